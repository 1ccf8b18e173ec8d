// Receiver side of a reduce-scatter: out[rows, N] = sum over the G GPUs of their partial row block,
// bf16 in, fp32 accumulate in ascending GPU order, one round-to-nearest-even to bf16.
//
// The paper leaves reduce-scatter out because a DMA engine cannot add (Sec. IV-E, the scenarios it
// studies); this kernel is the adding half, built so that it overlaps with the incoming
// transfers the way the GEMM overlaps with an all-gather: a block is cut into `pieces` row pieces,
// piece s of every peer's partial block arrives in step s, and one launch per reduction walks the
// pieces in step order, each tile waiting (bounded) until the G-1 incoming copies of its piece have
// landed. The work is pure streaming - (G + 1) x 2 bytes per output element, no reuse - so the
// kernel is built for HBM: 16-byte coalesced loads, every peer's vector in flight before the first
// add, four vectors per thread, workgroups striding over tiles so that the whole machine stays busy
// on whichever pieces have arrived.
#include "ficco_internal.h"

namespace ficco {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

static __device__ __forceinline__ uint32_t pack2_rne(float lo, float hi)
{
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    uint32_t ra = (a + 0x7FFFu + ((a >> 16) & 1u)) >> 16;
    uint32_t rb = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    if ((a & 0x7FFFFFFFu) > 0x7F800000u) ra = (a >> 16) | 0x0040u;
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) rb = (b >> 16) | 0x0040u;
    return (ra & 0xFFFFu) | (rb << 16);
}

// same bounded wait as the GEMM kernels use (one thread; see Gate)
static __device__ __forceinline__ int piece_ready(const Gate &g, int chunk)
{
    const uint64_t t0 = wall_clock64();
    const uint32_t *f = g.flags + (size_t)chunk * kFlagStrideWords;
    const int64_t *sv = g.sig_value ? reinterpret_cast<const int64_t *>(g.sig_value[chunk]) : nullptr;
    for (;;) {
        if (sv) {
            if (__hip_atomic_load(sv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) <= 0) return 1;
        } else {
            if (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == g.epoch) return 1;
        }
        if (__hip_atomic_load(g.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0u) return 0;
        if (wall_clock64() - t0 > g.spin_limit_ticks) {
            __hip_atomic_store(g.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(g.status_host, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            return 0;
        }
        __builtin_amdgcn_s_sleep(8);
    }
}

constexpr int kVecPerThread = 4;                       // 16-byte vectors per thread and tile
constexpr int kTileVecs = 256 * kVecPerThread;         // 1024 vectors = 8192 elements = 16 KiB of output

__global__ __launch_bounds__(256) void rs_reduce_kernel(ReduceLaunch r)
{
    __shared__ int s_ok;
    const int64_t piece_vecs = r.piece_vecs;
    const int tiles_per_piece = (int)((piece_vecs + kTileVecs - 1) / kTileVecs);
    const int tiles = r.pieces * tiles_per_piece;
    const u32x4_t *own = reinterpret_cast<const u32x4_t *>(r.own);
    const u32x4_t *in = reinterpret_cast<const u32x4_t *>(r.in);
    u32x4_t *out = reinterpret_cast<u32x4_t *>(r.out);
    const int64_t block_vecs = piece_vecs * r.pieces;

    for (int t = blockIdx.x; t < tiles; t += gridDim.x) {
        const int s = t / tiles_per_piece, tt = t % tiles_per_piece;
        if (r.gated) {
            if (threadIdx.x == 0) {
                // The first tile of a piece watches the G-1 transfers (their signals live in host memory:
                // thousands of workgroups polling them would swamp the host link). It then raises the
                // piece's word in device memory - the flag slot of the receiver's own piece, which no
                // transfer ever uses - and the piece's other tiles watch that word. No tile depends on
                // another workgroup being resident: a tile that has not seen the word after a quarter of
                // the wait limit (far longer than any piece takes to land; the watcher may never have
                // been dispatched if other work holds CUs) watches the transfers itself and raises the
                // word as well, so such a launch ends late instead of giving up.
                const int mine = r.block * r.pieces + s;
                uint32_t *word = const_cast<uint32_t *>(r.gate.flags) + (size_t)mine * kFlagStrideWords;
                int ok = 1, watch = tt == 0;
                if (!watch) {
                    const uint64_t t0 = wall_clock64();
                    while (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != r.gate.epoch) {
                        if (__hip_atomic_load(r.gate.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0u) { ok = 0; break; }
                        if (wall_clock64() - t0 > r.gate.spin_limit_ticks / 4) { watch = 1; break; }
                        __builtin_amdgcn_s_sleep(8);
                    }
                }
                if (watch && ok) {
                    for (int p = 0; p < r.G && ok; ++p)
                        if (p != r.block) ok = piece_ready(r.gate, p * r.pieces + s);
                    if (ok) __hip_atomic_store(word, r.gate.epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
                }
                s_ok = ok;
            }
            __syncthreads();               // also orders the tile's loads after the flag reads
            const int ok = s_ok;
            __syncthreads();
            if (!ok) continue;             // the wait gave up: every later tile sees the status word at once
        }
        const int64_t v0 = (int64_t)s * piece_vecs + (int64_t)tt * kTileVecs;
        const int64_t v_end = (int64_t)(s + 1) * piece_vecs;
        float acc[kVecPerThread][8];
        int64_t vi[kVecPerThread];
#pragma unroll
        for (int k = 0; k < kVecPerThread; ++k) vi[k] = v0 + threadIdx.x + k * 256;
        // peer 0 initialises, the others are added in ascending order; loads of four peers are in flight together
        for (int p0 = 0; p0 < r.G; p0 += 4) {
            u32x4_t v[4][kVecPerThread];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = p0 + j;
                if (p < r.G) {
                    const u32x4_t *src = p == r.block ? own : in + (int64_t)p * block_vecs;
#pragma unroll
                    for (int k = 0; k < kVecPerThread; ++k)
                        if (vi[k] < v_end) v[j][k] = __builtin_nontemporal_load(src + vi[k]);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = p0 + j;
                if (p < r.G) {
#pragma unroll
                    for (int k = 0; k < kVecPerThread; ++k) {
                        if (vi[k] < v_end) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float lo = __uint_as_float(v[j][k][e] << 16), hi = __uint_as_float(v[j][k][e] & 0xFFFF0000u);
                                if (p == 0) { acc[k][2 * e] = lo; acc[k][2 * e + 1] = hi; }
                                else { acc[k][2 * e] += lo; acc[k][2 * e + 1] += hi; }
                            }
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < kVecPerThread; ++k) {
            if (vi[k] < v_end) {
                u32x4_t o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = pack2_rne(acc[k][2 * e], acc[k][2 * e + 1]);
                __builtin_nontemporal_store(o, out + vi[k]);
            }
        }
    }
}

int reduce_grid_size(int device)
{
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, rs_reduce_kernel, 256, 0) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return per_cu * cus;
}

hipError_t launch_reduce(const ReduceLaunch &r, int grid, hipStream_t s)
{
    if (grid <= 0 || r.G < 1 || r.pieces < 1 || r.piece_vecs < 1 || r.block < 0 || r.block >= r.G) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rs_reduce_kernel, dim3((unsigned)grid), dim3(256), 0, s, r);
    return hipGetLastError();
}

}  // namespace ficco
