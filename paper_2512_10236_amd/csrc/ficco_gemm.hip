// bf16 MFMA GEMM kernels for gfx950 (CDNA4): C[rows, N] = A[rows, K] * W[K, N], fp32 accumulate,
// one round-to-nearest-even to bf16 at the end.
//
// This is the "chunk GEMM" of the overlap path (paper Sec. II-B for the operation, Sec. V-A for
// launching it per landed piece or per step). Two entry kernels share one tile routine:
//   * gemm_blocks_kernel   - one launch over a list of equal-height row blocks (a monolithic GEMM,
//                            one landed piece, or the G pieces of a fused step read in place);
//   * gemm_resident_kernel - one launch for the whole run; workgroups draw tiles from a ticket
//                            counter in arrival order and wait on the piece's ready flag.
//
// Data flow per workgroup tile (BM x BN, 256 threads = 4 wavefronts of 64):
//   global --16 B loads--> registers --> LDS (two stages of BK = 64, XOR-swizzled 16 B slots)
//   LDS --ds_read_b128--> 8-element bf16 fragments --> v_mfma_f32_32x32x16_bf16 --> fp32 accumulators
// The weight is read from a packed copy Wt[N, K] (k contiguous), so A and Wt fragments use the
// same access pattern. Every output element is accumulated over k ascending by the same
// instruction, whatever the tile shape or row block, which makes results bit-identical across
// schedules.
#include "ficco_internal.h"

namespace ficco {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

static __device__ __forceinline__ uint32_t pack2_bf16_rne(float lo, float hi)
{
    // fp32 -> bf16 round to nearest even; NaN stays NaN (quiet).
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    uint32_t ra = (a + 0x7FFFu + ((a >> 16) & 1u)) >> 16;
    uint32_t rb = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    if ((a & 0x7FFFFFFFu) > 0x7F800000u) ra = (a >> 16) | 0x0040u;
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) rb = (b >> 16) | 0x0040u;
    return (ra & 0xFFFFu) | (rb << 16);
}

template <int BM_, int BN_, int WGM_, int WGN_>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
    static constexpr int THREADS = WGM * WGN * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;       // wavefront tile
    static constexpr int FM = WTM / 32, FN = WTN / 32;         // 32x32 MFMA blocks per wavefront
    static constexpr int A_STAGE = BM * kBK * 2, B_STAGE = BN * kBK * 2;   // bytes
    static constexpr int LDS_BYTES = 2 * (A_STAGE + B_STAGE);
    static constexpr int AL = (BM * 8) / THREADS, BL = (BN * 8) / THREADS; // 16 B loads per thread per stage
    static_assert(THREADS == 256, "loaders assume 256 threads");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wavefront tile is made of 32x32 blocks");
    static_assert(AL >= 1 && BL >= 1, "tile too small for the loader");
};

// Computes one BM x BN tile. a_tile: first row of the tile in A; rows_valid in [1, BM] rows of
// it exist (the others are neither stored nor allowed to fault: their loads are clamped to the
// last valid row). wt_tile: first row (= output column) of the tile in Wt; cols_valid likewise.
template <class T>
static __device__ __forceinline__ void compute_tile(const uint16_t *__restrict__ a_tile, int rows_valid,
                                                    const uint16_t *__restrict__ wt_tile, int cols_valid,
                                                    uint16_t *__restrict__ c_tile, int64_t lda, int64_t ldw,
                                                    int64_t ldc, int K, unsigned char *smem)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / T::WGN, wn = wave % T::WGN;

    // ---- global -> LDS loader: 16-byte slot q = tid + 256*i holds row q/8, k-slot q%8
    const uint16_t *ga[T::AL];
    const uint16_t *gb[T::BL];
    int sa[T::AL], sb[T::BL];
#pragma unroll
    for (int i = 0; i < T::AL; ++i) {
        int q = tid + 256 * i, r = q >> 3, kc = q & 7;
        int rr = r < rows_valid ? r : rows_valid - 1;
        ga[i] = a_tile + (int64_t)rr * lda + kc * 8;
        sa[i] = r * 128 + ((kc ^ ((r >> 1) & 7)) << 4);
    }
#pragma unroll
    for (int i = 0; i < T::BL; ++i) {
        int q = tid + 256 * i, r = q >> 3, kc = q & 7;
        int rr = r < cols_valid ? r : cols_valid - 1;
        gb[i] = wt_tile + (int64_t)rr * ldw + kc * 8;
        sb[i] = r * 128 + ((kc ^ ((r >> 1) & 7)) << 4);
    }

    // ---- LDS -> fragment addresses: lane reads row (lane%32) of a 32-row block, k-slot
    //      2*kk + lane/32, un-swizzled by ((row>>1)&7) which only depends on the lane
    const int frow = lane & 31, fh = lane >> 5, fs = (lane >> 1) & 7;
    const int a_frag_base = (wm * T::WTM + frow) * 128;
    const int b_frag_base = (wn * T::WTN + frow) * 128;

    f32x16_t acc[T::FN][T::FM];
#pragma unroll
    for (int j = 0; j < T::FN; ++j)
#pragma unroll
        for (int i = 0; i < T::FM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.f;

    unsigned char *smA = smem;
    unsigned char *smB = smem + 2 * T::A_STAGE;

    u32x4_t ra[T::AL], rb[T::BL];
    const int KT = K / kBK;

#pragma unroll
    for (int i = 0; i < T::AL; ++i) ra[i] = *reinterpret_cast<const u32x4_t *>(ga[i]);
#pragma unroll
    for (int i = 0; i < T::BL; ++i) rb[i] = *reinterpret_cast<const u32x4_t *>(gb[i]);
#pragma unroll
    for (int i = 0; i < T::AL; ++i) *reinterpret_cast<u32x4_t *>(smA + sa[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < T::BL; ++i) *reinterpret_cast<u32x4_t *>(smB + sb[i]) = rb[i];
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int st = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) {
#pragma unroll
            for (int i = 0; i < T::AL; ++i) ra[i] = *reinterpret_cast<const u32x4_t *>(ga[i] + (kt + 1) * kBK);
#pragma unroll
            for (int i = 0; i < T::BL; ++i) rb[i] = *reinterpret_cast<const u32x4_t *>(gb[i] + (kt + 1) * kBK);
        }
        const unsigned char *cA = smA + st * T::A_STAGE;
        const unsigned char *cB = smB + st * T::B_STAGE;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            const int slot = ((2 * kk + fh) ^ fs) << 4;
            bf16x8_t fa[T::FM], fb[T::FN];
#pragma unroll
            for (int i = 0; i < T::FM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8_t *>(cA + a_frag_base + i * 32 * 128 + slot);
#pragma unroll
            for (int j = 0; j < T::FN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8_t *>(cB + b_frag_base + j * 32 * 128 + slot);
            // operands swapped on purpose: D[n][m], so each lane ends up with 4 consecutive
            // columns of one C row (8-byte stores in the epilogue)
#pragma unroll
            for (int j = 0; j < T::FN; ++j)
#pragma unroll
                for (int i = 0; i < T::FM; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[j][i], 0, 0, 0);
        }
        if (more) {
            unsigned char *nA = smA + (st ^ 1) * T::A_STAGE;
            unsigned char *nB = smB + (st ^ 1) * T::B_STAGE;
#pragma unroll
            for (int i = 0; i < T::AL; ++i) *reinterpret_cast<u32x4_t *>(nA + sa[i]) = ra[i];
#pragma unroll
            for (int i = 0; i < T::BL; ++i) *reinterpret_cast<u32x4_t *>(nB + sb[i]) = rb[i];
        }
        __syncthreads();
    }

    // ---- epilogue: acc[j][i][v] is C[m][n] with m = wm*WTM + 32 i + lane%32,
    //      n = wn*WTN + 32 j + 8 (v/4) + 4 (lane/32) + v%4
#pragma unroll
    for (int i = 0; i < T::FM; ++i) {
        const int m = wm * T::WTM + i * 32 + frow;
        if (m < rows_valid) {
            uint16_t *crow = c_tile + (int64_t)m * ldc;
#pragma unroll
            for (int j = 0; j < T::FN; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int n = wn * T::WTN + j * 32 + 8 * b + 4 * fh;
                    if (n < cols_valid) {
                        u32x2_t p;
                        p.x = pack2_bf16_rne(acc[j][i][4 * b + 0], acc[j][i][4 * b + 1]);
                        p.y = pack2_bf16_rne(acc[j][i][4 * b + 2], acc[j][i][4 * b + 3]);
                        *reinterpret_cast<u32x2_t *>(crow + n) = p;
                    }
                }
        }
    }
}

// Workgroups are dispatched round-robin over the 8 XCDs (each with its own L2). Renumber them so
// that consecutive logical ids run on the same XCD, then walk the tile grid in groups of GROUP_M
// row tiles so that one XCD works on few A row tiles and W column tiles at a time.
static __device__ __forceinline__ int xcd_contiguous_id(int pid, int total)
{
    const int q = total >> 3, r = total & 7;
    const int xcd = pid & 7, idx = pid >> 3;
    return (xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q) + idx;
}

template <class T>
__global__ __launch_bounds__(256) void gemm_blocks_kernel(GemmLaunch a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tiles_n = (a.N + T::BN - 1) / T::BN;
    const int rt_per_block = (a.rows_per_block + T::BM - 1) / T::BM;
    const int tiles_m = a.n_blocks * rt_per_block;
    const int total = tiles_m * tiles_n;
    const int lid = xcd_contiguous_id(blockIdx.x, total);
    constexpr int GROUP_M = 8;
    const int per_group = GROUP_M * tiles_n;
    const int group = lid / per_group;
    const int first_m = group * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (lid % per_group) % gsz;
    const int tn = (lid % per_group) / gsz;

    const int blk = tm / rt_per_block, rt = tm % rt_per_block;
    const int brow0 = a.block_row0 ? a.block_row0[blk] : a.row0;
    const int64_t row0 = (int64_t)brow0 + (int64_t)rt * T::BM;
    const int rows_valid = min(T::BM, a.rows_per_block - rt * T::BM);
    const int col0 = tn * T::BN;
    const int cols_valid = min(T::BN, a.N - col0);
    compute_tile<T>(a.A + row0 * a.lda, rows_valid, a.Wt + (int64_t)col0 * a.K, cols_valid,
                    a.C + row0 * a.ldc + col0, a.lda, a.K, a.ldc, a.K, smem);
}

template <class T>
__global__ __launch_bounds__(256) void gemm_resident_kernel(ResidentLaunch r)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int s_tile;
    __shared__ int s_ok;
    const GemmLaunch &a = r.g;
    const int tiles_n = (a.N + T::BN - 1) / T::BN;
    const int rt_per_chunk = (a.rows_per_block + T::BM - 1) / T::BM;
    const int per_chunk = rt_per_chunk * tiles_n;
    const int total = r.n_chunks * per_chunk;

    for (;;) {
        if (threadIdx.x == 0) s_tile = (int)(atomicAdd(r.ticket, 1u) - r.ticket_base);
        __syncthreads();
        const int t = s_tile;
        if (t >= total) break;            // every workgroup draws exactly one ticket past the end
        const int p = t / per_chunk, w = t % per_chunk;
        const int chunk = r.arrival[p];
        if (threadIdx.x == 0) {
            int ok = 1;
            if (chunk < r.local_chunk_begin || chunk >= r.local_chunk_end) {
                const uint32_t *f = r.flags + (size_t)chunk * kFlagStrideWords;
                const uint64_t t0 = wall_clock64();
                for (;;) {
                    // system scope: read past the caches, the writer is a copy engine
                    uint32_t v = __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    if (v == r.epoch) break;
                    if (__hip_atomic_load(r.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0u) { ok = 0; break; }
                    if (wall_clock64() - t0 > r.spin_limit_ticks) {
                        __hip_atomic_store(r.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        ok = 0;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(8);
                }
            }
            s_ok = ok;
        }
        __syncthreads();                   // also orders the tile's loads after the flag read
        if (s_ok) {
            const int rt = w % rt_per_chunk, tn = w / rt_per_chunk;
            const int64_t row0 = (int64_t)chunk * a.rows_per_block + (int64_t)rt * T::BM;
            const int rows_valid = min(T::BM, a.rows_per_block - rt * T::BM);
            const int col0 = tn * T::BN;
            const int cols_valid = min(T::BN, a.N - col0);
            compute_tile<T>(a.A + row0 * a.lda, rows_valid, a.Wt + (int64_t)col0 * a.K, cols_valid,
                            a.C + row0 * a.ldc + col0, a.lda, a.K, a.ldc, a.K, smem);
        }
        __syncthreads();                   // s_tile / s_ok / LDS stages are reused
    }
}

// W[K,N] -> Wt[N,K] through a 64x64 LDS tile (padded), 256 threads.
__global__ __launch_bounds__(256) void pack_weight_kernel(const uint16_t *__restrict__ W, uint16_t *__restrict__ Wt,
                                                          int64_t K, int64_t N)
{
    __shared__ uint16_t t[64][66];
    const int64_t k0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
    for (int e = threadIdx.x; e < 64 * 64; e += 256) {
        int kk = e >> 6, nn = e & 63;
        if (k0 + kk < K && n0 + nn < N) t[kk][nn] = W[(k0 + kk) * N + n0 + nn];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 64 * 64; e += 256) {
        int nn = e >> 6, kk = e & 63;
        if (k0 + kk < K && n0 + nn < N) Wt[(n0 + nn) * K + k0 + kk] = t[kk][nn];
    }
}

// ------------------------------------------------------------------------------------------ host
typedef TileCfg<256, 256, 2, 2> T256x256;
typedef TileCfg<128, 128, 2, 2> T128x128;
typedef TileCfg<256, 128, 2, 2> T256x128;
typedef TileCfg<128, 256, 2, 2> T128x256;
typedef TileCfg<64, 256, 1, 4> T64x256;
typedef TileCfg<32, 256, 1, 4> T32x256;

TileShape tile_shape(int tile)
{
    switch (tile) {
    case TILE_256x256: return {256, 256, T256x256::LDS_BYTES, 256};
    case TILE_128x128: return {128, 128, T128x128::LDS_BYTES, 256};
    case TILE_256x128: return {256, 128, T256x128::LDS_BYTES, 256};
    case TILE_128x256: return {128, 256, T128x256::LDS_BYTES, 256};
    case TILE_64x256:  return {64, 256, T64x256::LDS_BYTES, 256};
    case TILE_32x256:  return {32, 256, T32x256::LDS_BYTES, 256};
    default: return {0, 0, 0, 0};
    }
}

template <class T>
static hipError_t set_lds_limit(const void *fn)
{
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
}

template <class T>
static hipError_t launch_gemm_t(const GemmLaunch &a, hipStream_t s)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_blocks_kernel<T>));
    if (once != hipSuccess) return once;
    const int tiles_n = (a.N + T::BN - 1) / T::BN;
    const int rt = (a.rows_per_block + T::BM - 1) / T::BM;
    const int64_t total = (int64_t)a.n_blocks * rt * tiles_n;
    if (total <= 0 || total > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_blocks_kernel<T>, dim3((unsigned)total), dim3(256), T::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <class T>
static hipError_t launch_resident_t(const ResidentLaunch &r, hipStream_t s)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_resident_kernel<T>));
    if (once != hipSuccess) return once;
    if (r.grid <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_resident_kernel<T>, dim3((unsigned)r.grid), dim3(256), T::LDS_BYTES, s, r);
    return hipGetLastError();
}

template <class T>
static int resident_grid_t(int device)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_resident_kernel<T>));
    (void)once;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemm_resident_kernel<T>, 256, T::LDS_BYTES) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return per_cu * cus;
}

hipError_t launch_gemm(int tile, const GemmLaunch &a, hipStream_t s)
{
    switch (tile) {
    case TILE_256x256: return launch_gemm_t<T256x256>(a, s);
    case TILE_128x128: return launch_gemm_t<T128x128>(a, s);
    case TILE_256x128: return launch_gemm_t<T256x128>(a, s);
    case TILE_128x256: return launch_gemm_t<T128x256>(a, s);
    case TILE_64x256:  return launch_gemm_t<T64x256>(a, s);
    case TILE_32x256:  return launch_gemm_t<T32x256>(a, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_resident(int tile, const ResidentLaunch &r, hipStream_t s)
{
    switch (tile) {
    case TILE_256x256: return launch_resident_t<T256x256>(r, s);
    case TILE_128x128: return launch_resident_t<T128x128>(r, s);
    case TILE_256x128: return launch_resident_t<T256x128>(r, s);
    case TILE_128x256: return launch_resident_t<T128x256>(r, s);
    case TILE_64x256:  return launch_resident_t<T64x256>(r, s);
    case TILE_32x256:  return launch_resident_t<T32x256>(r, s);
    default: return hipErrorInvalidValue;
    }
}

int resident_grid_size(int tile, int device)
{
    switch (tile) {
    case TILE_256x256: return resident_grid_t<T256x256>(device);
    case TILE_128x128: return resident_grid_t<T128x128>(device);
    case TILE_256x128: return resident_grid_t<T256x128>(device);
    case TILE_128x256: return resident_grid_t<T128x256>(device);
    case TILE_64x256:  return resident_grid_t<T64x256>(device);
    case TILE_32x256:  return resident_grid_t<T32x256>(device);
    default: return 0;
    }
}

hipError_t launch_pack_weight(const uint16_t *W, uint16_t *Wt, int64_t K, int64_t N, hipStream_t s)
{
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64));
    hipLaunchKernelGGL(pack_weight_kernel, grid, dim3(256), 0, s, W, Wt, K, N);
    return hipGetLastError();
}

}  // namespace ficco
