// bf16 MFMA GEMM kernels for gfx950 (CDNA4): C[rows, N] = A[rows, K] * W[K, N], fp32 accumulate,
// one round-to-nearest-even to bf16 at the end.
//
// This is the "chunk GEMM" of the overlap path (paper Sec. II-B for the operation, Sec. V-A for
// launching it per landed piece or per step). Two entry kernels share one tile routine:
//   * gemm_blocks_kernel   - one launch over a list of equal-height row blocks (a monolithic GEMM,
//                            one landed piece, or the G pieces of a fused step read in place);
//   * gemm_resident_kernel - one launch for the whole run; workgroups draw tiles from a ticket
//                            counter in arrival order and wait until the tile's piece is ready.
//
// Data flow per workgroup tile (BM x BN, 256 threads = 4 wavefronts of 64):
//   global --global_load_lds_dwordx4--> LDS (two stages of BK = 64, XOR-swizzled 16 B slots)
//   LDS --ds_read_b128--> 8-element bf16 fragments --> v_mfma_f32_32x32x16_bf16 --> fp32 accumulators
// The weight is read from a packed copy Wt[N, K] (k contiguous), so A and Wt fragments use the
// same access pattern. Every output element is accumulated over k ascending by the same
// instruction, whatever the tile shape or row block, which makes results bit-identical across
// schedules.
#include "ficco_internal.h"
#include <stdlib.h>
#include <type_traits>
#include <algorithm>

namespace ficco {

#ifdef FICCO_PROBE
// profiling build only: per-wavefront-slot sums of {cycles waiting for loads, cycles at the barrier, cycles per k-step, k-steps}
__device__ unsigned long long g_probe[4][4];
__device__ unsigned long long g_probe_lgkm[4];
#define PROBE_T() clock64()
#endif

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

// 64 lanes x 16 B from global memory straight into 1 KiB of LDS starting at the wave-uniform byte address
// lds_base (lane l lands at lds_base + 16 l). The global address is a wave-uniform 64-bit base (scalar
// registers) plus a per-lane 32-bit byte offset, so that stepping along k costs scalar additions only and a
// load needs one vector register. Issued through inline assembly so that the waits are placed by hand
// (s_waitcnt vmcnt) and not widened by the compiler; M0 is declared clobbered, so the compiler keeps nothing
// of its own in it across the load.
static __device__ __forceinline__ void load_to_lds_16(const void *base, uint32_t lane_off, uint32_t lds_base)
{
    // (the base is the same in every lane by construction; the compiler cannot always see that - where it
    // comes out of a table in memory, say - and is told so, half by half)
    const uint64_t b = (uint64_t)base;
    const uint64_t ub = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(lane_off), "s"(ub), "s"(__builtin_amdgcn_readfirstlane(lds_base)) : "memory", "m0");
}
// Measuring builds (paper_2512_10236_amd/_build.py: build_variant) can take pieces out of the k loop to see what
// each costs; their results are wrong, their timing is the point. Every access stays where it was (addresses do not
// change) and no wait lasts longer than in the product build: FICCO_ABL_NOLOAD issues no global->LDS loads, FICCO_ABL_NOREAD no
// LDS fragment reads, FICCO_ABL_NOBAR no k-step barrier, FICCO_ABL_LATEWAIT gives the loads one more k-step before
// they are waited for. FICCO_PROBE adds clock reads around the waits (each costs a drain of the LDS counter).
template <int N>
static __device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
#ifdef FICCO_ABL_NOBAR
static __device__ __forceinline__ void wg_barrier() {}
#else
static __device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
#endif

template <int BM_, int BN_, int WGM_, int WGN_, int NSTAGE_, int BK_ = kBK>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
    static constexpr int NSTAGE = NSTAGE_;                     // LDS stages in the ring; loads run NSTAGE-1 k-tiles ahead
    static constexpr int BK = BK_;                             // k extent of one LDS stage: 64, or 32 (a deeper ring in the same LDS)
    static constexpr int KSUB = BK / 16;                       // sub-steps (one MFMA's k extent each) per stage
    static constexpr int ROWB = BK * 2;                        // bytes of a row of a stage
    static constexpr int SLOTS = BK / 8;                       // 16-byte slots per row
    static constexpr int RPL = 1024 / ROWB;                    // rows one load instruction (64 lanes x 16 B) fills
    static constexpr int SWZ_SHIFT = BK == 64 ? 1 : 2;         // rows that share a 256-byte bank line
    static constexpr int THREADS = WGM * WGN * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;       // wavefront tile
    static constexpr int FM = WTM / 32, FN = WTN / 32;         // 32x32 MFMA blocks per wavefront
    static constexpr int A_STAGE = BM * ROWB, B_STAGE = BN * ROWB;   // bytes
    static constexpr int STAGE = A_STAGE + B_STAGE;
    static constexpr int LDS_BYTES = NSTAGE * STAGE;
    static constexpr int NW = WGM * WGN;                       // wavefronts: 4 (one per SIMD) or 8 (two per SIMD)
    static constexpr int AB = BM / RPL / NW, BB = BN / RPL / NW; // 1 KiB blocks loaded per wavefront per stage
    static constexpr int LOADS = AB + BB;                      // load instructions per wavefront per k-tile
    static_assert(BK == 64 || BK == 32, "stages of 64 or 32 k values");
    static_assert(NSTAGE >= 2 && NSTAGE <= 4, "ring of 2 to 4 stages");
    static_assert(LDS_BYTES <= 160 * 1024 - 64, "LDS ring plus the kernels' few static words must fit one CU");
    static_assert(THREADS == 256 || THREADS == 512, "4 or 8 wavefronts");
    static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "every wavefront loads the same number of blocks");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wavefront tile is made of 32x32 blocks");
    static_assert(AB >= 1 && BB >= 1, "tile too small for the loader");
};

// Computes one BM x BN tile. a_tile: first row of the tile in A; rows_valid in [1, BM] rows of
// it exist (the others are neither stored nor allowed to fault: their loads are clamped to the
// last valid row). wt_tile: first row (= output column) of the tile in Wt; cols_valid likewise.
//
// LDS holds a ring of NSTAGE stages; a stage is BM + BN rows of 128 B (64 k values), the 16-byte
// slot kc of row r stored at slot kc ^ ((r >> 1) & 7) so that the 16 lanes of a ds_read_b128 phase
// hit 64 different banks. Loads go global -> LDS directly (no staging registers): a wavefront
// instruction fills 8 rows, lane l fetching the slot that belongs at position l. The big tile only
// has room for two stages; the smaller tiles use three or four, which is what keeps launches with
// few workgroups (small pieces) from being bound by load latency. The loop itself is described in
// tile_accumulate_from.
template <class T>
struct TileAcc {
    f32x16_t acc[T::FN][T::FM];
};

template <class T>
static __device__ __forceinline__ void tile_zero(TileAcc<T> &ta)
{
#pragma unroll
    for (int j = 0; j < T::FN; ++j)
#pragma unroll
        for (int i = 0; i < T::FM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) ta.acc[j][i][v] = 0.f;
}

struct NoHook {
    __device__ __forceinline__ void operator()() const {}
};

// Byte offset, from the first row of the tile, of what lane `lane` fetches for 1 KiB block `blk` of a stage:
// row blk*RPL + lane/SLOTS (clamped to the last row that exists), 16-byte slot (lane%SLOTS) ^ swizzle(row) of
// its k-tile. The swizzle - (row>>1)&7 for rows of 128 B, (row>>2)&3 for rows of 64 B - spreads the rows that
// share a 256-byte line of banks over different slots, so that the 16 lanes of a ds_read_b128 phase, which read
// the same k slot of 16 consecutive rows, hit 64 different banks.
template <class T>
static __device__ __forceinline__ uint32_t lane_offset(int blk, int lane, int rows_valid, int64_t row_stride_elems)
{
    const int row = blk * T::RPL + lane / T::SLOTS;
    const int kc = (lane % T::SLOTS) ^ ((row >> T::SWZ_SHIFT) & (T::SLOTS - 1));
    const int rr = row < rows_valid ? row : rows_valid - 1;
    return (uint32_t)(((int64_t)rr * row_stride_elems + kc * 8) * 2);
}

// Where the loader finds its part of k-tile kt of A. PlainA: one row-major block [rows, K] with row stride lda:
// a wave-uniform base that moves along k, and one per-lane byte offset per load (the tile's rows must span less
// than 4 GiB, which the shape rules guarantee: at most 256 rows of at most 2^31 elements... of 2 bytes - the
// launchers refuse row strides above kMaxK).
template <class T>
struct PlainA {
    uint32_t off[T::AB];
    const uint16_t *base;
    __device__ __forceinline__ PlainA(const uint16_t *a_tile, int rows_valid, int64_t lda, int wave, int lane) : base(a_tile)
    {
#pragma unroll
        for (int i = 0; i < T::AB; ++i) off[i] = lane_offset<T>(wave * T::AB + i, lane, rows_valid, lda);
    }
    __device__ __forceinline__ void seek(int) {}
    __device__ __forceinline__ const uint16_t *at(int kt) const { return base + (int64_t)kt * T::BK; }
};

// SlicedA: a run of consecutive k slices of the K-sliced layout (slice s = the [M][k0[s+1]-k0[s]] block that
// starts at element M*k0[s]), read as one k range. The issue stream walks the k-tiles in ascending order;
// `seek` moves to the slice a k-tile lies in and only then rebuilds the base and the per-lane offsets for that
// slice's row stride, so that inside a slice a load costs what it costs with PlainA.
template <class T>
struct SlicedA {
    uint32_t off[T::AB];
    const uint16_t *base;
    const uint16_t *A;
    const int32_t *k0;
    int64_t M, row0;
    int sl, kt_begin, kt_end, rows_valid, wave, lane;
    __device__ __forceinline__ SlicedA(const uint16_t *A_, const int32_t *k0_, int64_t M_, int64_t row0_, int first_slice, int rows_valid_,
                                       int wave_, int lane_)
        : base(A_), A(A_), k0(k0_), M(M_), row0(row0_), sl(first_slice - 1), kt_begin(0), kt_end(0), rows_valid(rows_valid_), wave(wave_), lane(lane_)
    {
    }
    __device__ __forceinline__ void seek(int kt)
    {
        while (kt >= kt_end) {               // uniform: every lane takes the same steps
            ++sl;
            const int kb = k0[sl], kw = k0[sl + 1] - kb;
            kt_begin = kt_end;
            kt_end += kw / T::BK;
            base = A + M * kb + row0 * kw;
#pragma unroll
            for (int i = 0; i < T::AB; ++i) off[i] = lane_offset<T>(wave * T::AB + i, lane, rows_valid, kw);
        }
    }
    __device__ __forceinline__ const uint16_t *at(int kt) const { return base + (int64_t)(kt - kt_begin) * T::BK; }
};

// Waits until at most `load_groups` k-tiles' worth of this wavefront's loads are outstanding (the counter wants
// a constant, hence the ladder; load_groups <= 2 with rings of at most four stages).
template <class T>
static __device__ __forceinline__ void wait_issued_after(int load_groups)
{
    if (load_groups >= 2) wait_vmem<2 * T::LOADS>();
    else if (load_groups == 1) wait_vmem<T::LOADS>();
    else wait_vmem<0>();
}

template <class T, class Hook = NoHook, class AddrA = PlainA<T>>
static __device__ __forceinline__ void tile_accumulate_from(TileAcc<T> &ta, AddrA &pa,
                                                            const uint16_t *__restrict__ wt_tile, int cols_valid,
                                                            int64_t ldw, int K, unsigned char *smem,
                                                            Hook after_first_wait = Hook())
{
    f32x16_t (&acc)[T::FN][T::FM] = ta.acc;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / T::WGN, wn = wave % T::WGN;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;

    uint32_t offb[T::BB];                  // per-lane byte offsets of the W loads from the tile's first row
#pragma unroll
    for (int i = 0; i < T::BB; ++i) offb[i] = lane_offset<T>(wave * T::BB + i, lane, cols_valid, ldw);
    // load l of the wavefront's LOADS loads of k-tile kt into `stage`: first the AB blocks of A, then the BB blocks
    // of W (k-tiles are issued in ascending order; load 0 of a k-tile comes first)
    auto issue_load = [&](int stage, int kt, int l) {
#ifdef FICCO_ABL_NOLOAD
        return;
#endif
        if (l == 0) pa.seek(kt);
        if (l < T::AB) load_to_lds_16(pa.at(kt), pa.off[l], lds0 + stage * T::STAGE + (wave * T::AB + l) * 1024);
        else load_to_lds_16(wt_tile + (int64_t)kt * T::BK, offb[l - T::AB], lds0 + stage * T::STAGE + T::A_STAGE + (wave * T::BB + (l - T::AB)) * 1024);
    };


    // LDS -> fragment addresses: lane reads row (lane%32) of a 32-row block, k-slot 2*kk + lane/32,
    // un-swizzled by the row's swizzle, which only depends on the lane
    const int frow = lane & 31, fh = lane >> 5, fs = (frow >> T::SWZ_SHIFT) & (T::SLOTS - 1);
    const int a_base = (wm * T::WTM + frow) * T::ROWB;
    const int b_base = T::A_STAGE + (wn * T::WTN + frow) * T::ROWB;

    const int KT = K / T::BK;
    constexpr int D = T::NSTAGE - 1;      // prefetch distance in k-tiles
    bf16x8_t fa[2][T::FM], fb[2][T::FN];
#ifdef FICCO_ABL_NOREAD
#pragma unroll
    for (int n = 0; n < 2; ++n) {
#pragma unroll
        for (int i = 0; i < T::FM; ++i) fa[n][i] = bf16x8_t{};
#pragma unroll
        for (int j = 0; j < T::FN; ++j) fb[n][j] = bf16x8_t{};
    }
#endif
    // fragment q of the FM + FN fragments of sub-step kk of the k-tile in the stage at `base`, into buffer n.
    // Order of arrival = order of first use by the MFMAs below (row block 0, then every column block, then the
    // other row blocks).
    auto read_frag = [&](const unsigned char *base, int kk, int n, int q) {
#ifdef FICCO_ABL_NOREAD
        return;
#endif
        const int slot = ((2 * kk + fh) ^ fs) << 4;
        if (q == 0) fa[n][0] = *reinterpret_cast<const bf16x8_t *>(base + a_base + slot);
        else if (q <= T::FN) fb[n][q - 1] = *reinterpret_cast<const bf16x8_t *>(base + b_base + (q - 1) * 32 * T::ROWB + slot);
        else fa[n][q - T::FN] = *reinterpret_cast<const bf16x8_t *>(base + a_base + (q - T::FN) * 32 * T::ROWB + slot);
    };
    constexpr int NM = T::FM * T::FN;           // MFMAs per sub-step
    constexpr int NR = T::FM + T::FN;           // fragment reads per sub-step
    constexpr int H1 = T::LOADS / 2, H2 = T::LOADS - H1;      // the two halves of a k-tile's loads

    // ---- prologue: the first D k-tiles' loads, the first barrier, the first fragments
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < KT) {
#pragma unroll
            for (int l = 0; l < T::LOADS; ++l) issue_load(d, d, l);
        }
    wait_issued_after<T>(min(D - 1, KT - 1));
    wg_barrier();                          // B_0: k-tile 0 has landed for everyone
    after_first_wait();
    if (D < KT) {
#pragma unroll
        for (int l = 0; l < H1; ++l) issue_load(D % T::NSTAGE, D, l);
    }
#pragma unroll
    for (int q = 0; q < NR; ++q) read_frag(smem, 0, 0, q);

    // ---- the loop, one k-tile (a stage of BK k values, KSUB sub-steps of one MFMA's k extent) per turn, rotated by
    // one sub-step: a turn runs all but the last sub-step of k-tile k out of the fragments read one sub-step earlier,
    // then waits for k-tile k+1 and for its own LDS reads and meets the others at barrier B_{k+1} (k-tile k+1 has
    // landed for everyone; everyone is done with the stage of k-tile k, which the loads of k-tile k+1+D may now
    // overwrite), and only then runs the last sub-step, whose MFMAs (16 in the big tiles) need registers only: under them go the first half of the loads of k-tile k+1+D and the reads of the first
    // fragments of k-tile k+1, so that neither the barrier nor the LDS latency behind it leaves the MFMA pipe
    // empty. The second half of those loads follows under sub-step 0 of the next turn. Every MFMA of the big
    // tiles is followed by at most one load or one read, and the order is pinned (sched_barrier), so that a
    // wavefront never issues a burst of loads: the four wavefronts share one address path, which takes about 16
    // cycles per load, and whatever a wavefront issues between two MFMAs beyond the 32 cycles one of them takes
    // leaves the MFMA pipe empty.
#ifdef FICCO_PROBE
    long long probe_vm = 0, probe_bar = 0, probe_step = 0, probe_last = 0, probe_n = 0, probe_lgkm = 0;
#endif
    // (A turn is compiled in two forms: the steady state, where every condition is known and the body has no
    // branch, and a general one for the first and last turns of a tile.)
    auto turn = [&](int k, auto l1st, auto l2nd, auto rn, auto steady_c) __attribute__((always_inline)) {
        constexpr bool steady = decltype(steady_c)::value;
        const unsigned char *cur = smem + (k % T::NSTAGE) * T::STAGE;
        const unsigned char *nxt = smem + ((k + 1) % T::NSTAGE) * T::STAGE;
        const int free_stage = k % T::NSTAGE;           // after B_{k+1}
#pragma unroll
        for (int kk = 0; kk < T::KSUB; ++kk) {
            const int c = kk & 1, n = c ^ 1;
            if (kk == T::KSUB - 1) {
                // everything this wavefront reads from the stage of k-tile k has arrived in registers
#ifdef FICCO_PROBE
                const long long pt0 = PROBE_T();
#endif
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#ifdef FICCO_PROBE
                const long long pt1 = PROBE_T();
#endif
                // ... and k-tile k+1 has landed: what may still be in flight are the loads issued after its own,
                // those of the k-tiles k+2 .. k+D that exist (memory operations complete in issue order)
#ifdef FICCO_ABL_LATEWAIT
                // timing-only ablation (results are wrong): the loads get one more k-step to arrive
                if constexpr (steady) wait_vmem<D * T::LOADS>();
#else
                if constexpr (steady) wait_vmem<(D - 1) * T::LOADS>();
#endif
                else if (rn) wait_issued_after<T>(min(D - 1, KT - 2 - k));
#ifdef FICCO_PROBE
                const long long pt2 = PROBE_T();
#endif
                wg_barrier();
#ifdef FICCO_PROBE
                const long long pt3 = PROBE_T();
                if (lane == 0) {
                    probe_vm += pt2 - pt1; probe_bar += pt3 - pt2; probe_lgkm += pt1 - pt0;
                    if (probe_last) probe_step += pt0 - probe_last;
                    probe_last = pt0; ++probe_n;
                }
#endif
            }
#pragma unroll
            for (int t = 0; t < NM; ++t) {
                const int i = t / T::FN, j = t % T::FN;
                // operands swapped on purpose: D[n][m], so each lane ends up with 4 consecutive
                // columns of one C row (8-byte stores in the epilogue)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c][j], fa[c][i], acc[j][i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                // under this MFMA: the reads and loads whose turn it is. Reads of the next sub-step's fragments go
                // behind the even MFMAs, loads behind the odd ones, where there are enough MFMAs to keep them apart.
#pragma unroll
                for (int q = 0; q < NR; ++q)
                    if (q * NM / NR == t) {
                        if (kk < T::KSUB - 1) read_frag(cur, kk + 1, n, q);
                        else if (rn) read_frag(nxt, 0, n, q);
                    }
                if (kk == T::KSUB - 1 && l1st) {
#pragma unroll
                    for (int l = 0; l < H1; ++l)
                        if (min(NM - 1, l * NM / H1 + ((NM / H1 / 2) | 1)) == t) issue_load(free_stage, k + 1 + D, l);
                }
                if (kk == 0 && l2nd) {
#pragma unroll
                    for (int l = 0; l < H2; ++l)
                        if (min(NM - 1, l * NM / H2 + ((NM / H2 / 2) | 1)) == t) issue_load((k + D) % T::NSTAGE, k + D, H1 + l);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    constexpr std::true_type yes{};
    constexpr std::false_type no{};
    int k = 0;
    for (; k + 1 < D && k + 1 + D < KT; ++k) turn(k, true, true, true, no);    // (rings of three or four stages only)
    for (; k + 1 + D < KT; ++k) turn(k, yes, yes, yes, yes);
    for (; k < KT; ++k) turn(k, false, k + D < KT, k + 1 < KT, no);
    // (the barrier before the last sub-step was the last one: every wavefront had finished reading the ring)
#ifdef FICCO_ABL_LATEWAIT
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
#ifdef FICCO_PROBE
    if (lane == 0) {
        atomicAdd(&g_probe[wave][0], (unsigned long long)probe_vm);
        atomicAdd(&g_probe[wave][1], (unsigned long long)probe_bar);
        atomicAdd(&g_probe[wave][2], (unsigned long long)probe_step);
        atomicAdd(&g_probe[wave][3], (unsigned long long)probe_n);
        atomicAdd(&g_probe_lgkm[wave], (unsigned long long)probe_lgkm);
    }
#endif
}


template <class T, class Hook = NoHook>
static __device__ __forceinline__ void tile_accumulate(TileAcc<T> &ta, const uint16_t *__restrict__ a_tile, int rows_valid,
                                                       const uint16_t *__restrict__ wt_tile, int cols_valid,
                                                       int64_t lda, int64_t ldw, int K, unsigned char *smem,
                                                       Hook after_first_wait = Hook())
{
    PlainA<T> pa(a_tile, rows_valid, lda, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), threadIdx.x & 63);
    tile_accumulate_from<T, Hook, PlainA<T>>(ta, pa, wt_tile, cols_valid, ldw, K, smem, after_first_wait);
}

// Rounds the accumulators to bf16 (nearest even) and stores the valid part of the tile.
template <class T>
static __device__ __forceinline__ void tile_store(const TileAcc<T> &ta, uint16_t *__restrict__ c_tile, int rows_valid,
                                                  int cols_valid, int64_t ldc)
{
    const f32x16_t (&acc)[T::FN][T::FM] = ta.acc;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / T::WGN, wn = wave % T::WGN;
    const int frow = lane & 31, fh = lane >> 5;
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

// The same result stored as whole row segments: a wavefront passes each 32-row block of its part of
// the tile through LDS (rows padded by 16 B so that they spread over the banks) and reads it back
// with consecutive lanes on consecutive 16-byte slots of a row, so a store instruction writes whole
// 128-byte lines instead of 16 bytes in each of 32 rows. Written through the caches (system scope):
// this is the epilogue for output that a copy engine reads while the kernel runs on, where partial
// lines would each go to memory on their own. Needs ldc % 8 == 0 and a 16-byte aligned C; uses the
// first 4 * 32 * (2 WTN + 16) bytes of the ring, which must be idle (tile_accumulate's final barrier)
// and stay idle until a workgroup barrier after the call.
template <class T>
static __device__ __forceinline__ void tile_store_rows_through(const TileAcc<T> &ta, uint16_t *__restrict__ c_tile, int rows_valid,
                                                               int cols_valid, int64_t ldc, unsigned char *smem)
{
    constexpr int SEG = T::WTN / 8;                 // 16-byte slots per row of the wavefront's part
    constexpr int STRIDE = T::WTN * 2 + 16;         // bytes between rows in LDS
    static_assert(T::NW * 32 * STRIDE <= T::LDS_BYTES, "staging area must fit the ring");
    static_assert((32 * SEG) % 64 == 0, "whole wavefront instructions");
    const f32x16_t (&acc)[T::FN][T::FM] = ta.acc;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / T::WGN, wn = wave % T::WGN;
    const int frow = lane & 31, fh = lane >> 5;
    unsigned char *mine = smem + wave * (32 * STRIDE);
#pragma unroll
    for (int i = 0; i < T::FM; ++i) {
#pragma unroll
        for (int j = 0; j < T::FN; ++j)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                u32x2_t p;
                p.x = pack2_bf16_rne(acc[j][i][4 * b + 0], acc[j][i][4 * b + 1]);
                p.y = pack2_bf16_rne(acc[j][i][4 * b + 2], acc[j][i][4 * b + 3]);
                *reinterpret_cast<u32x2_t *>(mine + frow * STRIDE + (j * 32 + 8 * b + 4 * fh) * 2) = p;
            }
        // same wavefront, LDS operations execute in order: no barrier between the two phases
#pragma unroll
        for (int it = 0; it < (32 * SEG) / 64; ++it) {
            const int q = it * 64 + lane;
            const int row = q / SEG, seg = q % SEG;
            const u32x4_t v = *reinterpret_cast<const u32x4_t *>(mine + row * STRIDE + seg * 16);
            const int m = wm * T::WTM + i * 32 + row;
            const int n = wn * T::WTN + seg * 8;
            if (m < rows_valid && n < cols_valid) {
                uint16_t *dst = c_tile + (int64_t)m * ldc + n;
                if (n + 8 <= cols_valid)
                    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(dst), "v"(v) : "memory");
                else   // N is a multiple of 4: the last slot of a row may be half there
                    __hip_atomic_store(reinterpret_cast<uint64_t *>(dst), (uint64_t)v.x | ((uint64_t)v.y << 32), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
    }
}

template <class T>
static __device__ __forceinline__ void compute_tile(const uint16_t *__restrict__ a_tile, int rows_valid,
                                                    const uint16_t *__restrict__ wt_tile, int cols_valid,
                                                    uint16_t *__restrict__ c_tile, int64_t lda, int64_t ldw,
                                                    int64_t ldc, int K, unsigned char *smem)
{
    TileAcc<T> ta;
    tile_zero(ta);
    tile_accumulate<T>(ta, a_tile, rows_valid, wt_tile, cols_valid, lda, ldw, K, smem);
    tile_store<T>(ta, c_tile, rows_valid, cols_valid, ldc);
}

// Bounded wait of one thread until a piece is ready (see Gate). Reads at system scope (past the
// caches): the writer is a copy engine. Returns 0 when the limit expires or another workgroup has
// already given up; the caller then skips its work, so every wave still reaches its exit.
static __device__ __forceinline__ int wait_ready(const Gate &g, int chunk)
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

// One look at a piece, without waiting: has it landed?
static __device__ __forceinline__ int peek_ready(const Gate &g, int chunk)
{
    if (g.sig_value) return __hip_atomic_load(reinterpret_cast<const int64_t *>(g.sig_value[chunk]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) <= 0;
    return __hip_atomic_load(g.flags + (size_t)chunk * kFlagStrideWords, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == g.epoch;
}

// Workgroups are dispatched round-robin over the 8 XCDs (each with its own L2). The tiles are cut
// into 8 runs of consecutive logical ids, one per XCD, and the tile grid is walked in groups of
// group_m row tiles, so that one XCD works on few A row tiles and W column tiles at a time. A launch
// with more tiles than the machine holds workgroups is started with that many workgroups only, and a
// workgroup takes every stride-th tile of its XCD's run: what is in flight on an XCD is the same run of
// ids that one workgroup per tile would give, without a workgroup start per tile.
struct XcdRun { int start, count, first, stride; };
static __device__ __forceinline__ XcdRun xcd_run(int pid, int grid, int total)
{
    const int q = total >> 3, r = total & 7;
    const int xcd = pid & 7;
    return {xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q, q + (xcd < r ? 1 : 0), pid >> 3, (grid - xcd + 7) >> 3};
}

template <class T>
__global__ __launch_bounds__(T::THREADS) void gemm_blocks_kernel(GemmLaunch a)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    if (a.n_wait > 0) {
        __shared__ int s_go;
        if (threadIdx.x == 0) {
            int ok = 1;
            for (int i = 0; i < a.n_wait && ok; ++i) ok = wait_ready(a.gate, a.wait_chunks[i]);
            s_go = ok;
        }
        __syncthreads();                   // also orders the tile's loads after the flag reads
        if (!s_go) return;
    }
    const int tiles_n = (a.N + T::BN - 1) / T::BN;
    const int rt_per_block = (a.rows_per_block + T::BM - 1) / T::BM;
    const int tiles_m = a.n_blocks * rt_per_block;
    const int total = tiles_m * tiles_n;
    const XcdRun run = xcd_run(blockIdx.x, gridDim.x, total);
    const int per_group = a.group_m * tiles_n;
    for (int t = run.first; t < run.count; t += run.stride) {
        const int lid = run.start + t;
        const int group = lid / per_group;
        const int first_m = group * a.group_m;
        const int gsz = min(tiles_m - first_m, a.group_m);
        const int tm = first_m + (lid % per_group) % gsz;
        const int tn = (lid % per_group) / gsz;

        const int blk = tm / rt_per_block, rt = tm % rt_per_block;
        const int brow0 = a.block_row0 ? a.block_row0[blk] : a.row0;
        const int64_t row0 = (int64_t)brow0 + (int64_t)rt * T::BM;
        const int rows_valid = min(T::BM, a.rows_per_block - rt * T::BM);
        const int col0 = tn * T::BN;
        const int cols_valid = min(T::BN, a.N - col0);
        // (tile_accumulate ends with a barrier after the last LDS read, so the next tile may refill the ring)
        compute_tile<T>(a.A + row0 * a.lda, rows_valid, a.Wt + (int64_t)col0 * a.K, cols_valid,
                        a.C + row0 * a.ldc + col0, a.lda, a.K, a.ldc, a.K, smem);
    }
}

// Tile order of the resident kernels. Row tiles are numbered in arrival order (R = arrival position x
// row tiles per piece + row tile in the piece) and dealt round-robin to kTicketLists lists, one per
// XCD, each with its own ticket counter: a workgroup first serves the list of the XCD it presumably
// runs on (workgroups are dispatched round-robin over the XCDs), so that the tiles sharing an L2 at
// any time are few row tiles times a run of column tiles, and then helps the other lists. Inside a
// list tiles go in groups of a few row tiles, row tile fastest: as many as one step delivers to the
// list (so that no workgroup draws a tile of the next step while tiles of this one are left), 1 to 8.
// When a step delivers few row tiles and there are many column tiles, one row tile times all columns
// per XCD would stream the whole weight through every L2 once per round; the row-piece kernel then
// splits the lists by column block as well (ResidentLaunch::col_lists), so that an XCD works on
// several row tiles of the step times a run of columns, as a launch over the step's pieces would.
//
// TileWalk hands a workgroup its next (list, tile) pair. The first tile of the first list is the
// workgroup's rank among the workgroups that start there (no memory access); later tiles are drawn
// from the list's counter. Before it turns to the other lists it reads their counters once, all
// loads in flight together: on a list that is already used up it only leaves its one
// past-the-end draw (an atomic whose result nobody waits for), and a list that the ranks of its own
// workgroups cover completely is never drawn from at all. Counter traffic is what a short launch
// pays at its start and end, since a draw goes to memory shared by all XCDs.
struct TileWalk {
    int turn;        // lists visited so far; the current list is (home + turn) % kTicketLists
    int first;       // the rank tile of the home list has not been handed out yet
    int looked;      // the other lists' counters have been read
    int spent;       // bit k: list (home + k) % kTicketLists was already used up at that look
    int x, t;        // the result: list and tile in the list, x < 0 when there is nothing left
};

// Issues, ahead of time, the draw that the next tile_walk_next() call would start with (if it would
// start with one) and returns 1 with the raw counter value in `drawn`; the caller puts this before
// work whose duration then hides the draw's round trip. Returns 0 when the next step is not a plain draw.
template <class TotalFn>
static __device__ __forceinline__ int tile_walk_predraw(const TileWalk &w, uint32_t *ticket, int grid, TotalFn total_of,
                                                        uint32_t &drawn)
{
    if (w.turn >= kTicketLists || w.first) return 0;
    const int y = (blockIdx.x + w.turn) % kTicketLists;
    if (total_of(y) <= resident_list_homes(grid, y)) return 0;
    if (w.turn > 0 && (!w.looked || ((w.spent >> w.turn) & 1))) return 0;
    drawn = __hip_atomic_fetch_add(ticket + y * kFlagStrideWords, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return 1;
}

template <class TotalFn>
static __device__ __forceinline__ void tile_walk_next(TileWalk &w, uint32_t *ticket, const uint32_t *base, int grid,
                                                      TotalFn total_of, int have_drawn = 0, uint32_t drawn = 0)
{
    const int home = blockIdx.x % kTicketLists, rank = blockIdx.x / kTicketLists;
    w.x = -1;
    while (w.turn < kTicketLists) {
        const int y = (home + w.turn) % kTicketLists;
        const int total = total_of(y), homes = resident_list_homes(grid, y);
        uint32_t *ctr = ticket + y * kFlagStrideWords;
        if (total <= homes) {
            // the ranks of the workgroups that start on this list cover it: nobody draws from its counter
            const bool mine = w.first && rank < total;
            w.first = 0;
            ++w.turn;
            if (mine) { w.x = y; w.t = rank; return; }
            continue;
        }
        if (w.turn > 0 && !w.looked) {
            uint32_t seen[kTicketLists];
#pragma unroll
            for (int k = 1; k < kTicketLists; ++k)
                seen[k] = __hip_atomic_load(ticket + ((home + k) % kTicketLists) * kFlagStrideWords, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
            int spent = 0;
#pragma unroll
            for (int k = 1; k < kTicketLists; ++k) {
                const int yk = (home + k) % kTicketLists;
                const int homes_k = resident_list_homes(grid, yk), total_k = total_of(yk);
                if (total_k > homes_k && (int)(seen[k] - base[yk]) + homes_k >= total_k) spent |= 1 << k;
            }
            w.spent = spent;
            w.looked = 1;
        }
        if (w.turn > 0 && ((w.spent >> w.turn) & 1)) {
            (void)__hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // result unused: no wait
            ++w.turn;
            continue;
        }
        int cand;
        if (w.first) {
            w.first = 0;
            if (rank >= total) continue;          // no tile at this rank: go on to the draws
            cand = rank;
        } else {
            const uint32_t raw = have_drawn ? drawn : __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            have_drawn = 0;
            cand = (int)(raw - base[y]) + homes;
        }
        if (cand < total) { w.x = y; w.t = cand; return; }
        ++w.turn;                                  // that was this workgroup's one draw past the end of list y
    }
}

// The lists of a resident launch as a grid of row classes x column blocks (see resident_list_tiles):
// which tiles list x holds and where tile t of it lies. Inside a list tiles go in groups of `group`
// row tiles, row tile fastest.
struct ListGrid {
    int row_tiles, tiles_n, group;
    int cl_shift;                // log2 of the number of column blocks (1, 2, 4 or 8 of them): shifts, not divisions
    __device__ __forceinline__ ListGrid(int row_tiles_, int tiles_n_, int col_lists, int group_)
        : row_tiles(row_tiles_), tiles_n(tiles_n_), group(group_), cl_shift(31 - __clz(col_lists)) {}
    __device__ __forceinline__ int class_shift() const { return 3 - cl_shift; }              // kTicketLists = 8 lists
    __device__ __forceinline__ int row_class(int x) const { return x & ((1 << class_shift()) - 1); }
    __device__ __forceinline__ int col_block(int x) const { return x >> class_shift(); }
    __device__ __forceinline__ int rows(int x) const
    {
        const int rc = row_class(x);
        return row_tiles > rc ? (row_tiles - rc + (1 << class_shift()) - 1) >> class_shift() : 0;
    }
    __device__ __forceinline__ int col_begin(int x) const { return (col_block(x) * tiles_n) >> cl_shift; }
    __device__ __forceinline__ int cols(int x) const { return (((col_block(x) + 1) * tiles_n) >> cl_shift) - col_begin(x); }
    __device__ __forceinline__ int total(int x) const { return rows(x) * cols(x); }
    // tile t of list x: R = its row tile in the arrival-ordered sequence, tn = its column tile
    __device__ __forceinline__ void position(int x, int t, int &R, int &tn) const
    {
        const int my_rows = rows(x), my_cols = cols(x);
        const int per_group = group * my_cols;
        const int g = t / per_group, first = g * group;
        const int gsz = min(my_rows - first, group);
        R = ((first + (t % per_group) % gsz) << class_shift()) + row_class(x);
        tn = col_begin(x) + (t % per_group) / gsz;
    }
};
static_assert(kTicketLists == 8, "ListGrid shifts assume 8 lists");

// A workgroup of a resident kernel has read everything it will read of A when it gets here (the data went
// through the MFMAs before its last tile was stored), so the last one out may let the next run's transfers
// into A start.
__device__ __forceinline__ void leave_run(const RunExit &e)
{
    if (e.release_value && threadIdx.x == 0) {
        const uint32_t before = __hip_atomic_fetch_add(e.count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (before + 1u == e.target)
            __hip_atomic_store(e.release_value, (int64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// STREAM_OUT: the GEMM -> reduce-scatter form (r.done_count set), a separate instantiation so that its
// epilogue and bookkeeping cost the all-gather form no registers.
template <class T, bool STREAM_OUT>
__global__ __launch_bounds__(T::THREADS) void gemm_resident_kernel(ResidentLaunch r)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __shared__ TileWalk s_walk;
    __shared__ int s_ok, s_chunk;
    const GemmLaunch &a = r.g;
    const int tiles_n = (a.N + T::BN - 1) / T::BN;
    const int rt_per_chunk = (a.rows_per_block + T::BM - 1) / T::BM;
    const int row_tiles = r.n_chunks * rt_per_chunk;
    const ListGrid lists(row_tiles, tiles_n, r.col_lists, r.group);
    auto total_of = [&](int x) { return lists.total(x); };

    if (threadIdx.x == 0) s_walk = TileWalk{0, 1, 0, 0, -1, 0};
    int have_drawn = 0;
    uint32_t drawn = 0;
    // Output streaming: a copy engine reads a piece of C while the kernel runs on, so
    // the tiles are written through the caches, and a tile is counted for its piece once every thread's
    // stores have been performed; whoever completes a piece lets its copy go. Ordering is by hand
    // (stores, their completion, barrier, counter, signal): a release fence would write back the whole
    // L2 once per tile. So that nobody waits for stores, a tile is counted under the next tile's
    // first k-step, or after the loop if it was the workgroup's last.
    int stored_chunk = -1;                 // thread 0: piece of the tile stored last and not yet counted
    auto count_stored = [&]() {
        if (STREAM_OUT && threadIdx.x == 0 && stored_chunk >= 0) {
            const uint32_t before = __hip_atomic_fetch_add(r.done_count + stored_chunk, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((before + 1u) % (uint32_t)r.tiles_per_chunk == 0u)
                __hip_atomic_store(reinterpret_cast<int64_t *>(r.done_sig[stored_chunk]), (int64_t)0, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_SYSTEM);
            stored_chunk = -1;
        }
    };
    for (;;) {
        if (threadIdx.x == 0) {
            TileWalk w = s_walk;
            tile_walk_next(w, r.ticket, r.ticket_base, r.grid, total_of, have_drawn, drawn);
            have_drawn = 0;
            int ok = 1;
            if (w.x >= 0) {
                int R, tn;
                lists.position(w.x, w.t, R, tn);
                const int chunk = r.arrival[R / rt_per_chunk];
                if (chunk < r.local_chunk_begin || chunk >= r.local_chunk_end) ok = wait_ready(a.gate, chunk);
                s_chunk = chunk;           // the others take it from here instead of the table in memory
            }
            s_walk = w;
            s_ok = ok;
        }
        __syncthreads();                   // also orders the tile's loads after the flag read
        const int x = s_walk.x, t = s_walk.t;
        if (x < 0) break;
        if (s_ok) {
            int R, tn;
            lists.position(x, t, R, tn);
            const int rt = R % rt_per_chunk;
            const int chunk = s_chunk;
            const int64_t row0 = (int64_t)chunk * a.rows_per_block + (int64_t)rt * T::BM;
            const int rows_valid = min(T::BM, a.rows_per_block - rt * T::BM);
            const int col0 = tn * T::BN;
            const int cols_valid = min(T::BN, a.N - col0);
            TileAcc<T> ta;
            tile_zero(ta);
            if constexpr (STREAM_OUT)
                tile_accumulate<T>(ta, a.A + row0 * a.lda, rows_valid, a.Wt + (int64_t)col0 * a.K, cols_valid, a.lda, a.K, a.K, smem,
                                   count_stored);
            else
                tile_accumulate<T>(ta, a.A + row0 * a.lda, rows_valid, a.Wt + (int64_t)col0 * a.K, cols_valid, a.lda, a.K, a.K, smem);
            // the next ticket's round trip runs under the epilogue
            if (threadIdx.x == 0) have_drawn = tile_walk_predraw(s_walk, r.ticket, r.grid, total_of, drawn);
            if constexpr (STREAM_OUT) {
                tile_store_rows_through<T>(ta, a.C + row0 * a.ldc + col0, rows_valid, cols_valid, a.ldc, smem);
                stored_chunk = chunk;
            } else {
                tile_store<T>(ta, a.C + row0 * a.ldc + col0, rows_valid, cols_valid, a.ldc);
            }
        }
        __syncthreads();                   // s_walk / s_ok / LDS stages are reused
    }
    if constexpr (STREAM_OUT) {
        wait_vmem<0>();
        __syncthreads();
        count_stored();
    }
    leave_run(r.leave);
}

// Column-piece variant of the resident kernel (the 2D communication shape of Sec. V-A, chosen when
// M <= K): step s delivers K-slice s of every shard, and every tile of C can make progress at every
// step. The accumulation order over k is that of the monolithic kernel, so the bits are the same.
template <class T>
__global__ __launch_bounds__(T::THREADS) void gemm_resident2d_kernel(Resident2DLaunch r)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __shared__ TileWalk s_walk;
    __shared__ int s_ok;
    const GemmLaunch &a = r.g;
    const int tiles_n = (a.N + T::BN - 1) / T::BN;
    const int row_tiles = (r.M + T::BM - 1) / T::BM;
    const ListGrid lists(row_tiles, tiles_n, r.col_lists, r.group);
    auto total_of = [&](int x) { return lists.total(x); };

    if (threadIdx.x == 0) s_walk = TileWalk{0, 1, 0, 0, -1, 0};
    int have_drawn = 0;
    uint32_t drawn = 0;
    for (;;) {
        if (threadIdx.x == 0) {
            TileWalk w = s_walk;
            tile_walk_next(w, r.ticket, r.ticket_base, r.grid, total_of, have_drawn, drawn);
            have_drawn = 0;
            s_walk = w;
        }
        __syncthreads();
        const int x = s_walk.x, t = s_walk.t;
        if (x < 0) break;
        int tm, tn;
        lists.position(x, t, tm, tn);
        const int64_t row0 = (int64_t)tm * T::BM;
        const int rows_valid = min(T::BM, r.M - (int)row0);
        const int col0 = tn * T::BN;
        const int cols_valid = min(T::BN, a.N - col0);
        const int j0 = (int)(row0 / r.rows_per_shard), j1 = (int)((row0 + rows_valid - 1) / r.rows_per_shard);
        TileAcc<T> ta;
        tile_zero(ta);
        int ok = 1;
        // The k loop takes runs of slices: it waits for the next slice, then looks (without waiting) how many of
        // the following ones have landed as well, and multiplies the whole run as one k range, so that the load
        // pipeline is only drained where the kernel has to wait anyway. With operands resident the run is all of K.
        for (int sl = 0; sl < r.slices && ok;) {
            int run_end = r.slices;
            if (r.gated) {
                if (threadIdx.x == 0) {
                    int o = 1;
                    for (int j = j0; j <= j1 && o; ++j) o = wait_ready(a.gate, sl * r.shards + j);
                    int e = sl + 1;
                    for (; o && e < r.slices; ++e) {
                        int landed = 1;
                        for (int j = j0; j <= j1 && landed; ++j) landed = peek_ready(a.gate, e * r.shards + j);
                        if (!landed) break;
                    }
                    s_ok = o ? e : 0;      // 0: gave up; else the slice after the run
                }
                __syncthreads();           // also orders the run's loads after the flag reads
                run_end = s_ok;
                ok = run_end != 0;
                __syncthreads();
            }
            if (ok) {
                const int kb = r.k0[sl], ke = r.k0[run_end];              // the run's columns: [kb, ke)
                SlicedA<T> pa(a.A, r.k0, r.M, row0, sl, rows_valid, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), threadIdx.x & 63);
                tile_accumulate_from<T, NoHook, SlicedA<T>>(ta, pa, a.Wt + (int64_t)col0 * a.K + kb, cols_valid, a.K, ke - kb, smem);
                sl = run_end;
            }
        }
        if (threadIdx.x == 0) have_drawn = tile_walk_predraw(s_walk, r.ticket, r.grid, total_of, drawn);
        if (ok) tile_store<T>(ta, a.C + row0 * a.ldc + col0, rows_valid, cols_valid, a.ldc);
        __syncthreads();                   // s_walk / s_ok / LDS stages are reused
    }
    leave_run(r.leave);
}

// Expert-parallel variant of the resident kernel (all-to-all token dispatch before the expert layers,
// Sec. II-A; unequal amounts per pair of GPUs, Sec. III-C): the rows of A are ragged segments, one per
// expert, each multiplied by that expert's weight. Row tiles never cross a segment; the host lists
// them in the order they become ready together with the pieces that cover them.
template <class T>
__global__ __launch_bounds__(T::THREADS) void gemm_grouped_kernel(GroupedLaunch r)
{
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    __shared__ TileWalk s_walk;
    __shared__ int s_ok;
    const GemmLaunch &a = r.g;
    const int tiles_n = (a.N + T::BN - 1) / T::BN;
    const ListGrid lists(r.n_row_tiles, tiles_n, r.col_lists, r.group);
    auto total_of = [&](int x) { return lists.total(x); };

    if (threadIdx.x == 0) s_walk = TileWalk{0, 1, 0, 0, -1, 0};
    int have_drawn = 0;
    uint32_t drawn = 0;
    for (;;) {
        if (threadIdx.x == 0) {
            TileWalk w = s_walk;
            tile_walk_next(w, r.ticket, r.ticket_base, r.grid, total_of, have_drawn, drawn);
            have_drawn = 0;
            int ok = 1;
            if (w.x >= 0 && r.gated) {
                int R, tn;
                lists.position(w.x, w.t, R, tn);
                const int32_t *rt = r.row_tiles + (size_t)R * kRowTileWords;
                for (int pc = rt[3]; pc <= rt[4] && ok; ++pc) ok = wait_ready(a.gate, pc);
            }
            s_walk = w;
            s_ok = ok;
        }
        __syncthreads();                   // also orders the tile's loads after the flag reads
        const int x = s_walk.x, t = s_walk.t;
        if (x < 0) break;
        if (s_ok) {
            int R, tn;
            lists.position(x, t, R, tn);
            const int32_t *rt = r.row_tiles + (size_t)R * kRowTileWords;
            const int64_t row0 = rt[0];
            const int rows_valid = rt[1];
            const int64_t expert = rt[2];
            const int col0 = tn * T::BN;
            const int cols_valid = min(T::BN, a.N - col0);
            TileAcc<T> ta;
            tile_zero(ta);
            tile_accumulate<T>(ta, a.A + row0 * a.lda, rows_valid, a.Wt + (expert * a.N + col0) * (int64_t)a.K, cols_valid,
                               a.lda, a.K, a.K, smem);
            if (threadIdx.x == 0) have_drawn = tile_walk_predraw(s_walk, r.ticket, r.grid, total_of, drawn);
            tile_store<T>(ta, a.C + row0 * a.ldc + col0, rows_valid, cols_valid, a.ldc);
        }
        __syncthreads();                   // s_walk / s_ok / LDS stages are reused
    }
}

__global__ __launch_bounds__(64) void wait_ready_kernel(Gate gate, const int32_t *chunks, int n)
{
    if (threadIdx.x == 0)
        for (int i = 0; i < n; ++i)
            if (!wait_ready(gate, chunks[i])) break;
}

// Nothing is published through the signal: what it orders is that the kernels before this one on the
// stream have finished reading A, which stream order has settled when this kernel starts. A relaxed store
// therefore does, and spares the cache write-back a release at system scope would add.
__global__ __launch_bounds__(64) void release_signal_kernel(int64_t *value)
{
    if (threadIdx.x == 0) __hip_atomic_store(value, (int64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
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

// Sender-side re-layout of column pieces out of a row-major matrix (see SliceLaunch). 16-byte vectors, a row
// of a piece is width/8 of them; the workgroup's threads stride over (row, vector) pairs of its block.
__global__ __launch_bounds__(256) void slice_source_kernel(SliceLaunch a)
{
    // blocks in arrival order, a bounded number of workgroups striding over them: the pieces of the first step
    // are finished - and their transfers released - first instead of every piece at the end
    const int total_blocks = a.n_pieces * a.blocks_per_piece;
    for (int blk = blockIdx.x; blk < total_blocks; blk += gridDim.x) {
        const int q = blk / a.blocks_per_piece, b = blk % a.blocks_per_piece;
        const int piece = a.arrival[q];
        const int sl = piece / a.shards, j = piece % a.shards;
        const int kb = a.k0[sl], kw = a.k0[sl + 1] - kb;
        const int r0 = b * a.rows_per_block, r1 = min(a.rows_per_shard, r0 + a.rows_per_block);
        const int vecs = kw / 8;
        const u32x4_t *src = reinterpret_cast<const u32x4_t *>(a.src + ((int64_t)j * a.rows_per_shard + r0) * a.K + kb);
        u32x4_t *dst = reinterpret_cast<u32x4_t *>(a.dst + a.M * kb + ((int64_t)j * a.rows_per_shard + r0) * kw);
        const int64_t src_pitch = a.K / 8;
        const int total = (r1 - r0) * vecs;
        for (int e = threadIdx.x; e < total; e += 4 * 256) {
            u32x4_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ee = e + u * 256;
                if (ee < total) v[u] = __builtin_nontemporal_load(src + (int64_t)(ee / vecs) * src_pitch + ee % vecs);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ee = e + u * 256;
                // written through the caches: the reader is a copy engine
                if (ee < total) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(dst + ee), "v"(v[u]) : "memory");
            }
        }
        // every store of the block has been performed (not just issued) before the block is counted
        wait_vmem<0>();
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t before = __hip_atomic_fetch_add(a.done_count + piece, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((before + 1u) % (uint32_t)a.blocks_per_piece == 0u)
                __hip_atomic_store(reinterpret_cast<int64_t *>(a.done_sig[piece]), (int64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

hipError_t launch_slice_source(const SliceLaunch &a, hipStream_t s)
{
    if (a.n_pieces <= 0 || a.blocks_per_piece <= 0 || a.rows_per_block <= 0) return hipErrorInvalidValue;
    const int64_t total = (int64_t)a.n_pieces * a.blocks_per_piece;
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(slice_source_kernel, dim3((unsigned)std::min<int64_t>(total, 1024)), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ host
// The big tile keeps two stages of 64 k values. Four stages of 32 (TileCfg<256, 256, 2, 2, 4, 32>) take the
// memory wait out of the loop but run 6-8 % slower: rows of 64 bytes double the cache lines each load
// instruction touches, and every 64 k values pay two barriers instead of one.
// Eight wavefronts (TileCfg<256, 256, 2, 4, 2> or <256, 256, 4, 2, 2>, two per SIMD, 128x64 each) give the
// same bits 2-5 % slower: a second wavefront per SIMD hides nothing that matters here, and the smaller
// wavefront tile reads half as much again from LDS per MFMA.
typedef TileCfg<256, 256, 2, 2, 2> T256x256;
typedef TileCfg<128, 128, 2, 2, 2> T128x128;       // two workgroups per CU: for launches that fill the machine
typedef TileCfg<128, 128, 2, 2, 4> T128x128D;      // deep ring, one workgroup per CU: for launches that do not
typedef TileCfg<256, 128, 2, 2, 3> T256x128;
typedef TileCfg<128, 256, 2, 2, 3> T128x256;
typedef TileCfg<64, 256, 1, 4, 3> T64x256;
typedef TileCfg<32, 256, 1, 4, 4> T32x256;
typedef TileCfg<128, 192, 2, 2, 3> T128x192;       // column counts that are multiples of 192 but not of 256
typedef TileCfg<256, 192, 2, 2, 2> T256x192;

// every tile shape, for the dispatch switches below
#define FICCO_FOR_EACH_TILE(X) \
    X(TILE_256x256, T256x256) X(TILE_128x128, T128x128) X(TILE_256x128, T256x128) X(TILE_128x256, T128x256) \
    X(TILE_64x256, T64x256) X(TILE_32x256, T32x256) X(TILE_128x128D, T128x128D) X(TILE_128x192, T128x192) \
    X(TILE_256x192, T256x192)

TileShape tile_shape(int tile)
{
    switch (tile) {
#define X(id, T) case id: return {T::BM, T::BN, T::LDS_BYTES, T::THREADS};
    FICCO_FOR_EACH_TILE(X)
#undef X
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
    if (total <= 0 || total > 0x7FFFFFFF || a.lda > kMaxK || a.K > kMaxK) return hipErrorInvalidValue;
    // at most as many workgroups as run at once (a multiple of 8, one share per XCD); the rest of the tiles
    // are taken by the kernel's loop
    int64_t grid = total;
    {
        static int fit_of[64];                       // per device: 0 = not asked yet, -1 = could not be asked
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
        int fit = dev < 64 ? fit_of[dev] : 0;
        if (fit == 0) {
            int per_cu = 0, cus = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemm_blocks_kernel<T>, T::THREADS, T::LDS_BYTES) == hipSuccess &&
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && per_cu * cus >= 8)
                fit = per_cu * cus / 8 * 8;
            else
                fit = -1;
            if (dev < 64) fit_of[dev] = fit;
        }
        if (fit > 0 && total > fit) grid = fit;
    }
    // group height of the tile order: matters when the launch runs for several rounds
    GemmLaunch b = a;
    if (b.group_m != 1 && b.group_m != 2 && b.group_m != 4 && b.group_m != 8) b.group_m = 0;
    if (!b.group_m) b.group_m = 8;
    if (!a.group_m && total > grid) {
        double best = -1;
        for (int g = 1; g <= 8; g *= 2) {
            const double c = tile_order_cost(T::BM, T::BN, tiles_n, (int64_t)a.n_blocks * rt, grid / 8, 1, g,
                                             (int64_t)a.n_blocks * a.rows_per_block * a.K * 2, (int64_t)a.N * a.K * 2);
            if (best < 0 || c < best) { best = c; b.group_m = g; }
        }
    }
    hipLaunchKernelGGL(gemm_blocks_kernel<T>, dim3((unsigned)grid), dim3(T::THREADS), T::LDS_BYTES, s, b);
    return hipGetLastError();
}

template <class T>
static hipError_t launch_resident_t(const ResidentLaunch &r, hipStream_t s)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_resident_kernel<T, false>));
    static hipError_t once_out = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_resident_kernel<T, true>));
    if (once != hipSuccess) return once;
    if (once_out != hipSuccess) return once_out;
    if (r.grid <= 0 || r.g.lda > kMaxK || r.g.K > kMaxK) return hipErrorInvalidValue;
    if (r.done_count)
        hipLaunchKernelGGL((gemm_resident_kernel<T, true>), dim3((unsigned)r.grid), dim3(T::THREADS), T::LDS_BYTES, s, r);
    else
        hipLaunchKernelGGL((gemm_resident_kernel<T, false>), dim3((unsigned)r.grid), dim3(T::THREADS), T::LDS_BYTES, s, r);
    return hipGetLastError();
}

template <class T>
static hipError_t launch_resident2d_t(const Resident2DLaunch &r, hipStream_t s)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_resident2d_kernel<T>));
    if (once != hipSuccess) return once;
    if (r.grid <= 0 || !r.k0 || r.g.K > kMaxK) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_resident2d_kernel<T>, dim3((unsigned)r.grid), dim3(T::THREADS), T::LDS_BYTES, s, r);
    return hipGetLastError();
}

template <class T>
static int resident2d_grid_t(int device)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_resident2d_kernel<T>));
    (void)once;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemm_resident2d_kernel<T>, T::THREADS, T::LDS_BYTES) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return per_cu * cus;
}

template <class T>
static hipError_t launch_grouped_t(const GroupedLaunch &r, hipStream_t s)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_grouped_kernel<T>));
    if (once != hipSuccess) return once;
    if (r.grid <= 0 || r.n_row_tiles <= 0 || r.g.lda > kMaxK || r.g.K > kMaxK) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_grouped_kernel<T>, dim3((unsigned)r.grid), dim3(T::THREADS), T::LDS_BYTES, s, r);
    return hipGetLastError();
}

template <class T>
static int grouped_grid_t(int device)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_grouped_kernel<T>));
    (void)once;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemm_grouped_kernel<T>, T::THREADS, T::LDS_BYTES) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return per_cu * cus;
}

template <class T>
static int resident_grid_t(int device)
{
    static hipError_t once = set_lds_limit<T>(reinterpret_cast<const void *>(&gemm_resident_kernel<T, false>));
    (void)once;
    int per_cu = 0, cus = 0;
    // (the output-streaming form may need more registers, but every tile shape is limited by LDS first)
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemm_resident_kernel<T, false>, T::THREADS, T::LDS_BYTES) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    return per_cu * cus;
}

#ifdef FICCO_PROBE
extern "C" int ficco_probe_read(unsigned long long *out16, int clear)
{
    if (hipMemcpyFromSymbol(out16, HIP_SYMBOL(g_probe), sizeof(unsigned long long) * 16) != hipSuccess) return -1;
    if (hipMemcpyFromSymbol(out16 + 16, HIP_SYMBOL(g_probe_lgkm), sizeof(unsigned long long) * 4) != hipSuccess) return -1;
    if (clear) {
        unsigned long long z[16] = {0};
        if (hipMemcpyToSymbol(HIP_SYMBOL(g_probe), z, sizeof(z)) != hipSuccess) return -1;
        if (hipMemcpyToSymbol(HIP_SYMBOL(g_probe_lgkm), z, sizeof(unsigned long long) * 4) != hipSuccess) return -1;
    }
    return 0;
}
#endif

hipError_t launch_gemm(int tile, const GemmLaunch &a, hipStream_t s)
{
    switch (tile) {
#define X(id, T) case id: return launch_gemm_t<T>(a, s);
    FICCO_FOR_EACH_TILE(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_resident(int tile, const ResidentLaunch &r, hipStream_t s)
{
    switch (tile) {
#define X(id, T) case id: return launch_resident_t<T>(r, s);
    FICCO_FOR_EACH_TILE(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_resident2d(int tile, const Resident2DLaunch &r, hipStream_t s)
{
    switch (tile) {
#define X(id, T) case id: return launch_resident2d_t<T>(r, s);
    FICCO_FOR_EACH_TILE(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

int resident2d_grid_size(int tile, int device)
{
    switch (tile) {
#define X(id, T) case id: return resident2d_grid_t<T>(device);
    FICCO_FOR_EACH_TILE(X)
#undef X
    default: return 0;
    }
}

int resident_grid_size(int tile, int device)
{
    switch (tile) {
#define X(id, T) case id: return resident_grid_t<T>(device);
    FICCO_FOR_EACH_TILE(X)
#undef X
    default: return 0;
    }
}

hipError_t launch_wait_ready(const Gate &gate, const int32_t *chunks, int n, hipStream_t s)
{
    hipLaunchKernelGGL(wait_ready_kernel, dim3(1), dim3(64), 0, s, gate, chunks, n);
    return hipGetLastError();
}

hipError_t launch_release_signal(uint64_t value_addr, hipStream_t s)
{
    if (!value_addr) return hipErrorInvalidValue;
    hipLaunchKernelGGL(release_signal_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<int64_t *>(value_addr));
    return hipGetLastError();
}

hipError_t launch_pack_weight(const uint16_t *W, uint16_t *Wt, int64_t K, int64_t N, hipStream_t s)
{
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((K + 63) / 64));
    hipLaunchKernelGGL(pack_weight_kernel, grid, dim3(256), 0, s, W, Wt, K, N);
    return hipGetLastError();
}

hipError_t launch_grouped(int tile, const GroupedLaunch &r, hipStream_t s)
{
    switch (tile) {
#define X(id, T) case id: return launch_grouped_t<T>(r, s);
    FICCO_FOR_EACH_TILE(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

int grouped_grid_size(int tile, int device)
{
    switch (tile) {
#define X(id, T) case id: return grouped_grid_t<T>(device);
    FICCO_FOR_EACH_TILE(X)
#undef X
    default: return 0;
    }
}

}  // namespace ficco
