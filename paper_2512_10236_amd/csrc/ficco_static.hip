// ficco_gemm_static: the resident GEMM over operands that are already in place, for callers that
// cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc). Everything the resident kernel needs beyond its inputs and outputs - the ticket
// counters of its tile lists, the status word of its bounded waits, the one-entry arrival table and
// the packed copy of the weight - lives in one file-scope device array instead of plan-owned
// allocations. See include/ficco.h for the contract.
#include "ficco_plan.h"

namespace ficco {
namespace {

constexpr size_t kHeadBytes = 4096;                                  // counters, status word, arrival table
constexpr size_t kStaticBytes = kHeadBytes + FICCO_STATIC_MAX_WEIGHT_BYTES;
// layout of the head, in 32-bit words: [0, 144) ticket counters (kTicketLists + 1 lines of 16 words),
// [160] status word, [176] arrival table (one entry)
constexpr int kStatusWord = 160, kArrivalWord = 176, kHeadWordsCleared = 192;

// Every GPU the library runs on holds its own copy of this array until the process ends. Host code
// never passes the array's name to a kernel or a copy: the name is a host-side stand-in, and the
// address of a device's copy comes from hipGetSymbolAddress (scratch_of below).
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

unsigned char *g_scratch_of[64];                                      // per device, filled on first use

int scratch_of(int dev, unsigned char **out)
{
    if (dev < 0 || dev >= 64) return FICCO_ERR_ARG;
    if (!g_scratch_of[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));       // the current device's copy
        if (!ptr) return FICCO_ERR_HIP;
        g_scratch_of[dev] = static_cast<unsigned char *>(ptr);
    }
    *out = g_scratch_of[dev];
    return FICCO_OK;
}

// The array keeps the last call's contents: counters, status and the arrival entry start every call from
// zero. A kernel rather than a memset, so that a caller may capture the call into a graph.
__global__ __launch_bounds__(256) void static_clear_kernel(uint32_t *head)
{
    if (threadIdx.x < kHeadWordsCleared) head[threadIdx.x] = 0u;
}

}  // namespace
}  // namespace ficco

using namespace ficco;

extern "C" int ficco_gemm_static(int64_t M, int64_t K, int64_t N, const void *A_dev, const void *W_dev, void *C_dev, void *stream)
{
    if (!A_dev || !W_dev || !C_dev) return FICCO_ERR_ARG;
    if (M < 1 || K < 1 || N < 1 || K % 64 || N % 8 || M > 0x7FFFFFFF || N > 0x7FFFFFFF || K > kMaxK) return FICCO_ERR_SHAPE;
    if ((uint64_t)K * (uint64_t)N * 2u > (uint64_t)FICCO_STATIC_MAX_WEIGHT_BYTES) return FICCO_ERR_SHAPE;
    bool dev_ptr = false;
    for (const void *ptr : {A_dev, W_dev, (const void *)C_dev}) {
        int rc = is_device_ptr(ptr, &dev_ptr);
        if (rc || !dev_ptr) return FICCO_ERR_ARG;
    }
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    unsigned char *base = nullptr;
    int rc = scratch_of(dev, &base);
    if (rc) return rc;
    uint32_t *head = reinterpret_cast<uint32_t *>(base);
    uint16_t *wt = reinterpret_cast<uint16_t *>(base + kHeadBytes);
    hipStream_t s = (hipStream_t)stream;

    // the shape as a one-piece resident plan (host-side bookkeeping only): same tile choice and tile order
    // as ficco_run gives such a plan, hence the same kernel
    ficco_plan_t shape;
    shape.M = M; shape.K = K; shape.N = N; shape.G = 1; shape.c = 1;
    shape.schedule = FICCO_FINE_PERSISTENT;
    shape.order = FICCO_ORDER_STEP_MAJOR;
    if ((rc = build_lists(&shape))) return rc;
    int cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    shape.tile = choose_tile(&shape, cus);
    const TileShape ts = tile_shape(shape.tile);
    if (ts.bm == 0) return FICCO_ERR_ARG;
    const int64_t row_tiles = (M + ts.bm - 1) / ts.bm, tn = (N + ts.bn - 1) / ts.bn;
    int grid = resident_grid_size(shape.tile, dev);
    if (grid <= 0) return FICCO_ERR_HIP;
    if (row_tiles * tn < grid) grid = (int)(row_tiles * tn);
    shape.resident_grid = grid;
    const ListGeometry lg = resident_lists(&shape);
    if (!lg.col_lists) return FICCO_ERR_ARG;
    int khz = 100000;
    (void)hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);

    hipLaunchKernelGGL(static_clear_kernel, dim3(1), dim3(256), 0, s, head);
    HIP_TRY(hipGetLastError());
    HIP_TRY(launch_pack_weight((const uint16_t *)W_dev, wt, K, N, s));

    ResidentLaunch r{};
    r.g.A = (const uint16_t *)A_dev;
    r.g.Wt = wt;
    r.g.C = (uint16_t *)C_dev;
    r.g.lda = K;
    r.g.ldc = N;
    r.g.N = (int32_t)N;
    r.g.K = (int32_t)K;
    r.g.n_blocks = 1;
    r.g.rows_per_block = (int32_t)M;
    r.g.group_m = 0;
    // nothing is waited for (the one piece is resident); the gate only has to point at valid words
    r.g.gate = Gate{head + kStatusWord + 4, nullptr, 1u, head + kStatusWord, head + kStatusWord, (uint64_t)khz * 2000u};
    r.arrival = reinterpret_cast<const int32_t *>(head + kArrivalWord);
    r.n_chunks = 1;
    r.ticket = head;
    for (int x = 0; x < kTicketLists; ++x) r.ticket_base[x] = 0;      // the counters were just cleared
    r.grid = grid;
    r.group = lg.group;
    r.col_lists = lg.col_lists;
    r.local_chunk_begin = 0;
    r.local_chunk_end = 1;
    HIP_TRY(launch_resident(shape.tile, r, s));
    return FICCO_OK;
}
