// Internal declarations shared by the kernel file and the C-ABI file of libficco. Not installed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ficco {

// Workgroup tile shapes. The k order (ascending, 16 at a time inside one 32x32x16 MFMA) is the
// same in all of them, so the output bits do not depend on the choice.
enum TileId : int { TILE_256x256 = 1, TILE_128x128 = 2, TILE_256x128 = 3, TILE_128x256 = 4,
                    TILE_64x256 = 5, TILE_32x256 = 6, TILE_COUNT = 7 };

struct TileShape { int bm, bn, lds_bytes, threads; };
TileShape tile_shape(int tile);

constexpr int kFlagStrideWords = 16;      // one ready flag per 64-byte line
constexpr int kBK = 64;                   // k extent of one LDS stage

// One GEMM launch over a list of equal-height row blocks of A/C (one block for a monolithic or
// per-piece launch, G blocks for a fused step).
struct GemmLaunch {
    const uint16_t *A;        // [*, K] bf16, leading dimension lda
    const uint16_t *Wt;       // packed weight [N, K] bf16
    uint16_t *C;              // [*, N] bf16, leading dimension ldc
    int64_t lda, ldc;
    int32_t N, K;
    const int32_t *block_row0;   // device table of n_blocks first rows, or nullptr
    int32_t row0;                // first row when block_row0 == nullptr (n_blocks == 1)
    int32_t n_blocks;
    int32_t rows_per_block;
    // Optional gate (copy-engine transfers raise flags instead of HIP events): every workgroup
    // waits until flags[wait_chunks[i]*kFlagStrideWords] == epoch for all i < n_wait.
    const uint32_t *flags;
    const int32_t *wait_chunks;
    int32_t n_wait;
    uint32_t epoch;
    uint32_t *status;             // [0] set to 1 when a bounded wait expires
    uint64_t spin_limit_ticks;    // in wall_clock64() ticks
};

// The resident kernel: tiles are taken from a ticket counter in arrival order; the tiles of the
// piece issued p-th wait until flags[arrival[p]*kFlagStrideWords] == epoch.
struct ResidentLaunch {
    GemmLaunch g;                 // block_row0/row0/n_blocks unused; rows_per_block = piece rows
    const int32_t *arrival;       // device, n_chunks chunk ids in arrival order
    int32_t n_chunks;
    const uint32_t *flags;        // device, n_chunks * kFlagStrideWords words
    uint32_t epoch;
    uint32_t *ticket;             // device, monotonically increasing across runs
    uint32_t ticket_base;         // value of *ticket when this run starts
    uint32_t *status;             // device, [0] set to 1 when a bounded wait expires
    uint64_t spin_limit_ticks;    // in wall_clock64() ticks
    int32_t grid;
    int32_t local_chunk_begin, local_chunk_end;   // chunk ids that need no flag (already resident), or empty
};

hipError_t launch_gemm(int tile, const GemmLaunch &a, hipStream_t s);
hipError_t launch_resident(int tile, const ResidentLaunch &a, hipStream_t s);
// One wavefront that waits (bounded) for the flags of chunks[0..n) to reach epoch; used to join the
// compute stream with copy-engine transfers when no GEMM consumes them.
hipError_t launch_wait_flags(const uint32_t *flags, const int32_t *chunks, int n, uint32_t epoch, uint32_t *status,
                             uint64_t spin_limit_ticks, hipStream_t s);
hipError_t launch_pack_weight(const uint16_t *W, uint16_t *Wt, int64_t K, int64_t N, hipStream_t s);
int resident_grid_size(int tile, int device);

}  // namespace ficco
