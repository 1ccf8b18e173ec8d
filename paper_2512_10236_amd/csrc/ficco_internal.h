// Internal declarations shared by the kernel file and the C-ABI file of libficco. Not installed.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace ficco {

// Workgroup tile shapes. The k order (ascending, 16 at a time inside one 32x32x16 MFMA) is the
// same in all of them, so the output bits do not depend on the choice.
enum TileId : int { TILE_256x256 = 1, TILE_128x128 = 2, TILE_256x128 = 3, TILE_128x256 = 4,
                    TILE_64x256 = 5, TILE_32x256 = 6, TILE_128x128D = 7, TILE_128x192 = 8, TILE_256x192 = 9, TILE_COUNT = 10 };

struct TileShape { int bm, bn, lds_bytes, threads; };
TileShape tile_shape(int tile);

constexpr int kFlagStrideWords = 16;      // one ready flag per 64-byte line
constexpr int kBK = 64;                   // k extent of one LDS stage
// Largest K (row stride of A and of the packed weight, in elements): the loaders address a tile's rows with 32-bit
// byte offsets from a 64-bit base, and 256 rows of 2^22 elements of 2 bytes span 2 GiB.
constexpr int64_t kMaxK = (int64_t)1 << 22;
constexpr int kTicketLists = 8;           // one tile list per XCD (each XCD has its own L2)

// Tiles of the resident kernels that list x (of kTicketLists) holds. The lists form a grid of
// kTicketLists / col_lists row classes by col_lists column blocks: list x takes the row tiles
// rc, rc + classes, rc + 2 classes, ... (rc = x % classes) of the arrival-ordered sequence of row
// tiles, times the column tiles of block x / classes (the column tiles cut into col_lists nearly
// equal runs). col_lists = 1: every list spans all column tiles.
__host__ __device__ inline int64_t resident_list_tiles(int64_t row_tiles, int64_t tiles_n, int x, int col_lists = 1)
{
    const int classes = kTicketLists / col_lists, rc = x % classes, cb = x / classes;
    const int64_t rows = row_tiles > rc ? (row_tiles - rc + classes - 1) / classes : 0;
    return rows * ((cb + 1) * tiles_n / col_lists - cb * tiles_n / col_lists);
}

// Relative cost of a tile order for one XCD, whose L2 is filled with what its workgroups have in
// flight: `slots` tiles taken from groups of g row tiles x `width` column tiles (width = the tn column
// tiles cut into col_lists blocks), i.e. part of one group or several whole groups. Counted in operand
// rows per k-step - rows of A plus rows of the packed weight - each weighted by where the fill comes
// from: the memory-side cache costs 1, HBM costs kHbmFillCost, and the kernels, whose rings hold two or
// three k-steps, feel that latency. A line is fetched from HBM by the first XCD that wants it; the
// XCDs that walk the same rows (the col_lists lists of a row class) or the same columns (the
// kTicketLists / col_lists lists of a column block) at the same time find it in the cache, and so do
// later passes over a group's rows and later groups' passes over the columns if the operand stays
// there (operands up to kCacheStayBytes do; a group's rows also do between its own rounds when the
// rows all row classes hold at that time fit). Among equal footprints groups of about three rounds of
// tiles were fastest. Fitted to sweeps of all 16 (col_lists, g) pairs on five shape/tile combinations
// (14 to 112 column tiles, 16 to 128 row tiles, 128x128 and 256x256 tiles) and checked against such
// sweeps on 8 shapes x 3 launch kinds: the pick is within 2 % of the best order in 23 of 24 cases.
// Known miss: with 128-row pieces of a short, very wide product (M = 4096, N = 14336) and the
// 128x128 tile (no longer chosen for it) the orders a step-bound group allows are all 6-16 % slower
// than the best free order, and the model picks the slowest of them.
constexpr double kHbmFillCost = 3.0;
constexpr int64_t kCacheStayBytes = 128ll << 20;       // of the 256 MB memory-side cache
__host__ inline double tile_order_cost(int bm, int bn, int64_t tn, int64_t row_tiles, int64_t slots, int col_lists, int g,
                                       int64_t a_bytes, int64_t w_bytes)
{
    const int classes = kTicketLists / col_lists;
    const int64_t rows_list = row_tiles / classes > 1 ? (row_tiles + classes - 1) / classes : 1;
    if (g > rows_list) g = (int)rows_list;
    const int64_t width = (tn + col_lists - 1) / col_lists;
    const int64_t per_group = (int64_t)g * width;
    const double rows_active = per_group >= slots ? (double)g : (double)g * (double)slots / (double)per_group;
    double cols_active = (double)slots / g > 1.0 ? (double)slots / g : 1.0;
    if (cols_active > (double)width) cols_active = (double)width;
    const double passes = per_group > slots ? (double)per_group / (double)slots : 1.0;       // rounds a group's rows stay in use
    const double groups = rows_list > g ? (double)rows_list / g : 1.0;                       // passes over a list's columns
    // a group's rows are needed for `passes` rounds in a row: the later ones find them cached if the rows that
    // all row classes hold at that time fit, even when the whole of A does not
    const int64_t group_rows_bytes = row_tiles > 0 ? a_bytes / row_tiles * g * classes : a_bytes;
    const double a_from_hbm = (a_bytes <= kCacheStayBytes || group_rows_bytes <= kCacheStayBytes) ? 1.0 / (col_lists * passes) : 1.0 / col_lists;
    const double w_from_hbm = w_bytes <= kCacheStayBytes ? 1.0 / (classes * groups) : 1.0 / classes;
    const double fill = rows_active * bm * (1.0 + (kHbmFillCost - 1.0) * a_from_hbm) +
                        cols_active * bn * (1.0 + (kHbmFillCost - 1.0) * w_from_hbm);
    const double off = log2((double)per_group / (3.0 * (double)slots));
    return fill * (1.0 + 0.02 * (off < 0 ? -off : off));
}

// Workgroups of a resident launch whose first list is x (workgroup b starts on list b % kTicketLists).
__host__ __device__ inline int resident_list_homes(int grid, int x) { return grid > x ? (grid - x + kTicketLists - 1) / kTicketLists : 0; }

// Atomic draws one resident launch makes on list x's counter: a workgroup's first tile of its first list
// is its rank there and needs no draw; if that covers the whole list nobody draws from it at all;
// otherwise every later tile is drawn and every workgroup draws exactly one ticket past the end of the
// list. The host advances its copy of each counter by this much per launch, so counters are never
// reset.
__host__ __device__ inline uint32_t resident_list_draws(int64_t list_tiles, int grid, int x)
{
    const int64_t homes = resident_list_homes(grid, x);
    return list_tiles > homes ? (uint32_t)(list_tiles - homes + grid) : 0u;
}

// How a kernel learns that piece `chunk` has landed:
//   flags     - flags[chunk*kFlagStrideWords] == epoch (a 4-byte copy or stream write queued behind the transfer)
//   sig_value - the 64-bit word at sig_value[chunk] has dropped to 0: the value field of the transfer's
//               own completion signal, decremented by the copy engine itself
// Both are read at system scope; the wait is bounded (status[0] = 1 when it expires).
struct Gate {
    const uint32_t *flags;
    const uint64_t *sig_value;    // device table of addresses, or nullptr to use flags
    uint32_t epoch;
    uint32_t *status;             // device word every waiting workgroup watches
    uint32_t *status_host;        // pinned host word set together with it, so that the host needs no copy to see it
    uint64_t spin_limit_ticks;    // in wall_clock64() ticks
};

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
    int32_t group_m;             // row tiles per group of the tile order: 1, 2, 4, 8, or 0 = the launcher chooses
    // Optional gate (copy-engine transfers): every workgroup waits until all of the pieces
    // wait_chunks[0..n_wait) are ready.
    Gate gate;
    const int32_t *wait_chunks;
    int32_t n_wait;
};

// What a resident kernel does on its way out when other plans' transfers wait for the end of this run
// (chained plans): every workgroup counts itself out, and the one that brings the counter (device,
// never reset) to `target` stores 0 into the value word of the signal those transfers depend on.
// release_value == nullptr: nothing to do.
struct RunExit {
    uint32_t *count;
    uint32_t target;
    int64_t *release_value;
};

// The resident kernel: tiles are taken from a ticket counter in arrival order; the tiles of the
// piece issued p-th wait until that piece is ready (g.gate).
struct ResidentLaunch {
    GemmLaunch g;                 // block_row0/row0/n_blocks/wait_chunks unused; rows_per_block = piece rows
    const int32_t *arrival;       // device, n_chunks chunk ids in arrival order
    int32_t n_chunks;
    uint32_t *ticket;             // device, kTicketLists counters kFlagStrideWords apart, monotonically increasing across runs
    uint32_t ticket_base[8];      // value of each counter when this run starts
    int32_t grid;
    int32_t group;                // row tiles per group of a list's tile order (1..8)
    int32_t col_lists;            // column blocks the lists are split into (1, 2, 4 or 8; see resident_list_tiles)
    int32_t local_chunk_begin, local_chunk_end;   // chunk ids that need no flag (already resident), or empty
    // GEMM -> reduce-scatter: when the last tile of a piece has been stored, the kernel releases the copy
    // that waits for the piece by storing 0 into the value word of the copy's dependency signal.
    uint32_t *done_count;         // device, one counter per chunk id, never reset: a run adds tiles_per_chunk to each
    const uint64_t *done_sig;     // device table: address of the value word of each chunk's dependency signal
    int32_t tiles_per_chunk;      // row tiles per piece x column tiles
    RunExit leave;
};

// The resident kernel for column (K) pieces: A is kept in K-sliced layout, slice after slice, slice s
// being the [M][k0[s+1] - k0[s]] row-major block of columns [k0[s], k0[s+1]) (equal widths unless the
// plan was given its own); piece s*shards + j is slice s of shard j (rows [j*rows_per_shard,
// (j+1)*rows_per_shard)). A workgroup owns one tile of C for all of K, keeps its accumulators in
// registers, and before each slice waits for the pieces that cover its rows.
struct Resident2DLaunch {
    GemmLaunch g;                 // A = K-sliced base, Wt, C, ldc, N, K (whole), gate; other fields unused
    int32_t M, slices, shards, rows_per_shard;
    const int32_t *k0;            // device, slices + 1 entries: first column of each slice, then K (multiples of the k-tile)
    uint32_t *ticket;
    uint32_t ticket_base[8];
    int32_t grid;
    int32_t gated;                // 0: operands resident, no waiting
    int32_t group, col_lists;     // tile order, as in ResidentLaunch
    RunExit leave;
};

// One receiver-side reduction (see ficco_reduce.hip): `in` is the landing buffer [G][rows][N] of the
// peers' partial blocks (slot `block` is not read), `own` this GPU's own partial block, `out` the
// reduced block; a block is `pieces` pieces of piece_vecs 16-byte vectors each; piece s of peer p is
// gate piece p * pieces + s.
struct ReduceLaunch {
    const uint16_t *in;
    const uint16_t *own;
    uint16_t *out;
    int64_t piece_vecs;
    int32_t G, block, pieces, gated;
    Gate gate;
};
hipError_t launch_reduce(const ReduceLaunch &r, int grid, hipStream_t s);
int reduce_grid_size(int device);

// Grouped (per-expert) resident GEMM over ragged row segments. row_tiles: n_row_tiles entries of
// kRowTileWords int32 {first row, rows (1..BM), expert, first piece, last piece, 0, 0, 0} in the order
// they become ready; a tile waits for pieces first..last (ids into the gate's tables) and multiplies
// its rows by Wt + expert * N * K.
constexpr int kRowTileWords = 8;
struct GroupedLaunch {
    GemmLaunch g;                 // A, Wt (all experts, [E][N][K]), C, lda, ldc, N, K, gate
    const int32_t *row_tiles;
    int32_t n_row_tiles;
    uint32_t *ticket;
    uint32_t ticket_base[8];
    int32_t grid;
    int32_t gated;
    int32_t group, col_lists;     // tile order, as in ResidentLaunch
};
hipError_t launch_grouped(int tile, const GroupedLaunch &a, hipStream_t s);
int grouped_grid_size(int tile, int device);

hipError_t launch_gemm(int tile, const GemmLaunch &a, hipStream_t s);
hipError_t launch_resident2d(int tile, const Resident2DLaunch &a, hipStream_t s);
int resident2d_grid_size(int tile, int device);
hipError_t launch_resident(int tile, const ResidentLaunch &a, hipStream_t s);
// One wavefront that waits (bounded) until the pieces chunks[0..n) are ready; used to join the
// compute stream with copy-engine transfers when no GEMM consumes them.
hipError_t launch_wait_ready(const Gate &gate, const int32_t *chunks, int n, hipStream_t s);
// One thread stores 0 into the value word of a completion signal (device-visible address) once everything
// before it on the stream has finished: transfers submitted with that signal as a dependency may start.
hipError_t launch_release_signal(uint64_t value_addr, hipStream_t s);
// Sender-side re-layout for column pieces out of a row-major matrix: piece (slice sl, shard j) = rows
// [j*rows_per_shard, (j+1)*rows_per_shard) x columns [k0[sl], k0[sl+1]) of src [M,K] is written as one
// contiguous block at element M*k0[sl] + j*rows_per_shard*width of dst (the K-sliced layout). Workgroups
// take blocks of rows_per_block rows of a piece, pieces in arrival order; stores go through the caches (a copy
// engine reads them next), and the workgroup that completes a piece (counter never reset: blocks_per_piece
// more per run) stores 0 into the value word of that piece's signal, which lets its transfer go.
struct SliceLaunch {
    const uint16_t *src;
    uint16_t *dst;
    int64_t M, K;
    int32_t shards, rows_per_shard;
    const int32_t *k0;            // device, slices + 1 entries
    const int32_t *arrival;       // device, piece ids (sl*shards + j) in arrival order
    int32_t n_pieces, rows_per_block, blocks_per_piece;
    uint32_t *done_count;         // device, per piece id
    const uint64_t *done_sig;     // device, per piece id: address of the signal's value word
};
hipError_t launch_slice_source(const SliceLaunch &a, hipStream_t s);
hipError_t launch_pack_weight(const uint16_t *W, uint16_t *Wt, int64_t K, int64_t N, hipStream_t s);
int resident_grid_size(int tile, int device);

}  // namespace ficco
