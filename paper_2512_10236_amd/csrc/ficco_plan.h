// Host side of libficco shared between its source files: the plan object, the small helpers every
// part uses, and the functions one part offers the others. Not installed; the public contract is
// include/ficco.h.
#pragma once

#include "../../include/ficco.h"
#include "ficco_internal.h"

#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>
#include <hsa/amd_hsa_signal.h>

#include <algorithm>
#include <cmath>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <new>
#include <vector>

namespace ficco {

extern thread_local int g_last_hip;      // hipError_t (or hsa_status_t) of the last failed call on this thread

#define HIP_TRY(expr)                                \
    do {                                             \
        hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) {                      \
            g_last_hip = (int)e_;                    \
            return FICCO_ERR_HIP;                    \
        }                                            \
    } while (0)

struct Group {
    int pos_begin, pos_end;      // arrival positions consumed by this launch
};

constexpr int kEpochSlots = 65536;   // pinned source words for flag writes; epoch e lives in slot e

// What a plan shares with the plans chained behind it (ficco_plan_chain): two signals used in turn, armed
// by the host when a run of the owning plan starts and released when that run ends on the compute stream
// (by the resident kernel's last workgroup out, or by a one-thread kernel). The owner re-arms a signal two of its runs later, by which time it has
// waited for the run in between, whose transfers could only start after every consumer of the older
// signal had finished. Outlives the owner while a dependent still holds it.
struct ChainLink {
    hsa_signal_t free_sig[2]{};
    uint64_t addr[2] = {0, 0};        // device-visible addresses of the value words
    bool made = false, alive = true;
    int last = -1;                    // signal armed by the owner's latest run (-1: none yet)
    ~ChainLink()
    {
        if (made)
            for (auto &sg : free_sig) (void)hsa_signal_destroy(sg);
    }
};

}  // namespace ficco

struct ficco_plan_s {
    int64_t M = 0, K = 0, N = 0;
    int G = 0, c = 0;
    int schedule = 0, direction = FICCO_DIR_AG_GEMM, order = FICCO_ORDER_STEP_MAJOR, mode = FICCO_MODE_PAIR;
    int timing = 0, tile_opt = 0, flag_write = 0, local_shard = -1, hold_flags = 0;
    int64_t spin_limit_us = 2000000;
    int backend_opt = FICCO_COPY_AUTO, links_opt = 0;
    int packing = 0;                     // fused schedule with explicit Gather / Scatter copies
    int repeat = 1;                      // GEMM-only runs: launches enqueued this many times inside one bracket
    int tile_group = 0, tile_col_lists = 0;   // forced tile order (0 = chosen from the shape)
    std::shared_ptr<ficco::ChainLink> link;        // released at the end of this plan's runs (plans are chained behind it)
    std::shared_ptr<ficco::ChainLink> chain_from;  // this plan's transfers wait for the latest run of that link's owner
    std::vector<int64_t> slice_k0;       // column pieces: first column of each slice, then K (c + 1 entries)
    bool own_widths = false;             // slice_k0 was given by the caller (ficco_plan_set_slice_widths)
    int src_layout = FICCO_LAYOUT_ROW_MAJOR;   // column pieces: how A_src holds the activation
    // column pieces out of a row-major device source: the sender-side staging copy (K-sliced), one dependency signal
    // per piece that the re-layout kernel releases, their value-word addresses and the kernel's block counters
    uint16_t *d_slice_src = nullptr;
    std::vector<hsa_signal_t> sig_packed;
    uint64_t *d_packed_value = nullptr;
    uint32_t *d_packed_count = nullptr;
    // expert-parallel (grouped) plans: E experts, ragged pieces, piece id (e*c + s)*G + j
    bool grouped = false;
    int E = 1;
    std::vector<int64_t> token_rows;     // [G][E]
    std::vector<int64_t> piece_row0, piece_nrows;   // by piece id
    std::vector<int64_t> expert_row0, expert_nrows;
    int32_t *d_row_tiles = nullptr;
    int n_row_tiles = 0;
    int backend = 0, links = 0;             // as resolved by the last run
    int device = 0;
    int n_chunks = 0;
    int64_t m = 0;                       // rows per chunk
    std::vector<int32_t> arrival;        // chunk ids in issue order
    std::vector<int32_t> group_of;       // per arrival position
    std::vector<ficco::Group> groups;

    // resources (allocated by finalize())
    bool finalized = false;
    int tile = 0;
    int resident_grid = 0;
    uint32_t *d_words = nullptr;         // flags | status | scratch: fine-grained device memory, polled while engines write it
    uint32_t *d_ticket_mem = nullptr;    // ticket counter: ordinary device memory (device-scope atomics)
    uint32_t *d_flags = nullptr, *d_ticket = nullptr, *d_status = nullptr;
    int32_t *d_tables = nullptr;         // arrival | block_row0 (by arrival position)
    int32_t *d_arrival = nullptr, *d_block_row0 = nullptr;
    int32_t *d_gather_idx = nullptr, *d_scatter_idx = nullptr;   // by arrival position: n + chunk, 2n + chunk
    int32_t *d_slice_k0 = nullptr;       // column pieces: slice_k0 on the device (behind the other tables)
    uint16_t *d_pack_a = nullptr, *d_pack_c = nullptr;            // packing: step inputs [M,K] and step outputs [M,N], arrival order
    uint32_t *h_epochs = nullptr;        // pinned
    volatile uint32_t *h_status = nullptr;   // pinned, behind h_epochs
    uint16_t *d_wt = nullptr;            // packed weight [N,K]
    const void *packed_from = nullptr;
    hipEvent_t ev_begin = nullptr, ev_end = nullptr, ev_copy_first = nullptr, ev_copy_last = nullptr;
    hipEvent_t ev_gemm_first = nullptr, ev_gemm_last = nullptr;
    bool last_lean = false;           // last run recorded ev_begin/ev_end only (GEMM alone, no per-launch timing)
    // HIP graph of one run (stream backend, per-launch schedules): ficco_graph_capture / ficco_graph_launch
    bool capturing = false, last_graph = false;
    hipStream_t cap_cs = nullptr, cap_xs = nullptr;
    hipEvent_t cap_fork = nullptr, cap_join = nullptr;
    std::vector<hipEvent_t> cap_dep;
    hipGraph_t graph = nullptr;
    hipGraphExec_t graph_exec = nullptr;
    int graph_copies = 0, graph_launches = 0;
    int64_t graph_copy_bytes = 0;
    std::vector<hipEvent_t> ev_dep;          // per group: transfers of the group done / launch done
    std::vector<hipEvent_t> ev_copy_b, ev_copy_e, ev_gemm_b, ev_gemm_e;   // TIMING=1
    int wall_clock_khz = 100000;
    std::vector<hsa_signal_t> sig_data, sig_flag;   // copy-engine backend: per chunk id
    std::vector<hsa_signal_t> sig_gather, sig_scatter;   // packing: per chunk id
    std::vector<hsa_signal_t> sig_done;              // resident GEMM -> RS: per chunk id, released by the kernel
    uint64_t *d_done_value = nullptr;                // device table: value-word addresses of sig_done
    uint32_t *d_done_count = nullptr;                // device: tiles of each piece stored so far (never reset)
    uint64_t *d_sig_value = nullptr;                 // device table: address of each data signal's value word
    int sig_poll = -1;                               // -1 unknown, 0 flags by 4-byte copies, 1 kernels poll the signals
    bool last_engines = false;
    bool last_reduce = false;                       // last run was ficco_rs_reduce (flops are adds, not a GEMM)
    int last_skip_shard = -1;                       // shard whose pieces the last run did not move (local shard, own block)
    double last_engine_copy_span_us = 0, last_engine_copy_busy_us = 0;

    // run state
    uint32_t run_index = 0;
    uint32_t ticket_total[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // tickets drawn from each list by all resident runs so far
    uint32_t exit_total = 0;                               // workgroups counted out by all runs that released a chain signal in the kernel
    bool last_had_copies = false, last_had_gemm = false, last_timing = false;
    int64_t last_copy_bytes = 0;
    int last_n_copies = 0, last_n_launches = 0;
};

namespace ficco {

inline bool is_2d(const ficco_plan_t *p) { return p->schedule == FICCO_FINE_2D; }

inline bool is_resident(const ficco_plan_t *p) { return p->schedule == FICCO_FINE_PERSISTENT || p->schedule == FICCO_FINE_2D; }

// shard a piece belongs to: row pieces are numbered shard-major (j*c + s), column pieces slice-major (s*G + j)
inline int shard_of(const ficco_plan_t *p, int chunk) { return is_2d(p) ? chunk % p->G : chunk / p->c; }

// Rows one launch covers as equal-height blocks: contiguous runs of chunks are merged so that a
// monolithic launch is one block of M rows and a shard-major fused step is one block too.
struct LaunchShape { int n_blocks; int64_t rows_per_block; bool contiguous; int64_t row0; };

// Geometry of the resident kernel's tile lists (see resident_list_tiles and the tile order notes in
// the kernel file). S = row tiles that become available together (a step of the step-major order
// brings G pieces, the other orders one piece). The lists are cut into col_lists column blocks so
// that what an XCD has in flight - groups of `group` row tiles of a step times a run of column tiles,
// one workgroup slot each - costs least by tile_order_cost. Ties go to the smaller col_lists and group.
struct ListGeometry { int group, col_lists; };

// Where a transferred piece of the activation sits (byte offset, the same in the source and in A_dev) and
// how long it is. Row pieces: m whole rows. Column pieces: the shard's rows of slice s, which are contiguous
// in the K-sliced layout.
struct Extent { size_t off, bytes; };

inline Extent piece_extent(const ficco_plan_t *p, int chunk)
{
    if (!is_2d(p)) return {(size_t)chunk * p->m * p->K * 2, (size_t)p->m * p->K * 2};
    const int sl = chunk / p->G, j = chunk % p->G;
    const size_t kb = (size_t)p->slice_k0[sl], kw = (size_t)p->slice_k0[sl + 1] - kb;
    return {((size_t)p->M * kb + (size_t)j * p->m * kw) * 2, (size_t)p->m * kw * 2};
}

// ---- plan construction and launches (ficco_plan.hip)
int build_lists(ficco_plan_t *p);
int choose_tile(const ficco_plan_t *p, int cus);
int finalize(ficco_plan_t *p);
void release(ficco_plan_t *p);
int make_events(std::vector<hipEvent_t> &v, size_t n);
int pack_weight(ficco_plan_t *p, const void *W_dev, hipStream_t s);
int is_device_ptr(const void *ptr, bool *is_dev);
LaunchShape launch_shape(const ficco_plan_t *p, const Group &g);
GemmLaunch make_launch(const ficco_plan_t *p, const Group &g, const void *A_dev, void *C_dev);
ListGeometry pick_lists(const ficco_plan_t *p, const TileShape &ts, int64_t tn, int64_t row_tiles, int64_t S, int64_t slots,
                        int64_t a_bytes, int64_t w_bytes);
ListGeometry resident_lists(const ficco_plan_t *p);
int launch_2d(ficco_plan_t *p, const Gate &gate, bool gated, int grid, const void *A_dev, void *C_dev, hipStream_t cs,
              uint64_t release_addr = 0);

// ---- copy-engine backend (ficco_engines.hip)
hsa_status_t make_signal(hsa_signal_t *out);
bool wait_signal(hsa_signal_t sgn, double limit_s);
uint64_t signal_value_address(hsa_signal_t sg);
double engine_ticks_per_us();
int engines_prepare(ficco_plan_t *p, bool touches_host, std::vector<int> &eng, int &links);
int run_grouped(ficco_plan_t *p, const void *A_src, void *A_dev, void *C_dev, hipStream_t cs, bool src_dev);
int run_engines(ficco_plan_t *p, const void *A_src, void *A_dev, void *C_dev, void *const *peer_out,
                hipStream_t cs, bool src_dev, const std::vector<char> &peer_dev);

}  // namespace ficco
