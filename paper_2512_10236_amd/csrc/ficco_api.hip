// C-ABI of libficco: plan construction, the transfer/launch scheduler, statistics, the
// decomposition/contention profiler and the static schedule heuristic. See include/ficco.h for the
// contract of every entry point.
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

using namespace ficco;

namespace {

thread_local int g_last_hip = 0;

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

// ------------------------------------------------------------------ copy-engine (SDMA) context
struct EngineCtx {
    bool ready = false;
    int status = FICCO_OK;
    int device = -1;                                  // HIP device the context was set up for (one per process)
    hsa_agent_t gpu{}, cpu{};
    uint32_t mask_dd = 0, mask_hd = 0, mask_dh = 0;   // engine-status hints: device->device, host->device, device->host
    uint32_t validated = 0, failed = 0;               // engines that passed / failed the one-time self test
    double ticks_per_us = 100.0;
};
EngineCtx g_engines;

struct AgentPick { int want_gpu_index; int seen_gpu; bool have_gpu, have_cpu; hsa_agent_t gpu, cpu; };

hsa_status_t pick_agents(hsa_agent_t a, void *data)
{
    AgentPick *pk = (AgentPick *)data;
    hsa_device_type_t t;
    if (hsa_agent_get_info(a, HSA_AGENT_INFO_DEVICE, &t) != HSA_STATUS_SUCCESS) return HSA_STATUS_SUCCESS;
    if (t == HSA_DEVICE_TYPE_GPU) {
        if (pk->seen_gpu == pk->want_gpu_index && !pk->have_gpu) { pk->gpu = a; pk->have_gpu = true; }
        pk->seen_gpu += 1;
    } else if (t == HSA_DEVICE_TYPE_CPU && !pk->have_cpu) {
        pk->cpu = a;
        pk->have_cpu = true;
    }
    return HSA_STATUS_SUCCESS;
}

// One-time set-up: the HSA runtime is already up underneath HIP (hsa_init only adds a reference,
// which is never dropped), agents are looked up, the usable engines are queried and copy
// timestamps are switched on.
int engines_init(int hip_device)
{
    EngineCtx &c = g_engines;
    if (c.ready) return c.device == hip_device ? c.status : FICCO_ERR_ARG;   // one device per process drives the engines
    c.ready = true;
    c.device = hip_device;
    c.status = FICCO_ERR_HIP;
    const bool dbg = getenv("FICCO_DEBUG") != nullptr;
    hsa_status_t hs = hsa_init();
    if (hs != HSA_STATUS_SUCCESS) { if (dbg) fprintf(stderr, "ficco: hsa_init 0x%x\n", (int)hs); return c.status; }
    AgentPick pk{hip_device, 0, false, false, {}, {}};
    hs = hsa_iterate_agents(pick_agents, &pk);
    if (hs != HSA_STATUS_SUCCESS || !pk.have_gpu || !pk.have_cpu) {
        if (dbg) fprintf(stderr, "ficco: agents 0x%x gpu=%d cpu=%d want=%d seen=%d\n", (int)hs, pk.have_gpu, pk.have_cpu, hip_device, pk.seen_gpu);
        return c.status;
    }
    c.gpu = pk.gpu;
    c.cpu = pk.cpu;
    if (hsa_amd_memory_copy_engine_status(c.gpu, c.gpu, &c.mask_dd) != HSA_STATUS_SUCCESS) c.mask_dd = 0;
    if (hsa_amd_memory_copy_engine_status(c.gpu, c.cpu, &c.mask_hd) != HSA_STATUS_SUCCESS) c.mask_hd = 0;
    if (hsa_amd_memory_copy_engine_status(c.cpu, c.gpu, &c.mask_dh) != HSA_STATUS_SUCCESS) c.mask_dh = 0;
    uint64_t freq = 0;
    if (hsa_system_get_info(HSA_SYSTEM_INFO_TIMESTAMP_FREQUENCY, &freq) == HSA_STATUS_SUCCESS && freq > 0)
        c.ticks_per_us = (double)freq * 1e-6;
    if (!getenv("FICCO_NO_COPY_PROFILING")) (void)hsa_amd_profiling_async_copy_enable(true);
    if (c.mask_hd == 0) c.mask_hd = 0xFFFFu;          // hint missing: let the self test decide
    c.status = FICCO_OK;
    if (getenv("FICCO_DEBUG"))
        fprintf(stderr, "ficco: copy engines d2d=0x%x h2d=0x%x d2h=0x%x ticks/us=%.1f status=%d\n", c.mask_dd, c.mask_hd,
                c.mask_dh, c.ticks_per_us, c.status);
    return c.status;
}

// Waits (bounded) until a signal has dropped below 1. Returns false on timeout or on an error value.
// A completion signal for copy-engine transfers: one without a host interrupt behind it (it is consumed
// by the engines, by kernels that read its value word, and by host polling). With the default,
// interrupt-capable kind an engine left about 6 us between two copies on its queue, with this kind
// about 3.8 us (cfg2, eight 1 MiB pieces per engine: copy span 287 -> 259 us).
// FICCO_INTERRUPT_SIGNALS=1 in the environment brings the default kind back.
hsa_status_t make_signal(hsa_signal_t *out)
{
    static const bool interrupt = getenv("FICCO_INTERRUPT_SIGNALS") != nullptr;
    if (interrupt) return hsa_signal_create(0, 0, nullptr, out);
    return hsa_amd_signal_create(0, 0, nullptr, HSA_AMD_SIGNAL_AMD_GPU_ONLY, out);
}

bool wait_signal(hsa_signal_t sgn, double limit_s)
{
    if (hsa_signal_load_scacquire(sgn) < 1) return true;       // the usual case: already complete
    const auto t0 = std::chrono::steady_clock::now();
    for (;;) {
        hsa_signal_value_t v = hsa_signal_wait_scacquire(sgn, HSA_SIGNAL_CONDITION_LT, 1, 2000000, HSA_WAIT_STATE_BLOCKED);
        if (v < 0) return false;
        if (v < 1) return true;
        if (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > limit_s) return false;
    }
}

// What a plan shares with the plans chained behind it (ficco_plan_chain): two signals used in turn, armed
// by the host when a run of the owning plan starts and released by a one-thread kernel at the end of that
// run on the compute stream. The owner re-arms a signal two of its runs later, by which time it has
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

}  // namespace

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
    std::shared_ptr<ChainLink> link;        // released at the end of this plan's runs (plans are chained behind it)
    std::shared_ptr<ChainLink> chain_from;  // this plan's transfers wait for the latest run of that link's owner
    std::vector<int64_t> slice_k0;       // column pieces: first column of each slice, then K (c + 1 entries)
    bool own_widths = false;             // slice_k0 was given by the caller (ficco_plan_set_slice_widths)
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
    std::vector<Group> groups;

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

namespace {

inline bool is_2d(const ficco_plan_t *p) { return p->schedule == FICCO_FINE_2D; }
inline bool is_resident(const ficco_plan_t *p) { return p->schedule == FICCO_FINE_PERSISTENT || p->schedule == FICCO_FINE_2D; }
// shard a piece belongs to: row pieces are numbered shard-major (j*c + s), column pieces slice-major (s*G + j)
inline int shard_of(const ficco_plan_t *p, int chunk) { return is_2d(p) ? chunk % p->G : chunk / p->c; }

// Grouped plans: piece (e, s, j) has id (e*c + s)*G + j; the T[j][e] rows of a (peer, expert) block are cut
// into c pieces as equal as integers allow (the first T mod c one row longer); rows follow in id
// order, so an expert's rows are contiguous and, inside them, what arrives in one step.
int build_lists_grouped(ficco_plan_t *p)
{
    const int G = p->G, c = p->c, E = p->E, n = E * c * G;
    p->n_chunks = n;
    p->m = 0;
    p->piece_nrows.assign(n, 0);
    p->piece_row0.assign(n, 0);
    p->expert_row0.assign(E, 0);
    p->expert_nrows.assign(E, 0);
    for (int e = 0; e < E; ++e)
        for (int j = 0; j < G; ++j) {
            const int64_t T = p->token_rows[(size_t)j * E + e];
            p->expert_nrows[e] += T;
            for (int s = 0; s < c; ++s) p->piece_nrows[(size_t)(e * c + s) * G + j] = T / c + (s < T % c ? 1 : 0);
        }
    int64_t r = 0;
    for (int i = 0; i < n; ++i) { p->piece_row0[i] = r; r += p->piece_nrows[i]; }
    r = 0;
    for (int e = 0; e < E; ++e) { p->expert_row0[e] = r; r += p->expert_nrows[e]; }
    if (p->order != FICCO_ORDER_CUSTOM) {
        p->arrival.clear();
        const bool by_peer = p->schedule == FICCO_SHARD || p->order == FICCO_ORDER_SHARD_MAJOR;
        if (by_peer) {
            for (int j = 0; j < G; ++j)
                for (int s = 0; s < c; ++s)
                    for (int e = 0; e < E; ++e) p->arrival.push_back((e * c + s) * G + j);
        } else {
            for (int s = 0; s < c; ++s)
                for (int j = 0; j < G; ++j)
                    for (int e = 0; e < E; ++e) p->arrival.push_back((e * c + s) * G + j);
        }
    }
    p->groups.clear();
    p->groups.push_back({0, n});
    p->group_of.assign(n, 0);
    return FICCO_OK;
}

int build_lists(ficco_plan_t *p)
{
    if (p->grouped) return build_lists_grouped(p);
    const int G = p->G, c = p->c, n = G * c;
    p->n_chunks = n;
    p->m = is_2d(p) ? p->M / p->G : p->M / n;      // rows of one piece (column pieces keep the shard's rows)
    if (is_2d(p) && !p->own_widths) {
        // as equal as whole k-tiles allow: the first (K/64) mod c slices are one k-tile wider
        const int64_t kt = p->K / kBK, base = kt / c, extra = kt % c;
        p->slice_k0.assign((size_t)c + 1, 0);
        for (int sl = 0; sl < c; ++sl) p->slice_k0[sl + 1] = p->slice_k0[sl] + kBK * (base + (sl < extra ? 1 : 0));
    }
    if (p->order != FICCO_ORDER_CUSTOM) {
        p->arrival.clear();
        if (is_2d(p)) {
            // column pieces: id s*G + j; step-major = slice by slice (ascending ids), shard-major = shard by shard
            if (p->order == FICCO_ORDER_SHARD_MAJOR) {
                for (int j = 0; j < G; ++j)
                    for (int sl = 0; sl < c; ++sl) p->arrival.push_back(sl * G + j);
            } else {
                for (int i = 0; i < n; ++i) p->arrival.push_back(i);
            }
        } else if (p->schedule == FICCO_SERIAL || p->schedule == FICCO_SHARD || p->order == FICCO_ORDER_SHARD_MAJOR) {
            for (int i = 0; i < n; ++i) p->arrival.push_back(i);
        } else {
            for (int s = 0; s < c; ++s)
                for (int j = 0; j < G; ++j) p->arrival.push_back(j * c + s);
        }
    }
    // "hetero" start: the local shard's pieces come first and need no transfer
    if (p->local_shard >= 0 && !is_2d(p)) {
        std::stable_partition(p->arrival.begin(), p->arrival.end(),
                              [&](int32_t i) { return i / c == p->local_shard; });
    }
    p->groups.clear();
    p->group_of.assign(n, 0);
    switch (p->schedule) {
    case FICCO_SERIAL:
    case FICCO_FINE_PERSISTENT:
    case FICCO_FINE_2D:
        p->groups.push_back({0, n});
        break;
    case FICCO_SHARD:
    case FICCO_FINE_UNFUSED:
        for (int q = 0; q < n; ++q) p->groups.push_back({q, q + 1});
        break;
    case FICCO_FINE_FUSED:
        for (int q = 0; q < n; q += G) p->groups.push_back({q, std::min(q + G, n)});
        break;
    default:
        return FICCO_ERR_ARG;
    }
    for (size_t g = 0; g < p->groups.size(); ++g)
        for (int q = p->groups[g].pos_begin; q < p->groups[g].pos_end; ++q) p->group_of[q] = (int32_t)g;
    return FICCO_OK;
}

// Rows one launch covers as equal-height blocks: contiguous runs of chunks are merged so that a
// monolithic launch is one block of M rows and a shard-major fused step is one block too.
struct LaunchShape { int n_blocks; int64_t rows_per_block; bool contiguous; int64_t row0; };

LaunchShape launch_shape(const ficco_plan_t *p, const Group &g)
{
    bool contig = true;
    for (int q = g.pos_begin + 1; q < g.pos_end; ++q)
        if (p->arrival[q] != p->arrival[q - 1] + 1) { contig = false; break; }
    if (contig) return {1, (int64_t)(g.pos_end - g.pos_begin) * p->m, true, (int64_t)p->arrival[g.pos_begin] * p->m};
    return {g.pos_end - g.pos_begin, p->m, false, 0};
}

// Tile choice. Estimated time of a launch = k-steps x [full rounds over the machine x step(1) +
// step(fill of the last, partial round)], where step(f) = base + slope * f is the time of one k-step
// of that tile shape when a fraction f of the machine's workgroup slots is occupied (microseconds,
// fitted to a sweep of launch sizes on MI355X; the full-machine cost base + slope of the mid-size
// tiles re-fitted to multi-round resident launches after the tile order changed: 128x256 and 256x128
// run at 0.87-0.95 of the 256x256 tile's throughput there, 128x128 at 0.84-0.88); padded (masked)
// rows and columns are paid in full.
int choose_tile(const ficco_plan_t *p, int cus)
{
    static const struct { int id; double base, slope; int occ; } cand[] = {
        {TILE_256x256, 1.40, 0.45, 1}, {TILE_128x256, 0.80, 0.25, 1}, {TILE_256x128, 0.80, 0.27, 1},
        {TILE_128x128, 0.60, 0.48, 2}, {TILE_128x128D, 0.48, 0.08, 1},
        {TILE_64x256, 0.57, 0.15, 1},  {TILE_32x256, 0.45, 0.05, 1},
        {TILE_128x192, 0.72, 0.12, 1}, {TILE_256x192, 1.10, 0.45, 1},
    };
    double best = 1e300;
    int best_id = TILE_128x128;
    for (auto &cd : cand) {
        TileShape ts = tile_shape(cd.id);
        const double cap = (double)cus * cd.occ;
        auto cost = [&](int64_t tiles) {
            const double full = std::floor((double)tiles / cap), rem = (double)tiles - full * cap;
            return full * (cd.base + cd.slope) + (rem > 0 ? cd.base + cd.slope * rem / cap : 0.0);
        };
        double total = 0;
        if (p->grouped) {
            int64_t rt = 0;
            for (int64_t me : p->expert_nrows) rt += (me + ts.bm - 1) / ts.bm;
            total = cost(rt * ((p->N + ts.bn - 1) / ts.bn));
        } else if (is_2d(p)) {
            total = cost(((p->M + ts.bm - 1) / ts.bm) * ((p->N + ts.bn - 1) / ts.bn));
        } else if (p->schedule == FICCO_FINE_PERSISTENT) {
            total = cost((int64_t)p->n_chunks * ((p->m + ts.bm - 1) / ts.bm) * ((p->N + ts.bn - 1) / ts.bn));
        } else {
            for (auto &g : p->groups) {
                LaunchShape ls = launch_shape(p, g);
                total += cost((int64_t)ls.n_blocks * ((ls.rows_per_block + ts.bm - 1) / ts.bm) * ((p->N + ts.bn - 1) / ts.bn));
            }
        }
        if (total < best * 0.999) { best = total; best_id = cd.id; }
    }
    return best_id;
}

void release(ficco_plan_t *p)
{
    auto ev = [](hipEvent_t &e) { if (e) { (void)hipEventDestroy(e); e = nullptr; } };
    ev(p->ev_begin); ev(p->ev_end); ev(p->ev_copy_first); ev(p->ev_copy_last);
    ev(p->ev_gemm_first); ev(p->ev_gemm_last);
    ev(p->cap_fork); ev(p->cap_join);
    if (p->graph_exec) { (void)hipGraphExecDestroy(p->graph_exec); p->graph_exec = nullptr; }
    if (p->graph) { (void)hipGraphDestroy(p->graph); p->graph = nullptr; }
    if (p->cap_cs) { (void)hipStreamDestroy(p->cap_cs); p->cap_cs = nullptr; }
    if (p->cap_xs) { (void)hipStreamDestroy(p->cap_xs); p->cap_xs = nullptr; }
    for (auto *v : {&p->ev_dep, &p->cap_dep, &p->ev_copy_b, &p->ev_copy_e, &p->ev_gemm_b, &p->ev_gemm_e}) {
        for (auto &e : *v) ev(e);
        v->clear();
    }
    for (auto *v : {&p->sig_data, &p->sig_flag, &p->sig_gather, &p->sig_scatter, &p->sig_done}) {
        for (auto &sg : *v) (void)hsa_signal_destroy(sg);
        v->clear();
    }
    if (p->d_words) (void)hipFree(p->d_words);
    if (p->d_ticket_mem) (void)hipFree(p->d_ticket_mem);
    if (p->d_sig_value) (void)hipFree(p->d_sig_value);
    if (p->d_done_value) (void)hipFree(p->d_done_value);
    if (p->d_done_count) (void)hipFree(p->d_done_count);
    p->d_done_value = nullptr;
    p->d_done_count = nullptr;
    p->d_sig_value = nullptr;
    p->sig_poll = -1;
    p->d_ticket_mem = nullptr;
    if (p->d_tables) (void)hipFree(p->d_tables);
    if (p->d_wt) (void)hipFree(p->d_wt);
    if (p->d_row_tiles) (void)hipFree(p->d_row_tiles);
    p->d_row_tiles = nullptr;
    if (p->d_pack_a) (void)hipFree(p->d_pack_a);
    if (p->d_pack_c) (void)hipFree(p->d_pack_c);
    p->d_pack_a = p->d_pack_c = nullptr;
    if (p->h_epochs) (void)hipHostFree(p->h_epochs);
    p->d_words = nullptr; p->d_tables = nullptr; p->d_wt = nullptr; p->h_epochs = nullptr;
    p->finalized = false;
}

int make_events(std::vector<hipEvent_t> &v, size_t n)
{
    while (v.size() < n) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        v.push_back(e);
    }
    return FICCO_OK;
}

int finalize(ficco_plan_t *p)
{
    if (p->finalized) return FICCO_OK;
    if (p->d_words || p->d_tables || p->h_epochs) release(p);      // a previous attempt failed half way
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (p->device >= 0 && dev != p->device) return FICCO_ERR_ARG;
    p->device = dev;
    int rc = build_lists(p);
    if (rc) return rc;
    int cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    p->tile = p->tile_opt ? p->tile_opt : choose_tile(p, cus);
    if (tile_shape(p->tile).bm == 0) return FICCO_ERR_ARG;
    int khz = 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0) p->wall_clock_khz = khz;

    const int n = p->n_chunks;
    const size_t words = (size_t)n * kFlagStrideWords + 2 * kFlagStrideWords + 32;   // flags | ticket | status | 128 B scratch
    // Flags and the status word are read by running kernels at system scope while a copy engine or
    // another queue writes them: that is only coherent for fine-grained memory (ordinary device
    // memory is coherent at kernel boundaries only).
    if (hipExtMallocWithFlags((void **)&p->d_words, words * 4, hipDeviceMallocFinegrained) != hipSuccess) { release(p); return FICCO_ERR_ALLOC; }
    HIP_TRY(hipMemset(p->d_words, 0, words * 4));
    // ticket counters of the lists, then the counter of workgroups that have left a run (chained plans)
    if (hipMalloc((void **)&p->d_ticket_mem, (kTicketLists + 1) * kFlagStrideWords * 4) != hipSuccess) { release(p); return FICCO_ERR_ALLOC; }
    HIP_TRY(hipMemset(p->d_ticket_mem, 0, (kTicketLists + 1) * kFlagStrideWords * 4));
    HIP_TRY(hipDeviceSynchronize());
    p->d_flags = p->d_words;
    p->d_ticket = p->d_ticket_mem;
    p->d_status = p->d_words + (size_t)n * kFlagStrideWords + kFlagStrideWords;
    const size_t n_k0 = is_2d(p) ? p->slice_k0.size() : 0;
    if (hipMalloc((void **)&p->d_tables, sizeof(int32_t) * (4 * (size_t)n + n_k0)) != hipSuccess) { release(p); return FICCO_ERR_ALLOC; }
    p->d_arrival = p->d_tables;
    p->d_block_row0 = p->d_tables + n;
    p->d_gather_idx = p->d_tables + 2 * (size_t)n;
    p->d_scatter_idx = p->d_tables + 3 * (size_t)n;
    p->d_slice_k0 = n_k0 ? p->d_tables + 4 * (size_t)n : nullptr;
    std::vector<int32_t> host(4 * (size_t)n + n_k0);
    for (size_t sl = 0; sl < n_k0; ++sl) host[4 * (size_t)n + sl] = (int32_t)p->slice_k0[sl];
    for (int q = 0; q < n; ++q) {
        host[q] = p->arrival[q];
        host[n + q] = (int32_t)(p->arrival[q] * p->m);
        host[2 * (size_t)n + q] = n + p->arrival[q];
        host[3 * (size_t)n + q] = 2 * n + p->arrival[q];
    }
    HIP_TRY(hipMemcpy(p->d_tables, host.data(), host.size() * 4, hipMemcpyHostToDevice));
    if (hipHostMalloc((void **)&p->h_epochs, sizeof(uint32_t) * (kEpochSlots + 16), hipHostMallocDefault) != hipSuccess) {
        release(p);
        return FICCO_ERR_ALLOC;
    }
    for (int i = 0; i < kEpochSlots; ++i) p->h_epochs[i] = (uint32_t)i;
    p->h_status = p->h_epochs + kEpochSlots;     // set by a kernel whose bounded wait expired
    for (int i = 0; i < 16; ++i) p->h_status[i] = 0;

    HIP_TRY(hipEventCreate(&p->ev_begin));
    HIP_TRY(hipEventCreate(&p->ev_end));
    HIP_TRY(hipEventCreate(&p->ev_copy_first));
    HIP_TRY(hipEventCreate(&p->ev_copy_last));
    HIP_TRY(hipEventCreate(&p->ev_gemm_first));
    HIP_TRY(hipEventCreate(&p->ev_gemm_last));
    rc = make_events(p->ev_dep, p->groups.size());
    if (rc) return rc;
    if (p->grouped) {
        // row tiles never cross an expert's segment; each lists the pieces that cover its rows (all of
        // them for the serial schedule); sorted by the step in which the last of those pieces arrives
        TileShape ts = tile_shape(p->tile);
        const int c = p->c, G = p->G;
        struct RT { int64_t row0; int32_t rows, expert, first, last, step; };
        std::vector<RT> rts;
        for (int e = 0; e < p->E; ++e) {
            int pc = e * c * G;                                   // first piece of the expert
            const int pc_end = (e + 1) * c * G;
            for (int64_t r0 = p->expert_row0[e]; r0 < p->expert_row0[e] + p->expert_nrows[e]; r0 += ts.bm) {
                const int64_t r1 = std::min<int64_t>(r0 + ts.bm, p->expert_row0[e] + p->expert_nrows[e]);
                while (pc < pc_end && p->piece_row0[pc] + p->piece_nrows[pc] <= r0) ++pc;
                int last = pc;
                while (last + 1 < pc_end && p->piece_row0[last + 1] < r1) ++last;
                while (p->piece_nrows[last] == 0 && last > pc) --last;   // trailing pieces without rows cover nothing
                RT t{r0, (int32_t)(r1 - r0), e, pc, last, (last / G) % c};
                if (p->schedule == FICCO_SERIAL) { t.first = 0; t.last = n - 1; t.step = 0; }
                rts.push_back(t);
            }
        }
        std::stable_sort(rts.begin(), rts.end(), [](const RT &a, const RT &b) { return a.step < b.step; });
        p->n_row_tiles = (int)rts.size();
        std::vector<int32_t> tab((size_t)std::max<size_t>(rts.size(), 1) * kRowTileWords, 0);
        for (size_t i = 0; i < rts.size(); ++i) {
            int32_t *w = &tab[i * kRowTileWords];
            w[0] = (int32_t)rts[i].row0; w[1] = rts[i].rows; w[2] = rts[i].expert; w[3] = rts[i].first; w[4] = rts[i].last;
        }
        if (hipMalloc((void **)&p->d_row_tiles, tab.size() * 4) != hipSuccess) { release(p); return FICCO_ERR_ALLOC; }
        HIP_TRY(hipMemcpy(p->d_row_tiles, tab.data(), tab.size() * 4, hipMemcpyHostToDevice));
        p->resident_grid = grouped_grid_size(p->tile, dev);
        if (p->resident_grid <= 0) return FICCO_ERR_HIP;
        const int64_t tiles = (int64_t)p->n_row_tiles * ((p->N + ts.bn - 1) / ts.bn);
        if (tiles < p->resident_grid) p->resident_grid = (int)std::max<int64_t>(tiles, 1);
    } else if (is_resident(p)) {
        p->resident_grid = is_2d(p) ? resident2d_grid_size(p->tile, dev) : resident_grid_size(p->tile, dev);
        if (p->resident_grid <= 0) return FICCO_ERR_HIP;
        TileShape ts = tile_shape(p->tile);
        int64_t tiles = is_2d(p) ? ((p->M + ts.bm - 1) / ts.bm) * ((p->N + ts.bn - 1) / ts.bn)
                                 : (int64_t)n * ((p->m + ts.bm - 1) / ts.bm) * ((p->N + ts.bn - 1) / ts.bn);
        if (tiles < p->resident_grid) p->resident_grid = (int)tiles;
    }
    p->finalized = true;
    return FICCO_OK;
}

int pack_weight(ficco_plan_t *p, const void *W_dev, hipStream_t s)
{
    const size_t one = (size_t)p->K * p->N;
    if (!p->d_wt) {
        if (hipMalloc((void **)&p->d_wt, one * 2 * (size_t)p->E) != hipSuccess) return FICCO_ERR_ALLOC;
    }
    for (int e = 0; e < p->E; ++e)       // one matrix per expert (a single one for the other plans)
        HIP_TRY(launch_pack_weight((const uint16_t *)W_dev + e * one, p->d_wt + e * one, p->K, p->N, s));
    p->packed_from = W_dev;
    return FICCO_OK;
}

// hipMemcpyAsync with an explicit kind taken from where the source/destination live.
int is_device_ptr(const void *ptr, bool *is_dev)
{
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, ptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return FICCO_ERR_ARG;            // ordinary (pageable) host memory is not accepted
    }
    if (at.type == hipMemoryTypeDevice) { *is_dev = true; return FICCO_OK; }
    if (at.type == hipMemoryTypeHost) { *is_dev = false; return FICCO_OK; }
    return FICCO_ERR_ARG;
}

GemmLaunch make_launch(const ficco_plan_t *p, const Group &g, const void *A_dev, void *C_dev)
{
    GemmLaunch a{};
    a.A = (const uint16_t *)A_dev;
    a.Wt = p->d_wt;
    a.C = (uint16_t *)C_dev;
    a.lda = p->K;
    a.ldc = p->N;
    a.N = (int32_t)p->N;
    a.K = (int32_t)p->K;
    LaunchShape ls = launch_shape(p, g);
    a.group_m = p->tile_group;          // 0: the launcher chooses
    a.n_blocks = ls.n_blocks;
    a.rows_per_block = (int32_t)ls.rows_per_block;
    if (ls.contiguous) {
        a.block_row0 = nullptr;
        a.row0 = (int32_t)ls.row0;
    } else {
        a.block_row0 = p->d_block_row0 + g.pos_begin;
        a.row0 = 0;
    }
    return a;
}

// ------------------------------------------------------------------ copy-engine backend
// Engines for a run, in order of preference. The runtime's engine-status query is only a hint
// (older ROCr releases report no engine for copies inside one device although the forced-SDMA copy
// works), so every engine is validated once per process by a 64-byte device-to-device copy inside
// plan-owned scratch with a bounded wait; that first use also creates the engine's queue, which
// takes milliseconds and must not fall into a timed run.
std::vector<int> usable_engines(bool touches_host, int want, void *scratch64x2)
{
    EngineCtx &c = g_engines;
    std::vector<int> order;
    if (touches_host) {
        for (int i = 0; i < 16; ++i) order.push_back(i);             // low ids sit closest to the host link
    } else {
        // Engines with neighbouring ids share a path: eight consecutive ones copying at once ran at 43-58 GB/s
        // each, every second one at 58 GB/s each. So even ids first, and 0/1 last within their half (the
        // runtime's own host copies use them).
        for (int i = 2; i < 16; i += 2) order.push_back(i);
        order.push_back(0);
        for (int i = 3; i < 16; i += 2) order.push_back(i);
        order.push_back(1);
    }
    std::vector<int> out;
    for (int e : order) {
        if ((int)out.size() >= want) break;
        const uint32_t bit = 1u << e;
        if (!(c.mask_hd & bit) || (c.failed & bit)) continue;         // the flag copy is host -> device
        if (!(c.validated & bit)) {
            hsa_signal_t sg;
            if (hsa_signal_create(1, 0, nullptr, &sg) != HSA_STATUS_SUCCESS) { c.failed |= bit; continue; }
            hsa_status_t st = hsa_amd_memory_async_copy_on_engine((char *)scratch64x2 + 64, c.gpu, scratch64x2, c.gpu, 64, 0, nullptr,
                                                                  sg, (hsa_amd_sdma_engine_id_t)bit, true);
            const bool ok = st == HSA_STATUS_SUCCESS && wait_signal(sg, 2.0);
            if (st != HSA_STATUS_SUCCESS || ok) (void)hsa_signal_destroy(sg);   // a copy that never finished keeps its signal
            if (!ok) { c.failed |= bit; continue; }
            c.validated |= bit;
        }
        out.push_back(e);
    }
    return out;
}

// Geometry of the resident kernel's tile lists (see resident_list_tiles and the tile order notes in
// the kernel file). S = row tiles that become available together (a step of the step-major order
// brings G pieces, the other orders one piece). The lists are cut into col_lists column blocks so
// that what an XCD has in flight - groups of `group` row tiles of a step times a run of column tiles,
// one workgroup slot each - costs least by tile_order_cost. Ties go to the smaller col_lists and group.
struct ListGeometry { int group, col_lists; };
inline ListGeometry pick_lists(const ficco_plan_t *p, const TileShape &ts, int64_t tn, int64_t row_tiles, int64_t S, int64_t slots,
                               int64_t a_bytes, int64_t w_bytes)
{
    ListGeometry best{0, 0};
    double best_cost = -1;
    for (int cl = 1; cl <= kTicketLists; cl *= 2) {
        if (cl > 1 && cl > tn) break;
        if (p->tile_col_lists && p->tile_col_lists != cl) continue;
        // a group must not span steps: no workgroup should draw a tile of the next step while tiles of this one are left
        const int64_t g_max = p->tile_group ? 8 : std::max<int64_t>(1, std::min<int64_t>(8, S / (kTicketLists / cl)));
        for (int g = 1; g <= g_max; g *= 2) {
            if (p->tile_group && p->tile_group != g) continue;
            const double cost = tile_order_cost(ts.bm, ts.bn, tn, row_tiles, std::max<int64_t>(1, slots), cl, g, a_bytes, w_bytes);
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = {g, cl}; }
        }
    }
    return best;                 // {0, 0}: the forced column split does not fit the column tiles
}

// row pieces: a step of the step-major order brings G pieces, the other orders one piece at a time
inline ListGeometry resident_lists(const ficco_plan_t *p)
{
    const TileShape ts = tile_shape(p->tile);
    const int64_t rt = (p->m + ts.bm - 1) / ts.bm;
    return pick_lists(p, ts, (p->N + ts.bn - 1) / ts.bn, (int64_t)p->n_chunks * rt, (p->order == FICCO_ORDER_STEP_MAJOR ? (int64_t)p->G : 1) * rt,
                      p->resident_grid / kTicketLists, p->M * p->K * 2, p->N * p->K * 2);
}

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

// One resident launch of the K-sliced schedule: every tile owns its part of C for the whole k range
// and waits, slice by slice, for the column pieces of the shards its rows come from.
int launch_2d(ficco_plan_t *p, const Gate &gate, bool gated, int grid, const void *A_dev, void *C_dev, hipStream_t cs,
              uint64_t release_addr = 0)
{
    Resident2DLaunch r{};
    if (release_addr)
        r.leave = RunExit{p->d_ticket_mem + (size_t)kTicketLists * kFlagStrideWords, p->exit_total + (uint32_t)grid,
                          reinterpret_cast<int64_t *>(release_addr)};
    r.g.A = (const uint16_t *)A_dev;
    r.g.Wt = p->d_wt;
    r.g.C = (uint16_t *)C_dev;
    r.g.lda = 0;                         // per slice: its width
    r.g.ldc = p->N;
    r.g.N = (int32_t)p->N;
    r.g.K = (int32_t)p->K;
    r.g.gate = gate;
    r.M = (int32_t)p->M;
    r.slices = p->c;
    r.shards = p->G;
    r.rows_per_shard = (int32_t)(p->M / p->G);
    r.k0 = p->d_slice_k0;
    r.ticket = p->d_ticket;
    r.grid = grid;
    r.gated = gated ? 1 : 0;
    TileShape ts = tile_shape(p->tile);
    const int64_t row_tiles = (p->M + ts.bm - 1) / ts.bm, tn = (p->N + ts.bn - 1) / ts.bn;
    // column pieces: every tile can start with the first step, so any group height goes
    const ListGeometry lg = pick_lists(p, ts, tn, row_tiles, row_tiles, grid / kTicketLists, p->M * p->K * 2, p->N * p->K * 2);
    if (!lg.col_lists) return FICCO_ERR_ARG;
    r.group = lg.group;
    r.col_lists = lg.col_lists;
    for (int x = 0; x < kTicketLists; ++x) {
        r.ticket_base[x] = p->ticket_total[x];
        p->ticket_total[x] += resident_list_draws(resident_list_tiles(row_tiles, tn, x, r.col_lists), grid, x);
    }
    HIP_TRY(launch_resident2d(p->tile, r, cs));
    if (release_addr) p->exit_total += (uint32_t)grid;      // counted only once the workgroups are on their way
    return FICCO_OK;
}

// Address, as this GPU sees it, of the value word of a user signal (amd_signal_t, the layout AQL consumers
// use), or 0 when the runtime does not report the word as accessible to the GPU.
uint64_t signal_value_address(hsa_signal_t sg)
{
    amd_signal_t *as = reinterpret_cast<amd_signal_t *>(sg.handle);
    if (!as || as->kind != AMD_SIGNAL_KIND_USER) return 0;
    void *vp = (void *)&as->value;
    hsa_amd_pointer_info_t info{};
    info.size = sizeof(info);
    uint32_t n_acc = 0;
    hsa_agent_t *acc = nullptr;
    if (hsa_amd_pointer_info(vp, &info, malloc, &n_acc, &acc) != HSA_STATUS_SUCCESS || info.type == HSA_EXT_POINTER_TYPE_UNKNOWN) {
        if (acc) free(acc);
        return 0;
    }
    bool mine = false;
    for (uint32_t k = 0; k < n_acc; ++k) mine |= acc[k].handle == g_engines.gpu.handle;
    if (acc) free(acc);
    const uintptr_t off = (uintptr_t)vp - (uintptr_t)info.hostBaseAddress;
    if (!mine || !info.agentBaseAddress || !info.hostBaseAddress || off + 8 > info.sizeInBytes) return 0;
    return (uint64_t)((uintptr_t)info.agentBaseAddress + off);
}

// What every run on the copy-engine backend needs before it submits anything: the runtime, one
// validated engine per emulated link (eng, links), one pair of completion signals per piece (plus the
// Gather / Scatter signals of a packing plan), and - decided once per plan - whether kernels can watch
// the signals' value words directly (p->sig_poll).
int engines_prepare(ficco_plan_t *p, bool touches_host, std::vector<int> &eng, int &links)
{
    const int n = p->n_chunks;
    int rc = engines_init(p->device);
    if (rc) return rc;
    EngineCtx &ctx = g_engines;

    // engines: one per emulated link
    links = p->links_opt > 0 ? p->links_opt : p->G;
    links = std::min(links, 16);
    eng = usable_engines(touches_host, links, p->d_status + kFlagStrideWords);
    if (eng.empty()) { if (getenv("FICCO_DEBUG")) fprintf(stderr, "ficco: no usable engine\n"); return FICCO_ERR_HIP; }
    links = std::min(links, (int)eng.size());
    p->links = links;

    // signals, one pair per chunk
    while ((int)p->sig_data.size() < n) {
        hsa_signal_t a, b;
        if (make_signal(&a) != HSA_STATUS_SUCCESS) return FICCO_ERR_ALLOC;
        p->sig_data.push_back(a);
        if (make_signal(&b) != HSA_STATUS_SUCCESS) return FICCO_ERR_ALLOC;
        p->sig_flag.push_back(b);
    }
    if (p->packing) {
        for (auto *v : {&p->sig_gather, &p->sig_scatter})
            while ((int)v->size() < n) {
                hsa_signal_t a;
                if (make_signal(&a) != HSA_STATUS_SUCCESS) return FICCO_ERR_ALLOC;
                v->push_back(a);
            }
    }
    // Can the kernels watch the transfers' own completion signals? The value word of a user signal
    // (amd_signal_t, the layout AQL consumers use) must lie in memory the runtime reports as
    // accessible to this GPU; its device-side address goes into a table. Otherwise, or when asked
    // for (FICCO_OPT_FLAG_WRITE = 2), every transfer is followed by a 4-byte flag copy instead.
    if (p->sig_poll < 0) {
        p->sig_poll = 0;
        // table entries: [0, n) transfers; with packing also [n, 2n) Gather and [2n, 3n) Scatter copies
        const int n_tab = p->packing ? 3 * n : n;
        std::vector<uint64_t> addr(n_tab, 0);
        bool ok = p->flag_write == 0;
        for (int i = 0; i < n_tab && ok; ++i) {
            const hsa_signal_t sg_i = i < n ? p->sig_data[i] : i < 2 * n ? p->sig_gather[i - n] : p->sig_scatter[i - 2 * n];
            addr[i] = signal_value_address(sg_i);
            ok = addr[i] != 0;
        }
        if (ok) {
            if (hipMalloc((void **)&p->d_sig_value, sizeof(uint64_t) * (size_t)n_tab) != hipSuccess) return FICCO_ERR_ALLOC;
            HIP_TRY(hipMemcpy(p->d_sig_value, addr.data(), sizeof(uint64_t) * (size_t)n_tab, hipMemcpyHostToDevice));
            p->sig_poll = 1;
        }
        if (getenv("FICCO_DEBUG")) fprintf(stderr, "ficco: kernels %s\n", p->sig_poll ? "poll the transfers' completion signals" : "wait on flags raised by 4-byte copies");
    }
    return FICCO_OK;
}

// One run of an expert-parallel plan: the grouped kernel is enqueued first and waits per tile for the
// pieces that cover its rows; piece (e, s, j) travels on peer j's link.
int run_grouped(ficco_plan_t *p, const void *A_src, void *A_dev, void *C_dev, hipStream_t cs, bool src_dev)
{
    const int mode = p->mode;
    const bool do_copy = mode != FICCO_MODE_GEMM_ONLY, do_gemm = mode != FICCO_MODE_COPY_ONLY;
    const bool dependent = mode == FICCO_MODE_PAIR;
    const int n = p->n_chunks, G = p->G;
    const bool touches_host = !src_dev;
    std::vector<int> eng;
    int links = 0;
    int rc = engines_prepare(p, touches_host, eng, links);
    if (rc) return rc;
    EngineCtx &ctx = g_engines;
    p->backend = FICCO_COPY_ENGINES;
    const bool poll_signals = p->sig_poll == 1 && !p->hold_flags && !touches_host;
    if (p->run_index > 0) {
        HIP_TRY(hipEventSynchronize(p->ev_end));
        for (int i = 0; i < n; ++i)
            if (!wait_signal(p->sig_data[i], 5.0) || !wait_signal(p->sig_flag[i], 5.0)) return FICCO_ERR_TIMEOUT;
    }
    p->run_index += 1;
    const uint32_t epoch = 1u + (p->run_index - 1u) % (uint32_t)(kEpochSlots - 1);
    const uint64_t spin_ticks = (uint64_t)p->spin_limit_us * (uint64_t)p->wall_clock_khz / 1000u;
    const Gate gate{p->d_flags, poll_signals ? p->d_sig_value : nullptr, epoch, p->d_status, (uint32_t *)p->h_status, spin_ticks};
    for (int i = 0; i < n; ++i) {
        hsa_signal_store_relaxed(p->sig_data[i], (do_copy && p->piece_nrows[i] > 0) ? 1 : 0);
        hsa_signal_store_relaxed(p->sig_flag[i], 0);
    }
    int n_copies = 0, n_launches = 0;
    int64_t copy_bytes = 0;
    HIP_TRY(hipEventRecord(p->ev_begin, cs));          // also the start of the GEMM span on this backend
    if (do_gemm && p->n_row_tiles > 0) {
        GroupedLaunch r{};
        r.g.A = (const uint16_t *)A_dev;
        r.g.Wt = p->d_wt;
        r.g.C = (uint16_t *)C_dev;
        r.g.lda = p->K; r.g.ldc = p->N; r.g.N = (int32_t)p->N; r.g.K = (int32_t)p->K;
        r.g.gate = gate;
        r.row_tiles = p->d_row_tiles;
        r.n_row_tiles = p->n_row_tiles;
        r.ticket = p->d_ticket;
        r.grid = p->resident_grid;
        r.gated = (dependent && do_copy) ? 1 : 0;
        TileShape ts = tile_shape(p->tile);
        const int64_t tn = (p->N + ts.bn - 1) / ts.bn;
        // ragged steps: a step brings about 1/c of the row tiles
        const ListGeometry lg = pick_lists(p, ts, tn, p->n_row_tiles, std::max<int64_t>(1, p->n_row_tiles / std::max(p->c, 1)), r.grid / kTicketLists,
                                           p->M * p->K * 2, (int64_t)p->E * p->N * p->K * 2);
        if (!lg.col_lists) return FICCO_ERR_ARG;
        r.group = lg.group;
        r.col_lists = lg.col_lists;
        for (int x = 0; x < kTicketLists; ++x) {
            r.ticket_base[x] = p->ticket_total[x];
            p->ticket_total[x] += resident_list_draws(resident_list_tiles(p->n_row_tiles, tn, x, r.col_lists), r.grid, x);
        }
        HIP_TRY(launch_grouped(p->tile, r, cs));
        ++n_launches;
    }
    HIP_TRY(hipEventRecord(p->ev_gemm_last, cs));
    if (do_copy && (!dependent || !do_gemm) && !p->hold_flags)
        HIP_TRY(launch_wait_ready(gate, p->d_arrival, n, cs));       // nothing else on the stream consumes the flags
    HIP_TRY(hipEventRecord(p->ev_end, cs));

    const bool chained = p->schedule == FICCO_SHARD || (p->schedule != FICCO_SERIAL && p->order == FICCO_ORDER_SHARD_MAJOR);
    int prev_chunk = -1;
    for (int q = 0; q < n && do_copy; ++q) {
        const int chunk = p->arrival[q];
        const hsa_amd_sdma_engine_id_t engine = (hsa_amd_sdma_engine_id_t)(1u << eng[(chunk % G) % links]);
        const size_t off = (size_t)p->piece_row0[chunk] * p->K * 2, bytes = (size_t)p->piece_nrows[chunk] * p->K * 2;
        hsa_status_t st;
        if (bytes) {
            hsa_signal_t dep{};
            int ndep = 0;
            if (chained && prev_chunk >= 0) { dep = p->sig_data[prev_chunk]; ndep = 1; }
            st = hsa_amd_memory_async_copy_on_engine((char *)A_dev + off, ctx.gpu, (const char *)A_src + off, src_dev ? ctx.gpu : ctx.cpu, bytes,
                                                     ndep, ndep ? &dep : nullptr, p->sig_data[chunk], engine, src_dev);
            if (st != HSA_STATUS_SUCCESS) { g_last_hip = (int)st; return FICCO_ERR_HIP; }
            prev_chunk = chunk;
            ++n_copies;
            copy_bytes += (int64_t)bytes;
        }
        if (!poll_signals && !p->hold_flags) {
            // the flag follows the piece's data; a piece without rows gets its flag at once
            hsa_signal_store_relaxed(p->sig_flag[chunk], 1);
            st = hsa_amd_memory_async_copy_on_engine(p->d_flags + (size_t)chunk * kFlagStrideWords, ctx.gpu, p->h_epochs + epoch, ctx.cpu, 4,
                                                     bytes ? 1 : 0, bytes ? &p->sig_data[chunk] : nullptr, p->sig_flag[chunk], engine, false);
            if (st != HSA_STATUS_SUCCESS) { hsa_signal_store_relaxed(p->sig_flag[chunk], 0); g_last_hip = (int)st; return FICCO_ERR_HIP; }
        }
    }
    p->last_had_copies = n_copies > 0;
    p->last_had_gemm = n_launches > 0;
    p->last_timing = false;
    p->last_copy_bytes = copy_bytes;
    p->last_n_copies = n_copies;
    p->last_n_launches = n_launches;
    p->last_engines = true;
    p->last_lean = false;
    p->last_graph = false;
    p->last_reduce = false;
    p->last_skip_shard = -1;
    return FICCO_OK;
}

int run_engines(ficco_plan_t *p, const void *A_src, void *A_dev, void *C_dev, void *const *peer_out,
                hipStream_t cs, bool src_dev, const std::vector<char> &peer_dev)
{
    const bool rs = p->direction == FICCO_DIR_GEMM_RS;
    const int mode = p->mode;
    const bool do_copy = mode != FICCO_MODE_GEMM_ONLY;
    const bool do_gemm = mode != FICCO_MODE_COPY_ONLY;
    const bool dependent = mode == FICCO_MODE_PAIR;
    const bool timing = p->timing != 0;
    const int n = p->n_chunks, c = p->c;
    // engines: one per emulated link
    bool touches_host = !src_dev;
    if (rs) {
        touches_host = false;
        for (int j = 0; j < p->G; ++j) touches_host |= !peer_dev[j];
    }
    std::vector<int> eng;
    int links = 0;
    int rc = engines_prepare(p, touches_host, eng, links);
    if (rc) return rc;
    EngineCtx &ctx = g_engines;
    const bool packed = p->packing && dependent && do_copy && do_gemm && !rs;
    // Signals live in host memory: when the transfers themselves cross the host link, hundreds of
    // polling workgroups would compete with them for it, so flags in device memory are used then.
    const bool poll_signals = p->sig_poll == 1 && !p->hold_flags && !touches_host;
    if (packed && p->sig_poll != 1) return FICCO_ERR_HIP;    // the packed launches watch the Gather copies' signals
    // the previous run must be over before its buffers, flags and signals are reused
    if (p->run_index > 0) {
        HIP_TRY(hipEventSynchronize(p->ev_end));
        for (int i = 0; i < n; ++i)
            if (!wait_signal(p->sig_data[i], 5.0) || !wait_signal(p->sig_flag[i], 5.0)) return FICCO_ERR_TIMEOUT;
        for (auto *v : {&p->sig_gather, &p->sig_scatter})
            for (auto &sg : *v)
                if (!wait_signal(sg, 5.0)) return FICCO_ERR_TIMEOUT;
    }
    if (timing) {
        if ((rc = make_events(p->ev_gemm_b, p->groups.size()))) return rc;
        if ((rc = make_events(p->ev_gemm_e, p->groups.size()))) return rc;
    }
    p->run_index += 1;
    const uint32_t epoch = 1u + (p->run_index - 1u) % (uint32_t)(kEpochSlots - 1);
    const uint64_t spin_ticks = (uint64_t)p->spin_limit_us * (uint64_t)p->wall_clock_khz / 1000u;
    const size_t row_bytes_a = (size_t)p->K * 2, row_bytes_c = (size_t)p->N * 2;
    auto is_local = [&](int chunk) { return !rs && p->local_shard >= 0 && shard_of(p, chunk) == p->local_shard; };
    // transfers are chained one after the other (peer-to-peer pattern) or run side by side (all-to-all)
    const bool chained = p->schedule == FICCO_SHARD ||
                         (p->schedule != FICCO_SERIAL && p->order == FICCO_ORDER_SHARD_MAJOR);
    const Gate gate{p->d_flags, poll_signals ? p->d_sig_value : nullptr, epoch, p->d_status, (uint32_t *)p->h_status, spin_ticks};
    // arm the signals before any kernel that watches them can start
    for (int i = 0; i < n; ++i) {
        hsa_signal_store_relaxed(p->sig_data[i], (do_copy && !is_local(i)) ? 1 : 0);
        hsa_signal_store_relaxed(p->sig_flag[i], 0);
        if (p->packing) {
            hsa_signal_store_relaxed(p->sig_gather[i], packed ? 1 : 0);
            hsa_signal_store_relaxed(p->sig_scatter[i], packed ? 1 : 0);
        }
    }

    // Chained plans (ficco_plan_chain). Behind another plan: every transfer of this run also waits for the
    // signal that plan's latest run releases when it ends. In front of others: this run arms one of its
    // two signals now and releases it from the compute stream when everything it enqueues there is done;
    // a run that fails half-way releases it from the host, so that nothing stays parked behind it.
    hsa_signal_t chain_dep{};
    bool has_chain_dep = false;
    if (rs && p->chain_from) return FICCO_ERR_ARG;       // defined for the transfers into A_dev only
    if (p->chain_from && p->chain_from->alive && p->chain_from->made && p->chain_from->last >= 0) {
        chain_dep = p->chain_from->free_sig[p->chain_from->last];
        has_chain_dep = true;
    }
    struct Disarm {
        hsa_signal_t sg{};
        bool on = false;
        ~Disarm() { if (on) hsa_signal_store_screlease(sg, 0); }
    } disarm;
    uint64_t release_addr = 0;
    if (p->link) {
        ChainLink &L = *p->link;
        if (!L.made) {
            for (int i = 0; i < 2; ++i) {
                if (make_signal(&L.free_sig[i]) != HSA_STATUS_SUCCESS) {
                    if (i) (void)hsa_signal_destroy(L.free_sig[0]);
                    return FICCO_ERR_ALLOC;
                }
            }
            L.made = true;
            for (int i = 0; i < 2; ++i)
                if (!(L.addr[i] = signal_value_address(L.free_sig[i]))) return FICCO_ERR_HIP;   // needs signals the GPU can write
        }
        if (!L.addr[0] || !L.addr[1]) return FICCO_ERR_HIP;
        const int idx = (L.last + 1) & 1;
        hsa_signal_store_relaxed(L.free_sig[idx], 1);
        L.last = idx;
        disarm.sg = L.free_sig[idx];
        disarm.on = true;
        release_addr = L.addr[idx];
    }

    int n_copies = 0, n_launches = 0;
    int64_t copy_bytes = 0;
    // one piece: data copy, then the 4-byte flag copy behind it on the same engine
    int prev_chunk = -1;
    std::vector<hsa_signal_t> *extra_dep = nullptr;      // per chunk id: one more signal every transfer waits for
    auto submit = [&](int q) -> int {
        const int chunk = p->arrival[q];
        if (is_local(chunk)) return FICCO_OK;
        const int lane = shard_of(p, chunk) % links;
        const hsa_amd_sdma_engine_id_t engine = (hsa_amd_sdma_engine_id_t)(1u << eng[lane]);
        void *dst;
        const void *src;
        size_t bytes;
        hsa_agent_t dst_agent = ctx.gpu, src_agent = ctx.gpu;
        bool force = true;
        if (!rs) {
            const Extent ex = piece_extent(p, chunk);
            bytes = ex.bytes;
            dst = (char *)A_dev + ex.off;
            src = (const char *)A_src + ex.off;
            if (!src_dev) { src_agent = ctx.cpu; force = false; }
        } else {
            const int peer = chunk / c;
            bytes = (size_t)p->m * row_bytes_c;
            src = (const char *)C_dev + (size_t)chunk * p->m * row_bytes_c;
            dst = (char *)peer_out[peer] + (size_t)(chunk % c) * p->m * row_bytes_c;
            if (!peer_dev[peer]) { dst_agent = ctx.cpu; force = false; }
        }
        hsa_signal_t dep[3];
        int ndep = 0;
        if (chained && prev_chunk >= 0) dep[ndep++] = p->sig_data[prev_chunk];
        if (extra_dep) dep[ndep++] = (*extra_dep)[chunk];
        if (has_chain_dep) dep[ndep++] = chain_dep;
        hsa_status_t st = hsa_amd_memory_async_copy_on_engine(dst, dst_agent, src, src_agent, bytes, ndep, ndep ? dep : nullptr,
                                                              p->sig_data[chunk], engine, force);
        if (st != HSA_STATUS_SUCCESS) { g_last_hip = (int)st; return FICCO_ERR_HIP; }
        prev_chunk = chunk;
        ++n_copies;
        copy_bytes += (int64_t)bytes;
        if (!poll_signals && !p->hold_flags && !packed) {
            hsa_signal_store_relaxed(p->sig_flag[chunk], 1);
            uint32_t *flag = p->d_flags + (size_t)chunk * kFlagStrideWords;
            st = hsa_amd_memory_async_copy_on_engine(flag, ctx.gpu, p->h_epochs + epoch, ctx.cpu, 4, 1, &p->sig_data[chunk],
                                                     p->sig_flag[chunk], engine, false);
            if (st != HSA_STATUS_SUCCESS) { hsa_signal_store_relaxed(p->sig_flag[chunk], 0); g_last_hip = (int)st; return FICCO_ERR_HIP; }
        }
        return FICCO_OK;
    };
    auto launch_group = [&](size_t g, bool gated) -> int {
        GemmLaunch a = make_launch(p, p->groups[g], A_dev, C_dev);
        if (gated) {
            // wait list = the group's pieces that arrive by transfer (arrival table slice)
            int first = p->groups[g].pos_begin, last = p->groups[g].pos_end;
            while (first < last && is_local(p->arrival[first])) ++first;     // local pieces sit at the front
            a.gate = gate;
            a.wait_chunks = p->d_arrival + first;
            a.n_wait = last - first;
            for (int q = first; q < last; ++q)
                if (is_local(p->arrival[q])) return FICCO_ERR_ARG;           // cannot happen: stable partition
        }
        if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_b[g], cs));
        HIP_TRY(launch_gemm(p->tile, a, cs));
        if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_e[g], cs));
        ++n_launches;
        return FICCO_OK;
    };

    // Every event record is a packet of its own on the stream and costs the device a microsecond or two, which
    // counts when steps follow each other without gaps: the begin event doubles as the start of the GEMM
    // span, and a run that is one resident launch and nothing else (all-gather pair) ends its span with the
    // end event.
    const bool span_is_run = !rs && !packed && is_resident(p) && do_gemm && dependent && !timing;
    // ... and in such a run the kernel itself lets the transfers of a plan chained behind this one go (its last
    // workgroup out); otherwise a one-thread kernel at the end of the run does
    const bool release_in_kernel = release_addr != 0 && span_is_run;
    HIP_TRY(hipEventRecord(p->ev_begin, cs));
    if (packed) {
        // ---- the fused schedule as the paper runs it with an unmodified GEMM (Sec. V-A): the G pieces of a
        // step are gathered by DMA into one contiguous input, multiplied into one contiguous output,
        // and the G output blocks are scattered by DMA to their rows of C.
        if (!p->d_pack_a && hipMalloc((void **)&p->d_pack_a, (size_t)p->M * p->K * 2) != hipSuccess) return FICCO_ERR_ALLOC;
        if (!p->d_pack_c && hipMalloc((void **)&p->d_pack_c, (size_t)p->M * p->N * 2) != hipSuccess) return FICCO_ERR_ALLOC;
        // Gather and Scatter run on engines of their own where the machine has spare ones
        std::vector<int> geng = usable_engines(false, 16, p->d_status + kFlagStrideWords);
        if (geng.empty()) return FICCO_ERR_HIP;
        auto aux_engine = [&](int chunk) {
            const int spare = (int)geng.size() > links ? (int)geng.size() - links : 0;
            const int lane = shard_of(p, chunk);
            const int e = spare ? geng[links + lane % spare] : geng[lane % (int)geng.size()];
            return (hsa_amd_sdma_engine_id_t)(1u << e);
        };
        // The launches watch the Gather copies' completion signals, or, when the transfers cross the host
        // link (where polling host memory would compete with them), flags raised by a 4-byte copy
        // behind each Gather copy. The final wait for the Scatter copies is a single wavefront.
        const Gate pgate{p->d_flags, p->d_sig_value, epoch, p->d_status, (uint32_t *)p->h_status, spin_ticks};
        const Gate ggate = poll_signals ? pgate : gate;
        const size_t piece_a = (size_t)p->m * row_bytes_a, piece_c = (size_t)p->m * row_bytes_c;
        for (size_t g = 0; g < p->groups.size(); ++g) {
            const Group &gr = p->groups[g];
            GemmLaunch a{};
            a.A = p->d_pack_a;
            a.Wt = p->d_wt;
            a.C = p->d_pack_c;
            a.lda = p->K; a.ldc = p->N; a.N = (int32_t)p->N; a.K = (int32_t)p->K;
            a.block_row0 = nullptr;
            a.row0 = (int32_t)((int64_t)gr.pos_begin * p->m);
            a.n_blocks = 1;
            a.rows_per_block = (int32_t)((int64_t)(gr.pos_end - gr.pos_begin) * p->m);
            a.gate = ggate;
            a.wait_chunks = (poll_signals ? p->d_gather_idx : p->d_arrival) + gr.pos_begin;
            a.n_wait = gr.pos_end - gr.pos_begin;
            if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_b[g], cs));
            HIP_TRY(launch_gemm(p->tile, a, cs));
            if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_e[g], cs));
            HIP_TRY(hipEventRecord(p->ev_dep[g], cs));
            ++n_launches;
        }
        HIP_TRY(hipEventRecord(p->ev_gemm_last, cs));
        // the run's last stage on the compute stream: wait (bounded) for every Scatter copy
        HIP_TRY(launch_wait_ready(pgate, p->d_scatter_idx, n, cs));
        for (int q = 0; q < n; ++q) {
            const int chunk = p->arrival[q];
            if ((rc = submit(q))) return rc;
            // Gather: the piece's rows of A_dev -> position q of the packed input, behind its transfer
            hsa_signal_t dep = p->sig_data[chunk];
            const bool has_dep = !is_local(chunk);
            hsa_status_t st = hsa_amd_memory_async_copy_on_engine((char *)p->d_pack_a + (size_t)q * piece_a, ctx.gpu,
                                                                  (const char *)A_dev + (size_t)chunk * piece_a, ctx.gpu, piece_a,
                                                                  has_dep ? 1 : 0, has_dep ? &dep : nullptr, p->sig_gather[chunk],
                                                                  aux_engine(chunk), true);
            if (st != HSA_STATUS_SUCCESS) { g_last_hip = (int)st; return FICCO_ERR_HIP; }
            ++n_copies;
            copy_bytes += (int64_t)piece_a;
            if (!poll_signals) {
                hsa_signal_store_relaxed(p->sig_flag[chunk], 1);
                st = hsa_amd_memory_async_copy_on_engine(p->d_flags + (size_t)chunk * kFlagStrideWords, ctx.gpu, p->h_epochs + epoch, ctx.cpu, 4,
                                                         1, &p->sig_gather[chunk], p->sig_flag[chunk], aux_engine(chunk), false);
                if (st != HSA_STATUS_SUCCESS) { hsa_signal_store_relaxed(p->sig_flag[chunk], 0); g_last_hip = (int)st; return FICCO_ERR_HIP; }
            }
        }
        // Scatter: a launch's output blocks leave when the launch is done (the host relays the event:
        // a copy engine cannot wait on it)
        for (size_t g = 0; g < p->groups.size(); ++g) {
            HIP_TRY(hipEventSynchronize(p->ev_dep[g]));
            for (int q = p->groups[g].pos_begin; q < p->groups[g].pos_end; ++q) {
                const int chunk = p->arrival[q];
                hsa_status_t st = hsa_amd_memory_async_copy_on_engine((char *)C_dev + (size_t)chunk * piece_c, ctx.gpu,
                                                                      (const char *)p->d_pack_c + (size_t)q * piece_c, ctx.gpu, piece_c,
                                                                      0, nullptr, p->sig_scatter[chunk], aux_engine(chunk), true);
                if (st != HSA_STATUS_SUCCESS) { g_last_hip = (int)st; return FICCO_ERR_HIP; }
                ++n_copies;
                copy_bytes += (int64_t)piece_c;
            }
        }
    } else if (!rs) {
        // ---- The kernels wait on flags or signals inside, so the order of the two sides is free. Short runs
        // enqueue the GEMM side first so that it is resident before data lands; long ones (a MiB or more per
        // link) start the engines first and enqueue the launches while the first pieces are on their way,
        // which takes the launch latency off the critical path.
        const bool copies_first = do_copy && do_gemm && (size_t)p->M * row_bytes_a / (size_t)std::max(links, 1) >= ((size_t)1 << 20);
        if (copies_first)
            for (int q = 0; q < n; ++q)
                if ((rc = submit(q))) return rc;
        if (do_gemm) {
            if (is_2d(p)) {
                if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_b[0], cs));
                if ((rc = launch_2d(p, gate, dependent, p->resident_grid, A_dev, C_dev, cs, release_in_kernel ? release_addr : 0))) return rc;
                if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_e[0], cs));
                ++n_launches;
            } else if (p->schedule == FICCO_FINE_PERSISTENT) {
                ResidentLaunch r{};
                if (release_in_kernel)
                    r.leave = RunExit{p->d_ticket_mem + (size_t)kTicketLists * kFlagStrideWords, p->exit_total + (uint32_t)p->resident_grid,
                                      reinterpret_cast<int64_t *>(release_addr)};
                Group all{0, n};
                r.g = make_launch(p, all, A_dev, C_dev);
                r.g.block_row0 = nullptr; r.g.row0 = 0; r.g.n_blocks = n; r.g.rows_per_block = (int32_t)p->m;
                r.arrival = p->d_arrival;
                r.n_chunks = n;
                r.g.gate = gate;
                r.ticket = p->d_ticket;
                r.grid = p->resident_grid;
                const ListGeometry lg = resident_lists(p);
                if (!lg.col_lists) return FICCO_ERR_ARG;
                r.group = lg.group;
                r.col_lists = lg.col_lists;
                if (!dependent) { r.local_chunk_begin = 0; r.local_chunk_end = n; }
                else if (p->local_shard >= 0) { r.local_chunk_begin = p->local_shard * c; r.local_chunk_end = (p->local_shard + 1) * c; }
                TileShape ts = tile_shape(p->tile);
                for (int x = 0; x < kTicketLists; ++x) {
                    r.ticket_base[x] = p->ticket_total[x];
                    p->ticket_total[x] += resident_list_draws(resident_list_tiles((int64_t)n * ((p->m + ts.bm - 1) / ts.bm),
                                                                                  (p->N + ts.bn - 1) / ts.bn, x, r.col_lists), r.grid, x);
                }
                if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_b[0], cs));
                HIP_TRY(launch_resident(p->tile, r, cs));
                if (release_in_kernel) p->exit_total += (uint32_t)p->resident_grid;
                if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_e[0], cs));
                ++n_launches;
            } else {
                for (size_t g = 0; g < p->groups.size(); ++g)
                    if ((rc = launch_group(g, dependent))) return rc;
            }
            if (!span_is_run) HIP_TRY(hipEventRecord(p->ev_gemm_last, cs));
        }
        if (do_copy) {
            for (int q = 0; q < n && !copies_first; ++q)
                if ((rc = submit(q))) return rc;
            if ((!dependent || !do_gemm) && !p->hold_flags) {
                // nothing on the compute stream consumes the flags: join through a small waiting kernel
                int first = 0;
                while (first < n && is_local(p->arrival[first])) ++first;
                if (first < n)
                    HIP_TRY(launch_wait_ready(gate, p->d_arrival + first, n - first, cs));
            }
        }
    } else if (p->schedule == FICCO_FINE_PERSISTENT) {
        // ---- GEMM -> RS with one resident kernel and no host in the loop: every transfer is submitted up
        // front with a dependency signal of its own; the kernel counts the tiles of each piece and the
        // one that completes a piece stores 0 into that signal's value word, which lets the copy go.
        if (!(do_gemm && do_copy && dependent)) return FICCO_ERR_ARG;        // the pair only
        while ((int)p->sig_done.size() < n) {
            hsa_signal_t a;
            if (make_signal(&a) != HSA_STATUS_SUCCESS) return FICCO_ERR_ALLOC;
            p->sig_done.push_back(a);
        }
        if (!p->d_done_value) {
            std::vector<uint64_t> addr(n);
            for (int i = 0; i < n; ++i)
                if (!(addr[i] = signal_value_address(p->sig_done[i]))) return FICCO_ERR_HIP;   // needs signals the GPU can write
            if (hipMalloc((void **)&p->d_done_value, sizeof(uint64_t) * (size_t)n) != hipSuccess) return FICCO_ERR_ALLOC;
            HIP_TRY(hipMemcpy(p->d_done_value, addr.data(), sizeof(uint64_t) * (size_t)n, hipMemcpyHostToDevice));
            if (hipMalloc((void **)&p->d_done_count, sizeof(uint32_t) * (size_t)n) != hipSuccess) return FICCO_ERR_ALLOC;
            HIP_TRY(hipMemset(p->d_done_count, 0, sizeof(uint32_t) * (size_t)n));
        }
        for (int i = 0; i < n; ++i) hsa_signal_store_relaxed(p->sig_done[i], 1);
        // transfers first (they wait for their pieces), then the launch
        extra_dep = &p->sig_done;
        for (int q = 0; q < n; ++q)
            if ((rc = submit(q))) return rc;
        extra_dep = nullptr;
        {
            ResidentLaunch r{};
            Group all{0, n};
            r.g = make_launch(p, all, A_dev, C_dev);
            r.g.block_row0 = nullptr; r.g.row0 = 0; r.g.n_blocks = n; r.g.rows_per_block = (int32_t)p->m;
            r.arrival = p->d_arrival;
            r.n_chunks = n;
            r.g.gate = gate;
            r.ticket = p->d_ticket;
            r.grid = p->resident_grid;
            const ListGeometry lg = resident_lists(p);
            if (!lg.col_lists) return FICCO_ERR_ARG;
            r.group = lg.group;
            r.col_lists = lg.col_lists;
            r.local_chunk_begin = 0; r.local_chunk_end = n;                   // A is resident: nothing to wait for
            TileShape ts = tile_shape(p->tile);
            const int64_t rt = (p->m + ts.bm - 1) / ts.bm, tn = (p->N + ts.bn - 1) / ts.bn;
            r.done_count = p->d_done_count;
            r.done_sig = p->d_done_value;
            r.tiles_per_chunk = (int32_t)(rt * tn);
            for (int x = 0; x < kTicketLists; ++x) {
                r.ticket_base[x] = p->ticket_total[x];
                p->ticket_total[x] += resident_list_draws(resident_list_tiles((int64_t)n * rt, tn, x, r.col_lists), r.grid, x);
            }
            HIP_TRY(launch_resident(p->tile, r, cs));
            ++n_launches;
        }
        HIP_TRY(hipEventRecord(p->ev_gemm_last, cs));
        if (!p->hold_flags) HIP_TRY(launch_wait_ready(gate, p->d_arrival, n, cs));
    } else {
        // ---- GEMM -> RS: a group's rows leave when its launch is done (the host relays the event)
        if (do_gemm) {
            for (size_t g = 0; g < p->groups.size(); ++g) {
                if ((rc = launch_group(g, false))) return rc;
                HIP_TRY(hipEventRecord(p->ev_dep[g], cs));
            }
            HIP_TRY(hipEventRecord(p->ev_gemm_last, cs));
        }
        if (do_copy) {
            for (size_t g = 0; g < p->groups.size(); ++g) {
                if (do_gemm && dependent) HIP_TRY(hipEventSynchronize(p->ev_dep[g]));
                for (int q = p->groups[g].pos_begin; q < p->groups[g].pos_end; ++q)
                    if ((rc = submit(q))) return rc;
            }
            if (!p->hold_flags) HIP_TRY(launch_wait_ready(gate, p->d_arrival, n, cs));
        }
    }
    if (release_addr) {
        if (!release_in_kernel) HIP_TRY(launch_release_signal(release_addr, cs));
        disarm.on = false;                               // the stream releases it from here on
    }
    HIP_TRY(hipEventRecord(p->ev_end, cs));

    p->last_had_copies = n_copies > 0;
    p->last_had_gemm = n_launches > 0;
    p->last_timing = timing;
    p->last_copy_bytes = copy_bytes;
    p->last_n_copies = n_copies;
    p->last_n_launches = n_launches;
    p->last_engines = true;
    p->last_lean = span_is_run;
    p->last_graph = false;
    p->last_skip_shard = rs ? -1 : p->local_shard;
    p->last_reduce = false;
    return FICCO_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" {

int ficco_static_descriptors(int64_t m, int64_t N, int64_t K, double *otb, double *mt_bytes)
{
    if (m < 0 || N < 0 || K < 0) return FICCO_ERR_ARG;
    const double bytes = 2.0 * ((double)m * K + (double)N * K + (double)m * N);
    if (mt_bytes) *mt_bytes = bytes;
    if (otb) *otb = bytes > 0 ? 2.0 * (double)m * (double)N * (double)K / bytes : 0.0;
    return FICCO_OK;
}

double ficco_ideal_overlap_us(double t_comm_us, double t_gemm_us, int n)
{
    if (n < 1) n = 1;
    // piece q's GEMM starts when its transfer has landed and the previous GEMM has finished
    double copy_done = 0, gemm_done = 0;
    for (int q = 0; q < n; ++q) {
        copy_done += t_comm_us / n;
        gemm_done = std::max(gemm_done, copy_done) + t_gemm_us / n;
    }
    return gemm_done;
}

int ficco_pick_schedule(int64_t M, int64_t K, int64_t N, int shards, int *schedule, int *chunks)
{
    if (M < 1 || K < 1 || N < 1 || shards < 1 || !schedule || !chunks) return FICCO_ERR_ARG;
    if (M % shards) return FICCO_ERR_SHAPE;
    // Static rule in the spirit of Sec. V-C: decomposition loss grows as the decomposed GEMM's combined
    // op-to-byte and memory-traffic metric (their product = its flop count) falls, so a shard is cut
    // into as many pieces as keep one piece's GEMM above a machine threshold (fitted on MI355X with
    // the sweep tool: 2.5e10 flop, piece rows a power of two, at least 256 rows, at most 16 pieces).
    // Among the schedules the resident kernel was the fastest at every point of the sweep, so the
    // schedule itself needs no threshold here.
    const int64_t ms = M / shards;
    const double kPieceFlops = 2.5e10;
    const double t = kPieceFlops / (2.0 * (double)N * (double)K);
    int64_t m = 1;
    while ((double)(m * 2) <= t && m < (int64_t)1 << 40) m *= 2;
    m = std::max<int64_t>(256, std::min(m, ms));
    int c = (int)std::max<int64_t>(1, std::min<int64_t>(16, ms / m));
    while (c > 1 && ms % c) c /= 2;
    const int sch = FICCO_FINE_PERSISTENT;
    *schedule = sch;
    *chunks = c;
    return FICCO_OK;
}

int ficco_plan(int64_t M, int64_t K, int64_t N, int shards, int chunks, int schedule, ficco_plan_t **out)
{
    if (!out) return FICCO_ERR_ARG;
    if (M < 1 || K < 1 || N < 1 || shards < 1) return FICCO_ERR_SHAPE;
    if (schedule == FICCO_AUTO) {
        int rc = ficco_pick_schedule(M, K, N, shards, &schedule, &chunks);
        if (rc) return rc;
    }
    if (schedule < FICCO_SERIAL || schedule > FICCO_FINE_2D) return FICCO_ERR_ARG;
    if (chunks < 1) return FICCO_ERR_SHAPE;
    if ((schedule == FICCO_SERIAL || schedule == FICCO_SHARD) && chunks != 1) return FICCO_ERR_SHAPE;
    if ((int64_t)shards * chunks > 4096) return FICCO_ERR_SHAPE;
    if (schedule == FICCO_FINE_2D) {
        // column pieces: every shard keeps its rows, k is cut into `chunks` slices of whole k-tiles
        if (M % shards || K % kBK || chunks > K / kBK) return FICCO_ERR_SHAPE;
    } else if (M % ((int64_t)shards * chunks)) {
        return FICCO_ERR_SHAPE;
    }
    if (K % 64 || N % 8) return FICCO_ERR_SHAPE;
    if (M > 0x7FFFFFFF || N > 0x7FFFFFFF || K > 0x7FFFFFFF) return FICCO_ERR_SHAPE;
    ficco_plan_t *p = new (std::nothrow) ficco_plan_t();
    if (!p) return FICCO_ERR_ALLOC;
    p->M = M; p->K = K; p->N = N; p->G = shards; p->c = chunks; p->schedule = schedule;
    p->device = -1;                      // bound to the current device on first use
    p->order = (schedule == FICCO_SERIAL || schedule == FICCO_SHARD) ? FICCO_ORDER_SHARD_MAJOR : FICCO_ORDER_STEP_MAJOR;
    int rc = build_lists(p);
    if (rc) { delete p; return rc; }
    *out = p;
    return FICCO_OK;
}

int ficco_plan_grouped(int64_t K, int64_t N, int peers, int experts, const int64_t *rows, int chunks, int schedule,
                       ficco_plan_t **out)
{
    if (!out || !rows) return FICCO_ERR_ARG;
    if (K < 1 || N < 1 || peers < 1 || experts < 1 || chunks < 1) return FICCO_ERR_SHAPE;
    if (schedule != FICCO_SERIAL && schedule != FICCO_SHARD && schedule != FICCO_FINE_PERSISTENT) return FICCO_ERR_ARG;
    if ((schedule == FICCO_SERIAL || schedule == FICCO_SHARD) && chunks != 1) return FICCO_ERR_SHAPE;
    if ((int64_t)peers * experts * chunks > 4096) return FICCO_ERR_SHAPE;
    if (K % 64 || N % 8 || K > 0x7FFFFFFF || N > 0x7FFFFFFF) return FICCO_ERR_SHAPE;
    int64_t M = 0;
    for (int i = 0; i < peers * experts; ++i) {
        if (rows[i] < 0) return FICCO_ERR_SHAPE;
        M += rows[i];
    }
    if (M < 1 || M > 0x7FFFFFFF) return FICCO_ERR_SHAPE;
    ficco_plan_t *p = new (std::nothrow) ficco_plan_t();
    if (!p) return FICCO_ERR_ALLOC;
    p->M = M; p->K = K; p->N = N; p->G = peers; p->E = experts; p->c = chunks; p->schedule = schedule;
    p->grouped = true;
    p->token_rows.assign(rows, rows + (size_t)peers * experts);
    p->device = -1;
    p->order = schedule == FICCO_SHARD ? FICCO_ORDER_SHARD_MAJOR : FICCO_ORDER_STEP_MAJOR;
    int rc = build_lists(p);
    if (rc) { delete p; return rc; }
    *out = p;
    return FICCO_OK;
}

int ficco_plan_pieces(const ficco_plan_t *p, int64_t *row0, int64_t *rows, int cap)
{
    if (!p || cap < p->n_chunks) return FICCO_ERR_ARG;
    for (int i = 0; i < p->n_chunks; ++i) {
        const int64_t r0 = p->grouped ? p->piece_row0[i] : (is_2d(p) ? (int64_t)(i % p->G) * p->m : (int64_t)i * p->m);
        const int64_t nr = p->grouped ? p->piece_nrows[i] : p->m;
        if (row0) row0[i] = r0;
        if (rows) rows[i] = nr;
    }
    return FICCO_OK;
}

int ficco_plan_chain(ficco_plan_t *p, ficco_plan_t *after)
{
    if (!p || p == after || p->grouped || (after && after->grouped)) return FICCO_ERR_ARG;
    if (!after) {
        p->chain_from.reset();
        return FICCO_OK;
    }
    if (!after->link) {
        after->link = std::shared_ptr<ChainLink>(new (std::nothrow) ChainLink());
        if (!after->link) return FICCO_ERR_ALLOC;
    }
    p->chain_from = after->link;
    return FICCO_OK;
}

int ficco_plan_set_slice_widths(ficco_plan_t *p, const int64_t *widths, int n)
{
    if (!p || !is_2d(p)) return FICCO_ERR_ARG;
    if (p->finalized) return FICCO_ERR_STATE;
    if (!widths) {
        p->own_widths = false;
        return build_lists(p);
    }
    if (n != p->c) return FICCO_ERR_SHAPE;
    std::vector<int64_t> k0((size_t)n + 1, 0);
    for (int sl = 0; sl < n; ++sl) {
        if (widths[sl] < kBK || widths[sl] % kBK || widths[sl] > p->K) return FICCO_ERR_SHAPE;
        k0[sl + 1] = k0[sl] + widths[sl];
    }
    if (k0[n] != p->K) return FICCO_ERR_SHAPE;
    p->slice_k0 = k0;
    p->own_widths = true;
    return build_lists(p);
}

int ficco_plan_slices(const ficco_plan_t *p, int64_t *k0, int64_t *widths, int cap)
{
    if (!p || !is_2d(p) || cap < p->c) return FICCO_ERR_ARG;
    for (int sl = 0; sl < p->c; ++sl) {
        if (k0) k0[sl] = p->slice_k0[sl];
        if (widths) widths[sl] = p->slice_k0[sl + 1] - p->slice_k0[sl];
    }
    return FICCO_OK;
}

int ficco_plan_set(ficco_plan_t *p, int option, int64_t value)
{
    if (!p) return FICCO_ERR_ARG;
    if (p->grouped && (option == FICCO_OPT_DIRECTION || option == FICCO_OPT_LOCAL_SHARD || option == FICCO_OPT_PACKING ||
                       option == FICCO_OPT_TIMING) && value != (option == FICCO_OPT_LOCAL_SHARD ? -1 : 0))
        return FICCO_ERR_ARG;          // expert-parallel plans: all-gather direction, every piece travels, no per-launch timing
    const bool late_ok = option == FICCO_OPT_MODE || option == FICCO_OPT_TIMING || option == FICCO_OPT_HOLD_FLAGS ||
                         option == FICCO_OPT_SPIN_LIMIT_US || option == FICCO_OPT_REPEAT || option == FICCO_OPT_TILE_GROUP ||
                         option == FICCO_OPT_TILE_COLUMN_LISTS;
    if (p->finalized && !late_ok) return FICCO_ERR_STATE;
    switch (option) {
    case FICCO_OPT_DIRECTION:
        if (value != FICCO_DIR_AG_GEMM && value != FICCO_DIR_GEMM_RS) return FICCO_ERR_ARG;
        if (value == FICCO_DIR_GEMM_RS && is_2d(p)) return FICCO_ERR_ARG;
        p->direction = (int)value;
        break;
    case FICCO_OPT_ORDER:
        if (value != FICCO_ORDER_STEP_MAJOR && value != FICCO_ORDER_SHARD_MAJOR) return FICCO_ERR_ARG;
        if (p->schedule == FICCO_SERIAL || p->schedule == FICCO_SHARD) value = FICCO_ORDER_SHARD_MAJOR;
        p->order = (int)value;
        break;
    case FICCO_OPT_MODE:
        if (value < FICCO_MODE_PAIR || value > FICCO_MODE_INDEPENDENT) return FICCO_ERR_ARG;
        p->mode = (int)value;
        break;
    case FICCO_OPT_TIMING:
        if (value != 0 && value != 1) return FICCO_ERR_ARG;
        p->timing = (int)value;
        break;
    case FICCO_OPT_TILE:
        if (value != 0 && tile_shape((int)value).bm == 0) return FICCO_ERR_ARG;
        p->tile_opt = (int)value;
        break;
    case FICCO_OPT_FLAG_WRITE:
        if (value < 0 || value > 2) return FICCO_ERR_ARG;
        p->flag_write = (int)value;
        break;
    case FICCO_OPT_SPIN_LIMIT_US:
        if (value < 1 || value > 60000000) return FICCO_ERR_ARG;
        p->spin_limit_us = value;
        break;
    case FICCO_OPT_LOCAL_SHARD:
        if (value < -1 || value >= p->G) return FICCO_ERR_ARG;
        if (value >= 0 && is_2d(p)) return FICCO_ERR_ARG;
        p->local_shard = (int)value;
        break;
    case FICCO_OPT_HOLD_FLAGS:
        if (value != 0 && value != 1) return FICCO_ERR_ARG;
        p->hold_flags = (int)value;
        break;
    case FICCO_OPT_COPY_BACKEND:
        if (value < FICCO_COPY_AUTO || value > FICCO_COPY_ENGINES) return FICCO_ERR_ARG;
        p->backend_opt = (int)value;
        break;
    case FICCO_OPT_LINKS:
        if (value < 0 || value > 16) return FICCO_ERR_ARG;
        p->links_opt = (int)value;
        break;
    case FICCO_OPT_REPEAT:
        if (value < 1 || value > 10000) return FICCO_ERR_ARG;
        p->repeat = (int)value;
        break;
    case FICCO_OPT_TILE_GROUP:
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return FICCO_ERR_ARG;
        p->tile_group = (int)value;
        break;
    case FICCO_OPT_TILE_COLUMN_LISTS:
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return FICCO_ERR_ARG;
        p->tile_col_lists = (int)value;
        break;
    case FICCO_OPT_PACKING:
        if (value != 0 && value != 1) return FICCO_ERR_ARG;
        if (value == 1 && p->schedule != FICCO_FINE_FUSED) return FICCO_ERR_ARG;
        p->packing = (int)value;
        break;
    default:
        return FICCO_ERR_ARG;
    }
    if (!p->finalized) return build_lists(p);
    return FICCO_OK;
}

int ficco_plan_set_arrival(ficco_plan_t *p, const int32_t *chunk_ids, int n)
{
    if (!p || !chunk_ids) return FICCO_ERR_ARG;
    if (p->finalized) return FICCO_ERR_STATE;
    if (n != p->n_chunks) return FICCO_ERR_ARG;
    std::vector<char> seen(n, 0);
    for (int q = 0; q < n; ++q) {
        if (chunk_ids[q] < 0 || chunk_ids[q] >= n || seen[chunk_ids[q]]) return FICCO_ERR_ARG;
        seen[chunk_ids[q]] = 1;
    }
    p->arrival.assign(chunk_ids, chunk_ids + n);
    p->order = FICCO_ORDER_CUSTOM;
    return build_lists(p);
}

int ficco_plan_info(const ficco_plan_t *p, ficco_plan_info_t *out)
{
    if (!p || !out) return FICCO_ERR_ARG;
    ficco_plan_info_t o{};
    o.M = p->M; o.K = p->K; o.N = p->N;
    o.shards = p->G; o.chunks = p->c;
    o.schedule = p->schedule; o.direction = p->direction; o.order = p->order; o.mode = p->mode;
    o.n_chunks = p->n_chunks;
    o.n_groups = (int32_t)p->groups.size();
    o.chunk_rows = p->m;
    TileShape ts = tile_shape(p->tile);
    o.tile_m = ts.bm; o.tile_n = ts.bn; o.tile_k = p->tile ? kBK : 0;
    o.resident_grid = p->resident_grid;
    o.copy_backend = p->backend;
    o.links = p->links;
    // descriptors of one launch: the resident kernel's unit of work is one piece
    int64_t rows = is_resident(p) ? p->m
                                  : (int64_t)(p->groups[0].pos_end - p->groups[0].pos_begin) * p->m;
    if (p->grouped) rows = p->M / p->n_chunks;      // descriptors of an average piece
    ficco_static_descriptors(rows, p->N, is_2d(p) ? p->K / p->c : p->K, &o.otb, &o.mt_bytes);
    *out = o;
    return FICCO_OK;
}

int ficco_plan_arrival(const ficco_plan_t *p, int32_t *chunk_ids, int32_t *group_ids, int cap)
{
    if (!p) return FICCO_ERR_ARG;
    if (cap < p->n_chunks) return FICCO_ERR_ARG;
    for (int q = 0; q < p->n_chunks; ++q) {
        if (chunk_ids) chunk_ids[q] = p->arrival[q];
        if (group_ids) group_ids[q] = p->group_of[q];
    }
    return FICCO_OK;
}

int ficco_pack_weight(ficco_plan_t *p, const void *W_dev, void *stream)
{
    if (!p || !W_dev) return FICCO_ERR_ARG;
    int rc = finalize(p);
    if (rc) return rc;
    bool dev = false;
    rc = is_device_ptr(W_dev, &dev);
    if (rc || !dev) return FICCO_ERR_ARG;
    return pack_weight(p, W_dev, (hipStream_t)stream);
}

int ficco_run(ficco_plan_t *p, const void *A_src, void *A_dev, const void *W_dev, void *C_dev,
              void *const *peer_out, void *compute_stream, void *copy_stream)
{
    if (!p || !A_dev || !W_dev || !C_dev) return FICCO_ERR_ARG;
    hipStream_t cs = (hipStream_t)compute_stream, xs = (hipStream_t)copy_stream;
    if (cs == xs) return FICCO_ERR_ARG;
    const bool rs = p->direction == FICCO_DIR_GEMM_RS;
    const int mode = p->mode;
    const bool do_copy = mode != FICCO_MODE_GEMM_ONLY;
    const bool do_gemm = mode != FICCO_MODE_COPY_ONLY;
    const bool dependent = mode == FICCO_MODE_PAIR;
    if (rs) {
        if (A_src) return FICCO_ERR_ARG;
        if (do_copy && !peer_out) return FICCO_ERR_ARG;
        if (is_2d(p) || p->local_shard >= 0) return FICCO_ERR_ARG;
        // resident kernel: alone, or as the pair with its transfers released by the kernel itself (engines only)
        if (is_resident(p) && mode != FICCO_MODE_GEMM_ONLY &&
            (mode != FICCO_MODE_PAIR || p->backend_opt == FICCO_COPY_STREAM || p->timing))
            return FICCO_ERR_ARG;
        // its epilogue writes 16-byte row segments
        if (is_resident(p) && (p->N % 8 != 0 || ((uintptr_t)C_dev & 15) != 0)) return FICCO_ERR_ARG;
    } else {
        if (peer_out) return FICCO_ERR_ARG;
        if (do_copy && !A_src) return FICCO_ERR_ARG;
    }
    int rc = finalize(p);
    if (rc) return rc;
    if (p->tile_col_lists > 1 && (is_resident(p) || p->grouped)) {     // refuse before anything is enqueued
        const TileShape ts = tile_shape(p->tile);
        if (p->tile_col_lists > (p->N + ts.bn - 1) / ts.bn) return FICCO_ERR_ARG;
    }

    bool dev = false;
    for (const void *ptr : {(const void *)A_dev, W_dev, (const void *)C_dev}) {
        rc = is_device_ptr(ptr, &dev);
        if (rc || !dev) return FICCO_ERR_ARG;
    }
    bool src_dev = false;
    if (!rs && do_copy) {
        rc = is_device_ptr(A_src, &src_dev);
        if (rc) return rc;
    }
    std::vector<char> peer_dev;
    if (rs && do_copy) {
        peer_dev.resize(p->G);
        for (int j = 0; j < p->G; ++j) {
            if (!peer_out[j]) return FICCO_ERR_ARG;
            bool d = false;
            rc = is_device_ptr(peer_out[j], &d);
            if (rc) return rc;
            peer_dev[j] = d;
        }
    }
    if (do_gemm && p->packed_from != W_dev) {
        rc = pack_weight(p, W_dev, cs);
        if (rc) return rc;
    }
    if (p->grouped) {
        if (rs || p->backend_opt == FICCO_COPY_STREAM || p->flag_write == 1) return FICCO_ERR_ARG;   // copy engines only
        return run_grouped(p, A_src, A_dev, C_dev, cs, src_dev);
    }
    // resolve the transfer backend
    int backend = p->backend_opt;
    // AUTO: the copy engines driven directly. They beat the stream path for pinned sources as well
    // (a transfer costs the host about a microsecond to submit against about ten for a stream copy,
    // and launches are enqueued before data moves), and they are the only way to move device-resident
    // shards without a copy kernel. The stream path remains for callers that ask for it, and for flag
    // writes by stream operations.
    const bool packed = p->packing && mode == FICCO_MODE_PAIR;     // the other modes measure the plain launches and transfers
    if (packed && (rs || p->hold_flags || backend == FICCO_COPY_STREAM)) return FICCO_ERR_ARG;
    // Exception: output blocks that all go to pinned host buffers (GEMM -> RS) stay on the stream path, whose
    // device-to-host copies were faster than the engines picked here (cfg4: 5.0 ms against 5.9 ms).
    bool any_peer_dev = false;
    for (char d : peer_dev) any_peer_dev |= (bool)d;
    const bool host_peers_only = rs && do_copy && !any_peer_dev && !is_resident(p);
    if (backend == FICCO_COPY_AUTO)
        backend = (packed || (do_copy && p->flag_write != 1 && !host_peers_only)) ? FICCO_COPY_ENGINES : FICCO_COPY_STREAM;
    p->backend = backend;
    if (backend == FICCO_COPY_ENGINES) {
        if (p->flag_write == 1) return FICCO_ERR_ARG;     // stream writes belong to the stream backend
        return run_engines(p, A_src, A_dev, C_dev, peer_out, cs, src_dev, peer_dev);
    }
    if (p->link || p->chain_from) return FICCO_ERR_ARG;   // chained plans run on the copy engines
    p->last_engines = false;
    p->links = 1;

    const bool timing = p->timing != 0;
    const int n = p->n_chunks;
    if (timing) {
        if ((rc = make_events(p->ev_copy_b, n))) return rc;
        if ((rc = make_events(p->ev_copy_e, n))) return rc;
        if ((rc = make_events(p->ev_gemm_b, p->groups.size()))) return rc;
        if ((rc = make_events(p->ev_gemm_e, p->groups.size()))) return rc;
    }

    const bool first = p->run_index == 0;
    p->run_index += 1;
    const uint32_t epoch = 1u + (p->run_index - 1u) % (uint32_t)(kEpochSlots - 1);
    const size_t row_bytes_c = (size_t)p->N * 2;
    const int c = p->c;

    // Order this run after the previous one on both streams, then start the clock on the stream
    // that moves first.
    // A run without transfers never touches the copy stream, and without per-launch timing it is
    // bracketed by two events only, so that back-to-back launches stay close together.
    const bool lean = !do_copy && !timing;
    // Under graph capture (ficco_graph_capture) the compute stream is the capture's origin: the copy
    // stream joins through a fork event, only dependency events are recorded (from a set of their
    // own), and the timing events stay outside the graph.
    const bool cap = p->capturing;
    std::vector<hipEvent_t> &dep_ev = cap ? p->cap_dep : p->ev_dep;
    if (cap) {
        HIP_TRY(hipEventRecord(p->cap_fork, cs));
        if (do_copy) HIP_TRY(hipStreamWaitEvent(xs, p->cap_fork, 0));
    } else {
        if (!first) {
            if (do_copy) HIP_TRY(hipStreamWaitEvent(xs, p->ev_end, 0));
            HIP_TRY(hipStreamWaitEvent(cs, p->ev_end, 0));
        }
        hipStream_t lead = (rs || !do_copy) ? cs : xs, follow = (rs || !do_copy) ? xs : cs;
        HIP_TRY(hipEventRecord(p->ev_begin, lead));
        if (do_copy) HIP_TRY(hipStreamWaitEvent(follow, p->ev_begin, 0));
    }

    int n_copies = 0, n_launches = 0;
    int64_t copy_bytes = 0;
    bool copy_first_recorded = false, gemm_first_recorded = false;

    auto is_local = [&](int chunk) { return !rs && p->local_shard >= 0 && shard_of(p, chunk) == p->local_shard; };

    auto issue_copy_ag = [&](int q) -> int {
        const int chunk = p->arrival[q];
        if (is_local(chunk)) return FICCO_OK;
        const Extent ex = piece_extent(p, chunk);
        const size_t off = ex.off, bytes = ex.bytes;
        if (timing) HIP_TRY(hipEventRecord(p->ev_copy_b[q], xs));
        if (!copy_first_recorded) {
            if (timing) HIP_TRY(hipEventRecord(p->ev_copy_first, xs));
            copy_first_recorded = true;
        }
        HIP_TRY(hipMemcpyAsync((char *)A_dev + off, (const char *)A_src + off, bytes,
                               src_dev ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, xs));
        if (timing) HIP_TRY(hipEventRecord(p->ev_copy_e[q], xs));
        ++n_copies;
        copy_bytes += (int64_t)bytes;
        return FICCO_OK;
    };
    auto issue_copy_rs = [&](int q) -> int {
        const int chunk = p->arrival[q];
        const int peer = chunk / c;
        const size_t off = (size_t)chunk * p->m * row_bytes_c, bytes = (size_t)p->m * row_bytes_c;
        const size_t peer_off = (size_t)(chunk % c) * p->m * row_bytes_c;
        if (timing) HIP_TRY(hipEventRecord(p->ev_copy_b[q], xs));
        HIP_TRY(hipMemcpyAsync((char *)peer_out[peer] + peer_off, (const char *)C_dev + off, bytes,
                               peer_dev[peer] ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, xs));
        if (timing) HIP_TRY(hipEventRecord(p->ev_copy_e[q], xs));
        ++n_copies;
        copy_bytes += (int64_t)bytes;
        return FICCO_OK;
    };
    auto issue_gemm = [&](size_t g) -> int {
        if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_b[g], cs));
        if (!gemm_first_recorded) {
            if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_first, cs));
            gemm_first_recorded = true;
        }
        GemmLaunch a = make_launch(p, p->groups[g], A_dev, C_dev);
        HIP_TRY(launch_gemm(p->tile, a, cs));
        if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_e[g], cs));
        ++n_launches;
        return FICCO_OK;
    };

    if (!timing && !cap) {
        // span events: first/last of each kind are recorded once, outside the per-piece path
        if (do_copy && !rs) HIP_TRY(hipEventRecord(p->ev_copy_first, xs));
        if (do_gemm && !lean) HIP_TRY(hipEventRecord(p->ev_gemm_first, cs));
    }

    if (is_resident(p)) {
        // ---- one resident kernel; transfers raise per-piece flags
        if (do_gemm) {
            const Gate gate{p->d_flags, nullptr, epoch, p->d_status, (uint32_t *)p->h_status,
                            (uint64_t)p->spin_limit_us * (uint64_t)p->wall_clock_khz / 1000u};
            int grid = p->resident_grid;
            if (dependent && do_copy) {
                // On this backend the 4-byte flag writes are done by a helper kernel of the HIP runtime,
                // which needs a CU with free registers while the resident workgroups spin: leave 8 CUs'
                // worth of slots unoccupied.
                int cus = 0;
                HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, p->device));
                const int full = is_2d(p) ? resident2d_grid_size(p->tile, p->device) : resident_grid_size(p->tile, p->device);
                const int per_cu = std::max(1, full / std::max(cus, 1));
                grid = std::max(1, std::min(grid, per_cu * (cus - 8)));
            }
            if (timing) {
                HIP_TRY(hipEventRecord(p->ev_gemm_b[0], cs));
                HIP_TRY(hipEventRecord(p->ev_gemm_first, cs));
            }
            gemm_first_recorded = true;
            const int reps = lean ? p->repeat : 1;       // measuring aid: the same launch back to back
            for (int rp = 0; rp < reps; ++rp) {
            if (is_2d(p)) {
                if ((rc = launch_2d(p, gate, dependent, grid, A_dev, C_dev, cs))) return rc;
            } else {
                ResidentLaunch r{};
                Group all{0, n};
                r.g = make_launch(p, all, A_dev, C_dev);
                r.g.block_row0 = nullptr; r.g.row0 = 0; r.g.n_blocks = n; r.g.rows_per_block = (int32_t)p->m;
                r.arrival = p->d_arrival;
                r.n_chunks = n;
                r.g.gate = gate;
                r.ticket = p->d_ticket;
                r.grid = grid;
                const ListGeometry lg = resident_lists(p);
                if (!lg.col_lists) return FICCO_ERR_ARG;
                r.group = lg.group;
                r.col_lists = lg.col_lists;
                if (!dependent) { r.local_chunk_begin = 0; r.local_chunk_end = n; }
                else if (p->local_shard >= 0) { r.local_chunk_begin = p->local_shard * c; r.local_chunk_end = (p->local_shard + 1) * c; }
                else { r.local_chunk_begin = 0; r.local_chunk_end = 0; }
                TileShape ts = tile_shape(p->tile);
                for (int x = 0; x < kTicketLists; ++x) {
                    r.ticket_base[x] = p->ticket_total[x];
                    p->ticket_total[x] += resident_list_draws(resident_list_tiles((int64_t)n * ((p->m + ts.bm - 1) / ts.bm),
                                                                                  (p->N + ts.bn - 1) / ts.bn, x, r.col_lists), r.grid, x);
                }
                HIP_TRY(launch_resident(p->tile, r, cs));
            }
            ++n_launches;
            }
            if (timing) HIP_TRY(hipEventRecord(p->ev_gemm_e[0], cs));
        }
        if (do_copy) {
            for (int q = 0; q < n; ++q) {
                if ((rc = issue_copy_ag(q))) return rc;
                const int chunk = p->arrival[q];
                if (dependent && !is_local(chunk) && !p->hold_flags) {
                    uint32_t *flag = p->d_flags + (size_t)chunk * kFlagStrideWords;
                    if (p->flag_write == 0)
                        HIP_TRY(hipMemcpyAsync(flag, p->h_epochs + epoch, 4, hipMemcpyHostToDevice, xs));
                    else
                        HIP_TRY(hipStreamWriteValue32(xs, flag, epoch, 0));
                }
            }
        }
    } else if (!rs) {
        // ---- all-gather -> GEMM, one launch per group of landed pieces
        if (!dependent) {
            if (do_copy) for (int q = 0; q < n; ++q) if ((rc = issue_copy_ag(q))) return rc;
            if (do_gemm)
                for (int rp = 0; rp < (lean ? p->repeat : 1); ++rp)
                    for (size_t g = 0; g < p->groups.size(); ++g) if ((rc = issue_gemm(g))) return rc;
        } else {
            for (size_t g = 0; g < p->groups.size(); ++g) {
                bool any = false;
                for (int q = p->groups[g].pos_begin; q < p->groups[g].pos_end; ++q) {
                    if (!is_local(p->arrival[q])) any = true;
                    if ((rc = issue_copy_ag(q))) return rc;
                }
                if (any) {
                    // the copy stream is in order: the event after the group's last transfer covers all of them
                    HIP_TRY(hipEventRecord(dep_ev[g], xs));
                    HIP_TRY(hipStreamWaitEvent(cs, dep_ev[g], 0));
                }
                if ((rc = issue_gemm(g))) return rc;
            }
        }
    } else {
        // ---- GEMM -> reduce-scatter (data movement): a group's rows leave as soon as its launch is done
        if (!dependent) {
            if (do_gemm)
                for (int rp = 0; rp < (lean ? p->repeat : 1); ++rp)
                    for (size_t g = 0; g < p->groups.size(); ++g) if ((rc = issue_gemm(g))) return rc;
            if (do_copy) {
                if (!cap) HIP_TRY(hipEventRecord(p->ev_copy_first, xs));
                for (int q = 0; q < n; ++q) if ((rc = issue_copy_rs(q))) return rc;
            }
        } else {
            for (size_t g = 0; g < p->groups.size(); ++g) {
                if ((rc = issue_gemm(g))) return rc;
                HIP_TRY(hipEventRecord(dep_ev[g], cs));
                HIP_TRY(hipStreamWaitEvent(xs, dep_ev[g], 0));
                if (g == 0 && !cap) HIP_TRY(hipEventRecord(p->ev_copy_first, xs));
                for (int q = p->groups[g].pos_begin; q < p->groups[g].pos_end; ++q)
                    if ((rc = issue_copy_rs(q))) return rc;
            }
        }
    }

    // ---- join: the run ends when both streams are done; ev_end is recorded on the compute stream
    if (cap) {
        // the copy stream rejoins the capture's origin; nothing else is recorded inside the graph
        if (do_copy) {
            HIP_TRY(hipEventRecord(p->cap_join, xs));
            HIP_TRY(hipStreamWaitEvent(cs, p->cap_join, 0));
        }
        p->graph_copies = n_copies;
        p->graph_launches = n_launches;
        p->graph_copy_bytes = copy_bytes;
        return FICCO_OK;
    }
    if (do_gemm && !lean) HIP_TRY(hipEventRecord(p->ev_gemm_last, cs));
    if (do_copy) {
        HIP_TRY(hipEventRecord(p->ev_copy_last, xs));
        HIP_TRY(hipStreamWaitEvent(cs, p->ev_copy_last, 0));
    }
    HIP_TRY(hipEventRecord(p->ev_end, cs));
    if (do_copy) HIP_TRY(hipStreamWaitEvent(xs, p->ev_end, 0));
    p->last_lean = lean;
    p->last_graph = false;
    p->last_skip_shard = rs ? -1 : p->local_shard;
    p->last_reduce = false;

    p->last_had_copies = n_copies > 0;
    p->last_had_gemm = n_launches > 0;
    p->last_timing = timing;
    p->last_copy_bytes = copy_bytes;
    p->last_n_copies = n_copies;
    p->last_n_launches = n_launches;
    return FICCO_OK;
}

int ficco_rs_reduce(ficco_plan_t *p, int block, const void *P_src, void *P_dev, const void *own, void *out, void *stream)
{
    if (!p || !P_src || !P_dev || !own || !out) return FICCO_ERR_ARG;
    if (is_2d(p) || p->grouped || block < 0 || block >= p->G) return FICCO_ERR_ARG;
    if (p->backend_opt == FICCO_COPY_STREAM || p->flag_write == 1) return FICCO_ERR_ARG;   // copy engines only
    hipStream_t cs = (hipStream_t)stream;
    int rc = finalize(p);
    if (rc) return rc;
    bool dev = false, src_dev = false;
    for (const void *ptr : {(const void *)P_dev, own, (const void *)out}) {
        rc = is_device_ptr(ptr, &dev);
        if (rc || !dev) return FICCO_ERR_ARG;
    }
    if ((rc = is_device_ptr(P_src, &src_dev))) return rc;
    const int n = p->n_chunks, c = p->c;
    // modes as in ficco_run: the pair, the reduction alone on a landing buffer that is already filled,
    // the transfers alone, or both without dependency
    const bool do_copy = p->mode != FICCO_MODE_GEMM_ONLY, do_add = p->mode != FICCO_MODE_COPY_ONLY;
    const bool dependent = p->mode == FICCO_MODE_PAIR;
    const bool touches_host = !src_dev;
    std::vector<int> eng;
    int links = 0;
    if ((rc = engines_prepare(p, touches_host, eng, links))) return rc;
    EngineCtx &ctx = g_engines;
    p->backend = FICCO_COPY_ENGINES;
    const bool poll_signals = p->sig_poll == 1 && !p->hold_flags && !touches_host;
    if (p->run_index > 0) {
        HIP_TRY(hipEventSynchronize(p->ev_end));
        for (int i = 0; i < n; ++i)
            if (!wait_signal(p->sig_data[i], 5.0) || !wait_signal(p->sig_flag[i], 5.0)) return FICCO_ERR_TIMEOUT;
    }
    p->run_index += 1;
    const uint32_t epoch = 1u + (p->run_index - 1u) % (uint32_t)(kEpochSlots - 1);
    const uint64_t spin_ticks = (uint64_t)p->spin_limit_us * (uint64_t)p->wall_clock_khz / 1000u;
    const Gate gate{p->d_flags, poll_signals ? p->d_sig_value : nullptr, epoch, p->d_status, (uint32_t *)p->h_status, spin_ticks};
    for (int i = 0; i < n; ++i) {
        hsa_signal_store_relaxed(p->sig_data[i], (i / c == block || !do_copy) ? 0 : 1);
        hsa_signal_store_relaxed(p->sig_flag[i], 0);
    }
    const size_t piece_bytes = (size_t)p->m * (size_t)p->N * 2;

    // the reduction is enqueued first: its tiles wait for their pieces
    ReduceLaunch r{};
    r.in = (const uint16_t *)P_dev;
    r.own = (const uint16_t *)own;
    r.out = (uint16_t *)out;
    r.piece_vecs = (int64_t)(piece_bytes / 16);
    r.G = p->G; r.block = block; r.pieces = c; r.gated = dependent ? 1 : 0;
    r.gate = gate;
    int grid = reduce_grid_size(p->device);
    if (grid <= 0) return FICCO_ERR_HIP;
    const int64_t tiles = (int64_t)c * ((r.piece_vecs + 1023) / 1024);
    if (tiles < grid) grid = (int)tiles;
    HIP_TRY(hipEventRecord(p->ev_begin, cs));
    if (do_add) HIP_TRY(launch_reduce(r, grid, cs));
    if (do_copy && !dependent && !p->hold_flags) {
        // nothing on the stream consumes the flags: join through the small waiting kernel, one launch per
        // run of arrival positions that belong to other blocks (the receiver's own pieces never travel)
        for (int q = 0; q < n;) {
            if (p->arrival[q] / c == block) { ++q; continue; }
            int e = q;
            while (e < n && p->arrival[e] / c != block) ++e;
            HIP_TRY(launch_wait_ready(gate, p->d_arrival + q, e - q, cs));
            q = e;
        }
    }
    HIP_TRY(hipEventRecord(p->ev_end, cs));

    // incoming partial blocks: piece s of peer j's block travels on link j; side by side in step-major
    // order (all links at once), one after the other for the shard-level and shard-major patterns
    const bool chained = p->schedule == FICCO_SHARD || (p->schedule != FICCO_SERIAL && p->order == FICCO_ORDER_SHARD_MAJOR);
    int n_copies = 0, prev_chunk = -1;
    int64_t copy_bytes = 0;
    for (int q = 0; q < n && do_copy; ++q) {
        const int chunk = p->arrival[q];
        if (chunk / c == block) continue;
        const hsa_amd_sdma_engine_id_t engine = (hsa_amd_sdma_engine_id_t)(1u << eng[(chunk / c) % links]);
        hsa_signal_t dep{};
        int ndep = 0;
        if (chained && prev_chunk >= 0) { dep = p->sig_data[prev_chunk]; ndep = 1; }
        hsa_status_t st = hsa_amd_memory_async_copy_on_engine((char *)P_dev + (size_t)chunk * piece_bytes, ctx.gpu,
                                                              (const char *)P_src + (size_t)chunk * piece_bytes, src_dev ? ctx.gpu : ctx.cpu,
                                                              piece_bytes, ndep, ndep ? &dep : nullptr, p->sig_data[chunk], engine, src_dev);
        if (st != HSA_STATUS_SUCCESS) { g_last_hip = (int)st; return FICCO_ERR_HIP; }
        prev_chunk = chunk;
        ++n_copies;
        copy_bytes += (int64_t)piece_bytes;
        if (!poll_signals && !p->hold_flags) {
            hsa_signal_store_relaxed(p->sig_flag[chunk], 1);
            st = hsa_amd_memory_async_copy_on_engine(p->d_flags + (size_t)chunk * kFlagStrideWords, ctx.gpu, p->h_epochs + epoch, ctx.cpu, 4,
                                                     1, &p->sig_data[chunk], p->sig_flag[chunk], engine, false);
            if (st != HSA_STATUS_SUCCESS) { hsa_signal_store_relaxed(p->sig_flag[chunk], 0); g_last_hip = (int)st; return FICCO_ERR_HIP; }
        }
    }
    p->last_had_copies = n_copies > 0;
    p->last_had_gemm = false;
    p->last_timing = false;
    p->last_copy_bytes = copy_bytes;
    p->last_n_copies = n_copies;
    p->last_n_launches = do_add ? 1 : 0;
    p->last_engines = true;
    p->last_lean = false;
    p->last_graph = false;
    p->last_skip_shard = block;
    p->last_reduce = true;
    return FICCO_OK;
}

int ficco_graph_capture(ficco_plan_t *p, const void *A_src, void *A_dev, const void *W_dev, void *C_dev,
                        void *const *peer_out)
{
    if (!p || !A_dev || !W_dev || !C_dev) return FICCO_ERR_ARG;
    if (is_resident(p) || p->grouped || p->timing || p->packing || p->mode != FICCO_MODE_PAIR) return FICCO_ERR_ARG;
    if (p->backend_opt == FICCO_COPY_ENGINES) return FICCO_ERR_ARG;      // engine submissions are host calls, not stream work
    const bool rs = p->direction == FICCO_DIR_GEMM_RS;
    if (rs ? (A_src || !peer_out) : (!A_src || peer_out)) return FICCO_ERR_ARG;
    int rc = finalize(p);
    if (rc) return rc;
    // only pinned host memory on the far side: a device-to-device stream copy would be a copy kernel
    bool dev = true;
    if (!rs) {
        if ((rc = is_device_ptr(A_src, &dev))) return rc;
        if (dev) return FICCO_ERR_ARG;
    } else {
        for (int j = 0; j < p->G; ++j) {
            if (!peer_out[j]) return FICCO_ERR_ARG;
            if ((rc = is_device_ptr(peer_out[j], &dev))) return rc;
            if (dev) return FICCO_ERR_ARG;
        }
    }
    if (!p->cap_cs) HIP_TRY(hipStreamCreateWithFlags(&p->cap_cs, hipStreamNonBlocking));
    if (!p->cap_xs) HIP_TRY(hipStreamCreateWithFlags(&p->cap_xs, hipStreamNonBlocking));
    if (!p->cap_fork) HIP_TRY(hipEventCreateWithFlags(&p->cap_fork, hipEventDisableTiming));
    if (!p->cap_join) HIP_TRY(hipEventCreateWithFlags(&p->cap_join, hipEventDisableTiming));
    while (p->cap_dep.size() < p->groups.size()) {
        hipEvent_t e;
        HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        p->cap_dep.push_back(e);
    }
    // the weight is packed outside the graph
    if (p->packed_from != W_dev) {
        if ((rc = pack_weight(p, W_dev, p->cap_cs))) return rc;
        HIP_TRY(hipStreamSynchronize(p->cap_cs));
    }
    if (p->graph_exec) { (void)hipGraphExecDestroy(p->graph_exec); p->graph_exec = nullptr; }
    if (p->graph) { (void)hipGraphDestroy(p->graph); p->graph = nullptr; }

    const int saved_backend = p->backend_opt;
    const uint32_t saved_run = p->run_index;
    p->backend_opt = FICCO_COPY_STREAM;
    HIP_TRY(hipStreamBeginCapture(p->cap_cs, hipStreamCaptureModeRelaxed));
    p->capturing = true;
    rc = ficco_run(p, A_src, A_dev, W_dev, C_dev, peer_out, p->cap_cs, p->cap_xs);
    p->capturing = false;
    p->backend_opt = saved_backend;
    p->run_index = saved_run;            // a capture is not a run
    hipGraph_t g = nullptr;
    hipError_t e = hipStreamEndCapture(p->cap_cs, &g);
    if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
    if (e != hipSuccess || !g) { g_last_hip = (int)e; (void)hipGetLastError(); return FICCO_ERR_HIP; }
    p->graph = g;
    e = hipGraphInstantiate(&p->graph_exec, p->graph, nullptr, nullptr, 0);
    if (e != hipSuccess) { g_last_hip = (int)e; (void)hipGetLastError(); p->graph_exec = nullptr; return FICCO_ERR_HIP; }
    return FICCO_OK;
}

int ficco_graph_launch(ficco_plan_t *p, void *stream)
{
    if (!p) return FICCO_ERR_ARG;
    if (!p->graph_exec) return FICCO_ERR_STATE;
    hipStream_t s = (hipStream_t)stream;
    if (p->run_index > 0) HIP_TRY(hipStreamWaitEvent(s, p->ev_end, 0));
    HIP_TRY(hipEventRecord(p->ev_begin, s));
    HIP_TRY(hipGraphLaunch(p->graph_exec, s));
    HIP_TRY(hipEventRecord(p->ev_end, s));
    p->run_index += 1;
    p->last_graph = true;
    p->last_reduce = false;
    p->last_engines = false;
    p->last_lean = false;
    p->last_had_copies = false;
    p->last_had_gemm = false;
    p->last_timing = false;
    return FICCO_OK;
}

int ficco_query_stats(ficco_plan_t *p, ficco_stats_t *out)
{
    if (!p || !out) return FICCO_ERR_ARG;
    if (!p->finalized || p->run_index == 0) return FICCO_ERR_STATE;
    HIP_TRY(hipEventSynchronize(p->ev_end));
    ficco_stats_t s{};
    float ms = 0;
    HIP_TRY(hipEventElapsedTime(&ms, p->ev_begin, p->ev_end));
    s.wall_us = ms * 1e3;
    if (p->last_graph) {
        // a graph replay is bracketed by the two events only; what it holds was counted at capture
        s.run_index = (int32_t)p->run_index;
        s.n_copies = p->graph_copies;
        s.n_launches = p->graph_launches;
        s.copy_bytes = p->graph_copy_bytes;
        s.flops = 2 * p->M * p->N * p->K;
        s.eff_tflops = s.wall_us > 0 ? (double)s.flops / s.wall_us * 1e-6 : 0.0;
        *out = s;
        return FICCO_OK;
    }
    if (p->last_had_copies && p->last_engines) {
        // copy-engine timestamps (system clock ticks) of every transfer of the run
        uint64_t t_min = ~0ull, t_max = 0;
        double busy = 0;
        for (int q = 0; q < p->n_chunks; ++q) {
            const int chunk = p->arrival[q];
            if ((p->last_skip_shard >= 0 && shard_of(p, chunk) == p->last_skip_shard) || (p->grouped && p->piece_nrows[chunk] == 0)) continue;
            if (!wait_signal(p->sig_data[p->arrival[q]], 5.0) || !wait_signal(p->sig_flag[p->arrival[q]], 5.0)) {
                if (getenv("FICCO_DEBUG"))
                    fprintf(stderr, "ficco: transfer %d (chunk %d) did not complete: data signal %lld flag signal %lld\n", q, chunk,
                            (long long)hsa_signal_load_relaxed(p->sig_data[p->arrival[q]]), (long long)hsa_signal_load_relaxed(p->sig_flag[p->arrival[q]]));
                return FICCO_ERR_TIMEOUT;
            }
            hsa_amd_profiling_async_copy_time_t t{};
            if (hsa_amd_profiling_get_async_copy_time(p->sig_data[p->arrival[q]], &t) != HSA_STATUS_SUCCESS) continue;
            t_min = std::min(t_min, (uint64_t)t.start);
            t_max = std::max(t_max, (uint64_t)t.end);
            busy += (double)(t.end - t.start) / g_engines.ticks_per_us;
        }
        if (t_max > t_min) s.copy_span_us = (double)(t_max - t_min) / g_engines.ticks_per_us;
        p->last_engine_copy_span_us = s.copy_span_us;
        p->last_engine_copy_busy_us = busy;
    } else if (p->last_had_copies) {
        HIP_TRY(hipEventElapsedTime(&ms, p->ev_copy_first, p->ev_copy_last));
        s.copy_span_us = ms * 1e3;
    }
    if (p->last_had_gemm) {
        if (p->last_lean) HIP_TRY(hipEventElapsedTime(&ms, p->ev_begin, p->ev_end));
        else HIP_TRY(hipEventElapsedTime(&ms, p->last_engines ? p->ev_begin : p->ev_gemm_first, p->ev_gemm_last));
        s.gemm_span_us = ms * 1e3;
    }
    s.gemm_busy_us = s.gemm_span_us;
    s.copy_busy_us = s.copy_span_us;
    if (p->last_timing) {
        double gb = 0, cb = 0;
        if (p->last_had_gemm) {
            const size_t ng = is_resident(p) ? 1 : p->groups.size();
            for (size_t g = 0; g < ng; ++g) {
                HIP_TRY(hipEventElapsedTime(&ms, p->ev_gemm_b[g], p->ev_gemm_e[g]));
                gb += ms * 1e3;
            }
            s.gemm_busy_us = gb;
        }
        if (p->last_had_copies && !p->last_engines) {
            for (int q = 0; q < p->n_chunks; ++q) {
                const int chunk = p->arrival[q];
                if ((p->last_skip_shard >= 0 && shard_of(p, chunk) == p->last_skip_shard) || (p->grouped && p->piece_nrows[chunk] == 0)) continue;
                HIP_TRY(hipEventElapsedTime(&ms, p->ev_copy_b[q], p->ev_copy_e[q]));
                cb += ms * 1e3;
            }
            s.copy_busy_us = cb;
        }
    }
    if (p->last_had_copies && p->last_engines) s.copy_busy_us = p->last_engine_copy_busy_us;
    if (p->last_engines && p->last_had_copies && getenv("FICCO_DEBUG") && atoi(getenv("FICCO_DEBUG")) >= 2) {
        uint64_t t0 = ~0ull;
        std::vector<hsa_amd_profiling_async_copy_time_t> tt(p->n_chunks), tf(p->n_chunks);
        for (int q = 0; q < p->n_chunks; ++q) {
            hsa_amd_profiling_get_async_copy_time(p->sig_data[p->arrival[q]], &tt[q]);
            hsa_amd_profiling_get_async_copy_time(p->sig_flag[p->arrival[q]], &tf[q]);
            if (tt[q].start && tt[q].start < t0) t0 = tt[q].start;
        }
        for (int q = 0; q < p->n_chunks; ++q)
            fprintf(stderr, "ficco: run %u pos %d chunk %d data [%.1f, %.1f] us flag [%.1f, %.1f] us\n", p->run_index, q, p->arrival[q],
                    (tt[q].start - t0) / g_engines.ticks_per_us, (tt[q].end - t0) / g_engines.ticks_per_us,
                    (tf[q].start - t0) / g_engines.ticks_per_us, (tf[q].end - t0) / g_engines.ticks_per_us);
    }
    s.exposed_comm_us = s.wall_us - s.gemm_busy_us;
    s.flops = p->last_reduce ? (int64_t)(p->G - 1) * (p->M / p->G) * p->N      // the reduction's additions
                             : 2 * p->M * p->N * p->K;
    s.eff_tflops = s.wall_us > 0 ? (double)s.flops / s.wall_us * 1e-6 : 0.0;
    s.copy_bytes = p->last_copy_bytes;
    s.copy_gbps = s.copy_span_us > 0 ? (double)s.copy_bytes / s.copy_span_us * 1e-3 : 0.0;
    s.n_copies = p->last_n_copies;
    s.n_launches = p->last_n_launches;
    s.run_index = (int32_t)p->run_index;
    if ((is_resident(p) && p->last_had_gemm) || p->last_engines) {
        const uint32_t st = p->h_status[0];     // the run has completed (event above): no copy needed
        if (st) {
            if (getenv("FICCO_DEBUG")) {
                fprintf(stderr, "ficco: a kernel's bounded wait expired (run %u)\n", p->run_index);
                std::vector<uint32_t> fl((size_t)p->n_chunks * kFlagStrideWords);
                if (hipMemcpy(fl.data(), p->d_flags, fl.size() * 4, hipMemcpyDeviceToHost) == hipSuccess) {
                    fprintf(stderr, "ficco: flags now:");
                    for (int i = 0; i < p->n_chunks; ++i) fprintf(stderr, " %u", fl[(size_t)i * kFlagStrideWords]);
                    fprintf(stderr, "\n");
                }
                if (p->last_engines) {
                    uint64_t t0 = ~0ull;
                    std::vector<hsa_amd_profiling_async_copy_time_t> tt(p->n_chunks), tf(p->n_chunks);
                    for (int q = 0; q < p->n_chunks; ++q) {
                        hsa_amd_profiling_get_async_copy_time(p->sig_data[p->arrival[q]], &tt[q]);
                        hsa_amd_profiling_get_async_copy_time(p->sig_flag[p->arrival[q]], &tf[q]);
                        if (tt[q].start && tt[q].start < t0) t0 = tt[q].start;
                    }
                    for (int q = 0; q < p->n_chunks; ++q)
                        fprintf(stderr, "ficco: pos %d chunk %d data [%.1f, %.1f] us flag [%.1f, %.1f] us\n", q, p->arrival[q],
                                (tt[q].start - t0) / g_engines.ticks_per_us, (tt[q].end - t0) / g_engines.ticks_per_us,
                                (tf[q].start - t0) / g_engines.ticks_per_us, (tf[q].end - t0) / g_engines.ticks_per_us);
                }
            }
            s.timed_out = 1;
            for (auto &sg : p->sig_done) hsa_signal_store_screlease(sg, 0);   // let parked copies go
            HIP_TRY(hipMemset(p->d_status, 0, 4));
            p->h_status[0] = 0;
        }
    }
    *out = s;
    return s.timed_out ? FICCO_ERR_TIMEOUT : FICCO_OK;
}

int ficco_query_spans(ficco_plan_t *p, double *copy_begin_us, double *copy_end_us, int cap_chunks,
                      double *gemm_begin_us, double *gemm_end_us, int cap_groups)
{
    if (!p) return FICCO_ERR_ARG;
    if (!p->finalized || p->run_index == 0 || !p->last_timing) return FICCO_ERR_STATE;
    HIP_TRY(hipEventSynchronize(p->ev_end));
    float ms = 0;
    if (copy_begin_us || copy_end_us) {
        if (cap_chunks < p->n_chunks) return FICCO_ERR_ARG;
        for (int q = 0; q < p->n_chunks; ++q) {
            const int chunk = p->arrival[q];
            const bool local = (p->last_skip_shard >= 0 && shard_of(p, chunk) == p->last_skip_shard) || (p->grouped && p->piece_nrows[chunk] == 0);
            double b = 0, e = 0;
            if (p->last_had_copies && !local && p->last_engines) {
                // engine timestamps live on another clock: reported relative to the run's first transfer
                static thread_local uint64_t t_first;
                hsa_amd_profiling_async_copy_time_t t{};
                if (q == 0 || t_first == 0) {
                    t_first = ~0ull;
                    for (int r = 0; r < p->n_chunks; ++r) {
                        hsa_amd_profiling_async_copy_time_t u{};
                        if (hsa_signal_load_relaxed(p->sig_data[r]) == 0 &&
                            hsa_amd_profiling_get_async_copy_time(p->sig_data[r], &u) == HSA_STATUS_SUCCESS && u.end > u.start)
                            t_first = std::min(t_first, (uint64_t)u.start);
                    }
                }
                if (hsa_amd_profiling_get_async_copy_time(p->sig_data[p->arrival[q]], &t) == HSA_STATUS_SUCCESS && t.end > t.start) {
                    b = (double)(t.start - t_first) / g_engines.ticks_per_us;
                    e = (double)(t.end - t_first) / g_engines.ticks_per_us;
                }
            } else if (p->last_had_copies && !local) {
                HIP_TRY(hipEventElapsedTime(&ms, p->ev_begin, p->ev_copy_b[q])); b = ms * 1e3;
                HIP_TRY(hipEventElapsedTime(&ms, p->ev_begin, p->ev_copy_e[q])); e = ms * 1e3;
            }
            if (copy_begin_us) copy_begin_us[q] = b;
            if (copy_end_us) copy_end_us[q] = e;
        }
    }
    if (gemm_begin_us || gemm_end_us) {
        const int ng = (int)p->groups.size();
        if (cap_groups < ng) return FICCO_ERR_ARG;
        for (int g = 0; g < ng; ++g) {
            double b = 0, e = 0;
            if (p->last_had_gemm) {
                HIP_TRY(hipEventElapsedTime(&ms, p->ev_begin, p->ev_gemm_b[g])); b = ms * 1e3;
                HIP_TRY(hipEventElapsedTime(&ms, p->ev_begin, p->ev_gemm_e[g])); e = ms * 1e3;
            }
            if (gemm_begin_us) gemm_begin_us[g] = b;
            if (gemm_end_us) gemm_end_us[g] = e;
        }
    }
    return FICCO_OK;
}

int ficco_profile_losses(ficco_plan_t *p, const void *A_src, void *A_dev, const void *W_dev, void *C_dev,
                         void *compute_stream, void *copy_stream, int warmup, int iters, ficco_losses_t *out)
{
    if (!p || !out || !A_src || !A_dev || !W_dev || !C_dev || iters < 1 || warmup < 0) return FICCO_ERR_ARG;
    if (p->direction != FICCO_DIR_AG_GEMM || p->grouped) return FICCO_ERR_ARG;
    ficco_plan_t *whole = nullptr;
    int rc = ficco_plan(p->M, p->K, p->N, p->G, 1, FICCO_SERIAL, &whole);
    if (rc) return rc;
    whole->backend_opt = p->backend_opt;
    whole->links_opt = p->links_opt;
    whole->spin_limit_us = p->spin_limit_us;
    const int saved_mode = p->mode, saved_timing = p->timing;

    // mean span of one mode over `iters` runs after `warmup`
    auto measure = [&](ficco_plan_t *q, int mode, double *gemm_us, double *copy_us) -> int {
        int r = ficco_plan_set(q, FICCO_OPT_MODE, mode);
        if (r) return r;
        if ((r = ficco_plan_set(q, FICCO_OPT_TIMING, 0))) return r;
        double g = 0, cp = 0;
        for (int it = 0; it < warmup + iters; ++it) {
            if ((r = ficco_run(q, A_src, A_dev, W_dev, C_dev, nullptr, compute_stream, copy_stream))) return r;
            ficco_stats_t s;
            if ((r = ficco_query_stats(q, &s))) return r;
            if (it >= warmup) { g += s.gemm_span_us; cp += s.copy_span_us; }
        }
        if (gemm_us) *gemm_us = g / iters;
        if (copy_us) *copy_us = cp / iters;
        return FICCO_OK;
    };

    ficco_losses_t L{};
    do {
        if ((rc = measure(whole, FICCO_MODE_GEMM_ONLY, &L.t_gemm_whole_us, nullptr))) break;
        if ((rc = measure(whole, FICCO_MODE_COPY_ONLY, nullptr, &L.t_copy_whole_us))) break;
        if ((rc = measure(p, FICCO_MODE_GEMM_ONLY, &L.t_gemm_pieces_us, nullptr))) break;
        if ((rc = measure(p, FICCO_MODE_COPY_ONLY, nullptr, &L.t_copy_pieces_us))) break;
        if ((rc = measure(p, FICCO_MODE_INDEPENDENT, &L.t_gemm_pieces_cont_us, &L.t_copy_pieces_cont_us))) break;
    } while (0);
    ficco_destroy(whole);
    p->mode = saved_mode;
    p->timing = saved_timing;
    if (rc) return rc;
    L.gemm_dil = L.t_gemm_pieces_us / L.t_gemm_whole_us;
    L.gemm_cil = L.t_gemm_pieces_cont_us / L.t_gemm_pieces_us;
    L.comm_dil = L.t_copy_pieces_us / L.t_copy_whole_us;
    L.comm_cil = L.t_copy_pieces_cont_us / L.t_copy_pieces_us;
    L.ideal_us = ficco_ideal_overlap_us(L.t_copy_whole_us, L.t_gemm_whole_us, p->schedule == FICCO_SERIAL ? 1 : ((int)p->groups.size() > 1 ? (int)p->groups.size() : p->n_chunks));
    *out = L;
    return FICCO_OK;
}

void ficco_destroy(ficco_plan_t *p)
{
    if (!p) return;
    if (p->finalized && p->run_index > 0 && p->ev_end) (void)hipEventSynchronize(p->ev_end);
    for (auto &sg : p->sig_done) hsa_signal_store_screlease(sg, 0);      // nothing may stay parked behind a piece that never completed
    if (p->link) {
        // plans chained behind this one keep the link alive; their transfers no longer wait for it
        p->link->alive = false;
        if (p->link->made)
            for (auto &sg : p->link->free_sig) hsa_signal_store_screlease(sg, 0);
    }
    // transfers still in flight must not outlive their signals; one bound for all of them (a run that
    // failed half-way may have armed signals whose transfers were never submitted)
    const auto deadline = std::chrono::steady_clock::now() + std::chrono::seconds(5);
    for (auto *v : {&p->sig_data, &p->sig_flag, &p->sig_gather, &p->sig_scatter})
        for (auto &sg : *v) {
            const double left = std::chrono::duration<double>(deadline - std::chrono::steady_clock::now()).count();
            (void)wait_signal(sg, left > 0.001 ? left : 0.001);
        }
    release(p);
    delete p;
}

const char *ficco_strerror(int status)
{
    switch (status) {
    case FICCO_OK: return "ok";
    case FICCO_ERR_ARG: return "invalid argument";
    case FICCO_ERR_SHAPE: return "shape rule violated";
    case FICCO_ERR_ALLOC: return "allocation failed";
    case FICCO_ERR_HIP: return "HIP call failed";
    case FICCO_ERR_TIMEOUT: return "resident kernel gave up waiting for a ready flag";
    case FICCO_ERR_STATE: return "call not valid in this state";
    default: return "unknown status";
    }
}

int ficco_last_hip_error(void) { return g_last_hip; }

const char *ficco_version(void) { return "ficco-mi355x 0.1 (gfx950)"; }

}  // extern "C"
