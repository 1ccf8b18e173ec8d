// Copy-engine (SDMA) backend of libficco: the engines are driven directly through the HSA runtime that
// sits underneath HIP, one engine per emulated link; completion signals double as the ready flags
// kernels wait on. Also the receiver side of the reduce-scatter, which lives on the same machinery.
#include "ficco_plan.h"

namespace ficco {

namespace {

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

}  // namespace

double engine_ticks_per_us() { return g_engines.ticks_per_us; }

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

    // engines: one per emulated link
    links = p->links_opt > 0 ? p->links_opt : p->G;
    links = std::min(links, 16);
    eng = usable_engines(touches_host, links, p->d_status + kFlagStrideWords);
    if (eng.empty()) { if (getenv("FICCO_DEBUG")) fprintf(stderr, "ficco: no usable engine\n"); return FICCO_ERR_HIP; }
    links = std::min(links, (int)eng.size());
    p->links = links;

    // signals, one pair per chunk
    auto grow = [&](std::vector<hsa_signal_t> &v) -> int {         // each list on its own: a failure half-way leaves them consistent
        while ((int)v.size() < n) {
            hsa_signal_t a;
            if (make_signal(&a) != HSA_STATUS_SUCCESS) return FICCO_ERR_ALLOC;
            v.push_back(a);
        }
        return FICCO_OK;
    };
    if ((rc = grow(p->sig_data)) || (rc = grow(p->sig_flag))) return rc;
    if (p->packing && ((rc = grow(p->sig_gather)) || (rc = grow(p->sig_scatter)))) return rc;
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

// Chained plans (ficco_plan_chain), one run's share. Behind another plan: every transfer of this run also
// waits for the signal (dep) that plan's latest run releases when it ends. In front of others: the run
// arms one of its two signals now and has it released from the compute stream (release_addr) when
// everything it enqueues there is done; until the run has handed that over, a return - a run that fails
// half-way - releases the signal from the host, so that nothing stays parked behind it.
struct ChainScope {
    hsa_signal_t dep{};
    bool has_dep = false;
    uint64_t release_addr = 0;
    hsa_signal_t armed{};
    bool on = false;
    int begin(ficco_plan_t *p)
    {
        if (p->chain_from && p->chain_from->alive && p->chain_from->made && p->chain_from->last >= 0) {
            dep = p->chain_from->free_sig[p->chain_from->last];
            has_dep = true;
        }
        if (!p->link) return FICCO_OK;
        ChainLink &L = *p->link;
        if (!L.made) {
            for (int i = 0; i < 2; ++i) {
                if (make_signal(&L.free_sig[i]) != HSA_STATUS_SUCCESS) {
                    if (i) (void)hsa_signal_destroy(L.free_sig[0]);
                    return FICCO_ERR_ALLOC;
                }
            }
            L.made = true;
            for (int i = 0; i < 2; ++i) L.addr[i] = signal_value_address(L.free_sig[i]);
        }
        if (!L.addr[0] || !L.addr[1]) return FICCO_ERR_HIP;      // needs signals the GPU can write
        const int idx = (L.last + 1) & 1;
        hsa_signal_store_relaxed(L.free_sig[idx], 1);
        L.last = idx;
        armed = L.free_sig[idx];
        on = true;
        release_addr = L.addr[idx];
        return FICCO_OK;
    }
    void handed_over() { on = false; }
    ~ChainScope() { if (on) hsa_signal_store_screlease(armed, 0); }
};

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
    ChainScope chain;
    if ((rc = chain.begin(p))) return rc;
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
    if (chain.release_addr) {
        HIP_TRY(launch_release_signal(chain.release_addr, cs));
        chain.handed_over();                             // the stream releases it from here on
    }
    HIP_TRY(hipEventRecord(p->ev_end, cs));

    const bool chained = p->schedule == FICCO_SHARD || (p->schedule != FICCO_SERIAL && p->order == FICCO_ORDER_SHARD_MAJOR);
    int prev_chunk = -1;
    for (int q = 0; q < n && do_copy; ++q) {
        const int chunk = p->arrival[q];
        const hsa_amd_sdma_engine_id_t engine = (hsa_amd_sdma_engine_id_t)(1u << eng[(chunk % G) % links]);
        const size_t off = (size_t)p->piece_row0[chunk] * p->K * 2, bytes = (size_t)p->piece_nrows[chunk] * p->K * 2;
        hsa_status_t st;
        if (bytes) {
            hsa_signal_t dep[2];
            int ndep = 0;
            if (chained && prev_chunk >= 0) dep[ndep++] = p->sig_data[prev_chunk];
            if (chain.has_dep) dep[ndep++] = chain.dep;
            st = hsa_amd_memory_async_copy_on_engine((char *)A_dev + off, ctx.gpu, (const char *)A_src + off, src_dev ? ctx.gpu : ctx.cpu, bytes,
                                                     ndep, ndep ? dep : nullptr, p->sig_data[chunk], engine, src_dev);
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

    if (rs && p->chain_from) return FICCO_ERR_ARG;       // chaining is defined for the transfers into A_dev only
    ChainScope chain;
    if ((rc = chain.begin(p))) return rc;
    const hsa_signal_t chain_dep = chain.dep;
    const bool has_chain_dep = chain.has_dep;
    const uint64_t release_addr = chain.release_addr;

    int n_copies = 0, n_launches = 0;
    int64_t copy_bytes = 0;
    // one piece: data copy, then the 4-byte flag copy behind it on the same engine
    int prev_chunk = -1;
    std::vector<hsa_signal_t> *extra_dep = nullptr;      // per chunk id: one more signal every transfer waits for
    // Column pieces out of a row-major matrix (ficco_source_layout): rectangular engine copies from pinned host
    // memory; from device memory the sender-side re-layout kernel, which releases each piece's transfer.
    const bool row_src = !rs && is_2d(p) && p->src_layout == FICCO_LAYOUT_ROW_MAJOR && do_copy;
    const bool relayout = row_src && src_dev;
    if (relayout) {
        if (!p->d_slice_src && hipMalloc((void **)&p->d_slice_src, (size_t)p->M * p->K * 2) != hipSuccess) return FICCO_ERR_ALLOC;
        while ((int)p->sig_packed.size() < n) {
            hsa_signal_t a;
            if (make_signal(&a) != HSA_STATUS_SUCCESS) return FICCO_ERR_ALLOC;
            p->sig_packed.push_back(a);
        }
        if (!p->d_packed_value) {
            std::vector<uint64_t> addr(n);
            for (int i = 0; i < n; ++i)
                if (!(addr[i] = signal_value_address(p->sig_packed[i]))) return FICCO_ERR_HIP;   // needs signals the GPU can write
            if (hipMalloc((void **)&p->d_packed_value, sizeof(uint64_t) * (size_t)n) != hipSuccess) return FICCO_ERR_ALLOC;
            HIP_TRY(hipMemcpy(p->d_packed_value, addr.data(), sizeof(uint64_t) * (size_t)n, hipMemcpyHostToDevice));
            if (hipMalloc((void **)&p->d_packed_count, sizeof(uint32_t) * (size_t)n) != hipSuccess) return FICCO_ERR_ALLOC;
            HIP_TRY(hipMemset(p->d_packed_count, 0, sizeof(uint32_t) * (size_t)n));
        }
        for (int i = 0; i < n; ++i) hsa_signal_store_relaxed(p->sig_packed[i], 1);
        extra_dep = &p->sig_packed;
    }
    // the re-layout kernel goes onto the compute stream in front of the GEMM (a resident GEMM kernel would
    // otherwise hold every CU while it waits for transfers that wait for this kernel)
    auto launch_relayout = [&]() -> int {
        if (!relayout) return FICCO_OK;
        SliceLaunch sl{};
        sl.src = (const uint16_t *)A_src;
        sl.dst = p->d_slice_src;
        sl.M = p->M; sl.K = p->K;
        sl.shards = p->G;
        sl.rows_per_shard = (int32_t)p->m;
        sl.k0 = p->d_slice_k0;
        sl.arrival = p->d_arrival;
        sl.n_pieces = n;
        // blocks of about 64 KiB of the widest slice, walked in arrival order by at most 1024 workgroups
        int64_t widest = 0;
        for (int q = 0; q < c; ++q) widest = std::max<int64_t>(widest, p->slice_k0[q + 1] - p->slice_k0[q]);
        sl.rows_per_block = (int32_t)std::max<int64_t>(1, std::min<int64_t>(p->m, (64 << 10) / (widest * 2)));
        sl.blocks_per_piece = (int32_t)((p->m + sl.rows_per_block - 1) / sl.rows_per_block);
        sl.done_count = p->d_packed_count;
        sl.done_sig = p->d_packed_value;
        HIP_TRY(launch_slice_source(sl, cs));
        return FICCO_OK;
    };
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
        bool rect = false;
        if (!rs) {
            const Extent ex = piece_extent(p, chunk);
            bytes = ex.bytes;
            dst = (char *)A_dev + ex.off;
            src = (const char *)A_src + ex.off;
            if (relayout) src = (const char *)p->d_slice_src + ex.off;       // the sender-side staging copy, K-sliced like A_dev
            rect = row_src && !src_dev;                                      // a strided rectangle out of the row-major host matrix
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
        hsa_status_t st;
        if (rect) {
            // rows [j*m, (j+1)*m) x columns [kb, kb+kw) at pitch K -> the piece's contiguous block of A_dev; the
            // runtime picks the engine for rectangular copies itself (its host-to-device one)
            const int sl = chunk / p->G, j = chunk % p->G;
            const size_t kb = (size_t)p->slice_k0[sl], kw = (size_t)p->slice_k0[sl + 1] - kb;
            hsa_pitched_ptr_t ps{(void *)((const char *)A_src + ((size_t)j * p->m * p->K + kb) * 2), (size_t)p->K * 2, 0};
            hsa_pitched_ptr_t pd{dst, kw * 2, 0};
            const hsa_dim3_t zero{0, 0, 0}, range{(uint32_t)(kw * 2), (uint32_t)p->m, 1};
            st = hsa_amd_memory_async_copy_rect(&pd, &zero, &ps, &zero, &range, ctx.gpu, hsaHostToDevice, ndep, ndep ? dep : nullptr,
                                                p->sig_data[chunk]);
        } else {
            st = hsa_amd_memory_async_copy_on_engine(dst, dst_agent, src, src_agent, bytes, ndep, ndep ? dep : nullptr,
                                                     p->sig_data[chunk], engine, force);
        }
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
        if ((rc = launch_relayout())) return rc;
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
        chain.handed_over();                             // the stream releases it from here on
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

}  // namespace ficco

using namespace ficco;

extern "C" {

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

}  // extern "C"
