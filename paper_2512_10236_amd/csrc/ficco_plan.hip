// Plans of libficco: shape rules, arrival lists and launch groups, tile choice, resources, options and
// the static schedule heuristic. See include/ficco.h for the contract of every entry point.
#include "ficco_plan.h"

namespace ficco {

thread_local int g_last_hip = 0;

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
    for (auto *v : {&p->sig_data, &p->sig_flag, &p->sig_gather, &p->sig_scatter, &p->sig_done, &p->sig_packed}) {
        for (auto &sg : *v) (void)hsa_signal_destroy(sg);
        v->clear();
    }
    if (p->d_words) (void)hipFree(p->d_words);
    if (p->d_ticket_mem) (void)hipFree(p->d_ticket_mem);
    if (p->d_sig_value) (void)hipFree(p->d_sig_value);
    if (p->d_done_value) (void)hipFree(p->d_done_value);
    if (p->d_done_count) (void)hipFree(p->d_done_count);
    if (p->d_slice_src) (void)hipFree(p->d_slice_src);
    if (p->d_packed_value) (void)hipFree(p->d_packed_value);
    if (p->d_packed_count) (void)hipFree(p->d_packed_count);
    p->d_slice_src = nullptr; p->d_packed_value = nullptr; p->d_packed_count = nullptr;
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

ListGeometry pick_lists(const ficco_plan_t *p, const TileShape &ts, int64_t tn, int64_t row_tiles, int64_t S, int64_t slots,
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
ListGeometry resident_lists(const ficco_plan_t *p)
{
    const TileShape ts = tile_shape(p->tile);
    const int64_t rt = (p->m + ts.bm - 1) / ts.bm;
    return pick_lists(p, ts, (p->N + ts.bn - 1) / ts.bn, (int64_t)p->n_chunks * rt, (p->order == FICCO_ORDER_STEP_MAJOR ? (int64_t)p->G : 1) * rt,
                      p->resident_grid / kTicketLists, p->M * p->K * 2, p->N * p->K * 2);
}

// One resident launch of the K-sliced schedule: every tile owns its part of C for the whole k range
// and waits, slice by slice, for the column pieces of the shards its rows come from.
int launch_2d(ficco_plan_t *p, const Gate &gate, bool gated, int grid, const void *A_dev, void *C_dev, hipStream_t cs,
              uint64_t release_addr)
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

}  // namespace ficco

using namespace ficco;

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

// Pieces per shard (or per output block) from the overlap model, see ficco_pick_schedule. `row_bytes` = what one
// row of a piece puts on its link: K elements of the activation (all-gather) or N of the output (reduce-scatter).
static int pick_pieces(int64_t M, int64_t K, int64_t N, int shards, int64_t row_bytes)
{
    const int64_t ms = M / shards;
    const double Tc = (double)ms * (double)row_bytes / 58.0e3;                      // us
    const double Tg = 2.0 * (double)M * (double)N * (double)K / 1.2e9;              // us
    int c = 1;
    double best = -1.0;
    for (int cc = 1; cc <= 32; cc *= 2) {
        if (ms % cc || (cc > 1 && ms / cc < 256)) continue;
        const double T = std::max(Tc + cc * 16.0, Tg + cc * 8.0) + std::min(Tc, Tg) / cc;
        if (best < 0 || T < best * 0.999) { best = T; c = cc; }
    }
    return c;
}

int ficco_pick_schedule_rs(int64_t M, int64_t K, int64_t N, int shards, int *schedule, int *chunks)
{
    if (M < 1 || K < 1 || N < 1 || shards < 1 || !schedule || !chunks) return FICCO_ERR_ARG;
    if (M % shards) return FICCO_ERR_SHAPE;
    // GEMM -> reduce-scatter, data movement (Sec. IV-E leaves the reduction out): the mirror image of the all-gather
    // rule. Row block p of the output travels to peer p piece by piece as the GEMM completes it, so one link carries
    // (M/shards) x N elements and what stays exposed is the last piece's transfer. Same model, same constants (they
    // describe the engines and the kernel, not the direction); checked against the one reduce-scatter workload
    // measured here (M 16384, K 3584, N 8192: 8 pieces per block, the best of 1-16).
    *schedule = FICCO_FINE_PERSISTENT;
    *chunks = pick_pieces(M, K, N, shards, N * 2);
    return FICCO_OK;
}

int ficco_pick_schedule(int64_t M, int64_t K, int64_t N, int shards, int *schedule, int *chunks)
{
    if (M < 1 || K < 1 || N < 1 || shards < 1 || !schedule || !chunks) return FICCO_ERR_ARG;
    if (M % shards) return FICCO_ERR_SHAPE;
    // Static rule in the spirit of Sec. V-C, built on the overlap model of Sec. IV-A with the two losses of
    // Sec. IV-B as per-piece costs. With c pieces per shard, all links side by side, the pair takes about
    //     T(c) = max(Tc + c * a, Tg + c * b) + min(Tc, Tg) / c
    // Tc = one shard over one link, Tg = the whole GEMM, both from machine rates (58 GB/s per copy engine, 1.2e15
    // flop/s sustained by the GEMM kernel); a = 16 us is what one more piece costs a link (the gap an engine leaves
    // between copies and the lower rate of small copies: the communication DIL), b = 8 us what it costs the GEMM
    // (GEMM DIL). The first term is the longer side stretched by its own per-piece cost, the second what stays
    // exposed of the shorter side: the first piece's transfer or the last piece's GEMM. c = the power of two up to
    // 32 that divides the shard, keeps pieces of at least 256 rows and minimises T. Among the schedules the resident
    // kernel was the fastest at every point of the sweep, so the schedule itself needs no threshold. a, b and the
    // row limit were fitted to the 24-shape sweep and scored on 16 shapes off its grid.
    const int c = pick_pieces(M, K, N, shards, K * 2);
    const int sch = FICCO_FINE_PERSISTENT;
    *schedule = sch;
    *chunks = c;
    return FICCO_OK;
}

int ficco_pick_schedule_layout(int64_t M, int64_t K, int64_t N, int shards, int source_layout, int *schedule, int *chunks)
{
    if (source_layout < FICCO_LAYOUT_ROW_MAJOR || source_layout > FICCO_LAYOUT_ROW_MAJOR_HOST) return FICCO_ERR_ARG;
    int rc = ficco_pick_schedule(M, K, N, shards, schedule, chunks);
    if (rc) return rc;
    // Row-major shards in pinned host memory: the runtime puts every rectangular copy on one engine, which then
    // carries the whole matrix at 47-53 GB/s where row pieces use the host link's full rate; row pieces were ahead
    // at every shape tried (e.g. M 4096, K 16384, N 4096: 2.56 ms against 2.72-3.25 ms with 2-8 column pieces).
    if (source_layout == FICCO_LAYOUT_ROW_MAJOR_HOST) return FICCO_OK;
    // Column pieces (the paper's 2D shape, Sec. V-C picks it from M against K) pay off on this machine when
    // the output is no more than one round of 256x256 tiles over the 256 CUs: then every tile can make progress
    // with every slice, while row pieces would leave most tiles waiting for their own piece. With a second,
    // partly filled round every tile of it would wait for the whole first round (measured: 18 % more tiles than
    // CUs made column pieces 18-37 % slower than row pieces).
    if (K % kBK != 0 || ((M + 255) / 256) * ((N + 255) / 256) > 256) return FICCO_OK;
    const double flops = 2.0 * (double)M * (double)N * (double)K;
    const bool transfer_bound = (double)N * shards <= 8192.0;     // GEMM time over transfer time grows with N*shards
    int sl;
    if (source_layout == FICCO_LAYOUT_K_SLICED) {
        // The sender holds its slices ready for DMA. Two slices when the transfers are the longer side (see
        // ficco_pick_slice_widths for their cut), else 2, from 1e11 flop 4, from 4e11 flop 8 (the more the GEMM
        // weighs, the earlier it should start). Fitted to the 24-shape sweep and the M <= K workload of the bench.
        sl = transfer_bound ? 2 : flops < 1.0e11 ? 2 : flops < 4.0e11 ? 4 : 8;
    } else {
        // The caller's row-major matrix: the step also pays for the sender-side re-layout (device sources) or
        // moves strided rectangles (pinned host sources). Where the transfers are the longer side that delay
        // lands on the critical path and row pieces stay ahead (measured at all eight transfer-bound shapes
        // tried); where the GEMM is the longer side and weighs at least 2e11 flop the re-layout hides behind
        // it and column pieces keep a lead of 9-13 %.
        if (transfer_bound || flops < 2.0e11) return FICCO_OK;
        sl = flops < 4.0e11 ? 4 : 8;
    }
    while (sl > 1 && sl > K / kBK) sl /= 2;
    if (sl > 1) {
        *schedule = FICCO_FINE_2D;
        *chunks = sl;
    }
    return FICCO_OK;
}

int ficco_pick_schedule_any(int64_t M, int64_t K, int64_t N, int shards, int *schedule, int *chunks)
{
    return ficco_pick_schedule_layout(M, K, N, shards, FICCO_LAYOUT_ROW_MAJOR, schedule, chunks);
}

int ficco_pick_slice_widths(int64_t M, int64_t K, int64_t N, int shards, int slices, int64_t *widths)
{
    if (M < 1 || K < kBK || K % kBK || N < 1 || shards < 1 || slices < 1 || slices > K / kBK || !widths) return FICCO_ERR_ARG;
    const int64_t kt = K / kBK;
    if (slices == 2 && (double)N * shards <= 8192.0) {
        // Transfers are the longer side: what stays exposed is the GEMM of the last slice, so the first slice is
        // as wide as the GEMM can digest while the second one travels. Three quarters of K was the best cut, by
        // 2-7 % over two equal slices, at every transfer-bound shape tried (N 512-1024, K 4096-8192, M 4096-16384).
        int64_t first = (3 * kt + 2) / 4;
        first = std::max<int64_t>(1, std::min(first, kt - 1));
        widths[0] = first * kBK;
        widths[1] = (kt - first) * kBK;
        return FICCO_OK;
    }
    for (int sl = 0; sl < slices; ++sl) widths[sl] = kBK * (kt / slices + (sl < kt % slices ? 1 : 0));
    return FICCO_OK;
}

int ficco_plan(int64_t M, int64_t K, int64_t N, int shards, int chunks, int schedule, ficco_plan_t **out)
{
    if (!out) return FICCO_ERR_ARG;
    if (M < 1 || K < 1 || N < 1 || shards < 1) return FICCO_ERR_SHAPE;
    const bool any_shape = schedule == FICCO_AUTO_ANY;
    if (schedule == FICCO_AUTO || schedule == FICCO_AUTO_ANY) {
        int rc = schedule == FICCO_AUTO ? ficco_pick_schedule(M, K, N, shards, &schedule, &chunks)
                                        : ficco_pick_schedule_any(M, K, N, shards, &schedule, &chunks);
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
    if (M > 0x7FFFFFFF || N > 0x7FFFFFFF || K > kMaxK) return FICCO_ERR_SHAPE;
    ficco_plan_t *p = new (std::nothrow) ficco_plan_t();
    if (!p) return FICCO_ERR_ALLOC;
    p->M = M; p->K = K; p->N = N; p->G = shards; p->c = chunks; p->schedule = schedule;
    p->device = -1;                      // bound to the current device on first use
    p->order = (schedule == FICCO_SERIAL || schedule == FICCO_SHARD) ? FICCO_ORDER_SHARD_MAJOR : FICCO_ORDER_STEP_MAJOR;
    int rc = build_lists(p);
    if (rc) { delete p; return rc; }
    if (any_shape && schedule == FICCO_FINE_2D) {
        // the rule's cut of the k range comes with its answer
        std::vector<int64_t> w((size_t)chunks);
        rc = ficco_pick_slice_widths(M, K, N, shards, chunks, w.data());
        if (!rc) rc = ficco_plan_set_slice_widths(p, w.data(), chunks);
        if (rc) { delete p; return rc; }
    }
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
    if (K % 64 || N % 8 || K > kMaxK || N > 0x7FFFFFFF) return FICCO_ERR_SHAPE;
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
    if (!p || p == after) return FICCO_ERR_ARG;
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
    case FICCO_OPT_SOURCE_LAYOUT:
        if (value != FICCO_LAYOUT_ROW_MAJOR && value != FICCO_LAYOUT_K_SLICED) return FICCO_ERR_ARG;
        if (!is_2d(p) && value != FICCO_LAYOUT_ROW_MAJOR) return FICCO_ERR_ARG;      // row pieces leave a row-major source as they are
        p->src_layout = (int)value;
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

void ficco_destroy(ficco_plan_t *p)
{
    if (!p) return;
    if (p->finalized && p->run_index > 0 && p->ev_end) (void)hipEventSynchronize(p->ev_end);
    for (auto &sg : p->sig_done) hsa_signal_store_screlease(sg, 0);      // nothing may stay parked behind a piece that never completed
    for (auto &sg : p->sig_packed) hsa_signal_store_screlease(sg, 0);    // ... or behind a re-layout that never ran
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
