// Runs of libficco: ficco_run (backend choice and the stream backend), HIP-graph capture and replay,
// statistics and the decomposition / contention profiler. See include/ficco.h for the contract of
// every entry point.
#include "ficco_plan.h"

using namespace ficco;

extern "C" {

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
    // column pieces leave a row-major source as rectangular engine copies or through the re-layout kernel, both on
    // the engine backend; the stream backend moves K-sliced sources only
    if (is_2d(p) && do_copy && p->src_layout == FICCO_LAYOUT_ROW_MAJOR) return FICCO_ERR_ARG;
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

int ficco_graph_capture(ficco_plan_t *p, const void *A_src, void *A_dev, const void *W_dev, void *C_dev,
                        void *const *peer_out)
{
    if (!p || !A_dev || !W_dev || !C_dev) return FICCO_ERR_ARG;
    if (is_resident(p) || p->grouped || p->timing || p->packing || p->mode != FICCO_MODE_PAIR) return FICCO_ERR_ARG;
    if (p->backend_opt == FICCO_COPY_ENGINES) return FICCO_ERR_ARG;      // engine submissions are host calls, not stream work
    if (p->link || p->chain_from) return FICCO_ERR_ARG;                  // chained plans run on the engines
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
            busy += (double)(t.end - t.start) / engine_ticks_per_us();
        }
        if (t_max > t_min) s.copy_span_us = (double)(t_max - t_min) / engine_ticks_per_us();
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
                    (tt[q].start - t0) / engine_ticks_per_us(), (tt[q].end - t0) / engine_ticks_per_us(),
                    (tf[q].start - t0) / engine_ticks_per_us(), (tf[q].end - t0) / engine_ticks_per_us());
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
                                (tt[q].start - t0) / engine_ticks_per_us(), (tt[q].end - t0) / engine_ticks_per_us(),
                                (tf[q].start - t0) / engine_ticks_per_us(), (tf[q].end - t0) / engine_ticks_per_us());
                }
            }
            s.timed_out = 1;
            for (auto &sg : p->sig_done) hsa_signal_store_screlease(sg, 0);   // let parked copies go
            for (auto &sg : p->sig_packed) hsa_signal_store_screlease(sg, 0);
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
                    b = (double)(t.start - t_first) / engine_ticks_per_us();
                    e = (double)(t.end - t_first) / engine_ticks_per_us();
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

    // mean span of one mode over `iters` runs after `warmup`; `repeat` > 1 (GEMM alone): every run enqueues the
    // plan's launches that many times back to back inside its bracket of events and the span is divided by it
    auto measure = [&](ficco_plan_t *q, int mode, int timing, int repeat, double *gemm_us, double *copy_us, double *busy_us) -> int {
        int r = ficco_plan_set(q, FICCO_OPT_MODE, mode);
        if (r) return r;
        if ((r = ficco_plan_set(q, FICCO_OPT_TIMING, timing))) return r;
        if ((r = ficco_plan_set(q, FICCO_OPT_REPEAT, repeat))) return r;
        double g = 0, cp = 0, bz = 0;
        for (int it = 0; it < warmup + iters; ++it) {
            if ((r = ficco_run(q, A_src, A_dev, W_dev, C_dev, nullptr, compute_stream, copy_stream))) return r;
            ficco_stats_t s;
            if ((r = ficco_query_stats(q, &s))) return r;
            if (it >= warmup) { g += s.gemm_span_us / repeat; cp += s.copy_span_us; bz += s.gemm_busy_us; }
        }
        if (gemm_us) *gemm_us = g / iters;
        if (copy_us) *copy_us = cp / iters;
        if (busy_us) *busy_us = bz / iters;
        return ficco_plan_set(q, FICCO_OPT_REPEAT, 1);
    };

    ficco_losses_t L{};
    const int saved_repeat = p->repeat;
    constexpr int kRepeat = 8;
    do {
        // After an idle spell the shader clock needs some tens of milliseconds of load to settle: the whole GEMM
        // runs back to back until 40 ms of it have passed before anything is measured.
        {
            if ((rc = ficco_plan_set(whole, FICCO_OPT_MODE, FICCO_MODE_GEMM_ONLY))) break;
            if ((rc = ficco_plan_set(whole, FICCO_OPT_REPEAT, kRepeat))) break;
            double burnt_us = 0;
            while (burnt_us < 40e3 && !rc) {
                if ((rc = ficco_run(whole, A_src, A_dev, W_dev, C_dev, nullptr, compute_stream, copy_stream))) break;
                ficco_stats_t s;
                if ((rc = ficco_query_stats(whole, &s))) break;
                burnt_us += s.wall_us > 1.0 ? s.wall_us : 1.0;
            }
            if (rc) break;
        }
        // decomposition loss: both sides as launches back to back, clocks settled
        if ((rc = measure(whole, FICCO_MODE_GEMM_ONLY, 0, kRepeat, &L.t_gemm_whole_us, nullptr, nullptr))) break;
        if ((rc = measure(p, FICCO_MODE_GEMM_ONLY, 0, kRepeat, &L.t_gemm_pieces_us, nullptr, nullptr))) break;
        // the launches' own durations summed (an event before and after each): what is left of the span are dispatch gaps
        if ((rc = measure(p, FICCO_MODE_GEMM_ONLY, 1, 1, nullptr, nullptr, &L.t_gemm_pieces_busy_us))) break;
        // contention loss: one run per bracket on both sides, so that the two are taken the same way
        if ((rc = measure(p, FICCO_MODE_GEMM_ONLY, 0, 1, &L.t_gemm_pieces_single_us, nullptr, nullptr))) break;
        if ((rc = measure(whole, FICCO_MODE_COPY_ONLY, 0, 1, nullptr, &L.t_copy_whole_us, nullptr))) break;
        if ((rc = measure(p, FICCO_MODE_COPY_ONLY, 0, 1, nullptr, &L.t_copy_pieces_us, nullptr))) break;
        if ((rc = measure(p, FICCO_MODE_INDEPENDENT, 0, 1, &L.t_gemm_pieces_cont_us, &L.t_copy_pieces_cont_us, nullptr))) break;
    } while (0);
    ficco_destroy(whole);
    p->mode = saved_mode;
    p->timing = saved_timing;
    p->repeat = saved_repeat;
    if (rc) return rc;
    L.gemm_dil = L.t_gemm_pieces_us / L.t_gemm_whole_us;
    L.gemm_cil = L.t_gemm_pieces_cont_us / L.t_gemm_pieces_single_us;
    L.comm_dil = L.t_copy_pieces_us / L.t_copy_whole_us;
    L.comm_cil = L.t_copy_pieces_cont_us / L.t_copy_pieces_us;
    L.ideal_us = ficco_ideal_overlap_us(L.t_copy_whole_us, L.t_gemm_whole_us, p->schedule == FICCO_SERIAL ? 1 : ((int)p->groups.size() > 1 ? (int)p->groups.size() : p->n_chunks));
    *out = L;
    return FICCO_OK;
}

}  // extern "C"
