#!/usr/bin/env python3
"""Benchmark of the DART token-reduction hot path on one MI355X.

One step = one dart_reduce call (row norms, pivot selection, duplication scores,
score ordering, retained set, compaction) over one synthetic batch of the
headline shape: B=8 multi-crop images of N=2880 vision tokens, D=4096, bf16,
P=16 pivots, keep 320.  Inputs are resident in HBM before the timed region and
rotate through enough distinct copies (> 1 GB) that every step reads HBM-cold
data rather than the 256 MB last-level cache.

Prints ONE JSON line: throughput in input vision tokens per second; the roofline
position of the whole call (the bytes the method must move over the HIP-event
duration of one dart_reduce) with every streaming kernel's own figure beside it;
the same measurement for the video and the ragged batch (other_configs); and the
CPU oracle timed on the host cores as a baseline.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
STAGES = ["row_l1_norms", "select_pivots", "duplication_scores", "order_scores", "retain",
          "gather_compact"]
# (the score pass is k_scores_ksplit for bf16 and k_scores_f32 for fp32 rows: the prefix covers both)
STAGE_KERNELS = ["k_row_l1", "k_select_pivots", "k_scores", "k_order_scores", "k_retain",
                 "k_gather"]


TRAFFIC_FILES = {2: "hbm_traffic_multicrop_B8_N2880_D4096_bf16.txt",
                 3: "hbm_traffic_ragged_B32_D3584_bf16.txt",
                 4: "hbm_traffic_video_B4_N9216_D3584_bf16.txt"}


def measured_traffic(kernel_prefix, config=2):
    """HBM bytes per launch of a kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size); None if the
    kernel sources changed since the counters were taken.  An empty prefix sums all
    the kernels of one step."""
    import glob
    import hashlib
    try:
        lines = open(os.path.join(ROOT, "profiles", TRAFFIC_FILES[config])).read().splitlines()
    except (OSError, KeyError):
        return None
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2502_11494_amd", "csrc", "*"))):
        h.update(open(path, "rb").read())
    sha = [l.split()[1] for l in lines if l.startswith("source_sha256")]
    if not sha or sha[0] != h.hexdigest():
        return None
    total, found = 0, False
    for l in lines:
        f = l.split()
        if len(f) == 4 and f[0] == "kernel" and f[1].startswith("dart::" + kernel_prefix):
            if kernel_prefix:
                return int((float(f[2]) + float(f[3])) * 1024)
            total += int((float(f[2]) + float(f[3])) * 1024)
            found = True
    return total if found else None


class HipEvents:
    """Raw hipEvent_t handles from the HIP runtime the process already uses."""

    def __init__(self, n):
        self.hip = C.CDLL("libamdhip64.so.7")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.ev = []
        for _ in range(n):
            e = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(e)) == 0
            self.ev.append(e)

    def handles(self, lo, hi):
        return [e.value for e in self.ev[lo:hi]]

    def ms(self, a, b, missing=None):
        """Elapsed time between two events; `missing` (if given) for a pair that was never
        recorded (a stage without a kernel)."""
        out = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(out), self.ev[a], self.ev[b])
        if rc != 0 and missing is not None:
            self.hip.hipGetLastError()  # the failed query must not surface in a later HIP call
            return missing
        assert rc == 0, rc
        return out.value

    def close(self):
        for e in self.ev:
            self.hip.hipEventDestroy(e)


def bench_sequences(args):
    """Context run: the vision tokens of the workload sit inside whole sequences (text rows
    before and after); one step = dart_reduce on the spans (no gather) + dart_compact_sequences
    moving the hidden states, the key and value rows of two earlier layers and three planes of
    position ids.  Prints its own JSON line; not the headline measurement."""
    import numpy as np
    import torch

    import paper_2502_11494_amd as D
    from paper_2502_11494_amd import workloads as W

    torch.cuda.set_device(0)
    w = W.by_index(args.config)
    sq = W.sequences_around(w, seed=1, before=(30, 40), after=(20, 60), n_kv=4, kv_width=w.D)
    rows, total_N = sq.H.shape[0], int(w.cu[-1])
    total_K = sum(w.budget(b) for b in range(w.B))
    out_rows = rows - total_N + total_K

    def dev(a):
        if w.dtype == W.BF16:
            return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(a).cuda()

    srcs = [dev(sq.H)] + [dev(t) for t in sq.kv]
    copies = 6  # rotate the hidden states so that every step reads them from HBM
    Hs = [srcs[0]] + [srcs[0].clone() for _ in range(copies - 1)]
    dsts = [torch.empty((out_rows, t.shape[1]), dtype=t.dtype, device="cuda") for t in srcs]
    cu_dev, span_dev = torch.from_numpy(w.cu).cuda(), torch.from_numpy(sq.span_start).cuda()
    seq_dev = torch.from_numpy(sq.seq_cu).cuda()
    desc = D.make_desc(w.B, w.D, w.P, w.dtype, K=w.K, keep_num=w.keep_num, keep_den=w.keep_den,
                       cu_seqlens=cu_dev, total_N=total_N, max_N=int(w.lengths.max()),
                       span_start=span_dev, X_rows=rows)
    ws = D.alloc_workspace(desc)
    keep = torch.empty(total_K, dtype=torch.int32, device="cuda")
    row_map = torch.empty(out_rows, dtype=torch.int32, device="cuda")
    seq_out = torch.empty(w.B + 1, dtype=torch.int32, device="cuda")
    posd = torch.from_numpy(sq.pos).cuda()
    pos_out = torch.empty((3, out_rows), dtype=torch.int64, device="cuda")

    def compact(i):
        D.dart_compact_sequences(desc, seq_dev, keep, [(Hs[i % copies], dsts[0])] +
                                 list(zip(srcs[1:], dsts[1:])), seq_out, row_map, ws, pos=posd,
                                 pos_out=pos_out)

    def step(i):
        D.dart_reduce(desc, Hs[i % copies], None, keep, ws)
        compact(i)

    def timed(fn):
        for i in range(args.warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            fn(args.warmup + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    t_step = timed(step)
    t_compact = timed(compact)
    assert D.dart_device_status(desc, ws) == D.DART_OK and int(seq_out[-1]) == out_rows
    moved = 2 * out_rows * sum(t.shape[1] * t.element_size() for t in srcs) + 2 * 3 * 8 * out_rows
    print(json.dumps({
        "metric": "sequence_rows_per_s", "value": round(rows / t_step, 1), "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t_step * 1e3, 5), "higher_is_better": True, "data": "synthetic",
        "dtype": "bf16" if w.dtype == W.BF16 else "f32",
        "config": {"workload": f"configs[{args.config}] {w.name} inside whole sequences: "
                               f"{rows} rows, {total_N} vision tokens -> {total_K}, "
                               f"hidden states + 4 cached key/value tensors of width {w.D}"},
        "compaction": {"ms": round(t_compact * 1e3, 5), "rows_out": out_rows,
                       "algorithmic_bytes": moved,
                       "achieved_GBps": round(moved / t_compact / 1e9, 1),
                       "frac_of_hbm_peak": round(moved / t_compact / 1e9 / HBM_PEAK_GBS, 4),
                       "note": "wall clock over the call's kernels (offsets, row map, row "
                               "gather, position ids); the cached key/value tensors are not "
                               "rotated and fit the memory-side cache"}}))


def bench_norms_given(args):
    """Context run: the criterion norms come from the caller (dart_reduce_with_norms; here they
    are computed once, outside the timed region, by dart_select_pivots), so the step has no
    norm pass and reads the hidden states once.  Prints its own JSON line; not the headline
    measurement."""
    import torch

    import paper_2502_11494_amd as D
    from paper_2502_11494_amd import workloads as W

    torch.cuda.set_device(0)
    w = W.by_index(args.config)
    total_N = int(w.cu[-1])
    total_K = sum(w.budget(b) for b in range(w.B))
    esz = 2 if w.dtype == W.BF16 else 4
    X0 = (torch.from_numpy(w.X.view("int16")).view(torch.bfloat16) if w.dtype == W.BF16
          else torch.from_numpy(w.X)).cuda()
    copies = max(2, -(-(1 << 30) // (total_N * w.D * esz)))  # rotate through more than 1 GB
    Xs = [X0] + [X0.clone() for _ in range(copies - 1)]
    cu_dev = torch.from_numpy(w.cu).cuda() if w.ragged else None
    if w.ragged:
        desc = D.make_desc(w.B, w.D, w.P, w.dtype, keep_num=w.keep_num, keep_den=w.keep_den,
                           cu_seqlens=cu_dev, total_N=total_N, max_N=int(w.lengths.max()))
    else:
        desc = D.make_desc(w.B, w.D, w.P, w.dtype, N=int(w.lengths[0]), K=w.K)
    ws = D.alloc_workspace(desc)
    pos = torch.from_numpy(w.pos).cuda()
    Y = torch.empty((total_K, w.D), dtype=X0.dtype, device="cuda")
    keep = torch.empty(total_K, dtype=torch.int32, device="cuda")
    pos_out = torch.empty(total_K, dtype=torch.int64, device="cuda")
    piv = torch.empty(w.B * w.P, dtype=torch.int32, device="cuda")
    l1 = torch.empty(total_N, dtype=torch.float32, device="cuda")
    D.dart_select_pivots(desc, X0, piv, ws, l1_out=l1)  # the library's own fp32 norms
    torch.cuda.synchronize()
    rel_err = 2e-6  # above the norm pass's rounding bound for these row widths

    def step(i):
        D.dart_reduce_with_norms(desc, Xs[i % copies], Y, keep, ws, l1, rel_err, pos=pos,
                                 pos_out=pos_out)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps
    _, compulsory, _ = whole_call_bytes(total_N, total_K, w.D, esz)
    print(json.dumps({
        "metric": "vision tokens reduced/sec with the criterion norms supplied by the caller",
        "value": round(total_N / t_step, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(t_step * 1e3, 5),
        "higher_is_better": True, "data": "synthetic",
        "dtype": "bf16" if w.dtype == W.BF16 else "f32",
        "config": {"workload": workload_label(w, args.config, False),
                   "path": "dart_reduce_with_norms: no norm pass, the hidden states are read once",
                   "input_copies_rotated": copies},
        "whole_path_algorithmic_GBps": round(compulsory / t_step / 1e9, 1),
        "frac_of_hbm_peak": round(compulsory / t_step / 1e9 / HBM_PEAK_GBS, 4)}))


def whole_call_bytes(total_N, total_K, D_, esz):
    """Algorithmic HBM bytes of one dart_reduce call: what the method must move (read every
    hidden-state row once, write the retained rows, read and write their position ids), and
    what the two-pass schedule moves (the pivots are not known before every norm is, so X is
    read twice; the gather reads the retained rows once more)."""
    x_bytes = total_N * D_ * esz
    compulsory = x_bytes + total_K * D_ * esz + 16 * total_K
    two_pass = 2 * x_bytes + 2 * total_K * D_ * esz + 16 * total_K
    return x_bytes, compulsory, two_pass


def measure(w, args, config_index, steps, warmup, variants=True):
    """Times dart_reduce on one workload (HBM-cold inputs: the batch rotates through more
    than 1 GB of copies).  Returns the figures of the bench line for that workload."""
    import numpy as np
    import torch

    import paper_2502_11494_amd as D
    from paper_2502_11494_amd import workloads as W

    total_N = int(w.cu[-1])
    total_K = sum(w.budget(b) for b in range(w.B))
    esz = 2 if w.dtype == W.BF16 else 4
    x_bytes, compulsory, two_pass = whole_call_bytes(total_N, total_K, w.D, esz)
    # the counter figures under profiles/ were taken on the plain run of this workload only
    plain = (config_index in TRAFFIC_FILES and not args.workload and args.p_ext == 0
             and args.crit_d == 0 and args.score_mode == 0 and not args.hot and not args.fused)

    if w.dtype == W.BF16:
        X0 = torch.from_numpy(w.X.view(np.int16)).view(torch.bfloat16).cuda()
    else:
        X0 = torch.from_numpy(w.X).cuda()
    copies = max(2, -(-(1 << 30) // x_bytes) + 1)
    copies = min(copies, max(2, int(64e9 // x_bytes)))
    if args.hot:
        copies = 1
    Xs = [X0] + [X0.clone() for _ in range(copies - 1)]
    pos = torch.from_numpy(w.pos).cuda()
    cu_dev = torch.from_numpy(w.cu).cuda() if w.ragged else None
    lens = w.lengths
    ext = None
    if args.p_ext > 0:
        E = W.text_pivot_rows(w, args.p_ext).reshape(-1, w.D)
        ext = (torch.from_numpy(E.view(np.int16)).view(torch.bfloat16) if w.dtype == W.BF16
               else torch.from_numpy(E)).cuda()
    more = dict(score_mode=args.score_mode, ext_pivots=ext, P_ext=args.p_ext)
    if args.random_pivots >= 0:
        more.update(pivot_mode=D.DART_PIVOT_RANDOM, seed=args.random_pivots)
    if w.ragged:
        desc = D.make_desc(w.B, w.D, w.P, w.dtype, keep_num=w.keep_num, keep_den=w.keep_den,
                           cu_seqlens=cu_dev, total_N=total_N, max_N=int(lens.max()), **more)
    else:
        desc = D.make_desc(w.B, w.D, w.P, w.dtype, N=int(lens[0]), K=w.K, **more)
    ws = D.alloc_workspace(desc)
    tile_w, tile_ks = (D.dart_score_tile_shape_first_read(desc) if args.crit_d > 0 else
                       D.dart_score_tile_shape(desc))
    score_tile = (None if tile_w == 0 else
                  {"waves": tile_w, "groups": tile_ks, "rows": 16 * tile_w // tile_ks})
    Y = torch.empty((total_K, w.D), dtype=X0.dtype, device="cuda")
    keep = torch.empty(total_K, dtype=torch.int32, device="cuda")
    pos_out = torch.empty(total_K, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream()

    ckw = {}
    if args.crit_d > 0:
        cb = W.key_states(w, args.crit_d)
        crit = (torch.from_numpy(cb.view(np.int16)).view(torch.bfloat16) if w.dtype == W.BF16
                else torch.from_numpy(cb)).cuda()
        ckw = dict(crit=crit, crit_D=args.crit_d, crit_ld=args.crit_d)

    def step(i):
        D.dart_reduce(desc, Xs[i % copies], Y, keep, ws, pos=pos, pos_out=pos_out, stream=stream,
                      **ckw)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    tokens_per_s = total_N * steps / wall

    # spread of the step time: ten further groups of steps, each timed like the region above
    per = max(1, steps // 10)
    groups = []
    for gi in range(10):
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for i in range(per):
            step(warmup + gi * per + i)
        torch.cuda.synchronize()
        groups.append((time.perf_counter() - tg) * 1e3 / per)
    groups.sort()
    spread = {"median": round(groups[5], 5), "min": round(groups[0], 5), "max": round(groups[-1], 5),
              "groups": 10, "steps_per_group": per}

    # per-kernel durations: the same steps again (the kernel-per-step path), every stage's
    # kernels stamping a pair of HIP events with their own begin and end on the stream they
    # run on (start/stop events of the launch: no packets between the kernels)
    evs = HipEvents(12 * steps)
    for i in range(steps):
        D.dart_reduce_profiled(desc, Xs[(warmup + i) % copies], Y, keep, ws,
                               evs.handles(12 * i, 12 * i + 12), pos=pos, pos_out=pos_out,
                               stream=stream, **ckw)
    torch.cuda.synchronize()
    stage_ms = [sum(evs.ms(12 * i + 2 * s, 12 * i + 2 * s + 1, missing=0.0)
                    for i in range(steps)) / steps for s in range(6)]
    evs.close()
    # the whole call: one event pair around each plain dart_reduce (no events inside it)
    evs = HipEvents(2 * steps)
    for i in range(steps):
        assert evs.hip.hipEventRecord(evs.ev[2 * i], C.c_void_p(stream.cuda_stream)) == 0
        step(warmup + i)
        assert evs.hip.hipEventRecord(evs.ev[2 * i + 1], C.c_void_p(stream.cuda_stream)) == 0
    torch.cuda.synchronize()
    call_ms = sum(evs.ms(2 * i, 2 * i + 1) for i in range(steps)) / steps
    evs.close()
    # algorithmic bytes of one launch of each streaming kernel
    alg_bytes = {
        0: (total_N * args.crit_d * esz if args.crit_d > 0 else x_bytes) + 4 * total_N,  # norms
        2: x_bytes + 4 * w.P * total_N + w.B * w.P * w.D * esz,     # read X + pivots, write S
        5: 2 * total_K * w.D * esz + 16 * total_K + 4 * total_K,    # rows + position ids
    }
    kernels = {}
    for s_, name in ((0, STAGE_KERNELS[0]),
                     (2, "k_scores_f32" if w.dtype != W.BF16 else STAGE_KERNELS[2]),
                     (5, STAGE_KERNELS[5])):
        gbps = alg_bytes[s_] / (stage_ms[s_] * 1e-3) / 1e9
        kernels[name] = {"algorithmic_bytes": alg_bytes[s_], "event_us": round(stage_ms[s_] * 1e3, 2),
                         "achieved": round(gbps, 1), "frac": round(gbps / HBM_PEAK_GBS, 4),
                         "traffic": measured_traffic(STAGE_KERNELS[s_], config_index) if plain else None}
    dom = max((0, 2, 5), key=lambda s_: stage_ms[s_])
    dom_name = "k_scores_f32" if dom == 2 and w.dtype != W.BF16 else STAGE_KERNELS[dom]
    counter_bytes = measured_traffic("", config_index) if plain else None
    achieved = compulsory / (call_ms * 1e-3) / 1e9
    roofline = {
        # the whole call: the bytes the method must move over the event-timed duration of one
        # dart_reduce (all of its kernels, on the stream they run on)
        "bound": "hbm", "scope": "whole dart_reduce call (6 kernels; 7 with ragged offsets)",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "algorithmic_bytes": compulsory, "call_event_us": round(call_ms * 1e3, 2),
        "traffic": counter_bytes,
        "traffic_source": (("profiles/" + TRAFFIC_FILES[config_index] + " (rocprofv3 FETCH_SIZE + "
                            "WRITE_SIZE of an earlier run of this command on the same sources; "
                            "not a counter of this run)") if counter_bytes is not None else None),
        "two_pass_schedule": {"bytes": two_pass,
                              "achieved": round(two_pass / (call_ms * 1e-3) / 1e9, 1),
                              "frac": round(two_pass / (call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "counter_frac": (None if counter_bytes is None else
                         round(counter_bytes / (call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)),
        "dominant_kernel": dom_name,
        "kernels": kernels,
        "stage_us": {STAGES[s_]: round(stage_ms[s_] * 1e3, 2) for s_ in range(6)},
        "on_chip_us": round((stage_ms[1] + stage_ms[3] + stage_ms[4]) * 1e3, 2),
    }
    out = {
        "ms_per_step": round(ms_per_step, 5), "tokens_per_s": round(tokens_per_s, 1),
        "tokens_removed_per_s": round((total_N - total_K) * steps / wall, 1),
        "steps": steps, "warmup": warmup, "total_tokens": total_N, "retained_tokens": total_K,
        "input_copies_rotated": copies, "score_tile": score_tile,
        "whole_path_algorithmic_GBps": round(compulsory / (ms_per_step * 1e-3) / 1e9, 1),
        "whole_path_counter_GBps": (None if counter_bytes is None else
                                    round(counter_bytes / (ms_per_step * 1e-3) / 1e9, 1)),
        "ms_per_step_spread": spread, "roofline": roofline,
    }
    if not variants:
        return out

    # context: independent batches in flight on several streams (default priority), so that
    # the on-chip kernels of one batch overlap the streaming passes of another
    concurrent = None
    if args.streams > 1:
        ns = args.streams
        sts = [torch.cuda.Stream() for _ in range(ns)]
        wss = [D.alloc_workspace(desc) for _ in range(ns)]
        Ys = [torch.empty_like(Y) for _ in range(ns)]
        keeps = [torch.empty_like(keep) for _ in range(ns)]
        pouts = [torch.empty_like(pos_out) for _ in range(ns)]

        def cstep(i):
            q = i % ns
            D.dart_reduce(desc, Xs[i % copies], Ys[q], keeps[q], wss[q], pos=pos,
                          pos_out=pouts[q], stream=sts[q], **ckw)

        for i in range(warmup):
            cstep(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            cstep(warmup + i)
        torch.cuda.synchronize()
        cwall = time.perf_counter() - t0
        same = all(torch.equal(k, keep) for k in keeps)
        concurrent = {"streams": ns, "ms_per_step": round(cwall * 1e3 / steps, 5),
                      "tokens_per_s": round(total_N * steps / cwall, 1),
                      "outputs_equal_single_stream": bool(same)}

    # context: the same steps replayed from HIP graphs (one captured step per input copy)
    graphed = None
    if args.graph:
        side = torch.cuda.Stream()
        graphs = []
        with torch.cuda.stream(side):
            for c in range(copies):
                gph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gph, stream=side):
                    D.dart_reduce(desc, Xs[c], Y, keep, ws, pos=pos, pos_out=pos_out, **ckw)
                graphs.append(gph)
        torch.cuda.synchronize()
        for i in range(warmup):
            graphs[i % copies].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[(warmup + i) % copies].replay()
        torch.cuda.synchronize()
        gwall = time.perf_counter() - t0
        graphed = {"ms_per_step": round(gwall * 1e3 / steps, 5),
                   "tokens_per_s": round(total_N * steps / gwall, 1)}
    # context: the same steps with the criterion norms supplied by the caller (here: the
    # library's own fp32 norms of the first input copy, computed outside the timed region; the
    # copies hold the same rows), so that the step has no norm pass and reads X once
    norms_given = None
    plain_pivots = (args.score_mode == 0 and args.p_ext == 0 and args.crit_d == 0 and
                    args.random_pivots < 0)
    if plain_pivots:
        l1 = torch.empty(total_N, dtype=torch.float32, device="cuda")
        pivs = torch.empty(w.B * w.P, dtype=torch.int32, device="cuda")
        D.dart_select_pivots(desc, Xs[0], pivs, ws, l1_out=l1, stream=stream)
        keep_n, Y_n = torch.empty_like(keep), torch.empty_like(Y)

        def nstep(i):
            D.dart_reduce_with_norms(desc, Xs[i % copies], Y_n, keep_n, ws, l1, 2e-6, pos=pos,
                                     pos_out=pos_out, stream=stream)

        for i in range(warmup):
            nstep(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            nstep(warmup + i)
        torch.cuda.synchronize()
        nwall = time.perf_counter() - t0
        norms_given = {"entry": "dart_reduce_with_norms", "ms_per_step": round(nwall * 1e3 / steps, 5),
                       "tokens_per_s": round(total_N * steps / nwall, 1),
                       "whole_path_algorithmic_GBps": round(compulsory / (nwall / steps) / 1e9, 1),
                       "outputs_equal_plain_call": bool(torch.equal(keep_n, keep) and
                                                        torch.equal(Y_n, Y))}
    out["concurrent_streams"] = concurrent
    out["graph_replay"] = graphed
    out["norms_supplied_by_caller"] = norms_given
    return out


def workload_label(w, index, extra):
    lens = w.lengths
    return (f"{'extra' if extra else f'configs[{index}]'} {w.name}: B={w.B} "
            f"N={'ragged' if w.ragged else int(lens[0])} D={w.D} P={w.P} "
            f"K={w.K if w.K else f'floor({w.keep_num}/{w.keep_den} N)'}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload 0..4 (2 is the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the video and ragged batches that the default run times after "
                         "the headline shape (other_configs in the output)")
    ap.add_argument("--score-mode", type=int, default=0, choices=[0, 1, 2],
                    help="0 = a threshold per pivot (the headline), 1/2 = one threshold on the "
                         "min/max aggregate (variant, context only)")
    ap.add_argument("--p-ext", type=int, default=0,
                    help="variant, context only: the last P_EXT of the workload's pivots are "
                         "synthetic text-token rows from outside the samples")
    ap.add_argument("--random-pivots", type=int, default=-1, metavar="SEED",
                    help="context run: pivots drawn at random from SEED (DART_PIVOT_RANDOM, the "
                         "random rows of the pivot ablation) instead of the largest norms")
    ap.add_argument("--workload", default="", choices=["", "audio", "action", "wide13b", "wide72b"],
                    help="context only: a shape beyond the five configurations (audio tokens, "
                         "a vision-language-action model, 13B / 72B hidden sizes)")
    ap.add_argument("--crit-d", type=int, default=0,
                    help="variant, context only: pivots by the L1 norm of separate key-state "
                         "rows of this width (grouped-query shapes, e.g. 1024) instead of the "
                         "hidden states")
    ap.add_argument("--streams", type=int, default=2,
                    help="context only: after the headline measurement, run the same number of "
                         "steps spread over this many HIP streams (independent batches in "
                         "flight, each with its own workspace and outputs) and report that "
                         "rate as concurrent_streams")
    ap.add_argument("--graph", action="store_true",
                    help="context only: also time the steps replayed from captured HIP graphs")
    ap.add_argument("--sequences", action="store_true",
                    help="context run: spans inside whole sequences and whole-sequence "
                         "compaction (prints its own line)")
    ap.add_argument("--norms-given", action="store_true",
                    help="context run: the criterion norms are supplied by the caller "
                         "(dart_reduce_with_norms: no norm pass; prints its own line)")
    ap.add_argument("--fused", action="store_true",
                    help="context run: the one-launch persistent kernel (DART_FUSED=1) instead of "
                         "the default kernel-per-step path")
    ap.add_argument("--hot", action="store_true",
                    help="context run: the same input buffer every step (cache-hot), not the "
                         "headline measurement")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the reduction step is per-sample work with no "
              "cross-GPU exchange; shard the batch by sample and run one process per GPU "
              "(use --gpus 1).",
              file=sys.stderr)
        sys.exit(2)

    if args.fused:
        os.environ["DART_FUSED"] = "1"
    import torch

    from paper_2502_11494_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    from paper_2502_11494_amd.build import ensure_built
    ensure_built()  # loads what is built; compiles only a missing or stale library
    if args.sequences:
        return bench_sequences(args)
    if args.norms_given:
        return bench_norms_given(args)
    torch.cuda.set_device(0)
    w = W.by_name(args.workload) if args.workload else W.by_index(args.config)
    m = measure(w, args, args.config, args.steps, args.warmup)
    total_N = m["total_tokens"]

    # the other two shapes the bandwidth target names, timed the same way in this process
    default_run = (args.config == 2 and not args.workload and args.p_ext == 0 and args.crit_d == 0
                   and args.score_mode == 0 and not args.hot and not args.fused)
    others = None
    if default_run and not args.no_other_configs:
        others = {}
        for idx, steps in ((4, max(20, args.steps // 2)), (3, max(10, args.steps // 5))):
            wo = W.by_index(idx)
            mo = measure(wo, args, idx, steps, max(3, args.warmup // 4), variants=False)
            mo["workload"] = workload_label(wo, idx, False)
            others[f"configs[{idx}]"] = mo
            del wo
            torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.set_threads(0)
        t0 = time.perf_counter()
        reps = 0
        while True:
            for b in range(w.B):
                lo, hi = int(w.cu[b]), int(w.cu[b + 1])
                oracle.reduce(w.X[lo:hi], w.dtype, w.P, w.budget(b), pos=w.pos[lo:hi])
            reps += 1
            if time.perf_counter() - t0 > 10.0 or reps >= 20:
                break
        cpu_wall = time.perf_counter() - t0
        cpu = {"value": round(total_N * reps / cpu_wall, 1), "unit": "tokens/s", "cores": threads,
               "kind": "oracle",
               "sample": f"the whole {w.name} batch ({total_N} tokens), {reps} passes"}
        # the same oracle on one thread, one sample (context for the threaded figure)
        oracle.set_threads(1)
        lo, hi = int(w.cu[0]), int(w.cu[1])
        t0 = time.perf_counter()
        oracle.reduce(w.X[lo:hi], w.dtype, w.P, w.budget(0), pos=w.pos[lo:hi])
        cpu["single_thread_value"] = round((hi - lo) / (time.perf_counter() - t0), 1)
        try:
            with open("/proc/cpuinfo") as f:
                models = [l.split(":", 1)[1].strip() for l in f if l.startswith("model name")]
            cpu["cpu_model"] = models[0] if models else None
            cpu["host_logical_cpus"] = os.cpu_count()
        except OSError:
            pass
        oracle.set_threads(0)

    out = {
        "metric": "vision tokens reduced/sec (input tokens per dart_reduce call), "
                  "N=2880 D=4096 bf16",
        "value": m["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": m["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.dtype == W.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": workload_label(w, args.config, bool(args.workload)),
                   "path": ("one persistent kernel (DART_FUSED=1)" if args.fused
                            else "one kernel per step"),
                   "score_mode": ["per-pivot thresholds", "one threshold on the minimum",
                                  "one threshold on the maximum"][args.score_mode],
                   "pivots_from_outside": args.p_ext,
                   "criterion": (f"none: pivots drawn at random from seed {args.random_pivots}"
                                 if args.random_pivots >= 0 else
                                 f"separate key-state rows of width {args.crit_d}"
                                 if args.crit_d > 0 else "the hidden states themselves"),
                   "total_tokens": total_N, "retained_tokens": m["retained_tokens"],
                   "input_copies_rotated": m["input_copies_rotated"],
                   "score_tile": m["score_tile"]},
        "tokens_removed_per_s": m["tokens_removed_per_s"],
        "whole_path_algorithmic_GBps": m["whole_path_algorithmic_GBps"],
        "whole_path_counter_GBps": m["whole_path_counter_GBps"],
        "ms_per_step_spread": m["ms_per_step_spread"],
        "inputs": "cache-hot (same buffer every step)" if args.hot else "HBM-cold (rotating copies)",
        "concurrent_streams": m.get("concurrent_streams"),
        "graph_replay": m.get("graph_replay"),
        "norms_supplied_by_caller": m.get("norms_supplied_by_caller"),
        "roofline": m["roofline"],
        "other_configs": others,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
