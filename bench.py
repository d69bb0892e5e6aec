#!/usr/bin/env python3
"""Benchmark of the chunked sparse-attention decode step on one MI355X.

A "step" is one pass of the per-decode-step hot path -- chunk_score, then
chunk_select_attention_decode (selection + attention over the kept chunks in
one call) -- over every resident layer of the workload, inputs already in HBM.
The separate chunk_topk_select and sparse_chunk_attention_decode calls are
timed on their own as well.  kv_chunk_abstract_build is the prefill-time call;
it is timed on its own and reported under "abstract_build".  kv_chunk_compress
(the builder of the 8-bit / 4-bit store; it also writes the compressed
workload's store here), kv_chunk_abstract_append and chunk_tree_refine are
timed on their own under "compress", "abstract_append_us" and "tree_refine".

Prints ONE JSON line.  `value` is the algorithmic KV traffic of the step
(abstracts read + scores written and re-read + kept K/V rows read + q in + out
written; never the dense cache the method avoids) divided by the wall time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# resident layers per workload (every layer of c1/c2 fits; c3 keeps a spread of
# eight layers x sixteen sequences = 64 GiB of K/V so that one pass touches far
# more than any cache holds)
RESIDENT = {
    "c1": list(range(32)),
    "c2": list(range(32)),
    "c3": [0, 1, 2, 7, 15, 23, 30, 31],
    "c4": [0, 1, 2, 7, 15, 23, 30, 31],      # compressed store (8-bit / 4-bit chunks), 512K context
}
ELEM = {"f32": 4, "f16": 2, "bf16": 2}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=sorted(RESIDENT))
    ap.add_argument("--layers", type=int, default=0, help="use only the first n resident layers (0 = all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=5, help="passes of the per-kernel timing loops")
    ap.add_argument("--layer-ahead", choices=["auto", "on", "off"], default="auto",
                    help="time the layer-ahead schedules of DecodeStack as well (auto: for the batch-1 workloads c1, c2 "
                         "and c4, where they pay; their two-stream and all-layers launches would otherwise mix into the "
                         "profiler's per-kernel averages of the default c3 run)")
    return ap.parse_args()


def algorithmic_bytes(layer, case, elem, four_bit=None):
    """Bytes one layer-step has to move, by part (see module docstring).  With a
    compressed store (four_bit[b,c] given) a kept token costs 2*128 or 2*64 bytes
    and a kept chunk its 32-byte record; abstracts and q are fp16."""
    import numpy as np
    hkv, d, g = case.hkv, case.d, case.g
    chunks = int(case.n_chunks.sum().item()) * hkv                  # (b,h,c) triples
    kept_tokens = int(layer.sel_tokens.sum().item())                # over (b,h)
    kv = kept_tokens * 2 * d * elem
    if four_bit is not None:
        elem = 2
        sel = layer.sel_idx.cpu().numpy()
        sizes = np.diff(case.chunk_off.cpu().numpy().astype(np.int64), axis=1)
        kv = 0
        for b in range(sel.shape[0]):
            for h in range(sel.shape[1]):
                ids = sel[b, h][sel[b, h] >= 0]
                kv += int((sizes[b, ids] * np.where(four_bit[b, ids], d, 2 * d)).sum()) + 32 * len(ids)
    parts = {
        "abstract": chunks * 2 * d * elem,
        "score_wr_rd": chunks * 4 * 2,
        "kv": kv,
        "q_out": case.batch * case.hq * d * (elem + 4),
    }
    parts["total"] = sum(parts.values())
    parts["kept_tokens"] = kept_tokens
    parts["chunks"] = chunks
    return parts


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a plain
    copy of known size); None if there is no summary for this workload."""
    path = os.path.join(ROOT, "profiles", f"pmc_{workload}_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch") and kernel in line:
            return int(float(line.split("=")[1]))
    return None


def time_calls(fn, reps, torch):
    """Average wall time of fn() in ms over `reps` calls, HIP events on the current stream."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / reps


def percentiles(xs):
    """median, 10th and 90th percentile of a list of times"""
    import numpy as np
    a = np.asarray(xs, dtype=np.float64)
    return float(np.median(a)), float(np.percentile(a, 10)), float(np.percentile(a, 90))


def time_steps(fn, steps, torch):
    """Per-step times in ms of `steps` calls of fn(), from HIP events recorded between the steps on the
    current stream (the stream the library's kernels are launched on)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def compress_store(B, torch, case, four_bit, timed, retag=False):
    """kv_chunk_compress of one layer (Sec. 4.4 / 6.1).  Returns the blobs cut to the used bytes, the records and,
    if `timed`, the timing record: source bytes read plus code bytes written per second."""
    import numpy as np
    nb, hk, n_ctx = case.K.shape[0], case.K.shape[1], case.K.shape[2]
    c_max = case.chunk_off.shape[1] - 1
    shape = B.make_shape(nb, case.hq, hk, 128, n_ctx, c_max, 1, case.K.dtype)
    cap = B.leoam_compressed_bytes_bound(shape)
    kb = torch.empty(cap, dtype=torch.uint8, device="cuda")
    vb = torch.empty(cap, dtype=torch.uint8, device="cuda")
    qm = torch.empty(nb, hk, c_max, 8, dtype=torch.int32, device="cuda")
    used = torch.zeros(1, dtype=torch.int64, device="cuda")
    fbd = torch.from_numpy(np.ascontiguousarray(four_bit).astype(np.uint8)).cuda()
    call = lambda: B.kv_chunk_compress(shape, case.K, case.V, case.chunk_off, case.n_chunks, fbd, kb, vb, qm, used)
    rec = None
    if timed:
        ms = time_calls(call, 5, torch)
        n = int(used.item())
        src = 2 * case.K.numel() * case.K.element_size()
        rec = {"us_per_layer": round(ms * 1e3, 1), "source_bytes": src, "code_bytes": 2 * n, "four_bit_share_of_chunks": 0.5,
               "GBps_read_plus_written": round((src + 2 * n) / (ms * 1e-3) / 1e9, 1)}
        if retag:
            # the live store brought to tags that differ in a tenth of the chunks (kv_chunk_recompress):
            # only those chunks are read and encoded again
            flip = np.random.default_rng(1).random(four_bit.shape) < 0.1
            new_tags = torch.from_numpy(np.ascontiguousarray(np.logical_xor(four_bit, flip)).astype(np.uint8)).cuda()
            info = torch.zeros(3, dtype=torch.int64, device="cuda")
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            B.kv_chunk_recompress(shape, case.K, case.V, case.chunk_off, case.n_chunks, fbd, new_tags, kb, vb, qm, used, info)
            b.record()
            torch.cuda.synchronize()
            rec["recompress_tenth_of_the_tags"] = {"us": round(a.elapsed_time(b) * 1e3, 1), "chunks_encoded_again": int(info[1]),
                                                   "refused": int(info[0]), "fresh_room_bytes": int(info[2])}
    else:
        call()
        torch.cuda.synchronize()
        n = int(used.item())
    return kb[:n].clone(), vb[:n].clone(), qm, rec


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU path; run it with --gpus 1 "
              "(the path would shard by (sequence, kv head) with no exchange; that is not implemented here)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import gen
    import paper_2506_20187_amd as L

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    B = L.binding
    cfg = gen.CONFIGS[args.workload]
    layer_ids = RESIDENT[args.workload]
    if args.layers > 0:
        layer_ids = layer_ids[: args.layers]
    elem = ELEM[cfg["dtype"]]

    t0 = time.time()
    layers, cases, tags = [], [], []
    compress = None
    quant = args.workload == "c4"
    for lid in layer_ids:
        if quant:
            # the compressed store is written by the library's own compression call (half of the chunks,
            # those without a heavy token, as 4-bit); the first layer's call is timed
            case = gen.make_case("c4", layer=lid, device="cuda")
            case.q = case.q.to(torch.float16)
            fb = gen.tag_four_bit(case.chunk_off.cpu().numpy(), case.n_chunks.cpu().numpy(), case.extra["heavy"], 0.5)
            kblob, vblob, qmeta, rec = compress_store(B, torch, case, fb, timed=compress is None)
            compress = compress or rec
            lay = L.DecodeLayer(kblob, vblob, case.chunk_off, case.n_chunks, case.hq, case.k_max,
                                case.max_chunks, case.token_budget, qmeta=qmeta, n_kv_heads=case.hkv,
                                n_ctx=case.n_ctx)
            tags.append(fb)                 # (the 16-bit cache stays resident too: the policy section below compares with it)
        else:
            case = gen.make_case(args.workload, layer=lid, device="cuda")
            lay = L.DecodeLayer(case.K, case.V, case.chunk_off, case.n_chunks, case.hq, case.k_max, case.max_chunks,
                                case.token_budget)
            tags.append(None)
        layers.append(lay)
        cases.append(case)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    print(f"# generated {len(layers)} resident layers of {args.workload} in {gen_s:.1f} s", file=sys.stderr, flush=True)

    # ---- prefill-time abstract build, timed on its own -----------------------
    def build_all():
        for lay in layers:
            lay.build_abstract()
    ab_ms = time_calls(build_all, 2, torch)
    k_bytes = sum(lay.K.numel() * lay.K.element_size() for lay in layers)
    ab_out_bytes = sum(lay.abstract.numel() * lay.abstract.element_size() for lay in layers)

    # ---- the timed step ----------------------------------------------------------
    def step():
        for lay, case in zip(layers, cases):
            lay.step(case.q)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t1
    ms_per_step = wall * 1e3 / args.steps
    us_per_layer = ms_per_step * 1e3 / len(layers)

    # the same steps once more with a HIP event between them: spread of the eager step
    eager_ms = time_steps(step, args.steps, torch)
    # ... and replayed from a HIP graph that holds one step (captured on a side stream)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        graph.replay()
    graph_ms = time_steps(graph.replay, args.steps, torch)
    del graph

    parts = [algorithmic_bytes(lay, case, elem, fb) for lay, case, fb in zip(layers, cases, tags)]
    step_bytes = sum(p["total"] for p in parts)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel timing (HIP events on the launch stream) ----------------------
    def only_score():
        for lay, case in zip(layers, cases):
            B.chunk_score(lay.shape, case.q, lay.abstract, lay.n_chunks, lay.score, None)

    def only_select():
        for lay in layers:
            B.chunk_topk_select(lay.shape, lay.score, lay.chunk_off, lay.n_chunks, lay.max_chunks, lay.token_budget,
                                lay.sel_idx, lay.sel_count, lay.sel_tokens)

    def only_attention():
        for lay, case in zip(layers, cases):
            B.sparse_chunk_attention_decode(lay.shape, case.q, lay.K, lay.V, lay.chunk_off, lay.n_chunks, lay.sel_idx,
                                            lay.sel_count, lay.scale, lay.out, lay.lse, lay.att_workspace, None, lay.qmeta)

    def only_select_attention():
        for lay, case in zip(layers, cases):
            B.chunk_select_attention_decode(lay.shape, lay.score, case.q, lay.K, lay.V, lay.chunk_off, lay.n_chunks,
                                            lay.max_chunks, lay.token_budget, lay.scale, lay.sel_idx, lay.sel_count,
                                            lay.sel_tokens, lay.out, lay.lse, lay.workspace, None, lay.qmeta)

    nl = len(layers)
    score_us = time_calls(only_score, args.kernel_reps, torch) * 1e3 / nl
    select_us = time_calls(only_select, args.kernel_reps, torch) * 1e3 / nl
    attn_us = time_calls(only_attention, args.kernel_reps, torch) * 1e3 / nl
    fused_us = time_calls(only_select_attention, args.kernel_reps, torch) * 1e3 / nl
    # selection + attention: kept K/V rows, q, out, and the score rows the selection reads
    kv_bytes = sum(p["kv"] + p["q_out"] + p["score_wr_rd"] // 2 for p in parts) / nl
    abs_bytes = sum(p["abstract"] + p["score_wr_rd"] // 2 for p in parts) / nl
    attn_gbs = kv_bytes / (fused_us * 1e-6) / 1e9
    score_gbs = abs_bytes / (score_us * 1e-6) / 1e9

    # ---- layer-ahead evaluation (Sec. 4.4): the schedules of DecodeStack over the resident layers ----
    # The evaluation of a layer needs its query before the layer runs (a query supplied up front: the
    # previous step's, or a speculated one); the benchmark's queries are fixed, so every schedule
    # computes the same step.  us per layer-step, median of per-step HIP-event times.
    layer_ahead = None
    want_ahead = args.layer_ahead == "on" or (args.layer_ahead == "auto" and args.workload in ("c1", "c2", "c4"))
    if want_ahead:
        if quant:
            stack = L.DecodeStack([lay.K for lay in layers], [lay.V for lay in layers], [c.chunk_off for c in cases],
                                  [c.n_chunks for c in cases], cases[0].hq, max(c.k_max for c in cases),
                                  cases[0].max_chunks, cases[0].token_budget, qmetas=[lay.qmeta for lay in layers],
                                  n_kv_heads=cases[0].hkv, n_ctx=cases[0].n_ctx)
        else:
            stack = L.DecodeStack([c.K for c in cases], [c.V for c in cases], [c.chunk_off for c in cases],
                                  [c.n_chunks for c in cases], cases[0].hq, max(c.k_max for c in cases),
                                  cases[0].max_chunks, cases[0].token_budget)
        stack.build_abstract()
        q_all = torch.stack([c.q for c in cases]).contiguous()
        layer_ahead = {"what": "us per layer-step (median, p10, p90 of per-step HIP-event times)"}
        for name in ("step_sequential", "step_layer_ahead", "step_scores_ahead", "step_select_ahead"):
            fn = getattr(stack, name)
            for _ in range(args.warmup):
                fn(q_all)
            med, p10, p90 = percentiles(time_steps(lambda: fn(q_all), args.steps, torch))
            layer_ahead[name] = [round(med * 1e3 / nl, 2), round(p10 * 1e3 / nl, 2), round(p90 * 1e3 / nl, 2)]
        # the step must not have changed: same kept lists and outputs as the per-layer objects above
        step()
        stack.step_select_ahead(q_all)
        torch.cuda.synchronize()
        for l, lay in enumerate(layers):
            sl = slice(l * lay.shape.batch, (l + 1) * lay.shape.batch)
            assert torch.equal(stack.sel_idx[sl][:, :, : lay.shape.k_max], lay.sel_idx), "layer-ahead schedules changed a kept list"
            assert (stack.out[sl] - lay.out).abs().max().item() <= 1e-4
        del stack, q_all

    # ---- abstract maintenance for one appended token per sequence (dense stores) ----
    append_us = None
    if not quant:
        lay = layers[0]
        off2, nc2, ab2 = lay.chunk_off.clone(), (lay.n_chunks - 1).clamp(min=0), lay.abstract.clone()
        st = torch.empty(lay.shape.batch, dtype=torch.int32, device="cuda")      # last chunk dropped: >= 16 free slots
        append_us = time_calls(lambda: B.kv_chunk_abstract_append(lay.shape, lay.K, off2, nc2, 1 << 20, ab2, st), 14,
                               torch) * 1e3
        assert int(st.abs().sum()) == 0
        del off2, nc2, ab2

    # ---- tree-structured refinement (Sec. 4.2) from uniform chunks of 64 tokens --------------
    # (a) keys with planted runs of important tokens in a desert (the structure Sec. 3.5 reports for deep
    #     layers; 128 runs of 32 tokens per head, k = 4096), (b) layer 0 of the workload itself, whose
    #     Gaussian keys give loose bounds: the tree then grows towards single tokens until the round limit.
    tree = None
    if not quant:
        lay, case = layers[0], cases[0]
        cs, cap, rounds = 64, 32768, 64
        nb, hk, nctx = lay.shape.batch, lay.shape.n_kv_heads, lay.shape.n_ctx
        m0 = -(-nctx // cs)
        tshape = B.make_shape(nb, case.hq, hk, case.d, nctx, m0, 1, lay.K.dtype)
        u_off = torch.clamp(torch.arange(m0 + 1, dtype=torch.int32, device="cuda") * cs, max=nctx).repeat(nb, 1).contiguous()
        u_nc = torch.full((nb,), m0, dtype=torch.int32, device="cuda")
        u_ab = torch.empty(nb, hk, m0, 2, case.d, dtype=lay.K.dtype, device="cuda")
        r_off = torch.empty(nb, hk, cap + 1, dtype=torch.int32, device="cuda")
        r_score = torch.empty(nb, hk, cap, dtype=torch.float32, device="cuda")
        r_cnt = torch.empty(nb, hk, dtype=torch.int32, device="cuda")
        r_ev, r_st = torch.empty_like(r_cnt), torch.empty_like(r_cnt)
        tws = torch.empty(B.leoam_tree_workspace_bytes(tshape, cap), dtype=torch.uint8, device="cuda")
        Kd, qd, hot = gen.make_desert_keys(nb, hk, case.g, nctx, clusters=128, cluster_len=(32, 32), dtype=cfg["dtype"],
                                           device="cuda")
        tree = {"initial_chunk": cs, "initial_chunks_per_head": m0, "token_level_evaluations_per_head": nctx,
                "max_rounds": rounds}
        for name, Kt, qt, k_tok in (("planted_runs", Kd, qd, int(hot[0, 0].sum())), ("workload_layer", lay.K, case.q,
                                                                                  int(case.token_budget))):
            B.kv_chunk_abstract_build(tshape, Kt, u_off, u_nc, u_ab)
            tree_ms = time_calls(lambda: B.chunk_tree_refine(tshape, qt, Kt, u_ab, cs, k_tok, rounds, cap, r_off, r_score,
                                                             r_cnt, r_ev, r_st, tws), 5, torch)
            tree[name] = {"us_per_layer_step": round(tree_ms * 1e3, 1), "k_tokens": k_tok,
                          "evaluations_per_head_avg": round(float(r_ev.float().mean()), 1),
                          "final_chunks_per_head_avg": round(float(r_cnt.float().mean()), 1),
                          "node_cap_overflows": int(r_st.sum())}
        del u_ab, r_off, r_score, tws, Kd, qd

    # ---- compression of one layer's cache to the 8-bit / 4-bit store (Sec. 4.4 / 6.1), 16-bit stores -------
    if not quant and cfg["dtype"] in ("f16", "bf16"):
        case = cases[0]
        fb = gen.tag_four_bit(case.chunk_off.cpu().numpy(), case.n_chunks.cpu().numpy(), case.extra["heavy"], 0.5)
        compress = compress_store(B, torch, case, fb, timed=True, retag=True)[3]

    # ---- plain streams of known size: what this machine reads, and copies, per second -------------
    # (4 GiB: far beyond the last-level cache; the read-only rate is the measured ceiling the
    # path's HBM-bound kernels are reported against, next to the nominal 8 TB/s)
    nbytes = 1 << 32
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    read_ms = time_calls(lambda: B.leoam_read_probe(src, nbytes, sink), 10, torch)
    read_gbs = nbytes / (read_ms * 1e-3) / 1e9
    # the same read at the size of one launch of the dominant kernel (ramp-up and drain included)
    # (every repetition reads another window of the 4 GiB, so that none of it comes from the last-level cache)
    small = int(kv_bytes) // 256 * 256
    windows = [src[i * small:(i + 1) * small] for i in range(nbytes // small)]
    turn = [0]

    def read_window():
        turn[0] = (turn[0] + 1) % len(windows)
        B.leoam_read_probe(windows[turn[0]], small, sink)
    read_small_ms = time_calls(read_window, 2 * len(windows), torch)
    read_small_gbs = small / (read_small_ms * 1e-3) / 1e9
    nbytes = 1 << 30
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    copy_ms = time_calls(lambda: B.leoam_copy_probe(dst, src, nbytes), 10, torch)
    copy_gbs = 2 * nbytes / (copy_ms * 1e-3) / 1e9
    del src, dst
    # ---- dynamic compression policy (Sec. 4.4) from rates measured on this GPU, compressed workload only ----
    # The condition T0 + D (1 - theta + theta delta) / B <= Tc + D theta / R with: D = the kept K/V of a layer-step at
    # 16 bits; delta = 0.25 (16-bit -> 4-bit, Sec. 6.1); B = the rate at which a plain copy moves source bytes through
    # HBM (all tiers are in HBM here, so a copy is what a "transfer" is); T0 = the measured evaluation time
    # (chunk_score + chunk_topk_select); Tc = the measured attention over the same kept tokens at 16 bits; R from the
    # measured difference between the compressed-store attention and what its bytes alone would cost at the 16-bit
    # kernel's rate (no measurable difference: decompression is hidden, R is reported as null and taken as 1e15).
    policy = None
    if quant:
        bw = copy_gbs / 2 * 1e9
        policy = {"bandwidth_GBps": round(bw / 1e9, 1), "ratio": 0.25, "layers": {}}
        for lid, lay, case, p in zip(layer_ids, layers, cases, parts):
            dt16 = case.K.dtype
            s16 = B.make_shape(case.batch, case.hq, case.hkv, 128, case.n_ctx, lay.shape.c_max, lay.shape.k_max, dt16)
            q16 = case.q.to(dt16)
            ws16 = torch.empty((B.leoam_workspace_bytes(s16, lay.token_budget) + 15) // 16 * 16, dtype=torch.uint8, device="cuda")
            out16 = torch.empty_like(lay.out)
            t16 = time_calls(lambda: B.sparse_chunk_attention_decode(s16, q16, case.K, case.V, lay.chunk_off, lay.n_chunks,
                                                                     lay.sel_idx, lay.sel_count, lay.scale, out16, None, ws16),
                             30, torch) * 1e-3
            tq = time_calls(lambda: B.sparse_chunk_attention_decode(lay.shape, case.q, lay.K, lay.V, lay.chunk_off,
                                                                    lay.n_chunks, lay.sel_idx, lay.sel_count, lay.scale,
                                                                    lay.out, lay.lse, lay.att_workspace, None, lay.qmeta),
                            30, torch) * 1e-3
            t_eval = time_calls(lambda: (B.chunk_score(lay.shape, case.q, lay.abstract, lay.n_chunks, lay.score, None),
                                         B.chunk_topk_select(lay.shape, lay.score, lay.chunk_off, lay.n_chunks, lay.max_chunks,
                                                             lay.token_budget, lay.sel_idx, lay.sel_count, lay.sel_tokens)),
                                30, torch) * 1e-3
            d16 = p["kept_tokens"] * 2 * 128 * 2
            extra = tq - t16 * p["kv"] / d16
            rate = d16 / extra if extra > 0 else None
            theta = B.leoam_compression_share(d16, 0.25, bw, t_eval, t16, rate or 1e15)
            policy["layers"][str(lid)] = {"D_bytes_16bit": d16, "stored_bytes": p["kv"], "T0_eval_us": round(t_eval * 1e6, 2),
                                          "Tc_attention_16bit_us": round(t16 * 1e6, 2),
                                          "attention_compressed_us": round(tq * 1e6, 2),
                                          "decompress_rate_GBps": None if rate is None else round(rate / 1e9, 1),
                                          "theta": round(theta, 4)}
            del ws16, out16
        # the policy applied to the first layer: tags from the selection with a budget of (1 - theta) of the context
        # (chunk_compression_tags), then the live store brought to them by kv_chunk_recompress
        lay, case, fb0 = layers[0], cases[0], tags[0]
        theta = policy["layers"][str(layer_ids[0])]["theta"]
        shape16 = B.make_shape(case.batch, case.hq, case.hkv, 128, case.n_ctx, lay.shape.c_max, 1, case.K.dtype)
        cap = 2 * B.leoam_compressed_bytes_bound(shape16)
        kb2 = torch.empty(cap, dtype=torch.uint8, device="cuda")
        vb2 = torch.empty(cap, dtype=torch.uint8, device="cuda")
        qm2 = torch.empty_like(lay.qmeta)
        used = torch.zeros(1, dtype=torch.int64, device="cuda")
        info = torch.zeros(3, dtype=torch.int64, device="cuda")
        fb_old = torch.from_numpy(np.ascontiguousarray(fb0).astype(np.uint8)).cuda()
        B.kv_chunk_compress(shape16, case.K, case.V, case.chunk_off, case.n_chunks, fb_old, kb2, vb2, qm2, used)
        sel_shape = B.make_shape(case.batch, case.hq, case.hkv, 128, case.n_ctx, lay.shape.c_max, lay.shape.c_max, L.binding.Q8Q4)
        sel2 = torch.empty(case.batch, case.hkv, lay.shape.c_max, dtype=torch.int32, device="cuda")
        cnt2 = torch.empty(case.batch, case.hkv, dtype=torch.int32, device="cuda")
        B.chunk_topk_select(sel_shape, lay.score, lay.chunk_off, lay.n_chunks, 0, max(1, int((1.0 - theta) * case.n_ctx)), sel2,
                            cnt2, None)
        fb_new = torch.empty_like(fb_old)
        B.chunk_compression_tags(sel_shape, lay.n_chunks, sel2, cnt2, fb_new)
        torch.cuda.synchronize()
        t_a, t_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_a.record()
        B.kv_chunk_recompress(shape16, case.K, case.V, case.chunk_off, case.n_chunks, fb_old, fb_new, kb2, vb2, qm2, used, info)
        t_b.record()
        torch.cuda.synchronize()
        nvalid = int(case.n_chunks.sum())
        policy["retag_first_layer"] = {"theta": theta, "four_bit_share_of_chunks_before": round(float(fb_old.sum()) / nvalid, 4),
                                       "four_bit_share_of_chunks_after": round(float(fb_new.sum()) / nvalid, 4),
                                       "chunks_encoded_again": int(info[1]), "of_chunks": nvalid * case.hkv,
                                       "refused": int(info[0]), "fresh_room_bytes": int(info[2]),
                                       "kv_chunk_recompress_us": round(t_a.elapsed_time(t_b) * 1e3, 1)}
        del kb2, vb2, qm2, sel2
    e_med, e_p10, e_p90 = percentiles(eager_ms)
    g_med, g_p10, g_p90 = percentiles(graph_ms)

    out = {
        "metric": "decode-step sparse-attn algorithmic KV GB/s (score+select+attention) at 128K ctx"
        if cfg["n_ctx"] == 131072 else "decode-step sparse-attn algorithmic KV GB/s (score+select+attention)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "us_per_layer_step": round(us_per_layer, 2),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 1),
        "pct_of_measured_read": round(100.0 * value / read_gbs, 1),
        "step_timing": {
            "what": "us per layer-step; `ms_per_step` is the wall-clock mean of the timed steps, these are per-step HIP-event times",
            "eager": {"median": round(e_med * 1e3 / nl, 2), "p10": round(e_p10 * 1e3 / nl, 2), "p90": round(e_p90 * 1e3 / nl, 2)},
            "graph_replay": {"median": round(g_med * 1e3 / nl, 2), "p10": round(g_p10 * 1e3 / nl, 2),
                             "p90": round(g_p90 * 1e3 / nl, 2)},
            "GBps_at_eager_median": round(step_bytes / (e_med * 1e-3) / 1e9, 1),
        },
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8/u4 codes, f32 accumulate" if quant else cfg["dtype"],
        "data": "synthetic",
        "config": {
            "workload": f"{args.workload}: batch {cfg['batch']}, {cfg['hq']} q / {cfg['hkv']} kv heads, head_dim 128, "
                        f"ctx {cfg['n_ctx']}, {'8-bit/4-bit compressed' if quant else cfg['dtype']} K/V, token budget {cfg['token_budget']}",
            "resident_layers": layer_ids,
            "layer_steps_per_step": nl,
            "bytes_per_layer_step": int(step_bytes / nl),
            "kept_tokens_per_layer_step": int(sum(p["kept_tokens"] for p in parts) / nl),
            "chunks_per_layer_step": int(sum(p["chunks"] for p in parts) / nl),
        },
        "kernels_us_per_layer_step": {"chunk_score": round(score_us, 2), "chunk_topk_select": round(select_us, 2),
                                      "sparse_chunk_attention_decode": round(attn_us, 2),
                                      "chunk_select_attention_decode": round(fused_us, 2)},
        "roofline": {
            "kernel": "select_attention_q_kernel (layers over 8192 chunks: sixteen chunks per lane)"
            if quant else "select_attention_kernel",
            "bound": "hbm",
            "achieved": round(attn_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(attn_gbs / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic(args.workload, "select_attention"),
            "traffic_source": None if measured_traffic(args.workload, "select_attention") is None else
            f"profiles/pmc_{args.workload}_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
            "benchmark, scaled by the copy probe; counters cannot be read from inside the timed process)",
            "bytes_per_launch": int(kv_bytes),
            "us_per_launch": round(fused_us, 2),
            "frac_of_measured_read": round(attn_gbs / read_gbs, 4),
            "frac_of_measured_read_same_size": round(attn_gbs / read_small_gbs, 4),
        },
        "roofline_chunk_score": {"bound": "hbm", "achieved": round(score_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": round(score_gbs / HBM_PEAK_GBS, 4), "bytes_per_launch": int(abs_bytes),
                                 "us_per_launch": round(score_us, 2)},
        "abstract_build": {"GBps_of_K_streamed": round((k_bytes + ab_out_bytes) / (ab_ms * 1e-3) / 1e9, 1),
                           "ms_per_layer": round(ab_ms / nl, 3)},
        "layer_ahead": layer_ahead,
        "abstract_append_us": None if append_us is None else round(append_us, 2),
        "tree_refine": tree,
        "compress": compress,
        "compression_policy": policy,
        "read_probe_GBps": round(read_gbs, 1),
        "read_probe_GBps_at_launch_size": round(read_small_gbs, 1),
        "copy_probe_GBps": round(copy_gbs, 1),
    }

    # ---- the oracle on the host cores, bounded sample --------------------------------
    if not args.no_cpu_baseline:
        import oracle
        lay, case = layers[0], cases[0]
        nseq = case.batch
        qc = case.q[:nseq].cpu()
        off, nc = case.chunk_off[:nseq].cpu(), case.n_chunks[:nseq].cpu()
        if quant:
            kb, vb, qm = lay.K.cpu(), lay.V.cpu(), lay.qmeta.cpu()
            ab = np.nan_to_num(oracle.abstract_build_q(kb, qm, off, nc))   # prefill-time, not timed
        else:
            Kc, Vc = case.K[:nseq].cpu(), case.V[:nseq].cpu()
            ab = np.nan_to_num(oracle.abstract_build(Kc, off, nc))      # prefill-time, not timed
        def oracle_step(n):
            ub = oracle.chunk_score(qc[:n], ab[:n], nc[:n])
            sel, cnt, tok = oracle.topk_select(ub, off[:n], nc[:n], case.max_chunks, case.token_budget, case.k_max)
            if quant:
                oracle.sparse_attention_q(qc[:n], kb, vb, qm, off[:n], sel, cnt)
            else:
                oracle.sparse_attention(qc[:n], Kc[:n], Vc[:n], off[:n], sel, cnt)

        def timed(n, budget_s):
            """median seconds per repetition over >= 5 repetitions and about budget_s of CPU time"""
            ts = []
            while len(ts) < 5 or (sum(ts) < budget_s and len(ts) < 5000):
                t = time.perf_counter()
                oracle_step(n)
                ts.append(time.perf_counter() - t)
            return float(np.median(ts)), len(ts), sum(ts)

        all_threads = oracle.num_threads()
        per_seq_bytes = parts[0]["total"] / case.batch
        med_all, reps_all, cpu_all = timed(nseq, 8.0)
        n1 = 1 if quant else min(2, nseq)              # the one-thread sample: fewer sequences, same work each
        oracle.set_threads(1)
        med_one, reps_one, cpu_one = timed(n1, 6.0)
        oracle.set_threads(all_threads)
        out["cpu_baseline"] = {
            "value": round(per_seq_bytes * nseq / med_all / 1e9, 3),
            "unit": "GB/s",
            "cores": all_threads,
            "kind": "oracle",
            "sample": f"{nseq} of {case.batch} sequences of layer {case.layer}, score+select+attention, median of "
                      f"{reps_all} repetitions, {cpu_all:.1f} s",
            "ms_per_layer_step_per_sequence": round(med_all / nseq * 1e3, 3),
            "one_thread": {"value": round(per_seq_bytes * n1 / med_one / 1e9, 3), "unit": "GB/s", "cores": 1,
                           "sample": f"{n1} of {case.batch} sequences of layer {case.layer}, median of {reps_one} "
                                     f"repetitions, {cpu_one:.1f} s",
                           "ms_per_layer_step_per_sequence": round(med_one / n1 * 1e3, 3)},
            "nproc": os.cpu_count(),
            "cpu_model": cpu_model(),
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
