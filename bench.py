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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=sorted(RESIDENT))
    ap.add_argument("--layers", type=int, default=0, help="use only the first n resident layers (0 = all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=5, help="passes of the per-kernel timing loops")
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


def compress_store(B, torch, case, four_bit, timed):
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
            case.K = case.V = None          # only the compressed store stays resident
            tags.append(fb)
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
        compress = compress_store(B, torch, case, fb, timed=True)[3]

    # ---- plain copy of known size: the "what does this box stream" reference ------
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    copy_ms = time_calls(lambda: B.leoam_copy_probe(dst, src, nbytes), 10, torch)
    copy_gbs = 2 * nbytes / (copy_ms * 1e-3) / 1e9
    del src, dst

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
            "bytes_per_launch": int(kv_bytes),
            "us_per_launch": round(fused_us, 2),
        },
        "roofline_chunk_score": {"bound": "hbm", "achieved": round(score_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": round(score_gbs / HBM_PEAK_GBS, 4), "bytes_per_launch": int(abs_bytes),
                                 "us_per_launch": round(score_us, 2)},
        "abstract_build": {"GBps_of_K_streamed": round((k_bytes + ab_out_bytes) / (ab_ms * 1e-3) / 1e9, 1),
                           "ms_per_layer": round(ab_ms / nl, 3)},
        "abstract_append_us": None if append_us is None else round(append_us, 2),
        "tree_refine": tree,
        "compress": compress,
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
        reps, cpu_s = 0, 0.0
        while reps < 3 or (cpu_s < 10.0 and reps < 5000):
            t = time.perf_counter()
            ub = oracle.chunk_score(qc, ab, nc)
            sel, cnt, tok = oracle.topk_select(ub, off, nc, case.max_chunks, case.token_budget, case.k_max)
            if quant:
                oracle.sparse_attention_q(qc, kb, vb, qm, off, sel, cnt)
            else:
                oracle.sparse_attention(qc, Kc, Vc, off, sel, cnt)
            cpu_s += time.perf_counter() - t
            reps += 1
        sample_bytes = parts[0]["total"] * nseq // case.batch
        out["cpu_baseline"] = {
            "value": round(sample_bytes / (cpu_s / reps) / 1e9, 3),
            "unit": "GB/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{nseq} of {case.batch} sequences of layer {case.layer}, score+select+attention, "
                      f"{reps} repetitions, {cpu_s:.1f} s of CPU time",
            "ms_per_layer_step_per_sequence": round(cpu_s / reps / nseq * 1e3, 3),
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
