#!/usr/bin/env python3
"""Benchmark of the HIPPO hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_16k] [--layers L]

One *step* is one pass of the whole hot path over one synthetic request of the named workload:

  prune         hippo_score_tokens -> hippo_select_gather_kv   (layer 0's cache -> pruned draft cache)
  decode round  for each of L distinct layer caches:
                    hippo_verify_attention (gamma+1 rows, full cache)    on stream A
                 || hippo_draft_attention  (1 row, pruned cache)         on stream B

L distinct per-layer caches (default 28, the depth of a 7B-class model) make the KV stream of a
step ~1 GB at the 16K workload -- far beyond the last-level cache, and what a real decode step
reads.  Kernels of a few microseconds are launch-bound from Python, so the prune and the decode
round are each captured once into a HIP graph and replayed; all inputs, outputs and workspaces
are resident in HBM before the timed region starts and nothing is allocated inside it.

`value` is the verify-attention effective KV bandwidth of the decode round,
  L * B * H_kv * (ctx_len + q_len) * d * 2 (K,V) * sizeof(dtype) / (duration of the round),
the round timed with HIP events on the launching stream inside the timed region while the draft
attention runs beside it on the second stream.  Also reported: prune throughput (visual tokens
per second through score + select + gather), per-call times, the roofline block of the verify
kernels and the CPU oracle timed on the host cores (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3_16k", choices=["tiny", "draft", "c3_16k", "c4_long", "c5_large"])
    ap.add_argument("--layers", type=int, default=0, help="distinct layer caches per step (0 = auto)")
    ap.add_argument("--num-splits", type=int, default=0, help="verify KV splits (0 = library heuristic)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=0, help="layers the oracle is timed on (0 = auto)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2601_08273_amd as h
    import synth_inputs as si
    from parity_util import dev

    h.load()                                   # fails loudly if libhippo.so is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = si.CONFIGS[args.workload]
    dt = cfg.dtype
    esize = 2 if dt == "bf16" else 4
    n_ctx = cfg.ctx_len
    n_tot = n_ctx + cfg.q_len
    kv_bytes = cfg.batch * cfg.n_kv_heads * n_tot * cfg.head_dim * 2 * esize      # one layer, K and V
    L = args.layers or max(2, min(28, int(2.5e9 // kv_bytes)))

    # ---- synthetic inputs: L distinct layer caches drawn by the recipe, then moved to HBM ----
    t0 = time.time()
    with ThreadPoolExecutor(max_workers=min(8, L)) as ex:
        layers = list(ex.map(lambda s: si.make_inputs(cfg, s), range(L)))
    kd = [dev(x["k"], dt) for x in layers]
    vd = [dev(x["v"], dt) for x in layers]
    qd = [dev(x["q_new"], dt) for x in layers]
    q_txt = dev(layers[0]["q_txt"], dt)
    gen_s = time.time() - t0

    vid = h.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)
    k_keep = cfg.k_keep
    n_dctx = n_ctx - cfg.n_visual + k_keep          # context length of the pruned draft cache
    B, Hkv, d = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    tdt = kd[0].dtype

    # ---- every output and workspace is allocated here, once ----
    kvd = h.kv_desc(kd[0], cfg.n_q_heads)
    ws_score = torch.empty(h.workspace_bytes(h.CALL_SCORE_TOKENS, kvd, vid, cfg.l_txt, n_ctx), dtype=torch.uint8,
                           device="cuda")
    ws_sel = torch.empty(256, dtype=torch.uint8, device="cuda")
    ws_ver = torch.empty(h.workspace_bytes(h.CALL_VERIFY_ATTENTION, kvd, None, cfg.q_len, n_tot, 0, args.num_splits),
                         dtype=torch.uint8, device="cuda")
    scores = torch.empty((B, cfg.n_visual), dtype=torch.float32, device="cuda")
    idx = torch.empty((B, k_keep), dtype=torch.int32, device="cuda")
    out_ver = torch.empty_like(qd[0])
    # draft caches: room for the pruned context plus the new token's own K/V row
    kp = [torch.empty((B, Hkv, n_dctx + 1, d), dtype=tdt, device="cuda") for _ in range(L)]
    vp = [torch.empty((B, Hkv, n_dctx + 1, d), dtype=tdt, device="cuda") for _ in range(L)]
    qdraft = [q[:, :1].contiguous() for q in qd]
    out_dr = torch.empty_like(qdraft[0])
    ws_dr = torch.empty(h.workspace_bytes(h.CALL_DRAFT_ATTENTION, h.kv_desc(kp[0], cfg.n_q_heads), None, 1,
                                          n_dctx + 1), dtype=torch.uint8, device="cuda")

    def prune(layer: int):
        h.hippo_score_tokens(q_txt, kd[layer][:, :, :n_ctx], vid, scores_out=scores, workspace=ws_score)
        h.hippo_select_gather_kv(scores, k_keep, kd[layer][:, :, :n_ctx], vd[layer][:, :, :n_ctx], vid,
                                 cfg.n_q_heads, idx_out=idx, k_dst=kp[layer][:, :, :n_dctx],
                                 v_dst=vp[layer][:, :, :n_dctx], workspace=ws_sel)

    for l in range(L):                              # fill every layer's draft cache before timing
        prune(l)
        kp[l][:, :, n_dctx] = kd[l][:, :, n_ctx]
        vp[l][:, :, n_dctx] = vd[l][:, :, n_ctx]
    torch.cuda.synchronize()

    sB = torch.cuda.Stream()                        # default priority

    def verify_all(stream=None):
        for l in range(L):
            h.hippo_verify_attention(qd[l], kd[l], vd[l], n_ctx, num_splits=args.num_splits, out=out_ver,
                                     workspace=ws_ver, stream=stream)

    def draft_all(stream=None):
        for l in range(L):
            h.hippo_draft_attention(qdraft[l], kp[l], vp[l], n_dctx, out=out_dr, workspace=ws_dr, stream=stream)

    def decode_round():
        cur = torch.cuda.current_stream()
        sB.wait_stream(cur)
        for l in range(L):
            h.hippo_verify_attention(qd[l], kd[l], vd[l], n_ctx, num_splits=args.num_splits, out=out_ver,
                                     workspace=ws_ver)
            h.hippo_draft_attention(qdraft[l], kp[l], vp[l], n_dctx, out=out_dr, workspace=ws_dr, stream=sB)
        cur.wait_stream(sB)

    # appended-row fusion: the q_len new rows arrive as [B, q_len, Hkv, d] and reach the cache inside
    # the attention launch, versus a separate copy (two strided copies, K and V) followed by the call
    k_new = [kd[l][:, :, n_ctx:n_tot].transpose(1, 2).contiguous() for l in range(L)]
    v_new = [vd[l][:, :, n_ctx:n_tot].transpose(1, 2).contiguous() for l in range(L)]

    def verify_append_all():
        for l in range(L):
            h.hippo_verify_attention(qd[l], kd[l], vd[l], n_ctx, num_splits=args.num_splits, out=out_ver,
                                     workspace=ws_ver, k_new=k_new[l], v_new=v_new[l])

    def copy_then_verify_all():
        for l in range(L):
            kd[l][:, :, n_ctx:n_tot].copy_(k_new[l].transpose(1, 2))
            vd[l][:, :, n_ctx:n_tot].copy_(v_new[l].transpose(1, 2))
            h.hippo_verify_attention(qd[l], kd[l], vd[l], n_ctx, num_splits=args.num_splits, out=out_ver,
                                     workspace=ws_ver)

    # paged cache: the same rows in 16-token pages scattered over a pool (one pool per layer)
    PS = 16
    n_pg = (n_tot + PS - 1) // PS
    gen = torch.Generator(device="cpu").manual_seed(0)
    tables = torch.stack([torch.randperm(B * n_pg, generator=gen)[:B * n_pg].reshape(B, n_pg) for _ in range(1)])[0]
    table_d = tables.to(torch.int32).cuda()

    def to_pool(x):                                   # [B, Hkv, N, d] -> [B * n_pg, PS, Hkv, d]
        pad = torch.zeros((B, Hkv, n_pg * PS, d), dtype=x.dtype, device=x.device)
        pad[:, :, :x.shape[2]] = x
        pages = pad.permute(0, 2, 1, 3).reshape(B * n_pg, PS, Hkv, d).contiguous()
        pool = torch.empty_like(pages)
        pool[table_d.reshape(-1).long()] = pages
        return pool
    k_pool = [to_pool(kd[l]) for l in range(L)]
    v_pool = [to_pool(vd[l]) for l in range(L)]

    def verify_paged_all():
        for l in range(L):
            h.hippo_verify_attention_paged(qd[l], k_pool[l], v_pool[l], table_d, n_ctx, num_splits=args.num_splits,
                                           out=out_ver, workspace=ws_ver)

    # fp8 cache: the same rows as E4M3 codes with one multiplier per (batch element, KV head)
    have_fp8 = dt == "bf16"
    if have_fp8:                                     # written by the library's own quantiser
        q8 = [h.hippo_quantize_kv_e4m3(kd[l], vd[l]) for l in range(L)]
        k8, v8 = [(c[0], c[2]) for c in q8], [(c[1], c[3]) for c in q8]
        ws_q8 = torch.empty(int(h.load().hippo_quantize_kv_workspace_bytes(C.byref(kvd), n_tot)), dtype=torch.uint8,
                            device="cuda")

    def quantize_layer0():
        h.hippo_quantize_kv_e4m3(kd[0], vd[0], k_codes=k8[0][0], v_codes=v8[0][0], workspace=ws_q8)

    def verify_fp8_all():
        for l in range(L):
            h.hippo_verify_attention_fp8kv(qd[l], k8[l][0], v8[l][0], k8[l][1], v8[l][1], n_ctx,
                                           num_splits=args.num_splits, out=out_ver, workspace=ws_ver)

    # Eq. 2 summed over several layers: one call that sweeps them in shared launches, versus one
    # accumulate call per layer
    NLS = min(4, L)
    ws_layers = torch.empty(h.load().hippo_score_layers_workspace_bytes(C.byref(kvd), C.byref(vid), cfg.l_txt, NLS),
                            dtype=torch.uint8, device="cuda")
    mass = torch.zeros((B, cfg.n_visual), dtype=torch.float32, device="cuda")
    k_ctx = [kd[l][:, :, :n_ctx] for l in range(NLS)]

    def score_layers_one_call():
        h.hippo_score_tokens_layers([q_txt] * NLS, k_ctx, vid, emb_layer=NLS - 1, scores_out=scores, workspace=ws_layers)

    def score_layers_accumulate():
        mass.zero_()
        for l in range(NLS - 1):
            h.hippo_score_tokens(q_txt, k_ctx[l], vid, flags=h.SCORE_ACCUMULATE_ONLY, attn_mass_inout=mass,
                                 workspace=ws_score)
        h.hippo_score_tokens(q_txt, k_ctx[NLS - 1], vid, attn_mass_inout=mass, scores_out=scores, workspace=ws_score)

    def score_only():
        h.hippo_score_tokens(q_txt, kd[0][:, :, :n_ctx], vid, scores_out=scores, workspace=ws_score)

    # speculative-sampling verification of the round's gamma draft tokens over LM-head-sized logits
    # (outside the timed step: it widens the path beyond the attention calls the metric is quoted on)
    V = si.LM_VOCAB
    pl_h, ql_h, rng = si.make_logits(B, cfg.gamma, V, 0)
    p_log, q_log = dev(pl_h, dt), dev(ql_h, dt)
    sd_tok = torch.from_numpy(rng.integers(0, V, (B, cfg.gamma)).astype(np.int32)).cuda()
    sd_ua = torch.from_numpy(rng.random((B, cfg.gamma), dtype=np.float32)).cuda()
    sd_us = torch.from_numpy(rng.random(B, dtype=np.float32)).cuda()
    sd_nacc = torch.empty(B, dtype=torch.int32, device="cuda")
    sd_next = torch.empty(B, dtype=torch.int32, device="cuda")
    ws_sd = torch.empty(h.load().hippo_spec_verify_workspace_bytes(B, cfg.gamma, V, h._dtype_code(p_log)),
                        dtype=torch.uint8, device="cuda")

    SD_REPS = 20        # calls per graph, so that the graph's own launch cost is amortised as for the layers

    def spec_sampling():
        for _ in range(SD_REPS):
            h.hippo_spec_verify(p_log, q_log, sd_tok, sd_ua, sd_us, 1.0, n_accept_out=sd_nacc,
                                next_token_out=sd_next, workspace=ws_sd)

    def spec_greedy():
        for _ in range(SD_REPS):
            h.hippo_spec_verify(p_log, None, sd_tok, None, None, 0.0, n_accept_out=sd_nacc,
                                next_token_out=sd_next, workspace=ws_sd)

    def capture(fn):
        fn()                                        # eager once (also sets kernel attributes)
        torch.cuda.synchronize()
        if args.no_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g.replay

    run_prune = capture(lambda: prune(0))
    run_round = capture(decode_round)
    run_verify = capture(verify_all)
    run_draft = capture(draft_all)
    run_score = capture(score_only)
    run_verify_append = capture(verify_append_all)
    run_copy_verify = capture(copy_then_verify_all)
    run_verify_paged = capture(verify_paged_all)
    run_verify_fp8 = capture(verify_fp8_all) if have_fp8 else None
    run_quantize = capture(quantize_layer0) if have_fp8 else None
    run_layers_one = capture(score_layers_one_call)
    run_layers_acc = capture(score_layers_accumulate)
    run_sd_sampling = capture(spec_sampling)
    run_sd_greedy = capture(spec_greedy)
    torch.cuda.synchronize()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(rec=None):
        e = [ev(), ev(), ev()] if rec is not None else None
        if e: e[0].record()
        run_prune()
        if e: e[1].record()
        run_round()
        if e:
            e[2].record()
            rec.append(e)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    rec = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall / args.steps * 1e3
    t_prune = float(np.mean([e[0].elapsed_time(e[1]) for e in rec])) * 1e-3
    t_round = float(np.mean([e[1].elapsed_time(e[2]) for e in rec])) * 1e-3
    verify_gbs = L * kv_bytes / t_round / 1e9
    prune_tok_s = B * cfg.n_visual / t_prune

    # ---- breakdown, outside the timed region: each piece alone, best of a few replays ----
    def alone(fn, reps=7):
        best = 1e30
        for _ in range(reps):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b))
        return best * 1e-3

    t_verify_alone = alone(run_verify) / L
    t_draft_alone = alone(run_draft) / L
    t_score_alone = alone(run_score)
    t_prune_alone = alone(run_prune)
    t_verify_append = alone(run_verify_append) / L
    t_copy_verify = alone(run_copy_verify) / L
    t_verify_paged = alone(run_verify_paged) / L
    t_verify_fp8 = alone(run_verify_fp8) / L if have_fp8 else None
    t_quantize = alone(run_quantize) if have_fp8 else None
    t_layers_one = alone(run_layers_one)
    t_layers_acc = alone(run_layers_acc)
    t_sd_sampling = alone(run_sd_sampling) / SD_REPS
    t_sd_greedy = alone(run_sd_greedy) / SD_REPS

    if args.pmc_calibration:       # a plain copy of known size: reads 256 MiB, writes 256 MiB
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    traffic = None    # HBM bytes per verify call from a counter run, if one has been summarised
    tf = os.path.join(ROOT, "profiles", "verify_attention_%s_hbm_traffic.txt" % args.workload)
    if os.path.exists(tf):
        for line in open(tf):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])

    result = {
        "metric": "verify-attention effective KV GB/s (% HBM peak); prune tokens/s at 16K ctx",
        "value": round(verify_gbs, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if dt == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %d q heads / %d kv heads, d %d, %s, %d frames x %dx%d + %d text = %d ctx, "
                               "gamma %d, keep %d%%, batch %d; %d distinct layer caches per step; draft attention "
                               "concurrent on a second stream" % (
                                   cfg.name, cfg.n_q_heads, cfg.n_kv_heads, d, dt, cfg.n_frames, cfg.grid_h,
                                   cfg.grid_w, cfg.n_prefix + cfg.n_suffix, n_ctx, cfg.gamma, cfg.keep_pct, B, L),
                   "layers_per_step": L, "num_splits": args.num_splits, "hip_graph": not args.no_graph},
        "pct_hbm_peak": round(100.0 * verify_gbs / HBM_PEAK_GBS, 2),
        "prune_tokens_per_s": round(prune_tok_s, 1),
        "us": {"prune(score+select+gather)": round(t_prune * 1e6, 2),
               "decode_round_per_layer(verify||draft)": round(t_round / L * 1e6, 3),
               "alone:verify_per_layer": round(t_verify_alone * 1e6, 3),
               "alone:draft_per_layer": round(t_draft_alone * 1e6, 3),
               "alone:score_tokens": round(t_score_alone * 1e6, 2),
               "alone:prune": round(t_prune_alone * 1e6, 2),
               "alone:verify_with_fused_append_per_layer": round(t_verify_append * 1e6, 3),
               "alone:copy_new_rows_then_verify_per_layer": round(t_copy_verify * 1e6, 3),
               "alone:verify_paged(16-token pages)_per_layer": round(t_verify_paged * 1e6, 3),
               "alone:verify_fp8_cache_per_layer": round(t_verify_fp8 * 1e6, 3) if have_fp8 else None,
               "alone:quantize_one_layer_cache_to_fp8": round(t_quantize * 1e6, 2) if have_fp8 else None,
               "alone:score_%d_layers(one call)" % NLS: round(t_layers_one * 1e6, 2),
               "alone:score_%d_layers(accumulate calls)" % NLS: round(t_layers_acc * 1e6, 2),
               "alone:spec_verify(sampling, V=%d)" % V: round(t_sd_sampling * 1e6, 2),
               "alone:spec_verify(greedy, V=%d)" % V: round(t_sd_greedy * 1e6, 2)},
        "verify_alone_GBps": round(kv_bytes / t_verify_alone / 1e9, 1),
        "roofline": {"bound": "hbm", "achieved": round(verify_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(verify_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "kernel": "hippo_verify_attention = attn_partial_grid + attn_combine; %d algorithmic bytes "
                               "(K+V of one layer) per call, duration = decode round / layers" % kv_bytes},
        "input_generation_s": round(gen_s, 1),
    }

    # ---- CPU oracle on a bounded sample of the same workload ----
    if not args.no_cpu_baseline:
        import oracle
        n_cpu, t0 = 0, time.perf_counter()
        while True:                                  # whole layers until ~10 s of oracle time
            l = n_cpu % L
            oracle.attention(layers[l]["q_new"], layers[l]["k"], layers[l]["v"], n_ctx)
            n_cpu += 1
            t_cpu = time.perf_counter() - t0
            if t_cpu > 10.0 or (args.cpu_layers and n_cpu >= args.cpu_layers):
                break
        result["cpu_baseline"] = {
            "value": round(kv_bytes * n_cpu / t_cpu / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": "%d verify-attention calls cycling over the %d layer caches of this workload (all heads, "
                      "all %d query rows), float64 C oracle, %.1f s" % (n_cpu, L, cfg.q_len, t_cpu)}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
