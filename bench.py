#!/usr/bin/env python3
"""Benchmark of the HIPPO hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_16k] [--layers L] [--keep-pct P]

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
attention runs beside it on the second stream; the figure is the MEDIAN over the steps' event pairs.

Outside the timed region the same run also reports, in the `us` object (microseconds, medians):
  alone:*      each entry point and each cache-format variant on its own
  calib:*      what this machine gives ANY kernel of the verify call's shape: a chain of launches
               that do nothing, and plain device copies / reductions of one layer's K+V bytes,
               replayed from the same kind of graph over L distinct buffers (tensor-library kernels only)
  c4_long:*    the long-video configuration: verify alone and beside the draft, and the prune and
               draft calls at keep ratios 5 / 10 / 25 %
  c5_large:*   the batch-4 large-share configuration: verify alone and beside the draft
and the CPU oracle timed on the host cores, one leg per entry point (a reported baseline only).
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
    ap.add_argument("--keep-pct", type=int, default=0, help="percent of visual tokens kept (0 = the workload's own)")
    ap.add_argument("--num-splits", type=int, default=0, help="verify KV splits (0 = library heuristic)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip everything outside the timed step (alone:*, calib:*, c4_long:*, c5_large:*)")
    ap.add_argument("--cpu-layers", type=int, default=0, help="calls the oracle's verify leg is limited to (0 = by time)")
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
    if args.keep_pct:
        cfg = cfg.with_keep(args.keep_pct)
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

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def capture(fn):
        fn()                                        # eager once (also sets kernel attributes)
        torch.cuda.synchronize()
        if args.no_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g.replay

    def samples_us(fn, reps=9, per=1):
        """durations of `reps` runs of fn (HIP events on the launching stream), in us per `per` calls"""
        fn()
        out = []
        for _ in range(reps):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            out.append(a.elapsed_time(b) * 1e3 / per)
        return out

    def med(fn, reps=9, per=1):
        return float(np.median(samples_us(fn, reps, per)))

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

    def decode_round():
        cur = torch.cuda.current_stream()
        sB.wait_stream(cur)
        for l in range(L):
            h.hippo_verify_attention(qd[l], kd[l], vd[l], n_ctx, num_splits=args.num_splits, out=out_ver,
                                     workspace=ws_ver)
            h.hippo_draft_attention(qdraft[l], kp[l], vp[l], n_dctx, out=out_dr, workspace=ws_dr, stream=sB)
        cur.wait_stream(sB)

    run_prune = capture(lambda: prune(0))
    run_round = capture(decode_round)
    torch.cuda.synchronize()

    # ---- the timed region: K steps of prune + decode round, each bracketed by HIP events ----
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
    prune_s = np.array([e[0].elapsed_time(e[1]) for e in rec]) * 1e-3
    round_s = np.array([e[1].elapsed_time(e[2]) for e in rec]) * 1e-3
    t_prune = float(np.median(prune_s))
    t_round = float(np.median(round_s))
    verify_gbs = L * kv_bytes / t_round / 1e9
    prune_tok_s = B * cfg.n_visual / t_prune

    us = {"prune(score+select+gather)": round(t_prune * 1e6, 2),
          "decode_round_per_layer(verify||draft)": round(t_round / L * 1e6, 3),
          "decode_round_per_layer[min,max over the steps]": [round(float(round_s.min()) / L * 1e6, 3),
                                                             round(float(round_s.max()) / L * 1e6, 3)]}

    # ================================================================================================
    # outside the timed region: each piece alone, the cache-format variants, calibration, other configs
    # ================================================================================================
    verify_alone_gbs = None
    if not args.no_extras:
        def verify_all():
            for l in range(L):
                h.hippo_verify_attention(qd[l], kd[l], vd[l], n_ctx, num_splits=args.num_splits, out=out_ver,
                                         workspace=ws_ver)

        def draft_all():
            for l in range(L):
                h.hippo_draft_attention(qdraft[l], kp[l], vp[l], n_dctx, out=out_dr, workspace=ws_dr)

        def score_only():
            h.hippo_score_tokens(q_txt, kd[0][:, :, :n_ctx], vid, scores_out=scores, workspace=ws_score)

        t_verify_alone = med(capture(verify_all), per=L)
        verify_alone_gbs = kv_bytes / t_verify_alone / 1e3
        us["alone:verify_per_layer"] = round(t_verify_alone, 3)
        us["alone:draft_per_layer"] = round(med(capture(draft_all), per=L), 3)
        us["alone:score_tokens"] = round(med(capture(score_only)), 2)
        if dt == "bf16":
            # the draft call again on the same values held as an fp32 cache: that cache type runs the
            # vector-ALU split-KV kernel, the bf16 cache the MFMA kernel padded to one 16-row block
            kp32, vp32 = [x.float() for x in kp], [x.float() for x in vp]
            qdraft32 = [x.float() for x in qdraft]
            out_dr32 = torch.empty_like(qdraft32[0])
            ws_dr32 = torch.empty(h.workspace_bytes(h.CALL_DRAFT_ATTENTION, h.kv_desc(kp32[0], cfg.n_q_heads), None, 1,
                                                    n_dctx + 1), dtype=torch.uint8, device="cuda")

            def draft_fp32_all():
                for l in range(L):
                    h.hippo_draft_attention(qdraft32[l], kp32[l], vp32[l], n_dctx, out=out_dr32, workspace=ws_dr32)

            us["alone:draft_per_layer(fp32 cache: vector-ALU kernel)"] = round(med(capture(draft_fp32_all), per=L), 3)
            del kp32, vp32
        us["alone:prune"] = round(med(run_prune), 2)

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

        us["alone:verify_with_fused_append_per_layer"] = round(med(capture(verify_append_all), per=L), 3)
        us["alone:copy_new_rows_then_verify_per_layer"] = round(med(capture(copy_then_verify_all), per=L), 3)

        # paged cache: the same rows in 16-token pages scattered over a pool (one pool per layer)
        PS = 16
        n_pg = (n_tot + PS - 1) // PS
        gen = torch.Generator(device="cpu").manual_seed(0)
        table_d = torch.randperm(B * n_pg, generator=gen).reshape(B, n_pg).to(torch.int32).cuda()

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
                h.hippo_verify_attention_paged(qd[l], k_pool[l], v_pool[l], table_d, n_ctx,
                                               num_splits=args.num_splits, out=out_ver, workspace=ws_ver)

        us["alone:verify_paged(16-token pages)_per_layer"] = round(med(capture(verify_paged_all), per=L), 3)
        del k_pool, v_pool

        # fp8 cache: the same rows as E4M3 codes with one multiplier per (batch element, KV head)
        if dt == "bf16":                                 # written by the library's own quantiser
            q8 = [h.hippo_quantize_kv_e4m3(kd[l], vd[l]) for l in range(L)]
            ws_q8 = torch.empty(int(h.load().hippo_quantize_kv_workspace_bytes(C.byref(kvd), n_tot)),
                                dtype=torch.uint8, device="cuda")

            def quantize_layer0():
                h.hippo_quantize_kv_e4m3(kd[0], vd[0], k_codes=q8[0][0], v_codes=q8[0][1], workspace=ws_q8)

            def verify_fp8_all():
                for l in range(L):
                    h.hippo_verify_attention_fp8kv(qd[l], q8[l][0], q8[l][1], q8[l][2], q8[l][3], n_ctx,
                                                   num_splits=args.num_splits, out=out_ver, workspace=ws_ver)

            us["alone:verify_fp8_cache_per_layer"] = round(med(capture(verify_fp8_all), per=L), 3)
            us["alone:quantize_one_layer_cache_to_fp8"] = round(med(capture(quantize_layer0)), 2)
            del q8

        # Eq. 2 summed over several layers: one call that sweeps them in shared launches, versus one
        # accumulate call per layer
        NLS = min(4, L)
        ws_layers = torch.empty(h.load().hippo_score_layers_workspace_bytes(C.byref(kvd), C.byref(vid), cfg.l_txt, NLS),
                                dtype=torch.uint8, device="cuda")
        mass = torch.zeros((B, cfg.n_visual), dtype=torch.float32, device="cuda")
        k_ctx = [kd[l][:, :, :n_ctx] for l in range(NLS)]

        def score_layers_one_call():
            h.hippo_score_tokens_layers([q_txt] * NLS, k_ctx, vid, emb_layer=NLS - 1, scores_out=scores,
                                        workspace=ws_layers)

        def score_layers_accumulate():
            mass.zero_()
            for l in range(NLS - 1):
                h.hippo_score_tokens(q_txt, k_ctx[l], vid, flags=h.SCORE_ACCUMULATE_ONLY, attn_mass_inout=mass,
                                     workspace=ws_score)
            h.hippo_score_tokens(q_txt, k_ctx[NLS - 1], vid, attn_mass_inout=mass, scores_out=scores,
                                 workspace=ws_score)

        us["alone:score_%d_layers(one call)" % NLS] = round(med(capture(score_layers_one_call)), 2)
        us["alone:score_%d_layers(accumulate calls)" % NLS] = round(med(capture(score_layers_accumulate)), 2)

        # speculative-sampling verification of the round's gamma draft tokens over LM-head-sized logits
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

        us["alone:spec_verify(sampling, V=%d)" % V] = round(med(capture(spec_sampling), per=SD_REPS), 2)
        us["alone:spec_verify(greedy, V=%d)" % V] = round(med(capture(spec_greedy), per=SD_REPS), 2)

        us.update(calibration(torch, np, capture, med, kv_bytes, L))
        if args.workload == "c3_16k":                      # the same copies at the other configurations' sizes
            for name in ("c4_long", "c5_large"):
                c = si.CONFIGS[name]
                nbytes = c.batch * c.n_kv_heads * (c.ctx_len + c.q_len) * c.head_dim * 2 * 2
                us.update(calibration(torch, np, capture, med, nbytes, max(2, min(28, int(2.5e9 // nbytes))),
                                      copies_only=True))

        # ---- the other bandwidth-bound configurations, so that a default run records them too ----
        if args.workload == "c3_16k":
            us.update(other_workloads(h, si, torch, np, kd, vd, qd, layers, capture, samples_us))

    if args.pmc_calibration:       # a plain copy of known size: reads 256 MiB, writes 256 MiB
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # HBM bytes per verify call, from the rocprofv3 counter runs summarised under profiles/ (a run of this
    # script cannot read the counters itself); null when no summary exists for the workload
    traffic, traffic_src = None, None
    tf = os.path.join(ROOT, "profiles", "verify_attention_%s_hbm_traffic.txt" % args.workload)
    if os.path.exists(tf):
        for line in open(tf):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic, traffic_src = float(line.split(":")[1]), os.path.relpath(tf, ROOT)

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
                   "layers_per_step": L, "num_splits": args.num_splits, "hip_graph": not args.no_graph,
                   "statistic": "median over the steps' HIP-event pairs"},
        "pct_hbm_peak": round(100.0 * verify_gbs / HBM_PEAK_GBS, 2),
        "prune_tokens_per_s": round(prune_tok_s, 1),
        "us": us,
        "verify_alone_GBps": round(verify_alone_gbs, 1) if verify_alone_gbs else None,
        "roofline": {"bound": "hbm", "achieved": round(verify_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(verify_gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "hippo_verify_attention (split-KV partial kernel + split merge); %d algorithmic bytes "
                               "(K+V of one layer) per call, duration = decode round / layers" % kv_bytes},
        "input_generation_s": round(gen_s, 1),
    }

    # ---- CPU oracle on bounded samples of the same workload, one leg per entry point ----
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, cfg, layers, kv_bytes, L)
    print(json.dumps(result), flush=True)


def calibration(torch, np, capture, med, kv_bytes, L, copies_only=False):
    """What this machine gives any kernel of the verify call's shape, measured with tensor-library
    kernels only: L dependent launches over L distinct buffers of one layer's K+V bytes each, replayed
    from the same kind of graph as the verify calls."""
    out = {}
    n_el = kv_bytes // 2                                  # 16-bit elements in one layer's K+V
    half = [torch.randn(n_el // 2, device="cuda").to(torch.bfloat16) for _ in range(L)]
    dst = torch.empty(n_el // 2, dtype=torch.bfloat16, device="cuda")
    mb = kv_bytes / 1e6

    def copy_chain():                                     # reads kv_bytes / 2 and writes kv_bytes / 2 per launch
        for l in range(L):
            dst.copy_(half[l])

    out["calib:copy(%.1f MB in, %.1f MB out)" % (mb / 2, mb / 2)] = round(med(capture(copy_chain), per=L), 3)
    del half, dst
    if copies_only:
        torch.cuda.empty_cache()
        return out
    full = [torch.randn(n_el, device="cuda").to(torch.bfloat16) for _ in range(L)]
    tiny = torch.zeros(64, device="cuda")
    acc = list(torch.zeros(L, device="cuda").unbind(0))
    top = list(torch.zeros(L, dtype=torch.bfloat16, device="cuda").unbind(0))

    def empty_chain():
        for _ in range(2 * L):                            # as many launches as L verify calls make
            tiny.add_(1.0)

    def sum_chain():                                      # reads kv_bytes per call
        for l in range(L):
            torch.sum(full[l], dim=0, dtype=torch.float32, out=acc[l])

    def amax_chain():                                     # reads kv_bytes per call
        for l in range(L):
            torch.amax(full[l], dim=0, out=top[l])

    out["calib:launch_that_does_nothing(chain of %d)" % (2 * L)] = round(med(capture(empty_chain), per=2 * L), 3)
    for name, fn in (("calib:sum(%.1f MB read)" % mb, sum_chain), ("calib:amax(%.1f MB read)" % mb, amax_chain)):
        try:
            out[name] = round(med(capture(fn), per=L), 3)
        except Exception as exc:                          # a reduction the graph cannot hold: say so, go on
            torch.cuda.synchronize()
            out[name] = "unavailable (%s)" % type(exc).__name__
    return out


def other_workloads(h, si, torch, np, kd, vd, qd, layers, capture, samples_us):
    """Verify attention (alone and beside the draft call) at the long-video and the large-share
    configurations, and the long-video prune / draft calls at keep ratios 5, 10 and 25 %.

    Their caches are assembled ON THE DEVICE from rows of the 16K layers the recipe drew (text rows from
    text rows, whole frames from frames; other layers supply the additional heads, batch elements and
    frames), so the values keep the recipe's statistics without a minute of host time to draw 2.4 GB anew.
    `--workload c4_long | c5_large` times the same configurations on caches drawn directly by the recipe."""
    from parity_util import dev
    out = {}
    c3 = si.CONFIGS["c3_16k"]
    L3 = len(kd)
    d = c3.head_dim
    pre3, vis3, suf3 = c3.n_prefix, c3.n_visual, c3.n_suffix

    def stat3(xs):
        return [round(float(np.min(xs)), 3), round(float(np.median(xs)), 3), round(float(np.max(xs)), 3)]

    def assemble(cfg, n_layers, src):
        """n_layers caches [B, Hkv, ctx + q_len, d] of configuration cfg from rows of the 16K layers"""
        res = []
        for l in range(n_layers):
            per_b = []
            for b in range(cfg.batch):
                per_h = []
                for hk in range(cfg.n_kv_heads):
                    lay = l * 7 + b * 3 + hk // c3.n_kv_heads               # a different source layer per piece
                    hh = hk % c3.n_kv_heads

                    def span(lo, width, n):       # n rows out of rows [lo, lo + width) of successive source layers
                        parts, s = [], 0
                        while n > 0:
                            parts.append(src[(lay + s) % L3][0, hh, lo:lo + min(n, width)])
                            n -= parts[-1].shape[0]
                            s += 1
                        return parts
                    per_h.append(torch.cat(span(0, pre3, cfg.n_prefix) + span(pre3, vis3, cfg.n_visual) +
                                           span(pre3 + vis3, suf3, cfg.n_suffix) +
                                           span(pre3 + vis3 + suf3, c3.q_len, cfg.q_len)))
                per_b.append(torch.stack(per_h))
            res.append(torch.stack(per_b).contiguous())
        return res

    def queries(cfg, n_layers):
        res = []
        for l in range(n_layers):
            parts, need, s = [], cfg.n_q_heads, 0
            while need > 0:
                parts.append(qd[(l + s) % L3][:, :, :min(need, c3.n_q_heads)])
                need -= parts[-1].shape[2]
                s += 1
            q = torch.cat(parts, dim=2)                                     # [1, 6, H, d]
            q = torch.cat([q] * ((cfg.q_len + c3.q_len - 1) // c3.q_len), dim=1)[:, :cfg.q_len]
            res.append(torch.cat([q.roll(b, 1) for b in range(cfg.batch)], dim=0).contiguous())
        return res

    for name in ("c4_long", "c5_large"):
        cfg = si.CONFIGS[name]
        n_ctx, n_tot = cfg.ctx_len, cfg.ctx_len + cfg.q_len
        bytes_layer = cfg.batch * cfg.n_kv_heads * n_tot * d * 2 * 2
        Lx = max(2, min(28, int(2.5e9 // bytes_layer)))
        K, V = assemble(cfg, Lx, kd), assemble(cfg, Lx, vd)
        Q = queries(cfg, Lx)
        Q1 = [q[:, :1].contiguous() for q in Q]
        kvd = h.kv_desc(K[0], cfg.n_q_heads)
        ws_v = torch.empty(h.workspace_bytes(h.CALL_VERIFY_ATTENTION, kvd, None, cfg.q_len, n_tot), dtype=torch.uint8,
                           device="cuda")
        out_v, out_d = torch.empty_like(Q[0]), torch.empty_like(Q1[0])
        sB = torch.cuda.Stream()
        vid = h.video_desc(cfg.n_frames, cfg.grid_h, cfg.grid_w, cfg.n_prefix)

        def verify_all():
            for l in range(Lx):
                h.hippo_verify_attention(Q[l], K[l], V[l], n_ctx, out=out_v, workspace=ws_v)

        xs = samples_us(capture(verify_all), reps=20, per=Lx)
        out["%s:verify_alone_per_layer[min,median,max]" % name] = stat3(xs)
        out["%s:verify_alone_frac_of_hbm_peak(median)" % name] = round(bytes_layer / np.median(xs) / 1e3 / HBM_PEAK_GBS, 4)

        for pct in ((5, 10, 25) if name == "c4_long" else (cfg.keep_pct,)):
            k_keep = (cfg.n_visual * pct + 99) // 100
            n_d = n_ctx - cfg.n_visual + k_keep
            KP = [K[l][:, :, :n_d + 1].contiguous() for l in range(Lx)]     # pruned-cache stand-ins: n_d + 1 rows
            VP = [V[l][:, :, :n_d + 1].contiguous() for l in range(Lx)]
            ws_d = torch.empty(h.workspace_bytes(h.CALL_DRAFT_ATTENTION, h.kv_desc(KP[0], cfg.n_q_heads), None, 1,
                                                 n_d + 1), dtype=torch.uint8, device="cuda")
            if name == "c4_long":
                # the long video keeps the 16x16 frames of the 16K layers whole, so its prune is timed too
                # (layer 0's draft cache is then the library's own gather)
                q_txt = torch.cat([dev(layers[0]["q_txt"], "bf16"), dev(layers[1]["q_txt"], "bf16")], dim=1)
                scores = torch.empty((cfg.batch, cfg.n_visual), dtype=torch.float32, device="cuda")
                idx = torch.empty((cfg.batch, k_keep), dtype=torch.int32, device="cuda")
                ws_s = torch.empty(h.workspace_bytes(h.CALL_SCORE_TOKENS, kvd, vid, cfg.l_txt, n_ctx),
                                   dtype=torch.uint8, device="cuda")
                ws_sel = torch.empty(256, dtype=torch.uint8, device="cuda")

                def prune():
                    h.hippo_score_tokens(q_txt, K[0][:, :, :n_ctx], vid, scores_out=scores, workspace=ws_s)
                    h.hippo_select_gather_kv(scores, k_keep, K[0][:, :, :n_ctx], V[0][:, :, :n_ctx], vid,
                                             cfg.n_q_heads, idx_out=idx, k_dst=KP[0][:, :, :n_d],
                                             v_dst=VP[0][:, :, :n_d], workspace=ws_sel)
                out["%s:prune_keep%d%%" % (name, pct)] = round(float(np.median(samples_us(capture(prune)))), 2)

            def draft_all():
                for l in range(Lx):
                    h.hippo_draft_attention(Q1[l], KP[l], VP[l], n_d, out=out_d, workspace=ws_d)

            def round_():
                cur = torch.cuda.current_stream()
                sB.wait_stream(cur)
                for l in range(Lx):
                    h.hippo_verify_attention(Q[l], K[l], V[l], n_ctx, out=out_v, workspace=ws_v)
                    h.hippo_draft_attention(Q1[l], KP[l], VP[l], n_d, out=out_d, workspace=ws_d, stream=sB)
                cur.wait_stream(sB)

            out["%s:draft_alone_per_layer_keep%d%%" % (name, pct)] = round(
                float(np.median(samples_us(capture(draft_all), per=Lx))), 3)
            if pct == cfg.keep_pct:
                xs = samples_us(capture(round_), reps=20, per=Lx)
                out["%s:round(verify||draft)_per_layer[min,median,max]" % name] = stat3(xs)
                out["%s:round_frac_of_hbm_peak(median)" % name] = round(
                    bytes_layer / np.median(xs) / 1e3 / HBM_PEAK_GBS, 4)
            del KP, VP
        out["%s:[layers, KV bytes per layer]" % name] = [Lx, bytes_layer]
        del K, V, Q, Q1
        torch.cuda.empty_cache()
    return out


def cpu_baseline(args, cfg, layers, kv_bytes, L):
    """The float64 oracle as it stands, on the host cores, one bounded leg per entry point (about
    25 s in all).  The top-level value stays the verify-attention leg."""
    import numpy as np

    import oracle
    n_ctx = cfg.ctx_len
    x0 = layers[0]
    legs, res = {}, {}

    def loop(fn, budget_s, max_calls=0):
        n, t0 = 0, time.perf_counter()
        while True:
            fn(n)
            n += 1
            t = time.perf_counter() - t0
            if t > budget_s or (max_calls and n >= max_calls):
                return n, t

    def score(i):
        res["scores"], _ = oracle.score_tokens(x0["q_txt"], x0["k"][:, :, :n_ctx], cfg.n_prefix, cfg.n_frames,
                                               cfg.grid_h, cfg.grid_w)
    n, t = loop(score, 5.0)
    legs["score_tokens"] = {"value": round(cfg.batch * cfg.n_visual * n / t, 1), "unit": "visual tokens/s",
                            "seconds": round(t, 2), "sample": "%d whole scoring calls (Eq. 2-7) on layer 0" % n}
    sc = res["scores"].astype(np.float32)

    def select(i):
        idx = oracle.topk(sc, cfg.k_keep)
        res["kp"] = oracle.gather(x0["k"][:, :, :n_ctx], cfg.n_prefix, cfg.n_visual, idx)
        res["vp"] = oracle.gather(x0["v"][:, :, :n_ctx], cfg.n_prefix, cfg.n_visual, idx)
    n, t = loop(select, 4.0)
    legs["select_gather_kv"] = {"value": round(cfg.batch * cfg.n_visual * n / t, 1), "unit": "visual tokens/s",
                                "seconds": round(t, 2),
                                "sample": "%d whole top-k (literal ranking) + K and V gathers on layer 0" % n}
    kp = np.concatenate([res["kp"], x0["k"][:, :, n_ctx:n_ctx + 1]], axis=2)
    vp = np.concatenate([res["vp"], x0["v"][:, :, n_ctx:n_ctx + 1]], axis=2)
    n_d = kp.shape[2] - 1
    d_bytes = cfg.batch * cfg.n_kv_heads * (n_d + 1) * cfg.head_dim * 2 * (2 if cfg.dtype == "bf16" else 4)

    def draft(i):
        oracle.attention(x0["q_new"][:, :1], kp, vp, n_d)
    n, t = loop(draft, 3.0)
    legs["draft_attention"] = {"value": round(d_bytes * n / t / 1e9, 3), "unit": "GB/s", "seconds": round(t, 2),
                               "us_per_call": round(t / n * 1e6, 1),
                               "sample": "%d draft-attention calls (1 row, %d pruned cache rows)" % (n, n_d + 1)}

    def verify(i):
        l = i % L
        oracle.attention(layers[l]["q_new"], layers[l]["k"], layers[l]["v"], n_ctx)
    n, t = loop(verify, 10.0, args.cpu_layers)
    legs["verify_attention"] = {"value": round(kv_bytes * n / t / 1e9, 3), "unit": "GB/s", "seconds": round(t, 2),
                                "sample": "%d verify-attention calls cycling over the %d layer caches" % (n, L)}
    return {"value": legs["verify_attention"]["value"], "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": "%d verify-attention calls cycling over the %d layer caches of this workload (all heads, "
                      "all %d query rows), float64 C oracle, %.1f s; `legs` holds the other entry points" % (
                          n, L, cfg.q_len, t),
            "legs": legs}


if __name__ == "__main__":
    main()
