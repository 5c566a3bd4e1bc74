#!/usr/bin/env python3
"""Benchmark of the rollout + rescoring hot path on one MI355X.

One "step" = rollout_generate on a synthetic left-padded query batch, then score_sequences (the teacher-forced
forward pass that yields every position's log-probability and value) on the rollout's own (tokens, mask) output.
score_responses, the same pass restricted to the response positions PPO reads, is timed beside it (outside the
timed region) and reported as `score_responses`; --score-responses makes it the step's rescoring call.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12       # B/s, MI355X HBM3E
MFMA_PEAK = 2.5e15      # flop/s, dense fp16/bf16 MFMA


def measured_ceilings():
    """Runs the stand-alone ceilings driver (a streaming read of 2 GiB; a bare matrix-instruction loop on zero and
    on random fp16 operands) in a child process before this process touches the GPU.  None if it was not built."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2403_17031_amd", "ceilings_driver")
    if not os.path.exists(exe):
        return None
    try:
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        return json.loads(r.stdout.strip().splitlines()[-1]) if r.returncode == 0 else None
    except Exception:
        return None


def gemm_traffic_per_row(cfg):
    """L2-miss bytes per GEMM row and launch of the per-layer products (FETCH_SIZE + WRITE_SIZE on gemm_driver,
    scaled by a copy kernel of known size; written by paper_2403_17031_amd/pmc_summary.py): for the 2.8B width
    only, where it was measured.  Returns (bytes per row, commit it was measured at) or (None, None)."""
    path = os.path.join(ROOT, "profiles", "pmc_gemm_traffic_config4.json")
    if cfg.d_model != 2560 or cfg.dtype == "fp32" or not os.path.exists(path):
        return None, None
    d = json.load(open(path))
    return float(d["bytes_per_gemm_row"]), d.get("commit")


def work_counts(cfg, n, resp, N, score_all=False):
    """Algorithmic flops / bytes of the workload from the drawn lengths (real tokens only).  Unless score_all, the
    rescoring pass is counted as score_responses needs it: every row through all layers but the last and through
    the last layer's QKV product; the rows from the last query column on (resp + 1 per sequence) through the last
    layer's attention, out-projection and MLP; the LM head on the resp rows that predict a response token."""
    import numpy as np
    L, d, F, V = cfg.n_layers, cfg.d_model, cfg.d_ff, cfg.vocab
    es = 4 if cfg.dtype == "fp32" else 2
    P_l = 4 * d * d + 2 * d * F
    mm = 2 * L * P_l                     # matmul flop per token through all layers
    lm = 2 * V * d
    attn = lambda k: L * 4 * d * k * (k + 1) / 2
    n = n.astype(np.float64)
    m = n + resp
    B = len(n)
    kv_tok = L * 2 * d * es              # K+V bytes of one cached token
    W = (L * (P_l + 3 * d + d + F + d + 4 * d) + V * d) * es   # bytes streamed per decode pass (no embed_in)
    kv_read = sum(kv_tok * (n + t + 1) for t in range(N - 1)).sum()
    # Prefill of a rollout: the final layer forms K and V (and Q) for every row, but only the last row of each
    # sequence goes through its attention, out-projection and MLP.
    mm_pre = 2 * ((L - 1) * P_l + 3 * d * d) if L > 0 else 0
    last_rows = 2 * (d * d + 2 * d * F) if L > 0 else 0
    attn_pre = lambda k: (L - 1) * 4 * d * k * (k + 1) / 2 + 4 * d * k if L > 0 else 0 * k
    if score_all or L == 0:
        gemm_sc = float(m.sum() * mm)
        lm_sc = float(m.sum() * lm)
        attn_sc = float(attn(m).sum())
        gemm_rows = m.sum() * 3 * L
    else:
        r = np.where(n > 0, resp + 1, 0).astype(np.float64)   # rows of a sequence from the last query column on
        gemm_sc = float(m.sum() * 2 * ((L - 1) * P_l + 3 * d * d) + r.sum() * 2 * (d * d + 2 * d * F))
        lm_sc = float(resp.sum() * lm)
        tri = lambda k: k * (k + 1) / 2
        attn_sc = float(((L - 1) * 4 * d * tri(m) + 4 * d * (tri(m) - tri(m - r))).sum())
        gemm_rows = m.sum() * (3 * (L - 1) + 1) + r.sum() * 2
    # launches of the large per-layer products (QKV, FC1, out-projection + FC2 as one) and the rows they cover
    gemm_launches = 3 * L + (3 * (L - 1) + 1 if L > 0 else 0)
    gemm_rows += n.sum() * (3 * (L - 1) + 1 if L > 0 else 0)
    return dict(
        prefill_flops=float((n * mm_pre + attn_pre(n)).sum() + B * (last_rows + lm)),
        score_flops=gemm_sc + lm_sc + attn_sc,
        gemm_rows_per_launch=float(gemm_rows / gemm_launches) if gemm_launches else 0.0,
        decode_bytes=float((N - 1) * W + kv_read + (N - 1) * B * kv_tok),
        decode_kv_read_bytes=float(kv_read),
        decode_flops=float((N - 1) * B * (mm + lm)),
        gemm_flops_prefill=float(n.sum() * mm_pre), gemm_flops_score=gemm_sc,
        lm_flops_score=lm_sc, weights_bytes=float(W), real_score_tokens=float(m.sum()),
        # the packed causal attention kernel: every layer of scoring, all but the final layer of prefill
        attn_flops=float(attn(m).sum() + (attn(n).sum() * (L - 1) / L if L > 0 else 0.0)),  # as run: all queries
        real_query_tokens=float(n.sum()),
        # one update iteration: a forward pass over every row (LM head on the response rows) and twice its flops
        # for the gradients
        update_flops=3.0 * float((m * mm + attn(m)).sum() + resp.sum() * lm))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4, help="BASELINE config index 1..5 (default: the 2.8B target)")
    ap.add_argument("--batch", type=int, default=None, help="override the config's batch (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="do not run the ceilings driver first (e.g. under a profiler, which should see this process only)")
    ap.add_argument("--no-update-leg", action="store_true",
                    help="skip the PPO-update leg (forward keeping activations, backward, AdamW; ~10 s at config 4)")
    ap.add_argument("--profile-update", action="store_true",
                    help="add per-kernel times of one more update iteration to the ppo_update object")
    ap.add_argument("--score-responses", action="store_true",
                    help="rescoring with score_responses (log-probs and values of the response columns only) instead of "
                         "score_sequences")
    ap.add_argument("--no-extra-score-shapes", action="store_true",
                    help="skip timing score_sequences on the paper's other batch shapes: right-padded (B,638) and (B/4,2021)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU (sequences are independent, so a batch would shard by "
                 "sequence with no communication inside a pass; that is not built here): --gpus must be 1")

    import numpy as np
    import torch
    import paper_2403_17031_amd as P
    from synth import WORKLOADS, make_weights, make_queries

    ceil = None if a.no_ceilings else measured_ceilings()   # before this process holds the GPU
    wl = WORKLOADS[a.config]
    cfg = wl.model
    B = a.batch or wl.batch
    N = wl.new_tokens
    t0 = time.time()
    w = make_weights(cfg, wl.weight_seed, threads=16)
    queries, mask = make_queries(wl, batch=B)
    pol = P.Policy(cfg, w, device="cuda:0")
    q_d = torch.from_numpy(queries).cuda()
    m_d = torch.from_numpy(mask).cuda()
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def score(toks, omask):
        if a.score_responses:
            return pol.score_responses(toks, omask, wl.query_len, wl.temperature)
        return pol.score_sequences(toks, omask, wl.temperature)

    def step():
        toks, lps, lens, omask = pol.rollout_generate(q_d, m_d, wl.sample_seed, wl.temperature, N, return_mask=True)
        lp, val = score(toks, omask)
        return toks, lps, lens, omask, lp, val

    for _ in range(a.warmup):
        out = step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * a.steps)]
    t1 = time.time()
    for i in range(a.steps):
        ev[3 * i].record()
        r = pol.rollout_generate(q_d, m_d, wl.sample_seed, wl.temperature, N, return_mask=True)
        ev[3 * i + 1].record()
        s = score(r[0], r[3])
        ev[3 * i + 2].record()
    torch.cuda.synchronize()
    wall = time.time() - t1
    roll_ms = float(np.mean([ev[3 * i].elapsed_time(ev[3 * i + 1]) for i in range(a.steps)]))
    score_ms = float(np.mean([ev[3 * i + 1].elapsed_time(ev[3 * i + 2]) for i in range(a.steps)]))
    prefill_ms, decode_ms = pol.last_rollout_phases()
    lens = r[2].cpu().numpy()
    n_true = mask.sum(1)
    wc = work_counts(cfg, n_true, lens, N, score_all=not a.score_responses)
    # the restricted rescoring call beside the full one (outside the timed region): what a PPO step would run
    wc_r = work_counts(cfg, n_true, lens, N, score_all=False)
    er = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    pol.score_responses(r[0], r[3], wl.query_len, wl.temperature)
    er[0].record()
    pol.score_responses(r[0], r[3], wl.query_len, wl.temperature)
    er[1].record()
    torch.cuda.synchronize()
    sr_ms = er[0].elapsed_time(er[1])
    score_resp = {"ms": sr_ms, "mfma_frac": wc_r["score_flops"] / (sr_ms * 1e-3) / MFMA_PEAK,
                  "step_ms_with_it": roll_ms + sr_ms, "step_tok_s_with_it": B * N / ((roll_ms + sr_ms) * 1e-3),
                  "note": "score_responses(first_col = query length): log-probs of the response columns and values "
                          "from the last query column on; flops counted as that pass needs them"}

    # one more step with per-kernel HIP events (outside the timed region) for the roofline object
    pol.profile_enable(True)
    step()
    prof = pol.profile_read()
    pol.profile_enable(False)
    # the four decode products are recorded one by one; their sum is the "gemm_decode" class
    dec = [v for k, v in prof.items() if k.startswith("gemm_decode_")]
    if dec:
        prof["gemm_decode"] = (sum(v[0] for v in dec), sum(v[1] for v in dec))
    tot = sum(v[0] for k, v in prof.items() if k != "gemm_decode")
    kern = {k: {"ms": round(v[0], 3), "launches": v[1]} for k, v in sorted(prof.items(), key=lambda kv: -kv[1][0])}
    dom = max(prof.items(), key=lambda kv: kv[1][0])[0]
    rooflines = {}
    if "gemm" in prof:
        fl = wc["gemm_flops_prefill"] + wc["gemm_flops_score"]
        ach = fl / (prof["gemm"][0] * 1e-3)
        # Memory traffic of the per-layer GEMMs cannot be counted in this process (hardware counters are collected
        # on the stand-alone gemm_driver, see profiles/pmc_gemm_traffic_config4.md): what leaves the L2s per GEMM
        # row and launch, Infinity-Cache hits included (an upper bound of the HBM bytes), times this run's mean
        # rows per launch.
        per_row, traffic_commit = gemm_traffic_per_row(cfg)
        traffic = per_row * wc["gemm_rows_per_launch"] if per_row else None
        rooflines["gemm"] = {"bound": "mfma", "achieved": ach / 1e12, "peak": MFMA_PEAK / 1e12, "unit": "TFLOP/s",
                             "frac": ach / MFMA_PEAK, "traffic": traffic, "traffic_measured_at_commit": traffic_commit,
                             "avg_launch_ms": prof["gemm"][0] / prof["gemm"][1]}
    if "attn_decode" in prof:
        by = wc["decode_kv_read_bytes"]
        ach = by / (prof["attn_decode"][0] * 1e-3)
        # FETCH_SIZE + WRITE_SIZE of this kernel on the stand-alone attn_driver (head size 80, see
        # profiles/pmc_attn_decode_traffic_config4.md): 1.004 x the algorithmic K/V bytes, every row fetched once
        a_traffic = 1.004 * by / prof["attn_decode"][1] if cfg.head_dim == 80 and cfg.dtype != "fp32" else None
        rooflines["attn_decode"] = {"bound": "hbm", "achieved": ach / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                                    "frac": ach / HBM_PEAK, "traffic": a_traffic,
                                    "avg_launch_ms": prof["attn_decode"][0] / prof["attn_decode"][1]}
    # the smaller kernel classes, each against the roof that bounds it (algorithmic work over measured time)
    es = 4 if cfg.dtype == "fp32" else 2
    Lr, dm = cfg.n_layers, cfg.d_model
    tok_pre, tok_sc = wc["real_query_tokens"], wc["real_score_tokens"]

    def _hbm(name, nbytes):
        if name in prof and prof[name][0] > 0:
            a_ = nbytes / (prof[name][0] * 1e-3)
            rooflines[name] = {"bound": "hbm", "achieved": a_ / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                               "frac": a_ / HBM_PEAK, "traffic": None,
                               "avg_launch_ms": prof[name][0] / prof[name][1]}

    _hbm("layernorm", (tok_pre + tok_sc) * Lr * dm * (4 + 2 * es))       # fp32 row in, two normalised rows out
    _hbm("rope_kv", (tok_pre + tok_sc) * Lr * 3 * dm * es * 2)           # q, k, v in; q and the K/V rows out
    _hbm("gemm_decode", (N - 1) * (wc["weights_bytes"] - cfg.vocab * dm * es))  # layer weights once per pass
    if "attn_prefill" in prof and prof["attn_prefill"][0] > 0:
        a_ = wc["attn_flops"] / (prof["attn_prefill"][0] * 1e-3)
        rooflines["attn_prefill"] = {"bound": "mfma", "achieved": a_ / 1e12, "peak": MFMA_PEAK / 1e12,
                                     "unit": "TFLOP/s", "frac": a_ / MFMA_PEAK, "traffic": None,
                                     "avg_launch_ms": prof["attn_prefill"][0] / prof["attn_prefill"][1]}
    # fractions of what this box was measured to sustain, next to the fractions of the published peaks
    if ceil:
        for rf in rooflines.values():
            top = ceil["mfma_f16_random_TFLOPs"] if rf["bound"] == "mfma" else ceil["stream_read_GBps"]
            rf["frac_of_measured"] = rf["achieved"] / top
    roof = rooflines.get(dom) or rooflines.get("gemm") or {}
    roof = dict(roof, kernel=dom if dom in rooflines else "gemm")

    # The signals PPO consumes next (reward assembly, GAE, advantage whitening, the clipped objective with its
    # output gradients) on this step's outputs.
    # Outside the headline metric.  Stand-ins: the policy's own rescoring outputs serve as the reference
    # log-probs and the reward-model values (a second and third weight set would cost two more
    # score_sequences calls of the time reported as score_ms).
    toks_d, lps_d, _, _ = r
    lp_d, val_d = s
    Lq = wl.query_len
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    for i in range(reps + 2):
        if i == 2:
            e0.record()
        rew, _, _, kept = P.ppo_assemble_rewards(lps_d, lp_d, val_d, toks_d, Lq, cfg.eos_id, cfg.pad_id, 0.05)
        adv, ret = P.ppo_gae(rew, val_d, kept, 1.0, 0.95, value_offset=Lq - 1)
        wadv = P.ppo_whiten(adv, kept)
        # the clipped objective and its gradient w.r.t. the model outputs, as in the first PPO epoch
        # (new outputs = the rollout's own)
        P.ppo_loss(lps_d, lps_d, wadv, val_d[:, Lq - 1:Lq - 1 + N], val_d[:, Lq - 1:Lq - 1 + N], ret, kept)
    e1.record()
    torch.cuda.synchronize()
    signals_ms = e0.elapsed_time(e1) / reps

    # The optimizer step of the PPO update (AdamW over fp32 master weights, moments and the bf16 copy) on
    # 2^30 parameters: 16 bytes read and 14 written per element.  Outside the headline metric.
    n_opt = 1 << 30
    o_p = torch.zeros(n_opt, dtype=torch.float32, device="cuda")
    o_g = torch.full((n_opt,), 1e-3, dtype=torch.float32, device="cuda")
    o_m, o_v = torch.zeros_like(o_p), torch.zeros_like(o_p)
    o_b = torch.empty(n_opt, dtype=torch.bfloat16, device="cuda")
    for i in range(1 + 3):
        if i == 1:
            e0.record()
        P.adamw_step(o_p, o_g, o_m, o_v, i + 1, param_bf16=o_b)
    e1.record()
    torch.cuda.synchronize()
    adamw_ms = e0.elapsed_time(e1) / 3
    ach = 30.0 * n_opt / (adamw_ms * 1e-3)
    rooflines["adamw"] = {"bound": "hbm", "achieved": ach / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                          "frac": ach / HBM_PEAK, "traffic": None, "avg_launch_ms": adamw_ms}
    del o_p, o_g, o_m, o_v, o_b

    # The backward pass through the output heads over the batch's B*N response positions (what the PPO
    # update differentiates): three products of 2*T*V*d flop each (logits, dL/dh, dL/dW).  Outside the
    # headline metric.
    bwd_legs = a.config != 5   # the 6.9B shape fills the GPU with weights and the rollout workspace alone
    head_bwd_ms = None
    g_hb = torch.Generator(device="cuda").manual_seed(7)
    hb_peak = MFMA_PEAK if cfg.dtype != "fp32" else 157.3e12
    if bwd_legs:
        T_hb = B * N
        x_hb = torch.randn(T_hb, cfg.d_model, device="cuda", generator=g_hb) * 2.0
        y_hb = torch.randint(0, cfg.vocab, (T_hb,), device="cuda", generator=g_hb, dtype=torch.int32)
        gl_hb = torch.randn(T_hb, device="cuda", generator=g_hb) / T_hb
        gv_hb = torch.randn(T_hb, device="cuda", generator=g_hb) / T_hb
        for i in range(1 + 2):
            if i == 1:
                e0.record()
            hb = pol.head_backward(x_hb, y_hb, gl_hb, gv_hb, wl.temperature, grad_scale=64.0 * T_hb)
        e1.record()
        torch.cuda.synchronize()
        head_bwd_ms = e0.elapsed_time(e1) / 2
        ach = 3 * 2.0 * T_hb * cfg.vocab * cfg.d_model / (head_bwd_ms * 1e-3)
        rooflines["head_backward"] = {"bound": "mfma", "achieved": ach / 1e12, "peak": hb_peak / 1e12, "unit": "TFLOP/s",
                                      "frac": ach / hb_peak, "traffic": None, "avg_launch_ms": head_bwd_ms,
                                      "rows": T_hb}
        del x_hb, y_hb, gl_hb, gv_hb, hb

    # The backward pass through one decoder layer's MLP branch over the batch's packed rows (the rows the
    # scoring pass runs over): forward recomputation (1 product) + four gradient products of 2*T*d*d_ff flop.
    # Outside the headline metric.
    mlp_bwd_ms = None
    if cfg.n_layers > 0 and bwd_legs:
        T_mb = int(wc["real_score_tokens"])
        x_mb = torch.randn(T_mb, cfg.d_model, device="cuda", generator=g_hb) * 2.0
        g_mb = torch.randn(T_mb, cfg.d_model, device="cuda", generator=g_hb)
        for i in range(1 + 2):
            if i == 1:
                e0.record()
            mb = pol.mlp_backward(0, x_mb, g_mb)
        e1.record()
        torch.cuda.synchronize()
        mlp_bwd_ms = e0.elapsed_time(e1) / 2
        ach = 5 * 2.0 * T_mb * cfg.d_model * cfg.d_ff / (mlp_bwd_ms * 1e-3)
        rooflines["mlp_backward"] = {"bound": "mfma", "achieved": ach / 1e12, "peak": hb_peak / 1e12,
                                     "unit": "TFLOP/s", "frac": ach / hb_peak, "traffic": None,
                                     "avg_launch_ms": mlp_bwd_ms, "rows": T_mb}
        del x_mb, g_mb, mb

    # The backward pass through the packed causal attention of one layer over the same rows (sequence lengths
    # of the scoring pass): five contractions of 2*hd flop per (query, key <= query, head) pair.
    attn_bwd_ms = None
    if cfg.n_layers > 0 and cfg.dtype != "fp32" and bwd_legs:
        n_sc = (n_true + lens).astype(np.int64)
        cu_ab = np.concatenate([[0], np.cumsum(n_sc)]).astype(np.int32)
        T_ab = int(cu_ab[-1])
        qkvg = [(torch.randn(T_ab, cfg.d_model, device="cuda", generator=g_hb)).half() for _ in range(4)]
        cu_dev = torch.from_numpy(cu_ab).cuda()
        for i in range(1 + 2):
            if i == 1:
                e0.record()
            ab = P.attention_backward(*qkvg, cu_dev, cfg.n_heads, max_len=int(n_sc.max()))
        e1.record()
        torch.cuda.synchronize()
        attn_bwd_ms = e0.elapsed_time(e1) / 2
        ach = 5 * 2.0 * cfg.d_model * float((n_sc * (n_sc + 1) // 2).sum()) / (attn_bwd_ms * 1e-3)
        rooflines["attention_backward"] = {"bound": "mfma", "achieved": ach / 1e12, "peak": MFMA_PEAK / 1e12,
                                           "unit": "TFLOP/s", "frac": ach / MFMA_PEAK, "traffic": None,
                                           "avg_launch_ms": attn_bwd_ms, "rows": T_ab}
        del qkvg, ab

    # The paper's other scoring shapes (reward-model batches of 638 tokens, long-context batches of 2021),
    # right-padded with true lengths uniform in [L/4, L]; outside the headline metric.
    extra = None
    if not a.no_extra_score_shapes:
        extra = {}
        for L, Bx in ((638, B), (2021, max(1, B // 4))):
            g = np.random.default_rng(wl.data_seed + L)
            xl = g.integers(L // 4, L + 1, Bx)
            xt = g.integers(1, cfg.pad_id, (Bx, L)).astype(np.int32)
            xm = (np.arange(L)[None, :] < xl[:, None]).astype(np.uint8)
            xt[xm == 0] = cfg.pad_id
            xt_d, xm_d = torch.from_numpy(xt).cuda(), torch.from_numpy(xm).cuda()
            pol.score_sequences(xt_d, xm_d, 1.0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            pol.score_sequences(xt_d, xm_d, 1.0)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            n_ = xl.astype(np.float64)
            Lc, d_, F_, V_ = cfg.n_layers, cfg.d_model, cfg.d_ff, cfg.vocab
            fl = float((n_ * (2 * Lc * (4 * d_ * d_ + 2 * d_ * F_) + 2 * V_ * d_) + Lc * 4 * d_ * n_ * (n_ + 1) / 2).sum())
            extra[f"B{Bx}xL{L}"] = {"ms": ms, "real_tok_s": float(xl.sum()) / (ms * 1e-3),
                                    "mfma_frac": fl / (ms * 1e-3) / MFMA_PEAK}

    # One iteration of the PPO update over the rollout batch through rlhf_ppo_update (outside the headline metric):
    # forward pass keeping the layer inputs, the clipped objective, the whole backward pass, AdamW over every weight
    # and the refresh of the fp16 weight image; the paper's update is K = 4 such iterations.  Advantages and returns
    # are synthetic, the old log-probs and values are the rollout's own.  Config 5 (6.9B) is skipped: weights,
    # optimizer state and kept activations exceed one GPU.
    update = None
    if not a.no_update_leg and cfg.n_layers > 0 and cfg.dtype != "fp32" and bwd_legs:
        toks_u, mask_u = r[0], r[3]
        adv_u = torch.randn(B, N, device="cuda", generator=g_hb)
        ret_u = torch.randn(B, N, device="cuda", generator=g_hb)
        oldv_u = val_d[:, Lq - 1:Lq - 1 + N].contiguous()
        kept_u = r[2]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for it in range(2):                              # one untimed iteration, one timed
            if it == 1:
                ev[0].record()
            st_u = pol.ppo_update(toks_u, mask_u, Lq, lps_d, adv_u, oldv_u, ret_u, kept_u, wl.temperature, epochs=1,
                                  n_minibatches=1)
        ev[1].record()
        torch.cuda.synchronize()
        upd_ms = ev[0].elapsed_time(ev[1])
        free_b, total_b = torch.cuda.mem_get_info()
        update = {"iteration_ms": upd_ms, "rows": int(mask_u.sum().item()), "loss": float(st_u[0, 0]),
                  "hbm_in_use_gb": (total_b - free_b) / 1e9,   # whole process: rollout workspace, weights, optimizer state, kept activations
                  "tflops": wc["update_flops"] / (upd_ms * 1e-3) / 1e12,
                  "note": "one of the K = 4 iterations of an update; 3 x the forward pass's flops (every row through "
                          "the layers, the LM head on the response rows; twice that for the gradients) over its time, "
                          "AdamW and the weight-image refresh included"}
        if a.profile_update:   # one more iteration with per-kernel HIP events
            pol.profile_enable(True)
            pol.ppo_update(toks_u, mask_u, Lq, lps_d, adv_u, oldv_u, ret_u, kept_u, wl.temperature, epochs=1,
                           n_minibatches=1)
            up = pol.profile_read()
            pol.profile_enable(False)
            update["kernels_ms"] = {k: {"ms": round(v[0], 3), "launches": v[1]}
                                    for k, v in sorted(up.items(), key=lambda kv: -kv[1][0])}
        pol._train = None

    cpu = None
    if not a.no_cpu_baseline:
        cpu = cpu_baseline(cfg, w, queries, mask, wl, n_true)

    if ceil:
        for rf in rooflines.values():
            if "frac_of_measured" not in rf:
                top = ceil["mfma_f16_random_TFLOPs"] if rf["bound"] == "mfma" else ceil["stream_read_GBps"]
                rf["frac_of_measured"] = rf["achieved"] / top
    ms_step = wall / a.steps * 1e3
    out = {
        "metric": "rollout generated tokens/s (rollout_generate + %s per step)" % (
            "score_responses" if a.score_responses else "score_sequences"),
        "value": B * N / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "fp32" else "f16 operands / f32 accumulate (bf16 weights)",
        "data": "synthetic",
        "config": {"workload": wl.name, "batch": B, "query_len": wl.query_len, "new_tokens": N,
                   "temperature": wl.temperature, "real_query_tokens": int(n_true.sum()),
                   "mean_response_len": float(lens.mean()),
                   "seeds": [wl.weight_seed, wl.data_seed, wl.sample_seed]},
        "generated_tok_s": B * N / (roll_ms * 1e-3), "rollout_ms": roll_ms,
        "prefill_ms": prefill_ms, "decode_ms": decode_ms,
        "decode_tok_s": B * (N - 1) / (decode_ms * 1e-3),
        "decode_hbm_frac": wc["decode_bytes"] / (decode_ms * 1e-3) / HBM_PEAK,
        "prefill_mfma_frac": wc["prefill_flops"] / (prefill_ms * 1e-3) / MFMA_PEAK,
        "rescoring_tok_s": wc["real_score_tokens"] / (score_ms * 1e-3), "score_ms": score_ms,
        "rescoring_tok_s_padded": B * (wl.query_len + N) / (score_ms * 1e-3),
        "score_mfma_frac": wc["score_flops"] / (score_ms * 1e-3) / MFMA_PEAK,
        "score_responses": score_resp,
        "roofline": roof, "rooflines": rooflines, "kernels_ms": kern, "profiled_step_ms": tot,
        "ceilings": ceil,
        "decode_frac_of_measured_stream": (wc["decode_bytes"] / (decode_ms * 1e-3) / (ceil["stream_read_GBps"] * 1e9)) if ceil else None,
        "prefill_frac_of_measured_mfma": (wc["prefill_flops"] / (prefill_ms * 1e-3) / (ceil["mfma_f16_random_TFLOPs"] * 1e12)) if ceil else None,
        "score_frac_of_measured_mfma": (wc["score_flops"] / (score_ms * 1e-3) / (ceil["mfma_f16_random_TFLOPs"] * 1e12)) if ceil else None,
        "ppo_signals_ms": signals_ms, "adamw_ms_per_2p30_params": adamw_ms, "head_backward_ms": head_bwd_ms, "mlp_backward_ms_per_layer": mlp_bwd_ms, "attention_backward_ms_per_layer": attn_bwd_ms, "ppo_update": update, "extra_score_shapes": extra,
        "cpu_baseline": cpu, "setup_s": setup_s,
    }
    print(json.dumps(out))


def cpu_baseline(cfg, w, queries, mask, wl, n_true):
    """The oracle, as it stands, on a bounded sample of the same workload: rows 0 and B-1 of the batch (B-1 alone
    when the batch has one row), 2 new tokens each (prefill + 1 cached decode pass), then rescoring of those rows."""
    import numpy as np
    from oracle import neox_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    B = queries.shape[0]
    rows = sorted({0, B - 1})
    n_new = min(2, wl.new_tokens)
    m = O.OracleModel(w, cfg, cache_f64=False)
    t_roll = t_score = 0.0
    n_scored = 0
    for b in rows:
        t0 = time.time()
        toks, lps, lens = O.rollout_generate(m, queries[b:b + 1], mask[b:b + 1], wl.sample_seed, wl.temperature, n_new,
                                             seq_id_base=b)
        t_roll += time.time() - t0
        full = np.concatenate([mask[b:b + 1], (np.arange(n_new)[None, :] < lens[:, None]).astype(np.uint8)], axis=1)
        t0 = time.time()
        O.score_sequences(m, toks, full, wl.temperature)
        t_score += time.time() - t0
        n_scored += int(full.sum())
    n_gen = n_new * len(rows)
    return {"value": n_gen / (t_roll + t_score), "unit": "tokens/s", "cores": int(cores),
            "kind": "oracle",
            "oracle_is": "oracle/neox_oracle.py: float64 numpy; its matrix products run on the BLAS that numpy links, "
                         "everything else is plain numpy",
            "sample": f"rows {rows} (queries of {[int(n_true[b]) for b in rows]} tokens), {n_new} new tokens each, "
                      f"then rescoring of those rows",
            "generated_tok_s": n_gen / t_roll, "rescoring_tok_s": n_scored / t_score,
            "rollout_s": t_roll, "score_s": t_score}


if __name__ == "__main__":
    main()
