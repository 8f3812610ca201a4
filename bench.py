#!/usr/bin/env python3
"""Benchmark of the SampleAttention prefill hot path on one MI355X.

One *step* = one pass of the whole path over one layer's attention inputs:
sa_sample_scores -> sa_select_strips -> sa_sparse_attn, chained on one stream
with the inputs already resident in HBM.  Prints ONE JSON line:

  metric  sparse prefill attention ms/layer (the headline metric) on the
          workload named in config.workload (default: the S=128K ChatGLM3-6B-
          shaped config, alpha = 0.95, literal generator constants); value is
          the median of the per-step durations between HIP events on the launch
          stream, ms_per_step the wall-clock mean over the same steps
  roofline      the strip-masked flash kernel against the bf16 MFMA peak:
                4*d*(computed 32x64 tiles) flop / mean kernel duration taken
                from HIP events the library records around the launch, on the
                launch stream, inside the timed region
  cpu_baseline  the fp64 oracle timed on this host on a bounded sample of the
                same workload, extrapolated linearly to one layer

Everything else on the line (per-stage times, the in-library dense kernel,
speedup, kept fractions, useful rate, alpha sweep with the recall of each mask,
the same workload at block granularity and with two chunks, separate column /
slash thresholds on heads of one pattern each, the same step replayed from a
captured HIP graph, the peaks this GPU reaches on a bare MFMA loop and a plain
copy) is context.  --sampling-study replaces the run
by a comparison of sampled against full scores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
TILE_FLOP = 4 * 128 * 32 * 64   # QK^T + PV of one 32x64 (query rows x keys) score tile at d = 128


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def to_device(bits: np.ndarray):
    import torch
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
    return t[None].contiguous().cuda()


def kept_pairs_per_row(S: int, cols: np.ndarray, offs: np.ndarray, window: int) -> np.ndarray:
    """Number of kept keys in every row of the strip mask of one head: selected columns at
    or before the row, plus kept offsets (selected or inside the window) that fit, minus
    the pairs that are both - a correlation of the two indicator vectors, taken with an
    FFT (counting only; exact after rounding)."""
    c = np.zeros(S)
    c[np.asarray(cols, dtype=np.int64)] = 1.0
    o = np.zeros(S)
    o[np.asarray(offs, dtype=np.int64)] = 1.0
    o[:window] = 1.0
    n = 1 << int(np.ceil(np.log2(2 * S)))
    both = np.fft.irfft(np.fft.rfft(c, n) * np.fft.rfft(o, n), n)[:S]      # both[i] = sum_j c[j] o[i - j]
    return np.cumsum(c) + np.cumsum(o) - np.rint(both)


def mask_density(S: int, cols: np.ndarray, offs: np.ndarray, window: int) -> float:
    """Kept fraction of the causal triangle for one head."""
    return float(kept_pairs_per_row(S, cols, offs, window).sum() / (S * (S + 1) / 2.0))


def schedule_slots(S: int, cols: np.ndarray, offs: np.ndarray, window: int) -> int:
    """Wave-tile slots the strip-masked kernel's schedule spends on one head: for every
    256-row query tile, 8 waves times (64-key tiles of gathered columns at or before its
    last row + 64-key tiles whose 319 offsets against the tile's rows hold a kept one).
    A slot is spent whether or not the wave has work on the tile (counting only)."""
    keep = np.zeros(S, dtype=bool)
    keep[np.asarray(offs, dtype=np.int64)] = True
    keep[:window] = True
    c = np.concatenate([[0], np.cumsum(keep)])
    nq = (S + 255) // 256
    nd = (S + 63) // 64 + 3
    d = np.arange(nd)
    lo, hi = np.clip(64 * d - 255, 0, S), np.clip(64 * d + 63, -1, S - 1)
    touched = (c[hi + 1] - c[lo] > 0) & (hi >= lo)
    n_rng_upto = np.concatenate([[0], np.cumsum(touched)])             # touched diagonals d < x
    last_row = np.minimum(256 * np.arange(nq) + 255, S - 1)
    n_col = (np.searchsorted(np.asarray(cols, dtype=np.int64), last_row, side="right") + 63) // 64
    n_rng = n_rng_upto[np.minimum(4 * np.arange(nq) + 4, nd)]           # diagonals d <= 4 a + 3
    return int(8 * (n_col.sum() + n_rng.sum()))


def touched_block_fraction(S: int, cols: np.ndarray, offs: np.ndarray, window: int, blk: int = 128) -> float:
    """Fraction of the blk x blk blocks of the causal triangle that hold at least one kept
    (query, key) pair for one head - the paper's "ratio of calculated blocks" grid (counting only)."""
    nb = (S + blk - 1) // blk
    col_blk = np.zeros(nb, dtype=bool)
    col_blk[np.unique(cols.astype(np.int64) // blk)] = True
    off_keep = np.zeros(S, dtype=bool)
    off_keep[offs] = True
    off_keep[:window] = True
    oo = np.nonzero(off_keep)[0].astype(np.int64)
    touched = 0
    for bi in range(nb):
        row = col_blk[:bi + 1].copy()                # a kept column j touches every block row >= j // blk
        lo = np.maximum(bi * blk, oo)                # rows of this block row that have a key at offset o
        hi = min((bi + 1) * blk, S) - 1
        ok = lo <= hi
        row[(lo[ok] - oo[ok]) // blk] = True
        row[(hi - oo[ok]) // blk] = True
        touched += int(row.sum())
    return touched / (nb * (nb + 1) / 2.0)


def block_mask_density(S: int, col_blocks: np.ndarray, slash_blocks: np.ndarray, window: int, blk: int) -> float:
    """Kept fraction of the blk x blk blocks of the causal triangle under the block
    mask (Algorithm 1 at block granularity): block (I, J), J <= I, is kept when J is a
    selected key block or I - J is a kept block diagonal - b and b + 1 for a selected
    offset block b, and the diagonals the local window reaches."""
    nb = (S + blk - 1) // blk
    diag = np.zeros(nb + 1, dtype=bool)
    diag[np.asarray(slash_blocks, dtype=np.int64)] = True
    diag[np.asarray(slash_blocks, dtype=np.int64) + 1] = True
    diag[: (window + blk - 2) // blk + 1] = True
    diag = diag[:nb]
    colk = np.zeros(nb, dtype=bool)
    colk[np.asarray(col_blocks, dtype=np.int64)] = True
    # diagonal delta holds nb - delta blocks; a kept column J holds nb - J blocks (rows I >= J)
    n_diag = int(np.sum(nb - np.nonzero(diag)[0]))
    n_col = int(np.sum(nb - np.nonzero(colk)[0]))
    # counted twice: kept column J on kept diagonal delta with J + delta <= nb - 1
    dd = np.nonzero(diag)[0]
    both = int(np.sum(np.searchsorted(dd, nb - 1 - np.nonzero(colk)[0], side="right")))
    return (n_diag + n_col - both) / (nb * (nb + 1) / 2.0)


def cpu_baseline(wl, x, alpha: float, budget_s: float) -> dict:
    """Oracle timing on a bounded sample (about 2 x budget_s of CPU work), scaled
    linearly to ms per layer.  The oracle runs as it stands: numpy fp64 on the
    host cores of this machine."""
    from oracle import sample_attention as O        # CPU-baseline leg only
    from sa_inputs import bf16_bits_to_f32
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    S, n_s = wl.seq_len, wl.n_sample_rows
    q = bf16_bits_to_f32(x["q"][0]).astype(np.float64)
    k = bf16_bits_to_f32(x["k"][0]).astype(np.float64)
    v = bf16_bits_to_f32(x["v"][0]).astype(np.float64)

    def timed(fn):
        t0 = time.perf_counter()
        r = fn()
        return r, time.perf_counter() - t0

    # stage 1: probe with a few rows, then size the sample to the budget
    probe = min(64, n_s)
    _, tp = timed(lambda: O.sample_scores(q, k, probe))
    rows1 = int(min(n_s, max(probe, 64 * int(budget_s / max(tp, 1e-6) * probe / 64))))
    (col, slash, _), t1 = timed(lambda: O.sample_scores(q, k, rows1))
    a32 = float(np.float32(alpha))
    (Ic, Is), t2 = timed(lambda: (O.select(col, a32), O.select(slash, a32)))
    # attention: same idea
    pr = np.linspace(0, S - 1, 8).astype(np.int64)
    _, tp = timed(lambda: O.masked_attn(q, k, v, Ic, Is, wl.window, rows=pr))
    n_att = int(min(S, max(8, budget_s / max(tp, 1e-6) * 8)))
    rows = np.linspace(0, S - 1, n_att).astype(np.int64)
    _, t3 = timed(lambda: O.masked_attn(q, k, v, Ic, Is, wl.window, rows=rows))
    per_head = t1 * (n_s / rows1) + t2 + t3 * (S / n_att)
    layer_ms = per_head * wl.n_q_heads * 1e3
    return {
        "value": layer_ms, "unit": "ms/layer", "cores": int(cores), "kind": "oracle",
        "sample": (f"query head 0 of {wl.n_q_heads}: stage 1 on the last {rows1} of {n_s} sampled rows "
                   f"({t1:.2f} s), selection on those scores ({t2:.2f} s), masked attention on "
                   f"{n_att} of {S} rows ({t3:.2f} s); scaled linearly to all rows and heads"),
    }


def sampling_study(sa, torch, wl, q, k, v, shape) -> int:
    """How much recall does sampling cost?  (Appendix "effectiveness of sampling": CRA
    reached by top-k strips chosen from a few sampled rows against top-k strips chosen
    from the full attention matrix, at equal k.)  Strip budgets are fractions of S for
    columns and offsets alike; the scores come from sa_sample_scores (all rows = n_s =
    S), the top-k lists from torch.topk (harness code, not part of the path), the
    recall from the log-sum-exps of sa_sparse_attn and sa_dense_attn."""
    S, Hq, w = wl.seq_len, wl.n_q_heads, wl.window
    _, dense_lse = sa.sa_dense_attn(q, k, v, want_lse=True)
    sources = [("all rows", S)] + [(f"last {n} rows", n) for n in sorted({128, wl.n_sample_rows}) if n < S]
    rows = []
    for name, n_s in sources:
        col, slash = sa.sa_sample_scores(q, k, n_s)
        for frac in (0.025, 0.05, 0.1, 0.2):
            kk = max(1, int(round(frac * S)))
            ci = torch.zeros(Hq, S, dtype=torch.int32, device="cuda")
            si = torch.zeros_like(ci)
            ci[:, :kk] = torch.topk(col, kk, dim=1).indices.sort(dim=1).values.int()
            si[:, :kk] = torch.topk(slash, kk, dim=1).indices.sort(dim=1).values.int()
            cnt = torch.full((Hq,), kk, dtype=torch.int32, device="cuda")
            _, lse, tiles = sa.sa_sparse_attn(q, k, v, ci, cnt, si, cnt, w, want_lse=True, want_tiles=True)
            torch.cuda.synchronize()
            r = torch.exp(lse - dense_lse)
            # the sampled rows are scored exactly; the question is how the mask does elsewhere
            rows.append({"scores_from": name, "n_rows": n_s, "strip_fraction": frac, "k": kk,
                         "recall_mean": float(r.mean()), "recall_p05": float(torch.quantile(r.flatten()[::7], 0.05)),
                         "cra_min": float(r.min())})
            log(f"sampling study: {json.dumps(rows[-1])}")
        del col, slash
    # the paper's remedy for bottom-only sampling: chunk_n segments, each masked by the strips its own
    # bottom rows select (here at the same budgets, counted per segment)
    for C in (4,):
        if S % (256 * C) != 0:
            continue
        col, slash = sa.sa_sample_scores(q, k, 128, n_chunks=C)
        for frac in (0.025, 0.05, 0.1, 0.2):
            kk = max(1, int(round(frac * S)))
            ci = torch.zeros(C, Hq, S, dtype=torch.int32, device="cuda")
            si = torch.zeros_like(ci)
            ci[:, :, :kk] = torch.topk(col, kk, dim=2).indices.sort(dim=2).values.int()
            si[:, :, :kk] = torch.topk(slash, kk, dim=2).indices.sort(dim=2).values.int()
            cnt = torch.full((C, Hq), kk, dtype=torch.int32, device="cuda")
            _, lse, _ = sa.sa_sparse_attn_chunked(q, k, v, ci, cnt, si, cnt, w, C, want_lse=True)
            torch.cuda.synchronize()
            r = torch.exp(lse - dense_lse)
            rows.append({"scores_from": f"last 128 rows of each of {C} segments", "n_rows": 128 * C,
                         "strip_fraction": frac, "k": kk, "recall_mean": float(r.mean()),
                         "recall_p05": float(torch.quantile(r.flatten()[::7], 0.05)), "cra_min": float(r.min())})
            log(f"sampling study: {json.dumps(rows[-1])}")
    print(json.dumps({"study": "sampled vs full scores at equal strip budgets", "workload": wl.name,
                      "seq_len": S, "window": w, "rows": rows}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="glm128k")
    ap.add_argument("--seq-len", type=int, default=0, help="override the workload's sequence length")
    ap.add_argument("--alpha", type=float, default=0.95)
    ap.add_argument("--structure-gain", type=float, default=1.0,
                    help="multiply the planted sink gain / query bias (labelled variant workload)")
    ap.add_argument("--dense-iters", type=int, default=2)
    ap.add_argument("--no-sweep", action="store_true", help="skip the alpha sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-block", action="store_true", help="skip the block-granularity runs")
    ap.add_argument("--no-alpha-grid", action="store_true",
                    help="skip the grid of separate column / slash thresholds on the three head patterns")
    ap.add_argument("--no-peaks", action="store_true", help="skip the MFMA / copy peak probes")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the replay of the same steps from a captured HIP graph")
    ap.add_argument("--heads-per-pass", type=int, default=0,
                    help="bound the workspace (long sequences): stage 1 and the attention take this many heads at a "
                         "time (sa_sparse_attn_partitioned); 0 = all heads at once")
    ap.add_argument("--sampling-study", action="store_true",
                    help="compare masks chosen from sampled scores with masks chosen from the scores of ALL rows "
                         "at equal strip budgets (recall of the dense softmax), then exit")
    ap.add_argument("--copy-calib-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (calibrates HBM byte counters)")
    ap.add_argument("--cpu-seconds", type=float, default=8.0,
                    help="CPU work per oracle leg (stage 1, attention) of the cpu_baseline sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2406_15486_amd as sa
    from sa_inputs import CONFIGS, make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sa.load_library()

    wl = CONFIGS[args.workload]
    if args.seq_len:
        wl = wl.scaled(args.seq_len)
    if args.structure_gain != 1.0:
        wl = wl.with_structure_gain(args.structure_gain)
    S, Hq, Hkv, n_s, w = wl.seq_len, wl.n_q_heads, wl.n_kv_heads, wl.n_sample_rows, wl.window
    log(f"workload {wl.name}: S={S} Hq={Hq} Hkv={Hkv} n_s={n_s} window={w} alpha={args.alpha}")
    t0 = time.perf_counter()
    x = make_inputs(wl)
    log(f"inputs generated on the host in {time.perf_counter() - t0:.1f} s")
    q, k, v = to_device(x["q"]), to_device(x["k"]), to_device(x["v"])
    shape = sa.Shape(1, Hq, Hkv, S)
    plan = sa.SampleAttentionPlan(shape, n_s, heads_per_pass=args.heads_per_pass or None)
    log(f"plan workspace {plan.ws.numel() / 1e9:.2f} GB"
        + (f" ({args.heads_per_pass} heads per pass)" if args.heads_per_pass else ""))
    torch.cuda.synchronize()

    if args.sampling_study:
        return sampling_study(sa, torch, wl, q, k, v, shape)

    if args.copy_calib_mib > 0:
        # a plain copy of known size: what FETCH_SIZE / WRITE_SIZE read for it scales the counters
        src = torch.empty(args.copy_calib_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region: K whole steps ----------------------------------------------
    for _ in range(args.warmup):
        plan.run(q, k, v, args.alpha, args.alpha, w)
    torch.cuda.synchronize()
    sa.sa_profile_enable(True)
    # an event pair per step on the launch stream (the library enqueues on torch's current stream)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e0, e1 in ev:
        e0.record()
        plan.run(q, k, v, args.alpha, args.alpha, w)
        e1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    step_ms = [e0.elapsed_time(e1) for e0, e1 in ev]
    ms_median = float(np.median(step_ms))
    stage = {name: sa.sa_profile_read(name) for name in
             ("row_lse", "score_accum", "score_final", "select", "transpose_v", "mask_prep", "sparse_flash")}
    # a kernel may run several times per step (one launch per pass over a group of heads); the
    # library keeps the last 64 launches of each kernel, i.e. a whole number m of the last steps
    def per_step(vv):
        if not vv:
            return None
        if len(vv) % args.steps == 0 and len(vv) < 64:
            return float(np.sum(vv)) / args.steps
        per = max(1, -(-Hq // (args.heads_per_pass or Hq)))          # launches per step
        m = max(1, len(vv) // per)
        return float(np.sum(vv[-m * per:])) / m
    stage_ms = {n: per_step(vv) for n, vv in stage.items()}
    log(f"ms/step: median of events {ms_median:.3f}, wall-clock mean {ms_per_step:.3f}; stages {json.dumps(stage_ms)}")

    tiles = plan.tiles.cpu().numpy().astype(np.int64)
    flash_ms = stage_ms["sparse_flash"]
    flop = float(tiles.sum()) * TILE_FLOP
    achieved = flop / (flash_ms * 1e-3) / 1e12
    # tiles a dense causal sweep computes: every 32-row block against the key tiles up to its last row
    dense_tiles = sum(((32 * b + 31) // 64 + 1) for b in range((S + 31) // 32)) * Hq
    cc = plan.col_cnt.cpu().numpy()
    sc = plan.slash_cnt.cpu().numpy()
    ci = plan.col_idx[0, :int(cc[0])].cpu().numpy()
    si = plan.slash_idx[0, :int(sc[0])].cpu().numpy()
    density0 = mask_density(S, ci, si, w)
    blocks0 = touched_block_fraction(S, ci, si, w)
    # useful rate: 4 d flop per KEPT (query, key) pair of every head's mask over the same kernel time
    ci_all, si_all = plan.col_idx.cpu().numpy(), plan.slash_idx.cpu().numpy()
    kept_pairs = float(sum(kept_pairs_per_row(S, ci_all[h, :int(cc[h])], si_all[h, :int(sc[h])], w).sum()
                           for h in range(Hq)))
    useful_tflops = 4.0 * 128 * kept_pairs / (flash_ms * 1e-3) / 1e12
    # slots of the kernel's schedule (busy or idle) against the computed wave tiles
    slots = float(sum(schedule_slots(S, ci_all[h, :int(cc[h])], si_all[h, :int(sc[h])], w) for h in range(Hq)))
    del ci_all, si_all
    ws_bytes = {"sample_scores": sa.sa_workspace_bytes(sa.binding.SA_OP_SAMPLE_SCORES, shape, n_s),
                "sparse_attn": sa.sa_workspace_bytes(sa.binding.SA_OP_SPARSE_ATTN, shape),
                "sparse_attn_4_heads_per_pass": sa.sa_partitioned_workspace_bytes(shape, 4, 1),
                "dense_attn": sa.sa_workspace_bytes(sa.binding.SA_OP_DENSE_ATTN, shape)}
    log(f"workspace bytes: {json.dumps(ws_bytes)}")
    # stages 1-2 against HBM: algorithmic bytes (K once per KV head and pass, the sampled Q rows,
    # the row statistics, the two score vectors; five passes over the scores for the selection)
    kv_b, qr_b, lse_b, sc_b = Hkv * S * 128 * 2, Hq * n_s * 128 * 2, Hq * n_s * 4, 2 * Hq * S * 4
    stage_bytes = {
        "row_lse": kv_b + qr_b + lse_b,
        "score_accum": kv_b + qr_b + lse_b + sc_b,
        "select": 5 * sc_b + 4 * float(cc.sum() + sc.sum()),
    }
    stage_gbs = {n: stage_bytes[n] / (stage_ms[n] * 1e-3) / 1e9 for n in stage_bytes if stage_ms.get(n)}
    # ... and against what actually bounds them: one QK^T contraction and one exponential per
    # (sampled row, key <= row) pair in each of the two passes
    pairs = float(Hq) * sum(min(i + 1, S) for i in range(S - n_s, S))
    stage_compute = {n: {"mfma_tflops": 2.0 * 128 * pairs / (stage_ms[n] * 1e-3) / 1e12,
                         "gexp_per_s": pairs / (stage_ms[n] * 1e-3) / 1e9}
                     for n in ("row_lse", "score_accum") if stage_ms.get(n)}

    # ---- in-library dense kernel on the same inputs --------------------------------
    dense_ms = None
    if args.dense_iters > 0:
        plan.dense(q, k, v)
        torch.cuda.synchronize()
        sa.sa_profile_enable(True)
        for _ in range(args.dense_iters):
            plan.dense(q, k, v)
        torch.cuda.synchronize()
        dk = sa.sa_profile_read("dense_flash")
        dt = sa.sa_profile_read("transpose_v")
        dense_ms = float(np.mean(dk)) + float(np.mean(dt))
        dense_kernel_tflops = dense_tiles * TILE_FLOP / (float(np.mean(dk)) * 1e-3) / 1e12
        log(f"dense kernel {np.mean(dk):.3f} ms (+{np.mean(dt):.3f} ms V^T) -> {dense_kernel_tflops:.1f} TFLOP/s")

    # Recall of a mask on row i = sum of the dense softmax over the kept keys
    # = exp(lse_masked_i - lse_dense_i); its minimum over rows is the CRA of the mask
    # (Sec. 3.3).  Both log-sum-exps are optional outputs of the attention kernels.
    dense_lse = None
    if dense_ms is not None and (not args.no_sweep or not args.no_block):
        plan.lse = torch.empty(Hq, S, dtype=torch.float32, device="cuda")
        plan.dense(q, k, v)
        torch.cuda.synchronize()
        dense_lse = plan.lse.clone()

    def recall_stats(lse_masked):
        if dense_lse is None:
            return {}
        r = torch.exp(lse_masked - dense_lse)
        return {"recall_mean": float(r.mean()), "cra_min": float(r.min())}

    # ---- alpha sweep (selection + attention only; stage 1 does not depend on alpha) --
    sweep = []
    if not args.no_sweep and len(wl.alphas) > 1:
        plan.sample(q, k)
        for a in wl.alphas:
            plan.select(a, a)
            plan.attend(q, k, v, w)          # warm
            torch.cuda.synchronize()
            sa.sa_profile_enable(True)
            plan.select(a, a)
            plan.attend(q, k, v, w)
            torch.cuda.synchronize()
            t_sel = float(np.mean(sa.sa_profile_read("select")))
            t_prep = float(np.mean(sa.sa_profile_read("mask_prep"))) + float(np.mean(sa.sa_profile_read("transpose_v")))
            t_fl = float(np.mean(sa.sa_profile_read("sparse_flash")))
            tl = plan.tiles.cpu().numpy().astype(np.int64)
            stage1 = sum(stage_ms[n] for n in ("row_lse", "score_accum", "score_final"))
            total = stage1 + t_sel + t_prep + t_fl
            cca, sca = plan.col_cnt.cpu().numpy(), plan.slash_cnt.cpu().numpy()
            d0 = mask_density(S, plan.col_idx[0, :int(cca[0])].cpu().numpy(),
                              plan.slash_idx[0, :int(sca[0])].cpu().numpy(), w)
            sweep.append({
                "alpha": a, "ms_layer": total, "sparse_flash_ms": t_fl,
                "computed_tile_fraction": float(tl.sum()) / dense_tiles,
                "mask_density_head0": d0,
                "mean_k_c": float(cca.mean()), "mean_k_s": float(sca.mean()),
                "speedup_vs_dense": (dense_ms / total) if dense_ms else None,
                "flash_tflops": float(tl.sum()) * TILE_FLOP / (t_fl * 1e-3) / 1e12,
                **(recall_stats(plan.lse) if plan.lse is not None else {}),
            })
            log(f"alpha {a}: {json.dumps(sweep[-1])}")

    # ---- the same workload at block granularity (Algorithm 1 with blk = 128): with the
    #      workload's sampled rows, and with the paper's 128 sampled rows -----------------
    block_runs = []
    if not args.no_block:
        blk = 128
        variants = [(bn_s, 1) for bn_s in sorted({n_s, min(128, S)}, reverse=True)]
        if S % 512 == 0 and S >= 1024:
            variants.append((128, 2))         # Algorithm 1 as printed: chunk_n = 2, 128 rows per chunk
        for bn_s, n_chunks in variants:
            bplan = sa.SampleAttentionPlan(shape, bn_s, granularity=blk, n_chunks=n_chunks)
            bplan.lse = plan.lse
            for a in wl.alphas:
                bplan.run(q, k, v, a, a, w)          # warm
                torch.cuda.synchronize()
                sa.sa_profile_enable(True)
                bplan.run(q, k, v, a, a, w)
                torch.cuda.synchronize()
                # a kernel runs once per chunk: the step's time is the sum of its launches
                t = {n: float(np.sum(sa.sa_profile_read(n))) for n in
                     ("row_lse", "score_accum", "score_final", "select", "transpose_v", "mask_prep", "sparse_flash")}
                tl = bplan.tiles.cpu().numpy().astype(np.int64)
                cca, sca = bplan.col_cnt.cpu().numpy(), bplan.slash_cnt.cpu().numpy()
                total = sum(t.values())
                # head 0, last chunk: the mask of the bottom segment of the queries
                c0 = bplan.col_idx.reshape(-1, *bplan.col_idx.shape[-2:])[-1, 0, :int(cca.reshape(n_chunks, -1)[-1, 0])]
                s0 = bplan.slash_idx.reshape(-1, *bplan.slash_idx.shape[-2:])[-1, 0, :int(sca.reshape(n_chunks, -1)[-1, 0])]
                block_runs.append({
                    "granularity": blk, "n_sample_rows": bn_s, "n_chunks": n_chunks, "alpha": a, "ms_layer": total,
                    "sparse_flash_ms": t["sparse_flash"],
                    "computed_tile_fraction": float(tl.sum()) / dense_tiles,
                    "block_mask_density_head0": block_mask_density(S, c0.cpu().numpy(), s0.cpu().numpy(), w, blk),
                    "mean_k_c_blocks": float(cca.mean()), "mean_k_s_blocks": float(sca.mean()),
                    "speedup_vs_dense": (dense_ms / total) if dense_ms else None,
                    "flash_tflops": float(tl.sum()) * TILE_FLOP / (t["sparse_flash"] * 1e-3) / 1e12,
                    **(recall_stats(bplan.lse) if bplan.lse is not None else {}),
                })
                log(f"block: {json.dumps(block_runs[-1])}")
            del bplan
    # ---- separate thresholds for columns and slashes (Sec. 4.1: alpha decomposed into alpha_c and
    #      alpha_s; Sec. 5.3 studies them) on heads of one pattern each: strong columns only,
    #      diagonals only, both.  Kept fraction, recall and CRA of the mask per (alpha_c, alpha_s).
    grid = []
    if not args.no_alpha_grid:
        from sa_inputs import HEAD_PATTERNS
        grid_alphas = (0.0, 0.8, 0.9, 0.95)
        for pname, pwl in HEAD_PATTERNS.items():
            pwl = pwl.scaled(S)
            if S // 2 - 2 * pwl.window < pwl.n_slash:
                continue
            t0 = time.perf_counter()
            px = make_inputs(pwl)
            pq, pk, pv = to_device(px["q"]), to_device(px["k"]), to_device(px["v"])
            del px
            log(f"head pattern {pname}: inputs in {time.perf_counter() - t0:.1f} s")
            plan.lse = torch.empty(Hq, S, dtype=torch.float32, device="cuda") if plan.lse is None else plan.lse
            plan.dense(pq, pk, pv)
            torch.cuda.synchronize()
            p_dense_lse = plan.lse.clone()
            plan.sample(pq, pk)
            for ac in grid_alphas:
                for as_ in grid_alphas:
                    plan.select(ac, as_)
                    plan.attend(pq, pk, pv, w)          # warm
                    torch.cuda.synchronize()
                    sa.sa_profile_enable(True)
                    plan.select(ac, as_)
                    plan.attend(pq, pk, pv, w)
                    torch.cuda.synchronize()
                    t_fl = float(np.mean(sa.sa_profile_read("sparse_flash")))
                    tl = plan.tiles.cpu().numpy().astype(np.int64)
                    cca, sca = plan.col_cnt.cpu().numpy(), plan.slash_cnt.cpu().numpy()
                    r = torch.exp(plan.lse - p_dense_lse)
                    grid.append({
                        "head_pattern": pname, "alpha_c": ac, "alpha_s": as_, "sparse_flash_ms": t_fl,
                        "computed_tile_fraction": float(tl.sum()) / dense_tiles,
                        "mask_density_head0": mask_density(S, plan.col_idx[0, :int(cca[0])].cpu().numpy(),
                                                           plan.slash_idx[0, :int(sca[0])].cpu().numpy(), w),
                        "mean_k_c": float(cca.mean()), "mean_k_s": float(sca.mean()),
                        "recall_mean": float(r.mean()), "cra_min": float(r.min()),
                    })
                    log(f"grid: {json.dumps(grid[-1])}")
            del pq, pk, pv, p_dense_lse
    sa.sa_profile_enable(False)

    # ---- the same step replayed from a HIP graph (launch overhead; matters at short lengths) ----
    graph_ms = None
    if not args.no_graph and not args.heads_per_pass:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            plan.run(q, k, v, args.alpha, args.alpha, w)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            plan.run(q, k, v, args.alpha, args.alpha, w)
        g.replay()
        torch.cuda.synchronize()
        gev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for e0, e1 in gev:
            e0.record()
            g.replay()
            e1.record()
        torch.cuda.synchronize()
        graph_ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in gev]))
        log(f"graph replay: {graph_ms:.3f} ms/step (eager {ms_median:.3f})")
        del g

    # ---- what this GPU reaches on a bare MFMA loop and on a plain copy ---------------------
    peaks = None
    if not args.no_peaks:
        sink = torch.zeros(1, dtype=torch.float32, device="cuda")
        peaks = {}
        for wps in (1, 2):
            sa.sa_probe_mfma(2000, wps, sink)            # warm
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            probe_flop = sa.sa_probe_mfma(20000, wps, sink)
            e1.record()
            torch.cuda.synchronize()
            peaks[f"mfma_bf16_tflops_{wps}_waves_per_simd"] = probe_flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        sa.sa_probe_copy(src, dst)
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            moved = sa.sa_probe_copy(src, dst)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, moved / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        peaks["copy_1gib_read_plus_write_gbs"] = best
        del src, dst
        log(f"measured peaks: {json.dumps(peaks)}")

    cpu = None
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        cpu = cpu_baseline(wl, x, args.alpha, args.cpu_seconds)
        log(f"cpu baseline took {time.perf_counter() - t0:.1f} s: {cpu['value']:.0f} ms/layer")

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl.name}_alpha{args.alpha:g}.json")
    if os.path.exists(tpath):
        # HBM bytes per launch of the strip-masked flash kernel, from the committed rocprofv3 --pmc
        # FETCH_SIZE / WRITE_SIZE runs of this same command (see the file for the calibration)
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")

    line = {
        "metric": "sparse prefill attention ms/layer",
        "value": ms_median,
        "unit": "ms/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: batch 1, {Hq} q heads / {Hkv} kv heads, d=128, S={S}, causal, bf16, "
                        f"{wl.n_sinks} sinks + {wl.n_slash} slash offsets per kv head, alpha={args.alpha}, "
                        f"sample rows={n_s}, window={w}",
            "alpha": args.alpha, "seq_len": S, "n_sample_rows": n_s, "window": w,
        },
        "roofline": {
            "kernel": "flash_kernel<strip-masked>", "bound": "mfma", "achieved": achieved,
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
            "traffic": traffic,
            "flop_per_launch": flop, "kernel_ms": flash_ms,
            "useful_tflops": useful_tflops,
        },
        "cpu_baseline": cpu,
        "timing": {"value": "median of per-step HIP-event durations on the launch stream",
                   "ms_per_step": "wall-clock mean over the same steps", "step_ms": step_ms},
        "stage_ms": stage_ms,
        "graph_replay_ms_per_step": graph_ms,
        "useful_tflops": useful_tflops,
        "schedule_slot_fraction": slots / dense_tiles,
        "idle_slot_share": 1.0 - float(tiles.sum()) / slots,
        "kept_pair_fraction": kept_pairs / (Hq * S * (S + 1) / 2.0),
        "workspace_bytes": ws_bytes,
        "plan_workspace_bytes": int(plan.ws.numel()),
        "heads_per_pass": args.heads_per_pass or Hq,
        "measured_peaks": peaks,
        "computed_tile_fraction": float(tiles.sum()) / dense_tiles,
        "mask_density_head0": density0,
        "touched_128x128_block_fraction_head0": blocks0,
        "stage_hbm_gbs_algorithmic": stage_gbs,
        "stage_compute": stage_compute,
        "mean_k_c": float(cc.mean()), "mean_k_s": float(sc.mean()),
        "dense_ms": dense_ms,
        "dense_kernel_tflops": dense_kernel_tflops if dense_ms else None,
        "speedup_vs_dense": (dense_ms / ms_median) if dense_ms else None,
        "alpha_sweep": sweep,
        "block_granularity_runs": block_runs,
        "alpha_c_alpha_s_grid": grid,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
