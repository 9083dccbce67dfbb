#!/usr/bin/env python3
"""Benchmark of the SpecVocab draft-step hot path on one MI355X.

Workload (N=1): the Llama-3-8B-shaped chain-drafting configuration -- d=4096, V=128256, bf16
output embedding, one hidden row per draft step, k=8192 Zipf(1.1)-biased sorted unique indices,
1000 distinct seeded (h, idx) steps.  One "step" = subset logits (gathered rows of U) -> subset
softmax -> top-10 draft tokens.  The K timed steps are replayed from one HIP graph (the paper
benchmarks under device graphs for the same reason: launch overhead would hide the kernel).

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel (the row gather) alone, algorithmic bytes / launch duration, on the timed
                workload (one U: what a drafter sees) and cold (U rotated over 8 copies: every row from HBM);
                `traffic` is read from the committed counter summary under profiles/
  stream_read   a plain 16-byte-per-lane read of a 4 GiB buffer in the same harness: the read bandwidth a kernel
                can reach on this machine; bandwidths are quoted against it as well as against the 8 TB/s peak
  cpu_baseline  the CPU oracle on a bounded sample of the same steps (one thread), and the same oracle run on
                all host cores at once, one step per thread
  dense         the full-vocabulary projection on the same GPU and the resulting speed-up
  cold          the same step with U rotated over 8 copies, so that no row can be served from the
                256 MB last-level cache (the one-U numbers are what a drafter really sees)
                also: the same kernel over one contiguous block of k rows, cold -- the ceiling of a burst
  select        the selector (W_down, W_vocab, top-k) at the same shape, the step with it, and the selector
                with W_vocab rotated over 6 copies (cold: no copy survives in the last-level cache)
  aux_log_softmax_us   log q_aux over the whole vocabulary (Section 3.4) at the same shape
  break_even    the paper's Section 6 / Table 4 comparison: full vocabulary, a static 32K vocabulary
                (gathered and pre-packed), SpecVocab with k = 2048 and 8192, whole steps
  other_configs tree rows (config 3; also with selection, at 8 and at 60 rows), the 262144-token head with a
                k sweep (config 4), 512 hidden rows with selection (config 5), each next to the dense projection
  indexed_lm_head_microbenchmark   fused gather against materialise-then-multiply at four model
                shapes, k from 512 to 32768 (the paper's kernel microbenchmark in kind)
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

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, published peak


def note(msg):
    """progress line on stderr, flushed before each GPU leg so that a failure names its leg"""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=1000)
    p.add_argument("--warmup", type=int, default=1000)
    p.add_argument("--distinct", type=int, default=1000, help="distinct (h, idx) steps to draw")
    p.add_argument("--cold-copies", type=int, default=8)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-extras", action="store_true", help="skip dense / cold / select legs")
    p.add_argument("--cpu-seconds", type=float, default=12.0)
    p.add_argument("--counter-run", nargs="?", const="warm", choices=("warm", "cold"), default=None,
                   help="for rocprofv3 --pmc: 1 GiB reference copies, then a few eager (ungraphed) steps on one U "
                        "(warm) or on 8 rotating copies of U (cold); no timing, no JSON line")
    p.add_argument("--trace-config", type=int, choices=(3, 4, 5, 30), default=None,
                   help="for rocprofv3 --kernel-trace: a few eager passes of that configuration (its draft step and "
                        "the dense projection; config 5 also the selection; 30 = the tree of config 3 with sets that "
                        "overlap more, draft steps only), no timing, no JSON line")
    return p.parse_args()


def config5_setup(sv, torch, np, dev):
    """Config 5 (512 hidden rows, selector d' = 256, k = 8192, top-10) resident on the device; returns the
    config and closures for its three stages plus the buffer the selection writes."""
    from workloads import CONFIGS

    def dev_bf16(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    c = CONFIGS[5]
    U = dev_bf16(c.weights())
    Wd_np, Wv_np = c.selector()
    Wd, Wv = dev_bf16(Wd_np), dev_bf16(Wv_np)
    h = dev_bf16(c.hidden(1)[0])
    ws = torch.empty(sv.workspace_bytes(sv.SV_OP_SELECT, c.rows, c.d, c.V, c.k, c.d_prime, 0, sv.SV_BF16),
                     dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(1, sv.workspace_bytes(sv.SV_OP_DRAFT_STEP, c.rows, c.d, c.V, c.k, 0, c.kd, sv.SV_BF16,
                                                sv.SV_IDX_PER_ROW | sv.SV_IDX_SORTED)),
                      dtype=torch.uint8, device=dev)
    sel = torch.empty((c.rows, c.k), dtype=torch.int32, device=dev)
    z = torch.empty((c.rows, c.k), dtype=torch.float32, device=dev)
    tok = torch.empty((c.rows, c.kd), dtype=torch.int32, device=dev)
    prob = torch.empty((c.rows, c.kd), dtype=torch.float32, device=dev)
    zd = torch.empty((c.rows, c.V), dtype=torch.float32, device=dev)
    run_select = lambda: sv.select(h, Wd, Wv, c.k, idx_out=sel, ws=ws)
    # the selection emits ascending ids, and says so
    run_step = lambda: sv.draft_step(h, U, sel, c.kd, logits_out=z, tok_out=tok, prob_out=prob, ws=ws2,
                                     sorted_lists=True)
    run_dense = lambda: sv.dense_logits(h, U, out=zd)
    run_select()                                   # sel holds valid ids before anything gathers with it
    torch.cuda.synchronize()
    run_step.buffers = (h, U, z, tok, prob)
    return c, run_select, run_step, run_dense, sel


def config5_any_order(sv, torch, dev, c, sel, run_step_args):
    """The same step on the same sets with every list shuffled and nothing declared about its order."""
    h, U, z, tok, prob = run_step_args
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    shuffled = torch.stack([sel[r][torch.randperm(c.k, generator=g, device=dev)] for r in range(c.rows)]).contiguous()
    ws3 = torch.empty(max(1, sv.workspace_bytes(sv.SV_OP_DRAFT_STEP, c.rows, c.d, c.V, c.k, 0, c.kd, sv.SV_BF16,
                                                sv.SV_IDX_PER_ROW)), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    return lambda: sv.draft_step(h, U, shuffled, c.kd, logits_out=z, tok_out=tok, prob_out=prob, ws=ws3)


def other_configs(sv, torch, np, dev, capture, timed_replays):
    """The remaining configurations (tree rows, large vocabulary, full step with selection): median
    microseconds per step from graph replays, next to the dense projection at the same row count."""
    from workloads import CONFIGS, make_rng, zipf_subset

    def dev_bf16(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    def med_us(fn, n, reps=5):
        g = capture(fn, n)
        timed_replays(g, 1)
        r = sorted(timed_replays(g, reps))
        return r[len(r) // 2] * 1e3 / n

    out = {}
    # ---- config 3: 60 tree rows, own k=4096 subset each (half shared), top-10
    note("config 3: tree of 60 rows")
    c = CONFIGS[3]
    U = dev_bf16(CONFIGS[2].weights())
    nst = 4
    h = dev_bf16(c.hidden(nst).reshape(nst * c.rows, c.d)).reshape(nst, c.rows, c.d)
    idx = torch.from_numpy(c.indices(nst)).to(dev)
    z = torch.empty((c.rows, c.k), dtype=torch.float32, device=dev)
    tok = torch.empty((c.rows, c.kd), dtype=torch.int32, device=dev)
    prob = torch.empty((c.rows, c.kd), dtype=torch.float32, device=dev)
    zd = torch.empty((c.rows, c.V), dtype=torch.float32, device=dev)
    step_us = med_us(lambda t: sv.draft_step(h[t % nst], U, idx[t % nst], c.kd, logits_out=z, tok_out=tok,
                                             prob_out=prob), 20)
    dense_us = med_us(lambda t: sv.dense_logits(h[t % nst], U, out=zd), 10)
    uniq = float(np.mean([np.unique(idx[t].cpu().numpy()).size for t in range(nst)]))
    out["config3_tree60"] = {"rows": c.rows, "k": c.k, "step_us": round(step_us, 1), "dense_us": round(dense_us, 1),
                             "speedup_vs_dense": round(dense_us / step_us, 2),
                             "unique_rows_per_step": round(uniq), "unique_row_MB": round(uniq * c.d * 2 / 1e6, 1),
                             "dense_frac_hbm_peak": round(c.V * c.d * 2 / (dense_us * 1e-6) / 8e12, 3)}
    # the same tree with sets that overlap more (slices of the lists above: their shared part comes first), so that
    # the union is a few thousand rows -- its size is known on the device only, which picks the kernel there
    over = []
    for lo, kk in ((0, 1024), (1500, 1024), (1500, 2048)):
        idx_o = idx[:, :, lo:lo + kk].contiguous()
        z_o = torch.empty((c.rows, kk), dtype=torch.float32, device=dev)
        us = med_us(lambda t: sv.draft_step(h[t % nst], U, idx_o[t % nst], c.kd, logits_out=z_o, tok_out=tok,
                                            prob_out=prob), 20)
        uq = float(np.mean([np.unique(idx_o[t].cpu().numpy()).size for t in range(nst)]))
        over.append({"k": kk, "unique_rows_per_step": round(uq), "step_us": round(us, 1)})
    out["config3_tree60"]["sets_that_overlap_more"] = over
    # the same shape with selection, at the width of one level of a small draft tree (8 rows) and at 60:
    # the selector has random weights, so its sets are timed, and the draft step runs on config 3's recipe
    from workloads import tree_subsets
    c2 = CONFIGS[2]
    Wd_np, Wv_np = c2.selector()
    Wd, Wv = dev_bf16(Wd_np), dev_bf16(Wv_np)
    for rows in (8, c.rows):
        rng = make_rng(c.number, 100 + rows)
        idx_r = torch.from_numpy(np.stack([tree_subsets(rng, c.V, rows, c.k, c.k // 2)[0] for _ in range(nst)])).to(dev)
        h_r = h[:, :rows].contiguous()
        sel = torch.empty((rows, c.k), dtype=torch.int32, device=dev)
        ws_s = torch.empty(sv.workspace_bytes(sv.SV_OP_SELECT, rows, c.d, c.V, c.k, c2.d_prime, 0, sv.SV_BF16),
                           dtype=torch.uint8, device=dev)
        nb = sv.workspace_bytes(sv.SV_OP_DRAFT_STEP, rows, c.d, c.V, c.k, 0, c.kd, sv.SV_BF16)
        ws_g = torch.empty(max(nb, 16), dtype=torch.uint8, device=dev)
        zr = torch.empty((rows, c.k), dtype=torch.float32, device=dev)

        def level(t):
            sv.select(h_r[t % nst], Wd, Wv, c.k, idx_out=sel, ws=ws_s)
            sv.draft_step(h_r[t % nst], U, idx_r[t % nst], c.kd, logits_out=zr, tok_out=tok[:rows],
                          prob_out=prob[:rows], ws=ws_g)
        sel_us = med_us(lambda t: sv.select(h_r[t % nst], Wd, Wv, c.k, idx_out=sel, ws=ws_s), 20)
        lvl_us = med_us(level, 20)
        dn_us = med_us(lambda t: sv.dense_logits(h_r[t % nst], U, out=zd[:rows]), 10)
        out["config3_tree60"][f"with_selection_{rows}_rows"] = {
            "select_us": round(sel_us, 1), "select_plus_step_us": round(lvl_us, 1), "dense_us": round(dn_us, 1),
            "speedup_vs_dense": round(dn_us / lvl_us, 2)}
        del idx_r, h_r, sel, ws_s, ws_g, zr
    del U, h, idx, z, zd, Wd, Wv
    torch.cuda.empty_cache()

    # ---- config 4: V=262144, d=3840, 8 rows, k sweep, one set per step and one set per row
    note("config 4: 262144-token head, 8 rows, k sweep")
    c = CONFIGS[4]
    U = dev_bf16(c.weights())
    h = dev_bf16(c.hidden(nst).reshape(nst * c.rows, c.d)).reshape(nst, c.rows, c.d)
    zd = torch.empty((c.rows, c.V), dtype=torch.float32, device=dev)
    dense_us = med_us(lambda t: sv.dense_logits(h[t % nst], U, out=zd), 10)
    del zd
    rng = make_rng(4, 2)
    sweep = {}
    for k in c.k_sweep:
        shared = torch.from_numpy(np.stack([zipf_subset(rng, c.V, k) for _ in range(nst)])).to(dev)
        per_row = torch.from_numpy(np.stack([np.stack([zipf_subset(rng, c.V, k) for _ in range(c.rows)])
                                             for _ in range(nst)])).to(dev)
        z = torch.empty((c.rows, k), dtype=torch.float32, device=dev)
        tok = torch.empty((c.rows, c.kd), dtype=torch.int32, device=dev)
        prob = torch.empty((c.rows, c.kd), dtype=torch.float32, device=dev)
        sh_us = med_us(lambda t: sv.draft_step(h[t % nst], U, shared[t % nst], c.kd, logits_out=z, tok_out=tok,
                                               prob_out=prob), 20)
        pr_us = med_us(lambda t: sv.draft_step(h[t % nst], U, per_row[t % nst], c.kd, logits_out=z, tok_out=tok,
                                               prob_out=prob), 20)
        sweep[str(k)] = {"shared_set_step_us": round(sh_us, 1), "per_row_sets_step_us": round(pr_us, 1),
                         "speedup_vs_dense_shared": round(dense_us / sh_us, 2),
                         "speedup_vs_dense_per_row": round(dense_us / pr_us, 2)}
    out["config4_gemma262k"] = {"rows": c.rows, "dense_us": round(dense_us, 1),
                                "dense_frac_hbm_peak": round(c.V * c.d * 2 / (dense_us * 1e-6) / 8e12, 3),
                                "k": sweep}
    del U, h
    torch.cuda.empty_cache()

    # ---- config 5: 512 rows, selector d'=256, k=8192, top-10: select -> logits -> softmax/top-10
    note("config 5: 512 rows with selection")
    c, run_select, run_step, run_dense, sel = config5_setup(sv, torch, np, dev)
    # (long matrix-core kernels: the clock settles over the first replays, so the three are timed in turns and
    # the median of seven rounds is taken)
    graphs = [capture(lambda t: run_select(), 3), capture(lambda t: run_step(), 3), capture(lambda t: run_dense(), 3),
              capture(lambda t, f=config5_any_order(sv, torch, dev, c, sel, run_step.buffers): f(), 3)]
    # the selection on its own first (its kernels are short: between two long matrix-core passes they run at the
    # lower clock those leave behind, 10-15 % slower; both figures are reported, the sum uses the one in turn)
    alone = sorted(timed_replays(graphs[0], 1)[0] * 1e3 / 3 for _ in range(10))
    sel_alone_us = alone[len(alone) // 2]
    rounds = [[timed_replays(g, 1)[0] * 1e3 / 3 for g in graphs] for _ in range(8)][1:]
    sel_us, step_us, dense_us, any_us = (sorted(r[i] for r in rounds)[len(rounds) // 2] for i in range(4))
    del graphs
    flops = 2.0 * c.rows * c.V * c.d
    out["config5_qwen3_select"] = {"rows": c.rows, "k": c.k, "d_prime": c.d_prime, "select_us": round(sel_alone_us, 1),
                                   "select_us_between_matrix_core_passes": round(sel_us, 1),
                                   "logits_softmax_topk_us": round(step_us, 1),
                                   "logits_softmax_topk_us_lists_shuffled_order_not_declared": round(any_us, 1),
                                   "end_to_end_us": round(sel_us + step_us, 1), "dense_us": round(dense_us, 1),
                                   "dense_tflops": round(flops / dense_us / 1e6, 1),
                                   "dense_frac_mfma_peak": round(flops / (dense_us * 1e-6) / 2.5e15, 3),
                                   "union_of_selected_sets": int(torch.unique(sel).numel()),
                                   "note": "random-init selector: the 512 selected sets are unrelated, their union "
                                           "is (nearly) the whole vocabulary, so the subset logits cost a dense pass"}
    return out


def trace_config(number, sv, torch, np, dev):
    """A few eager passes of one of the other configurations, for a kernel trace."""
    from workloads import CONFIGS, make_rng, zipf_subset

    def dev_bf16(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    if number == 5:
        _, run_select, run_step, run_dense, _ = config5_setup(sv, torch, np, dev)
        for _ in range(3):
            run_select()
            run_step()
            run_dense()
        torch.cuda.synchronize()
        print("config 5 trace run done: 3 x (select, draft step, dense)", flush=True)
        return
    if number == 30:
        c = CONFIGS[3]
        U = dev_bf16(CONFIGS[2].weights())
        h = dev_bf16(c.hidden(1)[0])
        idx = torch.from_numpy(c.indices(1)[0]).to(dev)
        for lo, kk in ((0, 1024), (1500, 1024), (1500, 2048)):        # the slices `sets_that_overlap_more` times
            idx_o = idx[:, lo:lo + kk].contiguous()
            for _ in range(5):
                sv.draft_step(h, U, idx_o, c.kd)
            torch.cuda.synchronize()
            print(f"k={kk}: union of {int(torch.unique(idx_o).numel())} rows", flush=True)
        print("config 3 with sets that overlap more, trace run done: per slice 5 x draft step", flush=True)
        return
    if number == 3:
        c = CONFIGS[3]
        U = dev_bf16(CONFIGS[2].weights())
        h = dev_bf16(c.hidden(1)[0])
        idx = torch.from_numpy(c.indices(1)[0]).to(dev)
        zd = torch.empty((c.rows, c.V), dtype=torch.float32, device=dev)
        for _ in range(5):
            sv.draft_step(h, U, idx, c.kd)
            sv.dense_logits(h, U, out=zd)
        torch.cuda.synchronize()
        print("config 3 trace run done: 5 x (draft step over 60 per-row sets, dense)", flush=True)
        return
    c = CONFIGS[4]
    U = dev_bf16(c.weights())
    h = dev_bf16(c.hidden(1)[0])
    rng = make_rng(4, 2)
    zd = torch.empty((c.rows, c.V), dtype=torch.float32, device=dev)
    for k in c.k_sweep:
        shared = torch.from_numpy(zipf_subset(rng, c.V, k)).to(dev)
        per_row = torch.from_numpy(np.stack([zipf_subset(rng, c.V, k) for _ in range(c.rows)])).to(dev)
        for _ in range(5):
            sv.draft_step(h, U, shared, c.kd)
        torch.cuda.synchronize()
        for _ in range(5):
            sv.draft_step(h, U, per_row, c.kd)
        torch.cuda.synchronize()
    for _ in range(3):
        sv.dense_logits(h, U, out=zd)
    torch.cuda.synchronize()
    print("config 4 trace run done: per k in (2048, 8192, 32768): 5 x shared-set step, 5 x per-row-sets step; "
          "3 x dense", flush=True)


def counter_summary_traffic():
    """HBM-side bytes per launch of the row gather from the committed rocprofv3 counter summary
    (profiles/gather_gemv_config2_hbm_traffic.md: its lines '* fetched: ... = X MB per launch' and
    '* written: ... = Y MB per launch'); None if the file is missing or does not hold both."""
    import re
    path = os.path.join(ROOT, "profiles", "gather_gemv_config2_hbm_traffic.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    got = {}
    for key in ("fetched", "written"):
        m = re.search(r"^\* " + key + r":.*= ([0-9.]+) MB per launch", text, flags=re.M)
        if not m:
            return None
        got[key] = float(m.group(1)) * 1e6
    return got["fetched"] + got["written"]


def indexed_head_microbenchmark(sv, torch, dev, capture, timed_replays):
    """The paper's kernel microbenchmark in kind (Section 6, the paragraph on the kernel's speed-up): synthetic
    activations and weights at model dimensions, one hidden row, graph replay; the fused row gather
    against the indexed LM head done the naive way of Figure 3a (materialise U[idx] in memory, then a
    matrix-vector product over the copy), both from this library.  Dimensions are those of public
    model cards; values are seeded random (drawn on the device: only the timing matters here)."""
    shapes = {"qwen3-8b": (4096, 151936), "qwen3-4b": (2560, 151936),
              "olmo2-7b": (4096, 100352), "olmo2-1b": (2048, 100352)}
    gen = torch.Generator(device=dev)
    gen.manual_seed(13836)
    out = {}
    for name, (d, V) in shapes.items():
        note(f"indexed LM head microbenchmark: {name}")
        U = (torch.randn((V, d), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
        h = torch.randn((8, 1, d), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        per_k = {}
        # the paper's k axis (its Figure 4 sweeps k up to 32768) in full for the first shape
        for k in ((512, 1024, 2048, 4096, 8192, 16384, 32768) if name == "qwen3-8b" else (512, 2048, 8192)):
            idx = torch.stack([torch.randperm(V, generator=gen, device=dev)[:k].sort().values
                               for _ in range(8)]).to(torch.int32).reshape(8, 1, k).contiguous()
            z = torch.empty((1, k), dtype=torch.float32, device=dev)
            ws = torch.empty(sv.workspace_bytes(sv.SV_OP_INDEXED_HEAD_NAIVE, 1, d, V, k, 0, 0, sv.SV_BF16),
                             dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            g1 = capture(lambda t: sv.subset_logits(h[t % 8], U, idx[t % 8], out=z), 200)
            timed_replays(g1, 1)
            ours = sorted(timed_replays(g1, 5))[2] * 1e3 / 200
            g2 = capture(lambda t: sv.indexed_head_naive(h[t % 8], U, idx[t % 8], out=z, ws=ws), 200)
            timed_replays(g2, 1)
            ref = sorted(timed_replays(g2, 5))[2] * 1e3 / 200
            per_k[str(k)] = {"fused_gather_us": round(ours, 2), "materialise_then_matvec_us": round(ref, 2),
                             "speedup": round(ref / ours, 2),
                             "fused_gather_frac_hbm_peak": round(k * d * 2 / (ours * 1e-6) / 8e12, 3)}
            del g1, g2, ws
        out[name] = {"d": d, "V": V, "k": per_k}
        del U
        torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2602_13836_amd as sv
    from workloads import CONFIGS

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sv.load_library()                       # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    c = CONFIGS[2]
    K, W = int(args.steps), int(args.warmup)
    nd = max(1, min(int(args.distinct), c.steps))
    es = c.esize()

    def dev_bf16(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    t0 = time.time()
    U_np = c.weights()
    h_np = c.hidden(nd)                     # [nd, 1, d]
    idx_np = c.indices(nd)                  # [nd, 1, k]
    U = dev_bf16(U_np)
    h = dev_bf16(h_np.reshape(nd * c.rows, c.d)).reshape(nd, c.rows, c.d)
    idx = torch.from_numpy(idx_np).to(dev)
    z = torch.empty((nd, c.rows, c.k), dtype=torch.float32, device=dev)
    tok = torch.empty((nd, c.rows, c.kd), dtype=torch.int32, device=dev)
    prob = torch.empty((nd, c.rows, c.kd), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    t_setup = time.time() - t0

    stream = torch.cuda.Stream()            # default priority

    def step(t, U_t=U):
        """one draft step: gathered logits + subset softmax + top-kd (specvocab_draft_step)"""
        i = t % nd
        sv.draft_step(h[i], U_t, idx[i], c.kd, logits_out=z[i], tok_out=tok[i], prob_out=prob[i])


    def capture(fn, n):
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()            # inputs are made on the default stream; the calls below run on another
        with torch.cuda.stream(stream):
            fn(0)                           # eager once: loads code objects before capture
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=stream):
                for t in range(n):
                    fn(t)
        torch.cuda.synchronize()
        return g

    def timed_replays(g, reps):
        """ms per replay, HIP events on the replay stream."""
        out = []
        with torch.cuda.stream(stream):
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                g.replay()
                e1.record(stream)
                e1.synchronize()
                out.append(e0.elapsed_time(e1))
        return out

    if args.trace_config is not None:
        trace_config(args.trace_config, sv, torch, np, dev)
        return

    if args.counter_run:
        # hardware counters are read per dispatch; a plain copy of known size calibrates them
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(3):
            dst.copy_(src)
        del src, dst
        ncopy = max(1, int(args.cold_copies)) if args.counter_run == "cold" else 1
        copies = [U] + [U.clone() for _ in range(ncopy - 1)]
        for t in range(min(K, 40)):
            step(t, copies[t % ncopy])
        torch.cuda.synchronize()
        print(f"counter run done ({args.counter_run}): 3 x 1 GiB copies, then eager steps over {ncopy} "
              f"cop{'y' if ncopy == 1 else 'ies'} of U", flush=True)
        return

    # ---------------- the timed region: exactly K steps, one graph replay
    note(f"config 2: capturing {K} draft steps")
    g_step = capture(step, K)
    with torch.cuda.stream(stream):
        for _ in range((W + K - 1) // K if W > 0 else 0):
            g_step.replay()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    with torch.cuda.stream(stream):
        g_step.replay()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t1) * 1e3
    rep = sorted(timed_replays(g_step, 10))
    us_per_step = wall_ms * 1e3 / K
    us_per_step_median = rep[len(rep) // 2] * 1e3 / K

    # ---------------- roofline of the dominant kernel: the row gather (specvocab_subset_logits)
    # algorithmic bytes of one launch: the k gathered rows of U + idx + h + the logits written
    gather_bytes = c.k * c.d * es + c.k * 4 + c.d * es + c.k * 4
    # The kernel-only legs replay graphs of KG >= 200 launches whatever K is: a replay of 20 launches is a quarter
    # of a millisecond of work between two host synchronisations, and the launches right after such a pause run
    # slower (cold legs most: 12.0 against 11.75 us per launch) -- an artefact of the replay length, not of the
    # kernel.  The cold leg is reported in graphs of K launches as well.
    KG = max(K, 200)
    note("config 2: row gather alone")
    g_gather = capture(lambda t: sv.subset_logits(h[t % nd], U, idx[t % nd], out=z[t % nd]), KG)
    timed_replays(g_gather, 2)
    gr = sorted(timed_replays(g_gather, 10))
    gather_us = gr[len(gr) // 2] * 1e3 / KG
    gather_gbps = gather_bytes / (gather_us * 1e-6) / 1e9
    # ---------------- the same gather cold: U rotated over several copies, so that no row can come from the
    # 256 MB last-level cache (on one U successive Zipf-biased sets share a third of their rows)
    note("config 2: row gather alone, cold (rotating copies of U)")
    ncopy = max(1, int(args.cold_copies))
    copies = [U] + [U.clone() for _ in range(ncopy - 1)]
    g_coldg = capture(lambda t: sv.subset_logits(h[t % nd], copies[t % ncopy], idx[t % nd], out=z[t % nd]), KG)
    timed_replays(g_coldg, 2)
    cgr = sorted(timed_replays(g_coldg, 10))
    coldg_us = cgr[len(cgr) // 2] * 1e3 / KG
    coldg_gbps = gather_bytes / (coldg_us * 1e-6) / 1e9
    del g_coldg
    if KG != K:
        g_coldk = capture(lambda t: sv.subset_logits(h[t % nd], copies[t % ncopy], idx[t % nd], out=z[t % nd]), K)
        timed_replays(g_coldk, 2)
        ckr = sorted(timed_replays(g_coldk, 10))
        coldk_us = ckr[len(ckr) // 2] * 1e3 / K
        del g_coldk
    else:
        coldk_us = coldg_us

    # ---------------- what a plain read reaches here: 16 bytes per lane over a buffer far larger than the caches
    note("streaming-read peak (4 GiB buffer)")
    big = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    big.fill_(3)
    ws_probe = torch.empty(262144, dtype=torch.uint8, device=dev)
    nprobe = 10
    g_probe = capture(lambda t: sv.stream_read_probe(big, ws_probe), nprobe)
    timed_replays(g_probe, 2)
    pr = sorted(timed_replays(g_probe, 5))
    stream_gbps = big.numel() / (pr[len(pr) // 2] * 1e-3 / nprobe) / 1e9
    del g_probe, big
    torch.cuda.empty_cache()

    # HBM-side bytes per launch: rocprofv3 FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a
    # 1 GiB plain copy, from the committed summary of `bench.py --counter-run` (None if that file is missing)
    roofline = {"bound": "hbm",
                "kernel": "gemv_rows_once_kernel<bf16, 8 loads/lane, 1 row/wave, 8 waves/workgroup>: row gather of 8192 rows of U "
                          "(specvocab_subset_logits), 1 of the 2 launches of a step",
                "achieved": round(gather_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(gather_gbps / HBM_PEAK_GBPS, 4), "traffic": counter_summary_traffic(),
                "bytes_per_launch": gather_bytes, "us_per_launch": round(gather_us, 3),
                "protocol": "frac: the timed workload (one U, Zipf-biased sets that share a third of their rows from "
                            "step to step, so part of it comes from the last-level cache); cold_frac: U rotated over "
                            f"{ncopy} copies, every row from HBM -- the figure the >= 70 % target is judged on; both "
                            f"from graphs of {KG} launches (HIP events around a replay, gaps between launches included); "
                            "cold_*_in_graphs_of_K: the same in graphs of K launches, where the launches after each "
                            "host synchronisation weigh more",
                "launches_per_graph": KG,
                "cold_us_per_launch": round(coldg_us, 3), "cold_achieved": round(coldg_gbps, 1),
                "cold_frac": round(coldg_gbps / HBM_PEAK_GBPS, 4),
                "cold_us_per_launch_in_graphs_of_K": round(coldk_us, 3),
                "cold_frac_in_graphs_of_K": round(gather_bytes / (coldk_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                "stream_read_peak_GBps": round(stream_gbps, 1),
                "frac_of_stream_read_peak": round(gather_gbps / stream_gbps, 4),
                "cold_frac_of_stream_read_peak": round(coldg_gbps / stream_gbps, 4)}

    result = {
        "metric": "subset-logits us/draft-step",
        "value": round(us_per_step, 3),
        "unit": "us/draft-step",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(wall_ms / K, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config 2, Llama-3-8B-shaped chain drafting: d=4096 V=128256 bf16 U, rows=1, "
                               "k=8192 Zipf(1.1) sorted unique idx, kd=10; step = subset logits + softmax + top-10",
                   "distinct_steps": nd, "graph_replay": True, "d": c.d, "V": c.V, "k": c.k, "kd": c.kd,
                   "rows": c.rows},
        "us_per_step_median_of_10_replays": round(us_per_step_median, 3),
        "achieved_GBps_whole_step": round(gather_bytes / (us_per_step * 1e-6) / 1e9, 1),
        "pct_hbm_peak_whole_step": round(100 * gather_bytes / (us_per_step * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
        "roofline": roofline,
        "setup_s": round(t_setup, 1),
    }

    if not args.no_extras:
        # ---------------- dense full-vocabulary baseline on the same GPU
        note("config 2: dense baseline")
        nden = 50
        zd = torch.empty((c.rows, c.V), dtype=torch.float32, device=dev)
        g_dense = capture(lambda t: sv.dense_logits(h[t % nd], U, out=zd), nden)
        timed_replays(g_dense, 2)
        dr = sorted(timed_replays(g_dense, 5))
        dense_us = dr[len(dr) // 2] * 1e3 / nden
        dense_bytes = c.V * c.d * es + c.V * 4 + c.d * es
        result["dense"] = {"us_per_step": round(dense_us, 2),
                           "GBps": round(dense_bytes / (dense_us * 1e-6) / 1e9, 1),
                           "frac_hbm_peak": round(dense_bytes / (dense_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                           "frac_of_stream_read_peak": round(dense_bytes / (dense_us * 1e-6) / 1e9 / stream_gbps, 4),
                           "speedup_subset_logits_kernel": round(dense_us / gather_us, 2),
                           "speedup_whole_step": round(dense_us / us_per_step, 2)}
        del g_dense, zd

        # ---------------- cold: the whole step on rotating copies of U, and the kernel's ceiling for such a burst
        note("config 2: cold (rotating copies of U)")
        g_cold = capture(lambda t: step(t, copies[t % ncopy]), K)
        timed_replays(g_cold, 1)
        cr = sorted(timed_replays(g_cold, 5))
        cold_us = cr[len(cr) // 2] * 1e3 / K
        # the same number of bytes as ONE contiguous block of k rows (no index list, the same kernel), cold:
        # what a burst of this size can reach on this machine at all
        nwin = c.V // c.k
        zc = torch.empty((c.rows, c.k), dtype=torch.float32, device=dev)
        g_coldc = capture(lambda t: sv.dense_logits(
            h[t % nd], copies[t % ncopy][((t // ncopy) % nwin) * c.k:((t // ncopy) % nwin + 1) * c.k], out=zc), KG)
        timed_replays(g_coldc, 1)
        ccr = sorted(timed_replays(g_coldc, 5))
        coldc_us = ccr[len(ccr) // 2] * 1e3 / KG
        result["cold"] = {"copies_of_U": ncopy, "us_per_step": round(cold_us, 3),
                          "gather_kernel_us": round(coldg_us, 3),
                          "gather_GBps": round(coldg_gbps, 1),
                          "gather_frac_hbm_peak": round(coldg_gbps / HBM_PEAK_GBPS, 4),
                          "contiguous_block_of_k_rows_us": round(coldc_us, 3),
                          "note": "contiguous_block_of_k_rows_us: the same kernel streaming k consecutive rows "
                                  "(no index list), also cold -- the ceiling for a burst of this size"}
        del g_cold, g_coldc
        # ---------------- one U, but sets that share next to nothing from step to step: uniform draws instead of
        # Zipf-biased ones (cold without the eight-fold address range of the rotating copies)
        note("config 2: uniform index sets on one U")
        gen_u = torch.Generator(device=dev)
        gen_u.manual_seed(13836002)
        nu = min(nd, 64)
        idx_u = torch.stack([torch.randperm(c.V, generator=gen_u, device=dev)[:c.k].sort().values
                             for _ in range(nu)]).to(torch.int32).reshape(nu, 1, c.k).contiguous()
        g_uni = capture(lambda t: sv.subset_logits(h[t % nd], U, idx_u[t % nu], out=z[t % nd]), KG)
        timed_replays(g_uni, 2)
        ur = sorted(timed_replays(g_uni, 5))
        uni_us = ur[len(ur) // 2] * 1e3 / KG
        result["cold"]["uniform_sets_one_U_gather_us"] = round(uni_us, 3)
        result["cold"]["uniform_sets_one_U_frac_hbm_peak"] = round(gather_bytes / (uni_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)
        del g_uni, idx_u
        # ---------------- frequent tokens scattered over the vocabulary instead of sitting at the low ids: the same
        # Zipf-biased rank sets mapped through a seeded random permutation of the ids
        note("config 2: Zipf-biased sets with a random rank -> id map")
        perm = torch.from_numpy(np.random.Generator(np.random.PCG64(13836000 + 100 * 2 + 9)).permutation(c.V)
                                .astype(np.int64)).to(dev)
        ns = min(nd, 64)
        idx_s = perm[idx[:ns].long()].sort(dim=-1).values.to(torch.int32).contiguous()
        g_sc = capture(lambda t: sv.subset_logits(h[t % nd], U, idx_s[t % ns], out=z[t % nd]), KG)
        timed_replays(g_sc, 2)
        sr_ = sorted(timed_replays(g_sc, 5))
        sc_us = sr_[len(sr_) // 2] * 1e3 / KG
        result["scattered_rank_to_id"] = {"gather_kernel_us": round(sc_us, 3),
                                          "frac_hbm_peak": round(gather_bytes / (sc_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                                          "distinct_sets": ns,
                                          "note": "identity map (frequent tokens at the low ids) is roofline.us_per_launch"}
        del g_sc, idx_s, perm
        torch.cuda.empty_cache()

        # ---------------- the selector at the same shape, and the whole step including it
        note("config 2: selector")
        Wd_np, Wv_np = c.selector()
        Wd, Wv = dev_bf16(Wd_np), dev_bf16(Wv_np)
        ws = torch.empty(sv.workspace_bytes(sv.SV_OP_SELECT, c.rows, c.d, c.V, c.k, c.d_prime, 0, sv.SV_BF16),
                         dtype=torch.uint8, device=dev)
        sel = torch.empty((c.rows, c.k), dtype=torch.int32, device=dev)
        nsel = 200
        g_sel = capture(lambda t: sv.select(h[t % nd], Wd, Wv, c.k, idx_out=sel, ws=ws), nsel)
        timed_replays(g_sel, 2)
        sr = sorted(timed_replays(g_sel, 5))
        sel_us = sr[len(sr) // 2] * 1e3 / nsel

        def full(t):
            i = t % nd
            sv.select(h[i], Wd, Wv, c.k, idx_out=sel, ws=ws)
            sv.subset_logits(h[i], U, sel, out=z[i])
            sv.draft_topk(z[i], sel, c.kd, tok_out=tok[i], prob_out=prob[i])
        g_full = capture(full, nsel)
        timed_replays(g_full, 2)
        fr = sorted(timed_replays(g_full, 5))
        full_us = fr[len(fr) // 2] * 1e3 / nsel
        result["select"] = {"d_prime": c.d_prime, "select_us": round(sel_us, 2),
                            "step_with_select_us": round(full_us, 2),
                            "speedup_vs_dense": round(result["dense"]["us_per_step"] / full_us, 2)}
        del g_sel, g_full
        # the same with W_vocab coming from HBM: consecutive steps read different copies of it (together
        # larger than the 256 MB last-level cache), as after a target-model pass has swept the caches
        nwv = 6
        Wv_copies = [Wv] + [Wv.clone() for _ in range(nwv - 1)]
        g_selc = capture(lambda t: sv.select(h[t % nd], Wd, Wv_copies[t % nwv], c.k, idx_out=sel, ws=ws), nsel)
        timed_replays(g_selc, 2)
        result["select"]["select_us_cold_W_vocab"] = round(sorted(timed_replays(g_selc, 5))[2] * 1e3 / nsel, 2)
        del g_selc, Wv_copies
        # the wider selector the paper also studies (d'/d = 1/8)
        Wd8_np, Wv8_np = c.selector(c.d // 8)
        Wd8, Wv8 = dev_bf16(Wd8_np), dev_bf16(Wv8_np)
        ws8 = torch.empty(sv.workspace_bytes(sv.SV_OP_SELECT, c.rows, c.d, c.V, c.k, c.d // 8, 0, sv.SV_BF16),
                          dtype=torch.uint8, device=dev)
        g_sel8 = capture(lambda t: sv.select(h[t % nd], Wd8, Wv8, c.k, idx_out=sel, ws=ws8), nsel)
        timed_replays(g_sel8, 2)
        result["select"]["select_us_d_prime_512"] = round(sorted(timed_replays(g_sel8, 5))[2] * 1e3 / nsel, 2)
        del g_sel8, Wd8, Wv8, ws8
        # the training-side distribution of the vocabulary speculator (Section 3.4): log q_aux over all V
        logq = torch.empty((c.rows, c.V), dtype=torch.float32, device=dev)
        ws_aux = torch.empty(sv.workspace_bytes(sv.SV_OP_AUX_LOG_SOFTMAX, c.rows, c.d, c.V, 0, c.d_prime, 0,
                                                sv.SV_BF16), dtype=torch.uint8, device=dev)
        g_aux = capture(lambda t: sv.aux_log_softmax(h[t % nd], Wd, Wv, out=logq, ws=ws_aux), nsel)
        timed_replays(g_aux, 2)
        result["aux_log_softmax_us"] = round(sorted(timed_replays(g_aux, 5))[2] * 1e3 / nsel, 2)
        del g_aux, logq, ws_aux

        # ---------------- the paper's break-even (Section 6, Table 4): SpecVocab wins over a static reduced
        # vocabulary V' when V d'/d + k < |V'|.  Static V' = 32K most frequent tokens (the size the
        # static-vocabulary baselines use) against SpecVocab with k = 2048 (the paper's typical k) and 8192.
        note("config 2: break-even against a static 32K vocabulary")
        static_idx = torch.arange(32768, dtype=torch.int32, device=dev)
        zs = torch.empty((c.rows, 32768), dtype=torch.float32, device=dev)
        st_us = sorted(timed_replays(capture(
            lambda t: sv.draft_step(h[t % nd], U, static_idx, c.kd, logits_out=zs, tok_out=tok[t % nd],
                                    prob_out=prob[t % nd]), nsel), 5))[2] * 1e3 / nsel
        # the same static vocabulary in its own mode: rows packed once, then a dense projection per step
        U_static = sv.pack_rows(U, static_idx)

        def static_packed(t):
            i = t % nd
            sv.dense_logits(h[i], U_static, out=zs)
            sv.draft_topk(zs, static_idx, c.kd, tok_out=tok[i], prob_out=prob[i])
        stp_us = sorted(timed_replays(capture(static_packed, nsel), 5))[2] * 1e3 / nsel
        del U_static
        sel2k = torch.empty((c.rows, 2048), dtype=torch.int32, device=dev)
        z2k = torch.empty((c.rows, 2048), dtype=torch.float32, device=dev)

        def full2k(t):
            i = t % nd
            sv.select(h[i], Wd, Wv, 2048, idx_out=sel2k, ws=ws)
            sv.draft_step(h[i], U, sel2k, c.kd, logits_out=z2k, tok_out=tok[i], prob_out=prob[i])
        sp2k_us = sorted(timed_replays(capture(full2k, nsel), 5))[2] * 1e3 / nsel
        result["break_even"] = {
            "dense_full_vocab_us": result["dense"]["us_per_step"],
            "static_32k_vocab_us": round(min(st_us, stp_us), 2),
            "static_32k_gathered_us": round(st_us, 2),
            "static_32k_packed_us": round(stp_us, 2),
            "specvocab_k2048_us": round(sp2k_us, 2),
            "specvocab_k8192_us": round(full_us, 2),
            "rows_equivalent": {"static": 32768, "specvocab_k2048": c.V * c.d_prime // c.d + 2048,
                                "specvocab_k8192": c.V * c.d_prime // c.d + 8192},
            "note": "whole draft step incl. softmax + top-10; SpecVocab legs include the selector "
                    "(W_down, W_vocab, exact top-k); random-init selector, so timing only"}

    del copies
    torch.cuda.empty_cache()
    if not args.no_extras:
        del U, h, idx, z
        torch.cuda.empty_cache()
        result["other_configs"] = other_configs(sv, torch, np, dev, capture, timed_replays)
        result["indexed_lm_head_microbenchmark"] = indexed_head_microbenchmark(sv, torch, dev, capture, timed_replays)

    # ---------------- CPU oracle on a bounded sample of the same steps
    if not args.no_cpu_baseline:
        note("CPU oracle on a sample of the same steps")
        import oracle
        n_cpu, t_cpu = 0, 0.0
        tc0 = time.perf_counter()
        while n_cpu < nd and (time.perf_counter() - tc0) < args.cpu_seconds:
            i = n_cpu
            z_ref = oracle.subset_logits(h_np[i], U_np, idx_np[i])
            oracle.softmax_topk(z_ref, idx_np[i], c.kd)
            n_cpu += 1
        t_cpu = time.perf_counter() - tc0
        result["cpu_baseline"] = {"value": round(t_cpu / n_cpu * 1e6, 1), "unit": "us/draft-step", "cores": 1,
                                  "kind": "oracle",
                                  "sample": f"first {n_cpu} of the {nd} steps of the same workload "
                                            f"(subset logits + softmax + top-{c.kd}), single thread",
                                  "host_cpus": os.cpu_count()}
        # the same oracle, untouched, on all host cores at once: one step per thread (ctypes releases the
        # interpreter lock around the C calls), throughput of the whole host
        from concurrent.futures import ThreadPoolExecutor
        ncores = max(1, min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), os.cpu_count() or 1))

        def one(i):
            z_ref = oracle.subset_logits(h_np[i], U_np, idx_np[i])
            oracle.softmax_topk(z_ref, idx_np[i], c.kd)
        n_all = min(nd, max(ncores, int(ncores * max(1.0, args.cpu_seconds / 2.0) / max(t_cpu / n_cpu, 1e-3))))
        ta0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=ncores) as pool:
            list(pool.map(one, range(n_all)))
        t_all = time.perf_counter() - ta0
        result["cpu_baseline_all_cores"] = {"value": round(t_all / n_all * 1e6, 1), "unit": "us/draft-step",
                                            "cores": ncores, "kind": "oracle",
                                            "sample": f"first {n_all} steps, one step per thread on {ncores} threads; "
                                                      f"value = wall time / steps (throughput of the whole host)"}

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
