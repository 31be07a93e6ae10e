#!/usr/bin/env python3
"""Benchmark of the Medusa static-tree verify step on one MI355X.

One "step" = one pass of the whole hot path over one batch of seeded synthetic input, all four C-ABI
calls: medusa_heads -> tree_verify_step -> accept_longest_prefix -> kv_compact, inputs resident in HBM.
Prints ONE JSON line: steps/s (value), ms/step, achieved HBM GB/s of the whole step, a `roofline`
object for the dominant kernel family (the weight-streaming GEMMs, timed with HIP events on the launch
stream in instrumented steps that follow the timed region) and a `cpu_baseline` object (the float64
oracle timed on this machine's host cores on a bounded sample of the same workload).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3_step_1k] [--no-heads]
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

HBM_PEAK_GBPS = 8000.0            # MI355X published HBM3E peak
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a copy kernel
# of known size; see profiles/gemm_w64_cfg3_step_1k_pmc.md).  Measured offline; not re-measured by this script.
TRAFFIC_W64 = {"fetch_bytes_per_launch": 110.88e6, "write_bytes_per_launch": 6.33e6,
               "source": "profiles/gemm_w64_cfg3_step_1k_pmc.md"}


def algorithmic_bytes(w, with_heads: bool):
    """Bytes one step must move through HBM: every weight once, the prefix KV once, the T new KV rows
    written and read once, the embedding rows gathered.  Activations (<= 1.4 MB each) are not counted."""
    es = 4 if w.dtype == "fp32" else 2
    T, K = w.tree.n_nodes, w.n_medusa
    kvd = w.kv_heads * w.head_dim
    layer_w = (2 * w.d * w.d + 2 * kvd * w.d + 3 * w.d * w.ffn) * es
    gemm_layers = w.n_layers * layer_w
    lm = w.vocab * w.d * es
    heads = K * (w.d * w.d + w.vocab * w.d) * es if with_heads else 0
    # K and V of one slot, one layer; 8-bit rows: one byte per feature plus one fp32 scale per head and matrix
    kv_row = 2 * (kvd + 4 * w.kv_heads) if w.kv_quant else 2 * kvd * es
    kv_prefix = sum(w.prefix) * kv_row * w.n_layers
    kv_tree = 2 * w.batch * T * kv_row * w.n_layers               # written + read
    embed = w.batch * T * w.d * es
    gemm_w64 = gemm_layers + lm          # every 64-row launch: QKV, O, gate/up, down of each layer and the LM head
    return dict(gemm=gemm_layers + lm + heads, gemm_w64=gemm_w64,
                weights_layers=gemm_layers, lm_head=lm, heads=heads,
                kv_prefix=kv_prefix, kv_tree=kv_tree, embed=embed,
                total=gemm_layers + lm + heads + kv_prefix + kv_tree + embed)


def build_device(w, with_heads):
    import torch
    import workload as W
    import paper_2603_03383_amd as P
    dev = "cuda:0"
    dm = P.DeviceModel(d=w.d, n_heads=w.n_heads, head_dim=w.head_dim, ffn=w.ffn, vocab=w.vocab, n_layers=w.n_layers,
                       dtype=w.dtype, tree=w.tree.name, n_kv_heads=w.n_kv_heads, rms_eps=w.rms_eps, rope_base=w.rope_base, device=dev)
    for l in range(w.n_layers):
        mats = [W.layer_weight(w, l, m, dev) for m in W.LAYER_MATS]
        dm.add_layer(*mats, W.norm_gain(w, f"layer{l}.g_attn", dev), W.norm_gain(w, f"layer{l}.g_ffn", dev))
        del mats
    dm.set_embed(W.embedding(w, dev))
    dm.set_lm_head(W.lm_head(w, dev))
    dm.set_final_gain(W.norm_gain(w, "g_final", dev))
    if with_heads:
        for k in range(1, w.n_medusa + 1):
            dm.add_medusa_head(W.medusa_w1(w, k, dev), None, W.medusa_lm(w, k, dev))
    dm.finalize()
    max_prefix = max(w.prefix) + (w.n_medusa + 1)
    kv = P.DeviceKV(dm, batch=w.batch, cap=max_prefix + w.tree.n_nodes, quant=w.kv_quant)
    for b in range(w.batch):
        for l in range(w.n_layers):
            k, v = W.prefix_kv(w, l, b, dev)
            kv.write(l, b, 0, k, v)
    torch.cuda.empty_cache()
    return dm, kv, max_prefix


def cpu_baseline(w, with_heads, budget_s=20.0):
    """Times the oracle (as it stands) on sequence 0 of the workload: decoder layers one after the other until
    `budget_s` seconds of oracle time are spent (all of them if they fit), then the final norm / LM head / argmax /
    acceptance and the Medusa heads; layers not run are accounted for by linear scaling, and so are further
    sequences of a batch.  Weights are generated layer by layer outside the timed regions."""
    import numpy as np
    import workload as W
    from oracle import medusa as O
    from oracle import tree as OT
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    f32 = lambda t: t.detach().to("cpu").float().numpy()
    tree = OT.build_tree(w.tree.caps, w.tree.budgets)
    T = tree["T"]
    cfg = dict(n_layers=w.n_layers, d=w.d, n_heads=w.n_heads, n_kv_heads=w.kv_heads, head_dim=w.head_dim, ffn=w.ffn,
               vocab=w.vocab, rms_eps=w.rms_eps, rope_base=w.rope_base, dtype=w.dtype, kv_quant=w.kv_quant)
    gen = "cuda:0"
    S = w.prefix[0]
    x = f32(W.hidden_state(w, "bench_x", T, gen)).astype(np.float64)
    t_layers, nl = 0.0, 0
    for l in range(w.n_layers):
        lw = {m: f32(W.layer_weight(w, l, m, gen)) for m in W.LAYER_MATS}
        lw["g_attn"], lw["g_ffn"] = f32(W.norm_gain(w, f"layer{l}.g_attn", gen)), f32(W.norm_gain(w, f"layer{l}.g_ffn", gen))
        k, v = W.prefix_kv(w, l, 0, gen)
        kc = np.zeros((w.kv_heads, S + T, w.head_dim)); vc = np.zeros_like(kc)
        kc[:, :S] = f32(k); vc[:, :S] = f32(v)
        t0 = time.perf_counter()
        x = O.tree_verify_layer(x, lw, kc, vc, S, tree, cfg)
        t_layers += time.perf_counter() - t0
        nl += 1
        del lw, kc, vc
        if t_layers > budget_s:
            break
    model = dict(cfg=cfg, g_final=f32(W.norm_gain(w, "g_final", gen)), lm_head=f32(W.lm_head(w, gen)))
    t0 = time.perf_counter()
    hidden, logits = O._final(x, model)
    am = O.argmax_lowest(logits)
    tokens = np.arange(T) % w.vocab
    O.accept_longest_prefix(tree, tokens, am)
    t_final = time.perf_counter() - t0
    t_heads, nh = 0.0, 0
    if with_heads:
        for kh in range(1, w.n_medusa + 1):
            head = dict(w1=f32(W.medusa_w1(w, kh, gen)), b1=None, lm=f32(W.medusa_lm(w, kh, gen)))
            m1 = dict(model, medusa=[head])
            tr1 = dict(tree, caps=tree["caps"][:1], cand_slot=np.zeros(T, np.int32))
            t0 = time.perf_counter()
            O.medusa_heads(hidden[0], m1, tr1)
            t_heads += (time.perf_counter() - t0) / 2.0     # the call also evaluates the base head: ~half is the head
            nh += 1
            del head, m1
    per_seq = t_layers / nl * w.n_layers + t_final + (t_heads / nh * w.n_medusa if nh else 0.0)
    est = per_seq * w.batch
    return dict(value=1.0 / est, unit="steps/s", cores=int(cores), kind="oracle",
                sample=f"sequence 0: {nl} of {w.n_layers} layers ({t_layers:.2f} s) + final norm/LM head/argmax/accept "
                       f"({t_final:.2f} s)" + (f" + {nh} of {w.n_medusa} Medusa heads ({t_heads:.2f} s)" if with_heads else "")
                       + f"; {t_layers + t_final + t_heads:.1f} s of oracle time, scaled linearly to the full step of "
                       f"{w.batch} sequence(s): {est:.1f} s/step")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3_step_1k")
    ap.add_argument("--no-heads", action="store_true", help="time verify+accept+compact only")
    ap.add_argument("--prefix", type=int, default=None, help="override the workload's prefix length (every sequence)")
    ap.add_argument("--kv8", action="store_true", help="8-bit KV cache rows (E4M3 codes + one fp32 scale per row)")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-extras", action="store_true",
                    help="leave out the autoregressive baseline and the chained loop (profiling runs: only the timed steps are traced)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workload as W
    import paper_2603_03383_amd as P

    w = W.CONFIGS[args.workload]
    if args.kv8:
        w = w.with_(name=f"{w.name}+kv8", kv_quant="fp8e4m3")
    if args.prefix is not None:
        w = w.with_(name=f"{w.name}@prefix{args.prefix}", prefix=(args.prefix,) * w.batch)
    with_heads = not args.no_heads and w.n_layers > 1
    P.lib()                                         # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    dm, kv, max_prefix = build_device(w, with_heads)
    Bn, T = w.batch, w.tree.n_nodes
    buf = P.StepBuffers(dm, Bn, max_prefix)
    seq0 = torch.tensor(w.prefix, dtype=torch.int32, device=dm.device)
    seq_len = seq0.clone()
    hidden = W.hidden_state(w, "bench_h", Bn, dm.device).view(Bn, 1, w.d)
    root = W.random_tokens(w, "bench_root", (Bn,), dm.device)
    buf.tree_tokens.copy_(W.random_tokens(w, "bench_tree", (Bn, T), dm.device))
    layer_only = w.n_layers == 1
    x0 = W.hidden_state(w, "bench_x", Bn * T, dm.device).float()
    x = x0.clone()

    def one_step():
        seq_len.copy_(seq0)                        # compaction advanced the lengths: reset (4*B bytes)
        if layer_only:
            P.tree_verify_layer(dm.desc, dm.layer(0), 0, x, kv.desc, seq_len, Bn, max_prefix, buf.ws)
        else:
            P.run_step(dm, kv, buf, hidden, None, root, seq_len, with_heads=with_heads)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / args.steps * 1e3

    # instrumented steps: HIP events around every kernel launch, on the launch stream
    P.medusa_profile_begin(args.steps * (w.n_layers * 12 + 64))
    for _ in range(args.steps):
        one_step()
    prof = P.medusa_profile_end()
    torch.cuda.synchronize()

    # the autoregressive baseline (Section 4.1): the same weights and prefix, the single-node tree, timed the same way
    ar = None
    if not layer_only and not args.skip_extras:
        dm_ar = dm.view_with_tree("tree1")
        buf_ar = P.StepBuffers(dm_ar, Bn, max_prefix)
        h_ar = hidden

        def ar_step():
            seq_len.copy_(seq0)
            P.run_step(dm_ar, kv, buf_ar, h_ar, None, root, seq_len)

        for _ in range(args.warmup):
            ar_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ar_step()
        torch.cuda.synchronize()
        ms_ar = (time.perf_counter() - t0) / args.steps * 1e3
        from paper_2603_03383_amd import metrics as M
        ov = M.overhead(ms, ms_ar)
        ar = {"time_ar_ms": ms_ar, "time_spec_ms": ms, "overhead": ov, "break_even_ac": M.break_even_ac(ov),
              "speedup_at_paper_ac": {"1.78": M.speedup(1.78, ov), "1.65": M.speedup(1.65, ov)},
              "max_ac_of_this_tree": w.n_medusa + 1,
              "note": "Overhead = Time_spec / Time_AR, Speedup = AC / Overhead (Section 4.1); Time_AR is one step of the "
                      "single-node tree (M = 1 GEMMs, single-query attention) over the same weights and prefix; AC needs "
                      "trained heads, so the paper's own AC values (1.78 at length 128, 1.65 at 1024) are plugged in; "
                      "the paper reports overhead 1.32 / 1.77 on its NPU"}
        del buf_ar
        seq_len.copy_(seq0)

    # the chained on-device loop (Section 3.2's device-resident, static-shape decode): N steps back to back, each
    # step's root / hidden / lengths taken from the previous one on the device; eager launches vs one HIP graph replayed
    chain = None
    if not layer_only and with_heads and not args.skip_extras:
        n_chain = 16
        cap_chain = max(w.prefix) + n_chain * (w.n_medusa + 1)
        kv_c = P.DeviceKV(dm, batch=Bn, cap=cap_chain + T, quant=w.kv_quant)
        for b in range(Bn):
            for l in range(w.n_layers):
                k, v = W.prefix_kv(w, l, b, dm.device)
                kv_c.write(l, b, 0, k, v)
        chain = {"steps": n_chain}
        for mode, use_graph in (("eager", False), ("graph", True)):
            dec = P.ChainedDecoder(dm, kv_c, Bn, cap_chain, use_graph=use_graph)
            for rep in range(2):                                       # first pass warms up / captures
                dec.prime(hidden.view(Bn, w.d), root, seq0)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                toks, lens = dec.run(n_chain)
                torch.cuda.synchronize()
                dt_c = time.perf_counter() - t0
            chain[f"ms_per_step_{mode}"] = dt_c / n_chain * 1e3
            chain[f"tokens_per_s_{mode}"] = float(lens.sum().item()) / dt_c
            del dec
        chain["note"] = ("random-init heads accept only the root, so tokens/s here is steps/s x batch; multiply by a "
                         "trained model's AC (the paper: 1.65-1.78) for its token rate")
        del kv_c

    # practical read ceiling of this machine, measured now: the library's pure-read stream at 1 GB and at the dominant
    # kernel's average size
    from paper_2603_03383_amd.stream_calib import read_ceiling
    ceil = read_ceiling(sizes=(154_500_000, 1_048_576_000), pool_bytes=4 << 30)

    ab = algorithmic_bytes(w, with_heads)
    if layer_only:
        ab["gemm"] = ab["weights_layers"]
        ab["gemm_w64"] -= ab["lm_head"]
        ab["total"] = ab["weights_layers"] + ab["kv_prefix"] + ab["kv_tree"]
    # dominant kernel: gemm_mfma_kernel<4,1,2,128,E> (every 64-row GEMM launch: 128-column bands, 128-feature stages)
    gemm = prof.get("gemm_w64", dict(launches=0, total_us=0.0))
    gemm_us_per_step = gemm["total_us"] / args.steps
    gemm_gbps = ab["gemm_w64"] / (gemm_us_per_step * 1e-6) / 1e9 if gemm_us_per_step else 0.0
    all_gemm_us = sum(v["total_us"] for k, v in prof.items() if k.startswith("gemm")) / args.steps
    all_gemm_gbps = ab["gemm"] / (all_gemm_us * 1e-6) / 1e9 if all_gemm_us else 0.0
    step_gbps = ab["total"] / (ms * 1e-3) / 1e9

    out = {
        "metric": "tree_verify_steps_per_s", "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "tree_nodes": T, "prefix": list(w.prefix), "batch": Bn,
                   "layers": w.n_layers, "with_medusa_heads": with_heads, "kv_rows": w.kv_quant or w.dtype,
                   "step": "tree_verify_layer" if layer_only else "medusa_heads+tree_verify_step+accept_longest_prefix+kv_compact"},
        "hbm": {"algorithmic_bytes_per_step": ab["total"], "achieved_GBps": step_gbps,
                "frac_of_peak": step_gbps / HBM_PEAK_GBPS,
                "kv_share_of_bytes": (ab["kv_prefix"] + ab["kv_tree"]) / ab["total"]},
        "roofline": {"kernel": "gemm_mfma_kernel<4,1,2,128," + ("f16_t" if w.dtype == "fp16" else "bf16_t") + ",*> (gemm_w64: the QKV, O, gate/up, down launches of every layer and the LM head; the last template argument selects the epilogue: partial sums, or SwiGLU for gate/up)",
                     "bound": "hbm", "achieved": gemm_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gemm_gbps / HBM_PEAK_GBPS,
                     "traffic": TRAFFIC_W64["fetch_bytes_per_launch"] + TRAFFIC_W64["write_bytes_per_launch"],
                     "traffic_detail": TRAFFIC_W64,
                     "algorithmic_bytes_per_launch": ab["gemm_w64"] / max(1.0, gemm["launches"] / args.steps),
                     "launches_per_step": gemm["launches"] / args.steps,
                     "avg_launch_us": gemm["total_us"] / max(1, gemm["launches"]),
                     "all_gemm_launches_GBps": all_gemm_gbps,
                     "measured": "HIP events on the launch stream around every launch, %d instrumented steps "
                                 "after the timed region" % args.steps},
        "stream_read_ceiling_GBps": {"%.0fMB" % (k / 1e6): v for k, v in ceil.items()},
        "kernel_us_per_step": {k: v["total_us"] / args.steps for k, v in prof.items()},
        "kernel_launches_per_step": {k: v["launches"] / args.steps for k, v in prof.items()},
        "paper_metrics": ar,
        "chained_loop": chain,
        "paper_context": "paper reports only ratios: 1.35x end-to-end on an NPU, fp16, L=128 (not comparable)",
    }
    if "gemm_large" in prof and prof["gemm_large"]["launches"]:
        # several sequences at once: the layer GEMMs run at M = batch * T rows and are bound by the matrix cores
        gl = prof["gemm_large"]
        elems = w.n_layers * (2 * w.d * w.d + 2 * w.kv_heads * w.head_dim * w.d + 3 * w.d * w.ffn) + (0 if layer_only else w.vocab * w.d)
        flops = 2.0 * Bn * T * elems
        tf = flops / (gl["total_us"] / args.steps * 1e-6) / 1e12
        out["roofline"] = {"kernel": "gemm_large_kernel (every GEMM of the step at M = %d rows)" % (Bn * T), "bound": "mfma",
                           "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0, "traffic": None,
                           "algorithmic_flops_per_launch": flops / (gl["launches"] / args.steps),
                           "launches_per_step": gl["launches"] / args.steps,
                           "avg_launch_us": gl["total_us"] / gl["launches"],
                           "measured": "HIP events on the launch stream around every launch, %d instrumented steps "
                                       "after the timed region" % args.steps}
    if not args.skip_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, with_heads)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
