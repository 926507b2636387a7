#!/usr/bin/env python3
"""Benchmark of the WISV edge-side verification round on one MI355X.

One step = one whole verify round (target forward over the K drafted tokens of every stream against the
KV cache, decision head, first-reject scan) on synthetic inputs already resident in HBM.
Prints ONE JSON line: verified draft tokens/s and ms per round, the roofline of the dominant kernel
(HIP-event durations measured here), and the CPU oracle timed on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--no-cpu-baseline] [--verifier wisv|ss]

--verifier ss times the speculative-sampling verifier (Sec. II-A) on the same forward instead of the decision
head: same workload, synthetic drafter distributions and uniform numbers resident in HBM.
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

HBM_PEAK_GBS = 8000.0         # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def build_round(ctx, w, binding, gen, np, torch):
    """Synthetic cache contents, drafts (built against the path's own greedy chain at the workload's match
    rate), drafter hidden states and CSI for workload w; returns a DeviceRound ready to be re-enqueued."""
    dev = "cuda:0"
    pred_next = []
    for b in range(w.batch):
        for l in range(w.model.n_layers):
            k, v = gen.synthetic_kv(w, b, l, dev)
            binding.kv_fill(ctx._kv, w.model, l, b, k, v)
        pn = gen.synthetic_pred_next(w, b)
        pred_next.append(pn)
        ctx.wisv_set_state(b, w.ctx, pn)
    csi = gen.csi_features(w)
    sid = np.arange(w.batch)
    drafts = np.zeros((w.batch, w.k), np.int32)
    plans = [gen.draft_plan(w, b) for b in range(w.batch)]
    nc = binding.WISV_FLAG_NO_COMMIT
    for j in range(w.k):
        if j == 0:
            t = np.asarray(pred_next)
        else:
            r = ctx.wisv_verify_round(sid, drafts, w.protos, None, np.full(w.m, -1), csi, np.zeros(w.batch), w.k, nc)
            t = r["target_argmax"][:, j]
        for b in range(w.batch):
            keep, alt = plans[b]
            a = int(alt[j])
            drafts[b, j] = int(t[b]) if (keep[j] and not w.uniform_drafts) else \
                (a if a != int(t[b]) else (a + 1) % w.model.vocab)
    probe = ctx.wisv_verify_round(sid, drafts, w.protos, None, np.full(w.m, -1), csi, np.zeros(w.batch), w.k, nc)
    mism = [[j for j in range(w.k) if (int(probe["mismatch_mask"][b]) >> j) & 1] for b in range(w.batch)]
    hd, row_map = gen.pack_hidden(w, [gen.draft_hidden(w, b) for b in range(w.batch)], mism)
    tau = np.full(w.batch, w.taus[len(w.taus) // 2], np.float32)
    rnd = ctx.device_round(sid, drafts, w.protos, hd if hd.shape[0] else None, row_map, csi, tau, w.k, nc)
    return rnd, dict(drafts=drafts, hd=hd, row_map=row_map, csi=csi, tau=tau, pred_next=pred_next)


def measured_traffic(workload, kclass):
    """HBM bytes per launch (fetched + written) of the kernels of class `kclass`, from the committed rocprofv3
    counter summary of this workload - or None when there is none or the kernel sources changed since."""
    import bench_profiles as ps
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, "no counter summary for this workload under profiles/"
    sha, table = ps.read_traffic(path)
    if sha != ps.source_hash():
        return None, "kernel sources changed since the counters under profiles/ were taken"
    launches = bytes_ = 0.0
    for name, (n, fetch, write) in table.items():
        if ps.kernel_class(name) == kclass:
            launches += n
            bytes_ += n * (fetch + write)
    if not launches:
        return None, "the counter summary has no kernel of this class"
    return bytes_ / launches, f"profiles/{workload}_hbm_traffic.txt (FETCH_SIZE + WRITE_SIZE scaled by a copy kernel)"


def generation_loop(ctx, w, inputs, n_rounds, binding, gen, np):
    """n_rounds consecutive committed rounds per stream (Alg. 1's outer loop with a synthetic drafter): every block
    starts at the stream's pending token, the other drafts follow the target's own greedy chain with the
    workload's match rate (the chain is found with uncommitted rounds that are not timed).  Returns the average
    accepted length (Sec. IV-C) and the time of the committed rounds, host buffers and copies included."""
    sid = np.arange(w.batch)
    csi, tau = inputs["csi"], inputs["tau"]
    for b in range(w.batch):
        ctx.wisv_set_state(b, w.ctx, inputs["pred_next"][b])
    pending = np.asarray(inputs["pred_next"], np.int64)
    accepted, seconds = [], 0.0
    nc = binding.WISV_FLAG_NO_COMMIT
    for r in range(n_rounds):
        keep = gen.uniform01(w.seed, f"loop/keep/{r}", w.m).reshape(w.batch, w.k) < gen.match_rates(w)[:, None]
        alt = gen.randint(w.seed, f"loop/alt/{r}", (w.batch, w.k), w.model.vocab).numpy()
        drafts = np.zeros((w.batch, w.k), np.int32)
        drafts[:, 0] = pending
        for j in range(1, w.k):                       # the drafter's view of the target: one uncommitted round per position
            t = ctx.wisv_verify_round(sid, drafts, w.protos, None, np.full(w.m, -1), csi, np.zeros(w.batch), w.k, nc)["target_argmax"][:, j]
            drafts[:, j] = np.where(keep[:, j], t, np.where(alt[:, j] != t, alt[:, j], (alt[:, j] + 1) % w.model.vocab))
        probe = ctx.wisv_verify_round(sid, drafts, w.protos, None, np.full(w.m, -1), csi, np.zeros(w.batch), w.k, nc)
        mism = [[j for j in range(w.k) if (int(probe["mismatch_mask"][b]) >> j) & 1] for b in range(w.batch)]
        hd, row_map = gen.pack_hidden(w, [gen.draft_hidden(w, b) for b in range(w.batch)], mism)
        t0 = time.perf_counter()
        g = ctx.wisv_verify_round(sid, drafts, w.protos, hd if hd.shape[0] else None, row_map, csi, tau, w.k, 0)
        seconds += time.perf_counter() - t0
        accepted.append(g["accepted_len"].copy())
        pending = g["correction_token"].astype(np.int64)
    acc = np.concatenate(accepted)
    from paper_2604_17701_amd import link_model as lm
    return {"rounds": n_rounds, "AAL": lm.average_accepted_length(acc.tolist()),
            "ms_per_committed_round_host_io": seconds / n_rounds * 1e3,
            "generated_tokens_per_s": float(acc.sum()) / seconds,
            "final_context": [int(ctx.wisv_get_state(b)[0]) for b in range(min(w.batch, 4))]}


def profiled_duration(workload, kclass):
    """Average duration (microseconds) rocprofv3's kernel trace gave the kernels of class `kclass` in the committed
    summary of this workload, or None when there is none or the kernel sources changed since."""
    import bench_profiles as ps
    stats = os.path.join(ROOT, "profiles", f"{workload}_kernel_stats.txt")
    if not os.path.exists(stats) or ps.read_hash(stats) != ps.source_hash():
        return None
    calls = total = 0.0
    for name, (n, avg) in ps.read_kernels(stats).items():
        if ps.kernel_class(name) == kclass:
            calls += n
            total += n * avg
    return total / calls if calls else None


def link_model_rows(w, t_edge, res):
    """The paper's per-round latency model (Sec. IV) with this run's measured edge time T_T + T_J plugged in, on
    two example links: which upload option the model prefers, and the modelled communication + edge latency
    of a round for both (the drafter term is left out: it is the same for both options)."""
    from paper_2604_17701_amd import link_model as lm
    fr = lm.Framing(vocab=w.model.vocab, d_hidden=w.model.d_draft, bits_hidden=16, hdr_up=256, hdr_down=256, bits_pos=8)
    m = float(sum(bin(int(x)).count("1") for x in res["mismatch_mask"])) / max(len(res["mismatch_mask"]), 1)
    rows = []
    for name, link in (("50/100 Mbit/s, 2 ms", lm.Link(50e6, 100e6, 0.01, 0.01, 2e-3)),
                       ("50/100 Mbit/s, 20 ms", lm.Link(50e6, 100e6, 0.01, 0.01, 20e-3))):
        fh = lm.t_comm_fh(fr, link, w.k) + t_edge
        sh = (link.t_up(fr.b_up1_sh(w.k)) + link.t_down(fr.hdr_down + m * fr.bits_pos) + link.t_up(fr.hdr_up + m * fr.b_hid) +
              link.t_down(fr.b_fb) + 2 * link.tau_rtt) + t_edge
        rows.append({"link": name, "mean_requested_positions": m, "T_FH_ms": fh * 1e3, "T_SH_ms": sh * 1e3,
                     "model_prefers": "FH" if lm.choose_protocol(fr, link, w.k, m) == lm.PROTO_FH else "SH"})
    return rows


def cpu_baseline(w, weights_dev, inputs, gen, np, torch, budget_s=20.0):
    """The oracle, as it stands, on the host cores: whole rounds of stream 0 of the same workload."""
    from oracle import wisv_oracle as wo
    wh = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in weights_dev.items()}
    orc = wo.Oracle(w.model, wh)
    cache = orc.new_cache(w.ctx + w.k)
    for l in range(w.model.n_layers):
        k, v = gen.synthetic_kv(w, 0, l, "cuda:0")
        cache[l, 0, :, :w.ctx] = k.float().cpu().numpy()
        cache[l, 1, :, :w.ctx] = v.float().cpu().numpy()
    rows = inputs["row_map"][:w.k]
    args = (cache, w.ctx, inputs["pred_next"][0], inputs["drafts"][0], w.protos[0], inputs["hd"], rows,
            inputs["csi"][0], float(inputs["tau"][0]))
    orc.verify_round(*args)                                    # warm-up
    times = []
    t_start = time.perf_counter()
    while len(times) < 3 or (time.perf_counter() - t_start < budget_s and len(times) < 20):
        t0 = time.perf_counter()
        orc.verify_round(*args)
        times.append(time.perf_counter() - t0)
    med = sorted(times)[len(times) // 2]
    return {"value": w.k / med, "unit": "verified draft tokens/s", "cores": wo.num_threads(), "kind": "oracle",
            "sample": f"{len(times)} whole rounds of one stream (K={w.k}, context {w.ctx}) of this workload, "
                      f"median {med * 1e3:.1f} ms per round; one stream of {w.batch}"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="index into the five workloads (default: the headline one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--verifier", choices=("wisv", "ss"), default="wisv",
                    help="wisv: CSI-aware decision head (the headline path); ss: speculative sampling on the same forward")
    ap.add_argument("--loop", type=int, default=0,
                    help="also run N consecutive committed rounds per stream with a synthetic drafter and report the "
                         "average accepted length (not part of the timed steps)")
    ap.add_argument("--shape", default=None,
                    help="BATCH,CONTEXT,K: the chosen config's recipe at another batch / cached length / block size")
    ap.add_argument("--one-term", type=int, default=None,
                    help="mask of product classes (1 QKV, 2 O, 4 gate/up, 8 down, 16 LM head) that take their activations as one "
                         "half-precision term in rounds of more than 16 rows (default: the library's, all five)")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="also run N plain 1 GiB copy kernels (known traffic, for scaling rocprofv3 memory counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: the verify round runs on ONE GPU (streams are independent; nothing is sharded): "
                 "run with --gpus 1")

    import numpy as np
    import torch

    from paper_2604_17701_amd import binding
    from wisv_inputs import configs, gen

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU: the verify round has no CPU implementation")
    w = configs.get(a.config)
    if a.shape:
        from dataclasses import replace
        b_, l_, k_ = (int(x) for x in a.shape.split(","))
        w = replace(w, name=f"{w.name}_as_b{b_}_l{l_}_k{k_}", batch=b_, ctx=l_, k=k_,
                    protos=tuple(w.protos[i % len(w.protos)] for i in range(b_)))
    dev = "cuda:0"
    t0 = time.time()
    wd = gen.make_weights(w.model, w.seed if a.config == 0 else configs.get(1).seed, dev)
    m = w.model
    max_ctx = w.ctx + w.k + a.loop * w.k
    kv = binding.new_kv_cache(m, w.batch, max_ctx, dev)
    ctx = binding.Context(m, wd, w.batch, max_ctx, w.k, kv_cache=kv)
    if a.one_term is not None:
        ctx.wisv_set_option(binding.WISV_OPT_ONE_TERM_CLASSES, a.one_term)
    rnd, inputs = build_round(ctx, w, binding, gen, np, torch)
    if a.verifier == "ss":
        # same drafts; drafter distributions with a small mass on the drafted token, uniform numbers as inputs
        q = torch.from_numpy(gen.draft_distributions(w.seed, w.m, m.vocab, inputs["drafts"].reshape(-1), np.full(w.m, 2e-5)))
        rnd = ctx.ss_device_round(np.arange(w.batch), inputs["drafts"], q, gen.unit_uniforms(w.seed, "ss_u", w.m),
                                  gen.unit_uniforms(w.seed, "ss_v", w.batch), w.k, binding.WISV_FLAG_NO_COMMIT)
        del q
    log(f"{w.name}: inputs resident after {time.time() - t0:.1f}s")

    # ---- the timed region: exactly `steps` rounds between two synchronisations
    for _ in range(a.warmup):
        rnd.run()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(a.steps):
        rnd.run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    ms = elapsed / a.steps * 1e3
    res = rnd.results()
    verified = w.batch * w.k / (ms * 1e-3)

    if a.calibration_copies:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(a.calibration_copies):
            ctx.wisv_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # ---- per-kernel durations: the same rounds again with a HIP event pair around every launch
    ctx.wisv_profile_enable(True)
    for _ in range(a.steps):
        rnd.run()
    ctx.wisv_profile_collect()
    prof = ctx.wisv_profile_read()
    ctx.wisv_profile_enable(False)
    # an empty event pair per round measures what the bracketing adds to every launch; it is subtracted
    pair_us = 1e3 * prof["event_pair_overhead"][0] / max(prof["event_pair_overhead"][1], 1)
    kernels = {n: {"ms_per_round": (t - 1e-3 * pair_us * c) / a.steps, "launches_per_round": c // a.steps,
                   "avg_us": 1e3 * t / max(c, 1) - pair_us}
               for n, (t, c) in prof.items() if c and n != "event_pair_overhead"}
    # algorithmic bytes each weight-streaming kernel class must read per round
    esz = 2 if m.dtype == "bf16" else 4
    d, f, nl = m.d_model, m.d_ff, m.n_layers
    alg_bytes = {
        "gemm_gate_up": nl * 2 * f * d * esz,
        "gemm_qkv": nl * d * (m.d_q + 2 * m.d_kv) * esz,
        "gemm_o": nl * m.d_q * d * esz,
        "gemm_down": nl * d * f * esz,
        "lm_head": m.vocab * d * esz,
        "attention": w.batch * w.ctx * m.kv_bytes_per_token(),
    }
    def hbm_roofline(kclass):
        """Algorithmic bytes of one launch of this class / its average duration, against the HBM peak.  Two clocks:
        HIP event pairs recorded here (minus an empty pair) and, when the committed profile still describes these
        kernels, rocprofv3's kernel trace, which counts a kernel from its dispatch; `frac` takes the slower one."""
        kk = kernels[kclass]
        per_launch = alg_bytes[kclass] / kk["launches_per_round"]
        by_events = per_launch / (kk["avg_us"] * 1e-6) / 1e9
        prof_us = profiled_duration(w.name, kclass)
        by_trace = per_launch / (prof_us * 1e-6) / 1e9 if prof_us else None
        achieved = min(by_events, by_trace) if by_trace else by_events
        traffic, traffic_note = measured_traffic(w.name, kclass)
        return {"bound": "hbm", "kernel": kclass, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_note,
                "bytes_per_launch": per_launch, "avg_launch_us": kk["avg_us"], "event_pair_overhead_us": pair_us,
                "frac_by_event_pairs": by_events / HBM_PEAK_GBS,
                "rocprofv3_avg_launch_us": prof_us,
                "frac_by_rocprofv3_duration": by_trace / HBM_PEAK_GBS if by_trace else None,
                "timing": f"HIP event pair around every launch on the round's stream, {a.steps} rounds right after the timed "
                          "ones, minus the duration of an empty event pair; frac uses the slower of this and the committed "
                          "rocprofv3 kernel-trace average"}

    dom = max((n for n in alg_bytes if n in kernels), key=lambda n: kernels[n]["ms_per_round"])
    roofline = hbm_roofline(dom)
    # matrix-core work of the three GEMM classes: the method's own FLOP (2 x rows x weights; what the kernels execute
    # for it - two bf16 terms or one half-precision term per activation - is not counted) against the dense bf16 / fp16 peak
    gemm_classes = [n for n in ("gemm_gate_up", "gemm_qkv", "gemm_o", "gemm_down", "lm_head") if n in kernels]
    gemm_ms = sum(kernels[n]["ms_per_round"] for n in gemm_classes)
    gemm_flop = 2.0 * w.m * sum(alg_bytes[n] for n in gemm_classes) / esz
    roofline_gemm = None
    if gemm_ms > 0 and m.dtype == "bf16":
        tf = gemm_flop / (gemm_ms * 1e-3) / 1e12
        per_class = {n: 2.0 * w.m * alg_bytes[n] / esz / (kernels[n]["ms_per_round"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS
                     for n in gemm_classes}
        roofline_gemm = {"bound": "mfma", "kernel": "+".join(gemm_classes), "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                         "flop_per_round": gemm_flop, "gemm_ms_per_round": gemm_ms, "frac_per_class": per_class,
                         "one_term_classes": ctx.wisv_get_option(binding.WISV_OPT_ONE_TERM_CLASSES) if w.m > 16 else 0,
                         "note": "algorithmic FLOP of the three GEMM classes / their summed launch durations (HIP event pairs); "
                                 "meaningful where the products are bound by the matrix cores (hundreds of rows)"}
    round_alg = w.algorithmic_bytes()
    out = {
        "metric": ("verified draft tokens/sec + ms per verify round, " +
                   (f"8B-shaped target, K={w.k}" if m.n_layers == 32 else f"tiny fp32 target, K={w.k}") +
                   (f", {w.batch} streams" if w.batch > 1 else "")),
        "value": verified, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if m.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "context": w.ctx, "k": w.k, "rows": w.m,
                   "protocols": "FH" if set(w.protos) == {0} else ("SH" if set(w.protos) == {1} else "FH+SH"),
                   "tau": float(inputs["tau"][0])},
        "roofline": roofline,
        "round_hbm": {"algorithmic_bytes": round_alg, "achieved_GBs": round_alg / (ms * 1e-3) / 1e9,
                      "frac_of_peak": round_alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "accepted_tokens_per_s": float(res["accepted_len"].sum()) / (ms * 1e-3),
        "committed_tokens_per_s": float((res["accepted_len"] + 1).sum()) / (ms * 1e-3),
        "mean_accepted_len": float(res["accepted_len"].mean()),
        "roofline_gemm": roofline_gemm,
        "link_model": link_model_rows(w, ms * 1e-3, res) if a.verifier == "wisv" else None,
        "kernels": kernels,
    }
    if a.verifier == "ss":
        # the four decision kernels are bracketed by one event pair; they must read every logits row once and, for
        # one row per stream, the logits and the drafter's distribution once more
        ss_bytes = (w.m + 2 * w.batch) * m.vocab * 4
        out["config"]["verifier"] = "speculative sampling (Sec. II-A)"
        out["spec_sampling"] = {"us_per_round": kernels["spec_sampling"]["avg_us"], "algorithmic_bytes": ss_bytes,
                                "achieved_GBs": ss_bytes / (kernels["spec_sampling"]["avg_us"] * 1e-6) / 1e9,
                                "logits_written_by_lm_head_bytes": w.m * m.vocab * 4}
    if a.loop and a.verifier == "wisv":
        out["generation_loop"] = generation_loop(ctx, w, inputs, a.loop, binding, gen, np)
    if not a.no_cpu_baseline and a.verifier == "wisv":
        t2 = time.time()
        out["cpu_baseline"] = cpu_baseline(w, wd, inputs, gen, np, torch)
        log(f"cpu baseline took {time.time() - t2:.1f}s")
    ctx.wisv_destroy()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
