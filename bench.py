#!/usr/bin/env python3
"""Benchmark of the VADUSA speculative decode step on one MI355X.

One "step" = one vadusa_step: tree expansion, tree-masked forward of all tree
nodes through every layer, acceptance, KV compaction and the draft heads for the
next step.  Workload: the 12-layer d=1024 bf16 decoder at batch 1 with a 64-node
tree (64 text + 225 prompt tokens, then one whole 750-step generation with
random-init draft heads, i.e. one committed token per step, L = 289 -> 1039).
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(m, B, M, L_mean):
    """Bytes one step must move: every weight once, every committed KV row once, tree KV written once."""
    s = 2 if m.dtype == "bf16" else 4
    d, F, V1 = m.d_model, m.d_ffn, m.n_logits
    w_layers = m.n_layers * (3 * d * d + d * d + 2 * d * F) * s
    w_out = V1 * d * s
    w_draft = m.n_draft_heads * (d * d + V1 * d) * s
    kv_pos = m.n_layers * 2 * d * s
    return w_layers + w_out + w_draft + B * L_mean * kv_pos + B * M * kv_pos


def algorithmic_flops(m, B, M, L_mean):
    """Multiply-adds x 2 of one step: the linear maps on all B * M rows, the draft heads on B rows,
    attention of every row over the committed keys and (on average half of) the tree rows."""
    d, F, V1, R = m.d_model, m.d_ffn, m.n_logits, B * M
    maps = 2.0 * R * (m.n_layers * (3 * d * d + d * d + 2 * d * F) + V1 * d)
    draft = 2.0 * B * m.n_draft_heads * (d * d + V1 * d)
    attn = 4.0 * R * (L_mean + M / 2.0) * d * m.n_layers
    return maps + draft + attn


MFMA_PEAK_TFLOPS = 2500.0   # dense bf16


def measured_traffic(workload):
    """HBM bytes per k_step launch from the rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE, scaled by a
    copy kernel of known size); the summary under profiles/ carries the figure on a `traffic_bytes_per_launch:`
    line.  None when no such measurement exists for the workload."""
    path = os.path.join(ROOT, "profiles", f"k_step_{workload}_pmc.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(wl, W, text, prompt, tree, budget_s=15.0):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    from oracle import vadusa_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    model = O.Model(wl.model, W)
    sts = [O.prefill(model, t, p) for t, p in zip(text, prompt)]
    n, t0 = 0, time.perf_counter()
    while True:
        for st in sts:
            O.step(model, st, tree, 1, ignore_eos=True)
        n += 1
        el = time.perf_counter() - t0
        if el > budget_s or n >= 200:
            break
    return {"value": len(sts) * tree.n_nodes * n / el, "unit": "tree tokens/s", "cores": int(cores),
            "kind": "oracle", "us_per_step": el / n * 1e6,
            "sample": f"{n} oracle steps (numpy fp64) from L={len(text[0]) + len(prompt[0])} after an untimed oracle prefill"}


def timed_steps(workload, steps, warmup, tau, by_length=False, keep_open=False):
    """Warm-up, then `steps` timed steps of a workload (whole generations from L0, the prefill between them untimed),
    bracketed by events on the stream the kernels run on.  Returns the result record with its own roofline object
    and, if keep_open, the context and inputs for further legs."""
    import torch
    from synth import PRESETS, make_weights, make_tokens, make_tree
    from paper_2410_21951_amd import Vadusa, TreeArrays
    wl = PRESETS[workload]
    m = wl.model
    W = make_weights(m, wl.seed)
    text, prompt = make_tokens(wl)
    tree = make_tree(wl.tree_nodes, wl.topk_caps)
    tarr = TreeArrays(tree.parent, tree.rank)
    dev = Vadusa(m, max_batch=wl.batch, max_tree_nodes=wl.tree_nodes, ignore_eos=True)
    dev.load_weights(W)
    B, M = wl.batch, wl.tree_nodes
    L0 = [len(t) + len(p) for t, p in zip(text, prompt)]
    seg = wl.n_generate

    dev.prefill(text, prompt)
    for _ in range(warmup):
        dev.step(tarr, tau, sync=False)
    torch.cuda.synchronize()

    total_ms, done, L_sum = 0.0, 0, 0.0
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    while done < steps:
        k = min(seg, steps - done)
        dev.prefill(text, prompt)                 # untimed: back to L = L0
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(k):
            dev.step(tarr, tau, sync=False)
        ev1.record()
        torch.cuda.synchronize()
        total_ms += ev0.elapsed_time(ev1)
        n_out = [len(dev.read_output(b)) for b in range(B)]
        # mean committed length over the segment (linear growth from L0 to L0 + n_out)
        L_sum += k * (np.mean(L0) + np.mean(n_out) / 2.0)
        done += k
    ms_step = total_ms / steps
    # the same step binned by committed length (untimed for the headline figure): five equal
    # slices of one generation, each timed with its own pair of events
    by_L = []
    if steps >= 50 and by_length:
        dev.prefill(text, prompt)
        nb = 5
        per = min(seg, steps) // nb
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(nb + 1)]
        torch.cuda.synchronize()
        evs[0].record()
        for i in range(nb):
            for _ in range(per):
                dev.step(tarr, tau, sync=False)
            evs[i + 1].record()
        torch.cuda.synchronize()
        for i in range(nb):
            by_L.append({"L_from": int(np.mean(L0)) + i * per, "L_to": int(np.mean(L0)) + (i + 1) * per,
                         "us_per_step": evs[i].elapsed_time(evs[i + 1]) / per * 1e3})
    L_mean = L_sum / steps
    nbytes = algorithmic_bytes(m, B, M, L_mean)
    achieved = nbytes / (ms_step * 1e-3) / 1e9
    nflops = algorithmic_flops(m, B, M, L_mean)
    tflops = nflops / (ms_step * 1e-3) / 1e12
    out = {
        "metric": "verified_tree_tokens_per_s", "value": B * M / (ms_step * 1e-3), "unit": "tree tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_step,
        "us_per_step": ms_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": m.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {m.n_layers}L d={m.d_model} {m.dtype}, batch {B}, {M}-node tree, "
                               f"tau={tau}, L {int(np.mean(L0))}->{int(np.mean(L0) + np.mean(n_out))}",
                   "mean_committed_per_step": float(np.mean(n_out)) / min(seg, steps)},
        # dominant kernel: k_step, the persistent kernel that runs a whole step; one launch per step,
        # so its average launch duration is the event-timed region divided by the number of steps
        # the roof that bounds the step: HBM bytes at batch 1 (64 flop per weight byte); from ~1000
        # rows on the contractions at MFMA peak take longer than the bytes at HBM peak
        "roofline": ({"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                      "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(wl.name),
                      "kernel": "k_step (one launch = one speculative step)",
                      "avg_launch_us": ms_step * 1e3, "algorithmic_bytes_per_launch": nbytes,
                      "algorithmic_flops_per_launch": nflops, "tflops": tflops}
                     if nbytes / (HBM_PEAK_GBS * 1e9) >= nflops / (MFMA_PEAK_TFLOPS * 1e12) else
                     {"bound": "mfma", "achieved": tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": tflops / MFMA_PEAK_TFLOPS, "traffic": measured_traffic(wl.name),
                      "kernel": "k_step (one launch = one speculative step)",
                      "avg_launch_us": ms_step * 1e3, "algorithmic_bytes_per_launch": nbytes,
                      "algorithmic_flops_per_launch": nflops, "hbm_gbs": achieved}),
        "by_committed_length": by_L,
    }
    if keep_open:
        return out, (dev, wl, W, text, prompt, tree, tarr)
    dev.close()
    return out, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=750)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="valle_b1")
    ap.add_argument("--tau", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of longform_b1, hubert_b16 and throughput_b64 that follow the headline workload")
    ap.add_argument("--other-steps", type=int, default=20, help="timed steps of each of those workloads")
    ap.add_argument("--only-timed", action="store_true",
                    help="run the warm-up and the timed steps only (no by-length pass, AR / stochastic / dial legs, "
                         "no CPU baseline): every k_step launch of the run is then a step of the workload or a "
                         "prefill chunk, which is what a per-kernel profile should average over")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain copy kernel of known size (256 MiB read + 256 MiB written, 8 launches): "
                         "under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` its counters give the scale of the HBM byte counters")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (the step shards over sequences, "
              "but no multi-GPU path is built)", file=sys.stderr)
        sys.exit(2)
    import torch
    if a.copy_calibration:
        torch.cuda.set_device(0)
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(8):
            torch.mul(src, 1.0, out=dst)      # one elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"launches": 8, "bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4}}))
        return
    from synth import PRESETS, make_weights, make_tokens, make_tree
    from paper_2410_21951_amd import Vadusa, TreeArrays
    torch.cuda.set_device(0)
    out, keep = timed_steps(a.workload, a.steps, a.warmup, a.tau, by_length=not a.only_timed, keep_open=True)
    dev, wl, W, text, prompt, tree, tarr = keep
    m, B, M = wl.model, wl.batch, wl.tree_nodes
    L0 = [len(t) + len(p) for t, p in zip(text, prompt)]
    ms_step = out["ms_per_step"]
    achieved = out["roofline"]["achieved"] if out["roofline"]["bound"] == "hbm" else out["roofline"]["hbm_gbs"]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if a.only_timed:
        dev.close()
        print(json.dumps(out))
        return
    # Plain auto-regressive decoding through the same kernels: a "tree" of the root alone, one
    # token per step.  speedup = accepted tokens per step x t_AR / t_tree (Sec. 4.1's metric); the
    # accepted length is a property of trained draft heads, so the line quotes what the paper's
    # own accepted lengths (Table 1: 3.00 at tau=1, 3.87 at tau=3, four heads) would give here.
    from synth import chain_tree
    t1 = chain_tree(1)
    t1arr = TreeArrays(t1.parent, t1.rank)
    n_ar = min(a.steps, 300)
    dev.prefill(text, prompt)
    for _ in range(5):
        dev.step(t1arr, 1, sync=False)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(n_ar):
        dev.step(t1arr, 1, sync=False)
    ev1.record()
    torch.cuda.synchronize()
    ar_us = ev0.elapsed_time(ev1) / n_ar * 1e3
    out["ar_step"] = {"us_per_step": ar_us, "steps": n_ar, "tree_step_over_ar_step": ms_step * 1e3 / ar_us,
                      "speedup_at_paper_accepted_len": {"tau1_acc3.00": 3.00 * ar_us / (ms_step * 1e3),
                                                        "tau3_acc3.87": 3.87 * ar_us / (ms_step * 1e3)}}
    # What a plain copy kernel reaches on this GPU (1 GiB read + 1 GiB written per launch): the
    # measured ceiling next to the nominal 8 TB/s
    src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(10):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * src.numel() * 4 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst
    out["roofline"]["copy_kernel_gbs"] = copy_gbs
    out["roofline"]["hbm_gbs_over_copy_kernel"] = achieved / copy_gbs
    # Prefill (the call synchronises, so host time is the measure): in passes of max_tree_nodes rows
    # (the default) and in passes of up to 512 rows per sequence (vadusa_config.prefill_chunk), which
    # run in the many-row kernel from 256 rows on.
    def prefill_ms(d, reps=5):
        d.prefill(text, prompt)
        t0 = time.perf_counter()
        for _ in range(reps):
            d.prefill(text, prompt)
        return (time.perf_counter() - t0) / reps * 1e3
    n_prompt = int(sum(L0))
    ms_small = prefill_ms(dev)
    dev512 = Vadusa(m, max_batch=wl.batch, max_tree_nodes=wl.tree_nodes, ignore_eos=True, prefill_chunk=512)
    dev512.load_weights(W)
    ms_big = prefill_ms(dev512)
    dev512.close()
    out["prefill"] = {"prompt_tokens": n_prompt, "ms_passes_of_tree_size": ms_small, "ms_passes_of_512": ms_big,
                      "tokens_per_s_passes_of_512": n_prompt / (ms_big * 1e-3)}
    # The stochastic form of Algorithm 1 (temperature 0.9, top_p 0.9 as in Sec. 3.1.2's sampling runs):
    # the same step with the perturbed-score kernel between the base head and the acceptance; the
    # uniforms are drawn on the device beforehand (their generation is not part of the step).
    n_st = min(a.steps, 300)
    u_dev = torch.rand(B * M * (m.speech_vocab + 1), device="cuda").clamp_(2.0 ** -24, 1.0 - 2.0 ** -24)
    dev.prefill(text, prompt)
    for _ in range(5):
        dev.step(tarr, a.tau, sync=False, sample=(0.9, 0.9, u_dev))
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(n_st):
        dev.step(tarr, a.tau, sync=False, sample=(0.9, 0.9, u_dev))
    ev1.record()
    torch.cuda.synchronize()
    st_us = ev0.elapsed_time(ev1) / n_st * 1e3
    dev.prefill(text, prompt)                    # the deterministic step over the same span of lengths
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(n_st):
        dev.step(tarr, a.tau, sync=False)
    ev1.record()
    torch.cuda.synchronize()
    det_us = ev0.elapsed_time(ev1) / n_st * 1e3
    out["stochastic_step"] = {"temperature": 0.9, "top_p": 0.9, "us_per_step": st_us, "steps": n_st,
                              "deterministic_us_per_step_same_lengths": det_us,
                              "over_deterministic_step": st_us / det_us}
    # Acceptance dial (batch 1 only).  Random-init draft heads are never right, so the timed run
    # above commits one token per step.  To time acceptance and compaction with paper-shaped path
    # lengths, the draft lists are planted: the greedy continuation is recorded first (tau = 1 is
    # lossless, so the stream of the run above is that continuation), then head i's list gets
    # the true token i steps ahead at rank 0 with probability alpha (seeded), a wrong one
    # otherwise.  alpha = 0.755 gives sum_k alpha^k = 3.0 accepted tokens per step with four
    # heads (the paper's Table 1 at tau = 1).  Each step returns its accepted tokens to the host
    # (one synchronisation per step, included in the time).
    # bf16 rounding differs between a token verified as a tree node and the same token decoded as
    # a root, so an arg-max inside a near-tie can flip and the planted run then leaves the
    # recorded continuation: it is recorded again from there (untimed) and the run goes on.
    if B == 1 and a.tau == 1 and a.steps >= 50:
        rng = np.random.default_rng(wl.seed + 99)
        alpha, Hh, V = 0.755, m.n_draft_heads, m.speech_vocab
        cur = np.asarray(prompt[0], np.int32)

        def record(p, n):
            dev.prefill(text, [p])
            for _ in range(n):
                dev.step(tarr, 1, sync=False)
            f = dev.read_output(0).tolist()
            dev.prefill(text, [p])
            return f

        future = record(cur, 150)
        pos = n_steps = n_tok = rerecorded = 0
        el = 0.0
        while n_steps < 200 and len(cur) + pos + 160 < m.max_positions - M - len(text[0]):
            if pos + Hh + 2 >= len(future):
                cur = np.concatenate([cur, np.asarray(future[:pos], np.int32)])
                future, pos = record(cur, 150), 0
            lists = []
            for i in range(1, Hh + 1):      # the root is future[pos]; head i must propose future[pos + i]
                true = future[pos + i]
                ids = [(true + 1 + j) % V for j in range(16)]          # 16 wrong candidates
                if rng.random() < alpha:
                    ids[0] = true
                lists.append(ids)
            t0 = time.perf_counter()
            acc = dev.step(tarr, 1, override=[lists], sync=True)[0]
            el += time.perf_counter() - t0
            n_steps += 1
            n_tok += len(acc)
            if acc == future[pos:pos + len(acc)]:
                pos += len(acc)
            else:
                rerecorded += 1
                cur = np.concatenate([cur, np.asarray(dev.read_output(0), np.int32)])
                future, pos = record(cur, 150), 0
        out["acceptance_dial"] = {"alpha": alpha, "steps": n_steps, "mean_accepted_per_step": n_tok / max(n_steps, 1),
                                  "us_per_step_incl_host_sync": el / max(n_steps, 1) * 1e6,
                                  "accepted_tokens_per_s": n_tok / el if el else 0.0,
                                  "ar_tokens_per_s": 1e6 / ar_us,
                                  "speedup_over_ar_incl_host_sync": (n_tok / el) / (1e6 / ar_us) if el else 0.0,
                                  # device time only: accepted tokens per step x t_AR / t_tree, both without host round trips
                                  "speedup_over_ar_device_time": (n_tok / max(n_steps, 1)) * ar_us / (ms_step * 1e3),
                                  "continuation_recorded_again": rerecorded}
    dev.close()
    # The other single-GPU workloads through the same entry point, each with a roofline object of its own
    # (the bound named per workload: HBM bytes at batch 1, MFMA at 1024 and 2048 rows); the headline stays valle_b1.
    if a.workload == "valle_b1" and not a.no_other_workloads:
        out["workloads"] = []
        for name in ("longform_b1", "hubert_b16", "throughput_b64"):
            rec, _ = timed_steps(name, a.other_steps, 5, PRESETS[name].taus[0])
            out["workloads"].append({k: rec[k] for k in ("value", "unit", "steps", "warmup", "us_per_step", "dtype", "config", "roofline")})
            torch.cuda.empty_cache()
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, W, text, prompt, tree)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
