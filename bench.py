#!/usr/bin/env python3
"""Benchmark of the FastMTP draft path on one MI355X.

One "step" = one pass of the whole hot path over one batch: K recursive draft steps of the shared MTP head with the
compressed output head (mtp_draft_steps), then acceptance + rollback against a synthetic target chain (mtp_accept).
Inputs are seeded and synthetic (7B-shaped head, bf16 ~N(0,0.02) weights), resident in HBM before timing starts.

Prints ONE JSON line.  `value` = draft tokens/s of the headline workload (config 2: one sequence, context 2048,
32768-row head, K = 3).  Beside it:
  roofline       the kernel the timed path launches (the single-launch kernel: all phases of all K steps), its average
                 launch duration from HIP events on the launch stream, algorithmic bytes per launch, the 8 TB/s HBM
                 peak, HBM bytes from the committed counter runs; `phases`: every phase of a draft step from the
                 kernel's own time stamps; `k_lmhead`: the output-head kernel of the one-launch-per-phase mode
  stream_ceiling a plain streaming read and a device copy, timed here: what this machine sustains
  full_vocab     the same path with the uncompressed head
  configs        the other configurations (batch 16; the vocabulary sweep at context 8192 incl. the full head through
                 the identity list; batch 64), each timed the same way
  k_sweep        the K-step chain measured for K = 1..7 and the draft-length model of Sec. 3.5 fed with those times
  cpu_baseline   the CPU oracle timed on this machine's host cores on the headline workload
and, unless --no-next-rows, the block of new positions, the list builder and the teacher-forced forward.
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
PMC_SUMMARY = os.path.join(ROOT, "profiles", "pmc_hbm_traffic_c2_7b_b1.md")
EXPECTED_ACCEPT = {0.8: (3, 1.952), 0.7: (5, 1.94117)}  # sum_j p^j for (p, K) of configs 3 and 5


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE, each
    scaled by what the same counter reads for a copy of known size); None if the summary does not cover it."""
    try:
        for line in open(PMC_SUMMARY):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 5 and cells[1] == kernel:
                return float(cells[-2])
    except (OSError, ValueError):
        pass
    return None


def step_bytes(shape, n_rows: int, ctx, k_index: int, with_ids: bool):
    """HBM bytes one draft step must move, by phase: every weight of the head once, n_rows rows of the output head (+
    the id list), and the K/V entries of every sequence up to and including the new one (k_index = 1-based step)."""
    d, F = shape.d_model, shape.d_ffn
    ph = {"proj": 2.0 * 2 * d * d, "qkv": 2.0 * (shape.q_dim + 2 * shape.kv_dim) * d,
          "attn": sum((int(L) + k_index) * 2 * shape.kv_dim * 2.0 for L in ctx), "oproj": 2.0 * d * shape.q_dim,
          "gateup": 2.0 * 2 * F * d, "down": 2.0 * F * d,
          "lmhead": 2.0 * n_rows * d + (4.0 * n_rows if with_ids else 0.0)}
    return ph


def chain_bytes(shape, n_rows, ctx, K, with_ids) -> float:
    return sum(sum(step_bytes(shape, n_rows, ctx, k, with_ids).values()) for k in range(1, K + 1))


def device_state():
    """Name, unit count and, where the driver's sysfs files are readable, the engine and memory clock levels in force
    after the timed region (files are read, no other program is started: the GPU is initialised by now)."""
    import glob
    import torch
    prop = torch.cuda.get_device_properties(0)
    dev = {"name": prop.name, "arch": getattr(prop, "gcnArchName", None), "compute_units": prop.multi_processor_count,
           "hbm_gib": round(prop.total_memory / 2**30, 1)}
    cards = []
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))[:8]:
        card = {"card": path.split("/")[4]}
        for key, name in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk"), ("level", "power_dpm_force_performance_level")):
            try:
                with open(os.path.join(os.path.dirname(path), name)) as f:
                    lines = [l.strip() for l in f if l.strip()]
                starred = [l for l in lines if l.endswith("*")]
                card[key] = (starred or lines)[0] if lines else None
            except OSError:
                card[key] = None
        cards.append(card)
    dev["clock_levels"] = cards or "not readable"
    return dev


class Chain:
    """One workload on one engine: the K-step chain + acceptance, replayed on the same inputs."""

    def __init__(self, binding, synth, torch, wl, w, subsets, max_steps=None, act=None):
        self.binding, self.synth, self.torch, self.wl = binding, synth, torch, wl
        self.shape, self.B = wl.shape, wl.batch
        self.act = act if act is not None else synth.make_activations(wl, threads=16)
        self.cap = self.act["kv_capacity"]
        self.kmax = max_steps or wl.draft_steps
        self.eng = binding.DraftEngine(self.shape, w, subsets, self.B, self.cap, self.kmax, device="cuda:0")
        e = self.eng
        self.hidden, self.token = e.to_device_bits(self.act["hidden_in"]), e.to_device_i32(self.act["token_in"])
        self.kc, self.vc = e.to_device_bits(self.act["k_cache"]), e.to_device_bits(self.act["v_cache"])
        self.kv0 = e.to_device_i32(self.act["kv_len"])
        self.kv = self.kv0.clone()
        B, K = self.B, self.kmax
        self.draft_buf = {k: torch.empty((B, k), dtype=torch.int32, device="cuda:0") for k in range(1, K + 1)}
        self.acc = torch.empty(B, dtype=torch.int32, device="cuda:0")
        self.out_tok = torch.empty((B, K + 1), dtype=torch.int32, device="cuda:0")
        self.pend = torch.empty(B, dtype=torch.int32, device="cuda:0")

    def one(self, subset_index, K, target):
        b, e = self.binding, self.eng
        draft = self.draft_buf[K]
        st = b.mtp_draft_steps(e.handle, self.B, K, subset_index, self.hidden, self.token, self.kc, self.vc, self.kv,
                               None, draft, None, None, 0)
        assert st == 0, b.mtp_status_string(st)
        st = b.mtp_accept(e.handle, self.B, K, draft, target, 0, self.kv, self.acc, self.out_tok, self.pend, 0)
        assert st == 0, b.mtp_status_string(st)
        self.kv.copy_(self.kv0)  # replay the same cycle next time (4*B bytes, device to device)

    def target_for(self, subset_index, K):
        """Target chain built from this configuration's own drafts (stand-in for the target model's verification)."""
        torch = self.torch
        dummy = torch.zeros((self.B, K + 1), dtype=torch.int32, device="cuda:0")
        self.one(subset_index, K, dummy)
        torch.cuda.synchronize()
        assert self.eng.poll_error() == 0
        tg = self.synth.make_targets(self.wl, self.draft_buf[K].cpu().numpy())
        return self.eng.to_device_i32(tg)

    def timed(self, subset_index, steps, warmup, K=None):
        torch = self.torch
        K = K or self.wl.draft_steps
        target = self.target_for(subset_index, K)
        for _ in range(warmup):
            self.one(subset_index, K, target)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            self.one(subset_index, K, target)
        torch.cuda.synchronize()
        el = time.perf_counter() - t
        return el, float(self.acc.float().mean().item())

    def row(self, name, subset_index, steps, warmup, with_ids=None, K=None):
        """One line of the `configs` table."""
        K = K or self.wl.draft_steps
        el, mean_acc = self.timed(subset_index, steps, warmup, K)
        n_rows = self.eng.subset_size(subset_index)
        ids = (subset_index >= 0) if with_ids is None else with_ids
        cb = chain_bytes(self.shape, n_rows, self.act["kv_len"], K, ids)
        gbs = cb * steps / el / 1e9
        r = {"name": name, "batch": self.B, "draft_steps": K,
             "context": [int(self.act["kv_len"].min()), int(self.act["kv_len"].max())], "head_rows": n_rows,
             "us_per_mtp_step": el / (steps * K) * 1e6, "draft_tokens_per_s": self.B * K * steps / el,
             "algorithmic_bytes_per_step": cb / K, "achieved_gbs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
             "mean_accept_len": mean_acc}
        exp = EXPECTED_ACCEPT.get(self.wl.accept_prob)
        if exp and exp[0] == K:
            r["expected_accept_len"] = exp[1]
        return r


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="c2_7b_b1")
    ap.add_argument("--subset", type=int, default=0, help="index into the workload's subset list; -1 = full vocabulary")
    ap.add_argument("--launch-mode", default="auto", choices=("auto", "per-phase", "single"),
                    help="how the library enqueues a call; auto = the library's own choice (single launch for one "
                         "sequence); both are timed briefly for one sequence and reported")
    ap.add_argument("--extend", type=int, default=4,
                    help="also time the first draft step over a block of this many new positions per sequence "
                         "(mtp_draft_extend); reported beside the main figures, never part of `value`; 0: skip")
    ap.add_argument("--list-builder", type=int, default=26, metavar="LOG2_TOKENS",
                    help="also time the high-frequency list builder (mtp_subset_build) on a synthetic long-tailed "
                         "stream of 2^LOG2_TOKENS tokens over this workload's vocabulary")
    ap.add_argument("--train-loss", type=int, default=512, metavar="POSITIONS",
                    help="also time the teacher-forced K-step forward with its weighted cross-entropy "
                         "(mtp_train_loss, K = 3, beta = 0.6) over this many positions")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the three side measurements above (block of positions, list builder, training forward)")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations (3, 4, 5)")
    ap.add_argument("--no-k-sweep", action="store_true", help="skip the measured K = 1..7 chains")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-vocab", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--k-sweep-target-ms", type=float, default=2.6,
                    help="ASSUMED time of one target-model forward for the draft-length model of Sec. 3.5")
    ap.add_argument("--phase-table", default="",
                    help="also write the per-phase time stamps of the single-launch kernel as a markdown table here")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run one plain 256 MiB device copy (a known-size reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding are part of it); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if args.no_next_rows:
        args.extend = args.list_builder = args.train_loss = 0

    import numpy as np
    import torch
    from paper_2509_18362_amd import binding, ksweep, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = synth.WORKLOADS[args.workload]
    shape, K, B = wl.shape, wl.draft_steps, wl.batch
    t0 = time.time()
    w = synth.make_weights(wl if wl.shape is synth.TINY else synth.WORKLOADS["c2_7b_b1"], threads=16)
    subsets = synth.make_subsets(wl)
    kmax = 7 if (B == 1 and not args.no_k_sweep) else K
    main_chain = Chain(binding, synth, torch, wl, w, subsets, max_steps=kmax)
    gen_s = time.time() - t0
    eng, act, cap = main_chain.eng, main_chain.act, main_chain.cap
    w_dev = eng.w  # device tensors: later engines share them
    stream = 0     # the null stream, which is also torch's current stream here

    if args.copy_calib:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    # ---- headline: K draft steps + acceptance, launch mode as the library chooses (or as asked) -------------------
    mode_ids = {"per-phase": binding.LAUNCH_PER_PHASE, "single": binding.LAUNCH_SINGLE, "auto": binding.LAUNCH_AUTO}
    mode_us = {}
    if B == 1:
        for name in ("per-phase", "single"):
            assert binding.mtp_set_launch_mode(eng.handle, mode_ids[name]) == 0
            n_t = max(20, args.steps // 5)
            el, _ = main_chain.timed(args.subset, n_t, max(5, args.warmup // 3))
            mode_us[name] = el / (n_t * K) * 1e6
    assert binding.mtp_set_launch_mode(eng.handle, mode_ids[args.launch_mode]) == 0
    elapsed, mean_accept = main_chain.timed(args.subset, args.steps, args.warmup)
    n_rows = eng.subset_size(args.subset)
    cbytes = chain_bytes(shape, n_rows, act["kv_len"], K, args.subset >= 0)
    tok_s = B * K * args.steps / elapsed
    us_per_mtp_step = elapsed / (args.steps * K) * 1e6
    path_gbs = cbytes * args.steps / elapsed / 1e9
    single = B == 1 and args.launch_mode != "per-phase"  # the path that was timed is the single-launch kernel
    target = main_chain.target_for(args.subset, K)
    draft, kv, acc, out_tok, pend = main_chain.draft_buf[K], main_chain.kv, main_chain.acc, main_chain.out_tok, main_chain.pend

    # ---- the dominant kernel of the timed path, timed with HIP events on the launch stream -------------------------
    # What an event pair around ONE launch adds to the kernel's own duration (the dispatch of a dependent launch):
    # the same bracket around single launches of the acceptance kernel against back-to-back launches of it.
    brackets = []
    for _ in range(50):
        b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        b0.record()
        binding.mtp_accept(eng.handle, B, K, draft, target, 1, kv, acc, out_tok, pend, stream)
        b1.record()
        b1.synchronize()
        brackets.append(b0.elapsed_time(b1) * 1e3)
    bracket_us = float(np.median(brackets))
    n_acc = 200
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n_acc):
        binding.mtp_accept(eng.handle, B, K, draft, target, 1, kv, acc, out_tok, pend, stream)  # mode 1: kv_len unchanged
    e1.record()
    torch.cuda.synchronize()
    accept_us = e0.elapsed_time(e1) * 1e3 / n_acc

    # the whole call (one kernel in single-launch mode): events inside the library around mtp_draft_steps' launches
    binding.mtp_set_timing(eng.handle, binding.TIMING_CALL)
    chain_us = []
    for _ in range(min(args.steps, 100)):
        main_chain.one(args.subset, K, target)
        chain_us.append(binding.mtp_last_draft_ms(eng.handle) * 1e3)
    binding.mtp_set_timing(eng.handle, binding.TIMING_OFF)
    p10, p50, p90 = (float(np.percentile(chain_us, q)) for q in (10, 50, 90))

    # the output-head kernel of the one-launch-per-phase mode (the largest single phase)
    assert binding.mtp_set_launch_mode(eng.handle, binding.LAUNCH_PER_PHASE) == 0
    binding.mtp_set_timing(eng.handle, binding.timing_phase("lmhead"))
    durs = []
    for i in range(max(30, args.steps // 3)):
        main_chain.one(args.subset, K, target)
        if i % 10 == 9:  # reading the events waits for the stream: do it sparsely
            durs.append(binding.mtp_last_draft_ms(eng.handle))
    torch.cuda.synchronize()
    binding.mtp_set_timing(eng.handle, binding.TIMING_OFF)
    assert binding.mtp_set_launch_mode(eng.handle, mode_ids[args.launch_mode]) == 0
    head_ms = float(np.median(durs))
    head_bytes = step_bytes(shape, n_rows, act["kv_len"], 1, args.subset >= 0)["lmhead"]
    k_lmhead = {"what": "output-head kernel of the one-launch-per-phase mode, event pair around each launch",
                "bytes_per_launch": head_bytes, "avg_launch_us": head_ms * 1e3,
                "achieved": head_bytes / (head_ms * 1e-3) / 1e9, "frac": head_bytes / (head_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "traffic": measured_traffic("k_lmhead") if (args.workload == "c2_7b_b1" and args.subset == 0) else None}

    # per-phase breakdown of the single-launch kernel from its own time stamps
    phases = None
    if single:
        W = torch.cuda.get_device_properties(0).multi_processor_count
        tbuf = torch.zeros(binding.mtp_phase_trace_bytes(eng.cfg) // 8, dtype=torch.int64, device="cuda:0")
        assert binding.mtp_set_phase_trace(eng.handle, tbuf) == 0
        acc_t, reps_t = None, 20
        for _ in range(reps_t):
            tbuf.zero_()
            main_chain.one(args.subset, K, target)
            torch.cuda.synchronize()
            t = tbuf.cpu().numpy()[:K * 8 * 4 * W].reshape(K, 8, 4, W).astype(np.float64) * 0.01  # us
            t = t - t[0, 7, 0].min()
            acc_t = t if acc_t is None else acc_t + t
        assert binding.mtp_set_phase_trace(eng.handle, None) == 0
        t = acc_t / reps_t
        order = [(7, "proj_hidden_half"), (0, "proj_embedding_half"), (1, "qkv"), (2, "attn"), (3, "oproj"),
                 (4, "gateup"), (5, "down"), (6, "lmhead")]
        phases, prev_end = [], None
        for s in range(K):
            sb = step_bytes(shape, n_rows, act["kv_len"], s + 1, args.subset >= 0)
            for sec, name in order:
                nbytes = sb["proj"] / 2 if name.startswith("proj") else sb[name]
                end = float(t[s, sec, 3].max())
                start = prev_end if prev_end is not None else float(t[s, sec, 0].min())
                rel = t[s, sec, 1]
                phases.append({"step": s + 1, "phase": name, "bytes": nbytes, "span_us": end - start,
                               "gbs": nbytes / max(end - start, 1e-9) / 1e3,
                               "input_ready_after_previous_phase_us": [float(rel.min() - start), float(rel.max() - start)],
                               "staging_us": float(np.median(t[s, sec, 2] - rel)),
                               "compute_us_min_median_max": [float(np.min(t[s, sec, 3] - t[s, sec, 2])),
                                                             float(np.median(t[s, sec, 3] - t[s, sec, 2])),
                                                             float(np.max(t[s, sec, 3] - t[s, sec, 2]))]})
                prev_end = end
        interior_us = float(t[K - 1, 6, 3].max() - t[0, 7, 0].min())
        if args.phase_table:
            with open(args.phase_table, "w") as f:
                f.write(f"| step | phase | MB | span us | GB/s | input ready after previous phase ended, us (first..last "
                        f"workgroup) | staging us | compute us (min / median / max over workgroups) |\n|---|---|---|---|---|---|---|---|\n")
                for r in phases:
                    a, b2 = r["input_ready_after_previous_phase_us"]
                    c = r["compute_us_min_median_max"]
                    f.write(f"| {r['step']} | {r['phase']} | {r['bytes'] / 1e6:.1f} | {r['span_us']:.1f} | {r['gbs']:.0f} | "
                            f"{a:.1f}..{b2:.1f} | {r['staging_us']:.1f} | {c[0]:.1f} / {c[1]:.1f} / {c[2]:.1f} |\n")
                f.write(f"\nkernel interior (first request to last result): {interior_us:.1f} us for {K} steps\n")

    kname = "k_flow" if single else "k_lmhead"
    if single:
        k_us, k_bytes = p50, cbytes
    else:
        k_us, k_bytes = head_ms * 1e3, head_bytes
    roofline = {"bound": "hbm", "kernel": kname, "achieved": k_bytes / (k_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": k_bytes / (k_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "traffic": measured_traffic(kname) if (args.workload == "c2_7b_b1" and args.subset == 0) else None,
                "bytes_per_launch": k_bytes, "avg_launch_us": k_us,
                "what": (f"one launch = all phases of {K} draft steps" if single else "one launch = one output-head phase"),
                "whole_path_achieved": path_gbs, "whole_path_frac": path_gbs / HBM_PEAK_GBS,
                "event_pair_around_one_accept_launch_us": bracket_us,
                "event_pair_overhead_us": bracket_us - accept_us,  # at least this much of avg_launch_us is not the kernel
                "phases": phases, "k_lmhead": k_lmhead}

    # ---- what this machine sustains: a plain streaming read (the weight stream's own access pattern) and a device copy ---
    probe_bytes = (eng.w["lm_head"].numel() * 2) // 16384 * 16384
    out8 = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    for _ in range(3):
        assert binding.mtp_stream_probe(eng.w["lm_head"], probe_bytes, out8, stream) == 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        binding.mtp_stream_probe(eng.w["lm_head"], probe_bytes, out8, stream)
    e1.record()
    torch.cuda.synchronize()
    read_gbs = probe_bytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * (1 << 30) * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    stream_ceiling = {"read_gbs": read_gbs, "read_frac_of_peak": read_gbs / HBM_PEAK_GBS,
                      "read_what": f"mtp_stream_probe over the {probe_bytes / 1e6:.0f} MB output head, 10 passes",
                      "copy_gbs_read_plus_write": copy_gbs, "copy_what": "torch copy of 1 GiB, bytes read + written"}

    # ---- the uncompressed head on the same workload ----------------------------------------------------------------
    full = None
    if not args.no_full_vocab and args.subset >= 0:
        fs = max(10, args.steps // 4)
        el_f, _ = main_chain.timed(-1, fs, max(3, args.warmup // 4))
        full = {"value": B * K * fs / el_f, "unit": "draft tokens/s", "us_per_mtp_step": el_f / (fs * K) * 1e6,
                "rows": shape.vocab_size, "compressed_speedup": (el_f / fs) / (elapsed / args.steps),
                "roofline_speedup": chain_bytes(shape, shape.vocab_size, act["kv_len"], K, False) / cbytes}

    # ---- the K-step chain for K = 1..7 (Sec. 3.5) and the draft-length model fed with the measured times -----------
    k_sweep = None
    if kmax >= 7:
        chains = []
        for k in range(1, 8):
            n_k = max(20, args.steps // 6)
            tg = main_chain.target_for(args.subset, k)
            for _ in range(5):
                main_chain.one(args.subset, k, tg)
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(n_k):
                main_chain.one(args.subset, k, tg)
            torch.cuda.synchronize()
            chains.append((time.perf_counter() - t) / n_k)  # chain + acceptance, seconds
        rows = ksweep.sweep(chains, 0.0, args.k_sweep_target_ms * 1e-3)
        k_sweep = {"measured_chain_plus_accept_us": [c * 1e6 for c in chains],
                   "us_per_mtp_step_by_K": [c * 1e6 / (k + 1) for k, c in enumerate(chains)],
                   "model": {"assumed_target_forward_ms": args.k_sweep_target_ms,
                             "acceptance": "the paper's 0.81/0.56/0.36 cumulative (Sec. 3.4), later positions extrapolated",
                             "rows": rows, "best_K": max(rows, key=lambda r: r["speedup_vs_plain_decoding"])["K"]}}

    # ---- the other configurations ------------------------------------------------------------------------------------
    configs = None
    if not args.no_configs and args.workload == "c2_7b_b1":
        configs = []
        # config 3: batch 16, ragged contexts, acceptance probability 0.8
        c3 = Chain(binding, synth, torch, synth.WORKLOADS["c3_7b_b16"], w_dev, synth.make_subsets(synth.WORKLOADS["c3_7b_b16"]))
        configs.append(c3.row("c3_7b_b16", 0, 100, 10))
        c3.eng.close()
        del c3
        # config 4: the vocabulary sweep at context 8192 (Table 2's sizes), incl. the full head through the identity list
        wl4 = synth.WORKLOADS["c4_7b_vocab"]
        subs4 = list(synth.make_subsets(wl4)) + [np.arange(shape.vocab_size, dtype=np.int32)]
        c4 = Chain(binding, synth, torch, wl4, w_dev, subs4)
        rows4 = [c4.row("c4_full_dense", -1, 60, 6)]
        rows4.append(c4.row("c4_full_identity_list", len(subs4) - 1, 60, 6))
        for i in range(len(subs4) - 2, -1, -1):
            rows4.append(c4.row(f"c4_subset_{len(subs4[i])}", i, 100, 10))
        full_us, full_b = rows4[0]["us_per_mtp_step"], rows4[0]["algorithmic_bytes_per_step"]
        for r in rows4:
            r["speedup_over_full_dense"] = full_us / r["us_per_mtp_step"]
            r["bytes_ratio_to_full_dense"] = full_b / r["algorithmic_bytes_per_step"]
        configs.extend(rows4)
        c4.eng.close()
        del c4
        # config 5: batch 64, long ragged contexts, K = 5, acceptance probability 0.7
        wl5 = synth.WORKLOADS["c5_7b_b64"]
        c5 = Chain(binding, synth, torch, wl5, w_dev, synth.make_subsets(wl5))
        configs.append(c5.row("c5_7b_b64", 0, 20, 3))
        c5.eng.close()
        del c5
        torch.cuda.empty_cache()

    extend = None
    if args.extend > 0:
        m = args.extend
        assert int(act["kv_len"].max()) + m <= cap, "the block does not fit the workload's cache capacity"
        eng2 = binding.DraftEngine(shape, w_dev, subsets, B * m, cap, 1, device="cuda:0")
        rng = np.random.default_rng(7)
        std = float(synth.bf16_bits_to_f32(act["hidden_in"]).std())
        hid_m = eng2.to_device_bits(synth.f32_to_bf16_bits(
            (rng.standard_normal((m, B, shape.d_model)) * std).astype(np.float32)))
        tok_m = eng2.to_device_i32(rng.integers(0, shape.vocab_size, size=(m, B)).astype(np.int32))
        ext_len = eng2.to_device_i32(np.full(B, m, dtype=np.int32))
        draft_m = torch.empty((m, B), dtype=torch.int32, device="cuda:0")
        kc, vc, kv0 = main_chain.kc, main_chain.vc, main_chain.kv0

        def one_block():
            st = binding.mtp_draft_extend(eng2.handle, B, m, args.subset, hid_m, tok_m, ext_len, kc, vc, kv, draft_m,
                                          None, None, stream)
            assert st == 0, binding.mtp_status_string(st)
            kv.copy_(kv0)

        n_blk = max(20, args.steps // 3)
        for _ in range(max(3, args.warmup // 3)):
            one_block()
        torch.cuda.synchronize()
        assert eng2.poll_error() == 0
        t = time.perf_counter()
        for _ in range(n_blk):
            one_block()
        torch.cuda.synchronize()
        el_b = time.perf_counter() - t
        # what one pass has to read: every weight once, the head's rows once, the caches once per position
        blk_bytes = sum(step_bytes(shape, n_rows, act["kv_len"], 1, args.subset >= 0).values())
        extend = {"positions_per_sequence": m, "rows": B * m, "us_per_call": el_b / n_blk * 1e6,
                  "positions_per_s": B * m * n_blk / el_b,
                  "speedup_over_one_position_at_a_time": m * us_per_mtp_step / (el_b / n_blk * 1e6),
                  "weight_pass_bytes": blk_bytes}
        # One cycle of the drafting loop as Sec. 2.3 runs it after a verification that accepted m - 1 drafts: step 1
        # over the m new positions (target hidden states), K - 1 recursive steps from the last position's own output,
        # acceptance (against a dummy target chain: what is timed is the work, not the acceptance rate).
        if K >= 2 and int(act["kv_len"].max()) + m + K - 1 <= cap:
            hid_out = torch.empty((m, B, shape.d_model), dtype=torch.float32, device="cuda:0")
            draft_c = torch.empty((B, K - 1), dtype=torch.int32, device="cuda:0")
            draft_k = torch.empty((B, K), dtype=torch.int32, device="cuda:0")
            tok_c = torch.empty(B, dtype=torch.int32, device="cuda:0")  # the last position's draft, 16-byte aligned

            def one_cycle():
                st = binding.mtp_draft_extend(eng2.handle, B, m, args.subset, hid_m, tok_m, ext_len, kc, vc, kv,
                                              draft_m, None, hid_out, stream)
                assert st == 0, binding.mtp_status_string(st)
                tok_c.copy_(draft_m[m - 1])
                st = binding.mtp_draft_continue(eng.handle, B, K - 1, args.subset, hid_out[m - 1], tok_c, kc, vc,
                                                kv, None, draft_c, None, None, stream)
                assert st == 0, binding.mtp_status_string(st)
                draft_k[:, 0] = tok_c
                draft_k[:, 1:] = draft_c
                st = binding.mtp_accept(eng.handle, B, K, draft_k, target, 0, kv, acc, out_tok, pend, stream)
                assert st == 0, binding.mtp_status_string(st)
                kv.copy_(kv0)

            for _ in range(max(3, args.warmup // 3)):
                one_cycle()
            torch.cuda.synchronize()
            assert eng.poll_error() == 0 and eng2.poll_error() == 0
            t = time.perf_counter()
            for _ in range(n_blk):
                one_cycle()
            torch.cuda.synchronize()
            el_c = (time.perf_counter() - t) / n_blk
            extend["cycle"] = {"what": f"block of {m} positions, {K - 1} recursive steps, acceptance", "us": el_c * 1e6,
                               "draft_tokens_per_s": B * K / el_c}
        eng2.close()

    builder = None
    if args.list_builder > 0:
        n_tok = 1 << args.list_builder
        stream_host = synth.make_token_stream(shape.vocab_size, n_tok, seed=9)
        stream_dev = torch.from_numpy(stream_host).to("cuda:0")
        n_list = min(32768, shape.vocab_size)
        ws_bytes = binding.mtp_subset_workspace_bytes(shape.vocab_size)
        ws_b = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
        ids_b = torch.empty(n_list, dtype=torch.int32, device="cuda:0")

        def build_once():
            st = binding.mtp_subset_build(stream_dev, n_tok, shape.vocab_size, n_list, ws_b, ws_bytes, ids_b, None,
                                          None, stream)
            assert st == 0, binding.mtp_status_string(st)

        for _ in range(3):
            build_once()
        torch.cuda.synchronize()
        reps_b = 20
        t = time.perf_counter()
        for _ in range(reps_b):
            build_once()
        torch.cuda.synchronize()
        el_l = (time.perf_counter() - t) / reps_b
        t = time.perf_counter()
        from oracle import oracle as orc_list
        ref_l = orc_list.build_subset(stream_host, shape.vocab_size, n_list)
        cpu_l = time.perf_counter() - t
        assert np.array_equal(ids_b.cpu().numpy(), ref_l["ids"])
        builder = {"tokens": n_tok, "vocab": shape.vocab_size, "list_size": n_list, "us_per_build": el_l * 1e6,
                   "tokens_per_s": n_tok / el_l, "algorithmic_gbs": 4.0 * n_tok / el_l / 1e9,
                   "frac_of_hbm_peak": 4.0 * n_tok / el_l / 1e9 / HBM_PEAK_GBS,
                   "oracle_seconds": cpu_l, "matches_oracle": True}
        del stream_dev

    train = None
    if args.train_loss > 0:
        n_pos, Kt = args.train_loss, 3
        eng3 = binding.DraftEngine(shape, w_dev, [], n_pos, max(64, -(-n_pos // 64) * 64), 1, device="cuda:0")
        rng = np.random.default_rng(8)
        hid_t = eng3.to_device_bits(synth.f32_to_bf16_bits(rng.standard_normal((n_pos, shape.d_model)).astype(np.float32)))
        tok_t = eng3.to_device_i32(rng.integers(0, shape.vocab_size, size=n_pos + Kt + 1).astype(np.int32))
        for _ in range(2):
            loss_t = eng3.train_loss(hid_t, tok_t, Kt, 0.6)
        torch.cuda.synchronize()
        assert eng3.poll_error() == 0
        reps_t = 5
        t = time.perf_counter()
        for _ in range(reps_t):
            loss_t = eng3.train_loss(hid_t, tok_t, Kt, 0.6)
        torch.cuda.synchronize()
        el_t = (time.perf_counter() - t) / reps_t
        # multiply-adds of the head per position and step: the body's matrices and the full output head
        macs = (2 * shape.d_model * shape.d_model + (shape.q_dim + 2 * shape.kv_dim) * shape.d_model
                + shape.q_dim * shape.d_model + 3 * shape.d_ffn * shape.d_model + shape.vocab_size * shape.d_model)
        train = {"positions": n_pos, "K": Kt, "beta": 0.6, "ms_per_forward": el_t * 1e3,
                 "positions_per_s": n_pos / el_t, "tflops": 2.0 * macs * n_pos * Kt / el_t / 1e12,
                 "loss": [float(x) for x in loss_t.cpu().numpy()],
                 "note": "every matrix phase is one LDS-tiled MFMA matrix product over all positions (activations as "
                         "bf16 hi + lo: two MFMAs per product)"}
        eng3.close()

    cpu = None
    if not args.no_cpu_baseline:
        from oracle.oracle import Oracle
        orc = Oracle(shape, w, cap, "f32")
        ids = None if args.subset < 0 else subsets[args.subset]
        nseq = min(B, 4)  # a bounded sample: at most four sequences of the batch
        reps, t = 0, time.perf_counter()
        while True:
            orc.chain(K, act["hidden_in"][:nseq], act["token_in"][:nseq], act["k_cache"][:nseq].copy(),
                      act["v_cache"][:nseq].copy(), act["kv_len"][:nseq], ids, want_logits=False, want_hidden=False)
            reps += 1
            el_c = time.perf_counter() - t
            if el_c >= args.cpu_seconds and reps >= 2 or el_c >= 3 * args.cpu_seconds:
                break
        cpu = {"value": nseq * K * reps / el_c, "unit": "draft tokens/s", "cores": orc.threads, "kind": "oracle",
               "sample": f"{reps} repetitions of the oracle's K={K} chain on {nseq} of {B} sequences of {wl.name}",
               "us_per_mtp_step": el_c / (reps * K) * 1e6 / nseq * B}
        # the same on one thread (one sequence, at least one chain, about a third of the budget)
        all_threads = orc.threads
        orc.set_threads(1)
        reps1, t = 0, time.perf_counter()
        while True:
            orc.chain(K, act["hidden_in"][:1], act["token_in"][:1], act["k_cache"][:1].copy(),
                      act["v_cache"][:1].copy(), act["kv_len"][:1], ids, want_logits=False, want_hidden=False)
            reps1 += 1
            el_1 = time.perf_counter() - t
            if el_1 >= args.cpu_seconds / 3:
                break
        orc.set_threads(all_threads)
        cpu["single_thread"] = {"value": K * reps1 / el_1, "unit": "draft tokens/s",
                                "sample": f"{reps1} repetitions of the K={K} chain on 1 sequence"}
        try:
            with open("/proc/cpuinfo") as f:
                cpu["cpu_model"] = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), None)
        except OSError:
            pass

    line = {
        "metric": "draft tokens/sec (and us per MTP step, HBM GB/s vs peak), compressed vs full vocab",
        "value": tok_s, "unit": "draft tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 weights and KV, f32 accumulate", "data": "synthetic",
        "config": {"workload": wl.name, "batch": B, "draft_steps": K, "context": [int(act["kv_len"].min()),
                                                                                   int(act["kv_len"].max())],
                   "head_rows": n_rows, "vocab": shape.vocab_size, "d_model": shape.d_model,
                   "launch_mode": ("single" if single else "per-phase")},
        "launch_mode_trial_us_per_mtp_step": mode_us or None,
        "us_per_mtp_step": us_per_mtp_step, "mean_accept_len": mean_accept,
        "mean_accept_len_note": "one sequence, one fixed target chain: a single sample, not a rate (configs 3 and 5 "
                                "report rates over their batches)" if B == 1 else None,
        "chain_us": {"p10": p10, "p50": p50, "p90": p90, "what": f"{K} draft steps, one library call"},
        "accept_us": accept_us,
        "algorithmic_bytes_per_step": cbytes / K, "roofline": roofline, "stream_ceiling": stream_ceiling,
        "full_vocab": full, "configs": configs, "k_sweep": k_sweep,
        "extend": extend, "list_builder": builder, "train_loss": train,
        "cpu_baseline": cpu,
        "input_generation_s": gen_s,
        "device": device_state(),
    }
    eng.close()
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    status = main()
    if status:
        sys.exit(status)
