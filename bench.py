#!/usr/bin/env python3
"""Benchmark of the FastMTP draft path on one MI355X.

One "step" = one pass of the whole hot path over one batch: K recursive draft steps of the shared MTP head with the
compressed output head (mtp_draft_steps), then acceptance + rollback against a synthetic target chain (mtp_accept).
Inputs are seeded and synthetic (7B-shaped head, bf16 ~N(0,0.02) weights), resident in HBM before timing starts.

Prints ONE JSON line: draft tokens/s (value), ms per step, and the objects `roofline` (dominant kernel against the
8 TB/s HBM peak), `full_vocab` (same path with the uncompressed head) and `cpu_baseline` (the CPU oracle, timed on
this machine's host cores on the same workload).
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


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE, each
    scaled by what the same counter reads for a copy of known size); None if the summary does not cover it."""
    try:
        for line in open(PMC_SUMMARY):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 5 and cells[1] == kernel:
                return float(cells[-2])
    except OSError:
        pass
    return None


def algorithmic_bytes_per_mtp_step(shape, n_rows: int, ctx, k_index: int, with_ids: bool) -> float:
    """HBM bytes one draft step must move: every weight of the head once, n_rows rows of the output head (+ the id
    list), and the K/V entries of every sequence up to and including the new one (k_index = 1-based step)."""
    d, F = shape.d_model, shape.d_ffn
    body = 2.0 * (2 * d * d + (shape.q_dim + 2 * shape.kv_dim) * d + d * shape.q_dim + 3 * F * d)
    head = 2.0 * n_rows * d + (4.0 * n_rows if with_ids else 0.0)
    kv = sum((int(L) + k_index) * 2 * shape.kv_dim * 2.0 for L in ctx)
    return body + head + kv


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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="c2_7b_b1")
    ap.add_argument("--subset", type=int, default=0, help="index into the workload's subset list; -1 = full vocabulary")
    ap.add_argument("--identity-list", action="store_true",
                    help="time the indirect head with the identity id list (all V rows through the gather path)")
    ap.add_argument("--launch-mode", default="auto", choices=("auto", "per-phase", "single"),
                    help="how the library enqueues a call: one launch per phase, or one cooperative launch for all "
                         "phases of all K steps; auto times both briefly for one sequence and keeps the faster")
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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-vocab", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--k-sweep-target-ms", type=float, default=0.0,
                    help="if > 0: add a MODEL of the draft-length sweep (Sec. 3.5) for this assumed target-forward time")
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
    from paper_2509_18362_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = synth.WORKLOADS[args.workload]
    shape, K, B = wl.shape, wl.draft_steps, wl.batch
    t0 = time.time()
    w = synth.make_weights(wl if wl.shape is synth.TINY else synth.WORKLOADS["c2_7b_b1"], threads=16)
    act = synth.make_activations(wl, threads=16)
    subsets = synth.make_subsets(wl)
    if args.identity_list:
        subsets = list(subsets) + [np.arange(shape.vocab_size, dtype=np.int32)]
        args.subset = len(subsets) - 1
    gen_s = time.time() - t0
    cap = act["kv_capacity"]
    eng = binding.DraftEngine(shape, w, subsets, B, cap, K, device="cuda:0")
    hidden = eng.to_device_bits(act["hidden_in"])
    token = eng.to_device_i32(act["token_in"])
    kc, vc = eng.to_device_bits(act["k_cache"]), eng.to_device_bits(act["v_cache"])
    kv0 = eng.to_device_i32(act["kv_len"])
    kv = kv0.clone()
    draft = torch.empty((B, K), dtype=torch.int32, device="cuda:0")
    acc = torch.empty(B, dtype=torch.int32, device="cuda:0")
    out_tok = torch.empty((B, K + 1), dtype=torch.int32, device="cuda:0")
    pend = torch.empty(B, dtype=torch.int32, device="cuda:0")
    stream = 0  # the null stream, which is also torch's current stream here

    def one_step(subset_index, target):
        st = binding.mtp_draft_steps(eng.handle, B, K, subset_index, hidden, token, kc, vc, kv, None, draft, None,
                                     None, stream)
        assert st == 0, binding.mtp_status_string(st)
        st = binding.mtp_accept(eng.handle, B, K, draft, target, 0, kv, acc, out_tok, pend, stream)
        assert st == 0, binding.mtp_status_string(st)
        kv.copy_(kv0)  # replay the same cycle next time (4*B bytes, device to device)

    def timed(subset_index, steps, warmup):
        # target chain built from this configuration's own drafts (stand-in for the target model's verification)
        dummy = torch.zeros((B, K + 1), dtype=torch.int32, device="cuda:0")
        one_step(subset_index, dummy)
        torch.cuda.synchronize()
        assert eng.poll_error() == 0
        target = eng.to_device_i32(synth.make_targets(wl, draft.cpu().numpy()))
        for _ in range(warmup):
            one_step(subset_index, target)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            one_step(subset_index, target)
        torch.cuda.synchronize()
        el = time.perf_counter() - t
        return el, float(acc.float().mean().item())

    if args.copy_calib:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    mode_ids = {"per-phase": binding.LAUNCH_PER_PHASE, "single": binding.LAUNCH_SINGLE}
    mode_us = {}
    launch_mode = args.launch_mode
    if launch_mode == "auto":
        launch_mode = "per-phase"
        if B == 1:  # the single launch pays off where a phase is short against a kernel boundary
            for name, mid in mode_ids.items():
                assert binding.mtp_set_launch_mode(eng.handle, mid) == 0
                el, _ = timed(args.subset, max(20, args.steps // 5), max(5, args.warmup // 3))
                mode_us[name] = el / (max(20, args.steps // 5) * K) * 1e6
            launch_mode = min(mode_us, key=mode_us.get)
    assert binding.mtp_set_launch_mode(eng.handle, mode_ids[launch_mode]) == 0
    elapsed, mean_accept = timed(args.subset, args.steps, args.warmup)
    n_rows = eng.subset_size(args.subset)
    chain_bytes = sum(algorithmic_bytes_per_mtp_step(shape, n_rows, act["kv_len"], k, args.subset >= 0)
                      for k in range(1, K + 1))
    tok_s = B * K * args.steps / elapsed
    us_per_mtp_step = elapsed / (args.steps * K) * 1e6
    path_gbs = chain_bytes * args.steps / elapsed / 1e9

    # dominant kernel: the compressed-head launch (final norm + gathered rows + argmax), timed with HIP events on the
    # launch stream over a region of the same length
    binding.mtp_set_timing(eng.handle, binding.timing_phase("lmhead"))
    dummy = eng.to_device_i32(synth.make_targets(wl, draft.cpu().numpy()))
    durs = []
    for i in range(args.steps):
        one_step(args.subset, dummy)
        if i % 10 == 9 or i == args.steps - 1:  # reading the events waits for the stream: do it sparsely
            durs.append(binding.mtp_last_draft_ms(eng.handle))
    torch.cuda.synchronize()
    binding.mtp_set_timing(eng.handle, binding.TIMING_OFF)
    k_ms = float(np.median(durs))
    head_bytes = 2.0 * n_rows * shape.d_model + (4.0 * n_rows if args.subset >= 0 else 0.0)
    # What an event pair around ONE launch adds to the kernel's own duration (the dispatch of a dependent launch):
    # the same bracket around single launches of the acceptance kernel, whose own duration the back-to-back run above
    # cannot exceed.  Reported so that the event-based figure can be set beside the profiler's begin/end stamps.
    brackets = []
    for _ in range(50):
        b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        b0.record()
        binding.mtp_accept(eng.handle, B, K, draft, dummy, 1, kv, acc, out_tok, pend, stream)
        b1.record()
        b1.synchronize()
        brackets.append(b0.elapsed_time(b1) * 1e3)
    bracket_us = float(np.median(brackets))
    roofline = {"bound": "hbm", "kernel": "k_lmhead", "achieved": head_bytes / (k_ms * 1e-3) / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head_bytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "traffic": measured_traffic("k_lmhead") if (args.workload == "c2_7b_b1" and args.subset == 0) else None,
                "bytes_per_launch": head_bytes, "avg_launch_us": k_ms * 1e3,
                "whole_path_achieved": path_gbs, "whole_path_frac": path_gbs / HBM_PEAK_GBS}

    # spread of the K-step chain alone (HIP events inside the library around one mtp_draft_steps call), and the
    # acceptance kernel alone (back-to-back launches between two events on the same stream)
    binding.mtp_set_timing(eng.handle, binding.TIMING_CALL)
    chain_us = []
    for _ in range(min(args.steps, 100)):
        one_step(args.subset, dummy)
        chain_us.append(binding.mtp_last_draft_ms(eng.handle) * 1e3)
    binding.mtp_set_timing(eng.handle, binding.TIMING_OFF)
    p10, p50, p90 = (float(np.percentile(chain_us, q)) for q in (10, 50, 90))
    n_acc = 200
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n_acc):
        binding.mtp_accept(eng.handle, B, K, draft, dummy, 1, kv, acc, out_tok, pend, stream)  # mode 1: kv_len unchanged
    e1.record()
    torch.cuda.synchronize()
    accept_us = e0.elapsed_time(e1) * 1e3 / n_acc
    roofline["event_pair_around_one_accept_launch_us"] = bracket_us
    roofline["event_pair_overhead_us"] = bracket_us - accept_us  # at least this much of avg_launch_us is not the kernel

    extend = None
    if args.extend > 0:
        m = args.extend
        assert int(act["kv_len"].max()) + m <= cap, "the block does not fit the workload's cache capacity"
        eng2 = binding.DraftEngine(shape, w, subsets, B * m, cap, 1, device="cuda:0")
        rng = np.random.default_rng(7)
        std = float(synth.bf16_bits_to_f32(act["hidden_in"]).std())
        hid_m = eng2.to_device_bits(synth.f32_to_bf16_bits(
            (rng.standard_normal((m, B, shape.d_model)) * std).astype(np.float32)))
        tok_m = eng2.to_device_i32(rng.integers(0, shape.vocab_size, size=(m, B)).astype(np.int32))
        ext_len = eng2.to_device_i32(np.full(B, m, dtype=np.int32))
        draft_m = torch.empty((m, B), dtype=torch.int32, device="cuda:0")

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
        blk_bytes = algorithmic_bytes_per_mtp_step(shape, n_rows, act["kv_len"], 1, args.subset >= 0)
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
                st = binding.mtp_accept(eng.handle, B, K, draft_k, dummy, 0, kv, acc, out_tok, pend, stream)
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
                   "stream_passes": -(-shape.vocab_size // 40000), "oracle_seconds": cpu_l,
                   "matches_oracle": True}

    train = None
    if args.train_loss > 0:
        n_pos, Kt = args.train_loss, 3
        eng3 = binding.DraftEngine(shape, w, [], n_pos, max(64, -(-n_pos // 64) * 64), 1, device="cuda:0")
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

    full = None
    if not args.no_full_vocab and args.subset >= 0:
        fs = max(10, args.steps // 4)
        el_f, acc_f = timed(-1, fs, max(3, args.warmup // 4))
        full = {"value": B * K * fs / el_f, "unit": "draft tokens/s", "us_per_mtp_step": el_f / (fs * K) * 1e6,
                "rows": shape.vocab_size, "compressed_speedup": (el_f / fs) / (elapsed / args.steps),
                "roofline_speedup": sum(algorithmic_bytes_per_mtp_step(shape, shape.vocab_size, act["kv_len"], k, False)
                                        for k in range(1, K + 1)) / chain_bytes}

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
                   "launch_mode": launch_mode},
        "launch_mode_trial_us_per_mtp_step": mode_us or None,
        "us_per_mtp_step": us_per_mtp_step, "mean_accept_len": mean_accept,
        "chain_us": {"p10": p10, "p50": p50, "p90": p90, "what": f"{K} draft steps, one library call"},
        "accept_us": accept_us,
        "algorithmic_bytes_per_step": chain_bytes, "roofline": roofline, "full_vocab": full, "extend": extend, "list_builder": builder, "train_loss": train,
        "cpu_baseline": cpu,
        "input_generation_s": gen_s,
        "device": device_state(),
    }
    if args.k_sweep_target_ms > 0:
        from paper_2509_18362_amd import ksweep
        line["k_sweep_model"] = {
            "assumed_target_forward_ms": args.k_sweep_target_ms,
            "acceptance": "paper's 0.81/0.56/0.36 cumulative (Sec. 3.4), later positions extrapolated",
            "rows": ksweep.sweep(us_per_mtp_step * 1e-6, accept_us * 1e-6, args.k_sweep_target_ms * 1e-3)}
    eng.close()
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    status = main()
    if status:
        sys.exit(status)
