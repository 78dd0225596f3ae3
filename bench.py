#!/usr/bin/env python3
"""Benchmark of the HashEvict hot path on one MI355X.

Default (what the driver runs): the Llama-3-8B-shaped decode configuration -- batch 1,
32 layers x 8 KV heads, GQA 4, head_dim 128, bf16, r = 32, 4096-token prompt compressed to
2048 slots by ``lshe_prefill_compress``, then decode.  A *step* is one pass of the whole path
-- hash, Hamming score, select, in-place overwrite, decode attention -- for every (sequence,
layer, KV head) unit: one ``lshe_decode_step`` call (a single kernel for this workload).
All inputs are synthetic (``paper_2412_16187_amd/synth.py``) and resident in HBM before the
timed region starts.

Prints ONE JSON line.  ``value`` is decode steps per second over exactly ``--steps`` timed
steps.  ``roofline`` prices the step's kernel against the 8 TB/s HBM peak from its algorithmic
bytes and its average duration, measured with HIP events (on the stream the kernel is
launched on) over the timed region.  ``cpu_baseline`` times the
CPU oracle on a bounded sample of the same workload on this host's cores.

``--workload`` selects another of the five configurations (toy, llama8b_batch32,
long_context: decode steps/s; prefill: prompt tokens/s of ``lshe_prefill_compress``).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ALU_PEAK_TLANEOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz, one 32-bit op per lane-cycle
# HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE counters
# (separate profiling runs, see profiles/); None until measured for a workload.
# evict_mfma_kernel on the prefill workload: vector instructions per launch (SQ_INSTS_VALU) and
# the kernel's duration in the same profile (profiles/prefill_kernels_prefill_workload.md)
PREFILL_VALU_INSTS = {"prefill": 1.536e9}
PREFILL_EVICT_MS = {"prefill": 4.216}
TRAFFIC = {"llama8b_decode": 278355149 + 417792, "llama8b_batch32": 4347973290 + 13376496}   # profiles/decode_fused_solo_kernel_llama8b_decode.md


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def copy_calibration(torch):
    x = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    y = torch.empty_like(x)
    y.copy_(x)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(8):
        y.copy_(x)
    c1.record()
    torch.cuda.synchronize()
    ms = c0.elapsed_time(c1) / 8
    print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30,
                      "ms_per_copy": ms, "GBps_read_plus_write": 2 * (1 << 30) / ms / 1e6}))


def config_name(w):
    return ("%s: B%d L%d H%d G%d d%d %s r%d, prompt %d -> budget %d, %d decode steps"
            % (w.name, w.batch, w.n_layers, w.n_kv_heads, w.gqa_group, w.head_dim, w.dtype,
               w.hash_bits, w.n_prompt, w.budget, w.n_decode))


def decode_step_bytes(w, W):
    """Algorithmic bytes of one decode step: per unit, K and V slots read once, the code table
    read once, q/k/v in and out written, one slot (K, V, code, position) written."""
    e = 2 if w.dtype == "bf16" else 4
    d, G, Cn = w.head_dim, w.gqa_group, w.budget
    return w.n_units * (2 * Cn * d * e + Cn * W * 4 + (2 * G + 2) * d * e + 2 * d * e + W * 4 + 4)


def prefill_bytes(w, W):
    """Algorithmic bytes of one prompt compression: keys and the queries of tokens >= C read
    once for hashing, codes written and read back once, survivors' K/V gathered (read + write)."""
    e = 2 if w.dtype == "bf16" else 4
    d, G, Cn, N = w.head_dim, w.gqa_group, w.budget, w.n_prompt
    nq = max(N - Cn, 0)
    hash_b = (N + G * nq) * d * e
    codes_b = 2 * (N + G * nq) * W * 4
    gather_b = 2 * 2 * min(N, Cn) * d * e
    return w.n_units * (hash_b + codes_b + gather_b)


def bench_decode(w, args, torch, B, synth, DeviceCache, upload_workload):
    dev = torch.device("cuda:0")
    U, N, T, G, d, Cn = w.n_units, w.n_prompt, w.n_decode, w.gqa_group, w.head_dim, w.budget
    steps = args.steps if args.steps > 0 else T
    t0 = time.time()
    Kp, Vp, Qp, kd, vd, qd = upload_workload(w, threads=args.gen_threads)
    torch.cuda.synchronize()
    log("inputs generated and uploaded in %.1f s" % (time.time() - t0))

    dc = DeviceCache(w.batch, w.n_layers, w.n_kv_heads, G, d, w.hash_bits, Cn, w.dtype,
                     w.n_sink, w.n_recent, n_prompt_max=N, policy=w.policy)
    dc.init_projection(synth.projection(w))

    # ---- prompt compression (set-up for the decode loop; timed for the record) --------------
    dc.prefill(Kp, Vp, Qp, N)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    dc.prefill(Kp, Vp, Qp, N)
    e1.record()
    torch.cuda.synchronize()
    prefill_ms = e0.elapsed_time(e1)
    snap = dc.snapshot()
    del Kp, Vp, Qp

    n_calls = steps + args.warmup
    pos_all = torch.arange(N, N + n_calls + 1, dtype=torch.int32,
                           device=dev).repeat_interleave(w.batch).view(-1, w.batch)

    # Argument tuples are built once so that the timed loop is one foreign call per step.
    fn = B.lib().lshe_decode_step
    cfg_ref = C.byref(dc.cfg)
    vp = C.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    fixed_tail = (vp(dc.K.data_ptr()), vp(dc.V.data_ptr()), vp(dc.code.data_ptr()),
                  vp(dc.slot_pos.data_ptr()), vp(dc.n_valid.data_ptr()), vp(dc.out.data_ptr()),
                  vp(dc.evicted.data_ptr()), None, None, None, vp(dc.workspace.data_ptr()),
                  C.c_size_t(dc.workspace.numel()), stream)
    calls = []
    for i in range(n_calls):
        j = i % T
        calls.append((cfg_ref, vp(dc.R_dev.data_ptr()), vp(qd[j].data_ptr()), vp(kd[j].data_ptr()),
                      vp(vd[j].data_ptr()), vp(pos_all[i].data_ptr())) + fixed_tail)

    def step(i):
        rc = fn(*calls[i])
        if rc != 0:
            raise B.LsheError(rc, "lshe_decode_step")

    # ---- warm-up, then restore the post-prefill state ---------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    dc.restore(snap)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps ------------------------------------------------
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_wall = time.perf_counter()
    ev0.record()
    for i in range(steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall_ms / steps
    evicted_after_timed = dc.evicted.clone()

    # ---- second pass over the same steps with a HIP event pair around every launch ------------
    # (cross-check of the per-kernel time, and of determinism: same victims as the timed pass)
    dc.restore(snap)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(steps)]
    for i in range(steps):
        a, b = evs[i]
        a.record()
        step(i)
        b.record()
    torch.cuda.synchronize()
    per_launch_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    same = bool(torch.equal(evicted_after_timed, dc.evicted))

    # Average kernel duration: HIP events around the timed region / steps.  With one kernel per
    # step launched back to back there is no gap between kernels (rocprofv3's kernel trace
    # shows end(i) == start(i+1)), so this is the kernel's average duration; event pairs around
    # single launches (per_launch_ms) add about 4 us of event overhead each and are kept only as
    # a cross-check.
    kern_ms = gpu_ms / steps
    step_bytes = decode_step_bytes(w, dc.W)
    kern_gbs = step_bytes / (kern_ms * 1e-3) / 1e9
    kernel = B.lshe_decode_plan(dc.cfg)

    # ---- optional: Section 4.8's attention loss per step (mass on the evicted token) ----------
    loss = None
    if args.attention_loss:
        dc.restore(snap)
        mass = torch.zeros((min(T, steps), U, G), dtype=torch.float32, device=dev)
        for i in range(mass.shape[0]):
            dc.decode_step(qd[i], kd[i], vd[i], pos_all[i], evicted_mass=mass[i])
        torch.cuda.synchronize()
        loss = {"mean_evicted_mass": float(mass.mean()), "max_evicted_mass": float(mass.max()),
                "steps": int(mass.shape[0])}

    # ---- CPU oracle on a bounded sample of the same workload ---------------------------------
    cpu = None
    if args.cpu_steps > 0 and w.policy == "hash":
        import oracle
        dc.restore(snap)
        torch.cuda.synchronize()
        R = dc.projection_host()
        n_thr = oracle.max_threads()
        us = min(U, args.cpu_units)         # leading units only when the workload is huge
        Kh = dc.K[:us].float().cpu().numpy()
        Vh = dc.V[:us].float().cpu().numpy()
        ch = np.ascontiguousarray(dc.code[:us].cpu().numpy().view(np.uint32))
        ph = dc.slot_pos[:us].cpu().numpy().copy()
        nvh = dc.n_valid[:us].cpu().numpy().copy()
        ns = min(args.cpu_steps, T)
        qh = qd[:ns, :us].float().cpu().numpy()
        kh = kd[:ns, :us].float().cpu().numpy()
        vh = vd[:ns, :us].float().cpu().numpy()
        t1 = time.perf_counter()
        for i in range(ns):
            oracle.decode_step_units(Kh, Vh, ch, ph, nvh, R, qh[i], kh[i], vh[i],
                                     np.full(us, N + i, np.int32), G, w.hash_bits,
                                     w.n_sink, w.n_recent, n_threads=n_thr)
        cpu_s = time.perf_counter() - t1
        cpu = {"value": ns / cpu_s * us / U, "unit": "steps/s", "cores": n_thr, "kind": "oracle",
               "sample": "first %d decode steps of %d of %d units (plain C, fp64, OpenMP over "
                         "units), scaled to all units" % (ns, us, U)}

    return {
        "metric": "decode_steps_per_sec",
        "value": steps / (wall_ms * 1e-3),
        "unit": "steps/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": config_name(w), "units": U, "tokens_per_step": w.batch},
        "eviction_scores_per_sec": U * Cn * steps / (wall_ms * 1e-3),
        "step_algorithmic_gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "gpu_ms_per_step_events": gpu_ms / steps,
        "prefill_ms": prefill_ms,
        "prefill_tokens_per_sec": w.batch * N / (prefill_ms * 1e-3),
        "hash_bits": w.hash_bits, "policy": w.policy,
        "code_cache_bytes_packed": B.lshe_code_cache_bytes(dc.cfg),
        "code_cache_bytes_at_8_bits_per_bit": U * Cn * w.hash_bits,
        "per_launch_event_ms": per_launch_ms,
        "instrumented_pass_same_evictions": same,
        "attention_loss": loss,
        "roofline": {"kernel": kernel, "bound": "hbm", "achieved": kern_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kern_gbs / HBM_PEAK_GBS,
                     "traffic": TRAFFIC.get(w.name), "avg_kernel_ms": kern_ms,
                     "algorithmic_bytes": step_bytes},
        "cpu_baseline": cpu,
    }


def bench_prefill(w, args, torch, B, synth, DeviceCache, upload_workload):
    U, N, G, d, Cn = w.n_units, w.n_prompt, w.gqa_group, w.head_dim, w.budget
    steps = args.steps if args.steps > 0 else 8
    t0 = time.time()
    Kp, Vp, Qp, _, _, _ = upload_workload(w, threads=args.gen_threads)
    torch.cuda.synchronize()
    log("inputs generated and uploaded in %.1f s" % (time.time() - t0))
    dc = DeviceCache(w.batch, w.n_layers, w.n_kv_heads, G, d, w.hash_bits, Cn, w.dtype,
                     w.n_sink, w.n_recent, n_prompt_max=N, policy=w.policy)
    dc.init_projection(synth.projection(w))
    warm = max(1, min(args.warmup, 3))
    for _ in range(warm):
        dc.prefill(Kp, Vp, Qp, N)
    torch.cuda.synchronize()
    t_wall = time.perf_counter()
    for _ in range(steps):
        dc.prefill(Kp, Vp, Qp, N)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3
    ms = wall_ms / steps
    byts = prefill_bytes(w, dc.W)
    alu_ops = 2.0 * G * dc.W * Cn * max(N - Cn, 0) * U

    cpu = None
    if args.cpu_steps > 0:
        import oracle
        R = dc.projection_host()
        us = min(U, 4)
        t1 = time.perf_counter()
        for u in range(us):
            x = synth.gen_unit(w, u)
            o = oracle.UnitCache(Cn, d, w.hash_bits, G, R, w.n_sink, w.n_recent)
            o.prefill(synth.quantize(w, x["K"][:N]), synth.quantize(w, x["V"][:N]),
                      synth.quantize(w, x["Q"][:, :N]))
        cpu_s = time.perf_counter() - t1
        cpu = {"value": w.batch * N / (cpu_s * U / us), "unit": "tokens/s", "cores": 1,
               "kind": "oracle",
               "sample": "prompt stage of %d of %d units, single thread (incl. input generation), "
                         "scaled to all units" % (us, U)}
    return {
        "metric": "prefill_prompt_tokens_per_sec",
        "value": w.batch * N / (ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": config_name(w), "units": U, "tokens_per_step": w.batch * N},
        # The prompt stage is dominated by the sequential eviction (about two thirds of the
        # call), which is bound by the vector ALUs: the scores come from i8 MFMA (8 % busy), the
        # vector instructions unpack bits into MFMA operands and keep the running argmax.
        # `achieved` = vector lane-operations the eviction kernel issues per launch
        # (SQ_INSTS_VALU x 64, counted by rocprofv3 on this workload, see profiles/) divided by
        # the time of the WHOLE call measured here; against the kernel's own profiled duration
        # the same count gives `frac_of_kernel_time`.  The method's own arithmetic -- one XOR and
        # one popcount per (slot, step, query head, code word) -- is reported as a rate too.
        "roofline": {"kernel": "evict_mfma_kernel (rate over the whole lshe_prefill_compress call)",
                     "bound": "alu",
                     "achieved": (PREFILL_VALU_INSTS.get(w.name, 0) * 64 / (ms * 1e-3) / 1e12
                                  if w.name in PREFILL_VALU_INSTS and w.policy == "hash" else None),
                     "peak": ALU_PEAK_TLANEOPS, "unit": "Tlaneop/s",
                     "frac": (PREFILL_VALU_INSTS[w.name] * 64 / (ms * 1e-3) / 1e12 / ALU_PEAK_TLANEOPS
                              if w.name in PREFILL_VALU_INSTS and w.policy == "hash" else None),
                     "traffic": None,
                     "avg_call_ms": ms,
                     "frac_of_kernel_time": (PREFILL_VALU_INSTS[w.name] * 64 / (PREFILL_EVICT_MS[w.name] * 1e-3)
                                             / 1e12 / ALU_PEAK_TLANEOPS
                                             if w.name in PREFILL_VALU_INSTS and w.policy == "hash" else None),
                     "algorithmic_xor_popcount_lane_ops": alu_ops,
                     "algorithmic_tlaneops_over_whole_call": alu_ops / (ms * 1e-3) / 1e12,
                     "hbm_algorithmic_bytes": byts,
                     "hbm_gbs_over_whole_call": byts / (ms * 1e-3) / 1e9},
        "cpu_baseline": cpu,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0,
                    help="timed steps (default: the workload's own count, 256 for the default)")
    ap.add_argument("--warmup", type=int, default=256,
                    help="untimed warm-up steps (a full pass, ~13 ms, also lets the clocks ramp)")
    ap.add_argument("--workload", default="llama8b_decode")
    ap.add_argument("--cpu-steps", type=int, default=8,
                    help="decode steps the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--cpu-units", type=int, default=256,
                    help="at most this many leading units are given to the CPU oracle")
    ap.add_argument("--gen-threads", type=int, default=min(16, os.cpu_count() or 1))
    ap.add_argument("--hash-bits", type=int, default=0,
                    help="override the workload's hash width r (sweep of Section 4.7 / Appendix B: "
                         "4, 8, 16, 24, 32, 64)")
    ap.add_argument("--policy", choices=("hash", "l2"), default="hash",
                    help="hash = HashEvict; l2 = the L2-norm comparator the paper measures against "
                         "(same slots and attention, victim = largest key norm)")
    ap.add_argument("--scale", default="",
                    help="override fields of the workload, e.g. n_layers=1,batch=8 (one layer's call) or "
                         "gqa_group=8,n_layers=80; integers only")
    ap.add_argument("--kept", default="",
                    help="always-kept tokens as n_sink,n_recent (the paper's experiments keep the first "
                         "4 and the last 10: --kept 4,10; the benchmark configurations keep none)")
    ap.add_argument("--attention-loss", action="store_true",
                    help="also run the decode steps once with the evicted_mass output and report the "
                         "mean attention probability of the evicted tokens (Section 4.8, per step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy 8 times (known HBM bytes: 1 GiB read "
                         "+ 1 GiB written per launch) so that rocprofv3 FETCH_SIZE / WRITE_SIZE "
                         "readings can be scaled; prints the achieved copy bandwidth")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (units are independent and would shard "
                 "with no exchange, but no multi-GPU path is built); use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.copy_calibration:
        copy_calibration(torch)
        return
    from paper_2412_16187_amd import binding as B
    from paper_2412_16187_amd import synth
    from paper_2412_16187_amd.state import DeviceCache, upload_workload

    B.lib()   # fail loudly if the HIP library is missing
    w = synth.WORKLOADS[args.workload]
    if args.hash_bits:
        w = w.scaled(hash_bits=args.hash_bits, name="%s_r%d" % (w.name, args.hash_bits))
    if args.policy != "hash":
        w = w.scaled(policy=args.policy, name="%s_%s" % (w.name, args.policy))
    if args.scale:
        kv = {k: int(v) for k, v in (item.split("=") for item in args.scale.split(","))}
        w = w.scaled(name="%s[%s]" % (w.name, args.scale), **kv)
    if args.kept:
        n_sink, n_recent = (int(x) for x in args.kept.split(","))
        w = w.scaled(n_sink=n_sink, n_recent=n_recent, name="%s_kept%d_%d" % (w.name, n_sink, n_recent))
    fn = bench_decode if w.n_decode > 0 else bench_prefill
    print(json.dumps(fn(w, args, torch, B, synth, DeviceCache, upload_workload)), flush=True)


if __name__ == "__main__":
    main()
