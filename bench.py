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
steps (after ``--warmup`` untimed ones; before those, untimed steps for ``--settle-ms`` let the
clocks ramp, reported as ``clock_settle``).  ``roofline`` prices the step's kernel against the 8 TB/s HBM peak from its algorithmic
bytes and its average duration, measured with HIP events (on the stream the kernel is
launched on) over the timed region.  ``select_alone`` times ``lshe_decode_select`` (hash,
score, argmax, overwrite -- no attention) over the same steps: eviction scores per second
outside the fused step.  ``cpu_baseline`` times the CPU oracle on a bounded sample of the same
workload on this host's cores, single-threaded and with OpenMP over units; ``parity_sample``
counts, on the first steps of every unit, the hash bits the device computed differently from
the oracle (all of which must be bits whose projection is within 1e-5 |x| |w| of zero).

``--workload`` selects another of the five configurations (toy, llama8b_batch32,
long_context: decode steps/s; prefill: prompt tokens/s of ``lshe_prefill_compress``, with the
three stages of the call timed one by one through ``lshe_prefill_phases``).
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
INT8_MFMA_PEAK_TOPS = 5000.0                   # dense int8 matrix-core peak, 5.0 POP/s
ALU_PEAK_TLANEOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz, one 32-bit op per lane-cycle

# Counter readings that cannot be taken inside this process (rocprofv3 runs of this same
# command, summarised under profiles/).  A reading is attached to the JSON line only when the
# run is the one it was taken on: same workload with no override, same launch plan.
#   hbm_bytes: FETCH_SIZE + WRITE_SIZE per launch of the dominant kernel, scaled by what the
#   same counters read for a plain copy of known size.
PROFILED = {
    "llama8b_decode": {
        "plan": "decode_fused_solo_kernel", "hbm_bytes": 271653478 + 417792,
        "profile": "profiles/decode_fused_solo_kernel_llama8b_decode.md",
        "select_served_from": {"level": "beyond L2 on every launch (memory-side cache or HBM)",
                               "tcc_req": 61520, "tcc_hit": 39504, "tcc_miss": 22016,
                               "fetch_bytes": 2748416, "profile": "profiles/select_kernel_code_table.md"}},
    "llama8b_batch32": {
        "plan": "decode_fused_kernel", "hbm_bytes": 4347764531 + 13373747,
        "profile": "profiles/decode_kernels_batch32_long_context_toy.md",
        "select_served_from": {"level": "beyond L2 on every launch (memory-side cache or HBM)",
                               "tcc_req": 494758, "tcc_hit": 88236, "tcc_miss": 406522,
                               "fetch_bytes": 46860493, "profile": "profiles/select_kernel_code_table.md"}},
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def host_cores():
    """(physical cores, logical CPUs, CPUs this process may run on), read at run time."""
    logical = os.cpu_count() or 1
    try:
        allowed = len(os.sched_getaffinity(0))
    except AttributeError:
        allowed = logical
    phys = set()
    try:
        pid = cid = None
        for line in open("/proc/cpuinfo"):
            if line.startswith("physical id"):
                pid = line.split(":")[1].strip()
            elif line.startswith("core id"):
                cid = line.split(":")[1].strip()
            elif not line.strip():
                if pid is not None and cid is not None:
                    phys.add((pid, cid))
                pid = cid = None
        if pid is not None and cid is not None:
            phys.add((pid, cid))
    except OSError:
        pass
    return (len(phys) or logical), logical, allowed


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


def measured_copy_gbs(torch, nbytes=1 << 29, reps=4):
    """Read + write bandwidth of a plain device-to-device copy on this GPU, GB/s."""
    x = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    y = torch.empty_like(x)
    y.copy_(x)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(reps):
        y.copy_(x)
    c1.record()
    torch.cuda.synchronize()
    return 2.0 * nbytes * reps / (c0.elapsed_time(c1) * 1e-3) / 1e9


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


def select_bytes(w, W):
    """Algorithmic bytes of the select alone: the code table, the step inputs, one slot written."""
    e = 2 if w.dtype == "bf16" else 4
    d, G, Cn = w.head_dim, w.gqa_group, w.budget
    masked = 4 * Cn if (w.n_sink or w.n_recent) else 0
    return w.n_units * (Cn * W * 4 + masked + (G + 2) * d * e + 2 * d * e + W * 4 + 4)


def bench_decode(w, args, torch, B, synth, DeviceCache, upload_workload, pristine):
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
    L = B.lib()
    cfg_ref = C.byref(dc.cfg)
    vp = C.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    ws = (vp(dc.workspace.data_ptr()), C.c_size_t(dc.workspace.numel()), stream)
    cache = (vp(dc.K.data_ptr()), vp(dc.V.data_ptr()), vp(dc.code.data_ptr()),
             vp(dc.slot_pos.data_ptr()), vp(dc.n_valid.data_ptr()))
    step_calls, select_calls = [], []
    for i in range(n_calls):
        j = i % T
        head = (cfg_ref, vp(dc.R_dev.data_ptr()), vp(qd[j].data_ptr()), vp(kd[j].data_ptr()),
                vp(vd[j].data_ptr()), vp(pos_all[i].data_ptr())) + cache
        step_calls.append(head + (vp(dc.out.data_ptr()), vp(dc.evicted.data_ptr()), None, None, None) + ws)
        select_calls.append(head + (vp(dc.evicted.data_ptr()), None, None) + ws)

    def run(fn, calls, n, what):
        for i in range(n):
            rc = fn(*calls[i])
            if rc != 0:
                raise B.LsheError(rc, what)

    def timed(fn, calls, what):
        """Warm-up, restore the post-prompt state, then exactly `steps` calls between HIP events
        (recorded on the stream the kernels run on) and host clocks."""
        run(fn, calls, args.warmup, what)
        torch.cuda.synchronize()
        dc.restore(snap)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t_wall = time.perf_counter()
        ev0.record()
        run(fn, calls, steps, what)
        ev1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t_wall) * 1e3, ev0.elapsed_time(ev1)

    # ---- let the clocks settle: the chip raises its clocks over the first ~10 ms of sustained
    # load, and a call with few warm-up steps would time the ramp instead of the kernel.  Whole
    # steps on the same cache, untimed, reported in the JSON line; the post-prompt state is
    # restored before the warm-up steps (timed() does it again after them).
    settle_steps = 0
    if args.settle_ms > 0:
        t_s = time.perf_counter()
        while (time.perf_counter() - t_s) * 1e3 < args.settle_ms:
            run(L.lshe_decode_step, step_calls, n_calls, "lshe_decode_step")
            torch.cuda.synchronize()
            settle_steps += n_calls
        dc.restore(snap)
        torch.cuda.synchronize()

    # ---- the timed region: exactly `steps` whole steps ---------------------------------------
    wall_ms, gpu_ms = timed(L.lshe_decode_step, step_calls, "lshe_decode_step")
    ms_per_step = wall_ms / steps
    evicted_after_timed = dc.evicted.clone()

    # ---- the same timed region again (state restored each time): spread of the measurement ----
    rep_ms = [gpu_ms / steps]
    for _ in range(max(args.repeats - 1, 0)):
        _, g_ms = timed(L.lshe_decode_step, step_calls, "lshe_decode_step")
        rep_ms.append(g_ms / steps)
    copy_gbs = measured_copy_gbs(torch)

    # ---- the select alone (hash + score + argmax + overwrite, no attention) --------------------
    sel_wall_ms, sel_gpu_ms = timed(L.lshe_decode_select, select_calls, "lshe_decode_select")
    same_sel = bool(torch.equal(evicted_after_timed, dc.evicted))
    sel_ms = sel_gpu_ms / steps

    # ---- the same select over a code table at one byte per hash bit (the paper's storage) --------
    unpacked = None
    if w.policy == "hash" and d == 128 and w.dtype == "bf16" and not args.no_unpacked:
        dc.restore(snap)
        shifts = torch.arange(32, device=dev, dtype=torch.int32)
        tab0 = ((dc.code.view(U, Cn, dc.W, 1) >> shifts) & 1).to(torch.uint8).reshape(U, Cn, 32 * dc.W).contiguous()
        tab, spos_u, nv_u = tab0.clone(), dc.slot_pos.clone(), dc.n_valid.clone()
        ev_u = torch.zeros_like(dc.evicted)
        ucalls = []
        for i in range(n_calls):
            j = i % T
            ucalls.append((cfg_ref, vp(dc.R_dev.data_ptr()), vp(qd[j].data_ptr()), vp(kd[j].data_ptr()),
                           vp(pos_all[i].data_ptr()), vp(tab.data_ptr()), vp(spos_u.data_ptr()),
                           vp(nv_u.data_ptr()), vp(ev_u.data_ptr()), stream))
        run(L.lshe_decode_select_unpacked, ucalls, args.warmup, "lshe_decode_select_unpacked")
        torch.cuda.synchronize()
        tab.copy_(tab0); spos_u.copy_(snap[3]); nv_u.copy_(snap[4])
        u0, u1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        u0.record()
        run(L.lshe_decode_select_unpacked, ucalls, steps, "lshe_decode_select_unpacked")
        u1.record()
        torch.cuda.synchronize()
        ums = u0.elapsed_time(u1) / steps
        unpacked = {"call": "lshe_decode_select_unpacked", "ms": ums,
                    "code_table_bytes": int(tab.numel()),
                    "eviction_scores_per_sec": U * Cn / (ums * 1e-3),
                    "same_evictions_as_the_packed_select": bool(torch.equal(ev_u, evicted_after_timed)),
                    "packed_select_ms": sel_ms, "slowdown_vs_packed": ums / sel_ms}
        del tab, tab0

    # ---- second pass over the same steps with a HIP event pair around every launch ------------
    # (cross-check of the per-kernel time, and of determinism: same victims as the timed pass)
    dc.restore(snap)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(steps)]
    for i in range(steps):
        a, b = evs[i]
        a.record()
        run(L.lshe_decode_step, step_calls[i:i + 1], 1, "lshe_decode_step")
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
    plan = B.lshe_decode_plan(dc.cfg)
    prof = PROFILED.get(w.name) if pristine else None
    if prof is not None and prof["plan"] != plan:
        prof = None          # the kernels changed since the counters were read: say nothing

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
    cpu, parity = None, None
    if args.cpu_steps > 0 and w.policy == "hash":
        import oracle
        dc.restore(snap)
        torch.cuda.synchronize()
        R = dc.projection_host()
        phys, logical, allowed = host_cores()
        n_thr = min(oracle.max_threads(), allowed)
        us = min(U, args.cpu_units)         # leading units only when the workload is huge
        state = (dc.K[:us].float().cpu().numpy(), dc.V[:us].float().cpu().numpy(),
                 np.ascontiguousarray(dc.code[:us].cpu().numpy().view(np.uint32)),
                 dc.slot_pos[:us].cpu().numpy(), dc.n_valid[:us].cpu().numpy())
        ns = min(args.cpu_steps, T)
        qh = qd[:ns, :us].float().cpu().numpy()
        kh = kd[:ns, :us].float().cpu().numpy()
        vh = vd[:ns, :us].float().cpu().numpy()

        def oracle_leg(n_steps, threads):
            Kh, Vh, ch, ph, nvh = (x.copy() for x in state)
            t1 = time.perf_counter()
            for i in range(n_steps):
                oracle.decode_step_units(Kh, Vh, ch, ph, nvh, R, qh[i], kh[i], vh[i],
                                         np.full(us, N + i, np.int32), G, w.hash_bits,
                                         w.n_sink, w.n_recent, n_threads=threads)
            return n_steps / (time.perf_counter() - t1) * us / U

        ns1 = max(1, ns // 8)
        v_omp = oracle_leg(ns, n_thr)
        v_one = oracle_leg(ns1, 1)
        cpu = {"value": v_omp, "unit": "steps/s", "cores": n_thr, "kind": "oracle",
               "sample": "first %d decode steps of %d of %d units (plain C, fp64, OpenMP over "
                         "units), scaled to all units" % (ns, us, U),
               "single_thread": {"value": v_one, "unit": "steps/s", "cores": 1,
                                 "sample": "first %d decode steps of the same units" % ns1},
               "host": {"physical_cores": phys, "logical_cpus": logical, "cpus_allowed": allowed}}

        # ---- lock-step sample: the device's hash codes of the first steps against the oracle's --
        np_steps = min(8, T)
        dc.restore(snap)
        cdbg = torch.zeros((np_steps, U, G + 1, dc.W), dtype=torch.int32, device=dev)
        for i in range(np_steps):
            dc.decode_step(qd[i], kd[i], vd[i], pos_all[i], codes_dbg=cdbg[i])
        torch.cuda.synchronize()
        X = torch.cat([qd[:np_steps], kd[:np_steps].unsqueeze(2)], dim=2).float().cpu().numpy()
        ref, margin = oracle.hash_codes(X.reshape(-1, d), R, with_margin=True)
        diff = cdbg.cpu().numpy().view(np.uint32).reshape(ref.shape) ^ ref
        flagged = unexplained = 0
        for i, wd in zip(*np.nonzero(diff)):
            for b in range(32):
                if (int(diff[i, wd]) >> b) & 1:
                    if wd * 32 + b < w.hash_bits and margin[i, wd * 32 + b] < 1e-5:
                        flagged += 1
                    else:
                        unexplained += 1
        parity = {"hashed_bits": int(ref.shape[0]) * w.hash_bits, "flagged_bits": flagged,
                  "unexplained_bits": unexplained,
                  "sample": "query and key codes of the first %d decode steps of all %d units "
                            "against the oracle's (flagged: projection within 1e-5 |x||w| of zero)"
                            % (np_steps, U)}

    return {
        "metric": "decode_steps_per_sec",
        "value": steps / (wall_ms * 1e-3),
        "unit": "steps/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "clock_settle": {"ms": args.settle_ms, "steps": settle_steps,
                         "what": "untimed whole steps before the warm-up steps, state restored after"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": config_name(w), "units": U, "tokens_per_step": w.batch},
        "eviction_scores_per_sec": U * Cn * steps / (wall_ms * 1e-3),
        "step_algorithmic_gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "gpu_ms_per_step_events": gpu_ms / steps,
        "repeats": {"n": len(rep_ms), "median_ms_per_step": float(np.median(rep_ms)),
                    "min_ms_per_step": float(np.min(rep_ms)), "max_ms_per_step": float(np.max(rep_ms)),
                    "what": "HIP-event time per step of the timed region, run n times from the same state "
                            "(value and roofline are the first run's)"},
        "select_alone": {
            "call": "lshe_decode_select", "ms": sel_ms, "wall_ms": sel_wall_ms / steps,
            "eviction_scores_per_sec": U * Cn / (sel_ms * 1e-3),
            "algorithmic_bytes": select_bytes(w, dc.W),
            "gbs": select_bytes(w, dc.W) / (sel_ms * 1e-3) / 1e9,
            "code_table_bytes": B.lshe_code_cache_bytes(dc.cfg),
            "same_evictions_as_the_fused_step": same_sel,
            "served_from": prof["select_served_from"] if prof else None},
        "select_alone_one_byte_per_hash_bit": unpacked,
        "prefill_ms": prefill_ms,
        "prefill_tokens_per_sec": w.batch * N / (prefill_ms * 1e-3),
        "hash_bits": w.hash_bits, "policy": w.policy,
        "code_cache_bytes_packed": B.lshe_code_cache_bytes(dc.cfg),
        "code_cache_bytes_at_8_bits_per_bit": U * Cn * w.hash_bits,
        "per_launch_event_ms": per_launch_ms,
        "instrumented_pass_same_evictions": same,
        "attention_loss": loss,
        "roofline": {"kernel": plan, "bound": "hbm", "achieved": kern_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kern_gbs / HBM_PEAK_GBS,
                     "traffic": prof["hbm_bytes"] if prof else None,
                     "traffic_source": ({"profile": prof["profile"], "plan": prof["plan"]}
                                        if prof else None),
                     "avg_kernel_ms": kern_ms, "algorithmic_bytes": step_bytes,
                     "measured_copy_gbs": copy_gbs,
                     "frac_of_measured_copy": kern_gbs / copy_gbs,
                     "copy_what": "read + write rate of a plain 512 MiB device-to-device copy in this run"},
        "cpu_baseline": cpu,
        "parity_sample": parity,
    }


def bench_prefill(w, args, torch, B, synth, DeviceCache, upload_workload, pristine):
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

    # ---- the three stages one by one, HIP events between them (same kernels, same stream) -----
    names = ("hash", "evict", "gather")
    bits = (B.LSHE_PREFILL_HASH, B.LSHE_PREFILL_EVICT, B.LSHE_PREFILL_GATHER)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for r in range(steps):
        evs[r][0].record()
        for j, ph in enumerate(bits):
            B.lshe_prefill_phases(dc.cfg, dc.R_dev, Kp, Vp, Qp, N, dc.K, dc.V, dc.code, dc.slot_pos,
                                  dc.n_valid, None, dc.workspace, ph)
            evs[r][j + 1].record()
    torch.cuda.synchronize()
    phase_ms = {n: float(np.mean([evs[r][j].elapsed_time(evs[r][j + 1]) for r in range(steps)]))
                for j, n in enumerate(names)}

    e = 2 if w.dtype == "bf16" else 4
    W = dc.W
    nq = max(N - Cn, 0)
    l2 = w.policy == "l2"
    hashed_rows = N + (0 if l2 else G * nq)
    hash_bytes = U * hashed_rows * (d * e + W * 4)                # rows read, codes written
    gather_bytes = U * min(N, Cn) * (2 * 2 * d * e + 2 * W * 4 + 4)   # K, V read + written, code, position
    plan = B.lshe_prefill_plan(dc.cfg, N)
    # Work of the sequential stage in the terms of the unit that executes it.  Matrix-core
    # kernel: the summed Hamming distances of a step are one row of an int8 product
    # [steps x r] . [r x slots], 2 r int8 operations per (step, slot).  Vector-ALU kernels:
    # one XOR and one popcount per (step, slot, query head, code word).
    mfma_ops = 2.0 * w.hash_bits * Cn * nq * U
    alu_ops = 2.0 * G * W * Cn * nq * U
    phases = {
        "hash": {"ms": phase_ms["hash"], "bound": "hbm", "algorithmic_bytes": hash_bytes,
                 "achieved": hash_bytes / (phase_ms["hash"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                 "unit": "GB/s", "frac": hash_bytes / (phase_ms["hash"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "matrix_core_flops": 2.0 * d * 32 * W * hashed_rows * U,
                 "matrix_core_tflops": 2.0 * d * 32 * W * hashed_rows * U / (phase_ms["hash"] * 1e-3) / 1e12},
        "gather": {"ms": phase_ms["gather"], "bound": "hbm", "algorithmic_bytes": gather_bytes,
                   "achieved": gather_bytes / (phase_ms["gather"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                   "unit": "GB/s", "frac": gather_bytes / (phase_ms["gather"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    copy_gbs = measured_copy_gbs(torch)
    for ph in phases.values():
        ph["measured_copy_gbs"] = copy_gbs          # read + write rate of a plain 512 MiB copy in this run
        ph["frac_of_measured_copy"] = ph["achieved"] / copy_gbs
    ev_s = phase_ms["evict"] * 1e-3
    if plan and "evict_mfma_kernel" in plan:
        roof = {"kernel": "evict_mfma_kernel", "bound": "mfma", "achieved": mfma_ops / ev_s / 1e12,
                "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": mfma_ops / ev_s / 1e12 / INT8_MFMA_PEAK_TOPS,
                "algorithmic_int8_ops": mfma_ops}
    elif l2:
        # the comparator's sequential stage is a chain of dependent LDS accesses (a tournament per unit):
        # no throughput roofline applies to it; the call's dominant kernel by bytes is the gather
        roof = dict(phases["gather"], kernel="gather_kernel")
    else:
        kern = "evict_lds_kernel" if plan and "evict_lds" in plan else "evict_global_kernel"
        roof = {"kernel": kern, "bound": "alu", "achieved": alu_ops / ev_s / 1e12 if nq else None,
                "peak": ALU_PEAK_TLANEOPS, "unit": "Tlaneop/s",
                "frac": alu_ops / ev_s / 1e12 / ALU_PEAK_TLANEOPS if nq else None,
                "algorithmic_lane_ops": alu_ops}
    roof.update({"traffic": None, "evict_ms": phase_ms["evict"]})
    if not l2:
        roof.update({"avg_kernel_ms": phase_ms["evict"], "xor_popcount_lane_ops": alu_ops,
                     "xor_popcount_tlaneops": alu_ops / ev_s / 1e12 if nq else None})

    cpu = None
    if args.cpu_steps > 0:
        import oracle
        from concurrent.futures import ThreadPoolExecutor
        R = dc.projection_host()
        phys, logical, allowed = host_cores()
        n_thr = max(1, min(16, allowed, U))

        def inputs(u):
            x = synth.gen_unit(w, u)
            return tuple(synth.quantize(w, x[n][..., :N, :]) for n in ("K", "V", "Q"))

        def one(kvq):
            o = oracle.UnitCache(Cn, d, w.hash_bits, G, R, w.n_sink, w.n_recent, policy=w.policy)
            o.prefill(*kvq)

        data = [inputs(u) for u in range(n_thr)]
        t1 = time.perf_counter()
        one(data[0])
        one_s = time.perf_counter() - t1
        t1 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=n_thr) as ex:
            list(ex.map(one, data))
        par_s = time.perf_counter() - t1
        cpu = {"value": w.batch * N / (par_s * U / n_thr), "unit": "tokens/s", "cores": n_thr,
               "kind": "oracle",
               "sample": "prompt stage of %d of %d units, one thread each (plain C, fp64), scaled to "
                         "all units" % (n_thr, U),
               "single_thread": {"value": w.batch * N / (one_s * U), "unit": "tokens/s", "cores": 1,
                                 "sample": "prompt stage of 1 unit"},
               "host": {"physical_cores": phys, "logical_cpus": logical, "cpus_allowed": allowed}}
    return {
        "metric": "prefill_prompt_tokens_per_sec",
        "value": w.batch * N / (ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": config_name(w), "units": U, "tokens_per_step": w.batch * N},
        "plan": plan,
        # The dominant kernel is the sequential eviction; its work is priced in the terms of the
        # unit that executes it (int8 matrix-core operations, or vector lane operations for the
        # kernels that score with XOR + popcount), over its own duration measured in this run.
        "roofline": roof,
        "phases": phases,
        "phases_sum_ms": sum(phase_ms.values()),
        "cpu_baseline": cpu,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0,
                    help="timed steps (default: the workload's own count, 256 for the default)")
    ap.add_argument("--warmup", type=int, default=256,
                    help="untimed warm-up steps (a full pass, ~13 ms, also lets the clocks ramp)")
    ap.add_argument("--settle-ms", type=float, default=25.0,
                    help="run untimed decode steps for this long before the warm-up steps so that the "
                         "clocks have ramped (0 = off)")
    ap.add_argument("--repeats", type=int, default=5,
                    help="how many times the timed region is run in all (spread reported as `repeats`)")
    ap.add_argument("--workload", default="llama8b_decode")
    ap.add_argument("--cpu-steps", type=int, default=128,
                    help="decode steps the CPU oracle is timed on with OpenMP (an eighth of them "
                         "single-threaded; 0 = skip the CPU legs)")
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
    ap.add_argument("--query-corr", type=float, default=0.0,
                    help="weight of a component shared by all queries of a unit (synth.Workload.query_corr): "
                         "correlated queries, the stress case of the prompt stage's matrix-core kernel")
    ap.add_argument("--attention-loss", action="store_true",
                    help="also run the decode steps once with the evicted_mass output and report the "
                         "mean attention probability of the evicted tokens (Section 4.8, per step)")
    ap.add_argument("--no-unpacked", action="store_true",
                    help="skip the select over a code table at one byte per hash bit (the paper's storage, "
                         "Sections 4.6-4.7), which is timed beside the packed one for comparison")
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
    pristine = not (args.hash_bits or args.policy != "hash" or args.scale or args.kept or args.query_corr)
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
    if args.query_corr:
        w = w.scaled(query_corr=args.query_corr, name="%s_corr%g" % (w.name, args.query_corr))
    fn = bench_decode if w.n_decode > 0 else bench_prefill
    print(json.dumps(fn(w, args, torch, B, synth, DeviceCache, upload_workload, pristine)), flush=True)


if __name__ == "__main__":
    main()
