#!/usr/bin/env python3
"""Benchmark of the denoise-step path on one MI355X.

Headline workload ("c3"): LLaDA-8B-shaped model (32 layers, d 4096, 32 heads x 128, MLP 12288, vocab 126464),
bfloat16, random-init N(0, 0.02) weights drawn on the device, batch 1, prompt of 1024 random tokens, blocks of 32,
threshold 0.9, at least 2 unmasked per step.  A "step" is one denoising forward over the in-flight block against the
cached prefix (embed .. LM head with fused confidence) followed by the unmask selection, replayed as one captured HIP
graph.  The timed region is exactly --steps such steps with everything resident in HBM (wall clock, both sides
synchronised); the block is put back to all-[MASK] (a device-side copy) whenever it would run out of masked positions.

Untimed for `value`, reported in the same JSON line:
  * per-step HIP-event times of at least 50 replays (median, minimum);
  * a pass with per-kernel HIP events for the roofline object (dominant kernel) and the per-kernel table;
  * one whole generation (prefill, 8 blocks, refresh at block boundaries) and the same with multi-block decoding;
  * "c2": one layer + LM head at prefix 512, the small HBM-bound workload;
  * "large_batch": the long-context batch-32 step (Dream-7B-shaped, prefix 8192), bound by the matrix cores;
  * "attainable": a plain stream read and a loop of nothing but matrix instructions, same run, same chip;
  * "cpu_baseline": the CPU oracle on a bounded sample, all cores and one thread.

Prints ONE JSON line.  --workload c2 | c4 | c5 makes that workload the headline instead.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0
KCLASS = {0: "qkv", 1: "wo", 2: "gate_up", 3: "down", 4: "lm_head", 5: "attention"}


def event_times_ms(torch, fn, n):
    """Per-iteration durations of fn(i), i < n, from events on the current stream (the one the library launches on)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record()
    for i in range(n):
        fn(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]


def pmc_traffic(profile_name, key):
    """HBM bytes per launch of a kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE scaled by
    a plain copy of known size; measured with the commands that file lists, not in this run), or None."""
    path = os.path.join(ROOT, "profiles", profile_name)
    if os.path.exists(path):
        for line in open(path):
            if line.startswith(f"traffic_bytes_per_launch {key}:"):
                return float(line.split(":")[1])
    return None


# ----------------------------------------------------------------------------------------------- CPU oracle baseline

def cpu_baseline(ms, P, Q, n_masked, budget_s=24.0):
    """The CPU oracle as it stands, timed on the host on the workload's shape: one cached forward of a full-shape layer
    and one LM head + confidence + unmask, with all cores and with one thread; the step of the 32-layer model is
    extrapolated as layers x layer + head (the 32 layers in float64 do not fit a bounded sample), the one-layer + head
    workload (c2) is that sum itself, timed in full."""
    from oracle import dllm_oracle as O
    from paper_2601_07568_amd import synth
    try:
        from threadpoolctl import threadpool_limits
    except Exception:                                   # no way to pin BLAS to one thread: report all cores only
        threadpool_limits = None
    one = ms.with_layers(1)
    w = synth.Weights(one, 3)
    prompt = synth.random_tokens(one, 3, P)
    blk = synth.masked_block(one, 3, Q, n_masked)
    ck, cv = O.prefill(w, prompt, widen=synth.as_float)
    w.globals()
    O.forward_cached(w, blk, ck, cv, widen=synth.as_float, want_logits=False)          # page the weights in

    def timed(budget, max_n):
        t0 = time.perf_counter()
        n = 0
        while True:
            _, x = O.forward_cached(w, blk, ck, cv, widen=synth.as_float, want_logits=False)
            n += 1
            if time.perf_counter() - t0 > budget or n >= max_n:
                break
        t_layer = (time.perf_counter() - t0) / n
        t0 = time.perf_counter()
        logits = O.head_logits(w, x, widen=synth.as_float)
        cand, conf, ent, _ = O.confidence(logits, one.mask_id)
        O.unmask(blk, cand, conf, one.mask_id, 0.9, 2)
        return n, t_layer, time.perf_counter() - t0

    try:
        cores = len(os.sched_getaffinity(0))
    except Exception:
        cores = os.cpu_count()
    n, t_layer, t_head = timed(budget_s * 0.4, 32)
    out = {"value": 1.0 / (ms.n_layers * t_layer + t_head), "unit": "steps/s", "cores": cores, "kind": "oracle",
           "sample": f"{n} cached forwards of one full-shape layer ({t_layer*1e3:.0f} ms each) and one LM head + "
                     f"confidence + unmask ({t_head*1e3:.0f} ms), numpy float64, all cores; step time extrapolated as "
                     f"{ms.n_layers} x layer + head",
           "one_layer_plus_head_step_s": t_layer + t_head}
    # the tiny workload's whole decode (64 prompt tokens, one block of 32, threshold 0.9, floor 1), timed in full
    tiny_w = synth.Weights(synth.TINY, 0)
    tiny_p = synth.random_tokens(synth.TINY, 0, 64)

    def tiny_decode():
        t0 = time.perf_counter()
        _, n_fw = O.decode(tiny_w, tiny_p, 1, 32, 0.9, 1)
        return time.perf_counter() - t0, n_fw

    tiny_decode()
    t_tiny, n_fw = tiny_decode()
    out["tiny_whole_decode_s"] = t_tiny
    out["tiny_whole_decode_forwards"] = int(n_fw)
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            n1, t1_layer, t1_head = timed(budget_s * 0.4, 4)
            t1_tiny, _ = tiny_decode()
        out["single_thread"] = {"value": 1.0 / (ms.n_layers * t1_layer + t1_head), "unit": "steps/s", "cores": 1,
                                "sample": f"{n1} layer forward(s) ({t1_layer*1e3:.0f} ms each) and one head "
                                          f"({t1_head*1e3:.0f} ms), one BLAS thread",
                                "one_layer_plus_head_step_s": t1_layer + t1_head, "tiny_whole_decode_s": t1_tiny}
    return out


# ----------------------------------------------------------------------------------------------- attainable rates

def attainable(eng, torch, dev):
    """What the chip sustains in this run: a 2 GiB stream read (median of 5) and a matrix-instruction loop."""
    buf = torch.empty(1 << 29, dtype=torch.float32, device=dev)
    buf.normal_()
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    eng.probe_hbm_read(buf, sink)
    t = event_times_ms(torch, lambda i: eng.probe_hbm_read(buf, sink), 5)
    gbs = buf.numel() * 4 / (statistics.median(t) * 1e-3) / 1e9
    small = buf[: (100663296 // 4)]
    eng.probe_hbm_read(small, sink)
    t100 = event_times_ms(torch, lambda i: eng.probe_hbm_read(small, sink), 20)
    del buf, small
    fl = eng.probe_mfma(20000, sink)
    tm = event_times_ms(torch, lambda i: eng.probe_mfma(20000, sink), 3)
    eng.probe_mfma(20000, sink, True)
    tr = event_times_ms(torch, lambda i: eng.probe_mfma(20000, sink, True), 3)
    return {"hbm_GBps": gbs, "hbm_read_100MB_us": statistics.median(t100) * 1e3,
            "mfma_bf16_TFLOPs": fl / (statistics.median(tm) * 1e-3) / 1e12,
            "mfma_bf16_random_operands_TFLOPs": fl / (statistics.median(tr) * 1e-3) / 1e12,
            "how": "dllm_probe_hbm_read over 2 GiB and over 100 MB (one launch each, events); dllm_probe_mfma: "
                   "32x32x16 bf16 products on register operands, one wave per SIMD, with operands of one sign and exponent and "
                   "with random signs, exponents and mantissas (what the chip sustains depends on the switching activity)"}


# ----------------------------------------------------------------------------------------------- batch-1 workloads

def multiblock_generation(eng, ms, prompt, P, Q, n_blocks, table, torch, np, dev, theta=0.45, add_at=0.1, full_at=0.95,
                          delay=1, refresh_every=16):
    """One generation with the multi-block decoding of Section 3.2 (entropy threshold 0.45 nats, block-add at 10 %,
    fully-activate at 95 %, one stabilizing round, a periodic refresh after 16 cached rounds in a row): block states,
    transitions and the plan of the next round (forward type, cache length) live on the device (dllm_fsm_update,
    dllm_fsm_plan); the host reads five integers per round to pick the window and the call.  With random weights the
    entropies stay near ln(V), so the floors of the fully activated blocks drive the decode; the leg measures the
    machinery (windows of more than one block, forwards without cache, per-block floors), not the paper's parallelism."""
    NB = n_blocks
    gen = torch.full((1, NB * Q), ms.mask_id, dtype=torch.int32, device=dev)
    state = torch.zeros(1, NB, dtype=torch.int32, device=dev)
    state[0, 0] = 2
    counter = torch.zeros(1, NB, dtype=torch.int32, device=dev)
    floor = torch.full((1, NB), -1, dtype=torch.int32, device=dev)
    floor[0, 0] = 1
    summary = torch.zeros(1, 4, dtype=torch.int32, device=dev)
    since = torch.zeros(1, dtype=torch.int32, device=dev)           # cached rounds since the last forward without cache
    nocache = torch.zeros(1, dtype=torch.int32, device=dev)         # the next forward must not use the cache
    n_commit = torch.zeros(1, dtype=torch.int32, device=dev)        # positions the cache holds after such a forward
    base = eng.i32([P])
    Qmax = 4 * Q
    cand = torch.zeros(1, Qmax, dtype=torch.int32, device=dev)
    conf = torch.zeros(1, Qmax, dtype=torch.float32, device=dev)
    ent = torch.zeros(1, Qmax, dtype=torch.float32, device=dev)
    n_max = P + NB * Q
    c2 = torch.zeros(n_max, dtype=torch.int32, device=dev)
    f2 = torch.zeros(n_max, dtype=torch.float32, device=dev)
    e2 = torch.zeros(n_max, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.prefill_kv(prompt, eng.i32([0, P]), table, None, total_tokens=P, max_seqlen=P)
    lo, hi, stab = 0, 0, 0
    rounds = nocache_rounds = wide_rounds = 0
    while lo >= 0:
        if hi - lo + 1 > 4:
            hi = lo + 3                                            # the window this engine was sized for
        nw = hi - lo + 1
        window = gen[:, lo * Q:(hi + 1) * Q]
        fl = floor[:, lo:hi + 1]
        if stab:
            n_tok = P + (hi + 1) * Q
            seq = torch.cat([prompt, gen[0, :(hi + 1) * Q]])
            eng.refresh_cache(seq, eng.i32([0, n_tok]), table, n_commit, c2, f2, e2, total_tokens=n_tok, max_seqlen=n_tok)
            s0 = P + lo * Q
            eng.unmask_blocks(window, c2[s0:n_tok][None], e2[s0:n_tok][None], theta, fl, True, Q)
            nocache_rounds += 1
        else:
            eng.denoise_step(window, eng.i32([P + lo * Q]), table, cand[:, :nw * Q], conf[:, :nw * Q], ent[:, :nw * Q],
                             max_prefix_len=P + lo * Q)
            eng.unmask_blocks(window, cand[:, :nw * Q], ent[:, :nw * Q], theta, fl, True, Q)
        eng.fsm_update(gen, state, counter, Q, add_at, full_at, delay, None, floor, summary)
        eng.fsm_plan(state, counter, base, Q, refresh_every, since, nocache, n_commit)
        lo, hi, _, _ = summary[0].tolist()
        stab = int(nocache.item())
        rounds += 1
        wide_rounds += nw > 1
        if rounds > 8 * NB * Q:
            raise RuntimeError("multi-block decode does not terminate")
    torch.cuda.synchronize()
    sec = time.perf_counter() - t0
    assert int((gen == ms.mask_id).sum()) == 0
    return {"tokens": NB * Q, "forwards": rounds, "forwards_without_cache": nocache_rounds,
            "forwards_with_more_than_one_block": wide_rounds, "seconds": sec, "tokens_per_s": NB * Q / sec,
            "tokens_per_forward": NB * Q / rounds, "rule": f"entropy <= {theta}", "block_add": add_at,
            "fully_activate": full_at, "stabilizing_rounds": delay, "periodic_refresh_every": refresh_every}


def multiblock_generation_device(eng, ms, prompt, P, Q, n_blocks, table, torch, np, dev, theta=0.45, add_at=0.1,
                                 full_at=0.95, delay=1, refresh_every=16, W=2, max_rounds=400):
    """The same multi-block generation with no host read inside the decode: one fixed sequence of calls per round (the
    plan on the device picks, per sequence, the cached step or the packed forward without cache, whose total is
    device-resident), captured once as a HIP graph and replayed; the host looks at the tokens every 16 rounds only to
    stop.  Windows are at most W blocks; every launch is sized for that and for the longest sequence, which is what a
    round costs when nothing comes back to the host to size it."""
    NB, Bn = n_blocks, 1
    cap = P + NB * Q
    i32 = dict(dtype=torch.int32, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    gen = torch.full((Bn, NB * Q), ms.mask_id, **i32)
    state = torch.zeros(Bn, NB, **i32)
    state[:, 0] = 2
    counter = torch.zeros(Bn, NB, **i32)
    since, nocache, plan_commit = (torch.zeros(Bn, **i32) for _ in range(3))
    base = eng.i32([P])
    prompts = prompt.reshape(1, P).contiguous()
    win, wfl = torch.zeros(Bn, W * Q, **i32), torch.zeros(Bn, W, **i32)
    pre, qv, qvc, wlo = (torch.zeros(Bn, **i32) for _ in range(4))
    cand, conf, ent = torch.zeros(Bn, W * Q, **i32), torch.zeros(Bn, W * Q, **f32), torch.zeros(Bn, W * Q, **f32)
    ptok, cu, ncommit = torch.zeros(cap, **i32), torch.zeros(Bn + 1, **i32), torch.zeros(Bn, **i32)
    c2, f2, e2 = torch.zeros(cap, **i32), torch.zeros(cap, **f32), torch.zeros(cap, **f32)

    def one_round():
        eng.fsm_round_windows(gen, state, base, nocache, Q, W, 0, win, wfl, pre, qv, qvc, wlo)
        eng.denoise_step_var(win, pre, qvc, table, cand, conf, ent, max_prefix_len=cap)
        eng.fsm_pack(prompts, gen, state, base, nocache, plan_commit, Q, W, 0, ptok, cu, ncommit, max_seqlen=cap)
        eng.refresh_cache_dev(ptok, cu, table, ncommit, c2, f2, e2, max_seqlen=cap)
        eng.fsm_unpack(cu, pre, qv, nocache, c2, f2, e2, cand, conf, ent)
        eng.unmask_blocks(win, cand, ent, theta, wfl, True, Q)
        eng.fsm_scatter(win, wlo, qv, gen, NB, Q, W)
        eng.fsm_update(gen, state, counter, Q, add_at, full_at, delay, None, None, None)
        eng.fsm_plan(state, counter, base, Q, refresh_every, since, nocache, plan_commit)

    eng.prefill_kv(prompt, eng.i32([0, P]), table, None, total_tokens=P, max_seqlen=P)
    one_round()                                                    # warm-up outside the capture, then start over
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_round()
    gen.fill_(ms.mask_id)
    state.zero_()
    state[:, 0] = 2
    for t in (counter, since, nocache, plan_commit):
        t.zero_()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.prefill_kv(prompt, eng.i32([0, P]), table, None, total_tokens=P, max_seqlen=P)
    rounds = 0
    while rounds < max_rounds:
        for _ in range(16):
            graph.replay()
        rounds += 16
        if int((gen == ms.mask_id).sum()) == 0:
            break
    torch.cuda.synchronize()
    sec = time.perf_counter() - t0
    assert int((gen == ms.mask_id).sum()) == 0 and eng.read_status() == 0
    return {"tokens": NB * Q, "rounds_replayed": rounds, "seconds": sec, "tokens_per_s": NB * Q / sec,
            "ms_per_round": sec * 1e3 / rounds, "window_blocks": W, "launch": "one HIP graph per round, replayed",
            "host_reads": "the token array once per 16 rounds, to stop"}


def batch1(args, torch, np, synth, Engine, dev, workload, steps, warmup, extras):
    """Batch-1 step of the LLaDA-8B-shaped model: "c3" = the whole model, prompt 1024 (headline), "c2" = one layer +
    LM head, prefix 512.  extras: generation legs, attainable rates (they need the engine)."""
    if workload == "c3":
        ms, P, Q, n_blocks, tau, m_floor, n_masked0 = synth.LLADA_8B, 1024, 32, 8, 0.9, 2, 32
        name = "LLaDA-8B-shaped 32 layers, bf16, batch 1, prompt 1024, block 32, tau 0.9, min 2 unmasks/step"
    else:
        ms, P, Q, n_blocks, tau, m_floor, n_masked0 = synth.LLADA_8B.with_layers(1), 512, 32, 1, 0.9, 1, 24
        name = "one LLaDA-8B-shaped layer + LM head, bf16, batch 1, prefix 512, block 32 (24 masked), tau 0.9, min 1"
    if args.layers is not None:
        ms = ms.with_layers(args.layers)
        name += f" [depth overridden: {args.layers} layers]"
    pt = 64
    max_len = P + n_blocks * Q
    mp = (max_len + pt - 1) // pt
    eng = Engine(ms, None, page_tokens=pt, max_pages_per_seq=mp, n_pages=mp, max_batch=1, max_q=4 * Q,
                 max_tokens=max_len, device_weights=synth.device_weights(ms, torch, dev, 1))
    table = eng.i32(np.arange(mp)[None])
    prompt = eng.i32(synth.random_tokens(ms, 3, P))
    cu = eng.i32([0, P])
    eng.prefill_kv(prompt, cu, table, None, total_tokens=P, max_seqlen=P)
    torch.cuda.synchronize()

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    fresh = eng.i32(synth.masked_block(ms, 3, Q, n_masked0)[None])
    qt = fresh.clone()
    prefix = eng.i32([P])
    cand = torch.zeros(1, Q, dtype=torch.int32, device=dev)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=dev)
    nrem = torch.zeros(1, 1, dtype=torch.int32, device=dev)
    steps_per_block = max(1, n_masked0 // m_floor)

    def one_step(i):
        if i % steps_per_block == 0:
            qt.copy_(fresh)                       # device-side re-mask: keeps every step a full step
        eng.denoise_step(qt, prefix, table, cand, conf, None, max_prefix_len=P)
        eng.unmask(qt, cand, conf, tau, m_floor, n_remaining=nrem)

    for i in range(warmup):
        one_step(i)
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        # one step (forward + unmask) captured once; the calls only enqueue and read no device value on the
        # host, so the captured graph is the step itself
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eng.denoise_step(qt, prefix, table, cand, conf, None, max_prefix_len=P)
            eng.unmask(qt, cand, conf, tau, m_floor, n_remaining=nrem)
        torch.cuda.synchronize()

    def timed_step(i):
        if graph is None:
            one_step(i)
            return
        if i % steps_per_block == 0:
            qt.copy_(fresh)
        graph.replay()

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        timed_step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    assert eng.read_status() == 0

    # ---- per-step event times over at least 50 steps (the re-mask copy of every 16th step is inside its step)
    per = event_times_ms(torch, timed_step, max(steps, 50))

    # ---- per-kernel HIP-event pass over the same steps (separate from the timed region above)
    eng.profile_enable(True)
    n_prof = min(steps, 16)
    for i in range(n_prof):
        one_step(i)
    kern = {}
    for cls, nm in KCLASS.items():
        n, tms, by = eng.profile_read(cls)
        if n:
            kern[nm] = {"launches": n, "avg_us": tms / n * 1e3, "bytes_per_launch": by / n,
                        "GBps": by / (tms * 1e-3) / 1e9 if tms > 0 else None}
    eng.profile_enable(False)
    d, dq, dkv, F = ms.d_model, ms.n_q_heads * ms.head_dim, ms.n_kv_heads * ms.head_dim, ms.d_ff
    step_bytes = ms.n_layers * 2 * (d * (dq + 2 * dkv) + dq * d + 3 * d * F) + 2 * ms.vocab * d \
        + ms.n_layers * 2 * 2 * dkv * (P + Q)
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9
    weight_streamers = {k: v for k, v in kern.items() if k != "attention"}
    dom = max(weight_streamers, key=lambda k: weight_streamers[k]["avg_us"] * weight_streamers[k]["launches"]) \
        if weight_streamers else None
    roofline = None
    if dom:
        a = kern[dom]["GBps"]
        traffic = pmc_traffic("denoise_step_c3_hbm_traffic_pmc.txt", f"k_skinny({dom})") \
            if workload == "c3" and args.layers is None else None
        roofline = {"bound": "hbm", "step_frac_of_hbm_peak": step_gbs / HBM_PEAK_GBS, "kernel": f"k_skinny ({dom})",
                    "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS, "traffic": traffic,
                    "avg_us": kern[dom]["avg_us"], "bytes_per_launch": kern[dom]["bytes_per_launch"]}

    out = {
        "metric": "denoise_steps_per_s", "value": steps / elapsed, "unit": "steps/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "launch": "eager" if graph is None else "hip graph of one step, replayed"},
        "step_ms_median": statistics.median(per), "step_ms_min": min(per), "step_ms_events": len(per),
        "step_algorithmic_GB": step_bytes / 1e9, "step_GBps": step_gbs, "step_frac_of_hbm_peak": step_gbs / HBM_PEAK_GBS,
        "roofline": roofline, "kernels": kern,
    }
    if not extras:
        eng.close()
        return out

    # ---- one whole generation, end to end (prefill, blocks, refresh at each boundary)
    gen = gen_mb = None
    if not args.no_generation and n_blocks > 1:
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        seq = prompt.clone()
        eng.prefill_kv(seq, cu, table, None, total_tokens=P, max_seqlen=P)
        torch.cuda.synchronize()
        prefill_s = time.perf_counter() - g0
        refresh_s = 0.0
        forwards = 0
        cur = P
        for b in range(n_blocks):
            blk = torch.full((1, Q), ms.mask_id, dtype=torch.int32, device=dev)
            pl = eng.i32([cur])
            while True:
                eng.denoise_step(blk, pl, table, cand, conf, None, max_prefix_len=cur)
                eng.unmask(blk, cand, conf, tau, m_floor, n_remaining=nrem)
                forwards += 1
                if int(nrem.item()) == 0:
                    break
            seq = torch.cat([seq, blk[0]])
            cur += Q
            torch.cuda.synchronize()
            r0 = time.perf_counter()
            eng.refresh_cache(seq, eng.i32([0, cur]), table, None, total_tokens=cur, max_seqlen=cur)
            torch.cuda.synchronize()
            refresh_s += time.perf_counter() - r0
        torch.cuda.synchronize()
        gsec = time.perf_counter() - g0
        per_tok = ms.n_layers * 2 * (d * (dq + 2 * dkv) + dq * d + 3 * d * F)          # GEMM flops per row
        attn_fl = lambda S: ms.n_layers * 4 * ms.n_q_heads * S * S * ms.head_dim       # QK^T and PV once each
        refresh_lens = [P + (b + 1) * Q for b in range(n_blocks)]
        refresh_flops = sum(S * per_tok + attn_fl(S) for S in refresh_lens)
        gen = {"tokens": n_blocks * Q, "forwards": forwards, "seconds": gsec, "tokens_per_s": n_blocks * Q / gsec,
               "steps_per_s": forwards / gsec, "tokens_per_forward": n_blocks * Q / forwards,
               "prefill": {"tokens": P, "ms": prefill_s * 1e3, "TFLOPs": (P * per_tok + attn_fl(P)) / prefill_s / 1e12},
               "refresh": {"calls": n_blocks, "tokens": refresh_lens, "ms_total": refresh_s * 1e3,
                           "TFLOPs": refresh_flops / refresh_s / 1e12}}
        # ---- the same generation with multi-block decoding (entropy rule, block state machine on the device)
        gen_mb = multiblock_generation(eng, ms, prompt, P, Q, n_blocks, table, torch, np, dev)
        gen_mb["without_host_reads"] = multiblock_generation_device(eng, ms, prompt, P, Q, n_blocks, table, torch, np, dev)
    out["generation"] = gen
    out["generation_multiblock"] = gen_mb
    out["attainable"] = attainable(eng, torch, dev)
    eng.close()
    return out


# ----------------------------------------------------------------------------------------------- large batches

def large_batch(args, torch, np, synth, Engine, dev, steps, warmup):
    """Long-context large-batch step: Dream-7B-shaped model, batch 32, prefix KV of 8192 tokens per sequence drawn
    directly on the device, one block of 32 per sequence with 16 masked: 1024 query rows, LM head on the masked ones.
    Bound by the matrix cores."""
    ms = synth.DREAM_7B if args.layers is None else synth.DREAM_7B.with_layers(args.layers)
    Bn, P, Q, pt = 32, 8192, 32, 64
    mp = (P + Q + pt - 1) // pt
    eng = Engine(ms, None, page_tokens=pt, max_pages_per_seq=mp, n_pages=Bn * mp, max_batch=Bn, max_q=Q,
                 max_tokens=0, device_weights=synth.device_weights(ms, torch, dev, 5), pack=False)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    pool = eng.kv_pool.view(torch.bfloat16)
    for i in range(0, pool.numel(), 1 << 28):                      # N(0,1) K and V for every slot
        n = min(1 << 28, pool.numel() - i)
        pool[i:i + n] = torch.randn(n, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    table = eng.i32(np.arange(Bn * mp).reshape(Bn, mp))
    prefix = eng.i32([P] * Bn)
    fresh = eng.i32(np.stack([synth.masked_block(ms, 5, Q, 16, stream=b) for b in range(Bn)]))
    qt = fresh.clone()
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=dev)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)

    def one_step(i):
        if i % 8 == 0:
            qt.copy_(fresh)
        eng.denoise_step(qt, prefix, table, cand, conf, None, max_prefix_len=P)
        eng.unmask(qt, cand, conf, 0.9, 1)

    for i in range(warmup):
        one_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one_step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert eng.read_status() == 0
    per = event_times_ms(torch, one_step, max(steps, 8))
    eng.profile_enable(True)
    n_prof = min(steps, 4)
    lm_rows = 0
    for i in range(n_prof):
        lm_rows += int((qt == ms.mask_id).sum()) if i % 8 else Bn * 16     # rows the LM head really computes
        one_step(i)
    kern = {}
    for cls, nm in KCLASS.items():
        n, tms, work = eng.profile_read(cls)
        if n:
            kern[nm] = {"launches": n, "avg_us": tms / n * 1e3,
                        ("GBps" if nm == "attention" else "TFLOPs"): work / (tms * 1e-3) / (1e9 if nm == "attention" else 1e12)}
    eng.profile_enable(False)
    if "lm_head" in kern:
        # the library books the LM head with every query row; only the masked rows are computed
        k = kern["lm_head"]
        k["rows_avg"] = lm_rows / n_prof
        k["TFLOPs"] = 2.0 * k["rows_avg"] * ms.vocab * ms.d_model / (k["avg_us"] * 1e-6) / 1e12
    T = Bn * Q
    d, dq, dkv, F, G = ms.d_model, ms.n_q_heads * ms.head_dim, ms.n_kv_heads * ms.head_dim, ms.d_ff, ms.n_q_heads // ms.n_kv_heads
    per_layer = 2 * T * (d * (dq + 2 * dkv) + dq * d + 3 * d * F)
    attn = 4 * (Q * G) * (P + Q) * ms.head_dim * ms.n_kv_heads * Bn
    # LM head on the rows masked on average over a re-mask period of 8 steps with one unmask per step and sequence
    head_rows = Bn * (16 - 3.5)
    flops = ms.n_layers * (per_layer + attn) + 2 * head_rows * ms.vocab * d
    ms_per_step = elapsed / steps * 1e3
    gemm = {k: v for k, v in kern.items() if k not in ("attention", "lm_head")}
    dom = max(gemm, key=lambda k: gemm[k]["avg_us"] * gemm[k]["launches"]) if gemm else None
    roofline = None
    if dom:
        a = kern[dom]["TFLOPs"]
        traffic = pmc_traffic("denoise_step_c5_hbm_traffic_pmc.txt", f"k_gemm_t256({dom})") if args.layers is None else None
        roofline = {"bound": "mfma", "step_frac_of_mfma_peak": flops / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                    "kernel": f"k_gemm_t256 ({dom})", "achieved": a, "peak": MFMA_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": a / MFMA_PEAK_TFLOPS, "traffic": traffic, "avg_us": kern[dom]["avg_us"]}
    eng.close()
    return {"metric": "denoise_steps_per_s", "value": steps / elapsed, "unit": "steps/s", "n_gpus": 1,
            "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "Dream-7B-shaped %d layers, bf16, batch 32, prefix KV 8192 drawn N(0,1), block 32 with "
                                   "16 masked, tau 0.9, min 1" % ms.n_layers, "launch": "eager"},
            "step_ms_median": statistics.median(per), "step_ms_min": min(per), "step_ms_events": len(per),
            "query_tokens_per_s": T * steps / elapsed, "step_algorithmic_TFLOP": flops / 1e12,
            "step_TFLOPs": flops / (ms_per_step * 1e-3) / 1e12,
            "step_frac_of_mfma_peak": flops / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
            "roofline": roofline, "kernels": kern}


def prefill_batch(args, torch, np, synth, Engine, dev, steps, warmup):
    """Workload c4: Dream-7B-shaped model, 16 prompts of 2048 random tokens prefilled in one call (32768 rows through
    every GEMM, bidirectional attention inside each prompt), then denoise steps with two blocks of 32 in flight per
    sequence (64 query rows each, 1024 in all) against the 2048-token caches, tau 0.85, floor 1 per block.  Reports
    both: the prefill in TFLOP/s and the step in steps/s."""
    ms = synth.DREAM_7B if args.layers is None else synth.DREAM_7B.with_layers(args.layers)
    Bn, S, Q, bl, pt = 16, 2048, 64, 32, 64
    mp = (S + Q + pt - 1) // pt
    eng = Engine(ms, None, page_tokens=pt, max_pages_per_seq=mp, n_pages=Bn * mp, max_batch=Bn, max_q=Q,
                 max_tokens=Bn * S, device_weights=synth.device_weights(ms, torch, dev, 4), pack=False)
    table = eng.i32(np.arange(Bn * mp).reshape(Bn, mp))
    toks = eng.i32(np.concatenate([synth.random_tokens(ms, 40 + b, S) for b in range(Bn)]))
    cu = eng.i32(np.arange(Bn + 1) * S)
    d, dq, dkv, F, G = ms.d_model, ms.n_q_heads * ms.head_dim, ms.n_kv_heads * ms.head_dim, ms.d_ff, ms.n_q_heads // ms.n_kv_heads
    gemm_per_row = 2 * (d * (dq + 2 * dkv) + dq * d + 3 * d * F)

    def prefill():
        eng.prefill_kv(toks, cu, table, None, total_tokens=Bn * S, max_seqlen=S)

    prefill()
    torch.cuda.synchronize()
    n_pre = 2
    t0 = time.perf_counter()
    for _ in range(n_pre):
        prefill()
    torch.cuda.synchronize()
    pre_s = (time.perf_counter() - t0) / n_pre
    pre_flops = ms.n_layers * (Bn * S * gemm_per_row + 4 * Bn * ms.n_q_heads * S * S * ms.head_dim)
    eng.profile_enable(True)
    prefill()
    pk = {}
    for cls, nm in KCLASS.items():
        n, tms, work = eng.profile_read(cls)
        if n:
            pk[nm] = {"launches": n, "avg_us": tms / n * 1e3}
    eng.profile_enable(False)

    prefix = eng.i32([S] * Bn)
    fresh = eng.i32(np.stack([np.concatenate([synth.masked_block(ms, 5, bl, 24, stream=2 * b),
                                              synth.masked_block(ms, 5, bl, 32, stream=2 * b + 1)]) for b in range(Bn)]))
    qt = fresh.clone()
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=dev)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)

    def one_step(i):
        if i % 16 == 0:
            qt.copy_(fresh)
        eng.denoise_step(qt, prefix, table, cand, conf, None, max_prefix_len=S)
        eng.unmask(qt, cand, conf, 0.85, 1, block_len=bl)

    for i in range(warmup):
        one_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one_step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert eng.read_status() == 0
    per = event_times_ms(torch, one_step, max(steps, 8))
    T = Bn * Q
    # LM head on the rows masked on average over the re-mask period of 16 steps (56 at its start, two fewer per step)
    step_flops = ms.n_layers * (T * gemm_per_row + 4 * (Q * G) * (S + Q) * ms.head_dim * ms.n_kv_heads * Bn) \
        + 2 * (Bn * (56 - 15)) * ms.vocab * d
    ms_per_step = elapsed / steps * 1e3
    eng.close()
    return {"metric": "denoise_steps_per_s", "value": steps / elapsed, "unit": "steps/s", "n_gpus": 1,
            "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "Dream-7B-shaped %d layers, bf16, batch 16, prompts 2048 prefilled, 2 blocks of 32 in "
                                   "flight per sequence, tau 0.85, min 1 per block" % ms.n_layers, "launch": "eager"},
            "step_ms_median": statistics.median(per), "step_ms_min": min(per), "step_ms_events": len(per),
            "query_tokens_per_s": T * steps / elapsed, "step_algorithmic_TFLOP": step_flops / 1e12,
            "step_TFLOPs": step_flops / (ms_per_step * 1e-3) / 1e12,
            "step_frac_of_mfma_peak": step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
            "prefill": {"tokens": Bn * S, "seconds": pre_s, "tokens_per_s": Bn * S / pre_s,
                        "algorithmic_TFLOP": pre_flops / 1e12, "TFLOPs": pre_flops / pre_s / 1e12,
                        "frac_of_mfma_peak": pre_flops / pre_s / 1e12 / MFMA_PEAK_TFLOPS, "kernels": pk},
            "roofline": {"bound": "mfma", "kernel": "prefill (all kernels)", "achieved": pre_flops / pre_s / 1e12,
                         "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": pre_flops / pre_s / 1e12 / MFMA_PEAK_TFLOPS,
                         "traffic": None}}


def trimmed(leg):
    """A secondary workload's entry of the headline line: its own numbers without the line's fixed fields."""
    drop = ("metric", "unit", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "warmup")
    return {k: v for k, v in leg.items() if k not in drop}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="c3", choices=["c3", "c2", "c4", "c5"])
    ap.add_argument("--layers", type=int, default=None, help="override depth (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-generation", action="store_true")
    ap.add_argument("--no-extra-legs", action="store_true",
                    help="headline workload only: no c2 / large-batch legs in the same line")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every step eagerly instead of replaying a captured HIP graph of one step")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (known traffic) so that a rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE run of this command can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2601_07568_amd import synth
    from paper_2601_07568_amd.binding import Engine

    dev = torch.device("cuda:0")
    if args.workload == "c5":
        print(json.dumps(large_batch(args, torch, np, synth, Engine, dev, args.steps, args.warmup)))
        return
    if args.workload == "c4":
        print(json.dumps(prefill_batch(args, torch, np, synth, Engine, dev, args.steps, args.warmup)))
        return
    out = batch1(args, torch, np, synth, Engine, dev, args.workload, args.steps, args.warmup, extras=True)
    torch.cuda.empty_cache()
    if args.workload == "c3" and not args.no_extra_legs and args.layers is None:
        # the small HBM-bound workload and the matrix-core-bound one, each with its own roofline object
        out["c2"] = trimmed(batch1(args, torch, np, synth, Engine, dev, "c2", max(args.steps, 50), args.warmup, extras=False))
        torch.cuda.empty_cache()
        out["large_batch"] = trimmed(large_batch(args, torch, np, synth, Engine, dev, 50, 3))
        torch.cuda.empty_cache()
    att = out.get("attainable")
    if att:
        # the same fractions against what the probes of this run reached (stream read; matrix loop on random operands)
        out["roofline"]["step_frac_of_attainable_hbm"] = out["step_GBps"] / att["hbm_GBps"]
        if "c2" in out:
            out["c2"]["roofline"]["step_frac_of_attainable_hbm"] = out["c2"]["step_GBps"] / att["hbm_GBps"]
        if "large_batch" in out:
            out["large_batch"]["roofline"]["step_frac_of_attainable_mfma"] = \
                out["large_batch"]["step_TFLOPs"] / att["mfma_bf16_random_operands_TFLOPs"]
    if not args.no_cpu_baseline:
        base = cpu_baseline(synth.LLADA_8B if args.workload == "c3" else synth.LLADA_8B.with_layers(1),
                            1024 if args.workload == "c3" else 512, 32, 32 if args.workload == "c3" else 24)
        out["cpu_baseline"] = base
    print(json.dumps(out))


if __name__ == "__main__":
    main()
