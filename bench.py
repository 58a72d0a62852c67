"""Benchmark of the stage executor on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4]

A step is one jpp_stage_zero_grads + one jpp_stage_run of the configuration's whole task list
(all microbatches, all owned stages, forward and backward, gradient accumulation, boundary
copies), with inputs resident in HBM.  Prints one JSON line: value = algorithmic TFLOP/s of the
whole step (linear maps 2 T d_in d_out x 3, causal attention at half, x 3; nothing recomputed or
element-wise is counted), ms_per_step from the host clock around K steps (min and median from
events on the compute stream), config = the workload and the executor's settings, roofline = the
dominant kernel (the weight-gradient GEMM) timed alone with events on its own stream against
the dense bf16 matrix peak, cpu_baseline = the fp64 oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0


def algorithmic_flops_per_microbatch(w):
    """2*T*d_in*d_out per linear map x3 (forward, input grad, weight grad); causal attention at
    half of the full score matrix (forward 2*mb*Hq*seq^2*hd, backward twice that); norms and
    activations not counted; no recompute counted."""
    T = w.tokens
    nq, nkv = w.n_q_heads * w.head_dim, w.n_kv_heads * w.head_dim
    f1 = 2 * w.d_ffn if w.act == 2 else w.d_ffn
    lin = w.d_model * (nq + 2 * nkv) + nq * w.d_model + w.d_model * f1 + w.d_ffn * w.d_model
    per_layer = 3 * 2.0 * T * lin + 3 * 2.0 * w.microbatch * w.n_q_heads * w.seq_len ** 2 * w.head_dim
    total = per_layer * w.n_layers
    if w.loss_head:
        total += 3 * 2.0 * T * w.d_model * w.vocab
    return total * len(w.stage_ids)


def flops_full_attention(w):
    """The count above with attention taken over the whole seq x seq score matrix."""
    extra = 3 * 2.0 * w.microbatch * w.n_q_heads * w.seq_len ** 2 * w.head_dim * w.n_layers * len(w.stage_ids)
    return algorithmic_flops_per_microbatch(w) + extra


def wgrad_shapes(w):
    """(M, N, K) of the weight-gradient GEMMs that the backward task completing a group
    launches, in launch order: the contraction runs over the tokens of the whole group."""
    T = w.tokens * max(1, w.wgrad_group)
    nq, nkv = w.n_q_heads * w.head_dim, w.n_kv_heads * w.head_dim
    f1 = 2 * w.d_ffn if w.act == 2 else w.d_ffn
    per_layer = [(w.d_model, w.d_ffn, T), (f1, w.d_model, T), (w.d_model, nq, T), (nq + 2 * nkv, w.d_model, T)]
    out = per_layer * w.n_layers
    if w.loss_head:
        out = [(w.vocab, w.d_model, T)] + out
    return out


def time_dominant_kernel(w, torch, B, reps=3):
    """Average launch duration of the dominant kernel -- the weight-gradient GEMM with the fused
    fp32 accumulation, one template instantiation launched with the shapes above -- measured
    with HIP events on the stream it is launched on."""
    s = torch.cuda.Stream()
    shapes = wgrad_shapes(w)
    total_ms, total_flops, n = 0.0, 0.0, 0
    with torch.cuda.stream(s):
        for (M, N, K) in shapes:
            # operands with the value distributions the step feeds this kernel: an output-gradient
            # matrix at the cotangents' scale and an activation matrix of unit scale (the matrix
            # pipes' clock, hence the rate, depends on the data)
            A = (torch.randn((K, M), device="cuda:0") * w.cot_std).to(torch.bfloat16)
            Bm = torch.randn((K, N), device="cuda:0").to(torch.bfloat16)
            C = torch.zeros((M, N), dtype=torch.float32, device="cuda:0")
            # with the scratch the executor gives it (outputs of few tiles are cut along k)
            need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, B.OUT_ACC_F32)
            ws = torch.empty(max(need // 4, 4), dtype=torch.float32, device="cuda:0")
            args = (B.JPP_BF16, M, N, K, A.data_ptr(), M, 1, Bm.data_ptr(), N, 1, C.data_ptr(), N, B.OUT_ACC_F32,
                    None, None, ws.data_ptr() if need else None, need, s.cuda_stream)
            B.jpp_op_gemm_ws(*args)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s)
            for _ in range(reps):
                B.jpp_op_gemm_ws(*args)
            e1.record(s)
            s.synchronize()
            total_ms += e0.elapsed_time(e1)
            total_flops += reps * 2.0 * M * N * K
            n += reps
            del A, Bm, C, ws
    avg_ms = total_ms / n
    return avg_ms, total_flops / n


class ClockSampler:
    """Shader clock and board power read from the driver's sysfs files every 50 ms while a timed
    region runs (the matrix pipes' clock under load is far below the nominal 2.4 GHz and differs
    from box to box, so a rate means little without it).  Everything is None when the files
    cannot be read."""

    def __init__(self):
        import glob
        import threading
        self.sclk = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))[:1]
        self.power = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))[:1]
        self.mhz, self.watts = [], []
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._loop, daemon=True)

    def _read(self):
        try:
            for line in open(self.sclk[0]):
                if "*" in line:
                    self.mhz.append(float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip()))
            if self.power:
                self.watts.append(float(open(self.power[0]).read()) / 1e6)
        except Exception:
            pass

    def _loop(self):
        while not self._stop.is_set():
            self._read()
            self._stop.wait(0.05)

    def __enter__(self):
        if self.sclk:
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self.sclk:
            self._thread.join()

    def summary(self):
        if not self.mhz:
            return None
        out = {"sclk_mhz_min": min(self.mhz), "sclk_mhz_mean": sum(self.mhz) / len(self.mhz),
               "sclk_mhz_max": max(self.mhz), "samples": len(self.mhz), "nominal_mhz": 2400,
               "source": "sysfs pp_dpm_sclk / hwmon power1_input, sampled every 50 ms over the timed steps"}
        if self.watts:
            out["power_w_mean"] = sum(self.watts) / len(self.watts)
            out["power_w_max"] = max(self.watts)
        return out


def progress(msg):
    """One line on stderr when a part of the run is done (stdout carries the JSON line only)."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def run_stage(w, steps, warmup, torch, B, inp, Stage, opt_kind=None, optimizer_name=None):
    """K timed steps of one configuration (a step = jpp_stage_zero_grads + jpp_stage_run of the
    whole task list, inputs resident in HBM).  Returns the figures of the bench line's top level."""
    progress(f"{w.name}: wgrad_group {max(1, w.wgrad_group)}, {warmup} warm-up + {steps} timed steps")
    task_list = None
    if w.sched == inp.SCHED_GPIPE and w.V > 1:
        # GPipe on a circular placement: every forward of every owned stage, then every backward
        task_list = [(i, B.JPP_FWD, s) for s in w.stage_ids for i in range(w.n_microbatches)]
        task_list += [(i, B.JPP_BWD, s) for s in reversed(w.stage_ids) for i in range(w.n_microbatches)]
    st = Stage(w, tasks=task_list)
    streams = 3 - B.jpp_stage_stream_mode(st.h)
    arena_gb = B.jpp_stage_arena_bytes(st.cfg, st.M, st.max_in_flight) / 1e9
    stash_slots = st.max_in_flight
    st.set_params_random(seed=0)
    st.bind(None, None, None, seed=1)           # synthetic boundary tensors generated in HBM
    if opt_kind is not None:
        st.optimizer_bind(opt_kind)
    step_no = [0]
    progress(f"  arena {arena_gb:.1f} GB, parameters and boundary tensors in HBM")

    def update():
        if opt_kind is not None:
            step_no[0] += 1
            st.apply_gradients(opt_kind, lr=1e-4 / w.n_microbatches, weight_decay=0.01, step=step_no[0])

    for _ in range(warmup):
        st.zero_grads()
        st.run()
        update()
    st.sync()
    torch.cuda.synchronize()
    progress("  warm-up done")
    # per-step marks on the stage's compute stream (every run is joined back into it), recorded
    # without waiting: the host keeps enqueueing while the GPU works
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    with ClockSampler() as clocks:
        t0 = time.perf_counter()
        marks[0].record(st.compute)
        for k in range(steps):
            st.zero_grads()
            st.run()
            update()
            marks[k + 1].record(st.compute)
        st.sync()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    progress(f"  timed steps done: {ms_per_step:.1f} ms per step")
    per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(steps))
    flops_step = algorithmic_flops_per_microbatch(w) * w.n_microbatches
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12
    opt_info = None
    if opt_kind is not None:
        # the update alone: HBM-bound, 4 (g) + 2 x esz (w) bytes per parameter for SGD,
        # 16 read + 12 written in fp32 state plus esz written for AdamW
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st.compute)
        for _ in range(3):
            update()
        e1.record(st.compute)
        st.sync()
        ms_u = e0.elapsed_time(e1) / 3
        esz = 2 if w.dtype == inp.DT_BF16 else 4
        per = (4 + 2 * esz) if opt_kind == B.JPP_OPT_SGD else (28 + esz)
        nbytes = per * st.pcount * len(w.stage_ids)
        opt_info = {"kind": optimizer_name, "ms": ms_u, "bytes": nbytes, "achieved_GBps": nbytes / ms_u / 1e6,
                    "peak_GBps": PEAK_HBM_GBS, "frac": nbytes / ms_u / 1e6 / PEAK_HBM_GBS}
    # sanity: the run produced finite gradients
    finite = bool(torch.isfinite(st.grads_tensor(0)).all().item())
    st.close()
    del st
    torch.cuda.empty_cache()
    return {"tflops": tflops, "ms_per_step": ms_per_step, "per_step": per_step, "finite": finite,
            "streams": streams, "arena_gb": arena_gb, "stash_slots": stash_slots, "optimizer": opt_info,
            "clocks": clocks.summary(), "microbatches_per_s": w.n_microbatches / (ms_per_step * 1e-3)}


def brief(w, r, steps, warmup):
    """One configuration in a few fields (the secondary entries of the bench line)."""
    return {"workload": w.name, "value": r["tflops"], "unit": "TFLOP/s",
            "pct_of_bf16_mfma_peak": 100.0 * r["tflops"] / PEAK_BF16_TFLOPS, "ms_per_step": r["ms_per_step"],
            "microbatches_per_s": r["microbatches_per_s"], "steps": steps, "warmup": warmup,
            "wgrad_group": max(1, w.wgrad_group), "streams": r["streams"], "arena_gb": r["arena_gb"],
            "stash_slots": r["stash_slots"], "grads_finite": r["finite"],
            "sclk_mhz_mean": (r["clocks"] or {}).get("sclk_mhz_mean")}


def oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count()


# Structure-matched twins for the oracle's timed sample: the configuration's own norm, activation,
# bias, RoPE, head_dim and query/kv head ratio (and loss head), at a width that keeps one
# microbatch of one layer at 5-10 algorithmic TFLOP (10-30 s of host time).
CPU_TWINS = {
    "C2": dict(d_model=8192, n_q_heads=64, d_ffn=32768, seq_len=2048, microbatch=1),
    "C4": dict(d_model=8192, n_q_heads=64, d_ffn=32768, seq_len=2048, microbatch=1),
    "C3": dict(d_model=4096, n_q_heads=32, d_ffn=14336, seq_len=2048, microbatch=1),
    "C5": dict(d_model=4096, n_q_heads=32, d_ffn=16384, seq_len=2048, microbatch=1, vocab=50304),
}


def cpu_baseline(config, w):
    """The fp64 oracle, as it stands, timed on the host: for C1 the whole run (all microbatches,
    forward and backward, the configuration's own task list) on all cores and on one; for the
    other configurations one microbatch, forward + backward, of ONE layer (plus the loss head for
    C5) of a structure-matched twin, the rate extrapolated to the workload by FLOP count."""
    import numpy as np
    from dataclasses import replace
    from oracle import stage_oracle as so
    from paper_2412_14374_amd import binding as B
    from paper_2412_14374_amd import inputs as inp

    def spec_of(t):
        return so.StageSpec(n_layers=t.n_layers, d_model=t.d_model, n_q_heads=t.n_q_heads, n_kv_heads=t.n_kv_heads,
                            head_dim=t.head_dim, d_ffn=t.d_ffn, seq_len=t.seq_len, microbatch=t.microbatch,
                            norm=t.norm, act=t.act, use_bias=bool(t.use_bias), rope=bool(t.rope),
                            rope_theta=t.rope_theta, norm_eps=t.norm_eps, loss_head=bool(t.loss_head), vocab=t.vocab)

    if config == "C1":
        base = inp.C1
        spec = spec_of(base)
        params, x, cot, tg = inp.draw_stage_inputs(base, so.layer_param_shapes(spec), None)
        tasks = [(i, "fwd" if ty == B.JPP_FWD else "bwd", s_)
                 for (i, ty, s_) in B.jpp_schedule_make(base.sched, base.P, base.rank, base.V, base.n_microbatches)]
        flops = so.algorithmic_flops_per_microbatch(spec) * base.n_microbatches

        def whole_run():
            t0 = time.perf_counter()
            for _ in range(20):
                so.run_task_list(spec, params, tasks, x, cot, tg)
            return (time.perf_counter() - t0) / 20
        all_cores = whole_run()
        try:
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):
                one_core = whole_run()
        except Exception:
            one_core = None
        return {"value": flops / all_cores / 1e12, "unit": "TFLOP/s", "cores": oracle_threads(), "kind": "oracle",
                "seconds": all_cores, "seconds_one_core": one_core,
                "steps_per_s": 1.0 / all_cores, "steps_per_s_one_core": (1.0 / one_core) if one_core else None,
                "microbatches_per_s_extrapolated_to_workload": base.n_microbatches / all_cores,
                "sample": "fp64 numpy oracle, the WHOLE C1 step (4 microbatches, forward + backward, GPipe list), "
                          f"mean of 20 runs, on all cores and on one; {flops / 1e9:.2f} algorithmic GFLOP per step"}
    kw = dict(CPU_TWINS[config])
    ratio = w.n_q_heads // w.n_kv_heads
    t = replace(w, n_layers=1, n_kv_heads=kw["n_q_heads"] // ratio, n_microbatches=1, **kw)
    spec = spec_of(t)
    rng = np.random.default_rng(0)
    p = {"layers": [{k: rng.standard_normal(shp) * 0.02 for k, shp in so.layer_param_shapes(spec)}]}
    if t.loss_head:
        p["head"] = {k: rng.standard_normal(shp) * 0.02 for k, shp in so.head_param_shapes(spec)}
    x = rng.standard_normal((t.microbatch, t.seq_len, t.d_model))
    c = None if t.loss_head else rng.standard_normal((t.microbatch, t.seq_len, t.d_model))
    tg = rng.integers(0, t.vocab, size=(t.microbatch, t.seq_len)).astype(np.int32) if t.loss_head else None
    t0 = time.perf_counter()
    out, cache = so.stage_forward(spec, p, x, tg)
    so.stage_backward(spec, p, cache, c)
    dt = time.perf_counter() - t0
    flops = so.algorithmic_flops_per_microbatch(spec)
    what = ["LayerNorm", "RMSNorm"][t.norm] + ", " + ["GeLU", "tanh-GeLU", "SwiGLU"][t.act] + \
        (", RoPE" if t.rope else "") + (f", {t.n_q_heads}/{t.n_kv_heads} query/kv heads" if ratio > 1 else "") + \
        (f", final norm + LM head {t.vocab} + cross-entropy" if t.loss_head else "")
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle_threads(), "kind": "oracle",
            "seconds": dt,
            "microbatches_per_s_extrapolated_to_workload": (flops / dt) / algorithmic_flops_per_microbatch(w),
            "sample": "fp64 numpy oracle, forward+backward of ONE microbatch of ONE layer of a structure-matched twin of "
                      f"{config} (d_model {t.d_model}, {t.n_q_heads} heads x {t.head_dim}, FFN {t.d_ffn}, seq {t.seq_len}, "
                      f"{what}); {flops / 1e9:.0f} algorithmic GFLOP; the workload's rate is extrapolated by FLOP count"}


def bench_kernels(w, torch, B, inp, fixed_reps=False):
    """Every kernel of one layer (forward and backward) alone on the device at the
    configuration's shapes: milliseconds, achieved rate and fraction of the roofline that bounds
    it (MFMA peak for GEMMs and attention with the counted FLOPs, HBM peak for the row-wise and
    element-wise kernels with their algorithmic bytes).  One JSON line per kernel."""
    dev = "cuda:0"
    bf = torch.bfloat16
    T, d, f = w.tokens, w.d_model, w.d_ffn
    Tg = T * max(1, w.wgrad_group)     # a weight gradient contracts over its whole group's tokens
    nq, nkv = w.n_q_heads * w.head_dim, w.n_kv_heads * w.head_dim
    nqkv, f1 = nq + 2 * nkv, (2 * f if w.act == inp.ACT_SWIGLU else f)
    strm = torch.cuda.current_stream().cuda_stream

    warm = [False]

    def timed(fn, reps=5):
        if not warm[0]:
            # the first kernels after idle run at a lower clock: bring the device up to load first
            for _ in range(30):
                fn()
            warm[0] = True

        def once(n):
            fn(); fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        ms = once(reps)
        if ms * reps < 20.0 and not fixed_reps:
            # a short kernel: five launches are over before the queue is full and the clock has
            # settled; time 20 ms of back-to-back launches instead, as a step issues them
            ms = once(min(2000, int(20.0 / ms) + 1))
        return ms

    def emit(name, shape, ms, work, bound):
        peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_HBM_GBS
        ach = work / ms / (1e9 if bound == "mfma" else 1e6)
        print(json.dumps({"kernel": name, "shape": shape, "ms": round(ms, 4), "bound": bound,
                          "achieved": round(ach, 1), "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
                          "peak": peak, "frac": round(ach / peak, 3)}), flush=True)

    gemms = [("qkv fwd", T, nqkv, d, 0, 0, 0), ("attn-out fwd", T, d, nq, 0, 0, 0), ("ffn-up fwd", T, f1, d, 0, 0, 0),
             ("ffn-down fwd", T, d, f, 0, 0, 0), ("qkv dgrad", T, d, nqkv, 0, 1, 0), ("attn-out dgrad", T, nq, d, 0, 1, 0),
             ("ffn-up dgrad", T, d, f1, 0, 1, 0), ("ffn-down dgrad", T, f, d, 0, 1, 0),
             ("qkv wgrad", nqkv, d, Tg, 1, 1, 2), ("attn-out wgrad", d, nq, Tg, 1, 1, 2),
             ("ffn-up wgrad", f1, d, Tg, 1, 1, 2), ("ffn-down wgrad", d, f, Tg, 1, 1, 2)]
    for name, M, N, K, aks, bks, mode in gemms:
        A = torch.randn((K, M) if aks else (M, K), device=dev).to(bf)
        Bm = (torch.randn((K, N) if bks else (N, K), device=dev) * 0.02).to(bf)
        Cc = torch.zeros((M, N), dtype=bf if mode == 0 else torch.float32, device=dev)
        need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, mode)
        ws = torch.empty(max(need // 4, 4), dtype=torch.float32, device=dev)
        ms = timed(lambda: B.jpp_op_gemm_ws(B.JPP_BF16, M, N, K, A.data_ptr(), M if aks else K, aks, Bm.data_ptr(),
                                            N if bks else K, bks, Cc.data_ptr(), N, mode, None, None,
                                            ws.data_ptr() if need else None, need, strm))
        emit("gemm " + name, f"{M}x{N}x{K}", ms, 2.0 * M * N * K, "mfma")
        del A, Bm, Cc, ws
    mb, seq, Hq, Hkv, hd = w.microbatch, w.seq_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    qkv = torch.randn(T, nqkv, device=dev).to(bf)
    do = torch.randn(T, nq, device=dev).to(bf)
    out = torch.zeros(T, nq, dtype=bf, device=dev)
    lse = torch.zeros(mb, Hq, seq, dtype=torch.float32, device=dev)
    dqkv, delta = torch.zeros_like(qkv), torch.zeros_like(lse)
    fl = 2.0 * mb * Hq * seq * seq * hd
    ms = timed(lambda: B.jpp_op_attention_fwd(B.JPP_BF16, mb, seq, Hq, Hkv, hd, qkv.data_ptr(), out.data_ptr(),
                                              lse.data_ptr(), strm))
    emit("attention fwd", f"mb{mb} seq{seq} Hq{Hq} Hkv{Hkv} hd{hd}", ms, fl, "mfma")
    # with the scratch the executor gives it (grouped-query shapes spread a kv head's query heads)
    need = B.jpp_op_attention_bwd_scratch_bytes(B.JPP_BF16, mb, seq, Hq, Hkv, hd)
    scr = torch.empty(max(need // 4, 4), dtype=torch.float32, device=dev)
    ms = timed(lambda: B.jpp_op_attention_bwd_ws(B.JPP_BF16, mb, seq, Hq, Hkv, hd, qkv.data_ptr(), out.data_ptr(),
                                                 lse.data_ptr(), do.data_ptr(), dqkv.data_ptr(), delta.data_ptr(),
                                                 scr.data_ptr() if need else None, need, strm))
    emit("attention bwd (delta + dK/dV + dQ kernels)", f"mb{mb} seq{seq} Hq{Hq} Hkv{Hkv} hd{hd}", ms, 2 * fl, "mfma")
    del qkv, do, out, lse, dqkv, delta, scr
    x = torch.randn(T, d, device=dev).to(bf)
    y, dy, dx = torch.zeros_like(x), torch.randn(T, d, device=dev).to(bf), torch.zeros_like(x)
    gam, bet = torch.ones(d, dtype=bf, device=dev), torch.zeros(d, dtype=bf, device=dev)
    stats = torch.zeros(2 * T, dtype=torch.float32, device=dev)
    gg, gb = torch.zeros(d, dtype=torch.float32, device=dev), torch.zeros(d, dtype=torch.float32, device=dev)
    part = torch.zeros(B.jpp_op_colreduce_scratch(T, d), dtype=torch.float32, device=dev)
    ms = timed(lambda: B.jpp_op_norm_fwd(B.JPP_BF16, w.norm, T, d, w.norm_eps, x.data_ptr(), gam.data_ptr(),
                                         bet.data_ptr(), y.data_ptr(), stats.data_ptr(), strm))
    emit("norm fwd", f"{T}x{d}", ms, 4.0 * T * d, "hbm")
    ms = timed(lambda: B.jpp_op_norm_bwd(B.JPP_BF16, w.norm, T, d, x.data_ptr(), gam.data_ptr(), stats.data_ptr(),
                                         dy.data_ptr(), None, dx.data_ptr(), gg.data_ptr(), gb.data_ptr(),
                                         part.data_ptr(), strm))
    emit("norm bwd (+ gain/offset gradient partials and finish)", f"{T}x{d}", ms, 6.0 * T * d, "hbm")
    del x, y, dy, dx
    h = torch.randn(T, f1, device=dev).to(bf)
    a_ = torch.zeros(T, f, dtype=bf, device=dev)
    da, dh = torch.randn(T, f, device=dev).to(bf), torch.zeros(T, f1, dtype=bf, device=dev)
    swiglu = w.act == inp.ACT_SWIGLU
    ms = timed(lambda: B.jpp_op_act_fwd(B.JPP_BF16, w.act, T, f, h.data_ptr(), a_.data_ptr(), strm))
    emit("activation fwd", f"{T}x{f}", ms, (6.0 if swiglu else 4.0) * T * f, "hbm")
    ms = timed(lambda: B.jpp_op_act_bwd(B.JPP_BF16, w.act, T, f, h.data_ptr(), da.data_ptr(), dh.data_ptr(), strm))
    emit("activation bwd", f"{T}x{f}", ms, (10.0 if swiglu else 6.0) * T * f, "hbm")
    if not swiglu:
        # the same two activations applied by the epilogues of the GEMMs around them
        n2 = torch.randn(T, d, device=dev).to(bf)
        W1 = (torch.randn(f, d, device=dev) * 0.02).to(bf)
        b1 = torch.zeros(f, dtype=bf, device=dev)
        need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, T, f, d, 0)
        ws = torch.empty(max(need // 4, 4), dtype=torch.float32, device=dev)
        ms = timed(lambda: B.jpp_op_gemm_gelu(T, f, d, n2.data_ptr(), d, 0, W1.data_ptr(), d, 0, h.data_ptr(), f,
                                              b1.data_ptr(), w.act, 0, a_.data_ptr(), ws.data_ptr() if need else None,
                                              need, strm))
        emit("gemm ffn-up fwd with GeLU epilogue (h and a)", f"{T}x{f}x{d}", ms, 2.0 * T * f * d, "mfma")
        del n2, W1
        dy2 = torch.randn(T, d, device=dev).to(bf)
        W2 = (torch.randn(d, f, device=dev) * 0.02).to(bf)
        ms = timed(lambda: B.jpp_op_gemm_gelu(T, f, d, dy2.data_ptr(), d, 0, W2.data_ptr(), f, 1, dh.data_ptr(), f,
                                              None, w.act, 1, h.data_ptr(), ws.data_ptr() if need else None, need, strm))
        emit("gemm ffn-down dgrad with GeLU' epilogue (dh)", f"{T}x{f}x{d}", ms, 2.0 * T * f * d, "mfma")
        del dy2, W2, ws
    del h, a_, da, dh
    if w.loss_head:
        # the last stage's head: logits (fp32), cross-entropy with its gradient (bf16), the two backward GEMMs
        V = w.vocab
        nf = torch.randn(T, d, device=dev).to(bf)
        Wh = (torch.randn(V, d, device=dev) * 0.02).to(bf)
        z = torch.zeros(T, V, dtype=torch.float32, device=dev)
        dz = torch.zeros(T, V, dtype=bf, device=dev)
        dn = torch.zeros(T, d, dtype=bf, device=dev)
        G = torch.zeros(V, d, dtype=torch.float32, device=dev)
        tgt = torch.randint(0, V, (T,), dtype=torch.int32, device=dev)
        row_loss, loss = torch.zeros(T, dtype=torch.float32, device=dev), torch.zeros(1, dtype=torch.float32, device=dev)

        def gemm(M, N, K, A, lda, aks, Bm, ldb, bks, Cc, mode):
            need = B.jpp_op_gemm_workspace_bytes(B.JPP_BF16, M, N, K, mode)
            ws = torch.empty(max(need // 4, 4), dtype=torch.float32, device=dev)
            return timed(lambda: B.jpp_op_gemm_ws(B.JPP_BF16, M, N, K, A.data_ptr(), lda, aks, Bm.data_ptr(), ldb, bks,
                                                  Cc.data_ptr(), N, mode, None, None, ws.data_ptr() if need else None,
                                                  need, strm))
        emit("gemm head fwd (fp32 logits)", f"{T}x{V}x{d}", gemm(T, V, d, nf, d, 0, Wh, d, 0, z, 1), 2.0 * T * V * d, "mfma")
        ms = timed(lambda: B.jpp_op_cross_entropy(B.JPP_BF16, T, V, z.data_ptr(), tgt.data_ptr(), dz.data_ptr(),
                                                  row_loss.data_ptr(), loss.data_ptr(), strm))
        emit("cross-entropy (loss + dz)", f"{T}x{V}", ms, 6.0 * T * V, "hbm")
        emit("gemm head dgrad", f"{T}x{d}x{V}", gemm(T, d, V, dz, V, 0, Wh, d, 1, dn, 0), 2.0 * T * V * d, "mfma")
        # the head's weight gradient contracts over its group like the layers' (dz and the
        # normalised activations of the group's members are contiguous in the stash)
        del z, dz, nf
        dzg = torch.zeros(Tg, V, dtype=bf, device=dev).normal_(0, 1e-3)
        nfg = torch.randn(Tg, d, device=dev).to(bf)
        emit("gemm head wgrad", f"{V}x{d}x{Tg}", gemm(V, d, Tg, dzg, V, 1, nfg, d, 1, G, 2), 2.0 * Tg * V * d, "mfma")


def bench_pipeline(a, w, torch, B, inp):
    """The configuration as a whole pipeline on one device: P actors with one virtual stage of
    w.n_layers layers each (so P times the single-actor model), every actor running its own
    1F1B list of the same M microbatches, outputs handed from actor to actor."""
    from dataclasses import replace
    from paper_2412_14374_amd.harness import Pipeline
    wp = replace(w, V=1, sched=inp.SCHED_1F1B, rank=0)
    P, M = wp.P, wp.n_microbatches
    lists = [B.jpp_schedule_make(inp.SCHED_1F1B, P, r, 1, M) for r in range(P)]
    pipe = Pipeline(wp, lists)
    pipe.set_params_random(seed=0)
    pipe.bind_random(seed=1)
    for _ in range(a.warmup):
        pipe.zero_grads()
        pipe.run()
    pipe.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        pipe.zero_grads()
        pipe.run()
    pipe.sync()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / a.steps * 1e3
    # per actor: the body layers; the head, if any, on the last actor only
    body = algorithmic_flops_per_microbatch(replace(wp, loss_head=0))
    flops = (body * P + (algorithmic_flops_per_microbatch(wp) - body)) * M
    finite = all(bool(torch.isfinite(s.grads_tensor(0)).all().item()) for s in pipe.actors)
    pipe.close()
    print(json.dumps({"metric": "whole pipeline on one GPU, fwd+bwd TFLOP/s", "value": flops / (ms * 1e-3) / 1e12,
                      "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms,
                      "dtype": "bf16" if w.dtype == inp.DT_BF16 else "f32", "data": "synthetic",
                      "pct_of_bf16_mfma_peak": 100.0 * flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                      "grads_finite": finite,
                      "config": {"workload": w.name + " as a pipeline", "actors": P, "layers_per_actor": w.n_layers,
                                 "n_microbatches": M, "schedule": "1f1b per actor"}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the secondary entries of the default run (the same workload with per-task weight "
                         "gradients, and C2 / C3 / C5 with the same defaults)")
    ap.add_argument("--remat", action="store_true",
                    help="rematerialisation: keep only each layer's input, recompute the layer in the backward "
                         "(the recomputation is not counted in the TFLOP/s)")
    ap.add_argument("--wgrad-group", type=int, default=None,
                    help="microbatches per weight-gradient group (jpp_layer_config.wgrad_group); 1 = every "
                         "backward task accumulates its own weight gradients; default min(8, M), 1 with --remat")
    ap.add_argument("--schedule", choices=["gpipe", "1f1b", "interleaved"], default=None,
                    help="override the configuration's schedule (same P, rank, V)")
    ap.add_argument("--optimizer", choices=["sgd", "adamw"], default=None,
                    help="end every step with the parameter update (jpp_stage_apply_gradients) and report "
                         "its own bandwidth; off by default: the headline metric is the stage's fwd+bwd")
    ap.add_argument("--kernels", action="store_true",
                    help="time every kernel of one layer alone at the configuration's shapes and print one "
                         "JSON line per kernel with its rate against its own roofline")
    ap.add_argument("--fixed-reps", action="store_true",
                    help="with --kernels: 2 + 5 launches per kernel whatever their length (keeps a counter pass of "
                         "the profiler short); by default kernels shorter than 4 ms are timed over 20 ms of launches")
    ap.add_argument("--streams", type=int, choices=[1, 2, 3], default=None,
                    help="streams a run computes on: 3 = forward, input-gradient chain and weight-gradient GEMMs "
                         "on their own streams, 2 = forward + backward, 1 = everything on one; default: the "
                         "library picks 1 or 3 from the stage's GEMM sizes")
    ap.add_argument("--fused-activation", type=int, choices=[0, 1, 2, 3], default=None,
                    help="where GeLU is evaluated (jpp_set_fused_activation): bit 0 = in the FFN-up GEMM's epilogue, "
                         "bit 1 = in the FFN-down input-gradient GEMM's; default: the library's (3)")
    ap.add_argument("--pipeline", action="store_true",
                    help="run the configuration's layers as a whole pipeline of P actors on this one GPU "
                         "(one layer-stack slice per actor, 1F1B lists, real stage-to-stage hand-offs) "
                         "instead of a single actor; prints a line of its own")
    ap.add_argument("--kernel-only", action="store_true",
                    help="profiling aid: run only the dominant kernel's launches plus the reference copies that "
                         "calibrate the profiler's counters (one of 1 GiB, sixteen of 64 MiB)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2412_14374_amd import binding as B
    from paper_2412_14374_amd import inputs as inp
    from paper_2412_14374_amd.harness import Stage

    B.lib()                                     # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    w = inp.CONFIGS[a.config]
    B.jpp_set_stream_mode(-1 if a.streams is None else 3 - a.streams)
    B.jpp_set_fused_activation(-1 if a.fused_activation is None else a.fused_activation)
    from dataclasses import replace
    kind = {"gpipe": inp.SCHED_GPIPE, "1f1b": inp.SCHED_1F1B, "interleaved": inp.SCHED_INTERLEAVED,
            None: w.sched}[a.schedule]
    # weight-gradient groups: by default 8 microbatches (for C4: P, one run of backwards of a
    # virtual stage in the interleaved schedule); rematerialisation drops what a group keeps
    # (the whole-pipeline variant holds P actors' stashes in one HBM: per-task weight gradients there)
    group = a.wgrad_group if a.wgrad_group is not None else (1 if a.remat or a.pipeline else min(8, w.n_microbatches))
    w = replace(w, remat=1 if a.remat else 0, sched=kind, wgrad_group=group)
    if a.kernel_only:
        # References for the profiler's counters.  Bandwidth-bound: a 1 GiB copy (every read
        # misses every cache: the scale of FETCH_SIZE / WRITE_SIZE) and 16 copies of the same
        # 64 MiB (larger than the L2s together, far smaller than the 256 MB last-level cache).
        # Latency-bound (a few thousand 128-byte reads in flight, no queueing): 4096 random rows
        # of 128 bytes gathered (jpp_op_embed_fwd) from a 4 GiB table, of which that cache can
        # hold a sixteenth -- HBM answers -- and from the 64 MiB buffer right after its copies --
        # the last-level cache answers.  TCC_EA0_RDREQ_LEVEL / TCC_EA0_RDREQ of each is the
        # mean time a read request of the L2s spends outside them under that condition.
        dev = "cuda:0"
        strm = torch.cuda.current_stream().cuda_stream
        rows_out = torch.empty(4096, 64, dtype=torch.bfloat16, device=dev)

        def gather(table, n_rows):
            ids = torch.randint(0, n_rows, (4096,), dtype=torch.int32, device=dev)
            torch.cuda.synchronize()
            B.jpp_op_embed_fwd(B.JPP_BF16, 4096, 64, n_rows, ids.data_ptr(), table.data_ptr(), rows_out.data_ptr(), strm)
            torch.cuda.synchronize()

        table = torch.ones(1 << 31, dtype=torch.bfloat16, device=dev)         # 4 GiB
        gather(table, (1 << 31) // 64)
        del table
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device=dev)           # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        small = torch.ones(1 << 25, dtype=torch.bfloat16, device=dev)         # 64 MiB
        small2 = torch.empty_like(small)
        for _ in range(16):
            small2.copy_(small)
        torch.cuda.synchronize()
        gather(small, (1 << 25) // 64)
        del small, small2
        avg_ms, flops = time_dominant_kernel(w, torch, B)
        print(json.dumps({"kernel_only": True, "avg_launch_ms": avg_ms, "flops_per_launch": flops,
                          "tflops": flops / avg_ms / 1e9}))
        return
    if a.kernels:
        return bench_kernels(w, torch, B, inp, a.fixed_reps)
    if a.pipeline:
        return bench_pipeline(a, w, torch, B, inp)
    opt_kind = {None: None, "sgd": B.JPP_OPT_SGD, "adamw": B.JPP_OPT_ADAMW}[a.optimizer]
    r = run_stage(w, a.steps, a.warmup, torch, B, inp, Stage, opt_kind, a.optimizer)
    tflops, ms_per_step, per_step = r["tflops"], r["ms_per_step"], r["per_step"]
    mb_per_s, finite, opt_info = r["microbatches_per_s"], r["finite"], r["optimizer"]
    streams, arena_gb, stash_slots = r["streams"], r["arena_gb"], r["stash_slots"]

    out = {
        "metric": "stage fwd+bwd TFLOP/s, % of bf16 MFMA peak, microbatches/s (1 GPU)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == inp.DT_BF16 else "f32", "data": "synthetic",
        "pct_of_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
        "microbatches_per_s": mb_per_s,
        "ms_per_step_min": per_step[0], "ms_per_step_median": per_step[len(per_step) // 2],
        # the same time with attention counted over the full score matrix (no causal halving)
        "value_full_attention_count": tflops * flops_full_attention(w) / algorithmic_flops_per_microbatch(w),
        "grads_finite": finite,
        "optimizer": opt_info,
        "config": {"workload": w.name, "layers_per_stage": w.n_layers, "virtual_stages": w.V,
                   "d_model": w.d_model, "heads": w.n_q_heads, "kv_heads": w.n_kv_heads, "d_ffn": w.d_ffn,
                   "seq_len": w.seq_len, "microbatch": w.microbatch, "n_microbatches": w.n_microbatches,
                   "schedule": ["gpipe", "1f1b", "interleaved-1f1b"][w.sched], "P": w.P, "rank": w.rank,
                   "remat": bool(w.remat), "wgrad_group": max(1, w.wgrad_group), "streams": streams, "arena_gb": arena_gb, "stash_slots": stash_slots,
                   "algorithmic_tflop_per_microbatch": algorithmic_flops_per_microbatch(w) / 1e12},
    }
    out["clocks"] = r["clocks"]
    default_run = (a.config == "C4" and a.wgrad_group is None and not a.remat and a.schedule is None
                   and a.streams is None and a.optimizer is None)
    if default_run and not a.headline_only:
        # Section 3.1 has every backward task add its own microbatch's gradients; the headline
        # defers them to groups of 8 (more stash memory, a longer contraction).  The per-task form
        # of the same workload, in the same run:
        w1 = replace(w, wgrad_group=1)
        out["per_task_wgrad"] = brief(w1, run_stage(w1, 3, 1, torch, B, inp, Stage), 3, 1)
        # the other bf16 configurations with the same defaults
        out["other_configs"] = []
        for name in ("C2", "C3", "C5"):
            wc = inp.CONFIGS[name]
            wc = replace(wc, wgrad_group=min(8, wc.n_microbatches))
            out["other_configs"].append(brief(wc, run_stage(wc, 5, 2, torch, B, inp, Stage), 5, 2))
    if w.dtype == inp.DT_BF16:
        avg_ms, flops_per_launch = time_dominant_kernel(w, torch, B)
        progress(f"dominant kernel timed: {avg_ms:.3f} ms per launch")
        shapes = wgrad_shapes(w)
        # L2 <-> fabric bytes per launch from the profiler, for the C4 shapes only: groups of 8 / per task
        traffic = {8: 33.8e9, 1: 6.65e9}.get(max(1, w.wgrad_group)) if a.config == "C4" else None
        ach = flops_per_launch / (avg_ms * 1e-3) / 1e12
        out["roofline"] = {"bound": "mfma", "kernel": "gemm_bf16_kernel<..., k-strided A, k-strided B> "
                           "(weight gradient with fused fp32 accumulate)",
                           "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                           "frac": ach / PEAK_BF16_TFLOPS, "avg_launch_ms": avg_ms,
                           "flops_per_launch": flops_per_launch,
                           "traffic": traffic, "traffic_unit": "bytes/launch",
                           # not read in this run: the counters need the profiler (one pass each)
                           "traffic_source": ("profiles/gemm_wgrad_c4_hbm_traffic.md: rocprofv3 --pmc FETCH_SIZE, then "
                                              "WRITE_SIZE, of `bench.py --kernel-only`, scaled by the same counters "
                                              "of a 1 GiB copy; bytes between the L2s and the fabric, of which the "
                                              "256 MB last-level cache serves at least three quarters (mean read "
                                              "time 594 L2 cycles against 519 / 857 for that cache / HBM idle); "
                                              "27-32 GB of it fetched, varying from run to run")
                           if traffic else None,
                           "algorithmic_bytes_per_launch": sum(8.0 * m * n + 2.0 * k * (m + n) for m, n, k in shapes)
                           / len(shapes)}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a.config, w)
        progress(f"oracle timed on the host: {out['cpu_baseline']['seconds']:.1f} s")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
