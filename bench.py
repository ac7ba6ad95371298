#!/usr/bin/env python3
"""Benchmark of the token-sharded layer forward (one MI355X).

A step is one pass of the whole hot path (gather + norm, q/k/v shard GEMM with the rotary embedding, partial
attention over every (query-shard, kv-shard) pair with the running log-sum-exp merge, o projection,
norm, FFN shard GEMMs, scatter) over one batch of synthetic input that is already resident in HBM.
Prints ONE JSON line.  The float64 CPU oracle is timed next to it (cpu_baseline) on the host cores; the
other configurations of the list are timed as well, each with its own roofline record.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16
FP32_VECTOR_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_{key}_hbm_traffic.md")


def measured_traffic_bytes(key):
    """HBM bytes per launch of the dominant kernel, from the tracked summary of the rocprofv3 FETCH_SIZE / WRITE_SIZE
    runs of this workload (its line 'roofline.traffic bytes per launch: <number>'); None when there is none."""
    try:
        with open(TRAFFIC_PROFILE.format(key=key)) as f:
            for line in f:
                if line.startswith("roofline.traffic bytes per launch:"):
                    return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def layer_flops(cfg):
    T = cfg.batch * cfg.seq_len
    D, H, Hkv, d, f = cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ff
    qkv = 2.0 * T * D * (H + 2 * Hkv) * d
    o = 2.0 * T * (H * d) * D
    up = 2.0 * T * D * f * (2 if cfg.act == "swiglu" else 1)
    down = 2.0 * T * f * D
    attn = 4.0 * d * H * cfg.batch * cfg.seq_len * (cfg.seq_len + 1) / 2      # causal-useful pairs only
    return {"qkv_gemm": qkv, "o_proj": o, "ffn_up": up, "ffn_down": down, "attention": attn,
            "total": qkv + o + up + down + attn}


def device_inputs(cfg, seed):
    """Random-init weights and hidden states drawn on the device (bf16 grid for bf16 configs)."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    D, H, Hkv, d, f, s = cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ff, cfg.sigma

    def normal(shape, std):
        return (torch.randn(shape, device="cuda", generator=g, dtype=torch.float32) * std).to(tdt)

    # q, k, v weights live in one [(H + 2 H_KV) d, D] allocation (the usual fused layout); the library is
    # handed the three views and recognises that they are contiguous
    wqkv = normal(((H + 2 * Hkv) * d, D), s)
    w = {"wq": wqkv[:H * d], "wk": wqkv[H * d:(H + Hkv) * d], "wv": wqkv[(H + Hkv) * d:],
         "wo": normal((D, H * d), s), "w_up": normal((f, D), s), "w_down": normal((D, f), s),
         "norm1_g": (1.0 + normal((D,), s).float()).to(tdt), "norm2_g": (1.0 + normal((D,), s).float()).to(tdt)}
    if cfg.act == "swiglu":
        w["w_gate"] = normal((f, D), s)
    if cfg.norm == "layernorm":
        w["norm1_b"], w["norm2_b"] = normal((D,), s), normal((D,), s)
    if cfg.bias:
        bqkv = normal(((H + 2 * Hkv) * d,), s)
        w.update(bq=bqkv[:H * d], bk=bqkv[H * d:(H + Hkv) * d], bv=bqkv[(H + Hkv) * d:], bo=normal((D,), s),
                 b_up=normal((f,), s), b_down=normal((D,), s))
    h = normal((cfg.batch, cfg.seq_len, D), 1.0)
    return w, h


def time_steps(fn, steps):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def per_step_stats(fn, steps):
    """Each step timed on its own with events on the current stream: median, mean, 95 % interval of the mean."""
    import statistics
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    mean = statistics.fmean(ms)
    half = 1.96 * statistics.stdev(ms) / len(ms) ** 0.5 if len(ms) > 1 else 0.0
    return {"median_ms": statistics.median(ms), "mean_ms": mean, "ci95_ms": [mean - half, mean + half], "n": len(ms)}


def measured_ceilings(cas):
    """What this device sustains: MFMA-only kernels with random bf16 operands, and a plain device copy."""
    import torch
    out = {"mfma_bf16_registers_tflops": cas.cascade_mfma_ceiling(0, 200000),
           "mfma_bf16_lds_operands_tflops": cas.cascade_mfma_ceiling(1, 200000)}
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    out["copy_read_plus_write_GBs"] = 5 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return out


def vendor_gemm_reference(cfg):
    """For scale only, never used by the product: the vendor library's plain bf16 GEMM (torch.matmul, weight as
    [N, K]) on the four GEMM shapes of the layer, without the epilogues the shard GEMMs fuse (rotary, SwiGLU,
    residual).  TFLOP/s per shape."""
    import torch
    T, D, f = cfg.batch * cfg.seq_len, cfg.d_model, cfg.d_ff
    qw, hw = (cfg.n_heads + 2 * cfg.n_kv_heads) * cfg.head_dim, cfg.n_heads * cfg.head_dim
    shapes = {"qkv_gemm": (T, qw, D), "o_proj": (T, D, hw), "ffn_up": (T, (2 if cfg.act == "swiglu" else 1) * f, D),
              "ffn_down": (T, D, f)}
    out = {}
    for name, (m, n, k) in shapes.items():
        x = torch.randn(m, k, device="cuda", dtype=torch.bfloat16)
        w = torch.randn(n, k, device="cuda", dtype=torch.bfloat16)
        fn = lambda: x @ w.t()
        for _ in range(40):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(40):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 40
        out[name] = {"ms": ms, "tflops": 2.0 * m * n * k / (ms * 1e-3) / 1e12}
        del x, w
    return out


class Workload:
    """Inputs, plan, descriptors and workspaces of one configuration, resident on the device."""

    def __init__(self, cas, cfg):
        import torch
        from cascade_inputs import config_seed, make_assignment
        self.cas, self.cfg = cas, cfg
        seed = config_seed(cfg)
        self.a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, seed)
        self.w, self.h = device_inputs(cfg, seed)
        self.plan = cas.cascade_plan_create(cfg.batch, cfg.seq_len, cfg.n_shards, self.a)
        self.wts = cas.make_layer_weights(self.w)
        self.h_out = torch.empty_like(self.h)
        self.desc = cas.make_layer_desc(cfg, cas.ATTN_FUSED, cas.ROWS_ORIGINAL)
        self.ws = cas.new_workspace(cas.cascade_layer_workspace_bytes(self.plan, self.desc))
        self.flops = layer_flops(cfg)

    def step(self):
        self.cas.cascade_layer_forward(self.plan, self.desc, self.wts, self.h, self.h_out, self.ws)

    def timed(self, steps, warmup):
        """W untimed steps, then exactly K steps between two device synchronisations (host clock)."""
        for _ in range(warmup):
            self.step()
        return time_steps(self.step, steps)

    def staged(self, steps):
        return staged_times(self.cas, self.plan, self.desc, self.wts, self.h, self.h_out, self.ws, steps)

    def materialised(self, steps):
        """MATERIALISED mode: partial attention writes m, e, u~ to HBM, the merge reads them back."""
        cas = self.cas
        desc_m = cas.make_layer_desc(self.cfg, cas.ATTN_MATERIALISED, cas.ROWS_ORIGINAL)
        ws_m = cas.new_workspace(cas.cascade_layer_workspace_bytes(self.plan, desc_m))
        step = lambda: cas.cascade_layer_forward(self.plan, desc_m, self.wts, self.h, self.h_out, ws_m)
        for _ in range(3):
            step()
        sec = time_steps(step, steps)
        stages = staged_times(cas, self.plan, desc_m, self.wts, self.h, self.h_out, ws_m, steps)
        # the merge alone, launched back to back on the partials the last pass left in the workspace
        m, e, u = cas.cascade_layer_partials(self.plan, desc_m, ws_m, self.cfg.batch, self.cfg.n_heads, self.cfg.head_dim)
        import torch
        o = torch.empty(self.cfg.batch, self.cfg.seq_len, self.cfg.n_heads * self.cfg.head_dim, device="cuda",
                        dtype=self.h.dtype)
        merge = lambda: cas.cascade_lse_merge(self.plan, m, e, u, o, self.cfg.n_heads, self.cfg.n_kv_heads,
                                              self.cfg.head_dim)
        for _ in range(3):
            merge()
        merge_alone = event_time(merge, max(10, steps))
        self.step()                                # leave the fused result in h_out
        torch.cuda.synchronize()
        return sec, stages, merge_alone

    def graph_replay(self, steps, warmup):
        """The same step captured once in a HIP graph and replayed: max(W, 60) untimed replays, then K timed ones."""
        import torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step()
        torch.cuda.current_stream().wait_stream(side)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.step()
        for _ in range(max(warmup, 60)):           # capture left the device idle: at least 60 replays to be busy again
            g.replay()
        return time_steps(g.replay, steps)


def event_time(fn, reps):
    """Average duration of fn's device work over `reps` back-to-back calls, HIP events on the current stream (s)."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def dominant_kernel(cfg):
    """The FFN up (+ gate) shard GEMM instance the launcher picks for this workload (the dominant kernel); the
    committed rocprofv3 kernel statistics show the same names."""
    if cfg.dtype != "bf16":
        return "gemm_f32_kernel (FFN up shard GEMM)"
    known = {"C3-llama3-8b-bf16": "gemm2_kernel<256,224,4,1,64,2,true,false,false>",
             "C4-llama3-8b-long-bf16": "gemm2_kernel<256,256,2,2,64,2,true,false,false>",
             "C5-llama3-70b-bf16": "gemm2_kernel<256,256,2,2,64,2,true,false,false>",
             "C2-gpt2-small-bf16": "gemm2_kernel<256,192,2,2,64,2,false,false,false>"}
    return known.get(cfg.name, "gemm2_kernel") + " (FFN up shard GEMM" + (", gate and up fused)" if cfg.act == "swiglu" else ")")


def roofline_record(cfg, flops, stages, key):
    bf16 = cfg.dtype == "bf16"
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else FP32_VECTOR_PEAK_TFLOPS
    tf = flops["ffn_up"] / (stages["ffn_up"] * 1e-3) / 1e12
    return {"bound": "mfma" if bf16 else "alu", "kernel": dominant_kernel(cfg), "achieved": tf, "peak": peak,
            "unit": "TFLOP/s", "frac": tf / peak, "traffic": measured_traffic_bytes(key),
            "avg_launch_ms": stages["ffn_up"], "flops_per_launch": flops["ffn_up"],
            "timing": "HIP events around the kernel on its stream, mean over separate instrumented passes"}


def staged_times(cas, plan, desc, wts, h, h_out, ws, steps):
    import torch
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(cas.N_STAGE_EVENTS)] for _ in range(steps)]
    for row in evs:
        for ev in row:
            ev.record()                            # creates the underlying HIP event
    torch.cuda.synchronize()
    for row in evs:
        cas.cascade_layer_forward_staged(plan, desc, wts, h, h_out, ws, row)
    torch.cuda.synchronize()
    out = {}
    for i, name in enumerate(cas.STAGE_NAMES):
        out[name] = sum(row[i].elapsed_time(row[i + 1]) for row in evs) / steps
    out["total"] = sum(row[0].elapsed_time(row[-1]) for row in evs) / steps
    return out


def run_m_split(cas, cfg, steps):
    """The same layer with distinct shardings: (c, delta) row shards and their m-split as key/value
    shards (c = 8, delta = c * n_shards, m = 2): beta = 2 alpha partials per row."""
    import torch
    from cascade_inputs import config_seed
    c = 8
    a, alpha = cas.cascade_cdelta_assignment(cfg.seq_len, c, c * cfg.n_shards)
    kv = cas.cascade_m_split(a, alpha, 2)
    w, h = device_inputs(cfg, config_seed(cfg))
    plan = cas.cascade_plan_create_rs(cfg.batch, cfg.seq_len, alpha, a, 2 * alpha, kv)
    wts = cas.make_layer_weights(w)
    h_out = torch.empty_like(h)
    out = {"row_shards": alpha, "kv_shards": 2 * alpha, "c": c, "delta": c * cfg.n_shards, "m": 2}
    for name, mode in (("fused", cas.ATTN_FUSED), ("materialised", cas.ATTN_MATERIALISED)):
        desc = cas.make_layer_desc(cfg, mode, cas.ROWS_ORIGINAL)
        ws = cas.new_workspace(cas.cascade_layer_workspace_bytes(plan, desc))
        step = lambda: cas.cascade_layer_forward(plan, desc, wts, h, h_out, ws)
        for _ in range(2):
            step()
        out[name + "_ms_per_step"] = time_steps(step, steps) * 1e3
        st = staged_times(cas, plan, desc, wts, h, h_out, ws, steps)
        out[name + "_attention_ms"], out[name + "_lse_merge_ms"] = st["attention"], st["lse_merge"]
        del ws
    T, H, d = cfg.batch * cfg.seq_len, cfg.n_heads, cfg.head_dim
    out["partial_bytes"] = cfg.batch * 2 * alpha * H * cfg.seq_len * (d + 2) * 4
    out["merge_GBs"] = (out["partial_bytes"] + T * H * d * 2) / (out["materialised_lse_merge_ms"] * 1e-3) / 1e9
    return out


def run_decode(cas, cfg, steps, batch=32, cache_tokens=8192, shard_rows=128):
    """Token-sharded KV-cache decode of one new token per sequence: partial attention of the new query
    row against every cached kv shard, then the LSE merge.  HBM-bound: every cached K and V row is read once."""
    import numpy as np
    import torch
    H, Hkv, d = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    S = cache_tokens // shard_rows
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    q = torch.randn((batch, H, d), device="cuda", generator=g).to(torch.bfloat16)
    kc = torch.randn((batch, Hkv, S, shard_rows, d), device="cuda", generator=g).to(torch.bfloat16)
    vc = torch.randn((batch, Hkv, S, shard_rows, d), device="cuda", generator=g).to(torch.bfloat16)
    lens = torch.full((batch, S), shard_rows, dtype=torch.int32, device="cuda")
    m = torch.empty((batch, H, S), dtype=torch.float32, device="cuda")
    e = torch.empty_like(m)
    u = torch.empty((batch, S, H, d), dtype=torch.float32, device="cuda")
    o = torch.empty((batch, 1, H * d), dtype=torch.bfloat16, device="cuda")
    plan = cas.cascade_plan_create(batch, 1, S, np.zeros(1, dtype=np.int32))
    attn = lambda: cas.cascade_decode_partial_attn(q, kc, vc, lens, m, e, u, d ** -0.5)
    merge = lambda: cas.cascade_lse_merge(plan, m.view(batch, H, S, 1), e.view(batch, H, S, 1),
                                          u.view(batch, S, H, 1, d), o, H, Hkv, d)
    for _ in range(3):
        attn(); merge()
    t_attn = time_steps(attn, steps)
    t_merge = time_steps(merge, steps)
    cache_bytes = 2 * kc.numel() * 2
    partial_bytes = (2 * m.numel() + u.numel()) * 4
    return {"batch": batch, "cache_tokens": cache_tokens, "kv_shards": S, "n_heads": H, "n_kv_heads": Hkv, "head_dim": d,
            "partial_attn_us": t_attn * 1e6, "cache_bytes": cache_bytes,
            "partial_attn_GBs": (cache_bytes + partial_bytes) / t_attn / 1e9,
            "partial_attn_frac_of_hbm_peak": (cache_bytes + partial_bytes) / t_attn / 1e9 / HBM_PEAK_GBS,
            "lse_merge_us": t_merge * 1e6, "partial_bytes": partial_bytes}


def run_variants(cas, cfg, steps):
    """Post-norm bidirectional block (the BERT-shaped layer of the paper's timing runs) on the C2 shape,
    and a four-layer stack of the headline layer (packed order kept between layers)."""
    import torch
    from cascade_inputs import CONFIGS, config_seed, make_assignment
    out = {}
    c2 = CONFIGS["C2"].with_(norm_placement="post")
    a = make_assignment(c2.assignment, c2.seq_len, c2.n_shards, config_seed(c2))
    w, h = device_inputs(c2, config_seed(c2))
    plan = cas.cascade_plan_create(c2.batch, c2.seq_len, c2.n_shards, a, mask_kind=cas.MASK_NONE)
    desc = cas.make_layer_desc(c2, cas.ATTN_FUSED, cas.ROWS_ORIGINAL)
    wts = cas.make_layer_weights(w)
    h_out = torch.empty_like(h)
    ws = cas.new_workspace(cas.cascade_layer_workspace_bytes(plan, desc))
    step = lambda: cas.cascade_layer_forward(plan, desc, wts, h, h_out, ws)
    for _ in range(3):
        step()
    sec = time_steps(step, steps)
    out["post_norm_bidirectional_C2"] = {"ms_per_layer": sec * 1e3, "tokens_per_s": c2.batch * c2.seq_len / sec}
    del ws, w, h, h_out

    L = 4
    a = make_assignment(cfg.assignment, cfg.seq_len, cfg.n_shards, config_seed(cfg))
    plan = cas.cascade_plan_create(cfg.batch, cfg.seq_len, cfg.n_shards, a)
    desc = cas.make_layer_desc(cfg, cas.ATTN_FUSED, cas.ROWS_ORIGINAL)
    tensors = [device_inputs(cfg, config_seed(cfg) + l)[0] for l in range(L)]
    wl = [cas.make_layer_weights(t) for t in tensors]
    _, h = device_inputs(cfg, config_seed(cfg))
    h_out = torch.empty_like(h)
    ws = cas.new_workspace(cas.cascade_layer_stack_workspace_bytes(plan, desc, L))
    step = lambda: cas.cascade_layer_stack_forward(plan, desc, wl, h, h_out, ws)
    for _ in range(2):
        step()
    sec = time_steps(step, max(3, steps // 2))
    out["stack_of_4_layers"] = {"workload": cfg.name, "ms_per_layer": sec * 1e3 / L, "tokens_per_s": cfg.batch * cfg.seq_len / sec}
    del ws, tensors, wl, h_out

    # LM head on the sharded rows of the headline workload (Llama-3 vocabulary size): logits of every token
    # (one shard GEMM over the packed rows, MFMA-bound) and of the last token only (reads W_vocab once: HBM-bound)
    V = 128256
    D = cfg.d_model
    g = torch.Generator(device="cuda").manual_seed(config_seed(cfg))
    w_vocab = (torch.randn(V, D, device="cuda", generator=g) * cfg.sigma).to(h.dtype)
    gain = torch.ones(D, device="cuda", dtype=h.dtype)
    nk = {"layernorm": cas.NORM_LAYERNORM, "rmsnorm": cas.NORM_RMSNORM}[cfg.norm]
    dt = cas.BF16 if cfg.dtype == "bf16" else cas.F32
    for rows, name in ((cas.LM_ALL_ROWS, "lm_head_all_rows"), (cas.LM_LAST_ROW, "lm_head_last_row")):
        d = cas.LmHeadDesc(dt, D, V, nk, cfg.eps, rows, cas.ROWS_ORIGINAL, cas.ROWS_ORIGINAL)
        n_rows = cfg.batch * cfg.seq_len if rows == cas.LM_ALL_ROWS else cfg.batch
        logits = torch.empty(n_rows, V, device="cuda", dtype=h.dtype)
        tok = torch.empty(n_rows, device="cuda", dtype=torch.int32)
        ws = cas.new_workspace(cas.cascade_lm_head_workspace_bytes(plan, d))

        def step():
            cas.cascade_lm_head(plan, d, h, gain, None, w_vocab, logits, ws)
            cas.cascade_greedy_token(logits, tok)
        for _ in range(2):
            step()
        sec = time_steps(step, max(3, steps // 5))
        flops = 2.0 * n_rows * D * V
        bytes_w = V * D * w_vocab.element_size()
        out[name] = {"vocab": V, "rows": n_rows, "ms": sec * 1e3, "tflops": flops / sec / 1e12,
                     "weight_GB_per_s": bytes_w / sec / 1e9}
        del logits, ws
    return out


def cpu_baseline(cfg, host):
    """The oracle as it stands, on the host cores: the whole unsharded float64 layer, repeated for ~10 s."""
    import numpy as np
    from oracle import cascade_oracle as orc
    w, h, h_out, a = host
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    reps, sec, ref = 0, 0.0, None
    while reps < 10 and sec < 10.0:
        t0 = time.perf_counter()
        ref = np.stack([orc.layer_direct(h[b], w64, cfg) for b in range(cfg.batch)])
        sec += time.perf_counter() - t0
        reps += 1
    diff, scale = np.abs(h_out - ref), float(np.abs(ref).max())
    err = {"max_abs_err_over_max_abs_ref": float(diff.max() / scale),
           "elementwise_atol": 1e-3 * scale,
           "fraction_of_elements_within_atol": float((diff <= 1e-3 * scale).mean())}
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
    except Exception:
        cores = os.cpu_count()
    return {"value": reps * cfg.batch * cfg.seq_len / sec, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"whole {cfg.name} layer (all {cfg.batch * cfg.seq_len} tokens), float64 layer_direct, "
                      f"{reps} repetitions",
            "seconds": sec}, err


def other_config(cas, key, steps):
    """Another configuration of the list, timed the same way (W = 3), with its own roofline record."""
    import torch
    from cascade_inputs import CONFIGS
    cfg = CONFIGS[key]
    wl = Workload(cas, cfg)
    sec = wl.timed(steps, 3)
    st = wl.staged(max(3, steps // 2))
    peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_VECTOR_PEAK_TFLOPS
    tf = wl.flops["total"] / sec / 1e12
    out = {"workload": cfg.name, "steps": steps, "tokens_per_s": cfg.batch * cfg.seq_len / sec, "ms_per_step": sec * 1e3,
           "layer_tflops": tf, "layer_frac_of_mfma_peak": tf / peak, "roofline": roofline_record(cfg, wl.flops, st, key),
           "stages_ms": st}
    del wl
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C3", help="headline workload (C1..C5)")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the other configurations, the m-split, decode and variant measurements")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the MFMA-only and copy-only ceiling measurements")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs all shards on ONE GPU; --gpus N with N > 1 is not supported "
                 "(no inter-GPU path exists)")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    import paper_2507_05228_amd as cas
    from cascade_inputs import CONFIGS
    cas.load_library()

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Order of the run.  (1) The timed region as the first thing the device does after start-up: W + K steps on a
    # device that was idle (reported as from_idle).  (2) The CPU oracle (device idle meanwhile).  (3) Every other
    # measurement, ending with at least 100 individually timed steps of the headline workload.  (4) The timed
    # region again, W + K steps right behind (3): the device has been busy and holds the clock it sustains
    # under this load.  (4) is `value`; an idle MI355X takes about 60 of these
    # 0.8 ms steps to reach that clock, more than the W a short run asks for.
    cfg = CONFIGS[args.config]
    key = args.config
    bf16 = cfg.dtype == "bf16"
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else FP32_VECTOR_PEAK_TFLOPS
    wl = Workload(cas, cfg)
    fl = wl.flops
    sec_idle = wl.timed(args.steps, args.warmup)
    torch.cuda.synchronize()

    out_cpu = None
    if not args.no_cpu_baseline:
        host = ({k: v.float().cpu().numpy() for k, v in wl.w.items()}, wl.h.float().cpu().numpy(),
                wl.h_out.float().cpu().numpy(), wl.a)
        out_cpu = cpu_baseline(cfg, host)
        del host

    extra = {}
    if bf16 and not args.no_ceilings:
        extra["measured_ceilings"] = measured_ceilings(cas)
        extra["vendor_library_gemm_for_scale"] = vendor_gemm_reference(cfg)
    st = wl.staged(max(args.steps, 20))
    sec_m, stm, merge_alone = wl.materialised(max(5, args.steps // 4))
    if bf16 and not args.headline_only:
        torch.cuda.empty_cache()
        extra["m_split"] = run_m_split(cas, cfg, max(3, args.steps // 4))
        torch.cuda.empty_cache()
        extra["kv_cache_decode"] = run_decode(cas, cfg, args.steps)
        torch.cuda.empty_cache()
        extra["variants"] = run_variants(cas, cfg, max(5, args.steps // 2))
        others = {}
        for k in ("C2", "C4", "C5"):
            if k != key:
                torch.cuda.empty_cache()
                others[k] = other_config(cas, k, max(5, args.steps // 5))
        extra["other_configs"] = others
        torch.cuda.empty_cache()

    # per-step statistics of the headline step (events around every step), then the headline itself
    per_step = per_step_stats(wl.step, max(args.steps, 100))
    sec = wl.timed(args.steps, args.warmup)                       # the headline: W warm-up steps, K timed steps
    sec_graph = wl.graph_replay(args.steps, args.warmup)

    es = 2 if bf16 else 4
    T, D, H, d, S = cfg.batch * cfg.seq_len, cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.n_shards
    merge_bytes = cfg.batch * S * H * cfg.seq_len * (d + 2) * 4 + T * H * d * es
    gather_bytes = 2 * T * D * es
    tflops = fl["total"] / sec / 1e12
    roof = roofline_record(cfg, fl, st, key)
    if "measured_ceilings" in extra:
        roof["frac_of_measured_lds_fed_mfma_rate"] = roof["achieved"] / extra["measured_ceilings"]["mfma_bf16_lds_operands_tflops"]
    out = {
        "metric": "sharded-layer prefill tokens/sec/GPU", "value": T / sec, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "seq_len": cfg.seq_len, "n_shards": S,
                   "assignment": cfg.assignment, "d_model": D, "n_heads": H, "n_kv_heads": cfg.n_kv_heads,
                   "head_dim": d, "d_ff": cfg.d_ff,
                   "attn_mode": "fused (running log-sum-exp merge inside the attention kernel, no partials in HBM)",
                   "io_rows": "original"},
        "layer_tflops": tflops, "layer_frac_of_mfma_peak": tflops / peak, "layer_gflop_counted": fl["total"] / 1e9,
        "timing": {"ms_per_step": sec * 1e3, "clock": "host, device synchronised before and after the K steps",
                   "position": "last in the run, right behind the other measurements, the last of which are the per-step "
                               "event timings of this same step (per_step_events)",
                   "from_idle_ms_per_step": sec_idle * 1e3,
                   "from_idle_position": "first device work of the process, same W and K",
                   "hip_graph_replay_ms_per_step": sec_graph * 1e3,
                   "per_step_events": per_step},
        # the paper's own data flow (Algorithms 3 and 4 as written): partials m, e, u~ to HBM, merge as a pass of its own
        "value_materialised": T / sec_m, "ms_per_step_materialised": sec_m * 1e3,
        "layer_tflops_materialised": fl["total"] / sec_m / 1e12,
        "roofline": roof,
        "stages_ms": st,
        "stage_tflops": {k: fl[k] / (st[k] * 1e-3) / 1e12 for k in ("qkv_gemm", "attention", "o_proj", "ffn_up", "ffn_down")},
        "stage_frac_of_mfma_peak": {k: fl[k] / (st[k] * 1e-3) / 1e12 / peak
                                    for k in ("qkv_gemm", "attention", "o_proj", "ffn_up", "ffn_down")},
        "hbm_kernels": {
            "lse_merge": {"ms": merge_alone * 1e3, "bytes": merge_bytes, "GBs": merge_bytes / merge_alone / 1e9,
                          "frac_of_hbm_peak": merge_bytes / merge_alone / 1e9 / HBM_PEAK_GBS,
                          "timing": "back-to-back launches on the partials of a materialised pass, HIP events",
                          "ms_inside_the_layer": stm["lse_merge"],
                          "frac_of_hbm_peak_inside_the_layer": merge_bytes / (stm["lse_merge"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "gather_norm1": {"ms": st["gather_norm1"], "bytes": gather_bytes,
                             "GBs": gather_bytes / (st["gather_norm1"] * 1e-3) / 1e9,
                             "frac_of_hbm_peak": gather_bytes / (st["gather_norm1"] * 1e-3) / 1e9 / HBM_PEAK_GBS}},
        "materialised_mode": {"ms_per_step": sec_m * 1e3, "partial_attention_ms": stm["attention"],
                              "lse_merge_ms": stm["lse_merge"]},
    }
    if out_cpu is not None:
        out["cpu_baseline"], out["error_vs_oracle"] = out_cpu
        out["max_rel_err_vs_oracle"] = out_cpu[1]["max_abs_err_over_max_abs_ref"]
    out.update(extra)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
