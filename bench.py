#!/usr/bin/env python3
"""Benchmark of the denoise-stage hot path on one MI355X.

A step = one pass of the whole hot path over one chunk: the sink's rotary re-indexing (all layers) followed by
lvx_denoise_stage on 40 DiT blocks at the 14B shape
(3 latent frames x 1560 tokens against the rolling cache: sink 1560 + 4 past chunks + self = 24 960 keys),
synthetic seeded inputs and random-init weights, everything resident in HBM before the timed region.
Prints ONE JSON line: latent frames/s (whole job, one GPU), plus
  roofline      the chunk-to-cache attention kernel's TFLOP/s against the bf16 dense MFMA peak, its launch durations
                measured live with HIP events on the launch stream inside the timed region;
  cpu_baseline  the fp64 numpy oracle timed on this machine's host cores on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense FP8 MFMA, published
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per attention launch at the full cache, from two rocprofv3 --pmc runs (FETCH_SIZE 617994 KiB, WRITE_SIZE 46803 KiB
# per dispatch; both counters read 1.000x the known size of a plain copy kernel in the same runs).  Summary and commands:
# profiles/attention_gemm_14b_pmc_hbm_traffic.txt.  Only valid for the 24960-key, 4680-query, 40-head launch timed here.
ATTN_TRAFFIC_BYTES = (617994 + 46803) * 1024


def attention_flops(n_q, n_k, H, D):
    return 4.0 * n_q * n_k * D * H


def block_flops(n, d, f, n_k, n_ctx, H, D):
    gemm = 2.0 * n * d * (3 * d) + 2.0 * n * d * d + (2.0 * n * d * d + 2 * 2.0 * n_ctx * d * d + 2.0 * n * d * d) + 2 * 2.0 * n * d * f
    return gemm + attention_flops(n, n_k, H, D) + attention_flops(n, n_ctx, H, D)


def cpu_baseline(p, sample_tokens, n_threads_hint):
    """Oracle (as it stands: numpy fp64 on the BLAS threads of the host) on one DiT block for `sample_tokens` of the chunk's
    tokens against the FULL visible key set (sink + 4 past chunks + the whole current chunk = 24960 keys), through the
    oracle's row form; extrapolated linearly in tokens and layers to frames/s."""
    import numpy as np
    from oracle import lvx_oracle as O
    H, D = p["n_heads"], p["head_dim"]
    d = H * D
    fk = p["frame_h"] * p["frame_w"]
    chunk = fk * p["chunk_frames"]
    n_k = fk * p["sink_frames"] + (p["window"] + 1) * chunk
    rng = np.random.default_rng(0)
    cfg = O.StageConfig(H, D, p["frame_h"], p["frame_w"], p["chunk_frames"], p["window"], p["sink_frames"], p["rope_axes"])
    w = {}
    for name, shape in (("W_qkv", (3 * d, d)), ("W_o", (d, d)), ("Wc_q", (d, d)), ("Wc_k", (d, d)), ("Wc_v", (d, d)),
                        ("Wc_o", (d, d)), ("W_1", (p["ffn"], d)), ("W_2", (d, p["ffn"]))):
        w[name] = rng.standard_normal(shape, dtype=np.float32).astype(np.float64) * 0.02
    for g in ("g_q", "g_k", "gc_q", "gc_k"):
        w[g] = np.ones(d)
    k_vis = rng.standard_normal((n_k, H, D), dtype=np.float32).astype(np.float64)
    v_vis = rng.standard_normal((n_k, H, D), dtype=np.float32).astype(np.float64)
    x = rng.standard_normal((sample_tokens, d))
    ctx = rng.standard_normal((p["n_ctx"], d))
    pos = tuple(a[:sample_tokens] for a in O.token_positions(chunk, 1 + 3 * p["window"], p["frame_h"], p["frame_w"]))
    t0 = time.perf_counter()
    O.dit_block_rows(x, pos, w, k_vis, v_vis, ctx, None, cfg)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = n_threads_hint
    return dt, cores, n_k


class PowerSampler:
    """Polls the GPU's shader clock and socket power (amdsmi) from a host thread while the timed region runs."""

    def __init__(self, period=0.1):
        self.samples, self.cap_w, self.period, self._stop, self._t = [], None, period, False, None
        try:
            import amdsmi
            self.A = amdsmi
            amdsmi.amdsmi_init()
            self.h = amdsmi.amdsmi_get_processor_handles()[0]
            cap = amdsmi.amdsmi_get_power_info(self.h).get("power_limit")
            self.cap_w = cap / 1e6 if isinstance(cap, (int, float)) else None
        except Exception:
            self.A = None

    def _poll(self):
        while not self._stop:
            try:
                m = self.A.amdsmi_get_gpu_metrics_info(self.h)
                clk, pw = m.get("current_gfxclk"), m.get("current_socket_power")
                if isinstance(clk, (int, float)) and isinstance(pw, (int, float)):
                    self.samples.append((clk, pw))
            except Exception:
                pass
            time.sleep(self.period)

    def start(self):
        if self.A is not None:
            import threading
            self._t = threading.Thread(target=self._poll, daemon=True)
            self._t.start()

    def stop(self):
        self._stop = True
        if self._t is not None:
            self._t.join()
        if not self.samples:
            return None
        clk = [c for c, _ in self.samples]
        pw = [w for _, w in self.samples]
        return {"samples": len(self.samples), "gfx_clk_mhz_avg": round(sum(clk) / len(clk)), "gfx_clk_mhz_min": min(clk), "gfx_clk_mhz_max": max(clk),
                "socket_power_w_avg": round(sum(pw) / len(pw)), "socket_power_w_max": max(pw), "power_cap_w": self.cap_w,
                "note": "amdsmi current_gfxclk / current_socket_power polled every %.1f s during the timed region; the published peaks assume 2400 MHz" % self.period}


def kernel_classes(prof, steps, n, d, f, n_k, n_ctx, H, D, L, sink_n, fp8=False):
    """Per kernel class: ms per step, launches per step, and the class's rate against the roofline that bounds it
    (MFMA classes: algorithmic FLOPs against the dense MFMA peak of the class's operand type, bf16, or FP8 for the linears of an
    FP8 stage; memory classes: algorithmic bytes against the HBM peak)."""
    fl = {"attn_self": attention_flops(n, n_k, H, D), "gemm_qkv": 2.0 * n * d * 3 * d, "gemm_o": 2.0 * n * d * d, "gemm_cross": 2 * 2.0 * n * d * d,
          "gemm_ffn1": 2.0 * n * d * f, "gemm_ffn2": 2.0 * n * d * f, "attn_cross": attention_flops(n, n_ctx, H, D), "ctx_kv": 2 * 2.0 * n_ctx * d * d}
    # algorithmic bytes per layer: rope+norm reads q (bf16) and k (fp32; bf16 in an FP8 stage) and writes q^, k^ (bf16, k^ straight
    # into the cache); the append then reads and writes v only; each LayerNorm reads the fp32 stream and writes bf16 (3 per layer)
    by = {"rope_norm": n * d * (2 + 2 + 2 + 2) if fp8 else n * d * (2 + 4 + 2 + 2), "append": 2.0 * n * d * 2,
          "layernorm": 3.0 * n * d * (4 + 2), "cross_qnorm": 2.0 * n * d * 2}
    per_step = {"misc": n * d * (2 + 4) + n * d * (2 + 4 + 2), "sink_rope": L * sink_n * d * (4 + 2)}
    out = {}
    for k, (ms, cnt) in prof.items():
        if not cnt:
            continue
        e = {"ms_per_step": round(ms / steps, 3), "launches_per_step": round(cnt / steps, 2)}
        sec = ms / steps * 1e-3
        if k in fl:
            peak = PEAK_FP8_TFLOPS if (fp8 and (k.startswith("gemm_") or k == "ctx_kv")) else PEAK_BF16_TFLOPS
            e.update(bound="mfma", achieved=round(L * fl[k] / sec / 1e12, 1), peak=peak, unit="TFLOP/s", frac=round(L * fl[k] / sec / 1e12 / peak, 4))
        elif k in by or k in per_step:
            b = L * by[k] if k in by else per_step[k]
            e.update(bound="hbm", achieved=round(b / sec / 1e9, 1), unit="GB/s", frac=round(b / sec / 1e9 / PEAK_HBM_GBS, 4))
        out[k] = e
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=40, help="debug only: fewer layers is NOT the benchmark workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-level", type=int, default=1,
                    help="HIP events inside the timed region: 1 = around the attention launches only (what `roofline` needs), "
                         "2 = around every kernel class (costs ~1.3 % of the step)")
    ap.add_argument("--breakdown-steps", type=int, default=4,
                    help="untimed extra steps with events around every kernel class, for `kernel_ms_per_step` (0 = skip)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=2340)
    ap.add_argument("--no-fp8-extra", action="store_true", help="skip the separately reported FP8-linears pass after the bf16 run")
    ap.add_argument("--fp8", action="store_true",
                    help="NOT the headline: run every linear of the stage in FP8 E4M3 with per-tensor dynamic scaling (the paper's own "
                         "default, Appendix C); attention, norms and the residual stream are unchanged; dtype is reported as such")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (one denoise stage = one timestep of the pipeline on one GPU); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import lvx_synth as S
    import paper_2512_04677_amd as lvx

    lvx.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    p = S.PRESETS["attn14b"]
    H, D = p["n_heads"], p["head_dim"]
    d = H * D
    fk = p["frame_h"] * p["frame_w"]
    sink_n, n = fk * p["sink_frames"], fk * p["chunk_frames"]
    n_slots = p["window"] + 1
    n_k = sink_n + n_slots * n
    L = args.layers

    t_setup = time.perf_counter()
    ROW_PAD = 64  # weight rows padded by 128 bytes (row stride in_features + 64), see include/lvx.h
    layers = [S.block_weights(d, p["ffn"], l, "bench", std=0.02, device=dev, on_device_draw=True, row_pad=ROW_PAD) for l in range(L)]
    rope = lvx.rope_desc(H, D, p["rope_axes"], 10000.0, p["frame_h"], p["frame_w"])
    stage = lvx.StageHandle(layers, rope, p["ffn"], ldw_d=d + ROW_PAD, ldw_ffn=p["ffn"] + ROW_PAD, fp8=args.fp8, keep_bf16=not args.fp8)
    cache = lvx.KVCache(lvx.cache_desc(L, H, D, p["frame_h"], p["frame_w"], p["chunk_frames"], p["window"], p["sink_frames"]), dev)
    cache.attach_sink_source()   # un-rotated sink keys: the sink's rotary index is re-assigned before every forward (Rolling RoPE)
    for l in range(L):
        sk = S.randn_bf16_device((sink_n, d), S.seed_of("bench_sk", l), 1.0, dev)
        sv = S.randn_bf16_device((sink_n, d), S.seed_of("bench_sv", l), 1.0, dev)
        lvx.lvx_kvcache_reset_sink(cache, l, sk, sv)
    ws = torch.empty(lvx.lvx_workspace_bytes(stage, n, p["n_ctx"]), dtype=torch.uint8, device=dev)
    n_inputs = 8
    xs = [S.randn_bf16_device((n, d), S.seed_of("bench_x", i), 1.0, dev) for i in range(n_inputs)]
    ctxs = [S.randn_bf16_device((p["n_ctx"], d), S.seed_of("bench_ctx", i), 1.0, dev) for i in range(n_inputs)]
    x = torch.empty_like(xs[0])
    torch.cuda.synchronize()
    print("[bench] setup %.1f s: %d layers, %.1f GB weights, %.1f GB cache, %.2f GB workspace" % (
        time.perf_counter() - t_setup, L, (sum(t.numel() * t.element_size() for w in layers for t in w.values() if t is not None)
                                       + sum(t.numel() * t.element_size() for t in stage.fp8_tensors)) / 1e9,
        cache.storage.numel() / 1e9, ws.numel() / 1e9), file=sys.stderr, flush=True)

    chunk = [0]

    def step():
        i = chunk[0]
        x.copy_(xs[i % n_inputs])
        t0 = 1 + p["chunk_frames"] * i
        lvx.lvx_sink_rope_update(cache, rope, -1, t0 + p["chunk_frames"] + 1)   # Phi(sink): two frames ahead of the block's last
        lvx.lvx_denoise_stage(stage, cache, x, ctxs[i % n_inputs], None, -0.25, i, t0, ws)
        chunk[0] += 1

    # fill the ring (setup, untimed): the steady state the paper's stage runs in has all window+1 slots occupied
    for _ in range(max(0, n_slots - args.warmup)):
        step()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    print("[bench] ring full after %d chunks; timing %d steps" % (chunk[0], args.steps), file=sys.stderr, flush=True)

    lvx.lvx_profile_read()
    lvx.lvx_profile_set(args.profile_level)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # between steps, on the launch stream
    sampler = PowerSampler()
    torch.cuda.synchronize()
    sampler.start()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    seconds = time.perf_counter() - t0
    clocks = sampler.stop()
    lvx.lvx_profile_set(0)
    prof = lvx.lvx_profile_read()
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    assert bool(torch.isfinite(x.float()).all()), "stage output is not finite"

    ms_per_step = seconds / args.steps * 1e3
    frames_per_s = p["chunk_frames"] * args.steps / seconds
    attn_ms, attn_n = prof["attn_self"]
    attn_avg_ms = attn_ms / max(attn_n, 1)
    attn_fl = attention_flops(n, n_k, H, D)
    attn_tflops = attn_fl / (attn_avg_ms * 1e-3) / 1e12 if attn_n else 0.0
    stage_fl = L * block_flops(n, d, p["ffn"], n_k, p["n_ctx"], H, D)

    out = {
        "metric": "latent frames/s per denoise stage (chunk-attention TFLOP/s and % of bf16 MFMA peak in `roofline`)",
        "value": round(frames_per_s, 4), "unit": "latent frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8 e4m3 linears (per-tensor dynamic scaling), bf16 attention" if args.fp8 else "bf16", "data": "synthetic",
        "config": {"workload": "configs[4]: one denoise stage on one GPU, %d DiT blocks (hidden 5120, 40 heads x 128, FFN 13824, "
                               "544 context tokens), chunk 3x1560=4680 tokens, rolling cache full: sink 1560 + 4 past chunks + self "
                               "= 24960 keys per layer (the attention inside is configs[1])" % L,
                   "n_layers": L, "chunk_tokens": n, "keys": n_k, "ms_per_chunk": round(ms_per_step, 3),
                   "ms_per_chunk_median": round(step_ms[len(step_ms) // 2], 3), "ms_per_chunk_min": round(step_ms[0], 3),
                   "ms_per_chunk_max": round(step_ms[-1], 3),
                   "stage_tflops": round(stage_fl / (seconds / args.steps) / 1e12, 2),
                   "stage_frac_of_bf16_peak": round(stage_fl / (seconds / args.steps) / 1e12 / PEAK_BF16_TFLOPS, 4)},
        "roofline": {"kernel": "lvx_attention_kernel<128,8,2,2,true,false> (chunk-to-cache self-attention, configs[1] shape)", "bound": "mfma",
                     "achieved": round(attn_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4), "traffic": ATTN_TRAFFIC_BYTES,
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE); algorithmic: %d" % (2 * d * (2 * n + 2 * n_k)),
                     "flops_per_launch": attn_fl, "avg_launch_ms": round(attn_avg_ms, 4), "launches": attn_n,
                     "peak_note": "published dense bf16 MFMA peak (2.4 GHz). The chip is power-limited: under this kernel it clocks at about "
                                  "2.0 GHz (see `clocks`), and a register-only MFMA loop on random operands sustains 1800 TFLOP/s (0.72 of "
                                  "this peak), which is the ceiling a bf16 kernel faces here"},
    }
    out["clocks"] = clocks
    bd_prof, bd_steps, bd_ms = None, 0, ms_per_step
    if args.profile_level >= 2:
        bd_prof, bd_steps = prof, args.steps
    elif args.breakdown_steps > 0:
        # per-class kernel times from a separate, untimed pass (the events around every launch slow the step a little)
        lvx.lvx_profile_set(2)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.breakdown_steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        lvx.lvx_profile_set(0)
        bd_prof, bd_steps, bd_ms = lvx.lvx_profile_read(), args.breakdown_steps, e0.elapsed_time(e1) / args.breakdown_steps
    if bd_prof is not None:
        # every launch of a step belongs to one class; what is left of the step is the idle time between launches (and the
        # events themselves).  fp8_quant (FP8 stages) is also contained in its linear's class, so it is not added again.
        out["kernel_ms_per_step"] = {k: round(v[0] / bd_steps, 3) for k, v in bd_prof.items() if v[1]}
        out["kernel_classes"] = kernel_classes(bd_prof, bd_steps, n, d, p["ffn"], n_k, p["n_ctx"], H, D, L, sink_n, fp8=args.fp8)
        in_kernels = sum(v[0] for k, v in bd_prof.items() if k != "fp8_quant") / bd_steps
        out["kernel_ms_per_step_sum"] = round(in_kernels, 3)
        out["between_launches_ms_per_step"] = round(bd_ms - in_kernels, 3)
        out["breakdown_ms_per_step"] = round(bd_ms, 3)
    if not args.fp8 and not args.no_fp8_extra:
        # second, separately reported configuration: the same stage with every linear in FP8 E4M3 (Appendix C, the paper's own
        # default); same weights (quantised per tensor here), same cache, continuing the same chunk sequence
        stage8 = lvx.StageHandle(layers, rope, p["ffn"], ldw_d=d + ROW_PAD, ldw_ffn=p["ffn"] + ROW_PAD, fp8=True, keep_bf16=True)
        ws8 = torch.empty(lvx.lvx_workspace_bytes(stage8, n, p["n_ctx"]), dtype=torch.uint8, device=dev)
        steps8 = min(args.steps, 10)

        def step8():
            i = chunk[0]
            x.copy_(xs[i % n_inputs])
            t0 = 1 + p["chunk_frames"] * i
            lvx.lvx_sink_rope_update(cache, rope, -1, t0 + p["chunk_frames"] + 1)
            lvx.lvx_denoise_stage(stage8, cache, x, ctxs[i % n_inputs], None, -0.25, i, t0, ws8)
            chunk[0] += 1

        for _ in range(2):
            step8()
        torch.cuda.synchronize()
        lvx.lvx_profile_read()
        t0_ = time.perf_counter()
        for _ in range(steps8):
            step8()
        torch.cuda.synchronize()
        sec8 = time.perf_counter() - t0_
        assert bool(torch.isfinite(x.float()).all()), "FP8 stage output is not finite"
        bd8 = max(args.breakdown_steps, 2)   # per-class kernel times from an untimed pass
        lvx.lvx_profile_set(2)
        for _ in range(bd8):
            step8()
        torch.cuda.synchronize()
        lvx.lvx_profile_set(0)
        prof8 = lvx.lvx_profile_read()
        qkv_ms = (prof8["gemm_qkv"][0] - prof8["fp8_quant"][0] / 7.0) / max(prof8["gemm_qkv"][1], 1)   # 7 quantisations per block
        out["fp8_linears"] = {
            "note": "NOT the headline: same stage, every linear in FP8 E4M3 with per-tensor dynamic scaling (Appendix C); attention bf16",
            "value": round(p["chunk_frames"] * steps8 / sec8, 4), "unit": "latent frames/s", "steps": steps8,
            "ms_per_step": round(sec8 / steps8 * 1e3, 3),
            "qkv_gemm_tflops": round(2.0 * n * 3 * d * d / (qkv_ms * 1e-3) / 1e12, 1), "fp8_mfma_peak_tflops": 5000.0,
            "kernel_ms_per_step": {k: round(v[0] / bd8, 3) for k, v in prof8.items() if v[1]},
            # the linears' classes against the FP8 peak; a linear's class contains the quantisation of its input
            "kernel_classes": kernel_classes(prof8, bd8, n, d, p["ffn"], n_k, p["n_ctx"], H, D, L, sink_n, fp8=True)}
    if not args.no_cpu_baseline:
        t_cpu, cores, keys_cpu = cpu_baseline(p, args.cpu_sample_tokens, os.cpu_count())
        est_chunk_s = t_cpu * (n / args.cpu_sample_tokens) * L
        out["cpu_baseline"] = {"value": round(p["chunk_frames"] / est_chunk_s, 6), "unit": "latent frames/s", "cores": cores,
                               "kind": "oracle",
                               "sample": "the fp64 numpy oracle (BLAS threads of the host, not a compiled C oracle), ONE DiT block in row form on "
                                         "%d of the chunk's %d tokens against all %d visible keys (sink + 4 chunks + the whole current chunk): "
                                         "%.2f s measured; extrapolated x%.0f tokens x%d layers"
                                         % (args.cpu_sample_tokens, n, keys_cpu, t_cpu, n / args.cpu_sample_tokens, L)}
    print(json.dumps(out), flush=True)
    cache.close()


if __name__ == "__main__":
    main()
