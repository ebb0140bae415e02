"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only random draws, bf16 rounding of the drawn values and the
named shape presets.  Both the CPU oracle and the HIP path receive the *same bits*: tensors are drawn
in fp32 from a seeded CPU generator, rounded to bf16 (round-to-nearest-even, torch's cast), and the
oracle gets those bf16 values widened exactly to float64.

The presets mirror the five workload configurations (shapes only; they stand in for the paper's
720x400, 3-latent-block, window-4, one-sink-frame runtime workload, Sec. 4.1):
  tiny      2 heads x 64, frame 4x6, chunk 2 frames, 2 past chunks       (config 1)
  attn14b   40 heads x 128, frame 30x52, chunk 3 frames, window 4        (configs 2-5)
"""
import zlib

import numpy as np
import torch

PRESETS = {
    "tiny": dict(n_heads=2, head_dim=64, frame_h=4, frame_w=6, chunk_frames=2, window=2, sink_frames=1,
                 rope_axes=(24, 20, 20), ffn=256, n_ctx=24),
    "small": dict(n_heads=4, head_dim=128, frame_h=5, frame_w=7, chunk_frames=3, window=4, sink_frames=1,
                  rope_axes=(44, 42, 42), ffn=1280, n_ctx=40),
    # 130-token frames: 520 .. 1300 visible keys, i.e. both sides of the attention kernel's switch to two key tiles per phase
    "medium": dict(n_heads=4, head_dim=128, frame_h=10, frame_w=13, chunk_frames=3, window=2, sink_frames=1,
                   rope_axes=(44, 42, 42), ffn=1024, n_ctx=72),
    "attn14b": dict(n_heads=40, head_dim=128, frame_h=30, frame_w=52, chunk_frames=3, window=4, sink_frames=1,
                    rope_axes=(44, 42, 42), ffn=13824, n_ctx=544),
}


def seed_of(*names):
    """Stable 31-bit seed from a tuple of names/ints (config, layer, tensor name, step...)."""
    return zlib.crc32("/".join(str(n) for n in names).encode()) & 0x7FFFFFFF


def randn_bf16(shape, seed, std=1.0, mean=0.0, device="cpu"):
    """N(mean, std) drawn in fp32 on the CPU with a seeded generator, rounded to bf16."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    t = torch.randn(tuple(shape), generator=g, dtype=torch.float32) * std + mean
    t = t.to(torch.bfloat16)
    return t.to(device) if device != "cpu" else t


def randn_f32(shape, seed, std=1.0, mean=0.0, device="cpu"):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    t = torch.randn(tuple(shape), generator=g, dtype=torch.float32) * std + mean
    return t.to(device) if device != "cpu" else t


def randn_bf16_device(shape, seed, std, device):
    """Same distribution drawn directly on the GPU (for the 28 GB weight set of the full stage, where a
    CPU draw would dominate the run).  Bits differ from the CPU draw; parity checks on such tensors read
    the tensor back instead of re-drawing it."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return (torch.randn(tuple(shape), generator=g, dtype=torch.float32, device=device) * std).to(torch.bfloat16)


def to_f64(t):
    """Exact widening of a (bf16/fp32) torch tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def block_weight_shapes(d, ffn):
    """Names and shapes of one block's weights; linears are [out, in], gains are [d]."""
    return {
        "W_qkv": (3 * d, d), "W_o": (d, d),
        "Wc_q": (d, d), "Wc_k": (d, d), "Wc_v": (d, d), "Wc_o": (d, d),
        "W_1": (ffn, d), "W_2": (d, ffn),
    }


def block_weights(d, ffn, layer, tag, std=0.02, device="cpu", on_device_draw=False, row_pad=0):
    """One block's weights ~ N(0, std) in bf16, RMSNorm gains = 1 (fp32).  With row_pad > 0 each matrix is the
    [:, :in_features] view of an [out, in_features + row_pad] allocation (row stride in + row_pad)."""
    w = {}
    for name, shape in block_weight_shapes(d, ffn).items():
        s = seed_of(tag, "layer", layer, name)
        shape = (shape[0], shape[1] + row_pad)
        t = randn_bf16_device(shape, s, std, device) if on_device_draw else randn_bf16(shape, s, std, device=device)
        w[name] = t[:, :shape[1] - row_pad] if row_pad else t
    for g in ("g_q", "g_k", "gc_q", "gc_k"):
        w[g] = torch.ones(d, dtype=torch.float32, device=device)
    return w


def weights_to_f64(w):
    return {k: to_f64(v) for k, v in w.items()}
