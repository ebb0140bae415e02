"""GPU parity of the streaming causal convolution with a two-frame feature cache (Appendix C) against the fp64 oracle,
through the C ABI: frame-by-frame and chunked streaming must both equal the oracle's whole-sequence convolution."""
import math

import numpy as np
import pytest
import torch

import lvx_synth as S
from oracle import lvx_oracle as O
from test_gpu_parity import DEV, assert_close

pytestmark = pytest.mark.gpu


def conv_inputs(tag, T, H, W, Ci, Co, pad=0):
    x = S.randn_bf16((T, H, W, Ci), S.seed_of(tag, "x"), 1.0, device=DEV)
    w = S.randn_bf16((Co, 27 * Ci + pad), S.seed_of(tag, "w"), 1.0 / math.sqrt(27 * Ci), device=DEV)[:, :27 * Ci]
    b = S.randn_f32((Co,), S.seed_of(tag, "b"), 0.5, device=DEV)
    return x, w, b


@pytest.mark.parametrize("H,W,Ci,Co,chunks,act", [
    (5, 7, 64, 8, [1, 1, 1, 1], 0),          # one frame per step: the overlapping cache shift
    (9, 6, 64, 72, [3, 3, 1, 2], 1),         # ragged column tile, SiLU
    (20, 33, 128, 136, [2, 4, 1], 1),        # 660 pixels per frame: several 256-row tiles with a ragged tail, two column tiles
    (4, 4, 192, 64, [4], 0),                 # whole sequence in one step
])
def test_streaming_conv_equals_whole_sequence_oracle(lvx, H, W, Ci, Co, chunks, act):
    T = sum(chunks)
    x, w, b = conv_inputs("conv_%d_%d_%d_%d" % (H, W, Ci, Co), T, H, W, Ci, Co, pad=64)
    ref = O.causal_conv3d(S.to_f64(x), S.to_f64(w).reshape(Co, 3, 3, 3, Ci), S.to_f64(b))
    if act:
        ref = O.silu(ref)
    conv = lvx.CausalConv(Ci, Co, H, W, max(chunks), DEV)
    y = torch.empty((T, H, W, Co), dtype=torch.bfloat16, device=DEV)
    t = 0
    for n in chunks:
        conv.step(x[t:t + n], w, b, act, y[t:t + n])
        t += n
    torch.cuda.synchronize()
    assert_close(y, ref, "causal conv %dx%d C %d->%d chunks %s" % (H, W, Ci, Co, chunks))
    # causality through the cache: the same frames again after a reset give the same result; without a reset they see the
    # previous sequence's last two frames as history, as the oracle's cache does
    y2 = torch.empty_like(y[:chunks[0]])
    conv.step(x[:chunks[0]], w, b, act, y2)
    torch.cuda.synchronize()
    model = O.CausalConvCache()
    model.frames = S.to_f64(x)[-2:]
    want = model.step(S.to_f64(x[:chunks[0]]), S.to_f64(w).reshape(Co, 3, 3, 3, Ci), S.to_f64(b))
    assert_close(y2, O.silu(want) if act else want, "continuing the stream with the cached two frames")
    conv.reset()
    conv.step(x[:chunks[0]], w, None, 0, y2)
    torch.cuda.synchronize()
    want0 = O.causal_conv3d(S.to_f64(x[:chunks[0]]), S.to_f64(w).reshape(Co, 3, 3, 3, Ci), None)
    assert_close(y2, want0, "after reset, no bias")
    too_long = torch.empty((max(chunks) + 1, H, W, Ci), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(lvx.LvxError) as e:
        conv.step(too_long, w, b, act, torch.empty((max(chunks) + 1, H, W, Co), dtype=torch.bfloat16, device=DEV))
    assert e.value.status == 2
    conv.close()


def test_linear_bias_and_silu_epilogues(lvx):
    M, N, K = 300, 200, 192
    a = S.randn_bf16((M, K), 71, 1.0, device=DEV)
    w = S.randn_bf16((N, K), 72, 1.0 / math.sqrt(K), device=DEV)
    b = S.randn_f32((N,), 73, 0.5, device=DEV)
    ref = O.linear(S.to_f64(a), S.to_f64(w)) + S.to_f64(b)
    c = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    lvx.lvx_linear(a, w, c, lvx.EPI_BIAS, gate=b)
    torch.cuda.synchronize()
    assert_close(c, ref, "linear + bias")
    lvx.lvx_linear(a, w, c, lvx.EPI_BIAS_SILU, gate=b)
    torch.cuda.synchronize()
    assert_close(c, O.silu(ref), "linear + bias + silu")
