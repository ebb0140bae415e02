"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle's own code.

Each test is chosen so that a plausible slip in oracle/lvx_oracle.py (dropped term, sign, index,
transposed operand) fails it.  Nothing here touches the HIP path.
"""
import math

import numpy as np
import pytest
from scipy.special import erf

from oracle import lvx_oracle as O

rng = np.random.default_rng(1234)


# ---------------------------------------------------------------- attention
def brute_attention(q, k, v, scale):
    """Pure-Python definition: loops over query, head, key, channel."""
    nq, H, D = q.shape
    nk = k.shape[0]
    out = np.zeros((nq, H, D))
    for r in range(nq):
        for h in range(H):
            s = [scale * sum(q[r, h, c] * k[m, h, c] for c in range(D)) for m in range(nk)]
            mx = max(s)
            e = [math.exp(t - mx) for t in s]
            z = sum(e)
            for c in range(D):
                out[r, h, c] = sum(e[m] * v[m, h, c] for m in range(nk)) / z
    return out


def test_attention_brute_force_tiny():
    q = rng.standard_normal((5, 2, 8))
    k = rng.standard_normal((11, 2, 8))
    v = rng.standard_normal((11, 2, 8))
    np.testing.assert_allclose(O.attention(q, k, v, 0.37), brute_attention(q, k, v, 0.37), rtol=1e-12, atol=1e-13)


def test_attention_config1_shape_vs_loops():
    # 2 heads, D=64, 48 queries x 168 keys; loop reference on a row subset keeps it to seconds
    q = rng.standard_normal((48, 2, 64))
    k = rng.standard_normal((168, 2, 64))
    v = rng.standard_normal((168, 2, 64))
    rows = [0, 17, 47]
    ref = brute_attention(q[rows], k, v, 0.125)
    np.testing.assert_allclose(O.attention(q, k, v, 0.125)[rows], ref, rtol=1e-11, atol=1e-12)


def test_attention_rows_sum_to_one_and_special_cases():
    q = rng.standard_normal((7, 3, 16))
    k = rng.standard_normal((19, 3, 16))
    v = rng.standard_normal((19, 3, 16))
    out, p = O.attention(q, k, v, 0.25, return_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-14)
    assert (p >= 0).all()
    # one visible key -> its V exactly
    one = O.attention(q, k[:1], v[:1], 0.25)
    np.testing.assert_array_equal(one, np.broadcast_to(v[:1].transpose(1, 0, 2).reshape(1, 3, 16), one.shape))
    # all V rows equal -> that row
    vc = np.broadcast_to(v[3], v.shape)
    np.testing.assert_allclose(O.attention(q, k, vc, 0.25), np.broadcast_to(v[3], (7, 3, 16)), atol=1e-14)
    # key order does not matter when nothing is masked
    perm = rng.permutation(19)
    np.testing.assert_allclose(O.attention(q, k[perm], v[perm], 0.25), out, atol=1e-13)
    # heads are independent: changing head 1's keys leaves head 0 untouched
    k2 = k.copy(); k2[:, 1] += 1.0
    np.testing.assert_array_equal(O.attention(q, k2, v, 0.25)[:, 0], out[:, 0])
    # scale really multiplies the logits: scale=0 -> uniform average of V
    np.testing.assert_allclose(O.attention(q, k, v, 0.0), np.broadcast_to(v.mean(0), (7, 3, 16)), atol=1e-14)
    # shift invariance of softmax survives huge logits (max-subtraction)
    big = O.attention(q * 1e3, k, v, 1.0)
    assert np.isfinite(big).all()


# ---------------------------------------------------------------- rolling cache protocol
@pytest.mark.parametrize("window", [1, 2, 4])
def test_cache_protocol_matches_closed_form_100_steps(window):
    """Alg. 3: pop the oldest when L entries are held, then append => after step i the cache holds
    chunks max(0, i-L+1)..i, evicts chunk i-L at step i (i >= L), and a forward at step i sees
    chunks max(0, i-L)..i-1 plus itself."""
    c = O.RollingKVCache(window)
    c.set_sink(np.full((2, 1, 1), -7.0), np.full((2, 1, 1), -9.0))
    for i in range(100):
        k = np.full((3, 1, 1), float(i))
        kk, vv = c.visible(k, k + 0.5)
        ids = sorted(set(kk[2:, 0, 0].astype(int).tolist()))
        assert ids == list(range(max(0, i - window), i + 1))
        assert kk.shape[0] == 2 + 3 * (min(i, window) + 1)
        # sink is first and never changes
        assert (kk[:2] == -7.0).all() and (vv[:2] == -9.0).all()
        n_ev = len(c.evicted)
        c.append(i, k, k + 0.5)
        assert c.chunk_ids() == list(range(max(0, i - window + 1), i + 1))
        if i >= window:
            assert c.evicted[n_ev:] == [i - window]
        else:
            assert len(c.evicted) == n_ev == 0


def test_block_causal_mask_rule():
    m = O.block_causal_mask(n_chunks=7, chunk_tokens=3, sink_tokens=2, window=4)
    for r in range(21):
        i = r // 3
        for col in range(2 + 21):
            if col < 2:
                want = True
            else:
                j = (col - 2) // 3
                want = (i - 4 <= j <= i)
            assert m[r, col] == want


def test_streaming_attention_equals_block_causal_full_sequence():
    """Chunk-vs-cache attention at step i == rows of block i of ONE masked attention over
    [sink, c0..c_{n-1}] (mask rule Sec. 3.2 + window of Eq. 1), including warm-up steps."""
    H, D, nc, ns, W, n = 2, 8, 5, 3, 2, 7
    ks, vs = rng.standard_normal((ns, H, D)), rng.standard_normal((ns, H, D))
    q = rng.standard_normal((n * nc, H, D))
    k = rng.standard_normal((n * nc, H, D))
    v = rng.standard_normal((n * nc, H, D))
    mask = O.block_causal_mask(n, nc, ns, W)
    full = O.attention(q, np.concatenate([ks, k]), np.concatenate([vs, v]), 0.3, mask=mask)
    cache = O.RollingKVCache(W)
    cache.set_sink(ks, vs)
    for i in range(n):
        sl = slice(i * nc, (i + 1) * nc)
        o = O.chunk_attention_step(cache, q[sl], k[sl], v[sl], 0.3, i)
        np.testing.assert_allclose(o, full[sl], rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- RoPE
def complex_rope_1d(x, pos, theta):
    """Textbook 1-D RoPE written with complex numbers: z_k -> z_k * exp(i pos theta^(-2k/d))."""
    d = x.shape[-1]
    z = x[..., 0::2] + 1j * x[..., 1::2]
    w = np.exp(1j * pos[:, None, None] * theta ** (-2.0 * np.arange(d // 2) / d))
    z = z * w
    out = np.empty_like(x)
    out[..., 0::2], out[..., 1::2] = z.real, z.imag
    return out


def test_rope_reduces_to_textbook_per_axis():
    fh, fw = 3, 4
    x = rng.standard_normal((2 * fh * fw, 2, 128))
    y = O.rope3d(x, 5, fh, fw)
    t, r, c = O.token_positions(x.shape[0], 5, fh, fw)
    # positions: frame-major, then row, then column
    assert t.tolist() == [5] * 12 + [6] * 12 and r[:12].tolist() == [0] * 4 + [1] * 4 + [2] * 4 and c[:5].tolist() == [0, 1, 2, 3, 0]
    np.testing.assert_allclose(y[..., :44], complex_rope_1d(x[..., :44], t.astype(float), 1e4), atol=1e-12)
    np.testing.assert_allclose(y[..., 44:86], complex_rope_1d(x[..., 44:86], r.astype(float), 1e4), atol=1e-12)
    np.testing.assert_allclose(y[..., 86:], complex_rope_1d(x[..., 86:], c.astype(float), 1e4), atol=1e-12)


def test_rope_identity_norm_relative_and_composition():
    fh, fw = 3, 4
    n = fh * fw
    x = rng.standard_normal((n, 2, 128))
    y = O.rope3d(x, 0, fh, fw)
    np.testing.assert_array_equal(y[0], x[0])                      # position (0,0,0) is the identity
    pair = lambda a: a[..., 0::2] ** 2 + a[..., 1::2] ** 2
    np.testing.assert_allclose(pair(y), pair(x), rtol=1e-12)       # each pair keeps its norm
    # scores depend only on position differences: shift every t by the same amount
    q, k = rng.standard_normal((n, 2, 128)), rng.standard_normal((n, 2, 128))
    s0 = np.einsum("qhd,khd->hqk", O.rope3d(q, 3, fh, fw), O.rope3d(k, 1, fh, fw))
    s1 = np.einsum("qhd,khd->hqk", O.rope3d(q, 40003, fh, fw), O.rope3d(k, 40001, fh, fw))
    np.testing.assert_allclose(s0, s1, rtol=0, atol=1e-8)          # holds at the 4e4 indices of a 10 000 s rollout
    # rotations compose additively in t (on the first frame where y = x = 0 for token 0)
    one = x[:1]
    a = O.rope3d(O.rope3d(one, 7, fh, fw), 5, fh, fw)
    np.testing.assert_allclose(a, O.rope3d(one, 12, fh, fw), atol=1e-12)
    # rotation direction: pair (1,0) at angle pos*1 (k=0) goes to (cos, sin)
    e = np.zeros((1, 1, 128)); e[0, 0, 0] = 1.0
    r = O.rope3d(e, 2, fh, fw)
    np.testing.assert_allclose(r[0, 0, :2], [math.cos(2.0), math.sin(2.0)], atol=1e-15)
    # second pair of the t axis uses theta^(-2/44)
    e = np.zeros((1, 1, 128)); e[0, 0, 2] = 1.0
    r = O.rope3d(e, 2, fh, fw)
    ang = 2.0 * 1e4 ** (-2.0 / 44)
    np.testing.assert_allclose(r[0, 0, 2:4], [math.cos(ang), math.sin(ang)], atol=1e-15)


# ---------------------------------------------------------------- norms, GELU, linear
def test_rmsnorm_layernorm_closed_forms():
    x = rng.standard_normal((6, 64)) * 3 + 1
    y = O.rmsnorm(x, np.ones(64), eps=0.0)
    np.testing.assert_allclose(np.sqrt((y ** 2).mean(-1)), 1.0, rtol=1e-13)
    np.testing.assert_allclose(O.rmsnorm(17.0 * x, np.ones(64), eps=0.0), y, rtol=1e-12)
    g = rng.standard_normal(64)
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-6), x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6) * g, rtol=1e-14)
    # RMSNorm does not subtract the mean
    assert abs(O.rmsnorm(x, np.ones(64)).mean()) > 0.05
    z = O.layernorm(x, eps=0.0)
    np.testing.assert_allclose(z.mean(-1), 0.0, atol=1e-14)
    np.testing.assert_allclose(z.var(-1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(O.layernorm(x + 5.0, eps=0.0), z, atol=1e-12)
    np.testing.assert_allclose(O.modulate(x, 0.5, 2.0, 0.0), z * 3.0 + 0.5, rtol=1e-13)
    # eps sits inside the square root, added to the mean square / variance
    c = np.full((1, 4), 2.0)
    np.testing.assert_allclose(O.rmsnorm(c, np.ones(4), eps=5.0), 2.0 / 3.0, rtol=1e-15)
    np.testing.assert_allclose(O.layernorm(np.array([[1.0, -1.0]]), eps=3.0), [[0.5, -0.5]], rtol=1e-15)


def test_gelu_tanh():
    x = np.linspace(-6, 6, 2001)
    g = O.gelu_tanh(x)
    assert O.gelu_tanh(np.array(0.0)) == 0.0
    np.testing.assert_allclose(g - O.gelu_tanh(-x), x, atol=1e-14)
    np.testing.assert_allclose(O.gelu_tanh(np.array([30.0, -30.0])), [30.0, 0.0], atol=1e-12)
    assert np.abs(g - 0.5 * x * (1 + erf(x / math.sqrt(2)))).max() < 1e-3
    np.testing.assert_allclose(O.gelu_tanh(np.array(1.0)), 0.5 * (1 + math.tanh(math.sqrt(2 / math.pi) * 1.044715)), rtol=1e-15)


def test_linear_is_x_times_w_transposed():
    x = rng.standard_normal((4, 6))
    W = rng.standard_normal((5, 6))               # [out, in], non-square so a transposed operand cannot pass
    ref = np.array([[sum(x[n, i] * W[o, i] for i in range(6)) for o in range(5)] for n in range(4)])
    np.testing.assert_allclose(O.linear(x, W), ref, rtol=1e-13)
    np.testing.assert_array_equal(O.linear(x, np.eye(6)), x)


# ---------------------------------------------------------------- block / stage
def tiny_cfg():
    return O.StageConfig(n_heads=2, head_dim=8, frame_h=2, frame_w=3, chunk_frames=2, window=2, sink_frames=1,
                         rope_axes=(4, 2, 2))


def tiny_weights(cfg, ffn=24, std=0.3):
    d = cfg.d_model
    shapes = {"W_qkv": (3 * d, d), "W_o": (d, d), "Wc_q": (d, d), "Wc_k": (d, d), "Wc_v": (d, d), "Wc_o": (d, d),
              "W_1": (ffn, d), "W_2": (d, ffn)}
    w = {k: rng.standard_normal(s) * std for k, s in shapes.items()}
    for g in ("g_q", "g_k", "gc_q", "gc_k"):
        w[g] = 1.0 + 0.1 * rng.standard_normal(d)
    return w


def fresh_cache(cfg, seed):
    r = np.random.default_rng(seed)
    c = O.RollingKVCache(cfg.window)
    c.set_sink(r.standard_normal((cfg.frame_tokens, cfg.n_heads, cfg.head_dim)),
               r.standard_normal((cfg.frame_tokens, cfg.n_heads, cfg.head_dim)))
    return c


def test_block_identity_cases_and_mod6_default():
    cfg = tiny_cfg()
    d = cfg.d_model
    x = rng.standard_normal((cfg.chunk_tokens, d))
    ctx = rng.standard_normal((5, d))
    w = tiny_weights(cfg)
    # zero output projections -> the block passes x through
    w0 = dict(w, W_o=np.zeros((d, d)), Wc_o=np.zeros((d, d)), W_2=np.zeros_like(w["W_2"]))
    np.testing.assert_array_equal(O.dit_block(x, w0, fresh_cache(cfg, 1), ctx, None, 0, 1, cfg), x)
    # zero gates remove the self-attention and FFN branches; what is left is x + cross-attention(x)
    m = np.zeros((6, d))
    y = O.dit_block(x, w, fresh_cache(cfg, 1), ctx, m, 0, 1, cfg)
    np.testing.assert_allclose(y, x + O.cross_attention(x, ctx, w, cfg), rtol=1e-13)
    # mod6=None is shift=scale=0, gate=1
    m = np.zeros((6, d)); m[2] = 1.0; m[5] = 1.0
    np.testing.assert_array_equal(O.dit_block(x, w, fresh_cache(cfg, 1), ctx, None, 0, 1, cfg),
                                  O.dit_block(x, w, fresh_cache(cfg, 1), ctx, m, 0, 1, cfg))
    # the block appends exactly one entry: the K/V of this forward (post-norm, post-RoPE K; raw V)
    c = fresh_cache(cfg, 1)
    O.dit_block(x, w, c, ctx, None, 0, 1, cfg)
    q, k, v = O.qkv_for_cache(O.modulate(x, 0.0, 0.0), w, cfg, 1)
    assert c.chunk_ids() == [0]
    np.testing.assert_array_equal(c.blocks[0][1], k)
    np.testing.assert_array_equal(c.blocks[0][2], v)


def test_euler_step_sign_and_dt_zero():
    cfg = tiny_cfg()
    d = cfg.d_model
    x = rng.standard_normal((cfg.chunk_tokens, d))
    ctx = rng.standard_normal((5, d))
    layers = [tiny_weights(cfg), tiny_weights(cfg)]
    caches = [fresh_cache(cfg, 1), fresh_cache(cfg, 2)]
    np.testing.assert_array_equal(O.denoise_stage(x, layers, caches, ctx, None, 0.0, 0, 1, cfg), x)
    caches = [fresh_cache(cfg, 1), fresh_cache(cfg, 2)]
    h = x
    for l in range(2):
        h = O.dit_block(h, layers[l], fresh_cache(cfg, l + 1), ctx, None, 0, 1, cfg)
    np.testing.assert_allclose(O.denoise_stage(x, layers, caches, ctx, None, -0.25, 0, 1, cfg), x - 0.25 * h, rtol=1e-14)
    # flow matching (Sec. 2.1): x_t = (1-s) x0 + s xT, v = xT - x0.  T Euler steps with dt = -1/T and the exact
    # velocity carry xT to x0 -- fixes the sign convention of the update.
    x0, xT, T = rng.standard_normal(9), rng.standard_normal(9), 4
    z = xT.copy()
    for _ in range(T):
        z = z + (xT - x0) * (-1.0 / T)
    np.testing.assert_allclose(z, x0, atol=1e-14)


def test_streaming_stage_equals_full_sequence_stack():
    """Two-layer stack streamed chunk by chunk through per-layer rolling caches == the same stack run once over
    the whole sequence with the block-causal windowed mask (state of block j at layer l depends only on blocks
    j-w..j of layer l-1).  Covers warm-up (steps < w) and eviction (steps > w)."""
    cfg = tiny_cfg()
    d = cfg.d_model
    n_chunks = 6
    layers = [tiny_weights(cfg), tiny_weights(cfg)]
    xs = [rng.standard_normal((cfg.chunk_tokens, d)) for _ in range(n_chunks)]
    ctxs = [rng.standard_normal((5, d)) for _ in range(n_chunks)]
    mod6 = [rng.standard_normal((6, d)) * 0.3 + np.array([0, 0, 1, 0, 0, 1])[:, None] for _ in layers]
    caches = [fresh_cache(cfg, 10 + l) for l in range(2)]
    sinks = [fresh_cache(cfg, 10 + l).sink for l in range(2)]
    t0 = lambda i: 1 + cfg.chunk_frames * i
    full = O.full_sequence_stage(xs, layers, sinks, ctxs, mod6, -0.25, t0, cfg)
    for i in range(n_chunks):
        y = O.denoise_stage(xs[i], layers, caches, ctxs[i], mod6, -0.25, i, t0(i), cfg)
        np.testing.assert_allclose(y, full[i], rtol=1e-10, atol=1e-11)


def test_block_rows_form_equals_whole_chunk_block():
    """dit_block_rows (sampled tokens + explicit visible keys) is the same function as dit_block restricted to rows."""
    cfg = tiny_cfg()
    d = cfg.d_model
    w = tiny_weights(cfg)
    ctx = rng.standard_normal((5, d))
    mod6 = rng.standard_normal((6, d)) * 0.3
    cache = fresh_cache(cfg, 3)
    for i in range(4):
        x = rng.standard_normal((cfg.chunk_tokens, d))
        t0 = 1 + cfg.chunk_frames * i
        before = O.RollingKVCache(cfg.window)
        before.sink, before.blocks = cache.sink, type(cache.blocks)(cache.blocks)
        y = O.dit_block(x, w, cache, ctx, mod6, i, t0, cfg)
        k_new, v_new = cache.blocks[-1][1], cache.blocks[-1][2]
        k_vis, v_vis = before.visible(k_new, v_new)
        rows = np.array([0, 5, cfg.chunk_tokens - 1])
        pos = tuple(p[rows] for p in O.token_positions(cfg.chunk_tokens, t0, cfg.frame_h, cfg.frame_w))
        perm = rng.permutation(k_vis.shape[0])          # key order must not matter
        yr, kr, vr = O.dit_block_rows(x[rows], pos, w, k_vis[perm], v_vis[perm], ctx, mod6, cfg)
        np.testing.assert_allclose(yr, y[rows], rtol=1e-11, atol=1e-12)
        np.testing.assert_array_equal(kr, k_new[rows])
        np.testing.assert_array_equal(vr, v_new[rows])


# ---------------------------------------------------------------- Rolling RoPE / adaptive attention sink (Appendix D)
def test_rolling_sink_keeps_query_to_sink_scores_independent_of_rollout_position():
    """With the sink's temporal index held a fixed offset ahead of the current block's, the logits between a block's
    queries and the sink do not depend on how far the rollout has advanced (the relative distance stays bounded);
    with the sink left at index 0 they do."""
    cfg = tiny_cfg()
    H, D, n = cfg.n_heads, cfg.head_dim, cfg.frame_tokens
    q_raw = rng.standard_normal((n, H, D))
    c = O.RollingKVCache(cfg.window)
    c.set_sink_source(rng.standard_normal((n, H, D)), rng.standard_normal((n, H, D)))
    delta = 2

    def logits(t_q, t_sink):
        c.roll_sink(t_sink, cfg)
        q = O.rope3d(q_raw, t_q, cfg.frame_h, cfg.frame_w, cfg.rope_axes, cfg.theta)
        return np.einsum("nhd,mhd->hnm", q, c.sink[0])

    a = logits(1, 1 + delta)
    b = logits(40001, 40001 + delta)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-9)          # fp64 angles at 4e4 lose ~1e-11
    assert np.abs(logits(40001, 0) - logits(1, 0)).max() > 1e-2   # a static sink index drifts


def test_roll_sink_rotates_only_temporal_pairs_from_the_source():
    cfg = tiny_cfg()                       # rope axes (4, 2, 2): pairs 0,1 temporal; pair 2 row; pair 3 column
    H, D, n = cfg.n_heads, cfg.head_dim, cfg.frame_tokens
    src = rng.standard_normal((n, H, D))
    v = rng.standard_normal((n, H, D))
    c = O.RollingKVCache(cfg.window)
    c.set_sink_source(src, v)
    c.roll_sink(5, cfg)
    k5 = c.sink[0].copy()
    c.roll_sink(9, cfg)
    k9 = c.sink[0].copy()
    # values never change; spatial pairs do not depend on the temporal index
    np.testing.assert_array_equal(c.sink[1], v)
    np.testing.assert_array_equal(k5[..., 4:], k9[..., 4:])
    # temporal pair k as a complex number: index 9 = index 5 turned by 4 * theta^(-2k/4)
    for k in range(2):
        z5 = k5[..., 2 * k] + 1j * k5[..., 2 * k + 1]
        z9 = k9[..., 2 * k] + 1j * k9[..., 2 * k + 1]
        np.testing.assert_allclose(z9, z5 * np.exp(1j * 4 * cfg.theta ** (-2.0 * k / 4)), rtol=1e-12, atol=1e-13)
    # rolling is recomputed from the source: going 5 -> 9 -> 5 gives back the first result bit for bit
    c.roll_sink(5, cfg)
    np.testing.assert_array_equal(c.sink[0], k5)
    # index 0 on a one-row, one-column grid is no rotation at all
    one = O.StageConfig(n_heads=H, head_dim=D, frame_h=1, frame_w=1, chunk_frames=1, window=1, rope_axes=cfg.rope_axes)
    c1 = O.RollingKVCache(1)
    c1.set_sink_source(src[:1], v[:1])
    c1.roll_sink(0, one)
    np.testing.assert_array_equal(c1.sink[0], src[:1])


def test_sink_prefill_special_cases_and_reduction_to_block_rows():
    cfg = tiny_cfg()
    d, H, D = cfg.d_model, cfg.n_heads, cfg.head_dim
    layers = [tiny_weights(cfg), tiny_weights(cfg)]
    ctx = rng.standard_normal((5, d))
    mod6 = [rng.standard_normal((6, d)) * 0.3 + np.array([0, 0, 1, 0, 0, 1])[:, None] for _ in layers]
    x = rng.standard_normal((cfg.frame_tokens, d))
    caches = [fresh_cache(cfg, 20 + l) for l in range(2)]
    for c in caches:                                            # a ring with history, which prefill must not touch
        c.append(0, rng.standard_normal((cfg.chunk_tokens, H, D)), rng.standard_normal((cfg.chunk_tokens, H, D)))
    ring_before = [list(c.blocks) for c in caches]
    t_sink = 7
    y = O.sink_prefill(x, layers, caches, ctx, mod6, t_sink, cfg)
    for c, rb in zip(caches, ring_before):
        assert len(c.blocks) == len(rb) and all(a is b for a, b in zip(c.blocks, rb)) and c.evicted == []
    # layer by layer this is the block evaluated on the sink's tokens with the sink's own K/V as the only visible keys
    h = x
    pos = O.token_positions(cfg.frame_tokens, t_sink, cfg.frame_h, cfg.frame_w)
    for l, w in enumerate(layers):
        u = O.modulate(h, mod6[l][0], mod6[l][1], cfg.eps)
        q, k, v = O.qkv_for_cache(u, w, cfg, t_sink)
        np.testing.assert_allclose(caches[l].sink[0], k, rtol=1e-13, atol=1e-14)
        np.testing.assert_array_equal(caches[l].sink[1], v)
        # the stored source is K before RoPE: row block [d, 2d) of the fused weight, normalised over all channels
        k_lin = u @ w["W_qkv"][d:2 * d].T
        k_src = k_lin / np.sqrt((k_lin ** 2).mean(-1, keepdims=True) + cfg.eps) * w["g_k"]
        np.testing.assert_allclose(caches[l].sink_source.reshape(-1, d), k_src, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(v.reshape(-1, d), u @ w["W_qkv"][2 * d:].T, rtol=1e-12, atol=1e-13)
        h, _, _ = O.dit_block_rows(h, pos, w, k, v, ctx, mod6[l], cfg)
    np.testing.assert_allclose(y, h, rtol=1e-11, atol=1e-12)
    # one-token sink: softmax over a single key is 1, so the attention output is that token's V
    one = O.StageConfig(n_heads=H, head_dim=D, frame_h=1, frame_w=1, chunk_frames=1, window=1, rope_axes=cfg.rope_axes)
    w = layers[0]
    x1 = rng.standard_normal((1, d))
    c1 = [O.RollingKVCache(1)]
    y1 = O.sink_prefill(x1, [w], c1, ctx, None, 3, one)
    u = O.layernorm(x1, one.eps)
    mid = x1 + (u @ w["W_qkv"][2 * d:].T) @ w["W_o"].T
    mid = mid + O.cross_attention(mid, ctx, w, one)
    np.testing.assert_allclose(y1, mid + O.ffn(O.layernorm(mid, one.eps), w), rtol=1e-12, atol=1e-13)


def test_streaming_with_sink_swap_and_rolling_index_runs_the_documented_sequence():
    """Alg. 3 with both mechanisms, on the stage level: prefill the reference sink, run block 0, swap the sink for the
    model's own output (second warm-up), then run blocks 1.. with the sink index re-assigned before every forward.
    Checked against the same blocks evaluated row-wise with explicitly assembled visible keys."""
    cfg = tiny_cfg()
    d, H, D = cfg.d_model, cfg.n_heads, cfg.head_dim
    layers = [tiny_weights(cfg)]
    ctx = rng.standard_normal((5, d))
    caches = [O.RollingKVCache(cfg.window)]
    delta = 1
    t0 = lambda i: 1 + cfg.chunk_frames * i
    t_sink = lambda i: t0(i) + cfg.chunk_frames - 1 + delta
    O.sink_prefill(rng.standard_normal((cfg.frame_tokens, d)), layers, caches, ctx, None, t_sink(0), cfg)
    src_ref = caches[0].sink_source.copy()
    outs = []
    for i in range(5):
        caches[0].roll_sink(t_sink(i), cfg)
        x = rng.standard_normal((cfg.chunk_tokens, d))
        # expected: rows form with the visible set assembled by hand
        k_sink = O.rope3d(caches[0].sink_source, t_sink(i), cfg.frame_h, cfg.frame_w, cfg.rope_axes, cfg.theta)
        u = O.modulate(x, 0.0, 0.0, cfg.eps)
        q, k, v = O.qkv_for_cache(u, layers[0], cfg, t0(i))
        kv = np.concatenate([k_sink] + [b[1] for b in caches[0].blocks] + [k], 0)
        vv = np.concatenate([caches[0].sink[1]] + [b[2] for b in caches[0].blocks] + [v], 0)
        want, _, _ = O.dit_block_rows(x, O.token_positions(cfg.chunk_tokens, t0(i), cfg.frame_h, cfg.frame_w), layers[0], kv, vv,
                                      ctx, None, cfg)
        y = O.denoise_stage(x, layers, caches, ctx, None, -0.25, i, t0(i), cfg)
        np.testing.assert_allclose(y, x - 0.25 * want, rtol=1e-11, atol=1e-12)
        outs.append(y)
        if i == 0:   # sink swap: the first generated frame becomes the sink; its K/V come from a second warm-up
            assert np.array_equal(caches[0].sink_source, src_ref)
            O.sink_prefill(y[:cfg.frame_tokens], layers, caches, ctx, None, t_sink(1), cfg)
            assert not np.array_equal(caches[0].sink_source, src_ref)
            assert caches[0].chunk_ids() == [0]


def test_sample_chunk_is_T_stages_with_independent_per_step_caches():
    """Alg. 3 inner loop: T forwards of the same weights, each with its own cache and its own modulation; T = 1 is one
    stage; the cache of step s holds only K/V produced at step s (timestep forcing: a block and the cache it attends to
    share the noise level), so perturbing the history of step 1 cannot change what step 0 computes."""
    cfg = tiny_cfg()
    d, H, D = cfg.d_model, cfg.n_heads, cfg.head_dim
    layers = [tiny_weights(cfg)]
    ctx = rng.standard_normal((5, d))
    T = 3
    mod6 = [[rng.standard_normal((6, d)) * 0.3 + np.array([0, 0, 1, 0, 0, 1])[:, None]] for _ in range(T)]
    mk = lambda: [[fresh_cache(cfg, 40 + s)] for s in range(T)]
    caches, twin = mk(), mk()
    x0 = rng.standard_normal((cfg.chunk_tokens, d))
    outs = []
    for i in range(3):
        x = rng.standard_normal((cfg.chunk_tokens, d))
        want = x
        for s in range(T):
            want = O.denoise_stage(want, layers, twin[s], ctx, mod6[s], -1.0 / T, i, 1 + 2 * i, cfg)
        got = O.sample_chunk(x, layers, caches, ctx, mod6, -1.0 / T, i, 1 + 2 * i, cfg)
        np.testing.assert_array_equal(got, want)
        for s in range(T):
            assert caches[s][0].chunk_ids() == list(range(max(0, i + 1 - cfg.window), i + 1))
    one = O.sample_chunk(x0, layers, [[fresh_cache(cfg, 40)]], ctx, [mod6[0]], -0.5, 0, 1, cfg)
    np.testing.assert_array_equal(one, O.denoise_stage(x0, layers, [fresh_cache(cfg, 40)], ctx, mod6[0], -0.5, 0, 1, cfg))
    # independence of the per-step caches
    a, b = mk(), mk()
    b[1][0].append(0, rng.standard_normal((cfg.chunk_tokens, H, D)), rng.standard_normal((cfg.chunk_tokens, H, D)))
    a[1][0].append(0, rng.standard_normal((cfg.chunk_tokens, H, D)), rng.standard_normal((cfg.chunk_tokens, H, D)))
    xa = O.denoise_stage(x0, layers, a[0], ctx, mod6[0], -1.0 / T, 0, 1, cfg)
    xb = O.denoise_stage(x0, layers, b[0], ctx, mod6[0], -1.0 / T, 0, 1, cfg)
    np.testing.assert_array_equal(xa, xb)
    assert np.abs(O.denoise_stage(xa, layers, a[1], ctx, mod6[1], -1.0 / T, 1, 1, cfg)
                  - O.denoise_stage(xb, layers, b[1], ctx, mod6[1], -1.0 / T, 1, 1, cfg)).max() > 1e-6


# ---------------------------------------------------------------- FP8 E4M3 per-tensor linears (Appendix C)
def e4m3_decode_table():
    """All 256 codes decoded from the format's definition: s eeee mmm, bias 7, e = 0 subnormal, 0x7f / 0xff NaN."""
    vals = np.empty(256)
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = m * 2.0 ** -9
        else:
            v = (1 + m / 8.0) * 2.0 ** (e - 7)
        vals[c] = -v if s else v
    return vals


def test_e4m3_rounding_against_the_code_table_and_torch():
    import torch
    tab = e4m3_decode_table()
    fin = tab[np.isfinite(tab)]
    assert fin.max() == 448.0 and np.abs(fin[fin != 0]).min() == 2.0 ** -9
    # every grid value is a fixed point; midpoints go to the even mantissa; saturation
    np.testing.assert_array_equal(O.e4m3_round(fin), fin)
    pos = np.unique(np.abs(fin))                       # 127 values: 0, 7 subnormals, 119 normals
    assert len(pos) == 127
    mid = (pos[:-1] + pos[1:]) / 2
    even = np.where((np.arange(len(pos) - 1) % 2) == 0, pos[:-1], pos[1:])     # code parity = mantissa parity
    np.testing.assert_array_equal(O.e4m3_round(mid), even)
    np.testing.assert_array_equal(O.e4m3_round(-mid), -even)
    np.testing.assert_array_equal(O.e4m3_round(np.array([448.0, 449.0, 463.9, 1e6, -1e6])), [448, 448, 448, 448, -448])
    # nearest-neighbour brute force on random values, and the library's conversion of the same published format
    y = np.concatenate([rng.standard_normal(3000) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)])
    y = y[np.abs(y) <= 448].astype(np.float32).astype(np.float64)
    got = O.e4m3_round(y)
    d = np.abs(y[:, None] - fin[None, :])
    assert np.all(np.abs(got - y) <= d.min(1) + 0.0)
    lib = torch.from_numpy(y.astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(got, lib)
    # relative error of a normal value is at most half a mantissa step
    big = np.abs(y) >= 2.0 ** -6
    assert (np.abs(got[big] - y[big]) / np.abs(y[big])).max() <= 2.0 ** -4


def test_fp8_per_tensor_quantisation_and_linear():
    x = rng.standard_normal((37, 64)) * 3.0
    x[5, 7] = -11.5                                   # the amax element
    q, s = O.fp8_quantize_per_tensor(x)
    assert s == float(np.float32(11.5) / np.float32(448)) and q[5, 7] == -448.0
    assert set(np.unique(np.abs(q))) <= set(np.abs(e4m3_decode_table()[:127]))
    # dequantised values are within half a grid step of x: |x| <= amax, step <= 2^-4 of the value (normals) or 2^-9*s
    err = np.abs(q * s - x.astype(np.float32).astype(np.float64))
    assert (err <= np.maximum(np.abs(x) * 2.0 ** -4, 2.0 ** -10 * s) * (1 + 1e-6)).all()
    # scale invariance: quantising 4x gives the same grid values and 4x the scale (powers of two are exact in fp32)
    q4, s4 = O.fp8_quantize_per_tensor(4 * x)
    np.testing.assert_array_equal(q4, q)
    assert s4 == 4 * s
    zq, zs = O.fp8_quantize_per_tensor(np.zeros((3, 8)))
    assert zs == 1.0 and not zq.any()
    # operands already on the grid (times a power of two) pass through exactly: linear_fp8 == exact product
    tab = e4m3_decode_table()
    grid = tab[np.isfinite(tab)]
    a = rng.choice(grid, size=(9, 16)); a[0, 0] = 448.0
    w = rng.choice(grid, size=(5, 16)) * 0.25; w[0, 0] = 112.0
    np.testing.assert_allclose(O.linear_fp8(a, w), a @ w.T, rtol=1e-6, atol=0)
    # general operands: the error against the exact product is bounded by the two half-step bounds
    W = rng.standard_normal((24, 64)) * 0.05
    y, ref = O.linear_fp8(x, W), x @ W.T
    bound = (np.abs(x) * 2.0 ** -4 + 2.0 ** -10 * s) @ np.abs(W).T + np.abs(x) @ (np.abs(W) * 2.0 ** -4 + 1e-4).T
    assert (np.abs(y - ref) <= bound * 1.1).all() and np.abs(y - ref).max() > 1e-4


def test_block_with_fp8_linears_is_a_small_perturbation_of_the_exact_block():
    cfg, cfg8 = tiny_cfg(), tiny_cfg()
    cfg8.fp8_linears = True
    d = cfg.d_model
    x = rng.standard_normal((cfg.chunk_tokens, d))
    ctx = rng.standard_normal((5, d))
    w = tiny_weights(cfg)
    y = O.dit_block(x, w, fresh_cache(cfg, 1), ctx, None, 0, 1, cfg)
    y8 = O.dit_block(x, w, fresh_cache(cfg, 1), ctx, None, 0, 1, cfg8)
    rel = np.sqrt(((y8 - y) ** 2).mean() / ((y - x) ** 2).mean())       # against what the block adds to x
    assert 1e-3 < rel < 0.12, rel                                       # 3 mantissa bits: a few per cent per linear
    # zero output projections: an all-zero tensor quantises to zeros (scale 1), the block stays the identity
    w0 = dict(w, W_o=np.zeros((d, d)), Wc_o=np.zeros((d, d)), W_2=np.zeros_like(w["W_2"]))
    np.testing.assert_array_equal(O.dit_block(x, w0, fresh_cache(cfg, 1), ctx, None, 0, 1, cfg8), x)
    # what goes into the cache is computed from the quantised QKV projection
    c = fresh_cache(cfg, 1)
    O.dit_block(x, w, c, ctx, None, 0, 1, cfg8)
    qkv = O.linear_fp8(O.layernorm(x, cfg.eps), w["W_qkv"])
    np.testing.assert_array_equal(c.blocks[0][2].reshape(-1, d), qkv[:, 2 * d:])


# ---------------------------------------------------------------- streaming causal convolution (Appendix C)
def test_causal_conv3d_against_loops_and_the_library_convolution():
    import torch
    T, H, W, Ci, Co = 4, 3, 5, 2, 3
    x = rng.standard_normal((T, H, W, Ci))
    w = rng.standard_normal((Co, 3, 3, 3, Ci))
    b = rng.standard_normal(Co)
    got = O.causal_conv3d(x, w, b)
    ref = np.zeros((T, H, W, Co))
    for t in range(T):
        for y in range(H):
            for xx in range(W):
                for o in range(Co):
                    acc = b[o]
                    for dt in range(3):
                        for dy in range(3):
                            for dx in range(3):
                                tt, yy, xs = t + dt - 2, y + dy - 1, xx + dx - 1
                                if tt < 0 or yy < 0 or yy >= H or xs < 0 or xs >= W:
                                    continue
                                for c in range(Ci):
                                    acc += w[o, dt, dy, dx, c] * x[tt, yy, xs, c]
                    ref[t, y, xx, o] = acc
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)
    # library routine: conv3d (a cross-correlation) on the explicitly padded volume, channels first
    xt = torch.from_numpy(x).permute(3, 0, 1, 2)[None]                       # [1, Ci, T, H, W]
    xt = torch.nn.functional.pad(xt, (1, 1, 1, 1, 2, 0))                     # W, H by 1 each side; time by 2 in the past only
    wt = torch.from_numpy(w).permute(0, 4, 1, 2, 3).contiguous()             # [Co, Ci, 3, 3, 3]
    lib = torch.nn.functional.conv3d(xt, wt, torch.from_numpy(b))[0].permute(1, 2, 3, 0).numpy()
    np.testing.assert_allclose(got, lib, rtol=1e-11, atol=1e-11)
    # causality: a change in frame 2 leaves frames 0 and 1 of the output alone and changes frame 2
    x2 = x.copy(); x2[2] += 1.0
    got2 = O.causal_conv3d(x2, w, b)
    np.testing.assert_array_equal(got2[:2], got[:2])
    assert np.abs(got2[2] - got[2]).max() > 1e-3 and np.abs(got2[3] - got[3]).max() > 1e-3


@pytest.mark.parametrize("chunks", [[1, 1, 1, 1, 1, 1, 1], [3, 3, 1], [2, 5], [7], [1, 4, 2]])
def test_streaming_conv_with_two_frame_cache_equals_whole_sequence(chunks):
    T, H, W, Ci, Co = sum(chunks), 4, 3, 3, 2
    x = rng.standard_normal((T, H, W, Ci))
    w = rng.standard_normal((Co, 3, 3, 3, Ci))
    b = rng.standard_normal(Co)
    whole = O.causal_conv3d(x, w, b)
    cache = O.CausalConvCache()
    outs, t = [], 0
    for n in chunks:
        outs.append(cache.step(x[t:t + n], w, b))
        t += n
        np.testing.assert_array_equal(cache.frames, np.concatenate([np.zeros((2, H, W, Ci)), x[:t]])[-2:])
    np.testing.assert_allclose(np.concatenate(outs), whole, rtol=1e-12, atol=1e-12)
    assert O.silu(0.0) == 0.0 and abs(O.silu(30.0) - 30.0) < 1e-11 and abs(O.silu(-1.0) + 1.0 / (1.0 + math.e)) < 1e-15
