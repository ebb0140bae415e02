"""CPU oracle for one denoising stage of the streaming causal video DiT (Live Avatar, arXiv 2512.04677).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition that the HIP kernels are
checked against.  Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import it;
the product path never does.  It shares no code with the HIP path and imports nothing from it.

Everything is numpy float64.  Inputs are whatever values the caller hands over (the tests hand over
bf16-rounded values converted exactly to float64); no intermediate is rounded to a narrower type, and
there is no tiling, fusion or reordering beyond what each definition states.

What the paper fixes and where (own words):
  * Eq. 1 (Sec. 3.1): a block of 3 latent frames is denoised conditioned on the ``w`` previous blocks
    held in a KV cache at the same noise level, on a sink frame, and on audio / text embeddings.
  * Sec. 3.2, Stage 1: attention is full inside a block and strictly causal between blocks.
  * Alg. 3 / Alg. 4 (Appendix D): after the forward the cache drops its oldest entry if it already
    holds ``L`` entries and then appends the K/V the forward produced from the *noisy* block
    ("History Corrupt", Sec. 3.3); the latent moves by an Euler step ``x <- x + v*dt``, ``dt = -1/T``.
  * Sec. 3.3 / Sec. 4.1: one sink frame stays in the cache for ever; ``w = 4``; blocks of 3 latents.
  * Appendix D, "Rolling RoPE": rotary position indices grow per generated frame; the sink carries
    its own temporal index (0 unless re-assigned); with Rolling RoPE that index is re-assigned at
    every block step to a value slightly ahead of the current block's, by recomputing the rotary
    embedding of the cached sink keys (Phi(sink) in Alg. 3 / Alg. 4).  The offset itself is not
    given: the caller supplies the index ("parity unpinned" for its value, the transform is pinned).
  * Sec. 3.3 / Appendix D, Adaptive Attention Sink: after the first block the sink is replaced by
    the model's own first generated latent, which needs a second warm-up to produce its K/V.

What the paper does not give (hidden size, heads, FFN width, norm placement, RoPE split, GELU form) is
taken from the build's workload description; each such reading is stated where the function that uses it is defined.

Parity pins live in tests/test_oracle_*.py.  Unpinned by anything the paper prints (the paper has no
worked numeric example): the *placement* of RMSNorm / LayerNorm / gates inside the block ("parity
unpinned" for that wiring; each primitive itself is pinned by closed forms and brute force).
"""
from collections import deque

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------------------
# primitives
# --------------------------------------------------------------------------------------------------
def softmax_rows(s):
    """Row-wise softmax of a 2-D score matrix, max-subtracted (textbook definition)."""
    s = np.asarray(s, F64)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, scale, mask=None, return_probs=False):
    """Scaled dot-product attention, one softmax per (query, head) over all given keys.

    q [Nq, H, D]; k, v [Nk, H, D]; ``mask`` optional boolean [Nq, Nk] (True = visible).
    This is the operation the streaming path performs from the current block's queries to the
    concatenation {sink, cached blocks, current block} (Eq. 1; Appendix C, attention paragraph).
    With ``mask=None`` every key is visible, which is the chunk-to-cache case: the mask rule of
    Sec. 3.2 hides nothing that is in the cache.
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    v = np.asarray(v, F64)
    nq, H, D = q.shape
    out = np.empty((nq, H, v.shape[2]), F64)
    probs = np.empty((H, nq, k.shape[0]), F64) if return_probs else None
    for h in range(H):
        s = (q[:, h, :] @ k[:, h, :].T) * scale
        if mask is not None:
            s = np.where(mask, s, -np.inf)
        p = softmax_rows(s)
        out[:, h, :] = p @ v[:, h, :]
        if return_probs:
            probs[h] = p
    return (out, probs) if return_probs else out


def rmsnorm(x, g, eps=1e-6):
    """y = x / sqrt(mean_c(x^2) + eps) * g over the last axis (all channels of a token)."""
    x = np.asarray(x, F64)
    r = np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x / r * np.asarray(g, F64)


def layernorm(x, eps=1e-6):
    """Affine-free LayerNorm over the last axis (biased variance)."""
    x = np.asarray(x, F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def modulate(x, shift, scale, eps=1e-6):
    """u = LayerNorm(x) * (1 + scale) + shift."""
    return layernorm(x, eps) * (1.0 + np.asarray(scale, F64)) + np.asarray(shift, F64)


def gelu_tanh(x):
    """0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) ))."""
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def linear(x, W):
    """y[n, o] = sum_i x[n, i] W[o, i]   (weights stored [out, in], no bias)."""
    return np.asarray(x, F64) @ np.asarray(W, F64).T


# --------------------------------------------------------------------------------------------------
# FP8 (E4M3) linears with per-tensor dynamic scaling (Appendix C, "FP8 Quantization")
# --------------------------------------------------------------------------------------------------
E4M3_MAX = 448.0          # largest finite value of the 8-bit format: 1.75 * 2^8 (no infinities, one NaN pattern per sign)


def e4m3_round(y):
    """Round to the nearest value of the E4M3 grid (ties to even), saturating at +-448.

    Grid: sign, 4 exponent bits (bias 7), 3 mantissa bits; normals 2^e * (1 + m/8) for e = -6 .. 8, subnormals
    m * 2^-9.  The spacing around |y| in [2^e, 2^(e+1)) is 2^(e-3), floored at 2^-9."""
    y = np.asarray(y, F64)
    a = np.abs(y)
    e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6, 8)
    q = np.exp2(e - 3)
    r = np.rint(a / q) * q                      # rint = ties to even; a/q is exact (power-of-two divisor)
    return np.sign(y) * np.minimum(r, E4M3_MAX)


def fp8_quantize_per_tensor(x):
    """Per-tensor dynamic scaling: amax = max|x| over the whole tensor, grid value = e4m3_round(x * (448 / amax)),
    represented value = grid value * (amax / 448).  The two scale factors and the product x * (448/amax) are formed in
    fp32 -- the precision in which the kernel decides the 8-bit code -- so that both sides round the same number.
    Returns (grid values as float64, scale as float64); an all-zero tensor gets scale 1."""
    x32 = np.asarray(x, np.float32)
    amax = np.float32(np.abs(x32).max()) if x32.size else np.float32(0)
    if amax == 0:
        return np.zeros(x32.shape, F64), 1.0
    inv = np.float32(E4M3_MAX) / amax
    scale = amax / np.float32(E4M3_MAX)
    y = x32 * inv                                # fp32 product
    return e4m3_round(y.astype(F64)), float(scale)


def linear_fp8(x, W):
    """y = dequant(quant(x)) @ dequant(quant(W))^T: both operands on the E4M3 grid with their own per-tensor scale,
    the contraction itself exact (fp64)."""
    xq, sx = fp8_quantize_per_tensor(x)
    wq, sw = fp8_quantize_per_tensor(W)
    return (xq @ wq.T) * (sx * sw)


def token_positions(n_tokens, t0, frame_h, frame_w):
    """(t, y, x) of token n laid out frame-major, then row, then column; t = t0 + frame."""
    n = np.arange(n_tokens)
    per_frame = frame_h * frame_w
    return t0 + n // per_frame, (n // frame_w) % frame_h, n % frame_w


def rope3d(x, t0, frame_h, frame_w, axes=(44, 42, 42), theta=10000.0, positions=None):
    """Three-axis rotary embedding on x [N, H, D], D = sum(axes).

    The head dimension is cut into consecutive groups of ``axes`` dims for (t, y, x).  Inside a
    group of d_a dims, adjacent dims (2k, 2k+1) form pair k and are rotated by the angle
    ``pos_a * theta**(-2k/d_a)``:  (a, b) -> (a cos - b sin, a sin + b cos).
    Temporal positions count latent frames (Appendix: a 10 000 s rollout reaches an index near
    4e4, i.e. one index per latent frame).
    """
    x = np.asarray(x, F64)
    N, H, D = x.shape
    assert sum(axes) == D and all(a % 2 == 0 for a in axes)
    pos = positions if positions is not None else token_positions(N, t0, frame_h, frame_w)
    out = np.empty_like(x)
    base = 0
    for axis, d_a in enumerate(axes):
        kk = np.arange(d_a // 2)
        freq = theta ** (-2.0 * kk / d_a)                      # [d_a/2]
        ang = np.asarray(pos[axis], F64)[:, None] * freq[None, :]   # [N, d_a/2]
        c = np.cos(ang)[:, None, :]
        s = np.sin(ang)[:, None, :]
        a = x[:, :, base:base + d_a:2]
        b = x[:, :, base + 1:base + d_a:2]
        out[:, :, base:base + d_a:2] = a * c - b * s
        out[:, :, base + 1:base + d_a:2] = a * s + b * c
        base += d_a
    return out


# --------------------------------------------------------------------------------------------------
# rolling KV cache: the list-of-blocks protocol of Alg. 3 / Alg. 4, kept as a deque (never a ring)
# --------------------------------------------------------------------------------------------------
class RollingKVCache:
    """One layer's cache at one timestep: a permanent sink entry plus at most ``window`` past blocks."""

    def __init__(self, window):
        self.window = int(window)
        self.sink = None                 # (k, v) of the sink frame, never evicted (Sec. 3.3)
        self.sink_source = None          # un-rotated sink keys when the sink's RoPE index is re-assigned per step
        self.blocks = deque()            # (chunk_index, k, v), oldest first
        self.evicted = []                # chunk indices dropped so far, in order

    def set_sink(self, k, v):
        self.sink = (np.asarray(k, F64), np.asarray(v, F64))
        self.sink_source = None

    def set_sink_source(self, k_src, v):
        """Install a sink whose keys are kept UN-rotated (normalised, before RoPE), so that its temporal index can be
        re-assigned at every block step (Appendix D, "Rolling RoPE"); also what the sink swap of the Adaptive
        Attention Sink installs (Sec. 3.3; Alg. 3, the assignment after the first block).  The sink keys are
        undefined until ``roll_sink`` is called."""
        self.sink_source = np.asarray(k_src, F64)
        self.sink = (None, np.asarray(v, F64))

    def roll_sink(self, t_sink, cfg):
        """Phi(sink) of Alg. 3 / Alg. 4: the sink keys become RoPE(source) with the sink's first frame at temporal
        index ``t_sink`` (spatial indices are those of the frame grid).  Always recomputed from the un-rotated
        source, never from the previous rotation; the sink values are not touched."""
        k = rope3d(self.sink_source, int(t_sink), cfg.frame_h, cfg.frame_w, cfg.rope_axes, cfg.theta)
        self.sink = (k, self.sink[1])

    def visible(self, k_cur, v_cur):
        """Keys/values a forward of the current block sees: sink, cached blocks (oldest first), itself."""
        ks = [self.sink[0]] + [b[1] for b in self.blocks] + [np.asarray(k_cur, F64)]
        vs = [self.sink[1]] + [b[2] for b in self.blocks] + [np.asarray(v_cur, F64)]
        return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)

    def append(self, chunk_index, k, v):
        """After the forward: drop the oldest block if the cache is full, then append (Alg. 3)."""
        if len(self.blocks) == self.window:
            self.evicted.append(self.blocks.popleft()[0])
        self.blocks.append((int(chunk_index), np.asarray(k, F64), np.asarray(v, F64)))

    def chunk_ids(self):
        return [b[0] for b in self.blocks]


def chunk_attention_step(cache, q, k_cur, v_cur, scale, chunk_index):
    """One streaming step: attend to {sink, cache, self}, then evict/append.  Returns O [Nq, H, D]."""
    kk, vv = cache.visible(k_cur, v_cur)
    out = attention(q, kk, vv, scale)
    cache.append(chunk_index, k_cur, v_cur)
    return out


def block_causal_mask(n_chunks, chunk_tokens, sink_tokens, window):
    """Visibility over the sequence [sink, c_0 .. c_{n-1}] for the queries of c_0 .. c_{n-1}.

    Row block i sees the sink, itself in full, and the ``window`` blocks before it (Sec. 3.2 mask
    rule restricted to the cache window of Eq. 1)."""
    nq = n_chunks * chunk_tokens
    nk = sink_tokens + nq
    m = np.zeros((nq, nk), bool)
    m[:, :sink_tokens] = True
    for i in range(n_chunks):
        lo = max(0, i - window)
        m[i * chunk_tokens:(i + 1) * chunk_tokens,
          sink_tokens + lo * chunk_tokens: sink_tokens + (i + 1) * chunk_tokens] = True
    return m


# --------------------------------------------------------------------------------------------------
# DiT block and denoise stage
# --------------------------------------------------------------------------------------------------
class StageConfig:
    """Shapes of the stack.  Defaults are the 14B-scale workload; tests shrink them."""

    def __init__(self, n_heads=40, head_dim=128, frame_h=30, frame_w=52, chunk_frames=3, window=4,
                 sink_frames=1, rope_axes=(44, 42, 42), theta=10000.0, eps=1e-6, fp8_linears=False):
        self.n_heads, self.head_dim = n_heads, head_dim
        self.frame_h, self.frame_w = frame_h, frame_w
        self.chunk_frames, self.window, self.sink_frames = chunk_frames, window, sink_frames
        self.rope_axes, self.theta, self.eps = tuple(rope_axes), theta, eps
        # Appendix C: every linear projection of the block takes both operands on the E4M3 grid with per-tensor
        # dynamic scales (each weight matrix as stored -- the fused QKV matrix is one tensor -- and each activation
        # tensor as a whole).  Attention, norms, RoPE, GELU and the residual adds are not quantised.
        self.fp8_linears = bool(fp8_linears)

    @property
    def d_model(self):
        return self.n_heads * self.head_dim

    @property
    def frame_tokens(self):
        return self.frame_h * self.frame_w

    @property
    def chunk_tokens(self):
        return self.chunk_frames * self.frame_tokens


def _lin(cfg):
    return linear_fp8 if cfg is not None and cfg.fp8_linears else linear


def _mod6(mod6, d):
    """(shift1, scale1, gate1, shift2, scale2, gate2); None means shift = scale = 0, gate = 1."""
    if mod6 is None:
        z, o = np.zeros(d, F64), np.ones(d, F64)
        return z, z, o, z, z, o
    m = np.asarray(mod6, F64).reshape(6, d)
    return m[0], m[1], m[2], m[3], m[4], m[5]


def qkv_for_cache(u, w, cfg, t0, positions=None):
    """QKV projection, Q/K RMSNorm over all channels, 3-D RoPE on Q and K; V untouched."""
    H, D = cfg.n_heads, cfg.head_dim
    d = H * D
    qkv = _lin(cfg)(u, w["W_qkv"])
    q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    if w.get("g_q") is not None:
        q = rmsnorm(q, w["g_q"], cfg.eps)
    if w.get("g_k") is not None:
        k = rmsnorm(k, w["g_k"], cfg.eps)
    n = u.shape[0]
    q = rope3d(q.reshape(n, H, D), t0, cfg.frame_h, cfg.frame_w, cfg.rope_axes, cfg.theta, positions)
    k = rope3d(k.reshape(n, H, D), t0, cfg.frame_h, cfg.frame_w, cfg.rope_axes, cfg.theta, positions)
    return q, k, v.reshape(n, H, D)


def cross_attention(x, ctx, w, cfg):
    """Attention from LayerNorm(x) to the audio+text context; Q/K RMSNorm if gains given; no RoPE."""
    H, D = cfg.n_heads, cfg.head_dim
    n = x.shape[0]
    q = _lin(cfg)(layernorm(x, cfg.eps), w["Wc_q"])
    k = _lin(cfg)(ctx, w["Wc_k"])
    v = _lin(cfg)(ctx, w["Wc_v"])
    if w.get("gc_q") is not None:
        q = rmsnorm(q, w["gc_q"], cfg.eps)
    if w.get("gc_k") is not None:
        k = rmsnorm(k, w["gc_k"], cfg.eps)
    m = ctx.shape[0]
    o = attention(q.reshape(n, H, D), k.reshape(m, H, D), v.reshape(m, H, D), 1.0 / np.sqrt(D))
    return _lin(cfg)(o.reshape(n, H * D), w["Wc_o"])


def ffn(u, w, cfg=None):
    return _lin(cfg)(gelu_tanh(_lin(cfg)(u, w["W_1"])), w["W_2"])


def dit_block(x, w, cache, ctx, mod6, chunk_index, t0, cfg):
    """One transformer block on the current chunk's tokens x [N, d]; updates ``cache`` (this layer's).

    Order: modulated pre-norm -> QKV -> RMSNorm+RoPE -> attention over {sink, cache, self} ->
    gated output projection (residual) -> cross-attention (residual) -> modulated pre-norm ->
    GELU-tanh FFN (gated residual).  The K/V appended are the ones this very forward computed from
    the noisy chunk (History Corrupt): nothing is re-encoded afterwards.
    """
    x = np.asarray(x, F64)
    H, D = cfg.n_heads, cfg.head_dim
    d = H * D
    sh1, sc1, g1, sh2, sc2, g2 = _mod6(mod6, d)
    u = modulate(x, sh1, sc1, cfg.eps)
    q, k, v = qkv_for_cache(u, w, cfg, t0)
    o = chunk_attention_step(cache, q, k, v, 1.0 / np.sqrt(D), chunk_index)
    x = x + g1 * _lin(cfg)(o.reshape(-1, d), w["W_o"])
    x = x + cross_attention(x, np.asarray(ctx, F64), w, cfg)
    u2 = modulate(x, sh2, sc2, cfg.eps)
    x = x + g2 * ffn(u2, w, cfg)
    return x


def dit_block_rows(x_rows, positions, w, k_visible, v_visible, ctx, mod6, cfg):
    """The block's output for a SUBSET of the chunk's tokens, given all keys/values those tokens see.

    Same formulas as dit_block, row by row: every step of the block acts on each token independently except the
    self-attention, whose keys/values (sink, cached chunks and the current chunk, any order) are passed in.
    Used for sampled checks at sizes where the whole chunk is too much for the CPU.  Returns (x_out_rows,
    k_rows, v_rows): k_rows / v_rows are what the block stores in the cache for these tokens."""
    x = np.asarray(x_rows, F64)
    H, D = cfg.n_heads, cfg.head_dim
    d = H * D
    sh1, sc1, g1, sh2, sc2, g2 = _mod6(mod6, d)
    u = modulate(x, sh1, sc1, cfg.eps)
    q, k, v = qkv_for_cache(u, w, cfg, 0, positions)
    o = attention(q, k_visible, v_visible, 1.0 / np.sqrt(D))
    x = x + g1 * _lin(cfg)(o.reshape(-1, d), w["W_o"])
    x = x + cross_attention(x, np.asarray(ctx, F64), w, cfg)
    u2 = modulate(x, sh2, sc2, cfg.eps)
    x = x + g2 * ffn(u2, w, cfg)
    return x, k, v


def sink_keys_values(u, w, cfg):
    """Un-rotated sink keys and sink values of one layer: K projection + RMSNorm (no RoPE), V projection."""
    H, D = cfg.n_heads, cfg.head_dim
    d = H * D
    qkv = _lin(cfg)(u, w["W_qkv"])
    k, v = qkv[:, d:2 * d], qkv[:, 2 * d:]
    if w.get("g_k") is not None:
        k = rmsnorm(k, w["g_k"], cfg.eps)
    n = u.shape[0]
    return k.reshape(n, H, D), v.reshape(n, H, D)


def sink_prefill(x_sink, layers, caches, ctx, mod6_per_layer, t_sink, cfg):
    """Run the sink frame's tokens x_sink [sink_tokens, d] through the stack and install, per layer, the sink's
    un-rotated keys and its values in ``caches`` (the warm-up that the sink swap of the Adaptive Attention Sink needs,
    Appendix D).  Reading (the paper does not say what the sink attends to): the sink frame attends to itself only,
    with its own frame at temporal index ``t_sink``; every other step of the block is the one of ``dit_block``.
    The ring of past blocks is not touched.  Returns the stack's output for the sink tokens (not used by the method)."""
    x = np.asarray(x_sink, F64)
    H, D = cfg.n_heads, cfg.head_dim
    d = H * D
    for l, w in enumerate(layers):
        sh1, sc1, g1, sh2, sc2, g2 = _mod6(None if mod6_per_layer is None else mod6_per_layer[l], d)
        u = modulate(x, sh1, sc1, cfg.eps)
        k_src, v = sink_keys_values(u, w, cfg)
        caches[l].set_sink_source(k_src, v)
        caches[l].roll_sink(t_sink, cfg)
        q = _lin(cfg)(u, w["W_qkv"])[:, :d]
        if w.get("g_q") is not None:
            q = rmsnorm(q, w["g_q"], cfg.eps)
        q = rope3d(q.reshape(-1, H, D), t_sink, cfg.frame_h, cfg.frame_w, cfg.rope_axes, cfg.theta)
        o = attention(q, caches[l].sink[0], caches[l].sink[1], 1.0 / np.sqrt(D))
        x = x + g1 * _lin(cfg)(o.reshape(-1, d), w["W_o"])
        x = x + cross_attention(x, np.asarray(ctx, F64), w, cfg)
        u2 = modulate(x, sh2, sc2, cfg.eps)
        x = x + g2 * ffn(u2, w, cfg)
    return x


def denoise_stage(x, layers, caches, ctx, mod6_per_layer, dt, chunk_index, t0, cfg):
    """One timestep of the pipeline for one chunk: all blocks, then the Euler step x <- x + v*dt.

    The stack's output stands in for the velocity v (embedding and output head are outside the
    stage).  ``caches`` is one RollingKVCache per layer, all advanced once."""
    x_in = np.asarray(x, F64)
    h = x_in
    for l, w in enumerate(layers):
        m6 = None if mod6_per_layer is None else mod6_per_layer[l]
        h = dit_block(h, w, caches[l], ctx, m6, chunk_index, t0, cfg)
    return x_in + h * dt


def sample_chunk(x, layers, caches_per_step, ctx, mod6_per_step, dt, chunk_index, t0, cfg, t_sink=None):
    """Alg. 3, the inner loop over the T denoising steps of ONE block on one device: step s (the s-th to run, i.e. the
    paper's j = T - s) is a full stage forward with that step's own rolling caches ``caches_per_step[s]`` (one per
    layer) and that step's modulation, followed by the Euler update and that cache's pop/append.  All steps share the
    weights.  With ``t_sink`` given, every step first re-assigns its caches' sink index (Phi(sink))."""
    x = np.asarray(x, F64)
    for s, caches in enumerate(caches_per_step):
        if t_sink is not None:
            for c in caches:
                c.roll_sink(t_sink, cfg)
        m6 = None if mod6_per_step is None else mod6_per_step[s]
        x = denoise_stage(x, layers, caches, ctx, m6, dt, chunk_index, t0, cfg)
    return x


def full_sequence_stage(x_chunks, layers, sink_kv_per_layer, ctx_per_chunk, mod6_per_layer, dt, t0_of_chunk, cfg):
    """The same stack evaluated on ALL chunks at once with an explicit block-causal windowed mask.

    This is the non-streaming statement of Eq. 1 + the mask rule: a cross-check for the cache
    protocol, not something the HIP path mirrors.  Returns the list of per-chunk outputs."""
    H, D = cfg.n_heads, cfg.head_dim
    d = H * D
    n_chunks = len(x_chunks)
    nc = x_chunks[0].shape[0]
    x_in = np.concatenate([np.asarray(c, F64) for c in x_chunks], axis=0)
    h = x_in
    per_frame = cfg.frame_h * cfg.frame_w
    n = np.arange(n_chunks * nc)
    local = n % nc
    t = np.array([t0_of_chunk(i) for i in range(n_chunks)])[n // nc] + local // per_frame
    positions = (t, (local // cfg.frame_w) % cfg.frame_h, local % cfg.frame_w)
    for l, w in enumerate(layers):
        sh1, sc1, g1, sh2, sc2, g2 = _mod6(None if mod6_per_layer is None else mod6_per_layer[l], d)
        u = modulate(h, sh1, sc1, cfg.eps)
        q, k, v = qkv_for_cache(u, w, cfg, 0, positions)
        ks, vs = sink_kv_per_layer[l]
        mask = block_causal_mask(n_chunks, nc, ks.shape[0], cfg.window)
        o = attention(q, np.concatenate([np.asarray(ks, F64), k]), np.concatenate([np.asarray(vs, F64), v]),
                      1.0 / np.sqrt(D), mask=mask)
        h = h + g1 * _lin(cfg)(o.reshape(-1, d), w["W_o"])
        ca = [cross_attention(h[i * nc:(i + 1) * nc], np.asarray(ctx_per_chunk[i], F64), w, cfg)
              for i in range(n_chunks)]
        h = h + np.concatenate(ca, axis=0)
        u2 = modulate(h, sh2, sc2, cfg.eps)
        h = h + g2 * ffn(u2, w, cfg)
    out = x_in + h * dt
    return [out[i * nc:(i + 1) * nc] for i in range(n_chunks)]


# --------------------------------------------------------------------------------------------------
# Streaming causal 3-D convolution with a two-frame feature cache (Appendix C, "Streaming VAE Feature Caching")
# --------------------------------------------------------------------------------------------------
def causal_conv3d(x, w, bias=None):
    """Causal 3x3x3 convolution over a WHOLE frame sequence, channels last.

    x [T, H, W, Cin], w [Cout, 3, 3, 3, Cin] (taps ordered time, row, column), bias [Cout] or None.
    out[t, y, x, o] = bias[o] + sum_{dt,dy,dx,c} w[o, dt, dy, dx, c] * x[t + dt - 2, y + dy - 1, x + dx - 1, c],
    with zeros outside the frame (spatial padding 1) and before the first frame (temporal padding 2 on the past side
    only: frame t never sees a later frame).  Written as 27 shifted matrix products, nothing else."""
    x = np.asarray(x, F64)
    w = np.asarray(w, F64)
    T, H, W, Cin = x.shape
    Cout = w.shape[0]
    xp = np.zeros((T + 2, H + 2, W + 2, Cin), F64)
    xp[2:, 1:-1, 1:-1] = x
    out = np.zeros((T, H, W, Cout), F64)
    for dt in range(3):
        for dy in range(3):
            for dx in range(3):
                out += xp[dt:dt + T, dy:dy + H, dx:dx + W] @ w[:, dt, dy, dx, :].T
    if bias is not None:
        out += np.asarray(bias, F64)
    return out


def silu(x):
    x = np.asarray(x, F64)
    return x / (1.0 + np.exp(-x))


class CausalConvCache:
    """Feature cache of one causal convolution layer: the two most recent INPUT frames (zeros before the first frame)."""

    def __init__(self):
        self.frames = None      # [2, H, W, Cin]

    def step(self, x_chunk, w, bias=None):
        """Decode the next frames given only the cache: prepend the two cached frames as causal context, convolve,
        keep the outputs of the new frames, then retain the last two input frames for the next call."""
        x = np.asarray(x_chunk, F64)
        if self.frames is None:
            self.frames = np.zeros((2,) + x.shape[1:], F64)
        seq = np.concatenate([self.frames, x], axis=0)
        out = causal_conv3d(seq, w, bias)[2:]
        self.frames = seq[-2:]
        return out
