"""GPU parity at the benchmark's full sizes (14B-DiT shape), in the launch configuration bench.py times.

The CPU oracle cannot evaluate these sizes whole, so outputs are checked on SAMPLED rows the oracle computes one by one
(all heads / all channels of each sampled token), teacher-forced where a step depends on the whole chunk: the oracle is
handed the cache contents the GPU path holds (read back through lvx_kvcache_gather, itself gated bit-exactly by the
small-size tests) and the rows of that cache are in turn checked against the oracle's own K/V for the sampled tokens.
Inputs are drawn on the GPU (seeded) and read back, so both sides see the same bits.
"""
import math

import numpy as np
import pytest
import torch

import lvx_synth as S
from oracle import lvx_oracle as O
from test_gpu_parity import BF16_OUT_LINK, DEV, assert_close, assert_same_bf16, dims, make_cache

pytestmark = pytest.mark.gpu
P = S.PRESETS["attn14b"]


def sample_rows(n, k, seed):
    """Tile-boundary rows of the 256-query workgroup tile / 32-query wave tile, first / last rows, plus random ones."""
    fixed = [0, 31, 32, 255, 256, n - 257, n - 73, n - 72, n - 1]
    rnd = np.random.default_rng(seed).choice(n, size=k, replace=False).tolist()
    return np.array(sorted(set(fixed + rnd)))


def test_config2_attention_sampled_rows_all_warmup_key_counts(lvx):
    """40 heads x 128, 4680 queries; keys 6240 .. 24960 as the ring fills (6240 = 97.5 tiles: ragged last tile)."""
    d, sink_n, n = dims(P)
    H, D = P["n_heads"], P["head_dim"]
    cache = make_cache(lvx, P)
    sk = S.randn_bf16_device((sink_n, d), 2, 1.0, DEV)
    sv = S.randn_bf16_device((sink_n, d), 3, 1.0, DEV)
    lvx.lvx_kvcache_set_sink(cache, 0, sk, sv)
    ks, vs = [S.to_f64(sk).reshape(-1, H, D)], [S.to_f64(sv).reshape(-1, H, D)]
    q = S.randn_bf16_device((n, d), 1, 1.0, DEV)
    out = torch.empty_like(q)
    rows = sample_rows(n, 24, 5)
    q_rows = S.to_f64(q[torch.as_tensor(rows, device=DEV)]).reshape(-1, H, D)
    scale = 1.0 / math.sqrt(D)
    for i in range(P["window"] + 1):
        k = S.randn_bf16_device((n, d), 10 + i, 1.0, DEV)
        v = S.randn_bf16_device((n, d), 20 + i, 1.0, DEV)
        info = lvx.lvx_chunk_append_evict(cache, 0, k, v, i)
        lvx.lvx_chunk_attention(cache, 0, q, scale, out)
        torch.cuda.synchronize()
        ks.append(S.to_f64(k).reshape(-1, H, D))
        vs.append(S.to_f64(v).reshape(-1, H, D))
        assert info.key_count == sink_n + (i + 1) * n
        ref = O.attention(q_rows, np.concatenate(ks), np.concatenate(vs), scale)
        got = out[torch.as_tensor(rows, device=DEV)]
        assert_close(got, ref.reshape(len(rows), d), "config 2 attention, %d keys" % info.key_count)
    # whole-output property that holds at any size: each output row is a convex combination of V rows
    vmax = torch.stack([torch.as_tensor(np.concatenate(vs).reshape(-1, d).max(0)), torch.as_tensor(-np.concatenate(vs).reshape(-1, d).min(0))])
    o = out.float().cpu()
    assert bool((o <= vmax[0] + 1e-2).all()) and bool((-o <= vmax[1] + 1e-2).all())
    cache.close()


def test_config3_streaming_loop_100_steps(lvx):
    """100 chunk steps of rope/norm -> append/evict -> attention at the 14B shape.  Indices are checked against the
    list protocol at EVERY step; cache bits, rope parity and sampled-row attention parity at steps 0,1,3,4,5,50,99;
    the sink segment is bit-identical at the end."""
    d, sink_n, n = dims(P)
    H, D, W = P["n_heads"], P["head_dim"], P["window"]
    cache = make_cache(lvx, P)
    rope = lvx.rope_desc(H, D, P["rope_axes"], 10000.0, P["frame_h"], P["frame_w"])
    gains = torch.ones(d, dtype=torch.float32, device=DEV)
    # sink: normalised, rotated at t = 0
    sraw = S.randn_bf16_device((sink_n, 3 * d), 99, 1.0, DEV)
    lvx.lvx_rope3d(rope, sraw[:, :d], sraw[:, d:2 * d], gains, gains, sink_n, 0, sraw[:, :d], sraw[:, d:2 * d], ld_in=3 * d, ld_out=3 * d)
    sink_k, sink_v = sraw[:, d:2 * d].contiguous(), sraw[:, 2 * d:].contiguous()
    lvx.lvx_kvcache_set_sink(cache, 0, sink_k, sink_v)
    model = O.RollingKVCache(W)
    model.set_sink(np.zeros((1, 1, 1)), np.zeros((1, 1, 1)))
    scale = 1.0 / math.sqrt(D)
    rows = sample_rows(n, 8, 7)
    rows_t = torch.as_tensor(rows, device=DEV)
    cap = sink_n + (W + 1) * n
    out = torch.empty((n, d), dtype=torch.bfloat16, device=DEV)
    gk = torch.empty((cap, d), dtype=torch.bfloat16, device=DEV)
    gv = torch.empty((cap, d), dtype=torch.bfloat16, device=DEV)
    for i in range(100):
        qkv = S.randn_bf16_device((n, 3 * d), S.seed_of("cfg3", i), 1.0, DEV)
        check = i in (0, 1, 3, 4, 5, 50, 99)
        raw_rows = S.to_f64(qkv[rows_t]) if check else None
        t0 = 1 + 3 * i
        lvx.lvx_rope3d(rope, qkv[:, :d], qkv[:, d:2 * d], gains, gains, n, t0, qkv[:, :d], qkv[:, d:2 * d], ld_in=3 * d, ld_out=3 * d)
        visible = model.chunk_ids() + [i]
        info = lvx.lvx_chunk_append_evict(cache, 0, qkv[:, d:2 * d], qkv[:, 2 * d:], i, ld=3 * d)
        lvx.lvx_chunk_attention(cache, 0, qkv[:, :d], scale, out)
        st = lvx.lvx_kvcache_get_state(cache, 0)
        assert info.slot == i % (W + 1) and info.evicted_chunk == (i - (W + 1) if i > W else -1)
        assert sorted(c for c in st.slot_chunk[:st.n_slots] if c >= 0) == visible
        assert info.key_count == st.key_count == sink_n + len(visible) * n
        model.append(i, np.zeros((1, 1, 1)), np.zeros((1, 1, 1)))
        if not check:
            continue
        torch.cuda.synchronize()
        lvx.lvx_kvcache_gather(cache, 0, 0, cap, gk, gv)
        torch.cuda.synchronize()
        sl = slice(info.key_offset, info.key_offset + n)
        assert torch.equal(gk[sl].view(torch.int16), qkv[:, d:2 * d].view(torch.int16)), "K bits of step %d" % i
        assert torch.equal(gv[sl].view(torch.int16), qkv[:, 2 * d:].view(torch.int16)), "V bits of step %d" % i
        assert torch.equal(gk[:sink_n].view(torch.int16), sink_k.view(torch.int16)) and torch.equal(gv[:sink_n].view(torch.int16), sink_v.view(torch.int16))
        # rope + rmsnorm parity on the sampled tokens (positions of those tokens)
        pos = tuple(p[rows] for p in O.token_positions(n, t0, P["frame_h"], P["frame_w"]))
        for col, name in ((0, "q"), (d, "k")):
            ref = O.rope3d(O.rmsnorm(raw_rows[:, col:col + d], np.ones(d), 1e-6).reshape(-1, H, D), 0, P["frame_h"], P["frame_w"],
                           P["rope_axes"], 10000.0, positions=pos)
            assert_close(qkv[rows_t][:, col:col + d].contiguous(), ref.reshape(len(rows), d), "config 3 step %d rope+norm %s" % (i, name))
        # attention of the sampled queries against the cache the GPU holds
        nk = info.key_count
        ref = O.attention(S.to_f64(qkv[rows_t][:, :d].contiguous()).reshape(-1, H, D), S.to_f64(gk[:nk]).reshape(nk, H, D),
                          S.to_f64(gv[:nk]).reshape(nk, H, D), scale)
        assert_close(out[rows_t], ref.reshape(len(rows), d), "config 3 step %d attention (%d keys)" % (i, nk))
    cache.close()


def test_config4_dit_block_sampled_rows(lvx):
    """One full-size DiT block (weights N(0, 0.02)), cache pre-filled with 4 chunks: the block's output rows for sampled
    tokens against the oracle's row form, which is handed the keys the GPU cache holds; the cache rows the block wrote
    for those tokens are checked against the oracle's own K-hat / V.  All at the stated numbers: K-hat absolutely (unit RMS),
    V and the residual stream in units of their RMS (V = u W_v^T is not normalised, RMS 1.44).  The fp32-stream entry point
    carries the gate; the bf16 one must return its exact narrowing."""
    d, sink_n, n = dims(P)
    H, D, W = P["n_heads"], P["head_dim"], P["window"]
    w = S.block_weights(d, P["ffn"], 0, "cfg4", std=0.02, device=DEV, on_device_draw=True, row_pad=64)   # padded rows, as bench.py
    rope = lvx.rope_desc(H, D, P["rope_axes"], 10000.0, P["frame_h"], P["frame_w"])
    stage = lvx.StageHandle([w], rope, P["ffn"], ldw_d=d + 64, ldw_ffn=P["ffn"] + 64)
    cache, cache16 = make_cache(lvx, P), make_cache(lvx, P)
    for c in (cache, cache16):
        lvx.lvx_kvcache_set_sink(c, 0, S.randn_bf16_device((sink_n, d), 2, 1.0, DEV), S.randn_bf16_device((sink_n, d), 3, 1.0, DEV))
        for i in range(W):
            lvx.lvx_chunk_append_evict(c, 0, S.randn_bf16_device((n, d), 10 + i, 1.0, DEV), S.randn_bf16_device((n, d), 20 + i, 1.0, DEV), i)
    ws = torch.empty(lvx.lvx_workspace_bytes(stage, n, P["n_ctx"]), dtype=torch.uint8, device=DEV)
    x = S.randn_bf16_device((n, d), 31, 1.0, DEV)
    ctx = S.randn_bf16_device((P["n_ctx"], d), 32, 1.0, DEV)
    mod6 = S.randn_f32((6, d), 33, 0.1, device=DEV)
    mod6[2] += 1.0
    mod6[5] += 1.0
    rows = sample_rows(n, 6, 9)
    rows_t = torch.as_tensor(rows, device=DEV)
    x_rows = S.to_f64(x[rows_t])
    t0 = 1 + 3 * W
    x32 = x.float()
    lvx.lvx_dit_block_f32(stage, 0, cache, x32, ctx, mod6, W, t0, ws)
    lvx.lvx_dit_block(stage, 0, cache16, x, ctx, mod6, W, t0, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(x32).all())
    assert_same_bf16(x, x32.to(torch.bfloat16), "config 4: bf16 entry point = narrowing of the fp32 one")
    assert torch.equal(cache.storage, cache16.storage)
    cap = sink_n + (W + 1) * n
    gk = torch.empty((cap, d), dtype=torch.bfloat16, device=DEV)
    gv = torch.empty((cap, d), dtype=torch.bfloat16, device=DEV)
    lvx.lvx_kvcache_gather(cache, 0, 0, cap, gk, gv)
    torch.cuda.synchronize()
    cfg = O.StageConfig(H, D, P["frame_h"], P["frame_w"], P["chunk_frames"], W, P["sink_frames"], P["rope_axes"])
    pos = tuple(p[rows] for p in O.token_positions(n, t0, P["frame_h"], P["frame_w"]))
    ref, k_rows, v_rows = O.dit_block_rows(x_rows, pos, S.weights_to_f64(w), S.to_f64(gk).reshape(cap, H, D), S.to_f64(gv).reshape(cap, H, D),
                                           S.to_f64(ctx), S.to_f64(mod6), cfg)
    off = sink_n + (W % (W + 1)) * n
    assert_close(gk[off + rows_t], k_rows.reshape(len(rows), d), "config 4 cached K-hat rows")
    assert_close(gv[off + rows_t], v_rows.reshape(len(rows), d), "config 4 cached V rows", relative_to_rms=True)
    assert_close(x32[rows_t], ref, "config 4 block output rows, fp32 stream", relative_to_rms=True)
    assert_close(x[rows_t], ref, "config 4 block output rows, bf16 in/out", relative_to_rms=True, links=1.0 + BF16_OUT_LINK)
    cache.close()
    cache16.close()


@pytest.mark.parametrize("M,N,K,epi", [(4680, 15360, 5120, "store"), (4680, 13824, 5120, "gelu"), (4680, 5120, 5120, "resid_f32"),
                                       (4680, 5120, 13824, "resid_f32"), (544, 5120, 5120, "dual")])
def test_fullsize_linears_sampled_rows(lvx, M, N, K, epi):
    """The stage's GEMM shapes with the padded row strides bench.py uses (activation and weight rows of in_features + 64
    elements): QKV, FFN up (GELU), output / FFN down (fp32 gated residual), and the context's K | V pair."""
    a = S.randn_bf16_device((M, K + 64), S.seed_of("fl_a", M, N, K), 1.0, DEV)[:, :K]
    w = S.randn_bf16_device((N, K + 64), S.seed_of("fl_w", M, N, K), 0.02, DEV)[:, :K]
    rows = sample_rows(M, 10, 13) if M >= 4680 else np.array([0, 1, 127, 128, 255, 256, 511, 512, 543])
    rows_t = torch.as_tensor(rows, device=DEV)
    ref = O.linear(S.to_f64(a[rows_t]), S.to_f64(w))
    if epi == "store":
        c = torch.empty((M, N + 64), dtype=torch.bfloat16, device=DEV)[:, :N]
        lvx.lvx_linear(a, w, c, lvx.EPI_STORE)
        torch.cuda.synchronize()
        assert_close(c[rows_t], ref, "full-size linear %dx%dx%d" % (M, N, K), relative_to_rms=True)
        # the same projection as the block runs it: q | k columns in fp32, v columns in bf16
        d = N // 3
        c32 = torch.empty((M, 2 * d + 32), dtype=torch.float32, device=DEV)[:, :2 * d]
        cv = torch.empty((M, N + 64), dtype=torch.bfloat16, device=DEV)[:, 2 * d:N]
        lvx.lvx_linear_dual(a, w[:2 * d], w[2 * d:], c32, cv)
        torch.cuda.synchronize()
        e = np.abs(S.to_f64(c32[rows_t]) - ref[:, :2 * d])
        print("full-size QKV, fp32 q | k columns: max-abs %.3e" % e.max(), flush=True)
        assert e.max() <= 1e-5 * math.sqrt(K)
        assert torch.equal(cv, c[:, 2 * d:])
    elif epi == "gelu":
        c = torch.empty((M, N + 64), dtype=torch.bfloat16, device=DEV)[:, :N]
        lvx.lvx_linear(a, w, c, lvx.EPI_GELU_TANH)
        torch.cuda.synchronize()
        assert_close(c[rows_t], O.gelu_tanh(ref), "full-size linear + GELU %dx%dx%d" % (M, N, K))
    elif epi == "resid_f32":
        r = torch.randn((M, N), dtype=torch.float32, device=DEV, generator=torch.Generator(device=DEV).manual_seed(5)) * 3.0
        g = S.randn_f32((N,), 6, 0.2, 1.0, device=DEV)
        want = S.to_f64(r[rows_t]) + S.to_f64(g) * ref
        lvx.lvx_linear(a, w, r, lvx.EPI_RESID_GATE_F32, resid=r, gate=g)
        torch.cuda.synchronize()
        e = np.abs(S.to_f64(r[rows_t]) - want)
        print("full-size linear + fp32 gated residual %dx%dx%d: max-abs %.3e" % (M, N, K, e.max()), flush=True)
        assert e.max() <= 1e-5 * math.sqrt(K)
    else:
        w2 = S.randn_bf16_device((N, K + 64), S.seed_of("fl_w2", M, N, K), 0.02, DEV)[:, :K]       # same row stride as w
        c = torch.empty((M, 2 * N + 64), dtype=torch.bfloat16, device=DEV)
        lvx.lvx_linear_dual(a, w, w2, c[:, :N], c[:, N:2 * N])
        torch.cuda.synchronize()
        assert_close(c[rows_t][:, :N], ref, "context K projection (dual launch)", relative_to_rms=True)
        assert_close(c[rows_t][:, N:2 * N], O.linear(S.to_f64(a[rows_t]), S.to_f64(w2)), "context V projection (dual launch)",
                     relative_to_rms=True)


def test_config5_stage_40_layers_layerwise_and_bit_exact_chain(lvx):
    """Full-size stage in the benchmark's launch configuration (40 blocks, 28 GB of weights with padded rows, sink installed
    un-rotated and re-indexed before every forward), twelve chunks: warm-up key counts, then the full ring of 24960 keys with
    every slot overwritten twice (chunks 5..9 and 10, 11).  (a) lvx_denoise_stage must equal, bit for bit up to the last-place
    rounding of the Euler step, the chain widen -> 40 x lvx_dit_block_f32 -> Euler run on a second cache; (b) in that chain, at
    chunks 0, 5 and 11, layers 0, 20 and 39 are checked on sampled tokens against the oracle's row form, which is given the
    layer's fp32 input rows and the keys that layer's cache holds (teacher-forced, links = 1); (c) at chunks 5 and 11 the oracle
    also carries ITS OWN rows forward through layers 0..3 (only the visible keys are the GPU cache's): the drift of the chain,
    gated with one link per layer; (d) both caches end bit-identical."""
    d, sink_n, n = dims(P)
    H, D, W = P["n_heads"], P["head_dim"], P["window"]
    L = 40
    layers = [S.block_weights(d, P["ffn"], l, "cfg5", std=0.02, device=DEV, on_device_draw=True, row_pad=64) for l in range(L)]
    rope = lvx.rope_desc(H, D, P["rope_axes"], 10000.0, P["frame_h"], P["frame_w"])
    stage = lvx.StageHandle(layers, rope, P["ffn"], ldw_d=d + 64, ldw_ffn=P["ffn"] + 64)
    cache_a, cache_b = make_cache(lvx, P, L), make_cache(lvx, P, L)
    cache_a.attach_sink_source()
    cache_b.attach_sink_source()
    for l in range(L):
        sk = S.randn_bf16_device((sink_n, d), S.seed_of("cfg5_sk", l), 1.0, DEV)
        sv = S.randn_bf16_device((sink_n, d), S.seed_of("cfg5_sv", l), 1.0, DEV)
        lvx.lvx_kvcache_reset_sink(cache_a, l, sk, sv)
        lvx.lvx_kvcache_reset_sink(cache_b, l, sk, sv)
    ws = torch.empty(lvx.lvx_workspace_bytes(stage, n, P["n_ctx"]), dtype=torch.uint8, device=DEV)
    cfg = O.StageConfig(H, D, P["frame_h"], P["frame_w"], P["chunk_frames"], W, P["sink_frames"], P["rope_axes"])
    rows = sample_rows(n, 4, 11)
    rows_t = torch.as_tensor(rows, device=DEV)
    cap = sink_n + (W + 1) * n
    gk = torch.empty((cap, d), dtype=torch.bfloat16, device=DEV)
    gv = torch.empty((cap, d), dtype=torch.bfloat16, device=DEV)
    dt = -0.25
    DEPTH = 4
    for i in range(12):
        x = S.randn_bf16_device((n, d), S.seed_of("cfg5_x", i), 1.0, DEV)
        ctx = S.randn_bf16_device((P["n_ctx"], d), S.seed_of("cfg5_ctx", i), 1.0, DEV)
        t0 = 1 + 3 * i
        xa = x.clone()
        lvx.lvx_sink_rope_update(cache_a, rope, -1, t0 + 4)
        lvx.lvx_sink_rope_update(cache_b, rope, -1, t0 + 4)
        lvx.lvx_denoise_stage(stage, cache_a, xa, ctx, None, dt, i, t0, ws)
        h = x.float()
        carry = S.to_f64(x[rows_t]) if i in (5, 11) else None          # the oracle's own rows, carried from layer to layer
        pos = tuple(p[rows] for p in O.token_positions(n, t0, P["frame_h"], P["frame_w"]))
        nk = sink_n + min(i + 1, W + 1) * n
        for l in range(L):
            forced = l in (0, 20, 39) and i in (0, 5, 11)
            drift = carry is not None and l < DEPTH
            h_in_rows = S.to_f64(h[rows_t]) if forced else None
            lvx.lvx_dit_block_f32(stage, l, cache_b, h, ctx, None, i, t0, ws)
            if not (forced or drift):
                continue
            lvx.lvx_kvcache_gather(cache_b, l, 0, cap, gk, gv)
            torch.cuda.synchronize()
            w64 = S.weights_to_f64(layers[l])
            k64, v64 = S.to_f64(gk[:nk]).reshape(nk, H, D), S.to_f64(gv[:nk]).reshape(nk, H, D)
            if forced:
                ref, _, _ = O.dit_block_rows(h_in_rows, pos, w64, k64, v64, S.to_f64(ctx), None, cfg)
                assert_close(h[rows_t], ref, "config 5 chunk %d layer %d output rows" % (i, l), relative_to_rms=True)
            if drift:
                carry, _, _ = O.dit_block_rows(carry, pos, w64, k64, v64, S.to_f64(ctx), None, cfg)
                assert_close(h[rows_t], carry, "config 5 chunk %d layers 0..%d, oracle rows carried forward" % (i, l), relative_to_rms=True,
                             links=l + 1)
        torch.cuda.synchronize()
        want = (x.double() + dt * h.double()).to(torch.bfloat16)
        diff = (xa.view(torch.int16).int() - want.view(torch.int16).int()).abs()
        frac = float((diff != 0).float().mean())
        print("config 5 chunk %d: stage vs block chain, elements differing %.2e, max ulp %d" % (i, frac, int(diff.max())), flush=True)
        assert int(diff.max()) <= 1 and frac < 1e-3
        assert bool(torch.isfinite(xa.float()).all())
    assert torch.equal(cache_a.storage, cache_b.storage)
    cache_a.close()
    cache_b.close()


def test_fullsize_rolling_sink_update_all_layers_one_launch(lvx):
    """Phi(sink) at the benchmark's shape and launch: 4 layers x 1560 sink tokens x 5120 channels rotated in ONE launch
    (layer = -1) to an index near the 10 000 s rollout's; every layer's sink keys are compared with the oracle on sampled
    tokens, its values bit for bit; the chunk stored next to the sink (sharing the sink's last 64-key tile) is untouched and
    the attention over {sink, chunk} is checked on sampled rows."""
    d, sink_n, n = dims(P)
    H, D, W = P["n_heads"], P["head_dim"], P["window"]
    L = 4
    cfg = O.StageConfig(H, D, P["frame_h"], P["frame_w"], P["chunk_frames"], W, P["sink_frames"], P["rope_axes"])
    rope = lvx.rope_desc(H, D, P["rope_axes"], 10000.0, P["frame_h"], P["frame_w"])
    cache = make_cache(lvx, P, L)
    cache.attach_sink_source()
    srcs, vals = [], []
    ck = S.randn_bf16_device((n, d), 31, 1.0, DEV)
    cv = S.randn_bf16_device((n, d), 32, 1.0, DEV)
    for l in range(L):
        srcs.append(S.randn_bf16_device((sink_n, d), 40 + l, 1.0, DEV))
        vals.append(S.randn_bf16_device((sink_n, d), 50 + l, 1.0, DEV))
        lvx.lvx_kvcache_reset_sink(cache, l, srcs[l], vals[l])
        lvx.lvx_chunk_append_evict(cache, l, ck, cv, 0)
    t_sink = 39998
    lvx.lvx_sink_rope_update(cache, rope, -1, t_sink)
    toks = np.array(sorted(set([0, 1, 51, 52, 1535, 1536, 1559] + np.random.default_rng(3).choice(sink_n, 16, replace=False).tolist())))
    pos = tuple(a[toks] for a in O.token_positions(sink_n, t_sink, P["frame_h"], P["frame_w"]))
    q = S.randn_bf16_device((n, d), 33, 1.0, DEV)
    out = torch.empty_like(q)
    rows = sample_rows(n, 6, 9)
    for l in range(L):
        gk = torch.empty((sink_n + n, d), dtype=torch.bfloat16, device=DEV)
        gv = torch.empty_like(gk)
        lvx.lvx_kvcache_gather(cache, l, 0, sink_n + n, gk, gv)
        torch.cuda.synchronize()
        assert lvx.lvx_kvcache_get_sink_index(cache, l) == t_sink
        assert torch.equal(gv[:sink_n].view(torch.int16), vals[l].view(torch.int16))
        assert torch.equal(gk[sink_n:].view(torch.int16), ck.view(torch.int16)) and torch.equal(gv[sink_n:].view(torch.int16), cv.view(torch.int16))
        ti = torch.as_tensor(toks, device=DEV)
        ref = O.rope3d(S.to_f64(srcs[l][ti]).reshape(-1, H, D), 0, P["frame_h"], P["frame_w"], cfg.rope_axes, cfg.theta, pos)
        assert_close(gk[ti], ref.reshape(len(toks), d), "layer %d sink keys at t=%d (sampled tokens)" % (l, t_sink))
        if l in (0, L - 1):
            lvx.lvx_chunk_attention(cache, l, q, 1 / math.sqrt(D), out)
            torch.cuda.synchronize()
            k_all = S.to_f64(gk).reshape(-1, H, D)        # cache contents as the GPU holds them (gated above / bit-exact)
            v_all = S.to_f64(gv).reshape(-1, H, D)
            ri = torch.as_tensor(rows, device=DEV)
            want = O.attention(S.to_f64(q[ri]).reshape(-1, H, D), k_all, v_all, 1 / math.sqrt(D))
            assert_close(out[ri], want.reshape(len(rows), d), "layer %d attention over {rolled sink, chunk 0}" % l)
    cache.close()


def test_fullsize_fp8_qkv_linear_sampled_rows(lvx):
    """The FP8 QKV projection at the benchmark's shape (4680 x 15360 x 5120, padded row strides as in bench.py): codes of the
    activation and of a slice of the weight bit for bit, the scales exactly, the output on sampled rows against the oracle's
    quantise-dequantise product."""
    M, N, K = 4680, 15360, 5120
    a = S.randn_bf16_device((M, K + 64), 61, 1.0, DEV)[:, :K]
    w = S.randn_bf16_device((N, K + 64), 62, 0.02, DEV)[:, :K]
    aq, sa = lvx.lvx_fp8_quantize(a, row_pad=128)
    wq, sw = lvx.lvx_fp8_quantize(w, row_pad=128)
    c = torch.empty((M, N + 64), dtype=torch.bfloat16, device=DEV)[:, :N]
    lvx.lvx_linear_fp8(aq, sa, wq, sw, c)
    torch.cuda.synchronize()
    a_grid, s_a = O.fp8_quantize_per_tensor(S.to_f64(a))
    w_grid, s_w = O.fp8_quantize_per_tensor(S.to_f64(w))
    assert float(sa.item()) == np.float32(s_a) and float(sw.item()) == np.float32(s_w)
    from test_gpu_fp8 import e4m3_decode
    np.testing.assert_array_equal(e4m3_decode(aq.cpu().numpy()), a_grid)
    np.testing.assert_array_equal(e4m3_decode(wq[:2048].cpu().numpy()), w_grid[:2048])
    rows = sample_rows(M, 10, 11)
    ref = (a_grid[rows] @ w_grid.T) * (s_a * s_w)
    assert_close(c[torch.as_tensor(rows, device=DEV)], ref, "fp8 QKV linear at 4680x15360x5120 (sampled rows)")
