"""CPU-only checks of the C-ABI boundary: symbols, ring arithmetic against the list protocol, error paths.
No kernel is launched here (every error below is raised by host-side argument checks)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2512_04677_amd as lvx
from oracle import lvx_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = lvx.load()
    header = open(os.path.join(ROOT, "include", "lvx.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lvx_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 18
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(lvx.SIGNATURES), declared ^ set(lvx.SIGNATURES)
    assert "gfx950" in lvx.version()


def desc14b(**kw):
    d = dict(n_layers=40, n_heads=40, head_dim=128, frame_h=30, frame_w=52, chunk_frames=3, window_chunks=4, sink_frames=1)
    d.update(kw)
    return lvx.cache_desc(**d)


def test_cache_bytes_14b_shape():
    # 24960 keys x 40 heads x 128 x bf16 x (K+V) x 40 layers = 20.4 GB; 24960 is a multiple of the 64-key tile
    assert lvx.lvx_kvcache_bytes(desc14b()) == 2 * 2 * 40 * 40 * 24960 * 128
    # tiny config: 24 + 3*48 = 168 keys, padded to 192
    assert lvx.lvx_kvcache_bytes(desc14b(n_layers=1, n_heads=2, head_dim=64, frame_h=4, frame_w=6, chunk_frames=2,
                                         window_chunks=2)) == 2 * 2 * 2 * 192 * 64


@pytest.mark.parametrize("window", [1, 2, 4])
def test_ring_arithmetic_matches_list_protocol(window):
    """The ring (slot = i mod (w+1), written before the attention) must expose exactly the chunks the list protocol of
    Alg. 3 (attend to the cache + self, then pop-if-full and append) exposes, for 120 steps including warm-up."""
    desc = desc14b(window_chunks=window)
    sink, chunk = 1560, 4680
    model = O.RollingKVCache(window)
    model.set_sink(np.zeros((1, 1, 1)), np.zeros((1, 1, 1)))
    slots = {}
    for i in range(120):
        info = lvx.lvx_ring_slot(desc, i)
        assert info.slot == i % (window + 1)
        assert info.key_offset == sink + info.slot * chunk
        if info.slot in slots:
            assert info.evicted_chunk == slots[info.slot]
        else:
            assert info.evicted_chunk == -1
        slots[info.slot] = i
        visible_model = model.chunk_ids() + [i]            # what the forward of chunk i sees
        assert sorted(slots.values()) == visible_model
        assert info.n_valid_chunks == len(visible_model)
        assert info.key_count == sink + chunk * len(visible_model)
        # the chunk the ring overwrites was already gone from the list before this forward
        assert info.evicted_chunk not in visible_model
        model.append(i, np.zeros((1, 1, 1)), np.zeros((1, 1, 1)))
    assert info.key_count == sink + (window + 1) * chunk


def test_key_counts_during_warm_up():
    d = desc14b()
    assert [lvx.lvx_ring_slot(d, i).key_count for i in range(6)] == [6240, 10920, 15600, 20280, 24960, 24960]


def status_of(fn, *a, **k):
    with pytest.raises(lvx.LvxError) as e:
        fn(*a, **k)
    return e.value.status


def test_error_paths_without_a_device():
    lib = lvx.load()
    d = desc14b()
    info = lvx.SlotInfo()
    assert lib.lvx_ring_slot(None, 0, C.byref(info)) == 1
    assert lib.lvx_ring_slot(C.byref(d), 0, None) == 1
    assert lib.lvx_ring_slot(C.byref(d), -1, C.byref(info)) == 1
    assert b"negative" in lib.lvx_last_error()
    assert status_of(lvx.lvx_ring_slot, desc14b(head_dim=96), 0) == 4
    assert status_of(lvx.lvx_ring_slot, desc14b(window_chunks=16), 0) == 4
    assert status_of(lvx.lvx_ring_slot, desc14b(n_heads=0), 0) == 2
    assert lvx.lvx_kvcache_bytes(desc14b(head_dim=96)) == 0
    h = C.c_void_p()
    need = lvx.lvx_kvcache_bytes(d)
    assert lib.lvx_kvcache_init(C.byref(d), None, need, None, C.byref(h)) == 1
    assert lib.lvx_kvcache_init(C.byref(d), C.c_void_p(4096 + 16), need, None, C.byref(h)) == 1      # misaligned
    assert lib.lvx_kvcache_init(C.byref(d), C.c_void_p(4096), need - 1, None, C.byref(h)) == 2        # too small
    assert lib.lvx_kvcache_init(C.byref(d), C.c_void_p(4096), need, None, None) == 1
    assert lib.lvx_kvcache_destroy(None) == 1
    assert lib.lvx_chunk_append_evict(None, 0, C.c_void_p(4096), C.c_void_p(4096), 5120, 0, None, None) == 1
    assert lib.lvx_chunk_attention(None, 0, C.c_void_p(4096), 5120, 10, 1.0, C.c_void_p(4096), 5120, None) == 1
    assert lib.lvx_chunk_attention_prescaled(None, 0, C.c_void_p(4096), 5120, 10, C.c_void_p(4096), 5120, None) == 1
    # linear: shape checks come before any launch
    p = C.c_void_p(4096)
    assert lib.lvx_linear(p, 100, p, 100, p, 64, 4, 64, 100, 0, None, 0, None, None) == 2      # K % 64
    assert lib.lvx_linear(p, 128, p, 128, p, 64, 4, 60, 128, 0, None, 0, None, None) == 2      # N % 8
    assert lib.lvx_linear(p, 64, p, 128, p, 64, 4, 64, 128, 0, None, 0, None, None) == 2       # lda < K
    assert lib.lvx_linear(p, 128, p, 128, p, 64, 4, 64, 128, 7, None, 0, None, None) == 1      # epilogue enum
    assert lib.lvx_linear(p, 128, p, 128, p, 64, 4, 64, 128, 2, None, 0, None, None) == 1      # residual missing
    assert lib.lvx_linear(C.c_void_p(4100), 128, p, 128, p, 64, 4, 64, 128, 0, None, 0, None, None) == 1
    assert lib.lvx_linear(None, 128, p, 128, p, 64, 4, 64, 128, 0, None, 0, None, None) == 1
    # two projections in one launch
    assert lib.lvx_linear_dual(p, 128, p, p, 128, p, 64, 1, p, 64, 4, 64, 64, 100, None) == 2    # K % 64
    assert lib.lvx_linear_dual(p, 128, p, p, 128, p, 64, 1, p, 64, 4, 64, 60, 128, None) == 2    # N2 % 8
    assert lib.lvx_linear_dual(p, 128, p, p, 128, p, 56, 0, p, 64, 4, 64, 64, 128, None) == 2    # ldc1 < N1
    assert lib.lvx_linear_dual(p, 128, p, None, 128, p, 64, 0, p, 64, 4, 64, 64, 128, None) == 1
    assert lib.lvx_linear_dual(p, 128, p, p, 128, C.c_void_p(4104), 64, 1, p, 64, 4, 64, 64, 128, None) == 1
    # rope descriptor checks
    r = lvx.rope_desc(40, 128, (44, 42, 40), 1e4, 30, 52)
    assert lib.lvx_rope3d(C.byref(r), p, p, 5120, None, None, 4, 0, p, p, 5120, None) == 2
    r = lvx.rope_desc(40, 128, (44, 42, 42), 1e4, 30, 52)
    assert lib.lvx_rope3d(C.byref(r), p, p, 5000, None, None, 4, 0, p, p, 5120, None) == 2       # ld < d
    assert lib.lvx_rope3d(C.byref(r), None, None, 5120, None, None, 4, 0, None, None, 5120, None) == 1
    assert lib.lvx_rope3d(C.byref(r), p, None, 5120, None, None, 4, 0, None, None, 5120, None) == 1
    assert lib.lvx_rope3d_f32in(C.byref(r), p, p, 5000, None, None, 4, 0, p, p, 5120, None) == 2
    assert lib.lvx_rope3d_f32in(C.byref(r), p, None, 10240, None, None, 4, 0, None, p, 5120, None) == 1
    assert lib.lvx_layernorm_modulate(p, 5120, None, None, 1e-6, 4, 5124, p, 5120, None) == 2
    # stage / workspace
    blocks = (lvx.BlockWeights * 1)()
    st = lvx.Stage(1, 13824, 0, 0, r, C.cast(blocks, C.POINTER(lvx.BlockWeights)))
    ws = lib.lvx_workspace_bytes(C.byref(st), 4680, 544)
    assert ws >= 4680 * 5120 * 2 * 2 + 4680 * 15360 * 2
    st_bad = lvx.Stage(1, 13824 + 8, 0, 0, r, C.cast(blocks, C.POINTER(lvx.BlockWeights)))
    st_bad2 = lvx.Stage(1, 13824, 5120 + 4, 0, r, C.cast(blocks, C.POINTER(lvx.BlockWeights)))
    assert lib.lvx_workspace_bytes(C.byref(st_bad2), 4680, 544) == 0
    assert lib.lvx_workspace_bytes(C.byref(st_bad), 4680, 544) == 0
    assert lib.lvx_dit_block(C.byref(st), 0, None, p, 4680, p, 544, None, 0, 1, p, ws, None) == 1
    assert lib.lvx_denoise_stage(None, None, p, 4680, p, 544, None, -0.25, 0, 1, p, ws, None) == 1


def test_sink_management_host_checks():
    lib = lvx.load()
    d = desc14b()
    # un-rotated sink keys of all layers: 40 layers x 1560 tokens x 5120 channels x bf16 = 639 MB
    assert lvx.load().lvx_sink_source_bytes(C.byref(d)) == 40 * 1560 * 5120 * 4      # kept in fp32
    assert lvx.load().lvx_sink_source_bytes(C.byref(desc14b(head_dim=96))) == 0
    p = C.c_void_p(4096)
    r = lvx.rope_desc(40, 128, (44, 42, 42), 1e4, 30, 52)
    out = C.c_int32()
    assert lib.lvx_kvcache_attach_sink_source(None, p, 1 << 30) == 1
    assert lib.lvx_kvcache_reset_sink(None, 0, p, p, 5120, None) == 1
    assert lib.lvx_sink_rope_update(None, C.byref(r), 0, 1, None) == 1
    assert lib.lvx_kvcache_get_sink_index(None, 0, C.byref(out)) == 1
    assert lib.lvx_kvcache_gather_sink_source(None, 0, p, 5120, None) == 1
    blocks = (lvx.BlockWeights * 1)()
    st = lvx.Stage(1, 13824, 0, 0, r, C.cast(blocks, C.POINTER(lvx.BlockWeights)))
    assert lib.lvx_sink_prefill(C.byref(st), None, p, p, 544, None, 1, None, p, 1 << 30, None) == 1
    assert b"NULL" in lib.lvx_last_error()


def test_fp8_entry_points_host_checks():
    lib = lvx.load()
    p = C.c_void_p(4096)
    f = C.c_void_p(8192)
    assert lib.lvx_fp8_quantize(None, 64, 4, 64, p, 64, p, f, None) == 1
    assert lib.lvx_fp8_quantize(p, 64, 4, 60, p, 64, p, f, None) == 2            # cols % 16
    assert lib.lvx_fp8_quantize(p, 64, 4, 64, p, 72, p, f, None) == 2            # ldq % 16
    assert lib.lvx_fp8_quantize(p, 32, 4, 64, p, 64, p, f, None) == 2            # ld < cols
    assert lib.lvx_fp8_quantize(p, 64, 4, 64, p, 64, C.c_void_p(4100), f, None) == 1
    # the allocation-free form: same checks, plus its stated maximum, all before anything touches a device
    assert lib.lvx_fp8_quantize_static(None, 64, 4, 64, p, 64, f, None) == 1
    assert lib.lvx_fp8_quantize_static(p, 64, 4, 60, p, 64, f, None) == 2
    assert lib.lvx_fp8_quantize_static(p, 1 << 20, 1 << 12, 1 << 20, p, 1 << 20, f, None) == 2          # 2^32 elements > 2^31
    assert b"exceeds" in lib.lvx_last_error()
    assert lib.lvx_linear_fp8(p, 128, f, p, 128, f, p, 64, 4, 64, 192, 0, None, 0, None, None) == 2    # K % 128
    assert lib.lvx_linear_fp8(p, 128, f, p, 128, f, p, 64, 4, 60, 128, 0, None, 0, None, None) == 2    # N % 8
    assert lib.lvx_linear_fp8(p, 120, f, p, 128, f, p, 64, 4, 64, 128, 0, None, 0, None, None) == 2    # lda
    assert lib.lvx_linear_fp8(p, 128, None, p, 128, f, p, 64, 4, 64, 128, 0, None, 0, None, None) == 1 # scale missing
    assert lib.lvx_linear_fp8(p, 128, f, p, 128, f, p, 64, 4, 64, 128, 3, None, 0, None, None) == 1    # residual missing
    # an FP8 stage needs d_model and d_ffn in multiples of 128 and 16-byte multiples as row strides
    r = lvx.rope_desc(40, 128, (44, 42, 42), 1e4, 30, 52)
    blocks = (lvx.BlockWeights * 1)()
    b8 = (lvx.BlockWeightsFp8 * 1)()
    cast8 = C.cast(b8, C.POINTER(lvx.BlockWeightsFp8))
    castb = C.cast(blocks, C.POINTER(lvx.BlockWeights))
    ok = lvx.Stage(1, 13824, 0, 0, r, castb, cast8, 5120 + 128, 13824 + 128)
    plain = lvx.Stage(1, 13824, 0, 0, r, castb)
    # an FP8 stage holds, beside the bf16 activations and the fp32 stream, the quantised input of its widest linear
    assert lib.lvx_workspace_bytes(C.byref(ok), 4680, 544) >= 4680 * (5120 * 2 + 15360 * 2 + 5120 * 4 + 13824)
    # a bf16 stage: the fp32 copy of the projection's k columns instead
    assert lib.lvx_workspace_bytes(C.byref(plain), 4680, 544) >= 4680 * (5120 * 2 + 15360 * 2 + 5120 * 4 + 5120 * 4)
    assert lib.lvx_workspace_bytes(C.byref(lvx.Stage(1, 13824 + 64, 0, 0, r, castb, cast8, 0, 0)), 4680, 544) == 0
    assert lib.lvx_workspace_bytes(C.byref(lvx.Stage(1, 13824, 0, 0, r, castb, cast8, 5120 + 8, 0)), 4680, 544) == 0


def test_causal_conv_host_checks():
    lib = lvx.load()
    d = lvx.ConvDesc(384, 384, 100, 180, 4)
    assert lib.lvx_causal_conv_state_bytes(C.byref(d)) == 6 * 102 * 182 * 384 * 2
    assert lib.lvx_causal_conv_state_bytes(C.byref(lvx.ConvDesc(96, 96, 100, 180, 4))) == 0          # c_in % 64
    assert lib.lvx_causal_conv_state_bytes(C.byref(lvx.ConvDesc(384, 380, 100, 180, 4))) == 0        # c_out % 8
    assert lib.lvx_causal_conv_state_bytes(C.byref(lvx.ConvDesc(384, 384, 400, 720, 20))) == 0       # volume beyond 4 GiB
    h = C.c_void_p()
    need = lib.lvx_causal_conv_state_bytes(C.byref(d))
    assert lib.lvx_causal_conv_init(C.byref(d), None, need, None, C.byref(h)) == 1
    assert lib.lvx_causal_conv_init(C.byref(d), C.c_void_p(4096), need - 1, None, C.byref(h)) == 2
    assert lib.lvx_causal_conv_init(C.byref(d), C.c_void_p(4096 + 16), need, None, C.byref(h)) == 1
    assert lib.lvx_causal_conv_step(None, C.c_void_p(4096), 1, C.c_void_p(4096), 27 * 384, None, 0, C.c_void_p(4096), None) == 1
    assert lib.lvx_causal_conv_reset(None, None) == 1 and lib.lvx_causal_conv_destroy(None) == 1
