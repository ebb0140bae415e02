"""Python binding of liblvx.so (the gfx950 HIP path).  Argument marshalling only: every step runs in the library.

PyTorch supplies device memory and the current HIP stream, nothing else.  There is no CPU fallback: `load()` raises
if the library has not been built (`python -m paper_2512_04677_amd.build`), and every call raises `LvxError` on a
non-zero status.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblvx.so")
_lib = None

LVX_MAX_SLOTS = 16
EPI_STORE, EPI_GELU_TANH, EPI_RESID_GATE, EPI_RESID_GATE_F32, EPI_BIAS, EPI_BIAS_SILU, EPI_STORE_F32 = 0, 1, 2, 3, 4, 5, 6
STATUS_NAMES = {0: "LVX_OK", 1: "LVX_ERR_INVALID_ARG", 2: "LVX_ERR_SHAPE", 3: "LVX_ERR_STATE", 4: "LVX_ERR_UNSUPPORTED",
                5: "LVX_ERR_HIP"}


class LvxError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, status), message))
        self.status = status


class CacheDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "n_heads", "head_dim", "frame_h", "frame_w", "chunk_frames",
                                         "window_chunks", "sink_frames")]


class SlotInfo(C.Structure):
    _fields_ = [("slot", C.c_int32), ("evicted_chunk", C.c_int64), ("n_valid_chunks", C.c_int32),
                ("key_offset", C.c_int32), ("key_count", C.c_int32)]


class RingState(C.Structure):
    _fields_ = [("last_chunk", C.c_int64), ("sink_set", C.c_int32), ("n_valid_chunks", C.c_int32),
                ("key_count", C.c_int32), ("n_slots", C.c_int32), ("slot_chunk", C.c_int64 * LVX_MAX_SLOTS)]


class RopeDesc(C.Structure):
    _fields_ = [("n_heads", C.c_int32), ("head_dim", C.c_int32), ("axes", C.c_int32 * 3), ("theta", C.c_float),
                ("frame_h", C.c_int32), ("frame_w", C.c_int32), ("eps", C.c_float), ("apply_rope", C.c_int32)]


class BlockWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("W_qkv", "W_o", "Wc_q", "Wc_k", "Wc_v", "Wc_o", "W_1", "W_2",
                                          "g_q", "g_k", "gc_q", "gc_k")]


class ConvDesc(C.Structure):
    _fields_ = [("c_in", C.c_int32), ("c_out", C.c_int32), ("height", C.c_int32), ("width", C.c_int32), ("max_frames", C.c_int32)]


class BlockWeightsFp8(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("W_qkv", "W_o", "Wc_q", "Wc_k", "Wc_v", "Wc_o", "W_1", "W_2", "scales")]


FP8_WEIGHT_ORDER = ("W_qkv", "W_o", "Wc_q", "Wc_k", "Wc_v", "Wc_o", "W_1", "W_2")


class Stage(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_ffn", C.c_int32), ("ldw_d", C.c_int32), ("ldw_ffn", C.c_int32), ("rope", RopeDesc),
                ("blocks", C.POINTER(BlockWeights)), ("blocks_fp8", C.POINTER(BlockWeightsFp8)), ("ldw8_d", C.c_int32),
                ("ldw8_ffn", C.c_int32)]


# name -> (restype, argtypes); the list the header declares
_vp, _i32, _i64, _f32, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
SIGNATURES = {
    "lvx_last_error": (C.c_char_p, []),
    "lvx_version": (C.c_char_p, []),
    "lvx_kvcache_bytes": (_sz, [C.POINTER(CacheDesc)]),
    "lvx_ring_slot": (C.c_int, [C.POINTER(CacheDesc), _i64, C.POINTER(SlotInfo)]),
    "lvx_kvcache_init": (C.c_int, [C.POINTER(CacheDesc), _vp, _sz, _vp, C.POINTER(_vp)]),
    "lvx_kvcache_destroy": (C.c_int, [_vp]),
    "lvx_kvcache_set_sink": (C.c_int, [_vp, _i32, _vp, _vp, _i64, _vp]),
    "lvx_chunk_append_evict": (C.c_int, [_vp, _i32, _vp, _vp, _i64, _i64, C.POINTER(SlotInfo), _vp]),
    "lvx_kvcache_get_state": (C.c_int, [_vp, _i32, C.POINTER(RingState)]),
    "lvx_kvcache_set_state": (C.c_int, [_vp, _i32, C.POINTER(RingState)]),
    "lvx_kvcache_gather": (C.c_int, [_vp, _i32, _i32, _i32, _vp, _vp, _i64, _vp]),
    "lvx_rope3d": (C.c_int, [C.POINTER(RopeDesc), _vp, _vp, _i64, _vp, _vp, _i32, _i32, _vp, _vp, _i64, _vp]),
    "lvx_rope3d_f32in": (C.c_int, [C.POINTER(RopeDesc), _vp, _vp, _i64, _vp, _vp, _i32, _i32, _vp, _vp, _i64, _vp]),
    "lvx_chunk_attention": (C.c_int, [_vp, _i32, _vp, _i64, _i32, _f32, _vp, _i64, _vp]),
    "lvx_chunk_attention_prescaled": (C.c_int, [_vp, _i32, _vp, _i64, _i32, _vp, _i64, _vp]),
    "lvx_linear": (C.c_int, [_vp, _i64, _vp, _i64, _vp, _i64, _i32, _i32, _i32, C.c_int, _vp, _i64, _vp, _vp]),
    "lvx_linear_dual": (C.c_int, [_vp, _i64, _vp, _vp, _i64, _vp, _i64, _i32, _vp, _i64, _i32, _i32, _i32, _i32, _vp]),
    "lvx_fp8_quantize": (C.c_int, [_vp, _i64, _i32, _i32, _vp, _i64, _vp, _vp, _vp]),
    "lvx_fp8_quantize_static": (C.c_int, [_vp, _i64, _i32, _i32, _vp, _i64, _vp, _vp]),
    "lvx_linear_fp8": (C.c_int, [_vp, _i64, _vp, _vp, _i64, _vp, _vp, _i64, _i32, _i32, _i32, C.c_int, _vp, _i64, _vp, _vp]),
    "lvx_layernorm_modulate": (C.c_int, [_vp, _i64, _vp, _vp, _f32, _i32, _i32, _vp, _i64, _vp]),
    "lvx_workspace_bytes": (_sz, [C.POINTER(Stage), _i32, _i32]),
    "lvx_context_kv": (C.c_int, [C.POINTER(Stage), _i32, _i32, _vp, _i32, _vp, _vp, _i64, _vp, _sz, _vp]),
    "lvx_dit_block": (C.c_int, [C.POINTER(Stage), _i32, _vp, _vp, _i32, _vp, _i32, _vp, _i64, _i32, _vp, _sz, _vp]),
    "lvx_dit_block_f32": (C.c_int, [C.POINTER(Stage), _i32, _vp, _vp, _i32, _vp, _i32, _vp, _i64, _i32, _vp, _sz, _vp]),
    "lvx_denoise_stage": (C.c_int, [C.POINTER(Stage), _vp, _vp, _i32, _vp, _i32, _vp, _f32, _i64, _i32, _vp, _sz, _vp]),
    "lvx_sink_source_bytes": (_sz, [C.POINTER(CacheDesc)]),
    "lvx_kvcache_attach_sink_source": (C.c_int, [_vp, _vp, _sz]),
    "lvx_kvcache_reset_sink": (C.c_int, [_vp, _i32, _vp, _vp, _i64, _vp]),
    "lvx_sink_rope_update": (C.c_int, [_vp, C.POINTER(RopeDesc), _i32, _i32, _vp]),
    "lvx_kvcache_get_sink_index": (C.c_int, [_vp, _i32, C.POINTER(C.c_int32)]),
    "lvx_kvcache_set_sink_index": (C.c_int, [_vp, _i32, _i32]),
    "lvx_kvcache_gather_sink_source": (C.c_int, [_vp, _i32, _vp, _i64, _vp]),
    "lvx_sink_prefill": (C.c_int, [C.POINTER(Stage), _vp, _vp, _vp, _i32, _vp, _i32, _vp, _vp, _sz, _vp]),
    "lvx_sample_chunk": (C.c_int, [C.POINTER(Stage), C.POINTER(_vp), _i32, _vp, _i32, _vp, _i32, _vp, _f32, _i64, _i32, _i32, _vp, _sz,
                                   _vp]),
    "lvx_causal_conv_state_bytes": (_sz, [C.POINTER(ConvDesc)]),
    "lvx_causal_conv_init": (C.c_int, [C.POINTER(ConvDesc), _vp, _sz, _vp, C.POINTER(_vp)]),
    "lvx_causal_conv_destroy": (C.c_int, [_vp]),
    "lvx_causal_conv_reset": (C.c_int, [_vp, _vp]),
    "lvx_causal_conv_step": (C.c_int, [_vp, _vp, _i32, _vp, _i64, _vp, _i32, _vp, _vp]),
    "lvx_profile_set": (C.c_int, [_i32]),
    "lvx_profile_read": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
}
PROF_KINDS = ["attn_self", "gemm_qkv", "gemm_o", "gemm_cross", "gemm_ffn1", "gemm_ffn2", "attn_cross", "rope_norm", "append",
              "layernorm", "fp8_quant", "ctx_kv", "cross_qnorm", "misc", "sink_rope"]


def load():
    """Loads liblvx.so; raises if it is missing (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("liblvx.so is not built: run `python -m paper_2512_04677_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise LvxError(status, load().lvx_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def version():
    return load().lvx_version().decode()


def cache_desc(n_layers, n_heads, head_dim, frame_h, frame_w, chunk_frames, window_chunks, sink_frames):
    return CacheDesc(n_layers, n_heads, head_dim, frame_h, frame_w, chunk_frames, window_chunks, sink_frames)


def rope_desc(n_heads, head_dim, axes, theta, frame_h, frame_w, eps=1e-6, apply_rope=1):
    return RopeDesc(n_heads, head_dim, (C.c_int32 * 3)(*axes), theta, frame_h, frame_w, eps, apply_rope)


def lvx_kvcache_bytes(desc):
    return load().lvx_kvcache_bytes(C.byref(desc))


def lvx_ring_slot(desc, chunk_index):
    info = SlotInfo()
    _check(load().lvx_ring_slot(C.byref(desc), chunk_index, C.byref(info)))
    return info


class KVCache:
    """Owns the torch storage tensor and the library handle of one rolling cache."""

    def __init__(self, desc, device="cuda:0"):
        import torch
        self.desc = desc
        nbytes = lvx_kvcache_bytes(desc)
        if nbytes == 0:
            raise LvxError(2, load().lvx_last_error().decode())
        self.storage = torch.empty(nbytes, dtype=torch.uint8, device=device)
        h = C.c_void_p()
        _check(load().lvx_kvcache_init(C.byref(desc), _ptr(self.storage), nbytes, _stream(), C.byref(h)))
        self.handle = h
        self.sink_source = None

    def attach_sink_source(self):
        """Allocates and hands over the storage for the un-rotated sink keys (Rolling RoPE / sink swap)."""
        import torch
        nbytes = load().lvx_sink_source_bytes(C.byref(self.desc))
        self.sink_source = torch.empty(nbytes, dtype=torch.uint8, device=self.storage.device)
        _check(load().lvx_kvcache_attach_sink_source(self.handle, _ptr(self.sink_source), nbytes))

    def close(self):
        if self.handle is not None:
            load().lvx_kvcache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def lvx_kvcache_set_sink(cache, layer, k, v, ld=None):
    _check(load().lvx_kvcache_set_sink(cache.handle, layer, _ptr(k), _ptr(v), ld if ld is not None else k.stride(0), _stream()))


def lvx_kvcache_reset_sink(cache, layer, k_src, v, ld=None):
    _check(load().lvx_kvcache_reset_sink(cache.handle, layer, _ptr(k_src), _ptr(v), ld if ld is not None else k_src.stride(0), _stream()))


def lvx_sink_rope_update(cache, rope, layer, t_sink):
    _check(load().lvx_sink_rope_update(cache.handle, C.byref(rope), layer, t_sink, _stream()))


def lvx_kvcache_get_sink_index(cache, layer):
    out = C.c_int32()
    _check(load().lvx_kvcache_get_sink_index(cache.handle, layer, C.byref(out)))
    return out.value


def lvx_kvcache_set_sink_index(cache, layer, t_sink):
    _check(load().lvx_kvcache_set_sink_index(cache.handle, layer, t_sink))


def lvx_kvcache_gather_sink_source(cache, layer, k_src_out):
    _check(load().lvx_kvcache_gather_sink_source(cache.handle, layer, _ptr(k_src_out), k_src_out.stride(0), _stream()))


def lvx_chunk_append_evict(cache, layer, k, v, chunk_index, ld=None):
    info = SlotInfo()
    _check(load().lvx_chunk_append_evict(cache.handle, layer, _ptr(k), _ptr(v), ld if ld is not None else k.stride(0),
                                         chunk_index, C.byref(info), _stream()))
    return info


def lvx_kvcache_get_state(cache, layer):
    s = RingState()
    _check(load().lvx_kvcache_get_state(cache.handle, layer, C.byref(s)))
    return s


def lvx_kvcache_set_state(cache, layer, state):
    _check(load().lvx_kvcache_set_state(cache.handle, layer, C.byref(state)))


def lvx_kvcache_gather(cache, layer, first_key, n_keys, k_out, v_out):
    _check(load().lvx_kvcache_gather(cache.handle, layer, first_key, n_keys, _ptr(k_out), _ptr(v_out), k_out.stride(0), _stream()))


def lvx_rope3d(desc, q_in, k_in, g_q, g_k, n_tokens, t0, q_out, k_out, ld_in=None, ld_out=None):
    ref_in = q_in if q_in is not None else k_in
    ref_out = q_out if q_out is not None else k_out
    _check(load().lvx_rope3d(C.byref(desc), _ptr(q_in), _ptr(k_in), ld_in if ld_in is not None else ref_in.stride(0),
                             _ptr(g_q), _ptr(g_k), n_tokens, t0, _ptr(q_out), _ptr(k_out),
                             ld_out if ld_out is not None else ref_out.stride(0), _stream()))


def lvx_rope3d_f32in(desc, q_in, k_in, g_q, g_k, n_tokens, t0, q_out, k_out, ld_in=None, ld_out=None):
    """q_in / k_in fp32 (row stride in fp32 elements), outputs bf16."""
    ref_in = q_in if q_in is not None else k_in
    ref_out = q_out if q_out is not None else k_out
    _check(load().lvx_rope3d_f32in(C.byref(desc), _ptr(q_in), _ptr(k_in), ld_in if ld_in is not None else ref_in.stride(0),
                                   _ptr(g_q), _ptr(g_k), n_tokens, t0, _ptr(q_out), _ptr(k_out),
                                   ld_out if ld_out is not None else ref_out.stride(0), _stream()))


def lvx_chunk_attention(cache, layer, q, scale, out, n_q=None):
    _check(load().lvx_chunk_attention(cache.handle, layer, _ptr(q), q.stride(0), q.shape[0] if n_q is None else n_q,
                                      scale, _ptr(out), out.stride(0), _stream()))


def lvx_chunk_attention_prescaled(cache, layer, q_scaled, out, n_q=None):
    _check(load().lvx_chunk_attention_prescaled(cache.handle, layer, _ptr(q_scaled), q_scaled.stride(0),
                                                q_scaled.shape[0] if n_q is None else n_q, _ptr(out), out.stride(0), _stream()))


def lvx_linear(a, w, c, epi=EPI_STORE, resid=None, gate=None, M=None):
    M = a.shape[0] if M is None else M
    N, K = w.shape[0], w.shape[1]
    _check(load().lvx_linear(_ptr(a), a.stride(0), _ptr(w), w.stride(0), _ptr(c), c.stride(0), M, N, K, epi,
                             _ptr(resid), resid.stride(0) if resid is not None else 0, _ptr(gate), _stream()))


def lvx_linear_dual(a, w1, w2, c1, c2):
    """c1 = a w1^T (bf16 or fp32, by c1's dtype), c2 = a w2^T (bf16); w1 and w2 must share their row stride."""
    import torch
    assert w1.stride(0) == w2.stride(0) and w1.shape[1] == w2.shape[1]
    _check(load().lvx_linear_dual(_ptr(a), a.stride(0), _ptr(w1), _ptr(w2), w1.stride(0), _ptr(c1), c1.stride(0),
                                  1 if c1.dtype == torch.float32 else 0, _ptr(c2), c2.stride(0), a.shape[0], w1.shape[0], w2.shape[0],
                                  w1.shape[1], _stream()))


def lvx_fp8_quantize(x, q=None, row_pad=0):
    """Quantises the bf16 matrix x per tensor; returns (codes uint8 [rows][cols] view, scale fp32 [1])."""
    import torch
    rows, cols = x.shape
    if q is None:
        q = torch.empty((rows, cols + row_pad), dtype=torch.uint8, device=x.device)[:, :cols]
    scratch = torch.empty(256, dtype=torch.uint8, device=x.device)
    scale = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(load().lvx_fp8_quantize(_ptr(x), x.stride(0), rows, cols, _ptr(q), q.stride(0), _ptr(scratch), _ptr(scale), _stream()))
    return q, scale


def lvx_fp8_quantize_static(x, q, scale):
    """The allocation-free form: q (uint8 [rows][>= cols]) and scale (fp32 [1]) are the caller's; nothing is allocated here."""
    rows, cols = x.shape
    _check(load().lvx_fp8_quantize_static(_ptr(x), x.stride(0), rows, cols, _ptr(q), q.stride(0), _ptr(scale), _stream()))


def lvx_linear_fp8(aq, scale_a, wq, scale_w, c, epi=EPI_STORE, resid=None, gate=None):
    M, N, K = aq.shape[0], wq.shape[0], wq.shape[1]
    _check(load().lvx_linear_fp8(_ptr(aq), aq.stride(0), _ptr(scale_a), _ptr(wq), wq.stride(0), _ptr(scale_w), _ptr(c), c.stride(0),
                                 M, N, K, epi, _ptr(resid), resid.stride(0) if resid is not None else 0, _ptr(gate), _stream()))


def lvx_layernorm_modulate(x, shift, scale, eps, u):
    _check(load().lvx_layernorm_modulate(_ptr(x), x.stride(0), _ptr(shift), _ptr(scale), eps, x.shape[0], x.shape[1],
                                         _ptr(u), u.stride(0), _stream()))


class StageHandle:
    """Host-side stage descriptor: keeps the weight tensors alive and holds the C structs."""

    def __init__(self, layers, rope, d_ffn, ldw_d=0, ldw_ffn=0, fp8=False, fp8_row_pad=128, keep_bf16=True):
        """layers: list of dicts of bf16 weight tensors (+ fp32 gains).  fp8=True quantises every linear weight per tensor
        with lvx_fp8_quantize (E4M3 codes + one scale each) and makes the stage run its linears in FP8; with
        keep_bf16=False the bf16 matrices are dropped from the dicts afterwards (the gains stay)."""
        import torch
        self.layers = layers
        self.n = len(layers)
        self.blocks = (BlockWeights * self.n)()
        self.blocks_fp8 = None
        self.fp8_tensors = []
        ldw8_d = ldw8_ffn = 0
        if fp8:
            self.blocks_fp8 = (BlockWeightsFp8 * self.n)()
            for i, w in enumerate(layers):
                scales = torch.empty(len(FP8_WEIGHT_ORDER), dtype=torch.float32, device=w["W_qkv"].device)
                for j, name in enumerate(FP8_WEIGHT_ORDER):
                    q, s = lvx_fp8_quantize(w[name], row_pad=fp8_row_pad)
                    scales[j:j + 1].copy_(s)
                    setattr(self.blocks_fp8[i], name, q.data_ptr())
                    self.fp8_tensors.append(q)
                    if name == "W_qkv":
                        ldw8_d = q.stride(0)
                    if name == "W_2":
                        ldw8_ffn = q.stride(0)
                    if not keep_bf16:
                        w[name] = None
                self.blocks_fp8[i].scales = scales.data_ptr()
                self.fp8_tensors.append(scales)
        for i, w in enumerate(layers):
            for name, _ in BlockWeights._fields_:
                t = w.get(name)
                setattr(self.blocks[i], name, None if t is None else t.data_ptr())
        self.rope = rope
        self.c = Stage(self.n, d_ffn, ldw_d, ldw_ffn, rope, C.cast(self.blocks, C.POINTER(BlockWeights)),
                       C.cast(self.blocks_fp8, C.POINTER(BlockWeightsFp8)) if fp8 else None, ldw8_d, ldw8_ffn)


def lvx_workspace_bytes(stage, n_tokens, n_ctx):
    return load().lvx_workspace_bytes(C.byref(stage.c), n_tokens, n_ctx)


def lvx_context_kv(stage, layer0, n_layers, ctx, k_out, v_out, workspace):
    """k_out, v_out: bf16 [n_layers][n_ctx][d] (contiguous in the first two dims, row stride k_out.stride(1))."""
    _check(load().lvx_context_kv(C.byref(stage.c), layer0, n_layers, _ptr(ctx), ctx.shape[0], _ptr(k_out), _ptr(v_out), k_out.stride(1),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def lvx_dit_block(stage, layer, cache, x, ctx, mod6, chunk_index, t0, workspace):
    _check(load().lvx_dit_block(C.byref(stage.c), layer, cache.handle, _ptr(x), x.shape[0], _ptr(ctx), ctx.shape[0], _ptr(mod6),
                                chunk_index, t0, _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def lvx_dit_block_f32(stage, layer, cache, x32, ctx, mod6, chunk_index, t0, workspace):
    _check(load().lvx_dit_block_f32(C.byref(stage.c), layer, cache.handle, _ptr(x32), x32.shape[0], _ptr(ctx), ctx.shape[0], _ptr(mod6),
                                    chunk_index, t0, _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def lvx_denoise_stage(stage, cache, x, ctx, mod6_per_layer, dt, chunk_index, t0, workspace):
    _check(load().lvx_denoise_stage(C.byref(stage.c), cache.handle, _ptr(x), x.shape[0], _ptr(ctx), ctx.shape[0],
                                    _ptr(mod6_per_layer), dt, chunk_index, t0, _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream()))


def lvx_sink_prefill(stage, cache, x_sink, ctx, mod6_per_layer, t_sink, workspace, x_out=None):
    _check(load().lvx_sink_prefill(C.byref(stage.c), cache.handle, _ptr(x_sink), _ptr(ctx), ctx.shape[0], _ptr(mod6_per_layer), t_sink,
                                   _ptr(x_out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def lvx_sample_chunk(stage, caches, x, ctx, mod6_per_step_layer, dt, chunk_index, t0, t_sink, workspace):
    handles = (C.c_void_p * len(caches))(*[c.handle for c in caches])
    _check(load().lvx_sample_chunk(C.byref(stage.c), handles, len(caches), _ptr(x), x.shape[0], _ptr(ctx), ctx.shape[0],
                                   _ptr(mod6_per_step_layer), dt, chunk_index, t0, t_sink, _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()))


class CausalConv:
    """One causal convolution layer's streaming state (padded volume with the two-frame feature cache) and its handle."""

    def __init__(self, c_in, c_out, height, width, max_frames, device="cuda:0"):
        import torch
        self.desc = ConvDesc(c_in, c_out, height, width, max_frames)
        nbytes = load().lvx_causal_conv_state_bytes(C.byref(self.desc))
        if nbytes == 0:
            raise LvxError(2, load().lvx_last_error().decode())
        self.state = torch.empty(nbytes, dtype=torch.uint8, device=device)
        h = C.c_void_p()
        _check(load().lvx_causal_conv_init(C.byref(self.desc), _ptr(self.state), nbytes, _stream(), C.byref(h)))
        self.handle = h

    def step(self, x, w, bias, act, y):
        """x [n_frames][H][W][c_in], w [c_out][27*c_in] (row stride w.stride(0)), y [n_frames][H][W][c_out]."""
        _check(load().lvx_causal_conv_step(self.handle, _ptr(x), x.shape[0], _ptr(w), w.stride(0), _ptr(bias), int(act), _ptr(y), _stream()))

    def reset(self):
        _check(load().lvx_causal_conv_reset(self.handle, _stream()))

    def close(self):
        if self.handle is not None:
            load().lvx_causal_conv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def lvx_profile_set(level):
    _check(load().lvx_profile_set(level))


def lvx_profile_read():
    """{class: (total_ms, launches)} since the last read; waits for the recorded events."""
    ms = (C.c_double * len(PROF_KINDS))()
    n = (C.c_int64 * len(PROF_KINDS))()
    _check(load().lvx_profile_read(ms, n))
    return {k: (ms[i], n[i]) for i, k in enumerate(PROF_KINDS)}
