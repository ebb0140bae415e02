"""lvx_fp8_quantize_static (the entry point that allocates nothing: its amax slots live in a device array inside the library)
against lvx_fp8_quantize (scratch handed over by the caller), through the C ABI: codes and scale bit for bit, on two calls in a
row, the second on a smaller tensor whose amax is smaller too (a maximum left over from the first call would coarsen its grid)."""
import ctypes as C

import numpy as np
import pytest
import torch

import lvx_synth as S

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_static_scratch_quantize_matches_caller_scratch_quantize(lvx):
    lib = lvx.load()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # outputs and the reference path's scratch are allocated up front; the calls under test receive pointers only
    shapes = [(4680, 5120, 64, 3.0), (1000, 1280, 0, 0.05), (37, 16, 16, 1.0), (1, 512, 0, 0.0)]
    bufs = []
    for rows, cols, pad, std in shapes:
        x = (S.randn_bf16_device((rows, cols + pad), S.seed_of("na_x", rows, cols), 1.0, DEV).float() * std).to(torch.bfloat16)[:, :cols]
        ldq = (cols + 15) // 16 * 16 + (128 if pad else 0)
        bufs.append(dict(x=x, q_ref=torch.zeros((rows, ldq), dtype=torch.uint8, device=DEV), q=torch.zeros((rows, ldq), dtype=torch.uint8, device=DEV),
                         s_ref=torch.zeros(1, dtype=torch.float32, device=DEV), s=torch.zeros(1, dtype=torch.float32, device=DEV),
                         scratch=torch.empty(256, dtype=torch.uint8, device=DEV)))
    torch.cuda.synchronize()
    for rep in range(2):                      # the whole series twice: every call finds the array as some other call left it
        for (rows, cols, pad, std), b in zip(shapes, bufs):
            b["q"].zero_()
            b["s"].zero_()
            x = b["x"]
            st = lib.lvx_fp8_quantize(x.data_ptr(), x.stride(0), rows, cols, b["q_ref"].data_ptr(), b["q_ref"].stride(0),
                                      b["scratch"].data_ptr(), b["s_ref"].data_ptr(), stream)
            assert st == 0, lib.lvx_last_error()
            st = lib.lvx_fp8_quantize_static(x.data_ptr(), x.stride(0), rows, cols, b["q"].data_ptr(), b["q"].stride(0), b["s"].data_ptr(), stream)
            assert st == 0, lib.lvx_last_error()
            torch.cuda.synchronize()
            assert torch.equal(b["s"], b["s_ref"]), (rows, cols, float(b["s"]), float(b["s_ref"]))
            assert torch.equal(b["q"][:, :cols], b["q_ref"][:, :cols]), (rows, cols)
            assert bool((b["q"][:, cols:] == 0).all())
            if std == 0.0:
                assert float(b["s"]) == 1.0 and bool(((b["q"] & 0x7f) == 0).all())   # all-zero tensor: scale 1, codes +-0
            else:
                assert float(b["s"]) == float(np.float32(float(x.float().abs().max())) / np.float32(448.0))
    # beyond the stated maximum: refused on the host, nothing enqueued
    p = C.c_void_p(bufs[0]["x"].data_ptr())
    assert lib.lvx_fp8_quantize_static(p, 1 << 20, 1 << 12, 1 << 20, p, 1 << 20, C.c_void_p(bufs[0]["s"].data_ptr()), stream) == 2
    assert b"lvx_fp8_quantize_static" in lib.lvx_last_error()
    assert lib.lvx_fp8_quantize_static(None, 64, 4, 64, p, 64, C.c_void_p(bufs[0]["s"].data_ptr()), stream) == 1
