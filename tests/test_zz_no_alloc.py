"""The entry point that allocates nothing (zpp_op_attention_bwd_noalloc: scratch in a static device array)
against the entry point it is a variant of (zpp_op_attention_bwd, scratch passed by the caller), through
the C ABI, on two calls in a row, the second with a smaller input.  The kernels are the same and
deterministic, so the outputs must be bit-identical."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2402_03791_amd as zpp

pytestmark = pytest.mark.gpu


def _case(b, seq, nh, d, impl, dtype, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    h = nh * d
    qkv = torch.randn(b * seq, 3 * h, device="cuda", generator=g).to(dtype)
    dattn = (torch.randn(b * seq, h, device="cuda", generator=g) * 1e-2).to(dtype)
    attn = torch.empty(b * seq, h, device="cuda", dtype=dtype)
    lse = torch.empty(b * nh * seq, device="cuda", dtype=torch.float32)
    zpp.op_attention_fwd(qkv, attn, lse, b, seq, nh, d, impl=impl)
    return qkv, attn, dattn, lse


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


@pytest.mark.parametrize("impl,dtype,first,second", [
    (1, torch.bfloat16, (2, 512, 4, 128), (1, 256, 2, 128)),     # MFMA kernels
    (0, torch.float32, (2, 96, 3, 64), (1, 40, 2, 32)),          # generic kernels
])
def test_attention_backward_without_allocation_matches_the_caller_scratch_call(impl, dtype, first, second):
    L = zpp.lib()
    assert L.zpp_op_attention_bwd_noalloc_max_rows() == 1 << 20
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    dt = 1 if dtype == torch.bfloat16 else 0
    for seed, (b, seq, nh, d) in enumerate((first, second)):
        print(f"no-alloc attention backward impl={impl} b={b} seq={seq} nh={nh} d={d}", flush=True)
        qkv, attn, dattn, lse = _case(b, seq, nh, d, impl, dtype, 40 + seed)
        delta = torch.empty(2 * b * nh * seq, device="cuda", dtype=torch.float32)
        ref = torch.full((b * seq, 3 * nh * d), float("nan"), device="cuda", dtype=dtype)
        out = torch.full_like(ref, float("nan"))
        rc = L.zpp_op_attention_bwd(dt, impl, qkv.data_ptr(), attn.data_ptr(), dattn.data_ptr(), lse.data_ptr(),
                                    delta.data_ptr(), ref.data_ptr(), b, seq, nh, d, stream)
        assert rc == 0, L.zpp_last_error()
        rc = L.zpp_op_attention_bwd_noalloc(dt, impl, qkv.data_ptr(), attn.data_ptr(), dattn.data_ptr(),
                                            lse.data_ptr(), out.data_ptr(), b, seq, nh, d, stream)
        assert rc == 0, L.zpp_last_error()
        torch.cuda.synchronize()
        assert not torch.isnan(ref.float()).any()
        assert torch.equal(_bits(out), _bits(ref))


def test_no_alloc_entry_point_rejects_sizes_beyond_its_scratch():
    L = zpp.lib()
    t = torch.zeros(256, device="cuda")
    p = t.data_ptr()
    # 64 x 64 x 512 rows = 2^21 > 2^20: refused on the host, nothing is launched
    rc = L.zpp_op_attention_bwd_noalloc(1, 1, p, p, p, p, p, 64, 512, 64, 128, None)
    assert rc == -4 and b"static scratch" in L.zpp_last_error()
