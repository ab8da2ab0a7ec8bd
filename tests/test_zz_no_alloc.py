"""GPU test of specvlm_decode_attn_static (the entry point whose scratch lives inside the library):
same results as specvlm_decode_attn, which is itself checked against the oracle, on two calls in a
row, the second with a smaller input; no device memory is allocated by the call."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev_bf16, host_f64, rnd_bits, assert_attn_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2508_16201_amd import binding
    binding.lib()
    return binding


def _case(B, q_len, kv_len, hq, hkv, d, seed, num_splits=0):
    q, k, v = rnd_bits((q_len, hq, d), seed), rnd_bits((kv_len, hkv, d), seed + 1), rnd_bits((kv_len, hkv, d), seed + 2)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    scale = 1.0 / np.sqrt(d)
    ref, ref_lse = B.decode_attn(qd, kd, vd, scale, want_lse=True, num_splits=num_splits)
    out = torch.full_like(qd, float("nan"))
    lse = torch.full((q_len, hq), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    # torch's allocator counts every allocation it serves: the call must add none
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    B.decode_attn_static(qd, kd, vd, scale, out=out, lse=lse, num_splits=num_splits)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    # the same kernels on the same inputs: bitwise equal to the workspace entry point
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    assert torch.equal(lse, ref_lse)
    want, want_lse = oracle.decode_attn(q, k, v, scale)
    assert_attn_close(out, want, f"static q{q_len} kv{kv_len}")
    np.testing.assert_allclose(host_f64(lse), want_lse, atol=2e-3, rtol=1e-4)


def test_two_calls_in_a_row_second_smaller(B):
    _case(B, 6, 5000, 16, 2, 128, seed=810)               # split-K: partial results go through the scratch array
    _case(B, 6, 1900, 16, 2, 128, seed=820)               # fewer splits' worth of slots than the call before
    _case(B, 1, 700, 14, 2, 64, seed=830, num_splits=5)
    _case(B, 3, 40, 4, 1, 64, seed=840)                   # a single split: the scratch array is not used at all


def test_ragged_batch_through_the_static_scratch(B):
    lens, q_lens, hq, hkv, d = [700, 33, 2049, 1280], [6, 6, 1, 4], 16, 2, 128
    qs = [rnd_bits((ql, hq, d), 850 + i) for i, ql in enumerate(q_lens)]
    ks = [rnd_bits((n, hkv, d), 860 + i) for i, n in enumerate(lens)]
    vs = [rnd_bits((n, hkv, d), 870 + i) for i, n in enumerate(lens)]
    cu_q = torch.tensor(np.concatenate([[0], np.cumsum(q_lens)]), dtype=torch.int32).cuda()
    cu_kv = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32).cuda()
    qd, kd, vd = dev_bf16(np.concatenate(qs)), dev_bf16(np.concatenate(ks)), dev_bf16(np.concatenate(vs))
    out = torch.empty_like(qd)
    B.decode_attn_static(qd, kd, vd, 0.088, out=out, cu_q=cu_q, cu_kv=cu_kv, max_q_len=6, max_kv_len=max(lens))
    torch.cuda.synchronize()
    o = 0
    for i in range(len(lens)):
        want, _ = oracle.decode_attn(qs[i], ks[i], vs[i], 0.088)
        assert_attn_close(out[o:o + q_lens[i]], want, f"static, request {i}")
        o += q_lens[i]


def test_shapes_beyond_the_scratch_are_refused(B):
    lib = B.lib()
    cap = lib.specvlm_decode_attn_static_scratch_bytes()
    assert cap == 16 << 20
    # 64 rows x 256 splits x 16 heads of fp32 partials: far more than the array holds
    assert B.decode_attn_workspace_bytes(1, 8, 1 << 20, 128, 16, 128, 256) > cap
    q = torch.zeros((8, 128, 128), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((1 << 16, 16, 128), dtype=torch.bfloat16, device="cuda")
    rc = lib.specvlm_decode_attn_static(C.c_void_p(q.data_ptr()), 128 * 128, 128, C.c_void_p(kv.data_ptr()),
                                        C.c_void_p(kv.data_ptr()), 16 * 128, 128, None, None, 1, 8, 1 << 20,
                                        128, 16, 128, 0.1, C.c_void_p(q.data_ptr()), None, 256, None)
    assert rc == -3
