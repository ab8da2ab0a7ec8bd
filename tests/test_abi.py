"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2508_16201_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "specvlm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(specvlm_[a-z_0-9]+)\s*\(", header))
    assert {"specvlm_score", "specvlm_select", "specvlm_gather_kv", "specvlm_decode_attn",
            "specvlm_accept"} <= declared
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)


def test_status_strings_and_version(B):
    assert B.version() >= 100
    assert B.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert B.status_string(code)


def test_workspace_queries_are_pure_host_functions(B):
    assert B.decode_attn_workspace_bytes(1, 6, 12806, 64, 8, 128) > 0
    assert B.decode_attn_workspace_bytes(1, 6, 12806, 64, 8, 96) == 0       # unsupported head_dim
    assert B.decode_attn_workspace_bytes(1, 9, 12806, 64, 8, 128) > 0       # 72 rows per kv head: two row groups
    assert B.decode_attn_workspace_bytes(1, 65, 12806, 64, 8, 128) == 0     # more than 64 queries per request
    assert B.score_workspace_bytes(256, 12800, 12544, 64, 8, 128) > 0
    per_layer = B.score_workspace_bytes(256, 12800, 12544, 64, 8, 128)
    assert B.score_layers_workspace_bytes(1, 256, 12800, 12544, 64, 8, 128) == per_layer
    assert B.score_layers_workspace_bytes(80, 256, 12800, 12544, 64, 8, 128) > per_layer
    assert B.accept_workspace_bytes(1, 5, 152064, True) >= B.accept_workspace_bytes(1, 5, 152064, False) > 0
    assert B.lib().specvlm_select_workspace_bytes(8, 32768) == 0


def test_bad_arguments_are_rejected_before_any_launch(B):
    lib = B.lib()
    null = None
    # decode_attn: q_len > kv_len, heads not divisible, negative sizes
    rc = lib.specvlm_decode_attn(null, 0, 0, null, null, 0, 0, null, null, 1, 4, 2, 8, 2, 128, 0.1,
                                 null, null, 0, null, 0, null)
    assert rc == -1
    rc = lib.specvlm_decode_attn(null, 0, 0, null, null, 0, 0, null, null, 1, 1, 2, 8, 3, 128, 0.1,
                                 null, null, 0, null, 0, null)
    assert rc == -1
    rc = lib.specvlm_decode_attn(null, 0, 0, null, null, 0, 0, null, null, 1, 1, 2, 8, 2, 96, 0.1,
                                 null, null, 0, null, 0, null)
    assert rc == -2
    rc = lib.specvlm_decode_attn(null, 0, 0, null, null, 0, 0, null, null, 0, 1, 2, 8, 2, 128, 0.1,
                                 null, null, 0, null, 0, null)
    assert rc == 0                                                           # batch 0 is legal
    # score: video span beyond keys; gather: keep more than the video holds
    rc = lib.specvlm_score(null, 0, 0, null, 0, 0, null, null, null, 1, 4, 10, 8, 4, 12, 4, 2, 128, 0.1,
                           0, null, 0.0, null, null, 0, null)
    assert rc == -1
    # score_layers: the same checks, plus the layer count and the layer strides
    rc = lib.specvlm_score_layers(null, 0, 0, 0, null, 0, 0, 0, 2, null, null, null, 1, 4, 10, 8, 4, 12, 4, 2, 128,
                                  0.1, 0, null, 0, 0.0, null, null, 0, null)
    assert rc == -1
    rc = lib.specvlm_score_layers(null, 0, 0, 0, null, 0, 0, 0, -1, null, null, null, 1, 4, 10, 0, 4, 6, 4, 2, 128,
                                  0.1, 0, null, 0, 0.0, null, null, 0, null)
    assert rc == -1
    rc = lib.specvlm_score_layers(null, 4, 0, 0, null, 0, 0, 0, 2, null, null, null, 1, 4, 10, 0, 4, 6, 4, 2, 128,
                                  0.1, 0, null, 0, 0.0, null, null, 0, null)
    assert rc == -2                                                          # layer stride not a multiple of 8
    rc = lib.specvlm_gather_kv(null, null, 0, 0, 0, null, null, 0, 0, 0, 1, 10, 0, 4, null, 5,
                               null, null, null, 1, null, 2, 128, null)
    assert rc == -1
    # accept: gamma < 0, vocab < 1, draft logits without uniforms
    rc = lib.specvlm_accept(null, null, null, null, 1, -1, 10, 1.0, null, null, null, 0, null)
    assert rc == -1
    rc = lib.specvlm_accept(null, null, null, null, 1, 2, 0, 1.0, null, null, null, 0, null)
    assert rc == -1
    rc = lib.specvlm_accept(null, C.c_void_p(8), null, null, 1, 2, 10, 1.0, null, null, null, 0, null)
    assert rc == -1
    # select: negative sizes; batch > 1 without cu arrays
    rc = lib.specvlm_select(null, null, null, null, null, -1, 10, 1, null, null, null, null, 0, null)
    assert rc == -1
    rc = lib.specvlm_select(null, null, C.c_void_p(8), C.c_void_p(8), null, 2, 10, 1, null, null, null, null, 0, null)
    assert rc == -1
