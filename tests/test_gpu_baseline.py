"""GPU parity (bit-exact) of specvlm_baseline_keep against the oracle's retention sets of the
ablation pruners (Sec. 2.2 random pruning; Sec. 5.2 windows, SD-Uniform, SD-Frame)."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2508_16201_amd import binding
    binding.lib()
    return binding


def host(t):
    return t.cpu().numpy()


@pytest.mark.parametrize("mode", ["window-front", "window-middle", "window-end", "uniform"])
@pytest.mark.parametrize("V,Bud", [(1568, 157), (12544, 1254), (25088, 2509), (32768, 16384), (97, 41),
                                   (10, 3), (50, 50), (50, 0), (1, 1), (100000, 777)])
def test_closed_form_modes(B, mode, V, Bud):
    got = host(B.baseline_keep(mode, V, Bud))
    assert np.array_equal(got, oracle.baseline_keep(mode, V, Bud)), (mode, V, Bud)


@pytest.mark.parametrize("F,gh,gw,Bud", [(64, 14, 14, 1254), (64, 14, 14, 8 * 196), (128, 16, 16, 3277),
                                         (8, 14, 14, 195), (8, 14, 14, 8 * 196), (3, 5, 7, 36)])
def test_frame_drop(B, F, gh, gw, Bud):
    V = F * gh * gw
    got = host(B.baseline_keep("frame-drop", V, Bud, n_frames=F, grid_h=gh, grid_w=gw))
    assert np.array_equal(got, oracle.baseline_keep("frame-drop", V, Bud, n_frames=F, grid_h=gh, grid_w=gw))


@pytest.mark.parametrize("F,gh,gw,sh,sw", [(64, 14, 14, 3, 3), (128, 16, 16, 4, 2), (1, 5, 7, 2, 3),
                                           (4, 14, 14, 1, 1), (2, 14, 14, 14, 14), (2, 3, 3, 5, 5)])
def test_lattice(B, F, gh, gw, sh, sw):
    V = F * gh * gw
    kw = dict(n_frames=F, grid_h=gh, grid_w=gw, stride_h=sh, stride_w=sw)
    got = host(B.baseline_keep("lattice", V, 0, **kw))
    assert np.array_equal(got, oracle.baseline_keep("lattice", V, 0, **kw))


@pytest.mark.parametrize("F,gh,gw,Bud", [(64, 14, 14, 1254), (128, 16, 16, 3277), (8, 14, 14, 1), (8, 14, 14, 7),
                                         (8, 14, 14, 1568), (3, 2, 3, 4), (1, 5, 7, 11), (64, 14, 14, 0)])
def test_uniform_per_frame(B, F, gh, gw, Bud):
    V = F * gh * gw
    kw = dict(n_frames=F, grid_h=gh, grid_w=gw)
    got = host(B.baseline_keep("uniform-per-frame", V, Bud, **kw))
    assert np.array_equal(got, oracle.baseline_keep("uniform-per-frame", V, Bud, **kw))


@pytest.mark.parametrize("V,Bud,seed", [(1568, 157, 0), (12544, 1254, 1), (25088, 2509, 2), (65536, 6554, 3),
                                        (3000, 1500, 2**63 + 11), (97, 41, 5), (64, 64, 6), (1025, 1, 7),
                                        (40000, 39999, 8)])
def test_random_matches_oracle_stream(B, V, Bud, seed):
    got = host(B.baseline_keep("random", V, Bud, seed=seed))
    assert np.array_equal(got, oracle.baseline_keep("random", V, Bud, seed=seed)), (V, Bud, seed)


def test_baseline_argument_errors(B):
    from paper_2508_16201_amd.binding import SpecVLMError
    with pytest.raises(SpecVLMError):
        B.baseline_keep("uniform", 100, 101)                                  # budget above the token count
    with pytest.raises(SpecVLMError):
        B.baseline_keep("frame-drop", 1000, 100, n_frames=5, grid_h=14, grid_w=14)   # grid does not match V
    with pytest.raises(SpecVLMError):
        B.baseline_keep("lattice", 392, 0, n_frames=2, grid_h=14, grid_w=14, stride_h=0, stride_w=1)
    with pytest.raises(SpecVLMError):
        B.baseline_keep("random", 70000, 100)                                 # above the select kernel's limit


def test_baseline_sets_feed_the_gather(B):
    """A window set drives specvlm_gather_kv like any other keep_idx: the draft cache keeps those rows."""
    from gpu_util import dev_bf16, host_bits, rnd_bits
    V, L, hkv, d, Bud = 588, 20, 2, 64, 59
    k = rnd_bits((1, V + L, hkv, d), 7)
    keep = B.baseline_keep("window-middle", V, Bud)
    kd, _ = B.gather_kv(dev_bf16(k), None, 0, V, keep)
    torch.cuda.synchronize()
    want = oracle.gather_kv(k[0], 0, V, oracle.baseline_keep("window-middle", V, Bud))
    assert np.array_equal(host_bits(kd[0]), want)
