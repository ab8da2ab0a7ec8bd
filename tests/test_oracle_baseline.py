"""Pins for the oracle's attention-agnostic retention sets (the pruners the paper's
ablations compare against: Sec. 2.2 random pruning, Sec. 5.2 windows, SD-Uniform and
SD-Frame).  Each mode is checked against a closed form or a brute-force re-statement
that does not call the oracle, so a wrong start, stride or tie rule fails here."""
import numpy as np
import pytest

import oracle

# Outputs 0..4 of SplitMix64 seeded with 1234567, as printed by the generator's public
# reference program (Steele, Lea, Flood, "Fast splittable pseudorandom number generators", 2014;
# test values circulated with the public-domain C version).
SPLITMIX_1234567 = [6457827717110365317, 3203168211198807973, 9817491932198370423,
                    4593380528125082431, 16408922859458223821]


def test_splitmix64_published_vector():
    assert [oracle.splitmix64(1234567, j) for j in range(5)] == SPLITMIX_1234567


def test_windows_closed_forms():
    V, B = 1000, 100
    assert np.array_equal(oracle.baseline_keep("window-front", V, B), np.arange(0, 100))
    assert np.array_equal(oracle.baseline_keep("window-middle", V, B), np.arange(450, 550))
    assert np.array_equal(oracle.baseline_keep("window-end", V, B), np.arange(900, 1000))
    # odd slack: the middle window starts at floor((V-B)/2)
    assert np.array_equal(oracle.baseline_keep("window-middle", 10, 3), np.array([3, 4, 5]))
    for mode in ("window-front", "window-middle", "window-end", "uniform", "random"):
        assert oracle.baseline_keep(mode, 50, 0).size == 0
        assert np.array_equal(oracle.baseline_keep(mode, 50, 50), np.arange(50))


def test_uniform_flat_equals_stage_two_alone():
    """With nothing taken by Stage I the two-stage rule is the flat stride (Eq. 7 with V_R empty)."""
    rng = np.random.default_rng(1)
    for V, B in ((1000, 100), (1568, 157), (97, 41), (12544, 1254), (7, 7), (9, 1)):
        want, _ = oracle.select(rng.random(V, dtype=np.float32), 0, B)
        assert np.array_equal(oracle.baseline_keep("uniform", V, B), want), (V, B)
    assert np.array_equal(oracle.baseline_keep("uniform", 1200, 100), np.arange(0, 1200, 12))
    got = oracle.baseline_keep("uniform", 1001, 100)
    gaps = np.diff(got)
    assert got[0] == 0 and set(gaps.tolist()) <= {10, 11}


def test_frame_drop_keeps_whole_frames_at_regular_interval():
    F, gh, gw = 64, 14, 14
    tpf, V = gh * gw, F * gh * gw
    got = oracle.baseline_keep("frame-drop", V, 8 * tpf, n_frames=F, grid_h=gh, grid_w=gw)
    frames = np.arange(0, 64, 8)                                    # F_k divides F: every 8th frame
    want = (frames[:, None] * tpf + np.arange(tpf)[None, :]).reshape(-1)
    assert np.array_equal(got, want)
    # a budget that is not a whole number of frames keeps floor(B / tokens per frame) frames
    got = oracle.baseline_keep("frame-drop", V, 1254, n_frames=F, grid_h=gh, grid_w=gw)
    fk = 1254 // tpf
    assert got.size == fk * tpf
    kept_frames = np.unique(got // tpf)
    assert np.array_equal(kept_frames, np.array([(t * F) // fk for t in range(fk)]))
    assert np.array_equal(np.bincount(got // tpf, minlength=F)[kept_frames], np.full(fk, tpf))
    assert oracle.baseline_keep("frame-drop", V, tpf - 1, n_frames=F, grid_h=gh, grid_w=gw).size == 0
    with pytest.raises(ValueError):
        oracle.baseline_keep("frame-drop", V + 1, tpf, n_frames=F, grid_h=gh, grid_w=gw)


def test_lattice_brute_force():
    for F, gh, gw, sh, sw in ((3, 14, 14, 3, 3), (2, 16, 16, 4, 2), (1, 5, 7, 2, 3), (4, 14, 14, 1, 1)):
        V = F * gh * gw
        got = oracle.baseline_keep("lattice", V, 0, n_frames=F, grid_h=gh, grid_w=gw, stride_h=sh, stride_w=sw)
        j = np.arange(V)
        row, col = (j % (gh * gw)) // gw, j % gw
        want = j[(row % sh == 0) & (col % sw == 0)]
        assert np.array_equal(got, want)
        assert got.size == F * -(-gh // sh) * -(-gw // sw)


def _splitmix_py(seed, j):
    m = (1 << 64) - 1
    z = (seed + (j + 1) * 0x9E3779B97F4A7C15) & m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def test_uniform_per_frame_pins():
    """Restarted stride: (a) when B is a multiple of F every frame holds the flat stride of its own
    grid, shifted; (b) frame shares differ by at most one and add up to B; (c) every frame with a
    share keeps its first token; (d) a full budget keeps everything; (e) a hand-worked case."""
    F, gh, gw = 8, 14, 14
    tpf, V = gh * gw, F * gh * gw
    got = oracle.baseline_keep("uniform-per-frame", V, 8 * 20, n_frames=F, grid_h=gh, grid_w=gw)
    per = np.array([(u * tpf) // 20 for u in range(20)])
    assert np.array_equal(got, np.concatenate([f * tpf + per for f in range(F)]))
    for Bud in (157, 1, 7, 9, 1567):
        got = oracle.baseline_keep("uniform-per-frame", V, Bud, n_frames=F, grid_h=gh, grid_w=gw)
        assert len(got) == Bud and np.all(np.diff(got) > 0)
        share = np.bincount(got // tpf, minlength=F)
        assert share.max() - share.min() <= 1 and share.sum() == Bud
        for f in range(F):
            if share[f]:
                assert got[got // tpf == f][0] == f * tpf
    assert np.array_equal(oracle.baseline_keep("uniform-per-frame", V, V, n_frames=F, grid_h=gh, grid_w=gw),
                          np.arange(V))
    # 3 frames of 2x3 tokens, budget 4: shares 1, 1, 2 (positions floor(f*4/3)); the last frame keeps 0 and 3
    got = oracle.baseline_keep("uniform-per-frame", 18, 4, n_frames=3, grid_h=2, grid_w=3)
    assert got.tolist() == [0, 6, 12, 15]


def test_random_is_the_top_draws_of_the_stream():
    V, B, seed = 3000, 300, 99
    draws = np.array([_splitmix_py(seed, j) >> 34 for j in range(V)], dtype=np.int64)
    order = sorted(range(V), key=lambda j: (-draws[j], j))
    want = np.sort(np.array(order[:B], dtype=np.int32))
    assert np.array_equal(oracle.baseline_keep("random", V, B, seed=seed), want)


def test_random_subset_properties():
    V, B = 12544, 1254
    a = oracle.baseline_keep("random", V, B, seed=1)
    b = oracle.baseline_keep("random", V, B, seed=2)
    assert a.size == B and np.all(np.diff(a) > 0) and a[0] >= 0 and a[-1] < V
    assert not np.array_equal(a, b)
    assert np.array_equal(a, oracle.baseline_keep("random", V, B, seed=1))       # deterministic in the seed
    # nested in the budget: a larger budget under the same seed keeps a superset
    assert np.isin(a, oracle.baseline_keep("random", V, 2 * B, seed=1)).all()
    # every token is kept about B/V of the time over many seeds (4-sigma band on 16 position bins)
    hits = np.zeros(16)
    n_seeds = 200
    for s in range(n_seeds):
        hits += np.bincount(oracle.baseline_keep("random", 1600, 160, seed=1000 + s) // 100, minlength=16)
    mean = n_seeds * 10.0
    assert np.all(np.abs(hits - mean) < 4.0 * np.sqrt(mean)), hits
