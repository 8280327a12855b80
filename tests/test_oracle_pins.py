"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- a library routine (torch SDPA in fp64), brute-force Python
loops, closed forms, invariants, and the figures the paper prints for its own
settings (tests/golden/paper_settings.txt).  None of it needs a GPU."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as orc
from oracle import DENSE, SPATIAL, TEMPORAL, TEXTURAL, Layout, Params

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_settings.txt")


def golden():
    out, sens = {}, []
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if not line:
            continue
        if line[0] == "sensitivity":
            sens.append(tuple(float(x) for x in line[1:]))
        else:
            out[line[0]] = [float(x) for x in line[1:]]
    out["sensitivity"] = sens
    return out


def rand_head(N, D, seed, peaky=1.0):
    g = np.random.default_rng(seed)
    q = (g.standard_normal((N, D)) * peaky / math.sqrt(D)).astype(np.float32)
    k = (g.standard_normal((N, D))).astype(np.float32)
    v = g.standard_normal((N, D)).astype(np.float32)
    return q, k, v


def sdpa64(q, k, v, mask=None):
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))[None, None]
    m = None if mask is None else torch.from_numpy(mask)[None, None]
    return F.scaled_dot_product_attention(t(q), t(k), t(v), attn_mask=m)[0, 0].numpy()


SMALL = Layout(T=4, H=3, W=5, text_len=3)  # N = 63, frames of 15 tokens


# ---------------------------------------------------------------- attention arithmetic (Eq. 1-2)
def test_dense_equals_library_sdpa():
    N = orc.num_tokens(SMALL)
    q, k, v = rand_head(N, 16, 1)
    np.testing.assert_allclose(orc.attention(q, k, v, DENSE, SMALL), sdpa64(q, k, v), rtol=0, atol=1e-12)


def test_dense_equals_python_triple_loop():
    L = Layout(2, 2, 3)
    N, D = orc.num_tokens(L), 4
    q, k, v = rand_head(N, D, 2)
    O = orc.attention(q, k, v, DENSE, L)
    for i in range(N):
        s = [sum(float(q[i, d]) * float(k[j, d]) for d in range(D)) / math.sqrt(D) for j in range(N)]
        e = [math.exp(x - max(s)) for x in s]
        for d in range(D):
            ref = sum(e[j] * float(v[j, d]) for j in range(N)) / sum(e)
            assert abs(O[i, d] - ref) < 1e-12


@pytest.mark.parametrize("cls", [SPATIAL, TEMPORAL, TEXTURAL])
@pytest.mark.parametrize("peaky", [1.0, 8.0])
def test_masked_equals_library_sdpa_with_boolean_mask(cls, peaky):
    """Given the mask, the arithmetic is the library's masked SDPA."""
    P = Params(0.3, 0.3, 2)
    N = orc.num_tokens(SMALL)
    q, k, v = rand_head(N, 8, 3 + cls, peaky)
    M = orc.keep_matrix(cls, SMALL, P)
    np.testing.assert_allclose(orc.attention(q, k, v, cls, SMALL, P), sdpa64(q, k, v, M), rtol=0, atol=1e-12)


def test_spatial_radius_zero_is_per_frame_attention():
    L = Layout(3, 2, 4)
    HW, N = 8, 24
    q, k, v = rand_head(N, 8, 5)
    O = orc.attention(q, k, v, SPATIAL, L, Params(bw_spatial=0.0))
    for f in range(3):
        s = slice(f * HW, (f + 1) * HW)
        np.testing.assert_allclose(O[s], sdpa64(q[s], k[s], v[s]), atol=1e-12)


def test_patterns_that_reduce_to_dense():
    N = orc.num_tokens(SMALL)
    q, k, v = rand_head(N, 8, 6)
    ref = sdpa64(q, k, v)
    np.testing.assert_allclose(orc.attention(q, k, v, TEMPORAL, SMALL, Params(bw_temporal=1.0)), ref, atol=1e-12)
    np.testing.assert_allclose(orc.attention(q, k, v, SPATIAL, SMALL, Params(bw_spatial=1.0)), ref, atol=1e-12)
    np.testing.assert_allclose(orc.attention(q, k, v, TEXTURAL, SMALL, Params(tex_stride=1)), ref, atol=1e-12)


def test_textural_is_dense_attention_on_gathered_keys():
    """Eq. 5: Attn(Q, K_C, V_C, M_init) -- gather the kept keys, then plain SDPA."""
    L = Layout(3, 4, 6, text_len=2)
    N = orc.num_tokens(L)
    q, k, v = rand_head(N, 8, 7)
    C = [j for j in range(N) if orc.keep(TEXTURAL, 0, j, L, Params(tex_stride=3))]
    assert 0 < len(C) < N
    Nv = 3 * 4 * 6
    O = orc.attention(q, k, v, TEXTURAL, L, Params(tex_stride=3))
    np.testing.assert_allclose(O[:Nv], sdpa64(q[:Nv], k[C], v[C]), atol=1e-12)
    # text query rows attend every key under every pattern
    np.testing.assert_allclose(O[Nv:], sdpa64(q, k, v)[Nv:], atol=1e-12)


def test_softmax_rows_sum_to_one_and_masked_entries_are_zero():
    P = Params()
    N = orc.num_tokens(SMALL)
    q, k, v = rand_head(N, 8, 8, 4.0)
    for cls in (SPATIAL, TEMPORAL, TEXTURAL, DENSE):
        _, Pr = orc.attention_rows(q, k, v, cls, SMALL, P, np.arange(N), want_prob=True)
        np.testing.assert_allclose(Pr.sum(1), 1.0, atol=1e-13)
        M = orc.keep_matrix(cls, SMALL, P)
        assert (Pr[~M] == 0).all() and (Pr[M] > 0).all()


def test_constant_values_and_key_shift_invariance():
    N = orc.num_tokens(SMALL)
    q, k, v = rand_head(N, 8, 9)
    for cls in (SPATIAL, TEMPORAL, TEXTURAL):
        np.testing.assert_allclose(orc.attention(q, k, np.ones_like(v), cls, SMALL), 1.0, atol=1e-13)
        shift = np.full((1, 8), 0.37, dtype=np.float32)  # adds q.c to every score of a row
        np.testing.assert_allclose(orc.attention(q, k + shift, v, cls, SMALL),
                                   orc.attention(q, k, v, cls, SMALL), atol=1e-6)


@pytest.mark.parametrize("cls", [SPATIAL, TEMPORAL, TEXTURAL, DENSE])
@pytest.mark.parametrize("block", [8, 16])
def test_block_skipping_changes_nothing(cls, block):
    L = Layout(6, 3, 5, text_len=5)  # N = 95, ragged against both block sizes
    N = orc.num_tokens(L)
    q, k, v = rand_head(N, 8, 10, 3.0)
    P = Params(0.2, 0.2, 2)
    O, vis, tot = orc.attention_blockskip(q, k, v, cls, L, P, block)
    np.testing.assert_allclose(O, orc.attention(q, k, v, cls, L, P), atol=1e-12)
    assert tot == math.ceil(N / block) ** 2
    if cls in (SPATIAL,):
        assert vis < tot  # something really is skipped
    if cls == DENSE:
        assert vis == tot


def test_tiny_config_heads():
    """The tiny workload's forced classes: all-ones mask equals brute-force dense."""
    L = Layout(4, 8, 8)
    q, k, v = rand_head(256, 64, 11)
    ref = sdpa64(q, k, v)
    np.testing.assert_allclose(orc.attention(q, k, v, DENSE, L), ref, atol=1e-12)
    for cls in (SPATIAL, TEMPORAL, TEXTURAL):
        O64, _, _ = orc.attention_blockskip(q, k, v, cls, L, Params(), 64)
        np.testing.assert_allclose(O64, orc.attention(q, k, v, cls, L), atol=1e-12)


# ---------------------------------------------------------------- mask geometry (Sec. 3.2, 4.1)
def band_fraction(n, r):
    """kept fraction of an n x n band |a-b| <= r."""
    r = min(r, n - 1)
    return (n * (2 * r + 1) - r * (r + 1)) / n ** 2


def test_band_closed_forms():
    L = Layout(16, 4, 8)
    for bw in (0.0, 0.13, 0.25, 0.5):
        rs, rt = orc.radius(bw, 16), orc.radius(bw, 32)
        assert rs == math.floor(np.float32(bw) * 16) and rt == math.floor(np.float32(bw) * 32)
        assert orc.kept_fraction(SPATIAL, L, Params(bw_spatial=bw)) == pytest.approx(band_fraction(16, rs), abs=1e-12)
        assert orc.kept_fraction(TEMPORAL, L, Params(bw_temporal=bw)) == pytest.approx(band_fraction(32, rt), abs=1e-12)


def test_paper_default_band_is_nine_sixteenths_reduction():
    g = golden()
    w = g["default_bandwidth"][0]
    # a band of relative half-width w keeps 1-(1-w)^2; the paper calls that a 9/16 reduction
    assert 1 - (1 - w) ** 2 == pytest.approx(1 - g["default_band_reduction"][0])
    L = Layout(8, 32, 32)  # HW = 1024: large enough that the discrete band is at its limit
    assert orc.kept_fraction(TEMPORAL, L, Params(bw_temporal=w)) == pytest.approx(7 / 16, abs=2e-3)
    L = Layout(256, 2, 2)
    assert orc.kept_fraction(SPATIAL, L, Params(bw_spatial=w)) == pytest.approx(7 / 16, abs=5e-3)


def test_paper_cogvideox_sparsity_is_fifty_percent():
    """Latent (12,30,45) with bandwidth 1/4: floor(12/4)=3 frames each side keeps exactly half."""
    g = golden()
    T, H, W = (int(x) for x in g["cogvideox_latent"])
    L = Layout(T, 6, 9)  # frame band does not depend on H, W; keep the count cheap
    assert orc.kept_fraction(SPATIAL, L, Params(bw_spatial=g["default_bandwidth"][0])) == pytest.approx(
        g["default_sparsity"][0], abs=1e-12)


def test_paper_checkerboard_keeps_half_and_four_neighbours():
    g = golden()
    tau = int(g["default_tex_stride"][0])
    for (H, W) in ((30, 40), (30, 45), (45, 80), (5, 7)):
        L = Layout(2, H, W)
        kept = np.array([orc.keep(TEXTURAL, 0, j, L, Params(tex_stride=tau)) for j in range(2 * H * W)])
        assert kept.mean() == pytest.approx(g["default_tex_kept"][0], abs=0.5 / (H * W) + 1e-12)
        grid = kept.reshape(2, H, W)
        assert (grid[0] == grid[1]).all()  # same subset in every frame
        for y in range(H):
            for x in range(W):
                if not grid[0, y, x]:  # every dropped token has its 4-neighbours kept (Sec. 3.2)
                    for yy, xx in ((y - 1, x), (y + 1, x), (y, x - 1), (y, x + 1)):
                        if 0 <= yy < H and 0 <= xx < W:
                            assert grid[0, yy, xx]


def test_paper_sensitivity_speedups():
    """Tab. 3: 1.85x / 2.5x / 3.0x for (w, tau) = (.25,2) (.18,3) (.13,4), first 10 % steps dense."""
    g = golden()
    dense_share = g["dense_step_share"][0]
    for speed, w, tau in g["sensitivity"]:
        L = Layout(4, 30, 45)
        tex = orc.kept_fraction(TEXTURAL, L, Params(tex_stride=int(tau)))
        assert 1 / (dense_share + (1 - dense_share) * tex) == pytest.approx(speed, abs=0.1)
        Lb = Layout(2, 40, 50)  # HW = 2000
        band = orc.kept_fraction(TEMPORAL, Lb, Params(bw_temporal=w))
        assert 1 / (dense_share + (1 - dense_share) * band) == pytest.approx(speed, abs=0.2)


def test_mask_structure():
    L = Layout(5, 3, 4, text_len=2)
    HW, Nv, N = 12, 60, 62
    P = Params(0.25, 0.25, 2)
    S, Tm, X = (orc.keep_matrix(c, L, P) for c in (SPATIAL, TEMPORAL, TEXTURAL))
    for M in (S, Tm):
        assert (M == M.T).all() and M.diagonal().all()
    assert S[Nv:].all() and S[:, Nv:].all() and Tm[Nv:].all() and X[:, Nv:].all()
    # Spatial: constant on frame x frame tiles; Temporal: periodic with the frame length
    for fa in range(5):
        for fb in range(5):
            tile = S[fa * HW:(fa + 1) * HW, fb * HW:(fb + 1) * HW]
            assert tile.all() == (abs(fa - fb) <= 1) and tile.any() == (abs(fa - fb) <= 1)
            assert (Tm[fa * HW:(fa + 1) * HW, fb * HW:(fb + 1) * HW] == Tm[:HW, :HW]).all()
    p = np.arange(HW)
    assert (Tm[:HW, :HW] == (np.abs(p[:, None] - p[None, :]) <= 3)).all()
    # Textural: every video query row sees the same key subset; text rows see everything
    assert (X[:Nv] == X[0]).all() and X[Nv:].all()
    y, x = p // 4, p % 4
    assert (X[0, :HW] == ((y - x) % 2 == 0)).all()
    # Eq. 4 as printed: row and column index share their residue modulo tau
    X3 = orc.keep_matrix(TEXTURAL, L, Params(tex_stride=3))
    assert (X3[0, :HW] == (y % 3 == x % 3)).all() and (X3[0, HW:2 * HW] == X3[0, :HW]).all()


# ---------------------------------------------------------------- ARM (Sec. 3.3, Eq. 6, Alg. 1)
def test_sampling_sets():
    L = Layout(6, 4, 5, text_len=7)
    assert (orc.sample_tokens(L, Params(), False) == np.arange(20)).all()  # first frame
    assert (orc.sample_tokens(L, Params(), True) == np.arange(0, 120, 6)).all()  # omega = T
    assert (orc.sample_tokens(L, Params(sample_interval=7), True) == np.arange(0, 120, 7)).all()


def test_full_mask_gives_recall_one():
    L = Layout(4, 4, 4, text_len=3)
    q, k, _ = rand_head(orc.num_tokens(L), 8, 20, 5.0)
    for glob in (False, True):
        assert orc.arm_recall(q, k, L, Params(), glob, DENSE) == pytest.approx(1.0, abs=1e-14)
        assert orc.arm_recall(q, k, L, Params(bw_temporal=1.0), glob, TEMPORAL) == pytest.approx(1.0, abs=1e-14)


def test_uniform_attention_recall_is_mask_area():
    """Q = 0 makes every softmax row uniform, so recall = kept fraction of the sampled mask."""
    L = Layout(8, 4, 8)  # HW = 32 is a multiple of T = 8: 4 samples per frame under omega = T
    N = orc.num_tokens(L)
    _, k, _ = rand_head(N, 8, 21)
    q = np.zeros_like(k)
    P = Params(0.25, 0.25)
    assert orc.arm_recall(q, k, L, P, False, TEMPORAL) == pytest.approx(band_fraction(32, 8), abs=1e-13)
    assert orc.arm_recall(q, k, L, P, True, SPATIAL) == pytest.approx(band_fraction(8, 2), abs=1e-13)
    # local samples all sit in frame 0, so the Spatial mask cannot exclude anything there
    assert orc.arm_recall(q, k, L, P, False, SPATIAL) == pytest.approx(1.0, abs=1e-14)


def test_one_hot_shifted_keys_recall_counts_rows_inside_band():
    """Query a looks (almost) only at key (a + s) mod n: recall = share of rows whose target is in the band."""
    L = Layout(2, 4, 8)
    HW, D, g = 32, 32, 40.0
    N = orc.num_tokens(L)
    eye = np.eye(D, dtype=np.float32)
    for s in (0, 3, 9, 30):
        q = np.zeros((N, D), np.float32)
        k = np.zeros((N, D), np.float32)
        q[:HW] = g * eye
        k[:HW] = g * np.roll(eye, s, axis=0)  # key j carries e_{(j - s) mod HW}
        r = orc.radius(0.25, HW)
        inside = sum(abs(((a + s) % HW) - a) <= r for a in range(HW)) / HW
        got = orc.arm_recall(q, k, L, Params(), False, TEMPORAL)
        assert got == pytest.approx(inside, abs=1e-6)


def test_row_mean_reading_of_recall():
    L = Layout(3, 2, 4)
    q, k, _ = rand_head(orc.num_tokens(L), 8, 22, 6.0)
    r, rows = orc.arm_recall(q, k, L, Params(), True, SPATIAL, want_rows=True)
    assert r == pytest.approx(rows.mean(), abs=1e-14) and ((rows > 0) & (rows <= 1)).all()
    # each row's recall is the masked share of the library softmax over the sampled keys
    idx = orc.sample_tokens(L, Params(), True)
    S = torch.softmax(torch.from_numpy((q[idx].astype(np.float64) @ k[idx].astype(np.float64).T) / math.sqrt(8)), -1).numpy()
    M = orc.keep_matrix(SPATIAL, L, Params())[np.ix_(idx, idx)]
    np.testing.assert_allclose(rows, (S * M).sum(1), atol=1e-13)


def test_decision_rule_truth_table():
    a = 0.9
    assert orc.decide(0.95, 0.95, a) == TEMPORAL  # both above: Temporal has priority (Alg. 1)
    assert orc.decide(0.95, 0.10, a) == TEMPORAL
    assert orc.decide(0.10, 0.95, a) == SPATIAL
    assert orc.decide(0.10, 0.10, a) == TEXTURAL
    assert orc.decide(0.9, 0.0, a) == TEMPORAL and orc.decide(0.0, 0.9, a) == SPATIAL  # ">=" as printed
    assert orc.decide(np.nextafter(0.9, 0), np.nextafter(0.9, 0), a) == TEXTURAL


def test_classify_combines_recalls_and_rule():
    L = Layout(4, 4, 4)
    q, k, _ = rand_head(64, 8, 23, 3.0)
    for mode in (orc.SAMPLE_FIRST_FRAME, orc.SAMPLE_EQUAL_INTERVAL):
        c, (rh, rt) = orc.arm_classify(q, k, L, Params(), mode, 0.5)
        assert rh == orc.arm_recall(q, k, L, Params(), mode == orc.SAMPLE_EQUAL_INTERVAL, TEMPORAL)
        assert rt == orc.arm_recall(q, k, L, Params(), True, SPATIAL)
        assert c == orc.decide(rh, rt, 0.5)


# ---------------------------------------------------------------- RainFusion+ (Sec. 4.3)
BWS = (0.5, 0.25, 0.125)


def test_plus_with_one_candidate_is_algorithm_one():
    L = Layout(4, 4, 4)
    q, k, _ = rand_head(64, 8, 30, 3.0)
    for alpha in (0.3, 0.6, 0.9):
        c, idx, rec = orc.arm_classify_plus(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, alpha, [0.25])
        c1, (rh, rt) = orc.arm_classify(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, alpha)
        assert c == c1 and rec[0, 0] == rh and rec[1, 0] == rt
        assert idx == (-1 if c == TEXTURAL else 0)


def test_plus_recalls_grow_with_bandwidth_and_minimum_is_chosen():
    L = Layout(8, 4, 8)
    N = orc.num_tokens(L)
    _, k, _ = rand_head(N, 8, 31)
    q = np.zeros_like(k)  # uniform attention: recall = area of the sampled mask, a closed form
    hat = [band_fraction(32, math.floor(b * 32)) for b in BWS]
    til = [band_fraction(8, math.floor(b * 8)) for b in BWS]
    c, idx, rec = orc.arm_classify_plus(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, 0.7, BWS)
    np.testing.assert_allclose(rec[0], hat, atol=1e-13)
    np.testing.assert_allclose(rec[1], til, atol=1e-13)
    assert rec[0, 0] >= rec[0, 1] >= rec[0, 2] and rec[1, 0] >= rec[1, 1] >= rec[1, 2]
    # band_fraction(32, 16) = 0.742 is the only Temporal candidate above 0.7
    assert (c, idx) == (TEMPORAL, 0)
    c, idx, _ = orc.arm_classify_plus(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, 0.4, BWS)
    assert (c, idx) == (TEMPORAL, 1)  # 0.25 -> 0.43 still holds 40 %, 0.125 -> 0.23 does not: minimum that holds
    c, idx, _ = orc.arm_classify_plus(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, 0.8, BWS)
    assert (c, idx) == (SPATIAL, 0)  # Temporal never reaches 0.8; Spatial band_fraction(8, 4) = 0.81 does
    c, idx, _ = orc.arm_classify_plus(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, 0.95, BWS)
    assert (c, idx) == (TEXTURAL, -1)
    # candidate order must not matter
    c, idx, _ = orc.arm_classify_plus(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, 0.4, (0.125, 0.5, 0.25))
    assert (c, idx) == (TEMPORAL, 2)


def test_two_head_mode_sends_unmatched_heads_to_dense():
    """Tab. 2 "two mask" rows: without the Textural pattern a head that matches neither mask stays dense."""
    L = Layout(4, 4, 4)
    q, k, _ = rand_head(64, 8, 40, 3.0)
    for alpha in (0.2, 0.6, 0.99):
        c3, r3 = orc.arm_classify(q, k, L, Params(), orc.SAMPLE_FIRST_FRAME, alpha)
        c2, r2 = orc.arm_classify(q, k, L, Params(two_head=True), orc.SAMPLE_FIRST_FRAME, alpha)
        assert r2 == r3 and c2 == (DENSE if c3 == TEXTURAL else c3)
    c2, idx, _ = orc.arm_classify_plus(q, k, L, Params(two_head=True), orc.SAMPLE_FIRST_FRAME, 0.999, BWS)
    assert (c2, idx) == (DENSE, -1)


# ---------------------------------------------------------------- text tokens in front of the video
def test_text_first_mask_from_first_principles():
    """With the text tokens first, token n >= text_len is video token n - text_len; the predicate is
    rebuilt here from frames, rows and columns and compared entry by entry."""
    L, tl = Layout(4, 3, 4, text_len=5), 5
    HW, Nv, N = 12, 48, 53
    P = Params(0.25, 0.25, 2, text_first=True)
    n = np.arange(N)
    is_text = n < tl
    v = n - tl
    f, p = v // HW, v % HW
    y, x = p // 4, p % 4
    either_text = is_text[:, None] | is_text[None, :]
    want = {
        SPATIAL: either_text | (np.abs(f[:, None] - f[None, :]) <= 1),
        TEMPORAL: either_text | (np.abs(p[:, None] - p[None, :]) <= 3),
        TEXTURAL: either_text | np.broadcast_to(((y - x) % 2 == 0)[None, :], (N, N)),
        DENSE: np.ones((N, N), bool),
    }
    for cls, M in want.items():
        assert (orc.keep_matrix(cls, L, P) == M).all(), cls


def test_text_first_is_the_text_last_problem_rotated():
    """Moving the text rows from the end to the front and setting the flag must give the same
    attention rows (moved the same way), the same samples (shifted) and the same recalls."""
    L, tl = Layout(3, 3, 4, text_len=6), 6
    N, D = orc.num_tokens(L), 8
    q, k, v = rand_head(N, D, 41, peaky=6.0)
    front = np.r_[np.arange(N - tl, N), np.arange(N - tl)]  # new row i holds old row front[i]
    for cls in (SPATIAL, TEMPORAL, TEXTURAL):
        ref = orc.attention(q, k, v, cls, L, Params())
        got = orc.attention(q[front], k[front], v[front], cls, L, Params(text_first=True))
        np.testing.assert_allclose(got, ref[front], rtol=0, atol=1e-12)
        # and it is SDPA under the explicit boolean mask of the rotated problem
        M = orc.keep_matrix(cls, L, Params(text_first=True))
        np.testing.assert_allclose(got, sdpa64(q[front], k[front], v[front], M), rtol=0, atol=1e-12)
    for glob in (False, True):
        assert (orc.sample_tokens(L, Params(text_first=True), glob) == orc.sample_tokens(L, Params(), glob) + tl).all()
        for cls in (SPATIAL, TEMPORAL):
            assert orc.arm_recall(q[front], k[front], L, Params(text_first=True), glob, cls) == pytest.approx(
                orc.arm_recall(q, k, L, Params(), glob, cls), abs=1e-14)
    # without text tokens the flag changes nothing
    L0 = Layout(3, 3, 4)
    assert (orc.keep_matrix(TEMPORAL, L0, Params(text_first=True)) == orc.keep_matrix(TEMPORAL, L0, Params())).all()
