"""Host logic of the library, no GPU: the block lists against a brute-force scan of the
oracle's token predicate, the exported symbols against the header, and argument checks."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle as orc
import paper_2505_21036_amd as rf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

LAYOUTS = [
    (4, 8, 8, 0),      # tiny: block 64 == one frame
    (5, 6, 11, 19),    # frames of 66 tokens straddle 64-blocks, text tail
    (3, 20, 23, 70),   # frames of 460 tokens, text spans more than one 64-block
    (7, 10, 13, 50),
    (2, 5, 5, 0),      # frames smaller than a block
    (9, 3, 3, 200),    # mostly text
]
PARAMS = [(0.25, 0.25, 2), (0.13, 0.18, 3), (0.0, 0.0, 4), (1.0, 1.0, 1), (0.4, 0.05, 2)]


TILE = rf.RF_KEY_TILE


def brute_blocks(M, block):
    """(any, all-and-no-tail) per (query block, 64-key tile) pair from an explicit boolean mask."""
    N = M.shape[0]
    nb, nt = -(-N // block), -(-N // TILE)
    pad = np.zeros((nb * block, nt * TILE), dtype=bool)
    pad[:N, :N] = M
    t = pad.reshape(nb, block, nt, TILE)
    any_ = t.any(axis=(1, 3))
    # "full" means every existing query row keeps every key slot of the tile, tail slots included
    rows = np.zeros(nb * block, dtype=bool)
    rows[:N] = True
    full = np.ones((nb, nt), dtype=bool)
    for qb in range(nb):
        r = rows[qb * block:(qb + 1) * block]
        full[qb] = t[qb][r].all(axis=(0, 2))
    return any_, full


@pytest.mark.parametrize("lay", LAYOUTS)
@pytest.mark.parametrize("par", PARAMS)
@pytest.mark.parametrize("block", [64, 128, 256, 384])
def test_block_lists_match_brute_force(lay, par, block):
    L, P = orc.Layout(*lay), orc.Params(par[0], par[1], par[2])
    rl, rp = rf.rf_layout(*lay), rf.rf_params(par[0], par[1], par[2], 0)
    N = orc.num_tokens(L)
    nb = -(-N // block)
    for cls in (orc.SPATIAL, orc.TEMPORAL, orc.DENSE):
        any_, full = brute_blocks(orc.keep_matrix(cls, L, P), block)
        row_ptr, cols = rf.rf_plan_host(rl, rp, block, cls)
        assert len(row_ptr) == nb + 1 and row_ptr[0] == 0
        for qb in range(nb):
            ent = cols[row_ptr[qb]:row_ptr[qb + 1]]
            kbs = ent & ~rf.RF_PLAN_PARTIAL
            assert (np.diff(kbs) > 0).all()
            assert set(kbs.tolist()) == set(np.nonzero(any_[qb])[0].tolist())  # visited == has a kept pair
            partial = (ent & rf.RF_PLAN_PARTIAL) != 0
            assert (partial == ~full[qb, kbs]).all()  # predicate re-applied exactly where needed


@pytest.mark.parametrize("lay", LAYOUTS)
@pytest.mark.parametrize("par", PARAMS)
@pytest.mark.parametrize("block", [64, 128, 256, 384])
def test_position_major_temporal_lists(lay, par, block):
    """The list a Temporal head walks over the position-major copy: the oracle's mask, rows and
    columns permuted into that order, scanned by brute force."""
    L, P = orc.Layout(*lay), orc.Params(par[0], par[1], par[2])
    rl, rp = rf.rf_layout(*lay), rf.rf_params(par[0], par[1], par[2], 0)
    N, (T, H, W, tl) = orc.num_tokens(L), lay
    tok = rf.rf_plan_position_major(rl)
    assert sorted(tok.tolist()) == list(range(N))
    for f in range(T):
        for p in (0, H * W // 2, H * W - 1):
            assert tok[p * T + f] == f * H * W + p
    assert (tok[T * H * W:] == np.arange(T * H * W, N)).all()
    M = orc.keep_matrix(orc.TEMPORAL, L, P)[np.ix_(tok, tok)]
    any_, full = brute_blocks(M, block)
    row_ptr, cols = rf.rf_plan_host(rl, rp, block, rf.RF_LIST_TEMPORAL_POSITION_MAJOR)
    for qb in range(len(row_ptr) - 1):
        ent = cols[row_ptr[qb]:row_ptr[qb + 1]]
        kbs, partial = ent & ~rf.RF_PLAN_PARTIAL, (ent & rf.RF_PLAN_PARTIAL) != 0
        assert set(kbs.tolist()) == set(np.nonzero(any_[qb])[0].tolist())
        assert (partial == ~full[qb, kbs]).all()
    order = rf.rf_plan_order(rl, rp, block, rf.RF_LIST_TEMPORAL_POSITION_MAJOR)
    assert sorted(order.tolist()) == list(range(len(row_ptr) - 1))


@pytest.mark.parametrize("lay", LAYOUTS)
@pytest.mark.parametrize("tau", [1, 2, 3])
@pytest.mark.parametrize("block", [64, 128, 256, 384])
def test_textural_lists(lay, tau, block):
    """Video-only query blocks walk the compacted key sequence; blocks holding text rows walk token space."""
    L, P = orc.Layout(*lay), orc.Params(0.25, 0.25, tau)
    rl, rp = rf.rf_layout(*lay), rf.rf_params(0.25, 0.25, tau, 0)
    N, Nv = orc.num_tokens(L), lay[0] * lay[1] * lay[2]
    nb = -(-N // block)
    M = orc.keep_matrix(orc.TEXTURAL, L, P)
    Nc = int(M[0].sum()) if Nv > 0 else N
    any_, full = brute_blocks(M, block)
    row_ptr, cols = rf.rf_plan_host(rl, rp, block, orc.TEXTURAL)
    for qb in range(nb):
        ent = cols[row_ptr[qb]:row_ptr[qb + 1]]
        kbs, partial = ent & ~rf.RF_PLAN_PARTIAL, (ent & rf.RF_PLAN_PARTIAL) != 0
        if lay[3] == 0 or qb < Nv // block:  # no text rows in the block (a ragged last block of video rows included)
            nct = -(-Nc // TILE)
            assert kbs.tolist() == list(range(nct))
            assert partial.tolist() == [(kt + 1) * TILE > Nc for kt in range(nct)]
        else:
            assert set(kbs.tolist()) == set(np.nonzero(any_[qb])[0].tolist())
            assert (partial == ~full[qb, kbs]).all()


@pytest.mark.parametrize("lay", [l for l in LAYOUTS if l[3] > 0])
@pytest.mark.parametrize("block", [64, 128])
def test_text_first_lists_are_over_the_video_first_order(lay, block):
    """With the text tokens in front, the kernel still walks video tokens first: row r of the walked
    order is tensor row  text_len + r  (video) or  r - Nv  (text).  The lists must match the oracle's
    text-first mask brought into that order, and the gather tables must hold tensor rows."""
    par = (0.25, 0.18, 3)
    L, P = orc.Layout(*lay), orc.Params(par[0], par[1], par[2], text_first=True)
    rl, rp = rf.rf_layout(*lay), rf.rf_params(par[0], par[1], par[2], 0, rf.RF_FLAG_TEXT_FIRST)
    N, (T, H, W, tl) = orc.num_tokens(L), lay
    Nv = T * H * W
    row_of = np.r_[np.arange(Nv) + tl, np.arange(tl)]
    for cls in (orc.SPATIAL, orc.TEMPORAL):
        any_, full = brute_blocks(orc.keep_matrix(cls, L, P)[np.ix_(row_of, row_of)], block)
        row_ptr, cols = rf.rf_plan_host(rl, rp, block, cls)
        for qb in range(len(row_ptr) - 1):
            ent = cols[row_ptr[qb]:row_ptr[qb + 1]]
            kbs, partial = ent & ~rf.RF_PLAN_PARTIAL, (ent & rf.RF_PLAN_PARTIAL) != 0
            assert set(kbs.tolist()) == set(np.nonzero(any_[qb])[0].tolist())
            assert (partial == ~full[qb, kbs]).all()
    tok = rf.rf_plan_position_major(rl, rp)
    plain = rf.rf_plan_position_major(rl)
    assert (tok == row_of[plain]).all() and sorted(tok.tolist()) == list(range(N))
    # the flag is inert without text tokens
    rl0 = rf.rf_layout(T, H, W, 0)
    a = rf.rf_plan_host(rl0, rp, block, orc.TEMPORAL)
    b = rf.rf_plan_host(rl0, rf.rf_params(par[0], par[1], par[2], 0), block, orc.TEMPORAL)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


@pytest.mark.parametrize("lay", LAYOUTS + [(33, 45, 80, 256), (13, 30, 45, 226)])
@pytest.mark.parametrize("block", [64, 128, 256, 384])
def test_query_block_order_is_a_permutation(lay, block):
    rl = rf.rf_layout(*lay)
    nqb = -(-(lay[0] * lay[1] * lay[2] + lay[3]) // block)
    for cls in (rf.RF_SPATIAL, rf.RF_TEMPORAL, rf.RF_TEXTURAL, rf.RF_DENSE):
        order = rf.rf_plan_order(rl, None, block, cls)
        assert sorted(order.tolist()) == list(range(nqb))
    n_video = lay[0] * lay[1] * lay[2] // block if lay[3] else nqb  # blocks without text rows
    want = np.r_[np.arange(n_video, nqb), np.arange(n_video)]       # text-holding blocks first, then token order
    assert (rf.rf_plan_order(rl, None, block, rf.RF_DENSE) == want).all()


def test_query_block_order_keeps_neighbours_together():
    """Text-holding blocks (the long items) lead the order; the XCD queues are eighths of the rest, where
    blocks next to each other must be neighbours in the sequence (token order, or position-grouped for
    Temporal in token order)."""
    rl = rf.rf_layout(33, 45, 80, 256)
    for block in (128, 256):
        n_video = 33 * 45 * 80 // block
        for cls in (rf.RF_SPATIAL, rf.RF_TEXTURAL, rf.RF_DENSE, rf.RF_LIST_TEMPORAL_POSITION_MAJOR, rf.RF_TEMPORAL):
            order, first = rf.rf_plan_order(rl, None, block, cls, full=True)
            n_text = len(order) - n_video
            assert n_text >= 1 and (order[:n_text] == np.arange(n_video, len(order))).all()
            if cls != rf.RF_TEMPORAL:
                assert (order[n_text:] == np.arange(n_video)).all()
            else:
                pos = (order[n_text:].astype(np.int64) * block) % (45 * 80) // block
                assert (np.diff(pos) >= 0).all()  # grouped by in-frame position
            work = np.diff(rf.rf_plan_host(rl, None, block, cls)[0])
            assert ((first >= 0) & (first < np.maximum(work, 1))).all()


@pytest.mark.parametrize("lay", [(7, 10, 13, 50), (33, 45, 80, 256)])
def test_blocks_of_a_generation_start_at_a_common_tile(lay):
    """Banded lists: the blocks an XCD runs together (32 blocks of 256 rows out of its eighth of the
    text-free part of the order) begin their cyclic walk at the same key tile wherever their lists hold it."""
    rl = rf.rf_layout(*lay)
    block = 256
    n_video = lay[0] * lay[1] * lay[2] // block
    for cls in (rf.RF_SPATIAL, rf.RF_LIST_TEMPORAL_POSITION_MAJOR):
        row_ptr, cols = rf.rf_plan_host(rl, None, block, cls)
        order, first = rf.rf_plan_order(rl, None, block, cls, full=True)
        tiles = cols & ~rf.RF_PLAN_PARTIAL
        rest = order[len(order) - n_video:]
        per = -(-n_video // 8)
        for s0 in range(0, n_video, per):
            for g0 in range(s0, min(s0 + per, n_video), 32):
                blocks = rest[g0:min(g0 + 32, s0 + per, n_video)]
                lo = max(tiles[row_ptr[b]] for b in blocks)
                for b in blocks:
                    mine = tiles[row_ptr[b]:row_ptr[b + 1]]
                    start = mine[first[b]]
                    assert start == lo if lo in mine else first[b] == 0 or start > lo
    # lists that are not one sliding range keep the plain walk
    _, first = rf.rf_plan_order(rl, None, block, rf.RF_TEMPORAL, full=True)
    assert (first == 0).all()


def test_paper_shapes_executed_fractions():
    """At the 720p shape with block 128 about half of the (block, tile) pairs are visited per pattern."""
    rl = rf.rf_layout(33, 45, 80, 256)
    for cls, lo, hi in ((rf.RF_SPATIAL, 0.44, 0.47), (rf.RF_TEMPORAL, 0.46, 0.50), (rf.RF_TEXTURAL, 0.49, 0.52)):
        vis, part, tot = rf.plan_block_counts(rl, None, 128, cls)
        assert lo < vis / tot < hi, (cls, vis / tot)
    vis, part, tot = rf.plan_block_counts(rl, None, 128, rf.RF_DENSE)
    assert vis == tot and part == 931  # only the ragged last tile of each query block


def test_every_declared_symbol_is_exported():
    lib = rf.load_library()
    hdr = open(os.path.join(ROOT, "include", "rainfusion.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = re.findall(r"\b(rf_[a-z_]+)\s*\(", hdr)
    assert set(names) >= {"rf_arm_classify", "rf_sparse_attention", "rf_arm_workspace_bytes", "rf_plan_host",
                          "rf_attention_workspace_bytes", "rf_plan_order", "rf_arm_classify_plus",
                          "rf_sparse_attention_plus", "rf_plan_position_major", "rf_arm_classify_noalloc",
                          "rf_plan_clear", "rf_status_string", "rf_version"}
    for n in set(names):
        assert getattr(lib, n) is not None
    assert rf.rf_version() >= 100
    assert rf.rf_status_string(0) == "ok" and "block" in rf.rf_status_string(-5)


def test_bad_arguments_are_rejected_before_any_gpu_work():
    lib = rf.load_library()
    L = rf.rf_layout(4, 8, 8, 0)
    one = C.c_void_p(16)  # non-null dummy; never dereferenced because validation fails first
    ok_p = rf.rf_params.default()

    def attn(Q=one, K=one, V=one, hc=one, B=1, nH=2, D=64, lay=L, par=ok_p, block=64, O=one, ws=None, wsb=0):
        return lib.rf_sparse_attention(Q, K, V, hc, B, nH, D, C.byref(lay) if lay else None,
                                       C.byref(par) if par else None, block, O, ws, wsb, None)

    assert attn(Q=None) == -1 and attn(O=None) == -1 and attn(hc=None) == -1 and attn(lay=None) == -1
    assert attn(D=80) == -2 and attn(B=0) == -2 and attn(nH=-1) == -2
    assert attn(lay=rf.rf_layout(0, 8, 8, 0)) == -3 and attn(lay=rf.rf_layout(4, 8, 8, -1)) == -3
    assert attn(lay=rf.rf_layout(4096, 4096, 4096, 0)) in (-2, -3)
    assert attn(par=rf.rf_params(1.5, 0.25, 2, 0)) == -4 and attn(par=rf.rf_params(0.25, -0.1, 2, 0)) == -4
    assert attn(par=rf.rf_params(0.25, 0.25, 2, 0, 32)) == -4  # unknown flag
    # 64-row wavefronts exist for head_dim 128 with 256-row blocks only
    wide = rf.rf_params(0.25, 0.25, 2, 0, rf.RF_FLAG_WIDE_ROWS)
    assert attn(par=wide, D=64, block=256) == -4 and attn(par=wide, D=128, block=128) == -4
    assert attn(par=wide, D=128, block=256, ws=None) == -6  # accepted up to the workspace check
    assert attn(par=rf.rf_params(0.25, 0.25, 0, 0)) == -4 and attn(par=rf.rf_params(float("nan"), 0.25, 2, 0)) == -4
    assert attn(block=32) == -5 and attn(block=512) == -5 and attn(block=0) == -5
    assert attn(block=384, ws=None) == -6 and attn(block=320) == -5  # 384 accepted up to the workspace check
    need = rf.rf_attention_workspace_bytes(1, 2, 64, L)
    # the work-queue counters, then a copy of K and of V: 2 heads x 256 tokens x 64 channels, bf16
    assert need == rf.RF_ATTENTION_MIN_WORKSPACE + 2 * 2 * 256 * 64 * 2
    # the workspace is required, holds at least the counters, and is 256-byte aligned
    assert attn(ws=None) == -6 and attn(ws=C.c_void_p(256), wsb=rf.RF_ATTENTION_MIN_WORKSPACE - 1) == -6
    assert attn(ws=C.c_void_p(264), wsb=need) == -8
    # tensors are moved 16 bytes at a time
    odd = C.c_void_p(24)
    assert attn(Q=odd) == -8 and attn(K=odd) == -8 and attn(V=odd) == -8 and attn(O=odd) == -8
    assert "align" in rf.rf_status_string(-8)
    assert rf.rf_attention_workspace_bytes(1, 2, 80, L) == 0

    def arm(Q=one, K=one, B=1, nH=2, D=64, lay=L, mode=0, thr=0.9, hc=one, ws=one, wsb=1 << 20):
        return lib.rf_arm_classify(Q, K, B, nH, D, C.byref(lay) if lay else None, None, mode, thr, hc, None, ws, wsb,
                                   None)

    assert arm(Q=None) == -1 and arm(hc=None) == -1
    assert arm(D=32) == -2
    assert arm(mode=2) == -4 and arm(thr=1.5) == -4 and arm(thr=float("nan")) == -4
    assert arm(ws=None) == -6 and arm(wsb=8) == -6
    assert arm(Q=C.c_void_p(8)) == -8 and arm(K=C.c_void_p(40)) == -8

    # the variant without a workspace: same checks, and problems beyond its static scratch are refused
    def armn(Q=one, K=one, B=1, nH=2, D=64, lay=L, mode=0, thr=0.9, hc=one):
        return lib.rf_arm_classify_noalloc(Q, K, B, nH, D, C.byref(lay) if lay else None, None, mode, thr, hc, None, None)

    assert armn(Q=None) == -1 and armn(hc=None) == -1 and armn(lay=None) == -1
    assert armn(D=32) == -2 and armn(mode=2) == -4 and armn(thr=1.5) == -4 and armn(Q=C.c_void_p(8)) == -8
    big_layout = rf.rf_layout(33, 45, 80, 256)  # 3600 sampled rows per pass
    assert rf.rf_arm_workspace_bytes(24, 3, big_layout) <= rf.RF_ARM_STATIC_SCRATCH_BYTES < rf.rf_arm_workspace_bytes(25, 3, big_layout)
    assert armn(B=25, nH=3, lay=big_layout) == -6
    assert rf.rf_arm_workspace_bytes(1, 2, L) == 1 * 2 * 2 * 64 * 4
    assert rf.rf_arm_workspace_bytes(0, 2, L) == 0
    # per-head bandwidth variants: candidate list checked on the host before anything else
    bw3, bad = (C.c_float * 3)(0.5, 0.25, 0.125), (C.c_float * 2)(0.5, 1.5)
    big = 1 << 20

    def armp(bws=bw3, n=3, hbw=one, hc=one):
        return lib.rf_arm_classify_plus(one, one, 1, 2, 64, C.byref(L), None, 0, 0.9, bws, n, hc, hbw, None, one, big, None)

    assert armp(bws=None) == -1 and armp(hbw=None) == -1 and armp(hc=None) == -1
    assert armp(n=0) == -4 and armp(n=5) == -4 and armp(bws=bad, n=2) == -4

    def attnp(bws=bw3, n=3, hbw=one):
        return lib.rf_sparse_attention_plus(one, one, one, one, hbw, bws, n, 1, 2, 64, C.byref(L), None, 64, one, None, 0,
                                            None)

    assert attnp(bws=None) == -1 and attnp(hbw=None) == -1 and attnp(n=9) == -4 and attnp(bws=bad, n=2) == -4
    needed = C.c_size_t(0)
    assert lib.rf_plan_host(C.byref(L), None, 64, 7, None, None, 0, C.byref(needed)) == -4
    assert lib.rf_plan_host(C.byref(L), None, 48, 0, None, None, 0, C.byref(needed)) == -5
    small = (C.c_int32 * 2)()
    assert lib.rf_plan_host(C.byref(L), None, 64, 0, None, small, 2, C.byref(needed)) == -6 and needed.value == 10


def test_bench_refuses_more_than_one_gpu_and_counts_kept_pairs():
    """bench.py --gpus N with N > 1 exits with a message (this build is one GPU); its FLOP bookkeeping
    (kept token pairs per pattern) matches a count over the oracle's mask on a small layout."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
    sys.path.insert(0, ROOT)
    import bench
    import rf_inputs as inp
    w = inp.Workload("count", 1, 1, 64, 5, 6, 11, 19, 64, 1)
    L = orc.Layout(w.T, w.H, w.W, w.text_len)
    for cls in (orc.SPATIAL, orc.TEMPORAL, orc.TEXTURAL, orc.DENSE):
        for bw, tau in ((0.25, 2), (0.13, 3)):
            want = int(orc.keep_matrix(cls, L, orc.Params(bw, bw, tau)).sum())
            assert bench.kept_pairs(cls, w, bw, bw, tau) == want, (cls, bw, tau)
