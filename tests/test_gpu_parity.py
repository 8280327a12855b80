"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded
inputs.  Small shapes are compared element by element on every row; the paper-sized shapes
on sampled rows the oracle computes one by one, plus properties that hold at any size.

Tolerances (bf16 inputs, fp32 accumulation, bf16 output): max-abs 2e-2 and mean-abs 2e-3, the
contract for this path.  Because i.i.d. inputs give outputs of only ~1e-2..1e-3 in size, the
relative L2 error is asserted as well: 5.2e-3, twice the largest value any case of this suite
prints (2.6e-3, the bf16 rounding of P and of O); peaky and planted inputs with larger outputs
are included.  ARM: recalls within 1e-3; classes exact unless a recall lies within 1e-3 of the
threshold (those heads are printed and exempt).
"""
import math

import numpy as np
import pytest
import torch

import oracle as orc
import paper_2505_21036_amd as rf
import rf_inputs as inp

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS, REL_L2 = 2e-2, 2e-3, 5.2e-3
DEV = "cuda:0"


def lay(w):
    return rf.rf_layout(w.T, w.H, w.W, w.text_len), orc.Layout(w.T, w.H, w.W, w.text_len)


def par(bs=0.25, bt=0.25, tau=2, omega=0, two_head=False):
    return (rf.rf_params(bs, bt, tau, omega, rf.RF_FLAG_TWO_HEAD if two_head else 0),
            orc.Params(bs, bt, tau, omega, two_head))


def f32(t):
    return t.float().numpy()


def check(O_gpu_rows, O_ref, what):
    got = O_gpu_rows.float().cpu().numpy().astype(np.float64)
    err = np.abs(got - O_ref)
    rel = np.linalg.norm(got - O_ref) / max(np.linalg.norm(O_ref), 1e-30)
    print("%s: max-abs %.3e mean-abs %.3e rel-L2 %.3e |ref|max %.3e" % (what, err.max(), err.mean(), rel,
                                                                       np.abs(O_ref).max()), flush=True)
    assert np.isfinite(got).all(), what
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, what
    assert rel <= REL_L2, what


def run_attention(w, Q, K, V, classes, block, params=None, packed=False):
    rl, _ = lay(w)
    hc = torch.as_tensor(classes, dtype=torch.int32).reshape(w.B, w.nH).to(DEV)
    ws = None
    if packed:  # Textural heads pack K_C, V_C, Temporal heads a position-major copy, into this workspace first
        ws = torch.empty(rf.rf_attention_workspace_bytes(w.B, w.nH, w.D, rl, params), dtype=torch.uint8, device=DEV)
    O = rf.rf_sparse_attention(Q, K, V, hc, rl, params, block, workspace=ws)
    torch.cuda.synchronize()
    return O


SMALL = ["tiny", "ragged64", "ragged96", "ragged128"]


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("block", [64, 128, 256, 384])
@pytest.mark.parametrize("scale", [1.0, 12.0])
def test_small_shapes_every_class_every_row(name, block, scale):
    w = inp.WORKLOADS[name]
    print("case", name, block, scale, flush=True)
    rp, op = par()
    _, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV, scale)
    for cls, packed in ((rf.RF_SPATIAL, False), (rf.RF_TEMPORAL, False), (rf.RF_TEMPORAL, True),
                        (rf.RF_TEXTURAL, False), (rf.RF_TEXTURAL, True), (rf.RF_DENSE, False)):
        O = run_attention(w, Q, K, V, [cls] * (w.B * w.nH), block, rp, packed)
        for b in range(w.B):
            for h in range(w.nH):
                q, k, v = (f32(t) for t in inp.head_qkv(w, b, h, scale))
                ref = orc.attention(q, k, v, cls, ol, op)
                check(O[b, h], ref, "%s blk%d scale%g cls%d packed%d head(%d,%d)" % (name, block, scale, cls, packed, b, h))


def test_tiny_config_forced_classes():
    """Head 0 Spatial, head 1 Temporal; then both Textural."""
    w = inp.WORKLOADS["tiny"]
    _, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV)
    for classes in ([rf.RF_SPATIAL, rf.RF_TEMPORAL], [rf.RF_TEXTURAL, rf.RF_TEXTURAL]):
        O = run_attention(w, Q, K, V, classes, 64)
        for h in range(2):
            q, k, v = (f32(t) for t in inp.head_qkv(w, 0, h))
            check(O[0, h], orc.attention(q, k, v, classes[h], ol), "tiny head %d cls %d" % (h, classes[h]))


@pytest.mark.parametrize("bs,bt,tau", [(0.0, 0.0, 1), (1.0, 1.0, 3), (0.13, 0.18, 4), (0.5, 0.125, 3)])
def test_parameter_corners(bs, bt, tau):
    w = inp.WORKLOADS["ragged128"]
    print("case corners", bs, bt, tau, flush=True)
    rp, op = par(bs, bt, tau)
    _, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV, 6.0)
    classes = inp.round_robin_classes(w).flatten().tolist()
    for block, packed in ((64, False), (128, False), (128, True), (256, True)):
        O = run_attention(w, Q, K, V, classes, block, rp, packed)
        for b in range(w.B):
            for h in range(w.nH):
                q, k, v = (f32(t) for t in inp.head_qkv(w, b, h, 6.0))
                ref = orc.attention(q, k, v, classes[b * w.nH + h], ol, op)
                check(O[b, h], ref, "corner bs%g bt%g tau%d blk%d packed%d head(%d,%d)" % (bs, bt, tau, block, packed, b, h))


@pytest.mark.parametrize("shape", [(1, 5, 5, 0), (1, 3, 3, 40), (2, 2, 2, 1), (3, 7, 9, 0)])
def test_degenerate_layouts(shape):
    """Fewer tokens than one block, mostly-text sequences, single frame."""
    T, H, W, tl = shape
    print("case degenerate", shape, flush=True)
    w = inp.Workload("deg", 1, 4, 64, T, H, W, tl, 64, 2000 + T * 100 + H)
    _, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV, 4.0)
    classes = [0, 1, 2, 3]
    for block in (64, 128):
        O = run_attention(w, Q, K, V, classes, block)
        for h in range(4):
            q, k, v = (f32(t) for t in inp.head_qkv(w, 0, h, 4.0))
            check(O[0, h], orc.attention(q, k, v, classes[h], ol), "deg %s blk%d cls%d" % (shape, block, h))


def test_out_of_range_class_runs_dense_and_constant_values_give_ones():
    w = inp.WORKLOADS["ragged96"]
    _, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV)
    O = run_attention(w, Q, K, V, [7, -1, 3], 128)
    for h in range(3):
        q, k, v = (f32(t) for t in inp.head_qkv(w, 0, h))
        check(O[0, h], orc.attention(q, k, v, orc.DENSE, ol), "class out of range head %d" % h)
    ones = torch.ones_like(V)
    for block in (64, 128):
        O = run_attention(w, Q, K, ones, [0, 1, 2], block)
        assert (O.float() - 1).abs().max().item() <= 1e-2


# ----------------------------------------------------------------------------- text tokens first, forced dense
@pytest.mark.parametrize("name", ["ragged64", "ragged96", "ragged128"])
@pytest.mark.parametrize("block", [64, 128, 256, 384])
def test_text_first_every_class_every_row(name, block):
    """The same heads with their text rows moved to the front and RF_FLAG_TEXT_FIRST set, against
    the oracle's text-first reading; attention for every class, packed or not, and the ARM."""
    w = inp.WORKLOADS[name]
    print("case text-first", name, block, flush=True)
    tl, scale = w.text_len, 6.0
    rl, ol = lay(w)
    rp, op = rf.rf_params(0.25, 0.25, 2, 0, rf.RF_FLAG_TEXT_FIRST), orc.Params(text_first=True)
    Q, K, V = (torch.roll(t, tl, dims=2).contiguous() for t in inp.full_qkv(w, DEV, scale))
    heads = {(b, h): [np.roll(f32(t), tl, axis=0) for t in inp.head_qkv(w, b, h, scale)]
             for b in range(w.B) for h in range(w.nH)}
    for cls, packed in ((rf.RF_SPATIAL, False), (rf.RF_TEMPORAL, False), (rf.RF_TEMPORAL, True),
                        (rf.RF_TEXTURAL, False), (rf.RF_TEXTURAL, True), (rf.RF_DENSE, False)):
        O = run_attention(w, Q, K, V, [cls] * (w.B * w.nH), block, rp, packed)
        for (b, h), (q, k, v) in heads.items():
            check(O[b, h], orc.attention(q, k, v, cls, ol, op),
                  "%s text-first blk%d cls%d packed%d head(%d,%d)" % (name, block, cls, packed, b, h))
    for mode in (rf.RF_SAMPLE_FIRST_FRAME, rf.RF_SAMPLE_EQUAL_INTERVAL):
        hc, rec = rf.rf_arm_classify(Q, K, rl, rp, mode, 0.5)
        hc, rec = hc.cpu().numpy(), rec.cpu().numpy()
        near = []
        for (b, h), (q, k, v) in heads.items():
            c, (rh, rt) = orc.arm_classify(q, k, ol, op, mode, 0.5)
            check_arm_head((b, h), hc[b, h], rec[b, h], c, rh, rt, 0.5, near)
        print("%s text-first mode %d: heads within 1e-3 of the threshold (exempt): %s" % (name, mode, near), flush=True)


def test_force_dense_flag_ignores_the_classes():
    w = inp.WORKLOADS["ragged128"]
    print("case force-dense", flush=True)
    rl, ol = lay(w)
    rp = rf.rf_params(0.25, 0.25, 2, 0, rf.RF_FLAG_FORCE_DENSE)
    Q, K, V = inp.full_qkv(w, DEV, 6.0)
    ws = torch.empty(rf.rf_attention_workspace_bytes(w.B, w.nH, w.D, rl, rp), dtype=torch.uint8, device=DEV)
    sparse_classes = torch.as_tensor(inp.round_robin_classes(w), dtype=torch.int32).to(DEV)
    for hc, workspace in ((None, None), (sparse_classes, None), (sparse_classes, ws)):
        O = rf.rf_sparse_attention(Q, K, V, hc, rl, rp, 128, workspace=workspace)
        torch.cuda.synchronize()
        for b in range(w.B):
            for h in range(w.nH):
                q, k, v = (f32(t) for t in inp.head_qkv(w, b, h, 6.0))
                check(O[b, h], orc.attention(q, k, v, orc.DENSE, ol), "force-dense head(%d,%d)" % (b, h))
    with pytest.raises(rf.RfError):  # without the flag the classes are required
        rf.rf_sparse_attention(Q, K, V, None, rl, None, 128)


# ----------------------------------------------------------------------------- ARM
def check_arm_head(what, got_class, got_recalls, want_class, rh, rt, alpha, near):
    """Recalls within 1e-3 of the oracle's; the class exact unless the recall that DECIDES it (Alg. 1:
    R-hat, or R-tilde once R-hat is below the threshold) lies within 1e-3 of the threshold; such heads
    are appended to `near` (the caller prints them) and exempt."""
    assert abs(got_recalls[0] - rh) <= 1e-3 and abs(got_recalls[1] - rt) <= 1e-3, (what, got_recalls, rh, rt)
    if abs(rh - alpha) < 1e-3 or (rh < alpha and abs(rt - alpha) < 1e-3):
        near.append((what, float(rh), float(rt)))
        return
    assert got_class == want_class, (what, got_class, want_class, rh, rt)


def arm_compare(w, Q, K, mode, alpha, rparams, oparams, heads=None):
    rl, ol = lay(w)
    hc, rec = rf.rf_arm_classify(Q, K, rl, rparams, mode, alpha)
    hc2, rec2 = rf.rf_arm_classify(Q, K, rl, rparams, mode, alpha)
    torch.cuda.synchronize()
    assert torch.equal(hc, hc2) and torch.equal(rec, rec2)  # fixed reduction order: bitwise repeatable
    hc, rec = hc.cpu().numpy(), rec.cpu().numpy()
    near = []
    for b in range(w.B):
        for h in range(w.nH):
            if heads is not None and (b, h) not in heads:
                continue
            q, k, _ = (f32(t) for t in inp.head_qkv(w, b, h))
            c, (rh, rt) = orc.arm_classify(q, k, ol, oparams, mode, alpha)
            check_arm_head((b, h), hc[b, h], rec[b, h], c, rh, rt, alpha, near)
    print("%s mode %d alpha %g: heads within 1e-3 of the threshold (exempt): %s" % (w.name, mode, alpha, near),
          flush=True)
    return hc, rec


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("mode", [rf.RF_SAMPLE_FIRST_FRAME, rf.RF_SAMPLE_EQUAL_INTERVAL])
def test_arm_small_shapes(name, mode):
    w = inp.WORKLOADS[name]
    print("case arm", name, mode, flush=True)
    Q, K, _ = inp.full_qkv(w, DEV)
    for alpha in (0.3, 0.5, 0.9):
        arm_compare(w, Q, K, mode, alpha, *par())
    arm_compare(w, Q, K, mode, 0.5, *par(0.1, 0.4, 2, 3))  # other bandwidths, sampling interval 3
    hc, _ = arm_compare(w, Q, K, mode, 0.9, *par(two_head=True))  # i.i.d. heads match no mask at 0.9
    assert (hc == rf.RF_DENSE).all()


def test_arm_recovers_planted_structure():
    w = inp.WORKLOADS["planted"]
    print("case arm planted", flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    hc, rec = arm_compare(w, Q, K, rf.RF_SAMPLE_FIRST_FRAME, 0.9, *par())
    for b in range(w.B):
        for h in range(w.nH):
            assert hc[b, h] == inp.planted_class(w, b, h), (b, h, rec[b, h])
    # attention with the ARM-chosen classes, O(1) outputs, both block sizes, sampled rows
    _, ol = lay(w)
    rows = np.array(inp.sample_rows(w, 24))
    for block in (64, 128):
        O = run_attention(w, Q, K, V, hc.flatten().tolist(), block)
        for (b, h) in ((0, 0), (0, 1), (0, 2), (1, 7), (1, 15)):
            q, k, v = (f32(t) for t in inp.head_qkv(w, b, h))
            ref = orc.attention_rows(q, k, v, int(hc[b, h]), ol, orc.Params(), rows)
            check(O[b, h][torch.as_tensor(rows, device=DEV)], ref, "planted blk%d head(%d,%d) cls%d" % (block, b, h, hc[b, h]))


# ----------------------------------------------------------------------------- RainFusion+ (per-head bandwidth)
BWS = [0.5, 0.25, 0.125]


def plus_compare(w, Q, K, V, mode, alpha, bws, block, rows=None, heads=None):
    """ARM with candidate bandwidths, then attention with the per-head bandwidth it chose."""
    rl, ol = lay(w)
    hc, hbw, rec = rf.rf_arm_classify_plus(Q, K, rl, None, mode, alpha, bws)
    O = rf.rf_sparse_attention_plus(Q, K, V, hc, hbw, bws, rl, None, block)
    torch.cuda.synchronize()
    hc, hbw, rec = hc.cpu().numpy(), hbw.cpu().numpy(), rec.cpu().numpy()
    near = []
    for b in range(w.B):
        for h in range(w.nH):
            if heads is not None and (b, h) not in heads:
                continue
            q, k, v = (f32(t) for t in inp.head_qkv(w, b, h))
            c, idx, orec = orc.arm_classify_plus(q, k, ol, orc.Params(), mode, alpha, bws)
            assert np.abs(rec[b, h] - orec).max() <= 1e-3, (b, h, rec[b, h], orec)
            if np.abs(orec - alpha).min() < 1e-3:
                near.append((b, h))
            else:
                assert (hc[b, h], hbw[b, h]) == (c, idx), (b, h, hc[b, h], hbw[b, h], c, idx, orec)
            # the attention is checked with whatever the GPU chose, so near-threshold heads are covered too
            bw = bws[hbw[b, h]] if hbw[b, h] >= 0 else 0.25
            r = np.arange(w.N) if rows is None else rows
            ref = orc.attention_rows(q, k, v, int(hc[b, h]), ol, orc.Params(bw, bw, 2), r)
            check(O[b, h][torch.as_tensor(r, device=DEV)], ref,
                  "%s plus blk%d head(%d,%d) cls%d bw%g" % (w.name, block, b, h, hc[b, h], bw))
    print("%s plus alpha %g: heads within 1e-3 of the threshold (exempt from class check): %s" % (w.name, alpha, near),
          flush=True)
    return hc, hbw, rec


@pytest.mark.parametrize("name", ["tiny", "ragged64", "ragged96", "ragged128"])
def test_plus_small_shapes(name):
    w = inp.WORKLOADS[name]
    print("case plus", name, flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    for alpha in (0.3, 0.45, 0.8):  # i.i.d. heads: recalls ~ mask area, so these thresholds exercise every outcome
        for mode in (rf.RF_SAMPLE_FIRST_FRAME, rf.RF_SAMPLE_EQUAL_INTERVAL):
            plus_compare(w, Q, K, V, mode, alpha, BWS, 64 if name == "tiny" else 128)
    plus_compare(w, Q, K, V, rf.RF_SAMPLE_FIRST_FRAME, 0.45, [0.125, 0.5], 64)  # unsorted, two candidates


def test_plus_planted_structure_gets_the_narrowest_band():
    w = inp.WORKLOADS["planted"]
    print("case plus planted", flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    rows = np.array(inp.sample_rows(w, 24))
    heads = {(0, 0), (0, 1), (0, 2), (1, 5), (1, 15)}
    hc, hbw, rec = plus_compare(w, Q, K, V, rf.RF_SAMPLE_FIRST_FRAME, 0.9, BWS, 128, rows, heads)
    for b in range(w.B):
        for h in range(w.nH):
            cls = inp.planted_class(w, b, h)
            assert hc[b, h] == cls
            # the planted structure sits well inside even the narrowest band
            assert hbw[b, h] == (-1 if cls == rf.RF_TEXTURAL else 2), (b, h, rec[b, h])


@pytest.mark.parametrize("text_first", [False, True])
def test_plus_attention_with_a_workspace_and_two_bandwidths_per_pattern(text_first):
    """rf_sparse_attention_plus with the full workspace: Temporal heads walk position-major copies with
    the list of THEIR bandwidth, Textural heads the packed K_C/V_C; heads of one pattern at different
    bandwidths in one call, text tokens behind or in front."""
    w = inp.WORKLOADS["ragged128"]
    print("case plus workspace", text_first, flush=True)
    rl, ol = lay(w)
    tl, scale = w.text_len, 5.0
    shift = tl if text_first else 0
    rp = rf.rf_params(0.25, 0.25, 2, 0, rf.RF_FLAG_TEXT_FIRST if text_first else 0)
    Q, K, V = (torch.roll(t, shift, dims=2).contiguous() for t in inp.full_qkv(w, DEV, scale))
    bws = [0.5, 0.25, 0.125]
    classes = [rf.RF_TEMPORAL, rf.RF_TEMPORAL, rf.RF_SPATIAL, rf.RF_SPATIAL, rf.RF_TEXTURAL, rf.RF_TEMPORAL]
    chosen = [0, 2, 1, 2, -1, 1]
    hc = torch.as_tensor(classes, dtype=torch.int32).reshape(w.B, w.nH).to(DEV)
    hbw = torch.as_tensor(chosen, dtype=torch.int32).reshape(w.B, w.nH).to(DEV)
    ws = torch.empty(rf.rf_attention_workspace_bytes(w.B, w.nH, w.D, rl, rp), dtype=torch.uint8, device=DEV)
    rp_wide = rf.rf_params(0.25, 0.25, 2, 0, rp.flags | rf.RF_FLAG_WIDE_ROWS)  # the 64-row loop with a list per head
    for block, params in ((64, rp), (128, rp), (256, rp), (256, rp_wide)):
        for workspace in (ws, None):
            O = rf.rf_sparse_attention_plus(Q, K, V, hc, hbw, bws, rl, params, block, workspace=workspace)
            torch.cuda.synchronize()
            for b in range(w.B):
                for h in range(w.nH):
                    i = b * w.nH + h
                    bw = bws[chosen[i]] if chosen[i] >= 0 else 0.25
                    q, k, v = (np.roll(f32(t), shift, axis=0) for t in inp.head_qkv(w, b, h, scale))
                    ref = orc.attention(q, k, v, classes[i], ol, orc.Params(bw, bw, 2, 0, False, text_first))
                    check(O[b, h], ref, "plus ws%d text-first%d blk%d head(%d,%d) cls%d bw%g" % (
                        workspace is not None, text_first, block, b, h, classes[i], bw))


# ----------------------------------------------------------------------------- paper-sized layers
def sampled_parity(w, O, classes, heads, per_head, params=orc.Params(), tag=""):
    _, ol = lay(w)
    rows = np.array(inp.sample_rows(w, per_head))
    rows_dev = torch.as_tensor(rows, device=DEV)
    for (b, h) in heads:
        q, k, v = (f32(t) for t in inp.head_qkv(w, b, h))
        ref = orc.attention_rows(q, k, v, int(classes[b * w.nH + h]), ol, params, rows)
        check(O[b, h][rows_dev], ref, "%s %s head(%d,%d) cls%d" % (w.name, tag, b, h, classes[b * w.nH + h]))


def test_cogvideox_layer():
    w = inp.WORKLOADS["cogvideox"]
    print("case cogvideox", flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    classes = inp.round_robin_classes(w).flatten().tolist()
    O = run_attention(w, Q, K, V, classes, w.block)
    sampled_parity(w, O, classes, [(0, h) for h in (0, 1, 2, 10, 23, 47)], 40, tag="round-robin")
    other = 64 if w.block == 128 else 128
    Oo = run_attention(w, Q, K, V, classes, other)
    sampled_parity(w, Oo, classes, [(0, h) for h in (3, 4, 5)], 40, tag="round-robin blk%d" % other)
    # ARM-chosen classes, equal-interval sampling; i.i.d. heads have near-uniform attention -> Textural
    hc, rec = arm_compare(w, Q, K, rf.RF_SAMPLE_EQUAL_INTERVAL, 0.9, *par(), heads={(0, 0), (0, 17), (0, 47)})
    assert (hc == rf.RF_TEXTURAL).all()
    O = run_attention(w, Q, K, V, hc.flatten().tolist(), w.block)
    sampled_parity(w, O, hc.flatten().tolist(), [(0, 5), (0, 30)], 40, tag="arm-chosen")


def test_osp720p_layer_sparse_and_dense():
    w = inp.WORKLOADS["osp720p"]
    print("case osp720p", flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    classes = inp.thirds_classes(w).flatten().tolist()
    O = run_attention(w, Q, K, V, classes, w.block)
    sampled_parity(w, O, classes, [(0, 0), (0, 9), (0, 23)], 20, tag="thirds")
    O = run_attention(w, Q, K, V, classes, 128, packed=True)  # the block size the configuration names
    sampled_parity(w, O, classes, [(0, 1), (0, 10), (0, 22)], 20, tag="thirds, packed, block 128")
    O = run_attention(w, Q, K, V, classes, 256, packed=True)
    sampled_parity(w, O, classes, [(0, 2), (0, 12), (0, 19)], 12, tag="thirds, packed, block 256")
    dense = [rf.RF_DENSE] * w.nH
    O = run_attention(w, Q, K, V, dense, w.block)
    sampled_parity(w, O, dense, [(0, 11)], 12, tag="dense")


def test_hunyuan720p_headline_layer():
    """ARM on first-frame samples, then sparse attention, in the configuration bench.py times."""
    w = inp.WORKLOADS["hunyuan720p"]
    print("case hunyuan720p", flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    hc, rec = arm_compare(w, Q, K, rf.RF_SAMPLE_FIRST_FRAME, 0.9, *par(), heads={(0, 0), (0, 13)})
    assert (hc == rf.RF_TEXTURAL).all()  # i.i.d. inputs: recalls ~ mask area < 0.9
    classes = inp.thirds_classes(w).flatten().tolist()
    O = run_attention(w, Q, K, V, classes, w.block)
    sampled_parity(w, O, classes, [(0, 0), (0, 8), (0, 16)], 20, tag="thirds")
    O = run_attention(w, Q, K, V, classes, w.block, packed=True)
    sampled_parity(w, O, classes, [(0, 9), (0, 15), (0, 17)], 20, tag="thirds, packed")
    O = run_attention(w, Q, K, V, classes, 128, packed=True)
    sampled_parity(w, O, classes, [(0, 1), (0, 10), (0, 20)], 20, tag="thirds, packed, block 128")
    O = run_attention(w, Q, K, V, classes, 256, packed=True)
    sampled_parity(w, O, classes, [(0, 2), (0, 11), (0, 21)], 12, tag="thirds, packed, block 256")
    O = run_attention(w, Q, K, V, hc.flatten().tolist(), w.block, packed=True)  # as bench.py runs it
    sampled_parity(w, O, hc.flatten().tolist(), [(0, 5)], 12, tag="arm-chosen, packed")
    O = run_attention(w, Q, K, V, hc.flatten().tolist(), w.block)
    sampled_parity(w, O, hc.flatten().tolist(), [(0, 6)], 12, tag="arm-chosen, gathered")
    # property at full size: constant values must come back as that constant on every row
    O = run_attention(w, Q, K, torch.ones_like(V), classes, w.block)
    assert (O.float() - 1).abs().max().item() <= 1e-2


def test_hunyuan720p_planted_layer_arm_picks_all_three_patterns():
    """The headline shape with planted heads: the ARM must return the planted class for every head
    (Alg. 1 -> Eq. 3-5 on the device, all three list walks in one launch), equal to the oracle's on two
    heads per class, and the attention with those classes, run as bench.py runs it, must match the
    oracle on sampled rows."""
    w = inp.WORKLOADS["hunyuan720p_planted"]
    print("case hunyuan720p planted", flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    heads = [(0, 0), (0, 1), (0, 2), (0, 9), (0, 16), (0, 23)]
    hc, rec = arm_compare(w, Q, K, rf.RF_SAMPLE_FIRST_FRAME, 0.9, *par(), heads=set(heads))
    for h in range(w.nH):
        assert hc[0, h] == inp.planted_class(w, 0, h), (h, rec[0, h])
    classes = hc.flatten().tolist()
    O = run_attention(w, Q, K, V, classes, w.block, packed=True)
    sampled_parity(w, O, classes, heads, 16, tag="planted, arm-chosen, packed")
    O = run_attention(w, Q, K, V, classes, 128)
    sampled_parity(w, O, classes, [(0, 3), (0, 4), (0, 5)], 16, tag="planted, arm-chosen, block 128, no copies")


# ----------------------------------------------------------------------------- 64 query rows per wavefront
@pytest.mark.parametrize("scale", [1.0, 12.0])
@pytest.mark.parametrize("text_first", [False, True])
def test_wide_rows_variant_every_class_every_row(scale, text_first):
    """RF_FLAG_WIDE_ROWS (a wavefront owns 64 query rows, software-pipelined tile loop): every class,
    gathered and packed, all rows of a ragged head_dim-128 shape (text rows, a ragged last block and
    a ragged last key tile), also with the text rows first."""
    w = inp.WORKLOADS["ragged128"]
    print("case wide rows", scale, text_first, flush=True)
    tl = w.text_len if text_first else 0
    _, ol = lay(w)
    rp = rf.rf_params(0.25, 0.25, 2, 0, rf.RF_FLAG_WIDE_ROWS | (rf.RF_FLAG_TEXT_FIRST if text_first else 0))
    op = orc.Params(text_first=text_first)
    Q, K, V = (torch.roll(t, tl, dims=2).contiguous() for t in inp.full_qkv(w, DEV, scale))
    heads = {(b, h): [np.roll(f32(t), tl, axis=0) for t in inp.head_qkv(w, b, h, scale)]
             for b in range(w.B) for h in range(w.nH)}
    for cls, packed in ((rf.RF_SPATIAL, False), (rf.RF_TEMPORAL, False), (rf.RF_TEMPORAL, True),
                        (rf.RF_TEXTURAL, False), (rf.RF_TEXTURAL, True), (rf.RF_DENSE, False)):
        O = run_attention(w, Q, K, V, [cls] * (w.B * w.nH), 256, rp, packed)
        for (b, h), (q, k, v) in heads.items():
            check(O[b, h], orc.attention(q, k, v, cls, ol, op),
                  "wide rows scale%g text-first%d cls%d packed%d head(%d,%d)" % (scale, text_first, cls, packed, b, h))


def test_wide_rows_variant_at_the_headline_shape():
    """The same variant on the planted heads of the headline shape, classes mixed in one launch, as
    `bench.py --wide-rows` runs it: sampled rows against the oracle."""
    w = inp.WORKLOADS["hunyuan720p_planted"]
    print("case wide rows, hunyuan720p planted", flush=True)
    Q, K, V = inp.full_qkv(w, DEV)
    classes = [inp.planted_class(w, 0, h) for h in range(w.nH)]
    rp = rf.rf_params(0.25, 0.25, 2, 0, rf.RF_FLAG_WIDE_ROWS)
    O = run_attention(w, Q, K, V, classes, 256, rp, packed=True)
    sampled_parity(w, O, classes, [(0, 0), (0, 1), (0, 2)], 16, tag="wide rows, planted classes, packed")
    O = run_attention(w, Q, K, V, [rf.RF_DENSE] * w.nH, 256, rp)
    sampled_parity(w, O, [rf.RF_DENSE] * w.nH, [(0, 7)], 8, tag="wide rows, dense")


# ----------------------------------------------------------------------------- graphs and streams
def test_step_replays_from_a_hip_graph():
    """ARM + attention captured once (after a warm-up call has built the block lists) and replayed
    with other work and synchronisations in between; every replay must reproduce the eager result
    for whatever the input buffers hold at that moment."""
    w = inp.WORKLOADS["ragged128"]
    print("case graph", flush=True)
    rl, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV, 6.0)
    ws = torch.empty(rf.rf_attention_workspace_bytes(w.B, w.nH, w.D, rl, None), dtype=torch.uint8, device=DEV)
    arm_ws = torch.empty(rf.rf_arm_workspace_bytes(w.B, w.nH, rl), dtype=torch.uint8, device=DEV)
    hc = torch.empty(w.B, w.nH, dtype=torch.int32, device=DEV)
    rec = torch.empty(w.B, w.nH, 2, dtype=torch.float32, device=DEV)
    O = torch.empty_like(Q)

    fixed = rf.rf_params(0.25, 0.25, 2, 0, rf.RF_FLAG_FIXED_ORDER)  # bitwise reproducible attention

    def step():
        rf.rf_arm_classify(Q, K, rl, None, rf.RF_SAMPLE_FIRST_FRAME, 0.45, hc, rec, arm_ws)
        rf.rf_sparse_attention(Q, K, V, hc, rl, fixed, 128, out=O, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up: builds and uploads the lists, sets kernel attributes
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    for trial, scale in enumerate((6.0, 1.0, 9.0)):
        fresh = inp.full_qkv(w, DEV, scale)
        for dst, src in zip((Q, K, V), fresh):
            dst.copy_(src)
        O.zero_()
        hc.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        O_graph, hc_graph = O.clone(), hc.clone()
        junk = (Q.float() @ K.float().transpose(-1, -2)).sum()  # unrelated eager work between replays
        step()
        torch.cuda.synchronize()
        assert torch.equal(hc_graph, hc), trial
        assert torch.equal(O_graph, O), (trial, float(junk))  # same kernels, same order of work per row
        for b in range(w.B):
            for h in range(w.nH):
                q, k, v = (f32(t) for t in inp.head_qkv(w, b, h, scale))
                check(O_graph[b, h], orc.attention(q, k, v, int(hc_graph[b, h]), ol), "graph replay %d head(%d,%d)" % (trial, b, h))


def test_many_calls_on_three_streams_and_a_replayed_graph():
    """The work-queue counters live in each call's own workspace, so any number of calls may be in
    flight: 72 launches over three streams (each stream with its own workspace and output) while a
    captured graph with a fourth workspace is replayed in between; every output against the oracle."""
    w = inp.WORKLOADS["ragged96"]
    print("case many streams", flush=True)
    rl, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV, 6.0)
    kinds = (rf.RF_TEMPORAL, rf.RF_TEXTURAL, rf.RF_SPATIAL, rf.RF_DENSE)
    classes = [torch.full((w.B, w.nH), c, dtype=torch.int32, device=DEV) for c in kinds]
    full = rf.rf_attention_workspace_bytes(w.B, w.nH, w.D, rl, None)
    # two full workspaces (packed copies), one with the counters only, one full for the graph
    wss = [torch.empty(n, dtype=torch.uint8, device=DEV) for n in (full, rf.RF_ATTENTION_MIN_WORKSPACE, full, full)]
    outs = [torch.empty_like(Q) for _ in range(4)]
    blocks = (64, 384, 256, 128)
    for i in range(4):  # lists built, kernel attributes set
        rf.rf_sparse_attention(Q, K, V, classes[i], rl, None, blocks[i], out=outs[i], workspace=wss[i])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        rf.rf_sparse_attention(Q, K, V, classes[3], rl, None, blocks[3], out=outs[3], workspace=wss[3])
    torch.cuda.synchronize()
    for o in outs:
        o.zero_()
    streams = [torch.cuda.Stream() for _ in range(3)]
    for rep in range(24):
        for i, s in enumerate(streams):
            with torch.cuda.stream(s):
                rf.rf_sparse_attention(Q, K, V, classes[i], rl, None, blocks[i], out=outs[i], workspace=wss[i])
        if rep % 4 == 0:
            graph.replay()
    torch.cuda.synchronize()
    for i, cls in enumerate(kinds):
        for h in range(w.nH):
            q, k, v = (f32(t) for t in inp.head_qkv(w, 0, h, 6.0))
            check(outs[i][0, h], orc.attention(q, k, v, cls, ol), "stream %d head %d" % (i, h))


@pytest.mark.parametrize("shape", [(3, 5, 64, 3, 7, 9, 33), (1, 7, 96, 9, 8, 8, 0), (2, 9, 128, 2, 16, 17, 300), (5, 1, 64, 11, 5, 5, 7)])
def test_odd_batch_and_head_counts_through_the_queues(shape):
    """Head counts that are not multiples of 8, fewer query blocks than XCDs, more text than video:
    every (head, block) item must be processed exactly once whatever the queue shapes are."""
    B, nH, D, T, H, W, tl = shape
    print("case queues", shape, flush=True)
    w = inp.Workload("odd", B, nH, D, T, H, W, tl, 64, 3000 + B * 17 + nH)
    _, ol = lay(w)
    Q, K, V = inp.full_qkv(w, DEV, 5.0)
    classes = [(b * nH + h) % 4 for b in range(B) for h in range(nH)]
    for block, packed in ((64, False), (128, True), (256, True)):
        O = run_attention(w, Q, K, V, classes, block, packed=packed)
        for b in range(B):
            for h in range(nH):
                q, k, v = (f32(t) for t in inp.head_qkv(w, b, h, 5.0))
                check(O[b, h], orc.attention(q, k, v, classes[b * nH + h], ol), "odd %s blk%d head(%d,%d)" % (shape, block, b, h))


def test_random_small_configurations():
    """Seeded sweep over layouts, parameters, flags, blocks and class mixes that the hand-picked cases
    do not name: every head of every configuration against the oracle."""
    rng = np.random.default_rng(20250521)
    for case in range(28):
        T, H, W = int(rng.integers(1, 9)), int(rng.integers(1, 13)), int(rng.integers(1, 13))
        tl = int(rng.choice([0, 0, 1, 17, 64, 100, 200]))
        D = int(rng.choice([64, 96, 128]))
        B, nH = int(rng.integers(1, 3)), int(rng.integers(1, 6))
        bs, bt = float(rng.choice([0.0, 0.07, 0.25, 0.5, 1.0])), float(rng.choice([0.0, 0.03, 0.25, 0.6, 1.0]))
        tau = int(rng.integers(1, 6))
        block = int(rng.choice([64, 128, 256, 384]))
        packed, text_first = bool(rng.integers(0, 2)), bool(rng.integers(0, 2)) and tl > 0
        scale = float(rng.choice([1.0, 4.0, 10.0]))
        w = inp.Workload("rand%d" % case, B, nH, D, T, H, W, tl, block, 5000 + case)
        print("case random", case, (B, nH, D, T, H, W, tl), (bs, bt, tau), block, packed, text_first, scale, flush=True)
        rl, ol = lay(w)
        rp = rf.rf_params(bs, bt, tau, 0, rf.RF_FLAG_TEXT_FIRST if text_first else 0)
        op = orc.Params(bs, bt, tau, 0, False, text_first)
        shift = tl if text_first else 0
        Q, K, V = (torch.roll(t, shift, dims=2).contiguous() for t in inp.full_qkv(w, DEV, scale))
        classes = [int(c) for c in rng.integers(0, 4, size=B * nH)]
        O = run_attention(w, Q, K, V, classes, block, rp, packed)
        for b in range(B):
            for h in range(nH):
                q, k, v = (np.roll(f32(t), shift, axis=0) for t in inp.head_qkv(w, b, h, scale))
                check(O[b, h], orc.attention(q, k, v, classes[b * nH + h], ol, op),
                      "random %d head(%d,%d) cls%d" % (case, b, h, classes[b * nH + h]))


def test_random_small_arm_configurations():
    """Seeded sweep of the ARM: layouts, bandwidths, sampling intervals and modes, text in front or behind,
    one or several candidate bandwidths; recalls within 1e-3 of the oracle, classes exact away from the threshold."""
    rng = np.random.default_rng(60521)
    for case in range(16):
        T, H, W = int(rng.integers(1, 9)), int(rng.integers(2, 13)), int(rng.integers(2, 13))
        tl = int(rng.choice([0, 5, 64, 130]))
        D = int(rng.choice([64, 96, 128]))
        B, nH = 1, int(rng.integers(1, 5))
        bs, bt = float(rng.choice([0.0, 0.1, 0.25, 0.5])), float(rng.choice([0.0, 0.05, 0.25, 0.5]))
        omega = int(rng.choice([0, 1, 2, 3, 7]))
        mode = int(rng.integers(0, 2))
        alpha = float(rng.choice([0.3, 0.5, 0.7]))
        text_first = bool(rng.integers(0, 2)) and tl > 0
        w = inp.Workload("rarm%d" % case, B, nH, D, T, H, W, tl, 64, 7000 + case)
        print("case random arm", case, (nH, D, T, H, W, tl), (bs, bt, omega), mode, alpha, text_first, flush=True)
        rl, ol = lay(w)
        rp = rf.rf_params(bs, bt, 2, omega, rf.RF_FLAG_TEXT_FIRST if text_first else 0)
        op = orc.Params(bs, bt, 2, omega, False, text_first)
        shift = tl if text_first else 0
        Q, K, _ = (torch.roll(t, shift, dims=2).contiguous() for t in inp.full_qkv(w, DEV, 3.0))
        hc, rec = rf.rf_arm_classify(Q, K, rl, rp, mode, alpha)
        hc, rec = hc.cpu().numpy(), rec.cpu().numpy()
        bws = [0.5, 0.125, 0.25]
        hcp, hbw, recp = (t.cpu().numpy() for t in rf.rf_arm_classify_plus(Q, K, rl, rp, mode, alpha, bws))
        near = []
        for h in range(nH):
            q, k, _ = (np.roll(f32(t), shift, axis=0) for t in inp.head_qkv(w, 0, h, 3.0))
            c, (rh, rt) = orc.arm_classify(q, k, ol, op, mode, alpha)
            check_arm_head((case, h), hc[0, h], rec[0, h], c, rh, rt, alpha, near)
            cp, idx, orec = orc.arm_classify_plus(q, k, ol, op, mode, alpha, bws)
            assert np.abs(recp[0, h] - orec).max() <= 1e-3, (case, h, recp[0, h], orec)
            if np.abs(orec - alpha).min() >= 1e-3:
                assert (hcp[0, h], hbw[0, h]) == (cp, idx), (case, h, hcp[0, h], hbw[0, h], cp, idx)
            else:
                near.append(((case, h, "plus"), orec.round(4).tolist()))
        print("random arm case %d: heads within 1e-3 of the threshold (exempt): %s" % (case, near), flush=True)
