"""Host-side checks of the index arithmetic and of the three-term split the HIP kernels rely on.

Nothing here touches the GPU or the oracle: the formulas are restated in numpy and checked for
the properties the kernels need (bijections, bank spreading, exactness of the split and the size
of what it drops).  A kernel that used another formula would fail its parity test; these tests
say WHY the formulas are safe to use."""
import numpy as np
import pytest

from workloads import round_to_bf16


# ------------------------------------------------------------------ LDS rows: bank spreading
# A ds_read_b128 serves 16 lanes together; they read the same logical 16-byte piece c of 16
# consecutive rows.  LDS has 64 banks of 4 bytes = 16 groups of 16 bytes: the 16 reads must fall in
# 16 different groups.  Physical piece index of (row, c):
LAYOUTS = {
    "128-byte rows, c ^ ((r >> 1) & 7)": (8, lambda r, c: c ^ ((r >> 1) & 7)),          # tiled kernels
    "128-byte rows of 1 KB words, c ^ (r & 15)": (64, lambda r, c: c ^ (r & 15)),       # staged kernel (Hp = 512)
    "192-byte rows, (c + ((r >> 2) & 3)) % 12": (12, lambda r, c: (c + ((r >> 2) & 3)) % 12),   # three-term kernel
}


@pytest.mark.parametrize("name", list(LAYOUTS))
def test_lds_row_layout_is_a_bijection_and_conflict_free(name):
    pieces, pos = LAYOUTS[name]
    swizzled = min(pieces, 16)          # only the low bits of the piece index take part
    for r in range(64):
        assert sorted(pos(r, c) for c in range(swizzled)) == list(range(swizzled)), (name, r)
    for base in range(0, 64, 16):
        for c in range(swizzled):
            groups = {(pieces * r + pos(r, c)) % 16 for r in range(base, base + 16)}
            assert len(groups) == 16, (name, base, c)


def test_direct_load_side_inverts_the_rotation():
    """The direct global->LDS loads write LDS linearly, so lane i must fetch the logical piece that
    belongs at physical position i: the inverse map used by the loaders."""
    for r in range(64):
        for p in range(12):
            c = (p + 12 - ((r >> 2) & 3)) % 12
            assert (c + ((r >> 2) & 3)) % 12 == p
        for p in range(8):
            c = p ^ ((r >> 1) & 7)
            assert c ^ ((r >> 1) & 7) == p


# ------------------------------------------------------------------ MFMA-operand ("fragment") order
def frag_index(row, unit, KS):
    """Element index of (row, unit) in [rows / 32][KS][64 lanes][8]: lane 32 g + c of fragment
    (rb, ks) holds row 32 rb + c, units 16 ks + 8 g .. + 7."""
    rb, c = divmod(row, 32)
    ks, rest = divmod(unit, 16)
    g, e = divmod(rest, 8)
    return ((rb * KS + ks) * 64 + 32 * g + c) * 8 + e


@pytest.mark.parametrize("rows,H", [(32, 64), (64, 128), (96, 512)])
def test_fragment_order_is_a_bijection(rows, H):
    KS = H // 16
    idx = np.array([[frag_index(r, u, KS) for u in range(H)] for r in range(rows)])
    assert sorted(idx.ravel().tolist()) == list(range(rows * H))
    # one operand of a wave (fixed row block and k-step) is 1 KB contiguous
    block = idx[:32, :16].ravel()
    assert block.min() == 0 and block.max() == 511


def test_term_interleaved_layout_is_a_bijection():
    """[row][unit / 32][term][unit % 32]: a chunk of 32 units is 96 contiguous elements per row."""
    H = 128
    idx = sorted(((u >> 5) * 96 + t * 32 + (u & 31)) for u in range(H) for t in range(3))
    assert idx == list(range(3 * H))


# ------------------------------------------------------------------ three-term bf16 split
def split3(x):
    x = x.astype(np.float32)
    x1 = round_to_bf16(x)
    r1 = (x - x1).astype(np.float32)
    x2 = round_to_bf16(r1)
    r2 = (r1 - x2).astype(np.float32)
    x3 = round_to_bf16(r2)
    return x1, x2, x3


def test_three_bf16_terms_add_up_to_the_fp32_number_exactly():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e-3, 20000), rng.uniform(-0.5, 0.5, 20000),
                        np.array([0.0, 1.0, -1.0, 0.5, 2.0 ** -20, 1.0 + 2.0 ** -23, 1e30, 1.2e-30])]).astype(np.float32)
    # (holds up to the largest finite bf16; a number that rounds to infinity as bf16 is no weight)
    x1, x2, x3 = split3(x)
    total = x1.astype(np.float64) + x2.astype(np.float64) + x3.astype(np.float64)
    assert np.array_equal(total, x.astype(np.float64))
    # each term is at most half a unit in the last place of the one before it
    big = np.abs(x) > 1e-30
    assert np.all(np.abs(x2[big]) <= np.abs(x1[big]) * 2.0 ** -8)
    assert np.all(np.abs(x3[big]) <= np.abs(x1[big]) * 2.0 ** -16)


def test_the_six_kept_cross_terms_leave_less_than_three_ulp_of_bf16_cubed():
    """(w1 + w2 + w3)(d1 + d2 + d3) minus the six kept products = w2 d3 + w3 d2 + w3 d3, each at
    most 2^-24 |w1 d1|: the sum of the kept products is within 3 * 2^-24 of the fp32 product,
    relative, before any accumulation error."""
    rng = np.random.default_rng(6)
    w = rng.normal(0, 0.05, 50000).astype(np.float32)
    d = rng.uniform(-0.5, 0.5, 50000).astype(np.float32)
    w1, w2, w3 = (t.astype(np.float64) for t in split3(w))
    d1, d2, d3 = (t.astype(np.float64) for t in split3(d))
    kept = w1 * d1 + w1 * d2 + w2 * d1 + w1 * d3 + w3 * d1 + w2 * d2
    exact = w.astype(np.float64) * d.astype(np.float64)
    ok = np.abs(exact) > 1e-12
    assert np.max(np.abs(kept - exact)[ok] / np.abs(exact)[ok]) <= 3 * 2.0 ** -24
