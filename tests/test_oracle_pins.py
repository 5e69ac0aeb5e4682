"""Pins for the CPU oracle: closed forms, invariants, library routines, brute
force and the values the paper prints.  None of these re-use the oracle's own
formula; a dropped term, wrong sign/index or transposed operand fails one."""
import math
import os

import numpy as np
import pytest

import oracle
import workloads as W
from oracle import formats, selector

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_qkv(B, H, S, d, dtype="f16", seed=0, std=1.0):
    return W.qkv_bits(B, H, S, d, dtype, std, seed)


def dense_softmax_attention(Q, K, V, dtype):
    """Independent dense attention: numpy matmul + softmax in fp64."""
    q, k, v = (W.bits_to_f64(x, dtype) for x in (Q, K, V))
    s = np.einsum("bhid,bhjd->bhij", q, k) / math.sqrt(q.shape[-1])
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=-1, keepdims=True)
    return np.einsum("bhij,bhjd->bhid", p, v)


# -- conversions ------------------------------------------------------------

def test_f16_widening_matches_numpy_for_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.f16_to_f64(int(b)) for b in bits])
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref))
    assert oracle.f16_to_f64(0x3C00) == 1.0 and oracle.f16_to_f64(0x0001) == 2.0 ** -24
    assert oracle.f16_to_f64(0x7BFF) == 65504.0 and oracle.f16_to_f64(0xC000) == -2.0


def test_bf16_widening_known_values():
    assert oracle.bf16_to_f64(0x3F80) == 1.0
    assert oracle.bf16_to_f64(0xC040) == -3.0
    assert oracle.bf16_to_f64(0x3F81) == 1.0 + 2.0 ** -7
    assert oracle.bf16_to_f64(0x0080) == 2.0 ** -126


# -- attention: closed forms and invariants ------------------------------------

@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_all_ones_mask_equals_dense_attention(dtype):
    B, H, S, d = 2, 3, 37, 16
    Q, K, V = rand_qkv(B, H, S, d, dtype, seed=11)
    mask = np.ones((1, 1, S, S), np.uint8)
    got = oracle.masked_attention(Q, K, V, dtype, mask)
    ref = dense_softmax_attention(Q, K, V, dtype)
    assert np.abs(got - ref).max() < 1e-12


def test_single_key_per_row_returns_that_value_row_exactly():
    B, H, S, d = 1, 2, 29, 8
    Q, K, V = rand_qkv(B, H, S, d, seed=12)
    rng = np.random.default_rng(5)
    sel = rng.integers(0, S, size=S)
    mask = np.zeros((1, 1, S, S), np.uint8)
    mask[0, 0, np.arange(S), sel] = 1
    got = oracle.masked_attention(Q, K, V, "f16", mask)
    v = W.bits_to_f64(V, "f16")
    assert np.array_equal(got, v[:, :, sel, :])


def test_zero_queries_give_mean_of_values_over_unmasked_keys():
    B, H, S, d = 1, 2, 40, 8
    Q, K, V = rand_qkv(B, H, S, d, seed=13)
    Q[:] = 0
    c = W.config(1)
    mask = W.dense_mask(c.mask, B, H, S)
    got = oracle.masked_attention(Q, K, V, "f16", mask)
    v = W.bits_to_f64(V, "f16")
    m = mask[0, 0].astype(np.float64)
    ref = np.einsum("ij,bhjd->bhid", m / m.sum(axis=1, keepdims=True), v)
    assert np.abs(got - ref).max() < 1e-13
    # zero keys: every score is 0 as well
    Q, K, V = rand_qkv(B, H, S, d, seed=14)
    K[:] = 0
    got = oracle.masked_attention(Q, K, V, "f16", mask)
    ref = np.einsum("ij,bhjd->bhid", m / m.sum(axis=1, keepdims=True), W.bits_to_f64(V, "f16"))
    assert np.abs(got - ref).max() < 1e-13


def test_probabilities_sum_to_one_and_vanish_on_masked_keys():
    B, H, S, d = 2, 2, 64, 16
    Q, K, V = rand_qkv(B, H, S, d, seed=15, std=2.0)
    spec = W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=7, stride=16)
    mask = W.dense_mask(spec, B, H, S)
    full = oracle.masked_attention(Q, K, V, "f16", mask)
    for (b, h, i) in [(0, 0, 0), (1, 1, 63), (0, 1, 17), (1, 0, 32)]:
        p, o = oracle.row_probs(Q, K, V, "f16", mask, b, h, i)
        assert abs(p.sum() - 1.0) < 1e-14
        assert np.all(p[mask[0, 0, i] == 0] == 0.0)
        assert np.all(p[mask[0, 0, i] == 1] > 0.0)
        assert np.array_equal(o, full[b, h, i])
        v = W.bits_to_f64(V, "f16")[b, h]
        assert np.abs(p @ v - o).max() < 1e-14


def test_fully_masked_rows_are_zero_and_nothing_is_nan():
    B, H, S, d = 1, 2, 33, 8
    Q, K, V = rand_qkv(B, H, S, d, seed=16)
    spec = W.MaskSpec(flags=W.PADDING, valid_len=(20,))
    mask = W.dense_mask(spec, B, H, S)
    got = oracle.masked_attention(Q, K, V, "f16", mask)
    assert np.all(np.isfinite(got))
    assert np.all(got[:, :, 20:, :] == 0.0)
    assert np.all(np.abs(got[:, :, :20, :]).sum(axis=-1) > 0.0)
    # rows < 20 must equal dense attention over the first 20 tokens only
    ref = dense_softmax_attention(Q[:, :, :20].copy(), K[:, :, :20].copy(), V[:, :, :20].copy(), "f16")
    assert np.abs(got[:, :, :20] - ref).max() < 1e-12


def test_causal_first_row_and_zero_width_window():
    B, H, S, d = 1, 1, 21, 4
    Q, K, V = rand_qkv(B, H, S, d, seed=17)
    v = W.bits_to_f64(V, "f16")
    got = oracle.masked_attention(Q, K, V, "f16", W.dense_mask(W.MaskSpec(flags=W.CAUSAL), B, H, S))
    assert np.array_equal(got[0, 0, 0], v[0, 0, 0])
    got = oracle.masked_attention(Q, K, V, "f16", W.dense_mask(W.MaskSpec(flags=W.WINDOW), B, H, S))
    assert np.array_equal(got, v)


def brute_force(q, k, v, m, scale):
    """Dense scores with -inf fill, then a whole-row softmax: pure Python."""
    d = len(q[0])
    out = [[0.0] * d for _ in range(len(q))]
    for i in range(len(q)):
        row = []
        for j in range(len(k)):
            if m[i][j]:
                row.append(scale * math.fsum(q[i][t] * k[j][t] for t in range(d)))
            else:
                row.append(-math.inf)
        top = max(row)
        if top == -math.inf:
            continue
        e = [math.exp(x - top) for x in row]
        z = math.fsum(e)
        for t in range(d):
            out[i][t] = math.fsum(e[j] / z * v[j][t] for j in range(len(k)))
    return out


@pytest.mark.parametrize("S,d,seed", [(1, 1, 0), (3, 2, 1), (8, 4, 2), (7, 3, 3), (5, 4, 4)])
def test_brute_force_on_tiny_shapes(S, d, seed):
    Q, K, V = rand_qkv(1, 1, S, d, seed=100 + seed, std=1.5)
    rng = np.random.default_rng(seed)
    mask = (rng.random((1, 1, S, S)) < 0.5).astype(np.uint8)
    if S > 2:
        mask[0, 0, 1, :] = 0  # one fully masked row
    got = oracle.masked_attention(Q, K, V, "f16", mask, scale=0.37)
    q, k, v = (W.bits_to_f64(x, "f16")[0, 0].tolist() for x in (Q, K, V))
    ref = np.array(brute_force(q, k, v, mask[0, 0].tolist(), 0.37))
    assert np.abs(got[0, 0] - ref).max() < 1e-14


# -- fewer (or more) queries than keys ---------------------------------------

def rand_rect(B, H, Sq, Sk, d, dtype="f16", seed=0, std=1.0):
    Q, _, _ = W.qkv_bits(B, H, Sq, d, dtype, std, seed)
    _, K, V = W.qkv_bits(B, H, Sk, d, dtype, std, seed + 1)
    return Q, K, V


@pytest.mark.parametrize("Sq,Sk", [(1, 9), (5, 3), (7, 16)])
def test_rectangular_all_ones_equals_dense_attention_and_brute_force(Sq, Sk):
    Q, K, V = rand_rect(2, 2, Sq, Sk, 8, seed=40 + Sq)
    ones = np.ones((1, 1, Sq, Sk), dtype=np.uint8)
    got = oracle.masked_attention(Q, K, V, "f16", ones)
    assert got.shape == (2, 2, Sq, 8)
    assert np.abs(got - dense_softmax_attention(Q, K, V, "f16")).max() < 1e-12
    rng = np.random.default_rng(Sq * 31 + Sk)
    mask = (rng.random((2, 2, Sq, Sk)) < 0.5).astype(np.uint8)
    mask[1, 0, 0, :] = 0  # one fully masked row
    got = oracle.masked_attention(Q, K, V, "f16", mask, scale=0.41)
    for b in range(2):
        for h in range(2):
            q, k, v = (W.bits_to_f64(x, "f16")[b, h].tolist() for x in (Q, K, V))
            ref = np.array(brute_force(q, k, v, mask[b, h].tolist(), 0.41))
            assert np.abs(got[b, h] - ref).max() < 1e-14
    assert np.all(got[1, 0, 0] == 0.0)


def test_rectangular_closed_forms_and_row_subsets():
    # one key per query -> exactly that value row; zero queries -> mean over the unmasked keys
    Sq, Sk, d = 6, 11, 5
    Q, K, V = rand_rect(1, 2, Sq, Sk, d, seed=77)
    v = W.bits_to_f64(V, "f16")
    pick = np.array([10, 0, 3, 3, 7, 1])
    mask = np.zeros((1, 1, Sq, Sk), dtype=np.uint8)
    mask[0, 0, np.arange(Sq), pick] = 1
    got = oracle.masked_attention(Q, K, V, "f16", mask)
    assert np.array_equal(got[0, 1], v[0, 1, pick])
    rng = np.random.default_rng(5)
    mask = (rng.random((1, 1, Sq, Sk)) < 0.6).astype(np.uint8)
    mask[0, 0, :, 2] = 1
    got = oracle.masked_attention(np.zeros_like(Q), K, V, "f16", mask)
    for i in range(Sq):
        sel = mask[0, 0, i].astype(bool)
        assert np.abs(got[0, 0, i] - v[0, 0, sel].mean(axis=0)).max() < 1e-14
    # a sample of the query rows of a self-attention problem gives those rows of its result, bit for bit
    S = 33
    Q, K, V = rand_qkv(1, 2, S, 8, seed=78)
    full_mask = W.dense_mask(W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=4, stride=8), 1, 2, S)
    full = oracle.masked_attention(Q, K, V, "f16", full_mask)
    rows = np.array([0, 5, 17, 32])
    part = oracle.masked_attention(np.ascontiguousarray(Q[:, :, rows]), K, V, "f16",
                                   np.ascontiguousarray(full_mask[:, :, rows]))
    assert np.array_equal(part, full[:, :, rows])


def test_default_scale_is_inverse_sqrt_head_dim():
    Q, K, V = rand_qkv(1, 1, 6, 9, seed=18)
    mask = np.ones((1, 1, 6, 6), np.uint8)
    a = oracle.masked_attention(Q, K, V, "f16", mask)
    b = oracle.masked_attention(Q, K, V, "f16", mask, scale=1.0 / 3.0)
    assert np.array_equal(a, b)


def test_key_permutation_invariance_and_per_batch_per_head_masks():
    B, H, S, d = 2, 2, 24, 8
    Q, K, V = rand_qkv(B, H, S, d, seed=19)
    rng = np.random.default_rng(7)
    mask = (rng.random((B, H, S, S)) < 0.4).astype(np.uint8)
    base = oracle.masked_attention(Q, K, V, "f16", mask)
    perm = rng.permutation(S)
    got = oracle.masked_attention(Q, np.ascontiguousarray(K[:, :, perm]),
                                  np.ascontiguousarray(V[:, :, perm]), "f16",
                                  np.ascontiguousarray(mask[:, :, :, perm]))
    assert np.abs(got - base).max() < 1e-13
    # each (b, h) must have used its own mask: recompute one pair alone
    one = oracle.masked_attention(Q[1:2, 1:2].copy(), K[1:2, 1:2].copy(), V[1:2, 1:2].copy(), "f16",
                                  mask[1:2, 1:2].copy())
    assert np.array_equal(one[0, 0], base[1, 1])


def test_adding_a_row_constant_to_the_scores_changes_nothing():
    # append a feature: q gets c_i, k gets 1 -> every score of row i shifts by c_i
    B, H, S, d = 1, 1, 20, 8
    Q, K, V = rand_qkv(B, H, S, d + 1, seed=20)
    mask = W.dense_mask(W.MaskSpec(flags=W.CAUSAL), B, H, S)
    K[..., d] = 0x3C00  # 1.0
    shifted = oracle.masked_attention(Q, K, V, "f16", mask, scale=0.25)
    Q2 = Q.copy()
    Q2[..., d] = 0
    plain = oracle.masked_attention(Q2, K, V, "f16", mask, scale=0.25)
    assert np.abs(shifted - plain).max() < 1e-13


def test_softmax_is_not_applied_to_transposed_scores():
    # non-symmetric check: O depends on q_i . k_j, not q_j . k_i
    S, d = 4, 2
    q = np.array([[1, 0], [0, 1], [2, 0], [0, 2]], dtype=np.float64)
    k = np.array([[3, 0], [0, 0], [0, 0], [0, 0]], dtype=np.float64)
    v = np.arange(S * d, dtype=np.float64).reshape(S, d)
    Q, K, V = (W.f64_to_f16_bits(x).reshape(1, 1, S, d) for x in (q, k, v))
    got = oracle.masked_attention(Q, K, V, "f16", np.ones((1, 1, S, S), np.uint8), scale=1.0)
    w = np.array([math.exp(3.0), 1, 1, 1])
    assert np.abs(got[0, 0, 0] - (w / w.sum()) @ v).max() < 1e-14
    assert np.abs(got[0, 0, 1] - v.mean(axis=0)).max() < 1e-14


# -- mask generators against the paper's Table 2 ---------------------------------

def _table2():
    rows = {}
    with open(os.path.join(GOLD, "table2_sparsity.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, val = line.split()
                rows[name] = float(val)
    return rows


def test_mask_generators_reproduce_table2_sparsity():
    printed = _table2()
    S = 1024
    spars = {}
    for name in printed:
        m = W.dense_mask(W.table2_spec(name), 1, 1, S)[0, 0]
        spars[name] = 100.0 * (1.0 - m.mean())
    # exact to the printed digit for the deterministic, fully specified patterns
    assert round(spars["causal"], 1) == printed["causal"]
    assert round(spars["sliding_window"], 1) == printed["sliding_window"]
    # closed forms: causal keeps S(S+1)/2, band |i-j|<=w keeps S(2w+1) - w(w+1)
    assert W.dense_mask(W.table2_spec("causal"), 1, 1, S).sum() == S * (S + 1) // 2
    assert W.dense_mask(W.table2_spec("sliding_window"), 1, 1, S).sum() == S * 65 - 32 * 33
    # compounds: the paper does not state how the parts overlap -> loose pins
    assert abs(spars["longformer"] - printed["longformer"]) < 1.5
    assert abs(spars["bigbird"] - printed["bigbird"]) < 3.0


# -- formats ------------------------------------------------------------------

def _masks_for_formats():
    out = []
    for idx, S in [(1, 128), (2, 200), (3, 256), (4, 256), (5, 512)]:
        c = W.config(idx)
        spec = c.mask
        if spec.valid_len is not None:
            spec = W.MaskSpec(**{**spec.__dict__, "valid_len": (S - 37,)})
        out.append((c.name, S, W.dense_mask(spec, 1, 1, S)[0, 0]))
    out.append(("scattered", 100, W.scattered_spec(100, 5, 3)[0, 0]))
    out.append(("empty", 70, np.zeros((70, 70), np.uint8)))
    out.append(("ones", 130, np.ones((130, 130), np.uint8)))
    return out


@pytest.mark.parametrize("bs", [16, 32, 64])
def test_formats_round_trip_and_invariants(bs):
    for name, S, M in _masks_for_formats():
        rp, ci = formats.csr(M)
        assert rp[0] == 0 and rp[-1] == M.sum() == len(ci)
        assert np.all(np.diff(rp) >= 0)
        for i in range(S):
            seg = ci[rp[i]:rp[i + 1]]
            assert np.all(np.diff(seg) > 0)
        assert np.array_equal(formats.dense_from_csr(rp, ci, S), M), name
        f = formats.bsr(M, bs)
        assert np.array_equal(formats.dense_from_bsr(f, S, bs), M), name
        nb = -(-S // bs)
        lrp, frp, prp = f["load_row_ptr"], f["full_row_ptr"], f["part_row_ptr"]
        assert np.array_equal(lrp, frp + prp)
        for br in range(nb):
            load = f["load_col_idx"][lrp[br]:lrp[br + 1]].tolist()
            full = f["full_col_idx"][frp[br]:frp[br + 1]].tolist()
            part = f["part_col_idx"][prp[br]:prp[br + 1]].tolist()
            assert load == sorted(set(full) | set(part)) and not (set(full) & set(part))
        pop = sum(bin(int(w)).count("1") for w in f["bitmap"].ravel())
        nfull = int(frp[-1])
        assert pop + nfull * bs * bs == M.sum() == f["nnz"]
        for words in f["bitmap"]:
            c = sum(bin(int(w)).count("1") for w in words)
            assert 0 < c < bs * bs
        if S % bs:  # ragged tiles can never be full
            assert (nb - 1) not in f["full_col_idx"].tolist()


def test_format_hand_counts():
    c = W.config(1)
    M = W.dense_mask(c.mask, 1, 1, 128)[0, 0]
    f64 = formats.bsr(M, 64)
    assert f64["full_row_ptr"][-1] == 0 and f64["part_row_ptr"][-1] == 4
    f16 = formats.bsr(M, 16)
    assert f16["full_row_ptr"][-1] == 8 and f16["part_row_ptr"][-1] == 14
    # bitmap of tile (0, 1) at bs 64: row r keeps columns 64..r+16 -> tile columns 0..r-48
    words = f64["bitmap"][1]
    for r in range(64):
        expect = (1 << max(0, r - 47)) - 1
        assert int(words[r]) == expect
    c4 = W.config(4)
    M4 = W.dense_mask(c4.mask, 1, 2, 512)
    for h in range(2):
        f = formats.bsr(M4[0, h], 64)
        assert f["part_row_ptr"][-1] == 0 and f["full_row_ptr"][-1] * 4096 == M4[0, h].sum()
    assert not np.array_equal(M4[0, 0], M4[0, 1])


def test_inner_tile_bitmap_layout():
    M = np.zeros((64, 64), np.uint8)
    M[9, 18] = 1    # inner tile (1, 2), entry (1, 2) -> word 2*8+1, bit 8*1+2
    M[63, 0] = 1    # inner tile (7, 0), entry (7, 0) -> word 7, bit 56
    f = formats.bsr(M, 64)
    it = formats.bitmap_inner_tiles(f["bitmap"])
    assert int(it[0, 17]) == 1 << 10 and int(it[0, 7]) == 1 << 56
    assert sum(bin(int(w)).count("1") for w in it[0]) == 2


# -- selector -----------------------------------------------------------------

def test_selector_hand_values():
    specs = {"window16": W.config(1).mask, "longformer512": W.config(2).mask,
             "strided2048": W.config(3).mask}
    with open(os.path.join(GOLD, "eq1_hand_values.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for name, S, v16, thr in rows:
        S, v16, thr = int(S), int(v16), float(thr)
        M = W.dense_mask(specs[name], 1, 1, S)[0, 0]
        assert selector.valid16(M) == v16
        assert abs(selector.threshold(v16, S) - thr) < 1e-12
        assert selector.choose(v16, S) == "block"
    # sparse enough -> row-wise: one tile per tile-row at S = 4096 (n = 256): 1/256 - 1.2/64 < 0
    assert selector.choose(256, 4096) == "row"
    assert selector.threshold(256, 4096) == pytest.approx(1 / 256 - 1.2 / 64)
    assert selector.choose(1, 16) == "row" and selector.choose(1, 9) == "row"
    # dense mask at n = 2: 1 - 1.2/1 < 0 -> row-wise; at n = 4: 1 - 0.3 > 0 -> block
    assert selector.choose(4, 32) == "row" and selector.choose(16, 64) == "block"
    # fewer queries than keys (this build's reading: ratio over the nq x nk tiles, n = nk in the logarithm), by hand:
    # all ones, 64 queries x 512 keys: nq = 4, nk = 32, 128 tiles of 128 set, log2(32) = 5 -> 1 - 1.2/25
    assert selector.valid16(np.ones((64, 512), dtype=np.uint8)) == 128
    assert selector.threshold(128, 64, Sk=512) == pytest.approx(1.0 - 1.2 / 25.0, abs=1e-15)
    # one key tile column set, 48 queries x 4096 keys: nq = 3, nk = 256, 3 tiles of 768 -> 1/256 - 1.2/64
    assert selector.threshold(3, 48, Sk=4096) == pytest.approx(1.0 / 256.0 - 1.2 / 64.0, abs=1e-15)
    # more queries than keys, 512 x 64: nq = 32, nk = 4, half of the tiles set -> 0.5 - 1.2/4
    assert selector.threshold(64, 512, Sk=64) == pytest.approx(0.5 - 0.3, abs=1e-15)
