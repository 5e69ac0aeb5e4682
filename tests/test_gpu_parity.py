"""HIP kernels against the fp64 CPU oracle, element by element, through the C ABI.

Gate (fp16/bf16 inputs): max-abs <= 5e-3 and relative Frobenius <= 1e-3 on the fp32 or
fp16 output; bf16 *output* adds its own rounding (half an ulp = 2^-9 relative), so that case
is gated at 5e-3 + 2^-8 |ref|.  Index arrays are checked bit-exactly in test_plan_formats.
"""
from dataclasses import replace

import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

MAX_ABS = 5e-3
REL_FRO = 1e-3


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


@pytest.fixture(scope="module")
def smha():
    import paper_2506_06095_amd as m
    return m


def to_dev(torch, bits, dtype):
    t = torch.from_numpy(bits.view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == "f16" else torch.bfloat16)


def check(got, ref, what, bf16_out=False):
    got = got.astype(np.float64)
    assert np.all(np.isfinite(got)), what
    diff = np.abs(got - ref)
    if bf16_out:
        assert np.all(diff <= MAX_ABS + 2.0 ** -8 * np.abs(ref)), (what, diff.max())
        return
    fro = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert diff.max() <= MAX_ABS, (what, "max-abs", diff.max(), np.unravel_index(diff.argmax(), diff.shape))
    assert fro <= REL_FRO, (what, "rel-fro", fro)


def run_case(torch, smha, Q, K, V, dtype, masks, kernel, block=64, out_f32=False, scale=0.0,
             heads=None, plan=None, what=""):
    """GPU forward on everything; oracle on `heads` (list of (b, h)) or on everything."""
    B, H, S, d = Q.shape
    own = plan is None
    if own:
        plan = smha.Plan.from_dense(masks, block=block, build_both=True, head_dim=d)
    try:
        q, k, v = (to_dev(torch, x, dtype) for x in (Q, K, V))
        out = plan.forward(q, k, v, out_dtype=torch.float32 if out_f32 else None, scale=scale, kernel=kernel)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy()
    finally:
        if own:
            plan.close()
    sc = None if scale == 0.0 else scale
    Bm, Hm = masks.shape[:2]
    if heads is None:
        ref = oracle.masked_attention(Q, K, V, dtype, masks, sc)
        check(got, ref, what, bf16_out=(dtype == "bf16" and not out_f32))
    else:
        for (b, h) in heads:
            m1 = np.ascontiguousarray(masks[b if Bm > 1 else 0, h if Hm > 1 else 0][None, None])
            ref = oracle.masked_attention(*(np.ascontiguousarray(x[b:b + 1, h:h + 1]) for x in (Q, K, V)),
                                          dtype, m1, sc)
            check(got[b:b + 1, h:h + 1], ref, f"{what} b{b} h{h}", bf16_out=(dtype == "bf16" and not out_f32))
    return got


KERNELS = {"row": 1, "block": 2}


@pytest.mark.parametrize("kernel", ["block", "row"])
@pytest.mark.parametrize("idx", [1, 2, 3])
def test_configs_1_to_3_full_size(torch_mod, smha, idx, kernel):
    c = W.config(idx)
    Q, K, V = W.qkv_bits(c.B, c.H, c.S, c.d, c.dtype, c.std, c.seed)
    masks = W.dense_mask(c.mask, c.B, c.H, c.S)
    run_case(torch_mod, smha, Q, K, V, c.dtype, masks, KERNELS[kernel], block=c.block, what=f"{c.name}/{kernel}")


@pytest.mark.parametrize("kernel", ["block", "row"])
def test_config_4_bf16_full_size(torch_mod, smha, kernel):
    c = W.config(4)
    Q, K, V = W.qkv_bits(c.B, c.H, c.S, c.d, c.dtype, c.std, c.seed)
    masks = W.dense_mask(c.mask, c.B, c.H, c.S)
    heads = [(0, 0), (1, 7), (1, 15)] if kernel == "row" else None
    with smha.Plan.from_desc(c.mask, c.B, c.H, c.S, block=c.block, build_both=True, head_dim=c.d) as plan:
        run_case(torch_mod, smha, Q, K, V, c.dtype, masks, KERNELS[kernel], out_f32=True, heads=heads,
                 plan=plan, what=f"{c.name}/{kernel}/f32out")
        got = run_case(torch_mod, smha, Q, K, V, c.dtype, masks, KERNELS[kernel], out_f32=False,
                       heads=[(0, 3)], plan=plan, what=f"{c.name}/{kernel}/bf16out")
    # bfloat16 output against the oracle rounded to bfloat16 (nearest even): distance in units of the last place
    m1 = np.ascontiguousarray(masks[0, 3][None, None])
    ref = oracle.masked_attention(*(np.ascontiguousarray(x[:1, 3:4]) for x in (Q, K, V)), c.dtype, m1)

    def ordered(bits):  # bit patterns -> integers that are monotonic in the value
        b = bits.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b)

    ulps = np.abs(ordered(W.f64_to_bf16_bits(got[:1, 3:4].astype(np.float64))) - ordered(W.f64_to_bf16_bits(ref)))
    hist = np.bincount(np.minimum(ulps.ravel(), 4), minlength=5) / ulps.size
    print(f"{c.name}/{kernel}: bfloat16 output, ulp distance 0/1/2/3/4+ = " + " ".join(f"{x:.4f}" for x in hist))
    big = np.abs(ref) >= 2.0 ** -6        # (tiny outputs: a unit in the last place is far below the 5e-3 gate)
    assert hist[0] + hist[1] >= 0.99 and ulps[big].max() <= 2


def test_config_5_full_size_every_head(torch_mod, smha):
    c = W.config(5)
    Q, K, V = W.qkv_bits(c.B, c.H, c.S, c.d, c.dtype, c.std, c.seed)
    masks = W.dense_mask(c.mask, c.B, c.H, c.S)
    with smha.Plan.from_desc(c.mask, c.B, c.H, c.S, block=c.block, head_dim=c.d, build_both=True) as plan:
        info = plan.info()
        assert info["kernel"] == smha.SMHA_KERNEL_BLOCK and info["n_split_rows"] == 1
        got = run_case(torch_mod, smha, Q, K, V, c.dtype, masks, 0, plan=plan, what=c.name)     # the oracle on all 32 heads
        valid = c.mask.valid_len[0]
        assert np.all(got[:, :, valid:, :] == 0.0)          # padded queries: zero rows
        assert np.all(np.abs(got[:, :, :valid, :]).sum(axis=-1) > 0)
        # the row-wise kernel on the same workload (it is 25 times slower here, so two heads against the oracle,
        # the rest against the block kernel's output)
        row = run_case(torch_mod, smha, Q, K, V, c.dtype, masks, KERNELS["row"], heads=[(0, 5), (0, 30)], plan=plan,
                       what=c.name + "/row")
        assert np.all(row[:, :, valid:, :] == 0.0)
        assert np.abs(row.astype(np.float64) - got.astype(np.float64)).max() <= 2e-3


LONG = {
    # BigBird blocks with padding, as cfg5, at twice and eight times its length
    "bigbird_16k": (16384, 128, "f16", lambda S: W.MaskSpec(flags=W.BIGBIRD | W.PADDING, block=64, n_window_blocks=3,
                                                           n_global_blocks=2, n_random_blocks=3, seed=16,
                                                           per_head=True, valid_len=(S - 777,))),
    "bigbird_64k": (65536, 64, "bf16", lambda S: W.MaskSpec(flags=W.BIGBIRD, block=64, n_window_blocks=3,
                                                           n_global_blocks=1, n_random_blocks=2, seed=64)),
    # causal band plus strided columns (cfg3's pattern) and a Longformer band with global tokens
    "strided_causal_16k": (16384, 64, "f16", lambda S: W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=255,
                                                                 stride=256, stride_phase=3)),
    "longformer_64k": (65536, 128, "f16", lambda S: W.MaskSpec(flags=W.WINDOW | W.GLOBAL, window_left=128,
                                                              window_right=128, n_global=16)),
}


@pytest.mark.parametrize("name,kernel", [(n, "block") for n in sorted(LONG)] + [("bigbird_16k", "row"), ("strided_causal_16k", "row")])
def test_long_sequences_on_sampled_rows(torch_mod, smha, name, kernel):
    """Sequences of 16k and 64k (the paper reports up to 64k, Sec. 5.5): the whole output is computed on the
    GPU; the oracle recomputes a sample of query rows (first / last rows, tile edges, random ones) from mask
    rows generated on their own, never the S x S matrix."""
    S, d, dtype, make = LONG[name]
    spec = make(S)
    B, H = 1, 2
    Q, K, V = W.qkv_bits(B, H, S, d, dtype, 0.7, seed=S + d)
    rng = np.random.default_rng(S)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 127, 128, S // 2 - 1, S // 2, S - 778, S - 777, S - 65, S - 64, S - 1],
                                     rng.integers(0, S, 24)]))
    with smha.Plan.from_desc(spec, B, H, S, block=64, head_dim=d, force=KERNELS[kernel]) as plan:
        q, k, v = (to_dev(torch_mod, x, dtype) for x in (Q, K, V))
        out = plan.forward(q, k, v, out_dtype=torch_mod.float32)
        torch_mod.cuda.synchronize()
        got = out[:, :, torch_mod.from_numpy(rows).cuda()].cpu().numpy()
        whole_finite = bool(torch_mod.isfinite(out).all())
    assert whole_finite
    valid = int(spec.valid_len[0]) if spec.valid_len else S
    Hm = spec.n_head_masks(H)
    mrows = np.stack([W.mask_rows(spec, S, h, valid, rows) for h in range(Hm)])[None].astype(np.uint8)
    ref = oracle.masked_attention(np.ascontiguousarray(Q[:, :, rows]), K, V, dtype, np.ascontiguousarray(mrows))
    check(got, ref, f"{name}/{kernel}")
    if spec.valid_len:
        assert np.all(got[:, :, rows >= valid] == 0.0)


@pytest.mark.parametrize("kernel", ["block", "row"])
@pytest.mark.parametrize("Sq,Sk,d,dtype", [(64, 512, 64, "f16"), (100, 1000, 128, "f16"), (257, 130, 64, "bf16"),
                                           (1, 777, 128, "bf16"), (1024, 64, 64, "f16"), (300, 2100, 128, "f16")])
def test_fewer_or_more_queries_than_keys(torch_mod, smha, kernel, Sq, Sk, d, dtype):
    """Cross-attention shapes: a chunk of queries against a longer (or shorter) key sequence."""
    B, H = 2, 3
    Q, _, _ = W.qkv_bits(B, H, Sq, d, dtype, 1.0, seed=Sq + Sk)
    _, K, V = W.qkv_bits(B, H, Sk, d, dtype, 1.0, seed=Sq + Sk + 1)
    rng = np.random.default_rng(Sq * 7 + Sk)
    masks = (rng.random((1, H, Sq, Sk)) < 0.2).astype(np.uint8)
    masks[0, 0, :, : max(1, Sk // 3)] = 1                   # a dense band of keys: full tiles
    masks[0, 1, Sq // 2] = 0                                # a query with no key
    if Sk > 64:
        masks[0, 2, :, 64:] = 0                             # only the first key tile
    for dev in (False, True):
        m = torch_mod.from_numpy(masks).cuda() if dev else masks
        with smha.Plan.from_dense_rect(m, build_both=True, head_dim=d) as plan:
            assert (plan.info()["S"], plan.info()["Sk"]) == (Sq, Sk)
            q, k, v = (to_dev(torch_mod, x, dtype) for x in (Q, K, V))
            out = plan.forward(q, k, v, out_dtype=torch_mod.float32, kernel=KERNELS[kernel])
            torch_mod.cuda.synchronize()
            got = out.cpu().numpy()
            with pytest.raises(ValueError):
                plan.forward(q, q, q)
    ref = oracle.masked_attention(Q, K, V, dtype, masks)
    check(got, ref, f"rect {Sq}x{Sk}/{kernel}")
    assert np.all(got[:, 1, Sq // 2] == 0.0)


@pytest.mark.parametrize("d,dtype", [(64, "f16"), (128, "f16"), (64, "bf16"), (128, "bf16")])
@pytest.mark.parametrize("name", ["strided_cols", "scattered", "rect_scattered", "mixed_long_rows", "all_gathered_tiny",
                                  "many_gathered"])
def test_gathered_tiles(torch_mod, smha, name, d, dtype):
    """Tiles with few used key columns are repacked into gathered tiles (staged rows from arbitrary keys):
    same result as the oracle, and as the plan that visits every tile as it is."""
    rng = np.random.default_rng(len(name) + d)
    if name == "strided_cols":
        masks = W.dense_mask(W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=70, stride=37, stride_phase=5), 1, 1, 1000)
    elif name == "scattered":
        masks = W.scattered_spec(700, 3, 5)
    elif name == "rect_scattered":
        masks = (rng.random((1, 2, 200, 3000)) < 0.004).astype(np.uint8)
        masks[0, 1, :, 100:228] = 1
    elif name == "mixed_long_rows":
        masks = (rng.random((1, 1, 2300, 2300)) < 0.003).astype(np.uint8)
        masks[0, 0, :64] = 1
        masks[0, 0, :, :8] = 1
        masks[0, 0, 1000] = 0
    elif name == "many_gathered":  # every 5th key: 19 gathered tiles per 128 rows, more than one item may hold
        masks = W.dense_mask(W.MaskSpec(flags=W.STRIDED, stride=5, stride_phase=2), 1, 1, 6000)
    else:  # every tile is sparse: the first tile of each item is a gathered one
        masks = np.zeros((1, 1, 130, 400), dtype=np.uint8)
        masks[0, 0, np.arange(130), (np.arange(130) * 37) % 400] = 1
        masks[0, 0, np.arange(130), (np.arange(130) * 91 + 7) % 400] = 1
    Bm, Hm, Sq, Sk = masks.shape
    B, H = (1, 2) if name == "many_gathered" else (2, 2)
    Q, _, _ = W.qkv_bits(B, H, Sq, d, dtype, 1.0, seed=Sq + d)
    _, K, V = W.qkv_bits(B, H, Sk, d, dtype, 1.0, seed=Sk + d + 1)
    q, k, v = (to_dev(torch_mod, x, dtype) for x in (Q, K, V))
    outs = []
    for no_gather in (False, True):
        with smha.Plan.from_dense_rect(masks, head_dim=d, force=smha.SMHA_KERNEL_BLOCK, no_gather=no_gather) as plan:
            assert (plan.info()["n_gathered"] > 0) == (not no_gather)
            if name == "many_gathered" and not no_gather:
                assert plan.info()["n_split_rows"] > 0      # lists cut at 16 gathered tiles: partial results merged
            outs.append(plan.forward(q, k, v, out_dtype=torch_mod.float32).cpu().numpy())
    ref = oracle.masked_attention(Q, K, V, dtype, masks)
    check(outs[0], ref, f"gathered {name}")
    check(outs[1], ref, f"ungathered {name}")


@pytest.mark.parametrize("kernel", ["block", "row"])
@pytest.mark.parametrize("d,dtype", [(64, "f16"), (128, "f16"), (64, "bf16"), (128, "bf16")])
def test_ragged_lengths_and_degenerate_rows(torch_mod, smha, kernel, d, dtype):
    for S in (1, 37, 100, 130, 257):
        B, H = 2, 3
        Q, K, V = W.qkv_bits(B, H, S, d, dtype, 1.0, 1000 + S)
        rng = np.random.default_rng(S)
        masks = (rng.random((B, H, S, S)) < 0.35).astype(np.uint8)
        masks[0, 0] = 0                      # nothing attends: all-zero output
        masks[0, 1] = 1                      # dense attention
        masks[1, 0, S // 2] = 0              # one fully masked row
        masks[1, 1] = np.eye(S, dtype=np.uint8)  # one key per row: O = V
        got = run_case(torch_mod, smha, Q, K, V, dtype, masks, KERNELS[kernel], out_f32=True,
                       what=f"ragged S={S} d={d} {dtype} {kernel}")
        assert np.all(got[0, 0] == 0.0) and np.all(got[1, 0, S // 2] == 0.0)
        # one key per row: the only weight is 1 up to fp32 rounding of the exponent argument
        assert np.allclose(got[1, 1].astype(np.float64), W.bits_to_f64(V, dtype)[1, 1], rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("kernel", ["block", "row"])
@pytest.mark.parametrize("d,dtype", [(8, "f16"), (32, "f16"), (32, "bf16"), (40, "f16"), (80, "bf16"), (96, "f16"),
                                     (96, "bf16"), (120, "f16"), (136, "bf16"), (192, "f16"), (256, "f16"), (256, "bf16")])
def test_head_sizes_other_than_64_and_128(torch_mod, smha, kernel, d, dtype):
    """Any multiple of 8 up to 256: the kernels for 64, 128 and 256 columns run narrower heads (SURVEY's shape
    variants: 32, 96 and 256).  Rows are packed, so a read or a store past a row's d columns would hit its neighbour."""
    for S in (37, 257, 1000):
        B, H = 2, 2
        Q, K, V = W.qkv_bits(B, H, S, d, dtype, 1.0, 4000 + S + d)
        rng = np.random.default_rng(S + d)
        masks = (rng.random((B, H, S, S)) < 0.3).astype(np.uint8)
        masks[0, 1] = 1                      # dense attention
        masks[1, 0, S // 2] = 0              # one fully masked row
        masks[1, 1] = np.eye(S, dtype=np.uint8)  # one key per row: O = V
        for out_f32 in (True, False):
            got = run_case(torch_mod, smha, Q, K, V, dtype, masks, KERNELS[kernel], out_f32=out_f32,
                           what=f"head size {d} S={S} {dtype} {kernel} f32out={out_f32}")
            assert np.all(got[1, 0, S // 2] == 0.0)
    # split groups (partial results merged) and gathered tiles at a narrow head
    if kernel == "block":
        S = 2100
        for spec, want in ((W.MaskSpec(flags=W.WINDOW | W.GLOBAL, window_left=32, window_right=32, n_global=70), "n_split_rows"),
                           (W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=70, stride=37, stride_phase=5), "n_gathered")):
            Q, K, V = W.qkv_bits(1, 2, S, d, dtype, 1.0, 77 + d)
            masks = W.dense_mask(spec, 1, 2, S)
            with smha.Plan.from_desc(spec, 1, 2, S, head_dim=d, force=smha.SMHA_KERNEL_BLOCK) as plan:
                assert plan.info()[want] > 0
                for out_f32 in (True, False):
                    run_case(torch_mod, smha, Q, K, V, dtype, masks, 0, plan=plan, out_f32=out_f32,
                             what=f"head size {d} {want} f32out={out_f32}")


def test_head_sizes_that_are_refused(torch_mod, smha):
    masks = np.ones((1, 1, 64, 64), dtype=np.uint8)
    with smha.Plan.from_dense(masks, head_dim=64) as plan:
        for d in (4, 12, 100, 260, 264, 512):
            q = torch_mod.zeros(1, 1, 64, d, device="cuda", dtype=torch_mod.float16)
            with pytest.raises(smha.SmhaError):
                plan.forward(q, q, q)


def test_random_shapes_masks_and_sharing(torch_mod, smha):
    """Seeded sweep over query / key counts around the tile edges, both head sizes and dtypes, masks shared
    or not across batch and heads, five mask families (unstructured at several densities, 64-blocky, band
    plus columns, empty and full rows mixed), three block sizes; both kernels, fp32 and 16-bit output."""
    torch = torch_mod
    rng = np.random.default_rng(1234)
    for case in range(48):
        Sq = int(rng.choice([1, 2, 17, 63, 64, 65, 100, 127, 128, 129, 200, 300, 513]))
        Sk = Sq if rng.random() < 0.5 else int(rng.choice([1, 5, 64, 65, 130, 257, 700]))
        d = int(rng.choice([64, 128]))
        dtype = str(rng.choice(["f16", "bf16"]))
        B, H = int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 5, 9]))
        Bm, Hm = (B if rng.random() < 0.4 else 1), (H if rng.random() < 0.4 else 1)
        kind = int(rng.integers(0, 5))
        dens = float(rng.choice([0.0, 0.02, 0.2, 0.7, 1.0]))
        m = (rng.random((Bm, Hm, Sq, Sk)) < dens).astype(np.uint8)
        if kind == 1:
            blk = (rng.random((Bm, Hm, (Sq + 63) // 64, (Sk + 63) // 64)) < 0.4).astype(np.uint8)
            m = np.kron(blk, np.ones((64, 64), np.uint8))[:, :, :Sq, :Sk].copy()
        elif kind == 2:
            i, j = np.arange(Sq)[:, None], np.arange(Sk)[None, :]
            m = np.broadcast_to(((np.abs(i - j) <= 20) | (j % 97 == 3)).astype(np.uint8), (Bm, Hm, Sq, Sk)).copy()
        elif kind == 3:
            m[:, :, ::3, :] = 0
            m[:, :, 1::7, :] = 1
        block = int(rng.choice([16, 32, 64]))
        Qb, _, _ = W.qkv_bits(B, H, Sq, d, dtype, 1.0, 1000 + case)
        _, Kb, Vb = W.qkv_bits(B, H, Sk, d, dtype, 1.0, 2000 + case)
        q, k, v = (to_dev(torch, x, dtype) for x in (Qb, Kb, Vb))
        ref = oracle.masked_attention(Qb, Kb, Vb, dtype, m, None)
        what = f"case {case}: B{B} H{H} Sq{Sq} Sk{Sk} d{d} {dtype} Bm{Bm} Hm{Hm} kind{kind} density{dens} block{block}"
        make = smha.Plan.from_dense if Sq == Sk else smha.Plan.from_dense_rect
        with make(m, block=block, build_both=True, head_dim=d) as plan:
            for kernel in KERNELS.values():
                for f32 in (True, False):
                    out = plan.forward(q, k, v, out_dtype=torch.float32 if f32 else None, kernel=kernel)
                    torch.cuda.synchronize()
                    check(out.float().cpu().numpy(), ref, f"{what} kernel {kernel} fp32 out {f32}",
                          bf16_out=(dtype == "bf16" and not f32))


@pytest.mark.parametrize("bs", [16, 32, 64])
def test_block_sizes_and_scale_and_same_dtype_output(torch_mod, smha, bs):
    c = W.config(3)
    B, H, S, d = 1, 2, 512, 64
    Q, K, V = W.qkv_bits(B, H, S, d, "f16", 1.0, 77)
    masks = W.dense_mask(c.mask, B, H, S)
    for kernel in (1, 2):
        run_case(torch_mod, smha, Q, K, V, "f16", masks, kernel, block=bs, scale=0.2, what=f"bs{bs} k{kernel}")


def test_padding_per_batch_and_per_head_masks(torch_mod, smha):
    spec = W.MaskSpec(flags=W.BIGBIRD | W.PADDING, block=64, n_window_blocks=3, n_global_blocks=1,
                      n_random_blocks=2, seed=11, per_head=True, valid_len=(1024, 700, 1))
    B, H, S, d = 3, 4, 1024, 128
    Q, K, V = W.qkv_bits(B, H, S, d, "f16", 0.5, 5)
    masks = W.dense_mask(spec, B, H, S)
    assert masks.shape[:2] == (3, 4)
    with smha.Plan.from_desc(spec, B, H, S, build_both=True, head_dim=d) as plan:
        for kernel in (1, 2):
            run_case(torch_mod, smha, Q, K, V, "f16", masks, kernel, plan=plan, what=f"padding k{kernel}")


def test_split_rows_merge_matches_unsplit_semantics(torch_mod, smha):
    # a few very long tile rows among short ones forces the split + combine path at d = 64
    S, d = 4096, 64
    spec = W.MaskSpec(flags=W.WINDOW | W.GLOBAL, window_left=32, window_right=32, n_global=70)
    Q, K, V = W.qkv_bits(1, 2, S, d, "f16", 1.0, 8)
    masks = W.dense_mask(spec, 1, 2, S)
    with smha.Plan.from_desc(spec, 1, 2, S, head_dim=d, force=smha.SMHA_KERNEL_BLOCK) as plan:
        assert plan.info()["n_split_rows"] == 1
        run_case(torch_mod, smha, Q, K, V, "f16", masks, 0, plan=plan, what="split")


@pytest.mark.parametrize("d,dtype", [(64, "f16"), (128, "bf16")])
def test_few_heads_take_the_fine_work_items_and_agree_with_many_heads(torch_mod, smha, d, dtype):
    """One plan, one mask: a call with 2 heads leaves the chip mostly empty and walks the lists cut to 16
    steps (partials merged), a call with 160 heads walks the whole lists; the heads they share must agree
    with the oracle, and with each other to rounding."""
    torch = torch_mod
    S = 4096
    spec = W.table2_spec("causal")
    masks = W.dense_mask(spec, 1, 1, S)
    Q, K, V = W.qkv_bits(1, 2, S, d, dtype, 1.0, 21)
    with smha.Plan.from_desc(spec, 1, 2, S, head_dim=d, force=smha.SMHA_KERNEL_BLOCK) as plan:
        coarse = plan.export("kernel_items").reshape(-1, 8)
        fine = plan.export("kernel_items_fine").reshape(-1, 8)
        assert len(fine) > len(coarse) and (coarse[:, 3] == -1).all() and (fine[:, 3] >= 0).any()
        few = run_case(torch, smha, Q, K, V, dtype, masks, 0, plan=plan, out_f32=True, what="few heads")
        q, k, v = (to_dev(torch, np.ascontiguousarray(np.tile(x, (1, 80, 1, 1))), dtype) for x in (Q, K, V))
        many = plan.forward(q, k, v, out_dtype=torch.float32)
        torch.cuda.synchronize()
        many = many.cpu().numpy()
        assert np.array_equal(many[:, :2], many[:, 158:160])           # replicated heads: identical results
        assert np.abs(many[:, :2].astype(np.float64) - few).max() <= 1e-3


def test_one_plan_serves_many_batch_sizes_in_turn(torch_mod, smha):
    """The plan keeps a work order per (batch, heads) it has seen, a few at a time: going round more batch
    sizes than it keeps, twice, every call must still give each replicated head the same rows."""
    torch = torch_mod
    S, d, H = 700, 64, 3
    spec = W.MaskSpec(flags=W.WINDOW | W.GLOBAL, window_left=50, window_right=10, n_global=5)
    masks = W.dense_mask(spec, 1, 1, S)
    Q, K, V = W.qkv_bits(1, H, S, d, "f16", 1.0, 33)
    ref = oracle.masked_attention(Q, K, V, "f16", masks)
    with smha.Plan.from_desc(spec, 1, H, S, head_dim=d, force=smha.SMHA_KERNEL_BLOCK) as plan:
        for rnd in range(2):
            for B in (1, 2, 3, 5, 7, 11, 13, 4, 6, 9, 12):
                q, k, v = (to_dev(torch, np.ascontiguousarray(np.tile(x, (B, 1, 1, 1))), "f16") for x in (Q, K, V))
                out = plan.forward(q, k, v, out_dtype=torch.float32)
                torch.cuda.synchronize()
                got = out.cpu().numpy()
                assert all(np.array_equal(got[b], got[0]) for b in range(1, B)), (rnd, B)
                check(got[:1], ref, f"round {rnd} batch {B}")


def test_strided_tensors_device_mask_and_determinism(torch_mod, smha):
    torch = torch_mod
    c = W.config(2)
    B, H, S, d = 2, 4, 512, 64
    Q, K, V = W.qkv_bits(B, H, S, d, "f16", 1.0, 21)
    masks = W.dense_mask(c.mask, B, H, S)
    ref = oracle.masked_attention(Q, K, V, "f16", masks)
    dev_mask = torch.from_numpy(masks).cuda()
    with smha.Plan.from_dense(dev_mask, block=32, build_both=True) as plan:
        # [B,S,H,d] storage viewed as [B,H,S,d]: non-packed strides
        def bshd(x):
            t = to_dev(torch, x, "f16")
            return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        q, k, v = bshd(Q), bshd(K), bshd(V)
        assert not q.is_contiguous()
        for kernel in (1, 2):
            out = torch.empty(B, S, H, d, dtype=torch.float16, device="cuda").permute(0, 2, 1, 3)
            plan.forward(q, k, v, out=out, kernel=kernel)
            out2 = torch.empty_like(out)
            plan.forward(q, k, v, out=out2, kernel=kernel)
            torch.cuda.synchronize()
            check(out.float().cpu().numpy(), ref, f"strided k{kernel}")
            assert torch.equal(out, out2)            # same launch twice: bit-identical
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            out3 = plan.forward(q, k, v, kernel=2, stream=side)
        side.synchronize()
        check(out3.float().cpu().numpy(), ref, "side stream")


@pytest.mark.parametrize("S", [1, 63, 100, 130, 512, 1000])
def test_device_mask_is_packed_on_the_gpu_and_gives_the_host_plan(torch_mod, smha, S):
    """A mask that lives in device memory goes through the bit-packing kernel; every index array of
    the plan must equal, bit for bit, the one built from the same mask in host memory (and through
    it the format oracle, which the host path is tested against).  Any nonzero byte means attend."""
    torch = torch_mod
    rng = np.random.default_rng(S)
    masks = (rng.random((2, 3, S, S)) < 0.3).astype(np.uint8)
    masks[masks != 0] = rng.integers(1, 256, size=int(masks.sum()), dtype=np.uint8)   # 1..255, not just 1
    masks[1, 2] = 0                                                                    # an empty mask
    masks[0, 1, :, : min(S, 70)] = 255                                                 # full tiles
    dev = torch.from_numpy(masks).cuda()
    for bs in (16, 64):
        with smha.Plan.from_dense(masks, block=bs, build_both=True) as ph, \
                smha.Plan.from_dense(dev, block=bs, build_both=True) as pd:
            ih, idv = ph.info(), pd.info()
            for key in ("nnz", "n_valid", "n_full", "n_part", "n_valid16", "n_tiles64", "n_union", "n_items", "kernel"):
                assert ih[key] == idv[key], key
            for mi in range(6):
                for which in ("row_ptr", "col_idx", "load_row_ptr", "load_col_idx", "flags", "bitmap"):
                    np.testing.assert_array_equal(ph.export(which, mi), pd.export(which, mi), err_msg=f"{which} mask {mi} bs {bs}")


@pytest.mark.parametrize("Sq,Sk", [(1, 1), (63, 63), (100, 100), (130, 130), (512, 512), (1000, 1000), (200, 3000), (777, 91)])
def test_device_mask_is_analysed_on_the_gpu_and_gives_the_host_plan(torch_mod, smha, Sq, Sk):
    """A device mask whose plan needs no per-row lists (block kernel, 64-wide tiles) is classified tile by tile
    on the GPU; statistics, exported block format and the kernel's work lists must equal, bit for bit, those
    of the plan built from the same mask in host memory.  Any nonzero byte means attend."""
    torch = torch_mod
    rng = np.random.default_rng(Sq * 3 + Sk)
    masks = (rng.random((2, 3, Sq, Sk)) < 0.3).astype(np.uint8)
    masks[masks != 0] = rng.integers(1, 256, size=int(masks.sum()), dtype=np.uint8)
    masks[1, 2] = 0                                        # an empty mask
    masks[0, 1, :, : min(Sk, 70)] = 255                    # full tiles
    masks[1, 0, :, min(Sk - 1, 5)::max(1, Sk // 7)] = 0    # thinned columns
    masks[1, 1] = 0
    masks[1, 1, :, ::97] = 1                               # sparse columns: gathered tiles
    dev = torch.from_numpy(masks).cuda()
    kw = dict(force=smha.SMHA_KERNEL_BLOCK)
    with smha.Plan.from_dense_rect(masks, **kw) as ph, smha.Plan.from_dense_rect(dev, **kw) as pd:
        ih, idv = ph.info(), pd.info()
        for key in ("S", "Sk", "nnz", "n_valid", "n_full", "n_part", "n_valid16", "n_tiles64", "n_union", "n_items",
                    "n_gathered", "n_split_rows", "kernel", "eq1_threshold", "model_block_us", "model_row_us"):
            assert ih[key] == idv[key], key
        for which in ("kernel_entries", "kernel_bitmaps", "kernel_gather_keys"):
            np.testing.assert_array_equal(ph.export(which), pd.export(which), err_msg=which)
        for mi in range(6):
            for which in ("load_row_ptr", "load_col_idx", "flags", "bitmap", "full_col_idx", "part_row_ptr", "kernel_items"):
                np.testing.assert_array_equal(ph.export(which, mi), pd.export(which, mi), err_msg=f"{which} mask {mi}")
        Q, _, _ = W.qkv_bits(2, 3, Sq, 64, "f16", 1.0, seed=Sq)
        _, K, V = W.qkv_bits(2, 3, Sk, 64, "f16", 1.0, seed=Sk + 1)
        q, k, v = (to_dev(torch, x, "f16") for x in (Q, K, V))
        got = pd.forward(q, k, v, out_dtype=torch.float32).cpu().numpy()
    check(got, oracle.masked_attention(Q, K, V, "f16", (masks != 0).astype(np.uint8)), f"device-analysed {Sq}x{Sk}")
    # when the selector may take the row kernel the per-row lists are needed: same plan as from the host
    scat = np.zeros((1, 1, 600, 600), dtype=np.uint8)
    scat[0, 0, np.arange(600), (np.arange(600) * 131) % 600] = 1
    scat[0, 0, np.arange(600), (np.arange(600) * 17 + 3) % 600] = 1
    with smha.Plan.from_dense(scat) as ph, smha.Plan.from_dense(torch.from_numpy(scat).cuda()) as pd:
        assert ph.info()["kernel"] == pd.info()["kernel"] == smha.SMHA_KERNEL_ROW
        for which in ("row_ptr", "col_idx"):
            np.testing.assert_array_equal(ph.export(which), pd.export(which))


def test_selected_kernel_wins_on_its_own_ground(torch_mod, smha):
    """Scattered mask -> the calibrated selector picks row-wise; block-structured and dilated masks -> block-wise
    (what the plans say is asserted; the timings of both kernels are printed, and the sweep below checks them)."""
    torch = torch_mod

    def time_kernel(plan, q, k, v, kernel):
        out = plan.forward(q, k, v, kernel=kernel)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(20):
            plan.forward(q, k, v, out=out, kernel=kernel)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / 20

    B, H, S, d = 4, 16, 2048, 64
    Q, K, V = W.qkv_bits(B, H, S, d, "f16", 1.0, 31)
    q, k, v = (to_dev(torch, x, "f16") for x in (Q, K, V))
    scat = W.scattered_spec(S, 8, 3)
    with smha.Plan.from_dense(scat, build_both=True) as plan:
        assert plan.info()["kernel"] == smha.SMHA_KERNEL_ROW
        t_row, t_blk = time_kernel(plan, q, k, v, 1), time_kernel(plan, q, k, v, 2)
        print(f"scattered: row {t_row:.3f} ms, block {t_blk:.3f} ms")
        run_case(torch, smha, Q, K, V, "f16", scat, 0, heads=[(0, 0), (3, 15)], plan=plan, what="scattered")
    c = W.config(3)
    with smha.Plan.from_desc(c.mask, B, H, S, build_both=True) as plan:
        assert plan.info()["kernel"] == smha.SMHA_KERNEL_BLOCK
        t_row, t_blk = time_kernel(plan, q, k, v, 1), time_kernel(plan, q, k, v, 2)
        print(f"strided causal: row {t_row:.3f} ms, block {t_blk:.3f} ms")
        assert plan.info()["model_block_us"] < plan.info()["model_row_us"]
    # dilated attention (every 64th key, causal): as 2080 one-column tiles the row kernel would win;
    # repacked into 32 gathered tiles the block kernel is selected and wins
    dil = W.MaskSpec(flags=W.CAUSAL | W.STRIDED, stride=64, stride_phase=0)
    with smha.Plan.from_desc(dil, B, H, S, build_both=True) as plan:
        assert plan.info()["kernel"] == smha.SMHA_KERNEL_BLOCK and plan.info()["n_gathered"] > 0
        t_row, t_blk = time_kernel(plan, q, k, v, 1), time_kernel(plan, q, k, v, 2)
        print(f"dilated: row {t_row:.3f} ms, block with gathered tiles {t_blk:.3f} ms")
        run_case(torch, smha, Q, K, V, "f16", W.dense_mask(dil, B, H, S), 0, heads=[(1, 2)], plan=plan, what="dilated")
    with smha.Plan.from_desc(dil, B, H, S, no_gather=True) as plan:
        assert plan.info()["kernel"] == smha.SMHA_KERNEL_ROW


@pytest.mark.parametrize("case", ["split_rows", "gathered"])
def test_forward_replays_from_a_hip_graph(torch_mod, smha, case):
    """Once its shape is prepared, the very first forward can be captured into a HIP graph: every replay,
    with eager forwards of the same and of other batch sizes and synchronisation in between, gives the
    eager result (what the graph points at is never freed or moved by later calls)."""
    torch = torch_mod
    if case == "split_rows":    # global block rows make a split 128-row group: partial results merged in the launch
        spec = W.MaskSpec(flags=W.BIGBIRD, block=64, n_window_blocks=3, n_global_blocks=2, n_random_blocks=2, seed=9)
        B, H, S, d = 1, 4, 4096, 128
    else:
        spec = W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=100, stride=32, stride_phase=1)
        B, H, S, d = 2, 2, 1500, 64
    with smha.Plan.from_desc(spec, B, H, S, head_dim=d, force=smha.SMHA_KERNEL_BLOCK) as plan:
        info = plan.info()
        assert (info["n_split_rows"] > 0) if case == "split_rows" else (info["n_gathered"] > 0)
        gen = torch.Generator(device="cuda").manual_seed(5)
        q, k, v = (torch.randn(B, H, S, d, device="cuda", generator=gen).half() for _ in range(3))
        out = torch.empty_like(q)
        plan.prepare(B, H, d)                               # work order and workspaces: nothing is allocated after this
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                plan.forward(q, k, v, out=out)
        torch.cuda.synchronize()
        for rep in range(3):
            for t in (q, k, v):
                t.copy_(torch.randn(B, H, S, d, device="cuda", generator=gen).half())
            eager = plan.forward(q, k, v)                   # eager work between replays
            nb = B + 1 + rep                                # ... also with batch sizes the plan has not seen yet
            plan.forward(*(torch.randn(nb, H, S, d, device="cuda", generator=gen).half() for _ in range(3)))
            torch.cuda.synchronize()
            out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), (case, rep)
        masks = W.dense_mask(spec, B, H, S)
        Qb, Kb, Vb = (x.cpu().numpy().view(np.uint16) for x in (q, k, v))
        ref = oracle.masked_attention(*(np.ascontiguousarray(x[:1, :1]) for x in (Qb, Kb, Vb)), "f16", masks)
        check(out[:1, :1].float().cpu().numpy(), ref, f"graph replay {case}")


def test_forwards_on_one_plan_overlap_on_two_streams(torch_mod, smha):
    """Two forwards on one plan (split 128-row groups, so both use a workspace and arrival counters) run at
    the same time on two streams, several rounds in a row: each call takes its own workspace, so every
    output equals the one computed alone, and that one matches the oracle."""
    torch = torch_mod
    spec = W.MaskSpec(flags=W.BIGBIRD, block=64, n_window_blocks=3, n_global_blocks=2, n_random_blocks=2, seed=3)
    B, H, S, d = 1, 8, 4096, 128
    with smha.Plan.from_desc(spec, B, H, S, head_dim=d, force=smha.SMHA_KERNEL_BLOCK) as plan:
        assert plan.info()["n_split_rows"] > 0
        plan.prepare(B, H, d)
        gen = torch.Generator(device="cuda").manual_seed(11)
        sets = [[torch.randn(B, H, S, d, device="cuda", generator=gen).half() for _ in range(3)] for _ in range(2)]
        alone = [plan.forward(*qkv) for qkv in sets]
        torch.cuda.synchronize()
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        for rnd in range(4):
            outs = [torch.zeros_like(sets[i][0]) for i in range(2)]
            torch.cuda.synchronize()
            for rep in range(3):                            # several launches queued per stream
                for i in range(2):
                    plan.forward(*sets[i], out=outs[i], stream=streams[i])
            torch.cuda.synchronize()
            for i in range(2):
                assert torch.equal(outs[i], alone[i]), (rnd, i)
        masks = W.dense_mask(spec, B, H, S)
        Qb, Kb, Vb = (x.cpu().numpy().view(np.uint16) for x in sets[1])
        ref = oracle.masked_attention(*(np.ascontiguousarray(x[:1, 3:4]) for x in (Qb, Kb, Vb)), "f16", masks)
        check(alone[1][:1, 3:4].float().cpu().numpy(), ref, "two streams")


def test_selector_sweep_across_the_row_block_boundary(torch_mod, smha):
    """Masks on both sides of where the kernels cross over (2 to 64 scattered keys per row, narrow windows,
    sequences of 512 to 4096, both head sizes): the calibrated selector's choice is timed against the other
    kernel.  The cost model was fitted so that the choice is within 1.15x of the faster kernel on these; the
    assertion allows 1.5x (launch-bound cases and a busy machine move the ratio), and every ratio is printed."""
    torch = torch_mod

    def time_kernel(plan, q, k, v, kernel):
        out = plan.forward(q, k, v, kernel=kernel)
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(20):
                plan.forward(q, k, v, out=out, kernel=kernel)
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) / 20)
        return best

    B, H = 4, 16
    cases = [(64, 512, "scat", 8), (64, 512, "scat", 32), (64, 2048, "scat", 4), (64, 2048, "scat", 16), (64, 2048, "scat", 32),
             (64, 2048, "scat", 64), (64, 4096, "scat", 64), (128, 2048, "scat", 8), (128, 2048, "scat", 32), (128, 2048, "scat", 64),
             (128, 4096, "scat", 16), (64, 2048, "win", 8), (128, 4096, "win", 8)]
    worst = 0.0
    for d, S, kind, n in cases:
        gen = torch.Generator(device="cuda").manual_seed(S + d + n)
        q, k, v = (torch.randn(B, H, S, d, device="cuda", generator=gen).half() for _ in range(3))
        m = W.scattered_spec(S, n, 3) if kind == "scat" else W.dense_mask(W.MaskSpec(flags=W.WINDOW, window_left=n, window_right=n), 1, 1, S)
        with smha.Plan.from_dense(m, build_both=True, head_dim=d) as plan:
            chosen = plan.info()["kernel"]
            t = {kk: time_kernel(plan, q, k, v, kk) for kk in (1, 2)}
        ratio = t[chosen] / min(t.values())
        worst = max(worst, ratio)
        print(f"d {d} S {S} {kind}{n}: row {t[1] * 1e3:.1f} us, block {t[2] * 1e3:.1f} us, chose {'row' if chosen == 1 else 'block'} ({ratio:.2f}x of the faster)")
        assert ratio <= 1.5, (d, S, kind, n, t, chosen)
    print(f"worst choice: {worst:.2f}x of the faster kernel")


def test_nothing_is_written_outside_the_output(torch_mod, smha):
    """Guard bands: O sits in the middle of a larger buffer filled with a NaN pattern; after block-wise launches
    (ordinary, gathered and split work lists) and row-wise ones at ragged sequence lengths the bands are
    untouched bit for bit and everything inside is finite (a misdirected global -> LDS fill or store would show)."""
    torch = torch_mod
    cases = [
        (W.MaskSpec(flags=W.BIGBIRD, block=64, n_window_blocks=3, n_global_blocks=2, n_random_blocks=2, seed=4), 1, 3, 4000, 128, "split"),
        (W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=100, stride=32, stride_phase=1), 2, 2, 1501, 64, "gathered"),
        (W.MaskSpec(flags=W.WINDOW, window_left=40, window_right=9), 1, 5, 777, 128, "plain"),
    ]
    for spec, B, H, S, d, what in cases:
        with smha.Plan.from_desc(spec, B, H, S, head_dim=d, build_both=True) as plan:
            info = plan.info()
            if what == "split":
                assert info["n_split_rows"] > 0
            if what == "gathered":
                assert info["n_gathered"] > 0
            gen = torch.Generator(device="cuda").manual_seed(S)
            q, k, v = (torch.randn(B, H, S, d, device="cuda", generator=gen).half() for _ in range(3))
            n = B * H * S * d
            band = 1 << 16
            for kernel in (2, 1):
                for out_dtype in (torch.float16, torch.float32):
                    buf = torch.full((n + 2 * band,), float("nan"), dtype=out_dtype, device="cuda")
                    pattern = buf.view(torch.int16 if out_dtype == torch.float16 else torch.int32).clone()
                    out = buf[band:band + n].view(B, H, S, d)
                    plan.forward(q, k, v, out=out, kernel=kernel)
                    torch.cuda.synchronize()
                    after = buf.view(pattern.dtype)
                    assert torch.equal(after[:band], pattern[:band]), (what, kernel, out_dtype, "band before O")
                    assert torch.equal(after[band + n:], pattern[band + n:]), (what, kernel, out_dtype, "band after O")
                    assert bool(torch.isfinite(out).all()), (what, kernel, out_dtype)


@pytest.mark.parametrize("idx", [1, 2, 4, 5])
def test_second_form_of_the_block_kernel(torch_mod, smha, idx):
    """The block kernel's second form (score waves and value waves, asked for with the plan option) on the
    workloads it covers: every head against the oracle, and the padded rows exactly zero."""
    c = W.config(idx)
    Q, K, V = W.qkv_bits(c.B, c.H, c.S, c.d, c.dtype, c.std, c.seed)
    masks = W.dense_mask(c.mask, c.B, c.H, c.S)
    with smha.Plan.from_desc(c.mask, c.B, c.H, c.S, block=c.block, head_dim=c.d, force=smha.SMHA_KERNEL_BLOCK, block_form=2) as plan:
        assert plan.info()["n_gathered"] == 0                # (plans with gathered tiles run the first form)
        for out_f32 in ((True,) if c.dtype == "bf16" else (False, True)):
            got = run_case(torch_mod, smha, Q, K, V, c.dtype, masks, 0, out_f32=out_f32, plan=plan, what=f"{c.name}/form 2")
        if c.mask.valid_len:
            assert np.all(got[:, :, c.mask.valid_len[0]:, :] == 0.0)


@pytest.mark.parametrize("S,d,dtype", [(100, 64, "f16"), (130, 128, "f16"), (1000, 64, "bf16"), (2500, 128, "f16")])
def test_second_form_ragged_and_split(torch_mod, smha, S, d, dtype):
    """Second form at ragged lengths, with empty 128-row groups, fully masked rows, part tiles and (at 2500)
    groups that are split between workgroups."""
    B, H = 2, 3
    Q, K, V = W.qkv_bits(B, H, S, d, dtype, 1.0, seed=S + d)
    rng = np.random.default_rng(S)
    masks = np.zeros((1, H, S, S), dtype=np.uint8)
    ii, jj = np.indices((S, S))
    masks[0, 0] = (np.abs(ii - jj) <= 40) | (jj < 70) | (ii < 70)           # band + global rows and columns: a long list to split
    masks[0, 1] = (rng.random((S, S)) < 0.3) & (jj <= ii)                       # scattered causal: part tiles everywhere
    masks[0, 1, S // 2] = 0                                                    # a query without keys
    masks[0, 2, : S // 3, : S // 2] = 1                                        # full tiles, and query groups with nothing at all
    with smha.Plan.from_dense(masks, head_dim=d, force=smha.SMHA_KERNEL_BLOCK, no_gather=True, block_form=2) as plan:
        got = run_case(torch_mod, smha, Q, K, V, dtype, masks, 0, out_f32=True, plan=plan, what=f"form 2 ragged {S}")
        assert np.all(got[:, 1, S // 2] == 0.0) and np.all(got[:, 2, S // 3:] == 0.0)
        if dtype == "f16":
            run_case(torch_mod, smha, Q, K, V, dtype, masks, 0, plan=plan, what=f"form 2 ragged {S} f16 out")


@pytest.mark.parametrize("form", [1, 3])
def test_first_and_third_form_of_the_block_kernel_on_config_5(torch_mod, smha, form):
    """The block kernel's first form (four waves of 32 rows) and third form (eight waves of 16 rows), each asked
    for with the plan option, on the headline workload: every head against the oracle, both output types, and
    the padded rows exactly zero.  (Left to itself the library runs the third form here.)"""
    c = W.config(5)
    Q, K, V = W.qkv_bits(c.B, c.H, c.S, c.d, c.dtype, c.std, c.seed)
    masks = W.dense_mask(c.mask, c.B, c.H, c.S)
    with smha.Plan.from_desc(c.mask, c.B, c.H, c.S, block=c.block, head_dim=c.d, force=smha.SMHA_KERNEL_BLOCK, block_form=form) as plan:
        assert plan.info()["n_gathered"] == 0 and plan.info()["n_split_rows"] > 0
        assert smha.smha_kernel_name(plan.handle, c.d, smha.SMHA_F16) == ("smha_block_fwd16" if form == 3 else "smha_block_fwd")
        for out_f32 in (False, True):
            got = run_case(torch_mod, smha, Q, K, V, c.dtype, masks, 0, out_f32=out_f32, plan=plan, what=f"{c.name}/form {form}")
            assert np.all(got[:, :, c.mask.valid_len[0]:, :] == 0.0)


@pytest.mark.parametrize("form", [1, 3])
@pytest.mark.parametrize("S,d,dtype", [(100, 128, "f16"), (130, 128, "bf16"), (1000, 96, "f16"), (2500, 128, "f16"), (2500, 120, "bf16")])
def test_first_and_third_form_ragged_and_split(torch_mod, smha, S, d, dtype, form):
    """Both forms at ragged lengths, with empty 128-row groups, fully masked rows, part tiles, heads narrower
    than 128 and (at 2500) groups that are split between workgroups."""
    B, H = 2, 3
    Q, K, V = W.qkv_bits(B, H, S, d, dtype, 1.0, seed=S + d)
    rng = np.random.default_rng(S)
    masks = np.zeros((1, H, S, S), dtype=np.uint8)
    ii, jj = np.indices((S, S))
    masks[0, 0] = (np.abs(ii - jj) <= 40) | (jj < 70) | (ii < 70)           # band + global rows and columns: a long list to split
    masks[0, 1] = (rng.random((S, S)) < 0.3) & (jj <= ii)                       # scattered causal: part tiles everywhere
    masks[0, 1, S // 2] = 0                                                    # a query without keys
    masks[0, 2, : S // 3, : S // 2] = 1                                        # full tiles, and query groups with nothing at all
    with smha.Plan.from_dense(masks, head_dim=d, force=smha.SMHA_KERNEL_BLOCK, no_gather=True, block_form=form) as plan:
        got = run_case(torch_mod, smha, Q, K, V, dtype, masks, 0, out_f32=True, plan=plan, what=f"form {form} ragged {S}")
        assert np.all(got[:, 1, S // 2] == 0.0) and np.all(got[:, 2, S // 3:] == 0.0)
        run_case(torch_mod, smha, Q, K, V, dtype, masks, 0, plan=plan, what=f"form {form} ragged {S} 16-bit out")


def test_plan_that_holds_only_the_row_format(torch_mod, smha):
    """A scattered mask without build_both: the selector takes the row-wise kernel and the plan keeps no block
    lists at all; forward runs (and forcing the block kernel is refused)."""
    S, d = 2048, 64
    m = W.scattered_spec(S, 8, 3)
    Q, K, V = W.qkv_bits(2, 4, S, d, "f16", 1.0, 77)
    with smha.Plan.from_dense(m, head_dim=d) as plan:
        info = plan.info()
        assert info["kernel"] == smha.SMHA_KERNEL_ROW and not info["has_block_kernel_lists"]
        run_case(torch_mod, smha, Q, K, V, "f16", m, 0, heads=[(0, 0), (1, 3)], plan=plan, what="row-only plan")
        q = to_dev(torch_mod, Q, "f16")
        with pytest.raises(smha.SmhaError):
            plan.forward(q, q, q, kernel=smha.SMHA_KERNEL_BLOCK)
