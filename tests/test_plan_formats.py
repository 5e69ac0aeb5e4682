"""Host-side planner against the format oracle (bit-exact), the selector against the
paper's formula, and the C ABI surface.  No GPU needed: plans are built host-only."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2506_06095_amd as smha
import workloads as W
from oracle import formats, selector
from paper_2506_06095_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BSR_KEYS = ["load_row_ptr", "load_col_idx", "flags", "full_row_ptr", "full_col_idx",
            "part_row_ptr", "part_col_idx"]


def check_plan_against_oracle(plan, masks, bs):
    Bm, Hm, S, Sk = masks.shape
    info = plan.info()
    assert (info["S"], info["Sk"], info["Bm"], info["Hm"], info["block"]) == (S, Sk, Bm, Hm, bs)
    nnz = nvalid = nfull = npart = v16 = 0
    for mi in range(Bm * Hm):
        M = masks[mi // Hm, mi % Hm]
        f = formats.bsr(M, bs)
        for k in BSR_KEYS:
            got = plan.export(k, mi)
            assert got.dtype == f[k].dtype and np.array_equal(got, f[k]), (k, mi)
        assert np.array_equal(plan.export("bitmap", mi).reshape(-1, bs), f["bitmap"]), mi
        rp, ci = formats.csr(M)
        assert np.array_equal(plan.export("row_ptr", mi), rp)
        assert np.array_equal(plan.export("col_idx", mi), ci)
        if bs == 64:
            assert np.array_equal(plan.export("bitmap_it8", mi).reshape(-1, 64),
                                  formats.bitmap_inner_tiles(f["bitmap"]))
        nnz += f["nnz"]
        nvalid += len(f["load_col_idx"]); nfull += len(f["full_col_idx"]); npart += len(f["part_col_idx"])
        v16 += selector.valid16(M)
    assert (info["nnz"], info["n_valid"], info["n_full"], info["n_part"], info["n_valid16"]) == \
           (nnz, nvalid, nfull, npart, v16)
    thr = selector.threshold(v16 / (Bm * Hm), S, Sk=Sk)
    assert info["eq1_threshold"] == pytest.approx(thr, abs=1e-12) or (np.isinf(thr) and np.isinf(info["eq1_threshold"]))


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_benchmark_configs_dense_and_description_plans_match_oracle(idx):
    c = W.config(idx)
    masks = W.dense_mask(c.mask, c.B, c.H, c.S)
    if idx == 4:
        masks = masks[:, :3].copy()  # three of the sixteen per-head masks keep this quick
    with smha.Plan.from_dense(masks, block=c.block, build_both=True, device_id=-2, head_dim=c.d) as p:
        check_plan_against_oracle(p, masks, c.block)
    H = 3 if idx == 4 else c.H
    with smha.Plan.from_desc(c.mask, c.B, H, c.S, block=c.block, build_both=True, device_id=-2,
                             head_dim=c.d) as p:
        check_plan_against_oracle(p, masks, c.block)


@pytest.mark.parametrize("bs", [16, 32, 64])
@pytest.mark.parametrize("S", [1, 15, 64, 100, 130, 257])
def test_ragged_sizes_and_all_block_sizes(S, bs):
    rng = np.random.default_rng(S * 100 + bs)
    masks = (rng.random((2, 2, S, S)) < 0.3).astype(np.uint8)
    masks[0, 0] = 0                       # an empty mask
    masks[0, 1] = 1                       # a dense mask
    masks[1, 0, :, : S // 2] = 7          # nonzero bytes other than 1 count as "attend"
    with smha.Plan.from_dense(masks, block=bs, build_both=True, device_id=-2) as p:
        check_plan_against_oracle(p, (masks != 0).astype(np.uint8), bs)


@pytest.mark.parametrize("bs", [16, 32, 64])
@pytest.mark.parametrize("Sq,Sk", [(1, 500), (100, 300), (257, 64), (130, 131), (64, 1)])
def test_fewer_or_more_queries_than_keys(Sq, Sk, bs):
    rng = np.random.default_rng(Sq * 1000 + Sk + bs)
    masks = (rng.random((2, 2, Sq, Sk)) < 0.3).astype(np.uint8)
    masks[0, 0] = 0
    masks[0, 1] = 1
    masks[1, 0, :, Sk // 2:] = 0
    with smha.Plan.from_dense_rect(masks, block=bs, build_both=True, device_id=-2) as p:
        check_plan_against_oracle(p, masks, bs)
        rp, ci = p.export("row_ptr", 3), p.export("col_idx", 3)
        assert np.array_equal(formats.dense_from_csr(rp, ci, Sq, Sk), masks[1, 1])
        f = {k: p.export(k, 3) for k in ("load_row_ptr", "load_col_idx", "flags")}
        f["bitmap"] = p.export("bitmap", 3).reshape(-1, bs)
        assert np.array_equal(formats.dense_from_bsr(f, Sq, bs, Sk), masks[1, 1])
    with pytest.raises(ValueError):
        smha.Plan.from_dense(masks, device_id=-2) if Sq != Sk else (_ for _ in ()).throw(ValueError())


def test_description_patterns_match_dense_generators():
    S = 300
    specs = [
        W.MaskSpec(flags=0),
        W.MaskSpec(flags=W.CAUSAL),
        W.MaskSpec(flags=W.WINDOW, window_left=5, window_right=0),
        W.MaskSpec(flags=W.WINDOW | W.GLOBAL, window_left=9, window_right=3, n_global=4),
        W.MaskSpec(flags=W.CAUSAL | W.STRIDED, stride=7, stride_phase=3),
        W.MaskSpec(flags=W.BLOCK_RANDOM, block=24, keep_p=0.3, seed=99, per_head=True),
        W.MaskSpec(flags=W.BIGBIRD | W.CAUSAL, block=16, n_window_blocks=3, n_global_blocks=1,
                   n_random_blocks=2, seed=5, per_head=True),
        W.MaskSpec(flags=W.BIGBIRD | W.PADDING, block=32, n_window_blocks=1, n_global_blocks=2,
                   n_random_blocks=30, seed=6, valid_len=(300, 17, 0)),
        W.MaskSpec(flags=W.WINDOW | W.PADDING, window_left=400, window_right=400, valid_len=(1, 299, 150)),
    ]
    for spec in specs:
        B, H = 3, 2
        masks = W.dense_mask(spec, B, H, S)
        with smha.Plan.from_desc(spec, B, H, S, block=32, build_both=True, device_id=-2) as p:
            check_plan_against_oracle(p, masks, 32)


def test_selector_follows_eq1_and_can_be_forced():
    c = W.config(3)
    with smha.Plan.from_desc(c.mask, 1, 1, c.S, selector=smha.SMHA_SELECTOR_PAPER_EQ1, device_id=-2) as p:
        i = p.info()
        assert i["kernel"] == smha.SMHA_KERNEL_BLOCK and i["eq1_threshold"] > 0
        assert not i["has_row_format"]
        with pytest.raises(smha.SmhaError):
            p.export("row_ptr")
    # one 16x16 tile per tile row at S = 4096: 1/256 - 1.2/64 < 0 -> row-wise
    diag = W.MaskSpec(flags=W.WINDOW)
    with smha.Plan.from_desc(diag, 1, 1, 4096, selector=smha.SMHA_SELECTOR_PAPER_EQ1, device_id=-2) as p:
        i = p.info()
        assert i["kernel"] == smha.SMHA_KERNEL_ROW and i["eq1_threshold"] == pytest.approx(1 / 256 - 1.2 / 64)
        assert i["has_row_format"] and not i["has_block_kernel_lists"]
    with smha.Plan.from_desc(diag, 1, 1, 16, selector=smha.SMHA_SELECTOR_PAPER_EQ1, device_id=-2) as p:
        assert p.info()["kernel"] == smha.SMHA_KERNEL_ROW
    with smha.Plan.from_desc(diag, 1, 1, 4096, force=smha.SMHA_KERNEL_BLOCK, device_id=-2) as p:
        assert p.info()["kernel"] == smha.SMHA_KERNEL_BLOCK
    # calibrated model: scattered columns -> row-wise, block-structured -> block-wise
    scat = W.scattered_spec(2048, 8, 3)
    with smha.Plan.from_dense(scat, device_id=-2) as p:
        assert p.info()["kernel"] == smha.SMHA_KERNEL_ROW
    from dataclasses import replace
    bb = replace(W.config(5).mask, valid_len=(2000,))
    with smha.Plan.from_desc(bb, 1, 1, 2048, head_dim=128, device_id=-2) as p:
        assert p.info()["kernel"] == smha.SMHA_KERNEL_BLOCK


def test_work_items_cover_every_tile_exactly_once():
    c = W.config(5)
    with smha.Plan.from_desc(c.mask, 1, 1, c.S, device_id=-2) as p:
        i = p.info()
        assert i["n_split_rows"] == 1             # the 128-row group holding the two global tile rows
        assert i["n_tiles64"] == i["n_valid"]
        assert i["n_tiles64"] / 2 <= i["n_union"] <= i["n_tiles64"]
        assert i["n_items"] > 64


def test_error_paths_return_status_codes():
    ones = np.ones((1, 1, 8, 8), np.uint8)
    with pytest.raises(smha.SmhaError) as e:
        smha.Plan.from_dense(ones, block=48, device_id=-2)
    assert e.value.status == 2
    with pytest.raises(smha.SmhaError) as e:
        smha.Plan.from_dense(ones, force=9, device_id=-2)
    assert e.value.status == 1
    with pytest.raises(smha.SmhaError) as e:
        smha.Plan.from_desc(W.MaskSpec(flags=W.STRIDED, stride=0), 1, 1, 8, device_id=-2)
    assert e.value.status == 1
    with pytest.raises(smha.SmhaError) as e:
        smha.Plan.from_desc(W.MaskSpec(flags=W.PADDING), 1, 1, 8, device_id=-2)
    assert e.value.status == 1
    with pytest.raises(smha.SmhaError) as e:
        smha.Plan.from_desc(W.MaskSpec(flags=W.PADDING, valid_len=(9,)), 1, 1, 8, device_id=-2)
    assert e.value.status == 1
    lib = binding._load()
    assert lib.smha_plan_from_dense(None, 0, 1, 1, 8, None, None) == 1
    assert lib.smha_plan_info(None, None) == 1
    lib.smha_plan_destroy(None)
    assert smha.smha_status_string(0) == "ok" and "unknown" in smha.smha_status_string(77)
    # a host-only plan cannot run: forward must say so rather than fall back to anything
    with smha.Plan.from_dense(ones, device_id=-2) as p:
        buf = (ctypes.c_char * 4096)()
        addr = (ctypes.addressof(buf) + 15) & ~15
        st = lib.smha_forward(ctypes.c_void_p(p.handle), addr, addr, addr, addr, 1, 1, 64, 0, 0,
                              None, None, None, None, 0.0, 0, None)
        assert st == 5
        assert lib.smha_forward(ctypes.c_void_p(p.handle), addr, addr, addr, addr, 1, 1, 100, 0, 0,
                                None, None, None, None, 0.0, 0, None) == 2
        assert lib.smha_forward(ctypes.c_void_p(p.handle), addr + 2, addr, addr, addr, 1, 1, 64, 0, 0,
                                None, None, None, None, 0.0, 0, None) == 2
        assert lib.smha_forward(ctypes.c_void_p(p.handle), None, addr, addr, addr, 1, 1, 64, 0, 0,
                                None, None, None, None, 0.0, 0, None) == 1
        # strides: rows that overlap (seq stride < d), a stride that is not a multiple of 8, and a
        # (batch, head) slice beyond the 2 GiB the kernels address with 32-bit offsets
        I3 = ctypes.c_int64 * 3
        ok = I3(8 * 64, 8 * 64, 64)
        for bad in (I3(8 * 64, 8 * 64, 32), I3(8 * 64, 8 * 64, 68), I3(1 << 40, 1 << 34, 1 << 28)):
            for pos in range(4):
                strides = [ok, ok, ok, ok]
                strides[pos] = bad
                assert lib.smha_forward(ctypes.c_void_p(p.handle), addr, addr, addr, addr, 1, 1, 64, 0, 0,
                                        *strides, 0.0, 0, None) == 2
        assert lib.smha_forward(ctypes.c_void_p(p.handle), addr, addr, addr, addr, 1, 1, 64, 0, 0,
                                ok, ok, ok, ok, 0.0, 0, None) == 5
    with smha.Plan.from_dense(np.ones((2, 3, 8, 8), np.uint8), device_id=-2) as p:
        st = lib.smha_forward(ctypes.c_void_p(p.handle), addr, addr, addr, addr, 4, 3, 64, 0, 0,
                              None, None, None, None, 0.0, 0, None)
        assert st == 3


def test_bench_refuses_more_than_one_gpu_and_says_so():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "smha.h")).read()
    names = set(re.findall(r"\b(smha_[a-z_0-9]+)\s*\(", text))
    assert {"smha_plan_from_dense", "smha_plan_from_desc", "smha_plan_info", "smha_plan_export",
            "smha_forward", "smha_plan_destroy", "smha_status_string", "smha_kernel_name"} <= names
    lib = ctypes.CDLL(smha.library_path())
    for n in names:
        assert hasattr(lib, n), n


def check_work_order(plan, B, H, slots, fine=False):
    """Every (batch*head, item) once, on the XCD of its head, ranks compact, loads balanced."""
    info = plan.info()
    Bm, Hm = info["Bm"], info["Hm"]
    lengths, off = [], [0]
    for m in range(Bm * Hm):
        it = plan.export("kernel_items_fine" if fine else "kernel_items", m).reshape(-1, 8)
        lengths.append(it[:, 2] - it[:, 1])
        off.append(off[-1] + len(it))
    all_len = np.concatenate(lengths)
    table, per = plan.work_order(B, H, slots, fine)
    assert 0 < per <= slots
    pairs = table[16:].reshape(-1, 2)
    seen = set()
    ratio = 0.0
    for x in range(8):
        at, n = int(table[x]), int(table[8 + x])
        assert n % per == 0
        lst = pairs[at:at + n].reshape(-1, per, 2)          # [turn][rank]
        loads = np.zeros(per, np.int64)
        for r in range(per):
            live = lst[:, r, 0] >= 0
            assert not np.any(live[1:] & ~live[:-1])           # a rank's unused turns are its last ones
            for bh, idx in lst[live, r]:
                assert bh % 8 == x and 0 <= bh < B * H
                mask = (bh // H if Bm > 1 else 0) * Hm + (bh % H if Hm > 1 else 0)
                assert off[mask] <= idx < off[mask + 1]
                assert (bh, idx) not in seen
                seen.add((int(bh), int(idx)))
                loads[r] += 2 + all_len[idx]
            heads = lst[live, r, 0]
            assert np.all(np.diff(heads) >= 0)                 # head after head
        # greedy longest-first: no workgroup exceeds its XCD's mean by more than the longest item
        assert loads.max() <= loads.mean() + 2 + int(all_len.max())
        if loads.sum():
            ratio = max(ratio, float(loads.max() / loads.mean()))
    want = {(bh, i) for bh in range(B * H)
            for i in range(off[(bh // H if Bm > 1 else 0) * Hm + (bh % H if Hm > 1 else 0)],
                           off[(bh // H if Bm > 1 else 0) * Hm + (bh % H if Hm > 1 else 0) + 1])}
    assert seen == want
    return ratio


def test_work_order_covers_every_item_once_and_balances():
    c = W.config(2)
    with smha.Plan.from_desc(c.mask, c.B, c.H, c.S, block=64, head_dim=c.d, force=smha.SMHA_KERNEL_BLOCK) as plan:
        check_work_order(plan, c.B, c.H, 128)
        check_work_order(plan, c.B, c.H, 128, fine=True)
        check_work_order(plan, c.B, c.H, 3)      # many turns per workgroup
        check_work_order(plan, 1, 1, 64)         # fewer items than workgroups, seven idle XCDs
    # per-head masks of unequal weight, a head count that is no multiple of 8
    spec = W.MaskSpec(flags=W.WINDOW | W.GLOBAL | W.BLOCK_RANDOM | W.PADDING, window_left=64, window_right=64,
                      n_global=70, keep_p=0.2, seed=5, per_head=True, valid_len=(2048, 1500))
    with smha.Plan.from_desc(spec, 2, 5, 2048, block=64, head_dim=64, force=smha.SMHA_KERNEL_BLOCK) as plan:
        check_work_order(plan, 2, 5, 16)
        check_work_order(plan, 2, 5, 16, fine=True)
        assert check_work_order(plan, 2, 5, 3) <= 1.2
    with smha.Plan.from_dense(np.zeros((1, 1, 256, 256), np.uint8), force=smha.SMHA_KERNEL_BLOCK) as plan:
        check_work_order(plan, 4, 4, 64)         # empty lists only (the items still write zeros)
    with smha.Plan.from_dense(np.ones((2, 3, 64, 64), np.uint8), force=smha.SMHA_KERNEL_BLOCK) as plan:
        with pytest.raises(smha.SmhaError):
            plan.work_order(3, 3, 64)            # batch does not match the plan's masks


def mask_from_kernel_lists(plan, mi, Sq, Sk, which="kernel_items", longest=64):
    """Rebuild mask `mi` from the block kernel's work lists, counting how often each entry is visited."""
    items = plan.export(which, mi).reshape(-1, 8)
    ents = plan.export("kernel_entries").reshape(-1, 4)
    bmp = plan.export("kernel_bitmaps").reshape(-1, 64)
    keys = plan.export("kernel_gather_keys").reshape(-1, 64)
    cnt = np.zeros((Sq + 128, Sk + 192), dtype=np.int32)
    bit = np.arange(64, dtype=np.uint64)
    for qtile, begin, end, slot, gbegin, gcount, _, _ in items:
        gath = [e for e in range(begin, end) if ents[e, 3] > 0]
        assert len(gath) == gcount <= 16 and end - begin <= longest
        assert gath == list(range(end - gcount, end))        # gathered tiles close an item's list
        for t, e in enumerate(gath):
            assert ents[e, 3] - 1 == gbegin + t
        for e in range(begin, end):
            col, c0, c1, g = ents[e]
            kk = keys[g - 1] if g > 0 else np.arange(64) + 64 * col
            for side, code in enumerate((c0, c1)):
                if code == -2:
                    continue
                r0 = qtile * 128 + 64 * side
                if code == -1:
                    blk = np.ones((64, 64), dtype=np.int32)
                else:
                    blk = ((bmp[code][:, None] >> bit[None, :]) & np.uint64(1)).astype(np.int32)
                np.add.at(cnt, (np.arange(r0, r0 + 64)[:, None], np.minimum(kk, Sk + 191)[None, :]), blk)
    return cnt


def test_fine_work_items_cut_every_list_to_16_steps_and_number_their_partials():
    spec = W.table2_spec("causal")
    with smha.Plan.from_desc(spec, 1, 1, 4096, head_dim=64, device_id=-2, force=smha.SMHA_KERNEL_BLOCK) as p:
        coarse = p.export("kernel_items").reshape(-1, 8)
        fine = p.export("kernel_items_fine").reshape(-1, 8)
        assert len(coarse) == 32 and (coarse[:, 3] == -1).all()            # nothing split at the coarse grain
        assert (fine[:, 2] - fine[:, 1]).max() == 16 and len(fine) > len(coarse)
        for g in range(32):                                                # each group: its parts tile its list
            whole = coarse[coarse[:, 0] == g][0]
            parts = fine[fine[:, 0] == g]
            parts = parts[np.argsort(parts[:, 1])]
            assert parts[0, 1] == whole[1] and parts[-1, 2] == whole[2]
            assert np.array_equal(parts[1:, 1], parts[:-1, 2])
            if len(parts) == 1:
                assert parts[0, 3] == -1
            else:
                assert np.array_equal(parts[:, 3], parts[0, 3] + np.arange(len(parts)))   # consecutive scratch slots
        split = fine[fine[:, 3] >= 0][:, 3]
        assert np.array_equal(np.sort(split), np.arange(len(split)))      # slots dense from 0
    # a mask whose lists are short has one grain only: the fine export is the coarse one
    with smha.Plan.from_desc(W.table2_spec("sliding_window"), 1, 1, 2048, head_dim=64, device_id=-2,
                             force=smha.SMHA_KERNEL_BLOCK) as p:
        assert np.array_equal(p.export("kernel_items"), p.export("kernel_items_fine"))


@pytest.mark.parametrize("seed", range(12))
def test_kernel_work_lists_of_random_masks_cover_each_unmasked_entry_once_and_order_every_item(seed):
    """Random mixtures of bands, long rows, scattered columns and blocks, square and rectangular, ragged sizes."""
    rng = np.random.default_rng(500 + seed)
    Sq = int(rng.integers(1, 700))
    Sk = Sq if rng.random() < 0.6 else int(rng.integers(1, 1500))
    Hm = int(rng.integers(1, 3))
    i, j = np.arange(Sq)[:, None], np.arange(Sk)[None, :]
    masks = np.zeros((1, Hm, Sq, Sk), dtype=np.uint8)
    for h in range(Hm):
        m = np.zeros((Sq, Sk), dtype=bool)
        if rng.random() < 0.7:
            m |= np.abs(i * Sk // max(Sq, 1) - j) <= int(rng.integers(0, 90))
        if rng.random() < 0.5:
            m |= (i < int(rng.integers(0, 70))) | (j < int(rng.integers(0, 20)))
        if rng.random() < 0.5:
            m |= rng.random((Sq, Sk)) < rng.choice([0.002, 0.02])
        if rng.random() < 0.5:
            blk = rng.random(((Sq + 63) // 64, (Sk + 63) // 64)) < 0.15
            m |= np.kron(blk, np.ones((64, 64), dtype=bool))[:Sq, :Sk]
        if rng.random() < 0.3:
            m &= j <= i * Sk // max(Sq, 1)
        masks[0, h] = m
    make = smha.Plan.from_dense if Sq == Sk else smha.Plan.from_dense_rect
    with make(masks, device_id=-2, force=smha.SMHA_KERNEL_BLOCK, no_gather=bool(seed % 3 == 0)) as plan:
        assert plan.info()["nnz"] == int(masks.sum())
        for mi in range(Hm):
            for which, longest in (("kernel_items", 64), ("kernel_items_fine", 16)):
                cnt = mask_from_kernel_lists(plan, mi, Sq, Sk, which, longest)
                assert np.array_equal(cnt[:Sq, :Sk], masks[0, mi].astype(np.int32)), (seed, mi, which)
                assert cnt[Sq:].sum() == 0 and cnt[:, Sk:].sum() == 0
        for B, H, slots, fine in ((1, Hm, 64, False), (3, Hm if Hm > 1 else 5, 32, True)):
            check_work_order(plan, B, H, slots, fine=fine)


@pytest.mark.parametrize("name", ["cfg3", "strided_cols", "scattered", "rect_scattered", "mixed_long_rows"])
def test_kernel_work_lists_with_gathered_tiles_cover_the_mask_exactly_once(name):
    rng = np.random.default_rng(11)
    if name == "cfg3":
        c = W.config(3)
        masks = W.dense_mask(c.mask, 1, 1, c.S)
    elif name == "strided_cols":
        masks = W.dense_mask(W.MaskSpec(flags=W.WINDOW | W.STRIDED, window_left=40, window_right=40, stride=37, stride_phase=5), 1, 1, 1000)
    elif name == "scattered":
        masks = W.scattered_spec(700, 3, 5)
    elif name == "rect_scattered":
        masks = (rng.random((1, 2, 200, 3000)) < 0.004).astype(np.uint8)
        masks[0, 1, :, 100:228] = 1
    else:  # a few very long rows (global tokens) next to scattered ones: split groups with gathered tiles
        masks = (rng.random((1, 1, 4500, 4500)) < 0.002).astype(np.uint8)
        masks[0, 0, :64] = 1
        masks[0, 0, :, :8] = 1
    Bm, Hm, Sq, Sk = masks.shape
    make = smha.Plan.from_dense if Sq == Sk else smha.Plan.from_dense_rect
    with make(masks, device_id=-2, force=smha.SMHA_KERNEL_BLOCK) as p, \
            make(masks, device_id=-2, force=smha.SMHA_KERNEL_BLOCK, no_gather=True) as q:
        ip, iq = p.info(), q.info()
        assert ip["n_gathered"] > 0 and iq["n_gathered"] == 0
        assert ip["n_union"] < iq["n_union"]                       # repacking only when it saves steps
        assert ip["n_tiles64"] == iq["n_tiles64"]
        for plan in (p, q):
            for mi in range(Bm * Hm):
                for which, longest in (("kernel_items", 64), ("kernel_items_fine", 16)):
                    cnt = mask_from_kernel_lists(plan, mi, Sq, Sk, which, longest)
                    assert np.array_equal(cnt[:Sq, :Sk], masks[mi // Hm, mi % Hm].astype(np.int32)), (name, mi, which)
                    assert cnt[Sq:].sum() == 0 and cnt[:, Sk:].sum() == 0
        for k in ("load_row_ptr", "load_col_idx", "flags", "bitmap"):  # the exported formats do not change
            assert np.array_equal(p.export(k), q.export(k))


def test_which_form_of_the_block_kernel_a_plan_runs():
    """The library's own choice at 128 columns (host-only plans: nothing runs): the form with eight waves of 16
    rows, except for plans whose tiles are nearly all full and whose lists are long (dense causal), and except
    for plans with gathered tiles; at 256 columns always that form unless tiles are gathered; at 64 columns the
    first form; the plan option overrides."""
    c5 = W.config(5)
    cases = [
        (c5.mask, 1, 2, 8192, 128, {}, "smha_block_fwd16"),
        (W.MaskSpec(flags=W.CAUSAL), 1, 2, 4096, 128, {}, "smha_block_fwd"),        # full tiles, lists of 32 steps
        (W.MaskSpec(flags=W.CAUSAL), 1, 2, 1024, 128, {}, "smha_block_fwd16"),      # short lists
        (W.MaskSpec(flags=W.WINDOW, window_left=32, window_right=32), 1, 2, 4096, 128, {}, "smha_block_fwd16"),
        (W.MaskSpec(flags=W.WINDOW, window_left=32, window_right=32), 1, 2, 4096, 96, {}, "smha_block_fwd16"),
        (c5.mask, 1, 2, 8192, 64, {}, "smha_block_fwd"),
        (c5.mask, 1, 2, 8192, 256, {}, "smha_block_fwd16"),
        (c5.mask, 1, 2, 8192, 256, {"block_form": 1}, "smha_block_fwd"),
        (c5.mask, 1, 2, 8192, 128, {"block_form": 1}, "smha_block_fwd"),
        (c5.mask, 1, 2, 8192, 128, {"block_form": 2}, "smha_block_fwd2"),
        (W.MaskSpec(flags=W.CAUSAL), 1, 2, 4096, 128, {"block_form": 3}, "smha_block_fwd16"),
        (W.MaskSpec(flags=W.CAUSAL | W.WINDOW | W.STRIDED, window_left=70, stride=37, stride_phase=5), 1, 2, 2048, 128, {}, "smha_block_fwd"),
    ]
    for spec, B, H, S, d, extra, want in cases:
        with smha.Plan.from_desc(spec, B, H, S, head_dim=d, device_id=-2, force=smha.SMHA_KERNEL_BLOCK, **extra) as plan:
            got = smha.smha_kernel_name(plan.handle, d, smha.SMHA_F16)
            assert got == want, (spec, S, d, extra, got, want)
    with smha.Plan.from_desc(c5.mask, 1, 2, 8192, head_dim=128, device_id=-2, force=smha.SMHA_KERNEL_ROW) as plan:
        assert smha.smha_kernel_name(plan.handle, 128, smha.SMHA_F16) == "smha_row_fwd"
