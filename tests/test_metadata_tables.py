"""The segment-packing tables exactly as the kernels read them (exported by plora_debug_metadata,
include/plora_debug.h) against a brute-force construction from the description: plain loops over
rows, segments and adapters, nothing shared with the library.  Integer work, compared bit for bit
(section 2.4: a token row must reach the adapter of its own segment)."""
import numpy as np
import pytest

from paper_2508_02932_amd import plora


def pad(v, a):
    return (v + a - 1) // a * a


def brute_force(T, D, seg_off, seg_adapter, rank, ap_rows=None):
    ap_rows = D if ap_rows is None else ap_rows     # rows of the padded [rows][rp] operand: d_in, or d_out when W is [d_out][d_in]
    n_seg, n_ad = len(seg_adapter), len(rank)
    seg = []
    h = hb = zt = blk = 0
    blk_seg = []
    for s in range(n_seg):
        lo, hi, a = seg_off[s], seg_off[s + 1], seg_adapter[s]
        r = rank[a] if a >= 0 else 0
        rp, r16, lp = pad(r, 64), pad(r, 16), pad(hi - lo, 64)
        seg.append(dict(row0=lo, row1=hi, adapter=a, r=r, rp=rp, r16=r16, blk0=blk, lp=lp, h_off=h, hb_off=hb, zt_off=zt))
        if a >= 0:
            for t in range(lo, hi):                     # row by row: a new block every 128 rows of the segment
                if (t - lo) % 128 == 0:
                    blk_seg.append(s)
                    blk += 1
            h += (hi - lo) * r
            hb += (hi - lo) * rp
            zt += r16 * lp
    ad, at, ap, r16_off, list0 = [], 0, 0, 0, 0
    seg_list = []
    for k in range(n_ad):
        own = [s for s in range(n_seg) if seg_adapter[s] == k and seg_off[s + 1] > seg_off[s]]
        tokens = sum(seg_off[s + 1] - seg_off[s] for s in own)
        ad.append(dict(r=rank[k], rp=pad(rank[k], 64), r16=pad(rank[k], 16), at_off=at, ap_off=ap, r16_off=r16_off,
                       seg_list0=list0, n_own=len(own), tokens=tokens))
        seg_list += own
        list0 += len(own)
        at += pad(rank[k], 16) * D
        ap += pad(rank[k], 64) * ap_rows
        r16_off += pad(rank[k], 16)
    by_tokens = sorted(range(n_ad), key=lambda k: (-ad[k]["tokens"], k))
    row_seg = np.full(T, -1)
    for s in range(n_seg):
        row_seg[seg_off[s]:seg_off[s + 1]] = s
    tiles = []
    for m0 in range(0, T, 256):
        segs = []
        for t in range(m0, min(m0 + 256, T)):           # row by row
            s = int(row_seg[t])
            if seg_adapter[s] >= 0 and s not in segs:
                segs.append(s)
        tiles.append(dict(segs=segs, own_ext=sum(seg[s]["rp"] // 64 for s in segs)))
    for tl in tiles:
        tl["n_ext"] = tl["own_ext"]
    return seg, ad, by_tokens, seg_list, blk_seg, tiles, h, max([pad(rank[seg_adapter[s]], 16) for s in range(n_seg)
                                                                 if seg_adapter[s] >= 0 and seg_off[s + 1] > seg_off[s]] + [0])


def check(T, D, K, seg_off, seg_adapter, rank, scale, w_layout=0):
    d = plora.Desc(T, D, K, np.array(seg_off), np.array(seg_adapter), np.array(rank), np.array(scale), plora.PLORA_BF16,
                   w_layout)
    info, tabs, image = plora.plora_debug_metadata(d)
    seg, ad, by_tokens, seg_list, blk_seg, tiles, h_elems, max_r16 = brute_force(T, D, seg_off, seg_adapter, rank,
                                                                                 K if w_layout else D)
    n_seg = len(seg_adapter)
    hdr = tabs["hdr"]
    assert (hdr["T"], hdr["D"], hdr["K"], hdr["n_seg"], hdr["n_adapters"]) == (T, D, K, n_seg, len(rank))
    assert int(hdr["w_out_in"]) == w_layout and int(hdr["at_base"]) == 0
    assert hdr["n_blocks"] == len(blk_seg) == info.n_blocks and hdr["max_r16"] == max_r16 == info.max_r16
    assert info.h_elems == h_elems == plora.plora_h_elems(d)
    for s in range(n_seg):
        for f, v in seg[s].items():
            assert int(tabs["seg"][s][f]) == v, (s, f)
    for k in range(len(rank)):
        for f, v in ad[k].items():
            assert int(tabs["ad"][k][f]) == v, (k, f)
        assert float(tabs["ad"][k]["scale"]) == np.float32(scale[k])
        assert int(tabs["ad"][k]["by_tokens"]) == by_tokens[k]
        # exported without pointers: B is null, the packed A^T buffer starts at address 0
        assert int(tabs["ad"][k]["ext_b"]) == (2 * ad[k]["at_off"] if w_layout else 0)
    assert tabs["seg_list"].tolist() == seg_list
    assert tabs["blk_seg"].tolist() == blk_seg
    assert info.n_tiles == len(tiles)
    for i, tl in enumerate(tiles):
        rec = tabs["tile"][i]
        assert int(rec["n_ext"]) == tl["n_ext"] and int(rec["n_own"]) == len(tl["segs"]), i
        assert int(rec["first_seg"]) == (tl["segs"][0] if tl["segs"] else n_seg)
        assert int(rec["third_seg"]) == (tl["segs"][2] if len(tl["segs"]) > 2 else n_seg)
        for j, s in enumerate(tl["segs"][:2]):
            q = rec["s"][j]
            assert (int(q["row0"]), int(q["row1"]), int(q["rp"]), int(q["r"]), int(q["hb_off"]), int(q["ap_off"])) == \
                (seg[s]["row0"], seg[s]["row1"], seg[s]["rp"], seg[s]["r"], seg[s]["hb_off"], ad[seg_adapter[s]]["ap_off"])
            assert int(q["B"]) == (2 * ad[seg_adapter[s]]["at_off"] if w_layout else 0)
    # the order the GEMMs walk the row tiles in: longest extension first (8 steps and more are one class), ties in row order
    want_order = sorted(range(len(tiles)), key=lambda i: (-min(tiles[i]["n_ext"], 8), i))
    assert tabs["tile_order"].tolist() == want_order
    # launch plans and workspace: ranges and sizes
    for v in (info.shrink_splits, info.dh_splits, info.da_splits, info.db_splits):
        assert 1 <= v <= 8
    assert info.da_tile_cols in (128, 256) and info.db_tile_cols in (128, 256)
    assert info.r16_total == sum(pad(r, 16) for r in rank)
    assert info.n_active == sum(1 for a in ad if a["tokens"] > 0)
    offs = [info.ws_zero, info.ws_meta, info.ws_desc, info.ws_at, info.ws_ap, info.ws_hb, info.ws_zt_h, info.ws_zt_g,
            info.ws_hf, info.ws_gf, info.ws_part, info.ws_wpart, info.ws_total]
    assert all(b >= a for a, b in zip(offs, offs[1:])) and all(o % 256 == 0 for o in offs[:-1])
    assert info.ws_total == plora.plora_workspace_bytes(d)
    assert info.ws_desc - info.ws_meta >= info.table_bytes
    assert info.ws_ap - info.ws_at >= 2 * D * info.r16_total
    assert info.ws_hb - info.ws_ap >= 2 * (K if w_layout else D) * sum(pad(r, 64) for r in rank)
    hb_elems = sum((g["row1"] - g["row0"]) * g["rp"] for g in seg if g["adapter"] >= 0)
    zt_elems = sum(g["r16"] * g["lp"] for g in seg if g["adapter"] >= 0)
    assert info.ws_zt_h - info.ws_hb >= 2 * hb_elems
    assert info.ws_zt_g - info.ws_zt_h >= 2 * zt_elems and info.ws_hf - info.ws_zt_g >= 2 * zt_elems
    assert info.ws_gf - info.ws_hf >= 4 * h_elems
    assert info.ws_wpart - info.ws_part >= 4 * max(info.shrink_splits, info.dh_splits) * len(blk_seg) * 128 * max_r16
    need = max(info.da_splits * info.r16_total * D * 4 if info.da_splits > 1 else 0,
               info.db_splits * info.r16_total * K * 4 if info.db_splits > 1 else 0)
    assert info.ws_total - info.ws_wpart >= need
    return info


@pytest.mark.parametrize("seed", range(12))
def test_tables_equal_brute_force_random_layouts(seed):
    rng = np.random.default_rng(100 + seed)
    n_ad = int(rng.integers(1, 9))
    n_seg = int(rng.integers(1, 14))
    lens = rng.integers(0, 700, size=n_seg)
    lens[rng.integers(n_seg)] = 0                                   # an empty segment
    if seed % 3 == 0:
        lens[rng.integers(n_seg)] = 1
    seg_off = np.concatenate([[0], np.cumsum(lens)]).astype(int).tolist()
    seg_adapter = rng.integers(-1, n_ad, size=n_seg).tolist()       # base-only rows, repeated and unused adapters
    rank = rng.integers(1, 129, size=n_ad).tolist()
    scale = (rng.integers(1, 9, size=n_ad) / 4.0).tolist()
    check(seg_off[-1], 8 * int(rng.integers(1, 40)), 8 * int(rng.integers(1, 40)), seg_off, seg_adapter, rank, scale,
          w_layout=seed % 2)


def test_tables_many_blocks_and_tiny_segments():
    """More than 256 token blocks; several segments inside one 256-row tile (the third_seg walk)."""
    lens = [40000, 3, 5, 7, 60, 1, 255, 256, 257, 0, 130]
    seg_off = np.concatenate([[0], np.cumsum(lens)]).tolist()
    seg_adapter = [0, 1, 2, -1, 3, 1, 0, 2, 2, 3, -1]
    info = check(seg_off[-1], 64, 128, seg_off, seg_adapter, [128, 8, 65, 16], [2.0, 1.0, 0.5, 4.0])
    assert info.n_blocks > 256


def test_tables_edge_descriptions():
    check(0, 16, 16, [0, 0], [0], [8], [1.0])                       # empty batch
    check(300, 16, 24, [0, 300], [-1], [8], [1.0])                  # base only
    check(1, 8, 8, [0, 1], [0], [1], [1.0])                         # one token, rank 1
    d = plora.Desc(0, 16, 16, np.zeros(1), np.zeros(0), np.zeros(0), np.zeros(0), plora.PLORA_BF16)
    info, tabs, _ = plora.plora_debug_metadata(d)                   # no segments, no adapters
    assert info.n_tiles == 0 and info.n_blocks == 0


def test_the_five_configurations_fit_one_preparation_launch():
    """The compact description of every benchmark configuration travels in one kernel argument
    (3584 bytes), so a call needs a single preparation launch."""
    from paper_2508_02932_amd import workloads as wl
    for idx in range(1, 6):
        for lin in wl.config(idx):
            lay = lin.layout
            d = plora.Desc(lay.T, lin.D, lin.K, lay.seg_off, lay.seg_adapter, lay.rank, lay.scale,
                           plora.PLORA_BF16 if lin.dtype == "bf16" else plora.PLORA_F32)
            info, _, _ = plora.plora_debug_metadata(d)
            assert info.desc_words * 4 <= 3584, (lin.name, info.desc_words)
