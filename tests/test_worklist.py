"""Host work-list compiler against a brute-force enumeration of allowed pairs per tile."""
import itertools

import numpy as np
import pytest

from paper_2503_22796_amd import binding as B

FULL, ARROW, CACHE = 0, 1, 2


def allowed(mode, w, n_text, i, j):
    if mode == FULL:
        return True
    return i < n_text or j < n_text or abs(i - j) <= w


def brute_tiles(mode, w, n_text, N, i0, i1, bn):
    """(tiles with at least one allowed pair, tiles with every pair allowed and no key >= N)."""
    some, every = set(), set()
    for t in range((N + bn - 1) // bn):
        js = range(t * bn, (t + 1) * bn)
        flags = [(j < N) and allowed(mode, w, n_text, i, j) for i in range(i0, i1) for j in js]
        if any(flags):
            some.add(t)
        if all(flags):
            every.add(t)
    return some, every


CASES = [
    # n_text, n_img, bm, bn, [(mode, w)...]
    (5, 40, 8, 4, [(FULL, 0), (ARROW, 0), (ARROW, 3), (ARROW, 9), (CACHE, 0), (ARROW, 39), (ARROW, 100)]),
    (0, 33, 8, 4, [(ARROW, 0), (ARROW, 5), (FULL, 0)]),
    (16, 64, 16, 8, [(FULL, 0), (ARROW, 8), (ARROW, 16), (CACHE, 0)]),
    (7, 0, 8, 4, [(ARROW, 2), (FULL, 0)]),
    (3, 1, 8, 4, [(ARROW, 0)]),
    (12, 50, 8, 8, [(ARROW, 1), (ARROW, 7), (ARROW, 8), (ARROW, 20)]),
    (9, 31, 4, 8, [(ARROW, 2), (ARROW, 11)]),
]


@pytest.mark.parametrize("n_text,n_img,bm,bn,heads", CASES)
@pytest.mark.parametrize("batch", [1, 2])
@pytest.mark.parametrize("n_xcd", [1, 3, 8])
def test_records_match_brute_force(n_text, n_img, bm, bn, heads, batch, n_xcd):
    N = n_text + n_img
    hp = [m for m, _ in heads]
    win = [w for _, w in heads]
    H = len(heads)
    st, laid, copy_heads = B.difa_worklist_build(batch, H, hp, win, n_text, n_img, bm, bn, n_xcd)
    assert st == B.DIFA_OK
    assert list(copy_heads) == [h for h in range(H) if hp[h] == CACHE]
    n_q = (N + bm - 1) // bm
    computed = [h for h in range(H) if hp[h] != CACHE]
    items = laid[laid["q_tile"] >= 0]            # the rest is padding of short queues
    assert len(items) == batch * len(computed) * n_q
    seen = set()
    if n_xcd == 1:
        assert len(laid) == len(items)
        tiles = [int(x) for x in items["n_tiles"]]
        assert tiles == sorted(tiles, reverse=True), "records must be ordered heaviest first"
    else:
        # queue x = positions x, x + n_xcd, ...: equal cost, padding only behind a queue's records
        costs = []
        for x in range(n_xcd):
            q = laid[x::n_xcd]
            real = q["q_tile"] >= 0
            assert not (np.diff(real.astype(int)) > 0).any(), "padding inside a queue"
            costs.append(int(q["n_tiles"][real].sum()))
        heaviest = int(items["n_tiles"].max()) if len(items) else 0
        assert max(costs) - min(costs) <= 2 * heaviest, f"queues out of balance: {costs}"
        # a head is split over at most two neighbouring queues... unless it is cut more than once
        # because it alone outweighs a queue's share
        share = sum(costs) / n_xcd
        for bh in set(items["bh"].tolist()):
            where = sorted({int(i) % n_xcd for i in np.nonzero((laid["bh"] == bh) & (laid["q_tile"] >= 0))[0]})
            head_cost = int(items["n_tiles"][items["bh"] == bh].sum())
            assert len(where) <= 2 + int(head_cost // max(share, 1)), (bh, where)
    for r in items:
        b, h = divmod(int(r["bh"]), H)
        assert 0 <= b < batch and h in computed
        key = (b, h, int(r["q_tile"]))
        assert key not in seen
        seen.add(key)
        i0, i1 = int(r["q_tile"]) * bm, min(N, (int(r["q_tile"]) + 1) * bm)
        mode, w = hp[h], win[h]
        some, every = brute_tiles(mode, w, n_text, N, i0, i1, bn)
        assert r["kv1_begin"] >= r["kv0_end"]
        visited = set(range(0, r["kv0_end"])) | set(range(r["kv1_begin"], r["kv1_end"]))
        assert visited == some, "visited tiles must be exactly the tiles that hold an allowed pair"
        assert r["n_tiles"] == len(visited)
        mask_free = set(range(0, min(r["nm0_end"], r["kv0_end"]))) | \
            set(range(max(r["nm1_begin"], r["kv1_begin"]), min(r["nm1_end"], r["kv1_end"])))
        assert mask_free <= every, "a tile flagged mask-free holds a masked pair"
        assert mask_free == (every & visited), "every mask-free tile should be recognised as such"
        if mode == ARROW and w < n_img - 1:
            assert r["window"] == w
        else:
            assert r["window"] == -1
    assert len(seen) == len(items)


def test_flux_2k_shape_tile_counts():
    # image-only query tile of an arrow head visits 8 text tiles + the band tiles
    bm, bn = B.difa_tile_shape(128)
    st, items, _ = B.difa_worklist_build(1, 2, [ARROW, FULL], [512, 0], 512, 16384, bm, bn, 8)
    assert st == B.DIFA_OK
    items = items[items["q_tile"] >= 0]
    N = 16896
    assert len(items) == 2 * ((N + bm - 1) // bm)
    full = items[items["window"] == -1]
    assert (full["n_tiles"] == N // bn).all() and (full["nm0_end"] == N // bn).all()
    arrow = items[items["window"] == 512]
    mid = arrow[arrow["q_tile"] == 30][0]
    i0 = 30 * bm
    lo, hi = i0 - 512, i0 + bm - 1 + 512
    assert mid["kv0_end"] == 8 and mid["nm0_end"] == 8
    assert mid["kv1_begin"] == lo // bn and mid["kv1_end"] == hi // bn + 1
    # the paper's "single masking operation": only the tiles the two band edges cross are masked
    masked = mid["n_tiles"] - 8 - (mid["nm1_end"] - mid["nm1_begin"])
    assert 0 < masked <= 2 * (bm // bn + 1)


def test_invalid_plans_are_rejected():
    for hp, win in (([4], [0]), ([ARROW], [-1]), ([3], [-1]), ([-1], [0])):
        st, _, _ = B.difa_worklist_build(1, 1, hp, win, 4, 4, 8, 4)
        assert st == B.DIFA_ERR_INVALID_ARG
    st, _, _ = B.difa_worklist_build(1, 1, [ARROW], None, 4, 4, 8, 4)
    assert st == B.DIFA_ERR_INVALID_ARG
    st, _, _ = B.difa_worklist_build(1, 1, [FULL], [0], 0, 0, 8, 4)
    assert st == B.DIFA_ERR_INVALID_ARG


def test_residual_sharing_heads_get_the_records_of_arrow_heads_with_the_flag():
    args = (2, 3, 37, 300, 256, 64)
    st, plain, _ = B.difa_worklist_build(args[0], args[1], [FULL, ARROW, ARROW], [0, 17, 90], *args[2:])
    st2, res, _ = B.difa_worklist_build(args[0], args[1], [FULL, B.DIFA_HEAD_ARROW_RESIDUAL, ARROW], [0, 17, 90], *args[2:])
    assert st == B.DIFA_OK and st2 == B.DIFA_OK and len(plain) == len(res)
    names = [n for n in plain.dtype.names if n != "flags"]
    for a, b in zip(plain, res):
        assert all(a[n] == b[n] for n in names)
        assert a["flags"] == 0
        assert b["flags"] == (B.DIFA_ITEM_ADD_RESIDUAL if b["bh"] % 3 == 1 else 0)


# ----------------------------------------------------------------------------- the schedule
def _schedule(wl_args, n_wg, n_xcd):
    batch, H, hp, win, n_text, n_img, bm, bn = wl_args
    st, items, _ = B.difa_worklist_build(batch, H, hp, win, n_text, n_img, bm, bn, 1)
    assert st == B.DIFA_OK
    st, segs, wg_begin, merges, n_slots = B.difa_schedule_build(items, n_wg, n_xcd)
    assert st == B.DIFA_OK
    return items, segs, wg_begin, merges, n_slots


def _check_schedule(items, segs, wg_begin, merges, n_slots, n_wg, n_xcd):
    # the per-workgroup lists partition the segment array
    assert wg_begin[0] == 0 and wg_begin[n_wg] == len(segs)
    assert all(wg_begin[w] <= wg_begin[w + 1] for w in range(n_wg))
    # every (record, position) is covered exactly once, and a segment repeats its record's fields
    by_key = {(int(r["bh"]), int(r["q_tile"])): r for r in items}
    cover = {k: np.zeros(int(r["n_tiles"]), dtype=np.int32) for k, r in by_key.items()}
    pieces = {}
    for s in segs:
        k = (int(s["bh"]), int(s["q_tile"]))
        r = by_key[k]
        for f in ("kv0_end", "nm0_end", "kv1_begin", "kv1_end", "nm1_begin", "nm1_end", "window"):
            assert s[f] == r[f]
        assert 0 <= s["pos_begin"] < s["pos_end"] <= r["n_tiles"]
        cover[k][s["pos_begin"]:s["pos_end"]] += 1
        whole = s["pos_begin"] == 0 and s["pos_end"] == r["n_tiles"]
        assert (s["part_slot"] < 0) == whole
        if not whole:
            pieces.setdefault(k, []).append(int(s["part_slot"]))
    for k, c in cover.items():
        assert (c == 1).all(), f"record {k} is not covered exactly once"
    # the merge list names exactly the cut records and their slots; slots are used once
    assert len(merges) == len(pieces)
    used = []
    for m in merges:
        k = (int(m["bh"]), int(m["q_tile"]))
        slots = sorted(pieces[k])
        assert m["n_parts"] == len(slots) >= 2
        assert slots == list(range(int(m["first_slot"]), int(m["first_slot"]) + len(slots)))
        used += slots
    assert sorted(used) == list(range(n_slots)) and n_slots <= 2 * n_wg
    # heads are kept together: a head lies on the dies its share of the work spans, plus one for the cuts
    die_of = {}
    for w in range(n_wg):
        for s in segs[wg_begin[w]:wg_begin[w + 1]]:
            die_of.setdefault(int(s["bh"]), set()).add(w % n_xcd)
    total = float(items["n_tiles"].sum())
    for bh, dies in die_of.items():
        share = float(items["n_tiles"][items["bh"] == bh].sum()) / total * n_xcd
        assert len(dies) <= int(np.ceil(share * 1.5)) + 1, (bh, dies, share)


@pytest.mark.parametrize("n_wg,n_xcd", [(8, 1), (16, 8), (256, 8), (6, 3)])
@pytest.mark.parametrize("n_text,n_img,heads", [
    (512, 4096, [(FULL, 0)] * 3 + [(ARROW, 128), (ARROW, 1024), (CACHE, 0)]),
    (333, 1000, [(ARROW, 7), (FULL, 0), (ARROW, 500)]),
    (0, 64, [(ARROW, 3)]),
    (16, 64, [(FULL, 0), (ARROW, 8), (ARROW, 16), (CACHE, 0)]),
])
def test_schedule_covers_every_position_once(n_wg, n_xcd, n_text, n_img, heads):
    hp, win = [m for m, _ in heads], [w for _, w in heads]
    args = (2, len(heads), hp, win, n_text, n_img, 256, 64)
    items, segs, wg_begin, merges, n_slots = _schedule(args, n_wg, n_xcd)
    _check_schedule(items, segs, wg_begin, merges, n_slots, n_wg, n_xcd)


def test_schedule_of_the_2k_layers_is_balanced():
    from paper_2503_22796_amd import workloads as W
    for wl, bound in ((W.flux_2k_full(), 1.04), (W.flux_2k_mixed(), 1.12)):
        args = (wl.B, wl.H, wl.head_plan, wl.window, wl.n_text, wl.n_img, 256, 64)
        items, segs, wg_begin, merges, n_slots = _schedule(args, 256, 8)
        _check_schedule(items, segs, wg_begin, merges, n_slots, 256, 8)
        load = np.array([(segs["pos_end"][wg_begin[w]:wg_begin[w + 1]] -
                          segs["pos_begin"][wg_begin[w]:wg_begin[w + 1]]).sum() for w in range(256)])
        ideal = items["n_tiles"].sum() / 256
        assert load.max() <= bound * ideal, (wl.name, load.max(), ideal)
        assert len(merges) > 0           # the tail records are cut


def _predicted_loads(items, segs, wg_begin, n_wg):
    """Per-workgroup load under the measured cost model, written out again here (eighths of a plain key-tile
    iteration: 8 per tile, 7 more on a tile that needs the element mask, 36 to start and finish a whole record,
    72 for a piece of a cut record plus 40 per other piece for the one that folds, shared evenly)."""
    by_key = {(int(r["bh"]), int(r["q_tile"])): r for r in items}
    load = np.zeros(n_wg)
    for w in range(n_wg):
        for sg in segs[wg_begin[w]:wg_begin[w + 1]]:
            r = by_key[(int(sg["bh"]), int(sg["q_tile"]))]
            masked = 0
            for p in range(int(sg["pos_begin"]), int(sg["pos_end"])):
                if p < r["kv0_end"]:
                    masked += p >= min(r["nm0_end"], r["kv0_end"])
                else:
                    t = r["kv1_begin"] + (p - r["kv0_end"])
                    masked += not (r["nm1_begin"] <= t < r["nm1_end"])
            n = int(sg["pos_end"] - sg["pos_begin"])
            parts = int(sg["n_parts"])
            load[w] += 8 * n + 7 * masked + (36 if sg["part_slot"] < 0 else 72 + 40 * (parts - 1) / parts)
    return load


def test_schedule_quality_on_the_named_layers():
    """Every compute unit finishes together, as far as the cost model can tell, and a cut record has few pieces
    (the workgroup that folds them reads every other piece's partial result at the very end of its work)."""
    from paper_2503_22796_amd import workloads as W
    for wl, bound in ((W.flux_2k_full(), 1.02), (W.flux_2k_mixed(), 1.04), (W.sd3_2k(), 1.05),
                      (W.video_like(), 1.04)):
        bm = 256
        args = (wl.B, wl.H, wl.head_plan, wl.window, wl.n_text, wl.n_img, bm, 64)
        items, segs, wg_begin, merges, n_slots = _schedule(args, 256, 8)
        load = _predicted_loads(items, segs, wg_begin, 256)
        assert load.max() <= bound * load.mean(), (wl.name, load.max() / load.mean())
        assert max((int(m["n_parts"]) for m in merges), default=1) <= 3, wl.name


def test_schedule_of_short_layers_does_not_cut_records_it_cannot_afford():
    # a 1K layer has one or two records per compute unit, and a cut costs a sixth of such a record: few cuts
    from paper_2503_22796_amd import workloads as W
    wl = W.flux_1k()
    args = (wl.B, wl.H, wl.head_plan, wl.window, wl.n_text, wl.n_img, 256, 64)
    items, segs, wg_begin, merges, n_slots = _schedule(args, 256, 8)
    _check_schedule(items, segs, wg_begin, merges, n_slots, 256, 8)
    assert len(merges) <= len(items) // 8


def test_schedule_rejects_bad_arguments():
    st, items, _ = B.difa_worklist_build(1, 1, [FULL], [0], 4, 60, 256, 64, 1)
    assert B.difa_schedule_build(items, 12, 8)[0] == B.DIFA_ERR_INVALID_ARG      # n_wg not a multiple of n_xcd
    assert B.difa_schedule_build(items, 0, 1)[0] == B.DIFA_ERR_INVALID_ARG
    st, segs, wg_begin, merges, n_slots = B.difa_schedule_build(items[:0], 8, 8)
    assert st == B.DIFA_OK and len(segs) == 0 and n_slots == 0 and (wg_begin == 0).all()


# ----------------------------------------------------------------------------- block-granular band
@pytest.mark.parametrize("n_text,n_img,bm,bn,heads", CASES)
def test_block_band_records_visit_the_same_tiles_and_mask_only_the_tail(n_text, n_img, bm, bn, heads):
    N = n_text + n_img
    hp, win = [m for m, _ in heads], [w for _, w in heads]
    H = len(heads)
    st, exact, _ = B.difa_worklist_build(1, H, hp, win, n_text, n_img, bm, bn, 1)
    st2, block, _ = B.difa_worklist_build(1, H, hp, win, n_text, n_img, bm, bn, 1, flags=B.DIFA_FLAG_BLOCK_BAND)
    assert st == B.DIFA_OK and st2 == B.DIFA_OK and len(exact) == len(block)
    ex = {(int(r["bh"]), int(r["q_tile"])): r for r in exact}
    n_kv = (N + bn - 1) // bn
    for r in block:
        e = ex[(int(r["bh"]), int(r["q_tile"]))]
        for f in ("kv0_end", "kv1_begin", "kv1_end", "n_tiles"):
            assert r[f] == e[f]                      # a block is visited iff it holds a kept pair: unchanged
        assert r["window"] == -1                     # no band edge is masked inside a tile
        visited = set(range(0, r["kv0_end"])) | set(range(r["kv1_begin"], r["kv1_end"]))
        mask_free = set(range(0, min(r["nm0_end"], r["kv0_end"]))) | \
            set(range(max(r["nm1_begin"], r["kv1_begin"]), min(r["nm1_end"], r["kv1_end"])))
        ragged_tail = {n_kv - 1} if N % bn else set()
        assert mask_free == visited - ragged_tail
    assert B.difa_worklist_build(1, H, hp, win, n_text, n_img, bm, bn, 1, flags=12)[0] == B.DIFA_ERR_INVALID_ARG


# --------------------------------------------------------------------------- image tokens first
def allowed_image_first(mode, w, n_text, n_img, i, j):
    if mode == FULL:
        return True
    return i >= n_img or j >= n_img or abs(i - j) <= w


IMAGE_FIRST_CASES = CASES + [
    (8, 32, 8, 4, [(ARROW, 2), (FULL, 0), (ARROW, 40)]),      # image length a multiple of the key tile
    (6, 30, 8, 4, [(ARROW, 0), (ARROW, 5)]),                  # a key tile that holds image and text keys
    (20, 3, 8, 4, [(ARROW, 1)]),                              # fewer image tokens than one key tile
    (5, 64, 16, 16, [(ARROW, 3), (ARROW, 17), (CACHE, 0)]),
]


@pytest.mark.parametrize("n_text,n_img,bm,bn,heads", IMAGE_FIRST_CASES)
@pytest.mark.parametrize("n_xcd", [1, 8])
def test_image_first_records_match_brute_force(n_text, n_img, bm, bn, heads, n_xcd):
    N = n_text + n_img
    hp = [m for m, _ in heads]
    win = [w for _, w in heads]
    H = len(heads)
    st, laid, _ = B.difa_worklist_build(1, H, hp, win, n_text, n_img, bm, bn, n_xcd, flags=B.DIFA_FLAG_IMAGE_FIRST)
    assert st == B.DIFA_OK
    items = laid[laid["q_tile"] >= 0]
    T = (N + bn - 1) // bn
    rot = n_img // bn if (n_text > 0 and n_img > 0) else 0     # position u is tile (u + rot) % T
    n_q = (N + bm - 1) // bm
    assert len(items) == sum(1 for m in hp if m != CACHE) * n_q
    for r in items:
        h = int(r["bh"])
        i0, i1 = int(r["q_tile"]) * bm, min(N, (int(r["q_tile"]) + 1) * bm)
        mode, w = hp[h], win[h]
        some, every = set(), set()
        for t in range(T):
            flags = [(j < N) and allowed_image_first(mode, w, n_text, n_img, i, j)
                     for i in range(i0, i1) for j in range(t * bn, (t + 1) * bn)]
            if any(flags):
                some.add(t)
            if all(flags):
                every.add(t)
        assert 0 <= r["kv0_end"] <= r["kv1_begin"] <= r["kv1_end"] <= T
        positions = list(range(0, r["kv0_end"])) + list(range(r["kv1_begin"], r["kv1_end"]))
        visited = {(u + rot) % T for u in positions}
        assert len(visited) == len(positions) == r["n_tiles"]
        assert visited == some, "visited tiles must be exactly the tiles that hold an allowed pair"
        free_pos = list(range(0, min(r["nm0_end"], r["kv0_end"]))) + \
            list(range(max(r["nm1_begin"], r["kv1_begin"]), min(r["nm1_end"], r["kv1_end"])))
        mask_free = {(u + rot) % T for u in free_pos}
        assert mask_free <= every, "a tile flagged mask-free holds a masked pair"
        # the first range knows only a mask-free prefix: when the first text tile also holds image keys
        # outside the band, the text tiles behind it are (safely) treated as masked
        mixed = n_img // bn if (n_img % bn and n_text > 0) else None       # the tile holding image and text keys
        if mixed is None or mixed in every:
            assert mask_free == (every & visited), "every mask-free tile should be recognised as such"


def test_image_first_flux_2k_shape_tile_counts():
    bm, bn = B.difa_tile_shape(128)
    st, items, _ = B.difa_worklist_build(1, 2, [ARROW, FULL], [512, 0], 512, 16384, bm, bn, 8,
                                         flags=B.DIFA_FLAG_IMAGE_FIRST)
    assert st == B.DIFA_OK
    items = items[items["q_tile"] >= 0]
    T = 16896 // bn
    full = items[items["window"] == -1]
    assert (full["n_tiles"] == T).all()
    arrow = items[items["window"] == 512]
    mid = arrow[arrow["q_tile"] == 30][0]
    i0 = 30 * bm
    lo, hi = i0 - 512, i0 + bm - 1 + 512
    assert mid["kv0_end"] == 8 and mid["nm0_end"] == 8                      # the 8 text tiles, none masked
    assert mid["kv1_begin"] == 8 + lo // bn and mid["kv1_end"] == 8 + hi // bn + 1
    assert mid["n_tiles"] == 8 + (hi // bn - lo // bn + 1)
    # same cost as with the text in front
    st, tf, _ = B.difa_worklist_build(1, 2, [ARROW, FULL], [512, 0], 512, 16384, bm, bn, 8)
    tf = tf[tf["q_tile"] >= 0]
    assert int(tf["n_tiles"].sum()) == int(items["n_tiles"].sum())
