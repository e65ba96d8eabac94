"""CPU: the host-side tiling of the prefill path (tide_prefill_plan).  Which kernels a call launches,
with which tile height, over which part of the checkpoint-major tile list, is plain arithmetic on
(dtype, C, T, d, b, compute units, form); it needs no GPU, and a slip in it would silently skip or
double-count rows on shapes the GPU parity tests do not happen to visit.  The property that matters:
every row of every checkpoint belongs to exactly one tile of exactly one launch."""
import numpy as np
import pytest

from paper_2603_21365_amd import tide_route as tr

SPLITK, WIDE, WIDE_F32, TILE, STREAM128, STREAM64, RING, BAND, SPLITK_FUSED, SQUARE = 1, 2, 3, 4, 5, 6, 7, 8, 9, 10
ELEM = {tr.F32: 4, tr.F16: 2, tr.BF16: 2}


def covered_rows(plan, C, T):
    """Row ranges [(checkpoint, first, last+1)] of every tile of every launch."""
    out = []
    for L in plan:
        R, tpc = L["rows_per_tile"], L["tiles_per_ckpt"]
        assert tpc == -(-T // R), "tiles per checkpoint = ceil(T / rows per tile)"
        assert 0 <= L["tile_begin"] < L["total_tiles"] <= C * tpc
        for t in range(L["tile_begin"], L["total_tiles"]):
            c, j = divmod(t, tpc)
            out.append((c, j * R, min((j + 1) * R, T)))
    return out


def check_plan(dtype, C, T, d, b, cus, form):
    plan = tr.prefill_plan(dtype, C, T, d, b, cus=cus, form=form)
    what = f"dtype={dtype} C={C} T={T} d={d} b={b} cus={cus} form={form}: {plan}"
    assert 1 <= len(plan) <= 2, what
    # ---- every row exactly once
    seen = np.zeros((C, T), np.uint8)
    for c, lo, hi in covered_rows(plan, C, T):
        assert lo < hi, what                      # no tile made of padding only
        seen[c, lo:hi] += 1
    assert seen.min() == 1 and seen.max() == 1, what
    assert plan[-1]["total_tiles"] == C * plan[-1]["tiles_per_ckpt"], what   # the last launch runs to the end of the list
    halves = (b + 127) // 128
    ntile = d * ELEM[dtype] // 256
    for i, L in enumerate(plan):
        k, R, wg = L["kernel"], L["rows_per_tile"], L["workgroups"]
        assert wg >= 1, what
        if k == SPLITK_FUSED:
            assert R == 32 and halves == 1 and L["total_tiles"] <= 64 and (form & 0xff) in (0, 8) and ((form & 0xff) == 8 or T <= 16), what
        if k in (SPLITK, SPLITK_FUSED):
            assert len(plan) == 1 and d % 128 == 0, what
            assert R in (32, 64, 128) and (form >> 8 or R == 32 or T > R // 2), what   # its own choice: never a tile that is mostly padding
            assert L["k_slices"] in (2, 4, 8, ntile) and 2 <= L["k_slices"] <= min(8, ntile), what
            assert wg == L["total_tiles"] * halves * L["k_slices"], what
        else:
            assert L["k_slices"] == 1, what
        if k in (WIDE, WIDE_F32):
            assert i == 0 and L["tile_begin"] == 0 and d % 128 == 0, what
            assert R == (128 if halves == 2 else 256), what
            assert wg % 8 == 0 and wg <= cus, what                                   # one slice of the list per XCD
            assert wg == (cus if L["total_tiles"] >= cus else 8 * -(-L["total_tiles"] // 8)), what   # rounds of one tile per CU; the last may be partly filled
            assert (dtype == tr.F32) == (k == WIDE_F32), what
            assert not (k == WIDE_F32 and halves == 2), what
        if k == SQUARE:
            assert i == 0 and R == 256 and halves == 2 and dtype != tr.F32 and d % 128 == 0 and d >= 192, what
            assert L["tile_begin"] == 0 and wg == 8 * -(-L["total_tiles"] // 8), what
            assert (form & 0xff) in (0, 9), what
            all_tiles = C * L["tiles_per_ckpt"]
            if len(plan) == 2:  # whole rounds here, the rest on 128-row tiles behind it: at most half a round
                assert form == 0 and L["total_tiles"] % cus == 0 and 0 < all_tiles - L["total_tiles"] < cus, what
                assert 2 * (all_tiles - L["total_tiles"]) <= cus and plan[1]["kernel"] == TILE, what
            else:
                assert L["total_tiles"] == all_tiles, what
                if form == 0:   # its own choice: more than half the CUs get a tile, and a last round more than half full
                    rem = all_tiles % cus
                    assert 2 * all_tiles > cus and (all_tiles <= cus or rem == 0 or 2 * rem > cus), what
        if k == TILE:
            assert R == 128 and dtype != tr.F32 and d % 128 == 0, what
            assert wg == 8 * -(-(L["total_tiles"] - L["tile_begin"]) // 8), what
        if k in (STREAM128, STREAM64):
            assert R == (128 if k == STREAM128 else 64) and d % 128 == 0, what
            assert wg % 8 == 0 and wg <= cus * (1 if (R == 128 or halves == 2) else 2), what
            assert halves == 1 or k == STREAM64, what
        if k == RING:
            assert R == 64 and halves == 1, what
        if k == BAND:
            assert len(plan) == 1 and R == 32 and dtype != tr.F32 and halves == 1 and d % 128 == 0 and wg == cus, what
        if d % 128 != 0:
            assert k == RING and len(plan) == 1, what
    if len(plan) == 2:
        assert plan[0]["kernel"] in (WIDE, WIDE_F32, SQUARE) and plan[1]["kernel"] not in (WIDE, WIDE_F32, SPLITK, SQUARE), what
    return plan


SHAPES = [(8, 4096, 4096), (9, 16384, 4096), (10, 16384, 768), (10, 16384, 8192), (1, 1, 4096), (8, 8, 4096), (1, 64, 256),
          (8, 33, 2048), (3, 1000, 1024), (5, 8155, 256), (12, 16384 + 77, 128), (1, 300000, 128), (32, 513, 512),
          (7, 2049, 3072), (2, 12345, 5120), (8, 2048, 4096), (8, 3072, 4096), (8, 1536, 4096), (1, 16384, 4096)]


@pytest.mark.parametrize("form", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9])
@pytest.mark.parametrize("dtype", [tr.BF16, tr.F16, tr.F32])
def test_every_row_is_in_exactly_one_tile(dtype, form):
    for C, T, d in SHAPES:
        for b in (64, 128, 256):
            for cus in (256, 304, 64, 8):
                check_plan(dtype, C, T, d, b, cus, form)


def test_every_row_is_in_exactly_one_tile_on_random_shapes():
    rng = np.random.default_rng(0x71DE)
    for _ in range(3000):
        dtype = int(rng.choice([tr.BF16, tr.F16, tr.F32]))
        C = int(rng.integers(1, 33))
        T = int(rng.choice([rng.integers(1, 70), rng.integers(1, 3000), rng.integers(1, 40000)]))
        if C * T > 600000:
            T = 600000 // C
        d = int(rng.choice([128, 256, 384, 768, 1024, 2048, 2560, 4096, 5120, 8192, 16384]))
        b = int(rng.choice([64, 128, 256]))
        cus = int(rng.choice([8, 64, 128, 256, 304]))
        form = int(rng.integers(0, 10))
        check_plan(dtype, C, T, d, b, cus, form)


def check_schedule(L, b, k_tiles):
    """Every tile of a streaming-kernel launch is processed exactly once, whole or as pieces that add up."""
    R, grid, lo, hi = L["rows_per_tile"], L["workgroups"], L["tile_begin"], L["total_tiles"]
    rows = np.zeros((hi - lo, R), np.uint8)
    busy = 0
    for block in range(grid):
        items = tr.stream_schedule(R, b, k_tiles, grid, block, lo, hi)
        busy += bool(items)
        for n, (tile, row_off, nrows) in enumerate(items):
            assert lo <= tile < hi and nrows in (32, 64, 128) and nrows <= R and row_off % nrows == 0 and row_off + nrows <= R
            assert nrows == R or (n == len(items) - 1 and b <= 128 and k_tiles % (R // nrows) == 0)   # a piece is a workgroup's last item
            rows[tile - lo, row_off:row_off + nrows] += 1
    assert rows.min() == 1 and rows.max() == 1, (L, b, k_tiles)
    return busy


def test_the_persistent_schedule_covers_every_tile_once():
    """The streaming kernels' own schedule (the code they run, executed on the host), on the launches the
    plan produces: whole tiles round-robin within an XCD's slice, then the tiles of the last round cut into pieces."""
    rng = np.random.default_rng(7)
    cases = [(tr.BF16, 5, 8155, 256, 128, 256, 2), (tr.F16, 3, 16384, 512, 128, 256, 2), (tr.BF16, 7, 8192, 128, 128, 256, 2),
             (tr.BF16, 3, 16384, 256, 128, 256, 1), (tr.BF16, 1, 4096, 4096, 128, 256, 2), (tr.BF16, 8, 2048, 4096, 128, 256, 0),
             (tr.BF16, 8, 4096, 4096, 256, 256, 1), (tr.BF16, 9, 16384, 4096, 128, 256, 0), (tr.F32, 3, 16384 - 70, 256, 128, 256, 2)]
    for _ in range(150):
        cases.append((int(rng.choice([tr.BF16, tr.F16, tr.F32])), int(rng.integers(1, 13)), int(rng.integers(33, 20000)),
                      int(rng.choice([128, 256, 384, 1024, 4096])), int(rng.choice([64, 128, 256])), int(rng.choice([8, 64, 256, 304])),
                      int(rng.choice([0, 1, 2, 4]))))
    checked = 0
    for dtype, C, T, d, b, cus, form in cases:
        for L in tr.prefill_plan(dtype, C, T, d, b, cus=cus, form=form):
            if L["kernel"] in (STREAM128, STREAM64):
                busy = check_schedule(L, b, d * ELEM[dtype] // 256)
                # no workgroup idles while tiles wait (the last XCD's slice of the list may be up to 7 tiles short)
                assert busy >= min(L["workgroups"], L["total_tiles"] - L["tile_begin"]) - 7
                checked += 1
    assert checked > 60


def check_band_schedule(C, U, grid):
    """Every 32-row block of every checkpoint lies in exactly one tile of exactly one workgroup; a tile has 1 to 9
    blocks of one checkpoint; the workgroups' shares differ by at most one block; XCD x (workgroup id mod 8) owns
    a contiguous eighth of the list."""
    seen = np.zeros((C, U), np.uint8)
    share = []
    first = {}
    for block in range(grid):
        tiles = tr.band_schedule(C, U, grid, block)
        n = 0
        pos = None
        for c, b0, nb in tiles:
            assert 0 <= c < C and 1 <= nb <= 9 and 0 <= b0 and b0 + nb <= U, (C, U, grid, block, tiles)
            assert pos is None or pos == c * U + b0, "a workgroup's tiles are contiguous in the checkpoint-major list"
            pos = c * U + b0 + nb
            seen[c, b0:b0 + nb] += 1
            n += nb
        # as few tiles as cover each piece of the band: a piece of L blocks within one checkpoint takes ceil(L / 9)
        pieces = {}
        for c, b0, nb in tiles:
            pieces.setdefault(c, []).append(nb)
        for c, sizes in pieces.items():
            assert len(sizes) == -(-sum(sizes) // 9) and max(sizes) - min(sizes) <= 1, (C, U, grid, block, tiles)
        share.append(n)
        if tiles:
            first[block] = tiles[0][0] * U + tiles[0][1]
    assert seen.min() == 1 and seen.max() == 1, (C, U, grid)
    assert max(share) - min(share) <= 1, (C, U, grid, share)
    for x in range(8):                      # XCD x: workgroups x, x + 8, ... take ascending, adjacent bands
        starts = [first[b] for b in range(x, grid, 8) if b in first]
        assert starts == sorted(starts)
        if x and starts:
            prev = [first[b] for b in range(x - 1, grid, 8) if b in first]
            assert not prev or max(prev) < min(starts)


def test_the_band_schedule_covers_every_block_once():
    rng = np.random.default_rng(11)
    cases = [(9, 512, 256), (10, 512, 256), (8, 128, 256), (1, 1, 8), (1, 7, 256), (3, 1000, 304), (32, 17, 64), (2, 5000, 8)]
    for _ in range(200):
        cases.append((int(rng.integers(1, 33)), int(rng.choice([rng.integers(1, 40), rng.integers(1, 2000)])), int(rng.choice([8, 64, 256, 304]))))
    for C, U, grid in cases:
        check_band_schedule(C, U, grid)
    # the 36-layer batched prefill on 256 CUs: 18 blocks per workgroup, two tiles of 9 unless a checkpoint ends inside the band
    counts = [len(tr.band_schedule(9, 512, 256, block)) for block in range(256)]
    assert sorted(set(counts)) == [2, 3] and counts.count(3) == 8


def test_generic_hidden_sizes_take_the_register_ring_kernel():
    for dtype, d in ((tr.BF16, 200), (tr.F16, 72), (tr.F32, 100), (tr.BF16, 4104), (tr.F32, 708)):
        for form in range(10):
            for C, T in ((1, 1), (4, 300), (10, 16384)):
                plan = check_plan(dtype, C, T, d, 128, 256, form)
                assert [L["kernel"] for L in plan] == [RING]


def test_the_choices_on_the_named_workloads():
    """What the automatic choice is on a 256-CU device for the workloads the measurements quote."""
    kinds = lambda plan: [(L["kernel"], L["rows_per_tile"]) for L in plan]
    assert kinds(tr.prefill_plan(tr.BF16, 8, 4096, 4096)) == [(TILE, 128)]                       # one tile per CU
    assert kinds(tr.prefill_plan(tr.BF16, 9, 16384, 4096)) == [(BAND, 32)]                        # 18 blocks of 32 rows per CU: the band form
    assert kinds(tr.prefill_plan(tr.BF16, 10, 16384, 4096)) == [(BAND, 32)]                       # 20 per CU
    assert kinds(tr.prefill_plan(tr.BF16, 10, 16384, 4096, 256)) == [(SQUARE, 256), (TILE, 128)]  # width 256: two rounds of 256-row tiles, the other half round as 128-row tiles
    assert [L["workgroups"] for L in tr.prefill_plan(tr.BF16, 10, 16384, 4096, 256)] == [512, 256]
    assert kinds(tr.prefill_plan(tr.BF16, 10, 16384, 4096, 256, form=6)) == [(TILE, 128)]         # ... the one-tile kernel when forced: five rounds of 128-row tiles
    assert tr.prefill_plan(tr.BF16, 10, 16384, 4096, 256, form=6)[0]["workgroups"] == 1280
    assert kinds(tr.prefill_plan(tr.BF16, 10, 16384, 4096, 256, form=4)) == [(WIDE, 128)]         # ... or the wide-tile kernel
    assert kinds(tr.prefill_plan(tr.BF16, 8, 8192, 4096)) == [(BAND, 32)]                         # 8 per CU (= one round of 256-row tiles)
    assert kinds(tr.prefill_plan(tr.BF16, 8, 5120, 4096)) == [(BAND, 32)]                         # 5 per CU
    assert kinds(tr.prefill_plan(tr.BF16, 8, 5120, 4096, form=4)) == [(WIDE, 256)]                # ... forced: 160 wide tiles on 160 CUs
    assert kinds(tr.prefill_plan(tr.F32, 10, 16384, 4096)) == [(WIDE_F32, 256), (RING, 64)]
    assert kinds(tr.prefill_plan(tr.F16, 8, 8, 4096)) == [(SPLITK_FUSED, 32)]                     # a decode step on packed weights: split-k in one launch
    assert tr.prefill_plan(tr.F16, 8, 8, 4096)[0]["k_slices"] == 8
    assert kinds(tr.prefill_plan(tr.F16, 8, 16, 4096)) == [(SPLITK_FUSED, 32)]
    assert kinds(tr.prefill_plan(tr.F16, 8, 17, 4096)) == [(SPLITK, 32)]                          # more rows in use: the pair
    assert kinds(tr.prefill_plan(tr.F16, 8, 8, 4096, 256)) == [(SPLITK, 32)]                      # width 256: the pair
    assert kinds(tr.prefill_plan(tr.F16, 8, 8, 4096, form=5)) == [(SPLITK, 32)]                   # the pair when forced
    assert kinds(tr.prefill_plan(tr.BF16, 1, 1024, 4096, form=8)) == [(SPLITK_FUSED, 32)]         # one launch when forced: 32 tiles
    assert kinds(tr.prefill_plan(tr.BF16, 1, 4096, 4096, form=8)) == [(SPLITK, 32)]               # ... 128 tiles: more than there are counters
    assert kinds(tr.prefill_plan(tr.BF16, 1, 1024, 4096)) == [(SPLITK, 32)]                       # one checkpoint's call: 32 tiles x 8 slices
    assert tr.prefill_plan(tr.BF16, 1, 1024, 4096)[0]["workgroups"] == 256
    p4096 = tr.prefill_plan(tr.BF16, 1, 4096, 4096)[0]                                            # 64 tiles x 4 slices: still one workgroup per CU
    assert (p4096["kernel"], p4096["rows_per_tile"], p4096["k_slices"], p4096["workgroups"]) == (SPLITK, 64, 4, 256)
    assert kinds(tr.prefill_plan(tr.BF16, 1, 8192, 4096)) == [(STREAM128, 128)]                   # 64 tiles: pieces of the persistent kernel
    assert kinds(tr.prefill_plan(tr.BF16, 1, 1024, 1024)) == [(STREAM128, 128)]                   # short rows: the chain is short already
    assert kinds(tr.prefill_plan(tr.BF16, 8, 4096, 4096, 256)) == [(TILE, 128)]                   # width 256: one 128-row tile per CU, eight consumer waves
    assert kinds(tr.prefill_plan(tr.BF16, 8, 2048, 4096, 256)) == [(STREAM64, 64)]                # ... 128 tiles: a 64-row workgroup per CU
    assert kinds(tr.prefill_plan(tr.BF16, 8, 2048, 4096)) == [(STREAM64, 64)]                     # 128 tiles of 128 rows: a 64-row workgroup per CU
    assert kinds(tr.prefill_plan(tr.BF16, 8, 2080, 4096)) == [(TILE, 128)]                        # 136 tiles: the 64-row kernel would need two per CU
    assert kinds(tr.prefill_plan(tr.BF16, 8, 6144, 4096)) == [(BAND, 32)]                         # 6 blocks per CU
    assert kinds(tr.prefill_plan(tr.BF16, 8, 6144, 4096, form=4)) == [(WIDE, 256)]                # 192 wide tiles: three quarters of a round
    assert tr.prefill_plan(tr.BF16, 8, 6144, 4096, form=4)[0]["workgroups"] == 192
    assert kinds(tr.prefill_plan(tr.BF16, 8, 4608, 4096)) == [(BAND, 32)]                         # 4.5 blocks per CU
    assert kinds(tr.prefill_plan(tr.BF16, 8, 4608, 4096, form=4)) == [(WIDE, 256)]                # ... forced: 144 wide tiles
    assert kinds(tr.prefill_plan(tr.BF16, 8, 4096 + 128, 4096)) == [(BAND, 32)]                   # one block more than a 128-row tile per CU
    assert kinds(tr.prefill_plan(tr.BF16, 8, 4096, 4096)) == [(TILE, 128)]                        # exactly four blocks per CU: the one-tile kernel
    assert kinds(tr.prefill_plan(tr.BF16, 8, 3072, 4096, 256)) == [(TILE, 128)]                   # width 256: 192 tiles of 128 rows on 192 CUs
    assert kinds(tr.prefill_plan(tr.BF16, 8, 4352, 4096, 256)) == [(SQUARE, 256)]                 # ... 136 tiles of 256 rows: the square form from more than half the CUs on
    assert kinds(tr.prefill_plan(tr.BF16, 8, 7168, 4096, 256)) == [(SQUARE, 256)]                 # ... 224
    assert kinds(tr.prefill_plan(tr.BF16, 8, 8192, 4096, 256)) == [(SQUARE, 256)]                 # ... one round
    assert kinds(tr.prefill_plan(tr.BF16, 8, 8448, 4096, 256)) == [(TILE, 128)]                   # ... one round and 8 tiles: the small tiles take it all
    assert kinds(tr.prefill_plan(tr.BF16, 8, 12288, 4096, 256)) == [(SQUARE, 256), (TILE, 128)]   # ... a round and a half: one round, then 256 small tiles
    assert [L["tile_begin"] for L in tr.prefill_plan(tr.BF16, 8, 12288, 4096, 256)] == [0, 512]
    assert kinds(tr.prefill_plan(tr.BF16, 8, 13312, 4096, 256)) == [(SQUARE, 256)]                # ... 1.625 rounds: two rounds
    assert kinds(tr.prefill_plan(tr.BF16, 8, 15360, 4096, 256)) == [(SQUARE, 256)]                # ... 1.875
    assert kinds(tr.prefill_plan(tr.BF16, 8, 16384, 4096, 256)) == [(SQUARE, 256)]                # ... two rounds
    assert kinds(tr.prefill_plan(tr.F16, 9, 16384, 4096, 256)) == [(SQUARE, 256), (TILE, 128)]    # ... 2.25
    assert kinds(tr.prefill_plan(tr.F32, 8, 8192, 4096, 256)) != [(SQUARE, 256)]                  # (16-bit rows only)
    assert kinds(tr.prefill_plan(tr.BF16, 8, 8192, 128, 256)) != [(SQUARE, 256)]                  # (two 64-value stages: too short a row)
    assert kinds(tr.prefill_plan(tr.F32, 8, 7168, 4096)) == [(WIDE_F32, 256)]                     # fp32 rows: 224 wide tiles
    assert kinds(tr.prefill_plan(tr.F32, 1, 9216, 4096)) == [(RING, 64)]                          # fp32, 72 tiles: the split-k chain is too long
    assert kinds(tr.prefill_plan(tr.F32, 1, 8192, 4096)) == [(SPLITK, 64)]


def test_a_forced_split_k_shape_is_taken_as_given():
    for dtype, C, T, d, b in ((tr.BF16, 3, 333, 1408, 128), (tr.F16, 2, 200, 1024, 256), (tr.F32, 2, 150, 512, 128), (tr.BF16, 8, 1, 4096, 128)):
        for rows in (32, 64, 128):
            for slices in (2, 4, 8):
                plan = check_plan(dtype, C, T, d, b, 256, tr.splitk_form(rows, slices))
                assert [(L["kernel"], L["rows_per_tile"], L["k_slices"]) for L in plan] == [(SPLITK, rows, slices)]
    assert tr.prefill_plan(tr.BF16, 1, 100, 512, form=tr.splitk_form(64, 8))[0]["k_slices"] == 4     # 4 k-tiles: at most 4 slices
    for word in (2 | 64 << 8, 5 | 48 << 8, 5 | 3 << 16, 5 | 1 << 24, 0 | 8 << 16):
        with pytest.raises(tr.TideError):
            tr.prefill_plan(tr.BF16, 1, 100, 512, form=word)


def test_the_band_form_is_one_launch_over_all_blocks():
    for dtype in (tr.BF16, tr.F16):
        for C, T, d, b in ((9, 16384, 4096, 128), (10, 16384, 768, 64), (3, 1000, 1024, 128), (1, 1, 128, 128)):
            (L,) = tr.prefill_plan(dtype, C, T, d, b, form=7)
            assert (L["kernel"], L["rows_per_tile"], L["tiles_per_ckpt"], L["total_tiles"], L["tile_begin"], L["workgroups"]) == \
                   (BAND, 32, -(-T // 32), C * -(-T // 32), 0, 256)
    # fp32 rows, width 256 and other hidden sizes fall back to forms that apply
    assert BAND not in [L["kernel"] for L in tr.prefill_plan(tr.F32, 9, 16384, 4096, form=7)]
    assert BAND not in [L["kernel"] for L in tr.prefill_plan(tr.BF16, 9, 16384, 4096, 256, form=7)]
    assert [L["kernel"] for L in tr.prefill_plan(tr.BF16, 9, 16384, 200, form=7)] == [RING]


def test_plan_rejects_bad_arguments():
    bad = [dict(dtype=9), dict(C=0), dict(C=33), dict(T=0), dict(d=100000), dict(d=0), dict(b=96), dict(cus=100), dict(cus=0), dict(form=10)]
    # hidden sizes of the generic fallback that are copied into zero-padded rows first are planned at the padded size
    assert tr.prefill_plan(tr.BF16, 4, 1000, 130) == tr.prefill_plan(tr.BF16, 4, 1000, 131)[:] == tr.prefill_plan(tr.BF16, 4, 1000, 256)
    assert tr.prefill_plan(tr.BF16, 4, 1000, 200, 256) == tr.prefill_plan(tr.BF16, 4, 1000, 256, 256)
    for kw in bad:
        args = dict(dtype=tr.BF16, C=4, T=100, d=1024, b=128, cus=256, form=0)
        args.update(kw)
        with pytest.raises(tr.TideError):
            tr.prefill_plan(args["dtype"], args["C"], args["T"], args["d"], args["b"], cus=args["cus"], form=args["form"])
