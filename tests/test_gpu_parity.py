"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import oracle
from paper_1802_04924_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import torch
    from paper_1802_04924_amd import Context
    assert torch.cuda.is_available()
    c = Context(0)
    yield c
    c.close()


@pytest.fixture(params=[True, False], ids=["wave-per-tile", "tiled"])
def kernels(ctx, request):
    """Single node eliminations with little work: on the kernel they take by default, then on the tiled one."""
    ctx.set_small_product_kernel(request.param)
    yield request.param
    ctx.set_small_product_kernel(True)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def check_products(ctx, A, w, B, expect_keyed=None, expect_keyed_bounded=None):
    """A [batch][Ci][Cj] etc. as numpy; compares out and argmin of every product with the oracle, on both
    entry points: lwp_eliminate_node (ranges measured and variant picked on the device, per product)
    and lwp_eliminate_node_bounded (the caller promises ranges -- here the exact ones -- and the host
    picks the variant).  expect_keyed: whether packed keys (global or per row) must have been used
    by the tiled kernel.  A call below 3 * 2^25 cell updates (2^25 with promised ranges, unless it has at most four 64 x 64 tiles) is first checked on the kernel it takes by default, the wavefront-per-tile one
    (compare/select), then on the tiled kernel."""
    d_A, d_w, d_B = dev(A), dev(w), dev(B)
    batch = A.shape[0]
    ref = [oracle.minplus_argmin(A[b], w[b], B[b]) for b in range(batch)]
    bounds = (A.min(), A.max(), w.min(), w.max(), B.min(), B.max())
    updates = A.shape[0] * A.shape[1] * A.shape[2] * B.shape[2]
    if updates <= (3 << 25):
        ctx.profile_enable(True)
        tiles64 = batch * -(-A.shape[1] // 64) * -(-B.shape[2] // 64)
        for bnd in ((None, bounds) if updates <= (1 << 25) or tiles64 <= 4 else (None,)):
            ctx.profile_reset()
            out, arg = ctx.eliminate_node(d_A, d_w, d_B, bounds=bnd)
            ctx.synchronize()
            prof = ctx.profile_read()
            out, arg = out.cpu().numpy(), arg.cpu().numpy()
            for b in range(batch):
                assert np.array_equal(out[b], ref[b][0]), f"cost mismatch in product {b} (wavefront per tile, bounds {bnd})"
                assert np.array_equal(arg[b], ref[b][1]), f"argmin mismatch in product {b} (wavefront per tile, bounds {bnd})"
            assert prof["products_plain"] == batch and prof["products_keyed"] + prof["products_keyed_row"] + prof["products_value"] == 0
            assert prof["keyed_launches"] == 0
        ctx.profile_enable(False)
    ctx.set_small_product_kernel(False)
    try:
        return check_products_tiled(ctx, d_A, d_w, d_B, ref, bounds, expect_keyed, expect_keyed_bounded)
    finally:
        ctx.set_small_product_kernel(True)


def check_products_tiled(ctx, d_A, d_w, d_B, ref, bounds, expect_keyed, expect_keyed_bounded):
    batch = d_A.shape[0]
    ctx.profile_enable(True)
    ctx.profile_reset()
    out, arg = ctx.eliminate_node(d_A, d_w, d_B)
    ctx.synchronize()
    prof = ctx.profile_read()
    out, arg = out.cpu().numpy(), arg.cpu().numpy()
    for b in range(batch):
        assert np.array_equal(out[b], ref[b][0]), f"cost mismatch in product {b}"
        assert np.array_equal(arg[b], ref[b][1]), f"argmin mismatch in product {b}"
    keyed = prof["products_keyed"] + prof["products_keyed_row"]
    assert keyed + prof["products_plain"] == batch and prof["products_value"] == 0     # every product ran exactly once
    if expect_keyed is not None:
        assert keyed == (batch if expect_keyed else 0)
    ctx.profile_reset()
    out, arg = ctx.eliminate_node(d_A, d_w, d_B, bounds=bounds)
    ctx.synchronize()
    prof_b = ctx.profile_read()
    ctx.profile_enable(False)
    out, arg = out.cpu().numpy(), arg.cpu().numpy()
    for b in range(batch):
        assert np.array_equal(out[b], ref[b][0]), f"cost mismatch in product {b} (promised ranges)"
        assert np.array_equal(arg[b], ref[b][1]), f"argmin mismatch in product {b} (promised ranges)"
    if expect_keyed_bounded is None:
        expect_keyed_bounded = expect_keyed
    if expect_keyed_bounded is not None:
        assert (prof_b["keyed_launches"] == 1) == expect_keyed_bounded
    return prof


SHAPES = [(1, 1, 1, 1), (1, 3, 5, 4), (2, 17, 33, 9), (1, 128, 128, 128), (3, 130, 257, 140),
          (2, 256, 256, 256), (1, 64, 512, 192), (1, 129, 16, 260), (5, 40, 100, 24)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("hi", [1, 3, 1 << 20])
def test_eliminate_node_keyed_small_values(ctx, shape, hi):
    batch, Ci, Cj, Ck = shape
    rng = np.random.default_rng(hash((shape, hi)) % (1 << 32))
    A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    check_products(ctx, A, w, B, expect_keyed=True)


@pytest.mark.parametrize("shape", [(64, 128, 16, 128), (100, 70, 33, 90), (300, 40, 130, 56), (2100, 16, 5, 16), (1, 1, 1000, 1), (3, 2, 1024, 3), (1, 9, 1025, 9), (1, 3, 40000, 2), (7, 250, 40, 250), (4, 200, 60, 200),
                                   (3, 250, 201, 250), (1, 130, 1000, 140), (2, 33, 203, 500), (5, 250, 210, 250),
                                   (1, 64, 12000, 70)])
@pytest.mark.parametrize("hi", [2, 1 << 24])
def test_eliminate_node_many_small_products(ctx, shape, hi):
    # calls below 2^27 cell updates with enough output for a wavefront per 16 x 16 tile (at least 2048 of
    # them), ragged in every dimension, with ties (hi = 2) and without; then long rows, where four
    # wavefronts share an 8 x 8 tile, their shares of the candidates ragged; then two: between 4096 and
    # 8192 tiles of 8 x 8 (short chunks, a tile per wavefront) and between 1024 and 4096 (long chunks);
    # (the very last: two 64 x 64 tiles with rows of 12000, beyond 2^25 cell updates -- on the wavefront-per-tile
    # kernel also with promised ranges); the four before it: 64 to 1536 tiles of 16 x 16 with rows of at least 200 candidates, where four
    # wavefronts share a 16 x 16 tile (shares of 51, 51, 51, 48; of 250 each in chunks of 64; 51, 51, 51, 50)
    batch, Ci, Cj, Ck = shape
    rng = np.random.default_rng(abs(hash((shape, hi))) % (1 << 32))
    A = rng.integers(-hi, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(-hi, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    check_products(ctx, A, w, B)


def spread_case(shape, bits, seed):
    batch, Ci, Cj, Ck = shape
    hi = (1 << bits) - 1
    rng = np.random.default_rng(seed)
    A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    # force ties across chunk boundaries: duplicate some candidates exactly
    A[:, :, Cj // 2:] = A[:, :, :Cj - Cj // 2]
    w[:, Cj // 2:] = w[:, :Cj - Cj // 2]
    B[:, Cj // 2:, :] = B[:, :Cj - Cj // 2, :]
    return A, w, B


# The spread of A + w + B (3 * 2^bits here) decides the key width.  Launches with fewer than 2048
# tiles of 128 x 128 use 64 x 64 tiles, whose deeper stages leave one bit less for the cost; where
# the host picks the variant (promised ranges) a spread that needs that bit moves the launch to
# 128 x 128 tiles if those still fill the chip (>= 512 tiles).  Beyond that the plain variant runs
# (keys re-based per row are for launches of at least 2^28 cell updates, tested further down).
@pytest.mark.parametrize("bits,expect_keyed", [(22, True), (24, True), (25, False), (26, False), (29, False)])
@pytest.mark.parametrize("shape", [(2, 130, 257, 140), (1, 128, 512, 128), (1, 31, 1000, 17)])
def test_eliminate_node_key_widths_small_tiles(ctx, shape, bits, expect_keyed):
    A, w, B = spread_case(shape, bits, bits * 1000 + shape[2])
    check_products(ctx, A, w, B, expect_keyed=expect_keyed)


@pytest.mark.parametrize("bits,expect_keyed", [(20, True), (23, True), (24, True), (25, True), (26, False)])
@pytest.mark.parametrize("shape", [(512, 256, 80, 256), (130, 500, 33, 512), (40, 500, 600, 512)])
def test_eliminate_node_key_widths_large_tiles(ctx, shape, bits, expect_keyed):
    A, w, B = spread_case(shape, bits, bits * 77 + shape[2])
    # 40 products of 4 x 4 large tiles prefer 64 x 64 tiles; only the host's policy moves them to
    # 128 x 128 tiles for the extra key bit.  On the device their 25-bit case sits exactly at the limit
    # of keys re-based per row (it depends on whether the largest possible value was drawn): not asserted
    on_device = None if (bits == 25 and shape[0] == 40) else expect_keyed
    check_products(ctx, A, w, B, expect_keyed=on_device, expect_keyed_bounded=expect_keyed)


def test_eliminate_node_split_tiles_repeatedly(ctx):
    # few tiles: several workgroups share a tile and merge through global scratch; the per-tile
    # arrival counters must be left ready for the next launch, whatever its shape
    rng = np.random.default_rng(99)
    shapes = [(1, 64, 2048, 64), (3, 70, 700, 130), (1, 64, 64, 64), (2, 200, 4096, 100), (1, 512, 512, 512), (9, 33, 257, 65)]
    for rep in range(3):
        for batch, Ci, Cj, Ck in shapes:
            hi = [3, 1 << 20, (1 << 26) - 1][rep]          # heavy ties / keyed / plain variant
            A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
            w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
            B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
            check_products(ctx, A, w, B)


@pytest.mark.parametrize("shape", [(17, 512, 100, 512), (1, 2100, 300, 2100), (3, 1200, 2050, 1230), (65, 256, 512, 256)])
@pytest.mark.parametrize("hi", [3, 1 << 20, (1 << 28) - 1])
def test_eliminate_node_last_round_of_workgroups_shares_its_tiles(ctx, shape, hi):
    # launches of a few more tiles than a multiple of the 256 compute units: the tiles left over once
    # every unit has the same number of whole ones are shared by several workgroups each (one launch with
    # whole and shared tiles side by side); heavy ties / packed keys / compare-select, ragged edges, a
    # batch whose last product is cut in two
    batch, Ci, Cj, Ck = shape
    tiles = batch * (-(-Ci // 64)) * (-(-Ck // 64))
    assert tiles > 1024 and 0 < tiles % 256 <= 128
    rng = np.random.default_rng(tiles + hi % 1000)
    A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    check_products(ctx, A, w, B)
    out, _ = ctx.eliminate_node(dev(A), dev(w), dev(B), want_argmin=False)
    ctx.synchronize()
    for b in range(0, batch, max(1, batch // 4)):
        assert np.array_equal(out[b].cpu().numpy(), oracle.minplus_argmin(A[b], w[b], B[b])[0])


@pytest.mark.parametrize("shape", [(9, 512, 200, 512), (13, 512, 100, 500), (1, 1600, 300, 1550), (25, 500, 300, 510)])
@pytest.mark.parametrize("hi", [3, 1 << 20, (1 << 28) - 1])
def test_eliminate_node_tiles_left_over_after_whole_rounds_are_shared(ctx, shape, hi):
    # launches of two to six tiles per compute unit and a few more: what is left once every unit has had
    # the same number of whole tiles (tiles modulo 256, here 64, 64, 113, 64) is shared by several
    # workgroups each, the rest of the launch is whole tiles
    batch, Ci, Cj, Ck = shape
    tiles = batch * (-(-Ci // 64)) * (-(-Ck // 64))
    assert tiles > 512 and 0 < tiles % 256 <= 128
    rng = np.random.default_rng(tiles + hi % 1000)
    A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    check_products(ctx, A, w, B)


@pytest.mark.parametrize("shape", [(5, 512, 300, 512), (7, 500, 200, 512), (1, 1100, 520, 1150), (21, 512, 130, 512)])
def test_eliminate_node_one_to_five_whole_tiles_per_unit_and_leftovers(ctx, shape):
    # 320, 448, 324 and 1344 tiles: one whole tile (five in the last case) per compute unit, the other 64,
    # 192, 68 and 64 tiles shared -- 4, 4, 4 and 2 parts each
    batch, Ci, Cj, Ck = shape
    tiles = batch * (-(-Ci // 64)) * (-(-Ck // 64))
    assert tiles > 256 and tiles % 256 != 0
    rng = np.random.default_rng(tiles)
    for hi in (3, 1 << 20):
        A = rng.integers(0, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
        w = rng.integers(0, hi, size=(batch, Cj), endpoint=True, dtype=np.int32)
        B = rng.integers(0, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
        check_products(ctx, A, w, B)


@pytest.mark.parametrize("want_argmin", [True, False])
def test_eliminate_node_ranges_taken_tile_by_tile(ctx, want_argmin):
    # lwp_eliminate_node with few output tiles: every workgroup measures the rows of A, the columns of B and
    # the w its own tile reads, and picks its arithmetic from them.  Here the tiles of one product differ:
    # rows 0..63 of A and columns 0..63 of B are narrow (packed keys), the rest spreads over 2^28 (compare /
    # select), one block is negative; ties within the narrow blocks; three products at different levels.
    # The tiled kernel is forced (the call is small enough for the other one); then a batch of 700 products
    # of one tile each, the form batches of small products take.
    rng = np.random.default_rng(64)
    batch, Ci, Cj, Ck = 3, 200, 300, 260
    A = rng.integers(0, 3, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    A[:, 64:128] = rng.integers(0, 1 << 28, size=(batch, 64, Cj), dtype=np.int32)
    A[:, 128:] = rng.integers(-(1 << 27), 0, size=(batch, Ci - 128, Cj), dtype=np.int32)
    w = rng.integers(0, 5, size=(batch, Cj), endpoint=True, dtype=np.int32) + np.arange(batch, dtype=np.int32)[:, None] * 100000
    B = rng.integers(0, 3, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    B[:, :, 64:192] = rng.integers(0, 1 << 28, size=(batch, Cj, 128), dtype=np.int32)
    ctx.set_small_product_kernel(False)
    try:
        for a, ww, b in ((A, w, B), (A[:, :40, :33].repeat(234, axis=0)[:700] + 0, w[:, :33].repeat(234, axis=0)[:700] + 0,
                                     B[:, :33, 60:110].repeat(234, axis=0)[:700] + 0)):
            out, arg = ctx.eliminate_node(dev(a), dev(ww), dev(b), want_argmin=want_argmin)
            ctx.synchronize()
            out = out.cpu().numpy()
            for q in range(0, a.shape[0], max(1, a.shape[0] // 7)):
                ro, ra = oracle.minplus_argmin(a[q], ww[q], b[q])
                assert np.array_equal(out[q], ro)
                if want_argmin:
                    assert np.array_equal(arg[q].cpu().numpy(), ra)
    finally:
        ctx.set_small_product_kernel(True)


def test_split_tiles_never_read_a_previous_launchs_partials(ctx):
    # the parts of a tile meet in scratch memory that every launch reuses: with fresh data per launch
    # a part published too late (or read too early) would show as a result of the launch before
    rng = np.random.default_rng(4242)
    for rep in range(40):
        for batch, Ci, Cj, Ck in ((1, 64, 2048, 64), (1, 512, 512, 512), (3, 100, 700, 90)):
            A = rng.integers(0, 1 << 20, size=(batch, Ci, Cj), dtype=np.int32)
            w = rng.integers(0, 1 << 20, size=(batch, Cj), dtype=np.int32)
            B = rng.integers(0, 1 << 20, size=(batch, Cj, Ck), dtype=np.int32)
            out, arg = ctx.eliminate_node(dev(A), dev(w), dev(B))
            out, arg = out.cpu().numpy(), arg.cpu().numpy()
            for b in range(batch):
                ro, ra = oracle.minplus_argmin(A[b], w[b], B[b])
                assert np.array_equal(out[b], ro) and np.array_equal(arg[b], ra), (rep, batch, Ci, Cj, Ck)


def test_split_tiles_with_an_empty_part_and_costs_next_to_int32_max(ctx):
    # Cj = 257 is 9 stages of 32; split four ways (3 stages each) the last part has no candidates at
    # all and holds only padding.  With all costs just below INT32_MAX the padding must still lose.
    rng = np.random.default_rng(257)
    for Cj in (257, 260, 288):
        base = 1 << 30
        A = rng.integers(base, base + 1000, size=(1, 130, Cj), endpoint=True, dtype=np.int32)
        w = rng.integers(0, 1000, size=(1, Cj), endpoint=True, dtype=np.int32)
        B = rng.integers(base - 5000, base - 4000, size=(1, Cj, 140), endpoint=True, dtype=np.int32)
        check_products(ctx, A, w, B, expect_keyed=True)
        # the same through a search whose round mixes shapes (parts are sized for the longest product)
    Cn = np.array([70, 257, 40, 33, 64, 288, 50], np.int32)
    edges = wl.chain_edges(len(Cn))
    tc, ts, tx = wl.ragged_tables(len(Cn), edges, Cn, 5, 0, 1000)
    tx = (tx.astype(np.int64) + (1 << 28)).astype(np.int32)          # 6 edges: totals stay below 2^31
    ref = oracle.search_ragged(len(Cn), edges, Cn, tc, ts, tx)
    for undo in (0, 1):
        cost, S = ctx.search_graph_ragged(len(Cn), edges, Cn, dev(tc), dev(ts), dev(tx), 0, undo)
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])


# shapes of at least 2^28 cell updates (smaller launches are bound by latency and stay on the plain
# variant): ragged in every dimension, fewer rows than a tile, the longest c range, a batch, split tiles
@pytest.mark.parametrize("shape", [(1, 333, 1000, 900), (2, 130, 2570, 500), (40, 100, 330, 290), (1, 3, 65536, 1400),
                                   (1, 512, 1024, 512), (9, 257, 513, 257)])
@pytest.mark.parametrize("b_bits", [1, 12, 24])
def test_eliminate_node_keys_rebased_per_row(ctx, shape, b_bits):
    # A and w range over 2^29 (no global offset brings A + w + B into 26 bits) while B is narrow:
    # every row of A + w is re-based to its own minimum and the packed keys still apply
    batch, Ci, Cj, Ck = shape
    rng = np.random.default_rng(Cj * 31 + b_bits)
    A = rng.integers(-(1 << 28), 1 << 28, size=(batch, Ci, Cj), dtype=np.int32)
    w = rng.integers(-(1 << 28), 1 << 28, size=(batch, Cj), dtype=np.int32)
    B = rng.integers(1000, 1000 + (1 << b_bits) - 1, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    # ties: repeat candidates exactly, and rows whose minimum is attained many times
    A[:, :, Cj // 2:] = A[:, :, :Cj - Cj // 2]
    w[:, Cj // 2:] = w[:, :Cj - Cj // 2]
    B[:, Cj // 2:, :] = B[:, :Cj - Cj // 2, :]
    if Ci > 2:
        A[:, 1, :] = -w                                   # a whole row of A + w equal to 0
    check_products(ctx, A, w, B, expect_keyed=True)
    if b_bits == 1:                                       # the same launch below the size threshold: plain
        check_products(ctx, A[:1, :, :64], w[:1, :64], B[:1, :64, :], expect_keyed=False)


def test_search_with_wide_node_costs_stays_on_packed_keys(ctx):
    # node costs from microseconds to half a second, transfers up to a few milliseconds: the shape
    # of real cost tables (Sec. 5.1), at a size where arithmetic dominates
    p = wl.chain_problem(6, 700, 3, tc_range=(1000, 1 << 29), ts_range=(0, 1 << 20), tx_range=(0, 1 << 22))
    ctx.profile_enable(True)
    ctx.profile_reset()
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        run_search(ctx, p, schedule)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    # run_search runs every search twice: with stored argmin (every product on packed keys: on global
    # offsets where clamping at the largest possible result absorbs the width of the node costs, else
    # re-based per row) and with recomputed argmin (value-only)
    n_products = 2 * 2 * (p["n_nodes"] - 2)      # ... and each of those with the small-product kernel allowed and not
    assert prof["products_keyed"] + prof["products_keyed_row"] == n_products and prof["products_value"] == n_products
    assert prof["products_plain"] == 0
    Cn = np.array([700, 650, 701, 300, 900, 640], np.int32)      # the same with per-node counts
    edges = wl.chain_edges(6)
    tc, ts, tx = wl.ragged_tables(6, edges, Cn, 8, 0, 1 << 22)
    tc = (tc.astype(np.int64) * 100).astype(np.int32)
    ref = oracle.search_ragged(6, edges, Cn, tc, ts, tx)
    cost, S = ctx.search_graph_ragged(6, edges, Cn, dev(tc), dev(ts), dev(tx))
    assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])


def test_eliminate_node_negative_and_offset_values(ctx):
    rng = np.random.default_rng(11)
    A = rng.integers(-(1 << 20), 1 << 10, size=(2, 70, 90, ), dtype=np.int32).reshape(2, 70, 90)
    w = rng.integers(-5000, 5000, size=(2, 90), dtype=np.int32)
    B = rng.integers((1 << 29), (1 << 29) + 1000, size=(2, 90, 50), dtype=np.int32)
    check_products(ctx, A, w, B, expect_keyed=True)       # re-based into the key range
    A = rng.integers(-(1 << 30), 1 << 30, size=(1, 33, 47), dtype=np.int32)
    w = rng.integers(-(1 << 20), 1 << 20, size=(1, 47), dtype=np.int32)
    B = rng.integers(-(1 << 29), 1 << 29, size=(1, 47, 65), dtype=np.int32)
    check_products(ctx, A, w, B, expect_keyed=False)


def test_eliminate_node_closed_forms(ctx, kernels):
    C = 150
    rng = np.random.default_rng(2)
    A = rng.integers(0, 1000, size=(1, 77, C), dtype=np.int32)
    B = np.full((1, C, C), 1 << 24, np.int32)
    B[0][np.arange(C), np.arange(C)] = 0
    out, arg = ctx.eliminate_node(dev(A), dev(np.zeros((1, C), np.int32)), dev(B))
    assert np.array_equal(out.cpu().numpy(), A)
    assert np.array_equal(arg.cpu().numpy()[0], np.tile(np.arange(C, dtype=np.int32), (77, 1)))
    out, arg = ctx.eliminate_node(dev(np.full((1, 9, 40), 4)), dev(np.full((1, 40), 2)), dev(np.full((1, 40, 6), 1)))
    assert (out.cpu().numpy() == 7).all() and (arg.cpu().numpy() == 0).all()


@pytest.mark.parametrize("shape", [(2, 50, 60, 70), (1, 64, 2048, 64), (3, 130, 257, 140), (40, 256, 100, 256), (600, 128, 40, 256),
                                   (7, 250, 40, 250), (4, 200, 60, 200)])
@pytest.mark.parametrize("lo,hi", [(0, 3), (0, 1 << 20), (-(1 << 29), 1 << 29)])
def test_eliminate_node_value_only(ctx, kernels, shape, lo, hi):
    # no argmin requested: the value-only variant (any int32 range) must give the same minima
    batch, Ci, Cj, Ck = shape
    rng = np.random.default_rng(abs(hash((shape, lo, hi))) % (1 << 32))
    A = rng.integers(lo, hi, size=(batch, Ci, Cj), endpoint=True, dtype=np.int32)
    w = rng.integers(lo // 4, hi // 4 + 1, size=(batch, Cj), endpoint=True, dtype=np.int32)
    B = rng.integers(lo, hi, size=(batch, Cj, Ck), endpoint=True, dtype=np.int32)
    out, arg = ctx.eliminate_node(dev(A), dev(w), dev(B), want_argmin=False)
    assert arg is None
    out = out.cpu().numpy()
    for b in range(0, batch, max(1, batch // 7)):
        assert np.array_equal(out[b], oracle.minplus_argmin(A[b], w[b], B[b])[0]), b


def test_eliminate_node_overflow(ctx, kernels):
    from paper_1802_04924_amd import LwpError
    big = np.full((1, 4, 4), (1 << 31) - 1, np.int32)
    ones, zeros = np.ones((1, 4), np.int32), np.zeros((1, 4, 4), np.int32)
    for want_argmin in (True, False):
        ctx.eliminate_node(dev(big), dev(ones), dev(zeros), want_argmin=want_argmin)     # only enqueues
        with pytest.raises(LwpError) as e:
            ctx.synchronize()                                   # the device found the overflow
        assert e.value.code == -4
        ctx.synchronize()                                       # reported once
    # only one product of a batch overflows
    A = np.zeros((3, 70, 40), np.int32)
    A[1, 5, 7] = (1 << 31) - 1
    ctx.eliminate_node(dev(A), dev(np.ones((3, 40), np.int32)), dev(np.zeros((3, 40, 9), np.int32)))
    with pytest.raises(LwpError) as e:
        ctx.synchronize()
    assert e.value.code == -4
    with pytest.raises(LwpError) as e:                          # promised ranges: refused before any launch
        ctx.eliminate_node(dev(big), dev(ones), dev(zeros), bounds=(0, (1 << 31) - 1, 1, 1, 0, 0))
    assert e.value.code == -4
    ctx.synchronize()


def test_eliminate_node_batch_with_different_cost_levels(ctx):
    # Eq. 2 holds per product: products of one batch whose node costs w sit at different levels (the
    # layers of one round differ in compute time) must not share a value range.  Product b has w
    # shifted by 1000 b; with A and B in [0, 10] a range taken over the whole batch would clamp
    # every candidate of the later products.
    rng = np.random.default_rng(1000)
    for hi, batch in ((10, 2), (10, 9), (1, 5), (1 << 16, 4)):
        A = rng.integers(0, hi, size=(batch, 70, 90), endpoint=True, dtype=np.int32)
        B = rng.integers(0, hi, size=(batch, 90, 130), endpoint=True, dtype=np.int32)
        w = rng.integers(0, hi, size=(batch, 90), endpoint=True, dtype=np.int32)
        w += (1000 * np.arange(batch, dtype=np.int32))[:, None] * (1 if hi < 100 else 1 << 10)
        check_products(ctx, A, w, B, expect_keyed=True)
    # ... and products of one batch that need different variants: packed keys, and compare/select
    A = rng.integers(0, 1000, size=(3, 64, 100), dtype=np.int32)
    B = rng.integers(0, 1000, size=(3, 100, 64), dtype=np.int32)
    w = rng.integers(0, 1000, size=(3, 100), dtype=np.int32)
    B[1] = rng.integers(-(1 << 29), 1 << 29, size=(100, 64), dtype=np.int32)
    ctx.profile_enable(True)
    prof = check_products(ctx, A, w, B, expect_keyed_bounded=False)
    assert prof["products_keyed"] == 2 and prof["products_plain"] == 1


@pytest.mark.parametrize("shape", [(2, 200, 300, 150), (2, 100, 150, 75), (600, 32, 20, 32)])
def test_eliminate_node_promised_ranges_are_checked(ctx, kernels, shape):
    # (the first shape is past the size up to which a call with promised ranges takes the wavefront-per-tile
    # kernel, the second is within it, the third within it on that kernel's 16 x 16 tiles)
    from paper_1802_04924_amd import LwpError
    rng = np.random.default_rng(77)
    A = rng.integers(0, 1000, size=shape[:3], dtype=np.int32)
    w = rng.integers(0, 1000, size=(shape[0], shape[2]), dtype=np.int32)
    B = rng.integers(0, 1000, size=(shape[0], shape[2], shape[3]), dtype=np.int32)
    good = (0, 999, 0, 999, 0, 999)
    wide = (-5, 5000, -7, 1 << 20, -1, 1 << 12)              # true, though no value attains them
    for bounds in (good, wide):
        for want_argmin in (True, False):
            out, arg = ctx.eliminate_node(dev(A), dev(w), dev(B), bounds=bounds, want_argmin=want_argmin)
            ctx.synchronize()
            for b in range(shape[0]):
                ro, ra = oracle.minplus_argmin(A[b], w[b], B[b])
                assert np.array_equal(out[b].cpu().numpy(), ro)
                assert arg is None or np.array_equal(arg[b].cpu().numpy(), ra)
    # one element outside the promise, in any operand, anywhere: found on the device
    b, Ci, Cj, Ck = shape
    for which, idx in (("A", (b - 1, Ci - 1, Cj - 1)), ("A", (0, 0, 0)), ("w", (b - 1, Cj // 2)), ("B", (0, Cj - 1, Ck - 1)),
                       ("B", (b - 1, 3, Ck // 2))):
        for value in (1000, -1, (1 << 31) - 1, -(1 << 31)):
            X = {"A": A.copy(), "w": w.copy(), "B": B.copy()}
            X[which][idx] = value
            for want_argmin in (True, False):
                ctx.eliminate_node(dev(X["A"]), dev(X["w"]), dev(X["B"]), bounds=good, want_argmin=want_argmin)
                with pytest.raises(LwpError) as e:
                    ctx.synchronize()
                assert e.value.code == -1, (which, idx, value)
    ctx.synchronize()


def test_eliminate_edge_overflow(ctx):
    from paper_1802_04924_amd import LwpError
    e1 = np.full((1, 33, 47), 1 << 30, np.int32)
    e2 = np.zeros((1, 33, 47), np.int32)
    ctx.eliminate_edge(dev(e1), dev(e2))
    ctx.synchronize()
    e2[0, 32, 46] = 1 << 30
    ctx.eliminate_edge(dev(e1), dev(e2))
    with pytest.raises(LwpError) as e:
        ctx.synchronize()
    assert e.value.code == -4
    with pytest.raises(oracle.OracleError):
        oracle.edge_sum(e1[0], e2[0])
    ctx.synchronize()


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 17, 5), (2, 128, 128), (1, 1000, 999)])
def test_eliminate_edge(ctx, shape):
    rng = np.random.default_rng(sum(shape))
    e1 = rng.integers(-(1 << 29), 1 << 29, size=shape, dtype=np.int32)
    e2 = rng.integers(-(1 << 29), 1 << 29, size=shape, dtype=np.int32)
    out = ctx.eliminate_edge(dev(e1), dev(e2)).cpu().numpy()
    for b in range(shape[0]):
        assert np.array_equal(out[b], oracle.edge_sum(e1[b], e2[b]))
    d1 = dev(e1)
    ctx.eliminate_edge(d1, dev(e2), out=d1)            # in place
    assert np.array_equal(d1.cpu().numpy(), e1 + e2)


def run_search(ctx, p, schedule=None):
    """Both undo modes (stored argmin tables / recomputed argmin, as the paper's Alg. 1 does) must
    return the oracle's cost and strategy."""
    from paper_1802_04924_amd import UNDO_RECOMPUTE, UNDO_STORED
    schedule = p["schedule"] if schedule is None else schedule
    ref = oracle.search(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"], schedule)
    d_tc, d_ts, d_tx = dev(p["tc"]), dev(p["ts"]), dev(p["tx"])
    # a small search runs as one launch of one workgroup unless told otherwise (the library decides;
    # the bound here is wider than its own): such searches are checked down both paths
    nodes_gone = len(ref["steps"]) and int((ref["steps"]["kind"] == 0).sum())
    both = nodes_gone * p["C"] ** 3 <= (1 << 22)
    # and rounds with little work run on the wavefront-per-tile kernel unless told otherwise: both kernels
    for single in ((True, False) if both else (True,)):
        ctx.set_single_launch(single)
        for wave in (True, False):
            ctx.set_small_product_kernel(wave)
            for undo in (UNDO_STORED, UNDO_RECOMPUTE):
                cost, S = ctx.search_graph(p["n_nodes"], p["edges"], p["C"], d_tc, d_ts, d_tx, schedule, undo)
                assert cost == ref["cost"], (undo, single, wave)
                assert np.array_equal(S, ref["strategy"]), (undo, single, wave)
    ctx.set_single_launch(True)
    ctx.set_small_product_kernel(True)
    assert oracle.strategy_cost(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"], S) == cost
    return cost, S


def test_search_config0(ctx):
    from oracle import brute
    p = wl.config0()
    cost, S = run_search(ctx, p)
    best, _, _ = brute.brute_force(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"])
    assert cost == best
    run_search(ctx, p, wl.SCHEDULE_LEFT_FOLD)


def test_small_search_with_hundreds_of_products_per_round(ctx):
    # a search small enough for one launch of one workgroup (with stored argmin tables its tables fit
    # that kernel's LDS) whose rounds hold 259, 130, 65, ... node eliminations: more than, and fewer
    # than, the 256 products whose cells that kernel deals out together; its descriptors (70 KB) do
    # not fit the kernel arguments, those of the 12-layer chain do
    for n_layers, C in ((520, 2), (12, 5), (300, 2)):
        p = wl.chain_problem(n_layers, C, n_layers, tx_range=(0, 3))       # heavy ties
        run_search(ctx, p)
        run_search(ctx, p, wl.SCHEDULE_LEFT_FOLD)
        # the one launch is not a min-plus launch: a search down that path records none
        ctx.profile_enable(True)
        ctx.profile_reset()
        ctx.search_graph(p["n_nodes"], p["edges"], p["C"], dev(p["tc"]), dev(p["ts"]), dev(p["tx"]))
        single = ctx.profile_read()["node_launches"]
        ctx.set_single_launch(False)
        ctx.profile_reset()
        ctx.search_graph(p["n_nodes"], p["edges"], p["C"], dev(p["tc"]), dev(p["ts"]), dev(p["tx"]))
        general = ctx.profile_read()["node_launches"]
        ctx.set_single_launch(True)
        ctx.profile_enable(False)
        assert single == 0 and general > 0


def test_search_graph_entry_point_itself(ctx):
    # lwp_search_graph as the header declares it (stored argmin), called through ctypes directly
    import ctypes
    from paper_1802_04924_amd import binding
    lib = binding.load()
    for p in (wl.config0(), wl.forkjoin_problem(2, 40, 9)):
        ref = oracle.search(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"], p["schedule"])
        d_tc, d_ts, d_tx = dev(p["tc"]), dev(p["ts"]), dev(p["tx"])
        edges = np.ascontiguousarray(p["edges"], np.int32)
        cost = ctypes.c_int32(-1)
        S = np.full(p["n_nodes"], -1, np.int32)
        rc = lib.lwp_search_graph(ctx._h, p["n_nodes"], len(edges), edges.ctypes.data, p["C"], d_tc.data_ptr(), d_ts.data_ptr(),
                                  d_tx.data_ptr(), p["schedule"], ctypes.byref(cost), S.ctypes.data)
        assert rc == 0
        assert cost.value == ref["cost"] and np.array_equal(S, ref["strategy"])
        n = lib.lwp_search_workspace_bytes(p["n_nodes"], len(edges), edges.ctypes.data, p["C"], p["schedule"])
        assert n > 0


@pytest.mark.parametrize("n_layers,C,hi", [(2, 7, 50), (3, 130, 1000), (11, 24, 3), (33, 200, 1 << 20), (9, 257, 1 << 24)])
@pytest.mark.parametrize("schedule", [wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD])
def test_search_chains(ctx, n_layers, C, hi, schedule):
    p = wl.chain_problem(n_layers, C, seed=n_layers + C, tc_range=(0, hi), ts_range=(0, hi), tx_range=(0, hi))
    run_search(ctx, p, schedule)


@pytest.mark.parametrize("modules,C,hi", [(1, 5, 3), (2, 33, 100000), (10, 64, 100000), (3, 128, 1)])
@pytest.mark.parametrize("schedule", [wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD])
def test_search_forkjoin(ctx, modules, C, hi, schedule):
    p = wl.forkjoin_problem(modules, C, seed=modules * 7 + C, lo=0, hi=hi)
    run_search(ctx, p, schedule)


@pytest.mark.parametrize("seed", range(8))
def test_search_random_series_parallel(ctx, seed):
    # random topologies: non-topological node ids, shuffled edges, multi-way parallel edges, and
    # (odd seeds) dangling branches that leave residual components to enumerate
    C = [3, 17, 64, 130][seed % 4]
    p = wl.series_parallel_problem(30 + 7 * seed, C, seed, hi=[2, 1000, 1 << 20][seed % 3], p_branch=0.08 if seed % 2 else 0.0)
    from paper_1802_04924_amd import plan_graph
    K = plan_graph(p["n_nodes"], p["edges"])["n_residual_nodes"]
    if K > 2 and C ** K > (1 << 32):              # possibly more strategies than either side enumerates
        p = wl.series_parallel_problem(30 + 7 * seed, 3, seed, hi=5, p_branch=0.08)
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        run_search(ctx, p, schedule)


def test_eliminate_node_maximum_candidate_count(ctx):
    # Cj at its limit of 65536: one tile, split over workgroups, widest index field
    rng = np.random.default_rng(65536)
    Cj = 65536
    for hi in (3, 1 << 12):
        A = rng.integers(0, hi, size=(1, 40, Cj), endpoint=True, dtype=np.int32)
        w = rng.integers(0, hi, size=(1, Cj), endpoint=True, dtype=np.int32)
        B = rng.integers(0, hi, size=(1, Cj, 70), endpoint=True, dtype=np.int32)
        check_products(ctx, A, w, B, expect_keyed=True)


def test_invalid_arguments_are_refused_before_any_launch(ctx):
    import ctypes
    from paper_1802_04924_amd import binding
    lib, h = binding.load(), ctx._h
    t = dev(np.zeros((4, 4), np.int32))
    p = ctypes.c_void_p(t.data_ptr())
    assert lib.lwp_eliminate_node(h, 1, 4, 4, 4, None, p, p, p, p) == binding.E_INVAL
    assert lib.lwp_eliminate_node(h, 0, 4, 4, 4, p, p, p, p, p) == binding.E_INVAL
    assert lib.lwp_eliminate_node(h, 1, 4, 1 << 17, 4, p, p, p, p, p) == binding.E_INVAL
    assert lib.lwp_eliminate_node(h, 1, 4, 4, 4, ctypes.c_void_p(t.data_ptr() + 2), p, p, p, p) == binding.E_INVAL
    assert lib.lwp_eliminate_edge(h, 1, 4, 4, p, None, p) == binding.E_INVAL
    assert lib.lwp_eliminate_edge(h, 1, -1, 4, p, p, p) == binding.E_INVAL
    cost = ctypes.c_int32(7)
    S = np.full(2, -5, np.int32)
    e = np.array([[0, 1]], np.int32)
    assert lib.lwp_search_graph(h, 2, 1, e.ctypes.data, 0, p, p, p, 0, ctypes.byref(cost), S.ctypes.data) == binding.E_INVAL
    assert lib.lwp_search_graph(h, 2, 1, e.ctypes.data, 4, p, p, None, 0, ctypes.byref(cost), S.ctypes.data) == binding.E_INVAL
    assert lib.lwp_search_graph_ex(h, 2, 1, e.ctypes.data, 4, p, p, p, 0, 9, ctypes.byref(cost), S.ctypes.data) == binding.E_INVAL
    bad = np.array([[0, 2]], np.int32)
    assert lib.lwp_search_graph(h, 2, 1, bad.ctypes.data, 4, p, p, p, 0, ctypes.byref(cost), S.ctypes.data) == binding.E_GRAPH
    assert cost.value == 7 and (S == -5).all()              # outputs untouched on error
    assert b"endpoint" in lib.lwp_last_error(h)
    assert lib.lwp_eliminate_node(None, 1, 4, 4, 4, p, p, p, p, p) == binding.E_INVAL


def test_search_small_irregular_graphs(ctx):
    graphs = {
        "single": (1, []), "two_isolated": (2, []), "parallel3": (2, [(0, 1), (0, 1), (0, 1)]),
        "diamond_skip": (4, [(0, 1), (0, 2), (1, 3), (2, 3), (0, 3)]),
        "backward_ids": (4, [(3, 1), (1, 0), (0, 2)]),
        "two_chains": (6, [(0, 1), (1, 2), (3, 4), (4, 5)]),
        "residual": (6, [(0, 1), (1, 2), (2, 3), (1, 4), (4, 3), (3, 5), (3, 5)]),
    }
    for name, (n, e) in graphs.items():
        edges = np.asarray(e, np.int32).reshape(-1, 2)
        for C, hi in ((1, 9), (3, 2), (19, 1000)):
            tc, ts, tx = wl.random_tables(n, edges, C, 3, (0, hi), (0, hi), (0, hi))
            p = {"n_nodes": n, "edges": edges, "C": C, "tc": tc, "ts": ts, "tx": tx, "schedule": 0}
            run_search(ctx, p)


IRREDUCIBLE = {
    "star_out": (4, [(0, 1), (0, 2), (0, 3)]),
    "star_in": (4, [(1, 0), (2, 0), (3, 0)]),
    "two_sources": (4, [(0, 2), (1, 2), (2, 3)]),
    "bipartite": (4, [(0, 2), (0, 3), (1, 2), (1, 3)]),
    "two_towers": (7, [(0, 1), (1, 4), (2, 3), (3, 4), (4, 5), (5, 6), (4, 6)]),
    "mixed_components": (8, [(0, 1), (0, 2), (0, 3), (4, 5), (5, 6), (7, 6)]),
    "triple_in": (9, [(0, 1), (1, 8), (2, 3), (3, 8), (4, 5), (5, 6), (6, 8), (7, 8)]),
}


@pytest.mark.parametrize("name", sorted(IRREDUCIBLE))
@pytest.mark.parametrize("C,hi", [(1, 7), (2, 1), (5, 3), (23, 1000), (64, 1 << 20)])
def test_search_enumerates_residual_components(ctx, name, C, hi):
    # the largest component here has 5 nodes: at most 64^5 = 2^30 strategies, which both sides enumerate
    n, e = IRREDUCIBLE[name]
    edges = np.asarray(e, np.int32)
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        tc, ts, tx = wl.random_tables(n, edges, C, C + hi, (0, hi), (0, hi), (0, hi))
        p = {"n_nodes": n, "edges": edges, "C": C, "tc": tc, "ts": ts, "tx": tx, "schedule": schedule}
        run_search(ctx, p)


@pytest.mark.parametrize("C,hi", [(160, 1 << 20), (250, 1 << 20), (256, 3)])
def test_search_enumerates_up_to_2_pow_32_strategies(ctx, C, hi):
    # a layer feeding three layers that never rejoin: nothing can be eliminated and all C^4 strategies
    # of the final graph are enumerated (Alg. 1).  160^4 = 6.6e8 is the size the benchmark's residual
    # workload times, 250^4 = 3.9e9 lies just under the limit of 2^32, 256^4 is the limit itself (the
    # flat strategy index then uses all 32 bits; small costs make ties that only the index resolves)
    edges = np.array([[0, 1], [0, 2], [0, 3]], np.int32)
    tc, ts, tx = wl.random_tables(4, edges, C, 7, (0, hi), (0, hi), (0, hi))
    run_search(ctx, {"n_nodes": 4, "edges": edges, "C": C, "tc": tc, "ts": ts, "tx": tx, "schedule": wl.SCHEDULE_ROUNDS})


def test_search_refuses_more_than_2_pow_32_strategies(ctx):
    from paper_1802_04924_amd import LwpError
    edges = np.array([[0, 1], [0, 2], [0, 3]], np.int32)
    tc, ts, tx = wl.random_tables(4, edges, 257, 7, (0, 9), (0, 9), (0, 9))
    with pytest.raises(LwpError) as e:
        ctx.search_graph(4, edges, 257, dev(tc), dev(ts), dev(tx))
    assert e.value.code == -3
    with pytest.raises(oracle.OracleError) as e2:
        oracle.search(4, edges, 257, tc, ts, tx)
    assert e2.value.code == oracle.E_NOT_REDUCIBLE


def test_search_beyond_the_provable_bounds(ctx):
    # worst-case bounds grow by max t_x per elimination and leave int32 after ~16 steps here, while
    # the minima stay small: the search must neither refuse nor lose exactness
    p = wl.chain_problem(40, 48, 3, tc_range=(0, 1 << 20), ts_range=(0, 1 << 20), tx_range=(0, 1 << 27))
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        run_search(ctx, p, schedule)
    p = wl.forkjoin_problem(3, 40, 4, lo=0, hi=1 << 25)
    run_search(ctx, p)
    # the same above the size (2^29 cell updates) from which a search reads the value ranges back and
    # picks packed-key variants: unprovable bounds then meet keys whose width comes from measured ranges
    p = wl.chain_problem(40, 256, 5, tc_range=(0, 1 << 20), ts_range=(0, 1 << 20), tx_range=(0, 1 << 27))
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        run_search(ctx, p, schedule)


def test_search_picks_its_arithmetic_without_reading_values_back():
    # A search with stored argmin never reads value ranges back.  Small searches (bound by latency) run
    # on compare/select.  Larger ones are launched on packed keys speculatively; a product whose measured
    # ranges do not allow them is skipped and flagged on the device, and the search runs again on the
    # kernel that picks keys, keys per row or compare/select per product -- which later searches of the
    # same context then start with.  Whatever the search's arithmetic, a round with little work (here
    # the late rounds, one product each) runs on the wavefront-per-tile kernel, which is compare/select.
    from paper_1802_04924_amd import Context
    with Context(0) as c:
        c.profile_enable(True)
        for n_layers, C, expect, at_least in ((4, 160, "plain", 2), (5, 512, "plain", 3), (6, 512, "keyed", 2)):   # 3 * 2^27 and 4 * 2^27 updates
            p = wl.chain_problem(n_layers, C, n_layers, tc_range=(0, 1000), ts_range=(0, 1000), tx_range=(0, 1000))
            ref = oracle.search(p["n_nodes"], p["edges"], C, p["tc"], p["ts"], p["tx"])
            c.profile_reset()
            cost, S = c.search_graph(p["n_nodes"], p["edges"], C, dev(p["tc"]), dev(p["ts"]), dev(p["tx"]))
            prof = c.profile_read()
            assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
            assert prof["products_" + expect] >= at_least
            assert prof["products_keyed"] + prof["products_plain"] + prof["products_keyed_row"] == n_layers - 2
        # one table with values over 2^28: no global offset brings its products into the key range
        p = wl.chain_problem(6, 700, 9, tc_range=(0, 1000), ts_range=(0, 1000), tx_range=(0, 1000))
        p["tx"][2] = np.random.default_rng(5).integers(-(1 << 27), 1 << 27, size=(700, 700), dtype=np.int32)
        d = dev(p["tc"]), dev(p["ts"]), dev(p["tx"])
        for schedule in (wl.SCHEDULE_LEFT_FOLD, wl.SCHEDULE_ROUNDS):
            ref = oracle.search(6, p["edges"], 700, p["tc"], p["ts"], p["tx"], schedule)
            for rep in range(2):
                c.profile_reset()
                cost, S = c.search_graph(6, p["edges"], 700, *d, schedule)
                prof = c.profile_read()
                assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
                total = prof["products_keyed"] + prof["products_plain"] + prof["products_keyed_row"]
                first = schedule == wl.SCHEDULE_LEFT_FOLD and rep == 0
                # the first search of the context ran twice (products skipped by the first run are not counted)
                assert (4 < total <= 8) if first else total == 4
                # in the left fold the wide table is the B side of one product (compare/select); in rounds
                # it is an A side first (keys re-based per row) and its minima are narrow again
                assert prof["products_keyed"] >= 1
                assert prof["products_plain" if schedule == wl.SCHEDULE_LEFT_FOLD else "products_keyed_row"] >= 1
        # narrow tables again: the context stays on the picking kernel, results unchanged
        p = wl.chain_problem(6, 512, 6, tc_range=(0, 1000), ts_range=(0, 1000), tx_range=(0, 1000))
        ref = oracle.search(6, p["edges"], 512, p["tc"], p["ts"], p["tx"])
        cost, S = c.search_graph(6, p["edges"], 512, dev(p["tc"]), dev(p["ts"]), dev(p["tx"]))
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])


def test_search_overflow_found_on_the_device(ctx):
    from paper_1802_04924_amd import LwpError
    # parallel edges whose sum leaves int32
    edges = np.array([[0, 1], [0, 1], [0, 1], [1, 2]], np.int32)
    tc, ts, tx = wl.random_tables(3, edges, 8, 1, (0, 5), (0, 5), (1 << 30, (1 << 30) + 9))
    with pytest.raises(LwpError) as e:
        ctx.search_graph(3, edges, 8, dev(tc), dev(ts), dev(tx))
    assert e.value.code == -4
    with pytest.raises(oracle.OracleError):
        oracle.search(3, edges, 8, tc, ts, tx)
    # residual pair whose sum leaves int32
    edges = np.array([[0, 1]], np.int32)
    tc, ts, tx = wl.random_tables(2, edges, 8, 1, (1 << 29, (1 << 29) + 9), (0, 5), (1 << 30, (1 << 30) + 9))
    with pytest.raises(LwpError) as e:
        ctx.search_graph(2, edges, 8, dev(tc), dev(ts), dev(tx))
    assert e.value.code == -4


def test_small_search_sums_at_the_edges_of_int32(ctx):
    # The single-workgroup search reads overflow off the carries of its 32-bit additions: a sum of
    # three whose first two terms leave int32 while the total fits must pass, a total of exactly
    # INT32_MAX or INT32_MIN must pass, one beyond must be reported.  Three-layer chains, the middle
    # layer eliminated (Eq. 2); the end layers cost nothing, so the residual sums add nothing.
    from paper_1802_04924_amd import LwpError
    edges = np.array([[0, 1], [1, 2]], np.int32)
    C = 3
    def problem(a, w, b):
        tc = np.zeros((3, C), np.int32); ts = np.zeros((3, C), np.int32)
        tc[1] = w
        tx = np.stack([np.asarray(a, np.int64), np.asarray(b, np.int64)]).astype(np.int32)
        return dict(n_nodes=3, edges=edges, C=C, tc=tc, ts=ts, tx=tx, schedule=wl.SCHEDULE_ROUNDS)
    jitter = np.arange(C * C).reshape(C, C)
    fits = [
        # A + w = 2.4e9 leaves int32, A + w + B = 0.9e9 does not
        (1_200_000_000 + jitter, np.full(C, 1_200_000_000) + np.arange(C), -1_500_000_000 - jitter.T),
        # A + w = -2.4e9, total -0.9e9
        (-1_200_000_000 - jitter, np.full(C, -1_200_000_000) - np.arange(C), 1_500_000_000 + jitter),
        # the largest sum is exactly INT32_MAX, the smallest exactly INT32_MIN
        (np.full((C, C), 2**31 - 1 - 10) - jitter, np.full(C, 4), np.full((C, C), 6)),
        (np.full((C, C), -2**31 + 10) + jitter, np.full(C, -4), np.full((C, C), -6)),
    ]
    for a, w, b in fits:
        p = problem(a, w, b)
        ref = oracle.search(3, edges, C, p["tc"], p["ts"], p["tx"])
        ctx.set_single_launch(True)
        cost, S = ctx.search_graph(3, edges, C, dev(p["tc"]), dev(p["ts"]), dev(p["tx"]))
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
    beyond = [
        (np.full((C, C), 2**31 - 1 - 10) - jitter, np.full(C, 4), np.full((C, C), 6) + (jitter == 0)),     # one cell: 2^31
        (np.full((C, C), -2**31 + 10) + jitter, np.full(C, -4), np.full((C, C), -6) - (jitter == 0)),      # one cell: -2^31 - 1
        (np.full((C, C), 2**31 - 1), np.full(C, 2**31 - 1), np.full((C, C), 2**31 - 1)),                   # both additions carry
        (np.full((C, C), -2**31), np.full(C, -2**31), np.full((C, C), -2**31)),                            # neither does
    ]
    for a, w, b in beyond:
        p = problem(a, w, b)
        with pytest.raises(oracle.OracleError):
            oracle.search(3, edges, C, p["tc"], p["ts"], p["tx"])
        for single in (True, False):
            ctx.set_single_launch(single)
            with pytest.raises(LwpError) as e:
                ctx.search_graph(3, edges, C, dev(p["tc"]), dev(p["ts"]), dev(p["tx"]))
            assert e.value.code == -4
    ctx.set_single_launch(True)


def test_search_with_tables_that_are_only_ever_summed(ctx):
    # One Inception-shaped module with 512 configurations: its first round runs on the tiled kernel,
    # whose key widths follow value ranges measured on the device.  A table that is first added into a
    # parallel edge (Eq. 3) is not measured itself, only the sum is.  Here those tables (8 of 18) lie far
    # outside the range of all others, half of them negative: a range taken from the wrong table, or
    # none, would give wrong keys.
    from paper_1802_04924_amd import plan_graph
    p = wl.forkjoin_problem(1, 512, 7, lo=0, hi=1000)
    touched, direct, summed = set(), set(), set()
    for s in plan_graph(p["n_nodes"], p["edges"], p["schedule"])["steps"]:
        for e in (int(s["e1"]), int(s["e2"])):
            if e not in touched:
                (summed if s["kind"] == 1 else direct).add(e)
        touched.update((int(s["e1"]), int(s["e2"])))
    only_summed = sorted(summed - direct)
    assert len(only_summed) >= 4
    for q, e in enumerate(only_summed):
        p["tx"][e] += 3_000_000 if q % 2 == 0 else -5_000_000
    run_search(ctx, p)


def test_search_errors(ctx):
    from paper_1802_04924_amd import LwpError
    edges = np.array([[0, 1], [0, 2], [0, 3]], np.int32)
    tc, ts, tx = wl.random_tables(4, edges, 300, 0, (0, 5), (0, 5), (0, 5))
    with pytest.raises(LwpError) as e:
        ctx.search_graph(4, edges, 300, dev(tc), dev(ts), dev(tx))     # 300^4 > 2^32 strategies
    assert e.value.code == -3
    p = wl.chain_problem(4, 8, 1, tc_range=(1 << 30, (1 << 30) + 5))
    with pytest.raises(LwpError) as e:
        ctx.search_graph(4, p["edges"], 8, dev(p["tc"]), dev(p["ts"]), dev(p["tx"]))
    assert e.value.code == -4
    # the context stays usable after an error
    run_search(ctx, wl.config0())


# ------------------------------------------------------------------ analytic cost model (Sec. 5.1)
def test_build_cost_tables_alexnet_and_search(ctx):
    p = wl.config1()
    tc, ts, tx = ctx.build_cost_tables(p["layers"], p["edges"], p["configs"], p["machine"])
    rtc, rts, rtx = oracle.build_cost_tables(p["layers"], p["edges"], p["configs"], p["machine"])
    assert np.array_equal(tc.cpu().numpy(), rtc)
    assert np.array_equal(ts.cpu().numpy(), rts)
    assert np.array_equal(tx.cpu().numpy(), rtx)
    cost, S = ctx.search_graph(p["n_nodes"], p["edges"], p["C"], tc, ts, tx, p["schedule"])
    ref = oracle.search(p["n_nodes"], p["edges"], p["C"], rtc, rts, rtx, p["schedule"])
    assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
    assert oracle.strategy_cost(p["n_nodes"], p["edges"], p["C"], rtc, rts, rtx, S) == cost


def test_vgg16_tables_and_search(ctx):
    # second network shape through the cost model: 21-layer chain, tables built on the GPU
    p = wl.vgg16_problem()
    assert p["n_nodes"] == 21
    tc, ts, tx = ctx.build_cost_tables(p["layers"], p["edges"], p["configs"], p["machine"])
    rtc, rts, rtx = oracle.build_cost_tables(p["layers"], p["edges"], p["configs"], p["machine"])
    assert np.array_equal(tc.cpu().numpy(), rtc) and np.array_equal(ts.cpu().numpy(), rts)
    assert np.array_equal(tx.cpu().numpy(), rtx)
    ref = oracle.search(21, p["edges"], 256, rtc, rts, rtx)
    for undo in (0, 1):
        cost, S = ctx.search_graph(21, p["edges"], 256, tc, ts, tx, p["schedule"], undo)
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
    # every chosen configuration is one the layer can actually use
    assert (rtc[np.arange(21), S] < p["machine"]["invalid_cost"]).all()


def test_search_on_a_side_stream(ctx):
    # the context follows the stream it was created with; results must not depend on the default stream
    import torch
    from paper_1802_04924_amd import Context
    p = wl.forkjoin_problem(2, 96, 8)
    ref = oracle.search(p["n_nodes"], p["edges"], p["C"], p["tc"], p["ts"], p["tx"])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        d_tc, d_ts, d_tx = dev(p["tc"]), dev(p["ts"]), dev(p["tx"])
        with Context(0, stream=side) as c2:
            for _ in range(3):
                cost, S = c2.search_graph(p["n_nodes"], p["edges"], p["C"], d_tc, d_ts, d_tx)
                assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])
            A, w, B = wl.batched_products(2, 100, 300, 90, 4)
            out, arg = c2.eliminate_node(dev(A), dev(w), dev(B))
            c2.synchronize()
            ro, ra = oracle.minplus_argmin(A[1], w[1], B[1])
            assert np.array_equal(out[1].cpu().numpy(), ro) and np.array_equal(arg[1].cpu().numpy(), ra)
    side.synchronize()


def test_build_cost_tables_odd_shapes(ctx):
    # non power-of-two extents, strides, ragged splits, every layer kind as producer and consumer,
    # a skip edge, and a machine with other constants
    N = 6
    layers = np.asarray([
        (wl.KIND_CONV, N, 3, 23, 31, 10, 12, 16, 3, 3, 2, 2, 1, 1),
        (wl.KIND_POOL, N, 10, 12, 16, 10, 6, 8, 2, 2, 2, 2, 0, 0),
        (wl.KIND_CONV, N, 10, 6, 8, 7, 6, 8, 5, 3, 1, 1, 2, 1),
        (wl.KIND_POOL, N, 7, 6, 8, 7, 4, 6, 3, 3, 1, 1, 0, 0),
        (wl.KIND_FC, N, 7, 4, 6, 9, 1, 1, 4, 6, 1, 1, 0, 0),
        (wl.KIND_FC, N, 9, 1, 1, 5, 1, 1, 1, 1, 1, 1, 0, 0),
        (wl.KIND_CONV, N, 10, 6, 8, 7, 6, 8, 1, 1, 1, 1, 0, 0),
    ], np.int32)
    edges = np.array([[0, 1], [1, 2], [2, 3], [3, 4], [4, 5], [1, 6], [6, 3]], np.int32)
    rows = []
    for n in (1, 2, 3):
        for h in (1, 2, 3):
            for w in (1, 2):
                for c in (1, 2, 5):
                    d = n * h * w * c
                    for off in (0, 1, 5):
                        if off + d <= 12:
                            rows.append((n, h, w, c, off, 0))
    rows.append((0, 0, 0, 0, 0, 0))
    configs = np.asarray(rows, np.int32)
    m = {"n_devices": 12, "flop_per_ns": 7, "byte_per_ns": 3, "invalid_cost": 1 << 27}
    tc, ts, tx = ctx.build_cost_tables(layers, edges, configs, m)
    rtc, rts, rtx = oracle.build_cost_tables(layers, edges, configs, m)
    assert np.array_equal(tc.cpu().numpy(), rtc)
    assert np.array_equal(ts.cpu().numpy(), rts)
    assert np.array_equal(tx.cpu().numpy(), rtx)


def test_build_cost_tables_errors(ctx):
    from paper_1802_04924_amd import LwpError
    p = wl.config1()
    bad = p["layers"].copy()
    bad[3, 2] += 1                      # pool2 no longer accepts conv2's channels
    with pytest.raises(LwpError) as e:
        ctx.build_cost_tables(bad, p["edges"], p["configs"], p["machine"])
    assert e.value.code == -1
    slow = dict(p["machine"], byte_per_ns=1, flop_per_ns=1)
    with pytest.raises(LwpError) as e:
        ctx.build_cost_tables(p["layers"], p["edges"], p["configs"], slow)
    assert e.value.code == -4


@pytest.mark.parametrize("C,hi,bottleneck", [(3, 2, False), (40, 1000, False), (96, 1 << 20, True), (130, 100000, True)])
def test_search_resnet_shaped(ctx, C, hi, bottleneck):
    p = wl.resnet_problem(C, seed=C, bottleneck=bottleneck, lo=0, hi=hi)
    for schedule in (wl.SCHEDULE_ROUNDS, wl.SCHEDULE_LEFT_FOLD):
        run_search(ctx, p, schedule)


def test_search_long_chains(ctx):
    # thousands of layers: thousands of rounds under LEFT_FOLD, batches of thousands of tiny
    # products under ROUNDS
    p = wl.chain_problem(3000, 3, seed=30, tc_range=(0, 9), ts_range=(0, 9), tx_range=(0, 9))
    run_search(ctx, p, wl.SCHEDULE_ROUNDS)
    p = wl.chain_problem(1200, 5, seed=31, tc_range=(0, 1000), ts_range=(0, 1000), tx_range=(0, 1000))
    run_search(ctx, p, wl.SCHEDULE_LEFT_FOLD)
    # more layers than the undo pass keeps in LDS (4096) and more eliminations than it has threads (1024)
    p = wl.chain_problem(5000, 2, seed=32, tc_range=(0, 3), ts_range=(0, 3), tx_range=(0, 3))
    run_search(ctx, p, wl.SCHEDULE_ROUNDS)
    Cn = wl.ragged_counts(2500, 32, 1, 6)
    edges = wl.chain_edges(2500)
    tc, ts, tx = wl.ragged_tables(2500, edges, Cn, 33, 0, 50)
    ref = oracle.search_ragged(2500, edges, Cn, tc, ts, tx)
    for undo in (0, 1):
        cost, S = ctx.search_graph_ragged(2500, edges, Cn, dev(tc), dev(ts), dev(tx), 0, undo)
        assert cost == ref["cost"] and np.array_equal(S, ref["strategy"])


def test_measured_valu_rate_probe_reports_consistent_figures(ctx):
    # the register-only probe reports lane-operations/s and the cell updates/s they amount to: 64 updates
    # per 96 arithmetic instructions of its loop (64 adds, 32 three-way mins).  How close the
    # rate is to 256 CUs x 64 lanes x 2.4 GHz depends on the clock the box runs at, which is no matter
    # of parity: reported, not asserted.
    import warnings
    r = ctx.measure_valu_rate()
    assert r["lane_ops_per_s"] > 0
    assert abs(r["cell_updates_per_s"] / r["lane_ops_per_s"] - 64 / 96) < 1e-9
    ratio = r["lane_ops_per_s"] / 39.3216e12
    if not 0.80 < ratio < 1.15:
        warnings.warn(f"VALU probe at {ratio:.2f} of the 2.4 GHz peak: the box runs at an unusual clock")
