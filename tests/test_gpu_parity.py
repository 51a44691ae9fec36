"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on the same inputs."""
import ctypes

import numpy as np
import pytest

from paper_2402_10517_amd import inputs
from gpu_util import check_against_oracle, run_gemv

pytestmark = pytest.mark.gpu
ALL_BITS = list(range(3, 9))


@pytest.fixture(scope="module")
def B():
    from paper_2402_10517_amd import binding
    return binding


@pytest.fixture(scope="module")
def tiny(B):
    idx, luts, x = inputs.make_case(1, 512, 512)
    pm = B.ap_pack(idx, luts)
    yield idx, luts, x, pm
    pm.close()


@pytest.mark.parametrize("b", ALL_BITS)
def test_config1_tiny_all_bit_widths(B, tiny, b):
    idx, luts, x, pm = tiny
    y = run_gemv(pm, b, x)
    check_against_oracle(y, idx, luts[b], b, x)


def test_device_round_trip_is_bit_exact(B, tiny):
    idx, _, _, pm = tiny
    assert np.array_equal(B.ap_unpack(pm), idx)
    for (M, K) in [(37, 2048 + 160), (5, 96)]:
        idx2, luts2, _ = inputs.make_case(11, M, K)
        pm2 = B.ap_pack(idx2, luts2)
        assert np.array_equal(B.ap_unpack(pm2), idx2)
        pm2.close()


# several spans per row, a ragged last span, rows not a multiple of 4, 1/2/4 waves per group
RAGGED = [(37, 96), (4, 32), (70, 2048 + 160), (129, 4096 + 32), (66, 3 * 2048), (10, 5 * 2048 + 736),
          (257, 9 * 2048 + 32)]


@pytest.mark.parametrize("M,K", RAGGED)
@pytest.mark.parametrize("b", ALL_BITS)
def test_ragged_shapes(B, M, K, b):
    idx, luts, x = inputs.make_case(12, M, K)
    pm = B.ap_pack(idx, {b: luts[b]})
    y = run_gemv(pm, b, x)
    check_against_oracle(y, idx, luts[b], b, x)
    pm.close()


@pytest.mark.parametrize("batch", range(1, 9))
@pytest.mark.parametrize("b", [3, 4, 6, 8])
def test_batches_one_to_eight(B, batch, b):
    M, K = 132, 2048 + 512
    idx, luts, x = inputs.make_case(13, M, K, batch=batch, sigma=0.01)
    pm = B.ap_pack(idx, {b: luts[b]})
    y = run_gemv(pm, b, x)
    assert y.shape == (batch, M)
    check_against_oracle(y, idx, luts[b], b, x)
    # a row of a batched call equals the batch-1 call on that row, bit for bit or within tolerance
    y0 = run_gemv(pm, b, x[batch - 1:batch])
    check_against_oracle(y0, idx, luts[b], b, x[batch - 1:batch])
    pm.close()


@pytest.mark.parametrize("batch", [9, 12, 16])
def test_batches_nine_to_sixteen_run_as_two_passes(B, batch):
    # rows 8.. of a larger batch equal a separate call on those rows, bit for bit; canaries around y;
    # shapes that reach the ALU kernels and (K % 256 == 0, forced) the tile kernel in both passes
    import ctypes
    import torch
    for (M, K, opts) in [(132, 2048 + 96, {}), (70, 2048 + 768, dict(variant=9))]:
        idx, luts, x = inputs.make_case(29, M, K, batch=batch, sigma=0.01)
        pm = B.ap_pack(idx, luts).set_options(**opts)
        guard = 64
        sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        xd = torch.from_numpy(x).cuda()
        for b in (3, 5, 8):
            ybuf = torch.full((guard + batch * M + guard,), -7.0, dtype=torch.float16, device="cuda")
            assert B.lib.ap_gemv(pm.handle, b, xd.data_ptr(), ybuf.data_ptr() + 2 * guard, batch, sp) == 0
            torch.cuda.synchronize()
            out = ybuf.cpu().numpy()
            assert np.all(out[:guard] == -7.0) and np.all(out[-guard:] == -7.0)
            y = out[guard:-guard].reshape(batch, M)
            check_against_oracle(y, idx, luts[b], b, x)
            y_tail = run_gemv(pm, b, x[8:])
            assert np.array_equal(y[8:].view(np.uint16), y_tail.view(np.uint16))
        pm.close()


@pytest.mark.parametrize("b", ALL_BITS)
def test_one_hot_activation_is_exact(B, b):
    M, K = 64, 2048 + 96
    idx, luts, _ = inputs.make_case(14, M, K)
    pm = B.ap_pack(idx, {b: luts[b]})
    for j in (0, 1, 7, 8, 511, 512, 1023, 2047, 2048, 2049, K - 33, K - 1):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, j] = 1.0
        y = run_gemv(pm, b, x)
        expect = luts[b][np.arange(M), idx[:, j] >> (8 - b)]
        assert np.array_equal(y[0].view(np.uint16) & 0x7fff != 0, expect.view(np.uint16) & 0x7fff != 0)
        assert np.array_equal(y[0], expect), "column %d" % j
    pm.close()


@pytest.mark.parametrize("b", ALL_BITS)
def test_integer_table_pins_bit_order_end_to_end(B, b):
    M, K = 24, 2048 + 64
    idx, _, _ = inputs.make_case(15, M, K)
    lut = np.tile(np.arange(1 << b, dtype=np.float16), (M, 1))
    pm = B.ap_pack(idx, {b: lut})
    for j in (0, 5, 300, 2047, 2050, K - 1):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, j] = 1.0
        y = run_gemv(pm, b, x)
        assert np.array_equal(y[0].astype(np.int64), idx[:, j].astype(np.int64) >> (8 - b))
    # a short all-ones prefix keeps the exact integer sum below 2048, so binary16 holds it exactly
    ncols = max(1, 2048 // (1 << b) // 2)
    x = np.zeros((1, K), dtype=np.float16)
    x[0, :ncols] = 1.0
    y = run_gemv(pm, b, x)
    assert np.array_equal(y[0].astype(np.int64), (idx[:, :ncols].astype(np.int64) >> (8 - b)).sum(axis=1))
    pm.close()


# kernel families for the adversarial inputs: the dispatcher's own choice, the one-row-per-lane
# matrix-core kernel for every b, the matrix-core kernel with in-wave exchange, the matrix-core kernel
# on tiles of 16 rows (one and two tiles per workgroup); the matrix-core kernels need K % 128 == 0
# (K % 256 == 0 on tiles) and batch >= 3 / >= 2, which the shapes below satisfy
FAMILIES = [dict(), dict(mfma_min_batch=-3), dict(variant=3), dict(variant=9), dict(variant=10)]


@pytest.mark.parametrize("family", range(len(FAMILIES)))
@pytest.mark.parametrize("batch", [1, 3, 5, 8])
@pytest.mark.parametrize("b", ALL_BITS)
def test_adversarial_tables(B, b, batch, family):
    M, K = 48, 2048 + 256
    assert K % 256 == 0                                   # so that the matrix-core kernels are reachable
    idx, luts, x = inputs.make_case(16, M, K, batch=batch)
    rng = np.random.default_rng(b)
    E = 1 << b
    lut = luts[b].copy()
    lut = lut[:, rng.permutation(E)]                      # unsorted
    lut[0, :] = np.float16(6.0e-8)                        # subnormals
    lut[1, ::2] = np.float16(-0.0)
    lut[2, :] = np.float16(0.25)                          # all entries equal
    lut[3, 0] = np.float16(65504.0)
    lut[3, E - 1] = np.float16(-65504.0)
    idx[5, :] = 0xA5                                      # a row whose indices are all equal
    xs = (x.astype(np.float32) * 1e-3).astype(np.float16) # keeps 65504 * x finite
    pm = B.ap_pack(idx, {b: lut}).set_options(**FAMILIES[family])
    for xv in (xs, np.zeros_like(x)):
        y = run_gemv(pm, b, xv)
        check_against_oracle(y, idx, lut, b, xv)
    pm.close()


@pytest.mark.parametrize("family", range(len(FAMILIES)))
@pytest.mark.parametrize("batch", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("b", ALL_BITS)
def test_subnormal_centroids_are_not_flushed(B, b, batch, family):
    # every centroid is a binary16 subnormal (k * 2^-24), activations are large: a path that
    # flushed subnormal inputs to zero (the matrix instructions included) would return 0 where the
    # result is of order 10
    M, K = 20, 2048 + 256
    assert K % 256 == 0
    rng = np.random.default_rng(100 + b)
    idx = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    lut = (rng.integers(1, 1024, size=(M, 1 << b)).astype(np.uint16)).view(np.float16)
    x = np.full((batch, K), 512.0, dtype=np.float16)
    x[:, ::3] = -256.0
    pm = B.ap_pack(idx, {b: lut}).set_options(**FAMILIES[family])
    y = run_gemv(pm, b, x)
    assert np.all(np.abs(y.astype(np.float64)) > 0.05)
    check_against_oracle(y, idx, lut, b, x)
    pm.close()


@pytest.mark.parametrize("rg", [2, 3, 4])
@pytest.mark.parametrize("batch", [1, 2, 5, 8])
def test_several_row_groups_per_workgroup(B, rg, batch):
    # the variant that keeps activations in registers across row groups, forced on small ragged
    # shapes: rows not a multiple of 4*rg, a ragged last span, 1..4 waves per group
    for (M, K) in [(4 * rg * 3 + 5, 2048 + 160), (7, 96), (4 * rg + 1, 3 * 2048 + 32 * 17)]:
        idx, luts, x = inputs.make_case(18, M, K, batch=batch, sigma=0.01)
        pm = B.ap_pack(idx, luts).set_options(row_groups=rg)
        for b in ALL_BITS:
            y = run_gemv(pm, b, x)
            check_against_oracle(y, idx, luts[b], b, x)
        pm.close()


@pytest.mark.parametrize("batch", [3, 4, 5, 8])
def test_matrix_core_variant_for_every_bit_width(B, batch):
    # forced for every b (the dispatcher uses it for b >= 6 only): several spans, a ragged last span
    # of 4-chunk blocks, rows not a multiple of 4 or 16, one and four row groups per workgroup
    for rg in (1, 4):
        for (M, K) in [(37, 128), (70, 2048 + 640), (21, 3 * 2048 + 128)]:
            idx, luts, x = inputs.make_case(19, M, K, batch=batch, sigma=0.01)
            pm = B.ap_pack(idx, luts).set_options(mfma_min_batch=-3, row_groups=rg)
            for b in ALL_BITS:
                y = run_gemv(pm, b, x)
                check_against_oracle(y, idx, luts[b], b, x)
            pm.close()


@pytest.mark.parametrize("batch", [2, 3, 4, 5, 7, 8])
def test_matrix_core_variant_with_in_block_exchange(B, batch):
    # forced for every b and batch >= 2: one span, several spans with a ragged last span of 4-chunk
    # blocks, more spans than waves (a wave takes two spans), rows not a multiple of 4
    # one, two and four row groups per workgroup (the last two reuse the activations of a span)
    for rg in (1, 2, 4):
        for (M, K) in [(37, 128), (70, 2048 + 640), (21, 3 * 2048 + 128), (9, 9 * 2048 + 256)]:
            idx, luts, x = inputs.make_case(21, M, K, batch=batch, sigma=0.01)
            pm = B.ap_pack(idx, luts).set_options(variant=B.VARIANT_EXCHANGE, row_groups=rg)
            for b in ALL_BITS:
                y = run_gemv(pm, b, x)
                check_against_oracle(y, idx, luts[b], b, x)
            pm.close()


@pytest.mark.parametrize("batch", [2, 3, 4, 5, 6, 7, 8])
def test_matrix_core_variant_on_tiles_of_16_rows(B, batch):
    # forced for every b and batch >= 2: one octet of chunks, several spans with a ragged last span, an
    # odd number of octets, more octet pairs than waves, rows not a multiple of 4 or 16 (tiles and row
    # groups partly or wholly past the matrix), one and two tiles per workgroup; workgroups of 1, 2, 3, 4 and 8
    # waves (the pair tables of the 3- and 4-bit paths are built by a different loop at 4 and 8 waves)
    for variant in (B.VARIANT_TILE, B.VARIANT_TILE2):
        for (M, K) in [(37, 256), (70, 2048 + 768), (21, 3 * 2048 + 256), (9, 9 * 2048 + 512), (130, 4096), (16, 512),
                       (20, 768), (40, 1280)]:
            idx, luts, x = inputs.make_case(27, M, K, batch=batch, sigma=0.01)
            pm = B.ap_pack(idx, luts).set_options(variant=variant)
            for b in ALL_BITS:
                y = run_gemv(pm, b, x)
                check_against_oracle(y, idx, luts[b], b, x)
            pm.close()


@pytest.mark.parametrize("b", [7, 8])
def test_bank_per_lane_variant(B, b):
    # forced (the dispatcher does not choose it): one lane per LDS bank column, 8 copies of a table,
    # a lane owns one row of 4 chunks: ragged spans whose last quad is partly filled, rows not a
    # multiple of 4, 1..8 waves per group (1, 2, 4, 8 or 16 table pieces per thread), unsorted tables
    rng = np.random.default_rng(40 + b)
    for (M, K) in RAGGED + [(512, 512), (33, 8 * 2048), (6, 14 * 2048)]:
        idx, luts, x = inputs.make_case(24, M, K, bit_widths=[b])
        lut = luts[b][:, rng.permutation(1 << b)].copy()
        pm = B.ap_pack(idx, {b: lut}).set_options(variant=B.VARIANT_BANK_PER_LANE)
        y = run_gemv(pm, b, x)
        check_against_oracle(y, idx, lut, b, x)
        pm.close()


@pytest.mark.parametrize("b", ALL_BITS)
def test_two_row_groups_per_workgroup_variant(B, b):
    # forced (the dispatcher uses it on large matrices only): 2..8 spans, a ragged last span, an odd
    # number of row groups (the last workgroup holds one group), rows not a multiple of 4; the outputs
    # are bit-identical to the kernel with one group per workgroup, except where that kernel runs a ragged
    # last span of at most 32 chunks on both halves of the wave (b = 4, 5, 6), which this variant does not
    for (M, K) in [(70, 2048 + 160), (129, 4096 + 32), (66, 3 * 2048), (10, 5 * 2048 + 736), (4, 8 * 2048), (37, 2048 + 32)]:
        idx, luts, x = inputs.make_case(26, M, K, bit_widths=[b])
        pm = B.ap_pack(idx, luts).set_options(variant=B.VARIANT_PAIR)
        y = run_gemv(pm, b, x)
        check_against_oracle(y, idx, luts[b], b, x)
        pm.set_options(variant=B.VARIANT_NO_PAIR)
        y1 = run_gemv(pm, b, x)
        check_against_oracle(y1, idx, luts[b], b, x)
        ragged = (K // 32) % 64
        if not (b in (4, 5, 6) and 0 < ragged <= 32):
            assert np.array_equal(y.view(np.uint16), y1.view(np.uint16))
        pm.close()


@pytest.mark.parametrize("batch", [1, 2, 8])
def test_fused_launch_equals_separate_calls(B, batch):
    import torch
    K = 2048 + 256
    mats = []
    for k, M in enumerate([64, 37, 130, 8]):
        idx, luts, x = inputs.make_case(20, M, K, batch=batch, salt=k)
        mats.append((idx, luts, x, B.ap_pack(idx, luts)))
    shared_x = torch.from_numpy(mats[0][2]).cuda()
    for b in ALL_BITS:
        for count in (1, 3, 4):
            triples, ys = [], []
            for (idx, luts, x, pm) in mats[:count]:
                y = torch.full((batch, pm.M), -3.0, dtype=torch.float16, device="cuda")
                triples.append((pm, shared_x, y))
            B.ap_gemv_multi(triples, b)
            torch.cuda.synchronize()
            for (idx, luts, x, pm), (_, _, y) in zip(mats[:count], triples):
                sep = B.ap_gemv(pm, b, shared_x)
                torch.cuda.synchronize()
                if batch <= 2:   # same kernel as the single call: bit-identical
                    assert np.array_equal(y.cpu().numpy().view(np.uint16), sep.cpu().numpy().view(np.uint16))
                check_against_oracle(y.cpu().numpy(), idx, luts[b], b, mats[0][2])
    # row lengths must agree at batch >= 2; at batch 1 any shapes share the launch
    idx, luts, x = inputs.make_case(20, 16, 512, batch=batch)
    other = B.ap_pack(idx, luts)
    y0 = torch.empty((batch, 64), dtype=torch.float16, device="cuda")
    y1 = torch.full((batch, 16), -3.0, dtype=torch.float16, device="cuda")
    x1 = torch.from_numpy(x).cuda()
    if batch == 1:
        B.ap_gemv_multi([(mats[0][3], shared_x, y0), (other, x1, y1)], 4)
        torch.cuda.synchronize()
        check_against_oracle(y1.cpu().numpy(), idx, luts[4], 4, x)
        check_against_oracle(y0.cpu().numpy(), mats[0][0], mats[0][1][4], 4, mats[0][2])
    else:
        with pytest.raises(B.ApError) as e:
            B.ap_gemv_multi([(mats[0][3], shared_x, y0), (other, x1, y1)], 4)
        assert e.value.status == 2
    for m in mats:
        m[3].close()
    other.close()


@pytest.mark.parametrize("batch", [2, 3, 5, 8])
def test_fused_launch_on_the_tile_kernel(B, batch):
    # forced through the first handle (the library chooses it from 1024 row groups per launch on): rows not
    # a multiple of 16, a matrix smaller than a tile, a ragged last span, canaries around every output
    import torch
    K = 2048 + 768
    mats = []
    for k, M in enumerate([70, 37, 130, 8, 16]):
        idx, luts, x = inputs.make_case(31, M, K, batch=batch, salt=k)
        mats.append((idx, luts, x, B.ap_pack(idx, luts)))
    mats[0][3].set_options(variant=B.VARIANT_TILE)
    shared_x = torch.from_numpy(mats[0][2]).cuda()
    guard = 32
    for b in ALL_BITS:
        for count in (1, 3, 5):
            triples, bufs = [], []
            for (idx, luts, x, pm) in mats[:count]:
                buf = torch.full((guard + batch * pm.M + guard,), -3.0, dtype=torch.float16, device="cuda")
                bufs.append(buf)
                triples.append((pm, shared_x, buf[guard:guard + batch * pm.M].view(batch, pm.M)))
            B.ap_gemv_multi(triples, b)
            torch.cuda.synchronize()
            for (idx, luts, x, pm), buf in zip(mats[:count], bufs):
                out = buf.cpu().numpy()
                assert np.all(out[:guard] == -3.0) and np.all(out[-guard:] == -3.0)
                check_against_oracle(out[guard:-guard].reshape(batch, pm.M), idx, luts[b], b, mats[0][2])
                # the same arithmetic as a single call on the tile kernel: bit-identical
                pm.set_options(variant=B.VARIANT_TILE)
                sep = B.ap_gemv(pm, b, shared_x)
                torch.cuda.synchronize()
                assert np.array_equal(out[guard:-guard].reshape(batch, pm.M).view(np.uint16), sep.cpu().numpy().view(np.uint16))
    for m in mats:
        m[3].close()


@pytest.mark.parametrize("batch", [2, 5, 8])
def test_batched_work_list(B, batch):
    # items of several shapes and bit-widths: groups large enough for the tile kernel (same b, rows of one
    # class of length, >= 1024 row groups together) share a launch, the others run as single calls;
    # canaries around every output; a tile-kernel item is bit-identical to the single call on that kernel
    import ctypes
    import torch
    shapes = [(2100, 2048), (2050, 2304), (37, 256), (70, 2048 + 96), (2060, 12288), (2100, 12288 + 256), (16, 12544)]
    mats = []
    for k, (M, K) in enumerate(shapes):
        idx, luts, x = inputs.make_case(33, M, K, batch=batch, salt=k, bit_widths=[3, 4, 8], sigma=0.01)
        mats.append((idx, luts, x, B.ap_pack(idx, luts), torch.from_numpy(x).cuda()))
    guard = 32
    quads, bufs, meta = [], [], []
    for rep, bsel in enumerate([(3, 3, 4, 3, 4, 4, 4), (8, 8, 4, 8, 4, 4, 3)]):
        for (idx, luts, x, pm, xd), b in zip(mats, bsel):
            buf = torch.full((guard + batch * pm.M + guard,), -5.0, dtype=torch.float16, device="cuda")
            bufs.append(buf)
            quads.append((pm, b, xd, buf[guard:guard + batch * pm.M].view(batch, pm.M)))
            meta.append((idx, luts, x, pm, xd, b))
    B.ap_gemv_list_batch(quads, batch)
    torch.cuda.synchronize()
    for (idx, luts, x, pm, xd, b), buf in zip(meta, bufs):
        out = buf.cpu().numpy()
        assert np.all(out[:guard] == -5.0) and np.all(out[-guard:] == -5.0)
        y = out[guard:-guard].reshape(batch, pm.M)
        check_against_oracle(y, idx, luts[b], b, x)
    if batch == 2:
        # batch 2: every item ran in a list launch of the kernel that single calls use, bit for bit
        for k, (idx, luts, x, pm, xd, b) in enumerate(meta):
            sep = B.ap_gemv(pm, b, xd)
            torch.cuda.synchronize()
            assert np.array_equal(bufs[k].cpu().numpy()[guard:-guard].reshape(batch, pm.M).view(np.uint16),
                                  sep.cpu().numpy().view(np.uint16))
    else:
        # the first two items of the first half (b = 3, 2048 and 2304 columns: 1038 row groups together) ran on
        # the tile kernel with 4 waves per tile, like a single call on it
        for k in (0, 1):
            idx, luts, x, pm, xd, b = meta[k]
            pm.set_options(variant=B.VARIANT_TILE)
            sep = B.ap_gemv(pm, b, xd)
            torch.cuda.synchronize()
            assert np.array_equal(bufs[k].cpu().numpy()[guard:-guard].reshape(batch, pm.M).view(np.uint16),
                                  sep.cpu().numpy().view(np.uint16))
            pm.set_options(variant=B.VARIANT_AUTO)
    # argument checks: status of the first bad item, nothing enqueued; batch range
    bad = list(quads)
    bad[3] = (quads[3][0], 5, quads[3][2], quads[3][3])       # no table for b = 5
    with pytest.raises(B.ApError) as e:
        B.ap_gemv_list_batch(bad, batch)
    assert e.value.status == 3
    with pytest.raises(B.ApError) as e:
        B.ap_gemv_list_batch(quads, 9)
    assert e.value.status == 6
    for m in mats:
        m[3].close()


def test_work_list_mixed_shapes_and_bit_widths(B):
    # one launch per 32 items: 40 items of 7 different shapes (1..9 spans, ragged spans, rows not a
    # multiple of 4), each with its own bit-width; every output bit-identical to a separate ap_gemv
    # call and within tolerance of the oracle; canaries between the outputs stay untouched
    import torch
    shapes = [(37, 96), (64, 2048 + 160), (130, 4096 + 32), (8, 512), (21, 3 * 2048), (5, 9 * 2048 + 32), (257, 1024)]
    mats = []
    for k, (M, K) in enumerate(shapes):
        idx, luts, x = inputs.make_case(25, M, K, salt=k)
        mats.append((idx, luts, x, B.ap_pack(idx, luts), torch.from_numpy(x).cuda()))
    rng = np.random.default_rng(25)
    picks = [(int(rng.integers(0, len(shapes))), int(rng.integers(3, 9))) for _ in range(40)]
    guard = 16
    total = sum(mats[m][3].M + guard for m, _ in picks) + guard
    ybuf = torch.full((total,), -7.0, dtype=torch.float16, device="cuda")
    quads, offs, off = [], [], guard
    for m, b in picks:
        M = mats[m][3].M
        quads.append((mats[m][3], b, mats[m][4], ybuf[off:off + M]))
        offs.append(off)
        off += M + guard
    B.ap_gemv_list(quads)
    torch.cuda.synchronize()
    out = ybuf.cpu().numpy()
    mask = np.ones(total, dtype=bool)
    for (m, b), o in zip(picks, offs):
        idx, luts, x, pm, xd = mats[m]
        y = out[o:o + pm.M].reshape(1, -1)
        mask[o:o + pm.M] = False
        sep = B.ap_gemv(pm, b, xd)
        torch.cuda.synchronize()
        assert np.array_equal(y.view(np.uint16), sep.cpu().numpy().view(np.uint16)), (m, b)
        check_against_oracle(y, idx, luts[b], b, x)
    assert np.all(out[mask] == -7.0)
    # a bad item anywhere in the list: its status, and nothing is enqueued
    ybuf.fill_(-7.0)
    bad = list(quads)
    pm3 = B.ap_pack(mats[0][0], {3: mats[0][1][3]})
    bad[35] = (pm3, 5, mats[0][4], ybuf[offs[35]:offs[35] + pm3.M])          # no table for b = 5
    with pytest.raises(B.ApError) as e:
        B.ap_gemv_list(bad)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert np.all(ybuf.cpu().numpy() == -7.0)
    assert B.lib.ap_gemv_list(None, 1, None) == 1
    assert B.lib.ap_gemv_list(B.make_list(quads), 0, None) == 1
    pm3.close()
    for m in mats:
        m[3].close()


def test_graph_capture_and_replay_match_eager(B, tiny):
    # ap_gemv and ap_gemv_multi allocate nothing and synchronise nothing, so a stream capture can
    # record them; every replay (with eager work and synchronisations in between) must reproduce
    # the eager result bit for bit
    import torch
    idx, luts, x, pm = tiny
    xd = torch.from_numpy(x).cuda()
    eager = {b: B.ap_gemv(pm, b, xd).clone() for b in ALL_BITS}
    torch.cuda.synchronize()
    ys = {b: torch.zeros((1, pm.M), dtype=torch.float16, device="cuda") for b in ALL_BITS}
    ym = torch.zeros((1, pm.M), dtype=torch.float16, device="cuda")
    cap = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(cap):
        for b in ALL_BITS:                       # warm-up on the capture stream
            B.ap_gemv(pm, b, xd, y=ys[b], stream=cap)
        cap.synchronize()
        with torch.cuda.graph(g, stream=cap):
            for b in ALL_BITS:
                B.ap_gemv(pm, b, xd, y=ys[b], stream=cap)
            B.ap_gemv_multi([(pm, xd, ym)], 5, stream=cap)
    torch.cuda.synchronize()
    for rep in range(4):
        for b in ALL_BITS:
            ys[b].zero_()
        ym.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for b in ALL_BITS:
            assert torch.equal(ys[b], eager[b]), (rep, b)
        assert torch.equal(ym, eager[5])
        # eager work between replays
        assert torch.equal(B.ap_gemv(pm, 4 + rep % 3, xd), eager[4 + rep % 3])
        torch.cuda.synchronize()


def test_dispatch_sequence_without_repacking_and_determinism(B, tiny):
    import torch
    idx, luts, x, pm = tiny
    before = pm.buf.clone()
    fresh = {b: run_gemv(pm, b, x) for b in ALL_BITS}
    rng = np.random.default_rng(4)
    for b in rng.integers(3, 9, size=24).tolist():
        y = run_gemv(pm, b, x)
        assert np.array_equal(y.view(np.uint16), fresh[b].view(np.uint16))   # bit-identical repeats
    assert torch.equal(before, pm.buf)                                         # blob untouched


def test_output_canaries_and_sparse_support(B):
    import torch
    M, K = 100, 2048 + 64
    idx, luts, x = inputs.make_case(17, M, K, batch=3)
    pm = B.ap_pack(idx, {3: luts[3], 4: luts[4], 8: luts[8]})
    guard = 64
    ybuf = torch.full((guard + 3 * M + guard,), -7.0, dtype=torch.float16, device="cuda")
    xd = torch.from_numpy(x).cuda()
    sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for b in (3, 4, 8):
        st = B.lib.ap_gemv(pm.handle, b, xd.data_ptr(), ybuf.data_ptr() + 2 * guard, 3, sp)
        assert st == 0
        torch.cuda.synchronize()
        out = ybuf.cpu().numpy()
        assert np.all(out[:guard] == -7.0) and np.all(out[-guard:] == -7.0)
        check_against_oracle(out[guard:-guard].reshape(3, M), idx, luts[b], b, x)
    for b in (5, 6, 7, 2, 9):
        assert B.lib.ap_gemv(pm.handle, b, xd.data_ptr(), ybuf.data_ptr(), 3, sp) == 3
    assert B.lib.ap_gemv(pm.handle, 3, xd.data_ptr(), ybuf.data_ptr(), 0, sp) == 6
    assert B.lib.ap_gemv(pm.handle, 3, xd.data_ptr(), ybuf.data_ptr(), 17, sp) == 6
    assert B.lib.ap_gemv(pm.handle, 3, xd.data_ptr() + 2, ybuf.data_ptr(), 1, sp) == 1
    pm.close()


def test_option_values_are_checked(B, tiny):
    _, _, _, pm = tiny
    L = B.lib
    for opt, bad in ((0, 9), (0, -1), (1, 0), (1, 5), (2, 10), (3, 2), (3, 6), (3, 11), (9, 0)):
        assert L.ap_set_option(pm.handle, opt, bad) == 1, (opt, bad)
    for opt, good, default in ((0, 2, 0), (1, 1, -1), (2, 9, 0), (3, 1, 0)):
        assert L.ap_set_option(pm.handle, opt, good) == 0
        assert L.ap_set_option(pm.handle, opt, default) == 0


def test_smaller_parent_bit_width(B):
    n, M, K = 6, 40, 2048 + 32
    rng = np.random.default_rng(6)
    idx = rng.integers(0, 1 << n, size=(M, K), dtype=np.uint8)
    luts = {b: rng.normal(0, 0.02, size=(M, 1 << b)).astype(np.float16) for b in range(3, n + 1)}
    x = rng.normal(0, 1, size=(2, K)).astype(np.float16)
    pm = B.ap_pack(idx, luts, n=n)
    for b in range(3, n + 1):
        y = run_gemv(pm, b, x)
        check_against_oracle(y, idx, luts[b], b, x, n=n)
    pm.close()


def test_attach_to_a_device_copy(B, tiny):
    idx, luts, x, pm = tiny
    pm2 = pm.clone()
    assert pm2.buf.data_ptr() != pm.buf.data_ptr()
    for b in (3, 8):
        assert np.array_equal(run_gemv(pm2, b, x).view(np.uint16), run_gemv(pm, b, x).view(np.uint16))
    pm2.close()


@pytest.mark.parametrize("batch", [1, 4])
def test_quantised_model_end_to_end(B, batch):
    # weights -> incremental upscaling (host) -> pack -> GEMV at every bit-width; the oracle takes
    # the same indices and tables, and the b-bit result must approach the dense product as b grows
    rng = np.random.default_rng([20240210, 31, batch])
    M, K = 96, 2048 + 320
    W = rng.standard_t(5, (M, K)).astype(np.float32) * 0.02
    S = (rng.gamma(0.5, 1.0, (M, K)) + 1e-6).astype(np.float32)
    idx, luts = B.ap_quantize(W, S, 3, 8, 15)
    x = rng.normal(0, 1, (batch, K)).astype(np.float16)
    pm = B.ap_pack(idx, luts)
    dense = x.astype(np.float64) @ W.astype(np.float64).T
    errs = []
    for b in ALL_BITS:
        y = run_gemv(pm, b, x)
        check_against_oracle(y, idx, luts[b], b, x)
        errs.append(float(np.sqrt(np.mean((y.astype(np.float64) - dense) ** 2))))
    assert errs[-1] < errs[0] / 8 and errs[3] < errs[0]
    pm.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_bit_widths_and_batches(B, seed):
    # a seeded sweep over shapes the fixed cases do not name: any M, any K % 32 == 0 up to ~5 spans,
    # random supported sets of bit-widths, every batch size; default dispatch
    rng = np.random.default_rng([20240210, 99, seed])
    for _ in range(8):
        M = int(rng.integers(1, 300))
        K = 32 * int(rng.integers(1, 330))
        batch = int(rng.integers(1, 9))
        bits = sorted(set(int(v) for v in rng.integers(3, 9, size=3)))
        idx, luts, x = inputs.make_case(30 + seed, M, K, batch=batch, sigma=0.02, bit_widths=bits)
        pm = B.ap_pack(idx, luts)
        for b in bits:
            y = run_gemv(pm, b, x)
            check_against_oracle(y, idx, luts[b], b, x)
        assert np.array_equal(B.ap_unpack(pm), idx)
        pm.close()


def test_issue_probe_runs_every_kind(B):
    """The measurement aid launches and completes for every kind (it has no output to compare)."""
    import torch
    for kind in range(7):
        assert B.lib.ap_probe_issue(kind, 3, None) == 0
    torch.cuda.synchronize()

