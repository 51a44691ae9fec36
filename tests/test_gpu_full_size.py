"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times."""
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


@pytest.mark.parametrize("M,K", inputs.CONFIGS[2]["shapes"])
def test_config2_llama7b_shapes_every_row(B, M, K):
    idx, luts, x = inputs.make_case(2, M, K)
    pm = B.ap_pack(idx, luts)
    for b in ALL_BITS:
        y = run_gemv(pm, b, x)
        check_against_oracle(y, idx, luts[b], b, x)
    assert np.array_equal(B.ap_unpack(pm), idx)
    pm.close()


@pytest.mark.parametrize("M,K", inputs.CONFIGS[3]["shapes"])
def test_config3_llama13b_shapes_every_row(B, M, K):
    idx, luts, x = inputs.make_case(3, M, K)
    pm = B.ap_pack(idx, luts)
    for b in ALL_BITS:
        y = run_gemv(pm, b, x)
        check_against_oracle(y, idx, luts[b], b, x)
    pm.close()


@pytest.mark.parametrize("M,K", inputs.CONFIGS[2]["shapes"] + inputs.CONFIGS[3]["shapes"])
def test_config2_and_3_shapes_sampled_rows_at_batch_3_to_8(B, M, K):
    # the dispatcher's own choice at small batches: the tile kernel on the taller matrices, the ALU
    # kernels on the others
    idx, luts, x = inputs.make_case(3, M, K, batch=8)
    pm = B.ap_pack(idx, luts)
    rows = np.unique(np.concatenate([np.arange(0, 20), np.arange(M - 20, M),
                                     np.random.default_rng(M + K).integers(0, M, size=256)]))
    for b in ALL_BITS:
        for batch in (3, 4, 5, 8):
            y = run_gemv(pm, b, x[:batch])
            check_against_oracle(y, idx, luts[b], b, x[:batch], rows=rows)
    pm.close()


@pytest.mark.parametrize("batch", [4, 8])
def test_fused_projections_of_a_7b_layer_at_small_batch(B, batch):
    # q, k, v in one launch and gate, up in one launch, as the library chooses (the tile kernel)
    import torch
    rng = np.random.default_rng(5)
    for (M, K, n) in [(4096, 4096, 3), (11008, 4096, 2)]:
        mats = []
        for k in range(n):
            idx, luts, x = inputs.make_case(4, M, K, batch=batch, salt=k)
            mats.append((idx, luts, B.ap_pack(idx, luts)))
        xd = torch.from_numpy(x).cuda()
        rows = np.unique(np.concatenate([np.arange(0, 20), np.arange(M - 20, M), rng.integers(0, M, size=128)]))
        for b in (3, 5, 8):
            triples = [(pm, xd, torch.empty((batch, M), dtype=torch.float16, device="cuda")) for (_, _, pm) in mats]
            B.ap_gemv_multi(triples, b)
            torch.cuda.synchronize()
            for (idx, luts, pm), (_, _, y) in zip(mats, triples):
                check_against_oracle(y.cpu().numpy(), idx, luts[b], b, x, rows=rows)
        for m in mats:
            m[2].close()


def test_config4_one_layer_as_a_batched_work_list(B):
    # the seven matrices of a decoder layer at batch 8 in one call: the 4096-column ones share a launch of
    # the tile kernel, 4096x11008 runs on its own
    import torch
    batch, b = 8, 4
    rng = np.random.default_rng(9)
    mats, quads = [], []
    for k, (M, K) in enumerate(inputs.DECODE_LAYER_SHAPES):
        idx, luts, x = inputs.make_case(4, M, K, batch=batch, salt=k)
        pm = B.ap_pack(idx, luts)
        y = torch.empty((batch, M), dtype=torch.float16, device="cuda")
        mats.append((idx, luts, x, pm, y))
        quads.append((pm, b, torch.from_numpy(x).cuda(), y))
    B.ap_gemv_list_batch(quads, batch)
    torch.cuda.synchronize()
    for (idx, luts, x, pm, y) in mats:
        M = pm.M
        rows = np.unique(np.concatenate([np.arange(0, 20), np.arange(M - 20, M), rng.integers(0, M, size=128)]))
        check_against_oracle(y.cpu().numpy(), idx, luts[b], b, x, rows=rows)
        pm.close()


@pytest.mark.parametrize("M,K", inputs.CONFIGS[5]["shapes"])
def test_config5_llama70b_shapes_every_row_at_batch_1_sampled_rows_at_batch_2_to_8(B, M, K):
    idx, luts, x = inputs.make_case(5, M, K, batch=8, sigma=0.01)
    pm = B.ap_pack(idx, luts)
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(M - 4, M),
                                     np.random.default_rng(K).integers(0, M, size=256)]))
    for b in ALL_BITS:
        y = run_gemv(pm, b, x[:1])
        check_against_oracle(y, idx, luts[b], b, x[:1])
        for batch in range(2, 9):
            y = run_gemv(pm, b, x[:batch])
            check_against_oracle(y, idx, luts[b], b, x[:batch], rows=rows)
    pm.close()


def test_config4_decode_step_bit_width_sequence(B):
    """One decoder layer's seven matrices packed once; a seeded sequence of bit-widths is applied
    without repacking and every output is checked on sampled rows."""
    packed = []
    for k, (M, K) in enumerate(inputs.DECODE_LAYER_SHAPES):
        idx, luts, x = inputs.make_case(4, M, K, salt=k)
        packed.append((idx, luts, x, B.ap_pack(idx, luts)))
    seq = inputs.decode_bit_sequence(8)
    for step, b in enumerate(seq):
        for (idx, luts, x, pm) in packed:
            rows = np.random.default_rng(step).integers(0, idx.shape[0], size=64)
            y = run_gemv(pm, b, x)
            check_against_oracle(y, idx, luts[b], b, x, rows=rows)
    for p in packed:
        p[3].close()


def test_config4_one_layer_as_a_mixed_precision_work_list(B):
    """One decoder layer's seven matrices in ONE launch, each at its own bit-width: every row of every
    output against the oracle, and bit for bit against separate ap_gemv calls."""
    import torch
    packed = []
    for k, (M, K) in enumerate(inputs.DECODE_LAYER_SHAPES):
        idx, luts, x = inputs.make_case(4, M, K, salt=k)
        packed.append((idx, luts, x, B.ap_pack(idx, luts), torch.from_numpy(x).cuda()))
    for bits in ([3, 4, 5, 6, 7, 8, 3], [8, 8, 3, 3, 5, 4, 7]):
        quads = [(pm, b, xd, torch.full((1, pm.M), -3.0, dtype=torch.float16, device="cuda"))
                 for (idx, luts, x, pm, xd), b in zip(packed, bits)]
        B.ap_gemv_list(quads)
        torch.cuda.synchronize()
        for (idx, luts, x, pm, xd), (_, b, _, y) in zip(packed, quads):
            check_against_oracle(y.cpu().numpy(), idx, luts[b], b, x)
            sep = B.ap_gemv(pm, b, xd)
            torch.cuda.synchronize()
            assert torch.equal(sep, y)
    for p in packed:
        p[3].close()
