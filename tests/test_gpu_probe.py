"""The register-only MFMA rate probe (a measurement aid of the benchmark): its sink must hold what the loop's
contractions add up to, so that the rate it reports is the rate of real matrix work."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def A():
    import paper_2603_24840_amd as pkg
    pkg.lib()
    return pkg


@pytest.mark.parametrize("shape", [16, 32])
def test_probe_on_ones_counts_every_product(A, shape):
    ones = torch.ones(512, dtype=torch.bfloat16, device=DEV)
    iters, n_wg = 3, 5
    sink, flop = A.arrol_probe_mfma_rate(ones, ones, shape=shape, n_workgroups=n_wg, iters=iters)
    torch.cuda.synchronize()
    # every accumulator element receives K = 32 unit products per iteration; a lane holds 128 elements
    assert torch.all(sink == 128.0 * 32.0 * iters)
    assert flop == 2.0 * 16 * 16 * 32 * 32 * iters * 8 * n_wg
    # all products counted: flop / 2 multiply-adds in the whole launch
    assert float(sink.double().sum()) == flop / 2


@pytest.mark.parametrize("shape", [16, 32])
def test_probe_contracts_the_fragments_it_was_given(A, shape):
    """Small integers make fp32 exact.  Summed over a wavefront, the accumulators of block (i, j) hold
    sum_k colsum(A_i)[k] * colsum(B_j)[k], whatever lane holds which row: only the K index of a lane's
    eight values matters (16x16x32: 8 * (lane / 16) + e; 32x32x16: 8 * (lane / 32) + e)."""
    g = torch.Generator().manual_seed(91)
    n_wg, iters = 3, 2
    n_frag_a, n_frag_b = 50, 7     # neither a multiple of the 8 resp. 4 fragments per wavefront: exercises the wrap
    a = torch.randint(-2, 3, (n_frag_a, 64, 8), generator=g).to(torch.bfloat16)
    b = torch.randint(-2, 3, (n_frag_b, 64, 8), generator=g).to(torch.bfloat16)
    sink, _ = A.arrol_probe_mfma_rate(a.to(DEV).reshape(-1), b.to(DEV).reshape(-1), shape=shape, n_workgroups=n_wg,
                                      iters=iters)
    torch.cuda.synchronize()
    got = sink.cpu().double().reshape(n_wg * 8, 64).sum(dim=1).numpy()
    an, bn = a.double().numpy(), b.double().numpy()
    lanes_per_k = 16 if shape == 16 else 32

    def colsum(frag):               # [64, 8] -> per K index, summed over the rows
        return frag.reshape(64 // lanes_per_k, lanes_per_k, 8).sum(axis=1).reshape(-1)

    for w in range(n_wg * 8):
        fa = [colsum(an[(w * 8 + f) % n_frag_a]) for f in range(8)]
        fb = [colsum(bn[(w * 4 + f) % n_frag_b]) for f in range(4)]
        if shape == 16:             # 8 x 4 blocks, each A fragment against each B fragment
            want = sum(float(np.dot(fa[i], fb[j])) for i in range(8) for j in range(4))
        else:                       # 4 x 2 blocks of 32 x 32, two K halves: fragments (i, half) and (j, half)
            want = sum(float(np.dot(fa[i + 4 * h], fb[j + 2 * h])) for i in range(4) for j in range(2) for h in range(2))
        assert got[w] == iters * want, (w, got[w], iters * want)


def test_probe_zero_iterations_and_zero_operands(A):
    z = torch.zeros(1024, dtype=torch.bfloat16, device=DEV)
    r = torch.randn(1024, device=DEV).to(torch.bfloat16)
    sink, flop = A.arrol_probe_mfma_rate(r, r, iters=0, n_workgroups=2)
    assert flop == 0.0 and torch.all(sink == 0)
    sink, _ = A.arrol_probe_mfma_rate(z, r, iters=4, n_workgroups=2)
    assert torch.all(sink == 0)
