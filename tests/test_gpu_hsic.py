"""Parity of the HSIC sensitivity (aq_rbf_gram / aq_hsic_sensitivity, through the C ABI) against the fp64 oracle on
the same seeded inputs.  Bars: kernel-matrix entries within 2e-5 absolute (fp32 products and the r_i + r_j - 2 a.b form
of the squared distance: errors of 1e-6 * d in the exponent's argument times gamma); HSIC values within 1e-4
relative (plus 1e-9 absolute for the near-zero ones), Eq. 5's combination within 1e-4 of the larger of its terms."""
import numpy as np
import pytest

import aq_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2605_24011_amd as aq
    assert torch.cuda.is_available(), "these tests need the GPU"
    aq.lib()
    return torch, aq


@pytest.fixture(scope="module")
def ho():
    from oracle import aq_hsic_oracle
    return aq_hsic_oracle


@pytest.mark.parametrize("K,d", [(2, 1), (33, 7), (128, 16), (130, 40), (300, 129), (257, 1000)])
def test_rbf_gram_matches_oracle(gpu, ho, K, d):
    torch, aq = gpu
    X, _, _ = wl.draw_hsic_inputs(K, d, 4, 2, 91, K, d)
    gamma = ho.median_gamma(X) if K > 2 else 0.5
    G = aq.aq_rbf_gram(torch.from_numpy(X).cuda(), gamma).cpu().numpy().astype(np.float64)
    want = ho.rbf_gram(X, gamma)
    assert np.abs(G - want).max() <= 2e-5
    assert np.array_equal(np.diag(G), np.ones(K))


@pytest.mark.parametrize("K,d,offset", [(130, 40, 20.0), (257, 1000, 20.0), (300, 129, -300.0)])
def test_rbf_gram_with_a_common_offset_on_every_feature(gpu, ho, K, d, offset):
    """Activations share a mean offset; the kernel depends on differences only.  r_i + r_j - 2 a_i.a_j on the raw
    samples would lose about eps * d * offset^2 of the squared distance (1000 features at +20: 0.05 absolute, against
    distances of order d); relative to sample 0 the offset is gone before anything is squared."""
    torch, aq = gpu
    X, _, _ = wl.draw_hsic_inputs(K, d, 4, 2, 95, K, d)
    gamma = ho.median_gamma(X)
    Xo = (X + np.float32(offset)).astype(np.float32)
    G = aq.aq_rbf_gram(torch.from_numpy(Xo).cuda(), gamma).cpu().numpy().astype(np.float64)
    want = ho.rbf_gram(Xo.astype(np.float64), gamma)          # the oracle on the very floats the GPU was given
    assert np.abs(G - want).max() <= 2e-5
    assert np.array_equal(np.diag(G), np.ones(K))


def test_sensitivity_with_offsets(gpu, ho):
    torch, aq = gpu
    K = 200
    X, Z, Y = wl.draw_hsic_inputs(K, 96, 64, 7, 96, K)
    gx, gz, gy = ho.median_gamma(X), ho.median_gamma(Z), ho.median_gamma(Y)
    Xo, Zo = (X + np.float32(20.0)).astype(np.float32), (Z - np.float32(35.0)).astype(np.float32)
    out = aq.aq_hsic_sensitivity(torch.from_numpy(Xo).cuda(), gx, torch.from_numpy(Zo).cuda(), gz,
                                 torch.from_numpy(Y).cuda(), gy, 0.5, 3.0).cpu().numpy()
    h_xz, h_zy = ho.hsic(Xo.astype(np.float64), gx, Zo.astype(np.float64), gz), ho.hsic(Zo.astype(np.float64), gz, Y, gy)
    assert abs(out[0] - h_xz) <= 1e-4 * abs(h_xz) + 1e-9
    assert abs(out[1] - h_zy) <= 1e-4 * abs(h_zy) + 1e-9


@pytest.mark.parametrize("K,dx,dz,dy", [(2, 1, 1, 1), (64, 32, 48, 7), (200, 96, 64, 7), (513, 300, 260, 14),
                                        (1500, 160, 224, 7),       # 12 x 12 tiles, fp64 reductions over many workgroups
                                        (4096, 64, 48, 7)])        # the bench's sample count (528 tiles), few features
def test_sensitivity_matches_oracle(gpu, ho, K, dx, dz, dy):
    torch, aq = gpu
    X, Z, Y = wl.draw_hsic_inputs(K, dx, dz, dy, 92, K)
    if K > 2:
        gx, gz, gy = ho.median_gamma(X), ho.median_gamma(Z), ho.median_gamma(Y)
    else:
        gx = gz = gy = 0.7
    alpha, beta = 0.5, 3.0
    out = aq.aq_hsic_sensitivity(torch.from_numpy(X).cuda(), gx, torch.from_numpy(Z).cuda(), gz,
                                 torch.from_numpy(Y).cuda(), gy, alpha, beta).cpu().numpy()
    h_xz, h_zy = ho.hsic(X, gx, Z, gz), ho.hsic(Z, gz, Y, gy)
    assert abs(out[0] - h_xz) <= 1e-4 * abs(h_xz) + 1e-9
    assert abs(out[1] - h_zy) <= 1e-4 * abs(h_zy) + 1e-9
    s = ho.sensitivity(X, gx, Z, gz, Y, gy, alpha, beta)
    assert abs(out[2] - s) <= 1e-4 * max(alpha * abs(h_xz), beta * abs(h_zy)) + 1e-9


def test_strided_inputs_and_independent_variables(gpu, ho):
    torch, aq = gpu
    K = 150
    X, Z, Y = wl.draw_hsic_inputs(K, 40, 24, 7, 93)
    _, Z2, _ = wl.draw_hsic_inputs(K, 40, 24, 7, 94)            # independent of X
    gx, gz, gy = ho.median_gamma(X), ho.median_gamma(Z2), ho.median_gamma(Y)
    Xp = torch.zeros((K, 64), device="cuda"); Xp[:, :40] = torch.from_numpy(X).cuda()       # row stride 64
    out = aq.aq_hsic_sensitivity(Xp[:, :40], gx, torch.from_numpy(Z2).cuda(), gz, torch.from_numpy(Y).cuda(), gy,
                                 1.0, 1.0).cpu().numpy()
    h = ho.hsic(X, gx, Z2, gz)
    assert abs(out[0] - h) <= 1e-4 * abs(h) + 1e-9
    dep = aq.aq_hsic_sensitivity(Xp[:, :40], gx, torch.from_numpy(Z).cuda(), ho.median_gamma(Z),
                                 torch.from_numpy(Y).cuda(), gy, 1.0, 1.0).cpu().numpy()
    assert dep[0] > 1.5 * out[0] > 0.0                     # dependence shows; the estimator has a bias of order 1/K


def test_errors(gpu):
    torch, aq = gpu
    X = torch.zeros((8, 4), device="cuda")
    with pytest.raises(aq.AqError) as e:
        aq.aq_rbf_gram(X, 0.0)
    assert e.value.status == aq.AQ_EINVAL
    with pytest.raises(aq.AqError) as e:
        aq.aq_hsic_sensitivity(X[:1], 1.0, X[:1], 1.0, X[:1], 1.0, 1.0, 1.0)
    assert e.value.status == aq.AQ_EINVAL
    with pytest.raises(aq.AqError) as e:
        aq.aq_hsic_sensitivity(X, 1.0, X, 1.0, X, 1.0, 1.0, 1.0, workspace=torch.zeros(64, dtype=torch.uint8, device="cuda"))
    assert e.value.status == aq.AQ_ESIZE


def test_rbf_gram_at_the_bench_size_sampled_entries(gpu, ho):
    """K = 4096 samples of 11008 features, the largest Gram matrix of the bench's sensitivity (528 tiles, more than
    the GPU holds at once): exactly symmetric (every tile writes its mirror image), ones on the diagonal, and
    entries sampled all over the matrix against the oracle's row routine."""
    torch, aq = gpu
    K, d = 4096, 11008
    g = torch.Generator(device="cuda"); g.manual_seed(93)
    A = torch.randn((K, d), dtype=torch.float32, device="cuda", generator=g)
    gamma = 1.0 / (2.0 * d)
    G = aq.aq_rbf_gram(A, gamma)
    assert torch.equal(G, G.t())
    assert bool((torch.diagonal(G) == 1.0).all())
    rng = np.random.default_rng(93)
    rows = np.concatenate([[0, 127, 128, K - 1], rng.integers(0, K, size=8)])
    Ah = A.cpu().numpy().astype(np.float64)
    Gh = G.cpu().numpy().astype(np.float64)
    for i in rows:
        diff = Ah - Ah[i]
        want = np.exp(-gamma * np.sum(diff * diff, axis=1))          # the oracle's definition, one row
        assert np.abs(Gh[i] - want).max() <= 2e-5
    # the same rows through the oracle's own routine on a subset it finishes quickly
    sub = np.sort(rng.choice(K, size=64, replace=False))
    assert np.abs(Gh[np.ix_(sub, sub)] - ho.rbf_gram(Ah[sub], gamma)).max() <= 2e-5
