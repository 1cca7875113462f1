"""GPU parity of the EM codebook learner (Sec. 4.2 Algorithm 1, App. A.2) against the fp64 numpy oracle.

One iteration is a deterministic map phi -> phi*; the GPU runs it in fp32 (sums over N points, a Cholesky
solve of a 2Nc x 2Nc system), the oracle in fp64 with the paper's T matrix and a general solver.  Bar: after
one step from the same phi, max |phi_gpu - phi_ref| <= 2e-3 * max |phi_ref| (fp32 rounding amplified by the
conditioning of T^T S T; observed ~1e-5), and a few annealed iterations must lower the oracle's objective.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def em():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2506_18879_amd as cv
    cv.load_library()

    def step(data, phi, T, iters=1, decay=1.0):
        J, N, _ = data.shape
        Nc = phi.shape[1]
        d = torch.from_numpy(np.ascontiguousarray(data, np.float32)).cuda()
        p = torch.from_numpy(np.ascontiguousarray(phi, np.float32)).cuda()
        nb = cv.commvq_em_workspace_bytes(J, N, Nc)
        ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
        for _ in range(iters):
            cv.commvq_em_step(d, J, N, Nc, T, p, ws, nb)
            T *= decay
        torch.cuda.synchronize()
        return p.cpu().numpy().astype(np.float64)
    return step


def calibration(J, N, Nc, seed):
    """Synthetic 2-D 'keys': noisy samples of the centres of a hidden codebook, plus a start point."""
    rng = np.random.default_rng(seed)
    hidden = rng.standard_normal((J, Nc, 2)) * 0.7
    data = np.empty((J, N, 2), np.float32)
    for j in range(J):
        z = hidden[j, :, 0] + 1j * hidden[j, :, 1]
        cen = (z[:, None] + 1j * z[None, :]).reshape(-1)
        pick = cen[rng.integers(0, Nc * Nc, N)]
        data[j, :, 0] = pick.real + 0.05 * rng.standard_normal(N)
        data[j, :, 1] = pick.imag + 0.05 * rng.standard_normal(N)
    start = (hidden + 0.2 * rng.standard_normal((J, Nc, 2))).astype(np.float32)
    return data, start


@pytest.mark.parametrize("Nc,N,T", [(1, 300, 0.5), (4, 1000, 0.3), (8, 3000, 0.2), (64, 4096, 0.1), (64, 1500, 1.0)])
def test_one_em_step_matches_oracle(em, oracle, Nc, N, T):
    J = 3
    data, start = calibration(J, N, Nc, seed=Nc * 1000 + N)
    print(f"case Nc={Nc} N={N} T={T}", flush=True)
    got = em(data, start, T)
    worst = 0.0
    for j in range(J):
        ref, _ = oracle.em_step(data[j], start[j], temperature=T)
        worst = max(worst, np.abs(got[j] - ref).max() / np.abs(ref).max())
    print(f"  max relative deviation of phi: {worst:.3e}", flush=True)
    assert worst <= 2e-3


def test_annealed_iterations_lower_the_objective(em, oracle):
    J, N, Nc = 2, 2000, 8
    data, start = calibration(J, N, Nc, seed=5)
    out = em(data, start, 0.5, iters=6, decay=0.6)
    for j in range(J):
        _, e0 = oracle.em_step(data[j], start[j], temperature=None)     # hard-assignment squared error at phi
        _, e1 = oracle.em_step(data[j], out[j], temperature=None)
        print(f"  sub-space {j}: squared error {e0:.3f} -> {e1:.3f}", flush=True)
        assert e1 < e0


def test_em_argument_checks(em):
    import torch
    import paper_2506_18879_amd as cv
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    for args, status in (((buf, 1, 10, 65, 0.5, buf, buf, 1 << 16), 3), ((buf, 1, 10, 4, 0.0, buf, buf, 1 << 16), 2),
                         ((buf, 1, 10, 4, 0.5, buf, buf, 16), 4), ((None, 1, 10, 4, 0.5, buf, buf, 1 << 16), 1)):
        with pytest.raises(cv.CommVQError) as e:
            cv.commvq_em_step(*args)
        assert e.value.status == status


# ---------------------------------------------------------------- one code shared by a group of sub-spaces
@pytest.fixture(scope="module")
def em_shared():
    import torch
    import paper_2506_18879_amd as cv
    cv.load_library()

    def step(data, phi, T, iters=1, decay=1.0):
        N, J, _ = data.shape
        Nc = phi.shape[1]
        d = torch.from_numpy(np.ascontiguousarray(data, np.float32)).cuda()
        p = torch.from_numpy(np.ascontiguousarray(phi, np.float32)).cuda()
        nb = cv.commvq_em_shared_workspace_bytes(J, N, Nc)
        ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
        for _ in range(iters):
            cv.commvq_em_step_shared(d, J, N, Nc, T, p, ws, nb)
            T *= decay
        torch.cuda.synchronize()
        return p.cpu().numpy().astype(np.float64)
    return step


def shared_calibration(J, N, Nc, seed, noise=0.05):
    """Whole vectors that are noisy centres (a, b) of a hidden tied table, the same pair in all J sub-spaces."""
    rng = np.random.default_rng(seed)
    hidden = rng.standard_normal((J, Nc, 2)) * 0.7
    z = hidden[..., 0] + 1j * hidden[..., 1]                                 # [J][Nc]
    a, b = rng.integers(0, Nc, N), rng.integers(0, Nc, N)
    c = z[:, a] + 1j * z[:, b]                                               # [J][N]
    data = np.stack([c.real.T, c.imag.T], axis=2) + noise * rng.standard_normal((N, J, 2))
    start = hidden + 0.1 * rng.standard_normal((J, Nc, 2))
    return data.astype(np.float32), start.astype(np.float32)


@pytest.mark.parametrize("J,Nc,N,T", [(1, 4, 500, 0.3), (4, 3, 777, 0.5), (16, 8, 1000, 0.8), (64, 64, 1500, 2.0), (64, 64, 200, 4.0),
                                      (7, 5, 64, 0.6)])
def test_one_shared_em_step_matches_oracle(em_shared, oracle, J, Nc, N, T):
    data, start = shared_calibration(J, N, Nc, seed=J * 100 + Nc)
    print(f"case group={J} Nc={Nc} N={N} T={T}", flush=True)
    got = em_shared(data, start, T)
    ref, _ = oracle.em_step_shared(data, start, temperature=T)
    worst = np.abs(got - ref).max() / np.abs(ref).max()
    print(f"  max relative deviation of phi: {worst:.3e}", flush=True)
    assert worst <= 2e-3


def test_shared_group_of_one_equals_the_per_sub_space_entry_point(em, em_shared):
    data, start = calibration(1, 900, 6, seed=11)
    a = em(data, start, 0.4)
    b = em_shared(np.ascontiguousarray(data.transpose(1, 0, 2)), start, 0.4)
    assert np.abs(a - b).max() <= 1e-4 * np.abs(a).max()


def test_shared_annealed_iterations_lower_the_objective(em_shared, oracle):
    J, N, Nc = 8, 1500, 6
    data, start = shared_calibration(J, N, Nc, seed=21, noise=0.1)
    start = start + 0.2 * np.random.default_rng(3).standard_normal(start.shape).astype(np.float32)
    out = em_shared(data, start, 1.0, iters=6, decay=0.6)
    _, e0 = oracle.em_step_shared(data, start, temperature=None)
    _, e1 = oracle.em_step_shared(data, out, temperature=None)
    print(f"  squared error {e0:.3f} -> {e1:.3f}", flush=True)
    assert e1 < e0


def test_shared_em_argument_checks(em_shared):
    import torch
    import paper_2506_18879_amd as cv
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    for args, status in (((buf, 65, 10, 4, 0.5, buf, buf, 1 << 20), 3), ((buf, 4, 10, 65, 0.5, buf, buf, 1 << 20), 3),
                         ((buf, 4, 10, 4, -1.0, buf, buf, 1 << 20), 2), ((buf, 4, 10, 4, 0.5, buf, buf, 16), 4),
                         ((buf, 4, 10, 4, 0.5, None, buf, 1 << 20), 1)):
        with pytest.raises(cv.CommVQError) as e:
            cv.commvq_em_step_shared(*args)
        assert e.value.status == status
