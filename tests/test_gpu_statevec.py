"""End-to-end use the paper describes (Section 4.4): a state-vector simulation of a brickwork circuit of
random d-qubit unitaries, each gate applied as a complex product of the reshaped state (2^(N-d) x 2^d)
with the 2^d x 2^d gate matrix, the number of slices chosen automatically before every product.
The circuits of the paper are defined in a figure that is not available; this is the same kind of
computation on a seeded synthetic circuit. Every gate product and every chosen slice count is checked
bit for bit against the CPU oracle; the vendor complex GEMM and unitarity are extra context."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_11975_amd import ozimmu

pytestmark = pytest.mark.gpu


def random_unitary(dim, gen):
    g = torch.complex(torch.randn((dim, dim), generator=gen, dtype=torch.float64),
                      torch.randn((dim, dim), generator=gen, dtype=torch.float64))
    q, r = torch.linalg.qr(g)
    return q * (torch.diagonal(r) / torch.diagonal(r).abs())   # Haar-distributed


def apply_gate(state, U, first_qubit, d, N, product):
    """state: 2^N amplitudes; the gate acts on qubits first_qubit .. first_qubit + d - 1."""
    psi = state.reshape([2] * N)
    axes = list(range(first_qubit, first_qubit + d))
    rest = [a for a in range(N) if a not in axes]
    M = psi.permute(rest + axes).reshape(2 ** (N - d), 2 ** d).contiguous()
    out = product(M, U.T.contiguous())                          # row vector convention: psi' = psi U^T
    inv = np.argsort(rest + axes).tolist()
    return out.reshape([2] * N).permute(inv).reshape(-1).contiguous()


@pytest.mark.parametrize("one_call", [False, True])
@pytest.mark.parametrize("threshold,max_rel", [(0.0, 5e-14), (1.0, 5e-13)])
def test_brickwork_random_unitary_circuit(threshold, max_rel, one_call):
    """one_call: count and product by ozimmu_zgemm_auto, the count of the gate before as its guess."""
    N, d, layers = 16, 6, 4
    gen = torch.Generator().manual_seed(11)
    picked, confirmed = [], []

    def ozaki(M, V):
        m, k = M.shape
        n = V.shape[1]
        C = torch.empty((m, n), dtype=torch.complex128, device="cuda")
        if one_call:
            s, ok = ozimmu.zgemm_auto(M, V, C, threshold, guess=picked[-1] if picked else 0)
            confirmed.append(ok)
            assert ok == (bool(picked) and picked[-1] == s)
        else:
            s, _ = ozimmu.auto_num_slices(M, V, threshold)
            ozimmu.zgemm(M, V, C, s, ozimmu.alloc_workspace(m, n, k, s, is_complex=True))
        picked.append(s)
        # the oracle on the same operands: same slice count, same product, bit for bit
        Mh, Vh = M.cpu().numpy(), V.cpu().numpy()
        assert s == oracle.auto_num_slices(Mh, Vh, threshold)[0]
        want, got = oracle.zgemm(Mh, Vh, s), C.cpu().numpy()
        assert np.array_equal(got.real.copy().view(np.uint64), want.real.copy().view(np.uint64)), len(picked)
        assert np.array_equal(got.imag.copy().view(np.uint64), want.imag.copy().view(np.uint64)), len(picked)
        return C

    state0 = torch.zeros(2 ** N, dtype=torch.complex128, device="cuda")
    state0[0] = 1.0
    a, b = state0.clone(), state0.clone()
    for layer in range(layers):
        offset = (d // 2) * (layer % 2)
        for first in range(offset, N - d + 1, d):
            U = random_unitary(2 ** d, gen).cuda()
            a = apply_gate(a, U, first, d, N, ozaki)
            b = apply_gate(b, U, first, d, N, torch.matmul)
    torch.cuda.synchronize()
    a, b = a.cpu().numpy(), b.cpu().numpy()
    assert abs(np.linalg.norm(a) - 1.0) <= 1e-12
    assert np.max(np.abs(a - b)) <= max_rel * np.max(np.abs(b)) * 50
    # amplitude of |00...0>, the quantity the paper compares
    assert abs(a[0] - b[0]) <= max_rel * 50 * abs(b[0]) + 1e-16
    # a lossless split needs more slices than one that may drop a bit on average
    assert min(picked) >= 1 and max(picked) <= 16
    if threshold == 0.0:
        assert max(picked) >= 9
    else:
        assert max(picked) <= 10
    if one_call:
        assert any(confirmed)
