"""Interception of the vendor DGEMM/ZGEMM calls (Section 4.4, third extension): an unmodified rocBLAS /
hipBLAS program is started with libozimmu_preload.so first in the loader's preload list; its result
must then be the Ozaki result, bit for bit the oracle's, and the vendor's own result when the
interposer is told to pass calls through. The program is a child process: it reads the problem from a
file and writes C back (csrc/blas_client.cpp)."""
import os
import subprocess
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2306_11975_amd import ozimmu
from paper_2306_11975_amd import workloads as wl

pytestmark = pytest.mark.gpu

PKG = Path(ozimmu.__file__).resolve().parent
CLIENT, PRELOAD = PKG / "blas_client", PKG / "libozimmu_preload.so"
CODE = {"N": 0, "T": 1, "C": 2}


def bits(x):
    return np.ascontiguousarray(x).view(np.uint64)


def run_client(tmp_path, api, ta, tb, alpha, beta, A, B, C0, mode, repeats=1, streams=1, extra_env=None):
    """A, B, C0 as stored (column-major semantics are produced here). Returns (C, stderr)."""
    if not CLIENT.exists() or not PRELOAD.exists():
        pytest.skip("blas_client / libozimmu_preload.so have not been built (python -m paper_2306_11975_amd.build)")
    cplx = np.iscomplexobj(C0)
    dt = np.complex128 if cplx else np.float64
    m, n = C0.shape
    k = A.shape[0] if CODE[ta] else A.shape[1]
    prob, res = tmp_path / "problem.bin", tmp_path / "result.bin"
    with open(prob, "wb") as f:
        np.array([api, int(cplx), CODE[ta], CODE[tb], m, n, k, repeats, streams], dtype=np.int64).tofile(f)
        np.array([complex(alpha).real, complex(alpha).imag, complex(beta).real, complex(beta).imag]).tofile(f)
        for M in (A, B, C0):
            np.asfortranarray(M.astype(dt)).T.tofile(f)     # column-major bytes
    env = dict(os.environ)
    if mode is not None:
        # first in the list; whatever the environment already preloads stays in place behind it
        env["LD_PRELOAD"] = str(PRELOAD) + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
        env["OZIMMU_MODE"] = mode
        env["OZIMMU_VERBOSE"] = "1"
    env.update(extra_env or {})
    if res.exists():
        res.unlink()
    print(f"blas_client api={api} {ta}{tb} m={m} n={n} k={k} mode={mode}", flush=True)
    p = subprocess.run([str(CLIENT), str(prob), str(res)], env=env, capture_output=True, text=True, timeout=100)
    assert p.returncode == 0, p.stderr
    C = np.fromfile(res, dtype=dt).reshape(n, m).T
    return C, p.stderr


def real_problem(ta, tb, m, n, k, seed):
    opA, opB = wl.phi_pair(m, n, k, 1.0, seed)
    A = opA.T.copy() if ta != "N" else opA
    B = opB.T.copy() if tb != "N" else opB
    C0 = np.random.default_rng(seed + 7).standard_normal((m, n))
    return opA, opB, A, B, C0


@pytest.mark.parametrize("api", [0, 1])
def test_intercepted_dgemm_is_the_ozaki_result(tmp_path, api):
    name = ("rocblas_dgemm", "hipblasDgemm")[api]
    opA, opB, A, B, C0 = real_problem("T", "N", 150, 90, 260, seed=5)
    alpha, beta = 1.5, -0.25
    got, log = run_client(tmp_path, api, "T", "N", alpha, beta, A, B, C0, mode="9")
    want = oracle.dgemm_blas(True, False, alpha, A, B, beta, C0, 9)
    assert np.array_equal(bits(got), bits(want))
    assert f"[ozimmu] {name} TN m=150 n=90 k=260 slices=9" in log

    # automatic slice count, lossless split: the count the oracle picks for op(A), op(B)
    s_auto = oracle.auto_num_slices(opA, opB, 0.0)[0]
    got, log = run_client(tmp_path, api, "T", "N", 1.0, 0.0, A, B, C0, mode="auto")
    assert f"slices={s_auto} (auto)" in log
    assert np.array_equal(bits(got), bits(oracle.dgemm_blas(True, False, 1.0, A, B, 0.0, C0, s_auto)))
    # ... and with one bit of average loss admitted
    s_t1 = oracle.auto_num_slices(opA, opB, 1.0)[0]
    assert s_t1 < s_auto
    got, log = run_client(tmp_path, api, "T", "N", 1.0, 0.0, A, B, C0, mode="auto", extra_env={"OZIMMU_THRESHOLD": "1"})
    assert f"slices={s_t1} (auto)" in log
    assert np.array_equal(bits(got), bits(oracle.dgemm_blas(True, False, 1.0, A, B, 0.0, C0, s_t1)))


def test_vendor_mode_and_no_preload_give_the_vendor_result(tmp_path):
    opA, opB, A, B, C0 = real_problem("N", "T", 64, 130, 200, seed=6)
    plain, _ = run_client(tmp_path, 0, "N", "T", 2.0, 1.0, A, B, C0, mode=None)
    through, log = run_client(tmp_path, 0, "N", "T", 2.0, 1.0, A, B, C0, mode="vendor")
    assert np.array_equal(bits(plain), bits(through))
    assert "rocblas_dgemm -> vendor" in log and "slices=" not in log
    ref = 2.0 * (opA @ opB) + C0
    assert np.allclose(plain, ref, rtol=1e-11, atol=1e-11)
    # small calls can be left to the vendor
    small, log = run_client(tmp_path, 0, "N", "T", 2.0, 1.0, A, B, C0, mode="8", extra_env={"OZIMMU_MIN_WORK": "1e9"})
    assert "-> vendor" in log and np.array_equal(bits(small), bits(plain))


@pytest.mark.parametrize("api", [0, 1])
def test_intercepted_zgemm_is_the_ozaki_result(tmp_path, api):
    rng = np.random.default_rng(11)
    m, n, k = 100, 140, 300
    opA = rng.standard_normal((m, k)) + 1j * rng.standard_normal((m, k))
    opB = rng.standard_normal((k, n)) + 1j * rng.standard_normal((k, n))
    C0 = rng.standard_normal((m, n)) + 1j * rng.standard_normal((m, n))
    A, B = opA.conj().T.copy(), opB
    alpha, beta = 0.5 - 1.25j, 0.75 + 0.5j
    got, log = run_client(tmp_path, api, "C", "N", alpha, beta, A, B, C0, mode="7")
    assert np.array_equal(bits(got), bits(oracle.zgemm_blas("C", "N", alpha, A, B, beta, C0, 7)))
    assert ("rocblas_zgemm", "hipblasZgemm")[api] + " CN" in log
    s_auto = oracle.auto_num_slices(opA, opB, 0.0)[0]
    got, log = run_client(tmp_path, api, "C", "N", 1.0, 0.0, A, B, C0, mode="auto")
    assert f"slices={s_auto} (auto)" in log
    assert np.array_equal(bits(got), bits(oracle.zgemm_blas("C", "N", 1.0, A, B, 0.0, C0, s_auto)))


@pytest.mark.parametrize("threshold", [0.0, 1.0])
def test_small_complex_gate_in_automatic_mode_takes_one_call_per_product(tmp_path, threshold):
    """A gate of 64 x 64 on a wide state, plain product, three times: the count of the call before is the guess of the
    next (ozimmu_zgemm_auto); count and result stay those of the two-call path, i.e. the oracle's."""
    rng = np.random.default_rng(23)
    m, n, k = 64, 2500, 64
    opA = wl.unit_column_complex(m, k, seed=24)
    opB = rng.standard_normal((k, n)) + 1j * rng.standard_normal((k, n))
    opB /= np.linalg.norm(opB)
    C0 = np.zeros((m, n), dtype=np.complex128)
    s_auto = oracle.auto_num_slices(opA, opB, threshold)[0]
    got, log = run_client(tmp_path, 1, "N", "N", 1.0, 0.0, opA, opB, C0, mode="auto", repeats=3,
                          extra_env={"OZIMMU_THRESHOLD": str(threshold)})
    assert log.count(f"slices={s_auto} (auto) [one call]") == 1                       # no guess yet
    assert log.count(f"slices={s_auto} (auto) [one call, guess confirmed]") == 2
    assert np.array_equal(bits(got), bits(oracle.zgemm_blas("N", "N", 1.0, opA, opB, 0.0, C0, s_auto)))


@pytest.mark.parametrize("api,cplx", [(2, False), (2, True), (3, False), (3, True)])
def test_all_fp64_gemm_ex_calls_are_intercepted_too(tmp_path, api, cplx):
    name = {2: "rocblas_gemm_ex", 3: "hipblasGemmEx"}[api]
    rng = np.random.default_rng(17 + api)
    m, n, k = 90, 120, 200
    if cplx:
        opA = rng.standard_normal((m, k)) + 1j * rng.standard_normal((m, k))
        opB = rng.standard_normal((k, n)) + 1j * rng.standard_normal((k, n))
        C0 = rng.standard_normal((m, n)) + 1j * rng.standard_normal((m, n))
        alpha, beta = 1.5 + 0.5j, -0.5j
        got, log = run_client(tmp_path, api, "N", "C", alpha, beta, opA, opB.conj().T.copy(), C0, mode="8")
        want = oracle.zgemm_blas("N", "C", alpha, opA, opB.conj().T.copy(), beta, C0, 8)
    else:
        opA, opB = wl.phi_pair(m, n, k, 1.0, seed=9)
        C0 = rng.standard_normal((m, n))
        alpha, beta = -1.25, 2.0
        got, log = run_client(tmp_path, api, "N", "T", alpha, beta, opA, opB.T.copy(), C0, mode="8")
        want = oracle.dgemm_blas(False, True, alpha, opA, opB.T.copy(), beta, C0, 8)
    assert f"[ozimmu] {name} N" in log and "slices=8" in log
    assert np.array_equal(bits(got), bits(want))


def test_repeated_calls_on_several_streams_share_the_workspace_safely(tmp_path):
    """Six calls round-robin over three streams: the interposer orders them on the device (they share one
    workspace), so the result is that of a single call."""
    opA, opB, A, B, C0 = real_problem("N", "N", 520, 300, 1100, seed=8)
    got, log = run_client(tmp_path, 0, "N", "N", 1.0, 0.0, A, B, C0, mode="6", repeats=6, streams=3)
    assert log.count("slices=6") == 6
    assert np.array_equal(bits(got), bits(oracle.dgemm_blas(False, False, 1.0, A, B, 0.0, C0, 6)))


TORCH_CHILD = r'''
import sys
import numpy as np
import torch
d = np.load(sys.argv[1])
dev = lambda a: torch.from_numpy(a).cuda()
A, B, M, Za, Zb = (dev(d[k]) for k in ("A", "B", "M", "Za", "Zb"))
out = {}
out["mm"] = torch.mm(A, B)
out["mm_t"] = torch.mm(B.t(), A.t())
out["addmm"] = torch.addmm(M, A, B, beta=0.5, alpha=-1.75)
out["zmm"] = Za @ Zb
out["zmm_h"] = Zb.conj().t() @ Za.conj().t()
out["bmm"] = torch.bmm(torch.stack([A, 2 * A, -A]), torch.stack([B, B, 3 * B]))
torch.cuda.synchronize()
np.savez(sys.argv[2], **{k: v.cpu().numpy() for k, v in out.items()})
'''


def test_pytorch_fp64_matmul_is_intercepted(tmp_path):
    """PyTorch's FP64 and complex128 matmul on the GPU reach the vendor library through hipblasDgemm /
    hipblasZgemm (and the strided-batched form for bmm), loaded into a local scope by the extension
    module: started under the preload list an unmodified script computes the Ozaki products."""
    import sys

    if not PRELOAD.exists():
        pytest.skip("libozimmu_preload.so has not been built (python -m paper_2306_11975_amd.build)")
    rng = np.random.default_rng(31)
    A, B = wl.phi_pair(200, 150, 330, 1.0, seed=12)
    M = rng.standard_normal((200, 150))
    Za = rng.standard_normal((70, 90)) + 1j * rng.standard_normal((70, 90))
    Zb = rng.standard_normal((90, 40)) + 1j * rng.standard_normal((90, 40))
    np.savez(tmp_path / "in.npz", A=A, B=B, M=M, Za=Za, Zb=Zb)
    env = dict(os.environ)
    env["LD_PRELOAD"] = str(PRELOAD) + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env.update(OZIMMU_MODE="8", OZIMMU_VERBOSE="1")
    print("python child under the preload list", flush=True)
    p = subprocess.run([sys.executable, "-c", TORCH_CHILD, str(tmp_path / "in.npz"), str(tmp_path / "out.npz")], env=env,
                       capture_output=True, text=True, timeout=110)
    assert p.returncode == 0, p.stderr[-2000:]
    got = np.load(tmp_path / "out.npz")
    assert p.stderr.count("hipblasDgemm ") >= 3 and p.stderr.count("hipblasZgemm ") >= 2, p.stderr[-2000:]
    assert "hipblasDgemmStridedBatched" in p.stderr and "-> vendor" not in p.stderr
    s = 8
    assert np.array_equal(bits(got["mm"]), bits(oracle.dgemm(A, B, s)))
    assert np.array_equal(bits(got["mm_t"]), bits(oracle.dgemm(B.T.copy(), A.T.copy(), s)))
    assert np.array_equal(bits(got["addmm"]), bits(oracle.dgemm_blas(False, False, -1.75, A, B, 0.5, M, s)))
    assert np.array_equal(bits(got["zmm"]), bits(oracle.zgemm(Za, Zb, s)))
    assert np.array_equal(bits(got["zmm_h"]), bits(oracle.zgemm(Zb.conj().T.copy(), Za.conj().T.copy(), s)))
    for i, (fa, fb) in enumerate(((1, 1), (2, 1), (-1, 3))):
        assert np.array_equal(bits(got["bmm"][i]), bits(oracle.dgemm(fa * A, fb * B, s)))


SIMULATOR = r'''
# a plain PyTorch state-vector simulator: brickwork circuit of Haar-random d-qubit gates, every gate one
# complex128 matmul of the reshaped state with the gate matrix (knows nothing about ozimmu)
import sys
import numpy as np
import torch
N, d, layers = 16, 6, 4
gen = torch.Generator().manual_seed(11)

def random_unitary(dim):
    g = torch.complex(torch.randn((dim, dim), generator=gen, dtype=torch.float64),
                      torch.randn((dim, dim), generator=gen, dtype=torch.float64))
    q, r = torch.linalg.qr(g)
    return q * (torch.diagonal(r) / torch.diagonal(r).abs())

state = torch.zeros(2 ** N, dtype=torch.complex128, device="cuda")
state[0] = 1.0
gates = []
for layer in range(layers):
    offset = (d // 2) * (layer % 2)
    for first in range(offset, N - d + 1, d):
        U = random_unitary(2 ** d)
        gates.append(U.numpy().copy())
        U = U.cuda()
        axes = list(range(first, first + d))
        rest = [a for a in range(N) if a not in axes]
        M = state.reshape([2] * N).permute(rest + axes).reshape(2 ** (N - d), 2 ** d).contiguous()
        out = torch.matmul(M, U.T.contiguous())
        state = out.reshape([2] * N).permute(np.argsort(rest + axes).tolist()).reshape(-1).contiguous()
torch.cuda.synchronize()
np.save(sys.argv[1], state.cpu().numpy())
np.save(sys.argv[1] + ".gates.npy", np.stack(gates))      # the circuit, so that a checker can replay it
'''


def replay_with_oracle(gates, threshold, N=16, d=6, layers=4):
    """The same circuit on the CPU, every gate product by the oracle with the oracle's own automatic
    slice count. Reshapes and permutations move data without arithmetic, so a simulator whose products
    are the oracle's ends in exactly this state."""
    state = np.zeros(2 ** N, dtype=np.complex128)
    state[0] = 1.0
    picked, g = [], 0
    for layer in range(layers):
        offset = (d // 2) * (layer % 2)
        for first in range(offset, N - d + 1, d):
            axes = list(range(first, first + d))
            rest = [a for a in range(N) if a not in axes]
            M = np.ascontiguousarray(state.reshape([2] * N).transpose(rest + axes).reshape(2 ** (N - d), 2 ** d))
            V = np.ascontiguousarray(gates[g].T)
            g += 1
            s = oracle.auto_num_slices(M, V, threshold)[0]
            picked.append(s)
            out = oracle.zgemm(M, V, s)
            state = np.ascontiguousarray(out.reshape([2] * N).transpose(np.argsort(rest + axes).tolist()).reshape(-1))
    return state, picked


def test_unmodified_simulator_under_the_preload_list(tmp_path):
    """The use the paper reports (Section 4.4): a state-vector simulator that calls the vendor ZGEMM is run
    unchanged, once as it is and once with the interposer in automatic mode at thresholds 0 and 1."""
    import re
    import sys

    if not PRELOAD.exists():
        pytest.skip("libozimmu_preload.so has not been built (python -m paper_2306_11975_amd.build)")

    def run(mode, threshold=None):
        env = dict(os.environ)
        if mode is not None:
            env["LD_PRELOAD"] = str(PRELOAD) + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
            env.update(OZIMMU_MODE=mode, OZIMMU_VERBOSE="1")
            if threshold is not None:
                env["OZIMMU_THRESHOLD"] = str(threshold)
        out = tmp_path / f"state_{mode}_{threshold}.npy"
        print(f"simulator child, mode={mode} threshold={threshold}", flush=True)
        p = subprocess.run([sys.executable, "-c", SIMULATOR, str(out)], env=env, capture_output=True, text=True, timeout=110)
        assert p.returncode == 0, p.stderr[-2000:]
        return np.load(out), np.load(str(out) + ".gates.npy"), p.stderr

    ref, ref_gates, _ = run(None)
    assert abs(np.linalg.norm(ref) - 1.0) <= 1e-12
    for threshold, tol, lo, hi in ((0, 5e-14, 9, 16), (1, 5e-13, 3, 10)):
        got, gates, log = run("auto", threshold)
        picked = [int(x) for x in re.findall(r"hipblasZgemm \S+ m=\d+ n=\d+ k=\d+ slices=(\d+) \(auto\)", log)]
        assert len(picked) == 8, log[-1500:]             # 4 layers of 2 gates
        # every gate through the one-call path, its guess (the count of the gate before) confirmed whenever it was right
        assert log.count("[one call") == 8, log[-1500:]
        assert log.count("guess confirmed") == sum(a == b for a, b in zip(picked, picked[1:])), log[-1500:]
        assert lo <= max(picked) <= hi
        # the oracle's replay of the same circuit: same slice count at every gate, same final state bit for bit
        assert np.array_equal(gates, ref_gates)
        want, want_picked = replay_with_oracle(gates, float(threshold))
        assert picked == want_picked
        assert np.array_equal(bits(got.real.copy()), bits(want.real.copy()))
        assert np.array_equal(bits(got.imag.copy()), bits(want.imag.copy()))
        assert abs(np.linalg.norm(got) - 1.0) <= 1e-12
        assert np.max(np.abs(got - ref)) <= tol * 50 * np.max(np.abs(ref))
        assert abs(got[0] - ref[0]) <= tol * 50 * abs(ref[0]) + 1e-16     # the amplitude the paper compares
