"""kronmatmul_static, the entry point for callers that cannot allocate device memory, against
kronmatmul_ws (same plan, same kernels, so bit-identical results are the bar) and against the CPU
oracle (the bars of test_gpu_parity), through the C-ABI.  The calls run back to back on one GPU's one
static array, each problem smaller than the one before it, so stale contents of the array from the
larger problem would show."""
import ctypes

import numpy as np
import pytest

import kron_inputs
import oracle

torch = pytest.importorskip("torch")
import paper_2401_10187_amd as km  # noqa: E402

pytestmark = pytest.mark.gpu

REL_TOL = {np.dtype("float32"): 1e-5, np.dtype("float64"): 1e-12}

# every problem needs an intermediate (two launches); the intermediates shrink from call to call
SEQUENCE = [
    ("float32", 16, [(8, 8)] * 5),          # 2 MiB of workspace
    ("float32", 3, [(8, 8)] * 5),           # 384 KiB (a smaller input than the first)
    ("float64", 3, [(16, 16)] * 3),         # 96 KiB, other kernels
    ("float64", 2, [(70, 30), (110, 50)]),  # 55 KiB, generic kernel
]


def _raw_static(Xd, Fd, Yd):
    """Straight through ctypes: no Python-side allocation between the arguments and the C-ABI."""
    L = km.lib()
    n = len(Fd)
    p = (ctypes.c_int * n)(*[F.shape[0] for F in Fd])
    q = (ctypes.c_int * n)(*[F.shape[1] for F in Fd])
    f = (ctypes.c_void_p * n)(*[F.data_ptr() for F in Fd])
    code = km.KM_F32 if Xd.dtype == torch.float32 else km.KM_F64
    stream = torch.cuda.current_stream().cuda_stream
    return L.kronmatmul_static(Xd.shape[0], n, p, q, Xd.data_ptr(), ctypes.cast(f, ctypes.c_void_p), Yd.data_ptr(),
                               code, ctypes.c_void_p(stream))


def test_static_entry_point_matches_the_workspace_entry_point():
    if not torch.cuda.is_available():
        pytest.fail("gpu-marked tests need a GPU")
    km.lib()
    for rep in range(2):                                  # the whole sequence twice: large after small too
        for k, (dtype, M, shapes) in enumerate(SEQUENCE):
            X, Fs = kron_inputs.make_problem(M, shapes, dtype, seed=100 + 10 * rep + k)
            P, Q = [s[0] for s in shapes], [s[1] for s in shapes]
            need = km.workspace_size(M, P, Q, dtype)
            assert 0 < need <= km.KM_STATIC_SCRATCH_BYTES, "the case must use the static array"
            Xd = torch.from_numpy(X).cuda()
            Fd = [torch.from_numpy(F).cuda() for F in Fs]
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            want = km.kronmatmul(Xd, Fd, workspace=ws)
            got = torch.full_like(want, float("nan"))
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            print("kronmatmul_static %s M=%d %s" % (dtype, M, shapes), flush=True)
            assert _raw_static(Xd, Fd, got) == km.KM_OK
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
            assert torch.equal(got, want), "differs from kronmatmul_ws"
            ref = oracle.kron_matmul(X, Fs)
            err = float(np.abs(got.cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max())
            assert err <= REL_TOL[ref.dtype], err
    # integer inputs: bit-exact against the oracle
    Xi, Fi = kron_inputs.make_problem(16, [(8, 8)] * 5, "float32", "int2", "int1", seed=7)
    Yi = km.kronmatmul(torch.from_numpy(Xi).cuda(), [torch.from_numpy(F).cuda() for F in Fi], static=True)
    torch.cuda.synchronize()
    assert np.array_equal(Yi.cpu().numpy(), oracle.kron_matmul(Xi, Fi))
    km.release()
