"""The entry point that allocates nothing, `dk_decode_verify_static`, against
`dk_decode_verify` (which takes the same scratch memory from a caller's
workspace): bit-identical outputs, on two calls in a row -- the second with a
smaller input, so that whatever the first call left in the library's built-in
scratch array is still there -- and at the group limit."""
import ctypes as C
import sys

import numpy as np
import pytest

import dk_inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dk():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: torch.cuda.is_available() is False")
    import paper_2207_00083_amd as dk
    dk.load()
    return dk


def _case(dk, K, G, m, seed, corrupt_groups):
    """Synthetic encoded results with the null-vector property, some groups
    corrupted; returns device tensors and the expected verdicts."""
    rng = np.random.default_rng(seed)
    S = K + 2
    A, gamma = dk_inputs.sample_coeff_draws(rng, G, K)
    Ainv, nvec, _ = dk.dk_coeffs(A, gamma)
    # rows [y_1..y_K, W r, 0] . A  -> consistent encodings
    src = rng.standard_normal((G, S, m)).astype(np.float32)
    src[:, K] *= 10.0
    src[:, K + 1] = 0.0
    ybar = np.einsum("gij,gim->gjm", A.astype(np.float64), src.astype(np.float64)).astype(np.float32)
    for g in corrupt_groups:
        j = int(np.argmax(np.abs(nvec[g])))
        ybar[g, j, int(rng.integers(m))] += 0.5 * float(np.max(np.abs(ybar[g])))
    expect = np.zeros(G, dtype=np.int32)
    expect[list(corrupt_groups)] = 1
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return dev(ybar.reshape(G * S, m)), dev(Ainv), dev(nvec), expect


def _both(dk, K, G, m, seed, corrupt_groups):
    ybar, Ainv, nvec, expect = _case(dk, K, G, m, seed, corrupt_groups)
    f32 = dict(dtype=torch.float32, device="cuda")
    y_ref, v_ref, r_ref = dk.dk_decode_verify(ybar, Ainv, nvec, K, tol=1e-3)
    y = torch.full((G * K, m), 7.0, **f32)
    v = torch.full((G,), 7, dtype=torch.int32, device="cuda")
    r = torch.full((G,), 7.0, **f32)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    # straight through the C ABI
    st = dk.load().dk_decode_verify_static(
        C.c_void_p(ybar.data_ptr()), C.c_void_p(Ainv.data_ptr()), C.c_void_p(nvec.data_ptr()),
        C.c_float(1e-3), C.c_void_p(y.data_ptr()), C.c_void_p(v.data_ptr()), C.c_void_p(r.data_ptr()),
        G, K, C.c_longlong(m), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, dk.dk_status_str(st)
    torch.cuda.synchronize()
    assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == before
    assert v_ref.cpu().numpy().tolist() == expect.tolist()
    assert torch.equal(v, v_ref)
    assert torch.equal(r.view(torch.int32), r_ref.view(torch.int32))
    assert torch.equal(y.view(torch.int32), y_ref.view(torch.int32))


def test_static_entry_point_equals_the_workspace_one_twice_in_a_row(dk):
    say("dk_decode_verify_static: K=4, G=64, m=65536, groups 3 and 40 corrupted")
    _both(dk, 4, 64, 65536, seed=1, corrupt_groups=(3, 40))
    # smaller input next: fewer groups, fewer and shorter spans, other groups corrupted
    say("dk_decode_verify_static: K=2, G=5, m=1003 (ragged, scalar path), group 4 corrupted")
    _both(dk, 2, 5, 1003, seed=2, corrupt_groups=(4,))
    say("dk_decode_verify_static: K=8, G=3, m=4096, clean")
    _both(dk, 8, 3, 4096, seed=3, corrupt_groups=())


def test_static_entry_point_at_and_beyond_its_group_limit(dk):
    G = 4096
    say("dk_decode_verify_static: K=1, G=%d (the limit), m=64" % G)
    _both(dk, 1, G, 64, seed=4, corrupt_groups=(0, 4095))
    ybar, Ainv, nvec, _ = _case(dk, 1, 8, 64, 5, ())
    y = torch.empty((8, 64), dtype=torch.float32, device="cuda")
    v = torch.empty(8, dtype=torch.int32, device="cuda")
    st = dk.load().dk_decode_verify_static(
        C.c_void_p(ybar.data_ptr()), C.c_void_p(Ainv.data_ptr()), C.c_void_p(nvec.data_ptr()),
        C.c_float(1e-3), C.c_void_p(y.data_ptr()), C.c_void_p(v.data_ptr()), None,
        G + 1, 1, C.c_longlong(64), None)
    assert st == 8                      # refused on the host, nothing launched
