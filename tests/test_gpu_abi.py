"""Error behaviour of the C ABI with a live handle (needs the GPU for svgd_create)."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mod():
    assert torch.cuda.is_available()
    from paper_2306_06528_amd import svgd
    return svgd


def test_argument_errors(mod):
    lib = mod._lib
    X = torch.randn(4, 100, device="cuda")
    G = torch.randn(4, 100, device="cuda")
    P = torch.empty(4, 100, device="cuda")
    eng = mod.Svgd(4, 100)
    h = eng._h
    xp, gp, pp = X.data_ptr(), G.data_ptr(), P.data_ptr()
    assert lib.svgd_step(h, None, gp, 4, 100, 0.1, None) == -1
    assert lib.svgd_step(h, xp, None, 4, 100, 0.1, None) == -1
    assert lib.svgd_step(h, xp, gp, 0, 100, 0.1, None) == -1
    assert lib.svgd_step(h, xp, gp, 4, 0, 0.1, None) == -1
    assert lib.svgd_step(h, xp, gp, 4, 100, float("nan"), None) == -1
    assert lib.svgd_step(h, xp, gp, 4, 100, float("inf"), None) == -1
    assert lib.svgd_step(h, xp, xp, 4, 100, 0.1, None) == -1            # X aliases G
    assert lib.svgd_step(h, xp, xp + 400, 4, 100, 0.1, None) == -1      # partial overlap
    assert lib.svgd_step(h, xp, gp, 5, 100, 0.1, None) == -3
    assert lib.svgd_step(h, xp, gp, 4, 101, 0.1, None) == -3
    assert lib.svgd_phi(h, xp, gp, 4, 100, xp, None) == -1              # PHI aliases X
    assert lib.svgd_phi(h, xp, gp, 4, 100, None, None) == -1
    assert lib.svgd_bandwidth(h, None, 4, 100, None, None) == -1
    assert lib.svgd_get_last(h, None, None, None) == -1                 # nothing computed yet
    assert lib.svgd_set_bandwidth(h, float("nan")) == -1
    torch.cuda.synchronize()
    assert torch.isfinite(X).all()
    # a valid call still works afterwards, and the handle dies with destroy
    assert lib.svgd_phi(h, xp, gp, 4, 100, pp, None) == 0
    torch.cuda.synchronize()
    assert torch.isfinite(P).all()
    stale = ctypes.c_void_p(h.value)
    eng.close()
    assert lib.svgd_step(stale, xp, gp, 4, 100, 0.1, None) == -2        # use after destroy
    assert lib.svgd_destroy(stale) == -2


def test_binding_raises(mod):
    eng = mod.Svgd(4, 100)
    X = torch.randn(5, 100, device="cuda")
    with pytest.raises(mod.SvgdError):
        eng.step(X, torch.randn_like(X), 0.1)
    with pytest.raises(TypeError):
        eng.step(X.cpu(), X.cpu(), 0.1)
    with pytest.raises(ValueError):          # nothing computed yet
        eng.get_last(4)
    Y = torch.randn(3, 100, device="cuda")
    eng.step(Y, torch.randn_like(Y), 0.1)
    with pytest.raises(ValueError):          # K of the last call is 3 x 3: no room to get that wrong
        eng.get_last(2)
    h, K = eng.get_last(3)
    assert h > 0 and K.shape == (3, 3)
    eng.close()
    with pytest.raises(mod.SvgdError):
        mod.Svgd(65, 100)


def test_profiling_selects_kernel_kinds(mod):
    X = torch.randn(32, 50_000, device="cuda")
    G = torch.randn_like(X)
    with mod.Svgd(32, 50_000) as eng:
        eng.profile_begin()
        eng.step(X, G, 0.01)
        prof = eng.profile_end()
        assert [prof[k][1] for k in mod.KERNEL_KINDS] == [1, 1, 1, 1]
        assert all(prof[k][0] > 0 for k in mod.KERNEL_KINDS)
        eng.profile_begin(("update",))
        eng.step(X, G, 0.01)
        eng.step(X, G, 0.01)
        prof = eng.profile_end()
        assert [prof[k][1] for k in mod.KERNEL_KINDS] == [0, 0, 0, 2]
        assert mod._lib.svgd_profile_begin_kinds(eng._h, 0) == -1       # no kind selected
        eng.step(X, G, 0.01)                                            # recording is off again
        assert [v[1] for v in eng.profile_end().values()] == [0, 0, 0, 0]


@pytest.mark.parametrize("pattern", [0, 1, 2, 3])
@pytest.mark.parametrize("n,D,ld", [(64, 20_011, 20_032), (8, 70_001, 70_001), (33, 1000, 1003), (3, 63, 64)])
def test_diag_read_rows(mod, pattern, n, D, ld):
    """The read yardstick reads every element of the n x D window exactly once: with ones inside the
    window and large values in the padding, the workgroups' sums add up to n * D exactly (integers
    that fp32 holds), whatever the grid."""
    buf = torch.full((n, ld), 1e6, device="cuda")
    X = buf[:, :D]
    X.fill_(1.0)
    for workgroups in (1, 7, 300):
        sink = torch.full((workgroups,), float("nan"), device="cuda")
        mod.diag_read_rows(X, sink, pattern)
        torch.cuda.synchronize()
        assert float(sink.double().sum().item()) == float(n * D)
    sink = torch.zeros(4, device="cuda")
    assert mod._lib.svgd_diag_read_rows(X.data_ptr(), n, D, ld, sink.data_ptr(), 4, 4, None) == -1
    assert mod._lib.svgd_diag_read_rows(X.data_ptr(), n, D, ld, sink.data_ptr(), 0, 0, None) == -1
    assert mod._lib.svgd_diag_read_rows(X.data_ptr(), n, D, D - 1, sink.data_ptr(), 0, 4, None) == -1
    assert mod._lib.svgd_diag_read_rows(None, n, D, ld, sink.data_ptr(), 0, 4, None) == -1


@pytest.mark.parametrize("pattern", list(range(12)) + [16, 21, 27])
@pytest.mark.parametrize("n,D,ld", [(64, 20_011, 20_032), (8, 70_001, 70_001), (33, 1000, 1003), (3, 63, 64)])
def test_diag_axpy_rows(mod, pattern, n, D, ld):
    """The yardstick kernel does what it says (x += s * g on the n x D window, nothing outside)."""
    buf = torch.randn(n, ld, device="cuda")
    gbuf = torch.randn(n, ld, device="cuda")
    X, G = buf[:, :D], gbuf[:, :D]
    want = buf.clone()
    want[:, :D] += 0.25 * G
    mod.diag_axpy_rows(X, G, 0.25, pattern, 7)
    torch.cuda.synchronize()
    assert torch.allclose(buf, want, rtol=0, atol=1e-6)
    assert torch.equal(buf[:, D:], want[:, D:])
    assert mod._lib.svgd_diag_axpy_rows(X.data_ptr(), G.data_ptr(), n, D, ld, 0.25, 12, 7, None) == -1
    assert mod._lib.svgd_diag_axpy_rows(X.data_ptr(), G.data_ptr(), n, D, ld, 0.25, 32, 7, None) == -1
    assert mod._lib.svgd_diag_axpy_rows(X.data_ptr(), G.data_ptr(), n, D, ld, 0.25, 0, 0, None) == -1
