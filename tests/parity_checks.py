"""Shared checks of the GPU parity tests: the HIP path (through the C ABI) against the fp64 oracle.

Tolerances (the stated bar): max|dphi| / max|phi| <= 1e-4, |dh| / h <= 1e-5, max|dK| <= 1e-5.
eps * phi is only a few ulp of X at NN-like scales, so X_new alone cannot show phi: phi is compared
through the emit-phi variant of the same kernels (svgd_phi), and the in-place path (svgd_step) is
then checked against fl32(x + eps * phi_gpu) to one ulp on every entry.
"""
import numpy as np
import torch

from oracle import svgd_oracle as orc

TOL_PHI, TOL_H, TOL_K = 1e-4, 1e-5, 1e-5


def ulp_diff(a, b):
    """max distance of a (fp64) from b (fp32 result), in units of fp32 ulp of b."""
    a = a.astype(np.float64)
    b32 = b.astype(np.float32)
    ulp = np.spacing(np.abs(b32)).astype(np.float64)
    return float((np.abs(a - b32.astype(np.float64)) / ulp).max())


def ulp_diff_device(X_new, X_old, PHI, eps, block=1 << 27):
    """The in-place update against fl32(X_old + fl32(eps) * PHI) on ALL entries, evaluated on the
    device in fp64 (the product and the sum are exact to far below an fp32 ulp), a block of rows at
    a time to bound the fp64 temporaries.  Returns max |X_new - want| / allowed with
        allowed = ulp_fp32(max(|x_old|, |x_new|)) + 1e-6 * |eps| * max|PHI|:
    one rounding at the magnitude of the operands (x_new itself can cancel to almost nothing, its
    own ulp is no yardstick), plus a hundredth of the phi tolerance for the case that PHI comes
    from another handle whose h, hence whose fp32 coefficient table, differs in the last bit.
    An update that did nothing is off by |eps * phi|, 10^6 times the second term."""
    e = torch.tensor(float(np.float32(eps)), dtype=torch.float64, device=X_new.device)
    n, D = X_new.shape
    rows = max(1, block // D)
    phimax = max(float(PHI[r:r + rows].abs().max().item()) for r in range(0, n, rows))
    slack = 1e-6 * abs(float(np.float32(eps))) * phimax
    worst = 0.0
    for r in range(0, n, rows):
        xn, xo, ph = X_new[r:r + rows], X_old[r:r + rows], PHI[r:r + rows]
        want = torch.addcmul(xo.double(), ph.double(), e)
        mag = torch.maximum(xn.abs(), xo.abs())
        ulp = (torch.nextafter(mag, torch.full_like(mag, float("inf"))) - mag).double().clamp_min(1e-45)
        worst = max(worst, float(((xn.double() - want).abs() / (ulp + slack)).max().item()))
    return worst


def oracle_kernel_matrix(Xh):
    d2 = orc.pairwise_d2(Xh)
    h = orc.bandwidth(d2)
    K, _ = orc.kernel(d2, h)
    return h, K


def phi_error_all_columns(PHI, Xh, Gh, K_ref, h_ref, chunk=1 << 20):
    """max|phi_gpu - phi_oracle| / max|phi_oracle| over ALL columns; the oracle's phi is streamed in
    column chunks (an n x D fp64 array would not fit next to the inputs at the large sizes) and the
    normaliser is the oracle's own maximum."""
    n, D = Xh.shape
    worst = scale = 0.0
    for s in range(0, D, chunk):
        w = min(chunk, D - s)
        ref = orc.phi_cols(Xh, Gh, K_ref, h_ref, s, w)
        got = PHI[:, s:s + w].cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        worst = max(worst, float(np.abs(got - ref).max()))
        scale = max(scale, float(np.abs(ref).max()))
    return worst / (scale if scale > 0 else 1.0)


def assert_x_new(X_new_h, ref, eps, what=""):
    """The in-place result against the oracle's x + eps * phi at the phi tolerance: the error may be
    1e-4 of eps * max|phi| plus one fp32 rounding of x, nothing more - a bound that an update which
    did nothing (or used a visibly wrong phi) cannot meet."""
    phi_max = float(np.abs(ref["phi"]).max())
    x_max = float(np.abs(ref["X_new"]).max())
    tol = TOL_PHI * abs(eps) * phi_max + float(np.spacing(np.float32(x_max)))
    err = float(np.abs(X_new_h.astype(np.float64) - ref["X_new"]).max())
    assert err <= tol, f"{what}: |X_new - (x + eps*phi_oracle)| = {err:.3e} > {tol:.3e}"
    # the bound must be able to see phi at all
    assert abs(eps) * phi_max > 4 * tol or eps == 0.0 or phi_max == 0.0, \
        f"{what}: this check is blind to phi (eps*max|phi| = {abs(eps) * phi_max:.3e}, tol {tol:.3e})"


def padded_copy(svgd, t):
    """t in the layout the update kernels like best: rows ld = D rounded up to 32 floats apart on a
    128-byte-aligned allocation."""
    n, D = t.shape
    v = svgd.padded_rows(n, D, device=t.device)
    v.copy_(t)
    assert v.data_ptr() % 128 == 0 and (n == 1 or v.stride(0) % 32 == 0)
    return v


def check_carried_chain(svgd, X0, G, eps, padded, steps=2, chunk=1 << 20):
    """svgd_step with SVGD_FLAG_CARRY_GRAM, `steps` times in a row (every step after the first takes
    its pair sums from the previous update), each step checked completely:
      h, K of the step (svgd_get_last)                    vs the oracle on the pre-step X,
      phi_gpu = svgd_phi of a second, plain handle        vs the oracle at 1e-4 max|phi_oracle|,
      X_new                                               == fl32(x + eps * phi_gpu) to 1 ulp, on
                                                          all n * D entries, on the device.
    padded: X, G and PHI are laid out with every row on a 128-byte boundary (the layout that selects
    the update kernel's direct-store instance), else dense.  X0, G: dense (n, D) device tensors."""
    n, D = X0.shape
    if padded:
        X, Gv = padded_copy(svgd, X0), padded_copy(svgd, G)
        PHI = svgd.padded_rows(n, D, device=X0.device, fill=float("nan"))
    else:
        X, Gv, PHI = X0.clone(), G, torch.full_like(X0, float("nan"))
    Gh = G.cpu().numpy()
    out = []
    with svgd.Svgd(n, D, flags=svgd.FLAG_CARRY_GRAM) as eng, svgd.Svgd(n, D) as plain:
        for step in range(steps):
            X_old = X.clone()
            plain.phi(X, Gv, PHI)                 # recomputed from X: independent of the carried sums
            assert torch.equal(X, X_old), "svgd_phi must leave X untouched"
            eng.step(X, Gv, eps)
            h, K = eng.get_last(n)
            Xh = X_old.cpu().numpy()
            h_ref, K_ref = oracle_kernel_matrix(Xh)
            e_h = abs(h - h_ref) / h_ref
            e_K = float(np.abs(K.astype(np.float64) - K_ref).max())
            assert e_h <= TOL_H, f"step {step}: h {h} vs {h_ref} (rel {e_h:.3e})"
            assert e_K <= TOL_K, f"step {step}: K max abs err {e_K:.3e}"
            assert np.array_equal(K, K.T) and np.all(np.diag(K) == 1.0)
            e_phi = phi_error_all_columns(PHI, Xh, Gh, K_ref, h_ref, chunk)
            assert e_phi <= TOL_PHI, f"step {step}: phi err / max|phi| = {e_phi:.3e}"
            ulps = ulp_diff_device(X, X_old, PHI, eps)
            assert ulps <= 1.0, f"step {step}: in-place update differs from x + eps*phi_gpu by {ulps} ulp"
            out.append(dict(e_h=e_h, e_K=e_K, e_phi=e_phi, ulps=ulps))
            del X_old
    return out
