"""The allocation-free entry point osscar_gram_static against osscar_gram (+ finalize), through the C-ABI: two calls in a
row on the same GPU, the second with a smaller input, so that whatever the first call left in the library's fixed scratch
array must not reach the second result.  Both are also held against the float64 oracle."""
import numpy as np
import pytest
import torch

import osscar_inputs as inp
from oracle import osscar_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _reference(cfg, X, W):
    """H, G, lambda, c0 from the existing entry point."""
    import paper_2403_12983_amd as pkg
    from paper_2403_12983_amd import binding as B
    s = pkg.Solver(cfg.d1, cfg.m, cfg.p, cfg.q, cfg.k, 1, X.dtype, W.dtype, DEV)
    s.osscar_gram(X, True, W, cfg.lam_abs, cfg.lam_rel)
    H, G = s.osscar_get_tensor(B.T_H).clone(), s.osscar_get_tensor(B.T_G).clone()
    lam, c0 = s.osscar_get_scalars()
    s.close()
    return H, G, lam, c0


def _static(cfg, X, W, poison):
    import paper_2403_12983_amd as pkg
    H = torch.full((cfg.d1, cfg.d1), poison, dtype=torch.float32, device=DEV)
    G = torch.full((cfg.d1, cfg.m), poison, dtype=torch.float32, device=DEV)
    sc = torch.full((2,), poison, dtype=torch.float64, device=DEV)
    pkg.osscar_gram_static(X, W, H, G, sc, cfg.lam_abs, cfg.lam_rel)
    torch.cuda.synchronize()
    return H, G, float(sc[0].item()), float(sc[1].item())


def _compare(cfg, X, W, poison):
    Hr, Gr, lamr, c0r = _reference(cfg, X, W)
    Hs, Gs, lams, c0s = _static(cfg, X, W, poison)
    d = torch.sqrt(torch.diagonal(Hr).double())
    assert ((Hs.double() - Hr.double()).abs() / torch.outer(d, d)).max().item() < 1e-6
    assert (torch.linalg.norm(Gs.double() - Gr.double()) / torch.linalg.norm(Gr.double())).item() < 1e-6
    assert abs(lams - lamr) <= 1e-6 * abs(lamr) and abs(c0s - c0r) <= 1e-6 * abs(c0r)
    assert torch.equal(Hs, Hs.T)
    # and against the oracle (Section 3: H = X^T X + lambda I, G = H W)
    Ho, Go, c0o, lamo = orc.gram(X.cpu().double().numpy(), W.cpu().double().numpy(), cfg.lam_abs, cfg.lam_rel)
    do = np.sqrt(np.diag(Ho))
    assert np.max(np.abs(Hs.cpu().double().numpy() - Ho) / np.outer(do, do)) < 1e-6
    assert np.linalg.norm(Gs.cpu().double().numpy() - Go) / np.linalg.norm(Go) < 1e-6
    assert abs(lams - lamo) <= 1e-6 * lamo and abs(c0s - c0o) <= 1e-6 * c0o


def test_static_gram_matches_osscar_gram_on_two_calls_in_a_row():
    # first call: bf16 activations and weights, d1 = 328 (2.6 tiles), 3000 rows (two sub-steps, the second ragged)
    big = inp.scaled(inp.CONFIGS["cfg3"], p=328, m=136, n=3000, k=160, swaps=1)
    Xb, Wb = inp.gen_X(big, device=DEV), inp.gen_W(big, DEV)
    _compare(big, Xb, Wb, poison=float("nan"))
    # second call, smaller on every axis and in float32: the scratch array still holds the first call's accumulator,
    # weights and staged rows
    small = inp.CONFIGS["cfg1"]
    Xs, Ws = inp.gen_X(small, device=DEV), inp.gen_W(small, DEV)
    _compare(small, Xs, Ws, poison=7.0)
    # and a larger one again, conv-shaped groups in float32 with a relative ridge
    mid = inp.scaled(inp.CONFIGS["cfg2"], p=24, m=40, n=1500, k=12, swaps=1, mix=0.5)
    Xm, Wm = inp.gen_X(mid, device=DEV), inp.gen_W(mid, DEV)
    _compare(mid, Xm, Wm, poison=-3.0)


def test_static_gram_limits_and_errors():
    import paper_2403_12983_amd as pkg
    from paper_2403_12983_amd.binding import OsscarError
    d1, m = 1025, 8
    X = torch.zeros(4, d1, device=DEV)
    W = torch.zeros(d1, m, device=DEV)
    H = torch.zeros(d1, d1, device=DEV)
    G = torch.zeros(d1, m, device=DEV)
    sc = torch.zeros(2, dtype=torch.float64, device=DEV)
    with pytest.raises(OsscarError) as e:
        pkg.osscar_gram_static(X, W, H, G, sc, 1e-3, 0.0)
    assert e.value.status == 2 and "1024" in str(e.value)
    # no rows at all: H = lambda_abs I, G = lambda_abs W
    d1, m = 16, 8
    W = inp.gen_W(inp.scaled(inp.CONFIGS["cfg1"], p=16, m=8, n=64, k=8, swaps=1), DEV)
    H = torch.empty(d1, d1, device=DEV)
    G = torch.empty(d1, m, device=DEV)
    pkg.osscar_gram_static(torch.zeros(0, d1, device=DEV), W, H, G, sc, 0.5, 1e-2)
    torch.cuda.synchronize()
    assert torch.equal(H, 0.5 * torch.eye(d1, device=DEV)) and torch.allclose(G, 0.5 * W, rtol=1e-6, atol=0)
    assert sc[0].item() == 0.5
