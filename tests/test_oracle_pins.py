"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test names the plausible mistake it is meant to catch.  None of the expected values comes from
the HIP path; they are library routines (torch CPU nn.LSTM / nn.GRU in float64), an algebraically
different formulation differentiated by autograd (unstabilized sLSTM), closed forms, hand-worked
rational examples (tests/golden) and finite differences.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import CELL_ELMAN, CELL_GRU, CELL_GRU4, CELL_LSTM, CELL_SLSTM

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
CELLS = [CELL_LSTM, CELL_GRU, CELL_SLSTM, CELL_ELMAN, CELL_GRU4]


def _rand(cell, T, B, NH, D, seed, rscale=0.6, with_s0=True):
    rng = np.random.default_rng(seed)
    G, S = oracle.num_gates(cell), oracle.num_states(cell)
    Wx = rng.standard_normal((T, B, G, NH, D))
    R = rng.standard_normal((NH, D, G, D)) * rscale / math.sqrt(D)
    b = rng.standard_normal((NH, G, D)) * 0.3
    s0 = None
    if with_s0:
        s0 = rng.uniform(-0.5, 0.5, size=(S, B, NH, D))
        if cell == CELL_SLSTM:
            s0[2] = rng.uniform(0.5, 1.5, size=(B, NH, D))  # normalizer positive
            s0[3] = rng.uniform(-0.3, 0.3, size=(B, NH, D))
    dH = rng.standard_normal((T, B, NH, D))
    return Wx, R, b, s0, dH


def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


# ----------------------------------------------------------------------------------------------
# library special cases: NH = 1 reduces LSTM / GRU / Elman to the textbook cells (Sec. 3, App. A)
# ----------------------------------------------------------------------------------------------
def _torch_rnn_reference(kind, Wx, R, b, s0, dH):
    """Run torch's CPU nn.LSTM / nn.GRU in float64 with W_ih = identity so that its input is the
    gate pre-activation, W_hh / b_hh re-laid-out from R / b.  Returns h[T], final c, and autograd
    gradients (dWx, dR, db, dh0, dc0)."""
    T, B, G, NH, D = Wx.shape
    assert NH == 1
    mod = {"lstm": torch.nn.LSTM, "gru": torch.nn.GRU, "elman": torch.nn.RNN}[kind](G * D, D, bias=True).double()   # nn.RNN: tanh
    x = torch.tensor(Wx.reshape(T, B, G * D), requires_grad=True)
    # torch: weight_hh[g*D + e, d] multiplies h[d] into gate g of unit e;  ours: R[0, d, g, e]
    w_hh = torch.tensor(np.ascontiguousarray(R[0].transpose(1, 2, 0)).reshape(G * D, D), requires_grad=True)
    b_hh = torch.tensor(b[0].reshape(G * D), requires_grad=True)
    h0 = torch.tensor(s0[0].reshape(1, B, D), requires_grad=True)
    params = {"weight_ih_l0": torch.eye(G * D, dtype=torch.float64), "weight_hh_l0": w_hh,
              "bias_ih_l0": torch.zeros(G * D, dtype=torch.float64), "bias_hh_l0": b_hh}
    if kind == "lstm":
        c0 = torch.tensor(s0[1].reshape(1, B, D), requires_grad=True)
        out, (hn, cn) = torch.func.functional_call(mod, params, (x, (h0, c0)))
    else:
        c0, cn = None, None
        out, hn = torch.func.functional_call(mod, params, (x, h0))
    loss = (out * torch.tensor(dH.reshape(T, B, D))).sum()
    wrt = [x, w_hh, b_hh, h0] + ([c0] if c0 is not None else [])
    grads = torch.autograd.grad(loss, wrt)
    dWx = grads[0].numpy().reshape(T, B, G, 1, D)
    dR = grads[1].numpy().reshape(G, D, D).transpose(2, 0, 1)[None]  # [g,e,d] -> [1,d,g,e]
    db = grads[2].numpy().reshape(1, G, D)
    dh0 = grads[3].numpy().reshape(B, 1, D)
    dc0 = grads[4].numpy().reshape(B, 1, D) if c0 is not None else None
    return out.detach().numpy().reshape(T, B, 1, D), (cn.detach().numpy().reshape(B, 1, D) if cn is not None else None), \
        dWx, dR, db, dh0, dc0


@pytest.mark.parametrize("kind,cell", [("lstm", CELL_LSTM), ("gru", CELL_GRU), ("elman", CELL_ELMAN)])
def test_matches_torch_cpu_library_cell_fp64(kind, cell):
    """Catches: wrong gate order, transposed R, GRU bias outside the r-product, z applied to the wrong
    term, any wrong Jacobian term, the time index of dR / R^T dg."""
    T, B, NH, D = 7, 3, 1, 5
    Wx, R, b, s0, dH = _rand(cell, T, B, NH, D, seed=11)
    st = oracle.fwd(cell, Wx, R, b, s0)
    dWx, dR, db, ds0 = oracle.bwd(cell, Wx, R, b, st, dH)
    h_ref, c_ref, dWx_ref, dR_ref, db_ref, dh0_ref, dc0_ref = _torch_rnn_reference(kind, Wx, R, b, s0, dH)
    np.testing.assert_allclose(st[1:, 0], h_ref, rtol=1e-12, atol=1e-13)
    if c_ref is not None:
        np.testing.assert_allclose(st[T, 1], c_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dWx, dWx_ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dR, dR_ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(db, db_ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(ds0[0], dh0_ref, rtol=1e-10, atol=1e-12)
    if dc0_ref is not None:
        np.testing.assert_allclose(ds0[1], dc0_ref, rtol=1e-10, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# sLSTM: the stabilized recurrence equals the unstabilized one (different formula, torch autograd)
# ----------------------------------------------------------------------------------------------
def _slstm_unstabilized_torch(Wx, R, b, s0, dH):
    """c~_t = sig(f) c~_{t-1} + e^i tanh z,  n~_t = sig(f) n~_{t-1} + e^i,  h = sig(o) c~/n~ with
    c~_0 = c_0 e^{m_0}, n~_0 = n_0 e^{m_0}; no stabilizer anywhere.  Multi-head via einsum."""
    T, B, G, NH, D = Wx.shape
    Wx_t = torch.tensor(Wx, requires_grad=True)
    R_t = torch.tensor(R, requires_grad=True)
    b_t = torch.tensor(b, requires_grad=True)
    h = torch.tensor(s0[0], requires_grad=True)
    c0 = torch.tensor(s0[1], requires_grad=True)
    n0 = torch.tensor(s0[2], requires_grad=True)
    m0 = torch.tensor(s0[3])
    h0 = h
    c, n = c0 * torch.exp(m0), n0 * torch.exp(m0)
    hs = []
    for t in range(T):
        pre = Wx_t[t] + torch.einsum("bnd,ndge->bgne", h, R_t) + b_t.permute(1, 0, 2)[None]
        i, f, z, o = pre[:, 0], pre[:, 1], pre[:, 2], pre[:, 3]
        c = torch.sigmoid(f) * c + torch.exp(i) * torch.tanh(z)
        n = torch.sigmoid(f) * n + torch.exp(i)
        h = torch.sigmoid(o) * c / n
        hs.append(h)
    hs = torch.stack(hs)
    loss = (hs * torch.tensor(dH)).sum()
    g = torch.autograd.grad(loss, [Wx_t, R_t, b_t, h0, c0, n0])
    return hs.detach().numpy(), c.detach().numpy(), n.detach().numpy(), [x.numpy() for x in g]


def test_slstm_stabilized_equals_unstabilized_and_autograd():
    """Catches: wrong m recursion, swapped exp arguments, missing normalizer term, wrong sign in dn,
    missing sig(-f) factor in df, gradient leaking through m."""
    T, B, NH, D = 6, 2, 2, 4
    Wx, R, b, s0, dH = _rand(CELL_SLSTM, T, B, NH, D, seed=5)
    st = oracle.fwd(CELL_SLSTM, Wx, R, b, s0)
    dWx, dR, db, ds0 = oracle.bwd(CELL_SLSTM, Wx, R, b, st, dH)
    hs, cT, nT, (dWx_r, dR_r, db_r, dh0_r, dc0_r, dn0_r) = _slstm_unstabilized_torch(Wx, R, b, s0, dH)
    np.testing.assert_allclose(st[1:, 0], hs, rtol=1e-11, atol=1e-13)
    # c_t = c~_t e^{-m_t}, n_t = n~_t e^{-m_t}
    np.testing.assert_allclose(st[T, 1] * np.exp(st[T, 3]), cT, rtol=1e-11)
    np.testing.assert_allclose(st[T, 2] * np.exp(st[T, 3]), nT, rtol=1e-11)
    np.testing.assert_allclose(dWx, dWx_r, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dR, dR_r, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(db, db_r, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(ds0[0], dh0_r, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(ds0[1], dc0_r, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(ds0[2], dn0_r, rtol=1e-9, atol=1e-12)
    assert np.all(ds0[3] == 0.0)


def test_slstm_stabilizer_shift_invariance():
    """(c0, n0, m0) -> (c0 e^-a, n0 e^-a, m0 + a) leaves every h_t unchanged."""
    T, B, NH, D = 5, 2, 2, 3
    Wx, R, b, s0, _ = _rand(CELL_SLSTM, T, B, NH, D, seed=8)
    a = 0.7
    s0b = s0.copy()
    s0b[1] *= math.exp(-a)
    s0b[2] *= math.exp(-a)
    s0b[3] += a
    h1 = oracle.fwd(CELL_SLSTM, Wx, R, b, s0)[1:, 0]
    h2 = oracle.fwd(CELL_SLSTM, Wx, R, b, s0b)[1:, 0]
    np.testing.assert_allclose(h1, h2, rtol=1e-12, atol=1e-14)


def test_slstm_large_input_gate_is_stable():
    """The whole point of m: pre-activations of +-200 must neither overflow nor produce NaN, and
    with R = 0 and constant inputs h stays sig(o) tanh(z)."""
    T, B, NH, D = 8, 1, 1, 2
    Wx = np.zeros((T, B, 4, NH, D))
    Wx[:, :, 0] = 200.0
    Wx[:, :, 1, :, 1] = -200.0
    Wx[:, :, 2] = 0.3
    Wx[:, :, 3] = -0.4
    st = oracle.fwd(CELL_SLSTM, Wx, np.zeros((NH, D, 4, D)), np.zeros((NH, 4, D)))
    assert np.all(np.isfinite(st))
    np.testing.assert_allclose(st[1:, 0], math.tanh(0.3) / (1 + math.exp(0.4)), rtol=1e-12)


def test_slstm_saturated_gates_match_the_unstabilized_recurrence():
    """The synthetic "large_mix" recipe of the GPU parity tests (pre-activations shifted by 0, +-50, +-100, +-200): in
    float64 exp(+-200) is still representable, so over a few steps the unstabilized recurrence is computable and must give
    the same h.  Catches a stabilizer that is only right for small values (wrong max argument, lost log sig(f) for large |f|)."""
    from paper_2412_07752_amd import synth
    w = synth.Workload("sat", CELL_SLSTM, 3, 3, 2, 16, "f32", False, bias="forget3", init="uniform0.1", seed=3, wx="large_mix")
    inp = synth.make_inputs(w)
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    Wx, R, b, s0 = f64(inp["Wx"]), f64(inp["R"]), f64(inp["b"]), f64(inp["states0"])
    assert np.abs(Wx).max() > 150.0
    st = oracle.fwd(CELL_SLSTM, Wx, R, b, s0)
    assert np.all(np.isfinite(st))
    h, c, n = s0[0].copy(), s0[1] * np.exp(s0[3]), s0[2] * np.exp(s0[3])
    sg = lambda v: 1.0 / (1.0 + np.exp(-v))
    for t in range(w.T):
        pre = Wx[t] + np.einsum("bnd,ndge->bgne", h, R) + b.transpose(1, 0, 2)[None]
        i, f, z, o = pre[:, 0], pre[:, 1], pre[:, 2], pre[:, 3]
        c = sg(f) * c + np.exp(i) * np.tanh(z)
        n = sg(f) * n + np.exp(i)
        h = sg(o) * c / n
        assert np.all(np.isfinite(c)) and np.all(n > 0)
        np.testing.assert_allclose(st[t + 1, 0], h, rtol=1e-9, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# closed forms with R = 0 and constant inputs
# ----------------------------------------------------------------------------------------------
def test_closed_forms_R_zero_constant_inputs():
    """LSTM: c_T = sig(i) tanh(z) (1 - sig(f)^T)/(1 - sig(f)).  sLSTM: h_t = sig(o) tanh(z) for all t.
    GRU: h_T = tanh(x_n + sig(r) b_n) (1 - sig(z)^T).  Catches dropped terms and wrong carries."""
    T, B, NH, D = 9, 2, 2, 3
    sg = lambda v: 1.0 / (1.0 + math.exp(-v))
    pi, pf, pz, po = 0.3, 1.1, -0.7, 0.45
    Wx = np.zeros((T, B, 4, NH, D))
    Wx[:, :, 0], Wx[:, :, 1], Wx[:, :, 2], Wx[:, :, 3] = pi, pf, pz, po
    R0, b0 = np.zeros((NH, D, 4, D)), np.zeros((NH, 4, D))
    st = oracle.fwd(CELL_LSTM, Wx, R0, b0)
    for t in range(1, T + 1):
        c = sg(pi) * math.tanh(pz) * (1 - sg(pf) ** t) / (1 - sg(pf))
        np.testing.assert_allclose(st[t, 1], c, rtol=1e-12)
        np.testing.assert_allclose(st[t, 0], sg(po) * math.tanh(c), rtol=1e-12)
    st = oracle.fwd(CELL_SLSTM, Wx, R0, b0)
    np.testing.assert_allclose(st[1:, 0], sg(po) * math.tanh(pz), rtol=1e-12)
    # unstabilized normalizer: n~_t = e^i (1 - sig(f)^t)/(1 - sig(f)) = n_t e^{m_t}
    for t in range(1, T + 1):
        np.testing.assert_allclose(st[t, 2] * np.exp(st[t, 3]), math.exp(pi) * (1 - sg(pf) ** t) / (1 - sg(pf)), rtol=1e-12)
    pr, pzz, pn, bn = 0.2, 0.9, -0.3, 0.8
    Wx3 = np.zeros((T, B, 3, NH, D))
    Wx3[:, :, 0], Wx3[:, :, 1], Wx3[:, :, 2] = pr, pzz, pn
    b3 = np.zeros((NH, 3, D))
    b3[:, 2] = bn
    st = oracle.fwd(CELL_GRU, Wx3, np.zeros((NH, D, 3, D)), b3)
    for t in range(1, T + 1):
        np.testing.assert_allclose(st[t, 0], math.tanh(pn + sg(pr) * bn) * (1 - sg(pzz) ** t), rtol=1e-12)


# ----------------------------------------------------------------------------------------------
# hand-worked rational examples (tests/golden)
# ----------------------------------------------------------------------------------------------
def test_hand_worked_examples():
    ln2, ln3 = math.log(2.0), math.log(3.0)
    g = _read_golden("gru_hand_example.txt")
    Wx = np.array([[0.0, -ln3, ln2], [0.0, 0.0, ln3 - 0.45]]).reshape(2, 1, 3, 1, 1)
    R = np.array([0.0, 0.0, 2.0]).reshape(1, 1, 3, 1)
    st = oracle.fwd(CELL_GRU, Wx, R, np.zeros((1, 3, 1)))
    np.testing.assert_allclose([st[1, 0].item(), st[2, 0].item()], [g["h_1"], g["h_2"]], rtol=1e-13)

    g = _read_golden("gru4_hand_example.txt")
    Wx = np.array([[-ln3, ln3, ln2 - 0.45, ln2], [0.0, 0.0, ln3 - 0.4, ln3 - 0.9]]).reshape(2, 1, 4, 1, 1)
    R = np.array([0.0, 0.0, 0.0, 2.0]).reshape(1, 1, 4, 1)
    st = oracle.fwd(CELL_GRU4, Wx, R, np.zeros((1, 4, 1)))
    np.testing.assert_allclose([st[1, 0].item(), st[2, 0].item()], [g["h_1"], g["h_2"]], rtol=1e-13)

    g = _read_golden("slstm_hand_example.txt")
    Wx = np.array([[0.0, 0.0, ln2, ln3], [ln2, 0.0, ln3 - 0.9, 0.0]]).reshape(2, 1, 4, 1, 1)
    R = np.array([0.0, 0.0, 2.0, 0.0]).reshape(1, 1, 4, 1)
    st = oracle.fwd(CELL_SLSTM, Wx, R, np.zeros((1, 4, 1)))
    for t in (1, 2):
        for s, nm in enumerate("hcnm"):
            np.testing.assert_allclose(st[t, s].item(), g[f"{nm}_{t}"], rtol=1e-13, atol=1e-15)

    g = _read_golden("lstm_hand_example.txt")
    Wx = np.array([[ln3, 0.0, ln2, 0.0], [-ln3, ln3, ln3, 0.0]]).reshape(2, 1, 4, 1, 1)
    st = oracle.fwd(CELL_LSTM, Wx, np.zeros((1, 1, 4, 1)), np.zeros((1, 4, 1)))
    np.testing.assert_allclose([st[1, 1].item(), st[2, 1].item()], [g["c_1"], g["c_2"]], rtol=1e-13)


# ----------------------------------------------------------------------------------------------
# head-wise block-diagonal R (Sec. 4.2): NH heads == one dense RNN with block-diagonal R
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cell", CELLS)
def test_heads_equal_block_diagonal_dense(cell):
    """Catches any head/unit index mix-up in Wx, R, b, states and in the gradients."""
    T, B, NH, D = 4, 3, 3, 4
    Wx, R, b, s0, dH = _rand(cell, T, B, NH, D, seed=21)
    G, S = oracle.num_gates(cell), oracle.num_states(cell)
    st = oracle.fwd(cell, Wx, R, b, s0)
    dWx, dR, db, ds0 = oracle.bwd(cell, Wx, R, b, st, dH)
    H = NH * D
    Rd = np.zeros((1, H, G, H))
    for n in range(NH):
        Rd[0, n * D:(n + 1) * D, :, n * D:(n + 1) * D] = R[n]
    Wxd = Wx.reshape(T, B, G, 1, H)
    bd = b.transpose(1, 0, 2).reshape(1, G, H)
    s0d = s0.reshape(S, B, 1, H)
    std = oracle.fwd(cell, Wxd, Rd, bd, s0d)
    np.testing.assert_allclose(std.reshape(st.shape), st, rtol=1e-12, atol=1e-14)
    dWxd, dRd, dbd, ds0d = oracle.bwd(cell, Wxd, Rd, bd, std, dH.reshape(T, B, 1, H))
    np.testing.assert_allclose(dWxd.reshape(dWx.shape), dWx, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dbd.reshape(G, NH, D).transpose(1, 0, 2), db, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(ds0d.reshape(ds0.shape), ds0, rtol=1e-11, atol=1e-13)
    for n in range(NH):
        np.testing.assert_allclose(dRd[0, n * D:(n + 1) * D, :, n * D:(n + 1) * D], dR[n], rtol=1e-11, atol=1e-13)
    # and every head alone equals a single-head run on its slice
    for n in range(NH):
        st1 = oracle.fwd(cell, Wx[:, :, :, n:n + 1], R[n:n + 1], b[n:n + 1], s0[:, :, n:n + 1])
        np.testing.assert_allclose(st1, st[:, :, :, n:n + 1], rtol=1e-13, atol=1e-15)


# ----------------------------------------------------------------------------------------------
# backward against central finite differences of the forward (Sec. 4)
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cell", CELLS)
def test_backward_matches_finite_differences(cell):
    """L = sum_t <dH_t, h_t>.  Every entry of Wx, R, b, h0, c0, n0 is perturbed.  The stabilizer's
    initial value is excluded: its gradient is zero by convention (m is a stop-gradient quantity)."""
    T, B, NH, D = 3, 2, 2, 3
    Wx, R, b, s0, dH = _rand(cell, T, B, NH, D, seed=3, rscale=1.0)
    S = oracle.num_states(cell)

    def loss(Wx_, R_, b_, s0_):
        return float((oracle.fwd(cell, Wx_, R_, b_, s0_)[1:, 0] * dH).sum())

    st = oracle.fwd(cell, Wx, R, b, s0)
    dWx, dR, db, ds0 = oracle.bwd(cell, Wx, R, b, st, dH)
    eps = 1e-6
    args = [Wx, R, b, s0]
    for k, (arr, grad) in enumerate(zip(args, [dWx, dR, db, ds0])):
        fd = np.zeros_like(arr)
        flat = arr.reshape(-1)
        for j in range(flat.size):
            if k == 3 and cell == CELL_SLSTM and j // (B * NH * D) == 3:
                continue
            old = flat[j]
            flat[j] = old + eps
            lp = loss(*args)
            flat[j] = old - eps
            lm = loss(*args)
            flat[j] = old
            fd.reshape(-1)[j] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(grad, fd, rtol=2e-6, atol=2e-8, err_msg=f"cell {cell} arg {k}")
    assert S == ds0.shape[0]


# ----------------------------------------------------------------------------------------------
# invariants
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cell", CELLS)
def test_time_chunks_compose_and_grad_identities(cell):
    T, B, NH, D = 6, 3, 2, 4
    Wx, R, b, s0, dH = _rand(cell, T, B, NH, D, seed=17)
    G = oracle.num_gates(cell)
    st = oracle.fwd(cell, Wx, R, b, s0)
    # run 4 steps, then 2 more from the saved states
    a = oracle.fwd(cell, Wx[:4], R, b, s0)
    c = oracle.fwd(cell, Wx[4:], R, b, a[4])
    np.testing.assert_allclose(np.concatenate([a, c[1:]]), st, rtol=1e-13, atol=1e-15)
    dWx, dR, db, ds0 = oracle.bwd(cell, Wx, R, b, st, dH)
    # the same for the backward: last chunk first, its dstates0 is the first chunk's dstates_last
    dWx2, dR2, db2, dsm = oracle.bwd(cell, Wx[4:], R, b, st[4:], dH[4:])
    dWx1, dR1, db1, ds0c = oracle.bwd(cell, Wx[:4], R, b, st[:5], dH[:4], dsm)
    np.testing.assert_allclose(np.concatenate([dWx1, dWx2]), dWx, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(dR1 + dR2, dR, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(db1 + db2, db, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(ds0c, ds0, rtol=1e-11, atol=1e-14)
    # db = sum over t, b of the recurrent-side gate gradient (eq. (6)); equals sum of dWx except GRU gate n
    summed = dWx.sum(axis=(0, 1)).transpose(1, 0, 2)
    upto = G if cell != CELL_GRU else 2
    np.testing.assert_allclose(summed[:, :upto], db[:, :upto], rtol=1e-11, atol=1e-14)
    if cell == CELL_GRU:
        assert not np.allclose(summed[:, 2], db[:, 2])
    # linear in dH
    dWx3, dR3, _, _ = oracle.bwd(cell, Wx, R, b, st, 2.5 * dH)
    np.testing.assert_allclose(dWx3, 2.5 * dWx, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dR3, 2.5 * dR, rtol=1e-12, atol=1e-14)
    # batch permutation equivariance
    perm = np.array([2, 0, 1])
    stp = oracle.fwd(cell, Wx[:, perm], R, b, s0[:, perm])
    np.testing.assert_allclose(stp, st[:, :, perm], rtol=1e-13, atol=1e-15)


def test_zero_initial_state_is_default_and_T0():
    for cell in CELLS:
        Wx, R, b, _, _ = _rand(cell, 3, 2, 1, 4, seed=1, with_s0=False)
        S = oracle.num_states(cell)
        a = oracle.fwd(cell, Wx, R, b, None)
        z = oracle.fwd(cell, Wx, R, b, np.zeros((S, 2, 1, 4)))
        assert np.array_equal(a, z)
        assert np.all(np.isfinite(a))
        e = oracle.fwd(cell, Wx[:0], R, b, None)
        assert e.shape == (1, S, 2, 1, 4) and np.all(e == 0)


# ----------------------------------------------------------------------------------------------
# clipping of the recurrent gradient term (Sec. 4.1)
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cell", CELLS)
def test_recurrent_clip_single_step_is_clamp_of_unclipped(cell):
    """T = 1: nothing upstream is affected by the clip, so dstates0[h] = direct path + clamp(R^T dg_1) with the
    unclipped dg_1.  Catches: clip applied to the wrong term (direct path, dH, dWx), wrong bounds, clip ignored."""
    T, B, NH, D = 1, 3, 2, 6
    Wx, R, b, s0, dH = _rand(cell, T, B, NH, D, seed=21, rscale=3.0)
    st = oracle.fwd(cell, Wx, R, b, s0)
    dWx0, dR0, db0, ds0_0 = oracle.bwd(cell, Wx, R, b, st, dH)
    # recurrent term alone: R^T dg_1 = dstates0[h] of the unclipped run minus the direct path, which is what a run
    # with the recurrent term cut (clip 0) returns
    _, _, _, ds0_cut = oracle.bwd(cell, Wx, R, b, st, dH, recurrent_clip=0.0)
    rec = ds0_0[0] - ds0_cut[0]
    assert np.abs(rec).max() > 0.2
    c = 0.1
    dWx, dR, db, ds0 = oracle.bwd(cell, Wx, R, b, st, dH, recurrent_clip=c)
    np.testing.assert_allclose(ds0[0], ds0_cut[0] + np.clip(rec, -c, c), rtol=1e-12, atol=1e-14)
    for a, ref in ((dWx, dWx0), (dR, dR0), (db, db0), (ds0[1:], ds0_0[1:])):
        np.testing.assert_array_equal(a, ref)
    big = oracle.bwd(cell, Wx, R, b, st, dH, recurrent_clip=1e30)
    for a, ref in zip(big, (dWx0, dR0, db0, ds0_0)):
        np.testing.assert_array_equal(a, ref)


@pytest.mark.parametrize("cell", CELLS)
def test_recurrent_clip_composes_over_time(cell):
    """BPTT over T steps with the clip == T single-step backward passes chained through dstates_last, each of
    them clipping its own recurrent term (dR, db summed).  Catches: clip applied once at the end, or to the carried
    gradient instead of to the recurrent term of each step."""
    T, B, NH, D = 5, 2, 2, 4
    Wx, R, b, s0, dH = _rand(cell, T, B, NH, D, seed=22, rscale=3.0)
    st = oracle.fwd(cell, Wx, R, b, s0)
    c = 0.05
    dWx, dR, db, ds0 = oracle.bwd(cell, Wx, R, b, st, dH, recurrent_clip=c)
    carry, dR_sum, db_sum = None, 0.0, 0.0
    for t in range(T, 0, -1):
        g = oracle.bwd(cell, Wx[t - 1:t], R, b, st[t - 1:t + 1], dH[t - 1:t], carry, recurrent_clip=c)
        np.testing.assert_allclose(dWx[t - 1], g[0][0], rtol=1e-12, atol=1e-14)
        dR_sum, db_sum, carry = dR_sum + g[1], db_sum + g[2], g[3]
    np.testing.assert_allclose(dR, dR_sum, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(db, db_sum, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(ds0, carry, rtol=1e-12, atol=1e-14)
    unclipped = oracle.bwd(cell, Wx, R, b, st, dH)
    assert np.abs(dWx - unclipped[0]).max() > 1e-3   # the clip did bite


def test_recurrent_cut_equals_library_lstm_cell_with_detached_h():
    """clip = 0 removes the path through R from the backward pass: the same as autograd through torch's CPU LSTMCell
    (float64) when the hidden state entering the cell is detached.  dR and db still see every step."""
    T, B, NH, D = 6, 3, 1, 5
    Wx, R, b, s0, dH = _rand(CELL_LSTM, T, B, NH, D, seed=23)
    st = oracle.fwd(CELL_LSTM, Wx, R, b, s0)
    dWx, dR, db, ds0 = oracle.bwd(CELL_LSTM, Wx, R, b, st, dH, recurrent_clip=0.0)
    G = 4
    x = torch.tensor(Wx.reshape(T, B, G * D), requires_grad=True)
    w_hh = torch.tensor(np.ascontiguousarray(R[0].transpose(1, 2, 0)).reshape(G * D, D), requires_grad=True)
    b_hh = torch.tensor(b[0].reshape(G * D), requires_grad=True)
    h0 = torch.tensor(s0[0].reshape(B, D), requires_grad=True)
    c0 = torch.tensor(s0[1].reshape(B, D), requires_grad=True)
    cell = torch.nn.LSTMCell(G * D, D).double()
    params = {"weight_ih": torch.eye(G * D, dtype=torch.float64), "weight_hh": w_hh,
              "bias_ih": torch.zeros(G * D, dtype=torch.float64), "bias_hh": b_hh}
    h, c, loss = h0, c0, 0.0
    dHt = torch.tensor(dH.reshape(T, B, D))
    for t in range(T):
        h, c = torch.func.functional_call(cell, params, (x[t], (h.detach() if t > 0 else h * 0 + h.detach(), c)))
        loss = loss + (h * dHt[t]).sum()
    g = torch.autograd.grad(loss, [x, w_hh, b_hh, c0])
    np.testing.assert_allclose(dWx, g[0].numpy().reshape(T, B, G, 1, D), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dR, g[1].numpy().reshape(G, D, D).transpose(2, 0, 1)[None], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(db, g[2].numpy().reshape(1, G, D), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(ds0[1], g[3].numpy().reshape(B, 1, D), rtol=1e-10, atol=1e-12)
    np.testing.assert_array_equal(ds0[0], 0.0)   # h_0 reaches the loss only through R
