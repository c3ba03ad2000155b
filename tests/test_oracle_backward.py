"""Pins for the backward oracle: the derivatives must agree with central finite differences of
the forward oracle's plain layer definition (Sec. 2.1), with closed forms, and with reverse-mode
differentiation of the forward written with a tensor library."""
import math

import numpy as np
import pytest
import torch

from oracle import moe_backward as ob
from oracle import moe_layer as om
from oracle import planner as op


def _tiny(act, seed=3, T=14, d=6, f=5, E=4, k=2, N=2, c=3):
    rng = np.random.default_rng(seed)
    n1 = f * (2 if act == "swiglu" else 1)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    x = rng.standard_normal((T, d))
    w1 = rng.standard_normal((E, n1, d)) * 0.6
    w2 = rng.standard_normal((E, d, f)) * 0.6
    dy = rng.standard_normal((T, d))
    ids, gates = om.route(logits, k)
    t_e = np.bincount(ids.reshape(-1), minlength=E)
    r = op.allocate_replicas(t_e, N, c, 1)
    plan = np.array(op.place_mro(r, t_e, N, c), dtype=np.int32)
    off = np.array([(i * T) // N for i in range(N + 1)], dtype=np.int32)
    disp = om.plan_dispatch(ids, off, plan, E, N, c)
    return dict(logits=logits, x=x, w1=w1, w2=w2, dy=dy, ids=ids, gates=gates, plan=plan,
                disp=disp, act=act, k=k, E=E)


def _loss(c, x=None, w1=None, w2=None, gates=None):
    y = om.layer_output(c["x"] if x is None else x, c["ids"], c["gates"] if gates is None else gates,
                        c["w1"] if w1 is None else w1, c["w2"] if w2 is None else w2, c["act"])
    return float(np.sum(c["dy"] * y))


def _backward(c):
    d = c["disp"]
    return ob.layer_backward(c["dy"], c["x"], c["ids"], c["gates"], d["pair_to_row"], d["row_to_pair"],
                             d["slot_offsets"], c["plan"], c["w1"], c["w2"], c["act"])


def _fd(c, name, index, h=1e-5):
    base = c[name]
    plus, minus = base.copy(), base.copy()
    plus[index] += h
    minus[index] -= h
    return (_loss(c, **{name: plus}) - _loss(c, **{name: minus})) / (2 * h)


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_gradients_match_finite_differences_of_the_layer_definition(act):
    c = _tiny(act)
    g = _backward(c)
    rng = np.random.default_rng(17)
    checks = [("x", g["dx"]), ("w1", g["dw1"]), ("w2", g["dw2"]), ("gates", g["dgates"])]
    for name, grad in checks:
        assert grad.shape == c[name].shape
        flat = rng.choice(grad.size, size=min(40, grad.size), replace=False)
        for i in flat:
            index = np.unravel_index(i, grad.shape)
            ref = _fd(c, name, index)
            assert grad[index] == pytest.approx(ref, rel=2e-6, abs=2e-8), (name, index)


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_gradients_match_reverse_mode_autodiff(act):
    c = _tiny(act, seed=8, T=20, E=5, k=3, N=3, c=2)
    g = _backward(c)
    x = torch.tensor(c["x"], requires_grad=True)
    w1 = torch.tensor(c["w1"], requires_grad=True)
    w2 = torch.tensor(c["w2"], requires_grad=True)
    logits = torch.tensor(c["logits"].astype(np.float64), requires_grad=True)
    ids = torch.tensor(c["ids"].astype(np.int64))
    gates = torch.softmax(torch.gather(logits, 1, ids), dim=1)
    assert np.allclose(gates.detach().numpy(), c["gates"], rtol=1e-12)
    y = torch.zeros_like(x)
    for t in range(x.shape[0]):
        for kk in range(c["k"]):
            e = int(ids[t, kk])
            z = w1[e] @ x[t]
            if act == "gelu":
                h = torch.nn.functional.gelu(z)
            else:
                f = z.shape[0] // 2
                h = torch.nn.functional.silu(z[:f]) * z[f:]
            y[t] = y[t] + gates[t, kk] * (w2[e] @ h)
    (y * torch.tensor(c["dy"])).sum().backward()
    assert np.allclose(g["dx"], x.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["dw1"], w1.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(g["dw2"], w2.grad.numpy(), rtol=1e-10, atol=1e-12)
    dlogits = ob.route_backward(g["dgates"], c["gates"], c["ids"], c["E"])
    assert np.allclose(dlogits, logits.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_activation_derivatives_closed_forms_and_differences():
    assert ob.gelu_grad(np.array([0.0]))[0] == 0.5
    assert ob.silu_grad(np.array([0.0]))[0] == 0.5
    # gelu'(1) = Phi(1) + phi(1)
    assert ob.gelu_grad(np.array([1.0]))[0] == pytest.approx(0.8413447460685429 + 0.24197072451914337, rel=1e-14)
    # silu'(ln 3) = 3/4 (1 + ln3/4)
    assert ob.silu_grad(np.array([math.log(3.0)]))[0] == pytest.approx(0.75 * (1 + math.log(3.0) / 4), rel=1e-14)
    far = ob.gelu_grad(np.array([12.0, -12.0]))
    assert far[0] == pytest.approx(1.0, abs=1e-12) and abs(far[1]) < 1e-12
    v = np.linspace(-4, 4, 33)
    h = 1e-6
    assert np.allclose(ob.gelu_grad(v), (om.gelu(v + h) - om.gelu(v - h)) / (2 * h), rtol=1e-8, atol=1e-9)
    assert np.allclose(ob.silu_grad(v), (om.silu(v + h) - om.silu(v - h)) / (2 * h), rtol=1e-8, atol=1e-9)


def test_route_backward_against_differences_of_route_and_shift_invariance():
    rng = np.random.default_rng(2)
    T, E, k = 9, 7, 3
    logits = (rng.standard_normal((T, E)) * 2).astype(np.float32)
    ids, gates = om.route(logits, k)
    dg = rng.standard_normal((T, k))
    dl = ob.route_backward(dg, gates, ids, E)
    assert np.allclose(dl.sum(axis=1), 0.0, atol=1e-14)      # softmax ignores a common shift
    picked = np.zeros((T, E), dtype=bool)
    picked[np.arange(T)[:, None], ids] = True
    assert np.all(dl[~picked] == 0.0)
    h = 2.0 ** -10                                           # exactly representable steps in fp32
    for t, e in [(0, int(ids[0, 0])), (3, int(ids[3, 2])), (5, int(ids[5, 1])), (8, int(ids[8, 0]))]:
        up, dn = logits.copy(), logits.copy()
        up[t, e] += h
        dn[t, e] -= h
        iu, gu = om.route(up, k)
        idn, gd = om.route(dn, k)
        if not (np.array_equal(np.sort(iu[t]), np.sort(ids[t])) and np.array_equal(np.sort(idn[t]), np.sort(ids[t]))):
            continue                                         # the step changed the selection
        # gates are listed in descending-logit order; compare per expert
        def per_expert(i, g):
            out = np.zeros(E)
            out[i[t]] = g[t]
            return out
        dgt = np.zeros(E)
        dgt[ids[t]] = dg[t]
        ref = float(np.sum(dgt * (per_expert(iu, gu) - per_expert(idn, gd)))) / (2 * h)
        assert dl[t, e] == pytest.approx(ref, rel=1e-4, abs=1e-7)


def test_replica_sum_and_empty_slots():
    c = _tiny("gelu", seed=5)
    g = _backward(c)
    counts = np.diff(c["disp"]["slot_offsets"])
    for s, n in enumerate(counts):
        if n == 0:
            assert not g["dw1_slot"][s].any() and not g["dw2_slot"][s].any()
    for e in range(c["E"]):
        slots = [s for s, ee in enumerate(c["plan"]) if ee == e]
        assert np.allclose(g["dw2"][e], sum(g["dw2_slot"][s] for s in slots), rtol=1e-14, atol=1e-15)
    # rows outside every slot (none here) aside, dyp rows carry gate * dy of their pair
    p2r = c["disp"]["pair_to_row"].reshape(-1, c["k"])
    assert np.allclose(g["dyp"][p2r[4, 1]], c["gates"][4, 1] * c["dy"][4], rtol=1e-15)
