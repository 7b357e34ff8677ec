"""CPU pins of the gate-predictor oracle: a library's sigmoid(linear) and its reverse-mode gradients, a closed form."""
import numpy as np
import pytest

from oracle.gate import gate_backward, gate_forward


def test_gate_matches_library_linear_sigmoid_and_autograd():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    x, w, b = rng.standard_normal((37, 24)), rng.standard_normal((24, 12)) * 0.4, rng.standard_normal(12)
    dg = rng.standard_normal((37, 12))
    tx, tw, tb = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, w, b))
    g = torch.sigmoid(torch.nn.functional.linear(tx, tw.T, tb))
    (g * torch.tensor(dg)).sum().backward()
    assert np.allclose(gate_forward(x, w, b), g.detach().numpy(), rtol=1e-13, atol=1e-13)
    dx, dw, db = gate_backward(x, w, gate_forward(x, w, b), dg)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(dw, tw.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(db, tb.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_gate_closed_forms():
    x = np.array([[1.0, 2.0]])
    assert np.allclose(gate_forward(x, np.zeros((2, 3)), np.zeros(3)), 0.5)          # sigmoid(0)
    w = np.array([[np.log(3.0)], [0.0]])
    assert np.allclose(gate_forward(x, w, np.zeros(1)), 0.75)                         # sigmoid(ln 3) = 3/4
    dx, dw, db = gate_backward(x, w, gate_forward(x, w, np.zeros(1)), np.ones((1, 1)))
    assert np.allclose(db, 0.75 * 0.25) and np.allclose(dw[:, 0], [0.1875, 0.375]) and np.allclose(dx, [[0.1875 * np.log(3.0), 0.0]])
