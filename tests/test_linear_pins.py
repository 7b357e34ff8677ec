"""CPU pins of the linear-projection oracle: a library's linear layer and its reverse-mode gradients, closed forms."""
import numpy as np
import pytest

from oracle.linear import linear_backward, linear_forward


def test_linear_matches_library_linear_and_autograd():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    x, w, b = rng.standard_normal((29, 24)), rng.standard_normal((40, 24)), rng.standard_normal(40)
    dy = rng.standard_normal((29, 40))
    tx, tw, tb = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, w, b))
    y = torch.nn.functional.linear(tx, tw, tb)
    (y * torch.tensor(dy)).sum().backward()
    assert np.allclose(linear_forward(x, w, b), y.detach().numpy(), rtol=1e-13, atol=1e-13)
    dx, dw, db = linear_backward(x, w, dy)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(dw, tw.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(db, tb.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(linear_forward(x, w), y.detach().numpy() - b, rtol=1e-12, atol=1e-12)


def test_linear_closed_forms():
    """A non-square weight picked so that a transposed operand or swapped gradient cannot pass."""
    x = np.array([[1.0, 2.0, 3.0]])
    w = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 1.0]])          # y0 = x0, y1 = x1 + x2
    assert np.allclose(linear_forward(x, w, np.array([10.0, 20.0])), [[11.0, 25.0]])
    dx, dw, db = linear_backward(x, w, np.array([[1.0, -1.0]]))
    assert np.allclose(dx, [[1.0, -1.0, -1.0]])
    assert np.allclose(dw, [[1.0, 2.0, 3.0], [-1.0, -2.0, -3.0]])
    assert np.allclose(db, [1.0, -1.0])
