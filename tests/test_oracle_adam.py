"""Pin of the oracle's Adam step against a numerical library's optimizer (PyTorch CPU, fp64) and its closed
forms: the first step moves every weight by lr * sign(g) (up to eps), zero gradients leave the weights alone."""
import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")


def test_adam_matches_library_optimizer_over_several_steps():
    rng = np.random.default_rng(0)
    W0 = rng.normal(0, 1, 500)
    grads = [rng.normal(0, 10.0 ** rng.integers(-3, 1), 500) for _ in range(6)]
    p = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    W, m, v = W0.copy(), np.zeros(500), np.zeros(500)
    for t, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g)
        opt.step()
        W, m, v = oracle.adam_step(W, g, m, v, 1e-2, t)
        np.testing.assert_allclose(W, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adam_closed_forms():
    g = np.array([3.0, -0.5, 1e-3, -7.0])
    W, m, v = oracle.adam_step(np.zeros(4), g, np.zeros(4), np.zeros(4), 0.1, 1, eps=0.0)
    np.testing.assert_allclose(W, -0.1 * np.sign(g), rtol=1e-12)          # bias-corrected first step
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)
    W2, _, _ = oracle.adam_step(np.ones(4), np.zeros(4), np.zeros(4), np.zeros(4), 0.1, 1)
    np.testing.assert_array_equal(W2, np.ones(4))
