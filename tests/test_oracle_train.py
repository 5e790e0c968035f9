"""Pins for the oracle's training step (oracle/train.py)."""
import numpy as np
import torch

from oracle import dense, train
from paper_1902_04610_amd import synth


def make(dims, M, seed, exact=False):
    rng = np.random.default_rng(seed)
    if exact:      # small multiples of 1/4: every product, sum and activation is a bf16 number
        Wm = [(rng.integers(-2, 3, (K, N)) / 4.0).astype(np.float32) for K, N in zip(dims[:-1], dims[1:])]
        X = (rng.integers(-2, 3, (M, dims[0])) / 4.0).astype(np.float32)
    else:
        Wm = [(rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32) for K, N in zip(dims[:-1], dims[1:])]
        X = rng.standard_normal((M, dims[0])).astype(np.float32)
    Wb = [synth.f32_to_bf16_bits(w) for w in Wm]
    labels = rng.integers(0, dims[-1], M).astype(np.int32)
    return synth.f32_to_bf16_bits(X), labels, Wm, Wb


def torch_reference(Xb, labels, Wb):
    """Double-precision autograd on the same bf16-valued weights and inputs,
    without the intermediate roundings."""
    W = [torch.tensor(synth.bf16_bits_to_f32(w), dtype=torch.float64, requires_grad=True) for w in Wb]
    h = torch.tensor(synth.bf16_bits_to_f32(Xb), dtype=torch.float64)
    for l, w in enumerate(W):
        h = h @ w
        if l + 1 < len(W):
            h = torch.relu(h)
    loss = torch.nn.functional.cross_entropy(h, torch.tensor(labels, dtype=torch.long))
    loss.backward()
    return loss.item(), h.detach().numpy(), [w.grad.numpy() for w in W]


def test_gradients_match_double_autograd():
    dims, M = (24, 40, 32, 10), 16
    Xb, labels, Wm, Wb = make(dims, M, 0)
    ref_loss, ref_logits, ref_grads = torch_reference(Xb, labels, Wb)
    loss, logits, grads = train.train_step(Xb, labels, [w.copy() for w in Wm], [w.copy() for w in Wb], 0.0)
    assert abs(loss - ref_loss) < 2e-2 * abs(ref_loss)
    assert np.abs(logits - ref_logits).max() < 2e-2 * np.abs(ref_logits).max()
    for g, r in zip(grads, ref_grads):
        assert g.shape == r.shape
        # bf16 rounding of activations and of the incoming gradient: 2^-8 relative each
        assert np.abs(g - r).max() < 3e-2 * np.abs(r).max()


def test_exact_point_matches_autograd_tightly():
    """With inputs on a coarse grid nothing is rounded in the forward pass, so
    the loss and logits equal the double computation to float precision."""
    dims, M = (4, 4, 3), 4
    Xb, labels, Wm, Wb = make(dims, M, 1, exact=True)
    ref_loss, ref_logits, ref_grads = torch_reference(Xb, labels, Wb)
    loss, logits, grads = train.train_step(Xb, labels, [w.copy() for w in Wm], [w.copy() for w in Wb], 0.0)
    assert np.array_equal(logits, ref_logits.astype(np.float32))
    assert abs(loss - ref_loss) < 1e-12
    for g, r in zip(grads, ref_grads):
        assert np.abs(g - r).max() < 6e-3 * max(np.abs(r).max(), 1e-9)      # only bf16(dZ) differs


def test_finite_differences_of_the_loss():
    dims, M = (6, 5, 4), 3
    Xb, labels, Wm, Wb = make(dims, M, 4, exact=True)
    # the point must not sit on a ReLU kink, where a central difference is meaningless
    assert ((synth.bf16_bits_to_f32(Xb).astype(np.float64) @ Wm[0]) != 0).all()
    _, _, grads = train.train_step(Xb, labels, [w.copy() for w in Wm], [w.copy() for w in Wb], 0.0)

    def loss_at(Ws):
        h = synth.bf16_bits_to_f32(Xb).astype(np.float64)
        for l, w in enumerate(Ws):
            h = h @ w
            if l + 1 < len(Ws):
                h = np.maximum(h, 0)
        h = h - h.max(axis=1, keepdims=True)
        logp = h - np.log(np.exp(h).sum(axis=1, keepdims=True))
        return -logp[np.arange(M), labels].mean()

    base = [w.astype(np.float64) for w in Wm]
    for l, (k, n) in [(0, (1, 2)), (0, (5, 0)), (1, (0, 3)), (1, (4, 1))]:
        up, dn = [w.copy() for w in base], [w.copy() for w in base]
        up[l][k, n] += 1e-4
        dn[l][k, n] -= 1e-4
        fd = (loss_at(up) - loss_at(dn)) / 2e-4
        assert abs(fd - grads[l][k, n]) < 1e-2 * max(abs(fd), 1e-2), (l, k, n, fd, grads[l][k, n])


def test_sgd_semantics():
    dims, M = (16, 24, 8), 8
    Xb, labels, Wm, Wb = make(dims, M, 3)
    keep_m, keep_b = [w.copy() for w in Wm], [w.copy() for w in Wb]
    _, _, grads = train.train_step(Xb, labels, Wm, Wb, 0.0)
    for a, b in zip(Wm, keep_m):
        assert np.array_equal(a, b)                       # lr = 0 leaves the weights bit-identical
    for a, b in zip(Wb, keep_b):
        assert np.array_equal(a, b)
    lr = np.float32(0.05)
    _, _, grads = train.train_step(Xb, labels, Wm, Wb, lr)
    for w, k, g in zip(Wm, keep_m, grads):
        assert np.array_equal(w, k - lr * g)              # float multiply, float subtract
    for w, b in zip(Wm, Wb):
        assert np.array_equal(b, synth.f32_to_bf16_bits(w))
    # the loss goes down over a few steps with a sane learning rate
    losses = [train.train_step(Xb, labels, Wm, Wb, lr)[0] for _ in range(5)]
    assert losses[-1] < losses[0]


def test_relu_mask_uses_stored_activation():
    # one hidden unit that is exactly zero after ReLU: no gradient flows through it
    Xb = synth.f32_to_bf16_bits(np.array([[1.0, 1.0]], np.float32))
    W1 = np.array([[1.0, -1.0], [1.0, -1.0]], np.float32)      # hidden = [2, 0 after relu]
    W2 = np.array([[1.0, 0.0], [5.0, -5.0]], np.float32)
    Wm, Wb = [W1.copy(), W2.copy()], [synth.f32_to_bf16_bits(W1), synth.f32_to_bf16_bits(W2)]
    _, _, grads = train.train_step(Xb, np.array([0], np.int32), Wm, Wb, 0.0)
    assert (grads[0][:, 1] == 0).all() and (grads[0][:, 0] != 0).all()
    assert (grads[1][1, :] == 0).all()                          # dead unit: zero activation
