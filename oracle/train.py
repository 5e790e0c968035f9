"""CPU oracle for one training step of a hyper-parameter-tuning job.

TEST INFRASTRUCTURE ONLY.  Never imported by the product path.

The paper (Salus, arXiv 1902.04610, Section 2.1) describes training as a
forward pass, a backward pass that propagates gradients and a parameter update;
it fixes no arithmetic.  The workload fixes the rest: an MLP with ReLU between
layers and no biases, bf16 working weights with float master weights, softmax
cross-entropy averaged over the batch, plain SGD.  The step below is that
definition written out with the primitives of dense.c:

    H_0 = X                                  (bf16)
    Z_l = H_{l-1} . Wb_l                     (exact sum, rounded to float)
    H_l = bf16(relu(Z_l))         l < L
    loss, dZ_L = softmax_xent(Z_L, labels)   (mean over the batch)
    for l = L .. 1:
        G_l    = bf16(dZ_l)
        dW_l   = H_{l-1}^T . G_l
        dZ_{l-1} = (G_l . Wb_l^T) * [H_{l-1} > 0]      (l > 1; old Wb_l)
        Wm_l  <- Wm_l - lr * dW_l            (float multiply, float subtract)
        Wb_l  <- bf16(Wm_l)

Reading: the ReLU derivative is taken from the stored bf16 activation
(H > 0), which is what a backward pass has at hand.

The step is split into its two passes so that a test can hand the backward
pass the activations and logits another implementation produced: whether a
unit's derivative is 0 or 1 is decided by the sign of a stored activation, and
two forward passes that differ by one rounding can disagree on units that sit
within that rounding of zero.

Pins: tests/test_oracle_train.py (torch double autograd as a second opinion,
finite differences at a point where no rounding occurs, lr = 0).
"""
import numpy as np

from . import dense


def forward(Xb, Wb):
    """Returns (H, logits): H = [H_0 = X, H_1, ..., H_{L-1}] as bf16 bits."""
    L = len(Wb)
    H = [np.ascontiguousarray(Xb, np.uint16)]
    Z = None
    for l in range(L):
        act = dense.ACT_RELU if l + 1 < L else dense.ACT_NONE
        Z = dense.dense_bf16(H[l], Wb[l], act)          # relu already applied for hidden layers
        if l + 1 < L:
            H.append(dense.round_bf16(Z))
    return H, Z


def backward_update(H, logits, labels, Wm, Wb, lr):
    """Loss, gradients and the SGD update.  Wm (float32) and Wb (uint16) are
    updated IN PLACE.  Returns (loss, grads, G) with grads[l] the float dW_l and
    G[l] the bf16 gradient that entered layer l's backward products."""
    L = len(Wm)
    loss, dZ = dense.softmax_xent(logits, labels)
    grads, G = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        G[l] = dense.round_bf16(dZ)
        grads[l] = dense.dense_bwd_weight_bf16(H[l], G[l])
        if l > 0:
            dH = dense.dense_bwd_input_bf16(G[l], Wb[l])
            positive = dense.bf16_to_f32(H[l]) > 0
            dZ = np.where(positive, dH, np.float32(0)).astype(np.float32)
        dense.sgd_update(Wm[l], Wb[l], grads[l], lr)
    return loss, grads, G


def train_step(Xb, labels, Wm, Wb, lr):
    """Xb: (M, K0) bf16 bits; labels: (M,) int32; Wm: list of float32 (K, N)
    arrays, Wb: list of uint16 (K, N) arrays - both updated IN PLACE.
    Returns (loss, logits, grads) where grads are the float dW of every layer."""
    H, logits = forward(Xb, Wb)
    loss, grads, _ = backward_update(H, logits, labels, Wm, Wb, lr)
    return loss, logits, grads
