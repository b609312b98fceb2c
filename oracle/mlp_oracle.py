"""CPU oracle of the dense step -- TEST INFRASTRUCTURE (numpy, fp64).

Section 2.1: y^ = NN_{w_nn}(lookup_{w_emb}(x^ID), x^NID): the network takes the looked-up (pooled)
embeddings concatenated with the non-ID features.  Algorithm 2: forward of the mini-batch, backward for
F'^nn and F'^emb (the gradient of the loss w.r.t. the embedding activations, sent back to the embedding
side), update w^nn <- w^nn - Omega^nn(F'^nn).  The network is a feed-forward ReLU net with one logit
and the loss is binary cross-entropy on the logit; Omega^nn is plain SGD.  Readings where the paper is
silent: the loss is the MEAN over the batch (Algorithm 2 writes a sum; `loss_mean=False` gives it);
"bf16 MLP" means operands of every product are rounded to bf16 (inputs, weights, activations and the
back-propagated deltas as they are stored) while sums are exact here (fp32 on the GPU); master weights
and their update are fp32; the rounding is treated as the identity in the backward pass.
"""
import numpy as np


def bf16(x):
    """fp32 -> bf16 (round to nearest even) -> fp64, elementwise."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


# ---- the stages of one step, each from its own inputs (operands already in storage precision) ----
def layer_forward(h_prev, W, b, q):
    """Stored activation of the next layer: q(relu(h_prev W + b)); also returns the pre-activation."""
    a = h_prev @ q(W) + np.asarray(b, dtype=np.float64)
    return q(np.maximum(a, 0.0)), a


def logit_loss(h_last, w_last, b_last, y, scale):
    """Logit z = h_last w + b, loss = scale * sum BCE(z, y), dz = d loss / d z = scale * (sigmoid(z) - y)."""
    z = (h_last @ w_last + np.asarray(b_last, dtype=np.float64)).reshape(-1)
    loss = scale * np.sum(np.logaddexp(0.0, z) - y * z)
    dz = scale * (0.5 * (1.0 + np.tanh(0.5 * z)) - y)
    return z, loss, dz


def delta_from_logit(dz, w_last, h_last, q):
    """Delta at the input of the last layer: q(dz (x) w_last^T, kept where the stored activation is positive)."""
    return q(dz[:, None] * w_last.reshape(1, -1) * (h_last > 0))


def delta_back(delta, W, h_prev, q):
    """Delta one layer down: q((delta W^T) kept where the stored activation h_prev is positive)."""
    return q((delta @ q(W).T) * (h_prev > 0))


def weight_grad(h_prev, delta):
    """(dW, db) of the layer between h_prev and delta."""
    return h_prev.T @ delta, delta.sum(axis=0)


class MLP:
    def __init__(self, weights, biases, lr, loss_mean=True, rounding=True, delay=0):
        """weights[l]: fp32 [in_l, out_l]; biases[l]: fp32 [out_l]; the last layer has out = 1.
        delay > 0 models a fully asynchronous dense side (the comparison of section 3.1): step t works with
        weights that miss the gradients of the last `delay` steps (those of step t are applied at the beginning
        of step t + delay + 1)."""
        self.delay = int(delay)
        self.pending = []          # gradients computed but not applied yet, oldest first
        self.W = [np.array(w, dtype=np.float32) for w in weights]
        self.b = [np.array(b, dtype=np.float32) for b in biases]
        self.lr = np.float32(lr)
        self.loss_mean = loss_mean
        # storage rounding of every operand: through fp32 to bf16, or none at all (pure fp64, for the pins)
        self.q = (lambda x: bf16(np.asarray(x, dtype=np.float32))) if rounding else (
            lambda x: np.asarray(x, dtype=np.float64))

    def step(self, pooled, dense, labels, update=True):
        """One forward + backward (+ SGD update).  Returns (loss, d_pooled fp32 [B, P], grads) where grads is
        the list of (dW, db) in fp64."""
        q = self.q
        if self.delay and len(self.pending) == self.delay + 1:       # step t - delay - 1's gradients are due
            self._apply(self.pending.pop(0))
        B, P = pooled.shape
        y = np.asarray(labels, dtype=np.float64).reshape(B)
        h = [q(np.concatenate([pooled, dense], axis=1))]
        L = len(self.W)
        for l in range(L - 1):
            h.append(layer_forward(h[-1], self.W[l], self.b[l], q)[0])
        scale = 1.0 / B if self.loss_mean else 1.0
        _, loss, dz = logit_loss(h[-1], q(self.W[-1]), self.b[-1], y, scale)
        grads = [None] * L
        grads[L - 1] = (h[-1].T @ dz[:, None], np.array([dz.sum()]))
        delta = delta_from_logit(dz, q(self.W[-1]), h[-1], q)      # [B, width of the last hidden layer]
        for l in range(L - 2, -1, -1):
            grads[l] = weight_grad(h[l], delta)
            if l > 0:
                delta = delta_back(delta, self.W[l], h[l], q)
            else:
                d_x = delta @ q(self.W[0]).T                        # the input has no ReLU in front of it
        if update:
            if self.delay:
                self.pending.append(grads)
            else:
                self._apply(grads)
        return loss, d_x[:, :P].astype(np.float32), grads

    def _apply(self, grads):
        for l in range(len(self.W)):
            self.W[l] = (self.W[l].astype(np.float64) - float(self.lr) * grads[l][0]).astype(np.float32)
            self.b[l] = (self.b[l].astype(np.float64) - float(self.lr) * grads[l][1]).astype(np.float32)
