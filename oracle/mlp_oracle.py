"""CPU oracle for the dense tower between pull and push (test infrastructure, not product code).

Plain numpy, float64 arithmetic.  What it follows:
  * the network: fully connected ReLU layers over the concatenated slot embeddings with one
    logit and a sigmoid cross-entropy loss (the CTR model of Section 2.1; the paper gives no layer
    sizes, the build's configuration does);
  * the train_mini-batch step of Algorithm 1: forward, backward, gradient of the pooled input;
  * the dense optimizer: Algorithm 2 (k-step Adam) exactly as in the sparse oracle - m0 = 0,
    v0 = eps, no bias correction, x -= lr m / sqrt(den), shared denominator frozen between merges,
    merge = mean of v, then mean of the stepped x.

Precision: the HIP path feeds bf16 operands to the matrix cores and accumulates in fp32.  The
oracle rounds to bf16 (nearest-even) at the same storage points - the input, the weights used in
products, every hidden activation, every back-propagated hidden gradient - and evaluates the
products themselves exactly (float64).  Gradients of the parameters are rounded to fp32 (the HIP
path stores them so) before the optimizer, which evaluates each assignment in float64 from the
stored fp32 state and rounds once.  With ``exact=True`` no bf16 rounding is applied (used by the
finite-difference pin).

Pins (tests/test_mlp_oracle_pins.py): finite-difference check of every gradient, closed forms of
the loss and its derivative, a hand-computed two-layer example, the dense optimizer against the
sparse C++ oracle with every row touched (two independent implementations of Algorithm 2), and
the merge identities of the proof sketch on the dense parameters.
"""
from __future__ import annotations

import numpy as np

STEP_LOCAL, STEP_MERGE_PENDING = 0, 1
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xD1B54A32D192ED03)
_F1 = np.uint64(0xBF58476D1CE4E5B9)
_F2 = np.uint64(0x94D049BB133111EB)


def bf16_round(a):
    """Nearest-even rounding of float32 values to bfloat16, returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return (u << np.uint64(16)).astype(np.uint32).view(np.float32).reshape(a.shape)


def layer_shapes(in_dim, hidden):
    dims = [int(in_dim)] + [int(h) for h in hidden] + [1]
    return [(dims[i], dims[i + 1]) for i in range(len(dims) - 1)]


def n_params(in_dim, hidden):
    return sum(i * o + o for i, o in layer_shapes(in_dim, hidden))


def init_params(in_dim, hidden, seed):
    """Weights: the integer recipe of the row initialiser (64-bit finalizer of (key ^ seed*phi) + C,
    four 16-bit fields summed and centred) with key = layer << 48 | index, scaled to a standard
    deviation of sqrt(2 / fan_in); biases zero."""
    out = []
    with np.errstate(over="ignore"):
        seed_mul = np.uint64(seed) * _GOLD
        for l, (i, o) in enumerate(layer_shapes(in_dim, hidden)):
            idx = np.arange(i * o, dtype=np.uint64)
            z = ((np.uint64(l) << np.uint64(48)) | idx) ^ seed_mul
            z = z + _C1
            z = (z ^ (z >> np.uint64(30))) * _F1
            z = (z ^ (z >> np.uint64(27))) * _F2
            z = z ^ (z >> np.uint64(31))
            s = ((z & np.uint64(0xFFFF)) + ((z >> np.uint64(16)) & np.uint64(0xFFFF)) +
                 ((z >> np.uint64(32)) & np.uint64(0xFFFF)) + (z >> np.uint64(48))).astype(np.int64) - 131070
            scale = np.float32(np.sqrt(2.0 / i) / 37837.2)
            out.append((s.astype(np.float32) * scale).astype(np.float32))
            out.append(np.zeros(o, np.float32))
    return np.concatenate(out)


class MlpOracle:
    def __init__(self, in_dim, hidden, n_replicas=1, kstep=False, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                 init_seed=0, exact=False):
        if n_replicas != 1 and not kstep:
            raise ValueError("replicas exist to be merged")
        self.in_dim, self.hidden = int(in_dim), [int(h) for h in hidden]
        self.shapes = layer_shapes(in_dim, hidden)
        self.W, self.kstep, self.exact = int(n_replicas), bool(kstep), bool(exact)
        self.lr, self.b1, self.b2, self.eps = (float(np.float32(h)) for h in (lr, beta1, beta2, eps))
        p0 = init_params(in_dim, hidden, init_seed)
        self.n = p0.size
        self.params = [p0.copy() for _ in range(self.W)]
        self.m = [np.zeros(self.n, np.float32) for _ in range(self.W)]
        self.v = [np.full(self.n, np.float32(eps), np.float32) for _ in range(self.W)]
        self.vhat = np.full(self.n, np.float32(eps), np.float32) if kstep else None
        self.pending = [False] * self.W

    # -- helpers
    def _r(self, a):
        return a.astype(np.float64) if self.exact else bf16_round(a.astype(np.float32)).astype(np.float64)

    def _layers(self, flat):
        out, o = [], 0
        for i, k in self.shapes:
            W = flat[o:o + i * k].reshape(i, k)
            o += i * k
            b = flat[o:o + k]
            o += k
            out.append((W, b))
        return out

    def forward(self, replica, pooled, keep=False):
        """logits[B] (float64); with keep=True also the activations needed by backward."""
        layers = self._layers(self.params[replica])
        h = self._r(np.asarray(pooled, np.float32))
        acts = [h]
        for W, b in layers[:-1]:
            z = h @ self._r(W) + b.astype(np.float64)
            h = self._r(np.maximum(z, 0.0))
            acts.append(h)
        W, b = layers[-1]
        logits = (h @ self._r(W) + b.astype(np.float64))[:, 0]
        return (logits, acts, layers) if keep else logits

    def loss_and_grads(self, replica, pooled, labels):
        """(mean loss, flat parameter gradient float64, grad of pooled float64)."""
        logits, acts, layers = self.forward(replica, pooled, keep=True)
        y = np.asarray(labels, np.float64)
        B = y.size
        loss = np.mean(np.maximum(logits, 0.0) - logits * y + np.log1p(np.exp(-np.abs(logits))))
        with np.errstate(over="ignore"):                            # exp(-z) may overflow to inf: 1 / (1 + inf) = 0, as it should
            dz = ((1.0 / (1.0 + np.exp(-logits)) - y) / B)[:, None]  # output layer: kept in full precision
        grads = []
        for l in range(len(layers) - 1, -1, -1):
            W, b = layers[l]
            a_prev = acts[l]
            grads.append(dz.sum(axis=0))
            grads.append((a_prev.T @ dz).reshape(-1))
            da = dz @ self._r(W).T
            if l > 0:
                dz = self._r(da * (a_prev > 0))
            else:
                dpooled = da
        return loss, np.concatenate(grads[::-1]), dpooled

    def step(self, replica, pooled, labels, mode=STEP_LOCAL, grad_bf16=False):
        """One training step; returns (loss float32, grad_pooled float32).  With grad_bf16 the returned
        gradient is rounded to bf16 (as float32 values): the HIP path's variant that hands the input
        gradient back in the input's precision rounds it there, once, from the fp32 sums."""
        if mode == STEP_MERGE_PENDING and not self.kstep:
            raise ValueError("single-replica mode has no merge step")
        loss, g, dpooled = self.loss_and_grads(replica, pooled, labels)
        g = g.astype(np.float32).astype(np.float64)              # the HIP path stores fp32 gradients
        x, m, v = self.params[replica], self.m[replica], self.v[replica]
        m[:] = (self.b1 * m.astype(np.float64) + (1.0 - self.b1) * g).astype(np.float32)
        v[:] = (self.b2 * v.astype(np.float64) + (1.0 - self.b2) * g * g).astype(np.float32)
        if mode == STEP_LOCAL:
            den = (self.vhat if self.kstep else v).astype(np.float64)
            x[:] = (x.astype(np.float64) - self.lr * m.astype(np.float64) / np.sqrt(den)).astype(np.float32)
        else:
            self.pending[replica] = True
        if grad_bf16 and not self.exact:
            return np.float32(loss), bf16_round(dpooled.astype(np.float32))
        return np.float32(loss), dpooled.astype(np.float32)

    def kstep_merge(self):
        if not self.kstep:
            raise ValueError("no k-step mode")
        vs = np.zeros(self.n, np.float64)
        for j in range(self.W):
            vs += self.v[j].astype(np.float64)
        self.vhat[:] = (vs / self.W).astype(np.float32)
        den = np.sqrt(self.vhat.astype(np.float64))
        xs = np.zeros(self.n, np.float64)
        for j in range(self.W):
            y = self.params[j].astype(np.float64)
            if self.pending[j]:
                y = y - self.lr * self.m[j].astype(np.float64) / den
            xs += y
        xbar = (xs / self.W).astype(np.float32)
        for j in range(self.W):
            self.params[j][:] = xbar
            self.pending[j] = False
