"""CPU oracle for CADA (Communication-Adaptive Distributed Adam), fp64.

TEST INFRASTRUCTURE ONLY.  A plain, slow, step-by-step implementation of the
paper's Algorithm 1 used to check the GPU library; the product path never
imports, calls or links anything in this directory, and this file imports
nothing from the GPU package.

CADA is an iteration with a data-dependent discrete decision, so the oracle is
the algorithm itself, in the paper's order and notation:

  * server update, equations (CADA-1)-(CADA-3) of Section 1.2:
        h^{k+1}   = beta1 h^k + (1-beta1) nabla^k
        v^{k+1}   = beta2 vhat^k + (1-beta2) (nabla^k)^2      (vhat^k, as printed)
        vhat^{k+1}= max(v^{k+1}, vhat^k)
        theta^{k+1} = theta^k - alpha (eps I + Vhat^{k+1})^{-1/2} h^{k+1}
    with nabla^k = (1/M) sum_m (stored gradient of worker m);
  * CADA1 rule, condition (workerrule1); CADA2 rule, condition (workerrule2),
    both of Section 2.2; upload also when tau_m^k >= D (Algorithm 1);
  * tau_m^{k+1} = 1 after an upload, tau_m^k + 1 otherwise;
  * theta^{-D} = ... = theta^{-1} = theta^0 (supplement, "Supporting Lemmas"),
    i.e. the parameter differences before step 0 are zero.

Readings where the paper is silent (shared with the library by convention):
  h^0 = v^0 = vhat^0 = 0; tau_m^0 = D (every worker uploads at k = 0);
  upload iff LHS > RHS (the rule skips on "<="); eps inside the square root;
  no bias correction; constant stepsize; minibatch gradient = mean over the B
  rows; l2 regulariser (lambda/2)|theta|^2 inside the logistic loss; uniform
  1/M weights; ReLU'(0) = 0; CADA1's stored innovation is kept across snapshot
  refreshes.

Every function here is pinned in tests/test_oracle_pins.py against finite
differences, closed forms, special cases (c = 0, huge c, M = 1, beta = 0), the
incremental-aggregate identity, the supplement's Lemma bounds and a brute-force
transcription on tiny inputs.
"""
from __future__ import annotations

from typing import Callable, Optional, Sequence

import numpy as np
from scipy.special import expit, logsumexp

RULE_ALWAYS = 0      # every worker uploads at every iteration (the distributed Adam/AMSGrad baseline of Section 4)
RULE_CADA1 = 1
RULE_CADA2 = 2
RULE_LAG = 3         # stochastic LAG, condition (LAGrule) of Section 2.1: fresh gradient against the stored one
SERVER_AMSGRAD = 0   # equations (CADA-1)-(CADA-3)
SERVER_SGD = 1       # theta <- theta - alpha * nabla (the update stochastic LAG follows, Section 2.1)
REPLAY_FREE = 255


# --------------------------------------------------------------------------
# losses and minibatch gradients (Section 1, problem (1): l(theta; xi))
# --------------------------------------------------------------------------
def logreg_loss(theta, X, y, lam):
    """Mean logistic loss log(1+exp(-y x.theta)) over the rows + (lam/2)|theta|^2."""
    theta = np.asarray(theta, dtype=np.float64)
    z = np.asarray(X, dtype=np.float64) @ theta
    yy = np.asarray(y, dtype=np.float64)
    return float(np.mean(np.logaddexp(0.0, -yy * z)) + 0.5 * lam * theta @ theta)


def logreg_grad(theta, X, y, lam):
    theta = np.asarray(theta, dtype=np.float64)
    Xd = np.asarray(X, dtype=np.float64)
    yy = np.asarray(y, dtype=np.float64)
    z = Xd @ theta
    r = -yy * expit(-yy * z)
    return Xd.T @ r / Xd.shape[0] + lam * theta


def mlp_unpack(theta, dims: Sequence[int]):
    """Views (W_l [in,out], b_l [out]) into the flat parameter vector."""
    out, o = [], 0
    for i in range(len(dims) - 1):
        nw = dims[i] * dims[i + 1]
        W = theta[o:o + nw].reshape(dims[i], dims[i + 1])
        o += nw
        b = theta[o:o + dims[i + 1]]
        o += dims[i + 1]
        out.append((W, b))
    assert o == theta.size
    return out


def mlp_logits(theta, X, dims):
    theta = np.asarray(theta, dtype=np.float64)
    a = np.asarray(X, dtype=np.float64)
    layers = mlp_unpack(theta, dims)
    for i, (W, b) in enumerate(layers):
        a = a @ W + b
        if i + 1 < len(layers):
            a = np.maximum(a, 0.0)
    return a


def mlp_loss(theta, X, y, dims):
    """Mean softmax cross-entropy of a ReLU MLP."""
    a = mlp_logits(theta, X, dims)
    lse = logsumexp(a, axis=1)
    return float(np.mean(lse - a[np.arange(a.shape[0]), np.asarray(y, dtype=np.int64)]))


def mlp_grad(theta, X, y, dims):
    theta = np.asarray(theta, dtype=np.float64)
    layers = mlp_unpack(theta, dims)
    acts = [np.asarray(X, dtype=np.float64)]
    zs = []
    for i, (W, b) in enumerate(layers):
        z = acts[-1] @ W + b
        zs.append(z)
        acts.append(np.maximum(z, 0.0) if i + 1 < len(layers) else z)
    logits = zs[-1]
    Bn = logits.shape[0]
    P = np.exp(logits - logsumexp(logits, axis=1, keepdims=True))
    dz = P
    dz[np.arange(Bn), np.asarray(y, dtype=np.int64)] -= 1.0
    dz /= Bn
    grads = [None] * len(layers)
    for i in range(len(layers) - 1, -1, -1):
        W, _ = layers[i]
        grads[i] = (acts[i].T @ dz, dz.sum(axis=0))
        if i > 0:
            da = dz @ W.T
            dz = da * (zs[i - 1] > 0.0)
    return np.concatenate([np.concatenate([gw.ravel(), gb]) for gw, gb in grads])


# --------------------------------------------------------------------------
# Algorithm 1
# --------------------------------------------------------------------------
class CadaOracle:
    """State and one-iteration step of Algorithm 1 for all M workers.

    ``rows(m, local_rows) -> (X, y)`` returns worker m's samples (the same
    float32 values the GPU sees; they are widened to fp64 here).
    """

    def __init__(self, *, model: str, layer_dims: Sequence[int], M: int, rule: int, D: int,
                 d_max: int, c: float, alpha: float, beta1: float, beta2: float, eps: float,
                 lam: float, theta0, rows: Callable, server: int = SERVER_AMSGRAD, alpha_K0: int = 0):
        assert rule in (RULE_ALWAYS, RULE_CADA1, RULE_CADA2, RULE_LAG)
        assert server in (SERVER_AMSGRAD, SERVER_SGD)
        self.server = server
        self.alpha_K0 = alpha_K0      # 0: constant stepsize; else alpha_k = alpha K0/(k+K0) (Theorem 2's 2/(mu(k+K0)))
        self.model, self.dims, self.M, self.rule = model, tuple(layer_dims), M, rule
        self.D, self.d_max, self.c = D, d_max, c
        self.alpha, self.beta1, self.beta2, self.eps, self.lam = alpha, beta1, beta2, eps, lam
        self.rows = rows
        self.theta = np.array(theta0, dtype=np.float64)
        p = self.theta.size
        self.p = p
        self.h = np.zeros(p)
        self.v = np.zeros(p)
        self.vhat = np.zeros(p)
        self.nabla = np.zeros(p)
        self.G = np.zeros((M, p))                     # stored (possibly stale) gradients
        self.tau = np.full(M, D, dtype=np.int64)
        self.ring = np.zeros(d_max)                   # last d_max values of |theta^{j+1}-theta^j|^2
        self.k = 0
        self.uploads_total = 0
        if rule == RULE_CADA2:
            self.theta_hat = np.tile(self.theta, (M, 1))      # theta^{k - tau_m^k}
        elif rule == RULE_CADA1:
            self.theta_snap = self.theta.copy()               # snapshot theta-tilde
            self.delta_stored = np.zeros((M, p))              # stored delta-tilde_m^{k-tau}
        self.trace = {"mask": [], "own_mask": [], "lhs": [], "rhs": [], "tau": []}

    def grad(self, theta, X, y):
        """Minibatch stochastic gradient of l(theta; xi) on the rows (X, y)."""
        if self.model == "logreg":
            return logreg_grad(theta, X, y, self.lam)
        return mlp_grad(theta, X, y, self.dims)

    def step(self, idx, replay: Optional[np.ndarray] = None):
        """One iteration k.  ``idx[m]`` = worker m's minibatch rows; ``replay[m]`` in
        {0, 1} forces the upload decision, 255 (or replay=None) leaves it to the rule."""
        M = self.M
        if self.rule == RULE_CADA1 and self.k % self.D == 0:
            self.theta_snap = self.theta.copy()
        g = np.empty((M, self.p))
        lhs = np.empty(M)
        delta_t = np.empty((M, self.p)) if self.rule == RULE_CADA1 else None
        for m in range(M):
            X, y = self.rows(m, idx[m])               # the same samples for both gradients
            g[m] = self.grad(self.theta, X, y)
            if self.rule == RULE_CADA2:
                diff = g[m] - self.grad(self.theta_hat[m], X, y)
            elif self.rule == RULE_CADA1:
                delta_t[m] = g[m] - self.grad(self.theta_snap, X, y)
                diff = delta_t[m] - self.delta_stored[m]
            else:
                # (LAGrule): the stored gradient was taken at theta^{k-tau} on the samples of that
                # iteration.  RULE_ALWAYS records the same quantity but does not use it.
                diff = g[m] - self.G[m]
            lhs[m] = diff @ diff
        rhs = (self.c / self.d_max) * float(np.sum(self.ring))
        own = (lhs > rhs) | (self.tau >= self.D)
        if self.rule == RULE_ALWAYS:
            own = np.ones(M, dtype=bool)
        mask = own.copy()
        if replay is not None:
            rp = np.asarray(replay)
            forced = rp != REPLAY_FREE
            mask[forced] = rp[forced] != 0
        self.trace["mask"].append(mask.astype(np.uint8))
        self.trace["own_mask"].append(own.astype(np.uint8))
        self.trace["lhs"].append(lhs.copy())
        self.trace["rhs"].append(rhs)
        self.trace["tau"].append(self.tau.copy())
        for m in range(M):
            if mask[m]:
                self.G[m] = g[m]
                self.tau[m] = 1
                if self.rule == RULE_CADA2:
                    self.theta_hat[m] = self.theta
                elif self.rule == RULE_CADA1:
                    self.delta_stored[m] = delta_t[m]
            else:
                self.tau[m] += 1
        self.uploads_total += int(mask.sum())
        self.server_update(self.G.sum(axis=0) / M)
        return mask

    def server_update(self, nabla):
        """Equations (CADA-1)-(CADA-3) with the aggregate ``nabla``; records
        |theta^{k+1}-theta^k|^2 for the rules' right-hand side and advances k."""
        self.nabla = np.asarray(nabla, dtype=np.float64)
        alpha = self.alpha if self.alpha_K0 <= 0 else self.alpha * self.alpha_K0 / (self.k + self.alpha_K0)
        if self.server == SERVER_SGD:
            theta_new = self.theta - alpha * self.nabla
            dtheta = theta_new - self.theta
            self.ring[self.k % self.d_max] = dtheta @ dtheta
            self.theta = theta_new
            self.k += 1
            return
        self.h = self.beta1 * self.h + (1.0 - self.beta1) * self.nabla
        self.v = self.beta2 * self.vhat + (1.0 - self.beta2) * self.nabla * self.nabla
        self.vhat = np.maximum(self.v, self.vhat)
        theta_new = self.theta - alpha * self.h / np.sqrt(self.eps + self.vhat)
        dtheta = theta_new - self.theta
        self.ring[self.k % self.d_max] = dtheta @ dtheta
        self.theta = theta_new
        self.k += 1

    def evaluate(self, n_samples: Sequence[int]):
        """(L(theta), accuracy) on all the data: the objective of problem (1), Section 1,
        L = (1/M) sum_m L_m with L_m the mean loss over worker m's samples (plus the
        regulariser for the logistic model), and the fraction of correctly classified samples
        averaged over the workers in the same way (the y-axes of the figures of Section 4)."""
        loss = acc = 0.0
        for m in range(self.M):
            X, y = self.rows(m, np.arange(int(n_samples[m])))
            if self.model == "logreg":
                loss += logreg_loss(self.theta, X, y, self.lam)
                z = np.asarray(X, dtype=np.float64) @ self.theta
                acc += float(np.mean(np.asarray(y, dtype=np.float64) * z > 0.0))
            else:
                loss += mlp_loss(self.theta, X, y, self.dims)
                acc += float(np.mean(np.argmax(mlp_logits(self.theta, X, self.dims), axis=1) == np.asarray(y)))
        return loss / self.M, acc / self.M

    def run(self, schedule, replay_schedule=None):
        for k in range(len(schedule)):
            self.step(schedule[k], None if replay_schedule is None else replay_schedule[k])
        return self

    def trace_arrays(self):
        t = self.trace
        return {"mask": np.array(t["mask"], dtype=np.uint8).reshape(-1, self.M),
                "own_mask": np.array(t["own_mask"], dtype=np.uint8).reshape(-1, self.M),
                "lhs": np.array(t["lhs"], dtype=np.float64).reshape(-1, self.M),
                "rhs": np.array(t["rhs"], dtype=np.float64),
                "tau": np.array(t["tau"], dtype=np.int64).reshape(-1, self.M)}


def margins(lhs, rhs):
    """Relative distance of each rule test from its threshold: |LHS-RHS| / max(RHS, tiny)."""
    rhs = np.asarray(rhs, dtype=np.float64).reshape(-1, 1)
    return np.abs(np.asarray(lhs, dtype=np.float64) - rhs) / np.maximum(rhs, 1e-300)
