"""Pins for the fp64 oracle: it is checked against things other than itself.

The paper prints no worked numerical example, so every pin is structural:
finite differences and an autograd library for the gradients, hand-computed
numbers for the server update (CADA-1)-(CADA-3), special cases of Algorithm 1
(c = 0, huge c, M = 1, beta = 0), identities and bounds the paper states, and
a brute-force transcription that recomputes everything from the stored iterate
history on tiny inputs.
"""
import math

import numpy as np
import pytest
import torch

from cada_synth import configs, generators
from oracle import cada_oracle as co
from oracle.driver import oracle_for

TINY_LOG = configs.CFG1.scaled(name="tiny_log", layer_dims=(6,), M=4, N_m=40, B=5, K=60, D=7, d_max=3,
                               c=0.5, alpha=0.01, lam=1e-3, seed=11)
TINY_LOG1 = TINY_LOG.scaled(name="tiny_log1", rule=configs.RULE_CADA1, data="sparse_uniform", c=0.4, seed=12)
TINY_MLP = configs.CFG4.scaled(name="tiny_mlp", layer_dims=(7, 5, 3), M=3, N_m=30, B=6, K=40, D=6, d_max=4,
                               c=0.5, alpha=0.002, seed=13)
TINY_MLP1 = configs.CFG5.scaled(name="tiny_mlp1", layer_dims=(6, 5, 4, 3), M=3, N_m=30, B=6, K=40, D=6,
                                d_max=4, c=0.5, alpha=0.002, seed=14)
ALL_TINY = [TINY_LOG, TINY_LOG1, TINY_MLP, TINY_MLP1]


def setup(cfg, **kw):
    prob = generators.make_problem(cfg)
    sched = generators.make_schedule(cfg)
    return prob, sched, oracle_for(cfg, prob, **kw)


# ---------------------------------------------------------------- gradients
def fd_grad(f, theta, eps=1e-6):
    g = np.zeros_like(theta)
    for i in range(theta.size):
        e = np.zeros_like(theta)
        e[i] = eps
        g[i] = (f(theta + e) - f(theta - e)) / (2 * eps)
    return g


def test_logreg_grad_finite_differences():
    rng = np.random.default_rng(0)
    X = rng.normal(size=(9, 5)).astype(np.float32)
    y = np.where(rng.random(9) < 0.5, 1.0, -1.0).astype(np.float32)
    th = rng.normal(size=5)
    g = co.logreg_grad(th, X, y, 0.3)
    np.testing.assert_allclose(g, fd_grad(lambda t: co.logreg_loss(t, X, y, 0.3), th), rtol=1e-6, atol=1e-9)


def test_logreg_grad_matches_autograd():
    rng = np.random.default_rng(1)
    X = rng.normal(size=(11, 7)).astype(np.float32)
    y = np.where(rng.random(11) < 0.5, 1.0, -1.0).astype(np.float32)
    th = rng.normal(size=7)
    t = torch.tensor(th, dtype=torch.float64, requires_grad=True)
    Xt, yt = torch.tensor(X, dtype=torch.float64), torch.tensor(y, dtype=torch.float64)
    loss = torch.nn.functional.softplus(-yt * (Xt @ t)).mean() + 0.5 * 0.2 * (t @ t)
    loss.backward()
    assert abs(loss.item() - co.logreg_loss(th, X, y, 0.2)) < 1e-12
    np.testing.assert_allclose(co.logreg_grad(th, X, y, 0.2), t.grad.numpy(), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("dims", [(5, 4, 3), (6, 5, 4, 3)])
def test_mlp_grad_finite_differences_and_autograd(dims):
    rng = np.random.default_rng(2)
    X = rng.normal(size=(8, dims[0])).astype(np.float32)
    y = rng.integers(0, dims[-1], size=8).astype(np.int32)
    p = sum(dims[i] * dims[i + 1] + dims[i + 1] for i in range(len(dims) - 1))
    th = rng.normal(scale=0.5, size=p)
    g = co.mlp_grad(th, X, y, dims)
    np.testing.assert_allclose(g, fd_grad(lambda t: co.mlp_loss(t, X, y, dims), th), rtol=2e-6, atol=1e-8)
    # the same network written with torch.nn.functional, parameters in the documented layout
    t = torch.tensor(th, dtype=torch.float64, requires_grad=True)
    a, o = torch.tensor(X, dtype=torch.float64), 0
    for i in range(len(dims) - 1):
        W = t[o:o + dims[i] * dims[i + 1]].reshape(dims[i], dims[i + 1]); o += dims[i] * dims[i + 1]
        b = t[o:o + dims[i + 1]]; o += dims[i + 1]
        a = a @ W + b
        if i + 2 < len(dims):
            a = torch.relu(a)
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(y, dtype=torch.long))
    loss.backward()
    assert abs(loss.item() - co.mlp_loss(th, X, y, dims)) < 1e-12
    np.testing.assert_allclose(g, t.grad.numpy(), rtol=1e-11, atol=1e-14)


# ------------------------------------------------------- server update by hand
def test_server_update_hand_computed():
    """(CADA-1)-(CADA-3) on a scalar with nabla = 2, 1, 1.9 and beta1 = beta2 = 0.5,
    alpha = 0.1, eps = 0, worked by hand.  The third step separates the printed
    recursion v^{k+1} = beta2*vhat^k + ... (v = 2.805) from one driven by v^k (2.555)."""
    o = co.CadaOracle(model="logreg", layer_dims=(1,), M=1, rule=2, D=5, d_max=2, c=0.0, alpha=0.1,
                      beta1=0.5, beta2=0.5, eps=0.0, lam=0.0, theta0=np.zeros(1), rows=None)
    o.server_update(np.array([2.0]))
    assert (o.h[0], o.v[0], o.vhat[0]) == (1.0, 2.0, 2.0)
    assert o.theta[0] == pytest.approx(-0.1 / math.sqrt(2.0), rel=1e-15)
    o.server_update(np.array([1.0]))
    assert (o.h[0], o.v[0], o.vhat[0]) == (1.0, 1.5, 2.0)
    assert o.theta[0] == pytest.approx(-0.2 / math.sqrt(2.0), rel=1e-15)
    o.server_update(np.array([1.9]))
    assert o.h[0] == pytest.approx(1.45, rel=1e-15)
    assert o.v[0] == pytest.approx(2.805, rel=1e-15) and o.vhat[0] == pytest.approx(2.805, rel=1e-15)
    assert o.theta[0] == pytest.approx(-0.2 / math.sqrt(2.0) - 0.1 * 1.45 / math.sqrt(2.805), rel=1e-14)
    # ring holds the squared steps, slot k mod d_max: steps 1 and 2 (0-based) remain
    assert o.ring[1] == pytest.approx((0.1 / math.sqrt(2.0)) ** 2, rel=1e-12)
    assert o.ring[0] == pytest.approx((0.1 * 1.45 / math.sqrt(2.805)) ** 2, rel=1e-12)
    assert o.k == 3


# ------------------------------------------------- independent AMSGrad loop
def distributed_amsgrad(cfg, prob, sched, K, grad_fn):
    """Every worker uploads a fresh gradient every step (Section 1, the direct
    distributed implementation), followed by the paper's server update."""
    th = prob.theta0.astype(np.float64)
    h = np.zeros_like(th); vh = np.zeros_like(th)
    for k in range(K):
        nab = np.zeros_like(th)
        for m in range(cfg.M):
            X, y = prob.rows(m, sched[k, m])
            nab += grad_fn(th, X, y)
        nab /= cfg.M
        h = cfg.beta1 * h + (1 - cfg.beta1) * nab
        vh = np.maximum(cfg.beta2 * vh + (1 - cfg.beta2) * nab ** 2, vh)
        th = th - cfg.alpha * h / np.sqrt(cfg.eps + vh)
    return th


def grad_fn_for(cfg):
    if cfg.model == "logreg":
        return lambda th, X, y: co.logreg_grad(th, X, y, cfg.lam)
    return lambda th, X, y: co.mlp_grad(th, X, y, cfg.layer_dims)


@pytest.mark.parametrize("cfg", ALL_TINY, ids=lambda c: c.name)
def test_c_zero_is_distributed_amsgrad(cfg):
    cfg = cfg.scaled(c=0.0)
    if cfg.model == "logreg":
        # theta0 = 0 makes LHS = RHS = 0 at k = 0 only; start from a generic point instead
        pass
    prob, sched, o = setup(cfg)
    o.run(sched)
    masks = o.trace_arrays()["mask"]
    assert masks[1:].all(), "with c = 0 every worker uploads (LHS > 0 on generic data)"
    assert masks[0].all(), "step 0 is forced by tau^0 = D"
    ref = distributed_amsgrad(cfg, prob, sched, cfg.K, grad_fn_for(cfg))
    np.testing.assert_allclose(o.theta, ref, rtol=1e-12, atol=1e-15)


def test_single_worker_is_single_node_amsgrad():
    cfg = TINY_LOG.scaled(M=1, c=0.0)
    prob, sched, o = setup(cfg)
    o.run(sched)
    ref = distributed_amsgrad(cfg, prob, sched, cfg.K, grad_fn_for(cfg))
    np.testing.assert_allclose(o.theta, ref, rtol=1e-12, atol=1e-15)
    assert o.uploads_total == cfg.K


# --------------------------------------------------------------- huge c
@pytest.mark.parametrize("cfg", [TINY_LOG, TINY_LOG1, TINY_MLP], ids=lambda c: c.name)
def test_huge_c_no_upload_closed_form(cfg):
    """c = 1e30 and D > K: only step 0 uploads, nabla stays nabla^0, and every
    coordinate follows h^k = (1-beta1^k) g, vhat^k = (1-beta2^k) g^2."""
    K = 30
    cfg = cfg.scaled(c=1e30, D=K + 5, K=K)
    prob, sched, o = setup(cfg)
    o.run(sched)
    masks = o.trace_arrays()["mask"]
    assert masks[0].all() and not masks[1:].any()
    g0 = np.mean([grad_fn_for(cfg)(prob.theta0.astype(np.float64), *prob.rows(m, sched[0, m]))
                  for m in range(cfg.M)], axis=0)
    th = prob.theta0.astype(np.float64).copy()
    for k in range(1, K + 1):
        th = th - cfg.alpha * (1 - cfg.beta1 ** k) * g0 / np.sqrt(cfg.eps + (1 - cfg.beta2 ** k) * g0 ** 2)
    np.testing.assert_allclose(o.theta, th, rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(o.h, (1 - cfg.beta1 ** K) * g0, rtol=1e-10, atol=1e-16)
    np.testing.assert_allclose(o.vhat, (1 - cfg.beta2 ** K) * g0 ** 2, rtol=1e-10, atol=1e-30)


@pytest.mark.parametrize("cfg", [TINY_LOG, TINY_MLP1], ids=lambda c: c.name)
def test_huge_c_uploads_exactly_every_D(cfg):
    cfg = cfg.scaled(c=1e30)
    prob, sched, o = setup(cfg)
    o.run(sched)
    t = o.trace_arrays()
    for k in range(cfg.K):
        assert t["mask"][k].all() == (k % cfg.D == 0) and t["mask"][k].any() == (k % cfg.D == 0)
    assert t["tau"].max() == cfg.D and t["tau"][1:].min() == 1
    assert o.uploads_total == cfg.M * math.ceil(cfg.K / cfg.D)


def test_beta_zero_reduces_to_max_scaled_sgd():
    """beta1 = beta2 = 0: h = nabla, vhat = running max of nabla^2."""
    cfg = TINY_LOG.scaled(beta1=0.0, beta2=0.0, c=0.0, K=20)
    prob, sched, o = setup(cfg)
    th = prob.theta0.astype(np.float64).copy(); vmax = np.zeros_like(th)
    for k in range(cfg.K):
        nab = np.mean([co.logreg_grad(th, *prob.rows(m, sched[k, m]), cfg.lam) for m in range(cfg.M)], axis=0)
        vmax = np.maximum(vmax, nab ** 2)
        th = th - cfg.alpha * nab / np.sqrt(cfg.eps + vmax)
    o.run(sched)
    np.testing.assert_allclose(o.theta, th, rtol=1e-12, atol=1e-15)


# ------------------------------------------------------ identities, invariants
@pytest.mark.parametrize("cfg", ALL_TINY, ids=lambda c: c.name)
def test_invariants_and_incremental_identity(cfg):
    prob, sched, o = setup(cfg)
    thetas = [o.theta.copy()]
    nabla_inc = np.zeros(o.p)
    max_nab_norm, max_nab_sq = 0.0, np.zeros(o.p)
    beta3 = cfg.beta1 ** 2 / cfg.beta2
    step_bound = cfg.alpha ** 2 * o.p / ((1 - cfg.beta2) * (1 - beta3))
    for k in range(cfg.K):
        G_old, vhat_old = o.G.copy(), o.vhat.copy()
        mask = o.step(sched[k])
        # incremental aggregate of Section 1.2 equals the definition
        nabla_inc = nabla_inc + sum((o.G[m] - G_old[m]) for m in range(cfg.M) if mask[m]) / cfg.M
        np.testing.assert_allclose(nabla_inc, o.nabla, rtol=1e-10, atol=1e-14)
        assert (o.vhat >= vhat_old).all()
        assert (o.tau >= 1).all() and (o.tau <= cfg.D).all()
        thetas.append(o.theta.copy())
        # identity in the proof of Lemma 4 and its bound
        s = cfg.alpha ** 2 * np.sum(o.h ** 2 / (cfg.eps + o.vhat))
        assert o.ring[k % cfg.d_max] == pytest.approx(s, rel=1e-9)
        assert s <= step_bound
        # Lemma 3 with sigma replaced by the running maxima
        max_nab_norm = max(max_nab_norm, np.linalg.norm(o.nabla))
        max_nab_sq = np.maximum(max_nab_sq, o.nabla ** 2)
        assert np.linalg.norm(o.h) <= max_nab_norm * (1 + 1e-12)
        assert (o.vhat <= max_nab_sq * (1 + 1e-12)).all()
    t = o.trace_arrays()
    # right-hand side recomputed from the iterate history, theta^j = theta^0 for j < 0
    th = lambda j: thetas[max(j, 0)]
    for k in range(cfg.K):
        rhs = cfg.c / cfg.d_max * sum(np.sum((th(k + 1 - d) - th(k - d)) ** 2) for d in range(1, cfg.d_max + 1))
        assert t["rhs"][k] == pytest.approx(rhs, rel=1e-12, abs=1e-300)
    assert 0 < t["mask"][1:].sum() < t["mask"][1:].size, "the case must mix uploads and skips"


def test_cada1_snapshot_step_has_zero_fresh_innovation():
    """At k mod D = 0 the snapshot equals theta^k, so delta-tilde_m^k = 0 and the
    left-hand side is the squared norm of the stored innovation."""
    cfg = TINY_LOG1
    prob, sched, o = setup(cfg)
    for k in range(cfg.K):
        stored = o.delta_stored.copy()
        o.step(sched[k])
        if k % cfg.D == 0:
            np.testing.assert_allclose(o.trace["lhs"][-1], np.sum(stored ** 2, axis=1), rtol=1e-14, atol=0)


def test_cada2_lhs_lipschitz_bound():
    cfg = TINY_LOG
    prob, sched, o = setup(cfg)
    for k in range(cfg.K):
        ref = o.theta_hat.copy(); th = o.theta.copy()
        o.step(sched[k])
        for m in range(cfg.M):
            X, _ = prob.rows(m, sched[k, m])
            L = np.sum(X.astype(np.float64) ** 2) / (4 * cfg.B) + cfg.lam
            assert math.sqrt(o.trace["lhs"][-1][m]) <= L * np.linalg.norm(th - ref[m]) * (1 + 1e-9) + 1e-300


# ------------------------------------------------------------- brute force
def loop_logreg_grad(th, X, y, lam):
    g = [lam * t for t in th]
    n = len(y)
    for b in range(n):
        z = sum(float(X[b][j]) * th[j] for j in range(len(th)))
        s = float(y[b])
        coef = -s / (1.0 + math.exp(s * z)) / n
        for j in range(len(th)):
            g[j] += coef * float(X[b][j])
    return np.array(g)


def brute_force(cfg, prob, sched, K):
    """Algorithm 1 recomputed from definitions: the iterate history is kept, each
    worker remembers only the step u_m of its last upload, and every stored
    quantity (stale gradient, theta-hat, stored innovation, RHS) is re-derived
    from (history, u_m) at each step."""
    M, D = cfg.M, cfg.D
    thetas = [prob.theta0.astype(np.float64)]
    th = lambda j: thetas[max(j, 0)]
    u = [-D] * M
    h = np.zeros(cfg.p); vh = np.zeros(cfg.p)
    masks, lhss, rhss = [], [], []

    def grad_at(j, m, jsamp):
        return loop_logreg_grad(th(j), *prob.rows(m, sched[jsamp, m]), cfg.lam)

    def stored_grad(m):                       # gradient held by the server for worker m
        return np.zeros(cfg.p) if u[m] < 0 else grad_at(u[m], m, u[m])

    def dtilde(j, m):                         # CADA1 innovation computed at step j
        if j < 0:
            return np.zeros(cfg.p)
        return grad_at(j, m, j) - grad_at(D * (j // D), m, j)

    for k in range(K):
        rhs = cfg.c / cfg.d_max * sum(np.sum((th(k + 1 - d) - th(k - d)) ** 2) for d in range(1, cfg.d_max + 1))
        mask, lhs = [], []
        for m in range(M):
            tau = k - u[m]
            if cfg.rule == configs.RULE_CADA2:
                diff = grad_at(k, m, k) - grad_at(k - tau, m, k)
            elif cfg.rule == configs.RULE_CADA1:
                diff = dtilde(k, m) - dtilde(u[m], m)
            else:                             # (LAGrule): other iterate AND other samples
                diff = grad_at(k, m, k) - stored_grad(m)
            lhs.append(float(diff @ diff))
            mask.append(lhs[-1] > rhs or tau >= D or cfg.rule == configs.RULE_ALWAYS)
        for m in range(M):
            if mask[m]:
                u[m] = k
        nab = sum(stored_grad(m) for m in range(M)) / M
        if cfg.server == configs.SERVER_SGD:
            thetas.append(thetas[-1] - cfg.alpha * nab)
        else:
            h = cfg.beta1 * h + (1 - cfg.beta1) * nab
            vh = np.maximum(cfg.beta2 * vh + (1 - cfg.beta2) * nab * nab, vh)
            thetas.append(thetas[-1] - cfg.alpha * h / np.sqrt(cfg.eps + vh))
        masks.append(mask); lhss.append(lhs); rhss.append(rhs)
    return thetas, np.array(masks), np.array(lhss), np.array(rhss)


@pytest.mark.parametrize("rule", [configs.RULE_CADA1, configs.RULE_CADA2])
def test_brute_force_history_transcription(rule):
    cfg = TINY_LOG.scaled(rule=rule, M=3, layer_dims=(3,), B=2, N_m=12, K=26, D=4, d_max=3, c=0.6, seed=21)
    prob, sched, o = setup(cfg)
    o.run(sched)
    thetas, masks, lhss, rhss = brute_force(cfg, prob, sched, cfg.K)
    t = o.trace_arrays()
    assert (t["mask"] == masks).all()
    forced = t["tau"] >= cfg.D
    assert 0 < masks[~forced].sum() < (~forced).sum(), "rule decisions must mix uploads and skips"
    np.testing.assert_allclose(t["lhs"], lhss, rtol=1e-9, atol=1e-22)
    np.testing.assert_allclose(t["rhs"], rhss, rtol=1e-11, atol=0)
    np.testing.assert_allclose(o.theta, thetas[-1], rtol=1e-12, atol=1e-15)


# ------------------------------------- rule variants: always-upload, stochastic LAG
@pytest.mark.parametrize("server,c", [(configs.SERVER_SGD, 400.0), (configs.SERVER_AMSGRAD, 10.0)])
def test_lag_rule_brute_force_history_transcription(server, c):
    """Condition (LAGrule) of Section 2.1 with the SGD update it is stated for, and with the
    server update of (CADA-1)-(CADA-3), against the history-based transcription."""
    cfg = TINY_LOG.scaled(rule=configs.RULE_LAG, server=server, M=3, layer_dims=(3,), B=2, N_m=12, K=30, D=5, d_max=3,
                          c=c, alpha=0.05 if server == configs.SERVER_SGD else 0.01, seed=22)
    prob, sched, o = setup(cfg)
    o.run(sched)
    thetas, masks, lhss, rhss = brute_force(cfg, prob, sched, cfg.K)
    t = o.trace_arrays()
    assert (t["mask"] == masks).all()
    forced = t["tau"] >= cfg.D
    assert 0 < masks[~forced].sum() < (~forced).sum(), "rule decisions must mix uploads and skips"
    np.testing.assert_allclose(t["lhs"], lhss, rtol=1e-9, atol=1e-22)
    np.testing.assert_allclose(t["rhs"], rhss, rtol=1e-11, atol=0)
    np.testing.assert_allclose(o.theta, thetas[-1], rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("cfg", [TINY_LOG, TINY_MLP], ids=lambda c: c.name)
def test_always_rule_is_distributed_amsgrad_for_any_c(cfg):
    cfg = cfg.scaled(rule=configs.RULE_ALWAYS, c=1e30)
    prob, sched, o = setup(cfg)
    o.run(sched)
    assert o.trace_arrays()["mask"].all() and o.uploads_total == cfg.M * cfg.K
    ref = distributed_amsgrad(cfg, prob, sched, cfg.K, grad_fn_for(cfg))
    np.testing.assert_allclose(o.theta, ref, rtol=1e-12, atol=1e-15)


def test_lag_sgd_with_c_zero_is_distributed_sgd_and_huge_c_uploads_every_D():
    cfg = TINY_LOG.scaled(rule=configs.RULE_LAG, server=configs.SERVER_SGD, c=0.0, alpha=0.05)
    prob, sched, o = setup(cfg)
    o.run(sched)
    assert o.trace_arrays()["mask"].all()
    th = prob.theta0.astype(np.float64)
    for k in range(cfg.K):                    # plain distributed minibatch SGD
        nab = sum(co.logreg_grad(th, *prob.rows(m, sched[k, m]), cfg.lam) for m in range(cfg.M)) / cfg.M
        th = th - cfg.alpha * nab
    np.testing.assert_allclose(o.theta, th, rtol=1e-12, atol=1e-15)
    prob, sched, o = setup(cfg.scaled(c=1e30))
    o.run(sched)
    m = o.trace_arrays()["mask"]
    for k in range(cfg.K):
        assert m[k].all() == (k % cfg.D == 0) and m[k].any() == (k % cfg.D == 0)


def test_decaying_stepsize_is_the_plain_loop():
    """alpha_k = alpha K0/(k+K0) (Theorem 2's 2/(mu(k+K0))): always-upload + SGD server is
    distributed SGD with that schedule; with the AMSGrad server the schedule multiplies the
    same h/sqrt(eps+vhat) direction."""
    cfg = TINY_LOG.scaled(rule=configs.RULE_ALWAYS, server=configs.SERVER_SGD, alpha=0.2, alpha_K0=7)
    prob, sched, o = setup(cfg)
    o.run(sched)
    th = prob.theta0.astype(np.float64)
    for k in range(cfg.K):
        nab = sum(co.logreg_grad(th, *prob.rows(m, sched[k, m]), cfg.lam) for m in range(cfg.M)) / cfg.M
        th = th - (0.2 * 7.0 / (k + 7.0)) * nab
    np.testing.assert_allclose(o.theta, th, rtol=1e-12, atol=1e-15)
    cfg = TINY_LOG.scaled(rule=configs.RULE_ALWAYS, alpha=0.05, alpha_K0=5)
    prob, sched, o = setup(cfg)
    o.run(sched)
    th = prob.theta0.astype(np.float64); h = np.zeros_like(th); vh = np.zeros_like(th)
    for k in range(cfg.K):
        nab = sum(co.logreg_grad(th, *prob.rows(m, sched[k, m]), cfg.lam) for m in range(cfg.M)) / cfg.M
        h = cfg.beta1 * h + (1 - cfg.beta1) * nab
        vh = np.maximum(cfg.beta2 * vh + (1 - cfg.beta2) * nab ** 2, vh)
        th = th - (0.05 * 5.0 / (k + 5.0)) * h / np.sqrt(cfg.eps + vh)
    np.testing.assert_allclose(o.theta, th, rtol=1e-12, atol=1e-15)


# -------------------------------------------------------------- evaluation
def test_evaluate_closed_forms_and_direct_sum():
    """At theta = 0 the logistic objective is ln 2 and the C-class cross-entropy ln C; at a
    generic point it is the per-sample Python-loop mean, averaged over the workers."""
    for cfg, want in ((TINY_LOG, math.log(2.0)), (TINY_MLP, math.log(3.0))):
        prob = generators.make_problem(cfg)
        o = oracle_for(cfg, prob, theta0=np.zeros(cfg.p))
        loss, acc = o.evaluate([cfg.N_m] * cfg.M)
        assert loss == pytest.approx(want, rel=1e-14)
    cfg = TINY_LOG
    prob, sched, o = setup(cfg)
    o.run(sched[:5])
    loss, acc = o.evaluate([cfg.N_m] * cfg.M)
    tot = hits = 0.0
    for m in range(cfg.M):
        X, y = prob.rows(m, np.arange(cfg.N_m))
        lm = hm = 0.0
        for b in range(cfg.N_m):
            z = sum(float(X[b][j]) * o.theta[j] for j in range(cfg.p))
            lm += math.log1p(math.exp(-float(y[b]) * z))
            hm += 1.0 if float(y[b]) * z > 0 else 0.0
        tot += lm / cfg.N_m + 0.5 * cfg.lam * float(o.theta @ o.theta)
        hits += hm / cfg.N_m
    assert loss == pytest.approx(tot / cfg.M, rel=1e-12) and acc == pytest.approx(hits / cfg.M, rel=1e-12)
    assert acc > 0.5, "five steps of training beat chance on the planted direction"


# ------------------------------------------------------------------ replay
@pytest.mark.parametrize("cfg", [TINY_LOG, TINY_MLP1], ids=lambda c: c.name)
def test_replay_reproduces_and_overrides(cfg):
    prob, sched, o = setup(cfg)
    o.run(sched)
    t = o.trace_arrays()
    o2 = oracle_for(cfg, prob).run(sched, t["mask"])
    assert np.array_equal(o2.theta, o.theta) and np.array_equal(o2.trace_arrays()["own_mask"], t["mask"])
    # forcing all-ones reproduces distributed AMSGrad whatever c is; the rule is still logged
    o3 = oracle_for(cfg, prob).run(sched, np.ones_like(t["mask"]))
    ref = distributed_amsgrad(cfg, prob, sched, cfg.K, grad_fn_for(cfg))
    np.testing.assert_allclose(o3.theta, ref, rtol=1e-12, atol=1e-15)
    assert (o3.tau == 1).all()
    # forcing all-zero after step 0 with the rule's own decision ignored: nabla frozen
    rp = np.zeros_like(t["mask"]); rp[0] = 1
    o4 = oracle_for(cfg, prob)
    o4.step(sched[0], rp[0]); nab0 = o4.nabla.copy()
    for k in range(1, 10):
        o4.step(sched[k], rp[k])
        assert np.array_equal(o4.nabla, nab0)
    # 255 leaves the decision to the rule
    o5 = oracle_for(cfg, prob).run(sched, np.full_like(t["mask"], 255))
    assert np.array_equal(o5.theta, o.theta)
