"""CPU oracle for the DPPF consensus round and the local step -- TEST INFRASTRUCTURE ONLY.

Plain, slow, float64 numpy code that writes out the paper's definitions one by one, so that
a reader can check every line against the paper by eye.  It is used by the tests, by the
smoke check and by the benchmark's CPU-baseline leg; the product path never calls it and it
shares no code with the GPU kernels.

All functions take the M workers' parameter vectors as one array ``x`` of shape (M, d): row m
is worker m's whole model x_m in R^d (Sec. 1, Eq. 1: one shared model vector; a per-layer
tensor list is the concatenation of its tensors in list order).  Inputs of any float dtype
are converted to float64 first and all arithmetic is float64; nothing is rounded back.

Every output below has a closed form that the CPU tests pin independently (hand-worked
cases, algebraic invariants, exact rational arithmetic); no function here is "parity
unpinned".

Readings taken where the paper leaves a choice open:
  * momentum form (Alg. 1 shows plain SGD; the experiments state "SGD with momentum 0.9"):
    heavy-ball with a raw-gradient buffer, v <- mu*v + g, x <- x - eta*v, no dampening, no
    Nesterov; weight decay is the coupled L2 form g <- g + wd*x.
  * the distance is one norm over the whole model vector, not per layer.
  * the push direction uses the pre-update gap and the pre-update average for every worker
    (all workers move simultaneously from the same snapshot; appendix, gap-dynamics proof).
  * a worker at zero distance (r_m = 0) has no push direction: its displacement is the zero
    vector, so x_m is returned unchanged, r_m = 0 and the reported coefficient is alpha.
"""
from __future__ import annotations

import numpy as np


def _as_f64(a) -> np.ndarray:
    return np.array(a, dtype=np.float64, copy=True)


# --------------------------------------------------------------------------------------
# Local optimizer step between rounds (Alg. 1, the SGD line; momentum 0.9 per Sec. 6 /
# appendix "DPPF with Soft-Consensus Methods").
# --------------------------------------------------------------------------------------
def local_sgd_step(x, v, g, lr, momentum, weight_decay=0.0):
    """One heavy-ball SGD step for every worker.  Returns (x_new, v_new), both (M, d)."""
    x = _as_f64(x)
    v = _as_f64(v)
    g = _as_f64(g)
    g_eff = g + weight_decay * x
    v_new = momentum * v + g_eff
    x_new = x - lr * v_new
    return x_new, v_new


# --------------------------------------------------------------------------------------
# Consensus round (Alg. 1 consensus branch with x_C = x_A; Eq. 5, the single-line update).
# --------------------------------------------------------------------------------------
def replica_mean(x):
    """x_A = (1/M) sum_m x_m  (Alg. 1, last line; Sec. 4)."""
    x = _as_f64(x)
    M = x.shape[0]
    total = np.zeros(x.shape[1], dtype=np.float64)
    for m in range(M):
        total = total + x[m]
    return total / M


def dist_norms(x, x_avg=None):
    """r_m = || x_m - x_A ||_2 over the whole vector (Alg. 1 push line; Eq. 5)."""
    x = _as_f64(x)
    if x_avg is None:
        x_avg = replica_mean(x)
    M = x.shape[0]
    r = np.zeros(M, dtype=np.float64)
    for m in range(M):
        diff = x[m] - x_avg
        r[m] = np.sqrt(np.sum(diff * diff))
    return r


def pull_push_coefficients(r, pull, push):
    """c_m = alpha - lambda / r_m, the bracket of Eq. 5; alpha where r_m = 0."""
    r = _as_f64(r)
    c = np.full(r.shape, float(pull), dtype=np.float64)
    for m in range(r.shape[0]):
        if r[m] > 0.0:
            c[m] = pull - push / r[m]
    return c


def pull_push_round(x, pull, push):
    """Eq. 5: x_m <- x_m + (x_A - x_m) * (alpha - lambda / ||x_m - x_A||).

    Returns (x_new, r, c, x_avg) with r, c, x_avg taken BEFORE the update."""
    x = _as_f64(x)
    M = x.shape[0]
    x_avg = replica_mean(x)
    r = dist_norms(x, x_avg)
    c = pull_push_coefficients(r, pull, push)
    x_new = np.empty_like(x)
    for m in range(M):
        if r[m] > 0.0:
            x_new[m] = x[m] + (x_avg - x[m]) * c[m]
        else:
            x_new[m] = x[m]          # zero gap: zero displacement
    return x_new, r, c, x_avg


def dppf_round(x, v, g, lr, momentum, weight_decay, pull, push):
    """The last local step followed by the consensus round (same result as calling
    local_sgd_step and then pull_push_round).  Returns (x_new, v_new, r, c, x_avg)."""
    x1, v1 = local_sgd_step(x, v, g, lr, momentum, weight_decay)
    x2, r, c, x_avg = pull_push_round(x1, pull, push)
    return x2, v1, r, c, x_avg


# --------------------------------------------------------------------------------------
# Alg. 1 written literally: pull toward a consensus variable x_C, then push away from a
# reference point along the ALREADY PULLED gap.  With x_C = x_A and alpha < 1 this equals
# Eq. 5 (Sec. 5, paragraph before Eq. 5).  `push_from` selects the reference of the push:
# the average x_A (Alg. 1) or x_C itself (the variant of the LSGD remark in the appendix).
# --------------------------------------------------------------------------------------
def pull_then_push(x, x_c, pull, push, push_from="average"):
    """Returns (x_new, r_post) where r_post[m] is the norm of the post-pull gap that the
    push normalises by.  A zero post-pull gap gives no push."""
    x = _as_f64(x)
    x_c = _as_f64(x_c)
    M = x.shape[0]
    x_avg = replica_mean(x)                      # the average of the workers before the round
    ref = x_avg if push_from == "average" else x_c
    if push_from not in ("average", "consensus"):
        raise ValueError(push_from)
    x_new = np.empty_like(x)
    r_post = np.zeros(M, dtype=np.float64)
    for m in range(M):
        pulled = (1.0 - pull) * x[m] + pull * x_c
        gap = pulled - ref
        r_post[m] = np.sqrt(np.sum(gap * gap))
        if r_post[m] > 0.0:
            x_new[m] = pulled + push * gap / r_post[m]
        else:
            x_new[m] = pulled
    return x_new, r_post


# --------------------------------------------------------------------------------------
# Exact gradient of the relaxed Inverse-Mean-Valley regulariser (Eq. 4(a); appendix
# "Derivation of the Update Rule"): both terms kept.
# --------------------------------------------------------------------------------------
def pull_push_round_exact(x, pull, push_r):
    """x_m <- x_m - alpha*d_m + (lambda_r / M^2) * (M * d_m/||d_m|| - sum_j d_j/||d_j||),
    d_m = x_m - x_A.  lambda_r is the regulariser's coefficient (Eq. 4(a)); the simplified
    update of Eq. 5 corresponds to lambda = lambda_r / M with the sum dropped.  Workers at
    zero distance contribute a zero unit vector.  Returns (x_new, r, x_avg)."""
    x = _as_f64(x)
    M = x.shape[0]
    x_avg = replica_mean(x)
    r = dist_norms(x, x_avg)
    units = np.zeros_like(x)
    for j in range(M):
        if r[j] > 0.0:
            units[j] = (x[j] - x_avg) / r[j]
    unit_sum = np.zeros(x.shape[1], dtype=np.float64)
    for j in range(M):
        unit_sum = unit_sum + units[j]
    x_new = np.empty_like(x)
    for m in range(M):
        d_m = x[m] - x_avg
        x_new[m] = x[m] - pull * d_m + (push_r / (M * M)) * (M * units[m] - unit_sum)
    return x_new, r, x_avg


# --------------------------------------------------------------------------------------
# Round by-products the paper logs (appendix "Pull-Push Mechanism") and the push-strength
# schedules (appendix "How to Schedule The Pushing Force?").
# --------------------------------------------------------------------------------------
def round_statistics(r, pull, push, x_avg=None):
    """Relaxed MV (mean distance to the average), per-worker pull strength alpha*r_m and
    push strength lambda.  With the average x_A given, also its Euclidean norm ||x_A||_2 and
    the ratio of the valley width (the relaxed MV) to that norm, the two quantities the
    appendix section on hyper-parameter sensitivity tracks."""
    r = _as_f64(r)
    out = {
        "relaxed_mv": float(np.sum(r) / r.shape[0]),
        "pull_strength": pull * r,
        "push_strength": np.full(r.shape, float(push)),
    }
    if x_avg is not None:
        x_avg = _as_f64(x_avg)
        out["average_norm"] = float(np.sqrt(np.sum(x_avg * x_avg)))
        out["width_over_norm"] = out["relaxed_mv"] / out["average_norm"]
    return out


def push_schedule(kind, push, t, t_total):
    """lambda_t for the fixed / decreasing / increasing (flipped cosine) schedules."""
    if kind == "fixed":
        return float(push)
    if kind == "decreasing":
        return 0.5 * push * (1.0 + np.cos(np.pi * t / t_total))
    if kind == "increasing":
        return 0.5 * push * (1.0 - np.cos(np.pi * t / t_total))
    raise ValueError(kind)


# --------------------------------------------------------------------------------------
# AdamW local step (the ViT experiments use AdamW, lr 5e-4, weight decay 0.01).  The paper
# gives no formula; this is the published decoupled-weight-decay Adam (Loshchilov & Hutter):
#   x <- x - lr*wd*x ; m <- b1*m + (1-b1)*g ; s <- b2*s + (1-b2)*g^2 ;
#   x <- x - lr * (m / (1-b1^t)) / (sqrt(s / (1-b2^t)) + eps),  t = 1, 2, ...
# --------------------------------------------------------------------------------------
def local_adamw_step(x, m1, m2, g, lr, beta1, beta2, eps, weight_decay, step):
    x = _as_f64(x)
    m1 = _as_f64(m1)
    m2 = _as_f64(m2)
    g = _as_f64(g)
    x = x - lr * weight_decay * x
    m1_new = beta1 * m1 + (1.0 - beta1) * g
    m2_new = beta2 * m2 + (1.0 - beta2) * (g * g)
    m_hat = m1_new / (1.0 - beta1 ** step)
    s_hat = m2_new / (1.0 - beta2 ** step)
    x_new = x - lr * m_hat / (np.sqrt(s_hat) + eps)
    return x_new, m1_new, m2_new
