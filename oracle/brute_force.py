"""Pure-Python brute force of the SparQ step for ONE head (and, in `sparq_group`, for the query heads that
share one KV head under the paper's grouped-query rule) on tiny inputs.

Test infrastructure only.  It exists to pin the C oracle to something that is not
itself: lists of Python floats, full sorts, math.fsum, no numpy arithmetic, written
directly from Section 3 (Eqs. 2, 6-10) and Section 4 (Steps 1-3).
"""
import math


def softmax(xs):
    top = max(xs)
    es = [math.exp(x - top) for x in xs]
    tot = math.fsum(es)
    return [e / tot for e in es]


def dense(q, K, V):
    """Eq. (2)."""
    d_h = len(q)
    s = softmax([math.fsum(q[c] * row[c] for c in range(d_h)) / math.sqrt(d_h) for row in K])
    return [math.fsum(s[i] * V[i][c] for i in range(len(K))) for c in range(d_h)]


def top(values, count):
    """Indices of the `count` largest values, ties to the lower index, ascending."""
    order = sorted(range(len(values)), key=lambda i: (-values[i], i))
    return sorted(order[:count])


def sparq(q, K, V, r, k, realloc=True, tau_mode="l1", local_window=0):
    """Steps 1-3 for one query head.  q: [d_h], K, V: [S][d_h] (lists of floats).
    tau_mode: "l1" (Eq. 9), "sqrt_dh" or "sqrt_r" (the fixed temperatures of the ablation in
    Section 5.3); local_window: that many most recent positions are always kept."""
    d_h, S = len(q), len(K)
    k = min(k, S)
    # Step 1
    i1 = top([abs(x) for x in q], r)
    l1_all = math.fsum(abs(x) for x in q)
    l1_sel = math.fsum(abs(q[c]) for c in i1)
    tau = math.sqrt(d_h * l1_sel / l1_all) if l1_all > 0 else math.sqrt(d_h)
    tau = {"l1": tau, "sqrt_dh": math.sqrt(d_h), "sqrt_r": math.sqrt(r)}[tau_mode]
    z = [math.fsum(q[c] * K[i][c] for c in i1) / tau for i in range(S)]
    s_hat = softmax(z)
    # Step 2
    n_local = min(local_window, k)
    i2 = top(s_hat[:S - n_local], k - n_local) + list(range(S - n_local, S))   # top-k of the softmax output
    sub = softmax([math.fsum(q[c] * K[i][c] for c in range(d_h)) / math.sqrt(d_h) for i in i2])
    y3 = [math.fsum(sub[n] * V[i][c] for n, i in enumerate(i2)) for c in range(d_h)]
    # Step 3
    alpha = math.fsum(s_hat[i] for i in i2)
    v_bar = [math.fsum(V[i][c] for i in range(S)) / S for c in range(d_h)]
    y = [alpha * y3[c] + (1 - alpha) * v_bar[c] for c in range(d_h)] if realloc else y3
    return dict(i1=i1, tau=tau, z=z, s_hat=s_hat, i2=i2, alpha=alpha, y=y, y3=y3, v_bar=v_bar)


def sparse_v_reallocation(q, K, V, k):
    """Eq. (6): (s o m_s) V + (1 - s.m_s) v_bar with the exact scores s."""
    d_h, S = len(q), len(K)
    s = softmax([math.fsum(q[c] * row[c] for c in range(d_h)) / math.sqrt(d_h) for row in K])
    keep = top(s, min(k, S))
    v_bar = [math.fsum(V[i][c] for i in range(S)) / S for c in range(d_h)]
    mass = math.fsum(s[i] for i in keep)
    return [math.fsum(s[i] * V[i][c] for i in keep) + (1 - mass) * v_bar[c] for c in range(d_h)]


def sparq_group(qs, K, V, r, k, realloc=True):
    """Section 4 'Grouped query attention' for the g query heads qs (each [d_h]) of one KV head: the
    magnitudes |q| are summed over the group before the top-r, the approximate scores s-hat are summed over
    the group before the top-k; the temperature, alpha and the exact attention stay per query head.
    Returns the shared i1 and i2 and per head tau, alpha, y."""
    g, d_h, S = len(qs), len(qs[0]), len(K)
    k = min(k, S)
    i1 = top([math.fsum(abs(q[c]) for q in qs) for c in range(d_h)], r)
    s_hats, taus = [], []
    for q in qs:
        l1_all = math.fsum(abs(x) for x in q)
        l1_sel = math.fsum(abs(q[c]) for c in i1)
        tau = math.sqrt(d_h * l1_sel / l1_all) if l1_sel > 0 else math.sqrt(d_h)
        taus.append(tau)
        s_hats.append(softmax([math.fsum(q[c] * K[i][c] for c in i1) / tau for i in range(S)]))
    i2 = top([math.fsum(s[i] for s in s_hats) for i in range(S)], k)
    v_bar = [math.fsum(V[i][c] for i in range(S)) / S for c in range(d_h)]
    alphas, ys = [], []
    for q, s_hat in zip(qs, s_hats):
        sub = softmax([math.fsum(q[c] * K[i][c] for c in range(d_h)) / math.sqrt(d_h) for i in i2])
        y3 = [math.fsum(sub[n] * V[i][c] for n, i in enumerate(i2)) for c in range(d_h)]
        alpha = math.fsum(s_hat[i] for i in i2)
        alphas.append(alpha)
        ys.append([alpha * y3[c] + (1 - alpha) * v_bar[c] for c in range(d_h)] if realloc else y3)
    return dict(i1=i1, i2=i2, tau=taus, alpha=alphas, y=ys)
