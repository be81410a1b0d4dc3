"""The paper's runtime model (Sec. 3.3) fitted to what the library measures on this GPU.

    t(s) = N * (t_L(b, s) + s * t_S(b, 1)) / (l(s) + 1)                      (Eq. 1-3, 7)
    t_L(b, s) ~ alpha_b * s + beta                                           (Sec. 3.3.1, the linear approximation)
    l(s)      ~ c * s**gamma                                                 (Eq. 5)

Inputs are plain numbers: per-pass latencies from `spec_profile_and_choose_s` / `bench.py`'s verify grid, draft
pass latencies, accepted-length samples or histograms from `spec_read_output`.  Nothing here touches the GPU;
it explains the profiled look-up table in the paper's own terms (why s_opt falls as the batch grows).

All functions are pure and take / return Python floats and lists.
"""
import math


def fit_line(xs, ys):
    """Least-squares (slope, intercept) of y ~ slope * x + intercept: the paper's t_L(b, s) ~ alpha_b * s + beta
    for one batch size (Sec. 3.3.1)."""
    n = len(xs)
    if n < 2 or n != len(ys):
        raise ValueError("need at least two (x, y) pairs")
    mx, my = sum(xs) / n, sum(ys) / n
    sxx = sum((x - mx) ** 2 for x in xs)
    if sxx == 0.0:
        raise ValueError("all x are equal")
    slope = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sxx
    return slope, my - slope * mx


def l_from_samples(l_samples, s):
    """Eq. 4: mean of min(l_i, s) over measured accepted-prefix lengths l_i."""
    if not l_samples:
        raise ValueError("no samples")
    return sum(min(int(l), s) for l in l_samples) / len(l_samples)


def l_from_histogram(hist, s):
    """Eq. 4 on a histogram: hist[k] = number of rounds that accepted exactly k proposals when s_run = len(hist) - 1
    were offered.  A round that accepted all s_run may have matched further, so the estimate is exact for s <= s_run."""
    if s > len(hist) - 1:
        raise ValueError("histogram was taken with fewer proposals than s")
    total = sum(hist)
    if total <= 0:
        raise ValueError("empty histogram")
    return sum(min(k, s) * cnt for k, cnt in enumerate(hist)) / total


def l_iid(alpha, s):
    """Eq. 6 when every proposal is right with probability alpha independently: sum_{i=1..s} alpha**i."""
    if alpha >= 1.0:
        return float(s)
    return alpha * (1.0 - alpha ** s) / (1.0 - alpha)


def fit_power(ss, ls):
    """Least squares of log l = log c + gamma * log s over s >= 1, l > 0: the (c, gamma) of Eq. 5."""
    pts = [(math.log(s), math.log(l)) for s, l in zip(ss, ls) if s >= 1 and l > 0]
    if len(pts) < 2:
        raise ValueError("need two points with s >= 1 and l > 0")
    g, logc = fit_line([p[0] for p in pts], [p[1] for p in pts])
    return math.exp(logc), g


def total_time(N, t_L, t_S, s, l):
    """Eq. 1-3: N / (l + 1) iterations of one verification pass and s draft steps."""
    return N * (t_L + s * t_S) / (l + 1.0)


def model_time(s, alpha_b, beta, c, gamma, N=1.0):
    """Eq. 7 in its approximated form, t_S merged into alpha_b as the paper does."""
    return N * (alpha_b * s + beta) / (c * s ** gamma + 1.0)


def delta(s, alpha_b, beta, c, gamma):
    """Left-hand side of Eq. 11, K * alpha_b * s**gamma - L * s**(gamma - 1) + alpha_b with K = (1 - gamma) * c and
    L = c * beta * gamma: the numerator of dt/ds.  Increasing in s and in alpha_b for 0 < gamma < 1."""
    K, L = (1.0 - gamma) * c, c * beta * gamma
    return K * alpha_b * s ** gamma - L * s ** (gamma - 1.0) + alpha_b


def s_opt_continuous(alpha_b, beta, c, gamma, s_hi=1.0e4):
    """Root of Eq. 11 over real s > 0 by bisection (delta is increasing in s, -inf at 0+).  Returns s_hi when
    the model keeps improving up to s_hi (alpha_b <= 0: extra proposals cost nothing)."""
    if not (0.0 < gamma < 1.0) or c <= 0.0 or beta <= 0.0:
        raise ValueError("the model needs 0 < gamma < 1, c > 0, beta > 0")
    if alpha_b <= 0.0 or delta(s_hi, alpha_b, beta, c, gamma) < 0.0:
        return s_hi
    lo, hi = 1.0e-9, s_hi
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if delta(mid, alpha_b, beta, c, gamma) < 0.0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def s_opt_grid(s_list, t_L_by_s, t_S, l_of_s, N=1.0):
    """The profiling stage's arg-min written on the model's terms: the s of s_list minimising Eq. 1-3 with the
    measured t_L(b, s), t_S(b, 1) and l(s) (l_of_s[s] for every s of s_list); ties go to the smaller s."""
    best_s, best_t = None, None
    for s, tl in sorted(zip(s_list, t_L_by_s)):
        t = total_time(N, tl, t_S, s, l_of_s[s])
        if best_t is None or t < best_t:
            best_s, best_t = s, t
    return best_s


def explain(batch_sizes, s_list, t_L_grid, t_S_by_b, l_of_s):
    """Fit the model per batch size and set it beside the measured optimum.

    t_L_grid[i][k]: verification latency at batch_sizes[i] with s_list[k] proposals; t_S_by_b[i]: one draft
    step; l_of_s[s]: expected accepted proposals for s = 0..max(s_list).  Returns c and gamma (fitted once: they
    do not depend on the batch size) and one dict per batch size: alpha_b, alpha_b with t_S merged in (as in
    Eq. 7), beta, the continuous root of Eq. 11, and the arg-min of Eq. 1-3 over the measured s."""
    S = max(s_list)
    c, gamma = fit_power(list(range(1, S + 1)), [l_of_s[s] for s in range(1, S + 1)])
    out = {"c": c, "gamma": gamma, "rows": []}
    for b, row, ts in zip(batch_sizes, t_L_grid, t_S_by_b):
        a, beta = fit_line(list(s_list), list(row))
        a_merged = a + ts
        root = s_opt_continuous(a_merged, beta, c, gamma) if 0.0 < gamma < 1.0 and beta > 0 else float("nan")
        out["rows"].append({"B": b, "alpha_b": a, "alpha_b_with_draft": a_merged, "beta": beta,
                            "s_opt_model": root, "s_opt_grid": s_opt_grid(s_list, row, ts, l_of_s)})
    return out
