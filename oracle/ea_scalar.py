"""Scalar re-statement of the Expected-Attention compress step.  TEST INFRASTRUCTURE ONLY.

Pure-Python loops over plain floats (IEEE double), written from the equations one index at a
time: no numpy arithmetic, no matrices.  It exists to cross-check ea_oracle.py on tiny inputs
(a second, independently typed coding of Eq. 1 and Eq. 5-9 and of the top-k rule), and is far
too slow for anything else.  Same readings of the paper as ea_oracle.py.
"""
import math


def _pair(c, half, interleaved):
    return (2 * c, 2 * c + 1) if interleaved else (c, c + half)


def averaged_rotation(t_next, T, theta):
    """(c-bar, s-bar) of one channel pair: the mean over j = 0..T-1 of cos / sin of
    (t_next + j) * theta -- the two independent entries of that pair's 2x2 block of R-bar."""
    cb = sb = 0.0
    for j in range(T):
        cb += math.cos((t_next + j) * theta)
        sb += math.sin((t_next + j) * theta)
    return cb / T, sb / T


def query_stats(q, q_pos0, inv_freq, t_next, T, ddof=0, q_is_rotated=True, interleaved=False):
    """q: w lists of d floats (one query head).  Returns (mu[d], Sigma[d][d]) of Eq. 6."""
    w, d = len(q), len(q[0])
    half = d // 2
    # u_s = R_{p_s}^T q_s : turn every pair back by its own angle
    u = [[0.0] * d for _ in range(w)]
    for s in range(w):
        for c in range(half):
            a, b = _pair(c, half, interleaved)
            if q_is_rotated:
                ang = (q_pos0 + s) * inv_freq[c]
                co, si = math.cos(ang), math.sin(ang)
                u[s][a] = co * q[s][a] + si * q[s][b]
                u[s][b] = -si * q[s][a] + co * q[s][b]
            else:
                u[s][a], u[s][b] = q[s][a], q[s][b]
    m = [sum(u[s][c] for s in range(w)) / w for c in range(d)]
    S = [[sum((u[s][i] - m[i]) * (u[s][j] - m[j]) for s in range(w)) / (w - ddof)
          for j in range(d)] for i in range(d)]
    # R-bar acts on each pair as [[cb, -sb], [sb, cb]]
    rb = [averaged_rotation(t_next, T, inv_freq[c]) for c in range(half)]

    def apply(vec):
        out = [0.0] * d
        for c in range(half):
            a, b = _pair(c, half, interleaved)
            cb, sb = rb[c]
            out[a] = cb * vec[a] - sb * vec[b]
            out[b] = sb * vec[a] + cb * vec[b]
        return out

    mu = apply(m)
    left = [apply([S[i][j] for i in range(d)]) for j in range(d)]      # column j of R-bar S
    RS = [[left[j][i] for j in range(d)] for i in range(d)]
    sigma = [apply(RS[i]) for i in range(d)]                            # row i times R-bar^T
    return mu, sigma


def scores(k, v, mus, sigmas, epsilon):
    """One KV head.  k, v: n lists of d floats; mus / sigmas: the G heads of its group."""
    n, d = len(k), len(k[0])
    G = len(mus)
    att = [[0.0] * n for _ in range(G)]
    for g in range(G):
        lg = []
        for i in range(n):
            lin = sum(mus[g][c] * k[i][c] for c in range(d)) / math.sqrt(d)
            quad = sum(k[i][a] * sigmas[g][a][b] * k[i][b]
                       for a in range(d) for b in range(d)) / (2.0 * d)
            lg.append(lin + quad)
        mx = max(lg)
        z = [math.exp(x - mx) for x in lg]
        tot = sum(z)
        att[g] = [x / tot for x in z]
    out = []
    for i in range(n):
        a = sum(att[g][i] for g in range(G)) / G
        out.append((a + epsilon) * math.sqrt(sum(x * x for x in v[i])))
    return out


def select(sc, n_kept):
    """Repeatedly take the best remaining pair (first one on ties); ascending positions."""
    left = list(range(len(sc)))
    kept = []
    for _ in range(n_kept):
        best = left[0]
        for i in left:
            if sc[i] > sc[best]:
                best = i
        kept.append(best)
        left.remove(best)
    return sorted(kept)
