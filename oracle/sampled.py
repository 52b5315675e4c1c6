"""Selected rows of the attention of ONE long sample, in fp64 numpy.

TEST INFRASTRUCTURE ONLY, like the rest of this directory.  The C oracle walks
over whole samples, one (sample, head) per thread; for a single sample of tens
of thousands of tokens and a couple of heads that takes minutes.  The functions
here evaluate the same definition (section 2.2.1 (1): softmax attention over
the visible keys of the row's own sample; masks and notation as in
attn_oracle.c) for chosen rows only, each row written out on its own:

    s_ij = scale q_i . k_j   for lo(i) <= j < vis(i)
    LSE_i = ln sum_j exp(s_ij),  p_ij = exp(s_ij - LSE_i),  O_i = sum_j p_ij v_j
    delta_i = dO_i . O_i,  dS_ij = p_ij (dO_i . v_j - delta_i)
    dQ_i = scale sum_j dS_ij k_j
    dK_j = scale sum_h sum_i dS_ij q_i,   dV_j = sum_h sum_i p_ij dO_i   (h over the heads of the group)

Only causal masks are covered (optionally with a sliding window of W keys):
lo(i) = max(0, i + 1 - W), vis(i) = i + 1.  Inputs are one sample: q, dout
[L, Hq, D], k, v [L, Hkv, D], values already rounded to the storage type.
The tests pin these functions to the C oracle on short samples.
"""
import numpy as np


def _bounds(i, window):
    return (0 if window is None else max(0, i + 1 - window)), i + 1


def row_forward(q, k, v, scale, i, h, window=None):
    """(O_i [D], LSE_i) of query row i, head h."""
    g = h // (q.shape[1] // k.shape[1])
    lo, hi = _bounds(i, window)
    s = scale * (k[lo:hi, g].astype(np.float64) @ q[i, h].astype(np.float64))
    m = s.max()
    z = np.exp(s - m).sum()
    p = np.exp(s - m) / z
    return p @ v[lo:hi, g].astype(np.float64), m + np.log(z)


def row_dq(q, k, v, dout, scale, i, h, window=None):
    """dQ_i [D] of query row i, head h."""
    g = h // (q.shape[1] // k.shape[1])
    lo, hi = _bounds(i, window)
    kk, vv = k[lo:hi, g].astype(np.float64), v[lo:hi, g].astype(np.float64)
    s = scale * (kk @ q[i, h].astype(np.float64))
    p = np.exp(s - s.max())
    p /= p.sum()
    do = dout[i, h].astype(np.float64)
    delta = do @ (p @ vv)
    ds = p * (vv @ do - delta)
    return scale * (ds @ kk)


def row_stats(q, k, v, dout, scale, window=None, rows_per_pass=256):
    """(LSE [Hq, L], delta [Hq, L]) of every query row: what key_row_dk_dv needs of the rows that see a key.
    The same definition as row_forward, evaluated for `rows_per_pass` rows at a time with a dense score
    matrix and an explicit mask, so that a key near the start of a long sample (seen by every later row)
    does not cost one pass over the keys per row."""
    L, Hq, D = q.shape
    G = Hq // k.shape[1]
    lse = np.zeros((Hq, L))
    delta = np.zeros((Hq, L))
    cols = np.arange(L)
    for h in range(Hq):
        kk, vv = k[:, h // G].astype(np.float64), v[:, h // G].astype(np.float64)
        for r0 in range(0, L, rows_per_pass):
            rows = np.arange(r0, min(L, r0 + rows_per_pass))
            s = scale * (q[rows, h].astype(np.float64) @ kk.T)
            seen = cols[None, :] <= rows[:, None]
            if window is not None:
                seen &= rows[:, None] - cols[None, :] < window
            s = np.where(seen, s, -np.inf)
            m = s.max(axis=1)
            e = np.exp(s - m[:, None])
            z = e.sum(axis=1)
            lse[h, rows] = m + np.log(z)
            o = (e / z[:, None]) @ vv
            delta[h, rows] = (dout[rows, h].astype(np.float64) * o).sum(axis=1)
    return lse, delta


def key_row_dk_dv(q, k, v, dout, scale, j, g, window=None, stats=None):
    """(dK_j [D], dV_j [D]) of key row j, KV head g: sums over every query row that sees key j and over
    the heads of the group.  LSE and delta of those rows are computed here, row by row, unless `stats`
    (the pair row_stats returns) hands them over."""
    L, Hq, D = q.shape
    G = Hq // k.shape[1]
    last = L - 1 if window is None else min(L - 1, j + window - 1)
    dk = np.zeros(D)
    dv = np.zeros(D)
    kj, vj = k[j, g].astype(np.float64), v[j, g].astype(np.float64)
    for h in range(g * G, (g + 1) * G):
        if stats is not None:
            rows = slice(j, last + 1)
            qi, do = q[rows, h].astype(np.float64), dout[rows, h].astype(np.float64)
            p = np.exp(scale * (qi @ kj) - stats[0][h, rows])
            ds = p * (do @ vj - stats[1][h, rows])
            dk += scale * (ds @ qi)
            dv += p @ do
            continue
        for i in range(j, last + 1):
            o, lse = row_forward(q, k, v, scale, i, h, window)
            qi, do = q[i, h].astype(np.float64), dout[i, h].astype(np.float64)
            p = np.exp(scale * (qi @ kj) - lse)
            ds = p * (do @ vj - do @ o)
            dk += scale * ds * qi
            dv += p * do
    return dk, dv
