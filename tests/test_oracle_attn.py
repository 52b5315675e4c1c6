"""Pins for the fp64 attention oracle (CPU only).

The paper prints no formula and no worked example for attention, so the oracle
is pinned to what the mathematics fixes: closed forms, invariants, reductions
to library routines (numpy einsum, PyTorch CPU scaled_dot_product_attention in
float64), brute-force finite differences, and the defining property of the
method (paper section 2.2.1 (2) / 3.2: packing changes nothing in the result).
Each test is chosen so that a plausible slip in the oracle (wrong mask edge,
wrong head mapping, dropped scale, log base, transposed operand, missing term
in a gradient) fails at least one of them.
"""
import numpy as np
import pytest
import torch

from oracle import attn as oa
from paper_2603_11101_amd import workloads as wl

MODES = [oa.MASK_CAUSAL, oa.MASK_PREFIX_BIDIR_SUFFIX, oa.MASK_PREFIX_CAUSAL_SUFFIX]


def stream(seed, lens, Hq, Hkv, D, prefix="rand"):
    cu, pl, q, k, v, do = wl.random_stream(seed, lens, Hq, Hkv, D, prefix_frac=-1.0)
    return cu, pl, q, k, v, do


def dense_mask(L, P, mode):
    i = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    if mode == oa.MASK_CAUSAL:
        return j <= i
    if mode == oa.MASK_PREFIX_BIDIR_SUFFIX:
        return np.where(i < P, j < P, np.ones_like(j, dtype=bool))
    return np.where(i < P, j < P, j <= i)


def test_single_token_samples():
    # one-token samples: softmax over one key is 1, so O = V, LSE = scale q.k,
    # dV = sum of dO over the group's query heads, dQ = dK = 0
    Hq, Hkv, D = 4, 2, 8
    cu, pl, q, k, v, do = stream(1, [1, 1, 1], Hq, Hkv, D)
    for mode in MODES:
        pl1 = None if mode == oa.MASK_CAUSAL else np.array([1, 0, 1], dtype=np.int32)
        out, lse = oa.attn_fwd(q, k, v, cu, pl1, scale=0.37, mask_mode=mode)
        dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, pl1, scale=0.37, mask_mode=mode)
        for t in range(3):
            for h in range(Hq):
                g = h // (Hq // Hkv)
                assert np.array_equal(out[t, h], v[t, g].astype(np.float64))
                assert lse[h, t] == pytest.approx(0.37 * float(np.dot(q[t, h].astype(np.float64), k[t, g].astype(np.float64))), rel=1e-14)
            for g in range(Hkv):
                want = do[t, g * 2:(g + 1) * 2].astype(np.float64).sum(axis=0)
                assert np.allclose(dv[t, g], want, rtol=0, atol=1e-15)
        assert np.abs(dq).max() < 1e-15 and np.abs(dk).max() < 1e-15


@pytest.mark.parametrize("mode", MODES)
def test_uniform_keys_closed_form(mode):
    # every key of a sample equal: p_ij = 1 / #A(i), O_i = mean of V over A(i),
    # LSE_i = scale q_i.k + ln #A(i).  Pins the mask geometry and the log base.
    Hq, Hkv, D = 2, 1, 4
    lens = [7, 12]
    cu, _, q, k, v, do = stream(2, lens, Hq, Hkv, D)
    pl = np.array([3, 12], dtype=np.int32)
    for s in range(2):
        k[cu[s]:cu[s + 1]] = k[cu[s]]
    scale = 0.5
    out, lse = oa.attn_fwd(q, k, v, cu, None if mode == oa.MASK_CAUSAL else pl, scale=scale, mask_mode=mode)
    for s, L in enumerate(lens):
        c = cu[s]
        P = pl[s]
        for i in range(L):
            if mode == oa.MASK_CAUSAL:
                cnt = i + 1
            elif mode == oa.MASK_PREFIX_BIDIR_SUFFIX:
                cnt = P if i < P else L
            else:
                cnt = P if i < P else i + 1
            for h in range(Hq):
                mean_v = v[c:c + cnt, 0].astype(np.float64).mean(axis=0)
                assert np.allclose(out[c + i, h], mean_v, rtol=1e-13, atol=1e-14)
                s_i = scale * float(np.dot(q[c + i, h].astype(np.float64), k[c, 0].astype(np.float64)))
                assert lse[h, c + i] == pytest.approx(s_i + np.log(cnt), abs=1e-12)


@pytest.mark.parametrize("mode", MODES)
def test_rows_of_p_sum_to_one_and_rows_of_ds_to_zero(mode):
    Hq, Hkv, D = 4, 2, 8
    cu, pl, q, k, v, do = stream(3, [9, 1, 14], Hq, Hkv, D)
    plm = None if mode == oa.MASK_CAUSAL else pl
    for s in range(3):
        for h in range(Hq):
            p, ds = oa.attn_probs(q, k, v, do, cu, plm, s, h, mask_mode=mode)
            L = cu[s + 1] - cu[s]
            P = 0 if plm is None else plm[s]
            assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
            assert np.abs(ds.sum(axis=1)).max() < 1e-13
            assert np.all((p > 0) == dense_mask(L, P, mode))


@pytest.mark.parametrize("mode", MODES)
def test_dense_library_reduction(mode):
    # single-sample stream against numpy einsum and torch CPU SDPA (float64, boolean mask)
    Hq, Hkv, D, L = 4, 2, 16, 33
    cu, _, q, k, v, do = stream(4, [L], Hq, Hkv, D)
    P = 20
    pl = None if mode == oa.MASK_CAUSAL else np.array([P], dtype=np.int32)
    scale = 1.0 / np.sqrt(D)
    out, lse = oa.attn_fwd(q, k, v, cu, pl, scale=scale, mask_mode=mode)
    mask = dense_mask(L, P, mode)
    G = Hq // Hkv
    kk = np.repeat(k.astype(np.float64), G, axis=1)
    vv = np.repeat(v.astype(np.float64), G, axis=1)
    s = np.einsum("ihd,jhd->hij", q.astype(np.float64), kk) * scale
    s = np.where(mask[None], s, -np.inf)
    m = s.max(axis=2, keepdims=True)
    e = np.exp(s - m)
    p = e / e.sum(axis=2, keepdims=True)
    ref = np.einsum("hij,jhd->ihd", p, vv)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
    assert np.allclose(lse, (m[..., 0] + np.log(e.sum(axis=2))), rtol=0, atol=1e-12)
    tq = torch.from_numpy(q.astype(np.float64)).permute(1, 0, 2)[None]
    tk = torch.from_numpy(kk).permute(1, 0, 2)[None]
    tv = torch.from_numpy(vv).permute(1, 0, 2)[None]
    tref = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, attn_mask=torch.from_numpy(mask)[None, None], scale=scale)
    assert np.allclose(out, tref[0].permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("mode", MODES)
def test_gradients_against_torch_autograd(mode):
    # third opinion on the backward: autograd through the dense float64 definition
    Hq, Hkv, D = 4, 2, 8
    lens = [11, 6]
    cu, pl, q, k, v, do = stream(5, lens, Hq, Hkv, D)
    plm = None if mode == oa.MASK_CAUSAL else pl
    scale = 0.3
    dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, plm, scale=scale, mask_mode=mode)
    G = Hq // Hkv
    for s, L in enumerate(lens):
        c = cu[s]
        P = 0 if plm is None else plm[s]
        tq = torch.tensor(q[c:c + L].astype(np.float64), requires_grad=True)
        tk = torch.tensor(k[c:c + L].astype(np.float64), requires_grad=True)
        tv = torch.tensor(v[c:c + L].astype(np.float64), requires_grad=True)
        mask = torch.from_numpy(dense_mask(L, P, mode))
        sc = torch.einsum("ihd,jhd->hij", tq, tk.repeat_interleave(G, dim=1)) * scale
        sc = sc.masked_fill(~mask[None], float("-inf"))
        o = torch.einsum("hij,jhd->ihd", torch.softmax(sc, dim=-1), tv.repeat_interleave(G, dim=1))
        (o * torch.tensor(do[c:c + L].astype(np.float64))).sum().backward()
        assert np.allclose(dq[c:c + L], tq.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dk[c:c + L], tk.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dv[c:c + L], tv.grad.numpy(), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("mode", MODES)
def test_finite_differences(mode):
    # central differences of loss = sum(O * dO) on tiny inputs, every input element
    Hq, Hkv, D = 2, 1, 4
    lens = [1, 3, 5]
    cu, pl, q, k, v, do = stream(6, lens, Hq, Hkv, D)
    plm = None if mode == oa.MASK_CAUSAL else pl
    scale = 0.7
    dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, plm, scale=scale, mask_mode=mode)

    # the oracle takes float32 inputs; perturb in float32-representable steps
    h = np.float32(2.0 ** -10)

    def loss(qq, kk, vv):
        out, _ = oa.attn_fwd(qq, kk, vv, cu, plm, scale=scale, mask_mode=mode)
        return float((out * do.astype(np.float64)).sum())

    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for idx in np.ndindex(*x.shape):
            xp = x.copy()
            xm = x.copy()
            xp[idx] += h
            xm[idx] -= h
            args_p = {"q": q, "k": k, "v": v}
            args_m = dict(args_p)
            args_p[name] = xp
            args_m[name] = xm
            step = float(xp[idx].astype(np.float64) - xm[idx].astype(np.float64))
            fd = (loss(args_p["q"], args_p["k"], args_p["v"]) - loss(args_m["q"], args_m["k"], args_m["v"])) / step
            assert fd == pytest.approx(g[idx], rel=2e-5, abs=2e-6), (name, idx)


def test_key_shift_and_value_scaling():
    # adding u to every key of a sample leaves O unchanged and moves LSE_i by scale q_i.u;
    # scaling V scales O
    Hq, Hkv, D = 2, 2, 8
    cu, pl, q, k, v, do = stream(7, [10, 5], Hq, Hkv, D)
    u = wl.round_to_bf16(np.random.default_rng(0).standard_normal(D).astype(np.float32) * 0.25)
    out0, lse0 = oa.attn_fwd(q, k, v, cu, None, scale=0.4)
    # keep the shifted keys exactly representable: K and u are bf16 numbers, their float32 sum is exact here
    k2 = k.copy()
    k2[cu[1]:cu[2]] += u
    assert np.array_equal(k2[cu[1]:cu[2]].astype(np.float64), k[cu[1]:cu[2]].astype(np.float64) + u.astype(np.float64))
    out1, lse1 = oa.attn_fwd(q, k2, v, cu, None, scale=0.4)
    assert np.allclose(out1, out0, rtol=1e-12, atol=1e-13)
    shift = 0.4 * np.einsum("ihd,d->hi", q[cu[1]:cu[2]].astype(np.float64), u.astype(np.float64))
    assert np.allclose(lse1[:, cu[1]:cu[2]] - lse0[:, cu[1]:cu[2]], shift, atol=1e-12)
    assert np.array_equal(lse1[:, :cu[1]], lse0[:, :cu[1]])
    out2, _ = oa.attn_fwd(q, k, v * np.float32(2.0), cu, None, scale=0.4)
    assert np.allclose(out2, 2.0 * out0, rtol=1e-14)


def test_gqa_equals_mha_with_repeated_heads():
    Hq, Hkv, D = 6, 2, 8
    cu, pl, q, k, v, do = stream(8, [13, 4], Hq, Hkv, D)
    G = Hq // Hkv
    out, lse = oa.attn_fwd(q, k, v, cu, pl)
    dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, pl)
    kr = np.repeat(k, G, axis=1)
    vr = np.repeat(v, G, axis=1)
    out2, lse2 = oa.attn_fwd(q, kr, vr, cu, pl)
    dq2, dk2, dv2 = oa.attn_bwd(q, kr, vr, do, cu, pl)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2) and np.array_equal(dq, dq2)
    assert np.allclose(dk, dk2.reshape(-1, Hkv, G, D).sum(axis=2), rtol=1e-13, atol=1e-14)
    assert np.allclose(dv, dv2.reshape(-1, Hkv, G, D).sum(axis=2), rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("mode", MODES)
def test_packing_invariance_permutation_and_no_leak(mode):
    Hq, Hkv, D = 4, 2, 8
    lens = [5, 17, 1, 9]
    cu, pl, q, k, v, do = stream(9, lens, Hq, Hkv, D)
    plm = None if mode == oa.MASK_CAUSAL else pl
    out, lse = oa.attn_fwd(q, k, v, cu, plm, mask_mode=mode)
    dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, plm, mask_mode=mode)
    # each sample alone gives bit-identical rows
    for s, L in enumerate(lens):
        c = cu[s]
        sl = slice(c, c + L)
        cu1 = np.array([0, L], dtype=np.int32)
        pl1 = None if plm is None else plm[s:s + 1]
        o1, l1 = oa.attn_fwd(q[sl], k[sl], v[sl], cu1, pl1, mask_mode=mode)
        g1 = oa.attn_bwd(q[sl], k[sl], v[sl], do[sl], cu1, pl1, mask_mode=mode)
        assert np.array_equal(out[sl], o1) and np.array_equal(lse[:, sl], l1)
        assert np.array_equal(dq[sl], g1[0]) and np.array_equal(dk[sl], g1[1]) and np.array_equal(dv[sl], g1[2])
    # reversing the sample order permutes the results
    order = [3, 2, 1, 0]
    rows = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in order])
    cu_r = np.zeros(5, dtype=np.int32)
    cu_r[1:] = np.cumsum([lens[s] for s in order])
    pl_r = None if plm is None else plm[order]
    out_r, lse_r = oa.attn_fwd(q[rows], k[rows], v[rows], cu_r, pl_r, mask_mode=mode)
    assert np.array_equal(out_r, out[rows]) and np.array_equal(lse_r, lse[:, rows])
    # NaN/Inf in another sample never reaches this one
    q2, k2, v2, do2 = q.copy(), k.copy(), v.copy(), do.copy()
    bad = slice(cu[1], cu[2])
    q2[bad] = np.nan
    k2[bad] = np.inf
    v2[bad] = np.nan
    do2[bad] = np.nan
    out_n, lse_n = oa.attn_fwd(q2, k2, v2, cu, plm, mask_mode=mode)
    g_n = oa.attn_bwd(q2, k2, v2, do2, cu, plm, mask_mode=mode)
    keep = np.r_[0:cu[1], cu[2]:cu[4]]
    assert np.array_equal(out_n[keep], out[keep]) and np.array_equal(lse_n[:, keep], lse[:, keep])
    assert np.array_equal(g_n[0][keep], dq[keep]) and np.array_equal(g_n[1][keep], dk[keep]) and np.array_equal(g_n[2][keep], dv[keep])


def test_prefix_degenerate_cases_reduce_to_bidirectional_and_causal():
    Hq, Hkv, D = 2, 1, 8
    lens = [6, 9]
    cu, _, q, k, v, do = stream(10, lens, Hq, Hkv, D)
    full = np.array(lens, dtype=np.int32)
    zero = np.zeros(2, dtype=np.int32)
    a, la = oa.attn_fwd(q, k, v, cu, full, mask_mode=oa.MASK_PREFIX_BIDIR_SUFFIX)
    b, lb = oa.attn_fwd(q, k, v, cu, zero, mask_mode=oa.MASK_PREFIX_BIDIR_SUFFIX)
    assert np.array_equal(a, b) and np.array_equal(la, lb)       # P = L and P = 0: fully bidirectional
    c, lc = oa.attn_fwd(q, k, v, cu, zero, mask_mode=oa.MASK_PREFIX_CAUSAL_SUFFIX)
    d, ld = oa.attn_fwd(q, k, v, cu, None, mask_mode=oa.MASK_CAUSAL)
    assert np.array_equal(c, d) and np.array_equal(lc, ld)       # causal suffix with empty prefix = causal


def test_sel_restricts_to_chosen_samples_and_zero_length_samples_are_legal():
    Hq, Hkv, D = 2, 2, 4
    lens = [4, 0, 6, 3]
    cu, pl, q, k, v, do = stream(11, lens, Hq, Hkv, D)
    out, lse = oa.attn_fwd(q, k, v, cu, None)
    out_s, lse_s = oa.attn_fwd(q, k, v, cu, None, sel=[2])
    sl = slice(cu[2], cu[3])
    assert np.array_equal(out_s[sl], out[sl]) and np.isnan(out_s[:cu[2]]).all() and np.isnan(out_s[cu[3]:]).all()
    assert not np.isnan(out).any() and not np.isnan(lse).any()


# ---------------------------------------------------------------- three-block mask
#
# Blocks [0, P), [P, P2), [P2, L): a row sees its own block and the blocks before it.  The dense mask
# below is written from that sentence (by block index), not from the oracle's visible() rule.

def three_block_mask(L, P, P2):
    block = (np.arange(L) >= P).astype(int) + (np.arange(L) >= P2).astype(int)
    return block[None, :] <= block[:, None]


def test_three_block_against_dense_definition_and_autograd():
    Hq, Hkv, D = 4, 2, 8
    lens = [23, 9, 14]
    ends = np.array([[7, 15], [0, 4], [14, 14]], dtype=np.int32)   # ordinary; empty first block; empty last two
    cu, _, q, k, v, do = stream(11, lens, Hq, Hkv, D)
    scale = 0.41
    out, lse = oa.attn_fwd(q, k, v, cu, ends, scale=scale, mask_mode=oa.MASK_THREE_BLOCK)
    dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, ends, scale=scale, mask_mode=oa.MASK_THREE_BLOCK)
    G = Hq // Hkv
    for s, L in enumerate(lens):
        c = cu[s]
        mask = torch.from_numpy(three_block_mask(L, ends[s, 0], ends[s, 1]))
        tq = torch.tensor(q[c:c + L].astype(np.float64), requires_grad=True)
        tk = torch.tensor(k[c:c + L].astype(np.float64), requires_grad=True)
        tv = torch.tensor(v[c:c + L].astype(np.float64), requires_grad=True)
        sc = torch.einsum("ihd,jhd->hij", tq, tk.repeat_interleave(G, dim=1)) * scale
        sc = sc.masked_fill(~mask[None], float("-inf"))
        o = torch.einsum("hij,jhd->ihd", torch.softmax(sc, dim=-1), tv.repeat_interleave(G, dim=1))
        (o * torch.tensor(do[c:c + L].astype(np.float64))).sum().backward()
        assert np.allclose(out[c:c + L], o.detach().numpy(), rtol=1e-12, atol=1e-13)
        assert np.allclose(lse[:, c:c + L], torch.logsumexp(sc, dim=-1).detach().numpy(), rtol=0, atol=1e-12)
        assert np.allclose(dq[c:c + L], tq.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dk[c:c + L], tk.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dv[c:c + L], tv.grad.numpy(), rtol=1e-11, atol=1e-12)
        for h in range(Hq):
            p, ds = oa.attn_probs(q, k, v, do, cu, ends, s, h, scale=scale, mask_mode=oa.MASK_THREE_BLOCK)
            assert np.all((p > 0) == mask.numpy())
            assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14) and np.allclose(ds.sum(axis=1), 0.0, atol=1e-13)


def test_three_block_degenerate_cases_reduce_to_the_prefix_mask():
    Hq, Hkv, D = 2, 1, 8
    lens = [19, 8]
    cu, _, q, k, v, do = stream(12, lens, Hq, Hkv, D)
    P = np.array([6, 3], dtype=np.int32)
    L = np.array(lens, dtype=np.int32)
    want = oa.attn_fwd(q, k, v, cu, P, mask_mode=oa.MASK_PREFIX_BIDIR_SUFFIX)
    gwant = oa.attn_bwd(q, k, v, do, cu, P, mask_mode=oa.MASK_PREFIX_BIDIR_SUFFIX)
    for ends in (np.stack([P, P], axis=1), np.stack([P, L], axis=1)):    # no middle block; no last block
        got = oa.attn_fwd(q, k, v, cu, ends, mask_mode=oa.MASK_THREE_BLOCK)
        ggot = oa.attn_bwd(q, k, v, do, cu, ends, mask_mode=oa.MASK_THREE_BLOCK)
        assert all(np.array_equal(a, b) for a, b in zip(got + ggot, want + gwant))
    # uniform keys: LSE_i = scale q_i.k + ln(number of visible keys)
    k1 = np.repeat(k[:1], len(k), axis=0)
    ends = np.array([[5, 12], [2, 7]], dtype=np.int32)
    _, lse = oa.attn_fwd(q, k1, v, cu, ends, scale=0.5, mask_mode=oa.MASK_THREE_BLOCK)
    for s, Ls in enumerate(lens):
        for i in range(Ls):
            nvis = ends[s, 0] if i < ends[s, 0] else ends[s, 1] if i < ends[s, 1] else Ls
            for h in range(Hq):
                want_lse = 0.5 * float(q[cu[s] + i, h].astype(np.float64) @ k1[0, 0].astype(np.float64)) + np.log(nvis)
                assert abs(lse[h, cu[s] + i] - want_lse) < 1e-12


# ---------------------------------------------------------------- sliding window
#
# Row i sees the W most recent keys, itself included: 0 <= i - j < W.  The dense mask below is that
# sentence as a band matrix, not the oracle's first_visible() / visible() pair.

def window_mask(L, W):
    d = np.arange(L)[:, None] - np.arange(L)[None, :]
    return (d >= 0) & (d < W)


def test_sliding_window_against_dense_definition_and_autograd():
    Hq, Hkv, D = 4, 2, 8
    lens = [23, 9, 14, 1]
    W = np.array([5, 1, 40, 3], dtype=np.int32)         # ordinary; self only; wider than the sample; one token
    cu, _, q, k, v, do = stream(21, lens, Hq, Hkv, D)
    scale = 0.37
    out, lse = oa.attn_fwd(q, k, v, cu, W, scale=scale, mask_mode=oa.MASK_SLIDING_WINDOW)
    dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, W, scale=scale, mask_mode=oa.MASK_SLIDING_WINDOW)
    G = Hq // Hkv
    for s, L in enumerate(lens):
        c = cu[s]
        mask = torch.from_numpy(window_mask(L, int(W[s])))
        tq = torch.tensor(q[c:c + L].astype(np.float64), requires_grad=True)
        tk = torch.tensor(k[c:c + L].astype(np.float64), requires_grad=True)
        tv = torch.tensor(v[c:c + L].astype(np.float64), requires_grad=True)
        sc = torch.einsum("ihd,jhd->hij", tq, tk.repeat_interleave(G, dim=1)) * scale
        sc = sc.masked_fill(~mask[None], float("-inf"))
        o = torch.einsum("hij,jhd->ihd", torch.softmax(sc, dim=-1), tv.repeat_interleave(G, dim=1))
        (o * torch.tensor(do[c:c + L].astype(np.float64))).sum().backward()
        assert np.allclose(out[c:c + L], o.detach().numpy(), rtol=1e-12, atol=1e-13)
        assert np.allclose(lse[:, c:c + L], torch.logsumexp(sc, dim=-1).detach().numpy(), rtol=0, atol=1e-12)
        assert np.allclose(dq[c:c + L], tq.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dk[c:c + L], tk.grad.numpy(), rtol=1e-11, atol=1e-12)
        assert np.allclose(dv[c:c + L], tv.grad.numpy(), rtol=1e-11, atol=1e-12)
        for h in range(Hq):
            p, ds = oa.attn_probs(q, k, v, do, cu, W, s, h, scale=scale, mask_mode=oa.MASK_SLIDING_WINDOW)
            assert np.all((p > 0) == mask.numpy())
            assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14) and np.allclose(ds.sum(axis=1), 0.0, atol=1e-13)


def test_sliding_window_special_cases():
    Hq, Hkv, D = 2, 1, 8
    lens = [19, 8]
    cu, _, q, k, v, do = stream(22, lens, Hq, Hkv, D)
    # a window as long as the sample (or longer) is the causal mask, bit for bit
    want = oa.attn_fwd(q, k, v, cu, None, mask_mode=oa.MASK_CAUSAL) + oa.attn_bwd(q, k, v, do, cu, None, mask_mode=oa.MASK_CAUSAL)
    for W in (np.array(lens, dtype=np.int32), np.array([1000, 1000], dtype=np.int32)):
        got = oa.attn_fwd(q, k, v, cu, W, mask_mode=oa.MASK_SLIDING_WINDOW) + oa.attn_bwd(q, k, v, do, cu, W, mask_mode=oa.MASK_SLIDING_WINDOW)
        assert all(np.array_equal(a, b) for a, b in zip(got, want))
    # W = 1: every row sees itself only: O = V, LSE = scale q.k, dV = sum of dO over the group, dQ = dK = 0
    one = np.ones(2, dtype=np.int32)
    out, lse = oa.attn_fwd(q, k, v, cu, one, scale=0.5, mask_mode=oa.MASK_SLIDING_WINDOW)
    dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, one, scale=0.5, mask_mode=oa.MASK_SLIDING_WINDOW)
    assert np.array_equal(out, np.repeat(v.astype(np.float64), Hq // Hkv, axis=1))
    assert np.allclose(lse.T, 0.5 * np.einsum("thd,td->th", q.astype(np.float64), k[:, 0].astype(np.float64)), atol=1e-13)
    assert np.all(dq == 0) and np.all(dk == 0) and np.allclose(dv[:, 0], do.astype(np.float64).sum(axis=1), atol=1e-14)
    # uniform keys: LSE_i = scale q_i.k + ln(min(i + 1, W)), O_i = mean of the last min(i + 1, W) values
    k1 = np.repeat(k[:1], len(k), axis=0)
    W = np.array([6, 3], dtype=np.int32)
    out, lse = oa.attn_fwd(q, k1, v, cu, W, scale=0.5, mask_mode=oa.MASK_SLIDING_WINDOW)
    for s, Ls in enumerate(lens):
        for i in range(Ls):
            n = min(i + 1, int(W[s]))
            want_o = v[cu[s] + i + 1 - n:cu[s] + i + 1, 0].astype(np.float64).mean(axis=0)
            for h in range(Hq):
                want_lse = 0.5 * float(q[cu[s] + i, h].astype(np.float64) @ k1[0, 0].astype(np.float64)) + np.log(n)
                assert abs(lse[h, cu[s] + i] - want_lse) < 1e-12
                assert np.allclose(out[cu[s] + i, h], want_o, rtol=1e-13, atol=1e-14)


def test_row_by_row_functions_equal_the_oracle():
    # oracle/sampled.py evaluates chosen rows of one long sample; on a short one it must give what the
    # C oracle gives for whole samples
    from oracle import sampled
    Hq, Hkv, D, L = 4, 2, 8, 70
    cu, _, q, k, v, do = stream(31, [L], Hq, Hkv, D)
    scale = 0.3
    for window, mode, pl in ((None, oa.MASK_CAUSAL, None), (9, oa.MASK_SLIDING_WINDOW, np.array([9], dtype=np.int32))):
        out, lse = oa.attn_fwd(q, k, v, cu, pl, scale=scale, mask_mode=mode)
        dq, dk, dv = oa.attn_bwd(q, k, v, do, cu, pl, scale=scale, mask_mode=mode)
        for i in (0, 1, 8, 9, 33, 69):
            for h in range(Hq):
                o_i, lse_i = sampled.row_forward(q, k, v, scale, i, h, window)
                assert np.allclose(o_i, out[i, h], rtol=1e-12, atol=1e-14) and abs(lse_i - lse[h, i]) < 1e-12
                assert np.allclose(sampled.row_dq(q, k, v, do, scale, i, h, window), dq[i, h], rtol=1e-11, atol=1e-13)
        stats = sampled.row_stats(q, k, v, do, scale, window, rows_per_pass=16)     # several passes, a ragged last one
        assert np.allclose(stats[0], lse, rtol=1e-12, atol=1e-13)
        for j in (0, 5, 40, 69):
            for g in range(Hkv):
                dk_j, dv_j = sampled.key_row_dk_dv(q, k, v, do, scale, j, g, window)
                assert np.allclose(dk_j, dk[j, g], rtol=1e-11, atol=1e-13) and np.allclose(dv_j, dv[j, g], rtol=1e-11, atol=1e-13)
                dk_j, dv_j = sampled.key_row_dk_dv(q, k, v, do, scale, j, g, window, stats=stats)
                assert np.allclose(dk_j, dk[j, g], rtol=1e-11, atol=1e-13) and np.allclose(dv_j, dv[j, g], rtol=1e-11, atol=1e-13)
