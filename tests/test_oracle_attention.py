"""Pins for the oracle's floating part.  CPU only.

Each test checks the C oracle against something other than itself: a dense
masked softmax written with library routines (numpy / torch in float64),
torch autograd, central finite differences, closed forms and invariants."""
import numpy as np
import pytest
import torch

from paper_2505_19609_amd import workloads as W


def _rand(shape, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return W.bf16_bits_to_f32(W.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)))


def _dense_reference(q, k, v, q_begin, scale, do=None):
    """Textbook single-sequence attention with library ops (torch float64).
    q: [Lq, Hq, d]; k, v: [Lk, Hkv, d]; query i sits at position q_begin + i."""
    q = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    k = torch.tensor(k, dtype=torch.float64, requires_grad=True)
    v = torch.tensor(v, dtype=torch.float64, requires_grad=True)
    Lq, Hq, d = q.shape
    Lk, Hkv, _ = k.shape
    g = Hq // Hkv
    kk = k.repeat_interleave(g, dim=1)
    vv = v.repeat_interleave(g, dim=1)
    s = torch.einsum("ihd,jhd->hij", q, kk) * scale
    pos = torch.arange(Lq)[:, None] + q_begin
    mask = torch.arange(Lk)[None, :] <= pos
    s = s.masked_fill(~mask[None], float("-inf"))
    lse = torch.logsumexp(s, dim=-1)
    o = torch.einsum("hij,jhd->ihd", torch.softmax(s, dim=-1), vv)
    out = {"o": o.detach().numpy(), "lse": lse.detach().numpy()}
    if do is not None:
        o.backward(torch.tensor(do, dtype=torch.float64))
        out.update(dq=q.grad.numpy(), dk=k.grad.numpy(), dv=v.grad.numpy())
    return out


def _problem(S, N, r, Hq, Hkv, d, seed, oracle):
    desc = oracle.ranges(S, N, r)
    q = _rand((desc["total_q"], Hq, d), seed)
    k = _rand((desc["total_k"], Hkv, d), seed + 1)
    v = _rand((desc["total_k"], Hkv, d), seed + 2)
    do = _rand((desc["total_q"], Hq, d), seed + 3)
    return desc, q, k, v, do


def test_brute_force_no_max_subtraction(oracle):
    """Triple loop, exp without max subtraction, on a tiny case."""
    S, Hq, Hkv, d, scale = [7, 3], 2, 1, 4, 0.37
    desc, q, k, v, _ = _problem(S, [1, 1], [0, 0], Hq, Hkv, d, 5, oracle)
    O, LSE = oracle.attention_fwd(q, k, v, desc, scale)
    for kk in range(2):
        for h in range(Hq):
            for i in range(S[kk]):
                qi = q[desc["cu_q"][kk] + i, h].astype(np.float64)
                w = [np.exp(scale * sum(qi[t] * float(k[desc["cu_k"][kk] + j, 0, t]) for t in range(d)))
                     for j in range(i + 1)]
                z = sum(w)
                o = sum(w[j] / z * v[desc["cu_k"][kk] + j, 0].astype(np.float64) for j in range(i + 1))
                assert np.allclose(O[desc["cu_q"][kk] + i, h], o, rtol=1e-12, atol=1e-13)
                assert abs(LSE[h, desc["cu_q"][kk] + i] - np.log(z)) < 1e-12


@pytest.mark.parametrize("Hq,Hkv,d", [(4, 4, 8), (6, 2, 16), (4, 1, 64)])
def test_forward_and_backward_match_dense_library(oracle, Hq, Hkv, d):
    """Packed batch with a shard == dense masked softmax + autograd per sequence."""
    S, N, r = [33, 1, 50, 18], [1, 1, 5, 2], [0, 0, 3, 1]
    scale = 1.0 / np.sqrt(d)
    desc, q, k, v, do = _problem(S, N, r, Hq, Hkv, d, 11, oracle)
    O, LSE = oracle.attention_fwd(q, k, v, desc, scale)
    dQ, dK, dV, D = oracle.attention_bwd(q, k, v, do, desc, scale)
    for s in range(len(S)):
        qs, qe = desc["cu_q"][s], desc["cu_q"][s + 1]
        ks, ke = desc["cu_k"][s], desc["cu_k"][s + 1]
        ref = _dense_reference(q[qs:qe], k[ks:ke], v[ks:ke], int(desc["q_begin"][s]), scale, do[qs:qe])
        assert np.allclose(O[qs:qe], ref["o"], rtol=1e-11, atol=1e-12)
        assert np.allclose(LSE[:, qs:qe], ref["lse"], rtol=1e-11, atol=1e-12)
        assert np.allclose(dQ[qs:qe], ref["dq"], rtol=1e-10, atol=1e-11)
        assert np.allclose(dK[ks:ke], ref["dk"], rtol=1e-10, atol=1e-11)
        assert np.allclose(dV[ks:ke], ref["dv"], rtol=1e-10, atol=1e-11)
        assert np.allclose(D[:, qs:qe], np.einsum("ihd,ihd->hi", do[qs:qe].astype(np.float64), ref["o"]),
                           rtol=1e-10, atol=1e-11)


def test_backward_central_finite_differences(oracle):
    """L = sum(O * dO); directional derivative along a random direction E for
    each of Q, K, V must equal <grad, E>."""
    S, N, r = [12, 9], [1, 3], [0, 2]
    Hq, Hkv, d, scale = 4, 2, 8, 0.31
    desc, q, k, v, do = _problem(S, N, r, Hq, Hkv, d, 23, oracle)
    dQ, dK, dV, _ = oracle.attention_bwd(q, k, v, do, desc, scale)
    rng = np.random.Generator(np.random.PCG64(99))

    def loss(q_, k_, v_):
        O, _ = oracle.attention_fwd(q_, k_, v_, desc, scale)
        return float((O * do.astype(np.float64)).sum())

    # the oracle takes float32 inputs, so perturb with steps exactly representable there
    eps = 2.0 ** -10
    for name, grad in (("q", dQ), ("k", dK), ("v", dV)):
        E = np.sign(rng.standard_normal(grad.shape)).astype(np.float32)
        args_p = {"q": q, "k": k, "v": v}
        args_m = dict(args_p)
        args_p = dict(args_p)
        args_p[name] = (args_p[name] + eps * E).astype(np.float32)
        args_m[name] = (args_m[name] - eps * E).astype(np.float32)
        assert np.array_equal(args_p[name].astype(np.float64),
                              {"q": q, "k": k, "v": v}[name].astype(np.float64) + eps * E)
        fd = (loss(args_p["q"], args_p["k"], args_p["v"]) - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * eps)
        an = float((grad * E).sum())
        # central difference error is O(eps^2 * third derivative)
        assert abs(fd - an) <= 2e-4 * max(1.0, abs(an)), (name, fd, an)


def test_first_row_and_softmax_rows_sum_to_one(oracle):
    S = [20, 5]
    Hq, Hkv, d, scale = 2, 2, 8, 0.5
    desc, q, k, v, _ = _problem(S, [1, 1], [0, 0], Hq, Hkv, d, 31, oracle)
    O, LSE = oracle.attention_fwd(q, k, v, desc, scale)
    for s in range(2):
        r0, c0 = desc["cu_q"][s], desc["cu_k"][s]
        # row 0 sees only key 0: O_0 = V_0 and LSE_0 = s_00 exactly
        assert np.array_equal(O[r0], v[c0].astype(np.float64))
        s00 = scale * (q[r0].astype(np.float64) * k[c0].astype(np.float64)).sum(-1)
        assert np.allclose(LSE[:, r0], s00, rtol=0, atol=1e-14)
    # V = all ones -> O = sum_j P_ij = 1
    O1, _ = oracle.attention_fwd(q, k, np.ones_like(v), desc, scale)
    assert np.allclose(O1, 1.0, rtol=0, atol=1e-13)
    # identical keys -> uniform weights -> O_i = mean of the V prefix, LSE = s + log(i+1)
    k_same = np.broadcast_to(k[:1], k.shape).copy()
    O2, L2 = oracle.attention_fwd(q, k_same, v, desc, scale)
    for s in range(2):
        for i in range(S[s]):
            pref = v[desc["cu_k"][s]: desc["cu_k"][s] + i + 1].astype(np.float64).mean(0)
            assert np.allclose(O2[desc["cu_q"][s] + i], pref, rtol=1e-12, atol=1e-13)


def test_packed_equals_each_sequence_alone(oracle):
    S, N, r = [19, 40, 7], [1, 4, 1], [0, 1, 0]
    Hq, Hkv, d, scale = 4, 2, 16, 0.25
    desc, q, k, v, do = _problem(S, N, r, Hq, Hkv, d, 41, oracle)
    O, LSE = oracle.attention_fwd(q, k, v, desc, scale)
    dQ, dK, dV, _ = oracle.attention_bwd(q, k, v, do, desc, scale)
    for s in range(3):
        qs, qe = desc["cu_q"][s], desc["cu_q"][s + 1]
        ks, ke = desc["cu_k"][s], desc["cu_k"][s + 1]
        one = oracle.ranges([S[s]], [N[s]], [r[s]])
        O1, L1 = oracle.attention_fwd(q[qs:qe], k[ks:ke], v[ks:ke], one, scale)
        g1 = oracle.attention_bwd(q[qs:qe], k[ks:ke], v[ks:ke], do[qs:qe], one, scale)
        assert np.array_equal(O[qs:qe], O1) and np.array_equal(LSE[:, qs:qe], L1)
        assert np.array_equal(dQ[qs:qe], g1[0])
        assert np.array_equal(dK[ks:ke], g1[1]) and np.array_equal(dV[ks:ke], g1[2])


def test_shards_reassemble_the_unsharded_sequence(oracle):
    """Rows of a shard equal the matching rows of the whole sequence; zero-padded
    partial dK/dV summed over all shards equal the whole sequence's dK/dV."""
    S, N = 45, 4
    Hq, Hkv, d, scale = 4, 2, 8, 0.3
    full = oracle.ranges([S])
    q = _rand((S, Hq, d), 51)
    k = _rand((S, Hkv, d), 52)
    v = _rand((S, Hkv, d), 53)
    do = _rand((S, Hq, d), 54)
    O, LSE = oracle.attention_fwd(q, k, v, full, scale)
    dQ, dK, dV, _ = oracle.attention_bwd(q, k, v, do, full, scale)
    dKs, dVs = np.zeros_like(dK), np.zeros_like(dV)
    for r in range(N):
        sh = oracle.ranges([S], [N], [r])
        b, e = int(sh["q_begin"][0]), int(sh["kv_len"][0])
        Or, Lr = oracle.attention_fwd(q[b:e], k[:e], v[:e], sh, scale)
        gq, gk, gv, _ = oracle.attention_bwd(q[b:e], k[:e], v[:e], do[b:e], sh, scale)
        assert np.allclose(Or, O[b:e], rtol=0, atol=1e-14)
        assert np.allclose(Lr, LSE[:, b:e], rtol=0, atol=1e-14)
        assert np.allclose(gq, dQ[b:e], rtol=0, atol=1e-13)
        dKs[:e] += gk
        dVs[:e] += gv
    assert np.allclose(dKs, dK, rtol=0, atol=1e-12)
    assert np.allclose(dVs, dV, rtol=0, atol=1e-12)


def test_gradient_identities(oracle):
    """Scale invariance of q.k under Q -> aQ, K -> K/a gives
    sum_i dQ_i.Q_i = sum_j dK_j.K_j for every (sequence, KV group)."""
    S, N, r = [30, 21], [1, 3], [0, 2]
    Hq, Hkv, d, scale = 6, 2, 8, 0.35
    desc, q, k, v, do = _problem(S, N, r, Hq, Hkv, d, 61, oracle)
    dQ, dK, dV, _ = oracle.attention_bwd(q, k, v, do, desc, scale)
    g = Hq // Hkv
    for s in range(2):
        qs, qe = desc["cu_q"][s], desc["cu_q"][s + 1]
        ks, ke = desc["cu_k"][s], desc["cu_k"][s + 1]
        for c in range(Hkv):
            lhs = (dQ[qs:qe, c * g:(c + 1) * g] * q[qs:qe, c * g:(c + 1) * g]).sum()
            rhs = (dK[ks:ke, c] * k[ks:ke, c]).sum()
            assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))


def test_gqa_equals_mha_with_duplicated_kv_heads(oracle):
    S = [25, 14]
    Hq, Hkv, d, scale = 6, 2, 8, 0.3
    g = Hq // Hkv
    desc, q, k, v, do = _problem(S, [1, 1], [0, 0], Hq, Hkv, d, 71, oracle)
    kd, vd = np.repeat(k, g, axis=1), np.repeat(v, g, axis=1)
    O, LSE = oracle.attention_fwd(q, k, v, desc, scale)
    Od, Ld = oracle.attention_fwd(q, kd, vd, desc, scale)
    assert np.array_equal(O, Od) and np.array_equal(LSE, Ld)
    dQ, dK, dV, _ = oracle.attention_bwd(q, k, v, do, desc, scale)
    dQd, dKd, dVd, _ = oracle.attention_bwd(q, kd, vd, do, desc, scale)
    assert np.array_equal(dQ, dQd)
    assert np.allclose(dK, dKd.reshape(-1, Hkv, g, d).sum(2), rtol=0, atol=1e-12)
    assert np.allclose(dV, dVd.reshape(-1, Hkv, g, d).sum(2), rtol=0, atol=1e-12)


def test_sampled_entries_match_the_full_run(oracle):
    """The row / column sampling used at full size returns the same numbers as the full run."""
    S, N, r = [64, 31], [2, 1], [1, 0]
    Hq, Hkv, d, scale = 4, 2, 8, 0.3
    desc, q, k, v, do = _problem(S, N, r, Hq, Hkv, d, 81, oracle)
    O, LSE = oracle.attention_fwd(q, k, v, desc, scale)
    dQ, dK, dV, D = oracle.attention_bwd(q, k, v, do, desc, scale)
    ent = (np.array([0, 1, 0], np.int32), np.array([3, 0, 1], np.int32), np.array([31, 30, 0], np.int32))
    o, l = oracle.fwd_rows(q, k, v, desc, scale, ent)
    dq, dd = oracle.bwd_dq_rows(q, k, v, do, desc, scale, ent)
    for t in range(3):
        row = desc["cu_q"][ent[0][t]] + ent[2][t]
        assert np.array_equal(o[t], O[row, ent[1][t]]) and l[t] == LSE[ent[1][t], row]
        assert np.array_equal(dq[t], dQ[row, ent[1][t]]) and dd[t] == D[ent[1][t], row]
    cent = (np.array([0, 0, 1], np.int32), np.array([1, 0, 1], np.int32), np.array([0, 63, 30], np.int32))
    dk, dv = oracle.bwd_dkv_cols(q, k, v, do, LSE, D, desc, scale, cent)
    for t in range(3):
        row = desc["cu_k"][cent[0][t]] + cent[2][t]
        assert np.array_equal(dk[t], dK[row, cent[1][t]]) and np.array_equal(dv[t], dV[row, cent[1][t]])


def test_delta_rows_is_the_row_term_of_the_softmax_gradient(oracle):
    """delta_rows (D_i = dO_i . O_i from the forward's O) against (a) a value worked by hand,
    (b) the D that the C backward forms from its own recomputed O (itself pinned by autograd
    and finite differences above), (c) the identity D_i = sum_j P_ij dP_ij: dS rows sum to 0."""
    assert oracle.delta_rows(np.array([[1.0, -2.0, 0.5]]), np.array([[3.0, 0.25, -4.0]]))[0] == 0.5
    S, N, r = [40, 23], [2, 1], [1, 0]
    Hq, Hkv, d, scale = 4, 2, 8, 0.3
    desc, q, k, v, do = _problem(S, N, r, Hq, Hkv, d, 91, oracle)
    ent = oracle.all_row_entries(desc, Hq)
    rows = desc["cu_q"][ent[0]] + ent[2]
    o, lse = oracle.fwd_rows(q, k, v, desc, scale, ent)
    D = oracle.delta_rows(do[rows, ent[1]], o)
    _, d_c = oracle.bwd_dq_rows(q, k, v, do, desc, scale, ent)
    assert np.allclose(D, d_c, rtol=0, atol=1e-13)
    g = Hq // Hkv
    for t in range(0, len(rows), 7):
        s, h, i = int(ent[0][t]), int(ent[1][t]), int(ent[2][t])
        p = int(desc["q_begin"][s]) + i
        kk = k[desc["cu_k"][s]:desc["cu_k"][s] + p + 1, h // g].astype(np.float64)
        vv = v[desc["cu_k"][s]:desc["cu_k"][s] + p + 1, h // g].astype(np.float64)
        P = np.exp(scale * kk @ q[rows[t], h].astype(np.float64) - lse[t])
        assert abs(P @ (vv @ do[rows[t], h].astype(np.float64)) - D[t]) < 1e-12
