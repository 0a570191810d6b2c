"""Pins for the fp64 CPU oracle (CPU only).

The oracle is Algorithm 1 of the paper (standard attention, S and P materialised).  Nothing here
compares the oracle with itself: every check is a closed form, an invariant of the definition
(Section 2), a hand-worked example, a scalar brute force written independently, or a library
routine (torch's fp64 scaled_dot_product_attention / logsumexp).
"""
import math
import os

import numpy as np
import pytest

import oracle


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _rand_qkv(seed, B, Nq, H, d, Nk=None):
    r = _rng(seed)
    Nk = Nq if Nk is None else Nk
    return (r.standard_normal((B, Nq, H, d)), r.standard_normal((B, Nk, H, d)), r.standard_normal((B, Nk, H, d)))


# ---------------------------------------------------------------- hand-worked examples (golden file)
def _parse_examples(path):
    env = {"ln": math.log, "__builtins__": {}}
    ev = lambda tok: float(eval(tok, env))  # noqa: E731  (fixture is ours; tokens like 2*ln(3), 3/11)
    examples, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "example":
            cur = {"name": rest[0], "k": [], "v": []}
            examples.append(cur)
        elif key in ("k", "v"):
            cur[key].append([ev(t) for t in rest])
        elif key in ("q", "P", "O"):
            cur[key] = [ev(t) for t in rest]
        elif key in ("scale", "expLSE"):
            cur[key] = ev(rest[0])
    return examples


def test_hand_worked_examples(golden_dir):
    examples = _parse_examples(os.path.join(golden_dir, "hand_examples.txt"))
    assert len(examples) == 2
    for ex in examples:
        q = np.array(ex["q"]).reshape(1, 1, 1, -1)
        k = np.array(ex["k"]).reshape(1, -1, 1, q.shape[-1])
        v = np.array(ex["v"]).reshape(1, k.shape[1], 1, -1)
        assert v.shape[-1] == q.shape[-1]
        o, lse = oracle.attention(q, k, v, ex["scale"])
        np.testing.assert_allclose(o.ravel(), ex["O"], rtol=1e-14)
        np.testing.assert_allclose(math.exp(lse.ravel()[0]), ex["expLSE"], rtol=1e-14)
        _, p = oracle.head_probs(q, k, v, ex["scale"], 0, 0)
        np.testing.assert_allclose(p.ravel(), ex["P"], rtol=1e-14)


# ---------------------------------------------------------------- scalar brute force, own indexing
def _brute_force(qf, kf, vf, B, H, Nq, Nk, d, scale):
    """Attention written with Python scalars over *flat* lists; indexing typed out again here
    as ((b*N+n)*H+h)*d+k  (Section 2: shape (batch, seqlen, heads, headdim))."""
    O = [0.0] * (B * Nq * H * d)
    LSE = [0.0] * (B * H * Nq)
    for b in range(B):
        for h in range(H):
            for i in range(Nq):
                s = []
                for j in range(Nk):
                    s.append(scale * math.fsum(qf[((b * Nq + i) * H + h) * d + c] * kf[((b * Nk + j) * H + h) * d + c]
                                               for c in range(d)))
                den = math.fsum(math.exp(x) for x in s)       # no max-shift: tiny inputs cannot overflow
                for c in range(d):
                    O[((b * Nq + i) * H + h) * d + c] = math.fsum(
                        math.exp(s[j]) / den * vf[((b * Nk + j) * H + h) * d + c] for j in range(Nk))
                LSE[(b * H + h) * Nq + i] = math.log(den)
    return O, LSE


@pytest.mark.parametrize("B,H,Nq,Nk,d,scale", [(2, 2, 3, 5, 3, 0.7), (1, 3, 8, 8, 4, 0.5), (2, 2, 1, 7, 2, 1.3)])
def test_brute_force_tiny(B, H, Nq, Nk, d, scale):
    q, k, v = _rand_qkv(11 + Nq, B, Nq, H, d, Nk)
    O, LSE = _brute_force(q.ravel().tolist(), k.ravel().tolist(), v.ravel().tolist(), B, H, Nq, Nk, d, scale)
    o, lse = oracle.attention(q, k, v, scale, row_block=2)
    np.testing.assert_allclose(o.ravel(), O, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse.ravel(), LSE, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- invariants of the definition
def test_rows_of_P_sum_to_one_and_are_positive():
    q, k, v = _rand_qkv(3, 2, 40, 3, 16)
    for b in range(2):
        for h in range(3):
            s, p = oracle.head_probs(q, k, v, 0.25, b, h)
            assert np.all(p > 0)
            np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=0, atol=1e-14)
            # S is the scaled logit matrix of this head
            np.testing.assert_allclose(s, 0.25 * q[b, :, h, :] @ k[b, :, h, :].T, rtol=1e-13, atol=1e-13)


def test_constant_V_gives_constant_O():
    q, k, v = _rand_qkv(4, 1, 33, 2, 8)
    v[...] = 0.0
    v += np.array([1.5, -2.0, 0.25, 3.0, 0.0, -7.0, 9.0, 1.0])      # every key has the same value row
    o, _ = oracle.attention(q, k, v, 0.35)
    np.testing.assert_allclose(o, np.broadcast_to(v[:, :1], o.shape), rtol=1e-14, atol=1e-14)


def test_shift_invariance_through_a_constant_column():
    # Q[..., c0] = 1 and K[..., c0] = t add scale*t to every logit of a row: P (hence O) is unchanged
    # (Section 2: translating a row by a common value does not change its softmax); LSE moves by scale*t.
    q, k, v = _rand_qkv(5, 2, 24, 2, 6)
    scale, t = 0.4, 3.75
    q[..., 2] = 1.0
    k0 = k.copy(); k0[..., 2] = 0.0
    k1 = k.copy(); k1[..., 2] = t
    o0, l0 = oracle.attention(q, k0, v, scale)
    o1, l1 = oracle.attention(q, k1, v, scale)
    np.testing.assert_allclose(o1, o0, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(l1 - l0, scale * t, rtol=1e-12)


def test_single_key_and_identical_keys():
    q, k, v = _rand_qkv(6, 2, 9, 2, 5, Nk=1)
    scale = 0.6
    o, lse = oracle.attention(q, k, v, scale)
    np.testing.assert_allclose(o, np.broadcast_to(v, o.shape), rtol=1e-15)
    s0 = scale * np.einsum("bihc,bhc->bhi", q, k[:, 0])
    np.testing.assert_allclose(lse, s0, rtol=1e-13, atol=1e-14)
    # the same key and value repeated Nk times: O = V_0, LSE = s_0 + ln Nk
    Nk = 17
    kk, vv = np.repeat(k, Nk, axis=1), np.repeat(v, Nk, axis=1)
    o2, lse2 = oracle.attention(q, kk, vv, scale)
    np.testing.assert_allclose(o2, np.broadcast_to(v, o.shape), rtol=1e-13)
    np.testing.assert_allclose(lse2, s0 + math.log(Nk), rtol=1e-13, atol=1e-13)


def test_zero_Q_gives_uniform_P():
    q, k, v = _rand_qkv(7, 1, 4, 2, 8, Nk=50)
    q[...] = 0.0
    o, lse = oracle.attention(q, k, v, 0.3)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=1, keepdims=True), o.shape), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse, math.log(50), rtol=1e-14)      # natural logarithm
    _, p = oracle.head_probs(q, k, v, 0.3, 0, 1)
    np.testing.assert_allclose(p, 1.0 / 50, rtol=1e-14)


def test_two_keys_closed_form_sigmoid():
    # d = 1, two keys: P = (sigma(s1-s2), 1-sigma(s1-s2)), LSE = logaddexp(s1, s2)
    r = _rng(8)
    for _ in range(20):
        qv, k1, k2, v1, v2, scale = r.standard_normal(5).tolist() + [float(r.uniform(0.1, 2.0))]
        q = np.array(qv).reshape(1, 1, 1, 1)
        k = np.array([k1, k2]).reshape(1, 2, 1, 1)
        v = np.array([v1, v2]).reshape(1, 2, 1, 1)
        o, lse = oracle.attention(q, k, v, scale)
        s1, s2 = scale * qv * k1, scale * qv * k2
        sig = 1.0 / (1.0 + math.exp(-(s1 - s2)))
        assert o.item() == pytest.approx(sig * v1 + (1 - sig) * v2, rel=1e-13, abs=1e-15)
        assert lse.item() == pytest.approx(np.logaddexp(s1, s2), rel=1e-13, abs=1e-15)


def test_key_permutation_invariance():
    q, k, v = _rand_qkv(9, 2, 20, 2, 8, Nk=37)
    perm = _rng(90).permutation(37)
    o0, l0 = oracle.attention(q, k, v, 0.5)
    o1, l1 = oracle.attention(q, k[:, perm], v[:, perm], 0.5)
    np.testing.assert_allclose(o1, o0, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l1, l0, rtol=1e-13, atol=1e-14)


def test_query_rows_are_independent_and_in_order():
    # reversing the queries reverses the outputs: catches a row index slip in O / LSE placement
    q, k, v = _rand_qkv(10, 2, 19, 3, 4)
    o0, l0 = oracle.attention(q, k, v, 0.5, row_block=4)
    o1, l1 = oracle.attention(q[:, ::-1], k, v, 0.5, row_block=7)
    np.testing.assert_allclose(o1[:, ::-1], o0, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(l1[:, :, ::-1], l0, rtol=1e-13, atol=1e-15)


def test_split_key_merge_through_LSE():
    # attention over keys [0, Nk/2) and [Nk/2, Nk) recombined through the log-sum-exp equals the full
    # result: the identity behind Algorithm 2's rescaling, and the pin of LSE's scale convention.
    q, k, v = _rand_qkv(12, 2, 16, 2, 8, Nk=30)
    scale = 0.45
    o, lse = oracle.attention(q, k, v, scale)
    oa, la = oracle.attention(q, k[:, :11], v[:, :11], scale)
    ob, lb = oracle.attention(q, k[:, 11:], v[:, 11:], scale)
    lm = np.logaddexp(la, lb)
    wa = np.exp(la - lm).transpose(0, 2, 1)[..., None]     # [B,H,N] -> [B,N,H,1]
    wb = np.exp(lb - lm).transpose(0, 2, 1)[..., None]
    np.testing.assert_allclose(lm, lse, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(wa * oa + wb * ob, o, rtol=1e-12, atol=1e-14)


def test_one_dominant_logit_is_stable():
    # one key aligned with q and 50x longer: exp() of the raw logit would overflow fp64 without the
    # rowmax shift (Section 2); the output must collapse onto that key's value row.
    q, k, v = _rand_qkv(13, 1, 6, 1, 16, Nk=40)
    jstar = 23
    for i in range(1):
        k[0, jstar, 0, :] = 50.0 * q[0, 0, 0, :]
    scale = 4.0            # logit ~ 4*50*|q|^2 ~ 3200 > ln(DBL_MAX) ~ 709
    o, lse = oracle.attention(q[:, :1], k, v, scale)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    np.testing.assert_allclose(o[0, 0, 0], v[0, jstar, 0], rtol=1e-12, atol=1e-12)
    assert lse.item() == pytest.approx(scale * 50.0 * float(q[0, 0, 0] @ q[0, 0, 0]), rel=1e-13)


# ---------------------------------------------------------------- library cross-checks
def test_against_torch_sdpa_fp64_on_workload_1():
    import torch
    from paper_2312_11918_amd import workloads

    w, qb, kb, vb = workloads.make_workload(1)
    q, k, v = (oracle.widen(x, w.dtype) for x in (qb, kb, vb))
    o, lse = oracle.attention(q, k, v, w.scale)
    tq, tk, tv = (torch.from_numpy(x).permute(0, 2, 1, 3) for x in (q, k, v))          # [B,H,N,d]
    to = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=w.scale).permute(0, 2, 1, 3)
    np.testing.assert_allclose(o, to.numpy(), rtol=1e-11, atol=1e-13)
    tl = torch.logsumexp(w.scale * tq @ tk.transpose(-1, -2), dim=-1)                   # [B,H,N]
    np.testing.assert_allclose(lse, tl.numpy(), rtol=1e-12, atol=1e-13)


def test_against_numpy_dense_formula_multihead():
    # softmax(scale*QK^T)V by einsum/scipy on a ragged, multi-head, Nq != Nk case
    from scipy.special import logsumexp, softmax
    q, k, v = _rand_qkv(14, 3, 13, 4, 7, Nk=29)
    scale = 0.37
    s = scale * np.einsum("bihc,bjhc->bhij", q, k)
    o_ref = np.einsum("bhij,bjhc->bihc", softmax(s, axis=-1), v)
    o, lse = oracle.attention(q, k, v, scale, row_block=5)
    np.testing.assert_allclose(o, o_ref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, logsumexp(s, axis=-1), rtol=1e-13, atol=1e-14)


def test_sampled_rows_match_closed_forms():
    # attention_rows on an all-identical-keys problem: every sampled row has the closed form
    q, k, v = _rand_qkv(15, 2, 64, 3, 8, Nk=1)
    kk, vv = np.repeat(k, 21, axis=1), np.repeat(v, 21, axis=1)
    rows = np.array([[0, 0, 0], [1, 2, 63], [0, 1, 17], [1, 0, 5]], dtype=np.int32)
    o, lse = oracle.attention_rows(q, kk, vv, 0.5, rows)
    for t, (b, h, i) in enumerate(rows):
        np.testing.assert_allclose(o[t], v[b, 0, h], rtol=1e-13)
        assert lse[t] == pytest.approx(0.5 * float(q[b, i, h] @ k[b, 0, h]) + math.log(21), rel=1e-13, abs=1e-14)


def test_sampled_rows_against_dense_formula():
    from scipy.special import logsumexp, softmax
    q, k, v = _rand_qkv(16, 2, 12, 2, 5, Nk=9)
    rows = np.array([[b, h, i] for b in range(2) for h in range(2) for i in (0, 5, 11)], dtype=np.int32)
    o, lse = oracle.attention_rows(q, k, v, 0.8, rows)
    s = 0.8 * np.einsum("bihc,bjhc->bhij", q, k)
    o_ref = np.einsum("bhij,bjhc->bihc", softmax(s, axis=-1), v)
    for t, (b, h, i) in enumerate(rows):
        np.testing.assert_allclose(o[t], o_ref[b, i, h], rtol=1e-12, atol=1e-14)
        assert lse[t] == pytest.approx(logsumexp(s[b, h, i]), rel=1e-13)


# ---------------------------------------------------------------- Algorithm 2's recurrence (fp64, any tile)
def _alg2_fp64(q, k, v, scale, bM, bN):
    """Algorithm 2 (FlashAttention-2 forward) written tile by tile in fp64 numpy: running rowmax
    (new, old), running rowsum, rescaled accumulator, final division by the rowsum."""
    B, Nq, H, d = q.shape
    Nk = k.shape[1]
    O = np.zeros_like(q)
    LSE = np.zeros((B, H, Nq))
    for b in range(B):
        for h in range(H):
            for i0 in range(0, Nq, bM):
                Qi = q[b, i0:i0 + bM, h]
                Oi = np.zeros_like(Qi)
                m = np.full(Qi.shape[0], -np.inf)
                l = np.zeros(Qi.shape[0])
                for j0 in range(0, Nk, bN):
                    S = scale * Qi @ k[b, j0:j0 + bN, h].T
                    m_new = np.maximum(m, S.max(axis=1))
                    P = np.exp(S - m_new[:, None])
                    alpha = np.exp(m - m_new)
                    l = alpha * l + P.sum(axis=1)
                    Oi = alpha[:, None] * Oi + P @ v[b, j0:j0 + bN, h]
                    m = m_new
                O[b, i0:i0 + bM, h] = Oi / l[:, None]
                LSE[b, h, i0:i0 + bM] = m + np.log(l)
    return O, LSE


@pytest.mark.parametrize("bM,bN", [(4, 4), (8, 16), (5, 3), (64, 64)])
def test_algorithm2_recurrence_reaches_the_oracle(bM, bN):
    q, k, v = _rand_qkv(17, 2, 24, 2, 8, Nk=40)
    k[0, 31, 0] *= 12.0          # a late large logit forces a big rescale
    o, lse = oracle.attention(q, k, v, 0.5)
    o2, lse2 = _alg2_fp64(q, k, v, 0.5, bM, bN)
    np.testing.assert_allclose(o2, o, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse2, lse, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- argument handling
def test_oracle_rejects_bad_shapes():
    q, k, v = _rand_qkv(18, 1, 4, 2, 3)
    with pytest.raises(ValueError):
        oracle.attention(q, k[:, :, :1], v, 1.0)
    with pytest.raises(RuntimeError):
        oracle.attention_rows(q, k, v, 1.0, np.array([[0, 2, 0]]))     # head out of range
    with pytest.raises(RuntimeError):
        oracle.attention(q, k, v, float("nan"))


def test_widen_bit_patterns():
    assert oracle.widen(np.array([0x3C00, 0xC000, 0x0001], dtype=np.uint16), "fp16").tolist() == [1.0, -2.0, 2.0 ** -24]
    assert oracle.widen(np.array([0x3F80, 0xC040, 0x0080], dtype=np.uint16), "bf16").tolist() == [1.0, -3.0, 2.0 ** -126]


# ---------------------------------------------------------------- causal mask (optional masking of S, Section 2 footnote)
def test_causal_rows_equal_unmasked_attention_over_the_prefix():
    # row i of the causal result is plain attention of q_i over keys 0..i: the unmasked path, pinned above
    q, k, v = _rand_qkv(21, 2, 23, 2, 6)
    oc, lc = oracle.attention(q, k, v, 0.6, row_block=5, causal=True)
    for i in (0, 1, 7, 22):
        o, l = oracle.attention(q[:, i:i + 1], k[:, :i + 1], v[:, :i + 1], 0.6)
        np.testing.assert_allclose(oc[:, i:i + 1], o, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(lc[:, :, i:i + 1], l, rtol=1e-13, atol=1e-15)
    # first row sees only key 0
    np.testing.assert_allclose(oc[:, 0], v[:, 0], rtol=1e-15)
    np.testing.assert_allclose(lc[:, :, 0], 0.6 * np.einsum("bhc,bhc->bh", q[:, 0], k[:, 0]), rtol=1e-13, atol=1e-15)
    # last row sees everything: equals the unmasked result
    of, lf = oracle.attention(q, k, v, 0.6)
    np.testing.assert_allclose(oc[:, -1], of[:, -1], rtol=1e-13)


def test_causal_against_torch_sdpa_fp64_and_brute_force():
    import torch
    q, k, v = _rand_qkv(22, 2, 17, 3, 5)
    o, lse = oracle.attention(q, k, v, 0.45, causal=True)
    tq, tk, tv = (torch.from_numpy(x).permute(0, 2, 1, 3) for x in (q, k, v))
    to = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.45, is_causal=True).permute(0, 2, 1, 3)
    np.testing.assert_allclose(o, to.numpy(), rtol=1e-12, atol=1e-14)
    # scalar brute force of one head, own loops: sum over j <= i only
    b, h = 1, 2
    for i in range(17):
        s = [0.45 * math.fsum(q[b, i, h, c] * k[b, j, h, c] for c in range(5)) for j in range(i + 1)]
        den = math.fsum(math.exp(x) for x in s)
        for c in range(5):
            assert o[b, i, h, c] == pytest.approx(math.fsum(math.exp(s[j]) / den * v[b, j, h, c] for j in range(i + 1)), rel=1e-12, abs=1e-14)
        assert lse[b, h, i] == pytest.approx(math.log(den), rel=1e-12, abs=1e-14)


def test_causal_sampled_rows_and_shape_check():
    q, k, v = _rand_qkv(23, 1, 12, 2, 4)
    o, lse = oracle.attention(q, k, v, 0.5, causal=True)
    rows = np.array([[0, 0, 0], [0, 1, 11], [0, 1, 5]], dtype=np.int32)
    orow, lrow = oracle.attention_rows(q, k, v, 0.5, rows, causal=True)
    for t, (b, h, i) in enumerate(rows):
        np.testing.assert_allclose(orow[t], o[b, i, h], rtol=1e-14)
        assert lrow[t] == pytest.approx(lse[b, h, i], rel=1e-14)
    with pytest.raises(RuntimeError):
        oracle.attention(q, k[:, :5], v[:, :5], 0.5, causal=True)      # causal needs as many keys as queries
