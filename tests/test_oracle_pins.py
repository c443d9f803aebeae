"""Pins for the CPU oracle: each test checks it against something the paper or
the mathematics fixes, computed here by an independent textbook routine (numpy
fp64), never by the oracle itself.  CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
from workloads import bf16_bits, make_problem

TOL = 1e-10


def f64(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.float64).numpy()


def textbook_attention(q, K, V, scale):
    """softmax(scale * q K^T) V for ONE query vector: q [d], K [n, d], V [n, dv]."""
    s = scale * (K @ q)
    s = s - s.max()
    p = np.exp(s)
    p = p / p.sum()
    return p @ V, p


def gather_logical(p, b):
    """Logical (unpaged) cache of sequence b: state [h_c, L, d_v], rope [L, d_r]."""
    L = int(p.seq_lens[b])
    n = (L + p.page_size - 1) // p.page_size
    idx = p.table_compact[b, :n]
    st = f64(p.state_pages)[idx]                      # [n, h_c, P, d_v]
    st = st.transpose(1, 0, 2, 3).reshape(p.h_c, n * p.page_size, p.d_v)[:, :L]
    rp = f64(p.rope_pages)[idx].reshape(n * p.page_size, p.d_r)[:L]
    return st, rp


# ---------------------------------------------------------------- P1
def test_absorbed_equals_explicit_upprojection():
    """Section 2.1 / 3.3.2: absorbing W_UK into the query and W_UV into the output
    gives the same result as attention over explicitly up-projected per-head
    keys and values.  Integer-valued W_UK and raw queries keep the absorbed
    query exactly representable in bf16, so the identity is exact."""
    rng = np.random.default_rng(1)
    h_q, h_c, d_c, d_h, d_r, L = 6, 2, 16, 8, 4, 37
    g_q = h_q // h_c
    p = make_problem("p1", seq_lens=[L], h_q=h_q, h_c=h_c, d_v=d_c, d_r=d_r, page_size=8,
                     seed=11, scale=0.3)
    W_UK = rng.integers(-1, 2, size=(h_q, d_c, d_h)).astype(np.float64)
    W_UV = rng.standard_normal((h_q, d_c, d_h))
    q_raw = rng.integers(-2, 3, size=(h_q, d_h)).astype(np.float64)
    q_abs = np.einsum("hcd,hd->hc", W_UK, q_raw)        # |.| <= 16: exact in bf16
    p.q_nope = torch.from_numpy(q_abs).to(torch.bfloat16).reshape(1, 1, h_q, d_c)
    assert np.array_equal(f64(p.q_nope).reshape(h_q, d_c), q_abs)
    out, lse = oracle.decode_problem(p)
    st, rp = gather_logical(p, 0)
    qr = f64(p.q_rope)[0, 0]
    for h in range(h_q):
        g = h // g_q                                    # contiguous head blocks
        c = st[g]                                       # [L, d_c]
        K = np.concatenate([c @ W_UK[h], rp], axis=1)   # explicit per-head key
        V = c @ W_UV[h]                                 # explicit per-head value
        q = np.concatenate([q_raw[h], qr[h]])
        ref, _ = textbook_attention(q, K, V, p.scale)
        got = out[0, 0, h] @ W_UV[h]                    # up-projection after attention
        np.testing.assert_allclose(got, ref, rtol=0, atol=TOL)


def bits_of(x: np.ndarray) -> np.ndarray:
    """fp64 array of values that bf16 holds exactly -> their bf16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16)
    assert np.array_equal(f64(t), x), "value not representable in bf16"
    return bf16_bits(t)


def test_whole_absorbed_block_equals_explicit_attention_with_separate_projections():
    """Sections 2.1 and 3.3.2 end to end on a tiny case: raw per-head queries,
    W_UK absorbed on the query side (oracle.project, one matrix per head), the
    latent attention, then the grouped output projection with W^vo = W_UV W_O
    (oracle.project summed over the groups), against per-head attention over
    explicitly up-projected keys and values followed by the ordinary output
    projection sum_h o_h W_O^h.  Small integer weights keep every intermediate
    that crosses a bf16 interface exactly representable, except the latent
    output itself, which BOTH sides take rounded to bf16: the identity checked
    downstream of it is then exact."""
    rng = np.random.default_rng(21)
    h_q, h_c, d_c, d_h, d_r, D, L, B, T = 6, 2, 16, 8, 4, 10, 29, 2, 2
    g_q = h_q // h_c
    p = make_problem("block", seq_lens=[L, 7], T=T, h_q=h_q, h_c=h_c, d_v=d_c, d_r=d_r, page_size=8, seed=12, scale=0.3)
    W_UK = rng.integers(-1, 2, size=(h_q, d_c, d_h)).astype(np.float64)       # [head][latent dim n][head dim k]
    W_UV = rng.integers(-1, 2, size=(h_q, d_c, d_h)).astype(np.float64)
    W_O = rng.integers(-1, 2, size=(h_q, d_h, D)).astype(np.float64)
    q_raw = rng.integers(-2, 3, size=(B, T, h_q, d_h)).astype(np.float64)
    # --- query side: q~[m][h][n] = sum_k W_UK[h][n][k] q[m][h][k]
    q_abs = oracle.project(bits_of(q_raw.reshape(B * T, h_q, d_h)), bits_of(W_UK), sum_groups=False)
    np.testing.assert_array_equal(q_abs, np.einsum("hnk,mhk->mhn", W_UK, q_raw.reshape(B * T, h_q, d_h)))
    p.q_nope = torch.from_numpy(q_abs.reshape(B, T, h_q, d_c)).to(torch.bfloat16)
    assert np.array_equal(f64(p.q_nope).reshape(B * T, h_q, d_c), q_abs)      # |.| <= 16: exact in bf16
    out, _ = oracle.decode_problem(p)                                          # [B, T, h_q, d_c] latent-space outputs
    out_bf = torch.from_numpy(out).to(torch.bfloat16)                          # the interface between the two kernels
    # --- output side: W^vo of group g, output-major: [D][g_q * d_c], rows of head h inside it = W_UV[h] W_O[h]
    W_vo = np.einsum("hcd,hdn->hcn", W_UV, W_O)                                # [h_q][d_c][D], |.| <= 8
    W_vo_g = W_vo.reshape(h_c, g_q * d_c, D).transpose(0, 2, 1)                # [G][N = D][K = g_q * d_c]
    y = oracle.project(bf16_bits(out_bf.reshape(B * T, h_c, g_q * d_c)), bits_of(W_vo_g), sum_groups=True)
    # --- explicit: per-head keys / values, textbook attention, up-projected value output, ordinary W_O
    y_ref = np.zeros((B * T, D))
    qr = f64(p.q_rope)
    for b in range(B):
        st, rp = gather_logical(p, b)
        for t in range(T):
            n_vis = int(p.seq_lens[b]) - T + 1 + t
            for h in range(h_q):
                c = st[h // g_q][:n_vis]
                K = np.concatenate([c @ W_UK[h], rp[:n_vis]], axis=1)
                V = c @ W_UV[h]
                o_h, _ = textbook_attention(np.concatenate([q_raw[b, t, h], qr[b, t, h]]), K, V, p.scale)
                # the explicit per-head output equals the up-projected latent output (the identity of the test above) ...
                np.testing.assert_allclose(out[b, t, h] @ W_UV[h], o_h, rtol=0, atol=TOL)
                # ... and downstream of the bf16 interface both sides use the rounded latent output
                y_ref[b * T + t] += (f64(out_bf)[b, t, h] @ W_UV[h]) @ W_O[h]
    np.testing.assert_allclose(y, y_ref, rtol=0, atol=1e-9)


def test_projection_against_numpy_and_closed_forms():
    """oracle.project against numpy's fp64 products on random bf16 data, with and
    without the sum over groups; identity weights copy the input; a transposed
    weight operand or a group taken from the wrong stride would show."""
    g = torch.Generator().manual_seed(5)
    M, G, N, K = 7, 3, 11, 20
    a = torch.randn(M, G, K, generator=g).to(torch.bfloat16)
    w = torch.randn(G, N, K, generator=g).to(torch.bfloat16)
    ref = np.einsum("mgk,gnk->mgn", f64(a), f64(w))
    np.testing.assert_allclose(oracle.project(bf16_bits(a), bf16_bits(w), sum_groups=False), ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.project(bf16_bits(a), bf16_bits(w), sum_groups=True), ref.sum(axis=1), rtol=0, atol=1e-12)
    eye = torch.eye(K).repeat(G, 1, 1).to(torch.bfloat16)                      # N == K: C[m][g] = A[m][g]
    np.testing.assert_array_equal(oracle.project(bf16_bits(a), bf16_bits(eye), sum_groups=False), f64(a))
    one_hot = torch.zeros(G, N, K, dtype=torch.bfloat16)
    one_hot[1, 4, 9] = 1.0                                                     # picks A[m][1][9] into C[m][1][4] only
    got = oracle.project(bf16_bits(a), bf16_bits(one_hot), sum_groups=False)
    want = np.zeros((M, G, N))
    want[:, 1, 4] = f64(a)[:, 1, 9]
    np.testing.assert_array_equal(got, want)


def test_gqa_oracle_against_textbook_attention_and_as_generalisation_of_gta():
    """The grouped-query baseline (separate key and value caches): (a) textbook
    attention on the gathered keys / values of every row, causal rows included;
    (b) Section 3.3.1 read the other way round: a GTA problem IS the GQA problem
    whose key rows are [first half of the tied state | shared RoPE key] and whose
    values are the tied state, so both oracle functions must agree on it."""
    p = make_problem("gqa_pin", kind="gqa", seq_lens=[37, 5, 0, 16], T=2, h_q=8, h_c=2, d_v=16, page_size=8, seed=31,
                     poison_tail=True)
    out, lse = oracle.decode_problem(p)
    g_q = p.h_q // p.h_c
    for b in range(p.B):
        L = int(p.seq_lens[b])
        n = (L + p.page_size - 1) // p.page_size
        idx = p.table_compact[b, :n]
        K = f64(p.key_pages)[idx].transpose(1, 0, 2, 3).reshape(p.h_c, n * p.page_size, p.d_n)
        V = f64(p.state_pages)[idx].transpose(1, 0, 2, 3).reshape(p.h_c, n * p.page_size, p.d_v)
        for t in range(p.T):
            n_vis = L - p.T + 1 + t
            for h in range(p.h_q):
                if n_vis <= 0:
                    assert np.isneginf(lse[b, t, h]) and (out[b, t, h] == 0).all()
                    continue
                ref, _ = textbook_attention(f64(p.q_nope)[b, t, h], K[h // g_q][:n_vis], V[h // g_q][:n_vis], p.scale)
                np.testing.assert_allclose(out[b, t, h], ref, rtol=0, atol=TOL)
    # (b)
    pg = make_problem("gta_as_gqa", kind="gta", seq_lens=[29, 8, 3], T=2, h_q=8, h_c=2, d_v=16, d_r=4, page_size=8, seed=32)
    out_t, lse_t = oracle.decode_problem(pg)
    st = pg.state_pages                                              # [n, h_c, P, d_h]
    key = torch.cat([st[..., :pg.d_n], pg.rope_pages[:, None].expand(-1, pg.h_c, -1, -1)], dim=-1)
    q = torch.cat([pg.q_nope, pg.q_rope], dim=-1)
    out_q, lse_q = oracle.gqa_decode(bf16_bits(q), bf16_bits(key), bf16_bits(st), pg.table_compact, pg.seq_lens,
                                     scale=pg.scale, causal=pg.causal)
    np.testing.assert_allclose(out_q, out_t, rtol=0, atol=TOL)
    np.testing.assert_allclose(lse_q, lse_t, rtol=0, atol=TOL)


# ---------------------------------------------------------------- P2
def test_softmax_weights_are_a_distribution():
    p = make_problem("p2", seq_lens=[19, 64, 1], T=2, h_q=4, h_c=2, d_v=8, d_r=4, page_size=16,
                     seed=12)
    out, lse, w = oracle.decode_problem(p, return_weights=True)
    assert (w >= 0).all()
    w = w.reshape(p.B, p.T, p.h_q, -1)
    for b in range(p.B):
        for t in range(p.T):
            n_vis = int(p.seq_lens[b]) - p.T + 1 + t
            if n_vis <= 0:
                assert (w[b, t] == 0).all()
                continue
            np.testing.assert_allclose(w[b, t].sum(-1), 1.0, atol=1e-12)
            assert (w[b, t, :, n_vis:] == 0).all()


# ---------------------------------------------------------------- P3
@pytest.mark.parametrize("cuts", [[], [20], [1, 2], [5, 5, 30, 31, 40, 49]])
def test_split_then_merge_equals_single_pass(cuts):
    p = make_problem("p3", seq_lens=[50, 7], T=2, h_q=4, h_c=2, d_v=8, d_r=4, page_size=8, seed=13)
    full_out, full_lse = oracle.decode_problem(p)
    edges = [0] + cuts + [10 ** 9]
    parts = [oracle.decode_problem(p, key_range=(a, b)) for a, b in zip(edges[:-1], edges[1:])]
    out, lse = oracle.merge(np.stack([x[0] for x in parts]), np.stack([x[1] for x in parts]))
    np.testing.assert_allclose(out, full_out, atol=TOL)
    np.testing.assert_allclose(lse, full_lse, atol=TOL)


def test_merge_closed_form():
    """Two parts with equal lse average their outputs and add ln 2; an empty
    part (lse = -inf) is ignored."""
    o = np.array([[[1.0, 3.0]], [[3.0, 5.0]], [[100.0, 100.0]]])
    l = np.array([[0.5], [0.5], [-np.inf]])
    out, lse = oracle.merge(o, l)
    np.testing.assert_allclose(out, [[2.0, 4.0]], atol=1e-15)
    np.testing.assert_allclose(lse, [0.5 + math.log(2.0)], atol=1e-15)
    out, lse = oracle.merge(o[2:], l[2:])
    assert (out == 0).all() and np.isneginf(lse).all()


# ---------------------------------------------------------------- P4
def test_gta_equals_gqa_with_assembled_key():
    """Section 3.3.1: V = tied state, K = concat(first half of the tied state,
    shared RoPE key broadcast to every KV head)."""
    h_q, h_kv, d_h, L = 8, 4, 16, 45
    p = make_problem("p4", kind="gta", seq_lens=[L, 3], h_q=h_q, h_c=h_kv, d_v=d_h,
                     d_r=d_h // 2, page_size=8, seed=14)
    out, lse = oracle.decode_problem(p)
    g_q = h_q // h_kv
    for b in range(p.B):
        st, rp = gather_logical(p, b)
        for h in range(h_q):
            kv = st[h // g_q]                                    # [L, d_h]
            K = np.concatenate([kv[:, : d_h // 2], rp], axis=1)  # NoPE half first
            V = kv
            q = np.concatenate([f64(p.q_nope)[b, 0, h], f64(p.q_rope)[b, 0, h]])
            ref, _ = textbook_attention(q, K, V, p.scale)
            np.testing.assert_allclose(out[b, 0, h], ref, atol=TOL)


# ---------------------------------------------------------------- P5
def test_single_latent_no_rope_is_mqa_with_k_equal_v():
    """h_c = 1 and d_R = 0 reduce to multi-query attention with K = V; checked
    against torch's own softmax/matmul in fp64."""
    p = make_problem("p5", seq_lens=[33], h_q=5, h_c=1, d_v=12, d_r=4, page_size=4, seed=15)
    out, lse = oracle.decode(bf16_bits(p.q_nope), None, bf16_bits(p.state_pages), None,
                             p.table_compact, p.seq_lens, h_c=1, scale=p.scale)
    st, _ = gather_logical(p, 0)
    c = torch.from_numpy(st[0])
    q = p.q_nope[0, 0].to(torch.float64)
    s = p.scale * q @ c.T
    ref = torch.softmax(s, dim=-1) @ c
    np.testing.assert_allclose(out[0, 0], ref.numpy(), atol=TOL)
    np.testing.assert_allclose(lse[0, 0], torch.logsumexp(s, dim=-1).numpy(), atol=TOL)


def test_gla2_is_two_independent_single_latent_problems():
    """Section 3.3.2: O_0 uses (Q_0, c_0) only and O_1 uses (Q_1, c_1) only."""
    p = make_problem("p5b", seq_lens=[40, 9], h_q=6, h_c=2, d_v=8, d_r=4, page_size=8, seed=16)
    out, lse = oracle.decode_problem(p)
    g_q = p.g_q
    for g in range(2):
        o_g, l_g = oracle.decode(bf16_bits(p.q_nope[:, :, g * g_q:(g + 1) * g_q]),
                                 bf16_bits(p.q_rope[:, :, g * g_q:(g + 1) * g_q]),
                                 bf16_bits(p.state_pages[:, g:g + 1]), bf16_bits(p.rope_pages),
                                 p.table_compact, p.seq_lens, h_c=1, scale=p.scale)
        assert np.array_equal(o_g, out[:, :, g * g_q:(g + 1) * g_q])
        assert np.array_equal(l_g, lse[:, :, g * g_q:(g + 1) * g_q])


# ---------------------------------------------------------------- P6
def test_closed_forms():
    p = make_problem("p6", seq_lens=[1, 23], h_q=4, h_c=2, d_v=8, d_r=4, page_size=8, seed=17)
    out, lse = oracle.decode_problem(p)
    # one key: output is that key, lse is its score
    st, rp = gather_logical(p, 0)
    for h in range(4):
        np.testing.assert_allclose(out[0, 0, h], st[h // 2, 0], atol=0)
        s0 = p.scale * (f64(p.q_nope)[0, 0, h] @ st[h // 2, 0] + f64(p.q_rope)[0, 0, h] @ rp[0])
        np.testing.assert_allclose(lse[0, 0, h], s0, atol=1e-14)
    # zero query: uniform weights
    p.q_nope.zero_()
    p.q_rope.zero_()
    out, lse = oracle.decode_problem(p)
    st, rp = gather_logical(p, 1)
    for h in range(4):
        np.testing.assert_allclose(out[1, 0, h], st[h // 2].mean(0), atol=1e-14)
        np.testing.assert_allclose(lse[1, 0, h], math.log(23), atol=1e-14)


def test_constant_rope_key_shifts_lse_only():
    """If every cached RoPE key equals r, the RoPE term adds the same constant
    scale * q_rope . r to every score: weights unchanged, lse shifted by it."""
    p = make_problem("p6b", seq_lens=[29], h_q=4, h_c=2, d_v=8, d_r=4, page_size=8, seed=18)
    r = p.rope_pages[0, 0].clone()
    p.rope_pages[:] = r
    out, lse = oracle.decode_problem(p)
    out0, lse0 = oracle.decode(bf16_bits(p.q_nope), None, bf16_bits(p.state_pages), None,
                               p.table_compact, p.seq_lens, h_c=2, scale=p.scale)
    np.testing.assert_allclose(out, out0, atol=1e-13)
    shift = p.scale * (f64(p.q_rope)[0, 0] @ f64(r))
    np.testing.assert_allclose(lse[0, 0], lse0[0, 0] + shift, atol=1e-12)


def test_gta_score_uses_first_half_only():
    """Changing the second half of the tied state's dims must leave the WEIGHTS
    unchanged (they enter only through V), Section 3.3.1."""
    p = make_problem("p6c", kind="gta", seq_lens=[21], h_q=4, h_c=2, d_v=8, d_r=4, page_size=8,
                     seed=19)
    _, lse_a, w_a = oracle.decode_problem(p, return_weights=True)
    p.state_pages[..., 4:] = p.state_pages[..., 4:] * 2 + 1
    out_b, lse_b, w_b = oracle.decode_problem(p, return_weights=True)
    assert np.array_equal(w_a, w_b) and np.array_equal(lse_a, lse_b)
    st, _ = gather_logical(p, 0)
    np.testing.assert_allclose(out_b[0, 0, 3], w_b.reshape(1, 1, 4, -1)[0, 0, 3] @ st[1], atol=1e-13)


# ---------------------------------------------------------------- P7
def test_paging_invariance():
    p = make_problem("p7", seq_lens=[70, 33, 64], h_q=4, h_c=2, d_v=8, d_r=4, page_size=16,
                     seed=20, extra_table_cols=2)
    out, lse = oracle.decode_problem(p)
    rng = np.random.default_rng(5)
    n = p.state_pages.shape[0]
    perm = rng.permutation(n)                 # new slot of old page i is perm[i]
    inv = np.argsort(perm)
    state2 = p.state_pages[torch.from_numpy(inv)]
    rope2 = p.rope_pages[torch.from_numpy(inv)]
    table2 = np.where(p.table_compact >= 0, perm[np.maximum(p.table_compact, 0)], -1).astype(np.int32)
    out2, lse2 = oracle.decode(bf16_bits(p.q_nope), bf16_bits(p.q_rope), bf16_bits(state2),
                               bf16_bits(rope2), table2, p.seq_lens, h_c=2, scale=p.scale)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)
    # page size 1 with the same logical content
    for b in range(p.B):
        st, rp = gather_logical(p, b)
        L = st.shape[1]
        s1 = p.state_pages.new_zeros((L, 2, 1, 8))
        n_pg = (L + 15) // 16
        idx = torch.from_numpy(p.table_compact[b, :n_pg].astype(np.int64))
        s1[:, :, 0, :] = p.state_pages[idx].permute(0, 2, 1, 3).reshape(-1, 2, 8)[:L]
        r1 = p.rope_pages[idx].reshape(-1, 1, 4)[:L]
        o1, l1 = oracle.decode(bf16_bits(p.q_nope[b:b + 1]), bf16_bits(p.q_rope[b:b + 1]),
                               bf16_bits(s1), bf16_bits(r1),
                               np.arange(L, dtype=np.int32)[None], p.seq_lens[b:b + 1], h_c=2,
                               scale=p.scale)
        assert np.array_equal(o1[0], out[b]) and np.array_equal(l1[0], lse[b])


# ---------------------------------------------------------------- P8
def test_causal_row_equals_shorter_single_query_call():
    T = 4
    p = make_problem("p8", seq_lens=[37, 4, 2], T=T, h_q=4, h_c=2, d_v=8, d_r=4, page_size=8,
                     seed=21)
    out, lse = oracle.decode_problem(p)
    for t in range(T):
        lens = np.maximum(p.seq_lens - T + 1 + t, 0).astype(np.int32)
        o1, l1 = oracle.decode(bf16_bits(p.q_nope[:, t:t + 1]), bf16_bits(p.q_rope[:, t:t + 1]),
                               bf16_bits(p.state_pages), bf16_bits(p.rope_pages), p.table_compact,
                               lens, h_c=2, scale=p.scale)
        assert np.array_equal(o1[:, 0], out[:, t]) and np.array_equal(l1[:, 0], lse[:, t])
    # sequence 2 has L = 2 < T: rows 0 and 1 see nothing
    assert (out[2, 0] == 0).all() and np.isneginf(lse[2, 0]).all()
    assert (out[2, 1] == 0).all() and np.isneginf(lse[2, 1]).all()
    assert np.isfinite(lse[2, 2]).all()
    # non-causal: every row sees all L keys
    p.causal = 0
    out_nc, lse_nc = oracle.decode_problem(p)
    assert np.array_equal(out_nc[:, T - 1], out[:, T - 1])
    st, rp = gather_logical(p, 0)
    q = np.concatenate([f64(p.q_nope)[0, 0, 1], f64(p.q_rope)[0, 0, 1]])
    K = np.concatenate([st[0], rp], axis=1)
    ref, _ = textbook_attention(q, K, st[0], p.scale)
    np.testing.assert_allclose(out_nc[0, 0, 1], ref, atol=TOL)


# ---------------------------------------------------------------- P9
def test_poisoned_tail_and_unused_slots_do_not_leak():
    kw = dict(seq_lens=[19, 40, 0], T=2, h_q=4, h_c=2, d_v=8, d_r=4, page_size=16, seed=22,
              extra_table_cols=3)
    clean = make_problem("p9", **kw)
    dirty = make_problem("p9", poison_tail=True, **kw)
    assert torch.isnan(dirty.state_pages).any()
    assert (dirty.table_compact[:, -1] == -1).all()
    o1, l1 = oracle.decode_problem(clean)
    o2, l2 = oracle.decode_problem(dirty)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    assert (o1[2] == 0).all() and np.isneginf(l1[2]).all()     # empty sequence


# ---------------------------------------------------------------- brute force
def test_brute_force_tiny_all_rows():
    """Every row of a small ragged GLA problem against the textbook routine."""
    p = make_problem("bf", seq_lens=[13, 1, 30], T=3, h_q=6, h_c=3, d_v=6, d_r=2, page_size=4,
                     seed=23, q_gain=3.0)
    out, lse, w = oracle.decode_problem(p, return_weights=True)
    w = w.reshape(p.B, p.T, p.h_q, -1)
    for b in range(p.B):
        st, rp = gather_logical(p, b)
        for t in range(p.T):
            n_vis = int(p.seq_lens[b]) - p.T + 1 + t
            for h in range(p.h_q):
                if n_vis <= 0:
                    assert (out[b, t, h] == 0).all() and np.isneginf(lse[b, t, h])
                    continue
                c = st[h // p.g_q][:n_vis]
                K = np.concatenate([c, rp[:n_vis]], axis=1)
                q = np.concatenate([f64(p.q_nope)[b, t, h], f64(p.q_rope)[b, t, h]])
                ref, pw = textbook_attention(q, K, c, p.scale)
                np.testing.assert_allclose(out[b, t, h], ref, atol=TOL)
                np.testing.assert_allclose(w[b, t, h, :n_vis], pw, atol=TOL)
                s = p.scale * (K @ q)
                np.testing.assert_allclose(lse[b, t, h], math.log(np.exp(s - s.max()).sum()) + s.max(),
                                           atol=TOL)


def test_selected_rows_match_full():
    p = make_problem("sel", seq_lens=[25, 40], T=2, h_q=4, h_c=2, d_v=8, d_r=4, page_size=8, seed=24)
    out, lse = oracle.decode_problem(p)
    sel = [(1, 1, 3), (0, 0, 0), (1, 0, 2)]
    o, l = oracle.decode_problem(p, sel=sel)
    for i, (b, t, h) in enumerate(sel):
        assert np.array_equal(o[i], out[b, t, h]) and l[i] == lse[b, t, h]


def test_bad_arguments_are_rejected():
    p = make_problem("bad", seq_lens=[5], h_q=4, h_c=2, d_v=8, d_r=4, page_size=8, seed=25)
    with pytest.raises(ValueError):
        oracle.decode(bf16_bits(p.q_nope[:, :, :3]), bf16_bits(p.q_rope[:, :, :3]),
                      bf16_bits(p.state_pages), bf16_bits(p.rope_pages), p.table_compact,
                      p.seq_lens, h_c=2, scale=1.0)
