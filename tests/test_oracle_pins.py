"""Pins for the CPU oracle: closed forms, invariants, special cases and a dense brute force.

None of these call the oracle's own formula again: each fixes the oracle to something the
mathematics or the paper's printed numbers determine, chosen so that a dropped term, a wrong
index, a swapped operand or a wrong head map fails at least one of them.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import reference as ref

HERE = os.path.dirname(os.path.abspath(__file__))


def bf16(x):
    return torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)


def rand_bf16(rng, shape, scale=1.0):
    return bf16(rng.standard_normal(shape) * scale)


def f64(t):
    return t.to(torch.float64).numpy()


def make_store(rng, lens, Hkv=2, D=128, P=16, L=1, k=None, v=None, seed=3):
    n_pages = sum(-(-n // P) for n in lens) * L + 7
    st = ref.PagedStore(L, Hkv, D, P, n_pages, seed=seed)
    ks, vs = [], []
    for r, n in enumerate(lens):
        st.add_request(r)
        for l in range(L):
            kk = k[r] if k is not None else rand_bf16(rng, (n, Hkv, D))
            vv = v[r] if v is not None else rand_bf16(rng, (n, Hkv, D))
            st.write(r, l, 0, kk, vv)
            if l == 0:
                ks.append(kk)
                vs.append(vv)
    return st, ks, vs


def dense_longdouble(q, k, v, Hq, scale):
    """Independent dense path: no pages, long double, per-head loops written differently."""
    n, Hkv, D = k.shape
    G = Hq // Hkv
    qd = f64(q).astype(np.longdouble)
    kd = f64(k).astype(np.longdouble)
    vd = f64(v).astype(np.longdouble)
    out = np.zeros((Hq, D), dtype=np.longdouble)
    for h in range(Hq):
        g = h // G
        logits = np.array([np.dot(qd[h], kd[t, g]) for t in range(n)], dtype=np.longdouble) * np.longdouble(scale)
        e = np.exp(logits - logits.max())
        p = e / e.sum()
        for t in range(n):
            out[h] += p[t] * vd[t, g]
    return out.astype(np.float64)


# ------------------------------------------------------------------ closed forms

def test_single_token_returns_v_exactly():
    rng = np.random.default_rng(0)
    st, ks, vs = make_store(rng, [1, 1, 1], Hkv=2)
    q = rand_bf16(rng, (3, 8, 128), 3.0)
    o = ref.decode_attention(st, 0, [0, 1, 2], q, 8)
    for r in range(3):
        for h in range(8):
            assert np.array_equal(o[r, h], f64(vs[r])[0, h // 4])


@pytest.mark.parametrize("n", [17, 1000])
def test_identical_keys_give_mean_of_v(n):
    rng = np.random.default_rng(1)
    k1 = rand_bf16(rng, (1, 2, 128))
    k = [k1.expand(n, 2, 128).contiguous()]
    st, ks, vs = make_store(rng, [n], k=k)
    q = rand_bf16(rng, (1, 8, 128))
    o = ref.decode_attention(st, 0, [0], q, 8)
    mean = f64(vs[0]).mean(axis=0)                       # [Hkv][D]
    for h in range(8):
        np.testing.assert_allclose(o[0, h], mean[h // 4], rtol=0, atol=1e-13)


def test_zero_query_gives_mean_of_v_and_masks_partial_page():
    # n = 17: one full block plus one token; slots 1..15 of the second block hold NaN poison
    rng = np.random.default_rng(2)
    st, ks, vs = make_store(rng, [17])
    q = torch.zeros((1, 8, 128), dtype=torch.bfloat16)
    o = ref.decode_attention(st, 0, [0], q, 8)
    assert np.all(np.isfinite(o))
    np.testing.assert_allclose(o[0, 5], f64(vs[0]).mean(axis=0)[1], atol=1e-13)


def test_weights_sum_to_one_and_lie_in_unit_interval():
    rng = np.random.default_rng(3)
    st, ks, vs = make_store(rng, [777])
    q = rand_bf16(rng, (8, 128), 2.0)
    for h in (0, 7):
        w, o = ref.attention_weights(st, 0, 0, h, q[h], 8)
        assert abs(w.sum() - 1.0) < 1e-14
        assert np.all(w > 0) and np.all(w <= 1)
        # the output is the weighted sum of V with exactly those weights
        np.testing.assert_allclose(o, (w[:, None] * f64(vs[0])[:, h // 4]).sum(axis=0), atol=1e-13)


def test_two_token_closed_form_pins_default_scale():
    # k0 = e_0, k1 = 0, q = a*e_0  ->  s0 = a/sqrt(128), s1 = 0, weight0 = 1/(1+exp(-a/sqrt(128)))
    D, a = 128, 8.0
    k = torch.zeros((2, 1, D), dtype=torch.bfloat16)
    k[0, 0, 0] = 1.0
    v = torch.zeros((2, 1, D), dtype=torch.bfloat16)
    v[0, 0, :] = 1.0
    v[1, 0, :] = -1.0
    rng = np.random.default_rng(4)
    st, _, _ = make_store(rng, [2], Hkv=1, k=[k], v=[v])
    q = torch.zeros((1, 1, D), dtype=torch.bfloat16)
    q[0, 0, 0] = a
    o = ref.decode_attention(st, 0, [0], q, 1)
    w0 = 1.0 / (1.0 + math.exp(-a / math.sqrt(128.0)))
    np.testing.assert_allclose(o[0, 0], np.full(D, 2 * w0 - 1), atol=1e-15)
    # explicit scale 0.5: weight0 = sigmoid(4)
    o2 = ref.decode_attention(st, 0, [0], q, 1, scale=0.5)
    np.testing.assert_allclose(o2[0, 0], np.full(D, 2 / (1 + math.exp(-4.0)) - 1), atol=1e-15)


def test_scale_and_query_trade_off_exactly():
    rng = np.random.default_rng(5)
    st, ks, vs = make_store(rng, [100])
    q = rand_bf16(rng, (1, 8, 128))
    a = ref.decode_attention(st, 0, [0], q * 2, 8, scale=0.05)     # doubling is exact in bf16
    b = ref.decode_attention(st, 0, [0], q, 8, scale=0.10)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)


def test_one_hot_limit_without_overflow():
    rng = np.random.default_rng(6)
    st, ks, vs = make_store(rng, [300])
    j = 123
    q = (ks[0][j, 0] * 64.0).view(1, 1, 128).expand(1, 8, 128).contiguous()   # |s| ~ 1e3
    o = ref.decode_attention(st, 0, [0], q, 8, scale=1.0)
    assert np.all(np.isfinite(o))
    np.testing.assert_allclose(o[0, 0], f64(vs[0])[j, 0], atol=1e-9)


# ------------------------------------------------------------------ head map

def test_group_map_is_contiguous():
    rng = np.random.default_rng(7)
    st, ks, vs = make_store(rng, [64], Hkv=2)
    q1 = rand_bf16(rng, (128,))
    q = q1.view(1, 1, 128).expand(1, 8, 128).contiguous()
    o = ref.decode_attention(st, 0, [0], q, 8)
    for h in (1, 2, 3):
        assert np.array_equal(o[0, h], o[0, 0])              # heads 0..3 share KV head 0
    for h in (5, 6, 7):
        assert np.array_equal(o[0, h], o[0, 4])              # heads 4..7 share KV head 1
    assert not np.allclose(o[0, 0], o[0, 4])
    # swapping the two KV heads swaps the two groups' outputs
    st2, _, _ = make_store(rng, [64], Hkv=2, k=[ks[0].flip(1).contiguous()], v=[vs[0].flip(1).contiguous()])
    o2 = ref.decode_attention(st2, 0, [0], q, 8)
    assert np.array_equal(o2[0, 0], o[0, 4]) and np.array_equal(o2[0, 4], o[0, 0])


# ------------------------------------------------------------------ paging

def test_page_permutation_leaves_output_bit_identical():
    rng = np.random.default_rng(8)
    lens = [17, 256, 1000]
    st, ks, vs = make_store(rng, lens)
    q = rand_bf16(rng, (3, 8, 128))
    a = ref.decode_attention(st, 0, [0, 1, 2], q, 8)
    st.permute_pages(99)
    b = ref.decode_attention(st, 0, [0, 1, 2], q, 8)
    assert np.array_equal(a, b)


def test_pack_unpack_roundtrip_and_layout_formula():
    rng = np.random.default_rng(9)
    Hkv, D, P = 2, 128, 16
    st, ks, vs = make_store(rng, [37], Hkv=Hkv)
    k2, v2 = st.read(0, 0, 5, 30)
    assert np.array_equal(k2, ref.as_u16(ks[0])[5:35]) and np.array_equal(v2, ref.as_u16(vs[0])[5:35])
    # restate the documented element order with numpy reshapes and compare with the raw page
    page = st.arena[st.pages[(0, 0)][1]]                      # tokens 16..31
    kt = ref.as_u16(ks[0])[16:32]                             # [tok][g][dim]
    vt = ref.as_u16(vs[0])[16:32]
    for g in range(Hkv):
        k_tile = kt[:, g, :].reshape(P, D // 8, 8).transpose(1, 0, 2).reshape(-1)      # [c][tok][8]
        assert np.array_equal(page[g * P * D:(g + 1) * P * D], k_tile)
        # V tile order [dim/32][tok/4][dim%16][(dim/16)%2][tok%4]
        v5 = vt[:, g, :].reshape(P // 4, 4, D // 32, 2, 16)   # [j][i][nbp][e][m]
        v_tile = v5.transpose(2, 0, 4, 3, 1).reshape(-1)
        off = Hkv * P * D + g * P * D
        assert np.array_equal(page[off:off + P * D], v_tile)


def test_concatenation_identity():
    # o(n1+n2) from the two halves' (max, normaliser, output): the merge rule a split
    # implementation relies on, checked here inside the oracle.
    rng = np.random.default_rng(10)
    n1, n2, D = 300, 212, 128
    k = rand_bf16(rng, (n1 + n2, 2, D))
    v = rand_bf16(rng, (n1 + n2, 2, D))
    q = rand_bf16(rng, (1, 8, D), 2.0)
    scale = 1 / math.sqrt(D)
    full, _, _ = make_store(rng, [n1 + n2], k=[k], v=[v])
    a, _, _ = make_store(rng, [n1], k=[k[:n1].contiguous()], v=[v[:n1].contiguous()])
    b, _, _ = make_store(rng, [n2], k=[k[n1:].contiguous()], v=[v[n1:].contiguous()])
    o = ref.decode_attention(full, 0, [0], q, 8)
    oa = ref.decode_attention(a, 0, [0], q, 8)
    ob = ref.decode_attention(b, 0, [0], q, 8)
    for h in range(8):
        s = scale * (f64(k)[:, h // 4] @ f64(q)[0, h])
        m1, m2 = s[:n1].max(), s[n1:].max()
        z1, z2 = np.exp(s[:n1] - m1).sum(), np.exp(s[n1:] - m2).sum()
        m = max(m1, m2)
        c1, c2 = z1 * math.exp(m1 - m), z2 * math.exp(m2 - m)
        np.testing.assert_allclose(o[0, h], (c1 * oa[0, h] + c2 * ob[0, h]) / (c1 + c2), atol=1e-12)


# ------------------------------------------------------------------ brute force

@pytest.mark.parametrize("Hq,Hkv,D,P,lens", [
    (4, 2, 32, 4, [1, 3, 4, 5, 8]),
    (8, 2, 128, 16, [17, 40]),
    (16, 2, 64, 8, [9, 33]),          # group of 8
    (3, 3, 32, 16, [20]),             # multi-head attention (group of 1)
])
def test_dense_longdouble_brute_force(Hq, Hkv, D, P, lens):
    rng = np.random.default_rng(11)
    st, ks, vs = make_store(rng, lens, Hkv=Hkv, D=D, P=P)
    q = rand_bf16(rng, (len(lens), Hq, D), 1.5)
    scale = 0.37
    o = ref.decode_attention(st, 0, list(range(len(lens))), q, Hq, scale=scale)
    for r in range(len(lens)):
        want = dense_longdouble(q[r], ks[r], vs[r], Hq, scale)
        np.testing.assert_allclose(o[r], want, rtol=0, atol=1e-13)


def test_ctx_len_override_ignores_later_tokens():
    rng = np.random.default_rng(12)
    st, ks, vs = make_store(rng, [50])
    q = rand_bf16(rng, (1, 8, 128))
    o = ref.decode_attention(st, 0, [0], q, 8, ctx_len=[23])
    want = dense_longdouble(q[0], ks[0][:23], vs[0][:23], 8, 1 / math.sqrt(128))
    np.testing.assert_allclose(o[0], want, atol=1e-13)


def test_empty_context_is_an_error():
    st = ref.PagedStore(1, 2, 128, 16, 4)
    st.add_request(0)
    with pytest.raises(ValueError):
        ref.decode_attention(st, 0, [0], torch.zeros((1, 8, 128), dtype=torch.bfloat16), 8)


# ------------------------------------------------------------------ capacity, Eq. (1)

def _toy():
    with open(os.path.join(HERE, "golden", "toy_example.json")) as f:
        return json.load(f)


def _placement(n_layers, offloaded_1based):
    x = np.ones((len(offloaded_1based), n_layers), dtype=np.int64)
    for r, layers in enumerate(offloaded_1based):
        for l in layers:
            x[r, l - 1] = 0
    return x


def test_capacity_bound_on_the_papers_example():
    toy = _toy()
    L, cap = toy["n_layers"], toy["gpu_blocks"]
    b1, b16 = toy["step1"]["blocks_per_layer"], toy["step16"]["blocks_per_layer"]
    A = _placement(L, toy["placement_A"]["offloaded_layers_1based"])
    assert ref.prefetch_buffer_blocks(b1, A) == toy["placement_A"]["blocks_moved_per_offloaded_layer"]["step1"]
    assert ref.prefetch_buffer_blocks(b16, A) == toy["placement_A"]["blocks_moved_per_offloaded_layer"]["step16"]
    assert ref.gpu_blocks_needed(b1, A) == 63 and ref.feasible(b1, A, cap)
    assert ref.feasible(b16, A, cap) is toy["placement_A"]["feasible"]["step16"]
    A_less = _placement(L, [[3, 6], [3, 6]])
    assert ref.gpu_blocks_needed(b1, A_less) == 72
    assert ref.feasible(b1, A_less, cap) is toy["placement_A"]["one_less_offloaded_layer_feasible_step1"]
    B = _placement(L, [[], [3, 6, 9]])
    assert ref.gpu_blocks_needed(b1, B) == 69 and ref.feasible(b1, B, cap)
    assert ref.gpu_blocks_needed(b16, B) == toy["placement_B"]["gpu_blocks_used_step16"]
    assert ref.feasible(b16, B, cap) is toy["placement_B"]["feasible"]["step16"]
    C = _placement(L, [[4, 8], [3, 6, 9]])                 # disjoint offloaded layers
    assert ref.gpu_blocks_needed(b16, C) == 70 and ref.feasible(b16, C, cap)
    C_overlap = _placement(L, [[3, 6], [3, 6, 9]])
    assert not ref.feasible(b16, C_overlap, cap)


def test_block_growth_only_at_16_token_boundaries():
    assert list(ref.blocks([1, 16, 17, 32, 33, 48, 49, 63, 64])) == [1, 1, 2, 2, 3, 3, 4, 4, 4]
    # 15 more decode steps move a 3-block request to 4 blocks only if a boundary is crossed
    assert ref.blocks([48 + 15])[0] == 4 and ref.blocks([40 + 15])[0] == 4 and ref.blocks([33 + 15])[0] == 3
    # request 2 "still fits" in 6 blocks after 15 steps when it started at most at 81 tokens
    assert ref.blocks([81 + 15])[0] == 6


def test_bytes_per_token_of_the_8b_shape():
    # Section 5.1 footnote: about 2 GB hold roughly 16K tokens of LLaMA3-8B KV
    per_token = 32 * 2 * 8 * 128 * 2
    assert per_token == 128 * 1024
    assert 16 * 1024 * per_token == 2 * 1024 ** 3
