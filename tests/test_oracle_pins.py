"""Pins for the CPU oracle: what the paper prints, closed forms, invariants, brute force on
tiny inputs and fp64 library routines.  None of these call the GPU library."""
import cmath
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads
from tests.conftest import read_golden

RNG = np.random.default_rng(1234)


def tiny_desc(n_q=4, n_kv=4, d=8, H=32, I=48):
    return oracle.LayerDesc(H, n_q, n_kv, d, I, 1e-5, 10000.0)


def tiny_weights(desc, seed=0, std=0.2):
    r = np.random.default_rng(seed)
    H, d = desc.hidden, desc.head_dim
    QD, KD, I = desc.n_q_heads * d, desc.n_kv_heads * d, desc.intermediate
    f = lambda *s: (r.standard_normal(s) * std).astype(np.float32)
    return {"wq": f(QD, H), "wk": f(KD, H), "wv": f(KD, H), "wo": f(H, QD), "wgate": f(I, H),
            "wup": f(I, H), "wdown": f(H, I),
            "g1": (1 + 0.1 * r.standard_normal(H)).astype(np.float32),
            "g2": (1 + 0.1 * r.standard_normal(H)).astype(np.float32)}


# ------------------------------------------------------------------ split rule
def test_split_matches_paper_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "replication_split.txt"))
    n, k = int(g["batch"]), int(g["replicas"])
    b = oracle.split_bounds(n, k)
    assert [b[j + 1] - b[j] for j in range(k)] == [int(v) for v in g["slices"].split()]


@pytest.mark.parametrize("n,k", [(0, 1), (0, 3), (1, 4), (15, 2), (15, 4), (64, 4), (7, 7), (5, 8), (1000, 3)])
def test_split_is_a_partition_into_contiguous_near_equal_slices(n, k):
    b = oracle.split_bounds(n, k)
    assert b[0] == 0 and b[-1] == n and len(b) == k + 1
    sizes = [b[j + 1] - b[j] for j in range(k)]
    assert all(s >= 0 for s in sizes) and sum(sizes) == n
    assert max(sizes) - min(sizes) <= 1


# ------------------------------------------------------------------ rotary embedding
def test_rope_position_zero_is_identity():
    z = RNG.standard_normal(16)
    assert np.array_equal(oracle.rope(z, 0, 10000.0), z)


def test_rope_d2_is_plane_rotation_by_pos_radians():
    # d = 2: one pair, theta_0 = base^0 = 1, so position p rotates by p radians
    for p in (1, 2, 7):
        out = oracle.rope(np.array([1.0, 0.0]), p, 10000.0)
        assert np.allclose(out, [math.cos(p), math.sin(p)], atol=1e-15)
        out = oracle.rope(np.array([0.0, 1.0]), p, 10000.0)
        assert np.allclose(out, [-math.sin(p), math.cos(p)], atol=1e-15)


def test_rope_pairs_are_split_half_with_geometric_frequencies():
    # d = 4, base = 10000: theta = [1, 1/100]; pairs are (0,2) and (1,3)
    p = 3
    out = oracle.rope(np.array([1.0, 0.0, 0.0, 0.0]), p, 10000.0)
    assert np.allclose(out, [math.cos(3.0), 0, math.sin(3.0), 0], atol=1e-15)
    out = oracle.rope(np.array([0.0, 1.0, 0.0, 0.0]), p, 10000.0)
    assert np.allclose(out, [0, math.cos(0.03), 0, math.sin(0.03)], atol=1e-15)
    out = oracle.rope(np.array([0.0, 0.0, 0.0, 1.0]), p, 10000.0)
    assert np.allclose(out, [0, -math.sin(0.03), 0, math.cos(0.03)], atol=1e-15)


def test_rope_equals_complex_multiplication():
    d, base, p = 64, 10000.0, 37
    z = RNG.standard_normal(d)
    out = oracle.rope(z, p, base)
    for i in range(d // 2):
        w = complex(z[i], z[i + d // 2]) * cmath.exp(1j * p * base ** (-2.0 * i / d))
        assert abs(out[i] - w.real) < 1e-13 and abs(out[i + d // 2] - w.imag) < 1e-13


def test_rope_is_orthogonal_additive_and_relative():
    d, base = 32, 10000.0
    q, k = RNG.standard_normal(d), RNG.standard_normal(d)
    assert math.isclose(np.linalg.norm(oracle.rope(q, 11, base)), np.linalg.norm(q), rel_tol=1e-13)
    assert np.allclose(oracle.rope(oracle.rope(q, 5, base), 9, base), oracle.rope(q, 14, base), atol=1e-12)
    a = oracle.rope(q, 20, base) @ oracle.rope(k, 13, base)
    b = oracle.rope(q, 107, base) @ oracle.rope(k, 100, base)
    assert math.isclose(a, b, rel_tol=1e-11, abs_tol=1e-12)


# ------------------------------------------------------------------ attention of one query
def test_attention_probabilities_sum_to_one_and_uniform_on_equal_scores():
    d, n = 8, 11
    q = RNG.standard_normal(d)
    keys, vals = RNG.standard_normal((n, d)), RNG.standard_normal((n, d))
    _, p = oracle.attend(q, keys, vals)
    assert math.isclose(p.sum(), 1.0, rel_tol=1e-14) and (p > 0).all()
    same = np.tile(keys[:1], (n, 1))
    out, p = oracle.attend(q, same, vals)
    assert np.allclose(p, 1.0 / n, atol=1e-15)
    assert np.allclose(out, vals.mean(axis=0), atol=1e-14)


def test_attention_single_key_returns_its_value_exactly():
    d = 8
    q, k, v = RNG.standard_normal(d), RNG.standard_normal((1, d)), RNG.standard_normal((1, d))
    out, p = oracle.attend(q, k, v)
    assert p[0] == 1.0 and np.array_equal(out, v[0])


def test_attention_brute_force_pure_python():
    d, n = 4, 6
    q = RNG.standard_normal(d)
    keys, vals = RNG.standard_normal((n, d)), RNG.standard_normal((n, d))
    s = [sum(q[c] * keys[j][c] for c in range(d)) / math.sqrt(d) for j in range(n)]
    e = [math.exp(v) for v in s]          # no max subtraction: a different but equal form
    den = math.fsum(e)
    ref = [math.fsum(e[j] / den * vals[j][c] for j in range(n)) for c in range(d)]
    out, p = oracle.attend(q, keys, vals)
    assert np.allclose(out, ref, rtol=1e-13, atol=1e-14)
    assert np.allclose(p, [v / den for v in e], rtol=1e-13)


def test_attention_is_shift_invariant_for_large_scores():
    d, n = 4, 5
    q = np.array([300.0, 0, 0, 0])
    keys = np.zeros((n, d)); keys[:, 0] = [1, 2, 3, 4, 5]
    vals = np.eye(n, d)
    out, p = oracle.attend(q, keys, vals)     # scores 150..750: overflow without the max shift
    assert np.isfinite(out).all() and math.isclose(p.sum(), 1.0, rel_tol=1e-14)
    assert p[-1] > 0.999999


# ------------------------------------------------------------------ projection / norm vs fp64 library
def test_linear_matches_fp64_library_matmul_on_non_square_shapes():
    x = RNG.standard_normal((5, 37)).astype(np.float32)
    W = RNG.standard_normal((13, 37)).astype(np.float32)      # [out, in]
    ref = (torch.from_numpy(x).double() @ torch.from_numpy(W).double().T).numpy()
    y = oracle.linear(x, W)
    assert y.shape == (5, 13)
    assert np.allclose(y, ref, rtol=1e-6, atol=1e-6)
    # y[t, n] is row t of x against row n of W: a one-hot check that fails for any transposition
    x1 = np.zeros((2, 3), np.float32); x1[1, 2] = 1.0
    W1 = np.arange(12, dtype=np.float32).reshape(4, 3)
    assert np.array_equal(oracle.linear(x1, W1), np.array([[0, 0, 0, 0], [2, 5, 8, 11]], np.float32))


def test_rmsnorm_unit_rms_scale_invariance_and_library():
    x = RNG.standard_normal((3, 64)).astype(np.float32)
    g1 = np.ones(64, np.float32)
    y = oracle.rmsnorm(x, g1, 0.0).astype(np.float64)
    assert np.allclose(np.sqrt((y ** 2).mean(axis=1)), 1.0, atol=1e-6)
    assert np.allclose(oracle.rmsnorm(4.0 * x, g1, 0.0), oracle.rmsnorm(x, g1, 0.0), atol=1e-6)
    g = (1 + 0.1 * RNG.standard_normal(64)).astype(np.float32)
    ref = F.rms_norm(torch.from_numpy(x).double(), (64,), torch.from_numpy(g).double(), 1e-5).numpy()
    assert np.allclose(oracle.rmsnorm(x, g, 1e-5), ref, rtol=1e-6, atol=1e-6)
    # eps sits inside the square root, added to the mean square
    z = np.zeros((1, 4), np.float32); z[0, 0] = 2.0          # mean square 1
    assert np.allclose(oracle.rmsnorm(z, np.ones(4, np.float32), 3.0)[0, 0], 2.0 / math.sqrt(1.0 + 3.0), rtol=1e-7)


# ------------------------------------------------------------------ whole layer
def _rope_complex(t, base):
    """[rows, heads, d] fp64 rotated to positions 0..rows-1 by complex multiplication."""
    rows, heads, d = t.shape
    half = d // 2
    z = torch.complex(t[..., :half], t[..., half:])
    theta = torch.tensor([base ** (-2.0 * i / d) for i in range(half)], dtype=torch.float64)
    ang = torch.arange(rows, dtype=torch.float64)[:, None] * theta[None, :]
    z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def _library_prefill(desc, w, x_seq):
    """One unpadded sequence [len, H] through fp64 library routines (rms_norm, matmul,
    scaled_dot_product_attention, silu)."""
    W = {k: torch.from_numpy(v).double() for k, v in w.items()}
    x = torch.from_numpy(x_seq).double()
    n, d, nq, nkv = x.shape[0], desc.head_dim, desc.n_q_heads, desc.n_kv_heads
    h = F.rms_norm(x, (desc.hidden,), W["g1"], desc.rms_eps)
    q = _rope_complex((h @ W["wq"].T).view(n, nq, d), desc.rope_base)
    k = _rope_complex((h @ W["wk"].T).view(n, nkv, d), desc.rope_base)
    v = (h @ W["wv"].T).view(n, nkv, d)
    k = k.repeat_interleave(nq // nkv, dim=1)
    v = v.repeat_interleave(nq // nkv, dim=1)
    a = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                       v.transpose(0, 1)[None], is_causal=True)[0]
    a = a.transpose(0, 1).reshape(n, nq * d)
    x1 = x + a @ W["wo"].T
    h2 = F.rms_norm(x1, (desc.hidden,), W["g2"], desc.rms_eps)
    u = F.silu(h2 @ W["wgate"].T) * (h2 @ W["wup"].T)
    return (x1 + u @ W["wdown"].T).numpy(), k, v


@pytest.mark.parametrize("n_q,n_kv", [(4, 4), (4, 2), (4, 1)])
def test_prefill_layer_matches_fp64_library_composition(n_q, n_kv):
    desc = tiny_desc(n_q, n_kv)
    w = tiny_weights(desc, 3)
    B, S = 3, 9
    x = RNG.standard_normal((B, S, desc.hidden)).astype(np.float32)
    lens = np.array([9, 4, 1], np.int32)
    y = oracle.decoder_layer_prefill(desc, w, x, lens)
    for b in range(B):
        ref, _, _ = _library_prefill(desc, w, x[b, :lens[b]])
        assert np.allclose(y[b, :lens[b]], ref, rtol=2e-6, atol=2e-6)
        assert not y[b, lens[b]:].any()          # padded rows are written as zero


def test_prefill_is_causal_and_ignores_padding():
    desc = tiny_desc()
    w = tiny_weights(desc, 4)
    x = RNG.standard_normal((1, 8, desc.hidden)).astype(np.float32)
    y = oracle.decoder_layer_prefill(desc, w, x, np.array([8], np.int32))
    x2 = x.copy(); x2[0, 5:] += 1.0
    y2 = oracle.decoder_layer_prefill(desc, w, x2, np.array([8], np.int32))
    assert np.array_equal(y[0, :5], y2[0, :5]) and not np.allclose(y[0, 5:], y2[0, 5:])
    y3 = oracle.decoder_layer_prefill(desc, w, x2, np.array([5], np.int32))
    assert np.array_equal(y3[0, :5], y[0, :5])


def test_layer_special_cases_zero_projections():
    desc = tiny_desc()
    w = tiny_weights(desc, 5)
    x = RNG.standard_normal((2, 6, desc.hidden)).astype(np.float32)
    lens = np.array([6, 6], np.int32)
    w0 = dict(w, wo=np.zeros_like(w["wo"]), wdown=np.zeros_like(w["wdown"]))
    assert np.array_equal(oracle.decoder_layer_prefill(desc, w0, x, lens), x)   # both residual branches vanish
    # gate = 0 => silu(0) * up = 0 => y = x1 = x + attention branch; equal to a layer whose down is 0
    wg = dict(w, wgate=np.zeros_like(w["wgate"]))
    wd = dict(w, wdown=np.zeros_like(w["wdown"]))
    assert np.array_equal(oracle.decoder_layer_prefill(desc, wg, x, lens),
                          oracle.decoder_layer_prefill(desc, wd, x, lens))
    assert not np.allclose(oracle.decoder_layer_prefill(desc, wd, x, lens), x)


def test_first_prefill_row_attends_only_to_itself():
    # with one visible key attention returns v exactly, so row 0 has a closed form through
    # library routines without any softmax
    desc = tiny_desc(4, 2)
    w = tiny_weights(desc, 6)
    x = RNG.standard_normal((1, 3, desc.hidden)).astype(np.float32)
    y = oracle.decoder_layer_prefill(desc, w, x, np.array([3], np.int32))
    W = {k: torch.from_numpy(v).double() for k, v in w.items()}
    x0 = torch.from_numpy(x[0, :1]).double()
    h = F.rms_norm(x0, (desc.hidden,), W["g1"], desc.rms_eps)
    v = (h @ W["wv"].T).view(1, desc.n_kv_heads, desc.head_dim)
    a = v.repeat_interleave(desc.n_q_heads // desc.n_kv_heads, dim=1).reshape(1, -1)
    x1 = x0 + a @ W["wo"].T
    h2 = F.rms_norm(x1, (desc.hidden,), W["g2"], desc.rms_eps)
    ref = x1 + (F.silu(h2 @ W["wgate"].T) * (h2 @ W["wup"].T)) @ W["wdown"].T
    assert np.allclose(y[0, 0], ref.numpy()[0], rtol=2e-6, atol=2e-6)


@pytest.mark.parametrize("n_q,n_kv", [(4, 4), (4, 2)])
def test_prefill_then_decode_equals_longer_prefill(n_q, n_kv):
    """Prefill of S tokens fills the cache; one decode step with token S must reproduce row S
    of a prefill of S + 1 tokens.  Pins cache slot, rotary position and the L + 1 visible keys."""
    desc = tiny_desc(n_q, n_kv)
    w = tiny_weights(desc, 7)
    B, S, cap = 2, 6, 10
    x = RNG.standard_normal((B, S + 1, desc.hidden)).astype(np.float32)
    full = oracle.decoder_layer_prefill(desc, w, x, np.array([S + 1, S + 1], np.int32))
    kc = np.zeros((B, n_kv, cap, desc.head_dim), np.float32)
    vc = np.zeros_like(kc)
    lens = np.array([S, S - 2], np.int32)        # second sequence: shorter history
    oracle.decoder_layer_prefill(desc, w, np.ascontiguousarray(x[:, :S]), lens, kc, vc)
    assert not kc[1, :, S - 2:].any() and kc[0, :, S - 1].any()
    xd = np.stack([x[0, S], x[1, S - 2]])
    yd = oracle.decoder_layer_decode(desc, w, xd, lens, kc, vc)
    assert np.allclose(yd[0], full[0, S], rtol=1e-5, atol=1e-6)
    assert np.allclose(yd[1], full[1, S - 2], rtol=1e-5, atol=1e-6)
    assert kc[0, :, S].any() and vc[1, :, S - 2].any() and not kc[0, :, S + 1:].any()


def test_decode_with_empty_cache_returns_value_path():
    desc = tiny_desc()
    w = tiny_weights(desc, 8)
    x = RNG.standard_normal((2, desc.hidden)).astype(np.float32)
    kc = np.zeros((2, 4, 4, 8), np.float32); vc = np.zeros_like(kc)
    yd = oracle.decoder_layer_decode(desc, w, x, np.array([0, 0], np.int32), kc, vc)
    yp = oracle.decoder_layer_prefill(desc, w, x[:, None, :], np.array([1, 1], np.int32))
    assert np.allclose(yd, yp[:, 0], rtol=1e-6, atol=1e-7)


def test_gqa_equals_mha_on_repeated_kv_heads():
    dg = tiny_desc(4, 2)
    wg = tiny_weights(dg, 9)
    dm = tiny_desc(4, 4)
    d = dg.head_dim
    rep = lambda m: np.repeat(m.reshape(2, d, -1), 2, axis=0).reshape(4 * d, -1)
    wm = dict(wg, wk=rep(wg["wk"]), wv=rep(wg["wv"]))
    x = RNG.standard_normal((2, 5, dg.hidden)).astype(np.float32)
    lens = np.array([5, 3], np.int32)
    assert np.array_equal(oracle.decoder_layer_prefill(dg, wg, x, lens),
                          oracle.decoder_layer_prefill(dm, wm, x, lens))


# ------------------------------------------------------------------ split == unsplit
@pytest.mark.parametrize("k", [1, 2, 3, 4, 7])
def test_replica_split_output_is_bit_identical_to_unsplit(k):
    desc = tiny_desc(4, 2)
    w = tiny_weights(desc, 10)
    B, S = 5, 7
    x = RNG.standard_normal((B, S, desc.hidden)).astype(np.float32)
    lens = np.array([7, 3, 5, 1, 6], np.int32)
    whole = oracle.decoder_layer_prefill(desc, w, x, lens)
    parts = oracle.forward_split(
        lambda lo, hi: oracle.decoder_layer_prefill(desc, w, np.ascontiguousarray(x[lo:hi]), lens[lo:hi]), B, k)
    assert np.array_equal(parts, whole)
    # decode, and the single projection split over token rows
    kc = RNG.standard_normal((B, 2, 8, 8)).astype(np.float32); vc = RNG.standard_normal((B, 2, 8, 8)).astype(np.float32)
    xd = x[:, 0]
    k1, v1 = kc.copy(), vc.copy()
    whole = oracle.decoder_layer_decode(desc, w, xd, lens, k1, v1)
    k2, v2 = kc.copy(), vc.copy()
    parts = oracle.forward_split(
        lambda lo, hi: oracle.decoder_layer_decode(desc, w, np.ascontiguousarray(xd[lo:hi]), lens[lo:hi], k2[lo:hi], v2[lo:hi]), B, k)
    assert np.array_equal(parts, whole) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
    xl = RNG.standard_normal((15, 24)).astype(np.float32); W = RNG.standard_normal((10, 24)).astype(np.float32)
    assert np.array_equal(oracle.forward_split(lambda lo, hi: oracle.linear(xl[lo:hi], W), 15, k), oracle.linear(xl, W))


# ------------------------------------------------------------------ Table 1 / Section 2.1 accounting
def test_accounting_reproduces_table1(golden_dir):
    g = read_golden(os.path.join(golden_dir, "table1_llama13b.txt"))
    H, I, nh = int(g["d_model"]), int(g["d_ff"]), int(g["n_heads"])
    desc = oracle.LayerDesc(H, nh, nh, H // nh, I)
    pp = oracle.projection_params(desc)
    assert oracle.layer_params(desc) == 4 * H * H + 3 * H * I == 317_194_240
    assert round(oracle.layer_params(desc) / 1e6) == int(g["layer_params_millions"])
    mib = lambda n: n * 2 / 2 ** 20
    assert mib(pp["wq"]) == mib(pp["wo"]) == float(g["attn_proj_mib"])
    assert mib(pp["wgate"]) == mib(pp["wdown"]) == float(g["ffn_proj_mib"])
    assert mib(pp["wq"] + pp["wk"] + pp["wv"] + pp["wo"]) == float(g["self_attn_mib"])
    assert mib(oracle.layer_params(desc)) == float(g["decoder_layer_mib"])
    rows = int(g["batch"]) * int(g["seq"])
    gf = lambda f: round(f / 1e9, 2)
    assert gf(oracle.gemm_flops(rows, pp["wq"])) == float(g["attn_proj_gflops"])
    assert gf(oracle.gemm_flops(rows, pp["wup"])) == float(g["ffn_proj_gflops"])
    assert gf(oracle.attention_score_flops(int(g["seq"]), H)) == float(g["attn_score_gflops"])
    attn = 4 * oracle.gemm_flops(rows, pp["wq"]) + oracle.attention_score_flops(int(g["seq"]), H)
    # the paper adds its rounded figures: 4 x 13.42 + 1.34 = 55.02 (the unrounded sum is 55.029)
    assert round(4 * float(g["attn_proj_gflops"]) + float(g["attn_score_gflops"]), 2) == float(g["self_attn_gflops"])
    assert abs(attn / 1e9 - float(g["self_attn_gflops"])) < 0.011
    assert round(float(g["self_attn_gflops"]) / float(g["self_attn_mib"]), 3) == float(g["self_attn_gflops_per_mb"])
    assert round(float(g["ffn_proj_gflops"]) / float(g["ffn_proj_mib"]), 3) == float(g["ffn_gflops_per_mb"])
    # the printed layer figure counts two FFN projections; the true sum counts three
    assert round(float(g["self_attn_gflops"]) + 2 * float(g["ffn_proj_gflops"]), 1) == float(g["decoder_layer_gflops_as_printed"])


# ------------------------------------------------------------------ workload generator sanity
def test_workload_generator_is_seeded_and_storage_exact():
    c = workloads.scaled(workloads.CONFIGS["C2"], hidden=64, n_q_heads=2, n_kv_heads=2, head_dim=32,
                         intermediate=96, n_seqs=3, len_lo=5, len_hi=9)
    w1, w2 = workloads.make_weights(c), workloads.make_weights(c)
    assert all(np.array_equal(w1[k], w2[k]) for k in w1)
    i = workloads.make_inputs(c)
    assert i.k_cache.shape == (3, 2, c.cache_cap, 32) and ((i.lens >= 5) & (i.lens <= 9)).all()
    t = torch.from_numpy(w1["wq"])
    assert torch.equal(t.to(torch.bfloat16).float(), t)         # already bf16-representable
    assert abs(float(np.std(w1["wgate"])) - 0.02) < 0.004 and abs(float(np.mean(w1["g1"])) - 1.0) < 0.02
    n = workloads.bursty_token_counts()
    assert len(n) == 200 and min(n) >= 1 and n == workloads.bursty_token_counts()
    assert [workloads.replicas_for_tokens(v) for v in (1, 127, 128, 511, 512)] == [1, 1, 2, 2, 4]


# ---------------------------------------------------------------- runs of consecutive layers
def _stack_cfg(n_layers=2, **kw):
    base = workloads.scaled(workloads.CONFIGS["C1"], n_q_heads=4, n_kv_heads=2, hidden=64, head_dim=16,
                            intermediate=96, n_layers=n_layers)
    return workloads.scaled(base, **kw)


def _odesc(cfg):
    return oracle.LayerDesc(cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.intermediate,
                            cfg.rms_eps, cfg.rope_base)


def test_stack_is_the_composition_of_its_layers_and_one_layer_is_the_layer():
    """Section 3.1: consecutive layers feed each other, nothing else happens in between."""
    cfg = _stack_cfg(3, n_seqs=3, seq_pad=9, len_lo=2, len_hi=9)
    ws = workloads.make_weights(cfg, 7)
    inp = workloads.make_inputs(cfg, 7)
    d = _odesc(cfg)
    y = oracle.decoder_stack_prefill(d, ws, inp.x, inp.lens)
    z = inp.x
    for w in ws:
        z = oracle.decoder_layer_prefill(d, w, z, inp.lens)
    mask = np.arange(cfg.seq_pad)[None, :] < inp.lens[:, None]
    assert np.array_equal(y[mask], z[mask])
    one = oracle.decoder_stack_prefill(d, ws[:1], inp.x, inp.lens)
    assert np.array_equal(one[mask], oracle.decoder_layer_prefill(d, ws[0], inp.x, inp.lens)[mask])
    # every layer changes the result (none is skipped)
    assert not np.allclose(y[mask], oracle.decoder_stack_prefill(d, ws[:2], inp.x, inp.lens)[mask])


def test_stack_prefill_then_decode_equals_longer_prefill():
    """Each layer of the run keeps its own cache: prefilling S tokens and decoding token S + 1
    through the run gives the last row of prefilling S + 1 tokens."""
    cfg = _stack_cfg(2, n_seqs=2, seq_pad=7, len_lo=7, len_hi=7)
    ws = workloads.make_weights(cfg, 11)
    inp = workloads.make_inputs(cfg, 11)
    d = _odesc(cfg)
    S, B, cap = cfg.seq_pad, cfg.n_seqs, 8
    full = oracle.decoder_stack_prefill(d, ws, inp.x, inp.lens)
    kc = np.zeros((2, B, cfg.n_kv_heads, cap, cfg.head_dim), np.float32)
    vc = np.zeros_like(kc)
    lens_s = np.full(B, S - 1, np.int32)
    oracle.decoder_stack_prefill(d, ws, np.ascontiguousarray(inp.x[:, :S - 1]), lens_s, kc, vc)
    y = oracle.decoder_stack_decode(d, ws, np.ascontiguousarray(inp.x[:, S - 1]), lens_s, kc, vc)
    np.testing.assert_allclose(y, full[:, S - 1], rtol=2e-5, atol=2e-6)
    # layer 1's cache holds keys of layer 0's OUTPUT, not of x: the two layers' caches differ
    assert not np.allclose(kc[0], kc[1])


def test_stack_split_equals_unsplit():
    cfg = _stack_cfg(2, mode="decode", n_seqs=5, seq_pad=1, len_lo=0, len_hi=6)
    ws = workloads.make_weights(cfg, 13)
    inp = workloads.make_inputs(cfg, 13)
    d = _odesc(cfg)
    kc, vc = inp.k_cache.copy(), inp.v_cache.copy()
    y = oracle.decoder_stack_decode(d, ws, inp.x, inp.lens, kc, vc)
    parts = []
    bounds = oracle.split_bounds(cfg.n_seqs, 3)
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        k2 = np.ascontiguousarray(inp.k_cache[:, lo:hi]).copy()
        v2 = np.ascontiguousarray(inp.v_cache[:, lo:hi]).copy()
        parts.append(oracle.decoder_stack_decode(d, ws, inp.x[lo:hi], inp.lens[lo:hi], k2, v2))
        assert np.array_equal(k2, kc[:, lo:hi])
    assert np.array_equal(np.concatenate(parts), y)


# ---------------------------------------------------------------- the layer's two halves
def test_attention_block_then_ffn_block_is_the_layer():
    """Section 3.3, Table 1 treats self-attention and FFN as modules of their own; with their norm
    and residual inside, the layer is the one followed by the other - for prefill and for decode."""
    cfg = _stack_cfg(1, n_seqs=3, seq_pad=8, len_lo=2, len_hi=8)
    w = workloads.make_weights(cfg, 21)
    inp = workloads.make_inputs(cfg, 21)
    d = _odesc(cfg)
    mask = np.arange(cfg.seq_pad)[None, :] < inp.lens[:, None]
    y = oracle.decoder_layer_prefill(d, w, inp.x, inp.lens)
    x1 = oracle.decoder_layer_prefill(d, w, inp.x, inp.lens, attention_only=True)
    y2 = oracle.ffn_block(d, w, x1.reshape(-1, cfg.hidden)).reshape(x1.shape)
    np.testing.assert_allclose(y2[mask], y[mask], rtol=1e-6, atol=1e-6)   # x1 passes through fp32 once
    assert not np.allclose(x1[mask], y[mask])
    dcfg = workloads.scaled(cfg, mode="decode", seq_pad=1, len_lo=0, len_hi=6)
    di = workloads.make_inputs(dcfg, 22)
    yd = oracle.decoder_layer_decode(d, w, di.x, di.lens, di.k_cache.copy(), di.v_cache.copy())
    x1d = oracle.decoder_layer_decode(d, w, di.x, di.lens, di.k_cache.copy(), di.v_cache.copy(), attention_only=True)
    np.testing.assert_allclose(oracle.ffn_block(d, w, x1d), yd, rtol=1e-6, atol=1e-6)


def test_ffn_block_against_library_fp64_and_special_cases():
    cfg = _stack_cfg(1)
    w = workloads.make_weights(cfg, 23)
    d = _odesc(cfg)
    x = np.random.default_rng(5).standard_normal((7, cfg.hidden)).astype(np.float32)
    y = oracle.ffn_block(d, w, x)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    xd = t(x)
    h = xd * torch.rsqrt((xd * xd).mean(-1, keepdim=True) + cfg.rms_eps) * t(w["g2"])
    ref = xd + (F.silu(h @ t(w["wgate"]).T) * (h @ t(w["wup"]).T)) @ t(w["wdown"]).T
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-6, atol=1e-6)
    # silu(0) = 0: a zero gate projection leaves the residual stream untouched, bit for bit
    w0 = dict(w, wgate=np.zeros_like(w["wgate"]))
    assert np.array_equal(oracle.ffn_block(d, w0, x), x)
    # the attention weights are not read
    w1 = dict(w, wq=np.full_like(w["wq"], np.nan), g1=np.full_like(w["g1"], np.nan))
    assert np.array_equal(oracle.ffn_block(d, w1, x), y)


def test_attention_block_special_cases():
    cfg = _stack_cfg(1, n_seqs=2, seq_pad=6, len_lo=6, len_hi=6)
    w = workloads.make_weights(cfg, 24)
    inp = workloads.make_inputs(cfg, 24)
    d = _odesc(cfg)
    # zero output projection: y = x bit for bit; the FFN weights are not read
    w0 = dict(w, wo=np.zeros_like(w["wo"]), wgate=np.full_like(w["wgate"], np.nan), g2=np.full_like(w["g2"], np.nan))
    assert np.array_equal(oracle.decoder_layer_prefill(d, w0, inp.x, inp.lens, attention_only=True), inp.x)
    # first row: one visible key, softmax weight 1 -> x + (v_0 repeated per group) Wo^T
    y = oracle.decoder_layer_prefill(d, w, inp.x, inp.lens, attention_only=True)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x0 = t(inp.x[:, 0])
    h = x0 * torch.rsqrt((x0 * x0).mean(-1, keepdim=True) + cfg.rms_eps) * t(w["g1"])
    v = (h @ t(w["wv"]).T).reshape(cfg.n_seqs, cfg.n_kv_heads, cfg.head_dim)
    a = v.repeat_interleave(cfg.n_q_heads // cfg.n_kv_heads, dim=1).reshape(cfg.n_seqs, -1)
    np.testing.assert_allclose(y[:, 0], (x0 + a @ t(w["wo"]).T).numpy(), rtol=1e-6, atol=1e-6)
