"""CPU oracle of the module-replica hot path: TEST INFRASTRUCTURE, not product code.

Thin numpy/ctypes front of ``cocoserve_oracle.c`` (fp32 arrays in and out, fp64 arithmetic,
nothing rounded between steps) plus the split/gather rule written out in Python.  Only tests,
the smoke check and the benchmark's CPU-baseline leg may import this package; it imports
nothing from the GPU library and the GPU library imports nothing from it.

Paper passages followed: module inventory and dimensions (Section 2.1), module definition
(Section 1, footnote), replication = contiguous batch slices, 15 -> 7 + 8, results collected
in order (Section 3.1 "Replication"), prefill/decode and the KV cache (Section 2.1), Table 1
(weight bytes and FLOPs per module).  Whole-layer outputs at 7B/13B/70B shapes are printed
nowhere: parity unpinned at those sizes except through the pinned pieces.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        _LIB = ctypes.CDLL(path)
        _LIB.orc_omp_threads.restype = ctypes.c_int
    return _LIB


class _Desc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int), ("n_q_heads", ctypes.c_int), ("n_kv_heads", ctypes.c_int),
                ("head_dim", ctypes.c_int), ("intermediate", ctypes.c_int),
                ("rms_eps", ctypes.c_double), ("rope_base", ctypes.c_double)]


class _Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g1", "g2")]


@dataclass
class LayerDesc:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    def c(self):
        return _Desc(self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim,
                     self.intermediate, self.rms_eps, self.rope_base)


WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g1", "g2")


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _weights(desc: LayerDesc, w: dict):
    H, QD, KD, I = desc.hidden, desc.n_q_heads * desc.head_dim, desc.n_kv_heads * desc.head_dim, desc.intermediate
    shapes = {"wq": (QD, H), "wk": (KD, H), "wv": (KD, H), "wo": (H, QD), "wgate": (I, H),
              "wup": (I, H), "wdown": (H, I), "g1": (H,), "g2": (H,)}
    keep = {}
    cw = _Weights()
    for n in WEIGHT_NAMES:
        a = _f32(w[n])
        if a.shape != shapes[n]:
            raise ValueError(f"{n}: shape {a.shape}, expected {shapes[n]}")
        keep[n] = a
        setattr(cw, n, a.ctypes.data)
    return cw, keep


# ---- split / gather (Section 3.1 "Replication") ---------------------------------------------
def split_bounds(n: int, k: int):
    """Slice j of k is [floor(j n / k), floor((j+1) n / k)): 15 over 2 gives 7 then 8."""
    if k < 1 or n < 0:
        raise ValueError("k >= 1 and n >= 0 required")
    out = (ctypes.c_int64 * (k + 1))()
    lib().orc_split_bounds(ctypes.c_int64(n), ctypes.c_int(k), out)
    return [int(v) for v in out]


# ---- pieces ---------------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    x = _f32(x); g = _f32(g)
    T, H = x.shape
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), ctypes.c_double(eps), ctypes.c_int64(T), ctypes.c_int(H), _p(out))
    return out


def linear(x, W):
    """y = x W^T with W [out, in]; the single-projection module."""
    x = _f32(x); W = _f32(W)
    T, K = x.shape
    N, K2 = W.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    y = np.empty((T, N), dtype=np.float32)
    lib().orc_linear_module(_p(x), _p(W), ctypes.c_int64(T), ctypes.c_int(K), ctypes.c_int(N), _p(y))
    return y


def rope(z, pos: int, base: float):
    """Rotate one head vector (fp64 in, fp64 out) to absolute position pos."""
    z = np.array(z, dtype=np.float64, copy=True)
    lib().orc_rope_f64(_p(z), ctypes.c_int(z.shape[0]), ctypes.c_int64(pos), ctypes.c_double(base))
    return z


def attend(q, keys, vals):
    """One query [d] against keys/vals [n, d] (fp64): returns (out [d], probs [n])."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    keys = np.ascontiguousarray(keys, dtype=np.float64)
    vals = np.ascontiguousarray(vals, dtype=np.float64)
    n, d = keys.shape
    out = np.empty(d, dtype=np.float64)
    probs = np.empty(n, dtype=np.float64)
    lib().orc_attend_f64(_p(q), _p(keys), _p(vals), ctypes.c_int64(n), ctypes.c_int(d),
                         ctypes.c_int64(d), _p(out), _p(probs))
    return out, probs


# ---- whole modules --------------------------------------------------------------------------
def decoder_layer_prefill(desc: LayerDesc, w: dict, x, lens, k_cache=None, v_cache=None, attention_only=False):
    """x [B, S, H]; lens [B]; returns y [B, S, H] (padded rows 0).  Optional caches
    [B, n_kv, cap, d] are filled for positions < lens[b].  attention_only: stop after the
    attention block (y = x + attention output projection)."""
    x = _f32(x)
    B, S, H = x.shape
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    cw, keep = _weights(desc, w)
    y = np.empty_like(x)
    cap = 0
    kp = vp = None
    if k_cache is not None:
        assert k_cache.dtype == np.float32 and v_cache.dtype == np.float32
        assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
        cap = k_cache.shape[2]
        kp, vp = _p(k_cache), _p(v_cache)
    d = desc.c()
    fn = lib().orc_attention_block_prefill if attention_only else lib().orc_decoder_layer_prefill
    rc = fn(ctypes.byref(d), ctypes.byref(cw), _p(x), _p(lens), ctypes.c_int(B), ctypes.c_int(S), _p(y), kp, vp,
            ctypes.c_int(cap))
    if rc != 0:
        raise ValueError("oracle rejected the prefill arguments")
    return y


def decoder_layer_decode(desc: LayerDesc, w: dict, x, lens, k_cache, v_cache, attention_only=False):
    """x [B, H]; lens [B] cached lengths; caches [B, n_kv, cap, d] fp32 updated IN PLACE at
    slot lens[b]; returns y [B, H].  attention_only: stop after the attention block."""
    x = _f32(x)
    B, H = x.shape
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    assert k_cache.dtype == np.float32 and v_cache.dtype == np.float32
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    cap = k_cache.shape[2]
    cw, keep = _weights(desc, w)
    y = np.empty_like(x)
    d = desc.c()
    fn = lib().orc_attention_block_decode if attention_only else lib().orc_decoder_layer_decode
    rc = fn(ctypes.byref(d), ctypes.byref(cw), _p(x), _p(lens), ctypes.c_int(B), _p(k_cache), _p(v_cache),
            ctypes.c_int(cap), _p(y))
    if rc != 0:
        raise ValueError("oracle rejected the decode arguments")
    return y


def ffn_block(desc: LayerDesc, w: dict, x):
    """x [T, H] independent rows: y = x + (silu(h Wg^T) * (h Wu^T)) Wd^T with h = RMSNorm(x; g2)."""
    x = _f32(x)
    T, H = x.shape
    cw, keep = _weights(desc, w)
    y = np.empty_like(x)
    d = desc.c()
    lib().orc_ffn_block(ctypes.byref(d), ctypes.byref(cw), _p(x), ctypes.c_int64(T), _p(y))
    return y


def decoder_stack_prefill(desc: LayerDesc, layers, x, lens, k_caches=None, v_caches=None):
    """A run of consecutive decoder layers (Section 3.1): layer l's output is layer l + 1's
    input.  layers: list of weight dicts; optional caches [L, B, n_kv, cap, d], one per layer."""
    y = _f32(x)
    for l, w in enumerate(layers):
        kc = None if k_caches is None else k_caches[l]
        vc = None if v_caches is None else v_caches[l]
        y = decoder_layer_prefill(desc, w, y, lens, kc, vc)
    return y


def decoder_stack_decode(desc: LayerDesc, layers, x, lens, k_caches, v_caches):
    """One decode step through a run of layers; caches [L, B, n_kv, cap, d] updated in place
    (every layer appends its own key / value at slot lens[b])."""
    y = _f32(x)
    for l, w in enumerate(layers):
        y = decoder_layer_decode(desc, w, y, lens, k_caches[l], v_caches[l])
    return y


def forward_split(forward_slice, n: int, k: int):
    """The replicated forward as the paper states it: cut [0, n) into k contiguous slices,
    run the unmodified module on each, put the outputs back in order.
    forward_slice(lo, hi) -> array of hi - lo leading rows (may be empty)."""
    b = split_bounds(n, k)
    parts = [forward_slice(b[j], b[j + 1]) for j in range(k) if b[j + 1] > b[j]]
    return np.concatenate(parts, axis=0)


def omp_threads() -> int:
    return int(lib().orc_omp_threads())


# ---- size and FLOP accounting (Section 2.1 parameter count; Table 1) ------------------------
def projection_params(desc: LayerDesc):
    H, QD, KD, I = desc.hidden, desc.n_q_heads * desc.head_dim, desc.n_kv_heads * desc.head_dim, desc.intermediate
    return {"wq": QD * H, "wk": KD * H, "wv": KD * H, "wo": H * QD,
            "wgate": I * H, "wup": I * H, "wdown": H * I}


def layer_params(desc: LayerDesc) -> int:
    """Projection parameters of one decoder layer (norm gains excluded, as the paper's 317 M)."""
    return sum(projection_params(desc).values())


def gemm_flops(rows: int, n_params: int) -> int:
    return 2 * rows * n_params


def attention_score_flops(seq: int, hidden: int) -> int:
    """QK^T and PV over a full seq x seq score matrix, all heads: 4 seq^2 hidden."""
    return 4 * seq * seq * hidden
