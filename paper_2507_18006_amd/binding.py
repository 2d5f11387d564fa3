"""ctypes binding of libcocoserve_mi.so: same names as the C ABI, marshalling only.

PyTorch is used for what the library leaves to the caller: device allocations (weight arenas,
workspaces, activations, KV caches) and HIP streams.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libcocoserve_mi.so"

CCS_OK, CCS_EINVAL, CCS_ESTATE, CCS_ENOMEM, CCS_EUNSUPPORTED, CCS_EHIP = 0, -1, -2, -3, -4, -5
CCS_DECODER_LAYER, CCS_LINEAR, CCS_ATTN_BLOCK, CCS_FFN_BLOCK = 0, 1, 2, 3
CCS_F32, CCS_BF16 = 0, 1
CCS_PREFILL, CCS_DECODE, CCS_ROWS = 0, 1, 2
CCS_MAX_REPLICAS = 16
STAGES = ("rmsnorm1", "gemm_qkv", "gemm_qkv_reduce", "rope", "attn", "attn_combine", "gemm_o",
          "gemm_o_reduce", "rmsnorm2", "gemm_gu", "gemm_gu_reduce", "gemm_down", "gemm_down_reduce",
          "pack_x", "clone", "compact", "expand")
CCS_N_STAGES = len(STAGES)
_STATUS = {0: "CCS_OK", -1: "CCS_EINVAL", -2: "CCS_ESTATE", -3: "CCS_ENOMEM",
           -4: "CCS_EUNSUPPORTED", -5: "CCS_EHIP"}

EXPORTS = (
    "ccs_module_arena_bytes", "ccs_module_workspace_bytes", "ccs_module_create",
    "ccs_module_replicate", "ccs_module_replicas", "ccs_module_forward", "ccs_module_forward_static",
    "ccs_static_workspace_bytes", "ccs_module_forward_split", "ccs_module_forward_shares", "ccs_module_copy", "ccs_module_migrate", "ccs_cache_copy",
    "ccs_module_arena", "ccs_module_profile", "ccs_module_profile_read", "ccs_module_sync", "ccs_module_destroy", "ccs_last_error", "ccs_version",
    "ccs_speedup_homo", "ccs_speedup", "ccs_plan_scale_up", "ccs_shares_from_capacity",
)


class CcsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


class ccs_module_desc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("hidden", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("intermediate", ctypes.c_int32),
                ("in_features", ctypes.c_int32), ("out_features", ctypes.c_int32),
                ("rms_eps", ctypes.c_float), ("rope_base", ctypes.c_float),
                ("n_layers", ctypes.c_int32)]


class ccs_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g1", "g2", "w")]


class ccs_batch(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("n_seqs", ctypes.c_int32), ("seq_pad", ctypes.c_int32),
                ("x", ctypes.c_void_p), ("y", ctypes.c_void_p),
                ("lens_host", ctypes.c_void_p), ("lens_dev", ctypes.c_void_p),
                ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("cache_cap", ctypes.c_int32), ("cache_layer_stride", ctypes.c_int64)]


_lib = None


def lib_path() -> str:
    return os.path.join(HERE, _LIB_NAME)


def lib():
    """Load the HIP library; there is no fallback when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(hipcc --offload-arch=gfx950); there is no CPU fallback")
    L = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    L.ccs_module_arena_bytes.restype = sz
    L.ccs_module_arena_bytes.argtypes = [ctypes.POINTER(ccs_module_desc)]
    L.ccs_module_workspace_bytes.restype = sz
    L.ccs_module_workspace_bytes.argtypes = [ctypes.POINTER(ccs_module_desc), i32, i32, i32]
    L.ccs_module_create.argtypes = [ctypes.POINTER(ccs_module_desc), ctypes.POINTER(ccs_weights), vp, vp, sz, vp,
                                    ctypes.POINTER(vp)]
    L.ccs_module_replicate.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), sz, ctypes.POINTER(vp)]
    L.ccs_module_replicas.argtypes = [vp]
    L.ccs_module_forward.argtypes = [vp, i32, ctypes.POINTER(ccs_batch)]
    L.ccs_module_forward_static.argtypes = [vp, i32, ctypes.POINTER(ccs_batch)]
    L.ccs_module_forward_static.restype = ctypes.c_int
    L.ccs_static_workspace_bytes.restype = sz
    L.ccs_static_workspace_bytes.argtypes = []
    L.ccs_module_forward_split.argtypes = [vp, ctypes.POINTER(ccs_batch), vp]
    L.ccs_module_forward_shares.argtypes = [vp, ctypes.POINTER(ccs_batch), ctypes.POINTER(i32), vp]
    L.ccs_module_copy.argtypes = [vp, i32, vp, vp]
    L.ccs_module_migrate.argtypes = [vp, i32, vp, vp]
    L.ccs_cache_copy.argtypes = [vp, vp, sz, vp]
    L.ccs_module_arena.argtypes = [vp, i32, ctypes.POINTER(vp)]
    L.ccs_module_profile.argtypes = [vp, ctypes.c_uint32]
    L.ccs_module_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double),
                                          ctypes.POINTER(ctypes.c_int64), i32]
    L.ccs_module_sync.argtypes = [vp]
    L.ccs_module_destroy.argtypes = [vp]
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)
    L.ccs_speedup_homo.restype = ctypes.c_double
    L.ccs_speedup_homo.argtypes = [ip, i32, ctypes.c_double]
    L.ccs_speedup.restype = ctypes.c_double
    L.ccs_speedup.argtypes = [ip, i32, dp, dp, dp, ctypes.c_double, ctypes.c_double, ctypes.c_double]
    L.ccs_plan_scale_up.restype = ctypes.c_int
    L.ccs_plan_scale_up.argtypes = [ip, i32, ctypes.c_double, ctypes.POINTER(ctypes.c_int64), i32, ctypes.c_int64,
                                    ctypes.POINTER(ctypes.c_uint8), ip, ctypes.POINTER(ctypes.c_uint8), dp]
    L.ccs_shares_from_capacity.restype = ctypes.c_int
    L.ccs_shares_from_capacity.argtypes = [ctypes.c_int64, i32, dp, ip]
    L.ccs_last_error.restype = ctypes.c_char_p
    L.ccs_version.restype = ctypes.c_char_p
    for name in ("ccs_module_create", "ccs_module_replicate", "ccs_module_replicas", "ccs_module_forward",
                 "ccs_module_forward_split", "ccs_module_forward_shares", "ccs_module_copy", "ccs_module_migrate", "ccs_cache_copy",
                 "ccs_module_arena", "ccs_module_profile", "ccs_module_profile_read", "ccs_module_sync", "ccs_module_destroy"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def _check(rc: int):
    if rc < 0:
        raise CcsError(rc, lib().ccs_last_error().decode())
    return rc


@dataclass
class ModuleDesc:
    kind: int = CCS_DECODER_LAYER
    dtype: int = CCS_BF16
    hidden: int = 0
    n_q_heads: int = 0
    n_kv_heads: int = 0
    head_dim: int = 0
    intermediate: int = 0
    in_features: int = 0
    out_features: int = 0
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    n_layers: int = 1

    def c(self) -> ccs_module_desc:
        return ccs_module_desc(self.kind, self.dtype, self.hidden, self.n_q_heads, self.n_kv_heads,
                               self.head_dim, self.intermediate, self.in_features, self.out_features,
                               self.rms_eps, self.rope_base, self.n_layers)


def module_arena_bytes(desc: ModuleDesc) -> int:
    d = desc.c()
    return int(lib().ccs_module_arena_bytes(ctypes.byref(d)))


def module_workspace_bytes(desc: ModuleDesc, max_seqs: int, max_seq_pad: int = 1, max_cache_cap: int = 0) -> int:
    d = desc.c()
    return int(lib().ccs_module_workspace_bytes(ctypes.byref(d), max_seqs, max_seq_pad, max_cache_cap))


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _vp_array(items):
    arr = (ctypes.c_void_p * len(items))()
    for i, v in enumerate(items):
        arr[i] = v
    return arr


class Module:
    """One module (decoder layer or projection) with k >= 1 instances on one GPU.

    Holds the torch allocations the C ABI expects the caller to own (arenas, workspaces,
    streams) and forwards every operation to the library."""

    def __init__(self, desc: ModuleDesc, weights: dict, max_seqs: int, max_seq_pad: int = 1,
                 max_cache_cap: int = 0, device: str = "cuda:0"):
        import torch
        self._torch = torch
        self.desc = desc
        self.device = torch.device(device)
        self.L = lib()
        self.arena_bytes = module_arena_bytes(desc)
        self.ws_bytes = module_workspace_bytes(desc, max_seqs, max_seq_pad, max_cache_cap)
        if self.arena_bytes == 0 or self.ws_bytes == 0:
            raise CcsError(CCS_EINVAL, self.L.ccs_last_error().decode())
        self.torch_dtype = torch.bfloat16 if desc.dtype == CCS_BF16 else torch.float32
        self.arenas = [self._alloc(self.arena_bytes)]
        self.workspaces = [self._alloc(self.ws_bytes)]
        # replica 0 lives on the stream that is current at creation: a replicated forward issued
        # from that stream then needs no fork/join events for it (and none at all at k = 1)
        self.streams = [torch.cuda.current_stream(self.device)]
        # one dict of tensors, or a list of them for a run of n_layers decoder layers
        layers = list(weights) if isinstance(weights, (list, tuple)) else [weights]
        if len(layers) != max(1, desc.n_layers):
            raise ValueError(f"need the weights of {max(1, desc.n_layers)} layers, got {len(layers)}")
        cw = (ccs_weights * len(layers))()
        for l, wl in enumerate(layers):
            for name, t in wl.items():
                if t.dtype != self.torch_dtype or not t.is_cuda or not t.is_contiguous():
                    raise ValueError(f"weight {name}: need a contiguous {self.torch_dtype} CUDA tensor")
                setattr(cw[l], name, t.data_ptr())
        d = desc.c()
        h = ctypes.c_void_p()
        _check(self.L.ccs_module_create(ctypes.byref(d), cw, self.arenas[0].data_ptr(),
                                        self.workspaces[0].data_ptr(), self.ws_bytes,
                                        self.streams[0].cuda_stream, ctypes.byref(h)))
        self.handle = h
        self.streams[0].synchronize()   # caller's weight tensors may now be dropped

    def _alloc(self, nbytes: int):
        return self._torch.empty(max(nbytes, 256), dtype=self._torch.uint8, device=self.device)

    # -- module_replicate(k) ------------------------------------------------------------------
    def replicate(self, k: int):
        torch = self._torch
        cur = self.replicas()
        if k > CCS_MAX_REPLICAS or k < 1:
            _check(self.L.ccs_module_replicate(self.handle, k, None, None, 0, None))
        while len(self.arenas) < k:
            self.arenas.append(self._alloc(self.arena_bytes))
            self.workspaces.append(self._alloc(self.ws_bytes))
            self.streams.append(torch.cuda.Stream(device=self.device))
        a = _vp_array([t.data_ptr() for t in self.arenas[:k]])
        w = _vp_array([t.data_ptr() for t in self.workspaces[:k]])
        s = _vp_array([st.cuda_stream for st in self.streams[:k]])
        _check(self.L.ccs_module_replicate(self.handle, k, a, w, self.ws_bytes, s))
        if k < cur:
            del self.arenas[k:], self.workspaces[k:], self.streams[k:]

    def replicas(self) -> int:
        return _check(self.L.ccs_module_replicas(self.handle))

    # -- batches --------------------------------------------------------------------------------
    def batch(self, mode: int, x, y, lens_host=None, lens_dev=None, k_cache=None, v_cache=None,
              seq_pad: int = 1):
        """Marshal tensors into a ccs_batch.  x: prefill [B,S,H] / decode [B,H] / rows [T,in];
        caches [B, n_kv, cap, d], or [n_layers, B, n_kv, cap, d] for a run of layers."""
        n_seqs = x.shape[0]
        cap, stride = 0, 0
        if k_cache is not None:
            cap = k_cache.shape[-2]
            if k_cache.dim() == 5:
                stride = k_cache.stride(0) * k_cache.element_size()
        b = ccs_batch(mode, n_seqs, seq_pad, _ptr(x), _ptr(y),
                      None if lens_host is None else lens_host.data_ptr(), _ptr(lens_dev),
                      _ptr(k_cache), _ptr(v_cache), cap, stride)
        b._keep = (x, y, lens_host, lens_dev, k_cache, v_cache)
        return b

    def forward(self, replica: int, batch: ccs_batch):
        _check(self.L.ccs_module_forward(self.handle, replica, ctypes.byref(batch)))

    def forward_static(self, replica: int, batch: ccs_batch):
        """forward() in the library's built-in workspace: no allocation, no caller workspace."""
        _check(self.L.ccs_module_forward_static(self.handle, replica, ctypes.byref(batch)))

    def forward_split(self, batch: ccs_batch, stream=None):
        s = self._torch.cuda.current_stream(self.device) if stream is None else stream
        _check(self.L.ccs_module_forward_split(self.handle, ctypes.byref(batch), s.cuda_stream))

    def forward_shares(self, batch: ccs_batch, counts, stream=None):
        """Uneven replicated forward: slice j is the next counts[j] sequences."""
        s = self._torch.cuda.current_stream(self.device) if stream is None else stream
        c = (ctypes.c_int32 * len(counts))(*[int(v) for v in counts])
        if len(counts) != self.replicas():
            raise ValueError("one count per replica")
        _check(self.L.ccs_module_forward_shares(self.handle, ctypes.byref(batch), c, s.cuda_stream))

    # -- module_copy / module_migrate -----------------------------------------------------------
    def copy(self, replica: int, stream=None):
        """Clone a replica's weights into a fresh arena (returned)."""
        s = self._torch.cuda.current_stream(self.device) if stream is None else stream
        dst = self._alloc(self.arena_bytes)
        _check(self.L.ccs_module_copy(self.handle, replica, dst.data_ptr(), s.cuda_stream))
        return dst

    def copy_into(self, replica: int, dst, stream=None):
        s = self._torch.cuda.current_stream(self.device) if stream is None else stream
        _check(self.L.ccs_module_copy(self.handle, replica, dst.data_ptr(), s.cuda_stream))

    def migrate(self, replica: int, stream=None):
        """Move a replica's weights to a fresh arena; the old arena is released after the copy."""
        s = self._torch.cuda.current_stream(self.device) if stream is None else stream
        dst = self._alloc(self.arena_bytes)
        _check(self.L.ccs_module_migrate(self.handle, replica, dst.data_ptr(), s.cuda_stream))
        s.synchronize()
        old = self.arenas[replica]
        self.arenas[replica] = dst
        return old

    def arena_ptr(self, replica: int) -> int:
        p = ctypes.c_void_p()
        _check(self.L.ccs_module_arena(self.handle, replica, ctypes.byref(p)))
        return int(p.value)

    # -- per-kernel timing ------------------------------------------------------------------------
    def profile(self, stages=None):
        """Time the named stages (None: all; empty: off) with HIP events on the replica streams."""
        if stages is None:
            mask = (1 << CCS_N_STAGES) - 1
        else:
            mask = 0
            for s in stages:
                mask |= 1 << STAGES.index(s)
        _check(self.L.ccs_module_profile(self.handle, mask))

    def profile_read(self, replica: int = 0, reset: bool = True) -> dict:
        """{stage: (total_ms, launches)} for the stages that ran."""
        ms = (ctypes.c_double * CCS_N_STAGES)()
        cnt = (ctypes.c_int64 * CCS_N_STAGES)()
        _check(self.L.ccs_module_profile_read(self.handle, replica, ms, cnt, 1 if reset else 0))
        return {STAGES[i]: (float(ms[i]), int(cnt[i])) for i in range(CCS_N_STAGES) if cnt[i]}

    def sync(self):
        _check(self.L.ccs_module_sync(self.handle))

    def destroy(self):
        if getattr(self, "handle", None):
            _check(self.L.ccs_module_destroy(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def cache_copy(dst, src, stream=None):
    """Streaming device-to-device copy of a KV cache (same byte size, no overlap)."""
    import torch
    s = torch.cuda.current_stream(dst.device) if stream is None else stream
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(lib().ccs_cache_copy(dst.data_ptr(), src.data_ptr(), nbytes, s.cuda_stream))


# -- scale-up planning (host only) -----------------------------------------------------------------
def speedup_homo(p, gamma: float) -> float:
    a = (ctypes.c_int32 * len(p))(*[int(v) for v in p])
    return lib().ccs_speedup_homo(a, len(p), float(gamma))


def speedup(p, bs, capacity, bandwidth, d: float, l: float, delta: float) -> float:
    """bs, capacity, bandwidth: one list per layer with p[i] entries (instance 0 = the original)."""
    a = (ctypes.c_int32 * len(p))(*[int(v) for v in p])
    flat = lambda rows: (ctypes.c_double * sum(len(r) for r in rows))(*[float(v) for r in rows for v in r])
    return lib().ccs_speedup(a, len(p), flat(bs), flat(capacity), flat(bandwidth), float(d), float(l), float(delta))


def shares_from_capacity(n: int, capacity):
    """Integer shares of n sequences / rows over the instances, minimising max_j share_j / capacity_j."""
    k = len(capacity)
    c = (ctypes.c_double * max(k, 1))(*[float(v) for v in capacity])
    out = (ctypes.c_int32 * max(k, 1))()
    rc = lib().ccs_shares_from_capacity(int(n), k, c, out)
    if rc < 0:
        raise CcsError(rc, "ccs_shares_from_capacity: bad arguments")
    return list(out)[:k]


def plan_scale_up(p, gamma: float, node_available, replica_size: int, placed=None):
    """Algorithm 1: returns (p_new, placed[node][layer], speedup)."""
    n, g = len(p), len(node_available)
    a = (ctypes.c_int32 * n)(*[int(v) for v in p])
    av = (ctypes.c_int64 * max(g, 1))(*[int(v) for v in node_available])
    pin = None
    if placed is not None:
        pin = (ctypes.c_uint8 * (g * n))(*[1 if v else 0 for row in placed for v in row])
    out = (ctypes.c_int32 * n)()
    pout = (ctypes.c_uint8 * max(g * n, 1))()
    sp = ctypes.c_double()
    _check(lib().ccs_plan_scale_up(a, n, float(gamma), av, g, int(replica_size), pin, out, pout, ctypes.byref(sp)))
    return list(out), [[int(pout[i * n + j]) for j in range(n)] for i in range(g)], sp.value
