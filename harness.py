"""Glue shared by the GPU parity tests, smoke() and bench.py: run a workloads.Config through the
HIP library (via the C ABI binding) and, for the comparison legs only, through the CPU oracle.

The oracle is test infrastructure: it is imported inside the two functions that call it
(`oracle_forward`, `oracle_desc`), never at module load, so a process that only runs the GPU
path does not load it."""
import numpy as np
import torch

import workloads
from paper_2507_18006_amd import binding as B

DEV = "cuda:0"


def module_desc(cfg: workloads.Config) -> B.ModuleDesc:
    dt = B.CCS_BF16 if cfg.dtype == "bf16" else B.CCS_F32
    if cfg.kind == "linear":
        return B.ModuleDesc(kind=B.CCS_LINEAR, dtype=dt, in_features=cfg.in_features, out_features=cfg.out_features)
    kind = {"decoder_layer": B.CCS_DECODER_LAYER, "attn_block": B.CCS_ATTN_BLOCK, "ffn_block": B.CCS_FFN_BLOCK}[cfg.kind]
    return B.ModuleDesc(kind=kind, dtype=dt, hidden=cfg.hidden, n_q_heads=cfg.n_q_heads,
                        n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, intermediate=cfg.intermediate,
                        rms_eps=cfg.rms_eps, rope_base=cfg.rope_base, n_layers=cfg.n_layers)


def oracle_desc(cfg: workloads.Config):
    import oracle
    return oracle.LayerDesc(cfg.hidden, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.intermediate,
                            cfg.rms_eps, cfg.rope_base)


def tdtype(cfg):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def to_dev(a: np.ndarray, cfg):
    """Storage-exact upload (the generator already rounded bf16 configs)."""
    return torch.from_numpy(a).to(DEV).to(tdtype(cfg)).contiguous()


def make_module(cfg, weights=None, seed=0, max_seqs=None, max_seq_pad=None, max_cap=None) -> B.Module:
    w = workloads.make_weights(cfg, seed) if weights is None else weights
    wd = [{k: to_dev(v, cfg) for k, v in wl.items()} for wl in w] if isinstance(w, list) else {k: to_dev(v, cfg) for k, v in w.items()}
    decode = cfg.mode == "decode"
    m = B.Module(module_desc(cfg), wd,
                 max_seqs=cfg.n_seqs if max_seqs is None else max_seqs,
                 max_seq_pad=(cfg.seq_pad if cfg.mode == "prefill" else 1) if max_seq_pad is None else max_seq_pad,
                 max_cache_cap=(cfg.cache_cap if decode else 0) if max_cap is None else max_cap, device=DEV)
    return m


class DeviceBatch:
    """Device copies of one workloads.Inputs + the ccs_batch that points at them."""

    def __init__(self, m: B.Module, cfg, inp: workloads.Inputs, with_cache=None):
        self.cfg = cfg
        self.x = to_dev(inp.x, cfg)
        mode = {"prefill": B.CCS_PREFILL, "decode": B.CCS_DECODE, "linear": B.CCS_ROWS}[cfg.mode]
        if cfg.kind in ("linear", "ffn_block"):
            out = cfg.out_features if cfg.kind == "linear" else cfg.hidden
            self.y = torch.zeros((inp.x.shape[0], out), dtype=tdtype(cfg), device=DEV)
            self.batch = m.batch(B.CCS_ROWS, self.x, self.y)
            return
        self.y = torch.zeros_like(self.x)
        self.lens_host = torch.from_numpy(np.ascontiguousarray(inp.lens, dtype=np.int32))
        self.lens_dev = self.lens_host.to(DEV)
        self.k = self.v = None
        if inp.k_cache is not None:
            self.k, self.v = to_dev(inp.k_cache, cfg), to_dev(inp.v_cache, cfg)
        elif with_cache:
            shape = (inp.x.shape[0], cfg.n_kv_heads, with_cache, cfg.head_dim)
            if cfg.n_layers > 1:
                shape = (cfg.n_layers,) + shape
            self.k = torch.zeros(shape, dtype=tdtype(cfg), device=DEV)
            self.v = torch.zeros(shape, dtype=tdtype(cfg), device=DEV)
        self.batch = m.batch(mode, self.x, self.y, self.lens_host, self.lens_dev, self.k, self.v,
                             seq_pad=cfg.seq_pad if cfg.mode == "prefill" else 1)

    def out(self) -> np.ndarray:
        torch.cuda.synchronize()
        return self.y.float().cpu().numpy()


def gpu_forward(cfg, k: int, seed: int = 0, weights=None, inputs=None, return_caches=False):
    """forward_split at k replicas through the C ABI; returns y as fp32 numpy."""
    m = make_module(cfg, weights, seed)
    try:
        m.replicate(k)
        inp = workloads.make_inputs(cfg, seed) if inputs is None else inputs
        db = DeviceBatch(m, cfg, inp)
        m.forward_split(db.batch)
        m.sync()
        y = db.out()
        if return_caches:
            return y, db.k.float().cpu().numpy(), db.v.float().cpu().numpy()
        return y
    finally:
        m.destroy()


def oracle_forward(cfg, seed: int = 0, weights=None, inputs=None, seqs=None, return_caches=False):
    """The oracle on the same seeded inputs; `seqs` restricts it to some sequences / rows."""
    import oracle
    w = workloads.make_weights(cfg, seed) if weights is None else weights
    inp = workloads.make_inputs(cfg, seed) if inputs is None else inputs
    sel = slice(None) if seqs is None else seqs
    if cfg.kind == "linear":
        return oracle.linear(inp.x[sel], w["w"])
    d = oracle_desc(cfg)
    if cfg.kind == "ffn_block":
        return oracle.ffn_block(d, w, inp.x[sel])
    ao = cfg.kind == "attn_block"
    if cfg.n_layers > 1:   # a run of layers; caches [L, B, ...]
        if cfg.mode == "prefill":
            return oracle.decoder_stack_prefill(d, w, np.ascontiguousarray(inp.x[sel]), inp.lens[sel])
        kc = np.ascontiguousarray(inp.k_cache[:, sel]).copy()
        vc = np.ascontiguousarray(inp.v_cache[:, sel]).copy()
        y = oracle.decoder_stack_decode(d, w, np.ascontiguousarray(inp.x[sel]), inp.lens[sel], kc, vc)
        return (y, kc, vc) if return_caches else y
    if cfg.mode == "prefill":
        return oracle.decoder_layer_prefill(d, w, np.ascontiguousarray(inp.x[sel]), inp.lens[sel], attention_only=ao)
    kc = np.ascontiguousarray(inp.k_cache[sel]).copy()
    vc = np.ascontiguousarray(inp.v_cache[sel]).copy()
    y = oracle.decoder_layer_decode(d, w, np.ascontiguousarray(inp.x[sel]), inp.lens[sel], kc, vc, attention_only=ao)
    return (y, kc, vc) if return_caches else y


def valid_mask(cfg, lens, n_seqs=None):
    """Boolean [B, S] of rows that are part of the result (prefill: t < len)."""
    B_ = len(lens)
    return np.arange(cfg.seq_pad)[None, :] < np.asarray(lens)[:, None]


def l2_err(y, ref, mask=None) -> float:
    """||y - ref||_2 / ||ref||_2 over the rows that count (reported beside the max-error bar)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if mask is not None:
        y, ref = y[mask], ref[mask]
    if ref.size == 0:
        return 0.0
    if not np.isfinite(y).all():
        return float("inf")
    n = np.linalg.norm(ref.ravel())
    return float(np.linalg.norm((y - ref).ravel()) / n) if n > 0 else 0.0


def row_rel_err(y, ref, mask=None) -> float:
    """max over rows of max_c |y - ref| / max_c |ref|: every token row (decode: every sequence) is
    held to the bar by its own magnitude, so a row whose result is small is not hidden behind a
    large one elsewhere in the batch."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if mask is not None:
        y, ref = y[mask], ref[mask]
    y, ref = y.reshape(-1, y.shape[-1]), ref.reshape(-1, ref.shape[-1])
    if ref.size == 0:
        return 0.0
    if not np.isfinite(y).all():
        return float("inf")
    den = np.abs(ref).max(axis=1)
    num = np.abs(y - ref).max(axis=1)
    ok = den > 0
    if (num[~ok] > 0).any():
        return float("inf")
    return float((num[ok] / den[ok]).max()) if ok.any() else 0.0


def rel_err(y, ref, mask=None) -> float:
    """max |y - ref| / max |ref| over the rows that count (the parity bar of the build)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if mask is not None:
        y, ref = y[mask], ref[mask]
    if ref.size == 0:
        return 0.0
    if not np.isfinite(y).all():
        return float("inf")
    return float(np.abs(y - ref).max() / np.abs(ref).max())
