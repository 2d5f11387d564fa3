"""Host-only checks of the C ABI: the library loads, exports what include/cocoserve_mi.h
declares, and its size accounting agrees with the paper's Table 1.  No GPU compute."""
import ctypes
import os
import re

import pytest

from tests.conftest import ROOT, read_golden
from paper_2507_18006_amd import binding as B


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cocoserve_mi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ccs_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = B.lib()
    syms = declared_symbols()
    assert len(syms) >= 14
    for s in syms:
        assert hasattr(L, s), f"{s} declared in the header but not exported"
    assert sorted(B.EXPORTS) == syms
    assert b"gfx950" in L.ccs_version()


def test_arena_bytes_match_table1_weight_bytes(golden_dir):
    g = read_golden(os.path.join(golden_dir, "table1_llama13b.txt"))
    H, I, nh = int(g["d_model"]), int(g["d_ff"]), int(g["n_heads"])
    d = B.ModuleDesc(hidden=H, n_q_heads=nh, n_kv_heads=nh, head_dim=H // nh, intermediate=I)
    arena = B.module_arena_bytes(d)
    weights = int(float(g["decoder_layer_mib"]) * 2 ** 20)
    gains = 2 * H * 2
    assert weights + gains <= arena <= weights + gains + 6 * 256      # + alignment padding only
    lin = B.ModuleDesc(kind=B.CCS_LINEAR, in_features=I, out_features=H)
    assert B.module_arena_bytes(lin) == int(float(g["ffn_proj_mib"]) * 2 ** 20)
    # the layer's halves: self-attention 200 MiB, FFN 3 x 135 MiB (Table 1), + one gain vector each
    att = B.module_arena_bytes(B.ModuleDesc(kind=B.CCS_ATTN_BLOCK, hidden=H, n_q_heads=nh, n_kv_heads=nh,
                                            head_dim=H // nh, intermediate=I))
    ffn = B.module_arena_bytes(B.ModuleDesc(kind=B.CCS_FFN_BLOCK, hidden=H, n_q_heads=nh, n_kv_heads=nh,
                                            head_dim=H // nh, intermediate=I))
    mib = 2 ** 20
    assert int(float(g["self_attn_mib"])) * mib + H * 2 <= att <= int(float(g["self_attn_mib"])) * mib + H * 2 + 4 * 256
    assert 3 * int(float(g["ffn_proj_mib"])) * mib + H * 2 <= ffn <= 3 * int(float(g["ffn_proj_mib"])) * mib + H * 2 + 3 * 256
    assert att + ffn == arena
    # a run of layers is that many layer arenas back to back
    run = B.ModuleDesc(hidden=H, n_q_heads=nh, n_kv_heads=nh, head_dim=H // nh, intermediate=I, n_layers=3)
    assert B.module_arena_bytes(run) == 3 * arena


def test_arena_of_a_run_grows_like_table2_memory(golden_dir):
    """Table 2: every further replicated LLaMA-13B layer takes 608 of the table's MB (the slope is
    the same between all printed rows); a layer's weights are 605 MiB (Table 1), so the table's MB
    are MiB and a layer carries about 3 MiB beside its weights.  The library's replica memory
    per layer (the arena) must sit between the two figures."""
    g = read_golden(os.path.join(golden_dir, "table2_scaling_cost.txt"))
    t1 = read_golden(os.path.join(golden_dir, "table1_llama13b.txt"))
    n = [int(v) for v in g["layers"].split()]
    mem = [int(v) for v in g["replication_memory_mb"].split()]
    slopes = {(mem[i + 1] - mem[i]) // (n[i + 1] - n[i]) for i in range(len(n) - 1)}
    assert all((mem[i + 1] - mem[i]) % (n[i + 1] - n[i]) == 0 for i in range(len(n) - 1))
    assert slopes == {608}
    H, I, nh = int(t1["d_model"]), int(t1["d_ff"]), int(t1["n_heads"])
    mib = 2 ** 20
    for layers in n:
        d = B.ModuleDesc(hidden=H, n_q_heads=nh, n_kv_heads=nh, head_dim=H // nh, intermediate=I, n_layers=layers)
        per_layer = B.module_arena_bytes(d) / layers / mib
        assert int(t1["decoder_layer_mib"]) <= per_layer <= 608


def test_bad_descs_are_rejected_without_a_gpu():
    bad = B.ModuleDesc(hidden=4096, n_q_heads=32, n_kv_heads=5, head_dim=128, intermediate=11008)
    assert B.module_arena_bytes(bad) == 0 and b"n_kv" in B.lib().ccs_last_error()
    odd = B.ModuleDesc(hidden=4100, n_q_heads=32, n_kv_heads=32, head_dim=128, intermediate=11008)
    assert B.module_arena_bytes(odd) == 0 and b"multiples of 32" in B.lib().ccs_last_error()
    f32 = B.ModuleDesc(dtype=B.CCS_F32, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, intermediate=688)
    assert B.module_arena_bytes(f32) >= 4 * (4 * 256 * 256 + 3 * 256 * 688 + 512)
    assert B.module_workspace_bytes(f32, 4, 32, 0) > 0
    assert B.module_workspace_bytes(f32, -1, 1, 0) == 0


def test_null_handles_return_einval():
    L = B.lib()
    assert L.ccs_module_replicas(None) == B.CCS_EINVAL
    assert L.ccs_module_sync(None) == B.CCS_EINVAL
    assert L.ccs_module_destroy(None) == B.CCS_EINVAL
    assert L.ccs_module_forward(None, 0, None) == B.CCS_EINVAL
    assert L.ccs_cache_copy(None, None, 16, None) == B.CCS_EINVAL
    assert L.ccs_cache_copy(None, None, 0, None) == B.CCS_OK
    assert len(L.ccs_last_error()) > 0
