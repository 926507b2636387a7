"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad configurations before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2604_17701_amd import binding
from wisv_inputs import configs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = ""
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if name.endswith(".h"):
            with open(os.path.join(ROOT, "include", name)) as f:
                text += f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wisv_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.load_library()
    names = _declared_symbols()
    assert {"wisv_ctx_create", "wisv_verify_round", "wisv_destroy"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.EXPORTS)


def test_struct_sizes_match_the_header_layout():
    # 7 ints, 2 floats, 9 ints, then three pointer-sized members (8-byte aligned)
    assert C.sizeof(binding.wisv_config) == 18 * 4 + 3 * 8
    assert C.sizeof(binding.wisv_round_in) == 8 + 5 * 8 + 8 + 2 * 8 + 8
    assert C.sizeof(binding.wisv_round_out) == 6 * 8
    assert C.sizeof(binding.wisv_weights) == 16 * 8


def _create(cfg, weights=None):
    lib = binding.load_library()
    h = C.c_void_p()
    err = C.create_string_buffer(256)
    rc = lib.wisv_ctx_create(C.byref(cfg) if cfg is not None else None, weights, C.byref(h), err, 256)
    return rc, h, err.value.decode()


@pytest.mark.parametrize("field,value,needle", [
    ("n_layers", 0, "n_layers"), ("d_model", 100, "d_model"), ("n_kv_heads", 3, "n_heads"),
    ("head_dim", 48, "head_dim"), ("dtype", 7, "dtype"), ("max_k", 17, "max_k"), ("max_ctx", 4, "max_ctx"),
    ("d_csi", 0, "decision-head"), ("head_act", 5, "head_act"), ("vocab", 1, "vocab"), ("max_batch", 0, "max_batch"),
])
def test_create_rejects_bad_config_before_any_gpu_work(field, value, needle):
    cfg = binding.make_config(configs.TINY, max_batch=1, max_ctx=64, max_k=4)
    setattr(cfg, field, value)
    rc, h, msg = _create(cfg)
    assert rc == binding.WISV_EINVAL and not h.value and needle in msg


def test_create_rejects_null_arguments():
    cfg = binding.make_config(configs.TINY, max_batch=1, max_ctx=64, max_k=4)
    rc, h, msg = _create(cfg, None)
    assert rc == binding.WISV_EINVAL and "weights" in msg
    rc, h, msg = _create(None, None)
    assert rc == binding.WISV_EINVAL and "config" in msg
    lib = binding.load_library()
    assert lib.wisv_ctx_create(C.byref(cfg), None, None, None, 0) == binding.WISV_EINVAL
    # a borrowed cache that is too small
    cfg.kv_cache, cfg.kv_bytes = 4096, 16
    rc, _, msg = _create(cfg, C.pointer(binding.wisv_weights()))
    assert rc == binding.WISV_EINVAL and "kv_cache" in msg


def test_null_context_is_handled():
    lib = binding.load_library()
    assert lib.wisv_destroy(None) == binding.WISV_OK
    assert lib.wisv_verify_round(None, None, None) == binding.WISV_EINVAL
    assert lib.wisv_last_error(None) == b""
    assert lib.wisv_set_state(None, 0, 0, 0) == binding.WISV_EINVAL


def test_kv_fill_follows_the_documented_cache_layout():
    """K plane position-major, V plane in blocks of 32 positions with element (pos, dim) at
    ((pos // 32) * head_dim + dim) * 32 + pos % 32 (include/wisv.h, wisv_config.kv_cache)."""
    import torch
    m = configs.TINY
    kv = binding.new_kv_cache(m, 2, 70, "cpu")
    g, hd = m.n_kv_heads, m.head_dim
    assert kv.shape[-1] == binding.ctx_pad(70) * hd == 96 * hd
    gen_ = torch.Generator().manual_seed(1)
    k, v = torch.randn(g, 45, hd, generator=gen_), torch.randn(g, 45, hd, generator=gen_)
    binding.kv_fill(kv, m, 1, 1, k, v)
    for gh in range(g):
        for pos in (0, 1, 31, 32, 44):
            for dim in (0, 5, hd - 1):
                assert kv[1, 1, 1][gh, ((pos // 32) * hd + dim) * 32 + pos % 32] == v[gh, pos, dim]
                assert kv[1, 1, 0][gh, pos * hd + dim] == k[gh, pos, dim]
    assert float(kv[0].abs().sum()) == 0.0 and float(kv[1, 0].abs().sum()) == 0.0


def test_bench_refuses_more_than_one_gpu():
    """The round runs on one GPU: asking bench.py for more ends with a message, before anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_profile_summaries_parse_and_name_the_kernels_bench_looks_for():
    """The committed rocprofv3 summaries are what bench.py reads its traffic and duration figures from: they must
    parse, carry the hash of the sources they were taken at, and hold the kernel classes bench.py reports for each
    of the four 8B-shaped workloads."""
    import bench_profiles as ps
    prof = os.path.join(ROOT, "profiles")
    for index in (1, 2, 3, 4):
        workload = configs.get(index).name
        sha, table = ps.read_traffic(os.path.join(prof, f"{workload}_hbm_traffic.txt"))
        stats = os.path.join(prof, f"{workload}_kernel_stats.txt")
        kern = ps.read_kernels(stats)
        assert sha and len(sha) == 16 and ps.read_hash(stats) == sha, workload
        for names in (table, kern):
            classes = {ps.kernel_class(n) for n in names}
            assert {"gemm_gate_up", "gemm_qkv_o_down", "lm_head", "attention"} <= classes, (workload, classes)
        for n, fetch, write in table.values():
            assert n > 0 and fetch >= 0 and write >= 0
    assert ps.template_args("k_gemm_ws<1, 1, 7, 1, 16, 0, 1>") == ("k_gemm_ws", ["1", "1", "7", "1", "16", "0", "1"])
    assert ps.kernel_class("k_gemm_ws<1, 1, 7, 1, 16, 0, 1>") == "gemm_gate_up"
    assert ps.kernel_class("k_gemm_mm<4, 1, 8, 1, 2, 2, 2, 2, 1>") == "lm_head"
    assert ps.kernel_class("k_attn_mfma<1, 8, true>") == "attention"
    assert ps.template_args("k_decide") == ("k_decide", []) and ps.kernel_class("k_decide") is None
