"""C-ABI checks that need no GPU: the library loads, exports every symbol the header declares, and
the host-side argument checks answer with error codes instead of crashing."""
import ctypes as C
import os
import re

import pytest

from paper_2501_06589_amd import ladder

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ladder.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ladder_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ladder.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return ladder.lib()


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = declared_symbols()
    assert set(names) == set(ladder.EXPORTS), (names, sorted(ladder.EXPORTS))
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layout_matches_header():
    text = open(os.path.join(ROOT, "include", "ladder.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} ladder_config;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:int32_t|float)\s+([a-z_]+)\s*;", body)
    assert fields == [n for n, _ in ladder.ladder_config._fields_]
    assert C.sizeof(ladder.ladder_config) == 4 * len(fields)
    body = re.search(r"typedef struct \{(.*?)\} ladder_layer_weights;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    assert re.findall(r"const void\*\s+([a-z_]+)\s*;", body) == [n for n, _ in ladder.ladder_layer_weights._fields_]


def good_config(**kw):
    base = dict(n_layers=2, hidden=256, n_q_heads=2, n_kv_heads=1, head_dim=64, inter=344, tp_degree=2,
                n_real_shards=2, max_batch=1, max_seq=40, max_tokens=32, dtype=ladder.LADDER_FP32)
    base.update(kw)
    return ladder.make_config(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(n_layers=0), ladder.LADDER_E_ARG),
    (dict(hidden=-8), ladder.LADDER_E_ARG),
    (dict(dtype=7), ladder.LADDER_E_ARG),
    (dict(wiring=3), ladder.LADDER_E_ARG),
    (dict(rms_eps=0.0), ladder.LADDER_E_ARG),
    (dict(hidden=252), ladder.LADDER_E_SHAPE),
    (dict(n_q_heads=3, n_kv_heads=2), ladder.LADDER_E_SHAPE),
    (dict(head_dim=63), ladder.LADDER_E_SHAPE),
    (dict(head_dim=512), ladder.LADDER_E_SHAPE),
    (dict(n_real_shards=3), ladder.LADDER_E_SHAPE),
    (dict(max_tokens=64), ladder.LADDER_E_SHAPE),
    (dict(n_standard_layers=5), ladder.LADDER_E_SHAPE),
    (dict(tp_degree=4, peer_pool=2, peer_rows=0), ladder.LADDER_E_SHAPE),
])
def test_bad_config_is_rejected_before_any_gpu_call(lib, kw, code):
    h = C.c_void_p()
    cfg = good_config(**kw)
    assert lib.ladder_init(C.byref(cfg), None, C.byref(h)) == code
    assert not h
    assert len(lib.ladder_last_error(None)) > 0


def test_null_arguments(lib):
    h = C.c_void_p()
    assert lib.ladder_init(None, None, C.byref(h)) == ladder.LADDER_E_ARG
    cfg = good_config()
    assert lib.ladder_init(C.byref(cfg), None, None) == ladder.LADDER_E_ARG
    lib.ladder_free(None)                                     # no-op
    assert lib.ladder_prefill(None, None, 1, 1, None) == ladder.LADDER_E_ARG
    assert lib.ladder_decode_step(None, None, None) == ladder.LADDER_E_ARG
    assert lib.ladder_load_layer(None, 0, 0, None) == ladder.LADDER_E_ARG
    assert lib.ladder_position(None, None, None) == ladder.LADDER_E_ARG
    assert lib.ladder_device_bytes(None) == 0
    assert lib.ladder_profile_read(None, 0, None, None) == ladder.LADDER_E_ARG


def test_init_without_a_gpu_reports_a_hip_error_or_succeeds(lib):
    # on a machine without a GPU the first HIP call fails: that must come back as an error code
    h = C.c_void_p()
    cfg = good_config()
    rc = lib.ladder_init(C.byref(cfg), None, C.byref(h))
    assert rc in (ladder.LADDER_OK, ladder.LADDER_E_HIP)
    if rc == ladder.LADDER_OK:
        lib.ladder_free(h)
    else:
        assert not h and b"hip" in lib.ladder_last_error(None).lower()


def test_sizing_calls_need_no_gpu(lib):
    """ladder_workspace_bytes / ladder_weight_bytes walk the memory plan on the host: positive for a good
    configuration, 0 (with a text) for a rejected one, growing with the cache capacity, and the weight store of a
    tile-aligned bf16 configuration is exactly two bytes per projection parameter."""
    cfg = good_config()
    ws, wt = ladder.workspace_bytes(cfg), ladder.weight_bytes(cfg)
    assert ws > 0 and wt > 0
    assert ladder.workspace_bytes(good_config(max_seq=4000)) > ws
    assert ladder.weight_bytes(good_config(max_seq=4000)) == wt
    assert ladder.workspace_bytes(good_config(hidden=252)) == 0 and len(lib.ladder_last_error(None)) > 0
    assert lib.ladder_workspace_bytes(None) == 0
    h, nq, nkv, d, inter, n = 512, 8, 2, 64, 448, 3
    cfg = good_config(n_layers=n, hidden=h, n_q_heads=nq, n_kv_heads=nkv, head_dim=d, inter=inter, tp_degree=1,
                      n_real_shards=1, dtype=ladder.LADDER_BF16)
    params = h * (nq + 2 * nkv) * d + nq * d * h + 3 * h * inter
    assert ladder.weight_bytes(cfg) == n * params * 2
    # the KV cache dominates the workspace of a long-context configuration: capacity rounded up to 128 positions
    big = good_config(n_layers=n, hidden=h, n_q_heads=nq, n_kv_heads=nkv, head_dim=d, inter=inter, tp_degree=1,
                      n_real_shards=1, dtype=ladder.LADDER_BF16, max_batch=4, max_seq=10000, max_tokens=1)
    kv = n * 2 * 4 * nkv * 10112 * d * 2
    assert kv <= ladder.workspace_bytes(big) <= kv + (64 << 20)
