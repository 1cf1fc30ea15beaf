"""CPU-only checks of the boundary: the library loads, exports every symbol include/esp.h declares, and
rejects bad arguments on the host before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2404_09526_amd import build
    if build.is_stale():
        build.build_lib(force=True)
    from paper_2404_09526_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "esp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(esp_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(lib.EXPORTS)
    for n in names:
        assert getattr(lib.lib, n) is not None


def test_version_and_error_string(lib):
    assert "gfx950" in lib.version()
    assert isinstance(lib.last_error(), str)


def test_workspace_queries(lib):
    assert lib.esp_prefill_workspace_bytes(8192, 8192, 1, 32, 32, 128) >= 256
    assert lib.esp_prefill_workspace_bytes(8192, 8192, 1, 32, 32, 64) == 0        # unsupported head_dim
    a = lib.esp_decode_workspace_bytes(64, 860000, 131072, 32, 32, 128)
    assert 0 < a < 64 << 20
    assert lib.esp_decode_workspace_bytes(64, 860000, 131072, 32, 5, 128) == 0     # Hq % Hkv != 0: the call is refused
    for Hq, Hkv in [(32, 1), (8, 2), (12, 12), (24, 3), (40, 20)]:                # head counts of the matrix-core kernel
        assert 0 < lib.esp_decode_workspace_bytes(64, 860000, 131072, Hq, Hkv, 128) < 512 << 20


def test_host_side_argument_errors(lib):
    L = lib.lib
    nul = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)      # never dereferenced: every call below fails validation first
    # merge: P out of range, bad D, null arrays
    assert L.esp_merge_partials(one, one, 0, 4, 4, 128, one, nul, nul) == lib.ESP_ERR_INVALID_ARG
    assert L.esp_merge_partials(one, one, 17, 4, 4, 128, one, nul, nul) == lib.ESP_ERR_INVALID_ARG
    assert "P=17" in lib.last_error()
    arr = (ctypes.c_void_p * 1)(256)
    assert L.esp_merge_partials(arr, arr, 1, 4, 4, 64, one, nul, nul) == lib.ESP_ERR_UNSUPPORTED
    assert L.esp_merge_partials(nul, arr, 1, 4, 4, 128, one, nul, nul) == lib.ESP_ERR_INVALID_ARG
    # append
    assert L.esp_kv_append(one, one, one, -1, one, one, 8, 4, 128, nul) == lib.ESP_ERR_INVALID_ARG
    assert L.esp_kv_append(one, one, one, 4, one, one, 8, 4, 96, nul) == lib.ESP_ERR_UNSUPPORTED
    assert L.esp_kv_append(nul, one, one, 4, one, one, 8, 4, 128, nul) == lib.ESP_ERR_INVALID_ARG
    assert L.esp_kv_append(one, one, one, 0, one, one, 8, 4, 128, nul) == lib.ESP_OK     # nothing to do
    # decode
    f = ctypes.c_float(0.1)
    assert L.esp_partial_attn_decode(one, one, one, 8, one, one, 2, 10, 5, 6, 4, 128, f, one, one, one, 1 << 20, nul) \
        == lib.ESP_ERR_INVALID_ARG                                                         # Hq % Hkv
    assert L.esp_partial_attn_decode(one, one, one, 8, one, one, 2, 10, 5, 4, 4, 64, f, one, one, one, 1 << 20, nul) \
        == lib.ESP_ERR_UNSUPPORTED
    assert L.esp_partial_attn_decode(one, one, one, 8, one, one, 2, 10, 5, 4, 4, 128, f, one, one, nul, 0, nul) \
        == lib.ESP_ERR_WORKSPACE
    assert L.esp_partial_attn_decode(one, one, one, 8, one, one, 2, 10, 5, 4, 4, 128, f, one, one, one, 16, nul) \
        == lib.ESP_ERR_WORKSPACE
    assert L.esp_partial_attn_decode(one, one, one, 8, one, one, 2, 10, 5, 12, 12, 128, f, one, one, one, 16, nul) \
        == lib.ESP_ERR_WORKSPACE                                                           # every head count is covered
    assert L.esp_partial_attn_decode(one, one, one, 8, one, one, 0, 0, 0, 4, 4, 128, f, one, one, nul, 0, nul) == lib.ESP_OK
    # decode on the built-in scratch block: the same checks, and sizes beyond the block are refused before any GPU call
    assert L.esp_partial_attn_decode_static(one, one, one, 8, one, one, 2, 10, 5, 6, 4, 128, f, one, one, nul) == lib.ESP_ERR_INVALID_ARG
    assert L.esp_partial_attn_decode_static(one, one, one, 8, one, one, 2, 10, 5, 4, 4, 64, f, one, one, nul) == lib.ESP_ERR_UNSUPPORTED
    assert lib.esp_decode_workspace_bytes(256, 7_000_000, 1 << 20, 64, 32, 128) > lib.ESP_DECODE_STATIC_SCRATCH_BYTES
    assert L.esp_partial_attn_decode_static(one, one, one, 1 << 24, one, one, 256, 7_000_000, 1 << 20, 64, 32, 128, f, one, one, nul) \
        == lib.ESP_ERR_WORKSPACE
    assert "built-in block" in lib.last_error()
    assert L.esp_partial_attn_decode_static(one, one, one, 8, one, one, 0, 0, 0, 4, 4, 128, f, one, one, nul) == lib.ESP_OK
    # decode combined with the peers' partials: the same checks, the number of peers, null or overlapping arrays
    def decode_merge(n_peers, peer_O=one, peer_L=one, O=one, LSE=one, Hq=4, D=128, ws=one, ws_bytes=1 << 20):
        return L.esp_partial_attn_decode_merge(one, one, one, 8, one, one, 2, 10, 5, Hq, 4, D, f, peer_O, peer_L, n_peers,
                                               O, LSE, ws, ws_bytes, nul)
    far = (ctypes.c_void_p * 2)(1 << 20, 2 << 20)
    assert decode_merge(-1) == lib.ESP_ERR_INVALID_ARG
    assert decode_merge(16) == lib.ESP_ERR_INVALID_ARG and "n_peers=16" in lib.last_error()
    assert decode_merge(2, far, far, Hq=6) == lib.ESP_ERR_INVALID_ARG
    assert decode_merge(2, far, far, D=64) == lib.ESP_ERR_UNSUPPORTED
    assert decode_merge(2, nul, far) == lib.ESP_ERR_INVALID_ARG
    assert decode_merge(2, (ctypes.c_void_p * 2)(1 << 20, 0), far) == lib.ESP_ERR_INVALID_ARG          # a null partial
    assert decode_merge(2, far, far, O=ctypes.c_void_p((2 << 20) + 512)) == lib.ESP_ERR_INVALID_ARG     # O inside a peer's O
    assert "overlaps" in lib.last_error()
    assert decode_merge(2, far, far, LSE=ctypes.c_void_p((1 << 20) + 4)) == lib.ESP_ERR_INVALID_ARG
    assert decode_merge(2, far, far, ws=nul, ws_bytes=0) == lib.ESP_ERR_WORKSPACE
    # prefill
    args = dict(batch=1, Tq=16, Tkv=16, max_q=16, max_kv=16, Hq=4, Hkv=4, D=128)

    def prefill(ws=one, ws_bytes=1 << 20, cu_q=nul, cu_kv=nul, **kw):
        a = dict(args, **kw)
        return L.esp_partial_attn_prefill(one, one, one, one, one, cu_q, cu_kv, a["batch"], a["Tq"], a["Tkv"], a["max_q"],
                                          a["max_kv"], a["Hq"], a["Hkv"], a["D"], f, 1, one, one, ws, ws_bytes, nul)
    assert prefill(D=64) == lib.ESP_ERR_UNSUPPORTED
    assert prefill(Hq=6) == lib.ESP_ERR_INVALID_ARG
    assert prefill(batch=2) == lib.ESP_ERR_INVALID_ARG              # batch > 1 without cu arrays
    assert prefill(cu_q=one) == lib.ESP_ERR_INVALID_ARG             # only one of cu_q / cu_kv
    assert prefill(ws=nul, ws_bytes=0) == lib.ESP_ERR_WORKSPACE
    assert prefill(ws_bytes=8) == lib.ESP_ERR_WORKSPACE
    assert prefill(ws=ctypes.c_void_p(8)) == lib.ESP_ERR_WORKSPACE  # misaligned
    assert prefill(Tq=0, max_q=0) == lib.ESP_OK                     # nothing to do

    def prefill_direct(slots=one, num_slots=64, ws=one, ws_bytes=1 << 20, **kw):
        a = dict(args, **kw)
        return L.esp_partial_attn_prefill_pool_direct(one, one, one, num_slots, slots, one, one, nul, nul, a["batch"], a["Tq"],
                                                      a["Tkv"], a["max_q"], a["max_kv"], a["Hq"], a["Hkv"], a["D"], f, 1, 0,
                                                      one, one, ws, ws_bytes, nul)
    assert prefill_direct(slots=nul) == lib.ESP_ERR_INVALID_ARG
    assert prefill_direct(num_slots=0) == lib.ESP_ERR_INVALID_ARG
    assert prefill_direct(num_slots=-1) == lib.ESP_ERR_INVALID_ARG
    assert prefill_direct(D=64) == lib.ESP_ERR_UNSUPPORTED
    assert prefill_direct(Hq=6) == lib.ESP_ERR_INVALID_ARG
    assert prefill_direct(ws=nul, ws_bytes=0) == lib.ESP_ERR_WORKSPACE
    assert prefill_direct(Tq=0, max_q=0) == lib.ESP_OK


def test_no_oracle_or_fallback_in_product():
    """The product path must not import the oracle (it is test infrastructure)."""
    pkg = os.path.join(ROOT, "paper_2404_09526_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text, fn
                assert "esp_oracle" not in text, fn
