"""The decode entry point that allocates nothing (its split-K partials live in a block of device memory built into the
library) against the entry point that takes a workspace: same kernels, so the outputs must agree bit for bit, which is
within the parity bar by construction (the workspace variant is checked against the oracle by the other tests; one case
here is checked against the oracle as well).  Two calls in a row on the shared block, the second with a smaller input,
called through the raw C symbols."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from esp_checks import check_o_lse
from paper_2404_09526_amd import workloads as wl

pytestmark = pytest.mark.gpu


def raw_decode(esp, dc, static, O, LSE, ws=None):
    L = esp.lib
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    args = [p(dc.q), p(dc.k_pool), p(dc.v_pool), dc.num_slots, p(dc.slot_idx), p(dc.seq_offsets), dc.B, dc.total_tokens,
            int(dc.lens.max()), dc.Hq, dc.Hkv, dc.D, ctypes.c_float(dc.scale), p(O), p(LSE)]
    if static:
        return L.esp_partial_attn_decode_static(*args, stream)
    return L.esp_partial_attn_decode(*args, p(ws), ws.numel(), stream)


def test_decode_on_the_built_in_scratch_block(cuda):
    from paper_2404_09526_amd import binding as esp
    big = wl.decode_pool("static-big", wl.lognormal_lengths(24, 3000, 10, 40000, 31), 1 << 18, 8, 8, 31, cuda, n_new=0)
    small = wl.decode_pool("static-small", [0, 5, 700, 64, 0, 1], 4096, 32, 8, 32, cuda, n_new=0)
    for rep, dc in enumerate((big, small, big)):                     # the second call is smaller than the first
        print(f"[case] {dc.name}: B={dc.B} total={dc.total_tokens} Hq={dc.Hq} Hkv={dc.Hkv}", flush=True)
        need = esp.esp_decode_workspace_bytes(dc.B, dc.total_tokens, int(dc.lens.max()), dc.Hq, dc.Hkv, dc.D)
        assert 0 < need <= esp.ESP_DECODE_STATIC_SCRATCH_BYTES
        ws = torch.empty(need, dtype=torch.uint8, device=cuda)
        O_ws = torch.full_like(dc.q, float("nan")); L_ws = torch.full((dc.B, dc.Hq), float("nan"), dtype=torch.float32, device=cuda)
        O_st = torch.full_like(dc.q, float("nan")); L_st = torch.full_like(L_ws, float("nan"))
        assert raw_decode(esp, dc, False, O_ws, L_ws, ws) == 0, esp.last_error()
        assert raw_decode(esp, dc, True, O_st, L_st) == 0, esp.last_error()
        torch.cuda.synchronize()
        assert torch.equal(O_st.view(torch.int16), O_ws.view(torch.int16)) and torch.equal(L_st.view(torch.int32), L_ws.view(torch.int32)), rep
        assert not torch.isnan(O_st.float()).any() and not torch.isnan(L_st).any()
        if dc is small:
            O_small, L_small = O_st, L_st
    # the small case against the oracle as well (its own pool image, built by its own scatter)
    dc = small
    kp = np.zeros((dc.num_slots, dc.Hkv, dc.D), np.uint16); vp = np.zeros_like(kp)
    slots, off = wl.host_i32(dc.slot_idx), wl.host_i32(dc.seq_offsets)
    for b, (kr, vr) in dc.host_rows.items():
        oracle.kv_append(kr, vr, slots[off[b]:off[b + 1]], kp, vp)
    Or, Lr = oracle.partial_attn_decode_all(wl.bits(dc.q), kp, vp, slots, off, dc.scale)
    check_o_lse(O_small.float().cpu().numpy().reshape(-1, dc.D), L_small.cpu().numpy().reshape(-1), Or.reshape(-1, dc.D), Lr.reshape(-1),
                "static-small")


def test_a_call_beyond_the_block_is_refused(cuda):
    """Sizes whose split-K partials do not fit the block: a clear error, nothing launched (the pointers are never read)."""
    from paper_2404_09526_amd import binding as esp
    B, total, Hq, Hkv = 256, 7_000_000, 64, 32
    assert esp.esp_decode_workspace_bytes(B, total, 1 << 20, Hq, Hkv, 128) > esp.ESP_DECODE_STATIC_SCRATCH_BYTES
    one = ctypes.c_void_p(256)
    rc = esp.lib.esp_partial_attn_decode_static(one, one, one, 1 << 24, one, one, B, total, 1 << 20, Hq, Hkv, 128,
                                                ctypes.c_float(0.1), one, one, None)
    assert rc == esp.ESP_ERR_WORKSPACE and "built-in block" in esp.last_error()
