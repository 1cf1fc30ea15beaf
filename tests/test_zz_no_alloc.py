"""The decode entry point that allocates nothing (its split-K partials live in a block of device memory built into the
library) against the entry point that takes a workspace: same kernels, so the outputs must agree bit for bit, which is
within the parity bar by construction (the workspace variant is checked against the oracle by the other tests; one case
here is checked against the oracle as well).  Two calls in a row on the shared block, the second with a smaller input,
called through the raw C symbols; and a decode step recorded into a graph and replayed."""
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


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (32, 8)])
def test_decode_step_replayed_from_a_captured_graph(cuda, Hq, Hkv):
    """What the entry point is for: a decode step (append of the new tokens' rows, then decode on the built-in block)
    recorded into a graph, where nothing may allocate.  The graph is replayed several times with other queries and
    other new rows in the same buffers, with eager work and host synchronisation in between; every replay is compared
    bit for bit with the eager calls on the same inputs (append + decode with a workspace).  Both partial kernels."""
    from paper_2404_09526_amd import binding as esp
    dc = wl.decode_pool(f"graph-step-{Hq}/{Hkv}", [300, 0, 1500, 64, 9, 2200, 700, 1], 8192, Hq, Hkv, 61, cuda, n_new=6)
    ml = int(dc.lens.max())
    gen = torch.Generator(device=cuda).manual_seed(99)
    ws = torch.empty(esp.esp_decode_workspace_bytes(dc.B, dc.total_tokens, ml, Hq, Hkv, dc.D), dtype=torch.uint8, device=cuda)
    # the new tokens replace the LAST token's row of the six non-empty requests that have one (their slots are in the
    # slot list already, so that the decode reads what the append just wrote)
    off = wl.host_i32(dc.seq_offsets)
    last = [int(off[b + 1]) - 1 for b in range(dc.B) if off[b + 1] > off[b]][:6]
    tgt = dc.slot_idx[torch.tensor(last, device=cuda)].contiguous()
    new_k = wl.randn_bf16((len(last), Hkv, dc.D), gen, cuda); new_v = wl.randn_bf16((len(last), Hkv, dc.D), gen, cuda)
    q = dc.q.clone()
    O_g = torch.full_like(q, float("nan")); L_g = torch.full((dc.B, Hq), float("nan"), dtype=torch.float32, device=cuda)

    def step(static):
        esp.esp_kv_append(new_k, new_v, tgt, dc.k_pool, dc.v_pool)
        if static:
            esp.esp_partial_attn_decode_static(q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, ml, softmax_scale=dc.scale, O=O_g, LSE=L_g)
            return None
        return esp.esp_partial_attn_decode(q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, ml, softmax_scale=dc.scale, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                  # warm-up on a side stream (the block's address is looked up here)
        step(True)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(True)
    for rep in range(4):
        print(f"[case] graph replay {rep} of {dc.name}", flush=True)
        q.copy_(wl.randn_bf16(tuple(q.shape), gen, cuda))
        new_k.copy_(wl.randn_bf16(tuple(new_k.shape), gen, cuda)); new_v.copy_(wl.randn_bf16(tuple(new_v.shape), gen, cuda))
        O_g.fill_(float("nan")); L_g.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        O_e, L_e = step(False)                                     # eager, same inputs (the append rewrites the same rows)
        torch.cuda.synchronize()
        assert torch.equal(O_g.view(torch.int16), O_e.view(torch.int16)) and torch.equal(L_g.view(torch.int32), L_e.view(torch.int32)), rep
        assert torch.isfinite(L_g[[0, 2, 3, 4, 5, 6, 7]]).all() and torch.isneginf(L_g[1]).all()
        if rep == 0:
            first = O_g.clone()
        else:
            assert not torch.equal(O_g.view(torch.int16), first.view(torch.int16))   # the replay saw the new inputs


def test_a_call_beyond_the_block_is_refused(cuda):
    """Sizes whose split-K partials do not fit the block: a clear error, nothing launched (the pointers are never read)."""
    from paper_2404_09526_amd import binding as esp
    B, total, Hq, Hkv = 256, 7_000_000, 64, 32
    assert esp.esp_decode_workspace_bytes(B, total, 1 << 20, Hq, Hkv, 128) > esp.ESP_DECODE_STATIC_SCRATCH_BYTES
    one = ctypes.c_void_p(256)
    rc = esp.lib.esp_partial_attn_decode_static(one, one, one, 1 << 24, one, one, B, total, 1 << 20, Hq, Hkv, 128,
                                                ctypes.c_float(0.1), one, one, None)
    assert rc == esp.ESP_ERR_WORKSPACE and "built-in block" in esp.last_error()
