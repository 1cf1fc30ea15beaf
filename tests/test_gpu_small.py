"""GPU parity, small cases checked exhaustively against the CPU oracle (element by element):
several tiles plus ragged tails, all striped offsets, var-len batches, GQA, unsorted positions,
empty visible sets, empty requests, and config 1 of the benchmark in full."""
import math

import numpy as np
import pytest
import torch

import oracle
from esp_checks import check_o_lse
from paper_2404_09526_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def esp(cuda):
    from paper_2404_09526_amd import binding
    return binding


def say(msg):
    print(f"[case] {msg}", flush=True)


def seeded_positions(n, hi, seed, device):
    """n query positions drawn uniformly from [0, hi), the same in every run."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    return torch.randint(0, hi, (n,), generator=g, dtype=torch.int32).to(device)


def run_prefill_case(esp, pc, check_merged=True, workspace=None):
    """Runs every shard through the HIP path, with bf16 and with fp32 partial outputs, and checks each partial.  With
    several shards: the fp32 partials are merged and compared with the oracle's merge of ITS OWN fp64 partials, i.e.
    with attention over the union of the shards (the pipeline: one rounding to bf16, at the end); the bf16 partials are
    merged and compared with the oracle's merge of those very bf16 arrays (the merge kernel on its own).  Returns the
    bf16 partials."""
    qb, qp = wl.bits(pc.q), wl.host_i32(pc.q_pos)
    cu_q = wl.host_i32(pc.cu_q)
    Tq, Hq, D = pc.q.shape
    rows = np.repeat(np.arange(Tq, dtype=np.int64), Hq)
    heads = np.tile(np.arange(Hq, dtype=np.int64), Tq)
    req_of_row = np.searchsorted(cu_q, np.arange(Tq), side="right") - 1
    single = pc.batch == 1
    parts, parts32, refs = [], [], []
    for si, s in enumerate(pc.shards):
        say(f"{pc.name} shard {si}: Tq={Tq} Tkv={s.k.shape[0]} Hq={Hq} Hkv={pc.Hkv} batch={pc.batch} causal={pc.causal}")
        # outputs start as NaN: a row the launch never wrote cannot pass as a stale copy of an earlier result
        O = torch.full_like(pc.q, float("nan"))
        LSE = torch.full((Tq, Hq), float("nan"), dtype=torch.float32, device=pc.q.device)
        esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos,
                                     None if single else pc.cu_q, None if single else s.cu_kv,
                                     None if single else pc.max_q, None if single else s.max_kv,
                                     softmax_scale=pc.scale, causal=pc.causal, O=O, LSE=LSE, workspace=workspace)
        torch.cuda.synchronize()
        cu_kv = wl.host_i32(s.cu_kv)
        lo, hi = cu_kv[req_of_row[rows]], cu_kv[req_of_row[rows] + 1]
        Or, Lr = oracle.partial_attn(qb, wl.bits(s.k), wl.bits(s.v), qp, wl.host_i32(s.kv_pos), pc.scale, pc.causal,
                                     rows, heads, lo, hi)
        check_o_lse(O.float().cpu().numpy().reshape(-1, D), LSE.cpu().numpy().reshape(-1), Or, Lr,
                    f"{pc.name} shard {si}")
        O32 = torch.full(pc.q.shape, float("nan"), dtype=torch.float32, device=pc.q.device)
        LSE32 = torch.full_like(LSE, float("nan"))
        esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos,
                                     None if single else pc.cu_q, None if single else s.cu_kv,
                                     None if single else pc.max_q, None if single else s.max_kv,
                                     softmax_scale=pc.scale, causal=pc.causal, O=O32, LSE=LSE32, workspace=workspace)
        torch.cuda.synchronize()
        check_o_lse(O32.cpu().numpy().reshape(-1, D), LSE32.cpu().numpy().reshape(-1), Or, Lr, f"{pc.name} shard {si} (fp32 out)")
        # the two output types differ by the final rounding only
        assert torch.equal(O32.to(torch.bfloat16).view(torch.int16), O.view(torch.int16)) and torch.equal(LSE32.view(torch.int32), LSE.view(torch.int32))
        parts.append((O, LSE)); parts32.append((O32, LSE32)); refs.append((Or, Lr))
    if check_merged and len(parts) > 1:
        say(f"{pc.name} merge of {len(parts)} partials")
        Om, Lm = esp.esp_merge_partials([p[0] for p in parts32], [p[1] for p in parts32])
        torch.cuda.synchronize()
        # pipeline check: the oracle merges ITS OWN fp64 partials = attention over the union of the shards
        Oref, Lref = oracle.merge_partials(np.stack([r[0] for r in refs]), np.stack([r[1] for r in refs]))
        check_o_lse(Om.float().cpu().numpy().reshape(-1, D), Lm.cpu().numpy().reshape(-1), Oref, Lref, f"{pc.name} merged")
        # merge kernel on bf16 partials: against the oracle's merge of the very arrays the GPU merged
        Ob, Lb = esp.esp_merge_partials([p[0] for p in parts], [p[1] for p in parts])
        torch.cuda.synchronize()
        Oref, Lref = oracle.merge_partials(np.stack([oracle.bf16_bits_to_f64(wl.bits(p[0])).reshape(-1, D) for p in parts]),
                                           np.stack([p[1].cpu().numpy().astype(np.float64).reshape(-1) for p in parts]))
        check_o_lse(Ob.float().cpu().numpy().reshape(-1, D), Lb.cpu().numpy().reshape(-1), Oref, Lref, f"{pc.name} merge of bf16 partials")
    return parts


# ------------------------------------------------------------------ config 1, in full
def test_config1_prefill_exhaustive(esp, cuda):
    pc = wl.config1_prefill(cuda)
    assert pc.visible_pairs_per_head == 131072 + 98432
    run_prefill_case(esp, pc)


def test_config1_merged_equals_unpartitioned_attention(esp, cuda):
    """The GPU pipeline (2 partials -> merge) against the oracle run directly on the whole 1024-token KV."""
    pc = wl.config1_prefill(cuda)
    parts = [esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale, out_dtype=torch.float32)
             for s in pc.shards]
    Om, Lm = esp.esp_merge_partials([p[0] for p in parts], [p[1] for p in parts])
    torch.cuda.synchronize()
    k_all = np.concatenate([wl.bits(s.k) for s in pc.shards]); v_all = np.concatenate([wl.bits(s.v) for s in pc.shards])
    pos = np.concatenate([wl.host_i32(s.kv_pos) for s in pc.shards])
    Or, Lr = oracle.partial_attn_all(wl.bits(pc.q), k_all, v_all, wl.host_i32(pc.q_pos), pos, pc.scale, True)
    check_o_lse(Om.float().cpu().numpy().reshape(-1, 128), Lm.cpu().numpy().reshape(-1), Or.reshape(-1, 128), Lr.reshape(-1),
                "C1 pipeline")


def run_decode_case(esp, dc, heads=None):
    say(f"{dc.name}: B={dc.B} lens={dc.lens.tolist()[:8]}... total={dc.total_tokens} Hq={dc.Hq} Hkv={dc.Hkv} S={dc.num_slots}")
    # oracle's own pool image, built by its own scatter from the host copies of the rows
    kp = np.zeros((dc.num_slots, dc.Hkv, dc.D), np.uint16); vp = np.zeros_like(kp)
    slots, off = wl.host_i32(dc.slot_idx), wl.host_i32(dc.seq_offsets)
    for b, (kr, vr) in dc.host_rows.items():
        oracle.kv_append(kr, vr, slots[off[b]:off[b + 1]], kp, vp)
    O, LSE = esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets,
                                         int(dc.lens.max()) if dc.B else 0, softmax_scale=dc.scale)
    torch.cuda.synchronize()
    reqs = np.repeat(np.array(sorted(dc.host_rows), np.int64), dc.Hq)
    hs = np.tile(np.arange(dc.Hq, dtype=np.int64), len(dc.host_rows))
    Or, Lr = oracle.partial_attn_decode(wl.bits(dc.q), kp, vp, slots, off, dc.scale, reqs, hs)
    Og = O.float().cpu().numpy()[reqs, hs]; Lg = LSE.cpu().numpy()[reqs, hs]
    check_o_lse(Og, Lg, Or, Lr, dc.name)
    return O, LSE, kp, vp


def test_config1_decode_append_merge(esp, cuda):
    dc = wl.config1_decode(cuda)
    O, LSE, kp, vp = run_decode_case(esp, dc)
    # bit-exact pool before the append (the oracle image was built by the oracle's scatter)
    assert np.array_equal(wl.bits(dc.k_pool), kp) and np.array_equal(wl.bits(dc.v_pool), vp)
    # append 4 tokens to free slots: every slot of the pool is compared
    oracle.kv_append(wl.bits(dc.new_k), wl.bits(dc.new_v), wl.host_i32(dc.new_slots), kp, vp)
    esp.esp_kv_append(dc.new_k, dc.new_v, dc.new_slots, dc.k_pool, dc.v_pool)
    torch.cuda.synchronize()
    assert np.array_equal(wl.bits(dc.k_pool), kp) and np.array_equal(wl.bits(dc.v_pool), vp)
    # merge with 3 synthetic peer partials: kernel test on the very arrays given to the GPU
    Om, Lm = esp.esp_merge_partials([O] + list(dc.peer_O), [LSE] + list(dc.peer_LSE))
    torch.cuda.synchronize()
    Op = np.stack([oracle.bf16_bits_to_f64(wl.bits(t)) for t in [O] + list(dc.peer_O)])
    Lp = np.stack([t.cpu().numpy().astype(np.float64) for t in [LSE] + list(dc.peer_LSE)])
    Oref, Lref = oracle.merge_partials(Op, Lp)
    check_o_lse(Om.float().cpu().numpy().reshape(-1, 128), Lm.cpu().numpy().reshape(-1), Oref.reshape(-1, 128),
                Lref.reshape(-1), "C1 merge")


def test_decode_in_two_master_groups(esp, cuda):
    """Distributed decoding with several masters (Sec. 4.2): the requests this instance is master of and the ones it
    helps with are decoded by separate calls, each over its own part of the slot list; both against the oracle."""
    import dataclasses
    dc = wl.config1_decode(cuda)
    h = dc.B // 2
    off = wl.host_i32(dc.seq_offsets)
    for name, lo, hi in (("own", 0, h), ("helped", h, dc.B)):
        sub = dataclasses.replace(
            dc, name=f"{dc.name}-{name}", lens=dc.lens[lo:hi], q=dc.q[lo:hi].contiguous(),
            slot_idx=dc.slot_idx[int(off[lo]):int(off[hi])].contiguous(),
            seq_offsets=(dc.seq_offsets[lo:hi + 1] - int(off[lo])).contiguous(),
            host_rows={b - lo: r for b, r in dc.host_rows.items() if lo <= b < hi})
        run_decode_case(esp, sub)


def test_multi_master_decode_on_two_streams(esp, cuda):
    """Distributed decoding with several masters on one GPU (Sec. 4.2, Fig. 8): this instance is master of half of the
    requests and only helps with the others.  The helped requests' queries arrive by a host-to-device copy (pinned
    memory) on a second stream of default priority while the own requests are decoded; then the helped ones are decoded
    and their (O, LSE) go back by device-to-host copies on the second stream while the own results are merged with the
    peers' partials.  Several rounds in a row; both halves, what arrived on the host, and the merge against the oracle."""
    lens = [300, 0, 1500, 64, 9, 2200, 700, 1]
    dc = wl.decode_pool("multi-master", lens, 8192, 8, 4, 36, cuda, n_new=0)
    h = dc.B // 2
    off = wl.host_i32(dc.seq_offsets)
    off_h = int(off[h])
    own_off = dc.seq_offsets[:h + 1].contiguous(); peer_off = (dc.seq_offsets[h:] - off_h).contiguous()
    own_slots, peer_slots = dc.slot_idx[:off_h].contiguous(), dc.slot_idx[off_h:].contiguous()
    ml_own, ml_peer = int(dc.lens[:h].max()), int(dc.lens[h:].max())
    q_host = dc.q[h:].cpu().pin_memory()                           # the other masters' queries, as they come off the wire
    q_peer = torch.zeros_like(dc.q[h:])
    O_own = torch.empty_like(dc.q[:h]); L_own = torch.empty((h, dc.Hq), dtype=torch.float32, device=cuda)
    O_peer = torch.empty_like(dc.q[h:]); L_peer = torch.empty((dc.B - h, dc.Hq), dtype=torch.float32, device=cuda)
    O_back = torch.empty(O_peer.shape, dtype=O_peer.dtype).pin_memory(); L_back = torch.empty(L_peer.shape, dtype=L_peer.dtype).pin_memory()
    ws_own = torch.empty(esp.esp_decode_workspace_bytes(h, off_h, ml_own, dc.Hq, dc.Hkv, dc.D), dtype=torch.uint8, device=cuda)
    ws_peer = torch.empty(esp.esp_decode_workspace_bytes(dc.B - h, dc.total_tokens - off_h, ml_peer, dc.Hq, dc.Hkv, dc.D),
                          dtype=torch.uint8, device=cuda)
    mO, mL = torch.empty_like(O_own), torch.empty_like(L_own)
    wire = torch.cuda.Stream()                                      # default priority
    main = torch.cuda.current_stream()
    # the oracle's answers: its own pool image, every request, every head
    kp = np.zeros((dc.num_slots, dc.Hkv, dc.D), np.uint16); vp = np.zeros_like(kp)
    slots = wl.host_i32(dc.slot_idx)
    for b, (kr, vr) in dc.host_rows.items():
        oracle.kv_append(kr, vr, slots[off[b]:off[b + 1]], kp, vp)
    Or, Lr = oracle.partial_attn_decode_all(wl.bits(dc.q), kp, vp, slots, off, dc.scale)
    for rnd in range(3):
        say(f"multi-master round {rnd}")
        for t in (q_peer, O_own, O_peer, mO):
            t.fill_(float("nan"))
        O_back.fill_(float("nan")); L_back.fill_(float("nan"))
        wire.wait_stream(main)
        with torch.cuda.stream(wire):
            q_peer.copy_(q_host, non_blocking=True)                 # peers' queries arrive while the own requests are decoded
        esp.esp_partial_attn_decode(dc.q[:h], dc.k_pool, dc.v_pool, own_slots, own_off, ml_own, softmax_scale=dc.scale,
                                    O=O_own, LSE=L_own, workspace=ws_own)
        main.wait_stream(wire)
        esp.esp_partial_attn_decode(q_peer, dc.k_pool, dc.v_pool, peer_slots, peer_off, ml_peer, softmax_scale=dc.scale,
                                    O=O_peer, LSE=L_peer, workspace=ws_peer)
        wire.wait_stream(main)
        with torch.cuda.stream(wire):
            O_back.copy_(O_peer, non_blocking=True); L_back.copy_(L_peer, non_blocking=True)   # results go back to their masters
        esp.esp_merge_partials([O_own] + [p[:h] for p in dc.peer_O], [L_own] + [p[:h] for p in dc.peer_LSE], O=mO, LSE=mL)
        # the same master step as ONE call (local attention and merge together), while the copies still run
        fO, fL = esp.esp_partial_attn_decode_merge(dc.q[:h], dc.k_pool, dc.v_pool, own_slots, own_off, ml_own,
                                                   [p[:h] for p in dc.peer_O], [p[:h] for p in dc.peer_LSE],
                                                   softmax_scale=dc.scale, workspace=ws_own)
        main.wait_stream(wire)
        torch.cuda.synchronize()
        check_o_lse(O_own.float().cpu().numpy().reshape(-1, dc.D), L_own.cpu().numpy().reshape(-1), Or[:h].reshape(-1, dc.D),
                    Lr[:h].reshape(-1), f"own requests, round {rnd}")
        check_o_lse(O_back.float().numpy().reshape(-1, dc.D), L_back.numpy().reshape(-1), Or[h:].reshape(-1, dc.D),
                    Lr[h:].reshape(-1), f"helped requests as received by their masters, round {rnd}")
        assert torch.equal(O_back.view(torch.int16), O_peer.cpu().view(torch.int16)) and torch.equal(L_back.view(torch.int32), L_peer.cpu().view(torch.int32))
        Op = np.stack([oracle.bf16_bits_to_f64(wl.bits(t)) for t in [O_own] + [p[:h].contiguous() for p in dc.peer_O]])
        Lp = np.stack([t.cpu().numpy().astype(np.float64) for t in [L_own] + [p[:h] for p in dc.peer_LSE]])
        Oref, Lref = oracle.merge_partials(Op, Lp)
        check_o_lse(mO.float().cpu().numpy().reshape(-1, dc.D), mL.cpu().numpy().reshape(-1), Oref.reshape(-1, dc.D), Lref.reshape(-1),
                    f"merge at the master, round {rnd}")
        Op = np.stack([Or[:h]] + [oracle.bf16_bits_to_f64(wl.bits(p[:h].contiguous())) for p in dc.peer_O])
        Lp = np.stack([Lr[:h]] + [p[:h].cpu().numpy().astype(np.float64) for p in dc.peer_LSE])
        Oref, Lref = oracle.merge_partials(Op, Lp)
        check_o_lse(fO.float().cpu().numpy().reshape(-1, dc.D), fL.cpu().numpy().reshape(-1), Oref.reshape(-1, dc.D), Lref.reshape(-1),
                    f"the master's step as one call, round {rnd}")


# ------------------------------------------------------------------ prefill: layouts and edge cases
@pytest.mark.parametrize("r_q", [0, 1, 2, 3])
def test_striped_all_offsets(esp, cuda, r_q):
    """Striped layout, every stripe as the local query: rows that see nothing in a shard (LSE = -inf) occur."""
    pc = wl.striped_prefill(f"striped-rq{r_q}", [600], 4, r_q, 4, 4, 10 + r_q, cuda)
    run_prefill_case(esp, pc)


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (4, 1), (16, 8)])
def test_gqa_varlen_batch_ragged(esp, cuda, Hq, Hkv):
    """Var-len batch with lengths that are not multiples of the 64-row KV tile or the 256-row Q tile."""
    pc = wl.striped_prefill(f"varlen-{Hq}/{Hkv}", [1, 63, 257, 300, 64], 2, 0, Hq, Hkv, 20, cuda)
    run_prefill_case(esp, pc)


def test_non_causal_and_tail(esp, cuda):
    pc = wl.contiguous_prefill("noncausal", 130, 0, [(0, 200), (200, 333)], 4, 4, 21, cuda, causal=False)
    run_prefill_case(esp, pc)


def test_unsorted_positions(esp, cuda):
    """Positions in arbitrary order (any token-level placement is legal): results must still be exact."""
    pc = wl.contiguous_prefill("shuffled", 300, 500, [(0, 450), (450, 800)], 4, 2, 22, cuda)
    g = torch.Generator(device="cpu").manual_seed(5)
    for s in pc.shards:
        perm = torch.randperm(s.kv_pos.numel(), generator=g).to(cuda)
        s.kv_pos = s.kv_pos[perm].contiguous()           # rows keep their data, positions are shuffled
    perm = torch.randperm(pc.q_pos.numel(), generator=g).to(cuda)
    pc.q_pos = pc.q_pos[perm].contiguous()
    run_prefill_case(esp, pc)


def test_query_chunk_before_every_key(esp, cuda):
    """A whole workgroup of queries sees nothing: O = 0, LSE = -inf everywhere, and the merge ignores it."""
    pc = wl.contiguous_prefill("allhidden", 64, 0, [(1000, 1200), (0, 64)], 4, 4, 23, cuda)
    parts = run_prefill_case(esp, pc)
    assert torch.isneginf(parts[0][1]).all() and (parts[0][0] == 0).all()


def test_prefill_is_deterministic(esp, cuda):
    pc = wl.striped_prefill("det", [700], 4, 1, 4, 4, 24, cuda)
    s = pc.shards[2]
    a = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale)
    b = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale)
    torch.cuda.synchronize()
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16)) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


# ------------------------------------------------------------------ decode: edge cases
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 4), (32, 8), (32, 32), (16, 16)])
def test_decode_heads_and_empty_requests(esp, cuda, Hq, Hkv):
    lens = [0, 1, 2, 3, 0, 65, 700, 5000, 0]
    dc = wl.decode_pool(f"decode-{Hq}/{Hkv}", lens, 8192, Hq, Hkv, 30, cuda, n_new=7, skip_new_every=3)
    O, LSE, kp, vp = run_decode_case(esp, dc)
    assert torch.isneginf(LSE[[0, 4, 8]]).all() and (O[[0, 4, 8]] == 0).all()
    oracle.kv_append(wl.bits(dc.new_k), wl.bits(dc.new_v), wl.host_i32(dc.new_slots), kp, vp)
    esp.esp_kv_append(dc.new_k, dc.new_v, dc.new_slots, dc.k_pool, dc.v_pool)
    torch.cuda.synchronize()
    assert np.array_equal(wl.bits(dc.k_pool), kp) and np.array_equal(wl.bits(dc.v_pool), vp)


@pytest.mark.parametrize("Hq,Hkv", [(32, 1), (4, 1), (8, 2), (12, 12), (24, 3), (40, 20), (5, 5), (48, 2), (9, 3), (40, 1),
                                    (66, 2), (32, 4), (64, 8), (7, 1)])
def test_decode_any_head_counts(esp, cuda, Hq, Hkv):
    """MQA, two KV heads, KV head counts that are no multiple of 4, query groups of every size: all on the matrix-core
    kernel (40 / 1 and 66 / 2 need a second chunk of columns, 7 / 1, 5 / 5 and 66 / 2 leave columns of a tile unused;
    32 / 4 and 64 / 8 are row-burst layouts that go there because of their groups of 8).  Empty requests, requests
    shorter than one tile, requests across several token ranges."""
    lens = [0, 1, 2, 3, 5, 0, 65, 700, 5000, 129, 0]
    dc = wl.decode_pool(f"decode-any-{Hq}/{Hkv}", lens, 8192, Hq, Hkv, 34, cuda, n_new=0)
    O, LSE, kp, vp = run_decode_case(esp, dc)
    assert torch.isneginf(LSE[[0, 5, 10]]).all() and (O[[0, 5, 10]] == 0).all()


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5, 6, 7])
def test_decode_randomized_layouts(esp, cuda, seed):
    """Drawn from a seeded generator: head layout (both kernels), number of requests, and a length mix with many
    requests shorter than a tile (several of them, and empty ones, inside one token range), a few of several thousand
    tokens (cut by range boundaries) and lengths at and around multiples of 32; then the fused decode + merge of the
    same case.  Every request and head against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv = [(32, 32), (8, 8), (32, 8), (16, 2), (5, 1), (36, 3), (64, 32), (33, 1)][seed]
    B = int(rng.integers(3, 90))
    kinds = rng.integers(0, 6, B)
    lens = np.where(kinds == 0, 0, np.where(kinds <= 2, rng.integers(1, 40, B),
                    np.where(kinds == 3, 32 * rng.integers(1, 9, B) + rng.integers(-1, 2, B), rng.integers(200, 6000, B))))
    if lens.sum() == 0:
        lens[0] = 77
    dc = wl.decode_pool(f"decode-random-{seed} ({Hq}/{Hkv})", lens.tolist(), 1 << 17, Hq, Hkv, 2000 + seed, cuda, n_new=0)
    O, LSE, kp, vp = run_decode_case(esp, dc)
    empty = torch.from_numpy(np.flatnonzero(lens == 0)).to(cuda)
    assert torch.isneginf(LSE[empty]).all() and (O[empty] == 0).all()
    Of, Lf = esp.esp_partial_attn_decode_merge(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, int(dc.lens.max()),
                                               list(dc.peer_O), list(dc.peer_LSE), softmax_scale=dc.scale)
    torch.cuda.synchronize()
    off, slots = wl.host_i32(dc.seq_offsets), wl.host_i32(dc.slot_idx)
    Or, Lr = oracle.partial_attn_decode_all(wl.bits(dc.q), kp, vp, slots, off, dc.scale)
    Op = np.stack([Or] + [oracle.bf16_bits_to_f64(wl.bits(t)) for t in dc.peer_O])
    Lp = np.stack([Lr] + [t.cpu().numpy().astype(np.float64) for t in dc.peer_LSE])
    Oref, Lref = oracle.merge_partials(Op, Lp)
    check_o_lse(Of.float().cpu().numpy().reshape(-1, dc.D), Lf.cpu().numpy().reshape(-1), Oref.reshape(-1, dc.D), Lref.reshape(-1),
                f"{dc.name} decode + merge in one call")


def test_decode_mqa_many_ranges_and_merge(esp, cuda):
    """MQA 32 / 1 at a size that is cut into many token ranges, then merged with peer partials."""
    lens = wl.lognormal_lengths(16, 6000, 10, 60000, 35)
    dc = wl.decode_pool("decode-mqa", lens, 1 << 18, 32, 1, 35, cuda, n_new=0)
    O, LSE, _, _ = run_decode_case(esp, dc)
    Om, Lm = esp.esp_merge_partials([O] + list(dc.peer_O), [LSE] + list(dc.peer_LSE))
    torch.cuda.synchronize()
    Op = np.stack([oracle.bf16_bits_to_f64(wl.bits(t)) for t in [O] + list(dc.peer_O)])
    Lp = np.stack([t.cpu().numpy().astype(np.float64) for t in [LSE] + list(dc.peer_LSE)])
    Oref, Lref = oracle.merge_partials(Op, Lp)
    check_o_lse(Om.float().cpu().numpy().reshape(-1, 128), Lm.cpu().numpy().reshape(-1), Oref.reshape(-1, 128), Lref.reshape(-1), "MQA merge")


@pytest.mark.parametrize("Hq,Hkv", [(8, 4), (6, 3), (32, 32)])
def test_decode_merged_with_the_peers_partials_in_one_pass(esp, cuda, Hq, Hkv):
    """The master's step of a multi-master decode (Sec. 4.2): local partial attention and the combination with the
    peers' results in one call, against the oracle's merge of ITS OWN local partial (fp64, never rounded) with the same
    peer arrays.  Covers a request the master holds nothing of, a peer that holds nothing of a request (LSE = -inf, O
    garbage), a request nobody holds anything of, and n_peers = 0 (bit-identical to the plain call)."""
    lens = [300, 0, 1500, 64, 0, 2200, 9, 1]
    dc = wl.decode_pool(f"decode-merge-{Hq}/{Hkv}", lens, 8192, Hq, Hkv, 37, cuda, n_new=0)
    O_loc, L_loc, kp, vp = run_decode_case(esp, dc)
    peers_O = [t.clone() for t in dc.peer_O]; peers_L = [t.clone() for t in dc.peer_LSE]
    peers_L[1][2] = float("-inf"); peers_O[1][2] = float("nan")          # a peer without tokens of request 2
    for t_o, t_l in zip(peers_O, peers_L):                                # nobody holds a token of request 4
        t_l[4] = float("-inf"); t_o[4] = float("nan")
    O, LSE = esp.esp_partial_attn_decode_merge(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, int(dc.lens.max()),
                                               peers_O, peers_L, softmax_scale=dc.scale)
    torch.cuda.synchronize()
    off, slots = wl.host_i32(dc.seq_offsets), wl.host_i32(dc.slot_idx)
    Or, Lr = oracle.partial_attn_decode_all(wl.bits(dc.q), kp, vp, slots, off, dc.scale)
    Op = np.stack([Or] + [np.nan_to_num(oracle.bf16_bits_to_f64(wl.bits(t)), nan=0.0) for t in peers_O])
    Lp = np.stack([Lr] + [t.cpu().numpy().astype(np.float64) for t in peers_L])
    Oref, Lref = oracle.merge_partials(Op, Lp)
    check_o_lse(O.float().cpu().numpy().reshape(-1, dc.D), LSE.cpu().numpy().reshape(-1), Oref.reshape(-1, dc.D),
                Lref.reshape(-1), f"{dc.name} local + {len(peers_O)} peers")
    assert torch.isneginf(LSE[4]).all() and (O[4] == 0).all()
    assert torch.isfinite(O.float()).all()
    # request 1: the master holds nothing, so the result is the peers' combination alone
    Om, Lm = esp.esp_merge_partials([t[1:2].contiguous() for t in peers_O], [t[1:2].contiguous() for t in peers_L])
    torch.cuda.synchronize()
    assert torch.allclose(O[1:2].float(), Om.float(), rtol=2 ** -7, atol=1e-6) and torch.allclose(LSE[1:2], Lm, rtol=1e-6, atol=1e-6)
    # no peers: the plain call
    O0, L0 = esp.esp_partial_attn_decode_merge(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, int(dc.lens.max()),
                                               [], [], softmax_scale=dc.scale)
    torch.cuda.synchronize()
    assert torch.equal(O0.view(torch.int16), O_loc.view(torch.int16)) and torch.equal(L0.view(torch.int32), L_loc.view(torch.int32))
    # an output that overlaps a peer's array is refused
    with pytest.raises(esp.EspError) as e:
        esp.esp_partial_attn_decode_merge(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, int(dc.lens.max()),
                                          peers_O, peers_L, softmax_scale=dc.scale, O=peers_O[0])
    assert e.value.status == esp.ESP_ERR_INVALID_ARG


def test_decode_many_ranges(esp, cuda):
    """Enough tokens that the token list is cut into many ranges, with requests spanning several of them."""
    lens = wl.lognormal_lengths(24, 3000, 10, 40000, 31)
    dc = wl.decode_pool("decode-ranges", lens, 1 << 18, 8, 8, 31, cuda, n_new=0)
    run_decode_case(esp, dc)


def test_decode_is_deterministic(esp, cuda):
    dc = wl.decode_pool("decode-det", [900, 33, 4000], 8192, 8, 4, 32, cuda, n_new=0)
    a = esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, 4000)
    b = esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, 4000)
    torch.cuda.synchronize()
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16)) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


# ------------------------------------------------------------------ merge kernel on its own
@pytest.mark.parametrize("P", [1, 2, 4, 16])
def test_merge_kernel(esp, cuda, P):
    g = torch.Generator(device=cuda).manual_seed(40 + P)
    T, H = 37, 8
    Os = [wl.randn_bf16((T, H, 128), g, cuda) for _ in range(P)]
    Ls = [torch.randn((T, H), generator=g, device=cuda) * 4 for _ in range(P)]
    if P > 1:
        Ls[1][::3] = float("-inf")                       # an empty partial here and there
        for L in Ls:
            L[5] = float("-inf")                         # a row that is empty in every partial
        Os[1][::3] = float("nan")                        # garbage in an empty partial must not leak
    say(f"merge P={P}")
    Om, Lm = esp.esp_merge_partials(Os, Ls)
    torch.cuda.synchronize()
    Op = np.stack([oracle.bf16_bits_to_f64(wl.bits(o)) for o in Os]); Lp = np.stack([l.cpu().numpy().astype(np.float64) for l in Ls])
    Op = np.nan_to_num(Op, nan=0.0)
    Oref, Lref = oracle.merge_partials(Op, Lp)
    check_o_lse(Om.float().cpu().numpy().reshape(-1, 128), Lm.cpu().numpy().reshape(-1), Oref.reshape(-1, 128), Lref.reshape(-1),
                f"merge P={P}")
    # in place (O aliases the first partial) and without LSE output
    O0 = Os[0].clone()
    esp.esp_merge_partials([O0] + Os[1:], Ls, O=O0, want_lse=False)
    torch.cuda.synchronize()
    assert torch.equal(O0.view(torch.int16), Om.view(torch.int16))


def test_device_side_errors_are_reported_not_thrown(esp, cuda):
    q = torch.zeros((4, 4, 64), dtype=torch.bfloat16, device=cuda)
    with pytest.raises(esp.EspError) as e:
        esp.esp_merge_partials([q], [torch.zeros((4, 4), device=cuda)])
    assert e.value.status == esp.ESP_ERR_UNSUPPORTED


def test_request_without_keys_in_this_shard(esp, cuda):
    """Multi-request batch where the first request holds no row of the shard (cu_kv repeats an offset)."""
    pc = wl.striped_prefill("nokeys", [100, 80], 2, 0, 4, 4, 25, cuda)
    s = pc.shards[1]
    k, v, kv_pos = s.k[100:].contiguous(), s.v[100:].contiguous(), s.kv_pos[100:].contiguous()
    cu_kv = torch.tensor([0, 0, 80], dtype=torch.int32, device=cuda)
    say("nokeys: request 0 has queries but no keys")
    O, LSE = esp.esp_partial_attn_prefill(pc.q, k, v, pc.q_pos, kv_pos, pc.cu_q, cu_kv, 100, 80, softmax_scale=pc.scale)
    torch.cuda.synchronize()
    assert torch.isneginf(LSE[:100]).all() and (O[:100] == 0).all()
    rows = np.repeat(np.arange(100, 180, dtype=np.int64), 4); heads = np.tile(np.arange(4, dtype=np.int64), 80)
    Or, Lr = oracle.partial_attn(wl.bits(pc.q), wl.bits(k), wl.bits(v), wl.host_i32(pc.q_pos), wl.host_i32(kv_pos), pc.scale,
                                 True, rows, heads)
    check_o_lse(O[100:].float().cpu().numpy().reshape(-1, 128), LSE[100:].cpu().numpy().reshape(-1), Or, Lr, "nokeys")


@pytest.mark.parametrize("Hq,Hkv", [(32, 4), (64, 64)])
def test_decode_wide_groups_and_many_head_blocks(esp, cuda, Hq, Hkv):
    """G = 8 query heads per KV head; 64 KV heads = 16 one-KiB head blocks (two workgroups along y)."""
    dc = wl.decode_pool(f"decode-{Hq}/{Hkv}", [17, 0, 2049, 300], 4096, Hq, Hkv, 33, cuda, n_new=0)
    run_decode_case(esp, dc)


def test_prefill_shard_entirely_in_the_future(esp, cuda):
    """No tile of the shard is visible to any row: nothing is swept, O = 0 and LSE = -inf everywhere."""
    pc = wl.contiguous_prefill("future", 300, 0, [(5000, 5500)], 4, 4, 26, cuda)
    s = pc.shards[0]
    say("future shard")
    O, LSE = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale)
    torch.cuda.synchronize()
    assert torch.isneginf(LSE).all() and (O == 0).all()


def test_prefill_empty_shard_and_large_positions(esp, cuda):
    """Tkv = 0 (an instance that holds nothing of this request) and positions near the top of the int32 range."""
    pc = wl.contiguous_prefill("big-positions", 70, 2**31 - 400, [(2**31 - 600, 2**31 - 300)], 4, 4, 27, cuda)
    run_prefill_case(esp, pc)
    empty_k = torch.empty((0, 4, 128), dtype=torch.bfloat16, device=cuda)
    empty_p = torch.empty((0,), dtype=torch.int32, device=cuda)
    O, LSE = esp.esp_partial_attn_prefill(pc.q, empty_k, empty_k, pc.q_pos, empty_p, softmax_scale=pc.scale)
    torch.cuda.synchronize()
    assert torch.isneginf(LSE).all() and (O == 0).all()


def test_prefill_large_scores_refresh_the_softmax_offset(esp, cuda):
    """Scores far above the first tile's (a late 'attention sink') and far below it: the optimistic offset has to
    be refreshed by the sum check, and tiny probabilities must not be lost."""
    pc = wl.contiguous_prefill("sink", 64, 1000, [(0, 640)], 4, 4, 28, cuda, causal=False)
    s = pc.shards[0]
    s.k[300:303] *= 40.0          # a few keys with very large scores in tile 4
    s.k[0:64] *= 0.01
    run_prefill_case(esp, pc)
    pc2 = wl.contiguous_prefill("sink-first", 64, 1000, [(0, 640)], 4, 4, 29, cuda, causal=False)
    pc2.shards[0].k[3:5] *= 60.0  # the huge scores come first, everything later is ~2^-80 of them
    run_prefill_case(esp, pc2)


@pytest.mark.parametrize("late_keys", [((300, 1.5),), ((523, 1.5),), ((300, 1.5), (523, 2.5), (1004, 3.5))])
def test_prefill_offset_moves_for_the_whole_row_when_one_half_sees_the_large_key(esp, cuda, late_keys):
    """A query row is held by two lanes, each with half of a tile's keys (key index % 8 < 4 in one, >= 4 in the
    other).  A late key whose score lies 2^36 above everything before it makes the probability sum of ITS half
    exceed the limit that moves the softmax offset, while the other half's sum stays small: the offset, and
    everything rescaled with it, must still move for the whole row.  Nothing here leaves the range of the
    optimistic pass (every tile sum stays below 2^100 of the offset in use), so the pipelined path itself is what
    is compared with the oracle, not the exact re-sweep.  Keys 300 and 1004 fall into one half, 523 into the other;
    with all three the offset moves three times (by 36, 25 and 25 bits)."""
    Tq, Tkv = 300, 1100
    pc = wl.contiguous_prefill("half-row-offset", Tq, 2000, [(0, Tkv)], 4, 2, 43, cuda, causal=False)
    s = pc.shards[0]
    u = torch.ones(pc.D, dtype=torch.bfloat16, device=cuda)
    pc.q[:] = (pc.q.float() * 0.05 + 1.5).to(torch.bfloat16)      # every row close to 1.5 * u
    s.k[:] = (s.k.float() * 0.05).to(torch.bfloat16)              # scores near 0 ...
    for idx, c in late_keys:
        s.k[idx] = c * u                                           # ... but for these: 1.5 * c * 128 * scale = 17 c nats
    assert [i % 8 >= 4 for i, _ in late_keys] in ([True], [False], [True, False, True])
    run_prefill_case(esp, pc)


@pytest.mark.gpu
@pytest.mark.parametrize("causal", [False, True])
def test_prefill_scores_beyond_the_optimistic_range_take_the_exact_sweep(esp, cuda, causal):
    """A key whose score lies ~2^400 above every earlier one, for every query row, arriving in a late tile: the
    probabilities of the pipelined pass overflow there, so the kernel must notice and redo the rows with its plain
    sweep (a result from the optimistic pass alone would be NaN or far off).  Also a row set whose scores all lie
    ~2^300 below zero, where a probability taken against the stand-in offset underflows.  Ragged tail included."""
    Tq, Tkv = 300, 1000
    pc = wl.contiguous_prefill("overflow", Tq, 1000, [(0, Tkv)], 4, 2, 41, cuda, causal=causal)
    s = pc.shards[0]
    u = torch.ones(pc.D, dtype=torch.bfloat16, device=cuda)
    pc.q[:] = (pc.q.float() * 0.05 + 1.5).to(torch.bfloat16)      # every row close to 1.5 * u
    s.k[:] = (s.k.float() * 0.05).to(torch.bfloat16)
    s.k[777] = 16.0 * u                                            # score 1.5*16*128*scale = 271 nats above the rest
    s.k[990] = 15.5 * u                                            # close second, in the ragged last tile
    run_prefill_case(esp, pc)
    pc2 = wl.contiguous_prefill("underflow", Tq, 1000, [(0, Tkv)], 4, 2, 42, cuda, causal=causal)
    s2 = pc2.shards[0]
    pc2.q[:] = (pc2.q.float() * 0.05 + 1.5).to(torch.bfloat16)
    s2.k[:] = (s2.k.float() * 0.05 - 12.0).to(torch.bfloat16)      # every score about -200 nats
    s2.k[100:104] = (s2.k[100:104].float() + 24.0).to(torch.bfloat16)   # a few keys 400 nats above those, in tile 1
    run_prefill_case(esp, pc2)


@pytest.mark.gpu
@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (8, 8)])
def test_prefill_more_items_than_workgroups(esp, cuda, Hq, Hkv):
    """More (query tile, head) items than the launch has workgroups, so every persistent workgroup works through
    several items, back and forth; with 8 KV heads the items are split by XCD, otherwise dealt over all workgroups.
    Short KV keeps the oracle cheap; every query row is checked."""
    Tq = 256 * 72 + 40                                  # 73 query tiles (the last one ragged) x Hq heads > 256 items
    pc = wl.contiguous_prefill(f"many-items-{Hq}/{Hkv}", Tq, 200, [(0, 330), (330, 700)], Hq, Hkv, 51, cuda)
    pc.q_pos[:] = seeded_positions(Tq, 900, 901, cuda)       # every tile sees a different part
    run_prefill_case(esp, pc)


def test_debug_validation_of_index_arrays(esp, cuda):
    """esp_debug_set_validate(1) (what ESP_DEBUG_VALIDATE=1 in the environment sets at load time): slots outside the pool, slots named twice, offsets that decrease or do not end at the row
    count are refused with ESP_ERR_INVALID_ARG before anything is launched; sound arrays pass and give the usual result."""
    dc = wl.config1_decode(cuda)
    max_len = int(dc.lens.max())
    was = esp.esp_debug_set_validate(True)
    try:
        _validation_cases(esp, cuda, dc, max_len)
    finally:
        esp.esp_debug_set_validate(was)


def _validation_cases(esp, cuda, dc, max_len):
    O, L = esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, max_len, softmax_scale=dc.scale)
    bad = dc.slot_idx.clone(); bad[17] = dc.num_slots
    with pytest.raises(esp.EspError) as e:
        esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, bad, dc.seq_offsets, max_len, softmax_scale=dc.scale)
    assert e.value.status == -1 and "slot_idx[17]" in str(e.value)
    bad = dc.slot_idx.clone(); bad[3] = -1
    with pytest.raises(esp.EspError):
        esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, bad, dc.seq_offsets, max_len, softmax_scale=dc.scale)
    off = dc.seq_offsets.clone(); off[2] = off[1] - 1
    with pytest.raises(esp.EspError) as e:
        esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, off, max_len, softmax_scale=dc.scale)
    assert "decrease" in str(e.value)
    with pytest.raises(esp.EspError):                              # a request longer than the stated maximum
        esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, max_len - 1, softmax_scale=dc.scale)
    # append: distinct non-negative slots below the pool size; negative ones mean "not kept"
    kp, vp = dc.k_pool.clone(), dc.v_pool.clone()
    twice = dc.new_slots.clone(); twice[1] = twice[0]
    with pytest.raises(esp.EspError) as e:
        esp.esp_kv_append(dc.new_k, dc.new_v, twice, kp, vp)
    assert "twice" in str(e.value)
    high = dc.new_slots.clone(); high[0] = dc.num_slots + 5
    with pytest.raises(esp.EspError):
        esp.esp_kv_append(dc.new_k, dc.new_v, high, kp, vp)
    assert torch.equal(kp, dc.k_pool) and torch.equal(vp, dc.v_pool)      # nothing was written by the refused calls
    skipped = dc.new_slots.clone(); skipped[:2] = -1
    esp.esp_kv_append(dc.new_k, dc.new_v, skipped, kp, vp)
    # prefill: offsets of a var-len batch
    pc = wl.striped_prefill("validate", [70, 130], 2, 0, 4, 4, 90, cuda)
    s0 = pc.shards[0]
    esp.esp_partial_attn_prefill(pc.q, s0.k, s0.v, pc.q_pos, s0.kv_pos, pc.cu_q, s0.cu_kv, pc.max_q, s0.max_kv, softmax_scale=pc.scale)
    short = s0.cu_kv.clone(); short[-1] -= 1
    with pytest.raises(esp.EspError):
        esp.esp_partial_attn_prefill(pc.q, s0.k, s0.v, pc.q_pos, s0.kv_pos, pc.cu_q, short, pc.max_q, s0.max_kv, softmax_scale=pc.scale)
    torch.cuda.synchronize()
    esp.esp_debug_set_validate(False)
    O2, L2 = esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, max_len, softmax_scale=dc.scale)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(L, L2)


def pool_image(rng, shard, num_slots):
    """Host pool arrays holding the shard's rows at random distinct slots (built by the oracle's own scatter), plus noise
    in every other slot; returns (k_pool, v_pool, slots) as numpy arrays."""
    kb, vb = wl.bits(shard.k), wl.bits(shard.v)
    kp = rng.integers(0, 65536, (num_slots,) + kb.shape[1:]).astype(np.uint16); vp = rng.integers(0, 65536, kp.shape).astype(np.uint16)
    kp &= 0x3FFF; vp &= 0x3FFF                                   # noise, but finite bf16 values
    slots = rng.permutation(num_slots)[: kb.shape[0]].astype(np.int32)
    oracle.kv_append(kb, vb, slots, kp, vp)
    return kp, vp, slots


def test_kv_gather_bit_exact(esp, cuda):
    """Every gathered row against the oracle, bit for bit; slots outside the pool (negative, too large) give zero rows."""
    rng = np.random.default_rng(31)
    S, T, Hkv = 5000, 3001, 4
    kp = rng.integers(0, 65536, (S, Hkv, 128)).astype(np.uint16); vp = rng.integers(0, 65536, (S, Hkv, 128)).astype(np.uint16)
    slots = rng.integers(0, S, T).astype(np.int32)                # repeats allowed
    slots[::11] = -1; slots[5::97] = S; slots[7::101] = S + 12345
    say(f"gather: S={S} T={T} Hkv={Hkv}")
    to = lambda a: torch.from_numpy(a.view(np.int16)).to(cuda).view(torch.bfloat16)
    k, v = esp.esp_kv_gather(to(kp), to(vp), torch.from_numpy(slots).to(cuda))
    torch.cuda.synchronize()
    kr, vr = oracle.kv_gather(kp, vp, slots)
    assert np.array_equal(wl.bits(k), kr) and np.array_equal(wl.bits(v), vr)
    k0, v0 = esp.esp_kv_gather(to(kp), to(vp), torch.zeros(0, dtype=torch.int32, device=cuda))
    assert k0.shape == (0, Hkv, 128) and v0.shape == (0, Hkv, 128)


@pytest.mark.parametrize("layout", ["one-request", "var-len-gqa"])
def test_prefill_over_pool_resident_rows(esp, cuda, layout):
    """The shard's rows live in a token pool at random slots; the call over (pool, slot list) must give what the
    oracle gives on its own gathered rows.  Every query row is checked."""
    rng = np.random.default_rng(41)
    if layout == "one-request":
        pc = wl.contiguous_prefill("pool-1req", 300, 400, [(0, 700)], 4, 4, 61, cuda)
    else:
        pc = wl.striped_prefill("pool-varlen", [70, 257, 130], 2, 1, 8, 2, 62, cuda)
    qb, qp = wl.bits(pc.q), wl.host_i32(pc.q_pos)
    cu_q = wl.host_i32(pc.cu_q)
    Tq, Hq, D = pc.q.shape
    rows = np.repeat(np.arange(Tq, dtype=np.int64), Hq); heads = np.tile(np.arange(Hq, dtype=np.int64), Tq)
    req_of_row = np.searchsorted(cu_q, np.arange(Tq), side="right") - 1
    single = pc.batch == 1
    to = lambda a: torch.from_numpy(a.view(np.int16)).to(cuda).view(torch.bfloat16)
    for si, s in enumerate(pc.shards):
        S = 2048
        kp, vp, slots = pool_image(rng, s, S)
        say(f"{pc.name} shard {si}: Tq={Tq} Tkv={len(slots)} pool={S} Hq={Hq} Hkv={pc.Hkv} batch={pc.batch}")
        O = torch.full_like(pc.q, float("nan")); LSE = torch.full((Tq, Hq), float("nan"), dtype=torch.float32, device=cuda)
        esp.esp_partial_attn_prefill_pool(pc.q, to(kp), to(vp), torch.from_numpy(slots).to(cuda), pc.q_pos, s.kv_pos,
                                          None if single else pc.cu_q, None if single else s.cu_kv,
                                          None if single else pc.max_q, None if single else s.max_kv,
                                          softmax_scale=pc.scale, causal=pc.causal, O=O, LSE=LSE)
        torch.cuda.synchronize()
        kg, vg = oracle.kv_gather(kp, vp, slots)
        cu_kv = wl.host_i32(s.cu_kv)
        lo, hi = cu_kv[req_of_row[rows]], cu_kv[req_of_row[rows] + 1]
        Or, Lr = oracle.partial_attn(qb, kg, vg, qp, wl.host_i32(s.kv_pos), pc.scale, pc.causal, rows, heads, lo, hi)
        check_o_lse(O.float().cpu().numpy().reshape(-1, D), LSE.cpu().numpy().reshape(-1), Or, Lr, f"{pc.name} shard {si}")


def run_pool_direct_case(esp, pc, seed, spare_slots=777):
    """Every shard of the case is laid out in a pool at random distinct slots (noise everywhere else) and attended by
    the call whose tile transfers read the pool rows themselves; bf16 and fp32 output, every query row against the
    oracle on ITS OWN gathered rows; and bit for bit against the dense call on the same rows (same tiles, same order
    of operations: only where a row comes from differs)."""
    rng = np.random.default_rng(seed)
    qb, qp = wl.bits(pc.q), wl.host_i32(pc.q_pos)
    cu_q = wl.host_i32(pc.cu_q)
    Tq, Hq, D = pc.q.shape
    rows = np.repeat(np.arange(Tq, dtype=np.int64), Hq); heads = np.tile(np.arange(Hq, dtype=np.int64), Tq)
    req_of_row = np.searchsorted(cu_q, np.arange(Tq), side="right") - 1
    single = pc.batch == 1
    to = lambda a: torch.from_numpy(a.view(np.int16)).to(pc.q.device).view(torch.bfloat16)
    for si, s in enumerate(pc.shards):
        S = 2 * s.k.shape[0] + spare_slots
        kp, vp, slots = pool_image(rng, s, S)
        say(f"{pc.name} shard {si} from the pool: Tq={Tq} Tkv={len(slots)} pool={S} Hq={Hq} Hkv={pc.Hkv} batch={pc.batch} causal={pc.causal}")
        args = (pc.q, to(kp), to(vp), torch.from_numpy(slots).to(pc.q.device), pc.q_pos, s.kv_pos,
                None if single else pc.cu_q, None if single else s.cu_kv, None if single else pc.max_q, None if single else s.max_kv)
        O = torch.full_like(pc.q, float("nan")); LSE = torch.full((Tq, Hq), float("nan"), dtype=torch.float32, device=pc.q.device)
        esp.esp_partial_attn_prefill_pool_direct(*args, softmax_scale=pc.scale, causal=pc.causal, O=O, LSE=LSE)
        O32 = torch.full(pc.q.shape, float("nan"), dtype=torch.float32, device=pc.q.device); LSE32 = torch.full_like(LSE, float("nan"))
        esp.esp_partial_attn_prefill_pool_direct(*args, softmax_scale=pc.scale, causal=pc.causal, O=O32, LSE=LSE32)
        Od, Ld = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, *args[6:], softmax_scale=pc.scale, causal=pc.causal)
        torch.cuda.synchronize()
        if Tq > 0:
            kg, vg = oracle.kv_gather(kp, vp, slots)
            assert np.array_equal(kg, wl.bits(s.k)) and np.array_equal(vg, wl.bits(s.v))
            cu_kv = wl.host_i32(s.cu_kv)
            lo, hi = cu_kv[req_of_row[rows]], cu_kv[req_of_row[rows] + 1]
            Or, Lr = oracle.partial_attn(qb, kg, vg, qp, wl.host_i32(s.kv_pos), pc.scale, pc.causal, rows, heads, lo, hi)
            check_o_lse(O.float().cpu().numpy().reshape(-1, D), LSE.cpu().numpy().reshape(-1), Or, Lr, f"{pc.name} shard {si} from the pool")
            check_o_lse(O32.cpu().numpy().reshape(-1, D), LSE32.cpu().numpy().reshape(-1), Or, Lr, f"{pc.name} shard {si} from the pool (fp32 out)")
        assert torch.equal(O.view(torch.int16), Od.view(torch.int16)) and torch.equal(LSE.view(torch.int32), Ld.view(torch.int32))
        assert torch.equal(O32.to(torch.bfloat16).view(torch.int16), O.view(torch.int16)) and torch.equal(LSE32.view(torch.int32), LSE.view(torch.int32))


@pytest.mark.gpu
@pytest.mark.parametrize("layout", ["one-request", "var-len-gqa"])
def test_prefill_reading_pool_rows_in_the_tile_transfers(esp, cuda, layout):
    if layout == "one-request":
        run_pool_direct_case(esp, wl.contiguous_prefill("pool-direct-1req", 300, 400, [(0, 700)], 4, 4, 61, cuda), 141)
    else:
        run_pool_direct_case(esp, wl.striped_prefill("pool-direct-varlen", [70, 257, 130, 1, 64], 2, 1, 8, 2, 62, cuda), 142)


@pytest.mark.gpu
def test_prefill_from_pool_long_shard_ragged_tail_and_short_shards(esp, cuda):
    """Many tiles (the slot ring wraps many times; plain and masked iterations; tiles that only some wavefronts see),
    a ragged last tile, and shards of 1 .. 5 tiles (every branch of the start-up with few tiles)."""
    run_pool_direct_case(esp, wl.contiguous_prefill("pool-direct-long", 700, 3000, [(0, 3700 - 29)], 4, 2, 63, cuda), 143)
    for n in (1, 63, 64, 65, 128, 200, 256, 257, 320):
        run_pool_direct_case(esp, wl.contiguous_prefill(f"pool-direct-{n}", 130, 400, [(0, n)], 2, 2, 64 + n, cuda), 144 + n, spare_slots=50)


@pytest.mark.gpu
def test_prefill_from_pool_non_causal_unsorted_and_hidden_shards(esp, cuda):
    run_pool_direct_case(esp, wl.contiguous_prefill("pool-direct-noncausal", 100, 0, [(0, 1000)], 4, 4, 65, cuda, causal=False), 151)
    pc = wl.contiguous_prefill("pool-direct-unsorted", 200, 500, [(0, 900)], 4, 4, 66, cuda)
    g = torch.Generator(device="cpu").manual_seed(66)
    pc.q_pos[:] = torch.randint(0, 1500, (200,), generator=g, dtype=torch.int32).to(cuda)
    pc.shards[0].kv_pos[:] = torch.randint(0, 1500, (900,), generator=g, dtype=torch.int32).to(cuda)
    run_pool_direct_case(esp, pc, 152)
    # a shard that lies entirely after the queries: nothing visible, no tile is swept
    run_pool_direct_case(esp, wl.contiguous_prefill("pool-direct-future", 100, 0, [(5000, 5600)], 4, 4, 67, cuda), 153)


@pytest.mark.gpu
@pytest.mark.parametrize("causal", [False, True])
def test_prefill_from_pool_exact_sweep(esp, cuda, causal):
    """The rows' scores leave the range of the optimistic pass: the plain re-sweep also has to find its rows by slot."""
    Tq, Tkv = 300, 1000
    pc = wl.contiguous_prefill("pool-direct-overflow", Tq, 1000, [(0, Tkv)], 4, 2, 41, cuda, causal=causal)
    s = pc.shards[0]
    u = torch.ones(pc.D, dtype=torch.bfloat16, device=cuda)
    pc.q[:] = (pc.q.float() * 0.05 + 1.5).to(torch.bfloat16)
    s.k[:] = (s.k.float() * 0.05).to(torch.bfloat16)
    s.k[777] = 16.0 * u
    s.k[990] = 15.5 * u
    run_pool_direct_case(esp, pc, 154)


@pytest.mark.gpu
def test_prefill_from_pool_more_items_than_workgroups_and_empty_shard(esp, cuda):
    Tq = 256 * 40 + 7
    pc = wl.contiguous_prefill("pool-direct-many-items", Tq, 150, [(0, 400)], 8, 8, 68, cuda)
    pc.q_pos[:] = seeded_positions(Tq, 800, 902, cuda)
    run_pool_direct_case(esp, pc, 155)
    # no shard rows at all: O = 0, LSE = -inf, no slot is read
    q = wl.randn_bf16((70, 4, 128), torch.Generator(device=cuda).manual_seed(3), cuda)
    pool = torch.zeros((16, 2, 128), dtype=torch.bfloat16, device=cuda)
    none = torch.zeros(0, dtype=torch.int32, device=cuda)
    O, LSE = esp.esp_partial_attn_prefill_pool_direct(q, pool, pool, none, torch.arange(70, dtype=torch.int32, device=cuda), none)
    torch.cuda.synchronize()
    assert torch.isneginf(LSE).all() and (O == 0).all()


@pytest.mark.gpu
@pytest.mark.parametrize("fill", ["zeros", "ones", "random"])
def test_prefill_workspace_contents_do_not_matter(esp, cuda, fill):
    """The workspace holds the counter of the item pool, which the call neither expects cleared nor clears: whatever
    the block holds (nothing, all ones, noise, the count of the previous call: both shards reuse it), every item is
    worked on exactly once.  More items than workgroups, so that the pool is in use; every query row is checked."""
    Tq = 256 * 40 + 7
    pc = wl.contiguous_prefill(f"workspace-{fill}", Tq, 150, [(0, 400), (400, 650)], 8, 8, 77, cuda)
    pc.q_pos[:] = seeded_positions(Tq, 800, 903, cuda)
    nbytes = esp.esp_prefill_workspace_bytes(Tq, 400, 1, 8, 8, 128)
    if fill == "zeros":
        ws = torch.zeros(nbytes, dtype=torch.uint8, device=cuda)
    elif fill == "ones":
        ws = torch.full((nbytes,), 255, dtype=torch.uint8, device=cuda)
    else:
        ws = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=cuda, generator=torch.Generator(device=cuda).manual_seed(5))
    run_prefill_case(esp, pc, workspace=ws)


@pytest.mark.gpu
def test_prefill_calls_on_two_streams_with_a_workspace_each(esp, cuda):
    """Two calls that may run at the same time (two streams of default priority), each with its own workspace, as the
    header asks: both must give what they give alone (bit for bit; the single calls are checked against the oracle by
    the other tests).  More items than workgroups in both, so that both use their item pool."""
    cases = []
    for k, (Tq, Hq, Hkv) in enumerate([(256 * 40 + 7, 8, 8), (256 * 36 + 100, 16, 8)]):
        pc = wl.contiguous_prefill(f"two-streams-{k}", Tq, 150, [(0, 400)], Hq, Hkv, 81 + k, cuda)
        pc.q_pos[:] = seeded_positions(Tq, 800, 904, cuda)
        s = pc.shards[0]
        O_ref, L_ref = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale)
        ws = torch.empty(esp.esp_prefill_workspace_bytes(Tq, 400, 1, Hq, Hkv, 128), dtype=torch.uint8, device=cuda)
        cases.append((pc, s, O_ref, L_ref, ws, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(3):
        outs = []
        for pc, s, O_ref, L_ref, ws, st in cases:
            O = torch.full_like(O_ref, float("nan")); L = torch.full_like(L_ref, float("nan"))
            st.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(st):
                esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale, O=O, LSE=L, workspace=ws)
            outs.append((O, L))
        torch.cuda.synchronize()
        for (pc, s, O_ref, L_ref, ws, st), (O, L) in zip(cases, outs):
            assert torch.equal(O.view(torch.int16), O_ref.view(torch.int16)) and torch.equal(L.view(torch.int32), L_ref.view(torch.int32)), (pc.name, rep)


@pytest.mark.gpu
def test_prefill_replayed_from_a_captured_graph(esp, cuda):
    """A prefill call recorded into a graph and replayed: the replays carry the recorded launch's arguments, counters'
    tag included, and must still work every item exactly once.  Replays alternate with eager calls on the same
    workspace and with host synchronisation; every replay is compared bit for bit with the eager result (which the
    other tests check against the oracle).  More items than workgroups, so that the item pool is in use."""
    Tq = 256 * 40 + 7
    pc = wl.contiguous_prefill("graph-replay", Tq, 150, [(0, 400)], 8, 8, 78, cuda)
    pc.q_pos[:] = seeded_positions(Tq, 800, 905, cuda)
    s = pc.shards[0]
    ws = torch.empty(esp.esp_prefill_workspace_bytes(Tq, 400, 1, 8, 8, 128), dtype=torch.uint8, device=cuda)
    nan_like = lambda t: torch.full_like(t, float("nan"))
    O_ref, L_ref = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale, workspace=ws)
    torch.cuda.synchronize()
    assert not torch.isnan(O_ref.float()).any() and not torch.isnan(L_ref).any()
    O_g, L_g = nan_like(O_ref), nan_like(L_ref)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                  # warm-up on the capture's side stream, as torch asks
        esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale, O=O_g, LSE=L_g, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale, O=O_g, LSE=L_g, workspace=ws)
    for rep in range(4):
        say(f"graph replay {rep}")
        O_g.copy_(nan_like(O_g)); L_g.copy_(nan_like(L_g))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(O_g.view(torch.int16), O_ref.view(torch.int16)) and torch.equal(L_g.view(torch.int32), L_ref.view(torch.int32)), f"replay {rep}"
        if rep % 2 == 0:                                           # an eager call in between, same workspace
            O_e, L_e = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, softmax_scale=pc.scale, workspace=ws)
            torch.cuda.synchronize()
            assert torch.equal(O_e.view(torch.int16), O_ref.view(torch.int16))


@pytest.mark.gpu
@pytest.mark.parametrize("seed", list(range(10)))
def test_prefill_randomized_layouts(esp, cuda, seed):
    """Seeded random layouts: head counts, batch, ragged lengths up to several query tiles and a dozen KV tiles,
    striped shards with a random stripe offset, sometimes shuffled positions or no mask.  Every row is checked."""
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv = [(4, 4), (8, 2), (4, 1), (16, 8), (32, 8), (8, 8)][int(rng.integers(0, 6))]
    n_req = int(rng.integers(1, 5))
    chunks = [int(rng.integers(1, 900)) for _ in range(n_req)]
    n_shards = int(rng.integers(1, 4))
    pc = wl.striped_prefill(f"rand{seed}-{Hq}/{Hkv}", chunks, n_shards, int(rng.integers(0, n_shards)), Hq, Hkv, 2000 + seed, cuda)
    mode = int(rng.integers(0, 4))
    if mode == 1:                                   # positions shuffled inside every request (rows keep their data)
        g = torch.Generator(device="cpu").manual_seed(seed)
        cu = wl.host_i32(pc.cu_q)
        for t in [pc] + pc.shards:
            pos = t.q_pos if t is pc else t.kv_pos
            for r in range(n_req):
                lo, hi = int(cu[r]), int(cu[r + 1])
                pos[lo:hi] = pos[lo:hi][torch.randperm(hi - lo, generator=g).to(cuda)]
    elif mode == 2:
        pc.causal = False
    say(f"layout: chunks={chunks} shards={n_shards} mode={mode}")
    run_prefill_case(esp, pc)


# ------------------------------------------------------------------ prefill that keeps rows of the shard on the way
def run_retain_case(esp, pc, seed, keep_fraction=0.7, out_dtype=torch.bfloat16):
    """Every shard through esp_partial_attn_prefill_retain with seeded slots (distinct; some rows not kept) into a pool
    full of noise: O and LSE must match the oracle (and agree with esp_partial_attn_prefill); the pool
    must be, bit for bit, what the oracle's scatter makes of the same noise."""
    rng = np.random.default_rng(seed)
    qb, qp = wl.bits(pc.q), wl.host_i32(pc.q_pos)
    cu_q = wl.host_i32(pc.cu_q)
    Tq, Hq, D = pc.q.shape
    rows = np.repeat(np.arange(Tq, dtype=np.int64), Hq); heads = np.tile(np.arange(Hq, dtype=np.int64), Tq)
    req_of_row = np.searchsorted(cu_q, np.arange(Tq), side="right") - 1
    single = pc.batch == 1
    to = lambda a: torch.from_numpy(a.view(np.int16)).to(pc.q.device).view(torch.bfloat16)
    for si, s in enumerate(pc.shards):
        Tkv = s.k.shape[0]
        S = max(64, 2 * Tkv + 17)
        kp = (rng.integers(0, 65536, (S, pc.Hkv, D)).astype(np.uint16)) & 0x3FFF
        vp = (rng.integers(0, 65536, (S, pc.Hkv, D)).astype(np.uint16)) & 0x3FFF
        slots = rng.permutation(S)[:Tkv].astype(np.int32)
        slots[rng.random(Tkv) > keep_fraction] = -1
        say(f"{pc.name} shard {si} with retention: Tq={Tq} Tkv={Tkv} Hq={Hq} Hkv={pc.Hkv} batch={pc.batch} kept={int((slots >= 0).sum())} pool={S}")
        kp_d, vp_d = to(kp), to(vp)
        O = torch.full(pc.q.shape, float("nan"), dtype=out_dtype, device=pc.q.device)
        LSE = torch.full((Tq, Hq), float("nan"), dtype=torch.float32, device=pc.q.device)
        args = (None if single else pc.cu_q, None if single else s.cu_kv, None if single else pc.max_q, None if single else s.max_kv)
        esp.esp_partial_attn_prefill_retain(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, torch.from_numpy(slots).to(pc.q.device), kp_d, vp_d, *args,
                                            softmax_scale=pc.scale, causal=pc.causal, O=O, LSE=LSE)
        torch.cuda.synchronize()
        oracle.kv_append(wl.bits(s.k), wl.bits(s.v), slots, kp, vp)
        assert np.array_equal(wl.bits(kp_d), kp), f"{pc.name} shard {si}: K pool differs"
        assert np.array_equal(wl.bits(vp_d), vp), f"{pc.name} shard {si}: V pool differs"
        if Tq == 0:
            continue
        O0, L0 = esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, *args, softmax_scale=pc.scale, causal=pc.causal,
                                              out_dtype=out_dtype)
        torch.cuda.synchronize()
        # against the call that keeps nothing: the same log-sum-exp bit for bit; O may differ in the last bits (an item
        # that keeps rows runs the masked iteration on more tiles, and that one normalises by the rounded probabilities)
        assert torch.equal(LSE.view(torch.int32), L0.view(torch.int32))
        assert torch.allclose(O.float(), O0.float(), rtol=2.0 ** -7, atol=1e-6)
        cu_kv = wl.host_i32(s.cu_kv)
        lo, hi = cu_kv[req_of_row[rows]], cu_kv[req_of_row[rows] + 1]
        Or, Lr = oracle.partial_attn(qb, wl.bits(s.k), wl.bits(s.v), qp, wl.host_i32(s.kv_pos), pc.scale, pc.causal, rows, heads, lo, hi)
        check_o_lse(O.float().cpu().numpy().reshape(-1, D), LSE.cpu().numpy().reshape(-1), Or, Lr, f"{pc.name} shard {si} (retain)")


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2), (4, 1)])
def test_retain_striped_varlen_ragged(esp, cuda, Hq, Hkv):
    pc = wl.striped_prefill(f"retain-varlen-{Hq}/{Hkv}", [1, 63, 257, 300, 64, 700], 2, 0, Hq, Hkv, 120, cuda)
    run_retain_case(esp, pc, 1)


def test_retain_long_shard_plain_iterations_and_fp32_out(esp, cuda):
    """A chunk behind a long prefix: most tiles run the branch-free iteration, the slot ring wraps several times."""
    pc = wl.contiguous_prefill("retain-long", 300, 2300, [(0, 2000), (2000, 2600)], 4, 4, 121, cuda)
    run_retain_case(esp, pc, 2, out_dtype=torch.float32)


def test_retain_rows_no_query_can_see(esp, cuda):
    """The shard lies in the future of every query (and, second shard, of most): everything asked for is kept anyway."""
    pc = wl.contiguous_prefill("retain-future", 300, 0, [(5000, 5777), (100, 900)], 4, 2, 122, cuda)
    run_retain_case(esp, pc, 3, keep_fraction=1.0)


def test_retain_non_causal_and_unsorted(esp, cuda):
    pc = wl.contiguous_prefill("retain-noncausal", 130, 0, [(0, 200), (200, 533)], 4, 4, 123, cuda, causal=False)
    run_retain_case(esp, pc, 4)
    pc = wl.contiguous_prefill("retain-shuffled", 300, 500, [(0, 450), (450, 1100)], 4, 2, 124, cuda)
    g = torch.Generator(device="cpu").manual_seed(6)
    for s in pc.shards:
        s.kv_pos = s.kv_pos[torch.randperm(s.kv_pos.numel(), generator=g).to(cuda)].contiguous()
    pc.q_pos = pc.q_pos[torch.randperm(pc.q_pos.numel(), generator=g).to(cuda)].contiguous()
    run_retain_case(esp, pc, 5)


@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (8, 8)])
def test_retain_more_items_than_workgroups(esp, cuda, Hq, Hkv):
    Tq = 256 * 72 + 40
    pc = wl.contiguous_prefill(f"retain-many-items-{Hq}/{Hkv}", Tq, 200, [(0, 330), (330, 700)], Hq, Hkv, 125, cuda)
    pc.q_pos[:] = seeded_positions(Tq, 900, 906, cuda)
    run_retain_case(esp, pc, 6)


def test_retain_requests_without_queries_and_no_queries_at_all(esp, cuda):
    """A batch whose first and last requests have rows in the shard but no query row in this call: their rows are kept
    all the same.  Then no query row at all (Tq = 0): the call is a plain scatter."""
    import dataclasses
    pc = wl.striped_prefill("retain-noq", [100, 80, 70], 2, 0, 4, 2, 126, cuda)
    sub = dataclasses.replace(pc, name="retain-noq", q=pc.q[100:180].contiguous(), q_pos=pc.q_pos[100:180].contiguous(),
                              cu_q=torch.tensor([0, 0, 80, 80], dtype=torch.int32, device=cuda), max_q=80)
    run_retain_case(esp, sub, 7)
    none = dataclasses.replace(pc, name="retain-tq0", q=pc.q[:0].contiguous(), q_pos=pc.q_pos[:0].contiguous(),
                               cu_q=torch.tensor([0, 0, 0, 0], dtype=torch.int32, device=cuda), max_q=0)
    run_retain_case(esp, none, 8)
