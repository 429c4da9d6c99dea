"""HIP path vs CPU oracle, element by element, through the C-ABI (needs an MI355X).

Integer / index / payload outputs must be bit-exact.  Advantages are float32 results of
float64 arithmetic on both sides; the bar is rtol 1e-5 / atol 1e-6.
"""
import numpy as np
import pytest

import oracle
from paper_2507_13833_amd import workloads

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-6


def _gpu():
    import torch
    from paper_2507_13833_amd import binding, runner
    binding.load()                                   # raises if libdc.so is missing: no fallback
    assert torch.cuda.is_available()
    return torch, binding, runner


def oracle_step(w, align=1, cap=0):
    eps = float(w.eps)
    bal = oracle.balance(w.seq_len, w.n_shards, cap)
    adv = oracle.group_advantage(w.reward, w.group_off, eps, w.ddof)
    adv_tok = oracle.adv_broadcast(adv, w.seq_len, w.src_tok_off, w.src_shard_seq_off, w.src_shard_tokens,
                                   w.field_by_name("mask").shards)
    pl = oracle.plan(w.seq_len, bal.perm, bal.shard_seq_off, w.token_budget, align)
    return bal, adv, adv_tok, pl


def check_step(w, align=1, cap=0, label="", overlapped=False, fused=False, two_calls=False):
    torch, binding, runner = _gpu()
    print(f"[parity] {label or w.name}: N={w.n_seq} P={w.n_shards} T={w.total_tokens} align={align} cap={cap}",
          flush=True)
    d = runner.DeviceBatch(w, align_tokens=align, cap=cap, poison=True)
    if two_calls:
        d.step_two_calls()                               # balance, advantage stage and plan in one call, then the gather
    elif fused:
        d.step_fused()                                   # the launch configuration bench.py times: balance and the
                                                         # advantage stage in one launch
    elif overlapped:
        d.step_overlapped()                              # the same on two streams
    else:
        d.step()
    torch.cuda.synchronize()
    compare_step(d, w, align, cap)
    return d


def compare_step(d, w, align=1, cap=0):
    """Every output of one finished step on DeviceBatch d against the oracle's."""
    assert d.read_status() == 0

    bal, adv, adv_tok, pl = oracle_step(w, align, cap)
    N, P = w.n_seq, w.n_shards

    # a1 + a2: Algorithm 1
    assert np.array_equal(d.perm.cpu().numpy(), bal.perm)
    assert np.array_equal(d.shard_seq_off.cpu().numpy(), bal.shard_seq_off)
    assert np.array_equal(d.shard_of_seq.cpu().numpy(), bal.shard_of_seq)
    assert np.array_equal(d.shard_load.cpu().numpy(), bal.shard_load)

    # a3: advantages
    g_adv = d.adv_seq.cpu().numpy()
    np.testing.assert_allclose(g_adv, adv, rtol=RTOL, atol=ATOL)
    for s in range(w.n_src_shards):
        g = d.adv_tok_src[s].cpu().numpy()
        np.testing.assert_allclose(g, adv_tok[s], rtol=RTOL, atol=ATOL)
        m = w.field_by_name("mask").shards[s]
        assert not g.view(np.uint32)[m == 0].any()          # +0.0 exactly where no loss is taken

    # a4: plan
    M = int(d.n_mb.item())
    assert M == pl.n_mb
    assert np.array_equal(d.dst_tok_off.cpu().numpy(), pl.dst_tok_off)
    assert np.array_equal(d.shard_tok_off.cpu().numpy(), pl.shard_tok_off)
    assert np.array_equal(d.shard_mb_off.cpu().numpy(), pl.shard_mb_off)
    assert np.array_equal(d.mb_seq_off.cpu().numpy()[:M + 1], pl.mb_seq_off)
    assert np.array_equal(d.cu_seqlens.cpu().numpy()[:N + M], pl.cu_seqlens)

    # a5: gather, every field, whole arena (poison outside the shards must survive)
    arena = d.capacity
    valid = np.zeros(arena, bool)
    for k in range(P):
        valid[pl.shard_tok_off[k]: pl.shard_tok_off[k] + bal.shard_load[k]] = True
    for f in w.fields:
        want = oracle.gather(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, f.shards,
                             pl.dst_tok_off, arena)
        got = d.dst_fields[f.name].cpu().numpy().view(want.dtype)
        assert np.array_equal(got[valid], want[valid]), f.name
        poison = np.frombuffer(bytes([0x5A] * f.elem_bytes), dtype=want.dtype)[0]
        assert np.all(got[~valid] == poison), f.name
    want = oracle.gather(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, adv_tok, pl.dst_tok_off, arena)
    got = d.dst_fields["adv_tok"].cpu().numpy().view(np.float32)
    np.testing.assert_allclose(got[valid], want[valid], rtol=RTOL, atol=ATOL)
    assert np.all(got[~valid].view(np.uint32) == 0x5A5A5A5A)
    # the repacked advantage is a bit copy of what the advantage kernel wrote
    src_adv = [t.cpu().numpy() for t in d.adv_tok_src]
    base = np.concatenate([[0], np.cumsum(w.src_shard_tokens)])
    shard_of = np.searchsorted(w.src_shard_seq_off, np.arange(N), side="right") - 1
    for j in np.random.default_rng(1).integers(0, N, 64) if N else []:
        i = bal.perm[j]
        seg_src = src_adv[shard_of[i]][w.src_tok_off[i]: w.src_tok_off[i] + w.seq_len[i]]
        seg_dst = got[pl.dst_tok_off[j]: pl.dst_tok_off[j] + w.seq_len[i]]
        assert np.array_equal(seg_src.view(np.uint32), seg_dst.view(np.uint32))


# ---------------------------------------------------------------- the five configs, full size
@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_config(cfg):
    check_step(workloads.make_workload(cfg), label=f"config {cfg}")


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_full_config_as_benchmarked(cfg):
    """Same check on the step bench.py times (balance and the advantage stage in one launch, one stream)."""
    d = check_step(workloads.make_workload(cfg), label=f"config {cfg}, fused launch", fused=True)
    # a second pass over the same buffers must reproduce every output bit for bit
    import torch
    first = {k: v.clone() for k, v in d.dst_fields.items()}
    perm, cu, dst = d.perm.clone(), d.cu_seqlens.clone(), d.dst_tok_off.clone()
    d.step_fused()
    torch.cuda.synchronize()
    assert d.read_status() == 0
    assert torch.equal(perm, d.perm) and torch.equal(cu, d.cu_seqlens) and torch.equal(dst, d.dst_tok_off)
    for k, v in d.dst_fields.items():
        assert torch.equal(first[k], v), k


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_config_balance_and_plan_in_one_call(cfg):
    """dc_balance_plan_group_advantage + dc_gather (what bench.py times): on configs 3-5 the plan runs as the tail
    of the balance workgroup, on configs 1 and 2 (4 and 8 shards) the call issues the separate kernels."""
    import torch
    d = check_step(workloads.make_workload(cfg), label=f"config {cfg}, balance + plan in one call", two_calls=True)
    first = {k: v.clone() for k, v in d.dst_fields.items()}
    perm, cu, dst = d.perm.clone(), d.cu_seqlens.clone(), d.dst_tok_off.clone()
    d.step_two_calls()                                   # a second pass reproduces every output bit for bit
    torch.cuda.synchronize()
    assert d.read_status() == 0
    assert torch.equal(perm, d.perm) and torch.equal(cu, d.cu_seqlens) and torch.equal(dst, d.dst_tok_off)
    for k, v in d.dst_fields.items():
        assert torch.equal(first[k], v), k


def test_balance_and_plan_in_one_call_shapes():
    rng = np.random.default_rng(51)
    for P, N in ((16, 16), (32, 32 * 3), (64, 64 * 17), (64, 4096), (16, 16 * 1024), (32, 32 * 512)):
        lens = np.minimum(rng.geometric(0.004, N), 6000).astype(np.int32)
        check_step(_custom(lens, 1 if N < 64 else 4, P, 16384, n_src=2 if N >= 64 else 1), label=f"P={P} N={N}", two_calls=True)
    # tiny sequences: many slots per gather tile, hundreds per micro-batch
    check_step(_custom(rng.integers(1, 9, 8192), 8, 16, 64, n_src=4), label="lengths 1..8", two_calls=True)
    # shard starts aligned; a budget that one slot fills exactly
    lens = rng.integers(1, 700, 64 * 40).astype(np.int32)
    lens[5] = 4096
    for align in (3, 64):
        check_step(_custom(lens, 8, 64, 4096, n_src=2), align=align, label=f"align {align}", two_calls=True)
    # lengths of 2^16 and more leave the packed path (one word per sequence) for the general one, plan still in the call
    lens = rng.integers(1, 3000, 32 * 16).astype(np.int32)
    lens[7] = 70000; lens[100] = 65536; lens[101] = 65535
    check_step(_custom(lens, 4, 32, 1 << 17, fields=("i32",)), label="a sequence of 70000 tokens", two_calls=True)
    # all lengths equal (no sort pass), and a long tail that keeps one worker far above the others
    check_step(_custom(np.full(64 * 30, 77), 8, 64, 1024), label="all equal", two_calls=True)
    heavy = np.minimum(64 * (1.0 - rng.random(64 * 64)) ** (-1 / 1.3), 32768).astype(np.int32) + rng.integers(512, 4096, 64 * 64)
    check_step(_custom(heavy, 16, 64, 65536, fields=("i32",)), label="long tail", two_calls=True)
    # fewer than 32 workers (16- and 32-lane rounds with lanes that offer nothing), also with a length of 2^16 and more
    for P, C in ((8, 128), (4, 512), (2, 100), (1, 64), (5, 33), (12, 40), (15, 7), (17, 30), (24, 64), (31, 9)):
        check_step(_custom(np.minimum(rng.geometric(0.004, P * C), 6000), 1, P, 16384), label=f"P={P} C={C}", two_calls=True)
    lens = rng.integers(1, 3000, 8 * 64).astype(np.int32)
    lens[3] = 66000
    check_step(_custom(lens, 4, 8, 1 << 17, fields=("i32",)), label="P=8, a sequence of 66000 tokens", two_calls=True)
    # shapes the call hands to the separate kernels: partitions of unequal size, 48 shards, 128 shards
    check_step(_custom(rng.integers(1, 500, 1000), 5, 16, 4096), cap=70, label="cap 70", two_calls=True)
    check_step(_custom(rng.integers(1, 500, 48 * 40), 8, 48, 4096), label="P=48", two_calls=True)
    check_step(_custom(rng.integers(1, 300, 128 * 20), 8, 128, 2048, n_src=2), label="P=128", two_calls=True)
    # and the training-layout advantage field made by the gather behind it
    w = workloads.make_workload(2, n_shards=16)
    torch, binding, runner = _gpu()
    a, b = runner.DeviceBatch(w, poison=True), runner.DeviceBatch(w, poison=True)
    a.step_two_calls(per_token=False); b.step_no_rollout_adv()
    torch.cuda.synchronize()
    assert a.read_status() == 0 and b.read_status() == 0
    for k in a.dst_fields:
        assert torch.equal(a.dst_fields[k], b.dst_fields[k]), k


def test_balance_and_plan_in_one_call_status_codes():
    torch, binding, runner = _gpu()
    lens = np.random.default_rng(52).integers(1, 60, 64).astype(np.int32)
    lens[9] = 200
    w = _custom(lens, 4, 16, 100)                                      # 200 > budget 100
    d = runner.DeviceBatch(w)
    d.step_two_calls(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_SEQ_EXCEEDS_BUDGET
    w = _custom(lens, 4, 16, 4096)
    d = runner.DeviceBatch(w)
    d.seq_len[1] = 0                                                   # zero-length sequence
    d.step_two_calls(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_ZERO_LENGTH_SEQ
    d = runner.DeviceBatch(w)
    d.capacity -= 1                                                    # arena one token short
    d.step_two_calls(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_OVERFLOW
    d = runner.DeviceBatch(w, poison=True)
    d.src_tok_off[3] = w.total_tokens                                  # a sequence that would start beyond its buffer
    d.step_two_calls(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT
    # host errors come before anything is enqueued
    d = runner.DeviceBatch(w)
    with pytest.raises(binding.DcError) as e:
        binding.dc_balance_plan_group_advantage(d.prm, d.source, d.seq_len, d.perm, d.shard_seq_off, d.shard_of_seq,
                                                d.shard_load, d.reward, d.group_off, w.n_groups, d.src_fields["mask"],
                                                d.adv_seq, d.adv_tok_src, d.capacity, d.dst_tok_off, d.shard_tok_off,
                                                d.shard_mb_off, d.mb_seq_off, d.cu_seqlens, d.n_mb, d.ws, 16, d.status)
    assert e.value.code == binding.DC_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert not d.perm.any()                                            # nothing ran


@pytest.mark.parametrize("cfg", [2, 5])
def test_gather_whose_dispatch_carries_the_timing_events(cfg):
    """dc_gather_timed: the same arenas as dc_gather, bit for bit, and two events that hold the kernel's own begin
    and end: a positive duration that does not exceed the one of events recorded round the call."""
    torch, binding, runner = _gpu()
    w = workloads.make_workload(cfg)
    d = check_step(w, label=f"config {cfg}, then dc_gather_timed", two_calls=True)
    want = {k: v.clone() for k, v in d.dst_fields.items()}
    for v in d.dst_fields.values():
        v.view(torch.uint8).fill_(0x5A)
    inner = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    outer = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    if not inner[0].cuda_event:                          # torch creates the HIP event at its first record:
        with pytest.raises(ValueError):                  # before that there is no handle to pass
            d.gather(inner)
    for e in inner:
        e.record()
    torch.cuda.synchronize()
    outer[0].record()
    d.gather(inner)
    outer[1].record()
    torch.cuda.synchronize()
    assert d.read_status() == 0
    for k, v in d.dst_fields.items():
        assert torch.equal(want[k], v), k
    ti, to = inner[0].elapsed_time(inner[1]), outer[0].elapsed_time(outer[1])
    print(f"[parity] gather timed by its dispatch: {ti:.4f} ms, by events round the call: {to:.4f} ms", flush=True)
    assert 0.0 < ti <= to * 1.02
    # one event alone, and none at all
    d.gather((inner[0], None)); d.gather((None, None))
    torch.cuda.synchronize()
    assert d.read_status() == 0


def test_step_replayed_from_a_hip_graph():
    """Every call only enqueues kernels on the given stream and allocates nothing, so a step can be captured
    in a HIP graph.  Each replay (with eager work and synchronisations in between) must reproduce the eager
    step bit for bit, and the eager step matches the oracle (check_step)."""
    import torch
    w = workloads.make_workload(2)
    d = check_step(w, label="config 2, eager step before capture", fused=True)
    want = {k: v.clone() for k, v in d.dst_fields.items()}
    want_small = [t.clone() for t in (d.perm, d.shard_seq_off, d.shard_load, d.adv_seq, d.dst_tok_off, d.cu_seqlens,
                                      d.mb_seq_off, d.n_mb)]
    side = torch.cuda.Stream()
    for step in (d.step_fused, d.step_no_rollout_adv):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        for rep in range(3):
            for v in d.dst_fields.values():
                v.fill_(0x5A)                                # eager work between the replays
            d.perm.zero_(); d.cu_seqlens.zero_(); d.dst_tok_off.zero_(); d.adv_seq.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert d.read_status() == 0
            for k, v in d.dst_fields.items():
                assert torch.equal(want[k], v), (k, rep)
            got_small = (d.perm, d.shard_seq_off, d.shard_load, d.adv_seq, d.dst_tok_off, d.cu_seqlens, d.mb_seq_off, d.n_mb)
            for a, b in zip(want_small, got_small):
                assert torch.equal(a, b), rep
        del g


def test_double_buffered_steps_on_two_streams():
    """Sec. 6.5 (double buffer) on one GPU: the library keeps no state and every call takes its arenas and its
    workspace as arguments, so the step that fills one buffer set may run on a second stream while a consumer
    still reads the other set.  Two sets with different batches, each on a stream of its own (default
    priority), three alternations issued without a host synchronisation in between, a reduction over the
    set's arenas behind every step as the consumer: both sets match the oracle and the consumer reads the
    same bits every time."""
    torch, binding, runner = _gpu()
    rng = np.random.default_rng(65)
    ws = [workloads.make_workload(2), _custom(rng.integers(1, 3000, 3072), 8, 24, 8192, n_src=2)]
    ds = [runner.DeviceBatch(w, poison=True) for w in ws]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for s in streams:
        s.wait_stream(torch.cuda.current_stream())
    sums = [[], []]
    for rep in range(3):
        for k in (0, 1):
            with torch.cuda.stream(streams[k]):
                ds[k].step_fused()
                sums[k].append(torch.stack([v.view(torch.uint8).sum(dtype=torch.int64) for v in ds[k].dst_fields.values()]))
    for s in streams:
        s.synchronize()
    torch.cuda.synchronize()
    for k in (0, 1):
        print(f"[parity] double buffer, set {k}: N={ws[k].n_seq} P={ws[k].n_shards}", flush=True)
        compare_step(ds[k], ws[k])
        assert all(torch.equal(sums[k][0], x) for x in sums[k][1:])


def test_two_stream_step():
    """The step with the advantage stage on a second stream beside balance + plan (bench.py --two-streams)."""
    check_step(workloads.make_workload(3), label="config 3, two streams", overlapped=True)


def test_fused_launch_shapes():
    """Balance + advantage in one launch on small and odd shapes: fewer sequences than one workgroup's waves,
    more groups than sequences' waves would cover, many shards, an empty batch."""
    rng = np.random.default_rng(16)
    check_step(_custom(rng.integers(1, 200, 6), 3, 2, 512), fused=True, label="fused N=6")
    check_step(_custom(rng.integers(1, 50, 1000), 1, 8, 4096, n_src=2), fused=True, label="fused G=1")
    check_step(_custom(rng.integers(1, 300, 2048), 8, 128, 2048, n_src=4), fused=True, label="fused P=128")
    torch, binding, runner = _gpu()
    d = runner.DeviceBatch(_custom(np.zeros(0, np.int32), 1, 4, 128))
    d.step_fused(); torch.cuda.synchronize()
    assert d.read_status() == 0 and int(d.n_mb.item()) == 0


def test_padded_rollout_layout():
    """The paper's batches are padded (Sec. 7.1: prompts left-padded to a fixed width, responses
    right-padded): a sequence's valid tokens are one contiguous run inside its row, so the rollout
    offsets express that layout directly; only valid tokens are read."""
    rng = np.random.default_rng(21)
    N, G, max_prompt, max_resp = 1024, 8, 512, 1024
    p_len = np.repeat(rng.integers(16, max_prompt + 1, N // G), G)
    r_len = rng.integers(1, max_resp + 1, N)
    row = max_prompt + max_resp
    w = _custom((p_len + r_len).astype(np.int32), G, 8, 4096, n_src=2)
    per = N // 2
    w.src_tok_off = ((np.arange(N) % per) * row + (max_prompt - p_len)).astype(np.int64)
    w.src_shard_tokens = np.array([per * row, per * row], np.int64)
    for f in w.fields:                                    # padded buffers: sentinel bytes in the padding
        dt = f.shards[0].dtype
        f.shards = [rng.integers(0, 200, per * row).astype(dt) for _ in range(2)]
    check_step(w, label="padded rows of 1536 tokens")


def test_repack_equals_plan_then_gather_and_is_deterministic():
    torch, binding, runner = _gpu()
    w = workloads.make_workload(2)
    d = runner.DeviceBatch(w)
    d.step()
    torch.cuda.synchronize()
    first = {k: v.clone() for k, v in d.dst_fields.items()}
    cu = d.cu_seqlens.clone()
    perm = d.perm.clone()
    for v in d.dst_fields.values():
        v.zero_()
    d.group_advantage(); d.balance(); d.repack()
    torch.cuda.synchronize()
    assert d.read_status() == 0
    assert torch.equal(perm, d.perm) and torch.equal(cu, d.cu_seqlens)
    for k, v in d.dst_fields.items():
        assert torch.equal(first[k], v), k


# ---------------------------------------------------------------- shapes and edges
def _custom(seq_len, G, P, budget, n_src=1, seed=0, fields=("i32", "bf16", "u8")):
    """Small hand-shaped workload (same field kinds, arbitrary lengths)."""
    rng = np.random.default_rng(seed)
    seq_len = np.asarray(seq_len, np.int32)
    N = len(seq_len)
    assert N % G == 0 and N % n_src == 0
    per = N // n_src
    sso = (np.arange(n_src + 1) * per).astype(np.int32)
    sto = np.zeros(N, np.int64)
    stk = np.zeros(n_src, np.int64)
    for s in range(n_src):
        c = np.cumsum(seq_len[sso[s]:sso[s + 1]].astype(np.int64))
        sto[sso[s] + 1: sso[s + 1]] = c[:-1]
        stk[s] = c[-1] if len(c) else 0
    fl = []
    for kind in fields:
        if kind == "i32":
            fl.append(workloads.Field("token_id", 4, [rng.integers(0, 1 << 30, int(t), dtype=np.int32) for t in stk]))
        elif kind == "bf16":
            fl.append(workloads.Field("old_logprob", 2,
                                      [rng.integers(0, 1 << 16, int(t)).astype(np.uint16) for t in stk]))
    fl.append(workloads.Field("mask", 1, [(rng.random(int(t)) < 0.7).astype(np.uint8) for t in stk]))
    reward = rng.standard_normal(N).astype(np.float32)
    return workloads.Workload(name="custom", cfg=0, n_seq=N, group_size=G, n_shards=P, token_budget=budget,
                              eps=1e-6, ddof=1, align_tokens=1, seq_len=seq_len,
                              prompt_len=np.zeros(N, np.int32),
                              group_off=(np.arange(N // G + 1) * G).astype(np.int32), reward=reward,
                              src_shard_seq_off=sso, src_tok_off=sto, src_shard_tokens=stk, fields=fl)


def test_seeded_random_shapes():
    """Forty drawn shapes through the step as bench.py issues it and through the separate calls: shard counts on both
    sides of every path's limits, partitions of equal and unequal size, length mixes from all ones to one sequence a
    thousand times the others, 1 to 8 rollout shards, aligned shards, budgets that a single slot fills."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        P = int(rng.choice([1, 2, 3, 7, 16, 16, 32, 32, 64, 64, 65, 96, 200]))
        C = int(rng.choice([1, 2, 3, 5, 17, 40, 64]))
        n_src = int(rng.choice([1, 1, 2, 4, 8]))
        N = P * C
        G = int(rng.choice([g for g in (1, 2, 4, 8, 16) if N % g == 0]))
        while N % n_src:
            n_src //= 2
        kind = int(rng.integers(0, 5))
        if kind == 0:
            lens = np.ones(N, np.int64)
        elif kind == 1:
            lens = rng.integers(1, 40, N)
        elif kind == 2:
            lens = np.minimum(rng.geometric(0.003, N), 5000)
        elif kind == 3:
            lens = rng.integers(1, 60, N); lens[int(rng.integers(0, N))] = 70000          # one length of 2^16 or more
        else:
            lens = np.full(N, int(rng.integers(1, 3000)))                                   # all equal: nothing to sort
        if int(lens.sum()) > 6_000_000:
            lens = np.minimum(lens, 2000)
        budget = int(max(lens.max(), rng.choice([1, 64, 4096, 1 << 17])))
        align = int(rng.choice([1, 1, 3, 16, 256]))
        cap = 0 if rng.random() < 0.7 else C + int(rng.integers(1, 4))
        w = _custom(lens.astype(np.int32), G, P, budget, n_src=n_src, seed=case, fields=("i32", "bf16") if case % 2 else ("i32",))
        label = f"drawn shape {case}: P={P} C={C} kind={kind} G={G} rollout shards={n_src} budget={budget}"
        check_step(w, align=align, cap=cap, label=label, two_calls=bool(case % 3))


@pytest.mark.parametrize("align", [3, 16, 64, 4096])
def test_alignment_padding(align):
    check_step(workloads.make_workload(1), align=align, label=f"config 1 align {align}")


def test_unconstrained_lpt():
    w = workloads.make_workload(2, prompts=64)
    check_step(w, cap=w.n_seq, label="cap=N (textbook LPT)")
    check_step(w, cap=w.n_seq // w.n_shards + 3, label="cap=C+3")


def test_tiny_sequences_many_per_tile():
    rng = np.random.default_rng(4)
    # ~900 slots per 4096-token tile: several LDS passes per tile, most chunks straddle slots
    check_step(_custom(rng.integers(1, 9, 8192), 8, 16, 64, n_src=4), label="lengths 1..8")
    check_step(_custom(np.ones(4096, np.int32), 4, 64, 7, n_src=2), align=5, label="all length 1")


def test_equal_lengths_and_single_shard():
    check_step(_custom(np.full(512, 37, np.int32), 8, 1, 1000), label="equal lengths, P=1")
    check_step(_custom(np.full(64, 300, np.int32), 8, 64, 300), label="N=P, budget = one sequence")


def test_ragged_sizes():
    rng = np.random.default_rng(9)
    check_step(_custom(rng.integers(1, 3000, 1000), 5, 8, 4096, n_src=2), label="N=1000")
    check_step(_custom(rng.integers(1, 70000, 63 * 3), 3, 63, 70000, n_src=1), label="P=63, long")
    check_step(_custom(rng.integers(1, 200, 2), 2, 2, 512), label="N=2")


def test_partition_sizes_and_worker_counts():
    """N = P * C for many (P, C): the items are filed per worker while they are placed (row pitch C rounded up
    to 2 mod 4), for odd and even C, worker counts that are no power of two, one worker, one item per worker;
    and the same batches with a limit above C (partitions of unequal size: the other layout pass)."""
    torch, binding, runner = _gpu()
    rng = np.random.default_rng(23)
    for P in (1, 2, 3, 5, 17, 33, 64):
        for C in (1, 2, 3, 4, 7, 64, 255, 256):
            N = P * C
            if N > 16384:
                continue
            lens = np.minimum(rng.geometric(0.01, N), 1500).astype(np.int32)
            if (P + C) % 3 == 0:
                lens[:] = lens[0]                               # all equal: index order decides everything
            w = _custom(lens, 1, P, 4096, fields=("i32",))
            for cap in (0, C + 1):
                d = runner.DeviceBatch(w, cap=cap)
                d.balance()
                torch.cuda.synchronize()
                assert d.read_status() == 0
                bal = oracle.balance(w.seq_len, P, cap)
                assert np.array_equal(d.perm.cpu().numpy(), bal.perm), (P, C, cap)
                assert np.array_equal(d.shard_seq_off.cpu().numpy(), bal.shard_seq_off), (P, C, cap)
                assert np.array_equal(d.shard_of_seq.cpu().numpy(), bal.shard_of_seq), (P, C, cap)
                assert np.array_equal(d.shard_load.cpu().numpy(), bal.shard_load), (P, C, cap)


def test_one_pass_sort_of_the_packed_path():
    """16, 32 or 64 workers, equal partitions, lengths below 2^16: the sorted list comes from one counting pass
    over a bin per length (tickets from atomic adds issued in index order, wave after wave, and a check of the
    result), with the two radix passes as the way out.  Cases: runs of one length at, just below and just above
    the limit of the one-pass sort, and long runs below it (many adds meeting in one word); the shortest length
    (the last run, followed by the array's padding) as the most frequent; few distinct lengths (always the way
    out); a range of lengths at and beyond what the bins hold; batches that are no multiple of the workgroup,
    smaller than a wavefront, and the largest."""
    torch, binding, runner = _gpu()
    rng = np.random.default_rng(61)

    def check(lens, P, label):
        lens = np.asarray(lens, np.int32)
        w = _custom(lens, 1, P, 1 << 17, fields=("i32",))
        d = runner.DeviceBatch(w)
        d.balance()
        torch.cuda.synchronize()
        assert d.read_status() == 0, label
        bal = oracle.balance(w.seq_len, P, 0)
        assert np.array_equal(d.perm.cpu().numpy(), bal.perm), label
        assert np.array_equal(d.shard_seq_off.cpu().numpy(), bal.shard_seq_off), label
        assert np.array_equal(d.shard_of_seq.cpu().numpy(), bal.shard_of_seq), label
        assert np.array_equal(d.shard_load.cpu().numpy(), bal.shard_load), label

    def with_runs(n, run, lo=100, hi=9000):
        """n lengths in which one value occurs exactly `run` times and no other more often than three times"""
        vals = rng.permutation(np.arange(lo, hi))[: n]
        lens = np.concatenate([np.repeat(vals[: (n - run) // 3 + 1], 3)[: n - run], np.full(run, hi + 7)])
        return rng.permutation(lens)

    for run in (2, 33, 64, 65, 700, 1023, 1024, 1025):
        check(with_runs(64 * 64, run), 64, f"a run of {run}")
    lens = with_runs(32 * 100, 30)
    lens[lens == lens.max()] = 5                                       # the longest run is the last one
    check(lens, 32, "most frequent length is the shortest")
    check(np.concatenate([np.full(20, 3), rng.permutation(np.arange(50, 50 + 16 * 64 - 20))]), 16, "the list ends in a run of 20")
    check(rng.choice([700, 701, 9000], 64 * 128), 64, "three distinct lengths")
    check(rng.choice(np.arange(1000, 1040), 16 * 1024), 16, "forty distinct lengths, 16 384 sequences")
    for top in (41000, 41981, 41982, 41983, 41984, 65535):             # range = top - 1
        lens = rng.integers(1, top + 1, 64 * 200)
        lens[3] = top; lens[11] = 1
        check(lens, 64, f"lengths 1..{top}")
    check(rng.integers(40000, 65536, 64 * 256), 64, "long sequences, 16 384 of them")
    for P, C in ((16, 1), (16, 3), (32, 33), (64, 17), (64, 100), (16, 1000), (32, 511), (64, 255)):
        check(np.minimum(rng.geometric(0.002, P * C), 30000), P, f"P={P} C={C}")
        check(rng.integers(200, 200 + max(2, P * C // 5), P * C), P, f"P={P} C={C}, five of every length")


def test_max_sequences():
    rng = np.random.default_rng(10)
    lens = np.minimum(rng.geometric(0.02, 16384), 2000).astype(np.int32)
    check_step(_custom(lens, 16, 64, 8192, n_src=16), label="N=16384 (limit), 16 rollout shards")


def test_more_than_64_shards():
    """More workers than a wavefront has lanes: the assignment rounds run on the whole workgroup."""
    rng = np.random.default_rng(14)
    lens = np.minimum(rng.geometric(0.01, 16384), 3000).astype(np.int32)
    check_step(_custom(lens, 16, 128, 8192, n_src=4), label="N=16384 P=128")
    check_step(_custom(lens, 16, 1024, 8192, n_src=4), label="N=16384 P=1024 (limit)")
    lens = rng.integers(1, 5000, 65 * 48).astype(np.int32)
    check_step(_custom(lens, 8, 65, 16384), label="P=65")
    check_step(_custom(lens, 8, 65, 16384), align=16, label="P=65 align 16")
    lens = np.concatenate([rng.integers(2000, 2100, 2048), np.ones(2048, np.int64)]).astype(np.int32)   # heavy ties
    w = _custom(lens, 16, 256, 4096, n_src=2)
    check_step(w, label="P=256 ties")
    check_step(w, cap=w.n_seq, label="P=256 cap=N (textbook LPT)")
    check_step(w, cap=w.n_seq // 256 + 2, label="P=256 cap=C+2")
    check_step(_custom(rng.integers(1, 300, 200), 2, 200, 512), label="N=P=200")


def test_more_than_64_shards_key_widths():
    """The workgroup-wide rounds keep 32-bit keys while every length is below 2^16 (rebased whenever the smallest key
    has passed 2^30) and 64-bit keys otherwise; in one piece and in portions."""
    rng = np.random.default_rng(16)
    heavy = lambda n: np.minimum(64 * (1.0 - rng.random(n)) ** (-1 / 1.3), 32768).astype(np.int32) + rng.integers(512, 4096, n)
    # ~10 M tokens per worker: (load << 10) passes 2^32 several times over
    _check_balance_ws(rng.integers(30000, 65536, 65 * 200), 65, label="65 workers, long sequences: 32-bit keys rebased")
    _check_balance_ws(rng.integers(30000, 65536, 256 * 200), 256, label="256 workers in portions, 32-bit keys rebased")
    _check_balance_ws(np.concatenate([[65535], rng.integers(1, 3, 128 * 100 - 1)]), 128, label="128 workers, 65535 and ones")
    # one length of 2^16 or more: 64-bit keys, ranks by counting
    _check_balance_ws(np.concatenate([[70000], rng.integers(1, 5000, 128 * 64 - 1)]), 128, label="128 workers, one length above 2^16")
    _check_balance_ws(np.concatenate([[1 << 24], heavy(128 * 300 - 1)]), 128, label="128 workers in portions, the longest length there is")
    _check_balance_ws(np.concatenate([[65536], rng.integers(100, 200, 1000 * 30 - 1)]), 1000, label="1000 workers, 64-bit keys")


def test_packed_rounds_with_keys_rebased():
    """16, 32 and 64 workers with tens of millions of tokens each: (load << 6) passes 2^30 again and again inside the
    packed rounds (sure, tested and short ones), in one piece and in portions."""
    rng = np.random.default_rng(17)
    _check_balance_ws(rng.integers(30000, 65536, 16384), 16, label="16 workers, 49 M tokens each")
    _check_balance_ws(rng.integers(30000, 65536, 32 * 400), 32, label="32 workers, 19 M tokens each")
    _check_balance_ws(np.concatenate([[65535] * 3, rng.integers(20000, 24000, 64 * 256 - 3)]), 64, label="64 workers, three long ones")
    _check_balance_ws(rng.integers(30000, 65536, 32768), 16, label="16 workers in portions, 98 M tokens each")


def _check_balance_ws(lens, P, cap=0, label=""):
    torch, binding, runner = _gpu()
    lens = np.asarray(lens, np.int32)
    N = len(lens)
    print(f"[parity] balance_ws {label}: N={N} P={P} cap={cap}", flush=True)
    prm = binding.make_params(N, P, 1 << 20, 1e-6, 1, cap, 1)
    dev = torch.device("cuda:0")
    seq_len = torch.from_numpy(lens).to(dev)
    perm = torch.full((N,), -1, dtype=torch.int32, device=dev)
    shard_seq_off = torch.full((P + 1,), -1, dtype=torch.int32, device=dev)
    shard_of_seq = torch.full((N,), -1, dtype=torch.int32, device=dev)
    shard_load = torch.full((P,), -1, dtype=torch.int64, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    nb = binding.dc_balance_workspace_bytes(prm)
    assert (nb > 0) == (N > binding.DC_MAX_SEQ)
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device=dev) if nb else None
    binding.dc_balance_ws(prm, seq_len, perm, shard_seq_off, shard_of_seq, shard_load, ws, nb, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    bal = oracle.balance(lens, P, cap)
    assert np.array_equal(perm.cpu().numpy(), bal.perm)
    assert np.array_equal(shard_seq_off.cpu().numpy(), bal.shard_seq_off)
    assert np.array_equal(shard_of_seq.cpu().numpy(), bal.shard_of_seq)
    assert np.array_equal(shard_load.cpu().numpy(), bal.shard_load)


def test_balance_beyond_the_lds():
    """dc_balance_ws above DC_MAX_SEQ sequences: index arrays in a workspace, the assignment in portions."""
    rng = np.random.default_rng(31)
    heavy = lambda n: np.minimum(64 * (1.0 - rng.random(n)) ** (-1 / 1.3), 32768).astype(np.int32) + rng.integers(512, 4096, n)
    _check_balance_ws(heavy(16384 + 64), 64, label="one round more than the LDS holds")
    _check_balance_ws(heavy(32768), 64, label="two portions, long tail")
    _check_balance_ws(np.minimum(rng.geometric(0.002, 49152), 9000), 16, label="three portions, P=16")
    _check_balance_ws(rng.integers(1, 300, 100000), 8, label="N=100000, many equal lengths")
    _check_balance_ws(rng.integers(1, 5000, 40000), 7, cap=6000, label="partitions of unequal size")
    _check_balance_ws(rng.integers(1, 5000, 40003), 7, cap=40003 // 7 + 1, label="N no multiple of P")
    _check_balance_ws(np.full(20000, 77), 4, label="all equal")
    _check_balance_ws(rng.integers(1, 100, 30000), 1, label="one worker")
    _check_balance_ws(heavy(63 * 785), 63, label="P=63, portions that end inside a round")
    _check_balance_ws(heavy(8192), 32, label="below the limit: dc_balance itself, no workspace")
    _check_balance_ws(heavy(128 * 300), 128, label="128 workers")
    _check_balance_ws(rng.integers(1, 2000, 1000 * 40), 1000, label="1000 workers, lengths with many ties")
    _check_balance_ws(heavy(65 * 600), 65, cap=640, label="65 workers, partitions of unequal size")
    # the most a shard may hold above DC_MAX_SEQ sequences: a place inside a partition is a 16-bit number
    _check_balance_ws(rng.integers(1, 60, 2 * 65535), 2, label="65535 sequences per shard")
    # 16, 32 or 64 workers, all partitions of equal size, lengths below 2^16: the packed rounds, portion by portion
    _check_balance_ws(rng.integers(200, 6000, 65536), 32, label="packed rounds, four portions of 512 rounds")
    one_long = np.concatenate([[60000], rng.integers(1, 40, 16 * 2048 - 1)])
    _check_balance_ws(one_long, 16, label="packed rounds, a worker's row fills before the portion ends")
    _check_balance_ws(np.concatenate([[65535], heavy(64 * 300 - 1)]), 64, label="packed rounds, longest length 65535")
    _check_balance_ws(np.concatenate([[65536], heavy(64 * 300 - 1)]), 64, label="one length above the packed words")
    _check_balance_ws(heavy(64 * 1001), 64, label="packed rounds, a short last portion")
    # the most sequences the call takes
    _check_balance_ws(heavy(1 << 20), 64, label="2^20 sequences, packed rounds in 64 portions")
    _check_balance_ws(rng.integers(1, 2000, 1 << 20), 1024, label="2^20 sequences on 1024 workers")


def test_seeded_random_shapes_of_the_balance():
    """Thirty drawn shapes of Algorithm 1 alone, on both sides of the LDS limit: every rounds variant (packed, general,
    workgroup-wide with either key width), in one piece and in portions, equal and unequal partitions."""
    rng = np.random.default_rng(2025)
    for case in range(30):
        P = int(rng.choice([1, 5, 16, 16, 32, 32, 64, 64, 64, 100, 128, 512, 1024]))
        big = bool(rng.random() < 0.5)
        C = int(rng.integers(max(1, 16385 // P + 1), max(2, 70000 // P))) if big else int(rng.integers(1, max(2, 16384 // P + 1)))
        C = min(C, 65535)
        N = P * C
        kind = int(rng.integers(0, 5))
        if kind == 0:
            lens = np.minimum(64 * (1.0 - rng.random(N)) ** (-1 / 1.3), 32768).astype(np.int64) + rng.integers(512, 4096, N)
        elif kind == 1:
            lens = rng.integers(1, 10, N)                                                    # ties everywhere
        elif kind == 2:
            lens = rng.integers(20000, 65536, N)                                             # keys rebased again and again
        elif kind == 3:
            lens = rng.integers(1, 3000, N); lens[int(rng.integers(0, N))] = int(rng.choice([65536, 1 << 20, 1 << 24]))
        else:
            lens = np.full(N, int(rng.integers(1, 65536)))
        cap = 0
        if rng.random() < 0.3:
            cap = min(C + int(rng.integers(1, 50)), 65535)
        _check_balance_ws(lens, P, cap=cap, label=f"drawn shape {case}: kind={kind}")


def test_seeded_random_shapes_with_fewer_workers_than_lanes():
    """Twenty-five drawn batches of Algorithm 1 as printed on 1 to 32 workers: the packed rounds on an 8-, 16- or
    32-lane sort whose upper lanes have no worker, batches from one item per worker to the LDS limit, heavy ties,
    long tails, and a length of 2^16 or more (the general rounds with the same layout)."""
    torch, binding, runner = _gpu()
    rng = np.random.default_rng(2026)
    for case in range(25):
        P = int(rng.integers(1, 33))
        C = int(rng.choice([1, 2, 3, int(rng.integers(4, 200)), int(rng.integers(200, 16384 // P + 1))]))
        N = P * C
        kind = int(rng.integers(0, 5))
        if kind == 0:
            lens = np.minimum(64 * (1.0 - rng.random(N)) ** (-1 / 1.3), 32768).astype(np.int64) + rng.integers(512, 4096, N)
        elif kind == 1:
            lens = rng.integers(1, 6, N)
        elif kind == 2:
            lens = np.minimum(rng.geometric(0.002, N), 20000)
        elif kind == 3:
            lens = rng.integers(1, 3000, N); lens[int(rng.integers(0, N))] = int(rng.choice([65536, 100000]))
        else:
            lens = rng.integers(30000, 65536, N)
        w = _custom(lens.astype(np.int32), 1, P, 1 << 24, fields=("i32",))
        d = runner.DeviceBatch(w)
        d.balance()
        torch.cuda.synchronize()
        label = f"drawn shape {case}: P={P} C={C} kind={kind}"
        assert d.read_status() == 0, label
        bal = oracle.balance(w.seq_len, P, 0)
        assert np.array_equal(d.perm.cpu().numpy(), bal.perm), label
        assert np.array_equal(d.shard_seq_off.cpu().numpy(), bal.shard_seq_off), label
        assert np.array_equal(d.shard_of_seq.cpu().numpy(), bal.shard_of_seq), label
        assert np.array_equal(d.shard_load.cpu().numpy(), bal.shard_load), label


def test_more_sequences_than_the_lds_holds():
    """The whole path above DC_MAX_SEQ sequences: dc_balance_ws, the plan through workspace memory, and the
    kernels that never cared (advantage, gather, scatter, GAE)."""
    rng = np.random.default_rng(33)
    lens = np.minimum(rng.geometric(0.006, 32768), 2500).astype(np.int32)
    w = _custom(lens, 16, 64, 8192, n_src=4)
    check_step(w, label="N=32768 P=64")
    check_step(w, align=16, label="N=32768 P=64 align 16")
    check_gather_advantage(w, label="N=32768 P=64")
    check_scatter(w, label="N=32768 P=64")
    lens = rng.integers(1, 400, 50000).astype(np.int32)
    w = _custom(lens, 5, 8, 3000, n_src=2)
    check_step(w, label="N=50000 P=8, ~20 slots per micro-batch")
    check_step(w, cap=50000 // 8 + 7, label="N=50000 P=8 cap=C+7")
    w = _with_ppo_fields(_custom(np.minimum(rng.geometric(0.01, 20480), 1500).astype(np.int32), 4, 16, 100000, n_src=2))
    check_step(w, label="N=20480 P=16, ~60 slots per micro-batch... and more than two windows")
    check_gae(w, 0.99, 0.95, 0.0, label="N=20480")
    # many shards above the limit: the whole workgroup assigns, one lane per shard walks the micro-batches
    lens = rng.integers(1, 300, 128 * 200).astype(np.int32)
    check_step(_custom(lens, 8, 128, 2048, n_src=2), label="N=25600 P=128")


def test_longest_sequence_and_most_fields():
    # two sequences of DC_MAX_SEQ_LEN tokens next to tiny ones (LPT keys, 32-bit offsets inside a tile, int64 outside)
    L = 1 << 24
    w = _custom(np.array([L, 5, L - 3, 100], np.int32), 2, 2, 1 << 25, fields=("i32", "u8"))
    check_step(w, label="sequences of 2^24 tokens")
    # DC_MAX_FIELDS fields in one gather: seven payload fields of mixed widths plus the per-token advantage
    rng = np.random.default_rng(13)
    w = _custom(rng.integers(1, 700, 2048), 8, 8, 4096, n_src=2)
    for k, (eb, dt) in enumerate(((4, np.int32), (2, np.uint16), (1, np.uint8), (4, np.int32))):
        w.fields.insert(0, workloads.Field(f"extra{k}", eb,
                                           [rng.integers(0, 200, int(t)).astype(dt) for t in w.src_shard_tokens]))
    assert len(w.fields) + 1 == 8
    check_step(w, label="8 fields")
    check_scatter(w, label="8 fields")


def test_loads_beyond_the_32_bit_keys():
    # 20 M tokens per shard: (load << 6) passes 2^30 many times over, so the assignment's keys are rebased
    # again and again, with the check running only every 64th round (sequences of ~10 K tokens)
    rng = np.random.default_rng(15)
    w = _custom(rng.integers(8000, 12000, 4096), 2, 2, 1 << 20, fields=("i32", "u8"))
    check_step(w, label="P=2, 20 M tokens per shard")


def test_long_and_short_sequences_mixed():
    # a big batch (the narrow fields ride on the 4-byte fields' workgroups) whose shards end in
    # runs of very short sequences: tiles with more slots per granule than a record holds sit
    # next to tiles inside one long sequence
    rng = np.random.default_rng(11)
    lens = np.concatenate([rng.integers(3500, 4500, 8192), rng.integers(1, 120, 8192)])
    rng.shuffle(lens)
    check_step(_custom(lens, 16, 64, 16384, n_src=2), label="8192 long + 8192 short")


def test_group_sizes_and_ddof():
    torch, binding, runner = _gpu()
    rng = np.random.default_rng(12)
    for G, ddof in ((1, 1), (2, 0), (3, 1), (7, 0), (64, 1), (96, 1)):
        w = _custom(rng.integers(1, 50, G * 6), G, 2 if (G * 6) % 2 == 0 else 1, 4096)
        w.ddof = ddof
        w.reward[:G] = 0.1                                     # identical rewards, inexact value
        check_step(w, label=f"G={G} ddof={ddof}")
    w.eps = 0.0                                                # identical rewards are +0 by rule: 0 / 0 otherwise
    check_step(w, label="eps = 0")


def test_advantage_ill_conditioned_rewards():
    # large common offset: float32 statistics would lose the signal, float64 keeps it
    w = _custom(np.full(64, 20, np.int32), 16, 4, 4096)
    w.reward = (np.float32(1000.0) + np.random.default_rng(3).integers(0, 4, 64).astype(np.float32) / 1024).astype(np.float32)
    check_step(w, label="rewards 1000 + k/1024")


# ---------------------------------------------------------------- unchanged DP layout: plan in place, move nothing
def test_identity_plan_describes_the_rollout_layout_in_place():
    """Next stage with the same DP size (the paper's local-cache case, Sec. 6): no balancing, no gather.
    dc_plan with the identity permutation and the rollout shards as training shards yields offsets that
    ARE the packed rollout layout, so cu_seqlens and micro-batches apply to the rollout buffers as they lie."""
    torch, binding, runner = _gpu()
    w = workloads.make_workload(4)                                   # 8 packed rollout shards
    d = runner.DeviceBatch(w)
    P = w.n_src_shards
    prm = binding.make_params(w.n_seq, P, w.token_budget)
    d.perm.copy_(torch.arange(w.n_seq, dtype=torch.int32, device=d.dev))
    sso = torch.from_numpy(np.asarray(w.src_shard_seq_off, np.int32)).to(d.dev)
    shard_tok_off = torch.zeros(P + 1, dtype=torch.int64, device=d.dev)
    shard_mb_off = torch.zeros(P + 1, dtype=torch.int32, device=d.dev)
    ws_bytes = binding.dc_workspace_bytes(prm, d.capacity)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=d.dev)
    binding.dc_plan(prm, d.source, d.seq_len, d.perm, sso, d.capacity, d.dst_tok_off, shard_tok_off, shard_mb_off,
                    d.mb_seq_off, d.cu_seqlens, d.n_mb, ws, ws_bytes, d.status)
    torch.cuda.synchronize()
    assert d.read_status() == 0
    pl = oracle.plan(w.seq_len, np.arange(w.n_seq, dtype=np.int32), w.src_shard_seq_off, w.token_budget)
    assert np.array_equal(d.dst_tok_off.cpu().numpy(), pl.dst_tok_off)
    M = int(d.n_mb.item())
    assert M == pl.n_mb and np.array_equal(d.cu_seqlens.cpu().numpy()[: w.n_seq + M], pl.cu_seqlens)
    # offset inside its shard == offset inside its rollout buffer: nothing has to move
    sto = shard_tok_off.cpu().numpy()
    shard_of = np.repeat(np.arange(P), np.diff(w.src_shard_seq_off))
    assert np.array_equal(d.dst_tok_off.cpu().numpy()[:-1] - sto[shard_of], w.src_tok_off)
    assert np.array_equal(np.diff(sto), w.src_shard_tokens)


def test_plan_without_permutation_and_shard_table_keeps_the_rollout_shards():
    """The same case with nothing materialised on the device: d_perm = NULL (slot j holds sequence j) and
    d_shard_seq_off = NULL (the training shards are the rollout shards, Sec. 6 "Local Cache").  Every plan
    output against the oracle's plan of the identity permutation; then dc_repack with d_perm = NULL and an
    explicit shard table moves every field unpermuted."""
    torch, binding, runner = _gpu()
    for cfg in (4, 2):                                               # 8 rollout shards; one rollout shard
        w = workloads.make_workload(cfg)
        d = runner.DeviceBatch(w, poison=True)
        P = w.n_src_shards
        prm = binding.make_params(w.n_seq, P, w.token_budget)
        shard_tok_off = torch.zeros(P + 1, dtype=torch.int64, device=d.dev)
        shard_mb_off = torch.zeros(P + 1, dtype=torch.int32, device=d.dev)
        ws_bytes = binding.dc_workspace_bytes(prm, d.capacity)
        ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=d.dev)
        binding.dc_plan(prm, d.source, d.seq_len, None, None, d.capacity, d.dst_tok_off, shard_tok_off, shard_mb_off,
                        d.mb_seq_off, d.cu_seqlens, d.n_mb, ws, ws_bytes, d.status)
        torch.cuda.synchronize()
        assert d.read_status() == 0
        ident = np.arange(w.n_seq, dtype=np.int32)
        pl = oracle.plan(w.seq_len, ident, w.src_shard_seq_off, w.token_budget)
        M = int(d.n_mb.item())
        assert M == pl.n_mb
        assert np.array_equal(d.dst_tok_off.cpu().numpy(), pl.dst_tok_off)
        assert np.array_equal(shard_tok_off.cpu().numpy(), pl.shard_tok_off)
        assert np.array_equal(shard_mb_off.cpu().numpy(), pl.shard_mb_off)
        assert np.array_equal(d.mb_seq_off.cpu().numpy()[:M + 1], pl.mb_seq_off)
        assert np.array_equal(d.cu_seqlens.cpu().numpy()[: w.n_seq + M], pl.cu_seqlens)
        shard_of = np.repeat(np.arange(P), np.diff(w.src_shard_seq_off))
        assert np.array_equal(d.dst_tok_off.cpu().numpy()[:-1] - pl.shard_tok_off[shard_of], w.src_tok_off)
        # a shard table without a permutation: 4 training shards of N/4 consecutive sequences, fields moved as they lie
        prm4 = binding.make_params(w.n_seq, 4, w.token_budget)
        sso4 = torch.arange(5, dtype=torch.int32, device=d.dev) * (w.n_seq // 4)
        st4 = torch.zeros(5, dtype=torch.int64, device=d.dev)
        sm4 = torch.zeros(5, dtype=torch.int32, device=d.dev)
        binding.dc_repack(prm4, d.source, d.seq_len, None, sso4, d.moved_fields, d.capacity, d.dst_tok_off, st4, sm4,
                          d.mb_seq_off, d.cu_seqlens, d.n_mb, ws, ws_bytes, d.status)
        torch.cuda.synchronize()
        assert d.read_status() == 0
        pl4 = oracle.plan(w.seq_len, ident, sso4.cpu().numpy(), w.token_budget)
        assert np.array_equal(d.dst_tok_off.cpu().numpy(), pl4.dst_tok_off)
        arena = int(pl4.shard_tok_off[-1])
        for f in w.fields:
            want = oracle.gather(w.seq_len, ident, w.src_tok_off, w.src_shard_seq_off, f.shards, pl4.dst_tok_off, arena)
            assert np.array_equal(d.dst_fields[f.name].cpu().numpy().view(want.dtype)[:arena], want), f.name
    # host errors: a shard table may only be left out together with the permutation, and P must then be the
    # number of rollout shards
    with pytest.raises(binding.DcError) as e:
        binding.dc_plan(prm, d.source, d.seq_len, d.perm, None, d.capacity, d.dst_tok_off, shard_tok_off, shard_mb_off,
                        d.mb_seq_off, d.cu_seqlens, d.n_mb, ws, ws_bytes, d.status)
    assert e.value.code == binding.DC_ERR_INVALID_ARG
    with pytest.raises(binding.DcError) as e:
        binding.dc_plan(prm4, d.source, d.seq_len, None, None, d.capacity, d.dst_tok_off, st4, sm4,
                        d.mb_seq_off, d.cu_seqlens, d.n_mb, ws, ws_bytes, d.status)
    assert e.value.code == binding.DC_ERR_INVALID_ARG


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_repack_full_config(cfg):
    """dc_repack itself (one call: plan, then gather) on the large configurations, every output against the oracle
    and bit-equal to dc_plan followed by dc_gather."""
    torch, binding, runner = _gpu()
    w = workloads.make_workload(cfg)
    print(f"[parity] dc_repack config {cfg}: N={w.n_seq} T={w.total_tokens}", flush=True)
    d = runner.DeviceBatch(w, poison=True)
    d.group_advantage(); d.balance(); d.repack()
    torch.cuda.synchronize()
    compare_step(d, w)
    two = runner.DeviceBatch(w, poison=True)
    two.step()
    torch.cuda.synchronize()
    assert torch.equal(d.cu_seqlens, two.cu_seqlens) and torch.equal(d.dst_tok_off, two.dst_tok_off)
    for k, v in d.dst_fields.items():
        assert torch.equal(v, two.dst_fields[k]), k


# ---------------------------------------------------------------- per-token advantages made by the gather
def check_gather_advantage(w, align=1, cap=0, label="", against_copy=False):
    """dc_gather_advantage: the training-layout advantage field straight from adv_seq and the mask, against
    the oracle's definition (broadcast in the rollout layout, then gathered as one more field)."""
    torch, binding, runner = _gpu()
    print(f"[parity] gather_advantage {label or w.name}: N={w.n_seq} P={w.n_shards} T={w.total_tokens} "
          f"align={align} cap={cap}", flush=True)
    d = runner.DeviceBatch(w, align_tokens=align, cap=cap, poison=True)
    d.step_no_rollout_adv()
    torch.cuda.synchronize()
    assert d.read_status() == 0
    bal, adv, adv_tok, pl = oracle_step(w, align, cap)
    assert np.array_equal(d.perm.cpu().numpy(), bal.perm)
    np.testing.assert_allclose(d.adv_seq.cpu().numpy(), adv, rtol=RTOL, atol=ATOL)
    assert np.array_equal(d.dst_tok_off.cpu().numpy(), pl.dst_tok_off)
    for t in d.adv_tok_src:                                   # no per-token data in the rollout layout
        assert not t.any()
    arena = d.capacity
    valid = np.zeros(arena, bool)
    for k in range(w.n_shards):
        valid[pl.shard_tok_off[k]: pl.shard_tok_off[k] + bal.shard_load[k]] = True
    for f in w.fields:                                        # the other fields (the mask among them) as ever
        want = oracle.gather(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, f.shards, pl.dst_tok_off, arena)
        got = d.dst_fields[f.name].cpu().numpy().view(want.dtype)
        assert np.array_equal(got[valid], want[valid]), f.name
        poison = np.frombuffer(bytes([0x5A] * f.elem_bytes), dtype=want.dtype)[0]
        assert np.all(got[~valid] == poison), f.name
    want = oracle.gather(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, adv_tok, pl.dst_tok_off, arena)
    got = d.dst_fields["adv_tok"].cpu().numpy().view(np.float32)
    np.testing.assert_allclose(got[valid], want[valid], rtol=RTOL, atol=ATOL)
    assert np.all(got[~valid].view(np.uint32) == 0x5A5A5A5A)  # padding and the arena's tail are not written
    mask_dst = d.dst_fields["mask"].cpu().numpy()
    assert not got.view(np.uint32)[valid & (mask_dst == 0)].any()       # +0.0 exactly where no loss is taken
    # every token of a slot carries the bits of ITS sequence's advantage
    g_adv = d.adv_seq.cpu().numpy().view(np.uint32)
    for j in np.random.default_rng(2).integers(0, w.n_seq, 64) if w.n_seq else []:
        i = bal.perm[j]
        seg = got.view(np.uint32)[pl.dst_tok_off[j]: pl.dst_tok_off[j] + w.seq_len[i]]
        m = mask_dst[pl.dst_tok_off[j]: pl.dst_tok_off[j] + w.seq_len[i]]
        assert np.all(seg[m != 0] == g_adv[i])
    if against_copy:                                          # and the arena equals the copied one bit for bit
        d2 = runner.DeviceBatch(w, align_tokens=align, cap=cap, poison=True)
        d2.step_fused()
        torch.cuda.synchronize()
        for k in d.dst_fields:
            assert torch.equal(d.dst_fields[k], d2.dst_fields[k]), k
    return d


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_gather_advantage_full_config(cfg):
    check_gather_advantage(workloads.make_workload(cfg), label=f"config {cfg}", against_copy=cfg in (2, 4, 5))


def test_gather_advantage_shapes():
    rng = np.random.default_rng(21)
    # many slots per tile (slots staged in LDS), several passes per tile, rollout shards, padding between shards
    check_gather_advantage(_custom(rng.integers(1, 9, 8192), 8, 16, 64, n_src=4), label="lengths 1..8", against_copy=True)
    check_gather_advantage(_custom(np.ones(4096, np.int32), 4, 64, 7, n_src=2), align=5, label="all length 1")
    check_gather_advantage(_custom(rng.integers(1, 3000, 1000), 5, 8, 4096, n_src=2), align=3, label="N=1000 align 3")
    check_gather_advantage(_custom(rng.integers(1, 200, 2), 2, 2, 512), label="N=2")
    check_gather_advantage(_custom(rng.integers(1, 70000, 63 * 3), 3, 63, 70000), align=4096, label="P=63 align 4096")
    # records next to LDS-staged tiles, narrow fields riding
    lens = np.concatenate([rng.integers(3500, 4500, 8192), rng.integers(1, 120, 8192)])
    rng.shuffle(lens)
    check_gather_advantage(_custom(lens, 16, 64, 16384, n_src=2), label="8192 long + 8192 short", against_copy=True)
    # the mask is the only field; mask bytes other than 0 / 1 select like 1
    w = _custom(rng.integers(1, 900, 512), 8, 4, 4096, fields=())
    w.fields[0].shards[0][::3] *= 0x80
    check_gather_advantage(w, label="mask only, bytes 0 / 1 / 0x80")
    # sequences of 2^24 tokens
    L = 1 << 24
    check_gather_advantage(_custom(np.array([L, 5, L - 3, 100], np.int32), 2, 2, 1 << 25, fields=("i32",)),
                           label="sequences of 2^24 tokens")


# ---------------------------------------------------------------- reverse path
def check_scatter(w, label=""):
    """gather, then scatter the training arenas back: every rollout buffer must equal what the
    oracle's scatter writes (bit-exact), gaps between sequences untouched."""
    torch, binding, runner = _gpu()
    print(f"[parity] scatter {label or w.name}: N={w.n_seq} T={w.total_tokens}", flush=True)
    d = runner.DeviceBatch(w)
    d.step()
    d.prepare_scatter()
    d.scatter()
    torch.cuda.synchronize()
    assert d.read_status() == 0
    bal = oracle.balance(w.seq_len, w.n_shards)
    pl = oracle.plan(w.seq_len, bal.perm, bal.shard_seq_off, w.token_budget)
    for name in d.back_names:
        arena = d.dst_fields[name].cpu().numpy()             # what the gather produced (checked elsewhere)
        blank = [np.full(int(t), {1: 0x5A, 2: 0x5A5A, 4: 0x5A5A5A5A}[arena.dtype.itemsize], arena.dtype)
                 for t in w.src_shard_tokens]
        want = oracle.scatter(w.seq_len, bal.perm, w.src_tok_off, w.src_shard_seq_off, arena, pl.dst_tok_off, blank)
        for s_, (g, x) in enumerate(zip(d.back_fields[name], want)):
            assert np.array_equal(g.cpu().numpy(), x), (name, s_)
    # and the round trip restores the rollout payload itself
    for f in w.fields:
        for s_, src in enumerate(f.shards):
            got = d.back_fields[f.name][s_].cpu().numpy().view(src.dtype)
            valid = np.zeros(len(src), bool)
            for i in range(w.src_shard_seq_off[s_], w.src_shard_seq_off[s_ + 1]):
                valid[w.src_tok_off[i]: w.src_tok_off[i] + w.seq_len[i]] = True
            assert np.array_equal(got[valid], src[valid]), (f.name, s_)
    return d


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_scatter_full_config(cfg):
    check_scatter(workloads.make_workload(cfg), label=f"config {cfg}")


def test_scatter_shapes():
    rng = np.random.default_rng(31)
    check_scatter(_custom(rng.integers(1, 9, 8192), 8, 16, 64, n_src=4), label="lengths 1..8")
    check_scatter(_custom(rng.integers(1, 3000, 1000), 5, 8, 4096, n_src=2), label="N=1000")
    check_scatter(_custom(rng.integers(1, 200, 2), 2, 2, 512), label="N=2")
    lens = np.concatenate([rng.integers(3500, 4500, 8192), rng.integers(1, 120, 8192)])
    rng.shuffle(lens)
    check_scatter(_custom(lens, 16, 64, 16384, n_src=2), label="8192 long + 8192 short")


def test_scatter_padded_rows_and_errors():
    torch, binding, runner = _gpu()
    rng = np.random.default_rng(33)
    N, G, row = 512, 8, 700
    lens = rng.integers(1, row + 1, N).astype(np.int32)
    w = _custom(lens, G, 8, 4096, n_src=2)
    per = N // 2
    w.src_tok_off = ((np.arange(N) % per) * row + rng.integers(0, row - lens + 1)).astype(np.int64)
    w.src_shard_tokens = np.array([per * row, per * row], np.int64)
    for f in w.fields:
        f.shards = [rng.integers(0, 200, per * row).astype(f.shards[0].dtype) for _ in range(2)]
    check_scatter(w, label="padded rows")
    # overlapping sequences in the rollout layout are refused (nothing of the first one is written)
    d = runner.DeviceBatch(w)
    d.step(); d.prepare_scatter(); torch.cuda.synchronize()
    d.src_tok_off[1] = d.src_tok_off[0]
    d.scatter(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT
    # a slot beyond the arena is refused
    d = runner.DeviceBatch(w)
    d.step(); d.prepare_scatter(); torch.cuda.synchronize()
    d.dst_tok_off[3] = d.capacity
    d.scatter(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_OVERFLOW
    # perm that names a sequence twice (and so another one never) is refused
    d = runner.DeviceBatch(w)
    d.step(); d.prepare_scatter(); torch.cuda.synchronize()
    d.perm[5] = d.perm[9]
    d.scatter(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT


# ---------------------------------------------------------------- PPO advantage stage (GAE)
GAE_RTOL, GAE_ATOL = 1e-5, 1e-6          # both sides: float64 arithmetic, one rounding to float32


def _with_ppo_fields(w, seed=0):
    """Give a hand-shaped workload the float32 fields the PPO advantage stage reads."""
    rng = np.random.default_rng(seed)
    for name, gen in (("value", lambda n: rng.standard_normal(n)),
                      ("old_logprob", lambda n: -np.abs(rng.standard_normal(n))),
                      ("ref_logprob", lambda n: -np.abs(rng.standard_normal(n)))):
        w.fields = [f for f in w.fields if f.name != name]
        w.fields.append(workloads.Field(name, 4, [gen(int(t)).astype(np.float32) for t in w.src_shard_tokens]))
    return w


def check_gae(w, gamma, lam, kl_coef, label=""):
    torch, binding, runner = _gpu()
    print(f"[parity] gae {label or w.name}: N={w.n_seq} T={w.total_tokens} gamma={gamma} lambda={lam} kl={kl_coef}",
          flush=True)
    d = runner.DeviceBatch(w)
    d.prepare_gae()
    d.gae(gamma, lam, kl_coef)
    torch.cuda.synchronize()
    assert d.read_status() == 0
    f32 = lambda name: [a.view(np.float32) for a in w.field_by_name(name).shards]
    want_adv, want_ret = oracle.gae(w.reward, w.seq_len, w.src_tok_off, w.src_shard_seq_off, w.src_shard_tokens,
                                    f32("value"), w.field_by_name("mask").shards, gamma, lam, kl_coef,
                                    f32("old_logprob") if kl_coef else None, f32("ref_logprob") if kl_coef else None)
    for s_ in range(w.n_src_shards):
        inside = np.zeros(int(w.src_shard_tokens[s_]), bool)
        for i in range(w.src_shard_seq_off[s_], w.src_shard_seq_off[s_ + 1]):
            inside[w.src_tok_off[i]: w.src_tok_off[i] + w.seq_len[i]] = True
        m = w.field_by_name("mask").shards[s_] != 0
        for got_t, want in ((d.gae_adv[s_], want_adv[s_]), (d.gae_ret[s_], want_ret[s_])):
            got = got_t.cpu().numpy()
            np.testing.assert_allclose(got[inside], want[inside], rtol=GAE_RTOL, atol=GAE_ATOL)
            assert not got[inside & ~m].view(np.uint32).any()        # +0.0 exactly where no loss
            assert np.isnan(got[~inside]).all()                      # elements of no sequence: untouched
    return d


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_gae_full_config(cfg):
    w = workloads.make_workload(cfg)
    check_gae(w, 1.0, 0.95, 0.0, label=f"config {cfg}")
    check_gae(w, 0.99, 0.9, 0.05, label=f"config {cfg} with KL penalty")


def test_gae_shapes_and_special_cases():
    rng = np.random.default_rng(41)
    w = _with_ppo_fields(_custom(rng.integers(1, 9, 8192), 8, 16, 64, n_src=4))
    check_gae(w, 1.0, 1.0, 0.0, label="lengths 1..8, gamma=lambda=1")
    check_gae(w, 0.9, 0.0, 0.1, label="lengths 1..8, lambda=0")
    w = _with_ppo_fields(_custom(rng.integers(1, 3000, 1000), 5, 8, 4096, n_src=2))
    check_gae(w, 0.97, 0.8, 0.02, label="N=1000")
    w = _with_ppo_fields(_custom(np.array([255, 256, 257, 1, 513, 4, 3, 1024]), 2, 2, 4096))
    check_gae(w, 1.0, 0.95, 0.0, label="block-edge lengths")
    # sequences without any loss-bearing token, and one whose loss-bearing tokens are all in the middle
    w = _with_ppo_fields(_custom(np.array([300, 700, 64, 1000]), 2, 2, 4096))
    mk = w.field_by_name("mask").shards[0]
    mk[:300] = 0
    mk[300:600] = 0; mk[700:1000] = 0
    check_gae(w, 0.99, 0.95, 0.0, label="fully and partly masked sequences")
    # long sequences are started by the grid's first workgroups, one per set of every (N/32)-th sequence: three
    # long ones in one set (two of equal length), one alone in its set, one in each rollout shard's tail
    lens = rng.integers(100, 600, 96)
    lens[[5, 8, 11, 0, 95]] = [9000, 12000, 12000, 5000, 4096]
    w = _with_ppo_fields(_custom(lens, 8, 8, 16384, n_src=2))
    check_gae(w, 0.99, 0.95, 0.03, label="long sequences among short ones")
    check_gae(_with_ppo_fields(_custom(np.array([20000, 30, 17000]), 1, 1, 65536)), 1.0, 0.9, 0.0, label="N=3, two long")


def test_gae_padded_rows():
    rng = np.random.default_rng(43)
    N, row = 512, 700
    lens = rng.integers(1, row + 1, N).astype(np.int32)
    w = _custom(lens, 8, 8, 4096, n_src=2)
    per = N // 2
    w.src_tok_off = ((np.arange(N) % per) * row + rng.integers(0, row - lens + 1)).astype(np.int64)
    w.src_shard_tokens = np.array([per * row, per * row], np.int64)
    for f in w.fields:
        f.shards = [rng.integers(0, 2, per * row).astype(f.shards[0].dtype) for _ in range(2)]
    check_gae(_with_ppo_fields(w), 1.0, 0.95, 0.01, label="padded rows")


# ---------------------------------------------------------------- device-side error reporting
def test_device_status_codes():
    torch, binding, runner = _gpu()
    w = _custom(np.array([5, 9, 3, 7], np.int32), 2, 2, 8)          # 9 > budget 8
    d = runner.DeviceBatch(w)
    d.step(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_SEQ_EXCEEDS_BUDGET

    w = _custom(np.array([5, 4, 3, 7], np.int32), 2, 2, 64)
    d = runner.DeviceBatch(w)
    d.seq_len[1] = 0                                                   # zero-length sequence
    d.balance(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_ZERO_LENGTH_SEQ

    d = runner.DeviceBatch(w)
    d.capacity -= 1                                                    # arena one token short
    d.balance(); d.plan(); d.gather(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_OVERFLOW

    d = runner.DeviceBatch(w)
    d.balance(); torch.cuda.synchronize()
    d.perm[0] = d.perm[1]                                              # not a permutation
    d.plan(); d.gather(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT

    d = runner.DeviceBatch(w)
    d.group_off[1] = 5                                                 # group table not monotone
    d.group_advantage(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT

    # the PPO advantage stage refuses the same things, and writes nothing for the sequence it refuses
    wp = _with_ppo_fields(_custom(np.array([5, 4, 3, 7], np.int32), 2, 2, 64))
    d = runner.DeviceBatch(wp); d.prepare_gae()
    d.seq_len[2] = -3
    d.gae(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_ZERO_LENGTH_SEQ
    assert torch.isnan(d.gae_adv[0][9:12]).all() and not torch.isnan(d.gae_adv[0][:9]).any()
    d = runner.DeviceBatch(wp); d.prepare_gae()
    d.src_tok_off[3] = 14                                              # sequence 3 would end beyond its buffer
    d.gae(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT
    assert torch.isnan(d.gae_ret[0][12:]).all()


def test_device_status_codes_above_the_lds_limit():
    """The same refusals on the paths for more than DC_MAX_SEQ sequences."""
    torch, binding, runner = _gpu()
    rng = np.random.default_rng(35)
    lens = rng.integers(1, 200, 20480).astype(np.int32)
    w = _custom(lens, 4, 16, 4096, n_src=2, fields=("i32",))

    d = runner.DeviceBatch(w)
    d.seq_len[12345] = 0                                               # zero-length sequence
    d.balance(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_ZERO_LENGTH_SEQ

    d = runner.DeviceBatch(w)
    d.capacity -= 1                                                    # arena one token short
    d.balance(); d.plan(); d.gather(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_OVERFLOW

    d = runner.DeviceBatch(w, poison=True)
    d.balance(); torch.cuda.synchronize()
    d.perm[20000] = d.perm[3]                                          # not a permutation: the repeat moves nothing
    d.plan(); d.gather(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT

    d = runner.DeviceBatch(w)
    d.balance(); torch.cuda.synchronize()
    d.shard_seq_off[5] = d.shard_seq_off[4] - 1                        # shard table not monotone: nothing is planned
    d.plan(); d.gather(); torch.cuda.synchronize()
    assert d.read_status() == binding.DC_ERR_BAD_LAYOUT
    assert int(d.n_mb.item()) == 0

    w2 = _custom(np.concatenate([lens, [5000] * 16]).astype(np.int32), 4, 16, 4096, n_src=2, fields=("i32",))
    d = runner.DeviceBatch(w2)
    d.step(); torch.cuda.synchronize()                                 # 5000 > budget 4096
    assert d.read_status() == binding.DC_ERR_SEQ_EXCEEDS_BUDGET


def test_empty_batch():
    torch, binding, runner = _gpu()
    w = _custom(np.zeros(0, np.int32), 1, 4, 128)
    d = runner.DeviceBatch(w)
    d.step(); torch.cuda.synchronize()
    assert d.read_status() == 0
    assert int(d.n_mb.item()) == 0
    assert d.shard_seq_off.cpu().tolist() == [0] * 5
    assert d.shard_tok_off.cpu().tolist() == [0] * 5
    assert d.shard_mb_off.cpu().tolist() == [0] * 5
    # the same through the calls bench.py issues, on a shard count that would take the one-launch form
    for P in (4, 16):
        d = runner.DeviceBatch(_custom(np.zeros(0, np.int32), 1, P, 128))
        ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        for e in ev:
            e.record()
        d.step_two_calls(None, True, ev); torch.cuda.synchronize()       # (nothing is launched: the events stay as they are)
        assert d.read_status() == 0
        assert int(d.n_mb.item()) == 0
        assert d.shard_seq_off.cpu().tolist() == [0] * (P + 1)
        assert d.shard_tok_off.cpu().tolist() == [0] * (P + 1)
