"""The seeded input recipe: shapes, ranges and layout of the five synthetic workloads."""
import numpy as np
import pytest

from paper_2507_13833_amd import workloads


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_shapes_and_ranges(cfg):
    w = workloads.make_workload(cfg, prompts=64)
    w2 = workloads.make_workload(cfg, prompts=64)
    assert np.array_equal(w.seq_len, w2.seq_len) and np.array_equal(w.reward, w2.reward)
    for f, g in zip(w.fields, w2.fields):
        assert all(np.array_equal(a, b) for a, b in zip(f.shards, g.shards))
    lo, hi, rlo, rhi = {1: (64, 256, 16, 1024), 2: (128, 1024, 32, 4096), 3: (256, 2048, 64, 8192),
                        4: (256, 2048, 64, 8192), 5: (512, 4096, 64, 32768)}[cfg]
    r = w.seq_len - w.prompt_len
    assert w.prompt_len.min() >= lo and w.prompt_len.max() <= hi
    assert r.min() >= rlo and r.max() <= rhi
    assert w.n_seq % w.n_shards == 0 and w.seq_len.max() <= w.token_budget
    assert w.n_src_shards == (8 if cfg == 4 else 1)
    for s in range(w.n_src_shards):
        a, b = w.src_shard_seq_off[s], w.src_shard_seq_off[s + 1]
        assert w.src_tok_off[a] == 0
        assert np.array_equal(np.diff(w.src_tok_off[a:b]), w.seq_len[a:b - 1])
        assert w.src_shard_tokens[s] == w.seq_len[a:b].sum()
        for f in w.fields:
            assert len(f.shards[s]) == w.src_shard_tokens[s] and f.shards[s].itemsize == f.elem_bytes
    names = [f.name for f in w.fields]
    assert names[0] == "token_id" and names[-1] == "mask"
    assert w.payload_bytes_per_token == {1: 9, 2: 9, 3: 17, 4: 17, 5: 19}[cfg]
    # mask: 0 on prompts; response starts with 1
    m = w.field_by_name("mask").shards[0]
    a, b = w.src_shard_seq_off[0], w.src_shard_seq_off[1]
    for i in range(a, min(b, a + 40)):
        t0 = w.src_tok_off[i]
        assert not m[t0:t0 + w.prompt_len[i]].any()
        assert m[t0 + w.prompt_len[i]] == 1
        if cfg != 5:
            assert m[t0 + w.prompt_len[i]: t0 + w.seq_len[i]].all()


def test_full_size_token_counts():
    # headline sizes (lengths only are cheap to check): N, P, mean length
    for cfg, n in ((3, 8192), (5, 16384)):
        sh = workloads._SHAPES[cfg]
        assert sh["prompts"] * sh["G"] == n


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625], np.float32)
    b = workloads.f32_to_bf16_bits(x)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0)
    assert b.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x4049]


def test_sequence_lengths_are_the_workloads_own():
    """sequence_lengths draws what make_workload draws first: the same lengths without the payload."""
    for cfg in (1, 3, 5):
        w = workloads.make_workload(cfg, prompts=24)
        assert np.array_equal(workloads.sequence_lengths(cfg, w.n_seq), w.seq_len)
    big = workloads.sequence_lengths(5, 65536)
    assert big.shape == (65536,) and big.dtype == np.int32 and big.min() >= 512 + 64 and big.max() <= 4096 + 32768
    with pytest.raises(ValueError):
        workloads.sequence_lengths(5, 100)                 # not a multiple of the group size
