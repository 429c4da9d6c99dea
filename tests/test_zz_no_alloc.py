"""dc_repack_noalloc (the plan's workspace is a device array inside the library: the call allocates
nothing) against dc_repack with a caller's workspace: every output bit for bit, on two calls in a
row, the second with a smaller input, so the second call finds the first one's tables in the array.
The comparison runs through the C-ABI on an MI355X; the size check needs no GPU."""
import pytest

from paper_2507_13833_amd import workloads

PLAN_OUTPUTS = ("dst_tok_off", "shard_tok_off", "shard_mb_off", "n_mb")


def _one(cfg, torch, runner):
    w = workloads.make_workload(cfg)
    print(f"[noalloc] config {cfg}: N={w.n_seq} T={w.total_tokens}", flush=True)
    want = runner.DeviceBatch(w, poison=True)
    want.group_advantage(); want.balance(); want.repack()
    got = runner.DeviceBatch(w, poison=True)
    got.group_advantage(); got.balance(); got.repack_noalloc()
    torch.cuda.synchronize()
    assert want.read_status() == 0 and got.read_status() == 0
    M = int(want.n_mb.item())
    for name in PLAN_OUTPUTS:
        assert torch.equal(getattr(want, name), getattr(got, name)), name
    assert torch.equal(want.mb_seq_off[:M + 1], got.mb_seq_off[:M + 1])
    assert torch.equal(want.cu_seqlens[:w.n_seq + M], got.cu_seqlens[:w.n_seq + M])
    for name, arena in want.dst_fields.items():
        assert torch.equal(arena, got.dst_fields[name]), name      # poison outside the shards included
    return got


@pytest.mark.gpu
def test_repack_noalloc_matches_repack_twice_in_a_row():
    import torch
    from paper_2507_13833_amd import binding, runner
    binding.load()
    assert torch.cuda.is_available()
    _one(3, torch, runner)          # 24 M tokens: fills 1.7 MB of the array
    _one(1, torch, runner)          # then 0.24 M tokens over the same array


def test_repack_noalloc_rejects_sizes_beyond_its_array():
    """Host-side check only: returns before anything touches a GPU."""
    from paper_2507_13833_amd import binding as B
    B.load()
    prm = B.make_params(16, 4, 1 << 20)
    src = B.Source([0, 16], [1 << 20], 0x1000)
    too_many = 200_000_000                                   # tokens of capacity whose tables exceed 8 MiB
    assert B.dc_workspace_bytes(prm, too_many) > B.DC_REPACK_NOALLOC_WS_BYTES
    with pytest.raises(B.DcError) as e:                     # fails before anything is enqueued or dereferenced
        B.dc_repack_noalloc(prm, src, 0x1000, 0x1000, 0x1000, B.Fields([]), too_many, 0x1000, 0x1000, 0x1000, 0x1000,
                            0x1000, 0x1000, 0x1000, stream=0)
    assert e.value.code == B.DC_ERR_UNSUPPORTED_SIZE
