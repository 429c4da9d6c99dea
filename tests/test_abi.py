"""The C-ABI library loads and exports what include/dc.h declares; host-side argument
validation returns before anything touches a GPU (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

from paper_2507_13833_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2507_13833_amd import build
        build.build_lib()
    return B.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dc_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layouts_match_header():
    assert C.sizeof(B.dc_params) == 40
    assert B.dc_params.token_budget.offset == 16 and B.dc_params.eps.offset == 24
    assert C.sizeof(B.dc_source) == 32 and C.sizeof(B.dc_field) == 24
    text = open(os.path.join(ROOT, "include", "dc.h")).read()
    for name, val in (("DC_MAX_SEQ", B.DC_MAX_SEQ), ("DC_MAX_SEQ_LARGE", B.DC_MAX_SEQ_LARGE), ("DC_MAX_SHARDS", B.DC_MAX_SHARDS),
                      ("DC_MAX_FIELDS", B.DC_MAX_FIELDS), ("DC_MAX_SRC_SHARDS", B.DC_MAX_SRC_SHARDS)):
        assert re.search(rf"#define\s+{name}\s+{val}\b", text)
    codes = dict(re.findall(r"(DC_(?:OK|ERR_[A-Z_]+))\s*=\s*(\d+)", text))
    for k, v in codes.items():
        assert getattr(B, k) == int(v)


def test_strerror(lib):
    assert B.strerror(0) == "ok"
    assert "Algorithm 1" in B.strerror(B.DC_ERR_NOT_DIVISIBLE)
    assert all(B.strerror(c) for c in range(10))


FAKE = 0x1000          # never dereferenced: every call below fails validation first


def test_balance_host_errors(lib):
    with pytest.raises(B.DcError) as e:
        B.dc_balance(B.make_params(10, 4, 100), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_NOT_DIVISIBLE
    for prm, code in ((B.make_params(8, 0, 100), B.DC_ERR_INVALID_ARG),
                      (B.make_params(2050, 1025, 100), B.DC_ERR_UNSUPPORTED_SIZE),
                      (B.make_params(B.DC_MAX_SEQ + 64, 64, 100), B.DC_ERR_UNSUPPORTED_SIZE),
                      (B.make_params(8, 4, 0), B.DC_ERR_INVALID_ARG),
                      (B.make_params(8, 4, 100, cap=1), B.DC_ERR_INVALID_ARG),
                      (B.make_params(8, 4, 100, align_tokens=0), B.DC_ERR_INVALID_ARG),
                      (B.make_params(8, 4, 100, eps=-1.0), B.DC_ERR_INVALID_ARG)):
        with pytest.raises(B.DcError) as e:
            B.dc_balance(prm, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, stream=0)
        assert e.value.code == code
    with pytest.raises(B.DcError) as e:
        B.dc_balance(B.make_params(8, 4, 100), None, FAKE, FAKE, FAKE, FAKE, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG


def test_balance_ws_host_errors(lib):
    big = B.DC_MAX_SEQ * 4
    assert B.dc_balance_workspace_bytes(B.make_params(B.DC_MAX_SEQ, 64, 100)) == 0
    assert B.dc_balance_workspace_bytes(B.make_params(B.DC_MAX_SEQ_LARGE + 64, 64, 100)) == 0
    ws = B.dc_balance_workspace_bytes(B.make_params(big, 64, 100))
    assert ws >= 12 * big
    out = (FAKE,) * 5                                         # seq_len, perm, shard_seq_off, shard_of_seq, shard_load
    with pytest.raises(B.DcError) as e:                      # workspace too small
        B.dc_balance_ws(B.make_params(big, 64, 100), *out, 0x10000, ws - 1, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_WORKSPACE
    with pytest.raises(B.DcError) as e:                      # no workspace
        B.dc_balance_ws(B.make_params(big, 64, 100), *out, None, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # workspace misaligned
        B.dc_balance_ws(B.make_params(big, 64, 100), *out, 0x10010, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # more than 65535 sequences per shard
        B.dc_balance_ws(B.make_params(1 << 18, 2, 100), *out, 0x10000, 1 << 24, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_UNSUPPORTED_SIZE
    with pytest.raises(B.DcError) as e:                      # exactly one more than a shard may hold
        B.dc_balance_ws(B.make_params(2 * 65536, 2, 100), *out, 0x10000, 1 << 24, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_UNSUPPORTED_SIZE
    with pytest.raises(B.DcError) as e:                      # beyond DC_MAX_SEQ_LARGE
        B.dc_balance_ws(B.make_params(B.DC_MAX_SEQ_LARGE + 64, 64, 100), *out, 0x10000, 1 << 26, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_UNSUPPORTED_SIZE
    with pytest.raises(B.DcError) as e:                      # Algorithm 1's assertion
        B.dc_balance_ws(B.make_params(big + 1, 64, 100), *out, 0x10000, 1 << 24, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_NOT_DIVISIBLE
    with pytest.raises(B.DcError) as e:                      # dc_balance itself keeps its limit
        B.dc_balance(B.make_params(big, 64, 100), *out, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_UNSUPPORTED_SIZE


def test_plan_and_gather_host_errors(lib):
    prm = B.make_params(8, 4, 100)
    src = B.Source([0, 8], [64], FAKE)
    args = (FAKE,) * 6
    with pytest.raises(B.DcError) as e:                      # workspace too small
        B.dc_plan(prm, src, FAKE, FAKE, FAKE, 64, *args, 0x10000, 16, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_WORKSPACE
    with pytest.raises(B.DcError) as e:                      # workspace misaligned
        B.dc_plan(prm, src, FAKE, FAKE, FAKE, 64, *args, 0x10008, 1 << 20, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    bad_src = B.Source([0, 5], [64], FAKE)                    # rollout shards do not cover N
    with pytest.raises(B.DcError) as e:
        B.dc_plan(prm, bad_src, FAKE, FAKE, FAKE, 64, *args, 0x10000, 1 << 20, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    many = B.Source(list(range(0, 18)) + [8] * 0, [1] * 17, FAKE)
    with pytest.raises(B.DcError) as e:
        B.dc_plan(prm, many, FAKE, FAKE, FAKE, 64, *args, 0x10000, 1 << 20, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_UNSUPPORTED_SIZE

    ws = B.dc_workspace_bytes(prm, 64)
    assert ws > 0 and ws % 256 == 0
    f_bad_size = B.Fields([([0x2000], 0x3000, 3)])
    with pytest.raises(B.DcError) as e:
        B.dc_gather(prm, src, f_bad_size, 64, FAKE, 0x10000, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    f_misaligned = B.Fields([([0x2004], 0x3000, 4)])
    with pytest.raises(B.DcError) as e:
        B.dc_gather(prm, src, f_misaligned, 64, FAKE, 0x10000, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    nine = B.Fields([([0x2000], 0x3000, 4)] * 9)
    with pytest.raises(B.DcError) as e:
        B.dc_gather(prm, src, nine, 64, FAKE, 0x10000, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_UNSUPPORTED_SIZE
    with pytest.raises(B.DcError) as e:                      # repack validates fields before it plans
        B.dc_repack(prm, src, FAKE, FAKE, FAKE, f_bad_size, 64, *args, 0x10000, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG


def test_group_advantage_host_errors(lib):
    prm = B.make_params(8, 4, 100)
    src = B.Source([0, 8], [64], FAKE)
    with pytest.raises(B.DcError) as e:                      # more groups than sequences
        B.dc_group_advantage(prm, src, FAKE, FAKE, FAKE, 9, None, FAKE, None, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # per-token output without a mask
        B.dc_group_advantage(prm, src, FAKE, FAKE, FAKE, 2, None, FAKE, [0x4000], FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # misaligned per-token buffer
        B.dc_group_advantage(prm, src, FAKE, FAKE, FAKE, 2, [0x5000], FAKE, [0x4004], FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG


def test_fused_balance_advantage_host_errors(lib):
    src = B.Source([0, 8], [64], FAKE)
    out = (FAKE,) * 4                                         # perm, shard_seq_off, shard_of_seq, shard_load
    with pytest.raises(B.DcError) as e:                      # the balance half's check
        B.dc_balance_group_advantage(B.make_params(10, 4, 100), B.Source([0, 10], [64], FAKE), FAKE, *out,
                                     FAKE, FAKE, 2, None, FAKE, None, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_NOT_DIVISIBLE
    prm = B.make_params(8, 4, 100)
    with pytest.raises(B.DcError) as e:                      # the advantage half's: more groups than sequences
        B.dc_balance_group_advantage(prm, src, FAKE, *out, FAKE, FAKE, 9, None, FAKE, None, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # per-token output without a mask
        B.dc_balance_group_advantage(prm, src, FAKE, *out, FAKE, FAKE, 2, None, FAKE, [0x4000], FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # no permutation output
        B.dc_balance_group_advantage(prm, src, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 2, None, FAKE, None, FAKE,
                                     stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG


def test_scatter_host_errors(lib):
    prm = B.make_params(8, 4, 100)
    src = B.Source([0, 8], [64], FAKE)
    ws = B.dc_scatter_workspace_bytes(prm, src)
    assert ws > 0 and ws % 256 == 0
    ok = B.Fields([([0x2000], 0x3000, 4)])
    with pytest.raises(B.DcError) as e:                      # workspace too small
        B.dc_scatter(prm, src, FAKE, FAKE, ok, 64, FAKE, 0x10000, 16, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_WORKSPACE
    with pytest.raises(B.DcError) as e:                      # workspace misaligned
        B.dc_scatter(prm, src, FAKE, FAKE, ok, 64, FAKE, 0x10010, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # rollout buffer not 16-byte aligned
        B.dc_scatter(prm, src, FAKE, FAKE, B.Fields([([0x2008], 0x3000, 2)]), 64, FAKE, 0x10000, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # no permutation
        B.dc_scatter(prm, src, FAKE, None, ok, 64, FAKE, 0x10000, ws, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    # a rollout shard table that does not cover N has no workspace size
    assert B.dc_scatter_workspace_bytes(prm, B.Source([0, 5], [64], FAKE)) == 0


def test_gather_advantage_host_errors(lib):
    prm = B.make_params(8, 4, 100)
    src = B.Source([0, 8], [64], FAKE)
    ws = B.dc_workspace_bytes(prm, 64)
    fields = B.Fields([([0x2000], 0x3000, 4), ([0x4000], 0x5000, 1)])
    call = lambda f, mask_field, perm=FAKE, adv=FAKE, dst=0x6000, ws_ptr=0x10000, ws_bytes=ws: B.dc_gather_advantage(
        prm, src, f, mask_field, perm, adv, dst, 64, FAKE, ws_ptr, ws_bytes, FAKE, stream=0)
    for mask_field in (0, 2, -1):                            # a 4-byte field, beyond the table, negative
        with pytest.raises(B.DcError) as e:
            call(fields, mask_field)
        assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # no fields at all: no mask
        call(B.Fields([]), 0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # no per-sequence advantages
        call(fields, 1, adv=None)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # no permutation
        call(fields, 1, perm=None)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # advantage arena not 16-byte aligned
        call(fields, 1, dst=0x6004)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # workspace too small
        call(fields, 1, ws_bytes=16)
    assert e.value.code == B.DC_ERR_WORKSPACE


def test_gae_host_errors(lib):
    prm = B.make_params(8, 4, 100)
    src = B.Source([0, 8], [64], FAKE)
    buf = [0x4000]
    with pytest.raises(B.DcError) as e:                      # KL penalty without the log-prob fields
        B.dc_gae(prm, src, FAKE, FAKE, buf, buf, None, None, 1.0, 0.95, 0.1, buf, buf, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # misaligned output
        B.dc_gae(prm, src, FAKE, FAKE, buf, buf, None, None, 1.0, 0.95, 0.0, [0x4004], buf, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # NaN discount
        B.dc_gae(prm, src, FAKE, FAKE, buf, buf, None, None, float("nan"), 0.95, 0.0, buf, buf, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG
    with pytest.raises(B.DcError) as e:                      # no rewards
        B.dc_gae(prm, src, FAKE, None, buf, buf, None, None, 1.0, 0.95, 0.0, buf, buf, FAKE, stream=0)
    assert e.value.code == B.DC_ERR_INVALID_ARG


def test_product_does_not_reach_the_oracle():
    pkg = os.path.join(ROOT, "paper_2507_13833_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text, fn
                assert "dc_oracle" not in text, fn
    for fn in os.listdir(os.path.join(ROOT, "oracle")):
        if fn.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", fn)).read()
            assert "paper_2507_13833_amd" not in text and "libdc.so" not in text, fn
