"""The C-ABI library loads, exports what include/tidar.h declares, and validates arguments on the host (no GPU)."""
import ctypes as C
import os
import re

import pytest

import tidar_inputs as TI

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def T():
    import paper_2511_08923_amd as T
    return T


def _declared():
    text = open(os.path.join(ROOT, "include", "tidar.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tidar_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(T):
    names = _declared()
    assert len(names) >= 15
    lib = C.CDLL(T.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(T.EXPORTS) == names
    for n in names:                      # the binding carries the same names
        assert hasattr(T, n), n


def test_strerror(T):
    assert T.tidar_strerror(0) == "ok"
    assert "workspace" in T.tidar_strerror(2)


def test_create_rejects_bad_shapes(T):
    good = T.make_config(TI.TINY, T.TIDAR_F32, max_k=4)
    T.tidar_destroy(T.tidar_create(good))
    for field, val in [("page_size", 8), ("max_k", 17), ("n_kv_heads", 3), ("dtype", 7), ("head_dim", 130),
                       ("mask_token_id", 512), ("vocab", 500)]:
        cfg = T.make_config(TI.TINY, T.TIDAR_F32, max_k=4)
        setattr(cfg, field, val)
        with pytest.raises(T.TidarError) as e:
            T.tidar_create(cfg)
        assert e.value.status == 1
    bf = T.make_config(TI.TINY, T.TIDAR_BF16, max_k=4)      # the bf16 path needs head_dim 128
    with pytest.raises(T.TidarError):
        T.tidar_create(bf)
    T.tidar_destroy(T.tidar_create(T.make_config(TI.SHAPE_8B, T.TIDAR_BF16)))


def test_workspace_bytes_monotone_and_validated(T):
    ctx = T.tidar_create(T.make_config(TI.SHAPE_8B, T.TIDAR_BF16, max_k=16, max_batch=4))
    a = T.tidar_workspace_bytes(ctx, 1, 16, 4096)
    b = T.tidar_workspace_bytes(ctx, 4, 16, 8192)
    assert 0 < a <= b
    for args in [(0, 16, 10), (5, 16, 10), (1, 17, 10), (1, 0, 10), (1, 4, -1)]:
        with pytest.raises(T.TidarError):
            T.tidar_workspace_bytes(ctx, *args)
    T.tidar_destroy(ctx)


def test_step_rejects_null_and_capacity_before_any_launch(T):
    ctx = T.tidar_create(T.make_config(TI.TINY, T.TIDAR_F32, max_k=4))
    lib = C.CDLL(T.LIB_PATH)
    lib.tidar_step.restype = C.c_int32
    # null weights/cache -> EINVAL without touching a device
    mode = T.make_mode()
    rc = T._lib.tidar_step(ctx, None, None, 1, None, None, 4, C.byref(mode), None, None, None, None, 0, None, 0, None)
    assert rc == 1
    # fabricate non-null (never dereferenced on the host) pointers to reach the capacity / workspace checks
    dummy = (C.c_void_p * 4)(8, 8, 8, 8)
    arr = C.cast(dummy, C.POINTER(C.c_void_p))
    w = T.tidar_weights(8, 8, 8, arr, arr, arr, arr, arr, arr)
    kv = T.tidar_kv_cache(8, 8, 8, 2, 2)                      # 2 pages = 32 positions
    rc = T._lib.tidar_step(ctx, C.byref(w), C.byref(kv), 1, 8, 8, 4, C.byref(mode), 8, 8, 8, None, 30, 8, 1 << 30, None)
    assert rc == 3                                              # 30 + 4 > 32
    rc = T._lib.tidar_step(ctx, C.byref(w), C.byref(kv), 1, 8, 8, 4, C.byref(mode), 8, 8, 8, None, 8, 8, 16, None)
    assert rc == 2                                              # workspace of 16 bytes
    rc = T._lib.tidar_step(ctx, C.byref(w), C.byref(kv), 1, 8, 8, 5, C.byref(mode), 8, 8, 8, None, 8, 8, 1 << 30, None)
    assert rc == 1                                              # k above max_k
    bad = T.make_mode(sample=True, temperature=0.0)
    rc = T._lib.tidar_step(ctx, C.byref(w), C.byref(kv), 1, 8, 8, 4, C.byref(bad), 8, 8, 8, None, 8, 8, 1 << 30, None)
    assert rc == 1
    # a layer's pages beyond 2 GiB cannot be addressed with 32-bit offsets: 4 heads x 16 x 32 x 4 B = 8 KiB per page
    huge = T.tidar_kv_cache(8, 8, 8, 2, (1 << 31) // 8192)
    rc = T._lib.tidar_step(ctx, C.byref(w), C.byref(huge), 1, 8, 8, 4, C.byref(mode), 8, 8, 8, None, 8, 8, 1 << 30, None)
    assert rc == 1
    T.tidar_destroy(ctx)


def test_pack_weight_validation(T):
    assert T.tidar_packed_weight_bytes(T.TIDAR_BF16, 64, 128) == 64 * 128 * 2
    assert T._lib.tidar_pack_weight(T.TIDAR_BF16, 8, 20, 64, 8, 32, 0, 1, None) == 1       # rows not multiple of 16
    assert T._lib.tidar_pack_weight(T.TIDAR_BF16, 8, 32, 48, 8, 32, 0, 1, None) == 1       # cols not multiple of 32
    assert T._lib.tidar_pack_weight(T.TIDAR_BF16, 8, 32, 64, 8, 32, 1, 1, None) == 1       # does not fit


def test_select_block_len_follows_the_row_budget(T):
    """Host-only policy: largest power-of-two block whose rows batch*k*(k+1) fit the budget (default 160 rows)."""
    ctx = T.tidar_create(T.make_config(TI.SHAPE_8B, T.TIDAR_BF16, max_k=16, max_batch=32))
    try:
        assert T.tidar_select_block_len(ctx, 1) == 8            # 72 rows fit, 272 do not
        assert T.tidar_select_block_len(ctx, 1, row_budget=272) == 16
        assert T.tidar_select_block_len(ctx, 1, row_budget=271) == 8
        assert T.tidar_select_block_len(ctx, 4) == 4            # 80 rows
        assert T.tidar_select_block_len(ctx, 8) == 4            # 160 rows, exactly the budget
        assert T.tidar_select_block_len(ctx, 9) == 2
        assert T.tidar_select_block_len(ctx, 32) == 1           # 2*3*32 = 192 > 160
        assert T.tidar_select_block_len(ctx, 1, k_cap=4, row_budget=10 ** 6) == 4
        assert T.tidar_select_block_len(ctx, 0) == 0
        assert T.tidar_select_block_len(None, 1) == 0
        for batch in range(1, 40):                               # brute force over the definition
            for budget in (1, 5, 20, 72, 160, 1000, 10 ** 5):
                want = max([k for k in (1, 2, 4, 8, 16) if k == 1 or batch * k * (k + 1) <= budget])
                assert T.tidar_select_block_len(ctx, batch, 0, budget) == want
    finally:
        T.tidar_destroy(ctx)
    small = T.tidar_create(T.make_config(TI.TINY, T.TIDAR_F32, max_k=4))
    assert T.tidar_select_block_len(small, 1, row_budget=10 ** 6) == 4   # never above the context's max_k
    T.tidar_destroy(small)
