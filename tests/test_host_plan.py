"""Host logic that needs no GPU: the launch plans the library derives from a shape (the
decode path's strips and K split, the tiled path's tile mix and K parts) and the argument
checks of the loss entry point."""
import ctypes

import pytest

import workloads as wl


@pytest.fixture(scope="module")
def L():
    import paper_2312_03788_amd as sqp
    return sqp.lib()


def _decode_plan(L, M, N, K, group):
    nw, split, kspg = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    L.sqp_debug_decode_plan(M, N, K, group, ctypes.byref(nw), ctypes.byref(split), ctypes.byref(kspg))
    return nw.value, split.value, kspg.value


def _tile_plan(L, M, N, K, cus=256):
    full, half, ks = ctypes.c_long(), ctypes.c_long(), ctypes.c_int()
    L.sqp_debug_prefill_plan(M, N, K, cus, ctypes.byref(full), ctypes.byref(half), ctypes.byref(ks))
    return full.value, half.value, ks.value


def test_decode_plan_invariants(L):
    shapes = [s for m in ("7b", "13b", "34b") for s in wl.MODEL_SHAPES[m]] + [(128, 8), (1024, 264), (65536, 64)]
    for (K, N) in shapes:
        for group in (32, 64, 128, 256):
            if K % group:
                continue
            nw, split, kspg = _decode_plan(L, 16, N, K, group)
            chunk = 128 if group % 128 == 0 else group
            chunks = K // chunk
            assert nw in (2, 4) and kspg == {32: 1, 64: 2}.get(group, 4)
            assert 1 <= split <= max(1, chunks // 4)          # at least four chunks per workgroup
            tiles = -(-N // (64 * nw))
            if tiles <= 128:
                # narrow layers: never more than one workgroup per compute unit, and as many as
                # the chunk bound allows below that
                assert tiles * split <= 256
                if split < max(1, chunks // 4):
                    assert tiles * (split + 1) > 256
            elif split < max(1, chunks // 4):
                assert abs(tiles * split - 704) <= tiles
            if nw == 2:                                        # only narrow layers, and not with a long K range
                # (groups of 128, where a launch can take two chunks per iteration: up to 40 tiles
                # if each workgroup then still walks 16 chunks)
                assert -(-N // 256) <= ((40 if group == 128 else 32) if group % 128 == 0 else 24)
                if -(-N // 256) > 32:
                    assert chunks // split >= 16
                if group % 128 == 0 and not (group == 128 and chunks // split >= 16):
                    assert chunks <= 24 * split
    assert _decode_plan(L, 16, 1024, 1024, 24)[2] == 0        # other group sizes: generic kernel


def test_decode_plan_34b_values(L):
    """The plans the benchmark's launches run with (they are part of its configuration)."""
    got = {(K, N): _decode_plan(L, 16, N, K, 128)[:2] for (K, N) in wl.MODEL_SHAPES["34b"]}
    assert got == {(8192, 10240): (2, 3), (8192, 8192): (2, 4), (8192, 44032): (4, 4), (22016, 8192): (2, 4)}


def test_decode_slice_choice(L):
    """Which calls take the column-slice kernel: groups of 128 only; up to 8 rows, 64-column
    slices on the wide layers, 32-column slices on the narrow ones unless K is long and the
    slices are few; more than 8 rows only where x is small enough (short K) and the layer not
    too wide; the 16-row calls of the benchmark sweep (K = 8192 and 22016) keep the strip kernel."""
    L.sqp_debug_decode_slice_choice.restype = ctypes.c_int
    ch = lambda M, K, N, g=128: L.sqp_debug_decode_slice_choice(M, N, K, g)
    assert [ch(1, K, N) for (K, N) in wl.MODEL_SHAPES["34b"]] == [1, 0, 1, 0]
    assert [ch(4, K, N) for (K, N) in wl.MODEL_SHAPES["34b"]] == [1, 0, 1, 0]
    assert [ch(8, K, N) for (K, N) in wl.MODEL_SHAPES["34b"]] == [1, 0, 1, -1]     # K = 22016: two blocks of x are too many
    assert [ch(1, K, N) for (K, N) in wl.MODEL_SHAPES["13b"]] == [1, 0, 1, -1]
    assert [ch(4, K, N) for (K, N) in wl.MODEL_SHAPES["7b"]] == [1, 0, 1, -1]
    assert [ch(12, K, N) for (K, N) in wl.MODEL_SHAPES["34b"]] == [1, 0, -1, -1]
    assert [ch(9, K, N) for (K, N) in wl.MODEL_SHAPES["13b"]] == [1, 0, 1, -1]
    assert [ch(12, K, N) for (K, N) in wl.MODEL_SHAPES["7b"]] == [1, 0, 1, -1]
    assert [ch(16, K, N) for (K, N) in wl.MODEL_SHAPES["7b"]] == [1, 0, 1, -1]      # short K: x is small
    assert [ch(16, K, N) for (K, N) in wl.MODEL_SHAPES["13b"]] == [1, -1, -1, -1]
    for (K, N) in wl.MODEL_SHAPES["34b"]:
        assert ch(13, K, N) == -1 and ch(16, K, N) == -1 and ch(64, K, N) == -1
        assert ch(1, K, N, 64) == -1 and ch(1, K, N, 256) == -1
    assert ch(1, 4096, 1024) == -1 and ch(1, 128, 8) == -1      # few slices: the strip kernel and its K split


def test_slice_calls_need_no_workspace(L):
    """A call that takes the column-slice kernel reports no workspace; the 16-row calls of the
    34B sweep (strip kernel, K split across workgroups) report tickets plus partial sums."""
    L.sqp_debug_decode_slice_choice.restype = ctypes.c_int
    L.sqp_w4a16_gemm_workspace_bytes.restype = ctypes.c_size_t
    for model in ("7b", "13b", "34b"):
        for (K, N) in wl.MODEL_SHAPES[model]:
            for M in (1, 4, 8, 12, 16):
                need = L.sqp_w4a16_gemm_workspace_bytes(M, N, K, 128)
                if L.sqp_debug_decode_slice_choice(M, N, K, 128) >= 0:
                    assert need == 0
    for (K, N) in wl.MODEL_SHAPES["34b"]:
        assert L.sqp_w4a16_gemm_workspace_bytes(16, N, K, 128) > 512 << 10


def test_decode_plan_many_rows(L):
    """More than 32 rows: two strips per workgroup, the split of the 16-row plan."""
    for (K, N) in wl.MODEL_SHAPES["34b"]:
        tiles4, chunks = -(-N // 256), K // 128
        four_strip_split = min(256 // tiles4 if tiles4 <= 128 else (704 + tiles4 // 2) // tiles4, max(1, chunks // 4))
        assert _decode_plan(L, 48, N, K, 128)[:2] == (2, four_strip_split)
    assert _decode_plan(L, 64, 512, 256, 128)[:2] == (2, 1)            # short K: no split
    assert _decode_plan(L, 64, 65536, 256, 128)[:2] == (4, 1)


def test_decode_plan_small_model_values(L):
    """Shapes where the sweeps found the four-strip, rounded-up plan 10-25 % off the best."""
    assert _decode_plan(L, 16, 4096, 4096, 128)[:2] == (2, 8)      # narrow and short: two strips
    assert _decode_plan(L, 16, 5120, 5120, 128)[:2] == (2, 6)
    assert _decode_plan(L, 16, 4096, 11008, 128)[:2] == (2, 8)
    assert _decode_plan(L, 16, 5120, 13824, 128)[:2] == (2, 6)     # 40 two-strip tiles x 6 = 240 workgroups
    assert _decode_plan(L, 32, 5120, 13824, 128)[:2] == (2, 6)
    assert _decode_plan(L, 32, 8192, 22016, 128)[:2] == (2, 4)     # 17..32 rows: also with a long K
    assert _decode_plan(L, 16, 8192, 22016, 128)[:2] == (2, 4)     # up to 16 rows, groups of 128: two chunks per iteration, so too
    assert _decode_plan(L, 16, 8192, 22016, 256)[:2] == (4, 8)     # other groups: a long K keeps four strips
    assert _decode_plan(L, 32, 12288, 4096, 128)[:2] == (4, 5)     # 48 tiles: four strips
    assert _decode_plan(L, 16, 22016, 4096, 128)[:2] == (4, 2)     # 86 tiles: 172 workgroups, not 258


@pytest.mark.parametrize("shape", [1, 2])
def test_tile_plan_invariants(L, shape):
    """Both full-tile shapes (1: 128 x 512, 2: 256 x 256)."""
    bm, bn = (128, 512) if shape == 1 else (256, 256)
    L.sqp_debug_set_prefill_shape(shape)
    try:
        for M in (65, 128, 256, 300, 512, 1024, 2048, 4096):
            for (K, N) in wl.MODEL_SHAPES["34b"] + [(1024, 264), (256, 8), (8192, 256)]:
                for cus in (256, 304, 64):
                    full, half, ks = _tile_plan(L, M, N, K, cus)
                    tiles = -(-N // bn) * -(-M // bm)
                    assert full >= 0 and half >= 0 and ks >= 1
                    assert full + half // 2 == tiles and half % 2 == 0   # every tile exactly once
                    if ks >= 2:
                        assert full == 0 and 4 * tiles <= cus
                        assert half * ks <= cus                          # one round
                        assert K // 64 // ks >= 8                        # at least 8 stages per part
                    else:
                        assert full % cus == 0 or half == 0              # first launch: whole rounds only
                        assert half <= cus                               # the remainder is one round
    finally:
        L.sqp_debug_set_prefill_shape(0)


def test_tile_plan_bench_shapes(L):
    """The tile counts of the benchmark's M = 2048 launches are the same for both shapes."""
    for shape in (0, 1, 2):
        L.sqp_debug_set_prefill_shape(shape)
        try:
            assert _tile_plan(L, 2048, 8192, 8192) == (256, 0, 1)
            assert _tile_plan(L, 2048, 10240, 8192) == (256, 128, 1)
            assert _tile_plan(L, 2048, 44032, 8192) == (1280, 192, 1)
            assert _tile_plan(L, 4096, 8192, 22016) == (512, 0, 1)
            assert _tile_plan(L, 256, 8192, 8192) == (0, 64, 4)
        finally:
            L.sqp_debug_set_prefill_shape(0)


def test_quant_loss_argument_errors(L):
    P = ctypes.c_void_p
    good, odd, null = P(0x1000), P(0x1008), P(0)
    q = L.sqp_quant_loss
    assert q(4, 1024, 1024, 128, good, good, good, good, good, good, null, good, null) == -1
    assert q(0, 1024, 1024, 128, good, good, good, good, good, good, good, good, null) == -2
    assert q(4, 1024, 1024, 100, good, good, good, good, good, good, good, good, null) == -2
    assert q(4, 1024, 1024, 128, good, odd, good, good, good, good, good, good, null) == -3
    assert L.sqp_quant_loss_scratch_doubles(512, 8192) == 4 * 64
    assert L.sqp_quant_loss_scratch_doubles(129, 130) == 4
    assert L.sqp_quant_loss_scratch_doubles(0, 8) == 0


def test_mlp_entry_argument_errors(L):
    P = ctypes.c_void_p
    good, odd, null = P(0x1000), P(0x1008), P(0)
    f = ctypes.c_float
    assert L.sqp_rmsnorm(4, 1024, null, good, f(1e-5), good, null) == -1
    assert L.sqp_rmsnorm(4, 1020, good, good, f(1e-5), good, null) == -2
    assert L.sqp_rmsnorm(4, 1024, good, good, f(-1.0), good, null) == -4
    assert L.sqp_rmsnorm(4, 1024, good, good, f(float("nan")), good, null) == -4
    assert L.sqp_rmsnorm(4, 1024, good, odd, f(1e-5), good, null) == -3
    assert L.sqp_scale_columns(8, 1020, good, good, good, null) == -2
    assert L.sqp_scale_columns(8, 1024, good, null, good, null) == -1
    assert L.sqp_interleave_gate_up(8, 1024, good, good, odd, null) == -3
    assert L.sqp_interleave_gate_up(0, 1024, good, good, good, null) == -2
    g = L.sqp_w4a16_gemm_silu_mul
    assert g(4, 1032, 1024, 128, good, good, good, good, good, null) == -2   # N % 16
    assert g(4, 1024, 1024, 24, good, good, good, good, good, null) == -2    # group not covered by the fused store
    assert g(4, 1024, 1152, 192, good, good, good, good, good, null) == -2
    assert g(4, 1024, 1024, 128, good, good, null, good, good, null) == -1
    assert L.sqp_transpose_nk(1024, 1020, good, good, null) == -2
    assert L.sqp_transpose_nk(1024, 1024, good, odd, null) == -3
