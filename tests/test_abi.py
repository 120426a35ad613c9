"""Host-side checks that need no GPU: the built library exports what include/ac.h declares, and
argument validation rejects bad calls before any launch."""
import os
import re

import pytest

from paper_2505_18574_amd import ops

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ac_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = ops.lib()
    names = declared_symbols()
    assert set(names) == set(ops.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None


def test_version_and_status_strings():
    assert ops.ac_version() >= 100
    seen = set()
    for code in range(0, -9, -1):
        s = ops.status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert ops.status_string(-1234) == "unknown status"


def test_validation_without_gpu():
    # every call below fails validation (or is empty), so nothing is launched
    L = ops.lib()
    p = 0x1000  # never dereferenced
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, -1, 0, None, 0, None) == ops.AC_ERR_SHIFT
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 7, None, 0, None) == ops.AC_ERR_ACT
    assert L.ac_gemm_i8(p, 7, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 0, None, 0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, p + 768, 4, p + 512, 8, 8, 8, 8, 0, 0, None, 0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 0, None, 64, None) == ops.AC_ERR_WORKSPACE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, p + 512, 8, 8, 8, 8, 0, 0, p + 1, 64, None) == ops.AC_ERR_WORKSPACE
    assert L.ac_gemm_i8(p, 8, p + 256, 8, None, 0, None, 8, 8, 8, 8, 0, 0, None, 0, None) == ops.AC_ERR_NULL
    assert L.ac_gemm_i8(None, 8, None, 8, None, 0, None, 8, 0, 8, 8, 0, 0, None, 0, None) == ops.AC_OK
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 1, 4, 4, 16, 16, 3, 3, 1, -1, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 1, 40000, 4, 16, 16, 3, 3, 1, 1, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 1, 4, 4, 16, 0, 3, 3, 1, 1, 0, 0, None, 0, None) == ops.AC_OK
    assert L.ac_gemm_bf16(p, 8, p + 256, 8, p + 512, 4, 8, 8, 8, 1.0, 0.0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_bf16(p, 8, p + 256, 8, p + 512, 8, 8, 0, 8, 1.0, 0.0, None) == ops.AC_OK
    assert L.ac_batched_gemm_f32(p, p + 256, p + 512, None, None, None, 33, 4, None) == ops.AC_ERR_SHAPE
    assert L.ac_batched_gemm_f32(p, p + 256, p + 512, None, None, None, 12, -1, None) == ops.AC_ERR_SHAPE
    assert ops.ac_gemm_i8_workspace_bytes(0, 8, 8) == 0


def test_sizes_beyond_the_supported_range_are_refused():
    """Dimensions above 2^29, or more than 2^31 - 1 blocks of 64 x 64 outputs, are refused on the host by every GEMM-like
    entry point; the size and plan queries answer as for an empty problem."""
    L = ops.lib()
    p = 0x1000  # never dereferenced
    big, imax = (1 << 29) + 1, (1 << 31) - 1
    for M, N, K in [(big, 16, 16), (16, big, 16), (16, 16, big), (imax, 16, 16), (1 << 29, 1 << 21, 16)]:
        ld = 1 << 40
        assert L.ac_gemm_i8(p, ld, p + 256, ld, None, 0, p + 512, ld, M, N, K, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE
        assert L.ac_gemm_i8_acc32(p, ld, p + 256, ld, None, 0, p + 512, ld, M, N, K, None) == ops.AC_ERR_SHAPE
        assert L.ac_gemm_i8_t(p, ld, p + 256, ld, None, 0, p + 512, ld, M, N, K, 0, 0, 1, 1, None) == ops.AC_ERR_SHAPE
        assert L.ac_gemm_bf16(p, ld, p + 256, ld, p + 512, ld, M, N, K, 1.0, 0.0, None) == ops.AC_ERR_SHAPE
        assert L.ac_gemm_bf16_ws(p, ld, p + 256, ld, p + 512, ld, M, N, K, 1.0, 0.0, None, 0, None) == ops.AC_ERR_SHAPE
        assert L.ac_gemm_i8_planned(p, ld, p + 256, ld, None, 0, p + 512, ld, M, N, K, 0, 0, None, 0, 64, 1, None) == ops.AC_ERR_SHAPE
        assert ops.ac_gemm_i8_workspace_bytes(M, N, K) == 0 and ops.ac_gemm_bf16_workspace_bytes(M, N, K) == 0
        assert ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, 64, 2) == 0
        assert ops.ac_gemm_i8_auto_plan(M, N, K, True) == ops.ac_gemm_i8_auto_plan(0, 0, 0, True)
        assert ops.ac_gemm_bf16_auto_plan(M, N, K) == ops.ac_gemm_bf16_auto_plan(0, 0, 0)
    # a convolution whose implicit GEMM has more than 2^29 rows (input of 2^31 - 1 elements or fewer, so that only M decides)
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 40000, 120, 120, 1, 16, 1, 1, 1, 0, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE


def test_planned_entry_validation_without_gpu():
    """Tile / split arguments of the planned launches are checked on the host before anything else runs."""
    L = ops.lib()
    p = 0x1000  # never dereferenced
    i8 = lambda tile, splits, K=4096, ws=None, wsb=0: L.ac_gemm_i8_planned(
        p, K, p + 256, 64, None, 0, p + 512, 64, 64, 64, K, 0, 0, ws, wsb, tile, splits, None)
    assert i8(100, 1) == ops.AC_ERR_PLAN          # unknown tile
    assert i8(64, 0) == ops.AC_ERR_PLAN           # no slices
    assert i8(64, 33) == ops.AC_ERR_PLAN          # 4096 bytes of K are 32 tiles of 128 bytes
    assert i8(256, 65) == ops.AC_ERR_PLAN         # ... and 64 tiles of 64 bytes
    assert i8(64, 4) == ops.AC_ERR_WORKSPACE      # a split needs the workspace
    need = ops.ac_gemm_i8_planned_workspace_bytes(64, 64, 4096, 64, 4)
    assert need == 4 * 64 * 64 * 4
    assert i8(64, 4, ws=p + 4096, wsb=need - 1) == ops.AC_ERR_WORKSPACE
    # slices hold whole K tiles: 32 tiles over 5 slices are 7 per slice, which leaves 5 slices; over 12 are 3 -> 11
    assert ops.ac_gemm_i8_planned_workspace_bytes(64, 64, 4096, 64, 5) == 5 * 64 * 64 * 4
    assert ops.ac_gemm_i8_planned_workspace_bytes(64, 64, 4096, 64, 12) == 11 * 64 * 64 * 4
    assert ops.ac_gemm_i8_planned_workspace_bytes(64, 64, 4096, 64, 1) == 0
    assert ops.ac_gemm_i8_planned_workspace_bytes(64, 64, 4096, 7, 4) == 0
    # a split over operands that cannot take the direct-to-LDS kernels (K not a multiple of 16)
    assert L.ac_gemm_i8_planned(p, 1000, p + 256, 64, None, 0, p + 512, 64, 64, 64, 1000, 0, 0, p + 4096, 1 << 20, 64, 2, None) == ops.AC_ERR_PLAN
    # ... or whose rows lie so far apart that a tile's rows span more than 32 bits of byte offset
    need = ops.ac_gemm_i8_planned_workspace_bytes(64, 64, 4096, 64, 2)
    assert L.ac_gemm_i8_planned(p, 1 << 24, p + 256, 64, None, 0, p + 512, 64, 64, 64, 4096, 0, 0, p + 4096, need, 64, 2, None) == ops.AC_ERR_PLAN
    assert L.ac_gemm_i8_planned(p, 4096, p + 256, 1 << 26, None, 0, p + 512, 64, 64, 64, 4096, 0, 0, p + 4096, need, 64, 2, None) == ops.AC_ERR_PLAN
    assert L.ac_gemm_bf16_planned(p, 1 << 23, p + 256, 64, p + 512, 64, 64, 64, 4096, 1.0, 0.0, None, 0, 64, 2, None) == ops.AC_ERR_PLAN
    bf = lambda tile, splits, K=4096, ws=None, wsb=0: L.ac_gemm_bf16_planned(
        p, K, p + 256, 64, p + 512, 64, 64, 64, K, 1.0, 0.0, ws, wsb, tile, splits, None)
    assert bf(32, 1) == ops.AC_ERR_PLAN
    assert bf(128, 65) == ops.AC_ERR_PLAN         # 8192 bytes of K are 64 tiles of 128 bytes
    assert bf(64, -1) == ops.AC_ERR_PLAN
    assert L.ac_gemm_bf16_planned(p, 1004, p + 256, 64, p + 512, 64, 64, 64, 1004, 1.0, 0.0, None, 0, 64, 2, None) == ops.AC_ERR_PLAN
    need = ops.ac_gemm_bf16_planned_workspace_bytes(64, 64, 4096, 128, 4)
    assert need == 4 * 64 * 64 * 4
    assert bf(128, 4, ws=p + 4096, wsb=need - 4) == ops.AC_ERR_WORKSPACE
    assert bf(128, 4, ws=p + 4100, wsb=need) == ops.AC_ERR_WORKSPACE   # misaligned
    assert bf(128, 4, ws=None, wsb=64) == ops.AC_ERR_WORKSPACE
    assert "tile" in ops.status_string(ops.AC_ERR_PLAN)


def test_resident_operand_kernels_validation_without_gpu():
    """Tile codes of the weight-stationary (320 / 160) and convolution patch (321 / 161) kernels: what they cannot
    take is refused on the host with AC_ERR_PLAN, before any launch."""
    L = ops.lib()
    p = 0x1000  # never dereferenced; 16-byte aligned
    i8 = lambda tile, splits, M=512, N=64, K=512, bias=None, bias_ld=0: L.ac_gemm_i8_planned(
        p, K, p + (1 << 20), N, bias, bias_ld, p + (2 << 20), N, M, N, K, 8, 1, None, 0, tile, splits, None)
    assert i8(320, 2) == ops.AC_ERR_PLAN                            # all of K is resident: no K split
    assert i8(320, 1, K=1552) == ops.AC_ERR_PLAN                    # 13 K tiles do not fit beside the 256-row ring
    assert i8(160, 1, K=2064) == ops.AC_ERR_PLAN                    # ... nor 17 beside the 128-row ring
    assert i8(160, 1, bias=p + (3 << 20), bias_ld=64) == ops.AC_ERR_PLAN  # a bias matrix
    assert i8(160, 1, N=60) == ops.AC_ERR_PLAN                      # N not a multiple of 16
    assert i8(321, 1) == ops.AC_ERR_PLAN and i8(161, 1) == ops.AC_ERR_PLAN  # the patch kernel is a convolution kernel
    assert L.ac_gemm_bf16_planned(p, 512, p + (1 << 20), 64, p + (2 << 20), 64, 512, 64, 512, 1.0, 0.0, None, 0, 320, 1, None) == ops.AC_ERR_PLAN
    conv = lambda tile, splits, Nb=1, H=8, W=8, Cin=32, Cout=16, KH=3, KW=3, stride=1, pad=1, out=p + (2 << 20): L.ac_conv2d_i8_planned(
        p, p + (1 << 20), None, out, Nb, H, W, Cin, Cout, KH, KW, stride, pad, 8, 1, None, 0, tile, splits, None)
    assert conv(77, 1) == ops.AC_ERR_PLAN                           # unknown tile
    assert conv(321, 2) == ops.AC_ERR_PLAN                          # no K split
    assert conv(321, 1, Cin=16) == ops.AC_ERR_PLAN                  # a K-step would straddle two taps
    assert conv(161, 1, Cin=48) == ops.AC_ERR_PLAN                  # Cin not a multiple of 32
    assert conv(321, 1, Cin=3, Cout=8) == ops.AC_ERR_PLAN           # not even the direct-to-LDS path
    assert conv(321, 1, out=p + (2 << 20) + 4) == ops.AC_ERR_PLAN   # 16-byte output stores
    assert conv(321, 1, Nb=8, H=28, W=28, Cin=128, Cout=256, stride=2) == ops.AC_ERR_PLAN  # patch + weights exceed LDS
    assert conv(161, 1, Nb=8, H=28, W=28, Cin=128, Cout=256, stride=2) == ops.AC_ERR_PLAN
    assert conv(321, 1, H=300, W=300, Cin=256, Cout=64) == ops.AC_ERR_PLAN  # K = 2304: more than 64 K-steps
    assert conv(320, 1, Cin=256, Cout=64, KH=3, KW=3) == ops.AC_ERR_PLAN    # K = 2304 is not resident for 320 ...


def test_transposed_entry_validation_without_gpu():
    L = ops.lib()
    p = 0x1000  # never dereferenced
    t = lambda lda, ldb, ta, tb: L.ac_gemm_i8_t(p, lda, p + 256, ldb, None, 0, p + 512, 8, 4, 8, 16, 0, 0, ta, tb, None)
    assert t(15, 8, 0, 0) == ops.AC_ERR_STRIDE   # plain A: lda >= K = 16
    assert t(3, 8, 1, 0) == ops.AC_ERR_STRIDE    # A^T is K x M: lda >= M = 4
    assert t(4, 15, 1, 1) == ops.AC_ERR_STRIDE   # B^T is N x K: ldb >= K = 16
    assert L.ac_gemm_i8_t(p, 4, p + 256, 16, None, 0, p + 512, 8, 4, 8, 16, 40, 0, 1, 1, None) == ops.AC_ERR_SHIFT
    assert L.ac_gemm_i8_t(p, 4, p + 256, 16, None, 0, None, 8, 4, 8, 16, 0, 0, 1, 1, None) == ops.AC_ERR_NULL
    assert L.ac_gemm_i8_t(None, 4, None, 16, None, 0, None, 8, 0, 8, 16, 0, 0, 1, 1, None) == ops.AC_OK


def test_auto_plans_are_host_arithmetic():
    # the benchmark shapes: big square problems take the 256 tile; narrow ones fall back to 64
    assert ops.ac_gemm_bf16_auto_plan(4096, 4096, 4096) == (256, 1)
    assert ops.ac_gemm_i8_auto_plan(3136, 64, 576) == (32, 1)     # a few microseconds, short K: one wave per 32 x 32 tile
    assert ops.ac_gemm_i8_auto_plan(256, 256, 256) == (32, 1) and ops.ac_gemm_i8_auto_plan(3136, 256, 64) == (32, 1)
    assert ops.ac_gemm_i8_auto_plan(512, 768, 768) == (32, 1) and ops.ac_gemm_i8_auto_plan(128, 1024, 1024) == (32, 1)
    assert ops.ac_gemm_i8_auto_plan(1024, 1024, 512)[0] != 32     # 1024 tiles: the tiled kernels from K = 512
    assert ops.ac_gemm_i8_auto_plan(784, 512, 1152)[0] != 32      # beyond the depth for 400 tiles
    assert ops.ac_gemm_i8_auto_plan(128, 1024, 3072)[0] != 32     # deep K: cut instead (more loads in flight from HBM)
    assert ops.ac_gemm_i8_auto_plan(3136, 64, 600)[0] != 32       # K not in whole 64-byte tiles
    assert ops.ac_gemm_i8_auto_plan(3136, 64, 704) == (32, 1)     # any whole number of 64-byte tiles
    assert ops.ac_gemm_i8_auto_plan(2048, 1024, 192) == (32, 1) and ops.ac_gemm_i8_auto_plan(2048, 1024, 256)[0] != 32
    assert ops.ac_gemm_i8_auto_plan(12544, 256, 64)[0] != 32      # 3136 tiles: more than the small kernel is ahead for
    assert ops.ac_gemm_i8_auto_plan(49, 2048, 4608)[0] != 32      # too deep: K is cut instead
    assert ops.ac_gemm_i8_auto_plan(65536, 64, 576) == (320, 1)   # long, narrow, short K: weight-stationary kernel
    assert ops.ac_gemm_i8_auto_plan(65536, 64, 4096) == (64, 1)   # K too deep to stay resident
    # few output tiles: tile and K slices come from one cost estimate; slicing needs the workspace and is priced at
    # several microseconds, so the 18 K tiles of 196 x 1024 x 2304 stay whole while the weight-streaming
    # 49 x 2048 x 4608 is sliced
    assert ops.ac_gemm_i8_auto_plan(196, 1024, 2304, True) == (64, 1)
    assert ops.ac_gemm_i8_auto_plan(49, 2048, 4608, True) == (64, 8)
    assert ops.ac_gemm_i8_auto_plan(16, 4096, 4096, True) == (64, 4)      # weight streaming: slices although 64 tiles exist
    assert ops.ac_gemm_i8_auto_plan(49, 2048, 4608, False) == (64, 1)
    tile, splits = ops.ac_gemm_i8_auto_plan(49, 512, 9216, True)
    assert tile == 64 and splits > 1
    assert ops.ac_gemm_i8_auto_plan(49, 512, 9216, False) == (64, 1)
    assert ops.ac_gemm_i8_workspace_bytes(49, 512, 9216) == ops.ac_gemm_i8_planned_workspace_bytes(49, 512, 9216, tile, splits)
    assert ops.ac_gemm_i8_workspace_bytes(196, 1024, 2304) == 0
    assert ops.ac_gemm_i8_auto_plan(256, 256, 1048576, True) == (192, 128)  # very deep K: a big tile, the chip filled once
    assert ops.ac_gemm_i8_auto_plan(256, 256, 1048576, False) == (64, 1)
    for M, N, K in [(16, 16, 100000), (300, 260, 70000), (512, 512, 16384), (1024, 256, 8192)]:
        tile, splits = ops.ac_gemm_i8_auto_plan(M, N, K, True)
        assert splits > 1
        assert ops.ac_gemm_i8_workspace_bytes(M, N, K) == ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, tile, splits) > 0
    # more 64 x 64 tiles than the chip holds at once: the code with the lowest fitted time estimate
    assert ops.ac_gemm_i8_auto_plan(8192, 8192, 8192) == (256, 1) and ops.ac_gemm_bf16_auto_plan(4096, 8192, 8192) == (256, 1)
    assert ops.ac_gemm_bf16_auto_plan(2048, 4096, 8192) == (192, 1)      # 128 tiles of 256 x 256 would idle half the chip
    assert ops.ac_gemm_i8_auto_plan(3072, 3072, 768) == (256, 1)         # 144 big tiles in one round beat 288 in two
    assert ops.ac_gemm_i8_auto_plan(4096, 4096, 128) == (320, 1)         # short K: weight-stationary also on a wide output
    assert ops.ac_gemm_i8_auto_plan(4096, 4096, 2048)[0] in (128, 192, 256)   # K too deep to stay resident
    assert ops.ac_gemm_bf16_auto_plan(32768, 32768, 32) == (256, 1)      # beyond the fitted range: the big tile
    for M, N, K in [(5000, 3000, 100), (700, 9000, 3000), (100000, 64, 16), (64, 100000, 4000), (12345, 6789, 1011)]:
        assert ops.ac_gemm_i8_auto_plan(M, N, K, False)[1] == 1 and ops.ac_gemm_bf16_auto_plan(M, N, K)[1] == 1
        assert ops.ac_gemm_i8_auto_plan(M, N, K, False)[0] in (32, 64, 128, 192, 256, 160, 320)
        assert ops.ac_gemm_bf16_auto_plan(M, N, K)[0] in (64, 128, 192, 256)
        if K > 2048:
            assert ops.ac_gemm_i8_auto_plan(M, N, K, False)[0] not in (160, 320)
    # bf16 with few output tiles: tile and slice count come from one cost estimate; a very deep K takes a
    # big tile (operands requested fewer times) and enough slices to fill the chip once
    assert ops.ac_gemm_bf16_auto_plan(256, 256, 524288) == (192, 128)
    assert ops.ac_gemm_bf16_auto_plan(256, 256, 8192) == (64, 8)
    assert ops.ac_gemm_bf16_auto_plan(1024, 1024, 1024) == (64, 1)
    for M, N, K in [(1, 1, 1), (64, 64, 100000), (100, 36, 7), (768, 768, 32768), (32, 8192, 8192)]:
        tile, splits = ops.ac_gemm_bf16_auto_plan(M, N, K)
        bm, bn, ktb = {64: (64, 64, 128), 128: (128, 128, 128), 192: (256, 128, 128), 256: (256, 256, 64)}[tile]
        nkt = -(-2 * K // ktb)
        assert 1 <= splits <= max(1, nkt // 4 + 1)
        if splits > 1:  # one round of workgroups
            assert -(-M // bm) * -(-N // bn) * splits <= (512 if tile == 64 else 256)


def test_workspace_size_matches_the_automatic_plan():
    """The size ac_gemm_i8_workspace_bytes reports is the one the library's own plan needs (the call checks the
    caller's workspace against it), over a random sweep of shapes on both sides of every planner boundary."""
    import random
    rng = random.Random(7)
    dims = [1, 7, 49, 64, 65, 196, 256, 300, 784, 1000, 1024, 1100, 1280, 2048, 3136, 4096, 8192, 12544, 50176]
    ks = [1, 16, 64, 100, 256, 576, 1152, 2304, 4096, 4608, 9216, 16384, 65536, 524288]
    split_seen = bf16_split_seen = 0
    for _ in range(400):
        M, N, K = rng.choice(dims), rng.choice(dims), rng.choice(ks)
        tile, splits = ops.ac_gemm_i8_auto_plan(M, N, K, True)
        assert tile in (32, 64, 128, 192, 256, 160, 320) and splits >= 1
        need = ops.ac_gemm_i8_workspace_bytes(M, N, K)
        if tile == 32:
            # the size covers operands the one-wave-per-tile kernel does not take, whose plan may cut K; the plan
            # for operands it does take never uses the buffer
            assert splits == 1 and need % (M * N * 4) == 0 and ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, 32, 1) == 0
            continue
        assert need == ops.ac_gemm_i8_planned_workspace_bytes(M, N, K, tile, splits)
        assert (need > 0) == (splits > 1)
        if splits > 1:
            split_seen += 1
            assert need == splits * M * N * 4
        # without a workspace the plan never slices
        assert ops.ac_gemm_i8_auto_plan(M, N, K, False)[1] == 1
        t2, s2 = ops.ac_gemm_bf16_auto_plan(M, N, K)
        assert t2 in (64, 128, 192, 256) and s2 >= 1
        need2 = ops.ac_gemm_bf16_workspace_bytes(M, N, K)
        assert need2 == ops.ac_gemm_bf16_planned_workspace_bytes(M, N, K, t2, s2)
        assert need2 == (s2 * M * N * 4 if s2 > 1 else 0)
        bf16_split_seen += s2 > 1
    assert split_seen > 20 and bf16_split_seen > 20
    assert ops.ac_gemm_bf16_workspace_bytes(0, 8, 8) == 0 and ops.ac_gemm_bf16_workspace_bytes(8, 8, -1) == 0


def test_bf16_workspace_validation_without_gpu():
    """The workspace of ac_gemm_bf16_ws is checked on the host like the one of ac_gemm_i8."""
    L = ops.lib()
    p = 0x1000  # never dereferenced
    M, N, K = 64, 64, 65536
    need = ops.ac_gemm_bf16_workspace_bytes(M, N, K)
    assert need > 0
    call = lambda ws, wsb: L.ac_gemm_bf16_ws(p, K, p + 256, N, p + 512, N, M, N, K, 1.0, 0.0, ws, wsb, None)
    assert call(p + 4096, need - 4) == ops.AC_ERR_WORKSPACE    # too small
    assert call(p + 4100, need) == ops.AC_ERR_WORKSPACE        # misaligned
    assert call(None, 64) == ops.AC_ERR_WORKSPACE              # a size without a pointer
    assert call(p + 4096, 0) == ops.AC_ERR_WORKSPACE           # a pointer without a size
    assert L.ac_gemm_bf16_ws(p, K, p + 256, N, p + 512, N, M, N, -1, 1.0, 0.0, None, 0, None) == ops.AC_ERR_SHAPE
    assert L.ac_gemm_bf16_ws(p, K - 8, p + 256, N, p + 512, N, M, N, K, 1.0, 0.0, None, 0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_bf16_ws(None, K, p + 256, N, p + 512, N, 0, N, K, 1.0, 0.0, None, 0, None) == ops.AC_OK  # nothing to do


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(ops, "_lib", None)
    monkeypatch.setattr(ops, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libac_mi355x.so"))
    with pytest.raises(ImportError):
        ops.lib()


def test_static_entry_refuses_on_the_host():
    """ac_gemm_i8_static validates like ac_gemm_i8 and refuses partial sums beyond its buffer, all before any GPU call."""
    L = ops.lib()
    p = 0x1000  # never dereferenced
    assert L.ac_gemm_i8_static(p, 4608, p + 256, 2048, None, 0, p + 512, 2048, 49, 2048, 4608, 32, 0, None) == ops.AC_ERR_SHIFT
    assert L.ac_gemm_i8_static(p, 4608, p + 256, 2048, None, 0, p + 512, 2000, 49, 2048, 4608, 3, 0, None) == ops.AC_ERR_STRIDE
    assert L.ac_gemm_i8_static(p, 4608, p + 256, 2048, None, 0, None, 2048, 49, 2048, 4608, 3, 0, None) == ops.AC_ERR_NULL
    assert L.ac_gemm_i8_static(None, 8, None, 8, None, 0, None, 8, 0, 8, 8, 0, 0, None) == ops.AC_OK
    assert ops.ac_gemm_i8_workspace_bytes(1024, 1024, 65536) > ops.AC_STATIC_SCRATCH_BYTES
    assert L.ac_gemm_i8_static(p, 65536, p + 256, 1024, None, 0, p + 512, 1024, 1024, 1024, 65536, 3, 0, None) == ops.AC_ERR_WORKSPACE


def test_convolution_sizes_whose_products_would_overflow_are_refused():
    """A large stride keeps the implicit GEMM tiny while batch, image and channel counts are near 2^31: the input
    size is refused factor by factor, before any product can leave int64."""
    L = ops.lib()
    p = 0x1000  # never dereferenced
    big = (1 << 29) + 7
    for Nb, Cin in [(big, big), (1 << 30, 1 << 30), ((1 << 31) - 1, (1 << 31) - 1), (big, 16), (16, big)]:
        assert L.ac_conv2d_i8(p, p + 256, None, p + 512, Nb, 32767, 32767, Cin, 16, 1, 1, 32767, 0, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE
    # kernel taps times channels beyond int32
    assert L.ac_conv2d_i8(p, p + 256, None, p + 512, 1, 30000, 30000, 1 << 20, 16, 30000, 30000, 1, 0, 0, 0, None, 0, None) == ops.AC_ERR_SHAPE
    # the same geometry at a size that fits is only refused for what it is asked to read (NULL operands), not for its shape
    assert L.ac_conv2d_i8(None, None, None, p + 512, 2, 32767, 32767, 1, 16, 1, 1, 32767, 0, 0, 0, None, 0, None) == ops.AC_ERR_NULL
