"""Host-side checks of the C ABI: the library loads, exports every symbol the
header declares, and turns bad arguments into error codes before any launch.
No kernel is launched here, so no GPU is needed."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2310_09259_amd", "libquik.so")
HDR = os.path.join(ROOT, "include", "quik.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2310_09259_amd import build
        build.build()
    lib = C.CDLL(LIB)
    lib.quik_workspace_bytes.restype = C.c_size_t
    lib.quik_status_string.restype = C.c_char_p
    return lib


def test_every_declared_symbol_is_exported(lib):
    names = sorted(set(re.findall(r"\b(quik_[a-z0-9_]+)\s*\(", open(HDR).read())))
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n


def test_sizes_and_strings(lib):
    assert lib.quik_version() >= 1
    assert lib.quik_packed_row_bytes(480, 4) == 240
    assert lib.quik_packed_row_bytes(488, 4) == 256
    assert lib.quik_packed_row_bytes(480, 8) == 480
    assert lib.quik_packed_row_bytes(481, 4) == 0           # odd count cannot be nibble-packed
    assert lib.quik_packed_row_bytes(16, 5) == 0
    ws = lib.quik_workspace_bytes(2048, 4096, 11008, 256, 4)
    assert ws >= 2048 * 1920 + 2 * 2048 * 4 + 2048 * 256 * 2 and ws % 256 == 0
    assert lib.quik_workspace_bytes(0, 4096, 1, 0, 4) == 0
    assert lib.quik_workspace_bytes(16, 64, 1, 64, 4) == 0   # no base column left
    assert b"OK" in lib.quik_status_string(0)
    for code in range(-6, 0):
        assert lib.quik_status_string(code).startswith(b"QUIK_E")


def test_outlier_index_validator(lib):
    def chk(lst, K):
        a = np.asarray(lst, np.int32)
        return lib.quik_check_outlier_idx_host(a.ctypes.data_as(C.c_void_p), len(lst), K)
    assert chk([3, 1, 7], 8) == 0
    assert chk([3, 3], 8) == -1
    assert chk([8], 8) == -1
    assert chk([-1], 8) == -1


def test_bad_arguments_are_rejected_before_launch(lib):
    p = C.c_void_p(0x1000)          # never dereferenced: validation fails first
    u = C.c_void_p(0x1004)          # misaligned
    null = C.c_void_p(0)
    q = lib.quik_quantize
    q.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int,
                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    # (x, T, K, ldx, idx, n_out, bits, xq, ldq, scale, zero, x_out, ldo, workspace, workspace_bytes, stream)
    assert q(p, 4, 64, 64, p, 8, 5, p, 32, p, p, p, 8, p, 16, null) == -1        # bits
    assert q(p, 0, 64, 64, p, 8, 4, p, 32, p, p, p, 8, p, 16, null) == -1        # T
    assert q(p, 4, 64, 64, p, 64, 4, p, 32, p, p, p, 64, p, 16, null) == -1      # n_out == K
    assert q(p, 4, 64, 32, p, 8, 4, p, 32, p, p, p, 8, p, 16, null) == -1        # ldx < K
    assert q(p, 4, 64, 64, p, 8, 4, p, 16, p, p, p, 8, p, 16, null) == -1        # ldq too small
    assert q(null, 4, 64, 64, p, 8, 4, p, 32, p, p, p, 8, p, 16, null) == -2     # x NULL
    assert q(p, 4, 64, 64, null, 8, 4, p, 32, p, p, p, 8, p, 16, null) == -2     # idx NULL with n_out
    assert q(u, 4, 64, 64, p, 8, 4, p, 32, p, p, p, 8, p, 16, null) == -3        # x misaligned
    assert q(p, 4, 64, 64, p, 8, 4, p, 40, p, p, p, 8, p, 16, null) == -3        # ldq % 16
    assert q(p, 4, 60, 64, p, 8, 4, p, 32, p, p, p, 8, p, 16, null) == -4        # K % 8
    assert q(p, 4, 64, 64, p, 4, 4, p, 32, p, p, p, 8, p, 16, null) == -4        # n_out % 8
    assert q(p, 4, 65536, 65536, p, 8, 4, p, 32768, p, p, p, 8, p, 16, null) == -4   # K too large
    assert q(p, 4, 64, 64, p, 8, 4, p, 32, p, p, p, 8, p, 15, null) == -5        # workspace too small
    assert q(p, 4, 64, 64, p, 8, 4, p, 32, p, p, p, 8, C.c_void_p(0x1002), 16, null) == -3
    g = lib.quik_gemm_dequant
    g.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                  C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                  C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    # (xq, ldq, scale, zero, x_out, ldo, T, K_b, n_out, bits, w_q, ldw, w_scale, w_red, w_out, ldwo, bias, N,
    #  y, ldy, workspace, workspace_bytes, stream)
    assert g(p, 32, p, p, p, 8, 4, 64, 8, 4, p, 16, p, p, p, 8, null, 8, p, 8, p, 16, null) == -1   # ldw small
    assert g(p, 32, p, p, p, 8, 4, 64, 8, 4, p, 32, p, p, p, 8, null, 8, null, 8, p, 16, null) == -2
    assert g(p, 32, p, p, p, 8, 4, 64, 8, 4, p, 32, p, p, p, 8, null, 8, p, 4, p, 16, null) == -1   # ldy < N
    assert g(p, 32, p, p, p, 8, 4, 64, 8, 4, u, 32, p, p, p, 8, null, 8, p, 8, p, 16, null) == -3   # w_q align
    # 4-bit layers need the quantization workspace (side data); 8-bit layers do not look at it
    assert g(p, 32, p, p, p, 8, 4, 64, 8, 4, p, 32, p, p, p, 8, null, 8, p, 8, null, 0, null) == -2
    assert g(p, 32, p, p, p, 8, 4, 64, 8, 4, p, 32, p, p, p, 8, null, 8, p, 8, p, 12, null) == -5
    assert g(p, 32, p, p, p, 8, 4, 64, 8, 4, p, 32, p, null, p, 8, null, 8, p, 8, p, 16, null) == -2
    # (xq, ldq, w_q, ldw, T, N, K_b, bits, acc, ldacc, workspace, workspace_bytes, w_reduced, stream): the
    # workspace and w_reduced come together or not at all; both names of the hook behave alike
    for ig in (lib.quik_debug_int_gemm, lib.quik_int_gemm):
        ig.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                       C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        assert ig(p, 32, p, 32, 4, 8, 64, 4, p, 8, p, 16, null, null) == -2
        assert ig(p, 32, p, 32, 4, 8, 64, 4, p, 8, null, 0, p, null) == -2
        assert ig(p, 32, p, 32, 4, 8, 64, 4, null, 8, null, 0, null, null) == -2     # acc NULL
        assert ig(p, 32, p, 32, 4, 8, 64, 4, p, 8, p, 12, p, null) == -5
        assert ig(p, 32, p, 32, 4, 8, 64, 4, p, 4, null, 0, null, null) == -1        # ldacc < N
    lin = lib.quik_linear
    lin.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                    C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                    C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    need = lib.quik_workspace_bytes(4, 64, 8, 8, 4)
    assert lin(p, 4, 64, 64, p, 8, 4, p, 32, p, p, p, 8, null, 8, p, 8, C.c_void_p(0x1000), need - 1,
               null) == -5
    assert lin(p, 4, 64, 64, p, 8, 4, p, 32, p, p, p, 8, null, 8, p, 8, null, need, null) == -2


def test_side_buffer_sizes_and_workspace_regions(lib):
    lib.quik_quantize_workspace_bytes.restype = C.c_size_t
    lib.quik_w_reduced_bytes.restype = C.c_size_t
    assert lib.quik_quantize_workspace_bytes(2048, 4) == 4 * 2048
    assert lib.quik_quantize_workspace_bytes(2048, 8) > 0
    assert lib.quik_quantize_workspace_bytes(0, 4) == 0 and lib.quik_quantize_workspace_bytes(4, 5) == 0
    assert lib.quik_w_reduced_bytes(11008, 4) == 8 * 11008 and lib.quik_w_reduced_bytes(11008, 8) == 4 * 11008
    assert lib.quik_w_reduced_bytes(0, 4) == 0
    off = (C.c_size_t * 4)()
    ldq = C.c_int(0)
    reg = lib.quik_workspace_regions
    reg.argtypes = [C.c_int] * 5 + [C.c_void_p, C.c_void_p]
    assert reg(2048, 4096, 11008, 256, 4, C.cast(off, C.c_void_p), C.cast(C.pointer(ldq), C.c_void_p)) == 0
    assert ldq.value == 1920 and off[0] == 0 and off[1] >= 2048 * 1920
    assert off[2] >= off[1] + 4 * 2048 and off[3] >= off[2] + 4 * 2048
    assert off[3] + 2048 * 256 * 2 <= lib.quik_workspace_bytes(2048, 4096, 11008, 256, 4)
    assert all(o % 256 == 0 for o in off)
    assert reg(2048, 4096, 11008, 256, 4, None, None) == -2
    assert reg(0, 4096, 11008, 256, 4, C.cast(off, C.c_void_p), C.cast(C.pointer(ldq), C.c_void_p)) == -1


def _plan(lib, T, N, K_b, cus=256):
    plan = (C.c_int * 5)()
    fn = lib.quik_debug_gemm_plan
    fn.argtypes = [C.c_int] * 4 + [C.c_void_p]
    rc = fn(T, N, K_b, cus, C.cast(plan, C.c_void_p))
    return rc, tuple(plan)


def _tiles_of_workgroup(lib, T, N, K_b, b, cus=256):
    """The tiles (first token row, first channel, channels) workgroup b of the persistent kernel walks through,
    as the library's own tile order gives them."""
    fn = lib.quik_debug_gemm_tile
    fn.argtypes = [C.c_int] * 6 + [C.c_void_p]
    out, k = [], 0
    while True:
        tile = (C.c_int * 3)()
        rc = fn(T, N, K_b, cus, b, k, C.cast(tile, C.c_void_p))
        assert rc in (0, 1)
        if rc == 0:
            return out
        out.append(tuple(tile))
        k += 1


def test_persistent_kernel_tile_walk_matches_its_definition_on_random_shapes(lib):
    """The kernel finds its tiles with divisions replaced by multiplications with host-prepared constants; the
    hook fails (rc < 0, caught in _tiles_of_workgroup) if that walk ever differs from the definition with plain
    divisions.  Random shapes and CU counts, every workgroup, every tile; the tiles must also cover the output
    exactly once."""
    rng = np.random.default_rng(20231009)
    seen = 0
    for _ in range(60):
        cus = int(rng.choice([8, 16, 64, 104, 256, 304]))
        T = int(rng.integers(1, 9000))
        N = 2 * int(rng.integers(64, 20000))
        K_b = 2 * int(rng.integers(512, 6000))
        rc, plan = _plan(lib, T, N, K_b, cus)
        if rc == 0:
            continue
        tiles_m, tn, base, rem, grid = plan
        flat = [t for b in range(grid) for t in _tiles_of_workgroup(lib, T, N, K_b, b, cus)]
        assert len(flat) == len(set(flat)) == tiles_m * tn, (T, N, K_b, cus)
        assert sum(-(-t[2] // 32) for t in flat) == tiles_m * ((N + 31) // 32), (T, N, K_b, cus)
        seen += 1
    assert seen >= 20


def test_persistent_kernel_plan_covers_the_output_and_balances_the_cus(lib):
    """Host logic of the persistent 4-bit kernel's tile plan, on the benchmark shapes (256 CUs)."""
    for T, N, K_b in ((2048, 11008, 3840), (2048, 4096, 10752), (4096, 15360, 4864), (4096, 28672, 7936),
                      (1030, 9990, 1064), (1024, 15360, 4864)):
        rc, plan = _plan(lib, T, N, K_b)
        assert rc in (1, 2), (T, N, K_b)                           # the persistent kernel can run the shape
        tiles_m, tn, base, rem, grid = plan
        nb = (N + 31) // 32
        assert tiles_m == (T + 255) // 256 and grid == 256
        assert tn * base + rem == nb and 0 <= rem < tn            # the tiles of a panel cover its blocks exactly
        assert 1 <= base and base + (1 if rem else 0) <= 6         # no tile wider than six blocks
        tiles = [_tiles_of_workgroup(lib, T, N, K_b, b) for b in range(grid)]
        # every (token panel, channel range) of the output belongs to exactly one workgroup, channel ranges of a
        # token panel tile [0, N) without gaps, widths are whole blocks of 32 channels (the last one cut at N)
        flat = sorted(t for ts in tiles for t in ts)
        assert len(flat) == len(set(flat)) == tiles_m * tn
        for mp in range(tiles_m):
            row = [t for t in flat if t[0] == mp * 256]
            assert len(row) == tn and row[0][1] == 0
            for a, b2 in zip(row, row[1:]):
                assert a[1] + a[2] == b2[1] and a[2] % 32 == 0 and base * 32 <= a[2] <= (base + 1) * 32
            assert row[-1][1] + row[-1][2] == N
        loads = [sum(-(-t[2] // 32) for t in ts) for ts in tiles]
        assert sum(loads) == tiles_m * nb                          # every block belongs to exactly one workgroup
        assert min(loads) > 0
        # the busiest CU is within one tile's width of the ideal share (the old fixed 256 x 192 tiling of
        # the first shape gave 12 blocks to most CUs for an ideal of 10.75)
        assert max(loads) <= -(-tiles_m * nb // grid) + 6
    # the headline shape is where fixed tiles waste most (464 tiles of 256 x 192 on 256 CUs = 12 blocks for the
    # busiest CU): the persistent kernel is the automatic choice and gives no CU more than 11; an XCD's
    # workgroups take all of its eight channel panels with four of the eight token panels per round
    rc, plan = _plan(lib, 2048, 11008, 3840)
    per_wg = [_tiles_of_workgroup(lib, 2048, 11008, 3840, b) for b in range(256)]
    assert rc == 1 and max(sum(-(-t[2] // 32) for t in ts) for ts in per_wg) == 11
    first_round_xcd0 = [per_wg[b][0] for b in range(0, 256, 8)]
    assert len({t[1] for t in first_round_xcd0}) == 8 and {t[0] for t in first_round_xcd0} == {0, 256, 512, 768}
    # one 256 x 128 tile per CU already balances the down-projection, four-block tiles at 1024 tokens of the
    # 13B QKV shape, few K stages per tile: per-tile kernels
    assert _plan(lib, 2048, 4096, 10752)[0] == 2 and _plan(lib, 1030, 9990, 1064)[0] == 2
    assert _plan(lib, 1024, 15360, 4864)[0] == 2
    # whole rounds of six-block tiles either way (13B QKV at 4096 tokens), and the 70B up-projection: the
    # persistent kernel's K loop is the faster one
    assert _plan(lib, 4096, 15360, 4864)[0] == 1 and _plan(lib, 4096, 28672, 7936)[0] == 1
    # shapes the persistent kernel cannot run: too few tiles for the chip, shallow K, odd N
    assert _plan(lib, 16, 15360, 4864)[0] == 0
    assert _plan(lib, 2048, 11008, 512)[0] == 0
    assert _plan(lib, 2048, 11007, 3840)[0] == 0
    assert _plan(lib, 2048, 11008, 3840, cus=0)[0] == -1
    assert _plan(lib, 2048, 11008, 3841)[0] == -1
    fn = lib.quik_debug_gemm_plan
    assert fn(2048, 11008, 3840, 256, None) == -2
    assert lib.quik_debug_set_gemm_path(3) == -1 and lib.quik_debug_set_gemm_path(-1) == -1
    assert lib.quik_debug_set_gemm_path(1) == 0 and lib.quik_debug_set_gemm_path(0) == 0


def test_mix_probe_rejects_bad_arguments(lib):
    vp, i = C.c_void_p, C.c_int
    fn = lib.quik_debug_mix_probe
    fn.argtypes = [i, i, i, vp, vp, C.c_size_t, vp, vp]
    p, u, null = vp(0x1000), vp(0x1004), vp(0)
    assert fn(64, 256, 10, p, null, 0, null, null) == -1          # mix outside 0 .. 63, 97, 127
    assert fn(96, 256, 10, p, null, 0, null, null) == -1 and fn(128, 256, 10, p, null, 0, null, null) == -1
    assert fn(32, 256, 10, p, null, 0, null, null) == -1          # nibble operands without changing operands
    assert fn(-1, 256, 10, p, null, 0, null, null) == -1
    assert fn(0, 0, 10, p, null, 0, null, null) == -1
    assert fn(0, 256, 0, p, null, 0, null, null) == -1
    assert fn(0, 256, 10, null, null, 0, null, null) == -2         # sink NULL
    assert fn(8, 256, 10, p, null, 32 << 20, null, null) == -2     # copies asked for, no source
    assert fn(8, 256, 10, p, p, 1 << 20, null, null) == -1         # source too small
    assert fn(8, 256, 10, p, u, 32 << 20, null, null) == -3        # source misaligned


def test_fp6_sizes_and_bad_arguments(lib):
    vp, i = C.c_void_p, C.c_int
    lib.quik_workspace_bytes_fp6.restype = C.c_size_t
    assert lib.quik_fp6_row_bytes(64) == 48
    assert lib.quik_fp6_row_bytes(65) == 96                  # padded to whole stages of 64 columns
    assert lib.quik_fp6_row_bytes(3840) == 2880
    assert lib.quik_fp6_row_bytes(0) == 0
    ws = lib.quik_workspace_bytes_fp6(2048, 4096, 11008, 256)
    assert ws >= 2048 * 2880 + 2 * 2048 * 4 + 2048 * 256 * 2 and ws % 256 == 0
    assert lib.quik_workspace_bytes_fp6(16, 64, 1, 64) == 0
    p, u, null = vp(0x1000), vp(0x1004), vp(0)
    pk = lib.quik_weight_pack_fp6
    pk.argtypes = [vp, i, i, i, vp, vp]
    assert pk(p, 32, 8, 64, null, null) == -2
    assert pk(p, 16, 8, 64, p, null) == -1                   # ldw < K_b / 2
    assert pk(p, 32, 8, 63, p, null) == -1                   # odd K_b
    assert pk(p, 32, 8, 64, u, null) == -3
    q6 = lib.quik_quantize_fp6
    q6.argtypes = [vp, i, i, i, vp, i, vp, vp, vp, vp, i, vp]
    assert q6(p, 4, 64, 64, null, 8, p, p, p, p, 8, null) == -2           # idx NULL with n_out
    assert q6(p, 4, 60, 64, p, 8, p, p, p, p, 8, null) == -4              # K % 8
    assert q6(p, 4, 32768, 32768, p, 8, p, p, p, p, 8, null) == -4        # K beyond the FP6 form's limit
    g6 = lib.quik_gemm_dequant_fp6
    g6.argtypes = [vp, vp, vp, vp, i, i, i, i, vp, vp, vp, vp, i, vp, i, vp, i, vp]
    # (xq6, scale, zero, x_out, ldo, T, K_b, n_out, w6, w_scale, w_reduced, w_out, ldwo, bias, N, y, ldy, stream)
    assert g6(p, p, p, p, 8, 4, 64, 8, p, p, p, p, 8, null, 8, null, 8, null) == -2
    assert g6(p, p, p, p, 8, 4, 64, 8, p, p, p, p, 8, null, 8, p, 4, null) == -1      # ldy < N
    assert g6(u, p, p, p, 8, 4, 64, 8, p, p, p, p, 8, null, 8, p, 8, null) == -3
    assert g6(p, p, p, p, 4, 4, 64, 8, p, p, p, p, 8, null, 8, p, 8, null) == -1      # ldo < n_out
    ig = lib.quik_int_gemm_fp6
    ig.argtypes = [vp, vp, i, i, i, vp, i, vp]
    assert ig(p, p, 4, 8, 64, null, 8, null) == -2
    assert ig(p, p, 4, 8, 64, p, 4, null) == -1
    lin = lib.quik_linear_fp6
    lin.argtypes = [vp, i, i, i, vp, i, vp, vp, vp, vp, i, vp, i, vp, i, vp, C.c_size_t, vp]
    need = lib.quik_workspace_bytes_fp6(4, 64, 8, 8)
    assert lin(p, 4, 64, 64, p, 8, p, p, p, p, 8, null, 8, p, 8, vp(0x1000), need - 1, null) == -5
    assert lin(p, 4, 64, 64, p, 8, p, p, p, p, 8, null, 8, p, 8, null, need, null) == -2


def test_sp24_sizes_and_bad_arguments(lib):
    vp, i = C.c_void_p, C.c_int
    lib.quik_workspace_bytes_sp24.restype = C.c_size_t
    lib.quik_sp24_weight_bytes.restype = C.c_size_t
    assert lib.quik_sp24_act_row_bytes(64) == 32
    assert lib.quik_sp24_act_row_bytes(65) == 64             # padded to whole stages of 64 columns
    assert lib.quik_sp24_act_row_bytes(3840) == 1920
    assert lib.quik_sp24_act_row_bytes(0) == 0
    assert lib.quik_sp24_weight_bytes(8, 64) == 8 * 32
    assert lib.quik_sp24_weight_bytes(7, 130) == 3 * 7 * 32  # three stages
    assert lib.quik_sp24_weight_bytes(0, 64) == 0
    ws = lib.quik_workspace_bytes_sp24(2048, 4096, 11008, 256)
    assert ws >= 2048 * 1920 + 2 * 2048 * 4 + 2048 * 256 * 2 and ws % 256 == 0
    assert lib.quik_workspace_bytes_sp24(16, 64, 1, 64) == 0
    p, u, null = vp(0x1000), vp(0x1004), vp(0)
    pk = lib.quik_weight_pack_sp24
    pk.argtypes = [vp, i, i, i, vp, vp, vp]
    assert pk(p, 32, 8, 64, null, null, null) == -2
    assert pk(p, 16, 8, 64, p, null, null) == -1             # ldw < K_b / 2
    assert pk(p, 32, 8, 63, p, null, null) == -1             # odd K_b
    assert pk(p, 32, 8, 64, u, null, null) == -3
    assert pk(p, 32, 8, 64, p, vp(0x1002), null) == -3       # misaligned counter
    q = lib.quik_quantize_sp24
    q.argtypes = [vp, i, i, i, vp, i, vp, vp, vp, vp, i, vp]
    assert q(p, 4, 64, 64, null, 8, p, p, p, p, 8, null) == -2            # idx NULL with n_out
    assert q(p, 4, 60, 64, p, 8, p, p, p, p, 8, null) == -4               # K % 8
    assert q(p, 4, 32768, 32768, p, 8, p, p, p, p, 8, null) == -4         # K beyond this form's limit
    g = lib.quik_gemm_dequant_sp24
    g.argtypes = [vp, vp, vp, vp, i, i, i, i, vp, vp, vp, vp, i, vp, i, vp, i, vp]
    # (xq24, scale, zero, x_out, ldo, T, K_b, n_out, w24, w_scale, w_reduced, w_out, ldwo, bias, N, y, ldy, stream)
    assert g(p, p, p, p, 8, 4, 64, 8, p, p, p, p, 8, null, 8, null, 8, null) == -2
    assert g(p, p, p, p, 8, 4, 64, 8, p, p, p, p, 8, null, 8, p, 4, null) == -1       # ldy < N
    assert g(u, p, p, p, 8, 4, 64, 8, p, p, p, p, 8, null, 8, p, 8, null) == -3
    assert g(p, p, p, p, 4, 4, 64, 8, p, p, p, p, 8, null, 8, p, 8, null) == -1       # ldo < n_out
    ig = lib.quik_int_gemm_sp24
    ig.argtypes = [vp, vp, i, i, i, vp, i, vp]
    assert ig(p, p, 4, 8, 64, null, 8, null) == -2
    assert ig(p, p, 4, 8, 64, p, 4, null) == -1
    lin = lib.quik_linear_sp24
    lin.argtypes = [vp, i, i, i, vp, i, vp, vp, vp, vp, i, vp, i, vp, i, vp, C.c_size_t, vp]
    need = lib.quik_workspace_bytes_sp24(4, 64, 8, 8)
    assert lin(p, 4, 64, 64, p, 8, p, p, p, p, 8, null, 8, p, 8, vp(0x1000), need - 1, null) == -5
    assert lin(p, 4, 64, 64, p, 8, p, p, p, p, 8, null, 8, p, 8, null, need, null) == -2


def _decode_sp24_weights(panels, N, K_b):
    """include/quik.h's description of the sparse weight buffer read backwards, value by value."""
    S = panels.shape[0]
    dec = np.zeros((N, 64 * S), np.int64)
    for s in range(S):
        for n in range(N):
            blk = [int(v) for v in panels[s, n]]
            for kappa in range(16):
                h, qq = (kappa // 4) % 2, 4 * (kappa // 8) + kappa % 4
                word = blk[16 * h + 8] | blk[16 * h + 9] << 8 | blk[16 * h + 10] << 16 | blk[16 * h + 11] << 24
                for e in range(2):
                    c = 2 * qq + e
                    byte = blk[16 * h + 4 * (c // 8) + c % 4]
                    nib = (byte >> 4) if (c // 4) % 2 else (byte & 0xF)
                    pos = (word >> (2 * c)) & 3
                    dec[n, 64 * s + 4 * kappa + pos] += nib - 16 if nib >= 8 else nib
    return dec


def test_sp24_test_side_packers_round_trip_and_generator_is_2of4():
    """The packers the GPU tests compare against, checked on the CPU: decoding their output value by
    value gives back the matrix (and zeros in the padding); the synthetic 2:4 weights have at most two
    nonzero values in every group of four and are otherwise the dense draw."""
    import dataclasses
    import oracle
    from paper_2310_09259_amd import synth
    from tests.util import is_2of4, sp24_act_panels, sp24_weight_panels
    rng = np.random.default_rng(3)
    N, K_b = 5, 136
    w = rng.integers(-8, 8, size=(N, K_b // 4, 4))
    for n in range(N):
        for gidx in range(K_b // 4):
            w[n, gidx, rng.choice(4, 2 + (gidx % 3 == 0), replace=False)] = 0
    w = w.reshape(N, K_b)
    panels = sp24_weight_panels(w)
    assert panels.shape == (3, 5, 32) and not panels[:, :, 12:16].any() and not panels[:, :, 28:32].any()
    dec = _decode_sp24_weights(panels, N, K_b)
    assert np.array_equal(dec[:, :K_b], w) and not dec[:, K_b:].any()
    # index positions ascend inside every pair
    for s in range(3):
        for n in range(N):
            for h in range(2):
                word = int.from_bytes(bytes(panels[s, n, 16 * h + 8:16 * h + 12]), "little")
                for qq in range(8):
                    assert (word >> (4 * qq)) & 3 < (word >> (4 * qq + 2)) & 3
    q = rng.integers(-8, 8, size=(4, 70))
    act = sp24_act_panels(q)
    assert act.shape == (2, 4, 32)
    back = np.zeros((4, 128), np.int64)
    for s in range(2):
        for b in range(32):
            m, pp = b // 4, b % 4
            hi, lo = act[s, :, b].astype(np.int64) >> 4, act[s, :, b].astype(np.int64) & 15
            back[:, 64 * s + 8 * m + pp] = np.where(hi >= 8, hi - 16, hi)
            back[:, 64 * s + 8 * m + 4 + pp] = np.where(lo >= 8, lo - 16, lo)
    assert np.array_equal(back[:, :70], q) and not back[:, 70:].any()
    shp = synth.LayerShape("s", 4, 264, 9, 8, 4, seed=9)
    dense = synth.make_inputs(shp)
    sparse = synth.make_inputs(dataclasses.replace(shp, sparse24=True))
    wd, wsp = oracle.unpack(dense.w_packed, shp.K_b, 4), oracle.unpack(sparse.w_packed, shp.K_b, 4)
    assert is_2of4(wsp).all() and not is_2of4(wd).all()
    assert np.all((wsp == wd) | (wsp == 0))
    assert np.array_equal(dense.x, sparse.x) and np.array_equal(dense.w_out, sparse.w_out)


def test_e3m2_patterns_decode_to_the_integers():
    """The test-side FP6 encoder (tests/util.py) against the format's value formula: 1 sign bit,
    3 exponent bits with bias 3, 2 mantissa bits; e = 0 is subnormal."""
    from tests.util import e3m2_pattern, fp6_panels
    v = np.arange(-8, 9)
    p = e3m2_pattern(v).astype(np.int64)
    s, e, m = p >> 5, (p >> 2) & 7, p & 3
    val = np.where(e == 0, m / 4.0 * 2.0 ** (1 - 3), (1 + m / 4.0) * 2.0 ** (e - 3.0)) * np.where(s == 1, -1.0, 1.0)
    assert np.array_equal(val, v.astype(np.float64))
    # layout: one row, columns 0..63 -> one 48-byte block; column 0 in the low six bits of byte 0,
    # column 32 in the low six bits of byte 16, columns 21 / 53 straddle into bytes 32.. / 40..
    q = np.zeros((1, 64), np.int64)
    q[0, 0], q[0, 32], q[0, 31], q[0, 63] = 1, 2, -8, 7
    blk = fp6_panels(q)[0, 0]
    assert blk.shape == (48,)
    assert blk[0] & 63 == 12 and blk[16] & 63 == 16
    assert blk[39] >> 2 == 56 and blk[47] >> 2 == 23          # last column of each group: top six bits of its 24 bytes
