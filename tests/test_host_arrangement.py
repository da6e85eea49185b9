"""CPU-only tests of the library's host side: the arrangement engine must reproduce the
oracle's index maps bit for bit, the C ABI must export everything the header declares, and
argument errors must come back as status codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2507_11978_amd as nt
from oracle import arrangement as arr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _same(lib_res, ora_res):
    off, mask, shape = lib_res[:3]
    o_off, o_mask, o_shape = ora_res
    assert tuple(shape) == tuple(o_shape)
    assert np.array_equal(off, o_off), "offsets differ"
    assert np.array_equal(mask, o_mask), "masks differ"


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "nt.h")).read()
    names = set(re.findall(r"\b(nt_[a-z0-9_]+)\s*\(", text))
    assert {"nt_arrange_tile", "nt_gemm", "nt_bmm", "nt_conv2d_implicit"} <= names
    lib = ctypes.CDLL(nt.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in nt.h but not exported"


# ------------------------------------------------------------ generic meta-op programs
PROGRAMS = [
    ((4, 6), None, [("tile", (2, 4))]),
    ((9, 10), None, [("tile", (2, 5), (1, -1))]),
    ((9, 10), (1, 9), [("tile", (4, 3)), ("tile", (1, -1)), ("expand", (-1, 5)), ("descend",), ("squeeze", 0), ("ascend",)]),
    ((3, 4, 5), None, [("permute", (2, 0, 1)), ("tile", (2, 2, 3))]),
    ((3, 4, 5), None, [("flatten", 0, 2), ("tile", (5, 2))]),
    ((2, 3, 5, 6), None, [("tile", (1, 3, 3, 2), (-1, -1, 1, 1)), ("squeeze", 1), ("descend",), ("squeeze", 0),
                          ("ascend",), ("ravel",), ("flatten", 0, 3), ("flatten", 1, 4), ("tile", (4, 5))]),
    ((2, 3, 5, 6), None, [("tile", (1, 3, 3, 3), (-1, -1, 2, 1), ((0, 0), (0, 0), (1, 1), (1, 1))), ("squeeze", 1),
                          ("descend",), ("squeeze", 0), ("ascend",), ("ravel",), ("flatten", 0, 3), ("flatten", 1, 4),
                          ("tile", (8, 8))]),
    ((17,), None, [("tile", (4,)), ("tile", (2,))]),          # three levels, ragged at both
    ((6, 1), None, [("expand", (-1, 4)), ("tile", (4, 3))]),
]


@pytest.mark.parametrize("shape,strides,ops", PROGRAMS)
def test_generic_programs_match_oracle(shape, strides, ops):
    a = arr.run_program(arr.Tensor(shape, strides), ops)
    assert nt.arrange_levels(shape, strides, ops) == a.levels
    mids = a.levels[1:-1]
    mid_sets = [()] if not mids else [tuple(m) for m in np.ndindex(*[s for lv in mids for s in lv])]
    for pid in range(arr.num_programs([a])):
        for mid in mid_sets:
            _same(nt.arrange_tile(shape, strides, ops, pid, mid), arr.tile_index_set(a, pid, mid))


# ------------------------------------------------------------- the matmul arrangement
def _gemm_case(M, N, K, tile, sa=None, sb=None, sc=None):
    BM, BN, BK = tile
    o = arr.mm_arrangement(arr.Tensor((M, K), sa), arr.Tensor((K, N), sb), arr.Tensor((M, N), sc), BM, BN, BK)
    d = (((M, K), sa), ((K, N), sb), ((M, N), sc))
    return o, d


def test_c1_index_maps_fully_enumerated():
    # 256^3 with tile 64x64x32: 16 programs x 8 k steps, every element of every tile
    (a, b, c), d = _gemm_case(256, 256, 256, (64, 64, 32))
    grid, kt = nt.arrange_gemm(*d, tile=(64, 64, 32))
    assert grid == (1, 4, 4) and kt == 8 and a.levels[0] == (4, 4) and a.levels[1] == (8,)
    for pid in range(16):
        _same(nt.arrange_gemm(*d, tile=(64, 64, 32), operand=2, program_id=pid), arr.tile_index_set(c, pid))
        for k in range(8):
            _same(nt.arrange_gemm(*d, tile=(64, 64, 32), operand=0, program_id=pid, k=k), arr.tile_index_set(a, pid, (k,)))
            _same(nt.arrange_gemm(*d, tile=(64, 64, 32), operand=1, program_id=pid, k=k), arr.tile_index_set(b, pid, (k,)))


@pytest.mark.parametrize("M,N,K,tile", [
    (3001, 5003, 1999, (256, 256, 64)), (3001, 5003, 1999, (64, 64, 32)), (4096, 4096, 4096, (256, 256, 64)),
    (8192, 8192, 8192, (256, 256, 64)), (5, 7, 3, (64, 64, 32)),
])
def test_sampled_programs_of_large_configs(M, N, K, tile):
    (a, b, c), d = _gemm_case(M, N, K, tile)
    grid, kt = nt.arrange_gemm(*d, tile=tile)
    Mt, Nt = a.levels[0]
    assert grid == (1, Mt, Nt) and kt == a.levels[1][0]
    rng = np.random.default_rng(0)
    pids = {0, Nt - 1, (Mt - 1) * Nt, Mt * Nt - 1} | set(rng.integers(0, Mt * Nt, 3).tolist())
    for pid in pids:
        _same(nt.arrange_gemm(*d, tile=tile, operand=2, program_id=pid), arr.tile_index_set(c, pid))
        for k in {0, kt - 1, int(rng.integers(0, kt))}:
            _same(nt.arrange_gemm(*d, tile=tile, operand=0, program_id=pid, k=k), arr.tile_index_set(a, pid, (k,)))
            _same(nt.arrange_gemm(*d, tile=tile, operand=1, program_id=pid, k=k), arr.tile_index_set(b, pid, (k,)))


def test_strided_operands():
    # A and B given as transposed (column-major) views, C with a padded row pitch
    (a, b, c), d = _gemm_case(70, 50, 45, (64, 64, 32), sa=(1, 70), sb=(1, 45), sc=(64, 1))
    for pid in range(2):
        _same(nt.arrange_gemm(*d, tile=(64, 64, 32), operand=2, program_id=pid), arr.tile_index_set(c, pid))
        for k in range(2):
            _same(nt.arrange_gemm(*d, tile=(64, 64, 32), operand=0, program_id=pid, k=k), arr.tile_index_set(a, pid, (k,)))
            _same(nt.arrange_gemm(*d, tile=(64, 64, 32), operand=1, program_id=pid, k=k), arr.tile_index_set(b, pid, (k,)))


def test_bmm_arrangement():
    Bn, M, N, K, tile = 3, 70, 130, 40, (64, 64, 32)
    a, b, c = arr.bmm_arrangement(arr.Tensor((Bn, M, K)), arr.Tensor((Bn, K, N)), arr.Tensor((Bn, M, N)), *tile)
    d = (((Bn, M, K), None), ((Bn, K, N), None), ((Bn, M, N), None))
    grid, kt = nt.arrange_bmm(*d, tile=tile)
    assert grid == a.levels[0] == (3, 2, 3) and kt == 2
    for pid in range(18):
        _same(nt.arrange_bmm(*d, tile=tile, operand=2, program_id=pid), arr.tile_index_set(c, pid))
        for k in range(kt):
            _same(nt.arrange_bmm(*d, tile=tile, operand=0, program_id=pid, k=k), arr.tile_index_set(a, pid, (k,)))
            _same(nt.arrange_bmm(*d, tile=tile, operand=1, program_id=pid, k=k), arr.tile_index_set(b, pid, (k,)))


@pytest.mark.parametrize("shape,stride,pad,full", [
    ((2, 3, 9, 10, 5, 3, 3), (1, 1), (1, 1), True),
    ((1, 4, 11, 8, 3, 3, 2), (2, 2), (1, 0), True),
    ((32, 256, 56, 56, 256, 3, 3), (1, 1), (1, 1), False),       # the conv benchmark shape, sampled
])
def test_conv_arrangement(shape, stride, pad, full):
    N, C, H, W, K, R, S = shape
    P = (H + 2 * pad[0] - R) // stride[0] + 1
    Q = (W + 2 * pad[1] - S) // stride[1] + 1
    tile = (64, 64, 32) if full else (256, 128, 64)
    a, b, c = arr.conv2d_arrangement(arr.Tensor((N, C, H, W)), arr.Tensor((K, C, R, S)), arr.Tensor((N, K, P, Q)),
                                     *tile, stride, pad)
    d = (((N, C, H, W), None), ((K, C, R, S), None), ((N, K, P, Q), None))
    grid, kt = nt.arrange_conv2d(*d, stride, pad, tile=tile)
    assert grid == (1,) + a.levels[0] and kt == a.levels[1][0]
    G = grid[1] * grid[2]
    pids = range(G) if full else [0, 1, G - 1, G // 2 + 1, 21 * grid[2]]
    ks = range(kt) if full else [0, 1, kt - 1, 17]
    for pid in pids:
        _same(nt.arrange_conv2d(*d, stride, pad, tile=tile, operand=2, program_id=pid), arr.tile_index_set(c, pid))
        for k in ks:
            _same(nt.arrange_conv2d(*d, stride, pad, tile=tile, operand=0, program_id=pid, k=k), arr.tile_index_set(a, pid, (k,)))
            _same(nt.arrange_conv2d(*d, stride, pad, tile=tile, operand=1, program_id=pid, k=k), arr.tile_index_set(b, pid, (k,)))


# ----------------------------------------------------------------- program order swizzle
@pytest.mark.parametrize("batch,mt,nt_", [(1, 4, 4), (1, 16, 16), (1, 12, 20), (32, 8, 8), (1, 32, 32), (1, 392, 2),
                                          (1, 1, 1), (1, 7, 3), (2, 9, 1), (1, 47, 79), (19, 5, 3), (8, 1, 1)])
def test_program_order_is_a_bijection(batch, mt, nt_):
    order = nt.program_order(batch, mt, nt_)
    assert np.array_equal(np.sort(order), np.arange(batch * mt * nt_))
    per = mt * nt_
    full = batch // 8 * 8
    for g in range(full // 8):                   # a complete group of 8 problems: one whole problem per XCD (workgroup index mod 8)
        blk = order[g * 8 * per:(g + 1) * 8 * per]
        for x in range(8):
            assert set(blk[x::8].tolist()) == set(range((g * 8 + x) * per, (g * 8 + x + 1) * per))
    for b in range(full, batch):                 # the problems left over keep their own block of workgroups
        assert set(order[b * per:(b + 1) * per].tolist()) == set(range(b * per, (b + 1) * per))


# ------------------------------------------------------------------------- error paths
def test_errors_are_status_codes():
    with pytest.raises(nt.NtError) as e:
        nt.arrange_gemm(((4, 5), None), ((6, 7), None), ((4, 7), None), tile=(2, 2, 2))
    assert e.value.name == "NT_ERR_SHAPE_MISMATCH"
    with pytest.raises(nt.NtError) as e:
        nt.arrange_gemm(((4, 5), None), ((5, 7), None), ((4, 8), None), tile=(2, 2, 2))
    assert e.value.name == "NT_ERR_SHAPE_MISMATCH"
    with pytest.raises(nt.NtError) as e:
        nt.arrange_levels((2, 3), None, [("expand", (5, -1))])
    assert e.value.name == "NT_ERR_SHAPE_MISMATCH"
    with pytest.raises(nt.NtError) as e:
        nt.arrange_levels((2, 3), None, [("squeeze", 0)])
    assert e.value.name == "NT_ERR_SHAPE_MISMATCH"
    with pytest.raises(nt.NtError) as e:
        nt.arrange_levels((2, 3), None, [("permute", (0, 0))])
    assert e.value.name == "NT_ERR_INVALID_ARG"
    with pytest.raises(nt.NtError) as e:
        nt.arrange_tile((4, 6), None, [("tile", (2, 4))], 3, capacity=4)
    assert e.value.name == "NT_ERR_BUFFER_TOO_SMALL"
    with pytest.raises(nt.NtError) as e:
        nt.arrange_tile((4, 6), None, [("tile", (2, 4))], 4)
    assert e.value.name == "NT_ERR_INVALID_ARG"
    with pytest.raises(nt.NtError) as e:
        nt.arrange_conv2d(((1, 3, 8, 8), None), ((4, 3, 3, 3), None), ((1, 4, 8, 8), None), (1, 1), (0, 0), tile=(64, 64, 32))
    assert e.value.name == "NT_ERR_SHAPE_MISMATCH"            # P must be 6 without padding
    # a mismatch of outermost shapes built by hand: C tiled differently from A's expansion
    lib = nt.load()
    assert lib.nt_gemm(None, None, None, None, None, None, 0, 0, nt.TileCfg(0, 0, 0), None) == 1
    assert nt.tile_supported((64, 64, 32)) and nt.tile_supported(None) and not nt.tile_supported((48, 64, 32))
    d = nt.binding.make_desc((128, 128))
    st = lib.nt_gemm(1, ctypes.byref(d), 1, ctypes.byref(d), 1, ctypes.byref(d), 0, 0, nt.TileCfg(48, 64, 32), None)
    assert st == 3                                            # NT_ERR_UNSUPPORTED, nothing launched
    st = lib.nt_gemm(1, ctypes.byref(d), 1, ctypes.byref(d), 1, ctypes.byref(d), 2, 0, nt.TileCfg(0, 0, 0), None)
    assert st == 3                                            # fp32 inputs are not built


def test_k_zero_and_empty_shapes():
    grid, kt = nt.arrange_gemm(((3, 0), None), ((0, 4), None), ((3, 4), None), tile=(2, 2, 2))
    assert grid == (1, 2, 2) and kt == 0
    grid, kt = nt.arrange_gemm(((0, 5), None), ((5, 4), None), ((0, 4), None), tile=(2, 2, 2))
    assert grid == (1, 0, 2)


@pytest.mark.parametrize("G,Cg,Kg,stride,pad,dilation", [(2, 3, 2, (1, 1), (1, 1), (1, 1)), (4, 1, 1, (2, 1), (0, 2), (1, 2)), (3, 2, 1, (1, 1), (2, 2), (2, 2))])
def test_grouped_convolution_views_match_oracle(G, Cg, Kg, stride, pad, dilation):
    """The programs that write a grouped convolution as one batched view: level shapes and every element's offset / mask."""
    N, H, W, R, S = 2, 7, 6, 3, 3
    P = (H + 2 * pad[0] - (R - 1) * dilation[0] - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - (S - 1) * dilation[1] - 1) // stride[1] + 1
    progs = arr.grouped_conv2d_view_programs(G, Cg, Kg, R, S, stride, pad, P, Q, H, W, dilation)
    shapes = ((N, G * Cg, H, W), (G * Kg, Cg, R, S), (N, G * Kg, P, Q))
    for shape, ops in zip(shapes, progs):
        a = arr.run_program(arr.Tensor(shape), ops)
        assert nt.arrange_levels(shape, None, ops) == a.levels
        off, mask = arr.view_index_set(a)
        # a single-level view is a grid of one-element tiles: program p is element p of the view
        flat_off, flat_mask = off.ravel(), mask.ravel()
        for pid in np.linspace(0, flat_off.size - 1, 97).astype(int):
            o, m, _, _ = nt.arrange_tile(shape, None, ops, int(pid))
            assert int(o[0]) == int(flat_off[pid]) and int(m[0]) == int(flat_mask[pid]), (shape, pid)
