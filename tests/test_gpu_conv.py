"""GPU parity of the convolution entry points against the fp64 oracle.

Every case runs through the C ABI on the same seeded inputs as the oracle.
Bars: relative L2 <= 1e-5 for the fp32 path, <= 5e-3 for the bf16-input path
(oracle fed the bf16-rounded values); the result must not depend on the
algorithm or the workspace size (Sec. 3.5: workspaces do not affect the result).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_04380_amd as sn
from paper_1801_04380_amd import workloads as wl
from _parity import CODE, DT, TOL, elementwise_excess, f64, rel_l2, run_conv, shape_of

pytestmark = pytest.mark.gpu

L = wl._L
# (layer, N): sizes the oracle finishes in seconds, spanning several tiles and ragged tails
CASES = [
    (wl.CONFIGS[1]["layers"][0], 2),                                   # cfg1
    (L("ragged3x3", 19, 37, 29, 70, 3, 3, (1, 1), (1, 1)), 3),
    (L("k200", 24, 20, 20, 200, 3, 3, (1, 1), (1, 1)), 2),            # several M tiles
    (L("s2_3x3", 16, 33, 33, 40, 3, 3, (2, 2), (1, 1)), 2),
    (L("s2_valid", 32, 35, 35, 48, 3, 3, (2, 2), (0, 0)), 2),
    (L("alex1", 3, 67, 67, 96, 11, 11, (4, 4), (0, 0), relu_in=False), 2),
    (L("5x5", 24, 27, 27, 32, 5, 5, (1, 1), (2, 2)), 2),
    (L("1x7", 32, 17, 17, 40, 1, 7, (1, 1), (0, 3)), 2),
    (L("7x1", 40, 17, 17, 32, 7, 1, (1, 1), (3, 0)), 2),
    (L("1x1", 96, 14, 14, 160, 1, 1), 3),
    (L("1x1_s2", 64, 28, 28, 96, 1, 1, (2, 2)), 2),
    (L("first3", 3, 40, 40, 64, 3, 3, (1, 1), (1, 1), relu_in=False), 2),
    (L("tiny", 1, 1, 1, 1, 1, 1), 1),
    (L("one_pixel_out", 5, 3, 3, 7, 3, 3), 1),
    (L("big_pad", 4, 5, 5, 6, 3, 3, (1, 1), (2, 2)), 2),
    (L("stride_gt_filter", 8, 16, 16, 8, 2, 2, (3, 3), (0, 0)), 2),
    (L("deep_c", 512, 7, 7, 64, 3, 3, (1, 1), (1, 1)), 2),
    (L("wide", 20, 19, 100, 72, 3, 3, (1, 1), (1, 1)), 2),            # column tiles, ragged last tile
    (L("wide_k64", 16, 37, 70, 64, 3, 3, (1, 1), (1, 1)), 1),
    (L("small_imgs", 32, 7, 7, 96, 3, 3, (1, 1), (1, 1)), 9),         # one tile spans several images
    (L("1x1_small", 40, 7, 7, 48, 1, 1), 11),
    # 3x3 with more than 64 output channels (forward) or input channels (backward-data) and an even
    # width: the tilings of the packed-filter kernel that loads its patch straight into LDS
    (L("cols72", 40, 21, 72, 136, 3, 3, (1, 1), (1, 1)), 2),          # column tiles, 16-byte items, ragged rows
    (L("cols64_big", 24, 64, 64, 160, 3, 3, (1, 1), (1, 1)), 8),      # enough tiles for the largest tile size
    (L("w8", 48, 8, 8, 96, 3, 3, (1, 1), (1, 1)), 20),                # rows of several images in one tile
    (L("w24", 17, 11, 24, 80, 3, 3, (1, 1), (1, 1)), 3),
    (L("w28", 64, 28, 28, 128, 3, 3, (1, 1), (1, 1)), 3),             # 4-byte items
    (L("w14", 35, 14, 14, 96, 3, 3, (1, 1), (1, 1)), 7),
    (L("w6_pad0", 20, 9, 6, 70, 3, 3, (1, 1), (0, 0)), 5),
    (L("w28_big", 16, 28, 28, 256, 3, 3, (1, 1), (1, 1)), 48),
    (L("w28_k96", 32, 28, 28, 96, 3, 3, (1, 1), (1, 1)), 32),         # backward-filter with two wave sets per tile
    (L("c96_bwd", 96, 16, 16, 48, 3, 3, (1, 1), (1, 1)), 3),          # backward-data into 96 channels
    (L("c130_pad2", 130, 10, 12, 130, 3, 3, (1, 1), (2, 2)), 2),
    # few tiles of small images: two sets of waves share a tile's chunks (an even chunk count):
    # 4 chunks; 6 (an odd count per set); 8 with a partial last chunk, 8-wide rows (16-byte items)
    (L("w14_split", 64, 14, 14, 128, 3, 3, (1, 1), (1, 1)), 4),
    (L("w14_split_c96", 96, 14, 14, 160, 3, 3, (1, 1), (1, 1)), 5),
    (L("w8_split_c120", 120, 8, 8, 128, 3, 3, (1, 1), (1, 1)), 6),
    (L("w14_split_bwd", 128, 14, 14, 64, 3, 3, (1, 1), (1, 1)), 3),   # backward-data from 64 channels into 128
    # at most 64 output channels on 32-column patches: four waves along the pixels (forward: K, backward-data: C)
    (L("k64_w64", 96, 16, 64, 64, 3, 3, (1, 1), (1, 1)), 2),
    (L("k48_w72", 104, 12, 72, 48, 3, 3, (1, 1), (1, 1)), 3),
    (L("k64_w112_pad0", 128, 20, 112, 64, 3, 3, (1, 1), (0, 0)), 1),
    (L("c40_bwd_w72", 40, 12, 72, 112, 3, 3, (1, 1), (1, 1)), 2),      # backward-data: 112 channels into 40
    # 32-column patches with no padding, and with more than the filter needs
    (L("wide_pad0", 32, 20, 112, 96, 3, 3, (1, 1), (0, 0)), 1),
    (L("wide_pad2", 32, 12, 72, 96, 3, 3, (1, 1), (2, 2)), 2),
    # whole rows of 8 * odd bytes (28, 12, 20 columns) with channels on 16-byte boundaries: 16-byte patch loads
    # that start before the row; tiles that cross images; a plane that rules the form out (27 x 28)
    (L("w28_shift", 40, 28, 28, 136, 3, 3, (1, 1), (1, 1)), 2),
    (L("w28_shift_bwd", 136, 28, 28, 72, 3, 3, (1, 1), (1, 1)), 3),
    (L("w12_shift", 48, 12, 12, 130, 3, 3, (1, 1), (1, 1)), 5),
    (L("w20_shift_pad0", 32, 10, 20, 128, 3, 3, (1, 1), (0, 0)), 3),
    (L("w28_h27", 32, 27, 28, 128, 3, 3, (1, 1), (1, 1)), 2),
    # rows of 4 * odd bytes (14, 6, 10, 22 columns): two rows to a 16-byte-loaded unit; odd channel counts rule it out
    (L("w14_pairs", 48, 14, 14, 130, 3, 3, (1, 1), (1, 1)), 5),
    (L("w14_pairs_bwd", 130, 14, 14, 72, 3, 3, (1, 1), (1, 1)), 3),
    (L("w6_pairs", 32, 6, 6, 128, 3, 3, (1, 1), (1, 1)), 7),
    (L("w10_pairs_pad0", 32, 10, 10, 128, 3, 3, (1, 1), (0, 0)), 3),
    (L("w22_pairs", 24, 8, 22, 96, 3, 3, (1, 1), (1, 1)), 3),
    (L("w14_c35", 35, 14, 14, 128, 3, 3, (1, 1), (1, 1)), 2),
    # filters of more than 2 MB: the XCDs keep to their channel tiles (8 tiles: one each; 16: two each; 4: pairs of XCDs)
    (L("1x1_k1024", 1040, 7, 7, 1024, 1, 1), 2),
    (L("1x1_k2048", 528, 7, 7, 2048, 1, 1), 2),
    (L("3x3_k512", 272, 6, 8, 512, 3, 3, (1, 1), (1, 1)), 2),
    # strided shapes the STAGED algorithm runs as a stride-1 convolution over the phase planes of the input:
    # 3x3 / stride 2 / pad 1 on even and odd images, 1x1 with strides 2 and 3 (odd image: the last row and column
    # are read by no window), 5x5 / stride 2 / pad 2 (every tap of the 3x3 inner filter real), strides that differ
    # per axis, many channels (several tiles and chunks), a 1x3 filter striding along its own axis
    (L("s2_3x3_even", 48, 28, 28, 160, 3, 3, (2, 2), (1, 1)), 3),
    (L("s2_3x3_odd", 24, 15, 17, 72, 3, 3, (2, 2), (1, 1)), 2),
    (L("s2_3x3_c130", 130, 14, 14, 136, 3, 3, (2, 2), (1, 1)), 2),
    (L("s2_1x1_odd", 40, 7, 7, 96, 1, 1, (2, 2)), 5),
    (L("s3_1x1", 32, 20, 20, 48, 1, 1, (3, 3)), 2),
    (L("s2_5x5", 16, 16, 16, 40, 5, 5, (2, 2), (2, 2)), 2),
    (L("s21_3x3", 32, 16, 12, 64, 3, 3, (2, 1), (1, 1)), 2),
    (L("s12_1x3", 32, 9, 20, 48, 1, 3, (1, 2), (0, 1)), 2),
    (L("s2_1x1_big", 256, 56, 56, 128, 1, 1, (2, 2)), 2),
    # 3x3 / stride 2 as a 2x2 inner convolution over the four phases (forward, backward-data): without padding on
    # an odd image (planes one row / column larger than the output), many channels; and a plain 2x2 filter
    (L("s2_3x3_valid_odd", 48, 35, 35, 72, 3, 3, (2, 2), (0, 0)), 3),
    (L("s2_3x3_valid_c136", 136, 17, 17, 96, 3, 3, (2, 2), (0, 0)), 2),
    (L("2x2_pad1", 24, 13, 18, 40, 2, 2, (1, 1), (1, 1)), 2),
    # at most 64 channels in and out on 32-column patches (4 chunks; 2 chunks with a ragged channel tile; a ragged
    # last chunk and more padding than the filter needs)
    (L("rf_c64_k64", 64, 20, 40, 64, 3, 3, (1, 1), (1, 1)), 3),
    (L("rf_c32_k40_pad0", 32, 12, 72, 40, 3, 3, (1, 1), (0, 0)), 2),
    (L("rf_c50_k64_pad2", 50, 17, 48, 64, 3, 3, (1, 1), (2, 2)), 2),
    # few input channels (C*R*S <= 32: one MFMA operand holds the whole reduction): rows longer than one
    # 64-pixel unit with a ragged end, more than 64 output channels, stride 2 without padding on an odd
    # image, one channel under a 5x5 filter, two channels under a 4x4 filter with a large padding, a
    # 1x1 filter over 32 channels on rows shorter than a unit, strides that differ per axis
    (L("few_c3_w150", 3, 9, 150, 70, 3, 3, (1, 1), (1, 1), relu_in=False), 2),
    (L("few_c3_s2_valid", 3, 37, 41, 32, 3, 3, (2, 2), (0, 0), relu_in=False), 3),
    (L("few_c1_5x5", 1, 20, 75, 130, 5, 5, (1, 1), (2, 2), relu_in=False), 2),
    (L("few_c2_4x4_pad3", 2, 11, 13, 24, 4, 4, (1, 1), (3, 3), relu_in=False), 2),
    (L("few_c32_1x1", 32, 7, 9, 40, 1, 1), 5),
    (L("few_c3_s12", 3, 12, 90, 64, 3, 3, (1, 2), (1, 0), relu_in=False), 2),
    # 1x1 / stride 1 with channel counts that are multiples of 8 (the matrix-product kernel): enough pixels
    # for the largest tile with a ragged channel tile and a reduction that ends in half a 16-channel step,
    # forward and backward-data swapped, an odd plane size (2-byte accesses, tiles spanning images)
    (L("pw_c72_k136", 72, 82, 82, 136, 1, 1), 5),
    (L("pw_c136_k72", 136, 82, 82, 72, 1, 1), 5),
    (L("pw_odd_c80_k200", 80, 81, 83, 200, 1, 1), 5),
    (L("pw_c264_k64", 264, 12, 10, 64, 1, 1), 7),
    # backward-filter of 1x1 layers on small planes: several slices of the batch with a ragged last wave,
    # planes shorter than one 16-pixel step, a plane of exactly 8 pixels
    (L("pw_slices_6x5", 72, 6, 5, 40, 1, 1), 19),
    (L("pw_tiny_3x3", 16, 3, 3, 24, 1, 1), 5),
    (L("pw_2x4", 24, 2, 4, 72, 1, 1), 9),
    # ... and on planes of a multiple of 4 pixels (operands through LDS): two images per workgroup with a
    # ragged last slice, ragged channel tiles, a last stage of one 16-pixel step
    (L("pw_lds_10x8", 264, 10, 8, 520, 1, 1), 41),
    # 5x5 with at most 64 channels out (forward) and in (backward-data) on a 35-wide image: the smaller pixel tile
    (L("5x5_c48_k64_w35", 48, 35, 35, 64, 5, 5, (1, 1), (2, 2)), 3),
    # 5x5 backward-filter, a filter row per launch: 32-column tiles of a wide image, a narrow image, 136 output channels
    (L("5x5_w40", 16, 12, 40, 40, 5, 5, (1, 1), (2, 2)), 2),
    (L("5x5_w12_k136", 20, 9, 12, 136, 5, 5, (1, 1), (2, 2)), 5),
    # 1x7 and 7x1 backward-filter on the row-stationary kernel: 32-column tiles of a wide image, 136 output channels
    (L("1x7_w40", 24, 10, 40, 40, 1, 7, (1, 1), (0, 3)), 2),
    (L("7x1_w40", 24, 10, 40, 40, 7, 1, (1, 1), (3, 0)), 2),
    (L("1x7_w12_k136", 20, 9, 12, 136, 1, 7, (1, 1), (0, 3)), 5),
    (L("7x1_w12_k136", 20, 9, 12, 136, 7, 1, (1, 1), (3, 0)), 5),
    # forward as a matrix product over (tap, channel) with the input gathered pixel by pixel (channels a multiple of
    # 16): each tile size with ragged channel tiles, strides that differ per axis under a 5x5 filter with padding, a
    # 4x4 stride-1 filter no tile kernel takes, a 1x1 / stride-2 layer that goes to the phase planes when they fit
    (L("g_s2_3x3_k136_big", 16, 130, 130, 136, 3, 3, (2, 2), (1, 1)), 8),
    (L("g_s2_3x3_k72_big", 16, 130, 130, 72, 3, 3, (2, 2), (1, 1)), 8),
    (L("g_s2_3x3_c32_k136", 32, 40, 40, 136, 3, 3, (2, 2), (1, 1)), 6),
    (L("g_5x5_s32", 32, 23, 31, 40, 5, 5, (3, 2), (2, 1)), 3),
    (L("g_4x4_s1", 16, 12, 14, 24, 4, 4, (1, 1), (1, 1)), 3),
    (L("g_1x1_s2_k512", 32, 14, 14, 512, 1, 1, (2, 2)), 4),
    # 1x1 / stride-2 backward-data written with the zeros of its 2x2 cells: an odd output width (single pixels per lane)
    (L("sc_1x1_s2_q5", 24, 10, 10, 40, 1, 1, (2, 2)), 3),
    # 1x1 backward-filter through LDS on planes that are no whole number of 4-pixel items (1, 2 and 3 pixels over):
    # the item over a plane's end starts early and is moved down; ragged channel tiles, several slices
    (L("pw_lds_9x9", 72, 9, 9, 136, 1, 1), 5),
    (L("pw_lds_6x11", 136, 6, 11, 40, 1, 1), 3),
    (L("pw_lds_5x19", 40, 5, 19, 72, 1, 1), 9),
    (L("pw_lds_13x5", 24, 13, 5, 24, 1, 1), 2),
    # 1x1 backward-filter with x gathered under each output pixel (zero workspace): padding that puts the first row
    # and column of outputs on zeros, an output plane of 30 pixels (2 over a 4-pixel item), strides that differ
    (L("gw_1x1_s2_pad1", 136, 9, 11, 72, 1, 1, (2, 2), (1, 1)), 5),
    (L("gw_1x1_s13", 40, 6, 31, 136, 1, 1, (1, 3)), 3),
    # zero-workspace strided backward-data by residue classes of the input pixels: two ragged tiles of input channels,
    # output channels short of a whole step, a stride larger than one side of the filter (classes without taps store
    # zeros), an image shorter than the stride along one axis
    (L("cls_5x4_s32_c136", 136, 19, 22, 40, 5, 4, (3, 2), (2, 1)), 3),
    (L("cls_2x5_s43", 24, 21, 17, 24, 2, 5, (4, 3), (1, 2)), 2),
    (L("cls_short_image", 16, 2, 37, 16, 1, 3, (3, 2), (0, 1)), 2),
]
IDS = [c[0].name for c in CASES]

_cache = {}


def _inputs(i, dtype):
    key = (i, dtype)
    if key not in _cache:
        layer, N = CASES[i]
        x, w, dy = wl.conv_inputs(layer, N, dtype, seed=100 + i)
        xo, wo, dyo = f64(x), f64(w), f64(dy)
        want = {
            sn.SN_CONV_FWD: oracle.conv2d_fwd(xo, wo, layer.stride, layer.pad),
            sn.SN_CONV_BWD_DATA: oracle.conv2d_bwd_data(dyo, wo, xo.shape, layer.stride, layer.pad),
            sn.SN_CONV_BWD_FILTER: oracle.conv2d_bwd_filter(xo, dyo, wo.shape, layer.stride, layer.pad),
        }
        _cache[key] = (x, w, dy, want)
    return _cache[key]


def _algos(shape, direction):
    """(algo, workspace bytes) pairs to try: every algorithm at its least and its preferred workspace."""
    out = []
    for algo in (sn.SN_ALGO_DIRECT, sn.SN_ALGO_IM2COL_GEMM, sn.SN_ALGO_STAGED, sn.SN_ALGO_WINOGRAD):
        try:
            mn, pf = sn.sn_conv_workspace_query(shape, direction, algo)
        except sn.SnError:
            continue
        out.append((algo, mn))
        if pf != mn:
            out.append((algo, pf))
            mid = (mn + pf) // 2 // 256 * 256
            if mid not in (mn, pf):
                out.append((algo, mid))
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("direction", [sn.SN_CONV_FWD, sn.SN_CONV_BWD_DATA, sn.SN_CONV_BWD_FILTER])
@pytest.mark.parametrize("case", range(len(CASES)), ids=IDS)
def test_conv_matches_oracle(case, direction, dtype):
    layer, N = CASES[case]
    x, w, dy, want = _inputs(case, dtype)
    out_dtypes = ["f32"] if (dtype == "f32" or direction == sn.SN_CONV_BWD_FILTER) else ["f32", "bf16"]
    for od in out_dtypes:
        shape = shape_of(layer, N, dtype, od)
        a, b = {sn.SN_CONV_FWD: (x, w), sn.SN_CONV_BWD_DATA: (dy, w), sn.SN_CONV_BWD_FILTER: (x, dy)}[direction]
        ref = want[direction]
        results = []
        for algo, ws in _algos(shape, direction):
            print("case", layer.name, "dir", direction, dtype, "->", od, "algo", sn.ALGO_NAMES[algo], "ws", ws, flush=True)
            got = run_conv(direction, a, b, ref.shape, DT[od] if direction != sn.SN_CONV_BWD_FILTER else torch.float32,
                           shape, algo, ws)
            err = rel_l2(f64(got), ref)
            assert err <= TOL[dtype], (layer.name, sn.ALGO_NAMES[algo], ws, err)
            assert elementwise_excess(f64(got), ref, TOL[dtype], got.dtype == torch.bfloat16) <= 0, \
                (layer.name, sn.ALGO_NAMES[algo], ws, "element")
            results.append(f64(got))
        # the budget changes speed, never the function: all variants agree with each other too
        for r in results[1:]:
            assert rel_l2(r, results[0]) <= 2 * TOL[dtype]


def test_auto_uses_budget_and_matches():
    layer, N = CASES[1]
    x, w, dy, want = _inputs(1, "bf16")
    shape = shape_of(layer, N, "bf16", "f32")
    for direction, a, b in ((sn.SN_CONV_FWD, x, w), (sn.SN_CONV_BWD_DATA, dy, w), (sn.SN_CONV_BWD_FILTER, x, dy)):
        for budget in (0, 1 << 20, 64 << 20):
            got = run_conv(direction, a, b, want[direction].shape, torch.float32, shape, sn.SN_ALGO_AUTO, budget)
            assert rel_l2(f64(got), want[direction]) <= TOL["bf16"]
            assert elementwise_excess(f64(got), want[direction], TOL["bf16"]) <= 0


def test_named_algo_with_too_little_workspace_is_refused():
    layer, N = CASES[1]
    x, w, dy, _ = _inputs(1, "f32")
    shape = shape_of(layer, N, "f32")
    mn, _ = sn.sn_conv_workspace_query(shape, sn.SN_CONV_FWD, sn.SN_ALGO_IM2COL_GEMM)
    P, Q = wl.out_hw(layer)
    y = torch.zeros((N, layer.K, P, Q), device="cuda")
    ws = torch.empty(mn - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(sn.SnError) as e:
        sn.sn_conv2d_fwd(x.cuda(), w.cuda(), y, shape, sn.SN_ALGO_IM2COL_GEMM, ws)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert float(y.abs().sum()) == 0.0      # nothing was launched


def test_autotune_records_and_plan_follows():
    layer, N = CASES[1]
    x, w, dy, want = _inputs(1, "bf16")
    shape = shape_of(layer, N, "bf16", "f32")
    sn.sn_planner_clear()
    _, pf = sn.sn_conv_workspace_query(shape, sn.SN_CONV_FWD, sn.SN_ALGO_IM2COL_GEMM)
    ws = torch.empty(pf, dtype=torch.uint8, device="cuda")
    P, Q = wl.out_hw(layer)
    y = torch.empty((N, layer.K, P, Q), device="cuda")
    sn.sn_conv_autotune(sn.SN_CONV_FWD, x.cuda(), w.cuda(), y, shape, ws, iters=2)
    algo, used, ms = sn.sn_conv_plan(shape, sn.SN_CONV_FWD, pf)
    assert ms is not None and ms > 0 and used <= pf
    algo0, used0, ms0 = sn.sn_conv_plan(shape, sn.SN_CONV_FWD, 0)
    assert algo0 == sn.SN_ALGO_DIRECT and used0 == 0 and ms0 >= ms
    assert rel_l2(f64(y), want[sn.SN_CONV_FWD]) <= TOL["bf16"]
    sn.sn_planner_clear()


def _random_cases(n, seed):
    """Seeded 3x3 / 1x1 stride-1 layers over the ranges where the tile kernels switch tilings: widths on both
    sides of the multiples of 8, 32-column patches and whole rows, paddings 0..2, channel counts on both sides
    of 64 and 128, a ragged last chunk of channels."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        R = int(rng.choice([3, 3, 3, 1]))
        W = int(rng.choice([6, 8, 10, 14, 16, 24, 28, 30, 32, 40, 56, 64, 66, 72, 80, 112]))
        H = int(rng.integers(3, 20))
        C = int(rng.choice([3, 8, 20, 32, 48, 64, 72, 96, 104, 128, 136, 200]))
        K = int(rng.choice([16, 40, 64, 72, 96, 128, 136, 192, 260]))
        pad = int(rng.integers(0, 3)) if R == 3 else 0
        N = int(rng.integers(1, 4))
        if H + 2 * pad < R or W + 2 * pad < R:
            continue
        cases.append((L("rnd%d" % i, C, H, W, K, R, R, (1, 1), (pad, pad)), N))
    return cases


RANDOM_CASES = _random_cases(36, 2024) + _random_cases(36, 7)


@pytest.mark.parametrize("case", range(len(RANDOM_CASES)),
                         ids=["%d_c%d_%dx%d_k%d_r%d_p%d_n%d" % (i, c[0].C, c[0].H, c[0].W, c[0].K, c[0].R, c[0].pad[0], c[1])
                              for i, c in enumerate(RANDOM_CASES)])
def test_conv_random_geometries(case):
    """bf16, every direction and algorithm at its preferred workspace, against the oracle."""
    layer, N = RANDOM_CASES[case]
    x, w, dy = wl.conv_inputs(layer, N, "bf16", seed=500 + case)
    xo, wo, dyo = f64(x), f64(w), f64(dy)
    want = {sn.SN_CONV_FWD: lambda: oracle.conv2d_fwd(xo, wo, layer.stride, layer.pad),
            sn.SN_CONV_BWD_DATA: lambda: oracle.conv2d_bwd_data(dyo, wo, xo.shape, layer.stride, layer.pad),
            sn.SN_CONV_BWD_FILTER: lambda: oracle.conv2d_bwd_filter(xo, dyo, wo.shape, layer.stride, layer.pad)}
    shape = shape_of(layer, N, "bf16", "bf16")
    for direction in (sn.SN_CONV_FWD, sn.SN_CONV_BWD_DATA, sn.SN_CONV_BWD_FILTER):
        ref = want[direction]()
        a, b = {sn.SN_CONV_FWD: (x, w), sn.SN_CONV_BWD_DATA: (dy, w), sn.SN_CONV_BWD_FILTER: (x, dy)}[direction]
        od = torch.float32 if direction == sn.SN_CONV_BWD_FILTER else torch.bfloat16
        for algo in (sn.SN_ALGO_DIRECT, sn.SN_ALGO_STAGED, sn.SN_ALGO_IM2COL_GEMM):
            try:
                mn, pf = sn.sn_conv_workspace_query(shape, direction, algo)
            except sn.SnError:
                continue
            print("case", layer, "N", N, "dir", direction, "algo", sn.ALGO_NAMES[algo], "ws", pf, flush=True)
            got = run_conv(direction, a, b, ref.shape, od, shape, algo, pf)
            err = rel_l2(f64(got), ref)
            assert err <= TOL["bf16"], (layer, N, direction, sn.ALGO_NAMES[algo], err)
            assert elementwise_excess(f64(got), ref, TOL["bf16"], got.dtype == torch.bfloat16) <= 0, \
                (layer, N, direction, sn.ALGO_NAMES[algo], "element")
