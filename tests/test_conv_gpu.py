"""Parity of the HIP path with the CPU oracle, through the C-ABI (needs an MI355X).

Bar: |y_gpu - y_ref| <= 1e-5 * sum|x*w| + 1e-6 for every output element, the sum taken over the
element's receptive field; exact equality where the inputs are small integers (all partial sums are
then exact in fp32, so a dropped or duplicated tap cannot hide inside the tolerance).
"""
import ctypes
import sys

import numpy as np
import pytest

import oracle
from paper_2103_16234_amd import binding, inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
TAP = binding.CONV_KERNEL_TAP
GENERIC = binding.CONV_KERNEL_GENERIC
POINTWISE = binding.CONV_KERNEL_POINTWISE
PANEL = binding.CONV_KERNEL_PANEL

_ref_cache = {}


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _reference(shape):
    key = shape
    if key not in _ref_cache:
        x, w = inputs.make_inputs(shape)
        y, ya = oracle.conv_ref(x, w, shape.pad_h, shape.pad_w)
        if len(_ref_cache) > 8:
            _ref_cache.clear()
        _ref_cache[key] = (x, w, y, ya)
    return _ref_cache[key]


def _run(shape, kernel=None, variant=0, tile_pix=0, chunk_c=0, exact=False, loader=0):
    x, w, y_ref, ya_ref = _reference(shape)
    xd = torch.from_numpy(x).cuda()
    wd = torch.from_numpy(w).cuda()
    yd = torch.full(shape.y_shape, float("nan"), device="cuda", dtype=torch.float32)   # every element must be written
    _say(f"[case] {shape.name} dims={shape.dims} kernel={kernel} variant={variant} tile_pix={tile_pix} chunk_c={chunk_c} loader={loader}")
    if kernel is None:
        binding.conv_fwd(xd, wd, shape.pad_h, shape.pad_w, y=yd)
        plan = binding.conv_fwd_plan(*shape.dims)
    else:
        _, plan = binding.conv_fwd_planned(xd, wd, shape.pad_h, shape.pad_w, kernel, variant, tile_pix, chunk_c, y=yd, loader=loader)
        assert loader == 0 or plan.loader == loader
    torch.cuda.synchronize()
    y = yd.cpu().numpy().astype(np.float64)
    assert not np.isnan(y).any(), "some outputs were never written"
    if exact:
        np.testing.assert_array_equal(y, y_ref)
    ok, worst = oracle.within_tolerance(y, y_ref, ya_ref)
    assert ok, f"worst (|diff|-1e-6)/(1e-5*sum|xw|) = {worst:.3g} with plan {plan.as_dict()}"
    return plan, worst


def S(name, *dims, x="u01", w="he", seed=1):
    return inputs.ConvShape(name, *dims, x, w, 100 + seed, 200 + seed)


# Small enough for the oracle in well under a second, large enough for several tiles and a ragged tail
# in every dimension a kernel blocks over (K vs 16/32/64, pixels vs the tile, C vs the chunk of 4k).
SMALL = [
    S("s3x3_ragged", 2, 20, 9, 11, 37, 3, 3, 1, 1),
    S("s3x3_even_w", 3, 12, 14, 14, 70, 3, 3, 1, 1),
    S("s3x3_w_mult4", 2, 8, 10, 12, 16, 3, 3, 1, 1),
    S("s3x3_odd_c", 1, 7, 13, 13, 18, 3, 3, 1, 1),          # C not a multiple of 4: scalar loaders
    S("s3x3_pad0", 2, 16, 12, 10, 33, 3, 3, 0, 0),
    S("s3x3_pad2", 1, 8, 6, 6, 20, 3, 3, 2, 2),            # wider padding than "same"
    S("s5x5", 2, 12, 11, 12, 21, 5, 5, 2, 2),
    S("s5x5_pad0", 1, 16, 9, 9, 40, 5, 5, 0, 0),
    S("s1x1", 3, 40, 7, 8, 50, 1, 1, 0, 0),
    S("s1x1_pad1", 2, 12, 5, 6, 17, 1, 1, 1, 1),            # zero frame around the output
    S("s3x3_tiny_map", 5, 24, 3, 3, 19, 3, 3, 1, 1),        # several images per pixel tile
    S("s3x3_1pix", 4, 8, 1, 1, 9, 3, 3, 1, 1),              # 1x1 maps: every tap but the centre is padding
    S("s3x3_wide", 1, 4, 4, 70, 8, 3, 3, 1, 1),             # rows longer than a pixel tile
    S("s3x3_single", 1, 1, 5, 5, 1, 3, 3, 1, 1),
    S("s3x3_c3_w8", 2, 3, 6, 8, 20, 3, 3, 1, 1),            # first-layer like: dwordx4 input rows, dword filter rows
    S("s3x3_w900", 1, 8, 5, 900, 20, 3, 3, 1, 1),           # a map wider than every shape's halo tile but the wide one's
    S("s5x5_w501", 1, 4, 6, 501, 9, 5, 5, 2, 2),            # ... with rows of single dwords
    S("s5x5_c6_w12", 1, 6, 9, 12, 18, 5, 5, 2, 2),
]


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: s.name)
def test_default_plan_matches_oracle(shape):
    _run(shape)


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: s.name)
def test_generic_kernel_matches_oracle(shape):
    _run(shape, kernel=GENERIC)


# Layers for the loader that moves global memory straight into LDS: every padding width's column shift, a batch that
# makes it the default on an odd width, rows of whole dwordx4 with ragged channel chunks, a 7x7 filter.
DIRECT = [
    S("d3x3_w8_pad2", 2, 24, 7, 8, 33, 3, 3, 2, 2),
    S("d3x3_n33_w13", 33, 8, 13, 13, 20, 3, 3, 1, 1),
    S("d5x5_w16", 1, 36, 6, 16, 17, 5, 5, 2, 2),
    S("d3x3_w4_c68", 3, 68, 5, 4, 70, 3, 3, 1, 1),
    S("d1x1_w20", 2, 52, 3, 20, 35, 1, 1, 0, 0),
]
REGISTERS, DIRECT_LOADS, LOADER_WAVES, DEEP_RING = 1, 2, 3, 4


@pytest.mark.parametrize("loader", [REGISTERS, DIRECT_LOADS, LOADER_WAVES, DEEP_RING])
@pytest.mark.parametrize("variant", range(32))
@pytest.mark.parametrize("shape", SMALL + DIRECT, ids=lambda s: s.name)
def test_every_tap_variant_matches_oracle(shape, variant, loader):
    if variant >= binding.conv_variant_count(TAP):
        pytest.skip("no such variant")
    try:
        _run(shape, kernel=TAP, variant=variant, loader=loader)
    except binding.ConvError as e:
        # a tile shape may not fit a layer (too few channels for its channel-splitting waves, LDS), and the direct
        # loader needs filter slices of whole dwordx4 and rows of dwordx4 or dwords: the library must say so instead
        # of running it
        assert e.code == -6


# Tile shapes whose last pixel tile is a four-pixel tail, multiplied by the 4x4x1 matrix instruction: every count of
# valid tail pixels (cut 0..3) and tiles that end before the tail (cut 5, 20), tiles that start mid-row and run across
# images, ragged K and C, every loader.
TAIL_VARIANTS = {26: 196, 27: 100, 28: 100, 29: 100}
TAIL_LAYERS = [
    S("t14", 3, 20, 14, 14, 70, 3, 3, 1, 1),
    S("t7", 9, 12, 7, 7, 33, 3, 3, 1, 1),
    S("t1x1_14", 2, 24, 14, 14, 64, 1, 1, 0, 0),
    S("t_w12", 2, 16, 9, 12, 40, 3, 3, 1, 1),
    S("t_w13_c6", 2, 6, 13, 13, 17, 3, 3, 1, 1),
]


@pytest.mark.parametrize("loader", [REGISTERS, DIRECT_LOADS, LOADER_WAVES])
@pytest.mark.parametrize("cut", [0, 1, 2, 3, 5, 20])
@pytest.mark.parametrize("variant", sorted(TAIL_VARIANTS))
@pytest.mark.parametrize("shape", TAIL_LAYERS, ids=lambda s: s.name)
def test_four_pixel_tail_tiles_match_oracle(shape, variant, cut, loader):
    tile = TAIL_VARIANTS[variant] - cut
    try:
        plan, _ = _run(shape, kernel=TAP, variant=variant, tile_pix=tile, loader=loader)
    except binding.ConvError as e:
        # a tile that is not a whole image touches more rows than the staging slots of some loader hold, and the direct
        # loaders need filter rows of whole dwordx4: the library must refuse, not run (the test below names cases that
        # may not be refused)
        assert e.code == -6
        return
    assert plan.variant == variant and plan.tile_pix == tile
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_plan_request(*shape.dims, TAP, variant, TAIL_VARIANTS[variant] + 1)      # a fifth tail pixel


def test_every_count_of_tail_pixels_runs():
    """(No refusal may hide a tail of one, two or three pixels: these two layers take every cut.)"""
    for variant, cap in TAIL_VARIANTS.items():
        for cut in (0, 1, 2, 3):
            for shape, loader in ((TAIL_LAYERS[1], LOADER_WAVES), (TAIL_LAYERS[2], REGISTERS)):
                plan, _ = _run(shape, kernel=TAP, variant=variant, tile_pix=cap - cut, loader=loader)
                assert plan.tile_pix == cap - cut


def test_four_pixel_tail_tiles_are_exact_on_integers_and_take_the_epilogue():
    shape = inputs.ConvShape("ints_tail", 3, 20, 14, 14, 70, 3, 3, 1, 1, "int", "int", 41, 42)
    for variant, tile in TAIL_VARIANTS.items():
        _run(shape, kernel=TAP, variant=variant, tile_pix=tile, exact=True)
        _run(shape, kernel=TAP, variant=variant, tile_pix=tile, exact=True, loader=LOADER_WAVES)
    shape = TAIL_LAYERS[0]
    x, w = inputs.make_inputs(shape)
    b = inputs.uniform_pm1(977, shape.K) * np.float32(0.5)
    y_ref, ya_ref = oracle.conv_bias_relu_ref(x, w, b, shape.pad_h, shape.pad_w, True)
    for variant, tile in TAIL_VARIANTS.items():
        yd = torch.full(shape.y_shape, float("nan"), device="cuda")
        _say(f"[case] tail bias_relu {shape.name} variant={variant}")
        _, plan = binding.conv_fwd_bias_relu(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda(),
                                             shape.pad_h, shape.pad_w, True, TAP, variant, tile, y=yd)
        torch.cuda.synchronize()
        assert plan.variant == variant
        y = yd.cpu().numpy().astype(np.float64)
        assert not np.isnan(y).any()
        ok, worst = oracle.within_tolerance(y, y_ref, ya_ref)
        assert ok, worst


def test_every_work_group_numbering_matches_oracle():
    """Channel tile fast, pixel tile fast and every group size in between (the numbering only decides which work-group
    computes which tile): 6 channel tiles of 16, with and without channel shares in the grid."""
    shape = S("order_k96", 3, 24, 9, 10, 96, 3, 3, 1, 1)
    x, w, y_ref, ya_ref = _reference(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    for order, k_group, want in ((1, 0, 6), (2, 0, 1), (3, 2, 2), (3, 3, 3), (3, 0, None), (0, 0, None)):
        yd = torch.full(shape.y_shape, float("nan"), device="cuda")
        _say(f"[case] {shape.name} order={order} k_group={k_group}")
        _, plan = binding.conv_fwd_planned(xd, wd, 1, 1, TAP, 2, 32, y=yd, order=order, k_group=k_group)
        torch.cuda.synchronize()
        assert plan.tile_k == 16 and (want is None or plan.k_group == want) and 6 % plan.k_group == 0
        assert plan.order == (1 if plan.k_group == 6 else 2 if plan.k_group == 1 else 3)
        y = yd.cpu().numpy().astype(np.float64)
        assert not np.isnan(y).any()
        assert oracle.within_tolerance(y, y_ref, ya_ref)[0]
    for order, k_group in ((3, 4), (3, 6), (3, 1), (4, 0)):             # not a divisor / not in between / no such order
        with pytest.raises(binding.ConvError):
            binding.conv_fwd_plan_request(*shape.dims, TAP, 2, 32, order=order, k_group=k_group)
    with pytest.raises(binding.ConvError):                              # five channel tiles: no group in between
        binding.conv_fwd_plan_request(3, 24, 9, 10, 80, 3, 3, 1, 1, TAP, 2, 32, order=3)


def test_direct_loader_runs_where_it_should():
    ran = 0
    for shape in SMALL + DIRECT:
        can = shape.C % 4 == 0                 # (rows of dwordx2 go dword by dword when the direct loader is asked for by name)
        for variant in (2, 4, 7, 23):
            try:
                plan, _ = binding.conv_fwd_plan_request(*shape.dims, TAP, variant, 0, 0, DIRECT_LOADS)
            except binding.ConvError as e:
                assert e.code == -6
                continue
            assert can and plan.loader == DIRECT_LOADS and plan.x_vec in (1, 4) and plan.w_vec == 4
            ran += 1
    assert ran >= 30
    # the default: direct wherever filter rows are whole dwordx4 (rows of the maps as dwordx4 or as single dwords)
    assert binding.conv_fwd_plan(8, 64, 56, 56, 64, 3, 3, 1, 1).loader == DIRECT_LOADS
    assert binding.conv_fwd_plan(1, 128, 13, 13, 384, 3, 3, 1, 1).loader == DIRECT_LOADS
    assert binding.conv_fwd_plan(1, 256, 13, 13, 384, 3, 3, 1, 1).loader == DEEP_RING      # one round of work-groups, 8 chunks
    assert binding.conv_fwd_plan(32, 256, 13, 13, 384, 3, 3, 1, 1).loader == DIRECT_LOADS
    assert binding.conv_fwd_plan(32, 512, 14, 14, 512, 3, 3, 1, 1).loader == LOADER_WAVES   # deep, rows of dwordx2
    assert binding.conv_fwd_plan(64, 32, 14, 14, 64, 3, 3, 1, 1).loader == DIRECT_LOADS
    assert binding.conv_fwd_plan(32, 64, 14, 14, 64, 3, 3, 1, 1).loader == DEEP_RING        # 392 work-groups of 16 x 64
    assert binding.conv_fwd_plan(8, 3, 224, 224, 64, 3, 3, 1, 1).loader == REGISTERS   # C = 3: dword filter rows


@pytest.mark.parametrize("tile_pix,chunk_c", [(1, 0), (17, 0), (33, 0), (50, 0), (64, 0)])
def test_odd_tile_requests(tile_pix, chunk_c):
    shape = S("s3x3_tiles", 2, 20, 9, 11, 37, 3, 3, 1, 1)
    ran = 0
    for variant in range(binding.conv_variant_count(TAP)):
        _, cap, _ = binding.conv_variant_info(TAP, variant)
        try:
            _run(shape, kernel=TAP, variant=variant, tile_pix=min(tile_pix, cap), chunk_c=chunk_c)
            ran += 1
        except binding.ConvError as e:
            assert e.code == -6
    assert ran >= 5


POINTWISE_SHAPES = [
    S("p_ragged", 3, 40, 7, 8, 50, 1, 1, 0, 0),            # HW = 56 < 64, C = 40 (2.5 steps of 16), K = 50
    S("p_two_tiles", 2, 64, 10, 10, 16, 1, 1, 0, 0),       # HW = 100: a full and a ragged pixel tile per image
    S("p_small_c", 1, 4, 8, 8, 70, 1, 1, 0, 0),            # a single 4-channel group
    S("p_deep", 1, 272, 4, 6, 33, 1, 1, 0, 0),             # 17 steps: more than any wave count
    S("p_one_k", 2, 32, 4, 4, 1, 1, 1, 0, 0),
    S("p_wide_tiles", 2, 48, 12, 25, 20, 1, 1, 0, 0),      # HW = 300: full and ragged 256- and 128-pixel work-groups
    S("p_7x7", 2, 36, 7, 7, 24, 1, 1, 0, 0),               # HW = 49: pixels move as single dwords
    S("p_13x13", 1, 20, 13, 13, 40, 1, 1, 0, 0),           # HW = 169: three pixel tiles, the last one ragged
]


@pytest.mark.parametrize("variant", range(20))
@pytest.mark.parametrize("shape", POINTWISE_SHAPES, ids=lambda s: s.name)
def test_every_pointwise_variant_matches_oracle(shape, variant):
    if variant >= binding.conv_variant_count(POINTWISE):
        pytest.skip("no such variant")
    plan, _ = _run(shape, kernel=POINTWISE, variant=variant)
    assert plan.kernel == POINTWISE and plan.workspace_bytes == 0


PANEL_SHAPES = POINTWISE_SHAPES + [
    S("p_batch", 37, 24, 6, 6, 70, 1, 1, 0, 0),            # 1332 pixels = 20.8 tiles that span images; K = 64 + 6
    S("p_batch_7x7", 9, 20, 7, 7, 35, 1, 1, 0, 0),         # dword pixels, 441 of them; C = 20 pads to 64
    S("p_batch_deep", 5, 132, 8, 8, 18, 1, 1, 0, 0),       # 9 steps pad to 12: clamped channel indices
    S("p_batch_c64", 6, 64, 8, 10, 64, 1, 1, 0, 0),        # nothing ragged: the unclamped, unmasked instance
    S("p_batch_13x13", 7, 24, 13, 13, 40, 1, 1, 0, 0),     # 169 pixels: dwords over flattened tiles
    S("p_batch_27x27", 3, 16, 27, 27, 33, 1, 1, 0, 0),     # 729 pixels: twelve tiles per image (dword-aligned dwordx4), the last with 25 pixels
    S("p_batch_11x23", 4, 20, 11, 23, 19, 1, 1, 0, 0),     # 253 pixels: four tiles per image, 3 pixels short
]


@pytest.mark.parametrize("groups", [0, 1, 2])
@pytest.mark.parametrize("variant", range(12))
@pytest.mark.parametrize("shape", PANEL_SHAPES, ids=lambda s: s.name)
def test_every_panel_variant_matches_oracle(shape, variant, groups):
    """Filter panel resident in LDS, waves streaming pixel tiles; few work-groups make every wave loop over tiles."""
    if variant >= binding.conv_variant_count(PANEL):
        pytest.skip("no such variant")
    plan, _ = _run(shape, kernel=PANEL, variant=variant, tile_pix=groups)
    assert plan.kernel == PANEL and plan.workspace_bytes == 0


def test_panel_needs_filters_that_fit_lds():
    shape = S("p_too_deep", 1, 4096, 2, 2, 64, 1, 1, 0, 0)   # 64 x 4096 floats = 1 MB of filters per channel tile
    x, w = inputs.make_inputs(shape)
    with pytest.raises(binding.ConvError) as e:
        binding.conv_fwd_planned(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), 0, 0, kernel=PANEL, variant=0)
    assert e.value.code == -6


@pytest.mark.parametrize("shape", POINTWISE_SHAPES, ids=lambda s: s.name)
def test_pointwise_shapes_default_plan_and_other_families(shape):
    plan, _ = _run(shape)
    assert plan.kernel in (POINTWISE, PANEL)
    _run(shape, kernel=GENERIC)
    _run(shape, kernel=TAP, variant=2)


def test_pointwise_needs_its_preconditions():
    for dims in [(1, 6, 8, 8, 8, 1, 1, 0, 0), (1, 8, 8, 8, 8, 1, 1, 1, 1), (1, 8, 8, 8, 8, 3, 3, 1, 1)]:
        shape = S("p_not", *dims)       # C % 4 != 0, padded, 3x3
        x, w = inputs.make_inputs(shape)
        with pytest.raises(binding.ConvError) as e:
            binding.conv_fwd_planned(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), dims[7], dims[8],
                                     kernel=POINTWISE)
        assert e.value.code == -6
        plan, _ = _run(shape)
        assert plan.kernel != POINTWISE


@pytest.mark.parametrize("shape", SMALL + POINTWISE_SHAPES[:3], ids=lambda s: s.name)
def test_two_stage_scheme_matches_oracle(shape):
    """The paper's own two-stage method (Section 3), opt-in with an explicit workspace."""
    x, w, y_ref, ya_ref = _reference(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    need = binding.conv_two_stage_workspace_bytes(*shape.dims)
    assert need == (0 if shape.R * shape.S == 1 else 4 * shape.R * shape.S * int(np.prod(shape.y_shape)))
    yd = torch.full(shape.y_shape, float("nan"), device="cuda")
    _say(f"[case] two-stage {shape.name} dims={shape.dims} workspace={need}")
    binding.conv_fwd_two_stage(xd, wd, shape.pad_h, shape.pad_w, y=yd)
    torch.cuda.synchronize()
    ok, worst = oracle.within_tolerance(yd.cpu().numpy(), y_ref, ya_ref)
    assert ok, worst
    if need:
        small = torch.empty(need // 4 - 1, device="cuda")
        with pytest.raises(binding.ConvError) as e:
            binding.conv_fwd_two_stage(xd, wd, shape.pad_h, shape.pad_w, workspace=small, y=yd)
        assert e.value.code == -7


def test_two_stage_scheme_other_filter_sizes_and_exactness():
    for shape in list(NONSQUARE):
        x, w, y_ref, ya_ref = _reference(shape)
        y = binding.conv_fwd_two_stage(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), shape.pad_h, shape.pad_w)
        torch.cuda.synchronize()
        assert oracle.within_tolerance(y.cpu().numpy(), y_ref, ya_ref)[0]
    shape = inputs.ConvShape("ints2", 2, 12, 9, 10, 35, 3, 3, 1, 1, "int", "int", 31, 32)
    x, w, y_ref, _ = _reference(shape)
    y = binding.conv_fwd_two_stage(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), 1, 1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y.cpu().numpy().astype(np.float64), y_ref)


NONSQUARE = [
    S("g2x3", 2, 5, 8, 9, 7, 2, 3, 1, 0),
    S("g7x7", 1, 3, 12, 12, 6, 7, 7, 3, 3),
    S("g1x5", 2, 4, 6, 10, 5, 1, 5, 0, 2),
    S("g4x4_pad5", 1, 2, 3, 3, 3, 4, 4, 5, 5),               # windows that lie wholly in the padding give exact zeros
]


EPILOGUE_CASES = [   # (shape, kernel family or None for the default plan, variant, tile_pix)
    (SMALL[0], None, 0, 0), (SMALL[0], GENERIC, 0, 0), (SMALL[0], TAP, 2, 0), (SMALL[0], TAP, 5, 0), (SMALL[0], TAP, 12, 0),
    (SMALL[6], TAP, 4, 0), (SMALL[6], TAP, 2, 0), (SMALL[3], TAP, 2, 0), (SMALL[1], TAP, 10, 0),
    (POINTWISE_SHAPES[0], POINTWISE, 0, 0), (POINTWISE_SHAPES[0], POINTWISE, 9, 0), (POINTWISE_SHAPES[6], POINTWISE, 2, 0),
    (PANEL_SHAPES[8], PANEL, 7, 1), (PANEL_SHAPES[9], PANEL, 6, 2), (PANEL_SHAPES[10], PANEL, 3, 0), (PANEL_SHAPES[0], PANEL, 1, 0),
    (NONSQUARE[0], None, 0, 0),
]


@pytest.mark.parametrize("with_bias,relu", [(False, True), (True, False), (True, True)])
@pytest.mark.parametrize("case", EPILOGUE_CASES, ids=lambda c: f"{c[0].name}-k{c[1]}v{c[2]}")
def test_fused_bias_relu_matches_oracle(case, with_bias, relu):
    """y = act(conv + bias) in the store path of the same kernel (Section 2.1), every kernel family."""
    shape, kernel, variant, tile_pix = case
    x, w = inputs.make_inputs(shape)
    b = inputs.uniform_pm1(900 + shape.K, shape.K) * np.float32(0.5) if with_bias else None
    y_ref, ya_ref = oracle.conv_bias_relu_ref(x, w, b, shape.pad_h, shape.pad_w, relu)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    bd = torch.from_numpy(b).cuda() if with_bias else None
    yd = torch.full(shape.y_shape, float("nan"), device="cuda")
    _say(f"[case] bias_relu {shape.name} dims={shape.dims} kernel={kernel} variant={variant} bias={with_bias} relu={relu}")
    _, plan = binding.conv_fwd_bias_relu(xd, wd, bd, shape.pad_h, shape.pad_w, relu, kernel, variant, tile_pix, y=yd)
    torch.cuda.synchronize()
    if kernel is not None:
        assert plan.kernel == kernel
    y = yd.cpu().numpy().astype(np.float64)
    assert not np.isnan(y).any()
    ok, worst = oracle.within_tolerance(y, y_ref, ya_ref)
    assert ok, worst
    if relu:
        assert (y >= 0).all() and (y == 0).any() and (y > 0).any()


def test_fused_epilogue_integer_inputs_are_exact():
    shape = inputs.ConvShape("ints_b", 2, 12, 9, 10, 35, 3, 3, 1, 1, "int", "int", 31, 32)
    x, w = inputs.make_inputs(shape)
    b = inputs.small_ints(77, shape.K, -20, 20)
    y_ref, _ = oracle.conv_bias_relu_ref(x, w, b, 1, 1, True)
    y, _ = binding.conv_fwd_bias_relu(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda(), 1, 1, True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y.cpu().numpy().astype(np.float64), y_ref)


# Channel splitting across work-groups (the work redistribution Section 5 leaves as future work): layers with many channels
# on few pixels, shares that are ragged (C = 100 over chunks of 16 / 32 / 64), scalar filter rows (C = 30), several
# images per tile, every filter size of the tap family.
SPLIT_SHAPES = [
    S("split_3x3_deep", 1, 200, 7, 7, 48, 3, 3, 1, 1),
    S("split_3x3_ragged_c", 2, 100, 6, 5, 37, 3, 3, 1, 1),
    S("split_3x3_odd_c", 1, 30, 9, 9, 20, 3, 3, 1, 1),
    S("split_5x5", 1, 72, 8, 8, 24, 5, 5, 2, 2),
    S("split_1x1_pad", 3, 96, 5, 6, 33, 1, 1, 1, 1),
    S("split_3x3_w8", 2, 88, 5, 8, 20, 3, 3, 1, 1),          # rows of whole dwordx4, shares with a ragged last chunk
]


def _run_split(shape, variant, c_splits, tile_pix=0, bias=False, relu=False, exact=False, workspace=None, loader=0):
    x, w = inputs.make_inputs(shape)
    b = inputs.uniform_pm1(900 + shape.K, shape.K) * np.float32(0.5) if bias else None
    y_ref, ya_ref = oracle.conv_bias_relu_ref(x, w, b, shape.pad_h, shape.pad_w, relu)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    bd = torch.from_numpy(b).cuda() if bias else None
    yd = torch.full(shape.y_shape, float("nan"), device="cuda")
    _say(f"[case] split_c {shape.name} dims={shape.dims} variant={variant} c_splits={c_splits} tile_pix={tile_pix} bias={bias} relu={relu}")
    _, plan = binding.conv_fwd_split_c(xd, wd, shape.pad_h, shape.pad_w, bd, relu, c_splits, variant, tile_pix, workspace=workspace, y=yd, loader=loader)
    torch.cuda.synchronize()
    y = yd.cpu().numpy().astype(np.float64)
    assert not np.isnan(y).any(), "some outputs were never written"
    if exact:
        np.testing.assert_array_equal(y, y_ref)
    ok, worst = oracle.within_tolerance(y, y_ref, ya_ref)
    assert ok, f"worst ratio {worst:.3g} with plan {plan.as_dict()}"
    return plan, yd


@pytest.mark.parametrize("loader", [REGISTERS, DIRECT_LOADS, LOADER_WAVES, DEEP_RING])
@pytest.mark.parametrize("c_splits", [2, 3, 5, 16])
@pytest.mark.parametrize("variant", [2, 5, 13, 17, 20, 7])
@pytest.mark.parametrize("shape", SPLIT_SHAPES, ids=lambda s: s.name)
def test_channel_splitting_matches_oracle(shape, variant, c_splits, loader):
    try:
        plan, _ = _run_split(shape, variant, c_splits, loader=loader)
    except binding.ConvError as e:
        assert e.code == -6   # the tile shape does not fit the layer
        return
    chunks = -(-shape.C // plan.chunk_c)
    assert 1 <= plan.c_splits <= min(c_splits, chunks)
    tiles = -(-shape.K // plan.tile_k) * -(-shape.N * plan.P * plan.Q // plan.tile_pix)
    assert plan.grid == tiles * plan.c_splits
    assert plan.workspace_bytes == (4 * plan.c_splits * shape.N * shape.K * plan.P * plan.Q if plan.c_splits > 1 else 0)


@pytest.mark.parametrize("bias,relu", [(True, False), (False, True), (True, True)])
def test_channel_splitting_applies_the_epilogue_after_the_sum(bias, relu):
    plan, _ = _run_split(SPLIT_SHAPES[0], 13, 4, bias=bias, relu=relu)
    assert plan.c_splits == 4
    _run_split(SPLIT_SHAPES[1], 2, 3, tile_pix=17, bias=bias, relu=relu)


def test_channel_splitting_is_exact_on_integers_and_reproducible():
    shape = inputs.ConvShape("split_ints", 1, 80, 7, 7, 40, 3, 3, 1, 1, "int", "int", 41, 42)
    ys = []
    for rep in range(2):
        plan, yd = _run_split(shape, 13, 5, exact=True)
        ys.append(yd.clone())
    assert plan.c_splits == 5
    assert torch.equal(ys[0], ys[1])
    shape = S("split_repro", 1, 160, 7, 7, 32, 3, 3, 1, 1)
    a = _run_split(shape, 20, 4)[1].clone()
    b = _run_split(shape, 20, 4)[1]
    assert torch.equal(a, b)     # the shares are added in share order, whichever work-group finishes first


def test_channel_splitting_default_plan_and_workspace_checks():
    shape = S("split_default", 1, 512, 7, 7, 512, 3, 3, 1, 1)
    want = binding.conv_fwd_plan_split_c(*shape.dims)
    assert want.kernel == TAP and want.c_splits > 1 and want.workspace_bytes == 4 * want.c_splits * shape.K * 49
    plan, _ = _run_split(shape, None, 0)
    assert (plan.variant, plan.tile_pix, plan.c_splits) == (want.variant, want.tile_pix, want.c_splits)
    x, w = inputs.make_inputs(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    short = torch.empty(want.workspace_bytes // 4 - 1, device="cuda")
    with pytest.raises(binding.ConvError) as e:
        binding.conv_fwd_split_c(xd, wd, 1, 1, workspace=short)
    assert e.value.code == -7
    lib = binding.load_library()
    yd = torch.empty(shape.y_shape, device="cuda")
    assert lib.conv_fwd_split_c(xd.data_ptr(), wd.data_ptr(), None, yd.data_ptr(), None, 0, *shape.dims, 0, None, None) == -1
    # only the tap family splits; the workspace-free entry points refuse a plan that asks for shares
    req = binding.ConvPlan()
    req.kernel, req.c_splits = GENERIC, 2
    ws = torch.empty(want.workspace_bytes // 4, device="cuda")
    assert lib.conv_fwd_split_c(xd.data_ptr(), wd.data_ptr(), None, yd.data_ptr(), ws.data_ptr(), ws.numel() * 4, *shape.dims, 0,
                                ctypes.byref(req), None) == -6
    req.kernel, req.variant = TAP, 13
    assert lib.conv_fwd_planned(xd.data_ptr(), wd.data_ptr(), yd.data_ptr(), *shape.dims, ctypes.byref(req), None) == -6
    # a layer the planner maps to another family keeps that mapping and needs no workspace
    other = binding.conv_fwd_plan_split_c(1, 256, 56, 56, 64, 1, 1, 0, 0)
    assert other.kernel == POINTWISE and other.c_splits == 1 and other.workspace_bytes == 0


@pytest.mark.parametrize("shape", NONSQUARE, ids=lambda s: s.name)
def test_other_filter_sizes_match_oracle(shape):
    """Sizes the tap kernel is built for run on it; anything else (2x3 here) on the generic kernel."""
    plan, _ = _run(shape)
    assert plan.kernel == (GENERIC if (shape.R, shape.S) == (2, 3) else TAP)
    _run(shape, kernel=GENERIC)


# Filter rows and columns, even and 7x7 filters in the tap kernel (built for a few tile shapes each): ragged K, C not a
# multiple of the chunk, padding that differs per axis, and one scalar-loader case (C = 6) per orientation.
EXTRA_SIZE_SHAPES = [
    S("t1x3", 2, 20, 9, 11, 37, 1, 3, 0, 1),
    S("t3x1", 2, 20, 9, 12, 37, 3, 1, 1, 0),
    S("t1x5", 1, 12, 7, 16, 20, 1, 5, 0, 2),
    S("t5x1", 3, 24, 10, 6, 33, 5, 1, 2, 0),
    S("t1x7", 1, 16, 6, 17, 18, 1, 7, 0, 3),
    S("t7x1", 2, 8, 17, 8, 40, 7, 1, 3, 0),
    S("t7x1_c6", 1, 6, 12, 8, 10, 7, 1, 3, 0),
    S("t1x3_c6_odd_w", 2, 6, 5, 9, 10, 1, 3, 0, 1),
    S("t2x2", 2, 16, 8, 8, 24, 2, 2, 0, 0),
    S("t2x2_pad1", 1, 12, 7, 9, 17, 2, 2, 1, 1),
    S("t4x4", 2, 8, 10, 12, 19, 4, 4, 1, 2),
    S("t7x7", 1, 8, 12, 12, 20, 7, 7, 3, 3),
]


@pytest.mark.parametrize("variant", [None, 2, 5, 7, 14, 16, 20, 22, 0])
@pytest.mark.parametrize("shape", EXTRA_SIZE_SHAPES, ids=lambda s: s.name)
def test_tap_kernel_on_other_filter_sizes(shape, variant):
    if variant is None:
        plan, _ = _run(shape)
        assert plan.kernel == TAP
        return
    try:
        _run(shape, kernel=TAP, variant=variant)
    except binding.ConvError as e:
        assert e.code == -6      # tile shape not built for this size (variant 0 never is), or it does not fit the layer


def test_other_filter_sizes_are_exact_on_integers():
    for dims in [(2, 12, 9, 10, 35, 1, 3, 0, 1), (1, 16, 8, 8, 20, 5, 1, 2, 0), (2, 8, 9, 9, 18, 2, 2, 1, 1),
                 (1, 8, 10, 10, 12, 4, 4, 2, 2), (1, 4, 9, 12, 6, 7, 7, 3, 3), (1, 12, 6, 14, 9, 1, 7, 0, 3)]:
        shape = inputs.ConvShape("ints_rs", *dims, "int", "int", 51, 52)
        plan, _ = _run(shape, exact=True)
        assert plan.kernel == TAP
        for variant in (2, 5, 7, 14, 16, 20, 22):
            try:
                _run(shape, kernel=TAP, variant=variant, exact=True)
            except binding.ConvError as e:
                assert e.code == -6
    shape = S("split_1x7", 1, 96, 7, 7, 32, 1, 7, 0, 3)
    _run_split(shape, 20, 3)


@pytest.mark.parametrize("dims", [(2, 12, 9, 10, 35, 3, 3, 1, 1), (1, 16, 8, 8, 20, 5, 5, 2, 2),
                                  (2, 24, 6, 8, 18, 1, 1, 0, 0), (1, 6, 7, 7, 5, 3, 3, 1, 1)])
def test_integer_inputs_are_exact(dims):
    shape = inputs.ConvShape("ints", *dims, "int", "int", 31, 32)
    _run(shape, exact=True)
    _run(shape, kernel=GENERIC, exact=True)
    if dims[5] == dims[6] and dims[5] in (1, 3, 5):
        for variant in range(binding.conv_variant_count(TAP)):
            try:
                _run(shape, kernel=TAP, variant=variant, exact=True)
            except binding.ConvError as e:
                assert e.code == -6
    if dims[5] == 1:
        for variant in range(binding.conv_variant_count(POINTWISE)):
            _run(shape, kernel=POINTWISE, variant=variant, exact=True)


def test_identity_filter_copies_input_bitwise():
    x = inputs.uniform_pm1(5, 2 * 24 * 6 * 7).reshape(2, 24, 6, 7)
    w = np.eye(24, dtype=np.float32).reshape(24, 24, 1, 1)
    y = binding.conv_fwd(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), 0, 0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y.cpu().numpy(), x)


def test_all_padding_windows_are_exact_zero():
    shape = S("zeros", 1, 4, 2, 2, 16, 3, 3, 4, 4)
    x, w = inputs.make_inputs(shape)
    y = binding.conv_fwd(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), 4, 4).cpu().numpy()
    assert y.shape == (1, 16, 8, 8)
    assert not y[:, :, :2, :].any() and not y[:, :, -2:, :].any() and not y[:, :, :, :2].any()
    _run(shape)


def test_results_are_bitwise_reproducible():
    shape = S("repro", 2, 32, 14, 14, 48, 3, 3, 1, 1)
    x, w = inputs.make_inputs(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    y1 = binding.conv_fwd(xd, wd, 1, 1).clone()
    y2 = binding.conv_fwd(xd, wd, 1, 1)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)


def test_misaligned_pointers_fall_back_to_narrow_loads():
    shape = S("misaligned", 2, 8, 10, 12, 16, 3, 3, 1, 1)
    x, w, y_ref, ya_ref = _reference(shape)
    for off in (1, 2):
        xbuf = torch.zeros(x.size + 4, device="cuda")
        wbuf = torch.zeros(w.size + 4, device="cuda")
        xd = xbuf[off:off + x.size].view(x.shape)
        wd = wbuf[off:off + w.size].view(w.shape)
        xd.copy_(torch.from_numpy(x))
        wd.copy_(torch.from_numpy(w))
        _say(f"[case] misaligned by {off} floats")
        y = binding.conv_fwd(xd, wd, 1, 1)
        torch.cuda.synchronize()
        ok, worst = oracle.within_tolerance(y.cpu().numpy(), y_ref, ya_ref)
        assert ok, worst


def test_panel_kernel_with_dword_aligned_tensors():
    """x and y that are only 4-byte aligned: the panel kernel moves pixels as dwordx4 at dword-aligned addresses."""
    shape = S("p_misaligned", 3, 32, 10, 25, 40, 1, 1, 0, 0)      # 250 pixels: four tiles per image, 6 pixels short
    x, w, y_ref, ya_ref = _reference(shape)
    ny = int(np.prod(shape.y_shape))
    for off in (1, 3):
        xbuf = torch.zeros(x.size + 4, device="cuda")
        ybuf = torch.full((ny + 8,), float("nan"), device="cuda")
        xd = xbuf[off:off + x.size].view(x.shape)
        yd = ybuf[off:off + ny].view(shape.y_shape)
        xd.copy_(torch.from_numpy(x))
        _say(f"[case] panel kernel, x and y misaligned by {off} floats")
        _, plan = binding.conv_fwd_planned(xd, torch.from_numpy(w).cuda(), 0, 0, PANEL, 7, 0, y=yd)
        torch.cuda.synchronize()
        assert plan.kernel == PANEL and plan.x_vec == 4
        ok, worst = oracle.within_tolerance(yd.cpu().numpy(), y_ref, ya_ref)
        assert ok, worst
        guard = ybuf.cpu().numpy()
        assert np.isnan(guard[:off]).all() and np.isnan(guard[off + ny:]).all()    # nothing written outside y


def test_runs_on_the_callers_stream():
    shape = S("stream", 1, 16, 14, 14, 16, 3, 3, 1, 1)
    x, w, y_ref, ya_ref = _reference(shape)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        y = binding.conv_fwd(xd, wd, 1, 1)
    st.synchronize()
    assert oracle.within_tolerance(y.cpu().numpy(), y_ref, ya_ref)[0]
    binding.conv_set_stream(None)


def test_repeated_plan_requests_hit_the_cache_and_stay_apart():
    """Resolved requests are remembered per (shape, request): the same request twice gives the same bits, and requests
    that differ in one field only (tile shape, pixel tile, work-groups per channel tile) are not mixed up."""
    shape = SMALL[1]
    x, w, y_ref, ya_ref = _reference(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    seen = {}
    for rep in range(2):
        for variant, tile_pix in ((2, 0), (2, 16), (5, 0), (5, 17), (2, 0)):
            y, plan = binding.conv_fwd_planned(xd, wd, shape.pad_h, shape.pad_w, TAP, variant, tile_pix, 0)
            torch.cuda.synchronize()
            assert plan.variant == variant and (tile_pix == 0 or plan.tile_pix == tile_pix)
            ok, worst = oracle.within_tolerance(y.cpu().numpy().astype(np.float64), y_ref, ya_ref)
            assert ok, worst
            key = (variant, tile_pix)
            if key in seen:
                assert torch.equal(seen[key][0], y) and seen[key][1] == (plan.tile_pix, plan.grid)
            seen[key] = (y.clone(), (plan.tile_pix, plan.grid))
    assert seen[(2, 0)][1] != seen[(2, 16)][1] and seen[(5, 0)][1] != seen[(5, 17)][1]
    pshape = PANEL_SHAPES[8]
    x, w, y_ref, ya_ref = _reference(pshape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    grids = set()
    for rep in range(2):
        for groups in (0, 1, 3):
            y, plan = binding.conv_fwd_planned(xd, wd, 0, 0, PANEL, 7, groups, 0)
            torch.cuda.synchronize()
            assert oracle.within_tolerance(y.cpu().numpy().astype(np.float64), y_ref, ya_ref)[0]
            if groups:
                assert plan.tile_pix == groups
            grids.add((groups, plan.grid))
    assert len(grids) == 3


def test_bad_plan_requests_are_refused():
    shape = S("badplan", 1, 8, 6, 6, 8, 3, 3, 1, 1)
    x, w = inputs.make_inputs(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    for kw in (dict(kernel=TAP, variant=99), dict(kernel=TAP, variant=0, tile_pix=10 ** 6),
               dict(kernel=TAP, variant=0, chunk_c=6), dict(kernel=42)):
        with pytest.raises(binding.ConvError) as e:
            binding.conv_fwd_planned(xd, wd, 1, 1, **kw)
        assert e.value.code == -6
    shape = S("badplan2", 1, 8, 6, 6, 8, 2, 2, 0, 0)
    x, w = inputs.make_inputs(shape)
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_planned(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), 0, 0, kernel=TAP)


@pytest.mark.parametrize("i", [1, 2, 3, 4, 5])
def test_benchmark_layers_full_size(i):
    """The five benchmark layers at full size, in the launch configuration the benchmark times
    (conv_fwd with its own plan), every output element against the oracle."""
    shape = inputs.config(i)
    plan, worst = _run(shape)
    _say(f"[result] {shape.name}: worst tolerance ratio {worst:.3g}, plan {plan.as_dict()}")
    _ref_cache.clear()


def test_conv_fwd_replays_from_a_hip_graph():
    """conv_fwd enqueues one kernel and nothing else, so it can be captured; every replay (with eager launches and
    synchronisations in between) must reproduce the eager result bit for bit."""
    shapes = [SMALL[0], SMALL[2], POINTWISE_SHAPES[0], PANEL_SHAPES[8]]      # SMALL[2]: rows of dwordx4, the direct loader
    tensors = []
    for s in shapes:
        x, w = inputs.make_inputs(s)
        xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        eager = binding.conv_fwd(xd, wd, s.pad_h, s.pad_w)
        tensors.append((s, xd, wd, eager, torch.zeros_like(eager)))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream (plans, kernel attributes)
        for s, xd, wd, _, out in tensors:
            binding.conv_fwd(xd, wd, s.pad_h, s.pad_w, y=out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for s, xd, wd, _, out in tensors:
            binding.conv_fwd(xd, wd, s.pad_h, s.pad_w, y=out)
    torch.cuda.synchronize()
    for rep in range(3):
        for _, _, _, _, out in tensors:
            out.fill_(float("nan"))
        torch.cuda.synchronize()
        _say(f"[case] graph replay {rep}")
        graph.replay()
        torch.cuda.synchronize()
        for s, xd, wd, eager, out in tensors:
            assert torch.equal(out, eager), s.name
            again = binding.conv_fwd(xd, wd, s.pad_h, s.pad_w)     # eager work between replays
            torch.cuda.synchronize()
            assert torch.equal(again, eager)


@pytest.mark.parametrize("shape", [SMALL[0], SMALL[6], POINTWISE_SHAPES[0], PANEL_SHAPES[8], NONSQUARE[0]], ids=lambda s: s.name)
def test_find_keeps_the_fastest_mapping(shape):
    """conv_fwd_find times every mapping, leaves y correct, and later conv_fwd calls use the winner."""
    x, w, y_ref, ya_ref = _reference(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    yd = torch.full(shape.y_shape, float("nan"), device="cuda")
    _say(f"[case] find {shape.name} dims={shape.dims}")
    flush = torch.empty(1 << 20, device="cuda") if shape.R == 3 else None     # 4 MiB scratch: the cold-cache timing path
    _, plan, us = binding.conv_fwd_find(xd, wd, shape.pad_h, shape.pad_w, y=yd, flush=flush)
    torch.cuda.synchronize()
    assert us > 0 and plan.workspace_bytes == 0 and plan.grid >= 1
    ok, worst = oracle.within_tolerance(yd.cpu().numpy(), y_ref, ya_ref)
    assert ok, worst
    again = binding.conv_fwd_plan(*shape.dims)                  # aligned tensors: the same cache entry
    assert (again.kernel, again.variant, again.tile_pix, again.grid) == (plan.kernel, plan.variant, plan.tile_pix, plan.grid)
    y2 = binding.conv_fwd(xd, wd, shape.pad_h, shape.pad_w)
    torch.cuda.synchronize()
    assert torch.equal(y2, yd)                                    # same mapping, same bits


@pytest.mark.parametrize("dims,period", [((4095, 8, 256, 256, 3, 3, 3, 1, 1), 7),        # x: 2,146,959,360 elements
                                         ((4095, 4, 64, 64, 128, 1, 1, 0, 0), 7)],       # y: 2,146,959,360 elements
                         ids=["x_near_2^31", "y_near_2^31"])
def test_tensors_just_below_the_element_limit(dims, period):
    """Maximum sizes: the largest tensors the boundary accepts (2^31 - 1 elements). The batch repeats a block of
    `period` distinct seeded images, so the oracle can evaluate sampled outputs from the block alone."""
    N, C, H, W, K, R, S, ph, pw = dims
    block = inputs.ConvShape("block", period, C, H, W, K, R, S, ph, pw, "u01", "he", 71, 72)
    xb, w = inputs.make_inputs(block)
    assert N % period == 0 and N * C * H * W < 2 ** 31 and N * K * block.P * block.Q < 2 ** 31
    xd = torch.from_numpy(xb).cuda().repeat(N // period, 1, 1, 1)
    wd = torch.from_numpy(w).cuda()
    _say(f"[case] near-limit tensors dims={dims}")
    y = binding.conv_fwd(xd, wd, ph, pw)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    npts = 400
    coords = np.stack([rng.integers(0, d, npts) for d in (N, K, block.P, block.Q)], axis=1)
    coords[:40, 0] = N - 1                                   # the far end of the tensors
    coords[:20, 2], coords[:20, 3] = block.P - 1, block.Q - 1
    coords[40:60, 0] = 0
    got = y[tuple(torch.from_numpy(coords.T).cuda())].cpu().numpy().astype(np.float64)
    folded = coords.copy().astype(np.int32)
    folded[:, 0] %= period
    ref, ref_abs = oracle.conv_ref_points(xb, w, ph, pw, folded)
    ok, worst = oracle.within_tolerance(got, ref, ref_abs)
    assert ok, worst
    assert not torch.isnan(y[-1]).any() and not torch.isnan(y[0]).any()


@pytest.mark.parametrize("shape", inputs.sweep_shapes()[1::4], ids=lambda s: s.name)
def test_sweep_layers_at_full_size(shape):
    """A slice of the synthetic sweep (every family, batch 1..256) at full size with the default plan: sampled
    outputs against the oracle, plus the layer's corners and last image."""
    x, w = inputs.make_inputs(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    yd = torch.full(shape.y_shape, float("nan"), device="cuda")
    _say(f"[case] sweep layer {shape.name} dims={shape.dims}")
    binding.conv_fwd(xd, wd, shape.pad_h, shape.pad_w, y=yd)
    torch.cuda.synchronize()
    assert not torch.isnan(yd).any(), "some outputs were never written"
    rng = np.random.default_rng(11)
    coords = np.stack([rng.integers(0, d, 300) for d in shape.y_shape], axis=1).astype(np.int32)
    coords[:8] = [[n, k, p, q] for n in (0, shape.N - 1) for k in (0, shape.K - 1) for (p, q) in ((0, 0), (shape.P - 1, shape.Q - 1))]
    got = yd[tuple(torch.from_numpy(coords.T.astype(np.int64)).cuda())].cpu().numpy().astype(np.float64)
    ref, ref_abs = oracle.conv_ref_points(x, w, shape.pad_h, shape.pad_w, coords)
    ok, worst = oracle.within_tolerance(got, ref, ref_abs)
    assert ok, worst


def _small_random_layers(seed, count):
    """Small layers with every kind of ragged edge: C a multiple of 4 (so that both loaders can run), any K, maps from a
    single row or column up to 25 wide whose rows move as dwordx4 or single dwords, padding from none to more than "same"."""
    import random
    rng = random.Random(seed)
    out = []
    for i in range(count):
        r = rng.choice([1, 3, 3, 5])
        pad = rng.choice([0, r // 2, r // 2, r // 2 + 1])
        lo = max(1, r - 2 * pad)
        h, w = rng.randint(lo, 20), rng.choice([v for v in range(lo, 26) if v % 4 == 0 or v % 2 == 1])
        out.append(inputs.ConvShape(f"fuzz{i}_{r}x{r}", rng.choice([1, 1, 2, 3, 5, 9]), 4 * rng.randint(1, 18), h, w,
                                    rng.randint(1, 70), r, r, pad, pad, "upm1", "he", 5000 + i, 6000 + i))
    return out


@pytest.mark.parametrize("shape", _small_random_layers(7, 24), ids=lambda s: s.name)
def test_both_loaders_on_random_small_layers(shape):
    """Random tile shapes and pixel tiles, with and without channel shares, through the register loader and through the
    direct one: every element against the oracle."""
    import random
    rng = random.Random(shape.x_seed)
    ran = 0
    for variant in rng.sample(range(binding.conv_variant_count(TAP)), 6):
        cap = binding.conv_variant_info(TAP, variant)[1]
        tile_pix = rng.choice([0, rng.randint(1, cap)])
        for loader in (REGISTERS, DIRECT_LOADS, LOADER_WAVES, DEEP_RING):
            try:
                _run(shape, kernel=TAP, variant=variant, tile_pix=tile_pix, loader=loader)
                _run_split(shape, variant, rng.choice([2, 3, 4]), tile_pix=tile_pix, loader=loader)
                ran += 1
            except binding.ConvError as e:
                assert e.code == -6
    assert ran >= 2


def _random_layers(seed, count):
    """Layers inside the paper's ranges but off the sweep grid (other batches, channel counts, map sizes)."""
    import random
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        f = rng.choice([1, 3, 3, 5])
        n, h = rng.choice([1, 2, 4, 16, 64]), rng.choice([7, 10, 14, 17, 20, 28, 35, 40, 56, 80])
        c, k = rng.choice([16, 24, 48, 80, 128, 160, 320, 448, 640]), rng.choice([24, 48, 96, 160, 256, 320, 512])
        if (f == 5 and c > 128) or n * c * h * h > 2 ** 22 or n * k * h * h > 2 ** 22:
            continue
        out.append(inputs.ConvShape(f"rand_{f}x{f}_n{n}_c{c}_{h}_k{k}", n, c, h, h, k, f, f, f // 2, f // 2, "u01", "he",
                                    9000 + len(out), 9500 + len(out)))
    return out


@pytest.mark.parametrize("shape", _random_layers(21, 16), ids=lambda s: s.name)
def test_random_layers_off_the_grid(shape):
    """Whatever the planner picks for shapes nobody tuned - default mapping, channel-splitting mapping and, for the tap
    family, the measured-best one - matches the oracle on sampled outputs."""
    x, w = inputs.make_inputs(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    rng = np.random.default_rng(13)
    coords = np.stack([rng.integers(0, d, 200) for d in shape.y_shape], axis=1).astype(np.int32)
    coords[:8] = [[n, k, p, q] for n in (0, shape.N - 1) for k in (0, shape.K - 1) for (p, q) in ((0, 0), (shape.P - 1, shape.Q - 1))]
    ref, ref_abs = oracle.conv_ref_points(x, w, shape.pad_h, shape.pad_w, coords)
    index = tuple(torch.from_numpy(coords.T.astype(np.int64)).cuda())

    def check(yd, what):
        assert not torch.isnan(yd).any(), f"{what}: some outputs were never written"
        ok, worst = oracle.within_tolerance(yd[index].cpu().numpy().astype(np.float64), ref, ref_abs)
        assert ok, (what, worst)

    _say(f"[case] random layer {shape.name} dims={shape.dims}")
    yd = torch.full(shape.y_shape, float("nan"), device="cuda")
    binding.conv_fwd(xd, wd, shape.pad_h, shape.pad_w, y=yd)
    torch.cuda.synchronize()
    check(yd, "default")
    yd.fill_(float("nan"))
    _, plan = binding.conv_fwd_split_c(xd, wd, shape.pad_h, shape.pad_w, y=yd)
    torch.cuda.synchronize()
    check(yd, f"split plan with {plan.c_splits} shares")
    yd.fill_(float("nan"))
    _, found, _ = binding.conv_fwd_find(xd, wd, shape.pad_h, shape.pad_w, y=yd)
    torch.cuda.synchronize()
    check(yd, f"found plan {found.kernel}/{found.variant}")


def test_micro_probes_run_and_report_their_work():
    lib = binding.load_library()
    binding.conv_set_stream(torch.cuda.current_stream())
    sink = torch.zeros(1, device="cuda")
    assert lib.conv_probe_mfma(10, sink.data_ptr()) == 8192 * 10 * 16 * 2048
    assert lib.conv_probe_mfma(0, sink.data_ptr()) == -2 and lib.conv_probe_mfma(10, None) == -1
    src = torch.arange(1 << 16, device="cuda", dtype=torch.float32)
    dst = torch.zeros_like(src)
    assert lib.conv_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel() * 4) == 0
    torch.cuda.synchronize()
    assert torch.equal(src, dst) and float(sink) == 0.0
    assert lib.conv_probe_copy(src.data_ptr() + 4, dst.data_ptr(), 1024) == -2       # not 16-byte aligned


def test_every_built_tap_instance_runs_on_some_layer():
    """No dropped kernel can hide behind a refused plan: every (filter size, tile shape) pair the build is pinned to
    (tests/test_abi_cpu.py) runs on at least one small layer with the register loader, every pair whose direct-load
    build a small layer can reach runs with that one too, and each run matches the oracle."""
    from test_abi_cpu import BUILT_TAP_INSTANCES
    probes = ((2, 8, 8, 8, 16), (2, 8, 4, 4, 16), (1, 4, 4, 4, 16), (1, 4, 2, 2, 1), (3, 8, 5, 5, 16))
    ran = {REGISTERS: set(), DIRECT_LOADS: set()}
    reachable_direct = set()
    for (R, S_), variants in sorted(BUILT_TAP_INSTANCES.items()):
        for v in sorted(variants):
            for loader in (REGISTERS, DIRECT_LOADS):
                for N, C, H, W, tile in probes:
                    dims = (N, C, H, W, 20, R, S_, R // 2, S_ // 2)
                    try:
                        binding.conv_fwd_plan_request(*dims, TAP, v, tile, loader=loader)      # host-only
                    except binding.ConvError as e:
                        assert e.code == -6
                        continue
                    if loader == DIRECT_LOADS:
                        reachable_direct.add((R, S_, v))
                    shape = S(f"inst_{R}x{S_}_v{v}_l{loader}_h{H}", *dims)
                    plan, _ = _run(shape, kernel=TAP, variant=v, tile_pix=tile, loader=loader)   # a refusal here is a failure
                    assert plan.variant == v and plan.loader == loader
                    ran[loader].add((R, S_, v))
                    break
    # the builds with loader waves: the nine tile shapes of eight waves at two per SIMD, for every filter size they take
    waves_ran = set()
    for (R, S_), variants in sorted(BUILT_TAP_INSTANCES.items()):
        for v in sorted(variants & {6, 7, 12, 19, 21, 26, 27, 28, 29}):
            for N, C, H, W, tile in probes:
                dims = (N, C, H, W, 20, R, S_, R // 2, S_ // 2)
                try:
                    binding.conv_fwd_plan_request(*dims, TAP, v, tile, loader=LOADER_WAVES)
                except binding.ConvError as e:
                    assert e.code == -6
                    continue
                plan, _ = _run(S(f"inst_{R}x{S_}_v{v}_l3_h{H}", *dims), kernel=TAP, variant=v, tile_pix=tile, loader=LOADER_WAVES)
                assert plan.loader == LOADER_WAVES and plan.block == 768
                waves_ran.add((R, S_, v))
                break
    assert waves_ran >= {(R, S_, v) for (R, S_) in ((1, 1), (3, 3)) for v in (6, 7, 12, 19, 21, 26, 27, 28, 29)} | {(5, 5, 12), (5, 5, 28)}, sorted(waves_ran)
    # the builds with the deep ring of staging copies: the tile shapes whose waves hold one or two MFMA tiles
    ring_ran = set()
    for (R, S_), variants in sorted(BUILT_TAP_INSTANCES.items()):
        for v in sorted(variants & {2, 4, 10, 11, 13, 17, 18, 20, 24, 25}):
            for N, C, H, W, tile in probes:
                dims = (N, C, H, W, 20, R, S_, R // 2, S_ // 2)
                try:
                    direct, _ = binding.conv_fwd_plan_request(*dims, TAP, v, tile, loader=DIRECT_LOADS)
                    binding.conv_fwd_plan_request(*dims, TAP, v, tile, loader=DEEP_RING)
                except binding.ConvError as e:
                    assert e.code == -6
                    continue
                plan, _ = _run(S(f"inst_{R}x{S_}_v{v}_l4_h{H}", *dims), kernel=TAP, variant=v, tile_pix=tile, loader=DEEP_RING)
                assert plan.loader == DEEP_RING and plan.block == direct.block and plan.lds_bytes >= 2 * direct.lds_bytes - 4096
                ring_ran.add((R, S_, v))
                break
    assert ring_ran >= {(R, S_, v) for (R, S_) in ((1, 1), (3, 3)) for v in (2, 4, 10, 11, 13, 18, 20, 24, 25)}, sorted(ring_ran)
    for v in (0, 5, 7, 22):
        with pytest.raises(binding.ConvError):
            binding.conv_fwd_plan_request(2, 8, 8, 8, 20, 3, 3, 1, 1, TAP, v, 16, loader=DEEP_RING)
    for v in (0, 2, 5, 13, 22):                                     # other tile shapes have no such build
        with pytest.raises(binding.ConvError):
            binding.conv_fwd_plan_request(2, 8, 8, 8, 20, 3, 3, 1, 1, TAP, v, 16, loader=LOADER_WAVES)
    want = {(R, S_, v) for (R, S_), variants in BUILT_TAP_INSTANCES.items() for v in variants}
    assert ran[REGISTERS] == want, sorted(want - ran[REGISTERS])
    assert ran[DIRECT_LOADS] == reachable_direct
    assert len(reachable_direct) >= len(want) * 3 // 4, sorted(want - reachable_direct)
