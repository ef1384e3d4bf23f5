"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates arguments before touching a device, and plans without a workspace."""
import ctypes
import os
import re

import pytest

from paper_2103_16234_amd import binding, inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        binding.build_library()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "convfwd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(conv_\w+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_plan_struct_matches_header():
    header = open(os.path.join(ROOT, "include", "convfwd.h")).read()
    body = re.search(r"typedef struct conv_plan \{(.*?)\} conv_plan_t;", header, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        names += [n.strip() for n in decl.split(None, 2 if decl.startswith("long long") else 1)[-1].split(",")]
    assert names == [n for n, _ in binding.ConvPlan._fields_]


def test_argument_errors_are_codes_not_crashes(lib):
    plan = binding.ConvPlan()
    ok = (1, 4, 8, 8, 4, 3, 3, 1, 1)
    assert lib.conv_fwd_plan(*ok, ctypes.byref(plan)) == 0
    assert lib.conv_fwd_plan(*ok, None) == -1
    for i in range(7):                                  # a non-positive dimension
        bad = list(ok)
        bad[i] = 0
        assert lib.conv_fwd_plan(*bad, ctypes.byref(plan)) == -2
    assert lib.conv_fwd_plan(1, 4, 8, 8, 4, 3, 3, -1, 1, ctypes.byref(plan)) == -2
    assert lib.conv_fwd_plan(1, 4, 2, 8, 4, 5, 5, 1, 2, ctypes.byref(plan)) == -3      # P = 0
    assert lib.conv_fwd_plan(1 << 12, 1 << 10, 1 << 5, 1 << 5, 4, 1, 1, 0, 0, ctypes.byref(plan)) == -4
    assert lib.conv_fwd_plan(1, 1 << 20, 1, 1, 1 << 11, 1, 1, 0, 0, ctypes.byref(plan)) == -4
    # null device pointers and bad shapes are rejected before any HIP call
    assert lib.conv_fwd(None, None, None, *ok) == -1
    assert lib.conv_fwd(1 << 20, 1 << 20, None, *ok) == -1
    assert lib.conv_fwd(1 << 20, 1 << 20, 1 << 20, 1, 4, 8, 8, 0, 3, 3, 1, 1) == -2
    assert lib.conv_two_stage_workspace_bytes(2, 4, 8, 8, 3, 3, 3, 1, 1) == 4 * 9 * 2 * 3 * 8 * 8
    assert lib.conv_two_stage_workspace_bytes(2, 4, 8, 8, 3, 1, 1, 0, 0) == 0
    assert lib.conv_two_stage_workspace_bytes(2, 4, 2, 8, 3, 5, 5, 1, 2) == -3
    assert lib.conv_fwd_two_stage(None, None, None, None, 0, *ok) == -1
    assert lib.conv_fwd_two_stage(1 << 20, 1 << 20, 1 << 20, None, 0, *ok) == -1      # workspace needed but null
    assert lib.conv_fwd_two_stage(1 << 20, 1 << 20, 1 << 20, 1 << 20, 16, *ok) == -7   # too small
    assert lib.conv_fwd_two_stage(1 << 20, 1 << 20, 1 << 20, 1 << 20, 1 << 40, 1, 20000, 8, 8, 4, 3, 3, 1, 1) == -6
    assert lib.conv_fwd_find(None, None, None, *ok, None, 0, None, None) == -1
    assert lib.conv_fwd_find(1 << 20, 1 << 20, 1 << 20, 1, 4, 2, 8, 4, 5, 5, 1, 2, None, 0, None, None) == -3   # validated before any GPU call
    assert lib.conv_fwd_plan_split_c(*ok, None) == -1
    assert lib.conv_fwd_plan_split_c(1, 4, 2, 8, 4, 5, 5, 1, 2, ctypes.byref(plan)) == -3
    assert lib.conv_fwd_split_c(None, None, None, None, None, 0, *ok, 0, None, None) == -1
    assert lib.conv_fwd_split_c(1 << 20, 1 << 20, None, 1 << 20, None, 0, 1, 4, 8, 8, 4, 3, 3, -1, 1, 0, None, None) == -2
    for code in (0, -1, -2, -3, -4, -5, -6, -7, -99):
        assert binding.conv_strerror(code)
    with pytest.raises(binding.ConvError) as e:
        binding.conv_fwd_plan(1, 4, 2, 8, 4, 5, 5, 1, 2)
    assert e.value.code == -3


def test_variant_tables(lib):
    assert binding.conv_variant_count(binding.CONV_KERNEL_GENERIC) == 1
    n = binding.conv_variant_count(binding.CONV_KERNEL_TAP)
    assert n >= 3 and binding.conv_variant_count(77) == 0
    assert binding.conv_variant_count(binding.CONV_KERNEL_POINTWISE) >= 4
    for v in range(n):
        tk, mp, bl = binding.conv_variant_info(binding.CONV_KERNEL_TAP, v)
        assert tk % 16 == 0 and mp % 16 in (0, 4) and bl % 64 == 0 and bl <= 1024        # 4: shapes whose last tile is a four-pixel tail
    with pytest.raises(binding.ConvError):
        binding.conv_variant_info(binding.CONV_KERNEL_TAP, n)


@pytest.mark.parametrize("i", [1, 2, 3, 4, 5])
def test_plans_of_the_benchmark_layers(i):
    c = inputs.config(i)
    p = binding.conv_fwd_plan(*c.dims)
    assert p.workspace_bytes == 0
    assert (p.P, p.Q) == (c.P, c.Q)
    assert p.flops == c.flops and p.bytes == c.algorithmic_bytes
    assert p.kernel != binding.CONV_KERNEL_GENERIC          # 1x1, 3x3 and 5x5 have specialised kernels
    assert p.lds_bytes <= 160 * 1024 and p.grid >= 1 and p.block in (64, 128, 256, 512, 768)
    tiles_k = -(-c.K // p.tile_k)
    tiles_p = -(-(c.N * c.P * c.Q) // p.tile_pix)
    assert p.grid == tiles_k * tiles_p


def test_plans_cover_odd_shapes():
    shapes = [(1, 3, 7, 7, 5, 3, 3, 1, 1), (2, 5, 13, 13, 17, 5, 5, 2, 2), (1, 832, 7, 7, 32, 1, 1, 0, 0),
              (3, 6, 9, 11, 4, 2, 3, 0, 1), (1, 4, 224, 224, 16, 3, 3, 1, 1), (1, 8, 5, 5, 8, 3, 3, 4, 4),
              (1, 1, 1, 1, 1, 1, 1, 0, 0)]
    for dims in shapes:
        p = binding.conv_fwd_plan(*dims)
        N, C, H, W, K, R, S, ph, pw = dims
        assert p.P == H + 2 * ph - R + 1 and p.Q == W + 2 * pw - S + 1
        assert p.workspace_bytes == 0 and p.lds_bytes <= 160 * 1024
        if (R, S) == (2, 3):
            assert p.kernel == binding.CONV_KERNEL_GENERIC
    # filter rows / columns, even and 7x7 filters have tap kernels too (a few tile shapes each); other sizes do not
    for R, S in [(1, 3), (3, 1), (1, 5), (5, 1), (1, 7), (7, 1), (2, 2), (4, 4), (7, 7)]:
        p = binding.conv_fwd_plan(8, 64, 17, 17, 96, R, S, (R - 1) // 2, (S - 1) // 2)
        assert p.kernel == binding.CONV_KERNEL_TAP and p.variant in (2, 5, 7, 14, 16, 20, 22)
    for R, S in [(2, 3), (6, 6), (3, 5), (9, 9), (1, 2)]:
        assert binding.conv_fwd_plan(8, 64, 17, 17, 96, R, S, 0, 0).kernel == binding.CONV_KERNEL_GENERIC


def test_plans_of_the_sweep_grid_are_well_formed():
    """Host-only planner over the synthetic layers of the sweep grid: every plan is a launch the kernels accept."""
    tap, pw, panel = binding.CONV_KERNEL_TAP, binding.CONV_KERNEL_POINTWISE, binding.CONV_KERNEL_PANEL
    families = set()
    for s in inputs.sweep_shapes():
        p = binding.conv_fwd_plan(*s.dims)
        families.add(p.kernel)
        assert p.workspace_bytes == 0 and (p.P, p.Q) == (s.P, s.Q)
        assert p.flops == s.flops and p.bytes == s.algorithmic_bytes
        assert 1 <= p.grid < 2 ** 31 and p.block in (64, 128, 256, 512, 768, 1024) and 0 <= p.lds_bytes <= 160 * 1024
        assert p.kernel in (tap, pw, panel)                      # every sweep layer has a specialised kernel
        assert 0 <= p.variant < binding.conv_variant_count(p.kernel)
        tile_k, cap, block = binding.conv_variant_info(p.kernel, p.variant)
        assert p.block == block + (256 if p.loader == 3 else 0) and p.tile_k == tile_k     # (four loader waves)
        total = s.N * s.P * s.Q
        if p.kernel == tap:
            assert 1 <= p.tile_pix <= cap
            assert p.grid == -(-s.K // p.tile_k) * -(-total // p.tile_pix)
            ktiles = -(-s.K // p.tile_k)           # the work-group numbering walks whole groups of channel tiles
            assert 1 <= p.k_group <= ktiles and ktiles % p.k_group == 0
            assert p.order == (1 if p.k_group == ktiles else 2 if p.k_group == 1 else 3)
            assert p.chunk_c % 4 == 0 and p.x_vec in (1, 2, 4) and p.w_vec in (1, 4)
            assert s.W % p.x_vec == 0 and (p.w_vec == 1 or s.C % 4 == 0)
        elif p.kernel == pw:
            assert s.R == 1 and s.pad_h == 0 and s.C % 4 == 0
            assert p.grid == -(-s.K // p.tile_k) * s.N * -(-(s.H * s.W) // p.tile_pix)
        else:
            assert s.R == 1 and s.pad_h == 0 and s.C % 4 == 0
            groups = p.tile_pix                                  # work-groups per channel tile
            assert p.grid == -(-s.K // p.tile_k) * groups
            tiles = s.N * -(-(s.H * s.W) // 64)                      # at most: tiles cut per image
            assert 1 <= groups * (block // 64) <= tiles + block // 64   # no more waves than 64-pixel tiles (+ one work-group)
            assert p.lds_bytes >= 4 * p.tile_k * s.C                 # the whole filter panel of a channel tile
    assert families == {tap, pw, panel}


def test_channel_splitting_plans_are_well_formed():
    """Host-only: the splitting planner only ever changes tap-family layers, sizes its workspace as documented, keeps
    at most two work-groups per CU when it splits, and splits the deep batch-1 layers it exists for."""
    tap = binding.CONV_KERNEL_TAP
    split_layers = 0
    for s in inputs.sweep_shapes():
        base = binding.conv_fwd_plan(*s.dims)
        p = binding.conv_fwd_plan_split_c(*s.dims)
        assert base.c_splits == 1 and base.workspace_bytes == 0
        assert p.c_splits >= 1 and (p.P, p.Q) == (s.P, s.Q)
        if base.kernel != tap:
            assert (p.kernel, p.variant, p.tile_pix, p.grid, p.c_splits) == (base.kernel, base.variant, base.tile_pix, base.grid, 1)
        if p.c_splits == 1:
            assert p.workspace_bytes == 0
            continue
        split_layers += 1
        assert p.kernel == tap
        assert p.workspace_bytes == 4 * p.c_splits * s.N * s.K * s.P * s.Q
        tiles = -(-s.K // p.tile_k) * -(-(s.N * s.P * s.Q) // p.tile_pix)
        assert p.grid == tiles * p.c_splits <= 512
        assert p.c_splits <= -(-s.C // p.chunk_c)                # every share holds at least one chunk
    assert split_layers >= 3
    deep = binding.conv_fwd_plan_split_c(1, 512, 7, 7, 512, 3, 3, 1, 1)
    assert deep.c_splits > 1
    wide = binding.conv_fwd_plan_split_c(32, 64, 56, 56, 64, 3, 3, 1, 1)
    assert wide.c_splits == 1                                    # plenty of output tiles: nothing to gain


def test_plan_requests_resolve_on_the_host_and_the_planner_minimises_the_model():
    """conv_fwd_plan_request is conv_fwd_planned without the launch; for tap-family layers the default plan is the
    request with the smallest modelled cost among every tile shape at its capacity tile and at the default's tile."""
    tap = binding.CONV_KERNEL_TAP
    lib = binding.load_library()
    req, res = binding.ConvPlan(), binding.ConvPlan()
    ok = (1, 4, 8, 8, 4, 3, 3, 1, 1)
    assert lib.conv_fwd_plan_request(*ok, None, ctypes.byref(res), None) == -1
    assert lib.conv_fwd_plan_request(*ok, ctypes.byref(req), None, None) == -1
    assert lib.conv_fwd_plan_request(1, 4, 2, 8, 4, 5, 5, 1, 2, ctypes.byref(req), ctypes.byref(res), None) == -3
    req.kernel, req.variant = tap, 999
    assert lib.conv_fwd_plan_request(*ok, ctypes.byref(req), ctypes.byref(res), None) == -6
    req.kernel, req.variant = binding.CONV_KERNEL_POINTWISE, 0
    assert lib.conv_fwd_plan_request(*ok, ctypes.byref(req), ctypes.byref(res), None) == -6       # 3x3: not a pointwise layer
    checked = 0
    for s in inputs.sweep_shapes()[5::9]:
        base = binding.conv_fwd_plan(*s.dims)
        deep = base.loader == binding.CONV_LOADER_DIRECT_DEEP    # a measured substitution made after the model's choice
        same, cost = binding.conv_fwd_plan_request(*s.dims, base.kernel, base.variant, base.tile_pix,
                                                   loader=base.loader if deep else 0)
        assert (same.kernel, same.variant, same.tile_pix, same.grid, same.block, same.lds_bytes) == \
               (base.kernel, base.variant, base.tile_pix, base.grid, base.block, base.lds_bytes)
        if base.kernel != tap:
            assert cost == 0.0
            continue
        assert cost > 0.0
        if deep:
            continue
        if s.dims in [tuple(c.dims) for c in (inputs.config(i) for i in range(1, 6))]:
            continue                                             # the five benchmark layers use measured mappings
        for variant in range(binding.conv_variant_count(tap)):
            for tile in (0, base.tile_pix):
                try:
                    other, c = binding.conv_fwd_plan_request(*s.dims, tap, variant, tile)
                except binding.ConvError as e:
                    assert e.code == -6
                    continue
                assert c >= cost * 0.998, (s.name, variant, other.tile_pix, c, cost)
        checked += 1
    assert checked >= 5
    split, c2 = binding.conv_fwd_plan_request(1, 512, 7, 7, 512, 3, 3, 1, 1, tap, 13, 25, c_splits=8)
    whole, c1 = binding.conv_fwd_plan_request(1, 512, 7, 7, 512, 3, 3, 1, 1, tap, 13, 25)
    assert split.c_splits == 8 and split.grid == 8 * whole.grid and split.workspace_bytes == 4 * 8 * 512 * 49
    assert c2 < c1                                               # the model agrees that this layer wants shares


def test_panel_plans_follow_the_batch():
    """The panel kernel takes over from the register-streaming kernel once a 1x1 layer has enough tiles."""
    small = binding.conv_fwd_plan(1, 256, 56, 56, 64, 1, 1, 0, 0)
    big = binding.conv_fwd_plan(32, 256, 56, 56, 64, 1, 1, 0, 0)
    assert small.kernel == binding.CONV_KERNEL_POINTWISE and big.kernel == binding.CONV_KERNEL_PANEL
    deep = binding.conv_fwd_plan(128, 4096, 7, 7, 64, 1, 1, 0, 0)      # 16 x 4096 floats of filters do not fit LDS
    assert deep.kernel != binding.CONV_KERNEL_PANEL


def test_thin_small_pointwise_layers_stream_on_any_map():
    """Up to 32 channels and ~120 MFLOP the register-streaming shape takes a 1x1 layer whatever its 256-pixel tiles waste."""
    odd = binding.conv_fwd_plan(2, 16, 17, 17, 768, 1, 1, 0, 0)
    assert (odd.kernel, odd.variant) == (binding.CONV_KERNEL_POINTWISE, 8)
    big = binding.conv_fwd_plan(8, 32, 35, 35, 768, 1, 1, 0, 0)        # 480 MFLOP: the panel kernel keeps it
    assert big.kernel == binding.CONV_KERNEL_PANEL


def test_sixteen_channel_panels_stay_off_grids_just_over_the_cu_count():
    """1 x 256 x 56 x 56 -> 320 would make 260 work-groups of one tile per wave on 256 CUs: the pointwise kernel takes it with
    eight channel shares; with 768 filters the grid is 336 and the panel kernel keeps the layer."""
    over = binding.conv_fwd_plan(1, 256, 56, 56, 320, 1, 1, 0, 0)
    assert (over.kernel, over.variant) == (binding.CONV_KERNEL_POINTWISE, 3)
    fine = binding.conv_fwd_plan(1, 256, 40, 40, 768, 1, 1, 0, 0)
    assert (fine.kernel, fine.variant) == (binding.CONV_KERNEL_PANEL, 5)


def test_panel_shapes_on_unaligned_maps_follow_the_grid_they_would_get():
    """13 x 13 and 27 x 27 maps: the panel shape is the one whose grid fills the chip, not a threshold on the work.
    64 x 384 x 13 x 13 -> 384 has 169 tiles: 64-channel panels would make 258 work-groups of one tile per wave on 256 CUs
    (two rounds); twice the batch makes 510 of them, which is two clean rounds and the fastest shape measured."""
    panel = binding.CONV_KERNEL_PANEL
    awkward = binding.conv_fwd_plan(64, 384, 13, 13, 384, 1, 1, 0, 0)
    assert awkward.kernel == panel and awkward.variant != 6
    clean = binding.conv_fwd_plan(128, 384, 13, 13, 384, 1, 1, 0, 0)
    assert (clean.kernel, clean.variant, clean.grid) == (panel, 6, 510)
    few_filters = binding.conv_fwd_plan(128, 256, 13, 13, 64, 1, 1, 0, 0)   # one round of 32-channel panels, not two of 16
    assert (few_filters.kernel, few_filters.variant) == (panel, 7)
    thin = binding.conv_fwd_plan(48, 320, 27, 27, 48, 1, 1, 0, 0)           # three 16-channel tiles, none padded
    assert (thin.kernel, thin.variant) == (panel, 5)
    # every pick is a shape the kernel is built for and whose panel fits LDS
    for n, c, hw, k in [(16, 256, 7, 384), (256, 1024, 7, 256), (8, 640, 15, 512), (192, 128, 27, 768), (32, 2048, 13, 64)]:
        plan = binding.conv_fwd_plan(n, c, hw, hw, k, 1, 1, 0, 0)
        if plan.kernel == panel:
            assert plan.variant in (5, 6, 7, 8) and plan.lds_bytes <= 160 * 1024 and plan.grid >= 1


def test_tap_plans_name_their_loader():
    """Tap-family plans report how chunks reach LDS; a request may name the loader, and the direct one is refused
    where it cannot run (dword filter rows, input rows that move as dwordx2)."""
    tap, registers, direct = binding.CONV_KERNEL_TAP, binding.CONV_LOADER_REGISTERS, binding.CONV_LOADER_DIRECT
    for dims, want in [((8, 64, 56, 56, 64, 3, 3, 1, 1), direct),        # rows of whole dwordx4
                       ((1, 48, 28, 28, 128, 5, 5, 2, 2), direct),
                       ((1, 256, 13, 13, 384, 3, 3, 1, 1), binding.CONV_LOADER_DIRECT_DEEP),  # one round of work-groups, 8 chunks
                       ((1, 128, 13, 13, 384, 3, 3, 1, 1), direct),      # odd width: rows of single dwords
                       ((8, 256, 13, 13, 384, 3, 3, 1, 1), direct),
                       ((32, 192, 7, 7, 384, 3, 3, 1, 1), direct),       # 7x7 maps
                       ((32, 512, 14, 14, 512, 3, 3, 1, 1), binding.CONV_LOADER_DIRECT_WAVES),  # rows of dwordx2, deep: loader waves
                       ((32, 64, 14, 14, 64, 3, 3, 1, 1), binding.CONV_LOADER_DIRECT_DEEP),   # 392 work-groups of 16 x 64, 8 chunks
                       ((64, 32, 14, 14, 64, 3, 3, 1, 1), direct),       # rows of dwordx2 go dword by dword
                       ((8, 3, 224, 224, 64, 3, 3, 1, 1), registers)]:   # 3 input channels: dword filter rows
        plan = binding.conv_fwd_plan(*dims)
        assert plan.kernel == tap and plan.loader == want, (dims, plan.as_dict())
        for loader in (registers, direct):
            try:
                other, _ = binding.conv_fwd_plan_request(*dims, tap, plan.variant, plan.tile_pix, loader=loader)
            except binding.ConvError as e:
                assert e.code == -6 and loader == direct and dims[1] % 4 != 0, (dims, loader)
                continue
            assert other.loader == loader and other.grid == plan.grid
            assert other.block == plan.block - (256 if plan.loader == 3 else 0)
            assert other.lds_bytes <= 160 * 1024
            if plan.loader == binding.CONV_LOADER_DIRECT_DEEP and loader == direct:
                assert plan.lds_bytes == 2 * other.lds_bytes       # four staging copies instead of two
    assert binding.conv_fwd_plan(32, 256, 56, 56, 64, 1, 1, 0, 0).loader == 0      # panel kernel: not a tap plan
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_plan_request(8, 64, 56, 56, 64, 3, 3, 1, 1, tap, 7, 0, loader=5)
    # the deep ring: a build of the tile shapes whose waves hold one or two MFMA tiles; dwordx2 rows move as dwords
    ring, _ = binding.conv_fwd_plan_request(1, 512, 14, 14, 512, 3, 3, 1, 1, tap, 18, 28, loader=binding.CONV_LOADER_DIRECT_DEEP)
    assert ring.loader == 4 and ring.block == 512 and ring.x_vec == 1 and ring.lds_bytes <= 160 * 1024
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_plan_request(8, 64, 56, 56, 64, 3, 3, 1, 1, tap, 7, 0, loader=binding.CONV_LOADER_DIRECT_DEEP)  # 7 tiles per wave
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_plan_request(8, 6, 14, 14, 64, 3, 3, 1, 1, tap, 2, 64, loader=binding.CONV_LOADER_DIRECT_DEEP)  # dword filter rows
    # loader waves: a build of the eight-wave tile shapes only; four more waves in the work-group, rows of dwordx2 as dwords
    waves, _ = binding.conv_fwd_plan_request(32, 512, 14, 14, 512, 3, 3, 1, 1, tap, 6, 196, loader=binding.CONV_LOADER_DIRECT_WAVES)
    assert waves.loader == 3 and waves.block == 768 and waves.x_vec == 1 and waves.grid == 256
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_plan_request(32, 512, 14, 14, 512, 3, 3, 1, 1, tap, 0, 196, loader=3)       # four waves: no such build
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_plan_request(8, 6, 14, 14, 64, 3, 3, 1, 1, tap, 6, 196, loader=3)           # dword filter rows


# Which (filter size, tile shape) pairs of the tap family are built. Written out by hand from the rule in the
# kernels' header (a shape takes a filter size if its filter block per chunk fits the staging registers); a change
# of the build that drops or adds an instance must change this table too.
_ALL = set(range(31))
_EXTRA = {2, 5, 7, 14, 16, 20, 22}
BUILT_TAP_INSTANCES = {
    (1, 1): _ALL, (3, 3): _ALL, (5, 5): {2, 4, 8, 9, 10, 11, 12, 14, 15, 16, 22, 23, 24, 28, 30},
    (1, 3): _EXTRA, (3, 1): _EXTRA, (1, 5): _EXTRA, (5, 1): _EXTRA, (1, 7): _EXTRA, (7, 1): _EXTRA,
    (2, 2): _EXTRA, (4, 4): _EXTRA, (7, 7): {2, 14, 16, 22},
}


def built_tap_instances():
    """(R, S) -> tile shapes the library accepts for that filter size, asked of the host-only resolver on layers
    small enough for every tile shape's LDS and staging registers (a pair counts as built if any of them resolves)."""
    tap = binding.CONV_KERNEL_TAP
    found = {}
    for (R, S) in BUILT_TAP_INSTANCES:
        ok = set()
        for v in range(binding.conv_variant_count(tap)):
            for N, C, H, tile in ((2, 8, 8, 16), (2, 8, 4, 16), (1, 4, 4, 16), (1, 4, 2, 1)):
                try:
                    binding.conv_fwd_plan_request(N, C, H, H, 16, R, S, R // 2, S // 2, tap, v, tile)
                    ok.add(v)
                except binding.ConvError as e:
                    assert e.code == -6
        found[(R, S)] = ok
    return found


def test_the_set_of_built_tap_instances_is_pinned():
    assert binding.conv_variant_count(binding.CONV_KERNEL_TAP) == 31
    assert built_tap_instances() == BUILT_TAP_INSTANCES
    # sizes outside the table have no tap kernel at all
    for R, S in [(2, 3), (6, 6), (3, 5), (9, 9), (1, 2), (11, 11)]:
        with pytest.raises(binding.ConvError):
            binding.conv_fwd_plan_request(2, 8, 16, 16, 16, R, S, 0, 0, binding.CONV_KERNEL_TAP, 2, 16)


def test_direct_loaders_keep_their_byte_offsets_inside_32_bits():
    """The direct loaders address a tile's cells as a scalar base plus a 32-bit byte offset per slot: a layer whose images
    (x) or whose channel tile of filters (w) span 4 GiB or more must not get them (host-only; nothing is launched)."""
    tap, direct = binding.CONV_KERNEL_TAP, binding.CONV_LOADER_DIRECT
    big_images = (2, 1 << 17, 80, 80, 16, 3, 3, 1, 1)          # one image: 2^17 * 6400 * 4 B = 3.1 GiB, and a tile may touch two
    plan = binding.conv_fwd_plan(*big_images)
    assert plan.loader in (0, binding.CONV_LOADER_REGISTERS), plan.as_dict()
    for v in range(binding.conv_variant_count(tap)):
        for loader in (direct, binding.CONV_LOADER_DIRECT_WAVES, binding.CONV_LOADER_DIRECT_DEEP):
            with pytest.raises(binding.ConvError):
                binding.conv_fwd_plan_request(*big_images, tap, v, 0, loader=loader)
    big_filters = (1, 1 << 21, 4, 4, 64, 3, 3, 1, 1)            # 64 output channels of 2^21 * 9 floats: 4.5 GiB per channel tile
    with pytest.raises(binding.ConvError):
        binding.conv_fwd_plan_request(*big_filters, tap, 7, 16, loader=direct)       # 64-channel tile
    narrow, _ = binding.conv_fwd_plan_request(*big_filters, tap, 2, 16, loader=direct)   # 16-channel tile: 1.1 GiB
    assert narrow.loader == direct
    plan = binding.conv_fwd_plan(*big_filters)
    assert plan.loader == binding.CONV_LOADER_REGISTERS or plan.tile_k * (1 << 21) * 9 * 4 < (1 << 32) - 64, plan.as_dict()
    small = binding.conv_fwd_plan(2, 1 << 10, 80, 80, 16, 3, 3, 1, 1)
    assert small.kernel == tap and small.loader != binding.CONV_LOADER_REGISTERS


def test_wide_maps_stay_in_the_tap_family():
    """Halo tiles hold whole padded rows: up to ~580 pixels every layer finds a tile shape whose staging slots take them, and
    beyond that the wide shape (twice the slots of the 16 x 448 one, the whole LDS) does: up to ~1500 pixels for 3x3 filters
    on rows of dwordx4 (pixel tiles that divide a row keep the halo tile at three rows), about half of that on rows of single dwords or with 5x5 filters."""
    tap = binding.CONV_KERNEL_TAP
    for W in (224, 512, 580):
        assert binding.conv_fwd_plan(1, 16, 32, W, 16, 3, 3, 1, 1).kernel == tap
    for dims in ((1, 16, 32, 1000, 16, 3, 3, 1, 1), (2, 32, 128, 1200, 64, 3, 3, 1, 1), (1, 16, 32, 1400, 16, 3, 3, 1, 1), (1, 16, 32, 701, 16, 3, 3, 1, 1), (1, 8, 32, 800, 32, 5, 5, 2, 2)):
        p = binding.conv_fwd_plan(*dims)
        assert p.kernel == tap and p.variant == 30 and p.lds_bytes <= 160 * 1024, (dims, p.as_dict())
    assert binding.conv_fwd_plan(1, 16, 32, 4000, 16, 3, 3, 1, 1).kernel == binding.CONV_KERNEL_GENERIC


def test_halo_tiles_that_cannot_fit_lds_never_reach_the_tap_kernel():
    """Padded rows of millions of floats: every size of the halo tile is computed in 64 bits, and what cannot fit LDS goes
    to the generic kernel instead of a tap launch with wrapped-around sizes (host-only; nothing is launched)."""
    import time
    tap = binding.CONV_KERNEL_TAP
    for dims in [(1, 64, 3, 7, 16, 3, 3, 0, 5600000), (1, 4, 3, 7, 1, 3, 3, 0, 400000000), (1, 8, 5, 5, 8, 3, 3, 0, 30000),
                 (1, 16, 3, 40000, 16, 3, 3, 1, 1), (1, 5, 1, 46000, 3, 1, 1, 0, 0)]:
        t0 = time.perf_counter()
        p = binding.conv_fwd_plan(*dims)
        assert time.perf_counter() - t0 < 2.0, dims            # the search gives up early instead of walking every phase
        assert p.kernel == binding.CONV_KERNEL_GENERIC, (dims, p.as_dict())
        for v in (2, 17, 10):
            with pytest.raises(binding.ConvError):
                binding.conv_fwd_plan_request(*dims, tap, v, 0)
    # every tap plan of the grid holds its whole double-buffered halo tile inside the LDS it asks for
    for s in inputs.sweep_shapes():
        p = binding.conv_fwd_plan(*s.dims)
        if p.kernel == tap:
            assert p.lds_bytes >= 2 * 4 * p.chunk_c * p.lds_plane
            assert p.lds_plane >= p.lds_rows * p.lds_pitch - 16 and p.lds_pitch >= s.W + 2 * s.pad_w


def test_the_benchmark_layers_go_through_the_planner_like_any_other_shape():
    """No table of measured mappings: the five benchmark layers get what the cost model and the rules pick, and what they
    pick is the model's own minimum over every tile shape and candidate pixel tile (tap family)."""
    tap = binding.CONV_KERNEL_TAP
    picks = {}
    for i in range(1, 6):
        dims = inputs.config(i).dims
        p = binding.conv_fwd_plan(*dims)
        picks[i] = (p.kernel, p.variant, p.tile_pix, p.loader)
        if p.kernel != tap:
            continue
        _, cost = binding.conv_fwd_plan_request(*dims, tap, p.variant, p.tile_pix, loader=p.loader)
        for v in range(binding.conv_variant_count(tap)):
            cap = binding.conv_variant_info(tap, v)[1]
            for tile in {cap, cap // 2, p.tile_pix}:
                try:
                    q, c = binding.conv_fwd_plan_request(*dims, tap, v, tile)
                except binding.ConvError:
                    continue
                # (the rules may replace the model's pick by its deep-ring build, and keep sixteen-share shapes off thin layers)
                assert c >= cost * 0.999 or q.loader != p.loader or v in (17, 18), (i, v, tile, c, cost)
    assert picks[3] == (tap, 27, 98, binding.CONV_LOADER_DIRECT)            # 98-pixel tiles with a tail on all 256 CUs
    assert picks[5] == (tap, 26, 196, binding.CONV_LOADER_DIRECT_WAVES)     # one 14 x 14 image per tile, twelve tiles and a tail
    assert picks[2][0] == binding.CONV_KERNEL_POINTWISE
