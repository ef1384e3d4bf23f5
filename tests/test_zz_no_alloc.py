"""The allocation-free entry point (conv_fwd_split_c_static) against conv_fwd_split_c, through the C-ABI.

The two run the same kernels with the same mapping, once on the library's static scratch array and once on a caller's
workspace, so their outputs must agree bit for bit; both are also held to the oracle's tolerance. The second call uses
a smaller layer, so stale partial sums of the first call sit in the array beyond what the second one writes.
"""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2103_16234_amd import binding, inputs

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _layer(name, dims, seed):
    return inputs.ConvShape(name, *dims, "u01", "he", 700 + seed, 800 + seed)


def _both(shape, variant, c_splits, tile_pix=0, bias=False, relu=False):
    x, w = inputs.make_inputs(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    bd = torch.from_numpy(inputs.uniform_pm1(55, shape.K)).cuda() if bias else None
    y_ws = torch.full(shape.y_shape, float("nan"), device="cuda")
    y_st = torch.full(shape.y_shape, float("nan"), device="cuda")
    print(f"[case] {shape.name} dims={shape.dims} variant={variant} c_splits={c_splits} tile_pix={tile_pix}", flush=True)
    _, p_ws = binding.conv_fwd_split_c(xd, wd, shape.pad_h, shape.pad_w, bias=bd, relu=relu, c_splits=c_splits, variant=variant,
                                       tile_pix=tile_pix, y=y_ws)
    _, p_st = binding.conv_fwd_split_c_static(xd, wd, shape.pad_h, shape.pad_w, y_st, bias=bd, relu=relu, c_splits=c_splits,
                                              variant=variant, tile_pix=tile_pix)
    torch.cuda.synchronize()
    assert p_st.as_dict() == p_ws.as_dict()
    a, b = y_ws.cpu().numpy(), y_st.cpu().numpy()
    assert not np.isnan(b).any(), "some outputs were never written"
    np.testing.assert_array_equal(a, b)                      # same kernels, same mapping: bit for bit
    y_ref, ya_ref = oracle.conv_bias_relu_ref(x, w, bd.cpu().numpy() if bias else None, shape.pad_h, shape.pad_w, relu)
    ok, worst = oracle.within_tolerance(b.astype(np.float64), y_ref, ya_ref)
    assert ok, f"worst tolerance ratio {worst:.3g} with plan {p_st.as_dict()}"
    return p_st


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row():
    big = _layer("noalloc_3x3_c256_14", (2, 256, 14, 14, 96, 3, 3, 1, 1), 1)
    small = _layer("noalloc_3x3_c64_7", (1, 64, 7, 7, 40, 3, 3, 1, 1), 2)
    p1 = _both(big, variant=5, c_splits=8)
    assert p1.c_splits == 8 and p1.workspace_bytes == 4 * 8 * 2 * 96 * 196
    p2 = _both(small, variant=13, c_splits=4, bias=True, relu=True)       # smaller: the array still holds the first call's sums
    assert p2.c_splits == 4 and p2.workspace_bytes < p1.workspace_bytes
    p3 = _both(big, variant=5, c_splits=8)                                # and back again
    assert p3.as_dict() == p1.as_dict()


def test_static_scratch_default_plan_and_no_shares():
    deep = _layer("noalloc_3x3_c512_7", (1, 512, 7, 7, 512, 3, 3, 1, 1), 3)    # the splitting planner's own choice
    p = _both(deep, variant=None, c_splits=0)
    assert p.c_splits > 1
    plain = _layer("noalloc_3x3_c16_12", (2, 16, 12, 12, 24, 3, 3, 1, 1), 4)  # one share: the array is not touched
    p = _both(plain, variant=2, c_splits=1)
    assert p.c_splits == 1 and p.workspace_bytes == 0


def test_static_scratch_refuses_what_does_not_fit():
    """A mapping whose partial outputs exceed the array is refused with CONV_E_WORKSPACE before anything is launched;
    argument errors are the ones of conv_fwd_split_c."""
    lib = binding.load_library()
    shape = _layer("noalloc_too_big", (8, 128, 28, 28, 128, 3, 3, 1, 1), 5)   # 8 shares x 3.2 MB of partial outputs
    x, w = inputs.make_inputs(shape)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    yd = torch.zeros(shape.y_shape, device="cuda")
    req, res = binding.ConvPlan(), binding.ConvPlan()
    req.kernel, req.variant, req.c_splits = binding.CONV_KERNEL_TAP, 7, 8
    need, _ = binding.conv_fwd_plan_request(*shape.dims, binding.CONV_KERNEL_TAP, 7, 0, c_splits=8)
    assert need.workspace_bytes > binding.STATIC_SCRATCH_BYTES
    rc = lib.conv_fwd_split_c_static(xd.data_ptr(), wd.data_ptr(), None, yd.data_ptr(), *shape.dims, 0, ctypes.byref(req),
                                     ctypes.byref(res))
    assert rc == -7
    torch.cuda.synchronize()
    assert float(yd.abs().max()) == 0.0                                      # nothing ran
    assert lib.conv_fwd_split_c_static(None, None, None, None, *shape.dims, 0, None, None) == -1
    assert lib.conv_fwd_split_c_static(xd.data_ptr(), wd.data_ptr(), None, yd.data_ptr(), 8, 128, 28, 28, 128, 3, 3, -1, 1, 0,
                                       None, None) == -2
