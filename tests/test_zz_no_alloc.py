"""The entry point that allocates nothing (conv2d_forward_static_scratch) against the entry
point it is a variant of (conv2d_forward_variant with the same variant and a caller's
workspace): same kernels, so the outputs must be bit-identical.  Two calls in a row share the
library's static scratch array; the second is a smaller layer."""
import numpy as np
import pytest
import torch

from paper_1904_04174_amd import binding as B
from paper_1904_04174_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _case(shape_in, shape_f, stride, padding, dtype, seed):
    x, f = wl.make_case(shape_in, shape_f, "uniform", seed)
    n, h, w, c = shape_in
    r, s, _, k = shape_f
    in_dt = B.F32 if dtype == "f32" else B.BF16
    p = B.make_params(n, h, w, c, k, r, s, stride, stride, padding, in_dt, B.F32)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    xd = torch.from_numpy(x).cuda().to(tdt).contiguous()
    fd = torch.from_numpy(f).cuda().to(tdt).contiguous()
    g = B.conv2d_get_geometry(p)
    return p, xd, fd, (n, g.out_rows, g.out_cols, k)


def _scratch_variant(p):
    """A variant that uses scratch memory for `p` (repacked filter and, by preference, the
    partial sums of a split reduction), within the static array's size."""
    fits = []
    for v in range(B.conv2d_num_variants()):
        name = B.conv2d_variant_name(v)
        if name.startswith("winograd") or not B.conv2d_variant_supports(p, v):
            continue
        if 0 < B.conv2d_workspace_size(p, v) <= B.STATIC_SCRATCH_BYTES:
            fits.append((0 if name.endswith("_splitk") else 1, v))
    assert fits, "no variant of this case uses scratch memory"
    return min(fits)[1]


def _reference(p, xd, fd, out_shape, vid):
    need = B.conv2d_workspace_size(p, vid)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    out = torch.full(out_shape, float("nan"), dtype=torch.float32, device="cuda")
    rc = B.conv2d_forward_raw(p, xd.data_ptr(), fd.data_ptr(), out.data_ptr(),
                              ws.data_ptr() if need else 0, need,
                              torch.cuda.current_stream().cuda_stream, vid)
    assert rc == 0, B.status_string(rc)
    return out, need


# (first call, second and smaller call), each run twice: with the selector's own pick, and with
# a variant forced that keeps a repacked filter and the partial sums of a split reduction in
# the scratch array
CASES = [
    ("f32", ((2, 14, 14, 256), (3, 3, 256, 256), 1, wl.PAD_SAME),
            ((1, 9, 11, 32), (3, 3, 32, 48), 1, wl.PAD_SAME)),
    ("bf16", ((4, 28, 28, 128), (3, 3, 128, 128), 1, wl.PAD_SAME),
             ((2, 10, 10, 64), (1, 1, 64, 40), 2, wl.PAD_VALID)),
    ("f32", ((4, 56, 56, 64), (3, 3, 64, 64), 1, wl.PAD_SAME),
            ((1, 8, 8, 4), (3, 3, 4, 4), 1, wl.PAD_SAME)),
]


@pytest.mark.parametrize("forced", [False, True])
@pytest.mark.parametrize("dtype,first,second", CASES)
def test_static_scratch_matches_workspace_entry_point(dtype, first, second, forced):
    stream = torch.cuda.current_stream().cuda_stream
    prepared = []
    for i, (shape_in, shape_f, stride, padding) in enumerate((first, second)):
        p, xd, fd, out_shape = _case(shape_in, shape_f, stride, padding, dtype, 4242 + i)
        vid = (_scratch_variant(p) if forced
               else B.conv2d_select_variant(p, B.SELECT_DIRECT_SUM_ONLY))
        want, need = _reference(p, xd, fd, out_shape, vid)
        assert need <= B.STATIC_SCRATCH_BYTES
        assert need > 0 or not forced
        prepared.append((p, xd, fd, want, vid))
    torch.cuda.synchronize()
    # the two calls in a row, outputs allocated beforehand: nothing is allocated in between
    outs = [torch.full(tuple(w.shape), float("nan"), dtype=torch.float32, device="cuda")
            for _, _, _, w, _ in prepared]
    torch.cuda.synchronize()
    try:
        for (p, xd, fd, _, vid), out in zip(prepared, outs):
            if forced:
                B.conv2d_debug_force_variant(vid)
            rc = B.conv2d_forward_static_scratch_raw(p, xd.data_ptr(), fd.data_ptr(),
                                                     out.data_ptr(), stream)
            assert rc == 0, B.status_string(rc)
    finally:
        B.conv2d_debug_force_variant(None)
    torch.cuda.synchronize()
    for (_, _, _, want, _), out in zip(prepared, outs):
        got, ref = out.cpu().numpy(), want.cpu().numpy()
        assert not np.isnan(got).any()
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_static_scratch_rejects_what_does_not_fit():
    # 3x3x1024x1024 in fp32: the repacked filter of a direct-to-LDS tile alone is 36 MiB
    p = B.make_params(1, 8, 8, 1024, 1024, 3, 3, 1, 1, B.PAD_SAME, B.F32, B.F32)
    big = [v for v in range(B.conv2d_num_variants())
           if B.conv2d_variant_supports(p, v)
           and B.conv2d_variant_name(v).startswith("igemm_dma_")
           and B.conv2d_workspace_size(p, v) > B.STATIC_SCRATCH_BYTES]
    assert big
    x = torch.zeros((1, 8, 8, 1024), device="cuda")
    f = torch.zeros((3, 3, 1024, 1024), device="cuda")
    out = torch.full((1, 8, 8, 1024), 7.0, device="cuda")
    B.conv2d_debug_force_variant(big[0])
    try:
        rc = B.conv2d_forward_static_scratch_raw(p, x.data_ptr(), f.data_ptr(), out.data_ptr(), 0)
    finally:
        B.conv2d_debug_force_variant(None)
    torch.cuda.synchronize()
    assert rc == B.STATUS_SCRATCH_EXCEEDED
    assert "scratch" in B.status_string(rc)
    assert bool((out == 7.0).all()), "a rejected call must launch nothing"
