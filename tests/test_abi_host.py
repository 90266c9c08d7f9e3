"""Host-side checks of the C ABI (no GPU): the library loads, exports every
declared symbol, derives the same geometry as the oracle, reports errors, and
its selector only picks variants that support the parameters."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1904_04174_amd import binding as B
from paper_1904_04174_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "conv2d.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conv2d_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 11
    assert set(names) == set(B.EXPORTS)
    raw = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(raw, n) is not None


def test_version_and_status_strings():
    assert B.conv2d_version() >= 100
    assert B.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -6):
        assert B.status_string(code) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


def test_variant_table():
    n = B.conv2d_num_variants()
    assert n >= 2
    names = [B.conv2d_variant_name(i) for i in range(n)]
    assert names[0] == "direct"
    assert len(set(names)) == n
    assert B.conv2d_variant_name(n) is None and B.conv2d_variant_name(-1) is None


def test_geometry_matches_oracle(oracle):
    rng = np.random.default_rng(5)
    checked = 0
    for _ in range(400):
        h, w = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        r, s = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        sr, sc = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        pad = int(rng.integers(0, 2))
        p = B.make_params(2, h, w, 3, 5, r, s, sr, sc, pad)
        try:
            want = oracle.geometry(h, w, r, s, sr, sc, pad)
        except ValueError:
            with pytest.raises(B.Conv2dError) as ei:
                B.conv2d_get_geometry(p)
            assert ei.value.status == B.STATUS_INVALID_ARGUMENT
            continue
        g = B.conv2d_get_geometry(p)
        assert (g.out_rows, g.out_cols, g.pad_top, g.pad_bottom, g.pad_left, g.pad_right) == want
        checked += 1
    assert checked > 200


def test_geometry_of_named_layers():
    want = {"R7x7": (112, 2, 3), "L-s2": (28, 0, 1), "R1x1s2": (14, 0, 0), "L-valid": (54, 0, 0),
            "V224-N16": (224, 1, 1), "L-s2valid": (27, 0, 0)}
    for name, (o, a, b) in want.items():
        g = B.conv2d_get_geometry(B.params_of_layer(wl.LAYERS[name]))
        assert (g.out_rows, g.pad_top, g.pad_bottom) == (o, a, b)
        assert (g.out_cols, g.pad_left, g.pad_right) == (o, a, b)


BAD = [
    dict(batch=-1), dict(in_rows=0), dict(in_cols=-3), dict(channels=0), dict(features=0),
    dict(window_rows=0), dict(window_cols=0), dict(stride_rows=0), dict(stride_cols=-1),
    dict(padding=2), dict(in_dtype=5), dict(out_dtype=-1),
    dict(padding=B.PAD_VALID, in_rows=2, window_rows=3),
]


@pytest.mark.parametrize("bad", BAD)
def test_invalid_parameters_are_rejected_before_any_launch(bad):
    kw = dict(batch=1, in_rows=8, in_cols=8, channels=4, features=4, window_rows=3, window_cols=3,
              stride_rows=1, stride_cols=1, padding=B.PAD_SAME, in_dtype=B.F32, out_dtype=B.F32)
    kw.update(bad)
    p = B.make_params(**kw)
    # non-null dummy pointers: validation must fail before they are touched
    rc = B.conv2d_forward_raw(p, 16, 16, 16)
    assert rc == B.STATUS_INVALID_ARGUMENT
    rc = B.conv2d_forward_raw(p, 16, 16, 16, variant_id=0)
    assert rc == B.STATUS_INVALID_ARGUMENT
    with pytest.raises(B.Conv2dError):
        B.conv2d_workspace_size(p)


def test_null_pointers_and_bad_variant_ids():
    p = B.make_params(1, 8, 8, 4, 4, 3, 3)
    assert B.conv2d_forward_raw(p, 0, 16, 16) == B.STATUS_INVALID_ARGUMENT
    assert B.conv2d_forward_raw(p, 16, 0, 16) == B.STATUS_INVALID_ARGUMENT
    assert B.conv2d_forward_raw(p, 16, 16, 0) == B.STATUS_INVALID_ARGUMENT
    assert B.conv2d_forward_raw(p, 16, 16, 16, variant_id=10 ** 6) == B.STATUS_INVALID_ARGUMENT
    assert B.conv2d_forward_raw(p, 16, 16, 16, variant_id=-1) == B.STATUS_INVALID_ARGUMENT
    assert B.lib().conv2d_get_geometry(None, None) == B.STATUS_INVALID_ARGUMENT
    assert B.lib().conv2d_workspace_size(ctypes.byref(p), None) == B.STATUS_INVALID_ARGUMENT


def test_empty_batch_is_a_noop_without_pointers():
    p = B.make_params(0, 8, 8, 4, 4, 3, 3)
    assert B.conv2d_forward_raw(p, 0, 0, 0) == B.STATUS_OK


def test_f32_in_bf16_out_is_unsupported():
    p = B.make_params(1, 8, 8, 8, 8, 3, 3, in_dtype=B.F32, out_dtype=B.BF16)
    assert B.conv2d_forward_raw(p, 16, 16, 16) == B.STATUS_UNSUPPORTED


def test_too_large_is_reported():
    p = B.make_params(4096, 1024, 1024, 64, 64, 3, 3)
    assert B.conv2d_forward_raw(p, 16, 16, 16) == B.STATUS_TOO_LARGE


def test_forced_variant_that_cannot_run_is_unsupported():
    # C = 3 cannot use the 16-byte gathers of the implicit-GEMM variants
    p = B.make_params(1, 8, 8, 3, 8, 3, 3)
    n = B.conv2d_num_variants()
    unsupported = [i for i in range(n) if not B.conv2d_variant_supports(p, i)]
    assert unsupported, "expected at least one variant to refuse C=3"
    for i in unsupported:
        assert B.conv2d_forward_raw(p, 16, 16, 16, variant_id=i) == B.STATUS_UNSUPPORTED
    assert B.conv2d_variant_supports(p, 0)
    # a misaligned pointer also makes a vectorised variant refuse
    p = B.make_params(1, 8, 8, 8, 8, 3, 3)
    vec = [i for i in range(1, n) if B.conv2d_variant_supports(p, i)]
    assert vec
    assert B.conv2d_forward_raw(p, 4, 16, 16, variant_id=vec[0]) == B.STATUS_UNSUPPORTED


def test_selector_only_picks_supported_variants():
    rng = np.random.default_rng(9)
    layers = list(wl.LAYERS.values())
    for i in range(300):
        if i < len(layers):
            L = layers[i]
            shapes = [B.params_of_layer(L, dt, B.F32) for dt in (B.F32, B.BF16)]
        else:
            shapes = [B.make_params(int(rng.integers(1, 5)), int(rng.integers(1, 30)),
                                    int(rng.integers(1, 30)), int(rng.integers(1, 70)),
                                    int(rng.integers(1, 70)), int(rng.integers(1, 4)),
                                    int(rng.integers(1, 4)), int(rng.integers(1, 3)),
                                    int(rng.integers(1, 3)), B.PAD_SAME,
                                    int(rng.integers(0, 2)), B.F32)]
        for p in shapes:
            v = B.conv2d_selected_variant(p)
            assert 0 <= v < B.conv2d_num_variants()
            assert B.conv2d_variant_supports(p, v)
            assert B.conv2d_workspace_size(p) >= 0


def test_compute_bound_layers_use_the_matrix_cores():
    for name in wl.VGG_N16 + ["L-same", "L-valid", "L-s2", "R3x3"]:
        p = B.params_of_layer(wl.LAYERS[name])
        v = B.conv2d_selected_variant(p)
        assert B.conv2d_variant_name(v).startswith(("igemm_", "winograd2x2_")), name
        v = B.conv2d_select_variant(p, B.SELECT_DIRECT_SUM_ONLY)
        assert B.conv2d_variant_name(v).startswith("igemm_"), name


def test_empty_batch_has_a_selection_and_no_workspace():
    for dt in (B.F32, B.BF16):
        p = B.make_params(0, 14, 14, 512, 512, 3, 3, 1, 1, B.PAD_SAME, dt, B.F32)
        assert B.conv2d_selected_variant(p) == 0
        assert B.conv2d_workspace_size(p) == 0
        for v in range(B.conv2d_num_variants()):
            if B.conv2d_variant_supports(p, v):
                assert B.conv2d_workspace_size(p, v) >= 0


def test_split_reduction_variants_state_their_workspace():
    p = B.params_of_layer(wl.LAYERS["V14-N1"])
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    split = [v for v, n in enumerate(names) if n.endswith("_splitk") and B.conv2d_variant_supports(p, v)]
    assert split
    for v in split:
        ws = B.conv2d_workspace_size(p, v)
        # at least two fp32 partial outputs; the register-staged tiles need nothing else
        assert ws >= 2 * 4 * 196 * 512
        if names[v].startswith(("igemm_f32_", "igemm_bf16_")):
            assert ws % (4 * 196 * 512) == 0
    # one slice of reduction cannot be split
    p1 = B.make_params(1, 8, 8, 4, 8, 1, 1)
    for v, n in enumerate(names):
        if n.endswith("_splitk"):
            assert not B.conv2d_variant_supports(p1, v)


def test_patch_tiles_split_their_channel_blocks():
    """A patch tile's split reduction runs over its channel blocks: at most one split per four
    blocks, the partial sums behind the repacked filter (none for a filter read as it lies);
    tiles that walk several tiles per workgroup, and shapes with a single block, do not split."""
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    p = B.params_of_layer(wl.LAYERS["V14-N16"], B.BF16, B.F32)       # C = 512: 16 blocks of 32
    plane = 4 * 16 * 14 * 14 * 512
    nat = names.index("igemm_patch_bf16_224x128_w2x2_p384_m16_nat_splitk")
    assert B.conv2d_variant_supports(p, nat)
    assert B.conv2d_workspace_size(p, nat) == 4 * plane
    packed = names.index("igemm_patch_bf16_224x128_w2x2_p384_m16_splitk")
    assert B.conv2d_workspace_size(p, packed) == 4 * plane + 2 * 9 * 512 * 512
    assert not B.conv2d_variant_supports(
        p, names.index("igemm_patch_bf16_128x64_w2x2_p256_b16_nat_splitk"))
    one_block = B.make_params(2, 14, 14, 32, 64, 3, 3, 1, 1, wl.PAD_SAME, B.BF16, B.F32)
    assert B.conv2d_variant_supports(
        one_block, names.index("igemm_patch_bf16_224x128_w2x2_p384_m16_nat"))
    assert not B.conv2d_variant_supports(one_block, nat)


def test_workspace_is_checked_before_any_launch():
    # a variant that needs scratch: too little of it, or a misaligned pointer, is an error status
    p = B.params_of_layer(wl.LAYERS["V14-N1"])
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    v = next(i for i, n in enumerate(names)
             if n.startswith("igemm_dma_f32") and B.conv2d_variant_supports(p, i))
    need = B.conv2d_workspace_size(p, v)
    assert need > 0
    assert B.conv2d_forward_raw(p, 256, 512, 768, 0, 0, variant_id=v) == B.STATUS_WORKSPACE_TOO_SMALL
    assert B.conv2d_forward_raw(p, 256, 512, 768, 1024, need - 1,
                                variant_id=v) == B.STATUS_WORKSPACE_TOO_SMALL
    assert B.conv2d_forward_raw(p, 256, 512, 768, 1028, need,
                                variant_id=v) == B.STATUS_INVALID_ARGUMENT


def test_tuned_table_names_existing_variants():
    # every named layer has a tuned choice; it must resolve to a variant that supports the layer
    names = {B.conv2d_variant_name(v): v for v in range(B.conv2d_num_variants())}
    import os
    table = os.path.join(os.path.dirname(B.__file__), "csrc", "tuned_table.inc")
    rows = [l for l in open(table) if l.startswith("{")]
    assert len(rows) >= len(wl.LAYERS)
    seen = {}
    for l in rows:
        fields = l[1:l.index("}")].split(",")
        name = fields[-1].strip().strip('"')
        bf16, n, h, w, c, k, r, s_, sr, sc, pad = (int(f) for f in fields[:-1])
        p = B.make_params(n, h, w, c, k, r, s_, sr, sc, pad, B.BF16 if bf16 else B.F32, B.F32)
        assert name in names, name
        assert B.conv2d_variant_supports(p, names[name]), l
        # a shape has at most two rows, the transform (Winograd) variant first: that one is the
        # unrestricted choice, the other the choice among the direct-sum variants
        key = tuple(fields[:-1])
        seen.setdefault(key, []).append(name)
        if name.startswith("winograd"):
            assert len(seen[key]) == 1, l
            assert B.conv2d_selected_variant(p) == names[name], l
        else:
            assert len(seen[key]) <= 2, l
            assert B.conv2d_select_variant(p, B.SELECT_DIRECT_SUM_ONLY) == names[name], l
            if len(seen[key]) == 1:
                assert B.conv2d_selected_variant(p) == names[name], l


def test_select_variant_flags():
    p = B.make_params(16, 56, 56, 256, 256, 3, 3)
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    assert any(n.startswith("winograd2x2_") for n in names)
    assert B.conv2d_select_variant(p, 0) == B.conv2d_selected_variant(p)
    assert not names[B.conv2d_select_variant(p, B.SELECT_DIRECT_SUM_ONLY)].startswith("winograd")
    with pytest.raises(B.Conv2dError):
        B.conv2d_select_variant(p, 2)
    # Winograd runs fp32 3x3 stride-1 layers with C and K multiples of 4 only
    wino = [i for i, n in enumerate(names) if n.startswith("winograd2x2_") and n.endswith("_g")]
    assert B.conv2d_variant_supports(p, wino[0])
    for bad in (B.make_params(16, 56, 56, 256, 256, 3, 3, 2, 2),
                B.make_params(16, 56, 56, 256, 256, 5, 5),
                B.make_params(16, 56, 56, 254, 256, 3, 3),
                B.make_params(16, 56, 56, 256, 256, 3, 3, in_dtype=B.BF16)):
        assert not B.conv2d_variant_supports(bad, wino[0])
    # its workspace holds the transformed filter, input and products
    tiles = 16 * 28 * 28
    assert B.conv2d_workspace_size(p, wino[0]) >= 4 * 16 * (256 * 256 + 2 * tiles * 256)


def test_variant_names_are_unique():
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    assert len(set(names)) == len(names)
    assert B.conv2d_variant_name(-1) is None and B.conv2d_variant_name(len(names)) is None


def test_bias_act_arguments_are_validated_before_any_launch():
    p = B.make_params(1, 8, 8, 4, 4, 3, 3)
    l = B.lib()
    call = lambda bias, act, x=16: l.conv2d_forward_bias_act(ctypes.byref(p), x, 16, bias, act, 16,
                                                             0, 0, 0)
    assert call(0, 2) == B.STATUS_INVALID_ARGUMENT       # unknown activation
    assert call(0, -1) == B.STATUS_INVALID_ARGUMENT
    assert call(18, B.ACT_RELU) == B.STATUS_INVALID_ARGUMENT   # bias not 4-byte aligned
    assert call(16, B.ACT_RELU, x=0) == B.STATUS_INVALID_ARGUMENT  # null input
    empty = B.make_params(0, 8, 8, 4, 4, 3, 3)
    assert l.conv2d_forward_bias_act(ctypes.byref(empty), 0, 0, 0, B.ACT_RELU, 0, 0, 0, 0) == 0


def test_pool_arguments_and_workspace_sizes_on_the_host():
    p = B.make_params(1, 8, 8, 4, 4, 3, 3)
    l = B.lib()
    call = lambda bias, act, x=16: l.conv2d_forward_bias_act_pool(ctypes.byref(p), x, 16, bias, act,
                                                                  16, 0, 0, 0)
    assert call(0, 2) == B.STATUS_INVALID_ARGUMENT       # unknown activation
    assert call(18, B.ACT_RELU) == B.STATUS_INVALID_ARGUMENT   # bias not 4-byte aligned
    assert call(16, B.ACT_RELU, x=0) == B.STATUS_INVALID_ARGUMENT  # null input
    empty = B.make_params(0, 8, 8, 4, 4, 3, 3)
    assert l.conv2d_forward_bias_act_pool(ctypes.byref(empty), 0, 0, 0, B.ACT_RELU, 0, 0, 0, 0) == 0
    # an output of one row has no 2x2 window: nothing to do, no workspace asked for
    thin = B.make_params(2, 1, 9, 4, 4, 1, 1)
    assert l.conv2d_forward_bias_act_pool(ctypes.byref(thin), 16, 16, 0, B.ACT_NONE, 16, 0, 0, 0) == 0
    # (the empty output tensor may well have a null pointer)
    assert l.conv2d_forward_bias_act_pool(ctypes.byref(thin), 16, 16, 0, B.ACT_NONE, 0, 0, 0, 0) == 0
    # a variant that pools in its epilogue needs its own workspace only; any other also the
    # unpooled tensor behind it
    big = B.make_params(16, 224, 224, 64, 64, 3, 3, in_dtype=B.BF16, out_dtype=B.BF16)
    unpooled = 16 * 224 * 224 * 64 * 2
    for v in range(B.conv2d_num_variants()):
        if not B.conv2d_variant_supports(big, v):
            continue
        own = B.conv2d_workspace_size(big, v)
        pooled = B.conv2d_pool_workspace_size(big, v)
        name = B.conv2d_variant_name(v)
        if name.startswith("igemm_patch_") and name.endswith(("_b16", "_b16_nat")):
            assert pooled == own, name
        else:
            assert pooled == (own + 255) // 256 * 256 + unpooled, name
    sel = B.conv2d_selected_variant(big)
    assert B.conv2d_pool_workspace_size(big) == B.conv2d_pool_workspace_size(big, sel)
    # where conv2d_forward's pick cannot pool (a 16-row tile here), the pooled entry point takes a
    # variant that can, if the model prices it below that pick plus the second kernel: no room
    # for the unpooled tensor is asked for
    mid = B.make_params(16, 112, 112, 128, 128, 3, 3, in_dtype=B.BF16, out_dtype=B.F32)
    assert "_m16" in B.conv2d_variant_name(B.conv2d_selected_variant(mid))
    assert B.conv2d_pool_workspace_size(mid) < 16 * 112 * 112 * 128 * 4
    with pytest.raises(B.Conv2dError):
        B.conv2d_pool_workspace_size(big, B.conv2d_num_variants())


def test_packed_filter_sizes_and_argument_checks():
    p = B.make_params(2, 14, 14, 40, 24, 3, 3)       # Kg = 360: no multiple of a 16-wide slice
    l = B.lib()
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    seen = set()
    for v, name in enumerate(names):
        if not B.conv2d_variant_supports(p, v):
            continue
        n = ctypes.c_size_t(0)
        rc = l.conv2d_packed_filter_size(ctypes.byref(p), v, ctypes.byref(n))
        assert rc == 0, name
        if name.startswith("igemm_dma_f32_") and "_r64_" in name:
            # slices of 16 fp32 values: 360 -> 368 rows of 24 features
            assert n.value == (368 * 24 * 4 + 255) // 256 * 256, name
            seen.add("dma")
        elif name == "direct" or name.startswith("igemm_f32_"):
            assert n.value == (360 * 24 * 4 + 255) // 256 * 256, name
            seen.add("copy")
        # a buffer that is too small, null pointers: rejected before any device call
        assert l.conv2d_pack_filter(ctypes.byref(p), v, 16, 16, n.value - 1, 0) == \
            B.STATUS_WORKSPACE_TOO_SMALL
        assert l.conv2d_pack_filter(ctypes.byref(p), v, 0, 16, n.value, 0) == B.STATUS_INVALID_ARGUMENT
        assert l.conv2d_pack_filter(ctypes.byref(p), v, 16, 0, n.value, 0) == B.STATUS_INVALID_ARGUMENT
    assert seen == {"dma", "copy"}
    n = ctypes.c_size_t(0)
    assert l.conv2d_packed_filter_size(ctypes.byref(p), -1, ctypes.byref(n)) == B.STATUS_INVALID_ARGUMENT
    assert l.conv2d_packed_filter_size(ctypes.byref(p), len(names), ctypes.byref(n)) == \
        B.STATUS_INVALID_ARGUMENT
    assert l.conv2d_packed_filter_size(ctypes.byref(p), 0, None) == B.STATUS_INVALID_ARGUMENT
    assert l.conv2d_forward_packed(ctypes.byref(p), -1, 16, 16, 0, 0, 16, 0, 0, 0) == \
        B.STATUS_INVALID_ARGUMENT
    assert l.conv2d_forward_packed(ctypes.byref(p), 0, 16, 16, 0, 7, 16, 0, 0, 0) == \
        B.STATUS_INVALID_ARGUMENT   # unknown activation


def test_window_row_gather_kernel_support_rules():
    """The kernel for very few channels: fp32 only, at most 4 channels, a patch of at most 3072
    values and LDS within 64 KiB; no workspace; chosen for the 7x7 stride-2 layer on a 3-channel
    image at batch 32."""
    names = [B.conv2d_variant_name(v) for v in range(B.conv2d_num_variants())]
    vid = names.index("rowgather_f32_128x64")
    stem = B.make_params(32, 224, 224, 3, 64, 7, 7, 2, 2, wl.PAD_SAME, B.F32, B.F32)
    assert B.conv2d_variant_supports(stem, vid)
    assert B.conv2d_workspace_size(stem, vid) == 0
    assert B.conv2d_variant_name(B.conv2d_selected_variant(stem)) == "rowgather_f32_128x64"
    for bad in (B.make_params(32, 224, 224, 3, 64, 7, 7, 2, 2, wl.PAD_SAME, B.BF16, B.F32),
                B.make_params(4, 56, 56, 8, 64, 3, 3, 1, 1, wl.PAD_SAME, B.F32, B.F32),
                # 11x11 stride 4: the block's patch has 39 x 213 values
                B.make_params(2, 50, 50, 3, 96, 11, 11, 4, 4, wl.PAD_SAME, B.F32, B.F32)):
        assert not B.conv2d_variant_supports(bad, vid)
    # a single channel, a 1x1 window: supported (one padded reduction step)
    assert B.conv2d_variant_supports(
        B.make_params(2, 19, 23, 1, 5, 1, 1, 1, 1, wl.PAD_SAME, B.F32, B.F32), vid)
    # the bf16 twin: bf16 input only, pixels of a row an even number of values apart
    vb = names.index("rowgather_bf16_128x64")
    for out in (B.F32, B.BF16):
        assert B.conv2d_variant_supports(
            B.make_params(32, 224, 224, 3, 64, 7, 7, 2, 2, wl.PAD_SAME, B.BF16, out), vb)
    assert B.conv2d_workspace_size(
        B.make_params(32, 224, 224, 3, 64, 7, 7, 2, 2, wl.PAD_SAME, B.BF16, B.F32), vb) == 0
    assert not B.conv2d_variant_supports(stem, vb)
    assert not B.conv2d_variant_supports(
        B.make_params(5, 30, 17, 3, 64, 5, 5, 3, 1, wl.PAD_SAME, B.BF16, B.F32), vb)
