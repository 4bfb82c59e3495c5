"""Host-side checks of libconvfwd.so that need no GPU: exported symbols, descriptor validation,
shape/FLOP formulas against the paper's table, the cooperative-load rule, variant listing, cache files."""
import ctypes
import os
import re

import pytest

from paper_1611_06945_amd import binding as B
from paper_1611_06945_amd import workloads as wl
from paper_1611_06945_amd.workloads import config1, config2, config3, config4, config5_layers

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "convfwd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_]+)\s*\(", text)) - {"defined"})


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"conv_fwd", "conv_fwd_ws", "conv_autotune", "conv_out_shape", "maxpool_fwd", "conv_strerror",
            "conv_cache_load", "conv_cache_save", "conv_force_variant", "conv_variant_count",
            "conv_variant_name", "conv_workspace_bytes", "conv_coop_load_plan"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), "libconvfwd.so does not export %s" % n


def test_binding_mirrors_the_header():
    for n in declared_functions():
        assert hasattr(B, n) or n == "conv_strerror", n
    assert B.strerror(0) == "success"


def test_out_shape_and_flops_match_appendix_a(appendix_a):
    for row in appendix_a:
        d = B.make_desc(row["b"], row["in_c"], row["in_y"], row["in_x"], row["oc"], row["ksz"], row["ksz"],
                        row["stride"], row["pad"])
        assert B.conv_out_shape(d) == (row["out_y"], row["out_x"]), row
        assert "%.6g" % B.conv_flops(d) == "%.6g" % row["flops"], row


def test_out_shape_of_benchmark_configs():
    assert B.conv_out_shape(B.desc_of(config1().shape)) == (32, 32)
    assert B.conv_out_shape(B.desc_of(config2().shape)) == (28, 28)
    assert B.conv_out_shape(B.desc_of(config3().shape)) == (55, 55)
    assert B.conv_out_shape(B.desc_of(config4(5).shape)) == (13, 13)
    assert [B.conv_out_shape(B.desc_of(w.shape)) for w in config5_layers()] == [(55, 55), (27, 27), (13, 13), (13, 13), (13, 13)]


@pytest.mark.parametrize("field,value", [("N", 0), ("C", 0), ("H", 0), ("W", -1), ("K", 0), ("R", 0), ("S", 0),
                                         ("stride", 0), ("pad", -1), ("flags", 128)])
def test_invalid_descriptor_fields(field, value):
    d = B.make_desc(1, 3, 8, 8, 4, 3, 3, 1, 1)
    setattr(d, field, value)
    with pytest.raises(B.ConvError) as e:
        B.conv_out_shape(d)
    assert e.value.status == B.CONV_EINVAL
    assert B.conv_flops(d) == 0.0
    assert B.conv_workspace_bytes(d) == 0


def test_invalid_geometry_dtype_and_sizes():
    with pytest.raises(B.ConvError) as e:
        B.conv_out_shape(B.make_desc(1, 1, 4, 4, 1, 5, 5))  # window larger than the padded input
    assert e.value.status == B.CONV_EINVAL
    assert B.conv_out_shape(B.make_desc(1, 1, 4, 4, 1, 5, 5, 1, 1)) == (2, 2)
    assert B.conv_out_shape(B.make_desc(1, 1, 2, 2, 1, 2, 2, 1, 2)) == (5, 5)  # pad >= window is legal
    with pytest.raises(B.ConvError) as e:
        B.conv_out_shape(B.make_desc(1, 1, 4, 4, 1, 1, 1, dtype=7))
    assert e.value.status == B.CONV_EDTYPE
    with pytest.raises(B.ConvError) as e:
        B.conv_out_shape(B.make_desc(4096, 1024, 32, 32, 1, 1, 1))  # 2^32 input elements
    assert e.value.status == B.CONV_EINVAL
    assert B.lib().conv_out_shape(None, None, None) == B.CONV_EINVAL


def test_null_and_misaligned_pointers_are_rejected_before_any_gpu_call():
    d = B.make_desc(1, 3, 8, 8, 4, 3, 3, 1, 1)
    L = B.lib()
    assert L.conv_fwd(ctypes.byref(d), None, 256, None, 512, None) == B.CONV_EINVAL
    assert L.conv_fwd(ctypes.byref(d), 256, None, None, 512, None) == B.CONV_EINVAL
    assert L.conv_fwd(ctypes.byref(d), 256, 512, None, None, None) == B.CONV_EINVAL
    assert L.conv_fwd(ctypes.byref(d), 260, 512, None, 1024, None) == B.CONV_EINVAL  # not 16-byte aligned
    assert L.conv_fwd(None, 256, 512, None, 1024, None) == B.CONV_EINVAL
    assert L.conv_autotune(ctypes.byref(d), None, 256, None, 512, None, 0, None) == B.CONV_EINVAL
    us = ctypes.c_double(0.0)
    assert L.conv_time_us(ctypes.byref(d), 256, 512, None, 1024, None, 0, None, 0, ctypes.byref(us)) == B.CONV_EINVAL
    assert L.conv_time_us(ctypes.byref(d), 256, 512, None, 1024, None, 0, None, 10, None) == B.CONV_EINVAL
    assert L.conv_time_us(ctypes.byref(d), None, 512, None, 1024, None, 0, None, 10, ctypes.byref(us)) == B.CONV_EINVAL
    assert L.maxpool_fwd(1, 1, 2, 2, 3, 2, 0, 256, 512, None) == B.CONV_EINVAL  # window larger than input
    assert L.maxpool_fwd(1, 1, 5, 5, 3, 2, 9, 256, 512, None) == B.CONV_EDTYPE
    assert L.maxpool_fwd(1, 1, 5, 5, 3, 2, 0, None, 512, None) == B.CONV_EINVAL


def test_cooperative_load_plan_worked_example():
    # Section 3, "Metaprogramming for NN Convolutions": 96 threads loading 256 words issue three loads and only the
    # third is guarded; 64 threads loading 256 words issue four loads, none guarded.
    assert B.conv_coop_load_plan(96, 256) == (3, True)
    assert B.conv_coop_load_plan(64, 256) == (4, False)
    assert B.conv_coop_load_plan(256, 256) == (1, False)
    assert B.conv_coop_load_plan(256, 1) == (1, True)
    for threads in (1, 7, 64, 96, 256):
        for words in (1, 63, 64, 65, 255, 256, 257, 2048):
            n, g = B.conv_coop_load_plan(threads, words)
            assert n == -(-words // threads) and g == (words % threads != 0)
    with pytest.raises(B.ConvError):
        B.conv_coop_load_plan(0, 5)


def all_bench_descs():
    ws = [config1(), config2(), config3()] + [config4(n, dt) for n in (1, 5, 20) for dt in (0, 1, 2)] + config5_layers()
    return [(w.name, B.desc_of(w.shape, w.dtype, relu=True)) for w in ws]


def test_every_benchmark_shape_has_variants_with_unique_names():
    for name, d in all_bench_descs():
        n = B.conv_variant_count(d)
        assert n >= 2, name
        names = [B.conv_variant_name(d, i) for i in range(n)]
        assert len(set(names)) == n
        tag = {0: "_f32_", 1: "_f16_", 2: "_bf16_"}[d.dtype]
        assert all(tag in x for x in names), (name, names)
        assert B.conv_variant_name(d, -1) in names and B.conv_variant_name(d, -2) in names
        # the choice conv_fwd makes needs no workspace; the declared workspace covers every variant
        nows = names.index(B.conv_variant_name(d, -2))
        assert B.conv_variant_workspace(d, nows) == 0
        assert B.conv_workspace_bytes(d) == max(B.conv_variant_workspace(d, i) for i in range(n))
        with pytest.raises(B.ConvError) as e:
            B.conv_variant_name(d, n)
        assert e.value.status == B.CONV_ENOVARIANT


def test_pointwise_variants_only_offered_for_pointwise_shapes():
    d2 = B.desc_of(config2().shape, 0)
    names2 = [B.conv_variant_name(d2, i) for i in range(B.conv_variant_count(d2))]
    assert any(n.startswith("pw_") for n in names2)
    d4 = B.desc_of(config4(5).shape, 0)
    assert not any(B.conv_variant_name(d4, i).startswith("pw_") for i in range(B.conv_variant_count(d4)))
    # C*R*S = 363 is no multiple of the vector width: the gather kernel may only use its element-wise filter loader;
    # the scalar-offset kernel (ug_) loads fp32 rows of any length by vectors, but not 16-bit rows
    d3 = B.desc_of(config3().shape, 0)
    names3 = [B.conv_variant_name(d3, i) for i in range(B.conv_variant_count(d3))]
    assert all("_v" not in n for n in names3 if not n.startswith("ug_"))
    d3h = B.desc_of(config3().shape, 1)
    assert all("_v" not in B.conv_variant_name(d3h, i) for i in range(B.conv_variant_count(d3h)))


def test_force_variant_and_cache_roundtrip(tmp_path):
    B.conv_cache_clear()
    d = B.desc_of(config4(5).shape, 0)
    n = B.conv_variant_count(d)
    default = B.conv_variant_name(d, -1)
    B.conv_force_variant(d, n - 1)
    assert B.conv_variant_name(d, -1) == B.conv_variant_name(d, n - 1)
    with pytest.raises(B.ConvError):
        B.conv_force_variant(d, n)
    B.conv_force_variant(d, -1)
    assert B.conv_variant_name(d, -1) == default

    # a cache file naming a different (valid) variant changes the selection; clear restores the heuristic
    other = next(B.conv_variant_name(d, i) for i in range(n)
                 if B.conv_variant_name(d, i) != default and B.conv_variant_workspace(d, i) == 0)
    path = tmp_path / "cache.txt"
    path.write_text("# comment\n5 256 13 13 384 3 3 1 1 0 1 | %s | %s\n" % (other, other))
    B.conv_cache_load(str(path))
    assert B.conv_variant_name(d, -1) == other and B.conv_variant_name(d, -2) == other
    out = tmp_path / "saved.txt"
    B.conv_cache_save(str(out))
    assert ("5 256 13 13 384 3 3 1 1 0 1 | %s | %s" % (other, other)) in out.read_text()
    B.conv_cache_clear()
    assert B.conv_variant_name(d, -1) == default
    B.conv_cache_load(str(out))
    assert B.conv_variant_name(d, -1) == other
    B.conv_cache_clear()


def test_bad_cache_files_leave_the_cache_alone(tmp_path):
    B.conv_cache_clear()
    d = B.desc_of(config4(5).shape, 0)
    default = B.conv_variant_name(d, -1)
    with pytest.raises(B.ConvError) as e:
        B.conv_cache_load(str(tmp_path / "missing.txt"))
    assert e.value.status == B.CONV_EIO
    bad = tmp_path / "bad.txt"
    bad.write_text("5 256 13 13 384 3 3 1 1 0 1 | only-one-field\n")
    with pytest.raises(B.ConvError):
        B.conv_cache_load(str(bad))
    bad.write_text("5 256 13 x 384 3 3 1 1 0 1 | a | b\n")
    with pytest.raises(B.ConvError):
        B.conv_cache_load(str(bad))
    # unknown variant names (a cache from another build) are ignored, not an error
    bad.write_text("5 256 13 13 384 3 3 1 1 0 1 | nosuch | nosuch\n")
    B.conv_cache_load(str(bad))
    assert B.conv_variant_name(d, -1) == default
    with pytest.raises(B.ConvError) as e:
        B.conv_cache_save(str(tmp_path / "no_such_dir" / "x.txt"))
    assert e.value.status == B.CONV_EIO


def test_appendix_a_workload_list_is_the_papers_table(appendix_a):
    # the package's own copy of the benchmark set must be the table of Appendix A, row for row
    ws = wl.appendix_a(5, wl.F32)
    assert len(ws) == len(appendix_a) == 43
    for r, w in zip(appendix_a, ws):
        s = w.shape
        assert (s.N, s.R, s.S, s.stride, s.K, s.H, s.W, s.C, s.pad) == (
            r["b"], r["ksz"], r["ksz"], r["stride"], r["oc"], r["in_y"], r["in_x"], r["in_c"], r["pad"])
        assert (s.OH, s.OW) == (r["out_y"], r["out_x"])
        assert abs(s.flops - r["flops"]) <= 1e-5 * r["flops"]
    assert len({w.name for w in ws}) == 43
    assert len({w.seeds() for w in ws}) == 43


def test_layout_entry_points_validate_before_any_gpu_call():
    L = B.lib()
    assert L.conv_convert_layout(0, 4, 4, 0, 256, 512, None) == B.CONV_EINVAL      # extent < 1
    assert L.conv_convert_layout(2, 4, 4, 7, 256, 512, None) == B.CONV_EDTYPE
    assert L.conv_convert_layout(2, 4, 4, 0, None, 512, None) == B.CONV_EINVAL
    assert L.conv_convert_layout(2, 4, 4, 0, 256, 256, None) == B.CONV_EINVAL      # in place is not supported
    assert L.conv_convert_layout(70000, 4, 4, 0, 256, 512, None) == B.CONV_EINVAL  # more outer slices than grid rows
    assert L.maxpool_fwd_layout(1, 1, 2, 2, 3, 2, 0, 1, 0, 256, 512, None) == B.CONV_EINVAL  # window larger than input
    assert L.maxpool_fwd_layout(1, 1, 5, 5, 3, 2, 9, 0, 1, 256, 512, None) == B.CONV_EDTYPE
    assert L.maxpool_fwd_layout(1, 1, 5, 5, 3, 2, 0, 0, 1, None, 512, None) == B.CONV_EINVAL


def test_layout_flags_select_only_channel_innermost_kernels():
    from paper_1611_06945_amd.workloads import ConvShape

    sh = ConvShape(2, 32, 13, 13, 64, 3, 3, 1, 1)
    plain = B.desc_of(sh, 1)
    nh = B.desc_of(sh, 1, in_nhwc=True, out_nhwc=True, filt_krsc=True)
    names_plain = [B.conv_variant_name(plain, i) for i in range(B.conv_variant_count(plain))]
    names_nh = [B.conv_variant_name(nh, i) for i in range(B.conv_variant_count(nh))]
    assert names_plain and not any(n.startswith("nhwc_") for n in names_plain)
    assert names_nh and all(n.startswith("nhwc_") for n in names_nh)
    # the two descriptors are different cache keys: forcing a variant for one leaves the other alone
    B.conv_force_variant(nh, 0)
    try:
        assert B.conv_variant_name(nh, -1) == names_nh[0]
        assert B.conv_variant_name(plain, -1) in names_plain
    finally:
        B.conv_force_variant(nh, -1)
    # fully connected shapes are offered the weight-streaming kernels
    fc = B.desc_of(ConvShape(5, 256, 6, 6, 4096, 6, 6, 1, 0), 0)
    assert B.conv_variant_name(fc, -1).startswith("fc_f32_")


def test_winograd_variants_and_the_transformed_filter_format():
    from paper_1611_06945_amd.workloads import ConvShape

    sh = ConvShape(20, 256, 13, 13, 384, 3, 3, 1, 1)
    plain = B.desc_of(sh, 0)
    names = [B.conv_variant_name(plain, i) for i in range(B.conv_variant_count(plain))]
    wino = [i for i, n in enumerate(names) if n.startswith("wino_")]
    assert wino, names
    # they keep the transformed filters (16 values per filter) in the caller's workspace, except those that transform
    # the filters inside the product kernel ("_ff") ...
    assert all(B.conv_variant_workspace(plain, i) == (0 if names[i].endswith("_ff") else 16 * 384 * 256 * 4) for i in wino)
    assert any(names[i].endswith("_ff") for i in wino)
    assert B.conv_workspace_bytes(plain) >= 16 * 384 * 256 * 4
    # ... the cost model picks them where they pay (this layer at batch 20), not on a small batch of the same layer,
    # and only the workspace-free ones when the caller brings no workspace
    assert B.conv_variant_name(plain, -1).startswith("wino_")
    assert not B.conv_variant_name(B.desc_of(sh.with_batch(1), 0), -1).startswith("wino_")
    # filters handed over in the Winograd domain: only those variants, no workspace, its own cache key
    pre = B.desc_of(sh, 0, filt_winograd=True)
    names_pre = [B.conv_variant_name(pre, i) for i in range(B.conv_variant_count(pre))]
    assert names_pre and all(n.startswith("wino_") and "_c8_" in n for n in names_pre)
    assert all(B.conv_variant_workspace(pre, i) == 0 for i in range(len(names_pre)))
    assert B.conv_workspace_bytes(pre) == 0
    assert B.conv_transformed_filter_bytes(plain) == B.conv_transformed_filter_bytes(pre) == 16 * 384 * 256 * 4
    # K is padded to a multiple of 4 in that format
    assert B.conv_transformed_filter_bytes(B.desc_of(ConvShape(1, 8, 9, 9, 10, 3, 3, 1, 1), 0)) == 16 * 12 * 8 * 4
    L = B.lib()
    # 16-bit storage has no Winograd-domain format: its ahead-of-time format is the MFMA operand order (C % 16 == 0)
    assert B.conv_transformed_filter_bytes(B.desc_of(ConvShape(2, 16, 13, 13, 40, 3, 3, 1, 1), 1)) == 64 * 16 * 9 * 2
    for sh2, dt, kw in [(ConvShape(2, 8, 13, 13, 40, 3, 3, 1, 1), 1, {}),               # 16-bit storage, C % 16 != 0
                        (ConvShape(2, 16, 13, 13, 40, 5, 5, 1, 2), 0, {}),              # 5x5
                        (ConvShape(2, 16, 13, 13, 40, 3, 3, 2, 1), 0, {}),              # stride 2
                        (ConvShape(2, 12, 13, 13, 40, 3, 3, 1, 1), 0, {})]:             # C % 8 != 0
        d = B.desc_of(sh2, dt, **kw)
        assert B.conv_transformed_filter_bytes(d) == 0
        assert L.conv_transform_filters(ctypes.byref(d), 256, 512, None) == B.CONV_ENOVARIANT
        dw = B.desc_of(sh2, dt, filt_winograd=True)
        assert B.conv_variant_count(dw) == 0
        assert L.conv_fwd(ctypes.byref(dw), 256, 512, None, 1024, None) == B.CONV_ENOVARIANT
    # not combinable with the channel-innermost formats
    both = B.desc_of(sh, 0, filt_winograd=True, in_nhwc=True, filt_krsc=True)
    assert B.conv_variant_count(both) == 0
    assert B.conv_transformed_filter_bytes(B.desc_of(sh, 0, in_nhwc=True, filt_krsc=True)) == 0
    # pointer checks come before any GPU call
    assert L.conv_transform_filters(ctypes.byref(plain), None, 512, None) == B.CONV_EINVAL
    assert L.conv_transform_filters(ctypes.byref(plain), 256, 520, None) == B.CONV_EINVAL   # output not 256-byte aligned
    assert L.conv_transform_filters(ctypes.byref(plain), 256, 256, None) == B.CONV_EINVAL   # in place
    assert L.conv_transform_filters(None, 256, 512, None) == B.CONV_EINVAL


def test_strided_window_variants_for_first_layers():
    """The first-layer window kernel is offered exactly where its staging fits (host-side validity, no GPU needed), needs no
    workspace, and is what an unmeasured 16-bit first layer gets."""
    from paper_1611_06945_amd.workloads import ConvShape

    def names_of(sh, dt):
        d = B.desc_of(sh, dt)
        return d, [B.conv_variant_name(d, i) for i in range(B.conv_variant_count(d))]

    for dt, tag in ((1, "f16"), (2, "bf16")):
        d, names = names_of(ConvShape(20, 3, 227, 227, 96, 11, 11, 4, 0), dt)
        swin = [i for i, n in enumerate(names) if n.startswith("swin_%s_11x11s4_c3_" % tag)]
        assert [names[i] for i in swin] == ["swin_%s_11x11s4_c3_M96N128" % tag, "swin_%s_11x11s4_c3_M32N128" % tag], names
        assert all(B.conv_variant_workspace(d, i) == 0 for i in swin)
        assert B.conv_variant_name(d, -1) == "swin_%s_11x11s4_c3_M96N128" % tag
        d7, names7 = names_of(ConvShape(5, 3, 224, 224, 64, 7, 7, 2, 3), dt)
        assert [n for n in names7 if n.startswith("swin_")] == ["swin_%s_7x7s2_c3_M64N128" % tag, "swin_%s_7x7s2_c3_M32N128" % tag]
        assert B.conv_variant_name(d7, -1).startswith("swin_")
    # channel tiles that would be mostly empty are not offered: K = 40 fits the 32- and 64-row tiles, not the 96-row one
    _, n40 = names_of(ConvShape(3, 3, 23, 63, 40, 11, 11, 4, 0), 1)
    assert [n for n in n40 if n.startswith("swin_")] == ["swin_f16_11x11s4_c3_M64N128", "swin_f16_11x11s4_c3_M32N128"]
    for sh, dt in [(ConvShape(20, 3, 227, 227, 96, 11, 11, 4, 0), 0),     # fp32 storage
                   (ConvShape(20, 4, 227, 227, 96, 11, 11, 4, 0), 1),     # four channels
                   (ConvShape(20, 3, 227, 227, 96, 11, 11, 2, 0), 1),     # another stride
                   (ConvShape(20, 3, 227, 227, 96, 9, 9, 4, 0), 1),       # another window
                   (ConvShape(20, 3, 63, 63, 96, 11, 11, 4, 0), 1),       # short output rows: a tile would span too many
                   (ConvShape(1, 3, 227, 600, 96, 11, 11, 4, 0), 1),      # rows longer than a staged row
                   (ConvShape(20, 3, 227, 227, 96, 11, 11, 4, 11), 1)]:   # padding as wide as the window
        _, names = names_of(sh, dt)
        assert names and not any(n.startswith("swin_") for n in names), (sh, dt)


def test_every_valid_descriptor_has_a_variant_and_a_default():
    """Seeded random descriptors over the whole documented domain: each has at least one variant, unique names, and a
    default selection that names one of them (host logic only: no launch)."""
    import numpy as np

    rng = np.random.default_rng(4242)
    checked = 0
    for _ in range(3000):
        R, S = int(rng.integers(1, 13)), int(rng.integers(1, 13))
        pad = int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 260)), int(rng.integers(1, 260))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        shape = wl.ConvShape(int(rng.integers(1, 33)), int(rng.integers(1, 1100)), H, W, int(rng.integers(1, 1100)), R, S,
                             int(rng.integers(1, 5)), pad)
        n_in, n_out = shape.N * shape.C * H * W, shape.N * shape.K * shape.OH * shape.OW
        if 4 * max(n_in, n_out) >= 2 ** 32:
            continue  # every tensor stays below 4 GiB (documented limit of the descriptor)
        for dtype in (wl.F32, wl.F16, wl.BF16):
            descs = [B.desc_of(shape, dtype, relu=bool(rng.integers(0, 2)))]
            gib = 2 ** 30 - 2 ** 20  # channel-innermost kernels: input and filter tensors below 1 GiB each
            small = 2 * (n_in + pad * (W + 1) * shape.C) < gib and 2 * shape.K * shape.C * R * S < gib
            if dtype != wl.F32 and shape.C % 8 == 0 and small:
                descs.append(B.desc_of(shape, dtype, relu=True, in_nhwc=True, out_nhwc=False, filt_krsc=True))
                if shape.K % 8 == 0:
                    descs.append(B.desc_of(shape, dtype, relu=True, in_nhwc=True, out_nhwc=True, filt_krsc=True))
            for d in descs:
                n = B.conv_variant_count(d)
                assert n >= 1, (shape, dtype, d.flags)
                names = [B.conv_variant_name(d, i) for i in range(n)]
                assert len(set(names)) == n
                assert B.conv_variant_name(d, -1) in names
                checked += 1
    assert checked > 5000


def test_fused_maxpool_flag_host_rules():
    from paper_1611_06945_amd.workloads import ConvShape

    sh = ConvShape(20, 256, 13, 13, 256, 3, 3, 1, 1)
    fused = B.desc_of(sh, 1, maxpool=True)
    assert B.conv_out_shape(B.desc_of(sh, 1)) == (13, 13) and B.conv_out_shape(fused) == (6, 6)
    names = [B.conv_variant_name(fused, i) for i in range(B.conv_variant_count(fused))]
    assert names and all(n.startswith("wconv_f16_3x3") and "_sk" not in n for n in names)  # one band per image, no splits
    nh = B.desc_of(sh, 2, maxpool=True, in_nhwc=True, out_nhwc=True, filt_krsc=True)
    assert all(B.conv_variant_name(nh, i).startswith("nhwc_win_bf16_3x3") for i in range(B.conv_variant_count(nh)))
    assert B.conv_variant_count(nh) >= 1
    # conv output smaller than the pooling window, Winograd-domain filters: refused
    L = B.lib()
    tiny = B.desc_of(ConvShape(1, 16, 4, 4, 8, 3, 3, 1, 0), 1, maxpool=True)  # 2x2 conv output
    assert L.conv_variant_count(ctypes.byref(tiny)) == B.CONV_EINVAL
    f32 = B.desc_of(sh, 0, maxpool=True)   # fp32: the 3x3 window kernel pools too
    assert B.conv_variant_count(f32) >= 1
    assert all(B.conv_variant_name(f32, i).startswith("wconv_f32_3x3") for i in range(B.conv_variant_count(f32)))
    assert B.conv_variant_count(B.desc_of(ConvShape(20, 96, 13, 13, 256, 5, 5, 1, 2), 0, maxpool=True)) == 0  # fp32 5x5
    assert B.conv_variant_count(B.desc_of(sh, 0, maxpool=True, filt_winograd=True)) == 0


def test_static_scratch_entry_point_validates_and_refuses_oversized_variants_on_the_host():
    d = B.make_desc(20, 64, 56, 56, 192, 3, 3, 1, 1, B.CONV_F32, relu=True)
    with pytest.raises(B.ConvError) as ei:
        B.conv_fwd_static(d, None, 512, None, 1024)
    assert ei.value.status == B.CONV_EINVAL
    with pytest.raises(B.ConvError) as ei:
        B.conv_fwd_static(d, 256 + 4, 512, None, 1024)  # misaligned input pointer
    assert ei.value.status == B.CONV_EINVAL
    over = [i for i in range(B.conv_variant_count(d)) if B.conv_variant_workspace(d, i) > B.CONV_STATIC_SCRATCH_BYTES]
    assert over
    B.conv_force_variant(d, over[0])
    try:
        with pytest.raises(B.ConvError) as ei:  # refused before any HIP call: works without a GPU
            B.conv_fwd_static(d, 256, 512, None, 1024)
        assert ei.value.status == B.CONV_EWORKSPACE
        assert B.conv_variant_name(d, over[0]) in str(ei.value)
        assert str(B.CONV_STATIC_SCRATCH_BYTES) in str(ei.value)
    finally:
        B.conv_force_variant(d, -1)
    # the header's constant and the binding's agree
    text = open(os.path.join(ROOT, "include", "convfwd.h")).read()
    assert "#define CONV_STATIC_SCRATCH_BYTES (32u << 20)" in text and B.CONV_STATIC_SCRATCH_BYTES == 32 << 20


def test_packed_filter_flag_host_rules():
    # kernels that read filters in MFMA operand order: fp16/bf16, stride 1, C % 16 == 0, 3x3 / 5x5 windows with a border
    # narrower than the window, channel-innermost input; every other use of the flag finds no kernel
    from paper_1611_06945_amd.workloads import ConvShape

    ok = B.desc_of(ConvShape(1, 64, 13, 13, 64, 3, 3, 1, 1), wl.F16, in_nhwc=True, filt_packed=True)
    assert B.conv_variant_count(ok) > 0
    assert all(B.conv_variant_name(ok, i).startswith("pwin_") for i in range(B.conv_variant_count(ok)))
    assert B.conv_transformed_filter_bytes(ok) == 64 * 64 * 9 * 2
    ragged = B.desc_of(ConvShape(1, 64, 13, 13, 40, 3, 3, 1, 1), wl.BF16, in_nhwc=True, filt_packed=True)
    assert B.conv_transformed_filter_bytes(ragged) == 64 * 64 * 9 * 2   # rows padded to whole 32-row blocks
    for shape, dt, kw in [
        (ConvShape(1, 64, 13, 13, 64, 3, 3, 1, 1), wl.F32, dict(in_nhwc=True)),
        (ConvShape(1, 40, 13, 13, 64, 3, 3, 1, 1), wl.F16, dict(in_nhwc=True)),
        (ConvShape(1, 64, 13, 13, 64, 3, 3, 2, 1), wl.F16, dict(in_nhwc=True)),
        (ConvShape(1, 64, 13, 13, 64, 3, 3, 1, 1), wl.F16, dict(in_nhwc=False)),
        (ConvShape(1, 64, 13, 13, 64, 3, 3, 1, 1), wl.F16, dict(in_nhwc=True, filt_krsc=True)),
        (ConvShape(1, 64, 13, 13, 64, 3, 3, 1, 1), wl.F16, dict(in_nhwc=True, maxpool=True)),
        (ConvShape(1, 64, 13, 13, 64, 3, 3, 1, 3), wl.F16, dict(in_nhwc=True)),
        (ConvShape(1, 64, 13, 13, 64, 7, 7, 1, 3), wl.F16, dict(in_nhwc=True)),
    ]:
        d = B.desc_of(shape, dt, filt_packed=True, **kw)
        assert B.conv_variant_count(d) == 0, (shape, dt, kw)
    # the conversion call validates before any GPU call and names the target by the flag
    with pytest.raises(B.ConvError) as ei:
        B.conv_transform_filters(ok, 256, 512 + 16, None)   # output not 256-byte aligned
    assert ei.value.status == B.CONV_EINVAL
    none = B.desc_of(ConvShape(1, 40, 13, 13, 64, 3, 3, 1, 1), wl.F16, in_nhwc=True, filt_packed=True)
    assert B.conv_transformed_filter_bytes(none) == 0
    with pytest.raises(B.ConvError) as ei:
        B.conv_transform_filters(none, 256, 512, None)
    assert ei.value.status == B.CONV_ENOVARIANT


def test_saved_cache_carries_the_identity_of_device_and_kernels(tmp_path):
    B.conv_cache_clear()
    d = B.desc_of(config4(5).shape, 0)
    names = [B.conv_variant_name(d, i) for i in range(B.conv_variant_count(d))]
    other = names[-1]
    src = tmp_path / "in.txt"
    src.write_text("5 256 13 13 384 3 3 1 1 0 1 | %s | %s\n" % (other, other))
    B.conv_cache_load(str(src))
    out = tmp_path / "saved.txt"
    B.conv_cache_save(str(out))
    text = out.read_text()
    head = text.splitlines()[0]
    m = re.match(r"#! convfwd-cache device=(\S+) registry=([0-9a-f]{16})$", head)
    assert m, head
    B.conv_cache_clear()
    B.conv_cache_load(str(out))                      # its own file loads
    assert B.conv_variant_name(d, -1) == other
    B.conv_cache_clear()
    default = B.conv_variant_name(d, -1)
    # another set of kernels: refused, cache untouched
    reg = m.group(2)
    wrong = tmp_path / "wrong_registry.txt"
    wrong.write_text(text.replace(reg, ("0" if reg[0] != "0" else "1") + reg[1:]))
    with pytest.raises(B.ConvError) as e:
        B.conv_cache_load(str(wrong))
    assert e.value.status == B.CONV_EIO and B.conv_variant_name(d, -1) == default
    # a malformed identity line: refused
    wrong.write_text("#! convfwd-cache device=x\n" + "\n".join(text.splitlines()[1:]) + "\n")
    with pytest.raises(B.ConvError):
        B.conv_cache_load(str(wrong))
    # another device: refused when this host knows its own device; a host without a GPU ("none") accepts any
    wrong.write_text(text.replace("device=" + m.group(1), "device=gfx000/Other_Device/1cu"))
    if m.group(1) == "none":
        B.conv_cache_load(str(wrong))
    else:
        with pytest.raises(B.ConvError):
            B.conv_cache_load(str(wrong))
    B.conv_cache_clear()


def test_run_ops_validates_each_element_and_reports_the_failing_index():
    L = B.lib()
    assert L.conv_run_ops(None, 0, None, None) == B.CONV_EINVAL
    empty = (B.conv_op * 1)()
    assert L.conv_run_ops(empty, 0, None, None) == B.CONV_OK          # nothing to do
    assert L.conv_run_ops(empty, -1, None, None) == B.CONV_EINVAL
    bad_kind = B.conv_op(7, B.conv_desc(), 256, None, None, 512, None, 0, (ctypes.c_int32 * 9)())
    failed = ctypes.c_int32(-1)
    assert L.conv_run_ops((B.conv_op * 1)(bad_kind), 1, None, ctypes.byref(failed)) == B.CONV_EINVAL and failed.value == 0
    # element 0 is refused by its own validation before any GPU call (a pool window larger than the image), and nothing
    # after it is looked at
    ops = [B.op_maxpool(1, 8, 2, 2, 3, 2, B.CONV_F16, False, False, 256, 512),
           B.op_convert(0, 0, 0, B.CONV_F16, 256, 512)]
    with pytest.raises(B.ConvError) as e:
        B.conv_run_ops(ops)
    assert e.value.status == B.CONV_EINVAL and "operation 0" in str(e.value)
    # a convolution element is validated like conv_fwd_ws: a misaligned input pointer
    d = B.make_desc(1, 16, 8, 8, 16, 3, 3, 1, 1, B.CONV_F16, relu=True)
    with pytest.raises(B.ConvError) as e:
        B.conv_run_ops([B.op_conv(d, 256 + 2, 512, None, 1024)])
    assert e.value.status == B.CONV_EINVAL
    assert ctypes.sizeof(B.conv_op) == 4 + 44 + 5 * 8 + 8 + 36 + 4   # the C layout: int32, conv_desc, 5 pointers, size_t, 9 int32, tail padding
