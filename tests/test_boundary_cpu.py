"""Host-side tests of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, infers shapes like the oracle, and rejects invalid descriptors on the
host before anything is launched."""
import ctypes
import os
import re
import subprocess
import tempfile

import numpy as np
import pytest

import oracle
import paper_1801_08058_amd as ng

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ngconv.h")


def _good(**kw):
    base = dict(n=2, c=64, h=14, w=14, k=64, r=3, s=3, pad_below=(1, 1), pad_above=(1, 1))
    base.update(kw)
    return ng.make_desc(**base)


def test_library_exports_every_declared_symbol():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ngc_[a-z0-9_]+)\s*\(", text))
    assert declared == set(ng.EXPORTS), declared ^ set(ng.EXPORTS)
    lib = ctypes.CDLL(ng.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_size_matches_header():
    fields = re.findall(r"int32_t\s+([a-z_, ]+);", re.search(r"typedef struct \{(.*?)\} ngc_conv_desc;", open(HEADER).read(), re.S).group(1))
    names = [n.strip() for f in fields for n in f.split(",")]
    assert names == [n for n, _ in ng.ngc_conv_desc._fields_]
    assert ctypes.sizeof(ng.ngc_conv_desc) == 4 * len(names)


def test_out_shape_matches_oracle():
    rng = np.random.default_rng(3)
    for _ in range(200):
        h, w, r, s = (int(v) for v in rng.integers(1, 40, 4))
        sh, sw, dh, dw = (int(v) for v in rng.integers(1, 4, 4))
        pb = [int(v) for v in rng.integers(0, 4, 4)]
        a = oracle.Attrs(1, 3, h, w, 4, r, s, sh, sw, dh, dw, *pb)
        P, Q = oracle.out_shape(a)
        d = ng.make_desc(1, 3, h, w, 4, r, s, (sh, sw), (dh, dw), (pb[0], pb[1]), (pb[2], pb[3]))
        got = ng.ngc_conv_out_shape(d, check=False)
        if P < 1 or Q < 1:
            assert got == ng.NGC_BAD_SHAPE
        else:
            assert got == (P, Q)


@pytest.mark.parametrize("kw,status", [
    (dict(n=0), ng.NGC_BAD_SHAPE), (dict(c=-1), ng.NGC_BAD_SHAPE), (dict(stride=(0, 1)), ng.NGC_BAD_SHAPE),
    (dict(dilation=(1, 0)), ng.NGC_BAD_SHAPE), (dict(pad_below=(-1, 0)), ng.NGC_BAD_SHAPE),
    (dict(h=1, w=1, pad_below=(0, 0), pad_above=(0, 0)), ng.NGC_BAD_SHAPE),       # 3x3 window does not fit
    (dict(dtype=7), ng.NGC_BAD_ARG), (dict(x_layout=5), ng.NGC_BAD_ARG), (dict(w_layout=9), ng.NGC_BAD_ARG),
    (dict(epilogue=8), ng.NGC_BAD_ARG), (dict(n=1 << 20, h=1 << 10, w=1 << 10), ng.NGC_BAD_SHAPE),
])
def test_invalid_descriptors_are_rejected_before_launch(kw, status):
    d = _good(**kw)
    fake = 0x1000                       # never dereferenced: validation fails first
    assert ng.ngc_conv_out_shape(d, check=False) == status
    assert ng.ngc_conv_fwd(d, fake, fake, fake, fake, None, None, check=False) == status
    assert ng.ngc_conv_bwd_data(d, fake, fake, fake, None, None, check=False) == status
    assert ng.ngc_conv_bwd_filters(d, fake, fake, fake, None, None, check=False) == status
    assert ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_BWD_FILTERS) == 0
    assert ng.ngc_conv_variant(d, ng.NGC_OP_FWD) == "invalid"


def test_null_pointers_missing_bias_and_workspace():
    d = _good(epilogue=ng.NGC_EPI_BIAS | ng.NGC_EPI_RELU)
    fake = 0x1000
    assert ng.ngc_conv_fwd(d, None, fake, fake, fake, None, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_conv_fwd(d, fake, fake, None, fake, None, None, check=False) == ng.NGC_BAD_ARG     # bias flag, no bias
    assert ng.ngc_conv_fwd(d, fake + 2, fake, fake, fake, None, None, check=False) == ng.NGC_BAD_ARG  # misaligned
    # KCRS filters on the MFMA path need workspace for the re-layout
    assert ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_FWD) >= 64 * 64 * 9 * 2
    assert ng.ngc_conv_fwd(d, fake, fake, fake, fake, None, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv_bwd_filters(d, fake, fake, fake, None, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    with pytest.raises(ng.NgcError):
        ng.ngc_conv_fwd(d, fake, fake, fake, fake, None, None)
    assert ng.ngc_layout_convert(ng.NGC_BF16, 1, 0, 4, 4, fake, 0, fake, 1, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_layout_convert(3, 1, 4, 4, 4, fake, 0, fake, 1, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_filter_convert(d, fake, fake, ng.NGC_KCRS, None, check=False) == ng.NGC_BAD_ARG


def test_backward_compounds_validate_before_launch():
    d = _good(w_layout=ng.NGC_BLOCKED_BWD)
    fake = 0x1000
    assert ng.ngc_conv_bwd_data_relu(d, fake, fake, None, fake, None, None, check=False) == ng.NGC_BAD_ARG   # no x_in
    assert ng.ngc_conv_bwd_data_relu(d, fake, fake, fake + 2, fake, None, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_conv_bwd_data_relu(d, None, fake, fake, fake, None, None, check=False) == ng.NGC_BAD_ARG
    bad = _good(stride=(0, 1))
    assert ng.ngc_conv_bwd_data_relu(bad, fake, fake, fake, fake, None, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_bias_grad(bad, fake, fake, fake, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_conv_bwd_data_relu_db(d, fake, fake, fake, fake, None, None, None, check=False) == ng.NGC_BAD_ARG   # no db
    assert ng.ngc_conv_bwd_data_relu_db(d, fake, fake, None, fake, fake, None, None, check=False) == ng.NGC_BAD_ARG   # no x_in
    assert ng.ngc_conv_bwd_data_relu_db(bad, fake, fake, fake, fake, fake, None, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_conv_bwd_data_relu_db(d, fake, fake, fake, fake, fake, None, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv_variant(d, ng.NGC_OP_BWD_DATA_DB) == ng.ngc_conv_variant(d, ng.NGC_OP_BWD_DATA)
    # partial channel sums sit behind the backprop-data part of the workspace
    assert ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_BWD_DATA_DB) >= ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_BWD_DATA) + 64 * 4
    assert ng.ngc_bias_grad(d, None, fake, None, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_bias_grad(d, fake, fake, None, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    # one fp32 partial per (position chunk, channel), channels padded to 16
    big = _good(n=64, h=56, w=56)
    nb = ng.ngc_conv_workspace_bytes(big, ng.NGC_OP_BIAS_GRAD)
    assert nb % 256 == 0 and 64 * 4 <= nb <= 4096 * 64 * 4
    assert ng.ngc_conv_variant(big, ng.NGC_OP_BIAS_GRAD) == "bias_grad_blocked_bf16"
    assert ng.ngc_conv_variant(_good(dtype=ng.NGC_F32, x_layout=ng.NGC_NCHW, y_layout=ng.NGC_NCHW), ng.NGC_OP_BIAS_GRAD) \
        == "bias_grad_generic"
    assert ng.ngc_conv_variant(bad, ng.NGC_OP_BIAS_GRAD) == "invalid"


def test_softmax_validates_before_launch():
    fake = 0x1000
    assert ng.ngc_softmax(ng.NGC_BF16, 0, 8, fake, fake, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_softmax(ng.NGC_BF16, 4, 0, fake, fake, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_softmax(ng.NGC_BF16, 1 << 31, 8, fake, fake, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_softmax(ng.NGC_BF16, 1 << 30, 1 << 12, fake, fake, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_softmax(7, 4, 8, fake, fake, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_softmax(ng.NGC_BF16, 4, 8, None, fake, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_softmax(ng.NGC_BF16, 4, 8, fake + 1, fake, None, check=False) == ng.NGC_BAD_ARG      # not element aligned
    assert ng.ngc_softmax(ng.NGC_F32, 4, 8, fake, fake + 2, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_softmax_bwd(ng.NGC_F32, 4, 8, fake, None, fake, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_softmax_variant(ng.NGC_BF16, 1000) == "softmax_rows_wave"
    assert ng.ngc_softmax_variant(ng.NGC_BF16, 2048) == "softmax_rows_wave"            # 4 vectors of 8 per lane
    assert ng.ngc_softmax_variant(ng.NGC_BF16, 2056) == "softmax_rows_wg"
    assert ng.ngc_softmax_variant(ng.NGC_BF16, 32768, True) == "softmax_rows_wg"       # 16 vectors per thread, 256 threads
    assert ng.ngc_softmax_variant(ng.NGC_BF16, 32776) == "softmax_rows_block"
    assert ng.ngc_softmax_variant(ng.NGC_BF16, 1001) == "softmax_rows_block"           # rows off the 16-byte grid
    assert ng.ngc_softmax_variant(ng.NGC_F32, 1024) == "softmax_rows_wave"
    assert ng.ngc_softmax_variant(ng.NGC_F32, 16384) == "softmax_rows_wg"
    assert ng.ngc_softmax_variant(ng.NGC_F32, 16388) == "softmax_rows_block"
    assert ng.ngc_softmax_variant(9, 8) == "invalid"


def test_unsupported_is_reported_not_routed_elsewhere():
    # blocked filters with a shape only the direct kernels cover
    d = _good(c=5, k=7, w_layout=ng.NGC_BLOCKED_FWD)
    assert ng.ngc_conv_variant(d, ng.NGC_OP_FWD) == "unsupported"
    assert ng.ngc_conv_fwd(d, 0x1000, 0x1000, None, 0x1000, None, None, check=False) == ng.NGC_UNSUPPORTED


def test_kernel_selection_and_sizes():
    d = _good(n=64, h=56, w=56, w_layout=ng.NGC_BLOCKED_FWD)
    assert ng.ngc_conv_variant(d, ng.NGC_OP_FWD) == "strip_bf16"
    s2 = _good(n=64, h=56, w=56, stride=(2, 2), w_layout=ng.NGC_BLOCKED_FWD)
    assert ng.ngc_conv_variant(s2, ng.NGC_OP_FWD) == "strip_bf16"            # strided strips
    s2b = _good(n=64, h=56, w=56, stride=(2, 2), w_layout=ng.NGC_BLOCKED_BWD)
    assert ng.ngc_conv_variant(s2b, ng.NGC_OP_BWD_DATA) == "strip_bf16"      # one launch per residue class
    # stride 2 with dilation 2: no tap reaches the odd rows of dx -> cleared, the other classes run as strips
    s2d = _good(n=2, h=15, w=9, stride=(2, 1), dilation=(2, 1), pad_below=(2, 0), w_layout=ng.NGC_BLOCKED_BWD)
    assert ng.ngc_conv_variant(s2d, ng.NGC_OP_BWD_DATA) == "strip_bf16"
    big = _good(n=2, h=40, w=40, r=7, s=7, pad_below=(3, 3), pad_above=(3, 3), w_layout=ng.NGC_BLOCKED_BWD)   # 49 taps
    assert ng.ngc_conv_variant(big, ng.NGC_OP_BWD_DATA).startswith("igemm")
    one = _good(n=64, h=56, w=56, r=1, s=1, pad_below=(0, 0), pad_above=(0, 0), w_layout=ng.NGC_BLOCKED_FWD)
    assert ng.ngc_conv_variant(one, ng.NGC_OP_FWD) == "gemm1x1_bf16"
    assert ng.ngc_conv_variant(one, ng.NGC_OP_BWD_FILTERS) == "wgrad_gemm_bf16"
    assert ng.ngc_conv_variant(d, ng.NGC_OP_BWD_FILTERS).startswith("wgrad")
    # layout propagation: 1x1, stride 1, no padding, H*W % 8 == 0 runs on the GEMM kernels with NCHW tensors
    for xl, yl in ((ng.NGC_NCHW, ng.NGC_NCHW16C), (ng.NGC_NCHW16C, ng.NGC_NCHW), (ng.NGC_NCHW, ng.NGC_NCHW)):
        kw = dict(n=64, c=256, h=56, w=56, r=1, s=1, pad_below=(0, 0), pad_above=(0, 0), x_layout=xl, y_layout=yl)
        assert ng.ngc_conv_variant(_good(w_layout=ng.NGC_BLOCKED_FWD, **kw), ng.NGC_OP_FWD) == "gemm1x1_bf16"
        assert ng.ngc_conv_variant(_good(w_layout=ng.NGC_BLOCKED_BWD, **kw), ng.NGC_OP_BWD_DATA) == "gemm1x1_bf16"
        assert ng.ngc_conv_variant(_good(**kw), ng.NGC_OP_BWD_FILTERS) == "wgrad_gemm_bf16"
        kw7 = dict(kw, h=7, w=7)                                              # 49 positions per image
        # anything else with NCHW tensors runs on blocked copies in the workspace, with the kernel of the blocked node
        assert ng.ngc_conv_variant(_good(**kw7), ng.NGC_OP_FWD) == "staged:gemm1x1_bf16"
        assert ng.ngc_conv_variant(_good(**kw7), ng.NGC_OP_BWD_FILTERS) == "staged:wgrad_gemm_bf16"
        assert ng.ngc_conv_variant(_good(w_layout=ng.NGC_BLOCKED_FWD, **kw7), ng.NGC_OP_FWD) == "staged:gemm1x1_bf16"
        kws = dict(kw, stride=(2, 2))
        assert ng.ngc_conv_variant(_good(**kws), ng.NGC_OP_BWD_DATA) == "staged:gemm1x1_bf16"
        blocked = ng.ngc_conv_workspace_bytes(_good(**dict(kw7, x_layout=ng.NGC_NCHW16C, y_layout=ng.NGC_NCHW16C)), ng.NGC_OP_FWD)
        copies = (64 * 256 * 49 * 2 if xl == ng.NGC_NCHW else 0) + (64 * 64 * 49 * 2 if yl == ng.NGC_NCHW else 0)
        assert ng.ngc_conv_workspace_bytes(_good(**kw7), ng.NGC_OP_FWD) == blocked + copies
    # channel counts: multiples of 16 run on the MFMA kernels (partial last tiles), anything else on the direct kernels
    for c, k in ((48, 96), (80, 16), (16, 208)):
        t3 = dict(n=8, c=c, k=k, h=28, w=28)
        assert ng.ngc_conv_variant(_good(w_layout=ng.NGC_BLOCKED_FWD, **t3), ng.NGC_OP_FWD).startswith("strip")
        assert ng.ngc_conv_variant(_good(w_layout=ng.NGC_BLOCKED_BWD, **t3), ng.NGC_OP_BWD_DATA).startswith("strip")
        assert ng.ngc_conv_variant(_good(**t3), ng.NGC_OP_BWD_FILTERS) == "wgrad_gemm_bf16"
        t1 = dict(t3, r=1, s=1, pad_below=(0, 0), pad_above=(0, 0))
        assert ng.ngc_conv_variant(_good(w_layout=ng.NGC_BLOCKED_FWD, **t1), ng.NGC_OP_FWD) == "gemm1x1_bf16"
        assert ng.ngc_conv_variant(_good(w_layout=ng.NGC_BLOCKED_BWD, **t1), ng.NGC_OP_BWD_DATA) == "gemm1x1_bf16"
        ws = ng.ngc_conv_workspace_bytes(_good(**t1), ng.NGC_OP_BWD_FILTERS)
        assert ws >= ((k + 63) // 64) * ((c + 63) // 64) * 64 * 64 * 4      # partials cover whole tiles
    odd = dict(n=8, c=40, k=72, h=28, w=28)
    assert [ng.ngc_conv_variant(_good(**odd), o) for o in range(3)] == ["direct"] * 3
    three = _good(n=8, h=56, w=56, x_layout=ng.NGC_NCHW)                      # 3x3 with NCHW x: a blocked copy of x
    assert [ng.ngc_conv_variant(three, o) for o in range(3)] == ["staged:strip_bf16", "staged:strip_bf16", "staged:wgrad_strip_bf16"]
    xcopy = 8 * 64 * 56 * 56 * 2
    three_b = _good(n=8, h=56, w=56)
    assert ng.ngc_conv_workspace_bytes(three, ng.NGC_OP_BWD_DATA) == 2 * xcopy + ng.ngc_conv_workspace_bytes(three_b, ng.NGC_OP_BWD_DATA)
    assert ng.ngc_conv_workspace_bytes(three, ng.NGC_OP_BWD_FILTERS) == xcopy + ng.ngc_conv_workspace_bytes(three_b, ng.NGC_OP_BWD_FILTERS)
    # the low-channel first layer with an NCHW result: only y gets a copy, the kernel still reads the NCHW x itself
    stem_n = ng.make_desc(8, 3, 224, 224, 64, 7, 7, (2, 2), (1, 1), (3, 3), (3, 3), x_layout=ng.NGC_NCHW, y_layout=ng.NGC_NCHW)
    assert ng.ngc_conv_variant(stem_n, ng.NGC_OP_FWD) == "staged:stem_fwd_bf16"
    assert ng.ngc_conv_workspace_bytes(stem_n, ng.NGC_OP_FWD) == 8 * 64 * 112 * 112 * 2
    assert ng.ngc_data_elems(d, 0) == 64 * 64 * 56 * 56 and ng.ngc_data_elems(d, 1) == 64 * 64 * 56 * 56
    assert ng.ngc_filter_elems(d, ng.NGC_BLOCKED_FWD) == 9 * 4 * 64 * 16
    f32 = _good(dtype=ng.NGC_F32, x_layout=ng.NGC_NCHW, y_layout=ng.NGC_NCHW)
    assert [ng.ngc_conv_variant(f32, o) for o in range(3)] == ["direct"] * 3
    stem = ng.make_desc(64, 3, 224, 224, 64, 7, 7, (2, 2), (1, 1), (3, 3), (3, 3), x_layout=ng.NGC_NCHW)
    assert ng.ngc_conv_out_shape(stem) == (112, 112)
    assert ng.ngc_data_elems(stem, 0) == 64 * 3 * 224 * 224
    for s in range(-6, 1):
        assert ng.ngc_status_string(s)


def test_fastdiv_exact_on_host():
    """The runtime-constant division the kernels use for index decoding, checked on the host
    against integer division (compiled from the product header, host code only)."""
    src = r'''
#include "common.h"
#include <stdio.h>
#include <stdlib.h>
int main() {
    unsigned long long bad = 0; unsigned s = 12345;
    for (unsigned d = 1; d <= 20000; ++d) {
        ngc::FastDiv f = ngc::make_fastdiv(d);
        for (int t = 0; t < 200; ++t) {
            s = s * 1664525u + 1013904223u;
            unsigned n = (t < 4) ? (unsigned[]){0u, d - 1, d, 0xFFFFFFFFu}[t] : (t & 1 ? s : s >> 8);
            if (ngc::fd_div(n, f) != n / d) ++bad;
        }
    }
    for (unsigned d : {1u << 31, 0xFFFFFFFFu, 12544u * 128u, 3u, 7u, 49u}) {
        ngc::FastDiv f = ngc::make_fastdiv(d);
        for (unsigned n : {0u, 1u, d - 1, d, d + 1, 0x7FFFFFFFu, 0xFFFFFFFFu}) if (ngc::fd_div(n, f) != n / d) ++bad;
    }
    printf("%llu\n", bad);
    return bad != 0;
}
'''
    with tempfile.TemporaryDirectory() as td:
        cpp = os.path.join(td, "fd.cpp")
        open(cpp, "w").write(src)
        exe = os.path.join(td, "fd")
        subprocess.check_call(["/opt/rocm/bin/hipcc", "-O1", "-std=c++17", "-Wno-unused-value", "-I",
                               os.path.join(ROOT, "paper_1801_08058_amd", "csrc"), "-o", exe, cpp],
                              stderr=subprocess.DEVNULL)
        assert subprocess.run([exe], capture_output=True, text=True).stdout.strip() == "0"


# ---------------------------------------------------------------- convolution over three spatial axes
def _good3(**kw):
    base = dict(n=2, c=64, d=6, h=10, w=10, k=64, t=3, r=3, s=3, pad_below=(1, 1, 1), pad_above=(1, 1, 1))
    base.update(kw)
    return ng.make_desc3(**base)


def test_conv3d_struct_matches_header():
    body = re.search(r"typedef struct \{((?:(?!typedef struct).)*?)\} ngc_conv3d_desc;", open(HEADER).read(), re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = [n.strip() for f in re.findall(r"int32_t\s+([a-z_, ]+);", body) for n in f.split(",")]
    assert names == [n for n, _ in ng.ngc_conv3d_desc._fields_]
    assert ctypes.sizeof(ng.ngc_conv3d_desc) == 4 * len(names)


def test_conv3d_out_shape_matches_oracle():
    rng = np.random.default_rng(33)
    for _ in range(200):
        ext = [int(v) for v in rng.integers(1, 20, 3)]
        taps = [int(v) for v in rng.integers(1, 6, 3)]
        st = [int(v) for v in rng.integers(1, 4, 3)]
        dil = [int(v) for v in rng.integers(1, 4, 3)]
        pb = [int(v) for v in rng.integers(0, 4, 3)]
        pa = [int(v) for v in rng.integers(0, 4, 3)]
        a = oracle.Attrs3(1, 3, *ext, 4, *taps, *st, *dil, *pb, *pa)
        want = oracle.out_shape3(a)
        got = ng.ngc_conv3d_out_shape(ng.make_desc3(1, 3, *ext, 4, *taps, st, dil, pb, pa), check=False)
        assert got == (ng.NGC_BAD_SHAPE if min(want) < 1 else want)


@pytest.mark.parametrize("kw,status", [
    (dict(d=0), ng.NGC_BAD_SHAPE), (dict(t=0), ng.NGC_BAD_SHAPE), (dict(stride=(1, 0, 1)), ng.NGC_BAD_SHAPE),
    (dict(dilation=(0, 1, 1)), ng.NGC_BAD_SHAPE), (dict(pad_below=(-1, 0, 0)), ng.NGC_BAD_SHAPE),
    (dict(d=2, t=5, pad_below=(0, 1, 1), pad_above=(0, 1, 1)), ng.NGC_BAD_SHAPE), (dict(dtype=7), ng.NGC_BAD_ARG),
    (dict(x_layout=3), ng.NGC_BAD_ARG), (dict(w_layout=9), ng.NGC_BAD_ARG), (dict(epilogue=8), ng.NGC_BAD_ARG),
    (dict(n=4096, c=1024, d=64, h=64, w=64), ng.NGC_BAD_SHAPE),
])
def test_conv3d_invalid_descriptors_are_rejected_before_launch(kw, status):
    d = _good3(**kw)
    assert ng.ngc_conv3d_out_shape(d, check=False) == status
    assert ng.ngc_conv3d_workspace_bytes(d, ng.NGC_OP_FWD) == 0
    assert ng.ngc_conv3d_variant(d, ng.NGC_OP_FWD) == "invalid"
    # non-null, aligned dummies: validation must fail before anything could touch them
    assert ng.ngc_conv3d_fwd(d, 4096, 4096, None, 4096, None, check=False) == status
    assert ng.ngc_conv3d_bwd_data(d, 4096, 4096, 4096, None, check=False) == status
    assert ng.ngc_conv3d_bwd_filters(d, 4096, 4096, 4096, None, check=False) == status


def test_conv3d_null_pointers_bias_and_workspace():
    d = _good3(epilogue=ng.NGC_EPI_BIAS)
    assert ng.ngc_conv3d_fwd(d, None, 4096, 4096, 4096, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_conv3d_fwd(d, 4096, 4096, None, 4096, None, check=False) == ng.NGC_BAD_ARG      # bias flag without bias
    assert ng.ngc_conv3d_fwd(d, 4096, 4100, 4096, 4096, None, check=False) == ng.NGC_BAD_ARG      # misaligned
    d = _good3()
    assert ng.ngc_conv3d_workspace_bytes(d, ng.NGC_OP_FWD) > 0                                    # filter re-layout
    assert ng.ngc_conv3d_fwd(d, 4096, 4096, None, 4096, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv3d_bwd_data(d, 4096, 4096, 4096, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv3d_bwd_filters(d, 4096, 4096, 4096, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv3d_filter_convert(d, 4096, 4096, ng.NGC_KCRS, check=False) == ng.NGC_BAD_ARG


def test_conv3d_kernel_selection_and_sizes(monkeypatch):
    F, B, W = ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS
    d = _good3()
    assert [ng.ngc_conv3d_variant(d, op) for op in (F, B, W)] == ["strip3_bf16", "strip3_bf16", "wgrad_gemm3_bf16"]
    monkeypatch.setenv("NGC_CONV3D_STRIP", "0")
    assert [ng.ngc_conv3d_variant(d, op) for op in (F, B)] == ["igemm3_bf16_256x64"] * 2
    d = _good3(c=128, k=128)
    assert [ng.ngc_conv3d_variant(d, op) for op in (F, B)] == ["igemm3_bf16_128x128"] * 2
    monkeypatch.delenv("NGC_CONV3D_STRIP")
    # one tap in (h, w) with a stride there: not a rank-2 node, not a strip window -> gather kernel
    assert ng.ngc_conv3d_variant(_good3(r=1, s=1, stride=(1, 2, 2), pad_below=(1, 0, 0), pad_above=(1, 0, 0)), F).startswith("igemm3")
    # pre-blocked filters: no workspace for forward / backprop-data
    assert ng.ngc_conv3d_workspace_bytes(_good3(w_layout=ng.NGC_BLOCKED_FWD), F) == 0
    assert ng.ngc_conv3d_workspace_bytes(_good3(w_layout=ng.NGC_BLOCKED_BWD), B) == 0
    assert ng.ngc_conv3d_workspace_bytes(d, F) == 27 * 128 * 128 * 2
    # windows over one group of adjacent axes go to the rank-2 kernels
    t = _good3(t=3, r=1, s=1, pad_below=(1, 0, 0), pad_above=(1, 0, 0))
    assert ng.ngc_conv3d_variant(t, F).startswith("rank2:") and "unsupported" not in ng.ngc_conv3d_variant(t, F)
    p = _good3(t=1, r=1, s=1, pad_below=(0, 0, 0), pad_above=(0, 0, 0))
    assert ng.ngc_conv3d_variant(p, F) == "rank2:gemm1x1_bf16" and ng.ngc_conv3d_variant(p, W).startswith("rank2:wgrad_gemm")
    s_ = _good3(t=1, r=1, s=5, pad_below=(0, 0, 2), pad_above=(0, 0, 2))
    assert ng.ngc_conv3d_variant(s_, B).startswith("rank2:")
    assert ng.ngc_conv3d_workspace_bytes(t, F) == ng.ngc_conv_workspace_bytes(
        ng.make_desc(2, 64, 6, 100, 64, 3, 1, pad_below=(1, 0), pad_above=(1, 0)), F)
    # a 1x3x3 window keeps the depth axis: rank-3 kernels
    assert ng.ngc_conv3d_variant(_good3(t=1, pad_below=(0, 1, 1), pad_above=(0, 1, 1)), F) == "strip3_bf16"
    # fp32, NCDHW and odd channel counts: direct kernels; blocked filters without an MFMA kernel: unsupported
    assert ng.ngc_conv3d_variant(_good3(dtype=ng.NGC_F32), F) == "direct3"
    assert ng.ngc_conv3d_variant(_good3(x_layout=ng.NGC_NCHW), B) == "direct3"
    assert ng.ngc_conv3d_variant(_good3(c=20), W) == "direct3"
    assert ng.ngc_conv3d_variant(_good3(c=48), F) == "strip3_bf16"
    assert ng.ngc_conv3d_variant(_good3(c=20, w_layout=ng.NGC_BLOCKED_FWD), F) == "unsupported"
    assert ng.ngc_conv3d_fwd(_good3(c=20, w_layout=ng.NGC_BLOCKED_FWD), 4096, 4096, None, 4096, None, check=False) == ng.NGC_UNSUPPORTED
    # more classes than the gather kernel holds
    assert ng.ngc_conv3d_variant(_good3(stride=(3, 3, 2)), B) == "direct3"
    # element counts
    d = _good3(c=20, k=7)
    assert ng.ngc_conv3d_data_elems(d, 0) == 2 * 32 * 6 * 10 * 10 and ng.ngc_conv3d_data_elems(d, 1) == 2 * 16 * 6 * 10 * 10
    assert ng.ngc_conv3d_filter_elems(d, ng.NGC_KCRS) == 7 * 20 * 27
    assert ng.ngc_conv3d_filter_elems(d, ng.NGC_BLOCKED_FWD) == 27 * 2 * 7 * 16
    assert ng.ngc_conv3d_filter_elems(d, ng.NGC_BLOCKED_BWD) == 27 * 1 * 20 * 16


def test_wide_rows_stay_on_the_strip_kernel():
    """Rows wider than a strip holds are cut into column tiles instead of falling to the gather kernel; the channel
    sums of the backward compound then need the second pass (a larger workspace than the plain op)."""
    F, B = ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA
    d = ng.make_desc(1, 64, 8, 2000, 64, 3, 3, pad_below=(1, 1), pad_above=(1, 1), w_layout=ng.NGC_BLOCKED_FWD)
    assert ng.ngc_conv_variant(d, F) == "strip_bf16"
    d = ng.make_desc(1, 64, 8, 2000, 64, 3, 3, pad_below=(1, 1), pad_above=(1, 1), w_layout=ng.NGC_BLOCKED_BWD)
    assert ng.ngc_conv_variant(d, B) == "strip_bf16"
    assert ng.ngc_conv_workspace_bytes(d, ng.NGC_OP_BWD_DATA_DB) > ng.ngc_conv_workspace_bytes(d, B)
    # the temporal window of a video layer as the rank-2 node it is
    t = ng.make_desc3(2, 64, 16, 56, 56, 64, 3, 1, 1, pad_below=(1, 0, 0), pad_above=(1, 0, 0), w_layout=ng.NGC_BLOCKED_FWD)
    assert ng.ngc_conv3d_variant(t, F) == "rank2:strip_bf16"


def test_conv3d_backward_compounds_validate_before_launch():
    d = _good3()
    B, DB, BG = ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_DATA_DB, ng.NGC_OP_BIAS_GRAD
    assert ng.ngc_conv3d_workspace_bytes(d, DB) > ng.ngc_conv3d_workspace_bytes(d, B) > 0
    assert ng.ngc_conv3d_workspace_bytes(d, BG) > 0
    assert ng.ngc_conv3d_bwd_data_relu(d, 4096, 4096, None, 4096, None, check=False) == ng.NGC_BAD_ARG          # no x_in
    assert ng.ngc_conv3d_bwd_data_relu(d, 4096, 4096, 4100, 4096, None, check=False) == ng.NGC_BAD_ARG          # misaligned
    assert ng.ngc_conv3d_bwd_data_relu(d, 4096, 4096, 4096, 4096, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv3d_bwd_data_relu_db(d, 4096, 4096, 4096, 4096, None, None, check=False) == ng.NGC_BAD_ARG  # no db
    assert ng.ngc_conv3d_bwd_data_relu_db(d, 4096, 4096, 4096, 4096, 4096, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    assert ng.ngc_conv3d_bias_grad(d, 4096, None, None, check=False) == ng.NGC_BAD_ARG
    assert ng.ngc_conv3d_bias_grad(d, 4096, 4096, None, check=False) == ng.NGC_WORKSPACE_TOO_SMALL
    bad = _good3(d=0)
    assert ng.ngc_conv3d_bwd_data_relu_db(bad, 4096, 4096, 4096, 4096, 4096, None, check=False) == ng.NGC_BAD_SHAPE
    assert ng.ngc_conv3d_bias_grad(bad, 4096, 4096, 4096, check=False) == ng.NGC_BAD_SHAPE


def test_operands_past_two_gib_run_in_groups_of_images():
    """A bf16 node with blocked tensors whose x or y reaches 2 GiB keeps its kernels: the library launches them over
    groups of images that stay below (workspace of one group; backprop-filters adds one dw per group)."""
    F, B, W, DB = ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS, ng.NGC_OP_BWD_DATA_DB
    big = ng.make_desc(68, 64, 500, 500, 64, 3, 3, pad_below=(1, 1), pad_above=(1, 1))
    grp = ng.make_desc(67, 64, 500, 500, 64, 3, 3, pad_below=(1, 1), pad_above=(1, 1))       # 67 images: 2^31 - 3.4 MB
    assert [ng.ngc_conv_variant(big, op) for op in (F, B, W)] == ["sliced:" + ng.ngc_conv_variant(grp, op) for op in (F, B, W)]
    assert ng.ngc_conv_variant(grp, F) == "strip_bf16"
    assert ng.ngc_conv_workspace_bytes(big, F) == ng.ngc_conv_workspace_bytes(grp, F)
    assert ng.ngc_conv_workspace_bytes(big, W) > ng.ngc_conv_workspace_bytes(grp, W)
    assert ng.ngc_conv_workspace_bytes(big, DB) > ng.ngc_conv_workspace_bytes(big, B)
    # NCHW tensors and fp32 are not sliced: the kernels that take them index with 64 bits
    assert not ng.ngc_conv_variant(ng.make_desc(68, 64, 500, 500, 64, 3, 3, x_layout=ng.NGC_NCHW), F).startswith("sliced")
    # one image of 2 GiB: nothing to slice
    one = ng.make_desc(1, 64, 4100, 4100, 64, 3, 3)
    assert ng.ngc_conv_variant(one, F) == "igemm_bf16_256x64"


def test_noalloc_entry_point_refuses_large_nodes_before_touching_the_gpu():
    """Host-side part of ngc_conv_bwd_filters_noalloc: invalid descriptors and nodes whose partials exceed the static
    array are refused by the checks that run before any HIP call (this test runs without a GPU)."""
    assert ng.ngc_static_scratch_bytes() == 32 << 20
    big = ng.make_desc(128, 512, 56, 56, 512, 3, 3, pad_below=(1, 1), pad_above=(1, 1))
    assert ng.ngc_conv_workspace_bytes(big, ng.NGC_OP_BWD_FILTERS) > ng.ngc_static_scratch_bytes()
    assert ng.ngc_conv_bwd_filters_noalloc(big, 16, 16, 16, None, check=False) == ng.NGC_SCRATCH_EXCEEDED
    bad = ng.make_desc(1, 16, 8, 8, 16, 3, 3, stride=(0, 1))
    assert ng.ngc_conv_bwd_filters_noalloc(bad, 16, 16, 16, None, check=False) == ng.NGC_BAD_SHAPE
    ok = ng.make_desc(2, 64, 14, 14, 64, 3, 3, pad_below=(1, 1), pad_above=(1, 1))
    assert ng.ngc_conv_bwd_filters_noalloc(ok, None, 16, 16, None, check=False) == ng.NGC_BAD_ARG


def test_sliced_nodes_size_their_workspace_for_every_group():
    """A node that runs as launches over groups of images (tensors of 2 GiB or more) hands every group the same
    workspace; the split of a backprop-filters reduction is not monotone in the batch, so the remainder group can need
    more than a full one (n = 215, C = K = 128, 200x200: 209 + 6 images).  The size the library reports must cover
    both, for every op."""
    F, B, W, DB = ng.NGC_OP_FWD, ng.NGC_OP_BWD_DATA, ng.NGC_OP_BWD_FILTERS, ng.NGC_OP_BWD_DATA_DB
    mk = lambda n, c=128, k=128, hw=200, wl=ng.NGC_KCRS: ng.make_desc(n, c, hw, hw, k, 3, 3, pad_below=(1, 1), pad_above=(1, 1), w_layout=wl)
    per_image = 128 * 200 * 200 * 2
    full = ((1 << 31) - 1) // per_image
    checked = 0
    for n in list(range(full + 1, full + 40)) + [215, 2 * full + 3, 3 * full - 1]:
        d = mk(n)
        if not ng.ngc_conv_variant(d, W).startswith("sliced"):
            continue
        rem = n % full
        row = (128 * 128 * 9 + 15) // 16 * 16 * 4
        groups = (n + full - 1) // full
        dw_rows = (groups * row + 255) // 256 * 256
        for op in (F, B, W):
            total = ng.ngc_conv_workspace_bytes(d, op)
            base = total - (dw_rows if op == W else 0)
            for g in ([full] + ([rem] if rem else [])):
                need = ng.ngc_conv_workspace_bytes(mk(g), op)
                assert need <= base, (n, op, g, need, base)
        checked += 1
    assert checked >= 30


def test_host_time_per_dispatch_with_launches_stubbed():
    """Kernel selection is meant to be negligible next to kernels of 10-20 us: with NGC_DRY_RUN=1 (every launch
    skipped after the planning) a call through the C ABI with a descriptor the library has seen before has to stay
    under 2 us of host time.  Plain C program against the built library, 10^4 calls per entry point."""
    src = r'''
#include "ngconv.h"
#include <stdio.h>
#include <stdlib.h>
#include <time.h>
static double now_us(void) { struct timespec t; clock_gettime(CLOCK_MONOTONIC, &t); return t.tv_sec * 1e6 + t.tv_nsec * 1e-3; }
static ngc_conv_desc mk(int n, int c, int hw, int k, int r, int stride, int wl, int epi) {
    ngc_conv_desc d = {n, c, hw, hw, k, r, r, stride, stride, 1, 1, r / 2, r / 2, r / 2, r / 2, NGC_BF16, NGC_NCHW16C, NGC_NCHW16C, wl, epi};
    return d;
}
int main(void) {
    setenv("NGC_DRY_RUN", "1", 1);
    void *p = (void *)(size_t)0x100000;                     /* never dereferenced: nothing is launched */
    const size_t big = (size_t)1 << 40;
    const int shapes[6][5] = {{64, 64, 56, 64, 3}, {128, 256, 56, 64, 1}, {128, 128, 28, 128, 3}, {128, 512, 14, 512, 3},
                              {128, 1024, 14, 2048, 1}, {128, 128, 56, 128, 3}};
    double worst = 0;
    for (int s = 0; s < 6; ++s) {
        const int stride = s >= 4 ? 2 : 1;
        ngc_conv_desc f = mk(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], shapes[s][4], stride, NGC_BLOCKED_FWD, NGC_EPI_BIAS | NGC_EPI_RELU);
        ngc_conv_desc b = mk(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], shapes[s][4], stride, NGC_BLOCKED_BWD, 0);
        ngc_conv_desc w = mk(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], shapes[s][4], stride, NGC_KCRS, 0);
        for (int op = 0; op < 4; ++op) {
            double t0 = 0;
            for (int i = -100; i < 10000; ++i) {
                if (i == 0) t0 = now_us();
                int rc = op == 0 ? ngc_conv_fwd(&f, p, p, (const float *)p, p, p, big, 0)
                       : op == 1 ? ngc_conv_bwd_data(&b, p, p, p, p, big, 0)
                       : op == 2 ? ngc_conv_bwd_filters(&w, p, p, (float *)p, p, big, 0)
                                 : ngc_bias_grad(&w, p, (float *)p, p, big, 0);
                if (rc != NGC_OK) { printf("rc %d shape %d op %d\n", rc, s, op); return 2; }
            }
            const double us = (now_us() - t0) / 10000.0;
            if (us > worst) worst = us;
            printf("shape %d op %d: %.3f us per call\n", s, op, us);
        }
    }
    printf("worst %.3f\n", worst);
    return 0;
}
'''
    with tempfile.TemporaryDirectory() as td:
        c = os.path.join(td, "disp.c")
        open(c, "w").write(src)
        exe = os.path.join(td, "disp")
        libdir = os.path.dirname(ng.LIB_PATH)
        subprocess.check_call(["gcc", "-O1", "-D_GNU_SOURCE", "-I", os.path.join(ROOT, "include"), "-o", exe, c, "-L", libdir,
                               "-l:libngconv.so", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"])
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        assert r.returncode == 0, r.stdout + r.stderr
        worst = float(r.stdout.strip().splitlines()[-1].split()[1])
        assert worst < 2.0, r.stdout
