"""The C-ABI library loads without a GPU and exports every symbol the public header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "q8t.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(q8t_[a-z0-9_]+)\s*\(", text)))


def _lib_path():
    path = os.path.join(ROOT, "paper_1805_11046_amd", "libq8t.so")
    if not os.path.exists(path):
        import __graft_entry__
        __graft_entry__.build()
    return path


def test_header_declares_the_expected_calls():
    names = _declared_functions()
    for must in ("q8t_quantize", "q8t_quantize_with_range", "q8t_quantize_bifurcate", "q8t_dequantize",
                 "q8t_qgemm_fwd", "q8t_qgemm_dgrad", "q8t_qgemm_wgrad", "q8t_qconv_fwd", "q8t_qconv_dgrad",
                 "q8t_qconv_wgrad", "q8t_range_bn_fwd", "q8t_range_bn_bwd", "q8t_range_bn_scale"):
        assert must in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(_lib_path())
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_binding_covers_every_declared_symbol():
    _lib_path()
    from paper_1805_11046_amd import binding
    assert sorted(binding.EXPORTED) == _declared_functions()


def test_host_only_calls():
    # these entry points do no GPU work: the closed form of Section 3 and size queries
    _lib_path()
    from paper_1805_11046_amd import binding
    import math
    assert binding.range_bn_scale(401408) == (2 * math.log(401408)) ** -0.5
    assert binding._lib.q8t_quantize_workspace_size(1 << 20) >= 8
    d = binding.conv_desc(128, 64, 56, 56, 64, 3, 3, 1, 1)
    assert (d.P, d.Q) == (56, 56)
    for which in (0, 1, 2):
        assert binding._lib.q8t_qconv_workspace_size(ctypes.byref(d), which) >= 0
    # the first layer of a ResNet at batch 256 runs on the kernel that builds its operand in LDS: its workspace is
    # the packed filter, not 630 MB of explicit im2col rows
    d1 = binding.conv_desc(256, 3, 224, 224, 64, 7, 7, 2, 3)
    assert 0 < binding._lib.q8t_qconv_workspace_size(ctypes.byref(d1), 0) < (1 << 20)
    assert "gfx950" in binding.version()


def test_argument_errors_are_reported_before_any_launch():
    _lib_path()
    from paper_1805_11046_amd import binding
    L = binding._lib
    assert L.q8t_quantize(None, 16, 8, 0, 0, None, None, None, None) == -1      # NULL
    assert L.q8t_quantize(None, -1, 8, 0, 0, None, None, None, None) == -2      # shape
    assert L.q8t_quantize(None, 16, 17, 0, 0, None, None, None, None) == -3     # bits
    assert L.q8t_quantize_noalloc(None, (1 << 34) + 1, 8, 0, 0, None, None, None) == -2   # beyond the maximum
    assert L.q8t_quantize_noalloc(None, 16, 8, 0, 0, None, None, None) == -1
    assert L.q8t_qgemm_fwd(None, None, None, None, 0, 1, 1, None, None, None, None) == -2
    assert L.q8t_range_bn_fwd(None, 1, 1, 1, 1, None, None, 0.0, None, None, None, None, None, None) == -2


def test_packed_filter_sizes_follow_the_kernel_that_serves_the_shape():
    # host logic of the packed filters: codes rounded up to 256 bytes + one column sum per output channel of the product,
    # for the shapes the register-tile and wide-tile kernels take; nothing for the others
    _lib_path()
    from paper_1805_11046_amd import binding

    def size(case, which):
        return binding.qconv_pack_size(binding.conv_desc(*case), which)

    def expect(case, which):
        n, c, h, w, k, r, s, st, pad = case
        up = lambda v: (v + 255) // 256 * 256
        return up(k * c * r * s) + up(4 * (k if which == 0 else c))

    for case in ((256, 256, 14, 14, 256, 3, 3, 1, 1), (256, 512, 7, 7, 512, 3, 3, 1, 1), (256, 64, 56, 56, 64, 3, 3, 1, 1),
                 (8, 64, 28, 28, 128, 1, 1, 1, 0)):
        for which in (0, 1):
            assert size(case, which) == expect(case, which)
    lattice = (256, 64, 56, 56, 128, 1, 1, 2, 0)       # forward on the gathered positions; its layer gradient packs nothing
    assert size(lattice, 0) == expect(lattice, 0) and size(lattice, 1) == 0
    for case in ((256, 64, 56, 56, 128, 3, 3, 2, 1), (256, 3, 224, 224, 64, 7, 7, 2, 3), (2, 3, 7, 6, 4, 3, 3, 1, 1)):
        assert size(case, 0) == 0 and size(case, 1) == 0
    assert size(lattice, 2) == 0                       # the weight gradient reads no filter
    L = binding._lib
    assert L.q8t_qconv_pack_multi(1, None, None, None, None, None) == -1
    assert L.q8t_qconv_pack_multi(0, None, None, None, None, None) == 0
