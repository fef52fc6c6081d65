"""CPU-only checks of the C boundary: the built library exports every function
include/rmm.h declares, and argument errors are reported as status codes before
any GPU work is attempted."""
import ctypes
import os
import re

import pytest
import torch

import paper_2201_13195_amd as rmm
from paper_2201_13195_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(rmm.lib_path()):
        from paper_2201_13195_amd import build
        build.build()
    return rmm.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "rmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rmm_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"rmm_forward", "rmm_backward", "rmm_sketch", "rmm_workspace_bytes", "rmm_status_string",
            "rmm_debug_philox", "rmm_debug_sketch_tile", "rmm_version"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    seen = {rmm.rmm_status_string(s) for s in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6
    assert rmm.rmm_status_string(-99) == "unknown status"
    assert rmm.rmm_version() >= 100


def test_workspace_query(lib):
    assert rmm.rmm_workspace_bytes(4096, 768, 3072, 410, torch.bfloat16, rmm.GAUSSIAN, binding.OP_BACKWARD) \
        >= 410 * 3072 * 2
    assert rmm.rmm_workspace_bytes(256, 128, 128, 32, torch.float32, rmm.GAUSSIAN, binding.OP_BACKWARD) \
        >= 32 * 128 * 4
    # invalid descriptors -> 0
    assert rmm.rmm_workspace_bytes(0, 768, 3072, 410, torch.bfloat16, 0, binding.OP_BACKWARD) == 0
    assert rmm.rmm_workspace_bytes(4096, 768, 3072, 410, torch.bfloat16, 7, binding.OP_BACKWARD) == 0
    assert rmm.rmm_workspace_bytes(4096, 768, 3072, 410, torch.bfloat16, 0, 9) == 0
    assert lib.rmm_workspace_bytes(None, 0) == 0


def test_invalid_arguments_are_status_codes(lib):
    """Every call here fails validation, so nothing is launched (no GPU needed)."""
    D, S = binding._Desc, binding._State
    st = S(1, 2)
    good = D(64, 32, 32, 8, 0, 0)
    fake = ctypes.c_void_p(0x1000)       # aligned, never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    assert lib.rmm_forward(None, st, fake, fake, None, fake, fake, None, 0, None) == -1
    assert lib.rmm_forward(ctypes.byref(good), st, None, fake, None, fake, fake, None, 0, None) == -1
    assert lib.rmm_forward(ctypes.byref(good), st, odd, fake, None, fake, fake, None, 0, None) == -1
    for bad in (D(0, 32, 32, 8, 0, 0), D(64, -1, 32, 8, 0, 0), D(64, 32, 32, 0, 0, 0), D(64, 32, 32, 8, 5, 0),
                D(64, 32, 32, 8, 0, 3), D(1 << 31, 32, 32, 8, 0, 0)):
        assert lib.rmm_forward(ctypes.byref(bad), st, fake, fake, None, fake, fake, None, 0, None) == -1
        assert lib.rmm_backward(ctypes.byref(bad), st, fake, fake, fake, fake, fake, None, None, 0, None) == -1
    assert lib.rmm_backward(ctypes.byref(good), st, fake, fake, fake, fake, None, None, None, 0, None) == -1
    # bias / dbias are read and written with vector accesses: a misaligned one is refused
    assert lib.rmm_forward(ctypes.byref(good), st, fake, fake, odd, fake, fake, None, 0, None) == -1
    assert lib.rmm_backward(ctypes.byref(good), st, fake, fake, fake, fake, fake, odd, fake, 1 << 20, None) == -1
    assert lib.rmm_backward_accumulate(ctypes.byref(good), st, fake, fake, fake, fake, fake, odd, fake, 1 << 20, None) == -1
    # workspace missing / too small
    assert lib.rmm_backward(ctypes.byref(good), st, fake, fake, fake, fake, fake, None, None, 0, None) == -3
    assert lib.rmm_backward(ctypes.byref(good), st, fake, fake, fake, fake, fake, None, fake, 8, None) == -3
    assert lib.rmm_sketch(0, 4, 4, 0, 0, st, fake, fake, None, 0, None) == -1
    assert lib.rmm_sketch(8, 4, 4, 0, 0, st, None, fake, None, 0, None) == -1
    assert lib.rmm_sketch(8, 4, 4, 2, 0, st, fake, fake, None, 0, None) == -1
    assert lib.rmm_debug_philox(st, 0, 0, 0, fake, None) == -1
    assert lib.rmm_debug_philox(st, 0, 0, 4, None, None) == -1
    assert lib.rmm_debug_sketch_tile(0, st, -1, 0, 4, 4, fake, None) == -1
    assert lib.rmm_debug_sketch_tile(2, st, 0, 0, 4, 4, fake, None) == -1
    assert lib.rmm_debug_sketch_tile(0, st, 0, 0, 1 << 20, 1 << 12, fake, None) == -2      # more entries than one launch covers
    # variance monitors off the MFMA path: d_in sets the number of tile rows of the plain product
    wide = D(8, (1 << 22) + 4, 8, 2, 0, 0)
    assert lib.rmm_variance_stats(ctypes.byref(wide), fake, fake, fake, fake, 1 << 40, None) == -2


def test_binding_refuses_cpu_tensors(lib):
    X = torch.zeros(8, 4)
    W = torch.zeros(4, 4)
    with pytest.raises(ValueError):
        rmm.rmm_forward(X, W, None, 2, rmm.GAUSSIAN, 0, 0,
                        Y=torch.zeros(8, 4), X_proj=torch.zeros(2, 4), ws=torch.zeros(16, dtype=torch.uint8))


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2201_13195_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, os.path.join(dirpath, f)


def test_workspace_sizes_follow_the_documented_layout(lib):
    """Host-side planning only: forward = the partial sums of the sketch of X; backward = G (k x d_out
    in the layer's dtype, rounded to 256 bytes) + the partial sums of the sketch of dY; inside a layer
    pass the sketch may use fewer token slices than on its own, or up to a quarter more; partial-sum slices never
    outnumber the 128-token blocks; the fp32 path needs no sketch partials; the variance op always
    needs some."""
    bf16, f32 = torch.bfloat16, torch.float32
    for n, d_in, d_out, k in [(4096, 768, 3072, 410), (16384, 1024, 4096, 1638), (16384, 4096, 1024, 32),
                              (333, 200, 136, 77), (100, 8, 8, 3), (4100, 520, 264, 64), (1, 8, 8, 1)]:
        fwd = rmm.rmm_workspace_bytes(n, d_in, d_out, k, bf16, 0, binding.OP_FORWARD)
        bwd = rmm.rmm_workspace_bytes(n, d_in, d_out, k, bf16, 0, binding.OP_BACKWARD)
        sk_x = rmm.rmm_workspace_bytes(n, d_in, d_in, k, bf16, 0, binding.OP_SKETCH)
        sk_y = rmm.rmm_workspace_bytes(n, d_out, d_out, k, bf16, 0, binding.OP_SKETCH)
        g = (k * d_out * 2 + 255) // 256 * 256
        assert 0 <= fwd <= 1.25 * sk_x + 4 * k * d_in and g <= bwd <= g + 1.25 * sk_y + 4 * k * d_out, (n, d_in, d_out, k)
        assert (fwd > 0) == (sk_x > 0), (n, d_in, d_out, k)
        for sk, d in ((sk_x, d_in), (sk_y, d_out), (fwd, d_in), (bwd - g, d_out)):
            assert sk % 256 == 0
            slices = sk / (k * d * 4)
            assert slices == 0 or 2 <= slices <= (n + 127) // 128 + 0.01
        assert rmm.rmm_workspace_bytes(n, d_in, d_out, k, f32, 0, binding.OP_FORWARD) == 0
        assert rmm.rmm_workspace_bytes(n, d_in, d_out, k, f32, 0, binding.OP_BACKWARD) == (k * d_out * 4 + 255) // 256 * 256
        for dt in (bf16, f32):
            assert rmm.rmm_workspace_bytes(n, d_in, d_out, k, dt, 1, binding.OP_VARIANCE) >= 256
    # widths that are not multiples of 8 take the plain kernels: no partials
    assert rmm.rmm_workspace_bytes(300, 67, 101, 9, bf16, 0, binding.OP_FORWARD) == 0


def test_new_entry_points_validate_before_launching(lib):
    D, S = binding._Desc, binding._State
    st, good, fake = S(1, 2), D(64, 32, 32, 8, 0, 0), ctypes.c_void_p(0x1000)
    lib.rmm_variance_stats.restype = ctypes.c_int
    assert lib.rmm_variance_stats(None, fake, fake, fake, fake, 1 << 20, None) == -1
    assert lib.rmm_variance_stats(ctypes.byref(good), None, fake, fake, fake, 1 << 20, None) == -1
    assert lib.rmm_variance_stats(ctypes.byref(good), fake, fake, ctypes.c_void_p(0x1004), fake, 1 << 20, None) == -1
    assert lib.rmm_variance_stats(ctypes.byref(good), fake, fake, fake, None, 0, None) == -3
    assert lib.rmm_variance_stats(ctypes.byref(good), fake, fake, fake, fake, 8, None) == -3
    assert lib.rmm_backward_accumulate(ctypes.byref(good), st, fake, fake, fake, fake, None, None, None, 0, None) == -1
    assert lib.rmm_backward_accumulate(ctypes.byref(good), st, fake, fake, fake, fake, fake, None, None, 0, None) == -3
    assert lib.rmm_sketch_profiled(0, 4, 4, 0, 0, st, fake, fake, None, 0, None, None, None) == -1
    # the entry point on the library's static scratch: argument errors, then its size limit
    assert lib.rmm_sketch_static(0, 4, 4, 0, 0, st, fake, fake, None) == -1
    assert lib.rmm_sketch_static(8, 4, 4, 0, 0, st, fake, ctypes.c_void_p(0x1004), None) == -1
    assert rmm.rmm_workspace_bytes(16384, 4096, 4096, 1638, torch.bfloat16, 0, binding.OP_SKETCH) > rmm.STATIC_SCRATCH_BYTES
    assert lib.rmm_sketch_static(16384, 4096, 1638, 1, 0, st, fake, fake, None) == -5


def test_operands_of_two_gib_or_more_stay_on_the_mfma_path(lib):
    """The MFMA kernels address an operand with 32-bit offsets from the rows a work-group reads,
    so the operand's total size does not matter; what takes the plain kernels (no partial-sum
    workspace) is a width that is not a multiple of 8 or a row of 2^22 elements or more."""
    bf16 = torch.bfloat16
    below = rmm.rmm_workspace_bytes((1 << 20) - 128, 1016, 8, 70, bf16, 0, binding.OP_FORWARD)     # 2.13e9 bytes < 2^31
    above = rmm.rmm_workspace_bytes((1 << 20) + 128, 1024, 8, 70, bf16, 0, binding.OP_FORWARD)     # 2^31 + ...
    assert below > 0 and above > 0
    assert rmm.rmm_workspace_bytes(4096, 1 << 22, 8, 70, bf16, 0, binding.OP_FORWARD) == 0
    assert rmm.rmm_workspace_bytes(4096, 1020, 8, 70, bf16, 0, binding.OP_FORWARD) == 0


def test_sors_kind_at_the_boundary(lib):
    """The structured kind needs no token-slice scratch (its sketch products are one kernel), shares
    a launch with the plain product only where that leaves compute units idle, and has no
    variance monitor; unknown kinds stay invalid."""
    bf = torch.bfloat16
    assert rmm.SORS == 2
    assert rmm.rmm_workspace_bytes(4096, 768, 768, 410, bf, rmm.SORS, binding.OP_SKETCH) == 0
    assert rmm.rmm_workspace_bytes(4096, 768, 3072, 410, bf, rmm.SORS, binding.OP_FORWARD) == 0
    assert rmm.rmm_workspace_bytes(4096, 768, 3072, 410, bf, rmm.SORS, binding.OP_BACKWARD) == 410 * 3072 * 2
    assert rmm.rmm_workspace_bytes(4096, 768, 3072, 410, bf, 3, binding.OP_BACKWARD) == 0
    assert rmm.rmm_uses_paired_launch(4096, 768, 3072, 410, bf, rmm.SORS, binding.OP_FORWARD)       # 192 tiles on 256 CUs
    assert rmm.rmm_uses_paired_launch(4096, 768, 3072, 410, bf, rmm.SORS, binding.OP_BACKWARD)
    assert rmm.rmm_uses_paired_launch(16384, 1024, 4096, 1638, bf, rmm.SORS, binding.OP_FORWARD)      # few long strips beside 4 rounds of tiles
    assert not rmm.rmm_uses_paired_launch(16384, 1024, 4096, 1638, bf, rmm.SORS, binding.OP_BACKWARD) # as many strip groups as CUs
    assert rmm.rmm_uses_paired_launch(4096, 768, 768, 410, bf, rmm.SORS, binding.OP_FORWARD)          # 192 split tiles
    assert not rmm.rmm_uses_paired_launch(4096, 512, 768, 410, bf, rmm.SORS, binding.OP_FORWARD)      # 256-thread plain tiles
    assert not rmm.rmm_uses_paired_launch(2048, 768, 3072, 410, bf, rmm.SORS, binding.OP_FORWARD)     # a single chunk
    assert not rmm.rmm_uses_paired_launch(4096, 768, 3072, 2049, bf, rmm.SORS, binding.OP_FORWARD)    # too many sketch columns
    assert rmm.rmm_uses_paired_launch(4096, 768, 3072, 410, bf, rmm.GAUSSIAN, binding.OP_BACKWARD)
    D, fake = binding._Desc, ctypes.c_void_p(0x1000)
    lib.rmm_variance_stats.restype = ctypes.c_int
    assert lib.rmm_variance_stats(ctypes.byref(D(4096, 768, 3072, 410, 1, 2)), fake, fake, fake, fake, 1 << 30, None) == -2
