"""Host-only checks of the C boundary: the library loads without a GPU,
exports every symbol the header declares, and its argument validation
returns the documented codes without touching a device."""
import ctypes
import os
import re

import pytest

import workloads as wl
from paper_2501_05460_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="library not built")


def header_functions(names=("epd_encode.h", "epd_encode_test.h")):
    found = set()
    for name in names:
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        found |= set(re.findall(r"\b(epd_[a-z0-9_]+)\s*\(", text))
    return sorted(found)


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = header_functions()
    assert "epd_encode" in names and "epd_encode_range" in names and "epd_create" in names
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names
    # the serving header carries no test or measurement hook
    serving = header_functions(("epd_encode.h",))
    assert not [n for n in serving if n.startswith(("epd_op_", "epd_profile_", "epd_debug_"))]


def test_weight_count_matches_generator_order():
    for name in wl.ALL_WORKLOADS:
        d = wl.workload(name).desc
        assert B.weight_count(d) == len(wl.weight_specs(d))
    d = wl.workload("c4").desc
    assert B.weight_count(d.replace(qk_norm=wl.QKNORM_PER_HEAD, final_norm=1)) == \
        len(wl.weight_specs(d.replace(qk_norm=wl.QKNORM_PER_HEAD, final_norm=1)))
    scaled = d.replace(layer_scale=1)                      # two more vectors per layer
    assert B.weight_count(scaled) == B.weight_count(d) + 2 * d.layers == len(wl.weight_specs(scaled))
    assert B.weight_count(d.replace(layer_scale=2)) == B.EPD_ERR_INVALID_ARG
    with_cls = d.replace(class_token=1)                    # the class vector; pos grows by a row
    assert B.weight_count(with_cls) == B.weight_count(d) + 1 == len(wl.weight_specs(with_cls))
    assert wl.weight_specs(with_cls)[2][1] == (d.n_patches + 1, d.hidden)
    assert B.weight_count(d.replace(class_token=2)) == B.EPD_ERR_INVALID_ARG
    rs = wl.workload("c2").desc.replace(final_norm=1, proj_kind=wl.PROJ_RESAMPLER, proj_mid=64, proj_heads=28)
    assert B.weight_count(rs) == len(wl.weight_specs(rs))
    assert B.weight_count(rs.replace(proj_heads=27)) == B.EPD_ERR_SHAPE          # 3584 % 27 != 0
    assert B.weight_count(rs.replace(proj_heads=7)) == B.EPD_ERR_UNSUPPORTED     # head dim 512 in bf16 mode
    assert B.weight_count(rs.replace(pixel_shuffle=1)) < 0


def test_check_desc_accepts_the_five_configs():
    for name in wl.ALL_WORKLOADS:
        s, msg = B.check_desc(wl.workload(name).desc)
        assert s == B.EPD_OK, (name, msg)


def test_check_desc_accepts_any_patch_grid_and_a_class_token():
    d = wl.workload("c3").desc
    for change in (dict(tile_size=14 * 6, pixel_shuffle=0, proj_prenorm=0),      # 36 patches per slice
                   dict(tile_size=14 * 27, pixel_shuffle=0, proj_prenorm=0),     # 729
                   dict(class_token=1), dict(class_token=1, dtype=wl.DT_FP32)):
        s, msg = B.check_desc(d.replace(**change))
        assert s == B.EPD_OK, (change, msg)


@pytest.mark.parametrize("change,status", [
    (dict(dtype=7), B.EPD_ERR_INVALID_ARG),
    (dict(norm=2), B.EPD_ERR_INVALID_ARG),
    (dict(act=-1), B.EPD_ERR_INVALID_ARG),
    (dict(heads=7), B.EPD_ERR_SHAPE),               # 1024 % 7 != 0
    (dict(tile_size=450), B.EPD_ERR_SHAPE),         # not a multiple of the patch
    (dict(hidden=0), B.EPD_ERR_SHAPE),
    (dict(max_tiles_per_call=0), B.EPD_ERR_SHAPE),
    (dict(tile_size=14 * 15), B.EPD_ERR_SHAPE),     # odd grid with pixel shuffle
    (dict(heads=4), B.EPD_ERR_UNSUPPORTED),         # head dim 256 in bf16 mode
    (dict(proj_out=4100), B.EPD_ERR_UNSUPPORTED),   # not a multiple of 8 in bf16 mode
])
def test_check_desc_rejects(change, status):
    d = wl.workload("c3").desc.replace(**change)
    s, msg = B.check_desc(d)
    assert s == status, msg
    assert msg
    assert B.weight_count(d) == status


def test_check_desc_caps_the_fp32_sequence_at_what_its_attention_kernel_holds_in_lds():
    d = wl.workload("c1").desc
    s, msg = B.check_desc(d.replace(tile_size=14 * 128))      # 16384 patches + head dim 64 floats > 64 KiB
    assert s == B.EPD_ERR_UNSUPPORTED and "fp32" in msg
    s, msg = B.check_desc(d.replace(tile_size=14 * 127))
    assert s == B.EPD_OK, msg


def test_check_offsets():
    assert B.check_offsets([0, 13, 26], 2, 26) == B.EPD_OK
    assert B.check_offsets([0, 3, 3, 9], 3, 9) == B.EPD_OK          # empty request is legal
    assert B.check_offsets([0], 0, 0) == B.EPD_OK
    assert B.check_offsets([1, 3], 1, 3) == B.EPD_ERR_OFFSETS       # must start at 0
    assert B.check_offsets([0, 5, 4], 2, 4) == B.EPD_ERR_OFFSETS    # decreasing
    assert B.check_offsets([0, 5], 1, 6) == B.EPD_ERR_OFFSETS       # does not cover the batch
    assert B.check_offsets(None, 1, 1) == B.EPD_ERR_INVALID_ARG
    assert B.check_offsets([0, 1], -1, 1) == B.EPD_ERR_OFFSETS


def test_create_rejects_bad_arguments_before_touching_a_device():
    lib = B.lib()
    d = B.desc_to_c(wl.workload("c1").desc)
    handle = ctypes.c_void_p(1234)
    assert lib.epd_create(ctypes.byref(d), None, None, ctypes.byref(handle)) == B.EPD_ERR_INVALID_ARG
    assert handle.value is None
    w = B.WeightsC(None, 3)
    assert lib.epd_create(ctypes.byref(d), ctypes.byref(w), None, ctypes.byref(handle)) == B.EPD_ERR_INVALID_ARG
    ptrs = (ctypes.c_void_p * 3)(16, 32, 48)
    w = B.WeightsC(ctypes.cast(ptrs, ctypes.POINTER(ctypes.c_void_p)), 3)       # wrong tensor count
    assert lib.epd_create(ctypes.byref(d), ctypes.byref(w), None, ctypes.byref(handle)) == B.EPD_ERR_INVALID_ARG
    assert b"expected" in lib.epd_last_error(None)
    assert lib.epd_create(ctypes.byref(d), ctypes.byref(w), None, None) == B.EPD_ERR_INVALID_ARG
    assert lib.epd_encode(None, None, 0, None, 0, None, None) == B.EPD_ERR_INVALID_ARG
    assert lib.epd_tokens_per_tile(None) == -1
    lib.epd_destroy(None)   # no-op


def test_host_side_under_address_and_undefined_behaviour_sanitizers():
    """The host half of the library (validation, block manager, dispatch arithmetic) built with
    -fsanitize=address,undefined (`python -m paper_2501_05460_amd.build --sanitize`) runs this file's and the
    block manager's tests clean.  Skipped when that build is not there (it is not part of the default build)."""
    import subprocess
    import sys
    from paper_2501_05460_amd import build as bld
    if not os.path.exists(bld.SAN_LIB) or os.environ.get("EPD_LIB_PATH"):
        pytest.skip("sanitizer build not present (or already running under it)")
    newest_source = max(os.path.getmtime(os.path.join(d, f)) for d in (bld.CSRC, os.path.join(ROOT, "include"))
                        for f in os.listdir(d))
    if os.path.getmtime(bld.SAN_LIB) < newest_source:
        pytest.skip("sanitizer build is older than the sources: run `python -m paper_2501_05460_amd.build --sanitize`")
    r = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi_host.py"), os.path.join(ROOT, "tests", "test_mm_cache_host.py")],
                       env=bld.sanitized_env(), capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; `bench.py --gpus N` with N > 1 (or a WORLD_SIZE above 1) says so and exits with a
    status of its own before anything touches a device."""
    import subprocess
    import sys
    bench = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py")
    r = subprocess.run([sys.executable, bench, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, bench], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and "one GPU" in r.stderr
