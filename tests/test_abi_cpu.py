"""CPU-only checks of the C-ABI: the library loads, exports what include/dn.h declares, and validates
arguments on the host before touching a device (no compute is launched here)."""
import ctypes
import os
import re

import pytest

from paper_1802_00130_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_1802_00130_amd import build
        build.build_lib(verbose=False)
    return binding.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert "dn_gn_matvec" in names and "dn_cg" in names and len(names) >= 18
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def _create(lib, dims, C=1.0, l=100, s=10):
    h = ctypes.c_void_p()
    arr = (ctypes.c_int * len(dims))(*dims)
    rc = lib.dn_create(ctypes.byref(h), len(dims) - 1, arr, C, l, s)
    return rc, h


def test_create_validation_and_sizes(lib):
    rc, h = _create(lib, (784, 300, 300, 10), l=60000, s=3000)
    assert rc == 0 and lib.dn_num_params(h) == 328810
    # workspace holds at least the stored blocks |S| n_L sum_{m<L} n_m and the activations for l rows
    need = 4 * (3000 * 10 * 600 + 60000 * 610)
    assert lib.dn_workspace_bytes(h) >= need
    lib.dn_destroy(h)
    assert _create(lib, (4, 0, 2))[0] == -1
    assert _create(lib, (4, 2), C=0.0)[0] == -1
    assert _create(lib, (4, 2), l=0)[0] == -1
    assert _create(lib, (4,))[0] == -1
    assert _create(lib, tuple([3] * 11))[0] == -1
    assert lib.dn_create(None, 1, (ctypes.c_int * 2)(2, 2), 1.0, 1, 1) == -1
    assert lib.dn_num_params(None) == 0 and lib.dn_workspace_bytes(None) == 0


def test_call_order_and_argument_errors(lib):
    rc, h = _create(lib, (6, 5, 3))
    assert rc == 0
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every call below fails validation first
    f = ctypes.c_double()
    it = ctypes.c_int()
    assert lib.dn_forward(h, fake, fake, fake, 10, ctypes.byref(f), None) == -3      # not bound
    assert lib.dn_bind(h, None, 1 << 30, None) == -1
    assert lib.dn_bind(h, ctypes.c_void_p(0x1001), 1 << 30, None) == -1              # misaligned
    assert lib.dn_bind(h, fake, 16, None) == -2                                      # too small
    assert lib.dn_bind(h, fake, lib.dn_workspace_bytes(h), None) == 0
    assert lib.dn_forward(h, None, fake, fake, 10, ctypes.byref(f), None) == -1
    assert lib.dn_forward(h, fake, fake, fake, 0, ctypes.byref(f), None) == -1
    assert lib.dn_grad(h, fake, fake, fake, 0, fake, None) == -1
    assert lib.dn_jacobian_prep(h, fake, fake, 100, fake, 11) == -1                  # s > s_max
    assert lib.dn_gn_matvec(h, fake, fake, 0) == -3                                  # no Jacobian prepared
    assert lib.dn_gn_matvec(h, fake, fake, 5) == -1
    assert lib.dn_gn_matvec_rop(h, fake, fake) == -3 and lib.dn_gn_matvec_rop(h, None, fake) == -1
    assert lib.dn_cg(h, fake, 1.0, 0.0, 5, 0, fake, ctypes.byref(it), ctypes.byref(f)) == -3
    assert lib.dn_cg(h, fake, -1.0, 0.0, 5, 0, fake, ctypes.byref(it), ctypes.byref(f)) == -1
    assert lib.dn_cg_sync(h, fake, 1.0, 1e-3, 5, 1, 0, 50.0, fake, ctypes.byref(it), ctypes.byref(f)) == -3
    assert lib.dn_cg_sync(h, fake, 1.0, 1e-3, 5, 1, 0, 0.0, fake, ctypes.byref(it), ctypes.byref(f)) == -1
    assert lib.dn_cg_sync(h, fake, 1.0, 1e-3, 5, 1, -1, 50.0, fake, ctypes.byref(it), ctypes.byref(f)) == -1
    assert lib.dn_cg_sync(h, fake, 1.0, 1e-3, 5, 0, 0, 50.0, fake, ctypes.byref(it), ctypes.byref(f)) == -1   # full mode
    assert lib.dn_gn_matvec(h, fake, fake, 2) == -3                                  # no Jacobian / no split structure
    assert lib.dn_num_partitions(h) == 0
    assert lib.dn_set_split(h, (ctypes.c_int * 3)(1, 6, 1)) == -1                    # more groups than allowed / neurons
    assert lib.dn_set_split(h, (ctypes.c_int * 3)(0, 1, 1)) == -1
    assert lib.dn_set_split(h, None) == -1
    assert lib.dn_jacobian_read(h, 2, fake) == -1
    assert lib.dn_jacobian_read(h, 1, fake) == -3
    prm = binding.NewtonParams(1.0, 1e-3, 1e-4, 1e-5, 2.0 / 3.0, 1.5, 10, 0, 1, 30, 0, 0.0)
    st = binding.NewtonStats()
    args = (h, fake, fake, fake, 10, fake, 5, fake)
    for field, bad in (("eta", 0.0), ("eta", 1.0), ("drop", 0.0), ("boost", 0.5), ("cg_max", 0), ("mode", 7),
                       ("max_trials", 0), ("lam", -1.0), ("cg_min", -1), ("r_percent", 101.0)):
        good = getattr(prm, field)
        setattr(prm, field, bad)
        assert lib.dn_newton_step(*args, ctypes.byref(prm), ctypes.byref(st)) == -1, field
        setattr(prm, field, good)
    assert lib.dn_newton_step(h, fake, fake, fake, 10, fake, 11, fake, ctypes.byref(prm), ctypes.byref(st)) == -1
    assert lib.dn_newton_step(h, fake, fake, fake, 10, fake, 5, fake, None, ctypes.byref(st)) == -1
    assert lib.dn_set_stream_passes(h, 1) == -1 and lib.dn_set_stream_passes(h, 2) == 0
    assert lib.dn_set_stream_passes(None, 0) == -1 and lib.dn_set_spin_limit(None, 5) == -1
    assert lib.dn_set_spin_limit(h, 5) == 0
    assert lib.dn_strerror(-6).decode().startswith("a bounded wait")
    assert lib.dn_strerror(-2).decode() == "workspace too small"
    assert lib.dn_profile_num_classes() >= 10 and lib.dn_profile_class_name(0).decode() == "gemm_forward"
    lib.dn_destroy(h)


def test_forward_static_validates_on_the_host(lib):
    """The entry point that allocates nothing checks its arguments and the size of the problem against its fixed
    scratch before it touches a device."""
    fake = ctypes.c_void_p(0x1000)
    f = ctypes.c_double()
    dims = (ctypes.c_int * 4)(784, 300, 300, 10)
    call = lambda L, d, C, th, l: lib.dn_forward_static(L, d, C, th, fake, fake, l, None, ctypes.byref(f), None)
    assert call(3, dims, 1.0, fake, 20000) == -7        # 20000 rows x 612 floats > 32 MiB
    assert call(3, dims, 0.0, fake, 20) == -1
    assert call(3, dims, 1.0, None, 20) == -1
    assert call(3, dims, 1.0, fake, 0) == -1
    assert call(0, dims, 1.0, fake, 20) == -1
    assert call(3, None, 1.0, fake, 20) == -1
    assert lib.dn_forward_static(3, dims, 1.0, fake, fake, fake, 20, None, None, None) == -1
    assert lib.dn_strerror(-7).decode().startswith("problem exceeds")


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The library's host side compiled with -fsanitize=address,undefined (host code only: every -fsanitize= option
    directly after an -Xarch_host; the device code is compiled as usual and never runs here) and driven through
    the validation, planning and create/destroy paths by tests/abi_host_driver.cpp.  The driver checks the
    return codes; the sanitizers abort on a bad access, on undefined behaviour and on a leak."""
    import subprocess
    from paper_1802_00130_amd import build
    exe = tmp_path / "abi_host_asan"
    cmd = [build.hipcc_path(), "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-o", str(exe), os.path.join(build.CSRC, "dn_lib.hip"), os.path.join(ROOT, "tests", "abi_host_driver.cpp")]
    subprocess.run(cmd, check=True, capture_output=True, timeout=600)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120, env=env)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "host driver ok" in out.stdout


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message before touching anything (this build is single-GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=60)
    assert out.returncode == 2 and "ONE GPU" in out.stderr and out.stdout.strip() == ""


def test_product_plan_fits_the_workspace_for_every_subsample_size(lib):
    """The slice count of the sums over samples is not monotone in the number of samples; whatever it is for
    1 <= s <= s_max, its partial sums must fit the workspace the context asked for (small l_max, so that the
    gradient's plans do not hide the product's)."""
    for dims, l_max, s_max in (((3072, 1000, 500, 10), 500, 2500), ((784, 300, 300, 10), 300, 3000),
                               ((64, 40, 7), 10, 5000), ((200, 300, 260, 10), 50, 1777),
                               ((2048, 2000, 2000, 2000, 100), 10, 5000)):
        rc, h = _create(lib, dims, l=l_max, s=s_max)
        assert rc == 0
        counts = [lib.dn_product_slices(h, s) for s in range(1, s_max + 1)]
        assert min(counts) >= 1, (dims, counts.index(min(counts)) + 1)
        assert lib.dn_product_slices(h, 0) == -1 and lib.dn_product_slices(h, s_max + 1) == -1
        # the count is a step function of s that goes up and down (it follows how the work-groups fill the chip)
        assert len(set(counts)) >= 2
        lib.dn_destroy(h)
    assert lib.dn_product_slices(None, 1) == -1


def test_large_tiles_are_chosen_for_whole_rounds_only(lib):
    """Host logic of the tile engine: 128 x 128 tiles need at least 512 tiles that fill whole rounds of 256 and lose
    little to padding; a grouped launch may send its large problems through them and the rest through small tiles."""
    import ctypes

    def plan(*problems):
        n = len(problems)
        arr = lambda k: (ctypes.c_int * n)(*[p[k] for p in problems])
        large = (ctypes.c_int * n)()
        rc = lib.dn_gemm_large_tiles(n, arr(0), arr(1), arr(2), large)
        return rc, list(large)

    assert plan((200000, 4096, 4096)) == (1, [1])                  # forward pass of the largest configuration
    assert plan((2000000, 4096, 4096)) == (1, [1])                 # its sweeps over the stored blocks
    assert plan((100000, 2000, 2048)) == (1, [1])
    assert plan((2000, 4096, 4096)) == (1, [1])                    # 512 tiles: two rounds exactly
    assert plan((5000, 2000, 2048)) == (0, [0])                    # 640 tiles: two and a half rounds
    assert plan((3000, 300, 784)) == (0, [0])                      # too few tiles
    assert plan((60000, 300, 784)) == (0, [0])                     # 300 columns: 384 with large tiles, 320 with small
    # inner sums of the largest configuration: four layers of 512 large tiles, the narrow last layer on small tiles
    assert plan(*([(2000, 4096, 4096)] * 4 + [(2000, 1000, 4096)])) == (4, [1, 1, 1, 1, 0])
    # a group that passes as a whole stays whole
    assert plan((4096, 4097, 2000), (4096, 4097, 2000), (4096, 4097, 2000), (4096, 4097, 2000), (1000, 4097, 2000))[0] == 5
    # argument checks
    one = (ctypes.c_int * 1)(64)
    assert lib.dn_gemm_large_tiles(0, one, one, one, one) == -1
    assert lib.dn_gemm_large_tiles(9, one, one, one, one) == -1
    assert lib.dn_gemm_large_tiles(1, None, one, one, one) == -1
    zero = (ctypes.c_int * 1)(0)
    assert lib.dn_gemm_large_tiles(1, zero, one, one, one) == -1
