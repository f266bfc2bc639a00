"""The C-ABI library loads without a GPU, exports every declared symbol and rejects bad arguments on the host."""
import ctypes
import os
import re

import pytest

from paper_2211_14133_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "kfac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kfac_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    lib = binding.load()
    names = _declared_symbols()
    assert "kfac_curvature" in names and "kfac_invert" in names and "kfac_precondition" in names
    for n in names:
        assert hasattr(lib, n), n
        assert n in binding.SIGNATURES, n
    assert sorted(binding.SIGNATURES) == names


def test_version_and_status_strings():
    lib = binding.load()
    assert lib.kfac_version() >= 100
    seen = {lib.kfac_status_string(s) for s in range(5)}
    assert len(seen) == 5 and all(seen)


def test_workspace_queries_are_host_only():
    lib = binding.load()
    assert lib.kfac_invert_workspace(4096) >= 2 * 4096 * 4096 * 4
    assert lib.kfac_invert_workspace(0) == 0
    assert lib.kfac_precondition_workspace(1024, 4096) >= 1024 * 4096 * 4
    # a large factor needs no split, a small one does
    assert lib.kfac_curvature_workspace(4096, 4096, binding.KFAC_F32) == 0
    assert lib.kfac_curvature_workspace(4096, 768, binding.KFAC_F32) > 0


def test_bad_arguments_are_rejected_before_any_launch():
    lib = binding.load()
    ERR_ARG, ERR_UNSUP, ERR_WS = 1, 2, 3
    fake = ctypes.c_void_p(4096)  # never dereferenced on the host
    # null pointers
    assert lib.kfac_curvature(None, 0, 16, 8, 8, 1.0, 0.0, fake, 8, None, 0, None) == ERR_ARG
    assert lib.kfac_curvature(fake, 0, 16, 8, 8, 1.0, 0.0, None, 8, None, 0, None) == ERR_ARG
    # sizes and leading dimensions
    assert lib.kfac_curvature(fake, 0, 0, 8, 8, 1.0, 0.0, fake, 8, None, 0, None) == ERR_ARG
    assert lib.kfac_curvature(fake, 0, 16, -1, 8, 1.0, 0.0, fake, 8, None, 0, None) == ERR_ARG
    assert lib.kfac_curvature(fake, 0, 16, 8, 7, 1.0, 0.0, fake, 8, None, 0, None) == ERR_ARG
    assert lib.kfac_curvature(fake, 0, 16, 8, 8, 1.0, 0.0, fake, 7, None, 0, None) == ERR_ARG
    # dtype
    assert lib.kfac_curvature(fake, 7, 16, 8, 8, 1.0, 0.0, fake, 8, None, 0, None) == ERR_ARG
    # misaligned pointer
    assert lib.kfac_curvature(ctypes.c_void_p(4098), 0, 16, 8, 8, 1.0, 0.0, fake, 8, None, 0, None) == ERR_ARG
    # workspace needed (small factor -> split) but missing / too small / misaligned
    need = lib.kfac_curvature_workspace(4096, 768, 0)
    assert lib.kfac_curvature(fake, 0, 4096, 768, 768, 1.0, 0.0, fake, 768, None, 0, None) == ERR_WS
    assert lib.kfac_curvature(fake, 0, 4096, 768, 768, 1.0, 0.0, fake, 768, fake, need - 1, None) == ERR_WS
    assert lib.kfac_curvature(fake, 0, 4096, 768, 768, 1.0, 0.0, fake, 768, ctypes.c_void_p(4100), need + 8, None) == ERR_WS
    # inversion
    assert lib.kfac_invert(None, 8, 8, 0.1, fake, 8, fake, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_invert(fake, 8, 8, 0.1, fake, 8, None, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_invert(fake, 8, 8, 0.1, fake, 8, fake, fake, 1 << 20, None) == ERR_ARG  # inv aliases factor
    other = ctypes.c_void_p(8192)
    assert lib.kfac_invert(fake, 8, 4, 0.1, other, 8, fake, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_invert(fake, 8, 8, -1.0, other, 8, fake, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_invert(fake, 8, 8, 0.1, other, 8, fake, None, 0, None) == ERR_WS
    # precondition
    assert lib.kfac_precondition(None, 8, 8, fake, 4, 4, fake, 4, fake, 4, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_precondition(fake, 8, 8, fake, 4, 4, fake, 3, fake, 4, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_precondition(fake, 8, 8, fake, 4, 4, fake, 4, fake, 4, None, 0, None) == ERR_WS
    assert lib.kfac_precondition_grouped_f16x2(None, 1, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_precondition_grouped_f16x2(None, 0, None, 0, None) == 0
    assert lib.kfac_precondition_grouped_f16x2_workspace(None, 0) == 0
    assert lib.kfac_precondition_f16x2_prepare(None, 1, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_precondition_grouped_f16x2_prepared(None, 1, fake, 1 << 20, fake, 1 << 20, None) == ERR_ARG
    assert lib.kfac_precondition_f16x2_prepared_bytes(None, 0) == 0
    assert lib.kfac_precondition_grouped_f16x2_prepared_workspace(None, 0) == 0
    # empty groups are fine
    assert lib.kfac_curvature_grouped(None, 0, 0, 1.0, 0.0, None, 0, None) == 0
    assert lib.kfac_invert_batched(None, 0, 0.1, None, 0, None) == 0
    assert lib.kfac_precondition_grouped(None, 0, None, 0, None) == 0


def test_bf16_is_reported_unsupported_or_supported_consistently():
    lib = binding.load()
    fake = ctypes.c_void_p(4096)
    st = lib.kfac_curvature(fake, binding.KFAC_BF16, 16, 8, 8, 1.0, 0.0, None, 8, None, 0, None)
    assert st == 1  # null factor is an argument error whatever the dtype


def test_split_bf16_dtype_workspace_and_header_value():
    """KFAC_F32_BF16X3: the header's value is the binding's; its workspace holds three packed bfloat16 planes
    (2 bytes per element each, padded to 32 tokens and 256 columns), i.e. three times what KFAC_BF16 needs."""
    lib = binding.load()
    header = open(os.path.join(ROOT, "include", "kfac.h")).read()
    assert "KFAC_F32_BF16X3 = %d" % binding.KFAC_F32_BF16X3 in header
    for n, d in [(4096, 4096), (600, 5000), (1, 3584)]:
        need = lib.kfac_curvature_workspace(n, d, binding.KFAC_F32_BF16X3)
        plane = -(-n // 32) * 32 * (-(-d // 256) * 256) * 2
        assert need >= 3 * plane
        assert need == 3 * lib.kfac_curvature_workspace(n, d, binding.KFAC_BF16)
        # two float16 planes and one word per item for its largest magnitude
        need2 = lib.kfac_curvature_workspace(n, d, binding.KFAC_F32_F16X2)
        assert need2 == 2 * lib.kfac_curvature_workspace(n, d, binding.KFAC_BF16) + 256
    assert "KFAC_F32_F16X2 = %d" % binding.KFAC_F32_F16X2 in header
    dummy = ctypes.c_void_p(0x1000)
    assert lib.kfac_curvature(dummy, 4, 64, 64, 64, 1.0, 0.0, dummy, 64, None, 0, None) == 1
    assert lib.kfac_curvature(dummy, binding.KFAC_F32_F16X2, 64, 4096, 4096, 1.0, 0.0, dummy, 4096, None, 0, None) == 3
    assert lib.kfac_curvature(dummy, binding.KFAC_F32_BF16X3, 64, 4096, 4096, 1.0, 0.0, dummy, 4096, None, 0, None) == 3


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2211_14133_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("test oracle", ""), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2211_14133_amd" not in text and "kfac.h" not in text, f


def test_plan_and_host_functions_reject_bad_arguments():
    lib = binding.load()
    handle = ctypes.c_void_p()
    assert lib.kfac_invert_plan_create(None, 1, 0.1, None, 0, ctypes.byref(handle)) == 1
    assert handle.value is None
    assert lib.kfac_invert_plan_create(None, 0, 0.1, None, 0, None) == 1
    # an empty plan is valid and has no steps
    assert lib.kfac_invert_plan_create(None, 0, 0.1, None, 0, ctypes.byref(handle)) == 0
    assert lib.kfac_invert_plan_steps(handle) == 0 and lib.kfac_invert_plan_position(handle) == 0
    assert lib.kfac_invert_plan_run(handle, 5, None) == 0
    assert lib.kfac_invert_plan_step_flops(handle, 0) == -1.0
    assert lib.kfac_invert_plan_reset(handle) == 0
    lib.kfac_invert_plan_destroy(handle)
    assert lib.kfac_invert_plan_steps(None) == 0
    assert lib.kfac_invert_plan_run(None, 1, None) == 1
    assert lib.kfac_perf_model(1.0, 1.0, 1.0, 1.0, 0, 1.0, 1.0, 1.0, None) == 1
    assert lib.kfac_assign_work(0, None, None, 1.0, 0, None, None, None, None, None, None, None, None, None) == 1


def test_mfma_probe_rejects_bad_arguments():
    lib = binding.load()
    flops = ctypes.c_double(0.0)
    fake = ctypes.c_void_p(256)  # never dereferenced: every call below fails before a launch
    assert lib.kfac_mfma_probe(binding.KFAC_F32, 10, None, ctypes.byref(flops), None) == 1
    assert lib.kfac_mfma_probe(binding.KFAC_F32, 10, fake, None, None) == 1
    assert lib.kfac_mfma_probe(binding.KFAC_F32, 0, fake, ctypes.byref(flops), None) == 1
    assert lib.kfac_mfma_probe(7, 10, fake, ctypes.byref(flops), None) == 1
    assert lib.kfac_mfma_probe_data(binding.KFAC_BF16, 1, 10, None, ctypes.byref(flops), None) == 1
    assert lib.kfac_mfma_probe_data(binding.KFAC_F32_BF16X3, 1, 10, fake, ctypes.byref(flops), None) == 1


def test_header_is_plain_c_and_cxx():
    """The boundary is a C ABI: the header must compile on its own as C99 and as C++11."""
    import shutil
    import subprocess

    header = os.path.join(ROOT, "include", "kfac.h")
    for cc, flags in (("gcc", ["-std=c99", "-x", "c"]), ("g++", ["-std=c++11", "-x", "c++"])):
        if shutil.which(cc) is None:
            pytest.skip(cc + " not available")
        r = subprocess.run([cc, *flags, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", header],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_inversion_plans_are_built_on_the_host_for_every_size():
    """Recording a plan launches nothing, so the host side of the inversion (block structure, task
    dependencies, bounds of every operand, launch descriptors) runs here without a GPU: every size must
    give a plan whose steps are labelled and whose model cost is the d^3 of the three phases."""
    lib = binding.load()
    cases = [[1], [2], [127], [128], [129], [511, 513], [1024] * 5 + [4096, 640], [2049, 100], [4096] * 3, [8192],
             [96] * 80, [32640]]
    for ds in cases:
        n = len(ds)
        items = (binding.InvertItem * n)()
        base = 1 << 40  # made-up device addresses: nothing is dereferenced
        for i, d in enumerate(ds):
            items[i] = binding.InvertItem(base, d, d, base + 4 * d * d + 256, d, (1 << 39) + 4 * i)
            base += 8 * d * d + 4096
        need = lib.kfac_invert_batched_workspace(items, n)
        assert need >= sum(8 * d * d for d in ds)
        handle = ctypes.c_void_p()
        ws = ctypes.c_void_p(1 << 42)
        assert lib.kfac_invert_plan_create(items, n, 1e-3, ws, need - 256, ctypes.byref(handle)) == 3  # too small
        assert lib.kfac_invert_plan_create(items, n, 1e-3, ws, need, ctypes.byref(handle)) == 0, ds
        steps = lib.kfac_invert_plan_steps(handle)
        assert steps >= 3
        labels = [lib.kfac_invert_plan_step_label(handle, i) for i in range(steps)]
        assert all(lb for lb in labels) and labels[0] == b"copy + damping" and labels[-1] == b"inverse = W W^T"
        flops = sum(lib.kfac_invert_plan_step_flops(handle, i) for i in range(steps))
        want = sum(float(d) ** 3 for d in ds)
        if min(ds) >= 511:
            assert 0.98 * want <= flops <= 1.10 * want, (ds, flops / want)
        lib.kfac_invert_plan_destroy(handle)
    # one row more than the block indices can address
    items = (binding.InvertItem * 1)()
    items[0] = binding.InvertItem(1 << 40, 32641, 32641, 1 << 41, 32641, 1 << 39)
    handle = ctypes.c_void_p()
    need = lib.kfac_invert_batched_workspace(items, 1)
    assert lib.kfac_invert_plan_create(items, 1, 1e-3, ctypes.c_void_p(1 << 42), need, ctypes.byref(handle)) == 2
