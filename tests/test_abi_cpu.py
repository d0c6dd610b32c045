"""CPU-only checks of the C-ABI library and the host-side helpers (no compute calls)."""
import ctypes
import os
import re

import numpy as np

from paper_2605_10793_amd import binding, inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "conqur.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conqur_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names
    assert lib.conqur_version().decode().startswith("conqur-gfx950")


def test_config_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "conqur.h")).read()
    body = text[text.index("typedef struct {", text.index("conqur_dtype;")):text.index("} conqur_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:uint32_t|int32_t|float|void\*)\s+([a-z_]+);", body)
    assert fields == [f[0] for f in binding.Config._fields_]
    assert ctypes.sizeof(binding.Config) == 10 * 4 + 8   # ten 32-bit fields, one pointer


def test_stats_structs_match_header_field_order():
    text = open(os.path.join(ROOT, "include", "conqur.h")).read()
    for cname, cls in (("conqur_batch_stats", binding.BatchStats), ("conqur_update_stats", binding.UpdateStats)):
        end = text.index("} %s;" % cname)
        body = text[text.rindex("typedef struct {", 0, end):end]
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        fields = re.findall(r"\b(?:uint64_t|uint32_t|double)\s+([a-z_0-9]+);", body)
        assert fields == [f[0] for f in cls._fields_], cname
    assert ctypes.sizeof(binding.BatchStats) == 32 and ctypes.sizeof(binding.UpdateStats) == 64


def test_binding_holds_no_method_arithmetic():
    """The binding marshals arguments; Eq. 1 (the objective) comes from the library's conqur_batch_stats."""
    src = open(os.path.join(ROOT, "paper_2605_10793_amd", "binding.py")).read()
    assert "sqrt" not in src


def test_oversized_contexts_are_rejected_at_init():
    lib = binding.load()
    out = ctypes.c_void_p()
    R0 = np.eye(16, dtype=np.float32)
    big = binding.Config(8192, 1, binding.BF16, 1 << 20, 0.0, 0.0, 0, 0, 0, 0, None)   # 8192 * 2^20 operand elements
    assert lib.conqur_init(ctypes.byref(big), R0.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out)) == binding.EINVAL


def test_null_arguments_are_rejected_without_a_device():
    lib = binding.load()
    out = ctypes.c_void_p()
    assert lib.conqur_init(None, None, ctypes.byref(out)) == binding.EINVAL
    assert lib.conqur_step_batch(None, None, 1, 1) == binding.EINVAL
    assert lib.conqur_update_rotation(None, None) == binding.EINVAL
    lib.conqur_destroy(None)
    bad = binding.Config(60, 1, binding.BF16, 8, 0.0, 0.0, 0, 0, 0, 0, None)     # dh % 16 != 0
    R0 = np.eye(60, dtype=np.float32)
    assert lib.conqur_init(ctypes.byref(bad), R0.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out)) == binding.EINVAL
    bad = binding.Config(64, 1, 7, 8, 0.0, 0.0, 0, 0, 0, 0, None)                # unknown dtype
    assert lib.conqur_init(ctypes.byref(bad), R0.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out)) == binding.EINVAL
    bad = binding.Config(64, 1, binding.BF16, 8, 0.0, 0.0, 0, 3, 0, 0, None)     # polar_precision > 2
    assert lib.conqur_init(ctypes.byref(bad), R0.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out)) == binding.EINVAL
    bad = binding.Config(64, 1, binding.BF16, 8, 0.0, 0.0, 0, 0, 2, 0, None)     # polar_verify > 1
    assert lib.conqur_init(ctypes.byref(bad), R0.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out)) == binding.EINVAL


def test_input_streams_are_reproducible_and_shaped():
    for name, w in I.WORKLOADS.items():
        a = I.batch(w, 1, 32)
        b = I.batch(w, 1, 32)
        assert a.shape == (32, w.d) and a.dtype == np.float32 and np.array_equal(a, b)
        assert not np.array_equal(a, I.batch(w, 2, 32))
        if w.dtype == "bf16":
            assert np.array_equal(a, I.round_to_bf16(a))
            assert I.bf16_bits(a).dtype == np.uint16
    w = I.WORKLOADS["c3"]
    s = I.channel_scales(w)
    assert (s > 15).sum() == w.n_outliers                     # outlier channels x100 on log-normal(0, 0.5) scales
    w4 = I.WORKLOADS["c4"]
    R0 = I.initial_rotation(w4)
    assert R0.shape == (32, 128, 128)
    assert np.abs(R0[5].T.astype(np.float64) @ R0[5] - np.eye(128)).max() < 1e-5


def test_build_reports_register_spills():
    from paper_2605_10793_amd import build
    remarks = ("a.hip:1:1: remark: Function Name: kern_a [-Rpass-analysis=kernel-resource-usage]\n"
               "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
               "a.hip:9:1: remark: Function Name: kern_b [-Rpass-analysis=kernel-resource-usage]\n"
               "a.hip:9:1: remark:     ScratchSize [bytes/lane]: 576 [-Rpass-analysis=kernel-resource-usage]\n")
    assert build.kernels_with_scratch(remarks) == [("kern_b", 576)]
