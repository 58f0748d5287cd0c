"""The C-ABI library loads without a GPU and exports every symbol include/hata.h declares;
host-side validation (no kernel launch) behaves as the header says."""
import ctypes
import os
import re

import pytest

from paper_2506_02572_amd import hata

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="hata.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hata_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    lib = hata.load_library()
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in hata.h but not exported by libhata.so"
    assert sorted(hata.EXPORTS) == names


def test_trainer_symbols_are_exported_and_bound():
    from paper_2506_02572_amd import train
    lib = hata.load_library()
    names = [n for n in declared_symbols("hata_train.h") if n.startswith("hata_train_") and
             n not in ("hata_train_config", "hata_train_hparams", "hata_train_ctx")]
    assert sorted(names) == sorted(train.EXPORTS)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in hata_train.h but not exported by libhata.so"
    # host-side validation, no GPU needed
    train._lib()
    n = ctypes.c_size_t(0)
    assert lib.hata_train_workspace_bytes(ctypes.byref(train.hata_train_config(128, 128, 32768)), ctypes.byref(n)) == 0
    assert n.value > 256 * 128 * 128 * 4
    assert lib.hata_train_workspace_bytes(ctypes.byref(train.hata_train_config(128, 100, 10)), ctypes.byref(n)) == -2
    assert lib.hata_train_workspace_bytes(None, ctypes.byref(n)) == -1
    h = ctypes.c_void_p()
    assert lib.hata_train_create(ctypes.byref(h), ctypes.byref(train.hata_train_config(128, 128, 10)), None, 0) == -3
    assert lib.hata_train_step(None, None, None, None, 1, None, 1, None, None, None, None, None, None) == -1
    assert lib.hata_train_destroy(None) == 0


def test_strerror_and_workspace_validation():
    lib = hata.load_library()
    assert hata.strerror(0) == "ok"
    assert "gave up" in hata.strerror(-5)
    for code in (-1, -2, -3, -4, -5, -99):
        assert hata.strerror(code)
    n = ctypes.c_size_t(0)
    good = hata.hata_config(1, 32, 8, 128, 128, 32768, 512, 8 * 32768 * 128, 32768 * 128, 128)
    assert lib.hata_workspace_bytes(ctypes.byref(good), ctypes.byref(n)) == 0
    # scores (2 B/key) + chunk histograms + idx + partials: well under 4 MB for this shape
    assert 8 * 32768 * 2 < n.value < 4 << 20
    bad = [
        hata.hata_config(1, 32, 8, 64, 128, 32768, 512, 1, 1, 128),         # d != 128
        hata.hata_config(1, 32, 7, 128, 128, 32768, 512, 1 << 20, 1 << 20, 128),  # Hq % Hkv
        hata.hata_config(1, 32, 8, 128, 100, 32768, 512, 1 << 20, 1 << 20, 128),  # r % 32
        hata.hata_config(1, 32, 8, 128, 128, 256, 512, 1 << 20, 1 << 20, 128),    # k_max > L_cap
        hata.hata_config(1, 32, 8, 128, 128, 32768, 512, 1 << 20, 1 << 20, 100),  # row stride < d
        hata.hata_config(0, 32, 8, 128, 128, 32768, 512, 1 << 20, 1 << 20, 128),  # B_max < 1
    ]
    for cfg in bad:
        assert lib.hata_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)) < 0
    assert lib.hata_workspace_bytes(None, ctypes.byref(n)) == -1
    # create refuses a missing workspace before touching the device
    h = ctypes.c_void_p()
    assert lib.hata_create(ctypes.byref(h), ctypes.byref(good), None, 0) == -3
    assert not h.value
    # calls on a NULL context are rejected, nothing is launched
    assert lib.hata_encode_query(None, None, None, 1, None, None) == -1
    assert lib.hata_decode_step(None, None, None, None, None, None, None, None, 1, 0, 1.0, None, None, None) == -1
    assert lib.hata_decode_step_paged(None, None, None, None, None, None, None, 4, 256, 4, None, None, 1, 0, 1.0,
                                      None, None, None) == -1
    assert lib.hata_prefill_write_paged(None, None, None, None, None, 1, 16, None, None, None, None, 4, 256, 4,
                                        None, None) == -1
    assert lib.hata_prefill_write(None, None, None, None, None, 1, 16, None, None, None, None, None) == -1
    assert lib.hata_step_plan(None, 1, None, None, None) == -1
    assert lib.hata_set_step_mode(None, 0) == -1
    assert lib.hata_set_wait_limit(None, 0) == -1
    assert lib.hata_keep_step_scores(None, 0) == -1
    assert lib.hata_check(None, None) == -1
    assert lib.hata_host_device_pointer(None, None) == -1
    assert lib.hata_destroy(None) == 0


def test_binding_has_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(hata.HataError):
        hata.Context(1, 32, 8, 128, 128, 2048, 128)


def test_probe_rejects_bad_arguments_without_a_device():
    lib = hata.load_library()
    assert lib.hata_probe_mfma_stream(None, 1 << 30, 16, 3, None) == -1      # no buffer
    assert lib.hata_probe_mfma_stream(ctypes.c_void_p(4096), 1 << 20, 16, 3, None) == -1   # below 4 MiB
    assert lib.hata_probe_mfma_stream(ctypes.c_void_p(4096 + 8), 1 << 30, 16, 3, None) == -1  # misaligned
    assert lib.hata_probe_mfma_stream(ctypes.c_void_p(4096), 1 << 30, 16, 0, None) == -1   # no mode bit
    assert lib.hata_probe_mfma_stream(ctypes.c_void_p(4096), 1 << 30, -1, 3, None) == -1

