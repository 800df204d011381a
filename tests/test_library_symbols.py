"""The built C-ABI libraries load and export every function that include/*.h declares: libpcm.so everything of
pcm.h plus the stage timer of pcm_measure.h, libpcm_measure.so the stand-alone matrix-core rate probe.

No GPU work is issued here: only host-side queries are called.
"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pcm.h")
MEASURE_HEADER = os.path.join(ROOT, "include", "pcm_measure.h")
LIB = os.path.join(ROOT, "paper_2605_16154_amd", "libpcm.so")
MEASURE_LIB = os.path.join(ROOT, "paper_2605_16154_amd", "libpcm_measure.so")


def _declared(header=HEADER):
    text = open(header).read()
    return sorted(set(re.findall(r"^PCM_API\s+[\w\s\*]+?\b((?:pcm|grpo)_\w+)\s*\(", text, flags=re.M)))


@pytest.fixture(scope="module")
def cdll():
    if not (os.path.exists(LIB) and os.path.exists(MEASURE_LIB)):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_four_calls():
    names = _declared()
    for need in ("pcm_score_phases", "pcm_update_keep_probs", "pcm_sample_chunks", "grpo_masked_actor_step"):
        assert need in names
    assert len(names) >= 12


def test_every_declared_symbol_is_exported(cdll):
    for name in _declared():
        assert hasattr(cdll, name), name
    measure = ctypes.CDLL(MEASURE_LIB)
    for name in _declared(MEASURE_HEADER):
        assert hasattr(measure if name == "pcm_measure_mfma_rate" else cdll, name), name


def test_training_header_has_no_measurement_exports_and_product_library_no_probe(cdll):
    # the calls of pcm.h never allocate or synchronise; the probe that does lives in its own library
    names = _declared()
    assert not [n for n in names if "measure" in n or "profile" in n]
    assert not hasattr(cdll, "pcm_measure_mfma_rate")
    assert "pcm_score_phases_static" in names


def test_host_side_queries(cdll):
    cdll.pcm_version.restype = ctypes.c_char_p
    assert b"pcm" in cdll.pcm_version()
    cdll.pcm_state_bytes.restype = ctypes.c_size_t
    assert cdll.pcm_state_bytes(5) == 16 + 24 * 5
    assert cdll.pcm_state_bytes(0) == 0 and cdll.pcm_state_bytes(65) == 0
    cdll.pcm_score_phases_workspace_bytes.restype = ctypes.c_size_t
    assert cdll.pcm_score_phases_workspace_bytes(8, 8, 64, 56, 5) >= 8 * 2 * 5 * 56 * 8
    q = cdll.grpo_masked_actor_step_workspace_bytes
    q.restype = ctypes.c_size_t
    assert q(96, 56, 256, 1024, 256, 0, 1) > q(96, 56, 256, 1024, 256, 0, 0) > 0
    assert q(768, 56, 4096, 11008, 256, 1, 1) > 768 * 56 * 11008 * 2 * 3
    assert q(768, 56, 4000, 11008, 256, 1, 1) == 0          # bf16 path needs d % 256 == 0
    cdll.pcm_status_string.restype = ctypes.c_char_p
    assert cdll.pcm_status_string(-2).startswith(b"workspace")


def test_null_and_range_arguments_are_rejected_on_the_host(cdll):
    # argument validation happens before any GPU call, so these run without a device
    assert cdll.pcm_state_init(None, 5, None) == -1
    assert cdll.pcm_score_phases(None, None, None, None, 1, 1, 1, 1, 1, ctypes.c_double(0.0), None, None, None,
                                 None, None, ctypes.c_size_t(0), None) == -1
    assert cdll.pcm_update_keep_probs(None, None, None, 5, ctypes.c_double(0.1), 5, None, None) == -1
    assert cdll.pcm_sample_chunks(None, None, None, None, 1, 1, 1, 1, ctypes.c_uint64(0), ctypes.c_uint64(0),
                                  None, None, None, None, ctypes.c_size_t(0), None) == -1


def test_optimizer_entry_validates_on_the_host(cdll):
    q = cdll.pcm_adamw_clip_step_workspace_bytes
    q.restype = ctypes.c_size_t
    numel = (ctypes.c_int64 * 2)(4096 * 3 + 1, 5)
    assert q(2, numel) >= 5 * 8                     # one fp64 partial per 4096-element chunk
    assert q(0, numel) == 0 and q(9, numel) == 0
    d = ctypes.c_double
    step = cdll.pcm_adamw_clip_step
    assert step(2, numel, None, None, None, None, None, ctypes.c_int64(1), d(1e-5), d(0.9), d(0.999), d(1e-8), d(0.0),
                d(2.0), None, None, ctypes.c_size_t(0), None) == -1


def test_header_is_valid_c_and_a_plain_c_client_links(cdll, tmp_path):
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    exe = tmp_path / "abi_check"
    lib_dir = os.path.dirname(LIB)
    cmd = [cc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "abi_check.c"), "-o", str(exe), "-L", lib_dir, "-l:libpcm.so",
           "-Wl,-rpath," + lib_dir]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "pcm" in r.stdout


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    import paper_2605_16154_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(b.PcmError):
        b.lib()
