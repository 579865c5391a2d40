"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and its host-only entry points validate their arguments (no GPU work)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spd.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2404_08856_amd import spd
    lib = ctypes.CDLL(spd.LIB_PATH)
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in spd.h but not exported"
    assert sorted(spd.EXPORTS) == names


def test_model_bytes_and_shape_validation():
    from paper_2404_08856_amd import spd, synth
    s = synth.SHAPES["llama7b"]
    cfg = spd.make_config(s, max_seqs=1, max_positions=1024)
    packed, kv, ws = spd.spd_model_bytes(cfg)
    # packed = bf16 matrices (same byte count as row-major: all dims divide the tile) + embed + gains
    assert packed >= s.streamed_weight_bytes() + s.vocab * s.d_model * 2
    assert packed < 1.01 * (s.streamed_weight_bytes() + s.vocab * s.d_model * 2)
    assert kv == s.n_layers * 2 * 1 * s.n_heads * 1024 * s.head_dim * 2
    assert ws > 0
    bad = spd.make_config(s, 1, 1024)
    bad.head_dim = 96
    with pytest.raises(spd.SpdError) as e:
        spd.spd_model_bytes(bad)
    assert e.value.code == spd.SPD_ERR_SHAPE and "head_dim" in str(e.value)
    bad = spd.make_config(s, 1, 1024)
    bad.d_model = 4100
    with pytest.raises(spd.SpdError):
        spd.spd_model_bytes(bad)
    # K not a multiple of 32 is padded per 16-row tile (tiny config: d_ffn = 688)
    t = synth.SHAPES["tiny_target"]
    p2, _, _ = spd.spd_model_bytes(spd.make_config(t, 1, 128))
    assert p2 > t.streamed_weight_bytes()


def test_accept_workspace_bytes_and_argument_checks():
    from paper_2404_08856_amd import spd
    assert spd.spd_accept_workspace_bytes(64, 4, 32000) == 64 * 9 * 16
    with pytest.raises(spd.SpdError) as e:
        spd.spd_accept_workspace_bytes(0, 4, 32000)
    assert e.value.code == spd.SPD_ERR_INVALID_ARG


def test_binding_fails_loudly_without_the_library(tmp_path):
    """No CPU fallback: a copy of the package without libspd.so cannot even be imported."""
    import shutil
    import subprocess
    import sys
    pkg = os.path.join(ROOT, "paper_2404_08856_amd")
    dst = tmp_path / "paper_2404_08856_amd"
    dst.mkdir()
    for name in ("__init__.py", "spd.py", "synth.py"):
        shutil.copy(os.path.join(pkg, name), dst / name)
    r = subprocess.run([sys.executable, "-c", "import paper_2404_08856_amd.spd"], cwd=tmp_path, capture_output=True, text=True,
                       timeout=300, env={**os.environ, "PYTHONPATH": str(tmp_path)})
    assert r.returncode != 0 and "ImportError" in r.stderr and "libspd.so is missing" in r.stderr


def test_product_does_not_import_the_oracle():
    """The oracle is test infrastructure: nothing under the package (or the bench's GPU path) imports it."""
    import re
    pkg = os.path.join(ROOT, "paper_2404_08856_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            text = open(os.path.join(pkg, name)).read()
            assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"from oracle import", bench)]
    assert len(uses) == 1 and "def cpu_baseline" in bench[:uses[0]] and "def side_configs" not in bench[:uses[0]]


def test_product_reads_no_environment_variables():
    """Kernel selection is fixed at model creation or set through spd_model_set_tuning: no hidden knobs."""
    csrc = os.path.join(ROOT, "paper_2404_08856_amd", "csrc")
    for name in os.listdir(csrc):
        if name.endswith((".hip", ".h")):
            assert "getenv" not in open(os.path.join(csrc, name)).read(), name


def test_null_handles_are_refused_by_every_entry_point():
    """Host-side argument validation: a NULL model (or buffer) is an error code and a message, never a crash."""
    from paper_2404_08856_amd import spd
    lib = ctypes.CDLL(spd.LIB_PATH)
    lib.spd_last_error.restype = ctypes.c_char_p
    null = ctypes.c_void_p(None)
    i32, f32, sz = ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    calls = {
        "spd_kv_set_len": (null, null, i32(1)),
        "spd_kv_get_len": (null, null, i32(1)),
        "spd_kv_lens_to_device": (null, null),
        "spd_kv_lens_from_device": (null, null),
        "spd_device_status": (null, null),
        "spd_kv_export": (null, i32(0), i32(0), i32(0), i32(1), null, null, null),
        "spd_prefill": (null, i32(0), null, i32(1), null, null),
        "spd_prefill_tokens": (null, i32(0), null, i32(1), null, null),
        "spd_verify_forward": (null, null, i32(1), i32(5), null, null),
        "spd_draft_step": (null, null, i32(1), i32(1), f32(1.0), null, null, null, null),
        "spd_draft_step_strided": (null, null, i32(1), i32(1), i32(1), f32(1.0), null, i32(1), null, sz(16), null, i32(1), null),
        "spd_speculative_accept": (null, null, null, null, i32(1), i32(4), i32(16), f32(1.0), ctypes.c_uint32(0), null, null, null, null, sz(0), null),
        "spd_speculative_accept_static": (null, null, null, null, i32(1), i32(4), i32(16), f32(1.0), ctypes.c_uint32(0), null, null, null, null),
        "spd_block_finish": (null, null, null, null, null, null, i32(1), i32(4), f32(1.0), null, null, null, null, i32(0), null, null, sz(0), null),
        "spd_trace_enable": (null, i32(1)),
        "spd_trace_read": (null, i32(8), null, null),
        "spd_model_set_tuning": (null, null),
        "spd_probe_read_chain": (null, sz(0), null, i32(1), i32(1), null, null, null, null),
    }
    for name, args in calls.items():
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int32
        rc = fn(*args)
        assert rc == spd.SPD_ERR_INVALID_ARG, (name, rc)
        assert lib.spd_last_error(), name
