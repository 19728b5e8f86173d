"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
logic (argument validation, workspace sizing, status strings) behaves without a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2502_16982_amd import binding as b
    if not os.path.exists(b.library_path()):
        from paper_2502_16982_amd import build
        build.build_library()
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "muon.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(muon_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree(binding):
    assert declared_functions() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol(binding):
    L = binding.lib()
    for name in declared_functions():
        assert hasattr(L, name), name


def test_struct_layout_matches_header(binding):
    assert C.sizeof(binding.muon_param) == 3 * 8 + 2 * 8 + 2 * 4
    assert C.sizeof(binding.muon_hparams) == 8 * 8 + 4 * 4 + 8 + 8


def test_default_hparams_are_the_papers(binding):
    hp = binding.default_hparams()
    assert (hp.a, hp.b, hp.c) == (3.4445, -4.7750, 2.0315)
    assert hp.momentum == 0.95 and hp.ns_steps == 5 and hp.rms_scale == 0.2 and hp.nesterov == 1
    assert hp.scale_mode == binding.MUON_SCALE_ADJUSTED_LR and hp.reserved == 0 and hp.hidden_size == 0.0


def test_status_strings(binding):
    L = binding.lib()
    seen = set()
    for code in range(0, -10, -1):
        s = L.muon_status_string(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 10
    assert L.muon_status_string(-99).decode() == "unknown status"


def test_workspace_bytes_validation(binding):
    L = binding.lib()
    out = C.c_size_t(0)
    p = binding.param_array([(128, 256)], [0], [0])
    assert L.muon_workspace_bytes(None, 1, 1, 0, C.byref(out)) == -1
    assert L.muon_workspace_bytes(p, 0, 1, 0, C.byref(out)) == -1
    assert L.muon_workspace_bytes(p, 1, 1, 0, None) == -1
    assert L.muon_workspace_bytes(p, 1, 7, 0, C.byref(out)) == -2
    assert L.muon_workspace_bytes(p, 1, 4, 0, C.byref(out)) == -2
    bad = binding.param_array([(8, 8)], [binding.MUON_BF16X2], [0])      # the split forms are no buffer dtypes
    assert L.muon_workspace_bytes(bad, 1, 1, 0, C.byref(out)) == -2
    bad = binding.param_array([(0, 256)], [0], [0])
    assert L.muon_workspace_bytes(bad, 1, 1, 0, C.byref(out)) == -1
    bad = binding.param_array([(8, 8)], [5], [0])
    assert L.muon_workspace_bytes(bad, 1, 1, 0, C.byref(out)) == -2
    huge = binding.param_array([(2 ** 21, 8)], [0], [0])
    assert L.muon_workspace_bytes(huge, 1, 1, 0, C.byref(out)) == -1


def test_workspace_bytes_scale_with_dtype_and_cap(binding):
    shapes = [(1024, 1024)] * 4 + [(1024, 4096), (4096, 1024)]
    p = binding.param_array(shapes, [1] * 6, [1] * 6)
    bf = binding.muon_workspace_bytes(p, 6, binding.MUON_BF16)
    f32 = binding.muon_workspace_bytes(p, 6, binding.MUON_F32)
    # temporaries per matrix: fp32 path 3 m*n + 2 m*m elements (X, two transposes, A, B); bf16 path 2 m*n + 2 m*m, plus
    # one more m*n for matrices that are iterated on their transpose (rows > cols)
    elems32 = sum(3 * a * b + 2 * min(a, b) ** 2 for a, b in shapes)
    elems16 = sum((3 if a > b else 2) * a * b + 2 * min(a, b) ** 2 for a, b in shapes)
    assert bf >= 2 * elems16 and bf < 2 * elems16 * 1.2 + (1 << 22)
    assert f32 >= 4 * elems32 and f32 < 4 * elems32 * 1.2 + (1 << 22)
    capped = binding.muon_workspace_bytes(p, 6, binding.MUON_BF16, max_bytes=bf // 3)
    assert capped < bf and capped % 256 == 0
    # the split forms keep two / three bf16 planes of every temporary
    for planes, code in ((2, binding.MUON_BF16X2), (3, binding.MUON_BF16X3)):
        sp = binding.muon_workspace_bytes(p, 6, code)
        assert sp >= planes * 2 * elems16 and sp < planes * 2 * elems16 * 1.2 + (1 << 22)
    tiny = binding.muon_workspace_bytes(p, 6, binding.MUON_BF16, max_bytes=1)
    one = 2 * (3 * 1024 * 4096 + 2 * 1024 * 1024)     # the largest single matrix is the transposed 4096 x 1024
    assert one <= tiny < one + (1 << 22)


def test_init_rejects_bad_arguments_before_touching_the_device(binding):
    L = binding.lib()
    ctx = C.c_void_p(None)
    p = binding.param_array([(128, 256)], [0], [0])
    assert L.muon_init(None, p, 1, 1, C.c_void_p(256), 1 << 30) == -1
    assert L.muon_init(C.byref(ctx), p, 1, 1, None, 1 << 30) == -1
    assert L.muon_init(C.byref(ctx), p, 1, 1, C.c_void_p(257), 1 << 30) == -7
    assert L.muon_init(C.byref(ctx), p, 1, 1, C.c_void_p(256), 16) == -4
    assert L.muon_init(C.byref(ctx), p, 1, 9, C.c_void_p(256), 1 << 30) == -2
    assert ctx.value is None
    assert L.muon_step(None, p, 1, C.byref(binding.default_hparams()), None, None) == -1
    assert L.muon_plan_chunks(None) == -1
    L.muon_destroy(None)  # no-op


def test_missing_library_fails_loudly(binding, monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "library_path", lambda: str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.lib()


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_16982_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"(from\s+oracle|import\s+oracle|oracle\.|oracle/|muon_oracle)", text), f
    bench = open(os.path.join(ROOT, "bench.py")).read() if os.path.exists(os.path.join(ROOT, "bench.py")) else ""
    # bench may use the oracle only for its cpu_baseline leg
    for line in bench.splitlines():
        if "oracle" in line and "import" in line:
            assert "cpu_baseline" in bench


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message and a non-zero status before touching any device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    proc = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                          timeout=120)
    assert proc.returncode != 0
    assert "one GPU" in proc.stderr
    assert proc.stdout.strip() == ""


def test_schedule_helper_builds_a_host_array(binding):
    hp = binding.default_hparams(coeff_schedule=[(1.0, 2.0, 3.0), (4.0, 5.0, 6.0)])
    assert hp.ns_steps == 2
    assert [hp.coeff_schedule[i] for i in range(6)] == [1.0, 2.0, 3.0, 4.0, 5.0, 6.0]
    binding.set_coeff_schedule(hp, None)
    assert not hp.coeff_schedule
    with pytest.raises(ValueError):
        binding.default_hparams(coeff_schedule=[(1.0, 2.0)])
