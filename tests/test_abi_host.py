"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and argument validation returns the documented status codes."""
import ctypes
import os
import re

import pytest

from paper_2604_05426_amd import binding as ml

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "multi_lora.h")).read()
    declared = set(re.findall(r"\b(multi_lora_[a-z_]+)\s*\(", header))
    assert declared == set(ml.EXPORTS)
    L = ml.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert ml.version() == "0.1"


def test_header_constants_match_binding():
    header = open(os.path.join(ROOT, "include", "multi_lora.h")).read()
    for name, val in re.findall(r"(MLORA_ERR_[A-Z]+|MLORA_OK)\s*=\s*(-?\d+)", header):
        assert ml.STATUS_NAMES[int(val)] == name
    assert int(re.search(r"#define MLORA_MAX_RANK (\d+)", header).group(1)) == ml.MAX_RANK
    assert int(re.search(r"#define MLORA_MAX_ADAPTERS (\d+)", header).group(1)) == ml.MAX_ADAPTERS


V = ml.multi_lora_validate


def test_validate_accepts_legal_inputs():
    assert V(ml.BF16, 10, 8, 8, 2, [4, 0], [1.0, 2.0], [0, 4, 10]) == 0
    assert V(ml.F32, 0, 1, 1, 0, [], [], [0]) == 0            # no tokens, no adapters
    assert V(ml.BF16, 300, 8, 8, 0, None, None, None) == 0    # no adapters: all rows plain X W, metadata not read
    assert V(ml.F32, 5, 3, 7, 3, [1, 128, 2], [1, 1, 1], [0, 0, 5, 5]) == 0   # empty segments


@pytest.mark.parametrize("args,code", [
    ((7, 10, 8, 8, 1, [4], [1.0], [0, 10]), -5),                    # dtype
    ((ml.F32, -1, 8, 8, 0, [], [], [0]), -2),                       # T
    ((ml.F32, 10, 0, 8, 1, [4], [1.0], [0, 10]), -2),               # k
    ((ml.F32, 10, 8, 8, 5000, [1] * 5000, [1.0] * 5000, [0] * 5001), -2),  # N
    ((ml.F32, 10, 8, 8, 1, [4], [1.0], [1, 10]), -3),               # off[0] != 0
    ((ml.F32, 10, 8, 8, 2, [4, 4], [1.0, 1.0], [0, 6, 5]), -3),     # decreasing (overlap)
    ((ml.F32, 10, 8, 8, 1, [4], [1.0], [0, 9]), -3),                # off[N] != T
    ((ml.F32, 10, 8, 8, 1, [129], [1.0], [0, 10]), -4),             # rank too big
    ((ml.F32, 10, 8, 8, 1, [-1], [1.0], [0, 10]), -4),
    ((ml.F32, 10, 8, 8, 1, [4], [float("nan")], [0, 10]), -10),     # scale
    ((ml.F32, 10, 8, 8, 1, [4], [float("inf")], [0, 10]), -10),
])
def test_validate_rejects(args, code):
    assert V(*args) == code
    assert ml.last_error() != ""


def test_validate_null_pointers():
    assert V(ml.F32, 10, 8, 8, 1, None, [1.0], [0, 10]) == -1
    assert V(ml.F32, 10, 8, 8, 1, [4], [1.0], None) == -1


def test_plan_create_reports_errors_before_touching_the_gpu():
    with pytest.raises(ml.MultiLoraError) as e:
        ml.Plan(ml.BF16, 10, 8, 8, [4], [1.0], [0, 9])
    assert e.value.status == -3
    L = ml.lib()
    assert L.multi_lora_plan_destroy(None) == 0
    assert L.multi_lora_workspace_bytes(None) == 0
    assert L.multi_lora_fwd(None, None, None, None, None, None, None, None, 0, None) == -1
    assert L.multi_lora_bwd(None, None, None, None, None, None, None, None, None, None, None, 0, None) == -1


def test_header_is_plain_c(tmp_path):
    """include/multi_lora.h is a C header: it must compile as C99 on its own, with warnings as errors."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text('#include "multi_lora.h"\n'
                   'int main(void) { mlora_monitor_params p; mlora_admission_params q; (void)p; (void)q;\n'
                   '                 return multi_lora_plan_destroy(0) == MLORA_OK ? 0 : 1; }\n')
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
