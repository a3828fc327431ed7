"""The C-ABI library loads and exports every symbol include/rama.h declares (no GPU needed)."""
import ctypes as C
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rama.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rama_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    from paper_2109_01838_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2109_01838_amd import build
        build.build_hip()
    lib = binding.load_library()
    names = declared_symbols()
    assert {"rama_create", "rama_destroy", "rama_last_error", "rama_find_conflicted_cycles",
            "rama_message_passing", "rama_dual_rounds", "rama_contract", "rama_solve"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(binding.EXPORTS)


def test_params_default_and_struct_layout():
    from paper_2109_01838_amd import binding
    p = binding.default_params()
    assert (p.max_cycle_len_first, p.max_cycle_len_later, p.mp_iters_first, p.mp_iters_later) == (5, 3, 10, 5)
    assert p.matching_rounds_cap == 32 and p.contract_threshold == 0.0 and p.max_rounds == 0
    assert abs(p.forest_ratio - 0.1) < 1e-7
    assert p.shortest_cycles_only == 0 and p.dual_rounds == 1
    assert C.sizeof(binding.RamaParams) == 40
    assert C.sizeof(binding.RamaStats) == 112


def test_binding_structs_match_the_header(tmp_path):
    """sizeof / offsetof of every field as a C compiler sees include/rama.h vs the ctypes mirrors."""
    import subprocess
    from paper_2109_01838_amd import binding
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "rama.h"', 'int main(void) {',
             'printf("%d\\n", RAMA_MAX_CYCLE_LEN);', 'printf("%d\\n", RAMA_STATIC_MAX_NODES);',
             'printf("%d\\n", RAMA_STATIC_MAX_EDGES);']
    classes = (("rama_params", binding.RamaParams), ("rama_stats", binding.RamaStats),
               ("rama_round_stats", binding.RamaRoundStats), ("rama_alloc", binding.RamaAlloc))
    for cname, cls in classes:
        lines.append(f'printf("%zu\\n", sizeof({cname}));')
        for field, _ in cls._fields_:
            lines.append(f'printf("%zu\\n", offsetof({cname}, {field}));')
    lines += ['return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    want = [binding.MAX_CYCLE_LEN, binding.STATIC_MAX_NODES, binding.STATIC_MAX_EDGES]
    for _, cls in classes:
        want.append(C.sizeof(cls))
        want += [getattr(cls, field).offset for field, _ in cls._fields_]
    assert got == want


def test_no_cpu_fallback_without_gpu():
    import pytest
    import torch
    from paper_2109_01838_amd import Rama
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        Rama("cuda:0")


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2109_01838_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "rama_oracle" not in text, f
    for f in ("__init__.py", "rama_oracle.c"):
        text = open(os.path.join(ROOT, "oracle", f)).read()
        assert "paper_2109_01838_amd" not in text and "librama_hip" not in text


def test_stored_oracle_results_come_from_the_oracle_alone():
    """The script that writes tests/golden/*_oracle.json imports the oracle and the input generators, nothing of
    the HIP path; the stored files carry what the GPU tests compare."""
    import json
    text = open(os.path.join(ROOT, "tests", "golden", "make_oracle_goldens.py")).read()
    assert "import oracle" in text and "binding" not in text and "Rama" not in text and "librama_hip" not in text
    imports = [l.strip() for l in text.splitlines() if l.startswith(("import ", "from "))]
    assert all(("paper_2109_01838_amd import inputs" in l) or ("paper_2109_01838_amd" not in l) for l in imports), imports
    for name, edges in (("cfg4", 25034752), ("cfg5", 97996800)):
        g = json.load(open(os.path.join(ROOT, "tests", "golden", f"{name}_oracle.json")))
        assert g["n_edges"] == edges and g["oracle_precision"] == "f32" and g["oracle_threads"] == 1
        assert len(g["labels_sha256"]) == 64 and all(len(g["input_sha256"][k]) == 64 for k in "ijc")
        assert g["lower_bound"] <= g["primal"] < 0 and g["rounds"] > 1 and g["n_clusters"] > 1
        assert len(g["label_samples"]) >= 512 and g["n_cycles_first"][1] > 0
