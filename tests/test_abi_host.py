"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares,
validates parameter blocks and sizes its workspace.  No kernel is launched here."""
import ctypes
import math
import os
import re

import pytest

from paper_2603_14549_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_2603_14549_amd import build
        build.build_library(verbose=False)
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "asap.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(asap_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_stage_calls():
    names = declared_functions()
    for n in ("asap_score", "asap_select", "asap_merge", "asap_compact_kv"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert sorted(names) == sorted(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def good():
    return binding.params_from_config(synth.CONFIGS["C6"])


def test_check_params_accepts_all_benchmark_configs(lib):
    for cfg in synth.CONFIGS.values():
        st, msg = binding.asap_check_params(binding.params_from_config(cfg))
        assert st == binding.ASAP_OK, (cfg.name, msg)
        assert binding.asap_workspace_bytes(binding.params_from_config(cfg)) > 0


@pytest.mark.parametrize("field,value", [
    ("B", 0), ("k", 0), ("k", 2305), ("Hkv", 5), ("d", 96), ("D", 4100), ("V", 0), ("V", 20000),
    ("Tmax", 0), ("Tmax", 129), ("P", -1), ("P", (1 << 20) + 1), ("lambda_max", 0.0), ("lambda_max", 1.5), ("eps", 0.0),
    ("merge_weight", -1.0), ("sim_threshold", float("nan")), ("qk_dtype", 7), ("mask_mode", 3), ("route", 2),
    ("score_rows", 2),
])
def test_check_params_rejects(lib, field, value):
    p = good()
    setattr(p, field, value)
    st, msg = binding.asap_check_params(p)
    assert st == binding.ASAP_EINVAL and msg
    assert binding.asap_workspace_bytes(p) == 0


def test_k_equal_v_and_infinite_threshold_are_legal(lib):
    p = good()
    p.k = p.V
    p.sim_threshold = -math.inf
    assert binding.asap_check_params(p)[0] == binding.ASAP_OK


def test_workspace_size_formula(lib):
    # query sums + per-kv-head sums + fp64 mass + min/max keys + per-split row statistics
    # + per-head column sums (C6: one query chunk, one key split, 64 text rows)
    p = good()
    B, H, Hkv, d, V = p.B, p.H, p.Hkv, p.d, p.V
    al = lambda x: (x + 255) // 256 * 256
    want = (al(8 * B * H * 1 * d) + al(8 * B * Hkv * d) + al(2 * B * Hkv * 4 * d) + al(8 * B * V) + al(16 * B)
            + al(4 * B * H * 1 * 2 * 64) + al(4 * B * H * V))
    assert binding.asap_workspace_bytes(p) == want
    assert want >= al(4 * B * p.k)          # also covers the kept-row norms of asap_merge


def test_struct_layout_matches_header(lib):
    # 9 int32 + 3 enums + 4 floats + 3 enums, all 4 bytes, no padding
    assert ctypes.sizeof(binding.asap_params) == 19 * 4


def test_header_is_plain_c_and_the_binding_mirrors_its_structs(tmp_path):
    """include/asap.h compiles as C11 on its own, and the ctypes mirrors of its two structs have the
    size and the field offsets the C compiler gives them."""
    import subprocess
    fields = {"asap_params": [f[0] for f in binding.asap_params._fields_],
              "asap_stage_io": [f[0] for f in binding.asap_stage_io._fields_]}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "asap.h"', 'int main(void) {']
    for st, names in fields.items():
        lines.append(f'  printf("{st} %zu\\n", sizeof({st}));')
        for n in names:
            lines.append(f'  printf("{st}.{n} %zu\\n", offsetof({st}, {n}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.splitlines())
    for st, names in fields.items():
        cls = getattr(binding, st)
        assert int(out[st]) == ctypes.sizeof(cls), st
        for n in names:
            assert int(out[f"{st}.{n}"]) == getattr(cls, n).offset, f"{st}.{n}"


def read_golden(name):
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", name)):
        line = line.split("#")[0].strip()
        if line:
            rows.append(line.split())
    return rows


def test_flops_utility_against_the_printed_tables_and_the_oracle(lib):
    # Eq. 7 / Eq. 8 as the library computes them: the values the paper prints (Tables 1, 2, 5) ...
    for row in read_golden("eq7_flops.txt"):
        v, printed = int(row[0]), float(row[1])
        assert abs(binding.asap_theoretical_flops([32], [v], 4096, 11008) / 1e12 - printed) <= 0.0006
    for row in read_golden("eq8_ratio.txt"):
        v, v0, pct = int(row[0]), int(row[1]), float(row[2])
        assert abs(100.0 * binding.asap_flops_ratio([32], [v], v0, 4096, 11008) - pct) <= 0.006
    # ... and a multi-stage schedule against the oracle's own formula
    from oracle import asap_oracle as O
    layers, tokens = [2, 14, 16], [2304, 576, 160]
    assert binding.asap_theoretical_flops(layers, tokens, 5120, 13824) == O.theoretical_flops(layers, tokens, 5120, 13824)
    assert abs(binding.asap_flops_ratio(layers, tokens, 2304, 5120, 13824) -
               O.flops_ratio(layers, tokens, 2304, 5120, 13824)) <= 1e-15
    with pytest.raises(binding.AsapError):
        binding.asap_theoretical_flops([1], [-5], 64, 64)


def test_paper_route_needs_room_to_refill(lib):
    p = good()
    p.route = binding.ASAP_ROUTE_PAPER
    assert binding.asap_check_params(p)[0] == binding.ASAP_OK
    assert binding.asap_workspace_bytes(p) >= 4 * p.B * p.k
    p.k = p.V // 2 + 1
    st, msg = binding.asap_check_params(p)
    assert st == binding.ASAP_EINVAL and "V / 2" in msg


def test_a_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """The product path has one implementation: without the built library every entry fails at load
    time, and nothing under paper_2603_14549_amd imports the oracle."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libasap.so"))
    with pytest.raises(FileNotFoundError, match="no fallback"):
        binding.load()
    with pytest.raises(FileNotFoundError):
        binding.asap_workspace_bytes(binding.params_from_config(synth.CONFIGS["S1"]))
    pkg = os.path.dirname(os.path.abspath(binding.__file__))
    for root, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(root, f), encoding="utf-8").read()
                assert "import oracle" not in text and "from oracle" not in text and "asap_oracle" not in text, f
