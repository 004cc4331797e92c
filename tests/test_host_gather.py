"""Gathered indices never address outside the gathered axis.

Indices the compiler can read (constants) are validated when the graph is finalized; indices that arrive at run
time pass through a wrap-and-clamp helper in the generated code.  The helper is taken out of a generated kernel's
own source and run here on the CPU, under AddressSanitizer, over indices far outside the axis: on a GPU such a read
would be a memory fault, here it is a report."""
import os
import re
import subprocess
import sys
import tempfile

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
import unit_graphs as ug
from paper_2108_13342_amd import api


def _gather_source(spec):
    g, _ = api.graph_from_spec(spec)
    g.rewrite()
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    p = api.Plan(g, [1] * nw, fusion=1, profile=0)
    srcs = [p.block_source(b) for b in range(p.num_blocks()) if "Gather" in p.describe()[b]["ops"]]
    assert len(srcs) == 1
    return srcs[0]


def test_generated_gather_wraps_and_clamps_with_the_axis_extent():
    for axis, shape in ((0, (23, 40)), (1, (6, 17, 8))):
        src = _gather_source(ug.gather_block(np.zeros((3, 5), dtype=np.int64), table_shape=shape, axis=axis))
        calls = re.findall(r"dn_gidx\((\w+), (\d+)\)", src)
        assert calls and all(int(n) == shape[axis] for _, n in calls), calls
        # no address term multiplies a loaded index that has not gone through the helper
        assert not re.search(r"\(idx_t\)v\d+ \*", src)


def test_constant_indices_are_validated_on_the_host():
    ok = ug.gather_block(np.array([[0, -23, 22]]), const_ids=True)
    api.graph_from_spec(ok)
    for bad in (23, -24, 10 ** 6):
        with pytest.raises(api.DnnfError) as e:
            api.graph_from_spec(ug.gather_block(np.array([[0, bad]]), const_ids=True))
        assert "outside the axis" in str(e.value)


def test_index_helper_under_address_sanitizer():
    src = _gather_source(ug.gather_block(np.zeros((2, 2), dtype=np.int64)))
    helpers = [l for l in src.splitlines() if l.startswith("DEV long long dn_gidx(")]
    assert len(helpers) == 2
    n = 23
    ids = [0, 1, n - 1, n, n + 1, -1, -n, -n - 1, 2 ** 31, -2 ** 31, 2 ** 62, -2 ** 62, 10 ** 6, -10 ** 6]
    fids = ["0.0f", "22.9f", "23.0f", "-1.0f", "-23.0f", "-24.5f", "1e30f", "-1e30f", "__builtin_inff()", "-__builtin_inff()", "__builtin_nanf(\"\")", "16777217.0f"]
    prog = "#include <cstdio>\n#include <vector>\n#define DEV static inline\n" + "\n".join(helpers) + f"""
int main() {{
  std::vector<double> table({n});                      // exactly the axis: any index outside it is an ASan report
  for (int i = 0; i < {n}; ++i) table[i] = 100.0 + i;
  const long long ids[] = {{{", ".join(str(i) + "LL" for i in ids)}}};
  for (long long i : ids) printf("%.0f\\n", table[dn_gidx(i, {n}LL)]);
  const float fids[] = {{{", ".join(fids)}}};
  for (float f : fids) printf("%.0f\\n", table[dn_gidx(f, {n}LL)]);
  return 0;
}}
"""
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "g.cpp"), "w").write(prog)
        subprocess.run(["g++", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", os.path.join(d, "g.cpp"), "-o", os.path.join(d, "g")], check=True)
        r = subprocess.run([os.path.join(d, "g")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    got = [int(x) - 100 for x in r.stdout.split()]
    want = [min(max(i + n if i < 0 else i, 0), n - 1) for i in ids]
    want += [0, 22, 22, 22, 0, 0, 22, 0, 22, 0, 0, 22]       # floats: truncated, then wrapped and clamped; NaN reads position 0
    assert got == want, (got, want)
