"""The boundary as a C compiler sees it: both headers compile as strict C99, a C program links against libmosaic.so
with every declared function referenced by name, and the host-side calls give that program the same answers the
Python binding gets (same struct layout on both sides)."""
import ctypes
import os
import re
import shutil
import subprocess

import pytest

from paper_2601_06562_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")
GCC = shutil.which("gcc")


def declared_functions():
    names = []
    for header in ("mosaic.h", "mosaic_graph.h"):
        text = open(os.path.join(INC, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(mosaic_\w+)\s*\(", text)
    return sorted(set(names))


@pytest.mark.skipif(GCC is None, reason="no gcc")
def test_headers_are_c99_and_a_c_program_gets_the_bindings_answers(tmp_path):
    names = declared_functions()
    assert set(binding.EXPORTS) | set(binding.GRAPH_EXPORTS) == set(names)          # the binding lists what is declared
    src = tmp_path / "abi.c"
    refs = ",\n  ".join(f"(void (*)(void))&{n}" for n in names)
    src.write_text(f"""
#include <stdio.h>
#include "mosaic.h"
#include "mosaic_graph.h"
typedef void (*fn)(void);
static fn all[] = {{
  {refs}
}};
int main(void) {{
  mosaic_plan p;
  size_t i, n = 0;
  int rc;
  for (i = 0; i < sizeof all / sizeof all[0]; ++i) n += all[i] != 0;
  rc = mosaic_plan_workspace(4096, 4096, 4096, 126464, 0, 256, 0, &p);
  printf("%d %d %zu %lld %d %d %d %d %d %d\\n", mosaic_version(), rc, n, (long long)p.workspace_bytes, p.num_chunks,
         p.rows_per_chunk, p.vocab_splits, p.tile_panel, p.grid, p.flags);
  rc = mosaic_plan_workspace(131072, 58501, 4096, 126464, 1 << 20, 256, 1, &p);
  printf("%d %lld %d %d %d %d %d %d %zu\\n", rc, (long long)p.workspace_bytes, p.num_chunks, p.rows_per_chunk,
         p.vocab_splits, p.tile_panel, p.grid, p.flags, sizeof(mosaic_plan));
  printf("%s|%s\\n", mosaic_status_string(MOSAIC_ERR_WORKSPACE_TOO_SMALL), mosaic_status_string(12345));
  return 0;
}}
""")
    libdir = os.path.dirname(binding.LIB_PATH)
    exe = str(tmp_path / "abi")
    subprocess.run([GCC, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I" + INC, "-o", exe, str(src),
                    "-L" + libdir, "-lmosaic", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([exe], check=True, stdout=subprocess.PIPE, text=True).stdout.split("\n")
    first = out[0].split()
    assert int(first[0]) == binding.lib().mosaic_version() and int(first[1]) == 0 and int(first[2]) == len(names)
    a = binding.mosaic_plan_workspace(4096, 4096, 4096, 126464, 0)
    assert [int(x) for x in first[3:]] == [a.workspace_bytes, a.num_chunks, a.rows_per_chunk, a.vocab_splits, a.tile_panel,
                                          a.grid, a.flags]
    second = out[1].split()
    b = binding.mosaic_plan_workspace(131072, 58501, 4096, 126464, 1 << 20, sampling=True)
    assert int(second[0]) == 0 and b.workspace_bytes <= 1 << 20
    assert [int(x) for x in second[1:8]] == [b.workspace_bytes, b.num_chunks, b.rows_per_chunk, b.vocab_splits,
                                             b.tile_panel, b.grid, b.flags]
    assert int(second[8]) == ctypes.sizeof(binding.MosaicPlan)
    L = binding.lib()
    assert out[2].split("|") == [L.mosaic_status_string(binding.MOSAIC_ERR_WORKSPACE_TOO_SMALL).decode(),
                                 L.mosaic_status_string(12345).decode()]
