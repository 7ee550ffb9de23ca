"""The boundary is a C ABI: both public headers must compile as plain C99, and a C program that includes
nothing else must link against the built library and get through the host-side calls (no GPU needed)."""
from __future__ import annotations

import os
import subprocess

from paper_2507_10069_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")


def test_headers_are_plain_c99(tmp_path):
    for header in ("emm.h", "emm_prefix_cache.h"):
        src = tmp_path / ("use_" + header.replace(".h", ".c"))
        src.write_text('#include "%s"\nint main(void) { return 0; }\n' % header)
        subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", INCLUDE, str(src)],
                       check=True)


def test_c_program_links_and_runs_host_calls(tmp_path):
    lib = B.LIB_PATH
    assert os.path.exists(lib), "build the library first (python -c 'import __graft_entry__ as g; g.build()')"
    exe = tmp_path / "host_calls"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", INCLUDE,
                    os.path.join(ROOT, "tests", "c_abi", "host_calls.c"), "-o", str(exe), lib,
                    "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=120)
    assert out.stdout.strip() == "ok"
