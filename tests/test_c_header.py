"""include/adacomp.h is a C header: a C99 translation unit that includes it must compile with gcc
-pedantic, link against libadacomp.so and get sensible answers from the calls that need no GPU."""
import os
import subprocess

import paper_1702_04683_amd as ac

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include <stdio.h>
#include "adacomp.h"

int main(void) {
    uint64_t n[3] = {1000, 0, 7};
    uint64_t off[4] = {0, 10, 10, 11};
    size_t bytes = 0;
    uint64_t words = 0;
    adacomp_update_t u;
    adacomp_state_t st;
    adacomp_layer_t layer;
    adacomp_param_layer_t param;
    (void)u; (void)st; (void)layer; (void)param;
    if (adacomp_count(1000, 0.01) != 10) return 1;
    if (adacomp_select_workspace(n, 3, 0.01, NULL, &bytes) != ADACOMP_OK || bytes == 0) return 2;
    if (adacomp_select_workspace(n, 3, 2.0, NULL, &bytes) != ADACOMP_ERR_RATE) return 3;
    if (adacomp_wire_bound(off, 3, &words) != ADACOMP_OK || words != 4 + 3 + 2 + 1 + 11 + 11) return 4;
    if (adacomp_wire_workspace(off, 3, &bytes) != ADACOMP_OK || bytes % 256) return 5;
    if (adacomp_select(NULL, 1, 0.5, NULL, NULL, NULL, 0, NULL) != ADACOMP_ERR_NULL) return 6;
    printf("%s|%s|%d\n", adacomp_strerror(ADACOMP_ERR_WORKSPACE), adacomp_kernel_name(ADACOMP_KERNEL_FILTER),
           (int)ADACOMP_KERNEL_COUNT);
    return 0;
}
"""


def test_header_compiles_as_c99_and_links(tmp_path):
    lib = ac.library_path()
    assert os.path.exists(lib), "build the library first (python -c 'import __graft_entry__ as g; g.build()')"
    src = tmp_path / "use_abi.c"
    src.write_text(PROGRAM)
    exe = tmp_path / "use_abi"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), lib, "-Wl,-rpath," + os.path.dirname(lib)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.strip().split("|")
    assert "workspace" in out[0] and out[1] == "filter" and int(out[2]) == ac.binding.KERNEL_COUNT
