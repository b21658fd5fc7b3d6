"""include/ssrnn.h is a C header: a plain C program (gcc -std=c99 -pedantic) includes it, links the
library and calls the host-only entry points.  No GPU is touched."""
import os
import subprocess

import paper_1803_11389_amd as ss

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

C_SOURCE = r"""
#include <stdio.h>
#include <string.h>
#include "ssrnn.h"

int main(void) {
  size_t ws = ssrnn_workspace_bytes(8, 4096, 1, 4, SSRNN_F32);
  size_t w8 = ssrnn_weight_bytes(128, 1, SSRNN_FP8);
  size_t pk = ssrnn_packed_weight_bytes(1024, 2, SSRNN_BF16);
  const void* W[1] = {0};
  /* rejected on the host: W[0] is NULL */
  int rc = sru_forward(W, 0, 0, 0, 0, (float*)0x1000, 1, 128, 8, 4, SSRNN_F32, SSRNN_SCHED_WAVEFRONT | SSRNN_KERNEL_AUTO, 0, 0, 0);
  printf("%d %zu %zu %zu %d %d\n", ssrnn_version(), ws, w8, pk, rc, (int)strlen(ssrnn_last_error()) > 0);
  return 0;
}
"""


def test_header_compiles_as_c_and_links(tmp_path):
    if not os.path.exists(ss.LIB_PATH):
        from paper_1803_11389_amd.build import build
        build()
    src = tmp_path / "abi.c"
    src.write_text(C_SOURCE)
    exe = tmp_path / "abi"
    libdir = os.path.dirname(ss.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-lssrnn", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=120).stdout.split()
    version, ws, w8, pk, rc, has_msg = (int(v) for v in out)
    assert version == ss.version() and ws == ss.workspace_bytes(8, 4096, 1, 4, ss.F32) and ws > 0
    assert w8 == 3 * 128 * 128 + 12 * 128 and pk == 3 * 1024 * 2048 * 2
    assert rc == 1 and has_msg == 1
