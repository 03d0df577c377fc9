"""The boundary is a C ABI: a plain C99 program (no C++, no torch, no Python in the loop) includes the
header, links the library and exercises the host-side contract: size query, plan report, argument checks
of every entry point, status strings.  Nothing here touches a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_01875_amd", "csrc")

PROGRAM = r"""
#include <stdio.h>
#include <string.h>
#include "kdloss.h"

#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void) {
  kd_loss_params p;
  size_t bytes = 0, small = 0;
  int64_t chunk = 0, launches = 0;
  char* fake[10];
  int i;
  memset(&p, 0, sizeof p);
  p.T = 4096; p.H_t = 4096; p.H_s = 1024; p.V = 151936;
  p.in_dtype = KD_BF16; p.grad_dtype = KD_BF16; p.w_layout = KD_W_VH; p.kind = KD_FKL;
  p.tau = 1.0f; p.beta = 0.5f; p.loss_scale = 1.0f;
  CHECK(sizeof p == 80);
  CHECK(kd_loss_workspace_size(&p, &bytes) == KD_OK);
  CHECK(bytes > 0 && bytes < (size_t)2 * 4096 * 151936 / 3);       /* far below one [T,V] bf16 tensor */
  CHECK(kd_loss_plan_info(&p, &chunk, &launches) == KD_OK && chunk == 16384 && launches > 0);
  p.vocab_chunk = 2048;
  CHECK(kd_loss_workspace_size(&p, &small) == KD_OK && small < bytes);
  p.vocab_chunk = 100;
  CHECK(kd_loss_workspace_size(&p, &small) == KD_ERR_PARAM);
  p.vocab_chunk = 0;
  p.loss_scale = 0.0f;                                               /* a zeroed block is refused, not run */
  CHECK(kd_loss_workspace_size(&p, &small) == KD_ERR_PARAM);
  p.loss_scale = 1.0f;
  p.kind = KD_AKL; p.beta = 0.0f;
  CHECK(kd_loss_workspace_size(&p, &small) == KD_ERR_PARAM);
  p.kind = KD_FKL; p.beta = 0.5f;
  for (i = 0; i < 10; ++i) fake[i] = (char*)(size_t)(0x10000 * (i + 1));   /* never dereferenced */
  CHECK(kd_loss_fwd_bwd(&p, fake[0], fake[1], fake[2], fake[3], NULL, (float*)fake[4], NULL, fake[5], fake[6],
                        fake[7], bytes - 1, NULL) == KD_ERR_WORKSPACE);
  CHECK(kd_loss_fwd_bwd(&p, NULL, fake[1], fake[2], fake[3], NULL, (float*)fake[4], NULL, fake[5], fake[6],
                        fake[7], bytes, NULL) == KD_ERR_NULL);
  CHECK(kd_loss_fwd(&p, fake[0], fake[1], fake[2] + 4, fake[3], NULL, (float*)fake[4], NULL, fake[7], bytes,
                    NULL) == KD_ERR_ALIGN);
  CHECK(kd_loss_fwd_bwd_static(&p, fake[0], fake[1], fake[2], fake[3], NULL, NULL, NULL, fake[5], fake[6],
                               NULL) == KD_ERR_NULL);
  p.T = 32768; p.H_t = 5120; p.H_s = 4096;
  CHECK(kd_loss_fwd_bwd_static(&p, fake[0], fake[1], fake[2], fake[3], NULL, (float*)fake[4], NULL, fake[5],
                               fake[6], NULL) == KD_ERR_TOO_LARGE);
  CHECK(kd_quantize_e4m3(fake[0], KD_BF16, 0, 1.0f, fake[1], NULL) == KD_ERR_SHAPE);
  for (i = 0; i <= 8; ++i) CHECK(strlen(kd_status_string((kd_status)i)) > 0);
  printf("C ABI OK: workspace %zu bytes, chunk %lld, %lld launches\n", bytes, (long long)chunk, (long long)launches);
  return 0;
}
"""


def test_plain_c_program_uses_the_library(tmp_path):
    lib = os.path.join(CSRC, "libkdloss.so")
    if not os.path.exists(lib):
        pytest.fail("libkdloss.so is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    src = tmp_path / "use_kdloss.c"
    src.write_text(PROGRAM)
    exe = tmp_path / "use_kdloss"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                        "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe), "-L", CSRC, "-lkdloss",
                        "-Wl,-rpath," + CSRC, "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "C ABI OK" in r.stdout, r.stdout + r.stderr
