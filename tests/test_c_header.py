"""The public header is plain C: it must compile with a C compiler, and a C program that
names every entry point must link against the built library (nothing is executed)."""
import os
import shutil
import subprocess
import tempfile

import pytest

import paper_2505_23725_amd as mlc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include <stddef.h>
#include "muloco.h"
/* one reference per entry point, through pointers of the declared types */
typedef void (*any_fn)(void);
static const any_fn entry_points[] = {
  (any_fn)muloco_strerror, (any_fn)newton_schulz_workspace_bytes,
  (any_fn)newton_schulz_workspace_min_bytes, (any_fn)newton_schulz,
  (any_fn)muloco_inner_workspace_bytes, (any_fn)muloco_inner_workspace_min_bytes,
  (any_fn)muloco_inner_step, (any_fn)muloco_outer_step, (any_fn)muloco_quantize_delta,
  (any_fn)muloco_topk_workspace_bytes, (any_fn)muloco_topk_outer_step,
  (any_fn)muloco_adamw_step, (any_fn)muloco_timing_enable, (any_fn)muloco_timing_read,
};
int main(void) {
  mlc_outer_hparams hp = {0};
  mlc_muon_hparams mh = {0};
  mlc_adamw_hparams ah = {0};
  mlc_kernel_timing t[MLC_KERNEL_FAMILIES];
  (void)hp; (void)mh; (void)ah; (void)t;
  return entry_points[0] == NULL || sizeof(entry_points) / sizeof(entry_points[0]) != 14;
}
"""


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_header_is_plain_c_and_every_entry_point_links():
    lib = mlc.library_path()
    assert os.path.exists(lib), "build the library first"
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "use_header.c")
        with open(src, "w") as f:
            f.write(PROGRAM)
        exe = os.path.join(tmp, "use_header")
        cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
               src, "-o", exe, lib, "-Wl,-rpath," + os.path.dirname(lib), "-Wl,--allow-shlib-undefined"]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr
