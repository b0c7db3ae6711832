"""The C-ABI library loads, exports every symbol include/hdet.h declares, and the binding's
structures have the C compiler's layout.  No GPU needed (no compute calls)."""
import ctypes as C
import os
import re
import subprocess
import tempfile

import pytest

import paper_2604_24708_amd as H
from paper_2604_24708_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hdet.h")


def test_library_exports_every_declared_symbol():
    lib = H.load_library()
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(hdet_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_the_c_compiler():
    src = r'''
#include <stdio.h>
#include <stddef.h>
#include "hdet.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu ", sizeof(hdet_config), sizeof(hdet_buffers), sizeof(hdet_state),
         sizeof(hdet_channel), sizeof(hdet_model_dims));
  printf("%zu %zu %zu %zu %zu %zu\n", offsetof(hdet_config, dims), offsetof(hdet_config, extra),
         offsetof(hdet_config, stream), offsetof(hdet_state, rho), offsetof(hdet_state, perm),
         offsetof(hdet_buffers, plane_stride));
  return 0;
}'''
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "s.c")
        open(c, "w").write(src)
        exe = os.path.join(d, "s")
        subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), c, "-o", exe], check=True)
        got = [int(x) for x in subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()]
    want = [C.sizeof(B.hdet_config), C.sizeof(B.hdet_buffers), C.sizeof(B.hdet_state),
            C.sizeof(B.hdet_channel), C.sizeof(B.hdet_model_dims),
            B.hdet_config.dims.offset, B.hdet_config.extra.offset, B.hdet_config.stream.offset,
            B.hdet_state.rho.offset, B.hdet_state.perm.offset, B.hdet_buffers.plane_stride.offset]
    assert got == want


def test_validation_needs_no_gpu():
    cfg = H.make_config(n_replicas=4, sync_interval=4, total_steps=40, warm_steps=12, lr_max=0.05,
                        alpha=0.2, n_params=100)
    assert H.hdet_workspace_bytes(cfg, 100) == (1600, 0, 0)
    for bad in [dict(n_replicas=0), dict(n_replicas=65), dict(sync_interval=0), dict(alpha=-0.1),
                dict(lr_max=0.0), dict(optimizer=5), dict(pct_start=0.0)]:
        kw = dict(n_replicas=4, sync_interval=4, total_steps=40, warm_steps=12, lr_max=0.05,
                  alpha=0.2, n_params=100)
        kw.update(bad)
        with pytest.raises(H.HdetError) as e:
            H.hdet_workspace_bytes(H.make_config(**kw), 100)
        assert e.value.code == H.HDET_EINVAL
    with pytest.raises(H.HdetError):
        H.hdet_workspace_bytes(cfg, 98)          # stride < P
    with pytest.raises(H.HdetError):
        H.hdet_workspace_bytes(cfg, 102)         # not a multiple of 4
    assert H.hdet_destroy(None) is None


def test_product_path_does_not_touch_the_oracle():
    """Nothing under the package may import or name the oracle."""
    pkg = os.path.join(ROOT, "paper_2604_24708_amd")
    for base, _, files in os.walk(pkg):
        if "_build" in base:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(base, f)).read().lower(), f
