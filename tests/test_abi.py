"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2406_09827_amd as hipattn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hip_[a-z_]+)\s*\(", text)))


def _exported(path):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], check=True, capture_output=True, text=True).stdout
    return {line.split()[-1] for line in out.splitlines() if " T " in line}


def test_library_exports_every_declared_symbol():
    lib = hipattn.load()
    names = _declared_symbols("hipattn.h")
    assert set(names) >= {"hip_mask_estimate", "hip_sparse_attn", "hip_workspace_bytes", "hip_strerror"}
    for n in names:
        assert hasattr(lib, n), n
    assert lib.hip_attn_version() >= 100
    # the product library exports the declared calls and nothing else that looks like an entry point
    assert {n for n in _exported(hipattn.binding.LIB_PATH) if n.startswith("hip_")} == set(names)


def test_aux_library_exports_every_declared_symbol():
    from paper_2406_09827_amd import probes
    lib = probes.load()
    names = _declared_symbols("hipattn_aux.h")
    assert set(names) == set(probes.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    # every header of include/ is covered by one of the two tests
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["hipattn.h", "hipattn_aux.h"]


def _ok_problem():
    p = hipattn.HipProblem()
    p.batch, p.n_q_heads, p.n_kv_heads, p.head_dim = 1, 4, 2, 128
    p.q_len, p.max_kv_len, p.k, p.bq, p.bk, p.dtype = 64, 64, 32, 16, 2, hipattn.BF16
    return p


@pytest.mark.parametrize("mutate,code", [
    (lambda p: setattr(p, "k", 33), -3),
    (lambda p: setattr(p, "bq", 65), -3),
    (lambda p: setattr(p, "bk", 0), -3),
    (lambda p: setattr(p, "head_dim", 96), -4),
    (lambda p: setattr(p, "dtype", 7), -5),
    (lambda p: setattr(p, "n_kv_heads", 3), -2),
    (lambda p: setattr(p, "q_len", 65), -2),
    (lambda p: (setattr(p, "k", 4096), setattr(p, "bk", 2)), -6),
    (lambda p: (setattr(p, "page_table", 4096), setattr(p, "page_size", 3), setattr(p, "max_pages", 64)), -8),
    (lambda p: setattr(p, "q_strides", (ctypes.c_int64 * 3)(8192, 130, 2)), -7),
    (lambda p: setattr(p, "k_backing", 4096), -8),     # a backing pool / a map of pages read needs a page table
    (lambda p: setattr(p, "touched", 4096), -8),
    (lambda p: (setattr(p, "page_table", 4096), setattr(p, "page_size", 4), setattr(p, "max_pages", 64),
                setattr(p, "k_backing", 4100)), -7),
])
def test_argument_errors_before_launch(mutate, code):
    lib = hipattn.load()
    p = _ok_problem()
    mutate(p)
    fake = ctypes.c_void_p(4096)   # never dereferenced: validation fails first
    assert lib.hip_mask_estimate(ctypes.byref(p), fake, fake, fake, None) == code
    assert lib.hip_sparse_attn(ctypes.byref(p), fake, fake, fake, fake, fake, None) == code
    assert lib.hip_strerror(code) not in (None, b"", b"unknown error")


def test_null_and_misaligned_pointers():
    lib = hipattn.load()
    p = _ok_problem()
    fake = ctypes.c_void_p(4096)
    assert lib.hip_mask_estimate(None, fake, fake, fake, None) == -1
    assert lib.hip_mask_estimate(ctypes.byref(p), None, fake, fake, None) == -1
    assert lib.hip_sparse_attn(ctypes.byref(p), fake, fake, None, fake, fake, None) == -1
    assert lib.hip_mask_estimate(ctypes.byref(p), ctypes.c_void_p(4100), fake, fake, None) == -7
    assert lib.hip_workspace_bytes(ctypes.byref(p)) == 0


def test_workspace_rules_of_top_r():
    lib = hipattn.load()
    p = _ok_problem()
    fake = ctypes.c_void_p(4096)
    p.top_r = 16
    need = lib.hip_workspace_bytes(ctypes.byref(p))
    assert need == p.batch * p.n_q_heads * p.q_len * p.head_dim * 2
    assert lib.hip_mask_estimate(ctypes.byref(p), fake, fake, fake, None) == -1       # no workspace
    p.workspace, p.workspace_bytes = 4096 + 4, need
    assert lib.hip_mask_estimate(ctypes.byref(p), fake, fake, fake, None) == -7       # misaligned
    p.workspace, p.workspace_bytes = 4096, need - 1
    assert lib.hip_mask_estimate(ctypes.byref(p), fake, fake, fake, None) == -9       # too small
    assert lib.hip_strerror(-9) not in (None, b"", b"unknown error")
    p.top_r = -1
    assert lib.hip_mask_estimate(ctypes.byref(p), fake, fake, fake, None) == -2
    p.top_r = p.head_dim                                                              # all channels: no scratch
    assert lib.hip_workspace_bytes(ctypes.byref(p)) == 0


def test_ctypes_mirror_matches_the_header(tmp_path):
    """Size and field offsets of the ctypes mirror against what a C compiler makes of include/hipattn.h."""
    import subprocess
    fields = [n for n, _ in hipattn.HipProblem._fields_]
    src = tmp_path / "layout.c"
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "hipattn.h"', 'int main(void) {',
             '  printf("%zu\\n", sizeof(hip_problem));']
    lines += [f'  printf("%zu\\n", offsetof(hip_problem, {n}));' for n in fields]
    lines += ['  return 0; }']
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)], check=True)
    out = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == ctypes.sizeof(hipattn.HipProblem)
    assert out[1:] == [getattr(hipattn.HipProblem, n).offset for n in fields]


def test_binding_refuses_cpu_tensors():
    import torch
    q = torch.zeros(1, 1, 16, 64)
    with pytest.raises(RuntimeError):
        hipattn.hip_mask_estimate(q, q, 8, 4, 2)


def test_header_compiles_as_plain_c(tmp_path):
    """The C caller under tests/c_abi compiles with gcc (-Wall -Werror) against include/hipattn.h."""
    import subprocess
    src = os.path.join(ROOT, "tests", "c_abi", "c_abi_smoke.c")
    rocm_inc = "/opt/rocm/include"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
                    "-I", rocm_inc, "-c", src, "-o", str(tmp_path / "c_abi_smoke.o")], check=True)
