"""CPU-only checks of the C-ABI boundary: the built library loads, exports every symbol the
header declares, and its host-side validation rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(bd.lib_path()):
        from paper_2605_19726_amd import build
        build.build(verbose=False)
    return bd.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "basa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(basa_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in basa.h but not exported"
    assert sorted(bd.EXPORTS) == names


def test_version_and_status_strings(lib):
    assert "gfx950" in bd.basa_version()
    assert lib.basa_status_string(0) == b"BASA_OK"
    assert lib.basa_status_string(3) == b"BASA_ERR_WORKSPACE"


@pytest.mark.parametrize("n,s", [(16, 0.5), (591, 0.5), (591, 0.75), (1024, 0.9), (1024, 0.0),
                                 (590, 0.6), (1000, 0.7), (3, 0.99), (512, 0.3), (77, 0.123)])
def test_kappa_matches_oracle(lib, n, s):
    assert bd.basa_kappa(n, s) == o.kappa_from_sparsity(n, s)


def test_kappa_rejects_bad_input(lib):
    assert bd.basa_kappa(10, 1.0) == -1
    assert bd.basa_kappa(10, -0.5) == -1
    assert bd.basa_kappa(0, 0.5) == -1


def fake_tensor(ptr=0x1000, dtype=bd.BF16, batch=1, heads=2, L=256, d=128):
    return bd.BasaTensor(ptr, dtype, batch, heads, L, d, heads * L * d, L * d, d)


def status_of(lib, fn, *args):
    st = fn(*args)
    return lib.basa_status_string(st).decode(), lib.basa_last_error().decode()


def test_select_argument_validation(lib):
    q, k = fake_tensor(), fake_tensor()
    p = bd.params(128, 0.5)
    V = C.c_void_p
    dummy = V(0x2000)
    call = lambda q_, k_, p_, rc=dummy, ws=dummy, wsb=1 << 40: status_of(
        lib, lib.basa_select, C.byref(q_), C.byref(k_), C.byref(p_), None, rc, dummy, dummy, dummy,
        None, None, ws, wsb, None)
    assert call(fake_tensor(ptr=0), k, p)[0] == "BASA_ERR_INVALID_ARG"
    assert call(fake_tensor(d=96), k, p)[0] == "BASA_ERR_UNSUPPORTED"
    assert call(fake_tensor(heads=3), k, p)[0] == "BASA_ERR_INVALID_ARG"        # 3 % 2 != 0
    assert call(q, fake_tensor(dtype=bd.F32), p)[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(100, 0.5))[0] == "BASA_ERR_UNSUPPORTED"
    assert call(q, k, bd.params(128, 1.0))[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(128, 0.5, window=100))[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(128, 0.5, sort=7))[0] == "BASA_ERR_INVALID_ARG"
    assert call(fake_tensor(L=0), k, p)[0] == "BASA_ERR_INVALID_ARG"            # empty sequence
    assert call(q, fake_tensor(L=4097 * 128), p)[0] == "BASA_ERR_UNSUPPORTED"   # more than 4096 key blocks
    assert call(q, k, bd.params(128, 0.5, mass_target=1.5))[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(128, 0.5, mass_target=-0.1))[0] == "BASA_ERR_INVALID_ARG"
    bad = bd.params(128, 0.5)
    bad.causal = 2
    assert call(q, k, bad)[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(128, 0.5, select_path=3))[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(128, 0.5, select_path=-1))[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(128, 0.5, mass_target=0.9, min_keep=-1))[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, bd.params(128, 0.5, budget_total=-1))[0] == "BASA_ERR_INVALID_ARG"
    seg = lambda starts, **kw: bd.params(128, 0.5, segments=starts, **kw)
    assert call(q, k, seg([1, 5]))[0] == "BASA_ERR_INVALID_ARG"                 # must start at 0
    assert call(q, k, seg([0, 5, 5]))[0] == "BASA_ERR_INVALID_ARG"              # must ascend strictly
    assert call(q, k, seg([0, 1000]))[0] == "BASA_ERR_INVALID_ARG"              # last start must be below L = 256
    assert call(q, k, seg([0, 128], window=128))[0] == "BASA_ERR_INVALID_ARG"   # one or the other
    assert call(q, k, seg(list(range(64))))[0] == "BASA_ERR_INVALID_ARG"        # at most 63
    assert call(q, fake_tensor(L=2000), seg([0, 5]))[0] == "BASA_ERR_INVALID_ARG"   # L_q != L_k
    pn = bd.params(128, 0.5); pn.n_segments = 2
    assert call(q, k, pn)[0] == "BASA_ERR_INVALID_ARG"                          # count without the array
    assert call(q, k, seg([0, 5]), wsb=16)[0] == "BASA_ERR_WORKSPACE"           # a valid list gets past the checks
    assert call(q, k, p, rc=None)[0] == "BASA_ERR_INVALID_ARG"
    name, why = call(q, k, p, wsb=16)
    assert name == "BASA_ERR_WORKSPACE" and "need" in why
    assert call(q, k, p, ws=None)[0] == "BASA_ERR_WORKSPACE"
    assert call(fake_tensor(ptr=0x1004), k, p)[0] == "BASA_ERR_INVALID_ARG"     # misaligned


def test_attention_argument_validation(lib):
    q, k, v = fake_tensor(), fake_tensor(), fake_tensor()
    p = bd.params(128)
    dummy = C.c_void_p(0x2000)
    strides = lambda *v_: (C.c_int64 * 3)(*v_)
    call = lambda q_, k_, v_, out=dummy, wsb=16, ostr=None, p_=p: status_of(
        lib, lib.basa_sparse_attn, C.byref(q_), C.byref(k_), C.byref(v_), dummy, dummy, 4, None, None,
        C.byref(p_), out, ostr, None, dummy, wsb, None)
    assert call(q, k, fake_tensor(L=128))[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, v, out=None)[0] == "BASA_ERR_INVALID_ARG"
    assert call(q, k, v, out=C.c_void_p(0x2004))[0] == "BASA_ERR_INVALID_ARG"            # misaligned
    assert call(q, k, v)[0] == "BASA_ERR_WORKSPACE"
    # more key blocks than a workgroup can list: refused on the host, before any device call
    big = fake_tensor(L=128 * 16385)
    name, why = call(q, big, big, wsb=1 << 50)
    assert name == "BASA_ERR_UNSUPPORTED" and "key blocks per head exceed" in why
    for bad in (-1, 5):
        assert call(q, k, v, wsb=1 << 40, p_=bd.params(128, attn_shape=bad))[0] == "BASA_ERR_INVALID_ARG"
    # output strides: token-major is fine (and reaches the workspace check), the rest is refused
    assert call(q, k, v, ostr=strides(256 * 2 * 128, 128, 2 * 128))[0] == "BASA_ERR_WORKSPACE"
    assert call(q, k, v, ostr=strides(256 * 2 * 128, 128, 64))[0] == "BASA_ERR_INVALID_ARG"      # token stride < d
    assert call(q, k, v, ostr=strides(256 * 2 * 128, 132, 2 * 128))[0] == "BASA_ERR_INVALID_ARG"  # not 16-byte
    assert call(q, k, v, ostr=strides(-8, 128, 2 * 128))[0] == "BASA_ERR_INVALID_ARG"
    st = lib.basa_dense_attn(C.byref(q), C.byref(k), C.byref(v), C.byref(p), dummy, None, None, dummy, 16, None)
    assert lib.basa_status_string(st) == b"BASA_ERR_WORKSPACE"

def test_workspace_sizes(lib):
    q, k = fake_tensor(heads=4, L=1000), fake_tensor(heads=2, L=1000)
    p = bd.params(128, 0.5)
    sel = lib.basa_select_workspace_size(C.byref(q), C.byref(k), C.byref(p))
    att = lib.basa_attn_workspace_size(C.byref(q), C.byref(k), C.byref(p))
    # attention workspace: tiled K and transposed V, padded to whole blocks (Q needs no copy)
    # (+ 272 bytes per 64-key tile: the key indices of the causal variant; + the probe counters)
    kv = (2 + 2) * 1024 * 128 * 2
    assert kv + 2 * 16 * 272 <= att <= kv + 2 * 16 * 272 + 1024
    assert sel >= 2 * 4 * 1000 * 8
    assert lib.basa_select_workspace_size(C.byref(fake_tensor(d=96)), C.byref(k), C.byref(p)) == 0


def test_struct_layouts_match_the_c_header(tmp_path):
    """The ctypes structures of the binding against the header as a C compiler lays it out."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    fields = {"basa_tensor": [f for f, _ in bd.BasaTensor._fields_], "basa_params": [f for f, _ in bd.BasaParams._fields_]}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "basa.h"', 'int main(void) {']
    for st, fl in fields.items():
        lines.append(f'  printf("{st} %zu\\n", sizeof({st}));')
        for f in fl:
            lines.append(f'  printf("{st}.{f} %zu\\n", offsetof({st}, {f}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run([cc, "-std=c99", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe)], check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for st, cls in (("basa_tensor", bd.BasaTensor), ("basa_params", bd.BasaParams)):
        assert int(got[st]) == C.sizeof(cls), st
        for f, _ in cls._fields_:
            assert int(got[f"{st}.{f}"]) == getattr(cls, f).offset, f"{st}.{f}"


def test_static_norm_sort_validation_without_a_launch(lib):
    # the size check comes before the scratch address is resolved, so no GPU is needed
    assert lib.basa_static_scratch_size() == 32 << 20
    p = bd.params(128)
    call = lambda x_, perm=C.c_void_p(0x2000): status_of(lib, lib.basa_norm_sort_static, C.byref(x_), C.byref(p),
                                                          perm, None, None)
    assert call(fake_tensor(ptr=0))[0] == "BASA_ERR_INVALID_ARG"
    assert call(fake_tensor(), perm=None)[0] == "BASA_ERR_INVALID_ARG"
    name, why = call(fake_tensor(heads=33, L=1 << 16))                    # 33 * 65536 tokens > 2 Mi
    assert name == "BASA_ERR_WORKSPACE" and "static array holds" in why


def test_downsample_validation_without_a_launch(lib):
    p = bd.params(128)
    x = fake_tensor()
    V = C.c_void_p
    call = lambda x_, mean=V(0x2000), xs=None: status_of(lib, lib.basa_downsample, C.byref(x_), None, C.byref(p),
                                                         mean, None, xs, None)
    assert call(x, mean=None)[0] == "BASA_ERR_INVALID_ARG"
    assert call(x, xs=V(0x3004))[0] == "BASA_ERR_INVALID_ARG"             # misaligned x_sorted
    assert call(x, xs=V(0x1000))[0] == "BASA_ERR_INVALID_ARG"             # x_sorted aliases x
    assert call(fake_tensor(d=96))[0] == "BASA_ERR_UNSUPPORTED"
    # a bad descriptor gives no workspace size instead of a number
    assert lib.basa_block_mass_workspace_size(C.byref(fake_tensor(ptr=0)), C.byref(x)) == 0
    assert lib.basa_block_mass_workspace_size(C.byref(x), C.byref(fake_tensor(heads=3))) == 0
    assert lib.basa_block_mass_workspace_size(C.byref(x), C.byref(x)) > 0
