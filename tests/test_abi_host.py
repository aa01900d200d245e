"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

from paper_2510_08318_amd import binding as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# A fake, suitably aligned "device address": argument checks never dereference it.
P = 0x10000000


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    headers = sorted(f for f in os.listdir(inc) if f.endswith(".h"))
    assert headers == ["linattn.h", "linattn_bench.h"]
    declared = set()
    for f in headers:
        declared |= set(re.findall(r"\b(linattn_[a-z_]+)\s*\(", open(os.path.join(inc, f)).read()))
    assert declared == set(L.EXPORTS)
    lib = L.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_header_constants_match_binding():
    header = open(os.path.join(ROOT, "include", "linattn.h")).read()
    consts = dict((m.group(1), int(m.group(2))) for m in re.finditer(r"#define\s+LINATTN_(\w+)\s+(-?\d+)", header))
    for name in ("OK", "E_NULL", "E_SHAPE", "E_DTYPE", "E_ALIGN", "E_PHI", "E_WORKSPACE", "E_HIP", "E_STATE",
                 "E_ALIAS", "PHI_HEDGEHOG", "PHI_RELU", "BF16", "F32", "LAYOUT_BHND", "LAYOUT_BNHD"):
        assert consts[name] == getattr(L, name), name
    for code in range(0, -10, -1):
        assert L.linattn_strerror(code) != "unknown status"
    assert L.linattn_strerror(-99) == "unknown status"


def test_workspace_bytes_is_pure_and_monotone():
    w = L.linattn_workspace_bytes(1, 40, 75600, 128, L.PHI_HEDGEHOG, L.BF16)
    assert w == L.linattn_workspace_bytes(1, 40, 75600, 128, L.PHI_HEDGEHOG, L.BF16)
    # partials of at most 512 workgroups + state + operand image: tens of MB, not GB
    assert 2_000_000 < w < 64_000_000
    assert L.linattn_workspace_bytes(2, 40, 75600, 128, L.PHI_HEDGEHOG, L.BF16) >= w
    assert w % 256 == 0
    for bad in [(0, 1, 8, 64), (1, 0, 8, 64), (1, 1, 0, 64), (1, 1, 8, 32), (1, 1, 8, 96), (1, 1, -5, 128),
                (70000, 1, 8, 64)]:
        assert L.linattn_workspace_bytes(*bad, L.PHI_HEDGEHOG, L.BF16) == 0
    assert L.linattn_workspace_bytes(1, 1, 8, 64, 7, L.BF16) == 0
    assert L.linattn_workspace_bytes(1, 1, 8, 64, L.PHI_HEDGEHOG, 9) == 0


def test_phi_create_rejects_bad_descriptors():
    mk = lambda **kw: L.linattn_phi_create(**{**dict(kind=L.PHI_HEDGEHOG, dtype=L.BF16, H=2, d=64, wq=P, wk=P + 4096), **kw}, check=False)
    assert mk(kind=3) == L.E_PHI
    assert mk(dtype=5) == L.E_DTYPE
    assert mk(H=0) == L.E_SHAPE
    assert mk(d=48) == L.E_SHAPE
    assert mk(layout=2) == L.E_SHAPE
    assert mk(layout=-1) == L.E_SHAPE
    pid = mk(layout=L.LAYOUT_BNHD)
    assert pid >= 16 and L.linattn_phi_destroy(pid) == L.OK
    assert mk(wq=None) == L.E_NULL
    assert mk(wk=None) == L.E_NULL
    assert mk(wq=P + 2) == L.E_ALIGN
    assert mk(state=P + 8, state_bytes=1 << 20) == L.E_ALIGN
    one = 2 * 65 * 64 * 4                                           # H * (d+1) * d fp32: the state of one batch item
    assert mk(state=P + 4096) == L.E_STATE                          # a state buffer of unknown size
    assert mk(state=P + 4096, state_bytes=one - 4) == L.E_STATE
    pid = mk(state=P + 4096, state_bytes=one)
    assert pid >= 16 and L.linattn_phi_destroy(pid) == L.OK
    assert mk(workspace=P + 128, workspace_bytes=1 << 20) == L.E_ALIGN
    out = ctypes.c_int(0)
    assert L.lib().linattn_phi_create(None, ctypes.byref(out)) == L.E_NULL
    pid = mk()
    assert pid >= 16
    assert L.linattn_phi_destroy(pid, check=False) == L.OK
    assert L.linattn_phi_destroy(pid, check=False) == L.E_PHI
    assert L.linattn_phi_destroy(3, check=False) == L.E_PHI


def test_fwd_rejects_bad_calls_before_touching_the_gpu():
    B, H, n, d = 1, 2, 300, 64
    ws = L.linattn_workspace_bytes(B, H, n, d, L.PHI_HEDGEHOG, L.BF16)
    pid = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 8192, workspace=P + (1 << 20), workspace_bytes=ws)
    big = 1 << 24
    q, k, v, o = P + 2 * big, P + 3 * big, P + 4 * big, P + 5 * big
    f = lambda *a, **kw: L.linattn_fwd(*a, **kw, check=False)
    try:
        assert f(q, k, v, o, B, H, n, d, 5) == L.E_PHI
        assert f(q, k, v, o, B, H, n, d, pid + 1) == L.E_PHI
        assert f(None, k, v, o, B, H, n, d, pid) == L.E_NULL
        assert f(q, k, v, None, B, H, n, d, pid) == L.E_NULL
        assert f(q, k, v, o, B, H + 1, n, d, pid) == L.E_SHAPE
        assert f(q, k, v, o, B, H, n, 128, pid) == L.E_SHAPE
        assert f(q, k, v, o, B, H, 0, d, pid) == L.E_SHAPE
        assert f(q, k, v, o, 0, H, n, d, pid) == L.E_SHAPE
        assert f(q + 4, k, v, o, B, H, n, d, pid) == L.E_ALIGN
        assert f(q, k, v, o + 8, B, H, n, d, pid) == L.E_ALIGN
        assert f(q, k, v, q, B, H, n, d, pid) == L.E_ALIAS
        assert f(q, k, v, v + 32, B, H, n, d, pid) == L.E_ALIAS
        # a problem that needs more scratch than the descriptor has
        assert f(q, k, v, o, 64, H, 100000, d, pid) == L.E_WORKSPACE
        with pytest.raises(L.LinattnError) as ei:
            L.linattn_fwd(q, k, v, o, B, H, n, d, 5)
        assert ei.value.status == L.E_PHI
    finally:
        L.linattn_phi_destroy(pid)
    pid2 = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 8192)
    try:
        assert f(q, k, v, o, B, H, n, d, pid2) == L.E_WORKSPACE
    finally:
        L.linattn_phi_destroy(pid2)
    # a state buffer sized for B = 1 serves B = 1 but refuses B = 2 (forward and backward alike)
    ws2 = L.linattn_workspace_bytes(2, H, n, d, L.PHI_HEDGEHOG, L.BF16)
    pid3 = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 8192, state=P + 16384, state_bytes=H * (d + 1) * d * 4,
                                workspace=P + (1 << 20), workspace_bytes=ws2)
    try:
        assert f(q, k, v, o, 2, H, n, d, pid3) == L.E_STATE
        t = [P + (i + 2) * big for i in range(7)]
        assert L.linattn_bwd(*t, 2, H, n, d, pid3, check=False) == L.E_STATE
    finally:
        L.linattn_phi_destroy(pid3)


def test_bwd_rejects_bad_calls():
    B, H, n, d = 1, 2, 300, 64
    ws = L.linattn_workspace_bytes(B, H, n, d, L.PHI_HEDGEHOG, L.BF16)
    pid = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 8192, workspace=P + (1 << 20), workspace_bytes=ws)
    big = 1 << 24
    t = [P + (i + 2) * big for i in range(7)]
    try:
        assert L.linattn_bwd(*t, B, H, n, d, pid, check=False) == L.E_STATE
        assert L.linattn_bwd(*t[:3], None, *t[4:], B, H, n, d, pid, check=False) == L.E_NULL
        assert L.linattn_bwd(*t, B, H, n, d, 2, check=False) == L.E_PHI
    finally:
        L.linattn_phi_destroy(pid)


def test_descriptor_table_reuses_slots():
    ids = [L.linattn_phi_create(L.PHI_HEDGEHOG, L.F32, 1, 64, P, P) for _ in range(8)]
    assert len(set(ids)) == 8
    for i in ids:
        L.linattn_phi_destroy(i)
    again = L.linattn_phi_create(L.PHI_HEDGEHOG, L.F32, 1, 64, P, P)
    assert again in ids
    L.linattn_phi_destroy(again)


def test_blend_pointers_are_checked_on_the_host():
    mk = lambda **kw: L.linattn_phi_create(**{**dict(kind=L.PHI_HEDGEHOG, dtype=L.BF16, H=2, d=64, wq=P, wk=P + 4096), **kw}, check=False)
    assert mk(blend_in=P + 65536) == L.E_NULL                       # softmax branch without r
    assert mk(blend_r=P + 65536) == L.E_NULL                        # r without the softmax branch
    assert mk(blend_dr=P + 65536) == L.E_NULL                       # dr without either
    assert mk(blend_in=P + 65536 + 2, blend_r=P + 4) == L.E_ALIGN
    pid = mk(blend_in=P + 65536, blend_r=P + 4, blend_dr=P + 8)
    assert pid >= 16
    assert L.linattn_phi_set_blend(pid, None, None, None, check=False) == L.OK
    assert L.linattn_phi_set_blend(pid, P + 65536, None, None, check=False) == L.E_NULL
    assert L.linattn_phi_set_blend(pid, P + 65536, P + 4, None, check=False) == L.OK
    assert L.linattn_phi_set_blend(9999, None, None, None, check=False) == L.E_PHI
    assert L.linattn_phi_destroy(pid) == L.OK


def test_blend_input_may_not_alias_the_output():
    B, H, n, d = 1, 2, 256, 64
    ws = L.linattn_workspace_bytes(B, H, n, d, L.PHI_HEDGEHOG, L.BF16)
    q, k, v, out = P + (8 << 20), P + (9 << 20), P + (10 << 20), P + (11 << 20)
    pid = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 8192, workspace=P + (1 << 20), workspace_bytes=ws,
                               blend_in=out + 64, blend_r=P + 16)
    assert L.linattn_fwd(q, k, v, out, B, H, n, d, pid, None, check=False) == L.E_ALIAS
    L.linattn_phi_destroy(pid)


def test_relu_descriptors_take_no_weights_and_no_blend():
    mk = lambda **kw: L.linattn_phi_create(**{**dict(kind=L.PHI_RELU, dtype=L.BF16, H=2, d=64, wq=None, wk=None), **kw}, check=False)
    assert mk(wq=P) == L.E_PHI
    assert mk(dwk=P) == L.E_PHI
    assert mk(blend_in=P + 65536, blend_r=P + 4) == L.E_PHI
    assert mk(d=48) == L.E_SHAPE
    pid = mk()
    assert pid >= 16
    assert L.linattn_phi_set_blend(pid, P + 65536, P + 4, None, check=False) == L.E_PHI
    assert L.linattn_phi_set_blend(pid, None, None, None, check=False) == L.OK
    # same scratch with and without "weight gradients": there are none
    a = L.linattn_workspace_bytes(1, 12, 32760, 128, L.PHI_RELU, L.BF16)
    assert a > 0 and a == L.linattn_workspace_bytes_wgrads(1, 12, 32760, 128, L.PHI_RELU, L.BF16)
    assert L.linattn_workspace_bytes(1, 12, 32760, 128, 3, L.BF16) == 0
    # a call without workspace is refused on the host
    assert L.linattn_fwd(P, P + (1 << 20), P + (2 << 20), P + (3 << 20), 1, 2, 100, 64, pid, None, check=False) == L.E_WORKSPACE
    assert L.linattn_phi_destroy(pid) == L.OK


def test_noalloc_forward_checks_arguments_and_its_limit_on_the_host():
    """linattn_fwd_noalloc needs no workspace in the descriptor, rejects what linattn_fwd rejects, and refuses
    problems whose forward scratch exceeds its static array -- all before any HIP call."""
    header = open(os.path.join(ROOT, "include", "linattn.h")).read()
    limit = re.search(r"#define\s+LINATTN_NOALLOC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", header)
    limit = int(limit.group(1)) << int(limit.group(2))
    assert limit == 32 << 20
    H, d = 2, 128
    pid = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 65536)          # no workspace
    big = 1 << 30
    q, k, v, o = P + big, P + 2 * big, P + 3 * big, P + 4 * big
    f = lambda *a: L.linattn_fwd_noalloc(*a, check=False)
    try:
        assert f(None, k, v, o, 1, H, 64, d, pid, None) == L.E_NULL
        assert f(q, k, v, o, 1, H + 1, 64, d, pid, None) == L.E_SHAPE
        assert f(q, k, v, o + 2, 1, H, 64, d, pid, None) == L.E_ALIGN
        assert f(q, k, v, q, 1, H, 64, d, pid, None) == L.E_ALIAS
        assert f(q, k, v, o, 1, H, 64, d, 3, None) == L.E_PHI
        # 600 (b,h) pairs: one partial and one state each = 600 * 2 * 66048 bytes > 32 MiB
        assert 600 * 2 * (d + 1) * d * 4 > limit
        assert f(q, k, v, o, 300, H, 64, d, pid, None) == L.E_WORKSPACE
    finally:
        L.linattn_phi_destroy(pid)
    # the task's largest configuration fits: partials + states of config 4 (B=2, H=40, n=75600, d=128)
    assert L.linattn_workspace_bytes(2, 40, 75600, 128, L.PHI_HEDGEHOG, L.BF16) > 0


def test_bf16_storage_fp32_arithmetic_dtype_is_accepted_on_the_host():
    """LINATTN_BF16_F32MATH: sized like the fp32 mode's plan (no operand images), tensors of 2 bytes per element."""
    header = open(os.path.join(ROOT, "include", "linattn.h")).read()
    assert re.search(r"#define\s+LINATTN_BF16_F32MATH\s+3\b", header) and L.BF16_F32MATH == 3
    assert L.linattn_workspace_bytes(1, 2, 1000, 128, L.PHI_HEDGEHOG, L.BF16_F32MATH) > 0
    assert L.linattn_workspace_bytes(1, 2, 1000, 128, L.PHI_HEDGEHOG, 4) == 0
    H, d = 2, 128
    ws = L.linattn_workspace_bytes(1, H, 500, d, L.PHI_HEDGEHOG, L.BF16_F32MATH)
    pid = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16_F32MATH, H, d, P, P + 65536, workspace=P + (1 << 20), workspace_bytes=ws)
    big = 1 << 30
    q, k, v, o = P + big, P + 2 * big, P + 3 * big, P + 4 * big
    try:
        # tensors are 2 bytes per element: out right behind q (B*H*n*d*2 bytes further) does not alias it
        nbytes = 1 * H * 500 * d * 2
        assert L.linattn_fwd(q, k, v, q + nbytes - 16, 1, H, 500, d, pid, None, check=False) == L.E_ALIAS
        assert L.linattn_fwd(None, k, v, o, 1, H, 500, d, pid, None, check=False) == L.E_NULL
    finally:
        L.linattn_phi_destroy(pid)
    assert L.linattn_phi_create(L.PHI_HEDGEHOG, 4, H, d, P, P + 65536, check=False) == L.E_DTYPE


def test_descriptor_flags_are_checked_on_the_host():
    """LINATTN_FLAG_CENTRED goes with the Eq. 5 map in LINATTN_BF16 only; unknown flag bits are refused."""
    header = open(os.path.join(ROOT, "include", "linattn.h")).read()
    assert re.search(r"#define\s+LINATTN_FLAG_CENTRED\s+1u\b", header) and L.FLAG_CENTRED == 1
    H, d = 2, 128
    pid = L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 65536, flags=L.FLAG_CENTRED)
    assert pid >= 16 and L.linattn_phi_destroy(pid) == L.OK
    assert L.linattn_phi_create(L.PHI_HEDGEHOG, L.F32, H, d, P, P + 65536, flags=L.FLAG_CENTRED, check=False) == L.E_PHI
    assert L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16_F32MATH, H, d, P, P + 65536, flags=L.FLAG_CENTRED, check=False) == L.E_PHI
    assert L.linattn_phi_create(L.PHI_RELU, L.BF16, H, d, None, None, flags=L.FLAG_CENTRED, check=False) == L.E_PHI
    assert L.linattn_phi_create(L.PHI_HEDGEHOG, L.BF16, H, d, P, P + 65536, flags=2, check=False) == L.E_PHI
