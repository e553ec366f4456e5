"""The C-ABI library loads without a GPU, exports every symbol include/*.h
declare, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2402_02320_amd import spin
    if not os.path.exists(spin.LIB_PATH):
        from paper_2402_02320_amd import build
        build.build()
    return spin.lib()


def declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(spin[0-9]*_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_five_calls():
    syms = declared_symbols()
    for name in ("spin_share", "spin_open", "spin_beaver_matmul", "spin_beaver_mul", "spin_trunc"):
        assert name in syms


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    for expected in ("spin128_beaver_matmul", "spin_bshare", "spin_lincomb_trunc", "spin_profile_read"):
        assert expected in names
    for name in names:
        assert getattr(L, name) is not None


def test_argument_validation_needs_no_gpu(L):
    fake = ctypes.c_void_p(0x1000)          # aligned, never dereferenced: validation rejects first
    odd = ctypes.c_void_p(0x1008)
    EINVAL, ERANGE, EWORKSPACE = 1, 2, 3
    assert L.spin_share(None, 8, 2, 1, 1, fake, None) == EINVAL
    assert L.spin_share(fake, 0, 2, 1, 1, fake, None) == EINVAL
    assert L.spin_share(fake, 8, 0, 1, 1, fake, None) == EINVAL
    assert L.spin_share(fake, 8, 9, 1, 1, fake, None) == EINVAL
    assert L.spin_share(odd, 8, 2, 1, 1, fake, None) == EINVAL
    assert L.spin_share(fake, 1 << 40, 2, 1, 1, fake, None) == ERANGE
    assert L.spin_open(fake, None, 8, 9, fake, None) == EINVAL
    assert L.spin_open(fake, odd, 8, 2, fake, None) == EINVAL
    assert L.spin_random(None, 8, 1, 1, 1, 0, None) == EINVAL
    assert L.spin_beaver_mul(2, 8, fake, fake, fake, fake, None, fake, None) == EINVAL
    assert L.spin_trunc(2, 8, 0, fake, fake, fake, fake, fake, None) == EINVAL
    assert L.spin_trunc(2, 8, 62, fake, fake, fake, fake, fake, None) == EINVAL
    assert L.spin_trunc(2, 8, 16, fake, fake, fake, None, fake, None) == EINVAL
    # the call on the built-in workspace refuses, before any launch, what does not fit its 64 MiB
    st = L.spin_beaver_matmul_static
    assert st(2, 1, 2048, 2048, 2048, fake, fake, fake, fake, fake, fake, 0, None) == EWORKSPACE
    assert st(2, 1, 0, 8, 8, fake, fake, fake, fake, fake, fake, 0, None) == EINVAL
    assert st(2, 1, 8, 8, 8, fake, None, fake, fake, fake, fake, 0, None) == EINVAL
    mm = L.spin_beaver_matmul
    assert mm(2, 1, 0, 4, 4, fake, fake, fake, fake, fake, fake, 0, fake, 1 << 30, None) == EINVAL
    assert mm(2, 1, 4, 4, 4, fake, fake, fake, fake, fake, fake, 7, fake, 1 << 30, None) == EINVAL
    assert mm(2, 1, 4, 4, 4, fake, fake, fake, fake, fake, fake, 0, None, 0, None) == EWORKSPACE
    assert mm(2, 1, 4, 4, 4, fake, fake, fake, fake, fake, fake, 0, fake, 16, None) == EWORKSPACE
    assert mm(2, 1, 1 << 25, 4, 4, fake, fake, fake, fake, fake, fake, 0, fake, 1 << 30, None) == ERANGE
    nt = L.spin_beaver_matmul_nt
    assert nt(2, 1, 4, 4, 4, fake, None, fake, fake, fake, fake, 0, fake, 1 << 30, None) == EINVAL
    assert nt(2, 1, 4, 4, 4, fake, fake, fake, fake, fake, fake, 1, fake, 16, None) == EWORKSPACE


def test_workspace_query(L):
    q = L.spin_beaver_matmul_workspace_bytes
    assert q(0, 1, 4, 4, 4, 0) == 0 and q(2, 1, 4, 4, 4, 5) == 0
    # VALU path: E and F as plain ring matrices
    assert q(3, 2, 10, 7, 5, 1) == 8 * 2 * (10 * 5 + 5 * 7)
    # limb path: n+1 digit-fragment copies of the padded operands, 8 bytes per padded element
    got = q(5, 1, 4096, 4096, 4096, 0)
    assert got == 8 * 6 * (4096 * 4096 * 2)
    assert q(3, 1, 64, 64, 64, 0) >= 8 * 4 * (64 * 64 * 2)


def test_validation_of_the_wider_entry_points(L):
    fake = ctypes.c_void_p(0x1000)
    EINVAL, EWORKSPACE = 1, 3
    assert L.spin128_trunc(2, 8, 126, fake, fake, fake, fake, fake, None) == EINVAL
    assert L.spin128_trunc(2, 8, 0, fake, fake, fake, fake, fake, None) == EINVAL
    assert L.spin128_share(fake, 8, 9, 1, 1, fake, None) == EINVAL
    assert L.spin128_beaver_matmul(2, 1, 4, 4, 4, fake, fake, fake, fake, fake, fake, 0, None, 0, None) == EWORKSPACE
    q = L.spin128_beaver_matmul_workspace_bytes
    assert q(3, 2, 10, 7, 5, 1) == 16 * 2 * (10 * 5 + 5 * 7)
    assert q(2, 1, 2048, 2048, 2048, 0) == 16 * 3 * (2048 * 2048 * 2)
    assert L.spin_beaver_and(2, 8, fake, fake, fake, fake, None, fake, None) == EINVAL
    assert L.spin_bopen(fake, None, 0, 2, fake, None) == EINVAL
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    coef = (ctypes.c_uint64 * 2)(1, 2)
    assert L.spin_lincomb_trunc(2, 8, 9, ptrs, coef, 0, 0, None, None, None, fake, None) == EINVAL
    assert L.spin_lincomb_trunc(2, 8, 2, ptrs, coef, 0, 16, None, None, None, fake, None) == EINVAL
    assert L.spin_lincomb_trunc(2, 8, 2, None, coef, 0, 0, None, None, None, fake, None) == EINVAL


def test_status_strings(L):
    assert L.spin_status_string(0) == b"ok"
    assert b"workspace" in L.spin_status_string(3)
    assert L.spin_last_hip_error() == b""


def test_validation_of_the_32_bit_entry_points(L):
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    EINVAL, ERANGE, EWORKSPACE = 1, 2, 3
    assert L.spin32_share(fake, 8, 9, 1, 1, fake, None) == EINVAL
    assert L.spin32_share(odd, 8, 2, 1, 1, fake, None) == EINVAL
    assert L.spin32_open(fake, None, 0, 2, fake, None) == EINVAL
    assert L.spin32_trunc(2, 8, 30, fake, fake, fake, fake, fake, None) == EINVAL
    assert L.spin32_trunc(2, 8, 0, fake, fake, fake, fake, fake, None) == EINVAL
    assert L.spin32_beaver_mul(2, 8, fake, fake, None, fake, fake, fake, None) == EINVAL
    assert L.spin_cast_64_to_32(fake, 0, fake, None) == EINVAL
    assert L.spin_cast_64_to_32(None, 8, fake, None) == EINVAL
    assert L.spin_cast_64_to_32(fake, 1 << 40, fake, None) == ERANGE
    mm = L.spin32_beaver_matmul
    assert mm(2, 1, 4, 4, 4, fake, fake, fake, fake, fake, fake, 0, None, 0, None) == EWORKSPACE
    assert mm(2, 1, 4, 0, 4, fake, fake, fake, fake, fake, fake, 0, fake, 1 << 30, None) == EINVAL
    q = L.spin32_beaver_matmul_workspace_bytes
    assert q(3, 2, 10, 7, 5, 1) == 4 * 2 * (10 * 5 + 5 * 7)
    # limb path: n+1 digit-fragment copies of the operands padded to 128 x 128 tiles, 4 bytes per element
    assert q(2, 1, 1024, 1024, 1024, 0) == 4 * 3 * (1024 * 1024 * 2)
    assert q(2, 1, 100, 100, 100, 0) == 4 * 3 * (128 * 128 * 2)


def test_validation_of_the_tiled_multiplication(L):
    fake = ctypes.c_void_p(0x1000)
    EINVAL, ERANGE = 1, 2
    f = L.spin_beaver_mul_bcast
    assert f(2, 0, 4, 4, 1, fake, fake, fake, fake, fake, fake, None) == EINVAL
    assert f(2, 4, 4, 4, 1, fake, fake, None, fake, fake, fake, None) == EINVAL
    assert f(9, 4, 4, 4, 0, fake, fake, fake, fake, fake, fake, None) == EINVAL
    assert f(2, 1 << 20, 1 << 20, 4, 0, fake, fake, fake, fake, fake, fake, None) == ERANGE


def test_validation_of_the_fused_multiplication(L):
    fake = ctypes.c_void_p(0x1000)
    EINVAL = 1
    f = L.spin_beaver_mul_trunc
    assert f(2, 8, 0, fake, fake, fake, fake, fake, fake, fake, fake, fake, None) == EINVAL
    assert f(2, 8, 62, fake, fake, fake, fake, fake, fake, fake, fake, fake, None) == EINVAL
    assert f(2, 8, 16, fake, fake, fake, fake, fake, fake, None, fake, fake, None) == EINVAL
    assert f(2, 0, 16, fake, fake, fake, fake, fake, fake, fake, fake, fake, None) == EINVAL


def test_validation_of_the_grouped_matmul(L):
    from paper_2402_02320_amd.spin import _MatmulGroup
    EINVAL, ERANGE, EWORKSPACE = 1, 2, 3
    fake = 0x1000
    desc = (_MatmulGroup * 2)()
    for d in desc:
        d.batch, d.M, d.N, d.K = 1, 8, 8, 8
        d.X = d.Y = d.A = d.B = d.C = d.Z = fake
    ws = ctypes.c_void_p(0x10000)
    f, q = L.spin_beaver_matmul_grouped, L.spin_beaver_matmul_grouped_workspace_bytes
    # limb path: every group has its own fragment stores (the packs of all groups run before the GEMMs); the
    # baseline path runs the groups one after another on one workspace
    assert q(2, 2, desc, 0) == 2 * L.spin_beaver_matmul_workspace_bytes(2, 1, 8, 8, 8, 0)
    assert q(2, 2, desc, 1) == L.spin_beaver_matmul_workspace_bytes(2, 1, 8, 8, 8, 1)
    assert f(2, 0, desc, 0, ws, 1 << 30, None) == EINVAL
    assert f(2, 65, desc, 0, ws, 1 << 30, None) == EINVAL
    assert f(2, 2, None, 0, ws, 1 << 30, None) == EINVAL
    assert f(2, 2, desc, 0, ws, 16, None) == EWORKSPACE
    desc[1].K = 0                                            # the second group is bad: nothing may be launched
    assert f(2, 2, desc, 0, ws, 1 << 30, None) == EINVAL
    assert q(2, 2, desc, 0) == 0
    desc[1].K = 1 << 25
    assert f(2, 2, desc, 0, ws, 1 << 30, None) == ERANGE
    desc[1].K = 8
    desc[1].Z = None
    assert f(2, 2, desc, 0, ws, 1 << 30, None) == EINVAL
