"""CPU-only checks of the C ABI: the library loads, exports what the header declares, rejects bad
arguments before touching a device, and expands seeds to exactly the oracle's W."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2510_04008_amd as ra
from oracle import race_oracle as ro

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "race_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(race_[a-z_]+)\s*\(", header))
    assert {"race_attn_fwd", "race_attn_bwd", "race_attn_workspace_bytes", "race_attn_expand_projection",
            "race_attn_debug_hash", "race_attn_debug_buckets", "race_status_string"} <= names
    lib = ra.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    lib = ra.lib()
    texts = [lib.race_status_string(i).decode() for i in range(7)]
    assert texts[0] == "ok" and len(set(texts)) == 7 and all(texts)
    assert lib.race_attn_last_error().decode() == ""


def _desc(**kw):
    base = dict(B=1, H=2, N=100, d=64, L=4, P=4, sharpening=8.0, causal=False, dtype=ra.RACE_F32, chunk=0)
    base.update(kw)
    return ra.make_desc(**base)


@pytest.mark.parametrize("bad", [dict(B=0), dict(H=0), dict(N=-1), dict(d=0), dict(L=0), dict(P=0),
                                 dict(sharpening=0.0), dict(sharpening=-1.0), dict(sharpening=float("nan")),
                                 dict(sharpening=float("-inf")), dict(dtype=7), dict(chunk=-5)])
def test_invalid_descriptors_are_rejected(bad):
    d = _desc(**bad)
    if "causal" not in bad:
        assert ra.race_attn_workspace_bytes(d) == 0
    lib = ra.lib()
    fake = ctypes.c_void_p(256)
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    st = lib.race_attn_fwd(ctypes.byref(d), fake, fake, fake, seeds, fake, fake, fake, 1 << 40, None)
    assert st == ra.RACE_ERR_INVALID_ARG


def test_unit_norm_option_is_a_flag():
    d = _desc()
    assert d.unit_qk == 0 and ra.race_attn_workspace_bytes(d) > 0
    d1 = _desc(unit_qk=True)
    assert d1.unit_qk == 1 and ra.race_attn_workspace_bytes(d1) == ra.race_attn_workspace_bytes(d)
    d1.unit_qk = 2
    assert ra.race_attn_workspace_bytes(d1) == 0
    fake = ctypes.c_void_p(256)
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    st = ra.lib().race_attn_fwd(ctypes.byref(d1), fake, fake, fake, seeds, fake, fake, fake, 1 << 40, None)
    assert st == ra.RACE_ERR_INVALID_ARG


def test_infinite_temperature_is_the_hard_hash_forward_only():
    d = _desc(sharpening=float("inf"))
    need = ra.race_attn_workspace_bytes(d)
    assert need > 0
    lib = ra.lib()
    p = [ctypes.c_void_p(256 * (i + 1)) for i in range(10)]
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    ok_ws = ctypes.c_void_p(1 << 20)
    for entry in (lib.race_attn_bwd_beta, lib.race_attn_bwd_saved):
        assert entry(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], None, ok_ws, need, None) == ra.RACE_ERR_UNSUPPORTED
    assert lib.race_attn_bwd(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], ok_ws, need, None) == ra.RACE_ERR_UNSUPPORTED


def test_causal_flag_must_be_0_or_1():
    d = _desc()
    d.causal = 2
    assert ra.race_attn_workspace_bytes(d) == 0


@pytest.mark.parametrize("bad", [dict(P=9), dict(d=260), dict(d=60), dict(d=264), dict(P=8, d=256)])
def test_unsupported_shapes(bad):
    d = _desc(**bad)
    assert ra.race_attn_workspace_bytes(d) == 0 and ra.race_attn_kernel_family(d) == 0
    fake = ctypes.c_void_p(256)
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    st = ra.lib().race_attn_fwd(ctypes.byref(d), fake, fake, fake, seeds, fake, fake, fake, 1 << 40, None)
    assert st == ra.RACE_ERR_UNSUPPORTED


def test_null_pointers_workspace_and_aliasing_are_checked_before_any_launch():
    lib = ra.lib()
    d = _desc()
    need = ra.race_attn_workspace_bytes(d)
    assert need > 0 and need % 256 == 0
    p = [ctypes.c_void_p(256 * (i + 1)) for i in range(12)]
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    ok_ws = ctypes.c_void_p(1 << 20)
    assert lib.race_attn_fwd(None, p[0], p[1], p[2], seeds, p[3], p[4], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_fwd(ctypes.byref(d), None, p[1], p[2], seeds, p[3], p[4], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_fwd(ctypes.byref(d), p[0], p[1], p[2], None, p[3], p[4], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_fwd(ctypes.byref(d), p[0], p[1], p[2], seeds, p[2], p[4], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_fwd(ctypes.byref(d), p[0], p[1], p[2], seeds, p[3], p[4], None, need, None) == ra.RACE_ERR_WORKSPACE
    assert lib.race_attn_fwd(ctypes.byref(d), p[0], p[1], p[2], seeds, p[3], p[4], ok_ws, need - 1, None) == ra.RACE_ERR_WORKSPACE
    assert lib.race_attn_fwd(ctypes.byref(d), p[0], p[1], p[2], seeds, p[3], p[4], ctypes.c_void_p(1000), need, None) == ra.RACE_ERR_WORKSPACE
    assert lib.race_attn_bwd(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], None, ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_bwd(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[6], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_bwd(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], ok_ws, 0, None) == ra.RACE_ERR_WORKSPACE
    # the temperature's cotangent is optional, but must not alias anything if given
    assert lib.race_attn_bwd_beta(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], p[6], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_bwd_beta(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], p[0], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_bwd_beta(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], p[9], ok_ws, 0, None) == ra.RACE_ERR_WORKSPACE
    assert lib.race_attn_bwd_beta(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], None, ok_ws, 0, None) == ra.RACE_ERR_WORKSPACE
    # the variant that reads the forward's workspace checks its arguments the same way
    assert lib.race_attn_bwd_saved(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], None, None, ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_bwd_saved(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], p[7], ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_bwd_saved(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], None, None, need, None) == ra.RACE_ERR_WORKSPACE
    assert lib.race_attn_bwd_saved(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], None, ok_ws, need - 1, None) == ra.RACE_ERR_WORKSPACE
    assert lib.race_attn_debug_hash(ctypes.byref(d), p[0], seeds, None, None, ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_debug_buckets(ctypes.byref(d), p[0], p[1], seeds, p[2], None, ok_ws, need, None) == ra.RACE_ERR_INVALID_ARG


def test_empty_sequence_is_a_no_op():
    d = _desc(N=0)
    assert ra.race_attn_workspace_bytes(d) == 0
    p = [ctypes.c_void_p(256 * (i + 1)) for i in range(10)]
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    lib = ra.lib()
    assert lib.race_attn_fwd(ctypes.byref(d), p[0], p[1], p[2], seeds, p[3], p[4], None, 0, None) == ra.RACE_OK
    assert lib.race_attn_bwd(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], None, 0, None) == ra.RACE_OK
    assert lib.race_attn_bwd_beta(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], p[9], None, 0, None) == ra.RACE_OK
    assert lib.race_attn_bwd_saved(ctypes.byref(d), p[0], p[1], p[2], p[3], p[4], p[5], seeds, p[6], p[7], p[8], p[9], None, 0, None) == ra.RACE_OK


def test_workspace_grows_with_the_problem_and_families_are_reported():
    small = ra.race_attn_workspace_bytes(_desc(N=1000))
    big = ra.race_attn_workspace_bytes(_desc(N=100000))
    assert 0 < small < big
    assert ra.race_attn_kernel_family(_desc()) == 1            # fp32 is served by the generic kernels


@pytest.mark.parametrize("H,L,P,d,dtype", [(1, 4, 4, 64, ra.RACE_F32), (4, 8, 6, 128, ra.RACE_BF16),
                                           (3, 3, 3, 8, ra.RACE_F32), (2, 1, 1, 16, ra.RACE_BF16)])
def test_projection_expansion_is_bit_identical_to_the_oracle(H, L, P, d, dtype):
    seeds = [1, (1 << 63) + 12345, 0, 0xFFFFFFFFFFFFFFFF][:H]
    desc = ra.make_desc(1, H, 16, d, L, P, 8.0, False, dtype)
    W = ra.race_attn_expand_projection(desc, seeds)
    assert W.shape == (H, L * P, d) and W.dtype == np.float32
    for h in range(H):
        ref = ro.expand_projection(seeds[h], L, P, d, round_bf16=(dtype == ra.RACE_BF16)).astype(np.float32)
        assert np.array_equal(W[h].view(np.uint32), ref.view(np.uint32))


def test_calibration_copy_rejects_bad_arguments_on_the_host():
    lib = ra.lib()
    buf = ctypes.create_string_buffer(4096 + 64)
    base = (ctypes.addressof(buf) + 63) // 64 * 64
    assert lib.race_attn_calibration_copy(None, None, 0, None) == ra.RACE_OK            # nothing to copy
    assert lib.race_attn_calibration_copy(None, base, 64, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_calibration_copy(base, None, 64, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_calibration_copy(base + 1024, base, 24, None) == ra.RACE_ERR_INVALID_ARG   # not a multiple of 16
    assert lib.race_attn_calibration_copy(base + 1028, base, 64, None) == ra.RACE_ERR_INVALID_ARG   # misaligned
    assert lib.race_attn_calibration_copy(base + 32, base, 64, None) == ra.RACE_ERR_INVALID_ARG     # overlapping


def test_calibration_mfma_rejects_bad_arguments_on_the_host():
    lib = ra.lib()
    fake = ctypes.c_void_p(4096)
    assert lib.race_attn_calibration_mfma(1, 1, 0, None, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_calibration_mfma(0, 1, 0, fake, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_calibration_mfma(1, 0, 0, fake, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_calibration_mfma((1 << 20) + 1, 1, 0, fake, None) == ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_calibration_mfma(1, 1, 3, fake, None) == ra.RACE_ERR_INVALID_ARG


def test_decode_entry_points_check_arguments_on_the_host():
    lib = ra.lib()
    d = _desc()
    assert ra.race_attn_state_bytes(d) == d.B * d.H * d.L * (1 << d.P) * (d.d + 1) * 4
    assert ra.race_attn_state_bytes(_desc(N=0)) == ra.race_attn_state_bytes(_desc(N=10 ** 6))     # no N in it
    assert ra.race_attn_state_bytes(_desc(P=0)) == 0 and ra.race_attn_step_workspace_bytes(_desc(L=0)) == 0
    need = ra.race_attn_step_workspace_bytes(d)
    assert need > 0 and need % 256 == 0
    p = [ctypes.c_void_p(256 * (i + 1)) for i in range(8)]
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    ok_ws = ctypes.c_void_p(1 << 20)
    E = ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_step(ctypes.byref(d), None, p[1], p[2], seeds, p[3], p[4], p[5], ok_ws, need, None) == E
    assert lib.race_attn_step(ctypes.byref(d), p[0], p[1], p[2], seeds, None, p[4], p[5], ok_ws, need, None) == E
    assert lib.race_attn_step(ctypes.byref(d), p[0], p[1], p[2], seeds, p[3], p[2], p[5], ok_ws, need, None) == E
    assert lib.race_attn_step(ctypes.byref(d), p[0], p[1], p[2], seeds, p[3], p[4], p[5], ok_ws, need - 1, None) == ra.RACE_ERR_WORKSPACE
    assert lib.race_attn_state_init(ctypes.byref(d), p[0], p[1], seeds, None, ok_ws, 1 << 30, None) == E
    assert lib.race_attn_state_init(ctypes.byref(d), p[0], p[1], seeds, p[0], ok_ws, 1 << 30, None) == E
    assert lib.race_attn_state_init(ctypes.byref(d), p[0], p[1], seeds, p[2], ok_ws, 0, None) == ra.RACE_ERR_WORKSPACE


def test_forward_on_built_in_scratch_checks_everything_on_the_host():
    """race_attn_fwd_static (for callers that cannot allocate) validates like race_attn_fwd, refuses seeds whose pinned
    image no earlier call has made (making it would allocate) and problems beyond its 32 MiB array: all before any
    device call, so this runs without a GPU."""
    lib = ra.lib()
    d = _desc()
    p = [ctypes.c_void_p(256 * (i + 1)) for i in range(6)]
    seeds = (ctypes.c_uint64 * 2)(0xABCDEF12345, 77)          # used nowhere else in this process
    E = ra.RACE_ERR_INVALID_ARG
    assert lib.race_attn_fwd_static(None, p[0], p[1], p[2], seeds, p[3], p[4], None) == E
    assert lib.race_attn_fwd_static(ctypes.byref(d), None, p[1], p[2], seeds, p[3], p[4], None) == E
    assert lib.race_attn_fwd_static(ctypes.byref(d), p[0], p[1], p[2], None, p[3], p[4], None) == E
    assert lib.race_attn_fwd_static(ctypes.byref(d), p[0], p[1], p[2], seeds, p[1], p[4], None) == E
    assert lib.race_attn_fwd_static(ctypes.byref(_desc(P=9)), p[0], p[1], p[2], seeds, p[3], p[4], None) == ra.RACE_ERR_UNSUPPORTED
    assert lib.race_attn_fwd_static(ctypes.byref(_desc(N=0)), None, None, None, None, None, None, None) == ra.RACE_OK
    assert lib.race_attn_fwd_static(ctypes.byref(d), p[0], p[1], p[2], seeds, p[3], p[4], None) == ra.RACE_ERR_NOT_READY
    assert b"not been prepared" in lib.race_attn_last_error()
    # 200 heads of the headline shape need 200 x 258 KiB of statistics even with one segment each
    big = ra.make_desc(1, 200, 4096, 128, 8, 6, 8.0, True, ra.RACE_BF16)
    many = (ctypes.c_uint64 * 200)(*range(200))
    assert lib.race_attn_fwd_static(ctypes.byref(big), p[0], p[1], p[2], many, p[3], p[4], None) == ra.RACE_ERR_WORKSPACE
    assert b"32 MiB" in lib.race_attn_last_error()


def test_generic_kernels_refuse_long_contexts():
    """The generic kernels keep per-table partial results of every token (L * N * d floats per pass): beyond 16 GiB of
    them the descriptor is unsupported instead of asking for a workspace the design was never meant for."""
    ok = _desc(N=1 << 20)                                  # fp32, H = 2, d = 64, L = 4: 6 GiB of partial results
    assert ra.race_attn_kernel_family(ok) == 1 and ra.race_attn_workspace_bytes(ok) > 0
    big = _desc(N=1 << 22)                                 # 24 GiB
    assert ra.race_attn_kernel_family(big) == 0 and ra.race_attn_workspace_bytes(big) == 0
    fake = ctypes.c_void_p(256)
    seeds = (ctypes.c_uint64 * 2)(1, 2)
    st = ra.lib().race_attn_fwd(ctypes.byref(big), fake, fake, fake, seeds, fake, fake, fake, 1 << 50, None)
    assert st == ra.RACE_ERR_UNSUPPORTED
    # the same shape in bf16 at the MFMA family's headline shape has no such limit
    long_bf16 = ra.make_desc(1, 4, 1 << 25, 128, 8, 6, 8.0, True, ra.RACE_BF16)
    assert ra.race_attn_kernel_family(long_bf16) == 2 and ra.race_attn_workspace_bytes(long_bf16) > 0


def test_the_force_generic_switch_is_read_at_every_call():
    d = ra.make_desc(1, 2, 1000, 128, 8, 6, 8.0, True, ra.RACE_BF16)
    assert ra.race_attn_kernel_family(d) == 2
    os.environ["RACE_ATTN_FORCE_GENERIC"] = "1"
    try:
        assert ra.race_attn_kernel_family(d) == 1
    finally:
        del os.environ["RACE_ATTN_FORCE_GENERIC"]
    assert ra.race_attn_kernel_family(d) == 2
