"""The C-ABI boundary without a GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "velora.h")


@pytest.fixture(scope="module")
def vl():
    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    return vl


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(velora_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(vl):
    names = _declared_symbols()
    assert {"velora_init_v", "velora_compress", "velora_reconstruct", "velora_weight_grad",
            "velora_weight_grad_factor", "velora_expand_factor", "velora_update_v", "velora_compress_update",
            "velora_workspace_bytes", "velora_status_string", "velora_version"} <= set(names)
    lib = ctypes.CDLL(vl.lib_path())
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/velora.h but not exported"
    from paper_2405_17991_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_library_does_not_read_the_environment(vl):
    # a call depends on its arguments and the device alone: the shipped library imports no getenv
    # (the measurement knobs of the weight-gradient planner only exist in -DVELORA_TUNING builds)
    import subprocess
    out = subprocess.run(["nm", "-D", "--undefined-only", vl.lib_path()], check=True, stdout=subprocess.PIPE,
                         text=True).stdout
    assert "getenv" not in out


def test_workspace_query_is_repeatable(vl):
    # the planner remembers its answers per thread; the same question must keep the same answer, also after
    # more distinct shapes than it remembers have gone through
    from paper_2405_17991_amd.binding import raw
    q = lambda N, D, O, M: int(raw.velora_workspace_bytes(vl.OP_WEIGHT_GRAD, N, D, O, M, vl.BF16))
    first = {(N, M): q(N, 1024, 512, M) for N in (256, 4096, 16384) for M in (1, 4, 16, 64, 128, 256, 512)}
    for _ in range(2):
        for (N, M), need in first.items():
            assert q(N, 1024, 512, M) == need and need > 0


def test_version_and_status_strings(vl):
    assert vl.velora_version() >= 100
    for code, name in vl.STATUS.items():
        assert vl.velora_status_string(code).startswith(name)
    assert "unknown" in vl.velora_status_string(99)


P = 0x7F0000001000      # a 4096-aligned, never dereferenced "device pointer"


def test_compress_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    c = raw.velora_compress
    assert c(None, P, 4, 8, 2, vl.BF16, P, None) == 1
    assert c(P, None, 4, 8, 2, vl.BF16, P, None) == 1
    assert c(P, P, 4, 8, 2, vl.BF16, None, None) == 1
    assert c(P, P, 4, 8, 2, 7, P, None) == 3
    assert c(P, P, 0, 8, 2, vl.BF16, P, None) == 2
    assert c(P, P, 4, 8, 3, vl.BF16, P, None) == 2          # M does not divide D
    assert c(P, P, 4, 8, 0, vl.BF16, P, None) == 2
    assert c(P, P, 4, 8, 16, vl.BF16, P, None) == 2         # M > D
    assert c(P, P, -1, 8, 2, vl.F32, P, None) == 2
    assert c(P + 1, P, 4, 8, 2, vl.BF16, P, None) == 4      # odd address for a 2-byte type
    assert c(P + 2, P, 4, 8, 2, vl.F32, P, None) == 4
    assert c(P, P + 2, 4, 8, 2, vl.BF16, P, None) == 4      # v is float32
    # the one cell of configuration 5 whose sub-token size does not divide D
    assert c(P, P, 16384, 13824, 13, vl.BF16, P, None) == 2


def test_weight_grad_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    w = raw.velora_weight_grad
    N, O, D, M = 64, 32, 16, 4
    need = vl.velora_workspace_bytes(vl.OP_WEIGHT_GRAD, N, D, O, M, vl.BF16)
    assert need > 0
    ok = (P, P, P, N, O, D, M, vl.BF16, P, vl.F32, 0, P, need, None)

    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return w(*a)

    assert call(a0=None) == 1 and call(a1=None) == 1 and call(a2=None) == 1 and call(a8=None) == 1
    assert call(a7=5) == 3 and call(a9=5) == 3
    assert call(a3=0) == 2 and call(a4=0) == 2 and call(a6=3) == 2 and call(a5=-16) == 2
    assert call(a0=P + 1) == 4 and call(a8=P + 2) == 4
    assert call(a11=None) == 5
    assert call(a12=need - 1) == 5


def test_init_v_and_reconstruct_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    need = vl.velora_workspace_bytes(vl.OP_INIT_V, 64, 16, 0, 4, vl.F32)
    assert need > 0
    i = raw.velora_init_v
    assert i(None, 64, 16, 4, vl.F32, P, P, need, None) == 1
    assert i(P, 64, 16, 4, vl.F32, None, P, need, None) == 1
    assert i(P, 64, 16, 5, vl.F32, P, P, need, None) == 2
    assert i(P, 64, 16, 4, 9, P, P, need, None) == 3
    assert i(P, 64, 16, 4, vl.F32, P, None, need, None) == 5
    assert i(P, 64, 16, 4, vl.F32, P, P, need - 1, None) == 5
    assert i(P + 2, 64, 16, 4, vl.F32, P, P, need, None) == 4
    r = raw.velora_reconstruct
    assert r(None, P, 4, 8, 2, vl.BF16, P, None) == 1
    assert r(P, P, 4, 8, 3, vl.BF16, P, None) == 2
    assert r(P, P, 4, 8, 2, 4, P, None) == 3
    assert r(P, P, 4, 8, 2, vl.BF16, P + 1, None) == 4


def test_factor_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    need = vl.velora_workspace_bytes(vl.OP_WEIGHT_GRAD_FACTOR, 64, 4, 32, 4, vl.BF16)
    assert need > 0
    f = raw.velora_weight_grad_factor
    assert f(None, P, 64, 32, 4, vl.BF16, P, P, need, None) == 1
    assert f(P, P, 64, 32, 4, vl.BF16, None, P, need, None) == 1
    assert f(P, P, 64, 0, 4, vl.BF16, P, P, need, None) == 2
    assert f(P, P, 64, 32, 4, 3, P, P, need, None) == 3
    assert f(P + 1, P, 64, 32, 4, vl.BF16, P, P, need, None) == 4
    assert f(P, P, 64, 32, 4, vl.BF16, P, None, need, None) == 5
    assert f(P, P, 64, 32, 4, vl.BF16, P, P, need - 1, None) == 5
    e = raw.velora_expand_factor
    assert e(None, P, 32, 16, 4, P, vl.F32, 0, None) == 1
    assert e(P, P, 32, 16, 3, P, vl.F32, 0, None) == 2
    assert e(P, P, 32, 16, 4, P, 8, 0, None) == 3
    assert e(P, P, 32, 16, 4, P + 2, vl.F32, 0, None) == 4


def test_swiglu_compress_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    f = raw.velora_swiglu_compress
    assert f(None, P, P, 8, 16, 4, vl.BF16, P, P, None) == 1
    assert f(P, P, P, 8, 16, 4, vl.BF16, None, P, None) == 1
    assert f(P, P, P, 8, 16, 4, 9, P, P, None) == 3
    assert f(P, P, P, 8, 16, 5, vl.BF16, P, P, None) == 2
    assert f(P, P, P, 0, 16, 4, vl.BF16, P, P, None) == 2
    assert f(P, P + 1, P, 8, 16, 4, vl.BF16, P, P, None) == 4
    assert f(P, P, P + 2, 8, 16, 4, vl.F32, P, P, None) == 4


def test_linear_compress_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    f = raw.velora_linear_compress
    assert f(None, P, P, 8, 16, 4, 4, vl.BF16, P, P, None) == 1
    assert f(P, P, P, 8, 16, 4, 4, vl.BF16, P, None, None) == 1
    assert f(P, P, P, 8, 16, 4, 4, 9, P, P, None) == 3
    assert f(P, P, P, 8, 16, 4, 5, vl.BF16, P, P, None) == 2                    # M does not divide D
    assert f(P, P, P, 8, 16, 0, 4, vl.BF16, P, P, None) == 2                    # O < 1
    assert f(P, P, P, 8, 16, 65535 * 64 + 1, 4, vl.BF16, P, P, None) == 2       # O beyond the grid limit
    assert f(P, P + 1, P, 8, 16, 4, 4, vl.BF16, P, P, None) == 4
    assert f(P, P, P + 2, 8, 16, 4, 4, vl.F32, P, P, None) == 4


def test_grad_input_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    f = raw.velora_grad_input
    assert f(None, P, 8, 4, 16, vl.BF16, P, None) == 1
    assert f(P, P, 8, 4, 16, vl.BF16, None, None) == 1
    assert f(P, P, 8, 4, 16, 9, P, None) == 3
    assert f(P, P, 0, 4, 16, vl.BF16, P, None) == 2
    assert f(P, P, 8, 4, 65535 * 64 + 1, vl.BF16, P, None) == 2
    assert f(P, P + 1, 8, 4, 16, vl.BF16, P, None) == 4
    assert f(P, P, 8, 4, 16, vl.F32, P + 2, None) == 4


def test_rmsnorm_compress_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    f = raw.velora_rmsnorm_compress
    assert f(None, P, 1e-6, P, 8, 16, 4, vl.BF16, P, P, None) == 1
    assert f(P, None, 1e-6, P, 8, 16, 4, vl.BF16, P, P, None) == 1
    assert f(P, P, 1e-6, P, 8, 16, 4, 7, P, P, None) == 3
    assert f(P, P, 1e-6, P, 8, 16, 3, vl.BF16, P, P, None) == 2
    assert f(P, P, -1.0, P, 8, 16, 4, vl.BF16, P, P, None) == 2
    assert f(P, P + 2, 1e-6, P, 8, 16, 4, vl.BF16, P, P, None) == 4
    assert f(P + 1, P, 1e-6, P, 8, 16, 4, vl.BF16, P, P, None) == 4


def test_adamw_step_factor_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    a = raw.velora_adamw_step_factor
    ok = (1e-3, 0.9, 0.999, 1e-8, 0.01, 1, 1.0, None)
    assert a(None, P, 32, 16, 4, P, vl.F32, P, P, *ok) == 1
    assert a(P, P, 32, 16, 4, P, vl.F32, None, P, *ok) == 1
    assert a(P, P, 32, 16, 4, P, 5, P, P, *ok) == 3
    assert a(P, P, 32, 16, 3, P, vl.F32, P, P, *ok) == 2                           # M does not divide D
    assert a(P, P, 32, 16, 4, P, vl.F32, P, P, 1e-3, 0.9, 0.999, 1e-8, 0.01, 0, 1.0, None) == 2   # step < 1
    assert a(P, P, 32, 16, 4, P, vl.F32, P, P, 1e-3, 1.0, 0.999, 1e-8, 0.01, 1, 1.0, None) == 2   # beta1 = 1
    assert a(P, P, 32, 16, 4, P, vl.F32, P, P, 1e-3, 0.9, -0.1, 1e-8, 0.01, 1, 1.0, None) == 2    # beta2 < 0
    assert a(P, P, 32, 16, 4, P, vl.F32, P, P, 1e-3, 0.9, 0.999, -1.0, 0.01, 1, 1.0, None) == 2   # eps < 0
    assert a(P, P, 32, 16, 4, P, vl.F32, P, P, float("nan"), 0.9, 0.999, 1e-8, 0.01, 1, 1.0, None) == 2
    assert a(P, P, 32, 16, 4, P + 2, vl.F32, P, P, *ok) == 4
    assert a(P, P, 32, 16, 4, P + 1, vl.BF16, P, P, *ok) == 4
    assert a(P, P, 32, 16, 4, P, vl.F32, P + 2, P, *ok) == 4


def test_update_v_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    need = vl.velora_workspace_bytes(vl.OP_INIT_V, 64, 16, 0, 4, vl.F32)
    u = raw.velora_update_v
    assert u(None, 64, 16, 4, vl.F32, None, 0.5, P, P, need, None) == 1
    assert u(P, 64, 16, 4, vl.F32, None, 0.5, None, P, need, None) == 1
    assert u(P, 64, 16, 4, vl.F32, None, 1.5, P, P, need, None) == 2      # beta outside [0, 1]
    assert u(P, 64, 16, 4, vl.F32, None, -0.1, P, P, need, None) == 2
    assert u(P, 64, 16, 3, vl.F32, None, 0.5, P, P, need, None) == 2
    assert u(P, 64, 16, 4, vl.F32, P + 2, 0.5, P, P, need, None) == 4
    assert u(P, 64, 16, 4, vl.F32, None, 0.5, P, P, need - 1, None) == 5
    c = raw.velora_compress_update
    assert c(P, None, 64, 16, 4, vl.F32, P, None, 0.5, P, P, need, None) == 1
    assert c(P, P, 64, 16, 4, vl.F32, P, None, 0.5, None, P, need, None) == 1
    assert c(P, P, 64, 16, 4, 2, P, None, 0.5, P, P, need, None) == 3
    assert c(P, P, 64, 16, 4, vl.F32, P, None, 0.5, P, None, need, None) == 5


def test_weight_grad_static_argument_errors(vl):
    # the same host-side checks as velora_weight_grad, and a plan that needs more than the static array is
    # refused before any device call (so this runs without a GPU)
    from paper_2405_17991_amd.binding import raw
    w = raw.velora_weight_grad_static
    N, O, D, M = 64, 32, 16, 4
    ok = (P, P, P, N, O, D, M, vl.BF16, P, vl.F32, 0, None)

    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return w(*a)

    assert call(a0=None) == 1 and call(a1=None) == 1 and call(a2=None) == 1 and call(a8=None) == 1
    assert call(a7=5) == 3 and call(a9=5) == 3
    assert call(a3=0) == 2 and call(a4=0) == 2 and call(a6=3) == 2
    assert call(a0=P + 1) == 4 and call(a8=P + 2) == 4
    # 2^20 output features x 1024 groups: 4 GiB of partial sums per token range
    big = vl.velora_workspace_bytes(vl.OP_WEIGHT_GRAD, 1024, 1024 * 8, 1 << 20, 1024, vl.BF16)
    assert big > vl.STATIC_SCRATCH_BYTES
    assert w(P, P, P, 1024, 1 << 20, 1024 * 8, 1024, vl.BF16, P, vl.F32, 0, None) == 5


def test_bandwidth_probe_argument_errors(vl):
    from paper_2405_17991_amd.binding import raw
    b = raw.velora_bandwidth_probe
    assert b(3, P, P, 1024, P, None) == 2 and b(-1, P, P, 1024, P, None) == 2
    assert b(0, P, None, 0, P, None) == 2 and b(0, P, None, 1000, P, None) == 2      # bytes: positive multiple of 16
    assert b(0, None, None, 1024, P, None) == 1 and b(0, P, None, 1024, None, None) == 1
    assert b(1, None, None, 1024, None, None) == 1 and b(2, P, None, 1024, None, None) == 1
    assert b(2, None, P, 1024, None, None) == 1
    assert b(0, P + 8, None, 1024, P, None) == 4 and b(1, None, P + 4, 1024, None, None) == 4
    assert b(0, P, None, 1024, P + 2, None) == 4


def test_workspace_query(vl):
    q = vl.velora_workspace_bytes
    assert q(vl.OP_COMPRESS, 128, 64, 0, 4, vl.BF16) == 0
    assert q(vl.OP_RECONSTRUCT, 128, 64, 0, 4, vl.BF16) == 0
    assert q(vl.OP_WEIGHT_GRAD, 128, 64, 0, 4, vl.BF16) == 0      # O missing
    assert q(vl.OP_WEIGHT_GRAD, 128, 64, 32, 5, vl.BF16) == 0     # M does not divide D
    a = q(vl.OP_WEIGHT_GRAD, 16384, 4096, 4096, 16, vl.BF16)
    assert a > 0 and a % 4 == 0
    # partial-sum traffic stays a small fraction of what the kernels must move anyway
    assert 2 * a <= 0.25 * (16384 * 4096 * 2 + 4096 * 4096 * 4)


def test_no_fallback_when_library_missing(vl, monkeypatch):
    from paper_2405_17991_amd import binding
    monkeypatch.setattr(binding, "_LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(ImportError):
        binding._load()
