"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything touches a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cdq.h")


@pytest.fixture(scope="module")
def L():
    from paper_2406_17542_amd import cdq
    return cdq.lib()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cdq_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported(L):
    names = _declared()
    assert {"cdq_hessian", "cdq_init_rtn", "cdq_greedy_cd", "cdq_loss", "cdq_workspace_bytes", "cdq_strerror"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/cdq.h but not exported by libcdq.so"


def test_strerror(L):
    assert L.cdq_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(L.cdq_strerror(code)) > 3


def test_workspace_query(L):
    from paper_2406_17542_amd import cdq
    # greedy CD: room for G0 [d_out][d_in] fp32 and the Hessian diagonal
    assert cdq.workspace_bytes(cdq.OP_GREEDY_CD, 0, 64, 128) >= 64 * 128 * 4 + 128 * 4
    assert cdq.workspace_bytes(cdq.OP_LOSS, 0, 2048, 2048) >= 2048 * 16 * 8
    assert cdq.workspace_bytes(cdq.OP_HESSIAN, 16384, 0, 2048) >= 2048 * 2048 * 4
    assert cdq.workspace_bytes(cdq.OP_HESSIAN, 16384, 0, 0) == 0


def test_argument_checks_need_no_gpu(L):
    """Every rejection below happens on the host before any HIP call."""
    p = ctypes.c_void_p(0x1000)      # never dereferenced: the checks fail first
    n = ctypes.c_void_p(0)
    EINVAL, EWS, EUNSUP = -1, -2, -4
    assert L.cdq_init_rtn(n, 4, 8, 3, 8, p, p, p, n) == EINVAL                      # null Wt
    assert L.cdq_init_rtn(p, 4, 8, 5, 8, p, p, p, n) == EINVAL                      # bits
    assert L.cdq_init_rtn(p, 4, 8, 1, 8, p, p, p, n) == EINVAL
    assert L.cdq_init_rtn(p, 4, 8, 3, 3, p, p, p, n) == EINVAL                      # d_in % group
    assert L.cdq_init_rtn(p, 4, 8, 3, 16, p, p, p, n) == EINVAL                     # group > d_in
    assert L.cdq_init_rtn(p, -1, 8, 3, 8, p, p, p, n) == EINVAL
    assert L.cdq_hessian(p, 7, 16, 8, p, 0, 0.0, n, 0, n) == EINVAL                 # dtype
    assert L.cdq_hessian(p, 1, 16, 12, p, 0, 0.0, n, 0, n) == EINVAL                # bf16 needs d_in % 8 == 0
    assert L.cdq_hessian(p, 0, 16, 8, p, 0, -1.0, n, 0, n) == EINVAL                # negative damping
    assert L.cdq_hessian(p, 0, 16, 8, p, 1, 0.0, n, 0, n) == EWS                    # accumulate needs workspace
    assert L.cdq_greedy_cd(p, p, p, p, p, 4, 8, 3, 8, -1, n, p, 1 << 20, n) == EINVAL    # T < 0
    assert L.cdq_greedy_cd(p, p, p, p, p, 4, 8, 3, 8, 4, n, n, 0, n) == EWS             # no workspace
    assert L.cdq_greedy_cd(p, p, p, p, p, 4, 8, 3, 8, 4, n, ctypes.c_void_p(0x1010), 1 << 20, n) == EWS   # misaligned
    assert L.cdq_greedy_cd(p, p, p, p, p, 4, 8, 3, 8, 4, n, ctypes.c_void_p(0x1000), 16, n) == EWS        # too small
    assert L.cdq_greedy_cd(p, p, p, p, p, 4, 65536, 3, 65536, 4, n, p, 1 << 40, n) == EUNSUP              # d_in too large
    assert L.cdq_loss(p, p, p, p, p, 4, 8, 8, n, n, p, 1 << 20, n) == EINVAL             # no output requested
    assert L.cdq_loss(p, p, p, p, p, 4, 8, 8, p, n, n, 0, n) == EWS
    assert L.cdq_gradient(p, p, p, p, p, 4, 8, 8, n, n) == EINVAL
