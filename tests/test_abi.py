"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything touches a GPU."""
import ctypes
import glob
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))


@pytest.fixture(scope="module")
def L():
    from paper_2406_17542_amd import cdq
    return cdq.lib()


def _declared():
    names = set()
    for h in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(cdq_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_exported(L):
    names = _declared()
    assert {"cdq_hessian", "cdq_init_rtn", "cdq_greedy_cd", "cdq_loss", "cdq_workspace_bytes", "cdq_strerror",
            "cdq_probe_copy", "cdq_greedy_cd_shape"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/*.h but not exported by libcdq.so"


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


def test_argument_checks_of_the_wider_entry_points(L):
    """OWC-CD, BCD and cyclic CD reject bad arguments on the host as well."""
    from paper_2406_17542_amd import cdq
    p = ctypes.c_void_p(0x1000)
    n = ctypes.c_void_p(0)
    EINVAL, EWS, EUNSUP = -1, -2, -4
    i64 = ctypes.c_int64
    # cdq_init_owc_cd(H, Wt, d_out, d_in, bits, group, n_gamma, T, scale, zero, Q, gamma_idx, moves, trace, trace_cap, variant, ws, ws_bytes, stream)
    assert L.cdq_init_owc_cd(p, p, 4, 256, 3, 64, 0, 4, p, p, p, n, n, n, 0, 0, n, 0, n) == EINVAL       # empty grid
    assert L.cdq_init_owc_cd(p, p, 4, 256, 3, 64, 50, -1, p, p, p, n, n, n, 0, 0, n, 0, n) == EINVAL     # T < 0
    assert L.cdq_init_owc_cd(p, p, 4, 256, 3, 64, 50, 4, p, p, p, n, n, n, 0, 2, n, 0, n) == EINVAL      # unknown variant
    assert L.cdq_init_owc_cd(p, p, 4, 256, 3, 64, 50, 4, p, p, p, n, n, p, 0, 0, n, 0, n) == EINVAL      # trace without capacity
    assert L.cdq_init_owc_cd(p, p, 4, 256, 3, 64, 50, 4, n, p, p, n, n, n, 0, 0, n, 0, n) == EINVAL      # null scale
    assert L.cdq_init_owc_cd(p, p, 4, 256, 3, 64, 50, 4, p, p, p, n, n, n, 0, 0, n, 0, n) == EWS         # tiled kernel needs G64
    assert L.cdq_init_owc_cd(p, p, 4, 65536, 3, 128, 50, 4, p, p, p, n, n, n, 0, 1, n, 0, n) == EUNSUP   # state does not fit LDS
    assert cdq.workspace_bytes(cdq.OP_INIT_OWC_CD, 0, 16, 256) >= 16 * 256 * 8
    # cdq_bcd(H, Wt, scale, zero, Q, d_out, d_in, bits, group, k, parts, T, moves, G_out, trace, trace_cap, flags, ws, ws_bytes, stream)
    assert L.cdq_bcd(p, p, p, p, p, 4, 256, 3, 256, 0, p, 8, n, n, n, 0, 0, p, 1 << 30, n) == EINVAL     # k < 1
    assert L.cdq_bcd(p, p, p, p, p, 4, 256, 3, 256, 3, p, 8, n, n, n, 0, 0, p, 1 << 30, n) == EUNSUP     # only pairs are built
    assert L.cdq_bcd(p, p, p, p, p, 4, 255, 3, 255, 2, p, 8, n, n, n, 0, 0, p, 1 << 30, n) == EINVAL     # odd d_in
    assert L.cdq_bcd(p, p, p, p, p, 4, 256, 3, 256, 2, n, 8, n, n, n, 0, 0, p, 1 << 30, n) == EINVAL     # no partitions
    assert L.cdq_bcd(p, p, p, p, p, 4, 256, 3, 256, 2, p, 8, n, n, n, 0, 8, p, 1 << 30, n) == EINVAL     # unknown flag bit
    assert L.cdq_bcd(p, p, p, p, p, 4, 256, 3, 256, 2, p, 8, n, n, n, 0, 0, n, 0, n) == EWS
    assert L.cdq_bcd(p, p, p, p, p, 4, 65536, 3, 65536, 2, p, 8, n, n, n, 0, 0, p, 1 << 40, n) == EUNSUP # wider than the wide-layer kernel holds
    assert cdq.workspace_bytes(cdq.OP_BCD, 8, 4, 256) >= 4 * 256 * 4 + 8 * 128 * 12
    # cdq_cyclic_cd(H, Wt, scale, zero, Q, d_out, d_in, bits, group, T, stats, G_out, trace, trace_cap, ws, ws_bytes, stream)
    assert L.cdq_cyclic_cd(p, p, p, p, p, 4, 256, 3, 256, i64(-1), n, n, n, 0, p, 1 << 30, n) == EINVAL
    assert L.cdq_cyclic_cd(p, p, p, p, p, 4, 256, 7, 256, i64(8), n, n, n, 0, p, 1 << 30, n) == EINVAL   # bits
    assert L.cdq_cyclic_cd(p, p, p, p, p, 4, 256, 3, 256, i64(8), n, n, n, 0, n, 0, n) == EWS
    assert L.cdq_cyclic_cd(p, p, p, p, p, 4, 254, 3, 254, i64(8), n, n, n, 0, p, 1 << 30, n) == EUNSUP   # d_in % 4
    assert L.cdq_cyclic_cd(p, p, p, p, p, 0, 256, 3, 256, i64(8), n, n, n, 0, n, 0, n) == 0             # empty layer


def test_argument_checks_of_the_new_options(L):
    """Start gradient handed over, columns per compute unit, the grid search's margin: rejected on the host where wrong."""
    from paper_2406_17542_amd import cdq
    p = ctypes.c_void_p(0x1000)
    n = ctypes.c_void_p(0)
    EINVAL, EWS, EUNSUP = -1, -2, -4
    def opts(**kw):
        o = cdq.CdOptions()
        for k, v in kw.items():
            setattr(o, k, v)
        return ctypes.byref(o)
    # cdq_greedy_cd_ex(H, Wt, scale, zero, Q, d_out, d_in, bits, group, T, stats, opts, ws, ws_bytes, stream)
    assert L.cdq_greedy_cd_ex(p, p, p, p, p, 4, 8, 3, 8, 4, n, opts(G0=0x1004), p, 1 << 20, n) == EINVAL        # start gradient not 16-byte aligned
    assert L.cdq_greedy_cd_ex(p, p, p, p, p, 4, 8, 3, 8, 4, n, opts(G0=0x2000), n, 0, n) == EWS                 # the diagonal still needs room
    assert L.cdq_greedy_cd_ex(p, p, p, p, p, 4, 8, 3, 8, 4, n, opts(G0=0x2000), p, 16, n) == EWS
    assert L.cdq_greedy_cd_ex(p, p, p, p, p, 4, 8, 3, 8, 4, n, opts(waves_per_column=3, elems_per_lane=16), p, 1 << 20, n) == EINVAL
    # cdq_init_owc(H, Wt, d_out, d_in, bits, group, n_gamma, margin, scale, zero, Q, gamma, loss, researched, G_out, ws, ws_bytes, stream)
    f = ctypes.c_float
    assert L.cdq_init_owc(p, p, 4, 256, 3, 256, 50, f(-1.0), p, p, p, n, n, n, n, p, 1 << 30, n) == EINVAL      # negative margin
    assert L.cdq_init_owc(p, p, 4, 256, 3, 256, 50, f(2.0), p, p, p, n, n, n, n, p, 1 << 30, n) == EINVAL
    assert L.cdq_init_owc(p, p, 4, 256, 3, 128, 50, f(0.0), p, p, p, n, n, n, n, p, 1 << 30, n) == EUNSUP       # one strength per column only
    assert L.cdq_init_owc(p, p, 4, 256, 3, 256, 0, f(0.0), p, p, p, n, n, n, n, p, 1 << 30, n) == EINVAL        # empty grid
    assert L.cdq_init_owc(p, p, 4, 256, 3, 256, 50, f(0.0), p, p, p, n, n, n, p, n, 0, n) == EWS                # no workspace
    assert L.cdq_init_owc(p, p, 0, 256, 3, 256, 50, f(0.0), p, p, p, n, n, n, p, n, 0, n) == 0                  # empty layer
    # more start-grid workspace than before for the same shape is not required when no gradient is asked for
    assert cdq.workspace_bytes(cdq.OP_INIT_OWC, 0, 64, 256) >= 64 * 256 * 4


def test_launch_shape_query(L):
    """The default launch shape is a host-side rule: 16 coordinates per lane up to d_in = 16384, the kernels with the
    Hessian diagonal in LDS above, and a scalar-load shape when the rows are not 16-byte aligned."""
    from paper_2406_17542_amd import cdq
    assert cdq.greedy_cd_shape(2048, 2048, 2048) == (2, 16)
    assert cdq.greedy_cd_shape(32768, 8192, 8192) == (8, 16)
    assert cdq.greedy_cd_shape(2048, 16384, 16384) == (16, 16)
    assert cdq.greedy_cd_launch(2048, 16384, 16384) == (16, 16, 2)      # more columns than compute units: two resident per unit
    assert cdq.greedy_cd_launch(256, 16384, 16384) == (16, 16, 1)
    assert cdq.greedy_cd_launch(32768, 8192, 8192) == (8, 16, 1)
    assert cdq.greedy_cd_shape(3072, 24576, 24576) == (16, 24)
    assert cdq.greedy_cd_shape(3072, 24576, 24576, aligned16=False) == (16, 32)      # 24 per lane needs 16-byte chunks
    assert cdq.greedy_cd_shape(4608, 36864, 36864) == (16, 36)
    w, e = cdq.greedy_cd_shape(6, 2048, 2048)                                         # few columns: the chain is split further
    assert 64 * w * e >= 2048 and e < 16
    with pytest.raises(cdq.CdqError) as err:
        cdq.greedy_cd_shape(4608, 36864, 36864, aligned16=False)
    assert err.value.code == -4
    with pytest.raises(cdq.CdqError):
        cdq.greedy_cd_shape(16, 65536, 65536)
