"""ctypes face of the CPU oracle (oracle/gsgd_oracle.c) on numpy arrays.

Test infrastructure: imported only by tests/, the smoke check and the
benchmark's cpu_baseline leg.  It imports nothing from the GPU package.

All arrays are C-contiguous float32 of shape (k, ld) (replica rows) or (n,)
(shared vectors); a routine works on the first n columns of each row, which
stand for global columns col0 .. col0+n-1 of the full problem.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None

STREAM_GRAD, STREAM_INIT, STREAM_XSTAR, STREAM_H, STREAM_X0, STREAM_PERM = range(6)
NOISE_GAUSSIAN, NOISE_UNIFORM = 0, 1

_f32p = C.POINTER(C.c_float)
_i32p = C.POINTER(C.c_int32)
_i64p = C.POINTER(C.c_int64)
_u32p = C.POINTER(C.c_uint32)
_f64p = C.POINTER(C.c_double)


def lib():
    global _lib
    if _lib is None:
        # GSGD_ORACLE_LIB points the tests at another build of the same source (the sanitizer build)
        path = os.environ.get("GSGD_ORACLE_LIB") or (_build.LIB if os.path.exists(_build.LIB) else _build.build())
        L = C.CDLL(path)
        L.oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_u01.argtypes = [C.c_uint32]
        L.oracle_u01.restype = C.c_float
        L.oracle_noise4.argtypes = [_u32p, C.c_int, _f32p]
        L.oracle_noise4.restype = None
        L.oracle_fill.argtypes = [_f32p, C.c_int64, C.c_int64, C.c_uint64, C.c_int]
        L.oracle_fill.restype = C.c_int
        L.oracle_init_replicas.argtypes = [_f32p, _f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64,
                                           C.c_int64, C.c_uint64, C.c_int]
        L.oracle_init_replicas.restype = C.c_int
        L.oracle_gen_grad.argtypes = [_f32p, _f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, C.c_int64,
                                      C.c_float, C.c_uint64, C.c_uint32, C.c_int]
        L.oracle_gen_grad.restype = None
        L.oracle_expand_lr.argtypes = [C.c_float, C.c_int32, _i64p, _f32p, C.c_int64, C.c_int64, _f32p]
        L.oracle_expand_lr.restype = C.c_int
        L.oracle_step_gossip.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                         C.c_float, C.c_float, _i32p]
        L.oracle_step_gossip.restype = C.c_int
        L.oracle_step_allreduce.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p, C.c_float]
        L.oracle_step_allreduce.restype = C.c_int
        L.oracle_step_easgd.argtypes = [_f32p, _f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                        C.c_float, C.c_float]
        L.oracle_step_easgd.restype = C.c_int
        L.oracle_step_gossip_ext.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                             C.c_float, C.c_float, C.c_int, C.c_float, _i32p, C.c_int]
        L.oracle_step_gossip_ext.restype = C.c_int
        L.oracle_step_allreduce_ext.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                                C.c_float, C.c_float, C.c_int]
        L.oracle_step_allreduce_ext.restype = C.c_int
        L.oracle_step_easgd_ext.argtypes = [_f32p, _f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                            C.c_float, C.c_float, C.c_int, C.c_float]
        L.oracle_step_easgd_ext.restype = C.c_int
        L.oracle_make_targets.argtypes = [C.c_uint64, C.c_uint32, C.c_int32, C.c_int, _i32p]
        L.oracle_make_targets.restype = C.c_int
        L.oracle_step_gossip_push.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                              C.c_float, C.c_float, C.c_int, _i32p]
        L.oracle_step_gossip_push.restype = C.c_int
        L.oracle_async_tick.argtypes = [_f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                        C.c_float, C.c_float, C.c_int, C.c_float, C.c_int32, C.c_int32]
        L.oracle_async_tick.restype = C.c_int
        L.oracle_easgd_tick.argtypes = [_f32p, _f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f32p,
                                        C.c_float, C.c_float, C.c_int, C.c_float, C.c_int32]
        L.oracle_easgd_tick.restype = C.c_int
        L.oracle_gen_grad_row.argtypes = [_f32p, _f32p, _f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, C.c_int64,
                                          C.c_float, C.c_uint64, C.c_uint32, C.c_int]
        L.oracle_gen_grad_row.restype = None
        L.oracle_make_tick.argtypes = [C.c_uint64, C.c_uint32, C.c_int32, _i32p, _i32p]
        L.oracle_make_tick.restype = C.c_int
        L.oracle_make_perm.argtypes = [C.c_uint64, C.c_uint32, C.c_int32, _i32p]
        L.oracle_make_perm.restype = C.c_int
        L.oracle_stats.argtypes = [_f32p, _f32p, C.c_int32, C.c_int64, C.c_int64, _f64p]
        L.oracle_stats.restype = None
        L.oracle_set_num_threads.argtypes = [C.c_int]
        L.oracle_set_num_threads.restype = None
        L.oracle_num_threads.argtypes = []
        L.oracle_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _f32(a):
    assert isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags.c_contiguous, "need C-contiguous float32"
    return a.ctypes.data_as(_f32p)


def _rows(a):
    assert a.ndim == 2
    return a.shape[0], a.shape[1]


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(w) & 0xFFFFFFFF for w in ctr])
    k = (C.c_uint32 * 2)(*[int(w) & 0xFFFFFFFF for w in key])
    out = (C.c_uint32 * 4)()
    lib().oracle_philox4x32_10(c, k, out)
    return tuple(int(w) for w in out)


def u01(r):
    return np.float32(lib().oracle_u01(int(r) & 0xFFFFFFFF))


def noise4(words, kind):
    r = (C.c_uint32 * 4)(*[int(w) & 0xFFFFFFFF for w in words])
    out = np.zeros(4, np.float32)
    lib().oracle_noise4(r, int(kind), _f32(out))
    return out


def fill(n, seed, which, col0=0):
    dst = np.empty(int(n), np.float32)
    rc = lib().oracle_fill(_f32(dst), int(col0), int(n), int(seed), int(which))
    if rc:
        raise ValueError("oracle_fill: bad stream id")
    return dst


def init_replicas(x, v, center, x0, seed, mode, n=None, col0=0):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    rc = lib().oracle_init_replicas(_f32(x), _f32(v), _f32(center) if center is not None else None,
                                    _f32(x0) if x0 is not None else None, k, int(col0), n, ld, int(seed), int(mode))
    if rc:
        raise ValueError("oracle_init_replicas: bad arguments")


def gen_grad(x, h, xstar, g, sigma, seed, step, noise_kind=NOISE_GAUSSIAN, n=None, col0=0):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    assert g.shape == x.shape and h.shape[0] >= n and xstar.shape[0] >= n
    lib().oracle_gen_grad(_f32(x), _f32(h), _f32(xstar), _f32(g), k, int(col0), n, ld,
                          float(sigma), int(seed), int(step), int(noise_kind))


def expand_lr(lr, n, seg_offsets=None, seg_lr_scale=None, col0=0):
    out = np.empty(int(n), np.float32)
    if seg_offsets is None:
        rc = lib().oracle_expand_lr(float(lr), 0, None, None, int(col0), int(n), _f32(out))
    else:
        off = np.ascontiguousarray(seg_offsets, dtype=np.int64)
        sc = np.ascontiguousarray(seg_lr_scale, dtype=np.float32)
        assert off.shape[0] == sc.shape[0] + 1
        rc = lib().oracle_expand_lr(float(lr), sc.shape[0], off.ctypes.data_as(_i64p), _f32(sc),
                                    int(col0), int(n), _f32(out))
    if rc:
        raise ValueError("oracle_expand_lr: a column lies in no segment")
    return out


def _lr_col(lr, n):
    if isinstance(lr, np.ndarray):
        assert lr.dtype == np.float32 and lr.shape[0] >= n
        return lr
    return np.full(n, np.float32(lr), np.float32)


def step_gossip(x, v, g, lr, mu, beta, peer, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    p = np.ascontiguousarray(peer, dtype=np.int32)
    assert p.shape[0] == k
    rc = lib().oracle_step_gossip(_f32(x), _f32(v), _f32(g), k, n, ld, _f32(lrc), float(mu), float(beta),
                                  p.ctypes.data_as(_i32p))
    if rc:
        raise ValueError("oracle_step_gossip failed (%d)" % rc)


def step_allreduce(x, v, g, lr, mu, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    rc = lib().oracle_step_allreduce(_f32(x), _f32(v), _f32(g), k, n, ld, _f32(lrc), float(mu))
    if rc:
        raise ValueError("oracle_step_allreduce failed (%d)" % rc)


def step_easgd(x, v, g, center, lr, mu, alpha_e, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    rc = lib().oracle_step_easgd(_f32(x), _f32(v), _f32(g), _f32(center), k, n, ld, _f32(lrc),
                                 float(mu), float(alpha_e))
    if rc:
        raise ValueError("oracle_step_easgd failed (%d)" % rc)


def step_gossip_ext(x, v, g, lr, mu, beta, peer, wd=0.0, nesterov=False, stale=False, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    p = np.ascontiguousarray(peer, dtype=np.int32)
    assert p.shape[0] == k
    rc = lib().oracle_step_gossip_ext(_f32(x), _f32(v), _f32(g), k, n, ld, _f32(lrc), float(mu), float(wd),
                                      int(bool(nesterov)), float(beta), p.ctypes.data_as(_i32p), int(bool(stale)))
    if rc:
        raise ValueError("oracle_step_gossip_ext failed (%d)" % rc)


def step_allreduce_ext(x, v, g, lr, mu, wd=0.0, nesterov=False, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    rc = lib().oracle_step_allreduce_ext(_f32(x), _f32(v), _f32(g), k, n, ld, _f32(lrc), float(mu), float(wd),
                                         int(bool(nesterov)))
    if rc:
        raise ValueError("oracle_step_allreduce_ext failed (%d)" % rc)


def step_easgd_ext(x, v, g, center, lr, mu, alpha_e, wd=0.0, nesterov=False, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    rc = lib().oracle_step_easgd_ext(_f32(x), _f32(v), _f32(g), _f32(center), k, n, ld, _f32(lrc), float(mu),
                                     float(wd), int(bool(nesterov)), float(alpha_e))
    if rc:
        raise ValueError("oracle_step_easgd_ext failed (%d)" % rc)


def step_gossip_push(x, v, g, lr, mu, target, wd=0.0, nesterov=False, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    t = np.ascontiguousarray(target, dtype=np.int32)
    assert t.shape[0] == k
    rc = lib().oracle_step_gossip_push(_f32(x), _f32(v), _f32(g), k, n, ld, _f32(lrc), float(mu), float(wd),
                                       int(bool(nesterov)), t.ctypes.data_as(_i32p))
    if rc:
        raise ValueError("oracle_step_gossip_push failed (%d)" % rc)


def async_tick(x, v, g_row, lr, mu, beta, i, j, wd=0.0, nesterov=False, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    assert g_row.shape[0] >= n
    rc = lib().oracle_async_tick(_f32(x), _f32(v), _f32(g_row), k, n, ld, _f32(lrc), float(mu), float(wd),
                                 int(bool(nesterov)), float(beta), int(i), int(j))
    if rc:
        raise ValueError("oracle_async_tick: node index out of range")


def easgd_tick(x, v, g_row, center, lr, mu, alpha_e, i, wd=0.0, nesterov=False, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    lrc = _lr_col(lr, n)
    assert g_row.shape[0] >= n and center.shape[0] >= n
    rc = lib().oracle_easgd_tick(_f32(x), _f32(v), _f32(g_row), _f32(center), k, n, ld, _f32(lrc), float(mu),
                                 float(wd), int(bool(nesterov)), float(alpha_e), int(i))
    if rc:
        raise ValueError("oracle_easgd_tick: node index out of range")


def gen_grad_row(x, h, xstar, g_row, i, sigma, seed, tick, noise_kind=NOISE_GAUSSIAN, n=None, col0=0):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    assert 0 <= i < k and g_row.shape[0] >= n and h.shape[0] >= n and xstar.shape[0] >= n
    lib().oracle_gen_grad_row(_f32(x), _f32(h), _f32(xstar), _f32(g_row), int(i), int(col0), n, ld,
                              float(sigma), int(seed), int(tick), int(noise_kind))


def make_tick(seed, tick, k):
    i, j = C.c_int32(0), C.c_int32(0)
    rc = lib().oracle_make_tick(int(seed), int(tick), int(k), C.byref(i), C.byref(j))
    if rc:
        raise ValueError("oracle_make_tick: k < 1")
    return int(i.value), int(j.value)


def make_targets(seed, step, k, exclude_self=False):
    out = np.empty(int(k), np.int32)
    rc = lib().oracle_make_targets(int(seed), int(step), int(k), int(bool(exclude_self)), out.ctypes.data_as(_i32p))
    if rc:
        raise ValueError("oracle_make_targets: k too small")
    return out


def make_perm(seed, step, k):
    out = np.empty(int(k), np.int32)
    rc = lib().oracle_make_perm(int(seed), int(step), int(k), out.ctypes.data_as(_i32p))
    if rc:
        raise ValueError("oracle_make_perm: k < 1")
    return out


def stats(x, xstar, n=None):
    k, ld = _rows(x)
    n = ld if n is None else int(n)
    out = np.zeros(4, np.float64)
    lib().oracle_stats(_f32(x), _f32(xstar), k, n, ld, out.ctypes.data_as(_f64p))
    return out


def num_threads():
    return int(lib().oracle_num_threads())


def set_num_threads(n):
    lib().oracle_set_num_threads(int(n))


# ----------------------------------------------------------------------------
# Diffusion potential (Section 3.1), written out from its definition in fp64.
# Under gossip rounds alone, theta_i(r) = sum_j v_ij theta_j(0) with V = M_r ... M_1.

def mixing_matrix_pull(peer, beta):
    """M with theta' = M theta for one pull round: row i is (1 - beta) e_i + beta e_peer[i]."""
    k = len(peer)
    M = np.zeros((k, k), np.float64)
    for i in range(k):
        M[i, i] += 1.0 - float(beta)
        M[i, int(peer[i])] += float(beta)
    return M


def mixing_matrix_push(target):
    """M for one push round: row r averages r itself and every i != r with target[i] == r."""
    k = len(target)
    M = np.zeros((k, k), np.float64)
    for r in range(k):
        got = [r] + [i for i in range(k) if i != r and int(target[i]) == r]
        for i in got:
            M[r, i] = 1.0 / len(got)
    return M


def diffusion_potential(theta0, V):
    """sum_i sum_j || v_ij theta_j(0) - (1/p) sum_j' v_ij' theta_j'(0) ||^2, term by term."""
    theta0 = np.asarray(theta0, np.float64)
    V = np.asarray(V, np.float64)
    p = theta0.shape[0]
    total = 0.0
    for i in range(p):
        contrib = [V[i, j] * theta0[j] for j in range(p)]
        centre = sum(contrib) / p
        for j in range(p):
            diff = contrib[j] - centre
            total += float(diff @ diff)
    return total
