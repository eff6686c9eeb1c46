"""Thin ctypes binding over libgsgd.so: argument marshalling only.

Every step of the method runs in the library's HIP kernels.  PyTorch is used
for device memory (tensors are passed as raw pointers) and for the current HIP
stream.  There is no CPU fallback: if the library is missing or a call fails,
an exception is raised.

Names mirror include/gsgd.h without the gsgd_ prefix.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgsgd.so")

MAX_K = 512
OK, ERR_INVALID_ARG, ERR_BAD_PERM, ERR_BAD_SEGMENTS, ERR_HIP, ERR_UNSUPPORTED, ERR_NO_MEMORY = 0, -1, -2, -3, -4, -5, -6
ERR_BAD_STATE, ERR_TOO_LARGE = -7, -8
STATS_STATIC_MAX_D = 1 << 26
NOISE_GAUSSIAN, NOISE_UNIFORM = 0, 1
INIT_BROADCAST, INIT_PER_REPLICA = 0, 1
FILL_XSTAR, FILL_H, FILL_X0 = 2, 3, 4
ROW_SPLIT_AUTO, ROW_SPLIT_OFF, ROW_SPLIT_ON = 0, 1, 2
GOSSIP_AUTO, GOSSIP_WALK, GOSSIP_SWEEP, GOSSIP_SWEEP_SPLIT = 0, 1, 2, 3

KERNEL_GOSSIP, KERNEL_ALLREDUCE, KERNEL_EASGD, KERNEL_GEN_GRAD, KERNEL_GOSSIP_FUSED, KERNEL_LOCAL = range(6)
KERNEL_COUNT = 6
WALK_ROW_MASK, WALK_FIRST, WALK_LAST = 0x0FFF, 0x4000, 0x8000
WALK_TREE, WALK_DESCEND, WALK_SAVE = 0x2000, 0x1000, 0x40000
WALK_RESTORE_SHIFT, WALK_SLOT_SHIFT, WALK_SLOTS = 16, 20, 8
PUSH_HAS_SENDERS, PUSH_MODE_SHIFT, PUSH_SAVE_AFTER, PUSH_SLOT_SHIFT, PUSH_COUNT_SHIFT = 0x1000, 16, 0x40000, 19, 22


class GsgdError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


class _Config(C.Structure):
    _fields_ = [("k", C.c_int32), ("d", C.c_int64), ("ld", C.c_int64),
                ("lr", C.c_float), ("momentum", C.c_float), ("sigma", C.c_float),
                ("seed", C.c_uint64), ("noise_kind", C.c_int32), ("n_seg", C.c_int32),
                ("seg_offsets", C.POINTER(C.c_int64)), ("seg_lr_scale", C.POINTER(C.c_float)),
                ("block_columns", C.c_int64)]


_lib = None
_vp = C.c_void_p

# name -> (restype, argtypes); also the list of symbols include/gsgd.h declares
SIGNATURES = {
    "gsgd_create": (C.c_int, [C.POINTER(_Config), C.POINTER(_vp)]),
    "gsgd_destroy": (C.c_int, [_vp]),
    "gsgd_set_lr": (C.c_int, [_vp, C.c_float]),
    "gsgd_set_launch_width": (C.c_int, [_vp, C.c_int, C.c_int]),
    "gsgd_set_local_step": (C.c_int, [_vp, C.c_float, C.c_int]),
    "gsgd_set_row_split": (C.c_int, [_vp, C.c_int]),
    "gsgd_set_gossip_form": (C.c_int, [_vp, C.c_int]),
    "gsgd_comm_due": (C.c_int, [C.c_uint64, C.c_uint32]),
    "gsgd_step_gossip_stale": (C.c_int, [_vp, _vp, _vp, _vp, C.POINTER(C.c_int32), C.c_float, _vp]),
    "gsgd_step_local": (C.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "gsgd_step_gossip_pull": (C.c_int, [_vp, _vp, _vp, _vp, C.POINTER(C.c_int32), C.c_float, C.c_int, _vp]),
    "gsgd_step_gossip_push": (C.c_int, [_vp, _vp, _vp, _vp, C.POINTER(C.c_int32), _vp]),
    "gsgd_push_walk": (C.c_int, [C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_uint32), C.POINTER(C.c_int32)]),
    "gsgd_step_async_tick": (C.c_int, [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_float, _vp]),
    "gsgd_step_easgd_tick": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.c_int32, C.c_float, _vp]),
    "gsgd_step_async_tick_fused": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_float, C.c_uint64,
                                             _vp]),
    "gsgd_run_async_ticks": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.c_float, C.c_uint64, C.c_uint64, _vp]),
    "gsgd_make_tick": (C.c_int, [C.c_uint64, C.c_uint64, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "gsgd_make_targets": (C.c_int, [C.c_uint64, C.c_uint64, C.c_int32, C.c_int, C.POINTER(C.c_int32)]),
    "gsgd_pull_walk": (C.c_int, [C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_uint32), C.POINTER(C.c_int32)]),
    "gsgd_init_replicas": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.c_int, _vp]),
    "gsgd_fill": (C.c_int, [_vp, _vp, C.c_int, _vp]),
    "gsgd_gen_grad": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.c_uint64, _vp]),
    "gsgd_step_allreduce": (C.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "gsgd_step_gossip": (C.c_int, [_vp, _vp, _vp, _vp, C.POINTER(C.c_int32), C.c_float, _vp]),
    "gsgd_step_easgd": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.c_float, _vp]),
    "gsgd_step_gossip_fused": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.POINTER(C.c_int32), C.c_float, C.c_uint64, _vp]),
    "gsgd_step_gossip_pull_fused": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.POINTER(C.c_int32), C.c_float, C.c_int,
                                              C.c_uint64, _vp]),
    "gsgd_step_gossip_push_fused": (C.c_int, [_vp, _vp, _vp, _vp, _vp, C.POINTER(C.c_int32), C.c_uint64, _vp]),
    "gsgd_philox_raw": (C.c_int, [_vp, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int64, _vp, _vp]),
    "gsgd_noise_alu_probe": (C.c_int, [_vp, C.c_int32, C.c_uint32, _vp, _vp]),
    "gsgd_make_perm": (C.c_int, [C.c_uint64, C.c_uint64, C.c_int32, C.POINTER(C.c_int32)]),
    "gsgd_perm_walk": (C.c_int, [C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_uint16)]),
    "gsgd_stats": (C.c_int, [_vp, _vp, _vp, C.POINTER(C.c_double), _vp]),
    "gsgd_relayout": (C.c_int, [C.c_int32, C.c_int64, C.c_int64, C.c_int64, _vp, C.c_int64, C.c_int64, _vp, _vp]),
    "gsgd_stats_static": (C.c_int, [C.c_int32, C.c_int64, C.c_int64, C.c_int64, _vp, _vp, _vp, _vp]),
    "gsgd_row_sqnorms": (C.c_int, [_vp, _vp, C.POINTER(C.c_double), _vp]),
    "gsgd_weights_pull": (C.c_int, [C.POINTER(C.c_double), C.c_int32, C.POINTER(C.c_int32), C.c_double]),
    "gsgd_weights_push": (C.c_int, [C.POINTER(C.c_double), C.c_int32, C.POINTER(C.c_int32)]),
    "gsgd_diffusion_potential": (C.c_int, [C.POINTER(C.c_double), C.c_int32, C.POINTER(C.c_double),
                                           C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "gsgd_poke_tickets": (C.c_int, [_vp, C.c_uint32, C.c_uint32, _vp]),
    "gsgd_strerror": (C.c_char_p, [C.c_int]),
    "gsgd_last_hip_error": (C.c_int, [_vp]),
}


def lib():
    """Load libgsgd.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libgsgd.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        import torch  # noqa: F401  -- loads the HIP runtime the library binds to
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def strerror(code):
    return lib().gsgd_strerror(int(code)).decode()


def _check(rc, where):
    if rc != OK:
        raise GsgdError(rc, where)


def _ptr(t, need=0, dtype=None):
    """Raw device pointer of a torch tensor (or None), after checking that it is
    what the library will take it for: a contiguous GPU tensor of `dtype`
    (fp32 unless given) holding at least `need` elements.  A wrong tensor would
    otherwise become an out-of-bounds device access."""
    if t is None:
        return None
    import torch
    want = torch.float32 if dtype is None else dtype
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError("expected a GPU tensor, got %r" % (type(t).__name__ if not isinstance(t, torch.Tensor)
                                                            else t.device,))
    if t.dtype != want:
        raise ValueError("expected dtype %s, got %s" % (want, t.dtype))
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    if t.numel() < need:
        raise ValueError("tensor holds %d elements, the call touches %d" % (t.numel(), need))
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return C.c_void_p(int(stream))
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _perm_arg(peer_perm, k=None):
    p = np.ascontiguousarray(peer_perm, dtype=np.int32)
    if p.ndim != 1 or (k is not None and p.shape[0] != k):
        raise ValueError("a peer / target map needs exactly k = %s entries, got shape %s" % (k, p.shape))
    return p, p.ctypes.data_as(C.POINTER(C.c_int32))


class Context:
    """Owns a gsgd_ctx.  Tensors passed to the methods must be fp32 CUDA
    tensors laid out as the header describes (k x ld rows, row-major or, with
    block_columns > 0, in blocks of that many columns; or d-vectors)."""

    def __init__(self, k, d, ld=None, lr=0.05, momentum=0.9, sigma=0.1, seed=0x161104581,
                 noise_kind=NOISE_GAUSSIAN, seg_offsets=None, seg_lr_scale=None, block_columns=0):
        ld = d if ld is None else ld
        cfg = _Config()
        cfg.k, cfg.d, cfg.ld = int(k), int(d), int(ld)
        cfg.block_columns = int(block_columns)
        cfg.lr, cfg.momentum, cfg.sigma = float(lr), float(momentum), float(sigma)
        cfg.seed, cfg.noise_kind = int(seed), int(noise_kind)
        self._keep = None
        if seg_offsets is not None:
            off = np.ascontiguousarray(seg_offsets, dtype=np.int64)
            sc = np.ascontiguousarray(seg_lr_scale, dtype=np.float32)
            if off.shape[0] != sc.shape[0] + 1:
                raise ValueError("seg_offsets must have one more entry than seg_lr_scale")
            cfg.n_seg = int(sc.shape[0])
            cfg.seg_offsets = off.ctypes.data_as(C.POINTER(C.c_int64))
            cfg.seg_lr_scale = sc.ctypes.data_as(C.POINTER(C.c_float))
            self._keep = (off, sc)
        else:
            cfg.n_seg = 0
        self.k, self.d, self.ld, self.block_columns = cfg.k, cfg.d, cfg.ld, cfg.block_columns
        self._h = _vp()
        _check(lib().gsgd_create(C.byref(cfg), C.byref(self._h)), "gsgd_create")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value and _lib is not None:
            _lib.gsgd_destroy(self._h)
            self._h = _vp()

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _m(self, t):
        """a k x ld matrix: the last row (row-major) or the last block's last piece (blocked) may be short of
        the padding"""
        if self.block_columns > 0:
            b, last = self.block_columns, (self.d - 1) // self.block_columns
            return _ptr(t, last * self.k * b + (self.k - 1) * b + (self.d - last * b))
        return _ptr(t, (self.k - 1) * self.ld + self.d)

    def _vec(self, t):
        """a shared d-vector"""
        return _ptr(t, self.d)

    def set_lr(self, lr):
        _check(lib().gsgd_set_lr(self._h, float(lr)), "gsgd_set_lr")

    def set_local_step(self, weight_decay=0.0, nesterov=False):
        _check(lib().gsgd_set_local_step(self._h, float(weight_decay), int(bool(nesterov))), "gsgd_set_local_step")

    def set_row_split(self, mode):
        _check(lib().gsgd_set_row_split(self._h, int(mode)), "gsgd_set_row_split")

    def set_gossip_form(self, form):
        _check(lib().gsgd_set_gossip_form(self._h, int(form)), "gsgd_set_gossip_form")

    def set_launch_width(self, kernel, workgroups):
        _check(lib().gsgd_set_launch_width(self._h, int(kernel), int(workgroups)), "gsgd_set_launch_width")

    def init_replicas(self, x, v, center, x0, mode=INIT_BROADCAST, stream=None):
        _check(lib().gsgd_init_replicas(self._h, self._m(x), self._m(v), self._vec(center), self._vec(x0), int(mode), _stream(stream)),
               "gsgd_init_replicas")

    def fill(self, dst, which, stream=None):
        _check(lib().gsgd_fill(self._h, self._vec(dst), int(which), _stream(stream)), "gsgd_fill")

    def gen_grad(self, x, h, xstar, g, step, stream=None):
        _check(lib().gsgd_gen_grad(self._h, self._m(x), self._vec(h), self._vec(xstar), self._m(g), int(step), _stream(stream)),
               "gsgd_gen_grad")

    def step_allreduce(self, x, v, g, stream=None):
        _check(lib().gsgd_step_allreduce(self._h, self._m(x), self._m(v), self._m(g), _stream(stream)), "gsgd_step_allreduce")

    def step_gossip(self, x, v, g, peer_perm, beta=0.5, stream=None):
        keep, p = _perm_arg(peer_perm, self.k)
        _check(lib().gsgd_step_gossip(self._h, self._m(x), self._m(v), self._m(g), p, float(beta), _stream(stream)),
               "gsgd_step_gossip")

    def step_gossip_stale(self, x, v, g, peer_perm, beta=0.5, stream=None):
        keep, p = _perm_arg(peer_perm, self.k)
        _check(lib().gsgd_step_gossip_stale(self._h, self._m(x), self._m(v), self._m(g), p, float(beta), _stream(stream)),
               "gsgd_step_gossip_stale")

    def step_gossip_pull(self, x, v, g, peer, beta=0.5, stale=False, stream=None):
        keep, p = _perm_arg(peer, self.k)
        _check(lib().gsgd_step_gossip_pull(self._h, self._m(x), self._m(v), self._m(g), p, float(beta), int(bool(stale)),
                                           _stream(stream)), "gsgd_step_gossip_pull")

    def step_gossip_push(self, x, v, g, target, stream=None):
        keep, p = _perm_arg(target, self.k)
        _check(lib().gsgd_step_gossip_push(self._h, self._m(x), self._m(v), self._m(g), p, _stream(stream)),
               "gsgd_step_gossip_push")

    def step_async_tick(self, x, v, g, i, j, beta=0.5, stream=None):
        _check(lib().gsgd_step_async_tick(self._h, self._m(x), self._m(v), self._m(g), int(i), int(j), float(beta),
                                          _stream(stream)), "gsgd_step_async_tick")

    def step_easgd_tick(self, x, v, g, center, i, alpha_e, stream=None):
        _check(lib().gsgd_step_easgd_tick(self._h, self._m(x), self._m(v), self._m(g), self._vec(center), int(i), float(alpha_e),
                                          _stream(stream)), "gsgd_step_easgd_tick")

    def step_async_tick_fused(self, x, v, h, xstar, i, j, tick, beta=0.5, stream=None):
        _check(lib().gsgd_step_async_tick_fused(self._h, self._m(x), self._m(v), self._vec(h), self._vec(xstar), int(i), int(j),
                                                float(beta), int(tick), _stream(stream)),
               "gsgd_step_async_tick_fused")

    def run_async_ticks(self, x, v, h, xstar, first_tick, n_ticks, beta=0.5, stream=None):
        _check(lib().gsgd_run_async_ticks(self._h, self._m(x), self._m(v), self._vec(h), self._vec(xstar), float(beta),
                                          int(first_tick), int(n_ticks), _stream(stream)), "gsgd_run_async_ticks")

    def step_local(self, x, v, g, stream=None):
        _check(lib().gsgd_step_local(self._h, self._m(x), self._m(v), self._m(g), _stream(stream)), "gsgd_step_local")

    def step_easgd(self, x, v, g, center, alpha_e, stream=None):
        _check(lib().gsgd_step_easgd(self._h, self._m(x), self._m(v), self._m(g), self._vec(center), float(alpha_e),
                                     _stream(stream)), "gsgd_step_easgd")

    def step_gossip_fused(self, x, v, h, xstar, peer_perm, step, beta=0.5, stream=None):
        keep, p = _perm_arg(peer_perm, self.k)
        _check(lib().gsgd_step_gossip_fused(self._h, self._m(x), self._m(v), self._vec(h), self._vec(xstar), p, float(beta),
                                            int(step), _stream(stream)), "gsgd_step_gossip_fused")

    def step_gossip_pull_fused(self, x, v, h, xstar, peer, step, beta=0.5, stale=False, stream=None):
        keep, p = _perm_arg(peer, self.k)
        _check(lib().gsgd_step_gossip_pull_fused(self._h, self._m(x), self._m(v), self._vec(h), self._vec(xstar), p, float(beta),
                                                 int(bool(stale)), int(step), _stream(stream)),
               "gsgd_step_gossip_pull_fused")

    def step_gossip_push_fused(self, x, v, h, xstar, target, step, stream=None):
        keep, p = _perm_arg(target, self.k)
        _check(lib().gsgd_step_gossip_push_fused(self._h, self._m(x), self._m(v), self._vec(h), self._vec(xstar), p, int(step),
                                                 _stream(stream)), "gsgd_step_gossip_push_fused")

    def philox_raw(self, c1, c2, c3, n_blocks, out, stream=None):
        import torch
        _check(lib().gsgd_philox_raw(self._h, int(c1), int(c2), int(c3), int(n_blocks),
                                     _ptr(out, 4 * int(n_blocks), torch.int32 if out.dtype == torch.int32 else torch.uint32),
                                     _stream(stream)),
               "gsgd_philox_raw")

    def noise_alu_probe(self, workgroups, iters, out, stream=None):
        _check(lib().gsgd_noise_alu_probe(self._h, int(workgroups), int(iters), _ptr(out, int(workgroups) * 256),
                                          _stream(stream)), "gsgd_noise_alu_probe")

    def row_sqnorms(self, x, stream=None):
        out = (C.c_double * self.k)()
        _check(lib().gsgd_row_sqnorms(self._h, self._m(x), out, _stream(stream)), "gsgd_row_sqnorms")
        return np.array(list(out), dtype=np.float64)

    def poke_tickets(self, next_tile, finished, stream=None):
        _check(lib().gsgd_poke_tickets(self._h, int(next_tile), int(finished), _stream(stream)), "gsgd_poke_tickets")

    def stats(self, x, xstar, stream=None):
        out = (C.c_double * 4)()
        _check(lib().gsgd_stats(self._h, self._m(x), self._vec(xstar), out, _stream(stream)), "gsgd_stats")
        return np.array(list(out), dtype=np.float64)


def stats_static(k, d, ld, x, xstar, out, stream=None, block_columns=0):
    """gsgd_stats_static: out is a float64 GPU tensor of 4 elements; nothing is allocated and nothing waits."""
    import torch
    k, d, ld, b = int(k), int(d), int(ld), int(block_columns)
    if k < 1 or d < 1 or ld < d or b < 0:
        raise ValueError("bad geometry k=%d d=%d ld=%d block_columns=%d" % (k, d, ld, b))
    need = (k - 1) * ld + d
    if b > 0:
        last = (d - 1) // b
        need = last * k * b + (k - 1) * b + (d - last * b)
    _check(lib().gsgd_stats_static(k, d, ld, b, _ptr(x, need), _ptr(xstar, d), _ptr(out, 4, torch.float64),
                                   _stream(stream)), "gsgd_stats_static")


def _span(k, d, ld, b):
    """elements a k x ld matrix of d used columns spans in its layout (b = columns per block, 0 = row-major)"""
    if b > 0:
        last = (d - 1) // b
        return last * k * b + (k - 1) * b + (d - last * b)
    return (k - 1) * ld + d


def relayout(k, d, src, src_ld, src_block_columns, dst, dst_ld, dst_block_columns, stream=None):
    """gsgd_relayout: copy a k x d matrix between layouts on the device."""
    k, d = int(k), int(d)
    sl, sb, dl, db = int(src_ld), int(src_block_columns), int(dst_ld), int(dst_block_columns)
    if k < 1 or d < 1 or sl < d or dl < d or sb < 0 or db < 0:
        raise ValueError("bad geometry")
    _check(lib().gsgd_relayout(k, d, sl, sb, _ptr(src, _span(k, d, sl, sb)), dl, db, _ptr(dst, _span(k, d, dl, db)),
                               _stream(stream)), "gsgd_relayout")


def comm_due(step, tau):
    rc = lib().gsgd_comm_due(int(step), int(tau))
    if rc < 0:
        raise GsgdError(rc, "gsgd_comm_due")
    return bool(rc)


def make_perm(seed, step, k):
    out = np.empty(int(k), np.int32)
    _check(lib().gsgd_make_perm(int(seed), int(step), int(k), out.ctypes.data_as(C.POINTER(C.c_int32))),
           "gsgd_make_perm")
    return out


_f64p = C.POINTER(C.c_double)


def _weights_arg(V):
    if not (isinstance(V, np.ndarray) and V.dtype == np.float64 and V.flags.c_contiguous and V.ndim == 2
            and V.shape[0] == V.shape[1]):
        raise ValueError("V must be a C-contiguous square float64 array (updated in place)")
    return V.ctypes.data_as(_f64p)


def weights_pull(V, peer, beta=0.5):
    keep, p = _perm_arg(peer)
    _check(lib().gsgd_weights_pull(_weights_arg(V), int(V.shape[0]), p, float(beta)), "gsgd_weights_pull")


def weights_push(V, target):
    keep, p = _perm_arg(target)
    _check(lib().gsgd_weights_push(_weights_arg(V), int(V.shape[0]), p), "gsgd_weights_push")


def diffusion_potential(V, sqnorm_start, sqnorm_now):
    a = np.ascontiguousarray(sqnorm_start, dtype=np.float64)
    b = np.ascontiguousarray(sqnorm_now, dtype=np.float64)
    out = C.c_double(0.0)
    _check(lib().gsgd_diffusion_potential(_weights_arg(V), int(V.shape[0]), a.ctypes.data_as(_f64p),
                                          b.ctypes.data_as(_f64p), C.byref(out)), "gsgd_diffusion_potential")
    return float(out.value)


def make_tick(seed, tick, k):
    i, j = C.c_int32(0), C.c_int32(0)
    _check(lib().gsgd_make_tick(int(seed), int(tick), int(k), C.byref(i), C.byref(j)), "gsgd_make_tick")
    return int(i.value), int(j.value)


def make_targets(seed, step, k, exclude_self=False):
    out = np.empty(int(k), np.int32)
    _check(lib().gsgd_make_targets(int(seed), int(step), int(k), int(bool(exclude_self)),
                                   out.ctypes.data_as(C.POINTER(C.c_int32))), "gsgd_make_targets")
    return out


def pull_walk(peer):
    """(walk words, stack slots used) for an arbitrary peer map."""
    keep, p = _perm_arg(peer)
    out = np.empty(keep.shape[0], np.uint32)
    slots = C.c_int32(0)
    _check(lib().gsgd_pull_walk(p, int(keep.shape[0]), out.ctypes.data_as(C.POINTER(C.c_uint32)), C.byref(slots)),
           "gsgd_pull_walk")
    return out, int(slots.value)


def push_walk(target):
    """(walk words, stack slots used) of the push-gossip kernel for a target map."""
    keep, p = _perm_arg(target)
    out = np.empty(keep.shape[0], np.uint32)
    slots = C.c_int32(0)
    _check(lib().gsgd_push_walk(p, int(keep.shape[0]), out.ctypes.data_as(C.POINTER(C.c_uint32)), C.byref(slots)),
           "gsgd_push_walk")
    return out, int(slots.value)


def perm_walk(peer_perm):
    keep, p = _perm_arg(peer_perm)
    out = np.empty(keep.shape[0], np.uint16)
    _check(lib().gsgd_perm_walk(p, int(keep.shape[0]), out.ctypes.data_as(C.POINTER(C.c_uint16))), "gsgd_perm_walk")
    return out
