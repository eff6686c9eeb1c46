"""CPU-only checks of the library boundary: every symbol the header declares is
exported, the pure-host entry points (permutation generator, cycle walk) agree
with the oracle and with a definition-level replay, and bad arguments come
back as error codes.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import brute
from paper_1611_04581_amd import gsgd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SEED = 0x161104581


def _declared():
    text = open(os.path.join(ROOT, "include", "gsgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gsgd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert "gsgd_step_gossip" in names and "gsgd_init_replicas" in names
    assert "gsgd_step_allreduce" in names and "gsgd_step_easgd" in names
    L = gsgd.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(gsgd.SIGNATURES) == names       # the binding covers exactly the header


def test_make_perm_bit_exact_with_oracle(oracle):
    for k in [1, 2, 3, 4, 8, 31, 32, 128, 512, 1000]:
        for step in (0, 1, 7, 199, 2**32 - 1):
            a = gsgd.make_perm(SEED, step, k)
            assert np.array_equal(a, oracle.make_perm(SEED, step, k)), (k, step)
    assert np.array_equal(gsgd.make_perm(5, 3, 16), np.array(brute.make_perm(5, 3, 16), np.int32))
    with pytest.raises(gsgd.GsgdError):
        gsgd.make_perm(SEED, 0, 0)
    with pytest.raises(gsgd.GsgdError):
        gsgd.make_perm(SEED, 2**32, 4)


def _replay_walk(walk, xp, beta):
    """What the gossip kernel does with a walk, on plain Python floats:
    finish the previous row when the next one of its cycle arrives, finish the
    last row of a cycle with the first."""
    out = [None] * len(xp)
    first = prev = prev_row = None
    for wd in walk:
        row = int(wd) & gsgd.WALK_ROW_MASK
        cur = xp[row]
        if int(wd) & gsgd.WALK_FIRST:
            first = cur
        else:
            out[prev_row] = prev - beta * (prev - cur)
        if int(wd) & gsgd.WALK_LAST:
            out[row] = cur - beta * (cur - first)
        prev, prev_row = cur, row
    return out


def test_perm_walk_visits_cycles_and_realises_the_mix():
    rng = np.random.default_rng(0)
    perms = [[0], [0, 1], [1, 0], [1, 2, 0], [0, 2, 1], [3, 2, 1, 0], list(range(16)), [(i + 1) % 16 for i in range(16)]]
    perms += [list(rng.permutation(k)) for k in (5, 8, 32, 33, 128, 512) for _ in range(3)]
    for perm in perms:
        k = len(perm)
        walk = gsgd.perm_walk(perm)
        rows = [int(w) & gsgd.WALK_ROW_MASK for w in walk]
        assert sorted(rows) == list(range(k))
        n_first = sum(1 for w in walk if int(w) & gsgd.WALK_FIRST)
        n_last = sum(1 for w in walk if int(w) & gsgd.WALK_LAST)
        assert n_first == n_last >= 1
        assert int(walk[0]) & gsgd.WALK_FIRST and int(walk[-1]) & gsgd.WALK_LAST
        # consecutive rows inside a cycle are linked by the permutation
        for a, b in zip(walk[:-1], walk[1:]):
            if not int(a) & gsgd.WALK_LAST:
                assert perm[int(a) & gsgd.WALK_ROW_MASK] == int(b) & gsgd.WALK_ROW_MASK
                assert not int(b) & gsgd.WALK_FIRST
            else:
                assert int(b) & gsgd.WALK_FIRST
        xp = [float(t) for t in rng.integers(-64, 64, k)]
        got = _replay_walk(walk, xp, 0.5)
        want = [xp[i] - 0.5 * (xp[i] - xp[perm[i]]) for i in range(k)]
        assert got == want


def test_perm_walk_rejects_non_bijections():
    for bad in ([0, 0], [1, 1, 0], [0, 1, 3], [-1, 0], [2, 0, 2]):
        with pytest.raises(gsgd.GsgdError) as e:
            gsgd.perm_walk(bad)
        assert e.value.code == gsgd.ERR_BAD_PERM
    with pytest.raises(gsgd.GsgdError) as e:
        gsgd.perm_walk(list(range(gsgd.MAX_K + 1)))
    assert e.value.code == gsgd.ERR_INVALID_ARG


def _cfg(**kw):
    c = gsgd._Config()
    c.k, c.d, c.ld, c.lr, c.momentum, c.sigma, c.seed, c.noise_kind, c.n_seg = 4, 64, 64, 0.05, 0.9, 0.1, 1, 0, 0
    for name, val in kw.items():
        setattr(c, name, val)
    return c


def test_create_rejects_bad_configurations_before_touching_the_gpu():
    L = gsgd.lib()
    h = C.c_void_p()
    assert L.gsgd_create(None, C.byref(h)) == gsgd.ERR_INVALID_ARG
    for bad in (dict(k=0), dict(k=gsgd.MAX_K + 1), dict(d=0), dict(ld=60), dict(ld=66), dict(noise_kind=2),
                dict(sigma=-1.0), dict(n_seg=-1), dict(n_seg=2)):
        assert L.gsgd_create(C.byref(_cfg(**bad)), C.byref(h)) == gsgd.ERR_INVALID_ARG, bad
        assert not h.value
    sc = (C.c_float * 2)(1.0, 2.0)
    for off in ([1, 10, 64], [0, 10, 63], [0, 40, 40 - 1], [0, 0, 64]):
        arr = (C.c_int64 * 3)(*off)
        c = _cfg(n_seg=2)
        c.seg_offsets = C.cast(arr, C.POINTER(C.c_int64))
        c.seg_lr_scale = C.cast(sc, C.POINTER(C.c_float))
        assert L.gsgd_create(C.byref(c), C.byref(h)) == gsgd.ERR_BAD_SEGMENTS, off


def test_null_context_and_error_strings():
    L = gsgd.lib()
    assert L.gsgd_destroy(None) == gsgd.ERR_INVALID_ARG
    assert L.gsgd_step_allreduce(None, None, None, None, None) == gsgd.ERR_INVALID_ARG
    assert L.gsgd_step_gossip(None, None, None, None, None, 0.5, None) == gsgd.ERR_INVALID_ARG
    assert L.gsgd_step_easgd(None, None, None, None, None, 0.1, None) == gsgd.ERR_INVALID_ARG
    assert L.gsgd_stats(None, None, None, None, None) == gsgd.ERR_INVALID_ARG
    texts = {gsgd.strerror(c) for c in range(0, -9, -1)}
    assert len(texts) == 9 and "unknown error" not in texts
    assert L.gsgd_poke_tickets(None, 0, 0, None) == gsgd.ERR_INVALID_ARG
    assert gsgd.strerror(-99) == "unknown error"


def test_comm_due_follows_the_algorithm_boxes():
    """Algorithms 2-4 exchange at the top of iteration t when t > 0 and
    t = 0 mod tau; with the exchange fused to the end of the previous step
    call, call s exchanges iff s + 1 is such a t."""
    for tau in (1, 2, 3, 10):
        T = 50
        box = [t > 0 and t % tau == 0 for t in range(T + 1)]          # exchange at the top of iteration t
        for s in range(T):
            assert gsgd.comm_due(s, tau) == box[s + 1], (s, tau)
    assert all(gsgd.comm_due(s, 1) for s in range(20))
    with pytest.raises(gsgd.GsgdError):
        gsgd.comm_due(3, 0)


def test_make_tick_bit_exact_with_oracle(oracle):
    for k in (1, 2, 32, 512):
        for t in (0, 1, 1000, 2**32 - 1):
            assert gsgd.make_tick(SEED, t, k) == oracle.make_tick(SEED, t, k)
    with pytest.raises(gsgd.GsgdError):
        gsgd.make_tick(SEED, 2**32, 4)
