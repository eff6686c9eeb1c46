"""Runs the host-only tests of the library's generators and walk builders
against a CPU build of csrc/host_perm.hip with AddressSanitizer and
UndefinedBehaviorSanitizer (the recursion over deep trees and the fixed-size
stacks are where an out-of-bounds write would hide).  Started by
test_sanitizers.py in a process of its own, with the sanitizer runtime
preloaded; argv[1] = the sanitized library.  Exits non-zero on any finding."""
import ctypes as C
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
sys.path.insert(0, ROOT)
sys.path.insert(0, HERE)

from paper_1611_04581_amd import gsgd          # noqa: E402  (the binding; its library is swapped below)

HOST_ONLY = ["gsgd_make_perm", "gsgd_make_targets", "gsgd_make_tick", "gsgd_pull_walk", "gsgd_push_walk", "gsgd_perm_walk"]


def main():
    L = C.CDLL(sys.argv[1])
    for name in HOST_ONLY:
        fn = getattr(L, name)
        fn.restype, fn.argtypes = gsgd.SIGNATURES[name]
    gsgd.lib = lambda: L                        # every binding call now lands in the sanitized build
    gsgd.strerror = lambda code: "error %d" % code
    from oracle import oracle
    oracle.lib()
    import test_abi_host as A
    import test_oracle_maps as M
    A.test_make_perm_bit_exact_with_oracle(oracle)
    A.test_perm_walk_visits_cycles_and_realises_the_mix()
    A.test_perm_walk_rejects_non_bijections()
    A.test_make_tick_bit_exact_with_oracle(oracle)
    for ex in (False, True):
        M.test_targets_match_restatement_and_library(oracle, ex)
    for k in (1, 2, 5, 32, 33, 128, 512):
        M.test_pull_walk_realises_the_definition(k)
        M.test_push_walk_realises_the_definition(k)
    M.test_pull_walk_of_a_permutation_is_the_cycle_walk()
    # the shapes that stress the builders most: the longest chain, the bushiest star, complete trees, all at the
    # largest k, plus maps that must be refused
    k = gsgd.MAX_K
    for m in ([max(i - 1, 0) for i in range(k)], [0] * k, [(i - 1) // 2 if i else 0 for i in range(k)],
              [(i - 1) // 3 if i else 0 for i in range(k)], [(i + 1) % k for i in range(k)], list(range(k)),
              [k - 1 - i for i in range(k)]):
        gsgd.pull_walk(m)
        gsgd.push_walk(m)
    for bad in ([k] * k, [-1] * k):
        for fn in (gsgd.pull_walk, gsgd.push_walk, gsgd.perm_walk):
            try:
                fn(bad)
            except gsgd.GsgdError:
                pass
            else:
                raise SystemExit("a map outside 0..k-1 was accepted")
    print("host generators and walk builders: clean under the sanitizers")


if __name__ == "__main__":
    main()
