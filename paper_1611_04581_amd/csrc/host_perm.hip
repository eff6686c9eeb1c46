// Host-side peer selection: the per-step random permutation ("choose a target
// j" of Algorithms 3 and 4 of the paper, with every target used once) and its
// decomposition into cycles, which is the order the gossip kernel walks.
#include <string.h>

#include "gsgd_internal.hpp"

namespace gsgd {

// Philox4x32-10 on the host (Salmon et al., SC'11): ten rounds of two 32x32
// multiplies whose halves are crossed with the other counter words and the key.
void host_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t a = ctr[0], b = ctr[1], c = ctr[2], e = ctr[3];
    uint32_t ka = key[0], kb = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t prod_a = 0xD2511F53ull * a;
        const uint64_t prod_c = 0xCD9E8D57ull * c;
        const uint32_t na = static_cast<uint32_t>(prod_c >> 32) ^ b ^ ka;
        const uint32_t nb = static_cast<uint32_t>(prod_c);
        const uint32_t nc = static_cast<uint32_t>(prod_a >> 32) ^ e ^ kb;
        const uint32_t ne = static_cast<uint32_t>(prod_a);
        a = na; b = nb; c = nc; e = ne;
        ka += 0x9E3779B9u;
        kb += 0xBB67AE85u;
    }
    out[0] = a; out[1] = b; out[2] = c; out[3] = e;
}

int build_walk(const int32_t* perm, int32_t k, Walk* out)
{
    if (!perm || !out || k < 1 || k > GSGD_MAX_K) return GSGD_ERR_INVALID_ARG;
    bool hit[GSGD_MAX_K];
    memset(hit, 0, sizeof(hit));
    for (int32_t i = 0; i < k; ++i) {
        const int32_t j = perm[i];
        if (j < 0 || j >= k || hit[j]) return GSGD_ERR_BAD_PERM;
        hit[j] = true;
    }
    bool seen[GSGD_MAX_K];
    memset(seen, 0, sizeof(seen));
    int32_t t = 0;
    for (int32_t start = 0; start < k; ++start) {
        if (seen[start]) continue;
        const int32_t head = t;
        int32_t i = start;
        do {
            seen[i] = true;
            out->seq[t++] = static_cast<uint32_t>(i);
            i = perm[i];
        } while (i != start);
        out->seq[head] |= WALK_FIRST;
        out->seq[t - 1] |= WALK_LAST;
    }
    for (int32_t r = t; r < GSGD_MAX_K; ++r) out->seq[r] = 0;
    return t == k ? GSGD_OK : GSGD_ERR_BAD_PERM;
}

// Visiting order for an arbitrary pull map ("each node pulls from one uniformly
// chosen node", Section 3.1): the map is a functional graph, i.e. cycles with
// trees hanging off them.  Cycles are walked as for a permutation; right after
// a cycle node is loaded, every node that pulls from it is visited depth-first
// (children in ascending index).  A tree node's peer is its parent, which was
// loaded earlier and whose x' is still held (the cycle register at depth 1,
// stack level depth-2 otherwise), so tree nodes are finished the moment they
// are loaded.  *levels is the number of stack levels the kernel needs.
int build_pull_walk(const int32_t* peer, int32_t k, Walk* out, int* levels)
{
    if (!peer || !out || !levels || k < 1 || k > GSGD_MAX_K) return GSGD_ERR_INVALID_ARG;
    for (int32_t i = 0; i < k; ++i)
        if (peer[i] < 0 || peer[i] >= k) return GSGD_ERR_BAD_PERM;
    // which nodes lie on a cycle: follow the map k steps from everywhere (lands on a cycle), then mark that cycle
    bool on_cycle[GSGD_MAX_K];
    memset(on_cycle, 0, sizeof(on_cycle));
    for (int32_t s = 0; s < k; ++s) {
        int32_t i = s;
        for (int32_t step = 0; step < k; ++step) i = peer[i];
        while (!on_cycle[i]) { on_cycle[i] = true; i = peer[i]; }
    }
    // children lists (nodes pulling from j, cycle predecessors excluded), ascending by construction
    int32_t head[GSGD_MAX_K], next[GSGD_MAX_K], tail[GSGD_MAX_K];
    for (int32_t i = 0; i < k; ++i) head[i] = tail[i] = next[i] = -1;
    for (int32_t i = 0; i < k; ++i) {
        if (on_cycle[i]) continue;
        const int32_t j = peer[i];
        if (head[j] < 0) head[j] = i; else next[tail[j]] = i;
        tail[j] = i;
    }
    bool seen[GSGD_MAX_K];
    memset(seen, 0, sizeof(seen));
    int32_t t = 0, max_level = 0;
    int32_t stack_node[GSGD_MAX_K], stack_child[GSGD_MAX_K];
    for (int32_t start = 0; start < k; ++start) {
        if (!on_cycle[start] || seen[start]) continue;
        const int32_t first_slot = t;
        int32_t last_cycle_slot = t;
        int32_t c = start;
        do {
            seen[c] = true;
            last_cycle_slot = t;
            out->seq[t++] = static_cast<uint32_t>(c);
            // depth-first over the tree below cycle node c
            int32_t sp = 0;
            stack_node[0] = c;
            stack_child[0] = head[c];
            while (sp >= 0) {
                const int32_t child = stack_child[sp];
                if (child < 0) { --sp; continue; }
                stack_child[sp] = next[child];
                const int32_t depth = sp + 1;                 // distance of `child` to the cycle
                uint32_t word = static_cast<uint32_t>(child) | WALK_TREE | (static_cast<uint32_t>(depth) << WALK_DEPTH_SHIFT);
                if (head[child] >= 0) {
                    word |= WALK_PUSH;
                    if (depth > max_level) max_level = depth;  // uses stack level depth-1
                }
                seen[child] = true;
                out->seq[t++] = word;
                if (head[child] >= 0) { ++sp; stack_node[sp] = child; stack_child[sp] = head[child]; }
            }
            c = peer[c];
        } while (c != start);
        out->seq[first_slot] |= WALK_FIRST;
        out->seq[last_cycle_slot] |= WALK_LAST;
    }
    for (int32_t r = t; r < GSGD_MAX_K; ++r) out->seq[r] = 0;
    *levels = max_level;
    return t == k ? GSGD_OK : GSGD_ERR_BAD_PERM;
}

}  // namespace gsgd

extern "C" int gsgd_make_perm(uint64_t seed, uint64_t step, int32_t k, int32_t* out)
{
    if (!out || k < 1 || step > 0xFFFFFFFFull) return GSGD_ERR_INVALID_ARG;
    const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    for (int32_t i = 0; i < k; ++i) out[i] = i;
    for (int32_t i = k - 1; i >= 1; --i) {
        const uint32_t ctr[4] = {static_cast<uint32_t>(i), 0u, static_cast<uint32_t>(step), 5u};
        uint32_t r[4];
        gsgd::host_philox4x32_10(ctr, key, r);
        const int32_t j = static_cast<int32_t>((static_cast<uint64_t>(r[0]) * static_cast<uint64_t>(i + 1)) >> 32);
        const int32_t tmp = out[i];
        out[i] = out[j];
        out[j] = tmp;
    }
    return GSGD_OK;
}

extern "C" int gsgd_perm_walk(const int32_t* peer_perm, int32_t k, uint16_t* walk)
{
    if (!walk) return GSGD_ERR_INVALID_ARG;
    gsgd::Walk w;
    const int rc = gsgd::build_walk(peer_perm, k, &w);
    if (rc != GSGD_OK) return rc;
    for (int32_t t = 0; t < k; ++t) walk[t] = static_cast<uint16_t>(w.seq[t]);
    return GSGD_OK;
}
