// Host-side peer selection: the per-step random permutation (the target choice
// of Algorithms 3 and 4 of the paper, with every node chosen once) and its
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

// Visiting order for an arbitrary pull map (every node pulling from one node
// drawn uniformly, Section 3.1).  The map is a functional graph: cycles with trees
// hanging off them.  Cycles are walked as for a permutation; right after a
// cycle node, the trees of nodes that pull (directly or through others) from
// it are visited depth-first, parents before children, so that a tree node's
// peer has always been loaded already and the node is finished on the spot.
//
// Order of the children of a node: childless ones first, then the others by
// the number of stack slots their subtree needs, the neediest last.  Only a
// subtree that is not the last one forces its parent's value to be saved, so
// slots(n) = max(slots(last child), 1 + slots(any other child with children)),
// which grows like log2 of the subtree size instead of its height.
namespace {

struct PullWalkBuilder {
    Walk*          out;
    int32_t        t;
    int            max_slot;
    int32_t        head[GSGD_MAX_K], next[GSGD_MAX_K];   // children lists (tree nodes only), ascending index
    int32_t        need[GSGD_MAX_K];                     // slots the subtree below a tree node needs
    int32_t        pool[GSGD_MAX_K];                     // ordered children of the nodes on the current path
    int32_t        pool_top;

    bool inner(int32_t n) const { return head[n] >= 0; }

    // Writes the children of n in visiting order to kids; *first_inner is the
    // position of the first child that has children itself.
    int32_t ordered_children(int32_t n, int32_t* kids, int32_t* first_inner) const
    {
        int32_t m = 0;
        for (int32_t c = head[n]; c >= 0; c = next[c]) if (!inner(c)) kids[m++] = c;
        *first_inner = m;
        for (int32_t c = head[n]; c >= 0; c = next[c]) if (inner(c)) kids[m++] = c;
        for (int32_t a = *first_inner + 1; a < m; ++a) {          // stable insertion sort by need
            const int32_t c = kids[a];
            int32_t b = a;
            while (b > *first_inner && need[kids[b - 1]] > need[c]) { kids[b] = kids[b - 1]; --b; }
            kids[b] = c;
        }
        return m;
    }

    // Emits the subtree below n (n itself is already out).  On entry the
    // kernel's `par` holds n's value unless n is a cycle node, in which case
    // every child fetches it from the cycle register.  Slots below `base` are
    // in use by ancestors.
    void emit_children(int32_t n, int base, bool n_on_cycle)
    {
        int32_t* kids = pool + pool_top;
        int32_t first_inner = 0;
        const int32_t m = ordered_children(n, kids, &first_inner);
        pool_top += m;
        for (int32_t a = 0; a < m; ++a) {
            const int32_t c = kids[a];
            uint32_t word = static_cast<uint32_t>(c) | WALK_TREE;
            const bool c_inner = a >= first_inner;
            const bool last = a == m - 1;
            int child_base = base;
            if (n_on_cycle) {
                word |= WALK_RESTORE_PREV;
            } else if (c_inner && a > first_inner) {
                word |= WALK_RESTORE_SLOT | (static_cast<uint32_t>(base) << WALK_SLOT_SHIFT);
            }
            if (c_inner) {
                word |= WALK_DESCEND;
                if (!n_on_cycle && !last) {
                    // n's value is needed again after c's subtree: it sits in slot `base` meanwhile
                    if (a == first_inner) word |= WALK_SAVE | (static_cast<uint32_t>(base) << WALK_SLOT_SHIFT);
                    if (base > max_slot) max_slot = base;
                    child_base = base + 1;
                }
            }
            out->seq[t++] = word;
            if (c_inner) emit_children(c, child_base, false);
        }
        pool_top -= m;
    }
};

}  // namespace

int build_pull_walk(const int32_t* peer, int32_t k, Walk* out, int* has_trees, int* slots_used)
{
    if (!peer || !out || !has_trees || !slots_used || k < 1 || k > GSGD_MAX_K) return GSGD_ERR_INVALID_ARG;
    for (int32_t i = 0; i < k; ++i)
        if (peer[i] < 0 || peer[i] >= k) return GSGD_ERR_BAD_PERM;
    // which nodes lie on a cycle: follow the map from every unvisited node, tagging the path; a path that runs
    // into its own tag has closed a new cycle, one that runs into an older tag has joined a known component
    bool on_cycle[GSGD_MAX_K];
    int32_t tag[GSGD_MAX_K];
    memset(on_cycle, 0, sizeof(on_cycle));
    memset(tag, 0, sizeof(tag));
    for (int32_t s = 0; s < k; ++s) {
        int32_t i = s;
        while (tag[i] == 0) { tag[i] = s + 1; i = peer[i]; }
        if (tag[i] != s + 1) continue;
        for (int32_t j = i; !on_cycle[j]; j = peer[j]) on_cycle[j] = true;
    }
    PullWalkBuilder b;
    b.out = out;
    b.t = 0;
    b.max_slot = -1;
    b.pool_top = 0;
    int32_t tail[GSGD_MAX_K];
    for (int32_t i = 0; i < k; ++i) { b.head[i] = tail[i] = b.next[i] = -1; b.need[i] = 0; }
    int32_t n_tree = 0;
    for (int32_t i = 0; i < k; ++i) {
        if (on_cycle[i]) continue;
        ++n_tree;
        const int32_t j = peer[i];
        if (b.head[j] < 0) b.head[j] = i; else b.next[tail[j]] = i;
        tail[j] = i;
    }
    // slots needed below every tree node, children before parents (reverse breadth-first order)
    int32_t order[GSGD_MAX_K];
    int32_t n_order = 0;
    for (int32_t i = 0; i < k; ++i)
        if (on_cycle[i]) for (int32_t c = b.head[i]; c >= 0; c = b.next[c]) order[n_order++] = c;
    for (int32_t q = 0; q < n_order; ++q)
        for (int32_t c = b.head[order[q]]; c >= 0; c = b.next[c]) order[n_order++] = c;
    if (n_order != n_tree) return GSGD_ERR_BAD_PERM;        // cannot happen for a valid map
    for (int32_t q = n_order - 1; q >= 0; --q) {
        const int32_t n = order[q];
        int32_t largest = -1, second = -1;
        for (int32_t c = b.head[n]; c >= 0; c = b.next[c]) {
            if (!b.inner(c)) continue;
            if (b.need[c] > largest) { second = largest; largest = b.need[c]; }
            else if (b.need[c] > second) second = b.need[c];
        }
        b.need[n] = largest < 0 ? 0 : (second < 0 ? largest : (largest > second + 1 ? largest : second + 1));
    }
    bool seen[GSGD_MAX_K];
    memset(seen, 0, sizeof(seen));
    for (int32_t start = 0; start < k; ++start) {
        if (!on_cycle[start] || seen[start]) continue;
        const int32_t first_slot = b.t;
        int32_t last_cycle_slot = b.t;
        int32_t c = start;
        do {
            seen[c] = true;
            last_cycle_slot = b.t;
            out->seq[b.t++] = static_cast<uint32_t>(c);
            b.emit_children(c, 0, true);
            c = peer[c];
        } while (c != start);
        out->seq[first_slot] |= WALK_FIRST;
        out->seq[last_cycle_slot] |= WALK_LAST;
    }
    for (int32_t r = b.t; r < GSGD_MAX_K; ++r) out->seq[r] = 0;
    if (b.t != k) return GSGD_ERR_BAD_PERM;
    *has_trees = n_tree > 0 ? 1 : 0;
    *slots_used = b.max_slot + 1;
    return *slots_used <= WALK_SLOTS ? GSGD_OK : GSGD_ERR_UNSUPPORTED;
}

// Visiting order for push-gossip (Algorithm 4): target[i] is where node i sends
// its parameters (target[i] == i: nowhere).  A node is finished when all its
// senders have been visited, so trees are walked children first; the cycles of
// the map are walked in the direction of sending, each cycle node after the
// trees that send to it, its cycle predecessor's x' riding along in a register.
//
// Among the senders of a node, the one whose subtree needs most stack slots
// goes first (nothing is pending yet), the others follow with the partial sum
// parked in a slot, childless senders last: the same log2 bound on the number
// of slots as for the pull walk.
namespace {

struct PushWalkBuilder {
    Walk*   out;
    int32_t t;
    int     max_slot;
    int32_t head[GSGD_MAX_K], next[GSGD_MAX_K];   // tree senders of every node, ascending index
    int32_t n_senders[GSGD_MAX_K];                // tree senders only
    int32_t need[GSGD_MAX_K];
    int32_t pool[GSGD_MAX_K];
    int32_t pool_top;

    bool inner(int32_t n) const { return head[n] >= 0; }

    // senders of n in visiting order: those with senders of their own by descending need, then the rest
    int32_t ordered_senders(int32_t n, int32_t* kids, int32_t* n_inner) const
    {
        int32_t m = 0;
        for (int32_t c = head[n]; c >= 0; c = next[c]) if (inner(c)) kids[m++] = c;
        *n_inner = m;
        for (int32_t a = 1; a < m; ++a) {                       // stable insertion sort, descending need
            const int32_t c = kids[a];
            int32_t b = a;
            while (b > 0 && need[kids[b - 1]] < need[c]) { kids[b] = kids[b - 1]; --b; }
            kids[b] = c;
        }
        for (int32_t c = head[n]; c >= 0; c = next[c]) if (!inner(c)) kids[m++] = c;
        return m;
    }

    // Emits everything that sends (directly or not) to n through tree edges.
    // Afterwards the kernel's acc holds the sum of n's tree senders' x'.
    void emit_senders(int32_t n, int base)
    {
        int32_t* kids = pool + pool_top;
        int32_t n_inner = 0;
        const int32_t m = ordered_senders(n, kids, &n_inner);
        pool_top += m;
        for (int32_t a = 0; a < m; ++a) {
            const int32_t c = kids[a];
            const bool c_inner = a < n_inner;
            uint32_t word = static_cast<uint32_t>(c) | WALK_TREE
                          | (static_cast<uint32_t>(1 + n_senders[c]) << PUSH_COUNT_SHIFT);
            if (c_inner) word |= PUSH_HAS_SENDERS;
            if (a == 0) word |= PUSH_START;
            else if (c_inner) word |= PUSH_RESTORE_ADD | (static_cast<uint32_t>(base) << PUSH_SLOT_SHIFT);
            else word |= PUSH_ADD;
            if (a + 1 < n_inner) {                              // the next sender's subtree will use acc
                word |= PUSH_SAVE_AFTER | (static_cast<uint32_t>(base) << PUSH_SLOT_SHIFT);
                if (base > max_slot) max_slot = base;
            }
            if (c_inner) emit_senders(c, a == 0 ? base : base + 1);
            out->seq[t++] = word;
        }
        pool_top -= m;
    }
};

}  // namespace

int build_push_walk(const int32_t* target, int32_t k, Walk* out, int* slots_used)
{
    if (!target || !out || !slots_used || k < 1 || k > GSGD_MAX_K) return GSGD_ERR_INVALID_ARG;
    for (int32_t i = 0; i < k; ++i)
        if (target[i] < 0 || target[i] >= k) return GSGD_ERR_BAD_PERM;
    bool on_cycle[GSGD_MAX_K];
    int32_t tag[GSGD_MAX_K];
    memset(on_cycle, 0, sizeof(on_cycle));
    memset(tag, 0, sizeof(tag));
    for (int32_t s = 0; s < k; ++s) {
        int32_t i = s;
        while (tag[i] == 0) { tag[i] = s + 1; i = target[i]; }
        if (tag[i] != s + 1) continue;
        for (int32_t j = i; !on_cycle[j]; j = target[j]) on_cycle[j] = true;
    }
    PushWalkBuilder b;
    b.out = out;
    b.t = 0;
    b.max_slot = -1;
    b.pool_top = 0;
    int32_t tail[GSGD_MAX_K];
    for (int32_t i = 0; i < k; ++i) { b.head[i] = tail[i] = b.next[i] = -1; b.need[i] = 0; b.n_senders[i] = 0; }
    for (int32_t i = 0; i < k; ++i) {
        if (on_cycle[i]) continue;
        const int32_t j = target[i];
        if (b.head[j] < 0) b.head[j] = i; else b.next[tail[j]] = i;
        tail[j] = i;
        ++b.n_senders[j];
    }
    // slots needed to assemble every node's sum, senders before receivers (reverse breadth-first order);
    // cycle nodes last, they are receivers of trees too
    int32_t order[GSGD_MAX_K];
    int32_t n_order = 0;
    for (int32_t i = 0; i < k; ++i) if (on_cycle[i]) order[n_order++] = i;
    for (int32_t q = 0; q < n_order; ++q)
        for (int32_t c = b.head[order[q]]; c >= 0; c = b.next[c]) order[n_order++] = c;
    if (n_order != k) return GSGD_ERR_BAD_PERM;              // cannot happen for a valid map
    for (int32_t q = n_order - 1; q >= 0; --q) {
        const int32_t n = order[q];
        int32_t largest = -1, second = -1;
        for (int32_t c = b.head[n]; c >= 0; c = b.next[c]) {
            if (!b.inner(c)) continue;
            if (b.need[c] > largest) { second = largest; largest = b.need[c]; }
            else if (b.need[c] > second) second = b.need[c];
        }
        b.need[n] = largest < 0 ? 0 : (second < 0 ? largest : (largest > second + 1 ? largest : second + 1));
    }
    bool seen[GSGD_MAX_K];
    memset(seen, 0, sizeof(seen));
    for (int32_t start = 0; start < k; ++start) {
        if (!on_cycle[start] || seen[start]) continue;
        const bool self_loop = target[start] == start;
        int32_t first_slot = -1, last_slot = -1;
        int32_t c = start;
        do {
            seen[c] = true;
            b.emit_senders(c, 0);
            uint32_t word = static_cast<uint32_t>(c)
                          | (static_cast<uint32_t>(1 + b.n_senders[c] + (self_loop ? 0 : 1)) << PUSH_COUNT_SHIFT);
            if (b.inner(c)) word |= PUSH_HAS_SENDERS;
            if (first_slot < 0) first_slot = b.t;
            last_slot = b.t;
            out->seq[b.t++] = word;
            c = target[c];
        } while (c != start);
        out->seq[first_slot] |= WALK_FIRST;
        out->seq[last_slot] |= WALK_LAST;
    }
    for (int32_t r = b.t; r < GSGD_MAX_K; ++r) out->seq[r] = 0;
    if (b.t != k) return GSGD_ERR_BAD_PERM;
    *slots_used = b.max_slot + 1;
    return *slots_used <= WALK_SLOTS ? GSGD_OK : GSGD_ERR_UNSUPPORTED;
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

// Independent uniform targets, one draw per node (Section 3.1: j ~ Uniform over
// the nodes): node i takes word 0 of Philox(counter (i, 1, step, 5)).
extern "C" int gsgd_make_targets(uint64_t seed, uint64_t step, int32_t k, int exclude_self, int32_t* out)
{
    if (!out || k < 1 || step > 0xFFFFFFFFull || (exclude_self != 0 && exclude_self != 1)) return GSGD_ERR_INVALID_ARG;
    if (exclude_self && k < 2) return GSGD_ERR_INVALID_ARG;
    const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    const uint64_t range = static_cast<uint64_t>(exclude_self ? k - 1 : k);
    for (int32_t i = 0; i < k; ++i) {
        const uint32_t ctr[4] = {static_cast<uint32_t>(i), 1u, static_cast<uint32_t>(step), 5u};
        uint32_t r[4];
        gsgd::host_philox4x32_10(ctr, key, r);
        int32_t j = static_cast<int32_t>((static_cast<uint64_t>(r[0]) * range) >> 32);
        if (exclude_self && j >= i) ++j;          // skip over the node itself
        out[i] = j;
    }
    return GSGD_OK;
}

// Which node's clock ticks and whom it pulls from (Section 6.1.2): both uniform
// over the nodes and independent, words 0 and 1 of Philox(counter (tick, 2, 0, 5)).
extern "C" int gsgd_make_tick(uint64_t seed, uint64_t tick, int32_t k, int32_t* i_out, int32_t* j_out)
{
    if (!i_out || !j_out || k < 1 || tick > 0xFFFFFFFFull) return GSGD_ERR_INVALID_ARG;
    const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    const uint32_t ctr[4] = {static_cast<uint32_t>(tick), 2u, 0u, 5u};
    uint32_t r[4];
    gsgd::host_philox4x32_10(ctr, key, r);
    *i_out = static_cast<int32_t>((static_cast<uint64_t>(r[0]) * static_cast<uint64_t>(k)) >> 32);
    *j_out = static_cast<int32_t>((static_cast<uint64_t>(r[1]) * static_cast<uint64_t>(k)) >> 32);
    return GSGD_OK;
}

extern "C" int gsgd_pull_walk(const int32_t* peer, int32_t k, uint32_t* walk, int32_t* slots_used)
{
    if (!walk || !slots_used) return GSGD_ERR_INVALID_ARG;
    gsgd::Walk w;
    int has_trees = 0, slots = 0;
    const int rc = gsgd::build_pull_walk(peer, k, &w, &has_trees, &slots);
    if (rc != GSGD_OK) return rc;
    for (int32_t t = 0; t < k; ++t) walk[t] = w.seq[t];
    *slots_used = slots;
    return GSGD_OK;
}

extern "C" int gsgd_push_walk(const int32_t* target, int32_t k, uint32_t* walk, int32_t* slots_used)
{
    if (!walk || !slots_used) return GSGD_ERR_INVALID_ARG;
    gsgd::Walk w;
    int slots = 0;
    const int rc = gsgd::build_push_walk(target, k, &w, &slots);
    if (rc != GSGD_OK) return rc;
    for (int32_t t = 0; t < k; ++t) walk[t] = w.seq[t];
    *slots_used = slots;
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
