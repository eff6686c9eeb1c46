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
