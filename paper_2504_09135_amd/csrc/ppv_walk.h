// Prefix walk over the per-depth arrays, shared by the kernels of libppv_hip.so.
#pragma once
#include "ppv_device.h"
#include "ppv_internal.h"

namespace {

// ------------------------------------------------------------------------------------------
// Prefix walk, one wavefront per prefix (Section 3.2 "Parallel Verification": the search that
// locates a prefix in sorted S; here it descends the per-depth arrays, one 64-way search among
// the children of the current prefix per token, instead of log2|S| probes of whole rows).
// All 64 lanes call it with the same arguments; every result is wave-uniform.
struct Walk {
    uint32_t node;    // the prefix's entry (meaningful when found)
    uint32_t cb, ce;  // its children (when found)
    uint32_t tok;     // its entry's token word with flags (when found and t > 0)
    uint32_t lo, hi;  // rank range in sorted S; lo == hi == insertion rank when not found
    bool found;       // the prefix is a prefix of at least one member
    bool member;      // the prefix itself is in S
};

// Search `key` among the entries [begin, end) (strictly increasing tokens).  Returns the first
// position whose token is >= key; on a match *hit is that entry and *next_child the child offset
// of the entry after it (the end of the match's own children), else hit->tok = PPV_NO_SLOT.
__device__ inline uint32_t wave_search(const NodeEnt *__restrict__ ent, uint32_t begin, uint32_t end, uint32_t key,
                                       int lane, NodeEnt *hit, uint32_t *next_child) {
    uint32_t lo = begin, hi = end;
    while (hi - lo > (uint32_t)(WAVE - 1)) {
        uint32_t n = hi - lo;
        uint32_t step = (n + WAVE - 1) / WAVE;
        uint32_t p = (uint32_t)(lane + 1) * step;
        if (p > n) p = n;
        uint32_t v = ent[lo + p - 1].tok & PPV_NODE_TOKEN;  // 64 pivots, the last one is the last entry
        int c = __popcll(__ballot(v < key));                // pivots below the key
        if (c == WAVE) { lo = hi; break; }                  // everything is below the key
        uint32_t nlo = lo + (uint32_t)c * step;
        uint32_t nhi = lo + (uint32_t)(c + 1) * step;
        if (nhi > hi) nhi = hi;
        lo = nlo;
        hi = nhi;
    }
    // at most 63 candidates: lane l takes entry lo+l, one lane more takes the entry after them
    // (always there: the array ends with a sentinel), which closes the last candidate's children
    const uint32_t n = hi - lo;
    NodeEnt e;
    e.tok = PPV_NO_SLOT;
    e.child = 0;
    if ((uint32_t)lane <= n) e = ent[lo + lane];
    const bool in = (uint32_t)lane < n;
    const uint32_t v = e.tok & PPV_NODE_TOKEN;
    const int c = __popcll(__ballot(in && v < key));
    const uint64_t eq = __ballot(in && v == key);
    hit->tok = PPV_NO_SLOT;
    if (eq) {
        const int l = __ffsll((long long)eq) - 1;
        hit->tok = lane_value(e.tok, l);
        hit->child = lane_value(e.child, l);
        *next_child = lane_value(e.child, l + 1);
    }
    return lo + (uint32_t)c;
}

// The descent from a known node: token i of the prefix is searched among the children of the node reached
// by tokens 0..i-1, for i = start .. t-1.  `mine` is lane l's token l of the prefix (the first 64 tokens
// in one coalesced load; token i is broadcast from lane i).
__device__ inline Walk walk_from(const IndexView &ix, const int32_t *__restrict__ prefix, int t, int lane, int32_t mine,
                                 int start, uint32_t node, uint32_t tokw, uint32_t cb, uint32_t ce) {
    Walk w;
    w.node = node;
    w.cb = cb;
    w.ce = ce;
    w.tok = tokw;
    w.found = true;
    w.member = false;
    for (int i = start; i < t; i++) {
        const uint32_t key = (uint32_t)((i < WAVE) ? lane_value(mine, i) : prefix[i]);
        NodeEnt hit;
        uint32_t next_child = 0;
        const uint32_t j = wave_search(ix.ent, w.cb, w.ce, key, lane, &hit, &next_child);
        if (hit.tok == PPV_NO_SLOT || key > PPV_NODE_TOKEN) {
            // every member below child j sorts before the prefix; with no such child the prefix
            // sorts after the whole range of the current node
            const uint32_t rank = (j < w.ce) ? ix.node_lo[j] : (w.node ? ix.node_hi[w.node] : ix.n_rows);
            w.lo = rank;
            w.hi = rank;
            w.found = false;
            w.member = false;
            return w;
        }
        w.node = j;
        w.tok = hit.tok;
        w.cb = hit.child;
        w.ce = next_child;
    }
    w.lo = w.node ? ix.node_lo[w.node] : 0u;
    w.hi = w.node ? ix.node_hi[w.node] : ix.n_rows;
    w.member = (w.tok & PPV_NODE_TERMINAL) != 0u;
    return w;
}

// Hash of a token string: two polynomials over the tokens, H_d = sum_{i<=d} (tok_i + 1) * K^(d-i) mod 2^32 with
// two multipliers K, mixed into 64 bits at the end.  A polynomial, because its evaluation is associative:
// filling the table takes the tokens one at a time (Horner), while a query needs the hashes of ALL its
// prefixes at once, lane d that of tokens 0..d, and gets them from one prefix scan over the wavefront
// (seven DPP steps) instead of a loop as long as the prefix.
constexpr uint32_t PREFIX_HASH_K1 = 0x9E3779B1u, PREFIX_HASH_K2 = 0x85EBCA77u;   // odd
struct PrefixHash {
    uint32_t h1, p1, h2, p2;   // the two polynomial values and K^length for each
};
__device__ inline PrefixHash prefix_hash_token(uint32_t tok) { return {tok + 1u, PREFIX_HASH_K1, tok + 1u, PREFIX_HASH_K2}; }
// the hash of string a followed by string b
__device__ inline PrefixHash prefix_hash_join(const PrefixHash &a, const PrefixHash &b) {
    return {a.h1 * b.p1 + b.h1, a.p1 * b.p1, a.h2 * b.p2 + b.h2, a.p2 * b.p2};
}
__device__ inline void prefix_hash_finish(const PrefixHash &x, uint32_t size, uint32_t fp_mask, uint32_t *slot,
                                          uint32_t *fp) {
    uint64_t h = ((uint64_t)x.h1 << 32) | x.h2;
    h ^= h >> 32;
    h *= 0xD6E8FEB86659FD93ull;
    h ^= h >> 29;
    *slot = __umulhi((uint32_t)(h >> 32), size);
    *fp = ((uint32_t)h & fp_mask) | 1u;
}
// lane l receives the value of the lane CTRL points to, or the empty string's hash where there is none
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF> __device__ inline PrefixHash prefix_hash_dpp(const PrefixHash &x) {
    return {(uint32_t)__builtin_amdgcn_update_dpp(0, (int)x.h1, CTRL, ROW_MASK, BANK_MASK, false),
            (uint32_t)__builtin_amdgcn_update_dpp(1, (int)x.p1, CTRL, ROW_MASK, BANK_MASK, false),
            (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x.h2, CTRL, ROW_MASK, BANK_MASK, false),
            (uint32_t)__builtin_amdgcn_update_dpp(1, (int)x.p2, CTRL, ROW_MASK, BANK_MASK, false)};
}
// lane l: the hash of the tokens of lanes 0..l (x = the lane's own token as a one-token string)
__device__ inline PrefixHash prefix_hash_scan(const PrefixHash &x) {
    PrefixHash t = x;
    t = prefix_hash_join(prefix_hash_dpp<DPP_ROW_SHR1>(x), t);
    t = prefix_hash_join(prefix_hash_dpp<DPP_ROW_SHR2>(x), t);
    t = prefix_hash_join(prefix_hash_dpp<DPP_ROW_SHR3>(x), t);              // up to 4 consecutive lanes of the row
    t = prefix_hash_join(prefix_hash_dpp<DPP_ROW_SHR4, 0xF, 0xE>(t), t);
    t = prefix_hash_join(prefix_hash_dpp<DPP_ROW_SHR8, 0xF, 0xC>(t), t);    // prefix inside each row of 16
    t = prefix_hash_join(prefix_hash_dpp<DPP_ROW_BCAST15, 0xA>(t), t);
    t = prefix_hash_join(prefix_hash_dpp<DPP_ROW_BCAST31, 0xC>(t), t);
    return t;
}

// Locates the prefix.  With a look-up table every length of the prefix is probed at once (lane d hashes
// tokens 0..d); the deepest hit is checked exactly -- its node must have that depth and the first member
// under it must begin with these tokens -- and the descent then starts there: nothing is left to descend
// when the whole prefix is in the index, one failing step (which yields the rank) when it is not.  A hit
// that fails the check (a fingerprint collision) only costs the shortcut: the descent starts at the root.
// `mine` = first_tokens(prefix, stride, lane), requested by the caller before the prefix's length is known.
__device__ inline int32_t first_tokens(const int32_t *__restrict__ prefix, int stride, int lane) {
    return (lane < stride) ? prefix[lane] : 0;
}
__device__ inline Walk walk_prefix(const IndexView &ix, const int32_t *__restrict__ prefix, int32_t mine, int t,
                                   int lane) {
    const uint32_t root_cb = ix.ent[0].child, root_ce = ix.ent[1].child;
    int tl = t < WAVE ? t : WAVE;
    tl = tl < ix.l_max ? tl : ix.l_max;   // nothing longer than the longest member is in the index
    if (ix.lookup_size != 0u && tl > 0) {
        uint32_t slot, fp;
        prefix_hash_finish(prefix_hash_scan(prefix_hash_token((uint32_t)mine)), ix.lookup_size, ix.lookup_fp_mask, &slot,
                           &fp);
        uint32_t cand = PPV_NO_SLOT;
        if (lane < tl) {
            for (uint32_t n = 0; n < ix.lookup_size; n++) {   // ends at the first empty slot (the table is half empty)
                const uint64_t e = ix.lookup[slot];
                if (e == 0ull) break;
                if ((uint32_t)(e >> 32) == fp) {
                    cand = (uint32_t)e;
                    break;
                }
                slot = slot + 1u == ix.lookup_size ? 0u : slot + 1u;
            }
        }
        const uint64_t hits = __ballot(cand != PPV_NO_SLOT);
        if (hits) {
            const int D = 63 - __clzll((long long)hits);   // deepest level with a hit: prefix length D + 1
            const uint32_t g = lane_value(cand, D);
            // everything that depends on g alone goes out together (the table holds valid nodes only), the rank
            // range included; the member's tokens wait for the depth check, which is what says they are there
            const uint32_t d0 = ix.depth_base[D + 1], d1 = ix.depth_base[D + 2];
            const NodeEnt e0 = ix.ent[g], e1 = ix.ent[g + 1];
            const uint32_t a = ix.node_xpos[g];
            const uint32_t g_lo = ix.node_lo[g], g_hi = ix.node_hi[g];
            if (g >= d0 && g < d1) {   // a node of depth D+1: its first member has D+1 tokens or more
                const bool same = lane > D || ix.x_tok[(size_t)a + lane] == mine;
                if (__ballot(!same) == 0ull) {
                    if (D + 1 == t) {   // the whole prefix: nothing left to descend
                        Walk w;
                        w.node = g;
                        w.cb = e0.child;
                        w.ce = e1.child;
                        w.tok = e0.tok;
                        w.lo = g_lo;
                        w.hi = g_hi;
                        w.found = true;
                        w.member = (e0.tok & PPV_NODE_TERMINAL) != 0u;
                        return w;
                    }
                    return walk_from(ix, prefix, t, lane, mine, D + 1, g, e0.tok, e0.child, e1.child);
                }
            }
        }
    }
    return walk_from(ix, prefix, t, lane, mine, 0, 0u, 0u, root_cb, root_ce);
}

__device__ inline uint32_t heavy_slot_of(const IndexView &ix, uint32_t node) {
    return node < ix.heavy_limit ? ix.heavy_slot[node] : PPV_NO_SLOT;
}

}  // namespace
