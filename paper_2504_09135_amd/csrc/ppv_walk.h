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

__device__ inline Walk walk_prefix(const IndexView &ix, const int32_t *__restrict__ prefix, int t, int lane) {
    Walk w;
    w.node = 0;
    w.cb = ix.ent[0].child;
    w.ce = ix.ent[1].child;
    w.tok = 0;
    w.found = true;
    w.member = false;
    // the first 64 tokens in one coalesced load; token i is broadcast from lane i
    const int32_t mine = (lane < t) ? prefix[lane] : 0;
    for (int i = 0; i < t; i++) {
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

__device__ inline uint32_t heavy_slot_of(const IndexView &ix, uint32_t node) {
    return node < ix.heavy_limit ? ix.heavy_slot[node] : PPV_NO_SLOT;
}

}  // namespace
