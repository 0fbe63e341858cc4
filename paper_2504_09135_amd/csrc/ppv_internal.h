// Internal definitions shared by the sources of libppv_hip.so (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ppv.h"

// Device view of the index.  The distinct non-empty prefixes of members ("nodes") are stored in
// breadth-first order: all prefixes of length 1 in sorted order, then all of length 2, ...
// Node 0 is the empty prefix.  Because each depth is sorted, the children of consecutive nodes
// are consecutive, so one offsets array describes all of them: the children of node g are the
// nodes ent[g].child .. ent[g+1].child, in increasing token order.  Token and child offset sit
// side by side, so the one load that searches (or lists) a node's children also brings each
// child's own children range.
//
// Nodes with more than `heavy_min` children ("heavy": the root and a few shallow prefixes) also
// carry their valid set as a ready-made V-bit image plus, per 32-bit word of it, the number of
// children before that word, so that a copy replaces the scatter and the child carrying a given
// token is found with two loads.
constexpr uint32_t PPV_NODE_TERMINAL = 0x80000000u;  // flag in NodeEnt::tok: the prefix itself is in S
constexpr uint32_t PPV_NODE_HEAVY = 0x40000000u;     // flag in NodeEnt::tok: the node has an image
constexpr uint32_t PPV_NODE_TOKEN = 0x3FFFFFFFu;
constexpr uint32_t PPV_NO_SLOT = 0xFFFFFFFFu;
constexpr int PPV_LIST_MAX = 1024;  // a valid set of at most this many tokens is handled as a list

struct NodeEnt {
    uint32_t tok;    // last token of the prefix | flags
    uint32_t child;  // first child; the children end where the next entry's children begin
};

struct IndexView {
    const NodeEnt *ent;          // [n_nodes+1] (the last entry is a sentinel that closes the offsets)
    const uint32_t *node_lo;     // [n_nodes]   rank of the first member the prefix is a prefix of
    const uint32_t *node_hi;     // [n_nodes]   one past the rank of the last such member
    const uint32_t *heavy_slot;  // [heavy_limit] slot of a heavy node, PPV_NO_SLOT otherwise
    const uint32_t *heavy_bits;  // [n_heavy, n_words] valid-set images
    const uint32_t *heavy_rank;  // [n_heavy, n_words] children before each word
    // Hashed look-up of whole prefixes (all lengths of a query are probed at once instead of one level after
    // the other): open addressing, 8 bytes per slot = fingerprint << 32 | node, 0 = empty; lookup_size == 0:
    // no table.  A hit is only a hint: it is checked against the node's depth and the tokens of its first member.
    const uint64_t *lookup;      // [lookup_size]
    const uint32_t *depth_base;  // [l_max + 2] nodes of depth d are depth_base[d] .. depth_base[d+1]
    const uint32_t *node_xpos;   // [n_nodes] where the first member under the node starts in x_tok (with a table only)
    const int32_t *x_tok;        // sorted S, flat: row r is x_tok[x_off[r] .. x_off[r+1])
    const int64_t *x_off;        // [n_rows + 1]
    uint32_t lookup_size;
    uint32_t lookup_fp_mask;     // fingerprint bits in use (all of them; 0 in a test mode that makes every probe a false hit)
    uint32_t heavy_limit;        // nodes >= heavy_limit are not heavy
    uint32_t heavy_min;          // a node is heavy iff it has more than heavy_min children
    uint32_t n_heavy;            // heavy nodes, i.e. rows of heavy_bits / heavy_rank
    uint32_t n_nodes;            // including node 0
    uint32_t n_rows;             // |S| after de-duplication
    int32_t vocab;
    int32_t n_words;             // ceil(vocab / 32)
    int32_t l_max;
};

// A row spread over several workgroups (small batches: fewer rows than compute units).  Every workgroup reduces
// its share of the row's tiles and of the listed tokens and leaves the per-tile / per-slice statistics here; the
// workgroup that arrives last (one device-scope counter per row) reads them all back and finishes the row exactly
// as a single workgroup would: the statistics do not depend on who computed them, so results are bit for bit
// those of an unsplit row.  The counter is returned to zero by the workgroup that finishes the row.
constexpr int PPV_MAX_TILES = 256;          // PPV_MAX_VOCAB / 1024 (fp32 tiles are 1024 tokens)
constexpr int PPV_SPLIT_MAX_ROWS = PPV_NOALLOC_MAX_ROWS;   // larger batches fill the chip with one workgroup per row
constexpr int PPV_SPLIT_MAX_PARTS = 16;
struct SplitRow {
    float4 tile[PPV_MAX_TILES];             // (reference, sum over all tokens, sum over valid tokens, its reference)
    float list_e[PPV_LIST_MAX];
    float slice_m[PPV_LIST_MAX / 64], slice_z[PPV_LIST_MAX / 64];
};
struct SplitScratch {
    uint32_t arrivals[PPV_SPLIT_MAX_ROWS];
    SplitRow row[PPV_SPLIT_MAX_ROWS];
};
// The scratch area of (current device, stream), allocated at the first call that needs one; nullptr when it
// cannot be had (the stream is being captured and has none yet, or out of memory): the row is then not split.
SplitScratch *ppv_split_scratch(hipStream_t stream);

// Per-row decoding cursor kept between decode steps (PPV_STATE_WORDS x uint32).  The second half looks one level
// ahead: the entry of the node's first child and the child offset of the entry after it.  For a node with exactly
// one child -- nearly every node below the first few levels of a set of long sequences -- that is the whole valid
// set and the child's own children range, so a decode step on such a node needs no load from the index before it
// can ask for the listed token's logit.  `flags` says whether that half is filled in; it is a cache, never required.
struct RowState {
    uint32_t node;   // entry of the row's current prefix; PPV_NO_SLOT: not a prefix of any member
    uint32_t cb, ce; // its children
    uint32_t slot;   // heavy slot or PPV_NO_SLOT
    uint32_t tok0;   // ent[cb].tok   (token | flags of the first child)      -- when flags == 1
    uint32_t child0; // ent[cb].child (where the first child's children begin)
    uint32_t child1; // ent[cb + 1].child (where they end, if the node has one child)
    uint32_t flags;  // 1: tok0 / child0 / child1 are filled in; anything else: they are not
};
static_assert(sizeof(RowState) == PPV_STATE_WORDS * sizeof(uint32_t), "state layout");

struct ppv_index {
    IndexView view;
    NodeEnt *d_ent;
    uint32_t *d_node_lo, *d_node_hi;
    uint32_t *d_heavy_slot, *d_heavy_bits, *d_heavy_rank;
    uint64_t *d_lookup;
    uint32_t *d_depth_base, *d_node_xpos;
    int32_t *d_x_tok;    // sorted S, flat, no padding: row r is d_x_tok[d_x_off[r] .. d_x_off[r+1])
    int64_t *d_x_off;    // [n_rows + 1]
    int64_t n_tokens;
    int64_t n_heavy;
    int64_t device_bytes;
    int device;
};

// Current value of a tuning / test switch (PPV_TUNE_* of ppv.h): read from the environment once at load,
// changed by ppv_tuning_set.
int ppv_tuning(int knob);

#define PPV_HIP_TRY(expr)                          \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) {                    \
            (void)hipGetLastError();               \
            return (e_ == hipErrorOutOfMemory) ? PPV_ENOMEM : PPV_EDEVICE; \
        }                                          \
    } while (0)
