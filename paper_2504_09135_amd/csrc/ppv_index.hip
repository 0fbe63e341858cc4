// Index construction (Algorithm 2, "Prepare"; Section 3.2 "Array Preparation"), sizes, export, release.
#include <algorithm>
#include <new>
#include <vector>

#include "ppv_internal.h"

extern "C" const char *ppv_status_string(ppv_status s) {
    switch (s) {
        case PPV_OK: return "PPV_OK";
        case PPV_EINVAL: return "PPV_EINVAL: invalid argument";
        case PPV_ENOMEM: return "PPV_ENOMEM: out of memory";
        case PPV_EDEVICE: return "PPV_EDEVICE: HIP call failed";
        case PPV_ERANGE: return "PPV_ERANGE: size beyond what the library supports";
    }
    return "unknown ppv_status";
}

namespace {

template <typename T>
ppv_status upload(T **dst, const std::vector<T> &src, int64_t *bytes) {
    size_t n = src.size() * sizeof(T);
    PPV_HIP_TRY(hipMalloc((void **)dst, n ? n : sizeof(T)));
    if (n) PPV_HIP_TRY(hipMemcpy(*dst, src.data(), n, hipMemcpyHostToDevice));
    *bytes += (int64_t)(n ? n : sizeof(T));
    return PPV_OK;
}

ppv_status build_impl(const int32_t *tokens, const int64_t *offsets, int64_t n_seq, int32_t vocab, ppv_index *ix) {
    // ---- validate
    if (offsets[0] != 0) return PPV_EINVAL;
    for (int64_t i = 0; i < n_seq; i++)
        if (offsets[i + 1] <= offsets[i]) return PPV_EINVAL;  // empty sequence or decreasing offsets
    const int64_t total = offsets[n_seq];
    for (int64_t j = 0; j < total; j++)
        if (tokens[j] < 0 || tokens[j] >= vocab) return PPV_EINVAL;
    if (n_seq > 0xFFFFFFFEll) return PPV_ERANGE;

    // ---- sort row ids lexicographically (token order = integer order, prefix before extension)
    std::vector<int64_t> order((size_t)n_seq);
    for (int64_t i = 0; i < n_seq; i++) order[(size_t)i] = i;
    auto less = [&](int64_t a, int64_t b) {
        const int32_t *pa = tokens + offsets[a], *pb = tokens + offsets[b];
        int64_t la = offsets[a + 1] - offsets[a], lb = offsets[b + 1] - offsets[b];
        int64_t n = la < lb ? la : lb;
        for (int64_t k = 0; k < n; k++)
            if (pa[k] != pb[k]) return pa[k] < pb[k];
        return la < lb;
    };
    std::sort(order.begin(), order.end(), less);

    // ---- de-duplicate, flatten, longest common prefix with the previous row
    std::vector<int32_t> x_tok;
    std::vector<int64_t> x_off;
    std::vector<int32_t> lcp;  // lcp[r] = common prefix length of rows r-1 and r (0 for r = 0)
    x_tok.reserve((size_t)total);
    x_off.reserve((size_t)n_seq + 1);
    lcp.reserve((size_t)n_seq);
    x_off.push_back(0);
    int32_t l_max = 0;
    for (int64_t i = 0; i < n_seq; i++) {
        int64_t s = order[(size_t)i];
        const int32_t *p = tokens + offsets[s];
        int64_t len = offsets[s + 1] - offsets[s];
        int32_t c = 0;
        if (!lcp.empty() || x_off.size() > 1) {
            size_t r = x_off.size() - 2;
            const int32_t *q = x_tok.data() + x_off[r];
            int64_t ql = x_off[r + 1] - x_off[r];
            int64_t n = ql < len ? ql : len;
            while (c < n && p[c] == q[c]) c++;
            if (c == len && c == ql) continue;  // duplicate of the previous kept row
        }
        x_tok.insert(x_tok.end(), p, p + len);
        x_off.push_back((int64_t)x_tok.size());
        lcp.push_back(c);
        if (len > l_max) l_max = (int32_t)len;
    }
    const int64_t n_rows = (int64_t)x_off.size() - 1;

    // ---- per-depth arrays.  A row r opens a new prefix of length d+1 iff it is longer than d and
    // shares at most d tokens with the row before it; that prefix covers rows up to the next row
    // whose common prefix with its predecessor is at most d.
    std::vector<uint32_t> node_tok(1, 0u), node_lo(1, 0u), node_hi(1, (uint32_t)n_rows);
    std::vector<size_t> level_base((size_t)l_max + 2, 0);
    level_base[0] = 1;
    for (int32_t d = 0; d < l_max; d++) {
        size_t open = 0;
        bool have_open = false;
        for (int64_t r = 0; r < n_rows; r++) {
            if (lcp[(size_t)r] <= d || r == 0) {
                if (have_open) { node_hi[open] = (uint32_t)r; have_open = false; }
                if (x_off[(size_t)r + 1] - x_off[(size_t)r] > d) {
                    if (node_tok.size() >= 0xFFFFFFFEull) return PPV_ERANGE;
                    // the first row of a prefix's range is the prefix itself iff it ends at depth d
                    uint32_t term = (x_off[(size_t)r + 1] - x_off[(size_t)r] == d + 1) ? PPV_NODE_TERMINAL : 0u;
                    node_tok.push_back((uint32_t)x_tok[(size_t)(x_off[(size_t)r] + d)] | term);
                    node_lo.push_back((uint32_t)r);
                    node_hi.push_back(0u);
                    open = node_tok.size() - 1;
                    have_open = true;
                }
            }
        }
        if (have_open) node_hi[open] = (uint32_t)n_rows;
        level_base[(size_t)d + 1] = node_tok.size();
    }
    const size_t G = node_tok.size();
    // children of node g (depth d) = the nodes of depth d+1 whose first row lies in [lo, hi)
    std::vector<uint32_t> child_off(G + 1, 0u);
    {
        size_t lvl_begin = 0, lvl_end = 1;  // the level that holds node 0 alone
        for (int32_t d = 0; d <= l_max; d++) {  // d = depth of the children of the current level
            size_t cb = (d < l_max) ? level_base[(size_t)d] : G;
            size_t ce = (d < l_max) ? level_base[(size_t)d + 1] : G;
            size_t c = cb;
            for (size_t g = lvl_begin; g < lvl_end; g++) {
                child_off[g] = (uint32_t)c;
                while (c < ce && node_lo[c] < node_hi[g]) c++;
            }
            lvl_begin = cb;
            lvl_end = ce;
        }
        child_off[G] = (uint32_t)G;
    }

    // ---- heavy nodes: ready-made valid-set images and per-word child counts
    const int n_words = (vocab + 31) / 32;
    const uint32_t heavy_min = (uint32_t)std::min<int64_t>(vocab / 32, PPV_LIST_MAX);
    std::vector<uint32_t> heavy_slot, heavy_bits, heavy_rank;
    size_t n_heavy = 0;
    for (size_t g = 0; g < G; g++) {
        uint32_t cb = child_off[g], ce = child_off[g + 1];
        if (ce - cb <= heavy_min) continue;
        heavy_slot.resize(g + 1, PPV_NO_SLOT);
        heavy_slot[g] = (uint32_t)n_heavy;
        heavy_bits.resize((n_heavy + 1) * (size_t)n_words, 0u);
        heavy_rank.resize((n_heavy + 1) * (size_t)n_words, 0u);
        uint32_t *bits = heavy_bits.data() + n_heavy * (size_t)n_words;
        uint32_t *rank = heavy_rank.data() + n_heavy * (size_t)n_words;
        for (uint32_t c = cb; c < ce; c++) {
            uint32_t v = node_tok[c] & PPV_NODE_TOKEN;
            bits[v >> 5] |= 1u << (v & 31u);
        }
        uint32_t acc = 0;
        for (int w = 0; w < n_words; w++) {
            rank[w] = acc;
            acc += (uint32_t)__builtin_popcount(bits[w]);
        }
        n_heavy++;
    }

    // ---- upload
    ppv_status st;
    ix->device_bytes = 0;
    std::vector<NodeEnt> ent(G + 1);
    for (size_t g = 0; g <= G; g++) {
        ent[g].tok = g < G ? node_tok[g] : PPV_NODE_TOKEN;
        if (g < heavy_slot.size() && heavy_slot[g] != PPV_NO_SLOT) ent[g].tok |= PPV_NODE_HEAVY;
        ent[g].child = child_off[g];
    }
    if ((st = upload(&ix->d_ent, ent, &ix->device_bytes)) != PPV_OK) return st;
    if ((st = upload(&ix->d_node_lo, node_lo, &ix->device_bytes)) != PPV_OK) return st;
    if ((st = upload(&ix->d_node_hi, node_hi, &ix->device_bytes)) != PPV_OK) return st;
    if ((st = upload(&ix->d_heavy_slot, heavy_slot, &ix->device_bytes)) != PPV_OK) return st;
    if ((st = upload(&ix->d_heavy_bits, heavy_bits, &ix->device_bytes)) != PPV_OK) return st;
    if ((st = upload(&ix->d_heavy_rank, heavy_rank, &ix->device_bytes)) != PPV_OK) return st;
    if ((st = upload(&ix->d_x_tok, x_tok, &ix->device_bytes)) != PPV_OK) return st;
    if ((st = upload(&ix->d_x_off, x_off, &ix->device_bytes)) != PPV_OK) return st;
    ix->n_tokens = (int64_t)x_tok.size();
    ix->n_heavy = (int64_t)n_heavy;
    ix->view.ent = ix->d_ent;
    ix->view.node_lo = ix->d_node_lo;
    ix->view.node_hi = ix->d_node_hi;
    ix->view.heavy_slot = ix->d_heavy_slot;
    ix->view.heavy_bits = ix->d_heavy_bits;
    ix->view.heavy_rank = ix->d_heavy_rank;
    ix->view.heavy_limit = (uint32_t)heavy_slot.size();
    ix->view.heavy_min = heavy_min;
    ix->view.n_nodes = (uint32_t)G;
    ix->view.n_rows = (uint32_t)n_rows;
    ix->view.vocab = vocab;
    ix->view.n_words = n_words;
    ix->view.l_max = l_max;
    return PPV_OK;
}

void release(ppv_index *ix) {
    if (!ix) return;
    (void)hipFree(ix->d_ent);
    (void)hipFree(ix->d_node_lo);
    (void)hipFree(ix->d_node_hi);
    (void)hipFree(ix->d_heavy_slot);
    (void)hipFree(ix->d_heavy_bits);
    (void)hipFree(ix->d_heavy_rank);
    (void)hipFree(ix->d_x_tok);
    (void)hipFree(ix->d_x_off);
    delete ix;
}

}  // namespace

extern "C" ppv_status ppv_build_index(const int32_t *tokens, const int64_t *offsets, int64_t n_seq, int32_t vocab,
                                      ppv_index_t **out) {
    if (!out) return PPV_EINVAL;
    *out = nullptr;
    if (!tokens || !offsets || n_seq <= 0 || vocab <= 0) return PPV_EINVAL;
    if (vocab > PPV_MAX_VOCAB) return PPV_ERANGE;
    ppv_index *ix = new (std::nothrow) ppv_index();
    if (!ix) return PPV_ENOMEM;
    if (hipGetDevice(&ix->device) != hipSuccess) { delete ix; return PPV_EDEVICE; }
    ppv_status st;
    try {
        st = build_impl(tokens, offsets, n_seq, vocab, ix);
    } catch (const std::bad_alloc &) {
        st = PPV_ENOMEM;
    } catch (...) {
        st = PPV_EDEVICE;
    }
    if (st != PPV_OK) { release(ix); return st; }
    *out = ix;
    return PPV_OK;
}

extern "C" ppv_status ppv_index_info(const ppv_index_t *ix, int64_t *n_distinct, int32_t *l_max, int32_t *vocab,
                                     int64_t *n_prefixes, int64_t *device_bytes) {
    if (!ix) return PPV_EINVAL;
    if (n_distinct) *n_distinct = ix->view.n_rows;
    if (l_max) *l_max = ix->view.l_max;
    if (vocab) *vocab = ix->view.vocab;
    if (n_prefixes) *n_prefixes = (int64_t)ix->view.n_nodes - 1;
    if (device_bytes) *device_bytes = ix->device_bytes;
    return PPV_OK;
}

extern "C" ppv_status ppv_index_export(const ppv_index_t *ix, int32_t *tokens_out, int64_t *offsets_out,
                                       int64_t *n_tokens) {
    if (!ix) return PPV_EINVAL;
    if (n_tokens) *n_tokens = ix->n_tokens;
    if (tokens_out && ix->n_tokens)
        PPV_HIP_TRY(hipMemcpy(tokens_out, ix->d_x_tok, (size_t)ix->n_tokens * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (offsets_out)
        PPV_HIP_TRY(hipMemcpy(offsets_out, ix->d_x_off, ((size_t)ix->view.n_rows + 1) * sizeof(int64_t),
                              hipMemcpyDeviceToHost));
    return PPV_OK;
}

extern "C" void ppv_free_index(ppv_index_t *ix) { release(ix); }
