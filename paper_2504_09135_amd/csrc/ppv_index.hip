// Index construction on the device (Algorithm 2, "Prepare"; Section 3.2 "Array Preparation"),
// plus sizes, export and release.
//
// The host hands over S as CSR; everything else runs in kernels:
//   1. validate (no empty sequence, tokens inside [0, V));
//   2. sort the rows lexicographically -- token order = integer order, left to right, a sequence
//      that ends sorts before its extensions -- by a least-significant-digit radix sort over the
//      columns from the last to the first (key of a row at column d: token + 1, or 0 past its end),
//      8 bits per pass, each pass a stable counting sort (histogram / scan / scatter);
//   3. longest common prefix of neighbouring sorted rows; duplicates dropped (S is a set);
//   4. the per-depth arrays: row r opens a new prefix of length d+1 iff it is longer than d and
//      shares at most d tokens with the row before it.  One exclusive scan over the depth-major
//      flags (depth, row) numbers all prefixes in breadth-first order and, because every depth is
//      sorted, gives each prefix its first child for free;
//   5. rank ranges: lo = the opening row; hi bottom-up, deepest level first (a prefix ends where
//      its last child ends, or one row after it opens if it has no child);
//   6. images and per-word child counts of the heavy prefixes.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>

#include <cstdlib>

#include "ppv_device.h"
#include "ppv_internal.h"
#include "ppv_walk.h"

extern "C" const char *ppv_status_string(ppv_status s) {
    switch (s) {
        case PPV_OK: return "PPV_OK";
        case PPV_EINVAL: return "PPV_EINVAL: invalid argument";
        case PPV_ENOMEM: return "PPV_ENOMEM: out of memory";
        case PPV_EDEVICE: return "PPV_EDEVICE: HIP call failed";
        case PPV_ERANGE: return "PPV_ERANGE: size beyond what the library supports";
        case PPV_EIO: return "PPV_EIO: file could not be opened, read or written";
    }
    return "unknown ppv_status";
}

namespace {

constexpr int BT = 256;            // threads per workgroup of the build kernels
constexpr int SCAN_ITEMS = 8;      // consecutive items per thread in the scans
constexpr int SCAN_CHUNK = BT * SCAN_ITEMS;
constexpr int SORT_TILES = 16;     // tiles of BT rows per workgroup in a radix pass
constexpr int SORT_CHUNK = BT * SORT_TILES;
constexpr int RADIX = 256;
static_assert(RADIX == BT, "one thread per digit in the radix kernels");

// ------------------------------------------------------------------------------------------
// Exclusive scan of f(0..n-1) (uint32 sums; the callers keep totals below 2^32).
// Three launches: per-chunk sums, scan of the chunk sums by one workgroup, per-chunk scan + base.
__device__ inline uint32_t block_exclusive_scan(uint32_t x, uint32_t *wave_tot, uint32_t *block_total) {
    // exclusive prefix of x over the workgroup's BT threads in thread order
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    const uint32_t incl = wave_incl_scan(x);
    if (lane == WAVE - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
    for (int w = 0; w < BT / WAVE; w++) {
        const uint32_t t = wave_tot[w];
        if (w < wave) before += t;
        total += t;
    }
    __syncthreads();
    *block_total = total;
    return before + incl - x;
}

template <typename F> __global__ __launch_bounds__(BT) void scan_chunk_sums(uint64_t n, F f, uint32_t *__restrict__ sums) {
    __shared__ uint32_t wave_tot[BT / WAVE];
    const uint64_t base = (uint64_t)blockIdx.x * SCAN_CHUNK + (uint64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t s = 0;
    for (int k = 0; k < SCAN_ITEMS; k++)
        if (base + k < n) s += f(base + k);
    s = wave_sum(s);
    if ((threadIdx.x & (WAVE - 1)) == 0) wave_tot[threadIdx.x / WAVE] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = 0;
        for (int w = 0; w < BT / WAVE; w++) t += wave_tot[w];
        sums[blockIdx.x] = t;
    }
}

// in place exclusive scan of m values by ONE workgroup; the grand total goes to *total
__global__ __launch_bounds__(BT) void scan_of_sums(uint32_t *__restrict__ sums, uint64_t m, uint32_t *__restrict__ total) {
    __shared__ uint32_t wave_tot[BT / WAVE];
    uint32_t carry = 0;
    for (uint64_t b0 = 0; b0 < m; b0 += SCAN_CHUNK) {
        const uint64_t base = b0 + (uint64_t)threadIdx.x * SCAN_ITEMS;
        uint32_t v[SCAN_ITEMS], s = 0;
        for (int k = 0; k < SCAN_ITEMS; k++) {
            v[k] = (base + k < m) ? sums[base + k] : 0u;
            s += v[k];
        }
        uint32_t tot;
        uint32_t ex = carry + block_exclusive_scan(s, wave_tot, &tot);
        for (int k = 0; k < SCAN_ITEMS; k++) {
            if (base + k < m) sums[base + k] = ex;
            ex += v[k];
        }
        carry += tot;
    }
    if (threadIdx.x == 0) *total = carry;
}

template <typename F>
__global__ __launch_bounds__(BT) void scan_apply(uint64_t n, F f, const uint32_t *__restrict__ sums, uint32_t *out) {
    __shared__ uint32_t wave_tot[BT / WAVE];
    const uint64_t base = (uint64_t)blockIdx.x * SCAN_CHUNK + (uint64_t)threadIdx.x * SCAN_ITEMS;
    uint32_t v[SCAN_ITEMS], s = 0;
    for (int k = 0; k < SCAN_ITEMS; k++) {
        v[k] = (base + k < n) ? f(base + k) : 0u;
        s += v[k];
    }
    uint32_t tot;
    uint32_t ex = sums[blockIdx.x] + block_exclusive_scan(s, wave_tot, &tot);
    for (int k = 0; k < SCAN_ITEMS; k++) {
        if (base + k < n) out[base + k] = ex;
        ex += v[k];
    }
}

// out[i] = sum of f(0..i-1) for i in [0, n); *d_total = sum of all.  sums: scratch of ceil(n / SCAN_CHUNK) words.
// f may read `out` only at the index it is asked for (the in-place scan of the radix histogram does).
template <typename F>
ppv_status exclusive_scan(uint64_t n, F f, uint32_t *out, uint32_t *sums, uint32_t *d_total, hipStream_t st) {
    const uint64_t nb = (n + SCAN_CHUNK - 1) / SCAN_CHUNK;
    if (nb == 0) {
        hipLaunchKernelGGL(scan_of_sums, dim3(1), dim3(BT), 0, st, sums, (uint64_t)0, d_total);  // total = 0
        PPV_HIP_TRY(hipGetLastError());
        return PPV_OK;
    }
    hipLaunchKernelGGL(scan_chunk_sums<F>, dim3((unsigned)nb), dim3(BT), 0, st, n, f, sums);
    hipLaunchKernelGGL(scan_of_sums, dim3(1), dim3(BT), 0, st, sums, nb, d_total);
    hipLaunchKernelGGL(scan_apply<F>, dim3((unsigned)nb), dim3(BT), 0, st, n, f, (const uint32_t *)sums, out);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}

// ------------------------------------------------------------------------------------------
// 1. validation and the longest row
__global__ __launch_bounds__(BT) void check_rows(const int64_t *__restrict__ off, int64_t n, int32_t *__restrict__ err,
                                                 int32_t *__restrict__ l_max) {
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    int32_t len = 0;
    if (i < n) {
        const int64_t l = off[i + 1] - off[i];
        if (l <= 0 || l > 0x7FFFFFFF) atomicOr(err, 1);
        else len = (int32_t)l;
    }
    for (int o = WAVE / 2; o > 0; o >>= 1) len = max(len, __shfl_xor(len, o, WAVE));
    if ((threadIdx.x & (WAVE - 1)) == 0 && len > 0) atomicMax(l_max, len);   // one atomic per wave
}
__global__ __launch_bounds__(BT) void check_tokens(const int32_t *__restrict__ tok, int64_t total, int32_t vocab,
                                                   int32_t *__restrict__ err) {
    const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    if (i < total && (tok[i] < 0 || tok[i] >= vocab)) atomicOr(err, 2);
}
__global__ __launch_bounds__(BT) void iota_rows(uint32_t *__restrict__ perm, uint32_t n) {
    const uint32_t i = blockIdx.x * BT + threadIdx.x;
    if (i < n) perm[i] = i;
}

// ------------------------------------------------------------------------------------------
// 2. one stable counting-sort pass on 8 bits of the column key
__device__ inline uint32_t column_key(const int32_t *__restrict__ tok, const int64_t *__restrict__ off, uint32_t row,
                                      int col) {
    const int64_t a = off[row], b = off[row + 1];
    return (col < b - a) ? (uint32_t)tok[a + col] + 1u : 0u;  // 0: the row has ended; sorts first
}

__global__ __launch_bounds__(BT) void radix_histogram(const int32_t *__restrict__ tok, const int64_t *__restrict__ off,
                                                      const uint32_t *__restrict__ perm, uint32_t n, int col, int shift,
                                                      uint8_t *__restrict__ digits, uint32_t *__restrict__ hist,
                                                      uint32_t n_blocks) {
    __shared__ uint32_t h[RADIX];
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t start = blockIdx.x * SORT_CHUNK;
    for (int t = 0; t < SORT_TILES; t++) {
        const uint32_t i = start + t * BT + threadIdx.x;
        if (i < n) {
            const uint32_t d = (column_key(tok, off, perm[i], col) >> shift) & (RADIX - 1);
            digits[i] = (uint8_t)d;
            atomicAdd(&h[d], 1u);
        }
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * n_blocks + blockIdx.x] = h[threadIdx.x];  // digit-major for the scan
}

__global__ __launch_bounds__(BT) void radix_scatter(const uint32_t *__restrict__ perm_in, uint32_t n,
                                                    const uint8_t *__restrict__ digits,
                                                    const uint32_t *__restrict__ hist_scanned, uint32_t n_blocks,
                                                    uint32_t *__restrict__ perm_out) {
    __shared__ uint32_t base[RADIX];               // next free slot per digit for this workgroup
    __shared__ uint32_t cnt[BT / WAVE][RADIX];     // rows per digit in the current tile, per wave
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    base[threadIdx.x] = hist_scanned[(size_t)threadIdx.x * n_blocks + blockIdx.x];
    const uint32_t start = blockIdx.x * SORT_CHUNK;
    for (int t = 0; t < SORT_TILES; t++) {
        for (int w = 0; w < BT / WAVE; w++) cnt[w][threadIdx.x] = 0;
        __syncthreads();
        const uint32_t i = start + t * BT + threadIdx.x;
        const bool valid = i < n;
        const uint32_t d = valid ? digits[i] : 0u;
        // lanes of this wave that hold the same digit
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < 8; b++) {
            const uint64_t bal = __ballot(valid && ((d >> b) & 1u));
            peers &= ((d >> b) & 1u) ? bal : ~bal;
        }
        const uint32_t rank_in_wave = (uint32_t)__popcll(peers & ((1ull << lane) - 1ull));
        if (valid && rank_in_wave == 0) cnt[wave][d] = (uint32_t)__popcll(peers);
        __syncthreads();
        if (valid) {
            uint32_t pos = base[d] + rank_in_wave;
            for (int w = 0; w < wave; w++) pos += cnt[w][d];
            perm_out[pos] = perm_in[i];            // stable: thread order within the tile is kept
        }
        __syncthreads();
        uint32_t add = 0;
        for (int w = 0; w < BT / WAVE; w++) add += cnt[w][threadIdx.x];
        base[threadIdx.x] += add;
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// 3. common prefix with the previous sorted row; duplicates
__global__ __launch_bounds__(BT) void neighbour_lcp(const int32_t *__restrict__ tok, const int64_t *__restrict__ off,
                                                    const uint32_t *__restrict__ perm, uint32_t n,
                                                    int32_t *__restrict__ lcp, uint8_t *__restrict__ keep) {
    const uint32_t i = blockIdx.x * BT + threadIdx.x;
    if (i >= n) return;
    if (i == 0) { lcp[0] = 0; keep[0] = 1; return; }
    const uint32_t r = perm[i], q = perm[i - 1];
    const int32_t *a = tok + off[r], *b = tok + off[q];
    const int32_t la = (int32_t)(off[r + 1] - off[r]), lb = (int32_t)(off[q + 1] - off[q]);
    const int32_t m = la < lb ? la : lb;
    int32_t c = 0;
    while (c < m && a[c] == b[c]) c++;
    lcp[i] = c;
    keep[i] = (c == la && c == lb) ? 0 : 1;
}
struct HistValue {
    const uint32_t *h;
    __device__ uint32_t operator()(uint64_t i) const { return h[i]; }
};
struct KeepFlag {
    const uint8_t *keep;
    __device__ uint32_t operator()(uint64_t i) const { return keep[i]; }
};
struct KeptLen {  // length of sorted row i if it is kept, else 0
    const uint8_t *keep;
    const uint32_t *perm;
    const int64_t *off;
    __device__ uint32_t operator()(uint64_t i) const {
        if (!keep[i]) return 0u;
        const uint32_t r = perm[i];
        return (uint32_t)(off[r + 1] - off[r]);
    }
};
// kept sorted row i becomes row dst[i] of the index: its tokens, offset, common prefix
__global__ __launch_bounds__(BT) void compact_rows(const int32_t *__restrict__ tok, const int64_t *__restrict__ off,
                                                   const uint32_t *__restrict__ perm, uint32_t n,
                                                   const uint8_t *__restrict__ keep, const uint32_t *__restrict__ dst,
                                                   const uint32_t *__restrict__ tok_at, const int32_t *__restrict__ lcp,
                                                   int32_t *__restrict__ x_tok, int64_t *__restrict__ x_off,
                                                   int32_t *__restrict__ row_lcp, uint32_t n_rows, uint32_t n_tok) {
    const uint32_t i = blockIdx.x * BT + threadIdx.x;
    if (i == 0) x_off[n_rows] = n_tok;
    if (i >= n || !keep[i]) return;
    const uint32_t r = perm[i], d = dst[i], at = tok_at[i];
    const int64_t a = off[r];
    const int32_t len = (int32_t)(off[r + 1] - a);
    x_off[d] = at;
    row_lcp[d] = lcp[i];
    for (int32_t k = 0; k < len; k++) x_tok[at + k] = tok[a + k];
}

// ------------------------------------------------------------------------------------------
// 4. per-depth arrays.  Flattened depth-major index k = d * N + r.
struct OpensPrefix {  // 1 iff row r opens a new prefix of length d+1
    const int64_t *x_off;
    const int32_t *row_lcp;
    uint64_t n_rows;
    __device__ uint32_t operator()(uint64_t k) const {
        const uint64_t d = k / n_rows, r = k - d * n_rows;
        const int64_t len = x_off[r + 1] - x_off[r];
        return (len > (int64_t)d && row_lcp[r] <= (int32_t)d) ? 1u : 0u;
    }
};
// pos[k] = prefixes numbered before (d, r); a prefix's number + 1 is its entry (entry 0 = the empty prefix)
__global__ __launch_bounds__(BT) void fill_nodes(const int32_t *__restrict__ x_tok, const int64_t *__restrict__ x_off,
                                                 const int32_t *__restrict__ row_lcp, const uint32_t *__restrict__ pos,
                                                 uint64_t n_rows, int32_t l_max, uint32_t n_nodes,
                                                 NodeEnt *__restrict__ ent, uint32_t *__restrict__ node_lo) {
    const uint64_t k = (uint64_t)blockIdx.x * BT + threadIdx.x;
    if (k == 0) {  // the empty prefix and the closing sentinel
        ent[0].tok = 0u;
        ent[0].child = 1u;
        node_lo[0] = 0u;
        ent[n_nodes].tok = PPV_NODE_TOKEN;
        ent[n_nodes].child = n_nodes;
    }
    if (k >= n_rows * (uint64_t)l_max) return;
    const uint64_t d = k / n_rows, r = k - d * n_rows;
    const int64_t a = x_off[r];
    const int64_t len = x_off[r + 1] - a;
    if (!(len > (int64_t)d && row_lcp[r] <= (int32_t)d)) return;
    const uint32_t g = 1u + pos[k];
    uint32_t t = (uint32_t)x_tok[a + d];
    if (len == (int64_t)d + 1) t |= PPV_NODE_TERMINAL;  // the opening row is the prefix itself
    // first child: the first prefix of length d+2 at or after this row (this row itself if it goes on,
    // else the next row); depth-major numbering makes that a plain look-up of the scan
    uint32_t child = n_nodes;
    if (d + 1 < (uint64_t)l_max) {
        const uint64_t first = (len > (int64_t)d + 1) ? r : r + 1;   // first == n_rows: start of the next depth
        child = 1u + pos[(d + 1) * n_rows + first];
    }
    ent[g].tok = t;
    ent[g].child = child;
    node_lo[g] = (uint32_t)r;
}

// 5. hi of the entries [g0, g1) of one depth, deeper levels already done
__global__ __launch_bounds__(BT) void fill_hi(const NodeEnt *__restrict__ ent, const uint32_t *__restrict__ node_lo,
                                              uint32_t g0, uint32_t g1, uint32_t *__restrict__ node_hi) {
    const uint32_t g = g0 + blockIdx.x * BT + threadIdx.x;
    if (g >= g1) return;
    const uint32_t cb = ent[g].child, ce = ent[g + 1].child;
    node_hi[g] = (ce > cb) ? node_hi[ce - 1] : node_lo[g] + 1u;
}

// 6. heavy prefixes
struct IsHeavy {
    const NodeEnt *ent;
    uint32_t heavy_min;
    __device__ uint32_t operator()(uint64_t g) const { return (ent[g + 1].child - ent[g].child > heavy_min) ? 1u : 0u; }
};
__global__ __launch_bounds__(BT) void mark_heavy(NodeEnt *__restrict__ ent, uint32_t n_nodes, uint32_t heavy_min,
                                                 const uint32_t *__restrict__ slot_of, uint32_t heavy_limit,
                                                 uint32_t *__restrict__ heavy_slot, uint32_t *__restrict__ heavy_node) {
    const uint32_t g = blockIdx.x * BT + threadIdx.x;
    if (g >= n_nodes) return;
    const bool heavy = ent[g + 1].child - ent[g].child > heavy_min;
    if (g < heavy_limit) heavy_slot[g] = heavy ? slot_of[g] : PPV_NO_SLOT;
    if (heavy) {
        heavy_node[slot_of[g]] = g;
        atomicOr(&ent[g].tok, PPV_NODE_HEAVY);
    }
}
// one workgroup per heavy prefix: OR its children into the image, then count children before each word
__global__ __launch_bounds__(BT) void fill_heavy(const NodeEnt *__restrict__ ent, const uint32_t *__restrict__ heavy_node,
                                                 int n_words, uint32_t *__restrict__ bits, uint32_t *__restrict__ rank) {
    __shared__ uint32_t wave_tot[BT / WAVE];
    const uint32_t g = heavy_node[blockIdx.x];
    uint32_t *b = bits + (size_t)blockIdx.x * (size_t)n_words;
    uint32_t *rk = rank + (size_t)blockIdx.x * (size_t)n_words;
    for (uint32_t c = ent[g].child + threadIdx.x; c < ent[g + 1].child; c += BT) {
        const uint32_t v = ent[c].tok & PPV_NODE_TOKEN;
        atomicOr(&b[v >> 5], 1u << (v & 31u));   // the image was zeroed before the launch
    }
    __threadfence();
    __syncthreads();
    uint32_t carry = 0;
    for (int w0 = 0; w0 < n_words; w0 += BT) {
        const int w = w0 + threadIdx.x;
        const uint32_t c = (w < n_words) ? (uint32_t)__popc(__builtin_nontemporal_load(&b[w])) : 0u;
        uint32_t tot;
        const uint32_t ex = carry + block_exclusive_scan(c, wave_tot, &tot);
        if (w < n_words) rk[w] = ex;
        carry += tot;
    }
}

// ------------------------------------------------------------------------------------------
struct DeviceBuffers {  // temporaries of the build, all released at the end
    void *p[24];
    int n = 0;
    ~DeviceBuffers() {
        for (int i = 0; i < n; i++) (void)hipFree(p[i]);
    }
    template <typename T> ppv_status alloc(T **out, size_t count) {
        *out = nullptr;
        if (n >= 24) return PPV_EDEVICE;
        hipError_t e = hipMalloc((void **)out, (count ? count : 1) * sizeof(T));
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return e == hipErrorOutOfMemory ? PPV_ENOMEM : PPV_EDEVICE;
        }
        p[n++] = *out;
        return PPV_OK;
    }
};

template <typename T> ppv_status keep_alloc(T **out, size_t count, int64_t *bytes) {
    *out = nullptr;
    hipError_t e = hipMalloc((void **)out, (count ? count : 1) * sizeof(T));
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? PPV_ENOMEM : PPV_EDEVICE;
    }
    *bytes += (int64_t)((count ? count : 1) * sizeof(T));
    return PPV_OK;
}

#define TRY(x)                          \
    do {                                \
        ppv_status s_ = (x);            \
        if (s_ != PPV_OK) return s_;    \
    } while (0)

inline unsigned blocks_for(uint64_t n) { return (unsigned)((n + BT - 1) / BT); }

// 6. Images and per-word child counts of the heavy prefixes, from the finished entries (G of them plus the
// sentinel).  Sets the heavy part of the index and of its view.
ppv_status finish_heavy(ppv_index *ix, uint32_t G, int32_t vocab, hipStream_t st) {
    DeviceBuffers tmp;
    const int n_words = (vocab + 31) / 32;
    const uint32_t heavy_min = (uint32_t)std::min<int64_t>(vocab / 32, PPV_LIST_MAX);
    uint32_t *slot_of, *sums, *d_total;
    TRY(tmp.alloc(&slot_of, G));
    TRY(tmp.alloc(&sums, (size_t)(((uint64_t)G + SCAN_CHUNK - 1) / SCAN_CHUNK)));
    TRY(tmp.alloc(&d_total, 1));
    TRY(exclusive_scan(G, IsHeavy{ix->d_ent, heavy_min}, slot_of, sums, d_total, st));
    uint32_t n_heavy;
    PPV_HIP_TRY(hipMemcpyAsync(&n_heavy, d_total, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    PPV_HIP_TRY(hipStreamSynchronize(st));
    // Breadth-first order puts the heavy prefixes (shallow ones) at small entry numbers, so the slot
    // table only has to reach past the last of them: the first entry that has all n_heavy before it.
    uint32_t heavy_limit = 0;
    if (n_heavy > 0) {
        uint32_t lo = 0, hi = G;
        while (lo < hi) {
            const uint32_t mid = lo + (hi - lo) / 2;
            uint32_t v;
            PPV_HIP_TRY(hipMemcpy(&v, slot_of + mid, sizeof(uint32_t), hipMemcpyDeviceToHost));
            if (v >= n_heavy) hi = mid; else lo = mid + 1;
        }
        heavy_limit = lo;
    }
    uint32_t *heavy_node;
    TRY(tmp.alloc(&heavy_node, n_heavy));
    TRY(keep_alloc(&ix->d_heavy_slot, heavy_limit, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_heavy_bits, (size_t)n_heavy * n_words, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_heavy_rank, (size_t)n_heavy * n_words, &ix->device_bytes));
    PPV_HIP_TRY(hipMemsetAsync(ix->d_heavy_bits, 0, std::max<size_t>((size_t)n_heavy * n_words, 1) * sizeof(uint32_t), st));
    hipLaunchKernelGGL(mark_heavy, dim3(blocks_for(G)), dim3(BT), 0, st, ix->d_ent, G, heavy_min,
                       (const uint32_t *)slot_of, heavy_limit, ix->d_heavy_slot, heavy_node);
    if (n_heavy > 0)
        hipLaunchKernelGGL(fill_heavy, dim3(n_heavy), dim3(BT), 0, st, (const NodeEnt *)ix->d_ent,
                           (const uint32_t *)heavy_node, n_words, ix->d_heavy_bits, ix->d_heavy_rank);
    PPV_HIP_TRY(hipGetLastError());
    PPV_HIP_TRY(hipStreamSynchronize(st));
    ix->n_heavy = n_heavy;
    ix->view.heavy_slot = ix->d_heavy_slot;
    ix->view.heavy_bits = ix->d_heavy_bits;
    ix->view.heavy_rank = ix->d_heavy_rank;
    ix->view.heavy_limit = heavy_limit;
    ix->view.n_heavy = n_heavy;
    ix->view.heavy_min = heavy_min;
    ix->view.n_words = n_words;
    return PPV_OK;
}

// Nodes of depth d are h_base[d] .. h_base[d+1] (h_base has l_max + 2 entries): depth 0 is the empty prefix, and
// the nodes of depth d+1 start where the children of the first node of depth d start.  Reads one child offset
// per depth from the finished entries.
ppv_status depth_bases(const ppv_index *ix, uint32_t G, int32_t l_max, uint32_t *h_base) {
    h_base[0] = 0u;
    h_base[1] = 1u;
    for (int d = 1; d < l_max; d++) {
        if (h_base[d] >= G) {
            h_base[d + 1] = G;
            continue;
        }
        PPV_HIP_TRY(hipMemcpy(&h_base[d + 1], &ix->d_ent[h_base[d]].child, sizeof(uint32_t), hipMemcpyDeviceToHost));
        if (h_base[d + 1] < h_base[d] || h_base[d + 1] > G) return PPV_EINVAL;
    }
    h_base[l_max + 1] = G;
    return PPV_OK;
}

// 7. Look-up table of whole prefixes: every node is entered under the hash of its token string (the first
// tokens of the first member under it).  Also the per-depth node ranges the look-up checks a hit against.
__global__ __launch_bounds__(BT) void insert_nodes(const uint32_t *__restrict__ node_lo, const int32_t *__restrict__ x_tok,
                                                   const int64_t *__restrict__ x_off,
                                                   const uint32_t *__restrict__ depth_base, int32_t l_max,
                                                   uint32_t n_nodes, uint64_t *__restrict__ table, uint32_t size,
                                                   uint32_t fp_mask, int32_t *__restrict__ err) {
    const uint32_t g = 1u + blockIdx.x * BT + threadIdx.x;   // node 0 is the empty prefix: not looked up
    if (g >= n_nodes) return;
    int lo = 1, hi = l_max;                                   // depth d with depth_base[d] <= g < depth_base[d+1]
    while (lo < hi) {
        const int mid = (lo + hi + 1) / 2;
        if (depth_base[mid] <= g) lo = mid; else hi = mid - 1;
    }
    const uint32_t r = node_lo[g];
    const int64_t a = x_off[r];
    if (x_off[r + 1] - a < lo) {   // (a loaded file) the first member under a node is at least as long as the node is deep
        atomicOr(err, 4);
        return;
    }
    PrefixHash h = prefix_hash_token((uint32_t)x_tok[a]);   // a node is at least one token deep
    for (int i = 1; i < lo; i++) h = prefix_hash_join(h, prefix_hash_token((uint32_t)x_tok[a + i]));
    uint32_t slot, fp;
    prefix_hash_finish(h, size, fp_mask, &slot, &fp);
    const unsigned long long entry = ((unsigned long long)fp << 32) | g;
    for (uint32_t n = 0; n < size; n++) {   // the table has twice as many slots as nodes
        if (atomicCAS((unsigned long long *)&table[slot], 0ull, entry) == 0ull) return;
        slot = slot + 1u == size ? 0u : slot + 1u;
    }
}

__global__ __launch_bounds__(BT) void fill_xpos(const uint32_t *__restrict__ node_lo, const int64_t *__restrict__ x_off,
                                                uint32_t n_nodes, uint32_t *__restrict__ xpos) {
    const uint32_t g = blockIdx.x * BT + threadIdx.x;
    if (g < n_nodes) xpos[g] = (uint32_t)x_off[node_lo[g]];
}

ppv_status finish_lookup(ppv_index *ix, uint32_t G, int32_t l_max, hipStream_t st) {
    uint32_t *h_base = new (std::nothrow) uint32_t[(size_t)l_max + 2];
    if (!h_base) return PPV_ENOMEM;
    ppv_status rc = depth_bases(ix, G, l_max, h_base);
    if (rc == PPV_OK) rc = keep_alloc(&ix->d_depth_base, (size_t)l_max + 2, &ix->device_bytes);
    if (rc == PPV_OK && hipMemcpy(ix->d_depth_base, h_base, ((size_t)l_max + 2) * sizeof(uint32_t), hipMemcpyHostToDevice) !=
                            hipSuccess) {
        (void)hipGetLastError();
        rc = PPV_EDEVICE;
    }
    delete[] h_base;
    if (rc != PPV_OK) return rc;
    ix->view.depth_base = ix->d_depth_base;
    ix->view.x_tok = ix->d_x_tok;
    ix->view.x_off = ix->d_x_off;
    ix->view.lookup = nullptr;
    ix->view.lookup_size = 0;
    ix->view.lookup_fp_mask = 0xFFFFFFFFu;
    // PPV_TUNE_LOOKUP = 0: no table (every prefix is located by the descent; saves 16 bytes per prefix of device memory).
    // PPV_TUNE_LOOKUP_WEAK = 1 (tests): one fingerprint for all, so that every probe is a false hit and the exact check
    // has to turn it away.
    if (ppv_tuning(PPV_TUNE_LOOKUP) == 0) return PPV_OK;
    if (ppv_tuning(PPV_TUNE_LOOKUP_WEAK) == 1) ix->view.lookup_fp_mask = 0u;
    const uint64_t want = 2ull * G;
    const uint32_t size = (uint32_t)std::min<uint64_t>(want, 0xFFFFFFF0ull);
    DeviceBuffers tmp;
    int32_t *d_err;
    TRY(tmp.alloc(&d_err, 1));
    TRY(keep_alloc(&ix->d_lookup, size, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_node_xpos, G, &ix->device_bytes));
    hipLaunchKernelGGL(fill_xpos, dim3(blocks_for(G)), dim3(BT), 0, st, (const uint32_t *)ix->d_node_lo,
                       (const int64_t *)ix->d_x_off, G, ix->d_node_xpos);
    PPV_HIP_TRY(hipMemsetAsync(d_err, 0, sizeof(int32_t), st));
    PPV_HIP_TRY(hipMemsetAsync(ix->d_lookup, 0, (size_t)size * sizeof(uint64_t), st));
    if (G > 1)
        hipLaunchKernelGGL(insert_nodes, dim3(blocks_for(G - 1)), dim3(BT), 0, st, (const uint32_t *)ix->d_node_lo,
                           (const int32_t *)ix->d_x_tok, (const int64_t *)ix->d_x_off,
                           (const uint32_t *)ix->d_depth_base, l_max, G, ix->d_lookup, size, ix->view.lookup_fp_mask,
                           d_err);
    PPV_HIP_TRY(hipGetLastError());
    int32_t err = 0;
    PPV_HIP_TRY(hipMemcpyAsync(&err, d_err, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    PPV_HIP_TRY(hipStreamSynchronize(st));
    if (err != 0) return PPV_EINVAL;
    ix->view.lookup = ix->d_lookup;
    ix->view.node_xpos = ix->d_node_xpos;
    ix->view.lookup_size = size;
    return PPV_OK;
}

ppv_status build_on_device(const int32_t *tokens, const int64_t *offsets, int64_t n_seq, int32_t vocab, ppv_index *ix) {
    if (offsets[0] != 0) return PPV_EINVAL;
    const int64_t total = offsets[n_seq];
    if (total < n_seq) return PPV_EINVAL;                          // some sequence is empty (or offsets decrease)
    if (n_seq > 0xFFFFFFF0ll || total > 0xFFFFFFF0ll) return PPV_ERANGE;
    const uint32_t n = (uint32_t)n_seq;
    hipStream_t st = nullptr;
    DeviceBuffers tmp;

    // ---- inputs to the device
    int32_t *d_tok;
    int64_t *d_off;
    int32_t *d_flags;  // [0] error bits, [1] longest row
    uint32_t *d_total;
    TRY(tmp.alloc(&d_tok, (size_t)total));
    TRY(tmp.alloc(&d_off, (size_t)n + 1));
    TRY(tmp.alloc(&d_flags, 2));
    TRY(tmp.alloc(&d_total, 4));
    PPV_HIP_TRY(hipMemcpyAsync(d_tok, tokens, (size_t)total * sizeof(int32_t), hipMemcpyHostToDevice, st));
    PPV_HIP_TRY(hipMemcpyAsync(d_off, offsets, ((size_t)n + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    PPV_HIP_TRY(hipMemsetAsync(d_flags, 0, 2 * sizeof(int32_t), st));

    // ---- 1. validate
    hipLaunchKernelGGL(check_rows, dim3(blocks_for(n)), dim3(BT), 0, st, (const int64_t *)d_off, (int64_t)n, d_flags,
                       d_flags + 1);
    hipLaunchKernelGGL(check_tokens, dim3(blocks_for((uint64_t)total)), dim3(BT), 0, st, (const int32_t *)d_tok, total,
                       vocab, d_flags);
    int32_t h_flags[2];
    PPV_HIP_TRY(hipMemcpyAsync(h_flags, d_flags, sizeof(h_flags), hipMemcpyDeviceToHost, st));
    PPV_HIP_TRY(hipStreamSynchronize(st));
    if (h_flags[0] != 0) return PPV_EINVAL;                         // empty sequence or token outside [0, vocab)
    const int32_t l_max = h_flags[1];

    // ---- 2. sort rows: LSD radix over the columns, last column first
    uint32_t *perm_a, *perm_b, *hist, *sums;
    uint8_t *digits;
    const uint32_t sort_blocks = (n + SORT_CHUNK - 1) / SORT_CHUNK;
    const uint64_t hist_len = (uint64_t)RADIX * sort_blocks;
    TRY(tmp.alloc(&perm_a, n));
    TRY(tmp.alloc(&perm_b, n));
    TRY(tmp.alloc(&digits, n));
    TRY(tmp.alloc(&hist, (size_t)hist_len));
    // scratch for every scan of the build: the largest one runs over l_max * n flags
    const uint64_t biggest_scan = std::max<uint64_t>((uint64_t)l_max * n + 1, hist_len);
    TRY(tmp.alloc(&sums, (size_t)((biggest_scan + SCAN_CHUNK - 1) / SCAN_CHUNK)));
    hipLaunchKernelGGL(iota_rows, dim3(blocks_for(n)), dim3(BT), 0, st, perm_a, n);
    int key_bits = 1;
    while ((1ll << key_bits) <= (int64_t)vocab) key_bits++;         // keys run over 0 .. vocab
    for (int col = l_max - 1; col >= 0; col--) {
        for (int shift = 0; shift < key_bits; shift += 8) {
            hipLaunchKernelGGL(radix_histogram, dim3(sort_blocks), dim3(BT), 0, st, (const int32_t *)d_tok,
                               (const int64_t *)d_off, (const uint32_t *)perm_a, n, col, shift, digits, hist,
                               sort_blocks);
            TRY(exclusive_scan(hist_len, HistValue{hist}, hist, sums, d_total, st));
            hipLaunchKernelGGL(radix_scatter, dim3(sort_blocks), dim3(BT), 0, st, (const uint32_t *)perm_a, n,
                               (const uint8_t *)digits, (const uint32_t *)hist, sort_blocks, perm_b);
            std::swap(perm_a, perm_b);
        }
    }
    PPV_HIP_TRY(hipGetLastError());

    // ---- 3. neighbours: common prefix, duplicates; compact into the flat sorted S
    int32_t *lcp;
    uint8_t *keep;
    uint32_t *dst, *tok_at;
    TRY(tmp.alloc(&lcp, n));
    TRY(tmp.alloc(&keep, n));
    TRY(tmp.alloc(&dst, n));
    TRY(tmp.alloc(&tok_at, n));
    hipLaunchKernelGGL(neighbour_lcp, dim3(blocks_for(n)), dim3(BT), 0, st, (const int32_t *)d_tok,
                       (const int64_t *)d_off, (const uint32_t *)perm_a, n, lcp, keep);
    TRY(exclusive_scan(n, KeepFlag{keep}, dst, sums, d_total, st));
    TRY(exclusive_scan(n, KeptLen{keep, perm_a, d_off}, tok_at, sums, d_total + 1, st));
    uint32_t h_tot[2];
    PPV_HIP_TRY(hipMemcpyAsync(h_tot, d_total, sizeof(h_tot), hipMemcpyDeviceToHost, st));
    PPV_HIP_TRY(hipStreamSynchronize(st));
    const uint32_t n_rows = h_tot[0], n_tok = h_tot[1];
    ix->device_bytes = 0;
    TRY(keep_alloc(&ix->d_x_tok, n_tok, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_x_off, (size_t)n_rows + 1, &ix->device_bytes));
    int32_t *row_lcp;
    TRY(tmp.alloc(&row_lcp, n_rows));
    hipLaunchKernelGGL(compact_rows, dim3(blocks_for(n)), dim3(BT), 0, st, (const int32_t *)d_tok,
                       (const int64_t *)d_off, (const uint32_t *)perm_a, n, (const uint8_t *)keep,
                       (const uint32_t *)dst, (const uint32_t *)tok_at, (const int32_t *)lcp, ix->d_x_tok, ix->d_x_off,
                       row_lcp, n_rows, n_tok);

    // ---- 4. number the prefixes breadth-first: one scan over the (depth, row) flags
    const uint64_t n_flags = (uint64_t)l_max * n_rows;
    if (n_flags + 1 > 0xFFFFFFF0ull) return PPV_ERANGE;
    uint32_t *pos;
    TRY(tmp.alloc(&pos, (size_t)n_flags + 1));
    TRY(exclusive_scan(n_flags, OpensPrefix{ix->d_x_off, row_lcp, n_rows}, pos, sums, d_total + 2, st));
    uint32_t n_pref;
    PPV_HIP_TRY(hipMemcpyAsync(&n_pref, d_total + 2, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    PPV_HIP_TRY(hipStreamSynchronize(st));
    if (n_pref > 0xFFFFFFF0u - 2) return PPV_ERANGE;
    const uint32_t G = n_pref + 1;                                   // with the empty prefix
    // the scan value one past the end closes the last depth
    PPV_HIP_TRY(hipMemcpyAsync(pos + n_flags, d_total + 2, sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
    TRY(keep_alloc(&ix->d_ent, (size_t)G + 1, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_node_lo, G, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_node_hi, G, &ix->device_bytes));
    hipLaunchKernelGGL(fill_nodes, dim3(blocks_for(std::max<uint64_t>(n_flags, 1))), dim3(BT), 0, st,
                       (const int32_t *)ix->d_x_tok, (const int64_t *)ix->d_x_off, (const int32_t *)row_lcp,
                       (const uint32_t *)pos, (uint64_t)n_rows, l_max, G, ix->d_ent, ix->d_node_lo);

    // ---- 5. hi, deepest depth first (a prefix ends where its last child ends, so the children's depth comes first)
    uint32_t *h_base = new (std::nothrow) uint32_t[(size_t)l_max + 2];
    if (!h_base) return PPV_ENOMEM;
    PPV_HIP_TRY(hipStreamSynchronize(st));
    const ppv_status rc_base = depth_bases(ix, G, l_max, h_base);
    if (rc_base != PPV_OK) {
        delete[] h_base;
        return rc_base;
    }
    for (int d = l_max; d >= 1; d--) {
        const uint32_t g0 = h_base[d], g1 = h_base[d + 1];
        if (g1 > g0)
            hipLaunchKernelGGL(fill_hi, dim3(blocks_for(g1 - g0)), dim3(BT), 0, st, (const NodeEnt *)ix->d_ent,
                               (const uint32_t *)ix->d_node_lo, g0, g1, ix->d_node_hi);
    }
    delete[] h_base;
    hipLaunchKernelGGL(fill_hi, dim3(1), dim3(BT), 0, st, (const NodeEnt *)ix->d_ent, (const uint32_t *)ix->d_node_lo,
                       0u, 1u, ix->d_node_hi);                       // the empty prefix: all of S
    PPV_HIP_TRY(hipGetLastError());

    // ---- 6. heavy prefixes
    TRY(finish_heavy(ix, G, vocab, st));
    TRY(finish_lookup(ix, G, l_max, st));

    ix->n_tokens = n_tok;
    ix->view.ent = ix->d_ent;
    ix->view.node_lo = ix->d_node_lo;
    ix->view.node_hi = ix->d_node_hi;
    ix->view.n_nodes = G;
    ix->view.n_rows = n_rows;
    ix->view.vocab = vocab;
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
    (void)hipFree(ix->d_lookup);
    (void)hipFree(ix->d_depth_base);
    (void)hipFree(ix->d_node_xpos);
    (void)hipFree(ix->d_x_tok);
    (void)hipFree(ix->d_x_off);
    delete ix;
}

// ------------------------------------------------------------------------------------------
// Persistence.  The file holds what cannot be recomputed cheaply -- the entries (heavy flag cleared), the rank
// ranges and the flat sorted S -- behind a fixed header; the heavy prefixes' images are rebuilt at load.
// Little-endian, as the machine is.
struct FileHeader {
    char magic[8];
    uint32_t version, header_bytes;
    int32_t vocab, l_max;
    uint64_t n_rows, n_nodes, n_tokens;
    uint64_t checksum;      // over the sections, in file order
    uint64_t reserved[9];
};
static_assert(sizeof(FileHeader) == 128, "file header layout");
const char FILE_MAGIC[8] = {'P', 'P', 'V', 'I', 'D', 'X', 0, 1};
constexpr size_t IO_CHUNK = 32u << 20;   // bytes staged per copy

// 64-bit multiply-xor checksum over 8-byte words (the tail is zero-padded); `h` carries across calls whose
// lengths are multiples of 8 except the last of a section
inline uint64_t checksum_words(uint64_t h, const unsigned char *p, size_t n) {
    size_t i = 0;
    for (; i + 8 <= n; i += 8) {
        uint64_t w;
        memcpy(&w, p + i, 8);
        h = (h ^ w) * 0x100000001B3ull;
        h ^= h >> 29;
    }
    if (i < n) {
        uint64_t w = 0;
        memcpy(&w, p + i, n - i);
        h = (h ^ w) * 0x100000001B3ull;
        h ^= h >> 29;
    }
    return h;
}

struct Section {
    void *dev;
    size_t bytes;
    bool entries;   // NodeEnt array: the heavy flag is not stored
};

// structural checks of a loaded index: whatever the file held, the kernels must stay inside the arrays
__global__ __launch_bounds__(BT) void check_loaded_nodes(const NodeEnt *__restrict__ ent,
                                                         const uint32_t *__restrict__ node_lo,
                                                         const uint32_t *__restrict__ node_hi, uint32_t n_nodes,
                                                         uint32_t n_rows, uint32_t vocab, int32_t *__restrict__ err) {
    const uint32_t g = blockIdx.x * BT + threadIdx.x;
    if (g >= n_nodes) return;
    const uint32_t c0 = ent[g].child, c1 = ent[g + 1].child;
    bool bad = c0 > c1 || c1 > n_nodes || (c1 > c0 && c0 <= g);   // children lie after their parent
    bad = bad || (ent[g].tok & PPV_NODE_HEAVY) != 0u || (g > 0 && (ent[g].tok & PPV_NODE_TOKEN) >= vocab);
    bad = bad || !(node_lo[g] < node_hi[g] && node_hi[g] <= n_rows);
    if (g == 0) bad = bad || c0 != 1u;
    if (g == n_nodes - 1) bad = bad || c1 != n_nodes || (ent[n_nodes].tok & PPV_NODE_HEAVY) != 0u;
    if (!bad)
        for (uint32_t c = c0; c + 1 < c1; c++)   // siblings in strictly increasing token order
            if ((ent[c].tok & PPV_NODE_TOKEN) >= (ent[c + 1].tok & PPV_NODE_TOKEN)) {
                bad = true;
                break;
            }
    if (bad) atomicOr(err, 1);
}
__global__ __launch_bounds__(BT) void check_loaded_rows(const int32_t *__restrict__ x_tok, const int64_t *__restrict__ x_off,
                                                        uint64_t n_rows, uint64_t n_tokens, int32_t vocab, int32_t l_max,
                                                        int32_t *__restrict__ err) {
    const uint64_t i = (uint64_t)blockIdx.x * BT + threadIdx.x;
    bool bad = false;
    if (i < n_rows) {
        const int64_t a = x_off[i], b = x_off[i + 1];
        bad = a < 0 || b <= a || b - a > l_max || (uint64_t)b > n_tokens || (i == 0 && a != 0) ||
              (i == n_rows - 1 && (uint64_t)b != n_tokens);
    }
    if (i < n_tokens) bad = bad || x_tok[i] < 0 || x_tok[i] >= vocab;
    if (bad) atomicOr(err, 2);
}

ppv_status save_to_file(const ppv_index *ix, const char *path) {
    PPV_HIP_TRY(hipSetDevice(ix->device));
    FILE *f = fopen(path, "wb");
    if (!f) return PPV_EIO;
    unsigned char *stage = new (std::nothrow) unsigned char[IO_CHUNK];
    if (!stage) {
        fclose(f);
        return PPV_ENOMEM;
    }
    FileHeader h;
    memset(&h, 0, sizeof(h));
    memcpy(h.magic, FILE_MAGIC, 8);
    h.version = 1;
    h.header_bytes = sizeof(FileHeader);
    h.vocab = ix->view.vocab;
    h.l_max = ix->view.l_max;
    h.n_rows = ix->view.n_rows;
    h.n_nodes = ix->view.n_nodes;
    h.n_tokens = (uint64_t)ix->n_tokens;
    const Section sec[5] = {{ix->d_ent, ((size_t)h.n_nodes + 1) * sizeof(NodeEnt), true},
                            {ix->d_node_lo, (size_t)h.n_nodes * sizeof(uint32_t), false},
                            {ix->d_node_hi, (size_t)h.n_nodes * sizeof(uint32_t), false},
                            {ix->d_x_off, ((size_t)h.n_rows + 1) * sizeof(int64_t), false},
                            {ix->d_x_tok, (size_t)h.n_tokens * sizeof(int32_t), false}};
    ppv_status st = PPV_OK;
    if (fwrite(&h, sizeof(h), 1, f) != 1) st = PPV_EIO;
    uint64_t sum = 0xCBF29CE484222325ull;
    for (int k = 0; k < 5 && st == PPV_OK; k++)
        for (size_t at = 0; at < sec[k].bytes && st == PPV_OK; at += IO_CHUNK) {
            const size_t n = std::min(IO_CHUNK, sec[k].bytes - at);
            if (hipMemcpy(stage, (const unsigned char *)sec[k].dev + at, n, hipMemcpyDeviceToHost) != hipSuccess) {
                (void)hipGetLastError();
                st = PPV_EDEVICE;
                break;
            }
            if (sec[k].entries)
                for (size_t e = 0; e < n / sizeof(NodeEnt); e++) {
                    NodeEnt ne;
                    memcpy(&ne, stage + e * sizeof(NodeEnt), sizeof(NodeEnt));
                    ne.tok &= ~PPV_NODE_HEAVY;
                    memcpy(stage + e * sizeof(NodeEnt), &ne, sizeof(NodeEnt));
                }
            sum = checksum_words(sum, stage, n);
            if (fwrite(stage, 1, n, f) != n) st = PPV_EIO;
        }
    delete[] stage;
    if (st == PPV_OK) {
        h.checksum = sum;
        if (fseek(f, 0, SEEK_SET) != 0 || fwrite(&h, sizeof(h), 1, f) != 1) st = PPV_EIO;
    }
    if (fclose(f) != 0 && st == PPV_OK) st = PPV_EIO;
    return st;
}

ppv_status load_from_file(FILE *f, ppv_index *ix) {
    FileHeader h;
    if (fread(&h, sizeof(h), 1, f) != 1) return PPV_EINVAL;   // shorter than a header: not an index file
    if (memcmp(h.magic, FILE_MAGIC, 8) != 0 || h.version != 1 || h.header_bytes != sizeof(FileHeader)) return PPV_EINVAL;
    if (h.vocab <= 0 || h.l_max <= 0 || h.n_rows == 0 || h.n_nodes < 2 || h.n_tokens < h.n_rows) return PPV_EINVAL;
    if (h.vocab > PPV_MAX_VOCAB || h.n_rows > 0xFFFFFFF0ull || h.n_nodes > 0xFFFFFFF0ull || h.n_tokens > 0xFFFFFFF0ull)
        return PPV_ERANGE;
    const size_t bytes[5] = {((size_t)h.n_nodes + 1) * sizeof(NodeEnt), (size_t)h.n_nodes * sizeof(uint32_t),
                             (size_t)h.n_nodes * sizeof(uint32_t), ((size_t)h.n_rows + 1) * sizeof(int64_t),
                             (size_t)h.n_tokens * sizeof(int32_t)};
    if (fseek(f, 0, SEEK_END) != 0) return PPV_EIO;
    const long end = ftell(f);
    if (end < 0 || (uint64_t)end != sizeof(h) + bytes[0] + bytes[1] + bytes[2] + bytes[3] + bytes[4]) return PPV_EINVAL;
    if (fseek(f, (long)sizeof(h), SEEK_SET) != 0) return PPV_EIO;

    if (hipGetDevice(&ix->device) != hipSuccess) {
        (void)hipGetLastError();
        return PPV_EDEVICE;
    }
    ix->device_bytes = 0;
    TRY(keep_alloc(&ix->d_ent, (size_t)h.n_nodes + 1, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_node_lo, (size_t)h.n_nodes, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_node_hi, (size_t)h.n_nodes, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_x_off, (size_t)h.n_rows + 1, &ix->device_bytes));
    TRY(keep_alloc(&ix->d_x_tok, (size_t)h.n_tokens, &ix->device_bytes));
    void *dev[5] = {ix->d_ent, ix->d_node_lo, ix->d_node_hi, ix->d_x_off, ix->d_x_tok};
    unsigned char *stage = new (std::nothrow) unsigned char[IO_CHUNK];
    if (!stage) return PPV_ENOMEM;
    ppv_status st = PPV_OK;
    uint64_t sum = 0xCBF29CE484222325ull;
    for (int k = 0; k < 5 && st == PPV_OK; k++)
        for (size_t at = 0; at < bytes[k] && st == PPV_OK; at += IO_CHUNK) {
            const size_t n = std::min(IO_CHUNK, bytes[k] - at);
            if (fread(stage, 1, n, f) != n) {
                st = PPV_EIO;
                break;
            }
            sum = checksum_words(sum, stage, n);
            if (hipMemcpy((unsigned char *)dev[k] + at, stage, n, hipMemcpyHostToDevice) != hipSuccess) {
                (void)hipGetLastError();
                st = PPV_EDEVICE;
            }
        }
    delete[] stage;
    if (st != PPV_OK) return st;
    if (sum != h.checksum) return PPV_EINVAL;

    // the checksum guards against damage; these checks guard the kernels against a file that was wrong when written
    hipStream_t s0 = nullptr;
    DeviceBuffers tmp;
    int32_t *d_err;
    TRY(tmp.alloc(&d_err, 1));
    PPV_HIP_TRY(hipMemsetAsync(d_err, 0, sizeof(int32_t), s0));
    hipLaunchKernelGGL(check_loaded_nodes, dim3(blocks_for(h.n_nodes)), dim3(BT), 0, s0, (const NodeEnt *)ix->d_ent,
                       (const uint32_t *)ix->d_node_lo, (const uint32_t *)ix->d_node_hi, (uint32_t)h.n_nodes,
                       (uint32_t)h.n_rows, (uint32_t)h.vocab, d_err);
    hipLaunchKernelGGL(check_loaded_rows, dim3(blocks_for(std::max(h.n_rows, h.n_tokens))), dim3(BT), 0, s0,
                       (const int32_t *)ix->d_x_tok, (const int64_t *)ix->d_x_off, h.n_rows, h.n_tokens, h.vocab, h.l_max,
                       d_err);
    PPV_HIP_TRY(hipGetLastError());
    int32_t err = 0;
    PPV_HIP_TRY(hipMemcpy(&err, d_err, sizeof(int32_t), hipMemcpyDeviceToHost));
    if (err != 0) return PPV_EINVAL;

    TRY(finish_heavy(ix, (uint32_t)h.n_nodes, h.vocab, s0));
    TRY(finish_lookup(ix, (uint32_t)h.n_nodes, h.l_max, s0));
    ix->n_tokens = (int64_t)h.n_tokens;
    ix->view.ent = ix->d_ent;
    ix->view.node_lo = ix->d_node_lo;
    ix->view.node_hi = ix->d_node_hi;
    ix->view.n_nodes = (uint32_t)h.n_nodes;
    ix->view.n_rows = (uint32_t)h.n_rows;
    ix->view.vocab = h.vocab;
    ix->view.l_max = h.l_max;
    return PPV_OK;
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
    if (hipGetDevice(&ix->device) != hipSuccess) {
        (void)hipGetLastError();
        delete ix;
        return PPV_EDEVICE;
    }
    ppv_status st = build_on_device(tokens, offsets, n_seq, vocab, ix);
    if (st != PPV_OK) {
        (void)hipDeviceSynchronize();
        (void)hipGetLastError();
        release(ix);
        return st;
    }
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

extern "C" ppv_status ppv_index_save(const ppv_index_t *ix, const char *path) {
    if (!ix || !path || !path[0]) return PPV_EINVAL;
    return save_to_file(ix, path);
}

extern "C" ppv_status ppv_index_load(const char *path, ppv_index_t **out) {
    if (!out) return PPV_EINVAL;
    *out = nullptr;
    if (!path || !path[0]) return PPV_EINVAL;
    FILE *f = fopen(path, "rb");
    if (!f) return PPV_EIO;
    ppv_index *ix = new (std::nothrow) ppv_index();
    if (!ix) {
        fclose(f);
        return PPV_ENOMEM;
    }
    ix->device = -1;
    const ppv_status st = load_from_file(f, ix);
    fclose(f);
    if (st != PPV_OK) {
        if (ix->device >= 0) {   // the device was touched: let its work drain before the buffers go
            (void)hipDeviceSynchronize();
            (void)hipGetLastError();
            release(ix);
        } else {
            delete ix;
        }
        return st;
    }
    *out = ix;
    return PPV_OK;
}
