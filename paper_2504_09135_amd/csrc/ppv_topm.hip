// Algorithm 2 with M candidates (the variant the paper ran with M = 50): per row, the M tokens of
// largest probability, one verification per candidate row a + [t_i], and the extended mask.
//
// One workgroup per row.
//   select   P = softmax(logits) is increasing in the logit, so the top M are found on the logits'
//            bit patterns, through an order-preserving 32-bit key per token.  M is small against
//            |V|, so almost every token can be turned away with one comparison:
//              A. the maximum of every 16-byte group of tokens is histogrammed by its leading 11 key
//                 bits; the bin that holds the M-th largest group maximum gives a bound L that at
//                 least M tokens reach.  A wavefront holds eight chunks of the row (8 KB of bf16) in
//                 registers; when its share of the row is longer, A looks only at those eight --
//                 the M-th largest of a part of the row is still a lower bound of the row's --
//                 provided the list has room for what the looser bound lets through (else from as
//                 many more of its chunks as it takes).  When A has looked at one set of eight, the
//                 maxima inside the bound's bin are counted once more by their next five key bits
//                 and the bound moves up inside the bin;
//              B. the tokens that are not below L are listed in LDS in token order, each with its
//                 logit: usually 1.1 to 1.5 M of them, from registers when A saw the whole row,
//                 else about as many times more as the share is longer than eight chunks, from the
//                 one pass over the row (the next eight chunks are asked for before these eight are
//                 looked at).  bf16 rows are compared two tokens at a time on 16-bit keys, and a
//                 chunk in which no lane has a token for the list costs a ballot;
//              C. a radix select over that short list (the keys' upper halves, counted from L, in one
//                 histogram of 256 bins; two more digits of 8 bits for fp32) finds the key T of the
//                 M-th largest token; the list is then cut to the
//                 tokens above T and the first few equal to T, in increasing token id, so the set
//                 is unique.
//            If the list does not fit (a flat row with thousands of equal logits at the cut, or a
//            workgroup too small to hold it) the same radix select runs over the whole row instead,
//            one histogram pass per digit and two more passes to gather in token order.
//   verify   the M candidate rows share their first |a| tokens, so the prefix is located once
//            (the same walk the full-vocabulary mask uses) and each candidate then needs one
//            binary search for its last token among the prefix's children (their tokens are
//            copied to LDS while the row is on its way) -- or one bit test in the ready-made
//            image of a heavy prefix.  One thread per candidate.
//   extend   the mask row is assembled in LDS and written with whole words.
//   count    a caller that wants only the mask (no candidate list, no verdicts) does not need the top M at all
//            when the prefix has few continuations: token t is among the M most probable iff fewer than M
//            tokens come before it in the order (logit descending, token id ascending).  Those are counted
//            for each child in one pass over the row, two instructions per token and child, with no
//            histogram, no list and no second pass.
// Nothing here is a dense contraction; the row is read from HBM once (64 KB at V = 32k, bf16).
#include <cstdlib>

#include "ppv_device.h"
#include "ppv_internal.h"
#include "ppv_walk.h"

namespace {

constexpr int TOPM_BITS = 11;             // leading key bits of the first digit
constexpr int TOPM_BINS = 1 << TOPM_BITS;   // the histogram shares its LDS with the mask row
constexpr int TOPM_SHIFT = 32 - TOPM_BITS;
constexpr int TOPM_CBINS = 256;   // bins of the histogram over the listed tokens' keys, counted from the bound (the last one: all above)
constexpr int TOPM_WAVES = 16;
constexpr int TOPM_LIST_BIG = 4096, TOPM_LIST_SMALL = 1024;   // capacity of the candidate list (tokens not below the bound),
                                                              // split evenly over the wavefronts; the small one serves M <= 128 at V <= 65,536
constexpr int TOPM_SLOTS = 16;    // list entries per thread at most: the list path needs at least LIST / 16 threads
constexpr int TOPM_HELD = 8;      // chunks of the row a wavefront holds in registers at a time (128 bytes per lane)

// Bit pattern -> key with the same order as the float value (-0 and +0 share a key).
__device__ inline uint32_t order_key(uint32_t bits) {
    if (bits == 0x80000000u) bits = 0u;
    return bits ^ ((uint32_t)((int32_t)bits >> 31) | 0x80000000u);
}

// the bit pattern whose key is k
__device__ inline uint32_t key_to_bits(uint32_t k) { return (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k; }

template <typename T> struct KeyChunk;   // what one 16-byte load per lane covers
template <> struct KeyChunk<float> {
    static constexpr int EPL = 4;
    __device__ static inline void keys(const uint4 &r, uint32_t k[4]) {
        k[0] = order_key(r.x); k[1] = order_key(r.y); k[2] = order_key(r.z); k[3] = order_key(r.w);
    }
    __device__ static inline uint32_t bits_of(const float *row, int v) { return ((const uint32_t *)row)[v]; }
};
template <> struct KeyChunk<uint16_t> {
    static constexpr int EPL = 8;
    __device__ static inline void keys(const uint4 &r, uint32_t k[8]) {
        k[0] = order_key(r.x << 16); k[1] = order_key(r.x & 0xFFFF0000u);
        k[2] = order_key(r.y << 16); k[3] = order_key(r.y & 0xFFFF0000u);
        k[4] = order_key(r.z << 16); k[5] = order_key(r.z & 0xFFFF0000u);
        k[6] = order_key(r.w << 16); k[7] = order_key(r.w & 0xFFFF0000u);
    }
    __device__ static inline uint32_t bits_of(const uint16_t *row, int v) { return (uint32_t)row[v] << 16; }
};

// Keys of this lane's EPL consecutive tokens of chunk c (tokens c*64*EPL + lane*EPL + k).  Returns how
// many of them lie inside the row (the first n of k[]); memory at or beyond token V is never touched.
template <typename T>
__device__ inline int load_keys(const T *__restrict__ row, int V, int c, int lane, uint32_t k[KeyChunk<T>::EPL]) {
    constexpr int EPL = KeyChunk<T>::EPL;
    const int g = (c * WAVE + lane) * EPL;
    if (g + EPL <= V) {
        KeyChunk<T>::keys(*(const uint4 *)(row + g), k);
        return EPL;
    }
    int n = 0;
    for (int j = 0; j < EPL; j++) {
        k[j] = 0u;
        if (g + j < V) {
            k[j] = order_key(KeyChunk<T>::bits_of(row, g + j));
            n = j + 1;
        }
    }
    return n;
}

// This lane's 16 bytes of chunk c, from an address that is always inside the row: a chunk beyond the last one
// reads the last one again, a lane beyond the row's end reads the row's first bytes (the caller discards both,
// and the tokens of the row's last group that lie beyond its end).  No condition stands between the caller and
// the load, so loads for the next batch can be in flight while this batch is worked on.  STREAM: the bytes are
// not read again (they need not stay in cache).
template <typename T, bool STREAM = true>
__device__ inline uint4 load_raw_clamped(const T *__restrict__ row, int V, int nc, int c, int lane) {
    constexpr int EPL = KeyChunk<T>::EPL;
    const int cc = c < nc ? c : nc - 1;
    const int g = (cc * WAVE + lane) * EPL;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *at = (const u32x4 *)(row + (g < V ? g : 0));
    const u32x4 v = STREAM ? __builtin_nontemporal_load(at) : *at;
    return make_uint4(v.x, v.y, v.z, v.w);
}
// four chunks at once (c .. c+3): four loads in flight per lane
template <typename T, bool STREAM>
__device__ inline void load_chunks(const T *__restrict__ row, int V, int nc, int c, int lane, uint4 *r) {
#pragma unroll
    for (int u = 0; u < 4; u++) r[u] = load_raw_clamped<T, STREAM>(row, V, nc, c + u, lane);
}
// how many of this lane's tokens of chunk c lie inside the row
template <typename T> __device__ inline int n_inside(int V, int c, int lane) {
    constexpr int EPL = KeyChunk<T>::EPL;
    const int r = V - (c * WAVE + lane) * EPL;
    return r < 0 ? 0 : (r > EPL ? EPL : r);
}
template <typename T> __device__ inline void unpack_vals(const uint4 &r, float x[KeyChunk<T>::EPL]) {
    if (sizeof(T) == 4) {
        x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
        x[2 % KeyChunk<T>::EPL] = __uint_as_float(r.z); x[3 % KeyChunk<T>::EPL] = __uint_as_float(r.w);
    } else {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int j = 0; j < 4; j++) {
            x[(2 * j) % KeyChunk<T>::EPL] = __uint_as_float(w[j] << 16);
            x[(2 * j + 1) % KeyChunk<T>::EPL] = __uint_as_float(w[j] & 0xFFFF0000u);
        }
    }
}

// inclusive prefix sum of x over the workgroup's threads in thread order; nw wavefronts
__device__ inline uint32_t block_incl_scan(uint32_t x, uint32_t *wave_tot, int nw) {
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    const uint32_t incl = wave_incl_scan(x);
    if (lane == WAVE - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < nw; w++)
        if (w < wave) before += wave_tot[w];
    __syncthreads();
    return before + incl;
}

// The histogram hist[0..bins) is filled (bins <= 4096).  Finds the digit d with #(digit > d) < need <= #(digit >= d)
// and leaves it in bc[4], with need - #(digit > d) in bc[5].  If fewer than `need` entries were counted,
// bc[4] = 0 and bc[5] = need.  Every thread calls; ends with a barrier.
// The work is wavefront 0's alone, in two levels without a barrier between them: lane l sums a run of consecutive
// bins (runs ordered from the top bin down), a scan over the lanes finds the run in which the count reaches
// `need`, and that run's bins, one per lane, are scanned the same way.  (A scan over all the workgroup's threads
// costs three barriers and was 1.5 to 2.2 us of a 16 us call.)
__device__ inline void pick_digit(const uint32_t *hist, int bins, uint32_t need, uint32_t *wave_tot, uint32_t *bc,
                                  int nthreads) {
    (void)wave_tot;
    (void)nthreads;
    if (threadIdx.x < WAVE) {
        const int lane = threadIdx.x;
        const int per = (bins + WAVE - 1) / WAVE;        // bins per lane, at most 64
        const int top_bin = bins - 1 - lane * per;       // lane l: bins top_bin - per + 1 .. top_bin
        const int low_bin = top_bin - per + 1;
        uint32_t s = 0;
        if (low_bin >= 0 && (per & 3) == 0 && (bins & 3) == 0) {   // whole run present and 16-byte aligned
            for (int j = 0; j < per; j += 4) {
                const uint4 h = *(const uint4 *)(hist + low_bin + j);
                s += h.x + h.y + h.z + h.w;
            }
        } else {
            for (int j = 0; j < per; j++)
                if (top_bin - j >= 0) s += hist[top_bin - j];
        }
        const uint32_t incl = wave_incl_scan(s);
        const uint64_t reach = __ballot(incl >= need);
        uint32_t digit = 0u, rest = need;
        if (reach) {   // wave-uniform
            const int l = __ffsll((long long)reach) - 1;                 // the run in which the count reaches need
            const uint32_t above = lane_value(incl - s, l);              // entries in the runs above it
            const int run_top = bins - 1 - l * per;
            const int bin = run_top - lane;                               // level 2: lane j takes bin run_top - j
            const uint32_t h = (lane < per && bin >= 0) ? hist[bin] : 0u;
            const uint32_t incl2 = above + wave_incl_scan(h);
            const uint64_t reach2 = __ballot(lane < per && bin >= 0 && incl2 >= need);
            if (reach2) {   // always: the run's total reaches need
                const int j = __ffsll((long long)reach2) - 1;
                digit = (uint32_t)(run_top - j);
                rest = need - lane_value(incl2 - h, j);
            }
        }
        if (lane == 0) {
            bc[4] = digit;
            bc[5] = rest;
        }
    }
    __syncthreads();
}

// digit p of the radix select: key bits [shift, previous shift)
template <typename T> __device__ inline int digit_shift(int pass) {
    return pass == 0 ? TOPM_SHIFT : (sizeof(T) == 4 ? (pass == 1 ? TOPM_SHIFT - TOPM_BITS : 0) : 16);
}
// bf16: the low 16 bits of a key follow from its sign, so the upper half settles the whole key
template <typename T> __device__ inline uint32_t full_key(uint32_t hi_part) {
    return sizeof(T) == 4 ? hi_part : ((hi_part << 16) | ((hi_part >> 15) & 1u ? 0u : 0xFFFFu));
}

struct TopmLds {
    uint32_t *hist;       // [TOPM_BINS]
    uint32_t *hist3;      // [32] the group maxima inside the bound's bin, by their next five key bits
    uint32_t *hist2;      // [TOPM_CBINS] the listed tokens' keys, counted from the bound (filled while they are listed)
    uint32_t *list_tok;   // [LIST]
    uint32_t *list_key;   // [LIST] the listed tokens' logits (bit patterns, bf16 in the upper half)
    uint32_t *sel;        // [PPV_TOPM_MAX]
    uint32_t *seg_a, *seg_b, *wave_tot;   // [TOPM_WAVES] each
    uint32_t *bc;         // [8]
};

// Radix select over the whole row (any workgroup size, any row): fills sel[0..m) in increasing token id.
template <typename T>
__device__ inline void select_streaming(const T *__restrict__ row, int V, int c0, int c1, int m, const TopmLds &s,
                                        int lane, int wave, int nthreads) {
    constexpr int EPL = KeyChunk<T>::EPL;
    const int tid = threadIdx.x, nw = nthreads / WAVE;
    const int n_pass = sizeof(T) == 4 ? 3 : 2;
    uint32_t hi_part = 0;          // digits settled so far, as the key's leading bits
    uint32_t need = (uint32_t)m;   // how many tokens are still to be taken among those that match hi_part
    int prev_shift = 32;
    for (int pass = 0; pass < n_pass; pass++) {
        const int shift = digit_shift<T>(pass);
        const int bins = 1 << (prev_shift - shift);
        for (int i = tid; i < bins; i += nthreads) s.hist[i] = 0u;
        __syncthreads();
        for (int c = c0; c < c1; c++) {
            uint32_t k[EPL];
            const int n = load_keys<T>(row, V, c, lane, k);
#pragma unroll
            for (int j = 0; j < EPL; j++) {
                const bool match = pass == 0 || (k[j] >> prev_shift) == hi_part;
                if (j < n && match) atomicAdd(&s.hist[(k[j] >> shift) & (uint32_t)(bins - 1)], 1u);
            }
        }
        __syncthreads();
        pick_digit(s.hist, bins, need, s.wave_tot, s.bc, nthreads);
        hi_part = (hi_part << (prev_shift - shift)) | s.bc[4];
        need = s.bc[5];
        prev_shift = shift;
        __syncthreads();
    }
    const uint32_t T_key = full_key<T>(hi_part);
    const uint32_t take_eq = need;   // of the tokens whose key equals T_key, the first take_eq in token order

    // gather in token order: counts per wavefront share, then positions from prefix counts
    uint32_t n_gt = 0, n_eq = 0;
    for (int c = c0; c < c1; c++) {
        uint32_t k[EPL];
        const int n = load_keys<T>(row, V, c, lane, k);
#pragma unroll
        for (int j = 0; j < EPL; j++) {
            n_gt += (j < n && k[j] > T_key) ? 1u : 0u;
            n_eq += (j < n && k[j] == T_key) ? 1u : 0u;
        }
    }
    n_gt = wave_sum(n_gt);
    n_eq = wave_sum(n_eq);
    if (lane == 0) {
        s.seg_a[wave] = n_gt;
        s.seg_b[wave] = n_eq;
    }
    __syncthreads();
    uint32_t gt_base = 0, eq_base = 0;   // tokens of either kind in the wavefronts before this one
    for (int w = 0; w < nw; w++)
        if (w < wave) {
            gt_base += s.seg_a[w];
            eq_base += s.seg_b[w];
        }
    for (int c = c0; c < c1; c++) {
        uint32_t k[EPL];
        const int n = load_keys<T>(row, V, c, lane, k);
        uint32_t g = 0, e = 0;
#pragma unroll
        for (int j = 0; j < EPL; j++) {
            g += (j < n && k[j] > T_key) ? 1u : 0u;
            e += (j < n && k[j] == T_key) ? 1u : 0u;
        }
        const uint32_t gi = wave_incl_scan(g), ei = wave_incl_scan(e);
        uint32_t gt_before = gt_base + gi - g, eq_before = eq_base + ei - e;
        const uint32_t first_tok = (uint32_t)((c * WAVE + lane) * EPL);
#pragma unroll
        for (int j = 0; j < EPL; j++) {
            if (j >= n) continue;
            if (k[j] > T_key) {
                const uint32_t pos = gt_before + (eq_before < take_eq ? eq_before : take_eq);
                if (pos < (uint32_t)m) s.sel[pos] = first_tok + j;
                gt_before++;
            } else if (k[j] == T_key) {
                if (eq_before < take_eq) {
                    const uint32_t pos = gt_before + eq_before;
                    if (pos < (uint32_t)m) s.sel[pos] = first_tok + j;
                }
                eq_before++;
            }
        }
        gt_base += last_lane(gi);
        eq_base += last_lane(ei);
    }
    __syncthreads();
}

// Two bf16 values in one word -> their two 16-bit keys, ordered as the values are (-0 just below +0: the
// thresholds below allow for it).
typedef short topm_s2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pk_keys(uint32_t w) {
    const topm_s2 sign = __builtin_bit_cast(topm_s2, w) >> 15;   // 0xFFFF under a negative value
    return w ^ (__builtin_bit_cast(uint32_t, sign) | 0x80008000u);
}
// per half: 1 if the key is above the threshold, else 0.  Two packed 16-bit instructions (saturating subtraction,
// minimum with 1), written out because the compiler turns the same expression back into a comparison and a
// select per half.
__device__ inline uint32_t pk_above(uint32_t keys, uint32_t thresholds) {
    uint32_t d, r;
    const uint32_t ones = 0x00010001u;
    asm("v_pk_sub_u16 %0, %1, %2 clamp" : "=v"(d) : "v"(keys), "v"(thresholds));
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(r) : "v"(d), "v"(ones));
    return r;
}
// Bound, short list, radix select over the list.  Needs nthreads >= LIST / TOPM_SLOTS and nthreads <= LIST.
// Returns false (for every thread alike) when the list did not fit; sel is then untouched.  r arrives holding
// the wavefront's first TOPM_HELD chunks; hist, hist2 and bc[6] were cleared before the workgroup's last barrier.
// The row is read from memory once: a share longer than r gives the bound from its first chunks only (at least m
// of THEIR groups reach it, so at least m tokens of the row do) -- as many batches of TOPM_HELD chunks as it takes
// for the list to have room for what the looser bound lets through, which is about share / those chunks times
// more; B reads the batches after the first again, from cache, and the rest of the share for the first time.
template <typename T, int LIST>
__device__ inline bool select_listed(const T *__restrict__ row, int V, int c0, int c1, int m, const TopmLds &s, int lane,
                                     int wave, int nthreads, uint4 (&r)[TOPM_HELD]) {
    constexpr int EPL = KeyChunk<T>::EPL;
    const int tid = threadIdx.x, nw = nthreads / WAVE;
    // ---- A. maxima of the 16-byte groups, histogram of their leading key bits.  The row is taken TOPM_HELD
    // chunks at a time (as many loads in flight per lane), a_batches batches of each wavefront's share.
    const int nc = (V + WAVE * EPL - 1) / (WAVE * EPL);
    const int cpw = (nc + nw - 1) / nw;             // chunks per wavefront (the last ones may have fewer)
    const bool kept = cpw <= TOPM_HELD;             // r holds a wavefront's whole share
    // With the bound from the whole row the list holds 1.1 to 1.5 m tokens when the bound is taken to the key's
    // upper 16 bits (below: possible when A looks at one batch) and about 4 m of a row of noise when it stays at
    // the histogram's bin, a quarter of an octave; from a_batches batches of the share, cpw / (TOPM_HELD a_batches)
    // times more.  One batch if the list then has room for twice 1.3 m times that, else as few as leave room for
    // 4 m times that.  (A list that overflows all the same sends the row to the whole-row select.)
    const int all_batches = (cpw + TOPM_HELD - 1) / TOPM_HELD;
    const long long want = (long long)m * cpw <= 4ll * LIST ? 1 : ((long long)m * cpw + 2ll * LIST - 1) / (2ll * LIST);
    const int a_batches = want > all_batches ? all_batches : (int)want;
    const uint32_t R = (uint32_t)(LIST / nw);
    const uint32_t base = (uint32_t)wave * R;
    const int a_end = c0 + a_batches * TOPM_HELD < c1 ? c0 + a_batches * TOPM_HELD : c1;
    uint32_t gk[TOPM_HELD];   // the keys of this lane's group maxima in the batch A looked at last, and which of them count
    uint32_t gvalid = 0u;
    for (int c = c0; c < a_end; c += TOPM_HELD) {
        gvalid = 0u;
        if (c != c0) {   // (chunks that A reads from memory are read again in B: from cache)
            load_chunks<T, false>(row, V, nc, c, lane, r);
            load_chunks<T, false>(row, V, nc, c + 4, lane, r + 4);
        }
#pragma unroll
        for (int u = 0; u < TOPM_HELD; u++) {
            if (c + u >= c1) continue;   // (wave-uniform) short rows: most of r is unused
            float x[EPL];
            unpack_vals<T>(r[u], x);
            const int n = n_inside<T>(V, c + u, lane);
            if ((c + u + 1) * WAVE * EPL > V) {   // (wave-uniform) the row ends inside this chunk
#pragma unroll
                for (int j = 1; j < EPL; j++)
                    if (j >= n) x[j] = -INFINITY;
            }
            float gm = x[0];
#pragma unroll
            for (int j = 1; j < EPL; j++) gm = fmaxf(gm, x[j]);
            gk[u] = order_key(__float_as_uint(gm));
            if (n > 0) {
                atomicAdd(&s.hist[gk[u] >> TOPM_SHIFT], 1u);
                gvalid |= 1u << u;
            }
        }
    }
    __syncthreads();
    pick_digit(s.hist, TOPM_BINS, (uint32_t)m, s.wave_tot, s.bc, nthreads);
    // At least m groups have their maximum in this bin or above, so at least m tokens are not below the bin's
    // lower edge.  With fewer than m groups in the row the bin is 0 and its edge is a NaN: nothing is below it.
    uint32_t edge_key16 = s.bc[4] << (16 - TOPM_BITS);
    if (a_batches == 1 && s.bc[4] != 0u) {   // (uniform)
        // A bin is a quarter of an octave wide and holds several times m tokens of a row of noise.  The maxima that
        // A has just seen are still in registers: those inside the bin are counted by their next five key bits, and
        // the bound moves up to the thirty-second of the bin in which the count from the top reaches m.
        const uint32_t bin = s.bc[4], rest = s.bc[5];
#pragma unroll
        for (int u = 0; u < TOPM_HELD; u++)
            if (((gvalid >> u) & 1u) && (gk[u] >> TOPM_SHIFT) == bin) atomicAdd(&s.hist3[(gk[u] >> 16) & 31u], 1u);
        __syncthreads();
        pick_digit(s.hist3, 32, rest, s.wave_tot, s.bc, nthreads);
        edge_key16 |= s.bc[4];
    }
    const float L = __uint_as_float(key_to_bits(edge_key16 << 16));
    // ---- B. the tokens that are not below L, in token order, each wavefront into its own part of the list,
    // each with its logit
    uint32_t cnt = 0;   // wave-uniform
    // bf16 rows are compared two tokens at a time on 16-bit keys: everything whose key is not below the edge's.
    // (-0 has the key just under +0's here; an edge at +0 is lowered by one so that it stays listed.  The list may
    // hold more than the float comparison would put there, never less: C goes by the exact keys.)
    const uint32_t th16 = edge_key16 == 0x8000u ? 0x7FFEu : edge_key16 - 1u;   // listed: key above th16 (edge 0: all)
    const uint32_t th_pk = th16 | (th16 << 16);
    if (a_batches > 1) {   // A has left its last chunks in r
        load_chunks<T, true>(row, V, nc, c0, lane, r);
        load_chunks<T, true>(row, V, nc, c0 + 4, lane, r + 4);
    }
    auto list_chunk = [&](const uint4 &rr, int cc) {   // chunk cc of the row, this lane's 16 bytes of it in rr
        // a[i]: word i of the lane's group; bf16: a 1 in each half whose token is listed, fp32: 1 if it is
        uint32_t a[4];
        const uint32_t w[4] = {rr.x, rr.y, rr.z, rr.w};
        if (sizeof(T) == 2) {
            if (edge_key16 == 0u) {   // (uniform)
                a[0] = a[1] = a[2] = a[3] = 0x00010001u;
            } else {
#pragma unroll
                for (int i = 0; i < 4; i++) a[i] = pk_above(pk_keys(w[i]), th_pk);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; i++) a[i] = !(__uint_as_float(w[i]) < L) ? 1u : 0u;
        }
        if ((cc + 1) * WAVE * EPL > V) {   // (wave-uniform) the row's last chunk: nothing behind the row's end
            const int n = n_inside<T>(V, cc, lane);
#pragma unroll
            for (int i = 0; i < 4; i++) {
                if (sizeof(T) == 2) a[i] &= (2 * i < n ? 0x0000FFFFu : 0u) | (2 * i + 1 < n ? 0xFFFF0000u : 0u);
                else a[i] = i < n ? a[i] : 0u;
            }
        }
        const uint64_t hit = __ballot((a[0] | a[1] | a[2] | a[3]) != 0u);
        if (hit == 0ull) return;   // most chunks of a long row
        uint32_t pm;   // bit j: token j of this lane's group is listed
        if (sizeof(T) == 2) {
            pm = 0u;
#pragma unroll
            for (int i = 0; i < 4; i++) pm |= ((a[i] | (a[i] >> 15)) & 3u) << (2 * i);
        } else {
            pm = a[0] | (a[1] << 1) | (a[2] << 2) | (a[3] << 3);
        }
        const uint32_t pc = (uint32_t)__popc(pm);
        uint32_t at, tot;
        if (__ballot(pc > 1u) == 0ull) {   // (wave-uniform) one token per lane at most: positions from the ballot
            at = cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(hit >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)hit, 0u));
            tot = (uint32_t)__popcll(hit);
        } else {
            const uint32_t incl = wave_incl_scan(pc);
            tot = last_lane(incl);
            at = cnt + incl - pc;
        }
        const uint32_t first_tok = (uint32_t)((cc * WAVE + lane) * EPL);
        while (pm) {
            const uint32_t j = (uint32_t)__ffs((int)pm) - 1u;
            // the token's logit out of the group, by masks (no branch, no indexed register)
            uint32_t key;
            if (sizeof(T) == 2) {
                const uint32_t m4 = 0u - ((j >> 2) & 1u), m2 = 0u - ((j >> 1) & 1u);
                const uint32_t lo = (w[2] & m4) | (w[0] & ~m4), hi = (w[3] & m4) | (w[1] & ~m4);
                const uint32_t ww = (hi & m2) | (lo & ~m2);
                key = (ww << ((~j & 1u) << 4)) & 0xFFFF0000u;
            } else {
                const uint32_t m2 = 0u - ((j >> 1) & 1u), m1 = 0u - (j & 1u);
                const uint32_t lo = (w[1] & m1) | (w[0] & ~m1), hi = (w[3] & m1) | (w[2] & ~m1);
                key = (hi & m2) | (lo & ~m2);
            }
            if (at < R) {
                s.list_tok[base + at] = first_tok + j;
                s.list_key[base + at] = key;
            }
            // C's histogram, while the key is at hand: the upper key half, counted from the bound (NaNs that
            // slipped through the comparison lie below it and are left out here as they are in C)
            const uint32_t k16 = order_key(key) >> 16;
            if (k16 >= edge_key16) {
                const uint32_t rel = k16 - edge_key16;
                atomicAdd(&s.hist2[rel < (uint32_t)(TOPM_CBINS - 1) ? rel : (uint32_t)(TOPM_CBINS - 1)], 1u);
            }
            at++;
            pm &= pm - 1u;
        }
        cnt += tot;
    };
    if (kept) {
#pragma unroll
        for (int u = 0; u < TOPM_HELD; u++)
            if (c0 + u < c1) list_chunk(r[u], c0 + u);
    } else {
        // the two halves of r take turns: four chunks are asked for again as soon as they have been looked at,
        // from addresses that always lie inside the row, while the other four are looked at
        constexpr int HALF = TOPM_HELD / 2;
        for (int c = c0; c < c1; c += TOPM_HELD) {
#pragma unroll
            for (int h = 0; h < TOPM_HELD; h += HALF) {
#pragma unroll
                for (int u = h; u < h + HALF; u++)
                    if (c + u < c1) list_chunk(r[u], c + u);
#pragma unroll
                for (int u = h; u < h + HALF; u++) r[u] = load_raw_clamped<T, true>(row, V, nc, c + TOPM_HELD + u, lane);
            }
        }
    }
    if (lane == 0) {
        s.seg_a[wave] = cnt < R ? cnt : R;
        if (cnt > R) atomicOr(&s.bc[6], 1u);
    }
    __syncthreads();
    if (s.bc[6] != 0u) return false;
    const uint32_t edge16 = edge_key16;

    // ---- C. the key T of the m-th largest token, from the list.  Thread t answers for the entries t*S .. t*S+S-1
    // of the list, which lie in its own wavefront's part (S = R / 64).
    const int S = LIST / nthreads;
    const uint32_t mine = s.seg_a[wave];
    const uint32_t o0 = (uint32_t)(lane * S);
    const uint32_t n_mine = o0 < mine ? (mine - o0 < (uint32_t)S ? mine - o0 : (uint32_t)S) : 0u;   // entries of this thread
    const uint32_t *lk = s.list_key + base + o0, *lt = s.list_tok + base + o0;
    // Every listed token's key is at or above the edge key (NaNs that slipped through the float comparison
    // aside: they were left out), so the upper 16 key bits, counted from the edge, are small numbers: the one
    // histogram over them that B has filled settles the upper half of T.  A row whose m-th largest token lies
    // further above the bound than the histogram is long (TOPM_CBINS - 1 values of the upper half) goes to the
    // whole-row select.
    pick_digit(s.hist2, TOPM_CBINS, (uint32_t)m, s.wave_tot, s.bc, nthreads);
    if (s.bc[4] == (uint32_t)(TOPM_CBINS - 1)) return false;   // T lies in the overflow bin
    uint32_t hi_part = edge16 + s.bc[4], need = s.bc[5];
    if (sizeof(T) == 4) {   // fp32: the lower half of T, eight bits at a time
        for (int shift = 8; shift >= 0; shift -= 8) {
            __syncthreads();
            for (int i = tid; i < 256; i += nthreads) s.hist[i] = 0u;
            __syncthreads();
            for (uint32_t q = 0; q < n_mine; q++) {
                const uint32_t k = order_key(lk[q]);
                if ((k >> (shift + 8)) == hi_part) atomicAdd(&s.hist[(k >> shift) & 255u], 1u);
            }
            __syncthreads();
            pick_digit(s.hist, 256, need, s.wave_tot, s.bc, nthreads);
            hi_part = (hi_part << 8) | s.bc[4];
            need = s.bc[5];
        }
    }
    // (a key at or above T is at or above the edge: the entries dropped above do not come back below)
    const uint32_t T_key = full_key<T>(hi_part);
    const uint32_t take_eq = need;
    // positions: list order is token order, and threads hold consecutive entries
    uint32_t g = 0, e = 0;
    for (uint32_t q = 0; q < n_mine; q++) {
        const uint32_t k = order_key(lk[q]);
        g += k > T_key ? 1u : 0u;
        e += k == T_key ? 1u : 0u;
    }
    const uint32_t packed = g | (e << 16);   // both counts stay below 2^16 (the list has at most 4096 entries)
    const uint32_t before = block_incl_scan(packed, s.wave_tot, nw) - packed;
    uint32_t gt_before = before & 0xFFFFu, eq_before = before >> 16;
    for (uint32_t q = 0; q < n_mine; q++) {
        const uint32_t k = order_key(lk[q]);
        if (k > T_key) {
            const uint32_t pos = gt_before + (eq_before < take_eq ? eq_before : take_eq);
            if (pos < (uint32_t)m) s.sel[pos] = lt[q];
            gt_before++;
        } else if (k == T_key) {
            if (eq_before < take_eq) {
                const uint32_t pos = gt_before + eq_before;
                if (pos < (uint32_t)m) s.sel[pos] = lt[q];
            }
            eq_before++;
        }
    }
    __syncthreads();
    return true;
}


// ---- mask-only calls, prefixes with at most TOPM_COUNT_MAX children ----
constexpr int TOPM_COUNT_MAX = 8;

// The two thresholds of a child whose logit has the bits `b` (bf16 in the upper half), each in both halves of a
// word: a token at a smaller id comes before the child if its key is above ge, one at a larger id if above gt.
__device__ inline void pk_thresholds(uint32_t b, uint32_t &ge, uint32_t &gt) {
    const uint32_t h = b >> 16;
    const uint32_t key = h ^ ((h & 0x8000u) ? 0xFFFFu : 0x8000u);
    const bool zero = (h & 0x7FFFu) == 0u;
    const uint32_t k_ge = zero ? 0x7FFFu : key, k_gt = zero ? 0x8000u : key;   // -0 and +0 are equal
    const uint32_t t_ge = k_ge ? k_ge - 1u : 0u;
    ge = t_ge | (t_ge << 16);
    gt = k_gt | (k_gt << 16);
}

// Counts, for each of the n children (token tokc[j], logit thr[j], both wave-uniform), the tokens of chunk c that
// come before it in the order of the top-M selection: a larger logit, or an equal one at a smaller token id.
// cnt[j] is this lane's count; for bf16 rows two 16-bit counts side by side (a lane sees at most 4,096 tokens of
// a row), because whole chunks are then counted two tokens at a time on 16-bit keys: three instructions per word
// and child, none of them through a condition register.
template <typename T>
__device__ inline void count_chunk(const uint4 &raw, int V, int c, int lane, int n, const int (&tokc)[TOPM_COUNT_MAX],
                                   const float (&thr)[TOPM_COUNT_MAX], uint32_t (&cnt)[TOPM_COUNT_MAX]) {
    constexpr int EPL = KeyChunk<T>::EPL;
    constexpr bool PACKED = sizeof(T) == 2;
    const int first = c * WAVE * EPL;            // the chunk holds tokens first .. first + 64 * EPL - 1
    const int g = first + lane * EPL;
    const bool ragged = first + WAVE * EPL > V;  // (wave-uniform) the row ends inside this chunk
    float x[EPL];
    uint32_t keys[4] = {0u, 0u, 0u, 0u};
    if (PACKED) {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; i++) keys[i] = pk_keys(w[i]);
        if (ragged) {                            // tokens behind the row's end get the lowest key: above no threshold
#pragma unroll
            for (int i = 0; i < 4; i++)
                keys[i] &= (g + 2 * i < V ? 0x0000FFFFu : 0u) | (g + 2 * i + 1 < V ? 0xFFFF0000u : 0u);
        }
    } else {
        unpack_vals<T>(raw, x);
        if (ragged) {
#pragma unroll
            for (int e = 0; e < EPL; e++)
                if (g + e >= V) x[e] = -INFINITY;    // never before a child: compared with ">" (they follow every token)
        }
    }
#pragma unroll
    for (int j = 0; j < TOPM_COUNT_MAX; j++) {
        if (j >= n) break;                       // (wave-uniform)
        const float t = thr[j];
        const bool before = first + WAVE * EPL <= tokc[j];   // every token of the chunk has a smaller id: ties count
        const bool after = first > tokc[j];                   // every token has a larger id: ties do not count
        uint32_t k = 0;
        if (__builtin_expect(before || after, 1)) {   // (all chunks of a row but one per child: the rest is kept out of the loop's way)
            if (PACKED) {
                uint32_t ge, gt;
                pk_thresholds(__float_as_uint(t), ge, gt);
                const uint32_t th = before ? ge : gt;
#pragma unroll
                for (int i = 0; i < 4; i++) k += pk_above(keys[i], th);
            } else if (before) {
#pragma unroll
                for (int e = 0; e < EPL; e++) k += x[e] >= t ? 1u : 0u;
            } else {
#pragma unroll
                for (int e = 0; e < EPL; e++) k += x[e] > t ? 1u : 0u;
            }
        } else if (PACKED) {                     // the child's own chunk (one per child and row): the threshold
                                                 // of each half follows from which side of the child its token lies on
            uint32_t ge, gt;
            pk_thresholds(__float_as_uint(t), ge, gt);
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint32_t lo = g + 2 * i < tokc[j] ? ge : gt, hi = g + 2 * i + 1 < tokc[j] ? ge : gt;
                k += pk_above(keys[i], (lo & 0x0000FFFFu) | (hi & 0xFFFF0000u));
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPL; e++) k += (x[e] > t || (x[e] == t && g + e < tokc[j])) ? 1u : 0u;
        }
        cnt[j] += k;
    }
}

// The mask row of a prefix with n <= TOPM_COUNT_MAX children (entries cb .. cb + n - 1), restricted to the m most
// probable tokens.  Every thread of the workgroup calls; r holds the wavefront's first TOPM_HELD chunks; tot[] was
// cleared before the last barrier.
template <typename T>
__device__ inline void count_children(const IndexView &ix, const T *__restrict__ row, int V, int nc, int c0, int c1,
                                      int m, uint32_t cb, int n, uint4 (&r)[TOPM_HELD], uint32_t *tot,
                                      uint32_t *__restrict__ out, int n_words, int lane, int nthreads) {
    // child j in lane j: its token and that token's logit
    uint32_t ctok = 0u;
    float cthr = 0.f;
    if (lane < n) {
        ctok = ix.ent[cb + (uint32_t)lane].tok & PPV_NODE_TOKEN;
        ctok = ctok < (uint32_t)V ? ctok : 0u;   // (always inside for an index that was built or loaded)
        cthr = __uint_as_float(KeyChunk<T>::bits_of(row, (int)ctok));
    }
    int tokc[TOPM_COUNT_MAX];
    float thr[TOPM_COUNT_MAX];
    uint32_t cnt[TOPM_COUNT_MAX];
#pragma unroll
    for (int j = 0; j < TOPM_COUNT_MAX; j++) {
        tokc[j] = (int)lane_value(ctok, j);
        thr[j] = __uint_as_float(lane_value(__float_as_uint(cthr), j));
        cnt[j] = 0u;
    }
    // the pairs of r take turns: a pair of chunks is asked for again as soon as it has been counted, while the
    // other three pairs are counted or on their way
    for (int c = c0; c < c1; c += TOPM_HELD) {
#pragma unroll
        for (int h = 0; h < TOPM_HELD; h += 2) {
#pragma unroll
            for (int u = h; u < h + 2; u++)
                if (c + u < c1) count_chunk<T>(r[u], V, c + u, lane, n, tokc, thr, cnt);
#pragma unroll
            for (int u = h; u < h + 2; u++) r[u] = load_raw_clamped<T>(row, V, nc, c + TOPM_HELD + u, lane);
        }
    }
#pragma unroll
    for (int j = 0; j < TOPM_COUNT_MAX; j++) {
        if (j >= n) break;
        const uint32_t w = wave_sum(sizeof(T) == 2 ? (cnt[j] & 0xFFFFu) + (cnt[j] >> 16) : cnt[j]);
        if (lane == 0) atomicAdd(&tot[j], w);
    }
    __syncthreads();
    bool in[TOPM_COUNT_MAX];
#pragma unroll
    for (int j = 0; j < TOPM_COUNT_MAX; j++) in[j] = j < n && tot[j] < (uint32_t)m;
    auto word = [&](int i) {
        uint32_t w = 0u;
#pragma unroll
        for (int j = 0; j < TOPM_COUNT_MAX; j++)
            if (in[j] && (tokc[j] >> 5) == i) w |= 1u << (tokc[j] & 31);
        return w;
    };
    if ((n_words & 3) == 0 && (((uintptr_t)out) & 15u) == 0) {
        for (int i = (int)threadIdx.x; i < (n_words >> 2); i += nthreads)
            ((uint4 *)out)[i] = make_uint4(word(4 * i), word(4 * i + 1), word(4 * i + 2), word(4 * i + 3));
    } else {
        for (int i = (int)threadIdx.x; i < n_words; i += nthreads) out[i] = word(i);
    }
}

template <typename T, int LIST>
__global__ __launch_bounds__(TOPM_WAVES *WAVE) void topm_kernel(IndexView ix, const int32_t *__restrict__ prefixes,
                                                                int32_t stride, const int32_t *__restrict__ lens,
                                                                const T *__restrict__ logits, int64_t row_stride, int M,
                                                                int force_streaming, int32_t *__restrict__ top_ids,
                                                                uint8_t *__restrict__ mask_V,
                                                                uint32_t *__restrict__ mask) {
    constexpr int EPL = KeyChunk<T>::EPL;
    extern __shared__ __align__(16) uint32_t smem[];  // max(TOPM_BINS, n_words) words, then heavy_min words for kids
    uint32_t *img = smem;                             // [n_words] the row of the mask, once the histogram is done with
    __shared__ uint32_t list_tok[LIST], list_key[LIST];
    __shared__ uint32_t hist2[TOPM_CBINS], hist3[32];
    __shared__ uint32_t sel[PPV_TOPM_MAX];
    __shared__ uint32_t seg_a[TOPM_WAVES], seg_b[TOPM_WAVES], wave_tot[TOPM_WAVES];
    __shared__ uint32_t bc[8];
    const TopmLds lds = {smem, hist3, hist2, list_tok, list_key, sel, seg_a, seg_b, wave_tot, bc};
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const int nthreads = blockDim.x, nw = nthreads / WAVE;
    const int V = ix.vocab, n_words = ix.n_words;
    const int m = M < V ? M : V;                      // candidates of this row
    // the tokens of the prefix's children, when they are listed (not a heavy prefix: at most heavy_min of them)
    uint32_t *kids = smem + (n_words > TOPM_BINS ? n_words : TOPM_BINS);
    const T *row = logits + (size_t)b * (size_t)row_stride;

    // this wavefront's contiguous share of the row, in chunks of one 16-byte load per lane
    const int nc = (V + WAVE * EPL - 1) / (WAVE * EPL);
    const int cpw = (nc + nw - 1) / nw;
    const int c0 = wave * cpw, c1 = (c0 + cpw < nc) ? c0 + cpw : nc;

    const bool listed = force_streaming != 1 && nthreads * TOPM_SLOTS >= LIST && nthreads <= LIST;
    // a caller that asks for the mask alone: prefixes with few children are settled by counting (see count_children)
    const bool counting = force_streaming == 0 && !top_ids && !mask_V;
    uint4 r[TOPM_HELD];
    if (listed || counting) {   // in flight while the prefix is located
        load_chunks<T, true>(row, V, nc, c0, lane, r);
        if (cpw > 4) load_chunks<T, true>(row, V, nc, c0 + 4, lane, r + 4);   // (uniform; a short row has no second half)
    }
    if (counting && tid < TOPM_COUNT_MAX) seg_a[tid] = 0u;
    if (listed) {   // what the list select starts from
        for (int i = tid; i < TOPM_BINS; i += nthreads) smem[i] = 0u;
        for (int i = tid; i < TOPM_CBINS; i += nthreads) hist2[i] = 0u;
        if (tid < 32) hist3[tid] = 0u;
        if (tid == 0) bc[6] = 0u;
    }
    if (wave == 0) {   // the part every candidate row shares: locate the prefix once
        const int32_t mine = first_tokens(prefixes + (size_t)b * (size_t)stride, stride, lane);
        int t = lens[b];
        t = t < 0 ? 0 : (t > stride ? stride : t);
        const Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, mine, t, lane);
        if (lane == 0) {
            bc[0] = w.node;
            bc[1] = w.found ? 1u : 0u;
            bc[2] = w.found ? w.cb : 0u;
            bc[3] = w.found ? w.ce : 0u;
        }
    }
    __syncthreads();   // the walk's verdict
    const uint32_t node = bc[0];
    const bool found = bc[1] != 0u;
    const uint32_t cb = bc[2], ce = bc[3];
    const int n = (int)(ce - cb);
    if (counting) {
        uint32_t *out = mask + (size_t)b * (size_t)n_words;
        if (!found || n == 0) {   // no continuation at all: the row of the mask is empty, the logits do not matter
            if ((n_words & 3) == 0 && (((uintptr_t)mask) & 15u) == 0) {
                for (int i = tid; i < (n_words >> 2); i += nthreads) ((uint4 *)out)[i] = make_uint4(0u, 0u, 0u, 0u);
            } else {
                for (int i = tid; i < n_words; i += nthreads) out[i] = 0u;
            }
            return;
        }
        // Counting pays where the selection would hold the row in registers anyway (it skips the bound, the list and
        // the cut: 9 against 12 us at V = 32k) and where the selection would read part of the row twice; a long row
        // that the selection reads once (bound from its first chunks alone, see select_listed) is no faster counted
        // (V = 256k: 120 against 117 us).
        const bool select_reads_once = listed && (cpw <= TOPM_HELD || (long long)m * cpw <= 4ll * LIST);
        if (n <= TOPM_COUNT_MAX && (uint32_t)n <= ix.heavy_min && (cpw <= TOPM_HELD || !select_reads_once)) {
            count_children<T>(ix, row, V, nc, c0, c1, m, cb, n, r, seg_a, out, n_words, lane, nthreads);
            return;
        }
    }
    // the children's tokens go to LDS while the row is on its way: the candidates are then looked up there
    const bool kids_listed = found && (uint32_t)n <= ix.heavy_min;
    if (kids_listed)
        for (int i = tid; i < n; i += nthreads) kids[i] = ix.ent[cb + (uint32_t)i].tok & PPV_NODE_TOKEN;
    const uint32_t slot = (found && (uint32_t)n > ix.heavy_min) ? heavy_slot_of(ix, node) : PPV_NO_SLOT;
    // ---- select
    bool done = false;
    if (listed) done = select_listed<T, LIST>(row, V, c0, c1, m, lds, lane, wave, nthreads, r);
    if (!done) select_streaming<T>(row, V, c0, c1, m, lds, lane, wave, nthreads);
    for (int i = tid; i < n_words; i += nthreads) img[i] = 0u;   // the histogram's LDS becomes the mask row
    __syncthreads();

    // ---- verify: one candidate per thread
    const uint32_t *image = ix.heavy_bits + (size_t)(slot != PPV_NO_SLOT ? slot : 0u) * (size_t)n_words;
    for (int i = tid; i < M; i += nthreads) {
        int32_t t = -1;
        uint32_t ok = 0;
        if (i < m && sel[i] < (uint32_t)V) {
            t = (int32_t)sel[i];
            if (slot != PPV_NO_SLOT) {
                ok = (image[t >> 5] >> (t & 31)) & 1u;
            } else if (kids_listed) {   // first child whose token is not below t
                int lo = 0, hi = n;
                while (lo < hi) {
                    const int mid = lo + (hi - lo) / 2;
                    if (kids[mid] < (uint32_t)t) lo = mid + 1;
                    else hi = mid;
                }
                ok = (lo < n && kids[lo] == (uint32_t)t) ? 1u : 0u;
            }
            if (ok) atomicOr(&img[t >> 5], 1u << (t & 31));
        }
        if (top_ids) top_ids[(size_t)b * (size_t)M + i] = t;
        if (mask_V) mask_V[(size_t)b * (size_t)M + i] = (uint8_t)ok;
    }
    __syncthreads();

    // ---- extend
    uint32_t *out = mask + (size_t)b * (size_t)n_words;
    if ((n_words & 3) == 0 && (((uintptr_t)mask) & 15u) == 0) {
        for (int i = tid; i < (n_words >> 2); i += nthreads) ((uint4 *)out)[i] = ((const uint4 *)img)[i];
    } else {
        for (int i = tid; i < n_words; i += nthreads) out[i] = img[i];
    }
}

// wavefronts per row: a power of two, at most one per chunk; many for a small batch (latency), few for a large one
int topm_waves(int V, ppv_dtype dt, int B) {
    const int per = (dt == PPV_F32 ? 4 : 8) * WAVE;
    const int nc = (V + per - 1) / per;
    int cap = B <= 512 ? 8 : 4;   // measured at V = 32k, M = 50: B = 256: 11.1 / 11.9 us with 8 / 16; B = 4,096: 63 / 90 / 169 us with 4 / 8 / 16
    // long rows (bf16, us per call with 4 / 8 / 16 wavefronts, M = 50 and 1,000): V = 128k: B = 128: 36 / 23 / 19 and 48 / 32 / 23,
    // B = 1,024: 75 / 66 / 83 and 120 / 99 / 102; V = 256k: B = 128: 60 / 37 / 27 and 78 / 49 / 42, B = 1,024: 118 / 117 / 143 (M = 50)
    if (nc <= 4 && B > 512) cap = 2;   // 4 KB rows (V = 1,024 fp32), B = 4,096, M = 50 / 1,000: 39 / 85 us with 1, 32 / 57 with 2, 36 / 64 with 4
    if (nc >= 128 && B <= 256) cap = 16;
    if (nc >= 128 && B <= 2048 && cap < 8) cap = 8;
    if (const int v = ppv_tuning(PPV_TUNE_TOPM_WAVES)) cap = v < TOPM_WAVES ? v : TOPM_WAVES;   // tuning aid (0: the table above)
    int nw = 1;
    while (nw * 2 <= cap && nw * 2 <= nc) nw <<= 1;
    return nw;
}

}  // namespace

extern "C" ppv_status ppv_topm_mask(const ppv_index_t *ix, const int32_t *prefixes, int32_t prefix_stride,
                                    const int32_t *lens, const void *logits, ppv_dtype dt, int64_t row_stride,
                                    int32_t M, int32_t B, int32_t *top_ids, uint8_t *mask_V, uint32_t *mask,
                                    void *stream) {
    if (!ix || B < 0 || prefix_stride < 0 || M < 1) return PPV_EINVAL;
    if (M > PPV_TOPM_MAX) return PPV_ERANGE;
    if (B == 0) return PPV_OK;
    if (!prefixes || !lens || !mask || !logits) return PPV_EINVAL;
    if (dt != PPV_F32 && dt != PPV_BF16) return PPV_EINVAL;
    const int V = ix->view.vocab;
    const int64_t per16 = (dt == PPV_F32) ? 4 : 8;
    if (row_stride < V || row_stride % per16 != 0 || ((uintptr_t)logits & 15u) != 0) return PPV_EINVAL;
    const int threads = topm_waves(V, dt, B) * WAVE;
    // testing aid: PPV_TUNE_TOPM_STREAMING = 1 sends every row through the whole-row radix select; 2 keeps the usual
    // select but takes the top M also where counting would do (mask-only calls)
    const int force_streaming = ppv_tuning(PPV_TUNE_TOPM_STREAMING);
    const size_t lds = ((size_t)(ix->view.n_words > TOPM_BINS ? ix->view.n_words : TOPM_BINS) + ix->view.heavy_min) * sizeof(uint32_t);
    const dim3 grid((unsigned)B), block(threads);
    hipStream_t hs = (hipStream_t)stream;
#define PPV_LAUNCH_TOPM(T, LIST)                                                                                      \
    hipLaunchKernelGGL((topm_kernel<T, LIST>), grid, block, lds, hs, ix->view, prefixes, prefix_stride, lens,          \
                       (const T *)logits, row_stride, M, force_streaming, top_ids, mask_V, mask)
    // a few hundred tokens reach the bound when M is small and the row not too long (the bound's bin holds a share
    // of the row): then a quarter of the LDS does, and more rows fit a compute unit
    const bool small_list = M <= 128 && V <= 65536;
    if (dt == PPV_F32) {
        if (small_list) PPV_LAUNCH_TOPM(float, TOPM_LIST_SMALL);
        else PPV_LAUNCH_TOPM(float, TOPM_LIST_BIG);
    } else {
        if (small_list) PPV_LAUNCH_TOPM(uint16_t, TOPM_LIST_SMALL);
        else PPV_LAUNCH_TOPM(uint16_t, TOPM_LIST_BIG);
    }
#undef PPV_LAUNCH_TOPM
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}
