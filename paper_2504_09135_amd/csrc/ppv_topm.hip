// Algorithm 2 with M candidates (the variant the paper ran with M = 50): per row, the M tokens of
// largest probability, one verification per candidate row a + [t_i], and the extended mask.
//
// One workgroup per row.
//   select   P = softmax(logits) is increasing in the logit, so the top M are found on the logits'
//            bit patterns: an order-preserving 32-bit key per token, then a radix select from the
//            most significant digit down (11 + 11 + 10 bits for fp32; bf16 keys are settled after
//            the first two digits).  Each digit is one pass over the row with a histogram in LDS;
//            the passes after the first find the row in cache.  Equal logits are taken in
//            increasing token id, so the set is unique.
//   gather   one more pass writes the selected tokens in increasing token id (each wavefront owns a
//            contiguous part of the row, so positions come from prefix counts, not from atomics).
//   verify   the M candidate rows share their first |a| tokens, so the prefix is located once
//            (the same walk the full-vocabulary mask uses) and each candidate then needs one
//            binary search for its last token among the prefix's children -- or one bit test in
//            the ready-made image of a heavy prefix.  One thread per candidate.
//   extend   the mask row is assembled in LDS and written with whole words.
// Nothing here is a dense contraction; the row is read from HBM once (64 KB at V = 32k, bf16).
#include <cstdlib>

#include "ppv_device.h"
#include "ppv_internal.h"
#include "ppv_walk.h"

namespace {

constexpr int TOPM_BINS = 2048;   // 11-bit digits
constexpr int TOPM_WAVES = 16;

// Bit pattern -> key with the same order as the float value (-0 and +0 share a key).
__device__ inline uint32_t order_key(uint32_t bits) {
    if (bits == 0x80000000u) bits = 0u;
    return bits ^ ((uint32_t)((int32_t)bits >> 31) | 0x80000000u);
}

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

template <typename T>
__global__ __launch_bounds__(TOPM_WAVES *WAVE) void topm_kernel(IndexView ix, const int32_t *__restrict__ prefixes,
                                                                int32_t stride, const int32_t *__restrict__ lens,
                                                                const T *__restrict__ logits, int64_t row_stride, int M,
                                                                int32_t *__restrict__ top_ids,
                                                                uint8_t *__restrict__ mask_V,
                                                                uint32_t *__restrict__ mask) {
    constexpr int EPL = KeyChunk<T>::EPL;
    extern __shared__ __align__(16) uint32_t img[];   // [n_words] the row of the mask
    __shared__ uint32_t hist[TOPM_BINS];
    __shared__ uint32_t sel[PPV_TOPM_MAX];
    __shared__ uint32_t seg_gt[TOPM_WAVES], seg_eq[TOPM_WAVES], wave_tot[TOPM_WAVES];
    __shared__ uint32_t bc[8];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const int nthreads = blockDim.x, nw = nthreads / WAVE;
    const int V = ix.vocab, n_words = ix.n_words;
    const int m = M < V ? M : V;                      // candidates of this row
    const T *row = logits + (size_t)b * (size_t)row_stride;

    if (wave == 0) {   // the part every candidate row shares: locate the prefix once
        int t = lens[b];
        t = t < 0 ? 0 : (t > stride ? stride : t);
        const Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, t, lane);
        if (lane == 0) {
            bc[0] = w.node;
            bc[1] = w.found ? 1u : 0u;
            bc[2] = w.found ? w.cb : 0u;
            bc[3] = w.found ? w.ce : 0u;
        }
    }
    for (int i = tid; i < n_words; i += nthreads) img[i] = 0u;

    // this wavefront's contiguous share of the row, in chunks of one 16-byte load per lane
    const int nc = (V + WAVE * EPL - 1) / (WAVE * EPL);
    const int cpw = (nc + nw - 1) / nw;
    const int c0 = wave * cpw, c1 = (c0 + cpw < nc) ? c0 + cpw : nc;

    // ---- select: the key T of the m-th largest token, digit by digit
    const int n_pass = sizeof(T) == 4 ? 3 : 2;
    uint32_t hi_part = 0;      // digits settled so far, as the key's leading bits
    uint32_t need = (uint32_t)m;   // how many tokens are still to be taken among those that match hi_part
    for (int pass = 0; pass < n_pass; pass++) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const int bins = pass == 2 ? 1024 : 2048;
        for (int i = tid; i < TOPM_BINS; i += nthreads) hist[i] = 0u;
        __syncthreads();
        for (int c = c0; c < c1; c++) {
            uint32_t k[EPL];
            const int n = load_keys<T>(row, V, c, lane, k);
#pragma unroll
            for (int j = 0; j < EPL; j++) {
                const bool match = pass == 0 || (k[j] >> (pass == 1 ? 21 : 10)) == hi_part;
                if (j < n && match) atomicAdd(&hist[(k[j] >> shift) & (uint32_t)(bins - 1)], 1u);
            }
        }
        __syncthreads();
        // bins from the top: the digit d with  #(digit > d) < need <= #(digit >= d)
        const int per = bins / nthreads > 0 ? bins / nthreads : 1;   // consecutive bins per thread, descending
        uint32_t s = 0;
        const int top_bin = bins - 1 - tid * per;
        if (top_bin >= 0)
            for (int j = 0; j < per; j++) s += hist[top_bin - j];
        const uint32_t incl = block_incl_scan(s, wave_tot, nw);
        if (top_bin >= 0 && incl - s < need && need <= incl) {   // exactly one thread
            uint32_t acc = incl - s;
            for (int j = 0; j < per; j++) {
                const uint32_t h = hist[top_bin - j];
                if (acc + h >= need) {
                    bc[4] = (uint32_t)(top_bin - j);
                    bc[5] = need - acc;
                    break;
                }
                acc += h;
            }
        }
        __syncthreads();
        hi_part = (hi_part << (pass == 2 ? 10 : 11)) | bc[4];
        need = bc[5];
        __syncthreads();
    }
    // bf16: the low 16 bits of a key follow from its sign, so two digits settle the whole key
    const uint32_t T_key = sizeof(T) == 4 ? hi_part : ((hi_part << 10) | ((hi_part >> 21) & 1u ? 0u : 0x3FFu));
    const uint32_t take_eq = need;   // of the tokens whose key equals T_key, the first take_eq in token order

    // ---- gather in token order
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
        seg_gt[wave] = n_gt;
        seg_eq[wave] = n_eq;
    }
    __syncthreads();
    uint32_t gt_base = 0, eq_base = 0;   // tokens of either kind in the wavefronts before this one
    for (int w = 0; w < nw; w++)
        if (w < wave) {
            gt_base += seg_gt[w];
            eq_base += seg_eq[w];
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
                if (pos < (uint32_t)m) sel[pos] = first_tok + j;
                gt_before++;
            } else if (k[j] == T_key) {
                if (eq_before < take_eq) {
                    const uint32_t pos = gt_before + eq_before;
                    if (pos < (uint32_t)m) sel[pos] = first_tok + j;
                }
                eq_before++;
            }
        }
        gt_base += last_lane(gi);
        eq_base += last_lane(ei);
    }
    __syncthreads();

    // ---- verify: one candidate per thread
    const uint32_t node = bc[0];
    const bool found = bc[1] != 0u;
    const uint32_t cb = bc[2], ce = bc[3];
    const uint32_t slot = (found && ce - cb > ix.heavy_min) ? heavy_slot_of(ix, node) : PPV_NO_SLOT;
    const uint32_t *image = ix.heavy_bits + (size_t)(slot != PPV_NO_SLOT ? slot : 0u) * (size_t)n_words;
    for (int i = tid; i < M; i += nthreads) {
        int32_t t = -1;
        uint32_t ok = 0;
        if (i < m) {
            t = (int32_t)sel[i];
            if (slot != PPV_NO_SLOT) {
                ok = (image[t >> 5] >> (t & 31)) & 1u;
            } else if (found) {   // first child whose token is not below t
                uint32_t lo = cb, hi = ce;
                while (lo < hi) {
                    const uint32_t mid = lo + (hi - lo) / 2;
                    if ((ix.ent[mid].tok & PPV_NODE_TOKEN) < (uint32_t)t) lo = mid + 1;
                    else hi = mid;
                }
                ok = (lo < ce && (ix.ent[lo].tok & PPV_NODE_TOKEN) == (uint32_t)t) ? 1u : 0u;
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
    const int cap = B <= 512 ? TOPM_WAVES : (B <= 1024 ? 8 : 4);
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
    const size_t lds = (size_t)ix->view.n_words * sizeof(uint32_t);
    if (dt == PPV_F32)
        hipLaunchKernelGGL(topm_kernel<float>, dim3((unsigned)B), dim3(threads), lds, (hipStream_t)stream, ix->view,
                           prefixes, prefix_stride, lens, (const float *)logits, row_stride, M, top_ids, mask_V, mask);
    else
        hipLaunchKernelGGL(topm_kernel<uint16_t>, dim3((unsigned)B), dim3(threads), lds, (hipStream_t)stream, ix->view,
                           prefixes, prefix_stride, lens, (const uint16_t *)logits, row_stride, M, top_ids, mask_V,
                           mask);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}
