// Per-step kernels: prefix walk (rank range), next-token scatter (packed mask), masked
// log-softmax + inverse-CDF sample, and the fused decode step.  gfx950, wave64.
#include "ppv_internal.h"

namespace {

constexpr int WAVE = 64;
constexpr int MASK_THREADS = 256;    // workgroup of the mask kernel: one row per workgroup
constexpr int SAMPLE_THREADS = 256;  // workgroup of the sample kernel: one row per workgroup

// ------------------------------------------------------------------------------------------
// Prefix walk, one wavefront per prefix (Section 3.2 "Parallel Verification": the search that
// locates a prefix in sorted S; here it descends the per-depth arrays, one 64-way search among
// the children of the current prefix per token, instead of log2|S| probes of whole rows).
// All 64 lanes call it with the same arguments; every result is wave-uniform.
struct Walk {
    uint32_t node;   // the prefix's entry in the per-depth arrays (valid when found)
    uint32_t lo, hi; // rank range in sorted S; lo == hi == insertion rank when not found
    bool found;      // the prefix is a prefix of at least one member
};

__device__ inline uint32_t wave_lower_bound(const uint32_t *__restrict__ a, uint32_t begin, uint32_t end,
                                            uint32_t key, int lane, bool *match) {
    // first position in [begin, end) whose value is >= key; values are strictly increasing
    uint32_t lo = begin, hi = end;
    while (hi - lo > (uint32_t)WAVE) {
        uint32_t n = hi - lo;
        uint32_t step = (n + WAVE - 1) / WAVE;
        uint32_t p = (uint32_t)(lane + 1) * step;
        if (p > n) p = n;
        uint32_t v = a[lo + p - 1];                       // 64 pivots, the last one is a[hi-1]
        int c = __popcll(__ballot(v < key));              // pivots below the key
        if (c == WAVE) { lo = hi; break; }                // everything is below the key
        uint32_t nlo = lo + (uint32_t)c * step;
        uint32_t nhi = lo + (uint32_t)(c + 1) * step;
        if (nhi > hi) nhi = hi;
        lo = nlo;
        hi = nhi;
    }
    bool in = lo + (uint32_t)lane < hi;
    uint32_t v = in ? a[lo + lane] : 0xFFFFFFFFu;
    int c = __popcll(__ballot(in && v < key));
    *match = __ballot(in && v == key) != 0ull;
    return lo + (uint32_t)c;
}

__device__ inline Walk walk_prefix(const IndexView &ix, const int32_t *__restrict__ prefix, int t, int lane) {
    Walk w;
    w.node = 0;
    w.lo = 0;
    w.hi = ix.n_rows;
    w.found = true;
    for (int i = 0; i < t; i++) {
        uint32_t key = (uint32_t)prefix[i];
        uint32_t cb = ix.child_off[w.node], ce = ix.child_off[w.node + 1];
        bool match;
        uint32_t j = wave_lower_bound(ix.node_tok, cb, ce, key, lane, &match);
        if (!match) {
            // every member below child j sorts before the prefix; if there is no such child the
            // prefix sorts after the whole range of the current node
            uint32_t rank = (j < ce) ? ix.node_lo[j] : w.hi;
            w.lo = rank;
            w.hi = rank;
            w.found = false;
            return w;
        }
        w.node = j;
        w.lo = ix.node_lo[j];
        w.hi = ix.node_hi[j];
    }
    return w;
}

// the prefix itself is a member iff its first row is not the first row of its first child
__device__ inline bool node_is_member(const IndexView &ix, const Walk &w, int t) {
    if (!w.found || t == 0) return false;
    uint32_t cb = ix.child_off[w.node], ce = ix.child_off[w.node + 1];
    return cb == ce || ix.node_lo[cb] != w.lo;
}

// ------------------------------------------------------------------------------------------
// Next-token scatter: OR the children's tokens of the reached node into a bit image in LDS.
// Called by the whole workgroup; img has n_words words and must already be zero.
__device__ inline void scatter_children(const IndexView &ix, uint32_t node, uint32_t *img, int tid, int nthreads) {
    uint32_t cb = ix.child_off[node], ce = ix.child_off[node + 1];
    for (uint32_t i = cb + (uint32_t)tid; i < ce; i += (uint32_t)nthreads) {
        uint32_t v = ix.node_tok[i];
        atomicOr(&img[v >> 5], 1u << (v & 31u));
    }
}

__global__ __launch_bounds__(MASK_THREADS) void mask_kernel(IndexView ix, const int32_t *__restrict__ prefixes,
                                                            int32_t stride, const int32_t *__restrict__ lens,
                                                            uint32_t *__restrict__ mask, uint32_t *__restrict__ range_lo,
                                                            uint32_t *__restrict__ range_hi,
                                                            uint8_t *__restrict__ member, int n_words) {
    extern __shared__ __align__(16) uint32_t smem[];
    uint32_t *img = smem;                 // [n_words]
    uint32_t *bc = smem + n_words;        // [2]: node, found
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    for (int i = tid; i < n_words; i += MASK_THREADS) img[i] = 0u;
    if (wave == 0) {
        int t = lens[b];
        t = t < 0 ? 0 : (t > stride ? stride : t);
        Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, t, lane);
        if (lane == 0) {
            bc[0] = w.node;
            bc[1] = w.found ? 1u : 0u;
            if (range_lo) range_lo[b] = w.lo;
            if (range_hi) range_hi[b] = w.hi;
            if (member) member[b] = node_is_member(ix, w, t) ? 1 : 0;
        }
    }
    __syncthreads();
    if (bc[1]) scatter_children(ix, bc[0], img, tid, MASK_THREADS);
    __syncthreads();
    uint32_t *out = mask + (size_t)b * (size_t)n_words;
    for (int i = tid; i < n_words; i += MASK_THREADS) out[i] = img[i];
}

// ------------------------------------------------------------------------------------------
// Masked log-softmax + inverse-CDF sample of one row by one workgroup.
template <typename T> __device__ inline float load_logit(const T *p, int v);
template <> __device__ inline float load_logit<float>(const float *p, int v) { return p[v]; }
template <> __device__ inline float load_logit<uint16_t>(const uint16_t *p, int v) {
    return __uint_as_float(((uint32_t)p[v]) << 16);  // bf16 -> fp32 is exact
}

struct RowResult {
    int32_t id;
    float logZ_valid, logZ_all;
};

template <typename Op>
__device__ inline double block_reduce(double x, double *red, int tid, Op op) {
    // wave reduction by shuffles, then across the waves through LDS; fixed order => deterministic
    for (int o = WAVE / 2; o > 0; o >>= 1) x = op(x, __shfl_xor(x, o, WAVE));
    __syncthreads();
    if ((tid & (WAVE - 1)) == 0) red[tid / WAVE] = x;
    __syncthreads();
    double r = red[0];
    for (int w = 1; w < SAMPLE_THREADS / WAVE; w++) r = op(r, red[w]);
    return r;
}

// mask_bit(v) tells whether token v is valid; scratch: SAMPLE_THREADS doubles + 8 doubles + 4 ints
template <typename T, typename MaskFn>
__device__ inline RowResult sample_row(const T *__restrict__ row, int V, MaskFn mask_bit, float u, double *scratch,
                                       int tid) {
    double *red = scratch;                       // [SAMPLE_THREADS/WAVE]
    double *chunk_sum = scratch + 8;             // [SAMPLE_THREADS]
    int *ibc = (int *)(scratch + 8 + SAMPLE_THREADS);
    auto fmaxd = [](double a, double b) { return a > b ? a : b; };
    auto addd = [](double a, double b) { return a + b; };

    // pass 1: maxima over all tokens and over valid tokens
    float m_all = -INFINITY, m_val = -INFINITY;
    for (int v = tid; v < V; v += SAMPLE_THREADS) {
        float l = load_logit<T>(row, v);
        m_all = fmaxf(m_all, l);
        if (mask_bit(v)) m_val = fmaxf(m_val, l);
    }
    m_all = (float)block_reduce((double)m_all, red, tid, fmaxd);
    m_val = (float)block_reduce((double)m_val, red, tid, fmaxd);

    // pass 2: sum over all tokens; valid weights are summed per contiguous chunk in token order
    double z_all = 0.0;
    for (int v = tid; v < V; v += SAMPLE_THREADS) z_all += (double)expf(load_logit<T>(row, v) - m_all);
    z_all = block_reduce(z_all, red, tid, addd);

    RowResult r;
    r.logZ_all = m_all + (float)log(z_all);
    if (m_val == -INFINITY) {  // empty mask (or every valid logit is -inf)
        r.id = -1;
        r.logZ_valid = -INFINITY;
        return r;
    }
    const int chunk = (V + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
    const int v0 = tid * chunk, v1 = min(V, v0 + chunk);
    double mine = 0.0;
    for (int v = v0; v < v1; v++)
        if (mask_bit(v)) mine += (double)expf(load_logit<T>(row, v) - m_val);
    chunk_sum[tid] = mine;
    __syncthreads();
    if (tid == 0) {
        double z = 0.0;
        for (int i = 0; i < SAMPLE_THREADS; i++) z += chunk_sum[i];
        double tau = (double)u * z, c = 0.0;
        int pick = -1, last = -1;
        for (int i = 0; i < SAMPLE_THREADS; i++) {
            if (chunk_sum[i] > 0.0) last = i;
            if (c + chunk_sum[i] > tau) { pick = i; break; }
            c += chunk_sum[i];
        }
        if (pick < 0) { pick = last; c = -1.0; }  // rounding: take the last positive chunk's last token
        red[0] = z;
        red[1] = tau;
        red[2] = c;
        ibc[0] = pick;
    }
    __syncthreads();
    const double z_val = red[0], tau = red[1], base = red[2];
    const int pick = ibc[0];
    __syncthreads();
    if (tid == pick) {
        double c = base < 0.0 ? 0.0 : base;
        int id = -1, last = -1;
        for (int v = v0; v < v1; v++) {
            if (!mask_bit(v)) continue;
            double w = (double)expf(load_logit<T>(row, v) - m_val);
            c += w;
            if (w > 0.0) last = v;
            if (base >= 0.0 && c > tau) { id = v; break; }
        }
        ibc[1] = id >= 0 ? id : last;
    }
    __syncthreads();
    r.id = ibc[1];
    r.logZ_valid = (float)(((double)m_val + log(z_val)) - ((double)m_all + log(z_all)));
    return r;
}

constexpr int SAMPLE_SCRATCH_DOUBLES = 8 + SAMPLE_THREADS + 2;

template <typename T>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_kernel(const T *__restrict__ logits, int64_t row_stride,
                                                                const uint32_t *__restrict__ mask,
                                                                const float *__restrict__ uniforms, int V, int n_words,
                                                                int32_t *__restrict__ ids,
                                                                float *__restrict__ logZ_valid,
                                                                float *__restrict__ logZ_all) {
    __shared__ double scratch[SAMPLE_SCRATCH_DOUBLES];
    const int b = blockIdx.x, tid = threadIdx.x;
    const uint32_t *mrow = mask + (size_t)b * (size_t)n_words;
    auto bit = [=](int v) { return (mrow[v >> 5] >> (v & 31)) & 1u; };
    RowResult r = sample_row<T>(logits + (size_t)b * (size_t)row_stride, V, bit, uniforms[b], scratch, tid);
    if (tid == 0) {
        ids[b] = r.id;
        logZ_valid[b] = r.logZ_valid;
        if (logZ_all) logZ_all[b] = r.logZ_all;
    }
}

// ------------------------------------------------------------------------------------------
// Fused decode step: walk + scatter into LDS + sample + append + membership of the extended row.
template <typename T>
__global__ __launch_bounds__(SAMPLE_THREADS) void decode_step_kernel(
    IndexView ix, int32_t *__restrict__ prefixes, int32_t stride, int32_t *__restrict__ lens,
    uint8_t *__restrict__ active, const T *__restrict__ logits, int64_t row_stride,
    const float *__restrict__ uniforms, int n_words, int32_t *__restrict__ ids, float *__restrict__ logZ_valid,
    float *__restrict__ logx) {
    extern __shared__ __align__(16) uint32_t smem[];
    uint32_t *img = smem;                                        // [n_words]
    uint32_t *bc = smem + n_words;                               // [4]
    double *scratch = (double *)(smem + ((n_words + 4 + 1) & ~1));  // 8-byte aligned
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    if (!active[b]) return;                                      // uniform for the workgroup
    int t = lens[b];
    t = t < 0 ? 0 : (t > stride ? stride : t);
    for (int i = tid; i < n_words; i += SAMPLE_THREADS) img[i] = 0u;
    if (wave == 0) {
        Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, t, lane);
        if (lane == 0) {
            bc[0] = w.node;
            bc[1] = w.found ? 1u : 0u;
        }
    }
    __syncthreads();
    const uint32_t node = bc[0];
    const bool found = bc[1] != 0u;
    if (found) scatter_children(ix, node, img, tid, SAMPLE_THREADS);
    __syncthreads();
    auto bit = [=](int v) { return (img[v >> 5] >> (v & 31)) & 1u; };
    RowResult r = sample_row<T>(logits + (size_t)b * (size_t)row_stride, ix.vocab, bit, uniforms[b], scratch, tid);
    const bool room = t < stride;
    if (wave == 0) {
        bool done = true;  // no valid token or no room: the row cannot continue
        int32_t id = -1;
        if (r.id >= 0 && room) {
            id = r.id;
            // the extended row's entry is the child carrying the sampled token
            uint32_t cb = ix.child_off[node], ce = ix.child_off[node + 1];
            bool match;
            uint32_t j = wave_lower_bound(ix.node_tok, cb, ce, (uint32_t)id, lane, &match);
            if (match) {  // always true: the token came from this node's children
                Walk w2;
                w2.node = j;
                w2.lo = ix.node_lo[j];
                w2.hi = ix.node_hi[j];
                w2.found = true;
                done = node_is_member(ix, w2, t + 1);
            }
        }
        if (lane == 0) {
            if (id >= 0) {
                prefixes[(size_t)b * (size_t)stride + t] = id;
                lens[b] = t + 1;
                if (logx) logx[b] += r.logZ_valid;
            }
            if (ids) ids[b] = id;
            if (logZ_valid) logZ_valid[b] = r.logZ_valid;
            if (done) active[b] = 0;
        }
    }
}

ppv_status check_logits_args(const void *logits, ppv_dtype dt, int64_t row_stride, int32_t V) {
    if (!logits || V <= 0 || row_stride < V) return PPV_EINVAL;
    if (dt != PPV_F32 && dt != PPV_BF16) return PPV_EINVAL;
    const int64_t per16 = (dt == PPV_F32) ? 4 : 8;
    if (row_stride % per16 != 0 || ((uintptr_t)logits & 15u) != 0) return PPV_EINVAL;
    if (V > PPV_MAX_VOCAB) return PPV_ERANGE;
    return PPV_OK;
}

}  // namespace

extern "C" ppv_status ppv_next_token_mask(const ppv_index_t *ix, const int32_t *prefixes, int32_t prefix_stride,
                                          const int32_t *lens, int32_t B, uint32_t *mask, uint32_t *range_lo,
                                          uint32_t *range_hi, uint8_t *member, void *stream) {
    if (!ix || B < 0 || prefix_stride < 0) return PPV_EINVAL;
    if (B == 0) return PPV_OK;  // nothing to do; the (possibly null) buffers are not looked at
    if (!prefixes || !lens || !mask) return PPV_EINVAL;
    const int n_words = (ix->view.vocab + 31) / 32;
    const size_t lds = ((size_t)n_words + 2) * sizeof(uint32_t);
    hipLaunchKernelGGL(mask_kernel, dim3((unsigned)B), dim3(MASK_THREADS), lds, (hipStream_t)stream, ix->view,
                       prefixes, prefix_stride, lens, mask, range_lo, range_hi, member, n_words);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}

extern "C" ppv_status constrained_sample(const void *logits, ppv_dtype dt, int64_t row_stride, const uint32_t *mask,
                                         const float *uniforms, int32_t B, int32_t V, int32_t *ids,
                                         float *logZ_valid, float *logZ_all, void *stream) {
    if (B < 0) return PPV_EINVAL;
    if (B == 0) return PPV_OK;
    if (!mask || !uniforms || !ids || !logZ_valid) return PPV_EINVAL;
    ppv_status st = check_logits_args(logits, dt, row_stride, V);
    if (st != PPV_OK) return st;
    const int n_words = (V + 31) / 32;
    if (dt == PPV_F32)
        hipLaunchKernelGGL(sample_kernel<float>, dim3((unsigned)B), dim3(SAMPLE_THREADS), 0, (hipStream_t)stream,
                           (const float *)logits, row_stride, mask, uniforms, V, n_words, ids, logZ_valid, logZ_all);
    else
        hipLaunchKernelGGL(sample_kernel<uint16_t>, dim3((unsigned)B), dim3(SAMPLE_THREADS), 0, (hipStream_t)stream,
                           (const uint16_t *)logits, row_stride, mask, uniforms, V, n_words, ids, logZ_valid,
                           logZ_all);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}

extern "C" ppv_status ppv_decode_step(const ppv_index_t *ix, int32_t *prefixes, int32_t prefix_stride, int32_t *lens,
                                      uint8_t *active, const void *logits, ppv_dtype dt, int64_t row_stride,
                                      const float *uniforms, int32_t B, int32_t *ids, float *logZ_valid, float *logx,
                                      void *stream) {
    if (!ix || B < 0 || prefix_stride < 0) return PPV_EINVAL;
    if (B == 0) return PPV_OK;
    if (!prefixes || !lens || !active || !uniforms) return PPV_EINVAL;
    ppv_status st = check_logits_args(logits, dt, row_stride, ix->view.vocab);
    if (st != PPV_OK) return st;
    const int n_words = (ix->view.vocab + 31) / 32;
    const size_t lds = (((size_t)n_words + 4 + 1) & ~(size_t)1) * sizeof(uint32_t) + SAMPLE_SCRATCH_DOUBLES * sizeof(double);
    if (dt == PPV_F32)
        hipLaunchKernelGGL(decode_step_kernel<float>, dim3((unsigned)B), dim3(SAMPLE_THREADS), lds,
                           (hipStream_t)stream, ix->view, prefixes, prefix_stride, lens, active,
                           (const float *)logits, row_stride, uniforms, n_words, ids, logZ_valid, logx);
    else
        hipLaunchKernelGGL(decode_step_kernel<uint16_t>, dim3((unsigned)B), dim3(SAMPLE_THREADS), lds,
                           (hipStream_t)stream, ix->view, prefixes, prefix_stride, lens, active,
                           (const uint16_t *)logits, row_stride, uniforms, n_words, ids, logZ_valid, logx);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}
