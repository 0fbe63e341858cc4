// Per-step kernels for gfx950 (wave64): next-token scatter (packed mask) with the prefix's rank range,
// fused masked log-softmax + inverse-CDF sample, and the fused decode step (the prefix is located by
// walk_prefix, shared with the top-M kernel).
//
// The logits row is the only large operand.  It is streamed exactly once, in tiles of 4 KB per
// wavefront (four 16-byte loads per lane, issued before any index work so that they are in
// flight while the prefix is located).  Each tile yields (reference, sum of exp relative to it), the
// reference being a value near the tile's maximum; tiles are combined afterwards, so every tile is
// independent and a row can be spread over any number of wavefronts.  The valid set enters in one of two ways:
//   list   at most PPV_LIST_MAX valid tokens: their logits are gathered (they were just streamed,
//          so they come from cache), summed relative to their own maximum, and the sample is
//          located by a scan over the list -- no per-element mask work in the stream;
//   image  more valid tokens: a V-bit image is applied inside the stream (three more ALU
//          operations per element) and the sample is located by re-reading one tile.
// Nothing here is a dense contraction, so no MFMA; the bound is HBM bandwidth, with the exp
// (quarter-rate v_exp_f32) as the main ALU cost.
#include <cmath>
#include <mutex>
#include <type_traits>

#include "ppv_device.h"
#include "ppv_internal.h"
#include "ppv_walk.h"

namespace {

constexpr int MASK_THREADS = 256;
constexpr int MAX_WAVES = 16;                 // wavefronts per row (workgroup of up to 1024 threads)
constexpr int LOOP_WAVES = 8;                 // the decode-loop kernel holds more in registers: at most 512 threads
constexpr int CHAIN_WAVES = 10;               // ... or, with one wavefront that only draws tokens beside up to nine that stream, 640
constexpr int MAX_TILES = PPV_MAX_TILES;
constexpr float LN2F = 0.693147180559945309417f;
static_assert(PPV_MAX_VOCAB <= MAX_TILES * 1024, "tile bookkeeping too small");

__device__ inline float fast_exp2(float y) { return __builtin_amdgcn_exp2f(y); }  // v_exp_f32, 1 ulp
__device__ inline float fast_log2(float y) { return __builtin_amdgcn_logf(y); }   // v_log_f32, 1 ulp (normal inputs)
// exp(d) for d <= 0 with the rounding of d*log2(e) compensated (used once per tile, not per token)
// Temperature (Algorithm 1's input T): P = softmax(logits / T).  The division is folded into the constant of the
// exponentials, c = log2(e) / T, so that it costs nothing per token; differences of logits that enter a result
// as they are (a reference minus another) are multiplied by inv = 1 / T.  T = 1 gives c = log2(e), inv = 1.
struct Temper {
    float c;
    float inv;
    float guard;   // how far above a tile's reference a logit may lie (REF_GUARD * T, see tile_stats)
};

__device__ inline float exp_scale(float d, float c) {
    float hi = d * c;
    float lo = fmaf(d, c, -hi);
    return fast_exp2(hi) * fmaf(lo, LN2F, 1.0f);
}

// ------------------------------------------------------------------------------------------
// ppv_next_token_mask: one workgroup per prefix.
__global__ __launch_bounds__(MASK_THREADS) void mask_kernel(IndexView ix, const int32_t *__restrict__ prefixes,
                                                            int32_t stride, const int32_t *__restrict__ lens,
                                                            uint32_t *__restrict__ mask,
                                                            uint32_t *__restrict__ range_lo,
                                                            uint32_t *__restrict__ range_hi,
                                                            uint8_t *__restrict__ member) {
    extern __shared__ __align__(16) uint32_t smem[];
    const int n_words = ix.n_words;
    uint32_t *img = smem;            // [n_words]
    uint32_t *bc = smem + n_words;   // [4]: node, found, cb, ce
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    if (wave == 0) {
        const int32_t mine = first_tokens(prefixes + (size_t)b * (size_t)stride, stride, lane);
        int t = lens[b];
        t = t < 0 ? 0 : (t > stride ? stride : t);
        Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, mine, t, lane);
        if (lane == 0) {
            bc[0] = w.node;
            bc[1] = w.found ? 1u : 0u;
            bc[2] = w.found ? w.cb : 0u;
            bc[3] = w.found ? w.ce : 0u;
            if (range_lo) range_lo[b] = w.lo;
            if (range_hi) range_hi[b] = w.hi;
            if (member) member[b] = w.member ? 1 : 0;
        }
    }
    __syncthreads();
    const uint32_t node = bc[0];
    const bool found = bc[1] != 0u;
    const uint32_t cb = bc[2], ce = bc[3];
    uint32_t *out = mask + (size_t)b * (size_t)n_words;
    // rows are written 16 bytes per lane when every row starts on a 16-byte boundary
    const bool wide = (n_words & 3) == 0 && (((uintptr_t)mask) & 15u) == 0;
    const int n_quads = n_words >> 2;
    if (found && ce - cb > ix.heavy_min) {  // ready-made image: plain copy
        const uint32_t *src = ix.heavy_bits + (size_t)heavy_slot_of(ix, node) * (size_t)n_words;
        if (wide && (((uintptr_t)ix.heavy_bits) & 15u) == 0) {
            for (int i = tid; i < n_quads; i += MASK_THREADS) ((uint4 *)out)[i] = ((const uint4 *)src)[i];
        } else {
            for (int i = tid; i < n_words; i += MASK_THREADS) out[i] = src[i];
        }
        return;
    }
    if (cb == ce) {  // not in S, or a member without extensions
        if (wide) {
            for (int i = tid; i < n_quads; i += MASK_THREADS) ((uint4 *)out)[i] = make_uint4(0u, 0u, 0u, 0u);
        } else {
            for (int i = tid; i < n_words; i += MASK_THREADS) out[i] = 0u;
        }
        return;
    }
    for (int i = tid; i < n_words; i += MASK_THREADS) img[i] = 0u;
    __syncthreads();
    for (uint32_t i = cb + (uint32_t)tid; i < ce; i += MASK_THREADS) {
        uint32_t v = ix.ent[i].tok & PPV_NODE_TOKEN;
        atomicOr(&img[v >> 5], 1u << (v & 31u));
    }
    __syncthreads();
    if (wide) {
        for (int i = tid; i < n_quads; i += MASK_THREADS) ((uint4 *)out)[i] = ((const uint4 *)img)[i];
    } else {
        for (int i = tid; i < n_words; i += MASK_THREADS) out[i] = img[i];
    }
}

// The same for vocabularies of at most 2,048 tokens (a mask row is at most 64 words: one word per lane): one
// wavefront per prefix, four prefixes per workgroup, no LDS and no barrier.  A listed node has at most V / 32 <= 64
// children here, one per lane; each child's bit is set by the lane that holds its word.
constexpr int MASK_SMALL_WORDS = WAVE;
__global__ __launch_bounds__(MASK_THREADS) void mask_rows_kernel(IndexView ix, const int32_t *__restrict__ prefixes,
                                                                 int32_t stride, const int32_t *__restrict__ lens, int B,
                                                                 uint32_t *__restrict__ mask,
                                                                 uint32_t *__restrict__ range_lo,
                                                                 uint32_t *__restrict__ range_hi,
                                                                 uint8_t *__restrict__ member) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int b = blockIdx.x * (MASK_THREADS / WAVE) + threadIdx.x / WAVE;
    if (b >= B) return;  // uniform per wavefront
    const int n_words = ix.n_words;
    const int32_t mine = first_tokens(prefixes + (size_t)b * (size_t)stride, stride, lane);
    int t = lens[b];
    t = t < 0 ? 0 : (t > stride ? stride : t);
    const Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, mine, t, lane);
    if (lane == 0) {
        if (range_lo) range_lo[b] = w.lo;
        if (range_hi) range_hi[b] = w.hi;
        if (member) member[b] = w.member ? 1 : 0;
    }
    uint32_t word = 0u;
    const uint32_t nchild = w.found ? w.ce - w.cb : 0u;
    if (nchild > ix.heavy_min) {   // ready-made image
        if (lane < n_words) word = ix.heavy_bits[(size_t)heavy_slot_of(ix, w.node) * (size_t)n_words + lane];
    } else if (nchild > 0u) {      // nchild <= heavy_min <= 64
        const uint32_t tok = (uint32_t)lane < nchild ? (ix.ent[w.cb + (uint32_t)lane].tok & PPV_NODE_TOKEN) : 0u;
        for (uint32_t i = 0; i < nchild; i++) {   // uniform trip count
            const uint32_t v = (uint32_t)__builtin_amdgcn_readlane((int)tok, (int)i);
            if ((uint32_t)lane == (v >> 5)) word |= 1u << (v & 31u);
        }
    }
    if (lane < n_words) mask[(size_t)b * (size_t)n_words + lane] = word;
}

// ------------------------------------------------------------------------------------------
// Tiles.  A tile is what one wavefront loads with four 16-byte loads per lane: 2048 bf16 or 1024
// fp32 tokens.  Load j of lane l holds the EPL consecutive tokens starting at
// tile*TILE + j*64*EPL + l*EPL, so token order inside a tile is (j, lane, k).
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int EPL = 4;  // tokens per 16-byte load
    __device__ static inline void unpack(const uint4 &r, float x[4]) {
        x[0] = __uint_as_float(r.x); x[1] = __uint_as_float(r.y);
        x[2] = __uint_as_float(r.z); x[3] = __uint_as_float(r.w);
    }
    __device__ static inline uint32_t pad() { return 0xFF800000u; }  // -inf
};
template <> struct Elem<uint16_t> {  // bf16: widening to fp32 is exact
    static constexpr int EPL = 8;
    __device__ static inline void unpack(const uint4 &r, float x[8]) {
        x[0] = __uint_as_float(r.x << 16); x[1] = __uint_as_float(r.x & 0xFFFF0000u);
        x[2] = __uint_as_float(r.y << 16); x[3] = __uint_as_float(r.y & 0xFFFF0000u);
        x[4] = __uint_as_float(r.z << 16); x[5] = __uint_as_float(r.z & 0xFFFF0000u);
        x[6] = __uint_as_float(r.w << 16); x[7] = __uint_as_float(r.w & 0xFFFF0000u);
    }
    __device__ static inline uint32_t pad() { return 0xFF80FF80u; }  // two bf16 -inf
};
template <typename T> struct TileGeom {
    static constexpr int EPL = Elem<T>::EPL;
    static constexpr int PER_LOAD = WAVE * EPL;   // tokens covered by one load of the wave
    static constexpr int TILE = 4 * PER_LOAD;     // tokens per tile
    static constexpr int WORDS = TILE / 32;       // mask words per tile
    static constexpr int LANES_PER_WORD = 32 / EPL;
};

struct RawTile {
    uint4 r[4];
    uint32_t word;   // image path: this lane's word of the tile's mask (requested together with the tile)
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename T>
__device__ inline void load_tile(const T *__restrict__ row, int V, int tile, int lane, RawTile &rt) {
    using G = TileGeom<T>;
    const int base = tile * G::TILE + lane * G::EPL;
    if ((tile + 1) * G::TILE <= V) {  // wave-uniform: whole tile inside the row
#pragma unroll
        for (int j = 0; j < 4; j++) {
            u32x4 v = __builtin_nontemporal_load((const u32x4 *)(row + base + j * G::PER_LOAD));
            rt.r[j] = make_uint4(v.x, v.y, v.z, v.w);
        }
    } else {  // ragged tail: never touch memory at or beyond token V; missing tokens are -inf
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int g = base + j * G::PER_LOAD;
            if (g + G::EPL <= V) {
                rt.r[j] = *(const uint4 *)(row + g);
            } else {
                uint32_t w[4] = {Elem<T>::pad(), Elem<T>::pad(), Elem<T>::pad(), Elem<T>::pad()};
                if (sizeof(T) == 4) {
                    for (int k = 0; k < 4; k++)
                        if (g + k < V) w[k] = ((const uint32_t *)row)[g + k];
                } else {
                    for (int k = 0; k < 8; k++)
                        if (g + k < V) {
                            uint32_t h = ((const uint16_t *)row)[g + k];
                            w[k >> 1] = (k & 1) ? ((w[k >> 1] & 0x0000FFFFu) | (h << 16))
                                                : ((w[k >> 1] & 0xFFFF0000u) | h);
                        }
                }
                rt.r[j] = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    }
}

// a tile known to lie wholly inside the row: four unconditional streaming loads
template <typename T>
__device__ inline void load_full_tile(const T *__restrict__ row, int tile, int lane, RawTile &rt) {
    using G = TileGeom<T>;
    const u32x4 *p = (const u32x4 *)(row + (size_t)tile * G::TILE + lane * G::EPL);
#pragma unroll
    for (int j = 0; j < 4; j++) {
        u32x4 v = __builtin_nontemporal_load(p + j * WAVE);
        rt.r[j] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// A tile requested with four unconditional 16-byte loads wherever it lies: a group of tokens past the row's end is
// read from the row's last whole group instead (valid memory), and pad_tile_tail, called when the tile is used, puts
// -inf there.  Nothing is conditional between request and use, so the compiler can count the loads in flight and
// wait for exactly the ones a use needs.  Needs V % EPL == 0 (no group straddles the row's end).
template <typename T>
__device__ inline void load_tile_clamped(const T *__restrict__ row, int V, int tile, int lane, RawTile &rt) {
    using G = TileGeom<T>;
    const int base = tile * G::TILE + lane * G::EPL;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const int g = base + j * G::PER_LOAD;
        const int gc = g < V ? g : V - G::EPL;
        u32x4 v = __builtin_nontemporal_load((const u32x4 *)(row + gc));
        rt.r[j] = make_uint4(v.x, v.y, v.z, v.w);
    }
}
template <typename T> __device__ inline void pad_tile_tail(RawTile &rt, int V, int tile, int lane) {
    using G = TileGeom<T>;
    const int base = tile * G::TILE + lane * G::EPL;
#pragma unroll
    for (int j = 0; j < 4; j++)
        if (base + j * G::PER_LOAD >= V) rt.r[j] = make_uint4(Elem<T>::pad(), Elem<T>::pad(), Elem<T>::pad(), Elem<T>::pad());
}

// word wi of a V-bit image, with bits at positions >= V cleared (0 beyond the image).  The load
// itself is unconditional (clamped index): a conditional load would make later waits conservative.
__device__ inline uint32_t image_word(const uint32_t *__restrict__ image, int wi, int V) {
    const int n_words = (V + 31) / 32;
    const int last = n_words - 1;
    uint32_t w = image[wi < last ? wi : last];
    if (wi == last && (V & 31)) w &= (1u << (V & 31)) - 1u;
    return wi <= last ? w : 0u;
}
// the tile's mask word for this lane (lane l < WORDS holds word l of the tile)
template <typename T>
__device__ inline uint32_t tile_mask_word(const uint32_t *__restrict__ image, int tile, int lane, int V) {
    using G = TileGeom<T>;
    const uint32_t w = image_word(image, tile * G::WORDS + (lane < G::WORDS ? lane : 0), V);
    return lane < G::WORDS ? w : 0u;
}

// mask bits of this lane's EPL tokens of load j, from the tile's mask words (lane l < WORDS holds word l)
template <typename T> __device__ inline uint32_t lane_bits(uint32_t tile_word, int j, int lane) {
    using G = TileGeom<T>;
    uint32_t w = (uint32_t)__shfl((int)tile_word, j * (G::WORDS / 4) + lane / G::LANES_PER_WORD, WAVE);
    return (w >> ((lane % G::LANES_PER_WORD) * G::EPL)) & ((1u << G::EPL) - 1u);
}

// Statistics of one tile: a reference m, sum_all = sum exp(x - m), and (IMAGE) sum_val over valid tokens.
// Any reference near the tile's maximum gives the same sums up to rounding, so the reduction over the
// wavefront that the exact maximum would need is avoided: m is the maximum of lane 0's own tokens (one
// readfirstlane), as long as no token of the tile lies more than REF_GUARD * T above it (one compare over the
// lanes' maxima); otherwise, and when lane 0 holds nothing but -inf, m is the exact maximum.  Either way m
// depends on the row's values alone, not on how the row is split over wavefronts.  m = -inf: an empty tile.
constexpr float REF_GUARD = 40.f;   // exp(40) * 2048 tokens is far inside fp32
template <typename T, bool IMAGE>
__device__ inline void tile_stats(const RawTile &rt, uint32_t tile_word, int lane, const Temper &tp, float &m_out,
                                  float &zall_out, float &zval_out) {
    using G = TileGeom<T>;
    float x[4][G::EPL];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        Elem<T>::unpack(rt.r[j], x[j]);
#pragma unroll
        for (int k = 0; k < G::EPL; k++) mx = fmaxf(mx, x[j][k]);
    }
    float ref = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(mx)));
    if (ref == -INFINITY || __ballot(mx > ref + tp.guard) != 0ull) ref = wave_max(mx);   // wave-uniform branch
    m_out = ref;
    if (ref == -INFINITY) {  // nothing but -inf in this tile
        zall_out = 0.f;
        zval_out = 0.f;
        return;
    }
    // exp(x - m) = 2^(x*c - m*c); m*c is rounded once (mc), its residual is folded into the tile sums
    const float c = tp.c;
    const float mc = ref * c;
    const float resid = fmaf(ref, c, -mc);
    float zall = 0.f, zval = 0.f;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        uint32_t bits = 0;
        if (IMAGE) bits = lane_bits<T>(tile_word, j, lane);
#pragma unroll
        for (int k = 0; k < G::EPL; k++) {
            float e = fast_exp2(fmaf(x[j][k], c, -mc));
            zall += e;
            if (IMAGE) {
                uint32_t keep = (uint32_t)(-(int32_t)((bits >> k) & 1u));
                zval += __uint_as_float(__float_as_uint(e) & keep);
            }
        }
    }
    const float fix = fast_exp2(-resid);
    zall_out = wave_sum(zall) * fix;
    zval_out = IMAGE ? wave_sum(zval) * fix : 0.f;
}

// Rare path of the image mode (the valid tokens lie far below the row maximum, so sums relative
// to the tile maxima would lose them): maximum over the valid tokens of a tile ...
template <typename T>
__device__ inline float tile_valid_max(const RawTile &rt, uint32_t tile_word, int lane) {
    using G = TileGeom<T>;
    float mv = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        float x[G::EPL];
        Elem<T>::unpack(rt.r[j], x);
        const uint32_t bits = lane_bits<T>(tile_word, j, lane);
#pragma unroll
        for (int k = 0; k < G::EPL; k++)
            if ((bits >> k) & 1u) mv = fmaxf(mv, x[k]);
    }
    return wave_max(mv);
}
// ... and the valid sum of a tile relative to a given reference (finite)
template <typename T>
__device__ inline float tile_valid_sum(const RawTile &rt, uint32_t tile_word, int lane, float ref, float c) {
    using G = TileGeom<T>;
    const float mc = ref * c;
    const float fix = fast_exp2(-fmaf(ref, c, -mc));
    float z = 0.f;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        float x[G::EPL];
        Elem<T>::unpack(rt.r[j], x);
        const uint32_t bits = lane_bits<T>(tile_word, j, lane);
#pragma unroll
        for (int k = 0; k < G::EPL; k++)
            if ((bits >> k) & 1u) z += fast_exp2(fmaf(x[k], c, -mc));
    }
    return wave_sum(z) * fix;
}

// Locate the sample inside one tile (IMAGE path).  target is the cumulative valid weight to exceed,
// in units of exp(x - m_tile).  Returns the token id (wave-uniform), or -1 if the tile has no valid
// token with positive weight.  When rounding lets no token exceed the target, the last valid token
// with positive weight is returned.
template <typename T>
__device__ inline int locate_in_tile(const RawTile &rt, uint32_t tile_word, int tile, int lane, float m,
                                     double target, float tc) {
    using G = TileGeom<T>;
    const float mc = m * tc;
    const float fix = fast_exp2(-fmaf(m, tc, -mc));
    double before = 0.0;  // valid weight of the loads already passed
    int last_valid = -1;
    for (int j = 0; j < 4; j++) {
        float x[G::EPL], e[G::EPL];
        Elem<T>::unpack(rt.r[j], x);
        const uint32_t bits = lane_bits<T>(tile_word, j, lane);
        float grp = 0.f;
        int my_last = -1;
#pragma unroll
        for (int k = 0; k < G::EPL; k++) {
            e[k] = ((bits >> k) & 1u) ? fast_exp2(fmaf(x[k], tc, -mc)) * fix : 0.f;
            grp += e[k];
            if (e[k] > 0.f) my_last = k;
        }
        const double incl = before + wave_incl_scan((double)grp);
        const uint64_t cross = __ballot(incl > target);
        const int first_tok = tile * G::TILE + j * G::PER_LOAD;
        if (cross) {
            const int l = __ffsll((long long)cross) - 1;
            int id = -1;
            if (lane == l) {
                double c = incl - (double)grp;
                for (int k = 0; k < G::EPL; k++) {
                    c += (double)e[k];
                    if (e[k] > 0.f && c > target) { id = k; break; }
                }
                if (id < 0) id = my_last;  // rounding inside the group
                if (id >= 0) id += first_tok + lane * G::EPL;   // (-1: a target below zero met a lane without a valid token)
            }
            return lane_value(id, l);
        }
        const uint64_t have = __ballot(my_last >= 0);
        if (have) {
            const int l = 63 - __clzll((long long)have);
            last_valid = lane_value(first_tok + lane * G::EPL + my_last, l);
        }
        before = last_lane(incl);
    }
    return last_valid;
}

// ------------------------------------------------------------------------------------------
// One row by one workgroup of `nw` wavefronts.
template <int TILES, int LIST> struct RowSharedT {
    float tile_m[TILES];
    float tile_zall[TILES];
    float tile_zval[TILES];
    float tile_ref[TILES];             // what tile_zval is relative to (the tile maximum, or the valid maximum)
    uint32_t list_tok[LIST + 1];       // valid tokens in increasing order (list path), flags in the top bits
    uint32_t list_child[LIST + 1];     // decode step: child offsets of the listed entries
    float list_e[LIST];                // exp(l - slice max) per listed token
    float slice_m[LIST / WAVE];
    float slice_z[LIST / WAVE];
    int tile_cnt[TILES];               // valid tokens per tile (mask -> list conversion)
    int bc_i[8];
    float bc_f[4];
};
using RowShared = RowSharedT<MAX_TILES, PPV_LIST_MAX>;
// Rows of at most SMALL_TILES tiles whose lists hold at most SMALL_LIST tokens (V <= 2048: the list limit is
// V / 32): 1 KB of LDS per row instead of 18 KB, so that the compute unit is filled by registers, not by LDS.
constexpr int SMALL_TILES = 4, SMALL_LIST = 64;
using RowSharedSmall = RowSharedT<SMALL_TILES, SMALL_LIST>;

struct RowOut {
    int32_t id;        // sampled token or -1
    int32_t pos;       // list path: position of the sampled token in the list, else -1
    float logZ_valid;
    float logZ_all;
    bool mine;         // this thread holds the row's result (wavefront 0 of the workgroup that finishes the row;
                       // every thread of it with ALL)
};

// Words that the workgroups of a split row hand to one another are written and read with device-scope accesses
// (each goes to the level of the memory system that all compute units share), so that no fence over the whole
// cache is needed: a device-wide fence per wavefront cost 30 us per launch, these cost about two.
__device__ inline void shared_put(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ inline float shared_get(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void shared_put_tile(SplitRow *r, int k, float m, float zall, float zval, float ref) {
    float *t = (float *)&r->tile[k];
    shared_put(t + 0, m);
    shared_put(t + 1, zall);
    shared_put(t + 2, zval);
    shared_put(t + 3, ref);
}

// A row shared by `parts` workgroups (see SplitRow); parts == 1: one workgroup has the row to itself and
// nothing else here is looked at.
struct Split {
    int parts;
    int part;             // this workgroup's number, 0 .. parts-1
    SplitRow *row;        // the row's scratch
    uint32_t *arrivals;   // the row's arrival counter
};

enum ValidMode { VALID_NONE = 0, VALID_LIST = 1, VALID_IMAGE = 2 };

// Streams a row's tiles through one wavefront's share of the work: wave `wave` of `nw` takes the
// tiles wave, wave+nw, ...  Per tile the statistics go to LDS.
//
// Full tiles go through a software pipeline of three register tiles X, Y, Z.  Each is reduced and
// then at once reloaded with the tile three turns ahead, so that two tiles (8 KB per wavefront)
// are always in flight behind the one being reduced.  The steady loop has no conditional load:
// every wait in it is for loads issued a known number of loads ago, so the compiler's wait
// counters leave the younger loads in flight (a conditional load anywhere on the way to a use
// makes it wait for everything).  The row's ragged last tile, if any, is taken with the guarded
// loader by the wave whose turn it is.
// `mid` is work of the caller's that needs no tile (the sums over the listed tokens): it is run once, at the first
// point where this wavefront has just asked for a tile and would only wait for it; never, if there is no such point.
// `wave_v` of `nw`: the wavefront's number among all wavefronts that share the row (over all its workgroups);
// `pub`: where a split row's statistics are left for the workgroup that finishes it (nullptr: not split).
template <typename T, bool IMAGE, bool PIPE, typename SH, typename MID>
__device__ inline void stream_tiles(const T *__restrict__ row, int V, const RawTile &first,
                                    const uint32_t *__restrict__ image, SH &sh, int lane, int wave_v,
                                    int nw, const Temper &tp, MID &mid, SplitRow *pub) {
    using G = TileGeom<T>;
    const int wave = __builtin_amdgcn_readfirstlane(wave_v);   // scalar: loop control stays uniform
    const int nt = (V + G::TILE - 1) / G::TILE;
    const int nfull = V / G::TILE;
    if (wave >= nt) return;
    auto reduce_tile = [&](const RawTile &t, int k) {
        float m, zall, zval;
        tile_stats<T, IMAGE>(t, IMAGE ? t.word : 0u, lane, tp, m, zall, zval);
        if (lane == 0) {
            sh.tile_m[k] = m;
            sh.tile_zall[k] = zall;
            sh.tile_zval[k] = zval;
            sh.tile_ref[k] = m;
            if (pub) shared_put_tile(pub, k, m, zall, zval, m);
        }
    };
    auto fetch = [&](RawTile &t, int k) {   // a full tile and, on the image path, its mask word
        load_full_tile<T>(row, k, lane, t);
        if (IMAGE) t.word = tile_mask_word<T>(image, k, lane, V);
    };
    // this wave's full tiles are wave + i*nw for i in [0, cnt); `first` is i = 0 (or the ragged tile)
    const int cnt = wave < nfull ? (nfull - wave + nw - 1) / nw : 0;
    int i = 0;
    bool mid_done = false;
    RawTile X = first, Y, Z;   // the same three register tiles serve every path below
    if (IMAGE) X.word = tile_mask_word<T>(image, wave, lane, V);
    if (PIPE && cnt >= 6) {
        fetch(Y, wave + nw);
        fetch(Z, wave + 2 * nw);
        mid();
        mid_done = true;
        while (i + 5 < cnt) {
            reduce_tile(X, wave + i * nw);
            fetch(X, wave + (i + 3) * nw);
            reduce_tile(Y, wave + (i + 1) * nw);
            fetch(Y, wave + (i + 4) * nw);
            reduce_tile(Z, wave + (i + 2) * nw);
            fetch(Z, wave + (i + 5) * nw);
            i += 3;
        }
        reduce_tile(X, wave + i * nw);
        reduce_tile(Y, wave + (i + 1) * nw);
        reduce_tile(Z, wave + (i + 2) * nw);
        i += 3;
    } else if (!PIPE && cnt >= 2) {
        // a short turn (in the kernels without the three-tile pipeline, which have the registers for it): two tiles take turns in X and Y, the next one asked for before this one is reduced.  Every
        // fetch stands in straight-line code with the reduction that follows it, so the waits stay exact.
        while (i + 2 < cnt) {   // X holds tile i
            fetch(Y, wave + (i + 1) * nw);
            if (!mid_done) {
                mid();
                mid_done = true;
            }
            reduce_tile(X, wave + i * nw);
            fetch(X, wave + (i + 2) * nw);
            reduce_tile(Y, wave + (i + 1) * nw);
            i += 2;
        }
        if (i + 1 < cnt) {
            fetch(Y, wave + (i + 1) * nw);
            if (!mid_done) {
                mid();
                mid_done = true;
            }
            reduce_tile(X, wave + i * nw);
            reduce_tile(Y, wave + (i + 1) * nw);
            i += 2;
        } else {
            reduce_tile(X, wave + i * nw);
            i += 1;
        }
    } else if (cnt > 0 || wave == nfull) {
        reduce_tile(X, wave);   // a single full tile, or the ragged one when the wave has nothing else
        i = 1;
    }
    // what is left (a short turn in a kernel with the three-tile pipeline, tile by tile), and perhaps the ragged tail
    for (; i < cnt; i++) {
        fetch(Z, wave + i * nw);
        if (!mid_done) {
            mid();
            mid_done = true;
        }
        reduce_tile(Z, wave + i * nw);
    }
    if (nfull < nt && nfull % nw == wave && wave != nfull) {
        load_tile<T>(row, V, nfull, lane, Z);
        if (IMAGE) Z.word = tile_mask_word<T>(image, nfull, lane, V);
        reduce_tile(Z, nfull);
    }
}

// Row totals from the per-tile statistics in LDS: the largest tile reference M, the sum over all tokens relative
// to it and (image rows) the sum over valid tokens.  Called by a whole wavefront; results are uniform.  The sum over
// all tokens only ever enters a logarithm, so it is added up in fp32 (a tree over at most 256 positive terms: a few
// 1e-7 relative); the valid sum sets the sampling threshold and is added up in fp64.
template <typename SH>
__device__ inline void combine_tiles(const SH &sh, int nt, int lane, const Temper &tp, bool image, float &M, float &za,
                                     double &zv) {
    if (nt <= WAVE) {   // (uniform) one tile per lane at most: both words in one round of LDS reads, no loops; the
                        // same operations in the same order as below, so the same bits
        const bool have = lane < nt;
        const float m = have ? sh.tile_m[have ? lane : 0] : -INFINITY;
        const float z = have ? sh.tile_zall[have ? lane : 0] : 0.f;
        const float zval = (image && have) ? sh.tile_zval[have ? lane : 0] : 0.f;
        M = wave_max(m);
        float a = 0.f;
        double v = 0.0;
        if (m != -INFINITY) {
            const float sc = exp_scale(m - M, tp.c);
            a = z * sc;
            if (image) v = (double)zval * (double)sc;
        }
        za = wave_sum(a);
        zv = image ? wave_sum(v) : 0.0;
        return;
    }
    M = -INFINITY;
    for (int k = lane; k < nt; k += WAVE) M = fmaxf(M, sh.tile_m[k]);
    M = wave_max(M);
    za = 0.f;
    zv = 0.0;
    for (int k = lane; k < nt; k += WAVE) {
        const float m = sh.tile_m[k];
        if (m != -INFINITY) {
            const float sc = exp_scale(m - M, tp.c);
            za += sh.tile_zall[k] * sc;
            if (image) zv += (double)sh.tile_zval[k] * (double)sc;   // (the other modes have no per-tile valid sums)
        }
    }
    za = wave_sum(za);
    if (image) zv = wave_sum(zv);
}

// A list of at most 63 valid tokens that one wavefront holds in registers, entry i in lane i (the per-step decode
// kernel): the sums over the list and the sample, with the arithmetic of the list path of row_sample for a list of
// one slice, so that both give the same bits.  gx: lane i < n_list holds the listed token's logit, the others -inf.
struct RegList {
    bool on;         // (uniform) the row's valid set is held this way
    bool have_gx;    // (uniform) the listed logits have been requested already and are in gx
    uint32_t tokw;   // lane i < n_list: the entry's token word (token | flags)
    float gx;
};
struct ListPick {
    int id, pos;     // sampled token and its position in the list; -1: nothing can be sampled
    float Mv;        // largest listed logit (-inf: no listed token has positive weight)
    double zvl;      // sum of the listed tokens' weights relative to Mv
};
__device__ inline ListPick reg_list_pick(float gx, uint32_t tokw, int n_list, float u, int lane, const Temper &tp) {
    ListPick pk;
    pk.id = -1;
    pk.pos = -1;
    pk.zvl = 0.0;
    if (n_list == 1) {
        // One listed token: what the general case below computes, without its reductions and scans over the lanes
        // (every other lane contributes an exact zero): the weight exp(x - x), through the same rounded steps, is
        // the sum; the token is drawn whatever u is, unless its weight is 0.
        const float g = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(gx)));
        const float m = g == g ? g : -INFINITY;   // (a NaN is passed over, as the maximum over the lanes does)
        pk.Mv = m;
        if (m == -INFINITY) return pk;
        const float mc = m * tp.c;
        const float e = fast_exp2(fmaf(m, tp.c, -mc)) * fast_exp2(-fmaf(m, tp.c, -mc));
        pk.zvl = (double)e;
        if (e > 0.f) {
            pk.pos = 0;
            pk.id = (int)((uint32_t)__builtin_amdgcn_readfirstlane((int)tokw) & PPV_NODE_TOKEN);
        }
        return pk;
    }
    const float m = wave_max(gx);
    pk.Mv = m;
    if (m == -INFINITY) return pk;
    const float mc = m * tp.c;
    const float fix = fast_exp2(-fmaf(m, tp.c, -mc));
    float e = fast_exp2(fmaf(gx, tp.c, -mc)) * fix;   // gx = -inf gives 0
    const double zvl = (double)wave_sum(e);
    pk.zvl = zvl;
    const double tau = (double)u * zvl;
    double target;
    int s;
    if (zvl > tau) {
        s = 0;
        target = tau;
    } else {
        s = zvl > 0.0 ? 0 : -1;
        target = INFINITY;
    }
    if (!(s >= 0 && lane < n_list)) e = 0.f;
    const double ic = wave_incl_scan((double)e);
    const uint64_t c2 = __ballot(e > 0.f && ic > target);
    const uint64_t h2 = __ballot(e > 0.f);
    if (c2 | h2) {
        const int l = c2 ? __ffsll((long long)c2) - 1 : 63 - __clzll((long long)h2);
        pk.pos = l;
        pk.id = (int)(lane_value(tokw, l) & PPV_NODE_TOKEN);
    }
    return pk;
}

// Streams the row and samples.  Called by every thread of the workgroup with uniform arguments.
//   first        this wave's first tile, already loaded (the wave owns tiles wave, wave+nw, ...)
//   next_row     optional: another row whose first tile (per wave) is to be requested into *next_first
//   mode         VALID_LIST: sh.list_tok[0..n_list) holds the valid tokens (in LDS, barrier done)
//                VALID_IMAGE: image (global memory, V bits) is the valid set
//                VALID_NONE: the valid set is empty
//   ALL          every thread gets the result (one more barrier); otherwise only wavefront 0 does
//   sp           the row's split over workgroups: `first` is then tile sp.part * nw + wave, and only the
//                workgroup that arrives last goes on to sample (the others return with mine == false)
//   SPLIT        compiled in only for kernels that may share a row between workgroups (the others pay nothing for it)
template <typename T, bool PIPE, typename SH, bool ALL, bool SPLIT>
__device__ inline RowOut row_sample(const T *__restrict__ row, int V, const RawTile &first, int mode, int n_list,
                                    const uint32_t *__restrict__ image, float u, SH &sh, int tid, int nw,
                                    const Temper &tp, const Split &sp, const T *__restrict__ next_row = nullptr,
                                    RawTile *next_first = nullptr) {
    using G = TileGeom<T>;
    const int lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int nt = (V + G::TILE - 1) / G::TILE;
    // the wavefront's number and count over all workgroups of the row: tiles and list slices are dealt out by these
    const int parts = SPLIT ? sp.parts : 1;
    const int vwave = SPLIT ? sp.part * nw + wave : wave, vnw = parts * nw;
    SplitRow *pub = SPLIT && parts > 1 ? sp.row : nullptr;

    // ---- list path, part 1: ask for the listed tokens' logits now (they are being streamed
    // anyway, so these are cache hits) so that they arrive while the tiles are reduced
    const int ns = (n_list + WAVE - 1) / WAVE;
    float gx = -INFINITY;   // this lane's listed logit of the wave's first slice
    if (mode == VALID_LIST && vwave < ns) {
        const int i = vwave * WAVE + lane;
        if (i < n_list) {
            const uint32_t v = sh.list_tok[i] & PPV_NODE_TOKEN;
            if (sizeof(T) == 4) gx = __uint_as_float(((const uint32_t *)row)[v]);
            else gx = __uint_as_float(((uint32_t)((const uint16_t *)row)[v]) << 16);
        }
    }

    // ---- list path, part 2: sums per slice of 64 listed tokens, relative to the slice maximum.  Run from inside
    // the stream, while the wavefront waits for a tile it has just asked for; after it when there is no such wait.
    bool list_done = false;
    auto list_sums = [&]() {
        list_done = true;
        if (mode != VALID_LIST) return;
        for (int s = vwave; s < ns; s += vnw) {
            const int i = s * WAVE + lane;
            float x = gx;
            if (s != vwave) {
                x = -INFINITY;
                if (i < n_list) {
                    const uint32_t v = sh.list_tok[i] & PPV_NODE_TOKEN;
                    if (sizeof(T) == 4) x = __uint_as_float(((const uint32_t *)row)[v]);
                    else x = __uint_as_float(((uint32_t)((const uint16_t *)row)[v]) << 16);
                }
            }
            const float m = wave_max(x);
            float e = 0.f;
            if (m != -INFINITY) {
                const float mc = m * tp.c;
                const float fix = fast_exp2(-fmaf(m, tp.c, -mc));
                e = fast_exp2(fmaf(x, tp.c, -mc)) * fix;   // x = -inf gives 0
            }
            if (i < n_list) {
                sh.list_e[i] = e;
                if (pub) shared_put(&pub->list_e[i], e);
            }
            const float z = wave_sum(e);
            if (lane == 0) {
                sh.slice_m[s] = m;
                sh.slice_z[s] = z;
                if (pub) {
                    shared_put(&pub->slice_m[s], m);
                    shared_put(&pub->slice_z[s], z);
                }
            }
        }
    };
    // ---- stream: every tile once
    if (mode == VALID_IMAGE) stream_tiles<T, true, PIPE, SH>(row, V, first, image, sh, lane, vwave, vnw, tp, list_sums, pub);
    else stream_tiles<T, false, PIPE, SH>(row, V, first, image, sh, lane, vwave, vnw, tp, list_sums, pub);
    if (!list_done) list_sums();
    // (decode loop) the row of the next step is known already: ask for this wave's first tile of it
    // now, so that it travels while this row is combined and sampled
    if (next_row && wave < nt) load_tile<T>(next_row, V, wave, lane, *next_first);
    RowOut none;
    none.id = -1;
    none.pos = -1;
    none.logZ_valid = -INFINITY;
    none.logZ_all = 0.f;
    none.mine = false;
    if (SPLIT && parts > 1) {
        // Every wavefront waits until its device-scope stores have been taken by the memory system, then the
        // workgroup's arrival is counted.  The workgroup that finds all the others already there finishes the
        // row (its reads are device-scope too, and issued after the count has come back); nobody waits for anybody.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);     // vmcnt(0) expcnt(0) lgkmcnt(0)
        __syncthreads();
        if (tid == 0) {
            const uint32_t before = __hip_atomic_fetch_add(sp.arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool last = before + 1u == (uint32_t)parts;
            if (last) __hip_atomic_store(sp.arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // the next launch starts from zero
            sh.bc_i[0] = last ? 1 : 0;
        }
        __syncthreads();
        if (!sh.bc_i[0]) return none;      // uniform for the workgroup
        const int nthreads = nw * WAVE;
        for (int k = tid; k < nt; k += nthreads) {
            const float *t = (const float *)&pub->tile[k];
            sh.tile_m[k] = shared_get(t + 0);
            sh.tile_zall[k] = shared_get(t + 1);
            sh.tile_zval[k] = shared_get(t + 2);
            sh.tile_ref[k] = shared_get(t + 3);
        }
        if (mode == VALID_LIST) {
            for (int i = tid; i < n_list; i += nthreads) sh.list_e[i] = shared_get(&pub->list_e[i]);
            for (int q = tid; q < ns; q += nthreads) {
                sh.slice_m[q] = shared_get(&pub->slice_m[q]);
                sh.slice_z[q] = shared_get(&pub->slice_z[q]);
            }
        }
    }
    __syncthreads();

    // Nobody but wavefront 0 has anything left to do when the result goes to it alone and the set is not an
    // image (whose rare second pass needs every wavefront): the others leave its SIMD to it.
    if (!ALL && mode != VALID_IMAGE && wave != 0) return none;
    // ---- combine (every wave computes the same row totals from LDS; cheap, and saves a broadcast)
    float M, za;
    double zv;
    combine_tiles(sh, nt, lane, tp, mode == VALID_IMAGE, M, za, zv);
    float R = M;  // reference of the valid sums of the image path

    // ---- image path, rare case: the valid mass is below 2^-18 of the row's largest term, so sums
    // relative to the tile maxima are inaccurate or have underflowed.  Redo the valid sums relative
    // to the maximum over valid tokens (the row is re-read; it is still in cache).
    if (mode == VALID_IMAGE && zv < 3.814697265625e-06) {
        __syncthreads();  // everyone has read tile_zval
        RawTile rt;
        for (int k = wave; k < nt; k += nw) {
            load_tile<T>(row, V, k, lane, rt);
            const uint32_t word = tile_mask_word<T>(image, k, lane, V);
            const float mv = tile_valid_max<T>(rt, word, lane);
            if (lane == 0) sh.tile_ref[k] = mv;
        }
        __syncthreads();
        float Mv = -INFINITY;
        for (int k = lane; k < nt; k += WAVE) Mv = fmaxf(Mv, sh.tile_ref[k]);
        Mv = wave_max(Mv);
        __syncthreads();  // everyone has read the per-tile valid maxima
        if (Mv != -INFINITY) {
            for (int k = wave; k < nt; k += nw) {
                load_tile<T>(row, V, k, lane, rt);
                const uint32_t word = tile_mask_word<T>(image, k, lane, V);
                const float z = tile_valid_sum<T>(rt, word, lane, Mv, tp.c);
                if (lane == 0) {
                    sh.tile_zval[k] = z;
                    sh.tile_ref[k] = Mv;
                }
            }
        } else {
            for (int k = tid; k < nt; k += nw * WAVE) sh.tile_zval[k] = 0.f;
        }
        __syncthreads();
        R = Mv;
        zv = 0.0;
        for (int k = lane; k < nt; k += WAVE) zv += (double)sh.tile_zval[k];
        zv = wave_sum(zv);
    }

    // ---- locate: wave 0
    RowOut out = none;
    out.mine = ALL || wave == 0;
    if (wave == 0) {
        const float l2za = fast_log2(za);
        int id = -1, pos = -1;
        float lzv = -INFINITY;
        if (mode == VALID_IMAGE) {
            if (zv > 0.0) {
                lzv = fmaf(R - M, tp.inv, LN2F * (fast_log2((float)zv) - l2za));
                const double tau = (double)u * zv;
                // first tile whose cumulative valid weight exceeds tau
                double carry = 0.0, before = 0.0;
                int kstar = -1, klast = -1;
                for (int k0 = 0; k0 < nt && kstar < 0; k0 += WAVE) {
                    const int k = k0 + lane;
                    double w = 0.0;
                    if (k < nt && sh.tile_zval[k] > 0.f)
                        w = (double)sh.tile_zval[k] * (double)exp_scale(sh.tile_ref[k] - R, tp.c);
                    const double incl = carry + wave_incl_scan(w);
                    const uint64_t cross = __ballot(incl > tau);
                    const uint64_t have = __ballot(w > 0.0);
                    if (cross) {
                        const int l = __ffsll((long long)cross) - 1;
                        kstar = k0 + l;
                        before = lane_value(incl - w, l);
                    } else if (have) {
                        klast = k0 + 63 - __clzll((long long)have);
                    }
                    carry = last_lane(incl);
                }
                double target;
                int kt;
                if (kstar >= 0) {
                    kt = kstar;
                    target = (tau - before) / (double)exp_scale(sh.tile_ref[kt] - R, tp.c);
                } else {  // rounding: the total never exceeded tau; take the last valid token
                    kt = klast;
                    target = INFINITY;
                }
                if (kt >= 0) {   // (no tile qualifies only when NaNs have poisoned the sums: then nothing is sampled)
                    RawTile lt;
                    load_tile<T>(row, V, kt, lane, lt);
                    const uint32_t word = tile_mask_word<T>(image, kt, lane, V);
                    id = locate_in_tile<T>(lt, word, kt, lane, sh.tile_ref[kt], target, tp.c);
                }
            }
        } else if (mode == VALID_LIST) {
            float Mv = -INFINITY;
            if (ns == 1) {   // one slice (at most 64 listed tokens, the usual case): nothing to scan over
                Mv = sh.slice_m[0];
            } else {
                if (lane < ns) Mv = sh.slice_m[lane];
                Mv = wave_max(Mv);
            }
            if (Mv != -INFINITY) {
                int s;
                double target, zvl;
                if (ns == 1) {   // the general case below, written out for one slice: same values bit for bit
                    zvl = (double)sh.slice_z[0];
                    const double tau = (double)u * zvl;
                    if (zvl > tau) {
                        s = 0;
                        target = tau;
                    } else {
                        s = zvl > 0.0 ? 0 : -1;
                        target = INFINITY;
                    }
                } else {
                    double w = 0.0, sc = 0.0;
                    if (lane < ns && sh.slice_m[lane] != -INFINITY) {
                        sc = (double)exp_scale(sh.slice_m[lane] - Mv, tp.c);
                        w = (double)sh.slice_z[lane] * sc;
                    }
                    const double incl = wave_incl_scan(w);
                    zvl = last_lane(incl);
                    const double tau = (double)u * zvl;
                    const uint64_t cross = __ballot(incl > tau);
                    const uint64_t have = __ballot(w > 0.0);
                    if (cross) {
                        s = __ffsll((long long)cross) - 1;
                        target = (tau - lane_value(incl - w, s)) / lane_value(sc, s);
                    } else {
                        s = have ? 63 - __clzll((long long)have) : -1;
                        target = INFINITY;
                    }
                }
                lzv = fmaf(Mv - M, tp.inv, LN2F * (fast_log2((float)zvl) - l2za));
                // (no slice or no token qualifies only when NaNs have poisoned the sums: then nothing is sampled,
                // and above all no position outside the list is ever formed)
                const int i = s * WAVE + lane;
                const float e = (s >= 0 && i < n_list) ? sh.list_e[i] : 0.f;
                const double ic = wave_incl_scan((double)e);
                const uint64_t c2 = __ballot(e > 0.f && ic > target);
                const uint64_t h2 = __ballot(e > 0.f);
                if (c2 | h2) {
                    const int l = c2 ? __ffsll((long long)c2) - 1 : 63 - __clzll((long long)h2);
                    pos = s * WAVE + l;
                    id = (int)(sh.list_tok[pos] & PPV_NODE_TOKEN);
                }
            }
        }
        out.id = id;   // all four are wave-uniform
        out.pos = pos;
        out.logZ_valid = lzv;
        out.logZ_all = fmaf(M, tp.inv, LN2F * l2za);
        if (ALL && lane == 0) {
            sh.bc_i[0] = out.id;
            sh.bc_i[1] = out.pos;
            sh.bc_f[0] = out.logZ_valid;
            sh.bc_f[1] = out.logZ_all;
        }
    }
    if (ALL) {
        __syncthreads();
        out.id = sh.bc_i[0];
        out.pos = sh.bc_i[1];
        out.logZ_valid = sh.bc_f[0];
        out.logZ_all = sh.bc_f[1];
    }
    return out;
}

// ------------------------------------------------------------------------------------------
// constrained_sample: the valid set arrives as a packed mask.  Count its bits; a small set is
// unpacked into the token list, a large one is used as an image.
template <typename T, bool SMALL, bool PIPE, bool SPLIT>
__global__ __launch_bounds__(SMALL ? SMALL_TILES * WAVE : MAX_WAVES * WAVE) void sample_kernel(const T *__restrict__ logits, int64_t row_stride,
                                                                  const uint32_t *__restrict__ mask,
                                                                  const float *__restrict__ uniforms, int V,
                                                                  int n_words, int list_max,
                                                                  int32_t *__restrict__ ids,
                                                                  float *__restrict__ logZ_valid,
                                                                  float *__restrict__ logZ_all, Temper tp,
                                                                  int split_shift, SplitScratch *scratch) {
    using G = TileGeom<T>;
    using SH = typename std::conditional<SMALL, RowSharedSmall, RowShared>::type;
    __shared__ SH sh;
    // SPLIT: a row is shared by 1 << split_shift consecutive workgroups
    const int b = SPLIT ? (int)(blockIdx.x >> split_shift) : (int)blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int nw = blockDim.x / WAVE;
    Split sp;
    sp.parts = SPLIT ? 1 << split_shift : 1;
    sp.part = SPLIT ? (int)(blockIdx.x & (unsigned)(sp.parts - 1)) : 0;
    sp.row = SPLIT ? &scratch->row[b] : nullptr;
    sp.arrivals = SPLIT ? &scratch->arrivals[b] : nullptr;
    const int vwave = sp.part * nw + wave;
    const T *row = logits + (size_t)b * (size_t)row_stride;
    const uint32_t *mrow = mask + (size_t)b * (size_t)n_words;
    const int nt = (V + G::TILE - 1) / G::TILE;
    // The mask row is read as quads of four words per lane: one wavefront load covers 256 words (8,192 tokens), so a
    // wavefront has few loads to wait for, and those it has are requested two at a time and before the logits tile
    // (memory answers a wavefront in the order of its requests: the few bytes the next steps wait for must not queue
    // behind the 4 KB tile; one word per lane and tile at a time cost a memory round trip per tile, which at 63
    // tiles on 4 wavefronts was most of the kernel).  Words past the row read as 0.
    const int n_groups = ((n_words + 3) / 4 + WAVE - 1) / WAVE;   // <= 32 (PPV_MAX_VOCAB / 8192)
    struct Quad {
        uint32_t w[4];
    };
    auto load_quad = [&](int g) {
        Quad q;
        const int wi = (g * WAVE + lane) * 4;
        if (wi + 4 < n_words) {   // inside the row and not its last word: four loads off one address
            const uint32_t *p = mrow + wi;
#pragma unroll
            for (int j = 0; j < 4; j++) q.w[j] = p[j];
        } else {                  // the row's end: clamped loads, bits past V cleared, 0 beyond
#pragma unroll
            for (int j = 0; j < 4; j++) q.w[j] = image_word(mrow, wi + j, V);
        }
        return q;
    };
    auto bits_of = [](const Quad &q) { return (int)(__popc(q.w[0]) + __popc(q.w[1]) + __popc(q.w[2]) + __popc(q.w[3])); };
    const Quad q0 = load_quad(wave), q1 = load_quad(wave + nw);   // (a group past the row: all zero)
    RawTile first;
    if (vwave < nt) load_tile<T>(row, V, vwave, lane, first);   // in flight during the mask work

    // valid tokens per group of 64 quads (kept in the tile_cnt array: there are fewer groups than tiles)
    const int incl0 = wave_incl_scan(bits_of(q0));
    {
        const int incl1 = wave_incl_scan(bits_of(q1));
        if (lane == WAVE - 1) {
            if (wave < n_groups) sh.tile_cnt[wave] = incl0;
            if (wave + nw < n_groups) sh.tile_cnt[wave + nw] = incl1;
        }
    }
    for (int g = wave + 2 * nw; g < n_groups; g += nw) {   // long rows on few wavefronts
        const int c = wave_sum(bits_of(load_quad(g)));
        if (lane == 0) sh.tile_cnt[g] = c;
    }
    __syncthreads();
    const int total = wave_sum(lane < n_groups ? sh.tile_cnt[lane] : 0);
    const int mode = total == 0 ? VALID_NONE : (total <= list_max ? VALID_LIST : VALID_IMAGE);
    if (mode == VALID_LIST) {
        // a group's valid tokens go to their places in the list: after those of the groups before it, in lane order
        auto unpack_group = [&](int g, const Quad &q, int incl) {
            const int before = wave_sum(lane < g ? sh.tile_cnt[lane] : 0);
            int at = before + incl - bits_of(q);
            const int wi = (g * WAVE + lane) * 4;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                uint32_t w = q.w[j];
                while (w) {
                    const int bit = __ffs((int)w) - 1;
                    sh.list_tok[at++] = (uint32_t)((wi + j) * 32 + bit);
                    w &= w - 1u;
                }
            }
        };
        if (wave < n_groups && sh.tile_cnt[wave] != 0) unpack_group(wave, q0, incl0);
        for (int g = wave + nw; g < n_groups; g += nw) {
            if (sh.tile_cnt[g] == 0) continue;   // (uniform) most groups of a short list hold nothing
            const Quad q = g == wave + nw ? q1 : load_quad(g);
            unpack_group(g, q, wave_incl_scan(bits_of(q)));
        }
        __syncthreads();
    }
    RowOut r = row_sample<T, PIPE, SH, false, SPLIT>(row, V, first, mode, mode == VALID_LIST ? total : 0, mrow, uniforms[b], sh, tid, nw, tp, sp);
    if (r.mine && tid == 0) {
        ids[b] = r.id;
        logZ_valid[b] = r.logZ_valid;
        if (logZ_all) logZ_all[b] = r.logZ_all;
    }
}

// Rows of a single tile (V <= 1,024 fp32 / 2,048 bf16 tokens): one wavefront per row, four rows per workgroup,
// everything in registers -- no LDS, no barrier.  The valid set is applied as bits in the tile (as on the image
// path of the general kernel, with the same rescue when the valid tokens lie far below the row maximum).
constexpr int ONE_TILE_ROWS = 4;
template <typename T>
__global__ __launch_bounds__(ONE_TILE_ROWS *WAVE) void sample_one_tile_kernel(const T *__restrict__ logits, int64_t row_stride,
                                                                              const uint32_t *__restrict__ mask,
                                                                              const float *__restrict__ uniforms, int B,
                                                                              int V, int n_words, int32_t *__restrict__ ids,
                                                                              float *__restrict__ logZ_valid,
                                                                              float *__restrict__ logZ_all, Temper tp) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int b = blockIdx.x * ONE_TILE_ROWS + threadIdx.x / WAVE;
    if (b >= B) return;   // uniform per wavefront
    const T *row = logits + (size_t)b * (size_t)row_stride;
    const uint32_t word = tile_mask_word<T>(mask + (size_t)b * (size_t)n_words, 0, lane, V);
    const float u = uniforms[b];
    RawTile rt;
    load_tile<T>(row, V, 0, lane, rt);
    float m, zall, zval;
    tile_stats<T, true>(rt, word, lane, tp, m, zall, zval);
    const float l2za = fast_log2(zall);
    int id = -1;
    float lzv = -INFINITY, ref = m;
    if (__ballot(word != 0u)) {
        if (zval < 3.814697265625e-06f) {   // below 2^-18 of the largest term: sum again, relative to the valid maximum
            ref = tile_valid_max<T>(rt, word, lane);
            zval = ref != -INFINITY ? tile_valid_sum<T>(rt, word, lane, ref, tp.c) : 0.f;
        }
        if (zval > 0.f) {
            lzv = fmaf(ref - m, tp.inv, LN2F * (fast_log2(zval) - l2za));
            id = locate_in_tile<T>(rt, word, 0, lane, ref, (double)u * (double)zval, tp.c);
        }
    }
    if (lane == 0) {
        ids[b] = id;
        logZ_valid[b] = lzv;
        if (logZ_all) logZ_all[b] = fmaf(m, tp.inv, LN2F * l2za);
    }
}

// ppv_sample_next for rows of a single tile: the prefix walk of mask_rows_kernel and the arithmetic of
// sample_one_tile_kernel in one wavefront per row; the valid set never exists outside this wavefront's registers
// (lane l holds word l of it, which is also word l of the tile's mask).
template <typename T>
__global__ __launch_bounds__(ONE_TILE_ROWS *WAVE) void sample_next_one_tile_kernel(
    IndexView ix, const int32_t *__restrict__ prefixes, int32_t stride, const int32_t *__restrict__ lens,
    const T *__restrict__ logits, int64_t row_stride, const float *__restrict__ uniforms, int B, int32_t *__restrict__ ids,
    float *__restrict__ logZ_valid, uint8_t *__restrict__ member, Temper tp) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int b = blockIdx.x * ONE_TILE_ROWS + threadIdx.x / WAVE;
    if (b >= B) return;   // uniform per wavefront
    const int V = ix.vocab, n_words = ix.n_words;
    const int32_t mine = first_tokens(prefixes + (size_t)b * (size_t)stride, stride, lane);   // before the tile: answers come in order
    int t = lens[b];
    const float u = uniforms[b];
    RawTile rt;
    load_tile<T>(logits + (size_t)b * (size_t)row_stride, V, 0, lane, rt);   // in flight during the walk
    t = t < 0 ? 0 : (t > stride ? stride : t);
    const Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, mine, t, lane);
    uint32_t word = 0u;
    const uint32_t nchild = w.found ? w.ce - w.cb : 0u;
    if (nchild > ix.heavy_min) {   // ready-made image
        if (lane < n_words) word = ix.heavy_bits[(size_t)heavy_slot_of(ix, w.node) * (size_t)n_words + lane];
    } else if (nchild > 0u) {      // nchild <= heavy_min <= 64: one child per lane
        const uint32_t tok = (uint32_t)lane < nchild ? (ix.ent[w.cb + (uint32_t)lane].tok & PPV_NODE_TOKEN) : 0u;
        for (uint32_t i = 0; i < nchild; i++) {   // uniform trip count
            const uint32_t v = (uint32_t)__builtin_amdgcn_readlane((int)tok, (int)i);
            if ((uint32_t)lane == (v >> 5)) word |= 1u << (v & 31u);
        }
    }
    float m, zall, zval;
    tile_stats<T, true>(rt, word, lane, tp, m, zall, zval);
    const float l2za = fast_log2(zall);
    int id = -1;
    float lzv = -INFINITY, ref = m;
    if (__ballot(word != 0u)) {
        if (zval < 3.814697265625e-06f) {   // below 2^-18 of the largest term: sum again, relative to the valid maximum
            ref = tile_valid_max<T>(rt, word, lane);
            zval = ref != -INFINITY ? tile_valid_sum<T>(rt, word, lane, ref, tp.c) : 0.f;
        }
        if (zval > 0.f) {
            lzv = fmaf(ref - m, tp.inv, LN2F * (fast_log2(zval) - l2za));
            id = locate_in_tile<T>(rt, word, 0, lane, ref, (double)u * (double)zval, tp.c);
        }
    }
    if (lane == 0) {
        ids[b] = id;
        if (logZ_valid) logZ_valid[b] = lzv;
        if (member) member[b] = w.member ? 1 : 0;
    }
}

// ------------------------------------------------------------------------------------------
// ppv_decode_begin: one wavefront per row walks the row's current prefix and leaves the cursor.
__global__ __launch_bounds__(MASK_THREADS) void decode_begin_kernel(IndexView ix, const int32_t *__restrict__ prefixes,
                                                                    int32_t stride, const int32_t *__restrict__ lens,
                                                                    int B, RowState *__restrict__ state,
                                                                    uint8_t *__restrict__ active,
                                                                    float *__restrict__ logx) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int b = blockIdx.x * (MASK_THREADS / WAVE) + threadIdx.x / WAVE;
    if (b >= B) return;  // uniform per wave
    const int32_t mine = first_tokens(prefixes + (size_t)b * (size_t)stride, stride, lane);
    int t = lens[b];
    t = t < 0 ? 0 : (t > stride ? stride : t);
    const Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, mine, t, lane);
    if (lane == 0) {
        RowState st;
        st.node = w.found ? w.node : PPV_NO_SLOT;
        st.cb = w.found ? w.cb : 0u;
        st.ce = w.found ? w.ce : 0u;
        st.slot = (w.found && w.ce - w.cb > ix.heavy_min) ? heavy_slot_of(ix, w.node) : PPV_NO_SLOT;
        st.tok0 = st.child0 = st.child1 = st.flags = 0u;   // nothing looked ahead
        state[b] = st;
        active[b] = (w.found && !w.member) ? 1 : 0;
        if (logx) logx[b] = 0.f;
    }
}

// ppv_decode_begin_empty: every row starts from the empty candidate.  The cursor is the root's, the same for all
// rows: no prefix to read, no walk; the lengths are written too, so that a decode loop needs no separate fill.
__global__ __launch_bounds__(MASK_THREADS) void decode_begin_empty_kernel(IndexView ix, int B, int32_t *__restrict__ lens,
                                                                          RowState *__restrict__ state,
                                                                          uint8_t *__restrict__ active,
                                                                          float *__restrict__ logx) {
    const int b = blockIdx.x * MASK_THREADS + threadIdx.x;
    if (b >= B) return;
    RowState st;
    st.node = 0u;
    st.cb = ix.ent[0].child;
    st.ce = ix.ent[1].child;
    st.slot = st.ce - st.cb > ix.heavy_min ? heavy_slot_of(ix, 0u) : PPV_NO_SLOT;
    st.tok0 = st.child0 = st.child1 = st.flags = 0u;   // nothing looked ahead
    lens[b] = 0;
    state[b] = st;
    active[b] = 1;   // the empty sequence is a prefix of every member and is no member itself (members are not empty)
    if (logx) logx[b] = 0.f;
}

// ppv_decode_step / ppv_decode_loop: take the children of the row's prefix as the valid set (list, or
// the ready-made image of a heavy node), stream + sample, append, and report whether the extended
// row is in S.  LOOP: the same for n_steps steps in one launch, one workgroup staying with its row;
// the cursor lives in registers and the next step's first tiles are requested before the current
// step is sampled (only when no child of the current prefix is a member, i.e. the row is certain to
// go on, so nothing is fetched in vain).
template <typename T, bool LOOP, bool PIPE, bool SPLIT, bool REG>
__global__ __launch_bounds__(LOOP ? (REG ? CHAIN_WAVES : LOOP_WAVES) * WAVE : MAX_WAVES * WAVE) void decode_kernel(
    IndexView ix, int32_t *__restrict__ prefixes, int32_t stride, int32_t *__restrict__ lens,
    uint8_t *__restrict__ active, RowState *__restrict__ state, const T *__restrict__ logits, int64_t row_stride,
    int64_t step_stride, const float *__restrict__ uniforms, int n_steps, int B, int32_t *__restrict__ ids,
    float *__restrict__ logZ_valid, float *__restrict__ logx, Temper tp, int split_shift, SplitScratch *scratch,
    int flags) {
    // flags bit 1 (ppv_decode_first_step): every row starts from the empty candidate here and now -- no flags, length
    // or cursor are read, the root's cursor is taken instead, and all of them are written at the end.
    const int advance = flags & 1;
    const bool fresh = (flags & 2) != 0;
    // advance == 0 (ppv_sample_next): every row takes part, a token is drawn, and nothing of the caller's rows is
    // changed (no append, no cursor, no flags)
    using G = TileGeom<T>;
    constexpr bool STEP_REG = REG && !LOOP, LOOP_REG = REG && LOOP;
    // (the loop kernel's fast steps alternate between two sets of tile statistics, see below)
    __shared__ RowShared shs[LOOP_REG ? 2 : 1];
    RowShared &sh = shs[0];
    // SPLIT: a row is shared by 1 << split_shift consecutive workgroups (never in the loop kernel)
    static_assert(!(LOOP && SPLIT), "the loop kernel keeps a row in one workgroup");
    const int b = SPLIT ? (int)(blockIdx.x >> split_shift) : (int)blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int nw = blockDim.x / WAVE;
    Split sp;
    sp.parts = SPLIT ? 1 << split_shift : 1;
    sp.part = SPLIT ? (int)(blockIdx.x & (unsigned)(sp.parts - 1)) : 0;
    sp.row = SPLIT ? &scratch->row[b] : nullptr;
    sp.arrivals = SPLIT ? &scratch->arrivals[b] : nullptr;
    const int vwave = sp.part * nw + wave;
    // REG: the per-step kernel of small batches keeps a list of at most 63 children in wavefront 0's registers and
    // looks one level ahead for the next cursor (see RowState); the loop kernel, split rows, long rows and large
    // batches (where the registers this costs would mean fewer rows per compute unit) use the list in LDS
    static_assert(!REG || (!SPLIT && !PIPE), "the register list is for short turns in unsplit rows");
    // the independent per-row loads go out together
    uint8_t on = active ? active[b] : (uint8_t)1;
    int t = lens[b];
    RowState st;
    if (state) st = state[b];
    else st.flags = 0u;
    float u = uniforms[b];
    // the running score is read now, not when it is updated at the very end (a load there would stand between the
    // sample and the kernel's last store); unconditional, from an address that always exists
    float logx_in = (logx ? logx : uniforms)[b];
    if (fresh) {   // (uniform) what was loaded is set aside -- the loads themselves stay unconditional, so that the
                   // waits after them stay exact -- for the root's cursor, as ppv_decode_begin_empty writes it
        on = 1;
        t = 0;
        logx_in = 0.f;
        st.node = 0u;
        st.cb = ix.ent[0].child;
        st.ce = ix.ent[1].child;
        st.slot = st.ce - st.cb > ix.heavy_min ? heavy_slot_of(ix, 0u) : PPV_NO_SLOT;
        st.tok0 = st.child0 = st.child1 = st.flags = 0u;
    }
    if (!on) return;  // uniform for the workgroup
    const int V = ix.vocab;
    const T *row = logits + (size_t)b * (size_t)row_stride;
    const int nt = (V + G::TILE - 1) / G::TILE;
    // The cursor comes from memory that the caller owns.  One that cannot be a cursor of this index (a state
    // that never went through ppv_decode_begin, or of another index) must not send a load out of bounds:
    // such a row is treated as having no valid token and retires; a look-ahead that cannot be one is ignored.
    auto check_cursor = [&]() {
        const uint32_t nc = st.ce - st.cb;
        const bool sane = st.node < ix.n_nodes && st.cb <= st.ce && st.ce <= ix.n_nodes &&
                          (st.slot == PPV_NO_SLOT ? nc <= ix.heavy_min : st.slot < ix.n_heavy);
        if (!sane) {
            st.cb = st.ce = 0u;
            st.slot = PPV_NO_SLOT;
        }
        if (st.flags != 1u || (st.tok0 & PPV_NODE_TOKEN) >= (uint32_t)V || st.child0 > st.child1 || st.child1 > ix.n_nodes)
            st.flags = 0u;
    };
    // Register list (wavefront 0): entry i of the node's children in lane i, one entry more than there are children
    // (it closes the last child's own range), and under each child the look-ahead for the next cursor.
    RegList rl;
    rl.on = false;
    rl.have_gx = false;
    rl.tokw = 0u;
    rl.gx = -INFINITY;
    uint32_t rl_child = 0u;                              // lane i <= n: child offset of entry i
    uint32_t ahead_tok = 0u, ahead_child = 0u, ahead_next = 0u;   // lane i < n: ent[child_i].tok / .child, ent[child_i + 1].child
    auto look_ahead = [&](int n) {   // (wavefront 0) every address is clamped into the entry array
        if (lane < n) {
            const uint32_t a0 = rl_child < ix.n_nodes ? rl_child : ix.n_nodes;
            const uint32_t a1 = a0 < ix.n_nodes ? a0 + 1u : ix.n_nodes;
            const NodeEnt e0 = ix.ent[a0];
            ahead_tok = e0.tok;
            ahead_child = e0.child;
            ahead_next = ix.ent[a1].child;
        }
    };
    if (STEP_REG && state) {
        // with a cursor the small loads go out before the 4 KB tile: memory answers a wavefront in request order
        check_cursor();
        const uint32_t nc = st.ce - st.cb;
        rl.on = nc >= 1u && nc < (uint32_t)WAVE && st.slot == PPV_NO_SLOT;   // (uniform)
        if (rl.on && wave == 0) {
            if (nc == 1u && st.flags == 1u) {   // the cursor knows its only child: its logit can be asked for at once
                rl.tokw = lane == 0 ? st.tok0 : 0u;
                rl_child = lane == 0 ? st.child0 : st.child1;
                rl.have_gx = true;
                if (lane == 0) {
                    const uint32_t v = st.tok0 & PPV_NODE_TOKEN;
                    if (sizeof(T) == 4) rl.gx = __uint_as_float(((const uint32_t *)row)[v]);
                    else rl.gx = __uint_as_float(((uint32_t)((const uint16_t *)row)[v]) << 16);
                }
                look_ahead(1);
            } else if ((uint32_t)lane <= nc) {
                const NodeEnt e = ix.ent[st.cb + (uint32_t)lane];
                rl.tokw = e.tok;
                rl_child = e.child;
            }
        }
        rl.have_gx = __builtin_amdgcn_readfirstlane(rl.have_gx ? 1 : 0) != 0 && wave == 0;
    }
    RawTile first;
    if (vwave < nt) load_tile<T>(row, V, vwave, lane, first);   // in flight during the index work
    t = t < 0 ? 0 : (t > stride ? stride : t);
    if (!state) {  // no cursor: locate the prefix from the root (wave 0), then share it
        if (wave == 0) {
            const int32_t mine = first_tokens(prefixes + (size_t)b * (size_t)stride, stride, lane);
            const Walk w = walk_prefix(ix, prefixes + (size_t)b * (size_t)stride, mine, t, lane);
            if (lane == 0) {
                sh.bc_i[4] = (int)(w.found ? w.node : PPV_NO_SLOT);
                sh.bc_i[5] = (int)(w.found ? w.cb : 0u);
                sh.bc_i[6] = (int)(w.found ? w.ce : 0u);
            }
        }
        __syncthreads();
        st.node = (uint32_t)sh.bc_i[4];
        st.cb = (uint32_t)sh.bc_i[5];
        st.ce = (uint32_t)sh.bc_i[6];
        st.slot = (st.node != PPV_NO_SLOT && st.ce - st.cb > ix.heavy_min) ? heavy_slot_of(ix, st.node) : PPV_NO_SLOT;
        __syncthreads();
    }
    if (!(STEP_REG && state)) check_cursor();
    if (STEP_REG && rl.on) {
        // ---- a short list in wavefront 0's registers.  The sample depends on the listed logits alone, not on the
        // row's totals: wavefront 0 draws the token and works out the next cursor while its tile is still on its
        // way; after the barrier only the stores, the totals and the two masses are left.  (Nothing is stored before
        // the barrier: the other wavefronts read the row's flags and cursor when they start, and one that starts
        // late must not find them changed.)
        const int n = (int)(st.ce - st.cb);
        ListPick pk;
        pk.id = -1;
        pk.pos = -1;
        pk.Mv = -INFINITY;
        pk.zvl = 0.0;
        bool drew = false;
        RowState nx = st;
        uint32_t tokw = 0u;
        if (wave == 0) {
            if (!rl.have_gx) {   // (waits for the entries)
                if (lane < n) {
                    const uint32_t v = rl.tokw & PPV_NODE_TOKEN;
                    if (sizeof(T) == 4) rl.gx = __uint_as_float(((const uint32_t *)row)[v]);
                    else rl.gx = __uint_as_float(((uint32_t)((const uint16_t *)row)[v]) << 16);
                }
                look_ahead(n);
            }
            pk = reg_list_pick(rl.gx, rl.tokw, n, u, lane, tp);
            const bool room = t < stride || !advance;
            drew = pk.id >= 0 && room;
            if (drew) {   // (uniform) the sampled child's entry, the one after it and its look-ahead, out of the lanes
                nx.node = st.cb + (uint32_t)pk.pos;
                tokw = lane_value(rl.tokw, pk.pos);
                nx.cb = lane_value(rl_child, pk.pos);
                nx.ce = lane_value(rl_child, pk.pos + 1);
                nx.tok0 = lane_value(ahead_tok, pk.pos);
                nx.child0 = lane_value(ahead_child, pk.pos);
                nx.child1 = lane_value(ahead_next, pk.pos);
                nx.flags = 1u;
                nx.slot = (tokw & PPV_NODE_HEAVY) ? heavy_slot_of(ix, nx.node) : PPV_NO_SLOT;
            }
        }
        struct {
            __device__ void operator()() const {}
        } nothing;
        stream_tiles<T, false, false, RowShared>(row, V, first, nullptr, sh, lane, wave, nw, tp, nothing, nullptr);
        __syncthreads();
        if (wave != 0) return;
        if (lane == 0) {
            if (ids) ids[b] = drew ? pk.id : -1;
            if (drew) {
                if (advance) {
                    prefixes[(size_t)b * (size_t)stride + t] = pk.id;
                    lens[b] = t + 1;
                    state[b] = nx;
                    if (tokw & PPV_NODE_TERMINAL) active[b] = 0;   // the extended row is itself a member
                    else if (fresh) active[b] = 1;
                }
            } else if (advance) {   // the row stops outside S: no valid token of positive weight, or no room
                if (logx) logx[b] = -INFINITY;
                active[b] = 0;
                if (fresh) {
                    lens[b] = 0;
                    state[b] = st;
                }
            }
        }
        if (pk.Mv == -INFINITY) {   // (uniform) no listed token has positive weight
            if (lane == 0 && logZ_valid) logZ_valid[b] = -INFINITY;
            return;
        }
        float M, za;
        double zv;
        combine_tiles(sh, nt, lane, tp, false, M, za, zv);
        const float lzv = fmaf(pk.Mv - M, tp.inv, LN2F * (fast_log2((float)pk.zvl) - fast_log2(za)));
        if (lane == 0) {
            if (logZ_valid) logZ_valid[b] = lzv;
            if (advance && logx && drew) logx[b] = logx_in + lzv;
        }
        return;
    }
    // running log importance score (tid 0); started from the stored value so that the additions happen in
    // the same order as with one launch per step
    float lx = (LOOP && logx) ? logx_in : 0.f;
    bool done = false;
    // LOOP_REG: hand-over from wavefront 0 to the workgroup, written before a fast step's barrier and read after it
    __shared__ struct {
        int done, drew;
        RowState nx;
    } hand[2];
    for (int s = 0; s < n_steps; s++) {
        const uint32_t cb = st.cb, ce = st.ce, slot = st.slot;
        const int nchild = (int)(ce - cb);
        const int mode = nchild == 0 ? VALID_NONE : (slot != PPV_NO_SLOT ? VALID_IMAGE : VALID_LIST);
        if (LOOP_REG && mode == VALID_LIST && nchild == 1 && st.flags == 1u && V % G::EPL == 0 && nw >= 2 &&
            nt <= 2 * (nw - 1)) {
            // ---- A chain of prefixes with one child each, the cursor knowing the child (nearly all of a long
            // sequence below its first levels).  Wavefront 0 only draws tokens: each step it takes the listed
            // logit that it asked for a step earlier, advances the cursor, asks for the next step's logit and
            // look-ahead, and after the step's barrier adds up the row's totals.  The other wavefronts only stream:
            // two tiles each, the next row's tiles requested before this row's are reduced, in two sets of registers
            // that swap roles from step to step, so that there is no copy of, no condition on and no wait for a
            // tile that is still on its way.  One barrier per step; statistics and hand-over alternate between two
            // buffers as in the fast step below.  The chain ends with the row (its last step asks for 16 bytes of
            // its own row instead of a next row), or at a prefix that is not of this kind, which the code below
            // takes from there.
            const int ntw = nw - 1;
            const int wave_s = __builtin_amdgcn_readfirstlane(wave);
            auto next_in_chain = [&](const RowState &c) {
                return c.ce - c.cb == 1u && c.flags == 1u && c.slot == PPV_NO_SLOT;
            };
            // whether the row has a step after this one (known from the cursor before the token is drawn)
            auto row_goes_on = [&]() { return !(st.tok0 & PPV_NODE_TERMINAL) && s + 1 < n_steps && t + 1 < stride; };
            bool finished = false;   // the row is done, or out of steps
            if (wave_s == 0) {
                float gx = -INFINITY;
                uint32_t a_tok = 0u, a_child = 0u, a_next = 0u;
                auto ask = [&](const T *r, const RowState &c, float &g, uint32_t &x0, uint32_t &x1, uint32_t &x2) {
                    if (lane == 0) {
                        const uint32_t v = c.tok0 & PPV_NODE_TOKEN;
                        if (sizeof(T) == 4) g = __uint_as_float(((const uint32_t *)r)[v]);
                        else g = __uint_as_float(((uint32_t)((const uint16_t *)r)[v]) << 16);
                        const uint32_t a0 = c.child0 < ix.n_nodes ? c.child0 : ix.n_nodes;
                        const uint32_t a1 = a0 < ix.n_nodes ? a0 + 1u : ix.n_nodes;
                        const NodeEnt g0 = ix.ent[a0];
                        x0 = g0.tok;
                        x1 = g0.child;
                        x2 = ix.ent[a1].child;
                    }
                };
                ask(row, st, gx, a_tok, a_child, a_next);
                for (;;) {
                    const bool more = row_goes_on();
                    const ListPick pk = reg_list_pick(gx, lane == 0 ? st.tok0 : 0u, 1, u, lane, tp);
                    const bool drew = pk.id >= 0 && t < stride;
                    RowState nx = st;
                    nx.flags = 0u;
                    if (drew) {
                        nx.node = st.cb;
                        nx.cb = st.child0;
                        nx.ce = st.child1;
                        nx.tok0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)a_tok);
                        nx.child0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)a_child);
                        nx.child1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)a_next);
                        nx.flags = 1u;
                        nx.slot = (st.tok0 & PPV_NODE_HEAVY) ? heavy_slot_of(ix, nx.node) : PPV_NO_SLOT;
                    }
                    const bool chain_on = drew && more && next_in_chain(nx);
                    // (the answers go straight into the registers the next step reads, whose old contents are used up:
                    // a copy of a value that is still on its way would have to wait for it)
                    const float mv = pk.Mv;
                    const double zvl = pk.zvl;
                    const int drawn = pk.id;
                    if (chain_on) ask(row + step_stride, nx, gx, a_tok, a_child, a_next);
                    if (drew && s + 1 < n_steps) u = uniforms[(size_t)(s + 1) * (size_t)B + b];
                    const bool ends = !drew || (st.tok0 & PPV_NODE_TERMINAL) != 0u;
                    if (lane == 0) {
                        hand[s & 1].done = ends ? 1 : 0;
                        hand[s & 1].drew = drew ? 1 : 0;
                        hand[s & 1].nx = nx;
                        if (drew) prefixes[(size_t)b * (size_t)stride + t] = drawn;
                        if (ids) ids[(size_t)s * (size_t)B + b] = drew ? drawn : -1;
                        if (!drew) lx = -INFINITY;   // the row stops outside S
                        if (logZ_valid && mv == -INFINITY) logZ_valid[(size_t)s * (size_t)B + b] = -INFINITY;
                    }
                    __syncthreads();
                    if (mv != -INFINITY) {
                        float M, za;
                        double zv;
                        combine_tiles(shs[s & 1], nt, lane, tp, false, M, za, zv);
                        const float lzv = fmaf(mv - M, tp.inv, LN2F * (fast_log2((float)zvl) - fast_log2(za)));
                        if (lane == 0) {
                            if (logZ_valid) logZ_valid[(size_t)s * (size_t)B + b] = lzv;
                            if (drew) lx += lzv;
                        }
                    }
                    done = ends;
                    if (drew) {
                        t += 1;
                        st = nx;
                    }
                    if (ends || s + 1 == n_steps) {
                        finished = true;
                        break;
                    }
                    s += 1;
                    row += step_stride;
                    if (!chain_on) break;
                }
            } else {
                const int k0 = wave_s - 1, k1 = wave_s - 1 + ntw;   // (a tile past the row reads as -inf and is not recorded)
                RawTile A0, A1, B0, B1;
                load_tile_clamped<T>(row, V, k0, lane, A0);
                load_tile_clamped<T>(row, V, k1, lane, A1);
                auto reduce = [&](RawTile &tile, int k, RowShared &cur) {
                    pad_tile_tail<T>(tile, V, k, lane);
                    float m, zall, zval;
                    tile_stats<T, false>(tile, 0u, lane, tp, m, zall, zval);
                    if (lane == 0 && k < nt) {
                        cur.tile_m[k] = m;
                        cur.tile_zall[k] = zall;
                        cur.tile_zval[k] = zval;
                        cur.tile_ref[k] = m;
                    }
                };
                // one step on the tiles (c0, c1), the next row's tiles requested into (n0, n1) first.
                // Returns true while the chain goes on.
                auto chain_step = [&](RawTile &c0, RawTile &c1, RawTile &n0, RawTile &n1) {
                    const bool more = row_goes_on();
                    const T *nrow = more ? row + step_stride : row;   // no next row: one line of this one (same loads,
                    const int Vn = more ? V : G::EPL;                 // all clamped to the row's first 16 bytes)
                    load_tile_clamped<T>(nrow, Vn, k0, lane, n0);
                    load_tile_clamped<T>(nrow, Vn, k1, lane, n1);
                    reduce(c0, k0, shs[s & 1]);
                    reduce(c1, k1, shs[s & 1]);
                    __syncthreads();
                    const bool ends = hand[s & 1].done != 0;
                    const bool drew = hand[s & 1].drew != 0;
                    done = ends;
                    if (drew) {
                        t += 1;
                        st = hand[s & 1].nx;
                    }
                    if (ends || s + 1 == n_steps) {
                        finished = true;
                        return false;
                    }
                    s += 1;
                    row += step_stride;
                    return drew && more && next_in_chain(st);
                };
                while (chain_step(A0, A1, B0, B1) && chain_step(B0, B1, A0, A1)) {
                }
            }
            if (finished) break;
            // a prefix of another kind: its step starts below from the row's first tile as the other steps know it
            if (wave < nt) load_tile<T>(row, V, wave, lane, first);
            if (wave_s != 0) u = uniforms[(size_t)s * (size_t)B + b];
            s -= 1;
            continue;
        }
        if (LOOP_REG && mode == VALID_LIST && nchild < WAVE) {
            // ---- A fast step: the children are a short list in wavefront 0's registers.  Wavefront 0 draws the
            // token and works out the next cursor (with its look-ahead) while the tiles are on their way, and hands
            // both to the workgroup through LDS; the step's one barrier says that the tiles' statistics and the
            // hand-over are there.  After it the other wavefronts go straight on to the next step while wavefront 0
            // adds up the row's totals: statistics and hand-over alternate between two buffers, and a buffer is not
            // written again before everybody has passed the barrier after the one it was read behind.
            RowShared &cur = shs[s & 1];
            const bool known = nchild == 1 && st.flags == 1u;   // the cursor knows its only child
            uint32_t e_tok = 0u, e_child = 0u, a_tok = 0u, a_child = 0u, a_next = 0u;
            float gx = -INFINITY;
            if (wave == 0) {
                if (known) {
                    e_tok = lane == 0 ? st.tok0 : 0u;
                    e_child = lane == 0 ? st.child0 : st.child1;
                } else if (lane <= nchild) {
                    const NodeEnt e = ix.ent[cb + (uint32_t)lane];
                    e_tok = e.tok;
                    e_child = e.child;
                }
                if (lane < nchild) {
                    const uint32_t v = e_tok & PPV_NODE_TOKEN;
                    if (sizeof(T) == 4) gx = __uint_as_float(((const uint32_t *)row)[v]);
                    else gx = __uint_as_float(((uint32_t)((const uint16_t *)row)[v]) << 16);
                    const uint32_t a0 = e_child < ix.n_nodes ? e_child : ix.n_nodes;
                    const uint32_t a1 = a0 < ix.n_nodes ? a0 + 1u : ix.n_nodes;
                    const NodeEnt g0 = ix.ent[a0];
                    a_tok = g0.tok;
                    a_child = g0.child;
                    a_next = ix.ent[a1].child;
                }
            }
            ListPick pk;
            pk.id = -1;
            pk.pos = -1;
            pk.Mv = -INFINITY;
            pk.zvl = 0.0;
            if (wave == 0) {
                pk = reg_list_pick(gx, e_tok, nchild, u, lane, tp);
                const bool drew = pk.id >= 0 && t < stride;
                RowState nx = st;
                nx.flags = 0u;
                uint32_t tokw = 0u;
                if (drew) {
                    nx.node = cb + (uint32_t)pk.pos;
                    tokw = lane_value(e_tok, pk.pos);
                    nx.cb = lane_value(e_child, pk.pos);
                    nx.ce = lane_value(e_child, pk.pos + 1);
                    nx.tok0 = lane_value(a_tok, pk.pos);
                    nx.child0 = lane_value(a_child, pk.pos);
                    nx.child1 = lane_value(a_next, pk.pos);
                    nx.flags = 1u;
                    nx.slot = (tokw & PPV_NODE_HEAVY) ? heavy_slot_of(ix, nx.node) : PPV_NO_SLOT;
                }
                if (lane == 0) {
                    hand[s & 1].done = (!drew || (tokw & PPV_NODE_TERMINAL)) ? 1 : 0;
                    hand[s & 1].drew = drew ? 1 : 0;
                    hand[s & 1].nx = nx;
                    if (drew) prefixes[(size_t)b * (size_t)stride + t] = pk.id;
                    if (ids) ids[(size_t)s * (size_t)B + b] = drew ? pk.id : -1;
                    if (!drew) lx = -INFINITY;   // the row stops outside S
                    if (logZ_valid && pk.Mv == -INFINITY) logZ_valid[(size_t)s * (size_t)B + b] = -INFINITY;
                }
            }
            struct {
                __device__ void operator()() const {}
            } nothing;
            stream_tiles<T, false, false, RowShared>(row, V, first, nullptr, cur, lane, wave, nw, tp, nothing, nullptr);
            __syncthreads();
            done = hand[s & 1].done != 0;
            const bool drew = hand[s & 1].drew != 0;
            if (drew) {
                t += 1;
                st = hand[s & 1].nx;
            }
            if (wave == 0 && pk.Mv != -INFINITY) {
                float M, za;
                double zv;
                combine_tiles(cur, nt, lane, tp, false, M, za, zv);
                const float lzv = fmaf(pk.Mv - M, tp.inv, LN2F * (fast_log2((float)pk.zvl) - fast_log2(za)));
                if (lane == 0) {
                    if (logZ_valid) logZ_valid[(size_t)s * (size_t)B + b] = lzv;
                    if (drew) lx += lzv;
                }
            }
            if (done || s + 1 == n_steps) break;
            row += step_stride;
            if (wave < nt) load_tile<T>(row, V, wave, lane, first);
            u = uniforms[(size_t)(s + 1) * (size_t)B + b];
            continue;
        }
        if (LOOP_REG) __syncthreads();   // (wavefront 0 may still be reading the statistics of a fast step before this one)
        const uint32_t *image = ix.heavy_bits + (size_t)(slot != PPV_NO_SLOT ? slot : 0) * (size_t)ix.n_words;
        int member_child = 0;
        if (mode == VALID_LIST) {
            // children are sorted by token: the list is ready as it is.  One entry more than the
            // children is taken along: it closes the last child's own children range.
            for (int i = tid; i <= nchild; i += nw * WAVE) {
                const NodeEnt e = ix.ent[cb + i];
                sh.list_tok[i] = e.tok;
                sh.list_child[i] = e.child;
                if (i < nchild && (e.tok & PPV_NODE_TERMINAL)) member_child = 1;
            }
            if (LOOP) member_child = __syncthreads_or(member_child);
            else __syncthreads();
        }
        const bool more = LOOP && s + 1 < n_steps && t + 1 < stride && mode != VALID_NONE && !member_child;
        RawTile next_first;
        const T *next_row = more ? row + step_stride : nullptr;
        float next_u = 0.f;
        if (more) next_u = uniforms[(size_t)(s + 1) * (size_t)B + b];
        RowOut r = row_sample<T, PIPE, RowShared, LOOP, SPLIT>(row, V, first, mode, mode == VALID_LIST ? nchild : 0, image, u, sh,
                                                  tid, nw, tp, sp, next_row, &next_first);
        if (r.mine && tid == 0) {
            const bool room = t < stride || !advance;
            int32_t id = -1;
            done = true;  // no valid token or no room: the row cannot continue
            RowState nx = st;
            nx.flags = 0u;   // (the look-ahead belongs to the node it was made for)
            if (r.id >= 0 && room) {
                id = r.id;
                uint32_t tokw;
                if (mode == VALID_LIST) {
                    nx.node = cb + (uint32_t)r.pos;
                    tokw = sh.list_tok[r.pos];
                    nx.cb = sh.list_child[r.pos];
                    nx.ce = sh.list_child[r.pos + 1];
                } else {  // child index = children before the token's word + set bits below it in the word
                    const uint32_t wv = image[id >> 5];
                    nx.node = cb + ix.heavy_rank[(size_t)slot * (size_t)ix.n_words + (id >> 5)] +
                              (uint32_t)__popc(wv & ((1u << (id & 31)) - 1u));
                    if (nx.node >= ix.n_nodes) nx.node = ix.n_nodes - 1u;   // (only a cursor that paired a slot with another node's children)
                    const NodeEnt e0 = ix.ent[nx.node], e1 = ix.ent[nx.node + 1];
                    tokw = e0.tok;
                    nx.cb = e0.child;
                    nx.ce = e1.child;
                }
                nx.slot = (tokw & PPV_NODE_HEAVY) ? heavy_slot_of(ix, nx.node) : PPV_NO_SLOT;
                done = (tokw & PPV_NODE_TERMINAL) != 0u;   // the extended row is itself a member
                if (advance) prefixes[(size_t)b * (size_t)stride + t] = id;
                lx += r.logZ_valid;
            } else {
                lx = -INFINITY;   // the row stops outside S: its importance score is multiplied by a valid mass of 0
            }
            if (ids) ids[(size_t)s * (size_t)B + b] = id;
            if (logZ_valid) logZ_valid[(size_t)s * (size_t)B + b] = r.logZ_valid;
            if (LOOP) {
                sh.bc_i[2] = done ? 1 : 0;
                sh.bc_i[3] = id >= 0 ? 1 : 0;
                sh.bc_i[4] = (int)nx.node;
                sh.bc_i[5] = (int)nx.cb;
                sh.bc_i[6] = (int)nx.ce;
                sh.bc_i[7] = (int)nx.slot;
            } else if (advance) {
                if (id >= 0) {
                    lens[b] = t + 1;
                    if (state) state[b] = nx;
                } else if (fresh) {
                    lens[b] = 0;
                    if (state) state[b] = st;
                }
                if (logx) logx[b] = logx_in + lx;   // (-inf for a row that drew nothing)
                if (done) active[b] = 0;
                else if (fresh) active[b] = 1;
            }
        }
        if (!LOOP) return;
        __syncthreads();
        done = sh.bc_i[2] != 0;
        if (sh.bc_i[3]) {
            t += 1;
            st.node = (uint32_t)sh.bc_i[4];
            st.cb = (uint32_t)sh.bc_i[5];
            st.ce = (uint32_t)sh.bc_i[6];
            st.slot = (uint32_t)sh.bc_i[7];
            st.flags = 0u;   // the loop kernel does not look ahead
        }
        __syncthreads();   // everyone has the new cursor before LDS is reused
        if (done || s + 1 == n_steps) break;
        row += step_stride;
        if (more) {
            first = next_first;
            u = next_u;
        } else {
            if (wave < nt) load_tile<T>(row, V, wave, lane, first);
            u = uniforms[(size_t)(s + 1) * (size_t)B + b];
        }
    }
    if (LOOP && tid == 0) {
        lens[b] = t;
        if (state) state[b] = st;
        if (logx) logx[b] = lx;
        if (done) active[b] = 0;
    }
}

// T > 0 and finite, or the call is refused; the constants the kernels take (see Temper)
bool temper_for(float temperature, Temper *tp) {
    if (!(temperature > 0.f) || !std::isfinite(temperature)) return false;
    tp->c = (float)(1.44269504088896340736 / (double)temperature);   // log2(e) / T
    tp->inv = (float)(1.0 / (double)temperature);
    tp->guard = REF_GUARD * temperature;
    return std::isfinite(tp->c) && tp->c > 0.f;
}

ppv_status check_logits_args(const void *logits, ppv_dtype dt, int64_t row_stride, int32_t V) {
    if (!logits || V <= 0 || row_stride < V) return PPV_EINVAL;
    if (dt != PPV_F32 && dt != PPV_BF16) return PPV_EINVAL;
    const int64_t per16 = (dt == PPV_F32) ? 4 : 8;
    if (row_stride % per16 != 0 || ((uintptr_t)logits & 15u) != 0) return PPV_EINVAL;
    if (V > PPV_MAX_VOCAB) return PPV_ERANGE;
    return PPV_OK;
}

// Wavefronts per row: a power of two, at most one per tile and at most MAX_WAVES.  A small batch is
// bound by latency and wants every row spread over many wavefronts so that the whole row is in
// flight at once; a large batch is bound by throughput and wants several rows per compute unit, so
// that one row's reduction and sampling phase overlaps another row's loads.  The steps below are
// measured, on the N=1M, V=32k decode loop (TB/s of logits over the whole loop): B=256: 1.05 with
// 16 wavefronts per row, 1.08 with 8, 0.93 with 4; B=512: 1.31 / 1.64 / 1.57; B=1024: 2.28 with 8,
// 2.50 with 4, 2.37 with 2; B=4096: 2.1 with 16, 3.4 with 8, 4.3 with 4, 4.1 with 2; and at
// V=256k: B=256: 3.8 with 16, 1.3 with 2; B=1024: 5.05 with 4, 5.09 with 8, 4.4 with 16.
// `parts`: workgroups per row (see parts_for); the figures then hold for one workgroup's share of the row and for
// the number of workgroups in the launch.
// `cursor_step`: the per-step decode kernel with a cursor, which no longer waits for index entries behind the tiles
// it has asked for: one tile per wavefront, the whole row in flight at once, also at 256 rows (C3, us per launch
// with 8 / 16 wavefronts: 7.9 / 7.6 before the list moved into registers; tiles reduced 3.4 / 2.8 us after the
// cursor is in).
int waves_for(int V, ppv_dtype dt, int B, int parts = 1, bool cursor_step = false) {
    const int tile = (dt == PPV_F32) ? TileGeom<float>::TILE : TileGeom<uint16_t>::TILE;
    const int nt = ((V + tile - 1) / tile + parts - 1) / parts;
    B *= parts;
    int cap = B <= 128 ? 16 : (B <= 512 ? 8 : 4);
    if (cursor_step && B <= 256) cap = 16;
    // long rows in a small batch: one row per compute unit, all of it in flight (constrained_sample, B = 256, us per
    // call with 8 / 16 wavefronts: 32 tiles: 13.2 / 12.0 (fp32 V = 32k), 15.2 / 14.2 (bf16 V = 64k); 63 tiles: 23.6 / 20.6)
    if (nt >= 32 && B <= 256) cap = 16;
    if (const int v = ppv_tuning(PPV_TUNE_WAVES_PER_ROW)) cap = v;   // tuning aid (0: the table above)
    int nw = 1;
    while (nw < nt && nw * 2 <= cap) nw <<= 1;
    return nw;
}

// Whether some wavefront's turn has six tiles or more, i.e. whether the three-tile pipeline of stream_tiles can
// run at all.  Kernels for shorter turns are compiled without it: 62 instead of 92 registers (bf16), which is
// two more rows in flight per compute unit when a large batch keeps every compute unit full.
bool long_turns(int V, ppv_dtype dt, int nw) {   // nw: wavefronts per row over all its workgroups
    const int tile = (dt == PPV_F32) ? TileGeom<float>::TILE : TileGeom<uint16_t>::TILE;
    return (V / tile + nw - 1) / nw >= 6;
}

// Workgroups per row.  A batch of fewer rows than the chip has compute units leaves most of it idle with one
// workgroup per row, and a long row alone on a compute unit is bound by that unit's arithmetic (about 4.8 us per
// 256 KB of bf16 logits).  Such a row is spread over 2 .. 16 workgroups: a power of two, six tiles or more each, at
// most one workgroup per compute unit.  Handing the statistics from workgroup to workgroup costs about 3 us (three
// dependent trips to device-scope memory), so rows are split only where that is less than what the split saves:
// row bytes x (1 - 1 / parts) >= 160 KB.  Measured, constrained_sample, bf16, us per call without / with the split:
// V = 128,256: B = 32: 13.0 / 10.0 (list rows), 17.8 / 11.2 (image rows); B = 128: 13.6 / 14.0, 18.7 / 16.1 (two
// parts: not split); V = 32,000, B = 64: 7.4 / 9.1 (not split).  PPV_TUNE_ROW_SPLIT forces a number of parts.
// The scratch area the parts meet in comes with the stream; without one (see ppv_split_scratch) rows are not split.
int parts_wanted(int V, ppv_dtype dt, int B) {
    const int tile = (dt == PPV_F32) ? TileGeom<float>::TILE : TileGeom<uint16_t>::TILE;
    const int nt = (V + tile - 1) / tile;
    if (B > PPV_SPLIT_MAX_ROWS) return 1;
    int parts = ppv_tuning(PPV_TUNE_ROW_SPLIT);
    if (parts == 0) {
        parts = 1;
        while (B * parts * 2 <= 256 && parts * 2 <= PPV_SPLIT_MAX_PARTS && nt / (parts * 2) >= 6) parts *= 2;
        const double row_kb = (double)V * (dt == PPV_F32 ? 4.0 : 2.0) / 1024.0;
        if (row_kb * (1.0 - 1.0 / parts) < 160.0) parts = 1;
    }
    while (parts > 1 && ((parts & (parts - 1)) != 0 || parts * 2 > nt)) parts--;   // a power of two, two tiles each
    return parts;
}
int parts_for(int V, ppv_dtype dt, int B, hipStream_t hs, SplitScratch **scratch) {
    *scratch = nullptr;
    int parts = parts_wanted(V, dt, B);
    if (parts > 1) {
        *scratch = ppv_split_scratch(hs);
        if (!*scratch) parts = 1;
    }
    return parts;
}
int shift_of(int parts) {
    int sh = 0;
    while ((1 << sh) < parts) sh++;
    return sh;
}

template <typename T>
void launch_sample(bool small, bool pipe, dim3 grid, dim3 block, hipStream_t hs, const T *lg, int64_t row_stride,
                   const uint32_t *mask, const float *uniforms, int V, int n_words, int list_max, int32_t *ids,
                   float *logZ_valid, float *logZ_all, Temper tp, int split_shift, SplitScratch *scratch) {
    if (split_shift)   // (a split row's turns are short; the kernel without the three-tile pipeline serves all of them)
        hipLaunchKernelGGL((sample_kernel<T, false, false, true>), grid, block, 0, hs, lg, row_stride, mask, uniforms, V,
                           n_words, list_max, ids, logZ_valid, logZ_all, tp, split_shift, scratch);
    else if (small)
        hipLaunchKernelGGL((sample_kernel<T, true, false, false>), grid, block, 0, hs, lg, row_stride, mask, uniforms, V, n_words,
                           list_max, ids, logZ_valid, logZ_all, tp, split_shift, scratch);
    else if (pipe)
        hipLaunchKernelGGL((sample_kernel<T, false, true, false>), grid, block, 0, hs, lg, row_stride, mask, uniforms, V, n_words,
                           list_max, ids, logZ_valid, logZ_all, tp, split_shift, scratch);
    else
        hipLaunchKernelGGL((sample_kernel<T, false, false, false>), grid, block, 0, hs, lg, row_stride, mask, uniforms, V,
                           n_words, list_max, ids, logZ_valid, logZ_all, tp, split_shift, scratch);
}

constexpr int REG_MAX_ROWS = 1024;   // batches up to here run the per-step kernel with the list in registers
template <typename T>
void launch_decode_kernel(bool loop, bool pipe, dim3 grid, dim3 block, hipStream_t hs, const IndexView &view,
                          int32_t *prefixes, int32_t stride, int32_t *lens, uint8_t *active, RowState *rs, const T *lg,
                          int64_t row_stride, int64_t step_stride, const float *uniforms, int n_steps, int B, int32_t *ids,
                          float *logZ_valid, float *logx, Temper tp, int split_shift, SplitScratch *scratch, int flags) {
#define PPV_LAUNCH_DECODE(LOOP, PIPE, SPLIT, REG)                                                                     \
    hipLaunchKernelGGL((decode_kernel<T, LOOP, PIPE, SPLIT, REG>), grid, block, 0, hs, view, prefixes, stride, lens,   \
                       active, rs, lg, row_stride, step_stride, uniforms, n_steps, B, ids, logZ_valid, logx, tp,        \
                       split_shift, scratch, flags)
    if (split_shift && !loop) PPV_LAUNCH_DECODE(false, false, true, false);   // (a split row's turns are short)
    else if (loop && pipe) PPV_LAUNCH_DECODE(true, true, false, false);
    else if (loop && rs && B <= REG_MAX_ROWS) PPV_LAUNCH_DECODE(true, false, false, true);
    else if (loop) PPV_LAUNCH_DECODE(true, false, false, false);
    else if (pipe) PPV_LAUNCH_DECODE(false, true, false, false);
    else if (rs && B <= REG_MAX_ROWS) PPV_LAUNCH_DECODE(false, false, false, true);
    else PPV_LAUNCH_DECODE(false, false, false, false);
#undef PPV_LAUNCH_DECODE
}

}  // namespace

extern "C" ppv_status ppv_next_token_mask(const ppv_index_t *ix, const int32_t *prefixes, int32_t prefix_stride,
                                          const int32_t *lens, int32_t B, uint32_t *mask, uint32_t *range_lo,
                                          uint32_t *range_hi, uint8_t *member, void *stream) {
    if (!ix || B < 0 || prefix_stride < 0) return PPV_EINVAL;
    if (B == 0) return PPV_OK;  // nothing to do; the (possibly null) buffers are not looked at
    if (!prefixes || !lens || !mask) return PPV_EINVAL;
    if (ix->view.n_words <= MASK_SMALL_WORDS) {
        const int rows_per_wg = MASK_THREADS / WAVE;
        hipLaunchKernelGGL(mask_rows_kernel, dim3((unsigned)((B + rows_per_wg - 1) / rows_per_wg)), dim3(MASK_THREADS), 0,
                           (hipStream_t)stream, ix->view, prefixes, prefix_stride, lens, B, mask, range_lo, range_hi,
                           member);
    } else {
        const size_t lds = ((size_t)ix->view.n_words + 4) * sizeof(uint32_t);
        hipLaunchKernelGGL(mask_kernel, dim3((unsigned)B), dim3(MASK_THREADS), lds, (hipStream_t)stream, ix->view,
                           prefixes, prefix_stride, lens, mask, range_lo, range_hi, member);
    }
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}

// The scratch area of constrained_sample_noalloc: the same SplitScratch that other calls allocate per stream, here
// a fixed array in device memory (every GPU the library runs on holds its own copy until the process ends).  Host
// code never uses the array's name as an address: its address on the current device is looked up once per device.
static __device__ __align__(256) unsigned char scratch[sizeof(SplitScratch)];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_fixed_mu;
SplitScratch *g_fixed_scratch[MAX_DEVICES];   // per device: the address of `scratch` there

ppv_status fixed_scratch(SplitScratch **out) {
    int dev = -1;
    PPV_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return PPV_ERANGE;
    std::lock_guard<std::mutex> lock(g_fixed_mu);
    if (!g_fixed_scratch[dev]) {
        void *ptr = nullptr;
        PPV_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return PPV_EDEVICE;
        g_fixed_scratch[dev] = (SplitScratch *)ptr;
    }
    *out = g_fixed_scratch[dev];
    return PPV_OK;
}

ppv_status sample_call(const void *logits, ppv_dtype dt, int64_t row_stride, const uint32_t *mask, const float *uniforms,
                       int32_t B, int32_t V, int32_t *ids, float *logZ_valid, float *logZ_all, float temperature,
                       void *stream, bool no_alloc) {
    Temper tp;
    if (B < 0 || !temper_for(temperature, &tp)) return PPV_EINVAL;
    if (B == 0) return PPV_OK;
    if (!mask || !uniforms || !ids || !logZ_valid) return PPV_EINVAL;
    ppv_status st = check_logits_args(logits, dt, row_stride, V);
    if (st != PPV_OK) return st;
    const int n_words = (V + 31) / 32;
    const int list_max = V / 32 < PPV_LIST_MAX ? V / 32 : PPV_LIST_MAX;
    const int tile = (dt == PPV_F32) ? TileGeom<float>::TILE : TileGeom<uint16_t>::TILE;
    const bool small = (V + tile - 1) / tile <= SMALL_TILES && list_max <= SMALL_LIST;   // then threads <= SMALL_TILES * WAVE
    hipStream_t hs = (hipStream_t)stream;
    SplitScratch *scratch = nullptr;
    int parts = 1;
    if (no_alloc) {   // the fixed array: no allocation, a stated largest batch
        if (B > PPV_NOALLOC_MAX_ROWS) return PPV_ERANGE;
        st = fixed_scratch(&scratch);
        if (st != PPV_OK) return st;
        if (!small && V > tile) parts = parts_wanted(V, dt, B);
    } else if (!small && V > tile) {
        parts = parts_for(V, dt, B, hs, &scratch);
    }
    const int threads = waves_for(V, dt, B, parts) * WAVE;
    const bool pipe = long_turns(V, dt, parts * threads / WAVE);
    const dim3 grid((unsigned)B * (unsigned)parts), block(threads);
    if (V <= tile) {   // the whole row is one tile
        const dim3 g1((unsigned)((B + ONE_TILE_ROWS - 1) / ONE_TILE_ROWS)), b1(ONE_TILE_ROWS * WAVE);
        if (dt == PPV_F32)
            hipLaunchKernelGGL(sample_one_tile_kernel<float>, g1, b1, 0, hs, (const float *)logits, row_stride, mask, uniforms,
                               B, V, n_words, ids, logZ_valid, logZ_all, tp);
        else
            hipLaunchKernelGGL(sample_one_tile_kernel<uint16_t>, g1, b1, 0, hs, (const uint16_t *)logits, row_stride, mask,
                               uniforms, B, V, n_words, ids, logZ_valid, logZ_all, tp);
        PPV_HIP_TRY(hipGetLastError());
        return PPV_OK;
    }
    if (dt == PPV_F32)
        launch_sample<float>(small, pipe, grid, block, hs, (const float *)logits, row_stride, mask, uniforms, V, n_words,
                             list_max, ids, logZ_valid, logZ_all, tp, shift_of(parts), scratch);
    else
        launch_sample<uint16_t>(small, pipe, grid, block, hs, (const uint16_t *)logits, row_stride, mask, uniforms, V,
                                n_words, list_max, ids, logZ_valid, logZ_all, tp, shift_of(parts), scratch);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}
}  // namespace

extern "C" ppv_status constrained_sample(const void *logits, ppv_dtype dt, int64_t row_stride, const uint32_t *mask,
                                         const float *uniforms, int32_t B, int32_t V, int32_t *ids,
                                         float *logZ_valid, float *logZ_all, float temperature, void *stream) {
    return sample_call(logits, dt, row_stride, mask, uniforms, B, V, ids, logZ_valid, logZ_all, temperature, stream, false);
}

extern "C" ppv_status constrained_sample_noalloc(const void *logits, ppv_dtype dt, int64_t row_stride,
                                                 const uint32_t *mask, const float *uniforms, int32_t B, int32_t V,
                                                 int32_t *ids, float *logZ_valid, float *logZ_all, float temperature,
                                                 void *stream) {
    return sample_call(logits, dt, row_stride, mask, uniforms, B, V, ids, logZ_valid, logZ_all, temperature, stream, true);
}

extern "C" ppv_status ppv_decode_begin(const ppv_index_t *ix, const int32_t *prefixes, int32_t prefix_stride,
                                       const int32_t *lens, int32_t B, uint32_t *state, uint8_t *active, float *logx,
                                       void *stream) {
    if (!ix || B < 0 || prefix_stride < 0) return PPV_EINVAL;
    if (B == 0) return PPV_OK;
    if (!prefixes || !lens || !state || !active) return PPV_EINVAL;
    const int rows_per_wg = MASK_THREADS / WAVE;
    hipLaunchKernelGGL(decode_begin_kernel, dim3((unsigned)((B + rows_per_wg - 1) / rows_per_wg)), dim3(MASK_THREADS), 0,
                       (hipStream_t)stream, ix->view, prefixes, prefix_stride, lens, B, (RowState *)state, active,
                       logx);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}

extern "C" ppv_status ppv_decode_begin_empty(const ppv_index_t *ix, int32_t B, int32_t *lens, uint32_t *state,
                                             uint8_t *active, float *logx, void *stream) {
    if (!ix || B < 0) return PPV_EINVAL;
    if (B == 0) return PPV_OK;
    if (!lens || !state || !active) return PPV_EINVAL;
    hipLaunchKernelGGL(decode_begin_empty_kernel, dim3((unsigned)((B + MASK_THREADS - 1) / MASK_THREADS)), dim3(MASK_THREADS),
                       0, (hipStream_t)stream, ix->view, B, lens, (RowState *)state, active, logx);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}

namespace {
ppv_status launch_decode(const ppv_index_t *ix, int32_t *prefixes, int32_t prefix_stride, int32_t *lens, uint8_t *active,
                         uint32_t *state, const void *logits, ppv_dtype dt, int64_t row_stride, int64_t step_stride,
                         const float *uniforms, int32_t n_steps, int32_t B, int32_t *ids, float *logZ_valid, float *logx,
                         float temperature, void *stream, bool loop, bool advance = true, bool fresh = false) {
    Temper tp;
    if (!ix || B < 0 || prefix_stride < 0 || n_steps < 0 || !temper_for(temperature, &tp)) return PPV_EINVAL;
    if (B == 0 || n_steps == 0) return PPV_OK;
    if (!prefixes || !lens || (advance && !active) || !uniforms) return PPV_EINVAL;
    ppv_status st = check_logits_args(logits, dt, row_stride, ix->view.vocab);
    if (st != PPV_OK) return st;
    if (loop && n_steps > 1) {
        const int64_t per16 = (dt == PPV_F32) ? 4 : 8;
        if (step_stride % per16 != 0 || step_stride < 0) return PPV_EINVAL;
    }
    hipStream_t hs = (hipStream_t)stream;
    SplitScratch *scratch = nullptr;
    const int parts = (loop || fresh) ? 1 : parts_for(ix->view.vocab, dt, B, hs, &scratch);
    int nw = waves_for(ix->view.vocab, dt, B, parts, !loop && state != nullptr);
    if (loop && nw > LOOP_WAVES) nw = LOOP_WAVES;
    // The loop kernel in a large batch: a workgroup stays with its row for every step, so what hides one row's
    // dependent phases (cursor, barrier, draw) is other rows on the same compute unit, and two wavefronts per row
    // put twice as many there as four (C3 replicas, M prefix-steps/s with 1 / 2 / 4 / 8 wavefronts per row:
    // 4,096 rows: 72 / 81 / 66 / 39; 16,384 rows: 95 / 98 / 77 / 42 -- 6.3 TB/s; the per-step kernel is best with four).
    if (loop && B > REG_MAX_ROWS && nw > 2 && ppv_tuning(PPV_TUNE_WAVES_PER_ROW) == 0) nw = 2;
    {   // the loop kernel with the list in registers: one wavefront draws, the others stream two tiles each
        const int tile = (dt == PPV_F32) ? TileGeom<float>::TILE : TileGeom<uint16_t>::TILE;
        const int nt = (ix->view.vocab + tile - 1) / tile;
        if (loop && state && B <= REG_MAX_ROWS && !long_turns(ix->view.vocab, dt, nw) && nt >= 2 && (nt + 1) / 2 + 1 <= CHAIN_WAVES &&
            ppv_tuning(PPV_TUNE_WAVES_PER_ROW) == 0)
            nw = (nt + 1) / 2 + 1;
    }
    const dim3 grid((unsigned)B * (unsigned)parts), block(nw * WAVE);
    RowState *rs = (RowState *)state;
    const bool pipe = long_turns(ix->view.vocab, dt, parts * nw);
    if (!loop) n_steps = 1;
    if (dt == PPV_F32)
        launch_decode_kernel<float>(loop, pipe, grid, block, hs, ix->view, prefixes, prefix_stride, lens, active, rs,
                                    (const float *)logits, row_stride, step_stride, uniforms, n_steps, B, ids, logZ_valid,
                                    logx, tp, shift_of(parts), scratch, (advance ? 1 : 0) | (fresh ? 2 : 0));
    else
        launch_decode_kernel<uint16_t>(loop, pipe, grid, block, hs, ix->view, prefixes, prefix_stride, lens, active, rs,
                                       (const uint16_t *)logits, row_stride, step_stride, uniforms, n_steps, B, ids,
                                       logZ_valid, logx, tp, shift_of(parts), scratch, (advance ? 1 : 0) | (fresh ? 2 : 0));
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}
}  // namespace

extern "C" ppv_status ppv_decode_step(const ppv_index_t *ix, int32_t *prefixes, int32_t prefix_stride, int32_t *lens,
                                      uint8_t *active, uint32_t *state, const void *logits, ppv_dtype dt,
                                      int64_t row_stride, const float *uniforms, int32_t B, int32_t *ids,
                                      float *logZ_valid, float *logx, float temperature, void *stream) {
    return launch_decode(ix, prefixes, prefix_stride, lens, active, state, logits, dt, row_stride, 0, uniforms, 1, B, ids,
                         logZ_valid, logx, temperature, stream, false);
}

extern "C" ppv_status ppv_decode_first_step(const ppv_index_t *ix, int32_t *prefixes, int32_t prefix_stride, int32_t *lens,
                                            uint8_t *active, uint32_t *state, const void *logits, ppv_dtype dt,
                                            int64_t row_stride, const float *uniforms, int32_t B, int32_t *ids,
                                            float *logZ_valid, float *logx, float temperature, void *stream) {
    if (!state) return PPV_EINVAL;
    return launch_decode(ix, prefixes, prefix_stride, lens, active, state, logits, dt, row_stride, 0, uniforms, 1, B, ids,
                         logZ_valid, logx, temperature, stream, false, true, true);
}

extern "C" ppv_status ppv_decode_loop(const ppv_index_t *ix, int32_t *prefixes, int32_t prefix_stride, int32_t *lens,
                                      uint8_t *active, uint32_t *state, const void *logits, ppv_dtype dt,
                                      int64_t row_stride, int64_t step_stride, const float *uniforms, int32_t n_steps,
                                      int32_t B, int32_t *ids, float *logZ_valid, float *logx, float temperature,
                                      void *stream) {
    return launch_decode(ix, prefixes, prefix_stride, lens, active, state, logits, dt, row_stride, step_stride, uniforms,
                         n_steps, B, ids, logZ_valid, logx, temperature, stream, true);
}

extern "C" ppv_status ppv_sample_next(const ppv_index_t *ix, const int32_t *prefixes, int32_t prefix_stride,
                                      const int32_t *lens, int32_t B, const void *logits, ppv_dtype dt,
                                      int64_t row_stride, const float *uniforms, int32_t *ids, float *logZ_valid,
                                      float temperature, void *stream) {
    Temper tp;
    if (!ix || B < 0 || prefix_stride < 0 || !temper_for(temperature, &tp)) return PPV_EINVAL;
    if (B == 0) return PPV_OK;
    if (!prefixes || !lens || !uniforms || !ids) return PPV_EINVAL;
    const int V = ix->view.vocab;
    const ppv_status st = check_logits_args(logits, dt, row_stride, V);
    if (st != PPV_OK) return st;
    const int tile = (dt == PPV_F32) ? TileGeom<float>::TILE : TileGeom<uint16_t>::TILE;
    if (V <= tile && ix->view.n_words <= MASK_SMALL_WORDS) {   // the whole row is one tile: one wavefront per row
        const dim3 g1((unsigned)((B + ONE_TILE_ROWS - 1) / ONE_TILE_ROWS)), b1(ONE_TILE_ROWS * WAVE);
        if (dt == PPV_F32)
            hipLaunchKernelGGL(sample_next_one_tile_kernel<float>, g1, b1, 0, (hipStream_t)stream, ix->view, prefixes,
                               prefix_stride, lens, (const float *)logits, row_stride, uniforms, B, ids, logZ_valid,
                               (uint8_t *)nullptr, tp);
        else
            hipLaunchKernelGGL(sample_next_one_tile_kernel<uint16_t>, g1, b1, 0, (hipStream_t)stream, ix->view, prefixes,
                               prefix_stride, lens, (const uint16_t *)logits, row_stride, uniforms, B, ids, logZ_valid,
                               (uint8_t *)nullptr, tp);
        PPV_HIP_TRY(hipGetLastError());
        return PPV_OK;
    }
    // longer rows: the fused decode step without a cursor, told to change nothing of the caller's rows
    return launch_decode(ix, const_cast<int32_t *>(prefixes), prefix_stride, const_cast<int32_t *>(lens), nullptr, nullptr,
                         logits, dt, row_stride, 0, uniforms, 1, B, ids, logZ_valid, nullptr, temperature, stream, false,
                         false);
}
