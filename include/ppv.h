/*
 * ppv.h -- C ABI of the MI355X (gfx950) parallel prefix-verification library.
 *
 * The library implements the per-step hot path of set-constrained decoding: for a batch of
 * decoding prefixes it produces each prefix's valid-next-token mask over the whole vocabulary
 * (PPV with M = |V|, Section 3.2 "Selection of top candidate tokens": the exact valid set
 * A_{a,S} of Section 2.1), and a fused masked log-softmax that returns the probability mass the
 * model puts on valid tokens, |P (.) mask|_1, together with a token sampled from
 * P (.) mask / |P (.) mask|_1 (Algorithm 1, SampleCandidate).
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory on the
 *     GPU that was current when the index was built.  The caller owns every buffer it passes.
 *   - Every call returns a ppv_status and never throws or aborts across this boundary.  Outputs
 *     are unspecified when the status is not PPV_OK.
 *   - Calls that take a `stream` (a hipStream_t passed as void*, NULL = the default stream) only
 *     enqueue work on it and do not synchronise with the host.  Argument checks that need device
 *     data are not made; checks on host-visible arguments are.
 *   - An index is immutable after it is built; calls on different streams may run concurrently.
 *   - Token order is integer order (Section 2.1, footnote on the ordered vocabulary); sequences
 *     are ordered lexicographically, left to right, a proper prefix before its extensions
 *     (Section 3.2 "Array Preparation").  Query tokens are compared as unsigned 32-bit values:
 *     a token outside [0, V) matches nothing and sorts after every real token.
 *   - Logits are expected to be finite or -inf.  A row with NaN or +inf logits has no meaningful sums; it
 *     ends in a defined state (a token of its valid set, or id -1 and the row retires) and does not affect
 *     other rows, but its id, logZ_valid and logx are unspecified.
 *   - Mask layout: row b is ceil(V/32) uint32 words; token v is bit (v & 31), least significant
 *     first, of word (v >> 5); bits at positions >= V are 0.
 */
#ifndef PPV_H
#define PPV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ppv_index ppv_index_t; /* opaque; owns its device memory */

typedef enum {
    PPV_OK = 0,
    PPV_EINVAL = -1,  /* bad argument: null pointer, bad size, empty S, empty sequence, token out of range */
    PPV_ENOMEM = -2,  /* host or device allocation failed */
    PPV_EDEVICE = -3, /* a HIP call failed (no device, launch error) */
    PPV_ERANGE = -4,  /* a size exceeds what the library supports (see PPV_MAX_VOCAB) */
    PPV_EIO = -5      /* a file could not be opened, read or written */
} ppv_status;

typedef enum { PPV_F32 = 0, PPV_BF16 = 1 } ppv_dtype;

#define PPV_MAX_VOCAB 262144 /* the per-row bit image (V/8 bytes) is staged in one workgroup's LDS */
#define PPV_TOPM_MAX 1024    /* largest M of ppv_topm_mask (the paper's experiments use 50 to 1000) */

const char *ppv_status_string(ppv_status s);

/*
 * ppv_build_index -- Algorithm 2, "Prepare"; Section 3.2 "Array Preparation".
 * Builds the device-resident index of the constraint set S: S sorted lexicographically and
 * de-duplicated (S is a set), stored flat without padding, plus per-depth arrays that list, for
 * every distinct prefix of a member, its token, its rank range in sorted S and where its
 * children start at the next depth.
 *   tokens   host, int32[offsets[n_seq]]: sequence i is tokens[offsets[i] .. offsets[i+1])
 *   offsets  host, int64[n_seq + 1], non-decreasing, offsets[0] == 0
 *   n_seq    number of sequences given (duplicates allowed, any order), > 0
 *   vocab    |V|; every token must lie in [0, vocab); 0 < vocab <= PPV_MAX_VOCAB
 *   out      receives the handle; release with ppv_free_index
 * The inputs are copied; the caller keeps ownership.  Synchronous.
 * Errors: PPV_EINVAL (null pointer, n_seq <= 0, an empty sequence, a token outside [0, vocab),
 * decreasing offsets), PPV_ERANGE (vocab too large, or more than 2^32 - 2 rows or prefixes),
 * PPV_ENOMEM, PPV_EDEVICE.
 */
ppv_status ppv_build_index(const int32_t *tokens, const int64_t *offsets, int64_t n_seq, int32_t vocab,
                           ppv_index_t **out);

/* Sizes of a built index.  Any output pointer may be NULL.
 *   n_distinct   |S| after de-duplication        l_max   longest member
 *   n_prefixes   number of distinct non-empty prefixes of members (entries of the per-depth arrays)
 *   device_bytes device memory the index holds */
ppv_status ppv_index_info(const ppv_index_t *index, int64_t *n_distinct, int32_t *l_max, int32_t *vocab,
                          int64_t *n_prefixes, int64_t *device_bytes);

/* Copies the sorted, de-duplicated S back to the host (for inspection and tests).
 *   tokens_out   host, int32[sum of member lengths] or NULL     offsets_out  host, int64[n_distinct + 1] or NULL
 *   n_tokens     receives the total number of tokens, may be NULL.  Synchronous. */
ppv_status ppv_index_export(const ppv_index_t *index, int32_t *tokens_out, int64_t *offsets_out, int64_t *n_tokens);

void ppv_free_index(ppv_index_t *index); /* NULL is allowed */

/*
 * ppv_index_save / ppv_index_load -- Section 3.2 "Array Preparation": the array is prepared once and
 * kept (the paper splits it by length only to save disk space; the flat layout here has no padding to
 * save); Section 3.2 "Advantages over prefix trees" counts loading a prepared array, instead of
 * building a tree, among the gains.  The file holds the per-depth entries, the rank ranges and the flat
 * sorted S behind a 128-byte header with a checksum; the heavy prefixes' images are rebuilt at load.
 * Little-endian; a file is only good for the library version that wrote it (the header says which).
 *   path   host, NUL-terminated
 *   out    host; *out receives a new index on the current device, *out = NULL on failure
 * ppv_index_load trusts nothing in the file: sizes are checked against the file's length, the checksum
 * against its contents, and a device pass checks that every offset, rank and token stays inside its
 * array, so that an index that loads cannot send a kernel out of bounds.
 * Errors: PPV_EINVAL (null argument; not an index file; sizes, checksum or structure wrong),
 * PPV_EIO (open / read / write failed), PPV_ERANGE, PPV_ENOMEM, PPV_EDEVICE.
 */
ppv_status ppv_index_save(const ppv_index_t *index, const char *path);
ppv_status ppv_index_load(const char *path, ppv_index_t **out);

/*
 * ppv_next_token_mask -- Algorithm 2 with M = |V| (verification of every token at once);
 * valid set of Section 2.1; Section 3.2 "Parallel Verification".
 * For each prefix a_b (the first lens[b] tokens of row b of `prefixes`):
 *   mask[b]      the packed valid set A_{a_b,S} (all zero when a_b is a prefix of no member, and
 *                when a_b is a member without extensions)
 *   range_lo[b]  number of members that sort before a_b
 *   range_hi[b]  range_lo[b] + number of members that a_b is a prefix of; for a prefix of no
 *                member both equal the rank at which a_b would be inserted (the lower bound
 *                the binary search of Section 3.2 ends on)
 *   member[b]    1 iff a_b is itself in S (the loop condition of Algorithm 1), else 0
 * Arguments (all device pointers):
 *   prefixes  int32[B, prefix_stride] row-major; only the first lens[b] entries of a row are read
 *   lens      int32[B], 0 <= lens[b] <= prefix_stride (values outside are clamped into that range)
 *   mask      uint32[B, ceil(V/32)], fully written
 *   range_lo, range_hi  uint32[B], each may be NULL      member  uint8[B], may be NULL
 * B == 0 is allowed and does nothing.  Errors: PPV_EINVAL (null index/prefixes/lens/mask, B < 0,
 * prefix_stride < 0), PPV_EDEVICE.
 */
ppv_status ppv_next_token_mask(const ppv_index_t *index, const int32_t *prefixes, int32_t prefix_stride,
                               const int32_t *lens, int32_t B, uint32_t *mask, uint32_t *range_lo,
                               uint32_t *range_hi, uint8_t *member, void *stream);

/*
 * constrained_sample -- Algorithm 1, SampleCandidate, sampling step and update step: a token drawn from the
 * model's distribution restricted to the valid set and renormalised, and the valid mass |P (.) mask|_1 that
 * multiplies the importance score x, with P = softmax(logits / T), T the temperature that Algorithm 1 takes as
 * input (the experiments of Section 4.1 "Methods" use T = 1).  With l_v = logits[v] / T, per row b:
 *   logZ_valid[b] = log sum_{v in mask} exp(l_v) - log sum_{all v} exp(l_v)   (<= 0; -inf if the mask is empty
 *                   or every valid token has logit -inf)
 *   logZ_all[b]   = log sum_{all v} exp(l_v)
 *   ids[b]        = the first valid token, in increasing token id, whose cumulative weight
 *                   sum_{w <= v, w in mask} exp(l_w) exceeds uniforms[b] * sum_{w in mask} exp(l_w)
 *                   (inverse-CDF sampling; the paper fixes no procedure); if rounding lets no token
 *                   exceed it, the last valid token with positive weight; -1 if the mask is empty or no
 *                   valid token has positive weight (the renormalised distribution is undefined then).
 * Arguments (all device pointers):
 *   logits      [B rows] of V elements of type dt, row b starts at element b*row_stride
 *               (row_stride >= V; rows must be 16-byte aligned: row_stride a multiple of 4 (f32) / 8 (bf16))
 *   mask        uint32[B, ceil(V/32)] in the layout above
 *   uniforms    float[B], each in [0, 1)
 *   ids         int32[B]     logZ_valid  float[B]     logZ_all  float[B] or NULL
 *   temperature host, T > 0 and finite.  The division is folded into the constant of the exponentials
 *               (no pass over the logits, no cost per token); T = 1 leaves the logits as they are.
 * Logits must be finite or -inf; accumulation is in fp32 with fp64 across partial sums.
 * Errors: PPV_EINVAL (null pointer, B < 0, V <= 0, row_stride < V or misaligned, bad dt, temperature not
 * a positive finite number), PPV_ERANGE (V > PPV_MAX_VOCAB), PPV_EDEVICE.
 */
ppv_status constrained_sample(const void *logits, ppv_dtype dt, int64_t row_stride, const uint32_t *mask,
                              const float *uniforms, int32_t B, int32_t V, int32_t *ids, float *logZ_valid,
                              float *logZ_all, float temperature, void *stream);

/*
 * constrained_sample_noalloc -- constrained_sample for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  constrained_sample spreads the rows
 * of a small batch over several workgroups, which meet in a scratch area that it allocates per stream on first
 * use; this call uses a fixed scratch array in device memory instead (about 4.3 MB, held on every GPU the library
 * runs on until the process ends) and calls no hipMalloc, hipFree or other allocating routine, ever.  Same
 * arguments, same results bit for bit.
 *   B     at most PPV_NOALLOC_MAX_ROWS rows (what the array holds): PPV_ERANGE beyond.
 * All calls on one GPU share the array: two calls of this function that overlap on one GPU (different streams)
 * race; calls on one stream, or otherwise ordered, do not.  Nothing has to be cleared between calls: every call
 * leaves the arrival counters at zero, which is what the next one starts from, and writes the statistics it reads.
 * The first call on a device looks up the array's address on that device (no allocation); make that first call
 * outside stream capture.
 * Errors: as constrained_sample; PPV_ERANGE also for B > PPV_NOALLOC_MAX_ROWS.
 */
#define PPV_NOALLOC_MAX_ROWS 512
ppv_status constrained_sample_noalloc(const void *logits, ppv_dtype dt, int64_t row_stride, const uint32_t *mask,
                                      const float *uniforms, int32_t B, int32_t V, int32_t *ids, float *logZ_valid,
                                      float *logZ_all, float temperature, void *stream);

/*
 * ppv_decode_begin -- Algorithm 1, SampleCandidate, initialisation step: the empty candidate sequence with
 * importance score x = 1 (or resume from given prefixes).  Locates each row's current prefix once
 * and leaves a cursor in `state`, so that every following ppv_decode_step costs one level of the
 * index instead of a walk from the root.
 * Arguments (all device pointers):
 *   prefixes, prefix_stride, lens   as in ppv_next_token_mask (lens[b] = 0: start from the empty prefix)
 *   state     uint32[B, PPV_STATE_WORDS], written; opaque, only ppv_decode_step reads and updates it
 *   active    uint8[B], written: 1 iff the row's prefix is a prefix of a member of S and is not
 *             itself a member (the row has something left to decode)
 *   logx      float[B] or NULL: set to 0 (log of the importance score x = 1)
 * Errors: PPV_EINVAL (null index/prefixes/lens/state/active, B < 0, prefix_stride < 0), PPV_EDEVICE.
 */
#define PPV_STATE_WORDS 8
ppv_status ppv_decode_begin(const ppv_index_t *index, const int32_t *prefixes, int32_t prefix_stride,
                            const int32_t *lens, int32_t B, uint32_t *state, uint8_t *active, float *logx,
                            void *stream);

/*
 * ppv_decode_begin_empty -- the same initialisation step for the case Algorithm 1 itself starts from: every row's
 * candidate is the empty sequence.  No prefix is read and nothing is located: all rows get the root's cursor, and
 * the lengths are written as well, so that a decode loop needs no separate fill of `lens`.  The results are those of
 * ppv_decode_begin with lens[b] = 0 for every row, bit for bit.
 *   lens    int32[B], written: 0            state, active, logx   as in ppv_decode_begin (active[b] = 1: the empty
 *           sequence is a prefix of every member and, members being non-empty, no member itself)
 * Errors: PPV_EINVAL (null index/lens/state/active, B < 0), PPV_EDEVICE.
 */
ppv_status ppv_decode_begin_empty(const ppv_index_t *index, int32_t B, int32_t *lens, uint32_t *state, uint8_t *active,
                                  float *logx, void *stream);

/*
 * ppv_decode_step -- one iteration of the while loop of Algorithm 1's SampleCandidate for B rows,
 * fused: the valid set of the row's prefix, a token drawn from it, the token appended, the importance score
 * multiplied by the valid mass, and the test whether the extended row is in S.
 * Equals ppv_next_token_mask + constrained_sample + append + membership test, but the mask never
 * leaves the chip.  Rows with active[b] == 0 are left untouched.
 * Arguments (all device pointers):
 *   prefixes  int32[B, prefix_stride], in/out: the sampled token is written at position lens[b]
 *   lens      int32[B], in/out: incremented for rows that sampled a token
 *   active    uint8[B], in/out: cleared when the extended row is a member of S (the row is done),
 *             and also (with ids[b] = -1, nothing appended, logx[b] = -inf) when the row has no valid token
 *             of positive probability or no room left (lens[b] == prefix_stride): such a row stops outside S
 *   state     uint32[B, PPV_STATE_WORDS] from ppv_decode_begin, in/out; or NULL: the prefix is then
 *             located from the root in every call (same results, one index level per token slower).
 *             With a state the caller must not change prefixes/lens of active rows between steps.
 *             Words that cannot be a cursor of this index (never initialised, or written for another
 *             index) are recognised by range checks: such a row samples nothing (ids[b] = -1) and retires.
 *   logits, dt, row_stride, uniforms, temperature   as in constrained_sample; V is the index's vocabulary
 *   ids         int32[B] or NULL: token sampled this step (-1 if none); untouched for inactive rows
 *   logZ_valid  float[B] or NULL: this step's log valid mass; untouched for inactive rows
 *   logx        float[B] or NULL, in/out: logx[b] += logZ_valid[b] (log of the importance score x) for a row that
 *               drew a token; -inf for a row that stopped outside S (Algorithm 1's update multiplies x by a valid
 *               mass of 0: ppv_disc_select never accepts such a candidate and gives it weight 0)
 * Errors: as the two calls above.
 */
ppv_status ppv_decode_step(const ppv_index_t *index, int32_t *prefixes, int32_t prefix_stride, int32_t *lens,
                           uint8_t *active, uint32_t *state, const void *logits, ppv_dtype dt, int64_t row_stride,
                           const float *uniforms, int32_t B, int32_t *ids, float *logZ_valid, float *logx,
                           float temperature, void *stream);

/*
 * ppv_decode_first_step -- ppv_decode_begin_empty and the first ppv_decode_step in one launch: the first iteration
 * of Algorithm 1's SampleCandidate, which always starts from the empty candidate.  Same arguments as
 * ppv_decode_step; what lens, active, state and logx hold on entry does not matter (every row's entry is overwritten;
 * state must not be NULL).  The results are those of the two calls, bit for bit.
 */
ppv_status ppv_decode_first_step(const ppv_index_t *index, int32_t *prefixes, int32_t prefix_stride, int32_t *lens,
                                 uint8_t *active, uint32_t *state, const void *logits, ppv_dtype dt,
                                 int64_t row_stride, const float *uniforms, int32_t B, int32_t *ids,
                                 float *logZ_valid, float *logx, float temperature, void *stream);

/*
 * ppv_sample_next -- ppv_next_token_mask and constrained_sample in one call, for callers that want the token and
 * the valid mass but not the mask itself: the three steps of the loop body of Algorithm 1's SampleCandidate that
 * do not change the candidate (valid set by PPV with M = |V|, draw, valid mass).  The valid set is read off the
 * index inside the kernel and never written to memory: per row this saves the V/8 bytes of mask written and read
 * back, and one launch.  Nothing of the caller's rows is changed.
 * Arguments (all device pointers):
 *   prefixes, prefix_stride, lens   as in ppv_next_token_mask (read only)
 *   logits, dt, row_stride, uniforms, temperature   as in constrained_sample; V is the index's vocabulary
 *   ids         int32[B]: the drawn token; -1 when the prefix has no valid next token of positive probability
 *               (it is a prefix of no member, a member without extensions, or all its valid tokens are at -inf)
 *   logZ_valid  float[B] or NULL: log of the valid mass (-inf with ids[b] = -1)
 * Results equal ppv_next_token_mask followed by constrained_sample up to the rounding of sums taken in another
 * order (both are within the stated tolerance of the exact value).
 * Errors: PPV_EINVAL (null index/prefixes/lens/uniforms/ids, B < 0, prefix_stride < 0, bad logits arguments or
 * temperature), PPV_ERANGE, PPV_EDEVICE.
 */
ppv_status ppv_sample_next(const ppv_index_t *index, const int32_t *prefixes, int32_t prefix_stride,
                           const int32_t *lens, int32_t B, const void *logits, ppv_dtype dt, int64_t row_stride,
                           const float *uniforms, int32_t *ids, float *logZ_valid, float temperature, void *stream);

/*
 * ppv_decode_loop -- the whole while loop of Algorithm 1's SampleCandidate in one launch: n_steps
 * iterations of ppv_decode_step, each workgroup staying with its row (cursor in registers, the next
 * step's logits requested while the current step is sampled).  For callers that hold the logits of
 * every step up front, i.e. whose distributions do not depend on the sampled tokens (scoring a fixed
 * proposal, replay, benchmarking the path without a model in between).  Results are identical to
 * n_steps calls of ppv_decode_step.
 * Arguments as in ppv_decode_step, except:
 *   logits       step s, row b starts at element s*step_stride + b*row_stride
 *   step_stride  elements between the [B, V] blocks of consecutive steps (a multiple of 4 (f32) / 8 (bf16))
 *   uniforms     float[n_steps, B]
 *   ids, logZ_valid   int32 / float [n_steps, B] or NULL; entries of steps a row did not take are not written
 * Errors: as ppv_decode_step; PPV_EINVAL also for n_steps < 0 or a misaligned step_stride.
 */
ppv_status ppv_decode_loop(const ppv_index_t *index, int32_t *prefixes, int32_t prefix_stride, int32_t *lens,
                           uint8_t *active, uint32_t *state, const void *logits, ppv_dtype dt, int64_t row_stride,
                           int64_t step_stride, const float *uniforms, int32_t n_steps, int32_t B, int32_t *ids,
                           float *logZ_valid, float *logx, float temperature, void *stream);

/*
 * ppv_topm_mask -- Algorithm 2 with M < |V| candidates, as the paper ran it (M = 50; 100, 500, 1000
 * in the appendix study of M), all four of its steps: the M most probable tokens, the candidate rows
 * a + [t_i], one search of sorted S per candidate, and the verdicts scattered into a mask over the
 * vocabulary; Section 3.2 "Selection of top candidate tokens".  The result is the mask of
 * ppv_next_token_mask restricted to the top-M tokens; feed it to constrained_sample for the
 * sampling step of Algorithm 1.
 * The top M are the M largest logits of the row (P = softmax(logits) has the same order); equal
 * logits are taken in increasing token id, -0 and +0 are equal.  Logits are finite or +/-inf: a row
 * that holds NaNs ends in a defined state (ids inside [0, V) or -1, nothing out of bounds), but its
 * candidates are unspecified.
 * The M candidate rows share their first |a| tokens: the prefix is
 * located once per row and each candidate is then searched by its last token.
 * Arguments (device pointers unless noted):
 *   index, prefixes, prefix_stride, lens   as in ppv_next_token_mask
 *   logits      device, [B, row_stride] of dt, 16-byte aligned, row_stride >= V and a multiple of
 *               4 (f32) / 8 (bf16); the model's next-token logits per row (a temperature T > 0 does not
 *               change their order, so the call takes none)
 *   M           host, 1 .. PPV_TOPM_MAX; a row has min(M, V) candidates
 *   top_ids     int32[B, M] or NULL: the row's candidates t_i in increasing token id; -1 beyond min(M, V)
 *   mask_V      uint8[B, M] or NULL: mask_V[b, i] = 1 iff a + [top_ids[b, i]] is a prefix of a member
 *   mask        uint32[B, ceil(V/32)]: bit t set iff t is a candidate and its mask_V is 1
 * A call that asks for the mask alone (top_ids and mask_V both NULL) returns the same mask, but where the prefix
 * has no more than eight continuations it need not select the M candidates at all: a continuation t is a candidate
 * iff fewer than M tokens come before it in the order above, and those are counted in one pass over the row (the
 * library does so where that is the faster way); a prefix without continuations reads no logits.
 * Errors: PPV_EINVAL (null pointer, M < 1, bad dtype / alignment / stride), PPV_ERANGE (M > PPV_TOPM_MAX),
 * PPV_EDEVICE.  B == 0 is PPV_OK.
 */
ppv_status ppv_topm_mask(const ppv_index_t *index, const int32_t *prefixes, int32_t prefix_stride,
                         const int32_t *lens, const void *logits, ppv_dtype dt, int64_t row_stride, int32_t M,
                         int32_t B, int32_t *top_ids, uint8_t *mask_V, uint32_t *mask, void *stream);

/*
 * ppv_disc_select -- Algorithm 1 after SampleCandidate: a candidate is accepted with probability equal to its
 * importance score x, in at most K rounds, then importance resampling among K candidates with probability
 * x_k / sum x_k.  The candidates of all
 * queries have been drawn beforehand (rows of ppv_decode_step / ppv_decode_loop; logx is their log
 * importance score), so the selection is a function of logx and the supplied uniforms.
 * Arguments (all device pointers):
 *   logx        float[n_candidates, Q]: candidate c of query q; candidates 0..K-1 go through the
 *               accept/reject rounds in order, candidates K..2K-1 are the fallback's fresh ones
 *   n_candidates  >= 2K, or >= K with reuse_rejected
 *   accept_u    float[K, Q] in [0,1): candidate k is accepted iff exp(logx) > accept_u (compared in fp64)
 *   resample_u  float[Q] in [0,1): the fallback takes, in candidate order, the first whose cumulative
 *               score exceeds resample_u * (sum of scores); the last one of positive score if rounding lets
 *               none exceed it.  A candidate of score 0 (logx = -inf: it stopped outside S) is never returned
 *   reuse_rejected  0: the fallback uses K new candidates (the algorithm as printed); 1: it resamples among
 *               the K rejected ones (then K = 1 is plain constrained decoding, Section 4.1 "Methods")
 *   chosen      int32[Q]: index of the returned candidate; -1 when no accept round passed and every fallback
 *               candidate has score 0 (nothing can be returned)
 *   n_draws     int32[Q] or NULL: candidates consumed (the k of Theorem 3.1: round of acceptance, else 2K / K)
 *   accepted    uint8[Q] or NULL: 1 iff returned by an accept round
 * Errors: PPV_EINVAL (K <= 0, Q < 0, too few candidates, null pointer), PPV_EDEVICE.
 */
ppv_status ppv_disc_select(const float *logx, int32_t n_candidates, int32_t K, int32_t Q, const float *accept_u,
                           const float *resample_u, int32_t reuse_rejected, int32_t *chosen, int32_t *n_draws,
                           uint8_t *accepted, void *stream);

/*
 * ppv_tuning_set / ppv_tuning_get -- process-wide tuning and test switches (not part of the method).  Each is
 * read once from the environment variable of the same name without the TUNE_ part (PPV_WAVES_PER_ROW, ...)
 * when the library is loaded; no per-step call reads the environment.  Setting one while calls are being
 * issued from another thread is a race.
 *   PPV_TUNE_WAVES_PER_ROW   wavefronts per row of the sampling kernels, 1..16; 0 = the library's table
 *   PPV_TUNE_TOPM_WAVES      the same for ppv_topm_mask
 *   PPV_TUNE_TOPM_STREAMING  1: every row of ppv_topm_mask takes the whole-row select (tests); 2: the usual select,
 *                            but also for mask-only calls on prefixes with few children (no counting); 0 = as needed
 *   PPV_TUNE_LOOKUP          0: ppv_build_index / ppv_index_load leave out the look-up table of whole prefixes
 *   PPV_TUNE_LOOKUP_WEAK     1: the table is built with one fingerprint for all entries (tests: every probe is
 *                            a false hit that the exact check must turn away)
 *   PPV_TUNE_ROW_SPLIT       workgroups a row is spread over in small batches, 1, 2, 4, 8, 16; 0 = the library's table
 * Errors: PPV_EINVAL (unknown knob, null pointer), PPV_ERANGE (value outside the knob's range).
 */
enum {
    PPV_TUNE_WAVES_PER_ROW = 0,
    PPV_TUNE_TOPM_WAVES = 1,
    PPV_TUNE_TOPM_STREAMING = 2,
    PPV_TUNE_LOOKUP = 3,
    PPV_TUNE_LOOKUP_WEAK = 4,
    PPV_TUNE_ROW_SPLIT = 5,
    PPV_TUNE_COUNT = 6
};
ppv_status ppv_tuning_set(int32_t knob, int32_t value);
ppv_status ppv_tuning_get(int32_t knob, int32_t *value);

#ifdef __cplusplus
}
#endif
#endif /* PPV_H */
