// DISC outer loop (Algorithm 1 after SampleCandidate): accept / reject rounds on the importance score
// x = exp(log x), then importance resampling proportional to x among the fallback candidates.
// One thread per query; the work is a few dozen flops per query, so this is launch-latency bound.
#include "ppv_internal.h"

namespace {

constexpr int DISC_THREADS = 256;

__global__ __launch_bounds__(DISC_THREADS) void disc_select_kernel(const float *__restrict__ logx, int K, int Q,
                                                                   const float *__restrict__ accept_u,
                                                                   const float *__restrict__ resample_u, int reuse,
                                                                   int32_t *__restrict__ chosen,
                                                                   int32_t *__restrict__ n_draws,
                                                                   uint8_t *__restrict__ accepted) {
    const int q = blockIdx.x * DISC_THREADS + threadIdx.x;
    if (q >= Q) return;
    // accept candidate k with probability x_k: x_k > epsilon_k, in double like the decision's definition
    for (int k = 0; k < K; k++) {
        const double x = exp((double)logx[(size_t)k * Q + q]);
        if (x > (double)accept_u[(size_t)k * Q + q]) {
            chosen[q] = k;
            if (n_draws) n_draws[q] = k + 1;
            if (accepted) accepted[q] = 1;
            return;
        }
    }
    // all K rejected: one of the K fallback candidates, candidate j with probability x_j / sum x
    const int first = reuse ? 0 : K;
    double m = -INFINITY;
    for (int j = 0; j < K; j++) m = fmax(m, (double)logx[(size_t)(first + j) * Q + q]);
    if (n_draws) n_draws[q] = reuse ? K : 2 * K;
    if (accepted) accepted[q] = 0;
    if (m == -INFINITY) {   // every score is 0 (all candidates stopped outside S): nothing can be returned
        chosen[q] = -1;
        return;
    }
    double total = 0.0;
    for (int j = 0; j < K; j++) total += exp((double)logx[(size_t)(first + j) * Q + q] - m);
    const double tau = (double)resample_u[q] * total;
    double c = 0.0;
    int pick = -1;   // the last candidate of positive score when rounding lets none exceed tau
    for (int j = 0; j < K; j++) {
        const double w = exp((double)logx[(size_t)(first + j) * Q + q] - m);
        c += w;
        if (w > 0.0) {
            pick = j;
            if (c > tau) break;
        }
    }
    chosen[q] = first + pick;
}

}  // namespace

extern "C" ppv_status ppv_disc_select(const float *logx, int32_t n_candidates, int32_t K, int32_t Q,
                                      const float *accept_u, const float *resample_u, int32_t reuse_rejected,
                                      int32_t *chosen, int32_t *n_draws, uint8_t *accepted, void *stream) {
    if (K <= 0 || Q < 0 || n_candidates < (reuse_rejected ? K : 2 * K)) return PPV_EINVAL;
    if (Q == 0) return PPV_OK;
    if (!logx || !accept_u || !resample_u || !chosen) return PPV_EINVAL;
    hipLaunchKernelGGL(disc_select_kernel, dim3((unsigned)((Q + DISC_THREADS - 1) / DISC_THREADS)), dim3(DISC_THREADS), 0,
                       (hipStream_t)stream, logx, K, Q, accept_u, resample_u, reuse_rejected ? 1 : 0, chosen, n_draws,
                       accepted);
    PPV_HIP_TRY(hipGetLastError());
    return PPV_OK;
}
