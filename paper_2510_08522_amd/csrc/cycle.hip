// Per-cycle aggregation of the statistics records (the paper aggregates metrics over k consecutive
// iterations before each decision, and its reward for adaptive optimizers carries
// -eta (sigma_norm^2 + sigma_norm) and the batch size regulariser -delta (log2 b - 5)).
// Two tiny fp64 kernels: a running sum of the records on the device, and the summary that turns
// the sums into means, pooled ratios and the two reward terms.  Nothing here touches gradients.
#include "../../include/dynamix.h"
#include "dynamix_internal.h"

namespace dynamix {

constexpr int kCycleExtra = 4;

__global__ __launch_bounds__(256) void cycle_accumulate_kernel(const double* stats, int64_t count,
                                                               double* window, int first)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) window[i] = first ? stats[i] : window[i] + stats[i];
    if (i == count) window[i] = first ? 1.0 : window[i] + 1.0;   // iterations accumulated
}

struct CycleArgs {
    double b[kKWide];
    double B, eta, delta;
    const double* window;
    double* summary;
    int32_t K;
    int32_t records;
};

__global__ __launch_bounds__(256) void cycle_summary_kernel(const CycleArgs a)
{
    const int K = a.K;
    const int R = kHead + 2 * K;
    const int rec = blockIdx.x;
    const int tid = threadIdx.x;
    const double iters = a.window[(int64_t)a.records * R];
    if (rec < a.records) {
        const double* w = a.window + (int64_t)rec * R;
        double* out = a.summary + (int64_t)rec * (R + kCycleExtra);
        for (int j = tid; j < R; j += blockDim.x) out[j] = w[j] / iters;
        if (tid == 0) {
            const double A = w[0] / iters, T = w[1] / iters;
            const double s2 = T / (a.B * A);
            out[R + 0] = T / (A - T / a.B);
            out[R + 1] = s2;
            out[R + 2] = sqrt(s2 > 0.0 ? s2 : 0.0);
            out[R + 3] = -a.eta * (w[5] / iters + w[6] / iters);
        }
    } else {
        // one extra block: the per-worker batch size regulariser
        double* tail = a.summary + (int64_t)a.records * (R + kCycleExtra);
        if (tid < K) tail[tid] = -a.delta * (log2(a.b[tid]) - 5.0);
    }
}

}  // namespace dynamix

extern "C" {

int64_t dynamix_cycle_summary_count(int32_t K, int64_t num_segments)
{
    if (K < 1 || K > DYNAMIX_K_MAX || num_segments < 0) return -1;
    return (1 + num_segments) * (int64_t)(DYNAMIX_STATS_HEAD + 2 * K + dynamix::kCycleExtra) + K;
}

int dynamix_cycle_accumulate(const double* stats, int64_t count, double* window, int32_t first,
                             void* stream)
{
    if (!stats || !window) return DYNAMIX_ERR_NULL;
    if (count < 1 || count > (int64_t)1 << 40) return DYNAMIX_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(stats) & 7u) || (reinterpret_cast<uintptr_t>(window) & 7u))
        return DYNAMIX_ERR_ALIGN;
    const int64_t blocks = (count + 1 + 255) / 256;
    dynamix::cycle_accumulate_kernel<<<dim3((unsigned)blocks), dim3(256), 0,
                                       static_cast<hipStream_t>(stream)>>>(stats, count, window,
                                                                           first != 0);
    return hipGetLastError() == hipSuccess ? DYNAMIX_OK : DYNAMIX_ERR_HIP;
}

int dynamix_cycle_summary(const double* window, int32_t K, int64_t num_segments,
                          const int32_t* batch_sizes, double eta, double delta, double* summary,
                          void* stream)
{
    if (!window || !batch_sizes || !summary) return DYNAMIX_ERR_NULL;
    if (K < 1 || K > DYNAMIX_K_MAX) return DYNAMIX_ERR_ARG;
    if (num_segments < 0 || num_segments > INT32_MAX / 4) return DYNAMIX_ERR_SEGMENTS;
    for (int k = 0; k < K; ++k)
        if (batch_sizes[k] <= 0) return DYNAMIX_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(window) & 7u) || (reinterpret_cast<uintptr_t>(summary) & 7u))
        return DYNAMIX_ERR_ALIGN;
    dynamix::CycleArgs a;
    int64_t B = 0;
    for (int k = 0; k < dynamix::kKWide; ++k) a.b[k] = 0.0;
    for (int k = 0; k < K; ++k) {
        a.b[k] = (double)batch_sizes[k];
        B += batch_sizes[k];
    }
    a.B = (double)B;
    a.eta = eta;
    a.delta = delta;
    a.window = window;
    a.summary = summary;
    a.K = K;
    a.records = (int32_t)(1 + num_segments);
    dynamix::cycle_summary_kernel<<<dim3((unsigned)a.records + 1), dim3(256), 0,
                                    static_cast<hipStream_t>(stream)>>>(a);
    return hipGetLastError() == hipSuccess ? DYNAMIX_OK : DYNAMIX_ERR_HIP;
}

}  // extern "C"
