// Final reduction: folds the per-piece partial sums of the streaming pass into the statistics
// records, in double precision and in a fixed order (no atomics), then derives the scalars.
//
// One block per record.  Level 1: the pieces of the record are dealt round-robin to row groups
// and every (row group, column) thread adds its pieces in increasing order (four interleaved
// running sums, folded in a fixed order).  Level 2: the row
// groups of a column are added in increasing order.  The order depends only on the plan, so the
// result is bitwise reproducible.
#include "dynamix_internal.h"

namespace dynamix {

constexpr int kFinalBlock = 1024;

__global__ __launch_bounds__(kFinalBlock) void final_reduce_kernel(const FinalArgs a)
{
    const int K = a.K;
    const int W = 2 * K + 1;
    const int R = kHead + 2 * K;
    const int rec = blockIdx.x;
    const int tid = threadIdx.x;
    const int p0 = a.rec_range[2 * rec];
    const int p1 = a.rec_range[2 * rec + 1];
    const int groups = kFinalBlock / W;  // >= 7 because W <= 129

    __shared__ double part[kFinalBlock];
    __shared__ double tot[2 * kKMax + 1];

    if (tid < W * groups) {
        const int col = tid % W, grp = tid / W;
        // four independent running sums keep four loads in flight; they are folded in a fixed
        // order, so the result depends only on the plan
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        int p = p0 + grp;
        for (; p + 3 * groups < p1; p += 4 * groups) {
            s0 += a.partials[(int64_t)p * W + col];
            s1 += a.partials[(int64_t)(p + groups) * W + col];
            s2 += a.partials[(int64_t)(p + 2 * groups) * W + col];
            s3 += a.partials[(int64_t)(p + 3 * groups) * W + col];
        }
        for (; p < p1; p += groups) s0 += a.partials[(int64_t)p * W + col];
        part[tid] = (s0 + s1) + (s2 + s3);
    }
    __syncthreads();
    if (tid < W) {
        double s = 0.0;
        for (int grp = 0; grp < groups; ++grp) s += part[grp * W + tid];
        tot[tid] = s;
    }
    __syncthreads();

    double* out = a.out_stats + (int64_t)rec * R;
    if (tid < K) {
        out[kHead + tid] = tot[1 + tid];          // n_k
        out[kHead + K + tid] = tot[1 + K + tid];  // d_k
    }
    if (tid == 0) {
        const double A = tot[0];
        double wd = 0.0;
        for (int k = 0; k < K; ++k) wd += a.b[k] * tot[1 + K + k];
        const double T = K > 1 ? wd / (double)(K - 1) : 0.0;
        const double A_unb = A - T / a.B;
        const double s2 = T / (a.B * A);
        out[0] = A;
        out[1] = T;
        out[2] = A_unb;
        out[3] = T / A_unb;
        out[4] = T / A;
        out[5] = s2;
        out[6] = sqrt(s2 > 0.0 ? s2 : 0.0);
        out[7] = a.rec_count[rec];
    }
}

hipError_t launch_final_reduce(int records, const FinalArgs& a, hipStream_t s)
{
    final_reduce_kernel<<<dim3(records), dim3(kFinalBlock), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace dynamix
