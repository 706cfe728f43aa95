// Final reduction: folds the per-piece partial sums of the streaming pass into the statistics
// records, in double precision and in a fixed order (no atomics), then derives the scalars.
//
// One block per record.  Level 1: the pieces of the record are dealt round-robin to row groups
// and every (row group, column) thread adds its pieces in increasing order (four interleaved
// running sums, folded in a fixed order).  Level 2: the row
// groups of a column are added in increasing order.  The order depends only on the plan, so the
// result is bitwise reproducible.
//
// Record 0 folds every piece, which with many pieces is more than one compute unit reads quickly
// (a thousand pieces at K = 32: 0.7 MB, 15 us).  It is then cut into `slices` equal ranges of
// pieces, one block each; every block leaves the sums of its range in global memory, and a second,
// one-block kernel adds the ranges in increasing order and writes the record.  (One launch with
// the last block to finish doing that costs more than it saves: the fences it needs write back and
// invalidate the L2, 7 us.)
#include "dynamix_internal.h"

namespace dynamix {

constexpr int kFinalBlock = 1024;

// The record: per-worker sums as they are, the scalars derived from them by one thread.
__device__ void write_record(const FinalArgs& a, int rec, const double* tot, int tid)
{
    const int K = a.K;
    const int R = kHead + 2 * K;
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

__global__ __launch_bounds__(kFinalBlock) void final_reduce_kernel(const FinalArgs a)
{
    const int K = a.K;
    const int W = 2 * K + 1;
    // blocks [0, slices) share record 0, the others have a record each
    const int slices = a.slices;
    const bool shared = slices > 1 && (int)blockIdx.x < slices;
    const int rec = (int)blockIdx.x < slices ? 0 : (int)blockIdx.x - slices + 1;
    const int tid = threadIdx.x;
    int p0 = a.rec_range[2 * rec];
    int p1 = a.rec_range[2 * rec + 1];
    if (shared) {
        const int per = (p1 - p0 + slices - 1) / slices;
        p0 = min(p1, p0 + (int)blockIdx.x * per);
        p1 = min(p1, p0 + per);
    }
    const int groups = kFinalBlock / W;  // >= 1 because W <= 513
    // the streaming pass before this kernel has drawn all of its tail pieces
    if (blockIdx.x == 0 && tid == 0) *a.queue = 0;

    __shared__ double part[kFinalBlock];
    __shared__ double tot[2 * kKWide + 1];

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
    if (shared) {
        // leave the sums of this range to the kernel that follows
        if (tid < W) a.slice_sums[(int)blockIdx.x * W + tid] = tot[tid];
        return;
    }
    write_record(a, rec, tot, tid);
}

// Record 0 from the sums of its ranges (launched after final_reduce_kernel when slices > 1).
__global__ __launch_bounds__(2 * kKWide + 1) void final_fold_kernel(const FinalArgs a)
{
    const int W = 2 * a.K + 1;
    const int tid = threadIdx.x;
    __shared__ double tot[2 * kKWide + 1];
    if (tid < W) {
        double s = 0.0;
        for (int m = 0; m < a.slices; ++m) s += a.slice_sums[m * W + tid];
        tot[tid] = s;
    }
    __syncthreads();
    write_record(a, 0, tot, tid);
}

hipError_t launch_final_reduce(int records, const FinalArgs& a, hipStream_t s)
{
    final_reduce_kernel<<<dim3(records + a.slices - 1), dim3(kFinalBlock), 0, s>>>(a);
    if (a.slices > 1) final_fold_kernel<<<dim3(1), dim3(2 * kKWide + 1), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace dynamix
