// Internal declarations shared by the HIP translation units of libdynamix (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dynamix {

constexpr int kKMax = 64;        // most workers of the one-sweep kernels (all K values of a vector in registers)
constexpr int kKWide = 256;      // most workers per call (two-sweep kernel above kKMax); pointers
                                 // and weights travel by value in the kernel arguments
// Threads per block of the streaming pass: four wave64, one per SIMD of the compute unit the
// block has to itself, so that a wave may use up to 512 registers (four waves read as fast as
// eight: measured).
constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kHead = 8;         // scalars in front of the per-worker entries of a record

enum : int { kF32 = 0, kBF16 = 1, kF16 = 2 };
constexpr int kDtypes = 3;

// What the streaming pass does with the aggregate: write it (or apply plain SGD to the parameters
// in place of the write), or carry optimizer state through the same pass.  An update with state
// writes 1 + (number of state vectors) streams and reads them first.
enum : int { kOptNone = 0, kOptMomentum = 1, kOptAdam = 2 };
constexpr int kOpts = 3;
constexpr int kKMaxOpt = 32;     // most workers for the updates with state (register budget)
constexpr int kKWideLoadsOpt = 24;   // ... with 16-byte loads; above, they take 8-byte loads
constexpr int out_streams(int opt) { return 1 + opt; }

// Vectors (16-byte loads) per thread and block iteration.  Small K gets several so that each
// lane keeps enough independent loads in flight; K x U x 4 data registers stay live until the
// aggregate of the vector is known.  The updates with state also hold a vector of every state
// stream per unrolled vector, and park two or three streams instead of one, so they unroll less.
constexpr int unroll_for(int K, int opt = kOptNone)
{
    return opt == kOptNone ? (K <= 2 ? 8 : K <= 8 ? 4 : K <= 16 ? 2 : 1) : (K <= 2 ? 4 : K <= 8 ? 2 : 1);
}

// 32-bit words a lane loads at a time: four (128-bit loads) up to 32 workers, two up to 48, one
// above, so that the K vectors of a lane plus the 2K+1 running sums stay within the 256 vector
// registers an instruction can address.
constexpr int load_words_for(int K, int opt = kOptNone)
{
    return opt != kOptNone && K > kKWideLoadsOpt ? 2 : K > kKMax ? 4 : K > 48 ? 1 : K > 32 ? 2 : 4;
}
// Whether the streaming pass for K workers may take its tiles as interleaved 256-byte chunks
// (see stream_pass.h); the host then starts every block's span at a multiple of 4 KB.
constexpr bool interleaves(int K, int opt = kOptNone)
{
    return K >= 8 && K <= 32 && load_words_for(K, opt) == 4;
}
// elements per vector
constexpr int vec_elems(int K, int dtype, int opt = kOptNone)
{
    return load_words_for(K, opt) * (dtype == kF32 ? 1 : 2);
}

// One unit of streaming work: vectors v_begin, v_begin + v_step, ... below v_end are the
// starts of the block iterations; elements outside [e_lo, e_hi) are masked (segment edges and
// the ragged tail).  One partial record of 2K+1 sums is produced per piece.
struct Piece {
    int64_t v_begin;
    int64_t v_end;
    int64_t v_step;
    int64_t e_lo;
    int64_t e_hi;
    int64_t block;   // owning block, or -1 - round for a piece of the shared tail (diagnostics only)
};

struct StreamArgs {
    const void* g[kKWide];       // K device pointers
    float w[kKWide];             // b_k / B, rounded once to fp32
    const Piece* pieces;
    const int32_t* block_range;  // [grid][2] first and one-past-last piece of each block
    float* out_agg;              // may be null
    double* partials;            // [pieces][2K+1]: A, n_0..n_{K-1}, d_0..d_{K-1}
    // The pieces listed in tail_order belong to no block: a block that has finished its own
    // pieces draws them one at a time by adding 1 to *queue (zero at launch; the final reduction,
    // which follows every streaming pass on the same stream, sets it back).
    const int32_t* tail_order;   // [n_tail] piece indices
    int32_t* queue;
    int32_t n_tail;
    float* params;               // fused model update: p <- p - lr (G + wd p) in place; else null
    float lr, wd;
    // Updates with state (kOptMomentum: state1 = momentum buffer; kOptAdam: state1, state2 = first
    // and second moment), read and written in place like params.  hp: the update's constants,
    // prepared on the host (see optimizer_constants in api.hip); flags: bit 0 Nesterov / decoupled.
    float* state1;
    float* state2;
    float hp[8];
    int32_t flags;
    // Non-zero: every worker buffer and the output start at a multiple of 256 bytes, and the
    // kernel may take its tiles as 256-byte chunks of several 4 KB units (see stream_pass.h).
    int32_t spread;
};

struct FinalArgs {
    double b[kKWide];            // batch sizes
    double B;                    // their sum
    const double* partials;
    const int32_t* rec_range;    // [records][2]: first and one-past-last piece of each record
    const double* rec_count;     // [records] elements covered
    double* out_stats;           // [records][8 + 2K]
    int32_t* queue;              // the streaming pass's tail counter, reset here
    double* slice_sums;          // [slices][2K+1] sums of the ranges record 0 is cut into
    int32_t slices;              // >= 1 blocks that share record 0
    int32_t K;
};

// Enqueue the streaming pass for (K, dtype, opt); returns hipErrorInvalidValue for an unknown
// combination.
hipError_t launch_stream_pass(int K, int dtype, int opt, int grid, const StreamArgs& a, hipStream_t s);
// Resident blocks per compute unit of that kernel (0 on error).
int stream_pass_blocks_per_cu(int K, int dtype, int opt);
hipError_t launch_final_reduce(int records, const FinalArgs& a, hipStream_t s);
// The two-sweep kernel for kKMax < K <= kKWide (aggregate written or statistics only).
hipError_t launch_wide_pass(int K, int dtype, int grid, const StreamArgs& a, hipStream_t s);
int wide_pass_blocks_per_cu(int dtype);

// One instantiation unit per update kind, dtype and group of eight K:
// launch_stream_pass_<opt>_<dtype>_<first K>.
#define DYNAMIX_DECLARE_UNIT(OPT, DT, LO)                                                          \
    hipError_t launch_stream_pass_##OPT##_##DT##_##LO(int K, int grid, const StreamArgs& a, hipStream_t s); \
    int occupancy_stream_pass_##OPT##_##DT##_##LO(int K);
#define DYNAMIX_FOR_EACH_PLAIN_UNIT(X, DT) \
    X(0, DT, 1) X(0, DT, 9) X(0, DT, 17) X(0, DT, 25) X(0, DT, 33) X(0, DT, 41) X(0, DT, 49) X(0, DT, 57)
#define DYNAMIX_FOR_EACH_STATE_UNIT(X, OPT, DT) X(OPT, DT, 1) X(OPT, DT, 9) X(OPT, DT, 17) X(OPT, DT, 25)
DYNAMIX_FOR_EACH_PLAIN_UNIT(DYNAMIX_DECLARE_UNIT, 0)
DYNAMIX_FOR_EACH_PLAIN_UNIT(DYNAMIX_DECLARE_UNIT, 1)
DYNAMIX_FOR_EACH_PLAIN_UNIT(DYNAMIX_DECLARE_UNIT, 2)
DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_DECLARE_UNIT, 1, 0)
DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_DECLARE_UNIT, 1, 1)
DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_DECLARE_UNIT, 1, 2)
DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_DECLARE_UNIT, 2, 0)
DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_DECLARE_UNIT, 2, 1)
DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_DECLARE_UNIT, 2, 2)

}  // namespace dynamix
