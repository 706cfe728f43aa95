// Streaming pass for more than 64 workers (up to kKWide).
//
// The one-sweep kernel keeps the K values of a vector in registers until the aggregate of the
// vector is known; beyond 64 workers that no longer fits, even with 4-byte loads.  This kernel
// reads the gradients twice instead, a super-tile of T tiles at a time:
//   sweep 1  tile by tile: G = sum_k w_k g_k over all K workers, sixteen at a time, k ascending;
//            A += G^2; G is parked in the LDS;
//   flush    the block writes the T tiles of G in one burst, between two barriers, with none of
//            its loads in flight (the same separation of reads and writes as in the one-sweep
//            kernel);
//   sweep 2  sixteen workers at a time over the T tiles: n_k += g^2, d_k += (g - G)^2 with G read
//            back from the LDS; after the T tiles the 32 sums are reduced over the wave and added
//            to per-wave fp64 accumulators in the LDS.
// HBM traffic is therefore 2 K P s bytes read (the second sweep of a super-tile comes too long
// after the first, and from too many blocks at once, for any cache to serve it) plus 4 P written.
// Same work decomposition, partial records, shared tail and final reduction as the one-sweep
// kernel; the order of every sum is fixed by the plan, so results are bitwise reproducible.
#include "stream_pass.h"

namespace dynamix {
namespace {

constexpr int kChunk = 16;   // workers whose vectors a lane holds at a time

template <int DT>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void wide_pass_kernel(
    const StreamArgs a, const int K)
{
    constexpr int VEC = DT == kF32 ? 4 : 8;       // elements per 16-byte vector
    constexpr int Q = VEC / 4;                    // 16-byte pieces of G per vector
    constexpr int VB = 16;
    constexpr int T = 32 / Q;                     // tiles per super-tile: 128 KB of G in the LDS
    constexpr int kSize = DT == kF32 ? 4 : 2;
    typedef Words<4> Wd;
    __shared__ u32x4 stage[T * Q][kBlock];
    __shared__ double acc[kWaves][2 * kKWide + 1];   // per wave: A, n_0.., d_0..
    __shared__ int next_piece;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int W = 2 * K + 1;
    const int chunks = (K + kChunk - 1) / kChunk;
    float* const out = a.out_agg;
    const int p_first = a.block_range[2 * blockIdx.x];
    const int p_last = a.block_range[2 * blockIdx.x + 1];
    const int n_tail = a.n_tail;
    bool drawn = false;

    // this lane's fp32 sums of one chunk of workers, reduced over the wave into the accumulators
    auto fold_chunk = [&](const float (&n)[kChunk], const float (&d)[kChunk], int k0) {
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
            const float rn = wave_sum(n[j]);
            const float rd = wave_sum(d[j]);
            if (lane == 0 && k0 + j < K) {
                acc[wave][1 + k0 + j] += (double)rn;
                acc[wave][1 + K + k0 + j] += (double)rd;
            }
        }
    };

    for (int p = p_first;; ++p) {
        if (drawn || p >= p_last) {
            drawn = true;
            if (n_tail == 0) break;
            if (tid == 0) {
                const int q = atomicAdd(a.queue, 1);
                next_piece = q < n_tail ? a.tail_order[q] : -1;
            }
            __syncthreads();
            p = __builtin_amdgcn_readfirstlane(next_piece);
            if (p < 0) break;
        }
        const Piece pc = a.pieces[p];
        for (int j = lane; j < W; j += 64) acc[wave][j] = 0.0;   // each wave clears its own row
        float A = 0.f;

        int64_t body_begin = pc.v_begin, body_end = pc.v_end;
        const bool head_cut = pc.e_lo > pc.v_begin * VEC;
        const bool tail_cut = pc.e_hi < pc.v_end * VEC;
        if (head_cut) ++body_begin;
        if (tail_cut && pc.v_end - 1 >= body_begin) --body_end;

        // A boundary vector (the vector at the head or tail of the piece that also holds elements
        // of a neighbouring segment, or the ragged end): lane 0 of wave 0, element by element,
        // masked elements pushed out of the descriptor's range.
        auto boundary_vector = [&](int64_t v, int64_t lo, int64_t hi) {
            int off[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const int64_t e = v * VEC + c;
                off[c] = (tid == 0 && e >= lo && e < hi) ? c * kSize : kMasked;
            }
            auto load_elems = [&](int k, float (&x)[VEC]) {
                const __amdgpu_buffer_rsrc_t r = tile_rsrc(a.g[k], v * VB, VB);
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    if constexpr (DT == kF32) {
                        x[c] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, off[c], 0, 0));
                    } else {
                        const uint32_t h = __builtin_amdgcn_raw_buffer_load_b16(r, off[c], 0, 0);
                        x[c] = elem_lo<DT>(h & 0xffffu);
                    }
                }
            };
            float Ge[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) Ge[c] = 0.f;
            for (int k = 0; k < K; ++k) {
                float x[VEC];
                load_elems(k, x);
                const float wk = a.w[k];
#pragma unroll
                for (int c = 0; c < VEC; ++c) Ge[c] = __builtin_fmaf(wk, x[c], Ge[c]);
            }
#pragma unroll
            for (int c = 0; c < VEC; ++c) A = __builtin_fmaf(Ge[c], Ge[c], A);
            if (out != nullptr) {
                const __amdgpu_buffer_rsrc_t r = tile_rsrc(out, v * (VEC * 4), VEC * 4);
#pragma unroll
                for (int c = 0; c < VEC; ++c)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(Ge[c]), r,
                                                          off[c] == kMasked ? kMasked : c * 4, 0, 0);
            }
            for (int k = 0; k < K; ++k) {
                float x[VEC];
                load_elems(k, x);
                float nk = 0.f, dk = 0.f;
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    nk = __builtin_fmaf(x[c], x[c], nk);
                    const float t = x[c] - Ge[c];
                    dk = __builtin_fmaf(t, t, dk);
                }
                if (tid == 0) {   // (masked elements read zero and leave G zero: they add nothing)
                    acc[0][1 + k] += (double)nk;
                    acc[0][1 + K + k] += (double)dk;
                }
            }
        };
        if (tid < 64) {   // wave 0 only; its row of accumulators was cleared by its own lanes
            if (head_cut)
                boundary_vector(pc.v_begin, pc.e_lo, min(pc.e_hi, (pc.v_begin + 1) * VEC));
            if (tail_cut && pc.v_end - 1 >= body_begin)
                boundary_vector(pc.v_end - 1, (pc.v_end - 1) * VEC, pc.e_hi);
        }

        // ---- the body, a super-tile of T tiles (of kBlock vectors) at a time
        for (int64_t sv = body_begin; sv < body_end; sv += (int64_t)T * kBlock) {
            const int sup_vectors = (int)min((int64_t)T * kBlock, body_end - sv);
            const int tiles = (sup_vectors + kBlock - 1) / kBlock;
            // vectors of tile t that exist (the last tile of the body may be short: its
            // descriptors are short, the lanes beyond read zero and write nothing)
            auto tile_bytes = [&](int t) { return min(kBlock, sup_vectors - t * kBlock) * VB; };
            // One worker's vector for step `s` of a sweep (steps enumerate (tile, chunk) pairs; a
            // step past the end, or a worker beyond K, reads nothing).  Loads are issued one by
            // one, each into the registers whose previous vector has just been used, so sixteen
            // loads per lane stay in flight without a second set of registers; `tie` orders the
            // load after that use (otherwise the scheduler hoists the loads and the live ranges
            // double).
            auto load_one = [&](int t, int k, bool valid, float tie0, float tie1) -> u32x4 {
                int off = tid * VB;
                asm volatile("" : "+v"(off) : "v"(tie0), "v"(tie1));
                const int kk = k < K ? k : K - 1;
                return Wd::template load<kLoadPolicy>(
                    tile_rsrc(a.g[kk], (sv + (int64_t)t * kBlock) * VB,
                              valid && k < K ? tile_bytes(t) : 0), off);
            };

            // sweep 1: the aggregate of every tile, parked in the LDS
            {
                u32x4 x[kChunk];
#pragma unroll
                for (int j = 0; j < kChunk; ++j) x[j] = load_one(0, j, true, 0.f, 0.f);
                const int steps = tiles * chunks;
                float G[VEC];
                int t = 0, c = 0;              // tile and chunk of step s
                for (int s = 0; s < steps; ++s) {
                    int tn = t, cn = c + 1;    // ... and of step s + 1
                    if (cn == chunks) {
                        cn = 0;
                        ++tn;
                    }
                    const bool more = s + 1 < steps;
                    if (c == 0) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) G[e] = 0.f;
                    }
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) {
                        const int k = c * kChunk + j;
                        const float wk = k < K ? a.w[k] : 0.f;
#pragma unroll
                        for (int w4 = 0; w4 < 4; ++w4) {
                            const uint32_t q = x[j][w4];
                            if constexpr (DT == kF32) {
                                G[w4] = __builtin_fmaf(wk, __uint_as_float(q), G[w4]);
                            } else {
                                G[2 * w4] = __builtin_fmaf(wk, elem_lo<DT>(q), G[2 * w4]);
                                G[2 * w4 + 1] = __builtin_fmaf(wk, elem_hi<DT>(q), G[2 * w4 + 1]);
                            }
                        }
                        x[j] = load_one(tn, cn * kChunk + j, more, G[0], G[VEC - 1]);
                    }
                    if (c == chunks - 1) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) A = __builtin_fmaf(G[e], G[e], A);
#pragma unroll
                        for (int h = 0; h < Q; ++h) {
                            u32x4 q;
#pragma unroll
                            for (int w4 = 0; w4 < 4; ++w4) q[w4] = __float_as_uint(G[4 * h + w4]);
                            stage[t * Q + h][tid] = q;   // read back by this lane only
                        }
                    }
                    t = tn;
                    c = cn;
                }
            }

            // flush: the block writes the super-tile of G with none of its loads in flight
            if (out != nullptr) {
                __syncthreads();
                const __amdgpu_buffer_rsrc_t r = tile_rsrc(out, sv * (VEC * 4), sup_vectors * (VEC * 4));
                for (int t = 0; t < tiles; ++t)
#pragma unroll
                    for (int h = 0; h < Q; ++h)
                        Wd::template store<kStorePolicy>(stage[t * Q + h][tid], r,
                                                         (t * kBlock + tid) * (VEC * 4) + VB * h);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
            }

            // sweep 2: squared norms and squared deviations, sixteen workers at a time
            {
                u32x4 x[kChunk];
#pragma unroll
                for (int j = 0; j < kChunk; ++j) x[j] = load_one(0, j, true, 0.f, 0.f);
                const int steps = chunks * tiles;
                float n[kChunk], d[kChunk];
                int c = 0, t = 0;
                for (int s = 0; s < steps; ++s) {
                    int cn = c, tn = t + 1;
                    if (tn == tiles) {
                        tn = 0;
                        ++cn;
                    }
                    const bool more = s + 1 < steps;
                    if (t == 0) {
#pragma unroll
                        for (int j = 0; j < kChunk; ++j) n[j] = d[j] = 0.f;
                    }
                    float G[VEC];
#pragma unroll
                    for (int h = 0; h < Q; ++h) {
                        const u32x4 q = stage[t * Q + h][tid];
#pragma unroll
                        for (int w4 = 0; w4 < 4; ++w4) G[4 * h + w4] = __uint_as_float(q[w4]);
                    }
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) {
#pragma unroll
                        for (int w4 = 0; w4 < 4; ++w4) {
                            const uint32_t q = x[j][w4];
                            if constexpr (DT == kF32) {
                                const float g = __uint_as_float(q);
                                n[j] = __builtin_fmaf(g, g, n[j]);
                                const float u = g - G[w4];
                                d[j] = __builtin_fmaf(u, u, d[j]);
                            } else {
                                const float g0 = elem_lo<DT>(q), g1 = elem_hi<DT>(q);
                                n[j] = __builtin_fmaf(g0, g0, n[j]);
                                n[j] = __builtin_fmaf(g1, g1, n[j]);
                                const float u0 = g0 - G[2 * w4], u1 = g1 - G[2 * w4 + 1];
                                d[j] = __builtin_fmaf(u0, u0, d[j]);
                                d[j] = __builtin_fmaf(u1, u1, d[j]);
                            }
                        }
                        x[j] = load_one(tn, cn * kChunk + j, more, n[j], d[j]);
                    }
                    if (t == tiles - 1) fold_chunk(n, d, c * kChunk);
                    c = cn;
                    t = tn;
                }
            }
            // (the next super-tile overwrites the parked G: every lane reads and writes only its
            // own slots, so no barrier is needed in between)
        }

        // the piece's record: A over the wave, then the four waves' rows added in fp64
        {
            const float r = wave_sum(A);
            if (lane == 0) acc[wave][0] += (double)r;
        }
        __syncthreads();
        for (int j = tid; j < W; j += kBlock) {
            double s = 0.0;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) s += acc[wv][j];
            a.partials[static_cast<int64_t>(p) * W + j] = s;
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_wide_pass(int K, int dtype, int grid, const StreamArgs& a, hipStream_t s)
{
    if (K <= kKMax || K > kKWide) return hipErrorInvalidValue;
    switch (dtype) {
    case kF32: wide_pass_kernel<kF32><<<dim3(grid), dim3(kBlock), 0, s>>>(a, K); break;
    case kBF16: wide_pass_kernel<kBF16><<<dim3(grid), dim3(kBlock), 0, s>>>(a, K); break;
    case kF16: wide_pass_kernel<kF16><<<dim3(grid), dim3(kBlock), 0, s>>>(a, K); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

int wide_pass_blocks_per_cu(int dtype)
{
    int nb = 0;
    hipError_t e = hipErrorInvalidValue;
    switch (dtype) {
    case kF32: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, wide_pass_kernel<kF32>, kBlock, 0); break;
    case kBF16: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, wide_pass_kernel<kBF16>, kBlock, 0); break;
    case kF16: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, wide_pass_kernel<kF16>, kBlock, 0); break;
    default: break;
    }
    return e == hipSuccess ? nb : 0;
}

}  // namespace dynamix
