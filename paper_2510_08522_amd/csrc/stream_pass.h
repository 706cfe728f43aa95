// Streaming pass: one sweep over the K gradient buffers (Algorithm 1 of the paper: gradient
// synchronisation fused with the gradient part of metric collection).
//
// Per 16-byte vector a lane loads the K workers' values, forms the weighted aggregate
// G = sum_k w_k g_k in a fixed k order, and then, while the K values are still in registers,
// adds g^2 to the worker's squared norm, (g - G)^2 to its squared deviation and G^2 to the
// aggregate's squared norm.  Nothing is read twice and the only write is G.  The kernel is
// bound by HBM bandwidth (about one flop per byte), so there is no LDS tiling of the data and no
// MFMA: the work is coalesced 128-bit loads, fp32 FMAs and one block reduction per piece.
#pragma once
#include "dynamix_internal.h"

namespace dynamix {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// Sum over the 64 lanes of a wave, same bits in every lane.  Four DPP steps give each row of 16
// lanes its sum (swap inside pairs, swap pairs inside quads, mirror the half row, mirror the
// row); the four row sums are then read out and added in a fixed order.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);  // row_half_mirror
    v += dpp_move<0x140>(v);  // row_mirror
    const int b = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
    return (r0 + r1) + (r2 + r3);
}

template <int DT>
struct Elem;
template <>
struct Elem<kF32> {
    static constexpr int kVec = 4;   // elements per 16 bytes
    static constexpr int kSize = 4;
};
template <>
struct Elem<kBF16> {
    static constexpr int kVec = 8;
    static constexpr int kSize = 2;
};

// Buffer descriptor over one tile of a stream: the uniform 64-bit base (pointer + tile start)
// lives in scalar registers and every lane adds only a 32-bit byte offset, so no per-worker
// address pair occupies vector registers.  Accesses at or beyond `bytes` are dropped by the
// hardware: loads return zero and stores are discarded.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const void* base, int64_t byte_off,
                                                            int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(static_cast<const char*>(base)) + byte_off, /*stride=*/0,
        /*num_records=*/bytes, /*flags=*/0x00020000);
}

constexpr int kNT = 2;               // cache-policy bit "non-temporal": data is touched once
constexpr int kLoadPolicy = kNT;     // gradient loads of interior tiles
constexpr int kStorePolicy = kNT;    // aggregate stores of interior tiles
constexpr int kMasked = 0x7ffffff0;  // a lane offset beyond every tile: the access is dropped

template <int K, int DT, int U>
__global__ __launch_bounds__(kBlock) void stream_pass_kernel(const StreamArgs a)
{
    constexpr int VEC = Elem<DT>::kVec;
    constexpr int W = 2 * K + 1;
    __shared__ float wave_part[kWaves][W];

    const int tid = threadIdx.x;
    const int p_first = a.block_first[blockIdx.x];
    const int p_last = a.block_first[blockIdx.x + 1];

    for (int p = p_first; p < p_last; ++p) {
        const Piece pc = a.pieces[p];
        float n[K], d[K], A = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k) n[k] = d[k] = 0.f;

        for (int64_t v0 = pc.v_begin; v0 < pc.v_end; v0 += pc.v_step) {
            // block-uniform: every element of this iteration lies inside the piece
            const bool interior =
                v0 * VEC >= pc.e_lo && (v0 + (int64_t)kBlock * U) * VEC <= pc.e_hi;
            u32x4 x[U][K];
            if (interior) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int k = 0; k < K; ++k)
                        x[u][k] = __builtin_amdgcn_raw_buffer_load_b128(
                            tile_rsrc(a.g[k], v0 * 16, kBlock * U * 16),
                            (u * kBlock + tid) * 16, 0, kLoadPolicy);
            } else {
                // edge tile (segment boundary or ragged tail): element-wise loads whose lane
                // offset is pushed out of range for masked elements, which then read as zero
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    int off[VEC];
#pragma unroll
                    for (int c = 0; c < VEC; ++c) {
                        const int64_t e = (v0 + (u * kBlock + tid)) * VEC + c;
                        off[c] = (e >= pc.e_lo && e < pc.e_hi)
                                     ? ((u * kBlock + tid) * VEC + c) * Elem<DT>::kSize
                                     : kMasked;
                    }
#pragma unroll
                    for (int k = 0; k < K; ++k) {
                        const __amdgpu_buffer_rsrc_t r =
                            tile_rsrc(a.g[k], v0 * 16, kBlock * U * 16);
                        if constexpr (DT == kF32) {
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                x[u][k][c] = __builtin_amdgcn_raw_buffer_load_b32(r, off[c], 0, 0);
                        } else {
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const uint32_t lo =
                                    __builtin_amdgcn_raw_buffer_load_b16(r, off[2 * c], 0, 0);
                                const uint32_t hi =
                                    __builtin_amdgcn_raw_buffer_load_b16(r, off[2 * c + 1], 0, 0);
                                x[u][k][c] = (lo & 0xffffu) | (hi << 16);
                            }
                        }
                    }
                }
            }

#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t v = v0 + (u * kBlock + tid);
                // pass 1 over the K values in registers: the weighted aggregate
                float G[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) G[c] = 0.f;
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    const float wk = a.w[k];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const uint32_t q = x[u][k][c];
                        if constexpr (DT == kF32) {
                            G[c] = __builtin_fmaf(wk, __uint_as_float(q), G[c]);
                        } else {
                            // bf16 is the upper half of fp32: widening is a shift or a mask, exact
                            G[2 * c] = __builtin_fmaf(wk, __uint_as_float(q << 16), G[2 * c]);
                            G[2 * c + 1] =
                                __builtin_fmaf(wk, __uint_as_float(q & 0xffff0000u), G[2 * c + 1]);
                        }
                    }
                }
#pragma unroll
                for (int c = 0; c < VEC; ++c) A = __builtin_fmaf(G[c], G[c], A);

                // the only write of the pass, issued as soon as G is known
                if (a.out_agg != nullptr) {
                    const __amdgpu_buffer_rsrc_t r =
                        tile_rsrc(a.out_agg, v0 * (VEC * 4), kBlock * U * VEC * 4);
                    const int o = (u * kBlock + tid) * (VEC * 4);
                    if (interior) {
#pragma unroll
                        for (int h = 0; h < VEC / 4; ++h) {
                            u32x4 q = {__float_as_uint(G[4 * h]), __float_as_uint(G[4 * h + 1]),
                                       __float_as_uint(G[4 * h + 2]), __float_as_uint(G[4 * h + 3])};
                            __builtin_amdgcn_raw_buffer_store_b128(q, r, o + 16 * h, 0, kStorePolicy);
                        }
                    } else {
#pragma unroll
                        for (int c = 0; c < VEC; ++c) {
                            const int64_t e = v * VEC + c;
                            const int oc = (e >= pc.e_lo && e < pc.e_hi) ? o + 4 * c : kMasked;
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(G[c]), r, oc, 0, 0);
                        }
                    }
                }

                // pass 2 over the same registers: squared norms and squared deviations
#pragma unroll
                for (int k = 0; k < K; ++k) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        uint32_t q = x[u][k][c];
                        if constexpr (DT == kF32) {
                            const float g = __uint_as_float(q);
                            n[k] = __builtin_fmaf(g, g, n[k]);
                            const float t = g - G[c];
                            d[k] = __builtin_fmaf(t, t, d[k]);
                        } else {
                            // keep the packed pair live and widen it again here: without this
                            // the compiler holds all 8K widened values and halves the occupancy
                            asm volatile("" : "+v"(q));
                            const float g0 = __uint_as_float(q << 16);
                            const float g1 = __uint_as_float(q & 0xffff0000u);
                            n[k] = __builtin_fmaf(g0, g0, n[k]);
                            n[k] = __builtin_fmaf(g1, g1, n[k]);
                            const float t0 = g0 - G[2 * c], t1 = g1 - G[2 * c + 1];
                            d[k] = __builtin_fmaf(t0, t0, d[k]);
                            d[k] = __builtin_fmaf(t1, t1, d[k]);
                        }
                    }
                }
            }
        }

        // block reduction: DPP inside each wave (fp32), then the four wave sums in fp64, fixed order
        const int lane = tid & 63, wave = tid >> 6;
        {
            const float r = wave_sum(A);
            if (lane == 0) wave_part[wave][0] = r;
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const float rn = wave_sum(n[k]);
            const float rd = wave_sum(d[k]);
            if (lane == 0) {
                wave_part[wave][1 + k] = rn;
                wave_part[wave][1 + K + k] = rd;
            }
        }
        __syncthreads();
        if (tid < W) {
            double s = 0.0;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) s += static_cast<double>(wave_part[wv][tid]);
            a.partials[static_cast<int64_t>(p) * W + tid] = s;
        }
        __syncthreads();
    }
}

// Switch over K for one dtype; instantiated in one translation unit per dtype and K range so
// that the build can compile them in parallel.
template <int DT, int K>
hipError_t launch_one(int grid, const StreamArgs& a, hipStream_t s)
{
    stream_pass_kernel<K, DT, unroll_for(K)><<<dim3(grid), dim3(kBlock), 0, s>>>(a);
    return hipGetLastError();
}

template <int DT, int K>
int occupancy_one()
{
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &nb, stream_pass_kernel<K, DT, unroll_for(K)>, kBlock, 0) != hipSuccess)
        return 0;
    return nb;
}

}  // namespace dynamix
