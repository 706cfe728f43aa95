// Streaming pass: one sweep over the K gradient buffers (Algorithm 1 of the paper: gradient
// synchronisation fused with the gradient part of metric collection).
//
// Per 16-byte vector a lane loads the K workers' values, forms the weighted aggregate
// G = sum_k w_k g_k in a fixed k order, and then, while the K values are still in registers,
// adds g^2 to the worker's squared norm, (g - G)^2 to its squared deviation and G^2 to the
// aggregate's squared norm.  Nothing is read twice and the only write is G, or, with a model
// update fused in (template parameter OPT), the parameters and the optimizer's state vectors,
// which then travel through the pass as further streams: read a tile ahead like the gradients,
// rewritten in place through the same staging as G.  The kernel is
// bound by HBM bandwidth (about one flop per byte), so there is no LDS tiling of the data and no
// MFMA: the work is coalesced 128-bit loads, fp32 FMAs and one block reduction per piece.
#pragma once
#include <type_traits>

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

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// The two 16-bit elements packed in a 32-bit word, widened to fp32 (exact for both formats).
// bf16 is the upper half of the fp32 encoding, so widening is a shift or a mask; fp16 goes
// through the hardware conversion, subnormals included.
template <int DT>
__device__ __forceinline__ float elem_lo(uint32_t q)
{
    if constexpr (DT == kBF16) return __uint_as_float(q << 16);
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(q & 0xffffu));
}
template <int DT>
__device__ __forceinline__ float elem_hi(uint32_t q)
{
    if constexpr (DT == kBF16) return __uint_as_float(q & 0xffff0000u);
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(q >> 16));
}

constexpr int kNT = 2;               // cache-policy bit "non-temporal": data is touched once
constexpr int kLoadPolicy = kNT;     // gradient loads of interior tiles
constexpr int kStorePolicy = kNT;    // aggregate stores of interior tiles

// One "vector" is what a lane loads at a time: LW 32-bit words (4 up to K = 32, then 2, then 1, so
// that the K vectors of a lane and the 2K+1 sums still fit the register file), i.e. LW fp32 or
// 2 LW bf16 or fp16 elements.
template <int LW>
struct Words;
template <>
struct Words<4> {
    typedef u32x4 type;
    template <int POL>
    static __device__ __forceinline__ type load(__amdgpu_buffer_rsrc_t r, int off)
    {
        return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, POL);
    }
    template <int POL>
    static __device__ __forceinline__ void store(type v, __amdgpu_buffer_rsrc_t r, int off)
    {
        __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, POL);
    }
};
template <>
struct Words<2> {
    typedef u32x2 type;
    template <int POL>
    static __device__ __forceinline__ type load(__amdgpu_buffer_rsrc_t r, int off)
    {
        return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, POL);
    }
    template <int POL>
    static __device__ __forceinline__ void store(type v, __amdgpu_buffer_rsrc_t r, int off)
    {
        __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, POL);
    }
};

typedef uint32_t u32x1 __attribute__((ext_vector_type(1)));
template <>
struct Words<1> {
    typedef u32x1 type;
    template <int POL>
    static __device__ __forceinline__ type load(__amdgpu_buffer_rsrc_t r, int off)
    {
        type v;
        v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, POL);
        return v;
    }
    template <int POL>
    static __device__ __forceinline__ void store(type v, __amdgpu_buffer_rsrc_t r, int off)
    {
        __builtin_amdgcn_raw_buffer_store_b32(v[0], r, off, 0, POL);
    }
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

constexpr int kMasked = 0x7ffffff0;  // a lane offset beyond every tile: the access is dropped

// The waves of a block leave every barrier in lockstep and then want the memory pipeline at the
// same moments.  Wave w therefore idles w * 1024 clocks (a microsecond or so) when a piece starts
// and after each flush.
__device__ __forceinline__ void stagger_waves(int tid)
{
    for (int i = 0; i < (tid >> 6); ++i) __builtin_amdgcn_s_sleep(16);
}

// Staging of the aggregate.  A store that enters a compute unit's memory pipeline while that unit
// has loads in flight holds the pipeline up for hundreds of cycles (measured: one 16-byte store
// per lane and tile costs a 32-stream read 27 % of its bandwidth, whatever the store's cache
// policy, issuing wave or size), and a byte written to HBM costs the read stream of the whole
// chip several bytes, the more the thinner the writes are spread in time (measured).  So
// finished tiles of G are kept on chip as long as there is room, and the whole block (the only
// one on its compute unit) writes them out in one burst between two barriers, when none of its
// loads is outstanding.  Room is 152 KB of LDS (what the 160 KB leave beside the wave partials)
// and, up to K = 44, the 256 accumulation registers of every lane: when the LDS is full for the
// first time in a flush cycle every lane moves its own slots into a first bank of registers,
// when it is full again (as far as the remaining registers reach) into a second, and after the
// third filling everything is written out.  With fp32 inputs a lane reads back only what it
// wrote, so the moves need no synchronisation (16-bit inputs: see kSwap in the kernel).
constexpr int kStageBytes = 152 * 1024;

// The banks live in the accumulation half of the register file, which nothing else in this
// kernel uses; the moves are written out so that the register allocator never has to weigh these
// values against the vector registers of the hot loop (left to itself it produced
// instantiations with corrupted sums on this target).
__device__ __forceinline__ uint32_t to_acc(uint32_t v)
{
    uint32_t a;
    asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a) : "v"(v));
    return a;
}
__device__ __forceinline__ uint32_t from_acc(uint32_t a)
{
    uint32_t v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}
// A store offset beyond every piece-wide descriptor (at most 2^30 bytes), also after the few
// bytes added for the second half of a vector.
constexpr int kMaskedStore = 0x7fff0000;

template <int K, int DT, int U, int OPT>
struct Shape {
    static constexpr int NO = out_streams(OPT);
    static constexpr int kLW = load_words_for(K, OPT);             // words per lane and load
    static constexpr int kVB = kLW * 4;                            // bytes per lane and load
    static constexpr int kVec = vec_elems(K, DT, OPT);             // elements per vector
    static constexpr int kSize = DT == kF32 ? 4 : 2;               // bytes per element
    static constexpr int kQ = kVec / kLW;                          // LW-word pieces of G per vector
    static constexpr int kSlots = kStageBytes / (kBlock * kVB);    // LW-word slots per thread
    static constexpr int kPerTile = U * kQ * NO;                   // slots a parked tile takes (NO streams)
    static constexpr int kTiles = kSlots / kPerTile;               // tiles the LDS holds
    // a second, smaller bank in what the first leaves of the 256 accumulation registers
    static constexpr int kTiles2 = (256 - kTiles * kPerTile * kLW) / (kPerTile * kLW);
    static_assert(kTiles >= 1, "a tile of G must fit the staging area");
};

template <int K, int DT, int U, int OPT>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void stream_pass_kernel(
    const StreamArgs a)
{
    constexpr int NO = out_streams(OPT);   // streams written (and, but for the plain aggregate, read first)
    typedef Shape<K, DT, U, OPT> Sh;
    typedef Words<Sh::kLW> Wd;
    typedef typename Wd::type wvec;
    constexpr int LW = Sh::kLW, VB = Sh::kVB, VEC = Sh::kVec, Q = Sh::kQ, NB = Sh::kTiles;
    constexpr int NB2 = Sh::kTiles2;
    constexpr int W = 2 * K + 1;
    constexpr int64_t TILE = (int64_t)kBlock * U;   // vectors per block iteration
    __shared__ wvec stage[NB * U * Q * NO][kBlock];
    __shared__ float wave_part[kWaves][W];

    const int tid = threadIdx.x;
    const int p_first = a.block_range[2 * blockIdx.x];
    const int p_last = a.block_range[2 * blockIdx.x + 1];
    // What is written per element: the aggregate G, or, with the fused model update, the new
    // parameter p - lr (G + wd p) over the old one; nothing in statistics-only calls.  The updates
    // with state (momentum, Adam) read and write the parameters and one or two state vectors.
    const bool fused = OPT != kOptNone || a.params != nullptr;
    float* const out = fused ? a.params : a.out_agg;
    const bool want_agg = OPT != kOptNone || out != nullptr;
    const float neg_lr = -a.lr, wd = a.wd;
    // stream s of the output (the same buffer is its input where there is one)
    auto out_ptr = [&](int s) -> float* { return s == 0 ? out : s == 1 ? a.state1 : a.state2; };
    // One element: the aggregate g and the old values in[] of the NO streams give the new ones.
    auto update = [&](float g, const float (&in)[NO], float (&o)[NO]) {
        if constexpr (OPT == kOptNone) {
            o[0] = fused ? __builtin_fmaf(neg_lr, __builtin_fmaf(wd, in[0], g), in[0]) : g;
        } else if constexpr (OPT == kOptMomentum) {
            // g' = G + wd p;  buf' = mu buf + g';  p' = p - lr (Nesterov: g' + mu buf', else buf')
            const float mu = a.hp[0];
            const float gp = __builtin_fmaf(wd, in[0], g);
            const float b = __builtin_fmaf(mu, in[1], gp);
            const float step = (a.flags & 1) ? __builtin_fmaf(mu, b, gp) : b;
            o[0] = __builtin_fmaf(neg_lr, step, in[0]);
            o[1] = b;
        } else {
            // Adam.  hp: beta1, 1 - beta1, beta2, 1 - beta2, 1 / sqrt(1 - beta2^t), eps,
            // lr / (1 - beta1^t), and the factor on p (1 - lr wd when the decay is decoupled, else
            // 1; wd is then zero in the gradient)
            const float gp = __builtin_fmaf(wd, in[0], g);
            const float m = __builtin_fmaf(a.hp[0], in[1], a.hp[1] * gp);
            const float v = __builtin_fmaf(a.hp[2], in[2], (a.hp[3] * gp) * gp);
            const float denom = __builtin_fmaf(__builtin_sqrtf(v), a.hp[4], a.hp[5]);
            o[0] = __builtin_fmaf(-a.hp[6], m / denom, in[0] * a.hp[7]);
            o[1] = m;
            o[2] = v;
        }
    };

    // The block's own pieces, then pieces of the shared tail for as long as there are any: one
    // lane draws the next index from the counter and hands it to the others through the LDS (the
    // barrier that ends every piece keeps the draw apart from the previous read).
    __shared__ int next_piece;
    const int n_tail = a.n_tail;
    bool drawn = false;
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
        float n[K], d[K], A = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k) n[k] = d[k] = 0.f;

        // pass 1 over the K vectors of one lane: the weighted aggregate, k ascending
        // With 31 or 32 fp32 workers the K weights and buffer addresses are read from the kernel
        // arguments again for every tile (scalar loads that hit the scalar cache, at an offset the
        // compiler cannot see through): kept in scalar registers for the whole loop they push so
        // many other scalars into spill lanes of vector registers that the loop runs out of those.
        constexpr bool kReloadWeights = K >= 31 && K <= 32 && DT == kF32 && OPT == kOptNone;
        auto pass1 = [&](const wvec (&xu)[K], float (&Gu)[VEC], const float* kw) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) Gu[c] = 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const float wk = kReloadWeights ? kw[k] : a.w[k];
#pragma unroll
                for (int c = 0; c < LW; ++c) {
                    const uint32_t q = xu[k][c];
                    if constexpr (DT == kF32) {
                        Gu[c] = __builtin_fmaf(wk, __uint_as_float(q), Gu[c]);
                    } else {
                        Gu[2 * c] = __builtin_fmaf(wk, elem_lo<DT>(q), Gu[2 * c]);
                        Gu[2 * c + 1] = __builtin_fmaf(wk, elem_hi<DT>(q), Gu[2 * c + 1]);
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < VEC; ++c) A = __builtin_fmaf(Gu[c], Gu[c], A);
        };
        // pass 2 for worker k: squared norm and squared deviation from the aggregate
        auto pass2 = [&](const wvec& xk, const float (&Gu)[VEC], int k) {
#pragma unroll
            for (int c = 0; c < LW; ++c) {
                uint32_t q = xk[c];
                // pins this read between the loads around it (and, for bf16, keeps the packed
                // pair live instead of all 8K widened values)
                asm volatile("" : "+v"(q));
                if constexpr (DT == kF32) {
                    const float g = __uint_as_float(q);
                    n[k] = __builtin_fmaf(g, g, n[k]);
                    const float t = g - Gu[c];
                    d[k] = __builtin_fmaf(t, t, d[k]);
                } else {
                    const float g0 = elem_lo<DT>(q), g1 = elem_hi<DT>(q);
                    if constexpr (DT == kBF16) {
                        // both squares of the packed pair in one instruction, fp32 accumulate
                        n[k] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q),
                                                               __builtin_bit_cast(bf16x2, q), n[k],
                                                               false);
                    } else {
                        n[k] = __builtin_fmaf(g0, g0, n[k]);
                        n[k] = __builtin_fmaf(g1, g1, n[k]);
                    }
                    const float t0 = g0 - Gu[2 * c], t1 = g1 - Gu[2 * c + 1];
                    d[k] = __builtin_fmaf(t0, t0, d[k]);
                    d[k] = __builtin_fmaf(t1, t1, d[k]);
                }
            }
        };
        // A boundary vector: the one vector at the head or tail of a piece that also holds
        // elements outside [lo, hi) (a segment edge at any element offset, or the ragged end of
        // the gradient).  Lane 0 of wave 0 handles it with element-wise loads and stores whose
        // offset is pushed out of the descriptor's range for masked elements, which then read as
        // zero and are not written.  At most two per piece, so it favours few registers over
        // speed: the vector is read twice (once per pass), eight workers at a time.
        auto boundary_vector = [&](int64_t v, int64_t lo, int64_t hi) {
            constexpr int CH = 8;   // workers whose loads are in flight together
            // The two flags are derived again here, from pointers the compiler cannot trace back:
            // otherwise it keeps them in a register across the hot loop, which has none to spare.
            float* out_b = out;
            const float* params_b = a.params;
            asm volatile("" : "+s"(out_b), "+s"(params_b));
            const bool want_b = out_b != nullptr, fused_b = params_b != nullptr;
            int off[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const int64_t e = v * VEC + c;
                off[c] = (tid == 0 && e >= lo && e < hi) ? c * Sh::kSize : kMasked;
            }
            auto load_worker = [&](int k) {
                const __amdgpu_buffer_rsrc_t r = tile_rsrc(a.g[k], v * VB, VB);
                wvec xe;
#pragma unroll
                for (int c = 0; c < LW; ++c) {
                    if constexpr (DT == kF32) {
                        xe[c] = __builtin_amdgcn_raw_buffer_load_b32(r, off[c], 0, 0);
                    } else {
                        const uint32_t l16 = __builtin_amdgcn_raw_buffer_load_b16(r, off[2 * c], 0, 0);
                        const uint32_t h16 =
                            __builtin_amdgcn_raw_buffer_load_b16(r, off[2 * c + 1], 0, 0);
                        xe[c] = (l16 & 0xffffu) | (h16 << 16);
                    }
                }
                return xe;
            };
            float Ge[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) Ge[c] = 0.f;
#pragma unroll
            for (int k0 = 0; k0 < K; k0 += CH) {
                // start this batch only when the one before has been consumed
                asm volatile("" : "+v"(off[0]) : "v"(Ge[0]));
                wvec xe[CH];
#pragma unroll
                for (int j = 0; j < CH; ++j)
                    if (k0 + j < K) xe[j] = load_worker(k0 + j);
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    if (k0 + j >= K) continue;
                    const float wk = a.w[k0 + j];
#pragma unroll
                    for (int c = 0; c < LW; ++c) {
                        const uint32_t q = xe[j][c];
                        if constexpr (DT == kF32) {
                            Ge[c] = __builtin_fmaf(wk, __uint_as_float(q), Ge[c]);
                        } else {
                            Ge[2 * c] = __builtin_fmaf(wk, elem_lo<DT>(q), Ge[2 * c]);
                            Ge[2 * c + 1] = __builtin_fmaf(wk, elem_hi<DT>(q), Ge[2 * c + 1]);
                        }
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < VEC; ++c) A = __builtin_fmaf(Ge[c], Ge[c], A);
            if (want_b) {
                __amdgpu_buffer_rsrc_t r[NO];
                r[0] = tile_rsrc(out_b, v * (VEC * 4), VEC * 4);
                if constexpr (NO > 1) r[1] = tile_rsrc(a.state1, v * (VEC * 4), VEC * 4);
                if constexpr (NO > 2) r[2] = tile_rsrc(a.state2, v * (VEC * 4), VEC * 4);
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    const int oc = off[c] == kMasked ? kMasked : c * 4;
                    if constexpr (OPT == kOptNone) {
                        float res = Ge[c];
                        if (fused_b) {
                            const float pc_old =
                                __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r[0], oc, 0, 0));
                            res = __builtin_fmaf(neg_lr, __builtin_fmaf(wd, pc_old, Ge[c]), pc_old);
                        }
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(res), r[0], oc, 0, 0);
                    } else {
                        float in[NO], o[NO];
#pragma unroll
                        for (int s = 0; s < NO; ++s)
                            in[s] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r[s], oc, 0, 0));
                        update(Ge[c], in, o);
#pragma unroll
                        for (int s = 0; s < NO; ++s)
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[s]), r[s], oc, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int k0 = 0; k0 < K; k0 += CH) {
                if (k0 > 0) asm volatile("" : "+v"(off[0]) : "v"(n[k0 - 1]), "v"(d[k0 - 1]));
                wvec xe[CH];
#pragma unroll
                for (int j = 0; j < CH; ++j)
                    if (k0 + j < K) xe[j] = load_worker(k0 + j);
#pragma unroll
                for (int j = 0; j < CH; ++j)
                    if (k0 + j < K) pass2(xe[j], Ge, k0 + j);
            }
        };

        // The piece is: an optional boundary vector at its head, a body of whole vectors
        // [body_begin, body_end), an optional boundary vector at its tail.
        int64_t body_begin = pc.v_begin, body_end = pc.v_end;
        const bool head_cut = pc.e_lo > pc.v_begin * VEC;
        const bool tail_cut = pc.e_hi < pc.v_end * VEC;
        if (head_cut) ++body_begin;
        if (tail_cut && pc.v_end - 1 >= body_begin) --body_end;
        if (tid < 64) {   // wave 0 only
            if (head_cut)
                boundary_vector(pc.v_begin, pc.e_lo, min(pc.e_hi, (pc.v_begin + 1) * VEC));
            if (tail_cut && pc.v_end - 1 >= body_begin)
                boundary_vector(pc.v_end - 1, (pc.v_end - 1) * VEC, pc.e_hi);
        }

        if (body_begin < body_end) {
            // ---- the body: the hot loop.  A tile is kBlock * U vectors; the last one may be
            // shorter, in which case its descriptors are shorter and the lanes beyond read zero
            // and write nothing.
            //
            // Which vectors make up a tile.  The K buffers of a caller often sit at the same
            // offsets of equally aligned allocations; the same elements of all workers then fall
            // into the same memory channels, and with tiles of 4 KB consecutive bytes per worker
            // the K loads of a lane queue up behind each other (8 % of the bandwidth at K = 32
            // with buffers a multiple of 16 MB apart, measured).
            // So, with 16-byte vectors, the body is taken in groups of 16 tiles, and tile i of a
            // group takes from each of the group's 16 U units of 4 KB one chunk of 256 bytes
            // (chunk (i + unit) mod 16): every load instruction of a wave then touches four
            // units instead of a quarter of one.  What is left after the last whole group is
            // taken in consecutive tiles.  The aggregate is written in the same chunks, which
            // costs more than it gains where the write is a large part of the traffic: below
            // eight workers the tiles stay consecutive (measured: 2 to 4 % slower otherwise).
            constexpr bool kSpread = interleaves(K, OPT);
            // The chunks only pay when they are whole cache lines, so the groups start at a
            // multiple of 256 vectors (the caller says whether the buffers themselves are aligned;
            // a.spread is zero otherwise, and everything is taken in consecutive tiles); the
            // vectors in front of that are taken as one short tile of their own.
            const int64_t body_vectors = body_end - body_begin;
            const bool spread = kSpread && a.spread != 0;
            const int pre = spread ? (int)min((int64_t)((-body_begin) & 255), body_vectors) : 0;
            const int has_pre = pre > 0 ? 1 : 0;
            const int64_t groups_begin = body_begin + pre;
            constexpr int GS = kSpread ? 4 : 0;           // log2 of the tiles per group
            constexpr int GROUP = (int)TILE << GS;        // vectors per group
            // (tile counts fit 32 bits: a tile is at least 1024 elements)
            const int body_tiles = has_pre + (int)((body_end - groups_begin + TILE - 1) / TILE);
            const int full_groups = spread ? (int)((body_end - groups_begin) / GROUP) : 0;
            struct Where {
                int64_t v;    // first vector of the tile's group: where its descriptors start
                int count;    // vectors they cover, to the end of the group or of the body
            };
            auto where = [&](int t) -> Where {
                if (t >= body_tiles) return {body_end, 0};
                if (t < has_pre) return {body_begin, pre};
                const int64_t v = groups_begin + (int64_t)((t - has_pre) >> GS) * GROUP;
                return {v, (int)min((int64_t)GROUP, body_end - v)};
            };
            // the vector, counted from where(t).v, that this lane handles as its u-th of tile t
            auto lane_vec_of = [&](int lane, int t, int u) -> int {
                const int tq = t - has_pre;   // -1 for the short tile in front
                if (kSpread && tq >= 0 && (tq >> GS) < full_groups) {
                    const int i = tq & ((1 << GS) - 1);
                    const int unit = lane >> 4;
                    return ((((u * 16 + unit) << GS) + ((i + unit) & ((1 << GS) - 1))) << 4) + (lane & 15);
                }
                const int i = tq < 0 ? 0 : tq & ((1 << GS) - 1);
                return (i * U + u) * kBlock + lane;
            };
            auto lane_vec = [&](int t, int u) -> int { return lane_vec_of(tid, t, u); };
            int t = 0;   // tile of the body being processed
            const bool long_run = body_vectors > 8 * TILE;   // staggering pays only then
            if (long_run) stagger_waves(tid);
            // The K vectors of every lane.  A tile is always loaded one iteration ahead: by
            // pass 2 of the tile before it, or here for the first one.
            wvec x[U][K];
            // the old values of the NO output streams for the tile: the parameters (fused updates
            // only; else never read, through a descriptor of length zero) and the optimizer state
            wvec xs[NO][U][Q];
            auto load_streams = [&](const Where& w, int tw) {
#pragma unroll
                for (int s = 0; s < NO; ++s) {
                    const __amdgpu_buffer_rsrc_t rp = tile_rsrc(
                        s == 0 ? a.params : out_ptr(s), w.v * (VEC * 4), fused ? w.count * (VEC * 4) : 0);
#pragma unroll
                    for (int u = 0; u < U; ++u)
#pragma unroll
                        for (int h = 0; h < Q; ++h)
                            xs[s][u][h] = Wd::template load<kLoadPolicy>(
                                rp, lane_vec(tw, u) * (VEC * 4) + VB * h);
                }
            };
            {
                const Where w0 = where(0);
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int k = 0; k < K; ++k)
                        x[u][k] = Wd::template load<kLoadPolicy>(
                            tile_rsrc(a.g[k], w0.v * VB, w0.count * VB), lane_vec(0, u) * VB);
                load_streams(w0, 0);
            }
            int staged = 0;            // tiles parked in LDS
            int t_staged = 0;          // first of them
            // When to flush.  A flush is short (10 us for 400 KB), but what the chip loses to the
            // writes depends on how they are spread in time: blocks that flush whenever their own
            // staging is full drift apart (their first flushes already lie 75 us apart, the fifth
            // 200 us) and the memory sees a steady trickle of writes among the reads; all blocks
            // flushing within a few microseconds of each other costs a quarter less (C4: 2.70 ->
            // 2.64 ms).  So the blocks flush at common instants, the multiples of kFlushPeriod on
            // the device-wide clock, with whatever they have parked by then (and, as before, when
            // the staging is full or the piece ends).  The four waves of a block have to agree on
            // the tile after which they flush without meeting: wave 0 reads the clock once per
            // tile and, when an instant has passed, announces in the LDS "flush after tile t + 2";
            // it also publishes its progress, and no other wave passes the flush point of a tile
            // before wave 0 has decided about it, i.e. has been through the tile two before it.
            // Wave 0 never waits for the others except in barriers that they reach without
            // waiting for it, so nobody waits for ever.
            constexpr int kStagedMax = K <= 44 ? 2 * NB + NB2 : NB;
            // the period: four fifths of the time a block takes to fill its staging at full speed
            // (a tile at 26.5 GB/s per compute unit), in ticks of the 100 MHz clock
            constexpr uint32_t kFlushPeriod = (uint32_t)(
                0.8 * kStagedMax *
                ((double)(kBlock * U) * (K * VB + (OPT == kOptNone ? 1 : 2 * NO) * VEC * 4) / 265.0));
            constexpr int kNever = 0x7fffffff;
            __shared__ int wave0_progress, flush_after;
            // (only where a piece fills the staging several times: one that fits it once is
            // better off with its single flush at the end)
            const bool timed = want_agg && body_vectors >= 2 * kStagedMax * TILE;
            int announced = kNever;        // wave 0: the tile it has announced a flush after
            uint32_t next_instant = 0;     // wave 0: clock value of the next common instant
            if (timed) {
                if (tid == 0) {
                    wave0_progress = 0;
                    flush_after = kNever;
                }
                const uint32_t now = (uint32_t)wall_clock64();
                next_instant = now - now % kFlushPeriod + kFlushPeriod;
                __syncthreads();
            }
            // the register banks (accumulation registers): NB and NB2 more tiles, parked before
            // those in the LDS
            uint32_t bank[NB * U * Q * NO * LW];
            uint32_t bank2[(NB2 > 0 ? NB2 : 1) * U * Q * NO * LW];
            int t_bank = 0, t_bank2 = 0;   // first tile of each bank
            bool more = true;
            // 16-bit inputs: a vector of G is twice the width of a store, and a lane that wrote
            // its own two halves would leave every store instruction with gaps of its own width
            // between the lanes.  The h-th store of a lane therefore takes one half of another
            // lane's vector, so that the 256 lanes of an instruction write 256 consecutive
            // pieces: lane l stores half (l mod 2) of the vector that lane 128 h + l / 2 parked.
            // The data change lanes in the LDS, between the barriers of the flush or, for the
            // register banks, when the banks are filled (with barriers of their own).
            constexpr bool kSwap = Q == 2;
            auto src_lane = [&](int lane, int h) -> int {
                return kSwap ? h * (kBlock / 2) + (lane >> 1) : lane;
            };
            auto src_half = [&](int lane, int h) -> int { return kSwap ? (lane & 1) : h; };
            // One tile.  With the bank the loop over tiles exists twice (two instantiations of this
            // body): once for the first half of a flush cycle, while the bank is empty, and once
            // for the second half, during which the bank is only kept, never redefined, so that
            // it costs the loop no register copies.
            auto tile_body = [&](auto mode) {
                // 0: both banks empty; 1: first bank full; 2: both full; 3: kernel without banks
                constexpr int kMode = decltype(mode)::value;
                // Software pipeline without extra registers: as pass 2 finishes with a worker's
                // vector, the same registers take that worker's vector of the next tile, so
                // loads are issued all through the arithmetic.  After the last tile the
                // descriptor gets zero length and the loads touch no memory.
                const int tn = t + 1;
                const Where wn = where(tn);
                more = wn.count > 0;
                uint32_t hidden_zero = 0;
                if constexpr (kReloadWeights) asm volatile("" : "+s"(hidden_zero));
                const float* const kw = a.w + hidden_zero;
                const void* const* const kg = a.g + hidden_zero;   // (likewise the K addresses)

                float G[U][VEC];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    pass1(x[u], G[u], kw);
                    if (want_agg) {
                        // park what will be written (fp32 inputs: every thread later reads back
                        // only what it wrote itself; 16-bit inputs: see kSwap)
#pragma unroll
                        for (int h = 0; h < Q; ++h) {
                            wvec q[NO];
#pragma unroll
                            for (int c = 0; c < LW; ++c) {
                                float in[NO], o[NO];
#pragma unroll
                                for (int s = 0; s < NO; ++s) in[s] = __uint_as_float(xs[s][u][h][c]);
                                update(G[u][LW * h + c], in, o);
#pragma unroll
                                for (int s = 0; s < NO; ++s) q[s][c] = __float_as_uint(o[s]);
                            }
#pragma unroll
                            for (int s = 0; s < NO; ++s)
                                stage[((staged * U + u) * NO + s) * Q + h][tid] = q[s];
                        }
                    }
                }

                // Flush point: pass 1 has consumed every load of this tile and pass 2 has not
                // yet issued any for the next one, so once all waves are here the block has no
                // load in flight.  The parked tiles are written out and the stores waited for.
                if (want_agg) {
                    if (staged == 0) t_staged = t;
                    ++staged;
                    bool on_time = false;
                    if (timed) {
                        if (__builtin_amdgcn_readfirstlane(tid) < 64) {   // wave 0
                            if (announced == kNever) {
                                const uint32_t now = (uint32_t)wall_clock64();
                                if ((int32_t)(now - next_instant) >= 0) {
                                    announced = t + 2;
                                    if (tid == 0)
                                        __hip_atomic_store(&flush_after, announced, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                                }
                            }
                            // (released after the announcement: who sees the progress sees it too)
                            if (tid == 0)
                                __hip_atomic_store(&wave0_progress, t + 1, __ATOMIC_RELEASE,
                                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                            on_time = t == announced;
                        } else {
                            while (__hip_atomic_load(&wave0_progress, __ATOMIC_ACQUIRE,
                                                     __HIP_MEMORY_SCOPE_WORKGROUP) < t - 1)
                                __builtin_amdgcn_s_sleep(1);
                            on_time = __hip_atomic_load(&flush_after, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_WORKGROUP) == t;
                        }
                        on_time = __builtin_amdgcn_readfirstlane((int)on_time) != 0;
                    }
                    if (kMode <= 1 ? (!more || on_time) : (staged == NB || !more || on_time)) {
                        __syncthreads();
                        // the store addresses are worked out here, from a copy of the lane number
                        // the compiler cannot see through: otherwise it prepares them ahead of
                        // the loop and keeps them in registers the loop needs
                        int lane_f = tid;
                        asm volatile("" : "+v"(lane_f));
                        // one descriptor over the whole body for the stores (a piece has at most
                        // 2^18 vectors, so byte offsets inside it fit the 32-bit lane offset)
                        __amdgpu_buffer_rsrc_t r[NO];
#pragma unroll
                        for (int s = 0; s < NO; ++s)
                            r[s] = tile_rsrc(out_ptr(s), body_begin * (VEC * 4),
                                             (int)(body_vectors * (VEC * 4)));
                        // where this lane's h-th store of a tile goes (see kSwap)
                        auto out_off = [&](int tj, int u, int h) -> int {
                            const int tq = tj - has_pre;
                            const int lv = lane_vec_of(src_lane(lane_f, h), tj, u);
                            const int in_vec = VB * src_half(lane_f, h);
                            // (the short tile in front ends inside the piece, where this
                            // descriptor does not: its idle lanes are masked here)
                            if (tq < 0) return lv < pre ? lv * (VEC * 4) + in_vec : kMaskedStore;
                            return (pre + (tq >> GS) * GROUP + lv) * (VEC * 4) + in_vec;
                        };
                        if constexpr (kMode == 1 || kMode == 2) {
#pragma unroll
                            for (int j = 0; j < NB; ++j) {
                                const int tj = t_bank + j;
#pragma unroll
                                for (int u = 0; u < U; ++u)
#pragma unroll
                                    for (int h = 0; h < Q; ++h)
#pragma unroll
                                        for (int s = 0; s < NO; ++s) {
                                            wvec t;
#pragma unroll
                                            for (int c = 0; c < LW; ++c)
                                                t[c] = from_acc(
                                                    bank[((((j * U + u) * NO + s) * Q) + h) * LW + c]);
                                            Wd::template store<kStorePolicy>(t, r[s], out_off(tj, u, h));
                                        }
                            }
                        }
                        if constexpr (kMode == 2) {
#pragma unroll
                            for (int j = 0; j < NB2; ++j) {
                                const int tj = t_bank2 + j;
#pragma unroll
                                for (int u = 0; u < U; ++u)
#pragma unroll
                                    for (int h = 0; h < Q; ++h)
#pragma unroll
                                        for (int s = 0; s < NO; ++s) {
                                            wvec t;
#pragma unroll
                                            for (int c = 0; c < LW; ++c)
                                                t[c] = from_acc(
                                                    bank2[((((j * U + u) * NO + s) * Q) + h) * LW + c]);
                                            Wd::template store<kStorePolicy>(t, r[s], out_off(tj, u, h));
                                        }
                            }
                        }
                        for (int j = 0; j < staged; ++j) {
                            const int tj = t_staged + j;
#pragma unroll
                            for (int u = 0; u < U; ++u)
#pragma unroll
                                for (int h = 0; h < Q; ++h)
#pragma unroll
                                    for (int s = 0; s < NO; ++s)
                                        Wd::template store<kStorePolicy>(
                                            stage[((j * U + u) * NO + s) * Q + src_half(tid, h)]
                                                 [src_lane(tid, h)],
                                            r[s], out_off(tj, u, h));
                        }
                        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                        __syncthreads();
                        staged = 0;
                        if (on_time) {
                            announced = kNever;
                            const uint32_t now = (uint32_t)wall_clock64();
                            next_instant = now - now % kFlushPeriod + kFlushPeriod;
                        }
                        if (long_run) stagger_waves(tid);
                    }
                }

                const int next_bytes = wn.count * VB;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int next_vec = lane_vec(tn, u);
#pragma unroll
                    for (int k = 0; k < K; ++k) {
                        pass2(x[u][k], G[u], k);
                        // order the load after the last use of the registers it overwrites (the
                        // empty asm ties its address to this worker's updated sums), or the
                        // scheduler hoists all K loads and the live ranges double
                        int pf_off = next_vec * VB;
                        asm volatile("" : "+v"(pf_off) : "v"(n[k]), "v"(d[k]));
                        x[u][k] = Wd::template load<kLoadPolicy>(
                            tile_rsrc(kReloadWeights ? kg[k] : a.g[k], wn.v * VB, next_bytes), pf_off);
                    }
                }
                load_streams(wn, tn);
                t = tn;
            };
            // The banks are used up to K = 44.  Above, the loop itself needs all 256 vector
            // registers, the compiler would start to move values into accumulation registers on
            // its own, and some instantiations built that way gave wrong sums.
            constexpr bool kBank = K <= 44;
            while (!kBank && more) tile_body(std::integral_constant<int, 3>{});
            while (kBank && more) {
                // until the LDS is full (or the run ends, which flushes)
                do {
                    tile_body(std::integral_constant<int, 0>{});
                } while (more && staged != 0 && staged < NB);
                if (!more) break;
                if (staged == 0) continue;   // flushed on time, before the LDS was full: start again
                // every lane moves the slots it will store into the first bank, and the LDS fills
                // again
                if (kSwap) __syncthreads();
#pragma unroll
                for (int j = 0; j < NB * U * NO; ++j)   // (tile, vector, stream) in parking order
#pragma unroll
                    for (int h = 0; h < Q; ++h) {
                        const wvec t = stage[j * Q + src_half(tid, h)][src_lane(tid, h)];
#pragma unroll
                        for (int c = 0; c < LW; ++c) bank[(j * Q + h) * LW + c] = to_acc(t[c]);
                    }
                if (kSwap) {
                    __syncthreads();
                    if (long_run) stagger_waves(tid);
                }
                t_bank = t_staged;
                staged = 0;
                if constexpr (NB2 > 0) {
                    do {
                        tile_body(std::integral_constant<int, 1>{});
                    } while (more && staged != 0 && staged < NB2);
                    if (!more) break;
                    if (staged == 0) continue;
                    // the second, smaller bank
                    if (kSwap) __syncthreads();
#pragma unroll
                    for (int j = 0; j < NB2 * U * NO; ++j)
#pragma unroll
                        for (int h = 0; h < Q; ++h) {
                            const wvec t = stage[j * Q + src_half(tid, h)][src_lane(tid, h)];
#pragma unroll
                            for (int c = 0; c < LW; ++c) bank2[(j * Q + h) * LW + c] = to_acc(t[c]);
                        }
                    if (kSwap) {
                        __syncthreads();
                        if (long_run) stagger_waves(tid);
                    }
                    t_bank2 = t_staged;
                    staged = 0;
                }
                // until the flush of banks and LDS (which resets staged)
                do {
                    tile_body(std::integral_constant<int, 2>{});
                } while (staged != 0);
            }
        }

        // block reduction: DPP inside each wave (fp32), then the wave sums in fp64, fixed order
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
        // (the lane number is hidden from the compiler here so that the address of the store is
        // worked out now and not kept in registers from the start of the kernel)
        int tid_e = tid;
        asm volatile("" : "+v"(tid_e));
        if (tid_e < W) {
            double s = 0.0;
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) s += static_cast<double>(wave_part[wv][tid_e]);
            a.partials[static_cast<int64_t>(p) * W + tid_e] = s;
        }
        __syncthreads();
    }
}

// Switch over K for one dtype; instantiated in one translation unit per dtype and K range so
// that the build can compile them in parallel.
template <int DT, int K, int OPT>
hipError_t launch_one(int grid, const StreamArgs& a, hipStream_t s)
{
    stream_pass_kernel<K, DT, unroll_for(K, OPT), OPT><<<dim3(grid), dim3(kBlock), 0, s>>>(a);
    return hipGetLastError();
}

template <int DT, int K, int OPT>
int occupancy_one()
{
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &nb, stream_pass_kernel<K, DT, unroll_for(K, OPT), OPT>, kBlock, 0) != hipSuccess)
        return 0;
    return nb;
}

}  // namespace dynamix
