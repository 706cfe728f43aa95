// Measurement aid: plain streaming kernels with the access pattern of the streaming pass and no
// arithmetic to speak of, to measure what the memory system of the device gives a kernel of this
// shape: reading N streams and writing nothing, writing one stream and reading nothing, copying,
// and (two launches on two streams, on disjoint sets of compute units) reading while another
// kernel writes.  The streaming pass is judged against these figures; nothing in the product path
// calls this file.
#include "../../include/dynamix.h"
#include "dynamix_internal.h"

namespace dynamix {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeBlock = 256;
constexpr int kNT = 2;   // cache-policy bit "non-temporal"
// Every probe kernel reserves more than half of a compute unit's LDS, so that no two blocks, of
// the same or of different probe kernels, share a compute unit: a reading and a writing kernel
// launched together on n and 256 - n blocks then run on disjoint units.
constexpr int kReserveLds = 96 * 1024;

struct ProbeArgs {
    const char* src[32];
    char* dst;
    int64_t vectors;   // 16-byte vectors per buffer
    int32_t spread;    // 0: consecutive 4 KB tiles; L = 8, 16, 32: chunks of L vectors, see below
    float* sink;       // never written: keeps the loads alive
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* base, int64_t off, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(base)) + off,
                                             0, bytes, 0x00020000);
}

// Block b owns the contiguous span of tiles [b * per, (b + 1) * per) of every stream; a tile is
// 256 vectors (4 KB) per stream.  With spread = L, G = 256 / L tiles form a group and load i of a
// group takes, from each of the group's G units of 4 KB, the chunk of L vectors number
// (i + unit) mod G: L = 16 (256-byte chunks of sixteen units) is what the streaming pass does.
template <int NS>
__global__ __launch_bounds__(kProbeBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void probe_read_kernel(
    const ProbeArgs a)
{
    __shared__ char reserve[kReserveLds];
    const int tid = threadIdx.x;
    const int64_t tiles = a.vectors / kProbeBlock;          // whole tiles only
    const int L = a.spread ? a.spread : 16;      // vectors per chunk
    const int G = kProbeBlock / L;               // tiles per group = units per group = chunks per unit
    const int64_t per = (tiles + gridDim.x - 1) / gridDim.x / G * G + G;   // whole groups
    const int64_t t0 = (int64_t)blockIdx.x * per;
    const int64_t t1 = t0 + per < tiles ? t0 + per : tiles;
    float acc = 0.f;
    const int unit = tid / L;
    for (int64_t t = t0; t < t1; ++t) {
        u32x4 x[NS];
        const int64_t group = t / G * G;
        const bool whole = group + G <= t1;
        const int i = (int)(t - group);
        const int group_tiles = (int)(tiles - group < G ? tiles - group : G);   // inside the buffer
        const int lane_vec = a.spread && whole ? (unit * G + (i + unit) % G) * L + tid % L
                                               : i * kProbeBlock + tid;
#pragma unroll
        for (int k = 0; k < NS; ++k)
            x[k] = __builtin_amdgcn_raw_buffer_load_b128(
                rsrc(a.src[k], group * kProbeBlock * 16, group_tiles * kProbeBlock * 16),
                lane_vec * 16, 0, kNT);
#pragma unroll
        for (int k = 0; k < NS; ++k)
            acc += __uint_as_float(x[k][0]) + __uint_as_float(x[k][1]) + __uint_as_float(x[k][2]) +
                   __uint_as_float(x[k][3]);
    }
    if (acc == 123.456f) {
        reserve[tid] = 1;
        a.sink[0] = acc + reserve[(tid + 1) & 255];
    }
}

// Writes `vectors` vectors to dst: 4 KB per store instruction of a block, contiguous span per block.
__global__ __launch_bounds__(kProbeBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void probe_write_kernel(
    const ProbeArgs a)
{
    __shared__ char reserve[kReserveLds];
    const int tid = threadIdx.x;
    const int64_t tiles = a.vectors / kProbeBlock;
    const int64_t per = (tiles + gridDim.x - 1) / gridDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * per;
    const int64_t t1 = t0 + per < tiles ? t0 + per : tiles;
    u32x4 v = {(uint32_t)tid, 1u, 2u, 3u};
    for (int64_t t = t0; t < t1; ++t) {
        v[1] = (uint32_t)t;
        __builtin_amdgcn_raw_buffer_store_b128(v, rsrc(a.dst, t * kProbeBlock * 16, kProbeBlock * 16),
                                               tid * 16, 0, kNT);
    }
    if (a.vectors < 0) {   // never: keeps the LDS reservation
        reserve[tid] = 1;
        __syncthreads();
        a.dst[tid] = reserve[(tid + 1) & 255];
    }
}

// dst := src[0], eight loads in flight per lane.
__global__ __launch_bounds__(kProbeBlock) __attribute__((amdgpu_waves_per_eu(1, 1))) void probe_copy_kernel(
    const ProbeArgs a)
{
    __shared__ char reserve[kReserveLds];
    constexpr int UN = 8;
    const int tid = threadIdx.x;
    const int64_t tiles = a.vectors / (kProbeBlock * UN);
    const int64_t per = (tiles + gridDim.x - 1) / gridDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * per;
    const int64_t t1 = t0 + per < tiles ? t0 + per : tiles;
    for (int64_t t = t0; t < t1; ++t) {
        u32x4 x[UN];
        const int64_t off = t * kProbeBlock * UN * 16;
#pragma unroll
        for (int u = 0; u < UN; ++u)
            x[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc(a.src[0], off, kProbeBlock * UN * 16),
                                                         (u * kProbeBlock + tid) * 16, 0, kNT);
#pragma unroll
        for (int u = 0; u < UN; ++u)
            __builtin_amdgcn_raw_buffer_store_b128(x[u], rsrc(a.dst, off, kProbeBlock * UN * 16),
                                                   (u * kProbeBlock + tid) * 16, 0, kNT);
    }
    if (a.vectors < 0) {   // never: keeps the LDS reservation
        reserve[tid] = 1;
        __syncthreads();
        a.dst[tid] = reserve[(tid + 1) & 255];
    }
}

}  // namespace
}  // namespace dynamix

extern "C" int dynamix_hbm_probe(const void* const* buffers, int32_t count, int64_t bytes, int32_t mode,
                                 int32_t blocks, void* stream)
{
    using namespace dynamix;
    if (!buffers) return DYNAMIX_ERR_NULL;
    if (count < 1 || count > 32 || bytes < 4096 || blocks < 1 || blocks > 65536) return DYNAMIX_ERR_ARG;
    for (int k = 0; k < count; ++k) {
        if (!buffers[k]) return DYNAMIX_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(buffers[k]) & 255u) return DYNAMIX_ERR_ALIGN;
    }
    ProbeArgs a;
    a.vectors = bytes / 16;
    a.dst = nullptr;
    a.sink = nullptr;
    a.spread = 0;
    for (int k = 0; k < 32; ++k) a.src[k] = static_cast<const char*>(buffers[k < count ? k : 0]);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(blocks), block(kProbeBlock);
    switch (mode) {
    case DYNAMIX_PROBE_READ:
    case DYNAMIX_PROBE_READ_SPREAD:
    case DYNAMIX_PROBE_READ_SPREAD_128B:
    case DYNAMIX_PROBE_READ_SPREAD_512B:
        a.spread = mode == DYNAMIX_PROBE_READ ? 0 : mode == DYNAMIX_PROBE_READ_SPREAD ? 16
                 : mode == DYNAMIX_PROBE_READ_SPREAD_128B ? 8 : 32;
        a.sink = static_cast<float*>(const_cast<void*>(buffers[0]));   // (never written)
        switch (count) {
        case 1: probe_read_kernel<1><<<grid, block, 0, s>>>(a); break;
        case 2: probe_read_kernel<2><<<grid, block, 0, s>>>(a); break;
        case 4: probe_read_kernel<4><<<grid, block, 0, s>>>(a); break;
        case 8: probe_read_kernel<8><<<grid, block, 0, s>>>(a); break;
        case 16: probe_read_kernel<16><<<grid, block, 0, s>>>(a); break;
        case 32: probe_read_kernel<32><<<grid, block, 0, s>>>(a); break;
        default: return DYNAMIX_ERR_ARG;
        }
        break;
    case DYNAMIX_PROBE_WRITE:
        if (count != 1) return DYNAMIX_ERR_ARG;
        a.dst = static_cast<char*>(const_cast<void*>(buffers[0]));
        probe_write_kernel<<<grid, block, 0, s>>>(a);
        break;
    case DYNAMIX_PROBE_COPY:
        if (count != 2) return DYNAMIX_ERR_ARG;
        a.dst = static_cast<char*>(const_cast<void*>(buffers[1]));
        probe_copy_kernel<<<grid, block, 0, s>>>(a);
        break;
    default:
        return DYNAMIX_ERR_ARG;
    }
    return hipGetLastError() == hipSuccess ? DYNAMIX_OK : DYNAMIX_ERR_HIP;
}
