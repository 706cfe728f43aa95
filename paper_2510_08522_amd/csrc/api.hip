// C ABI of libdynamix: argument validation, the cached launch plan and the two launches.
// Everything before "plan" runs without touching HIP, so a bad call costs nothing on the device.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <vector>

#include "../../include/dynamix.h"
#include "dynamix_internal.h"

// Device memory of dynamix_grad_aggregate_stats_static, the entry point that allocates nothing:
// plan tables, tail counter and partial sums of the call in flight.  Every GPU the library runs on
// holds its own copy at its own address until the process ends; host code reaches it only through
// the per-device address that hipGetSymbolAddress returns (static_scratch_of below), never
// through this name.
static __device__ __align__(256) unsigned char scratch[DYNAMIX_STATIC_SCRATCH_BYTES];

namespace dynamix {

#define DYNAMIX_UNIT_ENTRY(OPT, DT, LO) \
    {launch_stream_pass_##OPT##_##DT##_##LO, occupancy_stream_pass_##OPT##_##DT##_##LO},
struct Unit {
    hipError_t (*launch)(int, int, const StreamArgs&, hipStream_t);
    int (*occupancy)(int);
};
// [update kind][dtype][(K - 1) / 8]; the updates with state exist up to kKMaxOpt workers
static const Unit kUnits[kOpts][kDtypes][kKMax / 8] = {
    {{DYNAMIX_FOR_EACH_PLAIN_UNIT(DYNAMIX_UNIT_ENTRY, 0)},
     {DYNAMIX_FOR_EACH_PLAIN_UNIT(DYNAMIX_UNIT_ENTRY, 1)},
     {DYNAMIX_FOR_EACH_PLAIN_UNIT(DYNAMIX_UNIT_ENTRY, 2)}},
    {{DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_UNIT_ENTRY, 1, 0)},
     {DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_UNIT_ENTRY, 1, 1)},
     {DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_UNIT_ENTRY, 1, 2)}},
    {{DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_UNIT_ENTRY, 2, 0)},
     {DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_UNIT_ENTRY, 2, 1)},
     {DYNAMIX_FOR_EACH_STATE_UNIT(DYNAMIX_UNIT_ENTRY, 2, 2)}}};

static const Unit* unit_for(int K, int dtype, int opt)
{
    if (K < 1 || K > kKMax || dtype < 0 || dtype >= kDtypes || opt < 0 || opt >= kOpts) return nullptr;
    if (opt != kOptNone && K > kKMaxOpt) return nullptr;
    const Unit* u = &kUnits[opt][dtype][(K - 1) / 8];
    return u->launch ? u : nullptr;
}

hipError_t launch_stream_pass(int K, int dtype, int opt, int grid, const StreamArgs& a, hipStream_t s)
{
    if (K > kKMax && opt == kOptNone) return launch_wide_pass(K, dtype, grid, a, s);
    const Unit* u = unit_for(K, dtype, opt);
    return u ? u->launch(K, grid, a, s) : hipErrorInvalidValue;
}

int stream_pass_blocks_per_cu(int K, int dtype, int opt)
{
    if (K > kKMax && K <= kKWide && opt == kOptNone) return wide_pass_blocks_per_cu(dtype);
    const Unit* u = unit_for(K, dtype, opt);
    return u ? u->occupancy(K) : 0;
}

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// The launch plan of one (device, stream, K, dtype, P, segments): how the vector range is dealt
// to blocks and cut at segment boundaries, plus the device workspace for the partial sums.
struct Plan {
    int device = 0;
    hipStream_t stream = nullptr;
    int K = 0, dtype = 0, opt = 0;
    int64_t P = 0;
    std::vector<int64_t> offsets;  // empty without segments
    int grid = 0, pieces = 0, n_tail = 0, records = 0, slices = 1;
    bool uploaded = false;
    std::vector<char> host;        // staging image of the tables
    size_t table_bytes = 0;
    size_t total_bytes = 0;        // tables and partial sums
    size_t o_block = 0, o_tail = 0, o_range = 0, o_count = 0, o_queue = 0, o_part = 0, o_slices = 0;
    bool owns_blob = true;         // false: the blob is the library's static scratch array
    char* blob = nullptr;          // device: tables followed by the partial sums
    const Piece* d_pieces = nullptr;
    const int32_t* d_block_range = nullptr;
    const int32_t* d_tail_order = nullptr;
    const int32_t* d_rec_range = nullptr;
    const double* d_rec_count = nullptr;
    double* d_partials = nullptr;
    int32_t* d_queue = nullptr;    // tail pieces drawn so far in the running launch; zero between launches
    double* d_slice_sums = nullptr;
    uint64_t last_use = 0;
    ~Plan()
    {
        if (blob && owns_blob) (void)hipFree(blob);
    }
};

std::mutex g_mutex;
std::vector<std::unique_ptr<Plan>> g_plans;
uint64_t g_clock = 0;
constexpr size_t kMaxPlans = 128;
constexpr double kPieceCostBytes = 128.0 * 1024.0;  // streaming time that one more piece costs a block

// Optional kernel timing: event triples (before the streaming pass, between the two kernels,
// after the final reduction) recorded on the call's stream, one triple per call.
struct Timing {
    std::vector<hipEvent_t> events;  // 3 per slot
    int capacity = 0;
    int used = 0;
    int every = 1;       // only every n-th call is timed (events cost the stream a few microseconds)
    int64_t calls = 0;   // calls seen since timing began
};
Timing g_timing;

int env_int(const char* name, int fallback)
{
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : fallback;
}

// The work decomposition (pure host arithmetic, no HIP): pieces, the pieces of every block, the
// order of the shared tail, and per record its piece range and element count.

// Longest piece, a multiple of every tile size.  Two reasons: the kernel addresses the aggregate
// of a piece with 32-bit byte offsets (2^25 vectors would still do), and a lane adds the squares of
// a piece in fp32 before they reach the fp64 partial sums, with an error that grows with their
// number (measured with fp16 inputs: 2e-5 relative after 121 000 elements per lane, 7e-6 after
// 32 000, 3e-7 after 500); 2^18 vectors are at most 8 192 elements per lane.
constexpr int64_t kMaxPieceVectors = (int64_t)1 << 18;
constexpr int kTailPermille = 30;           // share of the range that goes to the shared tail
constexpr int kMaxSlices = 16;              // blocks of the final reduction that share record 0
constexpr int kPiecesPerSlice = 96;         // ... one per that many pieces, from kMinSlicedPieces on
constexpr int kMinSlicedPieces = 512;
constexpr int kTailMinTiles = 2;            // tiles in its last (shortest) pieces
constexpr int kTailMinTilesPerBlock = 64;   // shorter inputs get no tail

struct Layout {
    int grid = 0;
    std::vector<Piece> pieces;        // in ascending order of position
    std::vector<int32_t> block_range; // [grid][2]: first and one-past-last piece of every block
    std::vector<int32_t> tail_order;  // pieces of the shared tail in the order they are drawn
    std::vector<int32_t> rec_range;
    std::vector<double> rec_count;
};

void make_layout(int K, int dtype, int opt, int64_t P, int S, const int64_t* offsets, int64_t max_grid,
                 Layout& L)
{
    const int VEC = vec_elems(K, dtype, opt);
    const int64_t tile = (int64_t)kBlock * unroll_for(K, opt);  // vectors per block iteration
    const int64_t nvec = ceil_div(P, VEC);
    // Spans start at multiples of a wave's worth of vectors (1 KB of every stream), so that the
    // 64 lanes of a wave stay on whole cache lines; a block's last tile may be partial.  Kernels
    // that interleave chunks of 4 KB units start their groups at multiples of 256 vectors, so
    // their spans start there (otherwise every block would begin with a short tile).
    const int64_t gran = interleaves(K, opt) ? 256 : 64;
    if (max_grid < 1) max_grid = 1;
    L.grid = (int)std::min<int64_t>(std::min(max_grid, ceil_div(nvec, gran)),
                                    std::max<int64_t>(1, nvec / 512));

    const int64_t ngran = ceil_div(nvec, gran);

    // Every block owns one contiguous span.  A span costs its length plus a fixed amount per
    // piece (pipeline start, boundary vectors, final flush, block reduction: about what
    // 128 KB of streaming takes), and the spans are cut so that the costs are equal; without
    // segments the lengths of two spans differ by at most one granule.  A block is started
    // for every 512 vectors at least, up to max_grid.
    std::vector<int64_t> span_begin(L.grid + 1, 0);                    // first vector of every span
    {
        const double gran_bytes = (double)gran * VEC * (dtype == kF32 ? 4 : 2) * K;
        const double piece_cost = kPieceCostBytes / gran_bytes;           // in granules
        std::vector<int64_t> cuts;                                         // vectors where a new piece starts
        for (int j = 1; j < S; ++j) cuts.push_back(offsets[j] / VEC);
        const double total_cost = (double)ngran + piece_cost * (double)cuts.size();
        size_t c = 0;        // cuts already behind the walk
        int64_t t = 0;       // granules already dealt
        for (int b = 1; b < L.grid; ++b) {
            const double want = total_cost * b / L.grid;
            // advance granule by granule over the cuts, in one jump between them
            while (t < ngran) {
                const double here = (double)t + piece_cost * (double)c;
                if (here >= want) break;
                const int64_t next_cut = c < cuts.size() ? cuts[c] / gran : ngran;
                if (next_cut > t) {
                    const int64_t need = (int64_t)std::ceil(want - here);
                    t = std::min<int64_t>(std::min(next_cut, t + std::max<int64_t>(need, 1)), ngran);
                } else {
                    ++c;     // the cut lies in the granule the walk stands on
                }
            }
            // every block keeps at least one granule and leaves one for each block after it
            t = std::max<int64_t>(t, span_begin[b - 1] / gran + 1);
            t = std::min<int64_t>(t, ngran - (L.grid - b));
            span_begin[b] = t * gran;
            while (c < cuts.size() && cuts[c] / gran < t) ++c;
        }
        span_begin[L.grid] = nvec;
    }

    // The shared tail.  Compute units do not stream equally fast (on MI355X the blocks of a
    // 2.7 ms launch finish over a range of 160 us, the units of every other XCD about 1 % later
    // than the rest), so with equal spans the launch ends with a few blocks running alone.  The
    // block of a long span therefore only owns its front; the last few percent are cut into short
    // pieces, each half of what is left and the last ones kTailMinTiles tiles, that any block
    // draws from a counter once its own part is done: first the longest piece of every span, then
    // the second of every span, and so on.  (They are taken from every span, not from the end of
    // the whole range: blocks that all work within a few megabytes of each other stream a third
    // slower per tile, measured.)  Environment, tuning aids read when a plan is built:
    // DYNAMIX_TAIL_PERMILLE, the share of a span; DYNAMIX_TAIL_MIN, the shortest piece.
    struct Sub {
        int64_t begin;   // first vector
        int owner;       // block, or -1 - round for a piece of the tail
    };
    std::vector<Sub> subs;
    {
        const int permille_env = env_int("DYNAMIX_TAIL_PERMILLE", -1);
        const int64_t permille = permille_env >= 0 ? std::min(permille_env, 500) : kTailPermille;
        const int64_t shortest = std::max(1, env_int("DYNAMIX_TAIL_MIN", kTailMinTiles));
        const int64_t min_tiles = permille_env >= 0 ? 4 : kTailMinTilesPerBlock;
        for (int b = 0; b < L.grid; ++b) {
            subs.push_back({span_begin[b], b});
            const int64_t tiles = (span_begin[b + 1] - span_begin[b]) / tile;
            int64_t rest = tiles >= min_tiles ? tiles * permille / 1000 : 0;
            if (rest < shortest) continue;
            int64_t v = span_begin[b] + (tiles - rest) * tile;
            for (int round = 0; rest > 0; ++round) {
                const int64_t size = std::max(shortest, rest / 2);
                const int64_t take = rest < size + shortest ? rest : size;   // no shorter rest
                subs.push_back({v, -1 - round});
                v += take * tile;    // (the last one also takes what the span has beyond whole tiles)
                rest -= take;
            }
        }
    }
    {
        const int nsubs = (int)subs.size();
        std::vector<int64_t> sub_begin(nsubs + 1);
        for (int i = 0; i < nsubs; ++i) sub_begin[i] = subs[i].begin;
        sub_begin[nsubs] = nvec;
        L.block_range.assign(2 * (size_t)L.grid, 0);
        std::vector<std::pair<int, int32_t>> tail;   // (round, piece)
        const int nseg = S > 0 ? S : 1;
        for (int j = 0; j < nseg; ++j) {
            const int64_t lo = S > 0 ? offsets[j] : 0, hi = S > 0 ? offsets[j + 1] : P;
            const int64_t v_lo = lo / VEC, v_hi = ceil_div(hi, VEC);
            // parts of spans that meet [v_lo, v_hi)
            int b = (int)(std::upper_bound(sub_begin.begin(), sub_begin.end(), v_lo) -
                          sub_begin.begin()) - 1;
            for (; b < nsubs && sub_begin[b] < v_hi; ++b) {
                // (no piece longer than kMaxPieceVectors)
                const int64_t p_begin = std::max(v_lo, sub_begin[b]);
                const int64_t p_end = std::min(v_hi, sub_begin[b + 1]);
                for (int64_t v = p_begin; v < p_end; v += kMaxPieceVectors) {
                    Piece pc;
                    pc.v_begin = v;
                    pc.v_end = std::min(p_end, v + kMaxPieceVectors);
                    pc.v_step = tile;
                    pc.e_lo = std::max(lo, pc.v_begin * VEC);
                    pc.e_hi = std::min(hi, pc.v_end * VEC);
                    pc.block = subs[b].owner;
                    const int32_t index = (int32_t)L.pieces.size();
                    L.pieces.push_back(pc);
                    if (subs[b].owner >= 0) {
                        // (segments ascend and so do the parts: a block's pieces are consecutive)
                        int32_t* r = &L.block_range[2 * (size_t)subs[b].owner];
                        if (r[1] == 0) r[0] = index;
                        r[1] = index + 1;
                    } else {
                        tail.push_back({-1 - subs[b].owner, index});
                    }
                }
            }
        }
        std::stable_sort(tail.begin(), tail.end(),
                         [](const auto& x, const auto& y) { return x.first < y.first; });
        for (const auto& t : tail) L.tail_order.push_back(t.second);
    }

    // record 0 folds every piece; record 1 + j the pieces of segment j (consecutive by construction)
    L.rec_range.push_back(0);
    L.rec_range.push_back((int32_t)L.pieces.size());
    L.rec_count.push_back((double)P);
    int32_t first = 0;
    size_t i = 0;
    for (int j = 0; j < S; ++j) {
        while (i < L.pieces.size() && L.pieces[i].e_lo < offsets[j + 1]) ++i;
        L.rec_range.push_back(first);
        L.rec_range.push_back((int32_t)i);
        L.rec_count.push_back((double)(offsets[j + 1] - offsets[j]));
        first = (int32_t)i;
    }
}

// The tables of a plan and where each lies in the device blob (host arithmetic plus two device
// queries; no device memory is touched).
int layout_plan(Plan& pl, int S, const int64_t* offsets)
{
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, pl.device) != hipSuccess) return DYNAMIX_ERR_HIP;
    const int per_cu = stream_pass_blocks_per_cu(pl.K, pl.dtype, pl.opt);
    if (per_cu <= 0) return DYNAMIX_ERR_HIP;

    Layout L;
    int64_t max_grid = (int64_t)prop.multiProcessorCount * per_cu;
    const int cap = env_int("DYNAMIX_MAX_BLOCKS", 0);   // tuning aid: another number of blocks
    if (cap > 0) max_grid = cap;
    make_layout(pl.K, pl.dtype, pl.opt, pl.P, S, offsets, max_grid, L);
    pl.grid = L.grid;
    pl.pieces = (int)L.pieces.size();
    pl.n_tail = (int)L.tail_order.size();
    pl.records = 1 + S;

    const int W = 2 * pl.K + 1;
    pl.o_block = align_up(L.pieces.size() * sizeof(Piece), 256);
    pl.o_tail = align_up(pl.o_block + L.block_range.size() * sizeof(int32_t), 256);
    pl.o_range = align_up(pl.o_tail + L.tail_order.size() * sizeof(int32_t), 256);
    pl.o_count = align_up(pl.o_range + L.rec_range.size() * sizeof(int32_t), 256);
    pl.o_queue = align_up(pl.o_count + L.rec_count.size() * sizeof(double), 256);
    pl.o_part = align_up(pl.o_queue + sizeof(int32_t), 256);
    // the final reduction shares record 0 among several blocks when it has many pieces
    pl.slices = pl.pieces >= kMinSlicedPieces ? std::min(kMaxSlices, pl.pieces / kPiecesPerSlice) : 1;
    pl.o_slices = align_up(pl.o_part + (size_t)pl.pieces * W * sizeof(double), 256);
    pl.total_bytes = pl.o_slices + (size_t)pl.slices * W * sizeof(double);
    pl.table_bytes = pl.o_part;
    pl.host.assign(pl.o_part, 0);   // (the tail counter at o_queue starts at zero)
    std::memcpy(pl.host.data(), L.pieces.data(), L.pieces.size() * sizeof(Piece));
    std::memcpy(pl.host.data() + pl.o_block, L.block_range.data(), L.block_range.size() * sizeof(int32_t));
    if (!L.tail_order.empty())
        std::memcpy(pl.host.data() + pl.o_tail, L.tail_order.data(), L.tail_order.size() * sizeof(int32_t));
    std::memcpy(pl.host.data() + pl.o_range, L.rec_range.data(), L.rec_range.size() * sizeof(int32_t));
    std::memcpy(pl.host.data() + pl.o_count, L.rec_count.data(), L.rec_count.size() * sizeof(double));
    return DYNAMIX_OK;
}

// Points the plan at its device memory: total_bytes at `blob`.
void bind_plan(Plan& pl, char* blob, bool owns)
{
    pl.blob = blob;
    pl.owns_blob = owns;
    pl.d_pieces = reinterpret_cast<const Piece*>(blob);
    pl.d_block_range = reinterpret_cast<const int32_t*>(blob + pl.o_block);
    pl.d_tail_order = reinterpret_cast<const int32_t*>(blob + pl.o_tail);
    pl.d_rec_range = reinterpret_cast<const int32_t*>(blob + pl.o_range);
    pl.d_rec_count = reinterpret_cast<const double*>(blob + pl.o_count);
    pl.d_queue = reinterpret_cast<int32_t*>(blob + pl.o_queue);   // zero in the uploaded image
    pl.d_partials = reinterpret_cast<double*>(blob + pl.o_part);
    pl.d_slice_sums = reinterpret_cast<double*>(blob + pl.o_slices);
}

int build_plan(Plan& pl, int S, const int64_t* offsets)
{
    const int rc = layout_plan(pl, S, offsets);
    if (rc != DYNAMIX_OK) return rc;
    void* dev = nullptr;
    if (hipMalloc(&dev, pl.total_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return DYNAMIX_ERR_NOMEM;
    }
    bind_plan(pl, static_cast<char*>(dev), true);
    return DYNAMIX_OK;
}

bool same_shape(const Plan& pl, int K, int dtype, int opt, int64_t P, int S, const int64_t* offsets)
{
    return pl.K == K && pl.dtype == dtype && pl.opt == opt && pl.P == P &&
           (int)pl.offsets.size() == (S > 0 ? S + 1 : 0) &&
           (S == 0 || std::memcmp(pl.offsets.data(), offsets, sizeof(int64_t) * (S + 1)) == 0);
}

// Finds or builds the plan; the caller holds g_mutex.
int get_plan(int device, hipStream_t stream, int K, int dtype, int opt, int64_t P, int S,
             const int64_t* offsets, Plan** out)
{
    for (auto& up : g_plans) {
        Plan& pl = *up;
        if (pl.device == device && pl.stream == stream &&
            same_shape(pl, K, dtype, opt, P, S, offsets)) {
            pl.last_use = ++g_clock;
            *out = &pl;
            return DYNAMIX_OK;
        }
    }
    if (g_plans.size() >= kMaxPlans) {
        // drop the least recently used plan; hipFree waits for work that may still read it
        auto it = std::min_element(g_plans.begin(), g_plans.end(),
                                   [](const auto& x, const auto& y) { return x->last_use < y->last_use; });
        g_plans.erase(it);
    }
    auto up = std::make_unique<Plan>();
    up->device = device;
    up->stream = stream;
    up->K = K;
    up->dtype = dtype;
    up->opt = opt;
    up->P = P;
    if (S > 0) up->offsets.assign(offsets, offsets + S + 1);
    const int rc = build_plan(*up, S, offsets);
    if (rc != DYNAMIX_OK) return rc;
    up->last_use = ++g_clock;
    *out = up.get();
    g_plans.push_back(std::move(up));
    return DYNAMIX_OK;
}

// ---- the entry point that allocates nothing (for callers that cannot call hipMalloc)
//
// Its plan lives in the static scratch array instead of a hipMalloc'ed blob, one plan per device:
// the tables of the last shape stay resident, another shape overwrites them.  The tables reach
// the device in the arguments of a small kernel, 3.5 KB per launch on the caller's stream (an
// asynchronous copy from pageable host memory would go through staging buffers that the runtime
// allocates).
constexpr int kPokeWords = 896;
struct PokeArgs {
    uint32_t words[kPokeWords];
};
__global__ __launch_bounds__(kPokeWords) void poke_kernel(uint32_t* dst, int n, const PokeArgs a)
{
    const int i = threadIdx.x;
    if (i < n) dst[i] = a.words[i];
}

constexpr int kMaxDevices = 64;
struct StaticDevice {
    char* ptr = nullptr;            // this device's copy of the scratch array
    std::unique_ptr<Plan> plan;     // the shape whose tables are resident (host side: layout only)
    // A call recorded into a graph uploads its tables whenever the graph is replayed, behind the
    // host's back: once that has happened on a device, no call can trust what is resident any
    // more, and every call uploads its own tables.
    bool recorded_into_a_graph = false;
};
StaticDevice g_static[kMaxDevices];

// The address of the current device's scratch array, looked up once per device.
int static_scratch_of(int device, char** out)
{
    if (device < 0 || device >= kMaxDevices) return DYNAMIX_ERR_ARG;
    StaticDevice& sd = g_static[device];
    if (!sd.ptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return DYNAMIX_ERR_HIP;
        }
        sd.ptr = static_cast<char*>(p);
    }
    *out = sd.ptr;
    return DYNAMIX_OK;
}

// Finds or lays out the plan of the static path; the caller holds g_mutex.
int get_static_plan(int device, hipStream_t stream, int K, int dtype, int64_t P, int S,
                    const int64_t* offsets, Plan** out)
{
    char* ptr = nullptr;
    const int rc = static_scratch_of(device, &ptr);
    if (rc != DYNAMIX_OK) return rc;
    StaticDevice& sd = g_static[device];
    if (!sd.plan || !same_shape(*sd.plan, K, dtype, kOptNone, P, S, offsets)) {
        auto up = std::make_unique<Plan>();
        up->device = device;
        up->K = K;
        up->dtype = dtype;
        up->P = P;
        if (S > 0) up->offsets.assign(offsets, offsets + S + 1);
        const int lrc = layout_plan(*up, S, offsets);
        if (lrc != DYNAMIX_OK) return lrc;
        if (up->total_bytes > (size_t)DYNAMIX_STATIC_SCRATCH_BYTES) return DYNAMIX_ERR_CAPACITY;
        bind_plan(*up, ptr, /*owns=*/false);
        sd.plan = std::move(up);    // (the tables of the shape before are overwritten below)
    }
    sd.plan->stream = stream;
    *out = sd.plan.get();
    return DYNAMIX_OK;
}

// Writes the plan's tables (with a zero tail counter) to its device memory with kernels on
// `stream` (the static path, and any call that is being recorded into a graph).
int upload_by_kernels(const Plan& pl, hipStream_t stream)
{
    PokeArgs pa;
    for (size_t off = 0; off < pl.table_bytes; off += sizeof pa.words) {
        const size_t nbytes = std::min(sizeof pa.words, pl.table_bytes - off);   // multiples of 256
        std::memcpy(pa.words, pl.host.data() + off, nbytes);
        poke_kernel<<<dim3(1), dim3(kPokeWords), 0, stream>>>(
            reinterpret_cast<uint32_t*>(pl.blob + off), (int)(nbytes / 4), pa);
    }
    return hipGetLastError() == hipSuccess ? DYNAMIX_OK : DYNAMIX_ERR_HIP;
}

int check_shape(int32_t K, int64_t P, int32_t dtype, const int64_t* offsets, int64_t S)
{
    if (K < 1 || K > kKWide || P < 1 || dtype < DYNAMIX_F32 || dtype > DYNAMIX_F16)
        return DYNAMIX_ERR_ARG;
    if (S < 0 || S > INT32_MAX / 4) return DYNAMIX_ERR_SEGMENTS;
    if ((S == 0) != (offsets == nullptr)) return DYNAMIX_ERR_SEGMENTS;
    if (S > 0) {
        if (offsets[0] != 0 || offsets[S] != P) return DYNAMIX_ERR_SEGMENTS;
        for (int64_t j = 0; j < S; ++j)
            if (offsets[j + 1] <= offsets[j]) return DYNAMIX_ERR_SEGMENTS;
    }
    return DYNAMIX_OK;
}

// The model update fused into the pass, if any: which kind, the buffers it reads and writes in
// place, and its constants as the kernel takes them.
struct Update {
    int opt = kOptNone;
    float* params = nullptr;   // also the plain SGD step of kOptNone
    float* state1 = nullptr;
    float* state2 = nullptr;
    float lr = 0.f, wd = 0.f;
    float hp[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int32_t flags = 0;
};

int run(const void* const* grads, const int32_t* batch_sizes, int32_t K, int64_t P, int32_t dtype,
        const int64_t* offsets, int64_t S, float* out_agg, double* out_stats, void* stream_v,
        const Update& up = Update(), bool use_static = false)
{
    float* const params = up.params;
    // ---- validation: no HIP call before this block has passed
    if (!grads || !batch_sizes || !out_stats) return DYNAMIX_ERR_NULL;
    int vrc = check_shape(K, P, dtype, offsets, S);
    if (vrc != DYNAMIX_OK) return vrc;
    for (int k = 0; k < K; ++k) {
        if (!grads[k]) return DYNAMIX_ERR_NULL;
        if (batch_sizes[k] <= 0) return DYNAMIX_ERR_ARG;
    }
    for (int k = 0; k < K; ++k)
        if (reinterpret_cast<uintptr_t>(grads[k]) & 15u) return DYNAMIX_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(out_agg) & 15u) || (reinterpret_cast<uintptr_t>(out_stats) & 7u) ||
        (reinterpret_cast<uintptr_t>(params) & 15u) || (reinterpret_cast<uintptr_t>(up.state1) & 15u) ||
        (reinterpret_cast<uintptr_t>(up.state2) & 15u))
        return DYNAMIX_ERR_ALIGN;
    if (up.opt != kOptNone && K > kKMaxOpt) return DYNAMIX_ERR_ARG;
    if (params && K > kKMax) return DYNAMIX_ERR_ARG;   // the two-sweep kernel has no fused update

    // ---- weights: B in 64-bit integers, w_k = b_k / B rounded once to fp32
    int64_t B = 0;
    for (int k = 0; k < K; ++k) B += batch_sizes[k];

    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return DYNAMIX_ERR_HIP;

    std::lock_guard<std::mutex> lock(g_mutex);
    Plan* pl = nullptr;
    const int rc = use_static ? get_static_plan(device, stream, K, dtype, P, (int)S, offsets, &pl)
                              : get_plan(device, stream, K, dtype, up.opt, P, (int)S, offsets, &pl);
    if (rc != DYNAMIX_OK) return rc;
    // A call that is being recorded into a graph executes nothing now: it must carry the upload
    // of its tables with it (as kernels: a copy from pageable host memory is no graph material),
    // and it may not change what the host believes to be on the device.
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (stream != nullptr && hipStreamIsCapturing(stream, &capture) != hipSuccess) {
        (void)hipGetLastError();
        capture = hipStreamCaptureStatusNone;
    }
    const bool recording = capture != hipStreamCaptureStatusNone;
    const bool was_uploaded = pl->uploaded;
    if (use_static && recording) g_static[device].recorded_into_a_graph = true;
    if (!pl->uploaded || recording || (use_static && g_static[device].recorded_into_a_graph)) {
        if (use_static || recording) {
            if (upload_by_kernels(*pl, stream) != DYNAMIX_OK) return DYNAMIX_ERR_HIP;
        } else if (hipMemcpyAsync(pl->blob, pl->host.data(), pl->table_bytes,
                                  hipMemcpyHostToDevice, stream) != hipSuccess) {
            return DYNAMIX_ERR_HIP;
        }
        pl->uploaded = true;
    }

    StreamArgs sa;
    std::memset(&sa, 0, sizeof sa);
    FinalArgs fa;
    std::memset(&fa, 0, sizeof fa);
    for (int k = 0; k < K; ++k) {
        sa.g[k] = grads[k];
        sa.w[k] = (float)((double)batch_sizes[k] / (double)B);
        fa.b[k] = (double)batch_sizes[k];
    }
    sa.pieces = pl->d_pieces;
    sa.block_range = pl->d_block_range;
    sa.tail_order = pl->d_tail_order;
    sa.out_agg = out_agg;
    sa.partials = pl->d_partials;
    sa.queue = pl->d_queue;
    sa.n_tail = pl->n_tail;
    sa.params = params;
    sa.lr = up.lr;
    sa.wd = up.wd;
    sa.state1 = up.state1;
    sa.state2 = up.state2;
    std::memcpy(sa.hp, up.hp, sizeof sa.hp);
    sa.flags = up.flags;
    {
        // The interleaved tile order reads and writes 256-byte chunks: it is used when every
        // buffer starts on such a boundary (DYNAMIX_SPREAD=0 turns it off, a tuning aid).
        uintptr_t low = reinterpret_cast<uintptr_t>(out_agg) | reinterpret_cast<uintptr_t>(params) |
                        reinterpret_cast<uintptr_t>(up.state1) | reinterpret_cast<uintptr_t>(up.state2);
        for (int k = 0; k < K; ++k) low |= reinterpret_cast<uintptr_t>(grads[k]);
        sa.spread = (low & 255u) == 0 && env_int("DYNAMIX_SPREAD", 1) != 0;
    }
    fa.B = (double)B;
    fa.partials = pl->d_partials;
    fa.rec_range = pl->d_rec_range;
    fa.rec_count = pl->d_rec_count;
    fa.out_stats = out_stats;
    fa.queue = pl->d_queue;
    fa.slice_sums = pl->d_slice_sums;
    fa.slices = pl->slices;
    fa.K = K;

    hipEvent_t* ev = nullptr;
    if (g_timing.used < g_timing.capacity && g_timing.calls++ % g_timing.every == 0)
        ev = &g_timing.events[3 * (size_t)g_timing.used++];
    if (ev && hipEventRecord(ev[0], stream) != hipSuccess) return DYNAMIX_ERR_HIP;
    if (launch_stream_pass(K, dtype, up.opt, pl->grid, sa, stream) != hipSuccess) return DYNAMIX_ERR_HIP;
    // From here on the tail counter is in use; only the final reduction sets it back.  Should
    // that not get enqueued, the tables (with a zero counter) are uploaded again next time.
    pl->uploaded = false;
    if (ev && hipEventRecord(ev[1], stream) != hipSuccess) return DYNAMIX_ERR_HIP;
    if (launch_final_reduce(pl->records, fa, stream) != hipSuccess) return DYNAMIX_ERR_HIP;
    pl->uploaded = recording ? was_uploaded : true;
    if (ev && hipEventRecord(ev[2], stream) != hipSuccess) return DYNAMIX_ERR_HIP;
    return DYNAMIX_OK;
}

}  // namespace
}  // namespace dynamix

extern "C" {

int dynamix_grad_aggregate_stats_ex(const void* const* grads, const int32_t* batch_sizes,
                                    int32_t K, int64_t P, int32_t dtype,
                                    const int64_t* segment_offsets, int64_t num_segments,
                                    float* out_agg, double* out_stats, void* stream)
{
    try {
        return dynamix::run(grads, batch_sizes, K, P, dtype, segment_offsets, num_segments, out_agg,
                            out_stats, stream);
    } catch (const std::bad_alloc&) {
        return DYNAMIX_ERR_NOMEM;
    } catch (...) {
        return DYNAMIX_ERR_HIP;
    }
}

int dynamix_grad_aggregate_stats_static(const void* const* grads, const int32_t* batch_sizes,
                                        int32_t K, int64_t P, int32_t dtype,
                                        const int64_t* segment_offsets, int64_t num_segments,
                                        float* out_agg, double* out_stats, void* stream)
{
    try {
        return dynamix::run(grads, batch_sizes, K, P, dtype, segment_offsets, num_segments, out_agg,
                            out_stats, stream, dynamix::Update(), /*use_static=*/true);
    } catch (const std::bad_alloc&) {
        return DYNAMIX_ERR_NOMEM;
    } catch (...) {
        return DYNAMIX_ERR_HIP;
    }
}

int dynamix_grad_aggregate_stats_sgd(const void* const* grads, const int32_t* batch_sizes,
                                     int32_t K, int64_t P, int32_t dtype,
                                     const int64_t* segment_offsets, int64_t num_segments,
                                     float* params, float lr, float weight_decay,
                                     double* out_stats, void* stream)
{
    if (!params) return DYNAMIX_ERR_NULL;
    if (!(lr == lr) || !(weight_decay == weight_decay)) return DYNAMIX_ERR_ARG;   // NaN
    try {
        dynamix::Update up;
        up.params = params;
        up.lr = lr;
        up.wd = weight_decay;
        return dynamix::run(grads, batch_sizes, K, P, dtype, segment_offsets, num_segments, nullptr,
                            out_stats, stream, up);
    } catch (const std::bad_alloc&) {
        return DYNAMIX_ERR_NOMEM;
    } catch (...) {
        return DYNAMIX_ERR_HIP;
    }
}

int dynamix_grad_aggregate_stats_sgd_momentum(const void* const* grads, const int32_t* batch_sizes,
                                              int32_t K, int64_t P, int32_t dtype,
                                              const int64_t* segment_offsets, int64_t num_segments,
                                              float* params, float* momentum_buf, float lr,
                                              float weight_decay, float momentum, int32_t nesterov,
                                              double* out_stats, void* stream)
{
    if (!params || !momentum_buf) return DYNAMIX_ERR_NULL;
    if (!(lr == lr) || !(weight_decay == weight_decay) || !(momentum == momentum))
        return DYNAMIX_ERR_ARG;   // NaN
    try {
        dynamix::Update up;
        up.opt = dynamix::kOptMomentum;
        up.params = params;
        up.state1 = momentum_buf;
        up.lr = lr;
        up.wd = weight_decay;
        up.hp[0] = momentum;
        up.flags = nesterov ? 1 : 0;
        return dynamix::run(grads, batch_sizes, K, P, dtype, segment_offsets, num_segments, nullptr,
                            out_stats, stream, up);
    } catch (const std::bad_alloc&) {
        return DYNAMIX_ERR_NOMEM;
    } catch (...) {
        return DYNAMIX_ERR_HIP;
    }
}

int dynamix_grad_aggregate_stats_adam(const void* const* grads, const int32_t* batch_sizes, int32_t K,
                                      int64_t P, int32_t dtype, const int64_t* segment_offsets,
                                      int64_t num_segments, float* params, float* exp_avg,
                                      float* exp_avg_sq, float lr, float beta1, float beta2, float eps,
                                      float weight_decay, int32_t decoupled, int64_t step,
                                      double* out_stats, void* stream)
{
    if (!params || !exp_avg || !exp_avg_sq) return DYNAMIX_ERR_NULL;
    if (!(lr == lr) || !(weight_decay == weight_decay) || !(eps == eps) || step < 1 ||
        !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
        return DYNAMIX_ERR_ARG;
    try {
        // the constants of the step, worked out once in double and rounded to fp32
        const double c1 = 1.0 - std::pow((double)beta1, (double)step);
        const double c2 = 1.0 - std::pow((double)beta2, (double)step);
        dynamix::Update up;
        up.opt = dynamix::kOptAdam;
        up.params = params;
        up.state1 = exp_avg;
        up.state2 = exp_avg_sq;
        up.lr = lr;
        up.wd = decoupled ? 0.f : weight_decay;
        up.hp[0] = beta1;
        up.hp[1] = (float)(1.0 - (double)beta1);
        up.hp[2] = beta2;
        up.hp[3] = (float)(1.0 - (double)beta2);
        up.hp[4] = (float)(1.0 / std::sqrt(c2));
        up.hp[5] = eps;
        up.hp[6] = (float)((double)lr / c1);
        up.hp[7] = decoupled ? (float)(1.0 - (double)lr * (double)weight_decay) : 1.f;
        return dynamix::run(grads, batch_sizes, K, P, dtype, segment_offsets, num_segments, nullptr,
                            out_stats, stream, up);
    } catch (const std::bad_alloc&) {
        return DYNAMIX_ERR_NOMEM;
    } catch (...) {
        return DYNAMIX_ERR_HIP;
    }
}

int dynamix_grad_aggregate_stats(const void* const* grads, const int32_t* batch_sizes, int32_t K,
                                 int64_t P, int32_t dtype, const int64_t* segment_offsets,
                                 float* out_agg, double* out_stats, void* stream)
{
    int64_t S = 0;
    if (segment_offsets) {
        // the array ends at the first entry equal to P; entries must rise strictly towards it
        if (P < 1) return DYNAMIX_ERR_ARG;
        if (segment_offsets[0] != 0) return DYNAMIX_ERR_SEGMENTS;
        while (segment_offsets[S] < P) {
            if (segment_offsets[S + 1] <= segment_offsets[S]) return DYNAMIX_ERR_SEGMENTS;
            ++S;
        }
        if (segment_offsets[S] != P || S == 0) return DYNAMIX_ERR_SEGMENTS;
    }
    return dynamix_grad_aggregate_stats_ex(grads, batch_sizes, K, P, dtype, segment_offsets, S,
                                           out_agg, out_stats, stream);
}

int64_t dynamix_stats_count(int32_t K, int64_t num_segments)
{
    if (K < 1 || K > DYNAMIX_K_MAX || num_segments < 0) return -1;
    return (1 + num_segments) * (int64_t)(DYNAMIX_STATS_HEAD + 2 * K);
}

const char* dynamix_status_string(int status)
{
    switch (status) {
    case DYNAMIX_OK: return "ok";
    case DYNAMIX_ERR_NULL: return "a required pointer is NULL";
    case DYNAMIX_ERR_ARG: return "invalid K, P, dtype or batch size";
    case DYNAMIX_ERR_SEGMENTS: return "invalid segment offsets";
    case DYNAMIX_ERR_ALIGN: return "misaligned pointer";
    case DYNAMIX_ERR_NOMEM: return "workspace allocation failed";
    case DYNAMIX_ERR_HIP: return "HIP runtime call failed";
    case DYNAMIX_ERR_CAPACITY: return "shape exceeds the static scratch buffer";
    default: return "unknown status";
    }
}

int64_t dynamix_plan_describe(int32_t K, int64_t P, int32_t dtype, const int64_t* segment_offsets,
                              int64_t num_segments, int64_t max_blocks, int64_t* pieces_out,
                              int64_t capacity)
{
    const int rc = dynamix::check_shape(K, P, dtype, segment_offsets, num_segments);
    if (rc != DYNAMIX_OK) return -rc;
    if (max_blocks < 1 || capacity < 0 || (capacity > 0 && !pieces_out)) return -DYNAMIX_ERR_ARG;
    try {
        dynamix::Layout L;
        dynamix::make_layout(K, dtype, dynamix::kOptNone, P, (int)num_segments, segment_offsets,
                             max_blocks, L);
        const int64_t n = (int64_t)L.pieces.size();
        for (int64_t i = 0; i < n && i < capacity; ++i) {
            const dynamix::Piece& pc = L.pieces[i];
            int64_t* o = pieces_out + 6 * i;
            o[0] = pc.v_begin; o[1] = pc.v_end; o[2] = pc.v_step;
            o[3] = pc.e_lo; o[4] = pc.e_hi; o[5] = pc.block;
        }
        return n;
    } catch (...) {
        return -DYNAMIX_ERR_NOMEM;
    }
}

int dynamix_timing_begin(int32_t capacity)
{
    if (capacity < 0 || capacity > (1 << 20)) return DYNAMIX_ERR_ARG;
    std::lock_guard<std::mutex> lock(dynamix::g_mutex);
    dynamix::Timing& t = dynamix::g_timing;
    for (hipEvent_t e : t.events) (void)hipEventDestroy(e);
    t.events.clear();
    t.capacity = t.used = 0;
    t.calls = 0;
    try {
        t.events.reserve(3 * (size_t)capacity);
    } catch (...) {
        return DYNAMIX_ERR_NOMEM;
    }
    for (int i = 0; i < 3 * capacity; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return DYNAMIX_ERR_HIP;
        t.events.push_back(e);
    }
    t.capacity = capacity;
    return DYNAMIX_OK;
}

int dynamix_timing_every(int32_t n)
{
    if (n < 1) return DYNAMIX_ERR_ARG;
    std::lock_guard<std::mutex> lock(dynamix::g_mutex);
    dynamix::g_timing.every = n;
    dynamix::g_timing.calls = 0;
    return DYNAMIX_OK;
}

int32_t dynamix_timing_count(void)
{
    std::lock_guard<std::mutex> lock(dynamix::g_mutex);
    return dynamix::g_timing.used;
}

int dynamix_timing_read(int32_t index, float* stream_pass_ms, float* final_reduce_ms)
{
    if (!stream_pass_ms || !final_reduce_ms) return DYNAMIX_ERR_NULL;
    std::lock_guard<std::mutex> lock(dynamix::g_mutex);
    dynamix::Timing& t = dynamix::g_timing;
    if (index < 0 || index >= t.used) return DYNAMIX_ERR_ARG;
    hipEvent_t* ev = &t.events[3 * (size_t)index];
    if (hipEventElapsedTime(stream_pass_ms, ev[0], ev[1]) != hipSuccess ||
        hipEventElapsedTime(final_reduce_ms, ev[1], ev[2]) != hipSuccess) {
        (void)hipGetLastError();
        return DYNAMIX_ERR_HIP;
    }
    return DYNAMIX_OK;
}

int dynamix_release_cached(void)
{
    std::lock_guard<std::mutex> lock(dynamix::g_mutex);
    dynamix::g_plans.clear();
    for (auto& sd : dynamix::g_static) sd.plan.reset();   // host side only: the array itself stays
    return DYNAMIX_OK;
}

}  // extern "C"
