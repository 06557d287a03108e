// libwagma: the per-iteration hot path of WAGMA-SGD (arXiv 2005.00124,
// Algorithm 2 lines 6-17 with the groups of Algorithm 1) for P model replicas
// stored as P rows in one MI355X's HBM.  gfx950 only.
//
// Work decomposition.  Every operation of the step is elementwise in the
// parameter index; only the P rows interact.  A thread therefore owns one
// 16-byte column slice (4 consecutive parameters) of one group and does the
// whole iteration for it: it loads W, G and the momentum of every member row
// (plus the send buffer of late members), applies the local update, sums the
// contributions in butterfly-phase order, and stores W, momentum and send
// buffer.  Each element is read once and written once, by one thread, so the
// in-place update needs no synchronisation, no LDS and no second buffer, and a
// wavefront's accesses are 1 KiB contiguous per row.  The step is bound by HBM
// bandwidth (about 0.25 flop per byte): no matrix cores are involved.
//
// Two kernels cover all group sizes:
//   step_rows_in_registers<S>  S <= 8 member rows are held in registers
//                              (3*S independent 128-bit loads in flight per lane).
//   step_rows_streamed         any S >= 8: member rows are streamed 8 at a time,
//                              the partial sums kept on a log2(S/8)-deep pairwise
//                              stack; late members re-read their own W' from the
//                              send buffer they just wrote.
// The global average (Algorithm 2 lines 15-16) is the same computation with
// one group of all P ranks in natural order and nobody late.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "wagma.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kMaskWords = WAGMA_MAX_P / 64;
constexpr int kChunk = 8;       // rows per chunk of the streaming kernel
constexpr int kStackDepth = 7;  // log2(WAGMA_MAX_P / kChunk)
constexpr int kNumXcd = 8;      // accelerator complex dies of an MI355X
constexpr int64_t kMaxN = int64_t(1) << 31;

thread_local int g_last_hip_error = 0;

struct TileRef {
    int32_t tensor;       // which tensor a tile of the per-tensor layout belongs to
    int32_t reserved;
    int64_t first_slice;  // first 16-byte slice of the tile inside that tensor
};

struct StepParams {
    float* w;
    const float* g;
    float* m;
    float* pub;
    const int32_t* table;  // P ranks, group-major, butterfly member order
    int64_t ld;            // row stride in floats
    int64_t nvec;          // 16-byte column slices per row = ceil(n/4)
    int64_t tiles;         // workgroups per group = ceil(nvec / block)
    int64_t blocks;        // groups * tiles (grid may be padded beyond this)
    uint64_t late[kMaskWords];
    float lr;
    float mu;
    float inv_members;     // 1/S (or 1/P): exact, a power of two
    float members_plus_1;  // S + 1
    int members;           // S, or P in a global iteration
    int log2_chunks;       // log2(members / kChunk) for the streaming kernel
    int swizzle;           // 1: contiguous block range per XCD
    int tile_major;        // 1: consecutive blocks walk the groups of one column tile
    int stripe_log2;       // log2 of the distance, in KiB, between a workgroup's wavefronts
    int xcd_chunk_log2;    // log2 of the run of consecutive tiles one XCD works on (0: 1 tile)
    // per-tensor layout only (device tables)
    float* const* tw;            // [P][T] base pointers, index rank * T + tensor
    const float* const* tg;
    float* const* tm;
    float* const* tpub;
    const TileRef* tile_ref;     // [tiles]
    const int64_t* tensor_size;  // [T] floats
    int num_tensors;
};

// Element types of the kernel bodies: v4f (one 16-byte column slice) and float
// (the ragged last elements of a tensor in the per-tensor layout).
template <bool NT, typename V>
__device__ __forceinline__ V load_v(const float* p)
{
    if (NT)
        return __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
    return *reinterpret_cast<const V*>(p);
}

template <bool NT, typename V>
__device__ __forceinline__ void store_v(float* p, V v)
{
    if (NT)
        __builtin_nontemporal_store(v, reinterpret_cast<V*>(p));
    else
        *reinterpret_cast<V*>(p) = v;
}

// a*b + c with one rounding per element (Algorithm 2 lines 6-7 are two of these).
__device__ __forceinline__ float fma_v(float a, float b, float c)
{
    return __builtin_fmaf(a, b, c);
}

__device__ __forceinline__ v4f fma_v(float a, v4f b, v4f c)
{
    v4f r;
    r.x = __builtin_fmaf(a, b.x, c.x);
    r.y = __builtin_fmaf(a, b.y, c.y);
    r.z = __builtin_fmaf(a, b.z, c.z);
    r.w = __builtin_fmaf(a, b.w, c.w);
    return r;
}

__device__ __forceinline__ bool is_late(const StepParams& p, int rank)
{
    return (p.late[rank >> 6] >> (rank & 63)) & 1u;
}

// Balanced pairwise sum of N = 2^k values: adjacent members first, i.e. the
// butterfly phases of Section 3.3 in the order Algorithm 1 runs them.
template <int N, typename V>
__device__ __forceinline__ V tree_sum(const V* c)
{
    if constexpr (N == 1) {
        return c[0];
    } else {
        V left = tree_sum<N / 2, V>(c);
        V right = tree_sum<N / 2, V>(c + N / 2);
        return left + right;
    }
}

// Where the lane's element of a rank's row lives.  Flat layout: P rows of ld floats;
// the row base is wave-uniform (scalar registers) and the lane adds one 32-bit offset.
struct FlatAddr {
    const StepParams& p;
    uint32_t lane_at;  // float index inside the row
    __device__ __forceinline__ float* w(int rank) const { return p.w + (int64_t)rank * p.ld + lane_at; }
    __device__ __forceinline__ const float* g(int rank) const { return p.g + (int64_t)rank * p.ld + lane_at; }
    __device__ __forceinline__ float* m(int rank) const { return p.m + (int64_t)rank * p.ld + lane_at; }
    __device__ __forceinline__ float* pub(int rank) const { return p.pub + (int64_t)rank * p.ld + lane_at; }
};

// Per-tensor layout: a table of P x T base pointers per array; the lane adds its
// float index inside the tensor.
struct TensorAddr {
    const StepParams& p;
    int tensor;
    uint32_t lane_at;
    __device__ __forceinline__ int64_t slot(int rank) const { return (int64_t)rank * p.num_tensors + tensor; }
    __device__ __forceinline__ float* w(int rank) const { return p.tw[slot(rank)] + lane_at; }
    __device__ __forceinline__ const float* g(int rank) const { return p.tg[slot(rank)] + lane_at; }
    __device__ __forceinline__ float* m(int rank) const { return p.tm[slot(rank)] + lane_at; }
    __device__ __forceinline__ float* pub(int rank) const { return p.tpub[slot(rank)] + lane_at; }
};

// One group of S <= 8 members, all member rows held in registers.
template <int S, bool NT, typename V, typename Addr>
__device__ __forceinline__ void registers_body(const StepParams& p, const int32_t* member, const Addr& at)
{
    bool late[S];
    int rank[S];
    V wv[S], gv[S], mv[S], contrib[S];
#pragma unroll
    for (int e = 0; e < S; ++e) {
        rank[e] = member[e];
        late[e] = is_late(p, rank[e]);
        wv[e] = load_v<NT, V>(at.w(rank[e]));
        gv[e] = load_v<NT, V>(at.g(rank[e]));
        mv[e] = load_v<NT, V>(at.m(rank[e]));
    }
#pragma unroll
    for (int e = 0; e < S; ++e)
        if (late[e])
            contrib[e] = load_v<NT, V>(at.pub(rank[e]));  // the send buffer of a late process

    // (Issuing the loads and stores one array at a time instead of row by row was measured:
    // no difference.)
#pragma unroll
    for (int e = 0; e < S; ++e) {
        const V m_new = fma_v(p.mu, mv[e], gv[e]);
        wv[e] = fma_v(-p.lr, m_new, wv[e]);  // W'
        store_v<NT, V>(at.m(rank[e]), m_new);
        store_v<NT, V>(at.pub(rank[e]), wv[e]);
        if (!late[e])
            contrib[e] = wv[e];
    }
    const V w_sum = tree_sum<S, V>(contrib);
#pragma unroll
    for (int e = 0; e < S; ++e) {
        V out;
        if (late[e])
            out = (w_sum + wv[e]) / p.members_plus_1;
        else
            out = w_sum * p.inv_members;
        store_v<NT, V>(at.w(rank[e]), out);
    }
}

// One group of any size >= 8: member rows streamed 8 at a time.
template <bool NT, typename V, typename Addr>
__device__ __forceinline__ void streamed_body(const StepParams& p, const int32_t* member, const Addr& at)
{
    const int chunks = p.members / kChunk;
    V stack[kStackDepth];
    V acc;
    for (int c = 0; c < chunks; ++c) {
        int rank[kChunk];
        bool late[kChunk];
        V wv[kChunk], gv[kChunk], mv[kChunk], contrib[kChunk];
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            rank[i] = member[c * kChunk + i];
            late[i] = is_late(p, rank[i]);
            wv[i] = load_v<NT, V>(at.w(rank[i]));
            gv[i] = load_v<NT, V>(at.g(rank[i]));
            mv[i] = load_v<NT, V>(at.m(rank[i]));
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
            if (late[i])
                contrib[i] = load_v<NT, V>(at.pub(rank[i]));
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            const V m_new = fma_v(p.mu, mv[i], gv[i]);
            wv[i] = fma_v(-p.lr, m_new, wv[i]);
            store_v<NT, V>(at.m(rank[i]), m_new);
            store_v<NT, V>(at.pub(rank[i]), wv[i]);
            if (!late[i])
                contrib[i] = wv[i];
        }
        acc = tree_sum<kChunk, V>(contrib);
        // Binary-counter carry: after chunk c the stack holds one partial sum per set
        // bit of c+1, so equal-sized neighbours are always added left + right.
        bool carry = true;
#pragma unroll
        for (int l = 0; l < kStackDepth; ++l) {
            if (carry) {
                if ((c >> l) & 1) {
                    acc = stack[l] + acc;
                } else {
                    stack[l] = acc;
                    carry = false;
                }
            }
        }
    }
    V w_sum = acc;
#pragma unroll
    for (int l = 0; l < kStackDepth; ++l)
        if (l == p.log2_chunks)
            w_sum = stack[l];
    const V fresh = w_sum * p.inv_members;

    for (int e = 0; e < p.members; ++e) {
        const int rank = member[e];
        V out = fresh;
        if (is_late(p, rank)) {
            // W' of this member: this thread stored it to the send buffer above.
            const V w_prime = load_v<false, V>(at.pub(rank));
            out = (w_sum + w_prime) / p.members_plus_1;
        }
        store_v<NT, V>(at.w(rank), out);
    }
}

// Which group and which 16-byte column slice does this lane own?  Workgroups are
// handed to the 8 XCDs round-robin; with `swizzle` each XCD instead walks one
// contiguous eighth of the work.  A wavefront always owns 64 consecutive slices
// (1 KiB per row).  The wavefronts of workgroup `tile` sit 2^stripe_log2 KiB apart
// and consecutive workgroups fill the gaps, so that a workgroup's simultaneous
// requests to one row hit addresses one stripe apart (stripe_log2 = 0: the plain
// contiguous tile).  Returns false for lanes and workgroups beyond the end.
template <int BLOCK>
__device__ __forceinline__ bool decode_block(const StepParams& p, int64_t& group, int64_t& col)
{
    int64_t b = blockIdx.x;
    if (p.swizzle) {
        const int64_t per_xcd = (p.blocks + kNumXcd - 1) / kNumXcd;
        b = (b % kNumXcd) * per_xcd + b / kNumXcd;
    }
    if (b >= p.blocks)
        return false;
    int64_t tile;
    if (p.tile_major) {
        const int64_t groups = p.blocks / p.tiles;
        group = b % groups;
        tile = b / groups;
    } else {
        group = b / p.tiles;
        tile = b % p.tiles;
    }
    if (p.xcd_chunk_log2 > 0) {
        // Workgroup b runs on XCD b % 8.  Give each XCD runs of 2^xcd_chunk_log2 consecutive
        // tiles: the XCD number moves from tile bits [0,3) up to bits [j, j+3).
        const int j = p.xcd_chunk_log2;
        const int64_t xcd = tile & (kNumXcd - 1);
        const int64_t hi = tile >> 3;
        tile = ((hi >> j) << (j + 3)) | (xcd << j) | (hi & ((int64_t(1) << j) - 1));
    }
    constexpr int kWavesPerBlock = BLOCK / 64;
    const int64_t wave = threadIdx.x >> 6;
    const int64_t lane = threadIdx.x & 63;
    const int64_t super = tile >> p.stripe_log2;
    const int64_t within = tile & ((int64_t(1) << p.stripe_log2) - 1);
    const int64_t chunk = ((super * kWavesPerBlock + wave) << p.stripe_log2) + within;
    col = chunk * 64 + lane;
    return col < p.nvec;
}

template <int S, bool NT, int BLOCK, int WAVES>
__global__ void __launch_bounds__(BLOCK, WAVES) step_rows_in_registers(const StepParams p)
{
    int64_t group, col;
    if (!decode_block<BLOCK>(p, group, col))
        return;
    const FlatAddr at{p, (uint32_t)col * 4u};
    registers_body<S, NT, v4f>(p, p.table + group * S, at);
}

template <bool NT, int BLOCK, int WAVES>
__global__ void __launch_bounds__(BLOCK, WAVES) step_rows_streamed(const StepParams p)
{
    int64_t group, col;
    if (!decode_block<BLOCK>(p, group, col))
        return;
    const FlatAddr at{p, (uint32_t)col * 4u};
    streamed_body<NT, v4f>(p, p.table + group * p.members, at);
}

// Per-tensor layout.  Workgroup b owns tile b % tiles of group b / tiles; the tile table
// names the tensor and the tile's first 16-byte slice inside it.  A lane whose slice is
// cut off by the end of the tensor does the remaining 1..3 elements one by one; nothing
// beyond a tensor's last element is touched.
template <int S, bool NT, int BLOCK>
__global__ void __launch_bounds__(BLOCK, 2) step_tensors_in_registers(const StepParams p)
{
    const int64_t group = blockIdx.x / p.tiles;
    const TileRef ref = p.tile_ref[blockIdx.x % p.tiles];
    const int64_t size = p.tensor_size[ref.tensor];
    const int64_t first = (ref.first_slice + threadIdx.x) * 4;
    if (first >= size)
        return;
    const int32_t* member = p.table + group * S;
    TensorAddr at{p, ref.tensor, (uint32_t)first};
    if (first + 4 <= size) {
        registers_body<S, NT, v4f>(p, member, at);
    } else {
        for (int64_t k = first; k < size; ++k) {
            at.lane_at = (uint32_t)k;
            registers_body<S, NT, float>(p, member, at);
        }
    }
}

template <bool NT, int BLOCK>
__global__ void __launch_bounds__(BLOCK, 2) step_tensors_streamed(const StepParams p)
{
    const int64_t group = blockIdx.x / p.tiles;
    const TileRef ref = p.tile_ref[blockIdx.x % p.tiles];
    const int64_t size = p.tensor_size[ref.tensor];
    const int64_t first = (ref.first_slice + threadIdx.x) * 4;
    if (first >= size)
        return;
    const int32_t* member = p.table + group * p.members;
    TensorAddr at{p, ref.tensor, (uint32_t)first};
    if (first + 4 <= size) {
        streamed_body<NT, v4f>(p, member, at);
    } else {
        for (int64_t k = first; k < size; ++k) {
            at.lane_at = (uint32_t)k;
            streamed_body<NT, float>(p, member, at);
        }
    }
}

// Schedule table: rows 0..period-1 hold the groups of iterations t = residue
// (mod period) after Algorithm 1; row `period` is the single group 0..P-1 of a
// global iteration.  Slot k*S + e of a row is member e of the group with the
// k-th smallest base.  The phase bits are b_r = (t*g + r) mod G, r = 0..g-1
// (Algorithm 1 lines 3, 6, 14); the base has those bits clear and the bits of k
// spread over the remaining positions; member e sets phase bit b_r iff digit r
// of e is set.
__global__ void build_schedule_table(int32_t* table, int P, int G, int g, int period)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (period + 1) * P)
        return;
    const int residue = idx / P;
    const int slot = idx % P;
    if (residue == period) {
        table[idx] = slot;
        return;
    }
    const int k = slot >> g;
    const int e = slot & ((1 << g) - 1);
    int phase_mask = 0, member_bits = 0;
    for (int r = 0; r < g; ++r) {
        const int b = (residue * g + r) % G;
        phase_mask |= 1 << b;
        if ((e >> r) & 1)
            member_bits |= 1 << b;
    }
    int base = 0, rest = k;
    for (int bit = 0; bit < G; ++bit) {
        if (!((phase_mask >> bit) & 1)) {
            base |= (rest & 1) << bit;
            rest >>= 1;
        }
    }
    table[idx] = base | member_bits;
}

// ---------------------------------------------------------------------------
// HBM-region placement.  Measured on MI355X: the 288 GB of HBM are split, by the
// top physical address bits, into a few regions tens of GiB wide (the ranks of
// the 12-high stacks, by all appearance).  Write streams that all fall into one
// region sustain about 5.9 TB/s, write streams spread over two regions about
// 7.2 TB/s; reads do not care.  The step writes W, the momentum and the send
// buffer of every member row at once, so it runs about 15% faster when these
// three arrays lie in different regions.  Regions cannot be queried, so the
// allocator finds them by timing: this kernel writes four streams through `a`
// and four through `b`; it is fast exactly when a and b lie in different regions.
// The probe must write well beyond the 256 MB Infinity Cache to see the HBM at all.
constexpr size_t kProbeSideMax = size_t(1) << 30;            // bytes written through each pointer
constexpr size_t kPlacementMinBytes = size_t(1) << 30;       // smaller arrays are not placed
constexpr int kMaxCandidates = 64;

__global__ void __launch_bounds__(256) placement_probe(float* a, float* b, uint32_t vec_per_stream)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= vec_per_stream)
        return;
    const v4f zero = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (uint32_t k = 0; k < 4; ++k) {
        __builtin_nontemporal_store(zero, reinterpret_cast<v4f*>(a) + (size_t)k * vec_per_stream + i);
        __builtin_nontemporal_store(zero, reinterpret_cast<v4f*>(b) + (size_t)k * vec_per_stream + i);
    }
}

// GB/s of the probe on (a, b); both must have side_bytes behind them.  < 0 on a HIP error.
double probe_gbs(float* a, float* b, size_t side_bytes, hipEvent_t start, hipEvent_t stop)
{
    const uint32_t vec = (uint32_t)(side_bytes / 4 / 16);
    const unsigned grid = (vec + 255) / 256;
    float best_ms = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {
        if (hipEventRecord(start, nullptr) != hipSuccess)
            return -1.0;
        hipLaunchKernelGGL(placement_probe, dim3(grid), dim3(256), 0, (hipStream_t) nullptr, a, b, vec);
        if (hipEventRecord(stop, nullptr) != hipSuccess || hipEventSynchronize(stop) != hipSuccess)
            return -1.0;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, start, stop) != hipSuccess)
            return -1.0;
        if (rep > 0 && ms < best_ms)
            best_ms = ms;
    }
    return 2.0 * 4.0 * 16.0 * (double)vec / (best_ms * 1e-3) / 1e9;
}

// The region search of wagma_alloc_buffers.  Candidates are whole arrays allocated one after
// another (the driver hands out physical memory in address order, so later candidates lie
// further on).  Probe rates fall into two clusters about 18% apart: both pointers in one
// region (slow) or in two regions (fast).  The threshold between them is re-estimated from
// all rates measured so far (the split of the sorted rates that maximises the between-class
// variance), and the roles are re-derived from the stored measurements after every new
// candidate, so that an unlucky first candidate cannot mislead the search.
struct RegionSearch {
    static constexpr double kMinSpread = 1.10;  // cluster means closer than this: only one cluster was seen
    float* cand[kMaxCandidates];
    double self[kMaxCandidates], ends[kMaxCandidates];
    double cross[kMaxCandidates][kMaxCandidates];  // 0 = not measured yet
    double vals[kMaxCandidates * 8];
    int n = 0, n_vals = 0;
    double threshold = 1e30;  // rates below: same region; at or above: different regions
    double slow_mean = 0.0, fast_mean = 0.0;
    size_t side = 0, tail = 0;
    hipEvent_t start = nullptr, stop = nullptr;
    int w = -1, m = -1, pub = -1, g = -1;  // indices into cand[]
    bool failed = false;

    void see(double v)
    {
        if (v <= 0.0) {
            failed = true;
            return;
        }
        if (n_vals < kMaxCandidates * 8)
            vals[n_vals++] = v;
        double sorted[kMaxCandidates * 8];
        for (int i = 0; i < n_vals; ++i)
            sorted[i] = vals[i];
        for (int i = 1; i < n_vals; ++i) {  // insertion sort: a few hundred values at most
            const double x = sorted[i];
            int j = i - 1;
            while (j >= 0 && sorted[j] > x) {
                sorted[j + 1] = sorted[j];
                --j;
            }
            sorted[j + 1] = x;
        }
        double total = 0.0;
        for (int i = 0; i < n_vals; ++i)
            total += sorted[i];
        slow_mean = total / n_vals;
        fast_mean = 0.0;
        threshold = 1e30;
        if (sorted[n_vals - 1] < kMinSpread * sorted[0])
            return;
        double best = -1.0, low_sum = 0.0;
        double split_at = 1e30, mean_lo_best = slow_mean, mean_hi_best = 0.0;
        for (int k = 1; k < n_vals; ++k) {  // k values in the slow class
            low_sum += sorted[k - 1];
            const double mean_lo = low_sum / k, mean_hi = (total - low_sum) / (n_vals - k);
            const double score = (double)k * (n_vals - k) * (mean_hi - mean_lo) * (mean_hi - mean_lo);
            if (score > best) {
                best = score;
                split_at = 0.5 * (sorted[k - 1] + sorted[k]);
                mean_lo_best = mean_lo;
                mean_hi_best = mean_hi;
            }
        }
        // two real clusters are about 18% apart; a split of mere noise is not
        if (mean_hi_best >= kMinSpread * mean_lo_best) {
            threshold = split_at;
            slow_mean = mean_lo_best;
            fast_mean = mean_hi_best;
        }
    }
    void add(float* c)
    {
        cand[n] = c;
        for (int k = 0; k <= n; ++k)
            cross[n][k] = cross[k][n] = 0.0;
        if (n == 0) {
            // The clocks of an idle GPU take a while to come up: time nothing before that.
            for (int rep = 0; rep < 40; ++rep)
                (void)probe_gbs(c, c + side / sizeof(float), side, start, stop);
        }
        self[n] = probe_gbs(c, c + side / sizeof(float), side, start, stop);
        see(self[n]);
        ends[n] = probe_gbs(c, c + tail, side, start, stop);
        see(ends[n]);
        ++n;
        if (n > 1)
            (void)between(0, n - 1);  // one rate per candidate that does not depend on the roles
    }
    void report() const
    {
        std::fprintf(stderr, "wagma placement: %d candidates, threshold %.0f GB/s (slow %.0f, fast %.0f), "
                             "w=%d g=%d m=%d pub=%d\n", n, threshold, slow_mean, fast_mean, w, g, m, pub);
        for (int i = 0; i < n; ++i) {
            std::fprintf(stderr, "  cand %2d %p self %.0f ends %.0f cross:", i, (void*)cand[i], self[i], ends[i]);
            for (int j = 0; j < n; ++j)
                if (cross[i][j] != 0.0)
                    std::fprintf(stderr, " %d:%.0f", j, cross[i][j]);
            std::fprintf(stderr, "\n");
        }
    }
    double between(int i, int j)
    {
        if (cross[i][j] == 0.0) {
            cross[i][j] = cross[j][i] = probe_gbs(cand[i], cand[j], side, start, stop);
            see(cross[i][j]);
        }
        return cross[i][j];
    }
    // a candidate that straddles two regions is of no use
    bool clean(int i) const { return self[i] < threshold && ends[i] < threshold; }
    // Greedy roles in allocation order; repeated while new probes keep moving the threshold.
    void assign()
    {
        for (int round = 0; round < 8 && !failed; ++round) {
            const double threshold_before = threshold;
            w = m = pub = g = -1;
            for (int i = 0; i < n && !failed; ++i) {
                if (!clean(i))
                    continue;
                if (w < 0) {
                    w = i;
                    continue;
                }
                const int placed[3] = {w, m, pub};
                bool apart = true, with_w = false;
                for (int k = 0; k < 3 && placed[k] >= 0; ++k) {
                    if (between(placed[k], i) < threshold) {
                        apart = false;
                        if (k == 0)
                            with_w = true;
                    }
                }
                if (apart && m < 0)
                    m = i;
                else if (apart && pub < 0)
                    pub = i;
                else if (with_w && g < 0)
                    g = i;
            }
            if (threshold == threshold_before)
                break;  // the yardstick did not move: the roles stand
        }
        if (threshold > 1e29)
            m = pub = -1;  // only one cluster seen: nothing is known to be apart
    }
    bool complete() const { return w >= 0 && m >= 0 && pub >= 0 && g >= 0; }
};

int exact_log2(int64_t x)
{
    if (x < 1 || (x & (x - 1)) != 0)
        return -1;
    int l = 0;
    while ((int64_t(1) << l) < x)
        ++l;
    return l;
}

int gcd_int(int a, int b)
{
    while (b) {
        const int r = a % b;
        a = b;
        b = r;
    }
    return a;
}

int hip_failed(hipError_t e)
{
    g_last_hip_error = (int)e;
    return WAGMA_EHIP;
}

// WAVES = resident wavefronts per SIMD the register allocation must allow
// (2, 3 or 4: at most 256, 168 or 128 vector registers per lane).
template <int S, bool NT, int BLOCK, int WAVES>
void launch_registers(const StepParams& p, unsigned grid, hipStream_t stream)
{
    hipLaunchKernelGGL((step_rows_in_registers<S, NT, BLOCK, WAVES>), dim3(grid), dim3(BLOCK), 0,
                       stream, p);
}

template <bool NT, int BLOCK, int WAVES>
void launch_variant(const StepParams& p, bool streamed, unsigned grid, hipStream_t stream)
{
    if (streamed) {
        hipLaunchKernelGGL((step_rows_streamed<NT, BLOCK, WAVES>), dim3(grid), dim3(BLOCK), 0,
                           stream, p);
        return;
    }
    switch (p.members) {
    case 1: launch_registers<1, NT, BLOCK, 4>(p, grid, stream); break;
    case 2: launch_registers<2, NT, BLOCK, 4>(p, grid, stream); break;
    case 4: launch_registers<4, NT, BLOCK, 4>(p, grid, stream); break;
    default: launch_registers<8, NT, BLOCK, WAVES>(p, grid, stream); break;
    }
}

template <bool NT, int BLOCK>
void launch_waves(const StepParams& p, bool streamed, int waves, unsigned grid, hipStream_t stream)
{
    switch (waves) {
    case 2: launch_variant<NT, BLOCK, 2>(p, streamed, grid, stream); break;
    case 3: launch_variant<NT, BLOCK, 3>(p, streamed, grid, stream); break;
    default: launch_variant<NT, BLOCK, 4>(p, streamed, grid, stream); break;
    }
}

template <bool NT>
void launch_block(const StepParams& p, bool streamed, int block, int waves, unsigned grid,
                  hipStream_t stream)
{
    if (block == 512)
        launch_waves<NT, 512>(p, streamed, waves, grid, stream);
    else
        launch_waves<NT, 256>(p, streamed, waves, grid, stream);
}

}  // namespace

struct wagma_ctx {
    int P, S, G, g, tau, period, device;
    int fixed_groups;  // 1: every group iteration uses the groups of iteration 0
    int64_t n, ld;
    int32_t* d_table;  // (period + 1) * P, device
    int32_t* h_table;  // host mirror
    int opt_block, opt_nontemporal, opt_force_stream, opt_swizzle, opt_tile_major, opt_waves, opt_stripe_log2, opt_xcd_chunk_log2;
    float* placed[4];        // w, g, m, pub handed out by wagma_alloc_buffers (or all NULL)
    int place_candidates;    // allocations tried by the last wagma_alloc_buffers
    int place_regions;       // how many of w, m, pub lie in pairwise different regions (1..3)
    int place_g_with_w;      // 1 if g was found a place in the region of w
    double place_same_gbs;   // probe rate inside one region
    double place_split_gbs;  // probe rate between the regions of w and m (0 if not separated)
};

struct wagma_tensors {
    wagma_ctx* ctx;
    int T;
    int64_t tiles;      // workgroups per group
    void* d_blob;       // one device allocation: four pointer tables, the sizes, the tile table
    float* const* tw;
    const float* const* tg;
    float* const* tm;
    float* const* tpub;
    const int64_t* tensor_size;
    const TileRef* tile_ref;
};

namespace {
constexpr int kTensorBlock = 256;  // threads per workgroup of the per-tensor kernels

template <bool NT>
void launch_tensors(const StepParams& p, unsigned grid, hipStream_t stream)
{
    const dim3 g(grid), b(kTensorBlock);
    switch (p.members) {
    case 1: hipLaunchKernelGGL((step_tensors_in_registers<1, NT, kTensorBlock>), g, b, 0, stream, p); break;
    case 2: hipLaunchKernelGGL((step_tensors_in_registers<2, NT, kTensorBlock>), g, b, 0, stream, p); break;
    case 4: hipLaunchKernelGGL((step_tensors_in_registers<4, NT, kTensorBlock>), g, b, 0, stream, p); break;
    case 8: hipLaunchKernelGGL((step_tensors_in_registers<8, NT, kTensorBlock>), g, b, 0, stream, p); break;
    default: hipLaunchKernelGGL((step_tensors_streamed<NT, kTensorBlock>), g, b, 0, stream, p); break;
    }
}
}  // namespace

namespace {

// The part of the kernel arguments that both layouts share.
void fill_common(const wagma_ctx* ctx, StepParams& p, bool global, const uint64_t* stale_mask,
                        float lr, float mu, int64_t iter)
{
    std::memset(&p, 0, sizeof(p));
    p.lr = lr;
    p.mu = mu;
    p.members = global ? ctx->P : ctx->S;
    p.inv_members = 1.0f / (float)p.members;
    p.members_plus_1 = (float)(p.members + 1);
    const int32_t* table = nullptr;
    wagma_group_schedule(ctx, iter, &table, nullptr);
    p.table = table;
    if (!global && stale_mask) {
        const int words = (ctx->P + 63) / 64;
        for (int k = 0; k < words; ++k)
            p.late[k] = stale_mask[k];
        if (ctx->P < 64)
            p.late[0] &= (UINT64_C(1) << ctx->P) - 1;
    }
}

}  // namespace

extern "C" {

int wagma_create(wagma_ctx** out, int P, int S, int64_t n, int tau)
{
    if (!out)
        return WAGMA_EINVAL;
    *out = nullptr;
    const int G = exact_log2(P), g = exact_log2(S);
    // lanes address their column with a 32-bit float offset inside a row
    if (G < 0 || g < 0 || P > WAGMA_MAX_P || S > P || n < 1 || tau < 0 || n > kMaxN)
        return WAGMA_EINVAL;

    wagma_ctx* ctx = new (std::nothrow) wagma_ctx();
    if (!ctx)
        return WAGMA_ENOMEM;
    ctx->P = P;
    ctx->S = S;
    ctx->G = G;
    ctx->g = g;
    ctx->tau = tau;
    ctx->n = n;
    ctx->period = (g == 0 || G == 0) ? 1 : G / gcd_int(g, G);
    // Row stride.  Measured on MI355X: rows on 16 KiB boundaries run about 1% faster than rows
    // on 256 B boundaries (and rows off a 128 B boundary up to 10% slower); strides that are a
    // multiple of 1 MiB put all member rows of a group on the same memory channels (20% slower),
    // so such a stride is skewed by a few row alignments.  Small models keep the padding small.
    const int64_t row_align = n >= (int64_t(1) << 20) ? 4096 : 64;  // floats
    ctx->ld = (n + row_align - 1) / row_align * row_align;
    if ((ctx->ld * 4) % (int64_t(1) << 20) == 0)
        ctx->ld += 5 * row_align;
    // measured best on MI355X for the P=64, S=8, 25.6M-parameter workload
    ctx->opt_block = 512;
    ctx->opt_nontemporal = 1;
    ctx->opt_force_stream = 0;
    ctx->opt_swizzle = 0;
    ctx->opt_tile_major = 0;
    ctx->opt_waves = 2;
    ctx->opt_stripe_log2 = 2;
    ctx->opt_xcd_chunk_log2 = 2;
    ctx->fixed_groups = 0;
    ctx->d_table = nullptr;
    ctx->h_table = nullptr;
    for (int k = 0; k < 4; ++k)
        ctx->placed[k] = nullptr;
    ctx->place_candidates = 0;
    ctx->place_regions = 0;
    ctx->place_g_with_w = 0;
    ctx->place_same_gbs = 0.0;
    ctx->place_split_gbs = 0.0;

    const size_t entries = (size_t)(ctx->period + 1) * (size_t)P;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) {
        delete ctx;
        return hip_failed(e);
    }
    ctx->h_table = (int32_t*)std::malloc(entries * sizeof(int32_t));
    if (!ctx->h_table) {
        delete ctx;
        return WAGMA_ENOMEM;
    }
    e = hipMalloc((void**)&ctx->d_table, entries * sizeof(int32_t));
    if (e != hipSuccess) {
        std::free(ctx->h_table);
        delete ctx;
        g_last_hip_error = (int)e;
        return e == hipErrorOutOfMemory ? WAGMA_ENOMEM : WAGMA_EHIP;
    }
    const unsigned threads = 256;
    const unsigned grid = (unsigned)((entries + threads - 1) / threads);
    hipLaunchKernelGGL(build_schedule_table, dim3(grid), dim3(threads), 0, (hipStream_t) nullptr,
                       ctx->d_table, P, G, g, ctx->period);
    e = hipGetLastError();
    if (e == hipSuccess)
        e = hipMemcpy(ctx->h_table, ctx->d_table, entries * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        (void)hipFree(ctx->d_table);
        std::free(ctx->h_table);
        delete ctx;
        return hip_failed(e);
    }
    *out = ctx;
    return WAGMA_OK;
}

int wagma_destroy(wagma_ctx* ctx)
{
    if (!ctx)
        return WAGMA_OK;
    int rc = wagma_free_buffers(ctx);
    if (ctx->d_table) {
        const hipError_t e = hipFree(ctx->d_table);
        if (e != hipSuccess)
            rc = hip_failed(e);
    }
    std::free(ctx->h_table);
    delete ctx;
    return rc;
}

int64_t wagma_row_stride(const wagma_ctx* ctx)
{
    return ctx ? ctx->ld : (int64_t)WAGMA_EINVAL;
}

int wagma_set_row_stride(wagma_ctx* ctx, int64_t ld)
{
    if (!ctx || ld % 4 != 0 || ld < (ctx->n + 3) / 4 * 4 || ld > 2 * kMaxN)
        return WAGMA_EINVAL;
    ctx->ld = ld;
    return WAGMA_OK;
}

int wagma_set_grouping(wagma_ctx* ctx, int mode)
{
    if (!ctx || (mode != WAGMA_GROUPING_DYNAMIC && mode != WAGMA_GROUPING_FIXED))
        return WAGMA_EINVAL;
    ctx->fixed_groups = mode == WAGMA_GROUPING_FIXED;
    return WAGMA_OK;
}

int wagma_schedule_period(const wagma_ctx* ctx)
{
    return ctx ? ctx->period : WAGMA_EINVAL;
}

int wagma_is_global_iteration(const wagma_ctx* ctx, int64_t iter)
{
    if (!ctx || iter < 0 || iter == INT64_MAX)
        return WAGMA_EINVAL;
    return (ctx->tau > 0 && (iter + 1) % ctx->tau == 0) ? 1 : 0;
}

int wagma_group_schedule(const wagma_ctx* ctx, int64_t iter, const int32_t** dev_table,
                         const int32_t** host_table)
{
    const int global = wagma_is_global_iteration(ctx, iter);
    if (global < 0)
        return global;
    const int64_t row = global ? ctx->period : (ctx->fixed_groups ? 0 : iter % ctx->period);
    if (dev_table)
        *dev_table = ctx->d_table + row * ctx->P;
    if (host_table)
        *host_table = ctx->h_table + row * ctx->P;
    return WAGMA_OK;
}

int wagma_step(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub,
               const uint64_t* stale_mask, float lr, float mu, int64_t iter, void* stream)
{
    const int global = wagma_is_global_iteration(ctx, iter);
    if (global < 0)
        return global;
    if (!w || !g || !m || !pub)
        return WAGMA_EINVAL;
    if ((((uintptr_t)w) | ((uintptr_t)g) | ((uintptr_t)m) | ((uintptr_t)pub)) & 15u)
        return WAGMA_EINVAL;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;

    StepParams p;
    fill_common(ctx, p, global != 0, stale_mask, lr, mu, iter);
    p.w = w;
    p.g = g;
    p.m = m;
    p.pub = pub;
    p.ld = ctx->ld;
    p.nvec = (ctx->n + 3) / 4;
    p.swizzle = ctx->opt_swizzle;
    p.tile_major = ctx->opt_tile_major;

    const bool streamed = p.members > kChunk || (ctx->opt_force_stream && p.members == kChunk);
    p.log2_chunks = streamed ? exact_log2(p.members / kChunk) : 0;
    const int block = ctx->opt_block;
    p.stripe_log2 = ctx->opt_stripe_log2;
    // whole stripes: tiles is a multiple of 2^stripe_log2 (the surplus lanes find col >= nvec)
    p.tiles = (p.nvec + block - 1) / block;
    p.xcd_chunk_log2 = ctx->opt_xcd_chunk_log2;
    // tiles is rounded up to whole stripes and whole XCD rounds (the surplus lanes find col >= nvec)
    int round_log2 = p.stripe_log2;
    if (p.xcd_chunk_log2 > 0 && p.xcd_chunk_log2 + 3 > round_log2)
        round_log2 = p.xcd_chunk_log2 + 3;
    p.tiles = ((p.tiles + (int64_t(1) << round_log2) - 1) >> round_log2) << round_log2;
    p.blocks = (int64_t)(ctx->P / p.members) * p.tiles;
    int64_t grid = p.blocks;
    if (p.swizzle)
        grid = (grid + kNumXcd - 1) / kNumXcd * kNumXcd;
    if (grid > 0x7fffffff)
        return WAGMA_EINVAL;

    if (ctx->opt_nontemporal)
        launch_block<true>(p, streamed, block, ctx->opt_waves, (unsigned)grid, (hipStream_t)stream);
    else
        launch_block<false>(p, streamed, block, ctx->opt_waves, (unsigned)grid, (hipStream_t)stream);
    e = hipGetLastError();
    if (e != hipSuccess)
        return hip_failed(e);
    return WAGMA_OK;
}

// ---- per-tensor layout ------------------------------------------------------------------

int wagma_tensors_create(wagma_ctx* ctx, wagma_tensors** out, int T, const int64_t* sizes,
                         float* const* w, const float* const* g, float* const* m, float* const* pub)
{
    if (!out)
        return WAGMA_EINVAL;
    *out = nullptr;
    if (!ctx || T < 1 || T > (1 << 20) || !sizes || !w || !g || !m || !pub)
        return WAGMA_EINVAL;
    int64_t total = 0, tiles = 0;
    for (int k = 0; k < T; ++k) {
        if (sizes[k] < 1 || sizes[k] > kMaxN)
            return WAGMA_EINVAL;
        total += sizes[k];
        tiles += ((sizes[k] + 3) / 4 + kTensorBlock - 1) / kTensorBlock;
    }
    if (total != ctx->n || tiles * (int64_t)ctx->P > 0x7fffffff)
        return WAGMA_EINVAL;
    const size_t slots = (size_t)ctx->P * (size_t)T;
    for (size_t i = 0; i < slots; ++i) {
        if (!w[i] || !g[i] || !m[i] || !pub[i])
            return WAGMA_EINVAL;
        if ((((uintptr_t)w[i]) | ((uintptr_t)g[i]) | ((uintptr_t)m[i]) | ((uintptr_t)pub[i])) & 15u)
            return WAGMA_EINVAL;
    }
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;

    // blob layout: [4 pointer tables][T sizes][tiles tile refs]; every part 16-byte aligned
    const size_t table_bytes = (slots * sizeof(void*) + 15) / 16 * 16;
    const size_t sizes_bytes = ((size_t)T * sizeof(int64_t) + 15) / 16 * 16;
    const size_t refs_bytes = (size_t)tiles * sizeof(TileRef);
    const size_t blob_bytes = 4 * table_bytes + sizes_bytes + refs_bytes;
    char* host = (char*)std::malloc(blob_bytes);
    wagma_tensors* plan = new (std::nothrow) wagma_tensors();
    if (!host || !plan) {
        std::free(host);
        delete plan;
        return WAGMA_ENOMEM;
    }
    std::memset(host, 0, blob_bytes);
    std::memcpy(host + 0 * table_bytes, w, slots * sizeof(void*));
    std::memcpy(host + 1 * table_bytes, g, slots * sizeof(void*));
    std::memcpy(host + 2 * table_bytes, m, slots * sizeof(void*));
    std::memcpy(host + 3 * table_bytes, pub, slots * sizeof(void*));
    std::memcpy(host + 4 * table_bytes, sizes, (size_t)T * sizeof(int64_t));
    TileRef* refs = (TileRef*)(host + 4 * table_bytes + sizes_bytes);
    int64_t at = 0;
    for (int k = 0; k < T; ++k) {
        const int64_t slices = (sizes[k] + 3) / 4;
        for (int64_t first = 0; first < slices; first += kTensorBlock) {
            refs[at].tensor = k;
            refs[at].first_slice = first;
            ++at;
        }
    }
    char* dev = nullptr;
    e = hipMalloc((void**)&dev, blob_bytes);
    if (e == hipSuccess)
        e = hipMemcpy(dev, host, blob_bytes, hipMemcpyHostToDevice);
    std::free(host);
    if (e != hipSuccess) {
        if (dev)
            (void)hipFree(dev);
        delete plan;
        g_last_hip_error = (int)e;
        return e == hipErrorOutOfMemory ? WAGMA_ENOMEM : WAGMA_EHIP;
    }
    plan->ctx = ctx;
    plan->T = T;
    plan->tiles = tiles;
    plan->d_blob = dev;
    plan->tw = (float* const*)(dev + 0 * table_bytes);
    plan->tg = (const float* const*)(dev + 1 * table_bytes);
    plan->tm = (float* const*)(dev + 2 * table_bytes);
    plan->tpub = (float* const*)(dev + 3 * table_bytes);
    plan->tensor_size = (const int64_t*)(dev + 4 * table_bytes);
    plan->tile_ref = (const TileRef*)(dev + 4 * table_bytes + sizes_bytes);
    *out = plan;
    return WAGMA_OK;
}

int wagma_tensors_destroy(wagma_tensors* plan)
{
    if (!plan)
        return WAGMA_OK;
    int rc = WAGMA_OK;
    const hipError_t e = hipFree(plan->d_blob);
    if (e != hipSuccess)
        rc = hip_failed(e);
    delete plan;
    return rc;
}

int wagma_step_tensors(wagma_ctx* ctx, const wagma_tensors* plan, const uint64_t* stale_mask, float lr,
                       float mu, int64_t iter, void* stream)
{
    const int global = wagma_is_global_iteration(ctx, iter);
    if (global < 0)
        return global;
    if (!plan || plan->ctx != ctx)
        return WAGMA_EINVAL;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;

    StepParams p;
    fill_common(ctx, p, global != 0, stale_mask, lr, mu, iter);
    p.tw = plan->tw;
    p.tg = plan->tg;
    p.tm = plan->tm;
    p.tpub = plan->tpub;
    p.tensor_size = plan->tensor_size;
    p.tile_ref = plan->tile_ref;
    p.num_tensors = plan->T;
    p.tiles = plan->tiles;
    p.blocks = (int64_t)(ctx->P / p.members) * p.tiles;
    p.log2_chunks = p.members > kChunk ? exact_log2(p.members / kChunk) : 0;
    if (ctx->opt_nontemporal)
        launch_tensors<true>(p, (unsigned)p.blocks, (hipStream_t)stream);
    else
        launch_tensors<false>(p, (unsigned)p.blocks, (hipStream_t)stream);
    e = hipGetLastError();
    if (e != hipSuccess)
        return hip_failed(e);
    return WAGMA_OK;
}

// 64-bit finaliser of the public splitmix64 generator (Steele, Lea, Flood 2014).
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * UINT64_C(0xBF58476D1CE4E5B9);
    z = (z ^ (z >> 27)) * UINT64_C(0x94D049BB133111EB);
    return z ^ (z >> 31);
}

int wagma_stale_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, uint32_t threshold,
                     uint64_t* mask_words)
{
    if (!ctx || iter < 0 || !mask_words)
        return WAGMA_EINVAL;
    const int words = (ctx->P + 63) / 64;
    const uint64_t iter_key = mix64(seed + ((uint64_t)iter + 1) * UINT64_C(0x9E3779B97F4A7C15));
    for (int k = 0; k < words; ++k) {
        uint64_t word = 0;
        for (int b = 0; b < 64 && k * 64 + b < ctx->P; ++b) {
            const uint64_t rank = (uint64_t)(k * 64 + b);
            const uint64_t h = mix64(iter_key + (rank + 1) * UINT64_C(0xD1B54A32D192ED03));
            if ((uint32_t)(h >> 32) < threshold)
                word |= UINT64_C(1) << b;
        }
        mask_words[k] = word;
    }
    return WAGMA_OK;
}

int wagma_straggler_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, int count,
                         uint64_t* mask_words)
{
    if (!ctx || iter < 0 || count < 0 || count > ctx->P || !mask_words)
        return WAGMA_EINVAL;
    const int words = (ctx->P + 63) / 64;
    for (int k = 0; k < words; ++k)
        mask_words[k] = 0;
    // the key differs from that of wagma_stale_mask by a tag, so the two models are independent
    const uint64_t iter_key =
        mix64((seed ^ UINT64_C(0x5354524147474C52)) + ((uint64_t)iter + 1) * UINT64_C(0x9E3779B97F4A7C15));
    int picked = 0;
    for (uint64_t draw = 1; picked < count; ++draw) {
        const uint64_t h = mix64(iter_key + draw * UINT64_C(0xD1B54A32D192ED03));
        const int rank = ctx->G == 0 ? 0 : (int)(h >> (64 - ctx->G));
        const uint64_t bit = UINT64_C(1) << (rank & 63);
        if (mask_words[rank >> 6] & bit)
            continue;  // already selected: draw again
        mask_words[rank >> 6] |= bit;
        ++picked;
    }
    return WAGMA_OK;
}

int wagma_clock_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, uint32_t tolerance_ms,
                     uint64_t* mask_words, uint32_t* step_ms)
{
    // 16 geometric steps from 2 s to 43.5 s: the tail of the step-time distribution
    static const uint32_t kTailMs[16] = {2000, 2456, 3016, 3703, 4548, 5585, 6858, 8422,
                                         10342, 12700, 15595, 19151, 23517, 28879, 35463, 43500};
    if (!ctx || iter < 0 || !mask_words)
        return WAGMA_EINVAL;
    uint32_t ms[WAGMA_MAX_P];
    const uint64_t iter_key =
        mix64((seed ^ UINT64_C(0x434C4F434B4D534B)) + ((uint64_t)iter + 1) * UINT64_C(0x9E3779B97F4A7C15));
    uint32_t first_done = UINT32_MAX;
    for (int rank = 0; rank < ctx->P; ++rank) {
        const uint64_t h = mix64(iter_key + ((uint64_t)rank + 1) * UINT64_C(0xD1B54A32D192ED03));
        const bool in_tail = (h >> 60) >= 9;  // seven steps in sixteen
        ms[rank] = in_tail ? kTailMs[(h >> 56) & 15] : 1700u + (uint32_t)((h >> 32) & 0xFF) * 300u / 256u;
        if (ms[rank] < first_done)
            first_done = ms[rank];
    }
    const int words = (ctx->P + 63) / 64;
    for (int k = 0; k < words; ++k)
        mask_words[k] = 0;
    for (int rank = 0; rank < ctx->P; ++rank) {
        if ((uint64_t)ms[rank] > (uint64_t)first_done + tolerance_ms)
            mask_words[rank >> 6] |= UINT64_C(1) << (rank & 63);
        if (step_ms)
            step_ms[rank] = ms[rank];
    }
    return WAGMA_OK;
}

int wagma_alloc_buffers(wagma_ctx* ctx, float** w, float** g, float** m, float** pub)
{
    if (!ctx || !w || !g || !m || !pub || ctx->placed[0])
        return WAGMA_EINVAL;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess)
        return hip_failed(e);
    if (device != ctx->device)
        return WAGMA_EINVAL;
    const size_t bytes = (size_t)ctx->P * (size_t)ctx->ld * sizeof(float);
    ctx->place_candidates = 0;
    ctx->place_regions = 1;
    ctx->place_g_with_w = 0;
    ctx->place_same_gbs = 0.0;
    ctx->place_split_gbs = 0.0;

    float* chosen[3] = {nullptr, nullptr, nullptr};  // w, m, pub: pairwise different regions
    float* grad = nullptr;  // g: read only; best in the region of w (never in that of pub)
    float* spare[kMaxCandidates];
    int n_spare = 0;
    int rc = WAGMA_OK;

    if (bytes >= kPlacementMinBytes) {
        RegionSearch* rs = new (std::nothrow) RegionSearch();
        if (rs && hipEventCreate(&rs->start) == hipSuccess && hipEventCreate(&rs->stop) == hipSuccess) {
            // each probe writes `side` bytes through either pointer: at most half an array
            rs->side = bytes / 2 < kProbeSideMax ? bytes / 2 : kProbeSideMax;
            rs->side = rs->side / 1024 * 1024;
            rs->tail = (bytes - rs->side) / sizeof(float) / 4 * 4;
            while (!rs->complete() && !rs->failed && rs->n < kMaxCandidates) {
                size_t free_b = 0, total_b = 0;
                if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < 3 * bytes)
                    break;  // keep room for the caller
                float* c = nullptr;
                if (hipMalloc((void**)&c, bytes) != hipSuccess) {
                    (void)hipGetLastError();
                    break;
                }
                rs->add(c);
                rs->assign();
            }
            if (std::getenv("WAGMA_DEBUG_PLACEMENT"))
                rs->report();
            ctx->place_candidates = rs->n;
            ctx->place_same_gbs = rs->slow_mean;
            ctx->place_split_gbs = rs->fast_mean;
            ctx->place_regions = (rs->w >= 0) + (rs->m >= 0) + (rs->pub >= 0);
            if (ctx->place_regions == 0)
                ctx->place_regions = 1;
            ctx->place_g_with_w = rs->g >= 0;
            for (int i = 0; i < rs->n; ++i) {
                if (i == rs->w)
                    chosen[0] = rs->cand[i];
                else if (i == rs->m)
                    chosen[1] = rs->cand[i];
                else if (i == rs->pub)
                    chosen[2] = rs->cand[i];
                else if (i == rs->g)
                    grad = rs->cand[i];
                else
                    spare[n_spare++] = rs->cand[i];
            }
        }
        if (rs) {
            if (rs->start)
                (void)hipEventDestroy(rs->start);
            if (rs->stop)
                (void)hipEventDestroy(rs->stop);
            delete rs;
        }
    }
    // whatever could not be placed takes any spare candidate, then a fresh allocation
    float** missing[4] = {&chosen[0], &chosen[1], &chosen[2], &grad};
    for (int k = 0; k < 4 && rc == WAGMA_OK; ++k) {
        if (*missing[k])
            continue;
        if (n_spare > 0) {
            *missing[k] = spare[--n_spare];
        } else if ((e = hipMalloc((void**)missing[k], bytes)) != hipSuccess) {
            *missing[k] = nullptr;
            g_last_hip_error = (int)e;
            rc = e == hipErrorOutOfMemory ? WAGMA_ENOMEM : WAGMA_EHIP;
        }
    }
    for (int k = 0; k < n_spare; ++k)
        (void)hipFree(spare[k]);
    if (rc == WAGMA_OK && (e = hipDeviceSynchronize()) != hipSuccess)
        rc = hip_failed(e);
    if (rc != WAGMA_OK) {
        for (int k = 0; k < 3; ++k)
            if (chosen[k])
                (void)hipFree(chosen[k]);
        if (grad)
            (void)hipFree(grad);
        (void)hipGetLastError();
        return rc;
    }
    ctx->placed[0] = *w = chosen[0];
    ctx->placed[1] = *g = grad;
    ctx->placed[2] = *m = chosen[1];
    ctx->placed[3] = *pub = chosen[2];
    return WAGMA_OK;
}

int wagma_free_buffers(wagma_ctx* ctx)
{
    if (!ctx)
        return WAGMA_EINVAL;
    int rc = WAGMA_OK;
    for (int k = 0; k < 4; ++k) {
        if (ctx->placed[k]) {
            const hipError_t e = hipFree(ctx->placed[k]);
            if (e != hipSuccess)
                rc = hip_failed(e);
            ctx->placed[k] = nullptr;
        }
    }
    return rc;
}

int wagma_placement_info(const wagma_ctx* ctx, int* candidates, int* regions, int* g_with_w,
                         double* same_gbs, double* split_gbs)
{
    if (!ctx)
        return WAGMA_EINVAL;
    if (g_with_w)
        *g_with_w = ctx->place_g_with_w;
    if (candidates)
        *candidates = ctx->place_candidates;
    if (regions)
        *regions = ctx->place_regions;
    if (same_gbs)
        *same_gbs = ctx->place_same_gbs;
    if (split_gbs)
        *split_gbs = ctx->place_split_gbs;
    return WAGMA_OK;
}

int wagma_set_option(wagma_ctx* ctx, int option, int64_t value)
{
    if (!ctx)
        return WAGMA_EINVAL;
    switch (option) {
    case WAGMA_OPT_BLOCK:
        if (value != 256 && value != 512)
            return WAGMA_EINVAL;
        ctx->opt_block = (int)value;
        return WAGMA_OK;
    case WAGMA_OPT_NONTEMPORAL:
        ctx->opt_nontemporal = value != 0;
        return WAGMA_OK;
    case WAGMA_OPT_FORCE_STREAM:
        ctx->opt_force_stream = value != 0;
        return WAGMA_OK;
    case WAGMA_OPT_XCD_SWIZZLE:
        ctx->opt_swizzle = value != 0;
        return WAGMA_OK;
    case WAGMA_OPT_TILE_MAJOR:
        ctx->opt_tile_major = value != 0;
        return WAGMA_OK;
    case WAGMA_OPT_STRIPE_LOG2:
        if (value < 0 || value > 16)
            return WAGMA_EINVAL;
        ctx->opt_stripe_log2 = (int)value;
        return WAGMA_OK;
    case WAGMA_OPT_XCD_CHUNK_LOG2:
        if (value < 0 || value > 13)
            return WAGMA_EINVAL;
        ctx->opt_xcd_chunk_log2 = (int)value;
        return WAGMA_OK;
    case WAGMA_OPT_WAVES:
        if (value < 2 || value > 4)
            return WAGMA_EINVAL;
        ctx->opt_waves = (int)value;
        return WAGMA_OK;
    default:
        return WAGMA_EINVAL;
    }
}

const char* wagma_strerror(int code)
{
    switch (code) {
    case WAGMA_OK: return "success";
    case WAGMA_EINVAL: return "invalid argument";
    case WAGMA_EHIP: return "HIP runtime error (see wagma_last_hip_error)";
    case WAGMA_ENOMEM: return "out of memory";
    default: return "unknown libwagma error";
    }
}

int wagma_last_hip_error(void)
{
    return g_last_hip_error;
}

}  // extern "C"
