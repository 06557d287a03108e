// Device code of libwagma: the fused WAGMA-SGD step (Algorithm 2 lines 6-17 of
// arXiv 2005.00124 with the groups of Algorithm 1) for gfx950.  Included by wagma.hip only.
#ifndef WAGMA_KERNELS_H
#define WAGMA_KERNELS_H

#include <hip/hip_runtime.h>

#include <cstdint>

#include "wagma.h"
#include "wagma_shapes.h"
#include "wagma_tiles.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kMaskWords = WAGMA_MAX_P / 64;
constexpr int kRegisterRows = 8;      // groups up to this size are held in registers by one wavefront,
constexpr int kCooperativeRows = 64;  // up to this size by the wavefronts of a workgroup, larger ones streamed
// Rows per chunk of the streaming kernels.  Without busy processes 8 rows (24 loads in flight
// per lane, 2 wavefronts per SIMD) are best; with them a chunk of 8 often holds only two or
// three rows that are loaded at all, and 4 rows with twice the wavefronts hide the latency
// better (S = 16, two thirds of the processes busy: +22 %).
constexpr int streamed_chunk(bool lag) { return lag ? 4 : 8; }
constexpr int streamed_stack_depth(bool lag) { return lag ? 8 : 7; }  // log2(WAGMA_MAX_P / chunk)
constexpr int kNumXcd = 8;      // accelerator complex dies of an MI355X
constexpr int64_t kMaxN = int64_t(1) << 31;

using wagma_detail::AffineTile;
using wagma_detail::SlotPointers;
using wagma_detail::TileRef;

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
    uint64_t late[kMaskWords];  // bit p: process p contributes its send buffer (late or still computing)
    uint64_t busy[kMaskWords];  // bit p: process p is still computing an earlier step (LAG kernels only)
    float lr;
    float mu;
    float inv_members;     // 1/S (or 1/P): exact, a power of two
    float members_plus_1;  // S + 1
    int members;           // S, or P in a global iteration
    int log2_chunks;       // log2(members / streamed_chunk(lag)) for the streaming kernels
    int stripe_log2;       // log2 of the distance, in KiB, between a workgroup's wavefronts
    int xcd_chunk_log2;    // log2 of the run of consecutive tiles one XCD works on (0: 1 tile)
    uint64_t map;          // not 0: replaces the two fields above, see slice_of()
    // per-tensor layout only (device tables)
    const TileRef* tile_ref;     // [tiles]
    const AffineTile* affine_tile;  // [tiles], for the kernels with AFFINE (they read nothing else)
    const SlotPointers* slot_ptrs;  // [units][P] of this iteration's schedule row, for the kernels without
    int64_t mapped_tiles;           // the first so many tiles of the tile table belong to mapped blocks of 64
    int num_ranks;               // P: places per unit in slot_ptrs
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

// A process that is still computing an earlier step when the group allreduce runs
// (Section 4, the execution snapshot, over more than one iteration): its send buffer is
// contributed once more, and nothing of it is read besides or written at all.
__device__ __forceinline__ bool is_busy(const StepParams& p, int rank)
{
    return (p.busy[rank >> 6] >> (rank & 63)) & 1u;
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

// Where the lane's element of a rank's row lives.  Flat layout: P rows of ld floats; the row
// base is wave-uniform and the lane adds its float index inside the row.
// Every address functor names a member's row twice, by its place in the group (`slot`, counted from
// the `member` pointer the kernel body was given) and by its rank; each uses what it needs.
struct FlatAddr {
    const StepParams& p;
    uint32_t lane_at;  // float index inside the row
    __device__ __forceinline__ float* w(int, int rank) const { return p.w + (int64_t)rank * p.ld + lane_at; }
    __device__ __forceinline__ const float* g(int, int rank) const { return p.g + (int64_t)rank * p.ld + lane_at; }
    __device__ __forceinline__ float* m(int, int rank) const { return p.m + (int64_t)rank * p.ld + lane_at; }
    __device__ __forceinline__ float* pub(int, int rank) const { return p.pub + (int64_t)rank * p.ld + lane_at; }
};

// Per-tensor layout with tensors spaced alike in every array: the tile's entry holds the tensor of
// process 0 and the distance to the next process, nothing else is looked up.
struct AffineAddr {
    const AffineTile& t;
    uint32_t lane_at;
    __device__ __forceinline__ float* w(int, int rank) const { return t.w + (int64_t)rank * t.stride + lane_at; }
    __device__ __forceinline__ const float* g(int, int rank) const { return t.g + (int64_t)rank * t.stride + lane_at; }
    __device__ __forceinline__ float* m(int, int rank) const { return t.m + (int64_t)rank * t.stride + lane_at; }
    __device__ __forceinline__ float* pub(int, int rank) const { return t.pub + (int64_t)rank * t.stride + lane_at; }
};

// Per-tensor layout, any placement of the tensors: the plan holds, for every row of the schedule
// table and every unit (a mapped block; or a tensor, for the tiles outside the blocks), the four
// pointers of the unit's tensor for the P places of that schedule row, in the order of the row.  A
// workgroup of a mapped block knows its unit and its first place from its number alone, so these
// pointers are asked for together with the tile's entry and the ranks: nothing waits for anything
// but the data.  The table is small enough to stay in the L2 (P x 32 bytes per unit and row).
struct SlotAddr {
    const SlotPointers* first;  // of the member that `member[0]` names
    uint32_t lane_at;
    __device__ __forceinline__ float* w(int slot, int) const { return first[slot].w + lane_at; }
    __device__ __forceinline__ const float* g(int slot, int) const { return first[slot].g + lane_at; }
    __device__ __forceinline__ float* m(int slot, int) const { return first[slot].m + lane_at; }
    __device__ __forceinline__ float* pub(int slot, int) const { return first[slot].pub + lane_at; }
};

// What a workgroup of the per-tensor kernels looks up about its tile: the tile table's entry and
// the way to its tensor's elements, from the entry itself where the tensors are spaced alike
// (AFFINE), else through the pointers by place.
template <bool AFFINE>
struct TileOf;
template <>
struct TileOf<true> {
    AffineTile entry;
    __device__ __forceinline__ TileOf(const StepParams& p, int64_t tile) : entry(p.affine_tile[tile]) {}
    __device__ __forceinline__ const TileRef& ref() const { return entry.ref; }
    __device__ __forceinline__ AffineAddr at(const StepParams&, const int32_t*, uint32_t lane_at) const
    {
        return AffineAddr{entry, lane_at};
    }
};
template <>
struct TileOf<false> {
    TileRef entry;
    int64_t unit;
    // (a tile of a mapped block does not wait for its entry to know its unit)
    __device__ __forceinline__ TileOf(const StepParams& p, int64_t tile) : entry(p.tile_ref[tile])
    {
        if (tile < p.mapped_tiles)
            unit = tile >> 6;
        else
            unit = wagma_detail::unit_of_tile(tile, p.mapped_tiles, entry.tensor);
    }
    __device__ __forceinline__ const TileRef& ref() const { return entry; }
    // `member` points into this iteration's row of the schedule table: its distance from the
    // row's beginning is the place of the kernel body's first member
    __device__ __forceinline__ SlotAddr at(const StepParams& p, const int32_t* member, uint32_t lane_at) const
    {
        return SlotAddr{p.slot_ptrs + unit * p.num_ranks + (member - p.table), lane_at};
    }
};

// The work of registers_body (below) in two stages, for the kernel that deals a large group's rows
// out to several wavefronts: the local update of S <= 8 rows with the stores of momentum and send
// buffer, which yields W' of every row and the sum of the rows' contributions; and, once the sum
// over the whole group is known, the stores of W.  (Only W' is handed from one stage to the other:
// with the ranks and the late/busy flags handed over as well the compiler keeps 120 registers more
// alive and spills.  registers_body is not built from the two stages: that form of the S = 8
// kernel measured 0.75 % slower, same arrays, side by side.)
template <int S, bool NT, bool LAG, typename V, typename Addr>
__device__ __forceinline__ V rows_update(const StepParams& p, const int32_t* member, const Addr& at,
                                         V (&w_prime)[S])
{
    V gv[S], mv[S], contrib[S];
    bool late[S], busy[S];
    int rank[S];
#pragma unroll
    for (int e = 0; e < S; ++e) {
        rank[e] = member[e];
        late[e] = is_late(p, rank[e]);
        busy[e] = LAG && is_busy(p, rank[e]);
        if (!busy[e]) {
            w_prime[e] = load_v<NT, V>(at.w(e, rank[e]));
            gv[e] = load_v<NT, V>(at.g(e, rank[e]));
            mv[e] = load_v<NT, V>(at.m(e, rank[e]));
        }
    }
#pragma unroll
    for (int e = 0; e < S; ++e)
        if (late[e])
            contrib[e] = load_v<NT, V>(at.pub(e, rank[e]));  // the send buffer of a late process

    // (Issuing the loads and stores one array at a time instead of row by row was measured:
    // no difference.)
#pragma unroll
    for (int e = 0; e < S; ++e) {
        if (busy[e])
            continue;
        const V m_new = fma_v(p.mu, mv[e], gv[e]);
        w_prime[e] = fma_v(-p.lr, m_new, w_prime[e]);  // W'
        store_v<NT, V>(at.m(e, rank[e]), m_new);
        store_v<NT, V>(at.pub(e, rank[e]), w_prime[e]);
        if (!late[e])
            contrib[e] = w_prime[e];
    }
    return tree_sum<S, V>(contrib);
}

template <int S, bool NT, bool LAG, typename V, typename Addr>
__device__ __forceinline__ void rows_average(const StepParams& p, const int32_t* member, const Addr& at,
                                             const V (&w_prime)[S], V w_sum)
{
#pragma unroll
    for (int e = 0; e < S; ++e) {
        const int rank = member[e];
        if (LAG && is_busy(p, rank))
            continue;  // the sum would wait in its receive buffer, unread
        V out;
        if (is_late(p, rank))
            out = (w_sum + w_prime[e]) / p.members_plus_1;
        else
            out = w_sum * p.inv_members;
        store_v<NT, V>(at.w(e, rank), out);
    }
}

// One group of S <= 8 members, all member rows held in registers.  LAG: some members may
// be still computing (is_busy); without it the busy mask is not looked at.
template <int S, bool NT, bool LAG, typename V, typename Addr>
__device__ __forceinline__ void registers_body(const StepParams& p, const int32_t* member, const Addr& at)
{
    bool late[S], busy[S];
    int rank[S];
    V wv[S], gv[S], mv[S], contrib[S];
#pragma unroll
    for (int e = 0; e < S; ++e) {
        rank[e] = member[e];
        late[e] = is_late(p, rank[e]);
        busy[e] = LAG && is_busy(p, rank[e]);
        if (!busy[e]) {
            wv[e] = load_v<NT, V>(at.w(e, rank[e]));
            gv[e] = load_v<NT, V>(at.g(e, rank[e]));
            mv[e] = load_v<NT, V>(at.m(e, rank[e]));
        }
    }
#pragma unroll
    for (int e = 0; e < S; ++e)
        if (late[e])
            contrib[e] = load_v<NT, V>(at.pub(e, rank[e]));  // the send buffer of a late process

    // (Issuing the loads and stores one array at a time instead of row by row was measured:
    // no difference.)
#pragma unroll
    for (int e = 0; e < S; ++e) {
        if (busy[e])
            continue;
        const V m_new = fma_v(p.mu, mv[e], gv[e]);
        wv[e] = fma_v(-p.lr, m_new, wv[e]);  // W'
        store_v<NT, V>(at.m(e, rank[e]), m_new);
        store_v<NT, V>(at.pub(e, rank[e]), wv[e]);
        if (!late[e])
            contrib[e] = wv[e];
    }
    const V w_sum = tree_sum<S, V>(contrib);
#pragma unroll
    for (int e = 0; e < S; ++e) {
        if (busy[e])
            continue;  // the sum would wait in its receive buffer, unread
        V out;
        if (late[e])
            out = (w_sum + wv[e]) / p.members_plus_1;
        else
            out = w_sum * p.inv_members;
        store_v<NT, V>(at.w(e, rank[e]), out);
    }
}

// One group of any size >= 8: member rows streamed a chunk (8 rows, or 4 with LAG) at a time.
template <bool NT, bool LAG, typename V, typename Addr>
__device__ __forceinline__ void streamed_body(const StepParams& p, const int32_t* member, const Addr& at)
{
    constexpr int kChunk = streamed_chunk(LAG);
    constexpr int kStackDepth = streamed_stack_depth(LAG);
    const int chunks = p.members / kChunk;
    V stack[kStackDepth];
    V acc;
    for (int c = 0; c < chunks; ++c) {
        int rank[kChunk];
        bool late[kChunk], busy[kChunk];
        V wv[kChunk], gv[kChunk], mv[kChunk], contrib[kChunk];
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            rank[i] = member[c * kChunk + i];
            late[i] = is_late(p, rank[i]);
            busy[i] = LAG && is_busy(p, rank[i]);
            if (!busy[i]) {
                wv[i] = load_v<NT, V>(at.w(c * kChunk + i, rank[i]));
                gv[i] = load_v<NT, V>(at.g(c * kChunk + i, rank[i]));
                mv[i] = load_v<NT, V>(at.m(c * kChunk + i, rank[i]));
            }
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
            if (late[i]) {
                // An ordinary load: this line is stored to below and read once more in the
                // second pass.  After a non-temporal load the L2 lets go of it early and that
                // last read goes out to memory again (measured: the late rows then cost twice
                // their bytes, and 6 % of the time in the per-tensor layout).
                contrib[i] = load_v<false, V>(at.pub(c * kChunk + i, rank[i]));
            }
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            if (busy[i])
                continue;
            const V m_new = fma_v(p.mu, mv[i], gv[i]);
            wv[i] = fma_v(-p.lr, m_new, wv[i]);
            store_v<NT, V>(at.m(c * kChunk + i, rank[i]), m_new);
            if (late[i]) {
                // read again below: an ordinary store, so that the line may stay in the L2
                store_v<false, V>(at.pub(c * kChunk + i, rank[i]), wv[i]);
            } else {
                store_v<NT, V>(at.pub(c * kChunk + i, rank[i]), wv[i]);
                contrib[i] = wv[i];
            }
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

    // Second pass, a chunk at a time: first the send buffers of the chunk's late members are
    // asked for (W' of such a member: this thread stored it there in the first pass), all of
    // them before any is waited for, then the chunk's rows are stored.
    for (int c = 0; c < chunks; ++c) {
        int rank[kChunk];
        bool late[kChunk], busy[kChunk];
        V w_prime[kChunk];
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            rank[i] = member[c * kChunk + i];
            busy[i] = LAG && is_busy(p, rank[i]);
            late[i] = !busy[i] && is_late(p, rank[i]);
            if (late[i])
                w_prime[i] = load_v<false, V>(at.pub(c * kChunk + i, rank[i]));
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            if (busy[i])
                continue;
            V out = fresh;
            if (late[i])
                out = (w_sum + w_prime[i]) / p.members_plus_1;
            store_v<NT, V>(at.w(c * kChunk + i, rank[i]), out);
        }
    }
}

// Which group and which 16-byte column slice does this lane own?  Workgroups are handed to
// the 8 XCDs round-robin (workgroup b runs on XCD b mod 8) and walk the column tiles of one
// group before the next group's (the chip sweeps one group's rows at a time).  A wavefront
// always owns 64 consecutive slices (1 KiB per row).  The wavefronts of workgroup `tile` sit
// 2^stripe_log2 KiB apart and consecutive workgroups fill the gaps, so that a workgroup's
// simultaneous requests to one row hit addresses one stripe apart (stripe_log2 = 0: the plain
// contiguous tile).  Returns false for lanes and workgroups beyond the end.
constexpr int kBlock = 256;  // threads per workgroup of every step kernel

// Which 16-byte column slice of a row lane `lane` of wavefront `wave` of the workgroup for column
// tile `tile` takes: by the launch shape's map, or by its stripe and XCD run length
// (wagma_shapes.h).
__device__ __forceinline__ int64_t slice_of(const StepParams& p, int64_t tile, int64_t wave, int64_t lane)
{
    if (p.map != 0)
        return wagma_detail::mapped_slice(p.map, tile, wave, lane);
    return wagma_detail::striped_slice(p.stripe_log2, p.xcd_chunk_log2, tile, wave, lane);
}

__device__ __forceinline__ bool decode_block(const StepParams& p, int64_t& group, int64_t& col)
{
    const int64_t b = blockIdx.x;
    if (b >= p.blocks)
        return false;
    group = b / p.tiles;
    static_assert(kBlock == 256, "slice_of deals a tile out to four wavefronts");
    col = slice_of(p, b % p.tiles, threadIdx.x >> 6, threadIdx.x & 63);
    return col < p.nvec;
}

// Resident wavefronts per SIMD the register allocation must allow: the S = 8 body holds 32
// 128-bit values per lane (136 registers: 3 wavefronts), the smaller ones fit 4 and more.
template <int S, bool NT, bool LAG>
__global__ void __launch_bounds__(kBlock, S == 8 ? 2 : 4) step_rows_in_registers(const StepParams p)
{
    int64_t group, col;
    if (!decode_block(p, group, col))
        return;
    const FlatAddr at{p, (uint32_t)col * 4u};
    registers_body<S, NT, LAG, v4f>(p, p.table + group * S, at);
}

template <bool NT, bool LAG>
__global__ void __launch_bounds__(kBlock, 2) step_rows_streamed(const StepParams p)
{
    int64_t group, col;
    if (!decode_block(p, group, col))
        return;
    const FlatAddr at{p, (uint32_t)col * 4u};
    streamed_body<NT, LAG, v4f>(p, p.table + group * p.members, at);
}

// One group of 16, 32 or 64 members, its rows dealt out to the OCTETS = S/8 wavefronts of a
// workgroup, 8 consecutive members each: every wavefront holds its 8 rows in registers exactly as
// the S = 8 kernel does, the sums of the octets meet in LDS and every wavefront adds them up in
// the same order (the pairwise tree over the group is the pairwise tree over its octets' trees),
// so that a late member's W' is still in registers when W is stored.  All wavefronts of a
// workgroup work on the same 64 column slices (1 KiB of every row).  Workgroups b, b+8, b+16, b+24
// (the same XCD) take the four 1 KiB pieces that one workgroup of the other kernels takes.
template <int OCTETS, bool NT, bool LAG>
__global__ void __launch_bounds__(64 * OCTETS, OCTETS <= 4 ? 2 : 1) step_rows_cooperative(const StepParams p)
{
    __shared__ v4f octet_sum[OCTETS][64];
    const int64_t b = blockIdx.x;  // p.blocks = groups * tiles * 4, tiles a multiple of 32
    if (b >= p.blocks)
        return;
    const int64_t per_group = p.tiles * 4;
    const int64_t group = b / per_group;
    const int64_t piece = b % per_group;
    const int octet = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t col = slice_of(p, ((piece >> 5) << 3) | (piece & 7), (piece >> 3) & 3, lane);
    const bool valid = col < p.nvec;  // the same lanes in every wavefront of the workgroup
    const FlatAddr at{p, (uint32_t)col * 4u};
    const int32_t* member = p.table + group * p.members + octet * 8;

    v4f w_prime[8];
    v4f mine = {0.f, 0.f, 0.f, 0.f};
    if (valid)
        mine = rows_update<8, NT, LAG, v4f>(p, member, at, w_prime);
    octet_sum[octet][lane] = mine;
    __syncthreads();  // reached by every wavefront of the workgroup, outside the lanes' branch
    if (!valid)
        return;
    v4f sums[OCTETS];
#pragma unroll
    for (int o = 0; o < OCTETS; ++o)
        sums[o] = octet_sum[o][lane];
    rows_average<8, NT, LAG, v4f>(p, member, at, w_prime, tree_sum<OCTETS, v4f>(sums));
}

// Per-tensor layout.  Workgroup b owns tile b % tiles of group b / tiles; the tile table
// names the tensor, its size and the tile's first 16-byte slice inside it.  A lane whose slice is
// cut off by the end of the tensor does the remaining 1..3 elements one by one; nothing
// beyond a tensor's last element is touched.
template <int S, bool NT, bool LAG, bool AFFINE>
__global__ void __launch_bounds__(kBlock, 2) step_tensors_in_registers(const StepParams p)
{
    const int64_t group = blockIdx.x / p.tiles;
    const TileOf<AFFINE> tile(p, blockIdx.x % p.tiles);
    const TileRef& ref = tile.ref();
    const int64_t size = ref.size;
    const int64_t first = wagma_detail::tensor_slice(p.map, ref, threadIdx.x >> 6, threadIdx.x & 63) * 4;
    if (first >= size)
        return;
    const int32_t* member = p.table + group * S;
    auto at = tile.at(p, member, (uint32_t)first);
    if (first + 4 <= size) {
        registers_body<S, NT, LAG, v4f>(p, member, at);
    } else {
        for (int64_t k = first; k < size; ++k) {
            at.lane_at = (uint32_t)k;
            registers_body<S, NT, LAG, float>(p, member, at);
        }
    }
}

template <bool NT, bool LAG, bool AFFINE>
__global__ void __launch_bounds__(kBlock, 2) step_tensors_streamed(const StepParams p)
{
    const int64_t group = blockIdx.x / p.tiles;
    const TileOf<AFFINE> tile(p, blockIdx.x % p.tiles);
    const TileRef& ref = tile.ref();
    const int64_t size = ref.size;
    const int64_t first = wagma_detail::tensor_slice(p.map, ref, threadIdx.x >> 6, threadIdx.x & 63) * 4;
    if (first >= size)
        return;
    const int32_t* member = p.table + group * p.members;
    auto at = tile.at(p, member, (uint32_t)first);
    if (first + 4 <= size) {
        streamed_body<NT, LAG, v4f>(p, member, at);
    } else {
        for (int64_t k = first; k < size; ++k) {
            at.lane_at = (uint32_t)k;
            streamed_body<NT, LAG, float>(p, member, at);
        }
    }
}

// The per-tensor form of step_rows_cooperative: workgroup b takes one quarter (64 slices, 1 KiB per
// row) of a tile of the tile table; workgroups b, b+8, b+16, b+24 (the same XCD) take the four
// quarters of one tile.  The slice that a tensor's end cuts off is done element by element in up
// to three more rounds; the number of rounds is the same for every wavefront of the workgroup
// (they all work on the same slices), so every wavefront meets every barrier.
template <int OCTETS, bool NT, bool LAG, bool AFFINE>
__global__ void __launch_bounds__(64 * OCTETS, OCTETS <= 4 ? 2 : 1) step_tensors_cooperative(const StepParams p)
{
    __shared__ v4f octet_sum[OCTETS][64];
    __shared__ float octet_sum_1[OCTETS][64];
    const int64_t b = blockIdx.x;  // p.blocks = groups * tiles * 4, tiles a multiple of 8
    if (b >= p.blocks)
        return;
    const int64_t per_group = p.tiles * 4;
    const int64_t group = b / per_group;
    const int64_t piece = b % per_group;
    const TileOf<AFFINE> tile(p, ((piece >> 5) << 3) | (piece & 7));
    const TileRef& ref = tile.ref();
    const int64_t size = ref.size;
    const int64_t quarter = (piece >> 3) & 3;
    // where a contiguous tile's quarter begins; in a mapped block (whole slices only, nothing cut
    // off) the lanes' slices lie apart and only `first` below matters
    const int64_t first_slice = (int64_t)ref.first_slice + quarter * 64;
    if (ref.tile_in_block == 0 && first_slice * 4 >= size)
        return;  // the whole workgroup: this quarter lies beyond the tensor (or the tile is padding)
    const int octet = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t first = wagma_detail::tensor_slice(p.map, ref, quarter, lane) * 4;
    const bool whole = first + 4 <= size;      // the same lanes in every wavefront of the workgroup
    const bool cut = !whole && first < size;   // at most one lane, and only in the tensor's last quarter
    const int32_t* member = p.table + group * p.members + octet * 8;
    {
        const auto at = tile.at(p, member, (uint32_t)first);
        v4f w_prime[8];
        v4f mine = {0.f, 0.f, 0.f, 0.f};
        if (whole)
            mine = rows_update<8, NT, LAG, v4f>(p, member, at, w_prime);
        octet_sum[octet][lane] = mine;
        __syncthreads();
        if (whole) {
            v4f sums[OCTETS];
#pragma unroll
            for (int o = 0; o < OCTETS; ++o)
                sums[o] = octet_sum[o][lane];
            rows_average<8, NT, LAG, v4f>(p, member, at, w_prime, tree_sum<OCTETS, v4f>(sums));
        }
    }
    // the elements of a slice cut off by the tensor's end, if that slice is in this quarter
    const int64_t cut_slice = size / 4;
    const int rounds = (ref.tile_in_block == 0 && size % 4 != 0 && cut_slice >= first_slice && cut_slice < first_slice + 64)
                           ? (int)(size % 4)
                           : 0;
    for (int k = 0; k < rounds; ++k) {
        const auto at = tile.at(p, member, (uint32_t)(first + k));
        float w_prime[8];
        float mine = 0.f;
        if (cut)
            mine = rows_update<8, NT, LAG, float>(p, member, at, w_prime);
        octet_sum_1[octet][lane] = mine;
        __syncthreads();
        if (cut) {
            float sums[OCTETS];
#pragma unroll
            for (int o = 0; o < OCTETS; ++o)
                sums[o] = octet_sum_1[o][lane];
            rows_average<8, NT, LAG, float>(p, member, at, w_prime, tree_sum<OCTETS, float>(sums));
        }
        __syncthreads();  // before the next round writes the sums again
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

}  // namespace

#endif  // WAGMA_KERNELS_H
