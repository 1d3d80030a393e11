// ts_densify: densify an assumed-sparse gradient and add the dense one, on gfx950.
//
// The result is the one defined by arXiv 1905.04035, Section 4 (Listing 1: an
// IndexedSlices gradient becomes a dense tensor) and Section 6 (Algorithm 2, added
// branch: every gradient becomes dense, then they are summed):
//
//     dense_out[v,:] = dense_in[v,:] + sum_{t : ids[t] == v} rows[t,:]
//
// Two launches per call (three when the pairs need more than one sort slice), all on the
// caller's stream, no host synchronisation, no allocation:
//
//   sort_kernel     stable counting sort of the pairs by id.  Work-group (g, s) owns `part`
//                   consecutive ids (128 .. 2048) and slice s of the pairs; its 16
//                   wavefronts load their sub-slices into registers, list the pairs the
//                   work-group owns in LDS, count them into LDS-private tables, an
//                   exclusive scan turns the counts into offsets, and a walk over the
//                   lists hands every owned pair its final position.
//                   A part's first position is the number of pairs with a smaller id,
//                   which the work-group counts itself while it scans, so parts never
//                   wait for one another.  With one slice (up to 57344 pairs) this is a
//                   single launch; with more, a counting launch (count_kernel: one LDS
//                   table per work-group, no lists) fills a [slice][id] table first.
//                   The sort leaves one 32-byte record per sorted pair.
//   reduce_kernel   the HBM-bound kernel.  First the work-groups that add value rows: each
//                   takes four consecutive pieces of C sorted positions (one per wavefront)
//                   and one block of 256 columns.  The pieces of a row with more than C
//                   pairs are added up through LDS by the wavefront that holds the row's
//                   last piece in the work-group.  A row that spans several work-groups
//                   leaves one fp32 share per work-group in scratch; arrival counters tell
//                   the work-group that brings the last share, which adds the shares in a
//                   fixed tree order, adds dense_in and writes the row.  Then work-groups
//                   that take one output row (1024 columns of it, if it is wider) per
//                   wavefront, 16 bytes per lane, streaming:
//                   they copy the rows that received no pair.  Rows with at most C pairs:
//                   in a call with few pairs or narrow rows the wavefront in whose piece such
//                   a row starts finishes it (dense_in + sum straight to dense_out); else
//                   the wavefront that would copy the row adds up its few value rows
//                   instead, and the pieces pass over them; there, with pieces of 16
//                   positions, one wavefront walks the four pieces of a group by itself
//                   and keeps their sums in registers (no LDS, no barrier).  Same order of
//                   additions, same bits in every form.
//
// The sort is a chain of latencies and instructions that moves almost nothing, so a sort of up to six
// slices also carries work-groups that copy dense rows [0, X) and keep HBM busy, before it
// is known which of them receive pairs (the reduce kernel, which runs later, overwrites
// those).  The reduce kernel copies the untouched rows of [X, V).
//
// No floating-point atomics anywhere: the position of every pair, the cut points and
// the order of every addition depend on the ids alone, so results are reproducible
// bit for bit.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <string.h>
#include <type_traits>

#include "ts_densify.h"
#include "ts_densify_tools.h"

// Built-in workspace of ts_densify_static, the entry point for callers that cannot allocate.
// One copy per GPU, held from the moment the library is loaded on it until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress: kernels and
// memory calls are given the device address that call returns (static_scratch() below).
static __device__ __align__(256) unsigned char scratch[TS_STATIC_SCRATCH_BYTES];

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// One sorted pair, as the sort leaves it for the reduce kernel: where its value row is, and
// everything the reduce kernel needs to know about the output row it belongs to.
struct alignas(32) SortedPair {
    uint64_t row_addr;
    int32_t id;
    int32_t pos;        // position of the pair in the input (concatenation order)
    int32_t count;      // pairs of this id
    int32_t row_start;  // sorted position of the id's first pair
    int32_t pad[2];
};
static_assert(sizeof(SortedPair) == 32, "two 16-byte accesses per record");

constexpr int kMaxPart = 2048;     // most ids one sort work-group owns (LDS: 18 x part x 4 B + 8 KiB of lists = 152 KiB)
constexpr int kMinPart = 128;
constexpr int kBigCopyRows = 2;    // rows per wavefront in the copying work-groups of 1024 threads
constexpr int kSortWaves = 16;     // wavefronts per sort work-group
constexpr int kColBlock = 256;     // fp32 columns per wavefront item (64 lanes x 4)
constexpr int kMaxSlices = 64;
constexpr int kSliceTokens = 16384;
constexpr int kFusedSortMax = 57344;   // up to here one launch sorts everything (measured against two launches)
constexpr int kPieceSmallMax = 96256;  // up to here pieces of 16 positions, above 32 (bf16 rows read 16 bytes
                                       // per lane: always 16) -- measured: equal up to 25600 pairs, 16 ahead by
                                       // 1-4 % from 51200 to 131072, 32 ahead by 1 % from 200000; the limit is set
                                       // where a call's workspace (more pieces, more shares) still fits the built-in one

// ------------------------------------------------------------------ device helpers
__device__ __forceinline__ uint64_t ballot64(bool p) { return __ballot(p); }

__device__ __forceinline__ uint32_t lanes_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t bcast(uint32_t x, int lane) { return __builtin_amdgcn_readlane(x, lane); }

__device__ __forceinline__ uint64_t bcast64(uint64_t x, int lane)
{
    uint32_t lo = __builtin_amdgcn_readlane((uint32_t)x, lane);
    uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(x >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// Waits until every vector memory operation of the wavefront has completed (vmcnt = 0, the
// other counters left alone).  The builtin, not an asm statement: the compiler takes note of it.
__device__ __forceinline__ void wait_vm_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Sums across the wavefront with the data-parallel-primitive moves of the vector unit (one
// instruction and a few cycles per step; a shuffle through the LDS crossbar is an LDS instruction with
// its latency, and six of them in a row stand in the sort work-groups' chain).  A wavefront is four
// rows of 16 lanes.  dpp_or_zero: the value of the lane that CTRL names, 0 where there is none or
// where the row is not in ROW_MASK.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xf, true);
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x, int)
{
    x += dpp_or_zero<0x111, 0xf>(x);        // lane - 1 of the row
    x += dpp_or_zero<0x112, 0xf>(x);        // lane - 2
    x += dpp_or_zero<0x114, 0xf>(x);        // lane - 4
    x += dpp_or_zero<0x118, 0xf>(x);        // lane - 8: every row holds its own inclusive scan
    x += dpp_or_zero<0x142, 0xa>(x);        // rows 1 and 3 add the last lane of the row before them
    x += dpp_or_zero<0x143, 0xc>(x);        // rows 2 and 3 add lane 31, the sum of rows 0 and 1
    return x;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x)
{
    return __builtin_amdgcn_readlane(wave_inclusive_scan(x, 0), 63);
}

// Value rows: 4 * NV consecutive columns per lane.  load() brings them as they lie in memory
// (Raw: what stays in registers while the load is in flight), widen() makes fp32 of them.  (The
// address arrives as an integer: say that it is global memory, or the compiler falls back to
// flat loads.)
template <typename RowT, int NV>
struct RowLoad;

template <>
struct RowLoad<float, 1> {
    typedef f4 Raw;
    static __device__ __forceinline__ Raw load(uint64_t row_addr, int col)
    {
        typedef const f4 __attribute__((address_space(1))) * global_f4;
        return __builtin_nontemporal_load(reinterpret_cast<global_f4>(row_addr + (uint64_t)col * 4u));
    }
    static __device__ __forceinline__ void widen(Raw b, f4 (&out)[1]) { out[0] = b; }
};

__device__ __forceinline__ f4 widen_bf16x4(uint32_t lo, uint32_t hi)
{
    f4 r;
    r.x = __uint_as_float(lo << 16);
    r.y = __uint_as_float(lo & 0xFFFF0000u);
    r.z = __uint_as_float(hi << 16);
    r.w = __uint_as_float(hi & 0xFFFF0000u);
    return r;
}

template <>
struct RowLoad<uint16_t, 1> {
    typedef u2 Raw;
    static __device__ __forceinline__ Raw load(uint64_t row_addr, int col)
    {
        typedef const u2 __attribute__((address_space(1))) * global_u2;
        return __builtin_nontemporal_load(reinterpret_cast<global_u2>(row_addr + (uint64_t)col * 2u));
    }
    static __device__ __forceinline__ void widen(Raw b, f4 (&out)[1]) { out[0] = widen_bf16x4(b.x, b.y); }
};

// bf16 rows with d % 8 == 0: one 16-byte load brings eight columns
template <>
struct RowLoad<uint16_t, 2> {
    typedef u4 Raw;
    static __device__ __forceinline__ Raw load(uint64_t row_addr, int col)
    {
        typedef const u4 __attribute__((address_space(1))) * global_u4;
        return __builtin_nontemporal_load(reinterpret_cast<global_u4>(row_addr + (uint64_t)col * 2u));
    }
    static __device__ __forceinline__ void widen(Raw b, f4 (&out)[2])
    {
        out[0] = widen_bf16x4(b.x, b.y);
        out[1] = widen_bf16x4(b.z, b.w);
    }
};


// A partial row that another work-group of the same launch will read: a 16-byte store at
// agent scope, i.e. written through to memory, so that once it has been acknowledged nothing
// of it sits dirty in this work-group's L2 slice.  (The compiler offers that scope for
// 4-byte atomic stores only, and four of those per lane turn every 16-byte store into four
// strided partial writes; hence the instruction is spelled out.)
__device__ __forceinline__ void store_f4_through(float* p, f4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}

// The matching loads: at agent scope, so they are answered from memory and not from a line
// that this L2 slice or this compute unit's cache may still hold from an earlier call.  Eight
// 16-byte loads and the wait for them in ONE statement, so that the compiler never sees a
// loaded register before its data is there.  All eight addresses must be readable.
__device__ __forceinline__ void load8_through(f4 (&x)[8], const float* const (&addr)[8])
{
    asm volatile(
        "global_load_dwordx4 %0, %8, off sc1\n\t"
        "global_load_dwordx4 %1, %9, off sc1\n\t"
        "global_load_dwordx4 %2, %10, off sc1\n\t"
        "global_load_dwordx4 %3, %11, off sc1\n\t"
        "global_load_dwordx4 %4, %12, off sc1\n\t"
        "global_load_dwordx4 %5, %13, off sc1\n\t"
        "global_load_dwordx4 %6, %14, off sc1\n\t"
        "global_load_dwordx4 %7, %15, off sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]), "=&v"(x[7])
        : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "v"(addr[4]), "v"(addr[5]), "v"(addr[6]), "v"(addr[7])
        : "memory");
}

// Streaming accesses for data that is touched once per call (value rows, dense_in,
// dense_out): the nontemporal hint keeps them from displacing the sort's arrays and the
// partial rows in the caches, and measures about 8 % faster on a plain [V, d] copy.
__device__ __forceinline__ f4 load_f4_stream(const float* p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
}
__device__ __forceinline__ void store_f4_stream(float* p, f4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<f4*>(p));
}

// What happens to a finished output row on its way to memory.  EPI_NONE: stored as it is
// (untouched rows are bit copies of dense_in).  EPI_SCALE: every element multiplied by one
// fp32 factor (an average over k contributions is scale = 1/k).  EPI_SCALE_BF16: the same,
// then rounded to bf16 (nearest, ties to even), which halves the bytes written.
enum { EPI_NONE = 0, EPI_SCALE = 1, EPI_SCALE_BF16 = 2 };

__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    const uint32_t b = __float_as_uint(x);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (b >> 16) | 0x0040u;      // NaN stays NaN (quiet)
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// Stores four consecutive output elements starting at element index idx of the output.
template <int EPI>
__device__ __forceinline__ void store_out(void* out, size_t idx, f4 v, float scale)
{
    if (EPI == EPI_NONE) {
        store_f4_stream(reinterpret_cast<float*>(out) + idx, v);
    } else if (EPI == EPI_SCALE) {
        store_f4_stream(reinterpret_cast<float*>(out) + idx, v * scale);
    } else {
        v = v * scale;
        u2 b;
        b.x = bf16_rne(v.x) | (bf16_rne(v.y) << 16);
        b.y = bf16_rne(v.z) | (bf16_rne(v.w) << 16);
        __builtin_nontemporal_store(b, reinterpret_cast<u2*>(reinterpret_cast<uint16_t*>(out) + idx));
    }
}

// One wavefront copies the dense rows v0 .. v0 + R - 1 that lie below vend, except those whose
// bit is set in `skip` (bit r: row v0 + r): all loads of all rows are issued before the first store.
template <int R, int EPI>
__device__ __forceinline__ void copy_rows(const float* dense_in, void* dense_out, uint32_t skip,
                                          int v0, int vend, int d, int lane, float scale)
{
    bool go[R];
    bool any = false;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        go[r] = v0 + r < vend && !((skip >> r) & 1u);
        any = any || go[r];
    }
    if (!any) return;
    for (int c0 = 0; c0 < d; c0 += 4 * kColBlock) {
        f4 x[R][4];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int col = c0 + u * kColBlock + lane * 4;
                x[r][u] = (f4)(0.0f);
                if (go[r] && dense_in && col < d) x[r][u] = load_f4_stream(dense_in + (size_t)(v0 + r) * d + col);
            }
        // With an epilogue every value is transformed before the first store is issued: a
        // multiply placed between two stores makes the compiler wait for the earlier store
        // (the empty asm statements keep it from moving the arithmetic down to the stores).
        u2 packed[R][4];
        if constexpr (EPI != EPI_NONE) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    x[r][u] = x[r][u] * scale;
                    if constexpr (EPI == EPI_SCALE_BF16) {
                        packed[r][u].x = bf16_rne(x[r][u].x) | (bf16_rne(x[r][u].y) << 16);
                        packed[r][u].y = bf16_rne(x[r][u].z) | (bf16_rne(x[r][u].w) << 16);
                        asm volatile("" : "+v"(packed[r][u]));
                    } else {
                        asm volatile("" : "+v"(x[r][u]));
                    }
                }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int col = c0 + u * kColBlock + lane * 4;
                if (go[r] && col < d) {
                    const size_t idx = (size_t)(v0 + r) * d + col;
                    if constexpr (EPI == EPI_SCALE_BF16)
                        __builtin_nontemporal_store(packed[r][u], reinterpret_cast<u2*>(reinterpret_cast<uint16_t*>(dense_out) + idx));
                    else
                        store_f4_stream(reinterpret_cast<float*>(dense_out) + idx, x[r][u]);
                }
            }
    }
}

// One wavefront copies columns [c0, c0 + 1024) of dense row v (the reduce kernel's copy of a row
// that received no pair).  A lane past the row's last column reads the row's last four columns
// again and stores nothing: no load depends on the lane, so the four loads stay back to back.
template <int EPI>
__device__ __forceinline__ void copy_chunk(const float* dense_in, void* dense_out, int v, int c0, int d, int lane,
                                           float scale)
{
    f4 x[4];
    if (dense_in) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            x[u] = load_f4_stream(dense_in + (size_t)v * d + min(c0 + u * kColBlock + lane * 4, d - 4));
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = (f4)(0.0f);
    }
    // every value is transformed before the first store is issued, as in copy_rows
    u2 packed[4];
    if constexpr (EPI != EPI_NONE) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            x[u] = x[u] * scale;
            if constexpr (EPI == EPI_SCALE_BF16) {
                packed[u].x = bf16_rne(x[u].x) | (bf16_rne(x[u].y) << 16);
                packed[u].y = bf16_rne(x[u].z) | (bf16_rne(x[u].w) << 16);
                asm volatile("" : "+v"(packed[u]));
            } else {
                asm volatile("" : "+v"(x[u]));
            }
        }
    }
    // One wait for all loads: the stores sit in blocks of their own (not every lane stores), and the
    // compiler would wait at each of them for everything before it, the store before it included.
    // (In the copies beside the sort, copy_rows, that chain of stores is left as it is: there it
    // measured 0.7-1 us faster per launch, the sort's own loads wait less behind gentler copies.)
    wait_vm_all();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int col = c0 + u * kColBlock + lane * 4;
        if (col < d) {
            const size_t idx = (size_t)v * d + col;
            if constexpr (EPI == EPI_SCALE_BF16)
                __builtin_nontemporal_store(packed[u], reinterpret_cast<u2*>(reinterpret_cast<uint16_t*>(dense_out) + idx));
            else
                store_f4_stream(reinterpret_cast<float*>(dense_out) + idx, x[u]);
        }
    }
}

// ------------------------------------------------------------------ shard table
struct ShardTable {
    int32_t k;
    int32_t off[TS_MAX_SHARDS + 1];          // first global pair index of each shard
    const int32_t* ids[TS_MAX_SHARDS];
    const char* rows[TS_MAX_SHARDS];
};

// Where pair idx lives: its id and the address of its value row.  Only shards j0..j1
// (those that overlap the wavefront's range) are looked at; j0, j1 are wave-uniform.
__device__ __forceinline__ void locate(const ShardTable& sh, int j0, int j1, int idx, bool valid,
                                       int row_bytes, const int32_t*& idp, uint64_t& row_addr)
{
    for (int j = j0; j <= j1; ++j) {
        const int lo = sh.off[j], hi = sh.off[j + 1];
        if (valid && idx >= lo && idx < hi) {
            idp = sh.ids[j] + (idx - lo);
            row_addr = (uint64_t)(uintptr_t)sh.rows[j] + (uint64_t)(idx - lo) * (uint64_t)row_bytes;
        }
    }
}

// ------------------------------------------------------------------ sort
struct SortParams {
    int32_t n, V, G, S, SL;
    // The rows of the call are ids id_base .. id_base + V - 1 of a vocabulary of V_total ids
    // (the whole vocabulary: id_base = 0, V_total = V).  Ids of the vocabulary outside the
    // call's range belong to another owner: skipped, but not counted as bad.
    int32_t id_base, V_total;
    int32_t part;       // ids owned by one work-group (power of two)
    int32_t list_cap;   // entries in a wavefront's list of owned pairs (a multiple of 64, at least 128)
    int32_t row_bytes;
    int32_t* count;
    int32_t* row_start;
    SortedPair* sorted;
    uint32_t* tot;      // [S][G * part]   pairs per (slice, id)
    uint32_t* below;    // [S][G]          pairs of the slice with a valid id below the part
    uint32_t* bad;      // [S]             pairs of the slice with an id outside [0, V)
    int32_t* n_valid;
    int32_t* n_bad;
    int32_t* arrive;    // arrival counters of the reduce kernel, cleared here (arrive_vec 16-byte words)
    int32_t arrive_vec;
    // Work-groups past the sorting ones copy dense rows [copy_row0, copy_row1) to the output
    // without knowing yet which rows receive pairs (the reduce kernel, which runs after,
    // overwrites those).  It keeps HBM busy while the latency-bound sort runs.
    const float* copy_in;
    void* copy_out;
    int32_t copy_row0, copy_row1, d;
    float scale;
};

enum { SORT_FUSED = 0, SORT_SCATTER = 2 };

// One wavefront walks its sub-slice [a, b) in rounds of kRoundTiles tiles of 64 pairs.
// All ids of a round are loaded before any is used, so a round costs one memory
// latency; with a single round (slices of at most 16384 pairs) the ids stay in
// registers between the counting and the ranking pass.
constexpr int kRoundTiles = 16;
constexpr int kRoundPairs = kRoundTiles * 64;

// ids0 / off0 describe shard j0; when the whole range lies in that shard (j0 == j1, the
// common case) no table look-up is needed per tile.
__device__ __forceinline__ void load_round(const ShardTable& sh, int j0, int j1, const int32_t* ids0, int off0,
                                           int a0, int b, int lane, int32_t (&idr)[kRoundTiles])
{
#pragma unroll
    for (int u = 0; u < kRoundTiles; ++u) {
        // lanes past the end re-read the last pair, so that every load is unconditional
        // and all of them are in flight together; such lanes are masked where ids are used
        const int idx = min(a0 + u * 64 + lane, b - 1);
        const int32_t* idp = ids0 + (idx - off0);
        if (j0 != j1) {
            uint64_t unused = 0;
            locate(sh, j0, j1, idx, true, 0, idp, unused);
        }
        idr[u] = *idp;
    }
}

// Walks the tiles of a round and appends the pairs that this work-group owns to the
// wavefront's list, in input order (tiles in order, lanes in order).  An entry is
// (id - lo) << 21 | position of the pair in the wavefront's sub-slice (ids per part <= 2^11,
// pairs per sub-slice <= 2^21).  Every work-group looks at every pair of its slice but owns
// few of them: counting and ranking walk the short list, which is kept from round to round.
// The list holds cap entries (1024 when LDS allows, kListCap otherwise); when the next tile
// might not fit, flush(list, count) consumes what is listed and the list starts again
// (flushed tells the caller that the list no longer holds all owned pairs).  nown is the
// number of entries in the list, before and after.
// With TALLY the pairs with a valid id below the part and those with an id outside [0, V)
// are counted as well (wave-uniform counts).
constexpr int kListCap = 128;
constexpr int kLdsBytes = 160 * 1024;       // LDS of a compute unit, the most a work-group can have

constexpr int kListPosBits = 21;

template <bool TALLY, bool FULL, typename Flush>
__device__ __forceinline__ void own_tiles(const int32_t (&idr)[kRoundTiles], int a0, int b, uint32_t pos0, int lane,
                                          int lo, uint32_t span, uint32_t id_base, uint32_t V_total, uint32_t* list,
                                          uint32_t cap, uint32_t& nown, uint32_t& below, uint32_t& bad,
                                          bool& flushed, Flush&& flush)
{
    // The tallies are kept per lane and added up over the wavefront once per round: a wavefront issues
    // one instruction at a time whatever its kind, and 16 of them share a compute unit here, so the
    // pass is bound by its instruction count (a ballot, a population count and a scalar add per tally
    // and tile cost more than a compare and an add-with-carry per lane).
    uint32_t below_l = 0, bad_l = 0;
#pragma unroll
    for (int u = 0; u < kRoundTiles; ++u) {
        if (FULL || a0 + u * 64 < b) {
            const bool valid = FULL || a0 + u * 64 + lane < b;
            const uint32_t idg = (uint32_t)idr[u];
            const uint32_t id = idg - id_base;          // row of the call; wraps to a huge number below the range
            const uint32_t rel = id - (uint32_t)lo;
            const bool own = valid && rel < span;
            const uint64_t m = ballot64(own);
            if (TALLY) {
                below_l += (valid && id < (uint32_t)lo) ? 1u : 0u;
                bad_l += (valid && idg >= V_total) ? 1u : 0u;
            }
            if (m) {
                if (nown > cap - 64u) {
                    flush(list, nown);
                    nown = 0;
                    flushed = true;
                }
                if (own) list[nown + lanes_below(m)] = (rel << kListPosBits) | (pos0 + (uint32_t)(u * 64 + lane));
                nown += (uint32_t)__popcll(m);
            }
        }
    }
    if (TALLY) {
        below += wave_sum(below_l);
        bad += wave_sum(bad_l);
    }
}

// A round whose 16 tiles are all full (every round but a sub-slice's last) needs no test of the
// lanes against the sub-slice's end.
template <bool TALLY, typename Flush>
__device__ __forceinline__ void own_pairs(const int32_t (&idr)[kRoundTiles], int a0, int b, uint32_t pos0, int lane,
                                          int lo, uint32_t span, uint32_t id_base, uint32_t V_total, uint32_t* list,
                                          uint32_t cap, uint32_t& nown, uint32_t& below, uint32_t& bad,
                                          bool& flushed, Flush&& flush)
{
    if (a0 + kRoundPairs <= b)
        own_tiles<TALLY, true>(idr, a0, b, pos0, lane, lo, span, id_base, V_total, list, cap, nown, below, bad, flushed, flush);
    else
        own_tiles<TALLY, false>(idr, a0, b, pos0, lane, lo, span, id_base, V_total, list, cap, nown, below, bad, flushed, flush);
}

// The counting launch of a sort that takes several slices: work-group (g, s) counts the pairs of
// slice s per id of part g (p.tot), those with a valid id below the part (p.below) and those
// with an id outside the vocabulary (p.bad).  One LDS table for the whole work-group: the order
// of the pairs does not matter here.  It also clears the arrival counters of the reduce kernel,
// and the work-groups past the counting ones copy dense rows like those of sort_kernel.
__global__ __launch_bounds__(1024) void count_kernel(SortParams p, ShardTable sh)
{
    extern __shared__ __align__(16) uint32_t tab[];     // [part]
    __shared__ uint32_t red[2 * kSortWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nsort = p.G * p.S;
    if ((int)blockIdx.x >= nsort) {
        const int cw = (int)blockIdx.x - nsort;
        const int v = p.copy_row0 + (cw * kSortWaves + w) * kBigCopyRows;
        copy_rows<kBigCopyRows, EPI_NONE>(p.copy_in, p.copy_out, 0u, v, p.copy_row1, p.d, lane, p.scale);
        return;
    }
    const int g = (int)blockIdx.x % p.G;
    const int sl = (int)blockIdx.x / p.G;
    const int part = p.part;
    const int lo = g * part;
    const uint32_t span = (uint32_t)min(part, p.V - lo);

    const int t0 = sl * p.SL;
    const int t1 = (int)min((int64_t)p.n, (int64_t)t0 + p.SL);
    const int L = p.SL / kSortWaves;
    const int a = (int)min((int64_t)t1, (int64_t)t0 + (int64_t)w * L);
    const int b = (int)min((int64_t)t1, (int64_t)a + L);
    const int rounds = (b - a + kRoundPairs - 1) / kRoundPairs;
    int j0 = 0;
    while (j0 < sh.k - 1 && sh.off[j0 + 1] <= a) ++j0;
    int j1 = j0;
    while (j1 < sh.k - 1 && sh.off[j1 + 1] < b) ++j1;
    const int32_t* const ids0 = sh.ids[j0];
    const int off0 = sh.off[j0];

    int32_t idr[kRoundTiles];
    if (rounds > 0) load_round(sh, j0, j1, ids0, off0, a, b, lane, idr);
    {
        u4* const z = reinterpret_cast<u4*>(p.arrive);
        for (int i = (int)blockIdx.x * 1024 + tid; i < p.arrive_vec; i += nsort * 1024) z[i] = (u4)(0u);
    }
    for (int i = tid; i < part; i += 1024) tab[i] = 0u;
    __syncthreads();

    uint32_t below = 0, bad = 0;
    // (tallies per lane, full rounds without the test against the sub-slice's end: as in own_tiles)
    uint32_t below_l = 0, bad_l = 0;
    auto count_tiles = [&](auto full_tag, int a0) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int u = 0; u < kRoundTiles; ++u) {
            if (FULL || a0 + u * 64 < b) {
                const bool valid = FULL || a0 + u * 64 + lane < b;
                const uint32_t idg = (uint32_t)idr[u];
                const uint32_t id = idg - (uint32_t)p.id_base;      // row of the call; wraps to a huge number below the range
                // a lane without a pair, or with another part's, holds no id of the part
                const uint32_t rel = (valid && id - (uint32_t)lo < span) ? id - (uint32_t)lo : 0xFFFFFFFFu;
                below_l += (valid && id < (uint32_t)lo) ? 1u : 0u;
                bad_l += (valid && idg >= (uint32_t)p.V_total) ? 1u : 0u;
                const uint64_t m = ballot64(rel != 0xFFFFFFFFu);
                if (m) {
                    // the pairs of the id that the first owning lane holds are counted by that lane
                    // alone (a hot id would otherwise be one LDS atomic per pair), the others one by one
                    const int ll = __builtin_ctzll(m);
                    const uint32_t rl = bcast(rel, ll);
                    const uint64_t sm = ballot64(rel == rl);
                    if (lane == ll) atomicAdd(&tab[rl], (uint32_t)__popcll(sm));
                    if (rel != rl && rel != 0xFFFFFFFFu) atomicAdd(&tab[rel], 1u);
                }
            }
        }
    };
    for (int r = 0; r < rounds; ++r) {
        const int a0 = a + r * kRoundPairs;
        if (r > 0) load_round(sh, j0, j1, ids0, off0, a0, b, lane, idr);
        if (a0 + kRoundPairs <= b)
            count_tiles(std::true_type{}, a0);
        else
            count_tiles(std::false_type{}, a0);
    }
    below += wave_sum(below_l);
    bad += wave_sum(bad_l);
    if (lane == 0) {
        red[w] = below;
        red[kSortWaves + w] = bad;
    }
    __syncthreads();
    const size_t GV = (size_t)p.G * part;
    for (int i = tid; i < part; i += 1024) p.tot[(size_t)sl * GV + lo + i] = tab[i];
    if (tid == 0) {
        uint32_t bl = 0, bd = 0;
#pragma unroll
        for (int ww = 0; ww < kSortWaves; ++ww) {
            bl += red[ww];
            bd += red[kSortWaves + ww];
        }
        p.below[sl * p.G + g] = bl;
        if (g == 0) p.bad[sl] = bd;
    }
}

// The scan phase of sort_kernel for one work-group (see there).  E: consecutive ids per thread.
constexpr uint32_t kSeveral = 0x80000000u;

template <int MODE, int E>
__device__ __forceinline__ void scan_part(const SortParams& p, uint32_t* cnt, uint32_t* id_total, uint32_t* id_start,
                                          uint32_t* wsum, uint32_t base, int part, int lo, uint32_t span, int sl,
                                          int tid, int lane, int w)
{
    typedef uint32_t vec __attribute__((ext_vector_type(E)));
    const int i = tid * E;                  // first of this thread's ids; part is a multiple of E
    const bool idt = i < part;
    vec c[kSortWaves];
    vec total = (vec)(0u), pre = (vec)(0u);
    if (idt) {
#pragma unroll
        for (int ww = 0; ww < kSortWaves; ++ww) {
            c[ww] = *reinterpret_cast<const vec*>(cnt + ww * part + i);
            total += c[ww];
        }
        if (MODE == SORT_SCATTER) {
            total = *reinterpret_cast<const vec*>(id_total + i);     // over all slices, fetched at the start of the kernel
            pre = *reinterpret_cast<const vec*>(id_start + i);
        }
    }
    uint32_t mine = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) mine += total[e];
    const uint32_t incl = wave_inclusive_scan(mine, lane);
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    // what the wavefronts before this one hold: their sums, one per lane, added up
    const uint32_t woff = wave_sum(lane < w ? wsum[lane] : 0u);
    uint32_t rs = base + woff + incl - mine;        // first sorted position of this thread's first id
    if (idt) {
        vec start;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            start[e] = rs;
            if (sl == 0 && (uint32_t)(i + e) < span) {
                p.count[lo + i + e] = (int32_t)total[e];
                p.row_start[lo + i + e] = (int32_t)rs;
                if (lo + i + e == p.V - 1) {
                    p.row_start[p.V] = (int32_t)(rs + total[e]);
                    *p.n_valid = (int32_t)(rs + total[e]);
                }
            }
            rs += total[e];
        }
        *reinterpret_cast<vec*>(id_total + i) = total;
        *reinterpret_cast<vec*>(id_start + i) = start;
        // a wavefront's running position of an id, with kSeveral set if the wavefront holds the id more
        // than once (sorted positions stay below 2^31); the ranking pass only has to work on those
        vec o = start + pre;
#pragma unroll
        for (int ww = 0; ww < kSortWaves; ++ww) {
            vec several;
#pragma unroll
            for (int e = 0; e < E; ++e) several[e] = c[ww][e] > 1u ? kSeveral : 0u;
            *reinterpret_cast<vec*>(cnt + ww * part + i) = o | several;
            o += c[ww];
        }
    }
    __syncthreads();
}

template <int MODE, int EPI>
__global__ __launch_bounds__(1024) void sort_kernel(SortParams p, ShardTable sh)
{
    // [kSortWaves][part] counts, then [2][part] per-id totals and starts, then
    // [kSortWaves][list_cap] lists of owned pairs
    extern __shared__ __align__(16) uint32_t cnt[];
    __shared__ uint32_t red[3 * kSortWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nsort = p.G * p.S;
    if ((int)blockIdx.x >= nsort) {
        const int cw = (int)blockIdx.x - nsort;
        const int v = p.copy_row0 + (cw * kSortWaves + w) * kBigCopyRows;
        copy_rows<kBigCopyRows, EPI>(p.copy_in, p.copy_out, 0u, v, p.copy_row1, p.d, lane, p.scale);
        return;
    }
    const int g = (int)blockIdx.x % p.G;
    const int sl = (int)blockIdx.x / p.G;
    const int part = p.part;
    const int lo = g * part;
    const uint32_t span = (uint32_t)min(part, p.V - lo);
    uint32_t* const mycnt = cnt + w * part;
    uint32_t* const id_total = cnt + kSortWaves * part;
    uint32_t* const id_start = id_total + part;
    uint32_t* const list = id_start + part + w * p.list_cap;

    const int t0 = sl * p.SL;
    const int t1 = (int)min((int64_t)p.n, (int64_t)t0 + p.SL);
    const int L = p.SL / kSortWaves;
    const int a = (int)min((int64_t)t1, (int64_t)t0 + (int64_t)w * L);
    const int b = (int)min((int64_t)t1, (int64_t)a + L);
    const int rounds = (b - a + kRoundPairs - 1) / kRoundPairs;
    int j0 = 0;
    while (j0 < sh.k - 1 && sh.off[j0 + 1] <= a) ++j0;
    int j1 = j0;
    while (j1 < sh.k - 1 && sh.off[j1 + 1] < b) ++j1;

    const int32_t* const ids0 = sh.ids[j0];
    const char* const rows0 = sh.rows[j0];
    const int off0 = sh.off[j0];

    int32_t idr[kRoundTiles];
    if (rounds > 0) load_round(sh, j0, j1, ids0, off0, a, b, lane, idr);

    if (MODE == SORT_FUSED) {
        // the first launch of a call clears the arrival counters of the reduce kernel
        u4* const z = reinterpret_cast<u4*>(p.arrive);
        for (int i = (int)blockIdx.x * 1024 + tid; i < p.arrive_vec; i += nsort * 1024) z[i] = (u4)(0u);
    }

    const size_t GV = (size_t)p.G * part;
    uint32_t base_fetched = 0, nbad_fetched = 0;
    if (MODE == SORT_SCATTER) {
        // Everything the counting launch has left, fetched here so that the latency runs beside
        // the ids'.  Per slice (lane s2 speaks for slice s2, at most 64 slices): the pairs below
        // the part and the bad ids.  Per id (thread tid speaks for ids lo + tid, lo + tid + 1024,
        // ...): its count in all slices and in the slices before this one, sixteen loads in flight
        // at a time, kept where the scan below finds them.  (Measured: issuing more of these loads
        // at once, or issuing them before the tables are cleared, lengthens the launch by 2-3 us.)
        const uint32_t bl = lane < p.S ? p.below[lane * p.G + g] : 0u;
        const uint32_t bd = lane < p.S ? p.bad[lane] : 0u;
        for (int i = tid; i < part; i += 1024) {
            uint32_t total = 0, pre = 0;
            for (int sb = 0; sb < p.S; sb += 16) {
                uint32_t x[16];
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    x[q] = sb + q < p.S ? p.tot[(size_t)(sb + q) * GV + lo + i] : 0u;
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    total += x[q];
                    if (sb + q < sl) pre += x[q];
                }
            }
            id_total[i] = total;
            id_start[i] = pre;
        }
        base_fetched = wave_sum(bl);
        nbad_fetched = wave_sum(bd);
    }
    // every wavefront clears its own table of counts, so none has to wait for the others before it
    // starts to list and count (the tables meet at the barrier before the scan)
    {
        u4* const c4 = reinterpret_cast<u4*>(mycnt);
        for (int i = lane; i < part / 4; i += 64) c4[i] = (u4)(0u);
    }

    // pass 1: list the owned pairs, count them per (wavefront, id); count what lies below the part
    uint32_t below = 0, bad = 0, nown = 0;
    bool flushed = false;
    auto count_listed = [&](const uint32_t* l, uint32_t cnt_l) {
        // the pairs of the id that the first entry holds are counted by one lane (a hot id
        // would otherwise be one LDS atomic per pair, all on one address), the others one by one
        for (uint32_t t0 = 0; t0 < cnt_l; t0 += 64) {
            // a lane without an entry holds no id of the part; ballots of bare comparisons (one of a
            // condition put together from several costs two more vector instructions)
            const uint32_t rel = t0 + lane < cnt_l ? l[t0 + lane] >> kListPosBits : 0xFFFFFFFFu;
            const uint32_t rl = bcast(rel, 0);
            const uint64_t sm = ballot64(rel == rl);
            if (lane == 0) atomicAdd(&mycnt[rl], (uint32_t)__popcll(sm));
            if (rel != rl && rel != 0xFFFFFFFFu) atomicAdd(&mycnt[rel], 1u);
        }
    };
    for (int r = 0; r < rounds; ++r) {
        const int a0 = a + r * kRoundPairs;
        if (r > 0) load_round(sh, j0, j1, ids0, off0, a0, b, lane, idr);
        own_pairs<MODE == SORT_FUSED>(idr, a0, b, (uint32_t)(r * kRoundPairs), lane, lo, span, (uint32_t)p.id_base,
                                      (uint32_t)p.V_total, list, (uint32_t)p.list_cap, nown, below, bad, flushed,
                                      count_listed);
    }
    count_listed(list, nown);
    if (lane == 0) {
        red[w] = below;
        red[kSortWaves + w] = bad;
    }
    __syncthreads();
    // the wavefronts' tallies, one per lane, added up across the wavefront (not 32 reads per thread)
    uint32_t below_wg = 0, bad_wg = 0;
    if (MODE == SORT_FUSED) {
        const uint32_t t = lane < 2 * kSortWaves ? red[lane] : 0u;
        below_wg = wave_sum(lane < kSortWaves ? t : 0u);
        bad_wg = wave_sum(lane < kSortWaves ? 0u : t);
    }

    uint32_t base = below_wg, nbad = bad_wg;       // first sorted position of the part; bad ids
    if (MODE == SORT_SCATTER) {
        base = base_fetched;
        nbad = nbad_fetched;
    }
    if (sl == 0 && g == 0 && tid == 0) *p.n_bad = (int32_t)nbad;

    // The ids of the part in one sweep: thread tid speaks for E = part / 1024 (at least 1)
    // consecutive ids lo + E*tid .., read and written with one LDS access per table (8 bytes
    // when E = 2).  Totals over the wavefronts (and slices), exclusive scan into first
    // positions, running positions per wavefront; each id's count and first position are kept
    // where the ranking pass reads them.
    if (part > 1024) {
        scan_part<MODE, 2>(p, cnt, id_total, id_start, red + 2 * kSortWaves, base, part, lo, span, sl, tid, lane, w);
    } else {
        scan_part<MODE, 1>(p, cnt, id_total, id_start, red + 2 * kSortWaves, base, part, lo, span, sl, tid, lane, w);
    }

    // pass 2: every owned pair takes the next position of its id.  The list keeps the pairs in
    // input order and wavefronts own consecutive sub-slices, so the sort is stable.  Per 64
    // list entries: one LDS read of the running positions, a scalar loop over the distinct
    // ids among them (pairs of one id are ranked by lane), one LDS write by the last lane of
    // each id.  If the owned pairs fitted the list, the list of pass 1 is still there; otherwise
    // the sub-slice is walked again.
    auto rank_listed = [&](const uint32_t* l, uint32_t cnt_l) {
        for (uint32_t e0 = 0; e0 < cnt_l; e0 += 64) {
            const bool own = e0 + lane < cnt_l;
            const uint32_t ent = own ? l[e0 + lane] : 0u;
            const uint32_t rel = ent >> kListPosBits;
            const int idx = a + (int)(ent & ((1u << kListPosBits) - 1u));
            // An id that the wavefront holds once takes the table's position as it is.  Only ids it
            // holds several times (flagged by the scan) go through the loop over distinct ids, which is
            // what this pass spends its time on (13 instructions per distinct id).
            const uint32_t tabv = own ? mycnt[rel] : 0u;
            const uint32_t basev = tabv & ~kSeveral;
            const uint32_t relx = tabv >= kSeveral ? rel : 0xFFFFFFFFu;     // no id to rank: equal to none
            uint64_t m = ballot64(tabv >= kSeveral);
            const uint32_t tot_l = own ? id_total[rel] : 0u;
            const uint32_t rs_l = own ? id_start[rel] : 0u;
            uint32_t pos = basev, next = 0;
            bool leader = false;
            while (m) {
                const int ll = __builtin_ctzll(m);
                const uint32_t rl = bcast(rel, ll);
                const uint64_t sm = ballot64(relx == rl);
                if (relx == rl) pos = basev + lanes_below(sm);
                if (lane == ll) {
                    leader = true;
                    next = (basev + (uint32_t)__popcll(sm)) | kSeveral;
                }
                m &= ~sm;
            }
            if (leader) mycnt[rel] = next;
            // lanes exchange running positions through LDS from one step to the next: the
            // hardware keeps a wavefront's LDS accesses in order, the compiler must too
            asm volatile("" ::: "memory");
            if (own) {
                uint64_t row_addr = (uint64_t)(uintptr_t)rows0 + (uint64_t)(idx - off0) * (uint64_t)p.row_bytes;
                if (j0 != j1) {
                    const int32_t* idp = nullptr;
                    locate(sh, j0, j1, idx, true, p.row_bytes, idp, row_addr);
                }
                u4* rec = reinterpret_cast<u4*>(p.sorted + pos);
                u4 r0, r1;
                r0.x = (uint32_t)row_addr;
                r0.y = (uint32_t)(row_addr >> 32);
                r0.z = (uint32_t)lo + rel;
                r0.w = (uint32_t)idx;
                r1.x = tot_l;
                r1.y = rs_l;
                r1.z = 0u;
                r1.w = 0u;
                rec[0] = r0;
                rec[1] = r1;
            }
        }
    };
    if (!flushed) {
        rank_listed(list, nown);
        return;
    }
    nown = 0;
    for (int r = 0; r < rounds; ++r) {
        const int a0 = a + r * kRoundPairs;
        if (rounds > 1) load_round(sh, j0, j1, ids0, off0, a0, b, lane, idr);
        uint32_t unused0 = 0, unused1 = 0;
        bool unused2 = false;
        own_pairs<false>(idr, a0, b, (uint32_t)(r * kRoundPairs), lane, lo, span, (uint32_t)p.id_base,
                         (uint32_t)p.V_total, list, (uint32_t)p.list_cap, nown, unused0, unused1, unused2, rank_listed);
    }
    rank_listed(list, nown);
}

// ------------------------------------------------------------------ reduce
struct ReduceParams {
    // the first 64 bytes: all that a wavefront which copies a row needs
    int32_t V, d, C, ncb;
    int32_t n_piece_groups;     // work-groups that sum pieces: (groups of kGroupPieces pieces) x column blocks
    int32_t row0;               // the work-groups after them take the rows from here on, one per wavefront
    int32_t short_max;          // rows with at most this many pairs are added up row by row (0 or C)
    int32_t copy_row0;          // untouched rows below this one have been copied by the sort launches
    const int32_t* count;
    const float* dense_in;
    void* dense_out;
    float scale;
    int32_t copy_untouched;     // 0: rows without pairs are left as they are (in place, no epilogue)
    int32_t row_chunks;         // a wavefront of those work-groups takes 1024 columns of a row: chunks per row
    // the rest
    const int32_t* row_start;
    const SortedPair* sorted;
    const int32_t* n_valid;
    int32_t n;                  // pairs in the call (records beyond n_valid hold nothing)
    int32_t nslots;             // 2 * groups
    float* partial;             // [2 * groups][d]: slot 2g holds group g's share of a row that began before it,
                                // slot 2g + 1 its share of a row that begins in it and goes on beyond it
    int32_t* arrive;            // [levels][2 * groups][ncb] arrival counters, all zero when the launch starts
    int32_t logC, logG;         // log2 C; log2 of the sorted positions of a group of pieces
};

constexpr int kGroupPieces = 4;     // pieces per work-group of the reduce kernel, one per wavefront
constexpr int kLogGroupPieces = 2;

// Fixed-order combine of a row that spans several work-groups, inside the launch that made
// the shares (a share: what one work-group's pieces hold of the row, already added up in
// piece order).  The shares of a row form a tree with a fan-in of 16: share j of a level belongs
// to group j / 16, and a group's sum is itself share j / 16 of the next level, until one
// group holds the whole row.  Every wavefront that has stored a share counts itself in at
// the share's group; the one that finds all the others there adds the group's shares in a
// fixed order (a batch at a time as a balanced tree, the batches in order), stores the sum
// in the slot of the group's first share and moves up a level; at the top dense_in is
// added and the output row is written.  Which wavefront does the adding depends on timing,
// what it adds and in which order does not.
//
// Ordering without a release fence (which writes the whole L2 back and costs more than the
// rest of the kernel) and without an acquire fence (which empties this L2 slice for
// everybody): shares are stored through to memory (store_f4_through); a wavefront counts
// itself in only after those stores have been acknowledged; the wavefront that sees the
// full count reads the shares from memory (load8_through), past its caches.
constexpr int kFanIn = 16;
constexpr int kLogFanIn = 4;

// A share this wavefront has stored: that of group k (of pieces) of the cut row `id`, whose
// c pairs start at sorted position s.
struct CutRef {
    int32_t k, id, s, c;
};

// k0: the group in which the row begins.
__device__ __forceinline__ size_t share_slot(int k0, int group_in_row)
{
    return group_in_row == 0 ? (size_t)(2 * k0 + 1) : (size_t)2 * (size_t)(k0 + group_in_row);
}

__device__ __forceinline__ int32_t* arrival_counter(const ReduceParams& p, int level, size_t first_slot, int cb)
{
    return p.arrive + ((size_t)level * p.nslots + first_slot) * p.ncb + cb;
}

// Counts a level-0 share in.  The caller has made sure that the share's stores are
// acknowledged.  Returns (in lane 0) how many shares of the group had arrived before.
__device__ __forceinline__ int announce_share(const ReduceParams& p, const CutRef& r, int cb, int lane)
{
    const int k0 = r.s >> p.logG;
    const int g = (r.k - k0) >> kLogFanIn;
    int arrived = 0;
    if (lane == 0)
        arrived = __hip_atomic_fetch_add(arrival_counter(p, 0, share_slot(k0, g << kLogFanIn), cb), 1, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    return arrived;
}

// arrived0: what announce_share returned for this share.  If the share was its group's
// last, adds the group up and climbs the tree for as long as it is the last to arrive.
template <int NV, int EPI>
__device__ __forceinline__ void combine_if_last(const ReduceParams& p, const CutRef& r, int cb, int col, bool colok,
                                                int lane, int arrived0)
{
    constexpr int kBatch = 8 / NV;                  // shares loaded together: eight 16-byte loads
    const int k0 = r.s >> p.logG;                                     // the row's first group of pieces
    int Pl = ((r.s + r.c - 1) >> p.logG) - k0 + 1;                    // shares at this level (groups at level 0)
    int j = r.k - k0;                                                 // this wavefront's share
    int shift = 0;                                                    // a share of this level spans 16^level groups
    int arrived = __builtin_amdgcn_readfirstlane(arrived0);
    for (int level = 0;; ++level) {
        const int g = j >> kLogFanIn;
        const int m = min(kFanIn, Pl - (g << kLogFanIn));             // shares in this group
        const size_t first_slot = share_slot(k0, (g << kLogFanIn) << shift);
        const bool top = Pl <= kFanIn;
        if (level > 0) {
            // the group sum stored below has to be in memory before it is counted in
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            int x = 0;
            if (lane == 0)
                x = __hip_atomic_fetch_add(arrival_counter(p, level, first_slot, cb), 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
            arrived = __builtin_amdgcn_readfirstlane(x);
        }
        if (arrived != m - 1) return;
        f4 dn[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) {
            dn[q] = (f4)(0.0f);
            if (top && colok && p.dense_in) dn[q] = load_f4_stream(p.dense_in + (size_t)r.id * p.d + col + 4 * q);
        }
        f4 tot[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) tot[q] = (f4)(0.0f);
        // lanes past the row's last column read column 0 and drop it; shares past the group's
        // last read the last one again and drop it: every load is to an address that exists
        const int safe_col = colok ? col : 0;
        for (int i0 = 0; i0 < m; i0 += kBatch) {
            f4 x[8];                    // share u of the batch, vector q: x[u * NV + q]
            const float* addr[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int i = min(i0 + t / NV, m - 1);
                addr[t] = p.partial + share_slot(k0, ((g << kLogFanIn) + i) << shift) * p.d + safe_col + 4 * (t % NV);
            }
            load8_through(x, addr);
#pragma unroll
            for (int t = 0; t < 8; ++t) x[t] = (i0 + t / NV < m && colok) ? x[t] : (f4)(0.0f);
#pragma unroll
            for (int w = 1; w < kBatch; w <<= 1)
#pragma unroll
                for (int u = 0; u + w < kBatch; u += 2 * w)
#pragma unroll
                    for (int q = 0; q < NV; ++q) x[u * NV + q] += x[(u + w) * NV + q];
#pragma unroll
            for (int q = 0; q < NV; ++q) tot[q] += x[q];
        }
        if (top) {
            if (colok) {
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    if constexpr (EPI == EPI_NONE)
                        store_f4_stream(reinterpret_cast<float*>(p.dense_out) + (size_t)r.id * p.d + col + 4 * q,
                                        tot[q] + dn[q]);
                    else
                        store_out<EPI>(p.dense_out, (size_t)r.id * p.d + col + 4 * q, tot[q] + dn[q], p.scale);
                }
            }
            return;
        }
        if (colok) {
#pragma unroll
            for (int q = 0; q < NV; ++q) store_f4_through(p.partial + first_slot * p.d + col + 4 * q, tot[q]);
        }
        j = g;
        Pl = (Pl + kFanIn - 1) >> kLogFanIn;
        shift += kLogFanIn;
    }
}

// Columns [c0, c0 + 1024) of one output row v, by one wavefront, when rows with at most short_max
// (> 0) pairs are added up row by row.  A row that received no pair is copied from dense_in, unless
// that has been done or is not wanted; of a row that received at most short_max pairs, the
// value rows are added up in sorted order and dense_in last.  (Longer rows belong to the
// pieces.)  dense_in is asked for before the row's count is known whenever it will most
// likely be needed: all but the few long rows need it then.
template <typename RowT, int EPI>
__device__ __forceinline__ void short_row(const ReduceParams& p, int v, int c0, int lane)
{
    const bool copy = p.copy_untouched && v >= p.copy_row0;    // what to do if the row received no pair
    const bool early = copy;                                   // then only a long row makes the early load useless
    constexpr int RB = sizeof(RowT) == 4 ? 4 : 8;      // value rows in flight together (16 KiB; 8 KiB measured 2 % slower
                                                       // where short rows have up to 32 pairs)
    typedef typename RowLoad<RowT, 1>::Raw Raw;
    const int d = p.d;
    f4 dn[4];
    // a lane past the row's last column reads the last four columns again (and stores nothing), so
    // that no load depends on the lane
    auto load_dense = [&](int c0) {
        if (p.dense_in) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                dn[u] = load_f4_stream(p.dense_in + (size_t)v * d + min(c0 + u * kColBlock + lane * 4, d - 4));
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) dn[u] = (f4)(0.0f);
        }
    };
    if (early) load_dense(c0);
    const int c = p.count[v];
    if (c > p.short_max || (c == 0 && !copy)) return;
    uint64_t addr = 0;
    if (lane < c) addr = p.sorted[p.row_start[v] + lane].row_addr;
    if (!early) load_dense(c0);
    if (c > 0) {
        f4 acc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] = (f4)(0.0f);
        for (int j0 = 0; j0 < c; j0 += RB) {
            Raw raw[RB][4];
#pragma unroll
            for (int t = 0; t < RB; ++t) {
                const uint64_t ra = bcast64(addr, min(j0 + t, c - 1));
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int col = min(c0 + u * kColBlock + lane * 4, d - 4);
                    raw[t][u] = Raw{};
                    if (j0 + t < c) raw[t][u] = RowLoad<RowT, 1>::load(ra, col);
                }
            }
#pragma unroll
            for (int t = 0; t < RB; ++t) {
                if (j0 + t < c) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        f4 r[1];
                        RowLoad<RowT, 1>::widen(raw[t][u], r);
                        acc[u] = acc[u] + r[0];
                    }
                }
            }
        }
        // dense_in has been in flight all along; the output row takes its place
#pragma unroll
        for (int u = 0; u < 4; ++u) dn[u] = acc[u] + dn[u];
    }
    // one wait for all that is still on its way, then the stores back to back
    wait_vm_all();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int col = c0 + u * kColBlock + lane * 4;
        if (col < d) store_out<EPI>(p.dense_out, (size_t)v * d + col, dn[u], p.scale);
    }
}

// Where short rows are added up row by row, the long rows are added up by wavefronts that
// work alone: one wavefront takes a whole group of kGroupPieces pieces (4C sorted positions)
// and one block of columns, walks the pieces one after the other and keeps in registers
// what the work-group form keeps in LDS.  The sums are the same, in the same order: a piece's
// pairs in sorted order, the pieces of the group in order; a row that lies inside the group is
// finished there, of any other the group's sum becomes a share.  No barrier, no LDS, and a
// wavefront that has to wait for its share to be acknowledged, or to combine shares, holds up
// nobody but itself.  For groups of at most 64 sorted positions (C <= 16): one per lane.
template <typename RowT, int NV, int EPI>
__device__ __forceinline__ void group_wave(const ReduceParams& p, int kg, int cb, int lane)
{
    typedef typename RowLoad<RowT, NV>::Raw Raw;
    constexpr int BATCH = 16;                   // value rows in flight together
    constexpr int NW = 1;                       // windows of 64 sorted positions
    const int C = p.C;
    const int G = C << kLogGroupPieces;          // sorted positions of the group (at most 64)
    const int gpos0 = kg << p.logG;
    const int col = (cb * kColBlock + lane * 4) * NV;
    const bool colok = col < p.d;
    const bool have_dense = p.dense_in != nullptr;

    // lane j of window w looks at sorted position gpos0 + 64 w + j; records are read before
    // n_valid is known, what lies at or beyond it is ignored
    u4 r0[NW], r1[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int jr = w * 64 + lane;
        r0[w] = (u4)(0u);
        r1[w] = (u4)(0u);
        if (jr < G && gpos0 + jr < p.n) {
            const u4* rec = reinterpret_cast<const u4*>(p.sorted + gpos0 + jr);
            r0[w] = rec[0];
            r1[w] = rec[1];
        }
    }
    const int nvalid = *p.n_valid;
    int32_t id[NW], c[NW], s[NW];
    uint64_t addr[NW];
    uint64_t L[NW], RS[NW], RE[NW];             // positions of long rows; where such a row starts; where it ends
    uint64_t INSIDE[NW];                        // positions of rows that start inside the group
    bool any = false;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int jr = w * 64 + lane;
        const int wpos = gpos0 + jr;
        const bool inwin = jr < G && wpos < p.n && wpos < nvalid;
        id[w] = inwin ? (int32_t)r0[w].z : -1;
        c[w] = inwin ? (int32_t)r1[w].x : 0;
        s[w] = inwin ? (int32_t)r1[w].y : 0;
        addr[w] = inwin ? (((uint64_t)r0[w].y << 32) | r0[w].x) : 0ull;
        const bool lng = inwin && c[w] > C;
        L[w] = ballot64(lng);
        RS[w] = ballot64(lng && wpos == s[w]);
        RE[w] = ballot64(lng && wpos == s[w] + c[w] - 1);
        INSIDE[w] = ballot64(lng && s[w] >= gpos0);
        any = any || L[w] != 0;
    }
    if (!any) return;
    const uint64_t PS = ballot64((lane & (C - 1)) == 0);            // first and last position of a piece
    const uint64_t PE = ballot64((lane & (C - 1)) == C - 1);        // (C divides 64)

    f4 acc[NV], tot[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) acc[q] = tot[q] = (f4)(0.0f);
    bool segfirst = true;       // the piece at hand is the first of its row within the group
    CutRef ref[2];
    ref[0].k = ref[1].k = -1;
    int nref = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        uint64_t rem = L[w];
        while (rem) {
            // the next BATCH positions of long rows: all loads are issued before the first is used
            int jj[BATCH];
            Raw raw[BATCH];
            f4 dn[2][NV];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q = 0; q < NV; ++q) dn[t][q] = (f4)(0.0f);
            static_assert(BATCH == 16, "two slots, one per 8 positions");
            // dense_in of a row that is finished here: one slot and one load instruction per half of
            // the batch, issued behind the half's value rows.  A long row has more than 8 pairs, so
            // no two of them end within 8 positions of long rows.  (Several conditional loads into
            // one slot, or a slot chosen at run time, make the compiler load into a spare register
            // and move the value afterwards, with a wait for it and for all loads before it.)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint64_t half = 0;
#pragma unroll
                for (int uu = 0; uu < 8; ++uu) {
                    const int u = 8 * h + uu;
                    jj[u] = -1;
                    raw[u] = Raw{};
                    if (rem) {
                        const int j = (int)__builtin_ctzll(rem);
                        rem &= rem - 1ull;
                        half |= 1ull << j;
                        jj[u] = j;
                        if (colok) raw[u] = RowLoad<RowT, NV>::load(bcast64(addr[w], j), col);
                    }
                }
                const uint64_t ends = half & RE[w] & INSIDE[w];
                if (have_dense && ends && colok) {
                    const int vj = (int)bcast((uint32_t)id[w], (int)__builtin_ctzll(ends));
#pragma unroll
                    for (int q = 0; q < NV; ++q) dn[h][q] = load_f4_stream(p.dense_in + (size_t)vj * p.d + col + 4 * q);
                }
            }
            // one wait for the whole batch: the compiler waits for all of it at the first use anyway, and
            // would then wait again at every later position, which after a row's store means for that store
            wait_vm_all();
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int j = jj[u];
                if (j >= 0) {
                    const bool rs = (RS[w] >> j) & 1ull, re = (RE[w] >> j) & 1ull;
                    const bool ps = (PS >> j) & 1ull, pe = (PE >> j) & 1ull;
                    const bool fresh = rs || ps;
                    if (fresh) segfirst = rs || (w == 0 && j == 0);
                    f4 r[NV];
                    RowLoad<RowT, NV>::widen(raw[u], r);
#pragma unroll
                    for (int q = 0; q < NV; ++q) acc[q] = (fresh ? (f4)(0.0f) : acc[q]) + r[q];
                    if (re || pe) {
                        // the row's pairs in this piece are in: the pieces of the group in order
#pragma unroll
                        for (int q = 0; q < NV; ++q) tot[q] = segfirst ? acc[q] : tot[q] + acc[q];
                        segfirst = false;
                        const bool gend = w * 64 + j == G - 1;
                        if (re || gend) {
                            const int sj = (int)bcast((uint32_t)s[w], j);
                            const int cj = (int)bcast((uint32_t)c[w], j);
                            const int idj = (int)bcast((uint32_t)id[w], j);
                            if (re && sj >= gpos0) {
                                // the row lies inside the group
                                f4 dj[NV];
#pragma unroll
                                for (int q = 0; q < NV; ++q) dj[q] = have_dense ? dn[u >> 3][q] : (f4)(0.0f);
                                if (colok) {
#pragma unroll
                                    for (int q = 0; q < NV; ++q)
                                        store_out<EPI>(p.dense_out, (size_t)idj * p.d + col + 4 * q, tot[q] + dj[q], p.scale);
                                }
                            } else {
                                // the group's share of a row that began before it or goes on beyond it
                                const int kg0 = (sj >> p.logC) >> kLogGroupPieces;
                                const size_t slot = share_slot(kg0, kg - kg0);
                                if (colok) {
#pragma unroll
                                    for (int q = 0; q < NV; ++q) store_f4_through(p.partial + slot * p.d + col + 4 * q, tot[q]);
                                }
                                CutRef x;
                                x.k = kg;
                                x.id = idj;
                                x.s = sj;
                                x.c = cj;
                                if (nref == 0) ref[0] = x; else ref[1] = x;
                                ++nref;
                            }
                        }
                    }
                }
            }
        }
    }
    if (nref == 0) return;
    // shares are counted in once their stores are acknowledged; whoever brings the last share
    // of a group of shares adds the group up
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int answer[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) answer[t] = ref[t].k >= 0 ? announce_share(p, ref[t], cb, lane) : 0;
#pragma unroll
    for (int t = 0; t < 2; ++t)
        if (ref[t].k >= 0) combine_if_last<NV, EPI>(p, ref[t], cb, col, colok, lane, answer[t]);
}

// NV: 16-byte fp32 vectors per lane (a wavefront of a piece covers 256 * NV columns); BATCH:
// sorted positions whose rows are loaded together.
//
// Output rows with more than C pairs are added up by pieces.  A work-group takes kGroupPieces
// consecutive pieces of C sorted positions, one per wavefront, and one block of columns.  A
// wavefront adds up the pairs of such a row that lie in its piece and leaves the sum in LDS.
// After one barrier the wavefront that holds a row's last piece within the work-group adds
// the work-group's pieces of that row in piece order; if the row lies inside the work-group it
// is finished there and then, otherwise the sum goes to scratch as the work-group's share of
// the row, and the shares are combined as described above.
//
// Output rows with at most C pairs, SHORT = 0: the wavefront in whose piece such a row
// starts adds it up completely (its window is two pieces long for that) and writes
// dense_in + sum; the work-groups after those of the pieces copy the rows without pairs, one
// per wavefront.  SHORT = 1 or 2: those work-groups take every row that is not long, one per
// wavefront (short_row), and the pieces pass over the positions of short rows; with
// SHORT = 1 (pieces of at most 16 positions) the long rows go to wavefronts that work alone
// (group_wave) instead of the work-groups described here.  The order of additions, and so
// every bit of the result, is the same in all three.
template <typename RowT, int NV, int BATCH, int EPI, int SHORT>
__global__ __launch_bounds__(256) void reduce_kernel(ReduceParams p)
{
    // SHORT: 0 short rows in the pieces; 1 row by row, long rows by lone wavefronts (group_wave);
    // 2 row by row, long rows by the work-groups below
    // [wavefront][0: of a row that began before the piece, 1: of a row that begins in it][vector][lane]
    __shared__ f4 chain[SHORT == 1 ? 1 : kGroupPieces][2][NV][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if ((int)blockIdx.x >= p.n_piece_groups) {
        // one wavefront per row and chunk of 1024 columns (wider rows: several wavefronts, so that
        // no wavefront has to work through its row chunk after chunk)
        const int item = ((int)blockIdx.x - p.n_piece_groups) * kGroupPieces + wave;
        int v = p.row0 + item, c0 = 0;
        if (p.row_chunks > 1) {
            const int r = item / p.row_chunks;
            v = p.row0 + r;
            c0 = (item - r * p.row_chunks) * 4 * kColBlock;
        }
        if constexpr (!SHORT) {
            // the pieces add up every row that received pairs: copy the row if it received none
            if (v < p.V && p.count[v] == 0) copy_chunk<EPI>(p.dense_in, p.dense_out, v, c0, p.d, lane, p.scale);
        } else {
            if (v < p.V) short_row<RowT, EPI>(p, v, c0, lane);
        }
        return;
    }

    if constexpr (SHORT == 1) {
        // Four wavefronts, four consecutive groups of pieces, one block of columns.  Work-groups b, b + 8,
        // b + 16, ... run on the same XCD (one of eight, each with an L2 of its own): the column blocks of
        // one quadruple of groups go to work-groups of one XCD, which then reads the quadruple's records
        // from memory once.  Quadruples beyond a multiple of eight keep the plain order.  (Measured: 0.6-1.2 %
        // of the call at 50-130 thousand pairs; the same mapping for the work-group form of the pieces
        // changed nothing or cost 0.5 %, and giving an XCD 16 consecutive rows in the row work-groups
        // cost 1.5-4 us: consecutive rows are better spread over the XCDs, as they are.)
        const int b = (int)blockIdx.x;
        const int nq = p.n_piece_groups / p.ncb;
        int kq, cb;
        if (b < (nq & ~7) * p.ncb) {
            const int i = b >> 3;
            const int q = i / p.ncb;
            cb = i - q * p.ncb;
            kq = q * 8 + (b & 7);
        } else {
            kq = b / p.ncb;
            cb = b - kq * p.ncb;
        }
        const int kg = kq * 4 + wave;
        if (kg < p.nslots / 2) group_wave<RowT, NV, EPI>(p, kg, cb, lane);
        return;
    }

    // ---- piece k: sorted positions [pos0, pos0 + C), columns [cb*256*NV, (cb+1)*256*NV)
    const int kg = (int)blockIdx.x / p.ncb;
    const int cb = (int)blockIdx.x - kg * p.ncb;
    const int k = kg * kGroupPieces + wave;
    const int col = (cb * kColBlock + lane * 4) * NV;
    const bool colok = col < p.d;
    const int C = p.C;
    const int pos0 = k * C;

    // lane j looks at sorted position pos0 + j; the window is two pieces long because
    // an output row with at most C pairs that starts in this piece is finished here (unless
    // such rows are added up row by row: then the piece itself is all there is to look at).  The records are read before n_valid is known (one
    // memory latency instead of two); what lies at or beyond n_valid is ignored.
    const int wpos = pos0 + lane;
    const bool inarr = lane < (SHORT ? C : 2 * C) && wpos < p.n;
    u4 r0 = (u4)(0u), r1 = (u4)(0u);
    if (inarr) {
        const u4* rec = reinterpret_cast<const u4*>(p.sorted + wpos);
        r0 = rec[0];
        r1 = rec[1];
    }
    const int nvalid = *p.n_valid;
    const bool inwin = inarr && wpos < nvalid;
    const int32_t id = inwin ? (int32_t)r0.z : -1;
    const int32_t c = inwin ? (int32_t)r1.x : 0;
    const int32_t s = inwin ? (int32_t)r1.y : 0;
    const uint64_t addr = inwin ? (((uint64_t)r0.y << 32) | r0.x) : 0ull;
    const bool whole = c <= C;       // output row small enough to be summed by one wavefront
    const bool active = inwin && (whole ? (!SHORT && s >= pos0 && s < pos0 + C) : (lane < C));
    const bool first = active && (wpos == s || (!whole && lane == 0));
    const bool last = active && (wpos == s + c - 1 || (!whole && lane == C - 1));
    const uint64_t A = ballot64(active);
    const uint64_t F = ballot64(first);
    const uint64_t Lm = ballot64(last);
    const uint64_t W = ballot64(whole);
    const uint64_t H = ballot64(s >= pos0);      // the row of this position begins in this piece
    const bool have_dense = p.dense_in != nullptr;

    if (A != 0) {
        typedef typename RowLoad<RowT, NV>::Raw Raw;
        f4 acc[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) acc[q] = (f4)(0.0f);
        // The active positions are consecutive, or (when short rows are added up elsewhere) lie in
        // two runs: the end of one long row and the beginning of another.
        uint64_t rem = A;
        while (rem) {
            const int a = (int)__builtin_ctzll(rem);
            int b = 64 - __builtin_clzll(rem);
            if constexpr (SHORT) {
                const uint64_t gap = ~(rem >> a);
                b = a + (gap ? (int)__builtin_ctzll(gap) : 64 - a);
            }
            rem &= b < 64 ? ~0ull << b : 0ull;
            for (int base = a; base < b; base += BATCH) {
                // all loads of a batch are issued before the first is used
                Raw raw[BATCH];
                f4 dn[BATCH][NV];
#pragma unroll
                for (int u = 0; u < BATCH; ++u) {
                    const int j = base + u;
                    raw[u] = Raw{};
#pragma unroll
                    for (int q = 0; q < NV; ++q) dn[u][q] = (f4)(0.0f);
                    if (j < b) {
                        if (colok) raw[u] = RowLoad<RowT, NV>::load(bcast64(addr, j), col);
                        if (have_dense && (((Lm & W) >> j) & 1ull)) {
                            const int vj = (int)bcast((uint32_t)id, j);
                            if (colok) {
#pragma unroll
                                for (int q = 0; q < NV; ++q)
                                    dn[u][q] = load_f4_stream(p.dense_in + (size_t)vj * p.d + col + 4 * q);
                            }
                        }
                    }
                }
                // (where only long rows are left to the pieces, the compiler's code waits before every
                // position for all memory operations, a finished row's store included: one wait instead)
                if constexpr (SHORT != 0) wait_vm_all();
#pragma unroll
                for (int u = 0; u < BATCH; ++u) {
                    const int j = base + u;
                    if (j < b) {
                        const bool fresh = (F >> j) & 1ull;
                        f4 r[NV];
                        RowLoad<RowT, NV>::widen(raw[u], r);
#pragma unroll
                        for (int q = 0; q < NV; ++q) acc[q] = (fresh ? (f4)(0.0f) : acc[q]) + r[q];
                        if ((Lm >> j) & 1ull) {
                            if ((W >> j) & 1ull) {
                                const int vj = (int)bcast((uint32_t)id, j);
                                if (colok) {
#pragma unroll
                                    for (int q = 0; q < NV; ++q)
                                        store_out<EPI>(p.dense_out, (size_t)vj * p.d + col + 4 * q, acc[q] + dn[u][q], p.scale);
                                }
                            } else {
                                const int portion = (int)((H >> j) & 1ull);
#pragma unroll
                                for (int q = 0; q < NV; ++q) chain[wave][portion][q][lane] = acc[q];
                            }
                        }
                    }
                }
            }
        }
    }
    __syncthreads();

    // The cut rows that pass through this piece (at most two: one that ends in it or covers
    // it, one that begins in it).  The wavefront with the row's last piece inside the
    // work-group adds the work-group's pieces of the row, in piece order.
    uint64_t cuts = Lm & ~W;
    const int g_first = kg * kGroupPieces, g_last = g_first + kGroupPieces - 1;
    CutRef ref[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        ref[t].k = -1;
        if (cuts) {
            const int j = __builtin_ctzll(cuts);
            cuts &= cuts - 1;
            const int idj = (int)bcast((uint32_t)id, j);
            const int sj = (int)bcast((uint32_t)s, j);
            const int cj = (int)bcast((uint32_t)c, j);
            const int piece_first = sj >> p.logC, piece_last = (sj + cj - 1) >> p.logC;
            if (k == min(piece_last, g_last)) {
                const bool inside = piece_first >= g_first && piece_last <= g_last;
                f4 dn[NV];
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    dn[q] = (f4)(0.0f);
                    if (inside && have_dense && colok) dn[q] = load_f4_stream(p.dense_in + (size_t)idj * p.d + col + 4 * q);
                }
                const int x0 = max(piece_first, g_first);
                f4 tot[NV];
#pragma unroll
                for (int q = 0; q < NV; ++q) tot[q] = chain[x0 - g_first][x0 == piece_first ? 1 : 0][q][lane];
                for (int x = x0 + 1; x <= k; ++x) {
#pragma unroll
                    for (int q = 0; q < NV; ++q) tot[q] += chain[x - g_first][0][q][lane];
                }
                if (inside) {
                    if (colok) {
#pragma unroll
                        for (int q = 0; q < NV; ++q) {
                            if constexpr (EPI == EPI_NONE)
                                store_f4_stream(reinterpret_cast<float*>(p.dense_out) + (size_t)idj * p.d + col + 4 * q,
                                                tot[q] + dn[q]);
                            else
                                store_out<EPI>(p.dense_out, (size_t)idj * p.d + col + 4 * q, tot[q] + dn[q], p.scale);
                        }
                    }
                } else {
                    // the work-group's share of a row that goes beyond it
                    const int kg0 = piece_first >> kLogGroupPieces;
                    const size_t slot = share_slot(kg0, kg - kg0);
                    if (colok) {
#pragma unroll
                        for (int q = 0; q < NV; ++q) store_f4_through(p.partial + slot * p.d + col + 4 * q, tot[q]);
                    }
                    ref[t].k = kg;
                    ref[t].id = idj;
                    ref[t].s = sj;
                    ref[t].c = cj;
                }
            }
        }
    }
    if (ref[0].k < 0 && ref[1].k < 0) return;
    // shares are counted in once their stores are acknowledged; whoever brings the last share
    // of a group of shares adds the group up
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int answer[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) answer[t] = ref[t].k >= 0 ? announce_share(p, ref[t], cb, lane) : 0;
#pragma unroll
    for (int t = 0; t < 2; ++t)
        if (ref[t].k >= 0) combine_if_last<NV, EPI>(p, ref[t], cb, col, colok, lane, answer[t]);
}

// ------------------------------------------------------------------ unique ids (introspection)
__global__ __launch_bounds__(1024) void unique_kernel(const int32_t* count, int V, int32_t* out,
                                                      int32_t* n_out)
{
    __shared__ uint32_t wsum[kSortWaves];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    uint32_t base = 0;
    for (int v0 = 0; v0 < V; v0 += 1024) {
        const int v = v0 + tid;
        const bool flag = v < V && count[v] > 0;
        const uint64_t m = ballot64(flag);
        if (lane == 0) wsum[w] = (uint32_t)__popcll(m);
        __syncthreads();
        uint32_t woff = 0, tot = 0;
        for (int ww = 0; ww < kSortWaves; ++ww) {
            if (ww < w) woff += wsum[ww];
            tot += wsum[ww];
        }
        if (flag) out[base + woff + lanes_below(m)] = v;
        base += tot;
        __syncthreads();
    }
    if (tid == 0) *n_out = (int32_t)base;
}

// ------------------------------------------------------------------ host side
struct Plan {
    int32_t S, SL, G, part, list_cap, C, NB, NBG, levels, ncb;   // NB pieces in NBG groups   // ncb: 256-column blocks of a row; levels of the combine tree
    size_t off_nvalid, off_nbad, off_arrive, arrive_bytes, off_count, off_row_start, off_sorted, off_tot,
        off_below, off_bad, off_partial, total;
};

int g_piece_override = 0;
int32_t g_short_rows = -1;       // -1: choose; 0: the pieces take the short rows along; 1: row by row
int64_t g_overlap_sort = -1;            // dense bytes (read + write) copied beside each sort launch; -1 = default
int32_t g_part_override = 0;
void* g_ws = nullptr;
int64_t g_ws_bytes = 0;
Plan g_last_plan;
void* g_last_ws = nullptr;              // the workspace the most recent call used (bound, or the built-in one)
int32_t g_last_V = 0;
int32_t g_last_info[8] = {0, 0, 0, 0, 0, 0, 0, 0};
bool g_have_last = false;

constexpr int kMaxProfile = 4096;
hipEvent_t g_ev[2 * kMaxProfile];
int g_ev_made = 0;
int g_prof_cap = 0;
int g_prof_used = 0;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Calls with at least this many pairs add up their short rows row by row, the others in the pieces.
// Row by row a wavefront has one output row's few value rows in flight, all columns of them, after
// three loads that depend on each other; in the pieces it has up to eight pairs of 256 (bf16: 512)
// columns in flight, and every block of columns repeats the bookkeeping.  So the wider the rows and
// the more pairs, the better the first does.  Measured on V = 8192 .. 131072, Zipf ids: narrower than
// 256 columns it never pays (half-empty wavefronts), at 256 from about 400 thousand pairs (2 %), at 512
// from 65 to 100 thousand, at 1024 from 25 thousand (bf16 rows, 6-13 % by 50 thousand) or 40-50
// thousand (fp32 rows, 0.5-5 %), and from there on the limit halves when the width doubles (d = 4096:
// 8 to 16 thousand; 3-10 % beyond); below those it loses up to 30 % on narrow rows and small V.
// A dense operand of half a gigabyte or more (V = 131072 at d = 1024): row by row at any number of pairs
// (2-5 % measured from 8192 pairs on; the launch is so long that what row-by-row costs at its start and
// end no longer counts).
int64_t short_rows_from(int32_t d, int32_t V, bool bf16)
{
    if (d < 256) return INT64_MAX;
    if (d < 512) return 393216;
    if (d < 1024) return 65536;
    if ((int64_t)V * d >= ((int64_t)128 << 20)) return 0;
    return (int64_t)(bf16 ? 24576 : 40960) * 1024 / d;
}

int piece_tokens_for(int64_t n, bool wide_bf16)
{
    if (g_piece_override) return g_piece_override;
    return (wide_bf16 || n <= kPieceSmallMax) ? 16 : 32;
}

// bound: size the arrays that depend on how the sort is split (slices, parts) for the largest
// split any call of at most n pairs and at most V rows can choose, so that the total never
// shrinks when n or V grows.
void make_plan(int64_t n, int32_t d, int32_t V, int32_t C, Plan* pl, bool bound = false)
{
    if (n <= kFusedSortMax) {
        pl->S = 1;
        pl->SL = (int32_t)align_up((size_t)(n > 0 ? n : 1), 1024);
    } else {
        int64_t SL = kSliceTokens;
        int64_t S = (n + SL - 1) / SL;
        if (S > kMaxSlices) {
            SL = (int64_t)align_up((size_t)((n + kMaxSlices - 1) / kMaxSlices), 1024);
            S = (n + SL - 1) / SL;
        }
        pl->S = (int32_t)S;
        pl->SL = (int32_t)SL;
    }
    // ids per sort work-group: smaller parts shorten the sort (fewer owned pairs per
    // work-group), but every sorting work-group holds half of a compute unit and slows the
    // copy that runs beside it; about 64 work-groups per slice measured best
    // (with several slices every part looks at every slice, and that dominates: the largest
    // parts that still give every compute unit a work-group)
    int part = (pl->S > 1 && (int64_t)((V + kMaxPart - 1) / kMaxPart) * pl->S >= 256) ? kMaxPart : 1024;
    while (pl->S == 1 && part > kMinPart && (int64_t)((V + part - 1) / part) < 64) part >>= 1;
    if (g_part_override) part = g_part_override;
    pl->part = part;
    // a list that holds a whole round never has to be rebuilt; parts of 2048 ids leave room
    // for short lists only
    pl->list_cap = part <= 1024 ? kRoundPairs : kListCap;
    // One launch that walks several rounds: a wavefront whose work-group owns more of its pairs than the
    // list holds (a dominating id) would have to walk its share a second time to rank them; give the
    // lists what the LDS has left, up to the wavefront's whole share.
    if (pl->S == 1 && n > (int64_t)kSortWaves * kRoundPairs && part <= 1024) {
        const int64_t share = (pl->SL / kSortWaves + 63) / 64 * 64;
        const int64_t room = (kLdsBytes - 256 - (int64_t)(kSortWaves + 2) * part * 4) / (kSortWaves * 4) / 64 * 64;
        const int64_t cap = share < room ? share : room;
        if (cap > pl->list_cap) pl->list_cap = (int32_t)cap;
    }
    pl->G = (V + part - 1) / part;
    pl->C = C;
    pl->NB = (int32_t)((n + pl->C - 1) / pl->C);
    // a work-group of the reduce kernel takes kGroupPieces pieces; the shares of a row that spans several
    // work-groups are added up in a tree with a fan-in of 16: levels needed for a row that spans them all
    pl->NBG = (pl->NB + kGroupPieces - 1) / kGroupPieces;
    pl->levels = 1;
    for (int64_t reach = kFanIn; reach < pl->NBG; reach *= kFanIn) ++pl->levels;
    pl->ncb = (d + kColBlock - 1) / kColBlock;
    size_t o = 0;
    pl->off_nvalid = o;
    pl->off_nbad = o + 4;
    o = 256;
    pl->off_arrive = o;
    pl->arrive_bytes = align_up((size_t)pl->levels * 2 * pl->NBG * pl->ncb * 4, 256);
    o += pl->arrive_bytes;
    pl->off_count = o;
    o = align_up(o + (size_t)V * 4, 256);
    pl->off_row_start = o;
    o = align_up(o + ((size_t)V + 1) * 4, 256);
    pl->off_sorted = o;
    o = align_up(o + (size_t)n * sizeof(SortedPair), 256);
    size_t S_tab = pl->S > 1 ? (size_t)pl->S : 0, ids_tab = (size_t)pl->G * pl->part, G_tab = (size_t)pl->G;
    if (bound && n > kFusedSortMax) {
        const size_t s16 = (size_t)((n + kSliceTokens - 1) / kSliceTokens);
        S_tab = s16 < (size_t)kMaxSlices ? s16 : (size_t)kMaxSlices;
        ids_tab = align_up((size_t)V, kMaxPart);
        G_tab = ((size_t)V + 63) / 64;
    }
    pl->off_tot = o;
    if (S_tab) o = align_up(o + S_tab * ids_tab * 4, 256);
    pl->off_below = o;
    if (S_tab) o = align_up(o + S_tab * G_tab * 4, 256);
    pl->off_bad = o;
    if (S_tab) o = align_up(o + S_tab * 4, 256);
    pl->off_partial = o;
    o = align_up(o + (size_t)2 * pl->NBG * (size_t)d * 4, 256);
    pl->total = o;
}

int check_hip(hipError_t e) { return e == hipSuccess ? TS_OK : TS_ERR_HIP; }

// Compute units of the current GPU (asked once per device; 0 if the question fails, which
// only switches a tuning rule off).
int compute_units()
{
    static int cached[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = -1;
        cached[dev] = n;
    }
    return cached[dev] > 0 ? cached[dev] : 0;
}

// Device address of the built-in workspace on the current GPU: every GPU holds its own copy
// of the array at its own address, looked up once per device and kept.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TS_ERR_HIP;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TS_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TS_OK;
}

// The three kinds of launches, one instantiation per epilogue (the epilogue is a template
// argument so that the plain path keeps its code).
template <int EPI>
void launch_sort_fused(dim3 grid, size_t lds, hipStream_t stream, const SortParams& sp, const ShardTable& sh)
{
    hipLaunchKernelGGL((sort_kernel<SORT_FUSED, EPI>), grid, dim3(1024), lds, stream, sp, sh);
}

// With events (benchmarks only) the launch goes through the variant that stamps them with the
// kernel's own begin and end, so that their difference is the kernel's duration.
template <typename Kernel>
void launch_timed(Kernel kernel, unsigned grid, hipStream_t stream, hipEvent_t begin, hipEvent_t end,
                  const ReduceParams& rp)
{
    if (begin)
        hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, stream, begin, end, 0, rp);
    else
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, stream, rp);
}

template <int EPI, int SHORT>
void launch_reduce_as(unsigned grid, bool wide, int32_t row_dtype, hipStream_t stream, hipEvent_t begin,
                      hipEvent_t end, const ReduceParams& rp)
{
    if (wide)
        launch_timed(reduce_kernel<uint16_t, 2, 4, EPI, SHORT>, grid, stream, begin, end, rp);
    else if (row_dtype == TS_ROW_BF16)
        launch_timed(reduce_kernel<uint16_t, 1, 8, EPI, SHORT>, grid, stream, begin, end, rp);
    else
        launch_timed(reduce_kernel<float, 1, 8, EPI, SHORT>, grid, stream, begin, end, rp);
}

template <int EPI>
void launch_reduce(unsigned grid, bool wide, int32_t row_dtype, hipStream_t stream, hipEvent_t begin,
                   hipEvent_t end, const ReduceParams& rp)
{
    // short rows row by row: long rows by lone wavefronts where a group of pieces fits the lanes of one
    if (rp.short_max > 0 && kGroupPieces * rp.C > 64)
        launch_reduce_as<EPI, 2>(grid, wide, row_dtype, stream, begin, end, rp);
    else if (rp.short_max > 0)
        launch_reduce_as<EPI, 1>(grid, wide, row_dtype, stream, begin, end, rp);
    else
        launch_reduce_as<EPI, 0>(grid, wide, row_dtype, stream, begin, end, rp);
}

#define TS_DISPATCH_EPI(epi, fn, ...)                              \
    do {                                                           \
        if ((epi) == EPI_NONE) fn<EPI_NONE>(__VA_ARGS__);          \
        else if ((epi) == EPI_SCALE) fn<EPI_SCALE>(__VA_ARGS__);   \
        else fn<EPI_SCALE_BF16>(__VA_ARGS__);                      \
    } while (0)

// V rows are produced: ids id_base .. id_base + V - 1 of a vocabulary of V_total ids.
int densify_impl(const ShardTable& sh, int64_t n, int32_t row_dtype, int32_t d, int32_t V, int32_t id_base,
                 int32_t V_total, const float* dense_in, void* dense_out, int epi, float scale, void* stream_v,
                 void* ws_v, int64_t ws_bytes)
{
    const bool wide = row_dtype == TS_ROW_BF16 && (d % 8) == 0;     // 16-byte loads of bf16 rows
    Plan pl;
    make_plan(n, d, V, piece_tokens_for(n, wide), &pl);
    if (!ws_v || (int64_t)pl.total > ws_bytes) return TS_ERR_WORKSPACE;
    if ((int64_t)pl.NB * pl.ncb + (int64_t)V * ((d + 4 * kColBlock - 1) / (4 * kColBlock)) >= ((int64_t)1 << 31) - 8)
        return TS_ERR_OVERFLOW;
    hipStream_t stream = (hipStream_t)stream_v;
    char* ws = (char*)ws_v;

    SortParams sp;
    sp.n = (int32_t)n;
    sp.V = V;
    sp.id_base = id_base;
    sp.V_total = V_total;
    sp.G = pl.G;
    sp.S = pl.S;
    sp.SL = pl.SL;
    sp.part = pl.part;
    sp.row_bytes = d * (row_dtype == TS_ROW_BF16 ? 2 : 4);
    sp.count = (int32_t*)(ws + pl.off_count);
    sp.row_start = (int32_t*)(ws + pl.off_row_start);
    sp.sorted = (SortedPair*)(ws + pl.off_sorted);
    sp.tot = (uint32_t*)(ws + pl.off_tot);
    sp.below = (uint32_t*)(ws + pl.off_below);
    sp.bad = (uint32_t*)(ws + pl.off_bad);
    sp.n_valid = (int32_t*)(ws + pl.off_nvalid);
    sp.n_bad = (int32_t*)(ws + pl.off_nbad);
    sp.arrive = (int32_t*)(ws + pl.off_arrive);
    sp.arrive_vec = (int32_t)(pl.arrive_bytes / 16);

    // In place, the plain path leaves untouched rows alone.  With an epilogue they still have
    // to be scaled, by the item that reads them; only the copy made before the pairs are
    // sorted must go, because the reduce kernel would read scaled values.
    const bool in_place = (const void*)dense_in == (const void*)dense_out;
    const bool skip_untouched = in_place && epi == EPI_NONE;
    // Rows copied by the sort launches: about as many bytes as HBM moves while a sort runs
    // (measured defaults).  One slice: 32 MiB plus 1 MiB per 1024 pairs up to 16384 pairs, 2.5 MiB
    // per 1024 pairs beyond (the wavefronts then walk their shares in several rounds).  A sort
    // of a few slices leaves compute units idle, and a smaller blind copy beside
    // each of its two launches still pays (+4 % at 3-4 slices); a sort of many slices keeps the
    // whole GPU busy by itself (a copying work-group beside every sorting one lengthens the sort
    // by more than the copy is worth), and with that many pairs a large share of the rows
    // copied blindly would be overwritten: no blind copy then.
    const int64_t budget_single = n <= 16384 ? (32ll << 20) + (n / 1024 << 20)
                                             : (48ll << 20) + (n - 16384) / 1024 * (5ll << 19);
    const int64_t budget_multi = pl.S <= 4 ? (32ll << 20) : (pl.S <= 6 ? (16ll << 20) : 0);
    const int64_t budget = g_overlap_sort >= 0 ? g_overlap_sort
                                               : (pl.S == 1 ? budget_single : budget_multi);
    int64_t rows_per_launch = (in_place || (pl.S > 1 && epi != EPI_NONE)) ? 0 : budget / ((int64_t)8 * d);
    rows_per_launch = rows_per_launch / (kBigCopyRows * kSortWaves) * (kBigCopyRows * kSortWaves);
    // A work-group of these launches holds a compute unit (1024 threads, most of the LDS).  Where the
    // default budget comes to a little less than one work-group per compute unit in all, make it exactly
    // one: fewer leave compute units idle, and a few more than one leave a second round of stragglers
    // (measured on 256 compute units, d = 1024: 192 copying work-groups beside 64 sorting ones take
    // 2048-12800 pairs 1-2 % faster than 136-178 do, and 208 cost 1.5 us more than 192 at 16384 pairs).
    if (pl.S == 1 && g_overlap_sort < 0 && rows_per_launch > 0) {
        const int64_t cus = compute_units();
        const int64_t wg_rows = kBigCopyRows * kSortWaves;
        const int64_t all = pl.G + rows_per_launch / wg_rows;
        if (cus > pl.G && 4 * all >= 3 * cus && all < cus) rows_per_launch = (cus - pl.G) * wg_rows;
    }
    const int32_t tail0 = V;
    int32_t copy_done = 0;
    auto sort_grid = [&](SortParams& q) {
        q.copy_row0 = copy_done;
        q.copy_row1 = (int32_t)(copy_done + rows_per_launch < tail0 ? copy_done + rows_per_launch : tail0);
        copy_done = q.copy_row1;
        return dim3((unsigned)(pl.G * pl.S + (q.copy_row1 - q.copy_row0 + kBigCopyRows * kSortWaves - 1) / (kBigCopyRows * kSortWaves)));
    };
    sp.copy_in = dense_in;
    sp.copy_out = dense_out;
    sp.d = d;
    sp.scale = scale;
    sp.list_cap = pl.list_cap;
    const size_t lds = ((size_t)(kSortWaves + 2) * pl.part + (size_t)kSortWaves * sp.list_cap) * sizeof(uint32_t);
    if (pl.S == 1) {
        const dim3 g1 = sort_grid(sp);
        TS_DISPATCH_EPI(epi, launch_sort_fused, g1, lds, stream, sp, sh);
    } else {
        const dim3 g1 = sort_grid(sp);
        hipLaunchKernelGGL(count_kernel, g1, dim3(1024), (size_t)pl.part * sizeof(uint32_t), stream, sp, sh);
        const dim3 g2 = sort_grid(sp);
        hipLaunchKernelGGL((sort_kernel<SORT_SCATTER, EPI_NONE>), g2, dim3(1024), lds, stream, sp, sh);
    }
    if (hipGetLastError() != hipSuccess) return TS_ERR_HIP;

    ReduceParams rp;
    rp.V = V;
    rp.d = d;
    rp.C = pl.C;
    rp.ncb = wide ? (d + 2 * kColBlock - 1) / (2 * kColBlock) : pl.ncb;
    rp.n_piece_groups = pl.NBG * rp.ncb;
    rp.count = sp.count;
    rp.sorted = sp.sorted;
    rp.n = (int32_t)n;
    rp.n_valid = sp.n_valid;
    rp.dense_in = dense_in;
    rp.dense_out = dense_out;
    rp.scale = scale;
    rp.partial = (float*)(ws + pl.off_partial);
    rp.arrive = sp.arrive;
    rp.nslots = 2 * pl.NBG;
    rp.logC = __builtin_ctz((unsigned)pl.C);
    rp.logG = rp.logC + kLogGroupPieces;
    rp.copy_row0 = copy_done;
    rp.copy_untouched = skip_untouched ? 0 : 1;
    rp.row_start = sp.row_start;
    // Output rows with at most C pairs: with many pairs in the call they are added up row by row, by the
    // wavefronts that would otherwise copy the row; with few, the pieces take them along.
    rp.short_max = (g_short_rows < 0 ? n >= short_rows_from(d, V, row_dtype == TS_ROW_BF16) : g_short_rows == 1) ? pl.C : 0;
    // ... and, with pieces of at most 16 positions, their long rows by wavefronts that work alone, four groups
    // of pieces to a work-group
    if (rp.short_max > 0 && kGroupPieces * pl.C <= 64) rp.n_piece_groups = (pl.NBG + 3) / 4 * rp.ncb;
    // after the work-groups of the pieces, one wavefront for every output row that may need one
    rp.row0 = rp.short_max > 0 ? 0 : (skip_untouched ? V : copy_done);
    rp.row_chunks = (d + 4 * kColBlock - 1) / (4 * kColBlock);
    const unsigned rgrid = (unsigned)(rp.n_piece_groups + ((int64_t)(V - rp.row0) * rp.row_chunks + kGroupPieces - 1) / kGroupPieces);

    const bool prof = g_prof_used < g_prof_cap && rgrid > 0;
    hipEvent_t ev_begin = prof ? g_ev[2 * g_prof_used] : nullptr;
    hipEvent_t ev_end = prof ? g_ev[2 * g_prof_used + 1] : nullptr;
    if (rgrid > 0) TS_DISPATCH_EPI(epi, launch_reduce, rgrid, wide, row_dtype, stream, ev_begin, ev_end, rp);
    if (prof) ++g_prof_used;
    if (hipGetLastError() != hipSuccess) return TS_ERR_HIP;

    g_last_plan = pl;
    g_last_ws = ws_v;
    g_last_V = V;
    g_last_info[0] = pl.C;
    g_last_info[1] = copy_done;
    g_last_info[2] = tail0;
    g_last_info[3] = pl.S;
    g_last_info[4] = pl.part;
    g_last_info[5] = pl.NB;
    g_last_info[6] = pl.levels;
    // bit 0: in place; bits 1-2: how short rows were added up (0 in the pieces, 1 row by row with the long
    // rows by lone wavefronts, 2 row by row with the long rows by work-groups)
    g_last_info[7] = (in_place ? 1 : 0) | ((rp.short_max == 0 ? 0 : (kGroupPieces * rp.C <= 64 ? 1 : 2)) << 1);
    g_have_last = true;
    return TS_OK;
}

int validate_common(int64_t n_total, int32_t d, int32_t V, const float* dense_in, const void* dense_out)
{
    if (!dense_out) return TS_ERR_NULL;
    if (n_total < 0 || V <= 0 || d <= 0 || (d % 4) != 0) return TS_ERR_SHAPE;
    if (n_total >= ((int64_t)1 << 31)) return TS_ERR_OVERFLOW;
    if (((uintptr_t)dense_out & 15u) || ((uintptr_t)dense_in & 15u)) return TS_ERR_ALIGN;
    return TS_OK;
}

int densify_shards(const int32_t* const* ids_k, const void* const* rows_k, const int64_t* n_k, int32_t k,
                   int32_t row_dtype, int32_t d, int32_t V, const float* dense_in, void* dense_out, int epi,
                   float scale, void* stream, int32_t v_begin = 0, int32_t v_end = -1, void* ws = nullptr,
                   int64_t ws_bytes = -1)
{
    if (ws_bytes < 0) {         // the bound workspace
        ws = g_ws;
        ws_bytes = g_ws_bytes;
    }
    if (v_end < 0) v_end = V;
    if (V <= 0 || v_begin < 0 || v_begin >= v_end || v_end > V) return TS_ERR_SHAPE;
    if (k < 1 || k > TS_MAX_SHARDS) return TS_ERR_SHAPE;
    if (row_dtype != TS_ROW_FP32 && row_dtype != TS_ROW_BF16) return TS_ERR_SHAPE;
    if (!ids_k || !rows_k || !n_k) return TS_ERR_NULL;
    int64_t n_total = 0;
    for (int j = 0; j < k; ++j) {
        if (n_k[j] < 0) return TS_ERR_SHAPE;
        n_total += n_k[j];
        if (n_total >= ((int64_t)1 << 31)) return TS_ERR_OVERFLOW;
    }
    int rc = validate_common(n_total, d, v_end - v_begin, dense_in, dense_out);
    if (rc != TS_OK) return rc;
    ShardTable sh;
    memset(&sh, 0, sizeof sh);
    sh.k = k;
    int64_t off = 0;
    for (int j = 0; j < k; ++j) {
        if (n_k[j] > 0 && (!ids_k[j] || !rows_k[j])) return TS_ERR_NULL;
        if ((uintptr_t)rows_k[j] & 15u) return TS_ERR_ALIGN;
        if ((uintptr_t)ids_k[j] & 3u) return TS_ERR_ALIGN;
        sh.off[j] = (int32_t)off;
        sh.ids[j] = ids_k[j];
        sh.rows[j] = (const char*)rows_k[j];
        off += n_k[j];
    }
    for (int j = k; j <= TS_MAX_SHARDS; ++j) sh.off[j] = (int32_t)off;
    return densify_impl(sh, n_total, row_dtype, d, v_end - v_begin, v_begin, V, dense_in, dense_out, epi, scale, stream,
                        ws, ws_bytes);
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

int ts_densify(const int32_t* ids, const float* rows, int64_t n, int32_t d, int32_t V,
               const float* dense_in, float* dense_out, void* stream)
{
    const void* r = rows;
    return densify_shards(&ids, &r, &n, 1, TS_ROW_FP32, d, V, dense_in, dense_out, EPI_NONE, 1.0f, stream);
}

int ts_densify_static(const int32_t* ids, const float* rows, int64_t n, int32_t d, int32_t V,
                      const float* dense_in, float* dense_out, void* stream)
{
    // the size check comes first: a call that does not fit touches nothing, not even the device
    if (n < 0 || V <= 0 || d <= 0 || (d % 4) != 0) return TS_ERR_SHAPE;
    if (n >= ((int64_t)1 << 31)) return TS_ERR_OVERFLOW;
    Plan pl;
    make_plan(n, d, V, piece_tokens_for(n, false), &pl);
    if ((int64_t)pl.total > (int64_t)TS_STATIC_SCRATCH_BYTES) return TS_ERR_CAPACITY;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != TS_OK) return rc;
    const void* r = rows;
    return densify_shards(&ids, &r, &n, 1, TS_ROW_FP32, d, V, dense_in, dense_out, EPI_NONE, 1.0f, stream, 0, -1, ws,
                          (int64_t)TS_STATIC_SCRATCH_BYTES);
}

int ts_densify_bf16(const int32_t* ids, const uint16_t* rows, int64_t n, int32_t d, int32_t V,
                    const float* dense_in, float* dense_out, void* stream)
{
    const void* r = rows;
    return densify_shards(&ids, &r, &n, 1, TS_ROW_BF16, d, V, dense_in, dense_out, EPI_NONE, 1.0f, stream);
}

int ts_densify_multi(const int32_t* const* ids_k, const void* const* rows_k, const int64_t* n_k,
                     int32_t k, int32_t row_dtype, int32_t d, int32_t V, const float* dense_in,
                     float* dense_out, void* stream)
{
    return densify_shards(ids_k, rows_k, n_k, k, row_dtype, d, V, dense_in, dense_out, EPI_NONE, 1.0f, stream);
}

int ts_densify_scaled(const int32_t* const* ids_k, const void* const* rows_k, const int64_t* n_k,
                      int32_t k, int32_t row_dtype, int32_t d, int32_t V, const float* dense_in,
                      void* out, int32_t out_dtype, float scale, void* stream)
{
    if (out_dtype != TS_OUT_FP32 && out_dtype != TS_OUT_BF16) return TS_ERR_SHAPE;
    if (!(scale - scale == 0.0f)) return TS_ERR_SHAPE;                  // infinite or NaN
    if (out_dtype == TS_OUT_BF16 && out && (const void*)dense_in == out) return TS_ERR_SHAPE;
    const int epi = out_dtype == TS_OUT_BF16 ? EPI_SCALE_BF16 : (scale == 1.0f ? EPI_NONE : EPI_SCALE);
    return densify_shards(ids_k, rows_k, n_k, k, row_dtype, d, V, dense_in, out, epi, scale, stream);
}

int ts_densify_range(const int32_t* const* ids_k, const void* const* rows_k, const int64_t* n_k,
                     int32_t k, int32_t row_dtype, int32_t d, int32_t V, int32_t v_begin, int32_t v_end,
                     const float* dense_in, float* dense_out, void* stream)
{
    if (v_end < 0) return TS_ERR_SHAPE;
    return densify_shards(ids_k, rows_k, n_k, k, row_dtype, d, V, dense_in, dense_out, EPI_NONE, 1.0f, stream,
                          v_begin, v_end);
}

int ts_fusion_place(int64_t capacity_bytes, int64_t used_bytes, int32_t d, int32_t V, int32_t out_dtype,
                    int64_t* offset_bytes, int64_t* used_after_bytes)
{
    if (!offset_bytes || !used_after_bytes) return TS_ERR_NULL;
    if (capacity_bytes < 0 || used_bytes < 0 || d <= 0 || V <= 0) return TS_ERR_SHAPE;
    if (out_dtype != TS_OUT_FP32 && out_dtype != TS_OUT_BF16) return TS_ERR_SHAPE;
    int64_t bytes, start, end;
    if (__builtin_mul_overflow((int64_t)V, (int64_t)d, &bytes) ||
        __builtin_mul_overflow(bytes, (int64_t)(out_dtype == TS_OUT_BF16 ? 2 : 4), &bytes) ||
        __builtin_add_overflow(used_bytes, (int64_t)255, &start))
        return TS_ERR_OVERFLOW;
    start = start / 256 * 256;
    if (__builtin_add_overflow(start, bytes, &end)) return TS_ERR_OVERFLOW;
    if (end > capacity_bytes) return TS_ERR_CAPACITY;
    *offset_bytes = start;
    *used_after_bytes = end;
    return TS_OK;
}

int ts_buffer_bytes(int64_t k, int64_t N, int32_t d, int32_t V, int32_t row_dtype, int64_t* gathered_bytes,
                    int64_t* dense_bytes)
{
    if (!gathered_bytes || !dense_bytes) return TS_ERR_NULL;
    if (k < 0 || N < 0 || d <= 0 || V <= 0) return TS_ERR_SHAPE;
    if (row_dtype != TS_ROW_FP32 && row_dtype != TS_ROW_BF16) return TS_ERR_SHAPE;
    const int64_t elem = row_dtype == TS_ROW_BF16 ? 2 : 4;
    int64_t per_slice, kn, g, dn;
    if (__builtin_mul_overflow(elem, (int64_t)d, &per_slice) || __builtin_add_overflow(per_slice, (int64_t)4, &per_slice) ||
        __builtin_mul_overflow(k, N, &kn) || __builtin_mul_overflow(kn, per_slice, &g) ||
        __builtin_mul_overflow((int64_t)4 * V, (int64_t)d, &dn))
        return TS_ERR_OVERFLOW;
    *gathered_bytes = g;
    *dense_bytes = dn;
    return TS_OK;
}

int ts_workspace_bytes(int64_t n_total, int32_t d, int32_t V, int64_t* bytes)
{
    if (!bytes) return TS_ERR_NULL;
    if (n_total < 0 || V <= 0 || d <= 0 || (d % 4) != 0) return TS_ERR_SHAPE;
    if (n_total >= ((int64_t)1 << 31)) return TS_ERR_OVERFLOW;
    // the smallest pieces a call of this size can use: the most pieces, the largest workspace
    Plan a;
    make_plan(n_total, d, V, piece_tokens_for(n_total, true), &a, true);
    *bytes = (int64_t)a.total;
    return TS_OK;
}

int ts_call_workspace_bytes(int64_t n_total, int32_t row_dtype, int32_t d, int32_t V, int64_t* bytes)
{
    if (!bytes) return TS_ERR_NULL;
    if (n_total < 0 || V <= 0 || d <= 0 || (d % 4) != 0) return TS_ERR_SHAPE;
    if (row_dtype != TS_ROW_FP32 && row_dtype != TS_ROW_BF16) return TS_ERR_SHAPE;
    if (n_total >= ((int64_t)1 << 31)) return TS_ERR_OVERFLOW;
    Plan a;
    make_plan(n_total, d, V, piece_tokens_for(n_total, row_dtype == TS_ROW_BF16 && (d % 8) == 0), &a);
    *bytes = (int64_t)a.total;
    return TS_OK;
}

int ts_bind_workspace(void* ws, int64_t bytes)
{
    if (!ws) {
        g_ws = nullptr;
        g_ws_bytes = 0;
        g_have_last = false;
        return TS_OK;
    }
    if (bytes <= 0) return TS_ERR_SHAPE;
    if ((uintptr_t)ws & 255u) return TS_ERR_ALIGN;
    g_ws = ws;
    g_ws_bytes = bytes;
    g_have_last = false;
    return TS_OK;
}

int ts_last_views(const int32_t** count, const int32_t** row_start, const void** sorted,
                  const int32_t** n_valid, const int32_t** n_bad_ids)
{
    if (!g_last_ws || !g_have_last) return TS_ERR_WORKSPACE;
    const char* ws = (const char*)g_last_ws;
    if (count) *count = (const int32_t*)(ws + g_last_plan.off_count);
    if (row_start) *row_start = (const int32_t*)(ws + g_last_plan.off_row_start);
    if (sorted) *sorted = (const void*)(ws + g_last_plan.off_sorted);
    if (n_valid) *n_valid = (const int32_t*)(ws + g_last_plan.off_nvalid);
    if (n_bad_ids) *n_bad_ids = (const int32_t*)(ws + g_last_plan.off_nbad);
    return TS_OK;
}

int ts_read_views(int32_t* count_out, int32_t* row_start_out, int64_t rows_capacity, void* sorted_out,
                  int64_t sorted_capacity, int32_t* n_valid_out, int32_t* n_bad_ids_out, void* stream)
{
    if (!g_last_ws || !g_have_last) return TS_ERR_WORKSPACE;
    if (sorted_out && sorted_capacity < 0) return TS_ERR_SHAPE;
    // the lengths of count and row_start come from the last call, not from this caller
    if ((count_out || row_start_out) && rows_capacity < (int64_t)g_last_V) return TS_ERR_CAPACITY;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return TS_ERR_HIP;
    const char* ws = (const char*)g_last_ws;
    int32_t n_valid = 0, n_bad = 0;
    if (hipMemcpy(&n_valid, ws + g_last_plan.off_nvalid, 4, hipMemcpyDeviceToHost) != hipSuccess) return TS_ERR_HIP;
    if (hipMemcpy(&n_bad, ws + g_last_plan.off_nbad, 4, hipMemcpyDeviceToHost) != hipSuccess) return TS_ERR_HIP;
    if (sorted_out && (int64_t)n_valid > sorted_capacity) return TS_ERR_CAPACITY;
    if (n_valid_out) *n_valid_out = n_valid;
    if (n_bad_ids_out) *n_bad_ids_out = n_bad;
    if (count_out && hipMemcpy(count_out, ws + g_last_plan.off_count, (size_t)g_last_V * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return TS_ERR_HIP;
    if (row_start_out && hipMemcpy(row_start_out, ws + g_last_plan.off_row_start, ((size_t)g_last_V + 1) * 4,
                                   hipMemcpyDeviceToHost) != hipSuccess)
        return TS_ERR_HIP;
    if (sorted_out) {
        if (n_valid > 0 && hipMemcpy(sorted_out, ws + g_last_plan.off_sorted, (size_t)n_valid * sizeof(SortedPair),
                                     hipMemcpyDeviceToHost) != hipSuccess)
            return TS_ERR_HIP;
    }
    return TS_OK;
}

int ts_last_launch_info(int32_t* info)
{
    if (!info) return TS_ERR_NULL;
    if (!g_have_last) return TS_ERR_WORKSPACE;
    for (int i = 0; i < 8; ++i) info[i] = g_last_info[i];
    return TS_OK;
}

int ts_unique_ids(int32_t* unique_ids_out, int32_t* n_unique_out, void* stream)
{
    if (!unique_ids_out || !n_unique_out) return TS_ERR_NULL;
    if (!g_last_ws || !g_have_last) return TS_ERR_WORKSPACE;
    const int32_t* count = (const int32_t*)((const char*)g_last_ws + g_last_plan.off_count);
    hipLaunchKernelGGL(unique_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, count, g_last_V,
                       unique_ids_out, n_unique_out);
    return check_hip(hipGetLastError());
}

int ts_profile_begin(int32_t capacity)
{
    if (capacity < 0 || capacity > kMaxProfile) return TS_ERR_SHAPE;
    while (g_ev_made < 2 * capacity) {
        if (hipEventCreate(&g_ev[g_ev_made]) != hipSuccess) return TS_ERR_HIP;
        ++g_ev_made;
    }
    g_prof_cap = capacity;
    g_prof_used = 0;
    return TS_OK;
}

int ts_profile_end(float* ms_out, int32_t capacity, int32_t* n_out)
{
    if (!ms_out || !n_out) return TS_ERR_NULL;
    int m = g_prof_used < capacity ? g_prof_used : capacity;
    if (m < 0) m = 0;
    for (int i = 0; i < m; ++i) {
        if (hipEventSynchronize(g_ev[2 * i + 1]) != hipSuccess) return TS_ERR_HIP;
        if (hipEventElapsedTime(&ms_out[i], g_ev[2 * i], g_ev[2 * i + 1]) != hipSuccess) return TS_ERR_HIP;
    }
    *n_out = m;
    g_prof_cap = 0;
    g_prof_used = 0;
    return TS_OK;
}

int ts_set_overlap_bytes(int64_t sort_bytes)
{
    if (sort_bytes < -1) return TS_ERR_SHAPE;
    g_overlap_sort = sort_bytes;
    return TS_OK;
}

int ts_set_sort_part(int32_t part)
{
    if (part != 0 && part != 64 && part != 128 && part != 256 && part != 512 && part != 1024 && part != kMaxPart)
        return TS_ERR_SHAPE;
    g_part_override = part;
    return TS_OK;
}

int ts_set_short_rows(int32_t mode)
{
    if (mode < -1 || mode > 1) return TS_ERR_SHAPE;
    g_short_rows = mode;
    return TS_OK;
}

int ts_set_piece_tokens(int32_t piece_tokens)
{
    if (piece_tokens != 0 && piece_tokens != 8 && piece_tokens != 16 && piece_tokens != 32) return TS_ERR_SHAPE;
    g_piece_override = piece_tokens;
    return TS_OK;
}

const char* ts_status_string(int status)
{
    switch (status) {
        case TS_OK: return "ok";
        case TS_ERR_NULL: return "a required pointer is NULL";
        case TS_ERR_SHAPE: return "bad shape or argument value";
        case TS_ERR_ALIGN: return "pointer not aligned";
        case TS_ERR_WORKSPACE: return "workspace not bound or too small";
        case TS_ERR_HIP: return "HIP runtime error";
        case TS_ERR_OVERFLOW: return "size overflow";
        case TS_ERR_CAPACITY: return "output buffer too small";
        default: return "unknown status";
    }
}

}  // extern "C"
