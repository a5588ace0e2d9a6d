// kvm_score_step: softmax attention mass per (row, 16-token block) unit.
//
// What is computed is Eq. 1 of the paper restricted to the HBM-resident tokens
// of each row, summed per token block, then the maximum (or mean) over the
// query heads that share the KV head (GQA grouping rule, section 3.4).
//
// Structure (all kernels in this file):
//   plan_*          build the list of tiles (a record per run of at most T blocks of an active
//                   row), on the device, so the scorer's grid has no idle workgroups whatever
//                   the spread of row lengths, and the list of the tiles the row merge has
//                   to visit.  T depends on the kernel (64 .. 512).
//   score_tile_*    one workgroup per tile, taken in an XCD-aware order.  Per (unit, query)
//                   the kernel forms lse = log sum_t exp(z_t) over the block's tokens (the
//                   block's softmax mass is exp(lse - row lse)) and the tile's lse per query.
//                   The dot2 and mfma kernels keep the block values in LDS: a row that fits
//                   one tile is finished on the spot (only its masses are written); otherwise
//                   the tile writes the block values of its resident blocks, packed, plus the
//                   tile value, and score_rowmerge combines the tiles of the row.  The wide
//                   kernel always writes block values and leaves every row to the merge.
//   score_rowmerge* a fixed grid strides over the tiles of the rows that are not finished yet
//                   (a list the plan also makes): row lse from the tile values, masses from
//                   the block values.
//   xfer_*          bytes of a deferred exchange that ride along with a tile kernel.
//       _dot2       g in {1, 2, 4, 8}, dim <= 128: queries in registers, v_dot2 with fp32
//                   accumulate, one wavefront per unit
//       _mfma       any other g <= 128, dim <= 256: queries as matrix-core operands in
//                   registers, one wavefront per unit
//       _wide       dim 576 (MLA latent): the four wavefronts split up to 128 queries and
//                   share each unit through LDS; frames go global -> LDS directly
//
// The tile kernels are the only ones that touch K; they read every resident unit
// exactly once with non-temporal 16-byte loads that cover 1 KiB contiguous per
// wavefront instruction.  With the [dim/8][16][8] frame layout lane l of load kk
// holds token l%16, channels 32*kk + 8*(l/16) .. +7, which is at once
//   - a lane-private share of q.k for the dot2 kernel (cross-lane work: a reduce-scatter
//     over the four 16-lane rows with two row swaps per four queries, then 16-lane DPP
//     reductions for the block maximum and sum), and
//   - the A operand of v_mfma_f32_16x16x32 for k-step kk (row = token, k = channel), so
//     K goes from the load straight into the matrix core.
#include <atomic>

#include "kvm_internal.h"

namespace kvm {
namespace {

// What a tile kernel needs to know of its tile, in one 32-byte record written by the plan, so that
// a workgroup reaches its table entries and queries after a single dependent load (tile -> row
// -> row arrays was two, and on workloads of short rows the set-up chain is a good part of a
// workgroup's lifetime).
struct alignas(16) Tile {
    int64_t uid0;       // uid of the tile's first block
    int64_t q_off;      // element offset of the row's queries
    int32_t b0;         // the tile's first block in its row
    int32_t ntok;       // tokens of the row
    int32_t pad[2];
};

constexpr int kThreads = 256;   // workgroup size of every scorer kernel (4 wavefronts)

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));

// ---- arithmetic on 16-bit pairs -------------------------------------------------
template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c);
template <>
__device__ __forceinline__ float dot2<KVM_BF16>(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
template <>
__device__ __forceinline__ float dot2<KVM_FP16>(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), c, false);
}

template <int DT>
__device__ __forceinline__ float dot8(const uint4& k, const uint4& q, float c) {
    c = dot2<DT>(k.x, q.x, c);
    c = dot2<DT>(k.y, q.y, c);
    c = dot2<DT>(k.z, q.z, c);
    c = dot2<DT>(k.w, q.w, c);
    return c;
}

template <int DT>
__device__ __forceinline__ f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
    if constexpr (DT == KVM_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                       0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0,
                                                      0, 0);
}

// ---- cross-lane helpers -------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// All-reduce over each aligned group of 16 lanes: xor 1, xor 2 (quad permutes),
// then mirror within 8 and within 16 lanes.
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    return v;
}

// v_permlane32_swap exchanges rows 2,3 of its first operand with rows 0,1 of its second;
// v_permlane16_swap exchanges the odd rows of the first with the even rows of the second
// (a row = 16 lanes).  The builtins return both registers.  hipcc 7.2 folds r[0] + r[1]
// into r[0] + r[0] when the two results feed one operation directly; passing them through
// an empty asm statement keeps them in distinct registers (the compiler still inserts the
// wait states the instruction needs).
__device__ __forceinline__ void swap32(float a, float b, float& x, float& y) {
    auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
    unsigned u = r[0], v = r[1];
    asm volatile("" : "+v"(u), "+v"(v));
    x = __builtin_bit_cast(float, u);
    y = __builtin_bit_cast(float, v);
}
__device__ __forceinline__ void swap16(float a, float b, float& x, float& y) {
    auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
    unsigned u = r[0], v = r[1];
    asm volatile("" : "+v"(u), "+v"(v));
    x = __builtin_bit_cast(float, u);
    y = __builtin_bit_cast(float, v);
}
// a, b hold partial sums in all four 16-lane rows.  Returns, in rows 0 and 1,
// a summed over row pairs (0,2) and (1,3); in rows 2 and 3 the same for b.
__device__ __forceinline__ float fold_halves(float a, float b) {
    float x, y;
    swap32(a, b, x, y);
    return x + y;
}
// a, b as returned by fold_halves.  Row 0 gets a's rows 0+1, row 1 b's rows 0+1,
// row 2 a's rows 2+3, row 3 b's rows 2+3.
__device__ __forceinline__ float fold_rows(float a, float b) {
    float x, y;
    swap16(a, b, x, y);
    return x + y;
}
// After fold_rows(fold_halves(a0, a1), fold_halves(a2, a3)) the 16-lane row
// `cg` holds the complete sum of a_{query_of_row(cg)}.
__device__ __forceinline__ int query_of_row(int cg) { return ((cg & 1) << 1) | (cg >> 1); }
// All-reduce over the four rows (lanes l, l^16, l^32, l^48).
__device__ __forceinline__ float rows4_max(float v) {
    float x, y;
    swap32(v, v, x, y);
    v = fmaxf(x, y);
    swap16(v, v, x, y);
    return fmaxf(x, y);
}
__device__ __forceinline__ float rows4_sum(float v) {
    float x, y;
    swap32(v, v, x, y);
    v = x + y;
    swap16(v, v, x, y);
    return x + y;
}

// Maximum (MAX) or sum over each aligned group of N lanes (N a power of two up to 64), result in
// every lane of the group: DPP permutes within a row of 16 lanes, lane swaps across rows.  No LDS
// crossbar traffic (ds_bpermute, which is what __shfl_xor becomes, takes an LDS issue slot per
// value and the row merge reduces dozens of values per thread).
template <int N, bool MAX>
__device__ __forceinline__ float lanes_allreduce(float v) {
    auto op = [](float a, float b) { return MAX ? fmaxf(a, b) : a + b; };
    if constexpr (N >= 2) v = op(v, dpp_f<0xB1>(v));
    if constexpr (N >= 4) v = op(v, dpp_f<0x4E>(v));
    if constexpr (N >= 8) v = op(v, dpp_f<0x141>(v));
    if constexpr (N >= 16) v = op(v, dpp_f<0x140>(v));
    if constexpr (N >= 32) {
        float x, y;
        swap16(v, v, x, y);
        v = op(x, y);
    }
    if constexpr (N >= 64) {
        float x, y;
        swap32(v, v, x, y);
        v = op(x, y);
    }
    return v;
}

// Running softmax statistics: maximum m and z = sum exp(x - m).
struct MZ {
    float m, z;
};
__device__ __forceinline__ MZ mz_combine(MZ a, MZ b) {
    const float M = fmaxf(a.m, b.m);
    if (M == -INFINITY) return MZ{M, 0.f};
    return MZ{M, a.z * __expf(a.m - M) + b.z * __expf(b.m - M)};
}

// ---- plan: tiles of the active rows ------------------------------------------
constexpr int kPlanThreads = 128;     // small workgroups: the emit loop of a long row is serial per thread

// Row metadata the plan needs; a row whose blocks or queries would fall outside the
// arrays is dropped here (it gets no tile) so that no kernel can index out of bounds.
struct PlanRows {
    int n_rows;
    int g, dim;
    int tile_blocks;
    int64_t n_uids, q_elems;
    const int32_t* row_ntok;
    const int64_t* row_off;
    const int64_t* row_q_off;
    const uint8_t* row_active;
    int merge_all;      // the row merge visits every tile (wide path), not only those of rows with several
};

__device__ __forceinline__ bool row_scorable(const PlanRows& p, int r) {
    if (r >= p.n_rows) return false;
    if (p.row_active && !p.row_active[r]) return false;
    const int n = p.row_ntok[r];
    if (n <= 0) return false;
    const int64_t nb = ((int64_t)n + 15) >> 4;
    const int64_t off = p.row_off[r], qo = p.row_q_off[r];
    if (off < 0 || off + nb > p.n_uids) return false;
    if (qo < 0 || (qo & 7) || qo + (int64_t)p.g * p.dim > p.q_elems) return false;
    return true;
}

__device__ __forceinline__ uint32_t tiles_of_row(const PlanRows& p, int r) {
    if (!row_scorable(p, r)) return 0;
    const uint32_t nb = ((uint32_t)p.row_ntok[r] + 15u) >> 4;
    return (nb + p.tile_blocks - 1) / p.tile_blocks;
}

// Exclusive scan of one value per thread over a workgroup of kPlanThreads; returns the
// exclusive prefix and stores the workgroup total in *total.
__device__ uint64_t wg_exclusive_scan(uint64_t v, uint64_t* total) {
    __shared__ uint64_t wave_sums[kPlanThreads / kWave];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t inc = v;
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t o = (uint64_t)__shfl_up((unsigned long long)inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    uint64_t base = 0, tot = 0;
    for (int w = 0; w < kPlanThreads / kWave; ++w) {
        const uint64_t s = wave_sums[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// What a row adds to the two counts the plan scans together: its tiles in the low half and, in
// the high half, those of them that the row merge has to visit (all of them if the row has
// more than one tile, none otherwise).  Both totals stay below 2^32 (checked on the host).
__device__ __forceinline__ uint64_t plan_counts(const PlanRows& p, uint32_t nt) {
    return (uint64_t)nt | ((uint64_t)((nt > 1 || p.merge_all) ? nt : 0) << 32);
}

// What the row merge needs to know of a tile it visits, in one 32-byte record, so that a
// workgroup reaches its data after a single dependent load.
struct alignas(16) MergeTile {
    int64_t uid0;       // first unit of the tile
    uint32_t tile0;     // first tile of its row (the row's tile statistics start there)
    int32_t nbt;        // blocks in the tile
    int32_t n_t;        // tiles of its row
    int32_t pad[3];
};

__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(PlanRows p, uint64_t* wg_sum) {
    const int r = blockIdx.x * kPlanThreads + threadIdx.x;
    uint64_t total;
    (void)wg_exclusive_scan(plan_counts(p, tiles_of_row(p, r)), &total);
    if (threadIdx.x == 0) wg_sum[blockIdx.x] = total;
}

// One workgroup: turns wg_sum[0..n) into exclusive prefixes in place and writes the grand totals:
// counts[0] = tiles, counts[1] = tiles of rows with more than one tile.  Rows that do not overlap in
// uid space cannot have more than tiles_max tiles together (the bound the workspace is carved for);
// if the caller's rows do overlap and exceed it, the plan is declared empty (counts[2] = 1, both
// counts 0): nothing is emitted and nothing is scored, instead of records written past their arrays.
__global__ __launch_bounds__(kPlanThreads) void plan_scan_kernel(int n, uint64_t* wg_sum, uint32_t* counts,
                                                                 uint64_t tiles_max) {
    uint64_t carry = 0;
    for (int base = 0; base < n; base += kPlanThreads) {
        const int i = base + threadIdx.x;
        const uint64_t v = i < n ? wg_sum[i] : 0;
        uint64_t total;
        const uint64_t ex = wg_exclusive_scan(v, &total);
        if (i < n) wg_sum[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) {
        const bool over = (carry & 0xffffffffull) > tiles_max || (carry >> 32) > tiles_max;
        counts[0] = over ? 0u : (uint32_t)carry;
        counts[1] = over ? 0u : (uint32_t)(carry >> 32);
        counts[2] = over ? 1u : 0u;
    }
}

__global__ __launch_bounds__(kPlanThreads) void plan_emit_kernel(PlanRows p, const uint64_t* wg_base,
                                                                 const uint32_t* counts, Tile* tiles,
                                                                 MergeTile* merge) {
    if (counts[2]) return;               // plan declared empty by the scan (same value for every thread)
    const int r = blockIdx.x * kPlanThreads + threadIdx.x;
    const uint32_t nt = tiles_of_row(p, r);
    uint64_t total;
    const uint64_t at = wg_base[blockIdx.x] + wg_exclusive_scan(plan_counts(p, nt), &total);
    const uint32_t first = (uint32_t)at, mfirst = (uint32_t)(at >> 32);
    if (nt == 0) return;
    const int32_t ntok = p.row_ntok[r];
    const int32_t nb = (int32_t)(((uint32_t)ntok + 15u) >> 4);
    const int64_t off = p.row_off[r], q_off = p.row_q_off[r];
    for (uint32_t i = 0; i < nt; ++i) {
        const int32_t b0 = (int32_t)(i * p.tile_blocks);
        tiles[first + i] = Tile{off + b0, q_off, b0, ntok, {0, 0}};
    }
    if (nt > 1 || p.merge_all) {
        for (uint32_t i = 0; i < nt; ++i) {
            const int32_t b0 = (int32_t)(i * p.tile_blocks);
            merge[mfirst + i] = MergeTile{off + b0, first, min(p.tile_blocks, nb - b0), (int32_t)nt, {0, 0, 0}};
        }
    }
}

// ---- bytes of a deferred exchange riding along with a scoring launch ----------------------
// `n` workgroups of a tile kernel's grid each swap one (frame, host tier record) pair in place
// (what kvm_exchange_begin prepared) while the rest of the grid scores: the host link works
// during the scoring instead of after it.  They are interleaved with the scoring workgroups at
// the front of the grid (every stride-th one; the host picks a stride that is no multiple of
// the number of XCDs, so that they spread over all of them): all at the very front they would
// fill every compute unit with waves that only wait for the link and scoring would start
// after them.  The frames involved belong to units the scoring cannot see (kvm_exchange_begin
// has taken them out of the table), so the two kinds of workgroup never touch the same memory.
struct Xfer {
    uint32_t n;
    uint32_t stride;        // every stride-th workgroup of the first n * stride moves pair number (index / stride)
    const int32_t* frame;   // [n] frame of pair i, -1 = skip
    const int64_t* host;    // [n] host tier slot of pair i
    uint4* k_pool;
    uint4* v_pool;
    uint4* tier;
    uint32_t k_v4, v_v4;
    uint32_t n_slots;       // frames of the pool: a frame number outside it is skipped like -1
    uint64_t tier_slots;    // records of the tier: likewise
};

// Pair i decoded: frame, host slot and direction (one-way = the frame is copied out, nothing comes back).
// Returns false for a pair to skip.
__device__ __forceinline__ bool xfer_decode(const Xfer& x, uint32_t i, int32_t* f, int64_t* h, bool* one_way) {
    *f = x.frame[i];
    const int64_t hv = x.host[i];
    *one_way = hv >= 0 && (hv & KVM_XFER_OUT_ONLY) != 0;
    *h = *one_way ? (hv & ~KVM_XFER_OUT_ONLY) : hv;
    return (uint32_t)*f < x.n_slots && (uint64_t)*h < x.tier_slots;
}

__device__ __forceinline__ void xfer_pair(const Xfer& x, uint32_t i) {
    int32_t f;
    int64_t h;
    bool one_way;
    if (!xfer_decode(x, i, &f, &h, &one_way)) return;
    uint4* rec = x.tier + (size_t)h * ((size_t)x.k_v4 + x.v_v4);
    uint4* kf = x.k_pool + (size_t)f * x.k_v4;
    if (one_way) {                                                        // uniform for the workgroup
        for (uint32_t v = threadIdx.x; v < x.k_v4; v += kThreads) rec[v] = kf[v];
        if (x.v_v4) {
            const uint4* vf = x.v_pool + (size_t)f * x.v_v4;
            for (uint32_t v = threadIdx.x; v < x.v_v4; v += kThreads) rec[x.k_v4 + v] = vf[v];
        }
        return;
    }
    for (uint32_t v = threadIdx.x; v < x.k_v4; v += kThreads) {
        const uint4 a = kf[v], b = rec[v];
        kf[v] = b;
        rec[v] = a;
    }
    if (x.v_v4) {
        uint4* vf = x.v_pool + (size_t)f * x.v_v4;
        for (uint32_t v = threadIdx.x; v < x.v_v4; v += kThreads) {
            const uint4 a = vf[v], b = rec[x.k_v4 + v];
            vf[v] = b;
            rec[x.k_v4 + v] = a;
        }
    }
}

__global__ __launch_bounds__(kThreads) void xfer_kernel(Xfer x) { xfer_pair(x, blockIdx.x); }

// Position in the tile kernels' work order of workgroup `b` of a grid of `n`.  Workgroups go to the
// eight XCDs in turn (b mod 8) and every XCD has its own L2, so eight neighbouring tiles, which
// mostly belong to one row and read the same queries (147 KB for a row of latent frames), would
// each fetch them into a different L2.  Inside every aligned run of 64 workgroups the order is
// transposed: positions 8x .. 8x + 7 are the eight workgroups that run on XCD x.  A bijection
// whatever the hardware does; the last, partial run keeps its order.
#ifndef KVM_XCD_ORDER
#define KVM_XCD_ORDER 1
#endif
#ifndef KVM_XCD_RUN
#define KVM_XCD_RUN 8
#endif
__device__ __forceinline__ uint32_t xcd_order(uint32_t b, uint32_t n) {
    constexpr uint32_t C = KVM_XCD_RUN, G = 8 * C;      // C neighbouring positions per XCD, groups of 8 C
    if (!KVM_XCD_ORDER || b >= n / G * G) return b;
    const uint32_t r = b % G;
    return b - r + (r & 7u) * C + (r >> 3);
}

// Which role the workgroup at position `b` of a tile kernel's work order plays: returns true and
// the pair number for a transfer workgroup, false and the tile number otherwise.
__device__ __forceinline__ bool xfer_role(const Xfer& x, uint32_t b, uint32_t* index) {
    const uint32_t region = x.n * x.stride;
    if (b < region) {
        const uint32_t q = b / x.stride;
        if (b - q * x.stride == 0) {
            *index = q;
            return true;
        }
        *index = b - (q + 1);        // transfer workgroups before b: q + 1
        return false;
    }
    *index = b - x.n;
    return false;
}

// ---- shared pieces of the tile kernels ---------------------------------------------

// What every tile kernel derives from its tile.
struct TileCtx {
    int b0;
    int ntok, nb, nbt;       // tokens and blocks of the row, blocks of this tile
    int64_t uid0;            // uid of the tile's block 0
    int64_t q_off;           // element offset of the row's queries
};
template <int T>
__device__ __forceinline__ TileCtx tile_ctx(const Tile* tiles, uint32_t tile_id) {
    const Tile tile = tiles[tile_id];
    TileCtx c;
    c.b0 = tile.b0;
    c.ntok = tile.ntok;
    c.nb = (int)(((uint32_t)c.ntok + 15u) >> 4);
    c.nbt = min(T, c.nb - tile.b0);
    c.uid0 = tile.uid0;
    c.q_off = tile.q_off;
    return c;
}

// The table entries of a tile, thread t holding blocks t, t + 256, ... (-1 past the end).
template <int T>
struct TileSlots {
    int v[(T + kThreads - 1) / kThreads];
};
template <int T>
__device__ __forceinline__ TileSlots<T> load_tile_slots(const int32_t* __restrict__ slot_tbl, int64_t uid0, int nbt) {
    TileSlots<T> s;
#pragma unroll
    for (int e = 0; e < (T + kThreads - 1) / kThreads; ++e) {
        const int b = e * kThreads + threadIdx.x;
        s.v[e] = b < nbt ? slot_tbl[uid0 + b] : -1;
    }
    return s;
}

// Resident units of a tile, compacted into LDS as (block index in tile, pool frame), in
// block order: every thread looks at up to T/256 table entries, a ballot + popcount
// gives each resident entry its place.  Returns the list length.  Contains two barriers.
template <int T>
__device__ __forceinline__ int build_unit_list(TileSlots<T> slots, uint32_t n_slots, int2* s_list,
                                               int* s_cnt /* [E * 4] */) {
    constexpr int E = (T + kThreads - 1) / kThreads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int slot[E], within[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        slot[e] = slots.v[e];
        if ((uint32_t)slot[e] >= n_slots) slot[e] = -1;
        const uint64_t bal = __ballot(slot[e] >= 0);
        within[e] = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) s_cnt[e * 4 + wave] = __popcll(bal);
    }
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        int base = total;
        for (int w = 0; w < 4; ++w) {
            const int c = s_cnt[e * 4 + w];
            if (w < wave) base += c;
            total += c;
        }
        if (slot[e] >= 0) s_list[base + within[e]] = make_int2(e * kThreads + threadIdx.x, slot[e]);
    }
    __syncthreads();
    return total;
}

template <int T>
__device__ __forceinline__ int build_unit_list(const int32_t* __restrict__ slot_tbl, int64_t uid0, int nbt,
                                               uint32_t n_slots, int2* s_list, int* s_cnt /* [E * 4] */) {
    return build_unit_list<T>(load_tile_slots<T>(slot_tbl, uid0, nbt), n_slots, s_list, s_cnt);
}

template <int NK>
__device__ __forceinline__ void load_unit(uint4 (&dst)[NK], const uint4* __restrict__ k_pool, uint32_t slot,
                                          int unit_v4, int lane) {
    const v4u_t* p = reinterpret_cast<const v4u_t*>(k_pool + (size_t)slot * unit_v4 + lane);
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
        // K is read once per step and never again: non-temporal, so it does not displace the tables in L2
        const v4u_t v = __builtin_nontemporal_load(p + kk * 64);
        dst[kk] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

__device__ __forceinline__ int2 list_entry(const int2* s_list, int idx) {      // wave-uniform LDS read
    const int2 e = s_list[idx];
    return make_int2(__builtin_amdgcn_readfirstlane(e.x), __builtin_amdgcn_readfirstlane(e.y));
}

// The unit loop shared by the tile kernels.  Wavefront w takes list entries w, w + 4, ...:
// balanced whatever the residency pattern.  Two units are in flight per wavefront; the
// loads of the following unit are issued unconditionally (past the end of the list they
// re-read the last unit, a cache hit): a branch around them would make the compiler wait
// for every outstanding load before the first use of the current unit, which serialises
// load and compute.  `unit(cur, block index in tile)` consumes one unit.
template <int NK, class UnitFn>
__device__ __forceinline__ void for_each_unit(const int2* s_list, int n_res, const uint4* __restrict__ k_pool,
                                              int unit_v4, UnitFn unit) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 cur[NK], nxt[NK];
    int idx = wave;
    int i_cur = -1;
    if (idx < n_res) {
        const int2 e = list_entry(s_list, idx);
        i_cur = e.x;
        load_unit<NK>(cur, k_pool, (uint32_t)e.y, unit_v4, lane);
    }
    while (i_cur >= 0) {
        idx += 4;
        const int2 e_nxt = list_entry(s_list, idx < n_res ? idx : n_res - 1);
        const int i_nxt = idx < n_res ? e_nxt.x : -1;
        load_unit<NK>(nxt, k_pool, (uint32_t)e_nxt.y, unit_v4, lane);
        unit(cur, i_cur);
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) cur[kk] = nxt[kk];
        i_cur = i_nxt;
    }
}

// The same with two units in flight per wavefront besides the one being consumed (three
// register sets, the loop unrolled three times so that no set is ever copied).  More bytes in
// flight per compute unit for kernels whose register budget allows it.
template <int NK, class UnitFn>
__device__ __forceinline__ void for_each_unit_deep(const int2* s_list, int n_res, const uint4* __restrict__ k_pool,
                                                   int unit_v4, UnitFn unit) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint4 b0[NK], b1[NK], b2[NK];
    int i0, i1, i2;
    auto fetch = [&](uint4 (&dst)[NK], int idx) -> int {
        const int2 e = list_entry(s_list, idx < n_res ? idx : n_res - 1);
        load_unit<NK>(dst, k_pool, (uint32_t)e.y, unit_v4, lane);
        return idx < n_res ? e.x : -1;
    };
    int idx = wave;
    if (idx >= n_res) return;
    i0 = fetch(b0, idx);
    i1 = fetch(b1, idx + 4);
    while (true) {
        i2 = fetch(b2, idx + 8);
        unit(b0, i0);
        if (i1 < 0) break;
        i0 = fetch(b0, idx + 12);
        unit(b1, i1);
        if (i2 < 0) break;
        i1 = fetch(b1, idx + 16);
        unit(b2, i2);
        if (i0 < 0) break;
        idx += 12;
    }
}

// Where a tile kernel leaves its results.
struct TileOut {
    int agg;
    float* mass;        // [n_uids]
    // Rows of more than one tile only.  Row stride of both: g rounded up to a power of two on the dot2 and
    // mfma paths (vector loads in the row merge stay aligned); on the wide path 128 and g.
    // part_lse: log sum exp of a block's logits per query.  Dot2 and mfma paths: the i-th resident block of
    // a tile at entry (tile's first uid + i); wide path: block of uid u at entry u.
    float* part_lse;    // [n_uids][stride]
    float* tile_lse;    // [n_tiles][stride]: log sum exp over the tile
};

// Group aggregation of N values per thread over the GP lanes / threads that hold the
// queries of one block.  For GP = 128 (two wavefronts per block) the wavefront results meet
// in LDS: s_v holds 4 * N floats and the call contains one barrier.
template <int GP, int N>
__device__ __forceinline__ void group_agg(float (&v)[N], int agg, float* s_v) {
    constexpr int IN_WAVE = GP <= 64 ? GP : 64;
    if (agg == KVM_AGG_MAX) {
#pragma unroll
        for (int k = 0; k < N; ++k) v[k] = lanes_allreduce<IN_WAVE, true>(v[k]);
    } else {
#pragma unroll
        for (int k = 0; k < N; ++k) v[k] = lanes_allreduce<IN_WAVE, false>(v[k]);
    }
    if constexpr (GP > 64) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        if (lane == 0)
#pragma unroll
            for (int k = 0; k < N; ++k) s_v[k * 4 + wave] = v[k];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const float x = s_v[k * 4 + (wave & ~1)], y = s_v[k * 4 + (wave | 1)];
            v[k] = agg == KVM_AGG_MAX ? fmaxf(x, y) : x + y;
        }
    }
}

// Per-query total of (m, z) over the whole workgroup; thread (bsub, j) = (tid / GP, tid % GP)
// contributes `acc` for query j.  Contains one barrier.
template <int GP>
__device__ __forceinline__ MZ wg_total(MZ acc, float2* s_red /* [256] */) {
    const int j = threadIdx.x & (GP - 1);
#pragma unroll
    for (int d = GP; d < 64; d <<= 1) acc = mz_combine(acc, MZ{__shfl_xor(acc.m, d), __shfl_xor(acc.z, d)});
    s_red[threadIdx.x] = make_float2(acc.m, acc.z);
    __syncthreads();
    MZ tot{-INFINITY, 0.f};
#pragma unroll
    for (int w = 0; w < 4; ++w)
        if (GP <= 64 || (w & 1) == (j >> 6)) {
            const float2 p = s_red[w * 64 + (GP <= 64 ? j : (j & 63))];
            tot = mz_combine(tot, MZ{p.x, p.y});
        }
    return tot;
}

// log(sum exp) of what an MZ has seen; -inf for nothing.
__device__ __forceinline__ float mz_lse(MZ a) { return a.z > 0.f ? a.m + __logf(a.z) : -INFINITY; }

// Epilogue of a tile kernel.  s_lse[b * g + j] = log sum_t exp(z_t) over the tokens of block b
// for query j (the block's softmax mass is exp(s_lse - row lse)), or -inf where the block is
// not resident.  GP = smallest power of two >= g; thread (bsub, j) sweeps blocks bsub,
// bsub + 256/GP, ...
template <int GP, int T>
__device__ __forceinline__ void tile_epilogue(const float* s_lse, float2* s_red /* [256] */, float* s_v, int g,
                                              const TileCtx& c, size_t tile_index, const TileOut& o,
                                              const int2* s_list, int n_res) {
    constexpr int BS = kThreads / GP;
    constexpr int SWEEPS = (T + BS - 1) / BS;
    const int j = threadIdx.x & (GP - 1), bsub = threadIdx.x / GP;
    const bool jv = j < g;
    MZ acc{-INFINITY, 0.f};
    if (jv)
        for (int b = bsub; b < c.nbt; b += BS) acc = mz_combine(acc, MZ{s_lse[b * g + j], 1.f});
    const float tile_lse = mz_lse(wg_total<GP>(acc, s_red));

    if (c.nb <= T) {
        // the row is this tile: finish it here, a few sweeps at a time to keep registers low
        constexpr int CH = SWEEPS < 8 ? SWEEPS : 8;
        for (int k0 = 0; k0 < SWEEPS; k0 += CH) {
            float v[CH];
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                const int b = (k0 + k) * BS + bsub;
                const float l = (b < c.nbt && jv) ? s_lse[b * g + j] : -INFINITY;
                v[k] = l > -INFINITY ? __expf(l - tile_lse) : 0.f;
            }
            if (GP > 64 && k0 > 0) __syncthreads();       // s_v of the previous chunk has been read
            group_agg<GP, CH>(v, o.agg, s_v);
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                const int b = (k0 + k) * BS + bsub;
                // query 0 tells whether the block is resident
                if (j == 0 && b < c.nbt && s_lse[b * g] > -INFINITY)
                    // non-temporal: a plain store leaves a dirty line in the L2 whose write-back competes with the
                    // streaming reads later (in-process A/B on 16,384 one-tile rows: -2 % on the launch)
                    __builtin_nontemporal_store(o.agg == KVM_AGG_MAX ? v[k] : v[k] / (float)g, &o.mass[c.uid0 + b]);
            }
        }
    } else {
        if (bsub == 0 && jv) o.tile_lse[tile_index * GP + j] = tile_lse;
        // The block values of the resident blocks, packed: the i-th resident block of the tile goes to
        // entry uid0 + i, GP floats per entry (the row merge rebuilds the same list from the table).
        // What these stores cost is the number of 128-byte lines they touch, not their bytes (measured:
        // 0.2 ns per line on the 70B-shaped launch, 13 % of it with one entry per block and half the
        // blocks resident), so they are written without holes.  Non-temporal: read back once.
        if (jv)
            for (int i = bsub; i < n_res; i += BS)
                __builtin_nontemporal_store(s_lse[s_list[i].x * g + j], &o.part_lse[(c.uid0 + i) * GP + j]);
    }
}

// LDS a tile kernel needs besides its block-value array.
template <int T, int GP>
struct TileLds {
    int2 list[T];
    int cnt[((T + kThreads - 1) / kThreads) * 4];
    float2 red[kThreads];
    float v[GP > 64 ? 4 * ((T + kThreads / GP - 1) / (kThreads / GP)) : 1];
};

// ---- score_tile_dot2: g in {1, 2, 4, 8}, queries in registers ----------------------
template <int G, int DIM, int DT, int T>
__global__ __launch_bounds__(kThreads) void score_tile_dot2_kernel(
    const Tile* __restrict__ tiles, const uint32_t* __restrict__ n_tiles,
    const int32_t* __restrict__ slot_tbl, const uint4* __restrict__ k_pool, uint32_t n_slots,
    const uint16_t* __restrict__ q, float scale, TileOut out, Xfer xf) {
    static_assert(G == 1 || G == 2 || G == 4 || G == 8, "power-of-two group sizes only");
    constexpr int NK = DIM / 32;          // 16-byte loads per lane per unit
    constexpr int QROW_V4 = DIM / 8;      // 16-byte vectors per query
    __shared__ float s_lse[T * G];        // log sum exp per (block, query); -inf = not resident
    __shared__ TileLds<T, G> lds;

    uint32_t tile_id;
    if (xfer_role(xf, xcd_order(blockIdx.x, gridDim.x), &tile_id)) {     // this workgroup moves bytes instead of scoring
        xfer_pair(xf, tile_id);
        return;
    }
    // record and tile count are loaded together; the record of a position past the count is never used
    const TileCtx c = tile_ctx<T>(tiles, tile_id);
    if (tile_id >= *n_tiles) return;
    const int lane = threadIdx.x & 63;
    const int t = lane & 15, cg = lane >> 4;
    const uint4* qrow = reinterpret_cast<const uint4*>(q + c.q_off);

    uint4 qv[G][NK];
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) qv[j][kk] = qrow[j * QROW_V4 + 4 * kk + cg];

    for (int i = threadIdx.x; i < c.nbt * G; i += kThreads) s_lse[i] = -INFINITY;
    const int n_res = build_unit_list<T>(slot_tbl, c.uid0, c.nbt, n_slots, lds.list, lds.cnt);
    if (n_res == 0) {                            // nothing resident in this tile (uniform)
        // a row of several tiles still folds this tile's statistic: it must read as empty
        if (c.nb > T && threadIdx.x < G) out.tile_lse[(size_t)tile_id * G + threadIdx.x] = -INFINITY;
        return;
    }

    for_each_unit_deep<NK>(lds.list, n_res, k_pool, DIM * 2, [&](const uint4 (&cur)[NK], int i_cur) {
        const bool valid = t < min(16, c.ntok - 16 * (c.b0 + i_cur));
        // four queries at a time: each 16-lane row ends up owning one of them
#pragma unroll
        for (int j0 = 0; j0 < G; j0 += 4) {
            float a[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (j0 + jj < G) {
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) a[jj] = dot8<DT>(cur[kk], qv[(j0 + jj) % G][kk], a[jj]);
                }
            const float z = fold_rows(fold_halves(a[0], a[1]), fold_halves(a[2], a[3])) * scale;
            const float zz = valid ? z : -INFINITY;
            const float mx = row16_max(zz);
            const float e = valid ? __expf(zz - mx) : 0.f;
            const float s = row16_sum(e);
            const int jq = j0 + query_of_row(cg);
            if (t == 0 && jq < G) s_lse[i_cur * G + jq] = mx + __logf(s);
        }
    });
    __syncthreads();
    tile_epilogue<G, T>(s_lse, lds.red, lds.v, G, c, tile_id, out, lds.list, n_res);
}


// ---- score_row: one large workgroup per row, block values never leave the chip -----------
// For launches made of long rows (thousands of blocks each, g <= 8).  The tile kernels hand the
// block values of a row of several tiles to the row merge through HBM; those stores cost far more
// than their bytes (measured: 13 % of the launch on rows of 8,192 blocks) and the merge is a second
// pass.  Here one workgroup of eight or twelve wavefronts owns the whole row: the log-sum-exp of
// every resident block per query stays in LDS (the 160 KB of a compute unit hold 4,456 blocks of
// eight queries; what does not fit spills to the workspace and is read back by the same workgroup),
// the row's log-sum-exp is folded at the end and the masses are written once.  No plan, no tile
// statistics, no merge launch.
//   - Logits: packed dot products for g < 8.  With eight queries those are 128 vector instructions
//     per block and the loop runs out of issue slots (the chip also lowers its clock under that
//     load: 1.8 GHz measured against 2.2 GHz for g 4), so g 8 takes them from the matrix cores:
//     four 16x16x32 products per block with the queries as a half-empty column tile, 16 registers
//     of query operands instead of 128 (measured on rows of 8,192 blocks: 6.55 -> 6.38 ms).
//   - The row is walked in segments of 4,096 blocks: table entries -> compacted list of frames in
//     LDS (ballot + popcount), then the unit loop.
//   - Wavefronts take units from the list through a counter in LDS, so a wavefront that starts
//     late (the one that moves transfer pairs first) or draws slower units simply takes fewer.
//   - Transfer pairs of a deferred exchange ride along: workgroup b moves pairs b, b + grid, ...
//     with its last wavefront before that wavefront joins the scoring.
constexpr int kRowSeg = 4096;
constexpr int kRowLdsBytes = 160 * 1024;
// Workgroup size by group size: twelve wavefronts for one or two queries in registers, eight otherwise
// (four queries at twelve wavefronts spill; the matrix-core variant measures the same at eight and twelve).
#ifndef KVM_ROW_MF_MIN_G
#define KVM_ROW_MF_MIN_G 8
#endif
#ifndef KVM_ROW_MF_THREADS
#define KVM_ROW_MF_THREADS 512
#endif
// Groups of at least this many queries take their logits from the matrix cores in the row kernel.
constexpr int kRowMfMinG = KVM_ROW_MF_MIN_G;
template <int G>
struct RowShape {
    static constexpr bool kMf = G >= kRowMfMinG;
    static constexpr int kThreads = kMf ? KVM_ROW_MF_THREADS : G >= 4 ? 512 : 768;
    static constexpr int kWaves = kThreads / 64;
    static constexpr int kE = (kRowSeg + kThreads - 1) / kThreads;              // table entries per thread and segment
    static constexpr int kFixed = kRowSeg * 4 + 512 + kThreads * 8 + 256;        // list, counts, reduction, misc
    static constexpr int kCap = (kRowLdsBytes - kFixed) / (4 * G);              // block values that stay in LDS
};

struct RowArgs {
    const int32_t* slot_tbl;
    const uint4* k_pool;
    uint32_t n_slots;
    const uint16_t* q;
    float scale;
    int agg;
    float* mass;        // [n_uids]
    float* spill;       // [n_uids][G]: block values beyond the LDS capacity, entry (row's first uid + rank)
};

// One wavefront swaps n 16-byte pieces between a frame and its host record, four loads of each in
// flight per lane (past the end a lane re-reads the last piece and stores nothing).
__device__ __forceinline__ void swap_pieces_wave(uint4* __restrict__ dev, uint4* __restrict__ host, uint32_t n, int lane) {
    for (uint32_t v0 = 0; v0 < n; v0 += 256) {
        const uint32_t i0 = v0 + lane, i1 = i0 + 64, i2 = i0 + 128, i3 = i0 + 192;
        const uint32_t c0 = i0 < n ? i0 : n - 1, c1 = i1 < n ? i1 : n - 1, c2 = i2 < n ? i2 : n - 1,
                       c3 = i3 < n ? i3 : n - 1;
        const uint4 a0 = dev[c0], a1 = dev[c1], a2 = dev[c2], a3 = dev[c3];
        const uint4 h0 = host[c0], h1 = host[c1], h2 = host[c2], h3 = host[c3];
        if (i0 < n) { dev[i0] = h0; host[i0] = a0; }
        if (i1 < n) { dev[i1] = h1; host[i1] = a1; }
        if (i2 < n) { dev[i2] = h2; host[i2] = a2; }
        if (i3 < n) { dev[i3] = h3; host[i3] = a3; }
    }
}
// One wavefront copies n 16-byte pieces of a frame to its host record, eight loads in flight per lane.
__device__ __forceinline__ void copy_pieces_wave(const uint4* __restrict__ dev, uint4* __restrict__ host, uint32_t n,
                                                 int lane) {
    for (uint32_t v0 = 0; v0 < n; v0 += 512) {
        uint4 a[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t i = v0 + j * 64 + lane;
            a[j] = dev[i < n ? i : n - 1];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t i = v0 + j * 64 + lane;
            if (i < n) host[i] = a[j];
        }
    }
}
// One wavefront moves pair i: frame and host record swapped in place, or the frame copied out.
__device__ __forceinline__ void xfer_pair_wave(const Xfer& x, uint32_t i, int lane) {
    int32_t f;
    int64_t h;
    bool one_way;
    if (!xfer_decode(x, i, &f, &h, &one_way)) return;
    uint4* rec = x.tier + (size_t)h * ((size_t)x.k_v4 + x.v_v4);
    if (one_way) {
        copy_pieces_wave(x.k_pool + (size_t)f * x.k_v4, rec, x.k_v4, lane);
        if (x.v_v4) copy_pieces_wave(x.v_pool + (size_t)f * x.v_v4, rec + x.k_v4, x.v_v4, lane);
        return;
    }
    swap_pieces_wave(x.k_pool + (size_t)f * x.k_v4, rec, x.k_v4, lane);
    if (x.v_v4) swap_pieces_wave(x.v_pool + (size_t)f * x.v_v4, rec + x.k_v4, x.v_v4, lane);
}

// Table entries of the up to kRowSeg blocks from uid_seg0 that this thread looks at (block e * THREADS +
// thread of the segment; -1 past the end or for a frame number outside the pool).
template <int THREADS, int E>
__device__ __forceinline__ void row_segment_load(const int32_t* __restrict__ slot_tbl, int64_t uid_seg0, int nbs,
                                                 uint32_t n_slots, int (&slot)[E]) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int b = e * THREADS + threadIdx.x;
        slot[e] = b < nbs ? slot_tbl[uid_seg0 + b] : -1;
    }
#pragma unroll
    for (int e = 0; e < E; ++e)
        if ((uint32_t)slot[e] >= n_slots) slot[e] = -1;
}

// Rank of each of these blocks among the resident blocks of the segment, in block order (-1 = not
// resident); with LIST the frames are also written to s_slot[rank].  Returns the number of resident
// blocks.  Two barriers.
template <bool LIST, int THREADS, int E>
__device__ __forceinline__ int row_segment_rank(const int (&slot)[E], int* s_slot, int* s_cnt, int (&rank)[E]) {
    constexpr int WAVES = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int within[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const uint64_t bal = __ballot(slot[e] >= 0);
        within[e] = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) s_cnt[e * WAVES + wave] = __popcll(bal);
    }
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        int base = total;
        for (int w = 0; w < WAVES; ++w) {
            const int c = s_cnt[e * WAVES + w];
            if (w < wave) base += c;
            total += c;
        }
        rank[e] = slot[e] >= 0 ? base + within[e] : -1;
        if (LIST && slot[e] >= 0) s_slot[rank[e]] = slot[e];
    }
    __syncthreads();
    return total;
}

template <int G, int DIM, int DT>
__global__ __launch_bounds__(RowShape<G>::kThreads) void score_row_kernel(PlanRows pr, RowArgs a, Xfer xf) {
    static_assert(G == 1 || G == 2 || G == 4 || G == 8, "power-of-two group sizes only");
    using RS = RowShape<G>;
    constexpr int THREADS = RS::kThreads, WAVES = RS::kWaves, E = RS::kE, CAP = RS::kCap;
    constexpr int NK = DIM / 32;
    constexpr int QROW_V4 = DIM / 8;
    constexpr int KEEP = 2;               // segments whose ranks stay in registers for the final phase
    extern __shared__ __align__(16) unsigned char row_smem[];
    int* s_slot = reinterpret_cast<int*>(row_smem);
    int* s_cnt = reinterpret_cast<int*>(row_smem + kRowSeg * 4);
    float2* s_red = reinterpret_cast<float2*>(row_smem + kRowSeg * 4 + 512);
    int* s_take = reinterpret_cast<int*>(row_smem + kRowSeg * 4 + 512 + THREADS * 8);
    float* s_val = reinterpret_cast<float*>(row_smem + RS::kFixed);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x;
    // This workgroup's transfer pairs are moved by its last wavefront once the first list is built (no barrier
    // follows until the segment's units are done, and the other wavefronts simply take more units meanwhile);
    // a workgroup without a row to score moves them at once.
    auto move_pairs = [&]() {
        if (xf.n && wave == WAVES - 1)
            for (uint32_t p = blockIdx.x; p < xf.n; p += gridDim.x) xfer_pair_wave(xf, p, lane);
    };
    if (!row_scorable(pr, row)) {                                         // uniform
        move_pairs();
        return;
    }
    // everything the loops below use, in plain locals (the argument block is not referenced from the lambdas)
    const int32_t* __restrict__ slot_tbl = a.slot_tbl;
    const uint4* __restrict__ k_pool = a.k_pool;
    float* __restrict__ spill = a.spill;
    float* __restrict__ mass = a.mass;
    const uint32_t n_slots = a.n_slots;
    const float scale = a.scale;
    const int agg = a.agg;
    const int ntok = pr.row_ntok[row];
    const int nb = (int)(((uint32_t)ntok + 15u) >> 4);
    const int64_t uid0 = pr.row_off[row];
    const int tail = ntok - 16 * (nb - 1);                                // tokens of the last block, 1..16
    constexpr bool MF = RS::kMf;
    const int t = lane & 15, cg = lane >> 4;   // dot2: token and channel group; MF: query column and token group
    const uint4* qrow = reinterpret_cast<const uint4*>(a.q + pr.row_q_off[row]);
    // table entries of the first segment, the queries and whether the row's last block is in HBM: one round trip
    int slot_cur[E], slot_nxt[E];
    row_segment_load<THREADS, E>(slot_tbl, uid0, min(kRowSeg, nb), n_slots, slot_cur);
    const bool last_resident = (uint32_t)slot_tbl[uid0 + nb - 1] < n_slots;
    // dot2: every lane holds its channel group of all G queries; MF: the B operands of one 16-column tile
    // (column = query t, zero beyond G)
    constexpr int NQ = MF ? 1 : G;
    uint4 qv[NQ][NK];
#pragma unroll
    for (int j = 0; j < NQ; ++j)
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
            if constexpr (MF) qv[j][kk] = t < G ? qrow[t * QROW_V4 + 4 * kk + cg] : make_uint4(0, 0, 0, 0);
            else qv[j][kk] = qrow[j * QROW_V4 + 4 * kk + cg];
        }

    int rank_keep[KEEP][E], nseg_keep[KEEP] = {0, 0};
    int n_tot = 0;                                                        // resident blocks so far (uniform)
    for (int seg0 = 0, si = 0; seg0 < nb; seg0 += kRowSeg, ++si) {
        const int nbs = min(kRowSeg, nb - seg0);
        if (threadIdx.x == 0) *s_take = 0;                                // the list's take counter
        int rank[E];
        const int n_seg = row_segment_rank<true, THREADS, E>(slot_cur, s_slot, s_cnt, rank);
        if (si == 0) move_pairs();
        if (si < KEEP) {
            nseg_keep[si < KEEP ? si : 0] = n_seg;
#pragma unroll
            for (int e = 0; e < E; ++e) rank_keep[si < KEEP ? si : 0][e] = rank[e];
        }
        // the next segment's table entries travel while this segment is scored
        const bool more = seg0 + kRowSeg < nb;
        if (more) row_segment_load<THREADS, E>(slot_tbl, uid0 + seg0 + kRowSeg, min(kRowSeg, nb - seg0 - kRowSeg), n_slots, slot_nxt);
        // is the row's last block (the only one that can be short) the last entry of this list?
        const bool last_listed = !more && last_resident;
        if (n_seg > 0) {
            auto fetch = [&](uint4 (&dst)[NK]) -> int {
                int v = 0;
                if (lane == 0) v = atomicAdd(s_take, 1);
                const int idx = __builtin_amdgcn_readfirstlane(v);
                const int sl = __builtin_amdgcn_readfirstlane(s_slot[idx < n_seg ? idx : n_seg - 1]);
                load_unit<NK>(dst, k_pool, (uint32_t)sl, DIM * 2, lane);
                return idx < n_seg ? idx : -1;
            };
            auto unit = [&](const uint4 (&cur)[NK], int i) {
                const int vi = n_tot + i;
                if constexpr (MF) {
                    // [16 tokens x DIM] . [DIM x 16 queries]: lane holds tokens 4 cg + 0..3 of query t
                    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) acc = mfma16<DT>(cur[kk], qv[0][kk], acc);
                    const int ntk = (last_listed && i == n_seg - 1) ? tail : 16;
                    float z[4];
                    float mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        z[r] = 4 * cg + r < ntk ? acc[r] * scale : -INFINITY;
                        mx = fmaxf(mx, z[r]);
                    }
                    mx = rows4_max(mx);                       // a block has at least one token: finite
                    float sm = 0.f;
#pragma unroll
                    for (int r = 0; r < 4; ++r) sm += __expf(z[r] - mx);
                    sm = rows4_sum(sm);
                    if (cg == 0 && t < G) {
                        const float lse = mx + __logf(sm);
                        if (vi < CAP) s_val[vi * G + t] = lse;
                        else spill[(size_t)(uid0 + vi) * G + t] = lse;
                    }
                    return;
                }
                const bool valid = !(last_listed && i == n_seg - 1) || t < tail;
#pragma unroll
                for (int j0 = 0; j0 < G; j0 += 4) {
                    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        if (j0 + jj < G) {
#pragma unroll
                            for (int kk = 0; kk < NK; ++kk) acc[jj] = dot8<DT>(cur[kk], qv[(j0 + jj) % NQ][kk], acc[jj]);
                        }
                    const float z = fold_rows(fold_halves(acc[0], acc[1]), fold_halves(acc[2], acc[3])) * scale;
                    const float zz = valid ? z : -INFINITY;
                    const float mx = row16_max(zz);
                    const float e = valid ? __expf(zz - mx) : 0.f;
                    const float sm = row16_sum(e);
                    const int jq = j0 + query_of_row(cg);
                    if (t == 0 && jq < G) {
                        const float lse = mx + __logf(sm);
                        if (vi < CAP) s_val[vi * G + jq] = lse;
                        else spill[(size_t)(uid0 + vi) * G + jq] = lse;
                    }
                }
            };
            uint4 b0[NK], b1[NK], b2[NK];
            int i0 = fetch(b0), i1, i2;
            if (i0 >= 0) {
                i1 = fetch(b1);
                while (true) {
                    i2 = fetch(b2);
                    unit(b0, i0);
                    if (i1 < 0) break;
                    i0 = fetch(b0);
                    unit(b1, i1);
                    if (i2 < 0) break;
                    i1 = fetch(b1);
                    unit(b2, i2);
                    if (i0 < 0) break;
                }
            }
        }
        n_tot += n_seg;
        if (more)
#pragma unroll
            for (int e = 0; e < E; ++e) slot_cur[e] = slot_nxt[e];
        __syncthreads();          // every value of the segment is written; list and counter may be reused
    }
    if (n_tot == 0) return;       // nothing of this row is in HBM (uniform)

    // ---- the row's log-sum-exp per query: maximum, then sum of exponentials, over the stored block values ------
    // (in a fixed order, so that the result does not depend on which wavefront scored which unit; keeping
    // running statistics in the unit loop instead was tried: the extra exponentials per unit made the launch
    // 4 % longer, with eight queries in registers the loop is short of issue slots, not of bytes)
    const int n_lds = min(n_tot, CAP);                // ranks below this are in LDS, the others in the spill array
    float L[G];
    {
        const int j = threadIdx.x % G;
        constexpr int STEP = THREADS / G, U = 8;      // U independent reads in flight per thread
        float mx = -INFINITY;
        for (int r0 = threadIdx.x / G; r0 < n_lds; r0 += STEP * U) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = s_val[min(r0 + u * STEP, n_lds - 1) * G + j];      // clamped: a repeat is harmless
#pragma unroll
            for (int u = 0; u < U; ++u) mx = fmaxf(mx, v[u]);
        }
        for (int r = CAP + threadIdx.x / G; r < n_tot; r += STEP) mx = fmaxf(mx, spill[(size_t)(uid0 + r) * G + j]);
#pragma unroll
        for (int d = G; d < 64; d <<= 1) mx = fmaxf(mx, __shfl_xor(mx, d));
        if (lane < G) s_red[wave * G + lane].x = mx;
        __syncthreads();
        float row_max = -INFINITY;
        for (int w = 0; w < WAVES; ++w) row_max = fmaxf(row_max, s_red[w * G + j].x);
        float sm = 0.f;
        if (row_max > -INFINITY) {
            for (int r0 = threadIdx.x / G; r0 < n_lds; r0 += STEP * U) {
                float v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = r0 + u * STEP < n_lds ? s_val[(r0 + u * STEP) * G + j] : -INFINITY;
#pragma unroll
                for (int u = 0; u < U; ++u) sm += __expf(v[u] - row_max);       // exp(-inf) = 0 past the end
            }
            for (int r = CAP + threadIdx.x / G; r < n_tot; r += STEP) sm += __expf(spill[(size_t)(uid0 + r) * G + j] - row_max);
        }
#pragma unroll
        for (int d = G; d < 64; d <<= 1) sm += __shfl_xor(sm, d);
        if (lane < G) s_red[wave * G + lane].y = sm;
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < G; ++jj) {
            float m2 = -INFINITY, z2 = 0.f;
            for (int w = 0; w < WAVES; ++w) {
                const float2 pz = s_red[w * G + jj];
                m2 = fmaxf(m2, pz.x);
                z2 += pz.y;
            }
            L[jj] = z2 > 0.f ? m2 + __logf(z2) : -INFINITY;
        }
    }
    // ---- masses: ranks from the scoring phase (kept for the first segments, the table once more beyond) -------
    int base = 0;
    for (int seg0 = 0, si = 0; seg0 < nb; seg0 += kRowSeg, ++si) {
        int rank[E];
        int n_seg = 0;
        if (si < KEEP) {
            n_seg = nseg_keep[si < KEEP ? si : 0];
#pragma unroll
            for (int e = 0; e < E; ++e) rank[e] = rank_keep[si < KEEP ? si : 0][e];
        } else {
            int slot[E];
            row_segment_load<THREADS, E>(slot_tbl, uid0 + seg0, min(kRowSeg, nb - seg0), n_slots, slot);
            n_seg = row_segment_rank<false, THREADS, E>(slot, s_slot, s_cnt, rank);
        }
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (rank[e] < 0) continue;
            const int r = base + rank[e];
            float l[G];
            if (r < CAP) {
#pragma unroll
                for (int j = 0; j < G; ++j) l[j] = s_val[r * G + j];
            } else {
#pragma unroll
                for (int j = 0; j < G; ++j) l[j] = spill[(size_t)(uid0 + r) * G + j];
            }
            float m = 0.f;                                               // masses are >= 0: neutral for max and sum
#pragma unroll
            for (int j = 0; j < G; ++j) {
                const float x = l[j] > -INFINITY ? __expf(l[j] - L[j]) : 0.f;
                m = agg == KVM_AGG_MAX ? fmaxf(m, x) : m + x;
            }
            // non-temporal: a plain store leaves a dirty line in the L2 whose write-back later competes with
            // the streaming reads (measured on rows of 8,192 blocks: 0.11 ms of a 6.7 ms launch)
            __builtin_nontemporal_store(agg == KVM_AGG_MAX ? m : m / (float)G,
                                        &mass[uid0 + seg0 + e * THREADS + threadIdx.x]);
        }
        base += n_seg;
    }
}

// ---- score_tile_mfma: any g <= 16 * NCT, queries as matrix-core operands -----------
// Per unit the logits are the dense product [16 tokens x dim] . [dim x g].  The queries
// are the B operands (column = query l%16 of a 16-query column tile, k = channel), loaded
// once per workgroup.  Result layout: lane l holds tokens 4*(l/16) + 0..3 of query l%16.
template <int NCT, int DIM, int DT, int T>
__global__ __launch_bounds__(kThreads) void score_tile_mfma_kernel(
    const Tile* __restrict__ tiles, const uint32_t* __restrict__ n_tiles, int G,
    const int32_t* __restrict__ slot_tbl, const uint4* __restrict__ k_pool, uint32_t n_slots,
    const uint16_t* __restrict__ q, float scale, TileOut out, Xfer xf) {
    constexpr int NK = DIM / 32;
    constexpr int QROW_V4 = DIM / 8;
    constexpr int GP = NCT * 16;          // 16, 32, 64 or 128
    __shared__ float s_lse[T * NCT * 16];
    __shared__ TileLds<T, GP> lds;

    uint32_t tile_id;
    if (xfer_role(xf, xcd_order(blockIdx.x, gridDim.x), &tile_id)) {     // this workgroup moves bytes instead of scoring
        xfer_pair(xf, tile_id);
        return;
    }
    // record and tile count are loaded together; the record of a position past the count is never used
    const TileCtx c = tile_ctx<T>(tiles, tile_id);
    if (tile_id >= *n_tiles) return;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, cg = lane >> 4;
    const uint4* qrow = reinterpret_cast<const uint4*>(q + c.q_off);

    uint4 qb[NCT][NK];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int j = ct * 16 + n;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk)
            qb[ct][kk] = j < G ? qrow[j * QROW_V4 + 4 * kk + cg] : make_uint4(0, 0, 0, 0);
    }
    for (int i = threadIdx.x; i < c.nbt * G; i += kThreads) s_lse[i] = -INFINITY;
    const int n_res = build_unit_list<T>(slot_tbl, c.uid0, c.nbt, n_slots, lds.list, lds.cnt);
    if (n_res == 0) {                            // nothing resident in this tile (uniform)
        // a row of several tiles still folds this tile's statistic: it must read as empty
        if (c.nb > T && (int)threadIdx.x < G) out.tile_lse[(size_t)tile_id * GP + threadIdx.x] = -INFINITY;
        return;
    }

    for_each_unit<NK>(lds.list, n_res, k_pool, DIM * 2, [&](const uint4 (&cur)[NK], int i_cur) {
        const int tok_in_block = min(16, c.ntok - 16 * (c.b0 + i_cur));
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) acc = mfma16<DT>(cur[kk], qb[ct][kk], acc);
            float z[4];
            float mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                z[r] = (4 * cg + r) < tok_in_block ? acc[r] * scale : -INFINITY;
                mx = fmaxf(mx, z[r]);
            }
            mx = rows4_max(mx);                      // the block has at least one token, so mx is finite
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) s += __expf(z[r] - mx);
            s = rows4_sum(s);
            const int j = ct * 16 + n;
            if (cg == 0 && j < G) s_lse[i_cur * G + j] = mx + __logf(s);
        }
    });
    __syncthreads();
    tile_epilogue<GP, T>(s_lse, lds.red, lds.v, G, c, tile_id, out, lds.list, n_res);
}

// ---- score_tile_wide: wide frames (MLA latent, dim 576) scored by up to 128 queries ---
// The 128 x dim query operands do not fit one wavefront's registers, so the four
// wavefronts of the workgroup split the queries (32 each, two column tiles) and share the
// unit through LDS.  Frames travel global -> LDS directly (global_load_lds, 16 bytes per
// lane, no staging registers) into a ring of kWideBufs buffers: while one unit is being
// multiplied the next kWideBufs - 1 are in flight, which is what the memory latency asks for
// at 18 KiB per unit and two workgroups per compute unit.  One barrier per unit.
// Every wavefront issues exactly kWideDma loads and one store per unit, all unconditional, so
// that "at most N vector memory operations outstanding" identifies which frames have landed.
// Block values go straight to part_lse (row stride 128 floats, padded queries land in the
// padding), the tile's own log-sum-exp per query is carried in registers; score_rowmerge_big
// finishes every row.
constexpr int kWideBufs = 4;
constexpr int kWideTileBlocks = 512;

template <int DIM, int DT, int TB>
__global__ __launch_bounds__(kThreads, 2) void score_tile_wide_kernel(
    const Tile* __restrict__ tiles, const uint32_t* __restrict__ n_tiles, int G,
    const int32_t* __restrict__ slot_tbl, const uint4* __restrict__ k_pool, uint32_t n_slots,
    const uint16_t* __restrict__ q, float scale, TileOut out, Xfer xf) {
    constexpr int NK = DIM / 32;
    constexpr int UNIT_V4 = DIM * 2;
    constexpr int QROW_V4 = DIM / 8;
    constexpr int PER_WAVE = UNIT_V4 / 4;          // 16-byte vectors each wavefront moves per unit
    constexpr int FULL = PER_WAVE / 64, REM = PER_WAVE % 64;
    constexpr int DMA = FULL + (REM ? 1 : 0);      // loads per wavefront per unit
    constexpr int OPS = DMA + 1;                   // vector memory operations per wavefront per unit
    static_assert(UNIT_V4 % 4 == 0, "unit must split over four wavefronts");
    __shared__ uint4 kb0[UNIT_V4];
    __shared__ uint4 kb1[UNIT_V4];
    __shared__ uint4 kb2[UNIT_V4];
    __shared__ uint4 kb3[UNIT_V4];
    __shared__ int2 s_list[TB];
    __shared__ int s_cnt[((TB + kThreads - 1) / kThreads) * 4];

    uint32_t tile_id;
    if (xfer_role(xf, xcd_order(blockIdx.x, gridDim.x), &tile_id)) {     // this workgroup moves bytes instead of scoring
        xfer_pair(xf, tile_id);
        return;
    }
    // record and tile count are loaded together; the record of a position past the count is never used
    const TileCtx c = tile_ctx<TB>(tiles, tile_id);
    if (tile_id >= *n_tiles) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, cg = lane >> 4;
    const uint4* qrow = reinterpret_cast<const uint4*>(q + c.q_off);

    uint4 qb[2][NK];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
        const int j = 32 * wave + ct * 16 + n;
        const uint4* qj = qrow + (j < G ? j : 0) * QROW_V4 + cg;       // padded queries repeat query 0
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) qb[ct][kk] = qj[4 * kk];
    }
    const int n_res = build_unit_list<TB>(slot_tbl, c.uid0, c.nbt, n_slots, s_list, s_cnt);
    constexpr float kLn2 = 0.6931471805599453f;
    const float scale2 = scale * 1.4426950408889634f;          // logits in log2 units
    MZ run[2] = {{-INFINITY, 0.f}, {-INFINITY, 0.f}};          // base-2 reference and sum of exp2(z - reference)
    if (n_res > 0) {                                  // uniform
        // global -> LDS, 16 bytes per lane, LDS destination = m0 + 16 * lane.  Written as asm so that
        // the waits stay under this kernel's control (see the wait counts below).
        auto dma_op = [&](const uint4* src, uint4* dst) {
            const uint32_t lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4*)dst;
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                         :
                         : "v"(src), "s"(__builtin_amdgcn_readfirstlane(lds))
                         : "memory", "m0");
        };
        auto dma = [&](uint4* buf, int idx) {
            const int2 e = list_entry(s_list, idx < n_res ? idx : n_res - 1);
            const uint4* src = k_pool + (size_t)(uint32_t)e.y * UNIT_V4 + wave * PER_WAVE + lane;
            uint4* dst = buf + wave * PER_WAVE;
#pragma unroll
            for (int i = 0; i < FULL; ++i) dma_op(src + 64 * i, dst + 64 * i);
            if (REM && lane < REM) dma_op(src + 64 * FULL, dst + 64 * FULL);
        };
        auto compute = [&](const uint4* buf, int idx) {
            const int i_cur = list_entry(s_list, idx).x;
            const uint4* kb = buf + lane;
            f32x4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
            constexpr int AHEAD = 4;
            uint4 a[AHEAD];
#pragma unroll
            for (int p = 0; p < AHEAD - 1; ++p) a[p] = kb[p * 64];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) {
                if (kk + AHEAD - 1 < NK) a[(kk + AHEAD - 1) % AHEAD] = kb[(kk + AHEAD - 1) * 64];
                acc[0] = mfma16<DT>(a[kk % AHEAD], qb[0][kk], acc[0]);
                acc[1] = mfma16<DT>(a[kk % AHEAD], qb[1][kk], acc[1]);
            }
            // Softmax statistics in the base-2 domain: one multiply takes the accumulator to
            // log2 units, v_exp / v_log are base 2 already; natural-log values are formed only
            // where they leave the kernel.
            const int tok_in_block = min(16, c.ntok - 16 * (c.b0 + i_cur));
            float* pl = out.part_lse + (size_t)(c.uid0 + i_cur) * 128 + 32 * wave + n;
            float z[2][4], ml[2];
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
#pragma unroll
                for (int r = 0; r < 4; ++r) z[ct][r] = acc[ct][r] * scale2;
                if (tok_in_block < 16) {              // only a row's last block can be short (uniform)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (4 * cg + r >= tok_in_block) z[ct][r] = -INFINITY;
                }
                ml[ct] = fmaxf(fmaxf(z[ct][0], z[ct][1]), fmaxf(z[ct][2], z[ct][3]));
            }
            // Exponentials are taken against a reference that the four rows of a query share: the
            // largest logit the query has met so far in this tile, refreshed only when a block
            // comes within 2^-60 of overflowing against it (first unit included; the branch is
            // uniform and almost never taken).  That saves the per-block maximum across rows and
            // makes the tile statistic a plain sum.  A block more than 2^126 below the reference
            // underflows to mass 0, which is what it is at any tolerance.
            if (__ballot(ml[0] - run[0].m > 60.f || ml[1] - run[1].m > 60.f)) {
#pragma unroll
                for (int ct = 0; ct < 2; ++ct) {
                    const float ref = rows4_max(fmaxf(run[ct].m, ml[ct]));
                    run[ct].z *= __builtin_amdgcn_exp2f(run[ct].m - ref);
                    run[ct].m = ref;
                }
            }
            float lse[2];
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                float sm = 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) sm += __builtin_amdgcn_exp2f(z[ct][r] - run[ct].m);
                sm = rows4_sum(sm);                   // every row of lanes now holds the block's sum
                lse[ct] = (run[ct].m + __builtin_amdgcn_logf(sm)) * kLn2;
                run[ct].z += sm;
            }
            // One store per wavefront and unit: lane rows 0 and 1 write the wavefront's 32 queries
            // (column tile 0 and 1), a whole 128-byte line; what block-value stores cost is the
            // number of line writes.  From asm for the same reason the loads are: the number of
            // vector memory operations per step must be exactly what the wait counts assume.
            if (cg < 2) {
                const float v = cg == 0 ? lse[0] : lse[1];
                asm volatile("global_store_dword %0, %1, off nt" : : "v"(pl + cg * 16), "v"(v) : "memory");
            }
        };
        // vmcnt(N): at most N vector memory operations of this wavefront still outstanding.  Behind
        // the loads of unit idx sit, in issue order, the rest of iteration idx - 3 (its store) and the
        // whole of iterations idx - 2 and idx - 1: 1 + 2 * OPS operations.
        constexpr int LAG = 1 + 2 * OPS;
        static_assert(kWideBufs == 4 && LAG < 64, "wait count assumes three units in flight");
        dma(kb0, 0);
        dma(kb1, 1);
        dma(kb2, 2);
        // the first three iterations have fewer operations behind the loads they wait for
        constexpr int W0 = 2 * DMA, W1 = 2 * DMA + 1, W2 = 2 * DMA + 2;
        int idx = 0;
#define KVM_VMCNT(N) (((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))
#define KVM_WIDE_STEP(CUR, TGT, N)                       \
    if (idx < n_res) {                                   \
        __builtin_amdgcn_s_waitcnt(KVM_VMCNT(N));        \
        __syncthreads();                                 \
        dma(TGT, idx + 3);                               \
        compute(CUR, idx);                               \
        ++idx;                                           \
    }
        KVM_WIDE_STEP(kb0, kb3, W0)
        KVM_WIDE_STEP(kb1, kb0, W1)
        KVM_WIDE_STEP(kb2, kb1, W2)
        KVM_WIDE_STEP(kb3, kb2, LAG)
        while (idx < n_res) {
            KVM_WIDE_STEP(kb0, kb3, LAG)
            KVM_WIDE_STEP(kb1, kb0, LAG)
            KVM_WIDE_STEP(kb2, kb1, LAG)
            KVM_WIDE_STEP(kb3, kb2, LAG)
        }
#undef KVM_VMCNT
#undef KVM_WIDE_STEP
    }
    if (cg == 0) {
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
            const int j = 32 * wave + ct * 16 + n;
            if (j < G)
                out.tile_lse[(size_t)tile_id * G + j] =
                    run[ct].z > 0.f ? (run[ct].m + __builtin_amdgcn_logf(run[ct].z)) * kLn2 : -INFINITY;
        }
    }
}

// Log-sum-exp of query j over the tile values first, first + STEP, ... of a row (n_t tiles, g
// values per tile), in two calls so that other loads can be issued in between: the first
// sixteen values are loaded at once, without a branch (most rows have no more), and folded
// later; a plain loop over the tiles would wait for every load in turn, and with sixteen tiles
// per row that chain was most of the kernel's time.
constexpr int kFoldBatch = 16;
struct TileVals {
    float x[kFoldBatch];
};
template <int STEP>
__device__ __forceinline__ TileVals load_tile_values(const float* __restrict__ tl, int g, int j, int first, int n_t) {
    TileVals t;
#pragma unroll
    for (int u = 0; u < kFoldBatch; ++u) {
        const int i = first + u * STEP;
        t.x[u] = tl[(size_t)(i < n_t ? i : 0) * g + j];
    }
    return t;
}
// (maximum, sum of exp(x - maximum)) of one batch whose first value is tile i0; no branches.
template <int STEP>
__device__ __forceinline__ MZ fold_batch(const TileVals& t, int i0, int n_t) {
    float x[kFoldBatch];
    float M = -INFINITY;
#pragma unroll
    for (int u = 0; u < kFoldBatch; ++u) {
        x[u] = i0 + u * STEP < n_t ? t.x[u] : -INFINITY;
        M = fmaxf(M, x[u]);
    }
    const float Ms = M == -INFINITY ? 0.f : M;
    float z = 0.f;
#pragma unroll
    for (int u = 0; u < kFoldBatch; ++u) z += __expf(x[u] - Ms);
    return MZ{M, z};
}
template <int STEP>
__device__ __forceinline__ MZ fold_tile_values(const TileVals& head, const float* __restrict__ tl, int g, int j,
                                               int first, int n_t) {
    MZ t = fold_batch<STEP>(head, first, n_t);
    for (int i0 = first + kFoldBatch * STEP; i0 < n_t; i0 += kFoldBatch * STEP) {     // rows of more than 16 tiles
        const TileVals more = load_tile_values<STEP>(tl, g, j, i0, n_t);
        t = mz_combine(t, fold_batch<STEP>(more, i0, n_t));
    }
    return t;
}

// ---- score_rowmerge: rows of more than one tile ---------------------------------------
// A fixed grid strides over the plan's list of tiles to visit (one 32-byte record each).  Per
// tile the first GP threads fold the tile values of the tile's row into the row's log sum exp
// (one query each, through LDS to the others); then every thread turns block values into
// masses, V = min(4, GP) queries of a block at a time from one vector load, GP / V lanes per
// block.  The kernel is bound by instruction issue and by the latency of its dependent loads,
// not by bytes: the record is the only load the data loads wait for, and those are issued, all
// of them, before anything is used.
template <int V>
struct RowVec;
template <>
struct RowVec<1> {
    typedef float type;
};
template <>
struct RowVec<2> {
    typedef float type __attribute__((ext_vector_type(2)));
};
template <>
struct RowVec<4> {
    typedef float type __attribute__((ext_vector_type(4)));
};
template <int V>
__device__ __forceinline__ float vec_elem(const typename RowVec<V>::type& v, int i) {
    if constexpr (V == 1)
        return v;
    else
        return v[i];
}

template <int GP, int T>
__global__ __launch_bounds__(kThreads) void score_rowmerge_kernel(
    const uint32_t* __restrict__ counts, const MergeTile* __restrict__ merge, int g,
    const int32_t* __restrict__ slot_tbl, uint32_t n_slots, TileOut o) {
    static_assert(GP <= 64, "larger groups take score_rowmerge_big");
    constexpr int V = GP < 4 ? GP : 4;      // queries per thread
    constexpr int LP = GP / V;              // lanes per block
    constexpr int BS = kThreads / LP;       // blocks per sweep
    constexpr int SWEEPS = (T + BS - 1) / BS;
    typedef typename RowVec<V>::type vec_t;
    __shared__ float s_row[GP];
    __shared__ int2 s_list[T];
    __shared__ int s_cnt[((T + kThreads - 1) / kThreads) * 4];
    const int l = threadIdx.x & (LP - 1), bsub = threadIdx.x / LP;
    const bool folds = threadIdx.x < GP;
    const int jf = folds && (int)threadIdx.x < g ? threadIdx.x : 0;
    const uint32_t n_merge = counts[1];
    for (uint32_t m = blockIdx.x; m < n_merge; m += gridDim.x) {
        const MergeTile e = merge[m];
        const int64_t uid0 = e.uid0;
        const float* tl = o.tile_lse + (size_t)e.tile0 * GP;
        // table entries and tile values first, in flight together; then the list of resident blocks
        // (the tile kernel packed its block values in the same order), then all the block values at once
        const TileSlots<T> slots = load_tile_slots<T>(slot_tbl, uid0, e.nbt);
        TileVals head;
        if (folds) head = load_tile_values<1>(tl, GP, jf, 0, e.n_t);
        const int n_res = build_unit_list<T>(slots, n_slots, s_list, s_cnt);
        vec_t v[SWEEPS];
#pragma unroll
        for (int k = 0; k < SWEEPS; ++k) {
            const int i = k * BS + bsub;
            v[k] = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(o.part_lse + (uid0 + (i < n_res ? i : 0)) * GP) + l);
        }
        if (folds) s_row[threadIdx.x] = mz_lse(fold_tile_values<1>(head, tl, GP, jf, 0, e.n_t));
        __syncthreads();
        float lse[V];
#pragma unroll
        for (int i = 0; i < V; ++i) lse[i] = s_row[l * V + i];
#pragma unroll
        for (int k = 0; k < SWEEPS; ++k) {
            // masses are >= 0, so 0 is neutral for the maximum as well as for the sum
            float r = 0.f;
#pragma unroll
            for (int i = 0; i < V; ++i) {
                const float x = l * V + i < g ? __expf(vec_elem<V>(v[k], i) - lse[i]) : 0.f;
                r = o.agg == KVM_AGG_MAX ? fmaxf(r, x) : r + x;
            }
            r = o.agg == KVM_AGG_MAX ? lanes_allreduce<LP, true>(r) : lanes_allreduce<LP, false>(r);
            const int i = k * BS + bsub;
            if (l == 0 && i < n_res) o.mass[uid0 + s_list[i].x] = o.agg == KVM_AGG_MAX ? r : r / (float)g;
        }
        __syncthreads();                     // s_row and the list are rebuilt for the next tile
    }
}

// The same for groups of more than 64 queries (g <= 128).  There a block's values fill 512
// bytes, so half a wavefront takes a whole resident block (one 16-byte load per lane, the
// group aggregate is a reduction over 32 lanes, no LDS exchange) and blocks that are not
// resident are never read: the workgroup first compacts the resident blocks of its tile into
// a list.
template <int TB /* blocks per tile of the plan */,
          bool ALL /* every tile of the plan (wide path: tile values have a row stride of g, not 128) */>
__global__ __launch_bounds__(kThreads) void score_rowmerge_big_kernel(
    const uint32_t* __restrict__ counts, const MergeTile* __restrict__ merge, int g,
    const int32_t* __restrict__ slot_tbl, uint32_t n_slots, TileOut o) {
    __shared__ int2 s_list[TB];
    __shared__ int s_cnt[((TB + kThreads - 1) / kThreads) * 4];
    __shared__ float2 s_mz[kThreads];
    __shared__ float s_rowlse[128];
    constexpr int gs = 128;                          // row stride of the block values
    const int ts = ALL ? g : 128;                    // row stride of the tile values
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t n_merge = counts[1];
    for (uint32_t m = blockIdx.x; m < n_merge; m += gridDim.x) {
        const MergeTile e = merge[m];
        const TileSlots<TB> slots = load_tile_slots<TB>(slot_tbl, e.uid0, e.nbt);   // in flight with the tile values
        // Row log-sum-exp per query, once per workgroup: thread (half, j) folds every second tile value
        // of query j, the two halves meet in LDS; then every lane picks up its two queries (lane, lane + 64).
        const float* tl = o.tile_lse + (size_t)e.tile0 * ts;
        {
            const int j = threadIdx.x & 127, half = threadIdx.x >> 7;
            const int jq = j < g ? j : 0;
            const MZ t = fold_tile_values<2>(load_tile_values<2>(tl, ts, jq, half, e.n_t), tl, ts, jq, half, e.n_t);
            s_mz[threadIdx.x] = make_float2(t.m, t.z);
        }
        const int n_res = build_unit_list<TB>(slots, n_slots, s_list, s_cnt);      // two barriers: s_mz is complete
        if (threadIdx.x < 128) {
            const float2 x = s_mz[threadIdx.x], y = s_mz[threadIdx.x + 128];
            s_rowlse[threadIdx.x] = mz_lse(mz_combine(MZ{x.x, x.y}, MZ{y.x, y.y}));
        }
        __syncthreads();
        // Half a wavefront per resident block: a lane takes four queries (one 16-byte load).
        const int ql = lane & 31, half = lane >> 5;
        float lse[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) lse[i] = s_rowlse[4 * ql + i];
        constexpr int U = 8;                             // loads in flight per lane
        for (int base = 0; base < n_res; base += 8 * U) {
            f32x4_t a[U];
            int blk[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = base + 8 * u + 2 * wave + half;
                blk[u] = s_list[i < n_res ? i : n_res - 1].x;
                a[u] = __builtin_nontemporal_load(
                    reinterpret_cast<const f32x4_t*>(o.part_lse + (size_t)(e.uid0 + (ALL ? blk[u] : (i < n_res ? i : n_res - 1))) * gs) + ql);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float r = 0.f;                           // masses are >= 0: neutral for maximum and sum
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float x = 4 * ql + i < g ? __expf(a[u][i] - lse[i]) : 0.f;
                    r = o.agg == KVM_AGG_MAX ? fmaxf(r, x) : r + x;
                }
                r = o.agg == KVM_AGG_MAX ? lanes_allreduce<32, true>(r) : lanes_allreduce<32, false>(r);
                if (ql == 0 && base + 8 * u + 2 * wave + half < n_res)
                    o.mass[e.uid0 + blk[u]] = o.agg == KVM_AGG_MAX ? r : r / (float)g;
            }
        }
        __syncthreads();                                 // the LDS arrays are rebuilt for the next tile
    }
}

// ---- host side ----------------------------------------------------------------
enum class Path { Dot2, Row, Mfma, Wide, None };

struct Choice {
    Path path;
    int tile_blocks;   // blocks per workgroup (what the plan cuts rows into)
    int nct;           // Mfma: 16-query column tiles (1, 2, 4 or 8)
};

// Larger groups of a small head go to the matrix-core kernel.  Eight queries as packed dot products are
// 128 vector instructions per block and 128 registers of query operands: measured against the matrix-core
// tile kernel (one half-empty column tile), rows of 512 blocks are a tie and rows of 128 blocks 8 % slower.
#ifndef KVM_DOT2_MAX_G
#define KVM_DOT2_MAX_G 4
#endif
constexpr int kDot2MaxG = KVM_DOT2_MAX_G;

// Which kernel scores (g, dim), and with what tile size.  The block-value array in LDS takes
// tile_blocks * (padded g) * 4 bytes: at most 32 KiB.
//
// Launches made of long rows go to the row kernel (one large workgroup per row, block values kept on
// chip): at least one row per compute unit and 2,048 blocks per row on average (uid space per row; the
// host does not see the lengths).  Shorter or fewer rows are cut into tiles as before.
constexpr int kRowMinRows = 256;
constexpr int kRowMinMeanBlocks = 2048;
Choice choose(int g, int dim, int64_t n_uids, int64_t n_rows) {
    if (dim <= 128 && (g == 1 || g == 2 || g == 4 || g == 8)) {
        if (n_rows >= kRowMinRows && n_uids / n_rows >= kRowMinMeanBlocks && n_rows <= 0x7fffffff)
            return Choice{Path::Row, kRowSeg, 0};
        if (g <= kDot2MaxG) return Choice{Path::Dot2, 512, 0};
    }
    if (dim <= 256) {
        const int nct = (g + 15) / 16;
        const int nct_p = nct <= 1 ? 1 : nct <= 2 ? 2 : nct <= 4 ? 4 : 8;
        return Choice{Path::Mfma, 512 / nct_p, nct_p};
    }
    if (dim == 576) return Choice{Path::Wide, kWideTileBlocks, 0};
    return Choice{Path::None, 256, 0};
}

inline int64_t max_tiles(int64_t n_uids, int64_t n_rows, int tile_blocks) {
    // rows do not overlap in uid space, so sum(ceil(nb_r / T)) <= n_uids / T + n_rows
    return n_uids / tile_blocks + n_rows;
}

struct ScoreWs {
    uint32_t* n_tiles;  // [3]: tiles of the plan, tiles of rows with more than one tile, "plan refused" flag
    uint64_t* wg_sum;
    Tile* tiles;
    MergeTile* merge;   // [tiles]: what the row merge visits
    float* tile_lse;    // [tiles][stride]
    float* part;        // block values [n_uids][g] (row stride 128 on the wide path)
    size_t bytes;
};

ScoreWs carve(void* ws, int64_t n_uids, int32_t n_rows, int32_t g, const Choice& ch) {
    if (ch.path == Path::Row) {          // only the spill array: block values that do not fit the LDS
        ScoreWs w{};
        w.part = reinterpret_cast<float*>(reinterpret_cast<uintptr_t>(ws) + 256);
        w.bytes = 256 + align_up((size_t)n_uids * (size_t)g * sizeof(float), 256);
        return w;
    }
    const int tile_blocks = ch.tile_blocks;
    const size_t n_wg = ((size_t)n_rows + kPlanThreads - 1) / kPlanThreads;
    const size_t tiles_max = (size_t)max_tiles(n_uids, n_rows, tile_blocks);
    const size_t off_sum = 256;
    const size_t off_tiles = off_sum + align_up(n_wg * sizeof(uint64_t), 256);
    const size_t off_merge = off_tiles + align_up(tiles_max * sizeof(Tile), 256);
    const size_t off_tmz = off_merge + align_up(tiles_max * sizeof(MergeTile), 256);
    // row stride of the block and tile values: see TileOut
    const size_t stride = ch.path == Path::Wide ? 128 : ch.path == Path::Mfma ? (size_t)ch.nct * 16 : (size_t)g;
    const size_t off_part = off_tmz + align_up(tiles_max * stride * sizeof(float), 256);
    const uintptr_t base = reinterpret_cast<uintptr_t>(ws);
    ScoreWs w;
    w.n_tiles = reinterpret_cast<uint32_t*>(base);
    w.wg_sum = reinterpret_cast<uint64_t*>(base + off_sum);
    w.tiles = reinterpret_cast<Tile*>(base + off_tiles);
    w.merge = reinterpret_cast<MergeTile*>(base + off_merge);
    w.tile_lse = reinterpret_cast<float*>(base + off_tmz);
    w.part = reinterpret_cast<float*>(base + off_part);
    w.bytes = off_part + align_up((size_t)n_uids * stride * sizeof(float), 256);
    return w;
}

struct ScoreArgs {
    const kvm_pool_t* pool;
    const kvm_rows_t* rows;
    const void* q;
    float scale;
    PlanRows pr;
    ScoreWs w;
    TileOut out;
    Xfer xf;           // n == 0: nothing rides along
    unsigned grid;     // scoring workgroups (upper bound on tiles); the tile kernels launch xf.n more
    hipStream_t st;
};

// Workgroups of a row-merge launch: enough to fill every compute unit several times over; they
// stride over the list of tiles to visit.
constexpr unsigned kMergeGrid = 8192;

template <int GP, int T>
int launch_rowmerge(const ScoreArgs& a) {
    TimedLaunch tl("score_finalize", a.st);
    const unsigned grid = a.grid < kMergeGrid ? a.grid : kMergeGrid;
    if constexpr (GP > 64) {
        score_rowmerge_big_kernel<T, false><<<grid, kThreads, 0, a.st>>>(a.w.n_tiles, a.w.merge, a.rows->g,
                                                                        a.rows->slot_tbl, (uint32_t)a.pool->n_slots, a.out);
        return launch_status("score_rowmerge_big");
    } else {
        score_rowmerge_kernel<GP, T><<<grid, kThreads, 0, a.st>>>(a.w.n_tiles, a.w.merge, a.rows->g, a.rows->slot_tbl,
                                                            (uint32_t)a.pool->n_slots, a.out);
        return launch_status("score_rowmerge");
    }
}

template <int G, int DIM, int DT>
int launch_dot2_path(const ScoreArgs& a) {
    {
        TimedLaunch tl("score_partial", a.st);
        score_tile_dot2_kernel<G, DIM, DT, 512><<<a.grid + a.xf.n, kThreads, 0, a.st>>>(
            a.w.tiles, a.w.n_tiles, a.rows->slot_tbl,
            static_cast<const uint4*>(a.pool->k_pool), (uint32_t)a.pool->n_slots, static_cast<const uint16_t*>(a.q),
            a.scale, a.out, a.xf);
        if (int rc = launch_status("score_tile_dot2")) return rc;
    }
    return launch_rowmerge<G, 512>(a);
}

template <int G, int DIM, int DT>
int launch_row_path(const ScoreArgs& a) {
    auto kern = score_row_kernel<G, DIM, DT>;
    // the kernel's 160 KB of dynamic LDS have to be allowed once per device (the attribute belongs to the
    // function as loaded on that device); later calls, also under stream capture, only launch
    static std::atomic<unsigned long long> allowed{0};
    int dev = 0;
    KVM_HIP_TRY(hipGetDevice(&dev));
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev > 63 || !(allowed.load(std::memory_order_acquire) & bit)) {
        KVM_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kRowLdsBytes));
        if (dev <= 63) allowed.fetch_or(bit, std::memory_order_release);
    }
    RowArgs ra{a.rows->slot_tbl, static_cast<const uint4*>(a.pool->k_pool), (uint32_t)a.pool->n_slots,
               static_cast<const uint16_t*>(a.q), a.scale, a.out.agg, a.out.mass, a.w.part};
    TimedLaunch tl("score_partial", a.st);
    kern<<<(unsigned)a.rows->n_rows, RowShape<G>::kThreads, kRowLdsBytes, a.st>>>(a.pr, ra, a.xf);
    return launch_status("score_row");
}

template <int NCT, int DIM, int DT>
int launch_mfma_path(const ScoreArgs& a) {
    constexpr int T = 512 / NCT;
    {
        TimedLaunch tl("score_partial", a.st);
        score_tile_mfma_kernel<NCT, DIM, DT, T><<<a.grid + a.xf.n, kThreads, 0, a.st>>>(
            a.w.tiles, a.w.n_tiles, a.rows->g, a.rows->slot_tbl, static_cast<const uint4*>(a.pool->k_pool), (uint32_t)a.pool->n_slots,
            static_cast<const uint16_t*>(a.q), a.scale, a.out, a.xf);
        if (int rc = launch_status("score_tile_mfma")) return rc;
    }
    return launch_rowmerge<NCT * 16, T>(a);
}

// Wide frames (dim 576): workgroup-cooperative matrix-core kernel.
template <int DIM, int DT>
int launch_wide_path(const ScoreArgs& a) {
    constexpr int TB = kWideTileBlocks;
    {
        // The kernel's wait counts assume that its only vector memory operations are the ones it issues
        // itself; register spills would add scratch traffic to the count.  Refuse to run such a build.
        static int scratch_bytes = -1;
        if (scratch_bytes < 0) {
            hipFuncAttributes attr;
            KVM_HIP_TRY(hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(score_tile_wide_kernel<DIM, DT, TB>)));
            scratch_bytes = (int)attr.localSizeBytes;
        }
        if (scratch_bytes != 0)
            return fail(KVM_EHIP, "kvm_score_step: the wide kernel was built with %d bytes of scratch per lane",
                        scratch_bytes);
    }
    {
        TimedLaunch tl("score_partial", a.st);
        score_tile_wide_kernel<DIM, DT, TB><<<a.grid + a.xf.n, kThreads, 0, a.st>>>(
            a.w.tiles, a.w.n_tiles, a.rows->g, a.rows->slot_tbl, static_cast<const uint4*>(a.pool->k_pool), (uint32_t)a.pool->n_slots,
            static_cast<const uint16_t*>(a.q), a.scale, a.out, a.xf);
        if (int rc = launch_status("score_tile_wide")) return rc;
    }
    TimedLaunch tl("score_finalize", a.st);
    score_rowmerge_big_kernel<TB, true><<<a.grid < kMergeGrid ? a.grid : kMergeGrid, kThreads, 0, a.st>>>(
        a.w.n_tiles, a.w.merge, a.rows->g, a.rows->slot_tbl, (uint32_t)a.pool->n_slots, a.out);
    return launch_status("score_rowmerge_big");
}

template <int DIM, int DT>
int launch_dim(const ScoreArgs& a, const Choice& ch) {
    if constexpr (DIM <= 128) {
        if (ch.path == Path::Row) {
            switch (a.rows->g) {
                case 1: return launch_row_path<1, DIM, DT>(a);
                case 2: return launch_row_path<2, DIM, DT>(a);
                case 4: return launch_row_path<4, DIM, DT>(a);
                default: return launch_row_path<8, DIM, DT>(a);
            }
        }
        if (ch.path == Path::Dot2) {
            switch (a.rows->g) {
                case 1: return launch_dot2_path<1, DIM, DT>(a);
                case 2: return launch_dot2_path<2, DIM, DT>(a);
                default: return launch_dot2_path<4, DIM, DT>(a);
            }
        }
    }
    if constexpr (DIM <= 256) {
        if (ch.path == Path::Mfma) {
            switch (ch.nct) {
                case 1: return launch_mfma_path<1, DIM, DT>(a);
                case 2: return launch_mfma_path<2, DIM, DT>(a);
                case 4: return launch_mfma_path<4, DIM, DT>(a);
                default: return launch_mfma_path<8, DIM, DT>(a);
            }
        }
    }
    if constexpr (DIM == 576) {
        if (ch.path == Path::Wide) return launch_wide_path<DIM, DT>(a);
    }
    return fail(KVM_ESHAPE, "kvm_score_step: no kernel for g %d, dim %d", a.rows->g, a.pool->dim);
}

template <int DT>
int launch_dtype(const ScoreArgs& a, const Choice& ch) {
    switch (a.pool->dim) {
        case 32: return launch_dim<32, DT>(a, ch);
        case 64: return launch_dim<64, DT>(a, ch);
        case 96: return launch_dim<96, DT>(a, ch);
        case 128: return launch_dim<128, DT>(a, ch);
        case 192: return launch_dim<192, DT>(a, ch);
        case 256: return launch_dim<256, DT>(a, ch);
        case 576: return launch_dim<576, DT>(a, ch);
        default: return fail(KVM_ESHAPE, "kvm_score_step: no kernel for dim %d", a.pool->dim);
    }
}

}  // namespace

size_t score_workspace_bytes(int64_t n_uids, int32_t n_rows, int32_t g, int32_t dim) {
    const Choice ch = choose(g, dim, n_uids, n_rows);
    return carve(nullptr, n_uids, n_rows, g, ch).bytes;
}

namespace {
int score_step(const kvm_pool_t* pool, const kvm_rows_t* rows, const void* q, float softmax_scale, int agg,
               float* mass, void* ws, size_t ws_bytes, const Xfer& xf, void* stream) {
    KVM_REQUIRE(pool && rows, KVM_EINVAL, "kvm_score_step: null descriptor");
    KVM_REQUIRE(rows->n_rows >= 0 && rows->n_uids >= 0 && rows->q_elems >= 0, KVM_EINVAL,
                "kvm_score_step: negative size");
    KVM_REQUIRE(agg == KVM_AGG_MAX || agg == KVM_AGG_MEAN, KVM_EINVAL, "kvm_score_step: agg %d", agg);
    KVM_REQUIRE(pool->dtype == KVM_BF16 || pool->dtype == KVM_FP16, KVM_ESHAPE, "kvm_score_step: dtype %d",
                pool->dtype);
    KVM_REQUIRE(pool->dim > 0 && pool->dim % 32 == 0, KVM_ESHAPE, "kvm_score_step: dim %d is not a multiple of 32",
                pool->dim);
    KVM_REQUIRE(pool->unit_k_bytes == (uint32_t)(KVM_BLOCK_TOKENS * pool->dim * 2), KVM_ESHAPE,
                "kvm_score_step: unit_k_bytes %u != 16 * dim * 2", pool->unit_k_bytes);
    KVM_REQUIRE(rows->g >= 1 && rows->g <= 128, KVM_ESHAPE, "kvm_score_step: g %d outside 1..128", rows->g);
    KVM_REQUIRE(pool->n_slots <= 0x7fffffffull, KVM_EINVAL, "kvm_score_step: n_slots exceeds int32 slot ids");
    if (rows->n_rows == 0 || rows->n_uids == 0) return KVM_OK;
    KVM_REQUIRE(pool->k_pool && q && mass && ws, KVM_EINVAL, "kvm_score_step: null buffer");
    KVM_REQUIRE(rows->row_ntok && rows->row_off && rows->row_q_off && rows->slot_tbl, KVM_EINVAL,
                "kvm_score_step: null row array");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(ws) % 256 == 0, KVM_EINVAL, "kvm_score_step: ws not 256-byte aligned");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(q) % 16 == 0 && reinterpret_cast<uintptr_t>(pool->k_pool) % 16 == 0,
                KVM_EINVAL, "kvm_score_step: q and k_pool must be 16-byte aligned");
    const Choice ch = choose(rows->g, pool->dim, rows->n_uids, rows->n_rows);
    ScoreArgs a;
    a.pool = pool;
    a.rows = rows;
    a.q = q;
    a.scale = softmax_scale;
    a.w = carve(ws, rows->n_uids, rows->n_rows, rows->g, ch);
    KVM_REQUIRE(ws_bytes >= a.w.bytes, KVM_ENOSPC, "kvm_score_step: workspace %zu < %zu bytes", ws_bytes, a.w.bytes);
    const int64_t tiles_max = max_tiles(rows->n_uids, rows->n_rows, ch.tile_blocks);
    KVM_REQUIRE(tiles_max <= 0x7fffffffll, KVM_ESHAPE, "kvm_score_step: too many tiles");
    a.out = TileOut{agg, mass, a.w.part, a.w.tile_lse};
    a.xf = xf;
    KVM_REQUIRE(tiles_max + xf.n <= 0x7fffffffll, KVM_ESHAPE, "kvm_score_step: grid too large");
    if (xf.n) {
        // Spread the transfers over the first half of the tiles, at most one workgroup in seven, and with
        // an odd stride: workgroups go to the eight XCDs in turn, so a stride of 8 puts every transfer
        // workgroup on the same XCD, whose compute units then finish late (the wide kernel's launch was
        // 4 % longer), and an even one on half or a quarter of them.
        int64_t stride = tiles_max / (2 * (int64_t)xf.n);
        stride = stride < 1 ? 1 : stride > 7 ? 7 : stride;
        if (stride % 2 == 0) --stride;
        a.xf.stride = (uint32_t)stride;
    }
    a.grid = (unsigned)tiles_max;
    a.st = static_cast<hipStream_t>(stream);
    a.pr = PlanRows{rows->n_rows, rows->g,        pool->dim,     ch.tile_blocks,  rows->n_uids,
                    rows->q_elems, rows->row_ntok, rows->row_off, rows->row_q_off, rows->row_active,
                    ch.path == Path::Wide};
    if (ch.path == Path::Row)            // no plan: workgroup r takes row r
        return pool->dtype == KVM_BF16 ? launch_dtype<KVM_BF16>(a, ch) : launch_dtype<KVM_FP16>(a, ch);
    const int n_wg = (rows->n_rows + kPlanThreads - 1) / kPlanThreads;
    {
        TimedLaunch tl("score_plan", a.st);
        plan_count_kernel<<<n_wg, kPlanThreads, 0, a.st>>>(a.pr, a.w.wg_sum);
        plan_scan_kernel<<<1, kPlanThreads, 0, a.st>>>(n_wg, a.w.wg_sum, a.w.n_tiles, (uint64_t)tiles_max);
        plan_emit_kernel<<<n_wg, kPlanThreads, 0, a.st>>>(a.pr, a.w.wg_sum, a.w.n_tiles, a.w.tiles, a.w.merge);
        if (int rc = launch_status("score_plan")) return rc;
    }
    return pool->dtype == KVM_BF16 ? launch_dtype<KVM_BF16>(a, ch) : launch_dtype<KVM_FP16>(a, ch);
}
}  // namespace
}  // namespace kvm

extern "C" int kvm_score_step(const kvm_pool_t* pool, const kvm_rows_t* rows, const void* q,
                              float softmax_scale, int agg, float* mass, void* ws, size_t ws_bytes,
                              void* stream) {
    kvm::clear_error();
    return kvm::score_step(pool, rows, q, softmax_scale, agg, mass, ws, ws_bytes, kvm::Xfer{}, stream);
}

extern "C" int kvm_score_step_xfer(const kvm_pool_t* pool, const kvm_rows_t* rows, const void* q,
                                   float softmax_scale, int agg, float* mass, void* ws, size_t ws_bytes,
                                   const int32_t* xfer_frame, const int64_t* xfer_host, int64_t n_pairs,
                                   void* host_tier, uint64_t tier_slots, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(pool, KVM_EINVAL, "kvm_score_step_xfer: null pool");
    KVM_REQUIRE(n_pairs >= 0 && n_pairs <= 0x7ffffffll, KVM_EINVAL, "kvm_score_step_xfer: n_pairs %lld out of range",
                (long long)n_pairs);
    Xfer xf{};
    if (n_pairs > 0) {
        KVM_REQUIRE(xfer_frame && xfer_host && host_tier, KVM_EINVAL, "kvm_score_step_xfer: null transfer buffer");
        KVM_REQUIRE(pool->unit_k_bytes % 16 == 0 && pool->unit_v_bytes % 16 == 0, KVM_ESHAPE,
                    "kvm_score_step_xfer: unit sizes must be multiples of 16");
        KVM_REQUIRE(pool->k_pool && (pool->v_pool || pool->unit_v_bytes == 0), KVM_EINVAL,
                    "kvm_score_step_xfer: null pool memory");
        KVM_REQUIRE(reinterpret_cast<uintptr_t>(host_tier) % 16 == 0, KVM_EINVAL,
                    "kvm_score_step_xfer: host tier must be 16-byte aligned");
        xf = Xfer{(uint32_t)n_pairs, 1u, xfer_frame, xfer_host, static_cast<uint4*>(pool->k_pool),
                  static_cast<uint4*>(pool->v_pool), static_cast<uint4*>(host_tier), pool->unit_k_bytes / 16,
                  pool->unit_v_bytes / 16, (uint32_t)(pool->n_slots < 0x7fffffffull ? pool->n_slots : 0x7fffffffull), tier_slots};
    }
    if (rows && (rows->n_rows == 0 || rows->n_uids == 0) && xf.n) {
        // nothing to score: the bytes still have to move
        hipStream_t st = static_cast<hipStream_t>(stream);
        TimedLaunch tl("swap", st);
        xfer_kernel<<<xf.n, kThreads, 0, st>>>(xf);
        return launch_status("xfer");
    }
    return score_step(pool, rows, q, softmax_scale, agg, mass, ws, ws_bytes, xf, stream);
}
