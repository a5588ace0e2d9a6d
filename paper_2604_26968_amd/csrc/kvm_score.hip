// kvm_score_step: softmax attention mass per (row, 16-token block) unit.
//
// What is computed is Eq. 1 of the paper restricted to the HBM-resident tokens
// of each row, summed per token block, then the maximum (or mean) over the
// query heads that share the KV head (GQA grouping rule, section 3.4).
//
// Structure (all kernels in this file):
//   plan_*            build the list of tiles = (row, first block) of at most 512 blocks
//                     for the active rows, on the device, so the scorer's grid has no
//                     idle workgroups whatever the spread of row lengths
//   score_tile        g in {1, 2, 4, 8}, queries in registers: one workgroup per tile, one
//                     wavefront per unit at a time.  Per (unit, query) block maximum m and
//                     sum s = sum exp(z - m) stay in LDS; the workgroup reduces them to the
//                     tile's (M, Z).  A row that fits one tile is finished on the spot (only
//                     the masses are written); otherwise the tile writes s*exp(m - M) per
//                     (unit, query), coalesced, plus its (M, Z), and
//   score_rowmerge    combines the tiles of such a row and writes its masses
//   score_partial_generic / score_finalize
//                     any g up to 128 and dim up to 576: queries staged in LDS, (m, s)
//                     pairs through global memory, one workgroup per row to finish
//
// The tile kernels are the only ones that touch K; they read every resident unit
// exactly once with non-temporal 16-byte loads that cover 1 KiB contiguous per
// wavefront instruction.  With the [dim/8][16][8] unit layout lane l holds token
// l%16, channel group 4*kk + l/16 of load kk, so a lane accumulates its share of
// q.k in registers and the only cross-lane traffic is a reduce-scatter over the
// four 16-lane rows (two row-swap instructions per four queries) followed by
// 16-lane DPP reductions for the block maximum and sum.
#include "kvm_internal.h"

namespace kvm {
namespace {

struct Tile {
    int32_t row;
    int32_t b0;
};

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

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
// The row-swap builtins return both swapped registers.  hipcc 7.2 folds r[0] + r[1]
// into r[0] + r[0] when the two results feed one add directly; passing them through an
// empty asm statement keeps them in distinct registers (the compiler still inserts the
// wait states the instruction needs).
__device__ __forceinline__ float add_swapped(unsigned x, unsigned y) {
    asm volatile("" : "+v"(x), "+v"(y));
    return __builtin_bit_cast(float, x) + __builtin_bit_cast(float, y);
}
// a, b hold partial sums in all four 16-lane rows.  Returns, in rows 0 and 1,
// a summed over row pairs (0,2) and (1,3); in rows 2 and 3 the same for b.
__device__ __forceinline__ float fold_halves(float a, float b) {
    auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
    return add_swapped(r[0], r[1]);
}
// a, b as returned by fold_halves.  Row 0 gets a's rows 0+1, row 1 b's rows 0+1,
// row 2 a's rows 2+3, row 3 b's rows 2+3.
__device__ __forceinline__ float fold_rows(float a, float b) {
    auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
    return add_swapped(r[0], r[1]);
}
// After fold_rows(fold_halves(a0, a1), fold_halves(a2, a3)) the 16-lane row
// `cg` holds the complete sum of a_{kQueryOfRow[cg]}.
__device__ __forceinline__ int query_of_row(int cg) { return ((cg & 1) << 1) | (cg >> 1); }

// ---- plan: tiles of the active rows ------------------------------------------
constexpr int kPlanThreads = 1024;

// Row metadata the plan needs; a row whose blocks or queries would fall outside the
// arrays is dropped here (it gets no tile) so that no kernel can index out of bounds.
struct PlanRows {
    int n_rows;
    int g, dim;
    int64_t n_uids, q_elems;
    const int32_t* row_ntok;
    const int64_t* row_off;
    const int64_t* row_q_off;
    const uint8_t* row_active;
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
    return (nb + kTileBlocks - 1) / kTileBlocks;
}

// Exclusive scan of one value per thread over a workgroup of kPlanThreads; returns the
// exclusive prefix and stores the workgroup total in *total.
__device__ uint32_t wg_exclusive_scan(uint32_t v, uint32_t* total) {
    __shared__ uint32_t wave_sums[kPlanThreads / kWave];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
    for (int w = 0; w < kPlanThreads / kWave; ++w) {
        const uint32_t s = wave_sums[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(PlanRows p, uint32_t* wg_sum) {
    const int r = blockIdx.x * kPlanThreads + threadIdx.x;
    uint32_t total;
    (void)wg_exclusive_scan(tiles_of_row(p, r), &total);
    if (threadIdx.x == 0) wg_sum[blockIdx.x] = total;
}

// One workgroup: turns wg_sum[0..n) into exclusive prefixes in place and writes the grand total.
__global__ __launch_bounds__(kPlanThreads) void plan_scan_kernel(int n, uint32_t* wg_sum, uint32_t* n_tiles) {
    uint32_t carry = 0;
    for (int base = 0; base < n; base += kPlanThreads) {
        const int i = base + threadIdx.x;
        const uint32_t v = i < n ? wg_sum[i] : 0;
        uint32_t total;
        const uint32_t ex = wg_exclusive_scan(v, &total);
        if (i < n) wg_sum[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) *n_tiles = carry;
}

__global__ __launch_bounds__(kPlanThreads) void plan_emit_kernel(PlanRows p, const uint32_t* wg_base, Tile* tiles,
                                                                 uint32_t* row_tile0) {
    const int r = blockIdx.x * kPlanThreads + threadIdx.x;
    const uint32_t nt = tiles_of_row(p, r);
    uint32_t total;
    const uint32_t first = wg_base[blockIdx.x] + wg_exclusive_scan(nt, &total);
    if (r < p.n_rows) row_tile0[r] = first;
    for (uint32_t i = 0; i < nt; ++i) tiles[first + i] = Tile{r, (int32_t)(i * kTileBlocks)};
}

// ---- shared pieces of the tile kernels ---------------------------------------------
constexpr int kTileThreads = 256;
constexpr int kEntriesPerThread = kTileBlocks / kTileThreads;
static_assert(kTileBlocks % kTileThreads == 0, "whole table entries per thread");

typedef unsigned v4u_t __attribute__((ext_vector_type(4)));

// Resident units of a tile, compacted into LDS as (block index in tile, pool frame), in
// block order: every thread looks at kEntriesPerThread table entries, a ballot + popcount
// gives each resident entry its place.  Returns the list length.  Ends with a barrier.
__device__ __forceinline__ int build_unit_list(const int32_t* __restrict__ slot_tbl, int64_t uid0, int nbt,
                                               uint32_t n_slots, int2* s_list, int* s_cnt /* [entries * 4] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int slot[kEntriesPerThread], within[kEntriesPerThread];
#pragma unroll
    for (int e = 0; e < kEntriesPerThread; ++e) {
        const int b = e * kTileThreads + threadIdx.x;
        slot[e] = b < nbt ? slot_tbl[uid0 + b] : -1;
        if ((uint32_t)slot[e] >= n_slots) slot[e] = -1;
        const uint64_t bal = __ballot(slot[e] >= 0);
        within[e] = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) s_cnt[e * 4 + wave] = __popcll(bal);
    }
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int e = 0; e < kEntriesPerThread; ++e) {
        int base = total;
        for (int w = 0; w < 4; ++w) {
            const int c = s_cnt[e * 4 + w];
            if (w < wave) base += c;
            total += c;
        }
        if (slot[e] >= 0) s_list[base + within[e]] = make_int2(e * kTileThreads + threadIdx.x, slot[e]);
    }
    __syncthreads();
    return total;
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

// Running softmax statistics: maximum m and z = sum exp(x - m).
struct MZ {
    float m, z;
};
__device__ __forceinline__ MZ mz_combine(MZ a, MZ b) {
    const float M = fmaxf(a.m, b.m);
    if (M == -INFINITY) return MZ{M, 0.f};
    return MZ{M, a.z * __expf(a.m - M) + b.z * __expf(b.m - M)};
}

// ---- score_tile: g in {1, 2, 4, 8}, queries in registers ----------------------------
template <int G, int DIM, int DT>
__global__ __launch_bounds__(kTileThreads) void score_tile_kernel(
    const Tile* __restrict__ tiles, const uint32_t* __restrict__ n_tiles, const int32_t* __restrict__ row_ntok,
    const int64_t* __restrict__ row_off, const int64_t* __restrict__ row_q_off,
    const int32_t* __restrict__ slot_tbl, const uint4* __restrict__ k_pool, uint32_t n_slots,
    const uint16_t* __restrict__ q, float scale, int agg, float* __restrict__ mass, float* __restrict__ part_r,
    float2* __restrict__ tile_mz) {
    static_assert(G == 1 || G == 2 || G == 4 || G == 8, "power-of-two group sizes only");
    constexpr int NK = DIM / 32;          // 16-byte loads per lane per unit
    constexpr int UNIT_V4 = DIM * 2;      // 16-byte vectors per unit
    constexpr int QROW_V4 = DIM / 8;      // 16-byte vectors per query
    constexpr int BS = kTileThreads / G;  // blocks per sweep of the epilogue
    __shared__ float2 s_ms[kTileBlocks * G];   // (m, s) per (block, query); (-inf, 0) = not resident
    __shared__ int2 s_list[kTileBlocks];
    __shared__ int s_cnt[kEntriesPerThread * 4];
    __shared__ float2 s_red[4][G];

    if (blockIdx.x >= *n_tiles) return;
    const Tile tile = tiles[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = lane & 15, cg = lane >> 4;
    const int ntok = row_ntok[tile.row];
    const int nb = (ntok + 15) >> 4;
    const int nbt = min(kTileBlocks, nb - tile.b0);
    const int64_t uid0 = row_off[tile.row] + tile.b0;
    const uint4* qrow = reinterpret_cast<const uint4*>(q + row_q_off[tile.row]);

    uint4 qv[G][NK];
#pragma unroll
    for (int j = 0; j < G; ++j)
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) qv[j][kk] = qrow[j * QROW_V4 + 4 * kk + cg];

    for (int i = threadIdx.x; i < nbt * G; i += kTileThreads) s_ms[i] = make_float2(-INFINITY, 0.f);
    const int n_res = build_unit_list(slot_tbl, uid0, nbt, n_slots, s_list, s_cnt);
    if (n_res == 0) return;                      // nothing resident in this tile (uniform)

    // Wavefront w takes list entries w, w + 4, ...: balanced whatever the residency pattern.
    // Two units in flight per wavefront.  The loads of the following unit are issued
    // unconditionally (past the end of the list they re-read the last unit, a cache hit): a
    // branch around them would make the compiler wait for every outstanding load before the
    // first use of the current unit, which serialises load and compute.
    uint4 cur[NK], nxt[NK];
    int idx = wave;
    int i_cur = -1;
    if (idx < n_res) {
        const int2 e = list_entry(s_list, idx);
        i_cur = e.x;
        load_unit<NK>(cur, k_pool, (uint32_t)e.y, UNIT_V4, lane);
    }
    while (i_cur >= 0) {
        idx += 4;
        const int2 e_nxt = list_entry(s_list, idx < n_res ? idx : n_res - 1);
        const int i_nxt = idx < n_res ? e_nxt.x : -1;
        load_unit<NK>(nxt, k_pool, (uint32_t)e_nxt.y, UNIT_V4, lane);

        const int tok_in_block = min(16, ntok - 16 * (tile.b0 + i_cur));
        const bool valid = t < tok_in_block;
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
            if (t == 0 && jq < G) s_ms[i_cur * G + jq] = make_float2(mx, s);
        }
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) cur[kk] = nxt[kk];
        i_cur = i_nxt;
    }
    __syncthreads();

    // Tile statistics per query: thread (bsub, j) sweeps blocks bsub, bsub + BS, ...
    const int j = threadIdx.x & (G - 1), bsub = threadIdx.x / G;
    MZ acc{-INFINITY, 0.f};
    for (int b = bsub; b < nbt; b += BS) {
        const float2 p = s_ms[b * G + j];
        acc = mz_combine(acc, MZ{p.x, p.y});
    }
#pragma unroll
    for (int d = G; d < 64; d <<= 1) acc = mz_combine(acc, MZ{__shfl_xor(acc.m, d), __shfl_xor(acc.z, d)});
    if (lane < G) s_red[wave][lane] = make_float2(acc.m, acc.z);
    __syncthreads();
    MZ tot{s_red[0][j].x, s_red[0][j].y};
#pragma unroll
    for (int w = 1; w < 4; ++w) tot = mz_combine(tot, MZ{s_red[w][j].x, s_red[w][j].y});

    if (nb <= kTileBlocks) {
        // the row is this tile: finish it here
        const float inv = 1.f / tot.z;                  // n_res > 0, so tot.z >= 1
        for (int b0 = 0; b0 < nbt; b0 += BS) {
            const int b = b0 + bsub;
            const float2 p = b < nbt ? s_ms[b * G + j] : make_float2(-INFINITY, 0.f);
            float v = p.y * __expf(p.x - tot.m) * inv;  // exp(-inf) = 0 for blocks that are not resident
#pragma unroll
            for (int d = G / 2; d >= 1; d >>= 1) {
                const float o = __shfl_xor(v, d);
                v = agg == KVM_AGG_MAX ? fmaxf(v, o) : v + o;
            }
            if (j == 0 && p.y > 0.f) mass[uid0 + b] = agg == KVM_AGG_MAX ? v : v * (1.f / G);
        }
    } else {
        // s * exp(m - M_tile) per (unit, query), contiguous for the whole tile; 0 where not resident
        for (int i = threadIdx.x; i < nbt * G; i += kTileThreads) {
            const float2 p = s_ms[i];
            part_r[uid0 * G + i] = p.y * __expf(p.x - tot.m);
        }
        if (threadIdx.x < G) tile_mz[(size_t)blockIdx.x * G + threadIdx.x] = make_float2(tot.m, tot.z);
    }
}

// ---- score_rowmerge: rows of more than one tile, g in {1, 2, 4, 8} -------------------
// One workgroup per tile again: it folds the (M, Z) of all tiles of its row (a few pairs,
// read by every thread) and rescales its own tile's values into masses.
template <int G>
__global__ __launch_bounds__(kTileThreads) void score_rowmerge_kernel(
    const Tile* __restrict__ tiles, const uint32_t* __restrict__ n_tiles, const int32_t* __restrict__ row_ntok,
    const int64_t* __restrict__ row_off, const uint32_t* __restrict__ row_tile0,
    const int32_t* __restrict__ slot_tbl, uint32_t n_slots, const float* __restrict__ part_r,
    const float2* __restrict__ tile_mz, int agg, float* __restrict__ mass) {
    constexpr int BS = kTileThreads / G;
    if (blockIdx.x >= *n_tiles) return;
    const Tile tile = tiles[blockIdx.x];
    const int nb = (row_ntok[tile.row] + 15) >> 4;
    if (nb <= kTileBlocks) return;                   // finished by its tile
    const int nbt = min(kTileBlocks, nb - tile.b0);
    const int64_t uid0 = row_off[tile.row] + tile.b0;
    const float2* tmz = tile_mz + (size_t)row_tile0[tile.row] * G;
    const int n_t = (nb + kTileBlocks - 1) / kTileBlocks;
    const int j = threadIdx.x & (G - 1), bsub = threadIdx.x / G;
    MZ tot{-INFINITY, 0.f};
    for (int i = 0; i < n_t; ++i) {
        const float2 p = tmz[i * G + j];
        tot = mz_combine(tot, MZ{p.x, p.y});
    }
    // this tile's factor exp(M_tile - M_row) / Z_row
    const float f = tot.z > 0.f ? __expf(tile_mz[(size_t)blockIdx.x * G + j].x - tot.m) / tot.z : 0.f;
    // All loads first (unconditional, clamped), then the arithmetic: one round trip per tile.
    constexpr int SWEEPS = kTileBlocks / BS;
    float r[SWEEPS];
    int32_t slot[SWEEPS];
#pragma unroll
    for (int k = 0; k < SWEEPS; ++k) {
        const int b = k * BS + bsub;
        const int bc = b < nbt ? b : 0;
        slot[k] = slot_tbl[uid0 + bc];
        r[k] = part_r[(uid0 + bc) * G + j];
    }
#pragma unroll
    for (int k = 0; k < SWEEPS; ++k) {
        const int b = k * BS + bsub;
        const bool res = b < nbt && (uint32_t)slot[k] < n_slots;
        float v = res ? r[k] * f : 0.f;
#pragma unroll
        for (int d = G / 2; d >= 1; d >>= 1) {
            const float o = __shfl_xor(v, d);
            v = agg == KVM_AGG_MAX ? fmaxf(v, o) : v + o;
        }
        if (res && j == 0) mass[uid0 + b] = agg == KVM_AGG_MAX ? v : v * (1.f / G);
    }
}

// ---- score_partial_generic: any g, queries staged in LDS, (m, s) pairs to global -----
template <int DIM, int DT>
__global__ __launch_bounds__(kTileThreads) void score_partial_generic_kernel(
    const Tile* __restrict__ tiles, const uint32_t* __restrict__ n_tiles, int G,
    const int32_t* __restrict__ row_ntok, const int64_t* __restrict__ row_off,
    const int64_t* __restrict__ row_q_off, const int32_t* __restrict__ slot_tbl,
    const uint4* __restrict__ k_pool, uint32_t n_slots, const uint16_t* __restrict__ q, float scale,
    float2* __restrict__ part) {
    constexpr int NK = DIM / 32;
    constexpr int UNIT_V4 = DIM * 2;
    constexpr int QROW_V4 = DIM / 8;
    extern __shared__ uint4 q_lds[];      // [g][QROW_V4]
    __shared__ int2 s_list[kTileBlocks];
    __shared__ int s_cnt[kEntriesPerThread * 4];

    if (blockIdx.x >= *n_tiles) return;
    const Tile tile = tiles[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = lane & 15, cg = lane >> 4;
    const int ntok = row_ntok[tile.row];
    const int nb = (ntok + 15) >> 4;
    const int nbt = min(kTileBlocks, nb - tile.b0);
    const int64_t uid0 = row_off[tile.row] + tile.b0;
    const uint4* qrow = reinterpret_cast<const uint4*>(q + row_q_off[tile.row]);
    for (int i = threadIdx.x; i < G * QROW_V4; i += kTileThreads) q_lds[i] = qrow[i];
    const int n_res = build_unit_list(slot_tbl, uid0, nbt, n_slots, s_list, s_cnt);   // barriers cover q_lds too

    uint4 cur[NK], nxt[NK];
    int idx = wave;
    int i_cur = -1;
    if (idx < n_res) {
        const int2 e = list_entry(s_list, idx);
        i_cur = e.x;
        load_unit<NK>(cur, k_pool, (uint32_t)e.y, UNIT_V4, lane);
    }
    while (i_cur >= 0) {
        idx += 4;
        const int2 e_nxt = list_entry(s_list, idx < n_res ? idx : n_res - 1);
        const int i_nxt = idx < n_res ? e_nxt.x : -1;
        load_unit<NK>(nxt, k_pool, (uint32_t)e_nxt.y, UNIT_V4, lane);

        const int tok_in_block = min(16, ntok - 16 * (tile.b0 + i_cur));
        const bool valid = t < tok_in_block;
        float2* out = part + (uid0 + i_cur) * G;
        for (int j0 = 0; j0 < G; j0 += 4) {
            float a[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (j0 + jj < G) {
                    const uint4* qj = q_lds + (j0 + jj) * QROW_V4 + cg;
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) a[jj] = dot8<DT>(cur[kk], qj[4 * kk], a[jj]);
                }
            const float z = fold_rows(fold_halves(a[0], a[1]), fold_halves(a[2], a[3])) * scale;
            const float zz = valid ? z : -INFINITY;
            const float mx = row16_max(zz);
            const float e = valid ? __expf(zz - mx) : 0.f;
            const float s = row16_sum(e);
            const int jq = j0 + query_of_row(cg);
            if (t == 0 && jq < G) out[jq] = make_float2(mx, s);
        }
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) cur[kk] = nxt[kk];
        i_cur = i_nxt;
    }
}

// ---- score_finalize -----------------------------------------------------------
// GP = smallest power of two >= g.  Thread (bsub, j) = (tid / GP, tid % GP)
// handles query j of blocks bsub, bsub + 256/GP, ...
template <int GP>
__global__ __launch_bounds__(256) void score_finalize_kernel(
    PlanRows pr, const int32_t* __restrict__ slot_tbl, uint32_t n_slots, const float2* __restrict__ part, int agg,
    float* __restrict__ mass) {
    constexpr int BS = 256 / GP;
    __shared__ float sM[256], sZ[256];
    __shared__ float sV[256];
    const int row = blockIdx.x;
    if (!row_scorable(pr, row)) return;
    const int g = pr.g;
    const int nb = (pr.row_ntok[row] + 15) >> 4;
    const int64_t uid0 = pr.row_off[row];
    const int j = threadIdx.x % GP, bsub = threadIdx.x / GP;
    const bool jv = j < g;

    float M = -INFINITY, Z = 0.f;
    for (int b = bsub; b < nb; b += BS) {
        if (!jv || (uint32_t)slot_tbl[uid0 + b] >= n_slots) continue;
        const float2 p = part[(uid0 + b) * g + j];
        if (p.x > M) {
            Z = Z * __expf(M - p.x) + p.y;
            M = p.x;
        } else {
            Z += p.y * __expf(p.x - M);
        }
    }
    sM[threadIdx.x] = M;
    sZ[threadIdx.x] = Z;
    __syncthreads();
    float Mj = -INFINITY;
    for (int i = 0; i < BS; ++i) Mj = fmaxf(Mj, sM[i * GP + j]);
    float Zj = 0.f;
    for (int i = 0; i < BS; ++i) {
        const float m = sM[i * GP + j];
        if (m > -INFINITY) Zj += sZ[i * GP + j] * __expf(m - Mj);
    }
    const float inv = Zj > 0.f ? 1.f / Zj : 0.f;

    for (int b0 = 0; b0 < nb; b0 += BS) {
        const int b = b0 + bsub;
        const bool res = b < nb && (uint32_t)slot_tbl[uid0 + (b < nb ? b : 0)] < n_slots;
        float v = 0.f;
        if (res && jv) {
            const float2 p = part[(uid0 + b) * g + j];
            v = p.y * __expf(p.x - Mj) * inv;
        }
        // combine the GP queries of the block (masses are >= 0, so 0 is neutral for max too)
        if constexpr (GP <= 64) {
#pragma unroll
            for (int d = GP / 2; d >= 1; d >>= 1) {
                const float o = __shfl_xor(v, d);
                v = agg == KVM_AGG_MAX ? fmaxf(v, o) : v + o;
            }
        } else {
            __syncthreads();
            sV[threadIdx.x] = v;
            __syncthreads();
            if (j == 0) {
                for (int i = 1; i < GP; ++i) {
                    const float o = sV[bsub * GP + i];
                    v = agg == KVM_AGG_MAX ? fmaxf(v, o) : v + o;
                }
            }
        }
        if (res && j == 0) mass[uid0 + b] = agg == KVM_AGG_MAX ? v : v / (float)g;
    }
}

// ---- host side ----------------------------------------------------------------
struct ScoreWs {
    uint32_t* n_tiles;
    uint32_t* wg_sum;
    Tile* tiles;
    uint32_t* row_tile0;
    float2* tile_mz;
    float2* part;       // (m, s) pairs [n_uids][g] (generic path) or floats [n_uids][g] (tile path)
    size_t bytes;
};

ScoreWs carve(void* ws, int64_t n_uids, int32_t n_rows, int32_t g) {
    const size_t n_wg = ((size_t)n_rows + kPlanThreads - 1) / kPlanThreads;
    const size_t tiles_max = (size_t)max_tiles(n_uids, n_rows);
    const size_t off_sum = 256;
    const size_t off_tiles = off_sum + align_up(n_wg * sizeof(uint32_t), 256);
    const size_t off_row0 = off_tiles + align_up(tiles_max * sizeof(Tile), 256);
    const size_t off_tmz = off_row0 + align_up((size_t)n_rows * sizeof(uint32_t), 256);
    const size_t off_part = off_tmz + align_up(tiles_max * (size_t)g * sizeof(float2), 256);
    const uintptr_t base = reinterpret_cast<uintptr_t>(ws);
    ScoreWs w;
    w.n_tiles = reinterpret_cast<uint32_t*>(base);
    w.wg_sum = reinterpret_cast<uint32_t*>(base + off_sum);
    w.tiles = reinterpret_cast<Tile*>(base + off_tiles);
    w.row_tile0 = reinterpret_cast<uint32_t*>(base + off_row0);
    w.tile_mz = reinterpret_cast<float2*>(base + off_tmz);
    w.part = reinterpret_cast<float2*>(base + off_part);
    w.bytes = off_part + align_up((size_t)n_uids * (size_t)g * sizeof(float2), 256);
    return w;
}

struct ScoreArgs {
    const kvm_pool_t* pool;
    const kvm_rows_t* rows;
    const void* q;
    float scale;
    int agg;
    float* mass;
    PlanRows pr;
    ScoreWs w;
    unsigned grid;
    hipStream_t st;
};

// g in {1, 2, 4, 8} with the queries small enough for registers: tile kernel + row merge.
template <int G, int DIM, int DT>
int launch_tile_path(const ScoreArgs& a) {
    const uint4* kp = static_cast<const uint4*>(a.pool->k_pool);
    const uint32_t ns = (uint32_t)a.pool->n_slots;
    {
        TimedLaunch tl("score_partial", a.st);
        score_tile_kernel<G, DIM, DT><<<a.grid, kTileThreads, 0, a.st>>>(
            a.w.tiles, a.w.n_tiles, a.rows->row_ntok, a.rows->row_off, a.rows->row_q_off, a.rows->slot_tbl, kp, ns,
            static_cast<const uint16_t*>(a.q), a.scale, a.agg, a.mass, reinterpret_cast<float*>(a.w.part),
            a.w.tile_mz);
        if (int rc = launch_status("score_tile")) return rc;
    }
    TimedLaunch tl("score_finalize", a.st);
    score_rowmerge_kernel<G><<<a.grid, kTileThreads, 0, a.st>>>(
        a.w.tiles, a.w.n_tiles, a.rows->row_ntok, a.rows->row_off, a.w.row_tile0, a.rows->slot_tbl, ns,
        reinterpret_cast<const float*>(a.w.part), a.w.tile_mz, a.agg, a.mass);
    return launch_status("score_rowmerge");
}

template <int DIM, int DT>
int launch_generic_path(const ScoreArgs& a) {
    const int g = a.rows->g;
    const uint32_t ns = (uint32_t)a.pool->n_slots;
    const size_t lds = (size_t)g * (DIM / 8) * sizeof(uint4);
    auto kern = score_partial_generic_kernel<DIM, DT>;
    if (lds + 8 * 1024 > 160 * 1024)
        return fail(KVM_ESHAPE, "kvm_score_step: g %d x dim %d queries do not fit LDS", g, DIM);
    if (lds > 32 * 1024)
        KVM_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    {
        TimedLaunch tl("score_partial", a.st);
        kern<<<a.grid, kTileThreads, lds, a.st>>>(a.w.tiles, a.w.n_tiles, g, a.rows->row_ntok, a.rows->row_off,
                                                  a.rows->row_q_off, a.rows->slot_tbl,
                                                  static_cast<const uint4*>(a.pool->k_pool), ns,
                                                  static_cast<const uint16_t*>(a.q), a.scale, a.w.part);
        if (int rc = launch_status("score_partial_generic")) return rc;
    }
    TimedLaunch tl("score_finalize", a.st);
    int gp = 1;
    while (gp < g) gp <<= 1;
#define KVM_FIN(GP)                                                                                             \
    case GP:                                                                                                    \
        score_finalize_kernel<GP><<<a.rows->n_rows, 256, 0, a.st>>>(a.pr, a.rows->slot_tbl, ns, a.w.part, a.agg, \
                                                                    a.mass);                                    \
        break;
    switch (gp) {
        KVM_FIN(1) KVM_FIN(2) KVM_FIN(4) KVM_FIN(8) KVM_FIN(16) KVM_FIN(32) KVM_FIN(64) KVM_FIN(128)
        default: return fail(KVM_ESHAPE, "kvm_score_step: g %d", g);
    }
#undef KVM_FIN
    return launch_status("score_finalize");
}

template <int DIM, int DT>
int launch_dim(const ScoreArgs& a) {
    if constexpr (DIM <= 128) {
        switch (a.rows->g) {
            case 1: return launch_tile_path<1, DIM, DT>(a);
            case 2: return launch_tile_path<2, DIM, DT>(a);
            case 4: return launch_tile_path<4, DIM, DT>(a);
            case 8: return launch_tile_path<8, DIM, DT>(a);
            default: break;
        }
    }
    return launch_generic_path<DIM, DT>(a);
}

template <int DT>
int launch_dtype(const ScoreArgs& a) {
    switch (a.pool->dim) {
        case 32: return launch_dim<32, DT>(a);
        case 64: return launch_dim<64, DT>(a);
        case 96: return launch_dim<96, DT>(a);
        case 128: return launch_dim<128, DT>(a);
        case 192: return launch_dim<192, DT>(a);
        case 256: return launch_dim<256, DT>(a);
        case 576: return launch_dim<576, DT>(a);
        default: return fail(KVM_ESHAPE, "kvm_score_step: no kernel for dim %d", a.pool->dim);
    }
}

}  // namespace

size_t score_workspace_bytes(int64_t n_uids, int32_t n_rows, int32_t g) {
    return carve(nullptr, n_uids, n_rows, g).bytes;
}

}  // namespace kvm

extern "C" int kvm_score_step(const kvm_pool_t* pool, const kvm_rows_t* rows, const void* q,
                              float softmax_scale, int agg, float* mass, void* ws, size_t ws_bytes,
                              void* stream) {
    using namespace kvm;
    clear_error();
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
    ScoreArgs a;
    a.pool = pool;
    a.rows = rows;
    a.q = q;
    a.scale = softmax_scale;
    a.agg = agg;
    a.mass = mass;
    a.w = carve(ws, rows->n_uids, rows->n_rows, rows->g);
    KVM_REQUIRE(ws_bytes >= a.w.bytes, KVM_ENOSPC, "kvm_score_step: workspace %zu < %zu bytes", ws_bytes, a.w.bytes);
    const int64_t tiles_max = max_tiles(rows->n_uids, rows->n_rows);
    KVM_REQUIRE(tiles_max <= 0x7fffffffll, KVM_ESHAPE, "kvm_score_step: too many tiles");
    a.grid = (unsigned)tiles_max;
    a.st = static_cast<hipStream_t>(stream);
    a.pr = PlanRows{rows->n_rows, rows->g,        pool->dim,       rows->n_uids,    rows->q_elems,
                    rows->row_ntok, rows->row_off, rows->row_q_off, rows->row_active};
    const int n_wg = (rows->n_rows + kPlanThreads - 1) / kPlanThreads;
    {
        TimedLaunch tl("score_plan", a.st);
        plan_count_kernel<<<n_wg, kPlanThreads, 0, a.st>>>(a.pr, a.w.wg_sum);
        plan_scan_kernel<<<1, kPlanThreads, 0, a.st>>>(n_wg, a.w.wg_sum, a.w.n_tiles);
        plan_emit_kernel<<<n_wg, kPlanThreads, 0, a.st>>>(a.pr, a.w.wg_sum, a.w.tiles, a.w.row_tile0);
        if (int rc = launch_status("score_plan")) return rc;
    }
    return pool->dtype == KVM_BF16 ? launch_dtype<KVM_BF16>(a) : launch_dtype<KVM_FP16>(a);
}
