// kvm_score_step: softmax attention mass per (row, 16-token block) unit.
//
// What is computed is Eq. 1 of the paper restricted to the HBM-resident tokens
// of each row, summed per token block, then the maximum (or mean) over the
// query heads that share the KV head (GQA grouping rule, section 3.4).
//
// Structure (all kernels in this file):
//   plan_*           build the list of tiles = (row, first block) of at most 64 blocks
//                    for the active rows, on the device, so the scorer's grid has no
//                    idle workgroups whatever the spread of row lengths
//   score_partial    one workgroup per tile, one wavefront per unit at a time:
//                    per (unit, query) block maximum m and sum s = sum exp(z - m)
//   score_finalize   one workgroup per row: combines the (m, s) pairs into the
//                    row's softmax normaliser and writes the unit masses
//
// score_partial is the only kernel that touches K; it reads every resident unit
// exactly once with 16-byte loads that cover 1 KiB contiguous per wavefront
// instruction.  With the [dim/8][16][8] unit layout lane l holds token l%16,
// channel group 4*kk + l/16 of load kk, so a lane accumulates its share of
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

__global__ __launch_bounds__(kPlanThreads) void plan_emit_kernel(PlanRows p, const uint32_t* wg_base, Tile* tiles) {
    const int r = blockIdx.x * kPlanThreads + threadIdx.x;
    const uint32_t nt = tiles_of_row(p, r);
    uint32_t total;
    const uint32_t first = wg_base[blockIdx.x] + wg_exclusive_scan(nt, &total);
    for (uint32_t i = 0; i < nt; ++i) tiles[first + i] = Tile{r, (int32_t)(i * kTileBlocks)};
}

// ---- score_partial ------------------------------------------------------------
// G     queries per row, compile-time when QREG (queries live in registers),
//       otherwise a run-time value and the queries are staged in LDS
// DIM   channels per token (multiple of 32)
// DT    element type
template <int G_CT, int DIM, int DT, bool QREG>
__global__ __launch_bounds__(256) void score_partial_kernel(
    const Tile* __restrict__ tiles, const uint32_t* __restrict__ n_tiles, int g_rt,
    const int32_t* __restrict__ row_ntok, const int64_t* __restrict__ row_off,
    const int64_t* __restrict__ row_q_off, const int32_t* __restrict__ slot_tbl,
    const uint4* __restrict__ k_pool, uint32_t n_slots, const uint16_t* __restrict__ q, float scale,
    float2* __restrict__ part) {
    constexpr int NK = DIM / 32;          // 16-byte loads per lane per unit
    constexpr int UNIT_V4 = DIM * 2;      // 16-byte vectors per unit
    constexpr int QROW_V4 = DIM / 8;      // 16-byte vectors per query
    extern __shared__ uint4 q_lds[];      // [g][QROW_V4] when !QREG

    if (blockIdx.x >= *n_tiles) return;
    const Tile tile = tiles[blockIdx.x];
    const int G = QREG ? G_CT : g_rt;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = lane & 15, cg = lane >> 4;
    const int ntok = row_ntok[tile.row];
    const int nb = (ntok + 15) >> 4;
    const int nbt = min(kTileBlocks, nb - tile.b0);
    const int64_t uid0 = row_off[tile.row] + tile.b0;
    const uint4* qrow = reinterpret_cast<const uint4*>(q + row_q_off[tile.row]);

    constexpr int GR = QREG ? G_CT : 1;
    uint4 qv[GR][NK];
    if constexpr (QREG) {
#pragma unroll
        for (int j = 0; j < G_CT; ++j)
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) qv[j][kk] = qrow[j * QROW_V4 + 4 * kk + cg];
    } else {
        for (int i = threadIdx.x; i < G * QROW_V4; i += 256) q_lds[i] = qrow[i];
        __syncthreads();
    }

    // Resident units of the tile; this wavefront takes every fourth one.
    int my_slot = lane < nbt ? slot_tbl[uid0 + lane] : -1;
    if ((uint32_t)my_slot >= n_slots) my_slot = -1;
    uint64_t mine = 0;
    {
        int rank = 0;
        for (uint64_t m = __ballot(my_slot >= 0); m; m &= m - 1)
            if ((rank++ & 3) == wave) mine |= m & (~m + 1);
    }

    auto pop = [&]() -> int {
        if (!mine) return -1;
        const int i = __builtin_ctzll(mine);
        mine &= mine - 1;
        return i;
    };
    auto load_unit = [&](uint4 (&dst)[NK], int i) {
        const uint32_t slot = (uint32_t)__builtin_amdgcn_readlane(my_slot, i);
        const uint4* p = k_pool + (size_t)slot * UNIT_V4 + lane;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) dst[kk] = p[kk * 64];
    };

    uint4 cur[NK], nxt[NK];
    int i_cur = pop();
    if (i_cur >= 0) load_unit(cur, i_cur);
    while (i_cur >= 0) {
        const int i_nxt = pop();
        if (i_nxt >= 0) load_unit(nxt, i_nxt);

        const int tok_in_block = min(16, ntok - 16 * (tile.b0 + i_cur));
        const bool valid = t < tok_in_block;
        float2* out = part + (uid0 + i_cur) * G;

        // four queries at a time: each 16-lane row ends up owning one of them
#pragma unroll
        for (int j0 = 0; j0 < G; j0 += 4) {
            float a[4] = {0.f, 0.f, 0.f, 0.f};
            if constexpr (QREG) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if (j0 + jj < G_CT) {
#pragma unroll
                        for (int kk = 0; kk < NK; ++kk) a[jj] = dot8<DT>(cur[kk], qv[(j0 + jj) % GR][kk], a[jj]);
                    }
            } else {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if (j0 + jj < G) {
                        const uint4* qj = q_lds + (j0 + jj) * QROW_V4 + cg;
#pragma unroll
                        for (int kk = 0; kk < NK; ++kk) a[jj] = dot8<DT>(cur[kk], qj[4 * kk], a[jj]);
                    }
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
    float2* part;
    size_t bytes;
};

ScoreWs carve(void* ws, int64_t n_uids, int32_t n_rows, int32_t g) {
    const size_t n_wg = ((size_t)n_rows + kPlanThreads - 1) / kPlanThreads;
    const size_t off_sum = 256;
    const size_t off_tiles = off_sum + align_up(n_wg * sizeof(uint32_t), 256);
    const size_t off_part = off_tiles + align_up((size_t)max_tiles(n_uids, n_rows) * sizeof(Tile), 256);
    const uintptr_t base = reinterpret_cast<uintptr_t>(ws);
    ScoreWs w;
    w.n_tiles = reinterpret_cast<uint32_t*>(base);
    w.wg_sum = reinterpret_cast<uint32_t*>(base + off_sum);
    w.tiles = reinterpret_cast<Tile*>(base + off_tiles);
    w.part = reinterpret_cast<float2*>(base + off_part);
    w.bytes = off_part + align_up((size_t)n_uids * (size_t)g * sizeof(float2), 256);
    return w;
}

template <int DIM, int DT>
int launch_partial(int g, dim3 grid, hipStream_t st, const ScoreWs& w, const kvm_rows_t* rows,
                   const kvm_pool_t* pool, const void* q, float scale) {
    const uint4* kp = static_cast<const uint4*>(pool->k_pool);
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint32_t ns = (uint32_t)pool->n_slots;
#define KVM_LAUNCH_QREG(GG)                                                                            \
    score_partial_kernel<GG, DIM, DT, true><<<grid, 256, 0, st>>>(                                     \
        w.tiles, w.n_tiles, g, rows->row_ntok, rows->row_off, rows->row_q_off, rows->slot_tbl, kp, ns, \
        qq, scale, w.part)
    if constexpr (DIM <= 128) {
        switch (g) {
            case 1: KVM_LAUNCH_QREG(1); return launch_status("score_partial");
            case 2: KVM_LAUNCH_QREG(2); return launch_status("score_partial");
            case 4: KVM_LAUNCH_QREG(4); return launch_status("score_partial");
            case 8: KVM_LAUNCH_QREG(8); return launch_status("score_partial");
            default: break;
        }
    }
#undef KVM_LAUNCH_QREG
    const size_t lds = (size_t)g * (DIM / 8) * sizeof(uint4);
    auto kern = score_partial_kernel<0, DIM, DT, false>;
    if (lds > 160 * 1024) return fail(KVM_ESHAPE, "kvm_score_step: g %d x dim %d queries do not fit LDS", g, DIM);
    if (lds > 48 * 1024)
        KVM_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<grid, 256, lds, st>>>(w.tiles, w.n_tiles, g, rows->row_ntok, rows->row_off, rows->row_q_off,
                                 rows->slot_tbl, kp, ns, qq, scale, w.part);
    return launch_status("score_partial");
}

template <int DT>
int launch_partial_dim(int dim, int g, dim3 grid, hipStream_t st, const ScoreWs& w, const kvm_rows_t* rows,
                       const kvm_pool_t* pool, const void* q, float scale) {
    switch (dim) {
        case 32: return launch_partial<32, DT>(g, grid, st, w, rows, pool, q, scale);
        case 64: return launch_partial<64, DT>(g, grid, st, w, rows, pool, q, scale);
        case 96: return launch_partial<96, DT>(g, grid, st, w, rows, pool, q, scale);
        case 128: return launch_partial<128, DT>(g, grid, st, w, rows, pool, q, scale);
        case 192: return launch_partial<192, DT>(g, grid, st, w, rows, pool, q, scale);
        case 256: return launch_partial<256, DT>(g, grid, st, w, rows, pool, q, scale);
        case 576: return launch_partial<576, DT>(g, grid, st, w, rows, pool, q, scale);
        default: return fail(KVM_ESHAPE, "kvm_score_step: no kernel for dim %d", dim);
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
    const ScoreWs w = carve(ws, rows->n_uids, rows->n_rows, rows->g);
    KVM_REQUIRE(ws_bytes >= w.bytes, KVM_ENOSPC, "kvm_score_step: workspace %zu < %zu bytes", ws_bytes, w.bytes);
    const int64_t tiles_max = max_tiles(rows->n_uids, rows->n_rows);
    KVM_REQUIRE(tiles_max <= 0x7fffffffll, KVM_ESHAPE, "kvm_score_step: too many tiles");

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n_wg = (rows->n_rows + kPlanThreads - 1) / kPlanThreads;
    const PlanRows pr{rows->n_rows, rows->g,        pool->dim,       rows->n_uids,    rows->q_elems,
                      rows->row_ntok, rows->row_off, rows->row_q_off, rows->row_active};
    {
        TimedLaunch tl("score_plan", st);
        plan_count_kernel<<<n_wg, kPlanThreads, 0, st>>>(pr, w.wg_sum);
        plan_scan_kernel<<<1, kPlanThreads, 0, st>>>(n_wg, w.wg_sum, w.n_tiles);
        plan_emit_kernel<<<n_wg, kPlanThreads, 0, st>>>(pr, w.wg_sum, w.tiles);
        if (int rc = launch_status("score_plan")) return rc;
    }
    {
        TimedLaunch tl("score_partial", st);
        const dim3 grid((unsigned)tiles_max);
        const int rc = pool->dtype == KVM_BF16
                           ? launch_partial_dim<KVM_BF16>(pool->dim, rows->g, grid, st, w, rows, pool, q, softmax_scale)
                           : launch_partial_dim<KVM_FP16>(pool->dim, rows->g, grid, st, w, rows, pool, q, softmax_scale);
        if (rc) return rc;
    }
    {
        TimedLaunch tl("score_finalize", st);
        int gp = 1;
        while (gp < rows->g) gp <<= 1;
#define KVM_FIN(GP)                                                                                        \
    case GP:                                                                                               \
        score_finalize_kernel<GP><<<rows->n_rows, 256, 0, st>>>(pr, rows->slot_tbl, (uint32_t)pool->n_slots, \
                                                                w.part, agg, mass);                          \
        break;
        switch (gp) {
            KVM_FIN(1) KVM_FIN(2) KVM_FIN(4) KVM_FIN(8) KVM_FIN(16) KVM_FIN(32) KVM_FIN(64) KVM_FIN(128)
            default: return fail(KVM_ESHAPE, "kvm_score_step: g %d", rows->g);
        }
#undef KVM_FIN
        if (int rc = launch_status("score_finalize")) return rc;
    }
    return KVM_OK;
}
