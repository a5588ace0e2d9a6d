// kvm_span_update and kvm_prefetch_keys: position-aware prefetching (section 3.5).
//
// span  : per row, the smallest number of trailing blocks that hold a fraction theta of the
//         row's mass; per layer, the prefetch window = 16 * ceil(mean span).  Exact integer
//         arithmetic on fixed-point masses, so the result does not depend on summation order.
// keys  : per unit, whether it is a prefetch candidate (on the host, inside the window around
//         the decode position) and its rank key 1 - reuse estimate x decay^distance.  The list
//         itself is kvm_select_victims(key, cand, k): the k lowest keys.
#include "kvm_internal.h"

namespace kvm {
namespace {

// floor(m * 2^32) for m in (0, 1], 0 for anything else (NaN included), clamped at 1 (a mass
// is a softmax share); a row's total then fits 64 bits for any row length.
__device__ inline uint64_t fixed_mass(float m, uint8_t st) {
    if (!(st & KVM_ST_RESIDENT) || !(m > 0.0f)) return 0;
    return (uint64_t)(fminf(m, 1.0f) * 4294967296.0f);
}

__device__ inline uint64_t shfl_u64(uint64_t v, int src) {
    const uint32_t lo = __shfl((uint32_t)v, src), hi = __shfl((uint32_t)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}
__device__ inline uint64_t shfl_up_u64(uint64_t v, int delta) {
    const uint32_t lo = __shfl_up((uint32_t)v, delta), hi = __shfl_up((uint32_t)(v >> 32), delta);
    return ((uint64_t)hi << 32) | lo;
}
__device__ inline uint64_t shfl_xor_u64(uint64_t v, int mask) {
    const uint32_t lo = __shfl_xor((uint32_t)v, mask), hi = __shfl_xor((uint32_t)(v >> 32), mask);
    return ((uint64_t)hi << 32) | lo;
}

// One wavefront per row.  Pass 1: the row's total.  Pass 2: walk back from the last block in
// chunks of 64 x kSeg blocks; lane l holds kSeg consecutive distances (so a wavefront load covers
// contiguous memory), one prefix scan over the lane sums per chunk finds the lane in which the
// running sum reaches theta * total, and that lane walks its kSeg values to the exact block.
constexpr int kSeg = 8;

// Span of one row (0 = the row does not count: inactive, empty, out of range, no mass).
__device__ inline int64_t row_span(int row, int lane, int64_t n_uids, int n_layers,
                                   const int32_t* __restrict__ row_ntok, const int64_t* __restrict__ row_off,
                                   const uint8_t* __restrict__ row_active, const int32_t* __restrict__ row_layer,
                                   const float* __restrict__ mass, const uint8_t* __restrict__ state,
                                   uint32_t theta_num, uint32_t theta_den) {
    const int n = row_ntok[row];                             // the row's four records in one round trip
    const int64_t off = row_off[row];
    const int layer = row_layer[row];
    const bool active = row_active ? row_active[row] != 0 : true;
    if (n <= 0 || !active) return 0;
    const int64_t nb = ((int64_t)n + 15) >> 4;
    if (off < 0 || off + nb > n_uids) return 0;
    if (layer < 0 || layer >= n_layers) return 0;

    uint64_t total = 0;
    for (int64_t b0 = lane; b0 < nb; b0 += 4 * kWave) {      // four blocks per lane and trip, loads first
        float m[4];
        uint8_t st[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t b = b0 + u * kWave;
            m[u] = mass[off + (b < nb ? b : b0)];
            st[u] = state[off + (b < nb ? b : b0)];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (b0 + u * kWave < nb) total += fixed_mass(m[u], st[u]);
    }
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) total += shfl_xor_u64(total, m);
    if (total == 0) return 0;
    const unsigned __int128 need = (unsigned __int128)theta_num * total;

    uint64_t before = 0;   // sum over earlier chunks
    for (int64_t base = 0; base < nb; base += kWave * kSeg) {
        uint64_t q[kSeg];
        uint64_t v = 0;
        const int64_t s0 = base + (int64_t)lane * kSeg;      // this lane's first distance
#pragma unroll
        for (int j = 0; j < kSeg; ++j) {
            const int64_t s1 = s0 + j;
            q[j] = 0;
            if (s1 < nb) {
                const int64_t uid = off + (nb - 1 - s1);
                q[j] = fixed_mass(mass[uid], state[uid]);
            }
            v += q[j];
        }
        uint64_t incl = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const uint64_t up = shfl_up_u64(incl, d);
            if (lane >= d) incl += up;
        }
        const uint64_t hit = __ballot(s0 < nb && (unsigned __int128)(before + incl) * theta_den >= need);
        if (hit) {
            const int first = __ffsll((unsigned long long)hit) - 1;
            int64_t mine = s0 + kSeg;
            if (lane == first) {                             // the crossing lies among this lane's values
                uint64_t acc = before + incl - v;
                bool found = false;
#pragma unroll
                for (int j = 0; j < kSeg; ++j) {
                    acc += q[j];
                    if (!found && (unsigned __int128)acc * theta_den >= need) {
                        found = true;
                        mine = s0 + j + 1;
                    }
                }
            }
            return (int64_t)shfl_u64((uint64_t)mine, first);
        }
        before += shfl_u64(incl, kWave - 1);
    }
    return nb;
}

// One wavefront per row; the row's span goes to row_span[row] (0 = the row does not count).
__global__ __launch_bounds__(256) void span_rows_kernel(int n_rows, int64_t n_uids, int n_layers,
                                                        const int32_t* __restrict__ row_ntok,
                                                        const int64_t* __restrict__ row_off,
                                                        const uint8_t* __restrict__ row_active,
                                                        const int32_t* __restrict__ row_layer,
                                                        const float* __restrict__ mass,
                                                        const uint8_t* __restrict__ state, uint32_t theta_num,
                                                        uint32_t theta_den, int32_t* __restrict__ row_span_out) {
    const int lane = threadIdx.x % kWave;
    const int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave;
    if (row >= n_rows) return;
    const int64_t span = row_span((int)row, lane, n_uids, n_layers, row_ntok, row_off, row_active, row_layer, mass,
                                  state, theta_num, theta_den);
    if (lane == 0) row_span_out[row] = (int32_t)span;        // at most 2^27 blocks in a row of 2^31 tokens
}

// Per-layer sums of the row spans.  Adding each row's span straight to its layer's accumulator
// costs far more than finding the span: the adds of one layer all meet at one address (32
// layers: 64 hot addresses for every row of the model) and are served one after the other.  So
// a workgroup folds kSpanFoldRows rows into per-layer cells in LDS first and then adds each cell
// it touched to the accumulators once.  n_layers <= kSpanFoldLayers.
constexpr int kSpanFoldLayers = 2048;
constexpr int kSpanFoldRows = 4096;
__global__ __launch_bounds__(1024) void span_fold_kernel(int n_rows, int n_layers,
                                                         const int32_t* __restrict__ row_layer,
                                                         const int32_t* __restrict__ row_span_in,
                                                         unsigned long long* span_sum, uint32_t* span_cnt) {
    __shared__ unsigned long long s_sum[kSpanFoldLayers];
    __shared__ uint32_t s_cnt[kSpanFoldLayers];
    for (int l = threadIdx.x; l < n_layers; l += blockDim.x) {
        s_sum[l] = 0;
        s_cnt[l] = 0;
    }
    __syncthreads();
    const int64_t row0 = (int64_t)blockIdx.x * kSpanFoldRows;
    constexpr int PER = kSpanFoldRows / 1024;
    int32_t span[PER], layer[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int64_t row = row0 + u * 1024 + threadIdx.x;
        span[u] = row < n_rows ? row_span_in[row] : 0;
        layer[u] = row < n_rows ? row_layer[row] : 0;
    }
#pragma unroll
    for (int u = 0; u < PER; ++u)
        if (span[u] > 0) {                                   // a counted row has a layer in range
            atomicAdd(&s_sum[layer[u]], (unsigned long long)span[u]);
            atomicAdd(&s_cnt[layer[u]], 1u);
        }
    __syncthreads();
    for (int l = threadIdx.x; l < n_layers; l += blockDim.x)
        if (s_cnt[l]) {
            atomicAdd(&span_sum[l], s_sum[l]);
            atomicAdd(&span_cnt[l], s_cnt[l]);
        }
}

// The same without the fold, for models of more layers than the fold has cells.
__global__ __launch_bounds__(256) void span_add_kernel(int n_rows, const int32_t* __restrict__ row_layer,
                                                       const int32_t* __restrict__ row_span_in,
                                                       unsigned long long* span_sum, uint32_t* span_cnt) {
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= n_rows) return;
    const int32_t span = row_span_in[row];
    if (span <= 0) return;
    atomicAdd(&span_sum[row_layer[row]], (unsigned long long)span);
    atomicAdd(&span_cnt[row_layer[row]], 1u);
}

__global__ void span_window_kernel(int n_layers, const unsigned long long* span_sum, const uint32_t* span_cnt,
                                   int32_t w_min, int32_t w_max, int32_t* layer_window) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= n_layers || span_cnt[l] == 0) return;
    const unsigned long long mean_up = (span_sum[l] + span_cnt[l] - 1) / span_cnt[l];
    unsigned long long w = mean_up * 16ull;
    if (w < (unsigned long long)w_min) w = (unsigned long long)w_min;
    if (w > (unsigned long long)w_max) w = (unsigned long long)w_max;
    layer_window[l] = (int32_t)w;
}

// LANES threads per row, striding over its blocks.
template <int LANES>
__global__ __launch_bounds__(256) void prefetch_keys_kernel(int n_rows, int64_t n_uids, int n_layers,
                                                            const int32_t* __restrict__ row_ntok,
                                                            const int64_t* __restrict__ row_off,
                                                            const int32_t* __restrict__ row_layer,
                                                            const int32_t* __restrict__ row_pos,
                                                            const int32_t* __restrict__ layer_window,
                                                            const uint8_t* __restrict__ state,
                                                            const uint8_t* __restrict__ pair,
                                                            const float* __restrict__ p_est, double lg_pos_decay,
                                                            float* __restrict__ key, uint8_t* __restrict__ cand) {
    __shared__ float pe[KVM_N_PAIRS];
    if (threadIdx.x < KVM_N_PAIRS) pe[threadIdx.x] = p_est[threadIdx.x];
    __syncthreads();
    constexpr int ROWS_PER_WG = 256 / LANES;
    const int row = blockIdx.x * ROWS_PER_WG + threadIdx.x / LANES;
    if (row >= n_rows) return;
    const int nt = row_ntok[row];
    if (nt <= 0) return;
    const int64_t nb = ((int64_t)nt + 15) >> 4;
    const int64_t off = row_off[row];
    if (off < 0 || off + nb > n_uids) return;
    const int layer = row_layer[row];
    const bool layer_ok = layer >= 0 && layer < n_layers;
    const int64_t n = row_pos[row];
    const int64_t w = layer_ok ? layer_window[layer] : -1;
    const bool row_asks = n >= 0 && w >= 0;
    const int64_t nblk = n >> 4;
    for (int64_t b = threadIdx.x % LANES; b < nb; b += LANES) {
        const int64_t uid = off + b;
        const uint8_t st = state[uid];
        const int64_t first = b * 16, last = first + 15;
        const bool on_host = (st & KVM_ST_ON_HOST) && !(st & KVM_ST_RESIDENT);
        const bool ok = row_asks && on_host && last >= n - w && first <= n;
        float k = INFINITY;
        if (ok) k = 1.0f - pe[pair[uid] & 15] * pow_by_distance(lg_pos_decay, nblk - b);
        key[uid] = k;
        cand[uid] = ok ? (uint8_t)(KVM_ST_RESIDENT | KVM_ST_SCORED) : (uint8_t)0;
    }
}

int check_rows(const char* who, const kvm_rows_t* rows, bool* nothing) {
    *nothing = false;
    KVM_REQUIRE(rows, KVM_EINVAL, "%s: null rows", who);
    KVM_REQUIRE(rows->n_rows >= 0 && rows->n_uids >= 0, KVM_EINVAL, "%s: negative size", who);
    if (rows->n_rows == 0 || rows->n_uids == 0) {
        *nothing = true;
        return KVM_OK;
    }
    KVM_REQUIRE(rows->row_ntok && rows->row_off, KVM_EINVAL, "%s: null row array", who);
    return KVM_OK;
}

}  // namespace

size_t span_workspace_bytes(int32_t n_rows) { return ((size_t)(n_rows > 0 ? n_rows : 0) * sizeof(int32_t) + 255) & ~(size_t)255; }

}  // namespace kvm

extern "C" int kvm_span_update(const kvm_rows_t* rows, const int32_t* row_layer, int32_t n_layers, const float* mass,
                               const uint8_t* state, uint32_t theta_num, uint32_t theta_den, uint64_t* span_sum,
                               uint32_t* span_cnt, int32_t w_min, int32_t w_max, int32_t* layer_window, void* ws,
                               size_t ws_bytes, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(n_layers > 0, KVM_EINVAL, "kvm_span_update: n_layers %d <= 0", n_layers);
    KVM_REQUIRE(theta_den > 0 && theta_den <= 65536 && theta_num <= theta_den, KVM_EINVAL,
                "kvm_span_update: theta %u / %u must lie in [0, 1] with a denominator of at most 65536", theta_num,
                theta_den);
    KVM_REQUIRE(w_min >= 0 && w_max >= w_min, KVM_EINVAL, "kvm_span_update: window bounds [%d, %d]", w_min, w_max);
    KVM_REQUIRE(span_sum && span_cnt && layer_window, KVM_EINVAL, "kvm_span_update: null accumulator or output");
    bool nothing;
    if (int rc = check_rows("kvm_span_update", rows, &nothing)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!nothing) {
        KVM_REQUIRE(row_layer && mass && state, KVM_EINVAL, "kvm_span_update: null buffer");
        KVM_REQUIRE(ws && reinterpret_cast<uintptr_t>(ws) % 4 == 0, KVM_EINVAL,
                    "kvm_span_update: workspace null or not 4-byte aligned");
        KVM_REQUIRE(ws_bytes >= span_workspace_bytes(rows->n_rows), KVM_ENOSPC,
                    "kvm_span_update: workspace of %zu bytes, %zu needed", ws_bytes,
                    span_workspace_bytes(rows->n_rows));
    }
    TimedLaunch tl("span", st);
    if (!nothing) {
        const int n_rows = rows->n_rows;
        int32_t* row_span_buf = static_cast<int32_t*>(ws);
        span_rows_kernel<<<(unsigned)((n_rows + 3) / 4), 256, 0, st>>>(
            n_rows, rows->n_uids, n_layers, rows->row_ntok, rows->row_off, rows->row_active, row_layer, mass, state,
            theta_num, theta_den, row_span_buf);
        unsigned long long* sum = reinterpret_cast<unsigned long long*>(span_sum);
        if (n_layers <= kSpanFoldLayers)
            span_fold_kernel<<<(unsigned)((n_rows + kSpanFoldRows - 1) / kSpanFoldRows), 1024, 0, st>>>(
                n_rows, n_layers, row_layer, row_span_buf, sum, span_cnt);
        else
            span_add_kernel<<<(unsigned)((n_rows + 255) / 256), 256, 0, st>>>(n_rows, row_layer, row_span_buf, sum,
                                                                             span_cnt);
    }
    span_window_kernel<<<(unsigned)((n_layers + 255) / 256), 256, 0, st>>>(
        n_layers, reinterpret_cast<const unsigned long long*>(span_sum), span_cnt, w_min, w_max, layer_window);
    return launch_status("span");
}

extern "C" int kvm_prefetch_keys(const kvm_rows_t* rows, const int32_t* row_layer, const int32_t* row_pos,
                                 const int32_t* layer_window, int32_t n_layers, const uint8_t* state,
                                 const uint8_t* pair, const float* p_est, float pos_decay, float* key, uint8_t* cand,
                                 void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(n_layers > 0, KVM_EINVAL, "kvm_prefetch_keys: n_layers %d <= 0", n_layers);
    KVM_REQUIRE(pos_decay > 0.f && pos_decay <= 1.f, KVM_EINVAL,
                "kvm_prefetch_keys: positional decay %g outside (0, 1]", (double)pos_decay);
    bool nothing;
    if (int rc = check_rows("kvm_prefetch_keys", rows, &nothing)) return rc;
    if (nothing) return KVM_OK;
    KVM_REQUIRE(row_layer && row_pos && layer_window && state && pair && p_est && key && cand, KVM_EINVAL,
                "kvm_prefetch_keys: null buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("prefetch_keys", st);
    const double lg = std::log2((double)pos_decay);
    if (rows->n_uids / rows->n_rows >= 192) {
        prefetch_keys_kernel<256><<<(unsigned)rows->n_rows, 256, 0, st>>>(
            rows->n_rows, rows->n_uids, n_layers, rows->row_ntok, rows->row_off, row_layer, row_pos, layer_window,
            state, pair, p_est, lg, key, cand);
    } else {
        prefetch_keys_kernel<64><<<(unsigned)((rows->n_rows + 3) / 4), 256, 0, st>>>(
            rows->n_rows, rows->n_uids, n_layers, rows->row_ntok, rows->row_off, row_layer, row_pos, layer_window,
            state, pair, p_est, lg, key, cand);
    }
    return launch_status("prefetch_keys");
}
