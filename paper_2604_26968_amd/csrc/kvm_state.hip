// kvm_beta_update and kvm_ema_update: the small per-step state updates.
//
// beta  : reuse / miss counters of the 16 (block type, transition type) pairs
//         and their posterior means (section 3.3, Eq. 5).  Integer counters, so
//         the result does not depend on the order atomics arrive in.
// ema   : exponential moving average of the unit masses and the eviction
//         priority = head weight x EMA x posterior mean (section 3.4).
#include "kvm_internal.h"

namespace kvm {
namespace {

// ---- beta -----------------------------------------------------------------------
constexpr int kBetaThreads = 256;
constexpr int kBetaMaxGrid = 256;

__global__ __launch_bounds__(kBetaThreads) void beta_count_kernel(const uint8_t* __restrict__ ev_pair,
                                                                  const uint8_t* __restrict__ ev_outcome,
                                                                  int64_t n, uint32_t* hits, uint32_t* misses,
                                                                  uint32_t* n_bad) {
    __shared__ uint32_t h[33];   // 0..15 hits, 16..31 misses, 32 bad
    if (threadIdx.x < 33) h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * kBetaThreads;
    for (int64_t e = (int64_t)blockIdx.x * kBetaThreads + threadIdx.x; e < n; e += stride) {
        const uint32_t p = ev_pair[e], o = ev_outcome[e];
        if (p >= KVM_N_PAIRS || o > 1)
            atomicAdd(&h[32], 1u);
        else
            atomicAdd(&h[p + (o ? 0 : 16)], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 16) {
        if (h[threadIdx.x]) atomicAdd(&hits[threadIdx.x], h[threadIdx.x]);
    } else if (threadIdx.x < 32) {
        if (h[threadIdx.x]) atomicAdd(&misses[threadIdx.x - 16], h[threadIdx.x]);
    } else if (threadIdx.x == 32) {
        if (n_bad && h[32]) atomicAdd(n_bad, h[32]);
    }
}

__global__ void beta_mean_kernel(const uint32_t* hits, const uint32_t* misses, float alpha0, float beta0,
                                 float* p_hat) {
    const int i = threadIdx.x;
    if (i < KVM_N_PAIRS) {
        const float a = alpha0 + (float)hits[i];
        const float b = beta0 + (float)misses[i];
        p_hat[i] = a / (a + b);
    }
}

// ---- ema + priority -------------------------------------------------------------
// LANES threads per row (64 = one wavefront per row, for fleets of short rows; 256 = one
// workgroup per row, for long rows); they stride over the row's blocks.
template <int LANES>
__global__ __launch_bounds__(256) void ema_prio_kernel(int n_rows, int64_t n_uids, const int32_t* __restrict__ row_ntok,
                                                       const int64_t* __restrict__ row_off,
                                                       const uint8_t* __restrict__ row_active,
                                                       const float* __restrict__ mass, float decay,
                                                       const float* __restrict__ row_weight,
                                                       const uint8_t* __restrict__ pair,
                                                       const float* __restrict__ p_hat, uint8_t* __restrict__ state,
                                                       float* __restrict__ S, float* __restrict__ prio) {
    __shared__ float ph[KVM_N_PAIRS];
    if (threadIdx.x < KVM_N_PAIRS) ph[threadIdx.x] = p_hat[threadIdx.x];
    __syncthreads();
    constexpr int ROWS_PER_WG = 256 / LANES;
    const int row = blockIdx.x * ROWS_PER_WG + threadIdx.x / LANES;
    if (row >= n_rows) return;
    const int n = row_ntok[row];
    if (n <= 0) return;
    const int64_t nb = ((int64_t)n + 15) >> 4;
    const int64_t off = row_off[row];
    if (off < 0 || off + nb > n_uids) return;
    const bool active = row_active ? row_active[row] != 0 : true;
    const float w = row_weight[row];
    const float keep = decay, take = 1.0f - decay;
    for (int64_t b = threadIdx.x % LANES; b < nb; b += LANES) {
        const int64_t uid = off + b;
        uint8_t st = state[uid];
        float s = S[uid];
        if (active && (st & KVM_ST_RESIDENT)) {
            const float x = mass[uid];
            if (!(st & KVM_ST_SCORED)) {
                s = x;
                st |= KVM_ST_SCORED;
                state[uid] = st;
            } else {
                s = keep * s + take * x;
            }
            S[uid] = s;
        }
        prio[uid] = (st & KVM_ST_SCORED) ? w * s * ph[pair[uid] & 15] : INFINITY;
    }
}

}  // namespace
}  // namespace kvm

extern "C" int kvm_beta_update(const uint8_t* ev_pair, const uint8_t* ev_outcome, int64_t n_events, uint32_t* hits,
                               uint32_t* misses, float alpha0, float beta0, float* p_hat, uint32_t* n_bad,
                               void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(n_events >= 0, KVM_EINVAL, "kvm_beta_update: n_events %lld < 0", (long long)n_events);
    KVM_REQUIRE(hits && misses && p_hat, KVM_EINVAL, "kvm_beta_update: null counter or output");
    KVM_REQUIRE(n_events == 0 || (ev_pair && ev_outcome), KVM_EINVAL, "kvm_beta_update: null event array");
    KVM_REQUIRE(alpha0 > 0.f && beta0 > 0.f, KVM_EINVAL, "kvm_beta_update: prior (%g, %g) must be positive",
                (double)alpha0, (double)beta0);
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("beta", st);
    if (n_events > 0) {
        int64_t grid = (n_events + kBetaThreads * 16 - 1) / (kBetaThreads * 16);
        if (grid > kBetaMaxGrid) grid = kBetaMaxGrid;
        beta_count_kernel<<<(unsigned)grid, kBetaThreads, 0, st>>>(ev_pair, ev_outcome, n_events, hits, misses, n_bad);
    }
    beta_mean_kernel<<<1, 64, 0, st>>>(hits, misses, alpha0, beta0, p_hat);
    return launch_status("beta");
}

extern "C" int kvm_ema_update(const kvm_rows_t* rows, const float* mass, float ema_decay, const float* row_weight,
                              const uint8_t* pair, const float* p_hat, uint8_t* state, float* S, float* prio,
                              void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(rows, KVM_EINVAL, "kvm_ema_update: null rows");
    KVM_REQUIRE(rows->n_rows >= 0 && rows->n_uids >= 0, KVM_EINVAL, "kvm_ema_update: negative size");
    KVM_REQUIRE(ema_decay >= 0.f && ema_decay <= 1.f, KVM_EINVAL, "kvm_ema_update: decay %g outside [0, 1]",
                (double)ema_decay);
    if (rows->n_rows == 0 || rows->n_uids == 0) return KVM_OK;
    KVM_REQUIRE(rows->row_ntok && rows->row_off, KVM_EINVAL, "kvm_ema_update: null row array");
    KVM_REQUIRE(mass && row_weight && pair && p_hat && state && S && prio, KVM_EINVAL,
                "kvm_ema_update: null buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("ema_prio", st);
    if (rows->n_uids / rows->n_rows >= 192) {
        ema_prio_kernel<256><<<(unsigned)rows->n_rows, 256, 0, st>>>(rows->n_rows, rows->n_uids, rows->row_ntok,
                                                                    rows->row_off, rows->row_active, mass, ema_decay,
                                                                    row_weight, pair, p_hat, state, S, prio);
    } else {
        ema_prio_kernel<64><<<(unsigned)((rows->n_rows + 3) / 4), 256, 0, st>>>(
            rows->n_rows, rows->n_uids, rows->row_ntok, rows->row_off, rows->row_active, mass, ema_decay, row_weight,
            pair, p_hat, state, S, prio);
    }
    return launch_status("ema_prio");
}
