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

// ---- sliding window + blended estimate (section 3.3, after Eq. 5) ------------------------
// Ring of the last `window` outcomes per pair.  The order of events matters here (only the
// newest `window` of a pair survive), so one workgroup walks the event array in chunks of
// 1024 and gives every valid event its rank among the events of its pair: rank inside the
// wavefront from ballots, plus the counts of earlier wavefronts and earlier chunks.  An event
// is written iff it is among the last `window` of its pair in this call, at ring place
// (head + rank) mod window: distinct places, no write race.
constexpr int kWinThreads = 1024;
constexpr int kWinWaves = kWinThreads / kWave;

__global__ __launch_bounds__(kWinThreads) void beta_window_kernel(const uint8_t* __restrict__ ev_pair,
                                                                  const uint8_t* __restrict__ ev_outcome, int64_t n,
                                                                  uint8_t* __restrict__ win,
                                                                  uint32_t* __restrict__ win_head, uint32_t window) {
    __shared__ uint32_t tot[KVM_N_PAIRS];    // valid events of each pair in this call
    __shared__ uint32_t run[KVM_N_PAIRS];    // ... of which in earlier chunks
    __shared__ uint32_t head0[KVM_N_PAIRS];
    __shared__ uint32_t wcnt[kWinWaves][KVM_N_PAIRS];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    if (tid < KVM_N_PAIRS) {
        tot[tid] = 0;
        run[tid] = 0;
        head0[tid] = win_head[tid] % window;
    }
    if (tid < kWinWaves * KVM_N_PAIRS) (&wcnt[0][0])[tid] = 0;
    __syncthreads();
    for (int64_t e = tid; e < n; e += kWinThreads) {
        const uint32_t p = ev_pair[e], o = ev_outcome[e];
        if (p < KVM_N_PAIRS && o <= 1) atomicAdd(&tot[p], 1u);
    }
    __syncthreads();
    for (int64_t base = 0; base < n; base += kWinThreads) {
        const int64_t e = base + tid;
        uint32_t p = 0, o = 0;
        bool valid = false;
        if (e < n) {
            p = ev_pair[e];
            o = ev_outcome[e];
            valid = p < KVM_N_PAIRS && o <= 1;
        }
        // lanes of this wavefront that hold a valid event of the same pair
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 4; ++bit) {
            const uint64_t b = __ballot((p >> bit) & 1);
            same &= ((p >> bit) & 1) ? b : ~b;
        }
        const uint32_t rank_in_wave = __popcll(same & ((1ull << lane) - 1));
        if (valid && rank_in_wave == 0) wcnt[wave][p] = __popcll(same);
        __syncthreads();
        if (valid) {
            uint32_t rank = run[p] + rank_in_wave;
            for (int w = 0; w < wave; ++w) rank += wcnt[w][p];
            if ((uint64_t)rank + window >= tot[p])
                win[(size_t)p * window + (head0[p] + rank) % window] = (uint8_t)o;
        }
        __syncthreads();
        if (tid < KVM_N_PAIRS) {
            uint32_t c = 0;
            for (int w = 0; w < kWinWaves; ++w) c += wcnt[w][tid];
            run[tid] += c;
        }
        __syncthreads();
        if (tid < kWinWaves * KVM_N_PAIRS) (&wcnt[0][0])[tid] = 0;
        __syncthreads();
    }
    if (tid < KVM_N_PAIRS) win_head[tid] = (uint32_t)(((uint64_t)head0[tid] + tot[tid]) % window);
}

// One workgroup per pair: window frequency, posterior mean, confidence, blend.
__global__ __launch_bounds__(256) void beta_blend_kernel(const uint32_t* __restrict__ hits,
                                                         const uint32_t* __restrict__ misses, float alpha0,
                                                         float beta0, const uint8_t* __restrict__ win,
                                                         uint32_t window, float kappa, float* __restrict__ p_hat,
                                                         float* __restrict__ conf, float* __restrict__ p_blend) {
    __shared__ uint32_t s_ones, s_seen;
    const int i = blockIdx.x;
    if (threadIdx.x == 0) s_ones = s_seen = 0;
    __syncthreads();
    uint32_t ones = 0, seen = 0;
    for (uint32_t j = threadIdx.x; j < window; j += 256) {
        const uint32_t v = win[(size_t)i * window + j];
        seen += v <= 1;
        ones += v == 1;
    }
    if (seen) {
        atomicAdd(&s_seen, seen);
        atomicAdd(&s_ones, ones);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const float a = alpha0 + (float)hits[i];
        const float b = beta0 + (float)misses[i];
        const float post = a / (a + b);
        const float n = (float)hits[i] + (float)misses[i];
        const float c = (n + kappa > 0.f) ? n / (n + kappa) : 0.f;
        const float f = s_seen ? (float)s_ones / (float)s_seen : post;
        p_hat[i] = post;
        conf[i] = c;
        p_blend[i] = c * post + (1.f - c) * f;
    }
}

// ---- ema + priority -------------------------------------------------------------
// Optional refinements of section 3.4 (positional distance decay) and sections 3.4 / 3.7
// (per-head multipliers during a task transition); all pointers device.
struct EmaEx {
    double lg_pos_decay;   // log2 of the positional decay
    int n_seq, n_heads;
    const int32_t* row_seq;
    const int32_t* row_head;
    const uint8_t* seq_transition;
    const float* head_mult;
};

// LANES threads per row (64 = one wavefront per row, for fleets of short rows; 256 = one
// workgroup per row, for long rows); they stride over the row's blocks.
template <int LANES, bool EX>
__global__ __launch_bounds__(256) void ema_prio_kernel(int n_rows, int64_t n_uids, const int32_t* __restrict__ row_ntok,
                                                       const int64_t* __restrict__ row_off,
                                                       const uint8_t* __restrict__ row_active,
                                                       const float* __restrict__ mass, float decay,
                                                       const float* __restrict__ row_weight,
                                                       const uint8_t* __restrict__ pair,
                                                       const float* __restrict__ p_hat, uint8_t* __restrict__ state,
                                                       float* __restrict__ S, float* __restrict__ prio, EmaEx ex) {
    __shared__ float ph[KVM_N_PAIRS];
    constexpr int ROWS_PER_WG = 256 / LANES;
    const int row = blockIdx.x * ROWS_PER_WG + threadIdx.x / LANES;
    // the row's entries are loaded together with the posterior means, ahead of the barrier: the kernel
    // is a chain of dependent round trips for short rows
    const int rc = row < n_rows ? row : n_rows - 1;
    const int n = row_ntok[rc];
    const int64_t off = row_off[rc];
    const bool active = row_active ? row_active[rc] != 0 : true;
    float w = row_weight[rc];
    if (threadIdx.x < KVM_N_PAIRS) ph[threadIdx.x] = p_hat[threadIdx.x];
    __syncthreads();
    if (row >= n_rows) return;
    if (n <= 0) return;
    const int64_t nb = ((int64_t)n + 15) >> 4;
    if (off < 0 || off + nb > n_uids) return;
    if (EX && ex.head_mult) {
        // Out-of-range indices cannot be reported from here: such a row keeps multiplier 1.
        const int sq = ex.row_seq[row], hd = ex.row_head[row];
        if (sq >= 0 && sq < ex.n_seq && hd >= 0 && hd < ex.n_heads) {
            const uint32_t t = ex.seq_transition[sq];
            if (t <= 3) w *= ex.head_mult[(size_t)t * ex.n_heads + hd];
        }
    }
    const float keep = decay, take = 1.0f - decay;
    // Four units per lane and trip, all sixteen loads before the first use: a mass loaded only after
    // the state byte has arrived would put two round trips in a row, and a long row handled by one
    // wavefront is a chain of such trips (the kernel is bound by that latency, not by bytes).
    constexpr int U = 4;
    for (int64_t b0 = threadIdx.x % LANES; b0 < nb; b0 += U * LANES) {
        uint8_t st[U], pr[U];
        float s[U], x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t b = b0 + u * LANES;
            const int64_t uid = off + (b < nb ? b : b0);
            st[u] = state[uid];
            s[u] = S[uid];
            x[u] = mass[uid];
            pr[u] = pair[uid];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t b = b0 + u * LANES;
            if (b >= nb) break;
            const int64_t uid = off + b;
            if (active && (st[u] & KVM_ST_RESIDENT)) {
                if (EX) x[u] *= pow_by_distance(ex.lg_pos_decay, nb - 1 - b);
                if (!(st[u] & KVM_ST_SCORED)) {
                    s[u] = x[u];
                    st[u] |= KVM_ST_SCORED;
                    state[uid] = st[u];
                } else {
                    s[u] = keep * s[u] + take * x[u];
                }
                S[uid] = s[u];
            }
            prio[uid] = (st[u] & KVM_ST_SCORED) ? w * s[u] * ph[pr[u] & 15] : INFINITY;
        }
    }
}

template <bool EX>
void launch_ema(const kvm_rows_t* rows, const float* mass, float ema_decay, const float* row_weight,
                const uint8_t* pair, const float* p_hat, uint8_t* state, float* S, float* prio, const EmaEx& ex,
                hipStream_t st) {
    if (rows->n_uids / rows->n_rows >= 192) {
        ema_prio_kernel<256, EX><<<(unsigned)rows->n_rows, 256, 0, st>>>(
            rows->n_rows, rows->n_uids, rows->row_ntok, rows->row_off, rows->row_active, mass, ema_decay, row_weight,
            pair, p_hat, state, S, prio, ex);
    } else {
        ema_prio_kernel<64, EX><<<(unsigned)((rows->n_rows + 3) / 4), 256, 0, st>>>(
            rows->n_rows, rows->n_uids, rows->row_ntok, rows->row_off, rows->row_active, mass, ema_decay, row_weight,
            pair, p_hat, state, S, prio, ex);
    }
}

int check_ema(const char* who, const kvm_rows_t* rows, const float* mass, float ema_decay, const float* row_weight,
              const uint8_t* pair, const float* p_hat, uint8_t* state, float* S, float* prio, bool* nothing) {
    *nothing = false;
    KVM_REQUIRE(rows, KVM_EINVAL, "%s: null rows", who);
    KVM_REQUIRE(rows->n_rows >= 0 && rows->n_uids >= 0, KVM_EINVAL, "%s: negative size", who);
    KVM_REQUIRE(ema_decay >= 0.f && ema_decay <= 1.f, KVM_EINVAL, "%s: decay %g outside [0, 1]", who,
                (double)ema_decay);
    if (rows->n_rows == 0 || rows->n_uids == 0) {
        *nothing = true;
        return KVM_OK;
    }
    KVM_REQUIRE(rows->row_ntok && rows->row_off, KVM_EINVAL, "%s: null row array", who);
    KVM_REQUIRE(mass && row_weight && pair && p_hat && state && S && prio, KVM_EINVAL, "%s: null buffer", who);
    return KVM_OK;
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

extern "C" int kvm_beta_blend_update(const uint8_t* ev_pair, const uint8_t* ev_outcome, int64_t n_events,
                                     uint32_t* hits, uint32_t* misses, float alpha0, float beta0, uint8_t* win,
                                     uint32_t* win_head, int32_t window, float kappa, float* p_hat, float* conf,
                                     float* p_blend, uint32_t* n_bad, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(n_events >= 0, KVM_EINVAL, "kvm_beta_blend_update: n_events %lld < 0", (long long)n_events);
    KVM_REQUIRE(hits && misses && p_hat && conf && p_blend && win && win_head, KVM_EINVAL,
                "kvm_beta_blend_update: null counter, window or output");
    KVM_REQUIRE(n_events == 0 || (ev_pair && ev_outcome), KVM_EINVAL, "kvm_beta_blend_update: null event array");
    KVM_REQUIRE(alpha0 > 0.f && beta0 > 0.f, KVM_EINVAL, "kvm_beta_blend_update: prior (%g, %g) must be positive",
                (double)alpha0, (double)beta0);
    KVM_REQUIRE(window >= 1 && window <= KVM_MAX_WINDOW, KVM_EINVAL,
                "kvm_beta_blend_update: window %d outside [1, %d]", window, KVM_MAX_WINDOW);
    KVM_REQUIRE(kappa >= 0.f, KVM_EINVAL, "kvm_beta_blend_update: kappa %g < 0", (double)kappa);
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("beta", st);
    if (n_events > 0) {
        beta_window_kernel<<<1, kWinThreads, 0, st>>>(ev_pair, ev_outcome, n_events, win, win_head, (uint32_t)window);
        int64_t grid = (n_events + kBetaThreads * 16 - 1) / (kBetaThreads * 16);
        if (grid > kBetaMaxGrid) grid = kBetaMaxGrid;
        beta_count_kernel<<<(unsigned)grid, kBetaThreads, 0, st>>>(ev_pair, ev_outcome, n_events, hits, misses, n_bad);
    }
    beta_blend_kernel<<<KVM_N_PAIRS, 256, 0, st>>>(hits, misses, alpha0, beta0, win, (uint32_t)window, kappa, p_hat,
                                                   conf, p_blend);
    return launch_status("beta_blend");
}

extern "C" int kvm_ema_update(const kvm_rows_t* rows, const float* mass, float ema_decay, const float* row_weight,
                              const uint8_t* pair, const float* p_hat, uint8_t* state, float* S, float* prio,
                              void* stream) {
    using namespace kvm;
    clear_error();
    bool nothing;
    if (int rc = check_ema("kvm_ema_update", rows, mass, ema_decay, row_weight, pair, p_hat, state, S, prio, &nothing))
        return rc;
    if (nothing) return KVM_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("ema_prio", st);
    launch_ema<false>(rows, mass, ema_decay, row_weight, pair, p_hat, state, S, prio, EmaEx{}, st);
    return launch_status("ema_prio");
}

extern "C" int kvm_ema_update_ex(const kvm_rows_t* rows, const float* mass, float ema_decay, const kvm_ema_ex_t* ex,
                                 const float* row_weight, const uint8_t* pair, const float* p_hat, uint8_t* state,
                                 float* S, float* prio, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(ex, KVM_EINVAL, "kvm_ema_update_ex: null options");
    KVM_REQUIRE(ex->pos_decay > 0.f && ex->pos_decay <= 1.f, KVM_EINVAL,
                "kvm_ema_update_ex: positional decay %g outside (0, 1]", (double)ex->pos_decay);
    KVM_REQUIRE(!ex->head_mult ||
                    (ex->row_seq && ex->row_head && ex->seq_transition && ex->n_seq > 0 && ex->n_heads > 0),
                KVM_EINVAL, "kvm_ema_update_ex: head multipliers given without row_seq / row_head / seq_transition");
    bool nothing;
    if (int rc = check_ema("kvm_ema_update_ex", rows, mass, ema_decay, row_weight, pair, p_hat, state, S, prio,
                           &nothing))
        return rc;
    if (nothing) return KVM_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("ema_prio", st);
    EmaEx e{std::log2((double)ex->pos_decay), ex->n_seq, ex->n_heads, ex->row_seq, ex->row_head, ex->seq_transition,
            ex->head_mult};
    launch_ema<true>(rows, mass, ema_decay, row_weight, pair, p_hat, state, S, prio, e, st);
    return launch_status("ema_prio_ex");
}
