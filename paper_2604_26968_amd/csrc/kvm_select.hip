// kvm_select_victims: the k eligible units of lowest (priority, uid), in uid order.
//
// The paper evicts the unit with the lowest weighted importance (section 3.4);
// under a capacity budget that becomes an order statistic: find the k-th
// smallest key, then emit everything below it plus the first ties in uid order.
//
// Method: three-pass most-significant-digit radix select (11 + 11 + 10 bits) on
// an order-preserving 32-bit image of the fp32 priority, with workgroup-local
// LDS histograms merged by atomics, then an order-preserving compaction
// (per-chunk counts, one scan over chunks, per-chunk emit).  Each pass streams
// prio (4 B) and state (1 B) once.
#include <mutex>

#include "kvm_internal.h"

// Scratch of kvm_select_victims_static: histograms, control block and per-chunk counts for up to
// KVM_SELECT_STATIC_MAX_UIDS units (2^26 / 4096 chunks and one entry of totals).  Every GPU the library runs on holds its
// own copy at its own address; host code reaches it only through the pointer that
// hipGetSymbolAddress returns for the current device, never through this name.
static __device__ __align__(256) unsigned char scratch[KVM_SELECT_STATIC_SCRATCH_BYTES];

namespace kvm {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 4096;          // uids per workgroup in the count / emit kernels
constexpr int kItems = kChunk / kThreads;
constexpr int kBins0 = 2048, kBins1 = 2048, kBins2 = 1024;
constexpr int kRep0 = 16;               // copies of the pass-0 histogram in global memory
constexpr int kRow0 = kBins0 + 32;      // entries per copy: the bins, the resident count, padding to a line
constexpr int kHistWords = kRep0 * kRow0 + kBins1 + kBins2;

struct Ctrl {
    unsigned long long n_resident, n_eligible;
    unsigned long long k;            // victims to emit
    unsigned long long remaining;    // still to find inside the current bin
    uint32_t prefix;                 // key bits fixed so far (high bits)
    uint32_t threshold;              // final: k-th smallest key
    unsigned long long ties;         // final: how many keys == threshold to take
};

__device__ __forceinline__ bool eligible(uint8_t st) {
    return (st & (KVM_ST_RESIDENT | KVM_ST_PROTECTED | KVM_ST_SCORED | KVM_ST_SHARED)) ==
           (KVM_ST_RESIDENT | KVM_ST_SCORED);
}

// Monotone map fp32 -> uint32 (a < b as floats  <=>  key(a) < key(b)); NaN ranks
// with +inf and -0 with +0.
__device__ __forceinline__ uint32_t order_key(float p) {
    uint32_t u = __float_as_uint(p);
    if ((u & 0x7fffffffu) > 0x7f800000u) u = 0x7f800000u;
    if (u == 0x80000000u) u = 0;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void select_init_kernel(uint32_t* hist, int n, Ctrl* c) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) hist[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) *c = Ctrl{0, 0, 0, 0, 0, 0, 0};
}

// PASS 0: bits 31..21 of every eligible key, plus resident / eligible counts.
// PASS 1: bits 20..10 of keys whose bits 31..21 equal ctrl->prefix.
// PASS 2: bits  9..0  of keys whose bits 31..10 equal ctrl->prefix.
template <int PASS>
__global__ __launch_bounds__(kThreads) void select_hist_kernel(const float* __restrict__ prio,
                                                               const uint8_t* __restrict__ state, int64_t n,
                                                               uint32_t* __restrict__ hist, Ctrl* __restrict__ ctrl) {
    constexpr int BINS = PASS == 0 ? kBins0 : PASS == 1 ? kBins1 : kBins2;
    __shared__ uint32_t h[BINS];
    __shared__ uint32_t cnt[2];
    for (int i = threadIdx.x; i < BINS; i += kThreads) h[i] = 0;
    if (threadIdx.x < 2) cnt[threadIdx.x] = 0;
    __syncthreads();
    if (PASS > 0 && ctrl->k == 0) return;
    const uint32_t prefix = PASS == 0 ? 0u : ctrl->prefix;
    uint32_t n_res = 0;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    // Four elements per thread and trip: all eight loads first, unconditionally (a priority loaded only
    // once its state byte says "eligible" makes every element two dependent round trips, and the
    // pass is bound by that latency, not by its bytes or its LDS atomics).
    constexpr int B = 4;
    for (int64_t u0 = (int64_t)blockIdx.x * kThreads + threadIdx.x; u0 < n; u0 += stride * B) {
        uint8_t st[B];
        float pr[B];
#pragma unroll
        for (int i = 0; i < B; ++i) {
            const int64_t u = u0 + i * stride;
            st[i] = u < n ? state[u] : 0;
            pr[i] = prio[u < n ? u : 0];
        }
#pragma unroll
        for (int i = 0; i < B; ++i) {
            if (PASS == 0 && (st[i] & KVM_ST_RESIDENT)) ++n_res;
            if (!eligible(st[i])) continue;
            const uint32_t key = order_key(pr[i]);
            if (PASS == 0) {
                atomicAdd(&h[key >> 21], 1u);
            } else if (PASS == 1) {
                if ((key >> 21) == prefix) atomicAdd(&h[(key >> 10) & 2047u], 1u);
            } else if (PASS == 2) {
                if ((key >> 10) == prefix) atomicAdd(&h[key & 1023u], 1u);
            }
        }
    }
    if (PASS == 0) {
        if (n_res) atomicAdd(&cnt[0], n_res);
    }
    __syncthreads();
    // Pass 0: the priorities of one launch crowd into a few dozen neighbouring top-digit bins, i.e. into
    // one or two cache lines of the global histogram, and thousands of workgroups adding to one line are
    // served one after the other by one L2 channel (measured: 44 of the pass's 67 us on 21 M units).  So
    // pass 0 folds into one of kRep0 copies, chosen by workgroup; the scan sums the copies.  The resident
    // count travels in a spare bin of the same copy; the eligible count is the histogram's total.
    uint32_t* hg = PASS == 0 ? hist + (blockIdx.x % kRep0) * kRow0 : hist;
    for (int i = threadIdx.x; i < BINS; i += kThreads)
        if (h[i]) atomicAdd(&hg[i], h[i]);
    if (PASS == 0 && threadIdx.x == 0 && cnt[0]) atomicAdd(&hg[kBins0], cnt[0]);
}

// One workgroup.  Finds the bin in which the cumulative count reaches
// ctrl->remaining and narrows the prefix.  PASS 0 first turns the arguments
// into k.
template <int PASS>
__global__ __launch_bounds__(1024) void select_scan_kernel(const uint32_t* __restrict__ hist, Ctrl* __restrict__ ctrl,
                                                           int64_t k_or_neg1, int64_t budget, int64_t cap,
                                                           int64_t* __restrict__ n_victims) {
    constexpr int BINS = PASS == 0 ? kBins0 : PASS == 1 ? kBins1 : kBins2;
    constexpr int PER = BINS / 1024 > 0 ? BINS / 1024 : 1;
    __shared__ unsigned long long wave_sum[16];
    __shared__ unsigned long long s_remaining, s_k;
    // inclusive scan of the histogram, PER consecutive bins per thread (pass 0: the copies summed first)
    const int first = threadIdx.x * PER;
    unsigned long long local[PER];
    unsigned long long run = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        unsigned long long c = 0;
        if (first + i < BINS) {
            if (PASS == 0) {
                for (int r = 0; r < kRep0; ++r) c += hist[r * kRow0 + first + i];
            } else {
                c = hist[first + i];
            }
        }
        run += c;
        local[i] = run;
    }
    unsigned long long inc = run;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        if (PASS == 0) {
            unsigned long long n_resident = 0, n_eligible = 0;
            for (int r = 0; r < kRep0; ++r) n_resident += hist[r * kRow0 + kBins0];
            for (int w = 0; w < 16; ++w) n_eligible += wave_sum[w];
            ctrl->n_resident = n_resident;
            ctrl->n_eligible = n_eligible;
            unsigned long long k;
            if (k_or_neg1 >= 0)
                k = (unsigned long long)k_or_neg1;
            else
                k = n_resident > (unsigned long long)budget ? n_resident - (unsigned long long)budget : 0;
            if (k > n_eligible) k = n_eligible;
            if (k > (unsigned long long)cap) k = (unsigned long long)cap;
            ctrl->k = k;
            ctrl->remaining = k;
            *n_victims = (int64_t)k;
        }
        s_remaining = ctrl->remaining;
        s_k = ctrl->k;
    }
    __syncthreads();
    const unsigned long long want = s_remaining;
    if (s_k == 0) {
        if (PASS == 2 && threadIdx.x == 0) {
            ctrl->threshold = 0;
            ctrl->ties = 0;
        }
        return;
    }
    unsigned long long base = 0;
    for (int w = 0; w < wave; ++w) base += wave_sum[w];
    const unsigned long long excl = base + inc - run;     // keys in bins before `first`
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const unsigned long long before = excl + (i ? local[i - 1] : 0ull);
        const unsigned long long upto = excl + local[i];
        if (first + i < BINS && before < want && want <= upto) {       // exactly one bin satisfies this
            const uint32_t bin = (uint32_t)(first + i);
            if (PASS == 0) {
                ctrl->prefix = bin;
                ctrl->remaining = want - before;
            } else if (PASS == 1) {
                ctrl->prefix = (ctrl->prefix << 11) | bin;
                ctrl->remaining = want - before;
            } else {
                ctrl->threshold = (ctrl->prefix << 10) | bin;
                ctrl->ties = want - before;
            }
        }
    }
}

// Per chunk of kChunk uids: how many eligible keys are below / equal to the threshold.
__global__ __launch_bounds__(kThreads) void select_count_kernel(const float* __restrict__ prio,
                                                                const uint8_t* __restrict__ state, int64_t n,
                                                                const Ctrl* __restrict__ ctrl,
                                                                uint32_t* __restrict__ chunk_less,
                                                                uint32_t* __restrict__ chunk_eq) {
    __shared__ uint32_t s_less, s_eq;
    if (threadIdx.x == 0) s_less = s_eq = 0;
    __syncthreads();
    const uint32_t thr = ctrl->threshold;
    const bool any = ctrl->k != 0;
    uint32_t less = 0, eq = 0;
    const int64_t base = (int64_t)blockIdx.x * kChunk;
    if (any) {
        // both loads of an element issued before either is looked at (see select_hist_kernel)
#pragma unroll 8
        for (int i = 0; i < kItems; ++i) {
            const int64_t u = base + i * kThreads + threadIdx.x;
            const uint8_t st = u < n ? state[u] : 0;
            const uint32_t key = order_key(prio[u < n ? u : 0]);
            const bool el = eligible(st);
            less += el && key < thr;
            eq += el && key == thr;
        }
    }
    if (less) atomicAdd(&s_less, less);
    if (eq) atomicAdd(&s_eq, eq);
    __syncthreads();
    if (threadIdx.x == 0) {
        chunk_less[blockIdx.x] = s_less;
        chunk_eq[blockIdx.x] = s_eq;
    }
}

// One workgroup: exclusive scans of the two per-chunk count arrays, in place, with the totals
// stored behind the last chunk (entry n_chunks), so that a chunk's own counts are the difference
// of two neighbours (64-bit running sums are not needed: totals are bounded by n_uids < 2^32,
// which the entry point enforces).
__global__ __launch_bounds__(1024) void select_chunk_scan_kernel(int n_chunks, uint32_t* chunk_less,
                                                                 uint32_t* chunk_eq) {
    __shared__ uint32_t ws_a[16], ws_b[16];
    uint32_t carry_a = 0, carry_b = 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int base = 0; base < n_chunks; base += 1024) {
        const int i = base + threadIdx.x;
        const uint32_t a = i < n_chunks ? chunk_less[i] : 0, b = i < n_chunks ? chunk_eq[i] : 0;
        uint32_t ia = a, ib = b;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t oa = __shfl_up(ia, d), ob = __shfl_up(ib, d);
            if (lane >= d) {
                ia += oa;
                ib += ob;
            }
        }
        if (lane == 63) {
            ws_a[wave] = ia;
            ws_b[wave] = ib;
        }
        __syncthreads();
        uint32_t ba = 0, bb = 0, ta = 0, tb = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) {
                ba += ws_a[w];
                bb += ws_b[w];
            }
            ta += ws_a[w];
            tb += ws_b[w];
        }
        if (i < n_chunks) {
            chunk_less[i] = carry_a + ba + ia - a;
            chunk_eq[i] = carry_b + bb + ib - b;
        }
        carry_a += ta;
        carry_b += tb;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        chunk_less[n_chunks] = carry_a;
        chunk_eq[n_chunks] = carry_b;
    }
}

// Per chunk: write the selected uids at their rank in uid order.  A chunk that holds no key below
// the threshold and no tie that is still wanted (most chunks, when k is a small part of n) reads
// nothing.  VEC: prio and state are 16-byte aligned, so a thread fetches its kItems consecutive
// elements as 16-byte vectors (chunks that end inside the arrays only).
template <bool VEC>
__global__ __launch_bounds__(kThreads) void select_emit_kernel(const float* __restrict__ prio,
                                                               const uint8_t* __restrict__ state, int64_t n,
                                                               const Ctrl* __restrict__ ctrl,
                                                               const uint32_t* __restrict__ chunk_less,
                                                               const uint32_t* __restrict__ chunk_eq,
                                                               int64_t* __restrict__ victims) {
    __shared__ uint32_t w_less[kThreads / kWave], w_eq[kThreads / kWave];
    if (ctrl->k == 0) return;
    const uint32_t thr = ctrl->threshold;
    const unsigned long long ties = ctrl->ties;
    const int64_t base = (int64_t)blockIdx.x * kChunk;
    const uint32_t less0 = chunk_less[blockIdx.x], eq0 = chunk_eq[blockIdx.x];
    if (chunk_less[blockIdx.x + 1] == less0 && (chunk_eq[blockIdx.x + 1] == eq0 || eq0 >= ties)) return;
    // Thread t owns the kItems consecutive uids base + t*kItems .. so that ranks follow uid order.
    uint32_t flag_less = 0, flag_eq = 0;   // bit i: item i is below / equal
    uint32_t c_less = 0, c_eq = 0;
    static_assert(kItems == 16, "the vector path fetches 16 elements per thread");
    if (VEC && base + kChunk <= n) {
        const int64_t u0 = base + (int64_t)threadIdx.x * kItems;
        const uint4 sv = *reinterpret_cast<const uint4*>(state + u0);
        const float4* pv = reinterpret_cast<const float4*>(prio + u0);
        const float4 p0 = pv[0], p1 = pv[1], p2 = pv[2], p3 = pv[3];
        const uint32_t sw[4] = {sv.x, sv.y, sv.z, sv.w};
        const float pr[16] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w,
                              p2.x, p2.y, p2.z, p2.w, p3.x, p3.y, p3.z, p3.w};
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const uint8_t st = (uint8_t)(sw[i >> 2] >> (8 * (i & 3)));
            const uint32_t key = order_key(pr[i]);
            const bool el = eligible(st);
            const bool lt = el && key < thr, eq = el && key == thr;
            flag_less |= (uint32_t)lt << i;
            flag_eq |= (uint32_t)eq << i;
            c_less += lt;
            c_eq += eq;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int64_t u = base + (int64_t)threadIdx.x * kItems + i;
            if (u < n && eligible(state[u])) {
                const uint32_t key = order_key(prio[u]);
                if (key < thr) {
                    flag_less |= 1u << i;
                    ++c_less;
                } else if (key == thr) {
                    flag_eq |= 1u << i;
                    ++c_eq;
                }
            }
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t il = c_less, ie = c_eq;
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t ol = __shfl_up(il, d), oe = __shfl_up(ie, d);
        if (lane >= d) {
            il += ol;
            ie += oe;
        }
    }
    if (lane == 63) {
        w_less[wave] = il;
        w_eq[wave] = ie;
    }
    __syncthreads();
    unsigned long long less_before = less0, eq_before = eq0;
    for (int w = 0; w < wave; ++w) {
        less_before += w_less[w];
        eq_before += w_eq[w];
    }
    less_before += il - c_less;
    eq_before += ie - c_eq;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int64_t u = base + (int64_t)threadIdx.x * kItems + i;
        const bool lt = flag_less >> i & 1u, eq = flag_eq >> i & 1u;
        if (lt || (eq && eq_before < ties)) {
            const unsigned long long pos = less_before + (eq_before < ties ? eq_before : ties);
            victims[pos] = u;
        }
        less_before += lt;
        eq_before += eq;
    }
}

struct SelectWs {
    uint32_t* hist;        // kHistWords: kRep0 copies of the pass-0 histogram, then passes 1 and 2
    Ctrl* ctrl;
    uint32_t* chunk_less;
    uint32_t* chunk_eq;
    size_t bytes;
};

SelectWs carve(void* ws, int64_t n_uids) {
    const size_t n_chunks = (size_t)((n_uids + kChunk - 1) / kChunk);
    const size_t off_ctrl = align_up(kHistWords * sizeof(uint32_t), 256);
    const size_t off_less = off_ctrl + align_up(sizeof(Ctrl), 256);
    const size_t off_eq = off_less + align_up((n_chunks + 1) * sizeof(uint32_t), 256);
    const uintptr_t base = reinterpret_cast<uintptr_t>(ws);
    SelectWs w;
    w.hist = reinterpret_cast<uint32_t*>(base);
    w.ctrl = reinterpret_cast<Ctrl*>(base + off_ctrl);
    w.chunk_less = reinterpret_cast<uint32_t*>(base + off_less);
    w.chunk_eq = reinterpret_cast<uint32_t*>(base + off_eq);
    w.bytes = off_eq + align_up((n_chunks + 1) * sizeof(uint32_t), 256);
    return w;
}

}  // namespace

size_t select_workspace_bytes(int64_t n_uids) { return carve(nullptr, n_uids).bytes; }

static_assert(KVM_SELECT_STATIC_SCRATCH_BYTES ==
                  kHistWords * 4 + 256 + 2 * ((KVM_SELECT_STATIC_MAX_UIDS / kChunk) * 4 + 256),
              "the header's scratch size follows the workspace layout of carve()");

}  // namespace kvm

extern "C" size_t kvm_workspace_bytes(int op, int64_t n_uids, int32_t n_rows, int32_t g, int32_t dim) {
    if (n_uids < 0 || n_rows < 0) return 0;
    if (op == KVM_OP_SCORE) return kvm::score_workspace_bytes(n_uids, n_rows, g < 1 ? 1 : g, dim);
    if (op == KVM_OP_SELECT) return kvm::select_workspace_bytes(n_uids);
    if (op == KVM_OP_SPAN) return kvm::span_workspace_bytes(n_rows);
    return 0;
}

namespace kvm {
namespace {

// The launches of one selection over a carved workspace.  `timed` brackets the two phases with the
// library's timing events (which may create events on first use).
int launch_select(const float* prio, const uint8_t* state, int64_t n_uids, int64_t k_or_neg1, int64_t budget_units,
                  int64_t* victims, int64_t victims_cap, int64_t* n_victims, const SelectWs& w, hipStream_t st,
                  bool timed) {
    const int n_chunks = (int)((n_uids + kChunk - 1) / kChunk);
    int64_t hist_grid = (n_uids + (int64_t)kThreads * 16 - 1) / ((int64_t)kThreads * 16);
    if (hist_grid > 2048) hist_grid = 2048;
    if (hist_grid < 1) hist_grid = 1;
    uint32_t* h0 = w.hist;
    uint32_t* h1 = w.hist + kRep0 * kRow0;
    uint32_t* h2 = h1 + kBins1;
    {
        TimedLaunch tl(timed ? "select_hist" : nullptr, st);
        select_init_kernel<<<16, 256, 0, st>>>(w.hist, kHistWords, w.ctrl);
        select_hist_kernel<0><<<(unsigned)hist_grid, kThreads, 0, st>>>(prio, state, n_uids, h0, w.ctrl);
        select_scan_kernel<0><<<1, 1024, 0, st>>>(h0, w.ctrl, k_or_neg1, budget_units, victims_cap, n_victims);
        select_hist_kernel<1><<<(unsigned)hist_grid, kThreads, 0, st>>>(prio, state, n_uids, h1, w.ctrl);
        select_scan_kernel<1><<<1, 1024, 0, st>>>(h1, w.ctrl, 0, 0, 0, n_victims);
        select_hist_kernel<2><<<(unsigned)hist_grid, kThreads, 0, st>>>(prio, state, n_uids, h2, w.ctrl);
        select_scan_kernel<2><<<1, 1024, 0, st>>>(h2, w.ctrl, 0, 0, 0, n_victims);
        if (int rc = launch_status("select_hist")) return rc;
    }
    if (n_chunks > 0) {
        TimedLaunch tl(timed ? "select_emit" : nullptr, st);
        select_count_kernel<<<n_chunks, kThreads, 0, st>>>(prio, state, n_uids, w.ctrl, w.chunk_less, w.chunk_eq);
        select_chunk_scan_kernel<<<1, 1024, 0, st>>>(n_chunks, w.chunk_less, w.chunk_eq);
        const bool vec = reinterpret_cast<uintptr_t>(prio) % 16 == 0 && reinterpret_cast<uintptr_t>(state) % 16 == 0;
        if (vec)
            select_emit_kernel<true><<<n_chunks, kThreads, 0, st>>>(prio, state, n_uids, w.ctrl, w.chunk_less,
                                                                   w.chunk_eq, victims);
        else
            select_emit_kernel<false><<<n_chunks, kThreads, 0, st>>>(prio, state, n_uids, w.ctrl, w.chunk_less,
                                                                    w.chunk_eq, victims);
        if (int rc = launch_status("select_emit")) return rc;
    }
    return KVM_OK;
}

int check_select_args(const char* who, const float* prio, const uint8_t* state, int64_t n_uids, int64_t k_or_neg1,
                      int64_t budget_units, const int64_t* victims, int64_t victims_cap, const int64_t* n_victims) {
    KVM_REQUIRE(n_uids >= 0 && k_or_neg1 >= -1 && budget_units >= 0 && victims_cap >= 0, KVM_EINVAL,
                "%s: negative argument", who);
    KVM_REQUIRE(n_uids < (1ll << 32), KVM_ESHAPE, "%s: n_uids %lld needs 64-bit ranks", who, (long long)n_uids);
    KVM_REQUIRE(n_victims, KVM_EINVAL, "%s: null n_victims", who);
    KVM_REQUIRE(victims || victims_cap == 0, KVM_EINVAL, "%s: null victims", who);
    KVM_REQUIRE(n_uids == 0 || (prio && state), KVM_EINVAL, "%s: null input", who);
    return KVM_OK;
}

}  // namespace
}  // namespace kvm

extern "C" int kvm_select_victims(const float* prio, const uint8_t* state, int64_t n_uids, int64_t k_or_neg1,
                                  int64_t budget_units, int64_t* victims, int64_t victims_cap, int64_t* n_victims,
                                  void* ws, size_t ws_bytes, void* stream) {
    using namespace kvm;
    clear_error();
    if (int rc = check_select_args("kvm_select_victims", prio, state, n_uids, k_or_neg1, budget_units, victims,
                                   victims_cap, n_victims))
        return rc;
    KVM_REQUIRE(ws, KVM_EINVAL, "kvm_select_victims: null workspace");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(ws) % 256 == 0, KVM_EINVAL, "kvm_select_victims: ws not 256-byte aligned");
    const SelectWs w = carve(ws, n_uids);
    KVM_REQUIRE(ws_bytes >= w.bytes, KVM_ENOSPC, "kvm_select_victims: workspace %zu < %zu bytes", ws_bytes, w.bytes);
    return launch_select(prio, state, n_uids, k_or_neg1, budget_units, victims, victims_cap, n_victims, w,
                         static_cast<hipStream_t>(stream), true);
}

namespace kvm {
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};      // per device: address of its copy of `scratch`

// Address of the current device's scratch array, resolved once per device.
int static_scratch(void** out) {
    int dev = -1;
    KVM_HIP_TRY(hipGetDevice(&dev));
    KVM_REQUIRE(dev >= 0 && dev < kMaxDevices, KVM_EHIP, "kvm_select_victims_static: device %d out of range", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        KVM_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        KVM_REQUIRE(p && reinterpret_cast<uintptr_t>(p) % 256 == 0, KVM_EHIP,
                    "kvm_select_victims_static: bad scratch address %p on device %d", p, dev);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return KVM_OK;
}
}  // namespace
}  // namespace kvm

extern "C" int kvm_select_victims_static(const float* prio, const uint8_t* state, int64_t n_uids, int64_t k_or_neg1,
                                         int64_t budget_units, int64_t* victims, int64_t victims_cap,
                                         int64_t* n_victims, void* stream) {
    using namespace kvm;
    clear_error();
    if (int rc = check_select_args("kvm_select_victims_static", prio, state, n_uids, k_or_neg1, budget_units, victims,
                                   victims_cap, n_victims))
        return rc;
    KVM_REQUIRE(n_uids <= (int64_t)KVM_SELECT_STATIC_MAX_UIDS, KVM_ENOSPC,
                "kvm_select_victims_static: n_uids %lld exceeds the built-in scratch's limit of %lld units; "
                "use kvm_select_victims with a workspace",
                (long long)n_uids, (long long)KVM_SELECT_STATIC_MAX_UIDS);
    void* ptr = nullptr;
    if (int rc = static_scratch(&ptr)) return rc;
    const SelectWs w = carve(ptr, n_uids);
    KVM_REQUIRE(w.bytes <= (size_t)KVM_SELECT_STATIC_SCRATCH_BYTES, KVM_ENOSPC,
                "kvm_select_victims_static: scratch %zu < %zu bytes", (size_t)KVM_SELECT_STATIC_SCRATCH_BYTES, w.bytes);
    // Histograms and the control block are cleared by select_init_kernel, the per-chunk counts are
    // written before they are read: nothing of the previous call's contents is used.
    return launch_select(prio, state, n_uids, k_or_neg1, budget_units, victims, victims_cap, n_victims, w,
                         static_cast<hipStream_t>(stream), false);
}
