// kvm_pack / kvm_unpack: head-granular moves between the HBM pool (tier 0) and
// pinned host memory (tier 1), section 3.2 of the paper.
//
// A record is one unit's K frame followed by its V frame.  pack gathers the
// records of a uid list into a contiguous staging buffer with 16-byte loads and
// stores (one workgroup per record), flips the table / state entries, and the
// staging buffer travels to the host with hipMemcpyAsync; when no device
// staging buffer is given the gather writes pinned host memory directly.
// unpack is the mirror image.
#include "kvm_internal.h"

namespace kvm {
namespace {

constexpr int kThreads = 256;

// A unit may leave HBM only from a frame of its own: one that shares its frame with units of equal content
// (KVM_ST_SHARED) is refused like a unit that is not in HBM, so that frame is never handed out while read.
__device__ __forceinline__ bool in_own_frame(uint8_t st) {
    return (st & (KVM_ST_RESIDENT | KVM_ST_SHARED)) == KVM_ST_RESIDENT;
}

// first .. first + count of the list; record i lands at staging + (i - first) * rec.
__global__ __launch_bounds__(kThreads) void pack_kernel(const uint4* __restrict__ k_pool,
                                                        const uint4* __restrict__ v_pool, uint32_t n_slots,
                                                        uint32_t k_v4, uint32_t v_v4, int32_t* __restrict__ slot_tbl,
                                                        uint8_t* __restrict__ state, int64_t n_uids,
                                                        const int64_t* __restrict__ uids,
                                                        const int32_t* __restrict__ host_slots,
                                                        int32_t* __restrict__ freed_slots, int64_t first,
                                                        const int64_t* __restrict__ n_dev,
                                                        uint4* __restrict__ staging, uint32_t* n_bad) {
    __shared__ int32_t s_slot;
    const int64_t i = first + blockIdx.x;
    if (n_dev && i >= *n_dev) return;      // list shorter than the launch (uniform for the workgroup)
    if (threadIdx.x == 0) {
        const int64_t uid = uids[i];
        int32_t slot = -1;
        if (uid >= 0 && uid < n_uids && in_own_frame(state[uid])) slot = slot_tbl[uid];
        if ((uint32_t)slot >= n_slots) slot = -1;
        s_slot = slot;
        freed_slots[i] = slot;
        if (slot >= 0) {
            slot_tbl[uid] = -1 - host_slots[i];
            state[uid] = (uint8_t)((state[uid] & ~KVM_ST_RESIDENT) | KVM_ST_ON_HOST);
        } else if (n_bad) {
            atomicAdd(n_bad, 1u);
        }
    }
    __syncthreads();
    const int32_t slot = s_slot;
    if (slot < 0) return;
    uint4* dst = staging + (size_t)blockIdx.x * (k_v4 + v_v4);
    const uint4* ks = k_pool + (size_t)slot * k_v4;
    for (uint32_t v = threadIdx.x; v < k_v4; v += kThreads) dst[v] = ks[v];
    if (v_v4) {
        const uint4* vs = v_pool + (size_t)slot * v_v4;
        for (uint32_t v = threadIdx.x; v < v_v4; v += kThreads) dst[k_v4 + v] = vs[v];
    }
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(uint4* __restrict__ k_pool, uint4* __restrict__ v_pool,
                                                          uint32_t n_slots, uint32_t k_v4, uint32_t v_v4,
                                                          int32_t* __restrict__ slot_tbl, uint8_t* __restrict__ state,
                                                          int64_t n_uids, const int64_t* __restrict__ uids,
                                                          const int32_t* __restrict__ dst_slots, int64_t first,
                                                          const int64_t* __restrict__ n_dev,
                                                          const uint4* __restrict__ staging, uint32_t* n_bad) {
    __shared__ int32_t s_slot;
    const int64_t i = first + blockIdx.x;
    if (n_dev && i >= *n_dev) return;
    if (threadIdx.x == 0) {
        const int64_t uid = uids[i];
        int32_t slot = dst_slots[i];
        if (uid < 0 || uid >= n_uids || (state[uid] & KVM_ST_RESIDENT) || (uint32_t)slot >= n_slots) slot = -1;
        s_slot = slot;
        if (slot >= 0) {
            slot_tbl[uid] = slot;
            state[uid] = (uint8_t)((state[uid] & ~KVM_ST_ON_HOST) | KVM_ST_RESIDENT);
        } else if (n_bad) {
            atomicAdd(n_bad, 1u);
        }
    }
    __syncthreads();
    const int32_t slot = s_slot;
    if (slot < 0) return;
    const uint4* src = staging + (size_t)blockIdx.x * (k_v4 + v_v4);
    uint4* kd = k_pool + (size_t)slot * k_v4;
    for (uint32_t v = threadIdx.x; v < k_v4; v += kThreads) kd[v] = src[v];
    if (v_v4) {
        uint4* vd = v_pool + (size_t)slot * v_v4;
        for (uint32_t v = threadIdx.x; v < v_v4; v += kThreads) vd[v] = src[k_v4 + v];
    }
}

// pack + unpack in one pass over the list: record i of host_out receives the frame of
// out_uids[i], the same frame is then refilled from record i of host_in for in_uids[i].
// Both directions of the host link are busy at once; there is no device staging.
__global__ __launch_bounds__(kThreads) void swap_kernel(uint4* __restrict__ k_pool, uint4* __restrict__ v_pool,
                                                        uint32_t n_slots, uint32_t k_v4, uint32_t v_v4,
                                                        int32_t* __restrict__ slot_tbl, uint8_t* __restrict__ state,
                                                        int64_t n_uids, const int64_t* __restrict__ out_uids,
                                                        const int64_t* __restrict__ in_uids,
                                                        const int32_t* __restrict__ host_slots,
                                                        int32_t* __restrict__ freed_slots, int64_t first,
                                                        const int64_t* __restrict__ n_dev, uint4* __restrict__ host_out,
                                                        const uint4* __restrict__ host_in, uint32_t* n_bad) {
    __shared__ int32_t s_slot;
    __shared__ int s_refill;
    const int64_t i = first + blockIdx.x;
    if (n_dev && i >= *n_dev) return;
    if (threadIdx.x == 0) {
        const int64_t uo = out_uids[i], ui = in_uids[i];
        int32_t slot = -1;
        if (uo >= 0 && uo < n_uids && in_own_frame(state[uo])) slot = slot_tbl[uo];
        if ((uint32_t)slot >= n_slots) slot = -1;
        freed_slots[i] = slot;
        int refill = 0;
        uint32_t bad = 0;
        if (slot >= 0) {
            slot_tbl[uo] = -1 - host_slots[i];
            state[uo] = (uint8_t)((state[uo] & ~KVM_ST_RESIDENT) | KVM_ST_ON_HOST);
        } else {
            ++bad;
        }
        // the unpack half sees the table as the pack half left it
        if (slot >= 0 && ui >= 0 && ui < n_uids && !(state[ui] & KVM_ST_RESIDENT)) {
            refill = 1;
            slot_tbl[ui] = slot;
            state[ui] = (uint8_t)((state[ui] & ~KVM_ST_ON_HOST) | KVM_ST_RESIDENT);
        } else {
            ++bad;
        }
        if (bad && n_bad) atomicAdd(n_bad, bad);
        s_slot = slot;
        s_refill = refill;
    }
    __syncthreads();
    const int32_t slot = s_slot;
    if (slot < 0) return;
    const bool refill = s_refill != 0;
    const size_t rec_v4 = (size_t)k_v4 + v_v4;
    uint4* out = host_out + (size_t)blockIdx.x * rec_v4;
    const uint4* in = host_in + (size_t)blockIdx.x * rec_v4;
    uint4* kf = k_pool + (size_t)slot * k_v4;
    for (uint32_t v = threadIdx.x; v < k_v4; v += kThreads) {
        const uint4 x = kf[v];
        out[v] = x;
        if (refill) kf[v] = in[v];
    }
    if (v_v4) {
        uint4* vf = v_pool + (size_t)slot * v_v4;
        for (uint32_t v = threadIdx.x; v < v_v4; v += kThreads) {
            const uint4 x = vf[v];
            out[k_v4 + v] = x;
            if (refill) vf[v] = in[k_v4 + v];
        }
    }
}

// In-place exchange with a host tier addressed by slot: the frame of out_uids[i] and the tier
// record of in_uids[i] trade contents.  Every thread swaps its own 16-byte pieces (load both,
// store both), so no piece is overwritten before it has been read and neither a spare frame nor
// a spare tier slot is needed.
__global__ __launch_bounds__(kThreads) void exchange_kernel(uint4* __restrict__ k_pool, uint4* __restrict__ v_pool,
                                                            uint32_t n_slots, uint32_t k_v4, uint32_t v_v4,
                                                            int32_t* __restrict__ slot_tbl,
                                                            uint8_t* __restrict__ state, int64_t n_uids,
                                                            const int64_t* __restrict__ out_uids,
                                                            const int64_t* __restrict__ in_uids, int64_t first,
                                                            const int64_t* __restrict__ n_out_dev,
                                                            const int64_t* __restrict__ n_in_dev,
                                                            uint4* __restrict__ tier, uint64_t tier_slots,
                                                            uint32_t* n_bad) {
    __shared__ int32_t s_slot;
    __shared__ int64_t s_host;
    const int64_t i = first + blockIdx.x;
    if ((n_out_dev && i >= *n_out_dev) || (n_in_dev && i >= *n_in_dev)) return;
    if (threadIdx.x == 0) {
        const int64_t uo = out_uids[i], ui = in_uids[i];
        int32_t slot = -1;
        int64_t host = -1;
        if (uo >= 0 && uo < n_uids && in_own_frame(state[uo])) slot = slot_tbl[uo];
        if ((uint32_t)slot >= n_slots) slot = -1;
        if (ui >= 0 && ui < n_uids && ui != uo && (state[ui] & KVM_ST_ON_HOST) && !(state[ui] & KVM_ST_RESIDENT) &&
            slot_tbl[ui] < 0)
            host = -1 - (int64_t)slot_tbl[ui];
        if ((uint64_t)host >= tier_slots) host = -1;
        if (slot >= 0 && host >= 0) {
            slot_tbl[uo] = (int32_t)(-1 - host);
            state[uo] = (uint8_t)((state[uo] & ~KVM_ST_RESIDENT) | KVM_ST_ON_HOST);
            slot_tbl[ui] = slot;
            state[ui] = (uint8_t)((state[ui] & ~KVM_ST_ON_HOST) | KVM_ST_RESIDENT);
        } else {
            slot = -1;
            if (n_bad) atomicAdd(n_bad, 1u);
        }
        s_slot = slot;
        s_host = host;
    }
    __syncthreads();
    const int32_t slot = s_slot;
    if (slot < 0) return;
    const size_t rec_v4 = (size_t)k_v4 + v_v4;
    uint4* rec = tier + (size_t)s_host * rec_v4;
    uint4* kf = k_pool + (size_t)slot * k_v4;
    for (uint32_t v = threadIdx.x; v < k_v4; v += kThreads) {
        const uint4 a = kf[v], b = rec[v];
        kf[v] = b;
        rec[v] = a;
    }
    if (v_v4) {
        uint4* vf = v_pool + (size_t)slot * v_v4;
        for (uint32_t v = threadIdx.x; v < v_v4; v += kThreads) {
            const uint4 a = vf[v], b = rec[k_v4 + v];
            vf[v] = b;
            rec[k_v4 + v] = a;
        }
    }
}

// First and last part of an exchange whose bytes move during the next scoring launch.
__global__ __launch_bounds__(kThreads) void exchange_begin_kernel(uint32_t n_slots, int32_t* __restrict__ slot_tbl,
                                                                  uint8_t* __restrict__ state, int64_t n_uids,
                                                                  const int64_t* __restrict__ out_uids,
                                                                  const int64_t* __restrict__ in_uids, int64_t n,
                                                                  const int64_t* __restrict__ n_out_dev,
                                                                  const int64_t* __restrict__ n_in_dev,
                                                                  uint64_t tier_slots, int32_t* __restrict__ frame,
                                                                  int64_t* __restrict__ host, uint32_t* n_bad) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    int32_t slot = -1;
    int64_t h = -1;
    if (!((n_out_dev && i >= *n_out_dev) || (n_in_dev && i >= *n_in_dev))) {
        const int64_t uo = out_uids[i], ui = in_uids[i];
        if (uo >= 0 && uo < n_uids && in_own_frame(state[uo])) slot = slot_tbl[uo];
        if ((uint32_t)slot >= n_slots) slot = -1;
        if (ui >= 0 && ui < n_uids && ui != uo && (state[ui] & KVM_ST_ON_HOST) && !(state[ui] & KVM_ST_RESIDENT) &&
            slot_tbl[ui] < 0)
            h = -1 - (int64_t)slot_tbl[ui];
        if ((uint64_t)h >= tier_slots) h = -1;
        if (slot >= 0 && h >= 0) {
            slot_tbl[uo] = (int32_t)(-1 - h);
            state[uo] = (uint8_t)((state[uo] & ~KVM_ST_RESIDENT) | KVM_ST_ON_HOST);
        } else {
            slot = -1;
            if (n_bad) atomicAdd(n_bad, 1u);
        }
    }
    frame[i] = slot;
    host[i] = slot >= 0 ? h : -1;
}

// First part of a pack whose bytes move during the next scoring launch: entry i leaves HBM in the table
// exactly as pack_kernel's thread 0 does it, and the pair (frame, host slot | one-way flag) is noted.
__global__ __launch_bounds__(kThreads) void pack_begin_kernel(uint32_t n_slots, int32_t* __restrict__ slot_tbl,
                                                              uint8_t* __restrict__ state, int64_t n_uids,
                                                              const int64_t* __restrict__ uids, int64_t n,
                                                              const int64_t* __restrict__ n_dev,
                                                              const int32_t* __restrict__ host_slots,
                                                              uint64_t tier_slots, int32_t* __restrict__ frame,
                                                              int64_t* __restrict__ host, uint32_t* n_bad) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    int32_t slot = -1;
    int64_t h = -1;
    if (!(n_dev && i >= *n_dev)) {
        const int64_t uid = uids[i];
        h = host_slots[i];
        if (uid >= 0 && uid < n_uids && in_own_frame(state[uid])) slot = slot_tbl[uid];
        if ((uint32_t)slot >= n_slots || (uint64_t)h >= tier_slots) slot = -1;
        if (slot >= 0) {
            slot_tbl[uid] = (int32_t)(-1 - h);
            state[uid] = (uint8_t)((state[uid] & ~KVM_ST_RESIDENT) | KVM_ST_ON_HOST);
        } else if (n_bad) {
            atomicAdd(n_bad, 1u);
        }
    }
    frame[i] = slot;
    host[i] = slot >= 0 ? (h | KVM_XFER_OUT_ONLY) : -1;
}

__global__ __launch_bounds__(kThreads) void exchange_end_kernel(int32_t* __restrict__ slot_tbl,
                                                                uint8_t* __restrict__ state, int64_t n_uids,
                                                                const int64_t* __restrict__ in_uids,
                                                                const int32_t* __restrict__ frame, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const int32_t f = frame[i];
    if (f < 0) return;
    const int64_t ui = in_uids[i];
    if (ui < 0 || ui >= n_uids) return;       // cannot happen for a pair begin accepted
    slot_tbl[ui] = f;
    state[ui] = (uint8_t)((state[ui] & ~KVM_ST_ON_HOST) | KVM_ST_RESIDENT);
}

int check_common(const char* who, const kvm_pool_t* pool, const void* slot_tbl, const void* state, int64_t n_uids,
                 const void* uids, int64_t n, const void* slots, const void* staging_dev, size_t staging_dev_bytes,
                 const void* staging_host, size_t staging_host_bytes) {
    KVM_REQUIRE(pool, KVM_EINVAL, "%s: null pool", who);
    KVM_REQUIRE(n >= 0 && n_uids >= 0, KVM_EINVAL, "%s: negative count", who);
    KVM_REQUIRE(pool->unit_k_bytes > 0 && pool->unit_k_bytes % 16 == 0 && pool->unit_v_bytes % 16 == 0, KVM_ESHAPE,
                "%s: unit sizes (%u, %u) must be multiples of 16", who, pool->unit_k_bytes, pool->unit_v_bytes);
    KVM_REQUIRE(pool->n_slots <= 0x7fffffffull, KVM_EINVAL, "%s: n_slots exceeds int32 slot ids", who);
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(pool->k_pool && (pool->v_pool || pool->unit_v_bytes == 0), KVM_EINVAL, "%s: null pool memory", who);
    KVM_REQUIRE(slot_tbl && state && uids && slots, KVM_EINVAL, "%s: null buffer", who);
    KVM_REQUIRE(staging_host || staging_dev, KVM_EINVAL, "%s: no staging buffer at all", who);
    const size_t rec = (size_t)pool->unit_k_bytes + pool->unit_v_bytes;
    KVM_REQUIRE(!staging_host || staging_host_bytes / rec >= (size_t)n, KVM_ENOSPC,
                "%s: host staging %zu bytes < %lld records of %zu", who, staging_host_bytes, (long long)n, rec);
    KVM_REQUIRE(!staging_dev || staging_dev_bytes >= rec, KVM_ENOSPC, "%s: device staging smaller than one record", who);
    KVM_REQUIRE(staging_host || staging_dev_bytes / rec >= (size_t)n, KVM_ENOSPC,
                "%s: without a host buffer the device staging must hold all %lld records", who, (long long)n);
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(staging_host) % 16 == 0 && reinterpret_cast<uintptr_t>(staging_dev) % 16 == 0,
                KVM_EINVAL, "%s: staging buffers must be 16-byte aligned", who);
    return KVM_OK;
}

}  // namespace
}  // namespace kvm

extern "C" int kvm_pack(const kvm_pool_t* pool, int32_t* slot_tbl, uint8_t* state, int64_t n_uids, const int64_t* uids,
                        int64_t n, const int64_t* n_dev, const int32_t* host_slots, int32_t* freed_slots, void* staging_dev,
                        size_t staging_dev_bytes, void* staging_host, size_t staging_host_bytes, uint32_t* n_bad,
                        void* stream) {
    using namespace kvm;
    clear_error();
    if (int rc = check_common("kvm_pack", pool, slot_tbl, state, n_uids, uids, n, host_slots, staging_dev,
                              staging_dev_bytes, staging_host, staging_host_bytes))
        return rc;
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(freed_slots, KVM_EINVAL, "kvm_pack: null freed_slots");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t k_v4 = pool->unit_k_bytes / 16, v_v4 = pool->unit_v_bytes / 16;
    const size_t rec = (size_t)pool->unit_k_bytes + pool->unit_v_bytes;
    const uint4* kp = static_cast<const uint4*>(pool->k_pool);
    const uint4* vp = static_cast<const uint4*>(pool->v_pool);
    TimedLaunch tl("pack", st);
    if (!staging_dev) {
        for (int64_t first = 0; first < n; first += 0x40000000ll) {
            const int64_t cnt = n - first < 0x40000000ll ? n - first : 0x40000000ll;
            pack_kernel<<<(unsigned)cnt, kThreads, 0, st>>>(kp, vp, (uint32_t)pool->n_slots, k_v4, v_v4, slot_tbl, state,
                                                           n_uids, uids, host_slots, freed_slots, first, n_dev,
                                                           reinterpret_cast<uint4*>(static_cast<char*>(staging_host) + first * rec),
                                                           n_bad);
        }
        return launch_status("pack");
    }
    int64_t per_chunk = (int64_t)(staging_dev_bytes / rec);
    if (per_chunk > 0x40000000ll) per_chunk = 0x40000000ll;
    for (int64_t first = 0; first < n; first += per_chunk) {
        const int64_t cnt = n - first < per_chunk ? n - first : per_chunk;
        pack_kernel<<<(unsigned)cnt, kThreads, 0, st>>>(kp, vp, (uint32_t)pool->n_slots, k_v4, v_v4, slot_tbl, state,
                                                       n_uids, uids, host_slots, freed_slots, first, n_dev,
                                                       static_cast<uint4*>(staging_dev), n_bad);
        if (int rc = launch_status("pack")) return rc;
        if (staging_host)
            KVM_HIP_TRY(hipMemcpyAsync(static_cast<char*>(staging_host) + first * rec, staging_dev, (size_t)cnt * rec,
                                       hipMemcpyDeviceToHost, st));
    }
    return KVM_OK;
}

extern "C" int kvm_unpack(const kvm_pool_t* pool, int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                          const int64_t* uids, int64_t n, const int64_t* n_dev, const int32_t* dst_slots,
                          void* staging_dev,
                          size_t staging_dev_bytes, const void* staging_host, size_t staging_host_bytes,
                          uint32_t* n_bad, void* stream) {
    using namespace kvm;
    clear_error();
    if (int rc = check_common("kvm_unpack", pool, slot_tbl, state, n_uids, uids, n, dst_slots, staging_dev,
                              staging_dev_bytes, staging_host, staging_host_bytes))
        return rc;
    if (n == 0) return KVM_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t k_v4 = pool->unit_k_bytes / 16, v_v4 = pool->unit_v_bytes / 16;
    const size_t rec = (size_t)pool->unit_k_bytes + pool->unit_v_bytes;
    uint4* kp = static_cast<uint4*>(pool->k_pool);
    uint4* vp = static_cast<uint4*>(pool->v_pool);
    TimedLaunch tl("unpack", st);
    if (!staging_dev) {
        for (int64_t first = 0; first < n; first += 0x40000000ll) {
            const int64_t cnt = n - first < 0x40000000ll ? n - first : 0x40000000ll;
            unpack_kernel<<<(unsigned)cnt, kThreads, 0, st>>>(
                kp, vp, (uint32_t)pool->n_slots, k_v4, v_v4, slot_tbl, state, n_uids, uids, dst_slots, first, n_dev,
                reinterpret_cast<const uint4*>(static_cast<const char*>(staging_host) + first * rec), n_bad);
        }
        return launch_status("unpack");
    }
    int64_t per_chunk = (int64_t)(staging_dev_bytes / rec);
    if (per_chunk > 0x40000000ll) per_chunk = 0x40000000ll;
    for (int64_t first = 0; first < n; first += per_chunk) {
        const int64_t cnt = n - first < per_chunk ? n - first : per_chunk;
        if (staging_host)
            KVM_HIP_TRY(hipMemcpyAsync(staging_dev, static_cast<const char*>(staging_host) + first * rec,
                                       (size_t)cnt * rec, hipMemcpyHostToDevice, st));
        unpack_kernel<<<(unsigned)cnt, kThreads, 0, st>>>(kp, vp, (uint32_t)pool->n_slots, k_v4, v_v4, slot_tbl, state,
                                                         n_uids, uids, dst_slots, first, n_dev,
                                                         static_cast<const uint4*>(staging_dev), n_bad);
        if (int rc = launch_status("unpack")) return rc;
    }
    return KVM_OK;
}

extern "C" int kvm_swap(const kvm_pool_t* pool, int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                        const int64_t* out_uids, const int64_t* in_uids, int64_t n, const int64_t* n_dev,
                        const int32_t* host_slots, int32_t* freed_slots, void* host_out, size_t host_out_bytes,
                        const void* host_in, size_t host_in_bytes, uint32_t* n_bad, void* stream) {
    using namespace kvm;
    clear_error();
    if (int rc = check_common("kvm_swap", pool, slot_tbl, state, n_uids, out_uids, n, host_slots, nullptr, 0, host_out,
                              host_out_bytes))
        return rc;
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(in_uids && freed_slots && host_in && host_out, KVM_EINVAL, "kvm_swap: null buffer");
    const size_t rec = (size_t)pool->unit_k_bytes + pool->unit_v_bytes;
    KVM_REQUIRE(host_in_bytes / rec >= (size_t)n, KVM_ENOSPC, "kvm_swap: host_in %zu bytes < %lld records of %zu",
                host_in_bytes, (long long)n, rec);
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(host_in) % 16 == 0, KVM_EINVAL, "kvm_swap: host_in must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t k_v4 = pool->unit_k_bytes / 16, v_v4 = pool->unit_v_bytes / 16;
    TimedLaunch tl("swap", st);
    for (int64_t first = 0; first < n; first += 0x40000000ll) {
        const int64_t cnt = n - first < 0x40000000ll ? n - first : 0x40000000ll;
        swap_kernel<<<(unsigned)cnt, kThreads, 0, st>>>(
            static_cast<uint4*>(pool->k_pool), static_cast<uint4*>(pool->v_pool), (uint32_t)pool->n_slots, k_v4, v_v4,
            slot_tbl, state, n_uids, out_uids, in_uids, host_slots, freed_slots, first, n_dev,
            reinterpret_cast<uint4*>(static_cast<char*>(host_out) + first * rec),
            reinterpret_cast<const uint4*>(static_cast<const char*>(host_in) + first * rec), n_bad);
    }
    return launch_status("swap");
}

extern "C" int kvm_exchange(const kvm_pool_t* pool, int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                            const int64_t* out_uids, const int64_t* in_uids, int64_t n, const int64_t* n_out_dev,
                            const int64_t* n_in_dev, void* host_tier, uint64_t tier_slots, uint32_t* n_bad,
                            void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(pool, KVM_EINVAL, "kvm_exchange: null pool");
    KVM_REQUIRE(n >= 0 && n_uids >= 0, KVM_EINVAL, "kvm_exchange: negative count");
    KVM_REQUIRE(pool->unit_k_bytes > 0 && pool->unit_k_bytes % 16 == 0 && pool->unit_v_bytes % 16 == 0, KVM_ESHAPE,
                "kvm_exchange: unit sizes (%u, %u) must be multiples of 16", pool->unit_k_bytes, pool->unit_v_bytes);
    KVM_REQUIRE(pool->n_slots <= 0x7fffffffull && tier_slots <= 0x7fffffffull, KVM_EINVAL,
                "kvm_exchange: slot counts exceed int32 ids");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(pool->k_pool && (pool->v_pool || pool->unit_v_bytes == 0), KVM_EINVAL, "kvm_exchange: null pool memory");
    KVM_REQUIRE(slot_tbl && state && out_uids && in_uids && host_tier, KVM_EINVAL, "kvm_exchange: null buffer");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(host_tier) % 16 == 0, KVM_EINVAL,
                "kvm_exchange: host tier must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t k_v4 = pool->unit_k_bytes / 16, v_v4 = pool->unit_v_bytes / 16;
    TimedLaunch tl("swap", st);
    for (int64_t first = 0; first < n; first += 0x40000000ll) {
        const int64_t cnt = n - first < 0x40000000ll ? n - first : 0x40000000ll;
        exchange_kernel<<<(unsigned)cnt, kThreads, 0, st>>>(
            static_cast<uint4*>(pool->k_pool), static_cast<uint4*>(pool->v_pool), (uint32_t)pool->n_slots, k_v4, v_v4,
            slot_tbl, state, n_uids, out_uids, in_uids, first, n_out_dev, n_in_dev, static_cast<uint4*>(host_tier),
            tier_slots, n_bad);
    }
    return launch_status("exchange");
}

extern "C" int kvm_exchange_begin(const kvm_pool_t* pool, int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                                  const int64_t* out_uids, const int64_t* in_uids, int64_t n,
                                  const int64_t* n_out_dev, const int64_t* n_in_dev, uint64_t tier_slots,
                                  int32_t* frame, int64_t* host, uint32_t* n_bad, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(pool, KVM_EINVAL, "kvm_exchange_begin: null pool");
    KVM_REQUIRE(n >= 0 && n_uids >= 0, KVM_EINVAL, "kvm_exchange_begin: negative count");
    KVM_REQUIRE(pool->n_slots <= 0x7fffffffull && tier_slots <= 0x7fffffffull, KVM_EINVAL,
                "kvm_exchange_begin: slot counts exceed int32 ids");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(slot_tbl && state && out_uids && in_uids && frame && host, KVM_EINVAL,
                "kvm_exchange_begin: null buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("exchange_flip", st);
    exchange_begin_kernel<<<(unsigned)((n + kThreads - 1) / kThreads), kThreads, 0, st>>>(
        (uint32_t)pool->n_slots, slot_tbl, state, n_uids, out_uids, in_uids, n, n_out_dev, n_in_dev, tier_slots, frame,
        host, n_bad);
    return launch_status("exchange_begin");
}

extern "C" int kvm_pack_begin(const kvm_pool_t* pool, int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                              const int64_t* uids, int64_t n, const int64_t* n_dev, const int32_t* host_slots,
                              uint64_t tier_slots, int32_t* frame, int64_t* host, uint32_t* n_bad, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(pool, KVM_EINVAL, "kvm_pack_begin: null pool");
    KVM_REQUIRE(n >= 0 && n_uids >= 0, KVM_EINVAL, "kvm_pack_begin: negative count");
    KVM_REQUIRE(pool->n_slots <= 0x7fffffffull, KVM_EINVAL, "kvm_pack_begin: n_slots exceeds int32 slot ids");
    KVM_REQUIRE(tier_slots <= 0x7fffffffull, KVM_EINVAL, "kvm_pack_begin: tier_slots exceeds int32 slot ids");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(slot_tbl && state && uids && host_slots && frame && host, KVM_EINVAL, "kvm_pack_begin: null buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("exchange_flip", st);
    pack_begin_kernel<<<(unsigned)((n + kThreads - 1) / kThreads), kThreads, 0, st>>>(
        (uint32_t)pool->n_slots, slot_tbl, state, n_uids, uids, n, n_dev, host_slots, tier_slots, frame, host, n_bad);
    return launch_status("pack_begin");
}

extern "C" int kvm_exchange_end(int32_t* slot_tbl, uint8_t* state, int64_t n_uids, const int64_t* in_uids,
                                const int32_t* frame, int64_t n, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(n >= 0 && n_uids >= 0, KVM_EINVAL, "kvm_exchange_end: negative count");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(slot_tbl && state && in_uids && frame, KVM_EINVAL, "kvm_exchange_end: null buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("exchange_flip", st);
    exchange_end_kernel<<<(unsigned)((n + kThreads - 1) / kThreads), kThreads, 0, st>>>(slot_tbl, state, n_uids,
                                                                                       in_uids, frame, n);
    return launch_status("exchange_end");
}
