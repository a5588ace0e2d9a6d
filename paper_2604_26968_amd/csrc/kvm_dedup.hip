// kvm_hash_units, kvm_dedup_insert, kvm_dedup_release: content addressing of units
// (section 3.6 of the paper: blocks indexed by the SHA-256 of their content, a match raises
// a reference count instead of storing the block again).
//
// hash   : SHA-256 (FIPS 180-4) of a unit's record, K frame then V frame.  The hash is a
//          serial chain over the record's 64-byte blocks, so one lane hashes one unit; the
//          work is integer ALU (about 30 operations per byte), not memory.
// store  : open-addressing table in device memory keyed by the first 64 bits of the digest;
//          every match is confirmed on all 256 bits, so a collision of the 64-bit keys can
//          only cost a missed match, never a false one.
#include "kvm_internal.h"

namespace kvm {
namespace {

__device__ __constant__ uint32_t kShaK[64] = {
    0x428a2f98u, 0x71374491u, 0xb5c0fbcfu, 0xe9b5dba5u, 0x3956c25bu, 0x59f111f1u, 0x923f82a4u, 0xab1c5ed5u,
    0xd807aa98u, 0x12835b01u, 0x243185beu, 0x550c7dc3u, 0x72be5d74u, 0x80deb1feu, 0x9bdc06a7u, 0xc19bf174u,
    0xe49b69c1u, 0xefbe4786u, 0x0fc19dc6u, 0x240ca1ccu, 0x2de92c6fu, 0x4a7484aau, 0x5cb0a9dcu, 0x76f988dau,
    0x983e5152u, 0xa831c66du, 0xb00327c8u, 0xbf597fc7u, 0xc6e00bf3u, 0xd5a79147u, 0x06ca6351u, 0x14292967u,
    0x27b70a85u, 0x2e1b2138u, 0x4d2c6dfcu, 0x53380d13u, 0x650a7354u, 0x766a0abbu, 0x81c2c92eu, 0x92722c85u,
    0xa2bfe8a1u, 0xa81a664bu, 0xc24b8b70u, 0xc76c51a3u, 0xd192e819u, 0xd6990624u, 0xf40e3585u, 0x106aa070u,
    0x19a4c116u, 0x1e376c08u, 0x2748774cu, 0x34b0bcb5u, 0x391c0cb3u, 0x4ed8aa4au, 0x5b9cca4fu, 0x682e6ff3u,
    0x748f82eeu, 0x78a5636fu, 0x84c87814u, 0x8cc70208u, 0x90befffau, 0xa4506cebu, 0xbef9a3f7u, 0xc67178f2u};

__device__ __forceinline__ uint32_t rotr(uint32_t x, int n) { return __builtin_rotateright32(x, n); }

// One compression of the 16 big-endian message words in w (destroyed) into the state h.
__device__ __forceinline__ void sha_compress(uint32_t (&h)[8], uint32_t (&w)[16]) {
    uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], hh = h[7];
#pragma unroll
    for (int t = 0; t < 64; ++t) {
        if (t >= 16) {
            const uint32_t w15 = w[(t - 15) & 15], w2 = w[(t - 2) & 15];
            const uint32_t s0 = rotr(w15, 7) ^ rotr(w15, 18) ^ (w15 >> 3);
            const uint32_t s1 = rotr(w2, 17) ^ rotr(w2, 19) ^ (w2 >> 10);
            w[t & 15] = s1 + w[(t - 7) & 15] + s0 + w[t & 15];
        }
        const uint32_t S1 = rotr(e, 6) ^ rotr(e, 11) ^ rotr(e, 25);
        const uint32_t ch = (e & f) ^ (~e & g);
        const uint32_t t1 = hh + S1 + ch + kShaK[t] + w[t & 15];
        const uint32_t S0 = rotr(a, 2) ^ rotr(a, 13) ^ rotr(a, 22);
        const uint32_t maj = (a & b) ^ (a & c) ^ (b & c);
        hh = g;
        g = f;
        f = e;
        e = d + t1;
        d = c;
        c = b;
        b = a;
        a = t1 + S0 + maj;
    }
    h[0] += a;
    h[1] += b;
    h[2] += c;
    h[3] += d;
    h[4] += e;
    h[5] += f;
    h[6] += g;
    h[7] += hh;
}

__device__ __forceinline__ void sha_absorb(uint32_t (&h)[8], const uint4* __restrict__ p, uint32_t n_blocks) {
    for (uint32_t blk = 0; blk < n_blocks; ++blk) {
        uint32_t w[16];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const uint4 x = p[blk * 4 + v];
            w[4 * v + 0] = __builtin_bswap32(x.x);
            w[4 * v + 1] = __builtin_bswap32(x.y);
            w[4 * v + 2] = __builtin_bswap32(x.z);
            w[4 * v + 3] = __builtin_bswap32(x.w);
        }
        sha_compress(h, w);
    }
}

constexpr int kHashThreads = 64;   // one wavefront per workgroup: 64 units, spread over many compute units

__global__ __launch_bounds__(kHashThreads) void hash_units_kernel(const uint4* __restrict__ k_pool,
                                                                  const uint4* __restrict__ v_pool, uint32_t n_slots,
                                                                  uint32_t k_bytes, uint32_t v_bytes,
                                                                  const int32_t* __restrict__ slot_tbl,
                                                                  const uint8_t* __restrict__ state, int64_t n_uids,
                                                                  const int64_t* __restrict__ uids, int64_t n,
                                                                  uint32_t* __restrict__ digests, uint32_t* n_bad) {
    const int64_t i = (int64_t)blockIdx.x * kHashThreads + threadIdx.x;
    if (i >= n) return;
    const int64_t uid = uids[i];
    int32_t slot = -1;
    if (uid >= 0 && uid < n_uids && (state[uid] & KVM_ST_RESIDENT)) slot = slot_tbl[uid];
    if ((uint32_t)slot >= n_slots) slot = -1;
    uint32_t* out = digests + 8 * i;
    if (slot < 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) out[k] = 0;
        if (n_bad) atomicAdd(n_bad, 1u);
        return;
    }
    uint32_t h[8] = {0x6a09e667u, 0xbb67ae85u, 0x3c6ef372u, 0xa54ff53au,
                     0x510e527fu, 0x9b05688cu, 0x1f83d9abu, 0x5be0cd19u};
    sha_absorb(h, k_pool + (size_t)slot * (k_bytes / 16), k_bytes / 64);
    if (v_bytes) sha_absorb(h, v_pool + (size_t)slot * (v_bytes / 16), v_bytes / 64);
    // the record is a whole number of 64-byte blocks: the padding is one more block
    uint32_t w[16];
    w[0] = 0x80000000u;
#pragma unroll
    for (int k = 1; k < 14; ++k) w[k] = 0;
    const uint64_t bits = ((uint64_t)k_bytes + v_bytes) * 8;
    w[14] = (uint32_t)(bits >> 32);
    w[15] = (uint32_t)bits;
    sha_compress(h, w);
#pragma unroll
    for (int k = 0; k < 8; ++k) out[k] = __builtin_bswap32(h[k]);   // digest bytes are big-endian words
}

// ---- store ----------------------------------------------------------------------------------
constexpr uint32_t kNoItem = 0xffffffffu;
constexpr int kMaxProbe = 1 << 16;

struct Store {
    unsigned long long* tag;
    uint32_t* digest;   // [cap][8]
    long long* canon;
    uint32_t* refs;
    uint32_t* pending;
    uint64_t mask;
};

__device__ __forceinline__ unsigned long long tag_of(const uint32_t* d) {
    const unsigned long long t = ((unsigned long long)d[1] << 32) | d[0];
    return t ? t : 1ull;                 // 0 marks an empty place
}
__device__ __forceinline__ bool digest_is_zero(const uint32_t* d) {
    uint32_t o = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) o |= d[k];
    return o == 0;
}

// Pass 1: every item finds or claims the place of its 64-bit key and leaves its index there if it
// is the lowest so far.
__global__ __launch_bounds__(256) void dedup_claim_kernel(Store s, const uint32_t* __restrict__ digests, int64_t n,
                                                          int64_t* __restrict__ entry_of, uint32_t* n_full) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t* d = digests + 8 * i;
    int64_t where = -1;
    if (!digest_is_zero(d)) {
        const unsigned long long tag = tag_of(d);
        uint64_t pos = (tag >> 7) & s.mask;
        for (int probe = 0; probe < kMaxProbe && (uint64_t)probe <= s.mask; ++probe) {
            const unsigned long long prev = atomicCAS(&s.tag[pos], 0ull, tag);
            if (prev == 0ull || prev == tag) {
                where = (int64_t)pos;
                break;
            }
            pos = (pos + 1) & s.mask;
        }
        if (where < 0 && n_full) atomicAdd(n_full, 1u);
    }
    entry_of[i] = where;
    if (where >= 0) atomicMin(&s.pending[where], (uint32_t)i);
}

// Pass 2: the lowest item of a place that holds no live entry becomes its canonical copy.
__global__ __launch_bounds__(256) void dedup_settle_kernel(Store s, const uint32_t* __restrict__ digests,
                                                           const int64_t* __restrict__ uids, int64_t n,
                                                           const int64_t* __restrict__ entry_of) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t pos = entry_of[i];
    if (pos < 0 || s.pending[pos] != (uint32_t)i) return;
    if (s.canon[pos] >= 0 && s.refs[pos] > 0) return;      // live entry: nothing to settle
#pragma unroll
    for (int k = 0; k < 8; ++k) s.digest[8 * pos + k] = digests[8 * i + k];
    s.canon[pos] = uids[i];
}

// Pass 3: confirm the match on all 256 bits, count the reference, report the canonical copy.
__global__ __launch_bounds__(256) void dedup_resolve_kernel(Store s, const uint32_t* __restrict__ digests,
                                                            const int64_t* __restrict__ uids, int64_t n,
                                                            const int64_t* __restrict__ entry_of,
                                                            int64_t* __restrict__ canon_out, uint32_t* n_collide) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t pos = entry_of[i];
    int64_t canon = uids[i];
    if (pos >= 0) {
        bool same = true;
#pragma unroll
        for (int k = 0; k < 8; ++k) same &= s.digest[8 * pos + k] == digests[8 * i + k];
        if (same) {
            atomicAdd(&s.refs[pos], 1u);
            canon = s.canon[pos];
        } else if (n_collide) {
            atomicAdd(n_collide, 1u);
        }
        s.pending[pos] = kNoItem;
    }
    canon_out[i] = canon;
}

__global__ __launch_bounds__(256) void dedup_release_kernel(Store s, const uint32_t* __restrict__ digests, int64_t n,
                                                            uint32_t* n_bad) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t* d = digests + 8 * i;
    bool done = false;
    if (!digest_is_zero(d)) {
        const unsigned long long tag = tag_of(d);
        uint64_t pos = (tag >> 7) & s.mask;
        for (int probe = 0; probe < kMaxProbe && (uint64_t)probe <= s.mask; ++probe) {
            const unsigned long long cur = s.tag[pos];
            if (cur == 0ull) break;
            if (cur == tag) {
                bool same = true;
#pragma unroll
                for (int k = 0; k < 8; ++k) same &= s.digest[8 * pos + k] == d[k];
                if (same) {
                    uint32_t old = s.refs[pos];
                    while (old > 0) {
                        const uint32_t seen = atomicCAS(&s.refs[pos], old, old - 1);
                        if (seen == old) {
                            done = true;
                            break;
                        }
                        old = seen;
                    }
                }
                break;
            }
            pos = (pos + 1) & s.mask;
        }
    }
    if (!done && n_bad) atomicAdd(n_bad, 1u);
}

int check_store(const char* who, const kvm_store_t* st, Store* out) {
    KVM_REQUIRE(st, KVM_EINVAL, "%s: null store", who);
    KVM_REQUIRE(st->cap >= 2 && (st->cap & (st->cap - 1)) == 0, KVM_EINVAL, "%s: capacity %llu is not a power of two",
                who, (unsigned long long)st->cap);
    KVM_REQUIRE(st->tag && st->digest && st->canon && st->refs && st->pending, KVM_EINVAL, "%s: null store array", who);
    *out = Store{reinterpret_cast<unsigned long long*>(st->tag), reinterpret_cast<uint32_t*>(st->digest),
                 reinterpret_cast<long long*>(st->canon), st->refs, st->pending, st->cap - 1};
    return KVM_OK;
}

// ---- frames shared by duplicates ------------------------------------------------------------------
// Two launches: the first moves the duplicates (every item writes only its own unit's entries), the second
// flags the canonical units.  Several duplicates of one canonical unit then store the same byte, and no
// launch reads a state byte that another of its threads may be changing.

__global__ __launch_bounds__(256) void dedup_share_kernel(int32_t* __restrict__ slot_tbl, uint8_t* __restrict__ state,
                                                          int64_t n_uids, uint32_t n_slots,
                                                          const int64_t* __restrict__ uids,
                                                          const int64_t* __restrict__ canon, int64_t n,
                                                          uint32_t* __restrict__ frame_refs,
                                                          int32_t* __restrict__ freed, uint32_t* n_bad) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t u = uids[i], c = canon[i];
    int32_t out = -1;
    if (u < 0 || u >= n_uids || c < 0 || c >= n_uids) {
        if (n_bad) atomicAdd(n_bad, 1u);
    } else if (u != c) {
        const uint8_t su = state[u], sc = state[c];
        const int32_t fu = slot_tbl[u], fc = slot_tbl[c];
        if ((su & KVM_ST_RESIDENT) && (sc & KVM_ST_RESIDENT) && !(su & (KVM_ST_PROTECTED | KVM_ST_SHARED)) &&
            !(sc & KVM_ST_PROTECTED) && (uint32_t)fu < n_slots && (uint32_t)fc < n_slots && fu != fc) {
            slot_tbl[u] = fc;
            out = fu;
            state[u] = su | KVM_ST_SHARED;
            // the canonical unit's own reading is counted by whichever duplicate comes first
            if (atomicAdd(&frame_refs[fc], 1u) == 0) atomicAdd(&frame_refs[fc], 1u);
        }
    }
    freed[i] = out;
}

__global__ __launch_bounds__(256) void dedup_share_flag_kernel(uint8_t* __restrict__ state, const int64_t* __restrict__ canon,
                                                               int64_t n, const int32_t* __restrict__ freed) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n || freed[i] < 0) return;           // an accepted item: its canonical uid was checked by the first launch
    state[canon[i]] |= KVM_ST_SHARED;
}

// One workgroup per item: thread 0 decides, everyone copies.
__global__ __launch_bounds__(256) void dedup_unshare_kernel(uint4* __restrict__ k_pool, uint4* __restrict__ v_pool,
                                                            uint32_t n_slots, uint32_t k_v4, uint32_t v_v4,
                                                            int32_t* __restrict__ slot_tbl, uint8_t* __restrict__ state,
                                                            int64_t n_uids, const int64_t* __restrict__ uids,
                                                            const int32_t* __restrict__ new_frames,
                                                            uint32_t* __restrict__ frame_refs,
                                                            int32_t* __restrict__ freed, uint32_t* n_bad) {
    __shared__ int32_t s_from;
    const int64_t i = blockIdx.x;
    const int32_t nf = new_frames[i];
    if (threadIdx.x == 0) {
        const int64_t u = uids[i];
        int32_t from = -1;
        if (u < 0 || u >= n_uids || (uint32_t)nf >= n_slots) {
            if (n_bad) atomicAdd(n_bad, 1u);
        } else if ((state[u] & (KVM_ST_RESIDENT | KVM_ST_SHARED)) == (KVM_ST_RESIDENT | KVM_ST_SHARED)) {
            const int32_t f = slot_tbl[u];
            if ((uint32_t)f < n_slots && f != nf && frame_refs[f] != 0) from = f;
        }
        s_from = from;
        if (from < 0) freed[i] = nf;
    }
    __syncthreads();
    const int32_t f = s_from;
    if (f < 0) return;
    const uint4* ks = k_pool + (size_t)f * k_v4;
    uint4* kd = k_pool + (size_t)nf * k_v4;
    for (uint32_t v = threadIdx.x; v < k_v4; v += 256) kd[v] = ks[v];
    if (v_v4) {
        const uint4* vs = v_pool + (size_t)f * v_v4;
        uint4* vd = v_pool + (size_t)nf * v_v4;
        for (uint32_t v = threadIdx.x; v < v_v4; v += 256) vd[v] = vs[v];
    }
    __syncthreads();                       // the copy has been read before the old frame may be reported free
    if (threadIdx.x == 0) {
        const int64_t u = uids[i];
        slot_tbl[u] = nf;
        state[u] &= (uint8_t)~KVM_ST_SHARED;
        freed[i] = atomicSub(&frame_refs[f], 1u) == 1u ? f : -1;
    }
}

}  // namespace
}  // namespace kvm

extern "C" int kvm_dedup_share(int32_t* slot_tbl, uint8_t* state, int64_t n_uids, uint64_t n_slots, const int64_t* uids,
                               const int64_t* canon, int64_t n, uint32_t* frame_refs, int32_t* freed, uint32_t* n_bad,
                               void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(n >= 0 && n_uids >= 0, KVM_EINVAL, "kvm_dedup_share: negative count");
    KVM_REQUIRE(n_slots <= 0x7fffffffull, KVM_EINVAL, "kvm_dedup_share: n_slots exceeds int32 slot ids");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(slot_tbl && state && uids && canon && frame_refs && freed, KVM_EINVAL, "kvm_dedup_share: null buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("dedup", st);
    dedup_share_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(slot_tbl, state, n_uids, (uint32_t)n_slots, uids,
                                                                     canon, n, frame_refs, freed, n_bad);
    dedup_share_flag_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(state, canon, n, freed);
    return launch_status("dedup_share");
}

extern "C" int kvm_dedup_unshare(const kvm_pool_t* pool, int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                                 const int64_t* uids, const int32_t* new_frames, int64_t n, uint32_t* frame_refs,
                                 int32_t* freed, uint32_t* n_bad, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(pool, KVM_EINVAL, "kvm_dedup_unshare: null pool");
    KVM_REQUIRE(n >= 0 && n_uids >= 0 && n <= 0x7fffffffll, KVM_EINVAL, "kvm_dedup_unshare: count out of range");
    KVM_REQUIRE(pool->unit_k_bytes > 0 && pool->unit_k_bytes % 16 == 0 && pool->unit_v_bytes % 16 == 0, KVM_ESHAPE,
                "kvm_dedup_unshare: unit sizes (%u, %u) must be multiples of 16", pool->unit_k_bytes,
                pool->unit_v_bytes);
    KVM_REQUIRE(pool->n_slots <= 0x7fffffffull, KVM_EINVAL, "kvm_dedup_unshare: n_slots exceeds int32 slot ids");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(pool->k_pool && (pool->v_pool || pool->unit_v_bytes == 0), KVM_EINVAL,
                "kvm_dedup_unshare: null pool memory");
    KVM_REQUIRE(slot_tbl && state && uids && new_frames && frame_refs && freed, KVM_EINVAL,
                "kvm_dedup_unshare: null buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("dedup", st);
    dedup_unshare_kernel<<<(unsigned)n, 256, 0, st>>>(static_cast<uint4*>(pool->k_pool), static_cast<uint4*>(pool->v_pool),
                                                      (uint32_t)pool->n_slots, pool->unit_k_bytes / 16,
                                                      pool->unit_v_bytes / 16, slot_tbl, state, n_uids, uids, new_frames,
                                                      frame_refs, freed, n_bad);
    return launch_status("dedup_unshare");
}

extern "C" int kvm_hash_units(const kvm_pool_t* pool, const int32_t* slot_tbl, const uint8_t* state, int64_t n_uids,
                              const int64_t* uids, int64_t n, uint8_t* digests, uint32_t* n_bad, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(pool, KVM_EINVAL, "kvm_hash_units: null pool");
    KVM_REQUIRE(n >= 0 && n_uids >= 0, KVM_EINVAL, "kvm_hash_units: negative count");
    KVM_REQUIRE(pool->unit_k_bytes > 0 && pool->unit_k_bytes % 64 == 0 && pool->unit_v_bytes % 64 == 0, KVM_ESHAPE,
                "kvm_hash_units: unit sizes (%u, %u) must be multiples of 64", pool->unit_k_bytes,
                pool->unit_v_bytes);
    KVM_REQUIRE(pool->n_slots <= 0x7fffffffull, KVM_EINVAL, "kvm_hash_units: n_slots exceeds int32 slot ids");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(pool->k_pool && (pool->v_pool || pool->unit_v_bytes == 0), KVM_EINVAL, "kvm_hash_units: null pool memory");
    KVM_REQUIRE(slot_tbl && state && uids && digests, KVM_EINVAL, "kvm_hash_units: null buffer");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(digests) % 4 == 0, KVM_EINVAL, "kvm_hash_units: digests must be 4-byte aligned");
    KVM_REQUIRE(n <= 0x7fffffffll * kHashThreads, KVM_EINVAL, "kvm_hash_units: too many units for one call");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("hash", st);
    hash_units_kernel<<<(unsigned)((n + kHashThreads - 1) / kHashThreads), kHashThreads, 0, st>>>(
        static_cast<const uint4*>(pool->k_pool), static_cast<const uint4*>(pool->v_pool), (uint32_t)pool->n_slots,
        pool->unit_k_bytes, pool->unit_v_bytes, slot_tbl, state, n_uids, uids, n, reinterpret_cast<uint32_t*>(digests),
        n_bad);
    return launch_status("hash_units");
}

extern "C" int kvm_dedup_insert(const kvm_store_t* store, const uint8_t* digests, const int64_t* uids, int64_t n,
                                int64_t* canon_out, uint32_t* n_full, uint32_t* n_collide, void* ws, size_t ws_bytes,
                                void* stream) {
    using namespace kvm;
    clear_error();
    Store s;
    if (int rc = check_store("kvm_dedup_insert", store, &s)) return rc;
    KVM_REQUIRE(n >= 0 && n <= 0xfffffffell, KVM_EINVAL, "kvm_dedup_insert: item count %lld out of range", (long long)n);
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(digests && uids && canon_out, KVM_EINVAL, "kvm_dedup_insert: null buffer");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(digests) % 4 == 0, KVM_EINVAL, "kvm_dedup_insert: digests must be 4-byte aligned");
    KVM_REQUIRE(ws && ws_bytes >= (size_t)n * sizeof(int64_t) && reinterpret_cast<uintptr_t>(ws) % 8 == 0, KVM_ENOSPC,
                "kvm_dedup_insert: workspace needs %zu bytes, 8-byte aligned", (size_t)n * sizeof(int64_t));
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((n + 255) / 256);
    const uint32_t* d = reinterpret_cast<const uint32_t*>(digests);
    int64_t* entry_of = static_cast<int64_t*>(ws);
    TimedLaunch tl("dedup", st);
    dedup_claim_kernel<<<grid, 256, 0, st>>>(s, d, n, entry_of, n_full);
    dedup_settle_kernel<<<grid, 256, 0, st>>>(s, d, uids, n, entry_of);
    dedup_resolve_kernel<<<grid, 256, 0, st>>>(s, d, uids, n, entry_of, canon_out, n_collide);
    return launch_status("dedup_insert");
}

extern "C" int kvm_dedup_release(const kvm_store_t* store, const uint8_t* digests, int64_t n, uint32_t* n_bad,
                                 void* stream) {
    using namespace kvm;
    clear_error();
    Store s;
    if (int rc = check_store("kvm_dedup_release", store, &s)) return rc;
    KVM_REQUIRE(n >= 0, KVM_EINVAL, "kvm_dedup_release: negative count");
    if (n == 0) return KVM_OK;
    KVM_REQUIRE(digests, KVM_EINVAL, "kvm_dedup_release: null digests");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(digests) % 4 == 0, KVM_EINVAL, "kvm_dedup_release: digests must be 4-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("dedup", st);
    dedup_release_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(s, reinterpret_cast<const uint32_t*>(digests), n,
                                                                       n_bad);
    return launch_status("dedup_release");
}
