// Error text, version, kernel timing and the host-only sizing entry point.
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "kvm_internal.h"

namespace kvm {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = 0; }

// ---- timing ----------------------------------------------------------------
namespace {
struct Span {
    const char* name;
    hipEvent_t start, stop;
};
std::mutex g_mu;
bool g_on = false;
std::string g_only;                 // if not empty: the one span name that is timed
std::vector<Span> g_spans;          // spans recorded since the last reset
std::vector<hipEvent_t> g_free;     // events ready for reuse

hipEvent_t take_event() {
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

TimedLaunch::TimedLaunch(const char* name, hipStream_t stream) : slot_(-1), stream_(stream) {
    if (!name) return;                  // a launch that must not touch the event pool
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_on) return;
    if (!g_only.empty() && g_only != name) return;
    Span s{name, take_event(), take_event()};
    if (!s.start || !s.stop) return;
    if (hipEventRecord(s.start, stream) != hipSuccess) return;
    g_spans.push_back(s);
    slot_ = (int)g_spans.size() - 1;
}

TimedLaunch::~TimedLaunch() {
    if (slot_ < 0) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (slot_ < (int)g_spans.size()) (void)hipEventRecord(g_spans[slot_].stop, stream_);
}

}  // namespace kvm

namespace kvm {
namespace {
// Plain streaming read: every byte of the buffer once, 16-byte non-temporal loads, nothing else.
// A wavefront takes 4 KiB pieces (four loads of 1 KiB, the shape of a d = 128 frame), two pieces in
// flight; everything is folded into one word so that no load can be optimised away.  The rate of this
// kernel is the ceiling any kernel that has to read the same bytes can reach on the chip at hand.
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ p, size_t n_v4, uint32_t* out) {
    typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
    const v4u_t* q = reinterpret_cast<const v4u_t*>(p);
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (size_t)gridDim.x * 4;
    const size_t n_pieces = n_v4 / 256;                 // whole 4 KiB pieces
    constexpr int U = 2;
    uint32_t acc = 0;
    for (size_t c = wave * U; c < n_pieces; c += n_waves * U) {
        v4u_t v[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t cc = c + u < n_pieces ? c + u : c;
#pragma unroll
            for (int k = 0; k < 4; ++k) v[u][k] = __builtin_nontemporal_load(q + cc * 256 + k * 64 + lane);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (c + u < n_pieces)
#pragma unroll
                for (int k = 0; k < 4; ++k) acc ^= v[u][k].x ^ v[u][k].y ^ v[u][k].z ^ v[u][k].w;
    }
    // the tail that does not fill a piece
    for (size_t i = n_pieces * 256 + (size_t)blockIdx.x * 256 + threadIdx.x; i < n_v4; i += (size_t)gridDim.x * 256) {
        const v4u_t v = __builtin_nontemporal_load(q + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) atomicAdd(out, 1u);      // practically never: keeps the loads alive
}
}  // namespace
}  // namespace kvm

extern "C" {

const char* kvm_last_error(void) { return kvm::g_err; }

const char* kvm_version(void) { return "0.4"; }

int kvm_probe_read(const void* buf, size_t bytes, uint32_t* sink, void* stream) {
    using namespace kvm;
    clear_error();
    KVM_REQUIRE(buf && sink, KVM_EINVAL, "kvm_probe_read: null buffer");
    KVM_REQUIRE(reinterpret_cast<uintptr_t>(buf) % 16 == 0 && bytes % 16 == 0, KVM_EINVAL,
                "kvm_probe_read: buffer and size must be multiples of 16");
    if (bytes == 0) return KVM_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedLaunch tl("probe_read", st);
    probe_read_kernel<<<256 * 32, 256, 0, st>>>(static_cast<const uint4*>(buf), bytes / 16, sink);
    return launch_status("probe_read");
}

int kvm_timing_enable(int on) {
    std::lock_guard<std::mutex> lk(kvm::g_mu);
    kvm::g_on = on != 0;
    return KVM_OK;
}

int kvm_timing_only(const char* name) {
    std::lock_guard<std::mutex> lk(kvm::g_mu);
    kvm::g_only = name ? name : "";
    return KVM_OK;
}

void kvm_timing_reset(void) {
    std::lock_guard<std::mutex> lk(kvm::g_mu);
    for (auto& s : kvm::g_spans) {
        (void)hipEventSynchronize(s.stop);
        kvm::g_free.push_back(s.start);
        kvm::g_free.push_back(s.stop);
    }
    kvm::g_spans.clear();
}

int kvm_timing_read(const char* name, double* total_ms) {
    if (!name || !total_ms) return 0;
    std::lock_guard<std::mutex> lk(kvm::g_mu);
    int n = 0;
    double sum = 0.0;
    for (auto& s : kvm::g_spans) {
        if (std::strcmp(s.name, name) != 0) continue;
        if (hipEventSynchronize(s.stop) != hipSuccess) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, s.start, s.stop) != hipSuccess) continue;
        sum += ms;
        ++n;
    }
    *total_ms = sum;
    return n;
}

// ---------------------------------------------------------------------------
// Sizing: per-layer KV bytes by attention architecture (section 3.1, Eq. 3) and
// the largest batch that fits a memory target (Eq. 4 and the floor formula
// after it).  Integer arithmetic in bits so that sub-byte precisions stay exact.
// ---------------------------------------------------------------------------
int kvm_size(const kvm_model_t* m, uint64_t n_max, uint64_t mem_target_bytes, kvm_sizing_t* out) {
    kvm::clear_error();
    KVM_REQUIRE(m && out, KVM_EINVAL, "kvm_size: null argument");
    KVM_REQUIRE(m->n_layers > 0, KVM_EINVAL, "kvm_size: n_layers must be positive");
    KVM_REQUIRE(m->block_tokens > 0, KVM_EINVAL, "kvm_size: block_tokens must be positive");
    KVM_REQUIRE(m->head_divisor >= 1, KVM_EINVAL, "kvm_size: head_divisor must be >= 1");
    const int bits = m->bits_per_elem;
    KVM_REQUIRE(bits == 4 || bits == 8 || bits == 16 || bits == 32, KVM_EINVAL,
                "kvm_size: bits_per_elem %d not in {4, 8, 16, 32}", bits);
    kvm_sizing_t s;
    std::memset(&s, 0, sizeof s);
    uint64_t tok_layer_bits, unit_k_bits, unit_v_bits, kv_heads;
    if (m->d_latent > 0) {
        KVM_REQUIRE(m->d_rope >= 0 && m->n_q_heads > 0, KVM_EINVAL, "kvm_size: bad MLA dimensions");
        s.arch = KVM_ARCH_MLA;
        s.group_size = m->n_q_heads;
        kv_heads = 1;
        const uint64_t width = (uint64_t)m->d_latent + (uint64_t)m->d_rope;
        tok_layer_bits = width * bits;
        unit_k_bits = (uint64_t)m->block_tokens * width * bits;
        unit_v_bits = 0;
    } else {
        KVM_REQUIRE(m->n_q_heads > 0 && m->n_kv_heads > 0 && m->head_dim > 0, KVM_EINVAL,
                    "kvm_size: head counts and head_dim must be positive");
        KVM_REQUIRE(m->n_q_heads % m->n_kv_heads == 0, KVM_EINVAL,
                    "kvm_size: n_kv_heads %d does not divide n_q_heads %d", m->n_kv_heads, m->n_q_heads);
        KVM_REQUIRE(m->n_kv_heads % m->head_divisor == 0, KVM_EINVAL,
                    "kvm_size: head_divisor %d does not divide n_kv_heads %d", m->head_divisor, m->n_kv_heads);
        s.arch = m->n_q_heads == m->n_kv_heads ? KVM_ARCH_MHA
                 : m->n_kv_heads == 1          ? KVM_ARCH_MQA
                                               : KVM_ARCH_GQA;
        s.group_size = m->n_q_heads / m->n_kv_heads;
        kv_heads = (uint64_t)(m->n_kv_heads / m->head_divisor);
        tok_layer_bits = 2ull * kv_heads * (uint64_t)m->head_dim * bits;   // K and V
        unit_k_bits = unit_v_bits = (uint64_t)m->block_tokens * (uint64_t)m->head_dim * bits;
    }
    KVM_REQUIRE(tok_layer_bits % 8 == 0 && unit_k_bits % 8 == 0 && unit_v_bits % 8 == 0, KVM_EINVAL,
                "kvm_size: sizes are not whole bytes at %d bits per element", bits);
    s.bytes_per_token_layer = tok_layer_bits / 8;
    s.bytes_per_token = s.bytes_per_token_layer * (uint64_t)m->n_layers;
    s.bytes_per_seq = s.bytes_per_token * n_max;
    s.max_batch = s.bytes_per_seq ? mem_target_bytes / s.bytes_per_seq : 0;
    s.units_per_block = (uint32_t)((uint64_t)m->n_layers * kv_heads);
    s.unit_k_bytes = (uint32_t)(unit_k_bits / 8);
    s.unit_v_bytes = (uint32_t)(unit_v_bits / 8);
    s.pool_units = mem_target_bytes / ((uint64_t)s.unit_k_bytes + s.unit_v_bytes);
    // Head weights of the eviction priority (section 3.4): every head counts the same under MHA; a
    // grouped KV head stands for all the query heads that share it; MLA has one latent head per layer.
    s.head_weight = (s.arch == KVM_ARCH_GQA || s.arch == KVM_ARCH_MQA) ? (uint32_t)s.group_size : 1u;
    *out = s;
    return KVM_OK;
}

}  // extern "C"
