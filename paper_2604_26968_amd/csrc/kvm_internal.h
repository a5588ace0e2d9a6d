// Internal helpers shared by the translation units of libkvm (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "kvm.h"

namespace kvm {

// ---- error reporting -------------------------------------------------------
// Stores a printf-style message for kvm_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define KVM_HIP_TRY(expr)                                                                 \
    do {                                                                                  \
        hipError_t kvm_e_ = (expr);                                                       \
        if (kvm_e_ != hipSuccess)                                                         \
            return ::kvm::fail(KVM_EHIP, "%s: %s", #expr, hipGetErrorString(kvm_e_));     \
    } while (0)

#define KVM_REQUIRE(cond, code, ...)                     \
    do {                                                 \
        if (!(cond)) return ::kvm::fail(code, __VA_ARGS__); \
    } while (0)

// ---- kernel timing ---------------------------------------------------------
// Scope object: records a start event now and a stop event when it goes out of
// scope, both on `stream`, if timing is enabled.  Does nothing otherwise, and
// nothing at all when `name` is null.
class TimedLaunch {
  public:
    TimedLaunch(const char* name, hipStream_t stream);
    ~TimedLaunch();
    TimedLaunch(const TimedLaunch&) = delete;
    TimedLaunch& operator=(const TimedLaunch&) = delete;

  private:
    int slot_;
    hipStream_t stream_;
};

// Error of the most recent kernel launch on this thread, as a KVM code.
inline int launch_status(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(KVM_EHIP, "launch of %s: %s", what, hipGetErrorString(e));
    return KVM_OK;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- device arithmetic -----------------------------------------------------
// decay^d for an integer distance d >= 0, given lg = log2(decay) <= 0 in double.  The
// exponent d * lg is formed in double and split into its nearest integer and a fraction in
// [-0.5, 0.5]: the fraction goes through the fp32 exp2, the integer part is applied as an
// exact scaling, so the relative error stays at the level of one fp32 exp2 (~1e-7) however
// large d is.  Underflows to 0 (through denormals) like the exact value.
__device__ inline float pow_by_distance(double lg, int64_t d) {
    const double e = fmax((double)d * lg, -320.0);
    const double ei = rint(e);
    return ldexpf(exp2f((float)(e - ei)), (int)ei);
}

// ---- shapes ----------------------------------------------------------------
constexpr int kWave = 64;
// Workspace sizes, defined next to the kernels that use them.
size_t score_workspace_bytes(int64_t n_uids, int32_t n_rows, int32_t g, int32_t dim);
size_t select_workspace_bytes(int64_t n_uids);
size_t span_workspace_bytes(int32_t n_rows);

}  // namespace kvm
