// gpga_consensus_error_static: the consensus distance ||X - 1 xbar^T||_F (Sec. 4; App. B) for
// callers that cannot allocate device memory (code under HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc).  It runs the kernels of gpga_consensus_error /
// gpga_set_trace, with their per-workgroup partial sums in a file-scope device array
// instead of scratch owned by the context, writes the result to a caller-owned device
// double and never synchronises, allocates or frees.
//
// The array exists once per GPU the library runs on and is held until the process ends.
// Its name is only a host-side stand-in: the address a kernel may use comes from
// hipGetSymbolAddress, looked up once per device (with that device current) and kept.
// Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams,
// two threads) race on the partials.  Nothing in it has to start at zero - each call
// writes every partial it later reads - so no clearing is needed between calls.
#include <cstdio>
#include <mutex>

#include "gpga_internal.hpp"

namespace {

// 1 MiB: one double per 256-lane workgroup of the reduction pass, i.e. d up to
// 131072 x 1024 = 1.34e8 columns on the 128-bit path (3.3e7 on the scalar path).
constexpr size_t kStaticScratchDoubles = 131072;

// No `used` attribute here: the compiler gives a static device variable that host code
// refers to a global symbol in the code object, which is how the runtime finds it by name;
// with the attribute it stays a local symbol and the lookup cannot succeed.
static __device__ __align__(256) double scratch[kStaticScratchDoubles];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
double* g_scratch_ptr[kMaxDevices] = {nullptr};

}  // namespace

size_t static_scratch_doubles() { return kStaticScratchDoubles; }

hipError_t static_scratch_for_device(int device, double** ptr_out) {
    *ptr_out = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[device]) {
        int prev = -1;
        hipError_t e = hipGetDevice(&prev);
        if (e != hipSuccess) return e;
        if (prev != device) {
            e = hipSetDevice(device);
            if (e != hipSuccess) return e;
        }
        double* p = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
        if (prev != device) (void)hipSetDevice(prev);
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *ptr_out = g_scratch_ptr[device];
    return hipSuccess;
}

extern "C" gpga_status gpga_consensus_error_static(gpga_ctx* c, double* out_dev) {
    if (!c) return GPGA_EINVAL;
    auto fail = [&](gpga_status s, const char* msg) {
        snprintf(c->err, sizeof(c->err), "%s", msg);
        return s;
    };
    if (!out_dev || (reinterpret_cast<uintptr_t>(out_dev) & 7u)) return fail(GPGA_EINVAL, "out_dev must be an 8-byte aligned device pointer");
    if (!c->bound) return fail(GPGA_ESTATE, "buffers are not bound (gpga_bind)");
    const size_t need = consensus_partials_used(c);
    if (need > kStaticScratchDoubles) {
        snprintf(c->err, sizeof(c->err),
                 "d = %lld needs %zu partial sums, the static scratch holds %zu (d <= %zu on 16-byte aligned rows, "
                 "%zu otherwise): use gpga_consensus_error",
                 (long long)c->d, need, kStaticScratchDoubles, (kStaticScratchDoubles - 1) * 1024, kStaticScratchDoubles * 256);
        return GPGA_EINVAL;
    }
    double* ptr = nullptr;
    hipError_t e = static_scratch_for_device(c->device, &ptr);
    if (e != hipSuccess) {
        snprintf(c->err, sizeof(c->err), "static scratch address: %s", hipGetErrorString(e));
        return GPGA_EDEVICE;
    }
    int prev = -1;
    const bool switched = hipGetDevice(&prev) == hipSuccess && prev != c->device && hipSetDevice(c->device) == hipSuccess;
    e = launch_consensus_distance(c, ptr, kStaticScratchDoubles, out_dev);
    if (switched) (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        snprintf(c->err, sizeof(c->err), "consensus kernel launch: %s", hipGetErrorString(e));
        return GPGA_EDEVICE;
    }
    return GPGA_OK;
}
