// ctc_gate for callers that cannot allocate: no context, no workspace, no host staging.
//
// ctc_gate keeps the per-frame entropies and greedy labels in the caller's workspace and uploads the
// frame prefix sums through a pinned staging buffer it allocates on first use.  The variant here keeps
// the per-frame values in a file-scope device array of fixed size and takes the prefix sums as a device
// array, so that the call consists of kernel launches only: nothing is allocated, copied or waited for.
// It runs the same kernels as ctc_gate (Sec. 2.1: Eq. 2, collapse map, Eq. 3).
#include <mutex>

#include <stdarg.h>
#include <stdio.h>

#include "ssd_internal.h"

namespace {

// Per-frame scratch: entropies (fp32) in the first half, greedy labels (int32) in the second.  Every
// GPU the library runs on holds its own copy of this array until the process ends.
constexpr size_t SCRATCH_BYTES = (size_t)SSD_NOALLOC_MAX_FRAMES * 8;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

// Device address of `scratch` per GPU, looked up once per device with that device current.  In host
// code the array's name is only a handle for the symbol; kernels and copies get the looked-up address.
constexpr int MAX_DEVICES = 64;
void* scratch_addr[MAX_DEVICES] = {};
std::mutex scratch_mutex;

int report(char* err, size_t err_len, int code, const char* fmt, ...) {
    if (err && err_len) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(err, err_len, fmt, ap);
        va_end(ap);
    }
    return code;
}

hipError_t scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_addr[dev] = p;
    }
    *out = scratch_addr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int ctc_gate_noalloc(void* hip_stream, const void* logits, int dtype, const int32_t* cu_frames_dev, int B,
                                int64_t n_frames, int V_ctc, int blank_id, float tau_ctc, float* max_entropy,
                                uint8_t* gate_pass, int32_t* draft_ctc, int32_t* draft_len, char* err, size_t err_len) {
    if (err && err_len) err[0] = 0;
    if (!logits || !cu_frames_dev || !max_entropy || !gate_pass || !draft_ctc || !draft_len)
        return report(err, err_len, SSD_EINVAL, "ctc_gate_noalloc: NULL argument");
    if (B <= 0) return report(err, err_len, SSD_EINVAL, "ctc_gate_noalloc: B must be positive (got %d)", B);
    if (n_frames <= 0) return report(err, err_len, SSD_EINVAL, "ctc_gate_noalloc: n_frames must be positive (got %lld)", (long long)n_frames);
    if (V_ctc <= 0) return report(err, err_len, SSD_EINVAL, "ctc_gate_noalloc: V_ctc must be positive (got %d)", V_ctc);
    if (blank_id < 0 || blank_id >= V_ctc)
        return report(err, err_len, SSD_EINVAL, "ctc_gate_noalloc: blank_id %d outside [0, %d)", blank_id, V_ctc);
    if (dtype != SSD_F32 && dtype != SSD_BF16) return report(err, err_len, SSD_EUNSUPPORTED, "ctc_gate_noalloc: dtype %d", dtype);
    if (n_frames > SSD_NOALLOC_MAX_FRAMES)
        return report(err, err_len, SSD_ESHAPE, "ctc_gate_noalloc: %lld frames, the built-in scratch holds at most %d (use ctc_gate with a workspace)",
                      (long long)n_frames, SSD_NOALLOC_MAX_FRAMES);
    void* base = nullptr;
    hipError_t e = scratch_of_current_device(&base);
    if (e != hipSuccess) return report(err, err_len, SSD_EHIP, "ctc_gate_noalloc: scratch address: %s", hipGetErrorString(e));
    float* H = static_cast<float*>(base);
    int32_t* arg = reinterpret_cast<int32_t*>(static_cast<unsigned char*>(base) + (size_t)SSD_NOALLOC_MAX_FRAMES * 4);
    // Both scratch halves are written for every frame below n_frames before they are read (the second
    // kernel reads frames inside [0, n_frames) only), so nothing has to be cleared between calls.
    ssd::launch_gate(logits, dtype, n_frames, V_ctc, cu_frames_dev, B, blank_id, tau_ctc, H, arg, max_entropy, gate_pass,
                     draft_ctc, draft_len, static_cast<hipStream_t>(hip_stream));
    e = hipGetLastError();
    if (e != hipSuccess) return report(err, err_len, SSD_EHIP, "ctc_gate_noalloc: launch: %s", hipGetErrorString(e));
    return SSD_OK;
}
