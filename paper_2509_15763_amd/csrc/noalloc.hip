// unigist_decode_noalloc: unigist_decode for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  The split-K partial results, which
// unigist_decode keeps in a caller-supplied workspace, go to a fixed array in the library's device image instead.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process ends.  In
// host code the array's name is only a stand-in for the symbol: the device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what the kernels receive, exactly as they receive the caller's workspace
// in unigist_decode.
#include <mutex>

#include "common.h"

using namespace unigist;

namespace {

constexpr size_t kScratchBytes = UNIGIST_DECODE_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device ordinal, null until looked up

// address of the current device's copy of the array (null on failure)
void* scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" size_t unigist_decode_noalloc_scratch_bytes(void) { return kScratchBytes; }

extern "C" unigist_status unigist_decode_noalloc(const void* q, const void* kcache, const void* vcache, void* out,
                                                 float* lse, int B, int Hq, int Hkv, int Lk_max, const int* seqlens,
                                                 int D, unigist_dtype dt, void* hip_stream) {
    if (B < 1 || Hq < 1 || Hkv < 1 || Lk_max < 1 || D < 1) return UNIGIST_EINVAL;
    if (Hq % Hkv != 0) return UNIGIST_EINVAL;
    if (dt != UNIGIST_BF16 && dt != UNIGIST_F32) return UNIGIST_EUNSUPPORTED;
    if (B > 65535 || Hq > 65535) return UNIGIST_EUNSUPPORTED;
    if (!q || !kcache || !vcache || !out) return UNIGIST_EINVAL;
    const size_t need = unigist_decode_workspace(B, Hq, Hkv, Lk_max, D, dt);
    if (need == 0) return UNIGIST_EUNSUPPORTED;   // head dim the decode kernels are not built for
    if (need > kScratchBytes) return UNIGIST_ESCRATCH;
    void* ws = scratch_of_current_device();
    if (!ws) return UNIGIST_ELAUNCH;
    // The split kernel writes the (m, l, acc) slot of every (sequence, head, slice) -- also of an empty slice --
    // before the combine kernel reads it, so nothing of the previous call's contents has to be cleared.
    hipError_t e = launch_decode(q, kcache, vcache, out, lse, B, Hq, Hkv, Lk_max, seqlens, D, dt, (float*)ws,
                                 (hipStream_t)hip_stream);
    return e == hipSuccess ? UNIGIST_OK : UNIGIST_ELAUNCH;
}
