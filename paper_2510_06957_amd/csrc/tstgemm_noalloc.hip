// tstgemm_noalloc(): the product Y = X W + b for callers that can neither allocate device memory nor hand any in
// besides their operands -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It is
// tstgemm_ex() with the workspace argument pointing at a file-scope device array of this library instead of caller
// memory; the kernels are the same and take the array's address as they take any workspace.
//
// The array exists once per GPU the library is loaded on (each device holds its own copy at its own address, for as
// long as the process lives).  In host code the array's NAME is only a handle for the runtime: the device address of
// the current device's copy comes from hipGetSymbolAddress(), is looked up on the first call on that device and kept;
// everything below that touches the memory uses that address.
#include <mutex>

#include "tstgemm_internal.h"

namespace {

constexpr size_t kScratchBytes = TSTGEMM_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lookup_lock;
void *g_scratch_address[kMaxDevices];   // per device: where that device's copy of `scratch` lives (nullptr: not looked up yet)

// Device address of the current device's copy of the array.
int scratch_address(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return TSTGEMM_EHIP;
    std::lock_guard<std::mutex> guard(g_lookup_lock);
    if (dev < kMaxDevices && g_scratch_address[dev] != nullptr) {
        *out = g_scratch_address[dev];
        return TSTGEMM_OK;
    }
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return TSTGEMM_EHIP;
    if (dev < kMaxDevices) g_scratch_address[dev] = p;
    *out = p;
    return TSTGEMM_OK;
}

}  // namespace

extern "C" int tstgemm_noalloc(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream)
{
    if (!X || !t || !Y || M < 1 || K != t->K || N != t->N) return TSTGEMM_EINVAL;
    size_t need = 0;
    if (int rc = tstgemm_workspace_bytes(M, K, N, &need, nullptr)) return rc;
    if (need > kScratchBytes) return TSTGEMM_ESCRATCH;
    void *ws = nullptr;
    if (int rc = scratch_address(&ws)) return rc;
    // Nothing in the workspace has to start at zero: the packing pre-pass writes every entry of the tiles it lays out
    // (padding included) and every K slice stores its whole partial tile before the reduction reads it.
    tstgemm_opts_t o{};
    o.struct_size = sizeof(o);
    o.workspace = ws;
    o.workspace_bytes = kScratchBytes;
    return tstgemm_ex(X, t, b, Y, M, K, N, &o, stream);
}
