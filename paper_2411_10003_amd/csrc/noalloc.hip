// moe_expert_counts_static: the input distribution for callers that cannot allocate device memory or pass a
// workspace (code under graph capture, serving loops, harnesses that forbid hipMalloc).  The kernels are
// those of moe_expert_counts; the per-chunk histograms they pass between them live in an array built into
// the library's device image instead of the caller's workspace.
#include "internal.h"

// [chunk][expert] histograms of one call.  One copy per GPU the library is loaded on, at that GPU's own
// address, held until the process ends.
constexpr size_t SCRATCH_WORDS = (size_t)1 << 20;          // 4 MiB
static __device__ __align__(256) int32_t scratch[SCRATCH_WORDS];

namespace {

// The array's name is a host-side stand-in in host code; its device address is looked up once per device.
constexpr int MAX_DEVICES = 64;
std::atomic<int32_t*> g_scratch_ptr[MAX_DEVICES];

hipError_t scratch_for_current_device(int32_t** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    int32_t* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void* sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (sym == nullptr) return hipErrorInvalidSymbol;
        p = static_cast<int32_t*>(sym);
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // racing threads store the same address
    }
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" int moe_expert_counts_static(moe_handle_t h, const int32_t* idx, int32_t* counts, void* stream)
{
    if (!h || !idx || !counts) return MOE_ERR_NULL;
    if ((size_t)h->n_chunks * (size_t)h->s.E > SCRATCH_WORDS) return MOE_ERR_TOO_LARGE;
    int32_t* hist = nullptr;
    hipError_t e = scratch_for_current_device(&hist);
    hipStream_t st = (hipStream_t)stream;
    // every word counts_from_hist reads ([chunk < n_chunks][e < E]) is written by chunk_hist first
    if (e == hipSuccess) e = launch_chunk_hist(h->s, idx, hist, h->n_chunks, st);
    if (e == hipSuccess) e = launch_counts_from_hist(h->s, hist, h->n_chunks, counts, st);
    return moe_hip_status(e);
}
