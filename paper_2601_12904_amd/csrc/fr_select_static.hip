// fr_select_topk_static: the selection half of Query-Guided Selection for callers that cannot allocate device memory
// (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  Same kernels as fr_select_topk; the
// scratch of the multi-workgroup selection (state, histograms, the tiles' status words, candidate list) lives in a
// file-scope device array instead of a context's workspace.  Every GPU the library runs on holds its own copy of the
// array, at its own address, until the process ends; the address is resolved once per device and kept.
#include <mutex>

#include "fr_internal.hpp"

namespace {

constexpr int64_t STATIC_MAX_N = FR_SELECT_STATIC_MAX_SCORES;
constexpr size_t SCRATCH_WORDS = fr::select_workspace_words(STATIC_MAX_N);
static_assert(SCRATCH_WORDS * sizeof(uint32_t) <= (size_t)5 << 20, "the static scratch stays modest");

// In host code this name is only a handle for hipGetSymbolAddress; device addresses come from there.
static __device__ __align__(256) uint32_t scratch[SCRATCH_WORDS];

constexpr int MAX_DEVICES = 64;
std::mutex g_mutex;
uint32_t* g_scratch_ptr[MAX_DEVICES] = {};   // per device: address of its copy of `scratch`

// The current device's copy of the scratch array.
hipError_t scratch_of_current_device(uint32_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<uint32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

fr_status fail(fr_ctx* ctx, fr_status st, const char* msg) {
    if (ctx) ctx->err = msg;
    return st;
}

}  // namespace

namespace fr {
hipError_t select_static_prepare() {
    uint32_t* p = nullptr;
    return scratch_of_current_device(&p);
}
}  // namespace fr

extern "C" fr_status fr_select_topk_static(fr_ctx* ctx, const float* scores, int64_t n, int64_t k, int32_t nq,
                                           int32_t* q_index_out, void* stream) {
    if (ctx) ctx->err.clear();
    if (n < 0 || nq < 0 || k < 0 || k > n) return fail(ctx, FR_ERR_INVALID_ARG, "n, nq or k negative, or k > n");
    if (n > STATIC_MAX_N)
        return fail(ctx, FR_ERR_WORKSPACE, "n exceeds FR_SELECT_STATIC_MAX_SCORES: the static scratch serves at most that many "
                                           "scores (fr_select_topk has no such limit)");
    if (k + (int64_t)nq == 0) return FR_OK;
    if (!q_index_out || (reinterpret_cast<uintptr_t>(q_index_out) & 3u))
        return fail(ctx, FR_ERR_INVALID_ARG, "q_index_out is NULL or not 4-byte aligned");
    if (k > 0 && (!scores || (reinterpret_cast<uintptr_t>(scores) & 3u)))
        return fail(ctx, FR_ERR_INVALID_ARG, "scores is NULL or not 4-byte aligned");
    uint32_t* tmp = nullptr;
    hipError_t e = scratch_of_current_device(&tmp);
    if (e != hipSuccess) return fail(ctx, FR_ERR_DEVICE, hipGetErrorString(e));
    // what must start at zero (state, histograms, status words) is zero when the library is loaded, and every call
    // clears it again before it ends
    e = fr::launch_select(scores, n, k, nq, q_index_out, tmp, SCRATCH_WORDS * sizeof(uint32_t), (hipStream_t)stream);
    if (e != hipSuccess) return fail(ctx, FR_ERR_DEVICE, hipGetErrorString(e));
    return FR_OK;
}
