// llma_find_trigger_static: the trigger scan (paper: Method, the n-gram match step of Algorithm 1)
// for callers that may not allocate device memory -- code under HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc.  Same kernels as llma_find_trigger; the one buffer the
// scan needs beyond its inputs and outputs (the document index of every reference position) lives
// in a file-scope device array instead of a per-call allocation.
#include <mutex>

#include "../../include/llma.h"
#include "common.h"
#include "kernels.h"

// one int per reference token: 4 MiB per GPU the library runs on, held until the process ends
static __device__ __align__(256) int32_t trigger_scratch[LLMA_TRIGGER_STATIC_MAX_REF];

// The array's name is only a host-side handle for the symbol; its device address differs per GPU
// and is looked up once per device (with that device current) and kept.
#define MAX_DEVICES 64
static std::mutex g_scratch_mu;
static int32_t *g_scratch_ptr[MAX_DEVICES];

static hipError_t scratch_of_current_device(int32_t **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(trigger_scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = (int32_t *)p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

void llma_set_error_text(const char *text);     // llma_api.hip: text for llma_last_error(NULL)

extern "C" int llma_find_trigger_static(const int32_t *y_dev, int32_t y_len, const int32_t *ref_dev, int32_t ref_len,
                                        const int32_t *doc_offsets_dev, int32_t n_docs, int32_t n,
                                        int32_t *result_dev, void *hip_stream) {
    if (!result_dev || y_len < 0 || ref_len < 0 || n_docs < 0 || (!y_dev && y_len > 0) || (!ref_dev && ref_len > 0) ||
        (!doc_offsets_dev && n_docs > 0)) {
        llma_set_error_text("llma_find_trigger_static: null pointer or negative count");
        return LLMA_E_INVAL;
    }
    if (n < 1) {
        llma_set_error_text("llma_find_trigger_static: n must be >= 1");
        return LLMA_E_INVAL;
    }
    if (ref_len > LLMA_TRIGGER_STATIC_MAX_REF) {
        llma_set_error_text("llma_find_trigger_static: reference longer than LLMA_TRIGGER_STATIC_MAX_REF tokens "
                            "(the static scratch array); use llma_find_trigger");
        return LLMA_E_RANGE;
    }
    int32_t *scratch = nullptr;
    hipError_t e = scratch_of_current_device(&scratch);
    if (e != hipSuccess) {
        llma_set_error_text(hipGetErrorString(e));
        return LLMA_E_HIP;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    // scratch[p] = document of reference position p, for p < ref_len (every entry the scan reads is
    // written first, so what an earlier call left behind is never seen); then the scan, which checks
    // the document list itself because the host cannot
    if (ref_len > 0 && n_docs > 0) launch_fill_ref_doc(doc_offsets_dev, n_docs, scratch, ref_len, st);
    launch_trigger_plain(y_dev, y_len, ref_dev, doc_offsets_dev, scratch, ref_len, n_docs, n, result_dev, true, st);
    e = hipGetLastError();
    if (e != hipSuccess) {
        llma_set_error_text(hipGetErrorString(e));
        return LLMA_E_HIP;
    }
    return LLMA_OK;
}
