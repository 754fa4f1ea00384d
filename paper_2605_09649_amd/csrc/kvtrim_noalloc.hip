// kvtrim_select_global_noalloc: stage 2 for callers that cannot allocate device memory.
//
// The tables that kvtrim_select_global keeps in the context's workspace (chunk descriptors, radix
// histograms, per-sequence selection state, the device error flag) live here in one file-scope
// device array of fixed size, so the call needs no context and makes no allocation of any kind.  The
// array's name is only a host-side handle: its device address is looked up once per device with
// hipGetSymbolAddress (every GPU has its own copy at its own address) and that pointer is what the
// kernels get, exactly as they get the workspace pointers in kvtrim_select_global.
#include <string.h>

#include <mutex>

#include "kvtrim_internal.h"

static_assert(KVTRIM_NOALLOC_SCRATCH_BYTES % 256 == 0, "scratch size must keep the 256-byte alignment of its parts");

static __device__ __align__(256) unsigned char scratch[KVTRIM_NOALLOC_SCRATCH_BYTES];

namespace kvtrim {

constexpr int MAX_DEVICES = 64;
static unsigned char* g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each GPU, NULL until looked up
static std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch` (the device must be current); NULL and *err set on failure.
static unsigned char* scratch_on_current_device(hipError_t* err) {
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= MAX_DEVICES) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !p) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    return g_scratch_ptr[dev];
}

// Start of a call: the flag of the previous call on this GPU must not leak into this one.
__global__ void k_noalloc_begin(int32_t* err) { *err = 0; }

// End of a call: the flag becomes the caller's status word and is cleared.
__global__ void k_noalloc_end(int32_t* err, int32_t* status_out) {
    const int32_t e = *err;
    *err = 0;
    if (status_out) *status_out = (e & ERR_LAYOUT) ? KVTRIM_ELAYOUT : (e & ERR_CAP) ? KVTRIM_ECAP : (e & ERR_MISMATCH) ? KVTRIM_EMISMATCH : KVTRIM_OK;
}

}  // namespace kvtrim

using namespace kvtrim;

extern "C" kvtrim_status kvtrim_select_global_noalloc(const kvtrim_config* cfg, const kvtrim_cache* c, const float* score,
                                                      const int64_t* budget, uint8_t* keep_out, int32_t* kept_out,
                                                      uint32_t* thr_key_out, int32_t* status_out, void* hip_stream) {
    if (!config_valid(cfg) || !c) return KVTRIM_EINVAL;
    if (!c->log_beta || !c->pos || !c->seg_start || !c->seg_len) return KVTRIM_EINVAL;
    if (c->cap_entries < 1 || c->cap_entries > cfg->max_entries) return KVTRIM_EINVAL;
    if (!score || !budget || !keep_out || !kept_out) return KVTRIM_EINVAL;
    if (select_workspace(cfg, nullptr, nullptr) > (size_t)KVTRIM_NOALLOC_SCRATCH_BYTES) return KVTRIM_EINVAL;   // beyond the fixed array
    hipError_t herr = hipSuccess;
    unsigned char* base = scratch_on_current_device(&herr);
    if (!base) return KVTRIM_EHIP;

    kvtrim_ctx tmp;                                               // host-side stand-in for a context: shape + table pointers
    memset(&tmp, 0, sizeof(tmp));
    tmp.cfg = *cfg;
    shape_of(cfg, tmp.shape);
    select_workspace(cfg, reinterpret_cast<char*>(base), &tmp.ws);
    hipStream_t st = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(k_noalloc_begin, dim3(1), dim3(1), 0, st, tmp.ws.err);
    CacheView v;
    v.k = (const uint16_t*)c->k;
    v.v = (const uint16_t*)c->v;
    v.log_beta = c->log_beta;
    v.pos = c->pos;
    v.seg_start = c->seg_start;
    v.seg_len = c->seg_len;
    v.cap = c->cap_entries;
    v.log_tail = c->log_tail;
    const kvtrim_status rc = launch_select(&tmp, v, score, budget, keep_out, kept_out, thr_key_out, st);
    hipLaunchKernelGGL(k_noalloc_end, dim3(1), dim3(1), 0, st, tmp.ws.err, status_out);
    if (rc != KVTRIM_OK) return rc;
    return hipGetLastError() == hipSuccess ? KVTRIM_OK : KVTRIM_EHIP;
}
