// Per-stream scratch of a TAS handle (see Workspace in common.h) and the process-wide launch choices that
// tests and tuning runs may force.
#include "common.h"

#include <cstring>

namespace tensile {

Tuning g_tuning;

Workspace::~Workspace() {
    for (void *p : retired) (void)hipFree(p);
}

template <typename T>
int Workspace::provide(DevBuf<T> &b, size_t count, const char *what, bool *fresh) {
    if (fresh) *fresh = false;
    if (fixed_base) {
        // carve count elements out of the region, 256-byte aligned; nothing is kept from call to call
        const size_t bytes = ((count ? count : 1) * sizeof(T) + 255) / 256 * 256;
        if (bytes > fixed_bytes - fixed_used) {
            set_error("%s needs %zu more bytes of scratch than the %zu preallocated", what, bytes - (fixed_bytes - fixed_used),
                      fixed_bytes);
            return TENSILE_E_CAPACITY;
        }
        b.owned = false;
        b.p = reinterpret_cast<T *>(fixed_base + fixed_used);
        b.n = count;
        fixed_used += bytes;
        if (fresh) *fresh = true;
        return TENSILE_OK;
    }
    if (b.p && count <= b.n) return TENSILE_OK;
    size_t want = count ? count : 1;
    if (want < 2 * b.n) want = 2 * b.n;   // at least doubled: what is parked in `retired` stays below what is in use
    T *fresh_p = nullptr;
    const hipError_t e = hipMalloc(reinterpret_cast<void **>(&fresh_p), want * sizeof(T));
    if (e != hipSuccess) return hip_fail(e, what);
    if (b.p) retired.push_back(b.p);
    b.p = fresh_p;
    b.n = want;
    b.owned = true;
    if (fresh) *fresh = true;
    return TENSILE_OK;
}

template int Workspace::provide<int64_t>(DevBuf<int64_t> &, size_t, const char *, bool *);
template int Workspace::provide<int32_t>(DevBuf<int32_t> &, size_t, const char *, bool *);
template int Workspace::provide<unsigned long long>(DevBuf<unsigned long long> &, size_t, const char *, bool *);
template int Workspace::provide<unsigned int>(DevBuf<unsigned int> &, size_t, const char *, bool *);
template int Workspace::provide<int2>(DevBuf<int2> &, size_t, const char *, bool *);

WorkspaceLock acquire_workspace(const tensile_tas *tas, hipStream_t stream) {
    Workspace *ws;
    {
        std::lock_guard<std::mutex> g(tas->ws_mu);
        std::unique_ptr<Workspace> &slot = tas->workspaces[stream];
        if (!slot) {
            slot.reset(new Workspace());
            slot->stream = stream;
        }
        ws = slot.get();
    }
    WorkspaceLock l;
    l.ws = ws;
    l.lock = std::unique_lock<std::mutex>(ws->mu);
    ws->begin_call();
    return l;
}

namespace {
__global__ void fill_words_kernel(uint32_t *dst, size_t n, uint32_t value) {
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t k = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; k < n; k += stride) dst[k] = value;
}
}  // namespace

int fill_words(hipStream_t stream, void *dst, size_t n_words, uint32_t value) {
    if (n_words == 0) return TENSILE_OK;
    const size_t blocks = (n_words + 255) / 256;
    hipLaunchKernelGGL(fill_words_kernel, dim3(static_cast<uint32_t>(blocks < 1024 ? blocks : 1024)), dim3(256), 0, stream,
                       static_cast<uint32_t *>(dst), n_words, value);
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

}  // namespace tensile

using namespace tensile;

extern "C" int tensile_tuning_set(const char *knob, int value) {
    if (!knob) { set_error("tuning_set: knob is NULL"); return TENSILE_E_INVAL; }
    struct { const char *name; int Tuning::*field; } const table[] = {
        {"eval_r", &Tuning::eval_r},           {"eval_binned", &Tuning::eval_binned},
        {"eval_threads", &Tuning::eval_threads}, {"eval_segments", &Tuning::eval_segments},
        {"eval_persistent", &Tuning::eval_persistent}, {"eval_slots", &Tuning::eval_slots}, {"eval_nt", &Tuning::eval_nt},
        {"eval_seg_steps", &Tuning::eval_seg_steps},
        {"score_blocks", &Tuning::score_blocks}, {"link_packed", &Tuning::link_packed},
        {"step_fused", &Tuning::step_fused},
    };
    for (const auto &row : table)
        if (std::strcmp(knob, row.name) == 0) {
            g_tuning.*(row.field) = value;
            return TENSILE_OK;
        }
    set_error("tuning_set: unknown knob '%s'", knob);
    return TENSILE_E_INVAL;
}

extern "C" void tensile_tuning_reset(void) { g_tuning = Tuning(); }
