// ee_static.hip -- ee_exit_head_static: the exit head for callers that cannot allocate device
// memory and bring no workspace (code under HIP graph capture, tight serving loops, harnesses
// that forbid hipMalloc).  Same kernels as ee_exit_head; what that call keeps in the batch's
// workspace (the normalised operand rows and the per-tile softmax statistics, for fp32 models
// also the logits) lives here in a device array of the library's own, one copy per GPU.
#include "ee_internal.h"

#include <mutex>

static __device__ __align__(256) unsigned char scratch[EE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void*      g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once
std::mutex g_scratch_mutex;

// In host code the array's name is only a handle for the runtime; its address on the current
// device comes from hipGetSymbolAddress and differs from GPU to GPU.
int scratch_on_current_device(char** out) {
    int dev = -1;
    EE_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ee_fail(EE_ERR_HIP, "ee_exit_head_static: device ordinal out of range");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        EE_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return ee_fail(EE_ERR_HIP, "ee_exit_head_static: no device address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<char*>(g_scratch_ptr[dev]);
    return EE_OK;
}
}  // namespace

extern "C" int ee_exit_head_static(const ee_model* m, int exit_idx, float threshold, int force_exit, ee_batch* b,
                                   void* stream) {
    if (!m || !b || b->m != m) return ee_fail(EE_ERR_INVALID_ARG, "ee_exit_head_static: batch not bound to this model");
    if (exit_idx < 0 || exit_idx >= m->cfg.n_exits)
        return ee_fail(EE_ERR_INVALID_ARG, "ee_exit_head_static: exit index out of range");
    if (!m->exits[exit_idx].set) return ee_fail(EE_ERR_EXIT_NOT_RESIDENT, "ee_exit_head_static: exit head not set");
    if (threshold != threshold) return ee_fail(EE_ERR_INVALID_ARG, "ee_exit_head_static: threshold is NaN");
    const ee_model_config& c = m->cfg;
    const bool bf16 = c.dtype == EE_BF16;
    // the part of the workspace an exit head touches, laid out in the array
    ee_batch t = *b;
    t.W = WsLayout{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    const size_t Mpad = (size_t)b->Mpad;
    const size_t n_part = bf16 ? (size_t)c.vocab / 32 : 1;
    t.W.x = take(Mpad * c.d_model * (bf16 ? 2 : 4));
    t.W.part_max = take(Mpad * n_part * 4);
    t.W.part_sum = take(Mpad * n_part * 4);
    t.W.part_arg = take(Mpad * n_part * 4);
    t.W.logits = take(bf16 ? 0 : Mpad * (size_t)c.vocab * 4);
    t.W.total = o;
    if (o > EE_STATIC_SCRATCH_BYTES)
        return ee_fail(EE_ERR_CAPACITY, "ee_exit_head_static: " + std::to_string(o) + " bytes of scratch needed for this batch "
                                        "and model, the library's array holds " + std::to_string(EE_STATIC_SCRATCH_BYTES) +
                                        " (use ee_exit_head with a workspace)");
    char* base = nullptr;
    int rc = scratch_on_current_device(&base);
    if (rc != EE_OK) return rc;
    t.ws = base;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    return bf16 ? bf16_exit_head(m, exit_idx, threshold, force_exit ? 1 : 0, &t, nullptr, s)
                : f32_exit_head(m, exit_idx, threshold, force_exit ? 1 : 0, &t, nullptr, s);
}
