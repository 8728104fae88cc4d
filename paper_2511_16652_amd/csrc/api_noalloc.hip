// eggroll_perturbed_forward_noalloc: the population forward of one linear layer for callers that cannot
// allocate device memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// Its only scratch, the projections t[R][r], lives in a file-scope device array of fixed size instead of the
// context's growable buffer.  One copy of the array exists per GPU; every call on that GPU, from any context,
// shares it and it keeps the last call's contents (the projection pass overwrites every entry a call reads).
#include "common.hpp"

using namespace egg;

static constexpr size_t STATIC_T_FLOATS = size_t(1) << 20;  // 4 MiB per GPU, held until the process ends
static __device__ __align__(256) float scratch[STATIC_T_FLOATS];

// In host code the array's name is only a stand-in: its device address is looked up once per device, with that
// device current, and only that pointer is ever handed to kernels.
static constexpr int MAX_DEVICES = 64;
static float* scratch_ptr[MAX_DEVICES] = {};

static egg_status static_scratch(eggroll_ctx* c, float** out)
{
    if (c->device < 0 || c->device >= MAX_DEVICES) return fail(c, EGG_EUNSUPPORTED, "device ordinal %d has no static scratch slot", c->device);
    if (!scratch_ptr[c->device]) {
        if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
        float* p = nullptr;
        const hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(c, EGG_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        }
        scratch_ptr[c->device] = p;
    }
    *out = scratch_ptr[c->device];
    return EGG_OK;
}

extern "C" egg_status eggroll_perturbed_forward_noalloc(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype io_dtype,
                                                        egg_dtype y_dtype, float sigma, egg_act act, const void* W,
                                                        const void* X, void* Y, void* A_cache, void* B_cache)
{
    if (!c) return EGG_EINVAL;
    float* t = nullptr;
    egg_status s = static_scratch(c, &t);
    if (s != EGG_OK) return s;
    return checked_forward(c, key, shape, io_dtype, y_dtype, sigma, act, W, X, nullptr, false, Y, A_cache, B_cache, t, STATIC_T_FLOATS);
}
