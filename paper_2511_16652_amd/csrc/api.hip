// C ABI of libeggroll: argument validation, scratch management, and the sequencing of kernels for
// each entry point of include/eggroll.h.  No arithmetic of the method happens on the host.
#include <math.h>
#include <stdarg.h>
#include <string.h>

#include <mutex>

#include "common.hpp"

namespace egg {

egg_status fail(eggroll_ctx* c, egg_status s, const char* fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return s;
}

egg_status check_hip(eggroll_ctx* c, hipError_t e, const char* what)
{
    if (e == hipSuccess) return EGG_OK;
    return fail(c, EGG_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Scratch only grows.  A buffer that is too small is replaced by a larger one and parked on the retired list
// instead of being freed: kernels already enqueued, and HIP graphs captured earlier, keep valid addresses.
// Growth is geometric so that a slowly growing sequence of shapes retires O(log) buffers.
egg_status reserve(eggroll_ctx* c, eggroll_ctx::Buf& b, size_t bytes)
{
    if (b.bytes >= bytes) return EGG_OK;
    size_t want = (bytes + 255) & ~size_t(255);
    void* p = nullptr;
    hipError_t e = hipErrorOutOfMemory;
    if (b.p) {
        const size_t geo = (b.bytes + b.bytes / 2 + 255) & ~size_t(255);
        if (geo > want) {
            e = hipMalloc(&p, geo);
            if (e == hipSuccess) want = geo;
            else (void)hipGetLastError();
        }
    }
    if (e != hipSuccess) e = hipMalloc(&p, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(c, EGG_ENOMEM, "scratch of %zu bytes: %s", want, hipGetErrorString(e));
    }
    if (b.p) c->retired.push_back(b);
    b.p = p;
    b.bytes = want;
    ++c->scratch_generation;
    return EGG_OK;
}

egg_status ensure_dynamic_lds(eggroll_ctx* c, const void* kern, size_t bytes, const char* what)
{
    static std::mutex mu;
    static std::map<std::pair<int, const void*>, size_t> limit;  // (device, function) -> bytes already granted
    std::lock_guard<std::mutex> lock(mu);
    size_t& cur = limit[{c->device, kern}];
    if (bytes <= cur) return EGG_OK;
    egg_status st = check_hip(c, hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes), what);
    if (st == EGG_OK) cur = bytes;
    return st;
}

KernelScope::KernelScope(eggroll_ctx* ctx, const char* n) : c(ctx), name(n)
{
    if (!c->prof) return;
    auto get = [&]() {
        hipEvent_t e = nullptr;
        if (!c->free_events.empty()) {
            e = c->free_events.back();
            c->free_events.pop_back();
        } else if (hipEventCreate(&e) != hipSuccess) {
            e = nullptr;
        }
        return e;
    };
    a = get();
    b = get();
    if (a) (void)hipEventRecord(a, c->stream);
}

KernelScope::~KernelScope()
{
    if (!c->prof || !a || !b) return;
    (void)hipEventRecord(b, c->stream);
    c->recs.push_back({name, a, b});
}

// forward_pass: the entry point understands antithetic pairs (the others take pair ids as member ids)
egg_status validate_shape(eggroll_ctx* c, const egg_shape* s, bool need_rows, bool forward_pass)
{
    if (!s) return fail(c, EGG_EINVAL, "shape is NULL");
    if (s->member_count <= 0 || s->d_out <= 0 || s->d_in <= 0) return fail(c, EGG_EINVAL, "non-positive size");
    if (need_rows && s->rows_per_member <= 0) return fail(c, EGG_EINVAL, "rows_per_member must be positive");
    if (s->rank != 1 && s->rank != 2 && s->rank != 4 && s->rank != 8 && s->rank != 16)
        return fail(c, EGG_EINVAL, "rank %d not in {1,2,4,8,16}", s->rank);
    if (s->member_begin < 0 || s->member_begin + s->member_count > (int64_t(1) << 32))
        return fail(c, EGG_EINVAL, "member ids must lie in [0, 2^32)");
    if (s->antithetic != 0 && s->antithetic != 1) return fail(c, EGG_EINVAL, "antithetic must be 0 or 1");
    if (s->antithetic && !forward_pass)
        return fail(c, EGG_EINVAL, "antithetic applies to the forward passes; pass pair ids as member ids here");
    if (s->antithetic && ((s->member_begin | s->member_count) & 1))
        return fail(c, EGG_EINVAL, "antithetic pairs need an even member_begin and member_count");
    return EGG_OK;
}

// projection pre-pass + shared GEMM with the correction epilogue for one validated linear layer
egg_status forward_linear(eggroll_ctx* c, egg_key key, const egg_shape& shape, egg_dtype io_dtype, egg_dtype y_dtype, float sigma,
                          egg_act act, const void* W, const void* X, void* Y, void* A_cache, void* B_cache, const void* resid,
                          float* t_fixed, const float* t_ready, const NextProjection* next)
{
    const bool panel = c->cache_layout == EGG_CACHE_PANEL;
    const int64_t R = shape.member_count * (int64_t)shape.rows_per_member;
    float* t = nullptr;
    if (sigma != 0.0f && t_ready) {
        t = const_cast<float*>(t_ready);  // the producer of X already formed the projections
    } else if (sigma != 0.0f) {
        egg_status s = EGG_OK;
        if (t_fixed) {
            t = t_fixed;  // the caller's (static) projection buffer: nothing is allocated on this path
        } else {
            s = reserve(c, c->t_buf, (size_t)R * shape.rank * sizeof(float));
            if (s != EGG_OK) return s;
            t = (float*)c->t_buf.p;
        }
        s = launch_project(c, make_stream_key(key.seed, key.step, key.layer, 1), shape, io_dtype, X, t, B_cache, panel);
        if (s != EGG_OK) return s;
    }
    return launch_forward_gemm(c, make_stream_key(key.seed, key.step, key.layer, 0), shape, io_dtype, y_dtype, sigma, act, W, X, Y,
                               t, A_cache, resid, next);
}

// validation shared by the forward entry points; t_fixed != NULL: the projections go to that buffer of t_capacity
// values and nothing may be allocated on the way
egg_status checked_forward(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype io_dtype, egg_dtype y_dtype,
                                float sigma, egg_act act, const void* W, const void* X, const void* R_in, bool need_r, void* Y,
                                void* A_cache, void* B_cache, float* t_fixed, size_t t_capacity, const float* t_in, bool want_next,
                                uint32_t next_layer, float* t_next)
{
    if (!c) return EGG_EINVAL;
    egg_status s = validate_shape(c, shape, true, true);
    if (s != EGG_OK) return s;
    if (key.layer >> 31) return fail(c, EGG_EINVAL, "layer must be < 2^31");
    if (!W || !X || !Y || (need_r && !R_in)) return fail(c, EGG_EINVAL, "W, X, Y (and R_in) must be non-NULL");
    if (!aligned16(W) || !aligned16(X) || !aligned16(Y) || !aligned16(A_cache) || !aligned16(B_cache) || !aligned16(R_in))
        return fail(c, EGG_EINVAL, "pointers must be 16-byte aligned");
    if (io_dtype != EGG_BF16 && io_dtype != EGG_F32) return fail(c, EGG_EUNSUPPORTED, "io_dtype %d", (int)io_dtype);
    if (y_dtype != EGG_BF16 && y_dtype != EGG_F32) return fail(c, EGG_EUNSUPPORTED, "y_dtype %d", (int)y_dtype);
    if (io_dtype == EGG_F32 && y_dtype != EGG_F32) return fail(c, EGG_EUNSUPPORTED, "fp32 inputs need fp32 output");
    if (act != EGG_ACT_NONE && act != EGG_ACT_GELU) return fail(c, EGG_EINVAL, "unknown activation");
    const int kq = io_dtype == EGG_BF16 ? 8 : 4;
    if (shape->d_in % kq) return fail(c, EGG_EUNSUPPORTED, "d_in must be a multiple of %d", kq);
    if (shape->d_out % 4) return fail(c, EGG_EUNSUPPORTED, "d_out must be a multiple of 4");
    if (!(sigma == sigma) || sigma < 0.0f) return fail(c, EGG_EINVAL, "sigma must be >= 0");
    if (sigma == 0.0f && (A_cache || B_cache))
        return fail(c, EGG_EINVAL, "sigma == 0 generates no factors: caches must be NULL");
    const bool panel = c->cache_layout == EGG_CACHE_PANEL;
    if (panel && A_cache) return fail(c, EGG_EINVAL, "the panel cache layout keeps B only: A_cache must be NULL");
    const int64_t R = shape->member_count * (int64_t)shape->rows_per_member;
    if (R > (int64_t(1) << 31) - 512) return fail(c, EGG_EUNSUPPORTED, "more than 2^31 rows in one call");
    if (t_fixed) {
        if (c->prof) return fail(c, EGG_EINVAL, "per-kernel timing creates events: switch it off for the no-allocation entry point");
        if ((uint64_t)R * (uint64_t)shape->rank > t_capacity)
            return fail(c, EGG_EUNSUPPORTED, "rows * rank = %lld exceeds the static scratch of %zu values", (long long)R * shape->rank,
                        t_capacity);
        // the one other scratch user of this path: factors materialised for S > 1 or rank > 1 go to the caller's cache
        const bool regen = sigma == 0.0f || (shape->rank == 1 && shape->rows_per_member == 1 && !(shape->antithetic && A_cache));
        if (!regen && !A_cache)
            return fail(c, EGG_EINVAL, "more than one row per member or rank > 1 materialises A_i: pass A_cache (this entry point does not allocate)");
    }
    if (t_in && B_cache) return fail(c, EGG_EINVAL, "given projections skip the pass that would fill B_cache: pass one or the other");
    if (want_next) {
        if (!t_next) return fail(c, EGG_EINVAL, "t_next must be non-NULL");
        if (next_layer >> 31) return fail(c, EGG_EINVAL, "next_layer must be < 2^31");
        if (!forward_fuses_next_projection(*shape, io_dtype, y_dtype, sigma, act, R_in != nullptr))
            return fail(c, EGG_EUNSUPPORTED,
                        "the next layer's projections are formed only by bf16 GELU layers of rank 1, 2 or 4 without residual, sigma > 0, 64 | rows_per_member, "
                        "64 | d_in and at least 192 output tiles of 256 x 256");
    }
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    NextProjection np{nullptr, t_next};
    if (want_next) {
        // the next layer's B factors over this layer's outputs, exactly what eggroll_noise_gen writes for that layer
        const size_t bytes = (size_t)shape->member_count * shape->d_out * shape->rank * 2;
        s = reserve(c, c->next_b, bytes);
        if (s != EGG_OK) return s;
        s = launch_noise(c, make_stream_key(key.seed, key.step, next_layer, 1), (uint32_t)shape->member_begin, shape->member_count,
                         (int64_t)shape->d_out * shape->rank, EGG_BF16, EGG_NORMAL, 0, c->next_b.p);
        if (s != EGG_OK) return s;
        np.B = c->next_b.p;
    }
    return forward_linear(c, key, *shape, io_dtype, y_dtype, sigma, act, W, X, Y, A_cache, B_cache, R_in, t_fixed,
                          sigma != 0.0f ? t_in : nullptr, want_next ? &np : nullptr);
}

// z >= 0 with P(|Z| >= z) = erfc(z / sqrt 2) = alpha, 0 < alpha < 1: Newton's method on g(z) = log erfc(z / sqrt 2) - log alpha,
// which is concave and decreasing, so the iteration from z = 0 increases monotonically to the root
double two_sided_quantile(double alpha)
{
    const double la = log(alpha), rs2 = 0.70710678118654752440, c = 0.79788456080286535588;  // sqrt(2/pi)
    double z = 0.0;
    for (int it = 0; it < 200; ++it) {
        const double q = erfc(z * rs2);
        const double step = (log(q) - la) * q / (c * exp(-0.5 * z * z));  // -g/g', g' = -c exp(-z^2/2) / q
        z += step;
        if (fabs(step) <= 1e-16 * (1.0 + z)) break;
    }
    return z;
}

// The paper's integer noise (App. "Adding EGGROLL Perturbations": int8 values round(16 z), z ~ N(0,1), drawn from a
// pre-generated table that is indexed at random so that no floating point runs on the accelerator).  Table of 2^16
// entries indexed by 16 random bits: entry k is the value at the midpoint of the k-th of 65536 equal-probability cells,
// T[k] = round(16 Phi^-1((k + 1/2) / 65536)), rounded half away from zero and mirrored so that T[65535 - k] = -T[k]
// exactly (zero mean, symmetric: Assumption 1).  The largest magnitude is 69.
void normal_int_table(int8_t* out)
{
    for (int k = 32768; k < 65536; ++k) {
        const double q = (65535.5 - (double)k) / 65536.0;          // upper-tail probability of the cell midpoint
        const long v = lround(16.0 * two_sided_quantile(2.0 * q));  // P(|Z| >= z) = 2 q
        const int8_t t = (int8_t)(v > 127 ? 127 : v);
        out[k] = t;
        out[65535 - k] = (int8_t)-t;
    }
}

}  // namespace egg

using namespace egg;

extern "C" {

egg_status eggroll_create(eggroll_ctx** out, int device, void* hip_stream)
{
    if (!out) return EGG_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return EGG_EHIP;
    if (hipSetDevice(device) != hipSuccess) return EGG_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return EGG_EHIP;
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return EGG_EUNSUPPORTED;  // kernels are gfx950-only
    eggroll_ctx* c = new (std::nothrow) eggroll_ctx();
    if (!c) return EGG_ENOMEM;
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    if (prop.multiProcessorCount > 0) c->compute_units = prop.multiProcessorCount;
    egg_status s = reserve(c, c->zero_page, 256);
    if (s == EGG_OK && hipMemsetAsync(c->zero_page.p, 0, 256, c->stream) != hipSuccess) s = EGG_EHIP;
    if (s != EGG_OK) {
        delete c;
        return s;
    }
    *out = c;
    return EGG_OK;
}

egg_status eggroll_destroy(eggroll_ctx* c)
{
    if (!c) return EGG_EINVAL;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    eggroll_ctx::Buf* bufs[] = {&c->t_buf, &c->a_buf, &c->b_buf, &c->fnorm, &c->pack_a, &c->pack_b, &c->i8_a, &c->i8_b, &c->i8_h, &c->gru, &c->zero_page, &c->lut, &c->norm_tab, &c->model, &c->model_g, &c->proj_part, &c->next_b};
    for (auto* b : bufs)
        if (b->p) (void)hipFree(b->p);
    for (auto& b : c->retired) (void)hipFree(b.p);
    for (auto& r : c->recs) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    for (auto e : c->free_events) (void)hipEventDestroy(e);
    delete c;
    return EGG_OK;
}

const char* eggroll_strerror(egg_status s)
{
    switch (s) {
        case EGG_OK: return "ok";
        case EGG_EINVAL: return "invalid argument";
        case EGG_EUNSUPPORTED: return "unsupported dtype/shape combination or device";
        case EGG_EHIP: return "HIP runtime error";
        case EGG_ENOMEM: return "out of device memory for scratch";
    }
    return "unknown status";
}

const char* eggroll_last_error(const eggroll_ctx* c) { return c ? c->err.c_str() : "no context"; }

uint64_t eggroll_scratch_generation(const eggroll_ctx* c) { return c ? c->scratch_generation : 0; }

egg_status eggroll_trim(eggroll_ctx* c)
{
    if (!c) return EGG_EINVAL;
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c, EGG_EHIP, "sync before trimming scratch");
    for (auto& b : c->retired) (void)hipFree(b.p);
    c->retired.clear();
    return EGG_OK;
}

double eggroll_default_scale(int64_t population, double sigma, int rank)
{
    return 1.0 / ((double)population * sigma * sqrt((double)rank));
}

egg_status eggroll_set_conservative_waits(eggroll_ctx* c, int on)
{
    if (!c) return EGG_EINVAL;
    c->conservative_waits = on != 0;
    return EGG_OK;
}

egg_status eggroll_set_cache_layout(eggroll_ctx* c, egg_cache_layout layout)
{
    if (!c) return EGG_EINVAL;
    if (layout != EGG_CACHE_ROWS && layout != EGG_CACHE_PANEL) return fail(c, EGG_EINVAL, "unknown cache layout %d", (int)layout);
    c->cache_layout = (int)layout;
    return EGG_OK;
}

egg_status eggroll_noise_gen(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype dtype, egg_dist dist,
                             int int_bound, void* A_out, void* B_out)
{
    if (!c) return EGG_EINVAL;
    egg_status s = validate_shape(c, shape, false, false);
    if (s != EGG_OK) return s;
    if (key.layer >> 31) return fail(c, EGG_EINVAL, "layer must be < 2^31");
    const bool ok = (dist == EGG_NORMAL && (dtype == EGG_F32 || dtype == EGG_BF16)) ||
                    ((dist == EGG_UNIFORM_INT || dist == EGG_NORMAL_INT16) && dtype == EGG_I8) || (dist == EGG_RAW && dtype == EGG_U32);
    if (!ok) return fail(c, EGG_EUNSUPPORTED, "noise_gen: dist %d with dtype %d", (int)dist, (int)dtype);
    if (dist == EGG_UNIFORM_INT && !valid_int_bound(int_bound)) return fail(c, EGG_EINVAL, "int_bound outside [0,127]");
    if (dist == EGG_NORMAL_INT16) int_bound = EGG_INT_NOISE_NORMAL16;
    if ((A_out && !aligned16(A_out)) || (B_out && !aligned16(B_out))) return fail(c, EGG_EINVAL, "outputs must be 16-byte aligned");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    if (A_out) {
        s = launch_noise(c, make_stream_key(key.seed, key.step, key.layer, 0), (uint32_t)shape->member_begin,
                         shape->member_count, (int64_t)shape->d_out * shape->rank, dtype, dist, int_bound, A_out);
        if (s != EGG_OK) return s;
    }
    if (B_out) {
        s = launch_noise(c, make_stream_key(key.seed, key.step, key.layer, 1), (uint32_t)shape->member_begin,
                         shape->member_count, (int64_t)shape->d_in * shape->rank, dtype, dist, int_bound, B_out);
        if (s != EGG_OK) return s;
    }
    return EGG_OK;
}

egg_status eggroll_perturbed_forward(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype io_dtype,
                                     egg_dtype y_dtype, float sigma, egg_act act, const void* W, const void* X,
                                     void* Y, void* A_cache, void* B_cache)
{
    return checked_forward(c, key, shape, io_dtype, y_dtype, sigma, act, W, X, nullptr, false, Y, A_cache, B_cache, nullptr, 0);
}

egg_status eggroll_perturbed_forward_add(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype io_dtype,
                                         egg_dtype y_dtype, float sigma, egg_act act, const void* W, const void* X,
                                         const void* R_in, void* Y, void* A_cache, void* B_cache)
{
    return checked_forward(c, key, shape, io_dtype, y_dtype, sigma, act, W, X, R_in, true, Y, A_cache, B_cache, nullptr, 0);
}

egg_status eggroll_perturbed_forward_chained(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype io_dtype,
                                             egg_dtype y_dtype, float sigma, egg_act act, const void* W, const void* X,
                                             const void* R_in, void* Y, const float* t_in, int want_next, uint32_t next_layer,
                                             float* t_next)
{
    return checked_forward(c, key, shape, io_dtype, y_dtype, sigma, act, W, X, R_in, false, Y, nullptr, nullptr, nullptr, 0, t_in,
                           want_next != 0, next_layer, t_next);
}

egg_status eggroll_perturbed_forward_i8(eggroll_ctx* c, egg_key key, const egg_shape* shape, int int_bound,
                                        int corr_shift, int out_shift, int steps, const int8_t* W, const int8_t* H_in,
                                        int8_t* H_out)
{
    if (!c) return EGG_EINVAL;
    egg_status s = validate_shape(c, shape, false, true);
    if (s != EGG_OK) return s;
    if (key.layer >> 31) return fail(c, EGG_EINVAL, "layer must be < 2^31");
    if (!W || !H_in || !H_out) return fail(c, EGG_EINVAL, "W, H_in, H_out must be non-NULL");
    if (!aligned16(W) || !aligned16(H_in) || !aligned16(H_out)) return fail(c, EGG_EINVAL, "pointers must be 16-byte aligned");
    if (shape->rank != 1) return fail(c, EGG_EUNSUPPORTED, "integer path is rank 1");
    if (shape->d_out != shape->d_in && steps > 1) return fail(c, EGG_EUNSUPPORTED, "more than one step needs a square matrix");
    if (shape->d_out != shape->d_in && H_in == H_out) return fail(c, EGG_EINVAL, "H_in and H_out may alias only for a square matrix");
    if (shape->d_in % 16 || shape->d_out % 16) return fail(c, EGG_EUNSUPPORTED, "d_out and d_in must be multiples of 16");
    if (!valid_int_bound(int_bound)) return fail(c, EGG_EINVAL, "int_bound outside [0,127] (and not EGG_INT_NOISE_NORMAL16)");
    if (corr_shift < 0 || corr_shift > 31 || out_shift < 0 || out_shift > 31) return fail(c, EGG_EINVAL, "shift outside [0,31]");
    if (steps < 1) return fail(c, EGG_EINVAL, "steps must be >= 1");
    // int32 accumulators: |acc| <= d*127^2, |dot * A| <= d*127*bound^2
    if ((int64_t)shape->d_in * 127 * 127 + (int64_t)shape->d_in * 127 * noise_max(int_bound) * noise_max(int_bound) > 0x7FFFFFFFLL)
        return fail(c, EGG_EUNSUPPORTED, "d too large for int32 accumulation");
    if (shape->member_count > (int64_t(1) << 31) - 512) return fail(c, EGG_EUNSUPPORTED, "too many rows in one call");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_forward_i8(c, make_stream_key(key.seed, key.step, key.layer, 0),
                             make_stream_key(key.seed, key.step, key.layer, 1), *shape, int_bound, corr_shift,
                             out_shift, steps, W, H_in, H_out);
}

egg_status eggroll_gru_i8(eggroll_ctx* c, egg_key key, const egg_shape* shape, int int_bound, int corr_shift, int out_shift,
                          int steps, const int8_t* Wf, const int8_t* Uf, const int8_t* Wh, const int8_t* Uh, const int8_t* bf,
                          const int8_t* bh, const int8_t* U, const int8_t* S_in, int8_t* S_out)
{
    if (!c) return EGG_EINVAL;
    egg_status s = validate_shape(c, shape, false, true);
    if (s != EGG_OK) return s;
    if (key.layer > 0x7FFFFFFFu - 3u) return fail(c, EGG_EINVAL, "layer + 3 must be < 2^31");
    const void* ptrs[] = {Wf, Uf, Wh, Uh, bf, bh, U, S_in, S_out};
    for (const void* p : ptrs) {
        if (!p) return fail(c, EGG_EINVAL, "NULL pointer argument");
        if (!aligned16(p)) return fail(c, EGG_EINVAL, "pointers must be 16-byte aligned");
    }
    if (shape->rank != 1) return fail(c, EGG_EUNSUPPORTED, "integer path is rank 1");
    if (shape->d_out != shape->d_in) return fail(c, EGG_EUNSUPPORTED, "the cell's matrices are square");
    if (shape->d_in % 16) return fail(c, EGG_EUNSUPPORTED, "D must be a multiple of 16");
    if (!valid_int_bound(int_bound)) return fail(c, EGG_EINVAL, "int_bound outside [0,127] (and not EGG_INT_NOISE_NORMAL16)");
    if (corr_shift < 0 || corr_shift > 31 || out_shift < 0 || out_shift > 31) return fail(c, EGG_EINVAL, "shift outside [0,31]");
    if (steps < 1) return fail(c, EGG_EINVAL, "steps must be >= 1");
    if ((int64_t)shape->d_in * 127 * 127 + (int64_t)shape->d_in * 127 * noise_max(int_bound) * noise_max(int_bound) > 0x7FFFFFFFLL)
        return fail(c, EGG_EUNSUPPORTED, "D too large for int32 accumulation");
    if (shape->member_count > (int64_t(1) << 31) - 512) return fail(c, EGG_EUNSUPPORTED, "too many rows in one call");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    const int8_t* W[4] = {Wf, Uf, Wh, Uh};
    return launch_gru_i8(c, key, *shape, int_bound, corr_shift, out_shift, steps, W, bf, bh, U, S_in, S_out);
}

static bool pow2_in(int v, int lo, int hi) { return v >= lo && v <= hi && (v & (v - 1)) == 0; }

egg_status eggroll_layernorm_i8(eggroll_ctx* c, int64_t rows, int D, const int8_t* ln, const int8_t* U, int8_t* out)
{
    if (!c) return EGG_EINVAL;
    if (rows < 0) return fail(c, EGG_EINVAL, "rows must be >= 0");
    if (!pow2_in(D, 16, 1024)) return fail(c, EGG_EUNSUPPORTED, "D must be a power of two in [16, 1024]");
    if (!ln || !U || !out) return fail(c, EGG_EINVAL, "NULL pointer argument");
    if (!aligned16(ln) || !aligned16(U) || !aligned16(out)) return fail(c, EGG_EINVAL, "pointers must be 16-byte aligned");
    if (rows > (int64_t(1) << 31)) return fail(c, EGG_EUNSUPPORTED, "too many rows in one call");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    // with no residual to add the kernel only reads its y argument
    return launch_layernorm_i8(c, nullptr, const_cast<int8_t*>(U), ln, out, rows, D);
}

static egg_status validate_model_shape(eggroll_ctx* c, egg_key key, const egg_shape* shape, uint32_t noise_layers,
                                       int int_bound, int corr_shift)
{
    egg_status s = validate_shape(c, shape, false, true);
    if (s != EGG_OK) return s;
    if ((uint64_t)key.layer + noise_layers > 0x80000000ull) return fail(c, EGG_EINVAL, "noise layers must stay below 2^31");
    if (shape->rank != 1) return fail(c, EGG_EUNSUPPORTED, "integer path is rank 1");
    if (shape->d_out != shape->d_in) return fail(c, EGG_EINVAL, "d_out and d_in must both be the width D");
    if (!valid_int_bound(int_bound)) return fail(c, EGG_EINVAL, "int_bound outside [0,127] (and not EGG_INT_NOISE_NORMAL16)");
    if (corr_shift < 0 || corr_shift > 31) return fail(c, EGG_EINVAL, "shift outside [0,31]");
    if (shape->member_count > (int64_t(1) << 31) - 512) return fail(c, EGG_EUNSUPPORTED, "too many rows in one call");
    return EGG_OK;
}

egg_status eggroll_embed_i8(eggroll_ctx* c, egg_key key, const egg_shape* shape, int int_bound, int corr_shift,
                            const int8_t* emb, const uint8_t* tokens, int8_t* Y)
{
    if (!c) return EGG_EINVAL;
    egg_status s = validate_model_shape(c, key, shape, 1, int_bound, corr_shift);
    if (s != EGG_OK) return s;
    if (!pow2_in(shape->d_in, 16, 1024)) return fail(c, EGG_EUNSUPPORTED, "D must be a power of two in [16, 1024]");
    if (!emb || !tokens || !Y) return fail(c, EGG_EINVAL, "NULL pointer argument");
    if (!aligned16(emb) || !aligned16(Y)) return fail(c, EGG_EINVAL, "emb and Y must be 16-byte aligned");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_embed_i8(c, key, *shape, int_bound, corr_shift, emb, tokens, Y);
}

egg_status eggroll_egg_forward_i8(eggroll_ctx* c, egg_key key, const egg_shape* shape, int layers, int int_bound,
                                  int corr_shift, int steps, const egg_model_i8* model, const uint8_t* tokens,
                                  const int8_t* S_in, int8_t* S_out, int8_t* logits)
{
    if (!c) return EGG_EINVAL;
    if (layers < 0 || layers > 4096) return fail(c, EGG_EINVAL, "layers outside [0, 4096]");
    egg_status s = validate_model_shape(c, key, shape, 2u + 6u * (uint32_t)layers, int_bound, corr_shift);
    if (s != EGG_OK) return s;
    const int D = shape->d_in;
    if (D != 16 && D != 64 && D != 256 && D != 1024) return fail(c, EGG_EUNSUPPORTED, "D must be 16, 64, 256 or 1024 (a power of 4)");
    if (steps < 1) return fail(c, EGG_EINVAL, "steps must be >= 1");
    if (!model || !tokens || !logits) return fail(c, EGG_EINVAL, "NULL pointer argument");
    const void* always[] = {model->emb, model->ln_out, model->head, logits};
    for (const void* p : always)
        if (!p || !aligned16(p)) return fail(c, EGG_EINVAL, "model and output pointers must be non-NULL and 16-byte aligned");
    if (layers > 0) {
        const void* per_layer[] = {model->ln1, model->gru_w, model->gru_b, model->ln2, model->mlp1, model->mlp2, S_in, S_out};
        for (const void* p : per_layer)
            if (!p || !aligned16(p)) return fail(c, EGG_EINVAL, "model and state pointers must be non-NULL and 16-byte aligned");
        const size_t state_bytes = (size_t)layers * (size_t)shape->member_count * (size_t)D;
        const uintptr_t a = reinterpret_cast<uintptr_t>(S_in), b = reinterpret_cast<uintptr_t>(S_out);
        if (a < b + state_bytes && b < a + state_bytes) return fail(c, EGG_EINVAL, "S_in and S_out must not overlap");
    }
    // int32 accumulators of the widest contraction (4 D terms)
    if ((int64_t)4 * D * 127 * 127 + (int64_t)4 * D * 127 * noise_max(int_bound) * noise_max(int_bound) > 0x7FFFFFFFLL)
        return fail(c, EGG_EUNSUPPORTED, "D too large for int32 accumulation");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_egg_forward_i8(c, key, *shape, layers, int_bound, corr_shift, steps, *model, tokens, S_in, S_out, logits);
}

egg_status eggroll_loglik_i8(eggroll_ctx* c, int64_t rows, const int8_t* logits, const uint8_t* targets, int accumulate,
                             int32_t* out)
{
    if (!c) return EGG_EINVAL;
    if (rows < 0 || rows > (int64_t(1) << 31)) return fail(c, EGG_EINVAL, "rows outside [0, 2^31]");
    if (!logits || !targets || !out) return fail(c, EGG_EINVAL, "NULL pointer argument");
    if (!aligned16(logits) || !aligned16(out)) return fail(c, EGG_EINVAL, "logits and out must be 16-byte aligned");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_loglik_i8(c, rows, logits, targets, accumulate, out);
}

egg_status eggroll_egg_update_i8(eggroll_ctx* c, egg_key key, const egg_shape* shape, int layers, int int_bound,
                                 const int8_t* fitness, int32_t threshold, const egg_model_i8* model)
{
    if (!c) return EGG_EINVAL;
    if (layers < 0 || layers > 4096) return fail(c, EGG_EINVAL, "layers outside [0, 4096]");
    egg_status s = validate_shape(c, shape, false, false);
    if (s != EGG_OK) return s;
    if ((uint64_t)key.layer + 2u + 6u * (uint32_t)layers > 0x80000000ull) return fail(c, EGG_EINVAL, "noise layers must stay below 2^31");
    if (shape->rank != 1) return fail(c, EGG_EUNSUPPORTED, "integer path is rank 1");
    if (shape->d_out != shape->d_in) return fail(c, EGG_EINVAL, "d_out and d_in must both be the width D");
    const int D = shape->d_in;
    if (D % 16) return fail(c, EGG_EUNSUPPORTED, "D must be a multiple of 16");
    if (!valid_int_bound(int_bound)) return fail(c, EGG_EINVAL, "int_bound outside [0,127] (and not EGG_INT_NOISE_NORMAL16)");
    if (threshold < 0) return fail(c, EGG_EINVAL, "threshold must be >= 0");
    if (!fitness || !model || !model->emb || !model->head) return fail(c, EGG_EINVAL, "NULL pointer argument");
    if (layers > 0 && (!model->gru_w || !model->mlp1 || !model->mlp2)) return fail(c, EGG_EINVAL, "NULL pointer argument");
    if (!aligned16(model->emb) || !aligned16(model->head) || !aligned16(model->gru_w) || !aligned16(model->mlp1) || !aligned16(model->mlp2))
        return fail(c, EGG_EINVAL, "model pointers must be 16-byte aligned");
    if (shape->member_count * (int64_t)noise_max(int_bound) * noise_max(int_bound) > 0x7FFFFFFFLL)
        return fail(c, EGG_EUNSUPPORTED, "population too large for int32 accumulation");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    auto one = [&](uint32_t layer, int d_out, int d_in, int8_t* theta) {
        egg_shape sh = *shape;
        sh.d_out = d_out;
        sh.d_in = d_in;
        return launch_update_i8(c, make_stream_key(key.seed, key.step, layer, 0), make_stream_key(key.seed, key.step, layer, 1), sh,
                                int_bound, fitness, threshold, theta, nullptr);
    };
    if ((s = one(key.layer, 256, D, model->emb)) != EGG_OK) return s;
    const size_t DD = (size_t)D * D;
    for (int i = 0; i < layers; ++i) {
        const uint32_t base = key.layer + 1u + 6u * (uint32_t)i;
        for (int m = 0; m < 4; ++m)
            if ((s = one(base + m, D, D, model->gru_w + ((size_t)i * 4 + m) * DD)) != EGG_OK) return s;
        if ((s = one(base + 4, 4 * D, D, model->mlp1 + (size_t)i * 4 * DD)) != EGG_OK) return s;
        if ((s = one(base + 5, D, 4 * D, model->mlp2 + (size_t)i * 4 * DD)) != EGG_OK) return s;
    }
    return one(key.layer + 1u + 6u * (uint32_t)layers, 256, D, model->head);
}

egg_status eggroll_update(eggroll_ctx* c, egg_key key, const egg_shape* shape, egg_dtype noise_dtype,
                          const float* fitness, float scale, int accumulate, float* G, void* W, egg_dtype w_dtype,
                          float lr, const void* A_cache, const void* B_cache)
{
    if (!c) return EGG_EINVAL;
    egg_status s = validate_shape(c, shape, false, false);
    if (s != EGG_OK) return s;
    if (key.layer >> 31) return fail(c, EGG_EINVAL, "layer must be < 2^31");
    if (!fitness || !G) return fail(c, EGG_EINVAL, "fitness and G must be non-NULL");
    if (!aligned16(G) || !aligned16(W) || !aligned16(A_cache) || !aligned16(B_cache) || (reinterpret_cast<uintptr_t>(fitness) & 3))
        return fail(c, EGG_EINVAL, "misaligned pointer");
    if (noise_dtype != EGG_BF16 && noise_dtype != EGG_F32) return fail(c, EGG_EUNSUPPORTED, "noise_dtype %d", (int)noise_dtype);
    if (W && w_dtype != EGG_BF16 && w_dtype != EGG_F32) return fail(c, EGG_EUNSUPPORTED, "w_dtype %d", (int)w_dtype);
    if (shape->d_out % 4) return fail(c, EGG_EUNSUPPORTED, "d_out must be a multiple of 4");
    const bool b_panel = c->cache_layout == EGG_CACHE_PANEL && B_cache != nullptr;
    if (b_panel) {
        if (A_cache) return fail(c, EGG_EINVAL, "the panel cache layout keeps B only: A_cache must be NULL");
        if (noise_dtype != EGG_BF16 || shape->rank != 1 || shape->d_out % 2 || shape->d_in % 2)
            return fail(c, EGG_EUNSUPPORTED, "the panel cache layout needs bf16 factors, rank 1 and even dimensions");
    } else if ((A_cache == nullptr) != (B_cache == nullptr)) {
        return fail(c, EGG_EINVAL, "pass both caches or neither");
    }
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_update(c, make_stream_key(key.seed, key.step, key.layer, 0),
                         make_stream_key(key.seed, key.step, key.layer, 1), *shape, noise_dtype, fitness, scale,
                         accumulate, G, W, w_dtype, lr, A_cache, B_cache, b_panel);
}

egg_status eggroll_update_i8(eggroll_ctx* c, egg_key key, const egg_shape* shape, int int_bound, const int8_t* fitness,
                             int32_t threshold, int8_t* theta, int32_t* E_out)
{
    if (!c) return EGG_EINVAL;
    egg_status s = validate_shape(c, shape, false, false);
    if (s != EGG_OK) return s;
    if (key.layer >> 31) return fail(c, EGG_EINVAL, "layer must be < 2^31");
    if (!fitness || !theta) return fail(c, EGG_EINVAL, "fitness and theta must be non-NULL");
    if (!aligned16(theta) || !aligned16(E_out)) return fail(c, EGG_EINVAL, "theta and E_out must be 16-byte aligned");
    if (shape->rank != 1) return fail(c, EGG_EUNSUPPORTED, "integer path is rank 1");
    if (shape->d_out % 16 || shape->d_in % 16) return fail(c, EGG_EUNSUPPORTED, "d_out and d_in must be multiples of 16");
    if (!valid_int_bound(int_bound)) return fail(c, EGG_EINVAL, "int_bound outside [0,127] (and not EGG_INT_NOISE_NORMAL16)");
    if (threshold < 0) return fail(c, EGG_EINVAL, "threshold must be >= 0");
    // int32 E: |E| <= N * bound^2
    if (shape->member_count * (int64_t)noise_max(int_bound) * noise_max(int_bound) > 0x7FFFFFFFLL)
        return fail(c, EGG_EUNSUPPORTED, "population too large for int32 accumulation");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, EGG_EHIP, "hipSetDevice");
    return launch_update_i8(c, make_stream_key(key.seed, key.step, key.layer, 0),
                            make_stream_key(key.seed, key.step, key.layer, 1), *shape, int_bound, fitness, threshold,
                            theta, E_out);
}

void eggroll_normal_int_table(int8_t* out)
{
    if (out) egg::normal_int_table(out);
}

int64_t eggroll_int_threshold(double alpha, int64_t n_terms, double noise_std)
{
    if (!(alpha > 0.0)) return INT64_MAX;
    if (alpha >= 1.0 || n_terms <= 0 || !(noise_std > 0.0)) return 0;
    const double z = two_sided_quantile(alpha);
    const int64_t first = (int64_t)(noise_std * z);  // truncation
    const int64_t second = (int64_t)llround(noise_std * sqrt((double)n_terms));
    return first * second;
}

egg_status eggroll_profile_enable(eggroll_ctx* c, int on)
{
    if (!c) return EGG_EINVAL;
    c->prof = on != 0;
    return EGG_OK;
}

int eggroll_profile_read(eggroll_ctx* c, const char** names, int64_t* launches, double* total_ms, int cap)
{
    if (!c || cap < 0) return EGG_EINVAL;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c, EGG_EHIP, "profile sync");
    std::vector<const char*> order;
    std::map<std::string, std::pair<int64_t, double>> acc;
    for (auto& r : c->recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            auto it = acc.find(r.name);
            if (it == acc.end()) {
                order.push_back(r.name);
                acc[r.name] = {1, (double)ms};
            } else {
                it->second.first += 1;
                it->second.second += ms;
            }
        }
        c->free_events.push_back(r.a);
        c->free_events.push_back(r.b);
    }
    c->recs.clear();
    int n = 0;
    for (const char* nm : order) {
        if (n < cap) {
            if (names) names[n] = nm;
            if (launches) launches[n] = acc[nm].first;
            if (total_ms) total_ms[n] = acc[nm].second;
        }
        ++n;
    }
    return n;
}

}  // extern "C"
