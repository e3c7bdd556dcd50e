// Optimizer wrapper and loss-scale policy kernels (paper Sections 3.1 item 1, 3.2, 3.3).
//
// Both kernels of mp_unscale_check_update are pure streaming kernels bound by HBM:
//   inspect : reads 2 B/parameter  (fp16 gradient bit test, one ballot per wave)
//   update  : Adam reads g16 + w32 + m + v (14 B) and writes w32 + m + v + w16 (14 B) = 28 B/param,
//             SGD reads 6 B and writes 6 B = 12 B/param,
// with 16-byte accesses per lane, consecutive lanes on consecutive addresses.
#include "common.hpp"

#include <mutex>
#include <string.h>
#include <vector>

namespace mp {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
int hip_fail(hipError_t e, const char* what) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return MP_E_HIP;
}

// ------------------------------------------------------------------ scale state
__global__ void scale_state_init_kernel(mp_scale_state* st, int mode, float s, int interval, float smin,
                                        float smax) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < MP_HISTORY) {
        st->hist_scale[i]     = 0.f;
        st->hist_found_inf[i] = 0;
    }
    if (i == 0) {
        st->scale = s;
        st->inv_scale = 1.0f / s;
        st->min_scale = smin;
        st->max_scale = smax;
        st->mode = mode;
        st->growth_interval = interval;
        st->good_steps = 0;
        st->found_inf = 0;
        st->opt_step = 0;
        st->total_steps = 0;
        st->skipped_steps = 0;
        st->reserved = 0;
    }
}

__global__ void loss_scale_update_kernel(mp_scale_state* st) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const int   found = st->found_inf != 0;
    float       s     = st->scale;
    const int   slot  = st->total_steps % MP_HISTORY;
    st->hist_scale[slot]     = s;
    st->hist_found_inf[slot] = found;
    st->total_steps += 1;
    if (found) {
        st->skipped_steps += 1;
        st->good_steps = 0;
        if (st->mode == MP_SCALE_BACKOFF) s = fmaxf(s * 0.5f, st->min_scale);
    } else {
        st->opt_step += 1;
        int good = st->good_steps + 1;
        if (st->mode == MP_SCALE_BACKOFF && good >= st->growth_interval) {
            s = fminf(s * 2.0f, st->max_scale);
            good = 0;
        }
        st->good_steps = good;
    }
    st->scale     = s;
    st->inv_scale = 1.0f / s;
    st->found_inf = 0;
}

// ------------------------------------------------------------------ multi-tensor update
constexpr int UPD_THREADS     = 256;
constexpr int UPD_VEC         = 4;                                  // elements per lane per access
constexpr int UPD_ITERS       = 8;
constexpr int UPD_CHUNK       = UPD_THREADS * UPD_VEC * UPD_ITERS;  // 8192 elements per workgroup
constexpr int INS_VEC         = 8;                                  // the inspection pass reads fp16 only: 16 B per lane
constexpr int INS_ITERS       = UPD_CHUNK / (UPD_THREADS * INS_VEC);
constexpr int UPD_MAX_TENSORS = 32;                                 // descriptors per launch

struct UpdBatch {
    const uint16_t*    g16[UPD_MAX_TENSORS];
    float*             w32[UPD_MAX_TENSORS];
    uint16_t*          w16[UPD_MAX_TENSORS];
    float*             m[UPD_MAX_TENSORS];
    float*             v[UPD_MAX_TENSORS];
    unsigned long long n[UPD_MAX_TENSORS];
    int                chunk_start[UPD_MAX_TENSORS + 1];  // first workgroup of each tensor
    unsigned           vec_ok;                            // bit i: tensor i's pointers are 16-byte aligned
    int                ntensors;
};

struct UpdScalars {
    float  lr, beta1, beta2, eps, wd, omb1, omb2;
    double beta1d, beta2d;
    int    kind;
};

__device__ __forceinline__ int find_tensor(const UpdBatch& b, int bid) {
    int t = 0;
    while (t + 1 < b.ntensors && bid >= b.chunk_start[t + 1]) ++t;
    return t;
}

__global__ __launch_bounds__(UPD_THREADS) void inspect_kernel(UpdBatch b, mp_scale_state* st) {
    const int                 t   = find_tensor(b, blockIdx.x);
    const unsigned long long  n   = b.n[t];
    const unsigned long long  off = (unsigned long long)(blockIdx.x - b.chunk_start[t]) * UPD_CHUNK;
    const uint16_t*           g   = b.g16[t];
    const bool                vec = (b.vec_ok >> t) & 1u;
    bool                      bad = false;
#pragma unroll
    for (int it = 0; it < INS_ITERS; ++it) {
        const unsigned long long i = off + (unsigned long long)(it * UPD_THREADS + threadIdx.x) * INS_VEC;
        if (vec && i + INS_VEC <= n) {
            const uint4 q = *reinterpret_cast<const uint4*>(g + i);
            // both halves of each 32-bit word: exponent field 0x7C00 all ones
            const unsigned w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                bad |= ((w[k] & 0x7C00u) == 0x7C00u) | ((w[k] & 0x7C000000u) == 0x7C000000u);
            }
        } else {
            for (unsigned long long j = i; j < n && j < i + INS_VEC; ++j) bad |= half_nonfinite(g[j]);
        }
    }
    if (__any(bad)) {
        if ((threadIdx.x & 63) == 0) atomicOr(&st->found_inf, 1);
    }
}

// (1 - beta^t) in double by repeated squaring, rounded to fp32.
__device__ __forceinline__ float bias_correction(double beta, int t) {
    double r = 1.0, p = beta;
    for (int e = t; e > 0; e >>= 1) {
        if (e & 1) r *= p;
        p *= p;
    }
    return (float)(1.0 - r);
}

template <int KIND>
__device__ __forceinline__ void update_one(float g16v, float& w, float& m, float& v, const UpdScalars& s,
                                           float inv_scale, float bc1, float bc2) {
    float g = g16v * inv_scale;
    if (s.wd != 0.f) g = g + s.wd * w;
    if (KIND == MP_OPT_SGD) {
        w = w - s.lr * g;
    } else {
        m = s.beta1 * m + s.omb1 * g;
        v = s.beta2 * v + s.omb2 * (g * g);
        const float mhat = m / bc1;
        const float vhat = v / bc2;
        w = w - s.lr * mhat / (sqrtf(vhat) + s.eps);
    }
}

typedef float    f32x4v __attribute__((ext_vector_type(4)));
typedef unsigned u32x2v __attribute__((ext_vector_type(2)));

template <int KIND>
__global__ __launch_bounds__(UPD_THREADS) void update_kernel(UpdBatch b, UpdScalars s, const mp_scale_state* st) {
    if (st->found_inf != 0) return;  // overflow somewhere in this iteration: the whole step is skipped
    const float inv_scale = st->inv_scale;
    float       bc1 = 1.f, bc2 = 1.f;
    if (KIND == MP_OPT_ADAM) {
        const int t = st->opt_step + 1;
        bc1 = bias_correction(s.beta1d, t);
        bc2 = bias_correction(s.beta2d, t);
    }
    const int                t   = find_tensor(b, blockIdx.x);
    const unsigned long long n   = b.n[t];
    const unsigned long long off = (unsigned long long)(blockIdx.x - b.chunk_start[t]) * UPD_CHUNK;
    const uint16_t* __restrict__ g16 = b.g16[t];
    float* __restrict__          w32 = b.w32[t];
    uint16_t* __restrict__       w16 = b.w16[t];
    float* __restrict__          mm  = b.m[t];
    float* __restrict__          vv  = b.v[t];
    const bool                   vec = (b.vec_ok >> t) & 1u;

    // every access instruction of a wave covers one contiguous run (64 lanes x 16 B of fp32, 64 x 8 B of fp16),
    // so each 128-byte line is touched by exactly one load and one store per array
#pragma unroll
    for (int it = 0; it < UPD_ITERS; ++it) {
        const unsigned long long i = off + (unsigned long long)(it * UPD_THREADS + threadIdx.x) * UPD_VEC;
        if (vec && i + UPD_VEC <= n) {
            // streaming data, touched once per step: non-temporal accesses keep it from displacing cache contents
            const u32x2v gq = __builtin_nontemporal_load(reinterpret_cast<const u32x2v*>(g16 + i));
            f32x4v       w0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4v*>(w32 + i));
            f32x4v       m0 = {0.f, 0.f, 0.f, 0.f}, v0 = m0;
            if (KIND == MP_OPT_ADAM) {
                m0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4v*>(mm + i));
                v0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4v*>(vv + i));
            }
            const float gh[4] = {h2f((uint16_t)(gq.x & 0xFFFFu)), h2f((uint16_t)(gq.x >> 16)),
                                 h2f((uint16_t)(gq.y & 0xFFFFu)), h2f((uint16_t)(gq.y >> 16))};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float w = w0[k], m = m0[k], v = v0[k];
                update_one<KIND>(gh[k], w, m, v, s, inv_scale, bc1, bc2);
                w0[k] = w;
                m0[k] = m;
                v0[k] = v;
            }
            __builtin_nontemporal_store(w0, reinterpret_cast<f32x4v*>(w32 + i));
            if (KIND == MP_OPT_ADAM) {
                __builtin_nontemporal_store(m0, reinterpret_cast<f32x4v*>(mm + i));
                __builtin_nontemporal_store(v0, reinterpret_cast<f32x4v*>(vv + i));
            }
            u32x2v hq;
            hq.x = (unsigned)f2h(w0.x) | ((unsigned)f2h(w0.y) << 16);
            hq.y = (unsigned)f2h(w0.z) | ((unsigned)f2h(w0.w) << 16);
            *reinterpret_cast<u32x2v*>(w16 + i) = hq;  // read again by the next forward pass: ordinary store
        } else {
            for (unsigned long long j = i; j < n && j < i + UPD_VEC; ++j) {
                float w = w32[j], m1 = 0.f, v1 = 0.f;
                if (KIND == MP_OPT_ADAM) {
                    m1 = mm[j];
                    v1 = vv[j];
                }
                update_one<KIND>(h2f(g16[j]), w, m1, v1, s, inv_scale, bc1, bc2);
                w32[j] = w;
                if (KIND == MP_OPT_ADAM) {
                    mm[j] = m1;
                    vv[j] = v1;
                }
                w16[j] = f2h(w);
            }
        }
    }
}

}  // namespace mp

using namespace mp;

extern "C" const char* mp_last_error(void) { return g_err; }
extern "C" int         mp_version(void) { return 1; }

extern "C" int mp_scale_state_init(mp_scale_state* st, int mode, float init_scale, int growth_interval,
                                   float min_scale, float max_scale, mp_stream stream) {
    MP_REQUIRE(st != nullptr, "mp_scale_state_init: st is NULL");
    MP_REQUIRE(mode == MP_SCALE_STATIC || mode == MP_SCALE_BACKOFF, "mp_scale_state_init: bad mode %d", mode);
    MP_REQUIRE(growth_interval >= 1, "mp_scale_state_init: growth_interval %d < 1", growth_interval);
    MP_REQUIRE(init_scale > 0.f && min_scale > 0.f && min_scale <= init_scale && init_scale <= max_scale,
               "mp_scale_state_init: need 0 < min_scale <= init_scale <= max_scale (got %g %g %g)",
               (double)min_scale, (double)init_scale, (double)max_scale);
    hipLaunchKernelGGL(scale_state_init_kernel, dim3((MP_HISTORY + 255) / 256), dim3(256), 0, as_stream(stream),
                       st, mode, init_scale, growth_interval, min_scale, max_scale);
    MP_LAUNCH_CHECK("mp_scale_state_init");
    return MP_OK;
}

extern "C" int mp_loss_scale_update(mp_scale_state* st, mp_stream stream) {
    MP_REQUIRE(st != nullptr, "mp_loss_scale_update: st is NULL");
    hipLaunchKernelGGL(loss_scale_update_kernel, dim3(1), dim3(64), 0, as_stream(stream), st);
    MP_LAUNCH_CHECK("mp_loss_scale_update");
    return MP_OK;
}

extern "C" int mp_unscale_check_update(const mp_tensor_desc* tensors, int ntensors, const mp_opt_cfg* cfg,
                                       mp_scale_state* st, int flags, mp_stream stream) {
    MP_REQUIRE(st != nullptr && cfg != nullptr, "mp_unscale_check_update: st / cfg is NULL");
    MP_REQUIRE(ntensors >= 0 && (ntensors == 0 || tensors != nullptr), "mp_unscale_check_update: bad tensor list");
    MP_REQUIRE(cfg->kind == MP_OPT_SGD || cfg->kind == MP_OPT_ADAM, "mp_unscale_check_update: bad optimizer kind %d",
               cfg->kind);
    MP_REQUIRE((flags & ~MP_UPDATE_PRECHECKED) == 0, "mp_unscale_check_update: unknown flags 0x%x", flags);
    for (int i = 0; i < ntensors; ++i) {
        const mp_tensor_desc& d = tensors[i];
        if (d.n == 0) continue;
        MP_REQUIRE(d.g16 && d.w32 && d.w16, "mp_unscale_check_update: tensor %d has a NULL g16/w32/w16", i);
        MP_REQUIRE(cfg->kind != MP_OPT_ADAM || (d.m && d.v), "mp_unscale_check_update: tensor %d lacks Adam moments", i);
        MP_REQUIRE((reinterpret_cast<uintptr_t>(d.g16) & 1) == 0 && (reinterpret_cast<uintptr_t>(d.w16) & 1) == 0 &&
                       (reinterpret_cast<uintptr_t>(d.w32) & 3) == 0,
                   "mp_unscale_check_update: tensor %d is not element-aligned", i);
        MP_REQUIRE(d.n < (1ull << 40), "mp_unscale_check_update: tensor %d too large", i);
    }

    UpdScalars s;
    s.kind   = cfg->kind;
    s.lr     = (float)cfg->lr;
    s.beta1  = (float)cfg->beta1;
    s.beta2  = (float)cfg->beta2;
    s.eps    = (float)cfg->eps;
    s.wd     = (float)cfg->weight_decay;
    s.omb1   = (float)(1.0 - cfg->beta1);
    s.omb2   = (float)(1.0 - cfg->beta2);
    s.beta1d = cfg->beta1;
    s.beta2d = cfg->beta2;

    std::vector<UpdBatch> batches;
    UpdBatch              cur;
    cur = UpdBatch{};
    long long chunks = 0;
    auto      flush  = [&]() {
        if (cur.ntensors > 0) {
            cur.chunk_start[cur.ntensors] = (int)chunks;
            batches.push_back(cur);
        }
        cur = UpdBatch{};
        chunks = 0;
    };
    for (int i = 0; i < ntensors; ++i) {
        const mp_tensor_desc& d = tensors[i];
        if (d.n == 0) continue;
        const long long c = (long long)((d.n + UPD_CHUNK - 1) / UPD_CHUNK);
        if (cur.ntensors == UPD_MAX_TENSORS || chunks + c > 0x3FFFFFFF) flush();
        const int k = cur.ntensors++;
        cur.g16[k]  = d.g16;
        cur.w32[k]  = d.w32;
        cur.w16[k]  = d.w16;
        cur.m[k]    = d.m;
        cur.v[k]    = d.v;
        cur.n[k]    = d.n;
        cur.chunk_start[k] = (int)chunks;
        const bool ok = aligned16(d.g16) && aligned16(d.w32) && aligned16(d.w16) &&
                        (cfg->kind != MP_OPT_ADAM || (aligned16(d.m) && aligned16(d.v)));
        if (ok) cur.vec_ok |= (1u << k);
        chunks += c;
    }
    flush();

    hipStream_t hs = as_stream(stream);
    if (!(flags & MP_UPDATE_PRECHECKED)) {
        for (const UpdBatch& b : batches) {
            hipLaunchKernelGGL(inspect_kernel, dim3(b.chunk_start[b.ntensors]), dim3(UPD_THREADS), 0, hs, b, st);
            MP_LAUNCH_CHECK("mp_unscale_check_update(inspect)");
        }
    }
    for (const UpdBatch& b : batches) {
        if (cfg->kind == MP_OPT_ADAM)
            hipLaunchKernelGGL(update_kernel<MP_OPT_ADAM>, dim3(b.chunk_start[b.ntensors]), dim3(UPD_THREADS), 0, hs, b,
                               s, st);
        else
            hipLaunchKernelGGL(update_kernel<MP_OPT_SGD>, dim3(b.chunk_start[b.ntensors]), dim3(UPD_THREADS), 0, hs, b,
                               s, st);
        MP_LAUNCH_CHECK("mp_unscale_check_update(update)");
    }
    return MP_OK;
}
