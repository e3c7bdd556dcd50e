// Loss kernels: fp32 loss value and loss-scaled fp16 seed gradient (paper Section 3.1 item 1).
// Both are streaming kernels bound by HBM: every fp16 input is read once and the fp16 seed
// gradient written once; reductions are two-stage and deterministic (no float atomics).
#include "common.hpp"

namespace mp {

constexpr int LOSS_THREADS = 256;

// Sum `n` fp32 partials with one workgroup (fixed order), divide by `denom`, store to *out.
__global__ __launch_bounds__(LOSS_THREADS) void finish_mean_kernel(const float* __restrict__ part, int n, double denom,
                                                                   float* __restrict__ out) {
    __shared__ float red[LOSS_THREADS / 64];
    float            acc = 0.f;
    for (int i = threadIdx.x; i < n; i += LOSS_THREADS) acc += part[i];
    const float tot = block_sum<LOSS_THREADS / 64>(acc, red);
    if (threadIdx.x == 0) *out = tot / (float)denom;
}

// ------------------------------------------------------------------------------- MSE
template <bool VEC>
__global__ __launch_bounds__(LOSS_THREADS) void mse_kernel(int rows, int cols, int ld, const uint16_t* __restrict__ y,
                                                           const uint16_t* __restrict__ tg,
                                                           const mp_scale_state* __restrict__ st,
                                                           uint16_t* __restrict__ dy, float* __restrict__ part) {
    __shared__ float red[LOSS_THREADS / 64];
    const double     numel = (double)rows * (double)cols;
    const float      coef  = (float)(2.0 * (double)st->scale / numel);
    float            acc   = 0.f;
    if (VEC) {
        const int       vpr   = cols >> 3;  // vectors per row
        const long long nvec  = (long long)rows * vpr;
        for (long long v = (long long)blockIdx.x * LOSS_THREADS + threadIdx.x; v < nvec;
             v += (long long)gridDim.x * LOSS_THREADS) {
            const long long r   = v / vpr;
            const long long off = r * ld + (v - r * vpr) * 8;
            const uint4     a   = *reinterpret_cast<const uint4*>(y + off);
            const uint4     b   = *reinterpret_cast<const uint4*>(tg + off);
            const unsigned  aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
            unsigned        ow[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float d0 = h2f((uint16_t)(aw[k] & 0xFFFF)) - h2f((uint16_t)(bw[k] & 0xFFFF));
                const float d1 = h2f((uint16_t)(aw[k] >> 16)) - h2f((uint16_t)(bw[k] >> 16));
                acc += d0 * d0;
                acc += d1 * d1;
                ow[k] = (unsigned)f2h(coef * d0) | ((unsigned)f2h(coef * d1) << 16);
            }
            *reinterpret_cast<uint4*>(dy + off) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        }
    } else {
        const long long n = (long long)rows * cols;
        for (long long e = (long long)blockIdx.x * LOSS_THREADS + threadIdx.x; e < n;
             e += (long long)gridDim.x * LOSS_THREADS) {
            const long long r   = e / cols;
            const long long off = r * ld + (e - r * cols);
            const float     d   = h2f(y[off]) - h2f(tg[off]);
            acc += d * d;
            dy[off] = f2h(coef * d);
        }
    }
    const float tot = block_sum<LOSS_THREADS / 64>(acc, red);
    if (threadIdx.x == 0) part[blockIdx.x] = tot;
}

// ------------------------------------------------------------------------------- softmax cross-entropy
// One workgroup per row.  Cached variant (vocab a multiple of 8, at most 32 x THREADS): every lane keeps its 32
// logits in registers as fp32, overwrites them with exp(z - max) once and scales them on the way out, so HBM sees
// one read and one write of the row and each exponential is computed once.  THREADS is picked from the row length
// (256, 512 or 1024).  The generic variant re-reads the row (it then comes from L2).
constexpr int XENT_VECS = 4;  // 16-byte vectors per lane

template <int NW, bool MAX>
__device__ __forceinline__ float block_reduce_lds(float v, float* red) {
    v = MAX ? wave_max(v) : wave_sum(v);
    lds_barrier();  // everyone is done reading the previous result
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    lds_barrier();
    float t = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) t = MAX ? fmaxf(t, red[i]) : t + red[i];
    return t;
}

// Workgroups are persistent over rows (row = blockIdx.x, + gridDim.x, ...): the packed logits of the next row are
// requested before the current row is reduced, so the two reductions and the exponentials of a row run under the
// next row's memory latency.
// COLSUM: every workgroup also sums the gradient values it stores (the fp16 values, as stored) per column over its
// rows, and leaves the sums in colpart[blockIdx.x][vocab]: the bias gradient of the projection that made the logits
// then needs no second pass over the gradient matrix, only a sum over gridDim.x partial rows.
template <int THREADS, bool COLSUM = false>
__global__ __launch_bounds__(THREADS) void xent_cached_kernel(int vocab, int ld, const uint16_t* logits,
                                                              const int32_t* __restrict__ targets,
                                                              const mp_scale_state* __restrict__ st, int rows,
                                                              uint16_t* dlogits,  // may alias logits
                                                              float* __restrict__ row_loss,
                                                              float* __restrict__ colpart = nullptr) {
    __shared__ float red[THREADS / 64];
    const int        nvec  = vocab >> 3;
    const float      coef0 = (float)((double)st->scale / (double)rows);
    // a row's packed logits, its target and the target's logit; vectors beyond the row read as -inf
    auto fetch = [&](int row, uint4* q, int& tgt, float& zt) {
        const uint16_t* z = logits + (long long)row * ld;
        tgt               = targets[row];
        zt                = (tgt >= 0 && tgt < vocab) ? h2f(z[tgt]) : 0.f;
#pragma unroll
        for (int i = 0; i < XENT_VECS; ++i) {
            const int v = i * THREADS + threadIdx.x;
            q[i]        = make_uint4(0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u, 0xFC00FC00u);
            if (v < nvec) q[i] = *reinterpret_cast<const uint4*>(z + (long long)v * 8);
        }
    };
    uint4 raw[XENT_VECS];
    int   tgt = -1;
    float zt  = 0.f;
    int   row = blockIdx.x;
    float cs[COLSUM ? XENT_VECS : 1][8];
    if (COLSUM) {
#pragma unroll
        for (int i = 0; i < XENT_VECS; ++i)
#pragma unroll
            for (int k = 0; k < 8; ++k) cs[i][k] = 0.f;
    }
    if (row < rows) fetch(row, raw, tgt, zt);
    for (; row < rows; row += gridDim.x) {
        // (the next row is another row of the same matrix: it is read before anything is written to it, also when
        // dlogits aliases logits, because a row is only ever written by the workgroup that read it, afterwards)
        uint4 nraw[XENT_VECS];
        int   ntgt = -1;
        float nzt  = 0.f;
        if (row + (int)gridDim.x < rows) fetch(row + gridDim.x, nraw, ntgt, nzt);
        uint16_t*   dz    = dlogits + (long long)row * ld;
        const bool  valid = tgt >= 0 && tgt < vocab;
        const float coef  = valid ? coef0 : 0.f;  // invalid target: zero gradient row
        float       e[XENT_VECS][8];
        float       mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < XENT_VECS; ++i) {
            const unsigned w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                e[i][2 * k]     = h2f((uint16_t)(w[k] & 0xFFFF));
                e[i][2 * k + 1] = h2f((uint16_t)(w[k] >> 16));
                mx              = fmaxf(mx, fmaxf(e[i][2 * k], e[i][2 * k + 1]));
            }
        }
        mx = block_reduce_lds<THREADS / 64, true>(mx, red);
        float se = 0.f;
#pragma unroll
        for (int i = 0; i < XENT_VECS; ++i)
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                e[i][k] = __expf(e[i][k] - mx);  // exp(-inf) = 0 beyond the row
                se += e[i][k];
            }
        se = block_reduce_lds<THREADS / 64, false>(se, red);
        const float inv = 1.0f / se;
        if (threadIdx.x == 0) row_loss[row] = valid ? (mx + __logf(se)) - zt : 0.f;
        const int vt = valid ? (tgt >> 3) : -1;  // the vector that holds the target class
#pragma unroll
        for (int i = 0; i < XENT_VECS; ++i) {
            const int v = i * THREADS + threadIdx.x;
            if (v < nvec) {
                float p[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) p[k] = e[i][k] * inv;
                if (v == vt) {
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        if (k == (tgt & 7)) p[k] -= 1.0f;
                }
                unsigned o[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) o[k] = (unsigned)f2h(coef * p[2 * k]) | ((unsigned)f2h(coef * p[2 * k + 1]) << 16);
                *reinterpret_cast<uint4*>(dz + (long long)v * 8) = make_uint4(o[0], o[1], o[2], o[3]);
                if (COLSUM) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        cs[i][2 * k] += h2f((uint16_t)(o[k] & 0xFFFFu));
                        cs[i][2 * k + 1] += h2f((uint16_t)(o[k] >> 16));
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < XENT_VECS; ++i) raw[i] = nraw[i];
        tgt = ntgt;
        zt  = nzt;
    }
    if (COLSUM) {
        float* out = colpart + (long long)blockIdx.x * vocab;
#pragma unroll
        for (int i = 0; i < XENT_VECS; ++i) {
            const int v = i * THREADS + threadIdx.x;
            if (v < nvec) {
                *reinterpret_cast<float4*>(out + (long long)v * 8)     = make_float4(cs[i][0], cs[i][1], cs[i][2], cs[i][3]);
                *reinterpret_cast<float4*>(out + (long long)v * 8 + 4) = make_float4(cs[i][4], cs[i][5], cs[i][6], cs[i][7]);
            }
        }
    }
}

__global__ __launch_bounds__(LOSS_THREADS) void xent_kernel(int vocab, int ld, const uint16_t* logits,
                                                            const int32_t* __restrict__ targets,
                                                            const mp_scale_state* __restrict__ st, int rows,
                                                            uint16_t* dlogits,  // may alias logits
                                                            float* __restrict__ row_loss) {
    __shared__ float red[LOSS_THREADS / 64];
    const int        row  = blockIdx.x;
    const uint16_t*  z    = logits + (long long)row * ld;
    uint16_t*        dz   = dlogits + (long long)row * ld;
    const int        tgt  = targets[row];
    const bool       valid = tgt >= 0 && tgt < vocab;
    const float      coef = (float)((double)st->scale / (double)rows);
    // read before the first barrier; every write to dlogits (which may alias logits) comes after it
    const float      zt   = valid ? h2f(z[tgt]) : 0.f;
    float mx = -INFINITY;
    for (int e = threadIdx.x; e < vocab; e += LOSS_THREADS) mx = fmaxf(mx, h2f(z[e]));
    mx = block_max<LOSS_THREADS / 64>(mx, red);
    float se = 0.f;
    for (int e = threadIdx.x; e < vocab; e += LOSS_THREADS) se += __expf(h2f(z[e]) - mx);
    se = block_sum<LOSS_THREADS / 64>(se, red);
    const float inv = 1.0f / se;
    if (threadIdx.x == 0) row_loss[row] = valid ? (mx + __logf(se)) - zt : 0.f;
    for (int e = threadIdx.x; e < vocab; e += LOSS_THREADS) {
        float p = __expf(h2f(z[e]) - mx) * inv;
        if (e == tgt) p -= 1.0f;
        if (!valid) p = 0.f;
        dz[e] = f2h(coef * p);
    }
}

}  // namespace mp

using namespace mp;

static int loss_blocks(long long units) {
    long long b = (units + LOSS_THREADS * 4 - 1) / (LOSS_THREADS * 4);
    if (b < 1) b = 1;
    if (b > 2048) b = 2048;
    return (int)b;
}

extern "C" size_t mp_loss_workspace_bytes(int rows, int cols) {
    (void)cols;
    const size_t a = 2048 * sizeof(float);
    const size_t b = (size_t)(rows > 0 ? rows : 0) * sizeof(float);
    return a > b ? a : b;
}

extern "C" int mp_mse_scaled(int rows, int cols, const mp_half* y, const mp_half* target, int ld,
                             const mp_scale_state* st, float* loss, mp_half* dy, void* ws, size_t ws_bytes,
                             mp_stream stream) {
    MP_REQUIRE(rows > 0 && cols > 0 && ld >= cols, "mp_mse_scaled: bad shape rows=%d cols=%d ld=%d", rows, cols, ld);
    MP_REQUIRE(y && target && st && loss && dy, "mp_mse_scaled: NULL argument");
    if (!ws || ws_bytes < mp_loss_workspace_bytes(rows, cols)) {
        set_error("mp_mse_scaled: workspace of %zu bytes needed, %zu given", mp_loss_workspace_bytes(rows, cols), ws_bytes);
        return MP_E_WORKSPACE;
    }
    const bool vec = (cols % 8 == 0) && (ld % 8 == 0) && aligned16(y) && aligned16(target) && aligned16(dy);
    const int  nb  = loss_blocks(vec ? (long long)rows * cols / 8 : (long long)rows * cols);
    float*     part = static_cast<float*>(ws);
    hipStream_t hs = as_stream(stream);
    if (vec)
        hipLaunchKernelGGL(mse_kernel<true>, dim3(nb), dim3(LOSS_THREADS), 0, hs, rows, cols, ld, y, target, st, dy, part);
    else
        hipLaunchKernelGGL(mse_kernel<false>, dim3(nb), dim3(LOSS_THREADS), 0, hs, rows, cols, ld, y, target, st, dy, part);
    MP_LAUNCH_CHECK("mp_mse_scaled");
    hipLaunchKernelGGL(finish_mean_kernel, dim3(1), dim3(LOSS_THREADS), 0, hs, part, nb, (double)rows * (double)cols, loss);
    MP_LAUNCH_CHECK("mp_mse_scaled(finish)");
    return MP_OK;
}

// Rows per workgroup: with 1024 lanes per row only one workgroup fits a CU (the kernel's registers allow 5 waves per
// SIMD), and the workgroups are persistent so that the next row's loads overlap the current row's reductions (298 ->
// 247 us at 8192 x 32768).  Shorter rows have several workgroups per CU to overlap with and run one row each.
static int xent_grid(int rows, int threads) {
    if (threads < 1024) return rows;
    return rows < 256 ? rows : 256;
}

extern "C" int mp_softmax_xent_scaled(int rows, int vocab, const mp_half* logits, int ld, const int32_t* targets,
                                      const mp_scale_state* st, float* loss, mp_half* dlogits, void* ws,
                                      size_t ws_bytes, mp_stream stream) {
    MP_REQUIRE(rows > 0 && vocab > 0 && ld >= vocab, "mp_softmax_xent_scaled: bad shape rows=%d vocab=%d ld=%d", rows,
               vocab, ld);
    MP_REQUIRE(logits && targets && st && loss && dlogits, "mp_softmax_xent_scaled: NULL argument");
    if (!ws || ws_bytes < mp_loss_workspace_bytes(rows, vocab)) {
        set_error("mp_softmax_xent_scaled: workspace of %zu bytes needed, %zu given", mp_loss_workspace_bytes(rows, vocab),
                  ws_bytes);
        return MP_E_WORKSPACE;
    }
    float*      row_loss = static_cast<float*>(ws);
    hipStream_t hs       = as_stream(stream);
    const bool cache = (vocab % 8 == 0) && (ld % 8 == 0) && aligned16(logits) && aligned16(dlogits) &&
                       (vocab / 8 <= XENT_VECS * 1024);
    const int  nvec  = vocab / 8;
    if (cache && nvec <= XENT_VECS * 256)
        hipLaunchKernelGGL(xent_cached_kernel<256>, dim3(xent_grid(rows, 256)), dim3(256), 0, hs, vocab, ld, logits, targets, st, rows, dlogits,
                           row_loss);
    else if (cache && nvec <= XENT_VECS * 512)
        hipLaunchKernelGGL(xent_cached_kernel<512>, dim3(xent_grid(rows, 512)), dim3(512), 0, hs, vocab, ld, logits, targets, st, rows, dlogits,
                           row_loss);
    else if (cache)
        hipLaunchKernelGGL(xent_cached_kernel<1024>, dim3(xent_grid(rows, 1024)), dim3(1024), 0, hs, vocab, ld, logits, targets, st, rows, dlogits,
                           row_loss);
    else
        hipLaunchKernelGGL(xent_kernel, dim3(rows), dim3(LOSS_THREADS), 0, hs, vocab, ld, logits, targets, st, rows, dlogits,
                           row_loss);
    MP_LAUNCH_CHECK("mp_softmax_xent_scaled");
    hipLaunchKernelGGL(finish_mean_kernel, dim3(1), dim3(LOSS_THREADS), 0, hs, row_loss, rows, (double)rows, loss);
    MP_LAUNCH_CHECK("mp_softmax_xent_scaled(finish)");
    return MP_OK;
}

// ---- cross-entropy that also leaves the bias gradient of the projection behind the logits
static size_t round256(size_t n) { return (n + 255) / 256 * 256; }
// the fused path: rows cached in a 1024-lane workgroup, workgroups persistent over rows
static bool xent_db_fused(int rows, int vocab, int ld, const void* logits, const void* dlogits) {
    return (vocab % 8 == 0) && (ld % 8 == 0) && aligned16(logits) && aligned16(dlogits) && vocab / 8 <= XENT_VECS * 1024 &&
           vocab / 8 > XENT_VECS * 512 && rows >= 1;
}

extern "C" size_t mp_softmax_xent_db_workspace_bytes(int rows, int vocab) {
    if (rows <= 0 || vocab <= 0) return 0;
    const size_t fused = (size_t)xent_grid(rows, 1024) * (size_t)vocab * sizeof(float);
    const size_t plain = mp_colsum_workspace_bytes(rows, vocab);
    return round256(mp_loss_workspace_bytes(rows, vocab)) + (fused > plain ? fused : plain);
}

extern "C" int mp_softmax_xent_scaled_db(int rows, int vocab, const mp_half* logits, int ld, const int32_t* targets,
                                         mp_scale_state* st, float* loss, mp_half* dlogits, mp_half* db, void* ws,
                                         size_t ws_bytes, mp_stream stream) {
    MP_REQUIRE(rows > 0 && vocab > 0 && ld >= vocab, "mp_softmax_xent_scaled_db: bad shape rows=%d vocab=%d ld=%d", rows,
               vocab, ld);
    MP_REQUIRE(logits && targets && st && loss && dlogits && db, "mp_softmax_xent_scaled_db: NULL argument");
    if (!ws || ws_bytes < mp_softmax_xent_db_workspace_bytes(rows, vocab) || !aligned16(ws)) {
        set_error("mp_softmax_xent_scaled_db: 16-byte aligned workspace of %zu bytes needed, %zu given",
                  mp_softmax_xent_db_workspace_bytes(rows, vocab), ws_bytes);
        return MP_E_WORKSPACE;
    }
    const size_t head = round256(mp_loss_workspace_bytes(rows, vocab));
    float*       part = reinterpret_cast<float*>(static_cast<char*>(ws) + head);
    hipStream_t  hs   = as_stream(stream);
    if (!xent_db_fused(rows, vocab, ld, logits, dlogits)) {
        // small or unaligned vocabularies: the plain loss call, then a column sum over the gradient it stored
        const int rc = mp_softmax_xent_scaled(rows, vocab, logits, ld, targets, st, loss, dlogits, ws, head, stream);
        if (rc != MP_OK) return rc;
        return mp_colsum(rows, vocab, dlogits, ld, db, st, part, ws_bytes - head, stream);
    }
    float*    row_loss = static_cast<float*>(ws);
    const int grid     = xent_grid(rows, 1024);
    hipLaunchKernelGGL((xent_cached_kernel<1024, true>), dim3(grid), dim3(1024), 0, hs, vocab, ld, logits, targets, st, rows,
                       dlogits, row_loss, part);
    MP_LAUNCH_CHECK("mp_softmax_xent_scaled_db");
    hipLaunchKernelGGL(finish_mean_kernel, dim3(1), dim3(LOSS_THREADS), 0, hs, row_loss, rows, (double)rows, loss);
    MP_LAUNCH_CHECK("mp_softmax_xent_scaled_db(finish)");
    return finish_colsum_launch(part, grid, vocab, db, st, hs);
}
