// Bandwidth-bound pieces between the contractions: LayerNorm, attention softmax, LSTM cell,
// column sums (bias gradients), casts and fills.  fp32 arithmetic between fp16 storage points
// (paper Sections 3.1, 3.2).  Every kernel reads each stored input once and writes each stored
// output once; row reductions are wave-level (one 64-lane wave per row), column reductions are
// two-stage through a caller workspace and deterministic.
#include "cell_math.hpp"
#include "common.hpp"

#include <mutex>

namespace mp {

constexpr int GL_THREADS = 256;
constexpr int GL_WAVES   = GL_THREADS / 64;

__device__ __forceinline__ void unpack8(const uint4& q, float* f) {
    const unsigned w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        f[2 * k]     = h2f((uint16_t)(w[k] & 0xFFFF));
        f[2 * k + 1] = h2f((uint16_t)(w[k] >> 16));
    }
}
__device__ __forceinline__ uint4 pack8(const float* f) {
    unsigned w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = (unsigned)f2h(f[2 * k]) | ((unsigned)f2h(f[2 * k + 1]) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// --------------------------------------------------------------------------- partial-sum finish
// out16[c] = RNE16( sum_p part[p * stride + c] ) in a fixed order; optional non-finite flag.
// Workgroup = 32 columns x 8 part-lanes: lane q sums parts q, q+8, ... ; the 8 lane sums are then
// added in lane order.
struct FinishOuts {
    uint16_t* p[3];  // output of segment s covers partial columns [s*n, (s+1)*n)
};
__global__ __launch_bounds__(GL_THREADS) void finish_colsum_kernel(const float* __restrict__ part, int nparts,
                                                                   long long stride, int n, int nseg, FinishOuts outs,
                                                                   mp_scale_state* st) {
    __shared__ float sm[8][33];
    const int cl = threadIdx.x & 31, q = threadIdx.x >> 5;
    const int c  = blockIdx.x * 32 + cl;
    const int nt = n * nseg;
    float     acc = 0.f;
    if (c < nt) {
        // eight loads in flight per lane; the order of additions is fixed (p ascending)
        int p = q;
        for (; p + 56 < nparts; p += 64) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = part[(long long)(p + 8 * u) * stride + c];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += t[u];
        }
        for (; p < nparts; p += 8) acc += part[(long long)p * stride + c];
    }
    sm[q][cl] = acc;
    __syncthreads();
    bool bad = false;
    if (q == 0 && c < nt) {
        float t = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) t += sm[j][cl];
        const uint16_t h   = f2h(t);
        const int      seg = c / n;
        uint16_t*      o   = seg == 0 ? outs.p[0] : (seg == 1 ? outs.p[1] : outs.p[2]);
        o[c - seg * n]     = h;
        bad                = half_nonfinite(h);
    }
    if (st != nullptr && __any(bad)) {
        if ((threadIdx.x & 63) == 0) atomicOr(&st->found_inf, 1);
    }
}

// --------------------------------------------------------------------------- column sums
// Workgroup = 8 column-groups x 32 row-lanes; VEC columns per column-group (a row piece of 8 x 16 B =
// one 128-byte line per row when VEC = 8).
template <int VEC>
__global__ __launch_bounds__(GL_THREADS) void colsum_kernel(int rows, int cols, int ld, const uint16_t* __restrict__ dy,
                                                            int rows_per_block, float* __restrict__ part) {
    __shared__ float sm[32][8 * VEC + 1];
    const int cg = threadIdx.x & 7, rl = threadIdx.x >> 3;
    const int c0 = (blockIdx.x * 8 + cg) * VEC;
    const int r0 = blockIdx.y * rows_per_block;
    const int r1 = min(rows, r0 + rows_per_block);
    float     acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
    if (c0 < cols) {
        for (int r = r0 + rl; r < r1; r += 32) {
            if (VEC == 8) {
                float f[8];
                unpack8(*reinterpret_cast<const uint4*>(dy + (long long)r * ld + c0), f);
#pragma unroll
                for (int k = 0; k < 8; ++k) acc[k] += f[k];
            } else {
                acc[0] += h2f(dy[(long long)r * ld + c0]);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < VEC; ++k) sm[rl][cg * VEC + k] = acc[k];
    __syncthreads();
    for (int c = threadIdx.x; c < 8 * VEC; c += GL_THREADS) {
        float t = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) t += sm[j][c];
        const int gc = blockIdx.x * 8 * VEC + c;
        if (gc < cols) part[(long long)blockIdx.y * cols + gc] = t;
    }
}

// --------------------------------------------------------------------------- LayerNorm
// One wave per row.  MAXV 16-byte vectors per lane are kept in registers (d <= 64*8*MAXV).
constexpr int LN_MAXV = 4;

__global__ __launch_bounds__(GL_THREADS) void layernorm_fwd_kernel(int rows, int d, const uint16_t* __restrict__ x,
                                                                   const uint16_t* __restrict__ a,
                                                                   const uint16_t* __restrict__ gamma,
                                                                   const uint16_t* __restrict__ beta, float eps,
                                                                   uint16_t* __restrict__ y, float* __restrict__ mean_o,
                                                                   float* __restrict__ rstd_o) {
    const int lane = threadIdx.x & 63;
    const int row  = blockIdx.x * GL_WAVES + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int       nvec = d >> 3;
    const long long base = (long long)row * d;
    float           z[LN_MAXV][8];
    float           s = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        const int v = i * 64 + lane;
        if (v < nvec) {
            unpack8(*reinterpret_cast<const uint4*>(x + base + v * 8), z[i]);
            if (a != nullptr) {
                float t[8];
                unpack8(*reinterpret_cast<const uint4*>(a + base + v * 8), t);
#pragma unroll
                for (int k = 0; k < 8; ++k) z[i][k] += t[k];
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) s += z[i][k];
        }
    }
    const float mean = wave_sum(s) / (float)d;
    float       q    = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        const int v = i * 64 + lane;
        if (v < nvec) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                z[i][k] -= mean;
                q += z[i][k] * z[i][k];
            }
        }
    }
    const float var  = wave_sum(q) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    if (lane == 0) {
        mean_o[row] = mean;
        rstd_o[row] = rstd;
    }
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
        const int v = i * 64 + lane;
        if (v < nvec) {
            float g[8], b[8], o[8];
            unpack8(*reinterpret_cast<const uint4*>(gamma + v * 8), g);
            unpack8(*reinterpret_cast<const uint4*>(beta + v * 8), b);
#pragma unroll
            for (int k = 0; k < 8; ++k) o[k] = (z[i][k] * rstd) * g[k] + b[k];
            *reinterpret_cast<uint4*>(y + base + v * 8) = pack8(o);
        }
    }
}

// Backward: each wave walks rows  row = wave_global, wave_global + n_waves, ...  and keeps the
// column sums of dy*xhat and dy for its rows in registers; they are combined per workgroup in LDS
// and written as partials part[block][NS][d] (NS = 3 with ZSUM: also the column sums of the stored dz,
// which is the bias gradient of the linear layer whose output fed this LayerNorm).
// MAXV = 16-byte vectors per lane (d <= 64 * 8 * MAXV).  The raw vectors of the wave's next row are requested
// before the current row is reduced, so the two cross-lane reductions of a row overlap the next row's loads.
template <bool ZSUM, int MAXV>
__global__ __launch_bounds__(GL_THREADS) void layernorm_bwd_kernel(int rows, int d, const uint16_t* __restrict__ dy,
                                                                   const uint16_t* __restrict__ x,
                                                                   const uint16_t* __restrict__ a,
                                                                   const uint16_t* __restrict__ gamma,
                                                                   const float* __restrict__ mean_i,
                                                                   const float* __restrict__ rstd_i,
                                                                   uint16_t* __restrict__ dz, float* __restrict__ part) {
    extern __shared__ float sm[];  // [GL_WAVES][NS][d]
    constexpr int NS = ZSUM ? 3 : 2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nvec = d >> 3;
    float     gam[MAXV][8], sg[MAXV][8], sb[MAXV][8], sz[ZSUM ? MAXV : 1][8];
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int v = i * 64 + lane;
#pragma unroll
        for (int k = 0; k < 8; ++k) sg[i][k] = sb[i][k] = gam[i][k] = 0.f;
        if (ZSUM) {
#pragma unroll
            for (int k = 0; k < 8; ++k) sz[i][k] = 0.f;
        }
        if (v < nvec) unpack8(*reinterpret_cast<const uint4*>(gamma + v * 8), gam[i]);
    }
    const int stride = gridDim.x * GL_WAVES;
    uint4     rdy[MAXV], rx[MAXV], ra[MAXV];  // raw vectors of the row being worked on
    float     mean = 0.f, rstd = 0.f;
    auto fetch = [&](int row, uint4* qdy, uint4* qx, uint4* qa, float& mu, float& rs) {
        const long long base = (long long)row * d;
#pragma unroll
        for (int i = 0; i < MAXV; ++i) {
            const int v = i * 64 + lane;
            qdy[i] = qx[i] = qa[i] = make_uint4(0u, 0u, 0u, 0u);
            if (v < nvec) {
                qdy[i] = *reinterpret_cast<const uint4*>(dy + base + v * 8);
                qx[i]  = *reinterpret_cast<const uint4*>(x + base + v * 8);
                if (a != nullptr) qa[i] = *reinterpret_cast<const uint4*>(a + base + v * 8);
            }
        }
        mu = mean_i[row];
        rs = rstd_i[row];
    };
    int row = blockIdx.x * GL_WAVES + wave;
    if (row < rows) fetch(row, rdy, rx, ra, mean, rstd);
    for (; row < rows; row += stride) {
        uint4 ndy[MAXV], nx[MAXV], na[MAXV];
        float nmean = 0.f, nrstd = 0.f;
        if (row + stride < rows) fetch(row + stride, ndy, nx, na, nmean, nrstd);
        const long long base = (long long)row * d;
        float           xh[MAXV][8], g[MAXV][8];
        float           s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < MAXV; ++i) {
            const int v = i * 64 + lane;
            if (v < nvec) {
                float dyv[8];
                unpack8(rdy[i], dyv);
                unpack8(rx[i], xh[i]);
                if (a != nullptr) {
                    float t[8];
                    unpack8(ra[i], t);
#pragma unroll
                    for (int k = 0; k < 8; ++k) xh[i][k] += t[k];
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    xh[i][k] = (xh[i][k] - mean) * rstd;
                    g[i][k]  = dyv[k] * gam[i][k];
                    s1 += g[i][k];
                    s2 += g[i][k] * xh[i][k];
                    sg[i][k] += dyv[k] * xh[i][k];
                    sb[i][k] += dyv[k];
                }
            }
        }
        const float m1 = wave_sum(s1) / (float)d;
        const float m2 = wave_sum(s2) / (float)d;
#pragma unroll
        for (int i = 0; i < MAXV; ++i) {
            const int v = i * 64 + lane;
            if (v < nvec) {
                float o[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) o[k] = rstd * (g[i][k] - m1 - xh[i][k] * m2);
                *reinterpret_cast<uint4*>(dz + base + v * 8) = pack8(o);
                if (ZSUM) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) sz[i][k] += round16(o[k]);  // sums the stored (fp16) values
                }
            }
        }
#pragma unroll
        for (int i = 0; i < MAXV; ++i) {
            rdy[i] = ndy[i];
            rx[i]  = nx[i];
            ra[i]  = na[i];
        }
        mean = nmean;
        rstd = nrstd;
    }
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int v = i * 64 + lane;
        if (v < nvec) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                sm[(wave * NS + 0) * d + v * 8 + k] = sg[i][k];
                sm[(wave * NS + 1) * d + v * 8 + k] = sb[i][k];
                if (ZSUM) sm[(wave * NS + 2) * d + v * 8 + k] = sz[i][k];
            }
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < NS * d; c += GL_THREADS) {
        const int which = c / d, col = c - which * d;
        float     t     = 0.f;
#pragma unroll
        for (int w = 0; w < GL_WAVES; ++w) t += sm[(w * NS + which) * d + col];
        part[(long long)blockIdx.x * NS * d + c] = t;
    }
}

// --------------------------------------------------------------------------- attention softmax
// One wave per row, EPL consecutive elements per lane (cols <= 64 * EPL).
template <int EPL>
struct PackT;
template <> struct PackT<1> { typedef uint16_t T; };
template <> struct PackT<2> { typedef uint32_t T; };
template <> struct PackT<4> { typedef uint2 T; };
template <> struct PackT<8> { typedef uint4 T; };

template <int EPL>
__device__ __forceinline__ void load_epl(const uint16_t* p, float* f) {
    typename PackT<EPL>::T raw = *reinterpret_cast<const typename PackT<EPL>::T*>(p);
    const uint16_t*        h   = reinterpret_cast<const uint16_t*>(&raw);
#pragma unroll
    for (int k = 0; k < EPL; ++k) f[k] = h2f(h[k]);
}
template <int EPL>
__device__ __forceinline__ void store_epl(uint16_t* p, const float* f) {
    typename PackT<EPL>::T raw;
    uint16_t*              h = reinterpret_cast<uint16_t*>(&raw);
#pragma unroll
    for (int k = 0; k < EPL; ++k) h[k] = f2h(f[k]);
    *reinterpret_cast<typename PackT<EPL>::T*>(p) = raw;
}

template <int EPL>
__global__ __launch_bounds__(GL_THREADS) void softmax_fwd_kernel(long long rows, int cols, int ld, const uint16_t* s,
                                                                 uint16_t* p) {
    const int lane = threadIdx.x & 63;
    for (long long row = (long long)blockIdx.x * GL_WAVES + (threadIdx.x >> 6); row < rows;
         row += (long long)gridDim.x * GL_WAVES) {
        const int  c0 = lane * EPL;
        const bool on = c0 < cols;  // cols is a multiple of EPL on this path
        float      f[EPL];
        float      mx = -INFINITY;
        if (on) {
            load_epl<EPL>(s + row * ld + c0, f);
#pragma unroll
            for (int k = 0; k < EPL; ++k) mx = fmaxf(mx, f[k]);
        }
        mx       = wave_max(mx);
        float se = 0.f;
        if (on) {
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                f[k] = __expf(f[k] - mx);
                se += f[k];
            }
        }
        se = wave_sum(se);
        if (on) {
#pragma unroll
            for (int k = 0; k < EPL; ++k) f[k] = f[k] / se;
            store_epl<EPL>(p + row * ld + c0, f);
        }
    }
}

template <int EPL>
__global__ __launch_bounds__(GL_THREADS) void softmax_bwd_kernel(long long rows, int cols, int ld, const uint16_t* p,
                                                                 const uint16_t* dp, uint16_t* ds) {
    const int lane = threadIdx.x & 63;
    for (long long row = (long long)blockIdx.x * GL_WAVES + (threadIdx.x >> 6); row < rows;
         row += (long long)gridDim.x * GL_WAVES) {
        const int  c0 = lane * EPL;
        const bool on = c0 < cols;
        float      pv[EPL], dv[EPL];
        float      inner = 0.f;
        if (on) {
            load_epl<EPL>(p + row * ld + c0, pv);
            load_epl<EPL>(dp + row * ld + c0, dv);
#pragma unroll
            for (int k = 0; k < EPL; ++k) inner += dv[k] * pv[k];
        }
        inner = wave_sum(inner);
        if (on) {
#pragma unroll
            for (int k = 0; k < EPL; ++k) dv[k] = pv[k] * (dv[k] - inner);
            store_epl<EPL>(ds + row * ld + c0, dv);
        }
    }
}

// Generic rows (any cols / alignment): one wave per row, strided scalar accesses, three sweeps.
__global__ __launch_bounds__(GL_THREADS) void softmax_fwd_generic_kernel(long long rows, int cols, int ld,
                                                                         const uint16_t* s, uint16_t* p) {
    const int lane = threadIdx.x & 63;
    for (long long row = (long long)blockIdx.x * GL_WAVES + (threadIdx.x >> 6); row < rows;
         row += (long long)gridDim.x * GL_WAVES) {
        const uint16_t* sr = s + row * ld;
        uint16_t*       pr = p + row * ld;
        float           mx = -INFINITY;
        for (int c = lane; c < cols; c += 64) mx = fmaxf(mx, h2f(sr[c]));
        mx       = wave_max(mx);
        float se = 0.f;
        for (int c = lane; c < cols; c += 64) se += __expf(h2f(sr[c]) - mx);
        se = wave_sum(se);
        for (int c = lane; c < cols; c += 64) pr[c] = f2h(__expf(h2f(sr[c]) - mx) / se);
    }
}
__global__ __launch_bounds__(GL_THREADS) void softmax_bwd_generic_kernel(long long rows, int cols, int ld,
                                                                         const uint16_t* p, const uint16_t* dp,
                                                                         uint16_t* ds) {
    const int lane = threadIdx.x & 63;
    for (long long row = (long long)blockIdx.x * GL_WAVES + (threadIdx.x >> 6); row < rows;
         row += (long long)gridDim.x * GL_WAVES) {
        float inner = 0.f;
        for (int c = lane; c < cols; c += 64) inner += h2f(dp[row * ld + c]) * h2f(p[row * ld + c]);
        inner = wave_sum(inner);
        for (int c = lane; c < cols; c += 64) {
            const float pv    = h2f(p[row * ld + c]);
            ds[row * ld + c] = f2h(pv * (h2f(dp[row * ld + c]) - inner));
        }
    }
}

// --------------------------------------------------------------------------- LSTM cell
__global__ __launch_bounds__(GL_THREADS) void lstm_cell_fwd_kernel(int B, int H, const uint16_t* __restrict__ gates,
                                                                   int ldg, const float* __restrict__ c_prev,
                                                                   float* __restrict__ c, uint16_t* __restrict__ h1,
                                                                   int ldh, uint16_t* __restrict__ h2, int ldh2) {
    const int idx = blockIdx.x * GL_THREADS + threadIdx.x;
    if (idx >= B * H) return;
    const int       b = idx / H, j = idx - b * H;
    const uint16_t* g  = gates + (long long)b * ldg;
    uint16_t        hv;
    c[idx] = lstm_cell_forward(h2f(g[j]), h2f(g[H + j]), h2f(g[2 * H + j]), h2f(g[3 * H + j]), c_prev[idx], &hv);
    h1[(long long)b * ldh + j] = hv;
    if (h2 != nullptr) h2[(long long)b * ldh2 + j] = hv;
}

__global__ __launch_bounds__(GL_THREADS) void lstm_cell_bwd_kernel(int B, int H, const uint16_t* __restrict__ gates,
                                                                   int ldg, const float* __restrict__ c_prev,
                                                                   const float* __restrict__ c,
                                                                   const uint16_t* __restrict__ dh_a, int ld_a,
                                                                   const uint16_t* __restrict__ dh_b, int ld_b,
                                                                   float* __restrict__ dc_io,
                                                                   uint16_t* __restrict__ dgates) {
    const int idx = blockIdx.x * GL_THREADS + threadIdx.x;
    if (idx >= B * H) return;
    const int       b = idx / H, j = idx - b * H;
    const uint16_t* g  = gates + (long long)b * ldg;
    uint16_t*       dg = dgates + (long long)b * ldg;
    float           dh = 0.f;
    if (dh_a != nullptr) dh += h2f(dh_a[(long long)b * ld_a + j]);
    if (dh_b != nullptr) dh += h2f(dh_b[(long long)b * ld_b + j]);
    uint16_t d4[4];
    dc_io[idx] = lstm_cell_backward(h2f(g[j]), h2f(g[H + j]), h2f(g[2 * H + j]), h2f(g[3 * H + j]), c_prev[idx], c[idx], dh,
                                    dc_io[idx], d4);
    dg[j]         = d4[0];
    dg[H + j]     = d4[1];
    dg[2 * H + j] = d4[2];
    dg[3 * H + j] = d4[3];
}

// --------------------------------------------------------------------------- cast / fill
__global__ __launch_bounds__(GL_THREADS) void cast_kernel(size_t n, const float* __restrict__ src,
                                                          uint16_t* __restrict__ dst, bool vec) {
    const size_t stride = (size_t)gridDim.x * GL_THREADS;
    if (vec) {
        const size_t nv = n >> 3;
        for (size_t v = (size_t)blockIdx.x * GL_THREADS + threadIdx.x; v < nv; v += stride) {
            const float4 a = *reinterpret_cast<const float4*>(src + v * 8);
            const float4 b = *reinterpret_cast<const float4*>(src + v * 8 + 4);
            const float  f[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            *reinterpret_cast<uint4*>(dst + v * 8) = pack8(f);
        }
        for (size_t i = (nv << 3) + (size_t)blockIdx.x * GL_THREADS + threadIdx.x; i < n; i += stride) dst[i] = f2h(src[i]);
    } else {
        for (size_t i = (size_t)blockIdx.x * GL_THREADS + threadIdx.x; i < n; i += stride) dst[i] = f2h(src[i]);
    }
}

__global__ __launch_bounds__(GL_THREADS) void fill_kernel(size_t n, uint32_t value, uint32_t* __restrict__ dst) {
    const size_t stride = (size_t)gridDim.x * GL_THREADS;
    for (size_t i = (size_t)blockIdx.x * GL_THREADS + threadIdx.x; i < n; i += stride) dst[i] = value;
}

}  // namespace mp

using namespace mp;

static int grid_for(size_t units, int per_block, int cap) {
    size_t b = (units + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > (size_t)cap) b = cap;
    return (int)b;
}

// ---- column sums
static int colsum_row_blocks(int rows, int cols, int vec) {
    const int col_blocks = (cols + 8 * vec - 1) / (8 * vec);
    int       rb         = 1024 / (col_blocks > 0 ? col_blocks : 1);
    if (rb > 32) rb = 32;                 // partial rows the finish kernel has to add up
    const int max_rb = (rows + 63) / 64;  // at least 64 rows per workgroup
    if (rb > max_rb) rb = max_rb;
    if (rb < 1) rb = 1;
    return rb;
}

extern "C" size_t mp_colsum_workspace_bytes(int rows, int cols) {
    if (rows <= 0 || cols <= 0) return 0;
    // the scalar path (vec = 1) never uses more row blocks than the vector path allows for
    const int rb8 = colsum_row_blocks(rows, cols, 8), rb1 = colsum_row_blocks(rows, cols, 1);
    return (size_t)(rb8 > rb1 ? rb8 : rb1) * cols * sizeof(float);
}

int mp::finish_colsum_launch(const float* part, int nparts, int cols, mp_half* db, mp_scale_state* st, hipStream_t hs) {
    FinishOuts outs{{db, nullptr, nullptr}};
    hipLaunchKernelGGL(finish_colsum_kernel, dim3((cols + 31) / 32), dim3(GL_THREADS), 0, hs, part, nparts, (long long)cols,
                       cols, 1, outs, st);
    MP_LAUNCH_CHECK("column-sum finish");
    return MP_OK;
}

// Both launches of a column sum; `part` holds mp_colsum_workspace_bytes(rows, cols) bytes of partial sums, every one of
// which the first launch writes before the second reads it (nothing has to start at zero).
static int colsum_launch(int rows, int cols, const mp_half* dY, int ld, mp_half* db, mp_scale_state* st, float* part,
                         hipStream_t hs) {
    const bool  vec = (cols % 8 == 0) && (ld % 8 == 0) && aligned16(dY);
    const int   V   = vec ? 8 : 1;
    const int   rb  = colsum_row_blocks(rows, cols, V);
    const int   rpb = (rows + rb - 1) / rb;
    const dim3  grid((cols + 8 * V - 1) / (8 * V), rb);
    if (vec)
        hipLaunchKernelGGL(colsum_kernel<8>, grid, dim3(GL_THREADS), 0, hs, rows, cols, ld, dY, rpb, part);
    else
        hipLaunchKernelGGL(colsum_kernel<1>, grid, dim3(GL_THREADS), 0, hs, rows, cols, ld, dY, rpb, part);
    MP_LAUNCH_CHECK("mp_colsum");
    FinishOuts outs{{db, nullptr, nullptr}};
    hipLaunchKernelGGL(finish_colsum_kernel, dim3((cols + 31) / 32), dim3(GL_THREADS), 0, hs, part, rb,
                       (long long)cols, cols, 1, outs, st);
    MP_LAUNCH_CHECK("mp_colsum(finish)");
    return MP_OK;
}

extern "C" int mp_colsum(int rows, int cols, const mp_half* dY, int ld, mp_half* db, mp_scale_state* st, void* ws,
                         size_t ws_bytes, mp_stream stream) {
    MP_REQUIRE(rows > 0 && cols > 0 && ld >= cols, "mp_colsum: bad shape rows=%d cols=%d ld=%d", rows, cols, ld);
    MP_REQUIRE(dY && db, "mp_colsum: NULL argument");
    if (!ws || ws_bytes < mp_colsum_workspace_bytes(rows, cols)) {
        set_error("mp_colsum: workspace of %zu bytes needed, %zu given", mp_colsum_workspace_bytes(rows, cols), ws_bytes);
        return MP_E_WORKSPACE;
    }
    return colsum_launch(rows, cols, dY, ld, db, st, static_cast<float*>(ws), as_stream(stream));
}

// ---- column sums for callers that cannot allocate (code under HIP-graph capture, serving loops, harnesses that
// forbid hipMalloc): the partial sums live in a fixed array in the library's device image instead of a caller
// workspace.  Every GPU holds its own copy of the array at its own address; the array's NAME is only a host-side
// handle, so the device address is looked up once per device and only that pointer is ever handed to a kernel.
constexpr size_t kColsumScratchFloats = 262144;  // 1 MiB: covers every shape with cols <= 262144 (see the row-block rule)
static __device__ __align__(256) float scratch[kColsumScratchFloats];

constexpr int     kMaxDevices = 64;
static float*     g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, once looked up
static std::mutex g_scratch_mu;

static int colsum_scratch(float** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "mp_colsum_static: hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("mp_colsum_static: device index %d outside 0..%d", dev, kMaxDevices - 1);
        return MP_E_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // for the CURRENT device, which is `dev`
        if (e != hipSuccess || p == nullptr) return hip_fail(e, "mp_colsum_static: hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = static_cast<float*>(p);
    }
    *out = g_scratch_ptr[dev];
    return MP_OK;
}

extern "C" size_t mp_colsum_static_max_bytes(void) { return kColsumScratchFloats * sizeof(float); }

extern "C" int mp_colsum_static(int rows, int cols, const mp_half* dY, int ld, mp_half* db, mp_scale_state* st,
                                mp_stream stream) {
    MP_REQUIRE(rows > 0 && cols > 0 && ld >= cols, "mp_colsum_static: bad shape rows=%d cols=%d ld=%d", rows, cols, ld);
    MP_REQUIRE(dY && db, "mp_colsum_static: NULL argument");
    const size_t need = mp_colsum_workspace_bytes(rows, cols);
    if (need > kColsumScratchFloats * sizeof(float)) {
        set_error("mp_colsum_static: %d x %d needs %zu bytes of partial sums, the built-in scratch holds %zu; use mp_colsum "
                  "with a workspace", rows, cols, need, kColsumScratchFloats * sizeof(float));
        return MP_E_WORKSPACE;
    }
    float* part = nullptr;
    const int rc = colsum_scratch(&part);
    if (rc != MP_OK) return rc;
    return colsum_launch(rows, cols, dY, ld, db, st, part, as_stream(stream));
}

// ---- LayerNorm
static bool ln_shape_ok(int d) { return d % 8 == 0 && d <= 64 * 8 * LN_MAXV; }

extern "C" int mp_layernorm_fwd(int rows, int d, const mp_half* x, const mp_half* a, const mp_half* gamma,
                                const mp_half* beta, float eps, mp_half* y, float* mean, float* rstd, mp_stream stream) {
    MP_REQUIRE(rows > 0 && d > 0, "mp_layernorm_fwd: bad shape rows=%d d=%d", rows, d);
    MP_REQUIRE(x && gamma && beta && y && mean && rstd, "mp_layernorm_fwd: NULL argument");
    if (!ln_shape_ok(d)) {
        set_error("mp_layernorm_fwd: d=%d unsupported (need a multiple of 8, at most %d)", d, 64 * 8 * LN_MAXV);
        return MP_E_UNSUPPORTED;
    }
    MP_REQUIRE(aligned16(x) && (a == nullptr || aligned16(a)) && aligned16(gamma) && aligned16(beta) && aligned16(y),
               "mp_layernorm_fwd: pointers must be 16-byte aligned");
    hipLaunchKernelGGL(layernorm_fwd_kernel, dim3((rows + GL_WAVES - 1) / GL_WAVES), dim3(GL_THREADS), 0, as_stream(stream),
                       rows, d, x, a, gamma, beta, eps, y, mean, rstd);
    MP_LAUNCH_CHECK("mp_layernorm_fwd");
    return MP_OK;
}

static int ln_bwd_blocks(int rows) {
    int nb = (rows + GL_WAVES * 4 - 1) / (GL_WAVES * 4);  // about 4 rows per wave
    if (nb > 512) nb = 512;
    if (nb < 1) nb = 1;
    return nb;
}

extern "C" size_t mp_layernorm_bwd_workspace_bytes(int rows, int d) {
    if (rows <= 0 || d <= 0) return 0;
    return (size_t)ln_bwd_blocks(rows) * 3 * d * sizeof(float);
}

extern "C" int mp_layernorm_bwd(int rows, int d, const mp_half* dy, const mp_half* x, const mp_half* a,
                                const mp_half* gamma, const float* mean, const float* rstd, mp_half* dz, mp_half* dgamma,
                                mp_half* dbeta, mp_half* dz_colsum, mp_scale_state* st, void* ws, size_t ws_bytes,
                                mp_stream stream) {
    MP_REQUIRE(rows > 0 && d > 0, "mp_layernorm_bwd: bad shape rows=%d d=%d", rows, d);
    MP_REQUIRE(dy && x && gamma && mean && rstd && dz && dgamma && dbeta, "mp_layernorm_bwd: NULL argument");
    if (!ln_shape_ok(d)) {
        set_error("mp_layernorm_bwd: d=%d unsupported (need a multiple of 8, at most %d)", d, 64 * 8 * LN_MAXV);
        return MP_E_UNSUPPORTED;
    }
    MP_REQUIRE(aligned16(dy) && aligned16(x) && (a == nullptr || aligned16(a)) && aligned16(gamma) && aligned16(dz),
               "mp_layernorm_bwd: pointers must be 16-byte aligned");
    if (!ws || ws_bytes < mp_layernorm_bwd_workspace_bytes(rows, d)) {
        set_error("mp_layernorm_bwd: workspace of %zu bytes needed, %zu given", mp_layernorm_bwd_workspace_bytes(rows, d),
                  ws_bytes);
        return MP_E_WORKSPACE;
    }
    const int   nb   = ln_bwd_blocks(rows);
    const int   ns   = dz_colsum ? 3 : 2;
    float*      part = static_cast<float*>(ws);
    hipStream_t hs   = as_stream(stream);
    const size_t lds = (size_t)GL_WAVES * ns * d * sizeof(float);
    const bool small = d <= 64 * 8 * 2;  // two vectors per lane are enough: fewer registers, more waves per CU
    if (dz_colsum) {
        if (small)
            hipLaunchKernelGGL((layernorm_bwd_kernel<true, 2>), dim3(nb), dim3(GL_THREADS), lds, hs, rows, d, dy, x, a, gamma,
                               mean, rstd, dz, part);
        else
            hipLaunchKernelGGL((layernorm_bwd_kernel<true, LN_MAXV>), dim3(nb), dim3(GL_THREADS), lds, hs, rows, d, dy, x, a,
                               gamma, mean, rstd, dz, part);
    } else {
        if (small)
            hipLaunchKernelGGL((layernorm_bwd_kernel<false, 2>), dim3(nb), dim3(GL_THREADS), lds, hs, rows, d, dy, x, a, gamma,
                               mean, rstd, dz, part);
        else
            hipLaunchKernelGGL((layernorm_bwd_kernel<false, LN_MAXV>), dim3(nb), dim3(GL_THREADS), lds, hs, rows, d, dy, x, a,
                               gamma, mean, rstd, dz, part);
    }
    MP_LAUNCH_CHECK("mp_layernorm_bwd");
    FinishOuts outs{{dgamma, dbeta, dz_colsum}};
    hipLaunchKernelGGL(finish_colsum_kernel, dim3((ns * d + 31) / 32), dim3(GL_THREADS), 0, hs, part, nb, (long long)ns * d,
                       d, ns, outs, st);
    MP_LAUNCH_CHECK("mp_layernorm_bwd(finish)");
    return MP_OK;
}

// ---- attention softmax
template <typename F8, typename F4, typename F2, typename F1, typename FG>
static void softmax_dispatch(int cols, int ld, bool al16, bool al8, bool al4, F8 f8, F4 f4, F2 f2, F1 f1, FG fg) {
    if (cols <= 64) f1();
    else if (cols <= 128 && cols % 2 == 0 && ld % 2 == 0 && al4) f2();
    else if (cols <= 256 && cols % 4 == 0 && ld % 4 == 0 && al8) f4();
    else if (cols <= 512 && cols % 8 == 0 && ld % 8 == 0 && al16) f8();
    else fg();
}

extern "C" int mp_softmax_fwd(int64_t rows, int cols, const mp_half* s, mp_half* p, int ld, mp_stream stream) {
    MP_REQUIRE(rows > 0 && cols > 0 && ld >= cols, "mp_softmax_fwd: bad shape");
    MP_REQUIRE(s && p, "mp_softmax_fwd: NULL argument");
    const int   nb = grid_for((size_t)rows, GL_WAVES, 1 << 20);
    hipStream_t hs = as_stream(stream);
    auto        al = [&](int a) { return ((uintptr_t)s % a == 0) && ((uintptr_t)p % a == 0); };
    long long   r  = rows;
    softmax_dispatch(
        cols, ld, al(16), al(8), al(4),
        [&] { hipLaunchKernelGGL(softmax_fwd_kernel<8>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, s, p); },
        [&] { hipLaunchKernelGGL(softmax_fwd_kernel<4>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, s, p); },
        [&] { hipLaunchKernelGGL(softmax_fwd_kernel<2>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, s, p); },
        [&] { hipLaunchKernelGGL(softmax_fwd_kernel<1>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, s, p); },
        [&] { hipLaunchKernelGGL(softmax_fwd_generic_kernel, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, s, p); });
    MP_LAUNCH_CHECK("mp_softmax_fwd");
    return MP_OK;
}

extern "C" int mp_softmax_bwd(int64_t rows, int cols, const mp_half* p, const mp_half* dp, mp_half* ds, int ld,
                              mp_stream stream) {
    MP_REQUIRE(rows > 0 && cols > 0 && ld >= cols, "mp_softmax_bwd: bad shape");
    MP_REQUIRE(p && dp && ds, "mp_softmax_bwd: NULL argument");
    const int   nb = grid_for((size_t)rows, GL_WAVES, 1 << 20);
    hipStream_t hs = as_stream(stream);
    auto al = [&](int a) { return ((uintptr_t)p % a == 0) && ((uintptr_t)dp % a == 0) && ((uintptr_t)ds % a == 0); };
    long long r = rows;
    softmax_dispatch(
        cols, ld, al(16), al(8), al(4),
        [&] { hipLaunchKernelGGL(softmax_bwd_kernel<8>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, p, dp, ds); },
        [&] { hipLaunchKernelGGL(softmax_bwd_kernel<4>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, p, dp, ds); },
        [&] { hipLaunchKernelGGL(softmax_bwd_kernel<2>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, p, dp, ds); },
        [&] { hipLaunchKernelGGL(softmax_bwd_kernel<1>, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, p, dp, ds); },
        [&] { hipLaunchKernelGGL(softmax_bwd_generic_kernel, dim3(nb), dim3(GL_THREADS), 0, hs, r, cols, ld, p, dp, ds); });
    MP_LAUNCH_CHECK("mp_softmax_bwd");
    return MP_OK;
}

// ---- LSTM cell
extern "C" int mp_lstm_cell_fwd(int B, int H, const mp_half* gates, int ldg, const float* c_prev, float* c, mp_half* h_out,
                                int ldh, mp_half* h_out2, int ldh2, mp_stream stream) {
    MP_REQUIRE(B > 0 && H > 0 && ldg >= 4 * H && ldh >= H && (h_out2 == nullptr || ldh2 >= H), "mp_lstm_cell_fwd: bad shape");
    MP_REQUIRE(gates && c_prev && c && h_out, "mp_lstm_cell_fwd: NULL argument");
    MP_REQUIRE((long long)B * H < (1ll << 31), "mp_lstm_cell_fwd: B*H too large");
    hipLaunchKernelGGL(lstm_cell_fwd_kernel, dim3((B * H + GL_THREADS - 1) / GL_THREADS), dim3(GL_THREADS), 0,
                       as_stream(stream), B, H, gates, ldg, c_prev, c, h_out, ldh, h_out2, ldh2);
    MP_LAUNCH_CHECK("mp_lstm_cell_fwd");
    return MP_OK;
}

extern "C" int mp_lstm_cell_bwd(int B, int H, const mp_half* gates, int ldg, const float* c_prev, const float* c,
                                const mp_half* dh_a, int ld_a, const mp_half* dh_b, int ld_b, float* dc, mp_half* dgates,
                                mp_stream stream) {
    MP_REQUIRE(B > 0 && H > 0 && ldg >= 4 * H, "mp_lstm_cell_bwd: bad shape");
    MP_REQUIRE(gates && c_prev && c && dc && dgates, "mp_lstm_cell_bwd: NULL argument");
    MP_REQUIRE((dh_a == nullptr || ld_a >= H) && (dh_b == nullptr || ld_b >= H), "mp_lstm_cell_bwd: bad dh leading dimension");
    MP_REQUIRE((long long)B * H < (1ll << 31), "mp_lstm_cell_bwd: B*H too large");
    hipLaunchKernelGGL(lstm_cell_bwd_kernel, dim3((B * H + GL_THREADS - 1) / GL_THREADS), dim3(GL_THREADS), 0,
                       as_stream(stream), B, H, gates, ldg, c_prev, c, dh_a, ld_a, dh_b, ld_b, dc, dgates);
    MP_LAUNCH_CHECK("mp_lstm_cell_bwd");
    return MP_OK;
}

// ---- cast / fill
extern "C" int mp_cast_f32_to_f16(size_t n, const float* src, mp_half* dst, mp_stream stream) {
    if (n == 0) return MP_OK;
    MP_REQUIRE(src && dst, "mp_cast_f32_to_f16: NULL argument");
    const bool vec = aligned16(src) && aligned16(dst);
    hipLaunchKernelGGL(cast_kernel, dim3(grid_for(n / 8 + 1, GL_THREADS, 4096)), dim3(GL_THREADS), 0, as_stream(stream), n,
                       src, dst, vec);
    MP_LAUNCH_CHECK("mp_cast_f32_to_f16");
    return MP_OK;
}

extern "C" int mp_fill_u32(size_t n, uint32_t value, void* dst, mp_stream stream) {
    if (n == 0) return MP_OK;
    MP_REQUIRE(dst && ((uintptr_t)dst & 3) == 0, "mp_fill_u32: dst NULL or not 4-byte aligned");
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n, GL_THREADS, 4096)), dim3(GL_THREADS), 0, as_stream(stream), n, value,
                       static_cast<uint32_t*>(dst));
    MP_LAUNCH_CHECK("mp_fill_u32");
    return MP_OK;
}
