// Contractions: planner, split-K finish, generic fallback and the C entry points.  The matrix-core kernel templates are
// in gemm_kernels.hpp and are instantiated in gemm_kk.hip / gemm_ko.hip / gemm_oo.hip.
#include "gemm_dtl.hpp"

#include <cstdlib>
#include <cstring>

namespace mp {

extern template int launch_tile<true, true>(int, const GemmArgs&, dim3, hipStream_t);
extern template int launch_tile<true, false>(int, const GemmArgs&, dim3, hipStream_t);
extern template int launch_tile<false, false>(int, const GemmArgs&, dim3, hipStream_t);
extern template int launch_dtl_tile<true, true>(int, const GemmArgs&, int, hipStream_t);
extern template int launch_dtl_tile<true, false>(int, const GemmArgs&, int, hipStream_t);
extern template int launch_dtl_tile<false, false>(int, const GemmArgs&, int, hipStream_t);
extern template int launch_grouped<256, 256>(const GroupArgs&, int, hipStream_t);
extern template int launch_grouped<128, 128>(const GroupArgs&, int, hipStream_t);
extern template int launch_dtl_grouped<256, 256>(const GroupArgs&, int, hipStream_t);
extern template int launch_dtl_grouped<128, 128>(const GroupArgs&, int, hipStream_t);

// Sum split-K partials in split order, scale, round once, optional non-finite flag.
__global__ __launch_bounds__(256) void splitk_finish_kernel(const float* __restrict__ part, int splits, long long mn,
                                                            int N, int ldc, float alpha, const uint16_t* __restrict__ bias,
                                                            uint16_t* __restrict__ C, int* found_inf) {
    bool bad = false;
    for (long long v = (long long)blockIdx.x * 256 + threadIdx.x; v * 4 < mn; v += (long long)gridDim.x * 256) {
        const long long e = v * 4;  // N % 4 == 0 on this path
        float4          s = *reinterpret_cast<const float4*>(part + e);
        for (int p = 1; p < splits; ++p) {
            const float4 t = *reinterpret_cast<const float4*>(part + (long long)p * mn + e);
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        const long long m = e / N, n = e - m * N;
        s.x *= alpha; s.y *= alpha; s.z *= alpha; s.w *= alpha;
        if (bias) {
            s.x += h2f(bias[n]); s.y += h2f(bias[n + 1]); s.z += h2f(bias[n + 2]); s.w += h2f(bias[n + 3]);
        }
        const uint16_t h0 = f2h(s.x), h1 = f2h(s.y), h2 = f2h(s.z), h3 = f2h(s.w);
        *reinterpret_cast<uint2*>(C + m * ldc + n) =
            make_uint2((unsigned)h0 | ((unsigned)h1 << 16), (unsigned)h2 | ((unsigned)h3 << 16));
        bad |= half_nonfinite(h0) | half_nonfinite(h1) | half_nonfinite(h2) | half_nonfinite(h3);
    }
    if (found_inf && __any(bad)) {
        if ((threadIdx.x & 63) == 0) atomicOr(found_inf, 1);
    }
}

// Scalar kernel with the same contract, for shapes/alignments the matrix-core path does not take.
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmArgs g, int a_kc, int b_kc) {
    const long long mn  = (long long)g.M * g.N;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    bool            bad = false;
    if (idx < mn) {
        const int       m = (int)(idx / g.N), n = (int)(idx - (long long)m * g.N);
        const int       bo = blockIdx.y / g.batch_inner, bi = blockIdx.y - bo * g.batch_inner;
        const uint16_t* A = g.A + bo * g.sa_o + bi * g.sa_i;
        const uint16_t* B = g.B + bo * g.sb_o + bi * g.sb_i;
        float           acc = 0.f;
        for (int k = 0; k < g.K; ++k) {
            const float a = h2f(a_kc ? A[(long long)m * g.lda + k] : A[(long long)k * g.lda + m]);
            const float b = h2f(b_kc ? B[(long long)n * g.ldb + k] : B[(long long)k * g.ldb + n]);
            acc += a * b;
        }
        acc *= g.alpha;
        if (g.acc_in) acc += g.acc_in[(long long)m * g.N + n];
        if (g.C32) {
            g.C32[(long long)m * g.N + n] = acc;
        } else {
            if (g.bias) acc += h2f(g.bias[n]);
            if (g.relu) acc = (acc < 0.f) ? 0.f : acc;  // keeps a NaN, like the definition max(x, 0) on the reals extended by NaN
            uint16_t        h = f2h(acc);
            const long long coff = bo * g.sc_o + bi * g.sc_i;
            if (g.relu_src) {
                if (!(h2f(g.relu_src[coff + (long long)m * g.ld_aux + n]) > 0.f)) h = 0;
            } else if (g.add) {
                h = f2h(h2f(h) + h2f(g.add[coff + (long long)m * g.ld_aux + n]));
            }
            g.C[coff + (long long)m * g.ldc + n] = h;
            bad = half_nonfinite(h);
        }
    }
    if (g.found_inf && __any(bad)) {
        if ((threadIdx.x & 63) == 0) atomicOr(g.found_inf, 1);
    }
}

// ------------------------------------------------------------------------------------ host side
struct TileCfg {
    int   bm, bn;
    float eff;  // relative per-flop efficiency of the tile shape (bigger tiles reuse LDS data more)
};
static const TileCfg kTiles[] = {{256, 256, 1.00f}, {256, 128, 0.85f}, {128, 256, 0.85f}, {128, 128, 0.65f},
                                 {128, 64, 0.45f},  {64, 128, 0.45f},  {64, 64, 0.30f},   {32, 128, 0.25f},
                                 // only when both operands are stored contraction-contiguous (the transposing loader
                                 // wants a power-of-two tile edge): fills the chip evenly when N is a multiple of 192 only
                                 {256, 192, 0.88f}};
constexpr int   kTileKcOnly = 8;  // first index of the shapes restricted to that operand layout
constexpr int   kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
constexpr int   kCUs      = 256;

struct Plan {
    int tile, splits, k_per_split;
};
static int g_force_tile = -1, g_force_splits = 1;

// Which products take the direct-to-LDS kernels (mp_gemm_tuning_dtl): 0 = none, 1 (default) = weight-gradient products
// (both operands output-contiguous), 2 = every product they are built for.
static int g_dtl_mode = 1;
static int dtl_mode() { return g_dtl_mode; }

// Pick the tile shape (and split count when allowed) that minimises an estimate of run time:
// rounds of 256 workgroups x work per workgroup / shape efficiency.
static Plan make_plan(int M, int N, int K, long long batches, bool allow_split, bool kc_kc = false) {
    // tuning aid (mp_gemm_tuning_override): force a tile shape / split count
    if (g_force_tile >= 0) {
        int t = g_force_tile < (kc_kc ? kNumTiles : kTileKcOnly) ? g_force_tile : 0, sp = allow_split ? g_force_splits : 1;
        if (sp < 1) sp = 1;
        if (sp > 16) sp = 16;
        // every split must own at least one k-tile: (sp - 1) * k_per_split < K, as in the planner's own search
        int kps = ((K + sp - 1) / sp + BK - 1) / BK * BK;
        while (sp > 1 && (long long)(sp - 1) * kps >= K) {
            --sp;
            kps = ((K + sp - 1) / sp + BK - 1) / BK * BK;
        }
        return Plan{t, sp, kps > 0 ? kps : BK};
    }
    Plan   best{0, 1, 0};
    double best_cost = 1e300;
    for (int t = 0; t < (kc_kc ? kNumTiles : kTileKcOnly); ++t) {
        const long long tm = (M + kTiles[t].bm - 1) / kTiles[t].bm, tn = (N + kTiles[t].bn - 1) / kTiles[t].bn;
        const long long tiles = tm * tn * batches;
        const int       max_s = allow_split ? 16 : 1;
        for (int s = 1; s <= max_s; s *= 2) {
            const int kps = ((K + s - 1) / s + BK - 1) / BK * BK;
            if (s > 1 && (kps < 4 * BK || (long long)(s - 1) * kps >= K)) break;
            const long long wgs    = tiles * s;
            const long long rounds = (wgs + kCUs - 1) / kCUs;
            double cost = (double)rounds * kTiles[t].bm * kTiles[t].bn * ((double)kps + 2.0 * BK) / kTiles[t].eff;
            if (s > 1) cost += (double)M * N * s * 6.0;  // writing and re-reading fp32 partials
            if (cost < best_cost) {
                best_cost = cost;
                best      = Plan{t, s, kps};
            }
        }
    }
    if (best.splits == 1) best.k_per_split = (K + BK - 1) / BK * BK;
    if (best.k_per_split == 0) best.k_per_split = BK;
    return best;
}

static bool fast_path_ok(const GemmArgs& g) {
    auto m8 = [](long long v) { return (v & 7) == 0; };
    if (!aligned16(g.A) || !aligned16(g.B)) return false;
    if (g.C && !aligned16(g.C)) return false;
    if (!m8(g.lda) || !m8(g.ldb) || !m8(g.ldc)) return false;
    if (!m8(g.sa_o) || !m8(g.sa_i) || !m8(g.sb_o) || !m8(g.sb_i) || !m8(g.sc_o) || !m8(g.sc_i)) return false;
    if ((g.relu_src || g.add) && (!m8(g.ld_aux) || !aligned16(g.relu_src) || !aligned16(g.add))) return false;
    if (g.bias && !aligned16(g.bias)) return false;
    if ((g.N & 7) != 0) return false;  // the epilogue moves 8 columns at a time
    if ((g.acc_in || g.C32) && (!aligned16(g.acc_in) || !aligned16(g.C32))) return false;
    return true;
}

// ws: split-K partial buffer (may be NULL when !allow_split).
static int run_gemm(GemmArgs g, bool a_kc, bool b_kc, long long batches, bool allow_split, float* ws, size_t ws_floats,
                    hipStream_t hs) {
    if (g.M == 0 || g.N == 0 || batches == 0) return MP_OK;
    if (!fast_path_ok(g) || batches > 65535 || g.K == 0) {
        if (batches > 65535) {
            set_error("gemm: more than 65535 batches");
            return MP_E_UNSUPPORTED;
        }
        const long long mn = (long long)g.M * g.N;
        g.k_per_split      = g.K;
        hipLaunchKernelGGL(gemm_generic_kernel, dim3((unsigned)((mn + 255) / 256), (unsigned)batches), dim3(256), 0, hs, g,
                           (int)a_kc, (int)b_kc);
        MP_LAUNCH_CHECK("gemm (generic)");
        return MP_OK;
    }
    Plan p = make_plan(g.M, g.N, g.K, batches, allow_split && ws != nullptr && (g.N & 3) == 0 && batches == 1, a_kc && b_kc);
    if (p.splits > 1 && (size_t)p.splits * g.M * g.N > ws_floats) p = make_plan(g.M, g.N, g.K, batches, false, a_kc && b_kc);
    g.k_per_split = p.k_per_split;
    g.tiles_m     = (g.M + kTiles[p.tile].bm - 1) / kTiles[p.tile].bm;
    g.tiles_n     = (g.N + kTiles[p.tile].bn - 1) / kTiles[p.tile].bn;
    // persistent along x: at most as many workgroups as fit on the chip at once (a multiple of 8, see the tile
    // mapping); batches and splits keep their own grid dimensions
    const int  ntiles   = g.tiles_m * g.tiles_n;
    const int  lds_kib  = 2 * (kTiles[p.tile].bm + kTiles[p.tile].bn) * 128 / 1024;
    const int  resident = kCUs * (lds_kib > 80 ? 1 : 2);
    const long long others = batches * p.splits;
    const int  gx = (others == 1 && ntiles > resident) ? resident : ntiles;
    const dim3 grid((unsigned)gx, (unsigned)batches, (unsigned)p.splits);

    // interior, unbatched, unsplit problems on the large tiles: operands go straight from global memory into LDS
    // (built for all three operand layouts, used where it is the faster one: both operands output-contiguous, i.e. the
    // weight gradients.  A contraction-contiguous operand arrives there in 64-byte row pieces, which costs what the
    // saved LDS stores gain, so forward and input-gradient products stay on the register-staged kernel)
    const int bm = kTiles[p.tile].bm, bn = kTiles[p.tile].bn;
    if (dtl_mode() != 0 && others == 1 && bm >= 128 && bn >= 128 && g.M % bm == 0 && g.N % bn == 0 && g.K % DK == 0 && g.K >= DK &&
        (a_kc || !b_kc) && (dtl_mode() == 2 || (!a_kc && !b_kc))) {
        const int gxd = ntiles > kCUs ? kCUs : ntiles;   // one workgroup per compute unit (its ring of stages fills the LDS)
        if (a_kc && b_kc) return launch_dtl_tile<true, true>(p.tile, g, gxd, hs);
        if (a_kc && !b_kc) return launch_dtl_tile<true, false>(p.tile, g, gxd, hs);
        return launch_dtl_tile<false, false>(p.tile, g, gxd, hs);
    }
    GemmArgs k = g;
    if (p.splits > 1) {  // partials to workspace, epilogue (scale, bias, rounding, flag) in the finish kernel
        k.C32       = ws;
        k.C         = nullptr;
        k.found_inf = nullptr;
        k.bias      = nullptr;
    }
    int rc;
    if (a_kc && b_kc) rc = launch_tile<true, true>(p.tile, k, grid, hs);
    else if (a_kc && !b_kc) rc = launch_tile<true, false>(p.tile, k, grid, hs);
    else if (!a_kc && !b_kc) rc = launch_tile<false, false>(p.tile, k, grid, hs);
    else {
        set_error("gemm: operand layout combination not built");
        return MP_E_UNSUPPORTED;
    }
    if (rc != MP_OK) return rc;
    if (p.splits > 1) {
        const long long mn = (long long)g.M * g.N;
        long long       nb = (mn / 4 + 255) / 256;
        if (nb > 4096) nb = 4096;
        hipLaunchKernelGGL(splitk_finish_kernel, dim3((unsigned)nb), dim3(256), 0, hs, ws, p.splits, mn, g.N, g.ldc, g.alpha,
                           g.bias, g.C, g.found_inf);
        MP_LAUNCH_CHECK("gemm (split-K finish)");
    }
    return MP_OK;
}

static int check_desc(const mp_gemm_desc* d, const char* who) {
    MP_REQUIRE(d != nullptr, "%s: desc is NULL", who);
    MP_REQUIRE(d->M >= 0 && d->N >= 0 && d->K >= 0, "%s: negative dimension", who);
    MP_REQUIRE(d->batch_outer >= 1 && d->batch_inner >= 1, "%s: batch counts must be >= 1", who);
    MP_REQUIRE(d->trans_w == 0 || d->trans_w == 1, "%s: trans_w must be 0 or 1", who);
    MP_REQUIRE(d->ldx >= d->K && d->ldy >= d->N && d->ldw >= (d->trans_w ? d->N : d->K),
               "%s: leading dimension smaller than the row length (ldx=%d ldw=%d ldy=%d)", who, d->ldx, d->ldw, d->ldy);
    MP_REQUIRE(d->sx_outer >= 0 && d->sx_inner >= 0 && d->sw_outer >= 0 && d->sw_inner >= 0 && d->sy_outer >= 0 &&
                   d->sy_inner >= 0,
               "%s: negative batch stride", who);
    return MP_OK;
}

static void zero_args(GemmArgs& g) { g = GemmArgs{}; }

}  // namespace mp

using namespace mp;

// fp32 partial-sum floats the weight-gradient product [M,N] with contraction K will use
// (0 when the plan does not split the contraction).
static size_t splitk_floats(int M, int N, int K) {
    if (M <= 0 || N <= 0 || (N & 3) != 0) return 0;
    const Plan p = make_plan(M, N, K, 1, true);
    return p.splits > 1 ? (size_t)p.splits * (size_t)M * (size_t)N : 0;
}

static size_t splitk_floats_any(int M, int N, int K, bool allow, bool kc_kc) {
    if (M <= 0 || N <= 0 || (N & 3) != 0) return 0;
    const Plan p = make_plan(M, N, K, 1, allow, kc_kc);
    return p.splits > 1 ? (size_t)p.splits * (size_t)M * (size_t)N : 0;
}

extern "C" int mp_gemm_tuning_override(int tile, int splits) {
    MP_REQUIRE(tile < kNumTiles, "mp_gemm_tuning_override: tile index %d out of range (%d shapes)", tile, kNumTiles);
    MP_REQUIRE(tile < 0 || (splits >= 0 && splits <= 16), "mp_gemm_tuning_override: splits %d outside 0..16", splits);
    g_force_tile   = tile;
    g_force_splits = splits > 0 ? splits : 1;
    return MP_OK;
}

extern "C" int mp_gemm_tuning_dtl(int mode) {
    MP_REQUIRE(mode >= 0 && mode <= 2, "mp_gemm_tuning_dtl: mode %d outside 0..2", mode);
    g_dtl_mode = mode;
    return MP_OK;
}

extern "C" size_t mp_gemm_bwd_dw_workspace_bytes(const mp_gemm_desc* d, int with_db) {
    if (!d) return 0;
    const int rows = d->trans_w ? d->K : d->N, cols = d->trans_w ? d->N : d->K;
    size_t    b    = 0;
    if (d->batch_outer * (long long)d->batch_inner == 1) b = splitk_floats(rows, cols, d->M) * sizeof(float);
    if (with_db) b += mp_colsum_workspace_bytes(d->M, d->N);
    return b + 256;
}

// A product may split its contraction over grid.z (fp32 partials in `ws`, summed in split order by a finish launch)
// when the epilogue is one the finish launch can do: scale, bias, one rounding, overflow flag.
static bool split_ok(const GemmArgs& g, long long batches, const void* ws) {
    return ws != nullptr && aligned16(ws) && batches == 1 && !g.relu && !g.relu_src && !g.add && !g.acc_in && !g.C32;
}

extern "C" size_t mp_gemm_split_workspace_bytes(const mp_gemm_desc* d) {
    if (!d || d->M <= 0 || d->N <= 0 || d->K <= 0) return 0;
    // the larger of the forward (M x N over K) and dX (M x K over N) plans; 0 when neither would split
    const size_t a = splitk_floats_any(d->M, d->N, d->K, true, d->trans_w == 0);
    const size_t b = splitk_floats_any(d->M, d->K, d->N, true, d->trans_w == 1);
    return (a > b ? a : b) * sizeof(float);
}

extern "C" int mp_gemm_fwd(const mp_gemm_desc* d, const mp_half* X, const mp_half* W, const mp_half* bias,
                           const float* acc_in, mp_half* Y, float* y_f32, mp_stream stream) {
    return mp_gemm_fwd_ws(d, X, W, bias, acc_in, Y, y_f32, nullptr, 0, stream);
}

extern "C" int mp_gemm_fwd_ws(const mp_gemm_desc* d, const mp_half* X, const mp_half* W, const mp_half* bias,
                              const float* acc_in, mp_half* Y, float* y_f32, void* ws, size_t ws_bytes, mp_stream stream) {
    int rc = check_desc(d, "mp_gemm_fwd");
    if (rc) return rc;
    MP_REQUIRE(X && W && (Y || y_f32), "mp_gemm_fwd: NULL operand");
    MP_REQUIRE(d->epilogue >= MP_EPI_NONE && d->epilogue <= MP_EPI_BIAS_RELU, "mp_gemm_fwd: bad epilogue %d", d->epilogue);
    MP_REQUIRE((d->epilogue == MP_EPI_NONE) == (bias == nullptr), "mp_gemm_fwd: bias must be given iff the epilogue uses it");
    MP_REQUIRE(!(y_f32 && d->epilogue != MP_EPI_NONE), "mp_gemm_fwd: y_f32 needs MP_EPI_NONE");
    const long long batches = (long long)d->batch_outer * d->batch_inner;
    MP_REQUIRE(batches == 1 || (!acc_in && !y_f32), "mp_gemm_fwd: acc_in / y_f32 are not available for batched problems");
    GemmArgs g;
    zero_args(g);
    g.A = X; g.B = W; g.C = y_f32 ? nullptr : Y; g.C32 = y_f32; g.acc_in = acc_in; g.bias = bias;
    g.relu = d->epilogue == MP_EPI_BIAS_RELU;
    g.M = d->M; g.N = d->N; g.K = d->K;
    g.lda = d->ldx; g.ldb = d->ldw; g.ldc = d->ldy;
    g.sa_o = d->sx_outer; g.sa_i = d->sx_inner; g.sb_o = d->sw_outer; g.sb_i = d->sw_inner;
    g.sc_o = d->sy_outer; g.sc_i = d->sy_inner;
    g.batch_inner = d->batch_inner; g.alpha = d->alpha;
    const bool sp = split_ok(g, batches, ws);
    return run_gemm(g, true, d->trans_w == 0, batches, sp, sp ? static_cast<float*>(ws) : nullptr, sp ? ws_bytes / sizeof(float) : 0,
                    as_stream(stream));
}

extern "C" int mp_gemm_bwd_dx(const mp_gemm_desc* d, const mp_half* dY, const mp_half* W, const mp_half* relu_src,
                              const mp_half* add, int32_t ld_aux, mp_half* dX, mp_stream stream) {
    return mp_gemm_bwd_dx_ws(d, dY, W, relu_src, add, ld_aux, dX, nullptr, 0, stream);
}

extern "C" int mp_gemm_bwd_dx_ws(const mp_gemm_desc* d, const mp_half* dY, const mp_half* W, const mp_half* relu_src,
                                 const mp_half* add, int32_t ld_aux, mp_half* dX, void* ws, size_t ws_bytes, mp_stream stream) {
    int rc = check_desc(d, "mp_gemm_bwd_dx");
    if (rc) return rc;
    MP_REQUIRE(dY && W && dX, "mp_gemm_bwd_dx: NULL operand");
    MP_REQUIRE(!(relu_src && add), "mp_gemm_bwd_dx: relu_src and add may not both be given");
    MP_REQUIRE(!(relu_src || add) || ld_aux >= d->K, "mp_gemm_bwd_dx: ld_aux=%d smaller than K", ld_aux);
    GemmArgs g;
    zero_args(g);
    g.A = dY; g.B = W; g.C = dX; g.relu_src = relu_src; g.add = add; g.ld_aux = ld_aux;
    g.M = d->M; g.N = d->K; g.K = d->N;
    g.lda = d->ldy; g.ldb = d->ldw; g.ldc = d->ldx;
    g.sa_o = d->sy_outer; g.sa_i = d->sy_inner; g.sb_o = d->sw_outer; g.sb_i = d->sw_inner;
    g.sc_o = d->sx_outer; g.sc_i = d->sx_inner;
    g.batch_inner = d->batch_inner; g.alpha = d->alpha;
    // W[N,K] read as B(n'=k, k'=n) is output-contiguous; W[K,N] is contraction-contiguous.
    const long long batches = (long long)d->batch_outer * d->batch_inner;
    const bool      sp      = split_ok(g, batches, ws);
    return run_gemm(g, true, d->trans_w == 1, batches, sp, sp ? static_cast<float*>(ws) : nullptr, sp ? ws_bytes / sizeof(float) : 0,
                    as_stream(stream));
}

extern "C" int mp_gemm_bwd_dw(const mp_gemm_desc* d, const mp_half* dY, const mp_half* X, mp_half* dW, mp_half* db,
                              mp_scale_state* st, void* ws, size_t ws_bytes, mp_stream stream) {
    int rc = check_desc(d, "mp_gemm_bwd_dw");
    if (rc) return rc;
    MP_REQUIRE(dY && X && dW, "mp_gemm_bwd_dw: NULL operand");
    const long long batches = (long long)d->batch_outer * d->batch_inner;
    MP_REQUIRE(!(db && batches != 1), "mp_gemm_bwd_dw: db is not available for batched problems");
    const size_t need = mp_gemm_bwd_dw_workspace_bytes(d, db != nullptr);
    if (!ws || ws_bytes < need || !aligned16(ws)) {
        set_error("mp_gemm_bwd_dw: 16-byte aligned workspace of %zu bytes needed, %zu given", need, ws_bytes);
        return MP_E_WORKSPACE;
    }
    GemmArgs g;
    zero_args(g);
    g.C = dW; g.found_inf = st ? &st->found_inf : nullptr;
    g.K = d->M;
    g.ldc = d->ldw;
    g.sc_o = d->sw_outer; g.sc_i = d->sw_inner;
    g.batch_inner = d->batch_inner; g.alpha = d->alpha;
    if (!d->trans_w) {  // dW[N,K] = dY^T X
        g.A = dY; g.lda = d->ldy; g.sa_o = d->sy_outer; g.sa_i = d->sy_inner; g.M = d->N;
        g.B = X;  g.ldb = d->ldx; g.sb_o = d->sx_outer; g.sb_i = d->sx_inner; g.N = d->K;
    } else {  // dW[K,N] = X^T dY
        g.A = X;  g.lda = d->ldx; g.sa_o = d->sx_outer; g.sa_i = d->sx_inner; g.M = d->K;
        g.B = dY; g.ldb = d->ldy; g.sb_o = d->sy_outer; g.sb_i = d->sy_inner; g.N = d->N;
    }
    float*       wsf       = static_cast<float*>(ws);
    const size_t sk_floats = batches == 1 ? splitk_floats(g.M, g.N, g.K) : 0;
    rc = run_gemm(g, false, false, batches, sk_floats > 0, sk_floats > 0 ? wsf : nullptr, sk_floats, as_stream(stream));
    if (rc) return rc;
    if (db) {
        char*  cs_ws = static_cast<char*>(ws) + ((sk_floats * sizeof(float) + 255) / 256) * 256;
        size_t cs_b  = ws_bytes - (size_t)(cs_ws - static_cast<char*>(ws));
        return mp_colsum(d->M, d->N, dY, d->ldy, db, st, cs_ws, cs_b, stream);
    }
    return MP_OK;
}

extern "C" int mp_gemm_bwd_dw_grouped(const mp_gemm_group_item* items, int count, mp_scale_state* st, mp_stream stream) {
    MP_REQUIRE(items != nullptr && count >= 1 && count <= GROUP_MAX, "mp_gemm_bwd_dw_grouped: 1..%d items", GROUP_MAX);
    GemmArgs args[GROUP_MAX];
    bool     all256 = true, all128 = true;
    for (int i = 0; i < count; ++i) {
        const mp_gemm_desc* d = &items[i].desc;
        int rc = check_desc(d, "mp_gemm_bwd_dw_grouped");
        if (rc) return rc;
        MP_REQUIRE(items[i].dY && items[i].X && items[i].dW, "mp_gemm_bwd_dw_grouped: item %d has a NULL operand", i);
        GemmArgs& g = args[i];
        zero_args(g);
        g.C = items[i].dW; g.found_inf = st ? &st->found_inf : nullptr;
        g.K = d->M; g.ldc = d->ldw; g.batch_inner = 1; g.alpha = d->alpha;
        if (!d->trans_w) {  // dW[N,K] = dY^T X
            g.A = items[i].dY; g.lda = d->ldy; g.M = d->N;
            g.B = items[i].X;  g.ldb = d->ldx; g.N = d->K;
        } else {  // dW[K,N] = X^T dY
            g.A = items[i].X;  g.lda = d->ldx; g.M = d->K;
            g.B = items[i].dY; g.ldb = d->ldy; g.N = d->N;
        }
        g.k_per_split = g.K;
        const bool ok = d->batch_outer == 1 && d->batch_inner == 1 && fast_path_ok(g) && g.K > 0 && g.K % BK == 0 &&
                        g.M % 128 == 0 && g.N % 128 == 0;
        if (!ok) {
            set_error("mp_gemm_bwd_dw_grouped: item %d is batched, unaligned, or its shape is not a multiple of 128 "
                      "(weights) / 64 (rows); use mp_gemm_bwd_dw", i);
            return MP_E_UNSUPPORTED;
        }
        all256 = all256 && g.M % 256 == 0 && g.N % 256 == 0;
    }
    (void)all128;
    const int bm = all256 ? 256 : 128;
    // longest contraction first, so that the tiles that take longest start first
    int order[GROUP_MAX];
    for (int i = 0; i < count; ++i) order[i] = i;
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && args[order[j]].K > args[order[j - 1]].K; --j) std::swap(order[j], order[j - 1]);
    GroupArgs ga{};
    ga.count = count;
    long long total = 0;
    for (int i = 0; i < count; ++i) {
        GemmArgs g = args[order[i]];
        g.tiles_m  = g.M / bm;
        g.tiles_n  = g.N / bm;
        ga.p[i]          = g;
        ga.tile_start[i] = (int)total;
        total += (long long)g.tiles_m * g.tiles_n;
    }
    MP_REQUIRE(total < (1 << 24), "mp_gemm_bwd_dw_grouped: too many tiles");
    for (int i = count; i <= GROUP_MAX; ++i) ga.tile_start[i] = (int)total;
    // bias gradients: strips of BIAS_COLS columns of dY[M, N], numbered after the product tiles (same item order)
    int strips = 0;
    for (int i = 0; i < count; ++i) {
        const mp_gemm_group_item& it = items[order[i]];
        if (!it.db) continue;
        BiasItem& b = ga.b[ga.nbias];
        b.dY = reinterpret_cast<const unsigned short*>(it.dY);
        b.db = reinterpret_cast<unsigned short*>(it.db);
        b.ld = it.desc.ldy; b.rows = it.desc.M;
        ga.strip_start[ga.nbias++] = strips;
        strips += it.desc.N / BIAS_COLS;      // N is a multiple of 128 here (checked above for either orientation)
    }
    for (int i = ga.nbias; i <= GROUP_MAX; ++i) ga.strip_start[i] = strips;
    bool k32 = true;
    for (int i = 0; i < count; ++i) k32 = k32 && ga.p[i].K % DK == 0;
    if (dtl_mode() != 0 && k32)
        return all256 ? launch_dtl_grouped<256, 256>(ga, kCUs, as_stream(stream)) : launch_dtl_grouped<128, 128>(ga, kCUs, as_stream(stream));
    return all256 ? launch_grouped<256, 256>(ga, kCUs, as_stream(stream)) : launch_grouped<128, 128>(ga, 2 * kCUs, as_stream(stream));
}
