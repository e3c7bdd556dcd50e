// Fused scaled-dot-product self-attention for short sequences (seq_len <= 128, head size 64): one
// workgroup per (sequence, head), scores and probabilities never leave the chip except for the
// fp16 probability matrix the backward pass re-reads.  Same arithmetic and storage points as the
// unfused chain of products (paper Section 3.1: fp16 operands, fp32 accumulation, one RNE per stored
// tensor; softmax is an fp32 island, Section 3.2):
//     s  = RNE16(alpha q k^T)      p  = RNE16(softmax_fp32(s))      ctx = RNE16(p v)
//     dP = RNE16(dctx v^T)         dS = RNE16(p (dP - sum_n dP p))
//     dV = RNE16(p^T dctx)         dQ = RNE16(alpha dS k)           dK = RNE16(alpha dS^T q)
// What is saved is HBM traffic: the unfused chain writes and re-reads the [seq, seq] score-sized
// tensors nine times per layer.
//
// Matrix-core conventions (v_mfma_f32_32x32x16_f16, operands A then B): a lane supplies 8 k-values of row
// lane%32 of each operand, lanes 0-31 and 32-63 (half hf) covering two disjoint k-sets; the result lane
// holds D[i][j] for j = lane%32 and i = 8(r/4) + 4 hf + r%4, r = 0..15.  The k-order inside one
// instruction is free as long as both operands agree, which lets the probability registers of the
// score product feed the next product directly: for 32-key tile t and half-slice s a lane of half hf
// uses keys 32t + 16s + 4hf + {0..3} and 32t + 16s + 8 + 4hf + {0..3}.
#include "common.hpp"

#include <mutex>

namespace mp {

constexpr int AT_THREADS = 256;
constexpr int AT_S       = 128;  // maximum sequence length (keys held per workgroup)
constexpr int AT_D       = 64;   // head size
typedef unsigned u32x4a __attribute__((ext_vector_type(4)));
typedef unsigned u32x2a __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f16x8 as_f16x8(u32x4a v) {
    union { u32x4a u; f16x8 h; } c; c.u = v; return c.h;
}
__device__ __forceinline__ f16x8 join_f16x8(u32x2a lo, u32x2a hi) {
    union { u32x4a u; f16x8 h; } c; c.u = u32x4a{lo.x, lo.y, hi.x, hi.y}; return c.h;
}
__device__ __forceinline__ unsigned pack2(float a, float b) {  // RNE16 of both, one v_cvt_pk_f16_f32
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    typedef float    f2 __attribute__((ext_vector_type(2)));
    const h2 h = __builtin_convertvector(f2{a, b}, h2);
    return __builtin_bit_cast(unsigned, h);
}

// The matrix cores leave a lane (row lane%32, half hf) with packed pairs for columns 8 q + 4 hf + {0,1}, {2,3}.  Given the
// pairs of q = 2c (a0, a1) and q = 2c + 1 (b0, b1), lanes r and r + 32 trade so that each ends up with 8 consecutive
// columns, 16 c + 8 hf ... : 16-byte row pieces instead of 8-byte ones halve the cache accesses of a store.
__device__ __forceinline__ u32x4a gather8(unsigned a0, unsigned a1, unsigned b0, unsigned b1) {
    const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
    const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
    return u32x4a{s0[0], s1[0], s0[1], s1[1]};
}

// 16 bytes = 8 consecutive head-dimension values of row `row` (rows >= rows_valid read as zero)
__device__ __forceinline__ u32x4a load_row8(const uint16_t* base, int ld, int row, int rows_valid, int col) {
    if (row < rows_valid) return *reinterpret_cast<const u32x4a*>(base + (long long)row * ld + col);
    return u32x4a{0u, 0u, 0u, 0u};
}

// ------------------------------------------------------------------------------------ row-major LDS + transposing reads
// Matrices sit in LDS the way they sit in memory (row-major, staged with coalesced 16-byte accesses); whatever a product
// needs transposed comes out of the transposing LDS read (`ds_read_b64_tr_b16`: within 16 lanes, the four lanes
// 4 j .. 4 j + 3 address 8-byte chunks of matrix row k0 + j covering 16 consecutive columns, and lane i gets column i
// of rows k0 .. k0 + 3), two reads per 8-deep matrix-core fragment.
// slot (16-byte piece) swizzles: rows of X are 128 bytes (8 pieces), rows of P / dS 256 bytes (16 pieces).  Both make
// (a) the plain 16-byte fragment reads / stores of 16 consecutive rows at one logical piece and (b) the transposing
// reads, which touch 4 consecutive rows x 4 consecutive pieces, free of bank conflicts.
__device__ __forceinline__ int bx_swz(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }
__device__ __forceinline__ int bp_swz(int m) { return ((m & 3) << 2) | ((m >> 2) & 3); }

// Staging of a [rows_valid x 64] matrix into X in two halves, so that the global loads can be requested a phase ahead
// of the LDS stores: 1024 pieces of 8 columns, 4 per thread, fully coalesced (8 lanes per 128-byte row).
__device__ __forceinline__ void load_rows_x(const uint16_t* M, int ld, int rows_valid, u32x4a (&r4)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int v = threadIdx.x + AT_THREADS * j;
        r4[j]       = load_row8(M, ld, v >> 3, rows_valid, (v & 7) * 8);
    }
}
__device__ __forceinline__ void store_rows_x(char* X, const u32x4a (&r4)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int v = threadIdx.x + AT_THREADS * j;
        const int r = v >> 3, c = v & 7;
        *reinterpret_cast<u32x4a*>(X + r * 128 + ((c ^ bx_swz(r)) << 4)) = r4[j];
    }
}
// plain fragment: columns 16 kk + 8 hf ... of row `row` of X
__device__ __forceinline__ f16x8 x_frag(const char* X, int row, int kk, int hf) {
    return as_f16x8(*reinterpret_cast<const u32x4a*>(X + row * 128 + (((2 * kk + hf) ^ bx_swz(row)) << 4)));
}
typedef short s16x4a __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x2a lds_tr(const char* p) {
    const s16x4a v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4a*)((__attribute__((address_space(3))) void*)p));
    return __builtin_bit_cast(u32x2a, v);
}
// Transposed fragment of X (matrix rows = contraction index): for output row (column of X) col0 + lane % 32, the 4 + 4
// contraction indices k_lo .. k_lo + 3 and k_hi .. k_hi + 3.
__device__ __forceinline__ f16x8 x_frag_t(const char* X, int col0, int k_lo, int k_hi, int lane) {
    const int i16 = lane & 15, kq = i16 >> 2, c = col0 + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
    const int r0 = k_lo + kq, r1 = k_hi + kq;
    const u32x2a lo = lds_tr(X + r0 * 128 + (((c >> 3) ^ bx_swz(r0)) << 4) + (c & 4) * 2);
    const u32x2a hi = lds_tr(X + r1 * 128 + (((c >> 3) ^ bx_swz(r1)) << 4) + (c & 4) * 2);
    return join_f16x8(lo, hi);
}
// The same out of a [128][128] query-major matrix (P or dS): output row = key n0 + lane % 32, contraction over queries.
__device__ __forceinline__ f16x8 p_frag_t(const char* Pm, int n0, int k_lo, int k_hi, int lane) {
    const int i16 = lane & 15, kq = i16 >> 2, c = n0 + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
    const int r0 = k_lo + kq, r1 = k_hi + kq;
    const u32x2a lo = lds_tr(Pm + r0 * 256 + (((c >> 3) ^ bp_swz(r0)) << 4) + (c & 4) * 2);
    const u32x2a hi = lds_tr(Pm + r1 * 256 + (((c >> 3) ^ bp_swz(r1)) << 4) + (c & 4) * 2);
    return join_f16x8(lo, hi);
}

// scores / dP tile product for one wave: D[n][m] = sum_d Arows[n][d] * Brows[m][d]; the key-side operand A (all 128
// rows, used by every wave) comes from its staged copy in LDS (plain fragments: the contraction index is the
// column), the query-side operand B (this wave's 32 rows, used once) straight from global memory;
// m = 32 wave + lane % 32, n over four 32-key tiles.
__device__ __forceinline__ void rows_product(const char* An_lds, const uint16_t* Bm, int ldb, int S, int wave, int lane,
                                             f32x16 (&acc)[4]) {
    const int hf = lane >> 5, m = 32 * wave + (lane & 31);
    f16x8     bq[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) bq[kk] = as_f16x8(load_row8(Bm, ldb, m, S, 16 * kk + 8 * hf));
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        acc[t] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (32 * t < S) {  // wave-uniform
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x_frag(An_lds, 32 * t + (lane & 31), kk, hf), bq[kk], acc[t], 0, 0, 0);
        }
    }
}

// ------------------------------------------------------------------------------------ forward
__global__ __launch_bounds__(AT_THREADS, 4) void attention_fwd_kernel(int n_heads, int S, const uint16_t* __restrict__ qkv,
                                                                    int ld, int d_model, float alpha,
                                                                    uint16_t* __restrict__ P, uint16_t* __restrict__ ctx,
                                                                    int ld_ctx) {
    extern __shared__ __align__(16) char smem[];  // the rows of V (16 KB), then the rows of K (16 KB)
    char* Krows = smem + 128 * 128;
    const int b = blockIdx.x / n_heads, h = blockIdx.x - b * n_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hf = lane >> 5;
    const uint16_t* q = qkv + (long long)b * S * ld + h * AT_D;
    const uint16_t* k = q + d_model;
    const uint16_t* v = q + 2 * d_model;
    uint16_t*       Pb = P + (long long)blockIdx.x * S * S;

    {
        u32x4a rk[4], rv[4];
        load_rows_x(k, ld, S, rk);
        load_rows_x(v, ld, S, rv);
        store_rows_x(Krows, rk);
        store_rows_x(smem, rv);
    }
    __syncthreads();                   // rows of K and V complete

    f32x16 acc[4];
    rows_product(Krows, q, ld, S, wave, lane, acc);

    // softmax over the keys of query m; a lane holds 64 of its 128 scores, lane^32 the others
    const int m  = 32 * wave + (lane & 31);
    float     mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int   n = 32 * t + 8 * (r >> 2) + 4 * hf + (r & 3);
            const float s = (n < S) ? round16(alpha * acc[t][r]) : -INFINITY;
            acc[t][r]     = s;
            mx            = fmaxf(mx, s);
        }
    mx        = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float e = __expf(acc[t][r] - mx);  // exp(-inf) = 0 for masked keys
            acc[t][r]     = e;
            sum += e;
        }
    sum += __shfl_xor(sum, 32, 64);
    const float inv = 1.0f / sum;  // one division per query (the kernel is bound by vector ALU work); e * inv is within
                                   // one fp32 ulp of e / sum, far inside the rounding to fp16 that follows
    unsigned pk[4][8];  // probabilities as fp16 pairs: pk[t][2q], pk[t][2q+1] = keys 32t + 8q + 4hf + {0,1},{2,3}
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            pk[t][2 * qd]     = pack2(acc[t][4 * qd] * inv, acc[t][4 * qd + 1] * inv);
            pk[t][2 * qd + 1] = pack2(acc[t][4 * qd + 2] * inv, acc[t][4 * qd + 3] * inv);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const u32x4a row8 = gather8(pk[t][4 * c], pk[t][4 * c + 1], pk[t][4 * c + 2], pk[t][4 * c + 3]);
            const int    n    = 32 * t + 16 * c + 8 * hf;  // (S is a multiple of 8: a piece is inside or outside as a whole)
            if (m < S && n < S) *reinterpret_cast<u32x4a*>(Pb + (long long)m * S + n) = row8;
        }
    }

    // ctx[m][d] = sum_n p[m][n] v[n][d]: A = V^T rows d out of the rows of V, B = probability registers
    f32x16 o[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
        o[dt] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (32 * t < S) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const f16x8 pv = as_f16x8(u32x4a{pk[t][4 * s], pk[t][4 * s + 1], pk[t][4 * s + 2], pk[t][4 * s + 3]});
                    const int   n0 = 32 * t + 16 * s + 4 * hf;  // the registers' key order: 4 keys here, 4 more 8 further
                    const f16x8 vt = x_frag_t(smem, 32 * dt, n0, n0 + 8, lane);
                    o[dt]          = __builtin_amdgcn_mfma_f32_32x32x16_f16(vt, pv, o[dt], 0, 0, 0);
                }
            }
        }
    }
    if (m < S) {
        uint16_t* crow = ctx + ((long long)b * S + m) * ld_ctx + h * AT_D;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int q0 = 8 * c;  // accumulator registers of the column groups q = 2c, 2c + 1
                *reinterpret_cast<u32x4a*>(crow + 32 * dt + 16 * c + 8 * hf) =
                    gather8(pack2(o[dt][q0], o[dt][q0 + 1]), pack2(o[dt][q0 + 2], o[dt][q0 + 3]),
                            pack2(o[dt][q0 + 4], o[dt][q0 + 5]), pack2(o[dt][q0 + 6], o[dt][q0 + 7]));
            }
    }
}

// ------------------------------------------------------------------------------------ backward
// Every matrix sits in LDS the way it sits in memory (row-major, staged with coalesced 16-byte accesses); whatever a
// product needs transposed comes out of the transposing LDS read (`ds_read_b64_tr_b16`: within 16 lanes, the four
// lanes 4 j .. 4 j + 3 address 8-byte chunks of matrix row k0 + j covering 16 consecutive columns, and lane i gets
// column i of rows k0 .. k0 + 3), two reads per 8-deep matrix-core fragment.  No 2-byte LDS scatters, no transposing
// stagings.
// LDS: one [128][128] query-major buffer (32 KB) that holds P for the dV product and then dS for the dK product, plus one
// [128][64] buffer X (16 KB) that holds the rows of V (dP), dO (dV), K (dQ) and Q (dK) in turn: 48 KiB; the matrix that
// X takes next is always already on its way from memory in registers.  Two workgroups share a CU: the registers, not
// the LDS, set that (a third workgroup per CU would leave 168 registers per lane, and the spills that costs took the
// kernel from 36 to 65 us per layer).
constexpr int AT_BWD_LDS = 128 * 256 + 128 * 128;

__global__ __launch_bounds__(AT_THREADS, 2) void attention_bwd_kernel(int n_heads, int S, const uint16_t* __restrict__ qkv,
                                                                       int ld, int d_model, float alpha,
                                                                       const uint16_t* __restrict__ P,
                                                                       const uint16_t* __restrict__ dctx, int ld_ctx,
                                                                       uint16_t* __restrict__ dqkv, int ld_dqkv) {
    extern __shared__ __align__(16) char smem[];
    char* PS = smem;                 // [128][128] query-major: P for the dV product, then dS for the dK product
    char* X  = PS + 128 * 256;       // [128][64]: rows of V (dP), dO (dV), K (dQ), Q (dK), one after the other
    const int b = blockIdx.x / n_heads, h = blockIdx.x - b * n_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hf = lane >> 5;
    const uint16_t* q  = qkv + (long long)b * S * ld + h * AT_D;
    const uint16_t* k  = q + d_model;
    const uint16_t* v  = q + 2 * d_model;
    const uint16_t* dO = dctx + (long long)b * S * ld_ctx + h * AT_D;
    const uint16_t* Pb = P + (long long)blockIdx.x * S * S;
    uint16_t*       dq = dqkv + (long long)b * S * ld_dqkv + h * AT_D;
    uint16_t*       dk = dq + d_model;
    uint16_t*       dv = dq + 2 * d_model;
    const int       m  = 32 * wave + (lane & 31);

    // this lane's pieces of its query's probabilities
    u32x4a pw[4][2];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int n8 = 32 * t + 16 * c + 8 * hf;  // 16 bytes = keys n8 .. n8 + 7 of query m
            pw[t][c]     = u32x4a{0u, 0u, 0u, 0u};
            if (m < S && n8 < S) pw[t][c] = *reinterpret_cast<const u32x4a*>(Pb + (long long)m * S + n8);
        }
    u32x4a ra[4], rb[4];            // the matrix X takes next is requested a phase ahead
    load_rows_x(v, ld, S, ra);
    f16x8 bq[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) bq[kk] = as_f16x8(load_row8(dO, ld_ctx, m, S, 16 * kk + 8 * hf));
    load_rows_x(dO, ld_ctx, S, rb);
    store_rows_x(X, ra);            // rows of V
#pragma unroll
    for (int t = 0; t < 4; ++t)     // P goes into LDS as it comes from memory (query-major, 16-byte pieces)
#pragma unroll
        for (int c = 0; c < 2; ++c) *reinterpret_cast<u32x4a*>(PS + m * 256 + (((4 * t + 2 * c + hf) ^ bp_swz(m)) << 4)) = pw[t][c];
    __syncthreads();

    // dP[m][n] = sum_d dctx[m][d] v[n][d], same register layout as the scores (lane <-> query m)
    f32x16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        acc[t] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (32 * t < S) {  // wave-uniform
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x_frag(X, 32 * t + (lane & 31), kk, hf), bq[kk], acc[t], 0, 0, 0);
        }
    }
    __syncthreads();                // every wave is done with the rows of V
    store_rows_x(X, rb);            // the rows of dO
    load_rows_x(k, ld, S, ra);      // for the dQ product: on their way during the dS arithmetic and the dV product

    // dS = RNE16(p (dP - inner)), inner = sum_n dP p, in registers: lanes m and m + 32 trade halves of their pieces
    // (gather8 is its own inverse) and hold keys 8 q + 4 hf + {0..3} for q = 2c (words 0, 1) and q = 2c + 1 (words 2, 3)
    unsigned ds[4][8];
    {
        // this lane's own pieces of P come back out of LDS (it wrote them there itself) rather than waiting in registers
        auto own_p = [&](int t, int c) {
            const u32x4a w = *reinterpret_cast<const u32x4a*>(PS + m * 256 + (((4 * t + 2 * c + hf) ^ bp_swz(m)) << 4));
            return gather8(w[0], w[1], w[2], w[3]);
        };
        auto prob = [&](const u32x4a& w, int e) { return h2f((uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xFFFFu))); };
        float inner = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const u32x4a w = own_p(t, c);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int   r  = 8 * c + e;  // = 4 qd + (e % 4) with qd = 2c + e / 4
                    const float dp = round16(acc[t][r]);  // dP is a stored tensor
                    acc[t][r]      = dp;
                    inner += dp * prob(w, e);
                }
            }
        inner += __shfl_xor(inner, 32, 64);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const u32x4a w = own_p(t, c);  // (again: cheaper than keeping 64 floats)
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const int r       = 8 * c + e;
                    ds[t][4 * c + e / 2] = pack2(prob(w, e) * (acc[t][r] - inner), prob(w, e + 1) * (acc[t][r + 1] - inner));
                }
            }
    }
    __syncthreads();                // rows of dO (and P) complete

    // The 32 keys n of this wave, contraction over queries m in plain order (8 at 16 kk + 8 hf):
    //   dV[n][d] = sum_m p[m][n] dctx[m][d]          A = dO^T rows d out of the rows of dO, B = P^T rows n out of P
    //   dK[n][d] = alpha sum_m dS[m][n] q[m][d]      A = Q^T  rows d out of the rows of Q,  B = dS^T rows n out of dS
    auto key_product = [&](uint16_t* out, const float scale) {
        if (32 * wave < S) {  // wave-uniform
            f32x16 o[2];
            o[0] = o[1] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            // fragments of slice kk + 1 are requested before the matrix-core work of slice kk, and no further ahead
            f16x8 fb[2], fa[2][2];
            auto  fetch = [&](int kk, int buf) {
                const int m0 = 16 * kk + 8 * hf;  // (rows >= S of P / dS and of X hold zeros)
                fb[buf]      = p_frag_t(PS, 32 * wave, m0, m0 + 4, lane);
                fa[buf][0]   = x_frag_t(X, 0, m0, m0 + 4, lane);
                fa[buf][1]   = x_frag_t(X, 32, m0, m0 + 4, lane);
            };
            fetch(0, 0);
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                if (16 * kk < S) {
                    if (kk + 1 < 8) fetch(kk + 1, (kk + 1) & 1);
                    o[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[kk & 1][0], fb[kk & 1], o[0], 0, 0, 0);
                    o[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[kk & 1][1], fb[kk & 1], o[1], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            const int n = 32 * wave + (lane & 31);
            if (n < S) {
                uint16_t* row = out + (long long)n * ld_dqkv;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const int q0 = 8 * c;
                        *reinterpret_cast<u32x4a*>(row + 32 * dt + 16 * c + 8 * hf) =
                            gather8(pack2(scale * o[dt][q0], scale * o[dt][q0 + 1]), pack2(scale * o[dt][q0 + 2], scale * o[dt][q0 + 3]),
                                    pack2(scale * o[dt][q0 + 4], scale * o[dt][q0 + 5]), pack2(scale * o[dt][q0 + 6], scale * o[dt][q0 + 7]));
                    }
            }
        }
    };
    key_product(dv, 1.0f);

    __syncthreads();                // every wave is done with P and the rows of dO
    store_rows_x(X, ra);            // the rows of K
#pragma unroll
    for (int t = 0; t < 4; ++t)     // dS over P, traded back into 8 consecutive keys per lane
#pragma unroll
        for (int c = 0; c < 2; ++c)
            *reinterpret_cast<u32x4a*>(PS + m * 256 + (((4 * t + 2 * c + hf) ^ bp_swz(m)) << 4)) =
                gather8(ds[t][4 * c], ds[t][4 * c + 1], ds[t][4 * c + 2], ds[t][4 * c + 3]);
    load_rows_x(q, ld, S, rb);      // for the dK product: on their way during the dQ product
    __syncthreads();                // rows of K and dS complete

    // dQ[m][d] = alpha sum_n dS[m][n] k[n][d]: A = K^T rows d out of the rows of K (keys in the registers' order: 4 at
    // 32 t + 16 s + 4 hf and 4 more 8 further), B = dS registers
    {
        f32x16 o[2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
            o[dt] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (32 * t < S) {
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const f16x8 dsf = as_f16x8(u32x4a{ds[t][4 * s], ds[t][4 * s + 1], ds[t][4 * s + 2], ds[t][4 * s + 3]});
                        const int   n0  = 32 * t + 16 * s + 4 * hf;
                        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x_frag_t(X, 32 * dt, n0, n0 + 8, lane), dsf, o[dt], 0, 0, 0);
                    }
                }
            }
        }
        if (m < S) {
            uint16_t* row = dq + (long long)m * ld_dqkv;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int q0 = 8 * c;
                    *reinterpret_cast<u32x4a*>(row + 32 * dt + 16 * c + 8 * hf) =
                        gather8(pack2(alpha * o[dt][q0], alpha * o[dt][q0 + 1]), pack2(alpha * o[dt][q0 + 2], alpha * o[dt][q0 + 3]),
                                pack2(alpha * o[dt][q0 + 4], alpha * o[dt][q0 + 5]), pack2(alpha * o[dt][q0 + 6], alpha * o[dt][q0 + 7]));
                }
        }
    }
    __syncthreads();                // every wave is done with the rows of K
    store_rows_x(X, rb);            // the rows of Q
    __syncthreads();
    key_product(dk, alpha);
}

}  // namespace mp

using namespace mp;

static int attention_check(const char* who, int n_seq, int n_heads, int S, int d_head, const void* qkv, int ld,
                           const void* p, const void* ctx, int ld_ctx) {
    MP_REQUIRE(n_seq > 0 && n_heads > 0 && S > 0 && d_head > 0, "%s: bad shape", who);
    MP_REQUIRE(qkv && p && ctx, "%s: NULL argument", who);
    if (d_head != AT_D || S > AT_S || (S & 7) != 0) {
        set_error("%s: the fused kernel needs head size %d and seq_len a multiple of 8 up to %d (got %d, %d); "
                  "use the unfused chain of mp_gemm_* and mp_softmax_* calls instead", who, AT_D, AT_S, d_head, S);
        return MP_E_UNSUPPORTED;
    }
    const int d_model = n_heads * d_head;
    MP_REQUIRE(ld >= 3 * d_model && (ld & 7) == 0 && ld_ctx >= d_model && (ld_ctx & 7) == 0,
               "%s: leading dimensions must cover the row and be multiples of 8", who);
    MP_REQUIRE(aligned16(qkv) && aligned16(p) && aligned16(ctx), "%s: pointers must be 16-byte aligned", who);
    MP_REQUIRE((long long)n_seq * n_heads < (1ll << 31), "%s: too many (sequence, head) pairs", who);
    return MP_OK;
}

extern "C" int mp_attention_fwd(int n_seq, int n_heads, int seq_len, int d_head, const mp_half* qkv, int ld_qkv,
                                float alpha, mp_half* p, mp_half* ctx, int ld_ctx, mp_stream stream) {
    int rc = attention_check("mp_attention_fwd", n_seq, n_heads, seq_len, d_head, qkv, ld_qkv, p, ctx, ld_ctx);
    if (rc) return rc;
    hipLaunchKernelGGL(attention_fwd_kernel, dim3(n_seq * n_heads), dim3(AT_THREADS), 64 * 256 + 128 * 128, as_stream(stream), n_heads,
                       seq_len, qkv, ld_qkv, n_heads * d_head, alpha, p, ctx, ld_ctx);
    MP_LAUNCH_CHECK("mp_attention_fwd");
    return MP_OK;
}

extern "C" int mp_attention_bwd(int n_seq, int n_heads, int seq_len, int d_head, const mp_half* qkv, int ld_qkv,
                                float alpha, const mp_half* p, const mp_half* dctx, int ld_ctx, mp_half* dqkv,
                                int ld_dqkv, mp_stream stream) {
    int rc = attention_check("mp_attention_bwd", n_seq, n_heads, seq_len, d_head, qkv, ld_qkv, p, dctx, ld_ctx);
    if (rc) return rc;
    MP_REQUIRE(dqkv && aligned16(dqkv) && ld_dqkv >= 3 * n_heads * d_head && (ld_dqkv & 7) == 0,
               "mp_attention_bwd: bad dqkv / ld_dqkv");
    static std::once_flag once;
    static hipError_t     attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_bwd_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, AT_BWD_LDS);
    });
    if (attr_err != hipSuccess) return hip_fail(attr_err, "mp_attention_bwd: hipFuncSetAttribute(LDS size)");
    hipLaunchKernelGGL(attention_bwd_kernel, dim3(n_seq * n_heads), dim3(AT_THREADS), AT_BWD_LDS, as_stream(stream), n_heads,
                       seq_len, qkv, ld_qkv, n_heads * d_head, alpha, p, dctx, ld_ctx, dqkv, ld_dqkv);
    MP_LAUNCH_CHECK("mp_attention_bwd");
    return MP_OK;
}
