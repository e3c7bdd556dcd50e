// fp16 x fp16 -> fp32-accumulate contractions on the gfx950 matrix cores (the arithmetic of the paper's
// Section 3.1: half-precision operands, single-precision sums), with one RNE rounding to fp16 in the
// epilogue.
//
// One kernel template serves forward, input-gradient and weight-gradient products.  Internally a
// problem is  C[M,N] = alpha * sum_k A(m,k) B(n,k)  where each operand is either
//   KC ("contraction-contiguous"):  A(m,k) = A[m*lda + k]
//   OC ("output-contiguous")     :  A(m,k) = A[k*lda + m]
// Tiles are staged through LDS in a k-contiguous, XOR-swizzled layout (rows of 64 halves =
// 8 x 16-byte slots, slot index ^ f(row)), so that every matrix-core operand fragment is one
// 16-byte LDS read per lane whatever the global layout; OC operands are transposed 8x8 in
// registers (byte-permute instructions) between the global load and the LDS store.
//
// Matrix-core instruction: v_mfma_f32_32x32x16_f16.  The order of the 16 k-values inside one
// instruction is irrelevant as long as both operands use the same one (a sum over k), so both
// fragments are simply "8 consecutive k of one row".  Operands are issued swapped (B-tile rows as
// the instruction's first operand), which makes each lane own 4 consecutive output columns of one
// output row and allows 8-byte epilogue accesses:
//     lane l, accumulator register r  ->  row m = l % 32,  col n = 8*(r/4) + 4*(l/32) + r%4.
#pragma once
#include "common.hpp"

#include <mutex>
#include <type_traits>
#include <utility>

namespace mp {

constexpr int GEMM_THREADS = 256;
constexpr int BK           = 64;  // halves per LDS row = 128 bytes = 8 slots of 16 bytes
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct GemmArgs {
    const uint16_t* A;
    const uint16_t* B;
    uint16_t*       C;
    float*          C32;       // fp32 output (raw accumulator): y_f32 or split-K partials; ld = N
    const float*    acc_in;    // fp32 addend, ld = N
    const uint16_t* bias;      // [N]
    const uint16_t* relu_src;  // [M,N] ld_aux: zero output where <= 0
    const uint16_t* add;       // [M,N] ld_aux: second rounding after adding
    int*            found_inf;
    int             M, N, K;
    int             lda, ldb, ldc, ld_aux;
    long long       sa_o, sa_i, sb_o, sb_i, sc_o, sc_i;
    int             batch_inner;
    int             relu;
    float           alpha;
    int             k_per_split;  // multiple of BK; == K rounded up when not split
    int             tiles_m, tiles_n;
};

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}).
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// One accumulator register read / written where the statement stands.  The accumulators live in the AGPR half of the
// register file; left to itself the compiler copies the whole set into VGPRs ahead of the epilogue's first branch.
__device__ __forceinline__ float acc_get(float a) {
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}
__device__ __forceinline__ float acc_put(float v) {
    float a;
    asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a) : "v"(v));
    return a;
}

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// 16-byte global load of 8 halves starting at p[0], of which only the first `valid` (0..8) exist.
__device__ __forceinline__ u32x4 load8_guard(const uint16_t* p, int valid) {
    if (valid >= 8) return *reinterpret_cast<const u32x4*>(p);
    // ragged tail: element loads, assembled with compile-time indices only (no addressable local)
    unsigned w0 = 0, w1 = 0, w2 = 0, w3 = 0;
    if (valid > 0) w0 |= (unsigned)p[0];
    if (valid > 1) w0 |= (unsigned)p[1] << 16;
    if (valid > 2) w1 |= (unsigned)p[2];
    if (valid > 3) w1 |= (unsigned)p[3] << 16;
    if (valid > 4) w2 |= (unsigned)p[4];
    if (valid > 5) w2 |= (unsigned)p[5] << 16;
    if (valid > 6) w3 |= (unsigned)p[6];
    if (valid > 7) w3 |= (unsigned)p[7] << 16;
    return u32x4{w0, w1, w2, w3};
}

// ---- global -> registers -> LDS.  R = tile rows (BM or BN).  Up to 8 x 16 bytes per lane.
// Addresses are split into a wave-uniform part (tile origin, advanced per k-step; lives in scalar
// registers) and a per-lane part computed once, so the k-loop carries almost no address arithmetic.
// load<false> is straight-line code (no bounds tests) for tiles that lie fully inside the matrix
// and the k-range; load<true> tests every access and zero-fills, and is only taken at the edges.
template <int R>
struct KCLoader {  // operand stored [row][k]; `tile` points at element (row0, k0)
    static constexpr int NV = R / 32;  // vectors per lane (lane -> row tid/8 + 32 i, k-slot tid%8)
    static constexpr int N_LOADS = NV;
    u32x4                v[NV];
    unsigned             lane_off;     // elements from the tile origin
    int                  lds_off[2];   // byte offset inside the LDS tile for even / odd i (before + i*4096)
    __device__ __forceinline__ void init(int ld) {
        const int r0 = threadIdx.x >> 3, kv = threadIdx.x & 7;
        lane_off   = (unsigned)r0 * (unsigned)ld + kv * 8;
        lds_off[0] = r0 * 128 + ((kv ^ swz(r0)) << 4);
        lds_off[1] = r0 * 128 + ((kv ^ swz(r0) ^ 4) << 4);
    }
    template <bool GUARD, int I>
    __device__ __forceinline__ void load_one(const uint16_t* tile, int ld, int rows_left, int k_left) {
        const uint16_t* p = tile + (long long)(32 * I) * ld + lane_off;
        if (GUARD) {
            const int r = (threadIdx.x >> 3) + 32 * I;
            v[I] = (r < rows_left) ? load8_guard(p, k_left - (int)(threadIdx.x & 7) * 8) : u32x4{0u, 0u, 0u, 0u};
        } else {
            v[I] = *reinterpret_cast<const u32x4*>(p);
        }
    }
    template <int I>
    __device__ __forceinline__ void store_one(char* lds) const {
        *reinterpret_cast<u32x4*>(lds + lds_off[I & 1] + I * 4096) = v[I];
    }
    template <bool GUARD>
    __device__ __forceinline__ void load(const uint16_t* tile, int ld, int rows_left, int k_left) {
        static_for<NV>([&](auto ic) { load_one<GUARD, decltype(ic)::value>(tile, ld, rows_left, k_left); });
    }
    __device__ __forceinline__ void store(char* lds) const {
        static_for<NV>([&](auto ic) { store_one<decltype(ic)::value>(lds); });
    }
};

template <int R>
struct OCLoader {  // operand stored [k][row]; `tile` points at element (k0, row0).
    // Every lane owns a KB(k) x 8(row) block of the 64 x R tile, KB = R/32 (8 for R = 256): row group
    // rg = tid % (R/8), k group kg = tid / (R/8).  The block is transposed in registers with byte
    // permutes and written to LDS as 8 row pieces of KB halves.
    static constexpr int G = R / 8, KB = R / 32;
    static constexpr int N_LOADS = KB;
    u32x4    v[KB];
    unsigned lane_off;
    int      lds_row0;  // byte offset of (row rg*8, k kg*KB) before the slot swizzle: row*128 + within-slot bytes
    int      lds_slot;  // (slot of k = kg*KB) ^ (rg & 7); slot(i) = lds_slot ^ i   [swz(rg*8 + i) = (i ^ rg) & 7]
    // Which block a lane owns.  R = 128 stores 8 bytes per lane, and the LDS takes such a store 16 lanes (128 bytes, one
    // pass over its banks) at a time: with rg = tid % 16 the 16 lanes of a pass would share one k group, i.e. the same
    // 8-byte half of their 16-byte slots, and only 8 slots exist per pass: a two-way conflict on every store.  So a
    // pass holds 8 row groups x 2 adjacent k groups (the two halves of a slot) instead.
    static __device__ __forceinline__ int row_group(int t) { return R == 128 ? ((t & 7) | ((t >> 1) & 8)) : t % G; }
    static __device__ __forceinline__ int k_group(int t) { return R == 128 ? (((t >> 3) & 1) | ((t >> 5) << 1)) : t / G; }
    __device__ __forceinline__ void init(int ld) {
        const int rg = row_group(threadIdx.x), kg = k_group(threadIdx.x);
        const int k  = kg * KB;
        lane_off = (unsigned)k * (unsigned)ld + rg * 8;
        lds_row0 = rg * 8 * 128 + (k & 7) * 2;
        lds_slot = ((k >> 3) ^ rg) & 7;
    }
    template <bool GUARD, int J>
    __device__ __forceinline__ void load_one(const uint16_t* tile, int ld, int rows_left, int k_left) {
        const uint16_t* p = tile + (long long)J * ld + lane_off;
        if (GUARD) {
            const int rg = row_group(threadIdx.x), kg = k_group(threadIdx.x);
            v[J] = (kg * KB + J < k_left) ? load8_guard(p, rows_left - rg * 8) : u32x4{0u, 0u, 0u, 0u};
        } else {
            v[J] = *reinterpret_cast<const u32x4*>(p);
        }
    }
    // half (k = j, row I) of the block is the low or high half of word I/2 of v[j]
    template <int I>
    __device__ __forceinline__ unsigned pair(int j0) const {
        const unsigned lo = v[j0][I >> 1], hi = v[j0 + 1][I >> 1];
        return (I & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    }
    template <int I>
    __device__ __forceinline__ void store_row(char* lds) const {
        char* dst = lds + lds_row0 + I * 128 + ((lds_slot ^ I) << 4);
        if constexpr (KB == 8) {
            *reinterpret_cast<u32x4*>(dst) = u32x4{pair<I>(0), pair<I>(2), pair<I>(4), pair<I>(6)};
        } else if constexpr (KB == 4) {
            typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
            *reinterpret_cast<u32x2*>(dst) = u32x2{pair<I>(0), pair<I>(2)};
        } else if constexpr (KB == 2) {
            *reinterpret_cast<unsigned*>(dst) = pair<I>(0);
        } else {
            const unsigned w = v[0][I >> 1];
            *reinterpret_cast<uint16_t*>(dst) = (uint16_t)((I & 1) ? (w >> 16) : (w & 0xFFFFu));
        }
    }
    // store item J of KB covers 8/KB of the block's 8 LDS rows, so that items and loads pair up 1:1
    template <int J>
    __device__ __forceinline__ void store_one(char* lds) const {
        static_for<8 / KB>([&](auto rc) { store_row<J*(8 / KB) + decltype(rc)::value>(lds); });
    }
    template <bool GUARD>
    __device__ __forceinline__ void load(const uint16_t* tile, int ld, int rows_left, int k_left) {
        static_for<KB>([&](auto jc) { load_one<GUARD, decltype(jc)::value>(tile, ld, rows_left, k_left); });
    }
    __device__ __forceinline__ void store(char* lds) const {
        static_for<KB>([&](auto jc) { store_one<decltype(jc)::value>(lds); });
    }
};

template <int R, bool KC>
struct LoaderSel { typedef KCLoader<R> T; };
template <int R>
struct LoaderSel<R, false> { typedef OCLoader<R> T; };

// The operand stream of one workgroup: the two register sets per operand and the wave-uniform position of the next
// k-tile to load.  It outlives a tile.  When the workgroup goes on to another tile of the same problem, the two loads
// that would run past the end of the current tile fetch the first two k-tiles of the next one instead: that tile then
// starts with its k-tile 0 in LDS stage 0 and its k-tile 1 on the way into (la1, lb1) (`primed`), without a prologue,
// and those loads are queued ahead of the current tile's output stores instead of behind them.
template <int BM, int BN, bool A_KC, bool B_KC>
struct OperandStream {
    typename LoaderSel<BM, A_KC>::T la0, la1;
    typename LoaderSel<BN, B_KC>::T lb0, lb1;
    const uint16_t *ta, *tb;  // origin of the next k-tile to load
    int  k_next;              // its first k
    bool primed;
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    u32x2 bias[BN / 16];      // the coming tile's bias values for this lane's columns (4 per entry), when they start the sums
    __device__ __forceinline__ void init(int lda, int ldb) {
        la0.init(lda);
        la1.init(lda);
        lb0.init(ldb);
        lb1.init(ldb);
        ta = tb = nullptr;
        k_next  = 0;
        primed  = false;
    }
};

// ---- epilogue of one wave tile (TM x TN matrix-core tiles of 32 x 32), in the layout the matrix cores leave the result
// in.  mrow = first output row of this lane (row of the wave tile + lane % 32), ncol = first column of the wave tile.
template <int TM, int TN, bool EDGE>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, f32x16 (&acc)[TM][TN], const int mrow, const int ncol,
                                              const int bo, const int bi, const int bz, const bool split,
                                              const bool fold_bias, bool& bad) {
    const int eh = (threadIdx.x & 63) >> 5;
    // ---- epilogue, in the layout the matrix cores leave the result in.  Of the 32x32 tile (i, j) lane
    // (er = lane % 32, eh = lane / 32) holds row er and, for q = 0..3, the 4 consecutive columns 8 q + 4 eh ...
    // (acc[i][j][4 q + c]).  fp32 outputs are stored from there, 16 bytes per lane.  fp16 outputs are converted
    // and packed in pairs, then lanes er and er + 32 trade halves (one cross-half register swap per packed pair)
    // so that each lane ends up with 8 consecutive columns: 16-byte stores, and 16-byte loads of the residual /
    // ReLU-source operand, without a trip through LDS.
    asm volatile("s_nop 15\n\ts_nop 15");  // the last matrix-core results have landed before the explicit accumulator reads
    uint16_t*       C   = g.C ? g.C + bo * g.sc_o + bi * g.sc_i : nullptr;
    const uint16_t* aux = g.relu_src ? g.relu_src : g.add;
    if (aux) aux += bo * g.sc_o + bi * g.sc_i;
    float*     C32   = g.C32 ? g.C32 + (long long)bz * g.M * g.N : nullptr;

    // (N is a multiple of 8 on this path, so a 16-byte piece of a row is either fully inside or fully outside)
    if (C32) {  // raw accumulator out: split-K partial, or fp32 result with alpha and addend
        static_for<TM * TN * 4>([&](auto tc) {
            constexpr int t = decltype(tc)::value, i = t / (TN * 4), j = (t / 4) % TN, q = t % 4;
            const int m = mrow + 32 * i, n = ncol + 32 * j + 8 * q + 4 * eh;
            if (EDGE && (m >= g.M || n >= g.N)) return;
            f32x4 v = {acc_get(acc[i][j][4 * q]), acc_get(acc[i][j][4 * q + 1]), acc_get(acc[i][j][4 * q + 2]), acc_get(acc[i][j][4 * q + 3])};
            const long long mn = (long long)m * g.N + n;
            if (!split) {
                v *= g.alpha;
                if (g.acc_in) v += *reinterpret_cast<const f32x4*>(g.acc_in + mn);
            }
            *reinterpret_cast<f32x4*>(C32 + mn) = v;
        });
    } else {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        typedef float    f32x2 __attribute__((ext_vector_type(2)));
        typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
        // the uncommon terms first, in fp32: scale factor, fp32 addend, a bias that could not start the accumulators
        if (g.alpha != 1.f || g.acc_in || (g.bias && !fold_bias)) {
            static_for<TM * TN * 4>([&](auto tc) {
                constexpr int t = decltype(tc)::value, i = t / (TN * 4), j = (t / 4) % TN, q = t % 4;
                const int m = mrow + 32 * i, n = ncol + 32 * j + 8 * q + 4 * eh;
                const bool in = !EDGE || (m < g.M && n < g.N);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float x = acc_get(acc[i][j][4 * q + e]) * g.alpha;
                    if (g.acc_in && in) x += g.acc_in[(long long)m * g.N + n + e];
                    if (g.bias && !fold_bias && in) x += h2f(g.bias[n + e]);
                    acc[i][j][4 * q + e] = acc_put(x);
                }
            });
        }
        constexpr int NCH = TN * 2;  // 16-byte pieces per lane and 32-row block: tile j, piece c -> columns 32 j + 16 c + 8 eh ...
        u16x2         mag = {0, 0};  // running maximum of the magnitude bits of everything stored (non-finite: >= 0x7C00)
        // residual / ReLU-source pieces of block i; those of block i + 1 are requested before block i is worked on
        u32x4 av[2][NCH];
        auto  aux_load = [&](auto ic) {
            constexpr int i = decltype(ic)::value;
            static_for<NCH>([&](auto cc) {
                constexpr int ch = decltype(cc)::value;
                const int     m = mrow + 32 * i, n = ncol + 16 * ch + 8 * eh;
                av[i & 1][ch]   = u32x4{0u, 0u, 0u, 0u};
                if (!EDGE || (m < g.M && n < g.N)) av[i & 1][ch] = *reinterpret_cast<const u32x4*>(aux + (long long)m * g.ld_aux + n);
            });
        };
        if (aux) aux_load(std::integral_constant<int, 0>{});
        static_for<TM>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            if constexpr (i + 1 < TM) {
                if (aux) aux_load(std::integral_constant<int, i + 1>{});
            }
            __builtin_amdgcn_sched_barrier(0);
            const int m = mrow + 32 * i;
            static_for<TN>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                float         v[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = acc_get(acc[i][j][e]);
                if (g.relu) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) v[e] = (v[e] < 0.f) ? 0.f : v[e];  // max(v, 0) that keeps a NaN (the comparison is false for it)
                }
                // one rounding to fp16, packed in pairs: d[2 q], d[2 q + 1] = columns 8 q + 4 eh + {0, 1}, {2, 3}
                unsigned d[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const f16x2 hpair = __builtin_convertvector(f32x2{v[2 * e], v[2 * e + 1]}, f16x2);
                    d[e]              = __builtin_bit_cast(unsigned, hpair);
                }
                // lanes er (eh = 0) and er + 32 (eh = 1) trade: afterwards d[4 c .. 4 c + 3] hold, in order, the 8
                // consecutive columns 16 c + 8 eh ... of row er
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int w = 0; w < 2; ++w) {
                        const auto sw = __builtin_amdgcn_permlane32_swap(d[4 * c + w], d[4 * c + 2 + w], false, false);
                        d[4 * c + w]     = sw[0];
                        d[4 * c + 2 + w] = sw[1];
                    }
                static_for<2>([&](auto cc) {
                    constexpr int c = decltype(cc)::value;
                    const int     n = ncol + 32 * j + 16 * c + 8 * eh;
                    if (EDGE && (m >= g.M || n >= g.N)) return;
                    u32x4 out = {d[4 * c], d[4 * c + 1], d[4 * c + 2], d[4 * c + 3]};
                    if (aux) {
                        const u32x4 a = av[i & 1][2 * j + c];
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const unsigned ow = out[w], aw = a[w];  // (bit_cast wants whole objects, not vector elements)
                            const f16x2    hv = __builtin_bit_cast(f16x2, ow), tv = __builtin_bit_cast(f16x2, aw);
                            f16x2       rv;
                            if (g.relu_src) {
                                rv[0] = (tv[0] > (_Float16)0) ? hv[0] : (_Float16)0;
                                rv[1] = (tv[1] > (_Float16)0) ? hv[1] : (_Float16)0;
                            } else {
                                rv = __builtin_convertvector(__builtin_convertvector(hv, f32x2) + __builtin_convertvector(tv, f32x2), f16x2);
                            }
                            out[w] = __builtin_bit_cast(unsigned, rv);
                        }
                    }
                    if (g.found_inf) {
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const unsigned mw = out[w] & 0x7FFF7FFFu;
                            mag               = __builtin_elementwise_max(mag, __builtin_bit_cast(u16x2, mw));
                        }
                    }
                    *reinterpret_cast<u32x4*>(C + (long long)m * g.ldc + n) = out;
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        bad |= mag[0] >= 0x7C00 || mag[1] >= 0x7C00;
    }
}

// One output tile: tile number `pid` of problem g (tiles are numbered in bands of GROUP tile-rows), batch `by`, k-split
// `bz` of `nz`; `pid_next` is the tile this workgroup takes afterwards (same problem, batch and split), or -1.
// EDGE = false: every tile lies fully inside the matrices and K is a multiple of BK, so neither the
// loads nor the stores carry bounds tests.  EDGE = true: every access is tested (ragged shapes).
template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, bool EDGE>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const int pid, const int pid_next, const int by, const int bz,
                                          const int nz, char* smem, OperandStream<BM, BN, A_KC, B_KC>& S, bool& bad) {
    static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;            // 32x32 matrix-core tiles per wave
    static_assert(TM >= 1 && TN >= 1, "wave tile at least 32x32");
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;


    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int bo = by / g.batch_inner, bi = by - bo * g.batch_inner;
    const uint16_t* A = g.A + bo * g.sa_o + bi * g.sa_i;
    const uint16_t* B = g.B + bo * g.sb_o + bi * g.sb_i;
    const int kbeg = bz * g.k_per_split;
    const int kend = min(g.K, kbeg + g.k_per_split);
    const int nkt  = (kend - kbeg + BK - 1) / BK;

    auto tile_origin = [&](const int p, int& mm, int& nn) {
        constexpr int GROUP = 4;
        const int     band  = p / (GROUP * g.tiles_n);
        const int     first = band * GROUP;
        const int     gsz   = min(GROUP, g.tiles_m - first);
        const int     inb   = p - band * GROUP * g.tiles_n;
        mm                  = (first + inb % gsz) * BM;
        nn                  = (inb / gsz) * BN;
    };
    int m0, n0;
    tile_origin(pid, m0, n0);


    // The bias is a per-column constant of the fp32 sum, so it can start the accumulators (acc[i][j][4 q + c] is
    // column 32 j + 8 q + 4 (lane / 32) + c of the wave tile); not when a scale factor follows the sum.
    const int  er = lane & 31, eh = lane >> 5;
    const int  ncol = n0 + wn * WN;
    const bool fold_bias = g.bias != nullptr && g.C32 == nullptr && g.alpha == 1.f;
    f32x16     acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // (a primed stream brings the values along: they were requested ahead of the previous tile's output stores)
    typedef unsigned u32x2b __attribute__((ext_vector_type(2)));
    auto load_bias = [&](const int col0) {
        static_for<TN * 4>([&](auto tc) {
            constexpr int t = decltype(tc)::value, j = t / 4, q = t % 4;
            const int     n = col0 + 32 * j + 8 * q + 4 * eh;  // 4 consecutive columns: one 8-byte load
            S.bias[t]       = {0u, 0u};
            if (!EDGE || n < g.N) S.bias[t] = *reinterpret_cast<const u32x2b*>(g.bias + n);
        });
    };
    if (fold_bias) {
        if (!S.primed) load_bias(ncol);
        static_for<TN * 4>([&](auto tc) {
            constexpr int t = decltype(tc)::value, j = t / 4, q = t % 4;
            const auto    braw = S.bias[t];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float b = h2f((uint16_t)((e & 1) ? (braw[e >> 1] >> 16) : (braw[e >> 1] & 0xFFFFu)));
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[i][j][4 * q + e] = acc_put(b);
            }
        });
    }

    // Two register sets per operand: the global loads of k-tile t+2 are issued before the matrix-core
    // work of tile t and are first needed (for the LDS store) after the work of tile t+1, so a load has
    // two compute phases to arrive.  With one workgroup per CU and one wave per SIMD nothing else hides
    // the memory latency.
    // wave-uniform tile origins, advanced by one k-step per load
    const long long step_a = A_KC ? BK : (long long)BK * g.lda;
    const long long step_b = B_KC ? BK : (long long)BK * g.ldb;
    auto origin_a = [&](const int mm) { return A_KC ? A + (long long)mm * g.lda + kbeg : A + (long long)kbeg * g.lda + mm; };
    auto origin_b = [&](const int nn) { return B_KC ? B + (long long)nn * g.ldb + kbeg : B + (long long)kbeg * g.ldb + nn; };
    if (!S.primed) {
        S.ta     = origin_a(m0);
        S.tb     = origin_b(n0);
        S.k_next = kbeg;
    }
    // Where the stream goes behind this tile's last k-tile: on to the next tile (interior tiles with an even number of
    // at least 4 k-tiles: the register sets and LDS stages then end the tile in the roles they start one in), or
    // nowhere (see load_next).
    const bool      chain = !EDGE && pid_next >= 0 && nkt >= 4 && (nkt & 1) == 0;
    const uint16_t *nta = nullptr, *ntb = nullptr;
    int             ncol1 = 0;
    if (chain) {
        int m1, n1;
        tile_origin(pid_next, m1, n1);
        nta   = origin_a(m1);
        ntb   = origin_b(n1);
        ncol1 = n1 + wn * WN;
    }

    // matrix-core fragment addresses inside an LDS tile: row = base row + 32 i, k-slot = 2 kk + lane/32,
    // swizzled; only four distinct per-lane offsets exist (the rest are immediates), see swz().
    const int arow = wm * WM + (lane & 31), brow = wn * WN + (lane & 31);
    int       offa[4], offb[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        offa[c] = arow * 128 + ((((2 * c) | (lane >> 5)) ^ swz(arow)) << 4);
        offb[c] = brow * 128 + ((((2 * c) | (lane >> 5)) ^ swz(brow)) << 4);
    }

    // Loads never branch in the interior variant: past the last k-tile of the last tile the origin simply stops
    // advancing, so the (unused) extra loads re-read the last tile and stay in bounds.
    const int k_last = kbeg + (nkt > 0 ? nkt - 1 : 0) * BK;
    auto advance = [&] {
        const bool in = S.k_next < k_last;
        S.ta     = in ? S.ta + step_a : (chain ? nta : S.ta);
        S.tb     = in ? S.tb + step_b : (chain ? ntb : S.tb);
        S.k_next = in ? S.k_next + BK : (chain ? kbeg : S.k_next);
    };
    auto load_next = [&](auto& la, auto& lb) {
        la.template load<EDGE>(S.ta, g.lda, g.M - m0, kend - S.k_next);
        lb.template load<EDGE>(S.tb, g.ldb, g.N - n0, kend - S.k_next);
        advance();
    };
    // One pipeline step: issue the global loads of a later tile into (ln_a, ln_b), multiply the tile in
    // LDS stage `sa` and store the tile held in (st_a, st_b) into LDS stage `da`.  In the interior
    // variant this is one basic block, and the scheduling directives at its end interleave the memory
    // instructions with the matrix-core instructions (which run 8 passes each and leave the issue
    // port free): next-slice fragment reads right behind the first MFMAs of a slice, global loads
    // and LDS stores spread evenly over all slices but the last.
    // The workgroup barrier of a step stands in front of its LAST slice: by then every wave has issued all its
    // fragment reads of the stage being multiplied (the last slice's were issued a slice earlier) and all its stores
    // into the other stage, so behind the barrier the other stage may be read and this one overwritten.  The last
    // slice then runs out of registers while the first slice of the NEXT step is fetched from the other stage: a
    // step starts with its first fragments in registers instead of waiting an LDS round trip for them.
    constexpr int KS = BK / 16;   // k-slices per tile
    constexpr int NR = TM + TN;   // fragment reads per slice
    f16x8         af[2][TM], bf[2][TN];
    // fragment f of slice kk of the stage at `stage` into buffer kk&1 (f < TM: A rows, else B rows)
    auto read_frag = [&](const char* stage, auto kkc, auto fc) {
        constexpr int kk = decltype(kkc)::value, f = decltype(fc)::value;
        if constexpr (f < TM)
            af[kk & 1][f] = *reinterpret_cast<const f16x8*>(stage + offa[kk ^ ((f & 1) << 1)] + f * 4096);
        else
            bf[kk & 1][f - TM] =
                *reinterpret_cast<const f16x8*>(stage + A_BYTES + offb[kk ^ (((f - TM) & 1) << 1)] + (f - TM) * 4096);
    };
    auto step = [&](auto& ln_a, auto& ln_b, const auto& st_a, const auto& st_b, const char* sa, char* da) {
        constexpr int MS = TM * TN;                                // matrix-core instructions per slice
        constexpr int NM = MS * KS;                                // ... per step
        constexpr int NB = MS * (KS - 1);                          // ... in front of the barrier
        constexpr int NA = LoaderSel<BM, A_KC>::T::N_LOADS, NB_ = LoaderSel<BN, B_KC>::T::N_LOADS;
        constexpr int NG = NA + NB_;                               // global loads = LDS stores per step
        constexpr int RPM = (NR + MS - 1) / MS;                    // fragment reads issued behind one MFMA
        const int rows_a = g.M - m0, rows_b = g.N - n0, k_left = kend - S.k_next;
        auto gload = [&](auto gc) {
            constexpr int i = decltype(gc)::value;
            if constexpr (i < NA) ln_a.template load_one<EDGE, i>(S.ta, g.lda, rows_a, k_left);
            else ln_b.template load_one<EDGE, i - NA>(S.tb, g.ldb, rows_b, k_left);
        };
        auto lstore = [&](auto gc) {
            constexpr int i = decltype(gc)::value;
            if constexpr (i < NA) st_a.template store_one<i>(da);
            else st_b.template store_one<i - NA>(da + A_BYTES);
        };
        __builtin_amdgcn_sched_barrier(0);
        // Hand-placed order, pinned by scheduling barriers: behind matrix-core instruction m go the next
        // slice's fragment reads (at the start of a slice) and an even share of the step's global loads
        // and LDS stores.  An MFMA runs 8 passes and leaves the issue port free, so these overlap it.
        static_for<NM>([&](auto mc) {
            constexpr int m = decltype(mc)::value, kk = m / MS, q = m % MS, i = q / TN, j = q % TN;
            if constexpr (m == NB) {
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
            static_for<RPM>([&](auto rc) {
                constexpr int f = q * RPM + decltype(rc)::value;
                if constexpr (f < NR) {
                    if constexpr (kk + 1 < KS) read_frag(sa, std::integral_constant<int, kk + 1>{}, std::integral_constant<int, f>{});
                    else read_frag(da, std::integral_constant<int, 0>{}, std::integral_constant<int, f>{});  // next step
                }
            });
            if constexpr (m < NB) {
                constexpr int g0 = m * NG / NB, g1 = (m + 1) * NG / NB;
                static_for<g1 - g0>([&](auto gc) { gload(std::integral_constant<int, g0 + decltype(gc)::value>{}); });
                static_for<g1 - g0>([&](auto gc) { lstore(std::integral_constant<int, g0 + decltype(gc)::value>{}); });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        advance();
    };

    // prologue (unless the previous tile of this workgroup left the stream primed): k-tiles 0 and 1 into the two
    // register sets, k-tile 0 on into LDS stage 0
    if (!S.primed) {
        load_next(S.la0, S.lb0);
        load_next(S.la1, S.lb1);
        S.la0.store(smem);
        S.lb0.store(smem + A_BYTES);
        __syncthreads();
    }
    // step kt multiplies tile kt out of stage kt&1, stores tile kt+1 (loaded one step earlier) into the
    // other stage and loads tile kt+2 into the register set tile kt came from.  Unrolled by two so that
    // the register sets have static names.  Loads and stores past the last tile are redundant but
    // harmless (see load_next; the extra LDS store goes to the stage nobody reads any more), or belong to the next
    // tile (chain).
    static_for<NR>([&](auto fc) { read_frag(smem, std::integral_constant<int, 0>{}, fc); });  // first slice of the first step
    int kt = 0;
    for (; kt + 1 < nkt; kt += 2) {
        step(S.la0, S.lb0, S.la1, S.lb1, smem, smem + STAGE);
        step(S.la1, S.lb1, S.la0, S.lb0, smem + STAGE, smem);
    }
    if (kt < nkt) step(S.la0, S.lb0, S.la1, S.lb1, smem, smem + STAGE);  // odd tile count
    S.primed = chain;
    if (chain && fold_bias) load_bias(ncol1);

    gemm_epilogue<TM, TN, EDGE>(g, acc, m0 + wm * WM + er, ncol, bo, bi, bz, nz > 1, fold_bias, bad);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, bool EDGE>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(GemmArgs g) {
    extern __shared__ __align__(16) char smem[];
    bool bad = false;
    // Persistent over tiles: workgroup w takes tiles w, w + gridDim.x, ...  The stores of one tile's epilogue
    // drain while the next tile's first loads are in flight.
    const int ntiles = g.tiles_m * g.tiles_n;
    // consecutive ids are dispatched round-robin over the 8 XCDs (gridDim.x is a multiple of 8 whenever a
    // workgroup takes more than one tile), so id -> (id % 8) * (ntiles / 8) + id / 8 gives each XCD, and its
    // L2, a contiguous run of tiles
    auto tile_of = [&](const int vb) {
        const int q = ntiles >> 3, rem = ntiles & 7, x = vb & 7, local = vb >> 3;
        return x * q + min(x, rem) + local;
    };
    OperandStream<BM, BN, A_KC, B_KC> S;
    S.init(g.lda, g.ldb);
    for (int vb = blockIdx.x; vb < ntiles; vb += gridDim.x) {
        const int nvb = vb + gridDim.x;
        gemm_tile<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, EDGE>(g, tile_of(vb), nvb < ntiles ? tile_of(nvb) : -1, blockIdx.y,
                                                             blockIdx.z, gridDim.z, smem, S, bad);
    }
    if (g.found_inf && __any(bad)) {
        if ((threadIdx.x & 63) == 0) atomicOr(g.found_inf, 1);
    }
}

// Several independent problems of one operand layout in one launch (the weight-gradient products of a layer: each
// alone has too few tiles for the chip).  Tiles of all problems are numbered one after the other, largest problem
// first; no batches, no k-splits.
constexpr int GROUP_MAX = 8;
// A bias gradient riding in a grouped launch: column sums of dY[rows, cols], cut into strips of BIAS_COLS columns
// that are numbered after the product tiles (a strip is one work item for a workgroup, like a tile).
constexpr int BIAS_COLS = 128;
struct BiasItem {
    const unsigned short* dY;  // fp16 bits
    unsigned short*       db;
    int                   ld, rows;
};
struct GroupArgs {
    GemmArgs p[GROUP_MAX];
    int      tile_start[GROUP_MAX + 1];
    int      count;
    BiasItem b[GROUP_MAX];
    int      strip_start[GROUP_MAX + 1];  // strip_start[nbias] = number of strips
    int      nbias;
};

// db[strip] = RNE16(fp32 column sums of a 128-column strip of dY), by one workgroup of 256 threads: 16 lanes x 8
// columns (16-byte loads) by 16 row groups, 8 loads in flight per thread, rows summed in a fixed order (per thread
// ascending, then the 16 row groups ascending), so the result does not depend on scheduling.  16 x 128 floats of LDS.
__device__ inline void colsum_strip(const BiasItem it, int strip, char* smem, bool& bad) {
    constexpr int U = 8;
    const int     tid = threadIdx.x, cx = tid & 15, ry = tid >> 4;
    const unsigned short* src = it.dY + (size_t)strip * BIAS_COLS + cx * 8;
    float         acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int r0 = ry; r0 < it.rows; r0 += 16 * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + 16 * u;
            v[u]        = (r < it.rows) ? *reinterpret_cast<const uint4*>(src + (size_t)r * it.ld) : uint4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] += (float)__builtin_bit_cast(_Float16, (unsigned short)(w[e] & 0xffffu));
                acc[2 * e + 1] += (float)__builtin_bit_cast(_Float16, (unsigned short)(w[e] >> 16));
            }
        }
    }
    float* red = reinterpret_cast<float*>(smem);
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 8; ++e) red[ry * BIAS_COLS + cx * 8 + e] = acc[e];
    __syncthreads();
    if (tid < BIAS_COLS) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) s += red[j * BIAS_COLS + tid];
        const unsigned short h = __builtin_bit_cast(unsigned short, (_Float16)s);  // round to nearest even
        it.db[(size_t)strip * BIAS_COLS + tid] = h;
        bad |= (h & 0x7fffu) >= 0x7c00u;
    }
    __syncthreads();
}

// the strips of a grouped launch, work items total .. total + strips - 1
__device__ inline void group_bias_item(const GroupArgs& ga, int s, char* smem, bool& bad) {
    BiasItem it    = ga.b[0];
    int      first = 0;
#pragma unroll
    for (int q = 1; q < GROUP_MAX; ++q) {
        if (q < ga.nbias && s >= ga.strip_start[q]) {
            it    = ga.b[q];
            first = ga.strip_start[q];
        }
    }
    colsum_strip(it, s - first, smem, bad);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_grouped_kernel(GroupArgs ga) {
    extern __shared__ __align__(16) char smem[];
    bool      bad_any = false;
    int*      flag    = ga.p[0].found_inf;  // one flag for the whole group
    const int total   = ga.tile_start[ga.count];
    const int items   = total + ga.strip_start[ga.nbias];
    for (int vb0 = blockIdx.x; vb0 < items; vb0 += gridDim.x) {
        if (vb0 >= total) {  // a bias-gradient strip
            bool bad = false;
            group_bias_item(ga, vb0 - total, smem, bad);
            bad_any |= bad;
            continue;
        }
        // consecutive workgroup ids go round-robin over the 8 XCDs: give each XCD, and its L2, a contiguous run of
        // tiles (neighbouring tiles share operand panels)
        const int xq = total >> 3, xrem = total & 7, xx = vb0 & 7;
        const int vb = xx * xq + min(xx, xrem) + (vb0 >> 3);
        // the problem this tile belongs to: chosen with wave-uniform selects over statically indexed entries, so
        // the descriptor stays in scalar registers
        GemmArgs g     = ga.p[0];
        int      first = 0;
#pragma unroll
        for (int q = 1; q < GROUP_MAX; ++q) {
            if (q < ga.count && vb >= ga.tile_start[q]) {
                g     = ga.p[q];
                first = ga.tile_start[q];
            }
        }
        bool bad = false;
        OperandStream<BM, BN, A_KC, B_KC> S;
        S.init(g.lda, g.ldb);
        gemm_tile<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, false>(g, vb - first, -1, 0, 0, 1, smem, S, bad);
        bad_any |= bad;
        __syncthreads();  // (tiles of different problems: keep the LDS stages of one tile apart from the next)
    }
    if (flag && __any(bad_any)) {
        if ((threadIdx.x & 63) == 0) atomicOr(flag, 1);
    }
}

// ------------------------------------------------------------------------------------ launches
// The kernel templates are instantiated in one translation unit per operand layout (gemm_kk.hip, gemm_ko.hip,
// gemm_oo.hip: explicit instantiations of launch_tile / launch_grouped), which compile in parallel; gemm.hip holds
// the planner and the C entry points and only declares them.
template <int BM, int BN, int WM_, int WN_, bool AKC, bool BKC, bool EDGE>
static int launch_variant(const GemmArgs& g, dim3 grid, hipStream_t hs) {
    constexpr size_t  lds = 2 * (size_t)(BM + BN) * 128;
    static std::once_flag once;
    static hipError_t     attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<BM, BN, WM_, WN_, AKC, BKC, EDGE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (attr_err != hipSuccess) return hip_fail(attr_err, "gemm: hipFuncSetAttribute(LDS size)");
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM_, WN_, AKC, BKC, EDGE>), grid, dim3(GEMM_THREADS), lds, hs, g);
    MP_LAUNCH_CHECK("gemm launch");
    return MP_OK;
}

template <int BM, int BN, int WM_, int WN_, bool AKC, bool BKC>
static int launch_one(const GemmArgs& g, dim3 grid, hipStream_t hs) {
    const bool edge = (g.M % BM) != 0 || (g.N % BN) != 0 || (g.K % BK) != 0;
    return edge ? launch_variant<BM, BN, WM_, WN_, AKC, BKC, true>(g, grid, hs)
                : launch_variant<BM, BN, WM_, WN_, AKC, BKC, false>(g, grid, hs);
}

template <bool AKC, bool BKC>
int launch_tile(int t, const GemmArgs& g, dim3 grid, hipStream_t hs) {
    switch (t) {
        case 0: return launch_one<256, 256, 2, 2, AKC, BKC>(g, grid, hs);
        case 1: return launch_one<256, 128, 2, 2, AKC, BKC>(g, grid, hs);
        case 2: return launch_one<128, 256, 2, 2, AKC, BKC>(g, grid, hs);
        case 3: return launch_one<128, 128, 2, 2, AKC, BKC>(g, grid, hs);
        case 4: return launch_one<128, 64, 2, 2, AKC, BKC>(g, grid, hs);
        case 5: return launch_one<64, 128, 2, 2, AKC, BKC>(g, grid, hs);
        case 6: return launch_one<64, 64, 2, 2, AKC, BKC>(g, grid, hs);
        case 8:
            if constexpr (AKC && BKC) return launch_one<256, 192, 2, 2, AKC, BKC>(g, grid, hs);
            [[fallthrough]];
        default: return launch_one<32, 128, 1, 4, AKC, BKC>(g, grid, hs);
    }
}

template <int BM, int BN>
int launch_grouped(const GroupArgs& ga, int resident, hipStream_t hs) {
    constexpr size_t  lds = 2 * (size_t)(BM + BN) * 128;
    static std::once_flag once;
    static hipError_t     attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_grouped_kernel<BM, BN, 2, 2, false, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (attr_err != hipSuccess) return hip_fail(attr_err, "gemm: hipFuncSetAttribute(LDS size)");
    const int total = ga.tile_start[ga.count] + ga.strip_start[ga.nbias];
    hipLaunchKernelGGL((gemm_grouped_kernel<BM, BN, 2, 2, false, false>), dim3(total < resident ? total : resident),
                       dim3(GEMM_THREADS), lds, hs, ga);
    MP_LAUNCH_CHECK("grouped gemm launch");
    return MP_OK;
}

}  // namespace mp
