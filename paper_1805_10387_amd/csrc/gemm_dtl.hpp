// Contraction kernel whose operand tiles go from global memory straight into LDS (no staging registers, no LDS store
// instructions) through a ring of 32-deep k-tiles (as many stages as fit 160 KB of LDS: five for the 256 x 256 tile,
// up to eight for smaller tiles), for interior problems (every tile inside the matrices, K a multiple of 32).  Same
// arithmetic and epilogue as gemm_kernels.hpp (paper Section 3.1: fp16 operands, fp32 sums, one rounding); what
// differs is how the operands reach the matrix cores.
//
//   * `global_load_lds` (16 bytes per lane): a wave instruction deposits its 64 lanes' pieces as 1 KB of CONSECUTIVE
//     LDS bytes in lane order, whatever each lane's global address is.  The LDS layout is therefore chosen by choosing
//     which global piece each lane fetches:
//       contraction-contiguous operand ([row][k]): LDS rows of 32 k = 64 bytes = 4 pieces; piece s of row r sits in
//         slot s ^ ((r >> 2) & 3), which makes every 16-byte fragment read of 16 consecutive rows conflict-free;
//       output-contiguous operand ([k][row]): LDS keeps the global orientation, k-rows of R * 2 bytes; the 16-byte
//         piece g (8 rows) of k-row k sits at piece g ^ ((k & 3) << 2).  Fragments come out of it with the transposing
//         LDS read (`ds_read_b64_tr_b16`): within 16 lanes, lane i receives element i % 4 of the 8-byte chunks
//         addressed by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4, so four lanes that address the same k and four
//         consecutive 4-row groups hand every lane of the 16 its own row at 4 consecutive k.  Two such reads make the
//         8-k fragment of `v_mfma_f32_32x32x16_f16`; no byte permutes, no register transposes.
//   * ring of DNS stages: the loads of k-tile q + DNS are issued right behind the barrier inside k-tile q that retires
//     stage q % DNS, so a k-tile has DNS - 1 k-tiles of matrix-core work (about 1024 cycles each for the 256 x 256 tile)
//     to arrive, and the ring runs on across output tiles: the next tile's first k-tiles are requested during the
//     current tile's last ones.
//   * one workgroup barrier per k-tile, placed between its two 16-deep slices: behind it come the fragment reads of
//     the next k-tile's first slice, covered by the matrix-core work of this k-tile's second slice.
#pragma once
#include "gemm_kernels.hpp"

namespace mp {

constexpr int DK = 32;  // k per stage
// stages of the ring: as many as fit 160 KB of LDS, at most 8 (smaller tiles have less matrix-core work per k-tile, so
// a load needs more k-tiles of lead to cover the same memory latency)
constexpr int dtl_stages(int bm, int bn) { return (160 * 1024) / ((bm + bn) * 64) > 8 ? 8 : (160 * 1024) / ((bm + bn) * 64); }

#define MP_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define MP_GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

typedef short s16x4 __attribute__((ext_vector_type(4)));

// One operand (R tile rows) of the direct-to-LDS pipeline.
template <int R, bool KC>
struct DtlOperand {
    static_assert(R % 64 == 0 && (KC || R == 128 || R == 256), "tile edge");
    static constexpr int BYTES = R * 64;  // one stage: R rows x 32 k x 2 bytes
    static constexpr int NBLK  = R / 64;  // 1 KB blocks per wave and stage (R / 16 blocks, 4 waves)
    unsigned goff[NBLK];                  // this lane's global element offset inside block q, from the k-tile's origin
    int      foff[4];                     // fragment read offsets: KC [kk], OC [32-row tile i]

    // wave: wave index in the workgroup; row0: first row of this wave's tile rows inside the workgroup tile
    __device__ __forceinline__ void init(int ld, int wave, int lane, int row0) {
        const int r = lane & 31, h = lane >> 5;
#pragma unroll
        for (int q = 0; q < NBLK; ++q) {
            const int b = wave + 4 * q;
            if (KC) {
                const int row = 16 * b + (lane >> 2), s = (lane & 3) ^ ((lane >> 4) & 3);
                goff[q]       = (unsigned)row * (unsigned)ld + 8 * s;
            } else {
                const int P = 64 * b + lane, k = P / (R / 8), gp = P % (R / 8);
                goff[q]     = (unsigned)k * (unsigned)ld + 8 * (gp ^ ((k & 3) << 2));
            }
        }
        if (KC) {
            foff[0] = (row0 + r) * 64 + (((0 | h) ^ ((r >> 2) & 3)) << 4);
            foff[1] = (row0 + r) * 64 + (((2 | h) ^ ((r >> 2) & 3)) << 4);
            foff[2] = foff[3] = 0;
        } else {
            const int i16 = lane & 15, r16 = 16 * ((lane >> 4) & 1), kq = i16 >> 2;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int g = (((row0 + 32 * i) >> 3) ^ (kq << 2)) + (r16 >> 3) + ((i16 & 3) >> 1);
                foff[i]     = (8 * h + kq) * (2 * R) + (g << 4) + (i16 & 1) * 8;
            }
        }
    }
    // global -> LDS, block Q of this wave's share of one k-tile; `tile`: wave-uniform origin (first row, first k of the k-tile)
    // `stage`: LDS byte address of this operand's region in the target stage.
    // Written as assembly on purpose: the compiler orders every LDS read behind an LDS-writing load it knows of by
    // waiting for ALL loads in flight (it cannot tell the stages apart), which would serialise the ring.  The ring's
    // own accounting (the counted waits in front of the barriers) is what orders these loads against the reads.
    // (M0 holds the LDS destination; nothing else in these kernels uses M0.)
    template <int Q>
    __device__ __forceinline__ void issue_one(const uint16_t* tile, unsigned stage, int wave) const {
        const uint16_t* src = tile + goff[Q];
        const unsigned  dst = stage + (wave + 4 * Q) * 1024;
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(dst) : "memory");
    }
    // matrix-core fragment: 8 consecutive k of slice kk (16 k) for row (lane % 32) of 32-row tile i
    template <int KK, int I>
    __device__ __forceinline__ f16x8 frag(const char* stage) const {
        if constexpr (KC) {
            return *reinterpret_cast<const f16x8*>(stage + foff[KK] + I * 2048);
        } else {
            const char* p  = stage + foff[I] + KK * 16 * (2 * R);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)MP_LDS_PTR(p));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)MP_LDS_PTR(p + 4 * (2 * R)));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            return __builtin_bit_cast(f16x8, v);
        }
    }
};

// The output tiles vb0, vb0 + vb_step, ... (< tiles_m * tiles_n) of problem g, one after the other, with the ring of
// stages running on from tile to tile.  remap: number the tiles so that each XCD gets a contiguous run (a launch of one
// problem); otherwise vb is the tile number itself (the caller has placed the tiles).
template <int BM, int BN, bool A_KC, bool B_KC>
__device__ __forceinline__ void dtl_tiles(const GemmArgs& g, const int vb0, const int vb_step, const bool remap, char* smem,
                                          bool& bad) {
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    typedef DtlOperand<BM, A_KC> OpA;
    typedef DtlOperand<BN, B_KC> OpB;
    constexpr int STAGE = OpA::BYTES + OpB::BYTES;
    constexpr int DNS   = dtl_stages(BM, BN);
    constexpr int LPW   = OpA::NBLK + OpB::NBLK;  // loads per wave and k-tile
    constexpr int MS    = TM * TN;                // matrix-core instructions per 16-deep slice
    constexpr int NR    = TM + TN;                // fragments per slice

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds_base = (unsigned)(size_t)MP_LDS_PTR(smem);
    const int wm = wave >> 1, wn = wave & 1;
    const int er = lane & 31, eh = lane >> 5;
    const int nkt    = g.K / DK;
    const int ntiles = g.tiles_m * g.tiles_n;

    // tile numbering: XCD-contiguous runs, bands of 4 tile rows (as gemm_kernel)
    auto tile_of = [&](const int vb) {
        if (!remap) return vb;
        const int q = ntiles >> 3, rem = ntiles & 7, x = vb & 7, local = vb >> 3;
        return x * q + min(x, rem) + local;
    };
    auto tile_origin = [&](const int p, int& mm, int& nn) {
        constexpr int GROUP = 4;
        const int     band  = p / (GROUP * g.tiles_n);
        const int     first = band * GROUP;
        const int     gsz   = min(GROUP, g.tiles_m - first);
        const int     inb   = p - band * GROUP * g.tiles_n;
        mm                  = (first + inb % gsz) * BM;
        nn                  = (inb / gsz) * BN;
    };

    OpA oa;
    OpB ob;
    oa.init(g.lda, wave, lane, wm * WM);
    ob.init(g.ldb, wave, lane, wn * WN);
    const long long step_a = A_KC ? DK : (long long)DK * g.lda;
    const long long step_b = B_KC ? DK : (long long)DK * g.ldb;

    // ---- the load stream: k-tile after k-tile, output tile after output tile, into stage (count % DNS)
    int             l_vb = vb0, l_kt = 0, l_stage = 0;
    const uint16_t *l_pa = nullptr, *l_pb = nullptr;
    auto            l_origin = [&] {
        int m, n;
        tile_origin(tile_of(l_vb), m, n);
        l_pa = A_KC ? g.A + (long long)m * g.lda : g.A + m;
        l_pb = B_KC ? g.B + (long long)n * g.ldb : g.B + n;
    };
    l_origin();
    auto issue_one = [&](auto qc) {  // load instruction q of the k-tile the stream stands at
        constexpr int q = decltype(qc)::value;
        const unsigned st = lds_base + l_stage * STAGE;
        if constexpr (q < OpA::NBLK) oa.template issue_one<q>(l_pa, st, wave);
        else ob.template issue_one<q - OpA::NBLK>(l_pb, st + OpA::BYTES, wave);
    };
    auto advance = [&] {
        l_stage = l_stage + 1 == DNS ? 0 : l_stage + 1;
        // past the last k-tile of the last tile the position stays (the extra loads re-read that k-tile into a stage
        // nobody reads any more: in bounds, and they keep the count of loads in flight uniform)
        if (l_kt + 1 < nkt) {
            ++l_kt;
            l_pa += step_a;
            l_pb += step_b;
        } else if (l_vb + vb_step < ntiles) {
            l_vb += vb_step;
            l_kt = 0;
            l_origin();
        }
    };
    auto issue_next = [&] {
        static_for<LPW>([&](auto qc) { issue_one(qc); });
        advance();
    };

    f16x8 af[2][TM], bf[2][TN];
    auto  read_frags = [&](const char* stage, auto kkc, auto bufc) {
        constexpr int kk = decltype(kkc)::value, buf = decltype(bufc)::value;
        static_for<TM>([&](auto ic) { af[buf][decltype(ic)::value] = oa.template frag<kk, decltype(ic)::value>(stage); });
        static_for<TN>([&](auto jc) { bf[buf][decltype(jc)::value] = ob.template frag<kk, decltype(jc)::value>(stage + OpA::BYTES); });
    };
    auto read_frag_one = [&](const char* stage, auto kkc, auto bufc, auto fc) {
        constexpr int kk = decltype(kkc)::value, buf = decltype(bufc)::value, f = decltype(fc)::value;
        if constexpr (f < TM) af[buf][f] = oa.template frag<kk, f>(stage);
        else bf[buf][f - TM] = ob.template frag<kk, f - TM>(stage + OpA::BYTES);
    };

    // prologue: DNS k-tiles on their way, the first landed, its first fragments in registers
    static_for<DNS>([&](auto) { issue_next(); });
    static_assert((DNS - 1) * LPW <= 63, "loads in flight must fit the counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DNS - 1) * LPW) : "memory");
    __syncthreads();
    int c_stage = 0;
    read_frags(smem, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});

    for (int vb = vb0; vb < ntiles; vb += vb_step) {
        int m0, n0;
        tile_origin(tile_of(vb), m0, n0);
        const int  ncol      = n0 + wn * WN;
        const bool fold_bias = g.bias != nullptr && g.C32 == nullptr && g.alpha == 1.f;
        f32x16     acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (fold_bias) {
            typedef unsigned u32x2b __attribute__((ext_vector_type(2)));
            static_for<TN * 4>([&](auto tc) {
                constexpr int t = decltype(tc)::value, j = t / 4, q = t % 4;
                const u32x2b  braw = *reinterpret_cast<const u32x2b*>(g.bias + ncol + 32 * j + 8 * q + 4 * eh);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float b = h2f((uint16_t)((e & 1) ? (braw[e >> 1] >> 16) : (braw[e >> 1] & 0xFFFFu)));
#pragma unroll
                    for (int i = 0; i < TM; ++i) acc[i][j][4 * q + e] = acc_put(b);
                }
            });
        }
        for (int kt = 0; kt < nkt; ++kt) {
            const char* cur = smem + c_stage * STAGE;
            const char* nxt = smem + (c_stage + 1 == DNS ? 0 : c_stage + 1) * STAGE;
            __builtin_amdgcn_sched_barrier(0);
            // slice 0 out of buffer 0; behind its matrix-core instructions: the fragments of slice 1 into buffer 1
            static_for<MS>([&](auto mc) {
                constexpr int m = decltype(mc)::value, i = m / TN, j = m % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[0][j], af[0][i], acc[i][j], 0, 0, 0);
                if constexpr (m < NR) read_frag_one(cur, std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, mc);
                __builtin_amdgcn_sched_barrier(0);
            });
            // the next k-tile has landed (DNS - 2 later ones may still be in flight), and every wave is done with this stage:
            // its last fragments are in registers
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((DNS - 2) * LPW) : "memory");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // slice 1 out of buffer 1; behind its matrix-core instructions: the first fragments of the next k-tile into
            // buffer 0, and the loads of k-tile q + DNS into the stage just retired, one instruction at a time
            static_for<MS>([&](auto mc) {
                constexpr int m = decltype(mc)::value, i = m / TN, j = m % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[1][j], af[1][i], acc[i][j], 0, 0, 0);
                if constexpr (m < NR) read_frag_one(nxt, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, mc);
                constexpr int l0 = m * LPW / MS, l1 = (m + 1) * LPW / MS;
                static_for<l1 - l0>([&](auto lc) { issue_one(std::integral_constant<int, l0 + decltype(lc)::value>{}); });
                __builtin_amdgcn_sched_barrier(0);
            });
            advance();
            c_stage = c_stage + 1 == DNS ? 0 : c_stage + 1;
        }
        asm volatile("s_nop 15\n\ts_nop 15");
        gemm_epilogue<TM, TN, false>(g, acc, m0 + wm * WM + er, ncol, 0, 0, 0, false, fold_bias, bad);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the ring's last (unused) loads have landed before the LDS is reused
    __syncthreads();
}

template <int BM, int BN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_dtl_kernel(GemmArgs g) {
    extern __shared__ __align__(16) char smem[];
    bool bad = false;
    dtl_tiles<BM, BN, A_KC, B_KC>(g, blockIdx.x, gridDim.x, true, smem, bad);
    if (g.found_inf && __any(bad)) {
        if ((threadIdx.x & 63) == 0) atomicOr(g.found_inf, 1);
    }
}

// Several independent weight-gradient problems (both operands output-contiguous) in one launch, tiles numbered one
// problem after the other as in gemm_grouped_kernel; every tile runs its own ring (no chaining across problems).
template <int BM, int BN>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_dtl_grouped_kernel(GroupArgs ga) {
    extern __shared__ __align__(16) char smem[];
    bool      bad_any = false;
    int*      flag    = ga.p[0].found_inf;
    const int total   = ga.tile_start[ga.count];
    const int items   = total + ga.strip_start[ga.nbias];
    for (int vb0 = blockIdx.x; vb0 < items; vb0 += gridDim.x) {
        if (vb0 >= total) {  // a bias-gradient strip (no ring in flight between tiles here)
            bool bad = false;
            group_bias_item(ga, vb0 - total, smem, bad);
            bad_any |= bad;
            continue;
        }
        const int xq = total >> 3, xrem = total & 7, xx = vb0 & 7;
        const int vb = xx * xq + min(xx, xrem) + (vb0 >> 3);
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
        dtl_tiles<BM, BN, false, false>(g, vb - first, 1 << 30, false, smem, bad);
        bad_any |= bad;
    }
    if (flag && __any(bad_any)) {
        if ((threadIdx.x & 63) == 0) atomicOr(flag, 1);
    }
}

template <int BM, int BN>
int launch_dtl_grouped(const GroupArgs& ga, int resident, hipStream_t hs) {
    constexpr size_t  lds = (size_t)dtl_stages(BM, BN) * (BM + BN) * 64;
    static std::once_flag once;
    static hipError_t     attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dtl_grouped_kernel<BM, BN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (attr_err != hipSuccess) return hip_fail(attr_err, "gemm: hipFuncSetAttribute(LDS size)");
    const int total = ga.tile_start[ga.count] + ga.strip_start[ga.nbias];
    hipLaunchKernelGGL((gemm_dtl_grouped_kernel<BM, BN>), dim3(total < resident ? total : resident), dim3(GEMM_THREADS), lds, hs, ga);
    MP_LAUNCH_CHECK("grouped gemm launch (direct-to-LDS)");
    return MP_OK;
}

// Launch (host): the caller has checked that the problem is interior for this tile and unbatched, unsplit.
template <int BM, int BN, bool AKC, bool BKC>
int launch_dtl(const GemmArgs& g, int grid_x, hipStream_t hs) {
    constexpr size_t  lds = (size_t)dtl_stages(BM, BN) * (BM + BN) * 64;
    static std::once_flag once;
    static hipError_t     attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dtl_kernel<BM, BN, AKC, BKC>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (attr_err != hipSuccess) return hip_fail(attr_err, "gemm: hipFuncSetAttribute(LDS size)");
    hipLaunchKernelGGL((gemm_dtl_kernel<BM, BN, AKC, BKC>), dim3(grid_x), dim3(GEMM_THREADS), lds, hs, g);
    MP_LAUNCH_CHECK("gemm launch (direct-to-LDS)");
    return MP_OK;
}

// tile index as in the planner's table; returns MP_E_UNSUPPORTED for shapes this kernel is not built for
template <bool AKC, bool BKC>
int launch_dtl_tile(int t, const GemmArgs& g, int grid_x, hipStream_t hs) {
    switch (t) {
        case 0: return launch_dtl<256, 256, AKC, BKC>(g, grid_x, hs);
        case 1: return launch_dtl<256, 128, AKC, BKC>(g, grid_x, hs);
        case 2: return launch_dtl<128, 256, AKC, BKC>(g, grid_x, hs);
        case 3: return launch_dtl<128, 128, AKC, BKC>(g, grid_x, hs);
        case 8:
            if constexpr (AKC && BKC) return launch_dtl<256, 192, AKC, BKC>(g, grid_x, hs);
            [[fallthrough]];
        default: return MP_E_UNSUPPORTED;
    }
}

}  // namespace mp
