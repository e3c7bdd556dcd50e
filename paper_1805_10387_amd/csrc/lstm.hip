// Persistent recurrent-layer kernels: every time step of one LSTM layer in ONE launch per direction (the GNMT-like
// encoder of the paper's Section 2 configuration listing and Section 5.1; arithmetic of Sections 3.1 / 3.2: fp16
// operands, fp32 sums, fp16 storage points, fp32 cell state).
//
// A layer unrolled over time is a chain of small dependent products (batch rows x [4H, H]): launched one by one a time
// step costs its launches and first-load latencies, not its bytes.  Here each workgroup owns RL_UNITS hidden units of
// RL_ROWS batch rows for the whole sequence (batch rows never mix in the recurrence, so each block of rows is a grid
// of its own with its own step barrier):
//   forward : its 4 x RL_UNITS rows of the recurrent weight block W_h live in registers as matrix-core fragments for
//             all T steps; per step it reads h_{t-1} (all units, B x H fp16) from memory, forms its gate sums, adds
//             the input half x_t W_x^T (computed for all steps at once by one large product beforehand, kept fp32, so
//             the gate sum is still rounded once), updates its cells (c in registers, fp32) and publishes its slice
//             of h_t.
//   backward: its RL_UNITS columns of W_h (as W_h^T fragments) live in registers; per step it runs the cell backward
//             for its units (the recurrent gradient of its own units and the cell-state gradient never leave the
//             workgroup), publishes its slice of dgates_t, and after the step barrier contracts the whole dgates_t
//             (B x 4H) with its columns to get the recurrent gradient of its units for step t - 1.
// One grid-wide barrier per time step: every workgroup stores a step number into its own flag word and polls all flag
// words (no shared counter to serialise on).  All workgroups must be co-resident, so the grid never exceeds the number
// of compute units; the wait is bounded in wall-clock time and a workgroup that gives up raises *status, which makes
// every other workgroup give up too: the grid always drains.
#include "cell_math.hpp"
#include "common.hpp"

namespace mp {

constexpr int RL_THREADS = 256;  // 4 waves: each takes a quarter of the contraction
constexpr int RL_UNITS   = 16;   // hidden units per workgroup = one 16-row matrix-core block per gate
constexpr int RL_ROWS    = 16;   // batch rows per workgroup = one matrix-core block; more rows: more workgroups (grid y)
constexpr int RL_MAX_H   = 1024; // register budget of the fragment arrays below
constexpr int RL_FLAG_WORDS = 128;  // flag words per barrier group (one group per block of batch rows)
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

struct RlSync {
    int*      flags;        // nwait words, zero at launch; workgroup g stores the number of the step it has finished
    int*      status;       // 0 on entry; set nonzero by a workgroup whose wait ran out
    int       nwait;        // flags to wait for (= gridDim.x; tests may ask for more, which never arrive)
    long long limit_ticks;  // bound of one wait, in ticks of the constant 100 MHz clock
};

// This workgroup has finished `step`: its flag is raised once all its global stores of the step are visible
// device-wide.  The workgroup barrier waits until every wave's stores have left the compute unit and orders them
// before thread 0, whose device-scope release store then publishes them (one write-back of the cache level that
// other compute-unit clusters cannot see, per workgroup and step, instead of one per wave).
__device__ __forceinline__ void grid_arrive(const RlSync& s, int step) {
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(s.flags + blockIdx.x, step, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait until every flag has reached `step`.  Returns false (for the whole workgroup alike) when the wait was
// abandoned: its time ran out, or another workgroup had already given up.  Wave 0 polls (lane i watches flags i,
// i + 64, ...), takes the device-scope acquire, and hands the verdict to the other waves through `verdict` (LDS)
// and a workgroup barrier, which orders everything they read afterwards behind that acquire.
__device__ __forceinline__ bool grid_wait(const RlSync& s, int step, int* verdict) {
    if (threadIdx.x < 64) {
        const long long t0 = wall_clock64();
        int             ok = 1;
        for (;;) {
            int mine = 1;
            for (int i = threadIdx.x; i < s.nwait; i += 64)
                mine &= __hip_atomic_load(s.flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= step;
            if (__all(mine)) break;
            const int give_up = (wall_clock64() - t0 > s.limit_ticks) ||
                                __hip_atomic_load(s.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
            if (__any(give_up)) {  // (lanes read the clock a few ticks apart: the wave decides as one)
                ok = 0;
                break;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (threadIdx.x == 0) {
            if (!ok) atomicOr(s.status, 1);
            *verdict = ok;
        }
    }
    __syncthreads();
    return *verdict != 0;
}

__device__ __forceinline__ f16x8 as_frag(const u32x4& v) { return __builtin_bit_cast(f16x8, v); }

// ------------------------------------------------------------------------------------------------ forward
struct LstmFwdArgs {
    int             T, B, I, H;
    const float*    gx;     // [T*B, 4H] fp32: x_t W_x^T
    const uint16_t* w;      // [4H, ldw]; recurrent block = columns I .. I+H
    int             ldw;
    const uint16_t* bias;   // [4H]
    uint16_t*       gates;  // [T*B, 4H] out
    float*          c;      // [(T+1)*B, H]: rows of step 0 given, steps 1..T out
    uint16_t*       xh;     // [T*B, ldxh]: h_{t-1} is read from columns I.. of step t, h_t written to step t+1
    int             ldxh;
    uint16_t*       h_up;   // [T*B, ld_up] or NULL: h_t also goes here
    int             ld_up;
    RlSync          sync;
};

__global__ __launch_bounds__(RL_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1))) void lstm_layer_fwd_kernel(LstmFwdArgs a) {
    __shared__ float red[4][16][65];  // per wave: partial gate sums [batch row][16 g + unit]
    __shared__ int   verdict;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 15, lq = lane >> 4;
    const int H = a.H, I = a.I, B = a.B, T = a.T;
    const int j0  = blockIdx.x * RL_UNITS;   // this workgroup's hidden units
    const int b0  = blockIdx.y * RL_ROWS;    // ... and batch rows (the recurrence never mixes batch rows)
    const int nb  = min(RL_ROWS, B - b0);
    const int Kw  = H >> 2;             // this wave's share of the contraction over h
    const int nks = Kw >> 5;            // matrix-core steps of 32
    const int k0  = wave * Kw + 8 * lq; // first k of this lane's 8 consecutive values, + 32 ks
    RlSync    sync = a.sync;
    sync.flags += blockIdx.y * RL_FLAG_WORDS;  // one barrier group per block of batch rows

    // W_h fragments, resident for the whole sequence: gate g, unit lr, 8 consecutive k
    u32x4 wf[4][8];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            wf[g][ks] = u32x4{0u, 0u, 0u, 0u};
            if (ks < nks) wf[g][ks] = *reinterpret_cast<const u32x4*>(a.w + (long long)(g * H + j0 + lr) * a.ldw + I + k0 + 32 * ks);
        }

    // cell ownership: thread -> batch row b0 + cr, unit j0 + cu
    const int  cr = tid >> 4, cu = tid & 15;
    const bool cell = cr < nb;
    float      cst = 0.f, bia[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) bia[g] = h2f(a.bias[g * H + j0 + cu]);
    if (cell) cst = a.c[(long long)(b0 + cr) * H + j0 + cu];

    for (int t = 0; t < T; ++t) {
        const long long row0 = (long long)t * B + b0;
        // the input half of this thread's gate sums does not depend on the recurrence: request it ahead of the wait
        float gxv[4] = {0.f, 0.f, 0.f, 0.f};
        if (cell) {
#pragma unroll
            for (int g = 0; g < 4; ++g) gxv[g] = a.gx[(row0 + cr) * 4 * H + g * H + j0 + cu];
        }
        if (t > 0 && !grid_wait(sync, t, &verdict)) return;  // every workgroup's slice of h_{t-1} (these rows) is in memory
        const uint16_t* hprev = a.xh + row0 * a.ldxh + I;
        u32x4           af[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            af[ks] = u32x4{0u, 0u, 0u, 0u};
            if (ks < nks && lr < nb) af[ks] = *reinterpret_cast<const u32x4*>(hprev + (long long)lr * a.ldxh + k0 + 32 * ks);
        }
        f32x4 acc[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks < nks) {
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_frag(wf[g][ks]), as_frag(af[ks]), acc[g], 0, 0, 0);
            }
        }
        // acc[g][r] = partial sum of gate g, unit 4 lq + r, batch row lr
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][lr][16 * g + 4 * lq + r] = acc[g][r];
        __syncthreads();
        if (cell) {
            uint16_t g16[4], h16;
            float    gs[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int   n = 16 * g + cu;
                const float s = ((red[0][cr][n] + red[1][cr][n]) + red[2][cr][n]) + red[3][cr][n];
                g16[g]        = f2h((s + gxv[g]) + bia[g]);  // the gate sum's one rounding to storage
                gs[g]         = h2f(g16[g]);
            }
            cst = lstm_cell_forward(gs[0], gs[1], gs[2], gs[3], cst, &h16);
            const long long row = row0 + cr;
#pragma unroll
            for (int g = 0; g < 4; ++g) a.gates[row * 4 * H + g * H + j0 + cu] = g16[g];
            a.c[(row + B) * H + j0 + cu] = cst;
            if (t + 1 < T) a.xh[(row + B) * a.ldxh + I + j0 + cu] = h16;
            if (a.h_up != nullptr) a.h_up[row * a.ld_up + j0 + cu] = h16;
        }
        if (t + 1 < T) grid_arrive(sync, t + 1);  // (its workgroup barrier also keeps `red` of this step apart from the next)
    }
}

// ------------------------------------------------------------------------------------------------ backward
struct LstmBwdArgs {
    int             T, B, I, H;
    const uint16_t* w;         // [4H, ldw]
    int             ldw;
    const uint16_t* gates;     // [T*B, 4H]
    const float*    c;         // [(T+1)*B, H]
    const uint16_t* dh_above;  // [T*B, ld_above]: gradient reaching h_t from the layer above (or the loss)
    int             ld_above;
    uint16_t*       dgates;    // [T*B, 4H] out
    RlSync          sync;
};

__global__ __launch_bounds__(RL_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1))) void lstm_layer_bwd_kernel(LstmBwdArgs a) {
    __shared__ float red[4][16][17];  // per wave: partial recurrent gradient [batch row][unit]
    __shared__ int   verdict;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 15, lq = lane >> 4;
    const int H = a.H, I = a.I, B = a.B, T = a.T;
    const int j0  = blockIdx.x * RL_UNITS;
    const int b0  = blockIdx.y * RL_ROWS;
    const int nb  = min(RL_ROWS, B - b0);
    const int nks = H >> 5;                // this wave contracts over the H rows of gate block `wave`, 32 at a time
    const int n0  = wave * H + 8 * lq;     // first gate row of this lane's 8 consecutive values, + 32 ks
    RlSync    sync = a.sync;
    sync.flags += blockIdx.y * RL_FLAG_WORDS;

    // W_h^T fragments: unit lr, 8 consecutive gate rows n: W[n][I + j0 + lr] (a strided gather, once per launch)
    u32x4 wt[32];
#pragma unroll
    for (int ks = 0; ks < 32; ++ks) {
        wt[ks] = u32x4{0u, 0u, 0u, 0u};
        if (ks < nks) {
            const uint16_t* p = a.w + (long long)(n0 + 32 * ks) * a.ldw + I + j0 + lr;
            unsigned        q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                q[e] = (unsigned)p[(long long)(2 * e) * a.ldw] | ((unsigned)p[(long long)(2 * e + 1) * a.ldw] << 16);
            wt[ks] = u32x4{q[0], q[1], q[2], q[3]};
        }
    }

    const int  cr = tid >> 4, cu = tid & 15;
    const bool cell = cr < nb;
    float      dc = 0.f, dhrec = 0.f;

    // inputs of one cell-backward step for this thread's cell (they do not depend on the recurrence, so the next
    // step's are requested while the workgroup waits at the step barrier)
    struct CellIn {
        uint16_t gp[4], da;
        float    cp, cn;
    };
    auto load_cell = [&](int t) {
        CellIn q{};
        if (cell) {
            const long long row = (long long)t * B + b0 + cr;
#pragma unroll
            for (int g = 0; g < 4; ++g) q.gp[g] = a.gates[row * 4 * H + g * H + j0 + cu];
            q.cp = a.c[row * H + j0 + cu];
            q.cn = a.c[(row + B) * H + j0 + cu];
            q.da = a.dh_above[row * a.ld_above + j0 + cu];
        }
        return q;
    };
    CellIn in = load_cell(T - 1);

    for (int t = T - 1; t >= 0; --t) {
        const long long row0 = (long long)t * B + b0;
        if (cell) {
            uint16_t d4[4];
            dc = lstm_cell_backward(h2f(in.gp[0]), h2f(in.gp[1]), h2f(in.gp[2]), h2f(in.gp[3]), in.cp, in.cn, h2f(in.da) + dhrec, dc, d4);
#pragma unroll
            for (int g = 0; g < 4; ++g) a.dgates[(row0 + cr) * 4 * H + g * H + j0 + cu] = d4[g];
        }
        if (t == 0) break;
        const int step = T - t;                       // 1 .. T-1
        grid_arrive(sync, step);
        in = load_cell(t - 1);
        if (!grid_wait(sync, step, &verdict)) return;           // these rows of dgates_t are complete in memory
        // recurrent gradient of this workgroup's units: dgates_t[rows, 4H] W_h[:, j0 .. j0+16).  All of this lane's
        // pieces of dgates_t are requested at once (one memory latency), then multiplied.
        const uint16_t* dg = a.dgates + row0 * 4 * H;
        u32x4           af[32];
#pragma unroll
        for (int ks = 0; ks < 32; ++ks) {
            af[ks] = u32x4{0u, 0u, 0u, 0u};
            if (ks < nks && lr < nb) af[ks] = *reinterpret_cast<const u32x4*>(dg + (long long)lr * 4 * H + n0 + 32 * ks);
        }
        f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};  // two chains: even and odd steps
#pragma unroll
        for (int ks = 0; ks < 32; ++ks)
            if (ks < nks) acc[ks & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_frag(wt[ks]), as_frag(af[ks]), acc[ks & 1], 0, 0, 0);
        // acc[.][r] = partial sum for unit 4 lq + r, batch row lr
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][lr][4 * lq + r] = acc[0][r] + acc[1][r];
        __syncthreads();
        if (cell) {
            const float s = ((red[0][cr][cu] + red[1][cr][cu]) + red[2][cr][cu]) + red[3][cr][cu];
            dhrec         = round16(s);              // the recurrent gradient is a stored (fp16) tensor
        }
        // (`red` is next written behind the next step's barrier)
    }
}

}  // namespace mp

using namespace mp;

static int rl_check(const mp_lstm_layer_desc* d, const char* who, int* nwg) {
    MP_REQUIRE(d != nullptr, "%s: desc is NULL", who);
    MP_REQUIRE(d->T >= 1 && d->B >= 1 && d->I >= 0 && d->H >= 1, "%s: bad sizes T=%d B=%d I=%d H=%d", who, d->T, d->B, d->I, d->H);
    MP_REQUIRE(d->ldw >= d->I + d->H && d->ldxh >= d->I + d->H, "%s: leading dimension smaller than I + H", who);
    MP_REQUIRE(d->wait_limit_us >= 0 && d->debug_extra_participants >= 0 && d->debug_extra_participants <= 64,
               "%s: bad wait limit / debug participants", who);
    if (d->B > 32 || d->H % 128 != 0 || d->H > RL_MAX_H || d->I % 8 != 0 || d->ldw % 8 != 0 || d->ldxh % 8 != 0) {
        set_error("%s: the persistent kernel needs B <= 32, H a multiple of 128 up to %d, and I / ldw / ldxh multiples of 8 "
                  "(got B=%d H=%d I=%d ldw=%d ldxh=%d); run the layer step by step instead", who, RL_MAX_H, d->B, d->H, d->I,
                  d->ldw, d->ldxh);
        return MP_E_UNSUPPORTED;
    }
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_fail(e, who);
    *nwg = d->H / RL_UNITS;
    const int groups = (d->B + RL_ROWS - 1) / RL_ROWS;
    if (*nwg * groups > cus) {  // every workgroup must be resident at once, or the step barrier cannot complete
        set_error("%s: %d workgroups needed, the device has %d compute units", who, *nwg * groups, cus);
        return MP_E_UNSUPPORTED;
    }
    return MP_OK;
}

// step flags: two barrier groups (B <= 32 rows in blocks of 16) of up to 64 workgroups + 64 debug words each
extern "C" size_t mp_lstm_layer_workspace_bytes(void) { return 2 * RL_FLAG_WORDS * sizeof(int); }

static int rl_sync(const mp_lstm_layer_desc* d, int nwg, int32_t* status, void* ws, size_t ws_bytes, mp_stream stream,
                   const char* who, RlSync* out) {
    MP_REQUIRE(status != nullptr, "%s: status is NULL", who);
    if (!ws || ws_bytes < mp_lstm_layer_workspace_bytes() || (reinterpret_cast<uintptr_t>(ws) & 3u)) {
        set_error("%s: workspace of %zu bytes needed, %zu given", who, mp_lstm_layer_workspace_bytes(), ws_bytes);
        return MP_E_WORKSPACE;
    }
    const int rc = mp_fill_u32(mp_lstm_layer_workspace_bytes() / 4, 0u, ws, stream);  // flags start at zero (a kernel: capturable)
    if (rc != MP_OK) return rc;
    out->flags       = static_cast<int*>(ws);
    out->status      = status;
    out->nwait       = nwg + d->debug_extra_participants;
    out->limit_ticks = (d->wait_limit_us > 0 ? (long long)d->wait_limit_us : 2000000ll) * 100;  // 100 MHz clock
    return MP_OK;
}

extern "C" int mp_lstm_layer_fwd(const mp_lstm_layer_desc* d, const float* gx, const mp_half* w, const mp_half* bias,
                                 mp_half* gates, float* c, mp_half* xh, mp_half* h_up, int32_t* status, void* ws,
                                 size_t ws_bytes, mp_stream stream) {
    int nwg = 0;
    int rc  = rl_check(d, "mp_lstm_layer_fwd", &nwg);
    if (rc) return rc;
    MP_REQUIRE(gx && w && bias && gates && c && xh, "mp_lstm_layer_fwd: NULL argument");
    MP_REQUIRE(h_up == nullptr || (d->ld_up >= d->H && d->ld_up % 2 == 0), "mp_lstm_layer_fwd: ld_up=%d must be even and >= H", d->ld_up);
    MP_REQUIRE(aligned16(w) && aligned16(xh) && aligned16(gx) && aligned16(gates) && aligned16(c) && (h_up == nullptr || aligned16(h_up)),
               "mp_lstm_layer_fwd: pointers must be 16-byte aligned");
    LstmFwdArgs a{};
    rc = rl_sync(d, nwg, status, ws, ws_bytes, stream, "mp_lstm_layer_fwd", &a.sync);
    if (rc) return rc;
    a.T = d->T; a.B = d->B; a.I = d->I; a.H = d->H;
    a.gx = gx; a.w = w; a.ldw = d->ldw; a.bias = bias; a.gates = gates; a.c = c; a.xh = xh; a.ldxh = d->ldxh;
    a.h_up = h_up; a.ld_up = d->ld_up;
    hipLaunchKernelGGL(lstm_layer_fwd_kernel, dim3(nwg, (d->B + RL_ROWS - 1) / RL_ROWS), dim3(RL_THREADS), 0, as_stream(stream), a);
    MP_LAUNCH_CHECK("mp_lstm_layer_fwd");
    return MP_OK;
}

extern "C" int mp_lstm_layer_bwd(const mp_lstm_layer_desc* d, const mp_half* w, const mp_half* gates, const float* c,
                                 const mp_half* dh_above, mp_half* dgates, int32_t* status, void* ws, size_t ws_bytes,
                                 mp_stream stream) {
    int nwg = 0;
    int rc  = rl_check(d, "mp_lstm_layer_bwd", &nwg);
    if (rc) return rc;
    MP_REQUIRE(w && gates && c && dh_above && dgates, "mp_lstm_layer_bwd: NULL argument");
    MP_REQUIRE(d->ld_up >= d->H && d->ld_up % 2 == 0, "mp_lstm_layer_bwd: ld_up=%d (leading dimension of dh_above) must be even and >= H", d->ld_up);
    MP_REQUIRE(aligned16(w) && aligned16(gates) && aligned16(c) && aligned16(dh_above) && aligned16(dgates),
               "mp_lstm_layer_bwd: pointers must be 16-byte aligned");
    LstmBwdArgs a{};
    rc = rl_sync(d, nwg, status, ws, ws_bytes, stream, "mp_lstm_layer_bwd", &a.sync);
    if (rc) return rc;
    a.T = d->T; a.B = d->B; a.I = d->I; a.H = d->H;
    a.w = w; a.ldw = d->ldw; a.gates = gates; a.c = c; a.dh_above = dh_above; a.ld_above = d->ld_up; a.dgates = dgates;
    hipLaunchKernelGGL(lstm_layer_bwd_kernel, dim3(nwg, (d->B + RL_ROWS - 1) / RL_ROWS), dim3(RL_THREADS), 0, as_stream(stream), a);
    MP_LAUNCH_CHECK("mp_lstm_layer_bwd");
    return MP_OK;
}
