// LSTM cell arithmetic shared by the per-step cell kernels and the persistent recurrent-layer kernels: fp32 between
// fp16 storage points, the cell state never rounded (paper Section 3.2: explicitly fp32 parts of a mixed-precision
// model).  One definition, so that a layer gives the same bits whichever of the two paths runs it.
#pragma once
#include "common.hpp"

namespace mp {

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + __expf(-x)); }

// gi, gf, gg, go: the STORED (fp16) gate sums of one cell.  Returns c_t; *h16 = RNE16(sigma(o) tanh(c_t)).
__device__ __forceinline__ float lstm_cell_forward(float gi, float gf, float gg, float go, float c_prev, uint16_t* h16) {
    const float cn = sigmoidf_(gf) * c_prev + sigmoidf_(gi) * tanhf(gg);
    *h16           = f2h(sigmoidf_(go) * tanhf(cn));
    return cn;
}

// Backward of one cell for one time step.  dh: fp32 sum of the gradients reaching h_t; dc_in: cell-state gradient
// carried from step t + 1.  Writes RNE16 of (di, df, dg, do) and returns the cell-state gradient carried to t - 1.
__device__ __forceinline__ float lstm_cell_backward(float gi, float gf, float gg, float go, float c_prev, float c,
                                                    float dh, float dc_in, uint16_t* d4) {
    const float si = sigmoidf_(gi), sf = sigmoidf_(gf), tg = tanhf(gg), so = sigmoidf_(go);
    const float tc  = tanhf(c);
    const float d_o = dh * tc * so * (1.0f - so);
    const float dc  = dc_in + dh * so * (1.0f - tc * tc);
    const float d_i = dc * tg * si * (1.0f - si);
    const float d_f = dc * c_prev * sf * (1.0f - sf);
    const float d_g = dc * si * (1.0f - tg * tg);
    d4[0] = f2h(d_i);
    d4[1] = f2h(d_f);
    d4[2] = f2h(d_g);
    d4[3] = f2h(d_o);
    return dc * sf;
}

}  // namespace mp
