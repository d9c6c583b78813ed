// State set-up kernels and the pointwise half of the cellwise plan.
//
// The cellwise plan executes the unrolled cell grid one cell after another on one stream, the
// regime the paper attributes to a single GPU (Section 2.2, caption of the unfolded-RNN
// figure): per cell one recurrent product (gemm.hip, M = batch) and one launch of the kernel
// below, which adds the projection, applies the gate functions and updates the state.  The GRU
// that applies the reset gate before the candidate's recurrent product needs two products per
// cell with a pointwise kernel between them.
#include "common.h"
#include "kernels.h"

namespace rnn {
namespace {

template <int DT>
__global__ void state_init_kernel(const float* h0, const float* c0, float* h_f32, float* c_f32,
                                  void* h_st, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float h = h0 ? h0[i] : 0.0f;
    h_f32[i] = h;
    c_f32[i] = c0 ? c0[i] : 0.0f;
    if (DT == DT_BF16) ((bf16_t*)h_st)[i] = f32_to_bf16(h);
    else ((float*)h_st)[i] = h;
}

__global__ void state_export_kernel(const float* h_f32, const float* c_f32, float* hT, float* cT,
                                    size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (hT) hT[i] = h_f32[i];
    if (cT) cT[i] = c_f32[i];
}

template <int CELL, int DT>
__global__ void cell_step_kernel(CellStepArgs a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;  // (b, u)
    if (i >= a.B * a.H) return;
    const int b = i / a.H, u = i % a.H;
    int len = a.T;
    if (a.lengths) len = min(max(a.lengths[b], 0), a.T);
    const bool active = a.t < len;
    const size_t orow = ((size_t)a.t * a.B + b) * a.D * a.H + (size_t)a.d * a.H + u;
    if (!active) {  // state is held, the padded output position is +0.0
        if (DT == DT_BF16) ((bf16_t*)a.out)[orow] = 0;
        else ((float*)a.out)[orow] = 0.0f;
        return;
    }
    const float4 gx = *reinterpret_cast<const float4*>(
        a.gx + ((((size_t)a.t * a.B + b) * a.D + a.d) * a.H + u) * SLOTS);
    const float4 gh = *reinterpret_cast<const float4*>(a.gh + ((size_t)b * a.H + u) * SLOTS);
    const float4 bs = *reinterpret_cast<const float4*>(a.bias + (size_t)u * SLOTS);
    const float pre[SLOTS] = {gx.x + gh.x + bs.x, gx.y + gh.y + bs.y, gx.z + gh.z + bs.z,
                              gx.w + gh.w + bs.w};
    float c = a.c_f32[i];
    float h;
    if (CELL == CELL_GRU && a.gh_rh) {
        // the candidate's recurrent part was computed from r * h_{t-1}: nothing left to scale
        const float nh = a.gh_rh[((size_t)b * a.H + u) * SLOTS + 3] + bs.w;
        const float z = sigmoid_f(pre[1]);
        const float n = tanh_f(pre[2] + nh);
        h = (1.0f - z) * n + z * a.h_f32[i];
    } else {
        h = cell_update<CELL>(pre, a.h_f32[i], c);
    }
    if (DT == DT_BF16) {
        const bf16_t hb = f32_to_bf16(h);
        h = bf16_to_f32(hb);
        ((bf16_t*)a.h_st)[i] = hb;
        ((bf16_t*)a.out)[orow] = hb;
    } else {
        ((float*)a.h_st)[i] = h;
        ((float*)a.out)[orow] = h;
    }
    a.h_f32[i] = h;
    a.c_f32[i] = c;
}

template <int DT>
__global__ void gru_reset_kernel(CellStepArgs a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;  // (b, u)
    if (i >= a.B * a.H) return;
    const int b = i / a.H, u = i % a.H;
    const size_t g = ((((size_t)a.t * a.B + b) * a.D + a.d) * a.H + u) * SLOTS;
    const float r = sigmoid_f(a.gx[g] + a.gh[((size_t)b * a.H + u) * SLOTS] + a.bias[(size_t)u * SLOTS]);
    const float rh = r * a.h_f32[i];
    if (DT == DT_BF16) ((bf16_t*)a.rh_st)[i] = f32_to_bf16(rh);
    else ((float*)a.rh_st)[i] = rh;
}

}  // namespace

hipError_t launch_gru_reset(const CellStepArgs& a, hipStream_t stream) {
    const unsigned blocks = (unsigned)(((size_t)a.B * a.H + 255) / 256);
    if (a.dtype == DT_BF16) gru_reset_kernel<DT_BF16><<<blocks, 256, 0, stream>>>(a);
    else gru_reset_kernel<DT_F32><<<blocks, 256, 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_state_init(int dtype, const float* h0, const float* c0, float* h_f32,
                             float* c_f32, void* h_st, size_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (dtype == DT_BF16)
        state_init_kernel<DT_BF16><<<blocks, 256, 0, stream>>>(h0, c0, h_f32, c_f32, h_st, n);
    else
        state_init_kernel<DT_F32><<<blocks, 256, 0, stream>>>(h0, c0, h_f32, c_f32, h_st, n);
    return hipGetLastError();
}

hipError_t launch_state_export(const float* h_f32, const float* c_f32, float* hT, float* cT,
                               size_t n, hipStream_t stream) {
    if (n == 0 || (!hT && !cT)) return hipSuccess;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    state_export_kernel<<<blocks, 256, 0, stream>>>(h_f32, c_f32, hT, cT, n);
    return hipGetLastError();
}

hipError_t launch_cell_step(const CellStepArgs& a, hipStream_t stream) {
    const unsigned blocks = (unsigned)(((size_t)a.B * a.H + 255) / 256);
    if (a.cell == CELL_LSTM) {
        if (a.dtype == DT_BF16) cell_step_kernel<CELL_LSTM, DT_BF16><<<blocks, 256, 0, stream>>>(a);
        else cell_step_kernel<CELL_LSTM, DT_F32><<<blocks, 256, 0, stream>>>(a);
    } else {
        if (a.dtype == DT_BF16) cell_step_kernel<CELL_GRU, DT_BF16><<<blocks, 256, 0, stream>>>(a);
        else cell_step_kernel<CELL_GRU, DT_F32><<<blocks, 256, 0, stream>>>(a);
    }
    return hipGetLastError();
}

}  // namespace rnn
