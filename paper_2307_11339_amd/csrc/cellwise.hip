// State set-up kernels and the pointwise half of the cellwise plan.
//
// The cellwise plan executes the unrolled cell grid one cell after another on one stream, the
// regime the paper attributes to a single GPU (Section 2.2, caption of the unfolded-RNN
// figure): per cell one recurrent product (gemm.hip, M = batch) and one launch of the kernel
// below, which adds the projection, applies the gate functions and updates the state.  The GRU
// that applies the reset gate before the candidate's recurrent product needs two products per
// cell with a pointwise kernel between them.  The optional terms of the ONNX operators (peephole
// weights, clipping threshold) exist in this plan only.  Also here: the kernel that changes the
// layout of x and y for batch-first callers (used with every plan).
#include <algorithm>

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

// clip = 0: no clipping
__device__ inline float limit(float v, float clip) { return clip > 0.0f ? fminf(fmaxf(v, -clip), clip) : v; }

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
        const float z = sigmoid_f(limit(pre[1], a.clip));
        const float n = tanh_f(limit(pre[2] + nh, a.clip));
        h = (1.0f - z) * n + z * a.h_f32[i];
    } else if (a.peep != nullptr || a.clip > 0.0f) {
        const CellExt e = load_cell_ext(CELL == CELL_LSTM ? a.peep : nullptr, a.H, u, a.clip);
        h = cell_update_ext<CELL>(pre, a.h_f32[i], c, e);
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
    const float r = sigmoid_f(limit(a.gx[g] + a.gh[((size_t)b * a.H + u) * SLOTS] + a.bias[(size_t)u * SLOTS], a.clip));
    const float rh = r * a.h_f32[i];
    if (DT == DT_BF16) ((bf16_t*)a.rh_st)[i] = f32_to_bf16(rh);
    else ((float*)a.rh_st)[i] = rh;
}

__global__ void fill_zero_kernel(uint32_t* __restrict__ p, size_t words) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

template <class V>
__global__ void copy_2d_kernel(const char* __restrict__ src, size_t src_pitch, char* __restrict__ dst, size_t dst_pitch,
                               int rows, int units) {
    const size_t total = (size_t)rows * units;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t r = e / units, q = e - r * units;
        reinterpret_cast<V*>(dst + r * dst_pitch)[q] = reinterpret_cast<const V*>(src + r * src_pitch)[q];
    }
}

// dst[j][i][:] = src[i][j][:], rows of `units` elements of type V
template <class V>
__global__ void swap_outer_kernel(const V* __restrict__ src, V* __restrict__ dst, int n0, int n1, int units) {
    const size_t total = (size_t)n0 * n1 * units;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t row = e / units, q = e - row * units;       // row of dst = j * n0 + i
        const size_t j = row / n0, i = row - j * n0;
        dst[e] = src[(i * n1 + j) * units + q];
    }
}

}  // namespace

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream) {
    if (bytes == 0) return hipSuccess;
    if (!p || (bytes & 3) || ((uintptr_t)p & 3)) return hipErrorInvalidValue;
    const size_t words = bytes / 4;
    const unsigned blocks = (unsigned)std::min<size_t>((words + 255) / 256, 256 * 32);
    fill_zero_kernel<<<blocks, 256, 0, stream>>>((uint32_t*)p, words);
    return hipGetLastError();
}

hipError_t launch_copy_2d(const void* src, size_t src_pitch, void* dst, size_t dst_pitch, int rows, size_t row_bytes,
                          hipStream_t stream) {
    if (rows < 1 || row_bytes == 0) return hipSuccess;
    if (!src || !dst || (row_bytes & 1)) return hipErrorInvalidValue;
    const uintptr_t all = (uintptr_t)src | (uintptr_t)dst | src_pitch | dst_pitch | row_bytes;
    const size_t unit = (all & 15) == 0 ? 16 : (all & 3) == 0 ? 4 : 2;
    if (all & (unit - 1)) return hipErrorInvalidValue;
    const int units = (int)(row_bytes / unit);
    const size_t total = (size_t)rows * units;
    const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 256 * 64);
    const char* s = (const char*)src;
    char* d = (char*)dst;
    if (unit == 16) copy_2d_kernel<uint4><<<blocks, 256, 0, stream>>>(s, src_pitch, d, dst_pitch, rows, units);
    else if (unit == 4) copy_2d_kernel<uint32_t><<<blocks, 256, 0, stream>>>(s, src_pitch, d, dst_pitch, rows, units);
    else copy_2d_kernel<uint16_t><<<blocks, 256, 0, stream>>>(s, src_pitch, d, dst_pitch, rows, units);
    return hipGetLastError();
}

hipError_t launch_swap_outer(const void* src, void* dst, int n0, int n1, size_t row_bytes, hipStream_t stream) {
    if (n0 < 1 || n1 < 1 || row_bytes == 0 || (row_bytes & 1)) return hipErrorInvalidValue;
    const bool a16 = (((uintptr_t)src | (uintptr_t)dst | row_bytes) & 15) == 0;
    const bool a4 = (((uintptr_t)src | (uintptr_t)dst | row_bytes) & 3) == 0;
    const size_t unit = a16 ? 16 : a4 ? 4 : 2;
    const size_t total = (size_t)n0 * n1 * (row_bytes / unit);
    const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 256 * 64);
    const int units = (int)(row_bytes / unit);
    if (a16) swap_outer_kernel<uint4><<<blocks, 256, 0, stream>>>((const uint4*)src, (uint4*)dst, n0, n1, units);
    else if (a4) swap_outer_kernel<uint32_t><<<blocks, 256, 0, stream>>>((const uint32_t*)src, (uint32_t*)dst, n0, n1, units);
    else swap_outer_kernel<uint16_t><<<blocks, 256, 0, stream>>>((const uint16_t*)src, (uint16_t*)dst, n0, n1, units);
    return hipGetLastError();
}

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
