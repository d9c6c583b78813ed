// Shared device/host helpers of the gfx950 RNN library: bf16 conversion, gate functions,
// packed-layout constants.  Nothing in here is used by the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rnn {

// A hidden unit always owns SLOTS consecutive pre-activation values in the packed layouts:
//   LSTM: i, f, g, o
//   GRU : r, z, n_x, n_h   (n_x = input part of the candidate incl. b_in,
//                           n_h = recurrent part incl. b_hn, scaled by r before the tanh)
constexpr int SLOTS = 4;

enum : int { CELL_LSTM = 0, CELL_GRU = 1 };
enum : int { DT_F32 = 0, DT_BF16 = 1 };

typedef uint16_t bf16_t;  // raw bf16 bits

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
    union { uint32_t u; float f; } v;
    v.u = (uint32_t)b << 16;
    return v.f;
}

// round to nearest even; inputs are finite in this library
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
    union { uint32_t u; float f; } v;
    v.f = f;
    uint32_t lsb = (v.u >> 16) & 1u;
    return (bf16_t)((v.u + 0x7FFFu + lsb) >> 16);
}

__device__ inline float round_bf16(float f) { return bf16_to_f32(f32_to_bf16(f)); }

// v_rcp_f32 and v_exp_f32 are accurate to about 1 ulp, far inside the parity tolerances
__device__ inline float sigmoid_f(float a) { return __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }

// tanh(a) = 1 - 2 / (exp(2a) + 1); saturates cleanly to +-1 when exp overflows or underflows
__device__ inline float tanh_f(float a) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(__expf(2.0f * a) + 1.0f);
}

// One cell update from the four slot pre-activations (bias already added).
// Returns the new h (not yet rounded to the storage type); c is updated in place (LSTM only).
template <int CELL>
__device__ inline float cell_update(const float a[SLOTS], float h_prev, float& c) {
    if (CELL == CELL_LSTM) {
        const float ig = sigmoid_f(a[0]);
        const float fg = sigmoid_f(a[1]);
        const float gg = tanh_f(a[2]);
        const float og = sigmoid_f(a[3]);
        c = fg * c + ig * gg;
        return og * tanh_f(c);
    } else {
        const float r = sigmoid_f(a[0]);
        const float z = sigmoid_f(a[1]);
        const float n = tanh_f(a[2] + r * a[3]);
        return (1.0f - z) * n + z * h_prev;
    }
}

// The optional terms of the ONNX LSTM / GRU operators for one hidden unit: peephole weights (LSTM: i and f
// see c_{t-1}, o sees the new c_t) and the bound on the argument of every gate activation (never on the cell
// state inside o * tanh(c)).  The plain cell is {0, 0, 0, +infinity}: a + 0 * c == a and a value limited to
// [-inf, +inf] is itself, so one code path serves both and gives the plain cell's bits when the terms are off.
struct CellExt {
    float p_i, p_f, p_o;   // peephole weights of this unit (0 for a GRU)
    float lim;             // clipping threshold, +infinity for none
};

__device__ inline float limit_to(float v, float lim) { return fminf(fmaxf(v, -lim), lim); }

template <int CELL>
__device__ inline float cell_update_ext(const float a[SLOTS], float h_prev, float& c, const CellExt& e) {
    if (CELL == CELL_LSTM) {
        const float ig = sigmoid_f(limit_to(a[0] + e.p_i * c, e.lim));
        const float fg = sigmoid_f(limit_to(a[1] + e.p_f * c, e.lim));
        const float gg = tanh_f(limit_to(a[2], e.lim));
        c = fg * c + ig * gg;
        const float og = sigmoid_f(limit_to(a[3] + e.p_o * c, e.lim));
        return og * tanh_f(c);
    } else {
        const float r = sigmoid_f(limit_to(a[0], e.lim));
        const float z = sigmoid_f(limit_to(a[1], e.lim));
        const float n = tanh_f(limit_to(a[2] + r * a[3], e.lim));
        return (1.0f - z) * n + z * h_prev;
    }
}

// CellExt of hidden unit `unit`: peep = NULL or [3, H] (p_i, p_f, p_o), clip = 0 for none.
__device__ inline CellExt load_cell_ext(const float* peep, int H, int unit, float clip) {
    CellExt e;
    e.p_i = peep ? peep[unit] : 0.0f;
    e.p_f = peep ? peep[H + unit] : 0.0f;
    e.p_o = peep ? peep[2 * H + unit] : 0.0f;
    e.lim = clip > 0.0f ? clip : __builtin_inff();
    return e;
}

}  // namespace rnn
