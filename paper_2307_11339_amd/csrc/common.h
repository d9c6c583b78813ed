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

}  // namespace rnn
