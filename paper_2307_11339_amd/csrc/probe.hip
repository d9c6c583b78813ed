// Measurement aid: what the matrix cores of this GPU sustain, and at which shader clock, when a given number of
// compute units run nothing but dense bf16 matrix instructions.  The published peak of the chip assumes its highest
// clock; under a chip-wide matrix load the clock is lower, and the rate this probe reports is the ceiling that the
// contraction kernels (the recurrent kernels' products, the input projection) can be compared with.
#include "../../include/rnn.h"
#include "common.h"

namespace rnn {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// One workgroup of 4 waves per compute unit, one wave per SIMD: 16 independent 32 x 32 accumulators per wave (the
// register layout of a 128 x 128 wave tile), fragments fixed in registers, `iterations` rounds of 64 instructions.
// stamps[0..1] (workgroup 0): shader clocks and 100 MHz ticks spent in the loop.
__global__ __launch_bounds__(256, 1) void matrix_rate_kernel(float* sink, unsigned long long* stamps, int iterations,
                                                             float seed) {
    const int lane = threadIdx.x & 63;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[j][e] = (__bf16)(seed * (float)((lane * 7 + j * 3 + e) % 29 - 14));
            b[j][e] = (__bf16)(seed * (float)((lane * 5 + j * 11 + e) % 31 - 15));
        }
    f32x16 c[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) c[i][j][e] = 0.0f;
    const unsigned long long t0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + r) & 3], b[j], c[i][j], 0, 0, 0);
    }
    const unsigned long long t1 = clock64(), w1 = wall_clock64();
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) s += c[i][j][e];
    if (s == 1.2345e30f) sink[0] = s;                         // keeps the products alive; never true
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        stamps[0] = t1 - t0;
        stamps[1] = w1 - w0;
    }
}

}  // namespace
}  // namespace rnn

extern "C" int rnn_probe_matrix_rate(int compute_units, int iterations, double* clocks_per_instruction,
                                     double* shader_ghz, double* tflops, void* stream) {
    using namespace rnn;
    if (compute_units < 1 || compute_units > 4096 || iterations < 1 || iterations > (1 << 20) ||
        !clocks_per_instruction || !shader_ghz || !tflops)
        return RNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) return RNN_EDEVICE;
    if (cap != hipStreamCaptureStatusNone) return RNN_EUNSUPPORTED;   // allocates, synchronises and reads back
    unsigned char* buf = nullptr;
    if (hipMalloc((void**)&buf, 256) != hipSuccess) return RNN_ENOMEM;
    float* sink = (float*)buf;
    unsigned long long* stamps = (unsigned long long*)(buf + 64);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = RNN_EDEVICE;
    float ms = 0.0f;
    unsigned long long h[2] = {0, 0};
    do {
        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
        // an untimed pass of the same length first: the clock settles over tens of milliseconds
        matrix_rate_kernel<<<dim3(compute_units), dim3(256), 0, st>>>(sink, stamps, iterations, 0.01f);
        if (hipEventRecord(e0, st) != hipSuccess) break;
        matrix_rate_kernel<<<dim3(compute_units), dim3(256), 0, st>>>(sink, stamps, iterations, 0.01f);
        if (hipEventRecord(e1, st) != hipSuccess) break;
        if (hipGetLastError() != hipSuccess) break;
        if (hipStreamSynchronize(st) != hipSuccess) break;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) break;
        if (hipMemcpy(h, stamps, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) break;
        rc = RNN_OK;
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(buf);
    if (rc != RNN_OK) return rc;
    const double n = (double)iterations * 64.0;              // instructions per wave
    *clocks_per_instruction = (double)h[0] / n;
    *shader_ghz = h[1] ? (double)h[0] / (double)h[1] * 0.1 : 0.0;
    *tflops = ms > 0.0f ? (double)compute_units * 4.0 * n * 32768.0 / ((double)ms * 1e-3) / 1e12 : 0.0;
    return RNN_OK;
}
