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
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

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

// The exchange of the small-batch persistent kernels without their arithmetic: the launch is `groups` independent
// groups (the layers of a launch) of G workgroups; the workgroups of a group hold `words` tagged 64-bit words
// between them; in every step each publishes its share for that step (device-scope stores of the step's
// tag and a payload), then all four waves of every workgroup fetch the whole vector (device-scope 16-byte loads, a
// quarter per wave) until every tag is the step's, and join at a barrier.  Every step has its own slot, as in a
// state sequence.  A wait gives up after `spin_limit` polls and raises *status, after which the workgroup leaves;
// the others then give up the same way, so the grid always drains.
__global__ __launch_bounds__(256, 1) void exchange_step_kernel(uint64_t* all_seq, int G, int words, int steps,
                                                               uint32_t tag0, unsigned spin_limit, unsigned* status,
                                                               unsigned long long* stamps) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int group = blockIdx.x / G, member = blockIdx.x % G;
    const int per = words / G, quarter = words / 4;
    uint64_t* seq = all_seq + (size_t)group * (steps + 1) * words;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        seq, 0, (int)((size_t)(steps + 1) * words * 8), 0x00020000);
    const unsigned long long t0 = clock64();
    for (int s = 1; s <= steps; ++s) {
        const uint32_t tag = tag0 + (uint32_t)s;
        if (wave == 0 && lane < per)
            __hip_atomic_store(seq + (size_t)s * words + member * per + lane,
                               ((uint64_t)tag << 32) | (uint32_t)(member * per + lane), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        bool done = false;
        unsigned polls = 0;
        while (!done && polls < spin_limit) {
            bool ok = true;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i * 128 < quarter) {                      // uniform
                    int f = i * 128 + 2 * lane;
                    if (f >= quarter) f = quarter - 2;        // past the end: the last pair again, in bounds
                    const uint32_t off = (uint32_t)(((size_t)s * words + wave * quarter + f) * 8);
                    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 16 /* sc1 */);
                    ok = ok && v[1] == tag && v[3] == tag;
                }
            }
            done = __all(ok);
            ++polls;
        }
        if (__syncthreads_or(done ? 0 : 1)) {                 // some wave of this workgroup gave up
            if (threadIdx.x == 0) __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) stamps[0] = clock64() - t0;
}

}  // namespace
}  // namespace rnn

extern "C" int rnn_probe_exchange_step(int groups, int workgroups, int words, int steps, double* us_per_step,
                                       double* clocks_per_step, void* stream) {
    using namespace rnn;
    if (groups < 1 || groups > 64 || workgroups < 1 || words < 8 || words > 2048 || words % 8 != 0 || steps < 1 || steps > 100000 ||
        words % workgroups != 0 || words / workgroups > 64 || !us_per_step || !clocks_per_step)
        return RNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) return RNN_EDEVICE;
    if (cap != hipStreamCaptureStatusNone) return RNN_EUNSUPPORTED;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return RNN_EDEVICE;
    if (groups * workgroups > cus) return RNN_EINVAL;      // every workgroup must be resident: they wait for each other
    const size_t seq_bytes = (size_t)groups * (steps + 1) * words * 8;
    unsigned char* buf = nullptr;
    if (hipMalloc((void**)&buf, seq_bytes + 256) != hipSuccess) return RNN_ENOMEM;
    uint64_t* seq = (uint64_t*)buf;
    unsigned* status = (unsigned*)(buf + seq_bytes);
    unsigned long long* stamps = (unsigned long long*)(buf + seq_bytes + 64);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = RNN_EDEVICE;
    float ms = 0.0f;
    unsigned long long clocks = 0;
    unsigned gave_up = 0;
    do {
        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
        // two passes over the same slots with different tags (no word of the first pass can pass for one of the second)
        if (hipMemsetAsync(buf, 0, seq_bytes + 256, st) != hipSuccess) break;
        exchange_step_kernel<<<dim3(groups * workgroups), dim3(256), 0, st>>>(seq, workgroups, words, steps, 0x10000000u, 1u << 22, status, stamps);
        if (hipEventRecord(e0, st) != hipSuccess) break;
        exchange_step_kernel<<<dim3(groups * workgroups), dim3(256), 0, st>>>(seq, workgroups, words, steps, 0x20000000u, 1u << 22, status, stamps);
        if (hipEventRecord(e1, st) != hipSuccess) break;
        if (hipGetLastError() != hipSuccess) break;
        if (hipStreamSynchronize(st) != hipSuccess) break;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) break;
        if (hipMemcpy(&clocks, stamps, sizeof(clocks), hipMemcpyDeviceToHost) != hipSuccess) break;
        if (hipMemcpy(&gave_up, status, sizeof(gave_up), hipMemcpyDeviceToHost) != hipSuccess) break;
        rc = gave_up ? RNN_EDEVICE : RNN_OK;
    } while (0);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(buf);
    if (rc != RNN_OK) return rc;
    *us_per_step = (double)ms * 1e3 / steps;
    *clocks_per_step = (double)clocks / steps;
    return RNN_OK;
}

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
