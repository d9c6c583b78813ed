// Input-projection GEMM for gfx950:  C[m, n] = sum_k A[m, k] * W[n, k]   (both operands K-contiguous).
//
// In the unrolled cell grid every cell (l, t) consumes x_t (paper, Section 2.2); that part of
// the cell has no recurrent dependency, so it is computed for all time steps at once as one
// dense contraction: rows m = (t, b) pairs, columns n = packed gate rows of W_ih.
//
// bf16 path: 32x32x16 bf16 MFMA, fp32 accumulate.  A workgroup of 256 threads (4 waves, 2x2)
// owns a BM x BN tile of C; the K loop moves BK-wide slabs of A and W through LDS.
// fp32 path: plain FMA tiles (only the small fp32 workloads use it).
#include "common.h"
#include "kernels.h"

namespace rnn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

constexpr int BK = 64;              // K slab per iteration (bf16 elements)
constexpr int LDS_ROW = BK + 8;     // padded LDS row (elements): 144 B keeps 16 B alignment

// Tile BM x BN, 4 waves arranged 2 (m) x 2 (n); each wave owns (BM/2) x (BN/2).
template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_bf16_nt_kernel(const bf16_t* __restrict__ A, int lda,
                                                           const bf16_t* __restrict__ W, int ldw,
                                                           float* __restrict__ C, int ldc, int M,
                                                           int N, int K, int tiles_n) {
    constexpr int WM = BM / 2, WN = BN / 2;     // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;   // MFMA tiles per wave
    constexpr int A_CHUNKS = BM * (BK / 8) / 256;  // 16-byte chunks per thread
    constexpr int W_CHUNKS = BN * (BK / 8) / 256;
    __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LDS_ROW];
    __shared__ __attribute__((aligned(16))) bf16_t sW[BN * LDS_ROW];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    // consecutive workgroups walk down the M tiles of one N tile, so the workgroups that are
    // resident together share the same slab of W and stream disjoint rows of A
    const int tile_n = blockIdx.x % tiles_n;
    const int tile_m = blockIdx.x / tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    u32x4 ra[A_CHUNKS], rw[W_CHUNKS];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + i * 256;
            const int row = c / (BK / 8), kc = c % (BK / 8);
            const int m = m0 + row, k = k0 + kc * 8;
            u32x4 v = {0, 0, 0, 0};
            if (m < M && k < K) v = *reinterpret_cast<const u32x4*>(A + (size_t)m * lda + k);
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) {
            const int c = tid + i * 256;
            const int row = c / (BK / 8), kc = c % (BK / 8);
            const int n = n0 + row, k = k0 + kc * 8;
            u32x4 v = {0, 0, 0, 0};
            if (n < N && k < K) v = *reinterpret_cast<const u32x4*>(W + (size_t)n * ldw + k);
            rw[i] = v;
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int c = tid + i * 256;
            const int row = c / (BK / 8), kc = c % (BK / 8);
            *reinterpret_cast<u32x4*>(&sA[row * LDS_ROW + kc * 8]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < W_CHUNKS; ++i) {
            const int c = tid + i * 256;
            const int row = c / (BK / 8), kc = c % (BK / 8);
            *reinterpret_cast<u32x4*>(&sW[row * LDS_ROW + kc * 8]) = rw[i];
        }
    };

    load_global(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();  // previous slab fully consumed
        store_lds();
        __syncthreads();
        if (k0 + BK < K) load_global(k0 + BK);  // overlaps with the MFMAs below
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[TM], fw[TN];
            const int kof = ks * 16 + 8 * (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(
                    &sA[(wm * WM + i * 32 + (lane & 31)) * LDS_ROW + kof]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fw[j] = *reinterpret_cast<const bf16x8*>(
                    &sW[(wn * WN + j * 32 + (lane & 31)) * LDS_ROW + kof]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fw[j], acc[i][j], 0, 0, 0);
        }
    }

    // acc[i][j][e]: row = 8*(e/4) + 4*(lane/32) + e%4, column = lane%32 of the 32x32 tile
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * WM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m < M && n < N) C[(size_t)m * ldc + n] = acc[i][j][e];
            }
        }
}

// fp32: 64x64 tile, 256 threads, each thread a 4x4 micro-tile; K slabs of 16 through LDS.
__global__ __launch_bounds__(256) void gemm_f32_nt_kernel(const float* __restrict__ A, int lda,
                                                          const float* __restrict__ W, int ldw,
                                                          float* __restrict__ C, int ldc, int M,
                                                          int N, int K, int tiles_n) {
    constexpr int T = 64, KS = 16;
    __shared__ float sA[KS][T + 1];
    __shared__ float sW[KS][T + 1];
    const int tid = threadIdx.x;
    const int tile_n = blockIdx.x % tiles_n, tile_m = blockIdx.x / tiles_n;
    const int m0 = tile_m * T, n0 = tile_n * T;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += KS) {
        for (int i = tid; i < T * KS; i += 256) {
            const int r = i / KS, k = i % KS;
            sA[k][r] = (m0 + r < M && k0 + k < K) ? A[(size_t)(m0 + r) * lda + k0 + k] : 0.0f;
            sW[k][r] = (n0 + r < N && k0 + k < K) ? W[(size_t)(n0 + r) * ldw + k0 + k] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; w[i] = sW[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) C[(size_t)m * ldc + n] = acc[i][j];
        }
}

}  // namespace

hipError_t launch_gemm_nt(int dtype, const void* A, int lda, const void* W, int ldw, float* C,
                          int ldc, int M, int N, int K, hipStream_t stream) {
    if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
    if (dtype == DT_BF16) {
        // 16-byte loads: K, lda, ldw multiples of 8 and 16-byte aligned bases (checked by the caller)
        if (M >= 2048) {
            constexpr int BM = 128, BN = 128;
            const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
            gemm_bf16_nt_kernel<BM, BN><<<dim3(tm * tn), dim3(256), 0, stream>>>(
                (const bf16_t*)A, lda, (const bf16_t*)W, ldw, C, ldc, M, N, K, tn);
        } else {
            constexpr int BM = 64, BN = 64;
            const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
            gemm_bf16_nt_kernel<BM, BN><<<dim3(tm * tn), dim3(256), 0, stream>>>(
                (const bf16_t*)A, lda, (const bf16_t*)W, ldw, C, ldc, M, N, K, tn);
        }
    } else {
        const int tm = (M + 63) / 64, tn = (N + 63) / 64;
        gemm_f32_nt_kernel<<<dim3(tm * tn), dim3(256), 0, stream>>>(
            (const float*)A, lda, (const float*)W, ldw, C, ldc, M, N, K, tn);
    }
    return hipGetLastError();
}

}  // namespace rnn
