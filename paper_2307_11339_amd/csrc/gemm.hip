// Input-projection GEMM for gfx950:  C[m, n] = sum_k A[m, k] * W[n, k]   (both operands K-contiguous).
//
// In the unrolled cell grid every cell (l, t) consumes x_t (paper, Section 2.2); that part of
// the cell has no recurrent dependency, so it is computed for all time steps at once as one
// dense contraction: rows m = (t, b) pairs, columns n = packed gate rows of W_ih.
//
// bf16 path: 32x32x16 bf16 MFMA, fp32 accumulate.  A workgroup of 256 threads (4 waves, 2x2)
// owns a BM x BN tile of C; the K loop moves BK-wide slabs of A and W through LDS.
// fp32 path: plain FMA tiles (only the small fp32 workloads use it).
#include <type_traits>
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

// Large aligned shapes (the projection of a whole layer over all time steps): a 256 x 256 tile per workgroup, one
// workgroup per compute unit.  Each of the 4 waves owns 128 x 128 of it: 16 accumulator tiles of 32 x 32, which
// fill the 256 accumulation registers, so that one K step of 16 costs 8 fragment reads from LDS for 16 matrix
// instructions (the smaller tiles above read 6 for 8 and write every slab for half as many products).  With one
// wave per SIMD nothing else hides latency, so the loop is pipelined by hand and the instruction order is pinned
// with scheduling groups (one LDS read, or two LDS writes or global loads, per two matrix instructions):
//   quarter 0..2 of slab k   multiply the fragments read a quarter earlier, read the next quarter's;
//   quarter 2                the register set (slab k + 1, requested during slab k - 1) goes into the other stage;
//   barrier                  orders those writes before the reads below and the last reads of stage k % 2 (quarter 2)
//                            before the writes of slab k + 1's third quarter;
//   quarter 3                multiply, read quarter 0 of slab k + 1 from the other stage, request slab k + 2.
// K slabs of 64 in two LDS stages of 512 rows x 144 bytes (rows padded by 16 bytes: 16-byte reads and writes
// without bank conflicts, measured), 144 KiB.  Tile order follows the hardware: workgroup b runs on XCD b % 8, every
// XCD owns a band of M tiles and walks it in blocks of (up to) 8 x 4 tiles, one block per pass of its 32 compute
// units, whose A and W rows stay in its L2.  C leaves with non-temporal stores: it is 8 times the inputs and would
// only push them out of the L2.
// Needs M % 256 == 0, N % 256 == 0, K % 64 == 0, K >= 128, (M / 256) % 8 == 0, (N / 256) % 4 == 0 (the launcher checks).
__global__ __launch_bounds__(256, 1) void gemm_bf16_nt_wide_kernel(const bf16_t* __restrict__ A, int lda,
                                                                   const bf16_t* __restrict__ W, int ldw,
                                                                   float* __restrict__ C, int ldc, int K, int tiles_m,
                                                                   int tiles_n) {
    constexpr int BM = 256, BN = 256, BKW = 64;
    constexpr int WM = 128, WN = 128, TM = 4, TN = 4;
    constexpr int ROW = BKW + 8;                              // padded LDS row (elements)
    constexpr int CPR = BKW / 8;                              // 16-byte chunks per row
    constexpr int A_CH = BM * CPR / 256, W_CH = BN * CPR / 256;
    constexpr int STAGE = (BM + BN) * ROW;                    // elements per stage
    constexpr int BW = 4;                                     // N tiles per block of the tile order
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    int tile_m, tile_n;
    {
        const int b = blockIdx.x, x = b & 7, q = b >> 3;
        const int band = tiles_m / 8;                         // M tiles per XCD
        const int nb = tiles_n / BW;
        const int bh = band % 8 == 0 ? 8 : band % 4 == 0 ? 4 : band % 2 == 0 ? 2 : 1;   // block height divides the band
        const int per = bh * BW;
        const int g = q / per, r = q % per;
        const int gm = g / nb, gn = g % nb;
        tile_m = x * band + gm * bh + r % bh;
        tile_n = gn * BW + r / bh;
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    u32x4 ra[A_CH], rw[W_CH];
    const bf16_t* Ab = A + (size_t)(m0 + tid / CPR) * lda + (tid % CPR) * 8;
    const bf16_t* Wb = W + (size_t)(n0 + tid / CPR) * ldw + (tid % CPR) * 8;
    auto load_global = [&](int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) ra[i] = *reinterpret_cast<const u32x4*>(Ab + (size_t)(i * 32) * lda + k0);
#pragma unroll
        for (int i = 0; i < W_CH; ++i) rw[i] = *reinterpret_cast<const u32x4*>(Wb + (size_t)(i * 32) * ldw + k0);
    };
    const int st_off = (tid / CPR) * ROW + (tid % CPR) * 8;
    auto store_lds = [&](int stage) __attribute__((always_inline)) {
        bf16_t* sA = smem + stage * STAGE + st_off;
        bf16_t* sW = sA + BM * ROW;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *reinterpret_cast<u32x4*>(&sA[i * 32 * ROW]) = ra[i];
#pragma unroll
        for (int i = 0; i < W_CH; ++i) *reinterpret_cast<u32x4*>(&sW[i * 32 * ROW]) = rw[i];
    };
    // fragment of a 32 x 32 x 16 product: lane holds row lane % 32, K elements 8 * (lane / 32) .. + 7
    const int fa_off = (wm * WM + (lane & 31)) * ROW + 8 * (lane >> 5);
    const int fw_off = BM * ROW + (wn * WN + (lane & 31)) * ROW + 8 * (lane >> 5);
    bf16x8 fa[2][TM], fw[2][TN];
    auto read_frags = [&](int buf, int stage, int ks) __attribute__((always_inline)) {
        const bf16_t* sb = smem + stage * STAGE + ks * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(&sb[fa_off + i * 32 * ROW]);
#pragma unroll
        for (int j = 0; j < TN; ++j) fw[buf][j] = *reinterpret_cast<const bf16x8*>(&sb[fw_off + j * 32 * ROW]);
    };
    auto products = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fw[buf][j], acc[i][j], 0, 0, 0);
    };
    // scheduling group masks: 0x8 matrix instruction, 0x20 global load, 0x100 LDS read, 0x200 LDS write
    auto slab = [&](int k, auto write_next, auto load_next) __attribute__((always_inline)) {
        constexpr bool WRITE = decltype(write_next)::value, LOAD = decltype(load_next)::value;
        const int stage = k & 1;
        read_frags(1, stage, 1);
        products(0);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x8, 2, 0);
        }
        read_frags(0, stage, 2);
        products(1);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x8, 2, 0);
        }
        read_frags(1, stage, 3);
        if (WRITE) store_lds(stage ^ 1);
        products(0);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (WRITE) __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x8, 2, 0);
        }
        __syncthreads();
        if (WRITE) read_frags(0, stage ^ 1, 0);
        if (LOAD) load_global((k + 2) * BKW);
        products(1);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            if (WRITE) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (LOAD) __builtin_amdgcn_sched_group_barrier(0x20, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x8, 2, 0);
        }
    };
    const int nslab = K / BKW;                                // >= 2
    load_global(0);
    store_lds(0);
    load_global(BKW);
    __syncthreads();
    read_frags(0, 0, 0);
    int k = 0;
    for (; k + 2 < nslab; ++k) slab(k, std::true_type{}, std::true_type{});
    slab(k, std::true_type{}, std::false_type{});
    slab(k + 1, std::false_type{}, std::false_type{});
    // acc[i][j][e]: row = 8*(e/4) + 4*(lane/32) + e%4, column = lane%32 of the 32x32 tile
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * WM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                __builtin_nontemporal_store(acc[i][j][e], &C[(size_t)m * ldc + n]);
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
        constexpr int GM = 256, GN = 256;
        if (M % GM == 0 && N % GN == 0 && K % 64 == 0 && K >= 128 && (M / GM) % 8 == 0 && (N / GN) % 4 == 0 &&
            (size_t)(M / GM) * (N / GN) <= 0x7FFFFFFFu) {
            constexpr int smem = 2 * (GM + GN) * (64 + 8) * (int)sizeof(bf16_t);   // 144 KiB of the 160 KiB
            int dev = 0;
            hipError_t e = hipGetDevice(&dev);
            if (e != hipSuccess) return e;
            static bool configured[64] = {};
            if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
            if (!configured[dev]) {
                e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_nt_wide_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem);
                if (e != hipSuccess) return e;
                configured[dev] = true;
            }
            gemm_bf16_nt_wide_kernel<<<dim3((M / GM) * (N / GN)), dim3(256), smem, stream>>>(
                (const bf16_t*)A, lda, (const bf16_t*)W, ldw, C, ldc, K, M / GM, N / GN);
        } else if (M >= 2048) {
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
