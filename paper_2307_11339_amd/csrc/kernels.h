// Launchers of the gfx950 kernels (internal to the library; the public boundary is include/rnn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rnn {

// ---- input projection (gemm.hip) -----------------------------------------------------------
// C[m, n] = sum_k A[m, k] * W[n, k];  A is [M, K] with row stride lda, W is [N, K] with row
// stride ldw (both in `dtype`), C is fp32 with row stride ldc.  bf16 needs K, lda, ldw multiples
// of 8 and 16-byte aligned base pointers.
hipError_t launch_gemm_nt(int dtype, const void* A, int lda, const void* W, int ldw, float* C,
                          int ldc, int M, int N, int K, hipStream_t stream);

// ---- state set-up / tear-down and the cellwise plan (cellwise.hip) -------------------------
// h_f32, c_f32: [n] fp32 working state; h_st: [n] storage-type copy of h (operand of the next
// recurrent product).  h0 / c0 may be NULL (zeros).
hipError_t launch_state_init(int dtype, const float* h0, const float* c0, float* h_f32,
                             float* c_f32, void* h_st, size_t n, hipStream_t stream);
hipError_t launch_state_export(const float* h_f32, const float* c_f32, float* hT, float* cT,
                               size_t n, hipStream_t stream);

struct CellStepArgs {
    int cell, dtype;
    int B, H, D, d, t;
    const float* gx;      // [T*B, D, H, 4] projection of this layer (no bias)
    const float* gh;      // [B, H, 4] recurrent product of this step and direction
    const float* gh_rh;   // NULL, or (GRU with the reset gate applied before the product) [B, H, 4]
                          // product of W_hh with r * h_{t-1}: its slot n_h replaces gh's, unscaled
    void* rh_st;          // launch_gru_reset only: [B, H] storage type, receives r * h_{t-1}
    const float* bias;    // [H, 4]
    float* h_f32;         // [B, H] in/out
    float* c_f32;         // [B, H] in/out
    void* h_st;           // [B, H] storage type, out
    void* out;            // [T, B, D*H] storage type; this step writes row t, columns d*H..
    const int32_t* lengths;  // [B] or NULL
    int T;
    const float* peep;    // NULL, or (LSTM) [3, H] peephole weights p_i, p_f, p_o of this layer and direction
    float clip;           // clipping threshold of the gate arguments, 0 = none
};
hipError_t launch_cell_step(const CellStepArgs& a, hipStream_t stream);
// GRU variant that applies the reset gate before the candidate's recurrent product: from gx, gh and
// the bias compute r and write r * h_{t-1} (all sequences, storage type) to a.rh_st.
hipError_t launch_gru_reset(const CellStepArgs& a, hipStream_t stream);

// Zero `bytes` bytes (a multiple of 4) at the 4-byte aligned p with a kernel (a fill that may be
// recorded into a stream capture, where memset nodes are avoided).
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);

// `rows` rows of row_bytes bytes (a multiple of 2) from src (rows src_pitch bytes apart) to dst (dst_pitch):
// a block of sequences out of, or back into, a [.., B, ..] tensor.
hipError_t launch_copy_2d(const void* src, size_t src_pitch, void* dst, size_t dst_pitch, int rows, size_t row_bytes,
                          hipStream_t stream);

// dst[j][i][:] = src[i][j][:] for i < n0, j < n1, rows of row_bytes bytes (a multiple of 2): the
// batch-first <-> time-major change of layout of x and y.
hipError_t launch_swap_outer(const void* src, void* dst, int n0, int n1, size_t row_bytes, hipStream_t stream);

// ---- persistent wavefront kernel (wavefront.hip) -------------------------------------------
constexpr int WF_MAX_LAYERS = 16;  // layers that may run concurrently in one launch

struct WavefrontArgs {
    int cell, dtype;
    int T, B, H, D;
    int Bp;                      // B rounded up to a multiple of 4: row count of the blocked state
                                 // sequences, so that no cache line of one holds sequences of two chains
    int L_total;                 // layers of the model (for the hT / cT row index)
    int l0, LP;                  // this launch runs layers [l0, l0 + LP)
    int RT, CT;                  // 16-row tiles per workgroup, 16-column tiles per chain
    int NCH;                     // chains (independent column blocks) per workgroup, 1 or 2
    int nrb, ncb;                // row blocks and chains (column blocks) per (layer, direction)
    const void* whh[WF_MAX_LAYERS * 2];   // packed W_hh per (local layer, direction): [4H, H]
    const void* wih[WF_MAX_LAYERS * 2];   // packed W_ih (layers l0+1.. only, D = 1): [4H, H]
    const float* bias[WF_MAX_LAYERS * 2]; // [H, 4]
    const float* peep[WF_MAX_LAYERS * 2]; // NULL, or (LSTM) [3, H] peephole weights p_i, p_f, p_o per (local layer, direction)
    float clip;                           // clipping threshold of the gate arguments, 0 = none
    int ext;                              // 1 when clip > 0 or a peep[] entry is set: the launch runs the kernel
                                          // variants whose gate phase carries those terms
    const float* gx;             // projection of layer l0: [T*B, D, H, 4] (unused when xin is given)
    const void* xin;             // NULL, or the finished input of layer l0, which then multiplies it
                                 // with its resident W_ih inside the kernel instead of reading gx.
                                 // wavefront_x.hip: D = 1, width H, in the layout of a state sequence
                                 // [T][H/16][Bp][16]; wavefront_ll.hip: plain [T, B, xin_width2 * H / 2]
    int xin_width2;              // wavefront_ll.hip: twice the width of xin over H: 2 (as wide as the
                                 // layer), 1 (half as wide), 4 (a bidirectional layer above
                                 // the first, LP = 1)
    void* out[WF_MAX_LAYERS];    // output of each local layer: [T, B, D*H] storage type (the kernel of
                                 // wavefront_x.hip accepts NULL: output not wanted)
    void* hseq;                  // [LP*D, T+1, B, H] storage type: slot 0 = h0, slot s+1 = state
                                 // after step s; every address is written once per launch
    const float* h0;             // [L*D, B, H] or NULL
    const float* c0;
    float* hT;                   // [L*D, B, H] or NULL
    float* cT;
    const int32_t* lengths;      // [B] or NULL
    uint64_t* flagv;             // [LP*D, T, ncb, nrb] flag words {epoch, step}, never cleared
    unsigned* status;            // [1]: set to 1 if a workgroup gave up waiting
    unsigned long long* ticks;   // NULL, or [LP*D, T] device clock when a step was published
    unsigned spin_limit;         // polls before a wait is abandoned
    uint64_t* lseq;              // tag-in-data kernel only: [LP*D, T+1, B, row_words] tagged words
    uint32_t epoch;              // tag value of this launch (never 0), both kernels
};
// Returns hipErrorInvalidValue when no kernel variant exists for (dtype, RT, CT, NCH, H).
hipError_t launch_wavefront(const WavefrontArgs& a, hipStream_t stream);
// True when launch_wavefront has a variant for this combination.
bool wavefront_variant_exists(int dtype, int RT, int CT, int NCH, int H, bool fused);
// Workgroups per CU the variants with this CT are compiled for (1 or 2).
int wavefront_variant_occupancy(int CT);
// Write slot 0 of the state sequence (the state "before step 0") from h0.
hipError_t launch_wavefront_init(int dtype, const float* h0, int l0, int LP, int D, int T, int B, int Bp,
                                 int H, void* hseq, hipStream_t stream);

// ---- persistent kernel with the input product inside, one layer per launch (wavefront_x.hip) --
// Needs a.D == 1 and a.xin (the finished input sequence of layer l0, width H); a.gx is not read.  With
// a.LP > 1 the layers run side by side and a layer above the first reads the state sequence below it.
hipError_t launch_wavefront_x(const WavefrontArgs& a, hipStream_t stream);
// True when a variant exists for this combination and its LDS footprint fits the current device.
bool wavefront_x_variant_exists(int dtype, int RT, int CT, int NCH, int H, size_t lds_limit,
                                bool several_layers = false);  // host only
// src [T, B, H] -> dst [T][H/16][Bp][16] (the layout of a state sequence, Bp >= B rows per block); H % 16 == 0, T <= 65535,
// one row of 16 sequences must fit 64 KiB of LDS.
hipError_t launch_to_blocked(int dtype, const void* src, void* dst, int T, int B, int Bp, int H, hipStream_t stream);

// ---- persistent wavefront kernel, tag-in-data variant for CT == 1 (wavefront_ll.hip) --------
hipError_t launch_wavefront_ll(const WavefrontArgs& a, hipStream_t stream);
bool wavefront_ll_variant_exists(int dtype, int RT, int H);
// Write slot 0 of the tagged state sequences (h0, tagged with `epoch`).
hipError_t launch_wavefront_ll_init(int dtype, const float* h0, int l0, int LP, int D, int T, int B,
                                    int H, uint64_t* lseq, uint32_t epoch, hipStream_t stream);
// 8-byte words needed for `groups` (layer, direction) state sequences.
size_t wavefront_ll_words(int dtype, int groups, int T, int B, int H);

}  // namespace rnn
