/*
 * CPU oracle for the forward pass of a stacked LSTM / GRU.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the GPU library is checked against.  It is used by the tests,
 * by the smoke check and by the benchmark's CPU-baseline leg, and by nothing else; it shares
 * no code with the GPU path.
 *
 * What it computes.  The paper unrolls a recurrent network over layers and time steps into a
 * grid of cell operators A_t^l in which cell (l, t) depends on cell (l, t-1) and on cell
 * (l-1, t) (Section 1; Section 2.2, the figure of the folded and unfolded RNN).  The paper
 * names the cell ("LSTM", Section 1 and Section 6.2) but prints no cell equations, so the
 * cell below is the standard one:
 *
 *   LSTM (row blocks of W and b ordered i, f, g, o):
 *       a = W_ih x_t + b_ih + W_hh h_{t-1} + b_hh
 *       i = sigma(a_i)  f = sigma(a_f)  g = tanh(a_g)  o = sigma(a_o)
 *       c_t = f * c_{t-1} + i * g          h_t = o * tanh(c_t)
 *     optional peephole weights p_i, p_f, p_o (one value per hidden unit, the form of the ONNX LSTM
 *     operator, which is the model format the paper's system ingests, Section 1 and Section 4.1):
 *       i = sigma(a_i + p_i * c_{t-1})   f = sigma(a_f + p_f * c_{t-1})   o = sigma(a_o + p_o * c_t)
 *   GRU (row blocks ordered r, z, n):
 *       r = sigma(W_ir x + b_ir + W_hr h + b_hr)     z = sigma(W_iz x + b_iz + W_hz h + b_hz)
 *       variant 0 (reset applied after the product):  n = tanh(W_in x + b_in + r * (W_hn h + b_hn))
 *       variant 1 (reset applied before the product): n = tanh(W_in x + b_in + W_hn (r * h) + b_hn)
 *       h_t = (1 - z) * n + z * h_{t-1}
 *   optional clipping threshold clip > 0 (same operator): the argument of every gate activation
 *   (i, f, g, o with their peephole terms; r, z and the whole argument of n) is limited to
 *   [-clip, +clip] before sigma / tanh is applied; the cell state inside h_t = o * tanh(c_t) is not.
 *
 * Everything is evaluated in the plainest order: for each layer, each direction, each
 * sequence, each visited time step, each gate row, one dot product.  Arithmetic is double
 * precision throughout with libm exp() and tanh(); nothing is blocked, fused or reordered.
 * With nthreads > 1 the loop over hidden units of one cell is split among OpenMP threads;
 * every unit is still computed by exactly the same scalar code.
 *
 * Layout (all row-major, time-major):
 *   x  [T, B, I]            lengths [B] (NULL = all T), 1 <= lengths[b] <= T
 *   h0, c0 [L*D, B, H]      (NULL = zeros), row index l*D + d
 *   weights: L*D*4 pointers in order (l, d, {W_ih [G*H, I_l], W_hh [G*H, H], b_ih [G*H], b_hh [G*H]}),
 *            a NULL bias pointer means zeros; I_0 = I, I_l = D*H for l >= 1
 *   y  [T, B, D*H]          output of the last layer, +0.0 at padded positions (t >= lengths[b])
 *   hT, cT [L*D, B, H]      state after the last visited step of each sequence and direction
 *                           (cT is left untouched for a GRU, which has no cell state)
 *   layer_out (optional)    [L, T, B, D*H] outputs of every layer (NULL to skip)
 * Direction 0 visits t = 0 .. len-1; direction 1 visits t = len-1 .. 0, starting from the
 * initial state at each sequence's own last valid step.  Layer l >= 1 reads the concatenation
 * [forward half, backward half] of layer l-1.
 *
 * Parity pins (tests/test_oracle_pins.py): zero-weight closed forms, hidden-size-1 scalar
 * recursions, saturated-gate identities, split-sequence / layer / direction / batch
 * invariants, bounds, a term-by-term brute force, and an fp64 library LSTM/GRU cross-check; for
 * the peephole and clipping terms scalar recursions written out separately, closed forms (clip
 * so small that every gate sits at its clipped value) and the identities "zero peepholes" and
 * "threshold beyond every argument" = the plain cell.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_LSTM = 0, ORACLE_GRU = 1 };

static double sigmoid(double a) { return 1.0 / (1.0 + exp(-a)); }

/* clip <= 0 means no clipping */
static double limit(double a, double clip) {
    if (clip > 0.0) {
        if (a > clip) return clip;
        if (a < -clip) return -clip;
    }
    return a;
}

static double dot(const double *w, const double *v, int n) {
    double s = 0.0;
    for (int k = 0; k < n; ++k) s += w[k] * v[k];
    return s;
}

/* One LSTM cell for one sequence: reads x[In], h_prev[H], c_prev[H]; writes h_new[H], c_new[H].
 * peep: NULL or [3*H] peephole weights (p_i, p_f, p_o). */
static void lstm_cell(int In, int H, const double *W_ih, const double *W_hh, const double *b_ih,
                      const double *b_hh, const double *peep, double clip, const double *x,
                      const double *h_prev, const double *c_prev, double *h_new, double *c_new) {
#pragma omp parallel for schedule(static)
    for (int j = 0; j < H; ++j) {
        double a[4];
        for (int g = 0; g < 4; ++g) {
            const int row = g * H + j;
            a[g] = dot(W_ih + (size_t)row * In, x, In) + (b_ih ? b_ih[row] : 0.0) +
                   dot(W_hh + (size_t)row * H, h_prev, H) + (b_hh ? b_hh[row] : 0.0);
        }
        const double p_i = peep ? peep[j] : 0.0, p_f = peep ? peep[H + j] : 0.0, p_o = peep ? peep[2 * H + j] : 0.0;
        const double ig = sigmoid(limit(a[0] + p_i * c_prev[j], clip));
        const double fg = sigmoid(limit(a[1] + p_f * c_prev[j], clip));
        const double gg = tanh(limit(a[2], clip));
        const double c = fg * c_prev[j] + ig * gg;
        const double og = sigmoid(limit(a[3] + p_o * c, clip));
        c_new[j] = c;
        h_new[j] = og * tanh(c);
    }
}

/* One GRU cell for one sequence.  rh is scratch of H doubles (variant 1 only). */
static void gru_cell(int variant, int In, int H, const double *W_ih, const double *W_hh,
                     const double *b_ih, const double *b_hh, double clip, const double *x,
                     const double *h_prev, double *h_new, double *rgate, double *rh) {
    /* reset gate first: variant 1 needs r for every unit before the candidate's product */
#pragma omp parallel for schedule(static)
    for (int j = 0; j < H; ++j) {
        const int row = j; /* block r */
        const double a = dot(W_ih + (size_t)row * In, x, In) + (b_ih ? b_ih[row] : 0.0) +
                         dot(W_hh + (size_t)row * H, h_prev, H) + (b_hh ? b_hh[row] : 0.0);
        rgate[j] = sigmoid(limit(a, clip));
        rh[j] = rgate[j] * h_prev[j];
    }
#pragma omp parallel for schedule(static)
    for (int j = 0; j < H; ++j) {
        const int rz = H + j, rn = 2 * H + j;
        const double az = dot(W_ih + (size_t)rz * In, x, In) + (b_ih ? b_ih[rz] : 0.0) +
                          dot(W_hh + (size_t)rz * H, h_prev, H) + (b_hh ? b_hh[rz] : 0.0);
        const double z = sigmoid(limit(az, clip));
        const double nx = dot(W_ih + (size_t)rn * In, x, In) + (b_ih ? b_ih[rn] : 0.0);
        double nh;
        if (variant == 0)
            nh = rgate[j] * (dot(W_hh + (size_t)rn * H, h_prev, H) + (b_hh ? b_hh[rn] : 0.0));
        else
            nh = dot(W_hh + (size_t)rn * H, rh, H) + (b_hh ? b_hh[rn] : 0.0);
        const double n = tanh(limit(nx + nh, clip));
        h_new[j] = (1.0 - z) * n + z * h_prev[j];
    }
}

/* The input projection on its own: P[r, j] = sum_k in[r, k] * W[j, k] for r < rows, j < n_out.
 * This is the part of a cell that depends only on x_t (Section 2.2: every cell consumes its
 * own x_t), written as one dot product per output element. */
int rnn_oracle_projection(int rows, int n_out, int K, const double *in, const double *W, double *P) {
    if (!in || !W || !P || rows < 1 || n_out < 1 || K < 1) return 1;
    for (int r = 0; r < rows; ++r)
        for (int j = 0; j < n_out; ++j) P[(size_t)r * n_out + j] = dot(W + (size_t)j * K, in + (size_t)r * K, K);
    return 0;
}

/* peepholes: NULL, or L*D pointers (row l*D + d), each NULL or [3*H] (p_i, p_f, p_o), LSTM only;
 * clip: clipping threshold, <= 0 for none. */
int rnn_oracle_forward_ext(int cell, int gru_variant, int L, int D, int I, int H, int T, int B,
                           const double *const *weights, const double *const *peepholes, double clip,
                           const double *x, const int *lengths, const double *h0, const double *c0,
                           double *y, double *hT, double *cT, double *layer_out, int nthreads) {
    if (!weights || !x || !y) return 1;
    if (peepholes && cell != ORACLE_LSTM) return 1;
    if (cell != ORACLE_LSTM && cell != ORACLE_GRU) return 1;
    if (L < 1 || (D != 1 && D != 2) || I < 1 || H < 1 || T < 1 || B < 1) return 1;
    if (lengths)
        for (int b = 0; b < B; ++b)
            if (lengths[b] < 1 || lengths[b] > T) return 1;
#ifdef _OPENMP
    omp_set_num_threads(nthreads > 0 ? nthreads : 1);
#else
    (void)nthreads;
#endif
    const size_t out_sz = (size_t)T * B * D * H;
    double *in_buf = NULL;                 /* output of the previous layer */
    double *out_buf = (double *)malloc(out_sz * sizeof(double));
    double *h = (double *)malloc(sizeof(double) * H * 6);
    if (!out_buf || !h) { free(out_buf); free(h); return 3; }
    double *c = h + H, *h2 = h + 2 * H, *c2 = h + 3 * H, *rg = h + 4 * H, *rh = h + 5 * H;

    for (int l = 0; l < L; ++l) {
        const int In = (l == 0) ? I : D * H;
        const double *in = (l == 0) ? x : in_buf;
        for (size_t i = 0; i < out_sz; ++i) out_buf[i] = 0.0; /* padded positions stay +0.0 */
        for (int d = 0; d < D; ++d) {
            const double *const *w = weights + (size_t)(l * D + d) * 4;
            const double *W_ih = w[0], *W_hh = w[1], *b_ih = w[2], *b_hh = w[3];
            const double *peep = peepholes ? peepholes[l * D + d] : NULL;
            for (int b = 0; b < B; ++b) {
                const int len = lengths ? lengths[b] : T;
                const size_t st = ((size_t)(l * D + d) * B + b) * H;
                for (int j = 0; j < H; ++j) {
                    h[j] = h0 ? h0[st + j] : 0.0;
                    c[j] = c0 ? c0[st + j] : 0.0;
                }
                for (int s = 0; s < len; ++s) {
                    const int t = (d == 0) ? s : len - 1 - s;
                    const double *xt = in + ((size_t)t * B + b) * In;
                    if (cell == ORACLE_LSTM) {
                        lstm_cell(In, H, W_ih, W_hh, b_ih, b_hh, peep, clip, xt, h, c, h2, c2);
                        memcpy(c, c2, sizeof(double) * H);
                    } else {
                        gru_cell(gru_variant, In, H, W_ih, W_hh, b_ih, b_hh, clip, xt, h, h2, rg, rh);
                    }
                    memcpy(h, h2, sizeof(double) * H);
                    memcpy(out_buf + ((size_t)t * B + b) * D * H + (size_t)d * H, h,
                           sizeof(double) * H);
                }
                if (hT) memcpy(hT + st, h, sizeof(double) * H);
                if (cT && cell == ORACLE_LSTM) memcpy(cT + st, c, sizeof(double) * H);
            }
        }
        if (layer_out) memcpy(layer_out + (size_t)l * out_sz, out_buf, out_sz * sizeof(double));
        /* this layer's output becomes the next layer's input */
        if (!in_buf) {
            in_buf = (double *)malloc(out_sz * sizeof(double));
            if (!in_buf) { free(out_buf); free(h); return 3; }
        }
        double *tmp = in_buf; in_buf = out_buf; out_buf = tmp;
    }
    memcpy(y, in_buf, out_sz * sizeof(double));
    free(in_buf);
    free(out_buf);
    free(h);
    return 0;
}

/* The plain cells: no peepholes, no clipping. */
int rnn_oracle_forward(int cell, int gru_variant, int L, int D, int I, int H, int T, int B,
                       const double *const *weights, const double *x, const int *lengths,
                       const double *h0, const double *c0, double *y, double *hT, double *cT,
                       double *layer_out, int nthreads) {
    return rnn_oracle_forward_ext(cell, gru_variant, L, D, I, H, T, B, weights, NULL, 0.0, x, lengths,
                                  h0, c0, y, hT, cT, layer_out, nthreads);
}
