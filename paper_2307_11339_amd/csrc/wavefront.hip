// Persistent wavefront kernel: the whole layer x time grid of cells in one launch.
//
// The paper's observation (Section 1; Section 2.2, figure of the unfolded RNN): after unrolling,
// cell (l, t) depends only on cells (l, t-1) and (l-1, t), so the cells of one anti-diagonal
// can run side by side; a GPU that is handed the cells one at a time cannot use this.  Here
// the workgroups of one launch are divided into one group per (layer, direction).  A group
// walks along time; it starts step t as soon as its own step t-1 and the step t of the layer
// below have been published, so the groups settle on successive anti-diagonals of the grid.
//
// Inside a group, a workgroup owns RT*4 hidden units (RT tiles of 16 gate rows, the four
// pre-activation slots of a unit being adjacent rows) for CT*16 sequences.  Its slice of W_hh
// (and of W_ih for layers whose projection is fused) stays in registers for the whole launch as
// the A operand of 16-row MFMA tiles; the activations h_{t-1} (and x_t) are the B operand.  The
// four waves of a workgroup split K, so each wave reads a disjoint quarter of the activation
// vector straight from global memory; partial sums meet in LDS, then every (unit, sequence)
// pair is finished by one fixed lane that keeps c and h of that pair in registers.
//
// Steps are published through a vector of flag words per (layer, direction, column block, step),
// one 8-byte word per row block: a workgroup that has written its part of h_t stores
// {launch epoch, step} into its own word; a reader loads the whole vector with one instruction
// (one lane per row block) and polls until every word carries this launch's epoch.  (A shared
// counter bumped with atomic adds serialises the row blocks on one address and was measured at
// more than twice the cost.)  The epoch changes with every launch, so flags are never cleared.
// No bulk cache write-back or invalidate is used (every wave issuing one per step costs tens of
// microseconds).  Instead:
//   - everything a workgroup writes for others (h_t, layer outputs) goes out with device-scope
//     write-through stores, and the writer waits for their acknowledgement before its flag word
//     is stored;
//   - every exchanged address is written exactly once per launch (the state of step s has its
//     own slot, layer outputs are indexed by t) and is read only after its flag vector is
//     complete, and a cache line never holds data of two writers that finish at different times.
//     A reader's caches therefore cannot hold a stale copy, so activations are read with ordinary
//     cached loads and the workgroups of one XCD share them through that XCD's L2.
// The state sequence is stored in blocks of 16 hidden units: slot[unit / 16][row][unit % 16] with
// Bp = B rounded up to a multiple of 4 rows per block (rows >= B are padding nobody writes), so
// that a block is a whole number of 128-byte lines: without the padding a line at the end of one
// block would continue in the next block, whose first sequences belong to another chain, and a
// reader could cache that line before the other chain has written its part.
// A workgroup that owns 16 units then writes whole cache lines (32 bytes per sequence,
// sequences adjacent), and a fragment load of a wave covers 16 sequences x 32 contiguous bytes
// per unit block instead of 16 half lines 2 KiB apart.
// Every wait is bounded: a wave that exhausts its poll budget raises the status word and stops
// waiting, so the grid always drains.
#include "wf_traits.h"

// Every variant exists twice: with the plain cell, and (RNN_CELL_EXT = 1, the translation unit
// wavefront_b.hip) with the optional peephole and clipping terms in the gate phase, so that a model
// without those terms runs exactly the plain cell's instructions.
#ifndef RNN_CELL_EXT
#define RNN_CELL_EXT 0
#endif


namespace rnn {

namespace {

// Workgroups per CU a variant is compiled for.  (Two workgroups per CU with tiles of 32
// sequences were measured slower than one with 64: the step is bound by synchronisation and by
// L2 traffic, and doubling the number of workgroups raises both.)
constexpr int variant_occupancy(int /*CT*/) { return 1; }

// A workgroup owns RT*4 hidden units for NCH chains of CT*16 sequences each.  Chains are
// independent recurrences, so with NCH = 2 the workgroup alternates between them: once the
// matrix work of chain c has consumed the activation registers, the flags of the other chain
// (published half an iteration ago) are checked and its activations are requested; they travel
// while chain c runs its reduction, gates and publication.  Part of the flag wait and of the
// L2 round trip of the activations leaves the critical path this way.  (Requesting even
// earlier, before the matrix work, was measured slower: the flags are then only just being
// written and the wait is paid in full.  The store acknowledgement wait at the end of chain c
// also covers the loads in flight, which bounds what can be hidden.  Four chains of 16
// sequences were measured slower than two of 32: the fixed cost of a chain step, two barriers,
// a store acknowledgement and a flag poll, is paid twice as often.)
template <class TR, int CELL, int RT, int CT, int KB, bool FUSED, int NCH, bool EXT>
__global__ __launch_bounds__(256, variant_occupancy(CT)) void wavefront_kernel(WavefrontArgs p) {
    typedef typename TR::elem elem;
    typedef typename TR::frag frag;
    constexpr int KW = TR::KW;
    constexpr int NTILE = RT * CT;                 // 16x16 output tiles per chain
    constexpr int NOWN = (NTILE + 3) / 4;          // tiles of a chain finished by one wave
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    f32x4* red = reinterpret_cast<f32x4*>(smem_raw);  // [4 waves][NTILE][64 lanes]

    // every step of this kernel is on a dependency chain: when a projection kernel shares the CU,
    // these waves go first
    __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;

    const int v = xcd_contiguous_id();
    const int ngrp = p.ncb / NCH;                   // column block groups (ncb counts chains)
    const int wpg = p.nrb * ngrp;
    const int g = v / wpg;                          // local (layer, direction) index
    if (g >= p.LP * p.D) return;
    const int r = v - g * wpg;
    const int cbg = r / p.nrb, rb = r - cbg * p.nrb;
    const int ll = g / p.D, d = g - ll * p.D;
    const int l = p.l0 + ll;
    const bool fused = FUSED && ll > 0;
    const bool out_shared = FUSED && ll + 1 < p.LP;  // a fused layer above reads this layer's output
    const int H = p.H, B = p.B, T = p.T;
    const int Bp = p.Bp;                            // rows per 16-unit block of a state sequence
    const int kq = H / 4;                           // K range of one wave inside each part

    // per-workgroup rotation of the K blocks and of the column tiles (see load_part)
    const int rot_k = rb % KB;
    const int rot_c = (rb / KB) % CT;

    // ---- resident weights: A operand fragments ---------------------------------------------
    frag wh[RT][KB];
    frag wx[RT][KB];  // only live when FUSED
    {
        const elem* whh = static_cast<const elem*>(p.whh[g]);
        // a layer without a fused projection never uses wx; it loads W_hh again to stay branch-free
        const elem* wih = fused ? static_cast<const elem*>(p.wih[g]) : whh;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const size_t row = (size_t)(rb * RT + rt) * 16 + (lane & 15);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const int k = w * kq + wrap_kb<KB>(kb + rot_k) * KW + TR::koff(lane);
                wh[rt][kb] = TR::load(whh + row * H + k);
                if (FUSED) wx[rt][kb] = TR::load(wih + row * H + k);
            }
        }
    }

    // ---- per-lane state of the (unit, sequence) pairs this lane finishes ---------------------
    float c_reg[NCH][NOWN], h_reg[NCH][NOWN];
    int len_reg[NCH][NOWN], col_reg[NCH][NOWN];
    f32x4 bias_reg[NOWN];
    CellExt ext_reg[EXT ? NOWN : 1];                // peephole weights and clipping bound of the unit
    int unit_reg[NOWN];
    const size_t state_row = (size_t)(l * p.D + d) * B;
#pragma unroll
    for (int o = 0; o < NOWN; ++o) {
        const int j = w + 4 * o;                    // tile index = rt * CT + ct
        const int rt = j / CT, ct = j - rt * CT;
        const int unit = (rb * RT + rt) * 4 + (lane >> 4);
        unit_reg[o] = unit;
        bias_reg[o] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (j < NTILE) bias_reg[o] = *reinterpret_cast<const f32x4*>(p.bias[g] + (size_t)unit * SLOTS);
        if constexpr (EXT) ext_reg[o] = load_cell_ext(CELL == CELL_LSTM ? p.peep[g] : nullptr, H, min(unit, H - 1), p.clip);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int col = ((cbg * NCH + c) * CT + (ct + rot_c) % CT) * 16 + (lane & 15);
            col_reg[c][o] = col;
            c_reg[c][o] = 0.0f;
            h_reg[c][o] = 0.0f;
            len_reg[c][o] = 0;
            if (j < NTILE && col < B) {
                const size_t si = (state_row + col) * H + unit;
                if (p.h0) h_reg[c][o] = p.h0[si];
                if (p.c0) c_reg[c][o] = p.c0[si];
                len_reg[c][o] = p.lengths ? min(max(p.lengths[col], 0), T) : T;
            }
        }
    }

    // B operand columns of this lane (clamped so that loads stay in bounds; columns >= B are
    // computed from a duplicate of the last sequence and never stored)
    int bcol[NCH][CT];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
            bcol[c][ct] = min(((cbg * NCH + c) * CT + (ct + rot_c) % CT) * 16 + (lane & 15), B - 1);

    elem* hseq = static_cast<elem*>(p.hseq) + (size_t)g * (T + 1) * Bp * H;
    elem* out = static_cast<elem*>(p.out[ll]);
    const elem* below = fused ? static_cast<const elem*>(p.out[ll - 1]) : nullptr;
    const int out_ld = p.D * H;
    // flag word of (group, step, chain column block, row block): ((g*T + s)*ncb + cb)*nrb + rb
    const size_t flag_step = (size_t)p.ncb * p.nrb;
    uint64_t* my_flags = p.flagv + ((size_t)g * T * p.ncb + cbg * NCH) * p.nrb;          // chain 0
    const uint64_t* below_flags =
        fused ? p.flagv + ((size_t)(g - p.D) * T * p.ncb + cbg * NCH) * p.nrb : nullptr;
    const uint32_t epoch = p.epoch;
    bool aborted = false;
    const int kbase = w * kq + TR::koff(lane);
    // A wave reads only its own K quarter of an activation vector, so it waits only for the row
    // blocks that produce the cache lines of that quarter (a quarter of the flag vector, one cache
    // line at most, unless a quarter is narrower than a line).  A line of a state sequence holds 16
    // units, a line of a layer output (row-major) 128 bytes of one sequence.
    int fl0, nfl, xfl0, xnfl;
    flag_span(w * kq, kq, H, 16, RT * 4, fl0, nfl);
    flag_span(w * kq, kq, H, 128 / (int)sizeof(elem), RT * 4, xfl0, xnfl);

    // Addresses of the activation loads = uniform base of the step + uniform offset of the K block
    // + a 32-bit per-lane offset that does not change over the launch (one register per chain and
    // column tile; full per-load pointers do not fit beside two sets of resident weights).  In the
    // blocked layout a K block of KW units lies KW * B elements further when KW is a multiple of
    // 16; otherwise (fp32 fragments of 4 units) the offset is computed per load.
    constexpr bool LINEAR_K = (KW % 16) == 0;
    uint32_t hoff[NCH][CT], xoff[NCH][CT];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            hoff[c][ct] = (uint32_t)(hseq_off(kbase, bcol[c][ct], Bp) * sizeof(elem));
            xoff[c][ct] = (uint32_t)(((size_t)bcol[c][ct] * H + kbase) * sizeof(elem));
        }
    // h_{t-1} fragments of the chain that is processed next
    frag hbuf[KB][CT];
    auto fetch_h = [&](int c, int s) {  // wait for step s-1 of chain c, then request its state
        if (s > 0)
            wait_flags(my_flags + (size_t)(s - 1) * flag_step + (size_t)c * p.nrb + fl0, nfl, lane, epoch,
                       p.status, p.spin_limit, aborted);
        const elem* hprev = hseq + (size_t)s * Bp * H;  // state after step s-1
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int kr = wrap_kb<KB>(kb + rot_k);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                if (LINEAR_K)
                    hbuf[kb][ct] = TR::load(reinterpret_cast<const elem*>(
                        reinterpret_cast<const char*>(hprev) + (size_t)kr * KW * Bp * sizeof(elem) + hoff[c][ct]));
                else
                    hbuf[kb][ct] = TR::load(hprev + hseq_off(kbase + kr * KW, bcol[c][ct], Bp));
            }
        }
    };
    if (NCH > 1) fetch_h(0, 0);

    for (int s = 0; s < T; ++s) {
        const int t = d ? (T - 1 - s) : s;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            // projection of this step for the pairs this lane finishes (not needed until the
            // gates; issued first so that the loads fly during the matrix work)
            f32x4 gx_reg[NOWN];
#pragma unroll
            for (int o = 0; o < NOWN; ++o) {
                gx_reg[o] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (!fused && (w + 4 * o) < NTILE && col_reg[c][o] < B)
                    gx_reg[o] = *reinterpret_cast<const f32x4*>(
                        p.gx + ((((size_t)t * B + col_reg[c][o]) * p.D + d) * H + unit_reg[o]) * SLOTS);
            }

            f32x4 acc[RT][CT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) acc[rt][ct] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

            if (FUSED) {
                if (fused) {  // x_t = h_t of the layer below
                    wait_flags<true>(below_flags + (size_t)s * flag_step + (size_t)c * p.nrb + xfl0, xnfl, lane, epoch,
                                     p.status, p.spin_limit, aborted);
                    const char* xs = reinterpret_cast<const char*>(below + (size_t)t * B * H);
                    frag xbuf[KB][CT];
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                        for (int ct = 0; ct < CT; ++ct)
                            xbuf[kb][ct] = TR::load(reinterpret_cast<const elem*>(
                                xs + (size_t)wrap_kb<KB>(kb + rot_k) * KW * sizeof(elem) + xoff[c][ct]));
                    mma_part<TR, RT, CT, KB>(wx, xbuf, acc);
                }
            }

            if (NCH == 1) fetch_h(0, s);
            mma_part<TR, RT, CT, KB>(wh, hbuf, acc);
            if (NCH > 1) {  // request the state the next chain will need
                if (c + 1 < NCH) fetch_h(c + 1, s);
                else if (s + 1 < T) fetch_h(0, s + 1);
            }

            // partial sums of the four K quarters meet in LDS
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    red[(w * NTILE + rt * CT + ct) * 64 + lane] = acc[rt][ct];
            __syncthreads();

            elem* hcur = hseq + (size_t)(s + 1) * Bp * H;
            // all partial sums of the tiles this wave finishes are read before the first is used
            // (one LDS round trip instead of one per read)
            f32x4 part[NOWN][4];
#pragma unroll
            for (int o = 0; o < NOWN; ++o)
#pragma unroll
                for (int q = 0; q < 4; ++q) part[o][q] = red[(q * NTILE + min(w + 4 * o, NTILE - 1)) * 64 + lane];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int o = 0; o < NOWN; ++o) {
                const int j = w + 4 * o;
                if (j < NTILE) {  // uniform per wave
                    const bool valid = col_reg[c][o] < B;
                    f32x4 a = (part[o][0] + part[o][1]) + (part[o][2] + part[o][3]);
                    a += gx_reg[o];
                    a += bias_reg[o];
                    const bool active = valid && t < len_reg[c][o];
                    float c_new = c_reg[c][o];
                    const float pre[SLOTS] = {a[0], a[1], a[2], a[3]};
                    float hn;
                    if constexpr (EXT) hn = cell_update_ext<CELL>(pre, h_reg[c][o], c_new, ext_reg[o]);
                    else hn = cell_update<CELL>(pre, h_reg[c][o], c_new);
                    float kept = h_reg[c][o];
                    if (active) {
                        c_reg[c][o] = c_new;
                        (void)TR::store_val(hn, kept);
                        h_reg[c][o] = kept;
                    }
                    float unused;
                    const elem state_v = TR::store_val(h_reg[c][o], unused);   // held value when inactive
                    const elem out_v = active ? state_v : TR::zero();
                    // lanes n, n+16, n+32, n+48 hold units unit0 .. unit0+3 of sequence n
                    const int unit0 = unit_reg[o] - (lane >> 4);
                    const int colc = valid ? col_reg[c][o] : 0;
                    TR::publish(state_v, out_v, valid, out_shared, lane, hcur + hseq_off(unit0, colc, Bp),
                                out + ((size_t)t * B + colc) * out_ld + (size_t)d * H + unit0);
                }
            }

            // publish: wait until this wave's stores are acknowledged, meet the other waves, then
            // one thread stores this row block's flag word
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tid == 0) {
                st_dev_u64(my_flags + (size_t)s * flag_step + (size_t)c * p.nrb + rb,
                           ((uint64_t)epoch << 32) | (uint32_t)s);
                if (p.ticks && rb == 0 && cbg == 0 && c == 0) p.ticks[(size_t)g * T + s] = wall_clock64();
            }
        }
    }

#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int j = w + 4 * o;
            if (j < NTILE && col_reg[c][o] < B) {
                const size_t si = (state_row + col_reg[c][o]) * H + unit_reg[o];
                if (p.hT) p.hT[si] = h_reg[c][o];
                if (p.cT && CELL == CELL_LSTM) p.cT[si] = c_reg[c][o];
            }
        }
}

template <int DT>
__global__ void wavefront_init_kernel(const float* h0, int l0, int LP, int D, int T, int B, int Bp, int H,
                                      void* hseq) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t per = (size_t)B * H;
    const size_t n = (size_t)LP * D * per;
    if (i < n) {
        const size_t g = i / per, rem = i - g * per;
        const float h = h0 ? h0[((size_t)l0 * D) * per + i] : 0.0f;
        const size_t b = rem / H, u = rem - b * H;
        // slot 0 = state before step 0, blocked by 16 hidden units
        const size_t dst = g * (size_t)(T + 1) * Bp * H + ((u >> 4) * Bp + b) * 16 + (u & 15);
        if (DT == DT_BF16) ((bf16_t*)hseq)[dst] = f32_to_bf16(h);
        else ((float*)hseq)[dst] = h;
    }
}

template <class TR, int CELL, int RT, int CT, int KB, bool FUSED, int NCH>
hipError_t launch_variant(const WavefrontArgs& a, hipStream_t stream) {
    if (a.ncb % NCH != 0 || a.nrb % 4 != 0 || a.nrb > 256) return hipErrorInvalidValue;
    if ((size_t)a.Bp * a.H * sizeof(typename TR::elem) >= ((size_t)1 << 31)) return hipErrorInvalidValue;  // 32-bit lane offsets
    if (a.Bp < a.B || a.Bp % 4 != 0) return hipErrorInvalidValue;
    const int grid = a.LP * a.D * a.nrb * (a.ncb / NCH);
    const size_t smem = (size_t)4 * RT * CT * 64 * sizeof(f32x4);
    auto kern = wavefront_kernel<TR, CELL, RT, CT, KB, FUSED, NCH, RNN_CELL_EXT != 0>;
    if (smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    // every workgroup must be resident at once: check what the hardware can hold
    static int max_grid = 0;
    if (max_grid == 0) {
        int dev = 0, per_cu = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern),
                                                         256, smem) != hipSuccess)
            return hipErrorInvalidValue;
        const int want = variant_occupancy(CT);
        max_grid = prop.multiProcessorCount * (per_cu < want ? per_cu : want);
    }
    if (grid > max_grid) return hipErrorInvalidValue;
    kern<<<dim3(grid), dim3(256), smem, stream>>>(a);
    return hipGetLastError();
}

template <class TR, int RT, int CT, int KB, int NCH>
hipError_t launch_cell_fused(const WavefrontArgs& a, hipStream_t stream) {
    const bool fused = a.LP > 1;
    if (a.cell == CELL_LSTM)
        return fused ? launch_variant<TR, CELL_LSTM, RT, CT, KB, true, NCH>(a, stream)
                     : launch_variant<TR, CELL_LSTM, RT, CT, KB, false, NCH>(a, stream);
    return fused ? launch_variant<TR, CELL_GRU, RT, CT, KB, true, NCH>(a, stream)
                 : launch_variant<TR, CELL_GRU, RT, CT, KB, false, NCH>(a, stream);
}

// (dtype, RT, CT, KB, NCH) combinations that are compiled.  KB = H / (4 * KW); CT column tiles
// per chain, NCH chains per workgroup.
#define RNN_WF_VARIANTS(X)                                                        \
    X(TraitsBf16, 1, 4, 1, 1) X(TraitsBf16, 1, 4, 2, 1) X(TraitsBf16, 1, 4, 4, 1) \
    X(TraitsBf16, 4, 4, 4, 1) X(TraitsBf16, 4, 4, 8, 1)                           \
    X(TraitsBf16, 4, 2, 4, 2) X(TraitsBf16, 4, 2, 8, 2)                           \
    X(TraitsBf16, 4, 4, 3, 1) X(TraitsBf16, 4, 4, 5, 1) X(TraitsBf16, 4, 4, 6, 1) \
    X(TraitsBf16, 4, 4, 1, 1) X(TraitsBf16, 4, 4, 2, 1) X(TraitsBf16, 4, 2, 1, 2) X(TraitsBf16, 4, 2, 2, 2) \
    X(TraitsBf16, 2, 2, 10, 2) X(TraitsBf16, 2, 2, 12, 2)                                                      \
    X(TraitsBf16, 4, 2, 3, 2) X(TraitsBf16, 4, 2, 5, 2) X(TraitsBf16, 4, 2, 6, 2) \
    X(TraitsF32, 1, 4, 2, 1) X(TraitsF32, 1, 4, 4, 1) X(TraitsF32, 1, 4, 8, 1)    \
    X(TraitsF32, 1, 4, 16, 1) X(TraitsF32, 1, 4, 32, 1)

template <class TR> struct DtOf;
template <> struct DtOf<TraitsBf16> { static constexpr int value = DT_BF16; };
template <> struct DtOf<TraitsF32> { static constexpr int value = DT_F32; };

hipError_t launch_here(const WavefrontArgs& a, hipStream_t stream) {
    const int kw = a.dtype == DT_BF16 ? TraitsBf16::KW : TraitsF32::KW;
    if (a.H % (4 * kw) != 0) return hipErrorInvalidValue;
    const int KB = a.H / (4 * kw);
#define X(TR, rt, ct, kb, nch)                                                          \
    if (DtOf<TR>::value == a.dtype && a.RT == rt && a.CT == ct && KB == kb && a.NCH == nch)  \
        return launch_cell_fused<TR, rt, ct, kb, nch>(a, stream);
    RNN_WF_VARIANTS(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace

#if RNN_CELL_EXT
hipError_t launch_wavefront_ext(const WavefrontArgs& a, hipStream_t stream) { return launch_here(a, stream); }
#else
hipError_t launch_wavefront_ext(const WavefrontArgs& a, hipStream_t stream);   // wavefront_b.hip

bool wavefront_variant_exists(int dtype, int RT, int CT, int NCH, int H, bool fused) {
    if (fused && variant_occupancy(CT) > 1) return false;  // no room for W_ih at two workgroups per CU
    const int kw = dtype == DT_BF16 ? TraitsBf16::KW : TraitsF32::KW;
    if (H % (4 * kw) != 0) return false;
    const int KB = H / (4 * kw);
#define X(TR, rt, ct, kb, nch) \
    if (DtOf<TR>::value == dtype && RT == rt && CT == ct && KB == kb && NCH == nch) return true;
    RNN_WF_VARIANTS(X)
#undef X
    return false;
}

int wavefront_variant_occupancy(int CT) { return variant_occupancy(CT); }

hipError_t launch_wavefront(const WavefrontArgs& a, hipStream_t stream) {
    return a.ext ? launch_wavefront_ext(a, stream) : launch_here(a, stream);
}

hipError_t launch_wavefront_init(int dtype, const float* h0, int l0, int LP, int D, int T, int B, int Bp,
                                 int H, void* hseq, hipStream_t stream) {
    const size_t n = (size_t)LP * D * B * H;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (dtype == DT_BF16)
        wavefront_init_kernel<DT_BF16><<<blocks, 256, 0, stream>>>(h0, l0, LP, D, T, B, Bp, H, hseq);
    else
        wavefront_init_kernel<DT_F32><<<blocks, 256, 0, stream>>>(h0, l0, LP, D, T, B, Bp, H, hseq);
    return hipGetLastError();
}

#endif  // !RNN_CELL_EXT

}  // namespace rnn
