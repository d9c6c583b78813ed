// Persistent kernel for one layer whose input sequence is complete before the launch and has the
// layer's own width (every layer above the first of a unidirectional stack, and the first when its
// input is H wide): the input product W_ih x_t runs inside the recurrent kernel, cell by cell, as in
// the paper's cell (Section 2.2), so the projection never goes through HBM as fp32.
//
// Same decomposition and step protocol as the flag-vector kernel (a workgroup owns RT*4 hidden
// units for NCH chains of CT*16 sequences, the four waves split K, a vector of flag words per
// step, a write-once blocked state sequence).  What differs:
//   - W_hh stays in registers, because the recurrent product is the part of a step that sits on
//     the dependency chain; the workgroup's W_ih slice follows it into the accumulation registers
//     as far as they reach (wx_register_blocks), and the rest lives in LDS next to the partial-sum
//     exchange buffer, laid out fragment by fragment exactly as the MFMA reads its A operand (each
//     wave reads back only what it wrote itself);
//   - x has the layout of a state sequence (blocked by 16 units): a layer above the first reads
//     the state sequence of the layer below directly (and a layer that is not the last keeps no
//     other output), the first layer reads a re-laid-out copy of the caller's x.  Fragment loads
//     then ask for whole cache lines; the CU's path to L2 is bound by requests, not bytes;
//   - x_t needs no flags: with several chains, a chain step does its input part first (its
//     fragments were requested during the previous chain step) while the flags it will need
//     become visible, then the recurrent part;
//   - one wave writes a chain step to memory, from LDS, in whole cache lines, and is the only
//     one that needs a store acknowledged; it waits for the acknowledgement early in the next
//     chain step (the stores are then its only memory operations in flight: the state fragments
//     of the next chain step were requested before the gates) and stores the flag word there;
//   - a launch may hold several such layers side by side (template flag MULTI): a layer above the
//     first of the launch takes the state sequence of the group below as its x, as it is produced,
//     behind that group's flag vectors.
#include "wf_traits.h"

// Every variant exists twice: with the plain cell, and (RNN_CELL_EXT = 1, the translation unit
// wavefront_x_b.hip) with the optional peephole and clipping terms in the gate phase, so that a model
// without those terms runs exactly the plain cell's instructions.
#ifndef RNN_CELL_EXT
#define RNN_CELL_EXT 0
#endif


namespace rnn {

namespace {

// How many of the KB K blocks of a wave's W_ih slice stay in (accumulation) registers instead of LDS.
// Beside the RT * KB fragments of W_hh a lane has room for 224 weight registers in all (256 accumulation registers less the 32 accumulators); what
// fits there needs no LDS read in the input part, whose A fragments otherwise keep LDS as busy as the
// matrix unit (four 1 KiB reads per eight matrix instructions and wave).  (With all 256 accumulation
// registers given to weights and the accumulators in vector registers instead, both slices of 1024 units
// would fit, but matrix instructions whose C operand sits in the vector registers run much slower here:
// 2 layers of 512 units at batch 512 take 1.83 ms that way against 1.36.)  Only where the matrix
// instruction can take A from those registers, and for the interleaved-chain shapes.
template <class TR, int RT, int KB, int NCH>
constexpr int wx_register_blocks() {
    if (!TR::HAS_ACC_A || NCH != 2) return 0;
    constexpr int regs_per_frag = (int)(sizeof(typename TR::frag) / 4);
    constexpr int room = 224 - RT * KB * regs_per_frag;
    constexpr int fit = room > 0 ? room / (RT * regs_per_frag) : 0;
    return fit < KB ? fit : KB;
}

// MULTI: the launch runs p.LP layers side by side, one group of workgroups each; a layer above the first
// of the launch reads the state sequence of the group below as its x, behind that group's flags, so the
// groups settle on successive anti-diagonals of the layer x time grid (paper Section 2.2).
template <class TR, int CELL, int RT, int CT, int KB, int NCH, bool MULTI, bool EXT>
__global__ __launch_bounds__(256, 1) void wavefront_x_kernel(WavefrontArgs p) {
    // peephole weights of an extended LSTM cell: in LDS for the interleaved-chain shapes (no register to
    // spare beside the resident weights), in registers otherwise (no LDS to spare beside the W_ih slice)
    constexpr bool PEEP_LDS = EXT && CELL == CELL_LSTM && NCH == 2;
    constexpr bool PEEP_REG = EXT && CELL == CELL_LSTM && NCH != 2;
    static_assert(!MULTI || NCH > 1, "layers side by side need interleaved chains");
    typedef typename TR::elem elem;
    typedef typename TR::frag frag;
    constexpr int KW = TR::KW;
    constexpr int NTILE = RT * CT;                 // 16x16 output tiles per chain
    constexpr int NOWN = (NTILE + 3) / 4;          // tiles of a chain finished by one wave
    constexpr int KBR = wx_register_blocks<TR, RT, KB, NCH>();   // K blocks of the W_ih slice held in registers
    constexpr int KBL = KB - KBR;                  // ... and in LDS
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    f32x4* red = reinterpret_cast<f32x4*>(smem_raw);  // [4 waves][NTILE][64 lanes]
    frag* wxl = reinterpret_cast<frag*>(smem_raw + (size_t)4 * NTILE * 64 * sizeof(f32x4));  // [4][RT][KBL][64]
    // (PEEP_LDS) peephole weights of the workgroup's units [3][RT * 4] (zeros without them): read with the
    // partial sums in the gate phase, so that they cost no registers across the matrix parts
    float* peep_lds = reinterpret_cast<float*>(smem_raw + (size_t)4 * NTILE * 64 * sizeof(f32x4) +
                                               (size_t)4 * RT * KBL * 64 * sizeof(frag));

    __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;

    const int v = xcd_contiguous_id();
    const int ngrp = p.ncb / NCH;                   // column block groups (ncb counts chains)
    const int wpl = p.nrb * ngrp;                   // workgroups per layer
    const int g = MULTI ? v / wpl : 0;              // layer of the launch this workgroup belongs to
    if (v >= (MULTI ? p.LP : 1) * wpl) return;
    const int vr = v - g * wpl;
    const int cbg = vr / p.nrb, rb = vr - cbg * p.nrb;
    const int l = p.l0 + g;
    const bool xfused = MULTI && g > 0;             // x_t = state of the group below, guarded by its flags
    const int H = p.H, B = p.B, T = p.T;
    const int Bp = p.Bp;                            // rows per 16-unit block of a state sequence
    const int kq = H / 4;                           // K range of one wave inside each part

    // per-workgroup rotation of the K blocks and of the column tiles (see load_part)
    const int rot_k = rb % KB;
    const int rot_c = (rb / KB) % CT;

    // ---- resident weights: W_hh fragments in registers, W_ih fragments in LDS ------------------
    frag wh[RT][KB];
    frag wxr[RT][KBR > 0 ? KBR : 1];               // W_ih K blocks KBL.. (register slots)
    frag* wx_mine = wxl + (size_t)w * RT * KBL * 64 + lane;
    {
        const elem* whh = static_cast<const elem*>(p.whh[g]);
        const elem* wih = static_cast<const elem*>(p.wih[g]);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const size_t row = (size_t)(rb * RT + rt) * 16 + (lane & 15);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const int k = w * kq + wrap_kb<KB>(kb + rot_k) * KW + TR::koff(lane);
                wh[rt][kb] = TR::load(whh + row * H + k);
                if (kb < KBL) wx_mine[(rt * KBL + kb) * 64] = TR::load(wih + row * H + k);
                else wxr[rt][kb - KBL] = TR::load(wih + row * H + k);
            }
        }
    }

    // ---- per-lane state of the (unit, sequence) pairs this lane finishes ---------------------
    float c_reg[NCH][NOWN], h_reg[NCH][NOWN];
    int len_reg[NCH][NOWN];                         // valid steps of the pair's sequence; 0 for a column beyond the batch
    f32x4 bias_reg[NOWN];
    int unit_reg[NOWN];
    float peep_reg[PEEP_REG ? NOWN : 1][3];
    const size_t state_row = (size_t)l * B;
#pragma unroll
    for (int o = 0; o < NOWN; ++o) {
        const int j = w + 4 * o;                    // tile index = rt * CT + ct
        const int rt = j / CT, ct = j - rt * CT;
        const int unit = (rb * RT + rt) * 4 + (lane >> 4);
        unit_reg[o] = unit;
        bias_reg[o] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (j < NTILE) bias_reg[o] = *reinterpret_cast<const f32x4*>(p.bias[g] + (size_t)unit * SLOTS);
        if constexpr (PEEP_REG) {
            const CellExt e = load_cell_ext(p.peep[g], H, min(unit, H - 1), p.clip);
            peep_reg[o][0] = e.p_i; peep_reg[o][1] = e.p_f; peep_reg[o][2] = e.p_o;
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int col = ((cbg * NCH + c) * CT + (ct + rot_c) % CT) * 16 + (lane & 15);
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

    const float clip_lim = p.clip > 0.0f ? p.clip : __builtin_inff();   // uniform
    if constexpr (PEEP_LDS) {
        if (tid < 3 * RT * 4) {
            const int k = tid / (RT * 4), u = tid - k * (RT * 4);
            peep_lds[tid] = p.peep[g] ? p.peep[g][(size_t)k * H + rb * RT * 4 + u] : 0.0f;
        }
        // (the first barrier of the first chain step orders these writes before the first read)
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
    elem* out = static_cast<elem*>(p.out[g]);
    // x of a layer above the first of the launch: slot t + 1 of the state sequence of the group below
    const elem* xin = xfused ? hseq - (size_t)(T + 1) * Bp * H + (size_t)Bp * H : static_cast<const elem*>(p.xin);
    // flag word of (layer of the launch, step, chain column block, row block): ((g*T + s)*ncb + cb)*nrb + rb
    const size_t flag_step = (size_t)p.ncb * p.nrb;
    uint64_t* my_flags = p.flagv + (size_t)g * T * flag_step + (size_t)(cbg * NCH) * p.nrb;   // chain 0
    const uint64_t* x_flags = my_flags - (size_t)T * flag_step;     // the group below (xfused only)
    const uint32_t epoch = p.epoch;
    bool aborted = false;
    const int kbase = w * kq + TR::koff(lane);
    // a wave waits only for the row blocks that produce the cache lines (16 units each) of its own
    // K quarter of the state
    int fl0, nfl;
    flag_span(w * kq, kq, H, 16, RT * 4, fl0, nfl);

    frag hbuf[KB][CT];   // h_{t-1} fragments of the chain step that is processed next
    frag xbuf[KB][CT];   // x_t fragments of the chain step that is processed next
    // Loads are never predicated (the compiler can then count them and waits only for what an
    // instruction needs); past the last step they re-read the last one.
    auto poll_h = [&](int c, int s) {  // wait until step s-1 of chain c is published
        if (s > 0)
            wait_flags(my_flags + (size_t)(s - 1) * flag_step + (size_t)c * p.nrb + fl0, nfl, lane, epoch,
                       p.status, p.spin_limit, aborted);
    };
    // Addresses of the activation loads = uniform base of the step + uniform offset of the K block
    // + a 32-bit per-lane offset that does not change over the launch (one register per chain and
    // column tile; full per-load pointers would not fit beside the resident weights).  In the
    // blocked layout a K block of KW units lies KW * B elements further when KW is a multiple of
    // 16; otherwise (fp32 fragments of 4 units) the offset is computed per load.
    constexpr bool LINEAR_K = (KW % 16) == 0;
    uint32_t hoff[NCH][CT];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            hoff[c][ct] = (uint32_t)(hseq_off(kbase, bcol[c][ct], Bp) * sizeof(elem));
        }
    auto blocked_ptr = [&](const elem* step, int c, int ct, int kb) -> const elem* {
        const int kr = wrap_kb<KB>(kb + rot_k);
        if (LINEAR_K)
            return reinterpret_cast<const elem*>(reinterpret_cast<const char*>(step) +
                                                 (size_t)kr * KW * Bp * sizeof(elem) + hoff[c][ct]);
        return step + hseq_off(kbase + kr * KW, bcol[c][ct], Bp);
    };
    auto load_h = [&](int c, int s, int kb) {  // K block kb of the state after step s-1
        const elem* hprev = hseq + (size_t)min(s, T - 1) * Bp * H;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) hbuf[kb][ct] = TR::load(blocked_ptr(hprev, c, ct, kb));
    };
    auto load_x = [&](int c, int s, int kb) {  // K block kb of x at step s (same layout as the state)
        const elem* xs = xin + (size_t)min(s, T - 1) * Bp * H;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) xbuf[kb][ct] = TR::load(blocked_ptr(xs, c, ct, kb));
    };
    // wave 0: flag word of the chain step whose stores are still to be acknowledged
    uint64_t* pend_flag = nullptr;
    int pend_step = 0, pend_chain = 0;
    // Word touched by the L2 prefetch of x (wave 0).  Nothing uses it, but its register must stay
    // reserved until the load has returned: the empty asm that "uses" it sits behind a wait that
    // has covered the load anyway, so that it never causes a wait of its own.
    uint32_t pf = 0;
    auto store_pending_flag = [&]() {
        if (pend_flag != nullptr) {
            // every memory operation of this wave has completed, the stores of the chain step among them
            // (no counting: whatever else the wave has in flight, a spilled register included, is waited
            // for as well and was issued long before the stores)
            __builtin_amdgcn_s_waitcnt(0x0F70);
            asm volatile("" ::: "memory");
            asm volatile("" ::"v"(pf));
            if (lane == 0) {
                st_dev_u64(pend_flag, ((uint64_t)epoch << 32) | (uint32_t)pend_step);
                if (p.ticks && rb == 0 && cbg == 0 && pend_chain == 0) p.ticks[(size_t)g * T + pend_step] = wall_clock64();
            }
            pend_flag = nullptr;
        }
    };

    // acc += W_ih slice (A fragments from LDS, read one K block ahead of the matrix instructions)
    // x the x fragments.  The scheduling barriers keep the compiler from sinking each LDS read to
    // its first use, which would expose the LDS latency once per fragment.
    auto input_part = [&](f32x4 (&acc)[RT][CT], const uint64_t* xflag, uint64_t& seenx) {
        if (KBL == 0) {
            // the first matrix instructions read the freshly zeroed accumulators from inside an asm
            // statement: keep two wait states between those writes and them
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) asm volatile("s_nop 1" : "+a"(acc[rt][ct]));
        }
        frag abuf[2][RT];
        if (KBL > 0) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) abuf[0][rt] = wx_mine[(rt * KBL + 0) * 64];
        }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            if (kb + 1 < KBL) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) abuf[(kb + 1) & 1][rt] = wx_mine[(rt * KBL + kb + 1) * 64];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    if (kb < KBL) acc[rt][ct] = TR::mfma(abuf[kb & 1][rt], xbuf[kb][ct], acc[rt][ct]);
                    else TR::mfma_acc_a(wxr[rt][kb - KBL], xbuf[kb][ct], acc[rt][ct]);   // the recurrent part follows: no wait here
                }
            if (NCH > 1 && kb == KB / 8 && w == 0) store_pending_flag();
            // (a layer above the first of the launch) the flag word of the group below for the x fragments
            // that the recurrent part is about to request
            if (MULTI && kb == KB / 2 && xflag != nullptr) seenx = ld_dev_u64(xflag);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // acc += W_hh slice (registers) x the state fragments; the x fragments of chain step (cn, sn),
    // whose registers the input part has just released, are requested between the matrix
    // instructions, one K block per K block, so that the loads do not queue up in one burst.
    auto recurrent_part_prefetching_x = [&](f32x4 (&acc)[RT][CT], int cn, int sn, const uint64_t* flag,
                                            uint64_t& seen) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) TR::mfma_acc_a(wh[rt][kb], hbuf[kb][ct], acc[rt][ct]);
            // a little past half way the flag word this lane will poll is requested: by then it has
            // usually become visible (measured: earlier and the check fails too often, later and
            // the word comes back behind too many x fragments), and its round trip hides behind
            // the remaining instructions
            if (kb == (5 * KB) / 8) seen = ld_dev_u64(flag);
            load_x(cn, sn, kb);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (TR::HAS_ACC_A) wait_mfma_results();
    };

    // x comes from HBM, and every load a wave has in flight holds back the store acknowledgement
    // it waits for at the end of a chain step (memory operations return in order).  The workgroups
    // of a column group that share an XCD read the same x lines through the same L2, so wave 0 of
    // each of them touches a share of the lines two chain steps ahead with one-dword loads; the
    // fragment loads then hit L2.  Purely a hint: lines nobody touches are simply fetched later.
    const bool xcd_packed = (gridDim.x & 7) == 0;
    const int per_xcd = xcd_packed ? min((int)gridDim.x >> 3, p.nrb) : max(p.nrb >> 3, 1);
    const int pf_idx = xcd_packed ? rb % per_xcd : min(rb >> 3, per_xcd - 1);
    constexpr int LINE = 128 / (int)sizeof(elem);                 // elements per cache line
    constexpr int NLINES = CT * 16 * 16 / LINE;                    // lines of a chain per block of 16 units
    uint32_t pf_off[NCH];   // element offset, inside one step of x, of the line this lane touches
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col0 = (cbg * NCH + c) * CT * 16;
        const int line = min(pf_idx + per_xcd * lane, NLINES * (H / 16) - 1);
        const size_t off = ((size_t)(line / NLINES) * Bp + col0) * 16 + (size_t)(line % NLINES) * LINE;
        pf_off[c] = (uint32_t)(min(off, (size_t)Bp * H - 1) & ~(size_t)(LINE - 1));
    }
    auto touch_x = [&](int c, int s) -> uint32_t {
        return *reinterpret_cast<const uint32_t*>(xin + (size_t)min(s, T - 1) * Bp * H + pf_off[c]);
    };

    if (NCH > 1) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) load_h(0, 0, kb);
    }
    auto wait_x = [&](int c, int s) {  // wait until step s of chain c of the group below is published
        wait_flags<true>(x_flags + (size_t)s * flag_step + (size_t)c * p.nrb + fl0, nfl, lane, epoch, p.status,
                         p.spin_limit, aborted);
    };
    if (xfused) wait_x(0, 0);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) load_x(0, 0, kb);

    for (int s = 0; s < T; ++s) {
        const int t = s;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            f32x4 acc[RT][CT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) acc[rt][ct] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            // the chain step after this one
            const int cn = (c + 1 < NCH) ? c + 1 : 0;
            const int sn = (c + 1 < NCH) ? s : s + 1;

            if (NCH > 1) {
                // Input part first.  The flags this chain step will poll (those of the chain step
                // after it, the same chain as the one just published) were stored moments ago and
                // need about half a microsecond to become visible; both matrix parts run meanwhile.
                const uint64_t* xflag = (xfused && sn < T)
                    ? x_flags + (size_t)sn * flag_step + (size_t)cn * p.nrb + fl0 + min(lane, nfl - 1) : nullptr;
                uint64_t seenx = 0;
                input_part(acc, xflag, seenx);
                if (MULTI && xflag != nullptr && !__all((uint32_t)(seenx >> 32) == epoch)) wait_x(cn, sn);
                if (MULTI) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");  // the x requests stay below the flag check
                // flag word of this lane for step sn-1 of chain cn (clamped to a word that exists)
                const uint64_t* flag = my_flags + (size_t)max(sn - 1, 0) * flag_step + (size_t)cn * p.nrb + fl0 +
                                       min(lane, nfl - 1);
                uint64_t seen = 0;
                recurrent_part_prefetching_x(acc, cn, sn, flag, seen);
                if (sn > 0 && sn < T && !__all((uint32_t)(seen >> 32) == epoch)) poll_h(cn, sn);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");  // loads of the state stay below the flag check
                if (w == 0 && !xfused) pf = touch_x((c + 2) % NCH, s + (c + 2) / NCH);   // (never lines that are still being written)
                // The state of the next chain step (its flags have just been seen) is requested now: its
                // registers are free since the last matrix instruction, and the fragments travel while the
                // partial sums are exchanged and the gates run.
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) load_h(cn, sn, kb);
                __builtin_amdgcn_sched_barrier(0);
            } else {
                // One chain: the state is requested as late as possible, after the input part.
                uint64_t unused_x = 0;
                input_part(acc, nullptr, unused_x);
                poll_h(0, s);
                if (w == 0) pf = touch_x((c + 2) % NCH, s + (c + 2) / NCH);
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) load_h(0, s, kb);
                mma_part<TR, RT, CT, KB>(wh, hbuf, acc);
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
                for (int q = 0; q < 4; ++q)
                    part[o][q] = red[(q * NTILE + min(w + 4 * o, NTILE - 1)) * 64 + lane];
            CellExt ext[NOWN];
#pragma unroll
            for (int o = 0; o < NOWN; ++o) ext[o] = CellExt{0.0f, 0.0f, 0.0f, clip_lim};
            if constexpr (PEEP_LDS) {
#pragma unroll
                for (int o = 0; o < NOWN; ++o) {
                    const int ul = min(unit_reg[o] - rb * RT * 4, RT * 4 - 1);     // unit inside the workgroup's slice
                    ext[o].p_i = peep_lds[ul];
                    ext[o].p_f = peep_lds[RT * 4 + ul];
                    ext[o].p_o = peep_lds[2 * RT * 4 + ul];
                }
            }
            if constexpr (PEEP_REG) {
#pragma unroll
                for (int o = 0; o < NOWN; ++o) {
                    ext[o].p_i = peep_reg[o][0]; ext[o].p_f = peep_reg[o][1]; ext[o].p_o = peep_reg[o][2];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int o = 0; o < NOWN; ++o) {
                if (NCH == 1) {
                    // one chain: the input of the next step is requested in NOWN portions between
                    // the gate computations (its registers are free since the input part)
#pragma unroll
                    for (int kb = (o * KB) / NOWN; kb < ((o + 1) * KB) / NOWN; ++kb) load_x(cn, sn, kb);
                    __builtin_amdgcn_sched_barrier(0);
                }
                const int j = w + 4 * o;
                if (j < NTILE) {  // uniform per wave
                    f32x4 a = (part[o][0] + part[o][1]) + (part[o][2] + part[o][3]);
                    a += bias_reg[o];
                    const bool active = t < len_reg[c][o];
                    float c_new = c_reg[c][o];
                    const float pre[SLOTS] = {a[0], a[1], a[2], a[3]};
                    float hn;
                    if constexpr (EXT) hn = cell_update_ext<CELL>(pre, h_reg[c][o], c_new, ext[o]);
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
                    // Hand the values to wave 0 through LDS: [sequence n][unit u] inside the first
                    // partial-sum region of this tile, which only this wave has read and only wave 0
                    // will write again (in the next chain step, after it has read this).
                    elem* stage = reinterpret_cast<elem*>(red + (size_t)j * 64);
                    stage[(lane & 15) * 4 + (lane >> 4)] = state_v;
                    if (out) stage[64 + (lane & 15) * 4 + (lane >> 4)] = out_v;
                }
            }

            // Publish.  After the barrier wave 0 alone writes the chain step to memory, 4 units (one
            // piece) per lane, consecutive lanes consecutive addresses, so whole cache lines leave in
            // one instruction; it is then the only wave that has to see a store acknowledged.
            __syncthreads();
            if (w == 0) {
                typedef typename TR::piece piece;
#pragma unroll
                for (int it = 0; it < NOWN; ++it) {
                    const int pc = lane + 64 * it;           // piece = (sequence of the chain, tile row)
                    const int sl = pc / RT, rt = pc - sl * RT;
                    const int ct = ((sl >> 4) - rot_c + CT) % CT;
                    const int col = (cbg * NCH + c) * CT * 16 + sl;
                    const elem* stage = reinterpret_cast<const elem*>(red + (size_t)(rt * CT + ct) * 64) + (sl & 15) * 4;
                    const int unit0 = (rb * RT + rt) * 4;
                    if (col < B) {
                        TR::store_piece_dev(hcur + hseq_off(unit0, col, Bp), *reinterpret_cast<const piece*>(stage));
                        if (out)
                            *reinterpret_cast<piece*>(out + ((size_t)t * B + col) * H + unit0) =
                                *reinterpret_cast<const piece*>(stage + 64);
                    }
                }
            }
            asm volatile("" ::: "memory");
            if (NCH > 1) {
                // Wave 0 waits for the acknowledgement of these stores early in the input part of the
                // next chain step, where it hardly has to wait any more, and stores the flag word there.
                pend_flag = my_flags + (size_t)s * flag_step + (size_t)c * p.nrb + rb;
                pend_step = s;
                pend_chain = c;
            } else if (w == 0) {
                // one chain: the next step polls this flag at once
                __builtin_amdgcn_s_waitcnt(0x0F70);
                asm volatile("" ::: "memory");
                if (lane == 0) {
                    st_dev_u64(my_flags + (size_t)s * flag_step + rb, ((uint64_t)epoch << 32) | (uint32_t)s);
                    if (p.ticks && rb == 0 && cbg == 0) p.ticks[(size_t)g * T + s] = wall_clock64();
                }
            }
            if (NCH == 1) asm volatile("" ::"v"(pf));
        }
    }
    if (NCH > 1 && w == 0) store_pending_flag();

#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int j = w + 4 * o;
            const int col = ((cbg * NCH + c) * CT + (j % CT + rot_c) % CT) * 16 + (lane & 15);
            if (j < NTILE && col < B) {
                const size_t si = (state_row + col) * H + unit_reg[o];
                if (p.hT) p.hT[si] = h_reg[c][o];
                if (p.cT && CELL == CELL_LSTM) p.cT[si] = c_reg[c][o];
            }
        }
}

// [rows of H elements] -> blocked by 16 elements: dst[t][H/16][Bp][16] from src[t][B][H] (rows B..Bp-1
// of a block are padding and stay unwritten).  One
// workgroup moves 16 sequences of one step through LDS, so that it reads whole rows and writes
// runs of 16 sequences x 16 units (both sides in whole cache lines).  ES = element size in bytes.
template <int ES>
__global__ __launch_bounds__(256) void to_blocked_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                          int B, int Bp, int H) {
    extern __shared__ uint4 tile[];                 // [16 sequences][U] 16-byte units
    const int U = H * ES / 16;                      // 16-byte units per row
    const int t = blockIdx.y, b0 = blockIdx.x * 16;
    const int nb = min(16, B - b0);
    for (int i = threadIdx.x; i < nb * U; i += 256) {
        const int r = i / U, u = i - r * U;
        tile[r * U + u] = src[((size_t)t * B + b0 + r) * U + u];
    }
    __syncthreads();
    // output order: [block of 16 units][sequence][ES units of 16 bytes]
    for (int i = threadIdx.x; i < 16 * U; i += 256) {
        const int q = i % ES, r = (i / ES) % 16, blk = i / (ES * 16);
        if (r < nb) dst[(((size_t)t * (H / 16) + blk) * Bp + b0 + r) * ES + q] = tile[r * U + blk * ES + q];
    }
}

template <class TR, int RT, int CT, int KB, int NCH>
constexpr size_t lds_bytes() {
    return (size_t)4 * RT * CT * 64 * sizeof(f32x4) +
           (size_t)4 * RT * (KB - wx_register_blocks<TR, RT, KB, NCH>()) * 64 * sizeof(typename TR::frag) +
           ((RNN_CELL_EXT && NCH == 2) ? (size_t)3 * RT * 4 * sizeof(float) : 0);   // partial sums, W_ih blocks, (extended cell, two chains) peephole weights
}

int device_lds_limit() {
    static int limit = -1;
    if (limit < 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess)
            limit = v;
        else
            limit = 0;
    }
    return limit;
}

template <class TR, int CELL, int RT, int CT, int KB, int NCH, bool MULTI>
hipError_t launch_variant(const WavefrontArgs& a, hipStream_t stream) {
    if (a.ncb % NCH != 0 || a.nrb % 4 != 0 || a.nrb > 256) return hipErrorInvalidValue;
    if (a.LP < 1 || a.LP > WF_MAX_LAYERS || (!MULTI && a.LP != 1)) return hipErrorInvalidValue;
    if ((size_t)a.Bp * a.H * sizeof(typename TR::elem) >= ((size_t)1 << 31)) return hipErrorInvalidValue;  // 32-bit lane offsets
    if (a.Bp < a.B || a.Bp % 4 != 0) return hipErrorInvalidValue;
    const int grid = a.LP * a.nrb * (a.ncb / NCH);
    constexpr size_t smem = lds_bytes<TR, RT, CT, KB, NCH>();
    if (smem > (size_t)device_lds_limit()) return hipErrorInvalidValue;
    auto kern = wavefront_x_kernel<TR, CELL, RT, CT, KB, NCH, MULTI, RNN_CELL_EXT != 0>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    // every workgroup must be resident at once: one per compute unit
    static int max_grid = 0;
    if (max_grid == 0) {
        int dev = 0, per_cu = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern),
                                                         256, smem) != hipSuccess)
            return hipErrorInvalidValue;
        max_grid = prop.multiProcessorCount * (per_cu < 1 ? per_cu : 1);
    }
    if (grid > max_grid) return hipErrorInvalidValue;
    kern<<<dim3(grid), dim3(256), smem, stream>>>(a);
    return hipGetLastError();
}

template <class TR, int RT, int CT, int KB, int NCH>
hipError_t launch_cell(const WavefrontArgs& a, hipStream_t stream) {
    if (a.LP > 1) {   // several layers side by side: compiled for the interleaved-chain shapes only
        if constexpr (NCH > 1) {
            if (a.cell == CELL_LSTM) return launch_variant<TR, CELL_LSTM, RT, CT, KB, NCH, true>(a, stream);
            return launch_variant<TR, CELL_GRU, RT, CT, KB, NCH, true>(a, stream);
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (a.cell == CELL_LSTM) return launch_variant<TR, CELL_LSTM, RT, CT, KB, NCH, false>(a, stream);
    return launch_variant<TR, CELL_GRU, RT, CT, KB, NCH, false>(a, stream);
}

// (dtype, RT, CT, KB, NCH) combinations that are compiled: the same shapes as the flag-vector
// kernel's, so a plan chosen for that kernel can run either.
#define RNN_WFX_VARIANTS(X)                                                       \
    X(TraitsBf16, 1, 4, 1, 1) X(TraitsBf16, 1, 4, 2, 1) X(TraitsBf16, 1, 4, 4, 1) \
    X(TraitsBf16, 4, 4, 4, 1) X(TraitsBf16, 4, 4, 8, 1)                           \
    X(TraitsBf16, 4, 2, 4, 2) X(TraitsBf16, 4, 2, 8, 2)                           \
    X(TraitsBf16, 4, 4, 3, 1) X(TraitsBf16, 4, 4, 5, 1) X(TraitsBf16, 4, 4, 6, 1) \
    X(TraitsBf16, 4, 4, 1, 1) X(TraitsBf16, 4, 4, 2, 1) X(TraitsBf16, 4, 2, 1, 2) X(TraitsBf16, 4, 2, 2, 2) \
    X(TraitsBf16, 2, 2, 10, 2) X(TraitsBf16, 2, 2, 12, 2)                                                      \
    X(TraitsBf16, 4, 2, 3, 2) X(TraitsBf16, 4, 2, 5, 2) X(TraitsBf16, 4, 2, 6, 2) \
    X(TraitsF32, 1, 4, 2, 1) X(TraitsF32, 1, 4, 4, 1) X(TraitsF32, 1, 4, 8, 1)    \
    X(TraitsF32, 1, 4, 16, 1)

template <class TR> struct DtOf;
template <> struct DtOf<TraitsBf16> { static constexpr int value = DT_BF16; };
template <> struct DtOf<TraitsF32> { static constexpr int value = DT_F32; };

hipError_t launch_here(const WavefrontArgs& a, hipStream_t stream) {
    if (a.LP < 1 || a.D != 1 || a.xin == nullptr) return hipErrorInvalidValue;
    const int kw = a.dtype == DT_BF16 ? TraitsBf16::KW : TraitsF32::KW;
    if (a.H % (4 * kw) != 0) return hipErrorInvalidValue;
    const int KB = a.H / (4 * kw);
#define X(TR, rt, ct, kb, nch)                                                          \
    if (DtOf<TR>::value == a.dtype && a.RT == rt && a.CT == ct && KB == kb && a.NCH == nch)  \
        return launch_cell<TR, rt, ct, kb, nch>(a, stream);
    RNN_WFX_VARIANTS(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace

#if RNN_CELL_EXT
hipError_t launch_wavefront_x_ext(const WavefrontArgs& a, hipStream_t stream) { return launch_here(a, stream); }
#else
hipError_t launch_wavefront_x_ext(const WavefrontArgs& a, hipStream_t stream);   // wavefront_x_b.hip

bool wavefront_x_variant_exists(int dtype, int RT, int CT, int NCH, int H, size_t lds_limit, bool several_layers) {
    if (several_layers && NCH < 2) return false;
    const int kw = dtype == DT_BF16 ? TraitsBf16::KW : TraitsF32::KW;
    if (H % (4 * kw) != 0) return false;
    const int KB = H / (4 * kw);
#define X(TR, rt, ct, kb, nch)                                                               \
    if (DtOf<TR>::value == dtype && RT == rt && CT == ct && KB == kb && NCH == nch)          \
        return lds_bytes<TR, rt, ct, kb, nch>() <= lds_limit;
    RNN_WFX_VARIANTS(X)
#undef X
    return false;
}

hipError_t launch_to_blocked(int dtype, const void* src, void* dst, int T, int B, int Bp, int H, hipStream_t stream) {
    const int es = dtype == DT_BF16 ? 2 : 4;
    if (H % 16 != 0 || T < 1 || B < 1 || Bp < B || T > 65535) return hipErrorInvalidValue;
    const size_t smem = (size_t)16 * H * es;
    if (smem > 64 * 1024) return hipErrorInvalidValue;
    const dim3 grid((B + 15) / 16, T);
    if (es == 2)
        to_blocked_kernel<2><<<grid, 256, smem, stream>>>((const uint4*)src, (uint4*)dst, B, Bp, H);
    else
        to_blocked_kernel<4><<<grid, 256, smem, stream>>>((const uint4*)src, (uint4*)dst, B, Bp, H);
    return hipGetLastError();
}

hipError_t launch_wavefront_x(const WavefrontArgs& a, hipStream_t stream) {
    return a.ext ? launch_wavefront_x_ext(a, stream) : launch_here(a, stream);
}

#endif  // !RNN_CELL_EXT

}  // namespace rnn
