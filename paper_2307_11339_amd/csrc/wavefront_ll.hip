// Persistent wavefront kernel for small batches: the step synchronisation rides on the data.
//
// Same decomposition as wavefront.hip (one workgroup group per (layer, direction) of the
// unrolled cell grid, paper Section 2.2; weights resident in registers as MFMA A operands; four
// waves split K), for workgroups that own a single tile of 16 sequences.  At batch sizes like
// these a step is a few hundred nanoseconds of arithmetic, so the cost of a step is the number
// of device-memory round trips on its critical path.  Counters need about four (write h, wait
// for the acknowledgement, bump the counter, see the counter, read h).  Here every 8-byte word
// of the exchanged state carries its own tag:
//       word = { payload: two bf16 values (or one fp32 value), tag: 32-bit launch epoch }
// A producer simply stores the words; a consumer loads the words it needs and retries until
// all their tags equal the epoch of this launch.  8-byte accesses are single-copy atomic, so a
// word is either old (tag differs) or complete.  The state sequence has one slot per step
// (slot 0 = h0, slot s+1 = state after step s), each word is written once per launch, and the
// epoch changes with every launch, so nothing has to be cleared between launches.  Critical
// path per step: the store becoming visible and one load round trip (both overlap: a load issued
// right after the stores comes back about when they have landed), the matrix part, two workgroup
// barriers; no counters and no store acknowledgement wait.
//
// For a unidirectional stack the layer above reads the same state sequence as its x_t: where a
// sequence is still running the state is the layer's output, and where it is padded the cell
// above is inactive as well and ignores its input.
// Every wait is bounded (poll budget, shared status word), so the grid always drains.
#include "wf_traits.h"

// The variants of this kernel are compiled in three translation units so that the build runs in
// parallel: this file is part 0 (and holds the public functions); wavefront_ll_b.hip and
// wavefront_ll_c.hip include it with RNN_LL_PART set to 1 and 2.
#ifndef RNN_LL_PART
#define RNN_LL_PART 0
#endif
// Every variant exists twice: with the plain cell, and (RNN_CELL_EXT = 1, the translation units
// wavefront_ll_d/e/f.hip) with the optional peephole and clipping terms in the gate phase, so that a model
// without those terms runs exactly the plain cell's instructions.
#ifndef RNN_CELL_EXT
#define RNN_CELL_EXT 0
#endif

namespace rnn {
namespace {

struct LLBf16 : TraitsBf16 {
    static constexpr int WORDS_PER_KW = 16;  // 32 bf16 values = 16 tagged words
    static __device__ inline int row_words(int H) { return H / 2; }
    static __device__ inline int word_of(int k) { return k >> 1; }
    // fragment of 8 consecutive K values = the payloads of 4 tagged words, staged in LDS
    static __device__ inline frag frag_from_lds(const uint32_t* p) {
        union { u32x4 u; frag f; } v;
        v.u = *reinterpret_cast<const u32x4*>(p);
        return v.f;
    }
    // lanes n, n+16, n+32, n+48 hold units unit0..unit0+3 of sequence n; lane n writes them
    static __device__ inline void ll_publish(elem state, elem outv, bool valid, bool write_out,
                                             int lane, uint32_t epoch, uint64_t* state_dst,
                                             elem* out_dst) {
        uint32_t v0, v1, v2, v3;
        gather_rows((uint32_t)state | ((uint32_t)outv << 16), v0, v1, v2, v3);
        if (valid && lane < 16) {
            const uint64_t tag = (uint64_t)epoch << 32;
            st_dev_u64(state_dst, tag | (v0 & 0xFFFFu) | ((v1 & 0xFFFFu) << 16));
            st_dev_u64(state_dst + 1, tag | (v2 & 0xFFFFu) | ((v3 & 0xFFFFu) << 16));
            if (write_out) {
                const uint64_t ov = (uint64_t)(v0 >> 16) | ((uint64_t)(v1 >> 16) << 16) |
                                    ((uint64_t)(v2 >> 16) << 32) | ((uint64_t)(v3 >> 16) << 48);
                *reinterpret_cast<uint64_t*>(out_dst) = ov;
            }
        }
    }
};

struct LLF32 : TraitsF32 {
    static constexpr int WORDS_PER_KW = 4;
    static __device__ inline int row_words(int H) { return H; }
    static __device__ inline int word_of(int k) { return k; }
    static __device__ inline frag frag_from_lds(const uint32_t* p) { return __uint_as_float(*p); }
    static __device__ inline void ll_publish(elem state, elem outv, bool valid, bool write_out,
                                             int lane, uint32_t epoch, uint64_t* state_dst,
                                             elem* out_dst) {
        if (valid) {
            st_dev_u64(state_dst + (lane >> 4), ((uint64_t)epoch << 32) | __float_as_uint(state));
            if (write_out) out_dst[lane >> 4] = outv;
        }
    }
};

// One wave fetches the tagged words of its K quarter for all sequences of its column block
// (ncol rows of QW words), checks the tags and leaves the payloads in its own LDS staging area
// [col][QW + pad] as plain dwords.  Every lane loads 16 bytes (two tagged words) per
// instruction, so batch 1 with 1024 hidden units needs a single load instruction per source.
// Device-scope buffer loads (sc1): they see other workgroups' write-through stores and the
// compiler can keep many of them in flight.  `base` is the byte offset, inside the buffer
// resource, of word 0 of this wave's quarter for column 0 of the block; row_bytes separates
// consecutive sequences.
// ALL: every one of the NI instructions is issued and checked whatever ncol is (instructions past
// the end re-read the last pair), so that the compiler sees the same loads on every path and can
// tell what is still in flight; used where a request stays in flight across other work.
template <int QW, int NI = (16 * QW + 127) / 128, bool ALL = false>   // covers up to 128 * NI words
struct LLFetch {
    static constexpr int STRIDE = QW + 4;                  // padded staging row (dwords)
    u32x4 v[NI];
    // request the words (no wait)
    __device__ inline void issue(__amdgpu_buffer_rsrc_t rsrc, uint32_t base, uint32_t row_bytes, int ncol, int lane) {
        const int total = ncol * QW;                        // tagged words wanted by this wave
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int f = i * 128 + 2 * lane;               // first of this lane's two words
            if (ALL || i * 128 < total) {                   // uniform
                const int c = f / QW, wd = f % QW;
                // lanes past the end re-read the last pair (in bounds, result unused)
                const uint32_t off = (f < total) ? base + (uint32_t)c * row_bytes + (uint32_t)wd * 8u
                                                 : base + (uint32_t)(ncol - 1) * row_bytes + (uint32_t)(QW - 2) * 8u;
                v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 16 /* sc1 */);
            }
        }
    }
    // check the tags of what arrived and leave the payloads in the staging area; returns whether
    // every tag equals `epoch`
    __device__ inline bool land(int ncol, int lane, uint32_t epoch, uint32_t* stage) const {
        const int total = ncol * QW;
        bool ok = true;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int f = i * 128 + 2 * lane;
            if (ALL) {
                ok = ok && v[i][1] == epoch && v[i][3] == epoch;
                if (f < total) *reinterpret_cast<uint2*>(stage + (f / QW) * STRIDE + f % QW) = make_uint2(v[i][0], v[i][2]);
            } else if (i * 128 < total && f < total) {
                ok = ok && v[i][1] == epoch && v[i][3] == epoch;
                *reinterpret_cast<uint2*>(stage + (f / QW) * STRIDE + f % QW) = make_uint2(v[i][0], v[i][2]);
            }
        }
        return __all(ok);
    }
};

// A source too large to be fetched again and again (16 sequences x 64 or 128 words per wave) is
// requested outright in segments: one load instruction covers one cache line (16 words, the units of
// two to four producer workgroups) of 8 sequences, each is checked on its own, and only the
// segments whose producers were late are requested again.  A step then costs one round trip when
// everybody is on time, and a late producer costs its own segment only.  Needs QW % 16 == 0.
template <class TR, int KB>
__device__ inline void ll_wait_segments(uint32_t base, __amdgpu_buffer_rsrc_t rsrc, uint32_t row_bytes, int ncol,
                                        int lane, uint32_t* stage, uint32_t epoch, unsigned* status,
                                        unsigned spin_limit, bool& aborted) {
    constexpr int QW = KB * TR::WORDS_PER_KW;
    static_assert(QW % 16 == 0, "a sequence's quarter must be whole cache lines");
    constexpr int LB = QW / 16;                         // cache lines per sequence and K quarter
    constexpr int NI = 2 * LB;                          // instructions: two halves of 8 sequences each
    constexpr int STRIDE = QW + 4;
    const int sub = lane >> 3, pair = lane & 7;         // sequence inside the half, pair of words inside the line
    uint32_t off[2];
    uint32_t* dst[2];
    bool mine[2];
#pragma unroll
    for (int hs = 0; hs < 2; ++hs) {
        const int n = hs * 8 + sub;
        mine[hs] = n < ncol;
        off[hs] = base + (uint32_t)min(n, ncol - 1) * row_bytes + (uint32_t)pair * 16u;   // lanes past the end re-read the last sequence
        dst[hs] = stage + min(n, ncol - 1) * STRIDE + 2 * pair;
    }
    const int nhalf = ncol > 8 ? 2 : 1;
    u32x4 v[NI];
    unsigned pending = 0;
#pragma unroll
    for (int i = 0; i < NI; ++i)
        if (i / LB < nhalf) {                           // uniform
            v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off[i / LB] + (uint32_t)(i % LB) * 128u, 0, 16 /* sc1 */);
            pending |= 1u << i;
        }
    unsigned spins = 0;
    for (;;) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
            if (pending & (1u << i)) {                  // uniform
                const bool ok = !mine[i / LB] || (v[i][1] == epoch && v[i][3] == epoch);
                if (__all(ok)) {
                    if (mine[i / LB]) *reinterpret_cast<uint2*>(dst[i / LB] + (i % LB) * 16) = make_uint2(v[i][0], v[i][2]);
                    pending &= ~(1u << i);
                }
            }
        if (pending == 0u || aborted) break;
        if ((++spins & 63u) == 0u || spins == 8u) {
            const unsigned st = ld_dev_u32(status);
            if (st != 0u || spins >= spin_limit) {
                st_dev_u32(status, 1u);
                aborted = true;
                break;
            }
        }
#pragma unroll
        for (int i = 0; i < NI; ++i)
            if (pending & (1u << i))
                v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off[i / LB] + (uint32_t)(i % LB) * 128u, 0, 16 /* sc1 */);
    }
}

// Wait until the tagged words at `base` are complete and leave their payloads in the staging area.
// When the source needs more than one load instruction, waiting is done on a single probe
// instruction whose lanes sample the first word of every producer tile (4 hidden units written
// by one wave of one workgroup) over the sequences of the block; the full fetch follows and is
// repeated until every tag matches.
// MODE is a compile-time choice of the launch.  1: a source of two to four load instructions is fetched
// outright first.  2: a larger source is fetched outright in segments, see ll_wait_segments.  3: the
// source is known to fit one load instruction (the generic path carries a uniform branch per possible
// instruction, up to 16 of them, on the way in and on the way out of every fetch).
template <class TR, int KB, int MODE = 0>
__device__ inline void ll_wait(uint32_t base, __amdgpu_buffer_rsrc_t rsrc, uint32_t row_bytes, int ncol, int lane,
                               uint32_t probe_rel, uint32_t* stage, uint32_t epoch, unsigned* status,
                               unsigned spin_limit, bool& aborted) {
    constexpr int QW = KB * TR::WORDS_PER_KW;           // tagged words per sequence in one K quarter
    constexpr bool OUTRIGHT = MODE == 1;
    // load instructions the source can take: mode 1 promises at most four (each possible instruction is a
    // uniform branch on the way in and on the way out of a fetch)
    constexpr int NI_ALL = (16 * QW + 127) / 128;
    constexpr int NI = (OUTRIGHT && NI_ALL > 4) ? 4 : NI_ALL;
    if constexpr (MODE == 2) {
        ll_wait_segments<TR, KB>(base, rsrc, row_bytes, ncol, lane, stage, epoch, status, spin_limit, aborted);
        return;
    }
    unsigned spins = 0;
    // Called after 8 unsuccessful probes or fetches (no wait of a healthy launch in its steady state
    // lasts that long) and then every 256 probes or 64 fetches: the poll budget and the status word
    // (another workgroup may have given up) are only read here, off the path of a wait that succeeds.
    auto give_up = [&]() {
        const unsigned st = ld_dev_u32(status);
        if (st != 0u || spins >= spin_limit) {
            st_dev_u32(status, 1u);
            aborted = true;
        }
    };
    if constexpr (MODE == 3) {
        // the whole source is one load instruction: no code for the others
        for (;;) {
            LLFetch<QW, 1> f;
            f.issue(rsrc, base, row_bytes, ncol, lane);
            const bool ok = f.land(ncol, lane, epoch, stage);
            if (ok || aborted) break;
            if ((++spins & 63u) == 0u || spins == 8u) give_up();
        }
        return;
    }
    if (ncol * QW > 128) {
        // A source of two to four load instructions is first fetched outright: the waves of a layer are
        // aligned by the second barrier of the step, and a request issued right after one's own stores
        // comes back about when everybody's have landed, so it usually succeeds and the step pays one
        // round trip instead of two (2-layer GRU, 512 units, batch 8: 0.223 -> 0.190 ms; 4 layers of 1024
        // units at batch 2: 0.323 -> 0.265).  Any retry waits on the probe word.
        if constexpr (OUTRIGHT) {
            LLFetch<QW, NI> f;
            f.issue(rsrc, base, row_bytes, ncol, lane);
            if (f.land(ncol, lane, epoch, stage)) return;
        }
        while (!aborted) {
            const uint2 a = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(rsrc, base + probe_rel, 0, 16));
            if (__all(a.y == epoch)) break;
            if ((++spins & 255u) == 0u || spins == 8u) give_up();
        }
    }
    for (;;) {
        LLFetch<QW, NI> f;
        f.issue(rsrc, base, row_bytes, ncol, lane);
        const bool ok = f.land(ncol, lane, epoch, stage);
        if (ok || aborted) break;
        if ((++spins & 63u) == 0u || spins == 8u) give_up();
    }
}

// acc[rt] += W[rt][:] x (payloads in the staging area of this wave).  The B fragments are read from
// LDS a group ahead of the MFMAs that use them, so that the LDS latency is paid once per group, not
// once per K block.
template <class TR, int RT, int KB>
__device__ inline void ll_consume(const typename TR::frag (&wreg)[RT][KB], const uint32_t* stage, int ncol, int lane,
                                  f32x4 (&acc)[RT]) {
    constexpr int QW = KB * TR::WORDS_PER_KW;
    constexpr int STRIDE = QW + 4;
    constexpr int G = KB % 4 == 0 ? 4 : KB % 3 == 0 ? 3 : KB % 2 == 0 ? 2 : 1;   // fragments per group (a divisor of KB)
    // B operand fragments from the staging area: lane (n, q) reads sequence min(n, ncol-1)
    const uint32_t* mine = stage + min(lane & 15, ncol - 1) * STRIDE + TR::word_of(TR::koff(lane));
    typename TR::frag f[2][G];
#pragma unroll
    for (int i = 0; i < G; ++i) f[0][i] = TR::frag_from_lds(mine + i * TR::WORDS_PER_KW);
#pragma unroll
    for (int g = 0; g < KB / G; ++g) {
        if (g + 1 < KB / G) {
#pragma unroll
            for (int i = 0; i < G; ++i) f[(g + 1) & 1][i] = TR::frag_from_lds(mine + ((g + 1) * G + i) * TR::WORDS_PER_KW);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < G; ++i)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) acc[rt] = TR::mfma(wreg[rt][g * G + i], f[g & 1][i], acc[rt]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Waves 0..3 ("h waves") carry the recurrence: they fetch h_{t-1}, multiply, exchange partial sums,
// finish the gates and publish.  In a launch with fused layers the workgroup has four more waves
// ("x waves") that hold the W_ih slice and do nothing but the input product of the NEXT step: they
// request x_{t+1} (the state of the layer below) before the two barriers of step t, and multiply it
// right after them, i.e. while the h waves wait for h_t to come round.  The input product is then off
// the recurrent critical path, and neither wave type holds two sets of weights (with both sets in
// one wave the compiler parks one in the accumulator registers and copies it back before every MFMA).
// XW: 0 = no x waves; otherwise x waves, XW = twice the ratio of input width to H of the launch's first
// layer: 2 = as wide as the layer (also when that layer reads a projection), 1 = half as wide, 4 = twice as wide
// (a bidirectional layer above the first, which reads [forward, backward] of the layer below).
// XWO = XW + 8 * (mode of the h waves' state fetch, see ll_wait).
template <class TR, int CELL, int RT, int KB, int XWO, bool EXT>
__global__ __launch_bounds__((XWO & 7) ? 512 : 256) void wavefront_ll_kernel(WavefrontArgs p) {
    constexpr int XW = XWO & 7;
    constexpr int WAIT_MODE = (XWO >> 3) & 3;        // how the h waves fetch the state, see ll_wait
    constexpr bool FUSED = XW > 0;
    typedef typename TR::elem elem;
    typedef typename TR::frag frag;
    constexpr int KW = TR::KW;
    constexpr int NOWN = (RT + 3) / 4;               // tiles finished by one wave
    constexpr int QW = KB * TR::WORDS_PER_KW;        // tagged words per sequence and K quarter
    constexpr int STAGE_DW = 16 * (QW + 4);          // staging dwords per wave: 16 sequence rows
    constexpr int RED = 4 * RT * 64;                 // f32x4 entries of one set of partial sums
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    // partial sums of the h waves [4][RT][64 lanes]; of the x waves [2 (step parity)][4][RT][64];
    // then the per-wave staging areas
    f32x4* red = reinterpret_cast<f32x4*>(smem_raw);
    f32x4* xred = red + RED;
    uint32_t* stage = reinterpret_cast<uint32_t*>(smem_raw + (size_t)(FUSED ? 3 : 1) * RED * sizeof(f32x4)) +
                      (threadIdx.x >> 6) * STAGE_DW;

    // every step of this kernel is on a dependency chain: when a projection kernel shares the CU,
    // these waves go first
    __builtin_amdgcn_s_setprio(3);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = (tid >> 6) & 3;                    // K quarter of this wave
    const bool xwave = FUSED && (tid >> 8) != 0;
    const int v = xcd_contiguous_id();
    const int wpg = p.nrb * p.ncb;
    const int g = v / wpg;
    if (g >= p.LP * p.D) return;
    const int r = v - g * wpg;
    const int cb = r / p.nrb, rb = r - cb * p.nrb;
    const int ll = g / p.D, d = g - ll * p.D;
    const int l = p.l0 + ll;
    const bool fused = FUSED && ll > 0;
    // the first layer of the launch multiplies its input itself (from a plain [T, B, H] tensor) when the
    // host hands one over; otherwise it adds the projection gx
    const bool plain_x = FUSED && ll == 0 && p.xin != nullptr;
    const bool write_out = (ll == p.LP - 1);         // only the last layer of a launch is read later
    const int H = p.H, B = p.B, T = p.T;
    const int kq = H / 4;
    const uint32_t epoch = p.epoch;

    const int row_words = TR::row_words(H);
    const size_t seq_words = (size_t)(T + 1) * B * row_words;
    uint64_t* lseq = p.lseq + (size_t)g * seq_words;
    // one buffer resource over the state sequences of this group and (when fused) of the layer
    // below it, which lies directly before it (D == 1); offsets are bytes inside that window.
    // (The pieces are wave-uniform; saying so keeps the descriptor in scalar registers, otherwise
    // every load is wrapped in a loop over the distinct descriptors of the wave.)
    const uint64_t* window = fused ? lseq - seq_words : lseq;
    const uint32_t own_off = fused ? (uint32_t)(seq_words * 8) : 0u;
    const uint64_t wbits = reinterpret_cast<uint64_t>(window);
    const uint32_t wlo = __builtin_amdgcn_readfirstlane((uint32_t)wbits);
    const uint32_t whi = __builtin_amdgcn_readfirstlane((uint32_t)(wbits >> 32));
    const int wbytes = __builtin_amdgcn_readfirstlane((int)((fused ? 2 : 1) * seq_words * 8));
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<void*>(((uint64_t)whi << 32) | wlo), 0, wbytes, 0x00020000);
    const uint32_t row_bytes = (uint32_t)row_words * 8u;
    const int ncol = min(16, B - cb * 16);
    // byte offset (inside a slot) of word 0 of this wave's K quarter for column 0 of the block
    const uint32_t quarter_off = ((uint32_t)(cb * 16) * row_words + TR::word_of(w * kq)) * 8u;
    uint32_t probe_rel;  // probe word of this lane relative to quarter_off
    {
        const int ntile = kq / 4;                               // producer tiles in this K quarter
        const int ti = lane % ntile, ci = (lane / ntile) % ncol;
        probe_rel = (uint32_t)ci * row_bytes + (uint32_t)TR::word_of(ti * 4) * 8u;
    }
    const uint32_t slot_bytes = (uint32_t)B * row_bytes;
    bool aborted = false;

    if (xwave) {
        // ---- input product of the next step (fused layers); the x waves of the first layer of the
        // launch only keep the barriers company ----
        if (fused) {
            frag wx[RT][KB];
            const elem* wih = static_cast<const elem*>(p.wih[g]);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const size_t row = (size_t)(rb * RT + rt) * 16 + (lane & 15);
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) wx[rt][kb] = TR::load(wih + row * H + w * kq + kb * KW + TR::koff(lane));
            }
            // x_t = state of the layer below after its step t = slot t + 1 of its sequence (t == s when
            // D == 1).  A quarter that fits a few load instructions is requested a step early and stays
            // in flight across the barriers; a larger one is fetched after them.
            constexpr int XNI = WAIT_MODE == 3 ? 1 : ((16 * QW + 127) / 128 < 4 ? (16 * QW + 127) / 128 : 4);   // mode 3: one instruction covers it
            const bool early = ncol * QW <= 128 * XNI;
            LLFetch<QW, XNI, true> xq;
            if (early) xq.issue(rsrc, slot_bytes + quarter_off, row_bytes, ncol, lane);
            for (int sx = 0; sx < T; ++sx) {            // produces the input part of step sx
                if (sx > 0) {                           // steps sx-1 of the h waves: their two barriers
                    __syncthreads();
                    __syncthreads();
                }
                const uint32_t xbase = (uint32_t)(sx + 1) * slot_bytes + quarter_off;
                if (!(early && xq.land(ncol, lane, epoch, stage)))
                    ll_wait<TR, KB, WAIT_MODE == 3 ? 3 : 0>(xbase, rsrc, row_bytes, ncol, lane, probe_rel, stage, epoch, p.status, p.spin_limit, aborted);
                if (early) xq.issue(rsrc, (uint32_t)min(sx + 2, T) * slot_bytes + quarter_off, row_bytes, ncol, lane);
                __builtin_amdgcn_sched_barrier(0);
                f32x4 acc[RT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                ll_consume<TR, RT, KB>(wx, stage, ncol, lane, acc);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) xred[(((sx & 1) * 4 + w) * RT + rt) * 64 + lane] = acc[rt];
            }
            __syncthreads();
            __syncthreads();
        } else if (plain_x) {
            // first layer of the launch: x_t is a finished tensor without tags, read straight into MFMA
            // B fragments (lane (n, q) holds 8 consecutive inputs of sequence n), a step ahead
            constexpr int KBX = (XW > 0 ? XW * KB / 2 : 1) > 0 ? (XW > 0 ? XW * KB / 2 : 1) : 1;   // K blocks of this wave's quarter of the input
            const int IW = (XW > 0 ? XW : 2) * H / 2;     // input width
            frag wx[RT][KBX];
            // W_ih of all directions is one matrix [D * 4H, IW]; direction d owns rows d * 4H ...
            const elem* wih = static_cast<const elem*>(p.wih[g]) + (size_t)d * 4 * H * IW;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const size_t row = (size_t)(rb * RT + rt) * 16 + (lane & 15);
#pragma unroll
                for (int kb = 0; kb < KBX; ++kb)
                    wx[rt][kb] = TR::load(wih + row * IW + w * (IW / 4) + kb * KW + TR::koff(lane));
            }
            const elem* xrow = static_cast<const elem*>(p.xin) +
                               (size_t)(cb * 16 + min(lane & 15, ncol - 1)) * IW + w * (IW / 4) + TR::koff(lane);
            // x_t is requested NBUF steps ahead, between the two barriers of a step: the h waves are in
            // their gate phase then and have no polls in flight that the request could hold up.  Two
            // register sets used in turn where they fit beside the weights (x may come from HBM).
            constexpr int NBUF = (RT * KBX + 2 * KBX <= 48 && KB <= 4) ? 2 : 1;
            frag xb[NBUF][KBX];
            auto request = [&](int s, frag (&dst)[KBX]) {   // the step of this direction's order that is s-th
                const int sc = min(s, T - 1);
                const elem* src = xrow + (size_t)(d ? T - 1 - sc : sc) * B * IW;
#pragma unroll
                for (int kb = 0; kb < KBX; ++kb) dst[kb] = *reinterpret_cast<const frag*>(src + kb * KW);
            };
            auto produce = [&](int sx, frag (&cur)[KBX]) {
                f32x4 acc[RT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int kb = 0; kb < KBX; ++kb)
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) acc[rt] = TR::mfma(wx[rt][kb], cur[kb], acc[rt]);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) xred[(((sx & 1) * 4 + w) * RT + rt) * 64 + lane] = acc[rt];
                __syncthreads();            // first barrier of step sx: the partial sums are in LDS
                request(sx + NBUF, cur);
                __syncthreads();            // second barrier of step sx
            };
#pragma unroll
            for (int b = 0; b < NBUF; ++b) request(b, xb[b]);
            for (int sx = 0; sx < T; sx += NBUF) {
                produce(sx, xb[0]);
                if (NBUF > 1 && sx + 1 < T) produce(sx + 1, xb[NBUF - 1]);
            }
        } else {
            for (int s = 0; s < T; ++s) {
                __syncthreads();
                __syncthreads();
            }
        }
        return;
    }

    // ---- h waves ----
    frag wh[RT][KB];
    {
        const elem* whh = static_cast<const elem*>(p.whh[g]);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const size_t row = (size_t)(rb * RT + rt) * 16 + (lane & 15);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) wh[rt][kb] = TR::load(whh + row * H + w * kq + kb * KW + TR::koff(lane));
        }
    }

    float c_reg[NOWN], h_reg[NOWN];
    f32x4 bias_reg[NOWN];
    CellExt ext_reg[EXT ? NOWN : 1];                 // peephole weights and clipping bound of the unit
    int unit_reg[NOWN];
    const int col = cb * 16 + (lane & 15);
    const bool valid = col < B;
    const int colc = valid ? col : B - 1;            // clamped: loads stay in bounds
    const int len = valid ? (p.lengths ? min(max(p.lengths[col], 0), T) : T) : 0;
    const size_t state_row = (size_t)(l * p.D + d) * B;
#pragma unroll
    for (int o = 0; o < NOWN; ++o) {
        const int rt = w + 4 * o;
        const int unit = (rb * RT + rt) * 4 + (lane >> 4);
        unit_reg[o] = unit;
        c_reg[o] = 0.0f;
        h_reg[o] = 0.0f;
        bias_reg[o] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (EXT) ext_reg[o] = load_cell_ext(CELL == CELL_LSTM ? p.peep[g] : nullptr, H, min(unit, H - 1), p.clip);
        if (rt < RT && valid) {
            const size_t si = (state_row + col) * H + unit;
            if (p.h0) h_reg[o] = p.h0[si];
            if (p.c0) c_reg[o] = p.c0[si];
            bias_reg[o] = *reinterpret_cast<const f32x4*>(p.bias[g] + (size_t)unit * SLOTS);
        }
    }
    elem* out = static_cast<elem*>(p.out[ll]);
    const int out_ld = p.D * H;

    // Projection of a step for the pairs this lane finishes.  It is requested one step ahead, right
    // after the last poll of a step: loads return in order, so a request to HBM issued just before a
    // poll would hold back the poll's result for its whole latency; issued here it has the exchange,
    // the gates and the publication to travel.  Never predicated (indices are clamped), so that the
    // compiler can count the loads in flight.
    f32x4 gx_reg[NOWN];
    auto fetch_gx = [&](int s) {
        const int sc = min(s, T - 1);
        const int tt = d ? (T - 1 - sc) : sc;
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int unit = min(unit_reg[o], H - 1);
            gx_reg[o] = *reinterpret_cast<const f32x4*>(p.gx + ((((size_t)tt * B + colc) * p.D + d) * H + unit) * SLOTS);
        }
    };
    const bool has_x = fused || plain_x;   // the input part comes from the x waves
    if (!has_x) fetch_gx(0);

    for (int s = 0; s < T; ++s) {
        const int t = d ? (T - 1 - s) : s;
        f32x4 acc[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

        ll_wait<TR, KB, WAIT_MODE>(own_off + (uint32_t)s * slot_bytes + quarter_off, rsrc, row_bytes, ncol, lane,
                                  probe_rel, stage, epoch, p.status, p.spin_limit, aborted);
        ll_consume<TR, RT, KB>(wh, stage, ncol, lane, acc);

#pragma unroll
        for (int rt = 0; rt < RT; ++rt) red[(w * RT + rt) * 64 + lane] = acc[rt];
        f32x4 gx_now[NOWN];
#pragma unroll
        for (int o = 0; o < NOWN; ++o) gx_now[o] = gx_reg[o];
        if (!has_x) fetch_gx(s + 1);
        __syncthreads();

        // all partial sums this wave needs are read before the first is used (one LDS round trip)
        f32x4 part[NOWN][FUSED ? 8 : 4];
#pragma unroll
        for (int o = 0; o < NOWN; ++o)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                part[o][q] = red[(q * RT + min(w + 4 * o, RT - 1)) * 64 + lane];
                if constexpr (FUSED) part[o][4 + q] = xred[(((s & 1) * 4 + q) * RT + min(w + 4 * o, RT - 1)) * 64 + lane];
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int o = 0; o < NOWN; ++o) {
            const int rt = w + 4 * o;
            if (rt < RT) {  // uniform per wave
                f32x4 a = (part[o][0] + part[o][1]) + (part[o][2] + part[o][3]);
                if constexpr (FUSED) {
                    if (has_x) a += (part[o][4] + part[o][5]) + (part[o][6] + part[o][7]);
                }
                if (!has_x) a += gx_now[o];
                a += bias_reg[o];
                const bool active = valid && t < len;
                float c_new = c_reg[o];
                const float pre[SLOTS] = {a[0], a[1], a[2], a[3]};
                float hn;
                if constexpr (EXT) hn = cell_update_ext<CELL>(pre, h_reg[o], c_new, ext_reg[o]);
                else hn = cell_update<CELL>(pre, h_reg[o], c_new);
                if (active) {
                    float kept;
                    (void)TR::store_val(hn, kept);
                    c_reg[o] = c_new;
                    h_reg[o] = kept;
                }
                float unused;
                const elem state_v = TR::store_val(h_reg[o], unused);  // held value when inactive
                const elem out_v = active ? state_v : TR::zero();
                const int unit0 = unit_reg[o] - (lane >> 4);
                TR::ll_publish(state_v, out_v, valid, write_out, lane, epoch,
                               lseq + ((size_t)(s + 1) * B + colc) * row_words + TR::word_of(unit0),
                               out + ((size_t)t * B + colc) * out_ld + (size_t)d * H + unit0);
            }
        }
        if (p.ticks && tid == 0 && rb == 0 && cb == 0) p.ticks[(size_t)g * T + s] = wall_clock64();
        // Second barrier of the step: no wave starts polling for the next state before the waves that
        // finish tiles have issued their stores.  (Waves without a tile of their own otherwise poll
        // from here on, fail, and every failed poll costs a full round trip more than waiting would.)
        __syncthreads();
    }

#pragma unroll
    for (int o = 0; o < NOWN; ++o) {
        if ((w + 4 * o) < RT && valid) {
            const size_t si = (state_row + col) * H + unit_reg[o];
            if (p.hT) p.hT[si] = h_reg[o];
            if (p.cT && CELL == CELL_LSTM) p.cT[si] = c_reg[o];
        }
    }
}

// slot 0 of every state sequence of the launch = h0 (rounded to the storage type), tagged
template <int DT>
__global__ void wavefront_ll_init_kernel(const float* h0, int l0, int LP, int D, int T, int B, int H,
                                         uint64_t* lseq, uint32_t epoch) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // one tagged word each
    const int row_words = (DT == DT_BF16) ? H / 2 : H;
    const size_t per = (size_t)B * row_words;
    const size_t n = (size_t)LP * D * per;
    if (i >= n) return;
    const size_t g = i / per, rem = i - g * per;
    const size_t b = rem / row_words, wd = rem - b * row_words;
    const float* src = h0 ? h0 + (((size_t)l0 * D + g) * B + b) * H : nullptr;
    uint32_t payload;
    if (DT == DT_BF16) {
        const float a = src ? src[2 * wd] : 0.0f, c = src ? src[2 * wd + 1] : 0.0f;
        payload = (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(c) << 16);
    } else {
        payload = __float_as_uint(src ? src[wd] : 0.0f);
    }
    lseq[g * (size_t)(T + 1) * per + rem] = ((uint64_t)epoch << 32) | payload;
}

template <class TR, int CELL, int RT, int KB, int XWO>
hipError_t launch_ll_variant(const WavefrontArgs& a, hipStream_t stream) {
    constexpr int XW = XWO & 7;
    const int grid = a.LP * a.D * a.nrb * a.ncb;
    constexpr int QW = KB * TR::WORDS_PER_KW;
    const size_t smem = (size_t)(XW ? 3 : 1) * 4 * RT * 64 * sizeof(f32x4) +
                        (size_t)(XW ? 8 : 4) * 16 * (QW + 4) * sizeof(uint32_t);
    auto kern = wavefront_ll_kernel<TR, CELL, RT, KB, XWO, RNN_CELL_EXT != 0>;
    static bool configured = false;
    if (!configured && smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<dim3(grid), dim3(XW ? 512 : 256), smem, stream>>>(a);
    return hipGetLastError();
}

template <class TR, int RT, int KB, int XWO>
hipError_t launch_ll_cell2(const WavefrontArgs& a, hipStream_t stream) {
    if (a.cell == CELL_LSTM) return launch_ll_variant<TR, CELL_LSTM, RT, KB, XWO>(a, stream);
    return launch_ll_variant<TR, CELL_GRU, RT, KB, XWO>(a, stream);
}

template <class TR, int RT, int KB, int XW>
hipError_t launch_ll_cell(const WavefrontArgs& a, hipStream_t stream) {
    // the state of a step: min(16, B) sequences x one K quarter; two to four load instructions (128 words
    // each) are fetched outright
    constexpr int QW = KB * TR::WORDS_PER_KW;
    const int total = (a.B < 16 ? a.B : 16) * QW;
    // One load instruction per wave and source: the lean fetch loop (mode 3), for layers of at least 512 units
    // and for launches of a single layer.  Measured against the generic loop: 4 layers x 1024 units at batch 1
    // 0.267 -> 0.233 ms, 8 such layers 1.96 -> 1.70, 2 x 512 units 0.192 -> 0.181, one layer of 128 units
    // 0.048 -> 0.047; but stacks of 4 to 12 narrow layers (64 to 256 units) in one launch lose 6-13 % with it:
    // there the waves of every upper layer spin on the layer below, and the generic loop's extra
    // instructions pace those polls, whose traffic delays the stores everybody waits for.
    if (total <= 128 && (a.H >= 512 || a.LP * a.D == 1)) return launch_ll_cell2<TR, RT, KB, XW + 24>(a, stream);
    if constexpr (QW <= 256) {
        if (total > 128 && total <= 512) return launch_ll_cell2<TR, RT, KB, XW + 8>(a, stream);
    }
    // More than four load instructions: outright in segments, where that was measured to pay: quarters of
    // 64 words (512 units in bf16), 9 to 16 sequences (2 layers x 2 directions x 512 units, batch 64: 1.35 ->
    // 1.22 ms; batch 9 and 12 likewise 3 %).  Quarters of 128 words lose with it (4 layers x 1024 units at batch
    // 6: 0.36 -> 0.64 ms, batch 16: 0.58 -> 0.68), and so do sources of up to four instructions (batch 4:
    // 0.35 -> 0.46), which keep the probe word.
    if constexpr (QW == 64) {
        if (total > 512) return launch_ll_cell2<TR, RT, KB, XW + 16>(a, stream);
    }
    return launch_ll_cell2<TR, RT, KB, XW>(a, stream);
}

template <class TR, int RT, int KB>
hipError_t launch_ll_cell_fused(const WavefrontArgs& a, hipStream_t stream) {
    // workgroups with x waves: fused layers, or a first layer that multiplies its plain input itself
    // (a.xin_width2 = twice that input's width over H)
    if (a.xin != nullptr && a.xin_width2 == 4) {
        if constexpr (RT * KB * 2 <= 32) {       // the x waves hold RT * 2KB weight fragments
            if (a.LP != 1) return hipErrorInvalidValue;
            return launch_ll_cell<TR, RT, KB, 4>(a, stream);
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (a.xin != nullptr && a.xin_width2 == 1) {
        if constexpr (KB % 2 == 0) {
            return launch_ll_cell<TR, RT, KB, 1>(a, stream);
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (a.xin != nullptr && a.xin_width2 != 2) return hipErrorInvalidValue;
    if (a.LP > 1 || a.xin != nullptr) return launch_ll_cell<TR, RT, KB, 2>(a, stream);
    return launch_ll_cell<TR, RT, KB, 0>(a, stream);
}

// (dtype traits, RT, KB) combinations that are compiled; KB = H / (4 * KW), CT is always 1.  bf16: layers of
// 128 * KB units; fp32: 16 * KB units.  The taller tiles stop where the weight fragments of a wave (RT * KB,
// four registers each in bf16) no longer fit beside its other registers.
#define RNN_LL_VARIANTS_0(X)                                                     \
    X(LLBf16, 1, 1) X(LLBf16, 1, 2) X(LLBf16, 1, 4) X(LLBf16, 1, 8)               \
    X(LLBf16, 2, 1) X(LLBf16, 2, 2) X(LLBf16, 2, 4) X(LLBf16, 2, 8)               \
    X(LLBf16, 4, 1) X(LLBf16, 4, 2) X(LLBf16, 4, 4) X(LLBf16, 4, 8)
#define RNN_LL_VARIANTS_1(X)                                                     \
    X(LLF32, 1, 2) X(LLF32, 1, 4) X(LLF32, 1, 8)                                  \
    X(LLF32, 2, 2) X(LLF32, 2, 4) X(LLF32, 2, 8)                                  \
    X(LLF32, 4, 2) X(LLF32, 4, 4) X(LLF32, 4, 8)                                  \
    X(LLF32, 1, 16) X(LLF32, 2, 16) X(LLF32, 4, 16) X(LLF32, 2, 32) X(LLF32, 4, 32)
#define RNN_LL_VARIANTS_2(X)                                                     \
    X(LLBf16, 1, 3) X(LLBf16, 2, 3) X(LLBf16, 4, 3)                               \
    X(LLBf16, 1, 5) X(LLBf16, 2, 5) X(LLBf16, 4, 5)                               \
    X(LLBf16, 1, 6) X(LLBf16, 2, 6) X(LLBf16, 4, 6)                               \
    X(LLBf16, 1, 10) X(LLBf16, 2, 10) X(LLBf16, 1, 12) X(LLBf16, 2, 12)           \
    X(LLBf16, 1, 16) X(LLBf16, 2, 16)
#define RNN_LL_VARIANTS(X) RNN_LL_VARIANTS_0(X) RNN_LL_VARIANTS_1(X) RNN_LL_VARIANTS_2(X)
#if RNN_LL_PART == 0
#define RNN_LL_VARIANTS_HERE(X) RNN_LL_VARIANTS_0(X)
#elif RNN_LL_PART == 1
#define RNN_LL_VARIANTS_HERE(X) RNN_LL_VARIANTS_1(X)
#else
#define RNN_LL_VARIANTS_HERE(X) RNN_LL_VARIANTS_2(X)
#endif

template <class TR> struct LLDtOf;
template <> struct LLDtOf<LLBf16> { static constexpr int value = DT_BF16; };
template <> struct LLDtOf<LLF32> { static constexpr int value = DT_F32; };

// the variants compiled in this translation unit
hipError_t launch_here(const WavefrontArgs& a, hipStream_t stream, int KB) {
#define X(TR, rt, kb)                                                 \
    if (LLDtOf<TR>::value == a.dtype && a.RT == rt && KB == kb)       \
        return launch_ll_cell_fused<TR, rt, kb>(a, stream);
    RNN_LL_VARIANTS_HERE(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace

// every translation unit exports its variants under a name of its own: part 0..2, plain or extended cell
#define RNN_LL_FN2(part, ext) launch_wavefront_ll_part##part##_ext##ext
#define RNN_LL_FN(part, ext) RNN_LL_FN2(part, ext)
hipError_t RNN_LL_FN(RNN_LL_PART, RNN_CELL_EXT)(const WavefrontArgs& a, hipStream_t stream, int KB) { return launch_here(a, stream, KB); }

#if RNN_LL_PART == 0 && RNN_CELL_EXT == 0
hipError_t launch_wavefront_ll_part1_ext0(const WavefrontArgs& a, hipStream_t stream, int KB);
hipError_t launch_wavefront_ll_part2_ext0(const WavefrontArgs& a, hipStream_t stream, int KB);
hipError_t launch_wavefront_ll_part0_ext1(const WavefrontArgs& a, hipStream_t stream, int KB);
hipError_t launch_wavefront_ll_part1_ext1(const WavefrontArgs& a, hipStream_t stream, int KB);
hipError_t launch_wavefront_ll_part2_ext1(const WavefrontArgs& a, hipStream_t stream, int KB);

bool wavefront_ll_variant_exists(int dtype, int RT, int H) {
    const int kw = dtype == DT_BF16 ? TraitsBf16::KW : TraitsF32::KW;
    if (H % (4 * kw) != 0) return false;
    const int KB = H / (4 * kw);
#define X(TR, rt, kb) \
    if (LLDtOf<TR>::value == dtype && RT == rt && KB == kb) return true;
    RNN_LL_VARIANTS(X)
#undef X
    return false;
}

hipError_t launch_wavefront_ll(const WavefrontArgs& a, hipStream_t stream) {
    const int kw = a.dtype == DT_BF16 ? TraitsBf16::KW : TraitsF32::KW;
    if (a.H % (4 * kw) != 0 || a.CT != 1) return hipErrorInvalidValue;
    const int KB = a.H / (4 * kw);
#define X(TR, rt, kb) \
    if (LLDtOf<TR>::value == a.dtype && a.RT == rt && KB == kb) \
        return a.ext ? launch_wavefront_ll_part0_ext1(a, stream, KB) : launch_wavefront_ll_part0_ext0(a, stream, KB);
    RNN_LL_VARIANTS_0(X)
#undef X
#define X(TR, rt, kb) \
    if (LLDtOf<TR>::value == a.dtype && a.RT == rt && KB == kb) \
        return a.ext ? launch_wavefront_ll_part1_ext1(a, stream, KB) : launch_wavefront_ll_part1_ext0(a, stream, KB);
    RNN_LL_VARIANTS_1(X)
#undef X
#define X(TR, rt, kb) \
    if (LLDtOf<TR>::value == a.dtype && a.RT == rt && KB == kb) \
        return a.ext ? launch_wavefront_ll_part2_ext1(a, stream, KB) : launch_wavefront_ll_part2_ext0(a, stream, KB);
    RNN_LL_VARIANTS_2(X)
#undef X
    return hipErrorInvalidValue;
}

hipError_t launch_wavefront_ll_init(int dtype, const float* h0, int l0, int LP, int D, int T, int B,
                                    int H, uint64_t* lseq, uint32_t epoch, hipStream_t stream) {
    const size_t n = (size_t)LP * D * B * (dtype == DT_BF16 ? H / 2 : H);
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (dtype == DT_BF16)
        wavefront_ll_init_kernel<DT_BF16><<<blocks, 256, 0, stream>>>(h0, l0, LP, D, T, B, H, lseq, epoch);
    else
        wavefront_ll_init_kernel<DT_F32><<<blocks, 256, 0, stream>>>(h0, l0, LP, D, T, B, H, lseq, epoch);
    return hipGetLastError();
}

size_t wavefront_ll_words(int dtype, int groups, int T, int B, int H) {
    return (size_t)groups * (size_t)(T + 1) * B * (dtype == DT_BF16 ? H / 2 : H);
}

#endif  // RNN_LL_PART == 0 && RNN_CELL_EXT == 0

}  // namespace rnn
