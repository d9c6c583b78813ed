// Pieces shared by the two persistent kernels (counter-synchronised and tag-in-data):
// device-scope access helpers and the per-dtype MFMA traits.
#pragma once

#include "common.h"
#include "kernels.h"

namespace rnn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Device-scope (cross-XCD coherent) accesses for data exchanged between workgroups in flight.
__device__ inline uint64_t ld_dev_u64(const void* p) {
    return __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline uint32_t ld_dev_u32(const void* p) {
    return __hip_atomic_load(reinterpret_cast<const uint32_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_dev_u64(void* p, uint64_t v) {
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_dev_u16(void* p, uint16_t v) {
    __hip_atomic_store(reinterpret_cast<uint16_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_dev_u32(void* p, uint32_t v) {
    __hip_atomic_store(reinterpret_cast<uint32_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// For lanes 0..15: the value `mine` of lanes n, n + 16, n + 32, n + 48 (v0..v3), without a trip through
// LDS: v_permlane16_swap exchanges rows 1 and 3 (of 16 lanes) of its first operand with rows 0 and 2 of
// its second, v_permlane32_swap the upper half of the first with the lower half of the second.  In the
// other lanes the outputs hold other rows' values and are not used.
__device__ inline void gather_rows(uint32_t mine, uint32_t& v0, uint32_t& v1, uint32_t& v2, uint32_t& v3) {
    const auto r = __builtin_amdgcn_permlane16_swap(mine, mine, false, false);
    const auto q0 = __builtin_amdgcn_permlane32_swap(r[0], r[0], false, false);
    const auto q1 = __builtin_amdgcn_permlane32_swap(r[1], r[1], false, false);
    v0 = r[0]; v1 = r[1]; v2 = q0[1]; v3 = q1[1];
}

struct TraitsBf16 {
    typedef bf16_t elem;
    typedef bf16x8 frag;
    static constexpr int KW = 32;  // K elements consumed by one MFMA
    // lane -> first K element of its fragment inside a KW block
    static __device__ inline int koff(int lane) { return 8 * (lane >> 4); }
    static __device__ inline frag load(const elem* p) { return *reinterpret_cast<const frag*>(p); }
    static __device__ inline frag load_dev(const elem* p) {
        union { uint64_t u[2]; frag f; } v;
        v.u[0] = ld_dev_u64(p);
        v.u[1] = ld_dev_u64(p + 4);
        return v.f;
    }
    static __device__ inline f32x4 mfma(frag a, frag b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    // c += a x b with the A operand read from the accumulation registers (on gfx950 a matrix
    // instruction may take A or B from either half of the register file).  Resident weights beyond the
    // 256 vector registers live there; written this way they are operands, not spilled values that must
    // be copied back before every use.  The compiler does not see inside: the caller keeps dependent
    // instructions apart and waits (wait_mfma_results) before anything else reads c.
    static __device__ inline void mfma_acc_a(const frag& a, const frag& b, f32x4& c) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "a"(a), "v"(b));
    }
    static constexpr bool HAS_ACC_A = true;
    typedef uint64_t piece;  // 4 consecutive units of one sequence
    static __device__ inline void store_piece_dev(elem* dst, piece v) { st_dev_u64(dst, v); }
    // Write the state value and the output value of the 4 units held by lanes n, n+16, n+32,
    // n+48 (same sequence n) as two 8-byte device-scope stores issued by lane n.
    // out_shared: the layer output is read by another workgroup during this launch (a fused layer
    // above); otherwise it is an ordinary cached store that L2 can merge into whole lines.
    static __device__ inline void publish(elem state, elem outv, bool valid, bool out_shared, int lane,
                                          elem* state_dst, elem* out_dst) {
        // out_dst == nullptr: the layer output is not wanted (the consumer reads the state sequence)
        uint32_t v0, v1, v2, v3;
        gather_rows((uint32_t)state | ((uint32_t)outv << 16), v0, v1, v2, v3);
        if (valid && lane < 16) {
            const uint64_t st = (uint64_t)(v0 & 0xFFFFu) | ((uint64_t)(v1 & 0xFFFFu) << 16) |
                                ((uint64_t)(v2 & 0xFFFFu) << 32) | ((uint64_t)(v3 & 0xFFFFu) << 48);
            const uint64_t ov = (uint64_t)(v0 >> 16) | ((uint64_t)(v1 >> 16) << 16) |
                                ((uint64_t)(v2 >> 16) << 32) | ((uint64_t)(v3 >> 16) << 48);
            st_dev_u64(state_dst, st);
            if (out_dst) {
                if (out_shared) st_dev_u64(out_dst, ov);
                else *reinterpret_cast<uint64_t*>(out_dst) = ov;
            }
        }
    }
    // The same without the cross-lane exchange: every lane stores its own unit (2 bytes); the
    // lanes of a wave still cover 8 contiguous bytes per sequence.
    static __device__ inline void publish_own(elem state, elem outv, bool valid, int lane, elem* state_dst,
                                              elem* out_dst) {
        if (valid) {
            st_dev_u16(state_dst + (lane >> 4), state);
            if (out_dst) out_dst[lane >> 4] = outv;
        }
    }
    static __device__ inline elem store_val(float h, float& kept) {
        const bf16_t b = f32_to_bf16(h);
        kept = bf16_to_f32(b);
        return b;
    }
    static __device__ inline elem zero() { return 0; }
};

struct TraitsF32 {
    typedef float elem;
    typedef float frag;
    static constexpr int KW = 4;
    static __device__ inline int koff(int lane) { return lane >> 4; }
    static __device__ inline frag load(const elem* p) { return *p; }
    static __device__ inline frag load_dev(const elem* p) { return __uint_as_float(ld_dev_u32(p)); }
    static __device__ inline f32x4 mfma(frag a, frag b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ inline void mfma_acc_a(const frag& a, const frag& b, f32x4& c) { c = mfma(a, b, c); }
    static constexpr bool HAS_ACC_A = false;
    struct __attribute__((aligned(16))) piece { uint64_t lo, hi; };  // 4 consecutive units of one sequence
    static __device__ inline void store_piece_dev(elem* dst, piece v) {
        st_dev_u64(dst, v.lo);
        st_dev_u64(dst + 2, v.hi);
    }
    // every lane stores its own unit; state_dst / out_dst point at unit 4*(tile row) of sequence n
    static __device__ inline void publish(elem state, elem outv, bool valid, bool out_shared, int lane,
                                          elem* state_dst, elem* out_dst) {
        if (valid) {
            st_dev_u32(state_dst + (lane >> 4), __float_as_uint(state));
            if (out_dst) {
                if (out_shared) st_dev_u32(out_dst + (lane >> 4), __float_as_uint(outv));
                else out_dst[lane >> 4] = outv;
            }
        }
    }
    static __device__ inline void publish_own(elem state, elem outv, bool valid, int lane, elem* state_dst,
                                              elem* out_dst) {
        publish(state, outv, valid, false, lane, state_dst, out_dst);
    }
    static __device__ inline elem store_val(float h, float& kept) { kept = h; return h; }
    static __device__ inline elem zero() { return 0.0f; }
};


// After a run of mfma_acc_a: the results may be read 24 wait states after the last of them was issued
// (more than the deepest matrix pipeline needs; the compiler, which inserts such waits for the
// instructions it knows, cannot see these).
__device__ inline void wait_mfma_results() { asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory"); }

// Wait until the `n` flag words at `row` carry `epoch` (n <= 64, one word per lane).  Returns
// false when the wait was abandoned (poll budget exhausted, or another workgroup gave up).
// The poll budget and the status word are read every 1024 polls, off the path of a wait that
// succeeds; with EARLY_LOOK also after 8 unsuccessful polls (for the waits of a layer for the layer
// below it, which are long at the start of a launch: a tiny budget set by the host then ends them).
template <bool EARLY_LOOK = false>
__device__ inline bool wait_flags(const uint64_t* row, int n, int lane, uint32_t epoch,
                                  unsigned* status, unsigned spin_limit, bool& aborted) {
    if (aborted) return false;
    unsigned spins = 0;
    const int i0 = min(lane, n - 1);
    for (;;) {
        const bool ok = (uint32_t)(ld_dev_u64(row + i0) >> 32) == epoch;
        if (__all(ok)) break;
        if ((++spins & 1023u) == 0u || (EARLY_LOOK && spins == 8u)) {
            const unsigned st = ld_dev_u32(status);
            if (st != 0u || spins >= spin_limit) {
                st_dev_u32(status, 1u);
                aborted = true;
                return false;
            }
        }
    }
    // later loads must not be hoisted above the poll
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return true;
}

// Row blocks a wave must wait for before it reads units [k0, k0 + kn) of an activation vector with
// cached loads: those that write any unit sharing a cache line with that range, `line_units`
// consecutive units to a line (a line the wave brings into its caches must be complete, or a later
// reader of the same line, e.g. the wave of the next K quarter, would find the incomplete copy).
// `rb_units` = units per row block; line_units is a multiple of it.
__device__ inline void flag_span(int k0, int kn, int H, int line_units, int rb_units, int& first, int& count) {
    const int lo = (k0 / line_units) * line_units;
    const int hi = min(H, ((k0 + kn + line_units - 1) / line_units) * line_units);
    first = lo / rb_units;
    count = (hi - lo + rb_units - 1) / rb_units;
}

// i modulo KB for 0 <= i < 2 * KB (KB is a compile-time constant, usually a power of two)
template <int KB>
__device__ inline int wrap_kb(int i) {
    if constexpr ((KB & (KB - 1)) == 0) return i & (KB - 1);
    else return i >= KB ? i - KB : i;
}

// Activation fragments of one part (h_{t-1} or x_t) for CT column tiles: buf[kb][ct].  src[ct]
// points at this lane's first K element of the sequence in column tile ct.  Register slot kb
// holds K block (kb + rot) mod KB: workgroups that read the same activations at the same
// moment start at different K blocks, which spreads them over the L2 channels.  All loads are
// issued back to back, so a part costs one memory round trip, not one per fragment.
template <class TR, int CT, int KB>
__device__ inline void load_part(const typename TR::elem* const (&src)[CT], int rot,
                                 typename TR::frag (&buf)[KB][CT]) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) buf[kb][ct] = TR::load(src[ct] + wrap_kb<KB>(kb + rot) * TR::KW);
}

// acc[rt][ct] += W[rt][:] (resident fragments) x the loaded activation fragments
template <class TR, int RT, int CT, int KB>
__device__ inline void mma_part(const typename TR::frag (&wreg)[RT][KB],
                                const typename TR::frag (&buf)[KB][CT], f32x4 (&acc)[RT][CT]) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc[rt][ct] = TR::mfma(wreg[rt][kb], buf[kb][ct], acc[rt][ct]);
}

// Element offset of (hidden unit k, sequence col) inside one slot of the blocked state sequence.
__device__ inline size_t hseq_off(int k, int col, int B) {
    return ((size_t)(k >> 4) * B + col) * 16 + (k & 15);
}

// Renumber workgroups so that consecutive ids share an XCD (the dispatcher hands workgroups to
// the 8 XCDs round-robin): the workgroups of one (layer, direction, column block) chain then sit
// on as few XCDs as possible.
__device__ inline int xcd_contiguous_id() {
    int v = blockIdx.x;
    if ((gridDim.x & 7) == 0) v = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    return v;
}

}  // namespace rnn
