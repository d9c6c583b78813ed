// Host side of the library: the C ABI of include/rnn.h, weight repacking, workspace and the
// choice of execution plan.  All arithmetic of the forward pass runs in the HIP kernels.
#include "../../include/rnn.h"
#include "../../include/rnn_schedule.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "common.h"
#include "kernels.h"

using namespace rnn;

namespace {

struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
};

struct Plan {
    int kind = RNN_PLAN_CELLWISE;   // resolved plan (never AUTO)
    int LP = 1, RT = 1, CT = 1, NCH = 1, nrb = 0, ncb = 0;
    // the first layer runs in a launch of its own (it needs a projection, the layers above it run side
    // by side in the inside-product kernel): launches are {0}, {1..LP}, {LP+1..2LP}, ...
    bool first_alone = false;
    // > 0: the batch is larger than one pass of this plan can hold; it runs in passes of `chunk` sequences
    // (sequences are independent) through copies in the workspace, the last pass with a plan of its own
    int chunk = 0;
    // Which layers share a launch, as the scheduler placed the cell graph (derive_launches): per layer the launch
    // that holds it, per launch its first layer and its number of layers.  Empty (the cellwise plan): one layer
    // per launch.
    std::vector<int> layer_launch, launch_layer0, launch_layers;
};

// The launches of one (steps, layers per launch, first layer alone) combination, kept with the model.
struct LaunchTable {
    int steps = 0, LP = 0;
    bool first_alone = false;
    std::vector<int> layer_launch, launch_layer0, launch_layers;
};

}  // namespace

// Workspace of rnn_forward_static: callers that cannot allocate device memory run on pieces of this array.
// Every GPU the library runs on holds its own copy until the process ends.  In host code the array's name
// is only a handle for hipGetSymbolAddress; the address the kernels get is looked up once per device
// (static_scratch_of) and kept.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)RNN_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
char* scratch_ptr[MAX_DEVICES];   // per device: address of that device's copy of `scratch`, NULL = not looked up yet

// Address of the current device's copy of the static array (device must be the current HIP device).
char* static_scratch_of(int device) {
    if (device < 0 || device >= MAX_DEVICES) return nullptr;
    if (!scratch_ptr[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        scratch_ptr[device] = (char*)p;
    }
    return scratch_ptr[device];
}
}  // namespace

// About three seconds of polling: far beyond any wait of a healthy launch, short enough that a launch
// whose workgroups are not all resident (which would otherwise never end) drains.
constexpr unsigned DEFAULT_SPIN_LIMIT = 1u << 22;

struct rnn_model {
    int cell, L, I, H, D, dtype;   // H: the width the kernels work with (Hu padded, see padded_width)
    int Hu = 0;                    // the caller's hidden size
    int device = 0;
    int num_cus = 0;
    size_t lds_limit = 0;   // LDS bytes one workgroup may use
    int requested_plan = RNN_PLAN_AUTO;
    size_t esize = 4;  // bytes per stored element

    // packed weights per layer: W_ih for all directions [D*4H, I_l]; per (l, d): W_hh [4H, H], bias [H, 4]
    std::vector<DevBuf> wih, whh, bias;
    size_t weight_bytes = 0;

    DevBuf status;          // one word, raised by a kernel whose wait gave up (rnn_model_check)
    bool gru_reset_before = false;
    float clip = 0.0f;          // clipping threshold of the gate arguments, 0 = none
    std::vector<DevBuf> peep;   // empty, or per (layer, direction) [3, H] fp32 peephole weights (LSTM)
    bool batch_first = false;   // x is [B, T, I] and y [B, T, D*H]
    bool validate = false;      // check `lengths` on the host before every forward
    // the cell variant that only the cellwise plan implements (two dependent recurrent products per cell)
    bool cellwise_only() const { return gru_reset_before; }
    // Everything a forward pass keeps in device memory besides the weights.
    struct Workspace {
        DevBuf gx, hseq, flags, h_f32, c_f32, h_st, gh, ticks;
        DevBuf rh_st, gh2;      // reset-before-product GRU (cellwise plan): r * h and the second product
        DevBuf x_tm, y_tm;          // batch-first callers: time-major copies of x and y
        DevBuf x_ck, y_ck, st_ck[4];   // a batch run in passes: the pass's x, y, h0, c0, hT, cT
        DevBuf y_pad, st_pad[4];       // a padded model: y, h0, c0, hT, cT at the padded width
        DevBuf xblk;            // the caller's x in the layout of a state sequence (first layer of width H only)
        DevBuf lseq;            // tagged state sequences of the tag-in-data kernel (grown on demand)
        std::vector<DevBuf> ybuf;  // L-1 inter-layer activations
    };
    Workspace ws;           // allocated on demand, owned by the model
    Workspace ws_static;    // rnn_forward_static: the same buffers as pieces of the device's static array, per call
    // rnn_forward_static: the device's static array and how much of it this call has handed out
    struct Arena { char* base = nullptr; size_t used = 0; bool on = false; hipStream_t stream = nullptr; } arena;
    char* scratch = nullptr;   // this device's copy of the static array (NULL: the lookup failed)
    uint32_t epoch = 0;     // tag of the most recent tag-in-data launch
    size_t workspace_bytes = 0;
    bool want_ticks = false;
    bool capturing = false;     // the current rnn_forward is being recorded into a stream capture
    unsigned spin_limit = DEFAULT_SPIN_LIMIT;   // polls before a wait inside a persistent kernel is abandoned

    // optional profiling: HIP events around the kernels of each class
    bool profiling = false;
    struct ProfSlot { hipEvent_t a, b; int kind; };
    std::vector<ProfSlot> prof;      // event pairs, created once and reused
    size_t prof_used = 0;

    int layer_input(int l) const { return l == 0 ? I : D * H; }

    // launch tables already derived for this model (the scheduler runs once per combination, not per forward pass)
    mutable std::vector<LaunchTable> launch_tables;
};

namespace {

int dev_alloc(DevBuf& b, size_t bytes) {
    b.p = nullptr;
    b.bytes = 0;
    if (bytes == 0) return RNN_OK;
    if (hipMalloc(&b.p, bytes) != hipSuccess) {
        (void)hipGetLastError();
        b.p = nullptr;
        return RNN_ENOMEM;
    }
    b.bytes = bytes;
    return RNN_OK;
}

void dev_free(DevBuf& b) {
    if (b.p) (void)hipFree(b.p);
    b.p = nullptr;
    b.bytes = 0;
}

void free_workspace(rnn_model* m) {
    dev_free(m->ws.gx); dev_free(m->ws.hseq); dev_free(m->ws.flags); dev_free(m->ws.h_f32);
    dev_free(m->ws.c_f32); dev_free(m->ws.h_st); dev_free(m->ws.gh); dev_free(m->ws.ticks);
    for (auto& b : m->ws.ybuf) dev_free(b);
    dev_free(m->ws.lseq);
    dev_free(m->ws.xblk);
    dev_free(m->ws.rh_st);
    dev_free(m->ws.gh2);
    dev_free(m->ws.x_tm);
    dev_free(m->ws.y_tm);
    dev_free(m->ws.x_ck);
    dev_free(m->ws.y_ck);
    dev_free(m->ws.y_pad);
    for (auto& b : m->ws.st_pad) dev_free(b);
    for (auto& b : m->ws.st_ck) dev_free(b);
    m->workspace_bytes = 0;
}

constexpr int FLAG_COLBLOCKS_MAX = 16;

// The caller's x can be brought into the layout of a state sequence (launch_to_blocked's limits).
bool relayout_fits(const rnn_model* m, int T) {
    return T <= 65535 && (size_t)16 * m->H * m->esize <= 64 * 1024;
}

// Choose how the grid of cells is laid over the compute units for batch size B.
bool choose_wavefront(const rnn_model* m, int T, int B, Plan& plan) {
    if (m->H % 4 != 0) return false;
    const int row_tiles = m->H / 4;
    const int col_tiles = (B + 15) / 16;
    const int lp_max = (m->D == 1) ? (m->L < WF_MAX_LAYERS ? m->L : WF_MAX_LAYERS) : 1;
    // {row tiles, column tiles per chain, chains per workgroup}
    // ({2, 2, 2}: 8 hidden units per workgroup, for layers of more than 1024 units, whose slices of 16 units
    // no longer fit a workgroup's registers)
    static const int cand[][3] = {{1, 1, 1}, {2, 1, 1}, {4, 1, 1}, {1, 4, 1}, {4, 2, 2}, {4, 4, 1}, {2, 2, 2}};
    for (int launches = (m->L + lp_max - 1) / lp_max; launches <= m->L; ++launches) {
        const int LP = (m->L + launches - 1) / launches;
        const int budget = m->num_cus / (LP * m->D);
        int best = -1, best_cost = 0, best_rt = 0, best_nch = 0;
        bool best_first_alone = false;
        int tag_small = -1, tag_large = -1;   // tag-in-data candidates: smallest tile within 3/8 of the chip, largest tile
        for (int c = 0; c < (int)(sizeof(cand) / sizeof(cand[0])); ++c) {
            const int RT = cand[c][0], CT = cand[c][1], NCH = cand[c][2];
            if (row_tiles % RT) continue;
            if (RT == 2 && CT == 2 && m->H <= 1024) continue;
            const bool tagged = (CT == 1 && NCH == 1);  // single tile of 16 sequences: tag-in-data kernel
            // several layers of large tiles side by side: the inside-product kernel when every layer's
            // input is H wide, else the flag-vector kernel with a projection for the first layer
            // x-kernel launches of several layers: all layers when the model's input is H wide, the layers
            // above the first (which then runs alone, behind its projection) otherwise
            const bool side_by_side = !tagged && LP > 1 && m->D == 1 &&
                                      wavefront_x_variant_exists(m->dtype, RT, CT, NCH, m->H, m->lds_limit, true) &&
                                      (m->I == m->H ? relayout_fits(m, T)
                                                    : wavefront_variant_exists(m->dtype, RT, CT, NCH, m->H, false));
            const bool have = tagged ? wavefront_ll_variant_exists(m->dtype, RT, m->H)
                                     : (wavefront_variant_exists(m->dtype, RT, CT, NCH, m->H, LP > 1) || side_by_side);
            if (!have) continue;
            const int nrb = row_tiles / RT, ncb = (col_tiles + CT - 1) / CT;
            if (ncb % NCH) continue;
            // the tag-in-data kernel addresses two state sequences with 32-bit byte offsets
            if (tagged && wavefront_ll_words(m->dtype, 2, T, B, m->H) * 8 >= ((size_t)1 << 31)) continue;
            const int occ = tagged ? 1 : wavefront_variant_occupancy(CT);
            if (nrb * (ncb / NCH) > budget * occ || ncb > FLAG_COLBLOCKS_MAX) continue;
            if (tagged) {
                // The step of that kernel is an all-gather among the workgroups of a layer, and the more
                // workgroups poll, the longer a store takes to reach them (measured at batch 8, 2 layers of
                // 512 units: 256, 128, 64 workgroups in the launch take 3.6, 2.3-2.9, 2.15 us per step;
                // one layer of 1024 units at batch 1 on 256 or 64 workgroups: 1.95 and 2.05 us; 12 layers
                // of 64 units: 192, 96, 48 workgroups give 1.45, 1.3, 1.5 us).  So: the smallest tile that
                // keeps the whole launch within 3/8 of the compute units, else the largest tile.
                if (tag_small < 0 && LP * m->D * nrb * ncb <= m->num_cus * 3 / 8) tag_small = c;
                tag_large = c;
                continue;
            }
            // work per workgroup and step; at equal work prefer interleaved chains, then taller tiles
            const int cost = RT * CT * NCH;
            if (best < 0 || cost < best_cost || (cost == best_cost && NCH > best_nch) ||
                (cost == best_cost && NCH == best_nch && RT > best_rt)) {
                best = c; best_cost = cost; best_rt = RT; best_nch = NCH;
                best_first_alone = side_by_side && m->I != m->H;
            }
        }
        if (tag_large >= 0) best = tag_small >= 0 ? tag_small : tag_large;
        if (best >= 0) {
            plan.kind = RNN_PLAN_WAVEFRONT;
            plan.LP = LP;
            plan.RT = cand[best][0];
            plan.CT = cand[best][1];
            plan.NCH = cand[best][2];
            plan.nrb = row_tiles / plan.RT;
            plan.ncb = (col_tiles + plan.CT - 1) / plan.CT;
            plan.first_alone = best_first_alone && !(plan.CT == 1 && plan.NCH == 1);
            return true;
        }
    }
    return false;
}

// Which layers share a launch, and which group of workgroups of a launch runs which (layer, direction): taken from
// the scheduler, not from arithmetic on layer numbers.  The cell graph of the layers that run in the persistent
// kernels (Section 2.2; all of them, or those above a first layer that runs alone behind its projection) is built
// (rnn_schedule_grid), sorted (rnn_schedule_order: the topological sorting of Section 4.1) and placed
// (rnn_schedule_place_resident: the list scheduling of Section 3 with one kind of weights per processor and pass)
// on P = LP * D processors, one per group of workgroups that a launch of this plan has room for.  A pass of the
// placement is a launch; the processor of a (layer, direction) in its pass is its group.  Cell times: the products
// of a cell, 2 * gates * H * (input width + H) flops, relative to a layer above the first; an edge costs a quarter of
// such a cell across groups (a state vector through the L2).  The grid is uniform along time, so the first 256
// steps decide.  The kernels number the groups of a launch by ascending (layer, direction) and take the launch's
// first layer and layer count; processors are identical, so the groups of a pass are renumbered that way, and what
// the kernels cannot run (a layer split over passes, directions of one layer in different passes, layers of a
// pass that are not consecutive) is reported as an error instead of being run differently.
int derive_launches(const rnn_model* m, Plan& plan, int T) {
    const int steps = T < 256 ? T : 256;
    for (const LaunchTable& t : m->launch_tables)
        if (t.steps == steps && t.LP == plan.LP && t.first_alone == plan.first_alone) {
            plan.layer_launch = t.layer_launch; plan.launch_layer0 = t.launch_layer0; plan.launch_layers = t.launch_layers;
            return RNN_OK;
        }
    LaunchTable tab;
    tab.steps = steps; tab.LP = plan.LP; tab.first_alone = plan.first_alone;
    tab.layer_launch.assign(m->L, -1);
    const int lbase = plan.first_alone ? 1 : 0;         // layers below lbase run in launches of their own
    for (int l = 0; l < lbase; ++l) {
        tab.layer_launch[l] = l;
        tab.launch_layer0.push_back(l);
        tab.launch_layers.push_back(1);
    }
    const int Ls = m->L - lbase, D = m->D;
    if (Ls > 0) {
        int n = 0, ne = 0;
        int rc = rnn_schedule_grid_size(Ls, steps, D, &n, &ne);
        if (rc != RNN_OK) return rc;
        std::vector<int> off(n + 1), idx(ne > 0 ? ne : 1), order(n), kind(n), proc(n), pass(n);
        std::vector<double> exec(n), comm(ne > 0 ? ne : 1, 0.25);
        rc = rnn_schedule_grid(Ls, steps, D, off.data(), idx.data());
        if (rc != RNN_OK) return rc;
        const double unit = (double)(m->layer_input(m->L - 1) + m->H);
        for (int v = 0; v < n; ++v) {
            kind[v] = v / steps;                        // vertex (l * D + d) * steps + s
            exec[v] = (double)(m->layer_input(lbase + kind[v] / D) + m->H) / unit;
        }
        rc = rnn_schedule_order(n, off.data(), idx.data(), comm.data(), exec.data(), order.data());
        if (rc != RNN_OK) return rc;
        double latency = 0.0;
        int passes = 0;
        rc = rnn_schedule_place_resident(n, off.data(), idx.data(), order.data(), plan.LP * D, exec.data(), comm.data(),
                                         kind.data(), proc.data(), pass.data(), nullptr, &latency, &passes);
        if (rc != RNN_OK) return rc;
        std::vector<int> first(passes, -1), last(passes, -1);
        for (int k = 0; k < Ls * D; ++k) {
            const int l = lbase + k / D, r = pass[k * steps];
            for (int s = 1; s < steps; ++s)
                if (pass[k * steps + s] != r || proc[k * steps + s] != proc[k * steps]) return RNN_EDEVICE;
            if (k % D && r != pass[(k - 1) * steps]) return RNN_EDEVICE;     // the directions of a layer share a launch
            if (first[r] < 0) first[r] = l;
            if (l < first[r] || (last[r] >= 0 && l > last[r] + 1)) return RNN_EDEVICE;   // ascending and consecutive
            last[r] = l;
            tab.layer_launch[l] = lbase + r;
        }
        for (int r = 0; r < passes; ++r) {
            if (first[r] < 0 || (r > 0 && first[r] != last[r - 1] + 1)) return RNN_EDEVICE;
            tab.launch_layer0.push_back(first[r]);
            tab.launch_layers.push_back(last[r] - first[r] + 1);
        }
    }
    plan.layer_launch = tab.layer_launch; plan.launch_layer0 = tab.launch_layer0; plan.launch_layers = tab.launch_layers;
    if (m->launch_tables.size() >= 64) m->launch_tables.clear();
    m->launch_tables.push_back(std::move(tab));
    return RNN_OK;
}

int resolve_plan_shape(const rnn_model* m, int T, int B, Plan& plan, bool may_chunk);

// may_chunk: a batch that no persistent launch can hold may be split into passes
int resolve_plan(const rnn_model* m, int T, int B, Plan& plan, bool may_chunk = true) {
    const int rc = resolve_plan_shape(m, T, B, plan, may_chunk);
    if (rc != RNN_OK || plan.kind != RNN_PLAN_WAVEFRONT) return rc;
    return derive_launches(m, plan, T);
}

int resolve_plan_shape(const rnn_model* m, int T, int B, Plan& plan, bool may_chunk) {
    if (m->cellwise_only() && m->requested_plan == RNN_PLAN_WAVEFRONT) return RNN_EUNSUPPORTED;
    if (m->requested_plan == RNN_PLAN_CELLWISE || m->cellwise_only()) {
        plan = Plan();
        return RNN_OK;
    }
    if (choose_wavefront(m, T, B, plan)) return RNN_OK;
    if (may_chunk) {
        // the largest multiple of 16 sequences below B that has a plan (every workgroup's tiles full)
        for (int bc = ((B - 1) / 16) * 16; bc >= 16; bc -= 16)
            if (choose_wavefront(m, T, bc, plan)) {
                plan.chunk = bc;
                return RNN_OK;
            }
    }
    if (m->requested_plan == RNN_PLAN_WAVEFRONT) return RNN_EUNSUPPORTED;
    plan = Plan();
    return RNN_OK;
}

// First layer and number of layers of the launch that holds layer l (from the scheduler's table).
void launch_of(const rnn_model* m, const Plan& plan, int l, int& l0, int& n) {
    if (plan.layer_launch.empty()) { l0 = l; n = 1; return; }
    const int r = plan.layer_launch[l];
    l0 = plan.launch_layer0[r];
    n = plan.launch_layers[r];
}
bool first_of_launch(const rnn_model* m, const Plan& plan, int l) {
    int l0, n;
    launch_of(m, plan, l, l0, n);
    return l == l0;
}
int launch_count(const rnn_model* m, const Plan& plan) {
    return plan.layer_launch.empty() ? m->L : (int)plan.launch_layer0.size();
}

// Index of the launch that holds layer l (launches are numbered in stream order).
int launch_index(const Plan& plan, int l) { return plan.layer_launch.empty() ? l : plan.layer_launch[l]; }

// Only what is live is kept (the paper's memory model, Section 3, Equation 4, charges an operator's output
// while a successor still needs it): the output of layer l is read by layer l + 1 alone, and a state
// sequence by its own launch and by the launch after it.
//
// Entry of ws.ybuf that holds the output of layer l < L - 1, or -1 when that layer keeps none (its consumer
// reads its state sequence, or sits in the same launch of the tag-in-data kernel and reads the tagged words).
int ybuf_slot(const rnn_model* m, const Plan& plan, int l, int T);
// Layer regions of the state-sequence buffer: two launches' worth, used alternately.
int state_regions(const rnn_model* m, const Plan& plan) { return std::min(m->L, 2 * plan.LP); }
int state_region_index(const rnn_model* m, const Plan& plan, int l) {
    int l0, n;
    launch_of(m, plan, l, l0, n);
    if (state_regions(m, plan) == m->L) return l;   // every layer has its own
    return (launch_index(plan, l) % 2) * plan.LP + (l - l0);
}

// Gate row of the caller's [G*H, K] matrix that feeds slot s of unit u; -1 = no row (zeros).
// order: rnn_gate_order of the caller's row blocks.
int source_row(int cell, bool recurrent, int H, int u, int s, int order) {
    if (cell == CELL_LSTM) {                            // slots i, f, g, o
        static const int onnx_block[4] = {0, 2, 3, 1};  // ONNX row blocks are i, o, f, c
        return (order == RNN_ORDER_ONNX ? onnx_block[s] : s) * H + u;
    }
    const int r_blk = order == RNN_ORDER_ONNX ? 1 : 0;  // ONNX row blocks are z, r, h
    const int z_blk = order == RNN_ORDER_ONNX ? 0 : 1;
    if (s == 0) return r_blk * H + u;
    if (s == 1) return z_blk * H + u;
    if (s == 2) return recurrent ? -1 : 2 * H + u;      // n_x: input part of the candidate
    return recurrent ? 2 * H + u : -1;                  // n_h: recurrent part of the candidate
}

float elem_to_f32(const void* base, size_t i, int dtype) {
    if (dtype == DT_BF16) return bf16_to_f32(((const bf16_t*)base)[i]);
    return ((const float*)base)[i];
}

constexpr size_t PROF_MAX_SLOTS = 1 << 14;

// Record the start of a profiled launch; returns the slot index or -1 when profiling is off.
int prof_begin(rnn_model* m, int kind, hipStream_t st) {
    if (!m->profiling || m->capturing || m->prof_used >= PROF_MAX_SLOTS) return -1;
    if (m->prof_used == m->prof.size()) {
        if (m->arena.on) return -1;   // a call that must not allocate records into existing event pairs only
        rnn_model::ProfSlot s;
        if (hipEventCreate(&s.a) != hipSuccess) { (void)hipGetLastError(); return -1; }
        if (hipEventCreate(&s.b) != hipSuccess) { (void)hipGetLastError(); (void)hipEventDestroy(s.a); return -1; }
        s.kind = kind;
        m->prof.push_back(s);
    }
    const int i = (int)m->prof_used++;
    m->prof[i].kind = kind;
    (void)hipEventRecord(m->prof[i].a, st);
    return i;
}

void prof_end(rnn_model* m, int slot, hipStream_t st) {
    if (slot >= 0) (void)hipEventRecord(m->prof[slot].b, st);
}

#define HIP_TRY(expr)                       \
    do {                                    \
        if ((expr) != hipSuccess) {         \
            (void)hipGetLastError();        \
            return RNN_EDEVICE;             \
        }                                   \
    } while (0)

int forward_cellwise(rnn_model* m, const void* x, const int32_t* lengths, const float* h0,
                     const float* c0, void* y, float* hT, float* cT, int T, int B,
                     hipStream_t st) {
    const size_t per = (size_t)B * m->H;
    const size_t state = (size_t)m->L * m->D * per;
    HIP_TRY(launch_state_init(m->dtype, h0, c0, (float*)m->ws.h_f32.p, (float*)m->ws.c_f32.p,
                              m->ws.h_st.p, state, st));
    const int N4 = SLOTS * m->H;
    for (int l = 0; l < m->L; ++l) {
        const void* in = (l == 0) ? x : m->ws.ybuf[(l - 1) % 2].p;      // two buffers, used alternately
        void* out = (l == m->L - 1) ? y : m->ws.ybuf[l % 2].p;
        const int K = m->layer_input(l);
        const int ps = prof_begin(m, RNN_KERNEL_PROJECTION, st);
        HIP_TRY(launch_gemm_nt(m->dtype, in, K, m->wih[l].p, K, (float*)m->ws.gx.p, m->D * N4,
                               T * B, m->D * N4, K, st));
        prof_end(m, ps, st);
        for (int s = 0; s < T; ++s) {
            for (int d = 0; d < m->D; ++d) {
                const int g = l * m->D + d;
                float* gh = (float*)m->ws.gh.p + (size_t)d * B * N4;
                void* hst = (char*)m->ws.h_st.p + (size_t)g * per * m->esize;
                HIP_TRY(launch_gemm_nt(m->dtype, hst, m->H, m->whh[g].p, m->H, gh, N4, B, N4,
                                       m->H, st));
                CellStepArgs a;
                a.cell = m->cell; a.dtype = m->dtype;
                a.B = B; a.H = m->H; a.D = m->D; a.d = d; a.t = d ? (T - 1 - s) : s;
                a.gx = (const float*)m->ws.gx.p; a.gh = gh; a.bias = (const float*)m->bias[g].p;
                a.h_f32 = (float*)m->ws.h_f32.p + (size_t)g * per;
                a.c_f32 = (float*)m->ws.c_f32.p + (size_t)g * per;
                a.h_st = hst; a.out = out; a.lengths = lengths; a.T = T;
                a.gh_rh = nullptr; a.rh_st = nullptr;
                a.peep = m->peep.empty() ? nullptr : (const float*)m->peep[g].p;
                a.clip = m->clip;
                if (m->gru_reset_before) {  // r, then W_hh (r * h), whose candidate slot replaces gh's
                    a.rh_st = m->ws.rh_st.p;
                    HIP_TRY(launch_gru_reset(a, st));
                    HIP_TRY(launch_gemm_nt(m->dtype, m->ws.rh_st.p, m->H, m->whh[g].p, m->H, (float*)m->ws.gh2.p, N4, B,
                                           N4, m->H, st));
                    a.gh_rh = (const float*)m->ws.gh2.p;
                }
                HIP_TRY(launch_cell_step(a, st));
            }
        }
    }
    HIP_TRY(launch_state_export((const float*)m->ws.h_f32.p, (const float*)m->ws.c_f32.p, hT,
                                m->cell == CELL_LSTM ? cT : nullptr, state, st));
    return RNN_OK;
}

// Grow a workspace buffer to at least `bytes` (never shrinks).  Growing waits for the device, since
// work in flight may still use the old buffer.  `zeroed`: fresh memory is cleared once (flag words
// and tagged words: tag 0 is never used by a launch).
int grow(rnn_model* m, DevBuf& b, size_t bytes, bool zeroed = false) {
    if (b.bytes >= bytes) return RNN_OK;
    if (m->arena.on) {
        // rnn_forward_static: the buffer is the next piece of the device's static array (256-byte aligned);
        // the array keeps what the last call left, so what must start at zero is cleared on the stream
        const size_t at = (m->arena.used + 255) & ~(size_t)255;
        if (bytes > STATIC_SCRATCH_BYTES || at > STATIC_SCRATCH_BYTES - bytes) return RNN_ESCRATCH;
        b.p = m->arena.base + at;
        b.bytes = bytes;
        m->arena.used = at + bytes;
        if (zeroed) HIP_TRY(launch_fill_zero(b.p, (bytes + 3) & ~(size_t)3, m->arena.stream));
        return RNN_OK;
    }
    if (m->capturing) return RNN_EUNSUPPORTED;   // no allocation and no waiting inside a stream capture
    HIP_TRY(hipDeviceSynchronize());
    m->workspace_bytes -= b.bytes;
    dev_free(b);
    const int rc = dev_alloc(b, bytes);
    if (rc != RNN_OK) return rc;
    m->workspace_bytes += bytes;
    if (zeroed) HIP_TRY(hipMemset(b.p, 0, bytes));
    return RNN_OK;
}

// Rows per 16-unit block of a blocked sequence: B rounded up to a multiple of 4, so that a block
// (rows x 16 elements of 2 or 4 bytes) is a whole number of 128-byte cache lines and no line holds
// sequences of two chains.
inline size_t blocked_rows(int B) { return ((size_t)B + 3) & ~(size_t)3; }

// State sequences of the layers from l0 on (flag-vector kernels): every (layer, direction) owns
// T + 1 slots of blocked_rows(B) * H elements, so a layer can read the finished sequence of the
// layer below.
void* state_region(rnn_model* m, const Plan& plan, int l, int T, int B) {
    return (char*)m->ws.hseq.p +
           (size_t)state_region_index(m, plan, l) * m->D * (T + 1) * blocked_rows(B) * m->H * m->esize;
}

// One persistent launch: layers [l0, l0 + LP) over all T steps.
// gx: projection of layer l0, or NULL when the layer computes its input product itself, from xin
// (blocked like a state sequence) or, with x_from_state, from the state sequence of the layer below.
int launch_recurrent(rnn_model* m, const Plan& plan, int l0, int LP, int T, int B,
                     const float* gx, void* y, const int32_t* lengths, const float* h0,
                     const float* c0, float* hT, float* cT, hipStream_t st, const void* xin = nullptr,
                     bool x_from_state = false) {
    const bool tagged = plan.CT == 1 && plan.NCH == 1;
    if (++m->epoch == 0) {  // the tag wrapped: start over from cleared buffers
        HIP_TRY(launch_fill_zero(m->ws.lseq.p, m->ws.lseq.bytes, st));
        HIP_TRY(launch_fill_zero(m->ws.flags.p, m->ws.flags.bytes, st));
        m->epoch = 1;
    }
    if (tagged) {
        HIP_TRY(launch_wavefront_ll_init(m->dtype, h0, l0, LP, m->D, T, B, m->H,
                                         (uint64_t*)m->ws.lseq.p, m->epoch, st));
    } else {
        HIP_TRY(launch_wavefront_init(m->dtype, h0, l0, LP, m->D, T, B, (int)blocked_rows(B), m->H,
                                      state_region(m, plan, l0, T, B), st));
    }
    WavefrontArgs a;
    memset(&a, 0, sizeof(a));
    a.cell = m->cell; a.dtype = m->dtype;
    a.T = T; a.B = B; a.Bp = (int)blocked_rows(B); a.H = m->H; a.D = m->D; a.L_total = m->L;
    a.l0 = l0; a.LP = LP;
    a.RT = plan.RT; a.CT = plan.CT; a.NCH = plan.NCH; a.nrb = plan.nrb; a.ncb = plan.ncb;
    for (int ll = 0; ll < LP; ++ll) {
        const int l = l0 + ll;
        for (int d = 0; d < m->D; ++d) {
            a.whh[ll * m->D + d] = m->whh[l * m->D + d].p;
            a.wih[ll * m->D + d] = m->wih[l].p;  // fused layers have D = 1
            a.bias[ll * m->D + d] = (const float*)m->bias[l * m->D + d].p;
            a.peep[ll * m->D + d] = m->peep.empty() ? nullptr : (const float*)m->peep[l * m->D + d].p;
        }
        const int slot = (l == m->L - 1) ? -1 : ybuf_slot(m, plan, l, T);
        a.out[ll] = (l == m->L - 1) ? y : (slot >= 0 ? m->ws.ybuf[slot].p : nullptr);
        // a layer whose consumer reads the state sequence instead keeps no separate output
        if (!tagged && (xin || x_from_state) && l != m->L - 1) a.out[ll] = nullptr;
    }
    a.clip = m->clip;
    a.ext = (m->clip > 0.0f || !m->peep.empty()) ? 1 : 0;
    a.gx = gx;
    a.xin = xin;
    a.xin_width2 = (tagged && xin) ? 2 * m->layer_input(l0) / m->H : 0;
    if (x_from_state)  // x_t of layer l0 = state of layer l0 - 1 after step t = slot t + 1 of its sequence
        a.xin = (const char*)state_region(m, plan, l0 - 1, T, B) + blocked_rows(B) * m->H * m->esize;
    a.hseq = state_region(m, plan, l0, T, B);
    a.h0 = h0; a.c0 = c0; a.hT = hT; a.cT = cT; a.lengths = lengths;
    a.flagv = (uint64_t*)m->ws.flags.p;
    // the launch must stay inside the buffers the workspace holds (a kernel never checks)
    if (tagged) {
        if (wavefront_ll_words(m->dtype, LP * m->D, T, B, m->H) * sizeof(uint64_t) > m->ws.lseq.bytes) return RNN_EDEVICE;
    } else {
        const size_t flag_words = (size_t)LP * m->D * T * plan.ncb * plan.nrb;
        const size_t state_end = (size_t)(state_region_index(m, plan, l0) + LP) * m->D * (T + 1) * blocked_rows(B) * m->H * m->esize;
        if (flag_words * sizeof(uint64_t) > m->ws.flags.bytes || state_end > m->ws.hseq.bytes) return RNN_EDEVICE;
    }
    a.status = (unsigned*)m->status.p;
    a.ticks = m->want_ticks ? (unsigned long long*)m->ws.ticks.p + (size_t)l0 * m->D * T : nullptr;
    a.spin_limit = m->spin_limit;
    a.lseq = (uint64_t*)m->ws.lseq.p;
    a.epoch = m->epoch;
    const int ps = prof_begin(m, RNN_KERNEL_RECURRENT, st);
    if (tagged) HIP_TRY(launch_wavefront_ll(a, st));
    else if (a.xin) HIP_TRY(launch_wavefront_x(a, st));
    else HIP_TRY(launch_wavefront(a, st));
    prof_end(m, ps, st);
    return RNN_OK;
}

// A layer that runs alone in its launch, in one direction, on an input of its own width can do
// its input product inside the recurrent kernel (wavefront_x.hip) instead of through a projection.
// So can the first layer of a launch of the tag-in-data kernel (its x waves read the plain input).
bool input_product_inside(const rnn_model* m, const Plan& plan, int l, int T) {
    if (plan.kind != RNN_PLAN_WAVEFRONT) return false;
    if (plan.CT == 1 && plan.NCH == 1) {
        // tag-in-data kernel, first layer of a launch (layers above it in the launch are fused anyway): its
        // x waves hold the W_ih slice in registers, which fits for an input H wide, or 2H wide (a
        // bidirectional layer above the first) with small tiles
        if (!first_of_launch(m, plan, l)) return false;
        const int kw = (m->dtype == DT_BF16) ? 32 : 4;          // K elements per MFMA
        const int KB = m->H / (4 * kw);
        if (m->layer_input(l) == m->H) return true;
        if (2 * m->layer_input(l) == m->H) return KB % 2 == 0;
        return plan.LP == 1 && m->D == 2 && m->layer_input(l) == 2 * m->H && plan.RT * KB * 2 <= 32;
    }
    if (m->D != 1 || m->layer_input(l) != m->H) return false;
    // the first layer's input is first brought into the layout of a state sequence
    int l0, n;
    launch_of(m, plan, l, l0, n);
    if (n == 1) {
        if (l == 0 && !relayout_fits(m, T)) return false;
        return wavefront_x_variant_exists(m->dtype, plan.RT, plan.CT, plan.NCH, m->H, m->lds_limit);
    }
    // several layers per launch: all of them inside, or none (the launch's first layer would need gx)
    if (l0 == 0 && (m->I != m->H || !relayout_fits(m, T))) return false;
    return wavefront_x_variant_exists(m->dtype, plan.RT, plan.CT, plan.NCH, m->H, m->lds_limit, true);
}

int ybuf_slot(const rnn_model* m, const Plan& plan, int l, int T) {
    if (plan.kind != RNN_PLAN_WAVEFRONT) return l % 2;          // cellwise: two buffers, used alternately
    const bool tagged = plan.CT == 1 && plan.NCH == 1;
    int l0, n;
    launch_of(m, plan, l, l0, n);
    if (tagged) {
        // only the last layer of a launch writes an output (the layers inside a launch exchange tagged
        // words); the launch after it reads it: two buffers, used alternately
        return l == l0 + n - 1 ? launch_index(plan, l) % 2 : -1;
    }
    // flag-vector kernels: a layer that computes its input product inside keeps no output of its own unless it
    // is the last (the layer above it does the same and reads this layer's state sequence, slot t + 1); any
    // other layer keeps one (a fused layer of the same launch reads it while it is produced)
    return input_product_inside(m, plan, l, T) ? -1 : l;
}

// Size the workspace for one forward pass of T steps and B sequences under `plan`: only what that
// plan touches is allocated (the paper's memory model, Section 3, Equation 4, charges a model with
// its weights, outputs and temporaries; this is the temporaries part).
int prepare_workspace_pass(rnn_model* m, const Plan& plan, int T, int B) {
    const size_t rows = (size_t)T * B;
    const size_t state = (size_t)m->L * m->D * B * m->H;
    const bool wavefront = plan.kind == RNN_PLAN_WAVEFRONT;
    const bool tagged = wavefront && plan.CT == 1 && plan.NCH == 1;
    bool any_projection = !wavefront;
    if ((int)m->ws.ybuf.size() < m->L - 1) m->ws.ybuf.resize(m->L - 1);
    int rc = RNN_OK;
    for (int l = 0; l < m->L && rc == RNN_OK; ++l) {
        const bool inside = wavefront && input_product_inside(m, plan, l, T);
        if (!inside && (!wavefront || first_of_launch(m, plan, l))) any_projection = true;
        const int slot = l + 1 < m->L ? ybuf_slot(m, plan, l, T) : -1;
        if (slot >= 0) rc = grow(m, m->ws.ybuf[slot], rows * m->D * m->H * m->esize);
    }
    if (rc == RNN_OK && any_projection) rc = grow(m, m->ws.gx, rows * m->D * m->H * SLOTS * sizeof(float));
    if (rc == RNN_OK && wavefront && !tagged) {
        rc = grow(m, m->ws.hseq, (size_t)state_regions(m, plan) * m->D * (T + 1) * blocked_rows(B) * m->H * m->esize);
        // one flag word per (layer of a launch, direction, step, chain, row block); every launch stamps
        // them with its own tag, so all launches share the words of one
        if (rc == RNN_OK)
            rc = grow(m, m->ws.flags, (size_t)std::min(m->L, plan.LP) * m->D * T * plan.ncb * plan.nrb * sizeof(uint64_t), true);
        if (rc == RNN_OK && input_product_inside(m, plan, 0, T)) rc = grow(m, m->ws.xblk, (size_t)T * blocked_rows(B) * m->H * m->esize);
    }
    if (rc == RNN_OK && tagged)
        rc = grow(m, m->ws.lseq, wavefront_ll_words(m->dtype, plan.LP * m->D, T, B, m->H) * sizeof(uint64_t), true);
    if (rc == RNN_OK && !wavefront) {
        rc = grow(m, m->ws.h_f32, state * sizeof(float));
        if (rc == RNN_OK) rc = grow(m, m->ws.c_f32, state * sizeof(float));
        if (rc == RNN_OK) rc = grow(m, m->ws.h_st, state * m->esize);
        if (rc == RNN_OK) rc = grow(m, m->ws.gh, (size_t)m->D * B * m->H * SLOTS * sizeof(float));
        if (rc == RNN_OK && m->gru_reset_before) {
            rc = grow(m, m->ws.rh_st, (size_t)B * m->H * m->esize);
            if (rc == RNN_OK) rc = grow(m, m->ws.gh2, (size_t)B * m->H * SLOTS * sizeof(float));
        }
    }
    if (rc == RNN_OK) rc = grow(m, m->ws.ticks, (size_t)m->L * m->D * T * sizeof(unsigned long long));
    return rc;
}

// The workspace of a whole call: that of one pass (of the last, shorter pass too, whose plan may differ),
// the copies a batch run in passes goes through, and the time-major copies of a batch-first caller.
int prepare_workspace(rnn_model* m, const Plan& plan, int T, int B) {
    int rc;
    if (plan.chunk == 0) {
        rc = prepare_workspace_pass(m, plan, T, B);
    } else {
        Plan one = plan;
        one.chunk = 0;
        rc = prepare_workspace_pass(m, one, T, plan.chunk);
        const int tail = B % plan.chunk;
        if (rc == RNN_OK && tail != 0) {
            Plan last;
            rc = resolve_plan(m, T, tail, last, false);
            if (rc == RNN_OK) rc = prepare_workspace_pass(m, last, T, tail);
        }
        const size_t rows = (size_t)T * plan.chunk;
        if (rc == RNN_OK) rc = grow(m, m->ws.x_ck, rows * m->I * m->esize);
        if (rc == RNN_OK) rc = grow(m, m->ws.y_ck, rows * m->D * m->H * m->esize);
        for (int i = 0; i < 4 && rc == RNN_OK; ++i)
            rc = grow(m, m->ws.st_ck[i], (size_t)m->L * m->D * plan.chunk * m->H * sizeof(float));
    }
    if (rc == RNN_OK && m->H != m->Hu) {
        rc = grow(m, m->ws.y_pad, (size_t)T * B * m->D * m->H * m->esize);
        for (int i = 0; i < 4 && rc == RNN_OK; ++i)
            rc = grow(m, m->ws.st_pad[i], (size_t)m->L * m->D * B * m->H * sizeof(float));
    }
    if (rc == RNN_OK && m->batch_first) {
        const size_t rows = (size_t)T * B;
        rc = grow(m, m->ws.x_tm, rows * m->I * m->esize);
        if (rc == RNN_OK) rc = grow(m, m->ws.y_tm, rows * m->D * m->Hu * m->esize);
    }
    return rc;
}

// The persistent kernels exist for certain widths only (a wave's K quarter is a whole number of MFMA K
// blocks, and only some block counts are compiled).  Any other width is padded up to the next one that
// has them: the added units get zero weights, zero biases and a zero initial state, so they stay at zero
// (LSTM: c = 0.5 * 0 + 0.5 * tanh(0), h = 0.5 * tanh(0); GRU: h = 0.5 * tanh(0) + 0.5 * 0) and, their
// columns of W_hh and of the next layer's W_ih being zero as well, reach nothing.  Returns H when H is
// covered or beyond every compiled width.
int padded_width(int dtype, int H) {
    static const int bf16_blocks[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};   // x 128 units
    static const int f32_blocks[] = {2, 4, 8, 16, 32};                      // x 16 units
    const int unit = dtype == DT_BF16 ? 128 : 16;
    const int* blocks = dtype == DT_BF16 ? bf16_blocks : f32_blocks;
    const int n = dtype == DT_BF16 ? 10 : 5;
    const int need = (H + unit - 1) / unit;
    for (int i = 0; i < n; ++i)
        if (blocks[i] >= need) return blocks[i] * unit;
    return H;
}

// Shapes the library accepts (rnn_model_create_ordered, rnn_plan_query).
int check_model_shape(int cell, int num_layers, int input_size, int hidden_size, int num_directions, int dtype) {
    if (cell != RNN_LSTM && cell != RNN_GRU) return RNN_EINVAL;
    if (dtype != RNN_F32 && dtype != RNN_BF16) return RNN_EINVAL;
    if (num_layers < 1 || input_size < 1 || hidden_size < 1) return RNN_EINVAL;
    if (num_directions != 1 && num_directions != 2) return RNN_EINVAL;
    if (num_layers > 1024 || input_size > (1 << 20) || hidden_size > (1 << 16)) return RNN_EUNSUPPORTED;
    const int align = (dtype == RNN_BF16) ? 8 : 4;
    if (hidden_size % align != 0) return RNN_EUNSUPPORTED;
    if (dtype == RNN_BF16 && input_size % 8 != 0) return RNN_EUNSUPPORTED;
    return RNN_OK;
}

int forward_wavefront(rnn_model* m, const Plan& plan, const void* x, const int32_t* lengths,
                      const float* h0, const float* c0, void* y, float* hT, float* cT, int T,
                      int B, hipStream_t st) {
    const int N4 = SLOTS * m->H;
    for (int l0 = 0, LP = 0; l0 < m->L; l0 += LP) {
        int first;
        launch_of(m, plan, l0, first, LP);
        const int in_slot = l0 == 0 ? -1 : ybuf_slot(m, plan, l0 - 1, T);
        const void* in = (l0 == 0) ? x : (in_slot >= 0 ? m->ws.ybuf[in_slot].p : nullptr);
        if (plan.CT == 1 && plan.NCH == 1 && input_product_inside(m, plan, l0, T)) {
            // tag-in-data kernel: the x waves of the launch's first layer read the plain input
            const int rc = launch_recurrent(m, plan, l0, LP, T, B, nullptr, y, lengths, h0, c0, hT, cT, st, in);
            if (rc != RNN_OK) return rc;
            continue;
        }
        if (input_product_inside(m, plan, l0, T)) {
            // the first layer reads the caller's x, re-laid out; a layer above reads the state sequence below it
            if (l0 == 0) HIP_TRY(launch_to_blocked(m->dtype, x, m->ws.xblk.p, T, B, (int)blocked_rows(B), m->H, st));
            const int rc = launch_recurrent(m, plan, l0, LP, T, B, nullptr, y, lengths, h0, c0, hT, cT, st,
                                            l0 == 0 ? m->ws.xblk.p : nullptr, l0 > 0);
            if (rc != RNN_OK) return rc;
            continue;
        }
        const int K = m->layer_input(l0);
        const int ps = prof_begin(m, RNN_KERNEL_PROJECTION, st);
        HIP_TRY(launch_gemm_nt(m->dtype, in, K, m->wih[l0].p, K, (float*)m->ws.gx.p, m->D * N4,
                               T * B, m->D * N4, K, st));
        prof_end(m, ps, st);
        const int rc = launch_recurrent(m, plan, l0, LP, T, B, (const float*)m->ws.gx.p, y, lengths, h0,
                                        c0, hT, cT, st);
        if (rc != RNN_OK) return rc;
    }
    return RNN_OK;
}

int forward_one_pass(rnn_model* m, const Plan& plan, const void* x, const int32_t* lengths, const float* h0,
                     const float* c0, void* y, float* hT, float* cT, int T, int B, hipStream_t st) {
    return (plan.kind == RNN_PLAN_WAVEFRONT) ? forward_wavefront(m, plan, x, lengths, h0, c0, y, hT, cT, T, B, st)
                                             : forward_cellwise(m, x, lengths, h0, c0, y, hT, cT, T, B, st);
}

// A batch larger than one persistent launch can hold: passes of plan.chunk sequences, each gathered
// into contiguous copies, run, and scattered back (the sequences of a batch do not interact).
int forward_in_passes(rnn_model* m, const Plan& plan, const void* x, const int32_t* lengths, const float* h0,
                      const float* c0, void* y, float* hT, float* cT, int T, int B, hipStream_t st) {
    const size_t xrow = (size_t)m->I * m->esize, yrow = (size_t)m->D * m->H * m->esize;
    const size_t srow = (size_t)m->H * sizeof(float);
    const int groups = m->L * m->D;
    for (int b0 = 0; b0 < B; b0 += plan.chunk) {
        const int bc = (B - b0 < plan.chunk) ? B - b0 : plan.chunk;
        Plan pass = plan;
        pass.chunk = 0;
        if (bc != plan.chunk) {
            const int rc = resolve_plan(m, T, bc, pass, false);
            if (rc != RNN_OK) return rc;
        }
        HIP_TRY(launch_copy_2d((const char*)x + b0 * xrow, B * xrow, m->ws.x_ck.p, bc * xrow, T, bc * xrow, st));
        float* h0p = nullptr; float* c0p = nullptr;
        if (h0) {
            h0p = (float*)m->ws.st_ck[0].p;
            HIP_TRY(launch_copy_2d((const char*)h0 + b0 * srow, B * srow, h0p, bc * srow, groups, bc * srow, st));
        }
        if (c0) {
            c0p = (float*)m->ws.st_ck[1].p;
            HIP_TRY(launch_copy_2d((const char*)c0 + b0 * srow, B * srow, c0p, bc * srow, groups, bc * srow, st));
        }
        float* hTp = hT ? (float*)m->ws.st_ck[2].p : nullptr;
        float* cTp = cT ? (float*)m->ws.st_ck[3].p : nullptr;
        const int rc = forward_one_pass(m, pass, m->ws.x_ck.p, lengths ? lengths + b0 : nullptr, h0p, c0p, m->ws.y_ck.p, hTp,
                                        cTp, T, bc, st);
        if (rc != RNN_OK) return rc;
        HIP_TRY(launch_copy_2d(m->ws.y_ck.p, bc * yrow, (char*)y + b0 * yrow, B * yrow, T, bc * yrow, st));
        if (hT) HIP_TRY(launch_copy_2d(hTp, bc * srow, (char*)hT + b0 * srow, B * srow, groups, bc * srow, st));
        if (cT) HIP_TRY(launch_copy_2d(cTp, bc * srow, (char*)cT + b0 * srow, B * srow, groups, bc * srow, st));
    }
    return RNN_OK;
}

}  // namespace

extern "C" {

int rnn_model_create(rnn_model** out, int cell, int num_layers, int input_size, int hidden_size,
                     int num_directions, int dtype, const void* const* weights,
                     int weights_on_device) {
    return rnn_model_create_ordered(out, cell, num_layers, input_size, hidden_size, num_directions, dtype,
                                    weights, weights_on_device, RNN_ORDER_IFGO_RZN);
}

int rnn_model_create_ordered(rnn_model** out, int cell, int num_layers, int input_size, int hidden_size,
                             int num_directions, int dtype, const void* const* weights,
                             int weights_on_device, int gate_order) {
    if (!out || !weights) return RNN_EINVAL;
    if (gate_order != RNN_ORDER_IFGO_RZN && gate_order != RNN_ORDER_ONNX) return RNN_EINVAL;
    {
        const int rc = check_model_shape(cell, num_layers, input_size, hidden_size, num_directions, dtype);
        if (rc != RNN_OK) return rc;
    }
    const int G = (cell == RNN_LSTM) ? 4 : 3;
    for (int i = 0; i < num_layers * num_directions * 4; ++i)
        if ((i % 4) < 2 && !weights[i]) return RNN_EINVAL;  // the two matrices are mandatory

    rnn_model* m = new (std::nothrow) rnn_model();
    if (!m) return RNN_ENOMEM;
    m->cell = cell; m->L = num_layers; m->I = input_size; m->Hu = hidden_size;
    m->H = padded_width(dtype, hidden_size);
    m->D = num_directions; m->dtype = dtype;
    m->esize = (dtype == RNN_BF16) ? 2 : 4;
    int rc = RNN_OK;
    hipDeviceProp_t prop;
    if (hipGetDevice(&m->device) != hipSuccess ||
        hipGetDeviceProperties(&prop, m->device) != hipSuccess) {
        (void)hipGetLastError();
        delete m;
        return RNN_EDEVICE;
    }
    m->num_cus = prop.multiProcessorCount;
    m->lds_limit = prop.sharedMemPerBlock;
    m->scratch = static_scratch_of(m->device);   // the model's device is current here
    m->ws.ybuf.resize(num_layers > 1 ? num_layers - 1 : 0);
    m->ws_static.ybuf.resize(num_layers > 1 ? num_layers - 1 : 0);

    const int H = m->H, D = m->D;
    m->wih.resize(m->L);
    m->whh.resize((size_t)m->L * D);
    m->bias.resize((size_t)m->L * D);
    std::vector<unsigned char> src, packed;
    std::vector<float> bias_host((size_t)H * SLOTS);
    auto fetch = [&](const void* p, size_t bytes) -> const unsigned char* {
        if (!weights_on_device) return (const unsigned char*)p;
        src.resize(bytes);
        if (hipMemcpy(src.data(), p, bytes, hipMemcpyDeviceToHost) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        return src.data();
    };
    const int Hu = m->Hu;
    // Rows: the caller's [G*Hu, Ku] matrix; packed: [H units][SLOTS][K].  `parts` pieces of `piece`
    // columns each (the halves [forward, backward] of a layer's input, or one piece for anything else)
    // land `piece_to` columns apart, so that a padded layer below is read at its padded positions;
    // rows of added units and the columns between the pieces stay zero.
    auto pack_matrix = [&](const void* wsrc, bool recurrent, int parts, int piece, int piece_to,
                           unsigned char* dst) -> int {
        const int Ku = parts * piece, K = parts * piece_to;
        const unsigned char* s = fetch(wsrc, (size_t)G * Hu * Ku * m->esize);
        if (!s) return RNN_EDEVICE;
        const size_t rowb = (size_t)K * m->esize, srowb = (size_t)Ku * m->esize;
        for (int u = 0; u < Hu; ++u)
            for (int sl = 0; sl < SLOTS; ++sl) {
                const int r = source_row(cell, recurrent, Hu, u, sl, gate_order);
                if (r < 0) continue;                    // dst starts out zeroed
                unsigned char* d = dst + ((size_t)u * SLOTS + sl) * rowb;
                for (int q = 0; q < parts; ++q)
                    memcpy(d + (size_t)q * piece_to * m->esize, s + (size_t)r * srowb + (size_t)q * piece * m->esize,
                           (size_t)piece * m->esize);
            }
        return RNN_OK;
    };
    for (int l = 0; l < m->L && rc == RNN_OK; ++l) {
        const int K = m->layer_input(l);
        const size_t one = (size_t)SLOTS * H * K * m->esize;
        packed.assign(one * D, 0);
        for (int d = 0; d < D && rc == RNN_OK; ++d)
            rc = (l == 0) ? pack_matrix(weights[(l * D + d) * 4 + 0], false, 1, K, K, packed.data() + one * d)
                          : pack_matrix(weights[(l * D + d) * 4 + 0], false, D, Hu, H, packed.data() + one * d);
        if (rc == RNN_OK) rc = dev_alloc(m->wih[l], one * D);
        if (rc == RNN_OK && hipMemcpy(m->wih[l].p, packed.data(), one * D, hipMemcpyHostToDevice) != hipSuccess)
            rc = RNN_EDEVICE;
        m->weight_bytes += one * D;
        for (int d = 0; d < D && rc == RNN_OK; ++d) {
            const int g = l * D + d;
            const size_t hb = (size_t)SLOTS * H * H * m->esize;
            packed.assign(hb, 0);
            rc = pack_matrix(weights[g * 4 + 1], true, 1, Hu, H, packed.data());
            if (rc == RNN_OK) rc = dev_alloc(m->whh[g], hb);
            if (rc == RNN_OK && hipMemcpy(m->whh[g].p, packed.data(), hb, hipMemcpyHostToDevice) != hipSuccess)
                rc = RNN_EDEVICE;
            m->weight_bytes += hb;
            if (rc != RNN_OK) break;
            // biases: LSTM folds b_ih + b_hh per gate; GRU keeps b_in and b_hn apart
            const size_t bb = (size_t)G * Hu * m->esize;
            std::vector<unsigned char> bi(bb, 0), bh(bb, 0);
            if (weights[g * 4 + 2]) {
                const unsigned char* s = fetch(weights[g * 4 + 2], bb);
                if (!s) { rc = RNN_EDEVICE; break; }
                memcpy(bi.data(), s, bb);
            }
            if (weights[g * 4 + 3]) {
                const unsigned char* s = fetch(weights[g * 4 + 3], bb);
                if (!s) { rc = RNN_EDEVICE; break; }
                memcpy(bh.data(), s, bb);
            }
            std::fill(bias_host.begin(), bias_host.end(), 0.0f);
            for (int u = 0; u < Hu; ++u)
                for (int sl = 0; sl < SLOTS; ++sl) {
                    const int ri = source_row(cell, false, Hu, u, sl, gate_order);
                    const int rh = source_row(cell, true, Hu, u, sl, gate_order);
                    float v = 0.0f;
                    if (ri >= 0) v += elem_to_f32(bi.data(), ri, dtype);
                    if (rh >= 0) v += elem_to_f32(bh.data(), rh, dtype);
                    bias_host[(size_t)u * SLOTS + sl] = v;
                }
            const size_t pb = bias_host.size() * sizeof(float);
            rc = dev_alloc(m->bias[g], pb);
            if (rc == RNN_OK && hipMemcpy(m->bias[g].p, bias_host.data(), pb, hipMemcpyHostToDevice) != hipSuccess)
                rc = RNN_EDEVICE;
            m->weight_bytes += pb;
        }
    }
    if (rc == RNN_OK) rc = dev_alloc(m->status, sizeof(unsigned));
    if (rc == RNN_OK && hipMemset(m->status.p, 0, sizeof(unsigned)) != hipSuccess) rc = RNN_EDEVICE;
    if (rc == RNN_OK && hipDeviceSynchronize() != hipSuccess) rc = RNN_EDEVICE;
    if (rc != RNN_OK) {
        (void)hipGetLastError();
        rnn_model_destroy(m);
        return rc;
    }
    *out = m;
    return RNN_OK;
}

void rnn_model_destroy(rnn_model* m) {
    if (!m) return;
    free_workspace(m);
    for (auto& b : m->wih) dev_free(b);
    for (auto& b : m->whh) dev_free(b);
    for (auto& b : m->bias) dev_free(b);
    for (auto& b : m->peep) dev_free(b);
    dev_free(m->status);
    for (auto& e : m->prof) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    delete m;
}

int rnn_model_set_plan(rnn_model* m, int plan) {
    if (!m) return RNN_EINVAL;
    if (plan != RNN_PLAN_AUTO && plan != RNN_PLAN_CELLWISE && plan != RNN_PLAN_WAVEFRONT)
        return RNN_EINVAL;
    if (plan == RNN_PLAN_WAVEFRONT) {
        Plan p;
        if (m->cellwise_only() || !choose_wavefront(m, 1, 1, p)) return RNN_EUNSUPPORTED;
    }
    m->requested_plan = plan;
    return RNN_OK;
}

int rnn_model_set_gru_reset_before(rnn_model* m, int on) {
    if (!m || (on != 0 && on != 1)) return RNN_EINVAL;
    if (m->cell != CELL_GRU) return on ? RNN_EUNSUPPORTED : RNN_OK;
    if (on && m->requested_plan == RNN_PLAN_WAVEFRONT) return RNN_EUNSUPPORTED;
    m->gru_reset_before = on != 0;
    return RNN_OK;
}

int rnn_model_set_clip(rnn_model* m, float clip) {
    if (!m || !(clip >= 0.0f) || !isfinite(clip)) return RNN_EINVAL;
    m->clip = clip;
    return RNN_OK;
}

int rnn_model_set_peepholes(rnn_model* m, const float* const* peepholes, int on_device) {
    if (!m) return RNN_EINVAL;
    if (!peepholes) {   // back to the plain cell
        if (!m->peep.empty()) HIP_TRY(hipDeviceSynchronize());   // no forward still reads them
        for (auto& b : m->peep) { m->weight_bytes -= b.bytes; dev_free(b); }
        m->peep.clear();
        return RNN_OK;
    }
    if (m->cell != CELL_LSTM) return RNN_EUNSUPPORTED;
    const size_t bytes = (size_t)3 * m->H * sizeof(float);
    std::vector<DevBuf> fresh((size_t)m->L * m->D);
    int rc = RNN_OK;
    for (size_t g = 0; g < fresh.size() && rc == RNN_OK; ++g) {
        rc = dev_alloc(fresh[g], bytes);
        if (rc != RNN_OK) break;
        hipError_t e = hipMemset(fresh[g].p, 0, bytes);   // added units: zero weights
        for (int k = 0; k < 3 && e == hipSuccess && peepholes[g]; ++k)
            e = hipMemcpy((float*)fresh[g].p + (size_t)k * m->H, peepholes[g] + (size_t)k * m->Hu,
                          (size_t)m->Hu * sizeof(float), on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice);
        if (e != hipSuccess) { (void)hipGetLastError(); rc = RNN_EDEVICE; }
    }
    if (rc == RNN_OK && hipDeviceSynchronize() != hipSuccess) rc = RNN_EDEVICE;   // also: no forward still reads the old ones
    if (rc != RNN_OK) {
        for (auto& b : fresh) dev_free(b);
        return rc;
    }
    for (auto& b : m->peep) { m->weight_bytes -= b.bytes; dev_free(b); }
    m->peep.swap(fresh);
    m->weight_bytes += bytes * m->peep.size();
    return RNN_OK;
}

int rnn_model_set_batch_first(rnn_model* m, int on) {
    if (!m || (on != 0 && on != 1)) return RNN_EINVAL;
    m->batch_first = on != 0;
    return RNN_OK;
}

int rnn_model_set_validation(rnn_model* m, int on) {
    if (!m || (on != 0 && on != 1)) return RNN_EINVAL;
    m->validate = on != 0;
    return RNN_OK;
}

int rnn_model_reserve(rnn_model* m, int T, int B) {
    if (!m || T < 1 || B < 1) return RNN_EINVAL;
    Plan plan;
    const int rc = resolve_plan(m, T, B, plan);
    if (rc != RNN_OK) return rc;
    return prepare_workspace(m, plan, T, B);
}

// rnn_forward and rnn_forward_static: the second with the workspace carved from the device's static array.
static int forward_entry(rnn_model* m, const void* x, const int32_t* lengths, const float* h0,
                         const float* c0, void* y, float* hT, float* cT, int T, int B, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    HIP_TRY(hipStreamIsCapturing(st, &capture));
    m->capturing = capture != hipStreamCaptureStatusNone;
    struct Done { rnn_model* m; ~Done() { m->capturing = false; } } done{m};
    if (m->validate && lengths) {
        if (m->capturing) return RNN_EUNSUPPORTED;
        std::vector<int32_t> host((size_t)B);
        HIP_TRY(hipMemcpyAsync(host.data(), lengths, (size_t)B * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        for (int b = 0; b < B; ++b)
            if (host[b] < 1 || host[b] > T) return RNN_EINVAL;
    }
    Plan plan;
    int rc = resolve_plan(m, T, B, plan);
    if (rc != RNN_OK) return rc;
    rc = prepare_workspace(m, plan, T, B);   // no-op when rnn_model_reserve has seen this shape and plan
    if (rc != RNN_OK) return rc;
    if (m->capturing) {
        // The launches recorded now carry the tags chosen now, and every replay runs them again with
        // the same tags: what the previous replay (or any other forward) left in the flag words and
        // the tagged state words must not be taken for this run's, so a replay starts by clearing them.
        HIP_TRY(launch_fill_zero(m->ws.flags.p, m->ws.flags.bytes, st));
        HIP_TRY(launch_fill_zero(m->ws.lseq.p, m->ws.lseq.bytes, st));
    }
    if (m->cell == CELL_GRU) { c0 = nullptr; cT = nullptr; }
    void* y_caller = nullptr;
    if (m->batch_first) {   // the plans work on time-major copies
        HIP_TRY(launch_swap_outer(x, m->ws.x_tm.p, B, T, (size_t)m->I * m->esize, st));
        x = m->ws.x_tm.p;
        y_caller = y;
        y = m->ws.y_tm.p;
    }
    const bool padded = m->H != m->Hu;
    void* y_plain = y;             // time-major output at the caller's width
    float* hT_caller = hT;
    float* cT_caller = cT;
    const size_t srow_u = (size_t)m->Hu * sizeof(float), srow = (size_t)m->H * sizeof(float);
    const int state_rows = m->L * m->D * B;
    if (padded) {                  // the plans work at the padded width: states in, y and states out
        y = m->ws.y_pad.p;
        if (h0) {
            HIP_TRY(launch_fill_zero(m->ws.st_pad[0].p, (size_t)state_rows * srow, st));
            HIP_TRY(launch_copy_2d(h0, srow_u, m->ws.st_pad[0].p, srow, state_rows, srow_u, st));
            h0 = (const float*)m->ws.st_pad[0].p;
        }
        if (c0) {
            HIP_TRY(launch_fill_zero(m->ws.st_pad[1].p, (size_t)state_rows * srow, st));
            HIP_TRY(launch_copy_2d(c0, srow_u, m->ws.st_pad[1].p, srow, state_rows, srow_u, st));
            c0 = (const float*)m->ws.st_pad[1].p;
        }
        if (hT) hT = (float*)m->ws.st_pad[2].p;
        if (cT) cT = (float*)m->ws.st_pad[3].p;
    }
    rc = plan.chunk > 0 ? forward_in_passes(m, plan, x, lengths, h0, c0, y, hT, cT, T, B, st)
                        : forward_one_pass(m, plan, x, lengths, h0, c0, y, hT, cT, T, B, st);
    if (rc != RNN_OK) return rc;
    if (padded) {
        const size_t yrow = (size_t)m->D * m->H * m->esize, yrow_u = (size_t)m->D * m->Hu * m->esize;
        for (int d = 0; d < m->D; ++d)
            HIP_TRY(launch_copy_2d((const char*)y + (size_t)d * m->H * m->esize, yrow,
                                   (char*)y_plain + (size_t)d * m->Hu * m->esize, yrow_u, T * B,
                                   (size_t)m->Hu * m->esize, st));
        if (hT_caller) HIP_TRY(launch_copy_2d(hT, srow, hT_caller, srow_u, state_rows, srow_u, st));
        if (cT_caller) HIP_TRY(launch_copy_2d(cT, srow, cT_caller, srow_u, state_rows, srow_u, st));
    }
    if (m->batch_first)
        HIP_TRY(launch_swap_outer(y_plain, y_caller, T, B, (size_t)m->D * m->Hu * m->esize, st));
    return RNN_OK;
}

int rnn_forward(rnn_model* m, const void* x, const int32_t* lengths, const float* h0,
                const float* c0, void* y, float* hT, float* cT, int T, int B, void* stream) {
    if (!m || !x || !y || T < 1 || B < 1) return RNN_EINVAL;
    if (((uintptr_t)x | (uintptr_t)y) & 15) return RNN_EINVAL;
    if ((size_t)T * B > ((size_t)1 << 30)) return RNN_EUNSUPPORTED;
    return forward_entry(m, x, lengths, h0, c0, y, hT, cT, T, B, stream);
}

int rnn_forward_static(rnn_model* m, const void* x, const int32_t* lengths, const float* h0,
                       const float* c0, void* y, float* hT, float* cT, int T, int B, void* stream) {
    if (!m || !x || !y || T < 1 || B < 1) return RNN_EINVAL;
    if (((uintptr_t)x | (uintptr_t)y) & 15) return RNN_EINVAL;
    if ((size_t)T * B > ((size_t)1 << 30)) return RNN_EUNSUPPORTED;
    if (!m->scratch) return RNN_EDEVICE;    // the device's static array could not be looked up at create
    // For the length of this call the model's workspace is a set of empty buffers that grow() fills with
    // pieces of the static array; the model's own workspace is put back untouched afterwards.
    std::swap(m->ws, m->ws_static);
    for (auto& b : m->ws.ybuf) b = DevBuf();
    {
        std::vector<DevBuf> keep;
        keep.swap(m->ws.ybuf);              // no reallocation: the vector keeps its L-1 entries
        m->ws = rnn_model::Workspace();
        m->ws.ybuf.swap(keep);
    }
    m->arena.base = m->scratch;
    m->arena.used = 0;
    m->arena.stream = (hipStream_t)stream;
    m->arena.on = true;
    const int rc = forward_entry(m, x, lengths, h0, c0, y, hT, cT, T, B, stream);
    m->arena.on = false;
    std::swap(m->ws, m->ws_static);
    return rc;
}

int rnn_input_projection(rnn_model* m, int layer, const void* in, float* gx, int rows,
                         void* stream) {
    if (!m || !in || !gx || rows < 1 || layer < 0 || layer >= m->L) return RNN_EINVAL;
    if (m->H != m->Hu) return RNN_EUNSUPPORTED;   // a padded model has no projection in the caller's layout
    const int K = m->layer_input(layer);
    const int N = m->D * SLOTS * m->H;
    HIP_TRY(launch_gemm_nt(m->dtype, in, K, m->wih[layer].p, K, gx, N, rows, N, K,
                           (hipStream_t)stream));
    return RNN_OK;
}

int rnn_model_set_profiling(rnn_model* m, int flags) {
    if (!m || flags < 0 || flags > 3) return RNN_EINVAL;
    m->profiling = (flags & RNN_PROFILE_KERNELS) != 0;
    m->want_ticks = (flags & RNN_PROFILE_STEP_TICKS) != 0;
    m->prof_used = 0;
    return RNN_OK;
}

int rnn_model_profile_read(rnn_model* m, int kind, double* total_ms, long long* launches) {
    if (!m || !total_ms || !launches) return RNN_EINVAL;
    if (kind != RNN_KERNEL_PROJECTION && kind != RNN_KERNEL_RECURRENT) return RNN_EINVAL;
    double sum = 0.0;
    long long n = 0;
    for (size_t i = 0; i < m->prof_used; ++i) {
        if (m->prof[i].kind != kind) continue;
        float ms = 0.0f;
        HIP_TRY(hipEventSynchronize(m->prof[i].b));
        HIP_TRY(hipEventElapsedTime(&ms, m->prof[i].a, m->prof[i].b));
        sum += ms;
        ++n;
    }
    *total_ms = sum;
    *launches = n;
    return RNN_OK;
}

int rnn_model_read_step_ticks(rnn_model* m, uint64_t* ticks, size_t count) {
    if (!m || !ticks) return RNN_EINVAL;
    if (!m->ws.ticks.p || count * sizeof(uint64_t) > m->ws.ticks.bytes) return RNN_EINVAL;
    HIP_TRY(hipMemcpy(ticks, m->ws.ticks.p, count * sizeof(uint64_t), hipMemcpyDeviceToHost));
    return RNN_OK;
}

int rnn_model_check(rnn_model* m) {
    if (!m) return RNN_EINVAL;
    unsigned st = 0;
    HIP_TRY(hipMemcpy(&st, m->status.p, sizeof(st), hipMemcpyDeviceToHost));
    if (st == 0) return RNN_OK;
    // the word is only ever raised by the kernels: lower it, so that the next forward runs normally
    HIP_TRY(hipMemset(m->status.p, 0, sizeof(unsigned)));
    return RNN_EDEVICE;
}

int rnn_model_set_spin_limit(rnn_model* m, unsigned polls) {
    if (!m) return RNN_EINVAL;
    m->spin_limit = polls == 0 ? DEFAULT_SPIN_LIMIT : polls;
    return RNN_OK;
}

int rnn_model_set_launch_tag(rnn_model* m, uint32_t tag) {
    if (!m) return RNN_EINVAL;
    HIP_TRY(hipDeviceSynchronize());
    if (m->ws.lseq.p) HIP_TRY(hipMemset(m->ws.lseq.p, 0, m->ws.lseq.bytes));
    if (m->ws.flags.p) HIP_TRY(hipMemset(m->ws.flags.p, 0, m->ws.flags.bytes));
    HIP_TRY(hipDeviceSynchronize());
    m->epoch = tag;
    return RNN_OK;
}

int rnn_model_input_product_placement(const rnn_model* m, int T, int B, int layer, int* separate_launch) {
    if (!m || !separate_launch || T < 1 || B < 1 || layer < 0 || layer >= m->L) return RNN_EINVAL;
    Plan plan;
    const int rc = resolve_plan(m, T, B, plan);
    if (rc != RNN_OK) return rc;
    if (plan.kind != RNN_PLAN_WAVEFRONT) *separate_launch = 1;
    else if (input_product_inside(m, plan, layer, T)) *separate_launch = 0;
    else *separate_launch = first_of_launch(m, plan, layer) ? 1 : 0;  // layers above the first of a launch are fused
    return RNN_OK;
}

int rnn_plan_query(int cell, int num_layers, int input_size, int hidden_size, int num_directions, int dtype,
                   int requested_plan, int T, int B, int compute_units, size_t lds_bytes, int* plan_out,
                   int* separate_projection) {
    if (!plan_out || T < 1 || B < 1 || compute_units < 1) return RNN_EINVAL;
    if (requested_plan != RNN_PLAN_AUTO && requested_plan != RNN_PLAN_CELLWISE && requested_plan != RNN_PLAN_WAVEFRONT)
        return RNN_EINVAL;
    int rc = check_model_shape(cell, num_layers, input_size, hidden_size, num_directions, dtype);
    if (rc != RNN_OK) return rc;
    rnn_model m;   // shape and device figures only: no buffer is touched
    m.cell = cell; m.L = num_layers; m.I = input_size; m.Hu = hidden_size; m.H = padded_width(dtype, hidden_size);
    m.D = num_directions; m.dtype = dtype;
    m.esize = (dtype == RNN_BF16) ? 2 : 4;
    m.num_cus = compute_units;
    m.lds_limit = lds_bytes;
    m.requested_plan = requested_plan;
    Plan plan;
    rc = resolve_plan(&m, T, B, plan);
    if (rc != RNN_OK) return rc;
    const bool wavefront = plan.kind == RNN_PLAN_WAVEFRONT;
    plan_out[0] = plan.kind;
    plan_out[1] = wavefront ? plan.LP : 1;
    plan_out[2] = wavefront ? plan.RT : 0;
    plan_out[3] = wavefront ? plan.CT : 0;
    plan_out[4] = wavefront ? plan.NCH : 0;
    plan_out[5] = wavefront ? plan.nrb : 0;
    plan_out[6] = wavefront ? plan.ncb : 0;
    plan_out[7] = wavefront ? launch_count(&m, plan) * (plan.chunk > 0 ? (B + plan.chunk - 1) / plan.chunk : 1) : num_layers;
    if (separate_projection)
        for (int l = 0; l < num_layers; ++l)
            separate_projection[l] = !wavefront ? 1 : input_product_inside(&m, plan, l, T) ? 0 : first_of_launch(&m, plan, l) ? 1 : 0;
    return RNN_OK;
}

int rnn_plan_launches(int cell, int num_layers, int input_size, int hidden_size, int num_directions, int dtype,
                      int requested_plan, int T, int B, int compute_units, size_t lds_bytes, int* layer_launch,
                      int* layer_group) {
    if (!layer_launch || T < 1 || B < 1 || compute_units < 1) return RNN_EINVAL;
    if (requested_plan != RNN_PLAN_AUTO && requested_plan != RNN_PLAN_CELLWISE && requested_plan != RNN_PLAN_WAVEFRONT)
        return RNN_EINVAL;
    int rc = check_model_shape(cell, num_layers, input_size, hidden_size, num_directions, dtype);
    if (rc != RNN_OK) return rc;
    rnn_model m;   // shape and device figures only: no buffer is touched
    m.cell = cell; m.L = num_layers; m.I = input_size; m.Hu = hidden_size; m.H = padded_width(dtype, hidden_size);
    m.D = num_directions; m.dtype = dtype;
    m.esize = (dtype == RNN_BF16) ? 2 : 4;
    m.num_cus = compute_units;
    m.lds_limit = lds_bytes;
    m.requested_plan = requested_plan;
    Plan plan;
    rc = resolve_plan(&m, T, B, plan);
    if (rc != RNN_OK) return rc;
    for (int l = 0; l < num_layers; ++l) {
        int l0, n;
        launch_of(&m, plan, l, l0, n);
        layer_launch[l] = launch_index(plan, l);
        if (layer_group)
            for (int d = 0; d < num_directions; ++d) layer_group[l * num_directions + d] = (l - l0) * num_directions + d;
    }
    return RNN_OK;
}

size_t rnn_model_device_bytes(const rnn_model* m) {
    if (!m) return 0;
    return m->weight_bytes + m->workspace_bytes + sizeof(unsigned);
}

const char* rnn_status_string(int status) {
    switch (status) {
        case RNN_OK: return "ok";
        case RNN_EINVAL: return "invalid argument";
        case RNN_EUNSUPPORTED: return "unsupported shape or plan";
        case RNN_ENOMEM: return "out of memory";
        case RNN_EDEVICE: return "device error";
        case RNN_ESCRATCH: return "shape needs more workspace than the static scratch array holds";
        default: return "unknown status";
    }
}

}  // extern "C"
