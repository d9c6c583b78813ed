/*
 * rnn.h - C ABI of the MI355X (gfx950) stacked-RNN forward library.
 *
 * The operation.  A stacked recurrent network is unrolled over layers and time steps into a
 * grid of cell operators A_t^l; cell (l, t) may run as soon as cell (l, t-1) and cell (l-1, t)
 * have finished, so cells on one anti-diagonal are independent (paper: Section 1, where the
 * unrolled network is said to be parallel across layers and across time steps; Section 2.2,
 * figure of the folded and unfolded RNN).  Where the paper runs independent cells on CPU cores next to a
 * GPU that executes cells one by one, this library runs the whole grid inside one persistent
 * GPU kernel whose workgroups are split into one group per (layer, direction).
 *
 * The paper names the cell (LSTM) but prints no equations; this library uses the standard ones:
 *   LSTM  a = W_ih x_t + b_ih + W_hh h_{t-1} + b_hh  (row blocks i, f, g, o)
 *         c_t = sigma(a_f) c_{t-1} + sigma(a_i) tanh(a_g);   h_t = sigma(a_o) tanh(c_t)
 *   GRU   r = sigma(W_ir x + b_ir + W_hr h + b_hr),  z likewise        (row blocks r, z, n)
 *         n = tanh(W_in x + b_in + r (W_hn h + b_hn));   h_t = (1 - z) n + z h_{t-1}
 * Layer l >= 1 reads the concatenation [forward, backward] of layer l-1.  The forward
 * direction visits t = 0 .. len-1, the backward direction t = len-1 .. 0 of each sequence.
 *
 * Conventions for every entry point:
 *   - no C++ or framework types cross this boundary: plain pointers, ints and sizes;
 *   - "device pointer" means memory of the current HIP device, "host pointer" ordinary memory;
 *   - every function returning int returns an rnn_status; nothing throws; on failure outputs
 *     passed by pointer are left untouched;
 *   - a model belongs to the HIP device that was current when it was created, and at most one
 *     rnn_forward may be in flight per model (its workspace and step flags are per model);
 *   - what may run beside a forward pass.  The persistent kernels (RNN_PLAN_WAVEFRONT) size their grid for a GPU
 *     that is otherwise idle: every workgroup of a launch has to be resident at the same time, because workgroups
 *     wait for one another's steps.  Other kernels on other streams of the same GPU (another model's forward pass,
 *     the caller's own kernels, another process) can take compute units away and leave part of a launch
 *     unscheduled until they finish; the launch then makes no progress meanwhile.  It cannot hang for good: every
 *     wait inside the kernels is bounded (rnn_model_set_spin_limit), a launch whose waits run out drains, its
 *     outputs are undefined and rnn_model_check reports RNN_EDEVICE.  So: run forward passes of different models
 *     one after another (one stream, or ordered streams) when latency matters, and call rnn_model_check where a
 *     stall must be noticed.  Copies (hipMemcpyAsync) and kernels of the cellwise plan beside a forward pass are
 *     harmless;
 *   - the one-time set-up of a kernel variant (its LDS size, how many workgroups fit the GPU) is kept per
 *     process: calls into the library are made from one thread at a time, and the GPUs of a process are
 *     of one kind.
 */
#ifndef RNN_MI355X_H
#define RNN_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rnn_model rnn_model; /* opaque; created and destroyed by the library */

enum rnn_cell { RNN_LSTM = 0, RNN_GRU = 1 };

/* Storage type of x, y, the weights and the activations handed from layer to layer.
 * Accumulation, gate arithmetic, the cell state and h0/c0/hT/cT are always fp32.
 * With RNN_BF16 every h_t is rounded to bf16 (nearest even) when it is produced; that rounded
 * value is what the next step, the next layer, y and hT see. */
enum rnn_dtype { RNN_F32 = 0, RNN_BF16 = 1 };

enum rnn_status {
    RNN_OK = 0,
    RNN_EINVAL = 1,       /* NULL where a pointer is required, size <= 0, bad enum value */
    RNN_EUNSUPPORTED = 2, /* shape outside what the kernels support (see rnn_model_create) */
    RNN_ENOMEM = 3,       /* host or device allocation failed */
    RNN_EDEVICE = 4,      /* a HIP call failed, or a previous forward reported a stalled step */
    RNN_ESCRATCH = 5      /* rnn_forward_static: the shape needs more workspace than the static array holds */
};

/* How the cell grid is executed.
 *   RNN_PLAN_AUTO       wavefront when the shape allows it, otherwise cellwise.
 *   RNN_PLAN_CELLWISE   one launch sequence per cell, cells strictly one after another on the
 *                       stream: the single-GPU regime the paper describes in the caption of its
 *                       unfolded-RNN figure.  Kept as the reference path and as a baseline.
 *   RNN_PLAN_WAVEFRONT  one persistent kernel; workgroup groups per (layer, direction) advance
 *                       along anti-diagonals of the grid, synchronised by device-scope flags. */
enum rnn_plan { RNN_PLAN_AUTO = 0, RNN_PLAN_CELLWISE = 1, RNN_PLAN_WAVEFRONT = 2 };

/*
 * Create a model (paper, Section 1 / Section 4.1: the input of the system is a trained model).
 *   out                receives the handle.
 *   cell               rnn_cell.
 *   num_layers         L >= 1.
 *   input_size         I >= 1, width of x.
 *   hidden_size        H >= 1.
 *   num_directions     D = 1 or 2.
 *   dtype              rnn_dtype of the weights, x and y.
 *   weights            host array of L*D*4 pointers in order (l, d, {W_ih, W_hh, b_ih, b_hh}).
 *                      W_ih[l,d] is [G*H, I_l] row-major with I_0 = I and I_l = D*H for l >= 1;
 *                      W_hh[l,d] is [G*H, H] row-major; b_* are [G*H]; G = 4 (LSTM, row blocks
 *                      i,f,g,o) or 3 (GRU, row blocks r,z,n).  Elements have type `dtype`
 *                      (bf16 = the upper 16 bits of an IEEE float).  A NULL bias means zeros.
 *   weights_on_device  0: the pointed-to arrays are host memory; 1: device memory.
 * The library copies and repacks the weights; the caller keeps ownership of its arrays and may
 * free them when the call returns.  The call synchronises the device.
 * Supported shapes: hidden_size a multiple of 4 for RNN_F32 and a multiple of 8 for RNN_BF16,
 * input_size a multiple of 8 for RNN_BF16; otherwise RNN_EUNSUPPORTED.
 * The persistent kernels exist for certain hidden sizes (bf16: 128 x {1, 2, 3, 4, 5, 6, 8, 10, 12, 16};
 * fp32: 16 x {2, 4, 8, 16, 32}).  A model of another hidden size below the largest of them is held and run at
 * the next such size: the added units have zero weights, zero biases and a zero initial state, stay at zero
 * and reach nothing, and y, hT, cT are returned at the caller's size; rnn_model_device_bytes counts the padded
 * weights.  Larger models run one cell at a time (the cellwise plan).
 */
int rnn_model_create(rnn_model** out, int cell, int num_layers, int input_size, int hidden_size,
                     int num_directions, int dtype, const void* const* weights,
                     int weights_on_device);

/* Order of the gate row blocks inside the caller's W_ih, W_hh and bias arrays.
 *   RNN_ORDER_IFGO_RZN  LSTM i,f,g,o; GRU r,z,n (what rnn_model_create assumes).
 *   RNN_ORDER_ONNX      LSTM i,o,f,c; GRU z,r,h: the order of the ONNX operator set, the file
 *                       format the paper's system takes its models in (Section 1; Section 4.1). */
enum rnn_gate_order { RNN_ORDER_IFGO_RZN = 0, RNN_ORDER_ONNX = 1 };

/* rnn_model_create for weights whose gate row blocks are in `gate_order` (rnn_gate_order); every
 * other argument, the array list (l, d, {W_ih, W_hh, b_ih, b_hh}) and the error behaviour are those
 * of rnn_model_create.  Only the order of the row blocks differs; the GRU computed is the same
 * (reset gate applied after the recurrent product).  RNN_EINVAL for an unknown order. */
int rnn_model_create_ordered(rnn_model** out, int cell, int num_layers, int input_size, int hidden_size,
                             int num_directions, int dtype, const void* const* weights,
                             int weights_on_device, int gate_order);

/* Free the model, its device weights and its workspace.  NULL is accepted.  The caller must
 * have synchronised any stream that still runs a forward of this model. */
void rnn_model_destroy(rnn_model* model);

/* Choose the execution plan (rnn_plan) for later forwards.  RNN_EUNSUPPORTED when the model's
 * shape cannot run under that plan. */
int rnn_model_set_plan(rnn_model* model, int plan);

/* GRU only: on = 1 selects the GRU that applies the reset gate before the candidate's recurrent
 * product, n = tanh(W_in x + b_in + W_hn (r * h) + b_hn), the default of the ONNX operator set
 * (the file format the paper's system takes its models in, Section 1); on = 0 (the default)
 * applies it after the product, n = tanh(W_in x + b_in + r * (W_hn h + b_hn)).  The first form
 * needs two dependent recurrent products per cell and runs under the cellwise plan only:
 * RNN_EUNSUPPORTED for an LSTM model or while RNN_PLAN_WAVEFRONT is selected (and selecting that
 * plan afterwards is refused). */
int rnn_model_set_gru_reset_before(rnn_model* model, int on);

/* The two optional terms that the ONNX LSTM / GRU operators (the format of the models the paper's
 * system ingests, Section 1 and Section 4.1) add to the plain cell.  Both are part of the gate
 * arithmetic of every plan (the persistent kernels keep a unit's three peephole weights and the
 * threshold in registers beside its bias).  Either call takes effect with the next forward; no forward
 * of the model may be in flight.
 *
 * Clipping threshold: clip > 0 limits the argument of every gate activation (i, f, g, o including
 * their peephole terms; r, z and the whole argument of n) to [-clip, +clip]; the cell state inside
 * h = o * tanh(c) is not limited.  clip = 0 (the default) switches it off; negative or non-finite
 * values are RNN_EINVAL. */
int rnn_model_set_clip(rnn_model* model, float clip);

/* Peephole weights, LSTM only (RNN_EUNSUPPORTED for a GRU): i = sigma(a_i + p_i * c_{t-1}),
 * f = sigma(a_f + p_f * c_{t-1}), o = sigma(a_o + p_o * c_t).  peepholes: L*D pointers in order
 * (layer, direction), each to 3*H fp32 values (p_i, p_f, p_o: H values each) in host memory, or in
 * device memory when on_device != 0; a NULL entry means zeros.  The library copies them; the call
 * waits for the device.  peepholes = NULL removes them (the plain cell again). */
int rnn_model_set_peepholes(rnn_model* model, const float* const* peepholes, int on_device);

/* on = 1: rnn_forward takes x as [B, T, I] and writes y as [B, T, D*H] (padded positions of a
 * sequence still +0.0); the state tensors keep their layout.  Every plan works on time-major
 * copies kept in the workspace, so this costs one more pass over x and y.  on = 0 (the default):
 * time-major, as described at rnn_forward.  rnn_input_projection is not affected. */
int rnn_model_set_batch_first(rnn_model* model, int on);

/* Debug validation of the inputs of rnn_forward / rnn_forward_static.  on = 1: every call first copies `lengths`
 * to the host (waiting for `stream`) and returns RNN_EINVAL, with nothing enqueued, unless 1 <= lengths[b] <= T
 * for every sequence; such a call cannot be recorded into a HIP graph (RNN_EUNSUPPORTED while the stream is
 * capturing).  on = 0 (the default): no check on the host, out-of-range values are clamped on the device. */
int rnn_model_set_validation(rnn_model* model, int on);

/* Size the workspace now for forwards of T steps and B sequences under the current plan, so that
 * later rnn_forward calls of that shape allocate nothing.  Only what the plan chosen for (T, B)
 * touches is allocated (the paper's memory model, Section 3, Equation 4, counts exactly such
 * temporaries); a call of another shape may be given another plan and then grows the workspace
 * itself.  Buffers never shrink.  May synchronise the device. */
int rnn_model_reserve(rnn_model* model, int T, int B);

/*
 * Run the forward pass of the whole cell grid (Section 2.2, unfolded-RNN figure; Section 3,
 * the computation graph G = (V, E) whose vertices here are the cells).
 * All tensors are contiguous, time-major DEVICE pointers owned by the caller:
 *   x        [T, B, I]      dtype     input
 *   lengths  [B]            int32     valid steps per sequence, 1 <= lengths[b] <= T; NULL = all T.
 *                                      Values outside the range are clamped to [0, T] on the device (a sequence
 *                                      of length 0 keeps its initial state and gets +0.0 everywhere); with
 *                                      rnn_model_set_validation(model, 1) they are RNN_EINVAL instead.
 *   h0, c0   [L*D, B, H]    fp32      initial state, row l*D+d; NULL = zeros; c0 unused for GRU
 *   y        [T, B, D*H]    dtype     output of the last layer; positions t >= lengths[b] receive
 *                                      +0.0 (all-zero bits)
 *   hT, cT   [L*D, B, H]    fp32      state after the last valid step of each sequence in each
 *                                      direction; either may be NULL; cT unused for GRU
 *   T, B                               steps and sequences in this call (>= 1)
 *   stream                             hipStream_t passed as void* (NULL = the default stream)
 * The call enqueues work on `stream` and returns without waiting; outputs are valid once the
 * stream has reached the end of that work.  It allocates device memory only if this shape needs
 * more workspace than earlier calls or rnn_model_reserve provided (then it synchronises).
 * x and y must not overlap and must be 16-byte aligned (RNN_EINVAL otherwise: the kernels read and
 * write them in 16-byte pieces).  Inputs are not validated on the device beyond the clamping above.
 * A batch that no single persistent launch can hold (for example more than 256 sequences at 1024 units)
 * is run in passes over blocks of sequences, through copies in the workspace; results are the same.
 * Stream capture: the call may be recorded into a HIP graph (`stream` in capture mode) provided the
 * workspace already covers the shape (rnn_model_reserve, or an earlier call; RNN_EUNSUPPORTED
 * otherwise, with nothing recorded): it then records kernels only, the first of which clear the
 * model's step flags, because every replay reuses the tags chosen at capture time.  A replay counts
 * as a forward in flight (one at a time per model), the pointers recorded are the ones passed here,
 * and kernel timing (rnn_model_set_profiling) is not recorded.
 */
int rnn_forward(rnn_model* model, const void* x, const int32_t* lengths, const float* h0,
                const float* c0, void* y, float* hT, float* cT, int T, int B, void* stream);

/*
 * rnn_forward for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as rnn_forward, but
 * the call allocates and frees nothing, whatever shape it is given: its workspace (tagged state words, step
 * flags, inter-layer activations, projection and layout copies: everything rnn_forward keeps in the model's
 * own workspace) is laid out, per call, in one static device array of RNN_STATIC_SCRATCH_MIB mebibytes that
 * every GPU the library runs on holds from the first rnn_model_create on it until the process ends.
 *   - A shape whose plan needs more than that returns RNN_ESCRATCH with nothing enqueued (for example C3 of the
 *     named workloads needs about 3 MiB, a 2-layer bidirectional model of 512 units on 64 sequences of 256 steps
 *     about 140 MiB); RNN_EDEVICE if the array's address could not be obtained when the model was created.
 *   - All models of a device share the array, which keeps what the last call left: the call clears, on
 *     `stream`, the parts that must start at zero (step flags, tagged words).  Two calls that overlap in time
 *     on one GPU (different streams or different models) race on it and give undefined results; calls on one
 *     stream, or otherwise ordered, are fine.  It does not touch the workspace rnn_forward uses, so the two
 *     entry points may be mixed on one model (still one forward in flight per model).
 *   - Kernel timing (rnn_model_set_profiling) records only into event pairs that earlier rnn_forward calls
 *     created; otherwise the call goes untimed.
 */
#define RNN_STATIC_SCRATCH_MIB 64
int rnn_forward_static(rnn_model* model, const void* x, const int32_t* lengths, const float* h0,
                       const float* c0, void* y, float* hT, float* cT, int T, int B, void* stream);

/*
 * The input projection alone, for all time steps at once (the step that does not depend on the
 * recurrence: cell (l, t) consumes x_t, Section 2.2): for layer `layer`, all directions,
 *   gx[row, d, u, s] = sum_k in[row, k] * W_ih[l, d][s-th gate row of unit u, k]
 * in (DEVICE, [rows, I_l], dtype, row-major) -> gx (DEVICE, [rows, D, H, 4], fp32).
 * Slot s is i,f,g,o for LSTM and r,z,n,(zero) for GRU.  No bias is added.  Asynchronous on
 * `stream`.  Exposed so the projection can be tested and measured on its own.
 * RNN_EUNSUPPORTED for a model that runs at a padded width (see rnn_model_create): it has no projection
 * in the caller's layout.
 */
int rnn_input_projection(rnn_model* model, int layer, const void* in, float* gx, int rows,
                         void* stream);

/* Kernel classes for profiling. */
enum rnn_kernel { RNN_KERNEL_PROJECTION = 0, RNN_KERNEL_RECURRENT = 1 };
enum rnn_profile_flags { RNN_PROFILE_KERNELS = 1, RNN_PROFILE_STEP_TICKS = 2 };

/* Measurement aids for the two kernels that dominate the forward pass (projection over all
 * time steps; persistent recurrent kernel), the quantities the paper's profiler collects per
 * operator (Section 4.1: the model is profiled first, to obtain every operator's run time).
 *   flags & RNN_PROFILE_KERNELS     later forwards bracket every projection and every persistent
 *                                   launch with HIP events on the caller's stream;
 *   flags & RNN_PROFILE_STEP_TICKS  the persistent kernel stores the device wall clock (100 MHz)
 *                                   at which each (layer, direction, step) was published.
 * Calling it (with any flags, 0 = off) also discards the events recorded so far. */
int rnn_model_set_profiling(rnn_model* model, int flags);

/* After the caller has synchronised the stream: total milliseconds and number of launches of
 * kernel class `kind` (rnn_kernel) recorded since the last rnn_model_set_profiling.  Host pointers. */
int rnn_model_profile_read(rnn_model* model, int kind, double* total_ms, long long* launches);

/* After the caller has synchronised the stream: copy the step clocks of the last persistent
 * forward to host memory, `count` = L*D*T values in order (layer, direction, step s); the
 * backward direction's step s is time T-1-s. */
int rnn_model_read_step_ticks(rnn_model* model, uint64_t* ticks, size_t count);

/* After the stream has been synchronised: RNN_OK, or RNN_EDEVICE if a workgroup of a persistent
 * forward since the last check gave up waiting for another workgroup's step (the outputs of that
 * forward are then undefined).  The condition is latched on the device: while it stands, every wait
 * of a later forward gives up early as well, and this call lowers it again, so the forward after an
 * RNN_EDEVICE answer runs normally. */
int rnn_model_check(rnn_model* model);

/* Every wait inside the persistent kernels is bounded: a wave that has polled `polls` times without
 * success stops waiting, raises the condition that rnn_model_check reports, and runs on to the end of
 * the launch without waiting again (so the launch always drains).  The kernels read the budget only now
 * and then (every 64 to 1024 polls of a wait; where a layer waits for the layer below it, and in the
 * kernel for small batches, also after the first 8), so the value is rounded up to the next such
 * moment.  polls = 0 restores the default, about three seconds.  A tiny value makes healthy launches
 * of several layers give up, because an upper layer waits at the start of a launch for the layers below
 * it to get going; tests of the give-up path use that. */
int rnn_model_set_spin_limit(rnn_model* model, unsigned polls);

/* Test aid.  Every persistent launch stamps its step flags and tagged state words with a 32-bit tag, one more
 * than the launch before; after 2^32 launches of a model the tag wraps, and the launch that wraps first clears
 * those buffers (tag 0 means "never written").  This call sets the tag of the most recent launch to `tag`, so a
 * test reaches the wrap with the next launches instead of after 2^32; it waits for the device and clears the
 * flag and tagged-word buffers of the model's own workspace, so no earlier launch's tags can be met again. */
int rnn_model_set_launch_tag(rnn_model* model, uint32_t tag);

/* Where the input product W_ih x_t of `layer` is computed for a forward pass of T steps and B
 * sequences under the current plan: *separate_launch = 1 when it is a projection launch of its own
 * (RNN_KERNEL_PROJECTION: the product over all steps, hoisted out of the cell), 0 when it runs
 * inside the recurrent kernel (RNN_KERNEL_RECURRENT), cell by cell, beside the recurrent product
 * (the paper's cell, Section 2.2, takes x_t and h_{t-1} together).  Host only, no device work;
 * measurement code uses it to attribute the product's flops to the kernel that performs them.
 * RNN_EINVAL on a bad handle, layer, size or a NULL result pointer. */
int rnn_model_input_product_placement(const rnn_model* model, int T, int B, int layer,
                                      int* separate_launch);

/* Bytes of device memory the model currently holds: repacked weights plus workspace
 * (the quantity the paper's memory model sums per operator, Section 3, Equation 4). */
size_t rnn_model_device_bytes(const rnn_model* model);

/*
 * How the library would lay the cell grid (Section 2.2) of a model of this shape over a GPU with
 * `compute_units` compute units and `lds_bytes` of LDS per workgroup, for calls of T steps and B
 * sequences.  Pure host code: no model, no device and no GPU are needed (all pointers are HOST
 * pointers owned by the caller).  requested_plan as in rnn_model_set_plan.
 *   plan[8]: resolved plan (RNN_PLAN_CELLWISE or RNN_PLAN_WAVEFRONT), layers per launch, then for
 *            the persistent kernels the workgroup tile (16-row tiles, 16-sequence column tiles per
 *            chain, chains per workgroup), row blocks, chains (column blocks) and the number of
 *            recurrent launches per forward pass; zeros where the cellwise plan has no such figure.
 *            A batch larger than one persistent launch can hold runs in passes over blocks of
 *            sequences (they do not interact): the figures then describe one full pass (its row and
 *            column blocks say how many sequences: 16 * column tiles * chains), and the launch count
 *            covers all passes.
 *   separate_projection[num_layers] (may be NULL): 1 where W_ih x_t of that layer is a projection
 *            launch of its own, 0 where it is computed inside the recurrent kernel.
 * Returns RNN_EINVAL / RNN_EUNSUPPORTED for the shapes rnn_model_create rejects and for a requested
 * plan the shape cannot run under.
 */
int rnn_plan_query(int cell, int num_layers, int input_size, int hidden_size, int num_directions,
                   int dtype, int requested_plan, int T, int B, int compute_units, size_t lds_bytes,
                   int* plan, int* separate_projection);

/*
 * A stacked RNN whose layers have different hidden sizes (Section 2.2: a layer takes the output sequence of the layer
 * below as its input; nothing else ties their widths).  Consecutive layers of one hidden size form a run; every run
 * is an rnn_model of its own, padded to a kernel width, planned by the scheduler and launched on its own, and the
 * runs follow one another on the stream, each reading the output of the one before it from a buffer the stack owns.
 *   hidden_sizes[num_layers]   H_l >= 1, each as rnn_model_create accepts it
 *   weights                    as for rnn_model_create: L*D*4 host pointers in order (l, d, {W_ih, W_hh, b_ih, b_hh}),
 *                              W_ih[l,d] [G*H_l, I_l] with I_0 = input_size and I_l = D*H_{l-1}, W_hh[l,d] [G*H_l, H_l]
 * Errors as rnn_model_create (the first failing run decides); nothing is left allocated on failure.
 */
typedef struct rnn_stack rnn_stack;
int rnn_stack_create(rnn_stack** out, int cell, int num_layers, int input_size, const int* hidden_sizes,
                     int num_directions, int dtype, const void* const* weights, int weights_on_device);
/* Free the stack, its models and buffers.  NULL is accepted; streams that run it must have been synchronised. */
void rnn_stack_destroy(rnn_stack* stack);
/* Number of runs, and one run: its first layer, number of layers, hidden size and model (any result pointer may be
 * NULL).  The model stays owned by the stack; the per-model settings (rnn_model_set_plan, _set_clip, ...) apply to it. */
int rnn_stack_runs(const rnn_stack* stack);
int rnn_stack_run(const rnn_stack* stack, int run, int* first_layer, int* num_layers, int* hidden_size,
                  rnn_model** model);
/* Device bytes of all runs plus the buffers between them. */
size_t rnn_stack_device_bytes(const rnn_stack* stack);
/* rnn_forward through all runs.  x [T, B, I] and y [T, B, D*H_last] as there (DEVICE pointers, dtype).  h0, c0, hT,
 * cT: NULL, or HOST arrays of one DEVICE pointer per run (entries may be NULL), each [layers of the run * D, B, H of
 * the run] fp32.  The buffers between runs grow on demand (then the call synchronises the device; RNN_EUNSUPPORTED
 * instead while `stream` is being captured).  One forward in flight per stack. */
int rnn_stack_forward(rnn_stack* stack, const void* x, const int32_t* lengths, const float* const* h0,
                      const float* const* c0, void* y, float* const* hT, float* const* cT, int T, int B,
                      void* stream);

/* Which launch of a forward pass holds which layer (launches numbered in stream order), and which group of
 * workgroups of that launch runs which (layer, direction), for the plan rnn_plan_query reports for the same
 * arguments.  The split is the scheduler's: the cell grid (Section 2.2) sorted by the topological sorting of Section
 * 4.1 and placed by the list scheduling of Section 3 on as many processors as a launch has room for groups, each
 * processor holding the weights of one (layer, direction) per pass (rnn_schedule_place_resident); a pass is a
 * launch.  Under the cellwise plan every layer is a launch of its own.  Pure host code; HOST pointers:
 * layer_launch[num_layers], layer_group[num_layers * num_directions] (may be NULL).  Errors as rnn_plan_query. */
int rnn_plan_launches(int cell, int num_layers, int input_size, int hidden_size, int num_directions,
                      int dtype, int requested_plan, int T, int B, int compute_units, size_t lds_bytes,
                      int* layer_launch, int* layer_group);

/*
 * Measurement aid, no part of the forward pass: the rate at which `compute_units` workgroups (one per compute
 * unit, one wave per SIMD, 16 independent accumulators per wave) issue dense 32 x 32 x 16 bf16 matrix instructions
 * and nothing else, for `iterations` rounds of 64 instructions per wave, after one untimed pass of the same length.
 * The published matrix peak of the chip assumes its highest clock; under a chip-wide matrix load the clock is lower,
 * and this figure is the ceiling the contraction kernels (Section 2.2: the two products of every cell) can be
 * compared with.  Results (HOST pointers): shader clocks per instruction on one wave, the shader clock in GHz during
 * the loop (shader clocks over the 100 MHz constant counter), and the whole launch's rate in TFLOP/s from stream
 * events.  Allocates 256 bytes of device memory for the call, synchronises `stream`; RNN_EUNSUPPORTED while the
 * stream is being captured, RNN_EINVAL outside 1..4096 compute units, 1..2^20 iterations or on a NULL pointer.
 */
int rnn_probe_matrix_rate(int compute_units, int iterations, double* clocks_per_instruction,
                          double* shader_ghz, double* tflops, void* stream);

/*
 * Measurement aid, no part of the forward pass: one step of the exchange the small-batch persistent kernels are
 * built on, without their arithmetic.  `groups` independent groups (the layers of a launch) of `workgroups`
 * workgroups each; in every step each workgroup of a group publishes its share of the group's `words` tagged 64-bit
 * words (device-scope stores), then fetches all of them (device-scope loads, a quarter per wave) until every word
 * carries the step's tag, and joins its waves at a barrier: what a step of the cell grid (Section 2.2: h_t of every
 * unit is needed by every unit at t + 1) costs before any product or gate is computed.  Results (HOST pointers):
 * microseconds per step from stream events, shader clocks per step on workgroup 0; the second of two passes is
 * timed.  Allocates groups * (steps + 1) * words * 8 bytes for the call and synchronises `stream`.  RNN_EINVAL
 * unless 1 <= groups <= 64, groups * workgroups <= compute units (all must be resident), words a multiple of 8 and
 * of workgroups, 8 <= words <= 2048, words / workgroups <= 64, 1 <= steps <= 100000; RNN_EUNSUPPORTED while the
 * stream is being captured; RNN_EDEVICE if a wait gave up (the kernel's waits are bounded).
 */
int rnn_probe_exchange_step(int groups, int workgroups, int words, int steps, double* us_per_step,
                            double* clocks_per_step, void* stream);

/* Static, NUL-terminated description of an rnn_status value. */
const char* rnn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* RNN_MI355X_H */
