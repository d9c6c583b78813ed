// A stacked RNN whose layers differ in width, as a chain of models: consecutive layers of one hidden size form a run,
// every run is an rnn_model of its own (padded to a kernel width, planned by the scheduler and launched on its own),
// and the runs follow one another on the stream, the output of one being the input of the next (Section 2.2: a layer
// sees nothing of the layer below but its output sequence).  Host code on top of the calls of rnn.h.
#include "../../include/rnn.h"

#include <hip/hip_runtime.h>

#include <new>
#include <vector>

struct rnn_stack {
    int cell = 0, L = 0, I = 0, D = 1, dtype = 0;
    size_t esize = 4;
    std::vector<int> first, count, width;      // per run: first layer, layers, hidden size
    std::vector<rnn_model*> models;            // per run
    std::vector<void*> mid;                    // per run but the last: its output [T, B, D * width], dtype
    std::vector<size_t> mid_bytes;
};

extern "C" {

void rnn_stack_destroy(rnn_stack* s) {
    if (!s) return;
    for (rnn_model* m : s->models) rnn_model_destroy(m);
    for (void* p : s->mid)
        if (p) (void)hipFree(p);
    delete s;
}

int rnn_stack_create(rnn_stack** out, int cell, int num_layers, int input_size, const int* hidden_sizes,
                     int num_directions, int dtype, const void* const* weights, int weights_on_device) try {
    if (!out) return RNN_EINVAL;
    *out = nullptr;
    if (!hidden_sizes || !weights || num_layers < 1 || input_size < 1 || (num_directions != 1 && num_directions != 2))
        return RNN_EINVAL;
    for (int l = 0; l < num_layers; ++l)
        if (hidden_sizes[l] < 1) return RNN_EINVAL;
    rnn_stack* s = new rnn_stack();
    s->cell = cell; s->L = num_layers; s->I = input_size; s->D = num_directions; s->dtype = dtype;
    s->esize = dtype == RNN_BF16 ? 2 : 4;
    for (int l = 0; l < num_layers;) {
        int n = 1;
        while (l + n < num_layers && hidden_sizes[l + n] == hidden_sizes[l]) ++n;
        s->first.push_back(l); s->count.push_back(n); s->width.push_back(hidden_sizes[l]);
        l += n;
    }
    for (size_t r = 0; r < s->first.size(); ++r) {
        const int in = r == 0 ? input_size : num_directions * s->width[r - 1];
        rnn_model* m = nullptr;
        const int rc = rnn_model_create(&m, cell, s->count[r], in, s->width[r], num_directions, dtype,
                                        weights + (size_t)s->first[r] * num_directions * 4, weights_on_device);
        if (rc != RNN_OK) {
            rnn_stack_destroy(s);
            return rc;
        }
        s->models.push_back(m);
    }
    s->mid.assign(s->first.size() - 1, nullptr);
    s->mid_bytes.assign(s->first.size() - 1, 0);
    *out = s;
    return RNN_OK;
} catch (const std::bad_alloc&) {
    return RNN_ENOMEM;
}

int rnn_stack_runs(const rnn_stack* s) { return s ? (int)s->models.size() : 0; }

int rnn_stack_run(const rnn_stack* s, int run, int* first_layer, int* num_layers, int* hidden_size, rnn_model** model) {
    if (!s || run < 0 || run >= (int)s->models.size()) return RNN_EINVAL;
    if (first_layer) *first_layer = s->first[run];
    if (num_layers) *num_layers = s->count[run];
    if (hidden_size) *hidden_size = s->width[run];
    if (model) *model = s->models[run];
    return RNN_OK;
}

size_t rnn_stack_device_bytes(const rnn_stack* s) {
    if (!s) return 0;
    size_t total = 0;
    for (const rnn_model* m : s->models) total += rnn_model_device_bytes(m);
    for (size_t b : s->mid_bytes) total += b;
    return total;
}

int rnn_stack_forward(rnn_stack* s, const void* x, const int32_t* lengths, const float* const* h0,
                      const float* const* c0, void* y, float* const* hT, float* const* cT, int T, int B,
                      void* stream) {
    if (!s || !x || !y || T < 1 || B < 1) return RNN_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const size_t runs = s->models.size();
    for (size_t r = 0; r + 1 < runs; ++r) {
        const size_t need = (size_t)T * B * s->D * s->width[r] * s->esize;
        if (need <= s->mid_bytes[r]) continue;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cap) != hipSuccess) return RNN_EDEVICE;
        if (cap != hipStreamCaptureStatusNone) return RNN_EUNSUPPORTED;   // cannot grow a buffer while recording
        if (hipDeviceSynchronize() != hipSuccess) return RNN_EDEVICE;     // an earlier forward may still read the old one
        if (s->mid[r]) (void)hipFree(s->mid[r]);
        s->mid[r] = nullptr;
        s->mid_bytes[r] = 0;
        if (hipMalloc(&s->mid[r], need) != hipSuccess) {
            (void)hipGetLastError();
            return RNN_ENOMEM;
        }
        s->mid_bytes[r] = need;
    }
    for (size_t r = 0; r < runs; ++r) {
        const void* in = r == 0 ? x : s->mid[r - 1];
        void* outp = r + 1 == runs ? y : s->mid[r];
        const int rc = rnn_forward(s->models[r], in, lengths, h0 ? h0[r] : nullptr, c0 ? c0[r] : nullptr, outp,
                                   hT ? hT[r] : nullptr, cT ? cT[r] : nullptr, T, B, stream);
        if (rc != RNN_OK) return rc;
    }
    return RNN_OK;
}

}  // extern "C"
