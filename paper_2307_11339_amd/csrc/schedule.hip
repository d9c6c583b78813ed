// Host side only: the cell graph of a stacked RNN, the paper's topological sorting (Section 4.1)
// and list scheduling with its start / finish time rules (Section 3).  See include/rnn_schedule.h
// for the readings of the passages that are incomplete as printed.  Compiled with the device code
// for convenience; nothing here touches the GPU.
#include "../../include/rnn.h"
#include "../../include/rnn_schedule.h"

#include <deque>
#include <new>
#include <utility>
#include <vector>

namespace {

bool graph_ok(int n, const int* off, const int* idx) {
    if (n < 1 || !off || off[0] != 0) return false;
    for (int v = 0; v < n; ++v) {
        if (off[v + 1] < off[v]) return false;
        if (off[v + 1] > off[v] && !idx) return false;
        for (int e = off[v]; e < off[v + 1]; ++e) {
            if (idx[e] < 0 || idx[e] >= n || idx[e] == v) return false;
            if (e > off[v] && idx[e] <= idx[e - 1]) return false;
        }
    }
    return true;
}

}  // namespace

extern "C" {

int rnn_schedule_grid_size(int L, int T, int D, int* n_vertices, int* n_edges) {
    if (L < 1 || T < 1 || (D != 1 && D != 2) || !n_vertices || !n_edges) return RNN_EINVAL;
    const long long n = (long long)L * D * T;
    const long long e = (long long)L * D * (T - 1) + (long long)(L - 1) * D * T * D;
    if (n > (1LL << 30) || e > (1LL << 30)) return RNN_EUNSUPPORTED;
    *n_vertices = (int)n;
    *n_edges = (int)e;
    return RNN_OK;
}

int rnn_schedule_grid(int L, int T, int D, int* pred_offset, int* pred_index) {
    int n = 0, ne = 0;
    const int rc = rnn_schedule_grid_size(L, T, D, &n, &ne);
    if (rc != RNN_OK) return rc;
    if (!pred_offset || (ne > 0 && !pred_index)) return RNN_EINVAL;
    int e = 0;
    for (int g = 0; g < L * D; ++g) {
        const int l = g / D, d = g - l * D;
        for (int s = 0; s < T; ++s) {
            pred_offset[g * T + s] = e;
            // ascending ids: the layer below (smaller group index) comes before this group's own chain
            if (l > 0) {
                const int t = d == 0 ? s : T - 1 - s;
                for (int d2 = 0; d2 < D; ++d2) pred_index[e++] = ((l - 1) * D + d2) * T + (d2 == 0 ? t : T - 1 - t);
            }
            if (s > 0) pred_index[e++] = g * T + s - 1;
        }
    }
    pred_offset[n] = e;
    return e == ne ? RNN_OK : RNN_EINVAL;
}

int rnn_schedule_order(int n, const int* pred_offset, const int* pred_index, const double* comm,
                       const double* avg_exec, int* order) try {
    if (!graph_ok(n, pred_offset, pred_index) || !avg_exec || !order) return RNN_EINVAL;
    if (pred_offset[n] > 0 && !comm) return RNN_EINVAL;
    // successor lists, ascending because vertices are visited in ascending order
    std::vector<int> soff(n + 1, 0), sidx(pred_offset[n]);
    for (int e = 0; e < pred_offset[n]; ++e) ++soff[pred_index[e] + 1];
    for (int v = 0; v < n; ++v) soff[v + 1] += soff[v];
    {
        std::vector<int> fill(soff.begin(), soff.end() - 1);
        for (int v = 0; v < n; ++v)
            for (int e = pred_offset[v]; e < pred_offset[v + 1]; ++e) sidx[fill[pred_index[e]]++] = v;
    }
    std::vector<char> in_order(n, 0), queued(n, 0);
    std::deque<int> ready;
    for (int v = 0; v < n; ++v)
        if (pred_offset[v + 1] == pred_offset[v]) { ready.push_back(v); queued[v] = 1; }
    int placed = 0;
    std::vector<std::pair<int, int>> walk;  // (vertex, next successor slot) of the depth-first merge walk
    size_t pushed_back_in_a_row = 0;
    while (!ready.empty()) {
        const int v = ready.front();
        ready.pop_front();
        if (in_order[v]) continue;
        bool ok = true;
        for (int e = pred_offset[v]; e < pred_offset[v + 1] && ok; ++e) ok = in_order[pred_index[e]] != 0;
        if (!ok) {
            ready.push_back(v);
            if (++pushed_back_in_a_row > ready.size() + 1) return RNN_EINVAL;  // a cycle
            continue;
        }
        pushed_back_in_a_row = 0;
        in_order[v] = 1;
        order[placed++] = v;
        walk.clear();
        walk.emplace_back(v, soff[v]);
        while (!walk.empty()) {
            const int u = walk.back().first;
            const int slot = walk.back().second;
            if (slot == soff[u + 1]) { walk.pop_back(); continue; }
            walk.back().second = slot + 1;
            const int c = sidx[slot];
            if (in_order[c]) continue;
            const int e0 = pred_offset[c];
            if (pred_offset[c + 1] - e0 == 1 && comm[e0] > avg_exec[c]) {  // merge: keep the child with its parent
                in_order[c] = 1;
                queued[c] = 1;
                order[placed++] = c;
                walk.emplace_back(c, soff[c]);
            } else if (!queued[c]) {
                ready.push_back(c);
                queued[c] = 1;
            }
        }
    }
    return placed == n ? RNN_OK : RNN_EINVAL;
} catch (const std::bad_alloc&) {
    return RNN_ENOMEM;
}

int rnn_schedule_simulate(int n, const int* pred_offset, const int* pred_index, const int* order, int P,
                          const double* exec_time, const double* comm, int* proc, double* aft,
                          double* latency) try {
    if (!graph_ok(n, pred_offset, pred_index) || !order || P < 1 || !exec_time || !latency) return RNN_EINVAL;
    if (pred_offset[n] > 0 && !comm) return RNN_EINVAL;
    std::vector<double> free_at(P, 0.0), finish(n, 0.0);
    std::vector<int> where(n, -1);
    for (int i = 0; i < n; ++i) {
        const int v = order[i];
        if (v < 0 || v >= n || where[v] >= 0) return RNN_EINVAL;
        for (int e = pred_offset[v]; e < pred_offset[v + 1]; ++e)
            if (where[pred_index[e]] < 0) return RNN_EINVAL;  // not topological
        int best = -1;
        double best_eft = 0.0;
        for (int j = 0; j < P; ++j) {
            double est = free_at[j];
            for (int e = pred_offset[v]; e < pred_offset[v + 1]; ++e) {
                const int m = pred_index[e];
                const double ready = finish[m] + (where[m] != j ? comm[e] : 0.0);
                if (ready > est) est = ready;
            }
            const double eft = est + exec_time[v];
            if (best < 0 || eft < best_eft) { best = j; best_eft = eft; }
        }
        where[v] = best;
        finish[v] = best_eft;
        free_at[best] = best_eft;
    }
    double worst = 0.0;
    for (int v = 0; v < n; ++v) {
        if (finish[v] > worst) worst = finish[v];
        if (proc) proc[v] = where[v];
        if (aft) aft[v] = finish[v];
    }
    *latency = worst;
    return RNN_OK;
} catch (const std::bad_alloc&) {
    return RNN_ENOMEM;
}

int rnn_schedule_place_resident(int n, const int* pred_offset, const int* pred_index, const int* order, int P,
                                const double* exec_time, const double* comm, const int* kind, int* proc,
                                int* pass, double* aft, double* latency, int* n_passes) try {
    if (!graph_ok(n, pred_offset, pred_index) || !order || P < 1 || !exec_time || !kind || !latency || !n_passes)
        return RNN_EINVAL;
    if (pred_offset[n] > 0 && !comm) return RNN_EINVAL;
    std::vector<int> where(n, -1), placed_in(n, -1), waiting(order, order + n), left;
    {
        std::vector<char> seen(n, 0);
        for (int v : waiting) {
            if (v < 0 || v >= n || seen[v]) return RNN_EINVAL;
            seen[v] = 1;
        }
    }
    std::vector<double> finish(n, 0.0), free_at(P);
    std::vector<int> holds(P);
    std::vector<char> empty(P);
    double begin = 0.0;
    int r = 0;
    while (!waiting.empty()) {
        for (int j = 0; j < P; ++j) { free_at[j] = begin; empty[j] = 1; }
        left.clear();
        double end = begin;
        for (int v : waiting) {
            bool ready = true;
            for (int e = pred_offset[v]; e < pred_offset[v + 1] && ready; ++e) ready = placed_in[pred_index[e]] >= 0;
            int home = -1;                         // the processor that holds this kind in this pass
            for (int j = 0; j < P && home < 0; ++j)
                if (!empty[j] && holds[j] == kind[v]) home = j;
            int best = -1;
            double best_eft = 0.0;
            for (int j = 0; ready && j < P; ++j) {
                if (home >= 0 ? j != home : !empty[j]) continue;
                double est = free_at[j];
                for (int e = pred_offset[v]; e < pred_offset[v + 1]; ++e) {
                    const int m = pred_index[e];
                    const double at = finish[m] + (where[m] != j ? comm[e] : 0.0);
                    if (at > est) est = at;
                }
                const double eft = est + exec_time[v];
                if (best < 0 || eft < best_eft) { best = j; best_eft = eft; }
            }
            if (best < 0) {
                left.push_back(v);
                continue;
            }
            where[v] = best;
            placed_in[v] = r;
            finish[v] = best_eft;
            free_at[best] = best_eft;
            holds[best] = kind[v];
            empty[best] = 0;
            if (best_eft > end) end = best_eft;
        }
        if (left.size() == waiting.size()) return RNN_EINVAL;   // the order is not topological
        waiting.swap(left);
        begin = end;
        ++r;
    }
    double worst = 0.0;
    for (int v = 0; v < n; ++v) {
        if (finish[v] > worst) worst = finish[v];
        if (proc) proc[v] = where[v];
        if (pass) pass[v] = placed_in[v];
        if (aft) aft[v] = finish[v];
    }
    *latency = worst;
    *n_passes = r;
    return RNN_OK;
} catch (const std::bad_alloc&) {
    return RNN_ENOMEM;
}

}  // extern "C"
