/*
 * Host-side scheduling of the cell graph of a stacked RNN: the graph itself, the paper's
 * topological sorting and a list-scheduling simulation with its start/finish-time rules.
 * Pure host code (no device work, no allocation that outlives a call); part of librnn_mi355x.so.
 *
 * Graphs are passed in compressed form: vertex v has the predecessors
 * pred_index[pred_offset[v] .. pred_offset[v+1]), ascending; per-edge arrays (communication times)
 * are indexed like pred_index.  All arrays are HOST memory owned by the caller.  Functions return
 * an rnn_status value (rnn.h): RNN_OK, or RNN_EINVAL for NULL pointers, sizes < 1, indices out of
 * range, a graph with a cycle or an order that is not topological.
 */
#ifndef RNN_SCHEDULE_H
#define RNN_SCHEDULE_H

#ifdef __cplusplus
extern "C" {
#endif

/* Number of vertices and of edges of the unrolled RNN of L layers, T steps, D directions
 * (Section 2.2, figure of the folded and unfolded RNN): one vertex per cell. */
int rnn_schedule_grid_size(int L, int T, int D, int* n_vertices, int* n_edges);

/* Fill the graph of that unrolled RNN.  Vertex (l*D + d)*T + s is the cell of layer l, direction d,
 * s-th step in that direction's processing order (direction 0 visits time s, direction 1 time
 * T-1-s).  Its predecessors: the cell of step s-1 of the same layer and direction, and the cells of
 * layer l-1 at the same time, one per direction.  pred_offset has n_vertices + 1 entries,
 * pred_index n_edges (sizes from rnn_schedule_grid_size). */
int rnn_schedule_grid(int L, int T, int D, int* pred_offset, int* pred_index);

/* The topological sorting of Section 4.1 (Algorithm "Topological Sorting" and the text around it).
 * The printed pseudo-code never enqueues a successor and has no merge step although the text
 * describes one; the reading implemented: a ready queue seeded with the vertices without
 * predecessors in ascending order; the first element is popped and appended to the order when all
 * its predecessors are in the order, otherwise pushed back; after a vertex is appended its
 * successors are visited in ascending order, one that has exactly one predecessor and whose
 * communication time from it exceeds avg_exec of the successor is appended at once (and its own
 * successors are visited before the next sibling: depth first, for locality), any other one not yet
 * queued is pushed to the back of the queue (breadth first, for parallelism).
 *   comm      per edge: communication time of pred -> v
 *   avg_exec  per vertex: execution time averaged over the devices
 *   order     receives the n vertices in scheduling order */
int rnn_schedule_order(int n, const int* pred_offset, const int* pred_index, const double* comm,
                       const double* avg_exec, int* order);

/* List scheduling of the vertices, taken in `order`, on P identical processors with the rules of
 * Section 3 (earliest start time EST, earliest finish time EFT, latency L = the largest actual
 * finish time): on processor j a vertex can start when j is free and every predecessor has finished,
 * plus the edge's communication time when the predecessor ran on another processor (reading: the
 * printed EST adds the communication time of every edge; processors that share one memory pay it
 * only across processors); the vertex goes to the processor with the smallest EFT, ties to the
 * lowest index.
 *   exec_time per vertex; comm per edge
 *   proc      receives the processor of every vertex (may be NULL)
 *   aft       receives the finish time of every vertex (may be NULL)
 *   latency   receives the largest finish time */
int rnn_schedule_simulate(int n, const int* pred_offset, const int* pred_index, const int* order, int P,
                          const double* exec_time, const double* comm, int* proc, double* aft,
                          double* latency);

/* The same list scheduling under a residency rule, the form in which the persistent kernels meet the memory
 * constraint of Section 3 (Equation 4: what a device holds is bounded): every vertex has a kind (the weights it
 * needs: its layer and direction), a processor (a group of compute units) holds the weights of ONE kind for the
 * length of a launch, and a kind lives on ONE processor.  Reading implemented: the vertices are taken in `order`
 * in passes (a pass is a launch).  In a pass a vertex is placed when all its predecessors are placed and its kind's
 * processor, or else a processor that holds nothing yet, exists: on its kind's processor if the kind has one,
 * otherwise on the empty processor with the smallest EFT (ties to the lowest index), which then holds that kind.
 * A vertex that cannot be placed waits for the next pass, which starts, with all processors empty, when the last
 * vertex of this pass has finished (launches on one stream run one after the other).  Start times follow the rules
 * of rnn_schedule_simulate.  rnn_forward derives from the result which layers share a launch and which group of
 * workgroups runs which (layer, direction).
 *   kind      per vertex, any int
 *   proc, pass, aft (each may be NULL)  receive processor, pass and finish time of every vertex
 *   latency   receives the largest finish time; n_passes the number of passes */
int rnn_schedule_place_resident(int n, const int* pred_offset, const int* pred_index, const int* order, int P,
                                const double* exec_time, const double* comm, const int* kind, int* proc,
                                int* pass, double* aft, double* latency, int* n_passes);

#ifdef __cplusplus
}
#endif

#endif /* RNN_SCHEDULE_H */
