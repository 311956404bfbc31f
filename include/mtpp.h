/* mtpp: max-throughput partitioning of a computation graph by slicing a topological order.
 * HOST-only C ABI (no GPU): every pointer is host memory.
 *
 * Sections "Dynamic sharding of neural networks" (equations io, overflow, f, P*) and "Enhanced MTPP slicing of
 * topological order" (Algorithm 1): operations 0..n-1 with work, sizeparam and sizeout; edges (u, v) = v consumes
 * the output of u; bandwidth B, fast memory M.  For a block S (a run of consecutive operations of the order):
 *     io_in(S)    = (1/B) * sum of sizeout(u) over the u outside S that some operation of S consumes (each u once)
 *     io_out(S)   = (1/B) * sum of sizeout(v) over the v in S that some operation outside S consumes (each v once)
 *     peak(S)     = the largest working set of one operation of S: its sizeout plus the sizeout of its inputs
 *     overflow(S) = max(0, sizeparam(S) + peak(S) - M) / B + peak(S) / B
 *     f(S)        = io_in(S) + sum of work over S + overflow(S) + io_out(S)
 * The order is sliced into at most k blocks so that the largest f is as small as possible (dynamic programme
 * over all segment costs, O(n^2 + n m) to set up and O(n^2 k) to solve); ties go to fewer blocks.
 * (Readings of what the paper leaves open: the printed overflow adds bytes to seconds, here both terms are
 * times and the first is clamped at zero; peak as above; the listing's heuristic adjustment is the identity.) */
#ifndef MTPP_H
#define MTPP_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum { MTPP_OK = 0, MTPP_E_ARG = -1 /* null pointer, bad index, n or k out of range, B <= 0 */,
       MTPP_E_CYCLE = -2 /* the graph is not acyclic, or `order` is not a topological order of it */ };
#define MTPP_MAX_N 2048

/* Kahn's algorithm; among the operations that are ready the one with the smallest index goes first.
 * order_out: [n], written.  Returns MTPP_E_CYCLE if the graph has a cycle. */
int mtpp_kahn_order(int n, int m, const int32_t* edge_from /*[m]*/, const int32_t* edge_to /*[m]*/,
                    int32_t* order_out /*[n]*/);

/* f of the block order[first .. last] (inclusive positions in the order, 0-based). */
int mtpp_block_cost(int n, int m, const int32_t* edge_from, const int32_t* edge_to,
                    const double* work /*[n]*/, const double* sizeparam /*[n]*/, const double* sizeout /*[n]*/,
                    const int32_t* order /*[n]*/, int first, int last, double B, double M, double* cost_out);

/* Best slicing of `order` (NULL: Kahn's order) into at most k blocks.  block_end_out: [k]; entry i receives the
 * position after the last operation of block i (so the last used entry is n).  n <= MTPP_MAX_N, 1 <= k.
 * Nothing is written when an error is returned. */
int mtpp_slice_order(int n, int m, const int32_t* edge_from, const int32_t* edge_to,
                     const double* work, const double* sizeparam, const double* sizeout,
                     const int32_t* order /*[n] or NULL*/, int k, double B, double M,
                     double* bottleneck_out, int32_t* n_blocks_out, int32_t* block_end_out /*[k]*/);

#ifdef __cplusplus
}
#endif
#endif
