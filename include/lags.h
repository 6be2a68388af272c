/*
 * lags.h - C ABI of the MI355X (gfx950) per-layer error-compensated top-k
 * sparsifier of LAGS-SGD ("Layer-wise Adaptive Gradient Sparsification for
 * Distributed Deep Learning with Convergence Guarantees").
 *
 * One worker's step for one layer l (Algorithm 1, lines 6-7; TopK is Eq. 4):
 *     acc      = residual + lr * grad            (binary32, product rounded, then sum rounded)
 *     selected = the k entries of largest |acc|  (equal magnitudes: lower index first)
 *     out      = the (index, acc) pairs of the selected entries, index ascending
 *     residual = acc with the selected entries set to +0.0f
 * and the aggregation of P workers (Algorithm 1, lines 8-9; Eq. 5):
 *     update   = (sum over p = 0..P-1, in that order, of worker p's selected entries) / P
 *
 * Conventions for every entry point
 *   - Returns LAGS_OK (0) or a negative error code; never throws, never exits.
 *   - Pointers named grad, residual, out_idx, out_val, idx, val, update are DEVICE
 *     pointers owned by the caller; the library neither frees nor keeps them.
 *     Everything else (descriptors, handles, out-parameters) is host memory.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns without waiting for it.  A call may also use a
 *     side stream of the context; that work is ordered after everything enqueued on
 *     `hip_stream` before the call and before everything enqueued on it after the call.
 *   - Argument validation happens before anything is enqueued: on an error return
 *     no output buffer has been touched.
 *   - The sparsify, merge, apply and delta calls may be recorded into a HIP graph by stream
 *     capture (they enqueue kernels and event waits only, no memset and no copy), provided a
 *     call with the same table (and, for the merge-type calls, a P at least as large) has run
 *     outside capture before: that first call sizes the context's scratch with synchronous
 *     allocations.  Timing (lags_profile_*) must be off while capturing.  A recorded graph
 *     holds the addresses of the scratch it was recorded with: from the first recorded call on,
 *     scratch that a larger table (or a larger P) outgrows is kept allocated until lags_destroy
 *     instead of being freed, so graphs recorded earlier stay valid for as long as the context,
 *     their table and the caller's buffers live.
 *   - A context owns scratch memory only (histograms, counters, candidate slots);
 *     nothing in it influences results.  One context serves one stream at a time:
 *     calls on the same context must be ordered on one stream (or externally).
 *   - Indices are 0-based, local to their layer, int32.
 */
#ifndef LAGS_H
#define LAGS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lags_ctx lags_ctx;     /* opaque: device id + scratch arena            */
typedef struct lags_table lags_table; /* opaque: immutable prepared layer table       */

/* One layer (a "segment" of the flat arrays).  Section 3, Eq. 2: the model vector is
 * the concatenation of L layer vectors; a layer here is one tensor. */
typedef struct {
  int64_t offset; /* element offset of the layer in the flat grad/residual/update arrays, >= 0 */
  int64_t d;      /* elements in the layer, 1 <= d < 2^31                                      */
  double rho;     /* requested density k/d, 0 < rho <= 1 (the paper's 1/c, Section 4.2)        */
} lags_layer_desc;

enum {
  LAGS_OK = 0,
  LAGS_EINVAL = -1,   /* bad argument (null pointer, size or density out of range, overlap) */
  LAGS_ENOMEM = -2,   /* host or device allocation failed                                   */
  LAGS_EHIP = -3,     /* a HIP runtime call failed                                          */
  LAGS_ECAPACITY = -4 /* a size exceeds what the library supports                           */
};

/* k = max(1, min(d, ceil(rho * d))) with the product evaluated in double.  The paper
 * configures k per layer (Algorithm 1, input k^(l)); this is how a density becomes a k.
 * Returns -1 if d < 1 or rho is not in (0, 1]. */
int64_t lags_topk_count(int64_t d, double rho);

/* Create / destroy a context on HIP device `device`.  Scratch grows when a table is
 * created and is released by lags_destroy (which waits for the device first).  If an allocation
 * for a larger table fails, the context and the tables created before stay usable.
 * A context owns one side stream on which lags_sparsify_model runs the kernels of the small
 * layers beside those of the large ones (forked from and joined to the caller's stream with
 * events, so the caller sees one ordered call).  With LAGS_SIDE_STREAM=0 in the environment when
 * the context is created, every kernel stays on the caller's stream: meant for tools that
 * serialise the dispatches of all queues, such as counter collection. */
int lags_create(lags_ctx **out, int device);
int lags_destroy(lags_ctx *ctx);

/* Prepare a table of n >= 1 layers: derives k_l and the output position of each layer
 * (layer l's pairs start at sum_{j<l} k_j), builds the launch plan, uploads it and sizes
 * the context's scratch.  Layers must not overlap each other; gaps are allowed.
 * `layers` is read during the call only.  A caller may list P workers x L layers of one
 * flat buffer in a single table.  Synchronous (allocates and copies). */
int lags_table_create(lags_ctx *ctx, const lags_layer_desc *layers, int32_t n, lags_table **out);
int lags_table_destroy(lags_table *t); /* before lags_destroy of its context; not while work using it is in flight */
int32_t lags_table_num_layers(const lags_table *t);
int64_t lags_table_total_k(const lags_table *t);              /* sum_l k_l = length of out_idx/out_val */
int64_t lags_table_k(const lags_table *t, int32_t l);         /* -1 if l is out of range               */
int64_t lags_table_out_offset(const lags_table *t, int32_t l);/* -1 if l is out of range               */

/* Algorithm 1 lines 6-7 for ONE layer of d elements with a caller-chosen k (1 <= k <= d).
 *   grad      device, float[d], read only
 *   residual  device, float[d], read then overwritten with the new residual
 *   out_idx   device, int32[k], written: selected indices, ascending
 *   out_val   device, float[k], written: acc at those indices (bit exact)
 * Buffers must not overlap.  `lr` must be finite.  The first call for a new (d, k) prepares
 * and caches a one-layer plan (a synchronous allocation); later calls only enqueue. */
int lags_sparsify_layer(lags_ctx *ctx, const float *grad, float *residual, int64_t d, float lr,
                        int64_t k, int32_t *out_idx, float *out_val, void *hip_stream);

/* lags_sparsify_layer for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * (bit for bit) as lags_sparsify_layer, but no context: the plan and every scratch buffer live in
 * one fixed device array of 5 MiB inside the library (one copy per GPU, held until the process
 * ends), and the call performs no allocation of any kind: it enqueues kernels on `hip_stream`
 * of HIP device `device` and returns.
 *   d <= lags_noalloc_max_elements() (16,777,216), and tiles of 4096 elements x candidate slots
 *   per tile <= 2^19.  The slots per tile follow from k/d (a power of two, at least eight times
 *   the expected candidates of a tile): above 2^20 elements a layer that keeps up to 0.16 % of
 *   its entries uses 128 slots per tile (16.7 M elements fit), one that keeps up to 0.4 % uses
 *   256 (8.3 M elements fit), and so on; layers of up to 2^20 elements always fit.
 *   Larger requests return LAGS_ECAPACITY and enqueue nothing.
 * All calls on one GPU share the array: calls that overlap in time on one GPU (two streams, two
 * threads) race and give undefined results; calls ordered on one stream are fine, and nothing
 * has to be cleared between them. */
int lags_sparsify_layer_noalloc(int device, const float *grad, float *residual, int64_t d, float lr,
                                int64_t k, int32_t *out_idx, float *out_val, void *hip_stream);
int64_t lags_noalloc_max_elements(void);

/* Algorithm 1 lines 6-7 for every layer of a table in a few launches (the one-GPU
 * analogue of Section 5's buffering of many small tensors).
 *   grad_flat, residual_flat   device, float arrays covering every layer's [offset, offset+d)
 *   out_idx, out_val           device, length lags_table_total_k(t); layer l's k_l pairs
 *                              are at lags_table_out_offset(t, l)
 * The table must have been created from the same context. */
int lags_sparsify_model(lags_ctx *ctx, const lags_table *t, const float *grad_flat,
                        float *residual_flat, float lr, int32_t *out_idx, float *out_val,
                        void *hip_stream);

/* Algorithm 1 lines 8-9 / Eq. 5: dense averaged update from P workers' sparse sets.
 *   idx, val      device; worker p's pairs, laid out as lags_sparsify_model writes them for
 *                 this table, start at idx + p*stride_k and val + p*stride_k
 *                 (stride_k >= lags_table_total_k(t)); within a layer each worker's indices
 *                 must be strictly ascending and in [0, d)
 *   update_flat   device, float; every element of every layer is overwritten (sum in worker
 *                 order starting from +0.0f, then one division by (float)P); elements
 *                 outside all layers are left alone
 *   1 <= P <= 1024.  The parameter step v -= update is the caller's. */
int lags_merge_sparse(lags_ctx *ctx, const lags_table *t, const int32_t *idx, const float *val,
                      int32_t P, int64_t stride_k, float *update_flat, void *hip_stream);

/* Algorithm 1 line 9 / Eq. 5 applied in place, without materialising the dense update:
 *     param = param - (sum over p = 0..P-1, in that order, of worker p's selected entries) / P
 * for every element of every layer (binary32: the sum from +0.0f, one division by (float)P,
 * one subtraction).  Only elements some worker selected are read or written; all others keep
 * their bits.  idx, val, P, stride_k as for lags_merge_sparse; param_flat is a device float
 * array laid out like grad_flat.  The result equals subtracting lags_merge_sparse's update. */
int lags_apply_sparse(lags_ctx *ctx, const lags_table *t, const int32_t *idx, const float *val,
                      int32_t P, int64_t stride_k, float *param_flat, void *hip_stream);

/* Section 6.2: the per-layer metric delta^(l) that checks Assumption 1, with x^p = acc^p:
 *     delta = || sum_p (x^p - TopK(x^p)) ||^2 / ( (1 - k/d) * || sum_p x^p ||^2 )
 * (the denominator is the expectation over RandK, Section 4.2).  x^p - TopK(x^p) is worker p's
 * residual after sparsification, so the inputs are
 *   residual_flat  device float; worker p's residuals (after lags_sparsify_model) at
 *                  residual_flat + p*res_stride, laid out by this table
 *   idx, val       device; the selected pairs, worker p at + p*stride_k
 *   out3           device double[3 * n_layers], written: for layer l
 *                  out3[3l] = numerator, out3[3l+1] = ||sum_p x^p||^2, out3[3l+2] = delta
 *                  (NaN if the denominator is 0, e.g. k == d)
 * All sums are in double, over workers in worker order; reads P*4 bytes per element. */
int lags_delta_monitor(lags_ctx *ctx, const lags_table *t, const float *residual_flat,
                       int64_t res_stride, const int32_t *idx, const float *val, int32_t P,
                       int64_t stride_k, double *out3, void *hip_stream);

/* Section 5, Eq. 9: the layer-wise adaptive choice of the compression ratio c^(l) = d^(l)/k^(l).
 * Host only: no GPU work, no context.
 *
 * Layer l's sparse exchange is issued when its gradient is ready and overlaps the
 * backpropagation of the layer computed next, layer l-1 (Section 3, pipelining).  Eq. 9 picks
 * the smallest ratio whose exchange is hidden,
 *     c^(l) = min{ c_u, min{ c : t_comm^(l)(c) + t_spar^(l) <= t_comp^(l-1) } }
 * (the printed outer "max" with an upper bound c_u is read as "min"; an empty inner set gives
 * c_u).  With c = d/k for an integer k this is the LARGEST k in [1, d] whose exchange fits,
 * raised to at least ceil(d / c_u).
 *
 * Section 5 leaves the cost model of the collective open; this library's model is a ring
 * all-gather of one message per worker holding k (int32 index, float value) pairs:
 *     t_comm(k) = (P - 1) * (alpha + 8 * k * beta)      seconds. */
typedef struct {
  double alpha; /* start-up time of one message, seconds, >= 0 */
  double beta;  /* transfer time per byte, seconds, >= 0       */
  int32_t P;    /* workers, >= 1                                */
} lags_allgather_model;

/* t_comm(k) of the model above, evaluated in double in exactly this order:
 * ((double)(P-1)) * (alpha + (8.0 * (double)k) * beta).  NaN if net is NULL, P < 1 or k < 0. */
double lags_allgather_seconds(const lags_allgather_model *net, int64_t k);

/* Eq. 9 for n layers listed in forward order (layer 0 is computed last in backpropagation).
 *   d[l]       elements of layer l, 1 <= d[l] < 2^31
 *   t_comp[l]  backpropagation time of layer l, seconds, >= 0
 *   t_spar[l]  sparsification overhead of layer l (compression + de-compression), seconds, >= 0
 *   c_u        upper bound of the ratio, >= 1
 * The budget of layer l is t_comp[l-1]; layer 0 has nothing left to hide behind (budget 0).
 *   k_out[l]   the chosen k^(l)
 *   rho_out[l] a density for which lags_topk_count(d[l], rho_out[l]) == k_out[l] exactly
 *              (k/d, moved down by an ulp where the rounded product would give k+1);
 *              may be NULL
 * All arrays are host memory.  LAGS_EINVAL on a NULL pointer, a size out of range, a negative
 * or NaN time, or c_u < 1 (nothing is written then). */
int lags_adaptive_ratios(const lags_allgather_model *net, const int64_t *d, const double *t_comp,
                         const double *t_spar, int32_t n, double c_u, int64_t *k_out, double *rho_out);

/* Diagnostic: which route each layer took in the LAST sparsify call made on this context,
 * which must have been a lags_sparsify_model call with this table (the record lives in the
 * context's scratch, which every table and every lags_sparsify_layer call of the context
 * shares).  Host-synchronous: waits for the device.  route[l], l in [0, n):
 * 0 = one-workgroup route (small layer); 1 = sampled threshold accepted, the kept set was
 * read off the candidates collected by the streaming pass; 2 = sampled threshold rejected (too
 * few candidates, a tile's slots overflowed, too many entries tied around the k-th largest),
 * exact selection over the whole layer; 3 = layer not sampled, exact multi-pass route.
 * Results never depend on the route. */
int lags_last_routes(lags_ctx *ctx, const lags_table *t, int32_t *route, int32_t n);

/* Diagnostic: how a rejected threshold guess (route 2) is served.  mode 0 (default): by one
 * workgroup per rejected layer inside the same launches (nothing extra is enqueued while guesses
 * hold; a rejection is reported to the host through a pinned word, and the next 64 sparsify
 * calls of the context also enqueue the six multi-pass kernels, which then serve rejections);
 * mode 1: the multi-pass kernels are always enqueued; mode 2: never for rejections.
 * Results are the same in every mode. */
int lags_debug_fallback_chain(lags_ctx *ctx, int mode);

/* Diagnostic: address and size of the context's scratch buffer number `which` (0 <= which < 16),
 * and how many outgrown buffers the context keeps alive for recorded graphs. */
int lags_debug_scratch_info(lags_ctx *ctx, int which, const void **ptr, int64_t *bytes, int64_t *retired);

/* Diagnostic: overwrite every scratch buffer of the context with 0xFF bytes (enqueued on
 * `hip_stream`).  Results of later calls must not change: scratch carries nothing between calls. */
int lags_debug_poison_scratch(lags_ctx *ctx, void *hip_stream);

/* Optional per-kernel timing with HIP events recorded on the caller's stream (measurement
 * aid; off by default; no effect on results).  While enabled every kernel launch of this
 * context is bracketed by a pair of events (a kernel that is enqueued as a back-to-back group
 * of launches, like the streaming pass, is bracketed as a group and counted with its number
 * of launches).  lags_profile_read waits for all recorded
 * events, adds the elapsed milliseconds and launch count of kernel `kernel_id`
 * (0 <= kernel_id < lags_profile_num_kernels()) to *total_ms / *launches, and
 * lags_profile_reset drops everything recorded so far.  All three are host-synchronous.
 * The id named "sparsify_call" is not a kernel: it brackets a whole sparsify call on the
 * caller's stream, from its first enqueue to the join of the side stream.  The small layers'
 * kernels run on the side stream beside the streaming pass, so the per-kernel times of a call
 * can add up to more than the call takes. */
int lags_profile_enable(lags_ctx *ctx, int on);
/* Like lags_profile_enable(ctx, 1) but only launches of kernel `kernel_id` are bracketed
 * (two events per launch of that kernel instead of two per launch of every kernel). */
int lags_profile_enable_kernel(lags_ctx *ctx, int kernel_id);
int lags_profile_num_kernels(void);
const char *lags_profile_kernel_name(int kernel_id); /* NULL if out of range */
int lags_profile_read(lags_ctx *ctx, int kernel_id, double *total_ms, int64_t *launches);
int lags_profile_reset(lags_ctx *ctx);
/* Number of layer elements one launch of kernel `kernel_id` covers for table `t` (0 if that
 * kernel is not launched for it): the unit count for bytes-per-launch arithmetic. */
int64_t lags_profile_kernel_elements(const lags_table *t, int kernel_id);

/* Static, human-readable text for an error code. */
const char *lags_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LAGS_H */
