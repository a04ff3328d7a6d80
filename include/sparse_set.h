/*
 * sparse_set.h -- C ABI of libsparse_set.so: one truly sparse MLP layer trained with Sparse
 * Evolutionary Training (SET), as in "Truly Sparse Neural Networks at Scale" (arXiv 2102.01732),
 * computed by hand-written HIP kernels for gfx950 (MI355X).
 *
 * A layer maps n_in neurons to n_out neurons.  The paper's problem formulation writes its weights
 * as W^(l) in R^{n_in x n_out} (w_ij: neuron i of the previous layer -> neuron j); the library
 * stores the TRANSPOSE Wt in R^{n_out x n_in} as real CSR: row j lists the incoming connections of
 * neuron j (the set Gamma_j of eq. 4), columns ascending inside a row.  Only stored connections
 * exist: no dense matrix and no mask is ever formed.
 *
 * Dense operands (activations, their gradients) are DEVICE pointers to fp32 in feature-major
 * layout: element (neuron i, sample b) at i*ld + b, with B <= ld < 2^31, ld % 4 == 0 and a 16-byte
 * aligned base pointer.  Columns b >= B of a row are never written and never influence a result.
 *
 * Ownership: all device memory belongs to the caller.  `state_dev` holds everything that
 * persists between calls (CSR, CSC view, weights, velocities, gradients, biases, saved
 * activation signs); `scratch_dev` holds temporaries of a call and may be shared by all layers
 * that are used on the same stream.  Both must be 256-byte aligned and at least as large as
 * sparse_layer_query_sizes reports; the layer keeps both pointers until sparse_layer_destroy.
 * The sl_layer handle is a small host object owned by the library.
 *
 * Streams: `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 * forward / backward / update / sparse_loss_softmax_ce only enqueue work and return.
 * init / evolve / import / export read counts back and therefore synchronise the stream.
 * Calls on one layer must be issued from one host thread at a time.
 *
 * Errors: every function returns SL_OK (0) or a negative code; nothing is printed and nothing
 * aborts.  sparse_layer_last_error gives a text for the last failure on that layer.
 */
#ifndef SPARSE_SET_H
#define SPARSE_SET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SL_OK          0
#define SL_EINVAL     -1   /* null pointer, bad size, B <= 0, B > max_batch, ld < B, misalignment  */
#define SL_ESTATE     -2   /* call order: backward before forward, update before backward, ...     */
#define SL_ENOMEM     -3   /* caller's state or scratch buffer too small                           */
#define SL_EHIP       -4   /* HIP runtime error                                                    */
#define SL_EOVERFLOW  -5   /* nnz or a dimension exceeds the 32-bit index range                    */

typedef struct sl_layer sl_layer;

#define SL_FLAG_NEED_INPUT_GRAD 1u  /* backward also produces grad_x (false for the first layer)  */

typedef struct sl_config {
    int64_t  n_in, n_out;
    double   epsilon;       /* Erdos-Renyi density parameter of the problem formulation:           */
                            /* nnz = min(floor(epsilon*(n_in+n_out) + 0.5), n_in*n_out)            */
    int64_t  nnz_override;  /* -1: use epsilon; >= 0: exact number of connections                  */
    int32_t  act_kind;      /* 0 identity (output layer), 1 All-ReLU (eq. 3)                       */
    int32_t  act_parity;    /* l % 2 of the receiving neuron layer, input layer being l = 1:       */
                            /* 0 -> slope -alpha for z <= 0, 1 -> slope +alpha                     */
    float    alpha;         /* All-ReLU slope                                                      */
    float    init_limit;    /* new connections ~ U(-init_limit, init_limit), at init and regrowth  */
    float    lr, momentum;  /* eta and mu of eq. (1)                                               */
    float    weight_decay;  /* L2 coefficient added to the gradient (0 in every workload)          */
    uint64_t seed;          /* Philox key = (lo32(seed) ^ layer_id*0x9E3779B9, hi32(seed))         */
    uint32_t layer_id;
    int32_t  max_batch;     /* largest B any call will pass                                        */
    int32_t  prune_mode;    /* 0: remove the round(zeta*nnz) smallest |w|, ties by flat index      */
                            /* 1: Algorithm 2 literally: fraction zeta of the weights >= 0 and of  */
                            /*    the weights < 0 separately, each by magnitude                    */
    uint32_t flags;         /* SL_FLAG_*                                                           */
} sl_config;

/* Bytes of device memory a layer with this configuration needs.  Host only, no GPU required. */
int sparse_layer_query_sizes(const sl_config *cfg, size_t *state_bytes, size_t *scratch_bytes);

/* Problem formulation and the initialisation step of Algorithm 2: builds an Erdos-Renyi topology with
 * exactly nnz distinct connections (generation 0 of the Philox sampler), draws the weights,
 * zeroes biases and velocities, builds CSR and (if SL_FLAG_NEED_INPUT_GRAD) the CSC view.
 * Synchronises the stream. */
int sparse_layer_init(const sl_config *cfg, void *state_dev, size_t state_bytes, void *scratch_dev,
                      size_t scratch_bytes, void *hip_stream, sl_layer **out);

/* Forward, eq. (3) applied to z = Wt x + b:  a[j][b] = f_l(bias[j] + sum_{i in Gamma_j} Wt[j,i] x[i][b]).
 * x_dev [n_in][ldx], a_dev [n_out][lda] (device).  The sign of z needed by backward is kept in
 * the layer's state.  Asynchronous. */
int sparse_layer_forward(sl_layer *layer, const float *x_dev, int64_t ldx, int32_t B, float *a_dev,
                         int64_t lda, void *hip_stream);

/* Forward only (the paper's test-set evaluation, which its extreme-scale section names as a bottleneck): the same
 * computation as sparse_layer_forward, but nothing is saved for a backward pass and the layer's
 * training state is untouched, so it may be called between forward and backward.  Asynchronous. */
int sparse_layer_infer(sl_layer *layer, const float *x_dev, int64_t ldx, int32_t B, float *a_dev, int64_t lda,
                       void *hip_stream);

/* For callers that cannot allocate device memory or hand over a workspace at call time (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): sparse_layer_infer with the partial sums of
 * split rows kept in a buffer of SL_STATIC_SCRATCH_MIB MiB that is built into the library (one copy per GPU,
 * held until the process ends) instead of in the layer's scratch buffer.  Same arguments, same results bit for
 * bit.  Allocates nothing and creates no events.  SL_ENOMEM if the layer's partial sums (virtual rows x
 * round_up(max_batch, 32) floats; zero for layers without split rows) do not fit, SL_ESTATE while per-kernel
 * profiling is on.  The device of `hip_stream` must be current.  All calls on one GPU share that GPU's buffer:
 * calls that overlap in time on one GPU (two streams, two threads) race; nothing in it needs clearing between
 * calls.  Asynchronous. */
#define SL_STATIC_SCRATCH_MIB 16
int sparse_layer_infer_static(sl_layer *layer, const float *x_dev, int64_t ldx, int32_t B, float *a_dev, int64_t lda,
                              void *hip_stream);

/* Backward of the same minibatch (must follow forward with the same B):
 *   dz = grad_a * f_l'(z)                     (f' at z = 0 is the "z <= 0" branch of eq. 3)
 *   grad_bias[j] = sum_b dz[j][b]
 *   grad_val[p]  = sum_b dz[j][b] * x[i][b]   for every stored connection p = (j,i) only
 *   grad_x[i][b] = sum_{j:(j,i) stored} Wt[j,i] * dz[j][b]   (weights before the update)
 * grad_a_dev [n_out][ldg]; x_dev is the x passed to forward; grad_x_dev [n_in][ldgx] must be
 * non-NULL iff the layer was created with SL_FLAG_NEED_INPUT_GRAD (but see
 * sparse_layer_link_producer, which allows NULL for both gradients inside a chain).  The 1/B of the minibatch
 * mean (Algorithm 1's worker gradient) is carried by grad_a of the output layer.  Asynchronous. */
int sparse_layer_backward(sl_layer *layer, const float *x_dev, int64_t ldx, const float *grad_a_dev,
                          int64_t ldg, int32_t B, float *grad_x_dev, int64_t ldgx, void *hip_stream);

/* Dropout on the activations of a hidden layer (the paper's experiments use rates 0.3 / 0.4; none of
 * the benchmark workloads does).  Sets the rate p in [0,1) and the step index that selects the mask
 * for the NEXT forward/backward pair; call it before every training forward with a new step.  Element
 * (neuron j, sample b) is kept iff word b&3 of Philox(counter = (j, b>>2, 4, step)) >= floor(p*2^32);
 * kept activations and their gradients are multiplied by 1/(1-p), dropped ones are zero.  The keep
 * bits are saved next to the sign bits, so backward needs no regeneration.  sparse_layer_infer never
 * drops.  p = 0 switches it off. */
int sparse_layer_set_dropout(sl_layer *layer, float p, uint64_t step);

/* Chaining (optional).  Declares that `layer`'s input x is the activation output of `producer`
 * (same stream, same minibatch).  After that, sparse_layer_backward(layer, ...) may be called with
 * grad_x_dev == NULL: the input gradient is then multiplied by the producer's f' (eq. 3, from its
 * saved sign mask) and stored as the producer's dz, with its bias gradient, inside the same kernel,
 * and the producer's next sparse_layer_backward may be called with grad_a_dev == NULL.  This removes
 * one read and one write of the [n][B] gradient per hidden layer.  producer == NULL unlinks.
 * The producer must outlive the link. */
int sparse_layer_link_producer(sl_layer *layer, sl_layer *producer);

/* Momentum SGD over the stored connections and the biases, eq. (1) in velocity form:
 * vel <- mu*vel - eta*(grad + weight_decay*w);  w <- w + vel.  Must follow backward.  Asynchronous. */
int sparse_layer_update(sl_layer *layer, void *hip_stream);

/* Update fused behind the SDDMM (eq. 1 applied where Algorithm 1's worker gradient of a connection is
 * produced).  mode 0 (default): sparse_layer_backward stores the weight gradient and sparse_layer_update applies
 * eq. (1).  mode 1: sparse_layer_backward itself applies eq. (1) to every stored connection in the kernel that
 * finishes its gradient entry (same fp32 arithmetic, same result bit for bit) and does not store the gradient
 * (sparse_layer_export_grad then returns SL_ESTATE for grad_val); sparse_layer_update / sparse_layers_update must
 * still follow and update the biases only.  mode 2: as mode 1, and the gradient is stored as well.  The weights
 * that backward uses for the input gradient are those before the update in every mode.  SL_ESTATE between
 * backward and update. */
int sparse_layer_set_fused_update(sl_layer *layer, int32_t mode);

/* The prune / regrow cycle that Algorithm 2 runs after every epoch: removes k connections (see prune_mode), draws k
 * distinct empty positions with the Philox sampler at `generation` (>= 1, < 2^32; a different
 * value per call), gives them fresh weights and zero velocity, and rebuilds CSR and the CSC
 * view.  nnz is unchanged.  k = floor(zeta*nnz + 0.5) in double.  Synchronises the stream. */
int sparse_layer_evolve(sl_layer *layer, double zeta, uint64_t generation, void *hip_stream);

/* sparse_layer_evolve for up to 16 layers at once (Algorithm 2 evolves every layer after an epoch, and the layers'
 * cycles are independent of each other): layer k runs on hip_streams[k] (host array of `count` stream handles, any
 * of them may be the null stream) from a host thread of its own, so that one layer's waits overlap the others'
 * kernels.  Every layer ends exactly as after its own sparse_layer_evolve call.  The layers must have been
 * initialised with scratch buffers that do not overlap (SL_EINVAL otherwise).  The caller orders each stream after
 * the work that produced the layer's weights; all streams are synchronised on return.  Returns the first non-zero
 * code in layer order (that layer holds the message; the other layers still complete their cycle). */
int sparse_layers_evolve(sl_layer *const *layers, int32_t count, double zeta, uint64_t generation,
                         void *const *hip_streams);

/* Regrowth sampler of sparse_layer_evolve (sparse layers only).  Candidate positions t = 0, 1, 2, ... are
 * evaluated a window [0, W) at a time; a window that accepts fewer than k positions is evaluated again twice as
 * long.  first_window: W of the first attempt (0: chosen from the expected number of draws plus eight standard
 * deviations); max_window: largest W tried (0: what the scratch buffer holds).  The result never depends on
 * either; a window that cannot grow far enough makes sparse_layer_evolve return SL_ESTATE and leaves the layer
 * exactly as it was. */
int sparse_layer_set_sampler_window(sl_layer *layer, int64_t first_window, int64_t max_window);

/* Neuron importance, eq. (4): importance[j] = sum over the stored incoming connections of neuron j of
 * |Wt[j,i]|, added in fp32 in stored order.  importance_host: host array of n_out floats.
 * Synchronises the layer's last stream. */
int sparse_layer_importance(sl_layer *layer, float *importance_host);

/* Importance Pruning of Algorithm 2: removes ALL incoming connections of every neuron whose
 * importance (as above) is < threshold and compacts CSR, CSC view and velocities.  nnz shrinks (the
 * buffers keep their size); later evolutions preserve the reduced nnz.  *removed (host, may be
 * NULL) receives the number of removed connections.  Synchronises the stream. */
int sparse_layer_importance_prune(sl_layer *layer, float threshold, int64_t *removed, void *hip_stream);

/* Sparse model averaging: eq. (2) and the final step of Algorithm 1 (magnitude re-pruning of the averaged
 * model back to the sparsity level S): dst <- (1/K) * sum of the K replicas, where
 * a connection that a replica does not have counts as zero; the union of the patterns is then
 * pruned by magnitude (ordering key as in sparse_layer_evolve) back to dst's current number of
 * connections.  Each value is the fp32 sum in replica order divided by K.  Biases are averaged the
 * same way; all velocities of dst become zero.  dst may be one of the replicas; the replicas must
 * have dst's shape and at most dst's capacity (its nnz at creation) results.  1 <= K <= 16.
 * scratch_dev: device buffer of sparse_layers_average_query(sum of the replicas' nnz) bytes,
 * 256-byte aligned, used only during the call.  Synchronises the stream. */
int sparse_layers_average_query(int64_t total_entries, size_t *scratch_bytes);
int sparse_layers_average(sl_layer *dst, sl_layer *const *replicas, int32_t K, void *scratch_dev,
                          size_t scratch_bytes, void *hip_stream);

int sparse_layer_destroy(sl_layer *layer);

/* RetainValidUpdates of Algorithm 1 (asynchronous training on a parameter server): a gradient that
 * was computed on an older topology of this layer is restricted to the connections that still
 * exist; connections created since get a zero gradient.  The old pattern is CSR (old_rowptr_dev
 * int32[n_out+1], old_colidx_dev int32[old_nnz], columns ascending within a row) with
 * old_grad_dev float[old_nnz] in the same order and old_grad_bias_dev float[n_out]; all device
 * pointers, borrowed for the call's kernels only.  The result becomes the layer's pending gradient,
 * exactly as if sparse_layer_backward had produced it: sparse_layer_update applies it and
 * sparse_layer_export_grad reads it.  Row bounds outside [0, old_nnz] are clamped, never followed.
 * SL_ESTATE between forward and backward.  Asynchronous. */
int sparse_layer_retain_valid_updates(sl_layer *layer, const int32_t *old_rowptr_dev, const int32_t *old_colidx_dev,
                                      const float *old_grad_dev, int64_t old_nnz, const float *old_grad_bias_dev,
                                      void *hip_stream);

/* Softmax + cross-entropy over C output neurons (the loss is unnamed in the paper).
 * z_dev [C][ldz], y_dev int32[B] (device) -> dz_dev [C][lddz] = (softmax(z) - onehot(y)) / B and
 * *loss_sum_dev += sum_b -log softmax(z)[y_b] (device float; the caller zeroes and averages it;
 * may be NULL).  C <= 1024.  A label outside [0, C) means "no target": that sample adds nothing to the loss and
 * its dz is softmax(z) / B; the label is never used as an index.  Asynchronous. */
int sparse_loss_softmax_ce(const float *z_dev, int64_t ldz, const int32_t *y_dev, int32_t B, int32_t C,
                           float *dz_dev, int64_t lddz, float *loss_sum_dev, void *hip_stream);

/* The same loss written straight into an output layer (identity activation, n_out <= 1024) that has
 * just run forward with this B: dz and the bias gradient of `layer` are produced here, so its
 * sparse_layer_backward may be called with grad_a_dev == NULL and needs no separate pass.
 * z_dev is the a_dev that forward wrote.  Asynchronous. */
int sparse_loss_softmax_ce_into(sl_layer *layer, const float *z_dev, int64_t ldz, const int32_t *y_dev, int32_t B,
                                float *loss_sum_dev, void *hip_stream);

/* sparse_layer_update for up to 16 layers in one kernel launch (same arithmetic, same results).
 * Small networks are bound by the number of dependent launches per step.  Asynchronous. */
int sparse_layers_update(sl_layer *const *layers, int32_t count, void *hip_stream);

/* Inspection / parity / checkpoint.  Host pointers; each call synchronises the layer's last
 * stream.  Any output pointer may be NULL.  Arrays are in CSR order. */
int sparse_layer_nnz(const sl_layer *layer, int64_t *nnz);
int sparse_layer_export_csr(sl_layer *layer, int32_t *rowptr, int32_t *colidx, float *val, float *vel,
                            float *bias, float *bias_vel);
/* Replaces pattern and values; nnz must equal the layer's nnz, rows must be sorted and distinct. */
int sparse_layer_import_csr(sl_layer *layer, const int32_t *rowptr, const int32_t *colidx, const float *val,
                            const float *vel, const float *bias, const float *bias_vel);
int sparse_layer_export_grad(sl_layer *layer, float *grad_val, float *grad_bias);
int sparse_layer_set_lr(sl_layer *layer, float lr);
const char *sparse_layer_last_error(const sl_layer *layer);

/* Per-kernel timing (tracing aid, off by default).  Between profile_begin and profile_end every
 * kernel the layer launches is bracketed by HIP events on the caller's stream.  profile_end waits
 * for them and returns, per kernel id < n_ids, the number of launches and their summed duration
 * in milliseconds (host arrays).  Ids: see sparse_kernel_name (0 forward SpMM, 1 forward fix-up,
 * 2 activation gradient, 3 fused backward, 4 SDDMM, 5 backward fix-up, 6 update). */
int sparse_layer_profile_begin(sl_layer *layer);
int sparse_layer_profile_end(sl_layer *layer, int32_t *launches, float *total_ms, int32_t n_ids);
const char *sparse_kernel_name(int32_t id);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_SET_H */
