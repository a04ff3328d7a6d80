/*
 * set_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow CPU oracle for the per-minibatch compute of a truly sparse MLP
 * layer trained with Sparse Evolutionary Training (SET), written from the paper
 * "Truly Sparse Neural Networks at Scale" (arXiv 2102.01732).  It exists so that the GPU
 * library can be checked against something that can be read next to the paper by eye.  It is
 * NOT part of the product: only the tests, the smoke check and the benchmark's CPU-baseline leg
 * may load it, and it shares no code with the GPU path.
 *
 * Conventions (the paper's problem formulation writes W^(l) as n_{l-1} x n_l with w_ij the
 * connection from neuron i of layer l-1 to neuron j of layer l; we store the transpose):
 *   Wt  [n_out x n_in] in CSR: rowptr[n_out+1], colidx[nnz] ascending inside a row, val[nnz].
 *        Row j lists the incoming connections of neuron j, i.e. the set Gamma_j of eq. (4).
 *   dense operands are feature-major: element (neuron i, sample b) at i*ld + b.
 *   storage is fp32 (the paper's framework uses 32-bit floats); every reduction accumulates in
 *   double and rounds once on store.
 *
 * Functions and the passage each follows:
 *   or_philox4x32_10      counter-based generator of Salmon et al. (SC'11), used for the
 *                         Erdos-Renyi initialisation (problem formulation) and for the random
 *                         regrowth of Algorithm 2.
 *   or_weight_value       value of a freshly created connection (paper silent: uniform in
 *                         (-limit, limit), the same law at initialisation and at regrowth).
 *   or_sample_positions   k distinct empty positions, uniformly at random (Erdos-Renyi graph
 *                         with a fixed number of edges; Algorithm 2, regrowth step).
 *   or_forward            z = Wt x + b followed by All-ReLU, eq. (3).
 *   or_backward           backpropagation through one layer: delta through eq. (3)'s
 *                         derivative, weight gradient on existing connections only
 *                         (the worker gradient of Algorithm 1), input gradient.
 *   or_update             momentum SGD, eq. (1), in velocity form.
 *   or_dropout_keep/apply dropout on hidden activations (experiments' hyper-parameters).
 *   or_prune_select       Algorithm 2's removal step (magnitude based).
 *   or_softmax_ce         softmax + cross-entropy loss and its gradient (loss unnamed in the
 *                         paper; this is the reading used throughout).
 *   or_average_sorted,    sparse averaging of K replicas, eq. (2), and the magnitude re-pruning that
 *   or_keep_largest       follows it (WASAP-SGD phase 2, last step of Algorithm 1).
 *   or_importance(_f32)   neuron importance, eq. (4); Importance Pruning of Algorithm 2 removes the
 *                         incoming connections of neurons whose importance is below a threshold.
 *
 * Threads: when built with -fopenmp, the loops of or_forward, or_backward and or_update whose
 * iterations own disjoint outputs are shared among threads (rows j, or blocks of batch columns b for
 * the input gradient).  Every output element is still produced by ONE thread, by the same
 * additions in the same order as in the serial loop, so results do not depend on the thread count;
 * or_set_threads(1) gives the single-threaded run.  Nothing else is threaded.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -fPIC -shared set_oracle.c -o liboracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Storage type of the training step (or_all_relu, or_forward, or_backward, or_update, or_softmax_ce).  float is the
 * paper's precision and the only build the parity tests use; -DOR_REAL=double builds the same source with double
 * storage, which lets a finite-difference pin check the backward pass to 1e-6 instead of to what fp32 allows. */
#ifndef OR_REAL
#define OR_REAL float
#endif
typedef OR_REAL or_real;

/* Number of threads for the loops described in the header (0 or less: the OpenMP default).  Returns
 * the number that will be used (1 without OpenMP). */
int or_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3").  */
/* One round: two 32x32->64 multiplies of counter words 0 and 2 by fixed odd constants; the    */
/* high halves are xored with the other counter words and the round key, the low halves move   */
/* over unchanged.  The key is bumped by two Weyl constants between rounds.                    */
/* ------------------------------------------------------------------------------------------ */
void or_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Stream layout used by this method.  key = (seed_lo ^ layer_id * 0x9E3779B9, seed_hi);
 * counter = (index_lo, index_hi, purpose, generation).  purpose: 1 = candidate position,
 * 2 = dense-mode ordering key, 3 = weight value.  generation 0 is the initialisation, g >= 1 the
 * g-th topology evolution.  Every draw is a pure function of its arguments. */
static void draw(uint64_t seed, uint32_t layer_id, uint32_t purpose, uint32_t generation,
                 uint64_t index, uint32_t out[4])
{
    uint32_t key[2], ctr[4];
    key[0] = (uint32_t)seed ^ (uint32_t)(layer_id * 0x9E3779B9u);
    key[1] = (uint32_t)(seed >> 32);
    ctr[0] = (uint32_t)index;
    ctr[1] = (uint32_t)(index >> 32);
    ctr[2] = purpose;
    ctr[3] = generation;
    or_philox4x32_10(ctr, key, out);
}

/* Value of a connection created at `generation` at flat position p = j*n_in + i.
 * 23 random bits r -> odd integer 2r+1 - 2^23 in (-2^23, 2^23) -> v = that * 2^-23 in (-1,1),
 * never zero; w = v * limit with a single fp32 multiply. */
float or_weight_value(uint64_t seed, uint32_t layer_id, uint32_t generation, uint64_t p,
                      float init_limit)
{
    uint32_t w[4];
    draw(seed, layer_id, 3u, generation, p, w);
    uint32_t r = w[0] >> 9;
    int32_t odd = (int32_t)(2u * r + 1u) - (int32_t)(1 << 23);
    float v = (float)odd * (1.0f / 8388608.0f);
    return v * init_limit;
}

void or_weight_values(uint64_t seed, uint32_t layer_id, uint32_t generation, const uint64_t *p,
                      int64_t n, float init_limit, float *out)
{
    for (int64_t t = 0; t < n; ++t)
        out[t] = or_weight_value(seed, layer_id, generation, p[t], init_limit);
}

/* ------------------------------------------------------------------------------------------ */
/* Sampling k distinct empty positions.                                                        */
/* ------------------------------------------------------------------------------------------ */
static int contains_sorted(const uint64_t *a, int64_t n, uint64_t x)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo < n && a[lo] == x;
}

typedef struct { uint64_t key; uint64_t pos; } keypos;

static int cmp_keypos(const void *pa, const void *pb)
{
    const keypos *a = (const keypos *)pa, *b = (const keypos *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->pos != b->pos) return a->pos < b->pos ? -1 : 1;
    return 0;
}

static int cmp_u64(const void *pa, const void *pb)
{
    uint64_t a = *(const uint64_t *)pa, b = *(const uint64_t *)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

/* occupied: sorted flat positions already in use (|occupied| = n_occ).  Writes the k chosen
 * positions to out_pos in ASCENDING order.  Returns 0, or -1 if fewer than k empty positions
 * exist, -2 on allocation failure.
 *
 * dense mode  (n_in*n_out <= 4*(n_occ+k)): every empty position p gets the 64-bit ordering key
 *             (word0<<32 | word1) of draw(purpose 2, index p); the k empties with the smallest
 *             (key, p) are chosen.
 * sparse mode (otherwise): candidates t = 0,1,2,... with row j = (word0 * n_out) >> 32 and
 *             column i = (word1 * n_in) >> 32 of draw(purpose 1, index t); a candidate is
 *             accepted iff it is not occupied and was not accepted before; stop at k accepts. */
int or_sample_positions(int64_t n_in, int64_t n_out, int64_t k, const uint64_t *occupied,
                        int64_t n_occ, uint64_t seed, uint32_t layer_id, uint32_t generation,
                        uint64_t *out_pos)
{
    uint64_t total = (uint64_t)n_in * (uint64_t)n_out;
    if (k < 0 || (uint64_t)(n_occ + k) > total) return -1;
    if (k == 0) return 0;
    if (total <= 4u * (uint64_t)(n_occ + k)) {
        keypos *cand = (keypos *)malloc(sizeof(keypos) * (size_t)(total - (uint64_t)n_occ));
        if (!cand) return -2;
        int64_t n_empty = 0;
        for (uint64_t p = 0; p < total; ++p) {
            if (contains_sorted(occupied, n_occ, p)) continue;
            uint32_t w[4];
            draw(seed, layer_id, 2u, generation, p, w);
            cand[n_empty].key = ((uint64_t)w[0] << 32) | (uint64_t)w[1];
            cand[n_empty].pos = p;
            ++n_empty;
        }
        qsort(cand, (size_t)n_empty, sizeof(keypos), cmp_keypos);
        for (int64_t t = 0; t < k; ++t) out_pos[t] = cand[t].pos;
        free(cand);
    } else {
        /* accepted-so-far set: open addressing, empty slot = all ones (never a valid position
         * because total < 2^63 here). */
        uint64_t cap = 16;
        while (cap < 2u * (uint64_t)k + 2u) cap <<= 1;
        uint64_t *table = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)cap);
        if (!table) return -2;
        memset(table, 0xFF, sizeof(uint64_t) * (size_t)cap);
        int64_t accepted = 0;
        for (uint64_t t = 0; accepted < k; ++t) {
            uint32_t w[4];
            draw(seed, layer_id, 1u, generation, t, w);
            uint64_t j = ((uint64_t)w[0] * (uint64_t)n_out) >> 32;
            uint64_t i = ((uint64_t)w[1] * (uint64_t)n_in) >> 32;
            uint64_t p = j * (uint64_t)n_in + i;
            if (contains_sorted(occupied, n_occ, p)) continue;
            uint64_t slot = (p * 0x9E3779B97F4A7C15ull) & (cap - 1);
            int seen = 0;
            while (table[slot] != UINT64_MAX) {
                if (table[slot] == p) { seen = 1; break; }
                slot = (slot + 1) & (cap - 1);
            }
            if (seen) continue;
            table[slot] = p;
            out_pos[accepted++] = p;
        }
        free(table);
    }
    qsort(out_pos, (size_t)k, sizeof(uint64_t), cmp_u64);
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* All-ReLU, eq. (3): identity for x > 0; for x <= 0 the slope is -alpha when the receiving    */
/* neuron layer index l is even and +alpha when it is odd.  act_kind 0 = identity (output      */
/* layer, excluded by the paper from eq. (3)).                                                 */
/* ------------------------------------------------------------------------------------------ */
static or_real all_relu(or_real z, int act_kind, int parity, or_real alpha)
{
    if (act_kind == 0 || z > 0.0f) return z;
    return parity == 0 ? (-alpha) * z : alpha * z;
}

static or_real all_relu_slope(or_real z, int act_kind, int parity, or_real alpha)
{
    if (act_kind == 0 || z > 0.0f) return 1.0f;
    return parity == 0 ? -alpha : alpha;
}

void or_all_relu(const or_real *z, int64_t n, int act_kind, int parity, or_real alpha, or_real *a)
{
    for (int64_t t = 0; t < n; ++t) a[t] = all_relu(z[t], act_kind, parity, alpha);
}

/* Forward of one layer for a minibatch of B samples:
 *   z[j][b] = bias[j] + sum_{i in Gamma_j} Wt[j,i] * x[i][b];  a[j][b] = f_l(z[j][b]). */
void or_forward(int64_t n_out, const int32_t *rowptr, const int32_t *colidx, const or_real *val,
                const or_real *bias, const or_real *x, int64_t ldx, int32_t B, int act_kind,
                int parity, or_real alpha, or_real *z, or_real *a, int64_t ldo)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_out; ++j) {
        for (int32_t b = 0; b < B; ++b) {
            double acc = (double)bias[j];
            for (int32_t p = rowptr[j]; p < rowptr[j + 1]; ++p)
                acc += (double)val[p] * (double)x[(int64_t)colidx[p] * ldx + b];
            or_real zf = (or_real)acc;
            z[j * ldo + b] = zf;
            a[j * ldo + b] = all_relu(zf, act_kind, parity, alpha);
        }
    }
}

/* Backward of one layer.  Inputs: the layer's input x, its pre-activation z (from or_forward),
 * grad_a = dLoss/da.  Outputs:
 *   dz[j][b]     = grad_a[j][b] * f_l'(z[j][b])      (f' at z = 0 is the "<= 0" branch of eq. 3)
 *   grad_bias[j] = sum_b dz[j][b]
 *   grad_val[p]  = sum_b dz[j][b] * x[i][b]          for every STORED p = (j,i) only
 *   grad_x[i][b] = sum_{j : (j,i) stored} Wt[j,i] * dz[j][b]   (skipped when grad_x == NULL)
 * The 1/B of the minibatch mean lives in grad_a of the last layer (see or_softmax_ce). */
int or_backward(int64_t n_in, int64_t n_out, const int32_t *rowptr, const int32_t *colidx,
                const or_real *val, const or_real *x, int64_t ldx, const or_real *z,
                const or_real *grad_a, int64_t ldo, int32_t B, int act_kind, int parity,
                or_real alpha, or_real *dz, or_real *grad_val, or_real *grad_bias, or_real *grad_x,
                int64_t ldgx)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_out; ++j) {
        double sb = 0.0;
        for (int32_t b = 0; b < B; ++b) {
            or_real d = grad_a[j * ldo + b] * all_relu_slope(z[j * ldo + b], act_kind, parity, alpha);
            dz[j * ldo + b] = d;
            sb += (double)d;
        }
        grad_bias[j] = (or_real)sb;
        for (int32_t p = rowptr[j]; p < rowptr[j + 1]; ++p) {
            int64_t i = colidx[p];
            double s = 0.0;
            for (int32_t b = 0; b < B; ++b) s += (double)dz[j * ldo + b] * (double)x[i * ldx + b];
            grad_val[p] = (or_real)s;
        }
    }
    if (grad_x) {
        double *acc = (double *)calloc((size_t)n_in * (size_t)B, sizeof(double));
        if (!acc) return -2;
        /* blocks of eight batch columns are independent of each other: each (i, b) still receives its
         * terms in ascending (j, p) order */
#pragma omp parallel for schedule(static)
        for (int32_t b0 = 0; b0 < B; b0 += 8) {
            int32_t b1 = b0 + 8 < B ? b0 + 8 : B;
            for (int64_t j = 0; j < n_out; ++j)
                for (int32_t p = rowptr[j]; p < rowptr[j + 1]; ++p) {
                    int64_t i = colidx[p];
                    for (int32_t b = b0; b < b1; ++b)
                        acc[i * B + b] += (double)val[p] * (double)dz[j * ldo + b];
                }
        }
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n_in; ++i)
            for (int32_t b = 0; b < B; ++b) grad_x[i * ldgx + b] = (or_real)acc[i * B + b];
        free(acc);
    }
    return 0;
}

/* Dropout on the activations of a hidden layer (the paper's experiments train with a dropout rate
 * of 0.3; 0.4 at extreme scale).  Element (neuron j, sample b) is KEPT iff word (b & 3) of the Philox
 * draw with counter (j, b >> 2, purpose 4, step) is >= thr, thr = floor(p * 2^32); kept activations
 * are multiplied by scale = 1/(1-p) (inverted dropout), dropped ones are zero.  The same factor
 * multiplies the gradient that flows back. */
void or_dropout_keep(uint64_t seed, uint32_t layer_id, uint32_t step, int64_t n_out, int32_t B, uint32_t thr,
                     uint8_t *keep /* [n_out][B] */)
{
    for (int64_t j = 0; j < n_out; ++j)
        for (int32_t b = 0; b < B; ++b) {
            uint32_t key[2], ctr[4], w[4];
            key[0] = (uint32_t)seed ^ (uint32_t)(layer_id * 0x9E3779B9u);
            key[1] = (uint32_t)(seed >> 32);
            ctr[0] = (uint32_t)j; ctr[1] = (uint32_t)(b >> 2); ctr[2] = 4u; ctr[3] = step;
            or_philox4x32_10(ctr, key, w);
            keep[j * B + b] = w[b & 3] >= thr ? 1 : 0;
        }
}

void or_dropout_apply(float *a, const uint8_t *keep, int64_t n, float scale)
{
    for (int64_t t = 0; t < n; ++t) a[t] = keep[t] ? a[t] * scale : 0.0f;
}

/* Momentum SGD, eq. (1): w_{t+1} = w_t + mu (w_t - w_{t-1}) - eta grad.  With vel_t = w_t -
 * w_{t-1} (vel_0 = 0) this is vel <- mu*vel - eta*(grad + lambda*w);  w <- w + vel, evaluated in
 * fp32 in exactly this order (lambda = 0 in every workload). */
void or_update(int64_t n, or_real *val, or_real *vel, const or_real *grad, or_real lr, or_real momentum,
               or_real weight_decay)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        or_real g = grad[t] + weight_decay * val[t];
        or_real v = momentum * vel[t] - lr * g;
        vel[t] = v;
        val[t] = val[t] + v;
    }
}

/* ------------------------------------------------------------------------------------------ */
/* Algorithm 2, removal step.  Ordering key of a stored entry: (|w| as raw fp32 bits with the  */
/* sign cleared, flat position p = j*n_in + i); smaller keys are removed first.                */
/*   mode 0: remove the k = floor(zeta*nnz + 0.5) entries with the smallest keys.              */
/*   mode 1 (the algorithm's literal wording): split into P = {w >= 0} and N = {w < 0}; remove */
/*           floor(zeta*|P| + 0.5) smallest of P and floor(zeta*|N| + 0.5) of N closest to 0.  */
/* flat[p] must be ascending (CSR order).  remove[p] is set to 1/0.  Returns the number of     */
/* removed entries, or -2 on allocation failure.                                               */
/* ------------------------------------------------------------------------------------------ */
typedef struct { uint32_t mag; uint64_t pos; int64_t idx; } magpos;

static int cmp_magpos(const void *pa, const void *pb)
{
    const magpos *a = (const magpos *)pa, *b = (const magpos *)pb;
    if (a->mag != b->mag) return a->mag < b->mag ? -1 : 1;
    if (a->pos != b->pos) return a->pos < b->pos ? -1 : 1;
    return 0;
}

static int64_t round_half_up(double zeta, int64_t n)
{
    return (int64_t)floor(zeta * (double)n + 0.5);
}

static void remove_smallest(magpos *e, int64_t n, int64_t k, uint8_t *remove)
{
    qsort(e, (size_t)n, sizeof(magpos), cmp_magpos);
    for (int64_t t = 0; t < k && t < n; ++t) remove[e[t].idx] = 1;
}

int64_t or_prune_select(int64_t nnz, const float *val, const uint64_t *flat, double zeta, int mode,
                        uint8_t *remove)
{
    if (nnz < 0) return -1;
    magpos *pos_set = (magpos *)malloc(sizeof(magpos) * (size_t)(nnz > 0 ? nnz : 1));
    magpos *neg_set = (magpos *)malloc(sizeof(magpos) * (size_t)(nnz > 0 ? nnz : 1));
    if (!pos_set || !neg_set) { free(pos_set); free(neg_set); return -2; }
    memset(remove, 0, (size_t)nnz);
    int64_t n_pos = 0, n_neg = 0;
    for (int64_t p = 0; p < nnz; ++p) {
        uint32_t bits;
        memcpy(&bits, &val[p], 4);
        magpos e; e.mag = bits & 0x7FFFFFFFu; e.pos = flat[p]; e.idx = p;
        if (mode == 0 || val[p] >= 0.0f) pos_set[n_pos++] = e;   /* -0.0 >= 0 holds */
        else if (val[p] < 0.0f) neg_set[n_neg++] = e;
        else pos_set[n_pos++] = e;                               /* NaN: treated with P */
    }
    int64_t k_pos = round_half_up(zeta, n_pos), k_neg = round_half_up(zeta, n_neg);
    if (k_pos > n_pos) k_pos = n_pos;
    if (k_neg > n_neg) k_neg = n_neg;
    remove_smallest(pos_set, n_pos, k_pos, remove);
    remove_smallest(neg_set, n_neg, k_neg, remove);
    free(pos_set); free(neg_set);
    return k_pos + k_neg;
}

/* ------------------------------------------------------------------------------------------ */
/* Sparse model averaging, eq. (2): theta_f = (1/K) sum_i theta_i over K replicas whose topologies  */
/* have diverged; a connection absent from a replica counts as 0.  Input: the T stored entries of   */
/* all replicas sorted by flat position, entries of equal position in replica order.  Each run of   */
/* equal positions is added in fp32 in that order and divided by K.  Returns the size of the union. */
/* Algorithm 1's final step then keeps the largest magnitudes so that the sparsity level is        */
/* restored: or_keep_largest marks for removal everything but the n_keep largest (ordering key as   */
/* in or_prune_select: smaller (|w| bits, flat position) goes first).                               */
/* ------------------------------------------------------------------------------------------ */
int64_t or_average_sorted(int64_t T, const uint64_t *flat_sorted, const float *val_sorted, int32_t K,
                          uint64_t *out_flat, float *out_val)
{
    int64_t U = 0;
    int64_t x = 0;
    while (x < T) {
        float s = val_sorted[x];
        int64_t y = x + 1;
        while (y < T && flat_sorted[y] == flat_sorted[x]) { s = s + val_sorted[y]; ++y; }
        out_flat[U] = flat_sorted[x];
        out_val[U] = s / (float)K;
        ++U;
        x = y;
    }
    return U;
}

int64_t or_keep_largest(int64_t n, const float *val, const uint64_t *flat, int64_t n_keep, uint8_t *remove)
{
    if (n < 0) return -1;
    memset(remove, 0, (size_t)n);
    if (n_keep >= n) return 0;
    magpos *e = (magpos *)malloc(sizeof(magpos) * (size_t)(n > 0 ? n : 1));
    if (!e) return -2;
    for (int64_t p = 0; p < n; ++p) {
        uint32_t bits;
        memcpy(&bits, &val[p], 4);
        e[p].mag = bits & 0x7FFFFFFFu; e[p].pos = flat[p]; e[p].idx = p;
    }
    remove_smallest(e, n, n - n_keep, remove);
    free(e);
    return n - n_keep;
}

/* ------------------------------------------------------------------------------------------ */
/* Softmax + cross-entropy over C output neurons for B samples (feature-major z[c][b]).        */
/* p = softmax(z) in double with the maximum subtracted; loss = -(1/B) sum_b log p[y_b];       */
/* dz = (p - onehot(y)) / B rounded to fp32, B = the actual number of samples of this batch.   */
/* ------------------------------------------------------------------------------------------ */
double or_softmax_ce(const or_real *z, int64_t ldz, const int32_t *y, int32_t B, int32_t C,
                     or_real *dz, int64_t lddz)
{
    double loss = 0.0;
    for (int32_t b = 0; b < B; ++b) {
        double m = (double)z[b];
        for (int32_t c = 1; c < C; ++c)
            if ((double)z[c * ldz + b] > m) m = (double)z[c * ldz + b];
        double s = 0.0;
        for (int32_t c = 0; c < C; ++c) s += exp((double)z[c * ldz + b] - m);
        for (int32_t c = 0; c < C; ++c) {
            double p = exp((double)z[c * ldz + b] - m) / s;
            double t = (c == y[b]) ? 1.0 : 0.0;
            dz[c * lddz + b] = (or_real)((p - t) / (double)B);
        }
        loss -= ((double)z[(int64_t)y[b] * ldz + b] - m) - log(s);
    }
    return loss / (double)B;
}

/* Neuron importance, eq. (4), evaluated in the paper's precision: fp32 additions of |w| in stored
 * (CSR) order.  This is the value the Importance Pruning decision "I < t" of Algorithm 2 is taken
 * on, so that the decision does not depend on who evaluates it. */
void or_importance_f32(int64_t n_out, const int32_t *rowptr, const float *val, float *importance)
{
    for (int64_t j = 0; j < n_out; ++j) {
        float s = 0.0f;
        for (int32_t p = rowptr[j]; p < rowptr[j + 1]; ++p) s = s + fabsf(val[p]);
        importance[j] = s;
    }
}

/* Neuron importance, eq. (4): I_j = sum over incoming connections of |w_ij| (row sums of |Wt|). */
void or_importance(int64_t n_out, const int32_t *rowptr, const float *val, float *importance)
{
    for (int64_t j = 0; j < n_out; ++j) {
        double s = 0.0;
        for (int32_t p = rowptr[j]; p < rowptr[j + 1]; ++p) s += fabs((double)val[p]);
        importance[j] = (float)s;
    }
}
