// C ABI of libsparse_set.so (see include/sparse_set.h): argument checking, carving of the caller's
// state and scratch buffers, call-order tracking.  No kernel lives here.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <thread>
#include <vector>

#include "sl_internal.h"

namespace sl {

int set_err(sl_layer *L, int code, const char *fmt, ...)
{
    if (L) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(L->err, sizeof(L->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t take(size_t &cursor, size_t bytes)
{
    const size_t at = cursor;
    cursor = align_up(cursor + bytes);
    return at;
}

int64_t config_nnz(const sl_config &c)
{
    const double total = (double)c.n_in * (double)c.n_out;
    double want = c.nnz_override >= 0 ? (double)c.nnz_override : floor(c.epsilon * (double)(c.n_in + c.n_out) + 0.5);
    if (want > total) want = total;
    if (want < 0) want = 0;
    return (int64_t)want;
}

// Rows longer than the returned length are cut into virtual rows.  Matrices with at least 64 rows of
// moderate mean length (every Erdos-Renyi layer) keep their rows whole unless one is far above the
// mean; matrices with few or very long rows (narrow dense output layers: 2 or 10 rows of up to 10^6
// entries) are cut so that about 8192 groups exist.
int choose_seg(int64_t n_rows, int64_t nnz)
{
    const int64_t mean = (nnz + n_rows - 1) / (n_rows > 0 ? n_rows : 1);
    int64_t seg;
    if (n_rows >= 64 && mean <= 512) seg = 4 * mean;
    else seg = (nnz + 8191) / 8192;
    if (seg < 64) seg = 64;
    if (seg > (1 << 30)) seg = 1 << 30;
    return (int)seg;
}

// Window of candidates that yields k accepted positions with overwhelming probability: the
// expected number of draws is M*ln((M-occ)/(M-occ-k)); 5 % and eight standard deviations are
// added on top.
int64_t sampler_window(double M, double n_occ, double k)
{
    if (k <= 0) return 0;
    const double rest = M - n_occ - k;
    const double expect = rest > 0 ? M * log1p(k / rest) : 64.0 * M;
    return (int64_t)ceil(1.05 * expect + 8.0 * sqrt(expect) + 1024.0);
}

static int round_up32(int x) { return (x + 31) & ~31; }

int plan_state(const sl_config &c, int64_t nnz, StatePlan *sp)
{
    size_t cur = 0;
    const size_t n = (size_t)nnz, ni = (size_t)c.n_in, no = (size_t)c.n_out;
    const size_t ldz = (size_t)round_up32(c.max_batch);
    const bool csc = (c.flags & SL_FLAG_NEED_INPUT_GRAD) != 0;
    sp->rowptr = take(cur, 4 * (no + 1));
    sp->colidx = take(cur, 4 * n);
    sp->val = take(cur, 4 * n);
    sp->vel = take(cur, 4 * n);
    sp->grad = take(cur, 4 * n);
    sp->bias = take(cur, 4 * no);
    sp->bias_vel = take(cur, 4 * no);
    sp->grad_bias = take(cur, 4 * no);
    if (csc) {
        sp->colptr = take(cur, 4 * (ni + 1));
        sp->rowidx = take(cur, 4 * n);
        sp->csr_pos = take(cur, 4 * n);
        sp->valT = take(cur, 4 * n);
        sp->velT = take(cur, 4 * n);
    }
    sp->mask = take(cur, no * (ldz / 4));
    sp->dz = take(cur, 4 * no * ldz);
    sp->nv_cap_f = (int)(no + n / 64 + 2);
    sp->f_vptr = take(cur, 4 * ((size_t)sp->nv_cap_f + 1));
    sp->f_v2row = take(cur, 4 * (size_t)sp->nv_cap_f);
    sp->f_rvptr = take(cur, 4 * (no + 1));
    if (csc) {
        sp->nv_cap_b = (int)(ni + n / 64 + 2);
        sp->b_vptr = take(cur, 4 * ((size_t)sp->nv_cap_b + 1));
        sp->b_v2row = take(cur, 4 * (size_t)sp->nv_cap_b);
        sp->b_rvptr = take(cur, 4 * (ni + 1));
    }
    sp->sel = take(cur, 2 * sizeof(SelState));
    sp->total = cur;
    return SL_OK;
}

int plan_scratch(const sl_config &c, int64_t nnz, ScratchPlan *cp)
{
    const size_t n = (size_t)nnz, ni = (size_t)c.n_in, no = (size_t)c.n_out;
    const size_t ldz = (size_t)round_up32(c.max_batch);
    const bool csc = (c.flags & SL_FLAG_NEED_INPUT_GRAD) != 0;
    const double M = (double)c.n_in * (double)c.n_out;
    cp->dense_mode = M <= 4.0 * (double)nnz;
    // Importance Pruning can shrink nnz, which can move a dense-mode layer into the sparse mode (never
    // the other way round); the window is sized for whichever needs more.
    const double k_sparse = (double)nnz < floor(M / 4.0) ? (double)nnz : floor(M / 4.0);
    cp->w_cap = 2 * sampler_window(M, 0.0, k_sparse);
    if (cp->dense_mode && cp->w_cap < (int64_t)M) cp->w_cap = (int64_t)M;
    if (cp->w_cap < (int64_t)n) cp->w_cap = (int64_t)n;
    const size_t w = (size_t)cp->w_cap;
    // the regions of the training passes and of init/evolve never live at the same time
    size_t cur = 0;
    const size_t nv_cap = (no > (csc ? ni : 0) ? no : ni) + n / 64 + 2;
    cp->partial = take(cur, 4 * nv_cap * ldz);
    const size_t train_end = cur;
    cur = 0;
    cp->tie64 = take(cur, 8 * (n + 1));
    cp->trank = take(cur, 8 * (n + 1));
    cp->keep = take(cur, 4 * (n + 1));
    cp->kscan = take(cur, 4 * (n + 1));
    cp->s_col = take(cur, 4 * n);
    cp->s_val = take(cur, 4 * n);
    cp->s_vel = take(cur, 4 * n);
    cp->rowptr_s = take(cur, 4 * (no + 1));
    cp->new_p = take(cur, 8 * n);
    cp->keyA = take(cur, 8 * w);
    cp->keyB = take(cur, 8 * w);
    cp->payA = take(cur, 4 * w);
    cp->payB = take(cur, 4 * w);
    const size_t fl = (w > (ni > no ? ni : no) ? w : (ni > no ? ni : no)) + 1;
    cp->f0 = take(cur, 4 * fl);
    cp->f1 = take(cur, 4 * fl);
    cp->f2 = take(cur, 4 * fl);
    cp->f3 = take(cur, 4 * fl);
    cp->temp_bytes = ((size_t)32 << 20) + 2 * (w > n ? w : n);
    cp->temp = take(cur, cp->temp_bytes);
    cp->small = take(cur, 1024);
    cp->packed = take(cur, csc ? 16 * n : 0);   // (row, weight, velocity) per CSR slot while the transposed view is rebuilt
    cp->total = cur > train_end ? cur : train_end;
    return SL_OK;
}

static int check_config(const sl_config *c, int64_t *nnz_out)
{
    if (!c) return SL_EINVAL;
    if (c->n_in <= 0 || c->n_out <= 0 || c->max_batch <= 0) return SL_EINVAL;
    if (c->nnz_override < -1 || (c->nnz_override < 0 && !(c->epsilon >= 0.0))) return SL_EINVAL;
    if (c->act_kind < 0 || c->act_kind > 1 || c->act_parity < 0 || c->act_parity > 1) return SL_EINVAL;
    if (c->prune_mode < 0 || c->prune_mode > 1) return SL_EINVAL;
    if (!(c->init_limit > 0.f)) return SL_EINVAL;
    if (c->n_in >= ((int64_t)1 << 31) - 1 || c->n_out >= ((int64_t)1 << 31) - 1) return SL_EOVERFLOW;
    if (c->max_batch > (1 << 20)) return SL_EOVERFLOW;
    const int64_t nnz = config_nnz(*c);
    // 32-bit offsets and 32-bit sampler payloads
    if (nnz >= ((int64_t)1 << 30)) return SL_EOVERFLOW;
    const double M = (double)c->n_in * (double)c->n_out;
    if (M <= 4.0 * (double)nnz && M >= 2147483647.0) return SL_EOVERFLOW;
    const double k_sparse = (double)nnz < floor(M / 4.0) ? (double)nnz : floor(M / 4.0);
    if (2 * sampler_window(M, 0.0, k_sparse) >= ((int64_t)1 << 32) - 2) return SL_EOVERFLOW;
    *nnz_out = nnz;
    return SL_OK;
}

}  // namespace sl

using namespace sl;

extern "C" {

int sparse_layer_query_sizes(const sl_config *cfg, size_t *state_bytes, size_t *scratch_bytes)
{
    int64_t nnz = 0;
    int rc = check_config(cfg, &nnz);
    if (rc) return rc;
    StatePlan sp;
    ScratchPlan cp;
    plan_state(*cfg, nnz, &sp);
    plan_scratch(*cfg, nnz, &cp);
    if (state_bytes) *state_bytes = sp.total;
    if (scratch_bytes) *scratch_bytes = cp.total;
    return SL_OK;
}

int sparse_layer_init(const sl_config *cfg, void *state_dev, size_t state_bytes, void *scratch_dev,
                      size_t scratch_bytes, void *hip_stream, sl_layer **out)
{
    if (!out) return SL_EINVAL;
    *out = nullptr;
    int64_t nnz = 0;
    int rc = check_config(cfg, &nnz);
    if (rc) return rc;
    if (!state_dev || !scratch_dev) return SL_EINVAL;
    if (((uintptr_t)state_dev & 255) || ((uintptr_t)scratch_dev & 255)) return SL_EINVAL;
    sl_layer *L = new (std::nothrow) sl_layer();
    if (!L) return SL_ENOMEM;
    L->cfg = *cfg;
    L->nnz = nnz;
    plan_state(*cfg, nnz, &L->sp);
    plan_scratch(*cfg, nnz, &L->cp);
    if (state_bytes < L->sp.total || scratch_bytes < L->cp.total) {
        delete L;
        return SL_ENOMEM;
    }
    L->ldz = round_up32(cfg->max_batch);
    L->ldm = L->ldz / 4;
    L->has_csc = (cfg->flags & SL_FLAG_NEED_INPUT_GRAD) != 0;
    L->state = (char *)state_dev; L->state_bytes = state_bytes;
    L->scratch = (char *)scratch_dev; L->scratch_bytes = scratch_bytes;
    char *b = L->state;
    const StatePlan &sp = L->sp;
    L->rowptr = (int *)(b + sp.rowptr); L->colidx = (int *)(b + sp.colidx);
    L->val = (float *)(b + sp.val); L->vel = (float *)(b + sp.vel); L->grad = (float *)(b + sp.grad);
    L->bias = (float *)(b + sp.bias); L->bias_vel = (float *)(b + sp.bias_vel); L->grad_bias = (float *)(b + sp.grad_bias);
    if (L->has_csc) {
        L->colptr = (int *)(b + sp.colptr); L->rowidx = (int *)(b + sp.rowidx); L->csr_pos = (int *)(b + sp.csr_pos);
        L->valT = (float *)(b + sp.valT); L->velT = (float *)(b + sp.velT);
        L->bwd.vptr_store = (int *)(b + sp.b_vptr); L->bwd.v2row_store = (int *)(b + sp.b_v2row);
        L->bwd.rvptr_store = (int *)(b + sp.b_rvptr); L->bwd.nv_cap = sp.nv_cap_b;
    }
    L->mask = (uint8_t *)(b + sp.mask); L->dz = (float *)(b + sp.dz);
    L->fwd.vptr_store = (int *)(b + sp.f_vptr); L->fwd.v2row_store = (int *)(b + sp.f_v2row);
    L->fwd.rvptr_store = (int *)(b + sp.f_rvptr); L->fwd.nv_cap = sp.nv_cap_f;
    L->sel = (SelState *)(b + sp.sel);
    hipStream_t s = (hipStream_t)hip_stream;
    L->last_stream = s;
    rc = topo_init(L, s);
    if (rc == SL_OK) rc = static_scratch_setup(L, nullptr);   // address of the built-in buffer on this device
    if (rc == SL_OK) {
        hipError_t e = hipStreamSynchronize(s);
        if (e != hipSuccess) rc = SL_EHIP;
    }
    if (rc) {
        delete L;
        return rc;
    }
    *out = L;
    return SL_OK;
}

static int check_dense(sl_layer *L, const void *p, int64_t ld, int B, const char *what)
{
    if (!p) return set_err(L, SL_EINVAL, "%s is null", what);
    if (ld < B || (ld & 3) || ld > INT32_MAX)
        return set_err(L, SL_EINVAL, "%s: leading dimension %lld must be >= B, a multiple of 4 and below 2^31", what, (long long)ld);
    if ((uintptr_t)p & 15) return set_err(L, SL_EINVAL, "%s must be 16-byte aligned", what);
    return SL_OK;
}

int sparse_layer_forward(sl_layer *L, const float *x_dev, int64_t ldx, int32_t B, float *a_dev, int64_t lda,
                         void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (B <= 0 || B > L->cfg.max_batch) return set_err(L, SL_EINVAL, "B = %d outside 1..max_batch = %d", B, L->cfg.max_batch);
    int rc = check_dense(L, x_dev, ldx, B, "x");
    if (rc) return rc;
    rc = check_dense(L, a_dev, lda, B, "a");
    if (rc) return rc;
    L->last_stream = (hipStream_t)hip_stream;
    rc = launch_forward(L, x_dev, ldx, B, a_dev, lda, true, L->last_stream);
    if (rc) return rc;
    L->phase = 1;
    L->last_B = B;
    L->dz_ready = 0;
    return SL_OK;
}

int sparse_layer_infer(sl_layer *L, const float *x_dev, int64_t ldx, int32_t B, float *a_dev, int64_t lda,
                       void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (B <= 0 || B > L->cfg.max_batch) return set_err(L, SL_EINVAL, "B = %d outside 1..max_batch = %d", B, L->cfg.max_batch);
    int rc = check_dense(L, x_dev, ldx, B, "x");
    if (rc) return rc;
    rc = check_dense(L, a_dev, lda, B, "a");
    if (rc) return rc;
    L->last_stream = (hipStream_t)hip_stream;
    return launch_forward(L, x_dev, ldx, B, a_dev, lda, false, L->last_stream);
}

int sparse_layer_infer_static(sl_layer *L, const float *x_dev, int64_t ldx, int32_t B, float *a_dev, int64_t lda,
                              void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (B <= 0 || B > L->cfg.max_batch) return set_err(L, SL_EINVAL, "B = %d outside 1..max_batch = %d", B, L->cfg.max_batch);
    int rc = check_dense(L, x_dev, ldx, B, "x");
    if (rc) return rc;
    rc = check_dense(L, a_dev, lda, B, "a");
    if (rc) return rc;
    L->last_stream = (hipStream_t)hip_stream;
    return launch_forward_static(L, x_dev, ldx, B, a_dev, lda, L->last_stream);
}

int sparse_layer_set_dropout(sl_layer *L, float p, uint64_t step)
{
    if (!L) return SL_EINVAL;
    if (!(p >= 0.f && p < 1.f)) return set_err(L, SL_EINVAL, "dropout rate %g outside [0,1)", (double)p);
    if (p > 0.f && L->cfg.act_kind == 0) return set_err(L, SL_EINVAL, "dropout applies to hidden (All-ReLU) layers only");
    if (L->phase == 1) return set_err(L, SL_ESTATE, "set_dropout between forward and backward");
    L->drop_thr = (uint32_t)floor((double)p * 4294967296.0);
    L->drop_scale = 1.0f / (1.0f - p);
    L->drop_step = (uint32_t)step;
    return SL_OK;
}

int sparse_layer_link_producer(sl_layer *L, sl_layer *producer)
{
    if (!L) return SL_EINVAL;
    if (!producer) { L->producer = nullptr; return SL_OK; }
    if (producer == L) return set_err(L, SL_EINVAL, "a layer cannot be its own producer");
    if (!L->has_csc) return set_err(L, SL_EINVAL, "link: the layer was created without SL_FLAG_NEED_INPUT_GRAD");
    if (producer->cfg.n_out != L->cfg.n_in)
        return set_err(L, SL_EINVAL, "link: producer has %lld outputs, layer has %lld inputs",
                       (long long)producer->cfg.n_out, (long long)L->cfg.n_in);
    if (producer->cfg.max_batch < L->cfg.max_batch)
        return set_err(L, SL_EINVAL, "link: producer max_batch %d < layer max_batch %d", producer->cfg.max_batch,
                       L->cfg.max_batch);
    L->producer = producer;
    return SL_OK;
}

int sparse_layer_backward(sl_layer *L, const float *x_dev, int64_t ldx, const float *grad_a_dev, int64_t ldg,
                          int32_t B, float *grad_x_dev, int64_t ldgx, void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (L->phase < 1) return set_err(L, SL_ESTATE, "backward called before forward");
    if (B != L->last_B) return set_err(L, SL_ESTATE, "backward with B = %d after forward with B = %d", B, L->last_B);
    int rc = check_dense(L, x_dev, ldx, B, "x");
    if (rc) return rc;
    if (grad_a_dev || L->dz_ready != B) {
        L->dz_ready = 0;   // an explicit grad_a overrides anything a consumer handed over
        rc = check_dense(L, grad_a_dev, ldg, B, "grad_a");
        if (rc) return rc;
    }
    if (L->has_csc) {
        if (grad_x_dev) {
            rc = check_dense(L, grad_x_dev, ldgx, B, "grad_x");
            if (rc) return rc;
        } else if (!L->producer) {
            return set_err(L, SL_EINVAL, "grad_x is null and no producer layer is linked");
        } else if (L->producer->phase < 1 || L->producer->last_B != B) {
            return set_err(L, SL_ESTATE, "linked producer has not run forward with B = %d", B);
        }
    } else if (grad_x_dev) {
        return set_err(L, SL_EINVAL, "grad_x given but the layer was created without SL_FLAG_NEED_INPUT_GRAD");
    }
    L->last_stream = (hipStream_t)hip_stream;
    rc = launch_backward(L, x_dev, ldx, grad_a_dev, ldg, B, grad_x_dev, ldgx, L->last_stream);
    if (rc) return rc;
    L->phase = 2;
    return SL_OK;
}

int sparse_layer_update(sl_layer *L, void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (L->phase < 2) return set_err(L, SL_ESTATE, "update called before backward");
    L->last_stream = (hipStream_t)hip_stream;
    int rc = launch_update(L, L->last_stream);
    if (rc) return rc;
    L->phase = 0;
    L->weights_updated = false;
    return SL_OK;
}

int sparse_layer_set_fused_update(sl_layer *L, int32_t mode)
{
    if (!L) return SL_EINVAL;
    if (mode < 0 || mode > 2) return set_err(L, SL_EINVAL, "fused update mode %d outside 0..2", mode);
    if (L->phase == 2) return set_err(L, SL_ESTATE, "set_fused_update between backward and update");
    L->fuse_mode = mode;
    return SL_OK;
}

int sparse_layer_evolve(sl_layer *L, double zeta, uint64_t generation, void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (!(zeta >= 0.0 && zeta <= 1.0)) return set_err(L, SL_EINVAL, "zeta = %g outside [0,1]", zeta);
    if (generation == 0 || generation >= ((uint64_t)1 << 32)) return set_err(L, SL_EINVAL, "generation must be in 1..2^32-1");
    L->last_stream = (hipStream_t)hip_stream;
    int rc = topo_evolve(L, zeta, (uint32_t)generation, L->last_stream);
    if (rc) return rc;
    hipError_t e = hipStreamSynchronize(L->last_stream);
    if (e != hipSuccess) return set_err(L, SL_EHIP, "evolve: %s", hipGetErrorString(e));
    L->phase = 0;
    L->weights_updated = false;
    return SL_OK;
}

int sparse_layers_evolve(sl_layer *const *layers, int32_t count, double zeta, uint64_t generation, void *const *hip_streams)
{
    if (!layers || !hip_streams || count < 1 || count > SL_MAX_MULTI) return SL_EINVAL;
    for (int k = 0; k < count; ++k) {
        if (!layers[k]) return SL_EINVAL;
        for (int j = 0; j < k; ++j) {
            const char *a = layers[j]->scratch, *b = layers[k]->scratch;
            if (layers[j] == layers[k] || (a < b + layers[k]->scratch_bytes && b < a + layers[j]->scratch_bytes))
                return set_err(layers[k], SL_EINVAL, "layers %d and %d share a scratch buffer: they cannot evolve concurrently", j, k);
        }
    }
    int dev = 0;
    SL_HIP(layers[0], hipGetDevice(&dev));
    // The cycles of different layers touch nothing in common; each runs from a host thread of its own so that the
    // waits of one layer (survivor count, accepted candidates, longest row) overlap the kernels of the others.
    std::vector<int> rc((size_t)count, SL_OK);
    std::vector<std::thread> workers;
    std::vector<int> inline_later;   // layers for which no thread could be started: they run on this one
    for (int k = 1; k < count; ++k) {
        try {
            workers.emplace_back([&, k] {
                hipError_t e = hipSetDevice(dev);
                rc[k] = e != hipSuccess ? set_err(layers[k], SL_EHIP, "hipSetDevice: %s", hipGetErrorString(e))
                                        : sparse_layer_evolve(layers[k], zeta, generation, hip_streams[k]);
            });
        } catch (...) {
            inline_later.push_back(k);
        }
    }
    rc[0] = sparse_layer_evolve(layers[0], zeta, generation, hip_streams[0]);
    for (int k : inline_later) rc[k] = sparse_layer_evolve(layers[k], zeta, generation, hip_streams[k]);
    for (auto &w : workers) w.join();
    for (int k = 0; k < count; ++k)
        if (rc[k]) return rc[k];
    return SL_OK;
}

int sparse_layer_set_sampler_window(sl_layer *L, int64_t first_window, int64_t max_window)
{
    if (!L) return SL_EINVAL;
    if (first_window < 0 || max_window < 0) return set_err(L, SL_EINVAL, "sampler window must not be negative");
    L->sampler_first = first_window;
    L->sampler_max = max_window;
    return SL_OK;
}

int sparse_layer_retain_valid_updates(sl_layer *L, const int32_t *old_rowptr_dev, const int32_t *old_colidx_dev,
                                      const float *old_grad_dev, int64_t old_nnz, const float *old_grad_bias_dev,
                                      void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (!old_rowptr_dev || !old_grad_bias_dev) return set_err(L, SL_EINVAL, "retain_valid_updates: null rowptr or bias gradient");
    if (old_nnz < 0 || old_nnz > INT32_MAX) return set_err(L, SL_EINVAL, "retain_valid_updates: old_nnz = %lld", (long long)old_nnz);
    if (old_nnz > 0 && (!old_colidx_dev || !old_grad_dev)) return set_err(L, SL_EINVAL, "retain_valid_updates: null colidx or gradient");
    if (L->phase == 1) return set_err(L, SL_ESTATE, "retain_valid_updates between forward and backward");
    L->last_stream = (hipStream_t)hip_stream;
    int rc = topo_retain_valid(L, old_rowptr_dev, old_colidx_dev, old_grad_dev, old_nnz, L->last_stream);
    if (rc) return rc;
    SL_HIP(L, hipMemcpyAsync(L->grad_bias, old_grad_bias_dev, sizeof(float) * (size_t)L->cfg.n_out, hipMemcpyDeviceToDevice,
                             L->last_stream));
    L->phase = 2;
    L->dz_ready = 0;
    L->weights_updated = false;
    L->grad_stored = true;
    return SL_OK;
}

int sparse_layer_importance(sl_layer *L, float *importance_host)
{
    if (!L || !importance_host) return SL_EINVAL;
    float *imp = (float *)(L->scratch + L->cp.f0);
    int rc = topo_importance(L, imp, L->last_stream);
    if (rc) return rc;
    SL_HIP(L, hipMemcpyAsync(importance_host, imp, sizeof(float) * (size_t)L->cfg.n_out, hipMemcpyDeviceToHost, L->last_stream));
    SL_HIP(L, hipStreamSynchronize(L->last_stream));
    return SL_OK;
}

int sparse_layer_importance_prune(sl_layer *L, float threshold, int64_t *removed, void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (threshold != threshold) return set_err(L, SL_EINVAL, "threshold is NaN");
    L->last_stream = (hipStream_t)hip_stream;
    int rc = topo_importance_prune(L, threshold, removed, L->last_stream);
    if (rc) return rc;
    SL_HIP(L, hipStreamSynchronize(L->last_stream));
    L->phase = 0;
    L->dz_ready = 0;
    return SL_OK;
}

int sparse_layers_average_query(int64_t total_entries, size_t *scratch_bytes)
{
    if (total_entries < 0 || total_entries >= ((int64_t)1 << 32) - 2 || !scratch_bytes) return SL_EINVAL;
    *scratch_bytes = average_scratch_bytes(total_entries);
    return SL_OK;
}

int sparse_layers_average(sl_layer *dst, sl_layer *const *replicas, int32_t K, void *scratch_dev, size_t scratch_bytes,
                          void *hip_stream)
{
    if (!dst || !replicas) return SL_EINVAL;
    if (K < 1 || K > 16) return set_err(dst, SL_EINVAL, "average: K = %d outside 1..16", K);
    if (!scratch_dev || ((uintptr_t)scratch_dev & 255)) return set_err(dst, SL_EINVAL, "average: scratch null or not 256-byte aligned");
    int64_t total = 0;
    for (int k = 0; k < K; ++k) {
        const sl_layer *R = replicas[k];
        if (!R) return set_err(dst, SL_EINVAL, "average: replica %d is null", k);
        if (R->cfg.n_in != dst->cfg.n_in || R->cfg.n_out != dst->cfg.n_out)
            return set_err(dst, SL_EINVAL, "average: replica %d has another shape", k);
        total += R->nnz;
    }
    if (total >= ((int64_t)1 << 32) - 2) return set_err(dst, SL_EOVERFLOW, "average: %lld entries in total", (long long)total);
    hipStream_t s = (hipStream_t)hip_stream;
    dst->last_stream = s;
    int rc = topo_average(dst, replicas, K, (char *)scratch_dev, scratch_bytes, s);
    if (rc) return rc;
    SL_HIP(dst, hipStreamSynchronize(s));
    dst->phase = 0;
    dst->dz_ready = 0;
    return SL_OK;
}

static void drop_profile(sl_layer *L)
{
    for (auto &r : L->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    L->prof.clear();
}

int sparse_layer_profile_begin(sl_layer *L)
{
    if (!L) return SL_EINVAL;
    drop_profile(L);
    L->prof_on = true;
    return SL_OK;
}

int sparse_layer_profile_end(sl_layer *L, int32_t *launches, float *total_ms, int32_t n_ids)
{
    if (!L) return SL_EINVAL;
    L->prof_on = false;
    for (int i = 0; i < n_ids; ++i) {
        if (launches) launches[i] = 0;
        if (total_ms) total_ms[i] = 0.f;
    }
    int rc = SL_OK;
    for (auto &r : L->prof) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess) { rc = set_err(L, SL_EHIP, "profile: %s", hipGetErrorString(e)); break; }
        if (r.id < n_ids) {
            if (launches) launches[r.id] += 1;
            if (total_ms) total_ms[r.id] += ms;
        }
    }
    drop_profile(L);
    return rc;
}

const char *sparse_kernel_name(int32_t id)
{
    static const char *names[K_COUNT] = {"forward_spmm", "forward_fixup", "act_grad", "backward_fused",
                                         "sddmm", "backward_fixup", "update"};
    return (id >= 0 && id < K_COUNT) ? names[id] : "";
}

int sparse_layer_destroy(sl_layer *L)
{
    if (!L) return SL_EINVAL;
    drop_profile(L);
    delete L;
    return SL_OK;
}

int sparse_loss_softmax_ce(const float *z_dev, int64_t ldz, const int32_t *y_dev, int32_t B, int32_t C, float *dz_dev,
                           int64_t lddz, float *loss_sum_dev, void *hip_stream)
{
    if (!z_dev || !y_dev || !dz_dev || B <= 0 || C <= 0 || C > 1024 || ldz < B || lddz < B) return SL_EINVAL;
    return launch_softmax_ce(z_dev, ldz, y_dev, B, C, dz_dev, lddz, loss_sum_dev, nullptr, (hipStream_t)hip_stream);
}

int sparse_loss_softmax_ce_into(sl_layer *L, const float *z_dev, int64_t ldz, const int32_t *y_dev, int32_t B,
                                float *loss_sum_dev, void *hip_stream)
{
    if (!L) return SL_EINVAL;
    if (L->cfg.act_kind != 0) return set_err(L, SL_EINVAL, "loss_into: the layer must be an output layer (identity activation)");
    if (L->phase < 1 || L->last_B != B) return set_err(L, SL_ESTATE, "loss_into: the layer has not run forward with B = %d", B);
    if (!z_dev || !y_dev || ldz < B || L->cfg.n_out > 1024) return set_err(L, SL_EINVAL, "loss_into: bad argument");
    L->last_stream = (hipStream_t)hip_stream;
    int rc = launch_softmax_ce(z_dev, ldz, y_dev, B, (int)L->cfg.n_out, L->dz, L->ldz, loss_sum_dev, L->grad_bias, L->last_stream);
    if (rc) return set_err(L, rc, "loss_into: launch failed");
    L->dz_ready = B;
    return SL_OK;
}

int sparse_layers_update(sl_layer *const *layers, int32_t count, void *hip_stream)
{
    if (!layers || count < 1 || count > SL_MAX_MULTI) return SL_EINVAL;
    for (int k = 0; k < count; ++k) {
        if (!layers[k]) return SL_EINVAL;
        if (layers[k]->phase < 2) return set_err(layers[k], SL_ESTATE, "update called before backward");
    }
    hipStream_t s = (hipStream_t)hip_stream;
    int rc = launch_update_many(layers, count, s);
    if (rc) return rc;
    for (int k = 0; k < count; ++k) {
        layers[k]->phase = 0;
        layers[k]->weights_updated = false;
        layers[k]->last_stream = s;
    }
    return SL_OK;
}

int sparse_layer_nnz(const sl_layer *L, int64_t *nnz)
{
    if (!L || !nnz) return SL_EINVAL;
    *nnz = L->nnz;
    return SL_OK;
}

static int copy_out(sl_layer *L, void *host, const void *dev, size_t bytes)
{
    if (!host || bytes == 0) return SL_OK;
    SL_HIP(L, hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, L->last_stream));
    return SL_OK;
}

int sparse_layer_export_csr(sl_layer *L, int32_t *rowptr, int32_t *colidx, float *val, float *vel, float *bias,
                            float *bias_vel)
{
    if (!L) return SL_EINVAL;
    int rc = SL_OK;
    if (vel) rc = topo_sync_csr_vel(L, L->last_stream);
    const size_t n = (size_t)L->nnz, no = (size_t)L->cfg.n_out;
    if (!rc) rc = copy_out(L, rowptr, L->rowptr, 4 * (no + 1));
    if (!rc) rc = copy_out(L, colidx, L->colidx, 4 * n);
    if (!rc) rc = copy_out(L, val, L->val, 4 * n);
    if (!rc) rc = copy_out(L, vel, L->vel, 4 * n);
    if (!rc) rc = copy_out(L, bias, L->bias, 4 * no);
    if (!rc) rc = copy_out(L, bias_vel, L->bias_vel, 4 * no);
    if (rc) return rc;
    SL_HIP(L, hipStreamSynchronize(L->last_stream));
    return SL_OK;
}

int sparse_layer_import_csr(sl_layer *L, const int32_t *rowptr, const int32_t *colidx, const float *val,
                            const float *vel, const float *bias, const float *bias_vel)
{
    if (!L || !rowptr || !colidx || !val) return SL_EINVAL;
    const int64_t n = L->nnz, no = L->cfg.n_out, ni = L->cfg.n_in;
    if (rowptr[0] != 0 || rowptr[no] != n) return set_err(L, SL_EINVAL, "import: rowptr does not describe %lld entries", (long long)n);
    for (int64_t r = 0; r < no; ++r) {
        if (rowptr[r + 1] < rowptr[r]) return set_err(L, SL_EINVAL, "import: rowptr decreases at row %lld", (long long)r);
        for (int32_t p = rowptr[r]; p < rowptr[r + 1]; ++p) {
            if (colidx[p] < 0 || colidx[p] >= ni) return set_err(L, SL_EINVAL, "import: column out of range at %d", p);
            if (p > rowptr[r] && colidx[p] <= colidx[p - 1]) return set_err(L, SL_EINVAL, "import: row %lld not strictly ascending", (long long)r);
        }
    }
    hipStream_t s = L->last_stream;
    SL_HIP(L, hipStreamSynchronize(s));
    SL_HIP(L, hipMemcpy(L->rowptr, rowptr, 4 * (size_t)(no + 1), hipMemcpyHostToDevice));
    if (n > 0) {
        SL_HIP(L, hipMemcpy(L->colidx, colidx, 4 * (size_t)n, hipMemcpyHostToDevice));
        SL_HIP(L, hipMemcpy(L->val, val, 4 * (size_t)n, hipMemcpyHostToDevice));
        if (vel) SL_HIP(L, hipMemcpy(L->vel, vel, 4 * (size_t)n, hipMemcpyHostToDevice));
        else SL_HIP(L, hipMemset(L->vel, 0, 4 * (size_t)n));
    }
    if (bias) SL_HIP(L, hipMemcpy(L->bias, bias, 4 * (size_t)no, hipMemcpyHostToDevice));
    if (bias_vel) SL_HIP(L, hipMemcpy(L->bias_vel, bias_vel, 4 * (size_t)no, hipMemcpyHostToDevice));
    int rc = topo_finalize(L, s);
    if (rc) return rc;
    SL_HIP(L, hipStreamSynchronize(s));
    L->phase = 0;
    L->weights_updated = false;
    return SL_OK;
}

int sparse_layer_export_grad(sl_layer *L, float *grad_val, float *grad_bias)
{
    if (!L) return SL_EINVAL;
    if (L->phase < 2) return set_err(L, SL_ESTATE, "no gradient: backward has not run since the last update");
    if (grad_val && !L->grad_stored) return set_err(L, SL_ESTATE, "no gradient: the fused update (mode 1) does not store it");
    const size_t n = (size_t)L->nnz, no = (size_t)L->cfg.n_out;
    int rc = SL_OK;
    if (grad_val && n > 0) {
        if (L->has_csc) {
            // gradients live in CSC order; stage a CSR-ordered copy in scratch
            float *tmp = (float *)(L->scratch + L->cp.s_val);
            rc = topo_sync_csr_grad(L, tmp, L->last_stream);
            if (!rc) rc = copy_out(L, grad_val, tmp, 4 * n);
        } else {
            rc = copy_out(L, grad_val, L->grad, 4 * n);
        }
    }
    if (!rc) rc = copy_out(L, grad_bias, L->grad_bias, 4 * no);
    if (rc) return rc;
    SL_HIP(L, hipStreamSynchronize(L->last_stream));
    return SL_OK;
}

int sparse_layer_set_lr(sl_layer *L, float lr)
{
    if (!L) return SL_EINVAL;
    L->cfg.lr = lr;
    return SL_OK;
}

const char *sparse_layer_last_error(const sl_layer *L) { return L ? L->err : "null layer"; }

}  // extern "C"
