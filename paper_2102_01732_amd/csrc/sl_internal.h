// Internal declarations shared by the translation units of libsparse_set.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "sparse_set.h"

#define SL_MAX_MULTI 16   // layers per multi-layer launch

namespace sl {

// One orientation of the sparse matrix (CSR of Wt for the forward pass, CSC of Wt for the
// backward pass) together with its work decomposition.  A "virtual row" (vrow) is a run of at
// most `seg` consecutive stored entries of one row; rows longer than `seg` are cut into several
// vrows so that narrow layers (2 or 10 output neurons with up to 10^6 inputs each) still spread
// over the whole chip.  When no row is longer than `seg`, vptr aliases ptr and v2row is null.
struct SegMat {
    int n_rows = 0;
    int *ptr = nullptr;    // [n_rows+1] offsets into idx
    int *idx = nullptr;    // [nnz] index of the other dimension
    int *vptr = nullptr;   // [nv+1]
    int *v2row = nullptr;  // [nv] or null
    int *rvptr = nullptr;  // [n_rows+1] first vrow of each row (split only)
    int nv = 0;
    int split = 0;
    int seg = 0;
    // capacity-sized storage owned by the layer state
    int *vptr_store = nullptr, *v2row_store = nullptr, *rvptr_store = nullptr;
    int nv_cap = 0;
};

struct ScratchPlan {
    size_t total = 0;
    // forward/backward partial sums of split matrices
    size_t partial = 0;
    // evolve / init
    size_t tie64 = 0, trank = 0, keep = 0, kscan = 0, s_col = 0, s_val = 0, s_vel = 0, rowptr_s = 0, new_p = 0;
    size_t keyA = 0, keyB = 0, payA = 0, payB = 0, f0 = 0, f1 = 0, f2 = 0, f3 = 0, temp = 0, small = 0, packed = 0;
    size_t temp_bytes = 0;
    int64_t w_cap = 0;   // capacity of the sampler window (items)
    int dense_mode = 0;  // sampler mode of this layer (fixed: |occupied| + k == nnz always)
};

struct StatePlan {
    size_t total = 0;
    size_t rowptr = 0, colidx = 0, val = 0, vel = 0, grad = 0, bias = 0, bias_vel = 0, grad_bias = 0;
    size_t colptr = 0, rowidx = 0, csr_pos = 0, valT = 0, velT = 0;
    size_t mask = 0, dz = 0;
    size_t f_vptr = 0, f_v2row = 0, f_rvptr = 0, b_vptr = 0, b_v2row = 0, b_rvptr = 0;
    size_t sel = 0;
    int nv_cap_f = 0, nv_cap_b = 0;
};

struct SelState {            // radix-select state of one class of weights, lives on the device
    uint32_t prefix, krem, active, thresh, need, pad0, pad1, pad2;
    uint32_t hist[256];
};

}  // namespace sl

struct sl_layer {
    sl_config cfg;
    int64_t nnz = 0;
    int ldz = 0;       // leading dimension of dz and of partial sums (multiple of 32)
    int ldm = 0;       // bytes per row of the sign mask (ldz / 4)
    int has_csc = 0;
    sl::StatePlan sp;
    sl::ScratchPlan cp;
    char *state = nullptr;
    char *scratch = nullptr;
    size_t state_bytes = 0, scratch_bytes = 0;
    // CSR of Wt (forward orientation); val is always current.  vel/grad are in CSR order when
    // the layer has no CSC view; with a CSC view the master copies are valT/velT/grad in CSC order.
    int *rowptr = nullptr, *colidx = nullptr;
    float *val = nullptr, *vel = nullptr, *grad = nullptr, *bias = nullptr, *bias_vel = nullptr, *grad_bias = nullptr;
    int *colptr = nullptr, *rowidx = nullptr, *csr_pos = nullptr;
    float *valT = nullptr, *velT = nullptr;
    uint8_t *mask = nullptr;
    float *dz = nullptr;
    sl::SelState *sel = nullptr;
    sl::SegMat fwd, bwd;
    // optional per-kernel timing with HIP events on the caller's stream (off by default)
    struct ProfRec { int id; hipEvent_t start, stop; };
    bool prof_on = false;
    std::vector<ProfRec> prof;
    // Chaining: `producer` is the layer whose activation output is this layer's x.  When this layer's
    // backward is called without a grad_x buffer it writes the producer's dz (and bias gradient)
    // directly and sets the producer's dz_ready to the batch size; the producer's backward then
    // skips its own activation-derivative pass.
    sl_layer *producer = nullptr;
    int dz_ready = 0;
    // dropout on this layer's activations for the next forward/backward pair (0 = off)
    uint32_t drop_thr = 0, drop_step = 0;
    float drop_scale = 1.f;
    // Update fused behind the SDDMM: 0 off, 1 backward applies eq. (1) to the connections and does not store
    // the gradient, 2 applies it and stores the gradient as well.  weights_updated / grad_stored describe the
    // pending backward pass (phase 2).
    int fuse_mode = 0;
    bool weights_updated = false, grad_stored = true;
    int64_t sampler_first = 0, sampler_max = 0;   // window of the position sampler (0: automatic / the scratch capacity)
    int phase = 0;     // 0 idle, 1 forward done, 2 backward done
    int last_B = 0;
    hipStream_t last_stream = nullptr;
    char err[256] = {0};
};

namespace sl {

int set_err(sl_layer *L, int code, const char *fmt, ...);
#define SL_HIP(L, expr)                                                                       \
    do {                                                                                      \
        hipError_t e__ = (expr);                                                              \
        if (e__ != hipSuccess) return sl::set_err((L), SL_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies; the key is bumped by
// two Weyl constants between rounds.
__host__ __device__ inline void philox(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                       uint32_t out[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t a = (uint64_t)0xD2511F53u * c0;
        const uint64_t b = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(a >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)b;
        c3 = (uint32_t)a;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// kernel ids reported by the profiling calls
enum KernelId { K_FWD = 0, K_FWD_FIX, K_ACTGRAD, K_BWD_FUSED, K_SDDMM, K_BWD_FIX, K_UPDATE, K_COUNT };
struct ProfScope {
    sl_layer *L; hipStream_t s; hipEvent_t stop = nullptr;
    ProfScope(sl_layer *L_, int id, hipStream_t s_) : L(L_), s(s_)
    {
        if (!L->prof_on || L->prof.size() >= 65536) return;
        hipEvent_t a = nullptr;
        if (hipEventCreate(&a) != hipSuccess) return;
        if (hipEventCreate(&stop) != hipSuccess) { (void)hipEventDestroy(a); stop = nullptr; return; }
        (void)hipEventRecord(a, s);
        L->prof.push_back({id, a, stop});
    }
    ~ProfScope() { if (stop) (void)hipEventRecord(stop, s); }
};

// host-side planning (no GPU needed)
int64_t config_nnz(const sl_config &c);
int plan_state(const sl_config &c, int64_t nnz, StatePlan *sp);
int plan_scratch(const sl_config &c, int64_t nnz, ScratchPlan *cp);
int64_t sampler_window(double M, double n_occ, double k);
int choose_seg(int64_t n_rows, int64_t nnz);

// training kernels (sl_train.hip)
int launch_forward(sl_layer *L, const float *x, int64_t ldx, int B, float *a, int64_t lda, bool save_sign, hipStream_t s,
                   float *part = nullptr);   // part: where a split matrix puts its partial sums (null: the layer's scratch)
int launch_forward_static(sl_layer *L, const float *x, int64_t ldx, int B, float *a, int64_t lda, hipStream_t s);
int static_scratch_setup(sl_layer *L, void **ptr);
int launch_backward(sl_layer *L, const float *x, int64_t ldx, const float *ga, int64_t ldg, int B, float *gx,
                    int64_t ldgx, hipStream_t s);
int launch_update(sl_layer *L, hipStream_t s);
int launch_softmax_ce(const float *z, int64_t ldz, const int32_t *y, int B, int C, float *dz, int64_t lddz,
                      float *loss_sum, float *gb, hipStream_t s);
int launch_update_many(sl_layer *const *layers, int count, hipStream_t s);

// topology (sl_topology.hip)
int topo_init(sl_layer *L, hipStream_t s);
int topo_evolve(sl_layer *L, double zeta, uint32_t generation, hipStream_t s);
int topo_finalize(sl_layer *L, hipStream_t s, bool from_merge = false);   // vrows + CSC view from the CSR arrays
int topo_sync_csr_vel(sl_layer *L, hipStream_t s);    // CSC-master layers: velT -> vel (CSR order)
int topo_sync_csr_grad(sl_layer *L, float *grad_csr_dev, hipStream_t s);
int topo_check_temp(sl_layer *L, hipStream_t s);      // rocPRIM temporaries fit the reservation
size_t average_scratch_bytes(int64_t total_entries);
int topo_average(sl_layer *dst, sl_layer *const *replicas, int K, char *scratch, size_t scratch_bytes, hipStream_t s);
int topo_retain_valid(sl_layer *L, const int *old_rowptr, const int *old_col, const float *old_grad, int64_t old_nnz,
                      hipStream_t s);
int topo_importance(sl_layer *L, float *imp_dev, hipStream_t s);
int topo_importance_prune(sl_layer *L, float threshold, int64_t *removed, hipStream_t s);

}  // namespace sl
