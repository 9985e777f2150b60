/*
 * neus2.h - C ABI of libneus2: the training-step hot path of NeuS2 (arXiv 2212.05231)
 * as hand-written HIP kernels for gfx950 (MI355X), one GPU.
 *
 * Conventions for every call
 *  - Returns NEUS2_OK (0) or a negative NEUS2_ERR_* code; neus2_last_error() gives a
 *    thread-local message.  Arguments are validated on the host before anything is
 *    launched; a call that fails validation touches no device memory.
 *  - Pointers marked [device] are device pointers owned by the caller, 16-byte aligned,
 *    row-major, valid until the work queued on `stream` has finished.  Pointers marked
 *    [host] are read during the call only.  The library allocates no device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work; they never synchronise.
 *  - Arithmetic: fp32 throughout.  The matrix products of the two networks take their fp32
 *    factors as sums of bf16 terms on the bf16 matrix cores with fp32 accumulation: three terms
 *    (six term products) wherever a result is a forward output or decides a ReLU mask, which is
 *    as accurate as an fp32 product (about 2e-7 relative on the outputs); two terms (three term
 *    products) in the adjoint sweeps and weight gradients (about 1e-5 relative on the gradients).
 *  - n is the number of sample points; for ray workloads n = rays * samples_per_ray and a
 *    ray's samples are consecutive.
 *
 * Layouts
 *  - tables  [L][T][F]   F = 2 features per entry, fp16 or fp32 (cfg->table_dtype).
 *  - enc, q, d_enc: level-major [L][n][F] fp32 ("feature k = level*F + f of point i" is at
 *    (level*n + i)*F + f).  jac (de/dx, fp32): [L][3][n][2]; the six values J[f][a] of a point
 *    and level, in the order 3*f + a, are cut into three pairs, and pair c of point i is at
 *    ((level*3 + c)*n + i)*2 (a wavefront then reads and writes whole cache lines).
 *  - y, d_y [n][16]; normal, d_normal, pos, d_pos [n][3]; rgb, d_rgb [n][3].
 *  - SDF matrices H_l [n_l][n_{l-1}] and colour matrices W_l likewise, row-major fp32,
 *    bias-free (Definition 1 of the paper).
 */
#ifndef NEUS2_H
#define NEUS2_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NEUS2_MAX_LEVELS 32
#define NEUS2_MAX_MATS 4

enum {
    NEUS2_OK = 0,
    NEUS2_ERR_NULL = -1,        /* a required pointer is NULL */
    NEUS2_ERR_SHAPE = -2,       /* a size is negative, too large, or not a multiple it must be */
    NEUS2_ERR_CONFIG = -3,      /* the descriptor is inconsistent */
    NEUS2_ERR_ALIGN = -4,       /* a device pointer is not 16-byte aligned */
    NEUS2_ERR_UNSUPPORTED = -5, /* a valid request this build has no kernel for */
    NEUS2_ERR_HIP = -6          /* the HIP runtime reported an error at launch */
};

/* Shape descriptor.  Per-level resolution and dense flag are inputs, so that the caller's
 * reference computation and the kernels can never disagree on them.  A level is dense
 * (lexicographic vertex index) only if (res+1)^3 <= T; otherwise vertices are hashed. */
typedef struct neus2_config {
    int32_t n_levels;          /* L, 1..32 */
    int32_t n_features;        /* F, must be 2 */
    int32_t log2_table_size;   /* T = 1 << log2_table_size entries per level, 4..24 */
    int32_t active_levels;     /* lambda of Sec. 4.3: levels >= this contribute zeros */
    int32_t table_dtype;       /* 0 = fp32, 1 = fp16 */
    int32_t res[NEUS2_MAX_LEVELS];
    int32_t dense[NEUS2_MAX_LEVELS];
    int32_t n_sdf_mats;        /* K: 2 or 3 */
    int32_t sdf_dims[NEUS2_MAX_MATS + 1];   /* {L*F, 64, (64,) 16} */
    int32_t n_color_mats;      /* 0 (no colour network) or 3 */
    int32_t color_dims[NEUS2_MAX_MATS + 1]; /* {38, 64, 64, 3} */
    int32_t samples_per_ray;   /* 1..64 */
    int32_t loss_kind;         /* 0: mean(d^2) + beta*eikonal; 1: L1 colour + beta*eikonal;
                                  2: Huber colour (Eq. 4) + beta*eikonal */
    float s;                   /* slope of the logistic CDF Phi_s; calls that take s_dev read it
                                  from device memory instead when s_dev is not NULL */
    float beta;                /* weight of the eikonal term in Eq. 4 */
    float huber_delta;         /* loss_kind 2: |r| <= delta is quadratic, beyond it linear */
    int32_t frozen_levels;     /* levels [0, frozen_levels) are inputs, not parameters: encoded and
                                  differentiated with respect to the position like the others, but
                                  they get no table gradient and no Adam update.  Filled with the
                                  vertex coordinates (trilinear interpolation reproduces linear
                                  functions exactly) they feed the position x itself to the SDF
                                  network: Eq. 1's e = (x, h(x)) */
} neus2_config;

const char* neus2_last_error(void);
int neus2_version(void);

/* Check a descriptor without a GPU.  Returns NEUS2_OK or the error a compute call would give. */
int neus2_validate_config(const neus2_config* cfg /*[host]*/);

/* Bytes of scratch the scatter-add wants for n points (0 if it would not use any; -1 on a bad
 * descriptor).  The workspace is optional everywhere: without it (NULL, or too small) the
 * scatter-add falls back to its atomic kernel, same results. */
int64_t neus2_workspace_bytes(const neus2_config* cfg /*[host]*/, int64_t n);

/* Multi-resolution hash encoding (Sec. 3 "InstantNGP", Sec. 4.1) and its Jacobian de/dx,
 * which Eq. 2 (n = grad_x d) and Eq. 7 need.  Per level: the point is clamped to [0,1], the
 * grid coordinate is the single binary32 product x*res, the cell is its floor (at most
 * res-1), and the 8 cell vertices are interpolated trilinearly.  Levels >= active_levels
 * write zeros (Sec. 4.3).
 *   pos [device, n*3]  tables [device]  enc [device, L*n*F]  jac [device, L*n*F*3]
 *   dbg_idx [device, n*L*8 uint32] or NULL: the table slot of every corner, corner
 *   c = dx + 2*dy + 4*dz. */
int neus2_hash_encode(const neus2_config* cfg, const float* pos, const void* tables, int64_t n,
                      float* enc, float* jac, uint32_t* dbg_idx, void* stream);

/* SDF network forward (Eq. 1: (d,g) = f_Theta(e)) and analytic normal (Eq. 2) via
 * dd/de = H_K^(0,_) G ... G H_1 (supplement Sec. B).
 *   H [host array of K device pointers]
 *   y [device, n*16] (d = y[.,0]);  q [device, L*n*F] = dd/de;  normal [device, n*3] = q*jac.
 *   masks [device, 2*n*2 uint32] or NULL: if given, receives the ReLU masks m_l = [z_l > 0] of
 *   the hidden layers (Definition 1) for the backward call of the same inputs and matrices:
 *   word (l*n + i)*2 + h, l = 0, 1 (hidden layer), h = 0, 1, holds in bit 16*b + r the mask of
 *   neuron 32*b + 8*(r/4) + 4*h + r%4 of point i (with two matrices layer 1 is not written). */
int neus2_sdf_fwd_grad(const neus2_config* cfg, const float* enc, const float* jac,
                       const float* const* H, int64_t n, float* y, float* q, float* normal,
                       uint32_t* masks, void* stream);

/* The SDF network with more matrices than neus2_sdf_fwd_grad / neus2_sdf_mlp_bwd hold fused (the
 * deeper networks of the paper's Fig. 7, "speed-up of our 2nd-order derivative ... across MLP
 * layer numbers"): the same quantities, computed layer by layer, one launch per matrix and
 * direction, the per-point vectors passing through a workspace.
 *   n_mats K = 2..NEUS2_DEEP_MAX_MATS matrices: H[0] [64][enc_dim], H[1..K-2] [64][64],
 *   H[K-1] [16][64] (row-major, device; the array of pointers is host memory); enc_dim 16 or 32.
 *   enc [device, (enc_dim/2)*n*2], jac [device, (enc_dim/2)*3*n*2], q, d_enc like enc; layouts as
 *   in neus2_hash_encode with enc_dim/2 levels, all of them active.
 *   neus2_sdf_deep_fwd_grad: y [device, n*16], q = dd/de, normal [device, n*3] = q*jac (Eq. 1,
 *   Eq. 2, supplement Sec. B).
 *   neus2_sdf_deep_bwd: dH[l] (host array of K device pointers, shaped like H[l]) are ADDED into
 *   with delta_l a_{l-1}^T + S_l^T t_{l-1}^T (Theorem 1, Eqs. 7-8); d_enc is overwritten with
 *   dL/de.  It recomputes the forward pass itself and needs nothing from the forward call.
 *   workspace [device, at least neus2_sdf_deep_workspace_bytes(n_mats, n)]: required; contents
 *   are undefined afterwards.  The size query returns -1 for an unsupported n_mats or n < 0.
 * Errors: NEUS2_ERR_UNSUPPORTED (n_mats, enc_dim), NEUS2_ERR_NULL, NEUS2_ERR_SHAPE (workspace
 * too small, n < 0); nothing is launched then. */
#define NEUS2_DEEP_MAX_MATS 9
int64_t neus2_sdf_deep_workspace_bytes(int32_t n_mats, int64_t n);
int neus2_sdf_deep_fwd_grad(int32_t n_mats, int32_t enc_dim, const float* enc, const float* jac,
                            const float* const* H, int64_t n, float* y, float* q, float* normal,
                            void* workspace, int64_t workspace_bytes, void* stream);
int neus2_sdf_deep_bwd(int32_t n_mats, int32_t enc_dim, const float* enc, const float* jac,
                       const float* const* H, const float* d_y, const float* d_normal, int64_t n,
                       float* const* dH, float* d_enc, void* workspace, int64_t workspace_bytes,
                       void* stream);

/* Colour network forward (Eq. 3): rgb = sigmoid(W_3 relu(W_2 relu(W_1 cin))),
 * cin = [pos(3), normal(3), SH16(dir)(16), y(16)]; dirs [device, rays*3] are unit vectors,
 * sample i uses ray sample_ray[i] (sample_ray [device, n int32], rays with their own sample
 * counts) or, with sample_ray NULL, ray i / samples_per_ray.  rgb [device, n*3].
 * masks [device, 2*n*2 uint32] or NULL: as in neus2_sdf_fwd_grad, for neus2_color_bwd. */
int neus2_color_fwd(const neus2_config* cfg, const float* pos, const float* normal,
                    const float* dirs, const int32_t* sample_ray, const float* y,
                    const float* const* W, int64_t n, float* rgb, uint32_t* masks, void* stream);

/* First-order backward of the colour network (the paper needs no second-order term for
 * Upsilon, text after Eq. 6).
 *   rgb [device, n*3] in: the colours neus2_color_fwd wrote for the same inputs (the
 *   sigmoid's derivative is taken from them);
 *   d_rgb [device, n*3] in;  d_sdf [device, n] in or NULL (render's dL/dd, added to d_y[.,0]);
 *   dW [host array of 3 device pointers]: gradients are ADDED into them;
 *   d_y [device, n*16] is OVERWRITTEN with the colour network's dL/d(d,g) (+ d_sdf);
 *   d_normal [device, n*3] is ADDED into (it already holds the eikonal part);
 *   d_pos [device, n*3] or NULL is OVERWRITTEN with the colour network's dL/dx;
 *   masks [device, 2*n*2 uint32] or NULL: the masks neus2_color_fwd wrote for the same inputs
 *   and matrices.  The backward pass recomputes the hidden activations instead of reading them
 *   back.  Given the masks it does so at the accuracy its results are compared at (gradient
 *   tolerance, see "Arithmetic" above); without them it repeats the forward call's own
 *   arithmetic, which reproduces the masks bit for bit, at about 8 % more time. */
int neus2_color_bwd(const neus2_config* cfg, const float* pos, const float* normal,
                    const float* dirs, const int32_t* sample_ray, const float* y,
                    const float* const* W, const float* rgb,
                    const float* d_rgb, const float* d_sdf, int64_t n, float* const* dW,
                    float* d_y, float* d_normal, float* d_pos, const uint32_t* masks,
                    void* stream);

/* NeuS compositing (supplement Sec. E.3): alpha_i = max((Phi(d_i)-Phi(d_{i+1}))/Phi(d_i), 0),
 * alpha of the last sample is 0, T_i = prod_{j<i}(1-alpha_j), C = sum T_i alpha_i c_i.
 *   sdf [device]: d of sample i at sdf[i*sdf_stride];  rgb [device, n*3];
 *   s_dev [device, 1 float] or NULL: the slope s when it is a trained parameter that lives
 *   on the device (the paper keeps s learnable); NULL means cfg->s;
 *   C [device, rays*3];  weights [device, n] = T_i alpha_i. */
int neus2_render_rays(const neus2_config* cfg, const float* sdf, int64_t sdf_stride,
                      const float* rgb, const float* s_dev, int64_t rays, float* C,
                      float* weights, void* stream);

/* Backward of neus2_render_rays: dC [device, rays*3] -> d_sdf [device, n], d_rgb [device, n*3]
 * (both overwritten);  d_s [device, 1 float] or NULL: dL/ds is ADDED into it. */
int neus2_render_rays_bwd(const neus2_config* cfg, const float* sdf, int64_t sdf_stride,
                          const float* rgb, const float* dC, const float* s_dev, int64_t rays,
                          float* d_sdf, float* d_rgb, float* d_s, void* stream);

/* Loss of Eq. 4 and its first adjoints.
 *   loss_kind 1: loss = sum|C - target| / rays + beta * mean((|n|-1)^2); C, target
 *     [device, rays*3]; dC [device, rays*3] = sign(C-target)/rays.
 *   loss_kind 2: as 1 with the Huber function of huber_delta in place of |.|;
 *     dC = clamp(C-target, -delta, delta)/rays.
 *   loss_kind 0: loss = mean(d^2) + beta * mean((|n|-1)^2); C, target, dC are NULL and
 *     d_y [device, n*16] is overwritten with (2 d / n) e_0.  For loss_kind 1, 2 d_y may be NULL.
 *   d_normal [device, n*3] is overwritten with the eikonal part (2 beta / n)(|n|-1) n/|n|.
 *   loss [device, 2 floats]: {first term, beta * eikonal term}; ADDED into (zero it first). */
int neus2_loss(const neus2_config* cfg, const float* C, const float* target, const float* normal,
               const float* y, int64_t rays, int64_t n, float* loss, float* dC, float* d_normal,
               float* d_y, void* stream);

/* Backward through the SDF network and the encoding, first order plus the second-order term
 * of Eqs. 7-8 / Theorem 1:
 *   dH_l += delta_l a_{l-1}^T + S_l^T t_{l-1}^T,  t_0 = (de/dx) dL/dn,  t_l = G_l H_l t_{l-1};
 *   d_tables[slot_c][f] += w_c * dL/de_f + q_f * res * sum_a dL/dn_a * d_a w_c.
 *   d_y [device, n*16], d_normal [device, n*3]: total adjoints of (d,g) and n.
 *   dH [host array of K device pointers], d_tables [device, L*T*F fp32]: ADDED into.
 *   d_enc [device, L*n*F]: overwritten with dL/de (also the scratch between the two kernels).
 *   d_pos [device, n*3] or NULL: if given, ADDED into with (de/dx)^T dL/de plus the mixed
 *   second derivative of the interpolation contracted with q and dL/dn (needed only when
 *   positions are themselves functions of a learnable transform, Eq. 9).
 *   workspace [device, workspace_bytes] or NULL: scratch for the scatter-add, see
 *   neus2_workspace_bytes; contents are undefined afterwards.
 *   masks [device, 2*n*2 uint32] or NULL: the masks neus2_sdf_fwd_grad wrote for the same enc
 *   and H; meaning as in neus2_color_bwd. */
int neus2_sdf_bwd_2nd(const neus2_config* cfg, const float* pos, const void* tables,
                      const float* enc, const float* jac, const float* const* H, const float* q,
                      const float* d_y, const float* d_normal, int64_t n, float* const* dH,
                      float* d_tables, float* d_enc, float* d_pos, void* workspace,
                      int64_t workspace_bytes, const uint32_t* masks, void* stream);

/* The two halves of neus2_sdf_bwd_2nd as calls of their own (same arguments, same meaning):
 * the fused network backward (dH, d_enc, and the (de/dx)^T dL/de part of d_pos) ... */
int neus2_sdf_mlp_bwd(const neus2_config* cfg, const float* enc, const float* jac,
                      const float* const* H, const float* d_y, const float* d_normal, int64_t n,
                      float* const* dH, float* d_enc, float* d_pos, const uint32_t* masks,
                      void* stream);

/* ... and the scatter-add into the table gradient (Eq. 7's term included; with d_pos, the
 * mixed second derivative of the interpolation as well). */
int neus2_hash_scatter_bwd(const neus2_config* cfg, const float* pos, const void* tables,
                           const float* q, const float* d_enc, const float* d_normal, int64_t n,
                           float* d_tables, float* d_pos, void* workspace, int64_t workspace_bytes,
                           void* stream);

/* neus2_hash_scatter_bwd (without the position gradient) for callers that cannot allocate
 * device memory or pass a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results; the record lists live in a
 * buffer of NEUS2_STATIC_SCRATCH_BYTES that is part of the library's device image (every GPU the
 * library is used on holds one until the process ends).  The call allocates nothing, on the
 * device or through any library.  A batch whose lists do not fit (neus2_workspace_bytes minus
 * the 24 * n_levels * n bytes of its position-gradient part is the need; about 140 000 points
 * with 16 levels of 2^19 slots, more with fewer hashed levels) is rejected with
 * NEUS2_ERR_SHAPE and nothing is launched.  All calls on one GPU share the buffer: calls that
 * overlap in time on one GPU (different streams or threads) race; order them. */
#define NEUS2_STATIC_SCRATCH_BYTES (128 * 1024 * 1024)
int neus2_hash_scatter_bwd_static(const neus2_config* cfg, const float* pos, const void* tables,
                                  const float* q, const float* d_enc, const float* d_normal,
                                  int64_t n, float* d_tables, void* stream);

/* neus2_render_rays, neus2_loss (loss_kind 1 or 2) and neus2_render_rays_bwd in one launch,
 * same arguments and results (sdf is column 0 of y [device, n*16]); neus2_train_step uses
 * it.  A ray's samples stay in registers between the three stages. */
int neus2_render_loss_bwd(const neus2_config* cfg, const float* y, const float* rgb,
                          const float* normal, const float* target, const float* s_dev,
                          int64_t rays, float* C, float* weights, float* loss, float* dC,
                          float* d_sdf, float* d_rgb, float* d_normal, float* d_s, void* stream);

/* The same for rays with their own sample counts (an occupancy-grid ray marcher, supplement
 * Sec. E.3): ray r owns samples ray_offsets[r] .. ray_offsets[r+1]-1 of the n samples
 * (ray_offsets [device, rays+1 int32], non-decreasing, first 0, last n); any count, also 0
 * (such a ray renders black and still enters the colour term).  The last sample of a ray has
 * alpha 0.  The colour term is averaged over rays, the eikonal term over the n samples. */
int neus2_render_loss_bwd_ragged(const neus2_config* cfg, const float* y, const float* rgb,
                                 const float* normal, const float* target,
                                 const int32_t* ray_offsets, const float* s_dev, int64_t rays,
                                 int64_t n, float* C, float* weights, float* loss, float* dC,
                                 float* d_sdf, float* d_rgb, float* d_normal, float* d_s,
                                 void* stream);

/* Adam with bias correction over `count` parameters (the paper names no optimiser).
 *   param [device]: fp32 (dtype 0) or fp16 (dtype 1); with fp16 `master` [device, fp32] holds
 *   the full-precision copy, is updated, and param receives its round-to-nearest-even.
 *   grad, m, v [device, fp32].  t >= 1 is the step number (bias correction 1 - beta^t).
 *   flags: bit 0 (NEUS2_ADAM_CLEAR) clears grad; bit 1 (NEUS2_ADAM_LAZY) leaves every entry whose
 *   gradient is exactly zero as it is (value and both moments): the form used for hash tables of
 *   which a step touches a small part; the bias correction still uses the global step number. */
#define NEUS2_ADAM_CLEAR 1
#define NEUS2_ADAM_LAZY 2
int neus2_adam_step(void* param, float* master, float* grad, float* m, float* v, int64_t count,
                    int dtype, float lr, float beta1, float beta2, float eps, int t,
                    int flags, void* stream);

/* The same update over the hash tables [L][T][F] of a descriptor (fp16 tables with their fp32
 * master copy, or fp32 tables and master NULL), skipping the slots no point can address: a
 * dense level uses (res+1)^3 of its T slots; the rest never receive a gradient and the update
 * would leave them unchanged.  Same result as neus2_adam_step over L*T*F parameters.
 * flags bit 2 (NEUS2_ADAM_ACTIVE_LEVELS): the levels >= active_levels are skipped as well.  That
 * is the dense update exactly as long as those levels have never received a gradient (their
 * moments are zero and stay zero): the progressive schedule of Sec. 4.3 only ever adds levels.
 * neus2_adam_step, which knows no levels, rejects the bit. */
#define NEUS2_ADAM_ACTIVE_LEVELS 4
int neus2_adam_tables(const neus2_config* cfg, void* tables, float* master, float* grad, float* m,
                      float* v, float lr, float beta1, float beta2, float eps, int t,
                      int flags, void* stream);

/* neus2_adam_tables and, in the same launch, the dense update of a flat fp32 buffer of
 * small_count parameters (the matrices of both networks, a trained slope): small_param,
 * small_grad, small_m, small_v [device, fp32].  The lazy flag applies to the tables only.
 * Same results as the two separate calls. */
int neus2_adam_all(const neus2_config* cfg, void* tables, float* master, float* grad, float* m,
                   float* v, float* small_param, float* small_grad, float* small_m, float* small_v,
                   int64_t small_count, float lr, float beta1, float beta2, float eps, int t,
                   int flags, void* stream);

/* Global rigid transform of Eq. 9, x_c = R (x + T), then the affine map scale*x_c + offset
 * that takes world coordinates to the unit cube.  R [host, 9 row-major], T [host, 3]. */
int neus2_rigid_fwd(const float* pos, const float* R, const float* T, float scale, float offset,
                    int64_t n, float* out, void* stream);

/* Reductions for the transform's gradient: with g = scale * d_out,
 * Mb[0..8] += sum g (x+T)^T (= dL/dR, row-major), Mb[9..11] += sum g.  Mb [device, 12]. */
int neus2_rigid_bwd(const float* pos, const float* T, const float* d_out, float scale, int64_t n,
                    float* Mb, void* stream);

/* ---- The transform of a frame as six trained parameters (Sec. 5, Eqs. 9-10; the supplement's
 * training schedule optimises them alone for the first iterations of a frame) -------------------
 * A frame's points reach the canonical space through x_c = R_prev (R(omega) (x + T) + T_prev),
 * where (R_prev, T_prev) is the transform accumulated over the earlier frames and
 * R(omega) = exp([omega]_x).  That is the single rigid map x_c = Rc (x + Tc), Rc = R_prev R(omega),
 * Tc = T + R(omega)^T T_prev (the accumulation rule stated after Eq. 10).  All state lives in
 * device memory, so a training loop never reads anything back:
 *   param [device, 6]: omega (3), T (3);  m, v [device, 6]: their Adam moments;
 *   prev  [device, 12]: R_prev row-major (9), T_prev (3)  (identity and zero for the first frame);
 *   pose  [device, 12]: Rc (9), Tc (3), what the two calls below apply;
 *   Mb    [device, 12]: the reductions of neus2_rigid_bwd_dev.
 * Moving on to the next frame is a copy of pose into prev and new values in param. */

/* neus2_rigid_fwd / neus2_rigid_bwd with the transform read from device memory (pose). */
int neus2_rigid_fwd_dev(const float* pos, const float* pose, float scale, float offset, int64_t n,
                        float* out, void* stream);
int neus2_rigid_bwd_dev(const float* pos, const float* pose, const float* d_out, float scale,
                        int64_t n, float* Mb, void* stream);

/* apply = 1: the gradient of the six parameters from Mb (sum g (x+T)^T = M - b (R^T T_prev)^T,
 * dL/dR = R_prev^T of that, dL/domega_k = sum (dR/domega_k) o dL/dR, dL/dT = Rc^T b), one Adam
 * step on them (step number t >= 1, bias-corrected like neus2_adam_step), then pose is rebuilt
 * from the new parameters and Mb is cleared.  apply = 0: only pose is rebuilt from param and
 * prev and Mb cleared (the start of a frame; m, v may be NULL).  One thread, double precision. */
int neus2_pose_update(float* param, float* m, float* v, const float* prev, float* Mb, float* pose,
                      float lr, float beta1, float beta2, float eps, int t, int apply, void* stream);

/* All buffers of one training step, for neus2_train_step.  Every pointer is [device] except
 * H, W, dH, dW, which are [host] arrays of device pointers.  Sizes as in the calls above;
 * rays * samples_per_ray = n, unless ray_offsets / sample_ray describe the rays. */
typedef struct neus2_step_buffers {
    const float* pos; const float* dirs; const float* target; const void* tables;
    const float* const* H; const float* const* W;
    float* enc; float* jac; float* y; float* q; float* normal; float* rgb;
    float* C; float* weights; float* loss;
    float* dC; float* d_sdf; float* d_rgb; float* d_y; float* d_normal; float* d_enc;
    float* d_pos;              /* NULL unless the position gradient is wanted */
    float* const* dH; float* const* dW; float* d_tables;
    void* workspace;           /* optional scratch, see neus2_workspace_bytes */
    int64_t workspace_bytes;
    const float* s_dev;        /* optional, see neus2_render_rays */
    float* d_s;                /* optional, see neus2_render_rays_bwd (ADDED into) */
    const int32_t* ray_offsets;/* optional: rays with their own sample counts, see          */
    const int32_t* sample_ray; /*   neus2_render_loss_bwd_ragged and neus2_color_fwd; both or */
    int64_t n_rays;            /*   neither; n_rays is read only when they are given         */
    uint32_t* sdf_masks;       /* optional [2*n*2 each]: the ReLU masks pass from the forward    */
    uint32_t* color_masks;     /*   to the backward kernels, see neus2_color_bwd                 */
} neus2_step_buffers;

/* One forward + backward pass (everything above except Adam and the rigid transform), in the
 * order encode, SDF, colour, render, loss, render bwd, colour bwd, SDF bwd + scatter.
 * loss is zeroed first; dH, dW and d_tables are ADDED into.  Unlike neus2_hash_encode, the step
 * leaves the levels >= active_levels of enc and jac as they are (Sec. 4.3: those levels do not
 * enter the network; none of the step's kernels reads them) instead of writing zeros. */
int neus2_train_step(const neus2_config* cfg, const neus2_step_buffers* buf, int64_t n, void* stream);

/* ---- Occupancy grid and ray marching (supplement Sec. E.3 "Ray Marching Acceleration") ------
 * A grid of G^3 cells over the unit cube, G = 2^log2_res (2 <= log2_res <= 8), marks cells as
 * empty or not; the marcher leaves out samples in empty cells.  Cell (x,y,z) has the Morton
 * number with bit b of x, y, z at bit 3b, 3b+1, 3b+2.  density [device, G^3 fp32] holds one
 * non-negative value per cell in Morton order, bitfield [device, G^3/32 uint32] cell c in bit
 * c%32 of word c/32.  The paper refreshes the grid from the SDF through the logistic density
 * phi_s(d) = s e^{-sd} / (1+e^{-sd})^2 "in the same way as" the publication it cites: decay
 * all values, raise candidate cells to the density at a random point inside them, threshold. */

/* Sample points of m candidate cells: pos[i] = (cell coordinate + jitter[i]) / G.
 *   cells [device, m int32] Morton numbers (taken modulo G^3), jitter [device, m*3] in [0,1),
 *   pos [device, m*3].  The caller evaluates the SDF there (neus2_hash_encode,
 *   neus2_sdf_fwd_grad) and hands it to neus2_occupancy_update. */
int neus2_occupancy_points(int log2_res, const int32_t* cells, const float* jitter, int64_t m,
                           float* pos, void* stream);

/* One refresh: density *= decay for every cell; density[cells[i]] = max(., phi_s(sdf[i*sdf_stride]))
 * (a cell named twice keeps the larger; cell numbers outside the grid and non-finite values
 * are skipped); then bit c = density[c] > threshold for every cell.
 *   s_dev [device, 1] the trained slope, or NULL to use the argument s.  0 <= decay <= 1,
 *   threshold >= 0.  m may be 0 (decay and threshold only). */
int neus2_occupancy_update(int log2_res, float* density, const int32_t* cells, const float* sdf,
                           int64_t sdf_stride, int64_t m, const float* s_dev, float s, float decay,
                           float threshold, uint32_t* bitfield, void* stream);

/* Ray marching through the grid.  Ray r (origins, dirs [device, rays*3], unit-cube coordinates;
 * jitter [device, rays] in [0,1)) is clipped against [0,1]^3 (slab test, t_near >= 0); its
 * samples are the lattice points t_k = t_0 + k dt, t_0 = t_near + jitter dt, 0 <= k < max_steps,
 * with t_k < t_far whose cell clamp(floor((o + t_k d) G)) has its bit set.  All of this is
 * binary32 arithmetic, one rounding per operation, in the order written here.
 * Outputs, rays in order, a ray's samples in order of k:
 *   ray_offsets [device, rays+1 int32], pos [device, capacity*3], sample_ray [device, capacity
 *   int32] (the ray of each sample), t [device, capacity] or NULL (the parameters t_k).
 * At most `capacity` samples are written: the ray that crosses the capacity is cut there and
 * later rays get none (ray_offsets is clamped to capacity); n = ray_offsets[rays].  These are
 * the ray_offsets / sample_ray / pos that neus2_train_step takes for rays of unequal length. */
int neus2_march_rays(int log2_res, const uint32_t* bitfield, const float* origins, const float* dirs,
                     const float* jitter, int64_t rays, float dt, int32_t max_steps, int64_t capacity,
                     int32_t* ray_offsets, float* pos, int32_t* sample_ray, float* t, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NEUS2_H */
