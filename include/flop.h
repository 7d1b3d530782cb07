/*
 * flop.h - C ABI of the MI355X (gfx950) library for the gated factorized
 * linear layer of FLOP ("Structured Pruning of Large Language Models").
 *
 * Every weight matrix W (dout x d) is replaced by P G Q with P (dout x r),
 * Q (r x d) and G = diag(z_1..z_r), one Hard-Concrete gate per rank-1
 * component (Section 4.1).  In batched row form, for n tokens,
 *
 *     h = x Q^T        (n x r)
 *     g = h .* z       (column k scaled by z_k)
 *     y = g P^T        (n x dout)
 *
 * General conventions
 *  - All matrices are row-major.  Leading dimensions (ld*) are in ELEMENTS and
 *    must be >= the logical number of columns.
 *  - Every data pointer is a DEVICE pointer owned by the caller; the library
 *    allocates nothing, frees nothing and keeps no state between calls
 *    (flop_bwd_static's scratch array excepted, see there; the measurement aids of
 *    flop_bench.h, a separate header, keep state of their own).
 *    Scalars that are marked "host" are plain values.
 *  - x, Q, P, g, y and their gradients have the element type `dt` (float32 or
 *    bfloat16).  log_alpha, u, z, dzda, dlog_alpha and every reduction are
 *    float32; products are accumulated in float32 on the matrix cores and
 *    rounded once when stored.
 *  - `stream` is a hipStream_t passed as void*; work is enqueued on it and the
 *    call returns after host-side validation only.  NULL is the default stream.
 *  - Return value: FLOP_OK or a negative flop_status.  On error nothing has
 *    been enqueued.  No exception crosses this boundary.
 *  - Vector (16-byte) global loads are used when base pointers are 16-byte
 *    aligned and leading dimensions are multiples of 16 bytes; anything else
 *    is accepted and takes an element-wise path.  On the vector path a matrix
 *    of rows x cols is read as whole 16-byte chunks, so up to 15 bytes of a
 *    row's padding (between cols and ld) may be read, never written; their
 *    values do not reach any result.  Every row, the last included, must
 *    therefore be addressable up to the next multiple of 16 bytes.
 *  - Fastest layout: leading dimensions that are multiples of 128 bytes (64
 *    bfloat16).  The kernels move 128 contiguous bytes of a row per step; when
 *    rows do not start on 128-byte boundaries every such piece straddles two
 *    cache lines (measured: 10-15 % on 3056-wide bfloat16 matrices).  Matrices
 *    of any size are accepted; a matrix beyond 2 GiB that is read down its
 *    columns (dy in the weight gradient dP) makes flop_bwd cut that product
 *    along the tokens, using the k-split scratch of its workspace.
 */
#ifndef FLOP_H
#define FLOP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FLOP_OK = 0,
    FLOP_ERR_NULL = -1,      /* a required pointer is NULL */
    FLOP_ERR_SHAPE = -2,     /* a size is negative, zero where it must not be, or too large */
    FLOP_ERR_STRIDE = -3,    /* a leading dimension is smaller than the row length */
    FLOP_ERR_DTYPE = -4,     /* unknown flop_dtype / mode */
    FLOP_ERR_PARAM = -5,     /* hard-concrete constants need l < 0, r > 1, beta > 0 */
    FLOP_ERR_WORKSPACE = -6, /* workspace missing or smaller than flop_workspace_bytes() */
    FLOP_ERR_ALIGN = -7,     /* workspace not 256-byte aligned */
    FLOP_ERR_HIP = -8,       /* a HIP launch reported an error */
    FLOP_ERR_ALIAS = -9,     /* an output overlaps an input that the same launch still reads */
    FLOP_ERR_SCRATCH = -10   /* the problem needs more scratch than the library's static device array holds */
} flop_status;

typedef enum { FLOP_F32 = 0, FLOP_BF16 = 1 } flop_dtype;

/* Hard-Concrete constants: temperature beta and stretch interval (l, r), l < 0 < 1 < r.
 * beta = 1 gives the expressions exactly as printed in Section 3. */
typedef struct { float beta, l, r; } flop_hc;

typedef enum { FLOP_GATE_TRAIN = 0, FLOP_GATE_DETERMINISTIC = 1 } flop_gate_mode;

typedef enum { FLOP_OP_FWD = 0, FLOP_OP_BWD = 1, FLOP_OP_EXPECTED_L0 = 2, FLOP_OP_COMPACT = 3,
               FLOP_OP_EMBED_FWD = 4, FLOP_OP_EMBED_BWD = 5, FLOP_OP_GATE_GRAD = 6 } flop_op;

/*
 * Hard-Concrete gates (Section 3, the display defining s, s-bar and z):
 *   TRAIN:          s = sigmoid((log u_k - log(1 - u_k) + log_alpha_k) / beta)
 *   DETERMINISTIC:  s = sigmoid(log_alpha_k)            (u may be NULL)
 *   z_k = min(1, max(0, s (r - l) + l))
 * One gate per rank-1 component, shared by every token of the batch
 * (Section 4.3, last paragraph).  The uniform noise u is an input: the library
 * never draws random numbers.  u outside (0,1) yields z in {0,1}, no trap.
 * dzda (nullable) receives dz_k/dlog_alpha_k = (r-l) s (1-s) / beta where
 * 0 <= s-bar <= 1 and 0 elsewhere (no 1/beta in deterministic mode); flop_bwd
 * consumes it.  All arrays: device, float32, length n_gates.
 */
int flop_gate_sample(const float* log_alpha, const float* u, int64_t n_gates, flop_hc hc,
                     flop_gate_mode mode, float* z, float* dzda, void* stream);

/*
 * Forward (Section 4.1, W = P G Q):  g_saved = (x Q^T) .* z ;  y = g_saved P^T.
 *   x[n, d] ld ldx;  Q[r, d] ld ldq;  P[dout, r] ld ldp;  z[r] float32
 *   g_saved[n, r] ld ldg  - written once, rounded to dt; the only activation
 *                           the backward pass needs besides x
 *   y[n, dout] ld ldy
 * The gate is applied to the float32 accumulators before the single rounding.
 * n == 0 is a no-op.  workspace is optional (may be NULL): with
 * >= flop_workspace_bytes(FLOP_OP_FWD, ...) bytes, 256-byte aligned, a product
 * with few output tiles and a long contraction is split over k and added up in
 * a fixed order by a second kernel; without it every product is one launch.
 */
int flop_fwd(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
             const void* x, int64_t ldx, const void* Q, int64_t ldq, const void* P, int64_t ldp,
             const float* z, void* g_saved, int64_t ldg, void* y, int64_t ldy,
             void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward by the chain rule through the forward above and through
 * z = G(u; log_alpha) (Section 3: gradient steps reach theta and alpha):
 *   dg = dy P                       dP = dy^T g_saved
 *   dh = dg .* z                    dQ = dh^T x          dx = dh Q
 *   dz_k = sum_i dg_ik h_ik         dlog_alpha_k = dz_k * dzda_k
 * h is never stored: where dzda_k != 0 the gate is open and h = g_saved / z_k,
 * so dz_k = (sum_i dg_ik g_ik) / z_k; where dzda_k == 0 (or z_k == 0) the
 * result is exactly 0.  dh lives in the workspace only.
 *   dy[n, dout]; x, Q, P, z, g_saved as in flop_fwd; dzda[r] from flop_gate_sample
 *   dx[n, d], dQ[r, d], dP[dout, r]: overwritten (each nullable: skipped)
 *   dlog_alpha[r] float32 (nullable): overwritten, or added to when accumulate != 0
 * workspace: >= flop_workspace_bytes(FLOP_OP_BWD, ...), 256-byte aligned.
 * Results are deterministic (no floating-point atomics).
 */
int flop_bwd(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
             const void* dy, int64_t lddy, const void* x, int64_t ldx,
             const void* Q, int64_t ldq, const void* P, int64_t ldp,
             const float* z, const float* dzda, const void* g_saved, int64_t ldg,
             void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
             float* dlog_alpha, int accumulate,
             void* workspace, size_t workspace_bytes, void* stream);

/*
 * flop_bwd for callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same arguments without the workspace.  The
 * scratch that flop_bwd takes from its workspace (dh, the column-sum partials, k-split partials) lives in one
 * static device array of FLOP_STATIC_SCRATCH_BYTES inside the library, resolved once per device on the first
 * call there; this call allocates and frees nothing.  A problem whose
 * flop_workspace_bytes(FLOP_OP_BWD, dt, n, d, r, dout) exceeds FLOP_STATIC_SCRATCH_BYTES is refused with
 * FLOP_ERR_SCRATCH before anything is enqueued.  Results equal flop_bwd's bit for bit.  Nothing in the
 * array has to start at zero (every byte the kernels read has been written by the same call).  All calls on
 * one GPU share that GPU's array: calls that overlap in time on one GPU (different streams, or graphs
 * replayed concurrently) race and must be serialised by the caller.
 */
#define FLOP_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
int flop_bwd_static(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                    const void* dy, int64_t lddy, const void* x, int64_t ldx,
                    const void* Q, int64_t ldq, const void* P, int64_t ldp,
                    const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                    void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                    float* dlog_alpha, int accumulate, void* stream);

/*
 * flop_bwd with the last stage of the gate gradient left for later (the optimiser needs dlog_alpha
 * only once per step, so the model's layers can share one small launch instead of one each):
 * everything flop_bwd does, except that dlog_alpha is not written; instead *pending (host memory)
 * receives what flop_gate_grad_finish needs - the location of the partial column sums inside
 * `workspace` and the gate vectors of this call.  The workspace and z, dzda, dlog_alpha must stay
 * untouched until flop_gate_grad_finish has been called on the same stream for this item.
 * dlog_alpha must not be NULL here.
 */
typedef struct {
    const float* partial;      /* device, inside the call's workspace: chunks x r float32 partial sums */
    const float* z;            /* device, r */
    const float* dzda;         /* device, r */
    float* dlog_alpha;         /* device, r: overwritten, or added to when accumulate != 0 */
    const int32_t* r_active;   /* device int32 or NULL: gates at or beyond it get gradient 0 */
    int64_t r;
    int32_t chunks;
    int32_t accumulate;
} flop_gate_grad_pending;

int flop_bwd_deferred(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                      const void* dy, int64_t lddy, const void* x, int64_t ldx,
                      const void* Q, int64_t ldq, const void* P, int64_t ldp,
                      const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                      void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                      float* dlog_alpha, int accumulate,
                      void* workspace, size_t workspace_bytes, void* stream,
                      flop_gate_grad_pending* pending);

/*
 * Last stage of the gate gradient (Section 3) for `count` pending items (host array), sixteen to a launch:
 *   dlog_alpha_k = (sum_c partial[c][k]) / z_k^2 * dzda_k    (exactly 0 where z_k == 0 or dzda_k == 0)
 * The chunk sums are added in index order (deterministic); results equal flop_bwd's bit for bit.
 */
int flop_gate_grad_finish(const flop_gate_grad_pending* items, int32_t count, void* stream);

/*
 * flop_bwd_deferred with the weight gradients left for later as well.  Section 3's gradients dP = dy^T g and
 * dQ = dh^T x (dh = (dy P) .* z) feed only the optimiser's update of the step, not the rest of the backward pass; their
 * contraction runs over the n tokens, far longer than those of dh and dx on narrow layers, and a launch lasts as
 * long as its longest tile.  This call computes dx and the column sums of the gate gradient and writes to
 * *weights (host memory) the operands of the two products it left out: dy, g_saved, x, the gated dh inside
 * `workspace`, and the destinations dP, dQ (either may be NULL: that product is then not wanted).
 * flop_weight_grad_finish later computes them for many layers in shared launches of up to eight products.
 * Until that call has been made on the same stream, dy, x, g_saved and the workspace must stay untouched
 * (the workspace also holds the pending gate-gradient sums, as for flop_bwd_deferred).
 * dlog_alpha may be NULL here (then *pending is left untouched and may be NULL).
 */
typedef struct {
    int32_t dtype;             /* flop_dtype of the layer */
    int64_t n, d, r, dout;
    const void* dy; int64_t lddy;      /* device, n x dout */
    const void* g; int64_t ldg;        /* device, n x r: g_saved */
    const void* dh; int64_t ldh;       /* device, inside the call's workspace: (dy P) .* z, n x r; NULL if dQ is */
    const void* x; int64_t ldx;        /* device, n x d */
    void* dP; int64_t lddp;            /* device, dout x r, or NULL */
    void* dQ; int64_t lddq;            /* device, r x d, or NULL */
    void* split_ws; size_t split_bytes; /* device, inside the call's workspace: scratch for a product cut along k */
} flop_weight_grad_pending;

int flop_bwd_defer_weights(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                           const void* dy, int64_t lddy, const void* x, int64_t ldx,
                           const void* Q, int64_t ldq, const void* P, int64_t ldp,
                           const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                           void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                           float* dlog_alpha, int accumulate,
                           void* workspace, size_t workspace_bytes, void* stream,
                           flop_gate_grad_pending* pending, flop_weight_grad_pending* weights);

/*
 * dP = dy^T g and dQ = dh^T x (Section 3) for `count` pending layers (host array), up to eight products to a
 * launch.  Products that the bfloat16 transfer kernel can take unsplit (16-byte aligned rows, operands within
 * 2 GiB) and all float32 products are grouped in the order given; any other layer's pair is launched on its own
 * with the k-split scratch of its workspace.  Results agree with flop_bwd's to float32 summation order (a
 * different block shape may add the k steps in two interleaved halves); every run of this call on the same
 * items gives the same bits.  FLOP_ERR_NULL / FLOP_ERR_SHAPE / FLOP_ERR_STRIDE / FLOP_ERR_DTYPE for malformed
 * items (nothing is launched then).
 */
int flop_weight_grad_finish(const flop_weight_grad_pending* items, int32_t count, void* stream);

/*
 * The two small launches at the boundary between two training steps in one: flop_gate_grad_finish for the
 * step that ends (items, count) and flop_gate_sample_l0 for the step that begins (every other argument, as
 * there).  With count <= 16 and n_gates <= 4096 this is a single launch; otherwise the two calls are made one
 * after the other.  The finish reads the gates of the ending step while the new ones are written: z and dzda
 * given here (and l0_sum, l0_grad) must not overlap z, dzda or dlog_alpha of any item (keep two sets of gate
 * buffers and alternate), else FLOP_ERR_ALIAS.  Results equal those of the two separate calls (the Eq.(3) sum to float32 rounding).
 */
int flop_step_boundary(const flop_gate_grad_pending* items, int32_t count,
                       const float* log_alpha, const float* u, int64_t n_gates, flop_hc hc,
                       float* z, float* dzda, const float* w, float* l0_sum, float* l0_grad,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * flop_bwd for the layer whose backward pass ends a training step, with the step boundary attached: after
 * this call dlog_alpha of this layer and of every item of job->items is complete and the gates and
 * Eq.(3) of the next step are written, as if flop_bwd_deferred and flop_step_boundary(job->items + this
 * layer, ...) had been called.  Where the shapes allow it (bfloat16, 16-byte aligned rows, at most 16 gate
 * vectors in all, at most 4096 new gates) the boundary work rides as extra workgroups on this call's last
 * contraction launch and costs no launch of its own; otherwise it is launched separately.  The same
 * aliasing rule as flop_step_boundary applies, this layer's z, dzda and dlog_alpha included.
 * With job->n_gates == 0 only the gate gradients are finished (the gate arguments are then ignored): a training
 * loop that updates log_alpha between two steps samples the next gates after that update, with
 * flop_gate_sample_l0, and lets only the finish ride here.  With n_gates > 0 the next gates are sampled from
 * log_alpha as it is during this call, i.e. before an update that uses this step's dlog_alpha.
 * job and the arrays it points to are host memory, read before the call returns.
 */
typedef struct {
    const flop_gate_grad_pending* items;   /* earlier layers of the step (from flop_bwd_deferred); may be NULL */
    int32_t count;
    const float* log_alpha;                /* the arguments of flop_gate_sample_l0 for the next step */
    const float* u;
    int64_t n_gates;
    flop_hc hc;
    float* z;
    float* dzda;
    const float* w;
    float* l0_sum;
    float* l0_grad;
    void* workspace;
    size_t workspace_bytes;
} flop_boundary_job;

int flop_bwd_boundary(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                      const void* dy, int64_t lddy, const void* x, int64_t ldx,
                      const void* Q, int64_t ldq, const void* P, int64_t ldp,
                      const float* z, const float* dzda, const void* g_saved, int64_t ldg,
                      void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dP, int64_t lddp,
                      float* dlog_alpha, int accumulate,
                      void* workspace, size_t workspace_bytes, const flop_boundary_job* job, void* stream);

/*
 * flop_gate_sample_l0 for a whole step and flop_fwd of the step's first layer in one call: job (count == 0,
 * no items) describes the gate vectors of the model - log_alpha, u in, z, dzda, l0_sum, l0_grad out, as in
 * flop_gate_sample_l0 - and this layer's r gates are entries gate_offset .. gate_offset + r - 1 of them.
 * Where the first product runs on the asynchronous-transfer kernel (bfloat16, rows at least 4-byte aligned) and
 * the model has at most 4096 gates, the layer's gates are computed in that product's epilogue from log_alpha
 * and u, and extra workgroups of the same launch write z, dzda and Eq.(3) for all n_gates gates: the step
 * needs no gate launch.  Otherwise the gate kernel runs first and flop_fwd follows.  Results equal those of the
 * two separate calls bit for bit (Eq.(3) to float32 rounding).  Later layers of the step call flop_fwd with
 * their part of job->z.
 */
int flop_fwd_sampling(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                      const void* x, int64_t ldx, const void* Q, int64_t ldq, const void* P, int64_t ldp,
                      const flop_boundary_job* job, int64_t gate_offset, void* g_saved, int64_t ldg, void* y, int64_t ldy,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Gate-gradient step of the backward pass on its own (the reduction flop_bwd runs
 * after its contractions; Section 3: the gradient reaches alpha through z):
 *   dlog_alpha_k = (sum_i dh_ik g_ik) / z_k^2 * dzda_k,   dh = dg .* z,  g = h .* z,
 * i.e. dz_k * dz_k/dlog_alpha_k with dz_k = sum_i dg_ik h_ik; exactly 0 where
 * z_k == 0 or dzda_k == 0.  dh[n, r], g[n, r]: element type dt; dlog_alpha[r]
 * float32, overwritten or accumulated.  Rows are reduced in chunks of 32 and the
 * chunk sums added in a fixed order (deterministic).
 * workspace: >= flop_workspace_bytes(FLOP_OP_GATE_GRAD, dt, n, 0, r, 0), 256-byte aligned.
 */
int flop_gate_grad(flop_dtype dt, int64_t n, int64_t r, const void* dh, int64_t ldh, const void* g, int64_t ldg,
                   const float* z, const float* dzda, float* dlog_alpha, int accumulate,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Expected L0 norm, Eq.(3), with the temperature written out:
 *   p_k = sigmoid(log_alpha_k - beta * log(-l / r))        (= P[z_k > 0])
 *   out_sum[0] = sum_k w_k p_k        (w == NULL: w_k = 1)
 * w carries the parameter-block sizes that turn the sum into the expected
 * model size s(alpha) of Section 4.3 (d + dout for a rank-1 component).
 * grad (nullable) receives d out_sum / d log_alpha_k = w_k p_k (1 - p_k).
 * log_alpha may be the concatenation of the gates of many matrices.
 * out_sum: device float32[1].  n_gates == 0 writes 0.  The sum is carried in
 * float64 and is deterministic.
 * workspace: >= flop_workspace_bytes(FLOP_OP_EXPECTED_L0, FLOP_F32, n_gates,0,0,0).
 */
int flop_expected_l0(const float* log_alpha, const float* w, int64_t n_gates, flop_hc hc,
                     float* out_sum, float* grad,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * flop_gate_sample (TRAIN mode) and flop_expected_l0 of the same log_alpha in one
 * call: z, dzda as there; l0_sum[0] = sum_k w_k p_k and l0_grad[k] = w_k p_k (1 - p_k)
 * (w, dzda, l0_grad nullable).  Gate vectors of up to 4096 entries take one launch,
 * longer ones the two separate kernels.  workspace as for flop_expected_l0.
 */
int flop_gate_sample_l0(const float* log_alpha, const float* u, int64_t n_gates, flop_hc hc,
                        float* z, float* dzda, const float* w, float* l0_sum, float* l0_grad,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Compaction for inference (Section 4.1, last paragraph; Section 4.4):
 * component k is kept iff z[k] > 0 (exact comparison on the stored float32),
 * survivors keep ascending k.  With r' survivors:
 *   r_out[0] = r' (device int32)      idx[t] = k_t, t < r' (device int32, capacity r)
 *   Qc[t, :] = Q[k_t, :]  (r' x d, ld ldqc)        zc[t] = z[k_t]
 *   Pc[:, t] = P[:, k_t]  (dout x r', ld ldpc)
 * absorb_z_into_Q != 0 stores Qc[t, :] = round_dt(z[k_t] * Q[k_t, :]) instead
 * (the gate folded into one factor); zc then still holds z[k_t].
 * Rows t of Qc, columns t of Pc and entries of zc with r' <= t < min(r, 32*ceil(r'/32))
 * are zero-filled so that a following flop_fwd may use a rank rounded up to 32.
 * Outputs are sized by the caller for the worst case: Qc has r rows, ldpc >= r,
 * zc and idx have r entries.  Qc/Pc/zc are nullable (skipped).  Copies are
 * bit-exact.  r == 0 writes r_out = 0.
 * workspace: >= flop_workspace_bytes(FLOP_OP_COMPACT, dt, 0, d, r, dout).
 */
int flop_compact(flop_dtype dt, int64_t d, int64_t r, int64_t dout,
                 const float* z, const void* Q, int64_t ldq, const void* P, int64_t ldp,
                 int absorb_z_into_Q, int32_t* r_out, int32_t* idx,
                 void* Qc, int64_t ldqc, void* Pc, int64_t ldpc, float* zc,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Gated adaptive embedding (Section 4.2): word cluster c (clusters sorted by word
 * frequency) owns the vocabulary ids [id_begin, id_end), a table E_c[id_end-id_begin, dim],
 * a projection O_c[dim, d] and one Hard-Concrete gate per reduced dimension, so that
 * the embedding of id t is row t - id_begin of E_c G_c O_c:
 *     y[i, :] = (E_c[ids[i] - id_begin, :] .* z_c) O_c          (c = cluster of ids[i])
 * The struct is a HOST array entry; the pointers inside are DEVICE pointers.
 * Clusters must be ascending and disjoint; at most 8 clusters and 16384 tokens
 * per call (the batch is sorted by one workgroup in LDS).
 */
typedef struct {
    int64_t id_begin, id_end;     /* vocabulary range of the cluster */
    int64_t dim;                  /* reduced dimension d_c = number of gates */
    const void* E; int64_t lde;   /* E_c, element type dt */
    const void* O; int64_t ldo;   /* O_c, element type dt */
    const float* z;               /* gates z_c[dim] from flop_gate_sample */
    const float* dzda;            /* flop_embed_bwd only: dz/dlog_alpha[dim] (needed with dlog_alpha) */
    void* dE; int64_t ldde;       /* flop_embed_bwd only, nullable: gradient table, see below */
    void* dO; int64_t lddo;       /* flop_embed_bwd only, nullable: dO_c[dim, d], overwritten */
    float* dlog_alpha;            /* flop_embed_bwd only, nullable: [dim], overwritten */
} flop_embed_cluster;

/*
 * Forward.  ids[n_tokens]: device int64; y[n_tokens, d] (ld ldy) in the caller's
 * token order.  Tokens whose id lies in no cluster leave their row of y untouched.
 * `saved` (device, 256-byte aligned, >= flop_workspace_bytes(FLOP_OP_EMBED_FWD, dt,
 * n_tokens, d, sum of dim, 0) bytes) receives what the backward pass needs: the
 * sorted token order, the per-cluster segments and the gathered gated rows
 * g_c = E_c[rows] .* z_c (rounded to dt); keep it unchanged until flop_embed_bwd.
 */
int flop_embed_fwd(flop_dtype dt, int64_t n_tokens, const int64_t* ids, int32_t n_clusters,
                   const flop_embed_cluster* clusters, int64_t d, void* y, int64_t ldy,
                   void* saved, size_t saved_bytes, void* stream);

/*
 * Backward, per cluster over its tokens i (row_i = ids[i] - id_begin, g_i = E_c[row_i,:] .* z_c):
 *   dg_i = dy_i O_c^T               dO_c = sum_i g_i^T dy_i
 *   dE_c[row_i, :] += dg_i .* z_c   (tokens repeating a word accumulate)
 *   dz = sum_i dg_i .* E_c[row_i,:] dlog_alpha_c = dz .* dzda_c
 * dE_c is a table of the shape of E_c of which ONLY the rows of words that occur
 * in the batch are written (each with its complete sum, accumulated in token order
 * in float32, rounded once); all other rows are left as they are.  touched_ids
 * (device int64[n_tokens], nullable) receives the distinct ids of the batch in
 * ascending order and n_touched (device int32[1], nullable) their number.
 * Deterministic.  workspace: >= flop_workspace_bytes(FLOP_OP_EMBED_BWD, dt,
 * n_tokens, d, sum of dim, 0), 256-byte aligned.
 */
int flop_embed_bwd(flop_dtype dt, int64_t n_tokens, int32_t n_clusters, const flop_embed_cluster* clusters,
                   int64_t d, const void* dy, int64_t lddy, const void* saved, size_t saved_bytes,
                   int64_t* touched_ids, int32_t* n_touched,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Train-time active ranks.  The mask z is sampled once per step and shared by
 * the whole batch (Section 4.3, last paragraph), and a component with z_k = 0
 * adds nothing to y nor to any gradient (Section 4.1: y = sum_k z_k p_k q_k x),
 * so a step can run on the surviving components only: flop_gate_sample, then
 * flop_compact on the sampled z, flop_gather_gates for dz/dalpha, the two
 * calls below on the compacted factors, and flop_expand_grads to put the
 * gradients back in place.  The number of survivors stays on the device:
 * r_active is the device int32 that flop_compact wrote (r_out); r_cap is the
 * capacity of the compacted buffers (normally r) and only sizes the launches.
 * Everything else is as in flop_fwd / flop_bwd with r replaced by r_active[0]:
 * columns >= r_active[0] of g_saved, dPc and rows of dQc are not written,
 * dlog_alpha_c[k] = 0 for r_active[0] <= k < r_cap.
 */
int flop_fwd_active(flop_dtype dt, int64_t n, int64_t d, int64_t r_cap, int64_t dout,
                    const void* x, int64_t ldx, const void* Qc, int64_t ldqc, const void* Pc, int64_t ldpc,
                    const float* zc, const int32_t* r_active, void* g_saved, int64_t ldg, void* y, int64_t ldy,
                    void* workspace, size_t workspace_bytes, void* stream);
int flop_bwd_active(flop_dtype dt, int64_t n, int64_t d, int64_t r_cap, int64_t dout,
                    const void* dy, int64_t lddy, const void* x, int64_t ldx,
                    const void* Qc, int64_t ldqc, const void* Pc, int64_t ldpc,
                    const float* zc, const float* dzda_c, const int32_t* r_active, const void* g_saved, int64_t ldg,
                    void* dx, int64_t lddx, void* dQc, int64_t lddqc, void* dPc, int64_t lddpc,
                    float* dlog_alpha_c, int accumulate,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The per-step preparation of the active-rank path in two launches instead of
 * five: flop_gate_sample in TRAIN mode (z, dzda: nullable outputs of length r),
 * flop_compact of Q and P on the sampled z (r_active, idx, Qc, Pc, zc as
 * there, no absorption) and flop_gather_gates of dzda (dzda_c, nullable).
 */
int flop_active_prepare(flop_dtype dt, int64_t d, int64_t r, int64_t dout,
                        const float* log_alpha, const float* u, flop_hc hc,
                        const void* Q, int64_t ldq, const void* P, int64_t ldp,
                        float* z, float* dzda, int32_t* r_active, int32_t* idx,
                        void* Qc, int64_t ldqc, void* Pc, int64_t ldpc, float* zc, float* dzda_c, void* stream);

/* dst[t] = src[idx[t]] for t < r_active[0] (float32 vectors of gates, e.g. dzda);
 * idx, r_active as written by flop_compact; r is the capacity of idx and dst. */
int flop_gather_gates(const float* src, const int32_t* idx, const int32_t* r_active, int64_t r,
                      float* dst, void* stream);

/*
 * Gradients of the compacted factors back to the full-size layout:
 *   dQ[k_t, :] = dQc[t, :],  dP[:, k_t] = dPc[:, t],  dlog_alpha[k_t] = dlog_alpha_c[t]   (k_t = idx[t], t < r_active[0])
 * and exact zeros in every other row of dQ, column of dP and entry of dlog_alpha,
 * which is their true value (closed components receive no gradient).
 * Any of the three outputs may be NULL (then its source may be NULL too).
 */
int flop_expand_grads(flop_dtype dt, int64_t d, int64_t r, int64_t dout,
                      const int32_t* r_active, const int32_t* idx,
                      const void* dQc, int64_t lddqc, const void* dPc, int64_t lddpc, const float* dlog_alpha_c,
                      void* dQ, int64_t lddq, void* dP, int64_t lddp, float* dlog_alpha, void* stream);

/*
 * Train-time active ranks without compacted copies of the factors (Section 4.3, last
 * paragraph; Section 4.1: a closed component adds nothing to y nor to any gradient).
 * The contractions read the open components straight out of the full-size factors
 * through the ascending index list idx[0 .. r_active[0]) that flop_active_prepare
 * (with Qc = Pc = NULL: one launch) or flop_compact wrote, and write the gradients of
 * those components straight into the full-size gradients.  For both factors to be
 * gathered by rows, P is held transposed:
 *   Pt[r, dout] ld ldpt: row k is the column p_k of P;  dPt[r, dout] likewise.
 *   zc[r], dzda_c[r]: gates and dz/dalpha of the open components in idx order
 *   g_active[n, r_active] ld ldg (ldg >= r): the saved activation (x Q[idx]^T) .* zc
 * Forward: y = g_active Pt[idx].  Backward: dx; rows idx of dQ and dPt; dlog_alpha[idx];
 * every other row of dQ and dPt and (unless accumulate != 0) entry of dlog_alpha is set
 * to exact zero, their true value.  dx, dQ, dPt, dlog_alpha are nullable.
 * workspace of the backward: >= flop_workspace_bytes(FLOP_OP_BWD, dt, n, d, r, dout).
 * Same results as flop_fwd / flop_bwd on (Q, P = Pt^T, z) up to summation order.
 */
int flop_fwd_active_indexed(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                            const void* x, int64_t ldx, const void* Q, int64_t ldq, const void* Pt, int64_t ldpt,
                            const float* zc, const int32_t* idx, const int32_t* r_active,
                            void* g_active, int64_t ldg, void* y, int64_t ldy, void* stream);
int flop_bwd_active_indexed(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout,
                            const void* dy, int64_t lddy, const void* x, int64_t ldx,
                            const void* Q, int64_t ldq, const void* Pt, int64_t ldpt,
                            const float* zc, const float* dzda_c, const int32_t* idx, const int32_t* r_active,
                            const void* g_active, int64_t ldg,
                            void* dx, int64_t lddx, void* dQ, int64_t lddq, void* dPt, int64_t lddpt,
                            float* dlog_alpha, int accumulate,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * Deterministic mask for inference as Section 4.4 states it: each gate is scored
 * by its term of Eq.(3), p_k = sigmoid(log_alpha_k - beta * log(-l / r)), the
 * `keep` best are kept and the rest clipped to zero, so that the number of open
 * gates matches a chosen L0 norm:  z_k = p_k for the kept gates, 0 otherwise
 * (feed z to flop_compact).  p is increasing in log_alpha, so gates are ranked by
 * log_alpha itself; among equal values the lower index is kept first, which makes
 * the kept set unique.  keep: host value, clamped to [0, n_gates]; if keep_device
 * is not NULL it is a device float32 (e.g. the expected L0 written by
 * flop_expected_l0) and keep = rint(keep_device[0]) instead.  kept (nullable):
 * device int32, receives the number kept.  NaNs in log_alpha rank above or below
 * all numbers by their sign bit.  log_alpha may concatenate several matrices
 * (one global ranking) or be one matrix.  One workgroup does the selection.
 */
int flop_topk_mask(const float* log_alpha, int64_t n_gates, int64_t keep, const float* keep_device,
                   flop_hc hc, float* z, int32_t* kept, void* stream);

/*
 * Augmented-Lagrangian size constraint of Section 4.3:
 *   g(lambda, alpha) = lambda1 (s - t) + lambda2 (s - t)^2
 * with s = scale * size_sum[0], size_sum the block-size weighted Eq.(3) sum and
 * size_grad[k] = w_k p_k (1 - p_k) its gradient, both as written by
 * flop_expected_l0 (device), scale a host factor that brings the sum to the unit
 * of the target t (1 / total parameters for a fraction), lambda = {lambda1, lambda2}
 * (device float32[2]).  Writes
 *   dlog_alpha[k] (+)= (lambda1 + 2 lambda2 (s - t)) * scale * size_grad[k]     (nullable; accumulate != 0 adds)
 *   out[0] = g,  out[1] = dg/dlambda1 = s - t,  out[2] = dg/dlambda2 = (s - t)^2   (device float32[3], nullable)
 * The caller's optimiser descends on log_alpha and ascends on lambda with these.
 */
int flop_lagrangian(const float* size_sum, const float* size_grad, int64_t n_gates, float scale, float t,
                    const float* lambda, float* dlog_alpha, int accumulate, float* out, void* stream);

/* Bytes of 256-byte-aligned device workspace the op needs for these sizes
 * (0 when it needs none).  For FLOP_OP_EXPECTED_L0 pass the gate count as n; for the
 * embedding ops pass the token count as n and the sum of the cluster dimensions as r. */
size_t flop_workspace_bytes(int op, flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout);

/* Static description of a flop_status. */
const char* flop_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FLOP_H */
