/*
 * canz - per-rank matrix-optimizer (Muon) step of Canzona, arxiv 2602.06079,
 * for AMD MI355X (gfx950).  C ABI of libcanz.so.
 *
 * Three calls follow the paper's statement of the problem:
 *   canz_partition_alpha   Algorithm 1 (Sec. 3.2): which rank owns which whole matrix.  CPU.
 *                          (canz_partition_naive: the static rule of Eq. 1 it replaces.)
 *   canz_microgroup_plan   batches one rank's same-shape matrices for one launch.        CPU.
 *                          (canz_tp_schedule: TP micro-groups with rollback, Algorithms 2-4.)
 *   canz_muon_step         Delta W = Muon_step(G, States) (Sec. 4.1 stage (2), Sec. 3.3
 *                          stage (2)): momentum, Frobenius normalisation, k Newton-Schulz
 *                          steps, scaled update - enqueued on a HIP stream.
 *
 * General rules
 *   - Every function returns CANZ_OK (0) or a negative error code; nothing throws.
 *     canz_last_error() gives a message for the calling thread's last failure.
 *   - The library never allocates or frees device memory and never synchronises a
 *     stream or the device.  Host arrays passed in are read during the call only.
 *   - "host" / "device" in a comment says where a pointer must point.
 *   - An array whose stated size is zero may be passed as NULL.
 *   - Ranks are numbered 0 .. n_ranks-1 (the paper counts from 1).
 */
#ifndef CANZ_H
#define CANZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CANZ_OK = 0,
  CANZ_EINVAL = -1,       /* null pointer, value out of range, inconsistent sizes   */
  CANZ_ESHAPE = -2,       /* shape not supported by a kernel (alignment, tp split)  */
  CANZ_EWORKSPACE = -3,   /* workspace missing, misaligned or too small             */
  CANZ_EHIP = -4,         /* a HIP call or kernel launch failed                     */
  CANZ_EUNSUPPORTED = -5  /* unknown enum value                                     */
};

enum { CANZ_COST_NUMEL = 0, CANZ_COST_NS_FLOPS = 1, CANZ_COST_SHAMPOO_FLOPS = 2, CANZ_COST_SOAP_FLOPS = 3 };
#define CANZ_SOAP_COST_MAX_PRECOND_DIM 10000 /* the limit CANZ_COST_SOAP_FLOPS assumes for canz_soap_hparams.max_precond_dim */
enum { CANZ_DT_F32 = 0, CANZ_DT_BF16 = 1 };
enum { CANZ_SCALE_NONE = 0, CANZ_SCALE_ASPECT = 1, CANZ_SCALE_RMS = 2 };
enum { CANZ_PREC_BF16 = 0, CANZ_PREC_F32 = 1 };
enum { CANZ_OUT_PARAM = 0, CANZ_OUT_DELTA = 1 };

/* Message for the last error on this thread (static storage, never NULL). */
const char* canz_last_error(void);
/* Library version string, e.g. "0.1.0". */
const char* canz_version(void);

/*
 * canz_partition_alpha - alpha-balanced greedy LPT partitioning, Algorithm 1 (Sec. 3.2;
 * walkthrough in App. C "Detailed Walkthrough of Load-Balancing Algorithms").
 *
 * The flat parameter list is cut into n_buckets ordered buckets; bucket i holds the
 * parameters bucket_off[i] .. bucket_off[i+1]-1.  Buckets are visited by total load,
 * heaviest first (equal loads: lower index first).  For each bucket the deficits
 * d_r = max(0, mu - L_r) give v_fill = d / sum(d) (v_even if the sum is 0), the target is
 * W^k * ((1-alpha) v_even + alpha v_fill), and the running sum of targets is projected
 * onto the nearest parameter boundary (equal distance: the smaller index).
 *
 * All arguments are host pointers owned by the caller.
 *   rows, cols   [n_mats]  matrix shapes (used when cost == NULL)
 *   cost         [n_mats]  load W(p) >= 0 per parameter, or NULL to derive it from
 *                          cost_kind: CANZ_COST_NUMEL rows*cols (the paper's default),
 *                          CANZ_COST_NS_FLOPS 5*(4 m^2 n + 2 m^3), m = min, n = max,
 *                          CANZ_COST_SHAMPOO_FLOPS the FLOPs of canz_shampoo_step at its default
 *                          25 root iterations, (4 r c (r + c) + 200 (r^3 + c^3)) / 2^20 rounded
 *                          down (the cost follows the operator, App. D.5),
 *                          CANZ_COST_SOAP_FLOPS the FLOPs of canz_soap_step with a refresh every 10th
 *                          step and max_precond_dim = CANZ_SOAP_COST_MAX_PRECOND_DIM: with s1 and s3 the
 *                          sums of d and d^3 over the sides d (of r, c) within that limit, the only
 *                          ones that keep a basis, ((120 r c s1 + 7 s3) / 15) / 2^20, both divisions
 *                          rounded down
 *   bucket_off   [n_buckets+1] non-decreasing, bucket_off[0] = 0, last = n_mats
 *   alpha        blend factor in [0, 1]: 1 = fill deficits, 0 = even split per bucket
 *   cut_out      [n_buckets*(n_ranks+1)] cut vectors s_i in the original bucket order:
 *                rank r owns parameters cut[i][r] .. cut[i][r+1]-1 of bucket i
 *                (indices relative to the bucket)
 *   owner_out    [n_mats]  owning rank of each parameter
 *   load_out     [n_ranks] final accumulated load L_r
 * Real-valued steps run in IEEE fp64 in a fixed order (mu = total/R; deficits summed by
 * ascending rank; v = (1-alpha)*(1/R) + alpha*(d/D); target = W^k * v; C += target), so
 * results are reproducible bit for bit.  Total load must stay below 2^53 (integers above
 * that are not exact in fp64).
 * Errors: CANZ_EINVAL for null pointers, n_ranks < 1, alpha outside [0,1], malformed
 * bucket_off, negative cost, a load or a total load of 2^53 or more (computed without
 * wrap-around); CANZ_EUNSUPPORTED for an unknown cost_kind.
 */
int canz_partition_alpha(int64_t n_mats, const int64_t* rows, const int64_t* cols,
                         const int64_t* cost, int32_t cost_kind,
                         int64_t n_buckets, const int64_t* bucket_off,
                         int32_t n_ranks, double alpha,
                         int64_t* cut_out, int32_t* owner_out, int64_t* load_out);

/*
 * canz_partition_naive - the Atomic Ownership Rule (Sec. 3.1, Eq. 1): the static layout
 * without load balancing, kept as the baseline Algorithm 1 is compared with.  Applied to
 * every bucket on its own (each bucket is cut into R equal segments, App. B.1): with stride
 * S = |B_i| / R, rank r owns parameter p iff r S <= Start_Index(p) < (r + 1) S, the start
 * index taken inside the bucket; computed exactly as r = floor(Start_Index(p) * R / |B_i|).
 * One bucket spanning everything gives the rule over the whole buffer.
 *   numel [n_mats] elements per parameter, in buffer order; bucket_off [n_buckets+1] as in
 *   canz_partition_alpha; owner_out [n_mats]; load_out [n_ranks] elements owned per rank.
 * Host pointers, caller-owned.
 * Errors: CANZ_EINVAL for null pointers, n_ranks < 1, negative sizes, malformed bucket_off.
 */
int canz_partition_naive(int64_t n_mats, const int64_t* numel, int64_t n_buckets, const int64_t* bucket_off,
                         int32_t n_ranks, int32_t* owner_out, int64_t* load_out);

/*
 * canz_microgroup_plan - group the matrices one rank owns into same-shape batches.
 *
 * The paper's micro-groups fuse tensors for one collective (Sec. 4, Algorithm 2); here a
 * micro-group is the unit of one batched launch, so its members share (rows, cols, dtype).
 * Classes are ordered by per-matrix element count, largest first, ties by smallest member
 * id (the deterministic (W(p), ID_p) order of Algorithm 2, Phase 1); inside a class ids
 * ascend and are cut into consecutive chunks of at most max_mats matrices and at most
 * cmax_bytes bytes of bf16 matrix data (the role of C_max).
 *
 * Host pointers, caller-owned.
 *   rows, cols, dtype, owner [n_mats]; rank selects owner[p] == rank
 *   max_mats     0 = no cap;  cmax_bytes 0 = no cap
 *   n_groups_out number of groups G
 *   group_off_out [n_owned+1 capacity] offsets into member_out, G+1 entries written
 *   member_out   [n_owned capacity] matrix ids, group after group
 * Capacity n_mats+1 / n_mats always suffices.
 * Errors: CANZ_EINVAL for null pointers or negative caps; CANZ_ESHAPE if one matrix alone
 * exceeds cmax_bytes (Algorithm 3's "single item exceeds C_max").
 */
int canz_microgroup_plan(int64_t n_mats, const int64_t* rows, const int64_t* cols,
                         const int32_t* dtype, const int32_t* owner, int32_t rank,
                         int32_t max_mats, int64_t cmax_bytes,
                         int64_t* n_groups_out, int64_t* group_off_out, int64_t* member_out);

/*
 * canz_tp_schedule - micro-group construction with greedy rollback for tensor-parallel
 * fragments (Algorithm 2, Sec. 4.2; Algorithms 3 and 4 in App. C): which tensors are fused
 * into one gather/scatter round and which host rank computes each of them.
 *
 * Tensors are taken in LPT order (cost descending, equal costs by ascending id).  A group
 * grows one tensor at a time; after each addition it is scheduled onto the n_ranks host
 * ranks with the LPT rule on a min-heap of (load, rank) pairs (smallest load first, lower
 * rank among equals); if the largest rank load would exceed cmax, the addition is rolled
 * back, the group is final and the tensor opens the next group.
 *
 * Host pointers, caller-owned.
 *   cost          [n_mats] W(p) >= 0 (the paper uses numel)
 *   cmax          capacity C_max of one group, in cost units, per host rank
 *   n_groups_out  number of groups G
 *   group_off_out [n_mats+1] offsets into member_out / host_rank_out, G+1 entries written
 *   member_out    [n_mats] tensor ids, group after group, in the order the solver assigns
 *                 them (descending cost)
 *   host_rank_out [n_mats] host rank of member_out[i]
 *   group_load_out[n_mats] largest rank load L_max of each group, G entries written
 * Errors: CANZ_EINVAL for null pointers, n_ranks < 1, negative cost or capacity;
 * CANZ_ESHAPE if one tensor alone exceeds cmax (Algorithm 3's error case).
 */
int canz_tp_schedule(int64_t n_mats, const int64_t* cost, int32_t n_ranks, int64_t cmax,
                     int64_t* n_groups_out, int64_t* group_off_out, int64_t* member_out,
                     int32_t* host_rank_out, int64_t* group_load_out);

/*
 * One micro-group for canz_muon_step: n_mats matrices of identical shape and dtypes.
 * Every matrix is rows x cols, row-major, dense.  With tp > 1 the gradient (and, with
 * CANZ_OUT_DELTA, the output) of each matrix is held as tp column fragments of shape
 * rows x (cols/tp) in separate buffers (column-parallel split, App. B.2; gathered before
 * and scattered after the computation, Sec. 4.1 stages (1) and (3)).
 * The three pointer tables are HOST arrays of DEVICE pointers; they are read during the
 * call and may be freed on return.  The device buffers must stay valid until the stream
 * has finished the step.  Device pointers must be 16-byte aligned; with tp > 1 the
 * fragment width cols/tp must be a multiple of 8 (whole matrices may have any extents).
 * rows and cols are at most 4194240 each.  grad, mom and out buffers must not overlap.
 * Magnitudes: the normalisation is applied as a scalar after squares of the unnormalised
 * U = M (or G + beta M) have been formed in fp32, so the root-mean-square of U must lie within
 * about [1e-15, 1e+15] (sums of squares must neither underflow nor overflow fp32); gradients of
 * any realistic scale, including loss-scaled ones, are far inside.
 */
typedef struct {
  int64_t rows, cols;
  int32_t n_mats;
  int32_t tp;               /* 1 = whole matrices; >1 = column fragments (max 8)          */
  int32_t grad_dtype;       /* CANZ_DT_F32 or CANZ_DT_BF16                                 */
  int32_t out_dtype;        /* dtype of the out buffers                                    */
  const void* const* grad;  /* [n_mats*tp] fragment f of matrix i at grad[i*tp+f]          */
  void* const* mom;         /* [n_mats]    fp32 momentum, whole, updated in place          */
  void* const* out;         /* CANZ_OUT_PARAM: [n_mats] whole parameters, updated in place
                               CANZ_OUT_DELTA: [n_mats*tp] Delta W fragments, overwritten  */
} canz_group;

/*
 * Hyper-parameters of the step.  Per matrix (Sec. 4.1 stage (2); App. B.3, Eq. 5):
 *   M <- beta M + G;  U = M (nesterov: U = G + beta M)
 *   X = U / (||U||_F + eps); the iteration runs on the wide orientation
 *   ns_steps times: A = X X^T; B = b A + c A A; X <- a X + B X
 *   O = X; scale = 1 | sqrt(max(1, rows/cols)) | 0.2 sqrt(max(rows, cols))
 *   CANZ_OUT_PARAM: P <- P (1 - lr weight_decay) - lr scale O
 *   CANZ_OUT_DELTA: Delta W = - lr scale O
 */
typedef struct {
  float beta, lr, weight_decay, eps;
  int32_t nesterov;
  int32_t ns_steps;         /* >= 0 */
  float a, b, c;            /* c = 0 gives the cubic iteration */
  int32_t scale_mode;       /* CANZ_SCALE_* */
  int32_t precision;        /* CANZ_PREC_BF16: bf16 MFMA, fp32 accumulate; CANZ_PREC_F32: fp32 */
  int32_t out_mode;         /* CANZ_OUT_* */
} canz_muon_hparams;

/*
 * canz_muon_workspace_bytes - device scratch needed by canz_muon_step for these groups:
 * the maximum over the launch batches the call will form (consecutive matrices of equal
 * dtypes and equal shape up to a transpose, at most 128 / tp of them and at most 2^30
 * padded elements per batch unless one matrix alone is larger; up to four consecutive small
 * batches run side by side within the same 2^30 elements, otherwise batches run one after
 * another on the stream, so for matrices below 2^30 elements at most about 10 GB are
 * asked for in bf16 mode, twice that in fp32 mode, whatever the share).
 * g: host array [n_groups]; pointer tables inside may be NULL for this call.
 */
int canz_muon_workspace_bytes(const canz_group* g, int32_t n_groups,
                              const canz_muon_hparams* hp, size_t* bytes_out);

/*
 * canz_muon_step - enqueue one optimizer step for the given micro-groups on hip_stream.
 *   g               host array [n_groups]
 *   workspace       device, 256-byte aligned, at least canz_muon_workspace_bytes() bytes,
 *                   caller-owned; contents are scratch and need not be initialised
 *   hip_stream      a hipStream_t (NULL = the null stream)
 * Returns after enqueueing; completion follows stream order.  Results per matrix do not
 * depend on which other matrices share the group or the call, with one exception in bf16 mode:
 * Gram products with more than 12800 columns (k-steps) may have the tiles left over behind the
 * last full round of a launch summed in several k-slices, which changes fp32 rounding (far
 * below the tolerance) for matrices whose tiles fall there.  The call issues kernel
 * launches only (no memset, no copy, no allocation, no synchronisation), so with profiling
 * off it may be recorded into a HIP graph; the pointer tables are baked into the recorded
 * launches.  Calls on different streams may overlap if their workspaces are distinct.
 * Errors: CANZ_EINVAL (null pointers, n_mats < 0, tp outside 1..8, ns_steps < 0),
 * CANZ_ESHAPE (cols not divisible by tp, fragment width not a multiple of 8, an extent
 * above 4194240),
 * CANZ_EWORKSPACE, CANZ_EUNSUPPORTED (dtype / mode enums), CANZ_EHIP (launch failure;
 * earlier groups of the call may already be enqueued).
 */
int canz_muon_step(const canz_group* g, int32_t n_groups, const canz_muon_hparams* hp,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Shampoo, the second matrix optimizer the paper runs through the same planner ("Generalization
 * to Other Optimizers (Shampoo & SOAP)", App. C; "preconditioning matrices derived from the
 * Kronecker product of gradients", App. B.3), under the generic update of App. B.3, Eq. 5.
 * Per matrix G (rows x cols), with its two statistics as optimizer state:
 *   L <- beta L + G G^T   (rows x rows),   R <- beta R + G^T G   (cols x cols)
 *   O = (L + eps I)^(-1/4) G (R + eps I)^(-1/4)
 *   CANZ_OUT_PARAM: P <- P (1 - lr weight_decay) - lr O;   CANZ_OUT_DELTA: Delta W = - lr O
 * beta = 1 gives the running sums of the original algorithm (initialise L and R to eps0 I for
 * its L_0 = eps0 I, or to zero and pass eps).  The inverse fourth roots are computed in fp32
 * by root_iters rounds of a matmul-only coupled Newton iteration
 * (T = (5 I - M) / 4; X <- X T; M <- T^4 M; from M = z A, X = z^(1/4) I, z = 5 / (2 b) with
 * b = ||A|| ||A'^4||^(1/4), A' = A / ||A||, Frobenius norms: an upper bound of the largest eigenvalue
 * that is at most d^(1/8) above it, for two products before the first round),
 * which converges to A^(-1/4) for symmetric positive definite A = S + eps I once the
 * smallest eigenvalue of M has grown to 1: about log(d^(1/8) cond(A) / 2.5) / log(2.44) + 4 rounds
 * (22 rounds cover cond(A) <= 10^6 up to d = 32768; 25 is the default).  eps must be large enough that A is positive definite in fp32:
 * eps >= 10^-6 lambda_max(S) is safe; below that the iteration may diverge (NaN output).
 * Because the statistics are held in fp32, the update's relative error against exact arithmetic
 * grows like 1.3e-8 lambda_max(S) / eps: below 5e-3 for eps >= 10^-5 lambda_max(S).
 *
 * One micro-group: n_mats matrices of identical shape and dtypes; grad / out / tp as in
 * canz_group; left[i] (rows x rows) and right[i] (cols x cols) are fp32, dense, row-major,
 * device, 16-byte aligned, updated in place (they stay exactly symmetric).
 * Practical Shampoo recomputes the roots only every n-th step.  A caller that passes lroot / rroot
 * (same layout as left / right) gets the roots of a step with keep_roots = 0 written there, and a
 * step with keep_roots = 1 takes them from there instead of computing them: about 2 % of the cost
 * of a full step.
 * Consecutive groups of one call that agree in shape, tp, dtypes and in which tables they pass run as one group.
 */
typedef struct {
  int64_t rows, cols;
  int32_t n_mats;
  int32_t tp;
  int32_t grad_dtype;       /* CANZ_DT_F32 or CANZ_DT_BF16 */
  int32_t out_dtype;
  const void* const* grad;  /* [n_mats*tp] */
  void* const* left;        /* [n_mats] */
  void* const* right;       /* [n_mats] */
  void* const* out;         /* [n_mats] parameters, or [n_mats*tp] Delta W fragments */
  void* const* lroot;       /* [n_mats] rows x rows, or NULL: (L + eps I)^(-1/4) kept between steps */
  void* const* rroot;       /* [n_mats] cols x cols, or NULL (both tables or neither) */
} canz_shampoo_group;

typedef struct {
  float beta, lr, weight_decay, eps;
  int32_t root_iters;       /* >= 1; 25 is the default (also that of the cost model CANZ_COST_SHAMPOO_FLOPS) */
  int32_t out_mode;         /* CANZ_OUT_* */
  int32_t keep_roots;       /* 0: the roots are computed on every step (the algorithm as published);
                               1: the step uses the roots in lroot / rroot as they are (the statistics are
                               still updated): the amortised variant that recomputes them every n-th step */
} canz_shampoo_hparams;

/*
 * canz_shampoo_workspace_bytes - device scratch canz_shampoo_step needs for these groups (the
 * largest of its launch batches: same-shape matrices of one group, as many as fit in about
 * 8 GB of fp32 working matrices, at least one).  Pointer tables may be NULL for this call.
 */
int canz_shampoo_workspace_bytes(const canz_shampoo_group* g, int32_t n_groups,
                                 const canz_shampoo_hparams* hp, size_t* bytes_out);

/*
 * canz_shampoo_step - enqueue one Shampoo step for the given micro-groups on hip_stream.
 * Same conventions as canz_muon_step: host tables of device pointers read during the call,
 * caller-owned 256-byte aligned workspace whose contents are scratch, kernel launches only
 * (no allocation, copy, memset or synchronisation), completion in stream order.
 * Errors: CANZ_EINVAL (null pointers, n_mats < 0, tp outside 1..8, root_iters < 1, eps < 0, one root table
 * without the other, keep_roots without the tables),
 * CANZ_ESHAPE (cols not divisible by tp, fragment width not a multiple of 8, an extent above
 * 32768), CANZ_EWORKSPACE, CANZ_EUNSUPPORTED (dtype / mode enums), CANZ_EHIP.
 */
int canz_shampoo_step(const canz_shampoo_group* g, int32_t n_groups, const canz_shampoo_hparams* hp,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * SOAP, the third matrix optimizer the paper runs through the same planner ("Generalization to
 * Other Optimizers (Shampoo & SOAP)", App. C: "distinct cubic-complexity operations (SVD and
 * Eigendecomposition, respectively)"), under the generic update of App. B.3, Eq. 5: Adam run in
 * the eigenbasis of Shampoo's statistics.  Per matrix G (rows x cols) at step t = 1, 2, ...:
 *   M <- beta1 M + (1 - beta1) G                              (momentum, original space)
 *   G' = Q_L^T G Q_R,   M' = Q_L^T M Q_R                      (rotation into the bases)
 *   V <- beta2 V + (1 - beta2) G' * G'                        (elementwise, rotated space)
 *   N' = m / (sqrt(v) + eps),  m = M' / (1 - beta1^t), v = V / (1 - beta2^t) with bias
 *                              correction, m = M', v = V without
 *   N = Q_L N' Q_R^T;  CANZ_OUT_PARAM: P <- P (1 - lr weight_decay) - lr N;  CANZ_OUT_DELTA: Delta W = -lr N
 *   L <- beta2 L + (1 - beta2) G G^T,   R <- beta2 R + (1 - beta2) G^T G
 *   if refresh:  Q_L <- orthogonal factor of the QR decomposition of L Q_L,  Q_R likewise of R Q_R
 *                (one round of orthogonal iteration towards the eigenvectors; V is not rotated)
 * Between two refreshes the bases stand still, so M' obeys the momentum recurrence itself,
 * M' <- beta1 M' + (1 - beta1) G', and need not be rotated anew: a caller that passes mom_rot saves one
 * of the three rotations of a step.  With mom_rot_valid = 0 the step rotates M as above and leaves M'
 * in mom_rot; with mom_rot_valid = 1 it takes M' from mom_rot and updates it in place; a refresh step
 * leaves it rotated into the new bases.  So mom_rot is valid after every step, and a caller passes 0
 * only on the first step and after changing M or a basis itself.  M stays the state in the original space.
 * A side longer than max_precond_dim keeps no statistic and no basis (its Q is the identity and
 * its tables may be NULL); at least one side must be within the limit, and a side with a basis may
 * have at most 12288 rows or columns (the cited implementation's default limit is 10000).  Everything is fp32,
 * unless bf16_rotations is set: then the products that rotate G (and M) into the bases and N' back take their
 * operands (G, M, the bases, N' and the intermediate of a two-sided rotation) rounded to bf16 and accumulate in
 * fp32, about four times faster and with a relative error of the update near 5e-3 for a state with history (each
 * rounding is 2^-9 relative; on a first step from V = 0 the direction is nearly the sign of G', which the
 * rounding flips where |G'| is below it: about 7e-2 there); that includes the re-rotation of mom_rot after a refresh, whose last product still leaves its fp32
 * sums in mom_rot.  Momentum, second moment, the statistics' sums and the refresh stay in fp32.  Independently
 * of this switch, gradients that arrive as bf16 have their statistics G G^T and G^T G computed on the bf16 matrix
 * cores: their values are the exact operands, each product is exact in fp32 and the sums are kept in fp32.
 * The caller owns all state and decides when to refresh (every f-th step) and how the bases
 * start (identity, or eigenvectors of the first statistics computed elsewhere).  The QR step is
 * a blocked Householder factorisation: the basis it writes is orthonormal to fp32 rounding and
 * its columns are fixed up to sign (which the step does not depend on); where L Q_L is rank
 * deficient the trailing columns are some orthonormal completion.
 *
 * Consecutive groups of one call that agree in shape, tp, dtypes and in which tables they pass run as one
 * group (a matrix's result does not depend on what shares its launch; a refresh fills the chip better the
 * more matrices it holds).
 *
 * One micro-group: n_mats matrices of identical shape and dtypes; grad / out / tp as in
 * canz_group; all state is fp32, dense, row-major, device, 16-byte aligned, updated in place:
 * mom[i], var[i] rows x cols; left[i], qleft[i] rows x rows; right[i], qright[i] cols x cols
 * (the columns of a basis are its vectors).
 */
typedef struct {
  int64_t rows, cols;
  int32_t n_mats;
  int32_t tp;
  int32_t grad_dtype;       /* CANZ_DT_F32 or CANZ_DT_BF16 */
  int32_t out_dtype;
  const void* const* grad;  /* [n_mats*tp] */
  void* const* mom;         /* [n_mats] */
  void* const* var;         /* [n_mats] */
  void* const* left;        /* [n_mats] */
  void* const* right;       /* [n_mats] */
  void* const* qleft;       /* [n_mats] */
  void* const* qright;      /* [n_mats] */
  void* const* out;         /* [n_mats] parameters, or [n_mats*tp] Delta W fragments */
  void* const* mom_rot;     /* [n_mats] rows x cols, or NULL: the rotated momentum M' kept between steps */
} canz_soap_group;

typedef struct {
  float beta1, beta2, lr, weight_decay, eps;
  int32_t step;             /* t >= 1, used by the bias correction */
  int32_t bias_correction;  /* 0 or 1 */
  int32_t refresh;          /* 1: refresh the bases at the end of this step */
  int32_t max_precond_dim;  /* >= 1 */
  int32_t out_mode;         /* CANZ_OUT_* */
  int32_t mom_rot_valid;    /* 1: mom_rot holds Q_L^T M Q_R of the M and the bases passed in */
  int32_t bf16_rotations;   /* 0: everything in fp32; 1: the rotations of steps 3 and 6 on bf16 operands */
} canz_soap_hparams;

/*
 * canz_soap_workspace_bytes - device scratch canz_soap_step needs for these groups and these
 * hyper-parameters (a refresh step needs more).  Pointer tables may be NULL for this call.
 */
int canz_soap_workspace_bytes(const canz_soap_group* g, int32_t n_groups, const canz_soap_hparams* hp,
                              size_t* bytes_out);

/*
 * canz_soap_step - enqueue one SOAP step for the given micro-groups on hip_stream.
 * Same conventions as canz_muon_step: host tables of device pointers read during the call,
 * caller-owned 256-byte aligned workspace whose contents are scratch, kernel launches only
 * (no allocation, copy, memset or synchronisation), completion in stream order.
 * Errors: CANZ_EINVAL (null pointers, n_mats < 0, tp outside 1..8, betas outside [0, 1), eps < 0,
 * step < 1, max_precond_dim < 1), CANZ_ESHAPE (cols not divisible by tp, fragment width not a
 * multiple of 8, an extent above 32768, a side with a basis above 12288), CANZ_EWORKSPACE, CANZ_EUNSUPPORTED (dtype / mode enums,
 * both extents above max_precond_dim), CANZ_EHIP.
 */
int canz_soap_step(const canz_soap_group* g, int32_t n_groups, const canz_soap_hparams* hp,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * canz_muon_step_static - canz_muon_step without a workspace argument, for callers that
 * cannot allocate device memory or may not call an allocator where the step is issued
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 * The scratch is an array of CANZ_STATIC_WORKSPACE_BYTES bytes inside the library's device
 * code; each GPU the library runs on holds its own copy until the process ends.  Same
 * kernels, same launch batches and bit-identical results as canz_muon_step with a workspace
 * of its own.  The call allocates and frees nothing on the device; on its first use on a
 * device it looks up that device's address of the array (hipGetSymbolAddress), afterwards it
 * only enqueues kernels on hip_stream.
 * The array's contents are scratch: nothing in it has to start at zero and nothing is kept
 * from one call to the next.  All calls on one GPU share the array, so steps that may run at
 * the same time on one GPU (two streams, two threads) race: serialise them, or give the
 * others their own workspace through canz_muon_step.
 * Errors: as canz_muon_step; CANZ_EWORKSPACE if canz_muon_workspace_bytes() for these groups
 * exceeds CANZ_STATIC_WORKSPACE_BYTES (nothing is enqueued then); CANZ_EHIP if the array's
 * address cannot be obtained.
 */
#define CANZ_STATIC_WORKSPACE_BYTES (128u << 20)
int canz_muon_step_static(const canz_group* g, int32_t n_groups, const canz_muon_hparams* hp,
                          void* hip_stream);

/*
 * Per-kernel timing of canz_muon_step / canz_shampoo_step / canz_soap_step, for benchmarks (the measurement protocol of
 * App. C.1 reports the optimizer time; this splits it by kernel).  While enabled, every
 * kernel launch of a step is bracketed by a pair of HIP events on the step's own stream.
 * Process-wide state (guarded by a lock; with profiling off a step only reads one flag): meant for
 * one benchmark thread, with steps that do not overlap.
 *   canz_profile_enable   creates (host-side) events for up to max_launches launches per
 *                         collection period and starts recording; launches beyond that
 *                         are not recorded.
 *   canz_profile_collect  waits for the recorded events, adds elapsed milliseconds and
 *                         launch counts per kernel kind into ms_out / launches_out
 *                         (host arrays of CANZ_KERNEL_KINDS entries) and starts a new period.
 *   canz_profile_disable  stops recording.
 */
enum {
  CANZ_KERNEL_MOMENTUM = 0, /* momentum + gather + cast + norm partial sums */
  CANZ_KERNEL_NORM = 1,     /* 1 / (||U|| + eps)                            */
  CANZ_KERNEL_GRAM = 2,     /* A = X X^T                                    */
  CANZ_KERNEL_POLY = 3,     /* B = a I + b A + c A A                        */
  CANZ_KERNEL_UPDATE = 4,   /* X <- B X (both orientations)                 */
  CANZ_KERNEL_FINAL = 5,    /* last B X fused with the parameter update     */
  CANZ_KERNEL_APPLY = 6,    /* update without Newton-Schulz steps           */
  CANZ_KERNEL_SH_LOAD = 7,  /* Shampoo: gather + cast of G, both orientations */
  CANZ_KERNEL_SH_STAT = 8,  /* Shampoo: L, R statistics                       */
  CANZ_KERNEL_SH_INIT = 9,  /* Shampoo: norm and start of the root iteration  */
  CANZ_KERNEL_SH_ROOT = 10, /* Shampoo: products of the root iteration        */
  CANZ_KERNEL_SH_APPLY = 11,/* Shampoo: L^(-1/4) G and (.) R^(-1/4) + update   */
  CANZ_KERNEL_SOAP_LOAD = 12,   /* SOAP: momentum, gather + cast, padded copies of the bases */
  CANZ_KERNEL_SOAP_ROTATE = 13, /* SOAP: rotations into and out of the bases (+ update)    */
  CANZ_KERNEL_SOAP_ADAM = 14,   /* SOAP: second moment and Adam's direction                */
  CANZ_KERNEL_SOAP_STAT = 15,   /* SOAP: L, R statistics                                   */
  CANZ_KERNEL_SOAP_QR = 16,     /* SOAP refresh: products of the blocked QR                */
  CANZ_KERNEL_SOAP_PANEL = 17,  /* SOAP refresh: panel factorisation, fills, basis store   */
  CANZ_KERNEL_KINDS = 18
};
int canz_profile_enable(int32_t max_launches);
int canz_profile_collect(double* ms_out, int64_t* launches_out);
int canz_profile_disable(void);

#ifdef __cplusplus
}
#endif
#endif /* CANZ_H */
