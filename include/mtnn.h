/*
 * mtnn.h -- C ABI of the MI355X (gfx950) NT-operation library.
 *
 * The library computes the NT operation C = A x B^T of the MTNN paper (Shi, Xu, Chu,
 * "Supervised Learning Based Algorithm Selection for Deep Neural Networks") in the two ways
 * the paper compares, and selects between them per (m, n, k):
 *
 *   NT   one GEMM kernel that reads B as stored                      (Eq. 2)
 *   TNN  out-of-place transpose of B, then an NN GEMM                (Algorithm 1, Eq. 1)
 *   MTNN a boosted-tree predictor picks NT (+1) or TNN (-1)          (Algorithm 2)
 *
 * Conventions for every call
 *   - matrices are row-major fp32; leading dimensions are in ELEMENTS;
 *   - A, B, C, in, out and workspace are DEVICE pointers owned by the caller; the library keeps no
 *     reference to them after the enqueued work has run.  The library allocates and frees no device
 *     memory: the one buffer it uses beyond a call's arguments is the scratch the caller lends it
 *     per stream with mtnn_set_scratch;
 *   - the kernels exist for gfx950 only: a call that would launch one while the current device is
 *     missing or of another architecture returns MTNN_ERR_NO_DEVICE and launches nothing;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); work is enqueued
 *     on it and the call returns without synchronising;
 *   - alpha = 1 and there is no beta*C term (Section II): C is overwritten;
 *   - padding elements (columns at or beyond the logical width when ld > width) are never
 *     written in outputs and never influence results when present in inputs;
 *   - the same inputs, shape and scratch capacity of the stream give bit-identical outputs on every
 *     call, inside or outside a stream capture (no atomics; how a product is divided over workgroups
 *     depends on (operation, m, n, k, alignment, scratch bytes registered) and nothing else);
 *   - the return value is MTNN_OK (0) or one of the MTNN_ERR_* codes below.  Arguments are
 *     validated on the host before any device call, so a call that fails validation has
 *     touched neither the device nor the outputs.
 *   - degenerate sizes (the paper is silent): m == 0 or n == 0 is a successful no-op; k == 0
 *     writes +0.0f to the m x n region of C (the empty sum); a transpose with rows == 0 or
 *     cols == 0 is a successful no-op.
 */
#ifndef MTNN_H
#define MTNN_H

#include <stddef.h>

#if defined(__GNUC__)
#define MTNN_API __attribute__((visibility("default")))
#else
#define MTNN_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MTNN_OK = 0,
    MTNN_ERR_DIM = 1,        /* a dimension is negative                                   */
    MTNN_ERR_NULL = 2,       /* a NULL pointer with a non-empty problem                   */
    MTNN_ERR_LD = 3,         /* a leading dimension smaller than the logical row length   */
    MTNN_ERR_ALIAS = 4,      /* an output range overlaps an input range                   */
    MTNN_ERR_WORKSPACE = 5,  /* workspace (mtnn_tnn) or scratch (an explicit split) missing or too small */
    MTNN_ERR_LAUNCH = 6,     /* the HIP runtime refused a launch                          */
    MTNN_ERR_MODEL = 7,      /* model file missing, malformed or of the wrong arity       */
    MTNN_ERR_ARG = 8,        /* any other invalid argument (bad config id, bad label ...) */
    MTNN_ERR_NO_DEVICE = 9   /* no usable gfx950 device                                   */
};

/* ---- dense operations --------------------------------------------------------------- */

/* NT operation, Eq. 2: C[i][j] = sum_l A[i][l] * B[j][l].
 * A: m x k (lda >= k).  B: n x k (ldb >= k).  C: m x n (ldc >= n), overwritten. */
MTNN_API int mtnn_nt(void *stream, int m, int n, int k,
            const float *A, int lda, const float *B, int ldb, float *C, int ldc);

/* NN operation, Eq. 1: C[i][j] = sum_l A[i][l] * B[l][j].
 * A: m x k (lda >= k).  B: k x n (ldb >= n).  C: m x n (ldc >= n), overwritten. */
MTNN_API int mtnn_nn(void *stream, int m, int n, int k,
            const float *A, int lda, const float *B, int ldb, float *C, int ldc);

/* Out-of-place transpose (Section III; the "transposeOnGPU" step of Algorithm 1):
 * out[c][r] = in[r][c], copied as 32-bit words (bit-exact, NaN payloads and -0 included).
 * in: rows x cols (ldin >= cols).  out: cols x rows (ldout >= rows). */
MTNN_API int mtnn_transpose(void *stream, int rows, int cols,
                   const float *in, int ldin, float *out, int ldout);

/* In-place transpose of a square n x n matrix (ld >= n): X[c][r] <-> X[r][c], bit-exact.  The paper
 * names in-place transposition as future work for the case where the memory for B^T is missing
 * (Section III, Section VI); the square case decomposes into independent tile swaps. */
MTNN_API int mtnn_transpose_inplace(void *stream, int n, float *X, int ld);

/* In-place transpose of a dense rectangular matrix: X holds rows x cols (leading dimension cols) on
 * entry and cols x rows (leading dimension rows) on exit, bit-exact, with no second buffer -- the
 * paper's way out when the memory for B^T is missing (Section III; future work in Section VI).  The
 * index permutation is factored into two or three passes that each permute within rows or within
 * columns (three when rows and cols share a factor), every pass a set of independent LDS-sized
 * problems; see csrc/transpose_inplace_rect.hip.  rows == cols takes the square kernel; a vector
 * (rows or cols == 1) is a no-op.  Limits: rows, cols <= 32768 (else MTNN_ERR_ARG). */
MTNN_API int mtnn_transpose_inplace_rect(void *stream, int rows, int cols, float *X);

/* TNN without a workspace: B is transposed in place, the NN product runs on it, and B is transposed
 * back; B is unchanged once the enqueued work has run, but it is WRITTEN in between, so nothing else
 * may read it concurrently and it must not overlap A (MTNN_ERR_ALIAS).  A square B (n == k) may have
 * any leading dimension; a rectangular B must be dense (ldb == k) and within the limits of
 * mtnn_transpose_inplace_rect, else MTNN_ERR_ARG (mtnn_tnn_inplace_supported tells beforehand). */
MTNN_API int mtnn_tnn_inplace(void *stream, int m, int n, int k,
                     const float *A, int lda, float *B, int ldb, float *C, int ldc);
MTNN_API int mtnn_tnn_inplace_supported(int n, int k, int ldb);

/* Bytes of workspace TNN needs for B^T (n*k floats, rounded up to 256 B); 0 if n or k <= 0. */
MTNN_API size_t mtnn_tnn_workspace_bytes(int n, int k);

/* TNN, Algorithm 1: transpose B into `workspace` (k x n, ld = n), then the NN operation.
 * Unlike the listing, the B^T buffer is the caller's: no allocation happens inside.
 * Returns MTNN_ERR_WORKSPACE if workspace is NULL or smaller than mtnn_tnn_workspace_bytes(n, k).
 * The workspace must not overlap A, B or C. */
MTNN_API int mtnn_tnn(void *stream, int m, int n, int k,
             const float *A, int lda, const float *B, int ldb, float *C, int ldc,
             void *workspace, size_t workspace_bytes);

/* MTNN, Algorithm 2: label = mtnn_select(m, n, k); +1 runs NT, -1 runs TNN.
 * Memory rule of Section II: when the workspace is NULL or too small, NT runs whatever the
 * predictor says.  `chosen` (may be NULL) receives +1 or -1 for the path actually run.
 * Environment: MTNN_FORCE=nt or MTNN_FORCE=tnn (read once per process) replaces the predictor's
 * answer, for experiments; the memory rule still applies. */
MTNN_API int mtnn_auto(void *stream, int m, int n, int k,
              const float *A, int lda, const float *B, int ldb, float *C, int ldc,
              void *workspace, size_t workspace_bytes, int *chosen);

/* The choice among three alternatives that Section VI leaves as future work: NT (+1), TNN with the
 * caller's workspace (-1), or TNN through in-place transposes of B (-2) when there is no room for
 * B^T.  mtnn_select3 is the rule: the predictor's label decides between NT and TNN as in Algorithm 2;
 * where it answers TNN but have_workspace is 0, the in-place path is taken only if can_inplace is set
 * and the kernels' cost model puts the NN product plus two in-place transposes below the NT product,
 * otherwise NT (the memory rule of Section II).  Returns 0 for non-positive sizes.
 * mtnn_auto3 runs the chosen path; mode 0 = the rule, +1 / -1 / -2 force a path (-1 needs the
 * workspace: MTNN_ERR_WORKSPACE; -2 needs mtnn_tnn_inplace_supported: MTNN_ERR_ARG).  B is not const:
 * the in-place path writes it on the way and restores it.  *chosen (may be NULL) receives the path. */
MTNN_API int mtnn_select3(int m, int n, int k, int have_workspace, int can_inplace);
MTNN_API int mtnn_auto3(void *stream, int mode, int m, int n, int k,
               const float *A, int lda, float *B, int ldb, float *C, int ldc,
               void *workspace, size_t workspace_bytes, int *chosen);

/* ---- selection (Section IV) ----------------------------------------------------------- */

/* Predicted label for the NT operation of shape (m, n, k): +1 = NT, -1 = TNN; 0 if any of
 * m, n, k is <= 0.  Host only, pure, O(trees x depth).  The feature vector is
 * (m, n, k, n*k, m*n, m*k, m*n*k); the margin is the sum of the leaf values reached in each
 * tree (a node sends x left when x[feature] < threshold) and the label is +1 when the margin
 * is >= 0.  With no model loaded the answer is +1 (NT needs no extra memory).  If the environment
 * variable MTNN_MODEL names a readable model file and no model has been installed yet, the first
 * call loads it. */
MTNN_API int mtnn_select(int m, int n, int k);

/* mtnn_select over `count` (m, n, k) triples (HOST arrays; labels[i] as mtnn_select would return,
 * evaluated without the memo). */
MTNN_API int mtnn_select_batch(int count, const int *mnk, int *labels);

/* Number of features mtnn_select builds (7) and, into x[0..6], the features themselves. */
MTNN_API int mtnn_num_features(void);
MTNN_API int mtnn_features(int m, int n, int k, double *x);

/* Load a model file and make it the current predictor.  On failure the current predictor is
 * unchanged and MTNN_ERR_MODEL is returned.  mtnn_unload_model() returns to "always NT". */
MTNN_API int mtnn_load_model(const char *path);
MTNN_API int mtnn_save_model(const char *path);
MTNN_API void mtnn_unload_model(void);

/* Fit boosted regression trees on (X, labels) with the settings of Section IV-B and make the
 * result the current predictor: logistic loss on y = (label == +1), exact greedy CART splits,
 * `num_trees` rounds, depth <= max_depth, step eta, minimum loss reduction gamma, leaf penalty
 * lambda, minimum child hessian weight min_child_weight.  X is nrows x nfeat row-major HOST
 * doubles; labels are +1 / -1.  The paper's configuration is (8, 8, 1.0, 0.0) with the
 * library defaults lambda = 1, min_child_weight = 1. */
MTNN_API int mtnn_gbdt_train(int nrows, int nfeat, const double *X, const int *labels,
                    int num_trees, int max_depth, double eta, double gamma,
                    double lambda, double min_child_weight);

/* Convenience for the selector itself: rows are (m, n, k) triples, features built internally,
 * paper settings. */
MTNN_API int mtnn_train_selector(int nrows, const int *mnk, const int *labels);

/* Inspection of the current predictor (for tests and reports). */
MTNN_API int mtnn_model_num_trees(void);
MTNN_API int mtnn_model_num_features(void);
MTNN_API int mtnn_model_tree_size(int tree);                       /* nodes, or -1 */
/* node `idx` of `tree`, pre-order; feature = -1 for a leaf. */
MTNN_API int mtnn_model_node(int tree, int idx, int *feature, double *threshold,
                    int *left, int *right, double *value);
/* margin of an arbitrary feature vector under the current predictor */
MTNN_API int mtnn_model_margin(const double *x, int nfeat, double *margin);

/* ---- tile configurations (tuning, tests) -------------------------------------------------- */

/* The GEMM kernels come in several tile configurations, optionally with the k range split over
 * several workgroups per C tile (partial products summed in a fixed order by a second kernel);
 * mtnn_nt / mtnn_nn choose both per shape with a fixed cost model.  These calls run a given
 * configuration (cfg in [0, count), or -1 for the model's choice) and split count (1..32, or 0 for
 * the model's choice when cfg is -1 and no split when cfg is given).  op: 0 = NN, 1 = NT.
 * A configuration's name reads BMxBNxBK_wMxN[k2]_dmaS_xP: the C tile, the k slab, M x N waves per
 * workgroup ("k2": two such sets of waves on the same tile, each on half of every slab's k range),
 * S slab buffers, at most P workgroups per CU.
 *
 * Scratch.  A split launch keeps its partial products (m x n x splits floats) in scratch memory that
 * the CALLER owns and registers per stream: mtnn_set_scratch(stream, ptr, bytes) lends the library
 * `bytes` of device memory at `ptr` (256-byte aligned) for every later launch on that stream of the
 * current device, until it is replaced or withdrawn (ptr = NULL, bytes = 0); the memory must stay
 * valid while such launches are in flight, and launches on other streams must get other memory.  The
 * cost model only considers divisions whose partials fit what is registered (nothing registered:
 * unsplit launches only), so a call's result depends on the registered capacity and not on when or
 * where it is issued; an EXPLICIT split count (or even cut) that does not fit returns
 * MTNN_ERR_WORKSPACE.  mtnn_scratch_bytes_default() is the capacity the cost model was tuned with
 * (64 MiB) and the one mtnn_gemm_default_config / _splits assume; mtnn_gemm_scratch_bytes is what a
 * given (cfg, splits) launch needs (0 for an unsplit one or invalid arguments).
 *
 * splits = MTNN_GEMM_EVEN_CUT asks for the third way of dividing the work: the k ranges of all C
 * tiles, in units of 64, are laid in one line and cut into (CUs x workgroups per CU) equal pieces,
 * one per workgroup; tiles that a cut goes through are finished by a fix-up kernel that adds their
 * pieces in k order (same scratch, same reproducibility).  It runs only where the pipelined
 * kernel can (16-byte aligned operands, k % 4 = 0, ...) and there are at least as many units as
 * pieces; otherwise the call runs unsplit.  mtnn_gemm_default_splits may return it. */
#define MTNN_GEMM_EVEN_CUT (-2)
MTNN_API int mtnn_gemm_config_count(void);
MTNN_API const char *mtnn_gemm_config_name(int cfg);
MTNN_API int mtnn_gemm_default_config(int op, int m, int n, int k);
MTNN_API int mtnn_gemm_default_splits(int op, int m, int n, int k);
MTNN_API int mtnn_gemm_ex(void *stream, int op, int cfg, int splits, int m, int n, int k,
                 const float *A, int lda, const float *B, int ldb, float *C, int ldc);
/* mtnn_gemm_ex for callers that cannot allocate device memory and have none to lend: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments, validation,
 * kernels and results are those of mtnn_gemm_ex on a stream with MTNN_STATIC_SCRATCH_BYTES lent, but
 * the partial products of a divided launch live in an array inside the library's code object (one
 * copy per GPU, held until the process ends) and whatever mtnn_set_scratch registered is ignored.
 * The call allocates and frees nothing.  An explicit split count or even cut whose partials need
 * more than MTNN_STATIC_SCRATCH_BYTES returns MTNN_ERR_WORKSPACE and launches nothing (ask
 * mtnn_gemm_scratch_bytes beforehand); with cfg = -1 and splits = 0 the rule only considers what
 * fits.  All calls on one GPU share that GPU's array -- on every stream -- so two such calls that
 * overlap in time race on it: issue them on one stream, or order them yourself.  The first call on
 * a device asks the runtime for the array's address there (no stream operation, no allocation). */
#define MTNN_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
MTNN_API int mtnn_gemm_ex_static(void *stream, int op, int cfg, int splits, int m, int n, int k,
                        const float *A, int lda, const float *B, int ldb, float *C, int ldc);
MTNN_API int mtnn_set_scratch(void *stream, void *scratch, size_t bytes);
MTNN_API size_t mtnn_get_scratch_bytes(void *stream);      /* registered for (current device, stream); 0 if none */
MTNN_API size_t mtnn_scratch_bytes_default(void);
MTNN_API size_t mtnn_gemm_scratch_bytes(int cfg, int splits, int m, int n, int k);
/* What mtnn_nt (op 1) / mtnn_nn (op 0) choose for 16-byte aligned operands of this shape on a stream
 * with `scratch_bytes` registered: *cfg the configuration, *splits 1..32 or MTNN_GEMM_EVEN_CUT. */
MTNN_API int mtnn_gemm_choice(int op, int m, int n, int k, size_t scratch_bytes, int *cfg, int *splits);
/* How many launches of this process took the even-cut path (diagnostics, tests). */
MTNN_API long long mtnn_gemm_even_cut_launches(void);
/* How many products of this process ran with a fused epilogue (mtnn_fc_layer_forward,
 * mtnn_fc_weight_grad_sgd) rather than with the separate pass (diagnostics, tests). */
MTNN_API long long mtnn_gemm_fused_epilogue_launches(void);
/* enable = 0: mtnn_fc_layer_forward / mtnn_fc_weight_grad_sgd (and the training step built on them)
 * run the plain product followed by the separate pass everywhere, for before / after measurements in
 * one process; 1 (the default): fuse where possible.  Returns the previous setting.  Process-wide. */
MTNN_API int mtnn_set_fused_epilogues(int enable);

/* ---- one training step of a fully connected net (Section V-C, Table IX sizes) ---------------- */

/* The paper evaluates MTNN inside fully connected nets given only by their layer sizes: the forward
 * product of a layer (mini-batch of activations, mb x l1, times the transpose of the l2 x l1
 * weights) is an NT operation; the backward products are NN operations.  The rest of the step is
 * this library's reading (the paper is silent): bias on every layer, ReLU after every hidden layer,
 * softmax cross-entropy averaged over the mini-batch, plain SGD.  All buffers are device fp32
 * (labels: device int32), dense (ld = width), owned by the caller. */
typedef struct mtnn_fc_step_desc {
    int num_layers;          /* L >= 1 weight layers                                              */
    const int *dims;         /* HOST array of L+1 widths: input, hidden..., output                */
    int batch;               /* mini-batch size                                                   */
    const float *X;          /* batch x dims[0]                                                   */
    const int *labels;       /* batch class indices in [0, dims[L])                               */
    float *const *W;         /* HOST array of L device pointers, W[l]: dims[l+1] x dims[l]; updated in place */
    float *const *b;         /* HOST array of L device pointers, b[l]: dims[l+1]; updated in place */
    float *const *dW;        /* HOST array of L device pointers: gradients w.r.t. W[l] (outputs)  */
    float *const *db;        /* HOST array of L device pointers: gradients w.r.t. b[l] (outputs)  */
    float *logits;           /* optional output, batch x dims[L] (may be NULL)                    */
    float *loss;             /* output, 1 float: mean cross-entropy                               */
    void *workspace;         /* at least mtnn_fc_workspace_bytes(...)                             */
    size_t workspace_bytes;
    float lr;                /* SGD step                                                          */
    int forward_mode;        /* 0 = mtnn_auto (Algorithm 2), +1 = always NT, -1 = always TNN      */
} mtnn_fc_step_desc;

MTNN_API size_t mtnn_fc_workspace_bytes(int num_layers, const int *dims, int batch);
/* forward (NT per layer via the selected path) -> loss -> backward (dW = transpose + NN, dX = NN)
 * -> SGD update, all enqueued on `stream`. */
MTNN_API int mtnn_fc_train_step(void *stream, const mtnn_fc_step_desc *desc);
/* The forward half alone: activations, logits (if requested) and the loss (its gradient w.r.t. the
 * logits is left in the workspace); W, b, dW, db are not written and dW / db may be NULL.  Used to
 * split a step's time into forward and backward as in the paper's Table X. */
MTNN_API int mtnn_fc_forward(void *stream, const mtnn_fc_step_desc *desc);

/* The elementwise / reduction steps of the training step, exported for tests:
 * Z[i][j] += b[j] (then ReLU if relu != 0), in place, Z batch x width dense. */
MTNN_API int mtnn_fc_bias_act(void *stream, int batch, int width, float *Z, const float *b, int relu);
/* dZ = (softmax(logits) - onehot(labels)) / batch; row_loss[i] = -log softmax(logits_i)[label_i];
 * mean_loss[0] = mean of row_loss. */
MTNN_API int mtnn_fc_softmax_xent(void *stream, int batch, int classes, const float *logits, const int *labels,
                         float *dZ, float *row_loss, float *mean_loss);
/* dH[e] = H[e] > 0 ? dH[e] : 0 over `count` elements (H is the ReLU output). */
MTNN_API int mtnn_fc_relu_backward(void *stream, long long count, float *dH, const float *H);
/* db[j] = sum_i dZ[i][j], dZ batch x width dense.  scratch: optional 32 x width floats; with it the
 * rows are summed in up to 32 chunks by many workgroups and the chunks added in order (NULL: one
 * workgroup per 64 columns walks all rows).  Either way the order is fixed. */
MTNN_API int mtnn_fc_bias_grad(void *stream, int batch, int width, const float *dZ, float *db, float *scratch);
/* Both of the above in one pass over the gradient: dH = (H > 0 ? dH : 0) in place, then
 * db[j] = sum_i dH[i][j]; dH and H batch x width dense, scratch as for mtnn_fc_bias_grad. */
MTNN_API int mtnn_fc_relu_backward_bias_grad(void *stream, int batch, int width, float *dH, const float *H,
                                    float *db, float *scratch);
/* P[e] = fma(-lr, G[e], P[e]) over `count` elements. */
MTNN_API int mtnn_fc_sgd(void *stream, long long count, float *P, const float *G, float lr);

/* The two products of a layer with the elementwise step that follows them done in the product's
 * epilogue, so that the result makes one trip to memory instead of three (Section V-C: the forward
 * product of a layer is the NT operation, the weight gradient an NN operation; bias, ReLU and SGD are
 * this library's reading, as above).  Both give, bit for bit, what the separate calls give.
 *
 * mtnn_fc_layer_forward: Y = act(X x W^T + b), X m x k (mini-batch x inputs), W n x k, b n values,
 * Y m x n; relu = 1 clamps at zero, 0 does not.  mode: +1 the NT kernel, -1 TNN (Algorithm 1; needs
 * the workspace of mtnn_tnn), 0 the predictor's choice exactly as in mtnn_auto (Algorithm 2); the
 * path taken (+1 / -1) is stored in *chosen if it is non-NULL.  Arguments and errors as for
 * mtnn_nt / mtnn_tnn; b must not overlap Y (MTNN_ERR_ALIAS).
 *
 * mtnn_fc_weight_grad_sgd: dW = A x B (NN: A m x k, B k x n, dW m x n) and W = fma(-lr, dW, W) for the
 * m x n matrix W, which must not overlap A, B or dW.  In a layer: A = the transposed output
 * gradient (outputs x mini-batch), B = the layer's input activations.
 *
 * The epilogue is fused where the pipelined kernel runs (16-byte aligned operands, k % 4 = 0; for
 * the forward product also in the reduction kernel of a split-k launch); elsewhere the call runs the
 * plain product followed by the separate pass, with the same results. */
MTNN_API int mtnn_fc_layer_forward(void *stream, int mode, int m, int n, int k, const float *X, int ldx,
                          const float *W, int ldw, const float *b, int relu, float *Y, int ldy,
                          void *workspace, size_t workspace_bytes, int *chosen);
MTNN_API int mtnn_fc_weight_grad_sgd(void *stream, int m, int n, int k, const float *A, int lda,
                            const float *B, int ldb, float *dW, int lddw, float *W, int ldw, float lr);
/* dense device-to-device copy of a rows x cols matrix */
MTNN_API int mtnn_copy_rows(void *stream, int rows, int cols, const float *in, float *out);

/* ---- measurement aid ------------------------------------------------------------------------ */

/* Plain device-to-device streaming copy of `bytes` (a multiple of 16, both pointers 16-byte
 * aligned, ranges disjoint).  Not part of the paper's method: it is the known-traffic kernel
 * that hardware byte counters are scaled against, and the practical ceiling a read-once /
 * write-once kernel such as the transpose can be compared with. */
MTNN_API int mtnn_copy_bytes(void *stream, size_t bytes, const void *in, void *out);

/* One workgroup per compute unit, two waves per SIMD: one issues n_mfma fp32 matrix instructions,
 * the other n_valu fp32 vector multiply-adds (either count may be 0); `sink` is 512 floats of device
 * memory that are never written in practice.  Timing the three combinations shows whether the two
 * kinds of work overlap on this device (they do not: see csrc/probe.hip), which is what the kernels'
 * instruction budget around the k loop rests on. */
MTNN_API int mtnn_probe_lanes(void *stream, int n_mfma, int n_valu, float *sink);

/* ---- misc ---------------------------------------------------------------------------------- */

MTNN_API const char *mtnn_status_string(int status);
/* The hipError_t behind the most recent MTNN_ERR_LAUNCH in this process (0 if none); diagnostics. */
MTNN_API int mtnn_last_hip_error(void);
MTNN_API int mtnn_version(void);
/* 1 if `arch` (the architecture name the HIP runtime reports for a device, e.g.
 * "gfx950:sramecc+:xnack-") is the one the kernels are built for, else 0.  Every call that launches
 * a kernel applies this test to the current device and returns MTNN_ERR_NO_DEVICE when it fails. */
MTNN_API int mtnn_arch_supported(const char *arch);
/* A property of the current device, for reports: what = 0 compute units, 1 peak shader clock in kHz,
 * 2 peak memory clock in kHz, 3 memory bus width in bits.  Returns -1 if it cannot be read (no device,
 * unknown `what`). */
MTNN_API int mtnn_device_attribute(int what);

#ifdef __cplusplus
}
#endif
#endif /* MTNN_H */
