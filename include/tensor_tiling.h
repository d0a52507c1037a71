/* tensor_tiling.h - C ABI of the MI355X tensor-tiling execution library.
 *
 * Executes a chain of fully-connected / convolution layers under a k-cut tensor
 * tiling (arXiv 1805.04170): every tensor is cut k times, each cut splitting its
 * rows (R), its columns (C) or replicating it (r), giving 2^k shards that live
 * as 2^k separate buffers in one GPU's memory.
 *
 * Conventions (all entry points)
 *  - cut 0 is the first (outermost) cut.  Shard s in [0, 2^k) takes side
 *    ((s >> (k-1-j)) & 1) at cut j.  By the flattening theorem (Sec. 4.4) the shards
 *    of a rows x cols tensor form a grid of 2^kR row blocks x 2^kC column blocks;
 *    shard s holds row block = its side bits at the R cuts read outermost-first,
 *    column block likewise from the C cuts; bits at r cuts select a replica.
 *  - a shard buffer is dense row-major: (rows / 2^kR) x (cols / 2^kC), leading
 *    dimension = its column count.
 *  - "dev ptrs": a HOST array of 2^k DEVICE pointers, one per shard, owned by the
 *    caller.  The library never allocates or frees device memory; scratch comes from
 *    the caller's workspace argument.  All device work is enqueued on the caller's
 *    HIP stream (hipStream_t passed as void*, NULL = default stream) and is
 *    asynchronous; the pointer arrays themselves may be freed as soon as a call returns.
 *  - every call returns a tt_status; nothing throws across the ABI.  Argument and
 *    feasibility errors are detected on the host before anything is launched.
 *    Only even cuts exist (Sec. 4.1): an extent that does not divide gives TT_EINFEASIBLE.
 *  - calls are re-entrant.  The library keeps no mutable state between calls except guarded, once-only set-up
 *    (which kernels have had their LDS limit raised; the address of tt_fc_forward_static's scratch array per device),
 *    and it reads no environment variable: every launch decision is a function of the call's arguments.
 */
#ifndef TENSOR_TILING_H
#define TENSOR_TILING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TT_OK = 0,
    TT_EINVAL = 1,        /* bad argument (NULL, k out of range, unknown letter, ...) */
    TT_EINFEASIBLE = 2,   /* an uneven cut, or no feasible tiling / form sequence */
    TT_EUNSUPPORTED = 3,  /* valid request outside what this build implements */
    TT_ENOMEM = 4,        /* host allocation failed */
    TT_EDEVICE = 5,       /* a HIP launch reported an error */
    TT_EWORKSPACE = 6     /* workspace missing, too small or misaligned */
} tt_status;

enum { TT_MAX_K = 6, TT_MAX_LAYERS = 16 };
enum { TT_R = 0 /* split dim 0: rows / batch / input channel */,
       TT_C = 1 /* split dim 1: columns / channel / output channel */,
       TT_REP = 2 /* replicate */ };
/* aligned forms of a product Z = X Y (Sec. 4.2.1):
 * F1: X:R Y:r -> Z:R (M split); F2: X:r Y:C -> Z:C (N split); F3: X:C Y:R -> Z:red (K split, partial sums) */
enum { TT_F1 = 0, TT_F2 = 1, TT_F3 = 2 };
enum { TT_F32 = 0, TT_BF16 = 1 };
enum { TT_ACT_NONE = 0, TT_ACT_RELU = 1 };
enum { TT_FC = 0, TT_CONV2D = 1 };
enum { TT_PLAN_EXACT = 0, TT_PLAN_RECURSIVE = 1 };
enum { TT_OP_FWD = 0, TT_OP_DGRAD = 1, TT_OP_WGRAD = 2 };
enum { TT_TENSOR_X = 0, TT_TENSOR_G = 1, TT_TENSOR_W = 2 };

typedef struct { uint8_t cut[TT_MAX_K]; } tt_tiling; /* cut[j] in {TT_R, TT_C, TT_REP}; entries >= k ignored */

/* One layer x_out = act(x_in * W).
 * FC:     x_in is batch x n_in, W is n_in x n_out (W[i][j] joins input neuron i to output neuron j, Sec. 2.1).
 * CONV2D: stride-1 cross-correlation with zero padding; n_in = input channels C, n_out = output channels K,
 *         input H x W, filter R x S, output P = H + 2 pad - R + 1, Q = W + 2 pad - S + 1.
 *         Storage: activations NHWC, i.e. the row-major matrix (N*H*W) x C; filters [K][R][S][C].
 *         Cuts: R splits the batch (activations) / the input channels (filters);
 *               C splits the channels (activations) / the output channels (filters);
 *         image and filter-tap dimensions are never cut (Sec. 4.5). */
typedef struct {
    int32_t kind; /* TT_FC | TT_CONV2D */
    int32_t act;  /* TT_ACT_* applied to this layer's output */
    int64_t n_in, n_out;
    int64_t H, W, R, S, pad; /* CONV2D only; ignored for FC */
} tt_layer;

const char *tt_strerror(tt_status);

/* ---------------------------------------------------------------- geometry */

/* Shard extent of a rows x cols tensor under a k-cut tiling (Def. 1, Sec. 4.1).
 * TT_EINFEASIBLE if rows (cols) is not divisible by 2^kR (2^kC). */
tt_status tt_shard_shape(int64_t rows, int64_t cols, tt_tiling t, int k, int64_t *srows, int64_t *scols);

/* ------------------------------------------------------------------ planner
 * Host only, exact integer arithmetic (costs in elements).
 * Graph of an L-layer chain (Sec. 4.2): activations x_0..x_L, their gradients g_0..g_L, weights W_1..W_L;
 * products per layer  F_l: x_l = x_{l-1} W_l,  B_l: g_{l-1} = g_l W_l^T,  G_l: dW_l = x_{l-1}^T g_l,
 * with dW_l stored in the tiling of W_l.  Cost of a product = Eq. 2 per cut (conversion cost = area needed
 * for the local product minus area already held, Sec. 4.2.1), the area at cut j being the stored tile left by
 * cuts 0..j-1, summed as sum_j 2^j delta_j (Theorem 1) and minimised over feasible form sequences.
 * Chains may mix layer kinds the way AlexNet and VGG do (Sec. 6): convolutions first, then fully-connected layers.
 *  - A convolution whose H x W is smaller than the P x Q of the convolution before it: a pooling (or striding) stage
 *    lies between them; it works per image and per channel, moves nothing under any tiling (element-wise functions,
 *    Eq. 1 / Sec. 4.5), and the tensor between the layers is charged at the size the later layer reads.
 *  - A fully-connected layer after a convolution with K output channels: n_in = K * pixels (pixels <= what the
 *    convolution or the pooling after it left) is the flattened image; a column cut of that tensor is a channel cut.
 *  - Convolution after fully-connected: TT_EUNSUPPORTED.  Dimension mismatches: TT_EINVAL. */

typedef struct tt_plan tt_plan; /* opaque, host memory, freed by tt_plan_free */

/* Minimum-communication k-cut tiling of a chain (Eq. 3; Algorithm 1).
 * mode TT_PLAN_EXACT: global minimum over all joint k-cut tilings (dynamic program over layers, Eqs. 4-5,
 *   with k-cut sequences as states); supported for k <= 4.
 * mode TT_PLAN_RECURSIVE: Algorithm 1 as printed: one-cut dynamic program (Eqs. 4-5), fix it, recurse on the
 *   tile graph; ties resolved to the lexicographically first assignment in tensor order x_0,g_0,W_1,x_1,g_1,...
 *   with R < C < r; each product's form = lowest-index minimiser.
 * pin_*: NULL leaves the boundary tensor free, else fixes its tiling.
 * Errors: TT_EINVAL, TT_EINFEASIBLE (no feasible tiling), TT_EUNSUPPORTED, TT_ENOMEM. */
tt_status tt_plan_chain(const tt_layer *layers, int n_layers, int64_t batch, int k, uint32_t mode,
                        const tt_tiling *pin_x0, const tt_tiling *pin_g0, const tt_tiling *pin_xL,
                        const tt_tiling *pin_gL, tt_plan **out);

/* Cost of a given graph tiling: x[0..L], g[0..L], w[0..L-1] (w[l-1] tiles W_l).
 * delta_out (k entries, may be NULL) per-cut costs; forms_out (3*L*k entries, may be NULL): for layer l (0-based),
 * op in {FWD, DGRAD, WGRAD}, cut j at [(l*3 + op)*k + j], the first minimising form sequence. */
tt_status tt_plan_eval(const tt_layer *layers, int n_layers, int64_t batch, int k, const tt_tiling *x,
                       const tt_tiling *g, const tt_tiling *w, uint64_t *cost_elems, uint64_t *delta_out,
                       uint8_t *forms_out);

int tt_plan_k(const tt_plan *);
int tt_plan_layers(const tt_plan *);
uint64_t tt_plan_cost(const tt_plan *);          /* total, elements */
uint64_t tt_plan_delta(const tt_plan *, int cut); /* per-cut cost delta_j */
/* which = TT_TENSOR_X / _G (index 0..L) or TT_TENSOR_W (index 1..L) */
tt_status tt_plan_tiling(const tt_plan *, int which, int index, tt_tiling *out);
/* form sequence (k entries) of product op of layer (1..L) */
tt_status tt_plan_forms(const tt_plan *, int layer, int op, uint8_t *forms_out);
void tt_plan_free(tt_plan *);

/* ------------------------------------------------------------- conversions */

/* Tiling conversion A -> B of a rows x cols tensor (Sec. 5.2 step 1: slice, fetch, concatenate; on one GPU a
 * single gather-copy over the tile grid).  dst / src: 2^k dev ptrs.  elem_bytes in {1,2,4,8}.  Bit-exact.
 * src and dst buffers must not overlap.  Replicas in A are assumed identical (any one may be read). */
tt_status tt_retile(void *const *dst, tt_tiling B, const void *const *src, tt_tiling A, int k, int64_t rows,
                    int64_t cols, int elem_bytes, void *stream);

/* Element-wise gradient gate fused into a conversion (Sec. 2.1: df applied to the incoming gradient):
 * dst[B] = src[A] where mask[Am] > 0, else 0.  src and mask are rows x cols tensors of dtype (TT_F32 | TT_BF16)
 * under their own tilings; mask may be NULL (plain conversion). */
tt_status tt_retile_gate(void *const *dst, tt_tiling B, const void *const *src, tt_tiling A,
                         const void *const *mask, tt_tiling Am, int k, int64_t rows, int64_t cols, int dtype,
                         void *stream);

/* Tiling conversion between a convolution's and a fully-connected layer's view of the same [batch][channels][pixels]
 * tensor (Sec. 4.5: convolution tensors are cut along batch and channel only; Sec. 5.2 step 1).  Image side: per
 * shard a row-major (images * pixels) x channels matrix, the storage of tt_conv_*.  Matrix side: per shard a
 * row-major images x (channels * pixels) matrix with channel-major columns, so that a column cut (TT_C) is a channel
 * cut on both sides; TT_R cuts the batch on both sides.  to_matrix != 0: src is the image side under A, dst the matrix
 * side under B (the flatten in front of the first fully-connected layer); to_matrix == 0: src is the matrix side
 * under A, dst the image side under B (its gradient on the way back).  dst / src: 2^k dev ptrs.  elem_bytes in {2,4}.
 * Bit-exact; src and dst must not overlap; replicas in A are assumed identical; every replica in B is written.
 * Errors: TT_EINVAL, TT_EINFEASIBLE (batch or channels not divisible as a tiling asks), TT_EUNSUPPORTED (batch above
 * 65535, or batch * pixels >= 2^32). */
tt_status tt_flatten(void *const *dst, tt_tiling B, const void *const *src, tt_tiling A, int k, int64_t batch,
                     int64_t channels, int64_t pixels, int elem_bytes, int to_matrix, void *stream);

/* Reduction of the partial sums left by F3 cuts, fused with the output conversion (Sec. 4.2.1 "extra reduction";
 * Sec. 5.2 step 3).  partials: 2^k dev ptrs to fp32 buffers; shard s holds the (rows / 2^k1) x (cols / 2^k2)
 * block selected by its side bits at the F1 cuts (row block) and F2 cuts (column block); its bits at the F3
 * cuts number the partial sum.  Z = sum of partials in increasing partial number (fixed order, fp32), then act,
 * then conversion to out_dtype (TT_F32 | TT_BF16, round to nearest even) and scatter into the 2^k dst shards of
 * tiling B (replicas written once each).  forms: k entries.  Also valid with no F3 cut (cast + conversion). */
tt_status tt_reduce(void *const *dst, tt_tiling B, int out_dtype, const float *const *partials,
                    const uint8_t *forms, int k, int64_t rows, int64_t cols, int act, void *stream);

/* ---------------------------------------------- what an execution really moves
 * Elements that cross from one shard to another (Sec. 4.2.1: a device fetches the part of its tile under the new tiling
 * that it does not hold under the old one; with the third aligned form it fetches the other devices' partial sums of the
 * elements it is to store).  Counted block by block over the 2^k shards; host arithmetic, no device work.
 * For k = 1 the count of a product equals its cost under tt_plan_eval; for k > 1 the planner's cost is the paper's
 * recursive model and the two differ - callers report them side by side.
 * tt_conversion_cross_elems: a stored tensor of rows x cols going from tiling `from` to tiling `to`.
 * tt_product_cross_elems: Z = X Y (M x K times K x N) under stored tilings tX, tY, tZ and a form sequence (k entries,
 *   TT_F1..TT_F3): elems[0] input conversion of X, elems[1] of Y, elems[2] output conversion or partial-sum reduction.
 *   mult_*: elements per matrix entry (1 for fully-connected layers; pixels per channel entry / filter taps for
 *   convolutions, whose image and filter extents are never cut).
 * Errors: TT_EINVAL, TT_EINFEASIBLE (uneven cut, or M, N, K not divisible as the forms ask). */
tt_status tt_conversion_cross_elems(int64_t rows, int64_t cols, tt_tiling from, tt_tiling to, int k, uint64_t *elems);
tt_status tt_product_cross_elems(int64_t M, int64_t K, int64_t N, tt_tiling tX, tt_tiling tY, tt_tiling tZ,
                                 const uint8_t *forms, int k, uint64_t mult_x, uint64_t mult_y, uint64_t mult_z,
                                 uint64_t *elems /* [3] */);
/* one forward + backward pass over a chain of fully-connected layers (TT_EUNSUPPORTED for other kinds): the sum over its
 * 3 L products.  Tilings as tt_plan_eval takes them (x, g: L + 1; w: L); forms: 3 * L * k entries laid out as
 * tt_plan_eval's forms_out (layer, then forward / data gradient / weight gradient, then cut). */
tt_status tt_fc_chain_cross_elems(const tt_layer *layers, int n_layers, int64_t batch, int k, const tt_tiling *x,
                                  const tt_tiling *g, const tt_tiling *w, const uint8_t *forms, uint64_t *elems);

/* ------------------------------------------------- planner, general graphs
 * The tiling search on any dataflow graph (Sec. 4.2.2: operators organised into breadth-first levels, Eqs. 4-5 over
 * the tensors shared by adjacent levels; Sec. 4.3: Algorithm 1; Sec. 4.5: tensors with up to four dimensions - one
 * basic tiling per dimension plus replication - and operators other than products).  Host only.
 * A letter is a dimension index (the cut that halves it) or TT_LETTER_REP; a k-cut tiling is k letters, cut 0 first.
 * Cost model and readings as for tt_plan_chain (letters R and C there are dimensions 0 and 1 here).
 *   tensor: ndim, shape, same_as = index of an EARLIER tensor of the same shape whose tiling it shares (a weight
 *           gradient is stored like its weight), or -1.
 *   operator kinds and their aligned forms:
 *     TT_GOP_CONTRACT     z = x (.) y, in = {x, y}; m = {dim of x, dim of z} kept from x, n = {dim of y, dim of z} kept
 *                         from y, kk = {dim of x, dim of y} contracted.  Form 0: x cut along m, y replicated, z cut
 *                         along m;  1: x replicated, y cut along n, z cut along n;  2: both cut along kk, z partial sums.
 *                         x.y: m {0,0} n {1,1} kk {1,0};  x.y^T: n {0,1} kk {1,1};  x^T.y: m {1,0} kk {0,0};
 *                         convolution X[N,C,H,W] * W[K,C,R,S] -> Y[N,K,P,Q]: m {0,0} n {0,1} kk {1,1}.
 *     TT_GOP_ELEMENTWISE  1..4 inputs and the output of one shape; form d: every operand cut along dimension d.
 *     TT_GOP_BATCH        any other operator: every operand cut along dimension 0 (equal extents there).
 *     TT_GOP_SAMPLE_CHANNEL  operators that treat every (sample, channel) pair by itself: pooling, the flattening of
 *                         channel-major images [N,C,H,W] -> [N, C*H*W].  Operands need at least two dimensions, equal
 *                         extents in dimension 0, extents in dimension 1 that are multiples of the smallest one (the
 *                         channel count).  Form 0: all cut along dimension 0;  form 1: all cut along dimension 1.
 * pins: NULL, or n_tensors * k letters; a tensor whose first letter is TT_LETTER_FREE is left to the search.
 * mode TT_PLAN_EXACT: minimum over every joint assignment of k-cut sequences, found by minimising the tensors out
 * one at a time (TT_EUNSUPPORTED when every order would need a cost table of more than 2^24 entries);
 * TT_PLAN_RECURSIVE: Algorithm 1, each cut by the level-by-level dynamic program (cost = sum_j 2^j delta_j, forms
 * chosen cut by cut; TT_EUNSUPPORTED when a level has more than 2^28 joint one-cut states).
 * Errors: TT_EINVAL (malformed graph or letters), TT_EINFEASIBLE (no tiling with even cuts), TT_ENOMEM. */
enum { TT_GRAPH_MAX_DIMS = 4, TT_GRAPH_MAX_INPUTS = 4, TT_GRAPH_MAX_TENSORS = 4096, TT_GRAPH_MAX_OPS = 4096 };
enum { TT_LETTER_REP = 255, TT_LETTER_FREE = 253 };
enum { TT_GOP_CONTRACT = 0, TT_GOP_ELEMENTWISE = 1, TT_GOP_BATCH = 2, TT_GOP_SAMPLE_CHANNEL = 3 };
typedef struct { int32_t ndim; int32_t same_as; int64_t shape[4]; } tt_graph_tensor;
typedef struct { int32_t kind, n_in; int32_t in[4]; int32_t out; int32_t m[2], n[2], kk[2]; } tt_graph_op;
typedef struct tt_graph_plan tt_graph_plan; /* opaque; host memory owned by the library until tt_graph_plan_free */
tt_status tt_plan_graph(const tt_graph_tensor *tensors, int n_tensors, const tt_graph_op *ops, int n_ops, int k,
                        uint32_t mode, const uint8_t *pins, tt_graph_plan **out);
/* cost of given tilings (n_tensors * k letters; tensors stored alike must agree); delta_out (k) and forms_out
 * (n_ops * k, the cheapest feasible form sequence of every operator) may be NULL */
tt_status tt_graph_eval(const tt_graph_tensor *tensors, int n_tensors, const tt_graph_op *ops, int n_ops, int k,
                        const uint8_t *letters, uint64_t *cost_elems, uint64_t *delta_out, uint8_t *forms_out);
uint64_t tt_graph_plan_cost(const tt_graph_plan *p);
uint64_t tt_graph_plan_delta(const tt_graph_plan *p, int cut);
int tt_graph_plan_levels(const tt_graph_plan *p);              /* number of breadth-first levels */
int tt_graph_plan_level_of(const tt_graph_plan *p, int op);     /* level of an operator */
tt_status tt_graph_plan_tiling(const tt_graph_plan *p, int tensor, uint8_t *letters_out /* k */);
tt_status tt_graph_plan_forms(const tt_graph_plan *p, int op, uint8_t *forms_out /* k */);
void tt_graph_plan_free(tt_graph_plan *p);

/* --------------------------------------------------------- shard products */

/* 2^k (or any count of) independent products C_s = op(A_s) op(B_s) of identical shape in one launch
 * (Sec. 5.2 step 2: identical sub-operators).  Logical shapes: A is M x K, B is K x N, C is M x N row-major.
 * trans_a = 0: A stored M x K row-major;  1: stored K x M row-major (A = stored^T).
 * trans_b = 0: B stored K x N row-major;  1: stored N x K row-major.
 * in_dtype TT_BF16 (MFMA, fp32 accumulate) or TT_F32; out_dtype TT_BF16 | TT_F32; act applied before the store.
 * Buffers are dense (leading dimension = stored column count). */
tt_status tt_shard_gemm(int count, const void *const *A, const void *const *B, void *const *C, int64_t M,
                        int64_t N, int64_t K, int trans_a, int trans_b, int in_dtype, int out_dtype, int act,
                        void *stream);

/* ----------------------------------------------------------- layer execute
 * Three phases per product (Sec. 4.2.1, Sec. 5.2): convert inputs from their stored tilings to the aligned
 * tilings of the form sequence; run the 2^k identical shard products; convert (reduce, if any cut uses F3)
 * the temporary outputs to the stored output tiling.  forms: k entries per product, or NULL = the first
 * minimiser of the product's communication cost (as tt_plan_eval reports it).
 * dtype: TT_BF16 (bf16 storage, fp32 accumulate; partial sums fp32) or TT_F32.
 * workspace: device memory, 256-byte aligned, at least tt_*_workspace_bytes(...) bytes; may be NULL if 0. */

/* Exact workspace need of tt_fc_forward (op = TT_OP_FWD; tdY, tdX, forms_b ignored) or of tt_fc_backward
 * (op = TT_OP_DGRAD; forms_a = forms_dgrad, forms_b = forms_wgrad; with_dx = 0 if dX will be NULL) for the same
 * layer, tilings and forms (NULL forms = the same default as the execute call). */
tt_status tt_fc_workspace_bytes(const tt_layer *layer, int64_t batch, int k, int dtype, int op, tt_tiling tX,
                                tt_tiling tW, tt_tiling tY, tt_tiling tdY, tt_tiling tdX, const uint8_t *forms_a,
                                const uint8_t *forms_b, int with_dx, size_t *bytes);

/* Y = act(X W).  X: batch x n_in under tX;  W: n_in x n_out under tW;  Y: batch x n_out under tY. */
tt_status tt_fc_forward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                        tt_tiling tY, const uint8_t *forms, const void *const *X, const void *const *W,
                        void *const *Y, void *workspace, size_t ws_bytes, void *stream);

/* tt_fc_forward for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments, results and errors as tt_fc_forward; the
 * scratch comes from an array of TT_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the
 * library runs on holds its copy until the process ends).  The call allocates nothing and frees nothing.
 * TT_EWORKSPACE if the layer needs more scratch than that (tt_fc_workspace_bytes tells how much).  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads) race; the array keeps
 * the last call's contents and nothing in it needs clearing between calls. */
enum { TT_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024 };
tt_status tt_fc_forward_static(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                               tt_tiling tY, const uint8_t *forms, const void *const *X, const void *const *W,
                               void *const *Y, void *stream);

/* G = dY gated by [Y > 0] (act RELU) or dY;  dX = G W^T (under tdX);  dW = X^T G (under tW, dtype as W).
 * Y is the layer's stored output under tY (ignored when act is NONE; may then be NULL).
 * dX may be NULL to skip the activation gradient. */
tt_status tt_fc_backward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                         tt_tiling tY, tt_tiling tdY, tt_tiling tdX, const uint8_t *forms_dgrad,
                         const uint8_t *forms_wgrad, const void *const *X, const void *const *W,
                         const void *const *Y, const void *const *dY, void *const *dX, void *const *dW,
                         void *workspace, size_t ws_bytes, void *stream);

/* tt_fc_backward with the two products overlapped: the weight-gradient product (with its conversions) is enqueued
 * on aux_stream once G exists and runs beside the dX product on stream; the call makes aux_stream wait for stream's
 * earlier work and stream wait for the weight gradient before it returns, so callers keep ordering everything on
 * stream alone (and may capture stream into a HIP graph: aux_stream joins and leaves the capture inside the call).
 * Both streams must have default priority.  aux_stream NULL or equal to stream: same as tt_fc_backward.
 * The workspace need is that of tt_fc_backward (the two products never share scratch inside one call). */
tt_status tt_fc_backward_overlapped(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                                    tt_tiling tY, tt_tiling tdY, tt_tiling tdX, const uint8_t *forms_dgrad,
                                    const uint8_t *forms_wgrad, const void *const *X, const void *const *W,
                                    const void *const *Y, const void *const *dY, void *const *dX, void *const *dW,
                                    void *workspace, size_t ws_bytes, void *stream, void *aux_stream);

/* Convolution layer (layouts in tt_layer; the textbook stride-1 cross-correlation with zero padding, cut as Sec. 4.5
 * says: batch and channels only).  Supported cuts per product: F1 (batch), F2 (output channels for forward, input
 * channels for dgrad; out-channel / in-channel grid for wgrad), F3 (reduction split).  dtype TT_BF16: MFMA kernels,
 * channel counts per shard multiples of 8 and R * S <= 32 (else TT_EUNSUPPORTED).  dtype TT_F32: plain kernels that
 * follow the definition term by term, any channel count.  Arguments, ownership and errors as for tt_fc_*. */
tt_status tt_conv_workspace_bytes(const tt_layer *layer, int64_t batch, int k, int dtype, int op, tt_tiling tX,
                                  tt_tiling tW, tt_tiling tY, tt_tiling tdY, tt_tiling tdX, const uint8_t *forms_a,
                                  const uint8_t *forms_b, int with_dx, size_t *bytes);
tt_status tt_conv_forward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                          tt_tiling tY, const uint8_t *forms, const void *const *X, const void *const *W,
                          void *const *Y, void *workspace, size_t ws_bytes, void *stream);
tt_status tt_conv_backward(const tt_layer *layer, int64_t batch, int k, int dtype, tt_tiling tX, tt_tiling tW,
                           tt_tiling tY, tt_tiling tdY, tt_tiling tdX, const uint8_t *forms_dgrad,
                           const uint8_t *forms_wgrad, const void *const *X, const void *const *W,
                           const void *const *Y, const void *const *dY, void *const *dX, void *const *dW,
                           void *workspace, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------ kernel timing
 * Optional instrumentation for measurement (the counterpart of the paper's computation-only runs, Sec. 6.2: it
 * separates the time of the conversion / reduction kernels from the time of the shard products).
 * Between tt_profile_begin and tt_profile_end every kernel the calling thread launches through this library is
 * bracketed by a pair of HIP events on the launch stream.  tt_profile_end waits for the last event, fills the
 * records and disables recording.  Not to be used during stream capture.  The record list is per thread. */
enum { TT_K_CONVERT = 0, TT_K_GATE = 1, TT_K_REDUCE = 2, TT_K_GEMM_NN = 3, TT_K_GEMM_NT = 4, TT_K_GEMM_TN = 5,
       TT_K_GEMM_TT = 6, TT_K_GEMM_GENERIC = 7, TT_K_CONV_FWD = 8, TT_K_CONV_DGRAD = 9, TT_K_CONV_WGRAD = 10 };
typedef struct {
    int32_t kernel;      /* TT_K_* */
    int32_t count;       /* shards covered by the launch */
    int64_t d0, d1, d2;  /* products: M, N, K per shard; conversions / reductions: rows, cols, element bytes */
    uint64_t bytes;      /* algorithmic HBM bytes of the launch (operands read once + outputs written once) */
    uint64_t flops;      /* 2 M N K count for products, 0 otherwise */
    float ms;            /* elapsed between the two events */
} tt_kernel_record;
tt_status tt_profile_begin(void);
tt_status tt_profile_end(int *n_records);                 /* TT_EDEVICE if an event call fails */
tt_status tt_profile_get(int index, tt_kernel_record *out); /* valid until the next tt_profile_begin */

#ifdef __cplusplus
}
#endif
#endif /* TENSOR_TILING_H */
