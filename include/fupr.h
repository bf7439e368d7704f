/*
 * fupr - inference of a filter-pruned residual network whose non-parametric
 * operators have been folded into its convolutions, for AMD gfx950.
 *
 * The calls follow the paper's statement of the problem (Sec. IV-A): a
 * pre-trained model plus user options (what to fuse, how many filters to
 * prune) gives an optimised model, which is then run.
 *
 *   fupr_fold            batch norm as omega*x + lambda (Sec. IV-B-2, Eq. 3-5)
 *                        merged into the convolution before it (Sec. VI-B-3)
 *   fupr_xconv_fuse      aggressive fusion of a basic residual block: auxiliary and
 *                        padded convolutions concatenated to its two convolutions,
 *                        batch norms adjusted, the addition gone (Sec. IV-B-1, IV-B-2)
 *   fupr_select_filters  lowest-norm filters of a convolution (Sec. IV-C, Eq. 6)
 *   fupr_prune_count     how many filters a non-fused operator loses (Alg. 1)
 *   fupr_prune           removal of masked filters (Alg. 1, last step)
 *   fupr_pack            weights -> device layout
 *   fupr_conv_fused      convolution operator k x c x r x s (Sec. III, Sec. IV-B-1)
 *                        with bias, element-wise addition and ReLU in its epilogue
 *   fupr_proj_concat, fupr_conv_cat_fused   a projection shortcut accumulated in the accumulators of
 *                        its block's last convolution (Sec. IV-B-1, projection-shortcut recipe)
 *   fupr_conv_scatter_fused             a block's last convolution after its output filters were
 *                        pruned: the kept filters add into their channels of the block's
 *                        full-width output (Alg. 1 applied to every non-fused operator, Sec. V-A)
 *   fupr_maxpool, fupr_global_avgpool   the "Others" of Table II / Table VI
 *   fupr_conv_conv1x1_fused             two consecutive 1 x 1 convolutions (a bottleneck block's last,
 *                        the next block's first), the second from the first one's registers
 *   fupr_conv_maxpool_fused             Table II's ImageNet stem (7 x 7 convolution, stride 2, then
 *                        3 x 3 max pool, stride 2) in one kernel
 *   fupr_model_*, fupr_forward          a whole network (Table II) on one stream
 *
 * Conventions
 *   - Host calls (fold, select, prune, pack, model create) take HOST pointers.
 *     Device calls take DEVICE pointers, marked [dev] below.  The library never
 *     allocates, frees or copies device memory, creates no stream, and never
 *     synchronises a stream unless a call says so; device work is enqueued on
 *     the caller's stream (a hipStream_t passed as void*, NULL = the default
 *     stream) and, for fupr_forward only, on streams the caller has lent with
 *     fupr_model_set_side_streams.  Every device buffer is the caller's: packed
 *     parameters, the one-kernel schedule's table (fupr_model_table_*), the
 *     workspace.  The one exception is said where it is declared:
 *     fupr_forward_static works in a fixed device array inside the library.
 *   - Every call returns FUPR_OK (0) or a negative fupr_status.  On error no
 *     output buffer has been written and nothing has been launched.
 *   - Activations are NHWC.  A tensor of C channels has a channel stride
 *     c_stride >= C (elements between consecutive pixels) that is a multiple of
 *     8 for 16-bit types and of 4 for fp32; the lanes C..c_stride-1 of every
 *     pixel hold zeros (callers provide inputs that way, kernels write outputs
 *     that way).  Base pointers are 16-byte aligned.
 *   - Convolutions are cross-correlations with zero padding, square stride and
 *     padding; weights on the host are float32 in K x C x R x S order.
 *   - Calls are re-entrant and thread-safe.  Mutable state they share: (1) the
 *     tuning switches of fupr_tuning_set, process-wide, read at every launch;
 *     (2) a model's schedule, table and side streams, set by the
 *     fupr_model_set_* calls, which must not run concurrently with a forward
 *     pass of the same model; forward passes of one model that use its side
 *     streams are serialised with each other while they enqueue (they share the
 *     fork / join events); (3) the array fupr_forward_static works in.
 */
#ifndef FUPR_H
#define FUPR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t fupr_status;
enum {
  FUPR_OK = 0,
  FUPR_ERR_NULL = -1,       /* a required pointer is NULL                              */
  FUPR_ERR_SHAPE = -2,      /* sizes are non-positive or do not match each other       */
  FUPR_ERR_DTYPE = -3,      /* unknown dtype, or tensors of one call differ in dtype   */
  FUPR_ERR_MASK_EMPTY = -4, /* the mask keeps no filter                                */
  FUPR_ERR_BN_VAR = -5,     /* var + eps is not a positive finite number               */
  FUPR_ERR_WORKSPACE = -6,  /* workspace too small or misaligned                       */
  FUPR_ERR_ALIGN = -7,      /* pointer or channel stride violates the alignment rules  */
  FUPR_ERR_LAUNCH = -8,     /* the HIP runtime refused a launch, event or capture      */
  FUPR_ERR_ARG = -9,        /* any other invalid argument (flags, norm, counts, ids)   */
  FUPR_ERR_LIMIT = -10,     /* a size exceeds what the kernels index with 32 bits      */
  FUPR_ERR_BN_SCALE = -11   /* a batch-norm scale that must be inverted is zero        */
};
const char* fupr_status_str(fupr_status s); /* static string, never NULL */

typedef enum { FUPR_F32 = 0, FUPR_BF16 = 1, FUPR_F16 = 2 } fupr_dtype;

/* K filters, C input channels, R x S window, square stride and zero padding. */
typedef struct {
  int32_t K, C, R, S, stride, pad;
} fupr_conv_shape;

/* What fupr_fold merges / what the kernel epilogue applies.  FUPR_FUSE_SCATTER and
 * FUPR_FUSE_CAT are accepted in fupr_op_desc.epilogue only (see there). */
enum { FUPR_FUSE_BN = 1, FUPR_FUSE_RELU = 2, FUPR_FUSE_ADD = 4, FUPR_FUSE_SCATTER = 8, FUPR_FUSE_CAT = 16 };

/* In a channel-wise concatenation of two tensors (fupr_proj_concat, fupr_conv_cat_fused) the
 * second tensor's channels start at a multiple of this many channels: the kernels fetch
 * 64 channels of one pixel (one 128-byte line of a 16-bit tensor) per load and tensor. */
#define FUPR_CAT_ALIGN 64

/* ------------------------------------------------------------------ host -- */

/*
 * Batch norm merged into the preceding convolution (Sec. IV-B-2, Eq. 3-5;
 * Sec. VI-B-3).  With FUPR_FUSE_BN in fuse_flags:
 *     omega_k  = gamma_k / sqrt(var_k + eps)        lambda_k = beta_k - omega_k mean_k
 *     W_out[k] = omega_k W[k]                        b_out[k] = lambda_k + omega_k conv_bias[k]
 * computed in double, stored as float.  Without the flag W_out = W and
 * b_out = conv_bias.  conv_bias may be NULL (taken as zeros).  gamma, beta,
 * mean, var (K floats each) may be NULL only without FUPR_FUSE_BN.
 * W_out (K*C*R*S) and b_out (K) are caller-allocated and may alias W / conv_bias.
 * Errors: NULL, SHAPE, BN_VAR (var_k + eps <= 0 or not finite), ARG (unknown flag bits).
 */
fupr_status fupr_fold(const fupr_conv_shape* shape, const float* W, const float* conv_bias,
                      const float* gamma, const float* beta, const float* mean, const float* var,
                      float eps, uint32_t fuse_flags, float* W_out, float* b_out);

/* Batch-norm parameters of one operator (Sec. IV-B-2, Eq. 3-5): K floats each, host. */
typedef struct {
  const float* gamma;
  const float* beta;
  const float* mean;
  const float* var;
  float eps;
} fupr_bn;

/* The shortcut of a basic residual block (Table II). */
enum {
  FUPR_SHORTCUT_IDENTITY = 0,      /* y = F(x) + x                                            */
  FUPR_SHORTCUT_SUBSAMPLE_PAD = 1, /* x[:, ::stride, ::stride], zero channels up to conv2's K */
  FUPR_SHORTCUT_PROJECTION = 2     /* 1 x 1 convolution (stride of conv1) and its batch norm  */
};

/*
 * Aggressive operator fusion of a basic residual block (Sec. IV-B-1: the
 * basic-block recipe and the projection-shortcut recipe; batch norms per
 * Sec. IV-B-2).  The block
 *     h = relu(bn1(conv1(x)));  y = relu(bn2(conv2(h)) + shortcut(x))
 * with conv1 = k1 x c x r x s, conv2 = k2 x k1 x r x s (r, s odd, pad = r/2 = s/2,
 * conv2 of stride 1) becomes two dilated convolutions and no addition:
 *     [h ; x'] = relu(bn1'(conv1'(x)));  y = relu(bn2'(conv2'([h ; x'])))
 *   W1_out  (k1 + c) x c x r x s: conv1's filters, then the auxiliary convolution for
 *           channel-wise fusion: filter k1 + j has a single 1 at (channel j, centre tap),
 *           so its output is x at conv1's stride.
 *   bn1_out (k1 + c each): bn1, then the auxiliary batch norm omega = 1, lambda = 0
 *           (gamma = sqrt(1 + eps) rounded to float, beta = mean = 0, var = 1).
 *   W2_out  k2 x (k1 + c) x r x s: conv2's channels, then the auxiliary convolution for
 *           filter-wise fusion at the centre tap of channels k1 + j.  bn2 stays after the
 *           fused operator and would scale what these weights add, so they hold its
 *           inverse: 1 / omega2_k at j = k for FUPR_SHORTCUT_IDENTITY (needs c = k2,
 *           conv1 stride 1) and FUPR_SHORTCUT_SUBSAMPLE_PAD (c <= k2; rows k >= c stay
 *           zero); omega_p,k / omega2_k * Wp[k][j] for FUPR_SHORTCUT_PROJECTION (the
 *           1 x 1 convolution padded to r x s).
 *   beta2_out (k2): beta2, plus the projection's shift lambda_p,k for
 *           FUPR_SHORTCUT_PROJECTION; gamma, mean, var of bn2 are unchanged.
 * The copy of x passes through the block's first ReLU: the rewrite is exact for
 * block inputs that are themselves outputs of a ReLU.  All values are computed
 * in double and stored as float.  proj, Wp, bnp are read only for
 * FUPR_SHORTCUT_PROJECTION (proj = k2 x c x 1 x 1, pad 0, conv1's stride).
 * Outputs are caller-allocated and must not alias inputs.
 * Errors: NULL, SHAPE (sizes that do not fit the recipe), ARG (unknown shortcut),
 * BN_VAR, BN_SCALE (omega2_k = 0: the batch norm after conv2 cannot be inverted).
 */
typedef struct {
  float* gamma;
  float* beta;
  float* mean;
  float* var;
} fupr_bn_out;
fupr_status fupr_xconv_fuse(const fupr_conv_shape* conv1, const float* W1, const fupr_bn* bn1,
                            const fupr_conv_shape* conv2, const float* W2, const fupr_bn* bn2,
                            int32_t shortcut, const fupr_conv_shape* proj, const float* Wp,
                            const fupr_bn* bnp, float* W1_out, const fupr_bn_out* bn1_out,
                            float* W2_out, float* beta2_out);

/*
 * A projection shortcut accumulated in the accumulators of its block's last
 * convolution (Sec. IV-B-1, the projection-shortcut recipe, fused along the C
 * dimension): for a block that ends in a 1 x 1 convolution of h with weights W
 * and whose shortcut is a 1 x 1 convolution of the block input x with weights Wp,
 *     conv(h, W) + conv_p(x, Wp) = conv([h ; x], [W | Wp]),
 * so the addition disappears into one convolution over the concatenated
 * channels.  (The paper pads the 1 x 1 shortcut to the 3 x 3 of a basic block's
 * last convolution; a bottleneck block's last convolution is 1 x 1 already.)
 * Both batch norms have been merged beforehand (fupr_fold).  Writes
 *     W_out   K x (C1p + C2) x 1 x 1: W's C1 channels, zeros up to C1p = C1 rounded
 *             up to FUPR_CAT_ALIGN, then Wp's C2 channels;
 *     b_out   K: b + bp (one fp32 addition each; NULL inputs count as zeros);
 *     *out    the shape of the concatenated operator: K, C1p + C2, 1 x 1, stride 1, pad 0.
 * The device never builds [h ; x]: fupr_conv_cat_fused reads the first C1p
 * channels from h and the others from x at the shortcut's stride.
 * last, proj: 1 x 1, pad 0, equal K; last->stride = 1.  Outputs are
 * caller-allocated and must not alias inputs.  Errors: NULL, SHAPE.
 */
fupr_status fupr_proj_concat(const fupr_conv_shape* last, const float* W, const float* b,
                             const fupr_conv_shape* proj, const float* Wp, const float* bp,
                             fupr_conv_shape* out, float* W_out, float* b_out);

/*
 * Number of filters a non-fused operator with n filters loses at pruning rate
 * permille/1000: floor(n * permille / 1000) in integer arithmetic, capped at
 * n - 1 so that one filter always stays (Alg. 1).  Returns a negative status
 * for n <= 0 or permille outside 0..1000.  (A FUSED operator with n filters, m
 * of them original, loses n - m instead: pass that count to fupr_select_filters.)
 */
int32_t fupr_prune_count(int32_t n, int32_t permille);

/*
 * Filter importance (Sec. IV-C, Eq. 6): mask_out[k] = 0 for the n_prune filters
 * of smallest l1 (norm = 1) or l2 (norm = 2) norm over their C*R*S weights,
 * 1 for the others.  Norms are summed in double in (c, r, s) order; among
 * equal norms the lower filter index is pruned first.  0 <= n_prune < K.
 */
fupr_status fupr_select_filters(const fupr_conv_shape* shape, const float* W, int32_t norm,
                                int32_t n_prune, uint8_t* mask_out);

/*
 * Removal of masked filters (Alg. 1, last step).  mask has prod->K entries of
 * 0/1.  Writes *K_keep, keep_idx[0..K_keep) (ascending filter indices kept),
 * the producer's kept filters Wp_out (K_keep x C x R x S) and bias bp_out
 * (K_keep; bp may be NULL, then bp_out may be NULL), and for each of the
 * n_consumers convolutions that read the producer's output, its weights with
 * the removed input channels dropped, Wc_out[i] (cons[i].K x K_keep x R x S).
 * cons[i].C must equal prod->K.  All copies are exact.  Outputs are
 * caller-allocated (sizing them for K_keep = prod->K is always enough) and must
 * not alias inputs.
 * Errors: NULL, SHAPE, MASK_EMPTY, ARG (mask entry not 0/1, n_consumers < 0).
 */
fupr_status fupr_prune(const fupr_conv_shape* prod, const float* Wp, const float* bp,
                       const uint8_t* mask, int32_t n_consumers, const fupr_conv_shape* cons,
                       const float* const* Wc, int32_t* K_keep, int32_t* keep_idx, float* Wp_out,
                       float* bp_out, float* const* Wc_out);

/*
 * Device layout of one convolution's parameters: a blob of fupr_packed_bytes()
 * bytes, to be uploaded to a 256-byte aligned device address.
 *   16-bit types: [bias: Kp floats][weights: nchunk_pad x Kp x 8 elements]
 *       Kp = K rounded up to 16, Cp = C rounded up to 8, chunk j = (r*S + s)*(Cp/8) + c/8
 *       holds channels 8*(c/8)..+7 of tap (r, s); nchunk_pad = R*S*Cp/8 rounded up to 4.
 *   fp32:         [bias: Kp floats][weights: R*S*Cp x Kp floats], Kp = K rounded up to 4,
 *       Cp = C rounded up to 4, row (r*S + s)*Cp + c.
 * Padding entries are zero.  16-bit values are rounded to nearest even.
 * bias may be NULL (zeros).  Returns 0 bytes / an error for invalid shapes or dtypes.
 */
size_t fupr_packed_bytes(const fupr_conv_shape* shape, fupr_dtype dt);
fupr_status fupr_pack(const fupr_conv_shape* shape, const float* W, const float* bias,
                      fupr_dtype dt, void* blob_out);

/* ---------------------------------------------------------------- device -- */

/* An NHWC activation tensor in device memory. */
typedef struct {
  int32_t N, H, W, C, c_stride;
  fupr_dtype dt;
  void* ptr; /* [dev] */
} fupr_tensor;

/*
 * The tensor added before the final ReLU (the building block's shortcut,
 * Table II "add").  Output element (n, p, q, k) receives
 *     t[n, p*spatial_stride, q*spatial_stride, k - c_offset]   if c_offset <= k < c_offset + t.C
 *     0                                                         otherwise,
 * which covers the identity shortcut (stride 1, offset 0, t.C = K), the
 * parameter-free shortcut across a resolution change (stride 2, fewer
 * channels), and a projection shortcut's output.  c_offset is a multiple of 4.
 */
typedef struct {
  fupr_tensor t;
  int32_t spatial_stride, c_offset;
} fupr_residual;

/*
 * y[n,p,q,k] = act( b_k + sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] W[k,c,r,s] (+ res) )
 * (Sec. III; Sec. IV-B-1), accumulated in fp32; the residual is converted to
 * fp32 and added after the bias (this call; the one-kernel schedule of
 * fupr_forward orders the sum differently, see fupr_model_set_schedule); act is ReLU with FUPR_FUSE_RELU, else the
 * identity; one rounding to y's type at the end.  FUPR_FUSE_ADD requires res.
 * packed is [dev] the blob written by fupr_pack for the same shape and dtype.
 * x, y (and res) share one dtype; y->ptr is written, including its zero
 * padding lanes; y must not overlap x, and may overlap res only if res is the
 * identity shortcut with y's own geometry (same pointer, stride 1, offset 0).
 * Errors: NULL, SHAPE (y is not the conv's output shape, x->C != C, ...), DTYPE,
 * ALIGN, ARG, LIMIT, LAUNCH.
 */
fupr_status fupr_conv_fused(const fupr_conv_shape* shape, const fupr_tensor* x, const void* packed,
                            const fupr_residual* res, uint32_t epilogue_flags, const fupr_tensor* y,
                            void* stream);

/*
 * fupr_conv_fused over the channel-wise concatenation of two tensors that is
 * never built (the operator fupr_proj_concat constructs; Sec. IV-B-1): input
 * channel c < split is channel c of x1 at the output pixel (zero from x1->C on),
 * input channel c >= split is channel c - split of x2 at
 * (n, p * x2_spatial_stride, q * x2_spatial_stride), where split = x1->C rounded
 * up to FUPR_CAT_ALIGN.  shape: 1 x 1, stride 1, pad 0, C = split + x2->C.  x1 has the
 * output's extent; x2 has at least (P - 1) * x2_spatial_stride + 1 rows and
 * likewise columns; x2_spatial_stride is 1 or 2; 16-bit types only; everything
 * else (packed, res, flags, y, rounding) as in fupr_conv_fused.
 * Errors: as fupr_conv_fused; DTYPE for fp32 tensors.
 */
fupr_status fupr_conv_cat_fused(const fupr_conv_shape* shape, const fupr_tensor* x1,
                                const fupr_tensor* x2, int32_t x2_spatial_stride, const void* packed,
                                const fupr_residual* res, uint32_t epilogue_flags,
                                const fupr_tensor* y, void* stream);

/*
 * The last convolution of a building block whose OUTPUT filters were pruned
 * (Alg. 1 removes the lowest-norm filters of every non-fused operator, Sec. V-A;
 * fupr_prune with no consumer gives the kept filters and keep_idx).  The block's
 * output keeps its full width, because the shortcut still feeds every channel
 * (Table II "add"); the shape->K kept filters add into their own channels:
 *     y[n,p,q,keep_idx[j]] = act( b_j + conv_j(x)[n,p,q] + y[n,p,q,keep_idx[j]] ),  j < shape->K,
 * in place: on entry y holds the shortcut tensor (identity shortcut: the block's
 * input), every channel not listed is left as it is.  That equals the zero-masked
 * block (removed filters and their batch norm set to zero) whenever act leaves the
 * unlisted channels unchanged, i.e. for a shortcut that is the output of a ReLU.
 * One rounding per updated element; fp32 accumulation as in fupr_conv_fused.
 * keep_idx is [dev], shape->K int32 entries, strictly ascending, in 0 .. y->C - 1
 * (what fupr_prune writes); with any other content the values left in y are
 * unspecified, but no access leaves y.  y has the convolution's output
 * extent and y->C >= shape->K channels; x and y are 16-bit tensors of one type
 * and do not overlap.  epilogue_flags: FUPR_FUSE_RELU or 0.
 * Errors: NULL, SHAPE, DTYPE (fp32 tensors), ALIGN, ARG, LIMIT, LAUNCH.
 */
fupr_status fupr_conv_scatter_fused(const fupr_conv_shape* shape, const fupr_tensor* x,
                                    const void* packed, const int32_t* keep_idx,
                                    uint32_t epilogue_flags, const fupr_tensor* y, void* stream);

/* Max over the taps of a k x k window that fall inside the image (Table II, ImageNet stem). */
fupr_status fupr_maxpool(const fupr_tensor* x, int32_t k, int32_t stride, int32_t pad,
                         const fupr_tensor* y, void* stream);

/* y[n,0,0,c] = mean over H*W of x[n,:,:,c], fp32 accumulation (Table II, before fc). */
fupr_status fupr_global_avgpool(const fupr_tensor* x, const fupr_tensor* y, void* stream);

/*
 * The ImageNet stem of Table II as one operator: y = maxpool_{3x3, stride 2, pad 1}(
 * relu(conv(x) + bias)) without writing the convolution's output to memory
 * (the operator-fusion idea of Sec. IV-B applied to the one "Others" operator
 * that follows a convolution directly).  shape must be 7 x 7, stride 2, pad 3,
 * C <= 4, K = 64; x, y [dev] 16-bit NHWC, y->c_stride = 64, y->H/W the pool's
 * output extent; packed [dev] from fupr_pack.  The result equals fupr_conv_fused
 * (ReLU) followed by fupr_maxpool bit for bit: rounding is monotonic, so the
 * maximum of rounded values is the rounded maximum.
 * Errors: NULL, SHAPE, DTYPE, ALIGN; LIMIT when the shape is not the one above.
 */
fupr_status fupr_conv_maxpool_fused(const fupr_conv_shape* shape, const fupr_tensor* x,
                                    const void* packed, int32_t pool_k, int32_t pool_stride,
                                    int32_t pool_pad, const fupr_tensor* y, void* stream);

/*
 * Two 1 x 1 convolutions in one kernel: y = act1(conv1(x) + bias1 (+ res)) as
 * fupr_conv_fused computes it, and h = act2(conv2(y) + bias2) computed from the
 * rounded y while it is still in registers, so that the second convolution never
 * reads y from memory (a bottleneck block's last convolution and the next
 * block's first one, Table II; operator fusion in the sense of Sec. IV-B applied
 * across a block boundary).  Both y and h are written.  shape1, shape2: 1 x 1,
 * stride 1, pad 0, shape2.C = shape1.K <= 256, shape2.K <= 64, 16-bit types;
 * y->c_stride = shape1.K rounded up to 8.  Arguments as in fupr_conv_fused; the
 * second convolution has no shortcut.  h differs from fupr_conv_fused applied to
 * y only by the order of the fp32 summation inside a 32-channel step.
 * Errors: as fupr_conv_fused; LIMIT when the pair is not of the shape above.
 */
fupr_status fupr_conv_conv1x1_fused(const fupr_conv_shape* shape1, const fupr_tensor* x,
                                    const void* packed1, const fupr_residual* res, uint32_t flags1,
                                    const fupr_tensor* y, const fupr_conv_shape* shape2,
                                    const void* packed2, uint32_t flags2, const fupr_tensor* h,
                                    void* stream);

/* ----------------------------------------------------------------- model -- */

typedef enum { FUPR_OP_CONV = 0, FUPR_OP_MAXPOOL = 1, FUPR_OP_AVGPOOL = 2 } fupr_op_kind;

/*
 * One operator of the optimised network.  Tensors are numbered: 0 is the
 * network input, operator i (0-based) produces tensor i + 1.  A fully-connected
 * layer is a 1x1 convolution on the 1x1 image the global mean leaves.
 */
typedef struct {
  int32_t kind;          /* fupr_op_kind */
  int32_t in;            /* tensor read */
  int32_t res;           /* tensor added in the epilogue, -1 = none (conv only) */
  fupr_conv_shape conv;  /* conv: its shape.  maxpool: R = S = window, stride, pad */
  const void* packed;    /* [dev] conv only: blob from fupr_pack; must outlive the model */
  uint32_t epilogue;     /* conv only: FUPR_FUSE_RELU | FUPR_FUSE_ADD | FUPR_FUSE_SCATTER | FUPR_FUSE_CAT */
  int32_t res_spatial_stride, res_c_offset; /* see fupr_residual */
  /* With FUPR_FUSE_SCATTER (which needs FUPR_FUSE_ADD, 16-bit types, spatial stride 1 and
   * channel offset 0): the operator is fupr_conv_scatter_fused on tensor `res`, updated in
   * place; conv.K filters, keep_idx [dev] as described there, must outlive the model.  The
   * operator's output tensor IS tensor `res` afterwards (same memory, res's width), so `res`
   * must be an intermediate tensor (not 0) that no later operator reads under its old
   * number, and the operator must not be the network's last.  NULL otherwise. */
  const int32_t* keep_idx;
  /* With FUPR_FUSE_CAT (16-bit types): the operator is fupr_conv_cat_fused over tensor
   * `in` and tensor `in2` (an earlier tensor) read at spatial stride in2_spatial_stride;
   * conv.C = (channels of `in` rounded up to FUPR_CAT_ALIGN) + channels of `in2`.  Ignored
   * otherwise. */
  int32_t in2, in2_spatial_stride;
} fupr_op_desc;

typedef struct {
  fupr_dtype dt;
  int32_t C, H, W; /* one input image */
  int32_t n_ops;
  const fupr_op_desc* ops;
} fupr_graph_desc;

typedef struct fupr_model fupr_model;

/*
 * Checks the operator list (shapes chain, ids refer to earlier tensors, residual
 * geometry fits), copies it, and plans which intermediate tensors share memory.
 * Errors: NULL, SHAPE, DTYPE, ARG.  *out is untouched on error.
 */
fupr_status fupr_model_create(const fupr_graph_desc* g, fupr_model** out);
void fupr_model_destroy(fupr_model* m);

/*
 * How fupr_forward schedules the network.  AUTO (default): if every activation
 * tensor of one image fits in the compute unit's LDS (CIFAR-size networks of
 * Table II) and the caller has provided the table below, the whole network runs
 * as ONE kernel, one workgroup per image, activations never leaving LDS;
 * otherwise one kernel per launch group (an operator, or operators that have a
 * kernel together: stem convolution + max-pool, two 1 x 1 convolutions, a
 * bottleneck block).  PER_LAYER: always one kernel per operator.
 * The schedules compute the same operators but round differently: the
 * one-kernel schedule starts the fp32 accumulator from the bias and adds the
 * shortcut as one more MFMA step (before, not after, the last products), and the
 * fused launch groups sum inside a 32-channel step in another order.  Results
 * agree within the rounding of the storage type, not bit for bit.  The
 * one-kernel schedule also assumes FINITE activations: a shortcut value of
 * +-Inf turns all 16 filters of its tile at that pixel into NaN (0 x Inf), where
 * the per-operator kernels keep the other filters finite.
 * The one-kernel schedule is taken only when input->c_stride is the minimal one
 * (C rounded up to 8) and output->c_stride is at most the last operator's padded
 * width; other strides run one kernel per operator.
 */
enum { FUPR_SCHEDULE_AUTO = 0, FUPR_SCHEDULE_PER_LAYER = 1 };
fupr_status fupr_model_set_schedule(fupr_model* m, int32_t schedule);

/*
 * The table the one-kernel schedule walks (per layer: LDS offsets, strides, work
 * item shape, tap offsets).  It lives in device memory that the CALLER provides,
 * like packed parameters:
 *   fupr_model_table_bytes  its size; 0 when the network does not qualify for the
 *                           one-kernel schedule (or m is NULL).
 *   fupr_model_table_write  writes its image to host_out (that many bytes) as it
 *                           must appear at the 256-byte aligned [dev] address
 *                           dev_table (the image holds addresses inside itself and
 *                           the operators' `packed` addresses); the caller copies
 *                           it there.
 *   fupr_model_set_table    tells the model where the copy is; it must stay
 *                           valid and unchanged while the model is used.  NULL
 *                           takes it away again.  Without a table AUTO runs one
 *                           kernel per launch group.
 * Errors: NULL, ALIGN, ARG (the network has no such table).
 */
size_t fupr_model_table_bytes(const fupr_model* m);
fupr_status fupr_model_table_write(const fupr_model* m, const void* dev_table, void* host_out);
fupr_status fupr_model_set_table(fupr_model* m, const void* dev_table);

/*
 * Streams the per-operator schedule may use beside the caller's stream: batches
 * of 192 images or more then run as two sub-batches side by side (images are
 * independent; each sub-batch owns its slice of every workspace buffer), forked
 * from and joined to the stream passed to fupr_forward by events, so that the
 * call stays asynchronous, ordered on that stream, and capturable.  n = 0 .. 3
 * non-NULL hipStream_t of default priority, owned by the caller, alive until the
 * model is destroyed or the streams are replaced; n = 0 (the default) keeps
 * every launch on the caller's stream.  The library creates events here, never
 * streams.  Errors: NULL, ARG (n out of range), LAUNCH.
 */
fupr_status fupr_model_set_side_streams(fupr_model* m, int32_t n, void* const* streams);

/* Bytes of [dev] workspace fupr_forward needs for a batch (0 if m is NULL or batch <= 0). */
size_t fupr_model_workspace_bytes(const fupr_model* m, int32_t batch);

/* Shape of the network output for a batch: fills N, H, W, C, c_stride (minimal), dt; ptr = NULL. */
fupr_status fupr_model_output_shape(const fupr_model* m, int32_t batch, fupr_tensor* out);

/*
 * Runs the network on input (batch = input->N) and writes the last operator's
 * result into output->ptr.  workspace is [dev], 256-byte aligned, at least
 * fupr_model_workspace_bytes(m, batch) bytes, and is only used until the
 * enqueued work completes.  Asynchronous; creates nothing and allocates nothing,
 * so it is safe to capture in a HIP graph (with side streams: capture mode
 * thread-local or relaxed, and `stream` not the default stream).  If a launch
 * fails after sub-batches were forked, the side streams are still joined to
 * `stream` before the error is returned.
 * Errors: NULL, SHAPE, DTYPE, ALIGN, WORKSPACE, LIMIT, LAUNCH.
 */
fupr_status fupr_forward(const fupr_model* m, const fupr_tensor* input, const fupr_tensor* output,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * fupr_forward for the callers that cannot allocate device memory: code under
 * HIP-graph capture, tight serving loops, harnesses that forbid allocation.
 * The workspace is a fixed array of FUPR_STATIC_WORKSPACE_BYTES bytes of device
 * memory inside the library (a file-scope device array: every GPU the library
 * runs on holds its own copy from the moment the library is loaded there until
 * the process ends); its address on the current device is looked up once, at the
 * first call on that device.  The call itself allocates and frees nothing, on the
 * device or through any library.  input and output remain the caller's.
 * Networks and batch sizes whose fupr_model_workspace_bytes exceed the array are
 * refused with FUPR_ERR_WORKSPACE before anything is launched (32 MiB holds the
 * networks of Table II at one image, the paper's setting, and the CIFAR
 * networks up to a few hundred images; the one-kernel schedule needs no
 * workspace at any batch size).  The array keeps what the last call left in it;
 * nothing in it has to start at zero, because every tensor of the workspace is
 * written in full before it is read.  All calls on one GPU share the one array:
 * calls that overlap in time on one GPU (other streams, other threads) race, so
 * the caller orders them.  Otherwise identical to fupr_forward, bit for bit.
 * Errors: those of fupr_forward; WORKSPACE as said; LAUNCH if the runtime cannot
 * locate the array.
 */
#define FUPR_STATIC_WORKSPACE_BYTES (32u << 20)
size_t fupr_static_workspace_bytes(void);
fupr_status fupr_forward_static(const fupr_model* m, const fupr_tensor* input,
                                const fupr_tensor* output, void* stream);

/*
 * As fupr_forward, but brackets every kernel launch with HIP events on the
 * stream, waits for the stream, and writes elapsed times (milliseconds) to the
 * HOST array op_ms, which has fupr_model_num_ops entries: entry i is launch i;
 * entries past the number of launches are 0.  Synchronous.  For measurement only.
 */
fupr_status fupr_forward_timed(const fupr_model* m, const fupr_tensor* input,
                               const fupr_tensor* output, void* workspace, size_t workspace_bytes,
                               void* stream, float* op_ms);

/*
 * Algorithmic work of operator i at a batch size: flops = 2*C*R*S*K per output
 * pixel at the true (pruned) channel counts (0 for pools); bytes = input read
 * once + output written once + residual read once + parameters read once, at
 * the true channel counts and the model's element size.  kernel receives a
 * static string naming the kernel variant the operator launches.
 */
typedef struct {
  double flops, bytes;
  int64_t M;         /* output pixels N*P*Q */
  int32_t K, C, R, S, stride;
  int32_t first_op, n_ops; /* the operators covered: op itself for fupr_model_op_stats; a launch
                              may cover two (stem convolution + max-pool, two 1 x 1 convolutions) */
  const char* kernel;
} fupr_op_stats;
fupr_status fupr_model_op_stats(const fupr_model* m, int32_t batch, int32_t op, fupr_op_stats* out);
int32_t fupr_model_num_ops(const fupr_model* m);

/*
 * Kernel launches of one forward pass under the current schedule (1 for the
 * one-kernel schedule, else one per operator) and the algorithmic work of
 * launch i.  For the one-kernel schedule: all the network's flops; bytes = the
 * images read once + the result written once + every parameter read once.
 */
int32_t fupr_model_num_launches(const fupr_model* m);
fupr_status fupr_model_launch_stats(const fupr_model* m, int32_t batch, int32_t launch,
                                    fupr_op_stats* out);

/*
 * fupr_forward captured once into a HIP graph and replayed (the operators are
 * launch-bound at CIFAR sizes).  Capture happens on `stream`, which must be a
 * non-default stream with no other work in flight; pointers are baked in.
 */
typedef struct fupr_graph fupr_graph;
fupr_status fupr_graph_create(const fupr_model* m, const fupr_tensor* input,
                              const fupr_tensor* output, void* workspace, size_t workspace_bytes,
                              void* stream, fupr_graph** out);
fupr_status fupr_graph_launch(const fupr_graph* g, void* stream);
void fupr_graph_destroy(fupr_graph* g);

/* --------------------------------------------------------------- tuning -- */

/*
 * Process-wide switches that select among kernel instantiations or schedules
 * computing the same operators (for tests and sweeps; normal use needs none).
 * Each starts from the environment variable FUPR_<NAME IN CAPITALS>, read once
 * when the first switch is looked up, and changes only through this call; value
 * NULL or "" returns a switch to automatic.  Launchers read them at every launch.
 *   patch_tile, pipe_tile, stream_tile = <index>
 *                                                 force a tile of that kernel family (where it fits)
 *   conv_tile = <tile name>                       force a tile of the general kernel
 *   conv_patch, conv1x1_stream, conv1x1_pipe, conv1x1_fuse = 0
 *                                                 leave that kernel family out
 *   pipe_order = 0 | 1                            tiles of the pipelined 1 x 1 kernel as one contiguous
 *                                                 range per workgroup | consecutive tiles per XCD
 *   stream_blocks = 1 | 2                         the streaming 1 x 1 kernel built for one or two
 *                                                 workgroups per compute unit
 *   pair_filters = 16..128                        most filters of the second convolution of a pair of
 *                                                 1 x 1 convolutions in one launch
 *   split = 1..4                                  sub-batches of the per-operator schedule
 *   res_item = "M/FT/nsteps:MTxNT,..."            work-item shapes of the one-kernel schedule
 *   debug = 1                                     planner decisions and HIP error text on stderr
 * Errors: NULL, ARG (unknown name, value of 128 characters or more).
 */
fupr_status fupr_tuning_set(const char* name, const char* value);

#ifdef __cplusplus
}
#endif
#endif /* FUPR_H */
