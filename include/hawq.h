/*
 * hawq.h -- C interface of the MI355X (gfx950) integer-only inference kernels for
 * HAWQ-V3 ("Dyadic Neural Network Quantization").
 *
 * The library implements the inference-time arithmetic of the paper and nothing else:
 * low-bit integer convolution / matrix multiply with INT32 accumulation, INT32 bias add,
 * requantisation by a dyadic number b / 2^c (one integer multiply, one rounding right
 * shift; no floating point, no integer division), ReLU / clamp, the dyadic residual
 * addition and integer pooling.
 *
 * Conventions that hold for every entry point unless stated otherwise
 * -------------------------------------------------------------------
 *  - Every tensor / array pointer is DEVICE memory owned by the caller.  The library
 *    allocates nothing on these calls and keeps no reference after the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    only enqueue work; they never synchronise.
 *  - Layouts: activations NHWC, weights KRSC (K output channels, R x S window,
 *    C input channels); dense, innermost axis contiguous.
 *  - HAWQ_U4 / HAWQ_S4 tensors hold two elements per byte along the innermost
 *    (channel) axis: element 2i in bits 0..3, element 2i+1 in bits 4..7 (the same
 *    bytes as eight nibbles in a little-endian 32-bit word); S4 is two's complement.
 *    A 4-bit tensor's channel count must be even.
 *  - Dyadic rescaling of an integer t by (b, c):
 *        rq(t, b, c) = floor(t * b / 2^c + 1/2)         (ties toward +infinity)
 *    evaluated exactly in 64-bit integers.  Preconditions the library cannot check
 *    (the arrays live in device memory): 0 <= b < 2^31 and 1 <= c <= 62.
 *  - Accumulators must stay inside int32.  A static bound is checked from the shape and
 *    the operand ranges (HAWQ_ERR_OVERFLOW); within that bound the caller's bias must
 *    keep |acc + bias| < 2^31.
 *  - Errors are return codes; argument validation happens on the host before any launch
 *    (so it can be exercised without a GPU): a call that fails validation has enqueued nothing.
 *    The entry points that issue several launches (hawq_concat_dyadic: one per branch;
 *    hawq_forward_resnet: one per layer) validate everything they can first; should a later
 *    launch itself fail (HAWQ_ERR_DEVICE), the launches already issued stay enqueued, the
 *    streams are still joined, and the outputs are undefined.
 */
#ifndef HAWQ_H
#define HAWQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HAWQ_OK = 0,
    HAWQ_ERR_NULL = 1,        /* a required pointer is NULL */
    HAWQ_ERR_SHAPE = 2,       /* non-positive size, window larger than padded image, odd 4-bit channel count */
    HAWQ_ERR_DTYPE = 3,       /* dtype not allowed in this position / operand widths differ */
    HAWQ_ERR_RANGE = 4,       /* clamp interval empty or outside the output type */
    HAWQ_ERR_OVERFLOW = 5,    /* static bound says the INT32 accumulator could overflow */
    HAWQ_ERR_UNSUPPORTED = 6, /* valid request this build cannot serve (e.g. tensor >= 2 GiB) */
    HAWQ_ERR_DEVICE = 7,      /* a HIP call failed */
    HAWQ_ERR_WORKSPACE = 8    /* caller's workspace is too small */
} hawq_status;

typedef enum { HAWQ_U8 = 0, HAWQ_S8 = 1, HAWQ_U4 = 2, HAWQ_S4 = 3, HAWQ_S32 = 4 } hawq_dtype;

/* One quantised convolution layer (all fields int32 so the struct has no padding). */
typedef struct {
    int32_t N, H, W, C;            /* input  [N,H,W,C]                                        */
    int32_t K, R, S;               /* weights [K,R,S,C]                                       */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;          /* zero padding; output P = (H + 2 pad_h - R)/stride_h + 1 */
    int32_t x_dtype;               /* HAWQ_U8 | HAWQ_S8 | HAWQ_U4                             */
    int32_t w_dtype;               /* HAWQ_S8 with 8-bit x, HAWQ_S4 with HAWQ_U4 x            */
    int32_t y_dtype;               /* HAWQ_U8 | HAWQ_S8 | HAWQ_U4 | HAWQ_S4 | HAWQ_S32        */
    int32_t res_dtype;             /* HAWQ_U8 | HAWQ_S8 | HAWQ_U4 | HAWQ_S4 (ignored if residual == NULL) */
    int32_t relu;                  /* 1: y = max(y, 0) before the clamp                       */
    int32_t y_lo, y_hi;            /* clamp, e.g. [0,127], [0,15], [-128,127]                 */
    int32_t x_hi;                  /* largest |activation| the caller guarantees; 0 = the type's maximum.
                                      Used by the overflow bound; HAWQ_U8 data with x_hi <= 127 (the
                                      post-ReLU 8-bit range of the workloads) runs on the signed INT8
                                      matrix cores, larger values take a slower exact kernel.   */
    const void *w_blocked;         /* optional (NULL: none): device copy of the same weights made by
                                      hawq_conv_block_weights; the implicit-GEMM kernel then reads it instead of w
                                      (whole cache lines per fetch).  w is still required: other kernels read it. */
    const void *w_fragments;       /* optional (NULL: none): device copy of the same weights made by
                                      hawq_conv_fragment_weights; a 3x3 / stride 1 / pad 1 layer with 128, 256 or 512
                                      input channels (8-bit or packed 4-bit operands), or a 1x1 / stride 1 layer with
                                      512, 1024 or 2048 input channels and K % 256 == 0 (8-bit operands), then runs on
                                      a kernel that keeps its pixels in LDS and streams these.
                                      (hawq_conv2d_dual_int ignores the field: that kernel's two-convolution form needs
                                      a bound on the main branch's values that only hawq_net_create, which sees the
                                      weights on the host, can establish.) */
} hawq_conv_desc;

/*
 * Quantised convolution layer -- Section 3.1 (integer convolution accumulated in INT32, then
 * dyadic requantisation), Appendix D (INT32 bias of the folded batch norm added to the
 * accumulator), Section 3.3 (optional residual: each branch rescaled by its own dyadic
 * number, rounded separately, then added), Figure 1 (ReLU / clamp to the next layer's range).
 *
 *   acc[n,p,q,k] = sum_{r,s,c} x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c] * w[k,r,s,c]
 *   t = acc + bias[k]
 *   y = rq(t, b[k], c[k])  (+ rq(residual[n,p,q,k], res_b[k], res_c[k]) if residual != NULL)
 *   y = clamp(relu ? max(y,0) : y, y_lo, y_hi)          stored as y_dtype, [N,P,Q,K]
 *
 * bias, b, res_b: int32 [K]; c, res_c: uint8 [K].  b == c == NULL is allowed only with
 * y_dtype == HAWQ_S32 and no residual: y = t (raw accumulator + bias).
 * The INT32 accumulator never goes to memory; x and y must not overlap.
 * Every valid request is served; the matrix-core kernels need C a multiple of 64, 16-byte aligned x and w,
 * at most 304 reduction steps (R*S*C/64) and, for their vector epilogue, K a multiple of 16 with 16-byte aligned
 * y / residual / bias / b arrays -- anything else runs on a slower exact kernel with the same results.
 */
hawq_status hawq_conv2d_int(const hawq_conv_desc *desc, const void *x, const void *w, const int32_t *bias,
                            const int32_t *b, const uint8_t *c, const void *residual, const int32_t *res_b,
                            const uint8_t *res_c, void *y, void *stream);

/*
 * Block output with a convolution on both branches -- Section 3.3's residual equation in the form Figure 2 draws
 * for a block that changes shape: the main branch ends in a convolution, the shortcut is a convolution too, both
 * accumulators stay INT32 (neither is written to memory), each is rescaled by its own dyadic number, rounded
 * separately (Appendix G's example) and the integers are added:
 *   t_m = conv(x, w) + bias          t_s = conv(xs, ws) + bias_s
 *   y   = clamp( relu?( rq(t_m, b[k], c[k]) + rq(t_s, b_s[k], c_s[k]) ), y_lo, y_hi )
 * desc describes the main convolution and the output (y_dtype, relu, y_lo, y_hi; res_dtype is ignored); desc_s the
 * shortcut convolution, which must be 1x1 without padding and give the same N, P, Q, K (its y_dtype, relu and
 * clamp are ignored; its operand types follow the rule of hawq_conv2d_int on their own and may differ from the main
 * branch's).  All twelve pointers are device memory and required.  Errors as hawq_conv2d_int; a shortcut that is not
 * 1x1 / unpadded or whose output shape differs -> HAWQ_ERR_SHAPE.
 * 8-bit operands on both branches with C and Cs multiples of 64, K a multiple of 16 and 16-byte aligned arrays run
 * on the matrix cores in one launch; anything else runs on a slower exact kernel with the same results.
 */
hawq_status hawq_conv2d_dual_int(const hawq_conv_desc *desc, const void *x, const void *w, const int32_t *bias,
                                 const int32_t *b, const uint8_t *c, const hawq_conv_desc *desc_s, const void *xs,
                                 const void *ws, const int32_t *bias_s, const int32_t *b_s, const uint8_t *c_s, void *y,
                                 void *stream);

/*
 * Blocked copy of a layer's weights for hawq_conv2d_int / hawq_conv2d_dual_int (hawq_conv_desc::w_blocked): the
 * [K][R*S*C] byte matrix cut into [ceil(K/64)][row bytes / 64][64 channels][64 bytes] blocks, rows past K zero, so that
 * one reduction step of a 64- or 128-channel tile is contiguous memory.  Same integers, another order: results do not
 * change.  hawq_conv_blocked_weights_bytes: size of the copy, 0 if the layer has none (8-bit weights need C % 64 == 0,
 * packed 4-bit weights C % 128 == 0).  hawq_conv_block_weights: device to device, asynchronous on `stream`; w and
 * w_blocked 16-byte aligned device pointers; HAWQ_ERR_UNSUPPORTED if the layer has no blocked form.  Call once per
 * layer, outside the timed path.
 */
size_t hawq_conv_blocked_weights_bytes(const hawq_conv_desc *desc);
hawq_status hawq_conv_block_weights(const hawq_conv_desc *desc, const void *w, void *w_blocked, void *stream);

/*
 * Copy of a layer's weights in matrix-instruction fragment order: [ceil(K/32)][R*S*C/64][2][64 lanes][16 bytes], i.e. for
 * every group of 32 output channels and every 64-byte reduction step the two 1 KB operand fragments exactly as the 64
 * lanes of a wave hold them (channels past K zero).  A wave then loads its weights with fully coalesced reads straight
 * into registers.  Same integers, another order: results do not change.  C % 64 == 0; packed 4-bit weights are expanded
 * to signed bytes on the way (there is no 4-bit matrix instruction), even elements of every 32 before the odd ones -- the
 * order in which the kernel splits the packed activations -- so the copy of a 4-bit layer has the size of an 8-bit one's.
 * Otherwise hawq_conv_fragment_weights_bytes returns 0 and hawq_conv_fragment_weights HAWQ_ERR_UNSUPPORTED.
 * Device to device, asynchronous on `stream`, 16-byte aligned pointers; call once per layer, outside the timed path.
 */
size_t hawq_conv_fragment_weights_bytes(const hawq_conv_desc *desc);
hawq_status hawq_conv_fragment_weights(const hawq_conv_desc *desc, const void *w, void *w_fragments, void *stream);

/*
 * Tail of a bottleneck block in one launch -- Figure 2 / Section 3.3: the block's 3x3 convolution, its requantisation,
 * the 1x1 convolution that restores the channel count, its requantisation, the dyadic-rescaled shortcut, ReLU / clamp:
 *   h = clamp( relu2?( rq(conv3x3(x, w2) + bias2, b2, c2) ), lo2, hi2 )                    (desc2: y_dtype, relu, y_lo, y_hi)
 *   y = clamp( relu3?( rq(conv1x1(h, w3) + bias3, b3, c3) + rq(residual, res_b, res_c) ), lo3, hi3 )     (desc3)
 * -- the very integers of hawq_conv2d_int(desc2) followed by hawq_conv2d_int(desc3, residual), but the tensor h between
 * them stays inside the compute unit (INT32 accumulators in registers, h in LDS) and is never written to memory.
 * desc2: 3x3, stride 1, pad 1, C -> K = C channels, 8-bit operands within the signed range (HAWQ_S8, or HAWQ_U8 with
 * x_hi <= 127), y_dtype HAWQ_U8 / HAWQ_S8 with the clamp inside -128..127.  desc3: 1x1, stride 1, no padding, same N, H,
 * W, C = desc2.K, x_dtype = desc2.y_dtype, y_dtype and res_dtype HAWQ_U8 / HAWQ_S8.  w2_fragments / w3_fragments: the two
 * layers' weights as made by hawq_conv_fragment_weights.  residual [N,H,W,desc3.K] is required.  All pointers device
 * memory, 16-byte aligned tensors.  Shapes served: C = 128 with image width <= 28 and desc3.K a multiple of 128 up to 512;
 * C = 256 with width <= 14 and desc3.K a multiple of 256 up to 1024 (the stage-2 and stage-3 blocks of ResNet50);
 * anything else valid returns HAWQ_ERR_UNSUPPORTED (run the two layers separately).
 */
hawq_status hawq_bottleneck_tail_int(const hawq_conv_desc *desc2, const void *x, const void *w2_fragments, const int32_t *bias2,
                                     const int32_t *b2, const uint8_t *c2, const hawq_conv_desc *desc3, const void *w3_fragments,
                                     const int32_t *bias3, const int32_t *b3, const uint8_t *c3, const void *residual,
                                     const int32_t *res_b, const uint8_t *res_c, void *y, void *stream);

/*
 * Quantised fully connected layer / GEMM -- the matrix-multiply form of Section 3.1:
 *   y[m,n] = epilogue( sum_k x[m,k] * w[n,k] + bias[n] ),   x [M,Kdim], w [N,Kdim], y [M,N]
 * with the epilogue of hawq_conv2d_int (no residual).  b == c == NULL with y_dt == HAWQ_S32
 * returns the raw INT32 logits of the last layer.
 * HAWQ_U8 activations are taken over the type's whole range 0..255 (exact for every byte value).  With at most 512 rows and
 * Kdim a multiple of 512 they run on the matrix cores all the same (the kernel multiplies x - 128 and corrects with
 * 128 * sum(w), exact); other shapes with unsigned bytes take a slower exact kernel, and a caller whose unsigned
 * activations are known to stay within 0..127 (the post-ReLU range of the 8-bit layers) may pass the same buffer as
 * HAWQ_S8: same bytes, same result, every matrix-core form applies.
 */
hawq_status hawq_gemm_int(int32_t M, int32_t N, int32_t Kdim, int32_t x_dt, int32_t w_dt, int32_t y_dt, const void *x,
                          const void *w, const int32_t *bias, const int32_t *b, const uint8_t *c, int32_t relu,
                          int32_t y_lo, int32_t y_hi, void *y, void *stream);

/*
 * Stand-alone residual addition -- Section 3.3:
 *   y[p,k] = clamp( relu?( rq(m[p,k], m_b[k], m_c[k]) + rq(r[p,k], r_b[k], r_c[k]) ), y_lo, y_hi )
 * m: main branch, [n_pixels,K] of HAWQ_S32 (the INT32 accumulator) | S8 | U8 | U4 | S4;
 * r: shortcut, S8 | U8 | U4 | S4 | S32;  y: U8 | S8 | U4 | S4 | S32.  y may alias m or r when the types match.
 */
hawq_status hawq_residual_add_dyadic(int64_t n_pixels, int32_t K, int32_t m_dt, int32_t r_dt, int32_t y_dt,
                                     const void *m, const int32_t *m_b, const uint8_t *m_c, const void *r,
                                     const int32_t *r_b, const uint8_t *r_c, int32_t relu, int32_t y_lo,
                                     int32_t y_hi, void *y, void *stream);

/*
 * Integer global average pool -- Appendix E (pooling carried in INT32) with the paper's rule
 * that no integer division is used: 1/(H*W) is folded into the dyadic multiplier.
 *   s[n,k] = sum_{h,w} x[n,h,w,k]  (INT32);   y[n,k] = clamp(rq(s, b[k], c[k]), y_lo, y_hi)
 * x [N,H,W,C] U8 | S8 | U4 | S4;  y [N,C] U8 | S8 | U4 | S4 | S32.
 */
hawq_status hawq_avgpool_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t x_dt, int32_t y_dt, const void *x,
                             const int32_t *b, const uint8_t *c, int32_t y_lo, int32_t y_hi, void *y, void *stream);

/*
 * Max pool 3x3, stride 2, padding 1 on a quantised tensor (the pool that follows the first
 * convolution of a ResNet; an integer maximum over the in-image taps, then clamp).
 * x [N,H,W,C] U8 | S8 | U4 | S4;  y [N,P,Q,C] with P = (H-1)/2 + 1, of type U8 | S8 | U4 | S4.
 */
hawq_status hawq_maxpool_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t x_dt, int32_t y_dt, const void *x,
                             int32_t y_lo, int32_t y_hi, void *y, void *stream);

/*
 * Pooling carried in INT32 -- Appendix E (the pooling branch of an Inception module works on the INT32 feature map).
 * A window SUM: the divisor of an average pool (R*S with the padding counted, as in the Inception modules) is folded
 * into the dyadic number that follows -- the one given here or the concatenation's -- so there is no integer division.
 *   s[n,p,q,k] = sum over the in-image taps of x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + t, k]
 *   y = s (b == c == NULL, y_dt must be HAWQ_S32)   or   y = clamp(rq(s, b[k], c[k]), y_lo, y_hi)
 * x [N,H,W,C] HAWQ_S32 | U8 | S8 | U4 | S4;  y [N,P,Q,C].  The caller guarantees that a window's sum fits INT32
 * (|x| < 2^31 / (R*S) for INT32 input).  x and y must not overlap.
 */
hawq_status hawq_pool2d_sum_int(int32_t N, int32_t H, int32_t W, int32_t C, int32_t R, int32_t S, int32_t stride_h,
                                int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t x_dt, int32_t y_dt, const void *x,
                                const int32_t *b, const uint8_t *c, int32_t y_lo, int32_t y_hi, void *y, void *stream);

/*
 * Concatenation with one dyadic number per branch -- Appendix E: the branches of a module end at different scales
 * S_i; each is brought to the output scale S_a by its own DN(S_i / S_a), then the channels are laid side by side:
 *   y[p, off_i + k] = clamp( rq(q_i[p,k], b_i[k], c_i[k]), y_lo, y_hi ),   off_i = K_0 + ... + K_(i-1)
 * `branches` is a HOST array of n_branches descriptors whose q / b / c are DEVICE pointers: q [n_pixels,K] of `dtype`
 * (HAWQ_S32 for an accumulator or pooled sum, or a stored low-bit tensor), b int32 [K], c uint8 [K].
 * y [n_pixels, sum K_i] of y_dt.  With a 4-bit type every K_i must be even.  One launch per branch.
 */
typedef struct {
    const void *q;
    const int32_t *b;
    const uint8_t *c;
    int32_t K;
    int32_t dtype;
} hawq_concat_branch;
hawq_status hawq_concat_dyadic(int64_t n_pixels, int32_t n_branches, const hawq_concat_branch *branches, int32_t y_dt,
                               int32_t y_lo, int32_t y_hi, void *y, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Whole-network forward (integer-only ResNet18 / ResNet50, Figure 2 and Section 3.3).
 *
 * Canonical layer order: conv1, then for every stage and block c1, c2, [c3], [ds], finally fc.
 * ResNet50 puts the stride-2 on c1 of a stage's first block.  Storage rule for mixed precision
 * (Section 3.4: one bit width per layer for weights and activations): a tensor is stored at the
 * width of the convolution that reads it (8-bit: 0..127, 4-bit: 0..15, packed); ds shares c1's
 * width and reads the same stored block input; a ds output is signed 8-bit; conv1, the pooled
 * vector and fc are 8-bit (Appendix H).  A network that does not keep its activations may hold a
 * 4-bit tensor in an 8-bit container (values 0..15) and the weights of the 4-bit layers that read it
 * expanded to bytes, where the packed form would be slower (there is no 4-bit matrix instruction);
 * the integers are the same, hawq_net_step_output reports the container type.
 * ------------------------------------------------------------------------------------------- */
typedef struct hawq_net hawq_net;

/* Parameters of one layer, HOST pointers (copied to the device by hawq_net_create). */
typedef struct {
    const void *w;          /* [K,R,S,C] int8, or packed nibbles when bits == 4             */
    const int32_t *bias;    /* [K]                                                          */
    const int32_t *b;       /* [K]  (ignored for fc: raw INT32 logits)                      */
    const uint8_t *c;       /* [K]                                                          */
    const int32_t *res_b;   /* [K] for the last conv of a block (it adds the shortcut), else NULL */
    const uint8_t *res_c;   /* [K] likewise                                                 */
    int32_t bits;           /* 4 or 8; conv1 and fc must be 8; ds must equal its block's c1 */
    int32_t flags;          /* HAWQ_LAYER_* bits, 0 for the default behaviour                */
} hawq_layer_params;

/* On a ds layer: the transition convolution's INT32 accumulator is not stored as a signed 8-bit tensor but added
 * directly to the block's last convolution (hawq_conv2d_dual_int: Figure 2, both branches INT32).  The ds layer's
 * (b, c) then map its accumulator to the block's OUTPUT scale, and the last convolution's res_b / res_c are unused
 * (may be NULL).  One launch replaces two wherever the matrix-core form applies; otherwise the two raw INT32
 * accumulators pass through the workspace and a residual-addition launch. */
#define HAWQ_LAYER_INT32_SHORTCUT 1

/* Shape of layer `index` of the canonical order, for a square image of side image_hw. */
typedef struct {
    char name[24];          /* "conv1", "layer2.0.c1", "layer2.0.ds", "fc", ...             */
    int32_t C, K, R, S, stride, pad;
    int32_t H, W;           /* input size                                                   */
    int32_t P, Q;           /* output size                                                  */
    int32_t has_residual;   /* 1: res_b / res_c are required                                */
    int32_t is_ds;          /* 1: transition (shortcut) convolution                         */
} hawq_layer_info;

/* Host-only topology queries (no GPU needed).  arch = 18 or 50. */
int32_t hawq_net_num_layers(int32_t arch);
hawq_status hawq_net_layer_info(int32_t arch, int32_t image_hw, int32_t num_classes, int32_t index,
                                hawq_layer_info *out);

/*
 * Build a network: validates the parameters (here b and c are host data, so 0 <= b < 2^31 and
 * 1 <= c <= 62 ARE checked -> HAWQ_ERR_RANGE), allocates one device arena, uploads weights
 * (conv1 re-tiled for its kernel; every other layer also in the blocked order the implicit-GEMM kernel reads, so the
 * arena holds about twice the weights' size) and parameters, and creates the second stream and two events that
 * hawq_forward_resnet uses for large batches.  pool_b / pool_c: [C_last] host arrays of
 * the average pool's dyadic multiplier.  keep_activations != 0 gives every layer's output its own
 * workspace slot (for layer-by-layer comparison) instead of reusing buffers.
 * Synchronous; call outside any timed region.  Free with hawq_net_destroy.
 */
hawq_status hawq_net_create(int32_t arch, int32_t image_hw, int32_t num_classes, const hawq_layer_params *layers,
                            int32_t n_layers, const int32_t *pool_b, const uint8_t *pool_c,
                            int32_t keep_activations, hawq_net **out);
void hawq_net_destroy(hawq_net *net);

/* Bytes of caller-provided device workspace hawq_forward_resnet needs for a batch of N. */
size_t hawq_net_workspace_bytes(const hawq_net *net, int32_t N);

/* Images in the first of the two parts hawq_forward_resnet runs a batch of N as (see there); 0: one part. */
int32_t hawq_net_split_first(const hawq_net *net, int32_t N);

/* Number of launches of one forward: conv1, max pool, the convolutions, average pool, fc. */
int32_t hawq_net_num_steps(const hawq_net *net);

/*
 * Where step `step` leaves its output inside the workspace for batch N, and what it is
 * (valid until a later step reuses the slot; permanent with keep_activations).
 * name: at least 24 bytes.  dtype: hawq_dtype of the stored tensor.
 * The offsets describe a batch that runs as one part (always the case with keep_activations); when
 * hawq_net_split_first(net, N) is not 0 the two parts have their own regions of the workspace, the first laid out
 * as for a batch of that many images at the start, the second behind it.
 */
hawq_status hawq_net_step_output(const hawq_net *net, int32_t N, int32_t step, char *name, size_t *offset,
                                 size_t *bytes, int32_t *dtype, int32_t *dims4 /* N,P,Q,K */);

/*
 * Integer-only forward: x uint8 [N,image_hw,image_hw,3] (values 0..255) -> logits int32
 * [N,num_classes].  x, logits and workspace are device memory; workspace must hold
 * hawq_net_workspace_bytes(net, N) bytes, 256-byte aligned; x must be 16-byte aligned.  Enqueues every layer on
 * `stream`.  Unless the network keeps its activations, conv1 and the max pool run as one kernel and the conv1
 * tensor is never written to memory (its step reports an empty output).
 * Stream semantics: as if every launch were on `stream` -- the forward starts after all work queued on `stream`
 * before the call and work queued after the call sees the finished logits.  Inside, a batch of 96 images or more
 * (without kept activations) runs as two halves, the second on a stream the network owns (default priority, created
 * by hawq_net_create), forked and joined with events; images are independent, so the bits do not depend on it.
 * Because that stream and its two events belong to the network object, calls on one hawq_net must be issued from one
 * host thread at a time (any number may be in flight on the device).
 */
hawq_status hawq_forward_resnet(const hawq_net *net, const void *x, int32_t N, int32_t *logits, void *workspace,
                                size_t workspace_bytes, void *stream);

/*
 * The same forward for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Identical to hawq_forward_resnet except that the workspace is
 * a fixed array of hawq_noalloc_workspace_limit() bytes (64 MiB) inside the library's device code, one per GPU, held
 * until the process ends; x and logits are still the caller's device buffers.  The call allocates nothing (no
 * hipMalloc / hipFree, no allocating library routine).  hawq_net_workspace_bytes(net, N) must not exceed the limit --
 * HAWQ_ERR_WORKSPACE otherwise (ResNet50 at 224x224 fits up to a batch of about 28, ResNet18 about 100).
 * Every call on a GPU uses that GPU's one array (its contents are whatever the last call left; the forward reads
 * nothing it has not written): calls that overlap in time on one GPU -- from different streams, networks or
 * threads -- race.  Serialise them, e.g. by issuing them on one stream.  A network with kept activations may use it
 * too; hawq_net_step_output's offsets are then relative to the array, which the caller cannot read.
 */
size_t hawq_noalloc_workspace_limit(void);
hawq_status hawq_forward_resnet_noalloc(const hawq_net *net, const void *x, int32_t N, int32_t *logits, void *stream);

/*
 * Same forward with a pair of HIP events around every step, recorded on `stream`; on return the
 * stream has been synchronised and step_ms[i] (host array, hawq_net_num_steps entries) holds the
 * device time of step i in milliseconds.  For measurement only.
 */
hawq_status hawq_forward_resnet_timed(const hawq_net *net, const void *x, int32_t N, int32_t *logits,
                                      void *workspace, size_t workspace_bytes, void *stream, float *step_ms);

/* Static description of a step for reporting: multiply-accumulates and minimum HBM bytes
 * (input once + weights + parameters + output once + shortcut once) at batch N. */
hawq_status hawq_net_step_cost(const hawq_net *net, int32_t N, int32_t step, double *macs, double *bytes);

/* Measurement hook for tile-shape sweeps: 0 = the built-in heuristic (default), 1..3 = force one of the
 * matrix-core kernel's workgroup tiles (128x128 as four waves, 64x128, 64x64 channels x pixels) for every
 * later call in this process; any other value is taken as 0.  Process-wide state: set it only from a
 * single-threaded measurement program.  Results are identical for every setting. */
void hawq_tune_set_tile(int32_t tile);

/* Measurement hook for the batch split of hawq_forward_resnet: 0 = the built-in rule (default), -1 = never split,
 * n > 0 = first part of n images (the rest forms the second part) for every later call in this process.  Set it before
 * sizing the workspace.  Results are identical for every setting. */
void hawq_tune_set_split(int32_t n_first);

/* Measurement hook for the network plan: networks created by later hawq_net_create calls run the 3x3 and the closing 1x1 of
 * an identity-shortcut bottleneck block as one launch (the kernel of hawq_bottleneck_tail_int) wherever it applies (1),
 * only where the 3x3 has 256 input channels (2), or by the plan's own rule (0, default: the rule keeps two launches on the
 * ResNet50 shapes, where one launch measured slower).
 * Process-wide state, as hawq_tune_set_tile.  Results are identical for every setting. */
void hawq_tune_set_fusion(int32_t mode);

/*
 * Measurement helper: TOP/s of a register-only loop of independent INT8 matrix instructions (32x32x32, four
 * accumulators per wave, sixteen waves per compute unit, `iters` rounds, no memory traffic in the loop) on the current
 * device's default stream -- the sustained matrix-core rate to hold a convolution's TOP/s against, next to the
 * datasheet peak.  Synchronous; allocates and frees 1 MB of device memory.  tops: host pointer.
 * HAWQ_ERR_RANGE unless 1 <= iters <= 1000000.
 */
hawq_status hawq_probe_mfma_peak(int32_t iters, double *tops);

const char *hawq_status_string(hawq_status s);

#ifdef __cplusplus
}
#endif
#endif /* HAWQ_H */
