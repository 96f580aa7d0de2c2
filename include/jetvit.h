/*
 * jetvit.h -- C ABI of the MI355X (gfx950) token-mixer library for JetViT's
 * hybrid-attention Vision Transformer.
 *
 * The library computes the forward pass of the three token mixers that the
 * paper's Post-Training Attention Search assigns per layer -- ReLU-kernel
 * linear attention, non-overlapping 2-D window attention, and the retained
 * full softmax attention -- on caller-owned device buffers.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Pointers named q, k, v, o, workspace and every pointer documented as
 *    "device" are DEVICE pointers (HBM, current HIP device).  Pointers
 *    documented as "host" are host pointers.  Descriptor structs are host
 *    memory and are read before the call returns.
 *  - Ownership: the caller owns every buffer and the stream.  The library never
 *    allocates or frees device memory, never synchronises, and launches only on
 *    the stream it is given (hip_stream is a hipStream_t; NULL is the default
 *    stream).  Scratch memory comes in through `workspace`.
 *  - Tensors Q, K, V, O are logically [batch, heads, N, head_dim] with
 *    N = n_prefix + grid_h * grid_w tokens: the prefix tokens, then the grid in row-major
 *    raster order (grid cell (r, c) is token n_prefix + r*grid_w + c).
 *    The head_dim axis is contiguous; the other three axes have the element
 *    strides given in jv_strides, so a fused QKV projection output laid out
 *    [batch, N, 3, heads, head_dim] can be consumed without a transpose.
 *    Base pointers and all strides must keep every (b, h, n) row 16-byte aligned.
 *  - head_dim is 64, or 128 (the wide heads of the paper's largest backbones, Tab. 3/4) with
 *    JV_BF16 tensors: full, window and linear attention (prefix tokens included) and the
 *    linear-attention block with static or squeeze-dynamic filters are built for both; the
 *    focused map, token-wise filters and JV_F32 tensors for 64 only (JV_ERR_UNSUPPORTED
 *    otherwise).
 *  - Inputs are never written.  O must not overlap Q, K or V: the byte range that O's
 *    strides span may not intersect the range of any input (JV_ERR_INVALID_ARG).
 *  - Arithmetic: JV_F32 tensors are processed in fp32 throughout.  JV_BF16
 *    tensors feed bf16 matrix instructions with fp32 accumulation; softmax,
 *    normalisers and divisions are fp32.  O is rounded to `o_dtype` once, at the
 *    final store (round to nearest even).
 *  - Errors: every call validates its arguments on the host before any launch
 *    and returns a jv_status.  On any status other than JV_OK nothing was
 *    launched and no buffer was touched (JV_ERR_HIP excepted: a launch was
 *    attempted and the HIP runtime refused it).  No call aborts, throws or
 *    prints.  jv_last_error() returns a thread-local description of the last
 *    failure on the calling thread.
 *  - Thread safety: concurrent calls are safe as long as their output and
 *    workspace buffers do not overlap.  The only process-wide state is, per kernel
 *    that needs more than 64 KB of LDS, an atomic record of the devices on which
 *    that limit has been raised (done on the first call on each device, with that
 *    device current: make the first call on a device outside stream capture).
 */
#ifndef JETVIT_H
#define JETVIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    JV_OK = 0,
    JV_ERR_INVALID_ARG = 1,         /* null pointer, non-positive size, bad stride/alignment */
    JV_ERR_UNSUPPORTED = 2,         /* valid request this build does not implement */
    JV_ERR_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes below the *_workspace_bytes query */
    JV_ERR_HIP = 4                  /* the HIP runtime rejected a launch */
} jv_status;

typedef enum { JV_F32 = 0, JV_BF16 = 1 } jv_dtype;

/* Element strides of one [batch, heads, N, head_dim] tensor; head_dim stride is 1. */
typedef struct {
    int64_t stride_b, stride_h, stride_n;
} jv_strides;

typedef struct {
    int32_t batch, heads;
    int32_t grid_h, grid_w; /* token grid */
    int32_t head_dim;       /* 64 or 128 (128: bf16 tensors) */
    jv_dtype dtype;         /* element type of Q, K, V */
    jv_dtype o_dtype;       /* element type of O: equal to dtype, or JV_F32 with JV_BF16 inputs */
    jv_strides q, k, v, o;
    int32_t n_prefix;       /* tokens in front of the grid (class / register tokens), 0 .. 64;
                               N = n_prefix + grid_h * grid_w.  See "Prefix tokens" below. */
} jv_attn_desc;

/* Prefix tokens.  Backbones such as the paper's teachers carry a few tokens that belong to no
 * grid position (a class token, register tokens) in front of the patch tokens.  The paper does
 * not say how its mixers treat them; this library's rule, for a sequence of n_prefix such
 * tokens followed by the grid tokens in raster order:
 *  - full attention and linear attention take all N tokens as ordinary tokens;
 *  - window attention: a grid token attends to the grid tokens of its window (prefix tokens
 *    are in no window); a prefix token attends to all N tokens;
 *  - the depth-wise convolution of the linear-attention block runs over the grid only (zero
 *    padding at its border as before): prefix tokens receive no convolution term and feed
 *    none; the token average that generates the dynamic filters runs over all N tokens.
 * Token n of the tensors is prefix token n for n < n_prefix, else grid cell n - n_prefix. */

const char *jv_version(void);
const char *jv_status_string(jv_status status);
const char *jv_last_error(void);

/* ---------------------------------------------------------------------------
 * Linear attention (Sec. 3.2.1, Eq. 2 with the ReLU feature map the block keeps;
 * the output is normalised by the key sum):
 *     S = sum_j relu(k_j)^T v_j   (head_dim x head_dim, per batch and head)
 *     z = sum_j relu(k_j)
 *     o_i = relu(q_i) S / (relu(q_i) . z + eps)
 * Two passes: a streaming reduction of K and V into partial (S, z) states held
 * in `workspace`, then a pass over Q that sums the partials and applies them.
 * No 1/sqrt(d) scaling is applied.  eps is added to the denominator; eps < 0
 * or NaN is JV_ERR_INVALID_ARG.
 *
 * workspace: device, at least jv_linear_attn_workspace_bytes(desc) bytes,
 * 256-byte aligned; contents on entry are ignored, contents on return are
 * unspecified.  The query returns 0 for an invalid descriptor.
 * ------------------------------------------------------------------------- */
size_t jv_linear_attn_workspace_bytes(const jv_attn_desc *desc);
jv_status jv_linear_attn_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                             const void *v, void *o, float eps, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------
 * jv_linear_attn_fwd_static: jv_linear_attn_fwd for callers that cannot allocate device memory
 * or pass a workspace -- code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same kernels and same result as jv_linear_attn_fwd; the partial states live in a
 * fixed array of JV_STATIC_SCRATCH_BYTES of device memory that is part of the library's code
 * object (every GPU the library runs on holds one copy until the process ends).  The call
 * allocates and frees nothing; its first call on a device looks the array's address up.
 * Problems whose states need more than the array holds (jv_linear_attn_workspace_bytes(desc) >
 * JV_STATIC_SCRATCH_BYTES) are refused with JV_ERR_UNSUPPORTED before any launch.  All calls on
 * one GPU share the array: calls that may overlap in time on the same GPU (different streams or
 * threads) race with each other and must be serialised by the caller; calls on one stream are
 * ordered by the stream.  Nothing in the array has to be cleared between calls.
 * ------------------------------------------------------------------------- */
#define JV_STATIC_SCRATCH_BYTES (32u << 20)
jv_status jv_linear_attn_fwd_static(const jv_attn_desc *desc, const void *q, const void *k,
                                    const void *v, void *o, float eps, void *hip_stream);

/* ---------------------------------------------------------------------------
 * The paper's linear-attention block (Sec. 3.2.1, Eq. 4): the normalised ReLU linear attention
 * above plus a depth-wise convolution of V on the token grid,
 *     O = LA(Q, K, V) + DWC(V).
 * V is viewed as [batch, C = heads*64, grid_h, grid_w] (channel = head*64 + c); DWC is a
 * depth-wise (one filter per channel) ksize x ksize cross-correlation, stride 1, zero padding
 * ksize/2, no bias; its result is added in fp32 before O is rounded.
 *   JV_DWC_NONE             plain linear attention (same result as jv_linear_attn_fwd).
 *   JV_DWC_STATIC           one filter bank static_kernel, device fp32 [C, ksize, ksize].
 *   JV_DWC_SQUEEZE_DYNAMIC  the block the paper proposes ("Squeeze Dynamic Convolution"): the
 *       filter bank is generated per image from the token average of V by a two-layer MLP
 *       with SiLU and is shared by all tokens of that image:
 *           g = mean_n V[b, :, n];  u = silu(w1 g + b1);  kernel[b] = reshape(w2 u + b2, [C, k, k])
 *       w1 fp32 [hidden, C], b1 fp32 [hidden], w2 fp32 [C*k*k, hidden], b2 fp32 [C*k*k], device.
 *       The token sum of V is taken in the same pass that reduces K and V into the state.
 *   JV_DWC_TOKEN_DYNAMIC    the variant the paper tried first and rejected for its cost (Sec. 3.2.1;
 *       Tab. 1, "Token-wise Dynamic DWC"): the same generator applied to every grid token's own
 *       V row, so that each token carries a filter bank of its own, which weights that token's
 *       ksize x ksize neighbourhood:
 *           u_n = silu(w1 V[b, :, n] + b1);  kernel[b, n] = reshape(w2 u_n + b2, [C, k, k]);
 *           DWC(V)[b, c, n] = sum_taps kernel[b, n][c, tap] * V[b, c, n + tap]
 *       Weights as for the squeeze-dynamic mode; hidden a multiple of 64 (JV_ERR_UNSUPPORTED
 *       otherwise).  bf16 tensors: the generator runs as two matrix products with bf16
 *       operands and fp32 accumulation (w1, w2 and the hidden layer are rounded to bf16: pass
 *       weights that are bf16 values already and only the hidden layer is rounded; the filters
 *       stay fp32) over V as the matrix [batch * tokens, C] -- read in place when V's strides
 *       already describe one (head stride 64, batch stride = tokens * token stride), from a
 *       packed copy otherwise; the workspace holds the filters of all tokens (batch * tokens *
 *       C * k * k fp32), the cost the paper rejects the variant for.  fp32 tensors: plain fp32
 *       arithmetic throughout, one workgroup per token, only the hidden layer is kept (the
 *       workspace size is the same for both element types).  Prefix tokens get no convolution
 *       term.
 * ksize is 3 or 5; C <= 8192 and hidden <= 1024 (JV_ERR_UNSUPPORTED otherwise).  Pointers the
 * mode does not use are ignored.  workspace as for jv_linear_attn_fwd, sized by
 * jv_linear_block_workspace_bytes (0 for an invalid descriptor or parameter block).
 * ------------------------------------------------------------------------- */
typedef enum {
    JV_DWC_NONE = 0,
    JV_DWC_STATIC = 1,
    JV_DWC_SQUEEZE_DYNAMIC = 2,
    JV_DWC_TOKEN_DYNAMIC = 3
} jv_dwc_mode;

typedef struct {
    jv_dwc_mode mode;
    int32_t ksize;              /* 3 or 5 */
    int32_t hidden;             /* hidden width of the generator (dynamic modes) */
    const float *static_kernel; /* device, [C, ksize, ksize] (static only) */
    const float *w1, *b1, *w2, *b2; /* device (dynamic modes) */
} jv_dwc_params;

size_t jv_linear_block_workspace_bytes(const jv_attn_desc *desc, const jv_dwc_params *dwc);
jv_status jv_linear_block_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                              const void *v, void *o, float eps, const jv_dwc_params *dwc,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same block with the focused feature map in place of ReLU (Eq. 3: the kernel function
 * the paper tries on top of the convolution branch and rejects for its cost, Table 1 row
 * "+ DWC on V + Focusing Factor"; provided to measure that variant):
 *     phi_p(x) = |r| / |r^p| * r^p,   r = max(x, 0),
 * powers element-wise, Euclidean norms over the 64 channels of the token's head, phi_p(x) = 0
 * where r = 0.  (The printed denominator is read as the norm of the powered vector, which
 * makes phi_p norm-preserving.)  focus_p is an integer power, 1 <= focus_p <= 16;
 * focus_p = 1 is jv_linear_block_fwd.  Applied to q and k in fp32 from the stored values; for
 * bf16 tensors the mapped rows are rounded to bf16 again before the matrix products.
 * Everything else (arguments, workspace size, errors) as for jv_linear_block_fwd. */
jv_status jv_linear_block_focused_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                                      const void *v, void *o, float eps, int32_t focus_p,
                                      const jv_dwc_params *dwc, void *workspace,
                                      size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Window partition (Sec. 3.2.2: the feature map is split into non-overlapping
 * windows).  The grid is extended at the bottom and right to multiples of the
 * window (padded_h x padded_w); windows are anchored at (0, 0) and numbered
 * row-major; the win_h*win_w slots of a window are numbered row-major.
 *
 * jv_window_geometry: host computation; the three outputs are host pointers.
 *
 * jv_window_maps_host / jv_window_maps_device fill (any output may be NULL):
 *   token_index     int32 [n_windows * win_h*win_w]  token r*grid_w+c of the slot, -1 for padding
 *   pad_mask        uint8 [n_windows * win_h*win_w]  1 for a real token, 0 for padding
 *   window_of_token int32 [grid_h*grid_w]            window that holds each token
 * The _host variant takes host pointers and runs on the CPU; the _device
 * variant takes device pointers and runs one kernel on hip_stream.  Both give
 * identical bytes.
 * ------------------------------------------------------------------------- */
jv_status jv_window_geometry(int32_t grid_h, int32_t grid_w, int32_t win_h, int32_t win_w,
                             int32_t *padded_h, int32_t *padded_w, int32_t *n_windows);
jv_status jv_window_maps_host(int32_t grid_h, int32_t grid_w, int32_t win_h, int32_t win_w,
                              int32_t *token_index, uint8_t *pad_mask, int32_t *window_of_token);
jv_status jv_window_maps_device(int32_t grid_h, int32_t grid_w, int32_t win_h, int32_t win_w,
                                int32_t *token_index, uint8_t *pad_mask,
                                int32_t *window_of_token, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Window attention (Sec. 3.2.2): every token attends, with the softmax
 * attention of Eq. 1, to the real tokens of its own win_h x win_w window only.
 * Padding is virtual: Q, K, V, O hold the grid_h*grid_w real tokens; padded key
 * slots are excluded from the softmax (not merely zero-valued) and padded query
 * slots produce no output.  scale multiplies the logits; scale <= 0 or NaN
 * selects 1/sqrt(head_dim).
 * ------------------------------------------------------------------------- */
jv_status jv_window_attn_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                             const void *v, void *o, int32_t win_h, int32_t win_w, float scale,
                             void *hip_stream);

/* ---------------------------------------------------------------------------
 * Full softmax attention (Eq. 1): o_i = sum_j softmax_j(scale * q_i . k_j) v_j
 * over all N tokens, computed tile by tile with a running maximum and sum.
 * scale <= 0 or NaN selects 1/sqrt(head_dim).
 * ------------------------------------------------------------------------- */
jv_status jv_full_attn_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                           const void *v, void *o, float scale, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Encoder pieces.  The paper's hybrid encoder keeps the pretrained block around each token
 * mixer (Sec. 3.2.3: the MLP and the attention projections W_Q, W_K, W_V, W_O are inherited
 * unchanged); the block is the standard pre-LN transformer block.
 *
 * jv_layernorm_fwd: y[r, :] = (x[r, :] - mean) / sqrt(var + eps) * gamma + beta over `cols`
 * (population variance, fp32 statistics).  x is [rows, cols] of x_dtype, gamma and beta are
 * fp32 [cols], y is [rows, cols] of y_dtype; all device, rows contiguous, cols % 8 == 0.
 *
 * jv_gemm_bias_act: y = epilogue(a w^T + bias), a [M, K] bf16 and w [N, K] bf16 both row-major
 * (K contiguous), fp32 accumulation on the matrix cores.  bias is fp32 [N] or NULL.
 *   JV_EPI_NONE      y = acc + bias
 *   JV_EPI_GELU      y = gelu(acc + bias), the exact (erf) GELU x Phi(x), Phi to 5e-6 absolute
 *   JV_EPI_RESIDUAL  y = acc + bias + residual, residual [M, N] of y's element type (may be y
 *                    itself); the sum is formed in fp32 and rounded once
 *   JV_EPI_SILU      y = silu(acc + bias), silu(x) = x / (1 + exp(-x))
 * y is [M, N] of y_dtype (JV_BF16 or JV_F32).  K % 64 == 0 and N % 8 == 0 are required
 * (JV_ERR_UNSUPPORTED otherwise); M is arbitrary up to 2^30, K up to 2^21.  All pointers
 * device, 16-byte aligned.
 * ------------------------------------------------------------------------- */
typedef enum { JV_EPI_NONE = 0, JV_EPI_GELU = 1, JV_EPI_RESIDUAL = 2, JV_EPI_SILU = 3 } jv_epilogue;

jv_status jv_layernorm_fwd(const void *x, const float *gamma, const float *beta, void *y,
                           int64_t rows, int32_t cols, float eps, jv_dtype x_dtype,
                           jv_dtype y_dtype, void *hip_stream);
jv_status jv_gemm_bias_act(const void *a, const void *w, const float *bias, const void *residual,
                           void *y, int64_t M, int32_t N, int32_t K, jv_epilogue epilogue,
                           jv_dtype y_dtype, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Hybrid encoder forward (Fig. 2 of the paper: per layer, one of the three token mixers;
 * Sec. 4.4 works with a 24-layer ViT-Large).  For every block l:
 *     a = LN(x; ln1);  [Q K V] = a W_qkv^T + b_qkv, split into heads of width / heads channels;
 *     x += mix_{pattern[l]}(Q, K, V) W_o^T + b_o;
 *     x += gelu(LN(x; ln2) W_fc1^T + b_fc1) W_fc2^T + b_fc2.
 * The residual stream x is fp32 (stream_dtype JV_F32, the default) or bf16 (JV_BF16: what a
 * network converted to bf16 as a whole carries; every block then rounds the stream twice, and
 * each residual GEMM and LayerNorm moves half the bytes); GEMM operands and the tensors between
 * kernels are bf16.
 * No final norm: the output is the residual stream after the last block.
 *
 * jv_encoder_create copies the configuration and the table of weight POINTERS into a host
 * object; the weights themselves stay where they are (device memory owned by the caller,
 * which must outlive the object).  pattern is a host array of n_blocks values
 * (0 linear, 1 window, 2 full).  Weights per block: LayerNorm gamma/beta fp32 [width];
 * w_qkv bf16 [3*width, width] (rows: Q features, then K, then V), b_qkv fp32 [3*width];
 * w_o bf16 [width, width], b_o fp32; w_fc1 bf16 [mlp_hidden, width], b_fc1 fp32;
 * w_fc2 bf16 [width, mlp_hidden], b_fc2 fp32.  width = heads * 64 or heads * 128 (wide heads:
 * linear-attention blocks with the ReLU map only, static or squeeze-dynamic filters), width
 * and mlp_hidden multiples of 64.
 *
 * jv_encoder_forward: x and y are device [batch, n_prefix + grid_h*grid_w, width] of stream_dtype
 * (y may be x);
 * workspace is device memory of at least jv_encoder_workspace_bytes(...) bytes, 256-byte
 * aligned.  About 8 launches per block, all on hip_stream, no synchronisation.  Every shape the
 * pass would launch (its four matrix products, the window partition, the token counts) is
 * checked before the first launch; jv_encoder_workspace_bytes returns 0 for a (batch, grid) that
 * jv_encoder_forward would refuse.  With few tokens (the output of the second MLP product has
 * fewer than 128 tiles of 256 x 256) that product's K loop is split over two or four workgroups
 * per tile, whose fp32 partial results are added, with bias and residual, in a pass of their
 * own and in a fixed order; the workspace query accounts for the partial results.
 *
 * jv_encoder_forward_taps: the same forward pass that also hands out the residual stream after
 * chosen blocks, which is what a dense-prediction head attached to the encoder reads (the
 * paper's depth and segmentation heads take features of four intermediate layers, Sec. 4.1
 * and 4.2).  tap_blocks is a host array of n_taps block indices (0-based, strictly increasing,
 * each < n_blocks); tap_out is a host array of n_taps device pointers, each of stream_dtype,
 * [batch, grid_h*grid_w, width], 16-byte aligned, distinct from each other and from x and y.
 * tap_out[i] receives the stream after block tap_blocks[i].  The block's last GEMM writes
 * there directly and the next block reads it from there, so a tap costs no extra pass over the
 * stream (a tap on the last block is one device-to-device copy of y).  n_taps = 0 is
 * jv_encoder_forward.
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t n_blocks, width, heads, mlp_hidden;
    int32_t win_h, win_w;  /* window of the window-attention blocks */
    float ln_eps, la_eps;  /* LayerNorm epsilon; linear-attention denominator epsilon */
    const uint8_t *pattern; /* host, n_blocks entries: 0 linear, 1 window, 2 full */
    int32_t la_focus_p;     /* feature map of the linear-attention blocks: 0 or 1 = ReLU (the
                               paper's block), 2 .. 16 = focused map of that power (the ablation
                               variant, see jv_linear_block_focused_fwd) */
    int32_t n_prefix;       /* prefix tokens in front of the grid tokens of every image, 0 .. 64
                               (see "Prefix tokens" at jv_attn_desc); x and y are then
                               [batch, n_prefix + grid_h*grid_w, width] */
    jv_dtype stream_dtype;  /* element type of the residual stream: x, y and the taps */
} jv_encoder_config;

typedef struct {
    const float *ln1_g, *ln1_b;
    const void *w_qkv; const float *b_qkv;
    const void *w_o; const float *b_o;
    const float *ln2_g, *ln2_b;
    const void *w_fc1; const float *b_fc1;
    const void *w_fc2; const float *b_fc2;
    /* Linear-attention blocks only: the convolution branch of the paper's block (Eq. 4), as for
     * jv_linear_block_fwd; host pointer, copied by jv_encoder_create; NULL = plain linear
     * attention.  Ignored for window and full-attention blocks. */
    const jv_dwc_params *dwc;
} jv_block_weights;

typedef struct jv_encoder jv_encoder;

jv_status jv_encoder_create(const jv_encoder_config *config, const jv_block_weights *blocks,
                            jv_encoder **out);
size_t jv_encoder_workspace_bytes(const jv_encoder *enc, int32_t batch, int32_t grid_h,
                                  int32_t grid_w);
/* ---------------------------------------------------------------------------
 * jv_encoder_fold_layernorm (optional, once after jv_encoder_create): fold the block's two
 * LayerNorms into the matrix products behind them, so that a forward pass runs no LayerNorm pass
 * except the very first one.  The block is unchanged as a function (pre-LN block of Sec. 3.2.3's
 * inherited MLP and projections); what changes is where the normalisation is applied:
 *     W LN(x) + b = rstd (W diag(gamma)) x - rstd mean (W gamma) + (W beta + b),
 * so the products multiply the bf16 stream itself with the weights scaled by gamma (rounded to
 * bf16 once more), and mean and 1/sigma enter their epilogues; the residual products before
 * them write the stream's bf16 rows and per-row statistics next to their result.  Rounding
 * differs from the separate pass (the stream is rounded before the mean is removed, so the
 * relative error grows with |mean| / sigma of a token's features), the arithmetic does not.
 * buffer: device memory of jv_encoder_fold_bytes(enc) bytes, 256-byte aligned, owned by the
 * caller; the call launches the folding kernels on hip_stream and the encoder keeps the pointer:
 * the buffer must stay alive and unchanged while forward passes run.  Afterwards
 * jv_encoder_workspace_bytes asks for one more [tokens, width] bf16 buffer and the statistics.
 * buffer = NULL switches back to separate LayerNorm passes.
 * ------------------------------------------------------------------------- */
size_t jv_encoder_fold_bytes(const jv_encoder *enc);
jv_status jv_encoder_fold_layernorm(jv_encoder *enc, void *buffer, size_t buffer_bytes, void *hip_stream);
/* ---------------------------------------------------------------------------
 * jv_encoder_fuse_linear_projection (optional): in the linear-attention blocks, fold the apply
 * pass of Eq. 2 into the output projection the block inherits (Sec. 3.2.3).  With
 * o_h = relu(q_h) S_h / den_h and den_h = relu(q_h) . z_h + eps,
 *     concat_h(o_h) W_O^T = A' W'_b^T,   A'[t, 64 h + i] = relu(q_h[t, i]) / den_h[t],
 *                                        W'_b[n, 64 h + i] = sum_c W_O[n, 64 h + c] S_bh[i, c],
 * so a block runs the state pass, forms the per-image weights W'_b (bf16) and the scaled
 * queries A' (bf16) and multiplies them in the projection's GEMM (bias and residual as before);
 * the attention output itself is never written.  The block is unchanged as a function; the
 * roundings differ (S enters through W'_b rounded to bf16 instead of as a high + low bf16 pair).
 * Applies to blocks with 64-channel heads, the ReLU map and no convolution branch, with
 * separate LayerNorm passes, on images of a multiple of 256 tokens (prefix tokens included);
 * every other block runs as without the option.  enable != 0 switches it on, 0 off; afterwards
 * jv_encoder_workspace_bytes also asks for the summed states and [batch][width][width] bf16.
 * Host-only call: nothing is launched.  Returns JV_ERR_INVALID_ARG for a null encoder.
 * ------------------------------------------------------------------------- */
jv_status jv_encoder_fuse_linear_projection(jv_encoder *enc, int32_t enable);
jv_status jv_encoder_forward(const jv_encoder *enc, const void *x, void *y, int32_t batch,
                             int32_t grid_h, int32_t grid_w, void *workspace,
                             size_t workspace_bytes, void *hip_stream);
jv_status jv_encoder_forward_taps(const jv_encoder *enc, const void *x, void *y, int32_t batch,
                                  int32_t grid_h, int32_t grid_w, int32_t n_taps,
                                  const int32_t *tap_blocks, void *const *tap_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);
void jv_encoder_destroy(jv_encoder *enc);

#ifdef __cplusplus
}
#endif
#endif /* JETVIT_H */
