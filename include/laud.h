/*
 * laud.h -- C ABI of the MI355X (gfx950) dynamic-bottleneck library.
 *
 * The library implements the inference hot path of the LAUDNet block (Sec. 3.1-3.2,
 * Fig. 2): a spatial masker scores coarse S x S patches, the active patches are turned
 * into an index list, and the residual bottleneck (1x1 -> 3x3 -> 1x1) is evaluated on
 * those patches only and added back into the feature map in place of the skip value.
 * Channel skipping and layer skipping (Sec. 3.1) use the same compaction machinery.
 *
 * Conventions that hold for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never
 *     allocates, frees or keeps them.  Scratch memory is a caller-owned device workspace
 *     sized with laud_workspace_size(); its contents are undefined between calls.
 *   - Feature maps are dense NHWC: element (n,y,x,c) at ((n*H + y)*W + x)*C + c.  One
 *     pixel's channel vector is contiguous.  dtype is LAUD_F32 or LAUD_BF16; C, c_in,
 *     c_mid and c_out must be multiples of 8 and every tensor base 16-byte aligned.
 *     One feature map or scratch activation (N*H*W*max(c_in, c_mid) elements) has to stay
 *     below 2 GiB (the kernels address an operand with 32-bit byte offsets); larger
 *     shapes return LAUD_ERR_UNSUPPORTED.
 *   - Weights have the feature map's dtype: w1 [c_mid][c_in], w2 [c_mid][3][3][c_mid]
 *     (out, ky, kx, in; stride 1, zero padding 1, cross-correlation), w3 [c_out][c_mid].
 *     The per-channel affine (folded BN, Sec. 3.4) is float32: s1,t1,s2,t2 [c_mid],
 *     s3,t3 [c_out].  Accumulation, affine and the residual add are float32; h1, h2 and
 *     the output are rounded (nearest-even) to dtype.
 *   - Patch p of an H x W map with granularity S (S divides H and W; Hp = H/S, Wp = W/S)
 *     has flat index (n*Hp + py)*Wp + px and covers pixels [py*S, py*S+S) x [px*S, px*S+S).
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and never synchronises.  Data-dependent counts stay on the device.
 *   - Return value: LAUD_OK or a negative laud_status.  Arguments are validated on the
 *     host before anything is launched; on error nothing has been launched.
 *   - Threads: entry points may be called from several host threads at once as long as the calls
 *     use different workspaces (and, for in-place calls, different feature maps).  The library
 *     keeps no state between calls except (a) idempotent per-kernel launch attributes, requested on a
 *     kernel's first launch per device or all at once by laud_init(); (b) the optional stage-timing
 *     collector (laud_stage_timing_*), which is NOT re-entrant; (c) the fixed scratch array of
 *     laud_dyn_bottleneck_noalloc, shared by all calls on one GPU.  No environment variable is read.
 */
#ifndef LAUD_H
#define LAUD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LAUD_OK = 0,
  LAUD_ERR_INVALID_ARG = -1, /* null pointer, non-positive dim, S not dividing H/W, D not dividing c_mid */
  LAUD_ERR_UNSUPPORTED = -2, /* dtype/shape outside what the kernels cover (e.g. channels % 8 != 0) */
  LAUD_ERR_WORKSPACE = -3,   /* workspace missing or smaller than laud_workspace_size() */
  LAUD_ERR_HIP = -4,         /* a HIP launch failed */
  LAUD_ERR_SCRATCH_LIMIT = -5 /* laud_dyn_bottleneck_noalloc: the shapes need more scratch memory than the
                                 library's fixed LAUD_NOALLOC_SCRATCH_BYTES; use laud_dyn_bottleneck */
} laud_status;

typedef enum { LAUD_F32 = 0, LAUD_BF16 = 1 } laud_dtype;

typedef enum {
  LAUD_OP_MASK_GEN = 0,
  LAUD_OP_COMPACT = 1,
  LAUD_OP_GATHER = 2,
  LAUD_OP_DYN_BOTTLENECK = 3,
  LAUD_OP_CHANNEL_SKIP = 4
} laud_op;

/* Shape of a dense NHWC feature map. */
typedef struct {
  int32_t N, H, W, C;
  int32_t dtype; /* laud_dtype */
} laud_fmap;

/* Folded parameters of one residual bottleneck (Fig. 2(a); Sec. 3.4). Device pointers. */
typedef struct {
  int32_t c_in, c_mid, c_out; /* c_out must equal c_in (identity shortcut) */
  const void* w1;
  const void* w2;
  const void* w3;
  const float* s1;
  const float* t1;
  const float* s2;
  const float* t2;
  const float* s3;
  const float* t3;
  int32_t relu_out; /* non-zero: ReLU after the residual add, on computed pixels only */
  const void* packed; /* NULL, or the block's weights re-ordered once by laud_pack_weights() (device memory of
                         laud_packed_weights_size() bytes).  With it no call spends time re-ordering weights; without
                         it the entry points do the same re-ordering themselves on every call, into their workspace.
                         It must be re-made whenever w1 / w2 / w3 change. */
} laud_bottleneck;

/* Human-readable name of a status code (static storage). */
const char* laud_status_string(int status);

/* Library ABI version (increments when a signature changes). */
int laud_abi_version(void);

/*
 * Optional one-time set-up for the CURRENT device: requests the launch attributes of every kernel (large
 * dynamic LDS) and resolves the device address of the allocation-free entry point's scratch array, so that
 * no first call has to do it -- e.g. inside a stream capture.  Allocates nothing, launches nothing; may be
 * called again (per device, from any thread).  Entry points work without it.
 */
int laud_init(void);

/*
 * Weights in the order the MFMA kernels stream them (a data layout, no arithmetic: every 16-byte piece of w1, w2, w3
 * is copied to the place where the lane that multiplies it will read it, so that a wave loads 1 KB in a row straight
 * into registers).  Made once per block -- e.g. when a model is loaded -- and handed over in laud_bottleneck.packed.
 * laud_packed_weights_size returns 0 for shapes / dtypes whose kernels read the plain layout (then packed stays
 * NULL).  p->packed itself is ignored by both calls.
 */
size_t laud_packed_weights_size(const laud_bottleneck* p, int dtype);
int laud_pack_weights(const laud_bottleneck* p, int dtype, void* packed, void* stream);

/*
 * Workspace bytes an entry point needs for the given shapes.  `op` is a laud_op; `p` may be
 * NULL for ops that take no bottleneck; `S_or_D` is the spatial granularity S (mask-gen,
 * gather, dyn-bottleneck), the element count n (compact) or the number of channel groups D
 * (channel-skip).  Returns 0 for invalid arguments.
 */
size_t laud_workspace_size(int op, laud_fmap fx, const laud_bottleneck* p, int S_or_D);

/*
 * Spatial masker + index generation (Sec. 3.2 "Masker design"; App. B, operator fusion
 * items 1-2).  For every patch:  logit = bias + sum_c w[c] * mean over the S x S patch of
 * x[...,c]  (the one-channel form W_0 - W_1 of the two-logit masker), mask = logit > 0
 * (strict; 0 and NaN are inactive), optionally AND-ed with a per-sample layer gate.  Then
 * the ascending list of active flat patch indices and its length are produced.
 *   x        [N,H,W,C] dtype                      in
 *   w        [C] float32                          in
 *   keep     [N] bytes or NULL: sample n's patches are all inactive when keep[n] == 0
 *   mask     [N*Hp*Wp] bytes (0/1)                out
 *   idx      [N*Hp*Wp] int32, first *count valid  out
 *   count    [1] int32                            out
 *   sample_offsets [N+1] int32 or NULL: number of active patches before sample n  out
 *   logits   [N*Hp*Wp] float32 or NULL            out
 */
int laud_mask_gen(const void* x, laud_fmap fx, int S, const float* w, float bias,
                  const uint8_t* keep, uint8_t* mask, int32_t* idx, int32_t* count,
                  int32_t* sample_offsets, float* logits,
                  void* ws, size_t ws_bytes, void* stream);

/*
 * Stable compaction of a byte mask (Sec. 3.1 layer gates; App. B item 2 for patch masks
 * supplied from outside): idx = ascending positions i in [0,n) with keep[i] != 0,
 * *count = their number.  idx has capacity n.  n == 0 writes *count = 0.
 */
int laud_layer_skip_compact(const uint8_t* keep, int n, int32_t* idx, int32_t* count,
                            void* ws, size_t ws_bytes, void* stream);

/*
 * Stand-alone gather (Sec. 3.1, step 1 of the three-step schedule): for p < *count,
 * out[p][dy][dx][:] = x[n][py*S - halo + dy][px*S - halo + dx][:] if that pixel is inside
 * the image, else 0, with (n,py,px) decoded from idx[p]; halo is 0 or 1 (1 = the
 * neighbours a 3x3 kernel needs).  out is [cap][S+2*halo][S+2*halo][C] dtype with
 * cap >= *count (N*Hp*Wp always suffices); entries p >= *count are not written.
 */
int laud_gather_patches(const void* x, laud_fmap fx, int S, int halo,
                        const int32_t* idx, const int32_t* count, void* out, void* stream);

/*
 * Spatially adaptive bottleneck (Fig. 2(b); Sec. 3.4; App. B items 2-3).  For every pixel of
 * an active patch:  out = act(x + s3*conv1x1(h2;w3) + t3),  h2 = relu(s2*conv3x3(h1;w2) + t2),
 * h1 = relu(s1*conv1x1(x;w1) + t1) evaluated from the true x on the patch and its one-pixel
 * halo, with h1 := 0 outside the image (the padding is the 3x3's).  Pixels of inactive
 * patches: out == x bit for bit.  act = ReLU iff p->relu_out.
 *   idx/count  ascending active patch indices and their number (device), as produced by
 *              laud_mask_gen or laud_layer_skip_compact; with S == H == W the indices are
 *              sample ids and the call is layer skipping.
 *   out        [N,H,W,C]; may be the same pointer as x (in place, the scatter-add of
 *              App. B item 3); partial overlap is not allowed.
 */
int laud_dyn_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p, int S,
                        const int32_t* idx, const int32_t* count, void* out,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * laud_dyn_bottleneck for callers that cannot allocate or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results; the scratch activations (dilated pixel list, h1, h2) live in a fixed array of
 * LAUD_NOALLOC_SCRATCH_BYTES in the library's device image (one copy per GPU, held until the process ends)
 * instead of a caller workspace.  The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine).  Shapes whose laud_workspace_size(LAUD_OP_DYN_BOTTLENECK, ...) exceeds LAUD_NOALLOC_SCRATCH_BYTES
 * return LAUD_ERR_SCRATCH_LIMIT (e.g. one 56 x 56 x 256 float32 image with c_mid 64 needs 1.6 MB; batch 8 of the
 * bf16 stage-3 map 14 x 14 x 1024 with c_mid 256 needs 1.6 MB).  All calls on one GPU share the array, which keeps
 * the last call's contents: calls that overlap in time on one GPU (different streams or threads) race and must
 * be serialised by the caller; nothing in it needs clearing between calls.
 */
#define LAUD_NOALLOC_SCRATCH_BYTES (16u << 20)
int laud_dyn_bottleneck_noalloc(const void* x, laud_fmap fx, const laud_bottleneck* p, int S,
                                const int32_t* idx, const int32_t* count, void* out, void* stream);

/* What a group-convolution / squeeze-and-excitation bottleneck adds to laud_bottleneck (the RegNetY
 * backbones of Sec. 4; Sec. 3.2 states that the dynamic block carries over to group convolutions). */
typedef struct {
  int32_t group_width; /* g: channels per group of the 3x3 (as many in as out); divides c_mid; 8, 16, 32 or 64.
                          The block's w2 is then [c_mid][3][3][g]: output channel o reads the input channels
                          (o/g)*g .. (o/g)*g + g-1. */
  int32_t se_width;    /* hidden width of the SE module, <= 1024; 0 = no SE module (pointers below unused) */
  const float* w_se1;  /* [se_width][c_mid] float32, device */
  const float* b_se1;  /* [se_width] */
  const float* w_se2;  /* [c_mid][se_width] */
  const float* b_se2;  /* [c_mid] */
} laud_group_se;

/*
 * Spatially adaptive bottleneck whose 3x3 is a group convolution, with an optional squeeze-and-excitation
 * module between the 3x3 (after its affine and ReLU) and the last 1x1 (Sec. 4, RegNetY; Fig. 2(b) otherwise).
 * Everything is as in laud_dyn_bottleneck except
 *   h2 = relu(s2*groupconv3x3(h1;w2) + t2),
 *   gate[n][c] = sigmoid(w_se2 * relu(w_se1 * z[n] + b_se1) + b_se2),  z[n] = mean of h2 over the ACTIVE
 *   pixels of sample n (the paper does not say what the squeeze averages over when only some locations are
 *   computed; with every patch active, and for layer skipping with S == H == W, this is the ordinary
 *   global average),
 *   out = act(x + s3*conv1x1(h2 * gate[n]; w3) + t3) on active pixels.
 * h2 * gate is rounded to dtype before the last 1x1 (c_mid <= 4096 and N <= 65535 when se_width > 0).  Workspace:
 * laud_workspace_size(LAUD_OP_DYN_BOTTLENECK, ...).  Errors as laud_dyn_bottleneck; a group width other
 * than 8/16/32/64 returns LAUD_ERR_UNSUPPORTED, a null `e` or one that does not divide c_mid
 * LAUD_ERR_INVALID_ARG.
 */
int laud_dyn_group_se_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p,
                                 const laud_group_se* e, int S, const int32_t* idx, const int32_t* count,
                                 void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * The same block with the masker fused into the first 1x1 (Sec. 3.4 "Operator fusion for spatial
 * maskers"; App. B item 1): conv1 is evaluated on EVERY pixel (spatially static) and the masker's
 * per-pixel projection sum_c w[c]*x[n,y,x,c] is accumulated from the same reads of x; the
 * projection is pooled over S x S patches, thresholded and turned into the index list, and conv2 /
 * conv3 + scatter-add run on the active patches as in laud_dyn_bottleneck.  One call replaces
 * laud_mask_gen followed by laud_dyn_bottleneck and produces the same mask / idx / count /
 * sample_offsets / logits outputs (same meaning, same optional NULLs) and the same `out`; logits
 * differ from laud_mask_gen's only in float32 summation order.  It pays off when the dilated
 * activation ratio is close to 1 (small S); c_in <= 4096.  Workspace: as LAUD_OP_DYN_BOTTLENECK.
 * With a layer gate (`keep`) and logits == NULL the first 1x1 and the projection are evaluated on the kept samples
 * only (the gates are compacted first); with logits wanted they cover every sample, gated ones included.
 */
int laud_masker_dyn_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p, int S,
                               const float* w, float bias, const uint8_t* keep,
                               uint8_t* mask, int32_t* idx, int32_t* count,
                               int32_t* sample_offsets, float* logits, void* out,
                               void* ws, size_t ws_bytes, void* stream);

/*
 * The UNFUSED three-step schedule of Sec. 3.1 (gather, compute, scatter), kept as the baseline of
 * the operator-fusion ablation (Tab. 1): a stand-alone gather of the active patches with their halo
 * into a dense buffer, the three convolutions on that buffer (conv1 on all (S+2)^2 gathered
 * positions, with h1 := 0 at positions outside the image; the 3x3 inside the gathered tile; the last
 * 1x1 into a dense float32 buffer), and a stand-alone scatter that adds the residual.
 * Same arguments and same result as laud_dyn_bottleneck.  Workspace:
 * laud_dyn_bottleneck_unfused_workspace(fx, p, S) bytes.
 */
size_t laud_dyn_bottleneck_unfused_workspace(laud_fmap fx, const laud_bottleneck* p, int S);
int laud_dyn_bottleneck_unfused(const void* x, laud_fmap fx, const laud_bottleneck* p, int S,
                                const int32_t* idx, const int32_t* count, void* out,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * Channel-skipping bottleneck (Fig. 2(c); Sec. 3.1-3.2).  cmask is [N][D] bytes; group g of
 * sample n covers mid channels [g*G, (g+1)*G), G = c_mid / D.  The mask multiplies the input
 * and the output of the 3x3 conv.  Two schedules, same result: in general the kept-channel weight
 * gather is fused into the three convs and dropped channels are never computed (one set of tiles per
 * sample); for bf16 blocks with c_mid = 256, c_out = 1024, groups of whole 64-channel slices (D <= 4),
 * square maps and N <= 4096 the samples are ordered by mask pattern, the first 1x1 stores zeros in the
 * dropped groups of h1, and the fused 3x3 -> last 1x1 kernel skips every 64-channel input slice that no
 * row of a tile keeps and stores zeros in the dropped groups of h2 (p->packed is used when given).
 * out = act(x + s3*conv1x1(h2 masked; w3) + t3) on every pixel; with all groups dropped
 * out = act(x + t3).  out may be the same pointer as x.  Workspace: LAUD_OP_CHANNEL_SKIP.
 */
int laud_channel_skip_conv(const void* x, laud_fmap fx, const laud_bottleneck* p,
                           const uint8_t* cmask, int D, void* out,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * Static parts of the ResNet body (always executed, no mask).  The paper's
 * formulation assumes stride 1 inside dynamic blocks (Sec. 3.1); the first block of every stage
 * (projection shortcut, stride 2 in stages 2-4, placed on the 3x3 as in the torchvision models the
 * paper starts from) and the stem run as ordinary dense layers.
 *
 * laud_static_bottleneck: out = relu(s3*conv1x1(h2;w3)+t3 + s_sc*conv1x1_stride(x;w_sc)+t_sc), with
 * h1 = relu(affine1(conv1x1(x;w1))), h2 = relu(affine2(conv3x3 stride, pad 1 (h1;w2))).  x is
 * [N,H,W,c_in]; out is [N,Ho,Wo,c_out] with Ho = (H-1)/stride + 1 (stride 1 or 2) and must not alias x;
 * w_sc is [c_out][c_in] in x's dtype, s_sc/t_sc float32 [c_out]; p->c_out may differ from p->c_in.
 *
 * laud_stem: x [N,Hin,Win,3] dtype; 7x7 stride-2 pad-3 conv with w7 [c_out][7][7][3] (dtype),
 * affine s,t (float32), ReLU, then 3x3 stride-2 pad-1 max pooling; out [N,Hp,Wp,c_out] with
 * Hc = (Hin-1)/2 + 1, Hp = (Hc-1)/2 + 1; c_out a multiple of 8.
 *
 * laud_stem3x3 (the stem of the RegNet backbones, Sec. 4): x [N,Hin,Win,3] dtype; 3x3 stride-2 pad-1 conv with
 * w3 [c_out][3][3][3] (dtype), affine s,t (float32), ReLU, no pooling; out [N,Ho,Wo,c_out], Ho = (Hin-1)/2 + 1;
 * c_out a multiple of 8, at most 256.  No workspace.
 */
size_t laud_static_bottleneck_workspace(laud_fmap fx, const laud_bottleneck* p, int stride);
int laud_static_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p, const void* w_sc,
                           const float* s_sc, const float* t_sc, int stride, void* out,
                           void* ws, size_t ws_bytes, void* stream);
size_t laud_stem_workspace(int N, int Hin, int Win, int c_out, int dtype);
int laud_stem3x3(const void* x, int N, int Hin, int Win, int dtype, const void* w3, const float* s,
                 const float* t, int c_out, void* out, void* stream);
int laud_stem(const void* x, int N, int Hin, int Win, int dtype, const void* w7, const float* s,
              const float* t, int c_out, void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * Dynamic first block of a stage (Sec. 3.1: the mask decides at which OUTPUT locations the
 * convolutions run; locations that are not selected take the value of the skip connection, which in
 * this block is the strided 1x1 projection):
 *   out = act(s_sc*conv1x1_stride(x;w_sc)+t_sc + M * (s3*conv1x1(h2;w3)+t3)),
 * h1, h2 as in laud_static_bottleneck.  The mask lives on the output grid [N,Ho,Wo], Ho = (H-1)/stride+1,
 * in patches of S x S output pixels (S divides Ho and Wo); idx/count are the ascending list of active
 * patch indices (n*Hp + py)*Wp + px on that grid and its length, both device memory, e.g. from
 * laud_mask_gen called on x with granularity stride*S (adaptive pooling of x to the output patch grid,
 * Sec. 3.2) or from laud_layer_skip_compact.  conv1 runs only on the input pixels under the 3x3 windows
 * of active output pixels, conv2/conv3 only on active output pixels; the shortcut runs everywhere.
 * x [N,H,W,c_in], out [N,Ho,Wo,c_out] (must not alias x), stride 1 or 2, act = ReLU iff p->relu_out.
 * Errors as laud_static_bottleneck; LAUD_ERR_INVALID_ARG if S does not divide the output size.
 */
size_t laud_dyn_projection_workspace(laud_fmap fx, const laud_bottleneck* p, int stride);
int laud_dyn_projection_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p,
                                   const void* w_sc, const float* s_sc, const float* t_sc, int stride,
                                   int S, const int32_t* idx, const int32_t* count, void* out,
                                   void* ws, size_t ws_bytes, void* stream);

/*
 * The same first block for the group-convolution / SE backbones (Sec. 4, RegNetY): the stride sits on the group
 * 3x3 (w2 [c_mid][3][3][g]), and the SE gate (see laud_dyn_group_se_bottleneck) is taken over the sample's active
 * OUTPUT pixels.  With every patch of the output grid in the index list this is the static first block of a
 * stage.  Arguments, workspace (laud_dyn_projection_workspace) and errors as laud_dyn_projection_bottleneck and
 * laud_dyn_group_se_bottleneck.
 */
int laud_dyn_group_se_projection_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p,
                                            const laud_group_se* e, const void* w_sc, const float* s_sc,
                                            const float* t_sc, int stride, int S, const int32_t* idx,
                                            const int32_t* count, void* out, void* ws, size_t ws_bytes,
                                            void* stream);


/*
 * Channel masker (Sec. 3.2 "Masker design"; Fig. 3(b)): g = mean of x over H x W per sample and
 * channel; h = relu(wa*g + ba) (the paper does not name the non-linearity; ReLU is assumed);
 * l = wb*h + bb, 2D logits viewed row-major as [D][2]; group d is kept iff l[d][0] > l[d][1]
 * (strict; NaN drops the group).  The paper sets hidden = max(floor(D/16), 16); any positive
 * width is accepted.  All weights float32 device arrays: wa [hidden][C], ba [hidden],
 * wb [2*D][hidden], bb [2*D].  Outputs: cmask [N][D] bytes (the input of laud_channel_skip_conv),
 * logits2 [N][2*D] float32 or NULL.  Workspace: laud_channel_masker_workspace(fx) bytes.
 */
size_t laud_channel_masker_workspace(laud_fmap fx);
int laud_channel_masker(const void* x, laud_fmap fx, const float* wa, const float* ba, int hidden,
                        const float* wb, const float* bb, int D, uint8_t* cmask, float* logits2,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Instrumentation (host side; not part of the paper's method): per-stage GPU time of the
 * kernels the entry points launch.  While enabled, every stage is bracketed by a pair of HIP
 * events recorded on the call's stream (at most 65536 stage launches are kept per collection;
 * later ones are dropped).  laud_stage_timing_enable(1) clears what was collected and starts,
 * (0) stops.  laud_stage_timing_read() waits for the recorded events, adds up the elapsed
 * milliseconds and launch counts per stage into two HOST arrays of LAUD_STAGE_COUNT entries,
 * and clears the collection.  Not thread-safe against concurrent entry-point calls.
 */
typedef enum {
  LAUD_STAGE_MASK_LOGITS = 0, /* pooled masker + threshold */
  LAUD_STAGE_COMPACT = 1,     /* ordered index generation */
  LAUD_STAGE_GATHER = 2,      /* stand-alone gather */
  LAUD_STAGE_COPY_INACTIVE = 3,
  LAUD_STAGE_NEED = 4,        /* dilated active pixel list for conv1 */
  LAUD_STAGE_CONV1 = 5,
  LAUD_STAGE_CONV2 = 6,
  LAUD_STAGE_CONV3 = 7,
  LAUD_STAGE_CS1 = 8,
  LAUD_STAGE_CS2 = 9,
  LAUD_STAGE_CS3 = 10,
  LAUD_STAGE_SCATTER = 11,    /* stand-alone scatter + residual add (unfused schedule) */
  LAUD_STAGE_SE = 12,         /* squeeze-and-excitation gate + rescale (group-conv / SE blocks) */
  LAUD_STAGE_COUNT = 13
} laud_stage;
int laud_stage_timing_enable(int on);
int laud_stage_timing_read(double* total_ms, int64_t* launches);
const char* laud_stage_name(int stage);

/*
 * Achievable-peak probes (measurement aids, not part of the paper's method): the denominators a roofline fraction
 * can be read against besides the published peaks.  laud_probe_mfma launches `blocks` workgroups of 8 waves that
 * each issue 4*iters MFMAs (32x32x16 bf16, or the same FLOPs as 32x32x2 float32 steps) on register operands and
 * stores the FLOPs of the launch in *flops (host, may be NULL); sink is a device word nobody reads.
 * laud_probe_copy copies `bytes` (a multiple of 16, both pointers 16-byte aligned) with a plain grid-stride kernel;
 * laud_probe_read only reads them (sink: at least 16 device words nobody reads).
 * All only enqueue on `stream`; the caller times them with events.
 */
int laud_probe_mfma(int dtype, int iters, int blocks, double* flops, float* sink, void* stream);
int laud_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
int laud_probe_read(const void* src, size_t bytes, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LAUD_H */
