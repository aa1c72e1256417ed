/*
 * adadim.h - C ABI of the MI355X (gfx950) AdaDim layer-search library.
 *
 * AdaDim (paper Sec. 3.3, Eq. 1; procedure `rtn_ada` in App. B) decides, for
 * one linear layer, whether group-wise b-bit round-to-nearest quantization
 * should form its groups inside each output channel (per-OC) or inside each
 * input channel (per-IC, Sec. 3.2): it quantizes the weight both ways, scores
 * each by the output reconstruction error on calibration activations and
 * keeps the lower one.  This library is that search on one GPU.
 *
 * Conventions shared by every call
 *   - W is the layer weight, fp16, row-major [out, in] (torch.nn.Linear
 *     layout); X are calibration activations, fp16, row-major [tokens, in],
 *     so the layer output is X W^T (Eq. 1 writes the same product as W X).
 *   - Every data pointer is a DEVICE pointer owned by the caller unless the
 *     argument is documented as a host pointer.  The library never frees or
 *     keeps caller memory.  Internal scratch lives in the context.
 *   - Calls are asynchronous on the context's HIP stream; results are ready
 *     when that stream has caught up.  Three things wait for the stream:
 *     adadim_select with a host output; adadim_profile_read; and any call
 *     that finds one of the context's scratch buffers too small (it waits for
 *     the kernels that may still read the old buffer, frees it and allocates
 *     a larger one: the first call of a shape, never a repeat of it).
 *     adadim_layer_error_batch_select_noalloc has no scratch to grow.
 *   - Return value: ADADIM_OK or a negative ADADIM_E* code; the library does
 *     not throw or abort.  Arguments are validated before any device work, so
 *     a rejected call has touched nothing.  adadim_last_error gives a text.
 *   - Inf/NaN in W or X give undefined numbers, not an error.
 *   - A context may be used from one host thread at a time.
 */
#ifndef ADADIM_H
#define ADADIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADADIM_OK       0
#define ADADIM_EINVAL  (-1)  /* bad dim/bits/group/clip/shape/leading dimension */
#define ADADIM_ENULL   (-2)  /* a required pointer is NULL */
#define ADADIM_EALIGN  (-3)  /* a pointer or row pitch is not aligned as documented */
#define ADADIM_EHIP    (-4)  /* a HIP runtime call failed; see adadim_last_error */

#define ADADIM_DIM_OC 0      /* groups of `group` consecutive input channels inside an output row */
#define ADADIM_DIM_IC 1      /* groups of `group` consecutive output channels inside an input column */

#define ADADIM_DW_F32        0  /* dW written / read as fp32 */
#define ADADIM_DW_F16        1  /* dW written / read as fp16 (round to nearest even) */
#define ADADIM_DW_F16_SCALED 2  /* fp16 of dW[o,j] * colscale[j] in the scoring layout (see below) */

/*
 * Scoring layout.  The two fp16 operands of the error GEMM, the column-scaled dW
 * (ADADIM_DW_F16_SCALED) and the prepared Hs, are consumed 32 contraction elements at a
 * time from 256 consecutive rows.  When `in` is a multiple of 32 an [rows, in] operand is
 * therefore stored as [row tile of 256][column block of 32][256 rows][32 columns]: element
 * (r, c) at index (((r / 256) * (in / 32) + c / 32) * 256 + r % 256) * 32 + c % 32, the last
 * row tile padded to 256 rows (the padding is never read or written); otherwise plain
 * row-major (r * in + c).  adadim_score_elems gives the number of elements such a buffer
 * must hold: round_up(rows, 256) * in, or rows * in for the row-major form.
 */
int64_t adadim_score_elems(int64_t rows, int64_t cols);

typedef struct adadim_ctx adadim_ctx;

/* Creates a context bound to `hip_stream` (a hipStream_t passed as void*, NULL
 * = the default stream) on the device that is current at the time of the first
 * compute call.  Performs no device work itself.  *out receives the context. */
int adadim_create(adadim_ctx** out, void* hip_stream);

/* Frees the context and its device scratch.  NULL is allowed. */
void adadim_destroy(adadim_ctx* ctx);

/* Text for the last error recorded on this context (ctx == NULL: the text of
 * the last error of a failed adadim_create).  Owned by the library. */
const char* adadim_last_error(const adadim_ctx* ctx);

/* Library version string, e.g. "adadim-gfx950 0.3". Host pointer, static. */
const char* adadim_version(void);

/*
 * H (+)= X^T X, the Gram matrix that turns Eq. 1 into a quadratic form:
 * ||X W^T - X Q(W)^T||_F^2 = tr(dW H dW^T), dW = W - Q(W).
 *   X      fp16 [tokens, in], row pitch ldx >= in elements; X and ldx*2 must be
 *          16-byte aligned (EALIGN), in a multiple of 8.
 *   H      fp32 [in, in], full symmetric storage, 16-byte aligned.
 *   accumulate  0: H is overwritten; 1: the product is added to H, so a long
 *          calibration set can be fed in token chunks.
 * Products are exact (fp16 x fp16), sums are fp32 on the matrix cores.
 * tokens == 0 with accumulate == 0 zeroes H.
 */
int adadim_hessian(adadim_ctx* ctx, const void* X, int64_t tokens, int64_t in, int64_t ldx,
                   float* H, int accumulate);

/*
 * Group-wise asymmetric round-to-nearest quantization of W (Sec. 2.1: groups
 * of consecutive weights inside a channel share parameters; Sec. 3.2: the
 * channel is an output row for per-OC and an input column for per-IC; Sec. 4.1:
 * uniform asymmetric).  Per group, in fp32 with one rounding per operation:
 *     mx = clip*max(max w, 0)   mn = clip*min(min w, 0)
 *     scale = (mx-mn)/qmax, or 1 if mx == mn        qmax = 2^bits - 1
 *     zero  = clamp(rint(-mn/scale), 0, qmax)
 *     code  = clamp(rint(w/scale) + zero, 0, qmax)   (rint: ties to even)
 *     What  = scale*(code-zero)                      dW = w - What
 *   W      fp16 [out, in] contiguous, 16-byte aligned if in is a multiple of 8.
 *   dim    ADADIM_DIM_OC or ADADIM_DIM_IC.   bits in [2, 8].
 *   group  > 0 and dividing `in` (OC) / `out` (IC); 0 = the whole channel.
 *   clip   in (0, 1]; 1 is the paper's plain min/max range.
 * Outputs, each optional (NULL skips it):
 *   codes  u8  [out, in]
 *   scales f32 [out, in/g] (OC) or [out/g, in] (IC)
 *   zeros  u8  same shape as scales
 *   dW     [out, in] in the type named by dW_dtype.  ADADIM_DW_F16_SCALED
 *          multiplies column j by colscale[j] before the fp16 rounding and
 *          stores the result in the scoring layout (adadim_score_elems(out, in)
 *          elements).  colscale is fp32 [in] and must hold powers of two, as
 *          adadim_hessian_prepare writes them (the kernels fold the factor into
 *          the scale, which is exact only then); it must be non-NULL for this
 *          dtype and is ignored otherwise.
 *   packed u32 bitstream of the codes of each channel (row for OC, column for
 *          IC): code k of the channel at bits [k*bits, (k+1)*bits) of the
 *          channel's stream, little-endian 32-bit words, each channel padded
 *          to a whole word: [channels, ceil(len*bits/32)].
 */
int adadim_quantize(adadim_ctx* ctx, const void* W, int64_t out, int64_t in,
                    int dim, int bits, int group, float clip,
                    uint8_t* codes, float* scales, uint8_t* zeros,
                    void* dW, int dW_dtype, const float* colscale,
                    uint32_t* packed);

/*
 * The same quantizer writing the storage format of b + 16/g bits per weight, the figure the
 * paper counts with (Sec. 4.1: INT3/INT4 with groups of 128; "Avg Bits" of App. C: 4.125 for
 * b = 4, g = 128): the packed codes plus ONE 16-bit word per group.  The paper does not say
 * how scale and zero-point share the sixteen bits; here
 *     word = pattern << bits | zero
 *     pattern = the leading 16-bits bits of the 15-bit fp16 pattern of the scale (sign 0), i.e.
 *               an unsigned float with fp16's exponent and 11-bits fraction bits;
 *               scale = fp16(pattern << (bits-1)).
 * The fp32 scale of adadim_quantize is rounded to fp16 (nearest even), then to the nearest
 * pattern (ties to the even pattern; a pattern of 0 becomes 1), and zero, code, What and dW
 * are computed from the rounded scale with the formulas above: what is stored de-quantizes
 * to exactly the weights that dW (and so the search) saw.
 *   bits   2, 3 or 4.
 *   meta   u16, shape of `scales` above: [out, in/g] (OC) or [out/g, in] (IC); optional.
 * Everything else as in adadim_quantize.
 */
int adadim_quantize_meta16(adadim_ctx* ctx, const void* W, int64_t out, int64_t in,
                           int dim, int bits, int group, float clip,
                           uint8_t* codes, uint16_t* meta,
                           void* dW, int dW_dtype, const float* colscale,
                           uint32_t* packed);

/*
 * Both candidates of the search in one call: adadim_quantize(dim = OC) and adadim_quantize(dim = IC) of the same
 * W with the same bits, group and clip, each with its own outputs (any of them NULL to skip it), dW always as
 * ADADIM_DW_F16_SCALED.  meta16 = 1: the storage format of adadim_quantize_meta16 (scales_* are then u16 arrays
 * of group words and zeros_* are not written).  Same results as the two calls.  When both fast kernels take the
 * shape (groups of 32, 64 or 128 dividing both out and in, in a multiple of 32, both dW given, 2..4 bits if a
 * packed stream is asked for, then for both) it is one launch, which on a 4096 x 4096 layer costs what 1.6 of
 * the single launches cost; otherwise the two launches one after the other.
 */
int adadim_quantize_both(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int bits, int group, float clip,
                         int meta16, const float* colscale,
                         uint8_t* codes_oc, void* scales_oc, uint8_t* zeros_oc, void* dW_oc, uint32_t* packed_oc,
                         uint8_t* codes_ic, void* scales_ic, uint8_t* zeros_ic, void* dW_ic, uint32_t* packed_ic);

/*
 * Prepares H for scoring on the matrix cores.  With the power-of-two column
 * scales d_j = 2^(round(log2(H_jj)/2) - 6), i.e. about sqrt(H_jj)/64 (1 where H_jj <= 0):
 *   Hs     fp16 [in, in] in the scoring layout (adadim_score_elems(in, in) elements):
 *          Hs[n,k] = H[n,k]/(d_n d_k) for k < n, 0 elsewhere
 *   hmeta  f32  [2, in]:  hmeta[0,j] = d_j (the colscale of adadim_quantize),
 *                         hmeta[1,j] = H_jj
 * so that tr(dW H dW^T) = sum_o ( sum_j H_jj dW_oj^2 + 2 sum_{k<n} dW'_ok Hs_nk dW'_on ),
 * dW'_oj = dW_oj d_j.  The scaling keeps |Hs| <= 2^13 whatever the activation
 * outliers are.  Hs 16-byte aligned; in a multiple of 8.
 * Range: dW' is fp16, so a candidate is scored accurately while |dW_oj| sqrt(H_jj) lies
 * between 4e-3 and 4e6 for the entries that matter (an entry's share of the loss is about
 * that number squared).  With N(0, 0.02^2) weights, 65536 tokens and x100 outlier channels
 * the largest products are near 3e2 and the ordinary columns' near 1: activations 2^13 times
 * larger (fp16 cannot hold them) or 2^8 times smaller stay inside.  Beyond the upper end dW'
 * becomes inf and the loss inf or NaN, which never wins the selection (adadim_select); beyond
 * the lower end small entries are rounded to fp16 subnormals or zero and the loss reads low.
 */
int adadim_hessian_prepare(adadim_ctx* ctx, const float* H, int64_t in, void* Hs, float* hmeta);

/*
 * adadim_hessian (accumulate = 0) and adadim_hessian_prepare in one call: the pass that adds up the Gram
 * matrix's token-split partial tiles also writes Hs and hmeta for those tiles, and the tiles that were formed
 * whole get theirs from one read of their block of H, not of the full matrix.  Same outputs, bit for
 * bit, as the two calls one after the other.  For a calibration set fed in chunks use adadim_hessian with
 * accumulate = 1 and adadim_hessian_prepare after the last chunk.
 */
int adadim_hessian_prepared(adadim_ctx* ctx, const void* X, int64_t tokens, int64_t in, int64_t ldx,
                            float* H, void* Hs, float* hmeta);

/*
 * Reconstruction error of one candidate (Eq. 1, squared):
 *   loss = tr(dW H dW^T) = ||X dW^T||_F^2,   loss_rows[o] = dW_o H dW_o^T.
 *   dW        [out, in] of type dW_dtype (F32 or F16; not F16_SCALED).
 *   H         fp32 [in, in] as written by adadim_hessian.
 *   loss_rows optional fp32 [out];  loss  fp32 device scalar (required).
 * Prepares H internally on every call; use the _prepared form to score many
 * candidates against one H.
 */
int adadim_layer_error(adadim_ctx* ctx, const void* dW, int dW_dtype, int64_t out, int64_t in,
                       const float* H, float* loss_rows, float* loss);

/* Same result from a prepared H.  dW_dtype may also be ADADIM_DW_F16_SCALED
 * (dW already multiplied by hmeta[0,:], as adadim_quantize can emit). */
int adadim_layer_error_prepared(adadim_ctx* ctx, const void* dW, int dW_dtype, int64_t out, int64_t in,
                                const void* Hs, const float* hmeta, float* loss_rows, float* loss);

/*
 * The same for n candidates that share H, in one pass (the Hs tiles are fetched once for
 * all of them): dW is a HOST array of n device pointers, each [out, in] of type dW_dtype;
 * losses is a device array of n floats, loss_rows optional device [n, out].
 */
int adadim_layer_error_batch(adadim_ctx* ctx, int n, const void* const* dW, int dW_dtype, int64_t out,
                             int64_t in, const void* Hs, const float* hmeta, float* loss_rows, float* losses);

/*
 * adadim_layer_error_batch followed by adadim_select(losses, n, best_dev) in one call: the block that writes the
 * last loss also takes the argmin (same rule as adadim_select), one launch less per layer.  best_dev is a device
 * int32 and is required.
 */
int adadim_layer_error_batch_select(adadim_ctx* ctx, int n, const void* const* dW, int dW_dtype, int64_t out,
                                    int64_t in, const void* Hs, const float* hmeta, float* loss_rows, float* losses,
                                    int32_t* best_dev);

/*
 * adadim_layer_error_batch_select for callers that cannot allocate device memory: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The call above keeps its row partials, block
 * totals and counters in scratch that the context allocates and grows on demand; this one keeps them in a fixed
 * 16 MiB device array inside the library (one per GPU the library runs on, held until the process ends) and
 * calls no hipMalloc, hipFree or other allocating routine.  Same kernels, same launch shape, same results bit
 * for bit.
 *   n       1..8 candidates (one launch);  dW[c]  column-scaled fp16 in the scoring layout (ADADIM_DW_F16_SCALED),
 *           as adadim_quantize / adadim_quantize_both write it: the other dW types need a scaled copy of dW, which
 *           does not fit a fixed array.
 *   Sizes whose scratch exceeds the array are rejected with ADADIM_EINVAL and touch nothing;
 *   adadim_noalloc_scratch_bytes(n, out, in) gives the need (-1 for arguments out of range), the limit is
 *   16 MiB = 16777216 bytes: 512 + 64*ceil(out/256) + 4*n*slots*out with slots about ceil(in/256), e.g. 1.4 MB for
 *   two candidates of a 4096 x 11008 layer, 8.4 MB for eight of an 8192 x 8192 layer.
 *   Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two streams, two
 *   contexts, two threads) race and give undefined losses; calls on one stream, one after the other, are safe.
 * Everything else as in adadim_layer_error_batch_select.
 */
int adadim_layer_error_batch_select_noalloc(adadim_ctx* ctx, int n, const void* const* dW, int64_t out, int64_t in,
                                            const void* Hs, const float* hmeta, float* loss_rows, float* losses,
                                            int32_t* best_dev);
int64_t adadim_noalloc_scratch_bytes(int n, int64_t out, int64_t in);

/*
 * Eq. 1's argmin: index of the first minimum of losses[0..n) (a later
 * candidate wins only if strictly lower, as in App. B where 'oc' is visited
 * before 'ic').  NaN entries never win.
 *   losses    fp32 device array.   best_dev  optional device int32.
 *   host_best optional HOST int32*: if given, the call waits for the stream
 *             and stores the index there.
 */
int adadim_select(adadim_ctx* ctx, const float* losses, int n, int32_t* best_dev, int32_t* host_best);

/*
 * GPTQ in the dimension the search selected (Sec. 3.3 "Augmenting RTN and GPTQ", App. A.1, App. B
 * `gptq_ada`; GPTQ is Frantar et al. 2022): channels are quantized one after the other and each
 * channel's rounding error is spread over the channels not yet quantized.
 *
 * adadim_gptq_prepare works on H alone (shared by all layers with that input):
 *   dead[j] = 1 where H_jj == 0 (that diagonal entry is taken as 1 and the layer's weights of the
 *           channel as 0);  damping: percdamp * mean(diag H) is added to the diagonal;
 *   perm    visiting order, int32 [in]: perm[i] = original index of the channel visited i-th;
 *           act_order = 1: decreasing diag(H), equal values by index; 0: identity;
 *   U       fp32 [in, in], upper triangular, in visiting order: inv(P (H + damp I) P^T) = U^T U.
 *           Factorized in fp64 (device scratch: two in x in fp64 matrices), rounded once.
 * H fp32 [in, in] as adadim_hessian writes it; in <= 46340.
 */
int adadim_gptq_prepare(adadim_ctx* ctx, const float* H, int64_t in, float percdamp, int act_order, int32_t* perm,
                        uint8_t* dead, float* U);

/*
 * The sweep.  In blocks of 128 visited channels: q_i = Q(w_i), e_i = (w_i - q_i)/U_ii,
 * w_j -= e_i U_ij for the later channels j (inside the block at once, behind the block after it,
 * one channel's error at a time); all in fp32, every update a rounded product followed by a
 * rounded difference, so the result is reproducible bit for bit.  Q is the quantizer of
 * adadim_quantize (clip 1) with
 *   dim = OC: static groups: the parameters of (row, channel group) are static_scales /
 *           static_zeros [out, in/g] as adadim_quantize(dim = OC) writes them for the original W,
 *           looked up by the channel's original index (the paper's "reorder + static" setting);
 *           scales / zeros are not written (they are the static ones);
 *   dim = IC: the parameters of (row group, channel) are computed from the channel's current
 *           values when it is visited and written to scales f32 / zeros u8 [out/g, in]
 *           (the paper's "reorder" setting for per-IC); group 64 or 128.
 * Outputs in the original channel order: codes u8 [out, in]; optional dW fp32 [out, in] = W - What
 * (for adadim_layer_error); optional packed stream as in adadim_quantize.
 */
int adadim_gptq_quantize(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int dim, int bits, int group,
                         const float* U, const int32_t* perm, const uint8_t* dead, const float* static_scales,
                         const uint8_t* static_zeros, uint8_t* codes, float* scales, uint8_t* zeros, float* dW,
                         uint32_t* packed);

/*
 * The sweep in the b + 16/g storage format (see adadim_quantize_meta16): every scale is rounded into the 16-bit
 * group word before it is used, so the stored words de-quantize to exactly the weights whose errors were spread.
 *   dim = OC: static_meta u16 [out, in/g] as adadim_quantize_meta16(dim = OC) writes it for the original W;
 *   dim = IC: meta u16 [out/g, in] is written (the word of (row group, channel) when the channel is visited).
 * bits 2, 3 or 4; everything else as adadim_gptq_quantize.
 */
int adadim_gptq_quantize_meta16(adadim_ctx* ctx, const void* W, int64_t out, int64_t in, int dim, int bits, int group,
                                const float* U, const int32_t* perm, const uint8_t* dead, const uint16_t* static_meta,
                                uint8_t* codes, uint16_t* meta, float* dW, uint32_t* packed);

/*
 * Layer output for one activation vector from a per-IC quantized weight (Sec. 4.5 and App. D,
 * the per-IC kernel: weight [out x in] in b bits, input [in x 1] and output [out x 1] fp16):
 *     y[o] = sum_j scales[o/g, j] * (code[o, j] - zeros[o/g, j]) * x[j]
 * computed as sum_j (scales*x)[o/g, j] * code[o, j] - sum_j (scales*x)[o/g, j] * zeros[o/g, j]
 * in fp32 (the per-IC scale folded into the activation), rounded once to fp16.  (The kernel reads a code as
 * code + c with c a power of two fixed by the code's bit position, 4 .. 1024, and takes c * sum_j (scales*x)[o/g, j]
 * off again: a few more fp32 roundings of sums of that size, far below the fp16 rounding of y.)
 *   packed  the stream adadim_quantize(dim = IC, bits) writes: u32 [in, out*bits/32], 16-byte aligned
 *   scales  f32 [out/g, in] (16-byte aligned), zeros u8 [out/g, in] (4-byte aligned), as written there
 *   x       fp16 [in], 8-byte aligned;   y  fp16 [out]
 *   bits 2, 3 or 4; group a multiple of 32 dividing out (0 = out); in a multiple of 4.
 * The sum is split over fixed column chunks and added up in a fixed order: same bits every run.
 */
int adadim_gemv_ic(adadim_ctx* ctx, const uint32_t* packed, const float* scales, const uint8_t* zeros, const void* x,
                   int64_t out, int64_t in, int bits, int group, void* y);

/*
 * The same product from the b + 16/g format: `meta` u16 [out/g, in] as adadim_quantize_meta16(dim = IC)
 * writes it (8-byte aligned) in place of scales and zeros.  Half the parameter bytes of the call above.
 */
int adadim_gemv_ic_meta16(adadim_ctx* ctx, const uint32_t* packed, const uint16_t* meta, const void* x,
                          int64_t out, int64_t in, int bits, int group, void* y);

/*
 * Recording a sequence of calls as one HIP graph.  A layer's search is a dozen short kernels; launched one by
 * one the gaps between them are a tenth of the step on a 4096 x 4096 layer, replayed as a graph they close.
 *   adadim_capture_begin  starts recording on the context's stream, which must not be the default
 *           stream (EINVAL).  Calls made on the context until adadim_capture_end are recorded, not run.
 *           While recording, a call that would have to grow the context's scratch fails with EINVAL (make the
 *           same calls once beforehand), adadim_select takes no host output, adadim_profile records nothing,
 *           and the caller must not synchronise the stream or the device.
 *   adadim_capture_end    stops recording and returns the instantiated graph (a hipGraphExec_t as void*).  The
 *           graph holds the pointers and sizes of the recorded calls: the buffers must stay where they are,
 *           new contents are picked up on every launch.
 *   adadim_graph_launch   runs the graph on the context's stream (asynchronous like every other call).
 *   adadim_graph_destroy  frees it.  NULL is allowed.
 */
int adadim_capture_begin(adadim_ctx* ctx);
int adadim_capture_end(adadim_ctx* ctx, void** graph);
int adadim_graph_launch(adadim_ctx* ctx, void* graph);
void adadim_graph_destroy(void* graph);

/*
 * Measurement aid (not part of the method): per-kernel device timings.
 * adadim_profile(ctx, 1) clears the records and starts bracketing every kernel
 * the library launches on this context with a pair of HIP events on the
 * context's stream; adadim_profile(ctx, 0) stops.  At most 8192 launches are
 * recorded per enable; later ones are counted as `dropped`.
 * adadim_profile_read waits for the stream and returns the idx-th kernel's
 * record: name (host buffer of `cap` bytes), total milliseconds and number of
 * recorded launches.  Returns ADADIM_OK, or ADADIM_EINVAL when idx is past the
 * last record (use this to stop iterating).  adadim_profile_read_spread gives the
 * smallest, the median and the largest duration of the same launches (0 when there
 * are none).
 * An event pair costs a few microseconds of the stream's time (about 7 us per launch on an MI355X: 3 % of a
 * five-kernel step of 1.1 ms).  adadim_profile_only(ctx, name) restricts the bracketing to the kernel of that
 * name (as adadim_profile_read reports it, at most 31 characters) until it is called with NULL or "";
 * it changes no records and may be called while timing is on or off.
 */
int adadim_profile(adadim_ctx* ctx, int enable);
/*
 * Measurement aid: the rate the chip's matrix cores sustain on nothing but v_mfma_f32_32x32x16_f16 with
 * register-resident operands (1024 workgroups of four waves, 64 * iters instructions per wave), for all-zero
 * operands (random_operands = 0) or random fp16 operands in [-2, 2) (1).  The chip holds its power limit by
 * lowering the clock and the power depends on the operand bits, so the two rates differ; the second is the
 * ceiling a real fp16 contraction works under.  Waits for the stream.  tflops: the rate in TFLOP/s;
 * clock_mhz: the shader clock the loop ran at (clock64 against the 100 MHz wall_clock64).  Host pointers.
 */
int adadim_probe_mfma(adadim_ctx* ctx, int random_operands, int iters, double* tflops, double* clock_mhz);
/*
 * The same for the fp64 instruction the GPTQ factorization runs on: v_mfma_f64_16x16x4_f64, eight independent
 * accumulator chains per wave, 1024 workgroups of four waves, 8 * iters instructions per wave, operands near 1.
 * Outputs as above.  (On this chip the loop stays well below the published fp64 figure whatever the operands; the
 * factor's products are to be read against this rate.)
 */
int adadim_probe_mfma_f64(adadim_ctx* ctx, int iters, double* tflops, double* clock_mhz);
/*
 * Measurement aid: where the time of the Gram tile kernel goes, piece by piece.  Runs the 256-wide tile kernel of
 * adadim_hessian three times on X (device, fp16 [tokens, in], row pitch ldx; in > 1024) in a build that stamps the
 * 100 MHz clock around every piece, with the launch plan of an accumulating call (no whole tiles: those carry no
 * stamps), and reads the last launch's stamps back.  dispatcher = 1 launches one workgroup per piece in list order
 * whatever the plan, 0 as adadim_hessian would (a fixed order where the plan has short pieces).  H is not written and
 * the context's scratch for partial tiles is left with the stamps in it.  Waits for the stream.
 * records (host, cap * 8 floats): per piece {list (0 full piece, 1 rest, 2 short piece of a cut rest), XCD whose list
 * it is on, start and end in us from the first start, shader cycles, prologue us, main loop us, 0}.  n_records: the
 * number of pieces (also set when cap is too small, which is ADADIM_EINVAL).  plan_out (host, 8 ints): tiles, full
 * pieces per tile, their length in 32-token stages, tiles with a cut rest, pieces per cut rest, their length, whether
 * the order was fixed, places per XCD.
 */
/*
 * Measurement aid: what the access pattern of adadim_gemv_ic alone costs.  One launch that reads the code words of
 * `packed` (device, the [in][out * bits / 32] stream of adadim_gemv_ic, bits 2..4) with the grid, waves and column
 * ranges of the product's tile kernel and one xor per word in place of everything else; us (host): its duration
 * between two events on the context's stream.  Waits for the stream; uses the product's scratch for partial sums.
 */
int adadim_probe_gemv_read(adadim_ctx* ctx, const void* packed, int64_t out, int64_t in, int bits, double* us);
int adadim_probe_gram_timeline(adadim_ctx* ctx, const void* X, int64_t tokens, int64_t in, int64_t ldx,
                               int dispatcher, float* records, int cap, int* n_records, int* plan_out);
int adadim_profile_only(adadim_ctx* ctx, const char* name);
int adadim_profile_read(adadim_ctx* ctx, int idx, char* name, int cap, double* total_ms, int64_t* launches);
int adadim_profile_read_spread(adadim_ctx* ctx, int idx, double* min_ms, double* median_ms, double* max_ms);

#ifdef __cplusplus
}
#endif
#endif /* ADADIM_H */
