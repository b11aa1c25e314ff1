/*
 * sdgp.h -- C ABI of the SDGP backward-data library for AMD MI355X (gfx950).
 *
 * SDGP (Structured Data Gradient Pruning, arXiv 2202.00774) keeps n of every m
 * consecutive channels of the output data gradient dL/dO and zeroes the rest
 * (Alg. 1, Sec. III-A), then computes the input data gradient dL/dD from the
 * pruned tensor (Fig. 1, Fig. 2, Sec. II-A).  This library is that path and
 * nothing else: the prune primitive, and the backward-data product for linear
 * and convolution layers with the prune fused in.
 *
 * Conventions that hold for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or retains memory; scratch space, where a call needs
 *     it, is a workspace argument.  Inputs are const and are never
 *     written: dL/dO must survive because the weight gradient is computed from
 *     the unpruned tensor (Sec. III-A, last paragraph).
 *   - Tensors are contiguous, the pruned axis (channels) is the last one with
 *     stride 1 (Sec. III-A), and groups are the aligned runs
 *     [g*m, g*m+m) of that axis.  Groups never cross rows.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without synchronising.
 *   - All arguments are validated before anything is launched; a call that
 *     returns an error has had no effect on device memory.
 *   - A tensor with zero elements is a successful no-op.
 *   - Return value: SDGP_OK (0) or a negative sdgp_status.  No C++ exception
 *     crosses this boundary.
 */
#ifndef SDGP_H_
#define SDGP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SDGP_OK = 0,
    SDGP_ERR_NULL = -1,      /* a required pointer is NULL                                   */
    SDGP_ERR_NM = -2,        /* n < 1, n > m, m > 32 (Sec. III-A: group size at most 32)     */
    SDGP_ERR_SHAPE = -3,     /* channels not a multiple of m, negative size, element count
                                overflow, inconsistent convolution geometry, misaligned ptr  */
    SDGP_ERR_DTYPE = -4,     /* dtype is not an sdgp_dtype                                   */
    SDGP_ERR_RANKER = -5,    /* ranker is not an sdgp_ranker                                 */
    SDGP_ERR_WORKSPACE = -6, /* workspace is NULL or smaller than the size query returns     */
    SDGP_ERR_HIP = -7        /* the HIP runtime refused a launch (the HIP error is consumed) */
} sdgp_status;

typedef enum {
    SDGP_F32 = 0, /* IEEE binary32                                                     */
    SDGP_BF16 = 1 /* bfloat16 storage, fp32 arithmetic and accumulation, RNE on output */
} sdgp_dtype;

/* The three pruning functions of Sec. III-B.  "greedy" is the paper's Magnitude,
 * "greedy-adjusted" its Rescaled Magnitude. */
typedef enum {
    SDGP_RANDOM = 0,
    SDGP_GREEDY = 1,
    SDGP_GREEDY_ADJUSTED = 2
} sdgp_ranker;

/*
 * sdgp_prune -- Alg. 1 with the pruning function P of Sec. III-B.
 *
 *   dO      [rows, C] of `dt`, read only.
 *   n, m    keep n of every m consecutive channels; 1 <= n <= m <= 32, C % m == 0.
 *   rk      ranking rule.  The kept set of a group is the n positions with the
 *           largest (key, -position): larger key first, equal keys -> lower position.
 *             greedy, greedy-adjusted: key = |x| compared as the sign-cleared bit
 *               pattern (so -0 == +0, subnormals are not flushed).
 *             random: key = the 32-bit counter hash of (seed, flat element index
 *               row*C + channel); the values are not looked at.
 *           greedy-adjusted then multiplies the kept values of a group by
 *           s = (sum |x| over the group) / (sum |x| over the kept), both sums taken
 *           in fp32 in ascending channel order, one IEEE division, s = 1 when the
 *           denominator is 0; the product is rounded to `dt` (RNE).  This keeps
 *           the L1 norm of every group (Sec. III-B, Rescaled Magnitude).
 *   seed    only read by the random ranker.
 *   pruned  [rows, C] of `dt` or NULL: the dense-shaped pruned copy (the tensor
 *           Alg. 1 returns); dropped positions hold +0.
 *   vals    [rows, C*n/m] of `dt` or NULL: kept values in ascending channel order.
 *   idx     [rows, C*n/m] uint8 or NULL: position 0..m-1 of each kept value inside
 *           its group, strictly ascending inside a group.  vals and idx must be
 *           both NULL or both non-NULL.  At least one output must be requested.
 *
 * Pointers must be aligned to 16 bytes when C*sizeof(dt) is a multiple of 16
 * (any allocation from hipMalloc or torch is).
 */
int sdgp_prune(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, int rk, uint64_t seed,
               void* pruned, void* vals, uint8_t* idx, void* hip_stream);

/*
 * sdgp_linear_bwd_data -- dL/dD of a fully connected layer from the pruned dL/dO
 * (Fig. 2 right, Sec. II-A, with SDGP applied to dL/dO first).
 *
 *   dO  [rows, C_out] of `dt`       the layer's output data gradient (forward was O = D * W^T)
 *   W   [C_out, C_in] of `dt`       the layer's weights
 *   dD  [rows, C_in]  of `dt`       dD = prune(dO; n, m, rk, seed) * W, fp32 accumulation
 *
 * The prune is the one sdgp_prune defines (same keys, tie rule, rescale and flat
 * element index row*C_out + channel) and happens inside the kernel; no pruned
 * copy is written to memory.  n == m skips the ranker and is the dense product.
 */
int sdgp_linear_bwd_data(const void* dO, const void* W, void* dD, int64_t rows, int64_t C_out,
                         int64_t C_in, int dt, int n, int m, int rk, uint64_t seed,
                         void* hip_stream);

/*
 * sdgp_conv_bwd_data -- dL/dD of a 2-D convolution layer from the pruned dL/dO
 * (Fig. 3, Sec. III-A; convolution as a matrix product per Sec. II-A).
 *
 *   dO  [B, P, Q, C_out] NHWC      P = (H + 2*pad - R)/stride + 1, Q likewise from Wd and S
 *   W   [C_out, R, S, C_in]        (channels-last memory of a [C_out, C_in, R, S] weight)
 *   dD  [B, H, Wd, C_in] NHWC
 *
 *   dD[b,h,w,c] = sum over taps (r,s) and channels k of
 *                 prune(dO)[b,p,q,k] * W[k,r,s,c],   p = (h + pad - r)/stride, q = (w + pad - s)/stride,
 *   taking only taps for which p and q are integers inside [0,P) x [0,Q).
 *   The forward pass was a cross-correlation with dilation 1 and one group.
 *   Input pixels that no tap reaches receive 0.  Each dO element is pruned once,
 *   with flat element index ((b*P + p)*Q + q)*C_out + k.
 *
 *   workspace / workspace_bytes: scratch memory of at least
 *   sdgp_conv_bwd_data_workspace(...) bytes (16-byte aligned); may be NULL when the
 *   query returns 0.  Its contents are undefined afterwards.  Calls that share a
 *   workspace must be ordered on one stream.
 *
 * Requires 1 <= R,S <= 11, 1 <= stride <= 4, 0 <= pad < R and pad < S,
 * H + 2*pad >= R, Wd + 2*pad >= S.
 */
int sdgp_conv_bwd_data(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd,
                       int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt, int n,
                       int m, int rk, uint64_t seed, void* workspace, size_t workspace_bytes,
                       void* hip_stream);

/* Bytes of workspace sdgp_conv_bwd_data needs for these arguments; (size_t)-1 when
 * the arguments are invalid.  0 for most layers (the call is one fused kernel).
 *   - A first layer with a wide filter (C_in <= 4 and more than 32 (tap, channel)
 *     pairs) asks for room for a re-indexed copy of the filter that one small kernel
 *     builds before the fused one: 20 KB per 32 output channels for a 7x7 stride-2
 *     filter with padding 3 on an image of even size, 23 KB per 64 output channels
 *     for other 7x7 layers on three channels.
 *   - bf16 layers with n <= 2, m in {4, 8, 16} and C_out a multiple of 64 in which the
 *     fused kernel would rank a gradient element several times -- 1x1 filters with
 *     more than 256 input channels, strided filters up to 2*stride taps wide -- ask
 *     for room for the gradient ranked and compressed once (Sec. III-B: kept values
 *     and positions; 9/16 of the gradient's bytes), written by a pass of its own
 *     ahead of the product.
 *   - Small bf16 1x1 stride-1 layers (at most 2^24 elements in the gradient and in the
 *     filter) whose C_out is a multiple of 8 but not of 32 -- a classifier's 1000
 *     outputs -- ask for room for copies of the gradient and the filter with C_out
 *     rounded up to 32 (zeros in the new channels), on which the matrix-core kernel
 *     runs; without the workspace a slower kernel takes the layer.  The result does
 *     not depend on which one ran (the random ranker indexes rows of C_out elements
 *     either way). */
size_t sdgp_conv_bwd_data_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out,
                                    int R, int S, int stride, int pad, int dt, int n, int m);

/*
 * sdgp_conv_bwd_data_noalloc -- sdgp_conv_bwd_data for callers that cannot allocate device memory and therefore
 * cannot bring a workspace: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and error behaviour as sdgp_conv_bwd_data, minus the workspace: where that call
 * needs scratch memory (the re-indexed filter of a wide first layer), this one takes it from an array of
 * SDGP_NOALLOC_SCRATCH_BYTES that is part of the library's device image (each GPU the library runs on holds its own
 * copy until the process ends).  The call allocates and frees nothing.
 *
 *   - A first layer whose filter image exceeds SDGP_NOALLOC_SCRATCH_BYTES (the 7x7 stride-2 first layer of an
 *     ImageNet network with more than 384 output channels) returns SDGP_ERR_WORKSPACE and launches nothing;
 *     SDGP_ERR_HIP when the runtime cannot report the array's address.  Where the workspace of sdgp_conv_bwd_data
 *     only holds the gradient ranked ahead of the product, a problem whose arrays do not fit the scratch runs the
 *     fused kernel instead (same kept values, same result up to summation order); likewise a small 1x1 layer whose
 *     padded copies do not fit runs the kernel that needs none.
 *   - All calls on one GPU share that GPU's array, and it keeps the last call's contents (every call rewrites the
 *     part it reads, nothing has to start at zero).  Calls that overlap in time on one GPU -- different streams,
 *     or different host threads -- race on it: order them on one stream.
 */
#define SDGP_NOALLOC_SCRATCH_BYTES (256 * 1024)
int sdgp_conv_bwd_data_noalloc(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd,
                               int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt,
                               int n, int m, int rk, uint64_t seed, void* hip_stream);

/*
 * Rescaled Magnitude with one factor per channel.
 *
 * Sec. III-B defines Rescaled Magnitude on the group that P receives (what
 * SDGP_GREEDY_ADJUSTED does); the captions of the figures that show the rescaled
 * gradient instead state that the L1 norm is preserved per channel over the batch
 * and spatial dimensions.  The entry points below implement that second reading:
 * the kept set of every group is the Magnitude one, and channel c of the whole
 * tensor is multiplied by
 *     s[c] = (sum over rows of |dO[i,c]|) / (sum over the rows that kept c of |dO[i,c]|),
 * s[c] = 1 when the divisor is 0.  Both sums are accumulated in fp64 (in an order
 * that is fixed for a given shape, not the row order); s[c] is the fp64 quotient
 * rounded to fp32.
 *
 * sdgp_channel_scales       one read of dO [rows, C]: writes scale [C] (fp32, device) and, when
 *                           `sums` is not NULL, the two sums as sums[0..C) and sums[C..2C) (fp64,
 *                           device).  The result does not depend on the launch and is the same
 *                           from call to call (partial sums are added in a fixed order).
 *                           workspace: sdgp_channel_scales_workspace(...) bytes, 8-byte aligned.
 * sdgp_prune_channel_rescaled   Alg. 1 with P = Magnitude, kept values multiplied by scale[channel]
 *                           in fp32 and rounded to `dt` (RNE); dropped positions hold +0.
 *                           `scale` [C] is read from device memory (normally sdgp_channel_scales').
 * sdgp_scale_filter         W_scaled[k, :] = W[k, :] * scale[k] for W [C_out, inner] (inner = C_in for
 *                           a linear layer, R*S*C_in for a convolution), fp32 product rounded to
 *                           `dt`.  With it the rescaled product needs no second sweep over dO:
 *                           sum_k (x_k s_k) W[k,:] = sum_k x_k (s_k W[k,:]), so
 *                           sdgp_conv_bwd_data(dO, W_scaled, ..., SDGP_GREEDY, ...) is the backward-data
 *                           product of the rescaled gradient (rounding the filter instead of the
 *                           gradient: the same error bound, not the same bits).  W_scaled may
 *                           alias W.
 * sdgp_conv_bwd_data_channel_rescaled   the three steps above in one call: factors from dO, filter
 *                           rescaled into the workspace, fused Magnitude backward-data product.
 *                           A linear layer is the case B = rows, H = Wd = R = S = stride = 1, pad = 0.
 *                           workspace: sdgp_conv_bwd_data_channel_rescaled_workspace(...) bytes,
 *                           16-byte aligned; contents undefined afterwards.
 *
 * Shapes, n, m, alignment and error behaviour are those of sdgp_prune and sdgp_conv_bwd_data.
 * The workspace queries return (size_t)-1 for invalid arguments.
 */
size_t sdgp_channel_scales_workspace(int64_t rows, int64_t C, int dt, int n, int m);
int sdgp_channel_scales(const void* dO, int64_t rows, int64_t C, int dt, int n, int m, float* scale,
                        double* sums, void* workspace, size_t workspace_bytes, void* hip_stream);
int sdgp_prune_channel_rescaled(const void* dO, int64_t rows, int64_t C, int dt, int n, int m,
                                const float* scale, void* pruned, void* hip_stream);
int sdgp_scale_filter(const void* W, const float* scale, void* W_scaled, int64_t C_out, int64_t inner,
                      int dt, void* hip_stream);
size_t sdgp_conv_bwd_data_channel_rescaled_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                                                     int64_t C_out, int R, int S, int stride, int pad,
                                                     int dt, int n, int m);
int sdgp_conv_bwd_data_channel_rescaled(const void* dO, const void* W, void* dD, int64_t B, int64_t H,
                                        int64_t Wd, int64_t C_in, int64_t C_out, int R, int S,
                                        int stride, int pad, int dt, int n, int m, void* workspace,
                                        size_t workspace_bytes, void* hip_stream);

/*
 * sdgp_conv_bwd_data_grouped -- sdgp_conv_bwd_data for a grouped convolution (Sec. IV: RegNetX's 3x3 layers).
 * The channels split into `groups` independent convolutions: output channel k belongs to group
 * g = k / (C_out/groups) and saw the input channels [g*C_in/groups, (g+1)*C_in/groups) only, so
 *   W   [C_out, R, S, C_in/groups]
 *   dD[b,h,w,c] = sum over taps (r,s) and the output channels k of c's group of
 *                 prune(dO)[b,p,q,k] * W[k,r,s, c - g*C_in/groups].
 * dO is pruned along all of C_out as one row (Alg. 1 knows nothing of groups); C_out/groups must be a multiple of m
 * so that no m-group straddles two convolution groups (SDGP_ERR_SHAPE otherwise, and when groups does not divide
 * C_in and C_out).  groups == 1 is sdgp_conv_bwd_data.  For groups > 1:
 *   - bf16, 16 channels per group on both sides, 3x3, stride 1, padding 1 (RegNetX-400MF's layers), dO 16-byte and
 *     dD 8-byte aligned: one fused matrix-core kernel; the workspace holds the re-indexed filter (5 KB per group).
 *   - anything else: with n < m the gradient is pruned once into the workspace (the size of dO) and a plain kernel
 *     (one thread per dD element, fp32 accumulation) multiplies: correct for every shape and dtype, slow.
 * sdgp_conv_bwd_data_grouped_workspace(...) returns the bytes of the case the shape selects ((size_t)-1 for arguments
 * the call would refuse); a call of the first kind whose pointers are not aligned as stated falls to the second and
 * then needs the second's workspace (SDGP_ERR_WORKSPACE otherwise).
 */
size_t sdgp_conv_bwd_data_grouped_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R,
                                            int S, int stride, int pad, int64_t groups, int dt, int n, int m);
int sdgp_conv_bwd_data_grouped(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd,
                               int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int64_t groups,
                               int dt, int n, int m, int rk, uint64_t seed, void* workspace,
                               size_t workspace_bytes, void* hip_stream);

/*
 * Backward-data product from the compacted gradient (the K' = (n/m) * C_out form of Sec. III-A and of the ratio-4 and
 * ratio-8 estimates of Sec. IV-C): the prune pass writes the kept values and their positions into the workspace, then
 * every kept value adds its multiple of the matching row of W to its output pixels (one AXPY per kept value per tap,
 * fp32 FMAs on the vector ALUs; the rows differ from pixel to pixel, so this is not a matrix product).  Same result as
 * sdgp_conv_bwd_data up to summation order; its work falls with n/m, so it is the faster path only at high sparsity.
 *
 * bf16 only (SDGP_ERR_DTYPE otherwise); C_in a multiple of 8 and W, dD 16-byte aligned (SDGP_ERR_SHAPE otherwise, and
 * for a filter so large that m of its rows exceed 150 KB of LDS).  workspace:
 * sdgp_conv_bwd_data_compact_workspace(...) bytes, 16-byte aligned, contents undefined afterwards; the query returns
 * (size_t)-1 for arguments the call would refuse.  Everything else as sdgp_conv_bwd_data.
 */
size_t sdgp_conv_bwd_data_compact_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R,
                                            int S, int stride, int pad, int dt, int n, int m);
int sdgp_conv_bwd_data_compact(const void* dO, const void* W, void* dD, int64_t B, int64_t H, int64_t Wd,
                               int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt, int n,
                               int m, int rk, uint64_t seed, void* workspace, size_t workspace_bytes,
                               void* hip_stream);

/*
 * The two other products of a layer's training step (Sec. II-A, Fig. 1; Sec. IV-C, Fig. 9 times all three).
 * Neither prunes anything: SDGP touches only the data gradient, and Sec. III-A keeps the unpruned dL/dO for the
 * weight gradient.  They exist so that a whole step of a layer can run, and be timed, on this library's kernels.
 *
 * sdgp_conv_fwd          O[b,p,q,k] = sum_{r,s,c} D[b, p*stride + r - pad, q*stride + s - pad, c] * W[k,r,s,c]
 *                        D [B,H,Wd,C_in], W [C_out,R,S,C_in], O [B,P,Q,C_out], all `dt`; fp32 accumulation, RNE
 *                        on output; taps outside the image contribute nothing.  With stride 1 and R == S the
 *                        dense matrix-core kernels of the backward-data path compute it from a mirrored,
 *                        transposed copy of W that the call builds in the workspace; other layers take a
 *                        plain kernel.  O 16-byte aligned for the matrix-core path.
 * sdgp_conv_bwd_weight   dW[k,r,s,c] = sum_{b,p,q} dO[b,p,q,k] * D[b, p*stride + r - pad, q*stride + s - pad, c]
 *                        D and dO `dt`, dO UNPRUNED; dW [C_out,R,S,C_in] is written in fp32 whatever `dt` is.
 *                        bf16, stride 1, 3x3, C_in and C_out multiples of 64: matrix-core kernel whose workgroups
 *                        split the pixels and leave fp32 partial filters in the workspace, added in a fixed
 *                        order by a second kernel (the result is the same from call to call); other layers
 *                        take a plain reduction kernel.  D and dO 16-byte aligned for the matrix-core path.
 *
 * workspace: sdgp_conv_fwd_workspace(...) / sdgp_conv_bwd_weight_workspace(...) bytes (0 for layers that need none),
 * 16-byte aligned, contents undefined afterwards; the queries return (size_t)-1 for invalid arguments.  Geometry
 * rules and error behaviour are those of sdgp_conv_bwd_data (without n, m, ranker, seed).
 */
size_t sdgp_conv_fwd_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R, int S,
                               int stride, int pad, int dt);
int sdgp_conv_fwd(const void* D, const void* W, void* O, int64_t B, int64_t H, int64_t Wd, int64_t C_in,
                  int64_t C_out, int R, int S, int stride, int pad, int dt, void* workspace,
                  size_t workspace_bytes, void* hip_stream);
size_t sdgp_conv_bwd_weight_workspace(int64_t B, int64_t H, int64_t Wd, int64_t C_in, int64_t C_out, int R,
                                      int S, int stride, int pad, int dt);
int sdgp_conv_bwd_weight(const void* D, const void* dO, float* dW, int64_t B, int64_t H, int64_t Wd,
                         int64_t C_in, int64_t C_out, int R, int S, int stride, int pad, int dt,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Measurement aid: what the GPU sustains on the two resources the path is bound by (the benchmark reports its
 * roofline fractions against the published peaks and, beside them, against these).  One launch on `hip_stream`; the
 * caller times it.
 *   kind 0  copies `bytes` (rounded down to 16) from a to b with a plain streaming kernel
 *   kind 1  reads `bytes` of a; b receives one 4-byte word per workgroup (16 KB suffice)
 *   kind 2  `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16 per wavefront, two wavefronts per SIMD,
 *           operands in registers; a is ignored, b is not written (it must be a valid device pointer)
 *   kind 3  the same with v_smfmac_f32_32x32x32_bf16 (the structured-sparse instruction of the fused kernels)
 * a, b: device pointers, 16-byte aligned for kinds 0 and 1, never overlapping.  *work (HOST pointer) receives the
 * work of the launch: bytes moved (2 * bytes for the copy) or floating-point operations, dense-equivalent for kind 3
 * (2 * 32 * 32 * 32 per instruction).  Errors: SDGP_ERR_NULL, SDGP_ERR_SHAPE (kind, alignment, iters outside
 * 1 .. 2^20), SDGP_ERR_HIP.
 */
int sdgp_peak_probe(int kind, const void* a, void* b, size_t bytes, int iters, double* work, void* hip_stream);

/* Static, NUL-terminated description of a status code. */
const char* sdgp_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int sdgp_version(void);

#ifdef __cplusplus
}
#endif

#endif /* SDGP_H_ */
