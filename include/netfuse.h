/*
 * netfuse.h -- C ABI of the merged ("input-weight local") operators of NetFuse on MI355X (gfx950).
 *
 * NetFuse runs M instances of one architecture, each with its own weights and its own input,
 * as one set of merged operators in which a weight set is paired with its own input only
 * (Section 3).  Matrix multiplications merge into a batch matrix multiplication, convolutions
 * into a grouped convolution whose groups are the models, layer normalisations into a group
 * normalisation with one group per model; batch normalisation, pooling, activations and
 * element-wise operators merge by concatenation (Section 3.1, Table 1).  The merged result is
 * exactly the M separate results (Appendix A).
 *
 * Conventions for every entry point
 *   - All pointers are DEVICE pointers on the current HIP device, owned by the caller, who
 *     keeps them alive until `stream` has passed the call.  The library allocates nothing; calls
 *     may be made from any thread.  The only state it keeps is (a) one flag per kernel that needs
 *     more than 64 KB of LDS, set when its first launch has opted in to that size (idempotent),
 *     and (b) the calling thread's pending request of netfuse_time_next_launch.  It reads no
 *     environment variable.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call validates
 *     its arguments on the host BEFORE touching HIP, enqueues its kernels and returns; it
 *     never synchronises.  Kernels use no atomics and no hidden workspace: results are
 *     deterministic and the calls can be captured into a HIP graph.
 *   - Tensors are dense row-major (last index fastest) unless a stride is given.
 *   - `dt` is the STORAGE type of activations and weight tensors (float or bfloat16 bit
 *     patterns).  Arithmetic is always fp32 (fp32 accumulation); a bf16 output is rounded once,
 *     to nearest even, when it is stored.  Per-feature / per-channel vectors (bias, scale,
 *     shift, gamma, beta, mean, var) and attention masks are ALWAYS float, for either `dt`.
 *   - Inputs are never written.  Outputs are fully overwritten.  An output may alias the
 *     `residual` operand or (norms, pools excepted where stated) not alias anything else.
 *   - Model order: slice m of every operand belongs to model m; nothing else is assumed.
 *   - Errors: the return value only.  NF_EINVAL = a NULL required pointer, a non-positive or
 *     inconsistent size, an unknown enum, or an element count that does not fit 2^31-1 where
 *     a kernel indexes with 32 bits; NF_EUNSUPPORTED = valid arguments with no kernel;
 *     NF_ELAUNCH = the HIP runtime refused the launch.  On any error nothing is enqueued.
 */
#ifndef NETFUSE_H
#define NETFUSE_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { NF_OK = 0, NF_EINVAL = 1, NF_EUNSUPPORTED = 2, NF_ELAUNCH = 3 } nf_status;
typedef enum { NF_F32 = 0, NF_BF16 = 1 } nf_dtype;
typedef enum { NF_ACT_NONE = 0, NF_ACT_RELU = 1, NF_ACT_GELU = 2 /* 0.5 x (1 + erf(x / sqrt 2)) */ } nf_act;
/* Which dimension the M models are concatenated along (the d_i of Algorithm 1). */
typedef enum { NF_MERGE_BATCH = 0, NF_MERGE_CHANNEL = 1 } nf_merge_dim;

/*
 * Merged matrix multiplication = batch matrix multiplication (Section 3.1, "Matrix
 * multiplication"): for every model m,   Y[m] = act(X[m] . W[m] + bias[m]) + residual[m].
 *   X[M][N][K]   W[M][K][Nout]   bias[M][Nout] float or NULL   residual[M][N][Nout] or NULL
 *   Y[M][N][Nout]                (N = rows of model m: batch x sequence)
 * Y may alias residual.  The bf16 MFMA path needs K and Nout to be multiples of 8 and 16-byte
 * aligned pointers; other shapes take a slower general kernel.
 */
nf_status netfuse_linear(const void* X, const void* W, const float* bias, const void* residual,
                         void* Y, int M, int N, int K, int Nout, nf_dtype dt, nf_act act,
                         void* stream);

/*
 * The same merged matmul on weights re-laid out once, offline (Section 3.1, "Matrix multiplication":
 * the M weight matrices are concatenated once when the models are merged; at inference they are
 * static and are nearly all of the bytes a forward pass reads).
 *
 * Packed layout (K a multiple of 16, Nout a multiple of 32; same element count as W; bf16 only,
 * NF_EUNSUPPORTED for float): the operand fragments of the 32x32x16 matrix instruction,
 *   Wp[m][j][s][l][e] = W[m][16 s + 8 (l / 32) + e][32 j + l % 32]
 *   j < Nout/32 (column block), s < K/16 (k slice), l < 64 (lane), e < 8,
 * so the 1 KB a wavefront loads for one multiplication is contiguous, the slices of a column block
 * follow one another down k, then the next column block, then the next model.
 * netfuse_linear_packed_supported: 1 if netfuse_linear_packed has a kernel for (M, N, K, Nout)
 *   (N a multiple of 128 and Nout a multiple of 96 with K % 256 == 0, or of 128, 288 or 384 with
 *   K % 128 == 0; N a multiple of 64 and Nout of 96, 288 or 384 where M * (N / 64) * (Nout / width) lies in
 *   129 ... 256 -- 64-row tiles, one workgroup per compute unit when 128-row tiles would leave half of them
 *   idle; or N and Nout multiples of 256 with K % 32 == 0) AND the problem is large enough for it to pay (at
 *   least 128 of its tiles: with few models netfuse_linear's smaller tiles are faster), else 0 (then use
 *   netfuse_linear; netfuse_linear_packed still runs any shape it has a kernel for).
 * netfuse_linear_pack_weight: W[M][K][Nout] -> Wp; W and Wp must not overlap; Wp 16-byte aligned.
 * netfuse_linear_packed: Y[m] = act(X[m] . W[m] + bias[m]) + residual[m] as netfuse_linear (the
 *   products are summed in fp32 in a different order, so results can differ from it in the last bit);
 *   X, residual, Y, bias 16-byte aligned; NF_EUNSUPPORTED where ..._supported returns 0.
 */
int netfuse_linear_packed_supported(int M, int N, int K, int Nout, nf_dtype dt);
nf_status netfuse_linear_pack_weight(const void* W, void* Wp, int M, int K, int Nout, nf_dtype dt,
                                     void* stream);
nf_status netfuse_linear_packed(const void* X, const void* Wp, const float* bias, const void* residual,
                                void* Y, int M, int N, int K, int Nout, nf_dtype dt, nf_act act,
                                void* stream);

/*
 * Ragged merged matmul: the per-task output layers of fine-tuned models have a different number of
 * outputs per model (Section 5.1 leaves them unmerged for that reason; Section 6, common backbones).
 * They still pair each weight set with its own input only, so they run as ONE launch over the models:
 *   Y_m = act(X_m . W_m + bias_m),   X[M][N][K],   W_m[K][nout[m]],   bias_m[nout[m]],   Y_m[N][nout[m]]
 * W, bias and Y are the per-model blocks concatenated in model order, each block dense row-major (so
 * W_m starts K * (nout[0] + ... + nout[m-1]) elements into W, Y_m N times that sum into Y).
 * nout is a HOST array of M positive ints, read during the call.  bias float or NULL.
 * NF_EUNSUPPORTED for more than 256 models.
 */
nf_status netfuse_linear_ragged(const void* X, const void* W, const float* bias, void* Y, int M, int N,
                                int K, const int* nout, nf_dtype dt, nf_act act, void* stream);

/*
 * Merged convolution = grouped convolution with M*g groups (Section 3.1, "Convolution" and
 * "Operations with input-weight local computations"; Appendix A Eq. 2-6).  Inputs and weights
 * are concatenated along the channel dimension: x[Cin*m + ci] = x_m[ci], w[Cout*m + co] =
 * w_m[co], y_m[co] = y[Cout*m + co].  Merged output channel c belongs to group
 * G = c / (Cout/g) and reads merged input channels G*(Cin/g) ... G*(Cin/g) + Cin/g - 1.
 *   x[B][M*Cin][H][W]   w[M*Cout][Cin/g][KH][KW]   y[B][M*Cout][Ho][Wo]
 *   Ho = (H + 2 pad - dilation (KH-1) - 1)/stride + 1 (floor), Wo likewise.
 * Zero padding, cross-correlation (no kernel flip).  Fused epilogue per output element, in this
 * order:  v = conv + bias[c];  v = v*scale[c] + shift[c];  v += residual;  y = act(v)
 * with bias, scale, shift float[M*Cout] or NULL (scale and shift both or neither: an inference
 * batch normalisation folded per merged channel, see netfuse_bn_fold) and residual shaped like y
 * or NULL.  y may alias residual.
 */
nf_status netfuse_conv2d(const void* x, const void* w, const float* bias, const float* scale,
                         const float* shift, const void* residual, void* y, int M, int B, int Cin,
                         int Cout, int g, int H, int W, int KH, int KW, int stride, int pad,
                         int dilation, nf_dtype dt, nf_act act, void* stream);

/*
 * Merged layer normalisation = group normalisation with M groups (Section 3.1, "Layer
 * normalization"): mean and (biased) variance of a row are taken over ONE model's H features.
 *   layout NF_MERGE_BATCH:   x[M][rows][H]   (what the batch matmul produces)
 *   layout NF_MERGE_CHANNEL: x[rows][M*H]    (channel concatenation, the group-norm form)
 *   gamma, beta: float[M*H], the M affine vectors concatenated.
 *   y = gamma (v - mean)/sqrt(var + eps) + beta,  v = x + residual (residual: like x, or NULL).
 * y may alias x or residual.
 */
nf_status netfuse_layernorm(const void* x, const void* residual, const float* gamma,
                            const float* beta, void* y, int M, int rows, int H, float eps,
                            nf_merge_dim layout, nf_dtype dt, void* stream);

/*
 * Merged batch normalisation, inference mode (Section 3.1: per-channel, so the models'
 * channels are concatenated).  x[B][M*C][HW]; gamma, beta, mean, var: float[M*C].
 *   y = act(gamma (x - mean)/sqrt(var + eps) + beta + residual)     residual like x, or NULL.
 * y may alias x or residual.
 */
nf_status netfuse_batchnorm(const void* x, const float* gamma, const float* beta, const float* mean,
                            const float* var, const void* residual, void* y, int M, int B, int C,
                            int HW, float eps, nf_dtype dt, nf_act act, void* stream);

/*
 * Per merged channel constants of an inference batch normalisation, for netfuse_conv2d's
 * epilogue:  scale = gamma/sqrt(var + eps),  shift = beta - mean*scale.  All float[n], n = M*C.
 */
nf_status netfuse_bn_fold(const float* gamma, const float* beta, const float* mean, const float* var,
                          float* scale, float* shift, int n, float eps, void* stream);

/*
 * Merged attention.  QK^T and PV are batch matrix multiplications over (sequence, head) already;
 * merging M models multiplies the number of independent problems by M (Section 3.1, "Operations
 * with input-weight local computations"); softmax has no weights (Section 3.1, "Non-trainable
 * operations").  For every (m, b, head):
 *   s_ij = scale * sum_t Q_it K_jt + mask_j;   p_ij = softmax over keys j;   O_it = sum_j p_ij V_jt
 * Element (m, b, s, head, t) of Q, K and V lives at  ptr[m*stride_m + (b*S + s)*stride_row + head*d + t]
 * (element units), so the three may point into one packed [M][B*S][3*heads*d] buffer.
 * mask: float[M][B][S], additive over keys, or NULL.   O[M][B*S][heads*d] dense.
 * Softmax is evaluated in fp32 with the row maximum subtracted.  O must not alias Q, K or V.
 */
nf_status netfuse_attention(const void* Q, const void* K, const void* V, const float* mask, void* O,
                            int M, int B, int S, int heads, int d, long stride_m, long stride_row,
                            float scale, nf_dtype dt, void* stream);

/*
 * Merged relative-position attention (the "extra computations" of XLNet that Section 5.2 refers to;
 * the paper gives no equations, so this is the published Transformer-XL / XLNet form).  As
 * netfuse_attention, with a position term and per-model, per-head bias vectors added to the query:
 *   s_ij = scale * ( (Q_i + bias_w) . K_j  +  (Q_i + bias_r) . Kr[S - i + j] ) + mask_j
 * Kr[M][2 S][heads*d] (storage type of Q, dense): row p of model m is ITS projection of the encoding of
 * relative distance S - p, i.e. what netfuse_linear gives for the 2 S sinusoid rows of distances
 * S, S-1, ..., -S+1 and that model's position weights; rows 1 ... 2S-1 are used.  This indexing is
 * the "relative shift" of those models written out.  bias_w, bias_r: float[M][heads*d] or NULL.
 * A segment term that is constant over the keys of a query (single-segment inputs) cancels in the
 * softmax and is not part of this call.
 */
nf_status netfuse_attention_relpos(const void* Q, const void* K, const void* V, const void* Kr,
                                   const float* bias_w, const float* bias_r, const float* mask, void* O,
                                   int M, int B, int S, int heads, int d, long stride_m, long stride_row,
                                   float scale, nf_dtype dt, void* stream);

/*
 * Non-trainable operators merge by concatenation (Section 3.1, "Non-trainable operations"), so
 * these act per channel of the channel-merged tensor; Ctot = M*C.
 * Max pooling: x[B][Ctot][H][W] -> y[B][Ctot][Ho][Wo], window k x k, Ho = (H + 2 pad - k)/stride + 1;
 * padded positions never win (pad < k required).
 * Global average pooling: x[B][Ctot][HW] -> y[B][Ctot].
 */
nf_status netfuse_maxpool2d(const void* x, void* y, int B, int Ctot, int H, int W, int k, int stride,
                            int pad, nf_dtype dt, void* stream);
nf_status netfuse_avgpool_global(const void* x, void* y, int B, int Ctot, int HW, nf_dtype dt,
                                 void* stream);

/*
 * The reshape-and-transpose that Algorithm 1 inserts where consecutive merged operators disagree
 * on the merge dimension (Section 3.2):  to_channel != 0: src[M][rows][H] -> dst[rows][M*H];
 * to_channel == 0: the inverse.  src and dst must not overlap.
 */
nf_status netfuse_merge_transpose(const void* src, void* dst, int M, int rows, int H, int to_channel,
                                  nf_dtype dt, void* stream);

/*
 * Measurement hook (Section 5.1 times every configuration; this makes the per-kernel figures exact):
 * arms the calling thread so that the NEXT kernel this library launches from this thread records its
 * own begin and end timestamps on the device into the two HIP events (hipEvent_t passed as void*,
 * created by the caller with timing enabled; either may be NULL).  hipEventElapsedTime(start, stop)
 * then is that kernel's duration as a kernel trace would report it, without the host-side cost of an
 * event pair.  The request is consumed by one launch; passing two NULLs cancels it.  Not for use
 * under stream capture.
 */
nf_status netfuse_time_next_launch(void* start_event, void* stop_event);

/*
 * Measured roofs (the merged operators are priced against the matrix pipe and against HBM; Section 5.1
 * measures on the machine at hand): two kernels that do nothing but the limiting operation, launched
 * and timed like any operator (netfuse_time_next_launch applies to them).
 * netfuse_probe_mfma: `iters` rounds of four independent 32x32x16 bf16 matrix instructions per wavefront, from
 *   registers only, on 256 workgroups of 16 wavefronts; *flops (HOST pointer) receives the floating point
 *   operations the launch executes.  sink: 4 device bytes, never written.
 * netfuse_probe_hbm_read: reads src[0 .. bytes) (device, 16-byte aligned, bytes a multiple of 16) once with
 *   16-byte non-temporal loads and discards it.  sink: 4 device bytes, never written.
 */
nf_status netfuse_probe_mfma(void* sink, int iters, double* flops, void* stream);
nf_status netfuse_probe_hbm_read(const void* src, long long bytes, void* sink, void* stream);

/* Static description of a status code; never NULL. */
const char* netfuse_strerror(nf_status status);

#ifdef __cplusplus
}
#endif
#endif /* NETFUSE_H */
