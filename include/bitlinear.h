/*
 * bitlinear.h - C ABI of the MI355X (gfx950) BitLinear library.
 *
 * BitLinear is the 1-bit-weight, 8-bit-activation linear layer of BitNet
 * (arXiv 2310.11453, Section 2.1):
 *
 *     y = W~ Quant(LN(x)) * beta * gamma / Q_b                       (Eq. 11)
 *     W~ = Sign(W - alpha), alpha = mean(W), Sign(0) = -1             (Eq. 1-3)
 *     beta = mean(|W|)                                                (Eq. 12)
 *     Quant(x) = Clip(x * Q_b / gamma, ...), gamma = ||x||_inf        (Eq. 4-5)
 *     Q_b = 2^(b-1) = 128 for the paper's b = 8.
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte
 *     aligned, unless marked "host".  The library allocates nothing, never
 *     synchronises and never copies a scalar to the host: alpha, beta and
 *     gamma stay in device memory.  Work is enqueued on `stream` (a
 *     hipStream_t passed as void*; NULL = the default stream) and the call
 *     returns at once.
 *   - W is fp32 [N,K] row-major (K = fan-in, contiguous), X is fp32 [M,K],
 *     Y is fp32 [M,N].  K must be a multiple of 32.  M, N, K <= 2^30 and
 *     N * K <= 2^40 (else BL_ERR_SHAPE); the matmul and forward calls (plain,
 *     grouped, non-negative) take K <= 65536 (per K-group for the grouped
 *     calls), else BL_ERR_UNSUPPORTED: their int32 partial sums carry a factor
 *     of up to 2^14 per element of K.
 *   - Return value: BL_OK or a negative bl_status.  Argument errors are found
 *     on the host before any launch, in the order shape, flags, pointers,
 *     workspace.  M == 0 is a successful no-op (pointers are not looked at).
 *   - Inputs are never written; outputs must not alias inputs.  NaN/Inf in W
 *     or X is undefined behaviour.  Results are deterministic run to run.
 *   - Scratch memory is passed in as `workspace` (size from
 *     bitlinear_workspace_bytes); calls sharing one workspace must be ordered
 *     on one stream.
 */
#ifndef BITLINEAR_H
#define BITLINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BL_OK = 0,
    BL_ERR_NULL = -1,        /* a required pointer is NULL */
    BL_ERR_SHAPE = -2,       /* M,N,K out of range, K % 32 != 0, size overflow */
    BL_ERR_UNSUPPORTED = -3, /* unknown granularity / flag combination */
    BL_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than required */
    BL_ERR_HIP = -5          /* a HIP launch reported an error */
} bl_status;

/* Granularity of the activation scale gamma.  The paper quantises per tensor
 * while training and per token at inference (end of the paragraph after Eq. 6). */
typedef enum { BL_GAMMA_PER_TOKEN = 0, BL_GAMMA_PER_TENSOR = 1 } bl_granularity;

enum {
    BL_FLAG_SKIP_LN = 1u,       /* input is already normalised: skip LN of Eq. 12 */
    BL_FLAG_OUT_ACC_I32 = 2u,   /* forward/matmul: write the int32 accumulator of Eq. 7
                                   into Y (reinterpreted as int32 [M,N]) instead of Eq. 11 */
    BL_FLAG_BETA_CENTERED = 4u  /* pack: beta = mean|W - alpha| (prose above Eq. 1)
                                   instead of the literal mean|W| of Eq. 12 */
};

/* Operation selector for bitlinear_workspace_bytes. */
typedef enum { BL_OP_PACK = 0, BL_OP_QUANT = 1, BL_OP_FORWARD = 2, BL_OP_BACKWARD = 3,
               BL_OP_LN_BACKWARD = 4, BL_OP_FORWARD_NONNEG = 5, BL_OP_MATMUL = 6 } bl_op;

/* host: size in bytes of the packed-weight blob for an [N,K] matrix (0 on bad
 * shape).  The blob is the library's own tiled 1-bit layout (1 bit per weight,
 * N padded to 16 and K to 512). */
size_t bitlinear_packed_bytes(int64_t N, int64_t K, unsigned flags);

/* host: scratch bytes the given operation needs; 0 for an invalid argument.  BL_OP_MATMUL
 * is the one operation whose need may be 0 for a valid shape (its workspace is optional and
 * only some shapes have a use for it). */
size_t bitlinear_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, int granularity,
                                 unsigned flags);

/* Eq. 1-3 and Eq. 12: binarise and pack a latent weight.
 *   W       in   fp32 [N,K]
 *   packed  out  blob of bitlinear_packed_bytes(N,K,flags) bytes
 *   alpha   out  fp32 [1], mean of W (fp64 accumulation, rounded once)
 *   beta    out  fp32 [1], mean |W| (or mean |W - alpha| with BL_FLAG_BETA_CENTERED)
 * A weight's bit is 1 iff W[n,k] > alpha (so Sign(0) = -1). */
int bitlinear_pack_weights(const float* W, int64_t N, int64_t K, unsigned flags, void* packed,
                           float* alpha, float* beta, void* workspace, size_t workspace_bytes,
                           void* stream);

/* Inspection / interchange: blob -> canonical uint32 [N, K/32], where bit (k % 32)
 * of word [n, k/32] is 1 iff W~[n,k] = +1 (Eq. 1). */
int bitlinear_packed_to_canonical(const void* packed, int64_t N, int64_t K, uint32_t* canonical,
                                  void* stream);

/* Eq. 12 (LN) + Eq. 4-5: normalise each token over K, take gamma, round and clip.
 *   X          in   fp32 [M,K]
 *   ln_gain    in   fp32 [K] or NULL (no affine is shown in Eq. 12)
 *   ln_bias    in   fp32 [K] or NULL
 *   ln_eps          epsilon inside the square root of Eq. 12
 *   codes      out  int8 [M,K], round-half-even of x^ * (128/gamma), clamped to [-128,127]
 *   gamma      out  fp32 [M] (per token) or [1] (per tensor), floored at 1e-5
 *   rowsum     out  int32 [M] = sum_k codes[m,k], or NULL
 *   xhat_dump  out  fp32 [M,K] normalised input before quantisation, or NULL */
int bitlinear_quant_act(const float* X, int64_t M, int64_t K, const float* ln_gain,
                        const float* ln_bias, float ln_eps, int granularity, unsigned flags,
                        int8_t* codes, float* gamma, int32_t* rowsum, float* xhat_dump,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Eq. 7 + Eq. 11 on already-quantised activations:
 *   Y[m,n] = (sum_k codes[m,k] * W~[n,k]) * (beta * gamma_m / 128).
 *   rowsum  in  int32 [M] as produced by bitlinear_quant_act (required)
 *   Y       out fp32 [M,N] (int32 accumulators with BL_FLAG_OUT_ACC_I32)
 *   workspace   optional (may be NULL): with bitlinear_workspace_bytes(BL_OP_MATMUL, ...) bytes
 *               the library may split K over more workgroups (M <= 16: K > 16384; 16 < M <= 64:
 *               whenever N alone supplies too few workgroups for the chip) and fold the int32
 *               slices afterwards; the result is the same bit for bit */
int bitlinear_matmul(const int8_t* codes, const float* gamma, const int32_t* rowsum, int64_t M,
                     int64_t K, const void* packed, int64_t N, const float* beta, int granularity,
                     unsigned flags, float* Y, void* workspace, size_t workspace_bytes,
                     void* stream);

/* Eq. 11, the whole layer: bitlinear_quant_act into the workspace, then
 * bitlinear_matmul.  Arguments as above.  For one token (M = 1, K <= 32768 and
 * an N that one round of workgroups covers) both steps run in one launch: the
 * GEMM kernel normalises and quantises the row itself, with the quantiser's
 * arithmetic but its own summation order, so a code can differ from
 * bitlinear_quant_act's where x^ * 128 / gamma sits on a rounding tie.  The
 * workspace is required in every case
 * (bitlinear_workspace_bytes(BL_OP_FORWARD, ...)).  Afterwards it holds the codes,
 * gamma and row sums the matmul step read and, for M = 1, the normalised row x^ the
 * codes were rounded from (bitlinear_forward_workspace_layout says where); the rest
 * is unspecified. */
int bitlinear_forward(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                      const float* beta, const float* ln_gain, const float* ln_bias, float ln_eps,
                      int granularity, unsigned flags, float* Y, void* workspace,
                      size_t workspace_bytes, void* stream);

/* bitlinear_forward for callers that cannot allocate or pass scratch memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the workspace is a
 * 16 MiB array the library itself holds in device memory (one copy per GPU, kept until the
 * process ends).  The call allocates nothing and runs the same kernels as bitlinear_forward:
 * same arguments, same result bit for bit.  Shapes whose workspace
 * (bitlinear_workspace_bytes(BL_OP_FORWARD, ...)) exceeds 16 MiB = 16777216 bytes return
 * BL_ERR_UNSUPPORTED: roughly M * K <= 16 MiB less the K-split partial sums, i.e. every
 * decode batch (M <= 64 at K <= 65536), not the prefill batches.  All calls on one GPU share
 * the array: calls that overlap in time (different streams, or threads) race; calls ordered
 * on one stream do not.  The array's contents after a call are unspecified. */
int bitlinear_forward_static(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                             const float* beta, const float* ln_gain, const float* ln_bias,
                             float ln_eps, int granularity, unsigned flags, float* Y,
                             void* stream);

/* host: where bitlinear_forward leaves its intermediates in the workspace, for inspection.
 * offsets[0..3] = byte offsets of codes (int8 [M,K]), gamma (fp32 [M] or [1]), rowsum
 * (int32 [M]) and x^ (fp32 [K], M = 1 only; (size_t)-1 otherwise).  BL_ERR_SHAPE /
 * BL_ERR_UNSUPPORTED / BL_ERR_NULL as for bitlinear_forward. */
int bitlinear_forward_workspace_layout(int64_t M, int64_t N, int64_t K, int granularity,
                                       size_t offsets[4]);

/* ---- Group Quantization and Normalization (Eq. 13-15) -------------------------------
 * The paper splits weights and activations into G groups "along the partition dimension"
 * and estimates alpha, beta, gamma and the LayerNorm statistics per group, so that a
 * tensor-parallel shard needs no exchange.  Its symbols leave the axis open; both are here:
 *   groups_n  groups of N/groups_n output rows of W (column-parallel): alpha_g, beta_g per
 *             group, activations untouched;
 *   groups_k  groups of K/groups_k input columns (row-parallel): alpha_g, beta_g per slice
 *             of W, LayerNorm over each slice of a token (Eq. 15), gamma_g per slice (Eq. 14),
 *             and Y = sum_g acc_g * beta_g * gamma_g / 128 (each slice dequantised, then added
 *             in fp32 in the order g = 0, 1, ...).
 * Both at once give groups_n x groups_k blocks of W.  groups_n = groups_k = 1 is the plain
 * layer, bit for bit.  Requirements: groups in 1..64, N % groups_n == 0,
 * (N/groups_n) % 16 == 0 when groups_n > 1 (else BL_ERR_UNSUPPORTED), K % groups_k == 0,
 * (K/groups_k) % 32 == 0 (else BL_ERR_SHAPE).
 *   alpha, beta   fp32 [groups_n][groups_k]
 *   packed        groups_k consecutive blobs, blob g = the [N, K/groups_k] slice in the tile
 *                 layout; bitlinear_packed_bytes_grouped bytes
 *   gamma         fp32 [M][groups_k] (per token) or [groups_k] (per tensor)
 *   rowsum        int32 [M][groups_k]
 *   ln_gain/bias  fp32 [K] or NULL, applied per element after the group statistics
 * Everything else as in the functions above. */
size_t bitlinear_packed_bytes_grouped(int64_t N, int64_t K, int groups_n, int groups_k);
/* op = BL_OP_PACK, BL_OP_QUANT, BL_OP_FORWARD, BL_OP_LN_BACKWARD or BL_OP_FORWARD_NONNEG; 0 for
 * anything invalid */
size_t bitlinear_workspace_bytes_grouped(int op, int64_t M, int64_t N, int64_t K, int groups_n,
                                         int groups_k, int granularity);
int bitlinear_pack_weights_grouped(const float* W, int64_t N, int64_t K, int groups_n,
                                   int groups_k, unsigned flags, void* packed, float* alpha,
                                   float* beta, void* workspace, size_t workspace_bytes,
                                   void* stream);
/* canonical uint32 [N, K/32] as in bitlinear_packed_to_canonical */
int bitlinear_packed_to_canonical_grouped(const void* packed, int64_t N, int64_t K, int groups_k,
                                          uint32_t* canonical, void* stream);
int bitlinear_quant_act_grouped(const float* X, int64_t M, int64_t K, int groups_k,
                                const float* ln_gain, const float* ln_bias, float ln_eps,
                                int granularity, unsigned flags, int8_t* codes, float* gamma,
                                int32_t* rowsum, float* xhat_dump, void* workspace,
                                size_t workspace_bytes, void* stream);
/* flags: BL_FLAG_SKIP_LN only */
int bitlinear_forward_grouped(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                              int groups_n, int groups_k, const float* beta, const float* ln_gain,
                              const float* ln_bias, float ln_eps, int granularity, unsigned flags,
                              float* Y, void* workspace, size_t workspace_bytes, void* stream);

/* Section 2.2, straight-through estimator: Sign, Clip and rounding are treated
 * as identity, alpha/beta/gamma as constants.
 *   dY     in   fp32 [M,N], rounded to bf16 (nearest even) as the MFMA operand
 *   codes, gamma  in  as produced by bitlinear_quant_act in the forward
 *   packed, beta  in  as produced by bitlinear_pack_weights (needed when dX != NULL)
 *   dX     out  fp32 [M,K] = beta * dY W~           (gradient w.r.t. LN(x)), or NULL
 *   dW     out  fp32 [N,K] = dY^T (codes * gamma/128), or NULL; with a per-token gamma
 *               the factor gamma_m/128 is folded into row m of dY before the bf16 rounding
 * The workspace (bitlinear_workspace_bytes(BL_OP_BACKWARD, ...)) holds the operand copies:
 * dY as bf16 twice (rows and transposed), the codes transposed as bf16 and the weight signs
 * regrouped (one bit each for large operands, bf16 for small ones): about 2*(2*M*N + K*M)
 * + K*N/8 bytes for large operands, 2*(2*M*N + K*N + K*M) at most. */
int bitlinear_backward_ste(const float* dY, int64_t M, int64_t N, int64_t K, const int8_t* codes,
                           const float* gamma, int granularity, const void* packed,
                           const float* beta, float* dX, float* dW, void* workspace,
                           size_t workspace_bytes, void* stream);

/* ---- The non-negative quantiser of Eq. 6 ----------------------------------------------
 * For inputs of non-linear functions the paper shifts the activations by their minimum and
 * scales them into [0, Q_b]:  x~ = Clip((x - eta) * Q_b / gamma, eps, Q_b - eps), eta = min x.
 * Read here as: gamma = max(x - eta) (the value that makes the range [0, Q_b]), floored at
 * 1e-5; codes = clamp(rne((x^ - eta) * (128 / gamma)), 0, 127), x^ the LayerNorm output.
 * The paper does not write the matching dequantisation; putting x ~ x~ gamma/Q_b + eta into
 * Eq. 11 gives
 *   Y[m,n] = acc[m,n] * (beta * gamma_m / 128) + (beta * eta_m) * wsum[n],
 *   wsum[n] = sum_k W~[n,k]   (bitlinear_weight_rowsums, once per weight).
 * Per token or per tensor (one eta and one gamma for the whole tensor: the training-time
 * granularity of the paragraph after Eq. 6; the running minimum and maximum are integer
 * atomics on an order-preserving key, exact and order-free).
 *   eta   out/in  fp32 [M] (per token) or [1] (per tensor), like gamma
 *   wsum  out/in  int32 [N];   the rest as in the functions above.
 * bitlinear_quant_act_nonneg needs a workspace only per tensor
 * (bitlinear_workspace_bytes(BL_OP_QUANT, ...)); bitlinear_forward_nonneg needs
 * bitlinear_workspace_bytes(BL_OP_FORWARD_NONNEG, M, N, K, granularity, 0).
 *
 * With K-groups (Eq. 14 gives every group its own eta_g beside gamma_g):
 *   eta, gamma  fp32 [M][groups_k] or [groups_k];  wsum int32 [groups_k][N], wsum[g][n] the sum of
 *   W~[n, k] over the columns of group g (bitlinear_weight_rowsums_grouped);
 *   Y = sum_g ( acc_g * beta_g * gamma_g / 128 + (beta_g * eta_g) * wsum[g][n] ), each term two
 *   fp32 products and one sum as above, the groups added in fp32 in the order g = 0, 1, ...
 * bitlinear_forward_grouped_nonneg needs
 * bitlinear_workspace_bytes_grouped(BL_OP_FORWARD_NONNEG, M, N, K, groups_n, groups_k, granularity). */
int bitlinear_weight_rowsums(const void* packed, int64_t N, int64_t K, int32_t* wsum,
                             void* stream);
int bitlinear_quant_act_nonneg(const float* X, int64_t M, int64_t K, const float* ln_gain,
                               const float* ln_bias, float ln_eps, int granularity,
                               unsigned flags, int8_t* codes, float* gamma, float* eta,
                               int32_t* rowsum, float* xhat_dump, void* workspace,
                               size_t workspace_bytes, void* stream);
int bitlinear_matmul_nonneg(const int8_t* codes, const float* gamma, const float* eta,
                            const int32_t* rowsum, int64_t M, int64_t K, const void* packed,
                            int64_t N, const float* beta, const int32_t* wsum, int granularity,
                            unsigned flags, float* Y, void* stream);
int bitlinear_forward_nonneg(const float* X, int64_t M, int64_t K, const void* packed, int64_t N,
                             const float* beta, const int32_t* wsum, const float* ln_gain,
                             const float* ln_bias, float ln_eps, int granularity, unsigned flags,
                             float* Y, void* workspace, size_t workspace_bytes, void* stream);
int bitlinear_weight_rowsums_grouped(const void* packed, int64_t N, int64_t K, int groups_k,
                                     int32_t* wsum, void* stream);
int bitlinear_quant_act_grouped_nonneg(const float* X, int64_t M, int64_t K, int groups_k,
                                       const float* ln_gain, const float* ln_bias, float ln_eps,
                                       int granularity, unsigned flags, int8_t* codes, float* gamma,
                                       float* eta, int32_t* rowsum, float* xhat_dump,
                                       void* workspace, size_t workspace_bytes, void* stream);
int bitlinear_forward_grouped_nonneg(const float* X, int64_t M, int64_t K, const void* packed,
                                     int64_t N, int groups_n, int groups_k, const float* beta,
                                     const int32_t* wsum, const float* ln_gain, const float* ln_bias,
                                     float ln_eps, int granularity, unsigned flags, float* Y,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the LayerNorm of Eq. 12 (per K-group: Eq. 15).  With the straight-through
 * estimator of Section 2.2 the dX of bitlinear_backward_ste is the gradient with respect
 * to the LayerNorm output; this call carries it to the layer's input and, if asked, to the
 * LayerNorm gain and bias:
 *   xn = (x - mu) * rstd,  gh = dXhat * gain
 *   dX = rstd * (gh - mean(gh) - xn * mean(gh * xn)),  means over a token's K (or K-group)
 *   dgain[k] = sum_m dXhat[m,k] * xn[m,k],   dbias[k] = sum_m dXhat[m,k]
 *   dXhat    in   fp32 [M,K]
 *   X        in   fp32 [M,K], the input the forward call saw
 *   ln_gain  in   fp32 [K] or NULL;  ln_eps as in the forward call;  groups_k >= 1 as there
 *   dX       out  fp32 [M,K] or NULL; may be the same buffer as dXhat
 *   dgain, dbias  out fp32 [K] or NULL; they need the workspace
 *                 (bitlinear_workspace_bytes_grouped(BL_OP_LN_BACKWARD, M, N, K, 1, groups_k, 0))
 * Any K / groups_k that is a multiple of 32 (rows of more than 16384 elements are walked
 * from memory in three passes instead of being held in registers). */
int bitlinear_layernorm_backward(const float* dXhat, const float* X, int64_t M, int64_t K,
                                 int groups_k, const float* ln_gain, float ln_eps, float* dX,
                                 float* dgain, float* dbias, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* Measurement aid, no part of the layer: one launch that only reads `bytes` (a multiple of 16)
 * of device memory at `src` with the access pattern of the small-batch GEMM's weight stream
 * (16-byte streaming loads, `workgroups` x `threads` lanes sharing the range evenly) and
 * discards them.  Its duration is the floor for any kernel that has to fetch the same bytes,
 * which is what a decode-shape GEMM is measured against.  sink: uint32 [workgroups] or NULL,
 * never written for real data.  threads: a multiple of 64 up to 1024. */
int bitlinear_probe_read(const void* src, size_t bytes, int workgroups, int threads, uint32_t* sink,
                         void* stream);

/* host: launch-time switches for tests and benchmarks; results never depend on them.
 * spec = "name=value,name=value" (integers); every switch not named returns to 0 = the
 * library decides; NULL or "" resets all.  Process-wide, not thread-safe, takes effect on the
 * next call.  Unless this function has been called, the environment variable
 * BITLINEAR_TUNING (same syntax) is read once, at the first call that launches.
 *   decode_nofuse=1     bitlinear_forward at M = 1: quantiser and GEMM as two launches
 *   decode_nosplit=1    M <= 16: never split K over workgroups
 *   decode_tiles=t      M <= 16: weight tiles per workgroup
 *   mid_nosplit=1       16 < M <= 64: never split K over workgroups
 *   mid_split_tiles=c   16 < M <= 64: 512-element chunks of K per slice
 *   mid_only=1          16 < M <= 32: skip the register-streaming kernel
 *   mid_kernel=1        32 < M <= 64: the LDS-tiled kernel with the K split inside the workgroup
 *   prefill_tile=1|2    M > 64: 128 x 256 or 256 x 256 output tiles
 *   prefill_grid=g      M > 64: workgroups of the persistent kernel
 *   group_slices=1      grouped layers up to 64 tokens: every K-group a work item of its own instead of
 *                       several K-groups inside one workgroup
 *   prefill_xbm=r       M > 64: rows of tiles in the block of tiles an XCD owns (1, 2, 4, 8; 0 = 1, the fastest measured; more rows fetch fewer bytes)
 *   quant_wpr=w         quantiser: waves per row (1, 2, 4, 8)
 *   bwd_ring=1|2        backward GEMMs: the ring kernel / the small kernel
 *   bwd_grid=g, bwd_rowmajor=1   backward ring kernel: workgroups, plain tile order
 * Returns BL_OK, or BL_ERR_UNSUPPORTED (unknown name or bad syntax; nothing changes). */
int bitlinear_set_tuning(const char* spec);

/* host: static description of a status code. */
const char* bitlinear_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* BITLINEAR_H */
