/*
 * intfa -- INT-FlashAttention forward pass (arXiv 2409.16997) for AMD MI355X (gfx950).
 *
 * C ABI of libintfa.so.  Conventions shared by every entry point:
 *   - Every pointer is a DEVICE pointer into memory the caller owns, valid until the work
 *     enqueued by the call has finished, and 16-byte aligned.  The library keeps no pointer
 *     after a call returns and allocates no memory.
 *   - Tensors are contiguous and row-major: activations [B, H, N, d] with d fastest, per-token
 *     scales [B, H, N], per-head scales [B, H].  The paper states everything for one head
 *     [N, d]; batch and heads are independent copies of it.
 *   - Calls enqueue kernels on a HIP stream and return without synchronising.  The stream is
 *     the explicit argument where there is one, else the one given to ifa_set_stream()
 *     (the null stream until then).  No call synchronises, allocates or enqueues a memset, so the
 *     explicit-stream calls may be recorded into a HIP graph and replayed.
 *   - Return value: IFA_OK (0) or a negative ifa_status.  On any error nothing is enqueued.
 *     Arguments are validated on the host before a launch, so an unsupported shape is an
 *     error code, never a device fault.
 *   - R = 127 is the INT8 maximum of Algorithm 1 everywhere (quantizer grid and P grid).
 */
#ifndef INTFA_H
#define INTFA_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { IFA_F32 = 0, IFA_F16 = 1, IFA_BF16 = 2 } ifa_dtype;

typedef enum {
    IFA_OK = 0,
    IFA_ERR_NULL = -1,        /* a required pointer is null                                   */
    IFA_ERR_SHAPE = -2,       /* a size is <= 0 or overflows the index range                  */
    IFA_ERR_DTYPE = -3,       /* dtype enum out of range                                      */
    IFA_ERR_UNSUPPORTED = -4, /* valid but not built: d, N granularity, misaligned pointer    */
    IFA_ERR_HIP = -5,         /* the HIP runtime refused the launch (hipGetLastError != 0)    */
    IFA_ERR_WORKSPACE = -6    /* the shape needs more workspace than given / than is built in  */
} ifa_status;

/* Human-readable name of a status code (static storage, never null). */
const char *ifa_status_str(int status);

/* Sets the HIP stream (a hipStream_t passed as void*) used by the entry points that take no
 * stream argument.  Process-wide; not thread-safe against concurrent calls.  Returns IFA_OK. */
int ifa_set_stream(void *hip_stream);

/*
 * Token-level symmetric INT8 quantization of Q and K (Section 3.2: S_Q = rowmax|Q| / R,
 * S_K = rowmax|K| / R; symmetric, no zero point).
 *   X       [rows, d] real activations of dtype x_dtype (ifa_dtype), rows = B*H*N
 *   Xq      [rows, d] int8 out:  q = clamp(rint(x * (127 / a)), -127, 127), a = max_k |x[r,k]|
 *   scale   [rows] fp32 out:     a / 127  (fp32 divide); an all-zero row gets scale 1, q = 0
 * Arithmetic is fp32 with round-half-to-even and is bit-exact against that definition.
 * d must be one of 32, 64, 128, 256, 512.  NaN/Inf inputs are outside the contract.
 */
int quantize_tokenwise(const void *X, int x_dtype, long rows, int d,
                       signed char *Xq, float *scale);

/* Same, on an explicit stream, storing scale * scale_mul (one fp32 multiply after the divide) in
 * place of the scale.  scale_mul = 1/sqrt(d) folds the usual softmax scale into s_Q, which by the
 * linearity remark of Section 3.2 equals scaling S; Xq does not depend on it.  scale_mul must be a
 * finite positive number (else IFA_ERR_SHAPE). */
int quantize_tokenwise_ex(const void *X, int x_dtype, long rows, int d,
                          signed char *Xq, float *scale, float scale_mul, void *hip_stream);

/*
 * Token-level quantization of the Hadamard-rotated rows (Section 5 names the combination with Hadamard
 * transformations as future work).  Each row x is replaced by H_d x (Walsh-Hadamard, Sylvester order,
 * unnormalized, fp32 butterflies in the order h = 1, 2, 4, ...) before the rule of quantize_tokenwise is
 * applied; the stored scale is max|H_d x| / 127 * scale_mul.  H_d H_d = d I, so rotating the rows of both Q
 * and K multiplies Q K^T by exactly d: scale_mul = 1/sqrt(d) on both (or 1/d on one) restores S, and the
 * attention entry points are used unchanged.  Same argument rules as quantize_tokenwise_ex.
 */
int quantize_tokenwise_hadamard(const void *X, int x_dtype, long rows, int d,
                                signed char *Xq, float *scale, float scale_mul, void *hip_stream);

/*
 * Tensor-level symmetric INT8 quantization of V (Section 3.2: S_V = max|V| / R, a single
 * scalar for the head matrix V in R^{N x d}).
 *   X       [heads, N, d] real activations, heads = B*H
 *   Xq      [heads, N, d] int8 out, same rounding rule as quantize_tokenwise
 *   scale   [heads] fp32 out.  global_scale = 0: one scalar per head (the paper's single-head
 *           statement applied to each head).  global_scale = 1: one scalar for the whole
 *           array, written to every slot.
 * Uses `scale` itself as its only scratch (it holds the absmax between the two passes), so the
 * array is read twice.  N*d must be a multiple of 8.
 */
int quantize_headwise(const void *X, int x_dtype, long heads, long N, int d,
                      signed char *Xq, float *scale, int global_scale);

/* Same, on an explicit stream. */
int quantize_headwise_ex(const void *X, int x_dtype, long heads, long N, int d,
                         signed char *Xq, float *scale, int global_scale, void *hip_stream);

/*
 * Token-level quantization of Q and K (Section 3.2) in ONE launch: what the per-block-V and half-INT8 paths need in
 * front of the attention call (their V goes through quantize_blockwise, or stays fp16).
 *   Q, K        [rows, d] real activations of dtype x_dtype (same shape; rows = B*H*N)
 *   Q_i8, K_i8  [rows, d] int8 out;  s_Q, s_K [rows] fp32 out;  s_Q_mul folded into the stored s_Q (> 0)
 *   hadamard    non-zero: both tensors are rotated by H_d first, as in quantize_tokenwise_hadamard (Section 5)
 * Results are bit-identical to two quantize_tokenwise_ex (or quantize_tokenwise_hadamard) calls, whose argument rules
 * apply; nothing is enqueued on an error.
 */
int quantize_qk(const void *Q, const void *K, int x_dtype, long rows, int d, signed char *Q_i8, signed char *K_i8,
                float *s_Q, float *s_K, float s_Q_mul, int hadamard, void *hip_stream);

/*
 * The whole input preparation of Section 3.2 for one attention call, in three launches instead of the six the
 * three separate calls take: token-level quantization of Q and K in ONE launch, which also carries the absmax pass of V
 * (a few workgroups per head leave the maximum of their part in the tail of V_i8: no atomics, nothing to clear); then
 * the quantization pass of V; then one thread per head writes s_V and the tail of V_i8.  With fewer than 32 heads, or
 * heads of fewer than 512 elements, V goes through the general two-pass path of quantize_headwise instead (four launches).
 *   Q, K, V          [heads, N, d] real activations of dtype x_dtype, heads = B*H
 *   Q_i8, K_i8, V_i8 [heads, N, d] int8 out;  s_Q, s_K [heads, N] and s_V [heads] fp32 out
 *   s_Q_mul          multiplier folded into the stored s_Q (1/sqrt(d) for the usual softmax scale; 1 for none)
 * Results are bit-identical to quantize_tokenwise_ex(Q, ..., s_Q_mul), quantize_tokenwise_ex(K, ..., 1) and
 * quantize_headwise(V, ..., global_scale = 0).  Argument rules of those calls apply (d in {32 ... 512}, N*d a
 * multiple of 8, alignment); nothing is enqueued on an error.
 */
int quantize_qkv(const void *Q, const void *K, const void *V, int x_dtype, long heads, long N, int d,
                 signed char *Q_i8, signed char *K_i8, signed char *V_i8, float *s_Q, float *s_K, float *s_V,
                 float s_Q_mul, void *hip_stream);

/*
 * Algorithm 1 (INT-FlashAttention forward), lines 4-18, for every (b, h) head:
 *   S = diag(s_Q) (Q K^T) diag(s_K)          int8 x int8 -> int32 on MFMA, then fp32 scales
 *   m = max(m, rowmax S);  P = round(127 exp(S - m))  in [0, 127], int8
 *   l = l e^{m_old - m} + rowsum(P);  O = e^{m_old - m} O + P V      int8 x int8 -> int32
 *   O = diag(l)^-1 O s_V
 * over key blocks of ifa_block_cols() keys, taken in ascending order (the result depends on
 * that block size, because each block is rounded on the grid of the running max).
 *   Q_i8, K_i8, V_i8   [B, H, N, d] int8
 *   s_Q, s_K           [B, H, N] fp32, strictly positive;  s_V [B, H] fp32
 *   causal             0: every key (the paper's setting); 1: key index <= query index only
 *   O                  [B, H, N, d] out, fp16 for int_flash_attn_fwd, o_dtype for the _ex form
 * There is no softmax scale: the paper's S has none.  A caller that wants 1/sqrt(d) multiplies
 * s_Q by it (exact by the linearity remark of Section 3.2).
 * Supported: d in {64, 128}; any N >= 1 with N*d <= 0x7ff00000 (just under 2^31); keys at or beyond N are
 * masked in the last, ragged key block and rows at or beyond N are not written; B*H*N*d < 2^40.
 */
int int_flash_attn_fwd(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                       const float *s_Q, const float *s_K, const float *s_V,
                       int B, int H, int N, int d, int causal, void *O);

int int_flash_attn_fwd_ex(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                          const float *s_Q, const float *s_K, const float *s_V,
                          int B, int H, int N, int d, int causal, void *O, int o_dtype,
                          void *hip_stream);

/*
 * Algorithm 1 for N_q query rows against N_k keys (the paper states it for N_q = N_k; rows are independent, so
 * only the loop bounds change): a chunk of queries against a longer key sequence, or one query (decoding).
 *   Q_i8 [B, H, Nq, d], s_Q [B, H, Nq];  K_i8, V_i8 [B, H, Nk, d], s_K [B, H, Nk];  s_V [B, H];  O [B, H, Nq, d]
 *   causal = 1: the queries are the LAST Nq positions of the key sequence, i.e. query i sees keys
 *   j <= i + (Nk - Nq); needs Nk >= Nq (else IFA_ERR_UNSUPPORTED: some query would see no key).
 * Everything else as int_flash_attn_fwd_ex, which is this call with Nq = Nk.
 */
int int_flash_attn_fwd_rect(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                            const float *s_Q, const float *s_K, const float *s_V,
                            int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype, void *hip_stream);

/*
 * Algorithm 1 for a FEW queries per head against many keys (a decode step, a few speculative tokens, a short chunk),
 * with the key axis of every head split over the whole chip.  Shapes, mask rule and error rules of
 * int_flash_attn_fwd_rect, with Nq <= 32 (else IFA_ERR_UNSUPPORTED).  Lines 9-10 run first for every key block (the
 * block maxima go to the workspace; for Nq <= 8 the scaled scores too, for 9 <= Nq <= 32 the second pass computes
 * them again from K), so that each part of the key axis forms P on the grid of the running maximum the sequential
 * walk of Algorithm 1 would have at that block: P and the int32 P V are those of int_flash_attn_fwd_rect bit for bit,
 * and O differs from its result only by the order of the fp32 additions of lines 12-13 (the partial (m, l, O) of the
 * parts are merged with e^{m_part - m}, once per part instead of once per block).  With 9 <= Nq <= 32 and 96 heads
 * or more the split does not pay (K would be read twice by a chip that is already full) and the call runs the kernel
 * of int_flash_attn_fwd_rect.
 *   workspace         device memory, 256-byte aligned, at least ifa_splitk_workspace_bytes(B, H, Nq, Nk, d) bytes
 *                     (else IFA_ERR_WORKSPACE); owned by the caller, contents undefined before and after, must not be
 *                     shared by calls that may overlap.  Three kernel launches on hip_stream, nothing is allocated.
 * ifa_splitk_workspace_bytes returns 0 for a shape this entry point does not take.
 */
long ifa_splitk_workspace_bytes(int B, int H, int Nq, int Nk, int d);

int int_flash_attn_fwd_splitk(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                              const float *s_Q, const float *s_K, const float *s_V,
                              int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype,
                              void *workspace, long workspace_bytes, void *hip_stream);

/*
 * int_flash_attn_fwd_splitk for callers that cannot allocate device memory and have no buffer to lend: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same kernels, same results; the workspace is an array built into the library's device image
 * (ifa_static_workspace_bytes() bytes, 16 MiB, held by every GPU the library runs on until the process ends).  The
 * call allocates nothing and frees nothing.  A shape with ifa_splitk_workspace_bytes(...) beyond that size is refused
 * with IFA_ERR_WORKSPACE before any launch (16 MiB hold, e.g., B*H = 128 heads of 16384 keys at Nq = 1).
 * ifa_static_workspace_bytes() doubles as the set-up call: it looks the array's device address up for the current
 * device (once per device; otherwise the first int_flash_attn_fwd_splitk_static on that device does it).
 * Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (two streams, two threads) race
 * on it and must be serialized by the caller.  Nothing in it needs clearing between calls: every word a call reads
 * it has written before.
 */
long ifa_static_workspace_bytes(void);

int int_flash_attn_fwd_splitk_static(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                     const float *s_Q, const float *s_K, const float *s_V,
                                     int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype,
                                     void *hip_stream);

/*
 * Per-block quantization of V -- the scheme the paper names as its next step (Section 3.2, footnote;
 * Section 5, which names per-block quantization of V as the next step).
 * One scale per (head, block of block_keys consecutive keys) = per V_j of Algorithm 1:
 *   X [heads, N, d] -> Xq [heads, N, d] int8 (same rounding rule as above),
 *   scale [heads, ceil(N / block_keys)] fp32 = max|V_j| / 127 (1 for an all-zero block).
 * Single pass (the block is held in registers).  block_keys * d <= 16384, d a multiple of 8; to feed
 * int_flash_attn_fwd_vblock, block_keys must equal ifa_block_cols(d, causal).
 */
int quantize_blockwise(const void *X, int x_dtype, long heads, long N, int d, int block_keys,
                       signed char *Xq, float *scale, void *hip_stream);

/*
 * Algorithm 1 with the per-block V scales above: line 13 becomes O = e^{m_old - m} O + s_V,j (P V_j) and
 * line 16 divides by l only.  s_Vb is [B, H, ceil(N / ifa_block_cols(d, causal))] fp32, strictly positive.
 * Everything else as int_flash_attn_fwd_ex.
 */
int int_flash_attn_fwd_vblock(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                              const float *s_Q, const float *s_K, const float *s_Vb,
                              int B, int H, int N, int d, int causal, void *O, int o_dtype,
                              void *hip_stream);

/*
 * The same for N_q query rows against N_k keys: shapes and mask rule of int_flash_attn_fwd_rect, per-block V scales
 * s_Vb [B, H, ceil(Nk / ifa_block_cols(d, causal))] of int_flash_attn_fwd_vblock (blocks count from key 0).
 */
int int_flash_attn_fwd_vblock_rect(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                   const float *s_Q, const float *s_K, const float *s_Vb,
                                   int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype,
                                   void *hip_stream);

/*
 * Half-INT8 variant (Section 4: Q and K in INT8, V kept in FP16): lines 9-10 of
 * Algorithm 1 as above, then the softmax weights stay real and are rounded to FP16 for the second GEMM:
 *   P~ = fp16(exp(S - m))  (nearest even, no factor R);   l = e^{m_old - m} l + rowsum(P~)  (the rounded weights, fp32)
 *   O  = e^{m_old - m} O + P~ V_j  (fp16 x fp16 products, fp32 accumulation);   O = diag(l)^-1 O
 * over key blocks of ifa_block_cols_half() keys in ascending order.
 *   Q_i8, K_i8 [B, H, N, d] int8;  s_Q, s_K [B, H, N] fp32, strictly positive;  V_f16 [B, H, N, d] fp16 as the
 *   caller has it (not quantized, no s_V);  O [B, H, N, d] of o_dtype.
 * Supported: d in {64, 128}; any N >= 1 with 2*N*d <= 0x7ff00000 (just under 2^31).  Same error rules as int_flash_attn_fwd_ex.
 */
int int_flash_attn_fwd_half(const signed char *Q_i8, const signed char *K_i8, const void *V_f16,
                            const float *s_Q, const float *s_K,
                            int B, int H, int N, int d, int causal, void *O, int o_dtype, void *hip_stream);

/* The half-INT8 variant for N_q query rows against N_k keys; shapes and the causal convention as in
 * int_flash_attn_fwd_rect (V_f16 is [B, H, Nk, d]).  int_flash_attn_fwd_half is this call with Nq = Nk. */
int int_flash_attn_fwd_half_rect(const signed char *Q_i8, const signed char *K_i8, const void *V_f16,
                                 const float *s_Q, const float *s_K,
                                 int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype, void *hip_stream);

/* Key-block size of the half-INT8 kernel for (d, causal); 0 if that pair is unsupported. */
int ifa_block_cols_half(int d, int causal);

/* B_c of Algorithm 1 as the kernel for (d, causal) uses it; 0 if that pair is unsupported. */
int ifa_block_cols(int d, int causal);

/*
 * Test hook: Algorithm 1 on ONE head through the production kernel, with its integer stages written out.  The kernel
 * run here is the one int_flash_attn_fwd_ex launches, instantiated with stores below its accumulators; nothing else
 * differs (same MFMA loops, same biased accumulators, same staging).  N must be a multiple of 128, at most 8192.
 *   P_in    [N, N] int8 or null.  Non-null: these values replace the computed P of line 11 as the operand of the
 *           second GEMM (and in the row sum l), which lets a test drive line 13 to the ends of its range.
 *   S_i32   [N, N] int32 out or null: Q_i8 K_i8^T, the accumulator of line 9 (exact).  Under the causal mask, key
 *           tiles of 32 that lie wholly above the diagonal for a whole wavefront are not computed and not written.
 *   P_i8    [N, N] int8 out or null: P of line 11 as it enters the second GEMM (masked keys: 0; skipped tiles are
 *           not written).
 *   PV_i32  [N / B_c, N, d] int32 out or null: P_j V_j of line 13 for every key block j (exact); blocks a query
 *           block does not visit under the mask are not written.
 *   O       [N, d] fp32 out: the attention output, as from int_flash_attn_fwd_ex.
 * Same argument rules and error codes as int_flash_attn_fwd_ex.
 */
int ifa_debug_fwd(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                  const float *s_Q, const float *s_K, const float *s_V, int N, int d, int causal,
                  const signed char *P_in, int *S_i32, signed char *P_i8, int *PV_i32, float *O, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* INTFA_H */
