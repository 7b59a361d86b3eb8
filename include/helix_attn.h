/* helix_attn.h -- C ABI of the MI355X (gfx950) exact attention library.
 *
 * The operation is the parameter-free attention part of a GPT-3 style transformer
 * layer (paper Section 2.1 and Figure 1: the layer splits into pre-attention,
 * attention and post-attention, and only the attention part has no parameters),
 * computed per (batch, head) slice on [S, D] matrices:
 *
 *     O   = softmax(scale * Q K^T + causal mask) V          LSE_i = ln sum_j exp(scale * q_i.k_j)
 *
 * and its gradients dQ, dK, dV for a given dO.  Next-token prediction (Section 4.6)
 * makes the mask causal: query i sees keys j <= i.  Dropout and biases do not exist on
 * this path (Table 1 caption).  The backward pass works only from what the paper calls
 * the activations "saved by flash attention" (Section 4.4, recomputation without
 * attention): the inputs q, k, v and the outputs o, lse.  No S x S object is ever stored.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  bf16 tensors are
 *     contiguous [B, H, S, D] (D fastest), 16-byte aligned; fp32 tensors are contiguous
 *     [B, H, S], 4-byte aligned.  D must be 64 or 128.  B, H, S >= 1; S is arbitrary
 *     (ragged tails are masked), B*H*S*D must stay below 2^40 elements.
 *   - The library never allocates, frees or synchronises.  Work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = default stream) and the call returns as soon
 *     as the launches are queued.
 *   - Outputs are overwritten in full; inputs are never written; an output must not
 *     alias any other argument.
 *   - Arguments are validated on the host before the first HIP call.  The return value
 *     is a helix_status; anything but HELIX_OK means nothing (or, for HELIX_ERR_LAUNCH,
 *     only part of the work) was enqueued.
 *   - `scale` must be finite and > 0.  `causal` != 0 applies the mask j <= i; causal == 0
 *     runs full attention.
 */
#ifndef HELIX_ATTN_H
#define HELIX_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HELIX_OK = 0,
  HELIX_ERR_NULL_POINTER = 1,
  HELIX_ERR_BAD_SHAPE = 2,
  HELIX_ERR_UNSUPPORTED_HEAD_DIM = 3,
  HELIX_ERR_MISALIGNED = 4,
  HELIX_ERR_BAD_SCALE = 5,
  HELIX_ERR_WORKSPACE = 6,
  HELIX_ERR_LAUNCH = 7,
  HELIX_ERR_BAD_STRIDE = 8,
  HELIX_ERR_SCRATCH_LIMIT = 9
} helix_status;

/* Element strides of a logical [B, H, S, D] bf16 tensor whose D elements per row are
 * contiguous: element (b, h, s, d) lives at base + b*batch + h*head + s*row + d.  Used by
 * the *_strided entry points; a NULL helix_strides pointer there means contiguous
 * [B, H, S, D] (batch = H*S*D, head = S*D, row = D).  Host memory, read during the call.
 * Accepted strides: non-negative multiples of 8 elements (rows start on 16-byte
 * boundaries), D <= row <= 2^24, and nested -- ordered by stride, each dimension of extent
 * > 1 steps over at least the whole span of the next smaller one -- which every permutation
 * of the dimensions of a dense or padded buffer satisfies and which excludes overlap.
 * Anything else is HELIX_ERR_BAD_STRIDE. */
typedef struct helix_strides {
  long long batch;
  long long head;
  long long row;
} helix_strides;

/* Forward (Table 1, Attention column, "Forward": two matrix products per (query, key)
 * pair, 4*b*h*s^2 FLOPs for a full score matrix).
 *   q, k, v : in,  bf16 [B, H, S, D]
 *   o       : out, bf16 [B, H, S, D]
 *   lse     : out, fp32 [B, H, S], natural-log sum-exp of the scaled scores of each row */
int helix_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                   int B, int H, int S, int D, float scale, int causal, void* stream);

/* Backward (Table 1, "Backward B": gradients wrt the inputs only; attention has no
 * "Backward W").  Runs its kernels in order on `stream`: the row sums
 * delta_i = sum_d dO_id * O_id, for causal attention a refinement of delta on the first
 * HELIX_DELTA_HEAD_ROWS rows of every head (see helix_attn_bwd_delta_head), the dK/dV
 * pass and the dQ pass.
 *   q, k, v, o, lse : in, as given to / produced by helix_attn_fwd
 *   dO              : in,  bf16 [B, H, S, D]
 *   dq, dk, dv      : out, bf16 [B, H, S, D]
 *   workspace       : device scratch of at least helix_attn_bwd_workspace_bytes(B,H,S,D)
 *                     bytes, 256-byte aligned, owned by the caller; holds the row statistics
 *                     (see below) between the kernels; contents undefined afterwards. */
int helix_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                   const void* dO, void* dq, void* dk, void* dv,
                   void* workspace, size_t workspace_bytes,
                   int B, int H, int S, int D, float scale, int causal, void* stream);

/* helix_attn_bwd for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: the same kernels, with the
 * row statistics kept in a device array built into the library (HELIX_STATIC_SCRATCH_BYTES
 * = 32 MiB per GPU, held from the first call on that GPU until the process ends) instead of
 * a caller-provided workspace.  The call itself allocates and frees nothing.  Shapes whose
 * statistics do not fit (B*H*S > 4194304 rows, i.e. helix_attn_bwd_workspace_bytes >
 * HELIX_STATIC_SCRATCH_BYTES) return HELIX_ERR_SCRATCH_LIMIT and enqueue nothing.  All calls
 * on one GPU share the array: calls that may overlap in time (different streams) race; every
 * call overwrites the part it uses before reading it, so nothing needs clearing in between.
 * Otherwise same arguments, results (bit for bit) and error behaviour as helix_attn_bwd. */
#define HELIX_STATIC_SCRATCH_BYTES (32u << 20)
int helix_attn_bwd_static(const void* q, const void* k, const void* v, const void* o, const float* lse,
                          const void* dO, void* dq, void* dk, void* dv,
                          int B, int H, int S, int D, float scale, int causal, void* stream);

/* Bytes of scratch helix_attn_bwd needs: two fp32 planes [B, H, S], each rounded up to 256
 * bytes.  Returns 0 for an invalid shape.  Pure host arithmetic. */
size_t helix_attn_bwd_workspace_bytes(int B, int H, int S, int D);

/* The stages of helix_attn_bwd as separate calls, for per-kernel timing and profiling.
 * Same conventions.  `stats` is the backward's workspace (helix_attn_bwd_workspace_bytes
 * bytes, 256-byte aligned, device): plane 0 holds -delta_i = -sum_d dO_id * O_id, plane 1
 * holds lse_i * log2(e), both fp32 [B, H, S]; the second plane starts half way into the
 * buffer.  The gradient passes take the statistics in this form so that they spend no
 * vector instruction per score element on them (-delta is the initial accumulator of the
 * dO V^T product, and the probabilities are 2^(scale*log2(e)*s - lse*log2(e))).
 *   preprocess : stats <- (-rowsum(dO * O), lse * log2(e))               (memory bound)
 *   delta_head : -delta_i <- -sum_j p_ij * (dO_i . v_j) for query rows i < rows of every
 *                head, overwriting those entries of plane 0.  The two expressions are equal
 *                in exact arithmetic; the first rows of a causal head attend to few keys, so
 *                O is large there and its bf16 rounding would dominate the error of delta.
 *   dkdv       : dk, dv from q, k, v, dO, stats
 *   dq         : dq     from q, k, v, dO, stats */
#define HELIX_DELTA_HEAD_ROWS 2048
int helix_attn_bwd_preprocess(const void* o, const void* dO, const float* lse, void* stats,
                              int B, int H, int S, int D, void* stream);
int helix_attn_bwd_delta_head(const void* q, const void* k, const void* v, const void* dO,
                              const float* lse, void* stats, int rows,
                              int B, int H, int S, int D, float scale, int causal, void* stream);
int helix_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dO,
                        const void* stats, void* dk, void* dv,
                        int B, int H, int S, int D, float scale, int causal, void* stream);
int helix_attn_bwd_dq(const void* q, const void* k, const void* v, const void* dO,
                      const void* stats, void* dq,
                      int B, int H, int S, int D, float scale, int causal, void* stream);

/* Compute-unit count and peak engine clock (kHz) of the current HIP device, the two
 * factors of the MFMA roofline (CUs x 4096 bf16 FLOP/clk x clock).  Host pointers. */
int helix_attn_device_info(int* compute_units, int* clock_khz);

/* Measurement aid: enqueues a loop of independent 32x32x16 bf16 MFMA instructions and nothing
 * else -- `workgroups` workgroups of 8 waves, `iters` x 16 instructions per wave -- and writes
 * the number of FLOPs it performs to *flops (host).  Timed by the caller, it gives the rate the
 * matrix pipes sustain on this chip, the practical ceiling of the attention kernels beside the
 * nominal peak.  random_operands != 0: operand bits vary as on real data (the chip then lowers
 * its clock under its power limit); 0: constant operands.  `sink` is a device float that the
 * kernel never writes in practice; workgroups <= 2^20, iters <= 2^24. */
int helix_mfma_probe(float* sink, int workgroups, int iters, int random_operands, long long* flops, void* stream);

/* Measurement aid: the loop of helix_mfma_probe (random operands) in the company an MFMA has in
 * the attention kernels -- per MFMA one 1 KB operand read from LDS and, forward_mix == 0, two
 * fused multiply-adds and half an exp2 (the mix of the two backward passes) or, forward_mix != 0,
 * three and one (the forward's).  What it sustains is the rate a kernel with that instruction mix
 * can reach with no barrier, tile copy or dependency in its way.  Same arguments, limits and FLOP
 * count as helix_mfma_probe; uses 64 KB of LDS per workgroup. */
int helix_mfma_mix_probe(float* sink, int workgroups, int iters, int forward_mix, long long* flops, void* stream);

/* Human-readable name of a helix_status value (static storage, never NULL). */
const char* helix_status_string(int status);

/* Forward and backward on strided views.  The paper's activations are sequence-major
 * [s, b, h] tensors (Section 2.1), attention consumes the Q, K, V produced by the QKV linear
 * layer (Section 4.2) and, under sequence parallelism, each GPU works on h/t of the heads
 * over the full sequence (Section 2.2): with these entry points q, k, v can be views into
 * the [S, B, 3*H*D] (or per-head interleaved [S, B, H, 3*D]) output of that layer and
 * o, dO, dq, dk, dv views of [S, B, H*D] activations, with no transposing copy.
 * Same semantics, argument rules and error behaviour as helix_attn_fwd / helix_attn_bwd;
 * every *_strides argument is a host pointer or NULL (see helix_strides).  lse and the
 * workspace stay contiguous fp32 [B, H, S]. */
int helix_attn_fwd_strided(const void* q, const helix_strides* q_strides,
                           const void* k, const helix_strides* k_strides,
                           const void* v, const helix_strides* v_strides,
                           void* o, const helix_strides* o_strides, float* lse,
                           int B, int H, int S, int D, float scale, int causal, void* stream);
int helix_attn_bwd_strided(const void* q, const helix_strides* q_strides,
                           const void* k, const helix_strides* k_strides,
                           const void* v, const helix_strides* v_strides,
                           const void* o, const helix_strides* o_strides, const float* lse,
                           const void* dO, const helix_strides* dO_strides,
                           void* dq, const helix_strides* dq_strides,
                           void* dk, const helix_strides* dk_strides,
                           void* dv, const helix_strides* dv_strides,
                           void* workspace, size_t workspace_bytes,
                           int B, int H, int S, int D, float scale, int causal, void* stream);

/* The QKV linear layer on the attention stage.  HelixPipe sends the layer's input A and its
 * weights to the stage that runs attention instead of Q, K, V (Section 4.2, 2bsh + 3h^2
 * instead of 4bsh elements), so the product runs right before the attention kernels and, with
 * N = 3*H*D columns, writes the [S, B, 3, H, D] buffer that helix_attn_fwd_strided reads in
 * place (Table 1, "QKV Linear": 6bsh^2 FLOPs forward, as much for each backward product).
 *   forward : qkv[M][N] = a[M][K] * w[K][N]                      bf16 in, fp32 accumulate, bf16 out
 *   backward: da[M][K]  = dqkv[M][N] * w[K][N]^T                 bf16 out
 *             dw[K][N]  = a[M][K]^T * dqkv[M][N]                 fp32 out (overwritten, not accumulated)
 * M = S*B rows (tokens), K = hidden size, N = this GPU's share of the 3h output columns.
 * All matrices are row-major device memory, 16-byte aligned; ld* is the number of elements
 * between consecutive rows (>= the row length, a multiple of 8, at most 2^22).  K and N must be
 * multiples of 128; M is arbitrary for the forward and a multiple of 32 for the backward
 * (HELIX_ERR_BAD_SHAPE otherwise; HELIX_ERR_BAD_STRIDE for a bad ld).  No bias (Table 1 neglects it).
 * The backward keeps a transposed copy of w and cuts the weight gradient's contraction over the M
 * tokens into parts that run side by side and are then summed in a fixed order (bit-reproducible,
 * no atomics); both live in `workspace`: device memory of at least
 * helix_qkv_linear_bwd_workspace_bytes(M, K, N) bytes, 256-byte aligned, owned by the caller,
 * contents undefined afterwards (HELIX_ERR_NULL_POINTER / _MISALIGNED / _WORKSPACE otherwise).
 * Asynchronous on `stream`; nothing is allocated; inputs are not written. */
int helix_qkv_linear_fwd(const void* a, long long lda, const void* w, long long ldw,
                         void* qkv, long long ldqkv, int M, int K, int N, void* stream);
int helix_qkv_linear_bwd(const void* a, long long lda, const void* w, long long ldw,
                         const void* dqkv, long long lddqkv, void* da, long long ldda,
                         float* dw, long long lddw, void* workspace, size_t workspace_bytes,
                         int M, int K, int N, void* stream);
/* Bytes of scratch helix_qkv_linear_bwd needs (0 for an invalid shape).  Pure host arithmetic. */
size_t helix_qkv_linear_bwd_workspace_bytes(int M, int K, int N);

/* Whether `strides` (NULL: contiguous) is acceptable for a [B, H, S, D] view: HELIX_OK,
 * HELIX_ERR_BAD_STRIDE, or the shape errors of the other calls.  Pure host arithmetic: the
 * same check the *_strided entry points apply to each of their tensors. */
int helix_attn_check_strides(const helix_strides* strides, int B, int H, int S, int D);

/* Library version: major*10000 + minor*100 + patch. */
int helix_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HELIX_ATTN_H */
