/*
 * sparge.h -- C ABI of the MI355X (gfx950) implementation of SpargeAttn's hot path:
 * block-sparse, INT8-quantized attention O = softmax(QK^T/sqrt(d))V driven by a two-stage
 * online filter (arXiv 2502.18137, Algorithm 1).
 *
 * General rules for every entry point
 *   - Every data pointer is DEVICE memory owned by the caller unless marked "host".  The library
 *     allocates and frees no device memory and keeps no pointer after returning; intermediates live in the
 *     workspace `ws` the caller passes (sparge_workspace_bytes; 256-byte aligned).  A workspace carries no
 *     state between calls, but two calls that may run at the same time (different streams, replays of
 *     different graphs) must not share one: besides intermediates it holds the item counters of the
 *     attention kernel's work distribution.
 *   - What the library does own, per process: a thread-local error string and the thread-local timing-event
 *     arrays of sparge_set_timing_events; the compute-unit count of each device, looked up at the first
 *     attention launch there; and, for sparge_forward only, one extra HIP stream and two events per device,
 *     created at the first sparge_forward on that device and never destroyed (see there for what that
 *     means for stream capture and host threads).  sparge_tune uses host memory for its tables.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default stream).  No
 *     entry point except sparge_tune synchronises the host; results are valid after the stream reaches
 *     the end of the enqueued work.
 *   - Return value: SPARGE_OK or a negative error code; sparge_last_error() then describes it.
 *     Invalid arguments are rejected before anything is enqueued.
 *   - Tensors Q, K, V, O share one descriptor: logical shape [B, H, N, d], element strides
 *     stride_b / stride_h / stride_n, d contiguous (stride 1).  [B,H,N,d] and [B,N,H,d] both fit.
 *     Rows must be 16-byte aligned (base pointers 16-byte aligned, strides multiples of 8 elements).
 *   - Block geometry is fixed (Alg. 1 line 2; App. A.1): b_q = 128 query rows, b_k = 64 key rows,
 *     row groups of 32 query rows (b_q / c_w, c_w = 4) for the stage-2 test.
 *     T_m = ceil(N/128), T_n = ceil(N/64).  A partial last block uses its valid rows only.
 *   - Supported: d in {64, 128}; dtype fp16 or bf16; H <= SPARGE_MAX_HEADS; T_n <= SPARGE_MAX_TN.
 *   - Hyper-parameters (Sec. 3.6) are per head, host arrays of length H: tau in (0,1],
 *     theta any real (theta > 1 makes every block a fix block; theta = -inf disables the judge),
 *     lambda < 0 (-INFINITY = never skip).
 *   - sm_scale <= 0 selects 1/sqrt(d).
 */
#ifndef SPARGE_H
#define SPARGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SPARGE_OK = 0, SPARGE_EINVAL = -1, SPARGE_EUNSUPPORTED = -2, SPARGE_ENOSPACE = -3, SPARGE_EHIP = -4 };
enum { SPARGE_F16 = 0, SPARGE_BF16 = 1 };
enum { SPARGE_BQ = 128, SPARGE_BK = 64, SPARGE_ROW_GROUP = 32 };
enum { SPARGE_MAX_HEADS = 128, SPARGE_MAX_TN = 4096 };
/* see sparge_attn_quantized: how far (log2 units) a row's maximum may run ahead of the value subtracted inside exp */
enum { SPARGE_REF_SLACK_LOG2 = 8, SPARGE_REF_SLACK_LOG2_FP8 = 2 };
/* sparge_desc.pv_dtype: type of the P~V product (Alg. 1 line 16) */
enum { SPARGE_PV_16BIT = 0 /* the tensors' fp16/bf16 */, SPARGE_PV_FP8 = 1 /* OCP E4M3, see sparge_v_tiles */ };
/* sparge_desc.qk_dtype: type of the Q K^T product (Alg. 1 line 12).  SPARGE_QK_16BIT is the paper's
 * "SpargeAttn+FA2" variant (Sec. 4.3): the same two-stage filter on an unquantized kernel -- Q and K
 * enter the product as they are (no K smoothing is needed: it does not change the softmax), scores
 * accumulate in fp32, S = Q_i K_j^T * sm_scale.  Read by sparge_attn and sparge_forward only; not built
 * together with SPARGE_PV_FP8, for N <= 131072 (2048 key blocks). */
enum { SPARGE_QK_INT8 = 0, SPARGE_QK_16BIT = 1 };

/* which entry point a workspace is sized for */
enum { SPARGE_WS_QUANTIZE = 0, SPARGE_WS_PREDICT = 1, SPARGE_WS_ATTN = 2, SPARGE_WS_ATTN_QUANTIZED = 3,
       SPARGE_WS_FORWARD = 4, SPARGE_WS_ATTN_TILED = 5 };

typedef struct sparge_desc {
    int32_t B, H, N, d;
    int32_t dtype;                          /* SPARGE_F16 | SPARGE_BF16 */
    int64_t stride_b, stride_h, stride_n;   /* in elements; the d axis is contiguous */
    int32_t pv_dtype;                       /* SPARGE_PV_16BIT | SPARGE_PV_FP8; only the attention entry points read it */
    int32_t qk_dtype;                       /* SPARGE_QK_INT8 | SPARGE_QK_16BIT */
} sparge_desc;

/* Description of the last error on the calling thread (host string, never NULL). */
const char* sparge_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int sparge_version(void);

/* Bytes of device scratch `ws` the given entry point (SPARGE_WS_*) needs for this shape.
 * The workspace needs 256-byte alignment and carries no state between calls; calls that may overlap in
 * time need one each. */
int sparge_workspace_bytes(const sparge_desc* desc, int entry, size_t* bytes /* host, out */);

/*
 * Quant (Alg. 1 line 3; Sec. 3.5): per-block symmetric INT8 quantization of Q (128-row blocks)
 * and of K minus its per-(batch,head) token mean (64-row blocks).
 *   amax = max|x| over the block; scale = amax/127; x_hat = rint_half_even(x * (127/amax)), all fp32;
 *   a zero block gives x_hat = 0, scale = 0.  k_mean = fp32(sum_t K[t,:] (fp64) / N).
 * Outputs: Qq, Kq int8 [B,H,N,d] contiguous; q_scale fp32 [B,H,T_m]; k_scale fp32 [B,H,T_n];
 *          k_mean fp32 [B,H,d].
 */
int sparge_quantize(const void* Q, const void* K, const sparge_desc* desc,
                    int8_t* Qq, int8_t* Kq, float* q_scale, float* k_scale, float* k_mean,
                    void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Stage-1 predictor (Alg. 1 lines 4-6; Sec. 3.2): block means q_i, k_j; block self-similarity
 * s = mean pairwise cosine of a block's tokens; S_hat = sm_scale * q k^T with column j set to -inf
 * when s_kj < theta (and, if causal, when block j lies entirely after block i);
 * P_hat = row softmax; M[i,:] = TopCdf(P_hat[i], tau) (smallest descending prefix whose mass
 * reaches tau * sum; ties by ascending j; zero-probability entries never selected); then
 * M[i,:] = 1 if s_qi < theta, M[:,j] = 1 if s_kj < theta; if causal, entirely-future blocks are 0
 * and the block holding the first diagonal key of Q block i (j = 2i) is 1.
 * Outputs: mask uint8 [B,H,T_m,T_n] (1 = compute); optional sim_q fp64 [B,H,T_m] and
 *          sim_k fp64 [B,H,T_n] (NULL to skip).
 * tau, theta: host float arrays [H].
 */
int sparge_predict(const void* Q, const void* K, const sparge_desc* desc,
                   const float* tau, const float* theta, float sm_scale, int causal,
                   uint8_t* mask, double* sim_q, double* sim_k,
                   void* ws, size_t ws_bytes, void* hip_stream);

/*
 * sparge_predict for callers that cannot provide a workspace and must not trigger an allocation: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * sparge_predict, minus `ws`: the intermediates live in a static device array of the library,
 * SPARGE_STATIC_SCRATCH_BYTES per device, held until the process ends.  A shape whose predictor workspace
 * (sparge_workspace_bytes, SPARGE_WS_PREDICT) is larger is rejected with SPARGE_ENOSPACE.  The call
 * allocates nothing, on the device or through any library.  All calls on one device share that array:
 * calls that may overlap in time there (different streams or host threads) race and give undefined masks;
 * nothing in it needs clearing between calls (every intermediate is written before it is read).  The
 * array's address is looked up at the first call on a device: make that call outside a stream capture.
 */
enum { SPARGE_STATIC_SCRATCH_BYTES = 4 << 20 };
int sparge_predict_static(const void* Q, const void* K, const sparge_desc* desc,
                          const float* tau, const float* theta, float sm_scale, int causal,
                          uint8_t* mask, double* sim_q, double* sim_k, void* hip_stream);

/*
 * Sparse flash loop with the stage-2 filter (Alg. 1 lines 7-20; Sec. 3.1, 3.3, 3.4) on
 * pre-quantized Q/K (outputs of sparge_quantize; k_mean is not needed: softmax is invariant to it).
 * For every Q block i and every kept K block j (mask[i,j] != 0, ascending j):
 *   S = (Qq_i Kq_j^T in int32) * q_scale[i] * k_scale[j] * sm_scale (+ element-wise causal -inf),
 *   m_local = rowmax(S), m_ij = max(m_i,j-1, m_local), P~ = exp(S - m_ij),
 *   l_ij = exp(m_i,j-1 - m_ij) l_i,j-1 + rowsum(P~)            -- always;
 *   for each 32-row group: if max(m_local - m_ij) > lambda:
 *       O_ij = diag(exp(m_i,j-1 - m_ij)) O_i,j-1 + P~(rounded to V's dtype) V_j   -- else skipped;
 * finally O_i = diag(l)^-1 O_i.  Rows without any kept visible key get 0.
 * Rounding point of P~: the value subtracted inside exp is a per-row reference that lags the running
 * maximum (O and l are kept relative to it and rescaled when it moves, which leaves O_i unchanged in
 * real arithmetic): before a tile's softmax, if some valid row of a 32-row group has
 * m - m_ref > SPARGE_REF_SLACK_LOG2 * ln 2, the whole group's reference moves to its running maximum.
 * The stage-2 test always uses the running maximum m_ij itself.
 * mask: uint8 [B,H,T_m,T_n] or NULL (= all ones).  lambda: host float [H].
 * O: same dtype/strides as V (desc).  stats: optional uint64 [B,H,4] = {QK^T tiles executed,
 * P~V row-group products executed, tiles a full attention needs, row-group products a full
 * attention needs}; it is overwritten, not accumulated.
 * Work distribution: the launch is two resident workgroups per compute unit that take (head, Q block)
 * items from eight counters (one per XCD range of items) kept in `ws` and cleared by a one-wave kernel
 * enqueued in front of the launch; which workgroup computes an item depends on timing, the result does not.
 */
int sparge_attn_quantized(const int8_t* Qq, const int8_t* Kq, const float* q_scale, const float* k_scale,
                          const void* V, const sparge_desc* desc, const uint8_t* mask,
                          const float* lambda, float sm_scale, int causal,
                          void* O, uint64_t* stats, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Diagnostic, host only (no GPU work): the order in which the attention kernel hands out its (batch, head,
 * Q block) items for this shape.  order: host array of B*H*T_m entries; entry n is (b*H + h)*T_m + i.  The items
 * are cut into eight contiguous ranges (one per XCD), listed here one after the other; a range hands its items
 * out in the listed order, the ranges run side by side, and a work-group whose range is empty takes from the
 * next.  Non-causal: index order.  Causal: per range, first the later (longer) half of every head's Q blocks,
 * head by head and longest first, then the earlier halves.  The result of a call never depends on this order.
 */
int sparge_item_order(const sparge_desc* desc, int causal, int32_t* order /* host, out */);

/*
 * The block mask M_g (Sec. 3.2, Def. 2) as an index list, for callers whose own kernels walk lists of kept
 * blocks: lut int32 [B,H,T_m,T_n], row (b,h,i) holds the j with mask[b,h,i,j] != 0 in ascending order -- the
 * order in which Alg. 1 line 9 visits them -- followed by -1; lut_count int32 [B,H,T_m] their number.
 * mask: uint8 [B,H,T_m,T_n] as sparge_predict writes it.  All three are device memory.  (The library's own
 * attention kernel builds this list per Q block in LDS and does not need the call.)
 */
int sparge_mask_to_lut(const uint8_t* mask, const sparge_desc* desc, int32_t* lut, int32_t* lut_count,
                       void* hip_stream);

/*
 * The two halves of sparge_attn_quantized, for callers that reuse V across calls or time the loop
 * alone.  sparge_v_tiles re-tiles V for the P~V product (Alg. 1 line 16); sparge_v_tiles_bytes gives
 * the size of its output (16-byte aligned device memory).
 * pv_dtype = SPARGE_PV_16BIT: per (b,h) and key block j, d rows of 64 key slots, keys >= N
 *   zero-filled; within every 16 keys the slot order is {0-3, 8-11, 4-7, 12-15}; 16-bit [B,H,T_n,d,64].
 * pv_dtype = SPARGE_PV_FP8 (the FP8 product the paper credits to its SageAttention2-based kernel,
 *   Sec. 1 footnote; the paper gives no formulas, these are the library's):
 *   delta_V[b,h,c] = fp32(max_t |V[b,h,t,c]|) / 448 in fp32 (0 for a zero channel),
 *   V_hat = e4m3(fp32(V) / delta_V), OCP E4M3, round to nearest even; in the loop P~ is multiplied by
 *   448 / 2^SPARGE_REF_SLACK_LOG2_FP8 (its largest possible value then is 448; the reference maximum
 *   lags by at most SPARGE_REF_SLACK_LOG2_FP8 instead of SPARGE_REF_SLACK_LOG2) and rounded to E4M3;
 *   products accumulate in fp32; O = (sum P~_q V_hat) delta_V / (scaled l); l sums the unrounded P~.
 *   Output: E4M3 bytes [B,H,T_n,d/32,2,64,16]: (channel tile, key half h2, lane = c%32 + 32 g, byte b)
 *   holds channel c of key 64 j + 32 h2 + 8 (b/4) + 4 g + b%4 (keys >= N are 0); then, 256-byte
 *   aligned, delta_V fp32 [B,H,d]; then, 256-byte aligned, the fp32 bit patterns of the channel maxima.
 * sparge_attn_tiled is sparge_attn_quantized with V already in that form; its workspace
 * (SPARGE_WS_ATTN_TILED, 1 KB) holds the item counters only.
 */
int sparge_v_tiles_bytes(const sparge_desc* desc, size_t* bytes /* host, out */);
int sparge_v_tiles(const void* V, const sparge_desc* desc, void* v_tiles, void* hip_stream);
int sparge_attn_tiled(const int8_t* Qq, const int8_t* Kq, const float* q_scale, const float* k_scale,
                      const void* v_tiles, const sparge_desc* desc, const uint8_t* mask,
                      const float* lambda, float sm_scale, int causal,
                      void* O, uint64_t* stats, void* ws, size_t ws_bytes, void* hip_stream);

/* Same as sparge_quantize followed by sparge_attn_quantized, with Q-hat/K-hat kept in `ws`. */
int sparge_attn(const void* Q, const void* K, const void* V, const sparge_desc* desc,
                const uint8_t* mask, const float* lambda, float sm_scale, int causal,
                void* O, uint64_t* stats, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * All of Algorithm 1: Quant, predict M_g, masked loop with the lambda skip.  Q and K are each read
 * once for block statistics + Q quantization and K is read a second time for its quantization.
 * mask_out: optional uint8 [B,H,T_m,T_n] receiving M_g (NULL: kept in `ws` only).
 * Streams: the V tiles, the K mean and the K quantization run on a second stream that the library
 * keeps per device (created at the first call on that device, default priority, never destroyed),
 * forked from `hip_stream` after the block statistics and joined to it before the attention kernel,
 * next to the block predictor on `hip_stream`.  For the caller the call is ordered on `hip_stream`
 * like any other.  A stream capture of `hip_stream` takes the second stream into the capture at the fork
 * and releases it at the join, inside this call; make the first call on a device outside a capture (the
 * stream cannot be created inside one).  Host threads: calls are serialised by a mutex while they
 * enqueue and share the second stream, so their side passes run one after the other.  Graphs captured
 * from this call hold no reference to that stream and may be replayed concurrently on different
 * streams, each with its own workspace, outputs and mask.
 */
int sparge_forward(const void* Q, const void* K, const void* V, const sparge_desc* desc,
                   const float* tau, const float* theta, const float* lambda,
                   float sm_scale, int causal, void* O, uint8_t* mask_out, uint64_t* stats,
                   void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Relative L1 distance of Sec. 3.6, L1 = sum|O - O'| / sum|O| with O the reference: per (batch, head)
 * the two sums.  O, O_ref: 16-bit tensors laid out as desc says; out: device fp64 [B,H,2] =
 * {sum|O_ref - O|, sum|O_ref|}, overwritten.  The summation order is fixed (one workgroup per (batch, head)):
 * the same inputs give the same bits on every call.
 */
int sparge_rel_l1(const void* O, const void* O_ref, const sparge_desc* desc, double* out /* device */,
                  void* hip_stream);

/*
 * Hyper-parameter determination for one attention layer (Sec. 3.6), per head, from n_inputs inputs of
 * one shape.  The error of a setting on an input is the relative L1 distance between the sparse output
 * and the full attention computed by the same kernels (every block kept, nothing skipped).
 *   1. every (tau, theta) of the grid with the lambda test off: among the pairs whose error stays
 *      below l1 on every input, the one with the largest sparsity (mean over the inputs);
 *   2. every lambda of the grid at the head's chosen pair: among the values whose error stays below l2
 *      on every input, the one with the largest sparsity, if that beats leaving the test off.
 * The paper leaves open how five inputs "constrain" the error: here the worst input binds and the mean
 * sparsity is maximized; ties keep the earlier grid entry (tau outer, theta inner); if no pair is
 * admissible the pair with the smallest worst-input error is taken.
 * Q, K, V: host arrays of n_inputs device pointers.  Grids and results are host arrays.  Results:
 * tau, theta, lambda [H] (lambda = -INFINITY: stage 2 stays off); optional sparsity, l1_out [H] of the
 * chosen setting; optional tables stage1 [n_tau,n_theta,H,2] and stage2 [n_lambda,H,2] = {mean
 * sparsity, worst error}.  pv_dtype of desc selects the P~V product that is tuned.
 * This is the one entry point that synchronises: it reads counters back after every candidate, and it
 * blocks until the stream has finished.  Workspace: sparge_tune_workspace_bytes (256-byte aligned).
 */
int sparge_tune_workspace_bytes(const sparge_desc* desc, int n_inputs, size_t* bytes /* host, out */);
int sparge_tune(const void* const* Q, const void* const* K, const void* const* V, int n_inputs,
                const sparge_desc* desc, const float* tau_grid, int n_tau, const float* theta_grid, int n_theta,
                const float* lambda_grid, int n_lambda, float l1, float l2, float sm_scale, int causal,
                float* tau, float* theta, float* lambda, double* sparsity, double* l1_out,
                double* stage1, double* stage2, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * HilbertCurve permutation (Sec. 3.7; App. A).  sparge_hilbert_order: perm[s] = row-major index (t, h, w
 * with w fastest) of the s-th cell a Hilbert curve visits in a T x H x W grid; the curve fills the
 * enclosing 2^b cube (b = ceil(log2(max(T, H, W))), at least 1) and cells outside the grid are skipped;
 * T = 1 (a single frame, an image) selects the two-dimensional curve over (H, W).
 * Host function, perm: host int32 [T*H*W].
 * sparge_permute_tokens: dst[b,h,offset + s,:] = src[b,h,offset + perm[s],:] for s < L (inverse != 0:
 * dst[b,h,offset + perm[s],:] = src[b,h,offset + s,:]); tokens outside [offset, offset + L) are copied in
 * place (joint text-visual attention permutes the visual tokens only).  perm: device int32 [L], a
 * permutation of 0..L-1 (an entry outside that range leaves its token in place; duplicates are not detected).  src, dst: distinct 16-bit tensors laid out as desc says.
 */
int sparge_hilbert_order(int T, int H, int W, int32_t* perm /* host, out */);
int sparge_permute_tokens(const void* src, const sparge_desc* desc, const int32_t* perm /* device */, int L,
                          int offset, int inverse, void* dst, void* hip_stream);

/*
 * Profiling aid (not part of the method).  Hands the library `n` pairs of caller-created hipEvent_t
 * (host arrays of handles).  From then on, every launch of the attention kernel made by the calling
 * thread is bracketed on its stream by hipEventRecord(starts[k]), hipEventRecord(stops[k]), k counting
 * launches from 0; after n launches nothing more is recorded.  n = 0 (or NULL arrays) switches it off.
 * The arrays must stay valid until then; the library never creates, destroys or waits on an event.
 */
int sparge_set_timing_events(void* const* starts, void* const* stops, int n);

#ifdef __cplusplus
}
#endif
#endif /* SPARGE_H */
