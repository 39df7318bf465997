/*
 * fourier_attn.h -- C ABI of the MI355X (gfx950) FourierAttention hot path.
 *
 * Three operations of the paper's Section 3.3 ("Online Compression via
 * HiPPO-FourierT") and the calibration step of Section 3.4:
 *
 *   fa_compress  Eq. 1-4 (and Eq. 5 when `accumulate` is set): split the head
 *                dimensions of a middle token segment of K or of V into
 *                compressed and kept ones, project the compressed ones onto
 *                the first M real Fourier basis functions, and pack the kept
 *                ones.
 *   fa_compress_kv  the same for the K and the V segment of the same tokens in
 *                one call (fewer launches).
 *   fa_decode    Eq. 6: single-query attention over cat(sink+window rows,
 *                reconstructed middle rows) where the compressed dimensions
 *                of the middle rows are evaluated from their coefficients on
 *                the fly and never written to memory.
 *   fa_append    Eq. 5: the per-token update between two decode steps (the
 *                token leaving the recent window is folded into the state).
 *   fa_decode_mq    the same for several consecutive query tokens (causal
 *                among themselves).
 *   fa_select_dims  Section 3.4: rank the head dimensions of a segment by
 *                their reconstruction error and mark the Dc best for compression.
 *   fa_legt_compress / fa_legt_mse  Sections 3.2, 5.1: the translated-Legendre
 *                basis of the paper's basis comparison.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing and never synchronises: work is enqueued on
 *     `hip_stream` (a hipStream_t passed as void*, NULL = the default stream)
 *     and the call returns immediately.  The only state the library keeps
 *     between calls is per process: which kernels have had their dynamic-LDS
 *     ceiling raised, and (fa_decode_static) the device address of its static
 *     scratch array on each GPU; neither affects results.
 *   - Arguments are validated on the host before anything is launched; an
 *     invalid call launches nothing and returns a negative status.
 *   - Nothing throws, aborts or prints.
 *
 * Basis (Eq. 4, with the identically-zero sine of order 0 dropped): for
 * position p (relative to the first compressed token of the sequence),
 *   phi_0(p) = 1,  phi_{2n-1}(p) = cos(2 pi n p / T),  phi_{2n}(p) = sin(2 pi n p / T).
 * Coefficients are the plain inner products C[m,i] = sum_j phi_m(t0+j) X[j,i];
 * reconstruction weights each function by the inverse of its squared norm over
 * one period (1/T for the constant and for the cosine with 2n = T, else 2/T).
 */
#ifndef FOURIER_ATTN_H
#define FOURIER_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes: 0 = success, negative = error */
enum {
  FA_OK = 0,
  FA_ERR_NULL = -1,        /* a required pointer is NULL                      */
  FA_ERR_SHAPE = -2,       /* inconsistent or out-of-range sizes              */
  FA_ERR_UNSUPPORTED = -3, /* legal problem, but outside the compiled limits  */
  FA_ERR_WORKSPACE = -4,   /* workspace too small or misaligned               */
  FA_ERR_HIP = -5,         /* a HIP launch reported an error                  */
  FA_ERR_SCRATCH = -6      /* fa_decode_static: the sizes need more than FA_STATIC_SCRATCH_BYTES */
};

/* element type of q / K / V / kept-dimension tensors */
enum { FA_F32 = 0, FA_BF16 = 1 };

/* layout of the packed kept dimensions (K^mu / V^mu of Eq. 2), Du = D - Dc columns
 *   FA_KEEP_ROWS  [n_tokens, Dup]           one row per token, Dup = Du rounded up to a
 *                 multiple of 8; pad columns hold zeros (what fa_decode reads for K)
 *   FA_KEEP_TOK8  [ceil(n_tokens/8), Du, 8] eight consecutive tokens of one
 *                 dimension are contiguous    (what fa_decode reads for V)   */
enum { FA_KEEP_ROWS = 0, FA_KEEP_TOK8 = 1 };

/* compiled limits */
#define FA_MAX_HEAD_DIM 256   /* D, must be a multiple of 8                     */
#define FA_MAX_GROUP 16       /* query heads per KV head                         */
#define FA_MAX_STATES 1024    /* M accepted by fa_compress                        */
#define FA_MAX_DECODE_STATES 1024 /* M accepted by fa_decode for FA_BF16 (the paper's 2k = 1024) */
#define FA_MAX_DECODE_STATES_F32 256 /* M accepted by fa_decode for FA_F32           */
#define FA_MAX_KEPT_V_DIMS 128 /* D - Dvc accepted by fa_decode                     */
#define FA_MAX_SPLITS 256     /* token-axis chunks of fa_decode                  */

/*
 * fa_compress -- Eq. 2-3 for one tensor (K or V), optionally Eq. 5.
 *
 *   x           [B,H,N,D] middle segment (rows L_init .. L - L_local of Eq. 1),
 *               element type `dtype`, element strides sx_b/sx_h/sx_n, dim stride 1.
 *               Strides and base address must keep rows 16-byte aligned.
 *   dim_mask    [B,H,D] bytes, 1 = dimension is compressed.  Each row must
 *               contain exactly Dc ones (not checked: it would need a sync).
 *   M, T, t0    number of basis functions kept, period, position of x's
 *               first row;  1 <= M <= T, t0 >= 0, t0 + N <= T.
 *   accumulate  0: coeffs = projection;  1: coeffs += projection (Eq. 5 is the
 *               N = 1 case with t0 = number of tokens compressed so far).
 *   coeffs      [B,H,M,Dc] fp32, columns in ascending dimension order.
 *   x_keep      kept dimensions in ascending dimension order, layout
 *               `keep_layout`, element type `dtype`; slab (b,h) starts at
 *               x_keep + (b*H+h)*keep_stride_bh elements and token j of x is
 *               stored at token index keep_offset + j of that slab.  May be
 *               NULL (nothing is written).  keep_stride_bh = 0 means dense.
 *   workspace   at least fa_compress_workspace_bytes_for(dtype, ...) bytes, 256-byte
 *               aligned (fa_compress_workspace_bytes(...) suffices for either
 *               element type); it holds the per-token-chunk partial sums.
 *
 * N = 0 is legal (coeffs are zeroed unless accumulating).  Dc = 0 writes only
 * x_keep; Dc = D writes only coeffs.
 */
int fa_compress(const void* x, int dtype,
                int64_t sx_b, int64_t sx_h, int64_t sx_n,
                int B, int H, int N, int D,
                const uint8_t* dim_mask, int Dc,
                int M, int T, int t0, int accumulate,
                float* coeffs,
                void* x_keep, int keep_layout, int64_t keep_stride_bh, int keep_offset,
                void* workspace, size_t workspace_bytes, void* hip_stream);

size_t fa_compress_workspace_bytes(int B, int H, int N, int D, int Dc, int M);
/* The same for one element type: what a call with that `dtype` actually needs.  On long bf16
 * segments this is several times smaller than the figure above (fp32 inputs use shorter token
 * chunks, hence more partial sums); fa_compress accepts either. */
size_t fa_compress_workspace_bytes_for(int dtype, int B, int H, int N, int D, int Dc, int M);

/*
 * fa_decode -- Eq. 6 for one new query token per sequence.
 *
 *   q           [B,Hq,D] `dtype`; query head i uses KV head i / (Hq/Hkv).
 *   ck, cv      [B,Hkv,M,Dkc], [B,Hkv,M,Dvc] fp32 coefficients (K^mc, V^mc).
 *   kmask,vmask [B,Hkv,D] bytes; popcount Dkc / Dvc per row.
 *   M, T, t0, N basis size, period, position of the first middle row, number
 *               of middle rows (t0 + N <= T).
 *   k_keep      K^mu, FA_KEEP_ROWS layout, N tokens per (b,h) slab, slab stride
 *               kk_stride_bh elements (0 = dense).
 *   v_keep      V^mu, FA_KEEP_TOK8 layout, slab stride vk_stride_bh (0 = dense).
 *   k_full,v_full [B,Hkv,W,D] `dtype`: the L_init sink rows followed by the
 *               L_local window rows (their order does not affect the result);
 *               slab stride full_stride_bh elements (0 = dense).
 *   scale       softmax scale; <= 0 selects 1/sqrt(D).
 *   num_splits  token-axis chunks per (sequence, KV head) for the middle rows;
 *               0 lets the library choose.  The result does not depend on it
 *               beyond fp32 summation order.  With one chunk (num_splits = 1, or
 *               the library's choice from 192 (sequence, KV head) pairs on) shapes
 *               of the specialised bf16 kernel (D = 128, at most four query heads
 *               per KV head, 1 .. 32 kept dims on both sides, M <= 256, Dkc and Dvc
 *               multiples of 4) run as ONE launch: a workgroup per pair forms its
 *               series coefficients, walks its rows and merges, all in LDS.
 *   out         [B,Hq,D] fp32.
 *   workspace   at least fa_decode_workspace_bytes(...) bytes, 256-byte aligned.
 *
 * N = 0, W = 0, Dkc/Dvc = 0 or D are legal; N + W = 0 is FA_ERR_SHAPE.
 */
int fa_decode(const void* q, int dtype,
              int B, int Hq, int Hkv, int D,
              const float* ck, const uint8_t* kmask, int Dkc,
              const float* cv, const uint8_t* vmask, int Dvc,
              int M, int T, int t0, int N,
              const void* k_keep, int64_t kk_stride_bh,
              const void* v_keep, int64_t vk_stride_bh,
              const void* k_full, const void* v_full, int W, int64_t full_stride_bh,
              float scale, int num_splits,
              float* out,
              void* workspace, size_t workspace_bytes, void* hip_stream);

size_t fa_decode_workspace_bytes(int B, int Hq, int Hkv, int D, int Dkc, int Dvc,
                                 int M, int N, int W, int num_splits);

/*
 * fa_decode_varlen -- fa_decode for a batch whose sequences stand at different positions
 * (paper, Eq. 5: every sequence advances its own cache; batched serving).
 *
 * Same arguments, layouts, limits and workspace as fa_decode, with
 *   N_max, seq_n   seq_n: device pointer to B int32; sequence b has seq_n[b] middle rows (the first
 *                  seq_n[b] tokens of its k_keep / v_keep slabs).  Values are clamped into
 *                  [0, N_max]; N_max takes the place of N in every size, stride and workspace
 *                  rule.  seq_n = NULL: N_max rows for all.
 *   W_max, seq_w   the same for the full-width rows (rows 0 .. seq_w[b] - 1 of the k_full / v_full
 *                  slabs).  seq_w = NULL: W_max rows for all.
 * The launch plan is that of fa_decode(N = N_max, W = W_max): chunks past a sequence's rows leave
 * empty records; in the one-launch form (see num_splits) every workgroup simply walks its own
 * counts.  A sequence without any row gets out = 0.  The lists are read by the kernels, not by
 * the host: they may be written by earlier work on the same stream.
 */
int fa_decode_varlen(const void* q, int dtype,
                     int B, int Hq, int Hkv, int D,
                     const float* ck, const uint8_t* kmask, int Dkc,
                     const float* cv, const uint8_t* vmask, int Dvc,
                     int M, int T, int t0, int N_max, const int32_t* seq_n,
                     const void* k_keep, int64_t kk_stride_bh,
                     const void* v_keep, int64_t vk_stride_bh,
                     const void* k_full, const void* v_full, int W_max, const int32_t* seq_w,
                     int64_t full_stride_bh,
                     float scale, int num_splits,
                     float* out,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fa_decode_static -- fa_decode for callers that cannot allocate or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 *
 * Same arguments, kernels and results as fa_decode, without `workspace` / `workspace_bytes`: the
 * split-K state lives in a static device array of FA_STATIC_SCRATCH_BYTES inside the library (one
 * copy per GPU, held until the process ends; its device address is looked up on the first call on
 * each device).  The call allocates and frees nothing.  Sizes whose state
 * (fa_decode_workspace_bytes(...)) exceeds FA_STATIC_SCRATCH_BYTES return FA_ERR_SCRATCH and launch
 * nothing; the five benchmark configurations need 1 - 3 MB.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams,
 * two threads) race.  Calls on one stream, or otherwise ordered, are safe; nothing has to be
 * cleared between them.
 */
#define FA_STATIC_SCRATCH_BYTES (8u << 20)
int fa_decode_static(const void* q, int dtype,
                     int B, int Hq, int Hkv, int D,
                     const float* ck, const uint8_t* kmask, int Dkc,
                     const float* cv, const uint8_t* vmask, int Dvc,
                     int M, int T, int t0, int N,
                     const void* k_keep, int64_t kk_stride_bh,
                     const void* v_keep, int64_t vk_stride_bh,
                     const void* k_full, const void* v_full, int W, int64_t full_stride_bh,
                     float scale, int num_splits,
                     float* out, void* hip_stream);

/*
 * fa_append -- one decode step of cache maintenance (Eq. 5 and the recent window of Eq. 1).
 *
 * The recent window is a ring inside k_full / v_full (fa_decode does not care about the order of
 * their rows).  `slot` is the row that receives the new token.  With evict = 1 the window is full
 * and that row still holds its oldest token, which first becomes middle token number n_mid:
 *   ck[b,h,m,:] += phi_m(n_mid) * row[D^kc]        (the rank-one update of Eq. 5; same for cv)
 *   token n_mid of k_keep (FA_KEEP_ROWS) and of v_keep (FA_KEEP_TOK8) = row at the kept dims
 * With evict = 0 (window still filling) only the row is written and the arguments from kmask on
 * are ignored.  Afterwards fa_decode is called with N = n_mid + 1.
 *
 *   k_new,v_new [B,Hkv,D] `dtype`: the new token's key and value.
 *   k_full,v_full [B,Hkv,W,D] as for fa_decode, updated in place.
 *   n_mid       tokens folded so far = position of the evicted token; n_mid < T.
 *   ck, cv, k_keep, v_keep  as for fa_compress / fa_decode, updated in place; the slabs must
 *               have room for n_mid + 1 tokens (strides 0 = dense for exactly that many).
 *
 * Enqueues two small kernels on `hip_stream`; needs no workspace.
 */
int fa_append(const void* k_new, const void* v_new, int dtype,
              int B, int Hkv, int D,
              void* k_full, void* v_full, int W, int64_t full_stride_bh, int slot, int evict,
              const uint8_t* kmask, int Dkc, const uint8_t* vmask, int Dvc,
              int M, int T, int n_mid,
              float* ck, float* cv,
              void* k_keep, int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh,
              void* hip_stream);

/*
 * fa_append_varlen -- fa_append for a batch whose sequences stand at different positions (Eq. 5 per
 * sequence): every sequence has its own ring row and its own count of folded tokens.
 *
 *   seq_slot    device pointer to B int32: the ring row of sequence b that receives its new token.
 *               A value outside [0, W) leaves that sequence untouched (a finished sequence).
 *   seq_nmid    device pointer to B int32: the middle position the evicted token of sequence b
 *               takes (= tokens folded so far); negative: that sequence's window is still
 *               filling, nothing is folded and only the row is written.
 *   n_cap       tokens the k_keep / v_keep slabs have room for (strides 0 = dense for n_cap
 *               tokens); n_cap <= T.  A seq_nmid value >= n_cap is treated like a negative one.
 * Everything else as fa_append with evict = 1.  The lists are read by the kernels.
 */
int fa_append_varlen(const void* k_new, const void* v_new, int dtype,
                     int B, int Hkv, int D,
                     void* k_full, void* v_full, int W, int64_t full_stride_bh, const int32_t* seq_slot,
                     const uint8_t* kmask, int Dkc, const uint8_t* vmask, int Dvc,
                     int M, int T, const int32_t* seq_nmid, int n_cap,
                     float* ck, float* cv,
                     void* k_keep, int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh,
                     void* hip_stream);

/*
 * fa_compress_kv -- fa_compress for the K and the V segment of the same tokens in
 * one call (Eq. 2-4 applied to both caches, as prefill does).
 *
 * Equivalent to
 *   fa_compress(k, ..., kmask, Dkc, ..., ck, k_keep, FA_KEEP_ROWS, kk_stride_bh, keep_offset, ...)
 *   fa_compress(v, ..., vmask, Dvc, ..., cv, v_keep, FA_KEEP_TOK8, vk_stride_bh, keep_offset, ...)
 * (the layouts fa_decode reads); k and v share dtype, shape [B,H,N,D] and
 * strides.  When both sides qualify for the specialised projection kernel
 * (bf16, D = 128, at most 32 kept dims each, keep_offset a multiple of 8) the
 * two projections run as ONE launch and the two chunk reductions as one: two
 * kernel launches per call instead of four, and each tensor is cut into half
 * as many token chunks, so that the pair is one round of workgroups.  Kept
 * dims are identical to the two calls'; coefficients agree up to fp32
 * summation order (the chunk boundaries differ).
 * workspace: >= fa_compress_kv_workspace_bytes_for(dtype, B, H, N, D, Dkc, Dvc, M)
 * (fa_compress_kv_workspace_bytes(...) covers either element type), 256-byte aligned.  Everything else (argument meaning, errors, asynchrony) as fa_compress.
 */
size_t fa_compress_kv_workspace_bytes(int B, int H, int N, int D, int Dkc, int Dvc, int M);
size_t fa_compress_kv_workspace_bytes_for(int dtype, int B, int H, int N, int D, int Dkc, int Dvc, int M);
int fa_compress_kv(const void* k, const void* v, int dtype,
                   int64_t sx_b, int64_t sx_h, int64_t sx_n,
                   int B, int H, int N, int D,
                   const uint8_t* kmask, int Dkc, const uint8_t* vmask, int Dvc,
                   int M, int T, int t0, int accumulate,
                   float* ck, float* cv,
                   void* k_keep, int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh,
                   int keep_offset,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fa_decode_mq -- fa_decode for Tq consecutive query tokens per sequence (paper,
 * Section 3.3: the FlashAttention side of the fused kernel; chunked decoding or
 * the verification of drafted tokens).
 *
 * Same arguments, layouts and limits as fa_decode, except:
 *   q, out    [B, Hkv, Tq, G, D] (G = Hq / Hkv): the queries of one KV head are
 *             contiguous, token-major.  With Tq = 1 this is fa_decode's [B, Hq, D].
 *   k_full, v_full   the LAST Tq of the W rows are the Tq new tokens, in order;
 *             query token t sees every other row, every middle row, and new
 *             tokens 0 .. t (causal among the new tokens).  1 <= Tq <= W.
 *   Tq * G <= 16 (the group limit of fa_decode applies to tokens x heads).
 *   workspace >= fa_decode_workspace_bytes(B, Tq * Hq, Hkv, ...).
 * The middle rows and the older full-width rows are read once for all Tq tokens.
 */
int fa_decode_mq(const void* q, int dtype, int B, int Tq, int Hq, int Hkv, int D,
                 const float* ck, const uint8_t* kmask, int Dkc,
                 const float* cv, const uint8_t* vmask, int Dvc,
                 int M, int T, int t0, int N,
                 const void* k_keep, int64_t kk_stride_bh,
                 const void* v_keep, int64_t vk_stride_bh,
                 const void* k_full, const void* v_full, int W, int64_t full_stride_bh,
                 float scale, int num_splits, float* out,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fa_select_dims -- which head dimensions to compress (paper, Section 3.4).
 *
 * Every head dimension of the segment x[b,h] ([N, D], the middle rows of K or of V)
 * is compressed onto the first M basis functions and rebuilt (Eq. 3, then Eq. 6)
 * with the segment spanning exactly one period (T = N, positions 0 .. N-1);
 *     mse[b,h,d] = (1/N) sum_j ( x[j,d] - rebuilt[j,d] )^2 ,
 * and dim_mask[b,h,d] = 1 for the Dc dimensions of lowest mse (equal errors go to
 * the lower dimension index), 0 for the others: the mask fa_compress / fa_decode /
 * fa_append take.  Over one period the basis is orthogonal, so the error is
 * evaluated as (sum_j x^2 - sum_m w_m C[m,d]^2) / N from fp32 coefficients (bf16
 * segments are widened first); results below ~1e-5 of a dimension's mean square
 * are rounding noise and rank arbitrarily among themselves.
 *
 *   x         DEVICE, dtype elements, element strides as for fa_compress (rows
 *             16-byte aligned); read only
 *   M, Dc     1 <= M <= N; 0 <= Dc <= D
 *   dim_mask  DEVICE uint8 [B, H, D], written
 *   mse       DEVICE fp32 [B, H, D], written; may be NULL
 *   workspace DEVICE, 256-byte aligned, >= fa_select_workspace_bytes(...) bytes
 *             (holds the fp32 copy of a bf16 segment: 4*B*H*N*D bytes, the
 *             coefficients of all dims and the workspace of the projection)
 * Asynchronous on hip_stream; nothing is allocated.  Same limits as fa_compress.
 * Returns FA_OK or an FA_ERR_* code (arguments are checked on the host first).
 */
size_t fa_select_workspace_bytes(int dtype, int B, int H, int N, int D, int M);
int fa_select_dims(const void* x, int dtype,
                   int64_t sx_b, int64_t sx_h, int64_t sx_n,
                   int B, int H, int N, int D, int M, int Dc,
                   uint8_t* dim_mask, float* mse,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fa_legt_compress / fa_legt_mse -- the translated-Legendre (HiPPO-LegT) alternative basis that the
 * paper compares its Fourier basis with (Section 3.2; Section 5.1 and its reconstruction figure):
 * how well does each rebuild a KV dimension from the same number of states?  The paper gives no
 * formula for its LegT; the window is taken to be the segment itself, its N tokens at the cell
 * midpoints x_j = (2j+1)/N - 1 of [-1, 1]:
 *     coeffs[b,h,m,d] = sum_j P_m(x_j) x[b,h,j,d]                      (fa_legt_compress)
 *     mse[b,h,d] = (1/N) sum_j ( x[b,h,j,d] - sum_m (2m+1)/N coeffs[b,h,m,d] P_m(x_j) )^2   (fa_legt_mse)
 * with P_m the Legendre polynomial of degree m and (2m+1)/N the inverse of its squared norm under
 * the midpoint rule (sampled polynomials are orthogonal only up to that rule's O(1/N^2) error; the
 * oracle makes the same approximation).  The Fourier counterpart of mse is fa_select_dims' output.
 * All D head dims are processed (no mask): this is a calibration / ablation tool, not part of a
 * decode step.
 *
 *   x         DEVICE, dtype elements [B,H,N,D], element strides, dim stride 1; read only
 *   M         1 <= M <= N states per dimension (at most FA_MAX_STATES)
 *   coeffs    DEVICE fp32 [B,H,M,D]: written by fa_legt_compress, read by fa_legt_mse
 *   mse       DEVICE fp32 [B,H,D], written
 *   workspace DEVICE, 256-byte aligned, >= fa_legt_workspace_bytes(...) bytes
 * Asynchronous on hip_stream; nothing is allocated; arguments are checked on the host first.
 */
size_t fa_legt_workspace_bytes(int B, int H, int N, int D, int M);
int fa_legt_compress(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n,
                     int B, int H, int N, int D, int M, float* coeffs,
                     void* workspace, size_t workspace_bytes, void* hip_stream);
int fa_legt_mse(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n,
                int B, int H, int N, int D, int M, const float* coeffs, float* mse,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Measurement aids.  Same arguments and effect as fa_compress / fa_decode, but
 * synchronous: every kernel of the call is launched on `hip_stream` with its
 * own pair of HIP events, stamped by the runtime with the begin and the end of
 * that dispatch on the GPU (launch latency excluded); the call waits for the
 * stream, and the per-kernel durations in milliseconds are written to
 * `kernel_ms`, a HOST array:
 *   fa_compress_timed: 2 floats (projection, chunk reduction)
 *   fa_compress_kv_timed: 2 floats (projection of K and V, their chunk reductions;
 *                      sums over the two calls when the pair does not run as one launch)
 *   fa_decode_timed  : 3 floats (prepare, per-chunk partial, finish)
 * A kernel that was not launched for these sizes reports 0.
 */
int fa_compress_kv_timed(const void* k, const void* v, int dtype,
                         int64_t sx_b, int64_t sx_h, int64_t sx_n,
                         int B, int H, int N, int D,
                         const uint8_t* kmask, int Dkc, const uint8_t* vmask, int Dvc,
                         int M, int T, int t0, int accumulate,
                         float* ck, float* cv,
                         void* k_keep, int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh,
                         int keep_offset,
                         void* workspace, size_t workspace_bytes, void* hip_stream,
                         float* kernel_ms);
int fa_compress_timed(const void* x, int dtype,
                      int64_t sx_b, int64_t sx_h, int64_t sx_n,
                      int B, int H, int N, int D,
                      const uint8_t* dim_mask, int Dc,
                      int M, int T, int t0, int accumulate,
                      float* coeffs,
                      void* x_keep, int keep_layout, int64_t keep_stride_bh, int keep_offset,
                      void* workspace, size_t workspace_bytes, void* hip_stream,
                      float* kernel_ms);

int fa_decode_timed(const void* q, int dtype,
                    int B, int Hq, int Hkv, int D,
                    const float* ck, const uint8_t* kmask, int Dkc,
                    const float* cv, const uint8_t* vmask, int Dvc,
                    int M, int T, int t0, int N,
                    const void* k_keep, int64_t kk_stride_bh,
                    const void* v_keep, int64_t vk_stride_bh,
                    const void* k_full, const void* v_full, int W, int64_t full_stride_bh,
                    float scale, int num_splits,
                    float* out,
                    void* workspace, size_t workspace_bytes, void* hip_stream,
                    float* kernel_ms);

/* Number of middle-row chunks fa_decode will use for these sizes when
 * num_splits = 0 (exposed so callers can size and report); 0 for sizes
 * fa_decode rejects. */
int fa_decode_default_splits(int B, int Hq, int Hkv, int M, int N, int W);

/* Static description of a status code (never NULL). */
const char* fa_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FOURIER_ATTN_H */
