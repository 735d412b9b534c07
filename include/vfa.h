/*
 * vfa.h -- C ABI of libvfa.so: the VFA / VSA attention forward path for AMD MI355X (gfx950).
 *
 * Every pointer is a DEVICE pointer owned by the caller.  The library allocates nothing and
 * frees nothing.  Between calls it remembers only per-device facts that do not depend on the
 * arguments (the CU count, that a kernel's LDS limit has been raised, the address of its one
 * device array), held in atomics: calls may come from several host threads and for several
 * devices (the current device of the calling thread is used).  Calls are asynchronous: they
 * enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 * return; the caller keeps every buffer alive until the stream has passed the call.
 *
 * Tensor layouts (row-major, last index contiguous, 16-byte aligned base pointers):
 *   Q, O   [B, Hq,  N, d]  bf16
 *   K, V   [B, Hkv, N, d]  bf16       query head h reads KV head h / (Hq / Hkv)
 *   LSE    [B, Hq, N]      fp32       natural-log sum of exp of the scaled scores; may be NULL
 *   Krepr  [B, Hkv, ceil(N / block_n), d] bf16   key-block summaries (lives in `workspace`)
 *   skip_mask [B, Hq, ceil(N / block_m), ceil(N / block_n)] uint8; may be NULL
 *            0 = tile computed, 1 = tile skipped by the threshold test, 2 = tile not visited
 *
 * Supported shapes: d in {64, 128}; (block_m, block_n) in {(64, 64), (128, 64)}; any N >= 0
 * (ragged tails are masked); Hq a multiple of Hkv.  B == 0 or N == 0 is a successful no-op.
 * softmax_scale <= 0 selects 1 / sqrt(d).
 *
 * Return value: VFA_OK, or a negative code; vfa_strerror() names it.  Nothing is launched
 * when a negative code is returned, except VFA_ERR_HIP (a launch itself failed).
 * The functions never throw, abort or print.  Same inputs give bit-identical outputs.
 *
 * Calls may be recorded into a HIP graph (they only enqueue kernels; nothing is allocated, copied
 * or cleared).  One exception: the first launch, on each device, of an attention kernel that needs
 * more than 64 KiB of LDS (d = 128 with block_m = 128) sets that function attribute, so make one
 * ordinary call per entry point, device and process before capturing.
 */
#ifndef VFA_H_
#define VFA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VFA_OK 0
#define VFA_ERR_INVALID_ARG (-1) /* null/misaligned pointer, negative size, Hq % Hkv != 0, bad flag combination, workspace too small */
#define VFA_ERR_UNSUPPORTED (-2) /* d or block sizes outside the compiled set, sizes beyond 32-bit grid limits */
#define VFA_ERR_HIP (-3)         /* the HIP runtime reported a launch error */
#define VFA_ERR_TOO_LARGE (-4)   /* vfa_decode_noalloc_fwd only: the partial sums do not fit the library's fixed device array */

/* Bytes of `workspace` that vfa_attn_fwd / vsa_attn_fwd need (the Krepr tensor, rounded up
 * to 256 bytes).  Returns 0 for invalid arguments. */
size_t vfa_workspace_bytes(int B, int Hkv, int N, int d, int block_n);

/* Key-block summary pre-pass (Alg. 1, its first loop; Methods, Step 1):
 * Krepr[b, h, j, t] = the element of K[b, h, j*block_n : (j+1)*block_n, t] with the largest
 * absolute value, sign kept; when +a and -a tie, +a.  The result is an element of K, so bf16
 * is exact.  vfa_attn_fwd / vsa_attn_fwd run this themselves; it is exported for callers that
 * keep summaries across calls (a growing KV cache appends blocks). */
int vfa_kblock_summary(const void* K, void* Krepr, int B, int Hkv, int N, int d, int block_n,
                       void* stream);

/* The same pre-pass with the block representations of the k_repr ablation (Experiments, the
 * ablation of how k_repr is built): repr_mode 0 = sabsmax (as above), 1 = per-dimension maximum,
 * 2 = per-dimension mean (fp32 sum, rounded to bf16), 3 = per-dimension largest magnitude without
 * its sign.  VFA_ERR_INVALID_ARG for any other mode. */
int vfa_kblock_summary_mode(const void* K, void* Krepr, int B, int Hkv, int N, int d, int block_n,
                            int repr_mode, void* stream);

/* Conventional online-softmax forward (Table 1, FA column; Sec. 2.2 "Flash Attention"): key
 * blocks in ascending order, row max / rescale on every block.  The A/B comparison kernel. */
int fa_baseline_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B,
                    int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal,
                    float softmax_scale, void* stream);

/* Online softmax with conditional rescale: the second comparison kernel (related work, the
 * paragraph on FlashAttention-4; appendix, variant Blasst_FA4, its rescale-skip rule without the
 * block skipping).  As fa_baseline_fwd, except that a query
 * row adopts the new running max only when it exceeds the old one by more than
 * rescale_tau * ln 2 (rescale_tau >= 0, finite, in factors of two; 8 is the usual choice);
 * otherwise the row keeps its old max, its scale factor is exactly 1, and when this holds for
 * all 32 rows of a wave the rescale of l and O is not executed.  The output is the same exact
 * attention (the max cancels in O / l); exp(S - m) may reach 2^rescale_tau.  With rescale_tau = 0
 * every larger max is adopted, as in fa_baseline_fwd.  Same arguments, layouts and errors as
 * fa_baseline_fwd; VFA_ERR_INVALID_ARG for a negative or non-finite rescale_tau. */
int fa_lazy_rescale_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B,
                        int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal,
                        float softmax_scale, float rescale_tau, void* stream);

/* The second baseline with the other half of the same related work's recipe (FlashAttention-4, software
 * exponential): as fa_lazy_rescale_fwd, and every second exponential of a tile is computed without the
 * transcendental unit (range reduction, a cubic for 2^fraction on [0, 1) with relative error <= 2.1e-4,
 * the integer part added into the exponent field).  The result is the same attention to that error, far
 * below the bf16 rounding of P.  Same arguments, layouts and errors as fa_lazy_rescale_fwd. */
int fa_lazy_rescale_softexp_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B,
                                int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal,
                                float softmax_scale, float rescale_tau, void* stream);

/* VFA forward (Alg. 1).  For each query block: the running max starts at
 * m_init = max_j scale * Q_i . Krepr_j over the visible key blocks (use_minit = 1: the summaries
 * are computed into `workspace` first; use_minit = 2: `workspace` already holds them, e.g. from
 * vfa_kblock_summary on an earlier call; use_minit = 0: the max starts at -inf).  Key blocks
 * are visited as: the first n_sink blocks, then the local blocks (those overlapping the query
 * block's own token range plus the n_local-1 blocks before them; none if n_local == 0), then
 * all remaining visible blocks in ascending order, each block once.  Sink and
 * local blocks take the exact online-softmax update; all others reuse the frozen max (no row
 * max, no rescale).  O = acc / l, LSE = m + ln l.  Mathematically equal to exact attention.
 * use_minit == 0 with n_sink + n_local == 0 is rejected (the max would stay -inf).
 * `workspace` must hold vfa_workspace_bytes(...) bytes when use_minit != 0; use_minit = 1
 * overwrites it. */
int vfa_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq,
                 int Hkv, int N, int d, int block_m, int block_n, int causal, int n_sink,
                 int n_local, int use_minit, float softmax_scale, void* workspace,
                 size_t workspace_bytes, void* stream);

/* VSA forward (Alg. 2) = VFA plus the BLASST-style test on every visited tile: with
 * m~ = rowmax(S_ij) and m = the running max, the tile is skipped iff
 * m~ - max(m, m~) < -skip_threshold_nats for ALL rows of the query block
 * (skip_threshold_nats = -ln(lambda) > 0).  A skipped tile changes no state.  Rows whose
 * tiles were all skipped give O = 0, LSE = -inf.
 * What a skipped tile costs: its K tile, Q.K^T and the row max.  With d = 128 and block_m = 128
 * (the ping-pong kernel) its V tile is never requested, no exponential is computed and no P.V
 * runs: the decision is read one barrier after the vote, before any of them starts.  The other
 * shapes (generic kernel) save the exponentials and the P.V but have fetched V by then. */
int vsa_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int Hq,
                 int Hkv, int N, int d, int block_m, int block_n, int causal, int n_sink,
                 int n_local, int use_minit, float softmax_scale, float skip_threshold_nats,
                 unsigned char* skip_mask, void* workspace, size_t workspace_bytes, void* stream);

/* VFA / VSA with the switches of the ablation study and of the sparse-attention variants
 * (Experiments, the four ablation paragraphs: construction of k_repr, no m-initialisation, no
 * reordering, one summary per query block instead of row-wise approximate scores;
 * appendix: variants Blasst, Blasst_SWA, Blasst_Rowskip, Blasst_FA4).  As vfa_attn_fwd / vsa_attn_fwd,
 * plus:
 *   repr_mode  block representation used when use_minit == 1 (see vfa_kblock_summary_mode)
 *   q_repr_mode  0 = the approximate score uses each row of Q_i (the method); otherwise one summary
 *              q_repr_i of the query block replaces its rows, the scalar q_repr_i . k_repr_j seeds every
 *              row of the block alike: 1 = per-dimension largest magnitude of Q_i without its sign
 *              ("absmax"), 2 = sabsmax(Q_i), 3 = per-dimension mean of Q_i (fp32 sum, rounded to bf16).
 *              Needs use_minit == 1, and a workspace of vfa_workspace_bytes(B, Hkv, N, d, block_n) +
 *              vfa_workspace_bytes(B, Hq, N, d, block_m) bytes: the query-block summaries
 *              [B, Hq, ceil(N / block_m), d] are written behind the key-block summaries.
 *   reorder    1 = sink blocks, local blocks, then the rest (the method); 0 = ascending block
 *              order, the sink / local blocks keeping the exact-max update where they come
 *   freeze     1 = exact-max update on sink / local blocks only (the method); 0 = on every
 *              block (then n_sink = n_local = 0 with use_minit = 0 is allowed).  With freeze = 1 the
 *              max needs a value before the first frozen block: use_minit = 0 with reorder = 0 and
 *              n_sink = 0 (the first block in ascending order is an ordinary one) is rejected
 *   skip_threshold_nats  0 = no block skipping (skip_mask ignored); > 0 = the Alg. 2 skip test.
 *   rowskip    1 = Blasst_Rowskip: in a tile that is kept, a row that fails the threshold test is
 *              suppressed (scores -inf, its state untouched); needs skipping and freeze = 0
 *   lazy_rescale_tau  >= 0 = Blasst_FA4: on kept tiles a row keeps its old max while the new one
 *              exceeds it by at most tau * ln 2; negative = off; needs skipping and freeze = 0
 * reorder = freeze = 1, repr_mode = q_repr_mode = 0, rowskip = 0, tau < 0 is exactly vfa_attn_fwd /
 * vsa_attn_fwd.
 * Vanilla BLASST is (use_minit 0, reorder 0, freeze 0, threshold > 0); Blasst_SWA is the same with
 * reorder 1.
 * Every setting without skipping is exact attention; they differ in how far the frozen max sits
 * from the true one, which is what the ablation measures.  These run on the generic kernel. */
int vfa_variant_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B,
                    int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal,
                    int n_sink, int n_local, int use_minit, int repr_mode, int q_repr_mode, int reorder,
                    int freeze, int rowskip, float lazy_rescale_tau, float softmax_scale,
                    float skip_threshold_nats, unsigned char* skip_mask, void* workspace,
                    size_t workspace_bytes, void* stream);

/* Summaries of a growing key cache (Methods, Step 1: during decoding only newly appended key blocks
 * need their summary computed).  K is a cache
 * [B, Hkv, n_cap, d] whose first n_new rows are valid, of which rows [n_old, n_new) are new;
 * Krepr is [B, Hkv, ceil(n_cap / block_n), d] (vfa_workspace_bytes(B, Hkv, n_cap, d, block_n)
 * bytes).  Recomputes exactly the summaries of the blocks that contain new rows (a partly filled
 * last block is summarised over its valid rows); all others are left as they are.
 * VFA_ERR_INVALID_ARG unless 0 <= n_old <= n_new <= n_cap. */
int vfa_kblock_summary_append(const void* K, void* Krepr, int B, int Hkv, int n_cap, int n_old,
                              int n_new, int d, int block_n, void* stream);

/* Bytes of workspace vfa_decode_fwd needs (partial sums of n_splits key ranges per query head). */
size_t vfa_decode_workspace_bytes(int B, int Hq, int d, int n_splits);

/* Decode step (Alg. 1 with one query token per head that sees every cached key; the split over
 * key ranges uses Step 3: once the max is frozen, partial sums need no rescale).
 *   Q [B, Hq, d], O [B, Hq, d] bf16; LSE [B, Hq] fp32 or NULL
 *   K, V [B, Hkv, n_cap, d] bf16, rows [0, n_keys) valid (rows beyond are never read)
 *   Krepr  summaries of those n_keys rows, laid out for n_cap (see vfa_kblock_summary_append);
 *          read when use_minit == 1, may be NULL when use_minit == 0
 * The running max is m = max(m_init, exact row max over the first n_sink and the last n_local key
 * blocks), m_init = max_j scale * q . Krepr_j (or -inf); the cache is cut into n_splits ranges of
 * whole blocks; each range accumulates sum exp(s - m) and sum exp(s - m) v; the ranges are added in
 * index order (bit-identical results from run to run), divided, and LSE = m + ln l.  The result is
 * exact attention over the n_keys rows.  n_splits >= 1 (ranges may be empty; up to four (KV head, range) pairs
 * share a compute unit, and B * Hkv * n_splits of 1.5 to 4 times the number of compute units runs within a few
 * percent of the best); Hq / Hkv <= 32;
 * block_n = 64; d in {64, 128}.  workspace: vfa_decode_workspace_bytes(...) bytes, 16-byte aligned,
 * contents irrelevant on entry.  VFA_ERR_INVALID_ARG for n_keys < 1 or > n_cap, for
 * use_minit == 0 with n_sink + n_local == 0, and for the pointer / size errors listed above. */
int vfa_decode_fwd(const void* Q, const void* K, const void* V, const void* Krepr, void* O,
                   float* LSE, int B, int Hq, int Hkv, int n_cap, int n_keys, int d, int block_n,
                   int n_sink, int n_local, int use_minit, int n_splits, float softmax_scale,
                   void* workspace, size_t workspace_bytes, void* stream);

/* vfa_decode_fwd for callers that cannot allocate and have no workspace to hand over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, layouts, kernels
 * and results (bit for bit) as vfa_decode_fwd, minus the workspace: the partial sums of the key ranges live
 * in one fixed array of VFA_DECODE_NOALLOC_MAX_BYTES bytes of device memory that is part of the library's
 * code object (each device the library is used on holds one copy until the process ends).  The call
 * allocates nothing, frees nothing, clears nothing (every slot that is read is written earlier in the same
 * call) and enqueues the same three kernels on `stream`.
 * Limit: B * Hq * n_splits * (2 + d) * 4 bytes <= VFA_DECODE_NOALLOC_MAX_BYTES (4 MiB: 8065 (head, range)
 * rows at d = 128, e.g. B * Hq = 504 with 16 ranges), else VFA_ERR_TOO_LARGE and nothing is launched.
 * The first call on a device looks the array's address up (hipGetSymbolAddress; VFA_ERR_HIP if that fails):
 * make it outside graph capture.
 * All calls on one device share the array: two calls that may run at the same time on one device (different
 * streams, or replays of two graphs) race on it and must be serialised by the caller; calls on one stream are
 * ordered and safe.  The array keeps the last call's contents, which no later call reads. */
#define VFA_DECODE_NOALLOC_MAX_BYTES (4u << 20)
int vfa_decode_noalloc_fwd(const void* Q, const void* K, const void* V, const void* Krepr, void* O,
                           float* LSE, int B, int Hq, int Hkv, int n_cap, int n_keys, int d,
                           int block_n, int n_sink, int n_local, int use_minit, int n_splits,
                           float softmax_scale, void* stream);

/* The two decode calls for a batch whose sequences have different lengths.  old_lens / new_lens /
 * seq_lens are DEVICE arrays of B ints (4-byte aligned), read by the kernels (the host never looks at
 * them, so a serving loop can update them on the GPU): sequence b has seq_lens[b] valid rows in its
 * part of the cache, values are clamped to [1, n_cap] (to [0, n_cap] in the append call, where
 * old >= new means nothing to do).  Everything else as in vfa_kblock_summary_append / vfa_decode_fwd;
 * each sequence's key range is cut into n_splits ranges of its own length. */
int vfa_kblock_summary_append_varlen(const void* K, void* Krepr, int B, int Hkv, int n_cap,
                                     const int* old_lens, const int* new_lens, int d, int block_n,
                                     void* stream);
int vfa_decode_varlen_fwd(const void* Q, const void* K, const void* V, const void* Krepr, void* O,
                          float* LSE, int B, int Hq, int Hkv, int n_cap, const int* seq_lens, int d,
                          int block_n, int n_sink, int n_local, int use_minit, int n_splits,
                          float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

/* ---- FP8 (E4M3) path: the 8-bit tensor regime of the paper's performance discussion ("C8V32":
 * both matrix products in 8 bit, softmax arithmetic in fp32).  The paper gives no quantisation
 * scheme; this one is per-tensor: x8 = E4M3(x * inv_scale), round to nearest even, saturated at
 * +-448, and the attention call receives the matching descale factors (1 / inv_scale).
 * Only d = 128 with 128x64 blocks. ---- */

/* X (bf16, n elements, n a multiple of 8, 16-byte aligned) -> X8 (n E4M3 codes, same order). */
int vfa_fp8_quantize(const void* X, void* X8, long long n, float inv_scale, void* stream);

/* V [B, Hkv, N, 128] bf16 -> Vt8 [B, Hkv, ceil(N/64), 128, 64] E4M3: per 64-key tile a block of 128
 * feature rows by 64 keys, the keys in the order the P.V operand wants them (byte 32 h + j of a row
 * is key 32 (j/16) + 8 ((j%16)/4) + 4 h + j%4 of the tile); keys beyond N are written as zero.
 * vfa_fp8_v_bytes gives the size of Vt8. */
size_t vfa_fp8_v_bytes(int B, int Hkv, int N);
int vfa_fp8_pack_v(const void* V, void* Vt8, int B, int Hkv, int N, int d, float inv_scale, void* stream);

/* Attention forward on E4M3 operands.  frozen = 0: online softmax on every block (the FA column of
 * Table 1); frozen = 1: Alg. 1 (summaries are the sabsmax of the K codes, an element of K8 again;
 * n_sink, n_local, use_minit as in vfa_attn_fwd, with workspace >= B * Hkv * ceil(N/64) * 128 bytes).
 * Scores are (code products) * descale_q * descale_k * softmax_scale; exp(S - m) is rounded to E4M3
 * scaled by 2^8 (frozen = 0) or 2^4 (frozen = 1, leaving 4 binades for scores above the frozen max;
 * beyond them exp is capped, never NaN); l sums the unrounded values; O = descale_v * (P8 V8) / l is
 * written in bf16 and LSE in fp32 as in the bf16 entry points.  Q8, K8 [B, H, N, 128] codes.
 * With frozen = 1, a caller who quantises Q at a scale that makes descale_q * descale_k * softmax_scale *
 * log2(e) a power of two (to 2^-18 relative) gets a faster kernel with the same result: that factor is then
 * applied inside the matrix instruction and the frozen max enters as the accumulators' start value, so no
 * per-score multiply or subtract is left (the performance discussion's point that a max known in advance
 * takes vector work off the path; an online max cannot be folded this way).
 * Errors as vfa_attn_fwd; VFA_ERR_UNSUPPORTED unless d = 128, block_m = 128, block_n = 64. */
int vfa_fp8_attn_fwd(int frozen, const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE,
                     int B, int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal,
                     int n_sink, int n_local, int use_minit, float softmax_scale, float descale_q,
                     float descale_k, float descale_v, void* workspace, size_t workspace_bytes,
                     void* stream);

/* Alg. 1 on E4M3 operands WITHOUT exponentials.  Needs what the fast path of vfa_fp8_attn_fwd needs (descale_q *
 * descale_k * softmax_scale * log2(e) a power of two to 2^-18, else VFA_ERR_INVALID_ARG), because the scale and
 * the frozen max must sit inside the matrix instruction.  The code of a small float read as an integer is a
 * piecewise-linear logarithm of its value, so the E5M2 code of exp(S - m) is obtained from the score by a
 * multiply-add (folded into the instruction) and one float-to-byte conversion: each weight is within
 * [-11 %, +12 %] of the exact one (the format's own rounding would be +-12.5 %), and the row sum is taken over the
 * SAME rounded weights by one more matrix instruction, so O is a properly normalised average of V under those
 * weights (measured: mean-abs error as the rounded-exponential path, max-abs within 2^-3 max|V|).  LSE is computed
 * from that row sum: within 0.12 nats of the exact value.  This is the performance discussion's argument taken to
 * its end for 8-bit P: with the max known before the tile, no per-score vector arithmetic but a clamp and a
 * conversion is left.  Everything else as vfa_fp8_attn_fwd with frozen = 1 (sink / local blocks keep the
 * exact-max update, one exponential per row and block there). */
int vfa_fp8_attn_noexp_fwd(const void* Q8, const void* K8, const void* Vt8, void* O, float* LSE, int B,
                           int Hq, int Hkv, int N, int d, int block_m, int block_n, int causal,
                           int n_sink, int n_local, int use_minit, float softmax_scale, float descale_q,
                           float descale_k, float descale_v, void* workspace, size_t workspace_bytes,
                           void* stream);

/* ---- MXFP4 scores: the 4-bit tensor regime of the performance discussion (the "C4" configurations):
 * Q.K^T on operands in the published MX block format (E2M1 elements, two to a byte with the even
 * element in the low nibble, and one E8M0 scale byte 2^(byte - 127) per 32 consecutive features);
 * P.V as in the FP8 path (exp(S - m) and V in E4M3), softmax arithmetic in fp32.  The paper gives no
 * quantisation scheme; this is the MX one.  Only d = 128 with 128x64 blocks. ---- */

/* X (bf16, n elements, n a multiple of 32, 16-byte aligned; blocks of 32 never straddle rows when d is a
 * multiple of 32) -> X4 (n/2 bytes) and XS (n/32 scale bytes).  y = x * pre_scale in fp32; scale byte =
 * floor(log2(max|y| of the block)) - 2 + 127, at least 0 (an all-zero block gets 0); element = y / scale
 * rounded to the nearest of 0, 0.5, 1, 1.5, 2, 3, 4, 6, ties to the even mantissa, saturated at 6. */
int vfa_mxfp4_quantize(const void* X, void* X4, void* XS, long long n, float pre_scale, void* stream);

/* Bytes of workspace of vfa_mxfp4_attn_fwd (the key-block summaries), 0 for invalid arguments. */
size_t vfa_mxfp4_workspace_bytes(int B, int Hkv, int N);

/* Attention forward with MXFP4 scores.  Q4 [B, Hq, N, 64] and QS [B, Hq, N, 4], K4 [B, Hkv, N, 64] and
 * KS [B, Hkv, N, 4] from vfa_mxfp4_quantize (scale arrays 4-byte aligned); Vt8 from vfa_fp8_pack_v with
 * its descale_v.  Scores are (dequantised Q) . (dequantised K) * softmax_scale.  frozen = 0: online softmax
 * on every block; frozen = 1: Alg. 1, the summaries being the sabsmax of the dequantised keys held as MX
 * blocks of E5M2 elements (use_minit = 1 computes them into the workspace: [B, Hkv, Tc, 128] codes followed
 * by [B, Hkv, Tc, 4] scale bytes; 2 = the workspace already holds them).  l, O and LSE as in
 * vfa_fp8_attn_fwd; exp(S - m) is rounded to E4M3 scaled by 2^8 for frozen = 0 and to E5M2 scaled by 2^15 for
 * frozen = 1 (one mantissa bit less, 14 binades more: summaries of 4-bit keys collect the upward rounding
 * errors of a whole block, so the seeded max can sit many binades above the scores; the 4 binades of headroom
 * for scores ABOVE the frozen max are the same).  With frozen = 1 and softmax_scale * log2(e) = 1 (to 2^-18: the caller multiplied Q by
 * its scale * log2(e) before quantising and passes softmax_scale = ln 2) the frozen max enters as the start
 * value of the matrix instruction's accumulators and no per-score arithmetic but exp is left.
 * Errors as vfa_fp8_attn_fwd. */
int vfa_mxfp4_attn_fwd(int frozen, const void* Q4, const void* QS, const void* K4, const void* KS,
                       const void* Vt8, void* O, float* LSE, int B, int Hq, int Hkv, int N, int d,
                       int block_m, int block_n, int causal, int n_sink, int n_local, int use_minit,
                       float softmax_scale, float descale_v, void* workspace, size_t workspace_bytes,
                       void* stream);

/* vfa_mxfp4_attn_fwd's Alg. 1 without exponentials, as vfa_fp8_attn_noexp_fwd: needs softmax_scale * log2(e) = 1
 * (to 2^-18, else VFA_ERR_INVALID_ARG; the caller multiplied Q by its scale * log2(e) before quantising); the
 * factor 4 of the code scale rides in the queries' block-scale bytes (which must stay below 253).  Weights within
 * [-11 %, +12 %] of the exact ones, normalised by their own sum; LSE within 0.12 nats. */
int vfa_mxfp4_attn_noexp_fwd(const void* Q4, const void* QS, const void* K4, const void* KS,
                             const void* Vt8, void* O, float* LSE, int B, int Hq, int Hkv, int N, int d,
                             int block_m, int block_n, int causal, int n_sink, int n_local,
                             int use_minit, float softmax_scale, float descale_v, void* workspace,
                             size_t workspace_bytes, void* stream);

/* Static string for a return code. */
const char* vfa_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* VFA_H_ */
