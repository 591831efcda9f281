/*
 * svg.h -- C ABI of the MI355X (gfx950) sparse 3D attention library.
 *
 * The library implements the attention hot path of Sparse VideoGen
 * (arXiv 2502.01776): per-head online profiling (Alg. 1, Sec. 4.1), the layout
 * transformation that makes the temporal pattern block-contiguous and its
 * inverse (Sec. 4.2, Fig. 4), a block-sparse FlashAttention-style forward pass
 * over the kept tiles (Sec. 4.3), and a dense forward pass as the in-library
 * baseline (the paper's baseline is dense FlashAttention, Sec. 5.3); further the
 * fused QK-norm + rotary embedding pass in front of the attention (Sec. 4.3,
 * Table 2) and the FP8 variant of the sparse pass (Sec. 4.3 "Quantization").
 *
 * Conventions for every entry point
 *   - Tensors q, k, v, o are DEVICE pointers to contiguous bf16 arrays of shape
 *     [B, H, N, D], N = F*P + T, 16-byte aligned.  A video token of frame f and
 *     in-frame position p sits at row off + f*P + p ("F-outer" order), where
 *     off = T if text_first else 0; the T text tokens occupy [0,T) or [F*P,N).
 *     The transformed ("P-outer") order puts that token at row off + p*F + f.  With
 *     sink_first_frame set it keeps frame 0 together instead: row off + p for f = 0 and
 *     row off + P + p*(F-1) + (f-1) for the other frames, so that the first-frame keys,
 *     which every query keeps (Sec. 3.1), are ceil(P/block_n) contiguous key tiles for a
 *     temporal head as well.
 *   - All pointers are owned by the caller.  The library allocates no device
 *     memory, keeps no state between calls, and never synchronises the host:
 *     kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns.
 *   - Return value: SVG_OK (0) or a negative svg_status.  Arguments are checked on
 *     the host before anything is launched; on error nothing is enqueued.
 *   - Head labels: SVG_HEAD_SPATIAL (0) or SVG_HEAD_TEMPORAL (1), one uint8 per
 *     (b,h), index b*H + h.  Alg. 1's boolean best_mask_config is true for spatial.
 */
#ifndef SVG_H_
#define SVG_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct svg_shape {
  int32_t B, H;             /* batch, heads                                         */
  int32_t F, P, T;          /* frames, tokens per frame, text tokens; N = F*P + T   */
  int32_t D;                /* head dimension: 64 or 128                            */
  int32_t text_first;       /* 1: text rows are [0,T); 0: text rows are [F*P, N)    */
  int32_t w_s;              /* spatial half-window, frames:   keep |f_i-f_j| <= w_s */
  int32_t w_t;              /* temporal half-window, positions: keep |p_i-p_j| <= w_t */
  int32_t sink_first_frame; /* 0/1: both patterns also keep the keys of frame 0 (Sec. 3.1) */
  int32_t block_m, block_n; /* query-tile rows x key-tile columns: 128x64 or 32x32  */
  float softmax_scale;      /* <= 0 selects 1/sqrt(D)                               */
} svg_shape_t;

enum { SVG_HEAD_SPATIAL = 0, SVG_HEAD_TEMPORAL = 1 };
/* A third list pattern for svg_tile_list_build only (never a head label): the temporal
 * mask for a head LEFT in frame-major order, i.e. without the layout transformation.  It
 * exists for the comparison of Sec. 5.5 / Fig. 7 (sparse attention with and without the
 * transformation): in frame-major order the kept keys of a query tile are one short run
 * per frame, so many more tiles hold at least one of them. */
enum { SVG_LIST_TEMPORAL_FRAME_MAJOR = 2 };

typedef enum svg_status {
  SVG_OK = 0,
  SVG_ERR_INVALID_ARG = -1, /* NULL pointer, non-positive size, misaligned tensor, bad pattern */
  SVG_ERR_UNSUPPORTED = -2, /* D or tile size the kernels are not built for, N too large */
  SVG_ERR_WORKSPACE = -3,   /* workspace missing or smaller than svg_workspace_bytes() */
  SVG_ERR_ALIAS = -4,       /* in and out overlap where they must not */
  SVG_ERR_HIP = -5          /* the HIP runtime reported a launch error */
} svg_status;

/* Text for a status code; never NULL. */
const char* svg_strerror(int status);

/* Text of the HIP error behind the calling thread's most recent SVG_ERR_HIP
 * ("no error" if there was none). */
const char* svg_last_hip_error(void);

/* Library version, "major.minor". */
const char* svg_version(void);

/* Bytes of device workspace svg_profile_heads needs for `t` sampled rows (fp32
 * partial outputs of shape [B,H,t,D] and per-row softmax statistics for every part
 * the three passes of Alg. 1 are cut into, see svg_profile_plan, and an int32[t] row
 * order); also enough for every other call that takes a workspace.  0 if shape is
 * invalid. */
size_t svg_workspace_bytes(const svg_shape_t* shape, int32_t t);

/* How svg_profile_heads cuts the passes of Alg. 1 into workgroups for this shape and
 * t (a pure function of both; host side, nothing is launched).  The unmasked pass of a
 * group of sampled rows runs as *n_full parts over the key tiles
 * [full_bound[c], full_bound[c+1]), c < *n_full (full_bound: host array of 17
 * entries, ascending from 0 to nk; may be NULL), each masked pass as *n_masked <= 4
 * equal parts of its own tile sequence, *n_full <= 6; the parts are merged from per-row (output,
 * maximum, row sum) triples, so the plan changes the results only in fp32 rounding. */
int svg_profile_plan(const svg_shape_t* shape, int32_t t, int32_t* n_full, int32_t* n_masked,
                     int32_t* full_bound);

/* Number of query tiles and key tiles: ceil(N/block_m), ceil(N/block_n). */
int svg_tile_counts(const svg_shape_t* shape, int32_t* nq, int32_t* nk);

/*
 * Kept-tile list of one pattern (Fig. 4; Sec. 4.3 "block sparse attention").
 * HOST function, pure in its arguments.  pattern is SVG_HEAD_SPATIAL (rows and
 * columns in F-outer order), SVG_HEAD_TEMPORAL (P-outer order) or
 * SVG_LIST_TEMPORAL_FRAME_MAJOR (temporal mask, F-outer order).  Tile (a,b)
 * covers rows [a*block_m, min(N,(a+1)*block_m)) and columns
 * [b*block_n, min(N,(b+1)*block_n)) and is kept iff at least one (query, key)
 * pair inside it is kept by the pattern's element mask: either token is text, or
 * |f_i-f_j| <= w_s (spatial) / |p_i-p_j| <= w_t (temporal), or the key is in
 * frame 0 and sink_first_frame is set (Sec. 3.1, Sec. 3.3).
 *   row_ptr  host int32 [nq+1], written always
 *   col_idx  host int32 [cap], ascending within a row; may be NULL for a size query
 *   nnz_out  receives the number of kept tiles
 * If col_idx is non-NULL and cap < nnz: SVG_ERR_INVALID_ARG, nnz_out still set.
 */
int svg_tile_list_build(const svg_shape_t* shape, int pattern, int32_t* row_ptr,
                        int32_t* col_idx, int64_t cap, int64_t* nnz_out);

/*
 * Online profiling (Alg. 1; Sec. 4.1).  For every head and each of the t sampled
 * query rows, computes attention against ALL keys three times -- unmasked, with
 * the spatial element mask and with the temporal element mask, all in the
 * original F-outer order -- then MSE_x = mean over (row, channel) of
 * (O_full - O_x)^2, and label = spatial iff MSE_s < MSE_t (ties: temporal).
 *   q, k, v   device bf16 [B,H,N,D], F-outer order
 *   rows      device int32 [t], each in [0,N) (not checked: out-of-range rows are
 *             undefined behaviour); one set shared by all heads
 *   labels    device uint8 [B*H], written
 *   mse       device float [B*H*2] = {MSE_s, MSE_t} per head, written; may be NULL
 *   workspace device, >= svg_workspace_bytes(shape, t), 16-byte aligned
 * Runs bf16 MFMA with fp32 accumulation and fp32 softmax; results are
 * deterministic (no atomics).
 */
int svg_profile_heads(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                      const int32_t* rows, int32_t t, uint8_t* labels, float* mse,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * svg_profile_heads for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same computation, same kernels, same results bit for bit; the workspace is an
 * array of SVG_STATIC_SCRATCH_BYTES that is part of the library's code object (each GPU the
 * library runs on holds one copy until the process ends).  The call allocates and frees
 * nothing.  A shape and t with svg_workspace_bytes(shape, t) > SVG_STATIC_SCRATCH_BYTES is
 * refused with SVG_ERR_WORKSPACE before anything is enqueued (160 MiB covers every benchmark
 * shape at 1 % sampled rows, the 119k-token one needs 119 MB).  All calls on one GPU share
 * that GPU's array: calls that overlap in time on one GPU (other streams, other threads)
 * race; calls ordered on one stream do not.  Nothing in the array has to be cleared between
 * calls.
 */
#define SVG_STATIC_SCRATCH_BYTES (160u << 20)
int svg_profile_heads_static(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                             const int32_t* rows, int32_t t, uint8_t* labels, float* mse, void* stream);

/*
 * Layout transformation (Sec. 4.2, Fig. 4): for heads labelled temporal,
 * out[b,h, off + p*F + f, :] = in[b,h, off + f*P + p, :]; text rows and heads
 * labelled spatial are copied unchanged, so `out` is always fully written.
 * labels == NULL treats every head as temporal.  in and out must not overlap
 * (SVG_ERR_ALIAS).  Bit-exact data movement.
 */
int svg_layout_fwd(const svg_shape_t* shape, const void* in, void* out, const uint8_t* labels,
                   void* stream);

/* Inverse of svg_layout_fwd: out[b,h, off + f*P + p, :] = in[b,h, off + p*F + f, :]
 * for temporal heads; everything else copied. */
int svg_layout_inv(const svg_shape_t* shape, const void* in, void* out, const uint8_t* labels,
                   void* stream);

/*
 * Block-sparse attention forward (Sec. 4.3).  For each head and query tile a,
 * o[rows of a] = softmax(scale * q k^T) v over all in-range keys of the key tiles
 * listed for a in that head's tile list; tiles not listed are never read.
 * Head (b,h) uses the spatial list if labels[b*H+h] == SVG_HEAD_SPATIAL and the
 * temporal list otherwise; labels == NULL uses the spatial list for all heads.
 *   q, k, v, o  device bf16 [B,H,N,D]; temporal heads are expected in P-outer
 *               order (svg_layout_fwd applied) and o is written in the same order
 *               as q (apply svg_layout_inv afterwards)
 *   row_ptr_*   device int32 [nq+1];  col_idx_*  device int32 [nnz]  (CSR from
 *               svg_tile_list_build, uploaded by the caller; the temporal pair may
 *               be NULL when labels == NULL).  Entries are not range-checked on
 *               the device: a column >= nk is undefined behaviour.
 * A query tile with an empty list yields zeros.  workspace is reserved (may be
 * NULL, 0).
 */
int svg_sparse_attn_fwd(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                        void* o, const uint8_t* labels, const int32_t* row_ptr_s,
                        const int32_t* col_idx_s, const int32_t* row_ptr_t,
                        const int32_t* col_idx_t, void* workspace, size_t workspace_bytes,
                        void* stream);

/*
 * svg_sparse_attn_fwd with options.  flags == 0 is svg_sparse_attn_fwd itself.
 * SVG_ATTN_QO_TOKEN_ORDER folds two of the four layout passes of Sec. 4.2 into the
 * attention kernel (the paper fuses the transformation into its kernels as well,
 * Sec. 4.3): q is read and o is written in the original token order for every head,
 * the kernel gathering the query rows of a temporal head's tile and scattering its
 * output rows through the permutation; only k and v of temporal heads must be in
 * P-outer order.  Results are bit-identical to svg_layout_fwd(q) ->
 * svg_sparse_attn_fwd -> svg_layout_inv(o).
 * SVG_ATTN_ELEMENT_MASK applies the element mask of the head's pattern (Sec. 3.1: frames
 * within w_s of the query's frame for a spatial head, in-frame positions within w_t for a
 * temporal head; text keys, text queries and, if set, the first-frame sink always kept)
 * inside every visited tile, so that the result is attention under the exact mask
 * instead of its block cover.  The tile list still decides which tiles are visited (with
 * the lists of svg_tile_list_build no kept element is lost); temporal heads are expected in
 * P-outer order as usual.
 * SVG_ATTN_KV_TOKEN_ORDER folds the remaining two layout passes into the kernel as well
 * (Sec. 4.3): k and v of EVERY head stay in the original token order, and a temporal head's
 * key tile is gathered row by row (a row is 2*D contiguous bytes) from where the
 * transformation of Sec. 4.2 would have taken it.  Together with SVG_ATTN_QO_TOKEN_ORDER no
 * layout pass and no second copy of any tensor is left; results are bit-identical to the
 * passes it replaces.  It needs workspace_bytes >= 8 * nk * block_n (nk from svg_tile_counts;
 * svg_workspace_bytes covers it) for the table of source rows, which the call itself fills
 * (SVG_ERR_WORKSPACE if NULL or too small, SVG_ERR_ALIAS if it overlaps a tensor), and
 * block_m = 128; combined with SVG_ATTN_ELEMENT_MASK or block_m = 32: SVG_ERR_UNSUPPORTED.
 * Unknown flag bits: SVG_ERR_INVALID_ARG.
 */
enum { SVG_ATTN_QO_TOKEN_ORDER = 1, SVG_ATTN_ELEMENT_MASK = 2, SVG_ATTN_KV_TOKEN_ORDER = 4 };
int svg_sparse_attn_fwd_ex(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                           void* o, const uint8_t* labels, const int32_t* row_ptr_s,
                           const int32_t* col_idx_s, const int32_t* row_ptr_t,
                           const int32_t* col_idx_t, uint32_t flags, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * The sparse pass of one layer with as little layout traffic as the method needs (Sec. 4.2,
 * Sec. 4.3: the transformation is fused into the kernels).  Only k and v of the heads
 * labelled temporal are moved at all:
 *   svg_layout_kv_temporal   one launch: for every head labelled temporal,
 *       k_t[b,h, off + p*F + f, :] = k[b,h, off + f*P + p, :] and likewise v_t from v (text
 *       rows copied); the slots of heads labelled spatial in k_t, v_t are NOT written (and
 *       never read by the call below).  k_t, v_t: device bf16 [B,H,N,D], distinct from k, v
 *       and from each other (SVG_ERR_ALIAS).  labels must not be NULL.
 *   svg_sparse_attn_fwd_kv2  block-sparse attention in which a head labelled spatial reads k, v
 *       (original order) and a head labelled temporal reads k_t, v_t; q is read and o written
 *       in the original token order for every head (as with SVG_ATTN_QO_TOKEN_ORDER).  Results
 *       are bit-identical to svg_layout_fwd(q, k, v) -> svg_sparse_attn_fwd -> svg_layout_inv(o).
 *       flags: 0 or SVG_ATTN_ELEMENT_MASK.  labels and both tile lists are required.
 */
int svg_layout_kv_temporal(const svg_shape_t* shape, const void* k, const void* v, void* k_t, void* v_t,
                           const uint8_t* labels, void* stream);
int svg_sparse_attn_fwd_kv2(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                            const void* k_t, const void* v_t, void* o, const uint8_t* labels,
                            const int32_t* row_ptr_s, const int32_t* col_idx_s, const int32_t* row_ptr_t,
                            const int32_t* col_idx_t, uint32_t flags, void* stream);

/*
 * Dense attention forward, o = softmax(scale * q k^T) v per head: the baseline
 * the paper measures against (Sec. 5.3) and the pass used on the dense warm-up
 * steps (Sec. 5.1).  Same tensors and precision as svg_sparse_attn_fwd; every
 * tile is computed.  workspace is reserved (may be NULL, 0).
 */
int svg_dense_attn_fwd(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                       void* o, void* workspace, size_t workspace_bytes, void* stream);

/*
 * QK-norm and rotary position embedding of one tensor (q or k) in one pass: the two small
 * per-token operations in front of the attention that the paper customises for small head
 * dimensions (Sec. 4.3 "Efficient kernel customization", Table 2).  The paper gives no
 * formulas; these are the definitions of the models it evaluates:
 *   norm     SVG_NORM_NONE, SVG_NORM_RMS  y = x / sqrt(mean(x^2) + eps) * weight, or
 *            SVG_NORM_LAYER  y = (x - mean) / sqrt(var + eps) * weight + bias (biased
 *            variance), per token over the D channels of a head; weight, bias device
 *            float [D], NULL means 1 and 0
 *   rotation cos, sin device float [F*P, D/2], one row per VIDEO token in token order (both
 *            NULL: no rotation); channel pair i of video token v becomes
 *            (a cos[v,i] - b sin[v,i], b cos[v,i] + a sin[v,i]) with (a, b) = (x[2i], x[2i+1])
 *            for SVG_ROPE_INTERLEAVED and (x[i], x[i+D/2]) for SVG_ROPE_HALF; text tokens
 *            are not rotated.  The norm is applied first.
 *   x, y     device bf16 [B,H,N,D], token order; y == x (in place) is allowed, any other
 *            overlap is SVG_ERR_ALIAS.  Arithmetic in fp32, output rounded to bf16.
 */
enum { SVG_NORM_NONE = 0, SVG_NORM_RMS = 1, SVG_NORM_LAYER = 2 };
enum { SVG_ROPE_INTERLEAVED = 0, SVG_ROPE_HALF = 1 };
int svg_qk_norm_rope(const svg_shape_t* shape, const void* x, void* y, int norm, const float* weight,
                     const float* bias, float eps, const float* cos, const float* sin, int pairing,
                     void* stream);

/*
 * FP8 attention (Sec. 4.3 "Quantization", Sec. 5.2: FP8 quantisation of the sparse
 * attention, applied at head dimension 128).  The paper names no format or scaling;
 * this library uses OCP E4M3 (largest finite value 448) with one scale per head and
 * tensor, scale = float32(max|x| / 448) (1 for an all-zero head), x ~ code * scale, code =
 * the E4M3 value nearest to x / scale, ties to even.  The quotient is formed in float32 as
 * x * (1 / scale): where the exact quotient lies within two float32 roundings (2^-23
 * relative) of the midpoint of two E4M3 values, either neighbour may be returned.  Head
 * dimension 128 and 128 x 64 tiles only, otherwise SVG_ERR_UNSUPPORTED.
 *
 * svg_fp8_quantize converts q, k, v (device bf16 [B,H,N,128], token order) into
 *   q8      uint8 [B,H,N,128], token order
 *   k8      uint8 [B,H,nk*64,128]: rows beyond N are zero; heads labelled temporal are
 *           written in P-outer order (the layout transformation of Sec. 4.2 is applied on
 *           the way, so no svg_layout_fwd is needed)
 *   v8t     uint8 [B,H,nk,8192]: per 64-key tile a transposed image in the order the
 *           attention kernel stages it (opaque to the caller), same head order as k8
 *   scales  float [6*B*H]: [0,B*H) scale of q per head, then k, then v; the rest is
 *           scratch of the call
 * labels == NULL leaves every head in token order.  Buffer sizes in bytes:
 * svg_fp8_buffer_bytes(shape, SVG_FP8_Q / _K / _VT / _SCALES) (0 for an unsupported shape).
 * All buffers caller-owned, 16-byte aligned, and distinct from each other and from q, k, v
 * (SVG_ERR_ALIAS otherwise; likewise o of svg_sparse_attn_fp8_fwd against its inputs).
 *
 * svg_sparse_attn_fp8_fwd is svg_sparse_attn_fwd_ex(SVG_ATTN_QO_TOKEN_ORDER) on those
 * buffers: o (device bf16 [B,H,N,128]) is written in token order for every head, labels
 * and tile lists as for svg_sparse_attn_fwd (pass the labels given to svg_fp8_quantize).
 * Both matrix products run on the FP8 matrix cores with fp32 accumulation; the attention
 * weights are rounded to E4M3 for the second product and the row sums are taken over the
 * rounded weights.
 */
enum { SVG_FP8_Q = 0, SVG_FP8_K = 1, SVG_FP8_VT = 2, SVG_FP8_SCALES = 3 };
size_t svg_fp8_buffer_bytes(const svg_shape_t* shape, int which);
int svg_fp8_quantize(const svg_shape_t* shape, const void* q, const void* k, const void* v,
                     const uint8_t* labels, void* q8, void* k8, void* v8t, float* scales,
                     void* stream);
int svg_sparse_attn_fp8_fwd(const svg_shape_t* shape, const void* q8, const void* k8,
                            const void* v8t, const float* scales, void* o, const uint8_t* labels,
                            const int32_t* row_ptr_s, const int32_t* col_idx_s,
                            const int32_t* row_ptr_t, const int32_t* col_idx_t, void* stream);

/*
 * Measurement aid, not a step of the method: the rate the bf16 matrix cores sustain on this
 * GPU, which the roofline of the attention kernels (Sec. 5.3: kernel-level efficiency) is
 * read against besides the published peak.  Launches `workgroups` workgroups of 4
 * wavefronts (two resident per compute unit, three in form 2), each wavefront issuing 16 * iterations
 * products v_mfma_f32_32x32x16_bf16 on operands taken from `operands`.
 *   form 0   products only, operands in registers
 *   form 1   per product additionally one 1 KB operand read from LDS and the softmax
 *            instructions the D = 128 attention kernel spends per product (one FMA, one
 *            exponential, one addition, half a bf16 pack): an upper bound for that kernel
 *            design, without its staging, barriers and global memory traffic
 *   form 2   the same for the D = 64 kernel: three workgroups resident per compute unit, and
 *            per product the softmax instructions of two scores per lane (two FMAs, two
 *            exponentials, one bf16 pack, one packed dot product)
 *   operands device, 1 MiB, 16-byte aligned: bf16 values (random data draws the power real
 *            data draws; zeros would let the clock rise)
 *   sink     device float [workgroups * 256], written (keeps the products alive)
 *   flop_out host, may be NULL: receives the floating point operations of the launch
 *            (2 * 32 * 32 * 16 per product)
 * The caller times the launch (it should last >= 10 ms for the clock to settle).
 */
int svg_probe_mfma_bf16(int form, int32_t workgroups, int32_t iterations, const void* operands,
                        float* sink, double* flop_out, void* stream);

/* Measurement aid (no part of the method): what the LDS of one compute unit delivers for the
 * access patterns of the attention kernels (the roofline discussion needs to know whether the
 * LDS is a saturated unit).  One workgroup of `waves` wavefronts (1..16; 8 = two per SIMD, as
 * the D = 128 kernels run) issues `iterations` x 16 LDS instructions of one kind per wavefront:
 *   form 0   ds_read_b128, the K operand pattern (rows padded by 16 bytes)
 *   form 1   ds_read_b64_tr_b16, the V^T operand pattern on the swizzled row-major V tile
 *   form 2   the same read on plain row-major rows (shows what the swizzle is for)
 *   form 3   ds_write_b128 in the staging pattern
 *   scratch  device, 16-byte aligned, >= 16 * 8 + 1024 * 4 bytes, written: int64 [16], of which
 *            entry w receives the shader clocks wavefront w took for its iterations x 16
 *            instructions (followed by a sink that keeps the reads alive).  The caller reads it
 *            back after synchronising; bytes per clock of the unit = waves x iterations x 16 x
 *            (1024 for forms 0 and 3, 512 for forms 1 and 2) / max over w of entry w.
 * Errors: INVALID_ARG (form, waves, iterations, NULL or misaligned scratch), WORKSPACE (scratch too
 * small), HIP. */
int svg_probe_lds(int form, int32_t waves, int32_t iterations, void* scratch, size_t scratch_bytes,
                  void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVG_H_ */
