/*
 * libvista -- C ABI of the VISTA hot path on one MI355X (gfx950).
 *
 * Two stages (paper Sec. 3.1):
 *   stage 1  vista_summarize      S learned virtual seed embeddings, shared by all
 *                                 users, attend over each user's jagged history of
 *                                 L_b items and yield S summary tokens (Sec. 3.2);
 *   stage 2  vista_target_attend  every candidate item attends, independently, to
 *                                 its user's S cached summary tokens (Sec. 3.3).
 * The attention of both stages is the softmax form RowSoftmax(Q K^T) V of
 * Sec. 3.2.1 (unnumbered equation), multi-head, with scale 1/sqrt(d/H) unless
 * the descriptor overrides it.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers unless the name ends in _host.
 *     Tensors are row-major and packed; the innermost dimension is d.
 *   - The caller owns every buffer.  The library allocates nothing, keeps no
 *     state between calls, never synchronises; all work is enqueued on the
 *     given hipStream_t (passed as void*; NULL is the default stream).
 *   - Inputs are read-only; outputs are fully overwritten.
 *   - Errors are return codes.  Everything that can be checked on the host is
 *     checked before the first launch: on any status but VISTA_ERR_HIP nothing
 *     was enqueued.  VISTA_ERR_HIP reports that the runtime refused one of the
 *     call's launches; kernels launched before it may already be enqueued and the
 *     outputs are then undefined.
 *   - 64-bit row addressing throughout: N * d may exceed 2^31.
 */
#ifndef VISTA_H
#define VISTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  VISTA_OK = 0,
  VISTA_ERR_NULL = 1,        /* a required pointer is NULL */
  VISTA_ERR_SHAPE = 2,       /* a size is non-positive, d % H != 0, or a stride is inconsistent */
  VISTA_ERR_OFFSETS = 3,     /* offsets_host: not starting at 0, decreasing, or not ending at total_items */
  VISTA_ERR_UNSUPPORTED = 4, /* dtype / head width / S outside the supported set */
  VISTA_ERR_WORKSPACE = 5,   /* workspace pointer NULL, misaligned or too small */
  VISTA_ERR_HIP = 6,         /* the runtime refused a kernel launch of this call */
  VISTA_ERR_SCRATCH = 7      /* vista_summarize_static: the call needs more than VISTA_STATIC_SCRATCH_BYTES */
} vista_status;

/* storage dtype of every tensor of a call; accumulation is always fp32 */
enum { VISTA_F32 = 0, VISTA_BF16 = 1 };
/*
 * Attention form of stage 1 (desc.attn):
 *   VISTA_ATTN_SOFTMAX  RowSoftmax(scale Q_h K_h^T) V_h                      Sec. 3.2.1, unnumbered equation
 *   VISTA_ATTN_SILU     (1/L_b) sum_j SiLU(scale q . k_j) v_j                App. B, closing formula (SiLU
 *                       attention from targets to sources) with the 1/N factor of the appendix's opening
 *                       paragraph, N = the user's own length; the paper prints no score scale, so scale = 0
 *                       selects 1 here
 *   VISTA_ATTN_QLA      SiLU(Q_h) SiLU( SiLU(K_h)^T V_h )                    Sec. 3.2.2, target-side QLU equation
 *                       with the seeds as targets and the history as source; no normalisation, no scale
 *                       (desc.scale must be 0)
 */
enum { VISTA_ATTN_SOFTMAX = 0, VISTA_ATTN_SILU = 1, VISTA_ATTN_QLA = 2 };
/*
 * desc.flags.  VISTA_FLAG_SELF_TERM: every query also attends to itself and to no other
 * query (Eq. 3; the Delta term of Sec. 3.2.2; the identity block of App. B's mask).  In stage 1
 * the seed's own key and value are seed W_k and seed W_v; in stage 2 (no projections) the
 * candidate's own embedding is both.  Softmax: the own score joins the row's softmax.  SiLU form:
 * SiLU(scale q . k') v' joins the sum inside the same 1/L_b.  QLA: (SiLU(q) . SiLU(k')) v' is added.
 * Users without history still get zeros.
 */
enum { VISTA_FLAG_SELF_TERM = 1 };

/* ---------------------------------------------------------------- stage 1 */

typedef struct {
  int32_t B;              /* users                                                    */
  int32_t S;              /* virtual queries = summary tokens per user, 1..512        */
  int32_t d;              /* model width                                              */
  int32_t H;              /* heads; head h owns columns [h*d/H, (h+1)*d/H)            */
  int32_t dtype;          /* VISTA_F32 or VISTA_BF16                                  */
  int32_t attn;           /* VISTA_ATTN_SOFTMAX                                       */
  float   scale;          /* score scale; 0 selects 1/sqrt(d/H)                       */
  int32_t segment_items;  /* items per split-L segment, multiple of 32; 0 = default   */
  int64_t total_items;    /* N = offsets[B]                                           */
  int64_t q_user_stride;  /* 0: queries [S,d] shared by all users (Sec. 3.2);
                             S*d: per-user queries [B,S,d] (stacked layers)           */
  int32_t flags;          /* 0 or VISTA_FLAG_SELF_TERM                                */
  int32_t reserved;       /* must be 0                                                */
} vista_summarize_desc;

/*
 * Split-L schedule (the re-association of App. B: partial sums over blocks of
 * the history may be formed first and combined afterwards).  The packed history
 * of N rows is cut into G = ceil(N / segment_items) flat segments of equal size;
 * a segment is processed by one workgroup and is further cut at user
 * boundaries into pieces.  Piece (g, b) -- the rows of user b inside segment g
 * -- writes its running maximum, sum of exponentials and un-normalised output
 * to partial slot g + b; a merge pass combines a user's slots in an order fixed
 * by their count alone (ascending g; the quasi-linear form adds four interleaved
 * ascending sub-sums).  The schedule is a pure function of (offsets,
 * segment_items), never of the device, so results are bitwise reproducible.
 *
 * vista_summarize_segment_items: the segment size the call will use
 * (desc->segment_items, or the default derived from total_items and the
 * attention form alone: the history is cut into 256 k equal segments, k the
 * smallest count that keeps a segment at or below 8192 items -- 1024 k segments
 * of at most 2048 items for VISTA_ATTN_QLA, whose workgroups are small; at
 * least 256 items); 0 if the descriptor is invalid.
 */
int32_t vista_summarize_segment_items(const vista_summarize_desc* desc);

/*
 * The schedule itself, computed on the host by the very code the kernels run
 * (App. B: blocks of the history are summed first, in any grouping; this is the
 * grouping).  Every segment is walked as a stream of tiles of at most 32 rows;
 * a tile never spans two users.  Writes up to max_tiles records
 *     tiles[4 i + 0..3] = { segment, user, first flat row, rows in the tile (1..32) }
 * in the order the kernels visit them and returns the total number of tiles
 * (which may exceed max_tiles; pass max_tiles = 0, tiles = NULL to count), or -1
 * for an invalid descriptor or a NULL offsets_host.  offsets_host is NOT
 * validated here: for valid offsets the tiles cover every row of every user
 * exactly once; for any other contents every tile still lies inside
 * [0, total_items) and every user index inside [0, B), which is what keeps the
 * kernels from faulting on bad offsets.  Host-only: touches no device.
 */
int64_t vista_summarize_schedule(const vista_summarize_desc* desc, const int64_t* offsets_host,
                                 int64_t* tiles, int64_t max_tiles);

/* Bytes of device workspace vista_summarize needs for this descriptor (0 if invalid).
 * The workspace must be 256-byte aligned.  Its first 4 bytes receive an int32
 * device-side status (0 = offsets passed the on-device check, VISTA_ERR_OFFSETS
 * otherwise) that the caller may read after synchronising the stream. */
size_t vista_summarize_workspace_bytes(const vista_summarize_desc* desc);

/*
 * Stage 1 (Sec. 3.2; attention form of Sec. 3.2.1).  For each user b with rows
 * X_b = history_emb[offsets[b] .. offsets[b+1]-1]:
 *     K = X_b W_k,  V = X_b W_v,
 *     out[b][:, head h] = RowSoftmax(scale * Q_h K_h^T) V_h      for every head h,
 * Q = virtual_queries (shared) or virtual_queries[b] (q_user_stride = S*d).
 * The softmax of one query runs over all L_b items of that user; there is no
 * mask and no positional term.  A user with L_b = 0 gets zeros.
 *
 *   history_emb      device [N, d]        dtype
 *   offsets          device int64 [B+1]   offsets[0] = 0, non-decreasing, offsets[B] = N
 *   offsets_host     host   int64 [B+1]   optional mirror; when given it is validated
 *                                         here (VISTA_ERR_OFFSETS) before any launch.
 *                                         When NULL the check runs on the device and
 *                                         reports through the workspace status word;
 *                                         kernels clamp every row index to [0, N), so
 *                                         bad offsets give wrong numbers, never a fault.
 *   virtual_queries  device [S, d] or [B, S, d]   dtype
 *   W_k, W_v         device [d, d]        dtype; K = X @ W_k (input rows, output columns)
 *   out              device [B, S, d]     dtype (bf16: one round-to-nearest-even at the store)
 *   workspace        device, >= vista_summarize_workspace_bytes(desc), 256-byte aligned
 *
 * Supported: bf16 with (d, H) = (128, 4) or (256, 8), S in {64, 128, 256, 512} (MFMA path);
 * any dtype with d/H <= 64, d <= 512, S <= 512 (plain fp32-ALU path).
 * The workspace grows with the user count as well as with the history: the MFMA
 * path keeps (G + B) partial records of H * S * 144 bytes (G = segments), the
 * plain path the same count of H * S * (d/H + 2) * 4 bytes plus fp32 K and V.
 */
vista_status vista_summarize(const vista_summarize_desc* desc,
                             const void* history_emb,
                             const int64_t* offsets,
                             const int64_t* offsets_host,
                             const void* virtual_queries,
                             const void* W_k,
                             const void* W_v,
                             void* out,
                             void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/*
 * vista_summarize for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same computation, same kernels, same results bit for bit as
 * vista_summarize with the same descriptor; the workspace is a static device
 * array of VISTA_STATIC_SCRATCH_BYTES inside the library (one per GPU the
 * library runs on, held until the process ends).  The call allocates nothing.
 *
 *   - A descriptor whose vista_summarize_workspace_bytes exceeds
 *     VISTA_STATIC_SCRATCH_BYTES is rejected with VISTA_ERR_SCRATCH before any
 *     launch (64 MiB holds the 64-user, 0.77 M-item, S = 256, d = 128 batch with
 *     a third to spare).
 *   - The first call on a device looks up that device's copy of the array
 *     (no allocation, but make it outside a graph capture).
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one
 *     GPU (different streams, no ordering between them) race; order them.
 *   - The device-side offsets status (offsets_host == NULL) stays inside the
 *     library; pass offsets_host to have the offsets checked.
 */
#define VISTA_STATIC_SCRATCH_BYTES (64u << 20)
vista_status vista_summarize_static(const vista_summarize_desc* desc,
                                    const void* history_emb,
                                    const int64_t* offsets,
                                    const int64_t* offsets_host,
                                    const void* virtual_queries,
                                    const void* W_k,
                                    const void* W_v,
                                    void* out,
                                    void* hip_stream);

/* ---------------------------------------------------------------- stage 2 */

typedef struct {
  int32_t B;      /* users                         */
  int32_t C;      /* candidates per user           */
  int32_t S;      /* summary tokens per user       */
  int32_t d;      /* model width                   */
  int32_t H;      /* heads                         */
  int32_t dtype;  /* VISTA_F32 or VISTA_BF16       */
  float   scale;  /* 0 selects 1/sqrt(d/H)         */
  int32_t flags;  /* 0 or VISTA_FLAG_SELF_TERM     */
} vista_attend_desc;

/*
 * Stage 2 (Sec. 3.3).  For each user b, candidate c and head h:
 *     p = softmax over the S summary tokens of  scale * q . Y_h[j],   q = candidates[b,c,head h]
 *     out[b,c,head h] = sum_j p_j Y_h[j],                              Y = summaries[b]
 * The summaries are keys and values at once.  Each candidate is a query row of
 * its own: candidates never attend to each other (Sec. 3.2.1, remark after Eq. 2).
 *
 *   candidates  device [B, C, d]  dtype
 *   summaries   device [B, S, d]  dtype
 *   out         device [B, C, d]  dtype
 *
 * Supported: bf16 with d/H = 32, H even, S a multiple of 32 up to 256 or a multiple
 * of 64 up to 512 (MFMA path); any dtype with d/H <= 64, S <= 512 (plain path).
 * No workspace.
 */
vista_status vista_target_attend(const vista_attend_desc* desc,
                                 const void* candidates,
                                 const void* summaries,
                                 void* out,
                                 void* hip_stream);

/* ------------------------------------------------ gradients of quasi-linear attention */

/*
 * Backward of VISTA_ATTN_QLA (App. B.1: Eqs. 7, 9, 11 give dQ = dO Z, dK = V W^T, dV = K W for
 * the linear core, with the d_h x d_h intermediates Z = V^T K and W = Q^T dO; with the
 * activations of Sec. 3.2.2 in place every product is taken on the activated operand and
 * multiplied by the activation's derivative, as the appendix shows for its shifted-ELU
 * variant).  Per user and head, with A = SiLU(Q), P = SiLU(K), Zs = P^T V, G = SiLU(Zs):
 *     dQ  = (dO G^T) * SiLU'(Q)
 *     dZs = (A^T dO) * SiLU'(Zs)
 *     dV  = P dZs,      dK = (V dZs^T) * SiLU'(K)
 * K = X W_k and V = X W_v are recomputed from the history as in the forward call; the
 * gradients are with respect to these projected keys and values (their own backward --
 * dX = dK W_k^T + dV W_v^T, dW = X^T dK -- is a pair of plain matrix products outside this path).
 *
 * With VISTA_FLAG_SELF_TERM the forward output also holds the target-side diagonal term
 * (SiLU(q_i) . SiLU(k'_i)) v'_i with the seeds' own k' = q W_k, v' = q W_v (Sec. 3.2.2); its
 * gradients (App. B.1: the second term of Eq. 8, Eqs. 10 and 12, with the diagonals
 * U = Delta(SiLU(Q), SiLU(K')) and X = Delta(dO, V')) are
 *     dV' = U dO,   dK' = X SiLU(Q) * SiLU'(K'),   dQ += X SiLU(K') * SiLU'(Q)
 * with respect to k' and v' as values of their own (the chain through q W_k, q W_v is the
 * caller's, as for the history).
 *
 *   desc            as for the forward call: attn = VISTA_ATTN_QLA, scale = 0, flags = 0 or
 *                   VISTA_FLAG_SELF_TERM
 *   d_out           device [B, S, d]  dtype   gradient of the loss w.r.t. the forward output
 *   d_queries       device [B, S, d]  dtype   per user, also when the queries are shared
 *                                             (the gradient of shared seeds is the sum over users)
 *   d_keys, d_values device [N, d]    dtype   rows of users without history do not exist; every row is written
 *   d_self_keys, d_self_values  device [B, S, d]  dtype   with VISTA_FLAG_SELF_TERM only (else
 *                   ignored, may be NULL): per user, zeros for users without history
 *   workspace       >= vista_qla_backward_workspace_bytes(desc), 256-byte aligned
 * Supported: the shapes vista_summarize takes with VISTA_ATTN_QLA.
 */
size_t vista_qla_backward_workspace_bytes(const vista_summarize_desc* desc);
vista_status vista_qla_backward(const vista_summarize_desc* desc,
                                const void* history_emb,
                                const int64_t* offsets,
                                const int64_t* offsets_host,
                                const void* virtual_queries,
                                const void* W_k,
                                const void* W_v,
                                const void* d_out,
                                void* d_queries,
                                void* d_keys,
                                void* d_values,
                                void* d_self_keys,
                                void* d_self_values,
                                void* workspace, size_t workspace_bytes,
                                void* hip_stream);

/* ------------------------------------------------ cache codec (int8) */

/*
 * Sec. 3.1: the summaries are quantized when they are written to the cache and
 * dequantized when stage 2 reads them.  The paper fixes no scheme; this library's is
 * symmetric int8 with one fp32 scale per (summary token, head):
 *     amax = max |y_c| over the head's d/H channels,  scale = amax / 127,
 *     code_c = round-half-even(y_c * (127 / amax)),    y_c ~ code_c * scale,
 * every step in fp32; an all-zero group has scale 0 and zero codes.
 *   codes   int8  [B, S, d]      scales  float [B, S, H]
 * It halves the bytes stage 2 reads per user (S*d + 4*S*H instead of 2*S*d).
 */
typedef struct {
  int64_t rows;   /* B * S summary tokens          */
  int32_t d;      /* model width                   */
  int32_t H;      /* heads (scale groups per row)  */
  int32_t dtype;  /* dtype of y                    */
} vista_codec_desc;

/* y device [rows, d] dtype -> codes device int8 [rows, d], scales device float [rows, H].
 * Supported: d/H <= 64.  No workspace. */
vista_status vista_quantize_summaries(const vista_codec_desc* desc, const void* y, int8_t* codes, float* scales,
                                      void* hip_stream);

/*
 * vista_summarize with the codec fused into its last kernel: the normalised fp32 summaries
 * are quantized as they are produced and never stored in dtype.  Arguments as vista_summarize,
 * with out_codes (device int8 [B, S, d]) and out_scales (device float [B, S, H]) in place of out.
 * Supported: the shapes of the bf16 MFMA path, softmax and SiLU forms (else VISTA_ERR_UNSUPPORTED:
 * run vista_summarize, then vista_quantize_summaries).
 */
vista_status vista_summarize_q8(const vista_summarize_desc* desc,
                                const void* history_emb,
                                const int64_t* offsets,
                                const int64_t* offsets_host,
                                const void* virtual_queries,
                                const void* W_k,
                                const void* W_v,
                                int8_t* out_codes,
                                float* out_scales,
                                void* workspace, size_t workspace_bytes,
                                void* hip_stream);

/*
 * vista_target_attend on quantized summaries: keys and values are code * scale, formed on
 * the fly (the bf16 MFMA path rounds them to bf16 once, as it rounds every operand).
 * candidates / out device [B, C, d] dtype; codes device int8 [B, S, d]; scales device float [B, S, H].
 * Same supported set as vista_target_attend.
 */
vista_status vista_target_attend_q8(const vista_attend_desc* desc,
                                    const void* candidates,
                                    const int8_t* codes,
                                    const float* scales,
                                    void* out,
                                    void* hip_stream);

/* ------------------------------------------------ block between layers */

typedef struct {
  int64_t rows;   /* B * S                          */
  int32_t d;      /* model width                    */
  int32_t d_ff;   /* inner width                    */
  int32_t dtype;  /* VISTA_F32 or VISTA_BF16        */
  float   eps;    /* 0 selects 1e-6                 */
} vista_ffn_desc;

/*
 * SiLU-gated block that turns the summaries of one summarization layer into the
 * per-user queries of the next (Sec. 3.2.2 names a Simple Gated Linear Unit and
 * gives no formula; this is the reading this library fixes):
 *     yhat = y / sqrt(mean_d(y^2) + eps)
 *     out  = (SiLU(yhat W_g) * (yhat W_u)) W_o
 *   y    device [rows, d]     W_g, W_u  device [d, d_ff]    W_o  device [d_ff, d]
 *   out  device [rows, d]     all of dtype
 * Supported: d <= 512, d_ff <= 1024, both multiples of 32 (bf16 with d = 128 or 256
 * runs on the MFMA path, everything else on the plain one).  No workspace.
 */
vista_status vista_sglu_ffn(const vista_ffn_desc* desc,
                            const void* y,
                            const void* W_g, const void* W_u, const void* W_o,
                            void* out,
                            void* hip_stream);

/* Static, human-readable name of a status code. */
const char* vista_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* VISTA_H */
