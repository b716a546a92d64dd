/*
 * qvg.h - C ABI of the MI355X (gfx950) KV-cache codec of Quant VideoGen.
 *
 * The codec compresses the K or V tensor of one chunk of video tokens of one
 * attention head (paper Sec. 4.1: X in R^{N x d}) in two steps:
 *   1. semantic-aware smoothing: k-means groups the N tokens into K groups and
 *      the group centroid is subtracted from each token (Sec. 4.1, Eq. 5-6);
 *   2. progressive residual quantization: the residual is quantized to 2 bits
 *      per element in groups of B channels, and what that leaves is quantized
 *      again, n_stages times (Sec. 3.2 Eq. 1-2 applied to the residual of
 *      Sec. 4.2; each stage stores its own codes and per-group scales).
 * Decoding replays the stages (Sec. 4.2 Eq. 7); the fused entry point decodes
 * tile by tile inside an attention kernel, so the bf16 cache never exists.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer, 16-byte aligned, owned by the
 *     caller; the library allocates no device memory and keeps no state (the one exception is
 *     the static scratch array of qvg_encode_chunk_static, described there).
 *     `const qvg_params*`, `size_t*` are HOST pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work on it and never synchronise.
 *   - "bf16" is the upper 16 bits of an IEEE binary32; "f16" is IEEE binary16.
 *   - Return value: QVG_OK (0) or a negative qvg_status; on error nothing was
 *     enqueued unless the status is QVG_ERR_LAUNCH (outputs then undefined).
 *   - Inputs must be finite; non-finite values are not detected.
 *
 * Stored format of one chunk of one unit (n_heads counts independent units;
 * K and V of all heads and layers may be stacked into it):
 *   centroids [K][d]            bf16
 *   ids       [N]               uint8   index of the token's centroid
 *   codes     [N][T][d/4]       uint8   channel 4i+j in bits 2j..2j+1 of byte i, holding the
 *                                       level q in {-1,0,1} (Eq. 2, b = 2) as 2-bit two's
 *                                       complement: 0b00 = 0, 0b01 = +1, 0b11 = -1 (0b10 unused)
 *   scales    [N][T][d/B]       f16     per group of B consecutive channels
 * Format variants (Sec. 5 "Implementation"): with bits = 4 (INT4) the levels are -7..7 as 4-bit
 * two's complement, codes [N][T][d/2], channel 2i+j in bits 4j..4j+3 of byte i; with
 * scale_format = QVG_SCALE_E4M3 a scale is one byte in the OCP FP8 E4M3 layout (1 sign, 4
 * exponent bits with bias 7, 3 mantissa bits; largest finite value 448, no infinity, subnormals
 * m/8 * 2^-6), scales [N][T][d/B] uint8; the encoder never writes the NaN code 0x7F, and a
 * decoder that meets it reads 480.  E4M3 scale arrays need no alignment.
 * With more than 256 centroids (the codebook-size study of Sec. 5, Table 5, goes to K = 512) an id
 * is a 16-bit word: every "uint8_t *ids" argument then points at uint16 data, 2-byte aligned
 * (with S smoothing stages: S consecutive words per token).
 * The encoder writes ids below K only; a decoder (qvg_decode*, qvg_attn_decode*) that meets a
 * larger one, in a cache it did not write, reads the table's last row for it instead of memory
 * beyond the table.
 * A cache of several chunks concatenates ids/codes/scales along N and keeps one
 * centroid table per chunk: centroids [n_chunks][K][d].
 * Alignment inside a cache: qvg_encode_chunk wants every output pointer 16-byte aligned, so a chunk
 * can be encoded in place at token offset c * chunk_len only if chunk_len * T * (d/B) * 2 bytes of
 * binary16 scales (and chunk_len * T * d*b/8 bytes of codes) are multiples of 16: a chunk_len that
 * is a multiple of 8 tokens always is (E4M3 scale bytes need no alignment).  The attention entry
 * points read any chunk length and capacity; their fastest kernel needs the same property of
 * chunk_len and, with several units, of the capacity, and the others are read by a general kernel.
 *
 * With S = n_smooth_stages > 1 (the paper's progressive residual quantization, Sec. 4.2: the
 * residual of one k-means round is clustered again, S times, before it is quantized) a chunk
 * keeps S tables, centroids [n_chunks][S][K][d], and a token S ids, ids [N][S]; the residual
 * handed from one round to the next is rounded to bf16.  Everywhere below "[K][d]" then reads
 * "[S][K][d]" and "ids [N]" reads "ids [N][S]".
 */
#ifndef QVG_H
#define QVG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum qvg_status {
    QVG_OK = 0,
    QVG_ERR_NULL = -1,         /* a required pointer is NULL                      */
    QVG_ERR_BAD_PARAM = -2,    /* a size or parameter is out of its stated range  */
    QVG_ERR_UNSUPPORTED = -3,  /* valid in the paper, not built here              */
    QVG_ERR_WORKSPACE = -4,    /* workspace missing or too small                  */
    QVG_ERR_ALIGN = -5,        /* pointer or stride breaks the alignment rule     */
    QVG_ERR_LAUNCH = -6,       /* the HIP runtime refused a launch or a copy      */
    QVG_ERR_SCRATCH_LIMIT = -7 /* qvg_encode_chunk_static: the sizes need more scratch memory than
                                  QVG_STATIC_SCRATCH_BYTES                         */
} qvg_status;

/* Codec parameters, in the paper's symbols (Sec. 4, Sec. 5 "Implementation"). */
typedef struct qvg_params {
    int32_t n_heads;         /* H >= 1: independent units handled by one call           */
    int32_t head_dim;        /* d: 128                                                  */
    int32_t n_clusters;      /* K: 1..512; ids are uint8 up to 256 (Sec. 5: K = 256), uint16 beyond */
    int32_t group_size;      /* B: 16, 32, 64 or 128 consecutive channels of one token  */
    int32_t n_stages;        /* T: 1..8 rounds of b-bit quantization of the residual    */
    int32_t bits;            /* b: 2 or 4 bits per level (Sec. 5: INT2 / INT4)          */
    int32_t n_smooth_stages; /* S: 1..4 k-means smoothing rounds (QVG: 1, QVG-Pro: 4)        */
    int32_t kmeans_iters;    /* I >= 0 Lloyd iterations before the final assignment     */
    int32_t scale_format;    /* QVG_SCALE_F16 or QVG_SCALE_E4M3 (Sec. 5 "Implementation") */
} qvg_params;

#define QVG_SCALE_F16  0
#define QVG_SCALE_E4M3 1

/* which_entry values for qvg_workspace_bytes */
#define QVG_ENTRY_ENCODE 0
#define QVG_ENTRY_DECODE 1
#define QVG_ENTRY_ATTN   2
#define QVG_ENTRY_KMEANS_UPDATE 3
#define QVG_ENTRY_KMEANS_ASSIGN 4

/*
 * Encode one chunk (Sec. 4.1 and 4.2): I Lloyd iterations from init_centroids
 * (Sec. 4.3: the previous chunk's centroids, or any start the caller picks),
 * a final assignment, centroid subtraction (Eq. 5), then T rounds of 2-bit
 * group quantization of the residual (Eq. 1-2) with bit packing.
 *   x              [H][N][d] bf16 view: element (h,n,c) at x[h*stride_head + n*stride_token + c],
 *                  strides in elements, multiples of 8
 *   init_centroids [H][K][d] bf16 ([H][S][K][d]: one start table per smoothing round)
 *   centroids_out  [H][K][d] bf16, unit h at centroids_out + h*cent_out_stride_head elements
 *                  (0 = dense K*d; a multiple of 8; may equal init_centroids when I == 0 and dense)
 *   ids_out        [H][N]           codes_out [H][N][T][d/4]   scales_out [H][N][T][d/B] f16,
 *                  unit h starting out_stride_head_tokens tokens after unit h-1 (0 = dense N;
 *                  >= N).  The two strides let a chunk be written straight into a cache that
 *                  holds several chunks per unit: point the outputs at the chunk's first token
 *                  and table, and pass the cache's tokens and table elements per unit.
 *   workspace      qvg_workspace_bytes(p, QVG_ENTRY_ENCODE, N, 0) bytes (a few KB per unit when I == 0)
 * n_tokens in 0 .. 2^20.  n_tokens == 0 only copies the centroids.
 * Rounding rules that fix the stored integers: a group's scale is max|r| / qmax (one fp32
 * division; qmax = 2^(b-1) - 1, so 1 for b = 2), saturated at the scale format's largest finite
 * value (65504 or 448) and rounded to nearest even; q = round-half-even(r * (1/scale))
 * with 1/scale one correctly rounded fp32 division, clamped to [-qmax, qmax]; a zero scale gives
 * q = 0; the next round sees fma(-scale, q, r).  Assignment: smallest squared Euclidean
 * distance, the lowest index among exactly equal ones; a centroid is the mean of its
 * members summed in token order in fp64, rounded to fp32 then to bf16; an empty group
 * keeps its centroid.
 */
int qvg_encode_chunk(const qvg_params *p, int64_t n_tokens,
                     const void *x_bf16, int64_t stride_head, int64_t stride_token,
                     const void *init_centroids_bf16, void *centroids_bf16_out,
                     int64_t cent_out_stride_head,
                     uint8_t *ids_out, uint8_t *codes_out, void *scales_f16_out,
                     int64_t out_stride_head_tokens,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * qvg_encode_chunk for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same call without the workspace
 * arguments.  The workspace lives in a static device array inside the library,
 * QVG_STATIC_SCRATCH_BYTES per GPU the library runs on, held until the process ends; the call
 * allocates and frees nothing.  Arguments, results and errors are those of qvg_encode_chunk, plus
 *   QVG_ERR_SCRATCH_LIMIT  when qvg_workspace_bytes(p, QVG_ENTRY_ENCODE, n_tokens, 0) exceeds
 *                          QVG_STATIC_SCRATCH_BYTES (nothing was enqueued).  One layer's chunk of
 *                          every configuration this library is measured on fits (24 units x 4680
 *                          tokens, K = 256: 3.7 MB; 80 units x 10800 tokens, K = 128: 9 MB);
 *                          several smoothing stages need two bf16 copies of the chunk and fit only
 *                          for small chunks.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time (on
 * different streams, or from different threads on the same stream without ordering) race.  Calls
 * on one stream are ordered and safe.  The array keeps the previous call's contents; nothing in it
 * needs to start at zero.
 */
#define QVG_STATIC_SCRATCH_BYTES (16u << 20)
int qvg_encode_chunk_static(const qvg_params *p, int64_t n_tokens,
                            const void *x_bf16, int64_t stride_head, int64_t stride_token,
                            const void *init_centroids_bf16, void *centroids_bf16_out,
                            int64_t cent_out_stride_head,
                            uint8_t *ids_out, uint8_t *codes_out, void *scales_f16_out,
                            int64_t out_stride_head_tokens, void *stream);

/*
 * Decode (Sec. 4.2 "dequantization process", Eq. 7; Sec. 4.3 "Dequantization
 * kernel": all stages in one kernel, the running value kept in registers):
 * x_hat = centroid[id] + sum_t scale_t * q_t, fp32 fma in stage order, one
 * rounding to bf16 (S > 1: the S centroid rows are added first, in round order, in fp32).
 *   n_tokens (0 .. 2^31-1) tokens per unit in chunks of chunk_len (the last may be shorter;
 *   chunk_len >= n_tokens means one chunk); centroids [H][n_chunks][K][d].
 *   x_bf16_out: same view convention as the encoder's x.
 */
int qvg_decode(const qvg_params *p, int64_t n_tokens, int64_t chunk_len,
               const void *centroids_bf16, const uint8_t *ids, const uint8_t *codes,
               const void *scales_f16, void *x_bf16_out, int64_t stride_head,
               int64_t stride_token, void *stream);

/*
 * qvg_decode of a token range of caches that are allocated for more tokens than are decoded:
 * tokens first_token .. first_token + n_tokens - 1 of every unit, first_token a multiple of
 * chunk_len; unit h starts kv_capacity_tokens tokens (ids, codes, scales) and
 * ceil(kv_capacity_tokens / chunk_len) tables after unit h-1 (0 = first_token + n_tokens).
 * The array pointers are those of the whole cache (token 0 of unit 0); x_bf16_out receives
 * the range only, [H][n_tokens][d] in the view convention of qvg_decode.
 */
int qvg_decode_ex(const qvg_params *p, int64_t n_tokens, int64_t chunk_len,
                  int64_t kv_capacity_tokens, int64_t first_token,
                  const void *centroids_bf16, const uint8_t *ids, const uint8_t *codes,
                  const void *scales, void *x_bf16_out, int64_t stride_head,
                  int64_t stride_token, void *stream);

/*
 * Attention over the compressed cache: O = softmax(softmax_scale * Q K_hat^T) V_hat
 * per unit, no mask, where K_hat and V_hat are what qvg_decode would return (bf16),
 * produced tile by tile in LDS and never written to memory (or, with a workspace, written one
 * slab of chunks at a time into it: see `workspace`).
 *   q_bf16   [H][n_q][d] contiguous       out_bf16 [H][n_q][d] contiguous
 *   K and V caches: n_kv_tokens tokens in chunks of chunk_len, each with the
 *   layout qvg_decode reads; both use the parameters in *p.
 *   lse_out  [H][n_q] fp32 natural-log sum of exp of the scaled scores, or NULL
 *   workspace: optional device memory, 16-byte aligned.  Without it (NULL, 0) every block of 256
 *              queries decodes the cache for itself inside one kernel.  With it every 64-token tile
 *              is decoded ONCE per unit into the workspace (K_hat as bf16, V_hat as binary16, 512
 *              bytes per token and unit) and read from there by all query blocks: a slab of as many
 *              whole chunks as fit at a time, two launches per slab, the queries' running soft-max
 *              state (264 bytes per query and unit) carried in the workspace from slab to slab.
 *              The full-precision cache is never held beyond one slab.  Useful from 512 queries
 *              per unit upward (the dequantization is what bounds the one-kernel form).
 *              qvg_workspace_bytes(p, QVG_ENTRY_ATTN, tokens, n_q) gives the bytes that hold
 *              `tokens` tokens of decoded tiles plus the state, where tokens = number of chunks in
 *              a slab x chunk_len rounded up to a multiple of 64.  A workspace that cannot hold one
 *              chunk (plus the state, when the cache has more chunks than fit) is ignored, and so is
 *              any workspace when n_q <= 256.  Contents are
 *              scratch: nothing has to be initialised and nothing survives the call.  The result
 *              equals the one-kernel form's bit for bit (same operands, same order of operations).
 * n_kv_tokens >= 1; n_q == 0 is a no-op; softmax_scale must be positive and finite.
 */
int qvg_attn_decode(const qvg_params *p, int64_t n_q, const void *q_bf16,
                    int64_t n_kv_tokens, int64_t chunk_len,
                    const void *k_centroids, const uint8_t *k_ids, const uint8_t *k_codes,
                    const void *k_scales,
                    const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
                    const void *v_scales,
                    float softmax_scale, void *out_bf16, float *lse_out,
                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * qvg_attn_decode with what a generation step needs around it (Sec. 3.1: a chunk attends to the
 * cached chunks and to itself; Sec. 5 "Implementation": keys are cached BEFORE the rotary
 * position embedding):
 *   kv_capacity_tokens  the caches may be allocated for more tokens than they hold: unit h starts
 *                       kv_capacity_tokens tokens (ids, codes, scales) and
 *                       ceil(kv_capacity_tokens / chunk_len) tables (centroids) after unit h-1;
 *                       only the first n_kv_tokens tokens are read.  0 = n_kv_tokens.  Attention
 *                       of an earlier chunk's queries over a prefix of the cache (chunk-causal
 *                       order) is a call with a smaller n_kv_tokens.
 *   k_rope_f16          NULL, or [n_kv_tokens][d/2][2] f16 = (cos, sin) of the rotation angle of
 *                       token n and channel pair i, shared by all units: every decoded key,
 *                       rounded to bf16 as qvg_decode returns it, is rotated on interleaved pairs,
 *                       y[2i] = x[2i] cos - x[2i+1] sin, y[2i+1] = x[2i] sin + x[2i+1] cos (one
 *                       fp32 product and one fma each, then bf16), before the scores are taken.
 *                       The queries arrive already rotated.  V is not rotated.
 * Everything else as in qvg_attn_decode.
 */
int qvg_attn_decode_ex(const qvg_params *p, int64_t n_q, const void *q_bf16,
                       int64_t n_kv_tokens, int64_t chunk_len, int64_t kv_capacity_tokens,
                       const void *k_centroids, const uint8_t *k_ids, const uint8_t *k_codes,
                       const void *k_scales,
                       const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
                       const void *v_scales,
                       const void *k_rope_f16,
                       float softmax_scale, void *out_bf16, float *lse_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * qvg_attn_decode_ex with a prefix length per query: query i (of every unit) sees the cached
 * tokens 0 .. q_kv_len[i]-1 only.  With lengths that are multiples of chunk_len this is the
 * chunk-causal order of Sec. 3.1 for the queries of SEVERAL chunks in one call (each chunk
 * attends to the chunks before it; its own keys are not in the compressed cache: see
 * qvg_attn_merge).
 *   q_kv_len   [n_q] int32, device; values are clamped to 0 .. n_kv_tokens.  NULL = every query
 *              sees all n_kv_tokens tokens (the call is then qvg_attn_decode_ex).  A query with
 *              length 0 (the first chunk of a chunk-causal batch: nothing is cached before it)
 *              gets a zero output row and lse = -infinity, which qvg_attn_merge treats as a
 *              partial result without weight.
 * A workgroup stops at the longest prefix among its 256 queries, so queries sorted by length
 * cost what their prefixes cost (with a workspace every tile of the cache is still decoded once;
 * the query blocks stop reading at their longest prefix).
 */
int qvg_attn_decode_causal(const qvg_params *p, int64_t n_q, const void *q_bf16,
                           int64_t n_kv_tokens, int64_t chunk_len, int64_t kv_capacity_tokens,
                           const void *k_centroids, const uint8_t *k_ids, const uint8_t *k_codes,
                           const void *k_scales,
                           const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
                           const void *v_scales,
                           const void *k_rope_f16, const int32_t *q_kv_len,
                           float softmax_scale, void *out_bf16, float *lse_out,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * qvg_attn_decode_causal with the result left in fp32, [H][n_q][d] float, before the final rounding
 * to bf16 (no workspace arguments).  For checking the kernel's own arithmetic against a reference:
 * with a bf16 result, half an ulp of the output (2^-9 of its magnitude) hides what the kernel adds.
 * What the kernel adds: the scores are bf16 x bf16 products accumulated in fp32; the probabilities
 * enter the second contraction as binary16 rounded to nearest (the normaliser is the sum of the
 * rounded values), the decoded values as binary16 (exact: they are bf16 numbers; magnitudes beyond
 * 65504 are not supported).  The output error is therefore about 2^-12 of the magnitude of the
 * values a query attends to: below 2e-3 in absolute terms for |V| up to about 8, and it grows in
 * proportion beyond that (keys of any magnitude only sharpen the soft-max).
 */
int qvg_attn_decode_f32(const qvg_params *p, int64_t n_q, const void *q_bf16,
                        int64_t n_kv_tokens, int64_t chunk_len, int64_t kv_capacity_tokens,
                        const void *k_centroids, const uint8_t *k_ids, const uint8_t *k_codes,
                        const void *k_scales,
                        const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
                        const void *v_scales,
                        const void *k_rope_f16, const int32_t *q_kv_len,
                        float softmax_scale, float *out_f32, float *lse_out, void *stream);

/*
 * Merge two attention results over DISJOINT key sets (the compressed cache, from
 * qvg_attn_decode with lse_out, and the current chunk's own bf16 keys, from the model's
 * attention kernel) into the attention over their union (Sec. 3.1):
 *   lse = log(exp(lse_a) + exp(lse_b)),  out = exp(lse_a - lse) out_a + exp(lse_b - lse) out_b.
 *   out_a, out_b, out  [n_rows][head_dim] bf16 contiguous (out may be out_a or out_b)
 *   lse_a, lse_b       [n_rows] fp32 natural-log sum of exp of the scaled scores; at least one
 *                      of the two must be finite in every row
 *   lse_out            [n_rows] fp32 or NULL
 */
int qvg_attn_merge(int64_t n_rows, int32_t head_dim, const void *out_a_bf16, const float *lse_a,
                   const void *out_b_bf16, const float *lse_b, void *out_bf16, float *lse_out,
                   void *stream);

/*
 * The two k-means steps on their own (Sec. 4.1), as the encoder runs them.
 * assign: ids_out[h][n] = index of the nearest centroid of unit h; workspace
 *         qvg_workspace_bytes(p, QVG_ENTRY_KMEANS_ASSIGN, N, 0) bytes.
 * update: centroid = mean of its members (see qvg_encode_chunk for the rounding);
 *         counts_out [H][K] int32 may be NULL; workspace
 *         qvg_workspace_bytes(p, QVG_ENTRY_KMEANS_UPDATE, N, 0) bytes.
 */
int qvg_kmeans_assign(const qvg_params *p, int64_t n_tokens,
                      const void *x_bf16, int64_t stride_head, int64_t stride_token,
                      const void *centroids_bf16, uint8_t *ids_out,
                      void *workspace, size_t workspace_bytes, void *stream);
int qvg_kmeans_update(const qvg_params *p, int64_t n_tokens,
                      const void *x_bf16, int64_t stride_head, int64_t stride_token,
                      const uint8_t *ids, const void *centroids_prev_bf16,
                      void *centroids_bf16_out, int32_t *counts_out,
                      void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace an entry point needs for these sizes (host call, no GPU). */
int qvg_workspace_bytes(const qvg_params *p, int which_entry, int64_t n_tokens,
                        int64_t n_q, size_t *out);

/* Stored bytes of one chunk of n_tokens tokens for all H units: codes, scales,
 * ids and one centroid table per unit (Sec. 5 "Memory usage breakdown").
 * Negative qvg_status on bad parameters. */
int64_t qvg_compressed_bytes(const qvg_params *p, int64_t n_tokens);

/* Static, NUL-terminated description of a status code. */
const char *qvg_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int qvg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QVG_H */
