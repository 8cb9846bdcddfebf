/*
 * bitdecode.h -- C ABI of libbitdecode.so: decode-step attention over a quantized,
 * bit-packed KV cache on AMD MI355X (gfx950), after BitDecoding (arxiv 2503.18773).
 *
 * The library computes  Out = softmax(Q . D(K')^T) . D(V')  (Fig. 2 caption of the paper;
 * D = dequantization) for one new query token per sequence, plus the online
 * quantize-and-pack of the K/V tokens that feed the cache (Sec. III-A, Sec. IV-B).
 *
 * General conventions
 *  - Every pointer named "device" is a device (HBM) address owned by the caller; the
 *    library never allocates, frees, or synchronises.  Pointers named "host" are ordinary
 *    host addresses read or written synchronously inside the call.
 *  - All work is enqueued on the given hipStream_t (passed as void*; NULL = default
 *    stream) and the call returns at once.  Buffers must stay alive until the stream has
 *    passed the call.  Calls on one cache must be ordered on one stream.
 *  - For bd_cache, lengths are host integers and are uniform across the batch (the paper's
 *    "Batches" setting, Sec. V-A: same length, padded); bd_paged_cache (further down) keeps
 *    per-sequence lengths on the device (the "Page" setting).
 *  - head_dim is 128.  The residual block N_r (Eq. 1) is 128 tokens for every integer format; the
 *    quantization group is 128 as well, except for the _G64 / _G32 formats (64 / 32, with K
 *    channel-wise or, _KT_G64 / _KT_G32, per token); the MX group is 32 for BD_FMT_MXFP4, which
 *    keeps no residual.
 *  - Arguments are validated before anything is launched: a validation error (any status but
 *    BD_ERR_HIP) means nothing was enqueued and no state changed.  BD_ERR_HIP is a failed launch
 *    in the middle of a call: kernels enqueued before it stay enqueued, and the in-out lengths
 *    are those reached so far (see bd_decode_step).  Non-finite K/V/Q values are undefined behaviour.
 *
 * Cache layout (all little-endian, contiguous, 16-byte aligned), B = batch, H = n_kv_heads,
 * NBcap = capacity/128, D = 128, bits = 4 or 2, cpw = 32/bits codes per 32-bit word:
 *
 *  INT4 / INT2 and their _KT variants  (K channel-wise or per token, V per token -- Sec. IV-B(1), Sec. IV-C(1))
 *   k_codes  uint32 [B][H][NBcap][128 tokens][D/cpw]   word w of a token: channels cpw*w+n at bit bits*n
 *   v_codes  uint32 [B][H][NBcap][D channels][128/cpw] word w of a channel: block tokens cpw*w+n at bit bits*n
 *   k_params uint32 [B][H][NBcap][D]     half2: fp16 scale in bits 0..15, fp16 zero in bits 16..31
 *                                        (BD_FMT_INT4_KT / INT2_KT: [B][H][NBcap][128], one per token
 *                                        of the block, statistics over the token's 128 channels)
 *   v_params uint32 [B][H][NBcap][128]   half2 per token of the block
 *   k_res, v_res fp16 [B][H][128][D]     the L mod 128 newest tokens, unquantized (Sec. III-A(2))
 *   Quantizer: zero = group minimum (-0 stored as +0); scale = fp16((max - min) / (2^bits - 1))
 *   computed with one fp32 subtraction and one fp32 division; code = clamp(rint((x - zero) /
 *   scale), 0, 2^bits - 1) in fp32, ties to even, 0 where scale == 0;  x_hat = code*scale + zero.
 *
 *  MXFP4  (Sec. IV-D(2): e2m1 elements, one e8m0 scale per 32 contiguous channels of a token;
 *          every token is quantized on arrival, there is no residual)
 *   k_codes  uint8 [B][H][capacity tokens][D/2]   byte j: channel 2j low nibble, 2j+1 high nibble
 *   k_params uint8 [B][H][capacity tokens][D/32]  e8m0 (value 2^(byte-127))
 *   v_codes  uint8 [B][H][NBcap][D channels][64]  byte j of a channel: block tokens 2j (low), 2j+1 (high)
 *   v_params uint8 [B][H][capacity tokens][D/32]
 *   k_res, v_res unused (may be NULL).  Inputs (K, V, Q) and the output are bf16.
 *   Quantizer: shared exponent e = clamp(floor(log2(max|x|)) - 2, -127, 127) (byte 127 and zero
 *   codes for an all-zero group); element = nearest e2m1 to x / 2^e, ties to the even code,
 *   saturating at +-6, a zero magnitude stored as +0.
 */
#ifndef BITDECODE_H
#define BITDECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BD_OK = 0,
  BD_ERR_INVALID_ARG = -1,   /* NULL pointer, non-positive size, bad enum, bad length */
  BD_ERR_UNSUPPORTED = -2,   /* a shape this build has no kernel for (head_dim != 128; batch, KV heads times pieces of the query group, or batch times KV heads, beyond 65535, a launch grid dimension) */
  BD_ERR_ALIGNMENT = -3,     /* a device pointer is not 16-byte aligned */
  BD_ERR_CAPACITY = -4,      /* the cache cannot hold the tokens asked for */
  BD_ERR_HIP = -5            /* a HIP runtime call failed; see bd_last_hip_error() */
} bd_status;

typedef enum {
  BD_FMT_INT4 = 0,      /* K channel-wise, V per token (the paper's KC setting, its default) */
  BD_FMT_INT2 = 1,
  BD_FMT_MXFP4 = 2,
  BD_FMT_INT4_KT = 3,   /* K per token as well (the paper's KT setting, Sec. IV-C(1)) */
  BD_FMT_INT2_KT = 4,
  /* K channel-wise, V per token, with a quantization group smaller than the 128-token residual
   * block (Sec. IV-C(1): K_p of shape (T_n/group, d), V_p of shape (T_n, d/group)): K statistics
   * over 64 or 32 tokens per channel, V statistics over 64 or 32 channels per token.  Codes as
   * in BD_FMT_INT4 / INT2; k_params uint32 [B][H][NBcap][128/group][D], v_params uint32
   * [B][H][capacity][D/group] (paged: [P][H][128/group][D] and [P][H][128][D/group]). */
  BD_FMT_INT4_G64 = 5,
  BD_FMT_INT4_G32 = 6,
  BD_FMT_INT2_G64 = 7,
  BD_FMT_INT2_G32 = 8,
  /* K per token with a quantization group as well (the KT setting with a group; Sec. IV-C(1): tensor-wise
   * parameters of shape (T_n, d/group)): K statistics over 64 or 32 channels per token, exactly like V's.
   * Codes as in BD_FMT_INT4 / INT2; k_params and v_params both uint32 [B][H][capacity][D/group]
   * (paged: [P][H][128][D/group]). */
  BD_FMT_INT4_KT_G64 = 9,
  BD_FMT_INT4_KT_G32 = 10,
  BD_FMT_INT2_KT_G64 = 11,
  BD_FMT_INT2_KT_G32 = 12
} bd_format;

/* Element type of the attention output rows `out` (Fig. 2 caption: Out = softmax(Q D(K')^T) D(V')). */
typedef enum {
  BD_OUT_HALF = 0,   /* the type of the inputs: fp16 for the integer formats, bf16 for BD_FMT_MXFP4 */
  BD_OUT_F32 = 1     /* fp32: the kernels' fp32 result without the final rounding to 11 (fp16) or 8 (bf16) bits */
} bd_out_type;

/* Shape and buffers of one layer's cache.  Plain data, filled by the caller, passed by
 * const pointer; the six buffers are device pointers with the layouts given above. */
typedef struct bd_cache {
  int32_t batch;
  int32_t n_q_heads;     /* multiple of n_kv_heads; g_q = n_q_heads / n_kv_heads (Sec. IV-A) */
  int32_t n_kv_heads;
  int32_t head_dim;      /* 128 */
  int32_t format;        /* bd_format */
  int32_t capacity;      /* tokens per sequence the packed buffers can hold; multiple of 128 */
  void *k_codes, *v_codes;
  void *k_params, *v_params;
  void *k_res, *v_res;
  int32_t out_type;      /* bd_out_type of every `out` argument used with this cache (0 = BD_OUT_HALF) */
} bd_cache;

/* Size in bytes of buffer `which` (0 k_codes, 1 v_codes, 2 k_params, 3 v_params, 4 k_res,
 * 5 v_res) for the shape fields of `c` (pointers ignored).  0 on a bad argument. */
size_t bd_cache_bytes(const bd_cache* c, int which);

/* Split factor the library would pick for this shape and length (>= 1): how many
 * workgroups share the context of one (sequence, KV head), FlashDecoding-style split
 * over the context (the "split-partitioned" scheme named in Sec. V-A). */
int32_t bd_choose_splits(const bd_cache* c, int32_t packed_len);

/* Bytes of device workspace bd_decode_attn needs for `num_splits`: num_splits partial
 * results, each batch*n_q_heads*(128 + 2) floats (unnormalised output row, running max
 * in log2 units, running sum).  The residual tokens are shared out over the splits. */
size_t bd_workspace_bytes(const bd_cache* c, int32_t num_splits);

/* Prefill (Sec. IV-B(1)): quantize and pack the first L - (L mod 128) tokens of
 * k, v (device, [B][H][L][D] contiguous, fp16; bf16 for MXFP4) and copy the remaining
 * L mod 128 tokens into the fp16 residual.  For MXFP4 all L tokens are quantized.
 * Writes the resulting lengths to the host integers *packed_len, *res_len
 * (MXFP4: *packed_len = L, *res_len = 0).  L = 0 is allowed.  BD_ERR_CAPACITY if the
 * tokens to pack exceed capacity. */
bd_status bd_quant_pack_kv(const bd_cache* c, const void* k, const void* v, int32_t L,
                           int32_t* packed_len, int32_t* res_len, void* stream);

/* Decode-step append (Sec. IV-B(1)): store the new token k_new, v_new (device, [B][H][D])
 * in residual slot *res_len; when that fills the 128-token block, quantize and pack the
 * block as packed block packed_len/128 in the same call, so that on return
 * 0 <= *res_len <= 127 and prefill(L) followed by n appends equals prefill(L + n) bit for bit.
 * For MXFP4 the token is quantized directly.  *packed_len / *res_len are host in-out.
 * BD_ERR_CAPACITY (state unchanged) if the flush would not fit. */
bd_status bd_append_kv(const bd_cache* c, const void* k_new, const void* v_new,
                       int32_t* packed_len, int32_t* res_len, void* stream);

/* Decode attention (Fig. 2 caption; Sec. IV-A query transformation; Sec. IV-C fused
 * dequantize + QK^T + online softmax (Alg. 1) + PV; split over the context):
 * q device [B][n_q_heads][D] (fp16; bf16 for MXFP4); query head h attends KV head h / g_q
 * over the packed_len quantized tokens and the res_len residual tokens, logits scaled by
 * softmax_scale.  Writes num_splits partials into `workspace` (device, at least
 * bd_workspace_bytes(c, num_splits), 16-byte aligned; with num_splits == 1 and `out` given the
 * partials are not written: the attention kernel stores `out` itself, the same values, and no
 * merge kernel runs).  If `out` is non-NULL (device,
 * [B][n_q_heads][D], fp16 / bf16) the merge of the partials is enqueued too, so `out`
 * is complete when the stream passes this call; if NULL, call bd_splitk_combine.  (`out` has
 * the element type c->out_type names here and in every other call: fp16 / bf16, or fp32.)
 * num_splits >= 1 (any value; splits beyond the number of 128-token blocks stay empty).
 * With no tokens at all the output is zero. */
bd_status bd_decode_attn(const bd_cache* c, const void* q, int32_t packed_len, int32_t res_len,
                         float softmax_scale, int32_t num_splits, void* workspace, void* out,
                         void* stream);

/* bd_decode_attn for callers that cannot allocate device memory or pass a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the split partials go to a
 * static device array inside the library, BD_STATIC_SCRATCH_BYTES per GPU, held until the process
 * ends, instead of a caller's workspace.  Same kernels, same output bits as bd_decode_attn with
 * `out` given; `out` must be non-NULL.  Calls no allocating routine.  BD_ERR_CAPACITY if
 * bd_workspace_bytes(c, num_splits) exceeds BD_STATIC_SCRATCH_BYTES.  All calls on one GPU share
 * the array: calls that may overlap there (different streams, no ordering between them) race.  The
 * first call on a device looks the array's address up (do that call outside a graph capture). */
#define BD_STATIC_SCRATCH_BYTES (4u << 20)
bd_status bd_decode_attn_static(const bd_cache* c, const void* q, int32_t packed_len, int32_t res_len,
                                float softmax_scale, int32_t num_splits, void* out, void* stream);

/* One decode step in one call: exactly bd_append_kv(k_new, v_new) followed by
 * bd_decode_attn(q, ..., out) -- same cache contents, same lengths, same output bits -- in one
 * attention launch (plus the merge): the new token is attended straight from k_new / v_new and
 * filed into the residual by the attention kernel itself, and on the step that fills the residual
 * block the one workgroup that reads the new packed block quantizes it first (the fusion of the
 * paper's Residual Kernel, Sec. III-A(1) / Sec. IV-B, with the flush before the attention).
 * BD_FMT_MXFP4: the workgroup that reads the token's block quantizes the token into the cache before
 * it attends.  (The filling step of query groups above 16 heads -- 8 for the _G64 / _G32 formats -- runs
 * as the two calls.)  All pointers as in the two calls; `out` must be non-NULL.  Every argument is validated before the
 * append; only BD_ERR_HIP (a failed launch) can leave the token appended without the attention
 * having been enqueued, and *packed_len / *res_len then say so. */
bd_status bd_decode_step(const bd_cache* c, const void* k_new, const void* v_new, const void* q,
                         int32_t* packed_len, int32_t* res_len, float softmax_scale,
                         int32_t num_splits, void* workspace, void* out, void* stream);

/* The same step with the paper's own flush order (Sec. III-A(1), Sec. IV-B(1): the Residual Kernel
 * attends the half-precision residual block and quantizes it, in the same kernel, only once it holds N_r
 * tokens): identical to bd_decode_step on every step but the one that fills the residual block.  On
 * that step the attention reads the block's 128 tokens in fp16 -- no quantization error on them yet --
 * and the same launch packs them (one extra workgroup per KV head); on return the lengths and the
 * cache bytes are those bd_decode_step leaves.  Integer formats; BD_FMT_MXFP4 keeps no residual and
 * behaves as in bd_decode_step. */
bd_status bd_decode_step_lazy(const bd_cache* c, const void* k_new, const void* v_new, const void* q,
                              int32_t* packed_len, int32_t* res_len, float softmax_scale,
                              int32_t num_splits, void* workspace, void* out, void* stream);

/* Measurement aid, no part of the method: one launch that reads the packed K and V codes of the first
 * packed_len tokens (a multiple of 128) of every (sequence, KV head) unit of a cache, with the loads
 * bd_decode_attn uses, and computes nothing.  Its duration is the floor the memory system sets for a
 * decode launch over the same cache (where the breakdown of Sec. V-C ends up once loading the cache is all that is left).  `sink`
 * (device, 4 bytes, may be NULL) is written only for one value of the loaded data's checksum. */
bd_status bd_probe_stream_read(const bd_cache* c, int32_t packed_len, void* sink, void* stream);

/* Merge the num_splits partials left in `workspace` by bd_decode_attn (log-sum-exp
 * merge: m = max m_s, l = sum l_s 2^(m_s-m), O = sum O_s 2^(m_s-m) / l) into
 * out (device, [B][n_q_heads][D], fp16 / bf16). */
bd_status bd_splitk_combine(const bd_cache* c, const void* workspace, int32_t num_splits,
                            void* out, void* stream);

/* ---- Paged cache with per-sequence lengths (the "Page" setting of Sec. V-A / V-B) ----------
 *
 * The paper runs its kernels on a contiguous and on a page-managed KV cache and names no
 * layout.  Here a page is one 128-token quantization block: the packed blocks of all sequences
 * live in one pool, block n of sequence b is page block_table[b][n], and every sequence has its
 * own length, kept on the device.  P = num_pages; integer formats:
 *
 *   k_codes  uint32 [P][H][128 tokens][D/cpw]      v_codes  uint32 [P][H][D channels][128/cpw]
 *   k_params uint32 [P][H][D]                      v_params uint32 [P][H][128]
 *   k_res, v_res fp16 [B][H][128][D]               (per sequence, as in bd_cache)
 *   block_table int32 [B][max_pages_per_seq]       device; written by the caller, read by the library
 *   seq_lens    int32 [B]                          device; tokens cached per sequence; written by
 *                                                  bd_paged_quant_pack_kv / bd_paged_append_kv
 *   status      int32 [1]                          device, may be NULL; see below
 *
 * BD_FMT_MXFP4 quantizes every token on arrival, so there is no residual (k_res, v_res unused,
 * size 0) and the newest, partly filled block lives in a page as well: table entry n must be
 * valid before the sequence reaches token 128*n + 1.
 *
 *   k_codes  uint8 [P][H][128 tokens][D/2]         v_codes  uint8 [P][H][D channels][64]
 *   k_params uint8 [P][H][128][D/32]  (e8m0)       v_params uint8 [P][H][128][D/32]
 *
 * Inside a page every block has exactly the bytes it has in a bd_cache.  The caller owns the
 * page allocator: before a sequence reaches token 128*(n+1) its table entry n must name a page
 * no other block uses.  Because lengths live on the device the host cannot validate them; the
 * kernels do: a block whose table entry is missing (n >= max_pages_per_seq) or outside
 * [0, num_pages) is not read or written, bit 0 (decode) or bit 1 (append / prefill) of *status
 * is set, and an append that would have needed that block leaves the sequence's length as it
 * was (the token is dropped).  The caller clears *status. */
typedef struct bd_paged_cache {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;            /* 128 */
  int32_t format;              /* any bd_format */
  int32_t num_pages;
  int32_t max_pages_per_seq;
  void *k_codes, *v_codes;
  void *k_params, *v_params;
  void *k_res, *v_res;
  int32_t* block_table;
  int32_t* seq_lens;
  int32_t* status;
  int32_t out_type;            /* bd_out_type, as in bd_cache */
} bd_paged_cache;

/* Size in bytes of buffer `which` (0..5 as bd_cache_bytes, 6 block_table, 7 seq_lens). */
size_t bd_paged_cache_bytes(const bd_paged_cache* c, int which);

/* Workspace size for bd_paged_decode_attn (same layout as bd_workspace_bytes). */
size_t bd_paged_workspace_bytes(const bd_paged_cache* c, int32_t num_splits);

/* Prefill of sequence `seq` (Sec. IV-B(1)) from k, v (device, [H][L][D] fp16; bf16 for MXFP4):
 * the first L - (L mod 128) tokens are quantized into the sequence's pages, the rest copied to
 * its residual (MXFP4: all L tokens are quantized into pages), seq_lens[seq] = L.  Replaces
 * whatever the sequence held.  BD_ERR_CAPACITY if L needs more than max_pages_per_seq pages. */
bd_status bd_paged_quant_pack_kv(const bd_paged_cache* c, int32_t seq, const void* k, const void* v,
                                 int32_t L, void* stream);

/* One decode step of every sequence (Sec. IV-B): token b of k_new, v_new (device, [B][H][D]
 * fp16) goes to residual slot seq_lens[b] mod 128 of sequence b; a residual that reaches 128
 * tokens is quantized into page block_table[b][seq_lens[b] / 128]; seq_lens[b] += 1.
 * MXFP4 (bf16 inputs): the token is quantized straight into position seq_lens[b] mod 128 of that
 * page. */
bd_status bd_paged_append_kv(const bd_paged_cache* c, const void* k_new, const void* v_new, void* stream);

/* bd_decode_attn over the paged cache: sequence b attends its own seq_lens[b] tokens; a
 * sequence with no tokens gets a zero output row.  Every sequence is split num_splits ways
 * (pick it for the longest sequence, e.g. with bd_choose_splits on a bd_cache of the same
 * shape); workspace at least bd_paged_workspace_bytes(c, num_splits); `out` (device,
 * [B][n_q_heads][D] fp16; bf16 for MXFP4) must be non-NULL.  With num_splits == 1 the attention
 * kernel writes `out` itself and no merge runs. */
bd_status bd_paged_decode_attn(const bd_paged_cache* c, const void* q, float softmax_scale,
                               int32_t num_splits, void* workspace, void* out, void* stream);

/* One decode step of every sequence (Sec. III-A(1), IV-B: the step's append and its attention
 * in one call): the same results, bit for bit, as bd_paged_append_kv followed by
 * bd_paged_decode_attn, in fewer kernel launches.  With up to 16 query heads per KV head (8 for
 * the _G64 / _G32 formats): two -- the attention kernel reads the new token from k_new / v_new
 * and files it (integer formats: the workgroup that reads the block a step fills quantizes it
 * first; MXFP4: the workgroup that reads the token's block quantizes the token), and the merge,
 * the last kernel, raises the lengths.  Larger query groups: three -- append, attention, merge.
 * (With num_splits == 1 there is no merge and a small kernel raises the lengths.)  A sequence
 * whose token is dropped for want of a valid page (bit 1 of *status) attends the tokens it had. */
bd_status bd_paged_decode_step(const bd_paged_cache* c, const void* k_new, const void* v_new,
                               const void* q, float softmax_scale, int32_t num_splits,
                               void* workspace, void* out, void* stream);

/* The same step with the paper's own flush order (Sec. III-A(1), Sec. IV-B(1); see bd_decode_step_lazy): a
 * sequence whose residual block this step's token fills is attended with its 128 residual tokens in half
 * precision, and one extra workgroup per (sequence, KV head) of the same attention launch packs them into the
 * sequence's next page; the other sequences of the batch behave as in bd_paged_decode_step.  Two launches for
 * every query group size.  On return the pool, the lengths and *status are those bd_paged_decode_step leaves.
 * BD_FMT_MXFP4 keeps no residual and behaves as in bd_paged_decode_step. */
bd_status bd_paged_decode_step_lazy(const bd_paged_cache* c, const void* k_new, const void* v_new,
                                    const void* q, float softmax_scale, int32_t num_splits,
                                    void* workspace, void* out, void* stream);

/* Text for a status code (static storage). */
const char* bd_strerror(bd_status s);

/* hipError_t value of the last failing HIP call seen by this thread (0 if none). */
int bd_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BITDECODE_H */
