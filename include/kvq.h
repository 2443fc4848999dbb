/*
 * kvq.h -- C ABI of the key-prioritized mixed-precision KV cache for MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of "Quantize What Counts: More for Keys,
 * Less for Values" (arXiv 2502.15075): keys and values of one transformer layer are stored at
 * independent bit widths b_K, b_V (Sec. 1; Theorem 2: b_K > b_V when ||K||_F > ||V||_F; K4V2 is
 * the headline allocation), each quantized group-wise with the b-bit uniform scalar quantizer of
 * App. B "Preliminaries" in its asymmetric min-max form, and single-token decode attention
 * (App. A: A = softmax(q K^T / sqrt(d)), output A V) reads the packed codes directly.
 *
 * Conventions
 *   - Every pointer in kvq_cache and every tensor argument is a DEVICE pointer owned by the
 *     caller.  The library never allocates, frees or synchronizes; each call enqueues kernels on
 *     the given hipStream_t (passed as void*; NULL = the default stream) and returns.
 *   - Arguments are validated on the host before anything is launched; on error nothing ran.
 *   - Status codes only: the library never aborts, throws or prints.
 *   - Not checked (undefined results): non-finite inputs, |x| > 65504, overlapping buffers, concurrent
 *     calls that write the same cache, a v_scale_exp array that was not zeroed with the cache it belongs to.
 *
 * Quantizer (per tensor X in {K, V}, bits b, group size G; one group = G consecutive head_dim
 * elements of one token row -- token-wise grouping, Sec. 4 "Downstream Task Accuracy"):
 *     mn, mx   = min, max of the group in binary32 (mn = -0 is stored as +0)
 *     scale    = binary16( (mx - mn) / (2^b - 1) )        zero = binary16( mn )
 *     code_d   = clip( rint( (x_d - zero) * (1 / scale) ), 0, 2^b - 1 )   (all codes 0 if scale == 0)
 *     x^_d     = code_d * scale + zero                                   (App. B "Dequantization")
 *   every operation rounded once in binary32, round-to-nearest-even; codes use the STORED scale/zero.
 *
 * Rotation (rotate_k = 1; Sec. 4 "Integration with Rotation-Based Methods", Sec. 5.3: rotating the keys, not the
 * values, is what helps): every key row k is replaced by R k, R = H_128 diag(s) / sqrt(128) with H_128 the Sylvester
 * Hadamard matrix and s the signs of signs_k, before it is quantized, and the query is replaced by R q inside the
 * attention kernels, so the scores are those of the unrotated vectors up to rounding.  Arithmetic: signs first
 * (exact), then the butterfly network over strides 1, 2, 4, ..., 64 in that order, each butterfly one binary32
 * addition and one binary32 subtraction (lower index minus higher index), then one multiplication by
 * binary32(1/sqrt(128)).  R k goes to the quantizer in binary32; R q is rounded once to binary16.
 * kvq_dequantize returns keys in the input basis (R^T of the stored reconstruction: butterflies, scale, signs).
 * rotate_v = 1 does the same to value rows with R_v built from signs_v (the paper's study compares no rotation,
 * keys, values, both, and finds that values gain nothing): the attention kernels accumulate in the rotated basis and
 * apply R_v^T to the normalized output (binary32 butterflies) before it is stored.
 *
 * Channel-wise keys (axis_k = KVQ_AXIS_SEQ; Sec. 4 "Downstream Task Accuracy": the per-column back-end with its
 * full-precision residual buffer): a key group is G = group_k (32, 64 or 128) consecutive tokens of one channel.  The
 * newest tokens are kept as their 16-bit input patterns in a residual buffer of RL token slots, keys and values both
 * (k_resid, v_resid in kvq_cache, sizes from kvq_residual_bytes); RL = resid_len, or G when that field is 0; RL is 64
 * or 128 and a multiple of G (G = 32 therefore needs resid_len = 64 or 128; other lengths: KVQ_ERR_UNSUPPORTED, a buffer
 * that whole groups do not fill: KVQ_ERR_INVALID_ARG).  The token that completes a block of RL tokens triggers the
 * flush of that block: its key rows are quantized channel by channel (one scale/zero per channel and group of G tokens,
 * RL / G groups per block, same arithmetic as above with the group running over tokens), its value rows token-wise as
 * always.  Attention reads tokens below floor(seq_len / RL) * RL from the codes and the rest from the buffer.  Contract:
 * tokens are appended in order starting at 0 (pos = number of tokens appended so far), in_dtype = raw_dtype, and
 * seq_len of a decode call is that number.  Every quantized width for keys and values; bits 16 and rotate_v are not
 * combined with it; axis_v stays KVQ_AXIS_HEAD_DIM.  With rotate_k (Sec. 5.3's key-only rotation on this back-end) the
 * buffer keeps the input rows, a flush quantizes R k of every row of the block, and attention scores the flushed tokens
 * with binary16(R q) and the tail with q itself.  Attention needs a query of raw_dtype (KVQ_ERR_UNSUPPORTED otherwise);
 * kvq_decode_step is the append followed by the attention (several launches).  With per-sequence lengths
 * (kvq_decode_attention_varlen, kvq_decode_step_varlen) every sequence has its own count of appended tokens, its own
 * flushed blocks and its own tail in its residual buffer; kvq_decode_step_varlen appends sequence b's token at pos[b]
 * (= its count so far; in_dtype = raw_dtype).  kvq_dequantize and
 * kvq_reconstruction_error read the codes only: the caller keeps t1 at or below the number of flushed tokens.
 * Format: T_cap is a multiple of RL; k_meta is [B][H_kv][T_cap/G][D] entries {scale, zero},
 * entry (t/G, d); k_resid is [B][H_kv][RL][D] 16-bit patterns, token t in slot t%RL; v_resid is [B][H_kv][RL/32] blocks
 * in the v_codes order with b_V = 16, token t in block (t%RL)/32; the other planes are as below.
 *
 * Paged planes (page_tokens = P != 0; what a serving stack with a block table does): each plane is a pool
 * [n_pages][H_kv][...one head's share of a contiguous cache of capacity P...], and token t of sequence b lives in pool
 * page page_table[b][t / P] at local position t % P.  kvq_cache_bytes reports the pool sizes.  Every call takes the
 * table as it is at launch time; pages of different sequences must not alias unless they are only read.  With
 * channel-wise keys the four code and scale/zero planes are paged the same way (group_k = 64 with a 64-slot buffer only,
 * other lengths: KVQ_ERR_UNSUPPORTED; a 64-token block never straddles a page; k_meta holds P/64 blocks per page and
 * head) and the residual buffers stay per sequence.
 *
 * Storage format of one layer (sizes from kvq_cache_bytes; T_cap = max_seq rounded up to 32):
 *   k_codes  [B][H_kv][T_cap][D*b_K/8]      b_K in {1,2,4,8,16}: element d of a row at bits [d*b_K, (d+1)*b_K),
 *                                           little-endian.  b_K = 3 and 6: the row is cut into chunks of 32
 *                                           channels (4*b_K bytes); with LO = 2 (b_K = 3) or 4 (b_K = 6) and
 *                                           HI = b_K - LO, element x of a chunk has code mod 2^LO at bits
 *                                           [x*LO, (x+1)*LO) of the chunk and code >> LO at bits
 *                                           32*LO + [x*HI, (x+1)*HI)
 *   k_meta   [B][H_kv][T_cap/16][D/G_K][16] entries {uint16 scale, uint16 zero} (binary16 patterns);
 *                                           entry (t/16, g, t%16) is token t, group g
 *   v_codes  [B][H_kv][T_cap/32][512*b_V]   32-token blocks laid out in the order a 16x16x32 matrix
 *                                           instruction consumes a "tokens x channels" operand.  With
 *                                             u=t%32, x4=u/16, j=(u%16)/4, r=u%4, i=4*x4+r, x=i%2, v=i/2,
 *                                             q=4*(d/16)+v, P=16/b_V, e=q/P, p=q%P
 *                                           the code of (t, d) sits in the little-endian 32-bit word at
 *                                           byte (e/4)*1024 + (16*j + d%16)*16 + 4*(e%4) of the block,
 *                                           at bit 16*x + b_V*p; for b_V = 1 (a block is 512 bytes, P = 16) at
 *                                           byte (16*j + d%16)*8 + 4*e, bit 16*x + p.  b_V = 3 and 6: the block
 *                                           is a block of LO-bit fields (LO = 2, 4) holding code mod 2^LO
 *                                           followed by a block of (b_V - LO)-bit fields holding code >> LO,
 *                                           each in the order just given for its field width.
 *   v_meta   as k_meta with G_V.
 *   bits == 16 keeps the 16-bit input patterns (raw_dtype) in the same positions; no meta plane.
 */
#ifndef KVQ_H
#define KVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVQ_OK = 0,
  KVQ_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bits/group not allowed, bad head ratio */
  KVQ_ERR_UNSUPPORTED = 2, /* a valid request this build has no kernel for (head_dim != 128, axis) */
  KVQ_ERR_CAPACITY = 3,    /* pos + n_new > max_seq, seq_len > max_seq */
  KVQ_ERR_WORKSPACE = 4,   /* workspace smaller than kvq_decode_workspace_bytes */
  KVQ_ERR_DEVICE = 5,      /* the HIP runtime reported an error at launch */
  KVQ_ERR_STATIC_SCRATCH = 6 /* kvq_decode_attention_static only: the call needs more partial-record bytes than
                                KVQ_STATIC_SCRATCH_BYTES; use kvq_decode_attention with a workspace of the caller's */
} kvq_status;

typedef enum { KVQ_F16 = 0, KVQ_BF16 = 1, KVQ_F32 = 2 } kvq_dtype;

typedef enum {
  KVQ_AXIS_HEAD_DIM = 0, /* token-wise: groups of G channels inside one token row (Sec. 4, "per-row") */
  KVQ_AXIS_SEQ = 1       /* channel-wise: groups of tokens of one channel (Sec. 4, "per-column"); keys only, see
                            "Channel-wise keys" above */
} kvq_axis;

/* Immutable description of one layer's cache.  head_dim must be 128.  bits in {1,2,3,4,6,8,16} (the per-column
 * back-end's grid {1,2,4,6,8}, Table 1's 3-bit keys): 2^b - 1 steps.  Key rows are stored at their own width (a row
 * of 3-bit codes is 48 bytes), and so are value codes (a 32-token block of b-bit codes is 512 b bytes);
 * group in {32,64,128} (ignored for bits == 16).  raw_dtype (KVQ_F16 / KVQ_BF16) is the element
 * type of a plane whose bits == 16. */
typedef struct {
  int32_t batch, kv_heads, max_seq, head_dim;
  int32_t bits_k, bits_v;
  int32_t group_k, group_v;
  int32_t axis_k, axis_v;
  int32_t raw_dtype;
  int32_t rotate_k;     /* 0 / 1: key-only randomized Hadamard rotation (see "Rotation" above); needs bits_k < 16 */
  uint32_t signs_k[4];  /* the 128 signs of the rotation: bit d%32 of word d/32 set means s_d = -1 */
  int32_t rotate_v;     /* 0 / 1: the same rotation for value rows, with its own signs; needs bits_v < 16 */
  uint32_t signs_v[4];
  int32_t page_tokens;  /* 0: every (b, h) stream is contiguous.  Otherwise (a power of two, 64..65536) the planes are
                           pools of n_pages pages found through kvq_cache.page_table; see "Paged planes" above */
  int32_t n_pages;      /* pages in the pool (page_tokens != 0) */
  int32_t resid_len;    /* slots of the full-precision residual buffer: 0 (none; with axis_k = KVQ_AXIS_SEQ: group_k of
                           them), 64, or with channel-wise keys 128 (see "Channel-wise keys" above; the group sizes
                           are the grid {32, 64, 128} of the group-size study, Sec. 4 "Integration with Rotation-Based
                           Methods", the 64-token buffer is that of the downstream runs).
                           With axis_k = KVQ_AXIS_HEAD_DIM and 64 the keys stay token-wise and the
                           cache differs from the plain one only in that the newest seq_len mod 64 tokens are still in
                           the buffer (Sec. 4 "Downstream Task Accuracy": a 64-token buffer in front of 128-element
                           groups); everything said under "Channel-wise keys" about the buffer, the flush, the
                           appends in order and the calls holds for it, with the keys of a flushed block quantized row
                           by row as on the plain path.  rotate_k may be combined with it, bits 16 and rotate_v not. */
} kvq_layout;

/* Caller-owned device buffers of at least the sizes kvq_cache_bytes reports (16-byte aligned).
 * A meta pointer may be NULL iff the matching bits == 16. */
typedef struct {
  void *k_codes, *k_meta, *v_codes, *v_meta;
  void *k_resid, *v_resid; /* residual buffers (axis_k = KVQ_AXIS_SEQ, or resid_len = 64); NULL otherwise */
  const int32_t* page_table; /* paged planes: device, int32 [B][ceil(max_seq / page_tokens)]: logical page -> pool page
                                (each in [0, n_pages); entries of pages no call touches are never read); else NULL */
  int32_t* v_scale_exp;      /* device, int32 [B][H_kv], part of the cache's state whenever bits_v < 16 (else it may be
                                NULL): the largest binary16 exponent field of any value scale of 64 or more stored in
                                that (b, h) stream so far, 0 if there is none.  The caller zeroes it when the cache is
                                created or a batch slot is handed to a new sequence; every call that stores value scales
                                raises it, and the attention kernels read it: they form binary16 products of softmax
                                weight and value scale, and a stream that holds such a scale gets that many bits of
                                room (ordinary values, whose groups span less than 64 (2^b - 1), never touch it). */
} kvq_cache;

/* Host only.  bytes_out = sizes of k_codes, k_meta, v_codes, v_meta.  Pins the paper's memory
 * claim (Sec. 1): K4V2 code bytes are 3/4 of K4V4's. */
kvq_status kvq_cache_bytes(const kvq_layout* layout, size_t bytes_out[4]);

/* Host only.  bytes_out = sizes of k_resid, v_resid: 0, 0 unless the layout has a residual buffer (axis_k =
 * KVQ_AXIS_SEQ, or resid_len = 64). */
kvq_status kvq_residual_bytes(const kvq_layout* layout, size_t bytes_out[2]);

/* Bytes of scratch kvq_decode_attention needs for (q_heads, seq_len): the partial (max, sum, accumulator) records of its
 * split-sequence pass.  May be 0 (enough (b, h_kv) streams to fill the chip without splitting the sequence); then the
 * workspace pointer may be NULL.  Never shrinks as seq_len grows: a workspace sized once for the longest sequence
 * serves every shorter one.  Touches no device memory; the split plan follows the compute-unit count of the CURRENT
 * device (256 when no device is usable), so size the workspace with the device current that the decode calls run on. */
kvq_status kvq_decode_workspace_bytes(const kvq_layout* layout, int32_t q_heads, int32_t seq_len,
                                      size_t* bytes_out);

/* Quantize n_new tokens of keys and values and store them at positions [pos, pos + n_new)
 * (the per-step cache update of autoregressive decoding, Sec. 4 "Quantization-Error Evaluation").
 *   k_new, v_new   [B][H_kv][n_new][D] of in_dtype (KVQ_F16 / KVQ_BF16), element strides given,
 *                  the D axis contiguous.  For bits == 16, in_dtype must equal raw_dtype.
 * Writes only the bytes (for values: only the bit fields) of those tokens.  n_new == 0 is a no-op. */
kvq_status kvq_quantize_append(const kvq_layout* layout, const kvq_cache* cache, const void* k_new,
                               const void* v_new, kvq_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                               int64_t stride_t, int32_t pos, int32_t n_new, void* stream);

/* Decode attention of one query token per sequence over cached tokens [0, seq_len):
 *   out[b,hq,:] = softmax_t( softmax_scale * q[b,hq,:] . K^[b,hq/R,t,:] ) . V^[b,hq/R,t,:],  R = q_heads/kv_heads
 * (App. A; the caller passes softmax_scale = 1/sqrt(head_dim); it must be positive and finite).
 *   q    [B][q_heads][D] contiguous, KVQ_F16 or KVQ_BF16 (used exactly; values beyond binary16 range
 *        are not supported); q_heads / kv_heads in 1..8 (with 32-element groups on both tensors: up to 8, and the
 *        head count times the groups per row at most 32 after rounding the heads up to a power of two).
 *   out  [B][q_heads][D] contiguous, KVQ_F32 (the graded type), KVQ_F16 or KVQ_BF16 (rounded once).
 *   workspace  at least kvq_decode_workspace_bytes(layout, q_heads, seq_len) bytes, 16-byte aligned.
 * Unquantized tensors (bits == 16; both: the full-precision baseline; one: the ablation that quantizes only keys or
 * only values, Table 1's discussion): a 16-bit key plane is multiplied by the query as it is, so q_dtype must be
 * raw_dtype (KVQ_ERR_UNSUPPORTED otherwise).  With exactly one tensor unquantized the keys are token-wise, values are
 * not rotated, and the head count times the groups per row of the quantized tensor is at most 16
 * (KVQ_ERR_UNSUPPORTED otherwise). */
kvq_status kvq_decode_attention(const kvq_layout* layout, const kvq_cache* cache, const void* q,
                                kvq_dtype q_dtype, int32_t q_heads, int32_t seq_len, float softmax_scale,
                                void* out, kvq_dtype out_dtype, void* workspace, size_t workspace_bytes,
                                void* stream);

/* kvq_decode_attention for callers that cannot allocate device memory and so have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same arguments and the same
 * results bit for bit, but the partial (max, sum, accumulator) records of a split sequence go to an array of
 * KVQ_STATIC_SCRATCH_BYTES that is part of the library's device code (every GPU the library runs on holds its own copy
 * until the process ends; the array's device address is looked up once per device, on the first call with that device
 * current).  The call allocates nothing, frees nothing and calls no allocating routine.
 *   - a call that needs more than KVQ_STATIC_SCRATCH_BYTES of records (kvq_decode_workspace_bytes tells) returns
 *     KVQ_ERR_STATIC_SCRATCH and launches nothing;
 *   - every call on one GPU shares that GPU's array, whatever its stream: calls that can overlap in time on one GPU
 *     race on it (calls on one stream, or ordered by events, do not).  The array keeps the last call's records; nothing
 *     in it has to start at zero, because every record a call reads is one that the same call wrote. */
#define KVQ_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
kvq_status kvq_decode_attention_static(const kvq_layout* layout, const kvq_cache* cache, const void* q,
                                       kvq_dtype q_dtype, int32_t q_heads, int32_t seq_len, float softmax_scale,
                                       void* out, kvq_dtype out_dtype, void* stream);

/* One autoregressive decode step (Sec. 4: the cache grows by one quantized token per generated token): quantize the new
 * token's K/V row of every (b, h_kv) into position pos -- same bytes as kvq_quantize_append with n_new = 1 -- then
 * attend over tokens [0, pos].  Token-wise keys: the append is fused into the attention kernel (one launch, plus the
 * merge launch when the sequence is split).  Channel-wise keys: the append kernel, then the attention launches.
 * A cache with an unquantized tensor (bits == 16 for keys, values or both) has no fused step (KVQ_ERR_UNSUPPORTED):
 * call kvq_quantize_append with n_new = 1, then kvq_decode_attention.
 *   k_new, v_new   [B][H_kv][D] of in_dtype (KVQ_F16 / KVQ_BF16), element strides given, D contiguous.
 *   everything else as in kvq_decode_attention with seq_len = pos + 1. */
kvq_status kvq_decode_step(const kvq_layout* layout, const kvq_cache* cache, const void* k_new, const void* v_new,
                           kvq_dtype in_dtype, int64_t stride_b, int64_t stride_h, int32_t pos, const void* q,
                           kvq_dtype q_dtype, int32_t q_heads, float softmax_scale, void* out, kvq_dtype out_dtype,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Squared reconstruction error of cached tokens [t0, t1) against the full-precision rows they were made from:
 *   sums[b][h][0] = sum over t, d of (K[b,h,t,d] - K^[b,h,t,d])^2,  sums[b][h][1] the same for V,
 * the numerator of App. B's "Frobenius Norm (MSE) Perspective" (MSE = ||A - A^||_F^2 / number of entries; Table 1
 * reports it for keys at 3 and 4 bits); the caller divides by (t1-t0)*D (per head) or by the whole count.
 *   k_ref, v_ref  [B][H_kv][t1-t0][D] of ref_dtype (KVQ_F16 / KVQ_BF16): row 0 is token t0; element strides given,
 *                 D contiguous, 16-byte aligned rows; either may be NULL (its sums are then 0).
 *   sums          double[B][H_kv][2], overwritten.  x^ is the binary32 reconstruction of kvq_dequantize; differences
 *                 and the squares of 8 adjacent channels are summed in binary32 (relative error below 1e-6), the
 *                 rest in binary64; the order of those additions is not fixed (relative spread about 2^-50).
 * t0 == t1 writes zeros and reads no reference row. */
kvq_status kvq_reconstruction_error(const kvq_layout* layout, const kvq_cache* cache, const void* k_ref,
                                    const void* v_ref, kvq_dtype ref_dtype, int64_t stride_b, int64_t stride_h,
                                    int64_t stride_t, int32_t t0, int32_t t1, double* sums, void* stream);

/* The two calls above for sequences of different lengths in one batch (what a serving batch looks like):
 *   seq_lens  device, int32[B]: batch element b attends over tokens [0, seq_lens[b]); values are clamped to
 *             [1, max_seq_len] on the device.
 *   pos       device, int32[B]: the new token of batch element b goes to position pos[b] (clamped to [0, max_pos]) and
 *             its query attends over [0, pos[b]].
 *   max_seq_len / max_pos  host: an upper bound of the device values; the launch and the workspace
 *             (kvq_decode_workspace_bytes(layout, q_heads, max_seq_len), max_seq_len = max_pos + 1) are planned for it.
 * Everything else as in the uniform calls; channel-wise keys included (see "Channel-wise keys" above). */
kvq_status kvq_decode_attention_varlen(const kvq_layout* layout, const kvq_cache* cache, const void* q,
                                       kvq_dtype q_dtype, int32_t q_heads, const int32_t* seq_lens,
                                       int32_t max_seq_len, float softmax_scale, void* out, kvq_dtype out_dtype,
                                       void* workspace, size_t workspace_bytes, void* stream);
kvq_status kvq_decode_step_varlen(const kvq_layout* layout, const kvq_cache* cache, const void* k_new,
                                  const void* v_new, kvq_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                                  const int32_t* pos, int32_t max_pos, const void* q, kvq_dtype q_dtype,
                                  int32_t q_heads, float softmax_scale, void* out, kvq_dtype out_dtype, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* Reconstruct tokens [t0, t1) as x^ = code * scale + zero (App. B "Dequantization"):
 *   k_out, v_out  [B][H_kv][t1-t0][D] contiguous of out_dtype; either may be NULL to skip it.
 * KVQ_F32 output is exactly the binary32 value; 16-bit outputs round it once. */
kvq_status kvq_dequantize(const kvq_layout* layout, const kvq_cache* cache, int32_t t0, int32_t t1,
                          void* k_out, void* v_out, kvq_dtype out_dtype, void* stream);

/* Device self-test of the quantizer's arithmetic (App. B "Preliminaries": the scale factor (max - min) / (2^b - 1) and
 * the division by it).  Codes and scale bytes are bit-exact only if those two divisions are correctly rounded; the
 * kernels compute them in three operations each (a multiplication by the rounded reciprocal of 2^b - 1 with one exact
 * correction step; one refinement of the hardware's reciprocal approximation of the stored scale), which is exact
 * for every possible scale on gfx950.  This call checks it on the device it runs on.
 * counters: DEVICE pointer to two uint32, overwritten asynchronously on `stream`:
 *   counters[0] = how many of the 31743 positive finite binary16 scales get a reciprocal that differs from IEEE division,
 *   counters[1] = how many of 6 x 2^24 sampled quotients x / (2^b - 1), b in {1,2,3,4,6,8}, differ from IEEE division.
 * Both must read 0.  KVQ_ERR_INVALID_ARG for a null or misaligned pointer. */
kvq_status kvq_selftest_quantizer(uint32_t* counters, void* stream);

const char* kvq_status_string(kvq_status status);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
