/*
 * kvq_oracle.c -- plain, slow, single-purpose CPU oracle for the mixed-precision KV cache
 * ("Quantize What Counts: More for Keys, Less for Values", arXiv 2502.15075).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library; nothing on the product
 * path may call it.  It shares no code, header, table or helper with the GPU sources.
 *
 * What it computes, and which passage each part follows:
 *
 *   - the b-bit uniform scalar quantizer "scale, round, clip, reconstruct" of App. B
 *     "Preliminaries" (scale factor, Q = round(A/alpha) clipped to the code range,
 *     A^ = alpha Q), applied per group of G consecutive head_dim elements of one token row
 *     (token-wise grouping, Sec. 4 "Downstream Task Accuracy"; group sizes Sec. 4
 *     "Integration with Rotation-Based Methods"), in its asymmetric min-max form with
 *     2^b - 1 steps over the group range (the reading that reproduces the 3-bit/4-bit error
 *     ratio of Table 1), codes unsigned 0 .. 2^b - 1, scale and zero stored as binary16;
 *   - independent bit widths b_K and b_V for keys and values (Sec. 1, Theorem 2);
 *   - the reconstruction A^ = code * scale + zero (App. B "Dequantization");
 *   - decode attention of one query row over the reconstructed cache,
 *     A = softmax(q K^T * softmax_scale), out = A V  (App. A notation table and the
 *     "attention outputs" equation), summed in binary64;
 *   - the reconstruction MSE of App. B "Frobenius Norm (MSE) Perspective";
 *   - key-only randomized Hadamard rotation before quantization (Sec. 4 "Integration with
 *     Rotation-Based Methods", Sec. 5.3: rotating keys carries the gain, rotating values does
 *     not): every key row k becomes R k with R = H_D diag(s) / sqrt(D), H_D the Sylvester
 *     Hadamard matrix and s a fixed vector of signs; the query is rotated by the same R at
 *     decode time, so the scores q.k are those of the unrotated vectors up to rounding.  The
 *     paper leaves the arithmetic to its third-party rotation package; the reading taken here:
 *     the transform is the in-place butterfly network over strides 1, 2, 4, ..., D/2 in that
 *     order, each butterfly one binary32 addition and one binary32 subtraction (lower index
 *     minus higher index), then one multiplication by binary32(1/sqrt(D)); the rotated key row
 *     goes to the quantizer in binary32, the rotated query is rounded once to binary16 (the
 *     16-bit query a half-precision model hands to attention).
 *
 *   - channel-wise key groups with a full-precision residual buffer (Sec. 4 "Downstream Task
 *     Accuracy": the per-column back-end, with the most recent tokens kept in full precision
 *     and flushed periodically): with axis_k = 1 a key group is G_K consecutive TOKENS of one
 *     channel.  The reading taken here: the newest tokens live as their 16-bit input patterns
 *     in a residual buffer of G_K token slots (keys and values both); when token t with
 *     (t + 1) % G_K == 0 arrives the buffer is flushed: the G_K key rows are quantized channel
 *     by channel (one scale/zero per channel and block), the G_K value rows token-wise as
 *     always; attention reads tokens below floor(seq_len / G_K) * G_K from the codes and the
 *     rest from the buffer.  Tokens must be appended in order, starting at 0.
 *     The buffer's length is a parameter of its own (resid_len): the downstream runs pair a 64-token buffer with
 *     128-element groups, which can only be groups along head_dim (a 64-token flush cannot fill a 128-token group):
 *     with axis_k = 0 and resid_len = RL the keys are token-wise as on the plain path, and the only difference to it
 *     is that the newest n mod RL tokens are still in the buffer; with axis_k = 1 a flush of RL tokens quantizes
 *     RL / G_K groups per channel.
 *     With rotate_k (the study's best setting, K4V2 with key-only rotation, on the per-column back-end of the
 *     downstream runs: Sec. 5.3 and Sec. 4) the buffer still keeps the input rows; a flush quantizes R k of every
 *     row, channel by channel in the rotated basis; attention takes the scores of the flushed tokens from the
 *     rotated query (rounded once to binary16, as with token-wise keys) and those of the tail from the query
 *     itself: the same bilinear form in exact arithmetic, since R is orthogonal.
 *
 * Arithmetic of the quantizer is IEEE binary32, round-to-nearest-even, one rounding per
 * written operation (build with -ffp-contract=off, no fast-math).  The decisions that
 * produce integers (codes) are therefore taken in binary32, the precision the GPU kernel
 * uses; everything that is not an integer decision (attention) is binary64.
 *
 * Storage format (the paper is silent on layout; this is the library's own format, stated
 * here in full because bytes are compared one by one):
 *
 *   capacity   T_cap = max_seq rounded up to a multiple of 32 tokens.
 *   k_codes    [B][H][T_cap][D*b_K/8] bytes; for b_K = 1, 2, 4, 8, 16 element d of a token row
 *              occupies bits [d*b_K, (d+1)*b_K) of the row read as a little-endian bit string.
 *              b_K = 3 and 6 keep a power-of-two low part and the rest of every code in two
 *              runs: the row is cut into chunks of 32 channels (4*b_K bytes each); with
 *              LO = 2 (b_K = 3) or 4 (b_K = 6) and HI = b_K - LO, element x of a chunk has
 *              code mod 2^LO at bits [x*LO, (x+1)*LO) of the chunk and code >> LO at bits
 *              [32*LO + x*HI, 32*LO + (x+1)*HI)  (a row of 3-bit codes is 48 bytes, of
 *              6-bit codes 96: nothing is padded to a power of two).
 *   *_meta     [B][H][T_cap/16][D/G][16] entries of 4 bytes: little-endian uint16 scale
 *              then little-endian uint16 zero (both binary16 bit patterns); entry
 *              (t/16, g, t%16) belongs to token t, group g.
 *   v_codes    [B][H][T_cap/32][512*b_V] bytes: blocks of 32 tokens.  b_V = 3 and 6: a block is a block of LO-bit
 *              fields (LO = 2, 4) holding code mod 2^LO followed by a block of (b_V - LO)-bit fields holding
 *              code >> LO, each laid out as follows for its own field width.  Inside a block of b-bit fields the
 *              code of (token t, channel d) lives in a little-endian 32-bit word found as
 *                u = t%32; x4 = u/16; j = (u%16)/4; r = u%4; i = 4*x4 + r; x = i%2; v = i/2;
 *                q = 4*(d/16) + v; P = 16/b; e = q/P; p = q%P;
 *                word byte offset = (e/4)*(8*D) + (16*j + d%16)*16 + 4*(e%4);
 *                bit offset inside the word = 16*x + b*p;
 *              b = 1 (P = 16) has one piece of D/64 words per lane instead:
 *                word byte offset = (16*j + d%16)*(D/16) + 4*e   (8 bytes per lane for D = 128).
 *              (For D = 128 the stride 8*D is 1024 bytes: one 16-byte piece per wavefront
 *              lane.  The order is the one in which a 16x16x32 matrix instruction wants a
 *              "tokens x channels" operand, so a decode kernel needs no transpose.)
 *   bits == 16 the planes hold the 16-bit input patterns unchanged in the same positions
 *              (b = 16 in the formulas above); the meta planes are unused.
 *   residual buffer (RL = resid_len slots; RL = group_k when resid_len is 0 and axis_k == 1): T_cap = max_seq rounded
 *              up to a multiple of max(32, RL); all four planes as above for tokens below floor(n / RL) * RL, n the
 *              number of tokens appended; with axis_k == 1 (channel-wise keys, G = group_k, RL a multiple of G)
 *              k_meta is [B][H][T_cap/G][D] entries (scale, zero as above): entry (t/G, d);
 *              k_resid [B][H][RL][D] 16-bit patterns, token t in slot t % RL, row-major;
 *              v_resid [B][H][RL/32] blocks in the v_codes order with b = 16, token t in block
 *                      (t % RL) / 32 at u = t % 32.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { REF_F16 = 0, REF_BF16 = 1, REF_F32 = 2 };

typedef struct {
  int32_t batch, kv_heads, max_seq, head_dim;
  int32_t bits_k, bits_v;   /* 1, 2, 3, 4, 6, 8, or 16 = keep the 16-bit input unquantized.  Codes of both tensors
                               are stored at their own width */
  int32_t group_k, group_v; /* G: consecutive head_dim elements sharing one scale/zero */
  int32_t raw_dtype;        /* REF_F16 or REF_BF16: meaning of the planes when bits == 16 */
  int32_t rotate_k;         /* 1: key rows are stored as codes of R k (needs bits_k < 16) */
  uint32_t signs_k[4];      /* bit d of the 128-bit little-endian string set: s_d = -1 (D <= 128) */
  int32_t axis_k;           /* 0: key groups along head_dim (token-wise); 1: along tokens (channel-wise) */
  int32_t rotate_v;         /* 1: value rows are stored as codes of R_v v (needs bits_v < 16); the attention output is
                               taken back with R_v^T.  The paper's rotation study covers none / keys / values / both. */
  uint32_t signs_v[4];
  int32_t resid_len;        /* slots of the full-precision residual buffer: 0 = none (axis_k == 0) or group_k (axis_k == 1) */
} ref_layout;

/* tokens the residual buffer holds before it is flushed; 0: the layout has no buffer */
static int resid_slots(const ref_layout* L) { return L->resid_len ? L->resid_len : (L->axis_k == 1 ? L->group_k : 0); }

/* ------------------------------------------------------------------ number formats */

/* binary16 bit pattern -> binary32 value (exact). */
float ref_f16_to_f32(uint16_t h) {
  int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  float v;
  if (e == 0) v = ldexpf((float)m, -24);                 /* zero and subnormals */
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexpf((float)(1024 + m), e - 25);
  return sign ? -v : v;
}

/* binary32 value -> nearest binary16 bit pattern, ties to even, subnormals kept,
 * overflow to infinity.  Works on the real number, not on bit tricks: find the spacing of
 * binary16 numbers around |f| and round the quotient with rint (ties-to-even). */
uint16_t ref_f32_to_f16(float f) {
  uint16_t sign = signbit(f) ? 0x8000u : 0u;
  if (isnan(f)) return (uint16_t)(sign | 0x7E00u);
  double a = fabs((double)f);
  if (isinf(f) || a >= 65520.0) return (uint16_t)(sign | 0x7C00u); /* 65520 = halfway to 2^16 */
  if (a == 0.0) return sign;
  int ex;
  (void)frexp(a, &ex);            /* a = frac * 2^ex, frac in [0.5,1)  =>  2^(ex-1) <= a */
  int e = ex - 1;                 /* unbiased exponent of a */
  if (e < -14) e = -14;           /* subnormal range shares the spacing of 2^-14 */
  double ulp = ldexp(1.0, e - 10);
  double q = rint(a / ulp);       /* exact quotient (power-of-two divisor), RNE */
  /* q is in [0, 2048]; 2048 means the rounding carried into the next binade */
  uint32_t bits;
  if (e == -14 && q < 1024.0) bits = (uint32_t)q;                       /* subnormal */
  else {
    if (q >= 2048.0) { q = 1024.0; e += 1; }
    bits = ((uint32_t)(e + 15) << 10) | ((uint32_t)q - 1024u);
  }
  return (uint16_t)(sign | bits);
}

float ref_bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static float load_elem(const void* base, int dtype, int64_t idx) {
  if (dtype == REF_F16) return ref_f16_to_f32(((const uint16_t*)base)[idx]);
  if (dtype == REF_BF16) return ref_bf16_to_f32(((const uint16_t*)base)[idx]);
  return ((const float*)base)[idx];
}

/* Threads the loops over independent (batch, head) streams are shared out to (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int ref_threads(void) { return omp_get_max_threads(); }
#else
int ref_threads(void) { return 1; }
#endif

/* ------------------------------------------------------------------ sizes */

static int bits_allowed(int b) { return b == 1 || b == 2 || b == 3 || b == 4 || b == 6 || b == 8; }

static int64_t cap_tokens(const ref_layout* L) {
  int64_t unit = resid_slots(L) > 32 ? resid_slots(L) : 32;
  return ((int64_t)L->max_seq + unit - 1) / unit * unit;
}

/* bytes of k_codes, k_meta, v_codes, v_meta */
int ref_plane_bytes(const ref_layout* L, uint64_t out[4]) {
  int64_t rows = (int64_t)L->batch * L->kv_heads * cap_tokens(L);
  int D = L->head_dim;
  out[0] = (uint64_t)(rows * (D * L->bits_k / 8));
  out[1] = L->bits_k == 16 ? 0 : L->axis_k == 1 ? (uint64_t)(rows / L->group_k * D * 4) : (uint64_t)(rows * (D / L->group_k) * 4);
  out[2] = (uint64_t)(rows * (D * L->bits_v / 8));
  out[3] = L->bits_v == 16 ? 0 : (uint64_t)(rows * (D / L->group_v) * 4);
  return 0;
}

/* ------------------------------------------------------------------ where things live */

/* byte offset of meta entry (token t, group g) inside one (b,h) stream of a meta plane */
static int64_t meta_offset(int64_t t, int g, int ngroups) {
  return (((t / 16) * ngroups + g) * 16 + (t % 16)) * 4;
}

/* K codes: bit offset of (t, d) inside one (b,h) stream, widths 1, 2, 4, 8, 16 */
static int64_t k_bit_offset(int64_t t, int d, int D, int b) { return (t * D + d) * b; }

/* V codes, one 32-token block of b-bit fields (b = 1, 2, 4, 8, 16): byte offset of the 32-bit word of (u = t%32, d)
 * inside the block and bit offset inside the word */
static void v_in_block(int u, int d, int D, int b, int64_t* word_byte, int* bit) {
  int x4 = u / 16, j = (u % 16) / 4, r = u % 4;
  int i = 4 * x4 + r;
  int x = i % 2, v = i / 2;
  int q = 4 * (d / 16) + v;
  int P = 16 / b;
  int e = q / P, p = q % P;
  if (b == 1)                     /* 1-bit codes: a lane piece is D/64 words (8 bytes for D = 128), one piece per block */
    *word_byte = (16 * j + d % 16) * (D / 16) + 4 * e;
  else
    *word_byte = (int64_t)(e / 4) * (8 * D) + (16 * j + d % 16) * 16 + 4 * (e % 4);
  *bit = 16 * x + b * p;
}

static void put_bits_le(uint8_t* base, int64_t bit_offset, int nbits, uint32_t value) {
  for (int k = 0; k < nbits; ++k) {
    int64_t pos = bit_offset + k;
    uint8_t mask = (uint8_t)(1u << (pos % 8));
    if ((value >> k) & 1u) base[pos / 8] |= mask; else base[pos / 8] &= (uint8_t)~mask;
  }
}
static uint32_t get_bits_le(const uint8_t* base, int64_t bit_offset, int nbits) {
  uint32_t v = 0;
  for (int k = 0; k < nbits; ++k) {
    int64_t pos = bit_offset + k;
    v |= (uint32_t)((base[pos / 8] >> (pos % 8)) & 1u) << k;
  }
  return v;
}

/* K codes of any width: widths 3 and 6 are stored as a low and a high run per 32-channel chunk (see the format) */
static void k_put_code(uint8_t* cs, int64_t t, int d, int D, int b, uint32_t code) {
  if (b != 3 && b != 6) { put_bits_le(cs, k_bit_offset(t, d, D, b), b, code); return; }
  int lo = b == 3 ? 2 : 4, hi = b - lo, x = d % 32;
  int64_t chunk = (t * D + (d - x)) * b;                    /* first bit of the chunk: 32 channels of b bits */
  put_bits_le(cs, chunk + (int64_t)x * lo, lo, code & ((1u << lo) - 1u));
  put_bits_le(cs, chunk + 32 * lo + (int64_t)x * hi, hi, code >> lo);
}
static uint32_t k_get_code(const uint8_t* cs, int64_t t, int d, int D, int b) {
  if (b != 3 && b != 6) return get_bits_le(cs, k_bit_offset(t, d, D, b), b);
  int lo = b == 3 ? 2 : 4, hi = b - lo, x = d % 32;
  int64_t chunk = (t * D + (d - x)) * b;
  return get_bits_le(cs, chunk + (int64_t)x * lo, lo) | (get_bits_le(cs, chunk + 32 * lo + (int64_t)x * hi, hi) << lo);
}

/* V codes of any width in one (b,h) stream: a block of 32 tokens takes 4*D*b bytes; widths 3 and 6 keep the codes' low
 * 2 (4) bits as a block of 2-bit (4-bit) fields followed by their high 1 (2) bits as a block of 1-bit (2-bit) fields */
static void v_put_code(uint8_t* cs, int64_t t, int d, int D, int b, uint32_t code) {
  uint8_t* blk = cs + (t / 32) * (4 * (int64_t)D * b);
  int u = (int)(t % 32), bit;
  int64_t wb;
  if (b != 3 && b != 6) { v_in_block(u, d, D, b, &wb, &bit); put_bits_le(blk + wb, bit, b, code); return; }
  int lo = b == 3 ? 2 : 4, hi = b - lo;
  v_in_block(u, d, D, lo, &wb, &bit);
  put_bits_le(blk + wb, bit, lo, code & ((1u << lo) - 1u));
  v_in_block(u, d, D, hi, &wb, &bit);
  put_bits_le(blk + 4 * (int64_t)D * lo + wb, bit, hi, code >> lo);
}
static uint32_t v_get_code(const uint8_t* cs, int64_t t, int d, int D, int b) {
  const uint8_t* blk = cs + (t / 32) * (4 * (int64_t)D * b);
  int u = (int)(t % 32), bit;
  int64_t wb;
  if (b != 3 && b != 6) { v_in_block(u, d, D, b, &wb, &bit); return get_bits_le(blk + wb, bit, b); }
  int lo = b == 3 ? 2 : 4, hi = b - lo;
  v_in_block(u, d, D, lo, &wb, &bit);
  uint32_t code = get_bits_le(blk + wb, bit, lo);
  v_in_block(u, d, D, hi, &wb, &bit);
  return code | (get_bits_le(blk + 4 * (int64_t)D * lo + wb, bit, hi) << lo);
}

/* ------------------------------------------------------------------ Hadamard rotation */

/* In-place butterfly network of the Walsh-Hadamard transform in Sylvester (natural) order:
 * after the strides 1, 2, ..., n/2 the vector holds H_n y, H_n[i][j] = (-1)^popcount(i & j).
 * Every butterfly is one binary32 addition and one binary32 subtraction. */
static void butterflies_f32(float* y, int n) {
  for (int h = 1; h < n; h *= 2)
    for (int i = 0; i < n; ++i)
      if ((i & h) == 0) {
        float a = y[i], b = y[i + h];
        y[i] = a + b;
        y[i + h] = a - b;
      }
}

static int sign_is_minus(const uint32_t* signs, int d) { return (int)((signs[d / 32] >> (d % 32)) & 1u); }

/* y = R x,  R = H_n diag(s) / sqrt(n)   (Sec. 4 "Integration with Rotation-Based Methods"). */
void ref_rotate(const float* x, int n, const uint32_t* signs, float* y) {
  float c = (float)(1.0 / sqrt((double)n));
  for (int d = 0; d < n; ++d) y[d] = sign_is_minus(signs, d) ? -x[d] : x[d];
  butterflies_f32(y, n);
  for (int d = 0; d < n; ++d) y[d] = y[d] * c;
}

/* x = R^T y = diag(s) H_n y / sqrt(n)   (H_n is symmetric and H_n H_n = n I, so R^T R = I). */
void ref_unrotate(const float* y, int n, const uint32_t* signs, float* x) {
  float c = (float)(1.0 / sqrt((double)n));
  for (int d = 0; d < n; ++d) x[d] = y[d];
  butterflies_f32(x, n);
  for (int d = 0; d < n; ++d) { float v = x[d] * c; x[d] = sign_is_minus(signs, d) ? -v : v; }
}

/* ------------------------------------------------------------------ the quantizer */

/* Quantize one group of n binary32 values to `bits`-bit codes (1 <= bits <= 8).
 * Returns the binary16 patterns of scale and zero through *S, *Z.
 *   range  = max - min, scale = range / (2^b - 1)            (App. B scale factor, min-max form)
 *   code   = clip(round((x - zero) / scale), 0, 2^b - 1)      (App. B "Quantization")
 * with the stored (binary16) scale and zero used for the codes, so that reconstruction
 * with the stored numbers is the inverse map, and the division done as multiplication by
 * the once-rounded reciprocal of the scale. */
void ref_quantize_group(const float* x, int n, int bits, uint8_t* codes, uint16_t* S, uint16_t* Z) {
  float mn = x[0], mx = x[0];
  for (int d = 1; d < n; ++d) {
    if (x[d] < mn) mn = x[d];
    if (x[d] > mx) mx = x[d];
  }
  if (mn == 0.0f) mn = 0.0f;                      /* -0 -> +0 : one canonical zero */
  float levels = (float)((1 << bits) - 1);
  float s32 = (mx - mn) / levels;
  uint16_t sb = ref_f32_to_f16(s32);
  if ((sb & 0x7FFFu) == 0) sb = 0;                /* no negative zero scale */
  uint16_t zb = ref_f32_to_f16(mn);
  float s = ref_f16_to_f32(sb), z = ref_f16_to_f32(zb);
  *S = sb;
  *Z = zb;
  if (s == 0.0f) {                                /* constant group (or range below binary16) */
    for (int d = 0; d < n; ++d) codes[d] = 0;
    return;
  }
  float rcp = 1.0f / s;
  for (int d = 0; d < n; ++d) {
    float t = (x[d] - z) * rcp;                   /* two roundings: subtract, multiply */
    float q = rintf(t);                           /* ties to even */
    if (q < 0.0f) q = 0.0f;
    if (q > levels) q = levels;
    codes[d] = (uint8_t)q;
  }
}

/* reconstruction of one element: code * scale + zero, one rounding (the product is exact) */
float ref_reconstruct(uint32_t code, uint16_t S, uint16_t Z) {
  return (float)code * ref_f16_to_f32(S) + ref_f16_to_f32(Z);
}

/* Quantize tokens [pos, pos+n_new) of every (b,h) stream and write them into the planes.
 * k_new / v_new: [B][H][n_new][D] with the given element strides (D contiguous).
 * Returns 0, or a negative number for an argument the format cannot take. */
int ref_quantize_append(const ref_layout* L, uint8_t* k_codes, uint8_t* k_meta, uint8_t* v_codes,
                        uint8_t* v_meta, const void* k_new, const void* v_new, int in_dtype,
                        int64_t stride_b, int64_t stride_h, int64_t stride_t, int32_t pos, int32_t n_new) {
  int D = L->head_dim;
  if (pos < 0 || n_new < 0 || (int64_t)pos + n_new > L->max_seq) return -3;
  if (D % 64 || D > 1024) return -1;
  if (L->rotate_k && (L->bits_k == 16 || D > 128 || (D & (D - 1)))) return -1;
  if (L->rotate_v && (L->bits_v == 16 || D > 128 || (D & (D - 1)))) return -1;
  if (L->axis_k != 0 || L->resid_len != 0) return -1;       /* channel-wise keys, residual buffer: ref_seq_append */
  uint64_t pb[4];
  ref_plane_bytes(L, pb);
  int64_t streams = (int64_t)L->batch * L->kv_heads;
  for (int which = 0; which < 2; ++which) {
    int b = which ? L->bits_v : L->bits_k, G = which ? L->group_v : L->group_k;
    if (b != 16 && (D % G || !bits_allowed(b))) return -1;
  }
  for (int which = 0; which < 2; ++which) {                 /* 0 = keys, 1 = values */
    int b = which ? L->bits_v : L->bits_k;
    int G = which ? L->group_v : L->group_k;
    const void* src = which ? v_new : k_new;
    uint8_t* cplane = which ? v_codes : k_codes;
    uint8_t* mplane = which ? v_meta : k_meta;
    int64_t cstream = (int64_t)(pb[which ? 2 : 0] / (uint64_t)streams);
    int64_t mstream = (int64_t)(pb[which ? 3 : 1] / (uint64_t)streams);
    /* the (b,h) streams are independent and write disjoint bytes: one thread each (only the loop is shared out; the
     * arithmetic of a stream is untouched) */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < streams; ++bh) {
      float* row = (float*)malloc(sizeof(float) * (size_t)D);
      float* plain = (float*)malloc(sizeof(float) * (size_t)D);
      uint8_t* codes = (uint8_t*)malloc((size_t)D);
      int64_t bi = bh / L->kv_heads, hi = bh % L->kv_heads;
      uint8_t* cs = cplane + bh * cstream;
      uint8_t* ms = mplane ? mplane + bh * mstream : NULL;
      for (int64_t tn = 0; tn < n_new; ++tn) {
        int64_t t = pos + tn;
        int64_t base = bi * stride_b + hi * stride_h + tn * stride_t;
        if (b == 16) {                                      /* unquantized: copy the 16-bit patterns */
          for (int d = 0; d < D; ++d) {
            uint32_t bits16 = ((const uint16_t*)src)[base + d];
            if (!which) put_bits_le(cs, k_bit_offset(t, d, D, 16), 16, bits16);
            else v_put_code(cs, t, d, D, 16, bits16);
          }
          continue;
        }
        for (int d = 0; d < D; ++d) row[d] = load_elem(src, in_dtype, base + d);
        if (which ? L->rotate_v : L->rotate_k) {            /* quantize R x instead of x */
          memcpy(plain, row, sizeof(float) * (size_t)D);
          ref_rotate(plain, D, which ? L->signs_v : L->signs_k, row);
        }
        for (int g = 0; g < D / G; ++g) {
          uint16_t S, Z;
          ref_quantize_group(row + g * G, G, b, codes + g * G, &S, &Z);
          uint8_t* m = ms + meta_offset(t, g, D / G);
          m[0] = (uint8_t)(S & 0xFF); m[1] = (uint8_t)(S >> 8);
          m[2] = (uint8_t)(Z & 0xFF); m[3] = (uint8_t)(Z >> 8);
        }
        for (int d = 0; d < D; ++d) {
          if (!which) k_put_code(cs, t, d, D, b, codes[d]);
          else v_put_code(cs, t, d, D, b, codes[d]);
        }
      }
      free(row); free(plain); free(codes);
    }
  }
  return 0;
}

/* Reconstruct tokens [t0,t1) of both tensors as binary32 exactly as stored: k_out, v_out are
 * [B][H][t1-t0][D]; with rotate_k the key rows are reconstructions of R k (rotated basis). */
int ref_dequantize_stored(const ref_layout* L, const uint8_t* k_codes, const uint8_t* k_meta, const uint8_t* v_codes,
                          const uint8_t* v_meta, int32_t t0, int32_t t1, float* k_out, float* v_out) {
  int D = L->head_dim;
  if (t0 < 0 || t1 < t0 || t1 > L->max_seq) return -3;
  if (L->axis_k != 0 || L->resid_len != 0) return -1;       /* channel-wise keys, residual buffer: ref_seq_dequantize */
  uint64_t pb[4];
  ref_plane_bytes(L, pb);
  int64_t streams = (int64_t)L->batch * L->kv_heads;
  int64_t nt = t1 - t0;
  for (int which = 0; which < 2; ++which) {
    int b = which ? L->bits_v : L->bits_k;
    int G = which ? L->group_v : L->group_k;
    const uint8_t* cplane = which ? v_codes : k_codes;
    const uint8_t* mplane = which ? v_meta : k_meta;
    float* out = which ? v_out : k_out;
    if (!out) continue;
    int64_t cstream = (int64_t)(pb[which ? 2 : 0] / (uint64_t)streams);
    int64_t mstream = (int64_t)(pb[which ? 3 : 1] / (uint64_t)streams);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < streams; ++bh) {
      const uint8_t* cs = cplane + bh * cstream;
      const uint8_t* ms = mplane ? mplane + bh * mstream : NULL;
      for (int64_t t = t0; t < t1; ++t)
        for (int d = 0; d < D; ++d) {
          uint32_t code;
          if (!which) code = k_get_code(cs, t, d, D, b);
          else code = v_get_code(cs, t, d, D, b);
          float val;
          if (b == 16) val = L->raw_dtype == REF_BF16 ? ref_bf16_to_f32((uint16_t)code) : ref_f16_to_f32((uint16_t)code);
          else {
            const uint8_t* m = ms + meta_offset(t, d / G, D / G);
            uint16_t S = (uint16_t)(m[0] | (m[1] << 8)), Z = (uint16_t)(m[2] | (m[3] << 8));
            val = ref_reconstruct(code, S, Z);
          }
          out[((bh * nt) + (t - t0)) * D + d] = val;
        }
    }
  }
  return 0;
}

/* Reconstruct tokens [t0,t1) in the basis of the inputs: as ref_dequantize_stored, and with
 * rotate_k every reconstructed key row y is taken back to R^T y. */
int ref_dequantize(const ref_layout* L, const uint8_t* k_codes, const uint8_t* k_meta, const uint8_t* v_codes,
                   const uint8_t* v_meta, int32_t t0, int32_t t1, float* k_out, float* v_out) {
  int rc = ref_dequantize_stored(L, k_codes, k_meta, v_codes, v_meta, t0, t1, k_out, v_out);
  if (rc) return rc;
  int D = L->head_dim;
  int64_t rows = (int64_t)L->batch * L->kv_heads * (t1 - t0);
  float* tmp = (float*)malloc(sizeof(float) * (size_t)D);
  for (int which = 0; which < 2; ++which) {
    float* out = which ? v_out : k_out;
    if (!out || !(which ? L->rotate_v : L->rotate_k)) continue;
    for (int64_t r = 0; r < rows; ++r) {
      ref_unrotate(out + r * D, D, which ? L->signs_v : L->signs_k, tmp);
      memcpy(out + r * D, tmp, sizeof(float) * (size_t)D);
    }
  }
  free(tmp);
  return 0;
}

/* ------------------------------------------------------------------ attention */

/* Exact softmax attention of one query row per (b, h_q) over dense binary32 K, V:
 *   logit_t = softmax_scale * sum_d q_d K[t][d];  A = softmax(logit);  out = A V.
 * K, V: [B][H_kv][T][D] (T = seq_len rows used); q: [B][H_q][D] of dtype q_dtype;
 * query head h_q reads KV head h_q / (H_q/H_kv).  Two passes, binary64 sums. */
int ref_attention_dense(const float* K, const float* V, int32_t batch, int32_t kv_heads, int32_t q_heads,
                        int32_t seq_len, int32_t D, const void* q, int q_dtype, float softmax_scale, float* out) {
  if (seq_len <= 0 || q_heads % kv_heads) return -1;
  int R = q_heads / kv_heads;
  /* every (b, h_q) output row is independent: one thread each, with its own logits and sums */
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t bq = 0; bq < (int64_t)batch * q_heads; ++bq) {
    {
      int b = (int)(bq / q_heads), hq = (int)(bq % q_heads);
      double* logit = (double*)malloc(sizeof(double) * (size_t)seq_len);
      double* acc = (double*)malloc(sizeof(double) * (size_t)D);
      int hk = hq / R;
      const float* Kh = K + ((int64_t)b * kv_heads + hk) * seq_len * D;
      const float* Vh = V + ((int64_t)b * kv_heads + hk) * seq_len * D;
      int64_t qbase = ((int64_t)b * q_heads + hq) * D;
      double mx = -INFINITY;
      for (int t = 0; t < seq_len; ++t) {
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += (double)load_elem(q, q_dtype, qbase + d) * (double)Kh[(int64_t)t * D + d];
        logit[t] = (double)softmax_scale * s;
        if (logit[t] > mx) mx = logit[t];
      }
      double denom = 0.0;
      for (int d = 0; d < D; ++d) acc[d] = 0.0;
      for (int t = 0; t < seq_len; ++t) {
        double p = exp(logit[t] - mx);
        denom += p;
        for (int d = 0; d < D; ++d) acc[d] += p * (double)Vh[(int64_t)t * D + d];
      }
      for (int d = 0; d < D; ++d) out[qbase + d] = (float)(acc[d] / denom);
      free(logit); free(acc);
    }
  }
  return 0;
}

/* Decode attention over the packed cache = reconstruct tokens [0, seq_len) as stored, then the
 * dense definition above (with rotate_k: of the rotated query against the rotated keys, which is
 * the same bilinear form because R is orthogonal; rotated values are reconstructed in the input
 * basis first, so the output is in the input basis too).  out: [B][H_q][D] binary32. */
int ref_decode_attention(const ref_layout* L, const uint8_t* k_codes, const uint8_t* k_meta, const uint8_t* v_codes,
                         const uint8_t* v_meta, const void* q, int q_dtype, int32_t q_heads, int32_t seq_len,
                         float softmax_scale, float* out) {
  if (seq_len <= 0 || seq_len > L->max_seq) return -1;
  int64_t n = (int64_t)L->batch * L->kv_heads * seq_len * L->head_dim;
  float* Kd = (float*)malloc(sizeof(float) * (size_t)n);
  float* Vd = (float*)malloc(sizeof(float) * (size_t)n);
  if (!Kd || !Vd) { free(Kd); free(Vd); return -2; }
  /* keys as stored (rotated keys meet the rotated query); values in the input basis (R_v^T of the stored rows) */
  int rc = ref_dequantize_stored(L, k_codes, k_meta, v_codes, v_meta, 0, seq_len, Kd, NULL);
  if (!rc) rc = ref_dequantize(L, k_codes, k_meta, v_codes, v_meta, 0, seq_len, NULL, Vd);
  if (!rc && L->rotate_k) {
    /* scores against rotated keys need the rotated query: q' = binary16(R q), row by row */
    int D = L->head_dim;
    int64_t nq = (int64_t)L->batch * q_heads;
    float* qr = (float*)malloc(sizeof(float) * (size_t)(nq * D));
    float* tmp = (float*)malloc(sizeof(float) * (size_t)D);
    for (int64_t r = 0; r < nq; ++r) {
      for (int d = 0; d < D; ++d) tmp[d] = load_elem(q, q_dtype, r * D + d);
      ref_rotate(tmp, D, L->signs_k, qr + r * D);
      for (int d = 0; d < D; ++d) qr[r * D + d] = ref_f16_to_f32(ref_f32_to_f16(qr[r * D + d]));
    }
    rc = ref_attention_dense(Kd, Vd, L->batch, L->kv_heads, q_heads, seq_len, D, qr, REF_F32, softmax_scale, out);
    free(qr); free(tmp);
  } else if (!rc) {
    rc = ref_attention_dense(Kd, Vd, L->batch, L->kv_heads, q_heads, seq_len, L->head_dim, q, q_dtype, softmax_scale, out);
  }
  free(Kd); free(Vd);
  return rc;
}

/* ------------------------------------------------------------------ channel-wise keys + residual buffer */

/* bytes of k_resid and v_resid (axis_k == 1) */
int ref_resid_bytes(const ref_layout* L, uint64_t out[2]) {
  uint64_t n = (uint64_t)L->batch * L->kv_heads * resid_slots(L) * L->head_dim * 2;
  out[0] = n;
  out[1] = n;
  return 0;
}

static int seq_layout_ok(const ref_layout* L) {
  int G = L->group_k, D = L->head_dim;
  int RL = resid_slots(L);
  if ((L->axis_k != 0 && L->axis_k != 1) || L->rotate_v) return 0;
  if (RL != 32 && RL != 64 && RL != 128) return 0;
  if (L->axis_k == 1 ? (RL % G != 0) : (D % G != 0)) return 0;
  if (L->rotate_k && (D > 128 || (D & (D - 1)))) return 0;
  if (G != 32 && G != 64 && G != 128) return 0;
  if (D % 64 || D > 1024 || D % L->group_v) return 0;
  if (!bits_allowed(L->bits_k) || !bits_allowed(L->bits_v)) return 0;
  return 1;
}

/* 16-bit pattern of (slot, d) in the residual planes of one (b,h) stream */
static uint16_t resid_get_k(const uint8_t* rs, int slot, int d, int D) {
  const uint8_t* p = rs + ((int64_t)slot * D + d) * 2;
  return (uint16_t)(p[0] | (p[1] << 8));
}
static uint16_t resid_get_v(const uint8_t* rs, int slot, int d, int D) {
  return (uint16_t)v_get_code(rs, slot, d, D, 16);
}

/* Append tokens [pos, pos+n_new) to a cache with channel-wise keys: every token goes to its
 * residual slot; a token that completes a block of G = group_k tokens triggers the flush of
 * that block (keys channel by channel, values token by token).  pos must equal the number of
 * tokens appended so far.  in_dtype must be raw_dtype (the buffer keeps the input patterns). */
int ref_seq_append(const ref_layout* L, uint8_t* k_codes, uint8_t* k_meta, uint8_t* v_codes, uint8_t* v_meta,
                   uint8_t* k_resid, uint8_t* v_resid, const void* k_new, const void* v_new, int in_dtype,
                   int64_t stride_b, int64_t stride_h, int64_t stride_t, int32_t pos, int32_t n_new) {
  if (!seq_layout_ok(L)) return -1;
  if (in_dtype != L->raw_dtype) return -1;
  if (pos < 0 || n_new < 0 || (int64_t)pos + n_new > L->max_seq) return -3;
  int D = L->head_dim, G = L->group_k, GV = L->group_v, bk = L->bits_k, bv = L->bits_v, RL = resid_slots(L);
  uint64_t pb[4];
  ref_plane_bytes(L, pb);
  int64_t streams = (int64_t)L->batch * L->kv_heads;
  int64_t rstream = (int64_t)RL * D * 2;
  float* col = (float*)malloc(sizeof(float) * (size_t)(G > D ? G : D));
  uint8_t* codes = (uint8_t*)malloc((size_t)(G > D ? G : D));
  for (int64_t bh = 0; bh < streams; ++bh) {
    int64_t bi = bh / L->kv_heads, hi = bh % L->kv_heads;
    uint8_t* kc = k_codes + bh * (int64_t)(pb[0] / (uint64_t)streams);
    uint8_t* km = k_meta + bh * (int64_t)(pb[1] / (uint64_t)streams);
    uint8_t* vc = v_codes + bh * (int64_t)(pb[2] / (uint64_t)streams);
    uint8_t* vm = v_meta + bh * (int64_t)(pb[3] / (uint64_t)streams);
    uint8_t* kr = k_resid + bh * rstream;
    uint8_t* vr = v_resid + bh * rstream;
    for (int64_t tn = 0; tn < n_new; ++tn) {
      int64_t t = pos + tn;
      int slot = (int)(t % RL);
      int64_t base = bi * stride_b + hi * stride_h + tn * stride_t;
      for (int d = 0; d < D; ++d) {                           /* the newest token stays in full precision */
        uint32_t kb = ((const uint16_t*)k_new)[base + d], vb = ((const uint16_t*)v_new)[base + d];
        put_bits_le(kr, ((int64_t)slot * D + d) * 16, 16, kb);
        v_put_code(vr, slot, d, D, 16, vb);
      }
      if (slot != RL - 1) continue;
      /* flush the RL tokens that fill the buffer */
      int64_t t0 = t + 1 - RL;
      float* rows = (float*)malloc(sizeof(float) * (size_t)RL * (size_t)D);  /* the buffer's key rows (R k with rotate_k) */
      float* plain = (float*)malloc(sizeof(float) * (size_t)D);
      for (int i = 0; i < RL; ++i) {
        for (int d = 0; d < D; ++d) {
          uint16_t bits16 = resid_get_k(kr, i, d, D);
          plain[d] = L->raw_dtype == REF_BF16 ? ref_bf16_to_f32(bits16) : ref_f16_to_f32(bits16);
        }
        if (L->rotate_k) ref_rotate(plain, D, L->signs_k, rows + (size_t)i * D);
        else memcpy(rows + (size_t)i * D, plain, sizeof(float) * (size_t)D);
      }
      if (L->axis_k == 1) {
        for (int sub = 0; sub < RL / G; ++sub)                /* keys: one group = G tokens of channel d */
          for (int d = 0; d < D; ++d) {
            for (int i = 0; i < G; ++i) col[i] = rows[(size_t)(sub * G + i) * D + d];
            uint16_t S, Z;
            ref_quantize_group(col, G, bk, codes, &S, &Z);
            uint8_t* m = km + (((t0 + sub * G) / G) * D + d) * 4;
            m[0] = (uint8_t)(S & 0xFF); m[1] = (uint8_t)(S >> 8);
            m[2] = (uint8_t)(Z & 0xFF); m[3] = (uint8_t)(Z >> 8);
            for (int i = 0; i < G; ++i) k_put_code(kc, t0 + sub * G + i, d, D, bk, codes[i]);
          }
      } else {
        for (int i = 0; i < RL; ++i) {                        /* keys token-wise: groups of G channels of one row */
          for (int g = 0; g < D / G; ++g) {
            uint16_t S, Z;
            ref_quantize_group(rows + (size_t)i * D + g * G, G, bk, codes + g * G, &S, &Z);
            uint8_t* m = km + meta_offset(t0 + i, g, D / G);
            m[0] = (uint8_t)(S & 0xFF); m[1] = (uint8_t)(S >> 8);
            m[2] = (uint8_t)(Z & 0xFF); m[3] = (uint8_t)(Z >> 8);
          }
          for (int d = 0; d < D; ++d) k_put_code(kc, t0 + i, d, D, bk, codes[d]);
        }
      }
      free(rows); free(plain);
      for (int i = 0; i < RL; ++i) {                          /* values: token-wise groups as always */
        for (int d = 0; d < D; ++d) {
          uint16_t bits16 = resid_get_v(vr, i, d, D);
          col[d] = L->raw_dtype == REF_BF16 ? ref_bf16_to_f32(bits16) : ref_f16_to_f32(bits16);
        }
        for (int g = 0; g < D / GV; ++g) {
          uint16_t S, Z;
          ref_quantize_group(col + g * GV, GV, bv, codes + g * GV, &S, &Z);
          uint8_t* m = vm + meta_offset(t0 + i, g, D / GV);
          m[0] = (uint8_t)(S & 0xFF); m[1] = (uint8_t)(S >> 8);
          m[2] = (uint8_t)(Z & 0xFF); m[3] = (uint8_t)(Z >> 8);
        }
        for (int d = 0; d < D; ++d) v_put_code(vc, t0 + i, d, D, bv, codes[d]);
      }
    }
  }
  free(col); free(codes);
  return 0;
}

/* What attention sees of tokens [t0,t1) when the cache holds seq_len tokens: the reconstruction
 * of the flushed tokens (below floor(seq_len/G)*G), the 16-bit patterns of the rest, as binary32.
 * k_out, v_out: [B][H][t1-t0][D]. */
static int seq_dequantize_impl(const ref_layout* L, const uint8_t* k_codes, const uint8_t* k_meta, const uint8_t* v_codes,
                               const uint8_t* v_meta, const uint8_t* k_resid, const uint8_t* v_resid, int32_t seq_len,
                               int32_t t0, int32_t t1, float* k_out, float* v_out, int stored) {
  if (!seq_layout_ok(L)) return -1;
  if (t0 < 0 || t1 < t0 || t1 > seq_len || seq_len > L->max_seq) return -3;
  int D = L->head_dim, G = L->group_k, GV = L->group_v, bk = L->bits_k, bv = L->bits_v, RL = resid_slots(L);
  uint64_t pb[4];
  ref_plane_bytes(L, pb);
  int64_t streams = (int64_t)L->batch * L->kv_heads;
  int64_t rstream = (int64_t)RL * D * 2;
  int64_t n_flushed = (int64_t)seq_len / RL * RL;
  int64_t nt = t1 - t0;
  for (int64_t bh = 0; bh < streams; ++bh) {
    const uint8_t* kc = k_codes + bh * (int64_t)(pb[0] / (uint64_t)streams);
    const uint8_t* km = k_meta + bh * (int64_t)(pb[1] / (uint64_t)streams);
    const uint8_t* vc = v_codes + bh * (int64_t)(pb[2] / (uint64_t)streams);
    const uint8_t* vm = v_meta + bh * (int64_t)(pb[3] / (uint64_t)streams);
    const uint8_t* kr = k_resid + bh * rstream;
    const uint8_t* vr = v_resid + bh * rstream;
    for (int64_t t = t0; t < t1; ++t)
      for (int d = 0; d < D; ++d) {
        float kv, vv;
        if (t < n_flushed) {
          const uint8_t* m = L->axis_k == 1 ? km + ((t / G) * D + d) * 4 : km + meta_offset(t, d / G, D / G);
          kv = ref_reconstruct(k_get_code(kc, t, d, D, bk), (uint16_t)(m[0] | (m[1] << 8)), (uint16_t)(m[2] | (m[3] << 8)));
          const uint8_t* mv = vm + meta_offset(t, d / GV, D / GV);
          vv = ref_reconstruct(v_get_code(vc, t, d, D, bv), (uint16_t)(mv[0] | (mv[1] << 8)), (uint16_t)(mv[2] | (mv[3] << 8)));
        } else {
          uint16_t kb = resid_get_k(kr, (int)(t % RL), d, D), vb = resid_get_v(vr, (int)(t % RL), d, D);
          kv = L->raw_dtype == REF_BF16 ? ref_bf16_to_f32(kb) : ref_f16_to_f32(kb);
          vv = L->raw_dtype == REF_BF16 ? ref_bf16_to_f32(vb) : ref_f16_to_f32(vb);
        }
        if (k_out) k_out[((bh * nt) + (t - t0)) * D + d] = kv;
        if (v_out) v_out[((bh * nt) + (t - t0)) * D + d] = vv;
      }
    if (k_out && L->rotate_k && !stored) {                  /* flushed rows hold reconstructions of R k: back with R^T */
      float* tmp = (float*)malloc(sizeof(float) * (size_t)D);
      for (int64_t t = t0; t < t1 && t < n_flushed; ++t) {
        float* row = k_out + ((bh * nt) + (t - t0)) * D;
        ref_unrotate(row, D, L->signs_k, tmp);
        memcpy(row, tmp, sizeof(float) * (size_t)D);
      }
      free(tmp);
    }
  }
  return 0;
}

/* ... in the basis of the inputs (with rotate_k the flushed key rows are taken back with R^T) */
int ref_seq_dequantize(const ref_layout* L, const uint8_t* k_codes, const uint8_t* k_meta, const uint8_t* v_codes,
                       const uint8_t* v_meta, const uint8_t* k_resid, const uint8_t* v_resid, int32_t seq_len,
                       int32_t t0, int32_t t1, float* k_out, float* v_out) {
  return seq_dequantize_impl(L, k_codes, k_meta, v_codes, v_meta, k_resid, v_resid, seq_len, t0, t1, k_out, v_out, 0);
}

/* Decode attention over a cache with channel-wise keys and a residual buffer: the dense
 * definition on what ref_seq_dequantize returns for tokens [0, seq_len). */
int ref_seq_decode_attention(const ref_layout* L, const uint8_t* k_codes, const uint8_t* k_meta, const uint8_t* v_codes,
                             const uint8_t* v_meta, const uint8_t* k_resid, const uint8_t* v_resid, const void* q,
                             int q_dtype, int32_t q_heads, int32_t seq_len, float softmax_scale, float* out) {
  if (seq_len <= 0 || seq_len > L->max_seq) return -1;
  int64_t n = (int64_t)L->batch * L->kv_heads * seq_len * L->head_dim;
  float* Kd = (float*)malloc(sizeof(float) * (size_t)n);
  float* Vd = (float*)malloc(sizeof(float) * (size_t)n);
  if (!Kd || !Vd) { free(Kd); free(Vd); return -2; }
  /* keys as stored: flushed rows in the rotated basis when rotate_k, the tail as it came in */
  int rc = seq_dequantize_impl(L, k_codes, k_meta, v_codes, v_meta, k_resid, v_resid, seq_len, 0, seq_len, Kd, Vd, 1);
  if (!rc && !L->rotate_k)
    rc = ref_attention_dense(Kd, Vd, L->batch, L->kv_heads, q_heads, seq_len, L->head_dim, q, q_dtype, softmax_scale, out);
  else if (!rc) {
    /* the dense definition with the query that belongs to each token's basis: binary16(R q) for the flushed tokens,
     * q for the tail */
    int D = L->head_dim, R = q_heads / L->kv_heads;
    int64_t n_flushed = (int64_t)seq_len / resid_slots(L) * resid_slots(L);
    float* qp = (float*)malloc(sizeof(float) * (size_t)D);
    float* qr = (float*)malloc(sizeof(float) * (size_t)D);
    double* logit = (double*)malloc(sizeof(double) * (size_t)seq_len);
    double* acc = (double*)malloc(sizeof(double) * (size_t)D);
    for (int b = 0; b < L->batch; ++b)
      for (int hq = 0; hq < q_heads; ++hq) {
        int hk = hq / R;
        const float* Kh = Kd + ((int64_t)b * L->kv_heads + hk) * seq_len * D;
        const float* Vh = Vd + ((int64_t)b * L->kv_heads + hk) * seq_len * D;
        int64_t qbase = ((int64_t)b * q_heads + hq) * D;
        for (int d = 0; d < D; ++d) qp[d] = load_elem(q, q_dtype, qbase + d);
        ref_rotate(qp, D, L->signs_k, qr);
        for (int d = 0; d < D; ++d) qr[d] = ref_f16_to_f32(ref_f32_to_f16(qr[d]));
        double mx = -INFINITY;
        for (int t = 0; t < seq_len; ++t) {
          const float* qt = t < n_flushed ? qr : qp;
          double sdot = 0.0;
          for (int d = 0; d < D; ++d) sdot += (double)qt[d] * (double)Kh[(int64_t)t * D + d];
          logit[t] = (double)softmax_scale * sdot;
          if (logit[t] > mx) mx = logit[t];
        }
        double denom = 0.0;
        for (int d = 0; d < D; ++d) acc[d] = 0.0;
        for (int t = 0; t < seq_len; ++t) {
          double pw = exp(logit[t] - mx);
          denom += pw;
          for (int d = 0; d < D; ++d) acc[d] += pw * (double)Vh[(int64_t)t * D + d];
        }
        for (int d = 0; d < D; ++d) out[qbase + d] = (float)(acc[d] / denom);
      }
    free(qp); free(qr); free(logit); free(acc);
  }
  free(Kd); free(Vd);
  return rc;
}

/* ------------------------------------------------------------------ error metric */

/* MSE(A, A^) = ||A - A^||_F^2 / (number of entries)   (App. B, Frobenius / MSE perspective) */
double ref_mse(const float* a, const float* ahat, int64_t n) {
  double s = 0.0;
  for (int64_t i = 0; i < n; ++i) { double e = (double)a[i] - (double)ahat[i]; s += e * e; }
  return s / (double)n;
}
