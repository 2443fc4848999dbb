// Decode attention over the packed cache (gfx950): out = softmax(scale * q K^^T) V^  (App. A of
// arXiv 2502.15075) with K^, V^ the group-wise reconstructions code*scale+zero (App. B), computed
// without ever materializing K^ or V^:
//
//   logit[t,h]  = sum_g  sK[t,g] * (sum_{d in g} q[h,d] cK[t,d])  +  zK[t,g] * (sum_{d in g} q[h,d])
//   out[h,d]    = ( sum_t (p[t,h] sV[t,g(d)]) cV[t,d]  +  sum_t p[t,h] zV[t,g(d)] ) / sum_t p[t,h]
//
// Both inner sums over codes are 16x16x32 f16 matrix instructions.  A b-bit code c placed in the
// low mantissa bits of a binary16 lane is the subnormal c * 2^-24 (or c * 2^(k-24) when left at bit
// k): the products with the query are exact and the sum is taken in a window of about 24 bits (see
// the note at k_slot_elem), so "unpacking" is one AND per two codes; the power-of-two position
// factors are divided out of the query operand once per wavefront.
//
// Work split: one workgroup (4 or 8 wavefronts) walks a contiguous range of 32-token steps of one
// (batch, kv head); its wavefronts interleave the steps and each carries all query heads of that kv
// head as matrix columns (column c = g*R + h: key group g, head h), so every cache byte is read
// once.  Each wavefront keeps a ring of steps in registers: after a step is computed its registers
// are refilled with the step one ring length ahead, so several steps of streaming loads are always
// in flight per wavefront.  Wavefronts merge through LDS, workgroups through a workspace of
// (max, sum, acc) records and a small second kernel.
//
// Variants of the same kernel (template parameters): unquantized rows as operands (bits = 16), key
// codes of 3 and 6 bits as a low and a high run with a query operand each, two column sets (8 heads
// with 32-channel groups), channel-wise key groups (Sec. 4 "Downstream Task
// Accuracy": the scale moves into a per-block query operand), paged planes (a page-table lookup per
// step), per-sequence lengths, the fused append of a decode step, Hadamard-rotated keys and values
// (Sec. 4 "Integration with Rotation-Based Methods").
#include "kvq_internal.h"
#include "kvq_quantizer.h"

#include <atomic>
#include <type_traits>

namespace kvq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// D += A(16x32) * B(32x16); operands travel as 4 dwords (8 x 16-bit), binary16 or bfloat16.
template <bool BF>
__device__ __forceinline__ float4v mma(u32x4 a, u32x4 b, float4v c) {
  if constexpr (BF) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

constexpr float kCodeUnit = 5.9604644775390625e-08f;  // 2^-24: value of a code's lowest mantissa bit
constexpr float kInvCodeUnit = 16777216.0f;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;


template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
// Sum over the 16/R lanes of a 16-lane row that share x's query head (lanes c, c+R, c+2R, ...).
template <int R>
__device__ __forceinline__ float sum_over_groups(float x) {
  if (R <= 8) x += dpp_f32<0x128>(x);   // row_ror:8
  if (R <= 4) x += dpp_f32<0x124>(x);   // row_ror:4
  if (R <= 2) x += dpp_f32<0x122>(x);   // row_ror:2
  if (R <= 1) x += dpp_f32<0x121>(x);   // row_ror:1
  return x;
}

// ---- key codes: one lane holds 32 consecutive channels of one token (BK dwords) -------------
// Matrix step m (0..3) consumes 8 of them; slot i of that step is channel k_slot_elem(m,i) of the
// lane's 32, left at bit k of its 16-bit lane, i.e. read as code * 2^k * 2^-24, so the query operand of the slot is
// divided by k_slot_scale(i) = 2^k.
//
// Where the fields are left matters for accuracy.  A binary16 subnormal enters the matrix unit with the exponent
// 2^-14 whatever its leading zeros, and the unit keeps about 24 bits below the largest product exponent of a dot
// product: a code at bit 0 against an undivided query element loses everything below 2^-38 times that element (measured:
// up to 3e-4 code units per 32-term dot product, which the scale of a coarse key format on outlier-heavy keys turns
// into several 1e-3 of a logit), a code at bit k against the element divided by 2^k keeps 2^k times more.  The query
// operand in turn must stay a normal binary16 number, so k stays at or below 6.  Hence: 2-bit fields are moved to bits
// 4 and 6 (one more shift per matrix step), single bits to BASE..BASE+3; 4-bit fields stay at bits 0 and 4 and 8-bit
// fields at bit 0 (their scales are small and the error stays at the level of the value side's weight rounding; moving
// the 4-bit fields as well was measured: the same maximum error, 2.8 % more time for the headline format).
// BASE: lowest bit of the moved 1- and 2-bit fields (the high run of 3- and 6-bit codes is moved higher, its query
// operand carries the factor 2^LO and is still normal).
template <int BK> __device__ __forceinline__ constexpr int k_slot_elem(int m, int i) {
  const int v = i >> 1, x = i & 1;
  if (BK == 16) return 8 * m + i;
  if (BK == 1) return 4 * m + v + 16 * x;
  if (BK == 4) return 8 * m + v + 4 * x;
  if (BK == 8) return 8 * m + 4 * (v >> 1) + (v & 1) + 2 * x;
  return 16 * (m >> 1) + 4 * (m & 1) + v + 8 * x;  // BK == 2
}
template <int BK> constexpr int k_default_base() { return BK == 2 ? 4 : BK == 1 ? 3 : 0; }
template <int BK, int BASE = k_default_base<BK>()> __device__ __forceinline__ constexpr float k_slot_scale(int i) {
  const int v = i >> 1;
  if (BK == 4) return (v & 1) ? 16.0f : 1.0f;
  if (BK == 8 || BK == 16) return 1.0f;
  if (BK == 1) return (float)(1 << (BASE + v));
  return (float)(1 << (BASE + 2 * (v & 1)));       // BK == 2
}
// The same factor as a function of the channel (the slot a channel lands in fixes it), default BASE.
template <int BK> __device__ __forceinline__ constexpr float k_chan_scale(int d) {
  return BK == 4 ? ((d & 1) ? 16.0f : 1.0f) : BK == 2 ? ((d & 1) ? 64.0f : 16.0f) : 1.0f;
}
template <int BK> constexpr bool k_chan_scale_matches() {
  for (int m = 0; m < 4; ++m)
    for (int i = 0; i < 8; ++i)
      if (k_chan_scale<BK>(k_slot_elem<BK>(m, i)) != k_slot_scale<BK>(i)) return false;
  return true;
}
static_assert(k_chan_scale_matches<2>() && k_chan_scale_matches<4>() && k_chan_scale_matches<8>(), "slot factors");
// (shift left by s, right for negative s; s is a compile-time value after unrolling)
__device__ __forceinline__ uint32_t shl_signed(uint32_t w, int s) { return s >= 0 ? w << s : w >> (-s); }
template <int BK, int BASE = k_default_base<BK>()> __device__ __forceinline__ u32x4 unpack_k(const uint32_t* w, int m) {
  u32x4 a;
  if constexpr (BK == 16) {
    a = u32x4{w[4 * m], w[4 * m + 1], w[4 * m + 2], w[4 * m + 3]};      // unquantized: the 16-bit patterns themselves
  } else if constexpr (BK == 4) {
    const uint32_t lo = w[m], hi = w[m] >> 8;
    a = u32x4{lo & 0x000F000Fu, lo & 0x00F000F0u, hi & 0x000F000Fu, hi & 0x00F000F0u};
  } else if constexpr (BK == 8) {
    const uint32_t w0 = w[2 * m], w1 = w[2 * m + 1];
    a = u32x4{w0 & 0x00FF00FFu, (w0 >> 8) & 0x00FF00FFu, w1 & 0x00FF00FFu, (w1 >> 8) & 0x00FF00FFu};
  } else if constexpr (BK == 1) {
    // bit 4m+v of each half (channels 4m+v and 16+4m+v) to bit BASE+v.  What a shift carries across the middle of the
    // word lands outside the masks: left shifts reach bit 16+BASE-1 at most, right shifts bit 16-(4m-BASE) at least.
    static_assert(BASE >= 0 && BASE <= 7, "single-bit fields stay below bit 11");
    const uint32_t ws = shl_signed(w[0], BASE - 4 * m);
    constexpr uint32_t k1 = 0x00010001u << BASE;
    a = u32x4{ws & k1, ws & (k1 << 1), ws & (k1 << 2), ws & (k1 << 3)};
  } else {
    // fields 0,1 of the byte (bits 0-3) and fields 2,3 (bits 4-7) both to bits BASE..BASE+3 (same remark on carries)
    static_assert(BASE >= 4 && BASE <= 7, "two-bit fields stay below bit 11");
    const int byte0 = 8 * (m & 1);
    const uint32_t wl = shl_signed(w[m >> 1], BASE - byte0), wh = shl_signed(w[m >> 1], BASE - 4 - byte0);
    constexpr uint32_t k2 = 0x00030003u << BASE;
    a = u32x4{wl & k2, wl & (k2 << 2), wh & k2, wh & (k2 << 2)};
  }
  return a;
}
// Key codes of 3 and 6 bits are a low run (2 / 4 bits, the first dwords of the lane's 32 channels) and a high run
// (1 / 2 bits, the rest): two operands, multiplied by the query separately (the high run's query operand carries the
// factor 2^LO).
template <int BK> constexpr int k_lo() { return code_lo_bits<BK>(); }
template <int BK> constexpr int k_hi() { return code_hi_bits<BK>(); }
template <int BK> constexpr int k_hi_base() { return BK == 3 ? 5 : 6; }   // high run: single bits from bit 5, pairs from bit 6

// ---- value codes: one lane holds, per 32-token step, 2*BV dwords (index = 4*piece + dword; 1-bit codes: one piece
// of two dwords, d-tile dt's 8 codes in nibble dt%4 of each half of dword dt/4) ----
// Register v (0..3) of d-tile dt's operand holds slots 2v, 2v+1 and is left at bit offset v_slot_shift(v)
// of its 16-bit lane, i.e. it reads as code * 2^shift * 2^-24; the softmax weight of those slots is
// divided by 2^shift instead (an exponent offset, free).
// Value codes of 3 and 6 bits are a block of low parts (2 / 4 bits) and a block of high parts (1 / 2 bits): two
// operands per d-tile; v_slot_shift is the low part's, and the high part's weights carry the factor v_hi_factor.
template <int BV> constexpr int v_lo() { return code_lo_bits<BV>(); }
template <int BV> constexpr int v_hi() { return code_hi_bits<BV>(); }
template <int B> __device__ __forceinline__ constexpr int field_slot_shift(int v) {
  return B == 1 ? v : B == 2 ? 2 * v : (B == 4 ? 4 * (v & 1) : 0);
}
template <int BV> __device__ __forceinline__ constexpr int v_slot_shift(int v) { return field_slot_shift<v_lo<BV>()>(v); }
// code = lo + 2^LO hi, and the two operands sit at different bit offsets of their 16-bit lanes
template <int BV> __device__ __forceinline__ constexpr float v_hi_factor(int v) {
  return (float)(1 << (v_lo<BV>() + field_slot_shift<v_lo<BV>()>(v))) / (float)(1 << field_slot_shift<(v_hi<BV>() ? v_hi<BV>() : 1)>(v));
}
// Softmax weights are carried times 2^p_shift and divided by 2^shift of their slot: the largest of them is 2^10 (binary16
// headroom for weight x value scale up to 64), so p_shift is 10 plus the smallest slot shift, where the high part's
// slots count with their shift minus LO (their weights carry 2^LO).  The scale of a 1-bit group is its whole range:
// two bits more headroom (scale up to 255).  Larger scales: see weight_headroom.
template <int BV> constexpr float p_shift() {
  int m = field_slot_shift<v_lo<BV>()>(0);
  if (v_hi<BV>()) {
    const int h = field_slot_shift<(v_hi<BV>() ? v_hi<BV>() : 1)>(0) - v_lo<BV>();
    m = h < m ? h : m;
  }
  return (float)(10 + m - (BV == 1 ? 2 : 0));
}
template <int BV> __device__ __forceinline__ u32x4 unpack_v(const uint32_t* w, int dt) {
  u32x4 a;
  if (BV == 16) {
    a = u32x4{w[4 * dt], w[4 * dt + 1], w[4 * dt + 2], w[4 * dt + 3]};
  } else if (BV == 1) {
    const uint32_t ws = w[dt >> 2] >> (4 * (dt & 3));
    a = u32x4{ws & 0x00010001u, ws & 0x00020002u, ws & 0x00040004u, ws & 0x00080008u};
  } else if (BV == 2) {
    const uint32_t ws = w[dt >> 1] >> (8 * (dt & 1));
    a = u32x4{ws & 0x00030003u, ws & 0x000C000Cu, ws & 0x00300030u, ws & 0x00C000C0u};
  } else if (BV == 4) {
    const uint32_t lo = w[dt], hi = lo >> 8;
    a = u32x4{lo & 0x000F000Fu, lo & 0x00F000F0u, hi & 0x000F000Fu, hi & 0x00F000F0u};
  } else {
    const uint32_t w0 = w[2 * dt], w1 = w[2 * dt + 1];
    a = u32x4{w0 & 0x00FF00FFu, (w0 >> 8) & 0x00FF00FFu, w1 & 0x00FF00FFu, (w1 >> 8) & 0x00FF00FFu};
  }
  return a;
}

#ifndef KVQ_STAGES
#define KVQ_STAGES 4           // 32-token steps resident or in flight per wavefront (register ring)
#endif
#ifndef KVQ_WAVES_PER_SIMD
#define KVQ_WAVES_PER_SIMD 2   // occupancy the register allocation is held to
#endif

// Ring depth per instantiation: a step costs 2 b_K + 2 b_V + 4 registers per lane (and the scheduler wants room to
// start a refill before the old contents are dead); deeper rings for the narrow formats, two steps for the wide ones.
template <int BK, int BV, int NCK = 1, int NCV = 1, bool ROTV = false>
constexpr int ring_stages() {
  constexpr int regs = 2 * BK + 2 * BV + 4;
  constexpr int base = regs <= 16 ? KVQ_STAGES : regs <= 20 ? 3 : 2;
  constexpr int less = (NCK == 2 ? 2 : 0) + (NCV == 2 ? 1 : 0)    // a second column set costs registers (query operand,
                       + (code_hi_bits<BK>() ? 1 : 0)              // scale/zero entries, weights), so does a high run
                       + (code_hi_bits<BV>() ? 1 : 0)              // of keys or a high part of values (its weights)
                       + (ROTV ? 1 : 0)                            // (rotated values: the unrounded weights stay live)
                       + (BK == 2 && regs >= 16 ? 1 : 0);         // (moved 2-bit fields: two shifted copies of a word live)
  return base - less >= 1 ? base - less : 1;
}

// Everything one lane loads for one 32-token step (two 16-token tiles).
template <int BK, int BV>
struct StepRegs {
  uint32_t kc[2][BK];            // tile x4: row 16*x4 + c, this lane's 32 channels
  uint32_t vc[2 * BV];           // value codes: piece k, dword m at [4k + m]
  u32x4 meta;                    // 16 bytes of the step's scale/zero bytes, in plane order (lane l < 8 (ng_k + ng_v) holds
                                 // bytes 16 l ..); redistributed through LDS when the step is computed
};

struct LaneCtx {
  const uint8_t* kc; const uint8_t* vc;   // (b,h) stream bases of the code planes (wave-uniform)
  const uint8_t* meta_base;               // this lane's scale/zero plane: key plane for lanes < 8 ng_k, else value plane
  uint32_t meta_mul, meta_off;            // bytes of that plane per 32-token step; this lane's offset inside them
  uint32_t meta_step_mask;                // ~1 for the key lanes of channel-wise keys (one entry set per two steps)
  uint32_t kc_off, vc_off;                // this lane's byte offsets inside one step of the code planes
  uint32_t km_rd, vm_rd;                  // byte offsets of this lane's key / value scale-zero entries (tile 0) in the
                                          // wavefront's LDS copy of a step's scale/zero bytes
  uint8_t* meta_lds;                      // that LDS copy (1 KB per wavefront)
  int lane, c, j, gk, gv, ngk, ngv;
  static constexpr bool kRotV = false;
};
// Kernels for caches whose values are stored rotated (the output goes through R_v^T) mark their context so.
struct LaneCtxRotV : LaneCtx { static constexpr bool kRotV = true; };

// Cache bytes are read exactly once per decode step: streaming (non-temporal) loads.
__device__ __forceinline__ u32x4 ld16(const uint8_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// WIDE (paged planes): `step` counts 32-token steps in plane order from the plane base, so the uniform part of the
// address is formed in 64 bits; otherwise it counts inside the (b,h) stream that the bases point to.
// N consecutive dwords of a key tile (4 N bytes per lane: the lane's 32 channels), non-temporal; the address is a
// multiple of 4 N bytes only when N is a power of two (3- and 6-bit rows), so the vector types carry that alignment.
template <int N> __device__ __forceinline__ void load_dwords(uint32_t* dst, const uint8_t* p) {
  typedef uint32_t v2 __attribute__((ext_vector_type(2), aligned(8)));
  typedef uint32_t v3 __attribute__((ext_vector_type(3), aligned(4)));
  typedef uint32_t v4a8 __attribute__((ext_vector_type(4), aligned(8)));
  if constexpr (N == 1) {
    dst[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
  } else if constexpr (N == 2) {
    const v2 v = __builtin_nontemporal_load(reinterpret_cast<const v2*>(p));
    dst[0] = v.x; dst[1] = v.y;
  } else if constexpr (N == 3) {
    const v3 v = __builtin_nontemporal_load(reinterpret_cast<const v3*>(p));
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z;
  } else if constexpr (N == 6) {
    const v4a8 v = __builtin_nontemporal_load(reinterpret_cast<const v4a8*>(p));
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    load_dwords<2>(dst + 4, p + 16);
  } else {
    static_assert(N % 4 == 0, "key tile piece");
#pragma unroll
    for (int k = 0; k < N / 4; ++k) {
      const u32x4 v = ld16(p + 16 * k);
      dst[4 * k + 0] = v.x; dst[4 * k + 1] = v.y; dst[4 * k + 2] = v.z; dst[4 * k + 3] = v.w;
    }
  }
}

// lane_mask: ~0, or 0 for a refill past the wavefront's last step, which still issues its loads (every lane then reads
// the first 16 bytes of each part of the step it is given: one cache line per load, the data is never used).  A load
// that may or may not be issued sits behind a branch, and with a branch between the loads the compiler can no longer
// count how many newer loads follow a ring slot's: it then drains the ring before every use.
template <int BK, int BV, bool WIDE = false>
__device__ __forceinline__ void load_step(StepRegs<BK, BV>& r, const LaneCtx& L, int64_t step, uint32_t lane_mask = ~0u) {
  // uniform 64-bit base + 32-bit offset (a (b,h) stream of any plane is below 4 GiB)
  const uint8_t* kbase = WIDE ? L.kc + step * (512 * BK) : L.kc;
  const uint8_t* vbase = WIDE ? L.vc + step * (512 * BV) : L.vc;
  const uint8_t* mbase = WIDE ? L.meta_base + (step & (int64_t)(int32_t)L.meta_step_mask) * L.meta_mul : L.meta_base;
  const uint32_t ko = (WIDE ? 0u : (uint32_t)step * (512 * BK)) + (L.kc_off & lane_mask);
#pragma unroll
  for (int x4 = 0; x4 < 2; ++x4) load_dwords<BK>(r.kc[x4], kbase + (ko + x4 * (256 * BK)));
  // (every lane loads, for the same reason: lanes beyond the scale/zero bytes repeat the last 16 of them)
  if constexpr (BK != 16 || BV != 16)
    r.meta = ld16(mbase + ((WIDE ? 0u : ((uint32_t)step & L.meta_step_mask) * L.meta_mul) + (L.meta_off & lane_mask)));
  constexpr int VLO = v_lo<BV>(), VHI = v_hi<BV>();
  const uint32_t vstep = WIDE ? 0u : (uint32_t)step * (512 * BV);
  const uint32_t vo = vstep + (L.vc_off & lane_mask);
  if constexpr (BV == 1) load_dwords<2>(r.vc, vbase + vo);
#pragma unroll
  for (int k = 0; k < VLO / 2; ++k) {
    const u32x4 v = ld16(vbase + (vo + k * 1024));
    r.vc[4 * k + 0] = v.x; r.vc[4 * k + 1] = v.y; r.vc[4 * k + 2] = v.z; r.vc[4 * k + 3] = v.w;
  }
  // the block of high parts follows the block of low parts: 8 bytes per lane (single bits) or 16 (pairs)
  if constexpr (VHI == 1) load_dwords<2>(r.vc + 2 * VLO, vbase + (vstep + 512 * VLO + ((L.vc_off >> 1) & lane_mask)));
  if constexpr (VHI == 2) load_dwords<4>(r.vc + 2 * VLO, vbase + (vstep + 512 * VLO + (L.vc_off & lane_mask)));
}

__device__ __forceinline__ float meta_scale(uint32_t m) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(m & 0xFFFFu)); }
__device__ __forceinline__ float meta_zero(uint32_t m) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(m >> 16)); }

template <int NCV>
struct WaveState {
  float4v acc[8];       // out^T tile dt: rows d = 16*dt + 4*j + r, column c
  float m;              // running max of this lane's head, in log2 units
  float noff[4];        // p_shift - m - v_slot_shift(v): exponent offset of the slots in operand register v
  float l[4];           // per register class v: this lane's share of sum_t p * 2^(p_shift - shift(v))
  float zacc[NCV][4];   // same, weighted by zV[t, g] for this lane's value group of each column set
  float headroom;       // the running maximum is kept this far (in log2 units) above the largest logit seen, which holds
                        // every weight below 2^-headroom of its usual size (see weight_headroom); wave-uniform
};

// The softmax weights go into the matrix unit as binary16 products p * 2^p_shift * scale_V, and the largest of them
// (p = 1 at the running maximum) stays finite only for value scales below 2^(16 - p_shift) = 64 (256 for 1-bit values),
// i.e. for groups whose range is below 64 (2^b - 1) -- while inputs may be as large as binary16 goes.  The append
// kernels therefore keep, per (batch, kv head), the largest exponent field of any value scale they have stored
// (kvq_cache.v_scale_exp), and an attention launch over a stream that holds a scale of 64 or more holds ALL its
// weights down: the running maximum stays (that exponent - 5) above the logits, which divides every weight and every
// sum by that power of two (the final division by the sum of weights takes it out again).  What it costs is resolution
// of the smallest weights, which such a stream can spare: they multiply values of the same large scale.  Nothing of
// this is in the loop: the offset rides in the multiply-add that turns a logit into log2 units.
template <int BV> __device__ __forceinline__ float weight_headroom(int scale_exp_field) {
  const int need = scale_exp_field - 15 - (BV == 1 ? 7 : 5);   // scales below 2^6 (1-bit values: 2^8) need nothing
  return (float)(need < 0 ? 0 : need > 16 ? 16 : need);
}

// binary16 product of a binary32 weight and the binary16 held in the low half of `meta`, written to the
// low / high half of `dst` (one rounding: the compiler turns the fused multiply-add with a converted operand and the
// conversion of its result into one v_fma_mixlo/mixhi_f16).  Written in C and not as inline assembly on purpose: the
// weight comes straight from v_exp_f32, and the result of a transcendental instruction may not be read by the next
// vector instruction; the compiler keeps that distance for the instructions it emits itself, not for assembly text.
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void mix_lo(uint32_t& dst, float p, uint32_t meta) {
  const half2v r = {(_Float16)fmaf(p, meta_scale(meta), 0.0f), (_Float16)0.0f};
  dst = __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ void mix_hi(uint32_t& dst, float p, uint32_t meta) {
  half2v r = __builtin_bit_cast(half2v, dst);
  r.y = (_Float16)fmaf(p, meta_scale(meta), 0.0f);
  dst = __builtin_bit_cast(uint32_t, r);
}

// Round-to-nearest-even bfloat16 pattern of a finite binary32.
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ---- channel-wise keys (one scale/zero per channel and 64-token block) --------------------------------------------
// The scale of channel d cannot leave the contraction over d, so it is folded into the query: per block the operand
// q~[h,d] = q[h,d] * sK[blk,d] is rebuilt, as a high and a low binary16 part (the product of two 11-bit numbers has
// 22 bits; the low part carries the rest down to an absolute 2^-25, far below what the scores resolve).  The two parts
// are two matrix columns of the same head (column group 0 the high part, group 1 the low part: at most 8 heads fill
// 16 columns), so one matrix instruction multiplies the codes by both and the sum over column groups that the
// token-wise kernel uses for its key groups adds them.  The zero points enter as one constant per head and block,
// sum_d q[h,d] zK[blk,d].  logit[t,h] = sum_d q~[h,d] cK[t,d] + that constant.
struct KSeqState {
  u32x4 qop[4];            // query operand of the current block: this lane's part (high or low) of its head
  float zq_u;              // zero-point term of the current block, in code units (lanes of the high part; else 0)
};
struct KSeqState2 : KSeqState {
  u32x4 qoph[4];           // the same for the high run of 3- and 6-bit key codes (carries the factor 2^LO)
};
struct NoKSeq {};
// 2-, 4- and 8-bit keys: the staged query row is already divided by the position factor of each channel's code
// (k_chan_scale).  1-, 3- and 6-bit keys: the row is staged as it is and the factors of each run's slots are applied
// when the operands are built.
template <int BK> constexpr bool kseq_prescaled() { return BK == 2 || BK == 4 || BK == 8; }

// Rebuild the block's query operand from the staged query row and the block's 128 scale/zero entries (first 512 bytes
// of the wavefront's LDS copy of the step's scale/zero bytes).
// qrow: the head's query in binary32, channel d divided by k_chan_scale(d) (LDS; an all-zero row for a lane whose
// column carries nothing on the key side).  low_part: 1.0f in the lanes of the low part, 0.0f in those of the high part.
// The high part is the product rounded toward zero, h = rtz16(v); every lane forms v - low_part * h and converts
// again: v's own high part where low_part is 0, the exact rest where it is 1 — the same instructions in both.
template <int BK>
__device__ __forceinline__ void kseq_rebuild(KSeqState& ks, const LaneCtx& L, const float* qrow, float low_part) {
  constexpr int NC = BK == 8 ? 1 : 2;                        // classes of channels by k_chan_scale (even / odd)
  typedef __fp16 half2v __attribute__((ext_vector_type(2)));
  float zc[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) zc[c] = 0.f;
  const float nlow = -low_part;
#pragma unroll
  for (int half32 = 0; half32 < 2; ++half32) {     // 16 channels at a time: matrix steps 2*half32 and 2*half32 + 1
    float w[16];
#pragma unroll
    for (int quad = 0; quad < 4; ++quad) {
      const float4v qf = *reinterpret_cast<const float4v*>(qrow + 32 * L.j + 16 * half32 + 4 * quad);
      const u32x4 mv = *reinterpret_cast<const u32x4*>(L.meta_lds + 128 * L.j + 64 * half32 + 16 * quad);
      const uint32_t mw[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        w[4 * quad + e] = fmaf(qf[e], meta_scale(mw[e]), 0.0f);
        zc[e % NC] = fmaf(qf[e], meta_zero(mw[e]), zc[e % NC]);
      }
    }
#pragma unroll
    for (int mm = 0; mm < 2; ++mm) {
      const int m = 2 * half32 + mm;
      uint32_t op[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float a = w[k_slot_elem<BK>(m, 2 * v) - 16 * half32], b = w[k_slot_elem<BK>(m, 2 * v + 1) - 16 * half32];
        const half2v h = __builtin_amdgcn_cvt_pkrtz(a, b);
        const float xa = fmaf((float)h.x, nlow, a), xb = fmaf((float)h.y, nlow, b);
        op[v] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(xa, xb));
      }
      ks.qop[m] = u32x4{op[0], op[1], op[2], op[3]};
    }
  }
  float zq = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c) zq = fmaf(zc[c], k_chan_scale<BK>(c), zq);
  zq += __shfl_xor(zq, 16);
  zq += __shfl_xor(zq, 32);
  ks.zq_u = zq * (kCodeUnit - kCodeUnit * low_part);          // (only the high part's column adds the constant)
}

// The same for 1-, 3- and 6-bit keys: all 32 products q[d] sK[d] of the lane first (a single-bit run takes a matrix
// step's channels from both halves of the 32), then one operand set per run, each slot divided by the power of two at
// which the run's codes are left in their 16-bit lanes, the high run's times 2^LO.
template <int BK, typename KS>
__device__ __forceinline__ void kseq_rebuild_runs(KS& ks, const LaneCtx& L, const float* qrow, float low_part) {
  constexpr int KLO = k_lo<BK>(), KHI = k_hi<BK>();
  typedef __fp16 half2v __attribute__((ext_vector_type(2)));
  const float nlow = -low_part;
  float w[32];
  float zq = 0.f;
#pragma unroll
  for (int quad = 0; quad < 8; ++quad) {
    const float4v qf = *reinterpret_cast<const float4v*>(qrow + 32 * L.j + 4 * quad);
    const u32x4 mv = *reinterpret_cast<const u32x4*>(L.meta_lds + 128 * L.j + 16 * quad);
    const uint32_t mw[4] = {mv.x, mv.y, mv.z, mv.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w[4 * quad + e] = fmaf(qf[e], meta_scale(mw[e]), 0.0f);
      zq = fmaf(qf[e], meta_zero(mw[e]), zq);
    }
  }
  auto part16 = [&](float a, float b) -> uint32_t {          // this lane's part (high or low) of the pair, see above
    const half2v h = __builtin_amdgcn_cvt_pkrtz(a, b);
    const float xa = fmaf((float)h.x, nlow, a), xb = fmaf((float)h.y, nlow, b);
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(xa, xb));
  };
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    uint32_t op[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float f = 1.0f / k_slot_scale<KLO>(2 * v);
      op[v] = part16(w[k_slot_elem<KLO>(m, 2 * v)] * f, w[k_slot_elem<KLO>(m, 2 * v + 1)] * f);
    }
    ks.qop[m] = u32x4{op[0], op[1], op[2], op[3]};
    if constexpr (KHI != 0) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float f = (float)(1 << KLO) / k_slot_scale<KHI, k_hi_base<BK>()>(2 * v);
        op[v] = part16(w[k_slot_elem<KHI>(m, 2 * v)] * f, w[k_slot_elem<KHI>(m, 2 * v + 1)] * f);
      }
      ks.qoph[m] = u32x4{op[0], op[1], op[2], op[3]};
    }
  }
  zq += __shfl_xor(zq, 16);
  zq += __shfl_xor(zq, 32);
  ks.zq_u = zq * (kCodeUnit - kCodeUnit * low_part);
}

// One 32-token step.  MASKED: tokens at or beyond seq_len get weight 0 (garbage may sit there).
// BK == BV == 16 is the unquantized cache: no scale/zero, operands are the stored patterns (BF: bfloat16).
// NCK / NCV: column sets.  Columns are (group, head) pairs; when R * (groups) exceeds the 16 columns of a matrix tile
// (8 heads with 32-channel groups) the groups are spread over two column sets: set cs carries group grp + cs*(16/R).
// KS: KSeqState for channel-wise keys (then NEWBLK marks the first step of a 64-token block: the query operands are
// rebuilt from that block's scale/zero entries), NoKSeq otherwise.
template <int BK, int BV, int R, bool BF, int NCK, int NCV, bool MASKED, bool NEWBLK = false, typename KS = NoKSeq,
          typename LC = LaneCtx>
__device__ __forceinline__ void compute_step(const StepRegs<BK, BV>& r, const u32x4 (&qb)[NCK][4],
                                             const u32x4 (&qbh)[NCK][4], const float (&qsum_u)[NCK],
                                             float kappa, WaveState<NCV>& st, const LC& L, int step, int seq_len,
                                             KS& ks, const float* qrow = nullptr, float kseq_low = 0.f,
                                             bool rebuild = true) {
  // a tensor of bits = 16 is stored as its 16-bit patterns (BF: bfloat16) and multiplied as it is, no scale/zero
  constexpr bool RAWK = BK == 16, RAWV = BV == 16;
  constexpr bool BFK = RAWK && BF, BFV = RAWV && BF;
  constexpr int KLO = k_lo<BK>(), KHI = k_hi<BK>();   // qbh: the query operand of the high run (3- and 6-bit keys)
  constexpr bool KSEQ = !__is_same(KS, NoKSeq);
  constexpr int kSetStride = (16 / R) * 64;      // bytes between the scale/zero entries of a lane's groups in two sets
  uint32_t kmeta[NCK][8], vmeta[NCV][8];
  if constexpr (!RAWK || !RAWV) {
    // scale/zero bytes: plane order -> LDS -> the entries this lane needs (tokens 4j..4j+3 of both tiles, own groups)
    *reinterpret_cast<u32x4*>(L.meta_lds + L.lane * 16) = r.meta;     // (lanes beyond the bytes fill slots nobody reads)
    if constexpr (KSEQ && NEWBLK) {
      if (rebuild) {                             // (uniform; false only in the second step of a group of 64 or 128 tokens)
        if constexpr (kseq_prescaled<BK>()) kseq_rebuild<BK>(ks, L, qrow, kseq_low);
        else kseq_rebuild_runs<BK>(ks, L, qrow, kseq_low);
      }
    }
#pragma unroll
    for (int x4 = 0; x4 < 2; ++x4) {
#pragma unroll
      for (int cs = 0; cs < NCK; ++cs) {
        if constexpr (KSEQ || RAWK) continue;
        const u32x4 a = *reinterpret_cast<const u32x4*>(L.meta_lds + L.km_rd + cs * kSetStride + x4 * (64 * L.ngk));
        kmeta[cs][4 * x4 + 0] = a.x; kmeta[cs][4 * x4 + 1] = a.y; kmeta[cs][4 * x4 + 2] = a.z; kmeta[cs][4 * x4 + 3] = a.w;
      }
#pragma unroll
      for (int cs = 0; cs < NCV; ++cs) {
        if constexpr (RAWV) continue;
        const u32x4 b = *reinterpret_cast<const u32x4*>(L.meta_lds + L.vm_rd + cs * kSetStride + x4 * (64 * L.ngv));
        vmeta[cs][4 * x4 + 0] = b.x; vmeta[cs][4 * x4 + 1] = b.y; vmeta[cs][4 * x4 + 2] = b.z; vmeta[cs][4 * x4 + 3] = b.w;
      }
    }
  }

  // ---- scores: slot i = token 16*(i/4) + 4*j + i%4 of this step
  float s[8];
  {
    float part[8];
    if constexpr (KSEQ) {
      float4v d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < 4; ++m) {                // two independent accumulation chains (the two 16-token tiles)
        d0 = mma<BF>(unpack_k<KLO>(r.kc[0], m), ks.qop[m], d0);
        d1 = mma<BF>(unpack_k<KLO>(r.kc[1], m), ks.qop[m], d1);
        if constexpr (KHI != 0) {
          d0 = mma<BF>(unpack_k<KHI, k_hi_base<BK>()>(r.kc[0] + KLO, m), ks.qoph[m], d0);
          d1 = mma<BF>(unpack_k<KHI, k_hi_base<BK>()>(r.kc[1] + KLO, m), ks.qoph[m], d1);
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) part[i] = (i < 4 ? d0[i & 3] : d1[i & 3]) + ks.zq_u;
    }
#pragma unroll
    for (int cs = 0; cs < NCK; ++cs) {
      if constexpr (KSEQ) continue;
      float4v d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < 4; ++m) {                // two independent accumulation chains
        d0 = mma<BFK>(unpack_k<KLO>(r.kc[0], m), qb[cs][m], d0);
        d1 = mma<BFK>(unpack_k<KLO>(r.kc[1], m), qb[cs][m], d1);
        if constexpr (KHI != 0) {
          d0 = mma<BFK>(unpack_k<KHI, k_hi_base<BK>()>(r.kc[0] + KLO, m), qbh[cs][m], d0);
          d1 = mma<BFK>(unpack_k<KHI, k_hi_base<BK>()>(r.kc[1] + KLO, m), qbh[cs][m], d1);
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = i < 4 ? d0[i & 3] : d1[i & 3];
        float pt = d;
        if constexpr (!RAWK) pt = fmaf(d, meta_scale(kmeta[cs][i]), fmaf(meta_zero(kmeta[cs][i]), qsum_u[cs], 0.0f));
        part[i] = cs == 0 ? pt : part[i] + pt;
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = sum_over_groups<R>(part[i]);
  }
  bool valid[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    valid[i] = !MASKED || (step * 32 + 16 * (i >> 2) + 4 * L.j + (i & 3) < seq_len);
    if (MASKED && !valid[i]) s[i] = kNegBig;
  }
  // ---- running max (kept st.headroom above the logits): only when some lane sees a larger logit than its current max
  float lmax = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
  float lx = fmaf(lmax, kappa, st.headroom);
  if (__any(lx > st.m)) {
    lx = fmaxf(lx, __shfl_xor(lx, 16));
    lx = fmaxf(lx, __shfl_xor(lx, 32));
    const float m_new = fmaxf(st.m, lx);
    const float f = __builtin_amdgcn_exp2f(st.m - m_new);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) st.acc[dt] *= f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      st.l[v] *= f;
#pragma unroll
      for (int cs = 0; cs < NCV; ++cs) st.zacc[cs][v] *= f;
      st.noff[v] = p_shift<BV>() - (float)v_slot_shift<BV>(v) - m_new;
    }
    st.m = m_new;
  }
  // ---- softmax weights; quantized values: their binary16 products with the value scale, and the value-zero term
  constexpr int VLO = v_lo<BV>(), VHI = v_hi<BV>();
  uint32_t pw[NCV][4], pl[4];                    // pl: low-order bfloat16 part of the weights (bfloat16 cache only)
  uint32_t pwh[NCV][4];                          // weights of the high parts of 3- and 6-bit value codes
  constexpr bool ROTV = !RAWK && !RAWV && !KSEQ && LC::kRotV;   // (rotation is not combined with channel-wise keys)
  float pv[ROTV ? 8 : 1];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int v = i >> 1;
    float p = __builtin_amdgcn_exp2f(fmaf(s[i], kappa, st.noff[v]));
    if (MASKED && !valid[i]) p = 0.f;
    if constexpr (ROTV) pv[i] = p;
    st.l[v] += p;
    if constexpr (!RAWV) {
#pragma unroll
      for (int cs = 0; cs < NCV; ++cs) {
        uint32_t vm = vmeta[cs][i];
        if (MASKED && !valid[i]) vm = 0u;
        st.zacc[cs][v] = fmaf(p, meta_zero(vm), st.zacc[cs][v]);
        if (i & 1) mix_hi(pw[cs][v], p, vm); else mix_lo(pw[cs][v], p, vm);
        if constexpr (VHI != 0) {
          const float ph = p * v_hi_factor<BV>(v);
          if (i & 1) mix_hi(pwh[cs][v], ph, vm); else mix_lo(pwh[cs][v], ph, vm);
        }
      }
    } else if constexpr (!BF) {
      if (i & 1) mix_hi(pw[0][v], p, 0x3C00u); else mix_lo(pw[0][v], p, 0x3C00u);    // times binary16 1.0
    } else {
      // bfloat16 keeps 8 bits: carry the weight as two bfloat16 terms (16 bits) and multiply the values by both
      const uint32_t hi = bf16_rne(p);
      const uint32_t lo = bf16_rne(p - __uint_as_float(hi << 16));
      if (i & 1) { pw[0][v] |= hi << 16; pl[v] |= lo << 16; } else { pw[0][v] = hi; pl[v] = lo; }
    }
  }
  if constexpr (ROTV) {
    // Rotated values: the rounding error of a token's binary16 weight multiplies all of its group's codes alike, and
    // R_v^T gathers what is common to the channels into single output channels (times sqrt(D) for one group per row),
    // while the zero-point term beside it is summed with the unrounded weight.  What the rounding took from the weight
    // is therefore given back at the middle of the code range, through the zero-point sum: the error left is the
    // rounding error times the codes' distance from the middle, which has no common part to gather.
    constexpr float kMidLo = 0.5f * (float)((1 << VLO) - 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = i >> 1;
#pragma unroll
      for (int cs = 0; cs < NCV; ++cs) {
        uint32_t vm = vmeta[cs][i];
        if (MASKED && !valid[i]) vm = 0u;
        const float back = (float)__builtin_bit_cast(_Float16, (uint16_t)((i & 1) ? pw[cs][v] >> 16 : pw[cs][v] & 0xFFFFu));
        st.zacc[cs][v] = fmaf(kMidLo, fmaf(pv[i], meta_scale(vm), -back), st.zacc[cs][v]);
        if constexpr (VHI != 0) {
          constexpr float kMidHi = 0.5f * (float)((1 << VHI) - 1) * (float)(1 << VLO);
          const float f = v_hi_factor<BV>(v);
          const float backh = (float)__builtin_bit_cast(_Float16, (uint16_t)((i & 1) ? pwh[cs][v] >> 16 : pwh[cs][v] & 0xFFFFu));
          st.zacc[cs][v] = fmaf(kMidHi / f, fmaf(pv[i] * f, meta_scale(vm), -backh), st.zacc[cs][v]);
        }
      }
    }
  }
  // (Nothing is scheduled across this point.  The matrix instructions below cannot start before the weights are
  // complete anyway; left free, the scheduler pulls the unpacking of the value codes up into the softmax arithmetic,
  // which costs the kernel a dozen registers it does not have: with the fence no instance of the token-wise kernels
  // spills, without it most do.)
  if constexpr (!KSEQ) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) {
    constexpr int kDtPerSet = 8 / NCV;           // value groups of set 0 own the first d-tiles, of set 1 the rest
    const int cs = dt / kDtPerSet;
    const u32x4 pb = u32x4{pw[cs][0], pw[cs][1], pw[cs][2], pw[cs][3]};
    u32x4 a = unpack_v<VLO>(r.vc, dt);
    if constexpr (VHI != 0)
      st.acc[dt] = mma<BFV>(unpack_v<VHI>(r.vc + 2 * VLO, dt), u32x4{pwh[cs][0], pwh[cs][1], pwh[cs][2], pwh[cs][3]}, st.acc[dt]);
    if constexpr (RAWV && MASKED) {               // unquantized garbage may be Inf/NaN: clear the slots beyond seq_len
      uint32_t* aw = reinterpret_cast<uint32_t*>(&a);
#pragma unroll
      for (int v = 0; v < 4; ++v) aw[v] &= (valid[2 * v] ? 0x0000FFFFu : 0u) | (valid[2 * v + 1] ? 0xFFFF0000u : 0u);
    }
    st.acc[dt] = mma<BFV>(a, pb, st.acc[dt]);
    if constexpr (BFV) st.acc[dt] = mma<BFV>(a, u32x4{pl[0], pl[1], pl[2], pl[3]}, st.acc[dt]);
  }
}

// Record layout in the workspace: [b][hq][split] x (kHeadDim + 4) floats = acc[128], m, l, 0, 0.
constexpr int kRec = kHeadDim + 4;

// Fused decode step, first half: quantize the one new token of this (b,h) and store it at row t of the planes.  The
// first 16 lanes take the key row, the next 16 the value row (8 channels per lane; `raw` holds the lane's 16 input
// bytes, loaded by the caller).  Same arithmetic and bytes as the bulk quantize-append kernel.  The key codes and both
// scale/zero entries go to memory from here; the value codes go to `vstage` (128 bytes of LDS), from where the threads
// that own the block's words insert them after a barrier.  The reconstructed rows (code * scale + zero, one rounding as
// in App. B "Dequantization") go to `hat` (LDS: 128 key elements, then 128 value elements): the new token joins the
// attention from there, not from the cache.  bh: stream index in the planes (0 when paged: t is then a row number in
// plane order); sbh: the (batch, kv head) pair, for the stream's largest value-scale exponent.
template <int BK, int BV>
__device__ __forceinline__ void append_one(const DecodeArgs& a, int bh, int sbh, int tid, u32x4 raw, uint8_t* vstage, int64_t t,
                                           float* hat) {
  const Geom& g = a.g;
  const bool is_v = tid >= 16;
  const int lane16 = tid & 15, d0 = lane16 * 8;
  const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), a.in_bf16);
  if (g.rotate_k | g.rotate_v) {                   // both 16-lane rows run the butterflies; a row that is not rotated
    float xr[8];                                   // keeps its own numbers
#pragma unroll
    for (int e = 0; e < 8; ++e) xr[e] = x[e];
    rotate8(xr, lane16, is_v ? rot_sign_bits(g.signs_v, lane16) : rot_sign_bits(g.signs_k, lane16));
    const bool take = is_v ? g.rotate_v != 0 : g.rotate_k != 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = take ? xr[e] : x[e];
  }
  uint32_t codes[8];
  uint16_t S, Z;
  const int bits = is_v ? BV : BK;
  const int G = is_v ? g.g_v : g.g_k, ng = is_v ? g.ng_v : g.ng_k;
  const int lpg = G >> 3;
  quantize8(x, bits, lpg, codes, &S, &Z);
  if (is_v && (lane16 & (lpg - 1)) == 0) note_value_scale(a.cache.v_scale_exp + sbh, S);
  // (picked by integer arithmetic: a per-lane choice among pointers of the argument block becomes a lookup in private memory)
  const uintptr_t km = reinterpret_cast<uintptr_t>(a.cache.k_meta) + (uintptr_t)((int64_t)bh * g.km_stream);
  const uintptr_t vm = reinterpret_cast<uintptr_t>(a.cache.v_meta) + (uintptr_t)((int64_t)bh * g.vm_stream);
  uint32_t* meta = reinterpret_cast<uint32_t*>(km + (is_v ? vm - km : (uintptr_t)0));
  if ((lane16 & (lpg - 1)) == 0) meta[meta_index(t, lane16 >> lpg_shift(lpg), ng)] = (uint32_t)S | ((uint32_t)Z << 16);
  if (!is_v) {
    store_key_codes<BK>((uint8_t*)a.cache.k_codes + (int64_t)bh * g.kc_stream + t * (16 * BK), lane16, codes);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) vstage[d0 + e] = (uint8_t)codes[e];
  }
  const float sc = widen16(S, false), zp = widen16(Z, false);
#pragma unroll
  for (int e = 0; e < 8; ++e) hat[(is_v ? kHeadDim : 0) + d0 + e] = fmaf((float)codes[e], sc, zp);   // (exact product: one rounding)
}

// Second half of the fused append: thread d < 128 inserts channel d's code of the new token into its 32-bit word of
// the 32-token block (the other fields of the word belong to other tokens of the block and keep their bits).  With
// 2-bit fields channels d and d+16 share a word (with 1-bit fields d, d+16, d+32 and d+48), so the thread of the first
// of those 16-channel tiles owns the word.  The word is loaded at the top of the kernel (field_word), long before the
// codes exist, and stored from here.  `shift`: the field is bits [shift, shift + B) of the staged code.
template <int B> constexpr int field_tiles() { return B == 1 ? 4 : B == 2 ? 2 : 1; }   // 16-channel tiles per word
template <int B> __device__ __forceinline__ bool field_owner(int tid) {
  return tid < kHeadDim && !((tid >> 4) & (field_tiles<B>() - 1));
}
template <int B> __device__ __forceinline__ int field_word(int tid, int u) {
  int dw, bit;
  v_field(u, tid & (kHeadDim - 1), B, &dw, &bit);
  return dw;
}
template <int B>
__device__ __forceinline__ uint32_t field_insert(uint32_t w, int tid, const uint8_t* vstage, int u, int shift) {
  const uint32_t fmask = (1u << B) - 1u;
#pragma unroll
  for (int f = 0; f < field_tiles<B>(); ++f) {
    int dwf, bitf;
    v_field(u, tid + 16 * f, B, &dwf, &bitf);             // same word, the neighbouring tiles' fields
    w = (w & ~(fmask << bitf)) | ((((uint32_t)vstage[tid + 16 * f] >> shift) & fmask) << bitf);
  }
  return w;
}

// One output element in the caller's type (16-bit types: rounded once).
__device__ __forceinline__ void store_out(void* out, int out_dtype, int64_t i, float val) {
  if (out_dtype == KVQ_F32) ((float*)out)[i] = val;
  else if (out_dtype == KVQ_F16) ((_Float16*)out)[i] = (_Float16)val;
  else ((uint16_t*)out)[i] = (uint16_t)bf16_rne(val);
}
// Partial records travel between workgroups that may sit on different parts of the chip, each with a cache of its own:
// their stores and loads are device-scope atomic accesses (performed where every compute unit sees them).
__device__ __forceinline__ void store_device(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Final output of rotated values: the normalized row sits in the rotated basis (LDS, 128 floats); 16 threads take it
// back with R_v^T (8 channels each) and store it in the output type.
__device__ __forceinline__ void store_unrotated_row(const float* row, int lane16, const uint32_t signs[4], void* out,
                                                    int out_dtype, int64_t hq) {
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = row[8 * lane16 + e];
  unrotate8(x, lane16, rot_sign_bits(signs, lane16));
  const int64_t o = hq * kHeadDim + 8 * lane16;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (out_dtype == KVQ_F32) ((float*)out)[o + e] = x[e];
    else if (out_dtype == KVQ_F16) ((_Float16*)out)[o + e] = (_Float16)x[e];
    else ((uint16_t*)out)[o + e] = f32_to_bf16_bits(x[e]);
  }
}

// KSEQ: channel-wise keys (the caller passes the flushed part of the sequence: seq_len is a multiple of 64, nothing
// is appended); a wavefront then walks whole 64-token blocks (pairs of steps), rebuilding its query operands per block.
// PAGED: the planes are pools of pages; a step's data is found through this sequence's row of the page table.
// ROTV: the values are stored rotated (quantized caches with token-wise keys; compute_step then corrects its weights).
template <int BK, int BV, int R, int NW, bool BF, int NCK, int NCV, bool KSEQ = false, bool PAGED = false, bool ROTV = false>
__global__ __launch_bounds__(64 * NW, KVQ_WAVES_PER_SIMD) void decode_kernel(const DecodeArgs a) {
  constexpr int kSetGroups = 16 / R;             // groups per column set
  constexpr bool RAWK = BK == 16, RAWV = BV == 16;     // a tensor kept as its 16-bit patterns (either one, or both)
  constexpr bool RAW = RAWK;                          // (what the key side and the query staging ask)
  static_assert(!KSEQ || (!RAWK && !RAWV && NCK == 1), "channel-wise keys: quantized, one key column per head");
  static_assert(!ROTV || (!RAWK && !RAWV), "rotated values: both tensors quantized");
  constexpr int kRing = ring_stages<BK, BV, NCK, NCV, ROTV>();
#ifndef KVQ_KSEQ_STAGES
#define KVQ_KSEQ_STAGES 2
#endif
  // (channel-wise keys: the rebuild leaves registers for two steps, and the kernel, bound by its vector instructions,
  // measures no faster with a deeper ring)
  constexpr int kStages = KSEQ ? (kRing < KVQ_KSEQ_STAGES ? kRing : KVQ_KSEQ_STAGES) : kRing;
  constexpr int SPB = KSEQ ? 2 : 1;              // steps a wavefront takes in a row
  // codes enter the matrix unit as binary16 subnormals (code x 2^-24): the key side's factor goes into the logits'
  // scale, the value side's into the final accumulator
  constexpr float kUnit = RAWK ? 1.0f : kCodeUnit, kInvUnit = RAWK ? 1.0f : kInvCodeUnit;
  constexpr float kInvUnitV = RAWV ? 1.0f : kInvCodeUnit;
  __shared__ float sm_o[NW][R][kHeadDim];
  __shared__ float sm_m[NW][R], sm_l[NW][R];
  __shared__ __attribute__((aligned(16))) uint16_t sm_q[R][kHeadDim];
  // channel-wise keys: the query in binary32, channel d divided by k_chan_scale(d); row R is all zero
  __shared__ __attribute__((aligned(16))) float sm_qf[KSEQ ? R + 1 : 1][kHeadDim];
  __shared__ __attribute__((aligned(16))) uint8_t sm_meta[NW][1024];
  __shared__ uint8_t sm_vnew[kHeadDim];          // fused step: the new token's value codes,
  __shared__ float sm_hat[2][kHeadDim];           // its reconstructed key and value rows,
  __shared__ float sm_mnew[R];                    // and its logit per head in log2 units
  __shared__ float sm_qsum[R][4];
  const Geom& g = a.g;
  const kvq_cache& cache = a.cache;
  const uint16_t* __restrict__ q = a.q;
  const int q_bf16 = a.q_bf16, q_heads = a.q_heads, out_dtype = a.out_dtype;
  const int steps_per_split = a.steps_per_split;
  const float softmax_scale = a.softmax_scale;
  float* __restrict__ ws = a.ws;
  void* __restrict__ out = a.out;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int split = blockIdx.x, bh = blockIdx.y;
  const int b = bh / g.kv_heads, hk = bh % g.kv_heads;
  // this sequence's length: its own when the caller gave per-sequence lengths, inside what the launch was planned for
  int seq_len = a.seq_len;
  if (a.seq_lens) {
    int n = min(max(a.seq_lens[b] + a.lens_offset, 1), a.lens_bound);
    if (a.lens_mode == 1) n &= ~(a.lens_block - 1);         // a residual buffer of lens_block slots: the flushed blocks ...
    else if (a.lens_mode == 2) n &= a.lens_block - 1;       // ... or the tail in the buffer (either may be empty)
    seq_len = min(n, a.seq_len);
  }

  std::conditional_t<ROTV, LaneCtxRotV, LaneCtx> L;
  L.lane = lane; L.c = lane & 15; L.j = lane >> 4;
  L.ngk = g.ng_k; L.ngv = g.ng_v;
  const int h = L.c % R, grp = L.c / R;
  const bool act_k = grp < g.ng_k, act_v = grp < g.ng_v;
  L.gk = act_k ? grp : 0; L.gv = act_v ? grp : 0;
  const int64_t bh_base = PAGED ? 0 : bh;           // paged: rows are numbered from the plane base (virtual_token)
  L.kc = (const uint8_t*)cache.k_codes + bh_base * g.kc_stream;
  L.vc = (const uint8_t*)cache.v_codes + bh_base * g.vc_stream;
  L.kc_off = L.c * (16 * BK) + L.j * (4 * BK);
  L.vc_off = lane * (BV == 1 ? 8 : 16);
  {
    // channel-wise keys: 512 bytes of scale/zero per group of seq_g = 32, 64 or 128 tokens (32 lanes), fetched with
    // every step of the group (1, 2 or 4 of them)
    const int nk = RAWK ? 0 : KSEQ ? 32 : 8 * g.ng_k, nv = RAWV ? 0 : 8 * g.ng_v;   // (an unquantized tensor has none)
    const int ml = min(lane, nk + nv - 1);       // lanes beyond the scale/zero bytes of a step repeat the last 16
    const bool is_k = ml < nk;
    L.meta_base = is_k ? (const uint8_t*)cache.k_meta + bh_base * g.km_stream
                       : (const uint8_t*)cache.v_meta + bh_base * g.vm_stream;
    L.meta_mul = is_k ? (KSEQ ? 16384 / g.seq_g : 128 * g.ng_k) : 128 * g.ng_v;
    L.meta_off = 16 * (is_k ? ml : ml - nk);
    L.meta_step_mask = (KSEQ && is_k) ? ~(uint32_t)((g.seq_g >> 5) - 1) : ~0u;
    L.km_rd = (L.gk * 16 + 4 * L.j) * 4;                       // key bytes come first in the LDS copy
    L.vm_rd = 16 * nk + (L.gv * 16 + 4 * L.j) * 4;
    L.meta_lds = &sm_meta[wave][0];
  }

  // ---- what this launch reads.  A fused decode step does not read its new token (position seq_len - 1) back from the
  // cache: the workgroup that owns that position quantizes and stores it, and adds it to the attention as one more
  // partial record, computed from the reconstruction it holds in registers (no store -> load round trip, no fence).
  constexpr bool kCanAppend = !RAWK && !RAWV && !KSEQ;
  const bool fused = kCanAppend && a.k_new != nullptr;
  const int n_att = fused ? seq_len - 1 : seq_len;        // tokens attended through the cache planes
  const int n_steps = (n_att + 31) >> 5;
  const int step_begin = split * steps_per_split;
  const int step_end = min(step_begin + steps_per_split, n_steps);
  const bool do_append = fused && split == ((seq_len + 31) / 32 - 1) / steps_per_split;   // uniform over the workgroup
  // this wavefront's steps: step_begin + wave, + NW, ...; the last one may be the ragged tail of the sequence
  const int first = step_begin + SPB * wave;
  auto step_of = [&](int i) { return KSEQ ? first + 2 * NW * (i >> 1) + (i & 1) : first + NW * i; };
  const int n_my = first < step_end ? SPB * ((step_end - first + SPB * NW - 1) / (SPB * NW)) : 0;
  const bool ragged = (n_att & 31) != 0;
  const bool own_tail = ragged && n_my > 0 && step_of(n_my - 1) == n_steps - 1;
  const int n_full = own_tail ? n_my - 1 : n_my;   // complete steps of this wavefront
  // A step that is always there to load from: wavefronts with nothing to do still issue the ring's loads (see refill).
  const int safe_step = min(step_begin, max(n_steps - 1, 0));
  // paged: logical step -> step number in plane order (page of the pool, this head's share of it, step inside it)
  // (this workgroup's slice of its table row is copied to LDS first: a page number is needed before every step's
  // loads can be issued, and a global load in front of them costs the ring most of its depth)
  constexpr int kPageSlots = PAGED ? 2048 : 1;
  __shared__ int32_t sm_pages[kPageSlots];
  const int32_t* __restrict__ my_pages = PAGED ? cache.page_table + (int64_t)b * g.pages_per_seq : nullptr;
  const int step_shift = g.page_shift - 5;
  const int page0 = safe_step >> step_shift;
  const int last_needed = max(max(step_end - 1, safe_step), do_append ? (seq_len - 1) >> 5 : 0);
  const int n_pages_mine = (last_needed >> step_shift) - page0 + 1;
  const bool pages_in_lds = n_pages_mine <= kPageSlots;
  if constexpr (PAGED) {
    if (pages_in_lds) {
      for (int i = tid; i < n_pages_mine; i += 64 * NW) sm_pages[i] = my_pages[page0 + i];
      __syncthreads();
    }
  }
  auto page_of_step = [&](int step) -> int64_t {
    return pages_in_lds ? sm_pages[(step >> step_shift) - page0] : my_pages[step >> step_shift];
  };
  auto fetch = [&](StepRegs<BK, BV>& dst, int step, uint32_t lane_mask = ~0u) {
    if constexpr (PAGED) {
      load_step<BK, BV, true>(dst, L, ((page_of_step(step) * g.kv_heads + hk) << step_shift) + (step & ((1 << step_shift) - 1)), lane_mask);
    } else {
      load_step<BK, BV>(dst, L, step, lane_mask);
    }
  };

  // ---- the small loads of the prologue go first, none of them behind a branch, so that they return ahead of the
  // ring's first fill and the compiler can count what is in flight behind each: the query rows (every thread loads;
  // threads beyond the rows re-read the first 16 bytes), and in a fused step the new token's rows and the words of the
  // value block that take its codes (threads that have none of these re-read the query).
  int stream_scale_exp = 0;                        // largest exponent field of the stream's value scales (weight_headroom)
  if constexpr (!RAWV) stream_scale_exp = cache.v_scale_exp[bh];
  const int r_act = a.heads_per_kv;                // heads that exist (R is the next power of two)
  const bool q_lane = tid < R * 16 && (tid >> 4) < r_act;
  const uint16_t* qsrc = q + ((int64_t)b * q_heads + hk * r_act) * kHeadDim + (q_lane ? tid * 8 : 0);
  u32x4 qraw = *reinterpret_cast<const u32x4*>(qsrc);
  constexpr int VLO_ = v_lo<BV>(), VHI_ = v_hi<BV>();
  u32x4 nraw = u32x4{0u, 0u, 0u, 0u};
  uint32_t vw_lo = 0u, vw_hi = 0u;
  uint32_t* vw_lo_p = nullptr; uint32_t* vw_hi_p = nullptr;
  int64_t t_new = 0;
  int u_new = 0;                                   // the new token's place in its 32-token block
  if constexpr (kCanAppend) {
    // (paged: the new token's row number in plane order, with the stream index 0)
    if constexpr (PAGED) {
      const int64_t pg = do_append ? page_of_step((seq_len - 1) >> 5) : 0;
      t_new = ((pg * g.kv_heads + hk) << g.page_shift) + ((seq_len - 1) & ((1 << g.page_shift) - 1));
    } else {
      t_new = seq_len - 1;
    }
    // (the address is picked by integer arithmetic: a per-lane choice among pointers held in the argument block would
    // be turned into a lookup in private memory)
    const bool new_lane = do_append && tid < 32;
    const int64_t row_off = ((int64_t)b * a.nsb + (int64_t)hk * a.nsh + (tid & 15) * 8) * 2;
    const uintptr_t qp = reinterpret_cast<uintptr_t>(qsrc), kp = reinterpret_cast<uintptr_t>(a.k_new),
                    vp = reinterpret_cast<uintptr_t>(a.v_new);
    const uintptr_t nsrc = qp + (new_lane ? (kp - qp) + (tid >= 16 ? vp - kp : (uintptr_t)0) + (uintptr_t)row_off : (uintptr_t)0);
    nraw = *reinterpret_cast<const u32x4*>(nsrc);
    uint32_t* vblk = (uint32_t*)((uint8_t*)cache.v_codes + bh_base * g.vc_stream) + (t_new >> 5) * (int64_t)(128 * BV);
    u_new = (int)(t_new & 31);
    vw_lo_p = do_append && field_owner<VLO_>(tid) ? vblk + field_word<VLO_>(tid, u_new) : nullptr;
    vw_lo = *(vw_lo_p ? vw_lo_p : reinterpret_cast<const uint32_t*>(qsrc));
    if constexpr (VHI_ != 0) {
      vw_hi_p = do_append && field_owner<VHI_>(tid) ? vblk + 128 * VLO_ + field_word<VHI_>(tid, u_new) : nullptr;
      vw_hi = *(vw_hi_p ? vw_hi_p : reinterpret_cast<const uint32_t*>(qsrc));
    }
  }

  // ---- register ring of kStages steps, filled right away.
  // Ring slot k is refilled with the wavefront's i-th step (the ragged tail included); past its last step the loads
  // are still issued, at that last step (or at safe_step for a wavefront that has none) and collapsed to one cache line
  // each (see load_step), so that no load of the ring is conditional.
  StepRegs<BK, BV> buf[kStages];
  auto refill = [&](int k, int i) {
    fetch(buf[k], n_my > 0 ? step_of(min(i, n_my - 1)) : safe_step, i < n_my ? ~0u : 0u);
  };
  // Only the first half of the ring goes out in front of the query staging: the memory pipeline of a compute unit
  // takes in about what two steps of eight wavefronts ask for, a wavefront that issues more waits at the load until
  // earlier data has come back, and the barrier of the staging below would wait for the slowest of them.  The second
  // half follows the barrier, by when the first is on its way out of memory.
  constexpr int kEarly = (kStages + 1) / 2;
#pragma unroll
  for (int k = 0; k < kEarly; ++k) refill(k, k);

  // ---- fused step: quantize the new token (two 16-lane rows of the first wavefront), store keys and scale/zero, stage
  // the value codes for the threads that own the block's words
  if constexpr (kCanAppend) {
    if (do_append && tid < 32) append_one<BK, BV>(a, PAGED ? 0 : bh, bh, tid, nraw, sm_vnew, t_new, &sm_hat[0][0]);
  }

  // ---- query rows of this kv head -> LDS, then per-lane operands
  bool q_is_bf16 = q_bf16 != 0;
  if (tid < R * 16) {
    u32x4 raw = q_lane ? qraw : u32x4{0u, 0u, 0u, 0u};   // a surplus head is an all-zero query: uniform weights, never stored
    if constexpr (!RAW) {
      if (g.rotate_k) {
        // rotated keys: the scores need R q, rounded once to binary16 (16 threads hold one query row, 8 channels each)
        const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), q_is_bf16);
        rotate8(x, tid & 15, rot_sign_bits(g.signs_k, tid & 15));
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          w[e] = (uint32_t)f32_to_f16_bits(x[2 * e]) | ((uint32_t)f32_to_f16_bits(x[2 * e + 1]) << 16);
        raw = u32x4{w[0], w[1], w[2], w[3]};
      }
    }
    reinterpret_cast<u32x4*>(&sm_q[0][0])[tid] = raw;
    if constexpr (KSEQ) {
      const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
      const bool staged_bf16 = q_is_bf16 && !g.rotate_k;       // (a rotated query has been rounded to binary16 above)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        sm_qf[tid >> 4][8 * (tid & 15) + e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), staged_bf16) /
                                              (kseq_prescaled<BK>() ? k_chan_scale<BK>(e) : 1.0f);
    }
    if constexpr (!RAW) {
      // per-group sums of the (staged) query: the zero points of a key group enter the scores through them
      const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
      const bool f16_now = !q_is_bf16 || g.rotate_k;
      float part = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) part += widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), !f16_now);
      const int lpg = g.g_k >> 3;                    // lanes per key group: 4, 8 or 16
      for (int off = 1; off < lpg; off <<= 1) part += __shfl_xor(part, off, 16);
      if (((tid & 15) & (lpg - 1)) == 0) sm_qsum[tid >> 4][(tid & 15) >> lpg_shift(lpg)] = part;
    }
  }
  if constexpr (KSEQ) { if (tid < kHeadDim) sm_qf[R][tid] = 0.f; }
  if constexpr (!RAW) q_is_bf16 = q_is_bf16 && !g.rotate_k;      // the staged rotated query is binary16
  __syncthreads();
#pragma unroll
  for (int k = kEarly; k < kStages; ++k) refill(k, k);       // the second half of the ring's first fill
  auto widen = [&](uint16_t bits) -> float {
    return q_is_bf16 ? __uint_as_float((uint32_t)bits << 16) : (float)__builtin_bit_cast(_Float16, bits);
  };
  // ---- fused step, second half: the value codes go into their words (loaded at the top), and the new token becomes a
  // partial record of its own: logit of every head against the reconstructed key row (maximum = that logit, sum = one
  // weight of 1, accumulator = the reconstructed value row), which the merge below adds to the wavefronts' records
  if constexpr (kCanAppend) {
    if (do_append) {                               // uniform over the workgroup
      if (vw_lo_p) *vw_lo_p = field_insert<VLO_>(vw_lo, tid, sm_vnew, u_new, 0);
      if constexpr (VHI_ != 0) {
        if (vw_hi_p) *vw_hi_p = field_insert<VHI_>(vw_hi, tid, sm_vnew, u_new, VLO_);
      }
      if (tid < R * 16) {                            // 16 threads per head: 8 channels each, then a sum over the 16
        const int hh = tid >> 4, lane16 = tid & 15;
        const u32x4 qv = *reinterpret_cast<const u32x4*>(&sm_q[hh][8 * lane16]);
        const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) part = fmaf(widen((uint16_t)(qw[e >> 1] >> (16 * (e & 1)))), sm_hat[0][8 * lane16 + e], part);
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) part += __shfl_xor(part, off, 16);
        if (lane16 == 0) sm_mnew[hh] = part * (softmax_scale * kLog2e);
      }
    }
  }
  // column c of set cs carries head h restricted to key group grp + cs*kSetGroups (zero elsewhere); this lane's 32
  // channels are 32j..32j+31 and lie in one group
  constexpr int KLO = k_lo<BK>(), KHI = k_hi<BK>();
  u32x4 qb[NCK][4];
  u32x4 qbh[NCK][4];                             // operand of the high run of 3- and 6-bit key codes (else unused)
  float qsum_u[NCK];
  {
    uint16_t mych[32];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const u32x4 v = reinterpret_cast<const u32x4*>(&sm_q[h][32 * L.j])[k];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) mych[8 * k + e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
    }
#pragma unroll
    for (int cs = 0; cs < NCK; ++cs) {
      const int gcs = grp + cs * kSetGroups;
      const bool act = gcs < g.ng_k;
      const bool mine = act && ((32 * L.j) / g.g_k == gcs);
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        uint32_t w[4] = {0u, 0u, 0u, 0u}, wh[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint16_t bits = mych[k_slot_elem<KLO>(m, i)];
          uint32_t e;                              // unquantized: the query's own 16-bit pattern (same type as the cache)
          if constexpr (RAW) e = bits;
          else e = __builtin_bit_cast(uint16_t, (_Float16)(widen(bits) / k_slot_scale<KLO>(i)));
          if (mine) w[i >> 1] |= e << (16 * (i & 1));
          if constexpr (KHI != 0) {                // high run: its own slot order, and the codes' factor 2^LO
            const float qh = widen(mych[k_slot_elem<KHI>(m, i)]) * ((float)(1 << KLO) / k_slot_scale<KHI, k_hi_base<BK>()>(i));
            if (mine) wh[i >> 1] |= (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)qh) << (16 * (i & 1));
          }
        }
        qb[cs][m] = u32x4{w[0], w[1], w[2], w[3]};
        qbh[cs][m] = u32x4{wh[0], wh[1], wh[2], wh[3]};
      }
      float qsum = 0.f;
      if constexpr (!RAW) { if (act) qsum = sm_qsum[h][gcs]; }
      qsum_u[cs] = qsum * kUnit;
    }
  }
  const float kappa = softmax_scale * kLog2e * kInvUnit;

  WaveState<NCV> st;
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) st.acc[dt] = float4v{0.f, 0.f, 0.f, 0.f};
  st.m = kNegBig;
  st.headroom = 0.f;
  if constexpr (!RAWV) st.headroom = weight_headroom<BV>(stream_scale_exp);
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    st.l[v] = 0.f; st.noff[v] = 0.f;
#pragma unroll
    for (int cs = 0; cs < NCV; ++cs) st.zacc[cs][v] = 0.f;
  }

  // ---- main loop, unrolled over the ring: compute a step, then refill its registers with the step kStages
  // ahead, so that kStages-1 steps of loads are always in flight behind the one being computed.
  typename std::conditional<KSEQ, typename std::conditional<k_hi<BK>() != 0, KSeqState2, KSeqState>::type, NoKSeq>::type ks;
  const float* qrow = &sm_qf[KSEQ ? (grp < 2 ? h : R) : 0][0];   // (column groups 0 and 1 carry the key side)
  // one complete step out of ring slot k (for channel-wise keys an even slot starts a 64-token block, and the query
  // operands are rebuilt there: once per group of 64 tokens, twice per group of 128 -- the second time from the same
  // entries -- and in the odd steps too when a group is one step long)
  const bool rebuild_every_step = KSEQ && g.seq_g == 32;       // (uniform)
  auto full_step = [&](int k, int i) {
    if constexpr (KSEQ) {                        // an even step of this wavefront's sequence starts a block (uniform;
      const int odd = kStages % 2 == 0 ? (k & 1) : (i & 1);      // with an even ring it is the ring slot's parity)
      compute_step<BK, BV, R, BF, NCK, NCV, false, true>(buf[k], qb, qbh, qsum_u, kappa, st, L, step_of(i), n_att, ks, qrow,
                                                         grp == 1 ? 1.0f : 0.0f, !odd || rebuild_every_step);
    } else {
      compute_step<BK, BV, R, BF, NCK, NCV, false>(buf[k], qb, qbh, qsum_u, kappa, st, L, step_of(i), n_att, ks);
    }
  };
  // the ragged tail of the sequence out of ring slot k (it came through the ring like every other step): masked
  auto tail_step = [&](int k) {
    if constexpr (!KSEQ)
      compute_step<BK, BV, R, BF, NCK, NCV, true>(buf[k], qb, qbh, qsum_u, kappa, st, L, n_steps - 1, n_att, ks);
  };
  int it = 0;
  for (; it + kStages <= n_full; it += kStages) {
#pragma unroll
    for (int k = 0; k < kStages; ++k) {
      full_step(k, it + k);
      refill(k, it + k + kStages);
    }
  }
#pragma unroll
  for (int k = 0; k < kStages - 1; ++k)          // the last few complete steps are already in the ring,
    if (it + k < n_full) full_step(k, it + k);
  if (own_tail) {                                 // and so is the tail, in the slot after them
    const int kt = n_full - it;
#pragma unroll
    for (int k = 0; k < kStages; ++k)
      if (kt == k) tail_step(k);
  }

  // ---- wavefront totals: l and zacc over register classes and the 4 lane groups j; then this lane's output rows
  float l = 0.f;
#pragma unroll
  for (int v = 0; v < 4; ++v) l = fmaf(st.l[v], (float)(1 << v_slot_shift<BV>(v)), l);
  l += __shfl_xor(l, 16); l += __shfl_xor(l, 32);
#pragma unroll
  for (int cs = 0; cs < NCV; ++cs) {
    float z = 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) z = fmaf(st.zacc[cs][v], (float)(1 << v_slot_shift<BV>(v)), z);
    z += __shfl_xor(z, 16); z += __shfl_xor(z, 32);
    const int gcs = grp + cs * kSetGroups;                     // the value group this lane's column carries in set cs
    if (gcs < g.ng_v) {
      const int dtg = 8 / g.ng_v;                              // d-tiles per value group
#pragma unroll
      for (int dt = 0; dt < 8; ++dt)                           // (all eight tiles with their registers named at compile
        if (dt / dtg == gcs) {                                 // time; the stores of the other groups' tiles are skipped)
          float* dst = &sm_o[wave][h][16 * dt + 4 * L.j];
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) dst[rr] = fmaf(st.acc[dt][rr], kInvUnitV, z);
        }
    }
  }
  // (records of kernels that carry their weights times different powers of two meet in one merge when channel-wise keys
  // add the residual tail: the difference to 2^10 goes into the record's maximum)
  if (grp == 0 && L.j == 0) { sm_m[wave][h] = st.m + (10.0f - p_shift<BV>()); sm_l[wave][h] = l; }
  __syncthreads();

  // ---- merge the wavefronts; write a partial record, or the result when there is one split
  for (int idx = tid; idx < R * kHeadDim; idx += 64 * NW) {
    const int hh = idx / kHeadDim, d = idx % kHeadDim;
    float M = sm_m[0][hh];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w][hh]);
    if (do_append) M = fmaxf(M, sm_mnew[hh]);
    float o = 0.f, ll = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float f = exp2f(sm_m[w][hh] - M);
      o = fmaf(f, sm_o[w][hh][d], o);
      ll = fmaf(f, sm_l[w][hh], ll);
    }
    if (do_append) {                               // the new token: one weight of 1 (records carry their sums times 2^10)
      const float f = 1024.0f * exp2f(sm_mnew[hh] - M);
      o = fmaf(f, sm_hat[1][d], o);
      ll += f;
    }
    if (hh >= r_act) continue;
    const int64_t hq = (int64_t)b * q_heads + hk * r_act + hh;
    if (a.extra_splits != 0) {
      // one more record per head lies in the workspace, written by an earlier launch on the same stream (the flushed
      // part of a cache with a residual buffer, when this launch is the buffer's): it joins here, and no merge launch
      // follows
      const float* er = ws + hq * a.extra_splits * kRec;
      const float me = er[kHeadDim], le = er[kHeadDim + 1], oe = er[d];
      const float Mn = fmaxf(M, me);
      const float f0 = exp2f(M - Mn), fe = exp2f(me - Mn);
      o = fmaf(fe, oe, o * f0);
      ll = fmaf(fe, le, ll * f0);
    }
    if (a.rec_splits == 1) {
      const float val = o / ll;
      if (g.rotate_v) { sm_o[0][hh][d] = val; continue; }      // (only this thread touches element (hh, d))
      store_out(out, out_dtype, hq * kHeadDim + d, val);
    } else {
      // (device-scope stores: the record is read by a workgroup on another part of the chip, whose nearest cache is
      // not this one)
      float* rec = ws + (hq * a.rec_splits + a.rec_base + split) * kRec;
      store_device(rec + d, o);
      if (d == 0) { store_device(rec + kHeadDim, M); store_device(rec + kHeadDim + 1, ll); }
    }
  }
  bool wrote_rows = a.rec_splits == 1;               // this workgroup has left normalized rows (rotated values: in sm_o)
  if (a.merge_tag != 0) {                            // uniform: the launch's workgroups merge their records themselves
    // The workgroup of a (b, h_kv) stream that finishes last combines the stream's records: every workgroup counts
    // itself in (one device-scope increment, issued after all its record stores have been acknowledged), and the one
    // that brings the count to n_splits reads all records back.  Nobody waits for anybody.  Records and counter are
    // device-scope atomic accesses, which go past the caches that are private to a part of the chip; a device-scope
    // FENCE is not used on purpose: it writes back and invalidates the whole second-level cache of the workgroup's part
    // of the chip, under the streaming loads of every other workgroup there, and was measured to cost the 8B-layer
    // step 10 us (the barrier in front of the increment already waits for this workgroup's stores).  The counter word carries the launch's
    // tag above the count, so that whatever the word held before this launch -- another launch's tag, or the bytes of
    // a fresh workspace -- counts as zero; the last workgroup leaves the count at zero for a replay of the same launch.
    __shared__ int sm_last;
    __syncthreads();                                 // (all record stores of this workgroup are performed)
    if (tid == 0) {
      unsigned long long* cnt = reinterpret_cast<unsigned long long*>(ws + (int64_t)g.batch * q_heads * a.rec_splits * kRec) + bh;
      const unsigned long long tag = a.merge_tag << 16;
      unsigned long long seen = __hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), want;
      do {
        want = ((seen & ~0xFFFFull) == tag ? seen : tag) + 1ull;
      } while (!__hip_atomic_compare_exchange_strong(cnt, &seen, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      const int last = (int)(want & 0xFFFFull) == a.rec_splits;
      if (last) __hip_atomic_store(cnt, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sm_last = last;
    }
    __syncthreads();
    if (sm_last) {                                   // uniform over the workgroup
      const int n_rec = a.rec_splits;
      for (int idx = tid; idx < r_act * kHeadDim; idx += 64 * NW) {
        const int hh = idx / kHeadDim, d = idx % kHeadDim;
        const int64_t hq = (int64_t)b * q_heads + hk * r_act + hh;
        const float* rec = ws + hq * n_rec * kRec;
        // eight records at a time, all 24 loads of a round in flight together (a record's maximum and sum are the same
        // words for the 128 threads of a head); rounds are chained by a running maximum as in the main loop
        float M = kNegBig, o = 0.f, ll = 0.f;
        for (int s0 = 0; s0 < n_rec; s0 += 8) {
          float ms[8], ls[8], os[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float* r2 = rec + min(s0 + j, n_rec - 1) * kRec;
            ms[j] = load_device(r2 + kHeadDim); ls[j] = load_device(r2 + kHeadDim + 1); os[j] = load_device(r2 + d);
          }
          float Mc = M;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            if (s0 + j >= n_rec) { ms[j] = kNegBig; ls[j] = 0.f; os[j] = 0.f; }
            Mc = fmaxf(Mc, ms[j]);
          }
          const float fo = exp2f(M - Mc);
          o *= fo; ll *= fo;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float f = exp2f(ms[j] - Mc);
            o = fmaf(f, os[j], o);
            ll = fmaf(f, ls[j], ll);
          }
          M = Mc;
        }
        const float val = o / ll;
        if (g.rotate_v) sm_o[0][hh][d] = val;
        else store_out(out, out_dtype, hq * kHeadDim + d, val);
      }
      wrote_rows = true;
    }
  }
  if (wrote_rows && g.rotate_v) {                    // uniform over the workgroup
    __syncthreads();
    if (tid < R * 16 && (tid >> 4) < r_act)
      store_unrotated_row(&sm_o[0][tid >> 4][0], tid & 15, g.signs_v, out, out_dtype,
                          (int64_t)b * q_heads + hk * r_act + (tid >> 4));
  }
}

// Combine the split records of one (b, hq): log-sum-exp merge, then normalize (and take rotated values back).
// 512 threads: four groups of 128 channels, group k takes the records s = k, k+4, ...  Every load is independent of
// the ones before it (the maxima first, by one thread per record; then the weighted sums with the loop unrolled), so
// the kernel costs a few memory latencies rather than one per record.
struct RotV { int32_t on; uint32_t signs[4]; };
constexpr int kMergeGroups = 4;
__global__ __launch_bounds__(128 * kMergeGroups) void merge_kernel(const float* __restrict__ ws, void* __restrict__ out,
                                                                   int out_dtype, int32_t n_splits, RotV rot) {
  __shared__ float row[kHeadDim];
  __shared__ float s_part[kMergeGroups][kHeadDim + 1];     // partial sums of o (128) and l (1) per group
  __shared__ float s_max[128 * kMergeGroups / 64];
  const int64_t hq = blockIdx.x;
  const int tid = threadIdx.x, d = tid & (kHeadDim - 1), grp = tid >> 7;
  const float* rec = ws + hq * n_splits * kRec;
  // maximum over the records
  float M = kNegBig;
  for (int s = tid; s < n_splits; s += 128 * kMergeGroups) M = fmaxf(M, rec[s * kRec + kHeadDim]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
  if ((tid & 63) == 0) s_max[tid >> 6] = M;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < 128 * kMergeGroups / 64; ++w) M = fmaxf(M, s_max[w]);
  // weighted sums of this group's records
  float o = 0.f, l = 0.f;
#pragma unroll 8
  for (int s = grp; s < n_splits; s += kMergeGroups) {
    const float f = exp2f(rec[s * kRec + kHeadDim] - M);
    o = fmaf(f, rec[s * kRec + d], o);
    l = fmaf(f, rec[s * kRec + kHeadDim + 1], l);
  }
  s_part[grp][d] = o;
  if (d == 0) s_part[grp][kHeadDim] = l;
  __syncthreads();
  if (grp != 0) {
    if (!rot.on) return;
  } else {
    o = 0.f; l = 0.f;
#pragma unroll
    for (int k = 0; k < kMergeGroups; ++k) { o += s_part[k][d]; l += s_part[k][kHeadDim]; }
  }
  const float val = o / l;
  if (rot.on) {                                      // uniform
    if (grp == 0) row[d] = val;
    __syncthreads();
    if (tid < 16) store_unrotated_row(row, tid, rot.signs, out, out_dtype, hq);
    return;
  }
  if (out_dtype == KVQ_F32) ((float*)out)[hq * kHeadDim + d] = val;
  else if (out_dtype == KVQ_F16) ((_Float16*)out)[hq * kHeadDim + d] = (_Float16)val;
  else {
    uint32_t u = __float_as_uint(val);
    ((uint16_t*)out)[hq * kHeadDim + d] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
  }
}

inline RotV rot_v_of(const Geom& g) {
  RotV r{g.rotate_v, {g.signs_v[0], g.signs_v[1], g.signs_v[2], g.signs_v[3]}};
  return r;
}

// The same merge for up to 8 records (the plans of the short shapes: 2 to 8 splits): one wavefront pair per head, every
// record's maximum, sum and element loaded at once -- 24 independent loads, one memory latency -- and no step through
// LDS (the kernel above spends two latencies and two barriers, which is most of its 3.9 us at 4 records).
constexpr int kMergeFew = 8;
__global__ __launch_bounds__(kHeadDim) void merge_few_kernel(const float* __restrict__ ws, void* __restrict__ out,
                                                             int out_dtype, int32_t n_splits, RotV rot) {
  __shared__ float row[kHeadDim];
  const int64_t hq = blockIdx.x;
  const int d = threadIdx.x;
  const float* rec = ws + hq * n_splits * kRec;
  float m[kMergeFew], l[kMergeFew], o[kMergeFew];
#pragma unroll
  for (int j = 0; j < kMergeFew; ++j) {
    const float* r = rec + min(j, n_splits - 1) * kRec;       // (records past the last repeat it: same cache lines)
    m[j] = r[kHeadDim]; l[j] = r[kHeadDim + 1]; o[j] = r[d];
  }
  float M = m[0];
#pragma unroll
  for (int j = 1; j < kMergeFew; ++j) M = fmaxf(M, m[j]);
  float os = 0.f, ls = 0.f;
#pragma unroll
  for (int j = 0; j < kMergeFew; ++j) {
    const float f = j < n_splits ? exp2f(m[j] - M) : 0.f;
    os = fmaf(f, o[j], os);
    ls = fmaf(f, l[j], ls);
  }
  const float val = os / ls;
  if (rot.on) {                                      // uniform
    row[d] = val;
    __syncthreads();
    if (d < 16) store_unrotated_row(row, d, rot.signs, out, out_dtype, hq);
    return;
  }
  store_out(out, out_dtype, hq * kHeadDim + d, val);
}

// Merge `records` partial records per (batch, query head) into the output.
inline void launch_merge(const float* ws, void* out, int out_dtype, int32_t heads, int32_t records, RotV rot, hipStream_t stream) {
  if (records <= kMergeFew)
    hipLaunchKernelGGL(merge_few_kernel, dim3(heads), dim3(kHeadDim), 0, stream, ws, out, out_dtype, records, rot);
  else
    hipLaunchKernelGGL(merge_kernel, dim3(heads), dim3(128 * kMergeGroups), 0, stream, ws, out, out_dtype, records, rot);
}


template <int BK, int BV, int R, bool BF, int NCK, int NCV, bool KSEQ, bool PAGED>
void launch_nw(const DecodeArgs& a, const DecodePlan& plan, dim3 grid, hipStream_t stream) {
  if constexpr (BK != 16 && BV != 16 && !KSEQ) {
    if (a.g.rotate_v) {
      if (plan.waves_per_wg == 8)
        hipLaunchKernelGGL((decode_kernel<BK, BV, R, 8, BF, NCK, NCV, KSEQ, PAGED, true>), grid, dim3(512), 0, stream, a);
      else
        hipLaunchKernelGGL((decode_kernel<BK, BV, R, 4, BF, NCK, NCV, KSEQ, PAGED, true>), grid, dim3(256), 0, stream, a);
      return;
    }
  }
  if (plan.waves_per_wg == 8)
    hipLaunchKernelGGL((decode_kernel<BK, BV, R, 8, BF, NCK, NCV, KSEQ, PAGED>), grid, dim3(512), 0, stream, a);
  else
    hipLaunchKernelGGL((decode_kernel<BK, BV, R, 4, BF, NCK, NCV, KSEQ, PAGED>), grid, dim3(256), 0, stream, a);
}

// column sets: two only where 8 heads meet four groups (32 columns); quantized caches only
template <int BK, int BV, int R, bool BF, bool KSEQ, bool PAGED>
hipError_t launch_sets(const DecodeArgs& a, const DecodePlan& plan, dim3 grid, hipStream_t stream) {
  const bool k2 = R * a.g.ng_k > 16, v2 = R * a.g.ng_v > 16;
  if constexpr (R == 8 && BK != 16 && BV != 16) {
    if constexpr (KSEQ) {
      if (k2) return hipErrorInvalidValue;
      if (v2) launch_nw<BK, BV, R, BF, 1, 2, true, PAGED>(a, plan, grid, stream);
      else launch_nw<BK, BV, R, BF, 1, 1, true, PAGED>(a, plan, grid, stream);
    } else {
      if (k2 && v2) launch_nw<BK, BV, R, BF, 2, 2, false, PAGED>(a, plan, grid, stream);
      else if (k2) launch_nw<BK, BV, R, BF, 2, 1, false, PAGED>(a, plan, grid, stream);
      else if (v2) launch_nw<BK, BV, R, BF, 1, 2, false, PAGED>(a, plan, grid, stream);
      else launch_nw<BK, BV, R, BF, 1, 1, false, PAGED>(a, plan, grid, stream);
    }
  } else {
    if (k2 || v2) return hipErrorInvalidValue;
    launch_nw<BK, BV, R, BF, 1, 1, KSEQ, PAGED>(a, plan, grid, stream);
  }
  return hipGetLastError();
}

template <int BK, int BV, int R, bool BF = false, bool KSEQ = false>
hipError_t launch_one(const DecodeArgs& a, const DecodePlan& plan, hipStream_t stream) {
  dim3 grid(plan.n_splits, a.g.batch * a.g.kv_heads);
  hipError_t e;
  e = a.g.page_shift ? launch_sets<BK, BV, R, BF, KSEQ, true>(a, plan, grid, stream)
                     : launch_sets<BK, BV, R, BF, KSEQ, false>(a, plan, grid, stream);
  // the records of this launch are all there is: merge them, in the launch itself where that pays (merge_tag), else
  // here (otherwise the caller adds launches and merges)
  if (e != hipSuccess || a.rec_splits == 1 || a.rec_splits != plan.n_splits || a.merge_tag != 0) return e;
  launch_merge(a.ws, a.out, a.out_dtype, a.g.batch * a.q_heads, a.rec_splits, rot_v_of(a.g), stream);
  return hipGetLastError();
}

template <int BK, int BV, bool BF = false, bool KSEQ = false>
hipError_t launch_r(int R, const DecodeArgs& a, const DecodePlan& plan, hipStream_t stream) {
  switch (R) {
    case 1: return launch_one<BK, BV, 1, BF, KSEQ>(a, plan, stream);
    case 2: return launch_one<BK, BV, 2, BF, KSEQ>(a, plan, stream);
    case 4: return launch_one<BK, BV, 4, BF, KSEQ>(a, plan, stream);
    case 8: return launch_one<BK, BV, 8, BF, KSEQ>(a, plan, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace

#define KVQ_CAT2(a, b, c) a##b##_##c
#define KVQ_CAT(a, b, c) KVQ_CAT2(a, b, c)

#if defined(KVQ_INST_BK)
// ---- instance translation unit: the kernels of one (b_K, b_V) pair behind one launcher -------------------------------
hipError_t KVQ_CAT(launch_decode_inst_, KVQ_INST_BK, KVQ_INST_BV)(int R, const DecodeArgs& a, const DecodePlan& plan,
                                                                  hipStream_t stream) {
#if KVQ_INST_BK == 16 || KVQ_INST_BV == 16
  // one tensor or both unquantized: token-wise kernels only, typed by the 16-bit patterns' type
  return a.g.raw_dtype == KVQ_BF16 ? launch_r<KVQ_INST_BK, KVQ_INST_BV, true>(R, a, plan, stream)
                                   : launch_r<KVQ_INST_BK, KVQ_INST_BV, false>(R, a, plan, stream);
#else
  if (a.g.axis_k == KVQ_AXIS_SEQ) return launch_r<KVQ_INST_BK, KVQ_INST_BV, false, true>(R, a, plan, stream);
  return launch_r<KVQ_INST_BK, KVQ_INST_BV>(R, a, plan, stream);
#endif
}

#else
// ---- dispatcher translation unit ----------------------------------------------------------------------------------------
#ifndef KVQ_FOR_EACH_PAIR      // (a development build may name fewer pairs on the command line)
#define KVQ_FOR_EACH_PAIR(X) X(4, 2) X(2, 4) X(4, 4) X(8, 8) X(2, 2) X(8, 4) X(8, 2) X(4, 8) X(2, 8) X(16, 16) \
  X(3, 2) X(3, 4) X(3, 8) X(6, 2) X(6, 4) X(6, 8) X(1, 2) X(1, 4) X(1, 8) \
  X(1, 1) X(2, 1) X(3, 1) X(4, 1) X(6, 1) X(8, 1) \
  X(1, 3) X(2, 3) X(3, 3) X(4, 3) X(6, 3) X(8, 3) X(1, 6) X(2, 6) X(3, 6) X(4, 6) X(6, 6) X(8, 6) \
  X(16, 1) X(16, 2) X(16, 3) X(16, 4) X(16, 6) X(16, 8) X(1, 16) X(2, 16) X(3, 16) X(4, 16) X(6, 16) X(8, 16)
#endif
#define KVQ_DECL(BK_, BV_) \
  hipError_t KVQ_CAT(launch_decode_inst_, BK_, BV_)(int R, const DecodeArgs& a, const DecodePlan& plan, hipStream_t stream);
KVQ_FOR_EACH_PAIR(KVQ_DECL)
#undef KVQ_DECL

// Columns are laid out for a power-of-two number of heads per KV head.
int padded_heads(int r) { return r <= 1 ? 1 : r <= 2 ? 2 : r <= 4 ? 4 : 8; }

bool decode_supported(const Geom& g, int32_t q_heads) {
  const int r = q_heads / g.kv_heads;
  if (r < 1 || r > 8) return false;
  const int R = padded_heads(r);
  if (R * g.ng_k > 32 || R * g.ng_v > 32) return false;        // head x group columns: at most two 16-wide tiles
  if ((g.bits_k == 16) != (g.bits_v == 16)) {                  // one tensor unquantized, the other not:
    if (R * g.ng_k > 16 || R * g.ng_v > 16) return false;      // one column set, token-wise keys, values not rotated
    if (g.axis_k == KVQ_AXIS_SEQ || g.resid || g.rotate_v) return false;
  }
  return true;
}

// Compute units of the current device, asked once per device (a partitioned or binned part has fewer than the 256 of
// a whole MI355X).  Without a usable device (the host-only size queries on a machine with no GPU) the whole part's count.
int device_compute_units() {
  constexpr int kFull = 256, kMaxDevices = 64;
  static std::atomic<int> cached[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return kFull; }
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
      (void)hipGetLastError();
      n = kFull;
    }
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

namespace {
// Wavefronts per (b, h_kv) stream that fill the chip once, and what a sequence of n_steps steps can use of them.
struct WaveBudget { int waves, nw, splits; };
WaveBudget wave_budget(const Geom& g, int n_steps) {
  const int streams = g.batch * g.kv_heads;
  const int total_waves = device_compute_units() * 4 * KVQ_WAVES_PER_SIMD;
  int waves_per_stream = (total_waves + streams - 1) / streams;
  // at least two steps per wavefront (four or eight, i.e. fewer splits and at B=8, T=2048 the two-record merge inside
  // the launch instead of the merge launch, measure 13.7 and 14.6 us there against 11.9)
  const int max_waves = (n_steps + 1) / 2;
  if (waves_per_stream > max_waves) waves_per_stream = max_waves;
  if (waves_per_stream < 4) waves_per_stream = 4;
  const int nw = waves_per_stream >= 8 ? 8 : 4;
  int splits = waves_per_stream / nw;
  if (splits < 1) splits = 1;
  return WaveBudget{waves_per_stream, nw, splits};
}
int plan_steps(const Geom& g, int32_t seq_len) {
  return g.resid ? seq_len / g.resid * (g.resid / 32) : (seq_len + 31) / 32;      // (a residual buffer: the flushed tokens only)
}
}  // namespace

// Upper bound, over every length up to seq_len, of the partial records per (batch, query head) that one decode call
// writes (with a residual buffer: one per split of the flushed blocks plus one for the tail in the buffer): the number of splits
// before the steps are dealt out never shrinks as the sequence grows, and dealing them out in whole multiples of the
// workgroup's wavefronts only ever lowers it.  The workspace is sized for this bound, so a workspace sized once for the longest sequence serves every
// shorter one (the exact count is not monotone in the length).
int32_t decode_records_bound(const Geom& g, int32_t seq_len) {
  const int n_steps = plan_steps(g, seq_len);
  if (n_steps == 0) return 1;
  const int splits = wave_budget(g, n_steps).splits;
  return g.resid ? splits + 1 : splits;
}

DecodePlan plan_decode(const Geom& g, int32_t seq_len) {
  // Fill the chip exactly once: compute units x 4 SIMDs x KVQ_WAVES_PER_SIMD wavefronts, spread over the (b,h) streams.
  // Workgroups of 8 wavefronts halve the number of sequence splits (none at all from 256 streams up, where the
  // merge kernel and the workspace traffic disappear); each wavefront should still own a few steps.
  // Channel-wise keys: the plan covers the flushed tokens only (whole 64-token blocks, two steps each, taken in pairs);
  // n_splits = 0 when nothing is flushed yet.  The residual tail is a launch of its own.
  const int unit = g.axis_k == KVQ_AXIS_SEQ ? 2 : 1;
  const int n_steps = plan_steps(g, seq_len);
  if (n_steps == 0) return DecodePlan{0, 0, 4};
  const WaveBudget wb = wave_budget(g, n_steps);
  const int nw = wb.nw;
  int sps = (n_steps + wb.splits - 1) / wb.splits;
  sps = (sps + nw * unit - 1) / (nw * unit) * (nw * unit);
  const int splits = (n_steps + sps - 1) / sps;
  return DecodePlan{splits, sps, nw};
}

// A number that tells one launch's count of finished workgroups from whatever the counter word held before (48 bits,
// never 0).  A replayed graph launch carries the same number again: the last workgroup of a launch leaves the count at 0.
static unsigned long long next_merge_tag() {
  static std::atomic<unsigned long long> counter{0x9E3779B97F4Aull};
  unsigned long long t;
  do { t = counter.fetch_add(0x632BE59BD9B5ull, std::memory_order_relaxed) & 0xFFFFFFFFFFFFull; } while (t == 0);
  return t;
}

// Where the launch's own workgroups merge the records (two splits: the shapes that are bound by their launches; the 1 MiB
// cache of one sequence of 8 heads and 1024 tokens steps in 11.5 us this way and in 15.7 us with the merge kernel).  With
// four records and more the merge kernel is the faster way: the device-scope accesses of the counting and of reading
// the records back cost the last workgroup two trips to memory of 1.5 to 2 us each, as many as the second kernel
// needs, on top of slower record stores (measured: 22.4 against 20.9 us on the 8B layer's four splits, 64 against 30 us
// with 32 splits, where the workgroups' increments of one counter also queue up behind each other).
static unsigned long long merge_tag_for(int records) { return records == 2 ? next_merge_tag() : 0ull; }

hipError_t launch_decode_attention(const Geom& g, const kvq_cache& c, const void* q, int q_dtype, int32_t q_heads,
                                   int32_t seq_len, float softmax_scale, void* out, int out_dtype, float* workspace,
                                   const DecodePlan& plan, const AppendOne* app, hipStream_t stream,
                                   const int32_t* seq_lens, int32_t lens_offset) {
  const int R = padded_heads(q_heads / g.kv_heads);
  DecodeArgs a{};
  a.heads_per_kv = q_heads / g.kv_heads;
  a.seq_lens = seq_lens; a.lens_offset = lens_offset;
  a.g = g; a.cache = c;
  a.q = (const uint16_t*)q; a.q_bf16 = q_dtype == KVQ_BF16 ? 1 : 0; a.q_heads = q_heads;
  a.seq_len = seq_len; a.softmax_scale = softmax_scale;
  a.ws = workspace; a.out = out; a.out_dtype = out_dtype;
  a.n_splits = plan.n_splits; a.steps_per_split = plan.steps_per_split;
  a.rec_splits = plan.n_splits; a.rec_base = 0;
  a.merge_tag = 0;
  if (g.resid) {
    // a residual buffer: flushed blocks from the codes (plan; channel-wise or token-wise keys), the newest tokens from
    // the buffer by the unquantized kernel, all partial records merged at the end
    // (per-sequence lengths: seq_len is their bound; every sequence's own flushed part and tail are cut out on the
    // device, the tail launch always runs, and a sequence without one of the parts gets empty records for it)
    const bool varlen = seq_lens != nullptr;
    const int32_t RL = g.resid;
    const int32_t n_flushed = seq_len / RL * RL;
    const int32_t tail = varlen ? (n_flushed ? RL - 1 : seq_len) : seq_len - n_flushed;
    const int32_t records = plan.n_splits + (tail ? 1 : 0);
    // one split of flushed blocks and a tail: the tail's launch, which comes second, takes the first one's record in and
    // writes the result (one launch less than with the merge kernel)
    const bool tail_merges = n_flushed && tail && plan.n_splits == 1;
    a.lens_bound = seq_len; a.lens_block = RL;
    hipError_t e = hipSuccess;
    if (n_flushed) {
      a.seq_len = n_flushed; a.rec_splits = records; a.rec_base = 0; a.lens_mode = 1;
      a.merge_tag = !tail ? merge_tag_for(records) : 0;     // (a launch that writes every record may merge them itself)
#define KVQ_CASE(BK_, BV_) \
      if (g.bits_k == BK_ && g.bits_v == BV_) e = KVQ_CAT(launch_decode_inst_, BK_, BV_)(R, a, plan, stream);
      KVQ_FOR_EACH_PAIR(KVQ_CASE)
#undef KVQ_CASE
      if (e != hipSuccess) return e;
    }
    if (tail) {
      DecodeArgs t = a;
      t.merge_tag = 0;
      t.g.axis_k = KVQ_AXIS_HEAD_DIM; t.g.bits_k = t.g.bits_v = 16; t.g.g_k = t.g.g_v = kHeadDim; t.g.ng_k = t.g.ng_v = 1;
      t.g.rotate_k = 0;                                    // (the buffer holds the input rows: their scores take q itself)
      t.g.resid = 0; t.g.seq_g = 0;
      t.g.t_cap = RL; t.g.page_shift = 0; t.cache.page_table = nullptr;     // (the buffers are per sequence, never paged)
      t.g.kc_stream = t.g.vc_stream = (int64_t)RL * kHeadDim * 2; t.g.km_stream = t.g.vm_stream = 0;
      t.cache.k_codes = c.k_resid; t.cache.v_codes = c.v_resid; t.cache.k_meta = t.cache.v_meta = nullptr;
      t.seq_len = tail; t.n_splits = 1; t.steps_per_split = 4; t.lens_mode = 2;
      t.rec_splits = records; t.rec_base = records - 1;
      if (tail_merges) { t.rec_splits = 1; t.rec_base = 0; t.extra_splits = records; }
      e = launch_decode_inst_16_16(R, t, DecodePlan{1, 4, 4}, stream);
      if (e != hipSuccess) return e;
    }
    if (records > 1 && !(n_flushed && !tail) && !tail_merges) {     // (a launch that wrote all the records has merged them itself)
      launch_merge(workspace, out, out_dtype, g.batch * q_heads, records, rot_v_of(g), stream);
      e = hipGetLastError();
    }
    return e;
  }
  a.lens_mode = 0; a.lens_bound = seq_len; a.lens_block = 1;
  a.merge_tag = merge_tag_for(a.rec_splits);
  if (app) {
    a.k_new = (const uint16_t*)app->k_new; a.v_new = (const uint16_t*)app->v_new;
    a.in_bf16 = app->in_dtype == KVQ_BF16 ? 1 : 0; a.nsb = app->stride_b; a.nsh = app->stride_h;
  }
#define KVQ_CASE(BK_, BV_) \
  if (g.bits_k == BK_ && g.bits_v == BV_) return KVQ_CAT(launch_decode_inst_, BK_, BV_)(R, a, plan, stream);
  KVQ_FOR_EACH_PAIR(KVQ_CASE)
#undef KVQ_CASE
  return hipErrorInvalidValue;
}
#endif

}  // namespace kvq
