// Quantize-append (token-wise groups; channel-wise key groups with their residual buffer), dequantize and
// reconstruction-error kernels (gfx950).
//
// The quantizer is the b-bit uniform scalar quantizer of App. B ("Preliminaries": scale factor,
// round, clip, reconstruct) of arXiv 2502.15075 in its group-wise asymmetric min-max form; the
// exact arithmetic is stated in kvq.h.  Codes and scale/zero bytes must be identical on every
// machine, so this file is compiled with floating-point contraction off and every operation
// below is a single IEEE binary32 operation (hipcc's default division is correctly rounded).
#include "kvq_internal.h"
#include "kvq_quantizer.h"

namespace kvq {
namespace {

constexpr int kSpan = 64;                // tokens one workgroup covers (two 32-token value blocks)

// LDS staging of the value codes of one span, already in storage order: one element per code, the F = 32/b_V codes
// of an output word adjacent (so a word is assembled from one wide LDS read).  (Padding the area against the bank
// conflicts of the strided byte writes was measured: its address arithmetic costs more than the conflicts, 3 %.)

// Pack the codes held one per byte in w (first code in the lowest byte) into adjacent b-bit fields.
// (Bytes of tokens that were not staged hold garbage: they are masked to b bits so that they stay inside their field.)
// 16 bytes read once / written once: streaming accesses (see store_bytes)
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
  const u32x4v v = __builtin_nontemporal_load(reinterpret_cast<const u32x4v*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream16(void* p, uint4 w) {
  typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
  u32x4v v; v.x = w.x; v.y = w.y; v.z = w.z; v.w = w.w;
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4v*>(p));
}

template <int B> __device__ __forceinline__ uint32_t pack_bytes(uint32_t w) {
  if (B == 1) { w &= 0x01010101u; return (w | (w >> 7) | (w >> 14) | (w >> 21)) & 0xFu; }
  if (B == 2) { w &= 0x03030303u; return (w | (w >> 6) | (w >> 12) | (w >> 18)) & 0xFFu; }
  if (B == 4) return (w & 0xFu) | ((w >> 4) & 0xF0u) | ((w >> 8) & 0xF00u) | ((w >> 12) & 0xF000u);
  return w;
}

// Token row (0..63 of the span) -> (block, word family, field): the codes of the 8 channels d0..d0+7 of this lane go
// to 8 words one lane piece (LW = 4 words, 2 for 1-bit codes) apart; they are staged in LDS in storage order, one
// element per code.
template <int BV>
__device__ __forceinline__ void stage_value_codes(uint8_t* vstage, int row, int d0, const uint32_t codes[8]) {
  constexpr int F = 32 / BV, P = 16 / BV, ES = BV == 16 ? 2 : 1, LW = BV == 1 ? 2 : 4;
  const int sub = row >> 5, u = row & 31;
  const int j = (u >> 2) & 3, i = 4 * (u >> 4) + (u & 3);
  const int x = i & 1, v = i >> 1;
  const int q = 4 * (d0 >> 4) + v;
  const int e_idx = q / P, p = q % P;
  const int word0 = sub * (128 * BV) + (BV == 1 ? 0 : (e_idx >> 2) * 256) + (16 * j + (d0 & 15)) * LW + (e_idx & (LW - 1));
  const int a0 = (word0 * F + x * P + p) * ES;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int a = a0 + e * LW * F * ES;
    if (BV == 16) *reinterpret_cast<uint16_t*>(vstage + a) = (uint16_t)codes[e];
    else vstage[a] = (uint8_t)codes[e];
  }
}

// One thread per 32-bit word of the span (two blocks of 128*BV words, BW words apart in the plane: a block of 3- or
// 6-bit codes is a block of low parts followed by a block of high parts): assemble the word from the staged codes and
// store it; when the span is only partly covered by the new tokens [lo, hi), keep the fields of the other tokens.
template <int BV, int BW = 128 * BV, int SPAN = kSpan, bool NT = false>
__device__ __forceinline__ void store_value_words(uint32_t* vcp, const uint8_t* vstage, int tid, int lo, int hi) {
  constexpr int F = 32 / BV, P = 16 / BV, ES = BV == 16 ? 2 : 1;
  const bool full = lo == 0 && hi == SPAN;
  for (int w = tid; w < (SPAN / 32) * 128 * BV; w += 256) {
    uint32_t* vc = vcp + (w / (128 * BV)) * (BW - 128 * BV);      // vc[w]: the word's place in the plane
    const uint8_t* sp = vstage + w * F * ES;
    uint32_t bits;
    if (BV == 1) {
      const uint4 r0 = *reinterpret_cast<const uint4*>(sp), r1 = *reinterpret_cast<const uint4*>(sp + 16);
      bits = pack_bytes<1>(r0.x) | (pack_bytes<1>(r0.y) << 4) | (pack_bytes<1>(r0.z) << 8) | (pack_bytes<1>(r0.w) << 12) |
             (pack_bytes<1>(r1.x) << 16) | (pack_bytes<1>(r1.y) << 20) | (pack_bytes<1>(r1.z) << 24) | (pack_bytes<1>(r1.w) << 28);
    } else if (BV == 2) {
      const uint4 r = *reinterpret_cast<const uint4*>(sp);
      bits = pack_bytes<2>(r.x) | (pack_bytes<2>(r.y) << 8) | (pack_bytes<2>(r.z) << 16) | (pack_bytes<2>(r.w) << 24);
    } else if (BV == 4) {
      const uint2 r = *reinterpret_cast<const uint2*>(sp);
      bits = pack_bytes<4>(r.x) | (pack_bytes<4>(r.y) << 16);
    } else {
      bits = *reinterpret_cast<const uint32_t*>(sp);            // 8-bit: four codes; 16-bit: two patterns
    }
    if (full) {
      if (NT) __builtin_nontemporal_store(bits, vc + w); else vc[w] = bits;
      continue;
    }
    // partially covered span: keep the fields of tokens outside [lo, hi)
    const int sub = w / (128 * BV), wi = w % (128 * BV);
    const int piece = wi >> 8, rem = wi & 255;
    const int L = BV == 1 ? wi >> 1 : rem >> 2, m = BV == 1 ? wi & 1 : rem & 3;
    const int e_idx = 4 * piece + m;
    const int j = L >> 4;
    const uint32_t fmask = BV == 16 ? 0xFFFFu : ((1u << BV) - 1u);
    uint32_t mask = 0;
    for (int x = 0; x < 2; ++x)
      for (int p = 0; p < P; ++p) {
        const int q = e_idx * P + p;
        const int v = q & 3;
        const int i = 2 * v + x;
        const int tt = 32 * sub + 16 * (i >> 2) + 4 * j + (i & 3);
        if (tt >= lo && tt < hi) mask |= fmask << (16 * x + BV * p);
      }
    if (mask == 0) continue;
    vc[w] = (bits & mask) | (vc[w] & ~mask);
  }
}

// Bytes of LDS that stage the codes of one span: one staging area per part of a code (3- and 6-bit value codes are a
// low part and a high part, each packed into a block of its own).
template <int BV, int SPAN = kSpan> constexpr int stage_area() { return SPAN * kHeadDim * (BV == 16 ? 2 : 1); }
template <int BV, int SPAN = kSpan> constexpr int stage_total() { return stage_area<BV, SPAN>() * (code_hi_bits<BV>() ? 2 : 1); }

template <int BV, int SPAN = kSpan>
__device__ __forceinline__ void stage_value_row(uint8_t* vstage, int row, int d0, const uint32_t codes[8]) {
  constexpr int VLO = code_lo_bits<BV>(), VHI = code_hi_bits<BV>();
  if constexpr (VHI == 0) {
    stage_value_codes<BV>(vstage, row, d0, codes);
  } else {                                         // (the low parts are cut to their field when the words are packed)
    uint32_t high[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) high[e] = codes[e] >> VLO;
    stage_value_codes<VLO>(vstage, row, d0, codes);
    stage_value_codes<VHI>(vstage + stage_area<BV, SPAN>(), row, d0, high);
  }
}

// vc: the span's first block in the plane
template <int BV, int SPAN = kSpan, bool NT = false>
__device__ __forceinline__ void store_value_span(uint32_t* vc, const uint8_t* vstage, int tid, int lo, int hi) {
  constexpr int VLO = code_lo_bits<BV>(), VHI = code_hi_bits<BV>();
  if constexpr (VHI == 0) {
    store_value_words<BV, 128 * BV, SPAN, NT>(vc, vstage, tid, lo, hi);
  } else {
    store_value_words<VLO, 128 * BV, SPAN, NT>(vc, vstage, tid, lo, hi);
    store_value_words<VHI, 128 * BV, SPAN, NT>(vc + 128 * VLO, vstage + stage_area<BV, SPAN>(), tid, lo, hi);
  }
}

// One workgroup = `chain` consecutive spans of SPAN tokens (a multiple of 32: whole blocks of value codes) of one (b,h)
// stream, restricted to the new tokens in them.  The rows of the next span are loaded before the current one is
// quantized, so that a workgroup has loads in flight while it computes (with one span per workgroup the kernel waits on
// memory latency: 8 workgroups per compute unit do not keep enough bytes in flight on their own).  No load is
// conditional -- rows outside the new tokens re-read a row inside them, and the load "after the last span" is
// collapsed onto 16 bytes -- so that the compiler can count the loads in flight behind the ones it waits for (the last
// span peeled out of the loop instead, with nothing loaded behind it, costs 20 registers and 7 % of the rate).
template <int BK, int BV, bool BF, int SPAN>
__global__ __launch_bounds__(256) void quantize_append_kernel(Geom g, kvq_cache c, const uint16_t* __restrict__ k_new,
                                                              const uint16_t* __restrict__ v_new, int64_t sb, int64_t sh,
                                                              int64_t st, int32_t pos, int32_t n_new, int32_t chain) {
  constexpr int kSpan = SPAN;                      // (shadows the 64-token span of the other kernels in this file)
  constexpr int NR = SPAN / 16;                    // rows per thread and span
  __shared__ __attribute__((aligned(16))) uint8_t vstage[stage_total<BV, SPAN>()];
  const int tid = threadIdx.x;
  const int bh = blockIdx.y;
  const int b = bh / g.kv_heads, h = bh % g.kv_heads;
  const int lane16 = tid & 15;
  const int d0 = lane16 * 8;
  const int lpg_k = g.g_k >> 3, lpg_v = g.g_v >> 3;                  // lanes per group
  const int km_step = 16 * g.ng_k, vm_step = 16 * g.ng_v;
  const int blk_first = pos / kSpan + blockIdx.x * chain;
  const int blk_end = min(blk_first + chain, (pos + n_new - 1) / kSpan + 1);     // (the grid leaves no workgroup empty)
  const int64_t in_base = (int64_t)b * sb + (int64_t)h * sh;

  // the rows (tid/16) + 16*it of span blk; `live` = 0 collapses all loads onto the first 16 bytes of the span's first
  // new row
  auto load_span = [&](int blk, uint32_t live, uint4 (&kraw)[NR], uint4 (&vraw)[NR]) {
    const int lo = max(pos, blk * kSpan) - blk * kSpan;
    const int hi = min(pos + n_new, (blk + 1) * kSpan) - blk * kSpan;
#pragma unroll
    for (int it = 0; it < NR; ++it) {
      const int row = min(max((tid >> 4) + 16 * it, lo), hi - 1);
      const int64_t first_row = (int64_t)blk * kSpan + lo - pos;
      const int64_t src = in_base + first_row * st + (((int64_t)(row - lo) * st + d0) & (int64_t)(int32_t)live);
      kraw[it] = load_stream16(k_new + src);       // (streaming: the input rows are read once)
      vraw[it] = load_stream16(v_new + src);
    }
  };

  uint4 kraw[NR], vraw[NR], knext[NR], vnext[NR];
  load_span(blk_first, ~0u, kraw, vraw);
  for (int blk = blk_first; blk < blk_end; ++blk) {
    const bool more = blk + 1 < blk_end;           // uniform
    load_span(more ? blk + 1 : blk, more ? ~0u : 0u, knext, vnext);
    const int lo = max(pos, blk * kSpan) - blk * kSpan;
    const int hi = min(pos + n_new, (blk + 1) * kSpan) - blk * kSpan;
    // rows of all four planes are addressed by the span's first token in plane order (a span never straddles a page)
    const int64_t tv0 = virtual_token(g, c.page_table, b, h, (int64_t)blk * kSpan);
    uint32_t* vc = (uint32_t*)c.v_codes + (tv0 >> 5) * (128 * BV);
    // tv0 is a multiple of 32 (of the page size when paged), so row (tid/16) + 16*it sits at position tid/16 of the
    // span's it-th slab of 16 tokens in the scale/zero planes: one address per thread, a uniform stride per it
    uint8_t* kc = (uint8_t*)c.k_codes + (tv0 + (tid >> 4)) * (BK == 16 ? 256 : 16 * BK);
    uint32_t* km = (uint32_t*)c.k_meta + meta_index(tv0 + (tid >> 4), lane16 >> lpg_shift(lpg_k), g.ng_k);
    uint32_t* vm = (uint32_t*)c.v_meta + meta_index(tv0 + (tid >> 4), lane16 >> lpg_shift(lpg_v), g.ng_v);
#pragma unroll
    for (int it = 0; it < NR; ++it) {
      const int row = (tid >> 4) + 16 * it;
      if (row < lo || row >= hi) continue;         // whole 16-lane rows take the same branch
      // ---- keys: row-major codes
      {
        const uint4 raw = kraw[it];
        const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
        if (BK == 16) {
          store_stream16(kc + it * (16 * 256) + d0 * 2, raw);
        } else {
          float x[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), BF);
          if (g.rotate_k) rotate8(x, lane16, rot_sign_bits(g.signs_k, lane16));   // whole 16-lane rows are here together
          uint32_t codes[8];
          uint16_t S, Z;
          quantize8(x, BK, lpg_k, codes, &S, &Z);
          if ((lane16 & (lpg_k - 1)) == 0) __builtin_nontemporal_store((uint32_t)S | ((uint32_t)Z << 16), km + it * km_step);
          store_key_codes<BK, true>(kc + it * (16 * 16 * BK), lane16, codes);
        }
      }
      // ---- values: scale/zero straight to memory, codes to their place in the staged words
      {
        const uint4 raw = vraw[it];
        const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
        uint32_t codes[8];
        if (BV == 16) {
#pragma unroll
          for (int e = 0; e < 8; ++e) codes[e] = (rw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
        } else {
          float x[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), BF);
          if (g.rotate_v) rotate8(x, lane16, rot_sign_bits(g.signs_v, lane16));
          uint16_t S, Z;
          quantize8(x, BV, lpg_v, codes, &S, &Z);
          if ((lane16 & (lpg_v - 1)) == 0) {
            __builtin_nontemporal_store((uint32_t)S | ((uint32_t)Z << 16), vm + it * vm_step);
            note_value_scale(c.v_scale_exp + bh, S);
          }
        }
        stage_value_row<BV, SPAN>(vstage, row, d0, codes);
      }
    }
    __syncthreads();
    store_value_span<BV, SPAN, true>(vc, vstage, tid, lo, hi);
    if (more) __syncthreads();                     // (the staging area is reused by the next span)
#pragma unroll
    for (int it = 0; it < NR; ++it) { kraw[it] = knext[it]; vraw[it] = vnext[it]; }
  }
}

// The 8 fields of channels d0 .. d0+7 (d0 a multiple of 8) of token u in a 32-token block of B-bit fields: the same
// field of 8 words one lane piece (16 bytes, 8 for 1-bit fields) apart.
template <int B> __device__ __forceinline__ void block_fields8(const uint8_t* blkp, int u, int d0, uint32_t code[8]) {
  int dw, bit;
  v_field(u, d0, B, &dw, &bit);
  const uint32_t* blk = reinterpret_cast<const uint32_t*>(blkp) + dw;
#pragma unroll
  for (int e = 0; e < 8; ++e) code[e] = (blk[(B == 1 ? 2 : 4) * e] >> bit) & (B == 16 ? 0xFFFFu : ((1u << B) - 1u));
}
// The 8 codes of channels d0 .. d0+7 of value row t (3- and 6-bit codes: low parts from the block's first part, high
// parts from its second).
template <int B> __device__ __forceinline__ void value_codes8(const uint8_t* cs, int64_t t, int d0, uint32_t code[8]) {
  constexpr int LO = code_lo_bits<B>(), HI = code_hi_bits<B>();
  const uint8_t* blk = cs + (t >> 5) * (int64_t)(512 * B);
  block_fields8<LO>(blk, (int)(t & 31), d0, code);
  if constexpr (HI != 0) {
    uint32_t high[8];
    block_fields8<HI>(blk + 512 * LO, (int)(t & 31), d0, high);
#pragma unroll
    for (int e = 0; e < 8; ++e) code[e] |= high[e] << LO;
  }
}

// Channel-wise keys (Sec. 4 "Downstream Task Accuracy": the per-column back-end with its residual buffer).
// One workgroup = one block of RLT tokens (the residual buffer's length: 64 or 128) of one (b,h) stream, restricted to
// the new tokens [lo, hi) in it.  New tokens that no later token of this call overwrites go to their residual slot as
// 16-bit patterns.  A block that this call completes is flushed: rows below lo come back from the residual buffer (the
// launcher makes sure that no other workgroup of the same launch writes there), keys are quantized channel by channel
// (a group is g.seq_g = 32, 64 or 128 consecutive tokens of one channel, RLT / g.seq_g groups per channel and block),
// values token-wise exactly as in quantize_append_kernel.
// KTOK: the keys of a flushed block are quantized row by row like the values (a residual buffer in front of token-wise
// keys); otherwise channel by channel.
template <int BK, int BV, bool BF, bool KTOK, int RLT>
__global__ __launch_bounds__(256) void seq_append_kernel(Geom g, kvq_cache c, const uint16_t* __restrict__ k_new,
                                                         const uint16_t* __restrict__ v_new, int64_t sb, int64_t sh,
                                                         int64_t st, int32_t pos, int32_t n_new,
                                                         const int32_t* __restrict__ pos_arr, int32_t max_pos) {
  static_assert(RLT % kSpan == 0, "a flushed block is a whole number of value spans");
  constexpr int NIT = RLT / 16;                            // rows per thread: rg, rg + 16, ...
  constexpr int NGR = RLT / 32;                            // the most key groups a block can hold
  __shared__ __attribute__((aligned(16))) uint8_t vstage[stage_total<BV>()];
  __shared__ float s_mn[KTOK ? 1 : NGR][4][kHeadDim], s_mx[KTOK ? 1 : NGR][4][kHeadDim];
  const int tid = threadIdx.x;
  const int bh = blockIdx.y;
  const int b = bh / g.kv_heads, h = bh % g.kv_heads;
  if (pos_arr) pos = min(max(pos_arr[b], 0), max_pos);     // one token per sequence at its own position (n_new == 1)
  const int blk = pos / RLT + blockIdx.x;
  const int lo = max(pos, blk * RLT) - blk * RLT;
  const int hi = min(pos + n_new, (blk + 1) * RLT) - blk * RLT;
  const bool complete = hi == RLT;                         // this call brings the block's last token
  const int lane16 = tid & 15, rg = tid >> 4;
  const int d0 = lane16 * 8;
  uint8_t* kr = (uint8_t*)c.k_resid + (int64_t)bh * (RLT * kHeadDim * 2);
  uint8_t* vr = (uint8_t*)c.v_resid + (int64_t)bh * (RLT * kHeadDim * 2);

  uint4 kraw[NIT], vraw[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int row = rg + 16 * it;
    const int64_t t = (int64_t)blk * RLT + row;
    if (row >= lo && row < hi) {
      const int64_t src = (int64_t)b * sb + (int64_t)h * sh + (t - pos) * st + d0;
      kraw[it] = *reinterpret_cast<const uint4*>(k_new + src);
      vraw[it] = *reinterpret_cast<const uint4*>(v_new + src);
      if (t + RLT >= (int64_t)pos + n_new) {               // the last token of this call that lands in slot `row`
        *reinterpret_cast<uint4*>(kr + row * (kHeadDim * 2) + d0 * 2) = kraw[it];
        const uint32_t rw[4] = {vraw[it].x, vraw[it].y, vraw[it].z, vraw[it].w};
        int dw, bit;
        v_field(row & 31, d0, 16, &dw, &bit);
        uint16_t* blk16 = reinterpret_cast<uint16_t*>(vr + (row >> 5) * (512 * 16));
#pragma unroll
        for (int e = 0; e < 8; ++e) blk16[(dw + 4 * e) * 2 + (bit >> 4)] = (uint16_t)(rw[e >> 1] >> (16 * (e & 1)));
      }
    } else if (complete && row < lo) {                     // older tokens of the block being flushed
      kraw[it] = *reinterpret_cast<const uint4*>(kr + row * (kHeadDim * 2) + d0 * 2);
      uint32_t code[8];
      value_codes8<16>(vr, row, d0, code);
      vraw[it] = make_uint4(code[0] | (code[1] << 16), code[2] | (code[3] << 16), code[4] | (code[5] << 16),
                            code[6] | (code[7] << 16));
    }
  }
  if (!complete) return;                                   // uniform over the workgroup

  // rows of all four planes are addressed by the block's first token in plane order (a block never straddles a page)
  const int64_t tv0 = virtual_token(g, c.page_table, b, h, (int64_t)blk * RLT);
  uint8_t* kc = (uint8_t*)c.k_codes;
  uint32_t* km_tok = (uint32_t*)c.k_meta;                                  // token-wise keys: entries by token and group
  uint32_t* vm = (uint32_t*)c.v_meta;

  if constexpr (KTOK) {
    // ---- keys token-wise: every row on its own, exactly as quantize_append_kernel does it
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int64_t t = tv0 + rg + 16 * it;
      const uint32_t rw[4] = {kraw[it].x, kraw[it].y, kraw[it].z, kraw[it].w};
      float xk[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) xk[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), BF);
      if (g.rotate_k) rotate8(xk, lane16, rot_sign_bits(g.signs_k, lane16));
      uint32_t kcodes[8];
      uint16_t S, Z;
      const int lpg = g.g_k >> 3;
      quantize8(xk, BK, lpg, kcodes, &S, &Z);
      if ((lane16 & (lpg - 1)) == 0) km_tok[meta_index(t, lane16 >> lpg_shift(lpg), g.ng_k)] = (uint32_t)S | ((uint32_t)Z << 16);
      store_key_codes<BK>(kc + t * (16 * BK), lane16, kcodes);
    }
  } else {
    // ---- keys: minimum and maximum of every channel over the rows of each group.  A thread's rows rg + 16 it fall
    // into group it / gi (gi = seq_g / 16 of its rows in a row per group); within a group: this thread's rows, the 4 row
    // groups of its wavefront by two shuffles, the 4 wavefronts through LDS.
    const int gi = g.seq_g >> 4;                           // 2, 4 or 8 (uniform)
    uint32_t* km = (uint32_t*)c.k_meta + (tv0 / g.seq_g) * kHeadDim;       // the block's first group: 128 entries each
    float x[NIT][8];
    float mn[8], mx[8];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const uint32_t rw[4] = {kraw[it].x, kraw[it].y, kraw[it].z, kraw[it].w};
#pragma unroll
      for (int e = 0; e < 8; ++e) x[it][e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), BF);
      // rotated keys: the block's rows are quantized as R k (the buffer keeps the input rows; the 16 lanes of a row are
      // neighbours in one wavefront, and the whole workgroup is here)
      if (g.rotate_k) rotate8(x[it], lane16, rot_sign_bits(g.signs_k, lane16));
      const bool first = (it & (gi - 1)) == 0, last = ((it + 1) & (gi - 1)) == 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        mn[e] = first ? x[it][e] : fminf(mn[e], x[it][e]);
        mx[e] = first ? x[it][e] : fmaxf(mx[e], x[it][e]);
      }
      if (last) {                                          // (uniform)
        const int grp = it / gi;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float lo_e = fminf(mn[e], __shfl_xor(mn[e], 16)); lo_e = fminf(lo_e, __shfl_xor(lo_e, 32));
          float hi_e = fmaxf(mx[e], __shfl_xor(mx[e], 16)); hi_e = fmaxf(hi_e, __shfl_xor(hi_e, 32));
          if ((rg & 3) == 0) { s_mn[grp][tid >> 6][d0 + e] = lo_e; s_mx[grp][tid >> 6][d0 + e] = hi_e; }
        }
      }
    }
    __syncthreads();
    const float levels = (float)((1 << BK) - 1);
    const int n_grp = RLT / g.seq_g;
    for (int grp = 0; grp < n_grp; ++grp) {
      float sc[8], z[8], rcp[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float lo_v = fminf(fminf(s_mn[grp][0][d0 + e], s_mn[grp][1][d0 + e]), fminf(s_mn[grp][2][d0 + e], s_mn[grp][3][d0 + e]));
        const float hi_v = fmaxf(fmaxf(s_mx[grp][0][d0 + e], s_mx[grp][1][d0 + e]), fmaxf(s_mx[grp][2][d0 + e], s_mx[grp][3][d0 + e]));
        uint16_t S, Z;
        group_scale_zero(lo_v, hi_v, BK, &S, &Z);
        if (rg == 0) km[grp * kHeadDim + d0 + e] = (uint32_t)S | ((uint32_t)Z << 16);
        sc[e] = widen16(S, false); z[e] = widen16(Z, false);
        rcp[e] = sc[e] == 0.0f ? 0.0f : rcp_scale(sc[e]);    // (unused when the scale is 0)
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        if (it / gi != grp) continue;                      // (uniform)
        uint32_t codes[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) codes[e] = group_code(x[it][e], sc[e], z[e], rcp[e], levels);
        store_key_codes<BK>(kc + (tv0 + rg + 16 * it) * (16 * BK), lane16, codes);
      }
    }
  }

  // ---- values: token-wise, as in quantize_append_kernel for a full span, one span of kSpan tokens after the other
#pragma unroll
  for (int sp = 0; sp < RLT / kSpan; ++sp) {
    if (sp) __syncthreads();                               // (the staging area is reused)
#pragma unroll
    for (int k = 0; k < kSpan / 16; ++k) {
      const int it = sp * (kSpan / 16) + k;
      const int row = rg + 16 * k;                         // row inside the span
      const int64_t t = tv0 + sp * kSpan + row;
      const uint32_t rw[4] = {vraw[it].x, vraw[it].y, vraw[it].z, vraw[it].w};
      float xv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) xv[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), BF);
      uint32_t vcodes[8];
      uint16_t S, Z;
      const int lpg = g.g_v >> 3;
      quantize8(xv, BV, lpg, vcodes, &S, &Z);
      if ((lane16 & (lpg - 1)) == 0) {
        vm[meta_index(t, lane16 >> lpg_shift(lpg), g.ng_v)] = (uint32_t)S | ((uint32_t)Z << 16);
        note_value_scale(c.v_scale_exp + bh, S);
      }
      stage_value_row<BV>(vstage, row, d0, vcodes);
    }
    __syncthreads();
    store_value_span<BV>((uint32_t*)c.v_codes + ((tv0 + sp * kSpan) >> 5) * (128 * BV), vstage, tid, 0, kSpan);
  }
}

// Reconstruction x^ = code * scale + zero of 8 consecutive channels d0..d0+7 (d0 a multiple of 8) of the token with
// number t in plane order (virtual_token: contiguous and paged planes alike), as binary32 values; a 16-bit plane is
// widened exactly.  B: what a code takes in its plane (compile time); IS_V: values, else keys.
template <int B, bool IS_V>
__device__ __forceinline__ void reconstruct8_t(const Geom& g, const kvq_cache& c, int64_t t, int d0, float val[8]) {
  uint32_t code[8];
  if constexpr (IS_V) value_codes8<B>((const uint8_t*)c.v_codes, t, d0, code);
  else load_key_codes<B>((const uint8_t*)c.k_codes + t * (16 * B), d0 >> 3, code);
  if constexpr (B == 16) {
    const bool raw_bf16 = g.raw_dtype == KVQ_BF16;
#pragma unroll
    for (int e = 0; e < 8; ++e) val[e] = widen16((uint16_t)code[e], raw_bf16);
  } else {
    const uint32_t* ms = (const uint32_t*)(IS_V ? c.v_meta : c.k_meta);
    if (!IS_V && g.axis_k == KVQ_AXIS_SEQ) {       // channel-wise keys: one scale/zero per channel and group of seq_g tokens
      const uint4* mp = reinterpret_cast<const uint4*>(ms + (t / g.seq_g) * kHeadDim + d0);
      const uint4 m0 = mp[0], m1 = mp[1];
      const uint32_t mm[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e)
        val[e] = (float)code[e] * widen16((uint16_t)(mm[e] & 0xFFFF), false) + widen16((uint16_t)(mm[e] >> 16), false);
      return;
    }
    const int G = IS_V ? g.g_v : g.g_k, ng = IS_V ? g.ng_v : g.ng_k;
    const uint32_t m = ms[meta_index(t, d0 / G, ng)];
    const float s = widen16((uint16_t)(m & 0xFFFF), false);
    const float z = widen16((uint16_t)(m >> 16), false);
#pragma unroll
    for (int e = 0; e < 8; ++e) val[e] = (float)code[e] * s + z;
  }
}

// The same with the widths read from the geometry (the dequantize kernel: one token per thread, no loop to specialize).
__device__ __forceinline__ void reconstruct8(const Geom& g, const kvq_cache& c, int which, int64_t t, int d0, float val[8]) {
  if (which) {
    switch (g.bits_v) {
      case 1: return reconstruct8_t<1, true>(g, c, t, d0, val);
      case 2: return reconstruct8_t<2, true>(g, c, t, d0, val);
      case 3: return reconstruct8_t<3, true>(g, c, t, d0, val);
      case 4: return reconstruct8_t<4, true>(g, c, t, d0, val);
      case 6: return reconstruct8_t<6, true>(g, c, t, d0, val);
      case 8: return reconstruct8_t<8, true>(g, c, t, d0, val);
      default: return reconstruct8_t<16, true>(g, c, t, d0, val);
    }
  }
  switch (g.bits_k) {
    case 1: return reconstruct8_t<1, false>(g, c, t, d0, val);
    case 2: return reconstruct8_t<2, false>(g, c, t, d0, val);
    case 3: return reconstruct8_t<3, false>(g, c, t, d0, val);
    case 4: return reconstruct8_t<4, false>(g, c, t, d0, val);
    case 6: return reconstruct8_t<6, false>(g, c, t, d0, val);
    case 8: return reconstruct8_t<8, false>(g, c, t, d0, val);
    default: return reconstruct8_t<16, false>(g, c, t, d0, val);
  }
}

// One thread = 8 consecutive channels of one token.
__global__ __launch_bounds__(256) void dequantize_kernel(Geom g, kvq_cache c, int32_t t0, int32_t t1, void* k_out,
                                                         void* v_out, int out_dtype) {
  const int64_t nt = t1 - t0;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (bh, token, octet)
  const int64_t total = (int64_t)g.batch * g.kv_heads * nt * 16;
  if (idx >= total) return;
  const int oct = (int)(idx & 15);
  const int64_t row = idx >> 4;
  const int64_t bh = row / nt;
  const int64_t t = virtual_token(g, c.page_table, (int)(bh / g.kv_heads), (int)(bh % g.kv_heads), t0 + row % nt);
  const int d0 = oct * 8;

  for (int which = 0; which < 2; ++which) {
    void* out = which ? v_out : k_out;
    if (!out) continue;
    float val[8];
    reconstruct8(g, c, which, t, d0, val);
    if (which ? g.rotate_v : g.rotate_k)                                             // 16 threads = one row, all here
      unrotate8(val, oct, rot_sign_bits(which ? g.signs_v : g.signs_k, oct));
    const int64_t o = row * kHeadDim + d0;
    if (out_dtype == KVQ_F32) {
      float* p = (float*)out + o;
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = val[e];
    } else {
      uint16_t* p = (uint16_t*)out + o;
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = out_dtype == KVQ_F16 ? f32_to_f16_bits(val[e]) : f32_to_bf16_bits(val[e]);
    }
  }
}

// Squared reconstruction error (numerator of the MSE of App. B, "Frobenius Norm (MSE) Perspective").
// One thread = 8 consecutive channels of one token; a workgroup walks 16-token slabs of one (b,h) stream with
// stride gridDim.x; differences and the squares of a thread's 8 channels in binary32, everything above that summed
// in binary64, one atomic add per wavefront and tensor.
template <int BK, int BV>
__global__ __launch_bounds__(256) void sq_error_kernel(Geom g, kvq_cache c, const uint16_t* __restrict__ k_ref,
                                                       const uint16_t* __restrict__ v_ref, int ref_bf16, int64_t sb,
                                                       int64_t sh, int64_t st, int32_t t0, int32_t t1,
                                                       double* __restrict__ sums) {
  const int tid = threadIdx.x;
  const int64_t bh = blockIdx.y;
  const int64_t b = bh / g.kv_heads, h = bh % g.kv_heads;
  const int d0 = (tid & 15) * 8;
  const int64_t nt = t1 - t0;
  double acc[2] = {0.0, 0.0};
  for (int64_t r = (int64_t)blockIdx.x * 16 + (tid >> 4); r < nt; r += (int64_t)gridDim.x * 16) {
    const int64_t src = b * sb + h * sh + r * st + d0;
    uint4 raw[2];
    if (k_ref) raw[0] = *reinterpret_cast<const uint4*>(k_ref + src);
    if (v_ref) raw[1] = *reinterpret_cast<const uint4*>(v_ref + src);
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      if (!(which ? v_ref : k_ref)) continue;
      float val[8];
      const int64_t tv = virtual_token(g, c.page_table, (int)b, (int)h, t0 + r);
      if (which) reconstruct8_t<BV, true>(g, c, tv, d0, val);
      else reconstruct8_t<BK, false>(g, c, tv, d0, val);
      const uint32_t rw[4] = {raw[which].x, raw[which].y, raw[which].z, raw[which].w};
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), ref_bf16 != 0);
      // rotated rows are compared in the rotated basis: ||R x - y||_2 = ||x - R^T y||_2
      if (which ? g.rotate_v : g.rotate_k) rotate8(x, tid & 15, rot_sign_bits(which ? g.signs_v : g.signs_k, tid & 15));
      float sq = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float err = x[e] - val[e];
        sq += err * err;
      }
      acc[which] += (double)sq;
    }
  }
  // one atomic per workgroup and tensor: every head's two sums are hit by all the workgroups of that head, and atomics
  // on one address are served one after the other
  __shared__ double part[2][4];
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    double v = acc[which];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    if ((tid & 63) == 0) part[which][tid >> 6] = v;
  }
  __syncthreads();
  if (tid < 2) {
    const double v = (part[tid][0] + part[tid][1]) + (part[tid][2] + part[tid][3]);
    if (v != 0.0) atomicAdd(sums + bh * 2 + tid, v);
  }
}

// Checks the quantizer's fast divisions on the device it runs on: counters[0] counts the binary16 scales whose fast
// reciprocal differs from IEEE division (all 31743 positive finite patterns), counters[1] the sampled quotients
// (2^24 numerators per level count, spread over the binary32 exponent range) that differ.
__global__ __launch_bounds__(256) void selftest_quantizer_kernel(uint32_t* counters) {
#pragma clang fp contract(off)
  const uint32_t u = blockIdx.x * 256 + threadIdx.x;          // 0 .. 65535
  uint32_t bad_rcp = 0, bad_div = 0;
  if (u >= 1 && u < 0x7C00) {
    const float s = widen16((uint16_t)u, false);
    if (rcp_scale(s) != 1.0f / s) bad_rcp = 1;
  }
  const int widths[6] = {1, 2, 3, 4, 6, 8};
  for (uint32_t i = 0; i < 256; ++i) {
    const uint32_t bits = (uint32_t)(((uint64_t)(u * 256u + i) * 0x7F800000ull) >> 24);   // every 128th binary32 >= 0
    const float x = __uint_as_float(bits);
#pragma unroll
    for (int k = 0; k < 6; ++k) {
      const float levels = (float)((1 << widths[k]) - 1);
      const float fast = div_levels(x, levels, inv_levels(widths[k])), exact = x / levels;
      if (fast != exact || f32_to_f16_bits(fast) != f32_to_f16_bits(exact)) ++bad_div;
    }
  }
  if (bad_rcp) atomicAdd(counters, bad_rcp);
  if (bad_div) atomicAdd(counters + 1, bad_div);
}

__global__ __launch_bounds__(64) void zero_u32_kernel(uint32_t* p, int n) {
  if ((int)threadIdx.x < n) p[threadIdx.x] = 0u;
}

__global__ __launch_bounds__(256) void zero_f64_kernel(double* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.0;
}

}  // namespace

namespace {
template <int BK, int BV>
hipError_t launch_q(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype, int64_t sb,
                    int64_t sh, int64_t st, int32_t pos, int32_t n_new, hipStream_t stream) {
  // one workgroup per 32-token span (one block of value codes): against 64-token spans this doubles the workgroups of a
  // small call (a 2048-token chunk of one sequence: 6.5 instead of 7.9 us) and costs a large one nothing
  constexpr int kQSpan = 32;
  const int first = pos / kQSpan, last = (pos + n_new - 1) / kQSpan;
  // spans per workgroup: 4 in a row (each loaded while the one before is quantized) when that still leaves every
  // compute unit many rounds of workgroups (the 70B layer's bulk fill: 5.6 against 5.15 TB/s; 2 or 8 in a row
  // measure 5.4), one for smaller calls, which need their workgroups side by side
  const int64_t spans = (int64_t)(last - first + 1) * g.batch * g.kv_heads;
  const int chain = spans >= 65536 ? 4 : 1;
  dim3 grid((last - first + chain) / chain, g.batch * g.kv_heads);
  if (in_dtype == KVQ_BF16)
    hipLaunchKernelGGL((quantize_append_kernel<BK, BV, true, kQSpan>), grid, dim3(256), 0, stream, g, c, (const uint16_t*)k_new,
                       (const uint16_t*)v_new, sb, sh, st, pos, n_new, chain);
  else
    hipLaunchKernelGGL((quantize_append_kernel<BK, BV, false, kQSpan>), grid, dim3(256), 0, stream, g, c, (const uint16_t*)k_new,
                       (const uint16_t*)v_new, sb, sh, st, pos, n_new, chain);
  return hipGetLastError();
}
template <int BK>
hipError_t launch_qk(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype, int64_t sb,
                     int64_t sh, int64_t st, int32_t pos, int32_t n_new, hipStream_t stream) {
  switch (g.bits_v) {
    case 1: return launch_q<BK, 1>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 2: return launch_q<BK, 2>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 3: return launch_q<BK, 3>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 4: return launch_q<BK, 4>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 6: return launch_q<BK, 6>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 8: return launch_q<BK, 8>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 16: return launch_q<BK, 16>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
  }
  return hipErrorInvalidValue;
}
}  // namespace

hipError_t launch_quantize_append(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype,
                                  int64_t sb, int64_t sh, int64_t st, int32_t pos, int32_t n_new, hipStream_t stream) {
  if (n_new == 0) return hipSuccess;
  switch (g.bits_k) {
    case 1: return launch_qk<1>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 2: return launch_qk<2>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 3: return launch_qk<3>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 4: return launch_qk<4>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 6: return launch_qk<6>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 8: return launch_qk<8>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
    case 16: return launch_qk<16>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, stream);
  }
  return hipErrorInvalidValue;
}

namespace {
// pos_arr != nullptr: one token per sequence at pos_arr[b] (then pos and n_new are 0 and 1)
template <int BK, int BV>
hipError_t launch_sa(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype, int64_t sb,
                     int64_t sh, int64_t st, int32_t pos, int32_t n_new, const int32_t* pos_arr, int32_t max_pos,
                     hipStream_t stream) {
  const int first = pos / g.resid, last = (pos + n_new - 1) / g.resid;
  dim3 grid(last - first + 1, g.batch * g.kv_heads);
  const bool bf = in_dtype == KVQ_BF16, ktok = g.axis_k != KVQ_AXIS_SEQ;
#define KVQ_SA_LAUNCH(BF_, KTOK_, RL_)                                                                                     \
  hipLaunchKernelGGL((seq_append_kernel<BK, BV, BF_, KTOK_, RL_>), grid, dim3(256), 0, stream, g, c, (const uint16_t*)k_new, \
                     (const uint16_t*)v_new, sb, sh, st, pos, n_new, pos_arr, max_pos)
  if (ktok) { if (bf) KVQ_SA_LAUNCH(true, true, 64); else KVQ_SA_LAUNCH(false, true, 64); }
  else if (g.resid == 128) { if (bf) KVQ_SA_LAUNCH(true, false, 128); else KVQ_SA_LAUNCH(false, false, 128); }
  else { if (bf) KVQ_SA_LAUNCH(true, false, 64); else KVQ_SA_LAUNCH(false, false, 64); }
#undef KVQ_SA_LAUNCH
  return hipGetLastError();
}
template <int BK>
hipError_t launch_sak(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype, int64_t sb,
                      int64_t sh, int64_t st, int32_t pos, int32_t n_new, const int32_t* pos_arr, int32_t max_pos,
                      hipStream_t stream) {
  switch (g.bits_v) {
    case 1: return launch_sa<BK, 1>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 2: return launch_sa<BK, 2>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 3: return launch_sa<BK, 3>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 4: return launch_sa<BK, 4>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 6: return launch_sa<BK, 6>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 8: return launch_sa<BK, 8>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
  }
  return hipErrorInvalidValue;
}
hipError_t launch_sa_bits(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype, int64_t sb,
                          int64_t sh, int64_t st, int32_t pos, int32_t n_new, const int32_t* pos_arr, int32_t max_pos,
                          hipStream_t stream) {
  switch (g.bits_k) {
    case 1: return launch_sak<1>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 2: return launch_sak<2>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 3: return launch_sak<3>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 6: return launch_sak<6>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 4: return launch_sak<4>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
    case 8: return launch_sak<8>(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, pos_arr, max_pos, stream);
  }
  return hipErrorInvalidValue;
}
}  // namespace

hipError_t launch_seq_append_one(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype,
                                 int64_t sb, int64_t sh, const int32_t* pos_arr, int32_t max_pos, hipStream_t stream) {
  return launch_sa_bits(g, c, k_new, v_new, in_dtype, sb, sh, kHeadDim, 0, 1, pos_arr, max_pos, stream);
}

hipError_t launch_seq_append(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype,
                             int64_t sb, int64_t sh, int64_t st, int32_t pos, int32_t n_new, hipStream_t stream) {
  if (n_new == 0) return hipSuccess;
  // A first block that starts inside the residual buffer reads its older rows from there, while the workgroups of the
  // call's last tokens (as many as the buffer has slots) overwrite those slots: when the call goes on beyond that block, the block gets a launch of
  // its own and the rest follows in stream order.
  const int32_t first_end = (pos / g.resid + 1) * g.resid;
  if (pos % g.resid != 0 && pos + n_new > first_end) {
    const int32_t n1 = first_end - pos;
    hipError_t e = launch_seq_append(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n1, stream);
    if (e != hipSuccess) return e;
    return launch_seq_append(g, c, (const uint16_t*)k_new + (int64_t)n1 * st, (const uint16_t*)v_new + (int64_t)n1 * st,
                             in_dtype, sb, sh, st, first_end, n_new - n1, stream);
  }
  return launch_sa_bits(g, c, k_new, v_new, in_dtype, sb, sh, st, pos, n_new, nullptr, 0, stream);
}

hipError_t launch_dequantize(const Geom& g, const kvq_cache& c, int32_t t0, int32_t t1, void* k_out, void* v_out,
                             int out_dtype, hipStream_t stream) {
  const int64_t total = (int64_t)g.batch * g.kv_heads * (t1 - t0) * 16;
  if (total == 0) return hipSuccess;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;      // more than one launch can take: the caller splits [t0, t1)
  hipLaunchKernelGGL(dequantize_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, g, c, t0, t1, k_out, v_out, out_dtype);
  return hipGetLastError();
}

hipError_t launch_selftest_quantizer(uint32_t* counters, hipStream_t stream) {
  hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(64), 0, stream, counters, 2);
  hipLaunchKernelGGL(selftest_quantizer_kernel, dim3(256), dim3(256), 0, stream, counters);
  return hipGetLastError();
}

hipError_t launch_reconstruction_error(const Geom& g, const kvq_cache& c, const void* k_ref, const void* v_ref,
                                       int ref_dtype, int64_t sb, int64_t sh, int64_t st, int32_t t0, int32_t t1,
                                       double* sums, hipStream_t stream) {
  const int streams = g.batch * g.kv_heads;
  const int64_t n = (int64_t)streams * 2;
  // cleared by a kernel, not a memset, so that the call can be captured into a graph
  hipLaunchKernelGGL(zero_f64_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, sums, n);
  if (t1 == t0) return hipGetLastError();
  const int64_t slabs = ((int64_t)(t1 - t0) + 15) / 16;
  // about 32 workgroups per compute unit in all (measured: fewer leave latency exposed, more pile up on the atomics)
  int64_t per_stream = (8192 + streams - 1) / streams;
  if (per_stream > slabs) per_stream = slabs;
  const dim3 grid((unsigned)per_stream, streams);
  const int bf = ref_dtype == KVQ_BF16 ? 1 : 0;
#define KVQ_ERR_CASE(BK_, BV_)                                                                                          \
  if (g.bits_k == BK_ && g.bits_v == BV_)                                                                               \
    hipLaunchKernelGGL((sq_error_kernel<BK_, BV_>), grid, dim3(256), 0, stream, g, c, (const uint16_t*)k_ref,           \
                       (const uint16_t*)v_ref, bf, sb, sh, st, t0, t1, sums);
#define KVQ_ERR_ROW(BK_) KVQ_ERR_CASE(BK_, 1) KVQ_ERR_CASE(BK_, 2) KVQ_ERR_CASE(BK_, 3) KVQ_ERR_CASE(BK_, 4) \
  KVQ_ERR_CASE(BK_, 6) KVQ_ERR_CASE(BK_, 8) KVQ_ERR_CASE(BK_, 16)
  KVQ_ERR_ROW(1) KVQ_ERR_ROW(2) KVQ_ERR_ROW(3) KVQ_ERR_ROW(4) KVQ_ERR_ROW(6) KVQ_ERR_ROW(8) KVQ_ERR_ROW(16)
#undef KVQ_ERR_ROW
#undef KVQ_ERR_CASE
  return hipGetLastError();
}

}  // namespace kvq
