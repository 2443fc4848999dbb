// Decode attention over the packed cache (gfx950): out = softmax(scale * q K^^T) V^  (App. A of
// arXiv 2502.15075) with K^, V^ the group-wise reconstructions code*scale+zero (App. B), computed
// without ever materializing K^ or V^:
//
//   logit[t,h]  = sum_g  sK[t,g] * (sum_{d in g} q[h,d] cK[t,d])  +  zK[t,g] * (sum_{d in g} q[h,d])
//   out[h,d]    = ( sum_t (p[t,h] sV[t,g(d)]) cV[t,d]  +  sum_t p[t,h] zV[t,g(d)] ) / sum_t p[t,h]
//
// Both inner sums over codes are 16x16x32 f16 matrix instructions.  A b-bit code c placed in the
// low mantissa bits of a binary16 lane is the subnormal c * 2^-24 (or c * 2^(k-24) when left at bit
// k), which the matrix unit multiplies exactly, so "unpacking" is one AND per two codes; the
// power-of-two position factors are divided out of the query operand once per wavefront.
//
// Work split: one workgroup (4 wavefronts) walks a contiguous range of 64-token blocks of one
// (batch, kv head); each wavefront takes every 4th block and carries all R query heads of that kv
// head as matrix columns (column c = g*R + h: key group g, head h), so every cache byte is read
// once.  Wavefronts merge through LDS, workgroups through a workspace of (max, sum, acc) records
// and a small second kernel.
#include "kvq_internal.h"

namespace kvq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kCodeUnit = 5.9604644775390625e-08f;  // 2^-24: value of a code's lowest mantissa bit
constexpr float kInvCodeUnit = 16777216.0f;
constexpr float kPShift = 10.0f;                      // softmax weights are carried times 2^10 (binary16 headroom)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ half8 as_half8(u32x4 v) { return __builtin_bit_cast(half8, v); }

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
// lane's 32, stored times k_slot_scale(i).
template <int BK> __device__ __forceinline__ int k_slot_elem(int m, int i) {
  const int v = i >> 1, x = i & 1;
  if (BK == 4) return 8 * m + v + 4 * x;
  if (BK == 8) return 8 * m + 4 * (v >> 1) + (v & 1) + 2 * x;
  return 16 * (m >> 1) + 4 * (m & 1) + v + 8 * x;  // BK == 2
}
template <int BK> __device__ __forceinline__ float k_slot_scale(int i) {
  const int v = i >> 1;
  if (BK == 4) return (v & 1) ? 16.0f : 1.0f;
  if (BK == 8) return 1.0f;
  return (float)(1 << (2 * v));  // BK == 2
}
template <int BK> __device__ __forceinline__ half8 unpack_k(const uint32_t* w, int m) {
  u32x4 a;
  if (BK == 4) {
    const uint32_t lo = w[m], hi = w[m] >> 8;
    a = u32x4{lo & 0x000F000Fu, lo & 0x00F000F0u, hi & 0x000F000Fu, hi & 0x00F000F0u};
  } else if (BK == 8) {
    const uint32_t w0 = w[2 * m], w1 = w[2 * m + 1];
    a = u32x4{w0 & 0x00FF00FFu, (w0 >> 8) & 0x00FF00FFu, w1 & 0x00FF00FFu, (w1 >> 8) & 0x00FF00FFu};
  } else {
    const uint32_t ws = w[m >> 1] >> (8 * (m & 1));
    a = u32x4{ws & 0x00030003u, ws & 0x000C000Cu, ws & 0x00300030u, ws & 0x00C000C0u};
  }
  return as_half8(a);
}

// ---- value codes: one lane holds, per 64-token block, 4*BV dwords (index = 4*piece + dword) --
// Register v (0..3) of a step's operand holds slots 2v, 2v+1 and is left at bit offset v_slot_shift(v) of
// its 16-bit lane, i.e. it reads as code * 2^shift * 2^-24; the softmax weight of those slots is
// divided by 2^shift instead (an exponent offset, free).
template <int BV> __device__ __forceinline__ constexpr int v_slot_shift(int v) {
  return BV == 2 ? 2 * v : (BV == 4 ? 4 * (v & 1) : 0);
}
template <int BV> __device__ __forceinline__ half8 unpack_v(const uint32_t* w, int dt, int o) {
  u32x4 a;
  if (BV == 2) {
    const uint32_t ws = w[dt] >> (8 * o);
    a = u32x4{ws & 0x00030003u, ws & 0x000C000Cu, ws & 0x00300030u, ws & 0x00C000C0u};
  } else if (BV == 4) {
    const uint32_t lo = w[2 * dt + o], hi = lo >> 8;
    a = u32x4{lo & 0x000F000Fu, lo & 0x00F000F0u, hi & 0x000F000Fu, hi & 0x00F000F0u};
  } else {
    const uint32_t w0 = w[4 * dt + 2 * o], w1 = w[4 * dt + 2 * o + 1];
    a = u32x4{w0 & 0x00FF00FFu, (w0 >> 8) & 0x00FF00FFu, w1 & 0x00FF00FFu, (w1 >> 8) & 0x00FF00FFu};
  }
  return as_half8(a);
}

template <int BK, int BV>
struct BlockRegs {                 // everything one lane loads for one 64-token block
  uint32_t kc[4][BK];              // 4 tiles of 16 tokens
  u32x4 km[4];                     // key scale/zero of this lane's 4 tokens per tile (its own group)
  uint32_t vc[4 * BV];
  u32x4 vm[4];
};

struct LaneCtx {
  const uint8_t* kc; const uint32_t* km; const uint8_t* vc; const uint32_t* vm;   // (b,h) stream bases
  int lane, c, j, gk, gv, ngk, ngv;
};

template <int BK, int BV>
__device__ __forceinline__ void load_block(BlockRegs<BK, BV>& r, const LaneCtx& L, int blk) {
#pragma unroll
  for (int tile = 0; tile < 4; ++tile) {
    const int64_t t16 = (int64_t)blk * 4 + tile;
    const uint8_t* p = L.kc + ((t16 * 16 + L.c) * (16 * BK) + L.j * (4 * BK));
    if (BK == 4) {
      u32x4 v = *reinterpret_cast<const u32x4*>(p);
      r.kc[tile][0] = v.x; r.kc[tile][1] = v.y; r.kc[tile][2] = v.z; r.kc[tile][3] = v.w;
    } else if (BK == 8) {
      u32x4 v0 = *reinterpret_cast<const u32x4*>(p), v1 = *reinterpret_cast<const u32x4*>(p + 16);
      r.kc[tile][0] = v0.x; r.kc[tile][1] = v0.y; r.kc[tile][2] = v0.z; r.kc[tile][3] = v0.w;
      r.kc[tile][4] = v1.x; r.kc[tile][5] = v1.y; r.kc[tile][6] = v1.z; r.kc[tile][7] = v1.w;
    } else {
      uint2 v = *reinterpret_cast<const uint2*>(p);
      r.kc[tile][0] = v.x; r.kc[tile][1] = v.y;
    }
    r.km[tile] = *reinterpret_cast<const u32x4*>(L.km + ((t16 * L.ngk + L.gk) * 16 + 4 * L.j));
    r.vm[tile] = *reinterpret_cast<const u32x4*>(L.vm + ((t16 * L.ngv + L.gv) * 16 + 4 * L.j));
  }
  const uint8_t* vb = L.vc + (int64_t)blk * (1024 * BV) + L.lane * 16;
#pragma unroll
  for (int piece = 0; piece < BV; ++piece) {
    u32x4 v = *reinterpret_cast<const u32x4*>(vb + piece * 1024);
    r.vc[4 * piece + 0] = v.x; r.vc[4 * piece + 1] = v.y; r.vc[4 * piece + 2] = v.z; r.vc[4 * piece + 3] = v.w;
  }
}

__device__ __forceinline__ float meta_scale(uint32_t m) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(m & 0xFFFFu)); }
__device__ __forceinline__ float meta_zero(uint32_t m) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(m >> 16)); }

struct WaveState {
  float4v acc[8];   // out^T tile dt: rows d = 16*dt + 4*j + r, column c
  float m;          // running max of this lane's head, in log2 units
  float noff[4];    // kPShift - m - v_slot_shift(v): exponent offset of the slots in operand register v
  float l[4];       // per register class v: this lane's share of sum_t p * 2^(kPShift - shift(v))
  float zacc[4];    // same, weighted by zV[t, gv]
};

// binary16 product of a binary32 weight and the binary16 held in the low half of `meta`, written to the
// low / high half of `dst` (one rounding).
__device__ __forceinline__ void mix_lo(uint32_t& dst, float p, uint32_t meta) {
  asm("v_fma_mixlo_f16 %0, %1, %2, 0 op_sel_hi:[0,1,0]" : "=v"(dst) : "v"(p), "v"(meta));
}
__device__ __forceinline__ void mix_hi(uint32_t& dst, float p, uint32_t meta) {
  asm("v_fma_mixhi_f16 %0, %1, %2, 0 op_sel_hi:[0,1,0]" : "+v"(dst) : "v"(p), "v"(meta));
}

// One 64-token block.  MASKED: tokens at or beyond seq_len get weight 0 (garbage may sit there).
template <int BK, int BV, int R, bool MASKED>
__device__ __forceinline__ void compute_block(const BlockRegs<BK, BV>& r, const half8 (&qb)[4], float qsum_u, float kappa,
                                              WaveState& st, const LaneCtx& L, int blk, int seq_len) {
#pragma unroll
  for (int o = 0; o < 2; ++o) {                 // two steps of 32 tokens
    float s[8];                                  // slot i: token 16*(i/4) + 4*j + i%4 of this step
    {
      float4v d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < 4; ++m) {              // two independent accumulation chains
        d0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_k<BK>(r.kc[2 * o], m), qb[m], d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_k<BK>(r.kc[2 * o + 1], m), qb[m], d1, 0, 0, 0);
      }
      const uint32_t meta[8] = {r.km[2 * o].x, r.km[2 * o].y, r.km[2 * o].z, r.km[2 * o].w,
                                r.km[2 * o + 1].x, r.km[2 * o + 1].y, r.km[2 * o + 1].z, r.km[2 * o + 1].w};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float d = i < 4 ? d0[i & 3] : d1[i & 3];
        const float part = fmaf(d, meta_scale(meta[i]), meta_zero(meta[i]) * qsum_u);
        s[i] = sum_over_groups<R>(part);
      }
    }
    bool valid[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      valid[i] = !MASKED || (blk * 64 + 32 * o + 16 * (i >> 2) + 4 * L.j + (i & 3) < seq_len);
      if (MASKED && !valid[i]) s[i] = kNegBig;
    }
    // running max: only when some lane sees a larger logit than its current max
    float lmax = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
    float lx = lmax * kappa;
    if (__any(lx > st.m)) {
      lx = fmaxf(lx, __shfl_xor(lx, 16));
      lx = fmaxf(lx, __shfl_xor(lx, 32));
      const float m_new = fmaxf(st.m, lx);
      const float f = __builtin_amdgcn_exp2f(st.m - m_new);
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) st.acc[dt] *= f;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        st.l[v] *= f; st.zacc[v] *= f;
        st.noff[v] = kPShift - (float)v_slot_shift<BV>(v) - m_new;
      }
      st.m = m_new;
    }
    const uint32_t vmeta[8] = {r.vm[2 * o].x, r.vm[2 * o].y, r.vm[2 * o].z, r.vm[2 * o].w,
                               r.vm[2 * o + 1].x, r.vm[2 * o + 1].y, r.vm[2 * o + 1].z, r.vm[2 * o + 1].w};
    uint32_t pw[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = i >> 1;
      float p = __builtin_amdgcn_exp2f(fmaf(s[i], kappa, st.noff[v]));
      uint32_t vm = vmeta[i];
      if (MASKED && !valid[i]) { p = 0.f; vm = 0u; }
      st.l[v] += p;
      st.zacc[v] = fmaf(p, meta_zero(vm), st.zacc[v]);
      if (i & 1) mix_hi(pw[v], p, vm); else mix_lo(pw[v], p, vm);
    }
    const half8 pb = as_half8(u32x4{pw[0], pw[1], pw[2], pw[3]});
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
      st.acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(unpack_v<BV>(r.vc, dt, o), pb, st.acc[dt], 0, 0, 0);
  }
}

// Record layout in the workspace: [b][hq][split] x (kHeadDim + 4) floats = acc[128], m, l, 0, 0.
constexpr int kRec = kHeadDim + 4;

template <int BK, int BV, int R>
__global__ __launch_bounds__(256, 2) void decode_kernel(Geom g, kvq_cache cache, const uint16_t* __restrict__ q, int q_bf16,
                                                        int32_t q_heads, int32_t seq_len, float softmax_scale,
                                                        float* __restrict__ ws, void* __restrict__ out, int out_dtype,
                                                        int32_t n_splits, int32_t blocks_per_split) {
  __shared__ float sm_o[4][R][kHeadDim];
  __shared__ float sm_m[4][R], sm_l[4][R];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int split = blockIdx.x, bh = blockIdx.y;
  const int b = bh / g.kv_heads, hk = bh % g.kv_heads;

  LaneCtx L;
  L.lane = lane; L.c = lane & 15; L.j = lane >> 4;
  L.ngk = g.ng_k; L.ngv = g.ng_v;
  const int h = L.c % R, grp = L.c / R;
  const bool act_k = grp < g.ng_k, act_v = grp < g.ng_v;
  L.gk = act_k ? grp : 0; L.gv = act_v ? grp : 0;
  L.kc = (const uint8_t*)cache.k_codes + (int64_t)bh * g.kc_stream;
  L.km = (const uint32_t*)((const uint8_t*)cache.k_meta + (int64_t)bh * g.km_stream);
  L.vc = (const uint8_t*)cache.v_codes + (int64_t)bh * g.vc_stream;
  L.vm = (const uint32_t*)((const uint8_t*)cache.v_meta + (int64_t)bh * g.vm_stream);

  // ---- query operand: column c carries head h restricted to key group gk (zero elsewhere)
  const uint16_t* qrow = q + ((int64_t)b * q_heads + hk * R + h) * kHeadDim;
  auto qval = [&](int d) -> float {
    const uint16_t bits = qrow[d];
    return q_bf16 ? __uint_as_float((uint32_t)bits << 16) : (float)__builtin_bit_cast(_Float16, bits);
  };
  half8 qb[4];
  const bool mine = act_k && ((32 * L.j) / g.g_k == L.gk);   // this lane's 32 channels lie in one group
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = mine ? qval(32 * L.j + k_slot_elem<BK>(m, i)) / k_slot_scale<BK>(i) : 0.f;
      qb[m][i] = (_Float16)v;
    }
  float qsum = 0.f;
  if (act_k)
    for (int d = L.gk * g.g_k; d < (L.gk + 1) * g.g_k; ++d) qsum += qval(d);
  const float qsum_u = qsum * kCodeUnit;
  const float kappa = softmax_scale * kLog2e * kInvCodeUnit;

  WaveState st;
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) st.acc[dt] = float4v{0.f, 0.f, 0.f, 0.f};
  st.m = kNegBig;
#pragma unroll
  for (int v = 0; v < 4; ++v) { st.l[v] = 0.f; st.zacc[v] = 0.f; st.noff[v] = kPShift - (float)v_slot_shift<BV>(v) - kNegBig; }

  // ---- walk this wavefront's blocks: complete blocks in a two-deep register pipeline, then the ragged one
  const int n_blocks = (seq_len + 63) >> 6;
  const int blk_begin = split * blocks_per_split;
  const int blk_end = min(blk_begin + blocks_per_split, n_blocks);
  const int full_end = min(blk_end, seq_len >> 6);             // blocks below this index are complete
  {
    BlockRegs<BK, BV> ra, rb;
    int blk = blk_begin + wave;
    if (blk < full_end) load_block<BK, BV>(ra, L, blk);
    while (blk < full_end) {
      if (blk + 4 < full_end) load_block<BK, BV>(rb, L, blk + 4);
      compute_block<BK, BV, R, false>(ra, qb, qsum_u, kappa, st, L, blk, seq_len);
      blk += 4;
      if (blk >= full_end) break;
      if (blk + 4 < full_end) load_block<BK, BV>(ra, L, blk + 4);
      compute_block<BK, BV, R, false>(rb, qb, qsum_u, kappa, st, L, blk, seq_len);
      blk += 4;
    }
    // blk is now the first block of this wavefront's stride at or beyond full_end
    if (blk < blk_end) {
      load_block<BK, BV>(ra, L, blk);
      compute_block<BK, BV, R, true>(ra, qb, qsum_u, kappa, st, L, blk, seq_len);
    }
  }

  // ---- wavefront totals: l and zacc over register classes and the 4 lane groups j
  float l = 0.f, z = 0.f;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const float w = (float)(1 << v_slot_shift<BV>(v));
    l = fmaf(st.l[v], w, l); z = fmaf(st.zacc[v], w, z);
  }
  l += __shfl_xor(l, 16); l += __shfl_xor(l, 32);
  z += __shfl_xor(z, 16); z += __shfl_xor(z, 32);
  if (act_v) {
    const int dtg = 8 / g.ng_v;                                // d-tiles per value group
    for (int dt = L.gv * dtg; dt < (L.gv + 1) * dtg; ++dt)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) if (k == dt) a = st.acc[k][rr];   // static register indexing
        sm_o[wave][h][16 * dt + 4 * L.j + rr] = fmaf(a, kInvCodeUnit, z);
      }
    if (grp == 0 && L.j == 0) { sm_m[wave][h] = st.m; sm_l[wave][h] = l; }
  }
  __syncthreads();

  // ---- merge the 4 wavefronts; write a partial record, or the result when there is one split
  for (int idx = tid; idx < R * kHeadDim; idx += 256) {
    const int hh = idx / kHeadDim, d = idx % kHeadDim;
    float M = fmaxf(fmaxf(sm_m[0][hh], sm_m[1][hh]), fmaxf(sm_m[2][hh], sm_m[3][hh]));
    float o = 0.f, ll = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = exp2f(sm_m[w][hh] - M);
      o = fmaf(f, sm_o[w][hh][d], o);
      ll = fmaf(f, sm_l[w][hh], ll);
    }
    const int64_t hq = (int64_t)b * q_heads + hk * R + hh;
    if (n_splits == 1) {
      const float val = o / ll;
      if (out_dtype == KVQ_F32) ((float*)out)[hq * kHeadDim + d] = val;
      else if (out_dtype == KVQ_F16) ((_Float16*)out)[hq * kHeadDim + d] = (_Float16)val;
      else {
        uint32_t u = __float_as_uint(val);
        ((uint16_t*)out)[hq * kHeadDim + d] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
      }
    } else {
      float* rec = ws + (hq * n_splits + split) * kRec;
      rec[d] = o;
      if (d == 0) { rec[kHeadDim] = M; rec[kHeadDim + 1] = ll; }
    }
  }
}

// Combine the split records of one (b, hq): log-sum-exp merge, then normalize.
__global__ __launch_bounds__(128) void merge_kernel(const float* __restrict__ ws, void* __restrict__ out, int out_dtype,
                                                    int32_t n_splits) {
  const int64_t hq = blockIdx.x;
  const int d = threadIdx.x;
  const float* rec = ws + hq * n_splits * kRec;
  float M = kNegBig;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, rec[s * kRec + kHeadDim]);
  float o = 0.f, l = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float f = exp2f(rec[s * kRec + kHeadDim] - M);
    o = fmaf(f, rec[s * kRec + d], o);
    l = fmaf(f, rec[s * kRec + kHeadDim + 1], l);
  }
  const float val = o / l;
  if (out_dtype == KVQ_F32) ((float*)out)[hq * kHeadDim + d] = val;
  else if (out_dtype == KVQ_F16) ((_Float16*)out)[hq * kHeadDim + d] = (_Float16)val;
  else {
    uint32_t u = __float_as_uint(val);
    ((uint16_t*)out)[hq * kHeadDim + d] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
  }
}

template <int BK, int BV, int R>
hipError_t launch_one(const Geom& g, const kvq_cache& c, const void* q, int q_dtype, int32_t q_heads, int32_t seq_len,
                      float softmax_scale, void* out, int out_dtype, float* ws, const DecodePlan& plan, hipStream_t stream) {
  dim3 grid(plan.n_splits, g.batch * g.kv_heads);
  hipLaunchKernelGGL((decode_kernel<BK, BV, R>), grid, dim3(256), 0, stream, g, c, (const uint16_t*)q,
                     q_dtype == KVQ_BF16 ? 1 : 0, q_heads, seq_len, softmax_scale, ws, out, out_dtype, plan.n_splits,
                     plan.blocks_per_split);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || plan.n_splits == 1) return e;
  hipLaunchKernelGGL(merge_kernel, dim3(g.batch * q_heads), dim3(128), 0, stream, ws, out, out_dtype, plan.n_splits);
  return hipGetLastError();
}

template <int BK, int BV>
hipError_t launch_r(int R, const Geom& g, const kvq_cache& c, const void* q, int q_dtype, int32_t q_heads, int32_t seq_len,
                    float softmax_scale, void* out, int out_dtype, float* ws, const DecodePlan& plan, hipStream_t stream) {
  switch (R) {
    case 1: return launch_one<BK, BV, 1>(g, c, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, ws, plan, stream);
    case 2: return launch_one<BK, BV, 2>(g, c, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, ws, plan, stream);
    case 4: return launch_one<BK, BV, 4>(g, c, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, ws, plan, stream);
    case 8: return launch_one<BK, BV, 8>(g, c, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, ws, plan, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool decode_supported(const Geom& g, int32_t q_heads) {
  const int R = q_heads / g.kv_heads;
  if (R != 1 && R != 2 && R != 4 && R != 8) return false;
  if (g.bits_k == 16 || g.bits_v == 16) return false;          // unquantized planes: no kernel yet
  if (R * g.ng_k > 16 || R * g.ng_v > 16) return false;        // head x group columns must fit one 16-wide tile
  return true;
}

DecodePlan plan_decode(const Geom& g, int32_t seq_len) {
  const int n_blocks = (seq_len + 63) / 64;
  const int streams = g.batch * g.kv_heads;
  const int target_wgs = 256 * 2;                              // CUs x resident workgroups per CU
  int splits = (target_wgs + streams - 1) / streams;
  const int max_splits = (n_blocks + 3) / 4;                   // at least one block per wavefront
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  int bps = (n_blocks + splits - 1) / splits;
  bps = (bps + 3) / 4 * 4;
  splits = (n_blocks + bps - 1) / bps;
  return DecodePlan{splits, bps};
}

hipError_t launch_decode_attention(const Geom& g, const kvq_cache& c, const void* q, int q_dtype, int32_t q_heads,
                                   int32_t seq_len, float softmax_scale, void* out, int out_dtype, float* workspace,
                                   const DecodePlan& plan, hipStream_t stream) {
  const int R = q_heads / g.kv_heads;
#define KVQ_CASE(BK_, BV_)                                                                                          \
  if (g.bits_k == BK_ && g.bits_v == BV_)                                                                           \
    return launch_r<BK_, BV_>(R, g, c, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, workspace, plan, stream);
  KVQ_CASE(4, 2)
  KVQ_CASE(2, 4)
  KVQ_CASE(4, 4)
  KVQ_CASE(8, 8)
  KVQ_CASE(2, 2)
  KVQ_CASE(8, 4)
  KVQ_CASE(8, 2)
  KVQ_CASE(4, 8)
  KVQ_CASE(2, 8)
#undef KVQ_CASE
  return hipErrorInvalidValue;
}

}  // namespace kvq
