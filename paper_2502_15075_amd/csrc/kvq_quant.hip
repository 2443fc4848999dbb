// Quantize-append and dequantize kernels (gfx950).
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

constexpr int kLdsPitch = kHeadDim + 2;  // uint16 elements per staged value row (odd dword pitch)
constexpr int kSpan = 64;                // tokens one workgroup covers (two 32-token value blocks)

// One workgroup = one 64-token span of one (b,h) stream, restricted to the new tokens in it.
__global__ __launch_bounds__(256) void quantize_append_kernel(Geom g, kvq_cache c, const uint16_t* __restrict__ k_new,
                                                              const uint16_t* __restrict__ v_new, int in_bf16,
                                                              int64_t sb, int64_t sh, int64_t st, int32_t pos,
                                                              int32_t n_new) {
  __shared__ uint16_t vstage[kSpan * kLdsPitch];
  const int tid = threadIdx.x;
  const int bh = blockIdx.y;
  const int b = bh / g.kv_heads, h = bh % g.kv_heads;
  const int blk = pos / kSpan + blockIdx.x;
  const int lo = max(pos, blk * kSpan) - blk * kSpan;
  const int hi = min(pos + n_new, (blk + 1) * kSpan) - blk * kSpan;
  const int lane16 = tid & 15;
  const int d0 = lane16 * 8;

  uint8_t* kc = (uint8_t*)c.k_codes + (int64_t)bh * g.kc_stream;
  uint32_t* km = (uint32_t*)((uint8_t*)c.k_meta + (int64_t)bh * g.km_stream);
  uint32_t* vm = (uint32_t*)((uint8_t*)c.v_meta + (int64_t)bh * g.vm_stream);
  uint32_t* vc = (uint32_t*)((uint8_t*)c.v_codes + (int64_t)bh * g.vc_stream) + (int64_t)blk * (256 * g.bits_v);

  for (int row = lo + (tid >> 4); row < hi; row += 16) {
    const int64_t t = (int64_t)blk * kSpan + row;
    const int64_t src = (int64_t)b * sb + (int64_t)h * sh + (t - pos) * st + d0;
    // ---- keys: row-major codes
    {
      uint4 raw = *reinterpret_cast<const uint4*>(k_new + src);
      const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
      if (g.bits_k == 16) {
        *reinterpret_cast<uint4*>(kc + t * 256 + d0 * 2) = raw;
      } else {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), in_bf16);
        uint32_t codes[8];
        uint16_t S, Z;
        const int lpg = g.g_k >> 3;
        quantize8(x, g.bits_k, lpg, codes, &S, &Z);
        if ((lane16 & (lpg - 1)) == 0) km[meta_index(t, lane16 / lpg, g.ng_k)] = (uint32_t)S | ((uint32_t)Z << 16);
        uint8_t* rowp = kc + t * (16 * g.bits_k);
        if (g.bits_k == 4) {
          uint32_t w = 0;
#pragma unroll
          for (int e = 0; e < 8; ++e) w |= codes[e] << (4 * e);
          reinterpret_cast<uint32_t*>(rowp)[lane16] = w;
        } else if (g.bits_k == 2) {
          uint32_t w = 0;
#pragma unroll
          for (int e = 0; e < 8; ++e) w |= codes[e] << (2 * e);
          reinterpret_cast<uint16_t*>(rowp)[lane16] = (uint16_t)w;
        } else {
          uint32_t w0 = codes[0] | (codes[1] << 8) | (codes[2] << 16) | (codes[3] << 24);
          uint32_t w1 = codes[4] | (codes[5] << 8) | (codes[6] << 16) | (codes[7] << 24);
          reinterpret_cast<uint2*>(rowp)[lane16] = make_uint2(w0, w1);
        }
      }
    }
    // ---- values: codes staged in LDS, scale/zero straight to memory
    {
      uint4 raw = *reinterpret_cast<const uint4*>(v_new + src);
      const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
      uint16_t* dst = vstage + row * kLdsPitch + d0;
      if (g.bits_v == 16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e] = (uint16_t)(rw[e >> 1] >> (16 * (e & 1)));
      } else {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = widen16((uint16_t)(rw[e >> 1] >> (16 * (e & 1))), in_bf16);
        uint32_t codes[8];
        uint16_t S, Z;
        const int lpg = g.g_v >> 3;
        quantize8(x, g.bits_v, lpg, codes, &S, &Z);
        if ((lane16 & (lpg - 1)) == 0) vm[meta_index(t, lane16 / lpg, g.ng_v)] = (uint32_t)S | ((uint32_t)Z << 16);
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e] = (uint16_t)codes[e];
      }
    }
  }
  __syncthreads();

  // ---- values: assemble the span's dwords (two 32-token blocks) in storage order; keep the fields of other tokens
  const int bv = g.bits_v;
  const int P = 16 / bv;
  const uint32_t fmask = bv == 16 ? 0xFFFFu : ((1u << bv) - 1u);
  const int blk_dwords = 128 * bv;
  for (int w = tid; w < 2 * blk_dwords; w += 256) {
    const int sub = w / blk_dwords, wi = w % blk_dwords;
    const int piece = wi >> 8, rem = wi & 255;
    const int L = rem >> 2, m = rem & 3;
    const int e = 4 * piece + m;
    const int j = L >> 4, dl = L & 15;
    uint32_t bits = 0, mask = 0;
    for (int x = 0; x < 2; ++x)
      for (int p = 0; p < P; ++p) {
        const int q = e * P + p;
        const int dt = q >> 2, v = q & 3;
        const int i = 2 * v + x;
        const int tt = 32 * sub + 16 * (i >> 2) + 4 * j + (i & 3);
        if (tt >= lo && tt < hi) {
          const int sh_ = 16 * x + bv * p;
          bits |= ((uint32_t)vstage[tt * kLdsPitch + dt * 16 + dl] & fmask) << sh_;
          mask |= fmask << sh_;
        }
      }
    if (mask == 0) continue;
    if (mask != 0xFFFFFFFFu) bits |= vc[w] & ~mask;
    vc[w] = bits;
  }
}

// Reconstruction x^ = code * scale + zero.  One thread = 8 consecutive channels of one token.
__global__ __launch_bounds__(256) void dequantize_kernel(Geom g, kvq_cache c, int32_t t0, int32_t t1, void* k_out,
                                                         void* v_out, int out_dtype) {
  const int64_t nt = t1 - t0;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // (bh, token, octet)
  const int64_t total = (int64_t)g.batch * g.kv_heads * nt * 16;
  if (idx >= total) return;
  const int oct = (int)(idx & 15);
  const int64_t row = idx >> 4;
  const int64_t bh = row / nt;
  const int64_t t = t0 + row % nt;
  const int d0 = oct * 8;
  const bool raw_bf16 = g.raw_dtype == KVQ_BF16;

  for (int which = 0; which < 2; ++which) {
    void* out = which ? v_out : k_out;
    if (!out) continue;
    const int b = which ? g.bits_v : g.bits_k;
    const int G = which ? g.g_v : g.g_k;
    const int ng = which ? g.ng_v : g.ng_k;
    const uint8_t* cs = (const uint8_t*)(which ? c.v_codes : c.k_codes) + bh * (which ? g.vc_stream : g.kc_stream);
    const uint32_t* ms = (const uint32_t*)((const uint8_t*)(which ? c.v_meta : c.k_meta) + bh * (which ? g.vm_stream : g.km_stream));
    float val[8];
    float s = 0.f, z = 0.f;
    if (b != 16) {
      uint32_t m = ms[meta_index(t, d0 / G, ng)];
      s = widen16((uint16_t)(m & 0xFFFF), false);
      z = widen16((uint16_t)(m >> 16), false);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int d = d0 + e;
      uint32_t code;
      if (!which) {
        const int64_t bit = (t * kHeadDim + d) * b;
        const uint32_t wd = *reinterpret_cast<const uint32_t*>(cs + ((bit >> 5) << 2));
        code = (wd >> (bit & 31)) & (b == 16 ? 0xFFFFu : ((1u << b) - 1u));
      } else {
        int dw, bit;
        v_field((int)(t & 31), d, b, &dw, &bit);
        const uint32_t wd = reinterpret_cast<const uint32_t*>(cs + (t >> 5) * (int64_t)(512 * b))[dw];
        code = (wd >> bit) & (b == 16 ? 0xFFFFu : ((1u << b) - 1u));
      }
      val[e] = b == 16 ? widen16((uint16_t)code, raw_bf16) : (float)code * s + z;
    }
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

}  // namespace

hipError_t launch_quantize_append(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype,
                                  int64_t sb, int64_t sh, int64_t st, int32_t pos, int32_t n_new, hipStream_t stream) {
  if (n_new == 0) return hipSuccess;
  const int first = pos / kSpan, last = (pos + n_new - 1) / kSpan;
  dim3 grid(last - first + 1, g.batch * g.kv_heads);
  hipLaunchKernelGGL(quantize_append_kernel, grid, dim3(256), 0, stream, g, c, (const uint16_t*)k_new,
                     (const uint16_t*)v_new, in_dtype == KVQ_BF16 ? 1 : 0, sb, sh, st, pos, n_new);
  return hipGetLastError();
}

hipError_t launch_dequantize(const Geom& g, const kvq_cache& c, int32_t t0, int32_t t1, void* k_out, void* v_out,
                             int out_dtype, hipStream_t stream) {
  const int64_t total = (int64_t)g.batch * g.kv_heads * (t1 - t0) * 16;
  if (total == 0) return hipSuccess;
  const int64_t blocks = (total + 255) / 256;
  hipLaunchKernelGGL(dequantize_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, g, c, t0, t1, k_out, v_out, out_dtype);
  return hipGetLastError();
}

}  // namespace kvq
