// Internal declarations shared by the translation units of libkvq (host launchers + device helpers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvq.h"

namespace kvq {

constexpr int kHeadDim = 128;     // the only head_dim the kernels are written for
constexpr int kBlockTokens = 32;  // value codes are stored in blocks of this many tokens
constexpr int kSeqGroup = 64;     // tokens of the block the attention kernel walks channel-wise keys in (two steps), and the
                                  // residual buffer's usual length

// A layout with a residual buffer: channel-wise keys always, token-wise keys when resid_len says so.
inline bool has_residual(const kvq_layout& L) { return L.axis_k == KVQ_AXIS_SEQ || L.resid_len != 0; }
// Its slots: resid_len, or the group length of channel-wise keys when that field is 0.
inline int32_t residual_slots(const kvq_layout& L) {
  return L.resid_len ? L.resid_len : (L.axis_k == KVQ_AXIS_SEQ ? L.group_k : 0);
}

// Geometry derived once on the host and passed by value to every kernel.
struct Geom {
  int32_t batch, kv_heads, t_cap;   // t_cap = max_seq rounded up to kBlockTokens
  int32_t bits_k, bits_v, ng_k, ng_v, g_k, g_v;   // bits: 1, 2, 3, 4, 6, 8 (2^b - 1 steps, b bits per code in the plane), 16 = unquantized
  int32_t raw_dtype;
  int32_t axis_k;                   // KVQ_AXIS_SEQ: channel-wise key groups of seq_g tokens + residual buffer;
                                    // then g_k = 128 and ng_k = 1 (one matrix column per head on the key side)
  int32_t seq_g;                    // tokens per group of channel-wise keys (32, 64 or 128), 0 with token-wise keys
  int32_t resid;                    // slots of the residual buffer (64 or 128, a multiple of seq_g), 0 without one: the
                                    // planes then hold the tokens below seq_len rounded down to it, the buffer the rest
  int32_t rotate_k;                 // key rows are stored as codes of R k (randomized Hadamard rotation)
  uint32_t signs_k[4];              // bit d set: s_d = -1
  int32_t rotate_v;                 // value rows are stored as codes of R_v v; outputs are taken back with R_v^T
  uint32_t signs_v[4];
  int64_t kc_stream, km_stream, vc_stream, vm_stream;   // bytes per (b,h) stream in each plane
  // paged planes: a "stream" is then one head's share of one page (t_cap = page_tokens), the pool holds
  // n_pages * kv_heads of them, and sequence b finds its pages through the table (pages_per_seq entries per sequence)
  int32_t page_shift;               // log2(page_tokens), 0 = not paged
  int32_t pages_per_seq;
};

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

inline Geom make_geom(const kvq_layout& L) {
  Geom g{};
  g.batch = L.batch; g.kv_heads = L.kv_heads;
  g.axis_k = L.axis_k;
  g.resid = residual_slots(L);
  g.seq_g = L.axis_k == KVQ_AXIS_SEQ ? L.group_k : 0;
  g.t_cap = (int32_t)round_up(L.max_seq, g.resid ? g.resid : kBlockTokens);
  g.page_shift = 0; g.pages_per_seq = 0;
  if (L.page_tokens) {
    while ((1 << g.page_shift) < L.page_tokens) ++g.page_shift;
    g.pages_per_seq = (L.max_seq + L.page_tokens - 1) / L.page_tokens;
    g.t_cap = L.page_tokens;                       // the unit every plane is laid out for
  }
  g.bits_k = L.bits_k; g.bits_v = L.bits_v;                   // every code is packed at its own width
  g.g_k = (L.bits_k == 16 || L.axis_k == KVQ_AXIS_SEQ) ? kHeadDim : L.group_k;
  g.g_v = L.bits_v == 16 ? kHeadDim : L.group_v;
  g.ng_k = kHeadDim / g.g_k; g.ng_v = kHeadDim / g.g_v;
  g.raw_dtype = L.raw_dtype;
  g.rotate_k = L.rotate_k;
  for (int i = 0; i < 4; ++i) g.signs_k[i] = L.rotate_k ? L.signs_k[i] : 0u;
  g.rotate_v = L.rotate_v;
  for (int i = 0; i < 4; ++i) g.signs_v[i] = L.rotate_v ? L.signs_v[i] : 0u;
  g.kc_stream = (int64_t)g.t_cap * (kHeadDim * g.bits_k / 8);
  g.vc_stream = (int64_t)g.t_cap * (kHeadDim * g.bits_v / 8);
  g.km_stream = L.bits_k == 16 ? 0 : L.axis_k == KVQ_AXIS_SEQ ? (int64_t)(g.t_cap / g.seq_g) * kHeadDim * 4
                                                                : (int64_t)g.t_cap * g.ng_k * 4;
  g.vm_stream = L.bits_v == 16 ? 0 : (int64_t)g.t_cap * g.ng_v * 4;
  return g;
}

// Number of sequence splits the decode kernel uses for this problem (host-side plan).
struct DecodePlan {
  int32_t n_splits;         // workgroups per (b, h_kv)
  int32_t steps_per_split;  // 32-token steps each workgroup walks (a multiple of waves_per_wg)
  int32_t waves_per_wg;     // 4 or 8 wavefronts per workgroup
};

// The single new token of a fused decode step: [B][H_kv][D] rows with element strides.
struct AppendOne {
  const void* k_new; const void* v_new; int in_dtype; int64_t stride_b, stride_h;
};
DecodePlan plan_decode(const Geom& g, int32_t seq_len);
int32_t decode_records_bound(const Geom& g, int32_t seq_len);   // >= the records per head of every length up to seq_len
int device_compute_units();                                      // of the current device (256 without one)

// Everything the decode kernels need, passed by value.
struct DecodeArgs {
  Geom g;
  kvq_cache cache;
  const uint16_t* q; int q_bf16; int32_t q_heads;
  int32_t heads_per_kv;       // q_heads / kv_heads: 1..8; the kernels lay columns out for the next power of two and leave
                              // the surplus heads empty
  int32_t seq_len; float softmax_scale;
  // per-sequence lengths: batch element b attends over seq_lens[b] + lens_offset tokens (clamped to [1, seq_len]; seq_len
  // is then the upper bound the launch was planned for); nullptr: every sequence has seq_len tokens
  const int32_t* seq_lens; int32_t lens_offset;
  // channel-wise keys with per-sequence lengths: the length n = clamp(seq_lens[b] + lens_offset, 1, lens_bound) is cut
  // into its flushed blocks (lens_mode 1: n rounded down to the buffer's length, possibly 0) or its residual tail (lens_mode 2:
  // n modulo that length, possibly 0); a workgroup with nothing to read writes an empty record.  lens_mode 0: n as it is.
  int32_t lens_mode, lens_bound, lens_block;   // lens_block: the buffer's slots (a power of two)
  float* ws; void* out; int out_dtype;
  int32_t n_splits, steps_per_split;
  // partial records: a workgroup writes record rec_base + split of rec_splits per (batch, query head); rec_splits == 1
  // means there is nothing to merge and the result goes straight to `out`
  int32_t rec_splits, rec_base;
  // != 0 (only with rec_splits == 1): record 0 of extra_splits per (batch, query head) in the workspace, complete
  // before this launch starts, is merged into this launch's result
  int32_t extra_splits;
  // != 0: this launch writes all rec_splits records of every stream and merges them itself (the workgroup that finishes
  // a stream last does it; the streams' counters, one 64-bit word per (batch, kv head), follow the records in the
  // workspace); the number tells this launch's counts from what the words held before.  0: records are merged by
  // merge_kernel, or there is one record and nothing to merge.
  unsigned long long merge_tag;
  // fused decode step: the token at position seq_len-1 is quantized from k_new/v_new ([B][H_kv][D], element strides
  // nsb, nsh) by the workgroup that owns the last step, before it is read.  k_new == nullptr: plain attention.
  const uint16_t* k_new; const uint16_t* v_new; int in_bf16; int64_t nsb, nsh;
};


// Launchers (each validates nothing: the C ABI layer has done it).  Return hipGetLastError().
hipError_t launch_quantize_append(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new,
                                  int in_dtype, int64_t sb, int64_t sh, int64_t st, int32_t pos, int32_t n_new,
                                  hipStream_t stream);
// Channel-wise keys: tokens go to the residual buffer; completed blocks of g.resid tokens are flushed.
hipError_t launch_seq_append(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype,
                             int64_t sb, int64_t sh, int64_t st, int32_t pos, int32_t n_new, hipStream_t stream);
// ... one new token per sequence at that sequence's own position pos_arr[b] (device; clamped to [0, max_pos])
hipError_t launch_seq_append_one(const Geom& g, const kvq_cache& c, const void* k_new, const void* v_new, int in_dtype,
                                 int64_t sb, int64_t sh, const int32_t* pos_arr, int32_t max_pos, hipStream_t stream);
hipError_t launch_dequantize(const Geom& g, const kvq_cache& c, int32_t t0, int32_t t1, void* k_out, void* v_out,
                             int out_dtype, hipStream_t stream);
hipError_t launch_selftest_quantizer(uint32_t* counters, hipStream_t stream);
hipError_t launch_reconstruction_error(const Geom& g, const kvq_cache& c, const void* k_ref, const void* v_ref,
                                       int ref_dtype, int64_t sb, int64_t sh, int64_t st, int32_t t0, int32_t t1,
                                       double* sums, hipStream_t stream);
// Returns hipErrorInvalidValue if no kernel instance exists for (bits, groups, head ratio).
hipError_t launch_decode_attention(const Geom& g, const kvq_cache& c, const void* q, int q_dtype, int32_t q_heads,
                                   int32_t seq_len, float softmax_scale, void* out, int out_dtype, float* workspace,
                                   const DecodePlan& plan, const AppendOne* append, hipStream_t stream,
                                   const int32_t* seq_lens = nullptr, int32_t lens_offset = 0);
bool decode_supported(const Geom& g, int32_t q_heads);

#if defined(__HIPCC__)
// ---- device-side address helpers (the storage order documented in kvq.h) ----

// Index of (b, h, token t) in the row order of the planes: every plane is [stream][t_cap tokens] with a stream per
// (b, h) when contiguous and per (pool page, h) when paged, so one "virtual token" number addresses all four planes.
__device__ inline int64_t virtual_token(const Geom& g, const int32_t* __restrict__ page_table, int b, int h, int64_t t) {
  if (g.page_shift == 0) return ((int64_t)b * g.kv_heads + h) * g.t_cap + t;
  const int64_t page = page_table[(int64_t)b * g.pages_per_seq + (t >> g.page_shift)];
  return ((page * g.kv_heads + h) << g.page_shift) + (t & ((1 << g.page_shift) - 1));
}

// dword index of meta entry (token t, group g) inside one (b,h) stream
__host__ __device__ inline int64_t meta_index(int64_t t, int g, int ng) { return ((t >> 4) * ng + g) * 16 + (t & 15); }

// Position of value code (u = token inside its 32-token block, d) for bit width b:
// dword index inside the block and bit offset inside the dword.  A lane's piece is 4 dwords, for 1-bit codes 2.
__host__ __device__ inline void v_field(int u, int d, int b, int* dword, int* bit) {
  int x4 = u >> 4, j = (u >> 2) & 3, r = u & 3;
  int i = 4 * x4 + r;
  int x = i & 1, v = i >> 1;
  int q = 4 * (d >> 4) + v;
  int P = 16 / b;
  int e = q / P, p = q % P;
  *dword = b == 1 ? (16 * j + (d & 15)) * 2 + e : (e >> 2) * 256 + (16 * j + (d & 15)) * 4 + (e & 3);
  *bit = 16 * x + b * p;
}
#endif

}  // namespace kvq
