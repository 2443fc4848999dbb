// C ABI of libkvq: argument validation on the host, then one launcher call per entry point.
#include "kvq_internal.h"

#include <atomic>

namespace {

bool bits_ok(int b) { return b == 1 || b == 2 || b == 3 || b == 4 || b == 6 || b == 8 || b == 16; }
bool group_ok(int g) { return g == 32 || g == 64 || g == 128; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks everything about a layout that does not depend on the call.
kvq_status check_layout(const kvq_layout* L) {
  if (!L) return KVQ_ERR_INVALID_ARG;
  if (L->batch <= 0 || L->kv_heads <= 0 || L->max_seq <= 0 || L->head_dim <= 0) return KVQ_ERR_INVALID_ARG;
  if (!bits_ok(L->bits_k) || !bits_ok(L->bits_v)) return KVQ_ERR_INVALID_ARG;
  if (L->bits_k != 16 && (!group_ok(L->group_k) || L->head_dim % L->group_k)) return KVQ_ERR_INVALID_ARG;
  if (L->bits_v != 16 && (!group_ok(L->group_v) || L->head_dim % L->group_v)) return KVQ_ERR_INVALID_ARG;
  if ((L->axis_k != KVQ_AXIS_HEAD_DIM && L->axis_k != KVQ_AXIS_SEQ) ||
      (L->axis_v != KVQ_AXIS_HEAD_DIM && L->axis_v != KVQ_AXIS_SEQ))
    return KVQ_ERR_INVALID_ARG;
  if (L->raw_dtype != KVQ_F16 && L->raw_dtype != KVQ_BF16) return KVQ_ERR_INVALID_ARG;
  if (L->rotate_k != 0 && L->rotate_k != 1) return KVQ_ERR_INVALID_ARG;
  if (L->rotate_k && L->bits_k == 16) return KVQ_ERR_INVALID_ARG;   // the rotation exists for quantized keys only
  if (L->rotate_v != 0 && L->rotate_v != 1) return KVQ_ERR_INVALID_ARG;
  if (L->rotate_v && L->bits_v == 16) return KVQ_ERR_INVALID_ARG;
  if (L->page_tokens) {
    if (L->page_tokens < 64 || L->page_tokens > 65536 || (L->page_tokens & (L->page_tokens - 1)) || L->n_pages <= 0)
      return KVQ_ERR_INVALID_ARG;
    if ((int64_t)L->n_pages * L->kv_heads * L->page_tokens > ((int64_t)1 << 40)) return KVQ_ERR_UNSUPPORTED;
  }
  if (L->head_dim != kvq::kHeadDim) return KVQ_ERR_UNSUPPORTED;
  if (L->axis_v != KVQ_AXIS_HEAD_DIM) return KVQ_ERR_UNSUPPORTED;
  if (L->resid_len < 0) return KVQ_ERR_INVALID_ARG;
  if (kvq::has_residual(*L)) {
    // a residual buffer: quantized keys and values; keys may be rotated
    if (L->bits_k == 16 || L->bits_v == 16 || L->rotate_v) return KVQ_ERR_INVALID_ARG;
    const int32_t slots = kvq::residual_slots(*L);
    if (L->axis_k == KVQ_AXIS_SEQ) {
      // channel-wise keys: groups of 32, 64 or 128 tokens; a buffer of 64 or 128 slots that a whole number of groups fills
      if (slots % L->group_k != 0) return KVQ_ERR_INVALID_ARG;
      if (slots != 64 && slots != 128) return KVQ_ERR_UNSUPPORTED;
      // (paged planes: a 64-token page takes blocks of 64 tokens with one group each)
      if (L->page_tokens && (slots != 64 || L->group_k != 64)) return KVQ_ERR_UNSUPPORTED;
    } else if (slots != kvq::kSeqGroup) {
      return KVQ_ERR_UNSUPPORTED;                  // token-wise keys: a buffer of 64 slots
    }
  }
  if ((int64_t)L->batch * L->kv_heads > 65535) return KVQ_ERR_UNSUPPORTED;
  if (L->max_seq > (1 << 24)) return KVQ_ERR_UNSUPPORTED;   // a (b,h) stream of any plane stays below 4 GiB
  return KVQ_OK;
}

kvq_status check_cache(const kvq_layout* L, const kvq_cache* c) {
  if (!c || !c->k_codes || !c->v_codes) return KVQ_ERR_INVALID_ARG;
  if (L->bits_k != 16 && !c->k_meta) return KVQ_ERR_INVALID_ARG;
  if (L->bits_v != 16 && !c->v_meta) return KVQ_ERR_INVALID_ARG;
  if (!aligned16(c->k_codes) || !aligned16(c->v_codes) || !aligned16(c->k_meta) || !aligned16(c->v_meta))
    return KVQ_ERR_INVALID_ARG;
  if (kvq::has_residual(*L) && (!c->k_resid || !c->v_resid || !aligned16(c->k_resid) || !aligned16(c->v_resid)))
    return KVQ_ERR_INVALID_ARG;
  if (L->page_tokens && (!c->page_table || (reinterpret_cast<uintptr_t>(c->page_table) & 3u))) return KVQ_ERR_INVALID_ARG;
  if (L->bits_v != 16 && (!c->v_scale_exp || (reinterpret_cast<uintptr_t>(c->v_scale_exp) & 3u))) return KVQ_ERR_INVALID_ARG;
  return KVQ_OK;
}

}  // namespace

extern "C" {

kvq_status kvq_cache_bytes(const kvq_layout* layout, size_t bytes_out[4]) {
  kvq_status st = check_layout(layout);
  if (st != KVQ_OK) return st;
  if (!bytes_out) return KVQ_ERR_INVALID_ARG;
  const kvq::Geom g = kvq::make_geom(*layout);
  const int64_t streams = layout->page_tokens ? (int64_t)layout->n_pages * g.kv_heads : (int64_t)g.batch * g.kv_heads;
  bytes_out[0] = (size_t)(streams * g.kc_stream);
  bytes_out[1] = (size_t)(streams * g.km_stream);
  bytes_out[2] = (size_t)(streams * g.vc_stream);
  bytes_out[3] = (size_t)(streams * g.vm_stream);
  return KVQ_OK;
}

kvq_status kvq_residual_bytes(const kvq_layout* layout, size_t bytes_out[2]) {
  kvq_status st = check_layout(layout);
  if (st != KVQ_OK) return st;
  if (!bytes_out) return KVQ_ERR_INVALID_ARG;
  const size_t n = kvq::has_residual(*layout)
                       ? (size_t)layout->batch * layout->kv_heads * kvq::residual_slots(*layout) * kvq::kHeadDim * 2 : 0;
  bytes_out[0] = n;
  bytes_out[1] = n;
  return KVQ_OK;
}

kvq_status kvq_decode_workspace_bytes(const kvq_layout* layout, int32_t q_heads, int32_t seq_len, size_t* bytes_out) {
  kvq_status st = check_layout(layout);
  if (st != KVQ_OK) return st;
  if (!bytes_out || q_heads <= 0 || q_heads % layout->kv_heads || seq_len <= 0) return KVQ_ERR_INVALID_ARG;
  if (seq_len > layout->max_seq) return KVQ_ERR_CAPACITY;
  const kvq::Geom g = kvq::make_geom(*layout);
  // one record of (head_dim + 2) floats per (batch, query head, split), padded to 16 bytes; sized for the most records
  // any length up to seq_len writes, so that the figure never shrinks as seq_len grows
  const int32_t records = kvq::decode_records_bound(g, seq_len);
  // ... followed by one 64-bit counter of finished workgroups per (batch, kv head)
  *bytes_out = records == 1 ? 0 : (size_t)layout->batch * q_heads * records * (kvq::kHeadDim + 4) * sizeof(float) +
                                      (((size_t)layout->batch * layout->kv_heads * 8 + 15) & ~(size_t)15);
  return KVQ_OK;
}

kvq_status kvq_quantize_append(const kvq_layout* layout, const kvq_cache* cache, const void* k_new, const void* v_new,
                               kvq_dtype in_dtype, int64_t stride_b, int64_t stride_h, int64_t stride_t, int32_t pos,
                               int32_t n_new, void* stream) {
  kvq_status st = check_layout(layout);
  if (st != KVQ_OK) return st;
  st = check_cache(layout, cache);
  if (st != KVQ_OK) return st;
  if (pos < 0 || n_new < 0) return KVQ_ERR_INVALID_ARG;
  if ((int64_t)pos + n_new > layout->max_seq) return KVQ_ERR_CAPACITY;
  if (n_new == 0) return KVQ_OK;
  if (!k_new || !v_new) return KVQ_ERR_INVALID_ARG;
  if (in_dtype != KVQ_F16 && in_dtype != KVQ_BF16) return KVQ_ERR_INVALID_ARG;
  if ((layout->bits_k == 16 || layout->bits_v == 16) && (int)in_dtype != layout->raw_dtype) return KVQ_ERR_INVALID_ARG;
  // rows are read with 16-byte loads
  if (!aligned16(k_new) || !aligned16(v_new) || stride_b % 8 || stride_h % 8 || stride_t % 8 || stride_t < layout->head_dim)
    return KVQ_ERR_INVALID_ARG;
  const kvq::Geom g = kvq::make_geom(*layout);
  if (kvq::has_residual(*layout)) {
    if ((int)in_dtype != layout->raw_dtype) return KVQ_ERR_INVALID_ARG;   // the residual buffer keeps the input patterns
    hipError_t e = kvq::launch_seq_append(g, *cache, k_new, v_new, in_dtype, stride_b, stride_h, stride_t, pos, n_new,
                                          (hipStream_t)stream);
    return e == hipSuccess ? KVQ_OK : KVQ_ERR_DEVICE;
  }
  hipError_t e = kvq::launch_quantize_append(g, *cache, k_new, v_new, in_dtype, stride_b, stride_h, stride_t, pos, n_new,
                                             (hipStream_t)stream);
  return e == hipSuccess ? KVQ_OK : KVQ_ERR_DEVICE;
}

namespace {
// Everything that can be wrong with a decode call, checked without launching anything.
kvq_status decode_check(const kvq_layout* layout, const kvq_cache* cache, const void* q, kvq_dtype q_dtype, int32_t q_heads,
                        int32_t seq_len, float softmax_scale, void* out, kvq_dtype out_dtype, void* workspace,
                        size_t workspace_bytes, bool fused_append) {
  kvq_status st = check_layout(layout);
  if (st != KVQ_OK) return st;
  st = check_cache(layout, cache);
  if (st != KVQ_OK) return st;
  if (!q || !out || q_heads <= 0 || q_heads % layout->kv_heads || seq_len <= 0) return KVQ_ERR_INVALID_ARG;
  if (seq_len > layout->max_seq) return KVQ_ERR_CAPACITY;
  if (q_dtype != KVQ_F16 && q_dtype != KVQ_BF16) return KVQ_ERR_INVALID_ARG;
  if (out_dtype != KVQ_F32 && out_dtype != KVQ_F16 && out_dtype != KVQ_BF16) return KVQ_ERR_INVALID_ARG;
  if (!(softmax_scale > 0.0f) || softmax_scale > 3.0e38f) return KVQ_ERR_INVALID_ARG;   // positive and finite
  if (!aligned16(q) || !aligned16(out)) return KVQ_ERR_INVALID_ARG;
  const kvq::Geom g = kvq::make_geom(*layout);
  if (!kvq::decode_supported(g, q_heads)) return KVQ_ERR_UNSUPPORTED;
  if (kvq::has_residual(*layout) && (int)q_dtype != layout->raw_dtype) return KVQ_ERR_UNSUPPORTED;   // residual tail: as unquantized
  if (layout->bits_k == 16 && (int)q_dtype != layout->raw_dtype) return KVQ_ERR_UNSUPPORTED;   // matrix operands share a type
  if ((layout->bits_k == 16 || layout->bits_v == 16) && fused_append) return KVQ_ERR_UNSUPPORTED; // fused append: both tensors quantized
  size_t need = 0;
  st = kvq_decode_workspace_bytes(layout, q_heads, seq_len, &need);
  if (st != KVQ_OK) return st;
  if (need && (!workspace || workspace_bytes < need || !aligned16(workspace))) return KVQ_ERR_WORKSPACE;
  return KVQ_OK;
}

// seq_lens (device, may be null) + lens_offset: per-sequence lengths inside the bound seq_len.
kvq_status decode_common(const kvq_layout* layout, const kvq_cache* cache, const void* q, kvq_dtype q_dtype, int32_t q_heads,
                         int32_t seq_len, float softmax_scale, void* out, kvq_dtype out_dtype, void* workspace,
                         size_t workspace_bytes, const kvq::AppendOne* app, void* stream,
                         const int32_t* seq_lens = nullptr, int32_t lens_offset = 0) {
  kvq_status st = decode_check(layout, cache, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, workspace,
                               workspace_bytes, app != nullptr);
  if (st != KVQ_OK) return st;
  const kvq::Geom g = kvq::make_geom(*layout);
  const kvq::DecodePlan plan = kvq::plan_decode(g, seq_len);
  hipError_t e = kvq::launch_decode_attention(g, *cache, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype,
                                              (float*)workspace, plan, app, (hipStream_t)stream, seq_lens, lens_offset);
  return e == hipSuccess ? KVQ_OK : KVQ_ERR_DEVICE;
}
}  // namespace

kvq_status kvq_decode_attention(const kvq_layout* layout, const kvq_cache* cache, const void* q, kvq_dtype q_dtype,
                                int32_t q_heads, int32_t seq_len, float softmax_scale, void* out, kvq_dtype out_dtype,
                                void* workspace, size_t workspace_bytes, void* stream) {
  return decode_common(layout, cache, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, workspace,
                       workspace_bytes, nullptr, stream);
}

}  // extern "C"

// ---- the entry point that allocates nothing: its partial records live in an array of the device code -----------------
namespace {
// One copy per GPU, held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress: the
// kernels get the device address that call returns, never the name.
static __device__ __align__(256) unsigned char scratch[KVQ_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU (null: not looked up yet)

// The address of this GPU's copy of `scratch` (the current device's), looked up once per device.
hipError_t static_scratch(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // (two threads racing here store the same address)
  }
  *ptr = p;
  return hipSuccess;
}
}  // namespace

extern "C" {

kvq_status kvq_decode_attention_static(const kvq_layout* layout, const kvq_cache* cache, const void* q, kvq_dtype q_dtype,
                                       int32_t q_heads, int32_t seq_len, float softmax_scale, void* out,
                                       kvq_dtype out_dtype, void* stream) {
  size_t need = 0;
  kvq_status st = kvq_decode_workspace_bytes(layout, q_heads, seq_len, &need);
  if (st != KVQ_OK) return st;
  if (need > KVQ_STATIC_SCRATCH_BYTES) return KVQ_ERR_STATIC_SCRATCH;
  void* ws = nullptr;
  if (need && static_scratch(&ws) != hipSuccess) return KVQ_ERR_DEVICE;
  return decode_common(layout, cache, q, q_dtype, q_heads, seq_len, softmax_scale, out, out_dtype, ws,
                       need ? KVQ_STATIC_SCRATCH_BYTES : 0, nullptr, stream);
}

kvq_status kvq_decode_step(const kvq_layout* layout, const kvq_cache* cache, const void* k_new, const void* v_new,
                           kvq_dtype in_dtype, int64_t stride_b, int64_t stride_h, int32_t pos, const void* q,
                           kvq_dtype q_dtype, int32_t q_heads, float softmax_scale, void* out, kvq_dtype out_dtype,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (!layout) return KVQ_ERR_INVALID_ARG;
  if (pos < 0) return KVQ_ERR_INVALID_ARG;
  if (pos >= layout->max_seq) return KVQ_ERR_CAPACITY;
  if (!k_new || !v_new || (in_dtype != KVQ_F16 && in_dtype != KVQ_BF16)) return KVQ_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || stride_b % 8 || stride_h % 8) return KVQ_ERR_INVALID_ARG;
  if (kvq::has_residual(*layout)) {
    // the new token goes through the residual buffer (and may flush a block): two calls in a row,
    // the second one checked before the first one runs
    kvq_status st = decode_check(layout, cache, q, q_dtype, q_heads, pos + 1, softmax_scale, out, out_dtype, workspace,
                                 workspace_bytes, false);
    if (st != KVQ_OK) return st;
    st = kvq_quantize_append(layout, cache, k_new, v_new, in_dtype, stride_b, stride_h, layout->head_dim, pos, 1,
                                        stream);
    if (st != KVQ_OK) return st;
    return decode_common(layout, cache, q, q_dtype, q_heads, pos + 1, softmax_scale, out, out_dtype, workspace,
                         workspace_bytes, nullptr, stream);
  }
  const kvq::AppendOne app{k_new, v_new, (int)in_dtype, stride_b, stride_h};
  return decode_common(layout, cache, q, q_dtype, q_heads, pos + 1, softmax_scale, out, out_dtype, workspace,
                       workspace_bytes, &app, stream);
}

kvq_status kvq_decode_attention_varlen(const kvq_layout* layout, const kvq_cache* cache, const void* q, kvq_dtype q_dtype,
                                       int32_t q_heads, const int32_t* seq_lens, int32_t max_seq_len, float softmax_scale,
                                       void* out, kvq_dtype out_dtype, void* workspace, size_t workspace_bytes,
                                       void* stream) {
  if (!seq_lens || (reinterpret_cast<uintptr_t>(seq_lens) & 3u)) return KVQ_ERR_INVALID_ARG;
  return decode_common(layout, cache, q, q_dtype, q_heads, max_seq_len, softmax_scale, out, out_dtype, workspace,
                       workspace_bytes, nullptr, stream, seq_lens, 0);
}

kvq_status kvq_decode_step_varlen(const kvq_layout* layout, const kvq_cache* cache, const void* k_new, const void* v_new,
                                  kvq_dtype in_dtype, int64_t stride_b, int64_t stride_h, const int32_t* pos,
                                  int32_t max_pos, const void* q, kvq_dtype q_dtype, int32_t q_heads, float softmax_scale,
                                  void* out, kvq_dtype out_dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (!layout) return KVQ_ERR_INVALID_ARG;
  if (!pos || (reinterpret_cast<uintptr_t>(pos) & 3u) || max_pos < 0) return KVQ_ERR_INVALID_ARG;
  if (max_pos >= layout->max_seq) return KVQ_ERR_CAPACITY;
  if (!k_new || !v_new || (in_dtype != KVQ_F16 && in_dtype != KVQ_BF16)) return KVQ_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || stride_b % 8 || stride_h % 8) return KVQ_ERR_INVALID_ARG;
  if (kvq::has_residual(*layout)) {
    // every sequence's new token goes through its residual buffer at its own position (and may
    // flush a block there), then the attention with lengths pos[b] + 1; everything is checked before anything runs
    kvq_status st = decode_check(layout, cache, q, q_dtype, q_heads, max_pos + 1, softmax_scale, out, out_dtype, workspace,
                                 workspace_bytes, false);
    if (st != KVQ_OK) return st;
    if ((int)in_dtype != layout->raw_dtype) return KVQ_ERR_INVALID_ARG;     // the buffer keeps patterns of raw_dtype
    const kvq::Geom g = kvq::make_geom(*layout);
    if (kvq::launch_seq_append_one(g, *cache, k_new, v_new, (int)in_dtype, stride_b, stride_h, pos, max_pos,
                                   (hipStream_t)stream) != hipSuccess)
      return KVQ_ERR_DEVICE;
    return decode_common(layout, cache, q, q_dtype, q_heads, max_pos + 1, softmax_scale, out, out_dtype, workspace,
                         workspace_bytes, nullptr, stream, pos, 1);
  }
  const kvq::AppendOne app{k_new, v_new, (int)in_dtype, stride_b, stride_h};
  return decode_common(layout, cache, q, q_dtype, q_heads, max_pos + 1, softmax_scale, out, out_dtype, workspace,
                       workspace_bytes, &app, stream, pos, 1);
}

kvq_status kvq_dequantize(const kvq_layout* layout, const kvq_cache* cache, int32_t t0, int32_t t1, void* k_out,
                          void* v_out, kvq_dtype out_dtype, void* stream) {
  kvq_status st = check_layout(layout);
  if (st != KVQ_OK) return st;
  st = check_cache(layout, cache);
  if (st != KVQ_OK) return st;
  if (t0 < 0 || t1 < t0) return KVQ_ERR_INVALID_ARG;
  if (t1 > layout->max_seq) return KVQ_ERR_CAPACITY;
  if (out_dtype != KVQ_F32 && out_dtype != KVQ_F16 && out_dtype != KVQ_BF16) return KVQ_ERR_INVALID_ARG;
  if (!k_out && !v_out) return KVQ_ERR_INVALID_ARG;
  const kvq::Geom g = kvq::make_geom(*layout);
  hipError_t e = kvq::launch_dequantize(g, *cache, t0, t1, k_out, v_out, out_dtype, (hipStream_t)stream);
  return e == hipSuccess ? KVQ_OK : KVQ_ERR_DEVICE;
}

kvq_status kvq_reconstruction_error(const kvq_layout* layout, const kvq_cache* cache, const void* k_ref,
                                    const void* v_ref, kvq_dtype ref_dtype, int64_t stride_b, int64_t stride_h,
                                    int64_t stride_t, int32_t t0, int32_t t1, double* sums, void* stream) {
  kvq_status st = check_layout(layout);
  if (st != KVQ_OK) return st;
  st = check_cache(layout, cache);
  if (st != KVQ_OK) return st;
  if (t0 < 0 || t1 < t0) return KVQ_ERR_INVALID_ARG;
  if (t1 > layout->max_seq) return KVQ_ERR_CAPACITY;
  if (!sums || (reinterpret_cast<uintptr_t>(sums) & 7u)) return KVQ_ERR_INVALID_ARG;
  if (ref_dtype != KVQ_F16 && ref_dtype != KVQ_BF16) return KVQ_ERR_INVALID_ARG;
  if (t1 > t0) {                                       // an empty range reads no reference row
    if (!k_ref && !v_ref) return KVQ_ERR_INVALID_ARG;
    if (!aligned16(k_ref) || !aligned16(v_ref) || stride_b % 8 || stride_h % 8 || stride_t % 8 || stride_t < layout->head_dim)
      return KVQ_ERR_INVALID_ARG;
  }
  const kvq::Geom g = kvq::make_geom(*layout);
  hipError_t e = kvq::launch_reconstruction_error(g, *cache, k_ref, v_ref, ref_dtype, stride_b, stride_h, stride_t, t0, t1,
                                                  sums, (hipStream_t)stream);
  return e == hipSuccess ? KVQ_OK : KVQ_ERR_DEVICE;
}

kvq_status kvq_selftest_quantizer(uint32_t* counters, void* stream) {
  if (!counters || (reinterpret_cast<uintptr_t>(counters) & 3u)) return KVQ_ERR_INVALID_ARG;
  return kvq::launch_selftest_quantizer(counters, (hipStream_t)stream) == hipSuccess ? KVQ_OK : KVQ_ERR_DEVICE;
}

const char* kvq_status_string(kvq_status status) {
  switch (status) {
    case KVQ_OK: return "ok";
    case KVQ_ERR_INVALID_ARG: return "invalid argument";
    case KVQ_ERR_UNSUPPORTED: return "unsupported configuration";
    case KVQ_ERR_CAPACITY: return "beyond cache capacity";
    case KVQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KVQ_ERR_DEVICE: return "HIP runtime error at launch";
    case KVQ_ERR_STATIC_SCRATCH: return "needs more partial-record bytes than the static scratch array holds";
  }
  return "unknown status";
}

}  // extern "C"
