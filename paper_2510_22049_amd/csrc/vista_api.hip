// C ABI of libvista: argument validation, schedule resolution and dispatch to
// the kernel families.  No allocation, no synchronisation, no global state.
#include <math.h>

#include <mutex>

#include "common.hpp"

using namespace vista;

namespace {

bool dtype_ok(int32_t t) { return t == VISTA_F32 || t == VISTA_BF16; }

// Shape rules of vista_summarize that do not depend on pointers.
vista_status check_summarize_desc(const vista_summarize_desc* d) {
  if (!d) return VISTA_ERR_NULL;
  if (d->B <= 0 || d->S <= 0 || d->d <= 0 || d->H <= 0 || d->total_items < 0) return VISTA_ERR_SHAPE;
  if (d->d % d->H != 0) return VISTA_ERR_SHAPE;
  if (d->q_user_stride != 0 && d->q_user_stride != int64_t(d->S) * d->d) return VISTA_ERR_SHAPE;
  if (d->segment_items < 0 || d->segment_items % 32 != 0) return VISTA_ERR_SHAPE;
  if (!(d->scale >= 0.f) || isinf(d->scale)) return VISTA_ERR_SHAPE;
  if (d->attn < VISTA_ATTN_SOFTMAX || d->attn > VISTA_ATTN_QLA) return VISTA_ERR_UNSUPPORTED;
  if ((d->flags & ~VISTA_FLAG_SELF_TERM) != 0 || d->reserved != 0) return VISTA_ERR_SHAPE;
  if (d->attn == VISTA_ATTN_QLA && d->scale != 0.f) return VISTA_ERR_SHAPE;
  if (!dtype_ok(d->dtype)) return VISTA_ERR_UNSUPPORTED;
  if (d->S > 512 || d->d > 512 || d->d / d->H > 64) return VISTA_ERR_UNSUPPORTED;
  return VISTA_OK;
}

// Default segment size: a function of N alone (never of the device probed at
// run time).  The history is cut into 256 k equal segments -- one workgroup per
// compute unit of the target part and k rounds -- with k the smallest count
// that keeps a segment at or below 8192 items; a multiple of 32, at least 256.
int32_t resolve_segment(const vista_summarize_desc* d) {
  if (d->segment_items > 0) return d->segment_items;
  const int64_t N = d->total_items;
  // quasi-linear attention: a workgroup is four or eight waves with little state, several fit a
  // compute unit, so its history is cut four times finer
  const int64_t units = d->attn == VISTA_ATTN_QLA ? 1024 : 256;
  const int64_t cap = d->attn == VISTA_ATTN_QLA ? 2048 : 8192;
  const int64_t k = (N + units * cap - 1) / (units * cap) > 0 ? (N + units * cap - 1) / (units * cap) : 1;
  int64_t s = (N + units * k - 1) / (units * k);
  s = (s + 31) / 32 * 32;
  if (s < 256) s = 256;
  return int32_t(s);
}

// Scratch of vista_summarize_static: one array per GPU the library runs on, held until the
// process ends.  In host code the name below only stands for the symbol; the array's device
// address is looked up once per device and kept in static_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[VISTA_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* static_scratch_ptr[kMaxDevices] = {};
std::mutex static_scratch_mutex;

// Device address of the current device's scratch array (nullptr on failure).
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(static_scratch_mutex);
  if (!static_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    static_scratch_ptr[dev] = ptr;
  }
  return static_scratch_ptr[dev];
}

}  // namespace

extern "C" {

const char* vista_status_string(int status) {
  switch (status) {
    case VISTA_OK: return "VISTA_OK";
    case VISTA_ERR_NULL: return "VISTA_ERR_NULL: a required pointer is NULL";
    case VISTA_ERR_SHAPE: return "VISTA_ERR_SHAPE: inconsistent or non-positive sizes";
    case VISTA_ERR_OFFSETS: return "VISTA_ERR_OFFSETS: offsets must start at 0, not decrease, end at total_items";
    case VISTA_ERR_UNSUPPORTED: return "VISTA_ERR_UNSUPPORTED: dtype, head width or S outside the supported set";
    case VISTA_ERR_WORKSPACE: return "VISTA_ERR_WORKSPACE: workspace NULL, misaligned or too small";
    case VISTA_ERR_HIP: return "VISTA_ERR_HIP: a kernel launch failed";
    case VISTA_ERR_SCRATCH:
      return "VISTA_ERR_SCRATCH: the call needs more than the library's static scratch (VISTA_STATIC_SCRATCH_BYTES)";
    default: return "unknown vista status";
  }
}

int32_t vista_summarize_segment_items(const vista_summarize_desc* desc) {
  if (check_summarize_desc(desc) != VISTA_OK) return 0;
  return resolve_segment(desc);
}

int64_t vista_summarize_schedule(const vista_summarize_desc* desc, const int64_t* offsets_host, int64_t* tiles,
                                 int64_t max_tiles) {
  if (check_summarize_desc(desc) != VISTA_OK || !offsets_host || max_tiles < 0 || (max_tiles > 0 && !tiles))
    return -1;
  const int seg = resolve_segment(desc);
  const int64_t N = desc->total_items;
  const int64_t G = (N + seg - 1) / seg;
  int64_t n = 0;
  for (int64_t g = 0; g < G; ++g) {
    const int64_t seg_begin = g * seg;
    const int64_t seg_end = seg_begin + seg < N ? seg_begin + seg : N;
    TileCursor c;
    c.init(offsets_host, desc->B, find_user(offsets_host, desc->B, seg_begin), seg_begin, seg_end);
    while (c.valid) {
      if (n < max_tiles) {
        int64_t* t = tiles + 4 * n;
        t[0] = g;
        t[1] = c.user;
        t[2] = c.row;
        t[3] = c.rows();
      }
      ++n;
      c.advance(offsets_host, desc->B, seg_end);
    }
  }
  return n;
}

size_t vista_summarize_workspace_bytes(const vista_summarize_desc* desc) {
  if (check_summarize_desc(desc) != VISTA_OK) return 0;
  int seg = resolve_segment(desc);
  return mfma_summarize_supported(*desc) ? mfma_summarize_workspace(*desc, seg)
                                         : generic_summarize_workspace(*desc, seg);
}

static vista_status summarize_impl(const vista_summarize_desc* desc, const void* history_emb,
                                   const int64_t* offsets, const int64_t* offsets_host,
                                   const void* virtual_queries, const void* W_k, const void* W_v, void* out,
                                   float* out_scales, void* workspace, size_t workspace_bytes, void* hip_stream) {
  vista_status st = check_summarize_desc(desc);
  if (st != VISTA_OK) return st;
  if (out_scales && !mfma_summarize_supported(*desc)) return VISTA_ERR_UNSUPPORTED;
  if (!offsets || !virtual_queries || !W_k || !W_v || !out) return VISTA_ERR_NULL;
  if (desc->total_items > 0 && !history_emb) return VISTA_ERR_NULL;
  if (offsets_host) {
    if (offsets_host[0] != 0 || offsets_host[desc->B] != desc->total_items) return VISTA_ERR_OFFSETS;
    for (int b = 0; b < desc->B; ++b)
      if (offsets_host[b + 1] < offsets_host[b]) return VISTA_ERR_OFFSETS;
  }
  const size_t need = vista_summarize_workspace_bytes(desc);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < need)
    return VISTA_ERR_WORKSPACE;

  SummarizeArgs a;
  a.desc = *desc;
  a.seg = resolve_segment(desc);
  a.G = (desc->total_items + a.seg - 1) / a.seg;
  if (a.G + desc->B > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  // default scale: 1/sqrt(d_h) for the softmax form, none for the pointwise forms (as printed)
  const float scale = desc->scale > 0.f                  ? desc->scale
                      : desc->attn == VISTA_ATTN_SOFTMAX ? 1.f / sqrtf(float(desc->d / desc->H))
                                                         : 1.f;
  a.scale_log2 = scale * kLog2e;
  a.scale_plain = scale;
  a.X = history_emb;
  a.offsets = offsets;
  a.Q = virtual_queries;
  a.Wk = W_k;
  a.Wv = W_v;
  a.out = out;
  a.out_scales = out_scales;
  a.workspace = static_cast<char*>(workspace);
  a.stream = static_cast<hipStream_t>(hip_stream);

  // Offsets already checked on the host: the MFMA path finds each segment's first user
  // itself and its merge kernel clears the status word, so the plan kernel is not needed.
  if (offsets_host && mfma_summarize_supported(*desc)) {
    a.seg_user = nullptr;
    return mfma_summarize(a);
  }
  if (offsets_host && mfma_qla_supported(*desc)) {     // likewise; the finishing kernel clears the status word
    a.seg_user = nullptr;
    return generic_summarize(a);
  }
  int* seg_user = reinterpret_cast<int*>(a.workspace + kHeaderBytes);
  a.seg_user = seg_user;
  if (launch_plan(offsets, desc->B, desc->total_items, a.seg, a.G, reinterpret_cast<int*>(workspace), seg_user,
                  a.stream) != hipSuccess)
    return VISTA_ERR_HIP;
  return mfma_summarize_supported(*desc) ? mfma_summarize(a) : generic_summarize(a);
}

vista_status vista_summarize(const vista_summarize_desc* desc, const void* history_emb,
                             const int64_t* offsets, const int64_t* offsets_host,
                             const void* virtual_queries, const void* W_k, const void* W_v, void* out,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  return summarize_impl(desc, history_emb, offsets, offsets_host, virtual_queries, W_k, W_v, out, nullptr, workspace,
                        workspace_bytes, hip_stream);
}

vista_status vista_summarize_q8(const vista_summarize_desc* desc, const void* history_emb,
                                const int64_t* offsets, const int64_t* offsets_host,
                                const void* virtual_queries, const void* W_k, const void* W_v, int8_t* out_codes,
                                float* out_scales, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!out_scales) return VISTA_ERR_NULL;
  return summarize_impl(desc, history_emb, offsets, offsets_host, virtual_queries, W_k, W_v, out_codes, out_scales,
                        workspace, workspace_bytes, hip_stream);
}

vista_status vista_quantize_summaries(const vista_codec_desc* desc, const void* y, int8_t* codes, float* scales,
                                      void* hip_stream) {
  if (!desc) return VISTA_ERR_NULL;
  if (desc->rows <= 0 || desc->d <= 0 || desc->H <= 0 || desc->d % desc->H != 0) return VISTA_ERR_SHAPE;
  if (!dtype_ok(desc->dtype) || desc->d / desc->H > 64) return VISTA_ERR_UNSUPPORTED;
  if (!y || !codes || !scales) return VISTA_ERR_NULL;
  return generic_quantize(*desc, y, codes, scales, static_cast<hipStream_t>(hip_stream));
}

size_t vista_qla_backward_workspace_bytes(const vista_summarize_desc* desc) {
  if (check_summarize_desc(desc) != VISTA_OK || desc->attn != VISTA_ATTN_QLA) return 0;
  return qla_backward_workspace(*desc, resolve_segment(desc));
}

vista_status vista_qla_backward(const vista_summarize_desc* desc, const void* history_emb, const int64_t* offsets,
                                const int64_t* offsets_host, const void* virtual_queries, const void* W_k,
                                const void* W_v, const void* d_out, void* d_queries, void* d_keys, void* d_values,
                                void* d_self_keys, void* d_self_values, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  vista_status st = check_summarize_desc(desc);
  if (st != VISTA_OK) return st;
  if (desc->attn != VISTA_ATTN_QLA) return VISTA_ERR_UNSUPPORTED;
  if (!offsets || !virtual_queries || !W_k || !W_v || !d_out || !d_queries) return VISTA_ERR_NULL;
  if ((desc->flags & VISTA_FLAG_SELF_TERM) && (!d_self_keys || !d_self_values)) return VISTA_ERR_NULL;
  if (desc->total_items > 0 && (!history_emb || !d_keys || !d_values)) return VISTA_ERR_NULL;
  if (offsets_host) {
    if (offsets_host[0] != 0 || offsets_host[desc->B] != desc->total_items) return VISTA_ERR_OFFSETS;
    for (int b = 0; b < desc->B; ++b)
      if (offsets_host[b + 1] < offsets_host[b]) return VISTA_ERR_OFFSETS;
  }
  const size_t need = vista_qla_backward_workspace_bytes(desc);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < need)
    return VISTA_ERR_WORKSPACE;
  SummarizeArgs a;
  a.desc = *desc;
  a.seg = resolve_segment(desc);
  a.G = (desc->total_items + a.seg - 1) / a.seg;
  if (a.G + desc->B > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  a.scale_log2 = kLog2e;
  a.scale_plain = 1.f;
  a.X = history_emb;
  a.offsets = offsets;
  a.Q = virtual_queries;
  a.Wk = W_k;
  a.Wv = W_v;
  a.out = nullptr;
  a.out_scales = nullptr;
  a.workspace = static_cast<char*>(workspace);
  a.stream = static_cast<hipStream_t>(hip_stream);
  if (offsets_host && mfma_qla_supported(*desc)) {
    // offsets already checked on the host: the streaming kernels find each segment's first user
    // themselves and the state-gradient kernel clears the status word
    a.seg_user = nullptr;
    return qla_backward(a, d_out, d_queries, d_keys, d_values, d_self_keys, d_self_values);
  }
  int* seg_user = reinterpret_cast<int*>(a.workspace + kHeaderBytes);
  a.seg_user = seg_user;
  if (launch_plan(offsets, desc->B, desc->total_items, a.seg, a.G, reinterpret_cast<int*>(workspace), seg_user,
                  a.stream) != hipSuccess)
    return VISTA_ERR_HIP;
  return qla_backward(a, d_out, d_queries, d_keys, d_values, d_self_keys, d_self_values);
}

vista_status vista_summarize_static(const vista_summarize_desc* desc, const void* history_emb,
                                    const int64_t* offsets, const int64_t* offsets_host,
                                    const void* virtual_queries, const void* W_k, const void* W_v, void* out,
                                    void* hip_stream) {
  vista_status st = check_summarize_desc(desc);
  if (st != VISTA_OK) return st;
  const size_t need = vista_summarize_workspace_bytes(desc);
  if (need > size_t(VISTA_STATIC_SCRATCH_BYTES)) return VISTA_ERR_SCRATCH;
  void* ws = static_scratch();
  if (!ws) return VISTA_ERR_HIP;
  // Nothing in the scratch has to start at zero: every record the merge reads and the status
  // word are written by this call's own kernels before they are read.
  return vista_summarize(desc, history_emb, offsets, offsets_host, virtual_queries, W_k, W_v, out, ws,
                         size_t(VISTA_STATIC_SCRATCH_BYTES), hip_stream);
}

static vista_status target_attend_impl(const vista_attend_desc* desc, const void* candidates,
                                       const void* summaries, const int8_t* codes, const float* scales, void* out,
                                       void* hip_stream) {
  if (!desc) return VISTA_ERR_NULL;
  if (desc->B <= 0 || desc->C <= 0 || desc->S <= 0 || desc->d <= 0 || desc->H <= 0) return VISTA_ERR_SHAPE;
  if (desc->d % desc->H != 0) return VISTA_ERR_SHAPE;
  if (!(desc->scale >= 0.f) || isinf(desc->scale)) return VISTA_ERR_SHAPE;
  if ((desc->flags & ~VISTA_FLAG_SELF_TERM) != 0) return VISTA_ERR_SHAPE;
  if (!dtype_ok(desc->dtype)) return VISTA_ERR_UNSUPPORTED;
  if (desc->S > 512 || desc->d / desc->H > 64) return VISTA_ERR_UNSUPPORTED;
  if (!candidates || !out || (!summaries && !(codes && scales))) return VISTA_ERR_NULL;
  const float scale = desc->scale > 0.f ? desc->scale : 1.f / sqrtf(float(desc->d / desc->H));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // the MFMA path reads 16 codes at a time: rows of codes must then be 16-byte aligned
  const bool aligned = !codes || (desc->d % 16 == 0 && (reinterpret_cast<uintptr_t>(codes) & 15) == 0);
  if (mfma_target_attend_supported(*desc) && aligned)
    return mfma_target_attend(*desc, scale * kLog2e, candidates, summaries, codes, scales, out, s);
  return generic_target_attend(*desc, scale * kLog2e, candidates, summaries, codes, scales, out, s);
}

vista_status vista_target_attend(const vista_attend_desc* desc, const void* candidates,
                                 const void* summaries, void* out, void* hip_stream) {
  if (desc && !summaries) return VISTA_ERR_NULL;
  return target_attend_impl(desc, candidates, summaries, nullptr, nullptr, out, hip_stream);
}

vista_status vista_target_attend_q8(const vista_attend_desc* desc, const void* candidates, const int8_t* codes,
                                    const float* scales, void* out, void* hip_stream) {
  if (desc && (!codes || !scales)) return VISTA_ERR_NULL;
  return target_attend_impl(desc, candidates, nullptr, codes, scales, out, hip_stream);
}

vista_status vista_sglu_ffn(const vista_ffn_desc* desc, const void* y, const void* W_g, const void* W_u,
                            const void* W_o, void* out, void* hip_stream) {
  if (!desc) return VISTA_ERR_NULL;
  if (desc->rows <= 0 || desc->d <= 0 || desc->d_ff <= 0) return VISTA_ERR_SHAPE;
  if (!(desc->eps >= 0.f) || isinf(desc->eps)) return VISTA_ERR_SHAPE;
  if (!dtype_ok(desc->dtype)) return VISTA_ERR_UNSUPPORTED;
  if (desc->d > 512 || desc->d_ff > 1024 || desc->d % 32 != 0 || desc->d_ff % 32 != 0)
    return VISTA_ERR_UNSUPPORTED;
  if (!y || !W_g || !W_u || !W_o || !out) return VISTA_ERR_NULL;
  const float eps = desc->eps > 0.f ? desc->eps : 1e-6f;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (mfma_sglu_ffn_supported(*desc)) return mfma_sglu_ffn(*desc, eps, y, W_g, W_u, W_o, out, s);
  return generic_sglu_ffn(*desc, eps, y, W_g, W_u, W_o, out, s);
}

}  // extern "C"
