// Shared device helpers of libvista: storage types, the split-L piece walk and
// the launch-error check.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "vista.h"

namespace vista {

// bf16 travels as its 16 bit pattern; fp32 as float.
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float(uint32_t(v.bits) << 16); }

// Round-to-nearest-even fp32 -> bf16 (finite values; the paths never produce NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}
__device__ __forceinline__ void store_as(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_as(bf16_t* p, float v) { p->bits = f32_to_bf16_bits(v); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kHeaderBytes = 256;  // workspace header: int32 device status at byte 0
// Workspace layout of vista_summarize: [header 256 B][seg_user int32[G], padded to 256 B][path-specific data]
__host__ __device__ inline size_t plan_bytes(int64_t G) { return (size_t(G) * sizeof(int) + 255) & ~size_t(255); }

// ---------------------------------------------------------------------------
// Split-L piece walk (pure function of offsets and the segment size).
// Segment g owns flat rows [g*seg, min((g+1)*seg, N)).  find_user returns the
// last user whose first row is <= row; the walk then visits the non-empty
// intersections of the segment with consecutive users.  Every row handed to a
// caller lies inside the segment, hence inside [0, N), whatever offsets hold.
// ---------------------------------------------------------------------------
// offsets[] entries are read at workgroup-uniform addresses; telling the compiler
// so keeps the whole piece walk (and everything derived from it) in scalar registers.
// The walk is also compiled for the host (vista_summarize_schedule reports it).
__host__ __device__ __forceinline__ int64_t load_uniform(const int64_t* p) {
  const int64_t v = *p;
#if defined(__HIP_DEVICE_COMPILE__)
  const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(uint64_t(v)));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(uint64_t(v) >> 32));
  return int64_t((uint64_t(hi) << 32) | lo);
#else
  return v;
#endif
}

__host__ __device__ __forceinline__ int find_user(const int64_t* __restrict__ offsets, int B, int64_t row) {
  int lo = 0, hi = B;  // invariant: offsets[lo] <= row (offsets[0] = 0), answer in [lo, hi)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (load_uniform(offsets + mid) <= row) lo = mid; else hi = mid;
  }
  return lo;
}

struct Piece {
  int user;
  int64_t begin, end;  // flat rows [begin, end)
};

// Advances to the next piece of segment [pos, seg_end); returns false when done.
// `user` and `pos` carry the walk state between calls.
__host__ __device__ __forceinline__ bool next_piece(const int64_t* __restrict__ offsets, int B, int64_t seg_end,
                                                    int& user, int64_t& pos, Piece& out) {
  while (pos < seg_end && user < B) {
    int64_t uend = load_uniform(offsets + user + 1);
    if (uend > pos) {
      int64_t e = uend < seg_end ? uend : seg_end;
      out.user = user;
      out.begin = pos;
      out.end = e;
      pos = e;
      if (uend <= seg_end) ++user;
      return true;
    }
    ++user;
  }
  return false;
}

// A segment as one stream of tiles of `kTileItems` rows.  A tile never spans two
// users: the cursor walks the pieces of the segment and cuts each into tiles, the
// last of which may be ragged.  When the cursor runs off the segment it stays on
// its last tile (still in bounds) with valid = false.  All state is scalar.
constexpr int kTileItems = 32;
struct TileCursor {
  int wuser;        // piece walk: next user to look at
  int64_t wpos;     // piece walk: next flat row (= end of the current piece)
  int user;         // user of the current piece
  int64_t row;      // first row of the current tile
  int tiles_left;   // tiles of the current piece not yet passed, this one included
  int tail;         // valid rows of the piece's last tile, 1..32
  bool valid;

  __host__ __device__ __forceinline__ void enter(const Piece& pc) {
    const int64_t len = pc.end - pc.begin;            // 1 .. segment size: fits 32 bits
    user = pc.user;
    row = pc.begin;
    tiles_left = int((len + kTileItems - 1) / kTileItems);
    tail = int(len - int64_t(tiles_left - 1) * kTileItems);
  }
  // first_user: the user owning row seg_begin (last user whose first row is <= seg_begin)
  __host__ __device__ __forceinline__ void init(const int64_t* __restrict__ offsets, int B, int first_user,
                                                int64_t seg_begin, int64_t seg_end) {
    wuser = first_user;
    wpos = seg_begin;
    Piece pc;
    pc.user = 0;
    pc.begin = seg_begin;
    pc.end = seg_begin + 1;          // overwritten unless offsets are invalid; stays inside [0, N)
    valid = next_piece(offsets, B, seg_end, wuser, wpos, pc);
    enter(pc);
  }
  __host__ __device__ __forceinline__ void advance(const int64_t* __restrict__ offsets, int B, int64_t seg_end) {
    if (!valid) return;
    if (tiles_left > 1) {
      --tiles_left;
      row += kTileItems;
    } else {
      Piece nx;
      if (next_piece(offsets, B, seg_end, wuser, wpos, nx))
        enter(nx);
      else
        valid = false;               // stays on its last tile
    }
  }
  // valid rows of the current tile
  __host__ __device__ __forceinline__ int rows() const { return tiles_left == 1 ? tail : kTileItems; }
};

template <typename Tuple, size_t... I>
inline void fill_arg_pointers(void** ptrs, Tuple& vals, std::index_sequence<I...>) {
  ((ptrs[I] = static_cast<void*>(&std::get<I>(vals))), ...);
}

// Launches a kernel and reports this launch's own status (an error left behind by an
// earlier, unrelated call of the application is neither reported nor cleared).
template <typename... KArgs, typename... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                         Args... args) {
  std::tuple<KArgs...> vals{static_cast<KArgs>(args)...};
  void* ptrs[sizeof...(KArgs) > 0 ? sizeof...(KArgs) : 1];
  fill_arg_pointers(ptrs, vals, std::index_sequence_for<KArgs...>{});
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, stream);
}

#define VISTA_LAUNCH(...)                                              \
  do {                                                                 \
    if (::vista::launch(__VA_ARGS__) != hipSuccess) return VISTA_ERR_HIP; \
  } while (0)

// Launchers implemented in the kernel files (host side).
struct SummarizeArgs {
  vista_summarize_desc desc;
  int seg;            // resolved segment size
  int64_t G;          // segments
  const int* seg_user; // [G] first user of each segment (written by the plan kernel); null: found in the kernel
  float scale_log2;   // scale * log2(e)
  float scale_plain;  // scale
  const void* X;
  const int64_t* offsets;
  const void* Q;
  const void* Wk;
  const void* Wv;
  void* out;
  float* out_scales;  // non-null: out receives int8 codes and this their scales [B, S, H] (cache codec)
  char* workspace;
  hipStream_t stream;
};

size_t generic_summarize_workspace(const vista_summarize_desc& d, int seg);
size_t self_kv_bytes(const vista_summarize_desc& d);
hipError_t launch_self_kv(const vista_summarize_desc& d, const void* Q, const void* Wk, const void* Wv, float* Ks,
                          float* Vs, hipStream_t s);
vista_status generic_summarize(const SummarizeArgs& a);
bool mfma_summarize_supported(const vista_summarize_desc& d);
size_t mfma_summarize_workspace(const vista_summarize_desc& d, int seg);
vista_status mfma_summarize(const SummarizeArgs& a);

bool mfma_qla_supported(const vista_summarize_desc& d);
vista_status mfma_qla_state(const SummarizeArgs& a, float* partials);
// dz: dZs [B][H][32][32] fp32 (device); writes dK and dV rows of every item
vista_status mfma_qla_backward_items(const SummarizeArgs& a, const float* dz, void* d_keys, void* d_values);
size_t qla_backward_workspace(const vista_summarize_desc& d, int seg);
vista_status qla_backward(const SummarizeArgs& a, const void* d_out, void* d_queries, void* d_keys, void* d_values,
                          void* d_self_keys, void* d_self_values);

// summaries either as `summ` (dtype) or, when codes != null, as int8 codes with fp32 scales [B, S, H]
vista_status generic_target_attend(const vista_attend_desc& d, float scale_log2, const void* cand,
                                   const void* summ, const int8_t* codes, const float* scales, void* out,
                                   hipStream_t s);
vista_status generic_quantize(const vista_codec_desc& d, const void* y, int8_t* codes, float* scales, hipStream_t s);
bool mfma_target_attend_supported(const vista_attend_desc& d);
vista_status mfma_target_attend(const vista_attend_desc& d, float scale_log2, const void* cand,
                                const void* summ, const int8_t* codes, const float* scales, void* out,
                                hipStream_t s);

vista_status generic_sglu_ffn(const vista_ffn_desc& d, float eps, const void* y, const void* Wg,
                              const void* Wu, const void* Wo, void* out, hipStream_t s);
bool mfma_sglu_ffn_supported(const vista_ffn_desc& d);
vista_status mfma_sglu_ffn(const vista_ffn_desc& d, float eps, const void* y, const void* Wg,
                           const void* Wu, const void* Wo, void* out, hipStream_t s);

// Validates offsets on the device (status word) and records, for every segment,
// the user that owns its first row (seg_user[g], int32), so that the main
// kernels start their piece walk without a search.
hipError_t launch_plan(const int64_t* offsets, int B, int64_t N, int seg, int64_t G, int* status, int* seg_user,
                       hipStream_t s);

}  // namespace vista
