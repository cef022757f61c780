// Plain fp32-ALU kernels of libvista: any dtype, any S <= 512, head width <= 64.
// They carry the fp32 configuration and every shape the MFMA kernels do not
// take.  One thread owns one query (stage 1) or one (candidate, head) pair
// (stage 2) and streams the keys with an online softmax in base 2.
#include "common.hpp"

namespace vista {

constexpr int kMaxDh = 64;

// ------------------------------------------------------------------ checks

// Block 0 validates offsets and publishes the status word; every block takes a
// grid-stride share of the segments and finds each one's first user by binary search.
__global__ void plan_kernel(const int64_t* __restrict__ offsets, int B, int64_t N, int seg, int64_t G,
                            int* __restrict__ status, int* __restrict__ seg_user) {
  if (blockIdx.x == 0) {
    __shared__ int bad;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    int local = 0;
    for (int64_t b = threadIdx.x; b <= B; b += blockDim.x) {
      const int64_t o = offsets[b];
      if (b == 0 && o != 0) local = 1;
      if (b == B && o != N) local = 1;
      if (b < B && offsets[b + 1] < o) local = 1;
    }
    if (local) atomicOr(&bad, 1);
    __syncthreads();
    if (threadIdx.x == 0) *status = bad ? int(VISTA_ERR_OFFSETS) : 0;
  }
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t g = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; g < G; g += stride) {
    const int64_t row = g * seg;
    int lo = 0, hi = B;               // last user whose first row is <= row
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (offsets[mid] <= row) lo = mid; else hi = mid;
    }
    seg_user[g] = lo;
  }
}

hipError_t launch_plan(const int64_t* offsets, int B, int64_t N, int seg, int64_t G, int* status, int* seg_user,
                       hipStream_t s) {
  int blocks = int((G + 255) / 256);
  if (blocks < 1) blocks = 1;
  if (blocks > 1024) blocks = 1024;
  return launch(plan_kernel, dim3(blocks), dim3(256), 0, s, offsets, B, N, seg, G, status, seg_user);
}

// -------------------------------------------------- stage 1: K/V projection
// K = X W_k, V = X W_v in fp32 (Sec. 3.2.1: K and V of shape (L, d)).
// Block = 256 threads = (256/d') rows x d' columns; each thread one (row, col).
template <typename T>
__global__ void project_kernel(const T* __restrict__ X, const T* __restrict__ Wk, const T* __restrict__ Wv,
                               float* __restrict__ K, float* __restrict__ V, int64_t N, int d) {
  int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= N * d) return;
  int64_t row = idx / d;
  int col = int(idx - row * d);
  const T* x = X + row * d;
  float k = 0.f, v = 0.f;
  for (int t = 0; t < d; ++t) {
    float xv = to_f32(x[t]);
    k = fmaf(xv, to_f32(Wk[int64_t(t) * d + col]), k);
    v = fmaf(xv, to_f32(Wv[int64_t(t) * d + col]), v);
  }
  K[idx] = k;
  V[idx] = v;
}

// ------------------------------------------- stage 1: streaming attention
// Partial slot layout: [slot][h][query][dh + 2] fp32 = un-normalised O, then
// l (sum of 2^(s-m)) and m (running maximum of s, base-2 units).
// SILU = true: the pointwise score form of App. B, o += SiLU(s) v with no maximum and no
// denominator (the record's l and m stay 0; the merge divides by the user's length).  The
// score then arrives in natural units (scale_log2 carries the plain scale).
template <typename T, bool SILU>
__global__ void attend_history_kernel(const float* __restrict__ K, const float* __restrict__ V,
                                      const T* __restrict__ Q, int64_t q_user_stride,
                                      const int64_t* __restrict__ offsets, int B, int S, int d, int H,
                                      float scale_log2, int64_t N, int seg, const int* __restrict__ seg_user,
                                      float* __restrict__ partials) {
  const int dh = d / H;
  const int h = blockIdx.y;
  const int64_t seg_begin = int64_t(blockIdx.x) * seg;
  const int64_t seg_end = (seg_begin + seg < N) ? seg_begin + seg : N;
  int user = seg_user[blockIdx.x];
  int64_t pos = seg_begin;
  Piece pc;
  while (next_piece(offsets, B, seg_end, user, pos, pc)) {
    const int64_t slot = int64_t(blockIdx.x) + pc.user;
    for (int i = threadIdx.x; i < S; i += blockDim.x) {
      float q[kMaxDh], o[kMaxDh];
      const T* qrow = Q + q_user_stride * pc.user + int64_t(i) * d + h * dh;
      for (int t = 0; t < kMaxDh; ++t) {
        q[t] = t < dh ? to_f32(qrow[t]) * scale_log2 : 0.f;
        o[t] = 0.f;
      }
      float m = -INFINITY, l = 0.f;
      (void)m; (void)l;
      for (int64_t j = pc.begin; j < pc.end; ++j) {
        const float* kr = K + j * d + h * dh;
        const float* vr = V + j * d + h * dh;
        float s = 0.f;
        for (int t = 0; t < kMaxDh; ++t)
          if (t < dh) s = fmaf(q[t], kr[t], s);
        if (SILU) {
          const float p = s / (1.f + expf(-s));
          for (int t = 0; t < kMaxDh; ++t)
            if (t < dh) o[t] = fmaf(p, vr[t], o[t]);
        } else {
          float mn = fmaxf(m, s);
          float alpha = exp2f(m - mn);  // exp2(-inf) = 0 on the first item
          float p = exp2f(s - mn);
          l = l * alpha + p;
          for (int t = 0; t < kMaxDh; ++t)
            if (t < dh) o[t] = fmaf(o[t], alpha, p * vr[t]);
          m = mn;
        }
      }
      float* dst = partials + ((slot * H + h) * S + i) * (dh + 2);
      for (int t = 0; t < kMaxDh; ++t)
        if (t < dh) dst[t] = o[t];
      dst[dh] = SILU ? 0.f : l;
      dst[dh + 1] = SILU ? 0.f : m;
    }
  }
}

// ---------------------------------------- seeds as their own key and value
// Self term (Eq. 3; the Delta term of Sec. 3.2.2): K' = Q W_k, V' = Q W_v in fp32 for the
// S shared seeds or the B*S per-user ones.  One thread per (row, column).
template <typename T>
__global__ void self_kv_kernel(const T* __restrict__ Q, const T* __restrict__ Wk, const T* __restrict__ Wv,
                               float* __restrict__ Ks, float* __restrict__ Vs, int64_t rows, int d) {
  int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= rows * d) return;
  const int64_t row = idx / d;
  const int col = int(idx - row * d);
  const T* q = Q + row * d;
  float k = 0.f, v = 0.f;
  for (int t = 0; t < d; ++t) {
    const float qv = to_f32(q[t]);
    k = fmaf(qv, to_f32(Wk[int64_t(t) * d + col]), k);
    v = fmaf(qv, to_f32(Wv[int64_t(t) * d + col]), v);
  }
  Ks[idx] = k;
  Vs[idx] = v;
}

hipError_t launch_self_kv(const vista_summarize_desc& d, const void* Q, const void* Wk, const void* Wv, float* Ks,
                          float* Vs, hipStream_t s) {
  const int64_t rows = d.q_user_stride ? int64_t(d.B) * d.S : d.S;
  const int64_t blocks = (rows * d.d + 255) / 256;
  if (d.dtype == VISTA_BF16)
    return launch(self_kv_kernel<bf16_t>, dim3(unsigned(blocks)), dim3(256), 0, s, static_cast<const bf16_t*>(Q),
                  static_cast<const bf16_t*>(Wk), static_cast<const bf16_t*>(Wv), Ks, Vs, rows, d.d);
  return launch(self_kv_kernel<float>, dim3(unsigned(blocks)), dim3(256), 0, s, static_cast<const float*>(Q),
                static_cast<const float*>(Wk), static_cast<const float*>(Wv), Ks, Vs, rows, d.d);
}

// ------------------------------------------------------- stage 1: merge
// Combines a user's partial slots in ascending segment order.
//   softmax:  m = max m_c,  l = sum l_c 2^(m_c - m),  O = sum O_c 2^(m_c - m),  out = O / l;
//             the self term is one more slot: m = own score, l = 1, O = own value;
//   SiLU form: out = (sum O_c [+ SiLU(own score) own value]) / L_b.
// grid (B, H); threads stride over (query, channel).  scale_log2 / scale as in the main kernel.
template <typename T, bool SILU>
__global__ void merge_kernel(const float* __restrict__ partials, const int64_t* __restrict__ offsets,
                             int S, int d, int H, int seg, int64_t G, T* __restrict__ out,
                             const T* __restrict__ Q, int64_t q_user_stride, const float* __restrict__ Ks,
                             const float* __restrict__ Vs, float scale_log2) {
  const int dh = d / H;
  const int b = blockIdx.x, h = blockIdx.y;
  const int64_t begin = offsets[b], end = offsets[b + 1];
  T* dst = out + int64_t(b) * S * d + h * dh;
  if (end <= begin) {
    for (int e = threadIdx.x; e < S * dh; e += blockDim.x) store_as(dst + int64_t(e / dh) * d + (e % dh), 0.f);
    return;
  }
  int64_t g0 = begin / seg, g1 = (end - 1) / seg;
  if (g0 < 0) g0 = 0;
  if (g1 > G - 1) g1 = G - 1;
  const int64_t srow0 = q_user_stride ? int64_t(b) * S : 0;     // first row of this user's K', V'
  for (int e = threadIdx.x; e < S * dh; e += blockDim.x) {
    const int i = e / dh, t = e % dh;
    float s_self = 0.f, v_self = 0.f;
    if (Ks) {
      const T* q = Q + q_user_stride * b + int64_t(i) * d + h * dh;
      const float* ks = Ks + (srow0 + i) * d + h * dh;
      for (int c = 0; c < dh; ++c) s_self = fmaf(to_f32(q[c]), ks[c], s_self);
      s_self *= scale_log2;
      v_self = Vs[(srow0 + i) * d + h * dh + t];
    }
    if (SILU) {
      float o = 0.f;
      for (int64_t g = g0; g <= g1; ++g) o += partials[(((g + b) * H + h) * S + i) * (dh + 2) + t];
      if (Ks) o = fmaf(s_self / (1.f + expf(-s_self)), v_self, o);
      store_as(dst + int64_t(i) * d + t, o / float(end - begin));
      continue;
    }
    float m = Ks ? s_self : -INFINITY;
    for (int64_t g = g0; g <= g1; ++g) {
      const float* p = partials + (((g + b) * H + h) * S + i) * (dh + 2);
      m = fmaxf(m, p[dh + 1]);
    }
    float l = 0.f, o = 0.f;
    for (int64_t g = g0; g <= g1; ++g) {
      const float* p = partials + (((g + b) * H + h) * S + i) * (dh + 2);
      float w = exp2f(p[dh + 1] - m);
      l = fmaf(p[dh], w, l);
      o = fmaf(p[t], w, o);
    }
    if (Ks) {
      const float w = exp2f(s_self - m);
      l += w;
      o = fmaf(v_self, w, o);
    }
    store_as(dst + int64_t(i) * d + t, o / l);
  }
}

// ---------------------------------------------- quasi-linear attention (plain path)
// State of one piece: Z_h = SiLU(K_h)^T V_h, [dh x dh] fp32 per (slot, head) (Sec. 3.2.2; the
// block sums of App. B).  grid (G, H), 256 threads stride over the dh*dh entries.
__global__ void qla_state_kernel(const float* __restrict__ K, const float* __restrict__ V,
                                 const int64_t* __restrict__ offsets, int B, int d, int H, int64_t N, int seg,
                                 const int* __restrict__ seg_user, float* __restrict__ partials) {
  const int dh = d / H;
  const int h = blockIdx.y;
  const int64_t seg_begin = int64_t(blockIdx.x) * seg;
  const int64_t seg_end = (seg_begin + seg < N) ? seg_begin + seg : N;
  int user = seg_user[blockIdx.x];
  int64_t pos = seg_begin;
  Piece pc;
  while (next_piece(offsets, B, seg_end, user, pos, pc)) {
    const int64_t slot = int64_t(blockIdx.x) + pc.user;
    for (int e = threadIdx.x; e < dh * dh; e += blockDim.x) {
      const int a = e / dh, c = e % dh;
      float z = 0.f;
      for (int64_t j = pc.begin; j < pc.end; ++j) {
        const float k = K[j * d + h * dh + a];
        z = fmaf(k / (1.f + expf(-k)), V[j * d + h * dh + c], z);
      }
      partials[(slot * H + h) * dh * dh + e] = z;
    }
  }
}

// out_h = SiLU(Q_h) SiLU(Z_h) with Z_h the fixed-order sum of the user's states;
// the self term adds (SiLU(q) . SiLU(k')) v'.  grid (B, H), 1024 threads, Z staged in LDS.
// DH = the head width when it is known at compile time (32: the matrix-core shapes), else 0.
template <typename T, int DH>
__global__ __launch_bounds__(1024) void qla_finish_kernel(const float* __restrict__ partials,
                                                         const int64_t* __restrict__ offsets, int S, int d, int H,
                                                         int seg, int64_t G, T* __restrict__ out,
                                                         const T* __restrict__ Q, int64_t q_user_stride,
                                                         const float* __restrict__ Ks,
                                                         const float* __restrict__ Vs, int* status) {
  constexpr int kW = DH ? DH : kMaxDh;          // register rows are sized for it
  constexpr int kRun = 256;                     // queries per pass: four threads each at 1024 threads
  constexpr int kDeep = 8;                      // record loads a thread keeps in flight
  // without a plan kernel in front (offsets checked on the host) the status word is cleared here
  if (status && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *status = VISTA_OK;
  __shared__ float z[kW * kW];
  const int dh = DH ? DH : d / H;
  const int b = blockIdx.x, h = blockIdx.y;
  const int64_t begin = offsets[b], end = offsets[b + 1];
  T* dst = out + int64_t(b) * S * d + h * dh;
  if (end <= begin) {
    for (int e = threadIdx.x; e < S * dh; e += blockDim.x) store_as(dst + int64_t(e / dh) * d + (e % dh), 0.f);
    return;
  }
  int64_t g0 = begin / seg, g1 = (end - 1) / seg;
  if (g0 < 0) g0 = 0;
  if (g1 > G - 1) g1 = G - 1;
  // Sum of the user's records in a fixed order: four groups of 256 threads take every fourth
  // record each, ascending, a thread owning four neighbouring entries with eight 16-byte loads
  // in flight (a long user is not a chain of dependent round trips); the four sub-sums are then
  // added as ((s0 + s1) + s2) + s3.  The order depends on nothing but the record count.
  const int zz = dh * dh;
  if (zz % 4 == 0 && blockDim.x == 1024) {
    const int grp = threadIdx.x >> 8, t256 = threadIdx.x & 255;
    for (int e0 = 0; e0 < zz; e0 += 1024) {
      const int e = e0 + 4 * t256;
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e < zz) {
        for (int64_t g = g0 + grp; g <= g1; g += 4 * kDeep) {
          float4 v[kDeep];
#pragma unroll
          for (int u = 0; u < kDeep; ++u)
            v[u] = g + 4 * u <= g1 ? *reinterpret_cast<const float4*>(partials + ((g + 4 * u + b) * H + h) * zz + e)
                                   : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
          for (int u = 0; u < kDeep; ++u) {
            acc.x += v[u].x;
            acc.y += v[u].y;
            acc.z += v[u].z;
            acc.w += v[u].w;
          }
        }
      }
      for (int turn = 0; turn < 4; ++turn) {
        if (grp == turn && e < zz) {
          if (turn == 0) {
            z[e] = acc.x; z[e + 1] = acc.y; z[e + 2] = acc.z; z[e + 3] = acc.w;
          } else {
            z[e] += acc.x; z[e + 1] += acc.y; z[e + 2] += acc.z; z[e + 3] += acc.w;
          }
        }
        __syncthreads();
      }
    }
  } else {
    for (int e = threadIdx.x; e < zz; e += blockDim.x) {
      float acc = 0.f;
      for (int64_t g = g0; g <= g1; ++g) acc += partials[((g + b) * H + h) * zz + e];
      z[e] = acc;
    }
    __syncthreads();
  }
  for (int e = threadIdx.x; e < zz; e += blockDim.x) {
    const float v = z[e];
    z[e] = v / (1.f + expf(-v));
  }
  __syncthreads();
  const int64_t srow0 = q_user_stride ? int64_t(b) * S : 0;
  // Queries in runs of kRun: their activated rows go to LDS (coalesced reads), then a thread
  // walks the channels of one query in a rolled loop -- a row of the state per step -- with its
  // quarter of the outputs in registers (four threads per query).
  __shared__ float qs[kRun][kW + 1];
  const int qi = threadIdx.x % kRun, quarter = threadIdx.x / kRun;
  constexpr int kQ = (kW + 3) / 4;
  const int cq = (dh + 3) / 4, c0 = quarter * cq;
  for (int i0 = 0; i0 < S; i0 += kRun) {
    __syncthreads();                     // the previous run's rows are no longer read
    // (batches of eight elements per thread: the loads of a batch are all issued before the
    // first is used, so a run costs one round trip to memory, not eight)
    for (int e0 = threadIdx.x; e0 < kRun * dh; e0 += 8 * blockDim.x) {
      float qv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = e0 + j * blockDim.x;
        const int r = e / dh, a = e % dh;
        qv[j] = (e < kRun * dh && i0 + r < S) ? to_f32(Q[q_user_stride * b + int64_t(i0 + r) * d + h * dh + a]) : 0.f;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = e0 + j * blockDim.x;
        if (e < kRun * dh) qs[e / dh][e % dh] = qv[j] / (1.f + expf(-qv[j]));
      }
    }
    __syncthreads();
    const int i = i0 + qi;
    float o[kQ];
#pragma unroll
    for (int t = 0; t < kQ; ++t) o[t] = 0.f;
    if (i < S && quarter < 4) {
      float dot = 0.f;
#pragma unroll 1
      for (int a = 0; a < dh; ++a) {
        const float pa = qs[qi][a];
#pragma unroll
        for (int t = 0; t < kQ; ++t)
          if (t < cq && c0 + t < dh) o[t] = fmaf(pa, z[a * dh + c0 + t], o[t]);
        if (Ks) {
          const float k = Ks[(srow0 + i) * d + h * dh + a];
          dot = fmaf(pa, k / (1.f + expf(-k)), dot);
        }
      }
      if (Ks) {
#pragma unroll
        for (int t = 0; t < kQ; ++t)
          if (t < cq && c0 + t < dh) o[t] = fmaf(dot, Vs[(srow0 + i) * d + h * dh + c0 + t], o[t]);
      }
    }
    // the run's outputs go back through LDS so that neighbouring lanes store neighbouring channels
    __syncthreads();
    if (i < S && quarter < 4) {
#pragma unroll
      for (int t = 0; t < kQ; ++t)
        if (t < cq && c0 + t < dh) qs[qi][c0 + t] = o[t];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < kRun * dh; e += blockDim.x) {
      const int r = e / dh, a = e % dh;
      if (i0 + r < S) store_as(dst + int64_t(i0 + r) * d + a, qs[r][a]);
    }
  }
}

// ---------------------------------------------- quasi-linear attention: gradients (App. B.1)
__device__ __forceinline__ float silu_f(float x) { return x / (1.f + expf(-x)); }
__device__ __forceinline__ float silu_prime_f(float x) {
  const float sg = 1.f / (1.f + expf(-x));
  return sg * (1.f + x * (1.f - sg));
}

// Per (user, head): the state Zs (fixed-order sum of the user's records), G = SiLU(Zs),
//   dQ = (dO G^T) * SiLU'(Q)         written to d_queries,
//   dZs = (SiLU(Q)^T dO) * SiLU'(Zs) written to dz [B][H][dh][dh] fp32 for the item pass.
// grid (B, H), 1024 threads; queries pass through LDS in runs of 64.
template <typename T>
__global__ __launch_bounds__(1024) void qla_bwd_state_kernel(const float* __restrict__ partials,
                                                            const int64_t* __restrict__ offsets, int S, int d, int H,
                                                            int seg, int64_t G, const T* __restrict__ Q,
                                                            int64_t q_user_stride, const T* __restrict__ dO,
                                                            T* __restrict__ dQ, float* __restrict__ dz, int* status) {
  // without a plan kernel in front (offsets checked on the host) the status word is cleared here
  if (status && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *status = VISTA_OK;
  __shared__ float zs[kMaxDh * kMaxDh];        // Zs, then SiLU'(Zs)
  __shared__ float gt[kMaxDh * (kMaxDh + 1)];  // G transposed: gt[c][a]
  __shared__ float qa[64][kMaxDh + 1];         // SiLU(q) of the run
  __shared__ float dy[64][kMaxDh + 1];         // dO of the run
  const int dh = d / H;
  const int b = blockIdx.x, h = blockIdx.y;
  const int64_t begin = offsets[b], end = offsets[b + 1];
  const int zz = dh * dh;
  float* dzb = dz + (int64_t(b) * H + h) * zz;
  T* dq = dQ + int64_t(b) * S * d + h * dh;
  if (end <= begin) {       // no history: the forward output is zero whatever Q is
    for (int e = threadIdx.x; e < S * dh; e += blockDim.x) store_as(dq + int64_t(e / dh) * d + (e % dh), 0.f);
    for (int e = threadIdx.x; e < zz; e += blockDim.x) dzb[e] = 0.f;
    return;
  }
  int64_t g0 = begin / seg, g1 = (end - 1) / seg;
  if (g0 < 0) g0 = 0;
  if (g1 > G - 1) g1 = G - 1;
  // The user's records, summed in the forward finishing kernel's order: four groups of 256
  // threads take every fourth record each, ascending (a thread owns four neighbouring entries,
  // eight 16-byte loads in flight), and the sub-sums are added as ((s0 + s1) + s2) + s3; then
  // SiLU'(Zs) and G^T.
  if (zz % 4 == 0 && blockDim.x == 1024) {
    const int grp = threadIdx.x >> 8, t256 = threadIdx.x & 255;
    for (int e0 = 0; e0 < zz; e0 += 1024) {
      const int e = e0 + 4 * t256;
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e < zz) {
        for (int64_t g = g0 + grp; g <= g1; g += 32) {
          float4 v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u)
            v[u] = g + 4 * u <= g1 ? *reinterpret_cast<const float4*>(partials + ((g + 4 * u + b) * H + h) * zz + e)
                                   : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            acc.x += v[u].x;
            acc.y += v[u].y;
            acc.z += v[u].z;
            acc.w += v[u].w;
          }
        }
      }
      for (int turn = 0; turn < 4; ++turn) {
        if (grp == turn && e < zz) {
          if (turn == 0) {
            zs[e] = acc.x; zs[e + 1] = acc.y; zs[e + 2] = acc.z; zs[e + 3] = acc.w;
          } else {
            zs[e] += acc.x; zs[e + 1] += acc.y; zs[e + 2] += acc.z; zs[e + 3] += acc.w;
          }
        }
        __syncthreads();
      }
    }
  } else {
    for (int e = threadIdx.x; e < zz; e += blockDim.x) {
      float acc = 0.f;
      for (int64_t g = g0; g <= g1; ++g) acc += partials[((g + b) * H + h) * zz + e];
      zs[e] = acc;
    }
    __syncthreads();
  }
  for (int e = threadIdx.x; e < zz; e += blockDim.x) {
    const float acc = zs[e];
    zs[e] = silu_prime_f(acc);
    gt[(e % dh) * (dh + 1) + e / dh] = silu_f(acc);
  }
  // this thread's entries of dG = SiLU(Q)^T dO: e = threadIdx.x + blockDim.x k
  float dg[kMaxDh * kMaxDh / 256];
#pragma unroll
  for (int k = 0; k < kMaxDh * kMaxDh / 256; ++k) dg[k] = 0.f;
  for (int i0 = 0; i0 < S; i0 += 64) {
    __syncthreads();
    for (int e = threadIdx.x; e < 64 * dh; e += blockDim.x) {
      const int r = e / dh, a = e % dh;
      const bool on = i0 + r < S;
      const float q = on ? to_f32(Q[q_user_stride * b + int64_t(i0 + r) * d + h * dh + a]) : 0.f;
      qa[r][a] = silu_f(q);
      dy[r][a] = on ? to_f32(dO[(int64_t(b) * S + i0 + r) * d + h * dh + a]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kMaxDh * kMaxDh / 256; ++k) {
      const int e = threadIdx.x + int(blockDim.x) * k;
      if (e < zz) {
        const int a = e / dh, c = e % dh;
        float acc = dg[k];
        for (int r = 0; r < 64; ++r) acc = fmaf(qa[r][a], dy[r][c], acc);
        dg[k] = acc;
      }
    }
    // dQ of the run: one (query, channel) pair per thread and step
    for (int e = threadIdx.x; e < 64 * dh; e += blockDim.x) {
      const int r = e / dh, a = e % dh;
      if (i0 + r < S) {
        float acc = 0.f;
        for (int c = 0; c < dh; ++c) acc = fmaf(dy[r][c], gt[c * (dh + 1) + a], acc);
        const float q = to_f32(Q[q_user_stride * b + int64_t(i0 + r) * d + h * dh + a]);
        store_as(dq + int64_t(i0 + r) * d + a, acc * silu_prime_f(q));
      }
    }
  }
#pragma unroll
  for (int k = 0; k < kMaxDh * kMaxDh / 256; ++k) {
    const int e = threadIdx.x + int(blockDim.x) * k;
    if (e < zz) dzb[e] = dg[k] * zs[e];
  }
}

// The same for heads of width 32 (the matrix-core shapes), with the LDS traffic cut by register
// blocking: a thread owns four neighbouring key channels, so one 16-byte and one 4-byte LDS
// read feed four multiply-adds.  1024 threads; queries pass through LDS in runs of 256 (rows
// 36 floats apart: 16-byte aligned, spread over the banks).
//   dG:  thread (quarter g, key channels 4 ab .. 4 ab + 3, value channel c) sums over the
//        run's rows 64 g .. 64 g + 63; the four quarters are added at the end as ((s0+s1)+s2)+s3;
//   dQ:  thread (row, key channels 4 ab .. 4 ab + 3), two rows per thread and run.
__device__ __forceinline__ void load4(const float* p, float v[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load4(const bf16_t* p, float v[4]) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
}
__device__ __forceinline__ void store4(float* p, const float v[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(bf16_t* p, const float v[4]) {
  uint2 t;
  t.x = uint32_t(f32_to_bf16_bits(v[0])) | (uint32_t(f32_to_bf16_bits(v[1])) << 16);
  t.y = uint32_t(f32_to_bf16_bits(v[2])) | (uint32_t(f32_to_bf16_bits(v[3])) << 16);
  *reinterpret_cast<uint2*>(p) = t;
}

template <typename T>
__global__ __launch_bounds__(1024) void qla_bwd_state32_kernel(const float* __restrict__ partials,
                                                               const int64_t* __restrict__ offsets, int S, int d, int H,
                                                               int seg, int64_t G, const T* __restrict__ Q,
                                                               int64_t q_user_stride, const T* __restrict__ dO,
                                                               T* __restrict__ dQ, float* __restrict__ dz, int* status) {
  constexpr int dh = 32, zz = dh * dh, kRun = 256, kRow = 36;
  if (status && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *status = VISTA_OK;
  __shared__ __align__(16) float zs[zz];                 // Zs, then SiLU'(Zs)
  __shared__ __align__(16) float gt[dh * kRow];          // G transposed: gt[c][a]
  __shared__ __align__(16) float qa[kRun * kRow];        // SiLU(q) of the run; at the end the partial dG of the four quarters
  __shared__ __align__(16) float dy[kRun * kRow];        // dO of the run
  const int b = blockIdx.x, h = blockIdx.y;
  const int tid = threadIdx.x;
  const int64_t begin = offsets[b], end = offsets[b + 1];
  float* dzb = dz + (int64_t(b) * H + h) * zz;
  T* dq = dQ + int64_t(b) * S * d + h * dh;
  if (end <= begin) {       // no history: the forward output is zero whatever Q is
    for (int e = tid; e < S * dh; e += 1024) store_as(dq + int64_t(e / dh) * d + (e % dh), 0.f);
    dzb[tid] = 0.f;
    return;
  }
  int64_t g0 = begin / seg, g1 = (end - 1) / seg;
  if (g0 < 0) g0 = 0;
  if (g1 > G - 1) g1 = G - 1;
  const int grp = tid >> 8, t256 = tid & 255;
  {   // the user's records in the finishing kernel's order
    const int e = 4 * t256;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t g = g0 + grp; g <= g1; g += 32) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        v[u] = g + 4 * u <= g1 ? *reinterpret_cast<const float4*>(partials + ((g + 4 * u + b) * H + h) * zz + e)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        acc.x += v[u].x;
        acc.y += v[u].y;
        acc.z += v[u].z;
        acc.w += v[u].w;
      }
    }
    for (int turn = 0; turn < 4; ++turn) {
      if (grp == turn) {
        if (turn == 0) {
          zs[e] = acc.x; zs[e + 1] = acc.y; zs[e + 2] = acc.z; zs[e + 3] = acc.w;
        } else {
          zs[e] += acc.x; zs[e + 1] += acc.y; zs[e + 2] += acc.z; zs[e + 3] += acc.w;
        }
      }
      __syncthreads();
    }
  }
  {
    const float acc = zs[tid];             // entry (a, c) = (tid / 32, tid % 32)
    zs[tid] = silu_prime_f(acc);
    gt[(tid & 31) * kRow + (tid >> 5)] = silu_f(acc);
  }
  const int ab = t256 >> 5, c = t256 & 31;          // dG: key channels 4 ab .., value channel c
  float dg[4] = {0.f, 0.f, 0.f, 0.f};
  const T* Qb = Q + q_user_stride * b + h * dh;
  const T* Db = dO + int64_t(b) * S * d + h * dh;
  for (int i0 = 0; i0 < S; i0 += kRun) {
    __syncthreads();
    // eight elements of either array per thread, all loads issued before the first is used
    {
      float qv[8], yv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = tid + 1024 * j, r = e >> 5, a = e & 31;
        const bool on = i0 + r < S;
        qv[j] = on ? to_f32(Qb[int64_t(i0 + r) * d + a]) : 0.f;
        yv[j] = on ? to_f32(Db[int64_t(i0 + r) * d + a]) : 0.f;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = tid + 1024 * j, r = e >> 5, a = e & 31;
        qa[r * kRow + a] = silu_f(qv[j]);
        dy[r * kRow + a] = yv[j];
      }
    }
    __syncthreads();
    // dG += SiLU(Q)^T dO over this quarter's 64 rows
#pragma unroll 4
    for (int r = 64 * grp; r < 64 * grp + 64; ++r) {
      const float4 q4 = *reinterpret_cast<const float4*>(&qa[r * kRow + 4 * ab]);
      const float y = dy[r * kRow + c];
      dg[0] = fmaf(q4.x, y, dg[0]);
      dg[1] = fmaf(q4.y, y, dg[1]);
      dg[2] = fmaf(q4.z, y, dg[2]);
      dg[3] = fmaf(q4.w, y, dg[3]);
    }
    // dQ = (dO G^T) * SiLU'(Q): rows tid / 8 and tid / 8 + 128, key channels 4 (tid % 8) ..
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int r = (tid >> 3) + 128 * j, a4 = 4 * (tid & 7);
      if (i0 + r < S) {
        float o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int cc = 0; cc < dh; ++cc) {
          const float y = dy[r * kRow + cc];
          const float4 g4 = *reinterpret_cast<const float4*>(&gt[cc * kRow + a4]);
          o[0] = fmaf(y, g4.x, o[0]);
          o[1] = fmaf(y, g4.y, o[1]);
          o[2] = fmaf(y, g4.z, o[2]);
          o[3] = fmaf(y, g4.w, o[3]);
        }
        float q[4];
        load4(Qb + int64_t(i0 + r) * d + a4, q);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] *= silu_prime_f(q[k]);
        store4(dq + int64_t(i0 + r) * d + a4, o);
      }
    }
  }
  // the four quarters' partial dG, added in a fixed order, times SiLU'(Zs)
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) qa[grp * zz + (4 * ab + k) * dh + c] = dg[k];
  __syncthreads();
  dzb[tid] = (((qa[tid] + qa[zz + tid]) + qa[2 * zz + tid]) + qa[3 * zz + tid]) * zs[tid];
}

// Gradients of the target-side diagonal term (phi(q_i) . phi(k'_i)) v'_i (App. B.1: second term of
// Eq. 8, Eqs. 10 and 12, with phi = SiLU in place), one wave-sized group of dh threads per
// (user, query, head):
//   U = phi(q) . phi(k'),  X = dO . v',
//   dV' = U dO,   dK' = X phi(q) * phi'(k'),   dQ += X phi(k') * phi'(q)   (added to what the
//   state-gradient kernel has written).  Users without history get zeros (their output is zero).
template <typename T>
__global__ void qla_bwd_self_kernel(const T* __restrict__ Q, int64_t q_user_stride, const float* __restrict__ Ks,
                                    const float* __restrict__ Vs, const T* __restrict__ dO,
                                    const int64_t* __restrict__ offsets, int B, int S, int d, int H,
                                    T* __restrict__ dQ, T* __restrict__ dKs, T* __restrict__ dVs) {
  const int dh = d / H;
  const int64_t unit = int64_t(blockIdx.x) * blockDim.y + threadIdx.y;      // (user, query, head)
  if (unit >= int64_t(B) * S * H) return;
  const int h = int(unit % H);
  const int64_t bi = unit / H;                                            // user * S + query
  const int b = int(bi / S), i = int(bi % S);
  const int t = threadIdx.x;                                              // channel of the head (blockDim.x = 64)
  const int64_t at = bi * d + h * dh + t;
  const bool on = t < dh;
  if (offsets[b + 1] <= offsets[b]) {
    if (on) {
      store_as(dKs + at, 0.f);
      store_as(dVs + at, 0.f);
    }
    return;
  }
  const int64_t srow = (q_user_stride ? int64_t(b) * S : 0) + i;
  const float q = on ? to_f32(Q[q_user_stride * b + int64_t(i) * d + h * dh + t]) : 0.f;
  const float k = on ? Ks[srow * d + h * dh + t] : 0.f;
  const float v = on ? Vs[srow * d + h * dh + t] : 0.f;
  const float g = on ? to_f32(dO[at]) : 0.f;
  const float a = silu_f(q), pk = silu_f(k);
  float u = a * pk, x = g * v;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    u += __shfl_xor(u, off, 64);
    x += __shfl_xor(x, off, 64);
  }
  if (on) {
    store_as(dVs + at, u * g);
    store_as(dKs + at, x * a * silu_prime_f(k));
    store_as(dQ + at, to_f32(dQ[at]) + x * pk * silu_prime_f(q));
  }
}

// Per item and head (plain path): dV = SiLU(k) dZs, dK = (v dZs^T) * SiLU'(k), from fp32 K, V.
// One thread per (item, head).
template <typename T>
__global__ void qla_bwd_items_kernel(const float* __restrict__ K, const float* __restrict__ V,
                                     const int64_t* __restrict__ offsets, int B, int d, int H, int64_t N,
                                     const float* __restrict__ dz, T* __restrict__ dK, T* __restrict__ dV) {
  const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= N * H) return;
  const int64_t j = idx / H;
  const int h = int(idx - j * H);
  const int dh = d / H;
  int b = 0;                 // the last user starting at or before row j (empty users own no rows);
  {                          // searched per thread: rows of one wave belong to different users
    int hi = B;
    while (hi - b > 1) {
      const int mid = (b + hi) >> 1;
      if (offsets[mid] <= j) b = mid; else hi = mid;
    }
  }
  const float* z = dz + (int64_t(b) * H + h) * dh * dh;
  const float* k = K + j * d + h * dh;
  const float* v = V + j * d + h * dh;
  float p[kMaxDh], vv[kMaxDh];
  for (int a = 0; a < kMaxDh; ++a) {
    p[a] = a < dh ? silu_f(k[a]) : 0.f;
    vv[a] = a < dh ? v[a] : 0.f;
  }
  for (int c = 0; c < dh; ++c) {
    float acc = 0.f;
    for (int a = 0; a < kMaxDh; ++a)
      if (a < dh) acc = fmaf(p[a], z[a * dh + c], acc);
    store_as(dV + j * d + h * dh + c, acc);
  }
  for (int a = 0; a < dh; ++a) {
    float acc = 0.f;
    for (int c = 0; c < kMaxDh; ++c)
      if (c < dh) acc = fmaf(vv[c], z[a * dh + c], acc);
    store_as(dK + j * d + h * dh + a, acc * silu_prime_f(k[a]));
  }
}

static size_t generic_partials_bytes(const vista_summarize_desc& d, int seg) {
  int64_t G = (d.total_items + seg - 1) / seg;
  int dh = d.d / d.H;
  if (d.attn == VISTA_ATTN_QLA) return size_t(G + d.B) * d.H * dh * dh * sizeof(float);
  return size_t(G + d.B) * d.H * d.S * (dh + 2) * sizeof(float);
}

// fp32 K' and V' of the seeds (self term), each [S or B*S, d]; 0 without the flag
size_t self_kv_bytes(const vista_summarize_desc& d) {
  if (!(d.flags & VISTA_FLAG_SELF_TERM)) return 0;
  const size_t rows = d.q_user_stride ? size_t(d.B) * d.S : size_t(d.S);
  return (rows * d.d * sizeof(float) + 255) & ~size_t(255);
}

static size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

size_t generic_summarize_workspace(const vista_summarize_desc& d, int seg) {
  const int64_t G = (d.total_items + seg - 1) / seg;
  const size_t kv = mfma_qla_supported(d) ? 0 : 2 * align256(size_t(d.total_items) * d.d * sizeof(float));
  return kHeaderBytes + plan_bytes(G) + align256(generic_partials_bytes(d, seg)) + kv + 2 * self_kv_bytes(d);
}

template <typename T>
static vista_status generic_summarize_t(const SummarizeArgs& a) {
  const vista_summarize_desc& d = a.desc;
  const int64_t N = d.total_items;
  char* base = a.workspace + kHeaderBytes + plan_bytes(a.G);
  float* partials = reinterpret_cast<float*>(base);
  const size_t kv_each = mfma_qla_supported(d) ? 0 : align256(size_t(N) * d.d * sizeof(float));
  float* K = reinterpret_cast<float*>(base + align256(generic_partials_bytes(d, a.seg)));
  float* V = K + kv_each / sizeof(float);
  float* Ks = nullptr;
  float* Vs = nullptr;
  if (d.flags & VISTA_FLAG_SELF_TERM) {
    Ks = V + kv_each / sizeof(float);
    Vs = Ks + self_kv_bytes(d) / sizeof(float);
    if (launch_self_kv(d, a.Q, a.Wk, a.Wv, Ks, Vs, a.stream) != hipSuccess) return VISTA_ERR_HIP;
  }
  const T* Q = static_cast<const T*>(a.Q);
  const bool silu = d.attn == VISTA_ATTN_SILU, qla = d.attn == VISTA_ATTN_QLA;
  // the softmax form works in base-2 units; the pointwise forms take the score as it is
  const float score_scale = silu ? a.scale_plain : a.scale_log2;
  if (N > 0 && mfma_qla_supported(d)) {
    // bf16, head width 32: the state records come from the matrix-core kernel (same layout)
    const vista_status st = mfma_qla_state(a, partials);
    if (st != VISTA_OK) return st;
  } else if (N > 0) {
    int64_t total = N * d.d;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
    VISTA_LAUNCH(project_kernel<T>, dim3(unsigned(blocks)), dim3(256), 0, a.stream,
                       static_cast<const T*>(a.X), static_cast<const T*>(a.Wk), static_cast<const T*>(a.Wv),
                       K, V, N, d.d);
    if (qla)
      VISTA_LAUNCH(qla_state_kernel, dim3(unsigned(a.G), d.H), dim3(256), 0, a.stream, K, V, a.offsets, d.B, d.d,
                   d.H, N, a.seg, a.seg_user, partials);
    else if (silu)
      VISTA_LAUNCH((attend_history_kernel<T, true>), dim3(unsigned(a.G), d.H), dim3(64), 0, a.stream, K, V, Q,
                   d.q_user_stride, a.offsets, d.B, d.S, d.d, d.H, score_scale, N, a.seg, a.seg_user, partials);
    else
      VISTA_LAUNCH((attend_history_kernel<T, false>), dim3(unsigned(a.G), d.H), dim3(64), 0, a.stream, K, V, Q,
                   d.q_user_stride, a.offsets, d.B, d.S, d.d, d.H, score_scale, N, a.seg, a.seg_user, partials);
  }
  T* out = static_cast<T*>(a.out);
  if (qla && d.d / d.H == 32)
    VISTA_LAUNCH((qla_finish_kernel<T, 32>), dim3(d.B, d.H), dim3(1024), 0, a.stream, partials, a.offsets, d.S, d.d,
                 d.H, a.seg, a.G, out, Q, d.q_user_stride, Ks, Vs,
                 a.seg_user ? nullptr : reinterpret_cast<int*>(a.workspace));
  else if (qla)
    VISTA_LAUNCH((qla_finish_kernel<T, 0>), dim3(d.B, d.H), dim3(1024), 0, a.stream, partials, a.offsets, d.S, d.d,
                 d.H, a.seg, a.G, out, Q, d.q_user_stride, Ks, Vs,
                 a.seg_user ? nullptr : reinterpret_cast<int*>(a.workspace));
  else if (silu)
    VISTA_LAUNCH((merge_kernel<T, true>), dim3(d.B, d.H), dim3(256), 0, a.stream, partials, a.offsets, d.S, d.d,
                 d.H, a.seg, a.G, out, Q, d.q_user_stride, Ks, Vs, score_scale);
  else
    VISTA_LAUNCH((merge_kernel<T, false>), dim3(d.B, d.H), dim3(256), 0, a.stream, partials, a.offsets, d.S, d.d,
                 d.H, a.seg, a.G, out, Q, d.q_user_stride, Ks, Vs, score_scale);
  return VISTA_OK;
}

vista_status generic_summarize(const SummarizeArgs& a) {
  if (a.desc.d / a.desc.H > kMaxDh) return VISTA_ERR_UNSUPPORTED;
  return a.desc.dtype == VISTA_BF16 ? generic_summarize_t<bf16_t>(a) : generic_summarize_t<float>(a);
}

// Workspace of the backward call: the forward layout (header, plan, state records, fp32 K and V
// on the plain path) followed by dZs [B][H][dh][dh] fp32.
size_t qla_backward_workspace(const vista_summarize_desc& d, int seg) {
  const int dh = d.d / d.H;
  return generic_summarize_workspace(d, seg) + align256(size_t(d.B) * d.H * dh * dh * sizeof(float));
}

template <typename T>
static vista_status qla_backward_t(const SummarizeArgs& a, const void* d_out, void* d_queries, void* d_keys,
                                   void* d_values, void* d_self_keys, void* d_self_values) {
  const vista_summarize_desc& d = a.desc;
  const int64_t N = d.total_items;
  const int dh = d.d / d.H;
  char* base = a.workspace + kHeaderBytes + plan_bytes(a.G);
  float* partials = reinterpret_cast<float*>(base);
  const size_t kv_each = mfma_qla_supported(d) ? 0 : align256(size_t(N) * d.d * sizeof(float));
  float* K = reinterpret_cast<float*>(base + align256(generic_partials_bytes(d, a.seg)));
  float* V = K + kv_each / sizeof(float);
  float* dz = reinterpret_cast<float*>(a.workspace + generic_summarize_workspace(d, a.seg));
  const bool mfma = mfma_qla_supported(d);
  if (N > 0) {
    if (mfma) {
      const vista_status st = mfma_qla_state(a, partials);
      if (st != VISTA_OK) return st;
    } else {
      const int64_t blocks = (N * d.d + 255) / 256;
      if (blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
      VISTA_LAUNCH(project_kernel<T>, dim3(unsigned(blocks)), dim3(256), 0, a.stream, static_cast<const T*>(a.X),
                   static_cast<const T*>(a.Wk), static_cast<const T*>(a.Wv), K, V, N, d.d);
      VISTA_LAUNCH(qla_state_kernel, dim3(unsigned(a.G), d.H), dim3(256), 0, a.stream, K, V, a.offsets, d.B, d.d, d.H,
                   N, a.seg, a.seg_user, partials);
    }
  }
  int* status = a.seg_user ? nullptr : reinterpret_cast<int*>(a.workspace);
  if (dh == 32)
    VISTA_LAUNCH(qla_bwd_state32_kernel<T>, dim3(d.B, d.H), dim3(1024), 0, a.stream, partials, a.offsets, d.S, d.d, d.H,
                 a.seg, a.G, static_cast<const T*>(a.Q), d.q_user_stride, static_cast<const T*>(d_out),
                 static_cast<T*>(d_queries), dz, status);
  else
    VISTA_LAUNCH(qla_bwd_state_kernel<T>, dim3(d.B, d.H), dim3(1024), 0, a.stream, partials, a.offsets, d.S, d.d, d.H,
                 a.seg, a.G, static_cast<const T*>(a.Q), d.q_user_stride, static_cast<const T*>(d_out),
                 static_cast<T*>(d_queries), dz, status);
  if (d.flags & VISTA_FLAG_SELF_TERM) {
    // the seeds' own keys and values, then the diagonal term's gradients (dQ is added to)
    float* Ks = V + kv_each / sizeof(float);
    float* Vs = Ks + self_kv_bytes(d) / sizeof(float);
    if (launch_self_kv(d, a.Q, a.Wk, a.Wv, Ks, Vs, a.stream) != hipSuccess) return VISTA_ERR_HIP;
    const int64_t units = int64_t(d.B) * d.S * d.H;
    const int64_t blocks = (units + 3) / 4;
    if (blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
    VISTA_LAUNCH(qla_bwd_self_kernel<T>, dim3(unsigned(blocks)), dim3(64, 4), 0, a.stream, static_cast<const T*>(a.Q),
                 d.q_user_stride, Ks, Vs, static_cast<const T*>(d_out), a.offsets, d.B, d.S, d.d, d.H,
                 static_cast<T*>(d_queries), static_cast<T*>(d_self_keys), static_cast<T*>(d_self_values));
  }
  if (N > 0) {
    if (mfma) return mfma_qla_backward_items(a, dz, d_keys, d_values);
    const int64_t blocks = (N * d.H + 127) / 128;
    if (blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
    VISTA_LAUNCH(qla_bwd_items_kernel<T>, dim3(unsigned(blocks)), dim3(128), 0, a.stream, K, V, a.offsets, d.B, d.d,
                 d.H, N, dz, static_cast<T*>(d_keys), static_cast<T*>(d_values));
  }
  return VISTA_OK;
}

vista_status qla_backward(const SummarizeArgs& a, const void* d_out, void* d_queries, void* d_keys, void* d_values,
                          void* d_self_keys, void* d_self_values) {
  return a.desc.dtype == VISTA_BF16
             ? qla_backward_t<bf16_t>(a, d_out, d_queries, d_keys, d_values, d_self_keys, d_self_values)
             : qla_backward_t<float>(a, d_out, d_queries, d_keys, d_values, d_self_keys, d_self_values);
}

// ------------------------------------------------------------------ stage 2
// One thread per (user, candidate, head); keys = values = the user's summaries.
// Summaries come as `summ` or, when codes != null, as int8 codes times the scale of their (token, head).
template <typename T>
__global__ void target_attend_kernel(const T* __restrict__ cand, const T* __restrict__ summ,
                                     const int8_t* __restrict__ codes, const float* __restrict__ scales,
                                     T* __restrict__ out, int64_t total, int C, int S, int d, int H,
                                     float scale_log2, int self_term) {
  const int dh = d / H;
  int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int h = int(idx % H);
  const int64_t bc = idx / H;     // flat (user, candidate)
  const int64_t b = bc / C;
  const T* qrow = cand + bc * d + h * dh;
  const T* Y = codes ? nullptr : summ + b * S * d + h * dh;
  const int8_t* Yq = codes ? codes + b * S * d + h * dh : nullptr;
  float q[kMaxDh], o[kMaxDh];
  for (int t = 0; t < kMaxDh; ++t) {
    q[t] = t < dh ? to_f32(qrow[t]) * scale_log2 : 0.f;
    o[t] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  // with the self term the candidate's own embedding is one more key and value (Eq. 3)
  for (int j = 0; j < S + (self_term ? 1 : 0); ++j) {
    float y[kMaxDh];
    if (j < S && codes) {
      const float sc = scales[(b * S + j) * H + h];
      for (int t = 0; t < kMaxDh; ++t)
        if (t < dh) y[t] = float(Yq[int64_t(j) * d + t]) * sc;
    } else {
      const T* src = j < S ? Y + int64_t(j) * d : qrow;
      for (int t = 0; t < kMaxDh; ++t)
        if (t < dh) y[t] = to_f32(src[t]);
    }
    float s = 0.f;
    for (int t = 0; t < kMaxDh; ++t)
      if (t < dh) s = fmaf(q[t], y[t], s);
    float mn = fmaxf(m, s);
    float alpha = exp2f(m - mn);
    float p = exp2f(s - mn);
    l = l * alpha + p;
    for (int t = 0; t < kMaxDh; ++t)
      if (t < dh) o[t] = fmaf(o[t], alpha, p * y[t]);
    m = mn;
  }
  T* dst = out + bc * d + h * dh;
  const float inv = 1.f / l;
  for (int t = 0; t < kMaxDh; ++t)
    if (t < dh) store_as(dst + t, o[t] * inv);
}

vista_status generic_target_attend(const vista_attend_desc& d, float scale_log2, const void* cand,
                                   const void* summ, const int8_t* codes, const float* scales, void* out,
                                   hipStream_t s) {
  if (d.d / d.H > kMaxDh) return VISTA_ERR_UNSUPPORTED;
  int64_t total = int64_t(d.B) * d.C * d.H;
  int64_t blocks = (total + 127) / 128;
  if (blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  if (d.dtype == VISTA_BF16)
    VISTA_LAUNCH(target_attend_kernel<bf16_t>, dim3(unsigned(blocks)), dim3(128), 0, s,
                       static_cast<const bf16_t*>(cand), static_cast<const bf16_t*>(summ), codes, scales,
                       static_cast<bf16_t*>(out), total, d.C, d.S, d.d, d.H, scale_log2,
                       int(d.flags & VISTA_FLAG_SELF_TERM));
  else
    VISTA_LAUNCH(target_attend_kernel<float>, dim3(unsigned(blocks)), dim3(128), 0, s,
                       static_cast<const float*>(cand), static_cast<const float*>(summ), codes, scales,
                       static_cast<float*>(out), total, d.C, d.S, d.d, d.H, scale_log2,
                       int(d.flags & VISTA_FLAG_SELF_TERM));
  return VISTA_OK;
}

// ------------------------------------------------------- cache codec
// One thread per (token, head): amax over the head's channels, scale = amax / 127,
// code = round-half-even(y * (127 / amax)); every step in fp32 (Sec. 3.1 names the step,
// the scheme is this library's).
template <typename T>
__global__ void quantize_kernel(const T* __restrict__ y, int8_t* __restrict__ codes, float* __restrict__ scales,
                                int64_t groups, int d, int H) {
  const int64_t gidx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (gidx >= groups) return;
  const int dh = d / H;
  const int64_t row = gidx / H;
  const int h = int(gidx - row * H);
  const T* src = y + row * d + h * dh;
  float v[kMaxDh];
  float amax = 0.f;
  for (int t = 0; t < kMaxDh; ++t) {
    v[t] = t < dh ? to_f32(src[t]) : 0.f;
    amax = fmaxf(amax, fabsf(v[t]));
  }
  const float inv = amax > 0.f ? 127.f / amax : 0.f;
  scales[gidx] = amax > 0.f ? amax / 127.f : 0.f;
  int8_t* dst = codes + row * d + h * dh;
  for (int t = 0; t < kMaxDh; ++t)
    if (t < dh) dst[t] = int8_t(fminf(fmaxf(rintf(v[t] * inv), -127.f), 127.f));
}

vista_status generic_quantize(const vista_codec_desc& d, const void* y, int8_t* codes, float* scales, hipStream_t s) {
  const int64_t groups = d.rows * d.H;
  const int64_t blocks = (groups + 127) / 128;
  if (blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  if (d.dtype == VISTA_BF16)
    VISTA_LAUNCH(quantize_kernel<bf16_t>, dim3(unsigned(blocks)), dim3(128), 0, s, static_cast<const bf16_t*>(y), codes,
                 scales, groups, d.d, d.H);
  else
    VISTA_LAUNCH(quantize_kernel<float>, dim3(unsigned(blocks)), dim3(128), 0, s, static_cast<const float*>(y), codes,
                 scales, groups, d.d, d.H);
  return VISTA_OK;
}

// ------------------------------------------------------- gated block
// One workgroup per R rows: yhat and the gated hidden row live in LDS.
constexpr int kFfnRows = 4;

template <typename T>
__global__ void sglu_ffn_kernel(const T* __restrict__ y, const T* __restrict__ Wg, const T* __restrict__ Wu,
                                const T* __restrict__ Wo, T* __restrict__ out, int64_t rows, int d, int dff,
                                float eps) {
  extern __shared__ float lds[];
  float* yh = lds;                    // [R][d]
  float* hid = lds + kFfnRows * d;    // [R][dff]
  __shared__ float inv_rms[kFfnRows];
  const int64_t row0 = int64_t(blockIdx.x) * kFfnRows;
  const int nrow = int(rows - row0 < kFfnRows ? rows - row0 : kFfnRows);
  for (int e = threadIdx.x; e < kFfnRows * d; e += blockDim.x) {
    int r = e / d, t = e % d;
    yh[e] = r < nrow ? to_f32(y[(row0 + r) * d + t]) : 0.f;
  }
  __syncthreads();
  if (threadIdx.x < kFfnRows) {
    float ss = 0.f;
    for (int t = 0; t < d; ++t) ss = fmaf(yh[threadIdx.x * d + t], yh[threadIdx.x * d + t], ss);
    inv_rms[threadIdx.x] = 1.f / sqrtf(ss / d + eps);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < kFfnRows * d; e += blockDim.x) yh[e] *= inv_rms[e / d];
  __syncthreads();
  for (int f = threadIdx.x; f < dff; f += blockDim.x) {
    float g[kFfnRows], u[kFfnRows];
    for (int r = 0; r < kFfnRows; ++r) g[r] = u[r] = 0.f;
    for (int t = 0; t < d; ++t) {
      float wg = to_f32(Wg[int64_t(t) * dff + f]), wu = to_f32(Wu[int64_t(t) * dff + f]);
      for (int r = 0; r < kFfnRows; ++r) {
        g[r] = fmaf(yh[r * d + t], wg, g[r]);
        u[r] = fmaf(yh[r * d + t], wu, u[r]);
      }
    }
    for (int r = 0; r < kFfnRows; ++r) hid[r * dff + f] = g[r] / (1.f + expf(-g[r])) * u[r];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    float acc[kFfnRows];
    for (int r = 0; r < kFfnRows; ++r) acc[r] = 0.f;
    for (int f = 0; f < dff; ++f) {
      float w = to_f32(Wo[int64_t(f) * d + c]);
      for (int r = 0; r < kFfnRows; ++r) acc[r] = fmaf(hid[r * dff + f], w, acc[r]);
    }
    for (int r = 0; r < nrow; ++r) store_as(out + (row0 + r) * d + c, acc[r]);
  }
}

vista_status generic_sglu_ffn(const vista_ffn_desc& d, float eps, const void* y, const void* Wg,
                              const void* Wu, const void* Wo, void* out, hipStream_t s) {
  int64_t blocks = (d.rows + kFfnRows - 1) / kFfnRows;
  if (blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  size_t lds = size_t(kFfnRows) * (d.d + d.d_ff) * sizeof(float);
  if (d.dtype == VISTA_BF16)
    VISTA_LAUNCH(sglu_ffn_kernel<bf16_t>, dim3(unsigned(blocks)), dim3(256), lds, s,
                       static_cast<const bf16_t*>(y), static_cast<const bf16_t*>(Wg),
                       static_cast<const bf16_t*>(Wu), static_cast<const bf16_t*>(Wo),
                       static_cast<bf16_t*>(out), d.rows, d.d, d.d_ff, eps);
  else
    VISTA_LAUNCH(sglu_ffn_kernel<float>, dim3(unsigned(blocks)), dim3(256), lds, s,
                       static_cast<const float*>(y), static_cast<const float*>(Wg),
                       static_cast<const float*>(Wu), static_cast<const float*>(Wo),
                       static_cast<float*>(out), d.rows, d.d, d.d_ff, eps);
  return VISTA_OK;
}

}  // namespace vista
