// Stage 2 on the matrix cores (bf16 MFMA, fp32 accumulate), gfx950.
//
// One wave serves one (user, head): the user's S summary tokens of that head
// stay resident in registers twice -- as the K operand of S^T = K Q^T (keys x
// candidates) and, transposed, as the V operand of O^T = V^T P^T.  The
// transposed copy is made by the matrix core itself (K block times a 0/1
// selector matrix lands in the accumulator layout, which is the A-operand
// layout of the second product), so no LDS is used at all.  Candidates stream
// through in blocks of 32: two 16-byte loads per lane bring Q, the key blocks
// stream past it (scores -> 2^s -> P V accumulate, per-lane statistics because
// a lane owns one candidate column), and the normalised output is stored as
// four 8-byte pieces.
//
// Softmax reference: as in stage 1, when |q| |k| <= 60 (base-2 units) for the
// whole block the reference maximum is the constant 0; otherwise a running
// maximum with rescaling is kept across the key blocks.
#include "common.hpp"

namespace vista {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

namespace {

constexpr float kSafeBound2 = 3600.f;

struct AttendParams {
  const uint16_t* cand;
  const uint16_t* summ;
  uint16_t* out;
  int B, C, S, d, H;
  int chunk_blocks;   // candidate blocks (of 32) per workgroup
  int chunks;         // workgroups per (user, head group)
  float c;            // scale * log2(e)
};

union Pack8 {
  bf16x8 v;
  uint4 u;
  uint16_t h[8];
  uint32_t w[4];
};

__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 r = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float dot2_ones(uint32_t pk, float acc) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, acc, false);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// NKB = S / 32 key blocks; 4 waves = 4 heads per workgroup.
template <int NKB>
__global__ __launch_bounds__(256) void attend_mfma_kernel(AttendParams p) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int hf = lane >> 5, l32 = lane & 31;
  const int hgroups = p.H / 4;
  int id = blockIdx.x;
  const int chunk = id % p.chunks;
  id /= p.chunks;
  const int hg = id % hgroups;
  const int b = id / hgroups;
  const int h = hg * 4 + wave;
  const int64_t col = 32 * h + 8 * hf;          // first channel of this lane's 8-wide operand slice

  // ---- resident operands of this (user, head)
  bf16x8 kop[NKB][2], vop[NKB][2];
  float kmax2 = 0.f;
  {
    const uint16_t* Y = p.summ + int64_t(b) * p.S * p.d;
    Pack8 sel[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < 8; ++j) sel[ks].h[j] = (l32 == 16 * ks + 8 * hf + j) ? 0x3F80 : 0;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      Pack8 k[2];
      float n2 = 0.f;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        k[ks].u = *reinterpret_cast<const uint4*>(Y + int64_t(kb * 32 + l32) * p.d + col + 16 * ks);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float a = bf16_lo(k[ks].w[w]), c2 = bf16_hi(k[ks].w[w]);
          n2 = fmaf(a, a, fmaf(c2, c2, n2));
        }
      }
      n2 += __shfl_xor(n2, 32, 64);
      kmax2 = fmaxf(kmax2, n2);
      // V operand: (K block) x (selector) reproduces the block in accumulator layout
      f32x16 t = {0};
      t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k[0].v, sel[0].v, t, 0, 0, 0);
      t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k[1].v, sel[1].v, t, 0, 0, 0);
      Pack8 v0, v1;
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        v0.w[i / 2] = cvt_pk_bf16(t[i], t[i + 1]);
        v1.w[i / 2] = cvt_pk_bf16(t[8 + i], t[8 + i + 1]);
      }
      vop[kb][0] = v0.v;
      vop[kb][1] = v1.v;
      // K operand carries the score scale (one extra bf16 rounding of scale*log2e*k)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        Pack8 s;
#pragma unroll
        for (int w = 0; w < 4; ++w)
          s.w[w] = cvt_pk_bf16(bf16_lo(k[ks].w[w]) * p.c, bf16_hi(k[ks].w[w]) * p.c);
        kop[kb][ks] = s.v;
      }
    }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) kmax2 = fmaxf(kmax2, __shfl_xor(kmax2, off, 64));
    kmax2 *= p.c * p.c;
  }

  const int cb0 = chunk * p.chunk_blocks;
  const int nblocks_total = (p.C + 31) / 32;
  int cb1 = cb0 + p.chunk_blocks;
  if (cb1 > nblocks_total) cb1 = nblocks_total;
  const uint16_t* Tb = p.cand + int64_t(b) * p.C * p.d;
  uint16_t* Ob = p.out + int64_t(b) * p.C * p.d;

  auto load_q = [&](int cb, Pack8& q0, Pack8& q1) {
    int row = cb * 32 + l32;
    if (row > p.C - 1) row = p.C - 1;
    const uint16_t* src = Tb + int64_t(row) * p.d + col;
    q0.u = *reinterpret_cast<const uint4*>(src);
    q1.u = *reinterpret_cast<const uint4*>(src + 16);
  };

  // Candidate blocks are fetched kPrefetch blocks ahead: with one wave per SIMD
  // nothing else hides the HBM latency of the two 16-byte loads per lane.
  constexpr int kPrefetch = 4;
  Pack8 qr[kPrefetch][2];
#pragma unroll
  for (int u = 0; u < kPrefetch; ++u)
    if (cb0 + u < cb1) load_q(cb0 + u, qr[u][0], qr[u][1]);
  for (int cbb = cb0; cbb < cb1; cbb += kPrefetch) {
#pragma unroll
   for (int u = 0; u < kPrefetch; ++u) {
    const int cb = cbb + u;
    if (cb >= cb1) break;
    Pack8 c0 = qr[u][0], c1 = qr[u][1];
    if (cb + kPrefetch < cb1) load_q(cb + kPrefetch, qr[u][0], qr[u][1]);

    float qn2 = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float a0 = bf16_lo(c0.w[w]), a1 = bf16_hi(c0.w[w]), b0 = bf16_lo(c1.w[w]), b1 = bf16_hi(c1.w[w]);
      qn2 = fmaf(a0, a0, fmaf(a1, a1, fmaf(b0, b0, fmaf(b1, b1, qn2))));
    }
    qn2 += __shfl_xor(qn2, 32, 64);
    const bool general = __builtin_amdgcn_ballot_w64(qn2 * kmax2 > kSafeBound2) != 0;

    // Key blocks stream through: 32 keys x 32 candidates of scores at a time.
    f32x16 o = {0};
    float l[4] = {0.f, 0.f, 0.f, 0.f};
    float m = general ? -INFINITY : 0.f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      f32x16 sc = {0};
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kb][0], c0.v, sc, 0, 0, 0);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kb][1], c1.v, sc, 0, 0, 0);
      if (general) {
        float tmax = sc[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sc[i]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float mnew = fmaxf(m, tmax);
        const float alpha = __builtin_amdgcn_exp2f(m - mnew);
        m = mnew;
#pragma unroll
        for (int i = 0; i < 4; ++i) l[i] *= alpha;
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i] *= alpha;
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[i] -= mnew;
      }
      Pack8 p0, p1;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const uint32_t pk = cvt_pk_bf16(__builtin_amdgcn_exp2f(sc[i]), __builtin_amdgcn_exp2f(sc[i + 1]));
        l[(i / 2) & 3] = dot2_ones(pk, l[(i / 2) & 3]);
        if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
      }
      o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[kb][0], p0.v, o, 0, 0, 0);
      o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[kb][1], p1.v, o, 0, 0, 0);
    }
    float lsum = (l[0] + l[1]) + (l[2] + l[3]);
    lsum += __shfl_xor(lsum, 32, 64);
    const float inv = __builtin_amdgcn_rcpf(lsum);
    const int row = cb * 32 + l32;
    if (row < p.C) {
      uint16_t* dst = Ob + int64_t(row) * p.d + 32 * h + 4 * hf;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 pk;
        pk.x = cvt_pk_bf16(o[4 * g] * inv, o[4 * g + 1] * inv);
        pk.y = cvt_pk_bf16(o[4 * g + 2] * inv, o[4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(dst + 8 * g) = pk;
      }
    }
   }
  }
}

template <int NKB>
void launch(const AttendParams& p, hipStream_t s) {
  const unsigned blocks = unsigned(p.B) * unsigned(p.H / 4) * unsigned(p.chunks);
  hipLaunchKernelGGL(attend_mfma_kernel<NKB>, dim3(blocks), dim3(256), 0, s, p);
}

}  // namespace

bool mfma_target_attend_supported(const vista_attend_desc& d) {
  return d.dtype == VISTA_BF16 && d.d == 32 * d.H && d.H % 4 == 0 && d.S % 32 == 0 && d.S <= 256;
}

vista_status mfma_target_attend(const vista_attend_desc& d, float scale_log2, const void* cand,
                                const void* summ, void* out, hipStream_t s) {
  AttendParams p;
  p.cand = static_cast<const uint16_t*>(cand);
  p.summ = static_cast<const uint16_t*>(summ);
  p.out = static_cast<uint16_t*>(out);
  p.B = d.B; p.C = d.C; p.S = d.S; p.d = d.d; p.H = d.H;
  p.c = scale_log2;
  // Candidate blocks per workgroup: long enough to amortise the operand set-up
  // (about one block's worth of work), short enough to give the chip >= 1024 workgroups.
  const int nblocks = (d.C + 31) / 32;
  const int64_t groups = int64_t(d.B) * (d.H / 4);
  int chunk = 16;
  while (chunk > 2 && groups * ((nblocks + chunk - 1) / chunk) < 1024) chunk >>= 1;
  p.chunk_blocks = chunk;
  p.chunks = (nblocks + chunk - 1) / chunk;
  if (groups * p.chunks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  switch (d.S / 32) {
    case 1: launch<1>(p, s); break;
    case 2: launch<2>(p, s); break;
    case 3: launch<3>(p, s); break;
    case 4: launch<4>(p, s); break;
    case 5: launch<5>(p, s); break;
    case 6: launch<6>(p, s); break;
    case 7: launch<7>(p, s); break;
    default: launch<8>(p, s); break;
  }
  VISTA_LAUNCH_CHECK();
  return VISTA_OK;
}

}  // namespace vista
