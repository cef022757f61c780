// Stage 2 on the matrix cores (bf16 MFMA, fp32 accumulate), gfx950.
//
// One workgroup (8 waves) serves one user and four heads; a round scores 64
// candidates: wave (head h, half c) takes the 32 candidates of half c for
// head h.  The user's S summary tokens of a head are resident twice: as the K
// operand of S^T = K Q^T (keys x candidates) in each wave's registers, and,
// transposed, as the V operand of O^T = V^T P^T in LDS, shared by the head's two
// waves.  The transposed copy is made by the matrix core itself (K block times
// a 0/1 selector matrix lands in the accumulator layout, which is the A-operand
// layout of the second product).
//
// HBM traffic is fully coalesced and never touches vector registers on the way
// in: the 64 x 256 B candidate tile of the next round is brought in by direct
// global->LDS loads (each 16 lanes fetch one whole row) while this round is
// computed; the finished 64 x 256 B output tile is staged in LDS and stored as
// whole rows one round later.  Both tiles keep their 16-byte chunks at position
// chunk XOR (row mod 16), so row-wise fills and column-wise operand accesses are
// both free of bank conflicts.
//
// Key blocks stream past a candidate block (scores -> 2^s -> P V accumulate);
// a lane owns one candidate column, so the softmax statistics are per-lane.
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
constexpr int kRound = 64;                 // candidates per round
constexpr int kTileChunks = kRound * 16;   // 16-byte chunks of a 64 x 256 B tile

struct AttendParams {
  const uint16_t* cand;
  const uint16_t* summ;
  uint16_t* out;
  int B, C, S, d, H;
  int rounds_per_wg;  // rounds (of 64 candidates) a workgroup takes
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

__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int NKB>
struct AttendLds {
  uint4 qbuf[2][kTileChunks];        // candidate tiles: row r, chunk c at [r * 16 + (c ^ (r & 15))]
  uint4 obuf[2][kTileChunks];        // output tiles, same arrangement
  uint4 vop[4][NKB][2][64];          // V operands: [head][key block][half of the 16 registers][lane]
};

// NKB = S / 32 key blocks.
template <int NKB>
__global__ __launch_bounds__(512) void attend_mfma_kernel(AttendParams p) {
  __shared__ AttendLds<NKB> sm;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hl = wave >> 1;            // head within the group of four
  const int half = wave & 1;           // which 32 candidates of a round
  const int hf = lane >> 5, l32 = lane & 31;
  const int hgroups = p.H / 4;
  int id = blockIdx.x;
  const int chunk = id % p.chunks;
  id /= p.chunks;
  const int hg = id % hgroups;
  const int b = id / hgroups;
  const int h = hg * 4 + hl;
  const int row_bytes = p.d * 2;
  const int slice = hg * 256;          // byte offset of this head group's 128 channels inside a row

  const int nrounds_total = (p.C + kRound - 1) / kRound;
  const int r0 = chunk * p.rounds_per_wg;
  int r1 = r0 + p.rounds_per_wg;
  if (r1 > nrounds_total) r1 = nrounds_total;
  const char* Tb = reinterpret_cast<const char*>(p.cand) + int64_t(b) * p.C * row_bytes + slice;
  char* Ob = reinterpret_cast<char*>(p.out) + int64_t(b) * p.C * row_bytes + slice;

  // Direct global->LDS fill of one candidate tile: two 16-byte loads per lane; lane l of
  // instruction i of wave w fills LDS chunk j = (2 w + i) * 64 + l, i.e. tile row j / 16,
  // and fetches that row's chunk (j % 16) ^ (row % 16).  Rows past C are clamped.
  auto fill = [&](int round, int qb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int j = (2 * wave + i) * 64 + lane;
      const int row = j >> 4;
      int cand = round * kRound + row;
      if (cand > p.C - 1) cand = p.C - 1;
      const uint32_t voff = uint32_t(cand) * uint32_t(row_bytes) + uint32_t(((j & 15) ^ (row & 15)) * 16);
      const uint32_t lds_base = uint32_t(reinterpret_cast<uintptr_t>(
          (void __attribute__((address_space(3)))*)(&sm.qbuf[qb][(2 * wave + i) * 64])));
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(lds_base), "v"(voff), "s"(Tb)
                   : "memory", "m0");
    }
  };
  // Whole-row store of a finished output tile (rows past C are skipped).
  auto drain = [&](int round, int ob) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int j = (2 * wave + i) * 64 + lane;
      const int row = j >> 4;
      const int cand = round * kRound + row;
      if (cand < p.C) {
        const uint4 v = sm.obuf[ob][j];
        *reinterpret_cast<uint4*>(Ob + int64_t(cand) * row_bytes + ((j & 15) ^ (row & 15)) * 16) = v;
      }
    }
  };

  if (r0 < r1) fill(r0, 0);            // first tile on its way while the operands are set up

  // ---- resident operands of this (user, head): K in registers (both waves of the head),
  //      V through the selector MFMA into LDS (each wave builds half of the key blocks)
  bf16x8 kop[NKB][2];
  float kmax2 = 0.f;
  {
    const uint16_t* Y = p.summ + int64_t(b) * p.S * p.d + 32 * h + 8 * hf;
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
        k[ks].u = *reinterpret_cast<const uint4*>(Y + int64_t(kb * 32 + l32) * p.d + 16 * ks);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float a = bf16_lo(k[ks].w[w]), c2 = bf16_hi(k[ks].w[w]);
          n2 = fmaf(a, a, fmaf(c2, c2, n2));
        }
      }
      n2 += __shfl_xor(n2, 32, 64);
      kmax2 = fmaxf(kmax2, n2);
      if ((kb & 1) == half) {
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
        sm.vop[hl][kb][0][lane] = v0.u;
        sm.vop[hl][kb][1][lane] = v1.u;
      }
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

  // operand position of this lane inside a tile: row = 32 half + l32, chunk = 4 hl + 2 ks + hf
  const int orow = 32 * half + l32;
  const int osw = orow & 15;

  for (int r = r0; r < r1; ++r) {
    const int cur = (r - r0) & 1;
    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): this wave's part of tile r has landed
    lds_barrier();                               // ... and everybody else's; obuf[cur] is free again
    if (r + 1 < r1) fill(r + 1, cur ^ 1);
    if (r > r0) drain(r - 1, cur ^ 1);

    Pack8 c0, c1;
    c0.u = sm.qbuf[cur][orow * 16 + ((4 * hl + hf) ^ osw)];
    c1.u = sm.qbuf[cur][orow * 16 + ((4 * hl + 2 + hf) ^ osw)];
    float qn2 = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float a0 = bf16_lo(c0.w[w]), a1 = bf16_hi(c0.w[w]), b0 = bf16_lo(c1.w[w]), b1 = bf16_hi(c1.w[w]);
      qn2 = fmaf(a0, a0, fmaf(a1, a1, fmaf(b0, b0, fmaf(b1, b1, qn2))));
    }
    qn2 += __shfl_xor(qn2, 32, 64);
    const bool general = __builtin_amdgcn_ballot_w64(qn2 * kmax2 > kSafeBound2) != 0;
    // Key blocks stream through: 32 keys x 32 candidates of scores at a time.  The common
    // route is straight-line code over all key blocks (one scheduling region).
    f32x16 o = {0};
    float l[4] = {0.f, 0.f, 0.f, 0.f};
    if (!general) {
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
        f32x16 sc = {0};
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kb][0], c0.v, sc, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kb][1], c1.v, sc, 0, 0, 0);
        Pack8 v0, v1;
        v0.u = sm.vop[hl][kb][0][lane];
        v1.u = sm.vop[hl][kb][1][lane];
        Pack8 p0, p1;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const uint32_t pk = cvt_pk_bf16(__builtin_amdgcn_exp2f(sc[i]), __builtin_amdgcn_exp2f(sc[i + 1]));
          l[(i / 2) & 3] = dot2_ones(pk, l[(i / 2) & 3]);
          if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
        }
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0.v, p0.v, o, 0, 0, 0);
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1.v, p1.v, o, 0, 0, 0);
      }
    } else {
      float m = -INFINITY;
#pragma unroll 1
      for (int kb = 0; kb < NKB; ++kb) {
        f32x16 sc = {0};
        Pack8 ka, kb2;
        // dynamic key-block index: operands come back from LDS-free registers through a switch-free path
        ka.v = kop[0][0]; kb2.v = kop[0][1];
#pragma unroll
        for (int t = 1; t < NKB; ++t)
          if (t == kb) { ka.v = kop[t][0]; kb2.v = kop[t][1]; }
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, c0.v, sc, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb2.v, c1.v, sc, 0, 0, 0);
        Pack8 v0, v1;
        v0.u = sm.vop[hl][kb][0][lane];
        v1.u = sm.vop[hl][kb][1][lane];
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
        Pack8 p0, p1;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const uint32_t pk = cvt_pk_bf16(__builtin_amdgcn_exp2f(sc[i] - mnew), __builtin_amdgcn_exp2f(sc[i + 1] - mnew));
          l[(i / 2) & 3] = dot2_ones(pk, l[(i / 2) & 3]);
          if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
        }
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0.v, p0.v, o, 0, 0, 0);
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1.v, p1.v, o, 0, 0, 0);
      }
    }
    float lsum = (l[0] + l[1]) + (l[2] + l[3]);
    lsum += __shfl_xor(lsum, 32, 64);
    const float inv = __builtin_amdgcn_rcpf(lsum);
    // register group g holds channels 8 g + 4 hf + 0..3 of the head: 8 bytes at chunk 4 hl + g, half hf
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 pk;
      pk.x = cvt_pk_bf16(o[4 * g] * inv, o[4 * g + 1] * inv);
      pk.y = cvt_pk_bf16(o[4 * g + 2] * inv, o[4 * g + 3] * inv);
      reinterpret_cast<uint2*>(&sm.obuf[cur][orow * 16 + ((4 * hl + g) ^ osw)])[hf] = pk;
    }
  }
  if (r0 < r1) {
    lds_barrier();
    drain(r1 - 1, (r1 - 1 - r0) & 1);
  }
}

template <int NKB>
void launch(const AttendParams& p, hipStream_t s) {
  const unsigned blocks = unsigned(p.B) * unsigned(p.H / 4) * unsigned(p.chunks);
  hipLaunchKernelGGL(attend_mfma_kernel<NKB>, dim3(blocks), dim3(512), 0, s, p);
}

}  // namespace

bool mfma_target_attend_supported(const vista_attend_desc& d) {
  return d.dtype == VISTA_BF16 && d.d == 32 * d.H && d.H % 4 == 0 && d.S % 32 == 0 && d.S <= 256 &&
         int64_t(d.C) * d.d * 2 < (int64_t(1) << 32);
}

vista_status mfma_target_attend(const vista_attend_desc& d, float scale_log2, const void* cand,
                                const void* summ, void* out, hipStream_t s) {
  AttendParams p;
  p.cand = static_cast<const uint16_t*>(cand);
  p.summ = static_cast<const uint16_t*>(summ);
  p.out = static_cast<uint16_t*>(out);
  p.B = d.B; p.C = d.C; p.S = d.S; p.d = d.d; p.H = d.H;
  p.c = scale_log2;
  // Rounds per workgroup: long enough to amortise the operand set-up (about two rounds'
  // worth of work), short enough to give the chip >= 512 workgroups.
  const int nrounds = (d.C + kRound - 1) / kRound;
  const int64_t groups = int64_t(d.B) * (d.H / 4);
  int per = 8;
  while (per > 2 && groups * ((nrounds + per - 1) / per) < 512) per >>= 1;
  p.rounds_per_wg = per;
  p.chunks = (nrounds + per - 1) / per;
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
