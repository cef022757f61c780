// SiLU-gated block between two summarization layers on the matrix cores
// (bf16 MFMA, fp32 accumulate), gfx950.
//
//   yhat = y / sqrt(mean_d(y^2) + eps),   out = (SiLU(yhat W_g) * (yhat W_u)) W_o
//
// All three products are formed transposed, with the rows of y on the MFMA
// column index, so that a lane owns one row of y throughout:
//   G^T[f][m] = sum_k W_g[k][f] y[m][k]      (A = W_g^T block, B = y^T)
//   H^T[f][m] = SiLU(r_m G^T) * (r_m U^T)    per-lane scalar r_m = 1/rms(y_m): the norm is
//                                            applied to the accumulators, not to the operand
//   out^T[o][m] += sum_f W_o[f][o] H^T[f][m] (A = W_o^T block, B = H^T straight from the
//                                            accumulator registers of the first product)
// A workgroup (4 waves, one per SIMD: the out^T accumulators alone are 128 registers at
// d = 256) takes 128 rows, a wave 32 of them: its y^T operands stay in registers, the
// out^T accumulators too.  The hidden dimension is walked in steps of
// 32: per step the three weight panels that touch those 32 hidden units are turned
// into A operands -- the weights are row-major [in, out], the operand wants the
// input index along a lane's registers, so each 32x32 block is transposed by the
// matrix core itself (block times a 0/1 selector lands in accumulator layout, which
// is operand layout with the lane on the block's column index) -- and parked in
// LDS, double-buffered, where all four waves read them.  The order in which a
// lane's registers walk a 16-wide slice of a contraction index is the accumulator's
// ({4 hf + r, 8 + 4 hf + r}); both operands of every product use the same order.
#include "common.hpp"

namespace vista {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

namespace {

constexpr int kFfnWaves = 4;
constexpr int kFfnRows = 32 * kFfnWaves;   // rows of y per workgroup

struct FfnParams {
  const uint16_t* y;
  const uint16_t* Wg;
  const uint16_t* Wu;
  const uint16_t* Wo;
  uint16_t* out;
  int64_t rows;
  int dff;
  float eps;
};

union Pack8 {
  bf16x8 v;
  uint4 u;
  uint2 d[2];
  uint16_t h[8];
  uint32_t w[4];
};

__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 r = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Operands of one hidden step in LDS: W_g^T and W_u^T for every 16-slice of the input
// index, W_o^T for both 16-slices of the step's hidden units and every 32-block of outputs.
template <int D>
struct FfnLds {
  static constexpr int KS = D / 16, OB = D / 32;
  union {
    uint4 op[2][2 * KS + 2 * OB][64];
    uint4 stage[kFfnWaves][32 * 16];   // at the end: half of a wave's 32 output rows (256 B each)
  };
};

template <int D>
__global__ __launch_bounds__(64 * kFfnWaves) void ffn_mfma_kernel(FfnParams p) {
  constexpr int KS = D / 16;             // 16-slices of the input index
  constexpr int OB = D / 32;             // 32-blocks of the output index
  constexpr int NBLK = KS + OB;          // 32x32 weight blocks to transpose per hidden step
  __shared__ FfnLds<D> sm;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hf = lane >> 5, l32 = lane & 31;
  const int64_t row0 = int64_t(blockIdx.x) * kFfnRows + 32 * wave;
  int64_t myrow = row0 + l32;
  if (myrow > p.rows - 1) myrow = p.rows - 1;     // rows past the end repeat the last one; never stored

  // ---- y^T operands of this lane's row, and its 1/rms
  bf16x8 yop[KS];
  float ss = 0.f;
  {
    const char* yr = reinterpret_cast<const char*>(p.y) + myrow * (D * 2) + 8 * hf;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      Pack8 t;
      t.d[0] = *reinterpret_cast<const uint2*>(yr + 32 * s);         // k = 16 s + 4 hf + 0..3
      t.d[1] = *reinterpret_cast<const uint2*>(yr + 32 * s + 16);    // k = 16 s + 8 + 4 hf + 0..3
      yop[s] = t.v;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float a = bf16_lo(t.w[w]), b = bf16_hi(t.w[w]);
        ss = fmaf(a, a, fmaf(b, b, ss));
      }
    }
  }
  ss += __shfl_xor(ss, 32, 64);
  const float rinv = __builtin_amdgcn_rsqf(ss * (1.0f / D) + p.eps);

  // selector operands: Sel_q[c][j] = (16 q + c == j)
  Pack8 sel[2];
#pragma unroll
  for (int q = 0; q < 2; ++q)
#pragma unroll
    for (int j = 0; j < 8; ++j) sel[q].h[j] = (l32 == 16 * q + 8 * hf + j) ? 0x3F80 : 0;

  // Block b of hidden step n: b < KS/2 -> W_g rows 32 b.., columns 32 n..; b < KS -> W_u likewise;
  // else W_o rows 32 n.., columns 32 (b - KS)...  Its two operands go to slots s0, s0 + 1.
  constexpr int BPW = (NBLK + kFfnWaves - 1) / kFfnWaves;   // blocks a wave transposes per step
  auto load_block = [&](int n, int b, Pack8& a0, Pack8& a1) __attribute__((always_inline)) {
    const uint16_t* W;
    int ld, r0, c0;
    if (b < KS / 2) { W = p.Wg; ld = p.dff; r0 = 32 * b; c0 = 32 * n; }
    else if (b < KS) { W = p.Wu; ld = p.dff; r0 = 32 * (b - KS / 2); c0 = 32 * n; }
    else { W = p.Wo; ld = D; r0 = 32 * n; c0 = 32 * (b - KS); }
    const uint16_t* src = W + int64_t(r0 + l32) * ld + c0 + 8 * hf;
    a0.u = *reinterpret_cast<const uint4*>(src);
    a1.u = *reinterpret_cast<const uint4*>(src + 16);
  };
  auto store_block = [&](int buf, int b, const Pack8& a0, const Pack8& a1) __attribute__((always_inline)) {
    f32x16 t = {0};
    t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, sel[0].v, t, 0, 0, 0);
    t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, sel[1].v, t, 0, 0, 0);
    Pack8 o0, o1;
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
      o0.w[i / 2] = cvt_pk_bf16(t[i], t[i + 1]);
      o1.w[i / 2] = cvt_pk_bf16(t[8 + i], t[8 + i + 1]);
    }
    int s0;
    if (b < KS / 2) s0 = 2 * b;
    else if (b < KS) s0 = KS + 2 * (b - KS / 2);
    else s0 = 2 * KS + 2 * (b - KS);
    sm.op[buf][s0][lane] = o0.u;
    sm.op[buf][s0 + 1][lane] = o1.u;
  };

  const int nsteps = p.dff / 32;
  Pack8 raw[BPW][2];
#pragma unroll
  for (int i = 0; i < BPW; ++i) {
    const int b = wave + kFfnWaves * i;
    if (b < NBLK) load_block(0, b, raw[i][0], raw[i][1]);
  }
#pragma unroll
  for (int i = 0; i < BPW; ++i) {
    const int b = wave + kFfnWaves * i;
    if (b < NBLK) store_block(0, b, raw[i][0], raw[i][1]);
  }

  f32x16 acc[OB];
#pragma unroll
  for (int ob = 0; ob < OB; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[ob][i] = 0.f;

  for (int n = 0; n < nsteps; ++n) {
    const int buf = n & 1;
    lds_barrier();                     // step n's operands are in place; the other buffer is free
    const bool more = n + 1 < nsteps;
    if (more) {
#pragma unroll
      for (int i = 0; i < BPW; ++i) {
        const int b = wave + kFfnWaves * i;
        if (b < NBLK) load_block(n + 1, b, raw[i][0], raw[i][1]);
      }
    }
    f32x16 G = {0}, U = {0};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      Pack8 ag, au;
      ag.u = sm.op[buf][s][lane];
      au.u = sm.op[buf][KS + s][lane];
      G = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag.v, yop[s], G, 0, 0, 0);
      U = __builtin_amdgcn_mfma_f32_32x32x16_bf16(au.v, yop[s], U, 0, 0, 0);
    }
    Pack8 h0, h1;
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      float hv[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const float g = G[i + e] * rinv, u = U[i + e] * rinv;
        const float sig = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-kLog2e * g));
        hv[e] = g * sig * u;
      }
      const uint32_t pk = cvt_pk_bf16(hv[0], hv[1]);
      if (i < 8) h0.w[i / 2] = pk; else h1.w[(i - 8) / 2] = pk;
    }
#pragma unroll
    for (int ob = 0; ob < OB; ++ob) {
      Pack8 a0, a1;
      a0.u = sm.op[buf][2 * KS + 2 * ob][lane];
      a1.u = sm.op[buf][2 * KS + 2 * ob + 1][lane];
      acc[ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, h0.v, acc[ob], 0, 0, 0);
      acc[ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, h1.v, acc[ob], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < BPW; ++i) {
        const int b = wave + kFfnWaves * i;
        if (b < NBLK) store_block(buf ^ 1, b, raw[i][0], raw[i][1]);
      }
    }
  }

  // ---- out^T accumulators -> rows of out, through LDS so that the stores are whole rows.
  // Register group g of block ob holds outputs 32 ob + 8 g + 4 hf + 0..3 of the lane's row:
  // 8 bytes at 16-byte chunk 4 ob + g, half hf.  Two passes of 256 B per row.
  lds_barrier();                       // everybody is done with the operand buffers
  constexpr int HALF = OB / 2 > 0 ? OB / 2 : 1;    // output blocks per pass (128 channels)
#pragma unroll
  for (int pass = 0; pass < OB / HALF; ++pass) {
#pragma unroll
    for (int obh = 0; obh < HALF; ++obh) {
      const int ob = pass * HALF + obh;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 pk;
        pk.x = cvt_pk_bf16(acc[ob][4 * g], acc[ob][4 * g + 1]);
        pk.y = cvt_pk_bf16(acc[ob][4 * g + 2], acc[ob][4 * g + 3]);
        const int chunk = 4 * obh + g;             // < 4 HALF <= 16
        reinterpret_cast<uint2*>(&sm.stage[wave][l32 * 16 + (chunk ^ (l32 & 15))])[hf] = pk;
      }
    }
    // the wave reads back what it alone wrote (LDS keeps a wave's accesses in order; the
    // compiler must too)
    asm volatile("" ::: "memory");
    constexpr int CH = 4 * HALF;                   // 16-byte chunks per row in this pass
#pragma unroll
    for (int i = 0; i < (32 * CH) / 64; ++i) {
      const int q = i * 64 + lane;
      const int r = q / CH, c = q % CH;
      const uint4 v = sm.stage[wave][r * 16 + (c ^ (r & 15))];
      if (row0 + r < p.rows)
        *reinterpret_cast<uint4*>(reinterpret_cast<char*>(p.out) + (row0 + r) * (D * 2) + pass * (HALF * 64) + c * 16) = v;
    }
    asm volatile("" ::: "memory");
  }
}

}  // namespace

bool mfma_sglu_ffn_supported(const vista_ffn_desc& d) {
  return d.dtype == VISTA_BF16 && (d.d == 128 || d.d == 256) && d.d_ff >= 32 && d.d_ff % 32 == 0 &&
         d.rows > 0 && (int64_t(d.rows) + kFfnRows - 1) / kFfnRows <= 0x7FFFFFFF;
}

vista_status mfma_sglu_ffn(const vista_ffn_desc& d, float eps, const void* y, const void* Wg, const void* Wu,
                           const void* Wo, void* out, hipStream_t s) {
  FfnParams p;
  p.y = static_cast<const uint16_t*>(y);
  p.Wg = static_cast<const uint16_t*>(Wg);
  p.Wu = static_cast<const uint16_t*>(Wu);
  p.Wo = static_cast<const uint16_t*>(Wo);
  p.out = static_cast<uint16_t*>(out);
  p.rows = d.rows;
  p.dff = d.d_ff;
  p.eps = eps;
  const unsigned blocks = unsigned((int64_t(d.rows) + kFfnRows - 1) / kFfnRows);
  if (d.d == 128)
    VISTA_LAUNCH(ffn_mfma_kernel<128>, dim3(blocks), dim3(64 * kFfnWaves), 0, s, p);
  else
    VISTA_LAUNCH(ffn_mfma_kernel<256>, dim3(blocks), dim3(64 * kFfnWaves), 0, s, p);
  return VISTA_OK;
}

}  // namespace vista
