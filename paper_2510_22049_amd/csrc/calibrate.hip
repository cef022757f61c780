// Calibration kernels of the benchmark side (not on the product path): what this
// part really sustains, measured with the instructions the hot kernels are made of.
//
//   * matrix pipe alone: independent 32x32x16 bf16 MFMAs back to back -> achievable
//     MFMA rate and, from it, the shader clock under load (1024 flop per clock and SIMD);
//   * streaming read: every lane sums 16-byte loads over a large buffer -> achievable
//     HBM read bandwidth;
//   * vector-ALU issue costs: clocks per wave-instruction of v_exp_f32, v_add_f32,
//     v_cvt_pk_bf16_f32, and the issue-port time an MFMA takes away from them
//     (a loop of MFMAs plus a growing number of adds leaves the matrix-bound regime
//     where the port is full).
//
// Every loop body holds a known number of instructions on independent registers;
// the host divides the elapsed time by iterations x waves per SIMD.  One
// workgroup per compute unit, `waves_per_simd` x 4 waves each, so each SIMD runs
// exactly that many waves.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vista_calibrate.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;

template <int MODE>
__global__ void issue_kernel(float* sink, int iters, float seed) {
  float v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = seed + threadIdx.x * 1e-3f + i * 0.01f;
  f32x16 acc[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[k][i] = 0.f;
  f32x4 small[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(seed + i);
    b[i] = (__bf16)(seed - i);
  }
  uint32_t packed[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  uint32_t packed2[8] = {1, 1, 1, 1, 1, 1, 1, 1};
  bf16x8 qa = a, qb = b;
  float w[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) w[i] = seed * i;
  for (int it = 0; it < iters; ++it) {
    if constexpr (MODE == VISTA_CAL_EXP || MODE == VISTA_CAL_EXP_ADD) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = __builtin_amdgcn_exp2f(v[i]);
    }
    if constexpr (MODE == VISTA_CAL_ADD) {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] += seed;
    }
    if constexpr (MODE == VISTA_CAL_CVT) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        f32x2 f = {v[2 * i] + __uint_as_float(packed[i]), v[2 * i + 1]};   // keeps the conversions in the loop
        packed[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
      }
    }
    if constexpr (MODE == VISTA_CAL_EXP_ADD) {
      // 16 adds on registers the exponentials do not touch
#pragma unroll
      for (int i = 0; i < 16; ++i) w[i] += seed;
    }
    if constexpr (MODE == VISTA_CAL_MFMA || (MODE >= VISTA_CAL_MFMA_ADD16 && MODE <= VISTA_CAL_MFMA_ADD64) ||
                  MODE == VISTA_CAL_MFMA_EXP16) {
      constexpr int NADD = MODE == VISTA_CAL_MFMA_ADD16   ? 16
                           : MODE == VISTA_CAL_MFMA_ADD32 ? 32
                           : MODE == VISTA_CAL_MFMA_ADD48 ? 48
                           : MODE == VISTA_CAL_MFMA_ADD64 ? 64
                                                          : 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[k], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < NADD / 4; ++i) v[(k * (NADD / 4) + i) % 16] += seed;
        if constexpr (MODE == VISTA_CAL_MFMA_EXP16) {
#pragma unroll
          for (int i = 0; i < 4; ++i) v[4 * k + i] = __builtin_amdgcn_exp2f(v[4 * k + i]);
        }
      }
    }
    if constexpr (MODE == VISTA_CAL_MFMA_AGPR_ADD32) {
      // the same four MFMAs with their accumulators held in accumulation registers
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[k]) : "v"(a), "v"(b));
#pragma unroll
        for (int i = 0; i < 8; ++i) v[(8 * k + i) % 16] += seed;
      }
    }
    if constexpr (MODE == VISTA_CAL_MFMA4 || MODE == VISTA_CAL_MFMA4_ADD32) {
      const i16x4 a4 = {short(0x3F80), short(0x3F80), short(0x3F80), short(0x3F80)};
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const i16x4 b4 = {short(packed[(2 * k) % 8]), short(packed[(2 * k) % 8] >> 16), short(packed[(2 * k + 1) % 8]),
                          short(packed[(2 * k + 1) % 8] >> 16)};
        small[k % 4] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a4, b4, small[k % 4], 0, 0, 0);
        if constexpr (MODE == VISTA_CAL_MFMA4_ADD32) {
          v[(2 * k) % 16] += seed;
          v[(2 * k + 1) % 16] += seed;
        }
      }
    }
    if constexpr (MODE == VISTA_CAL_TILE_BODY) {
      // Two query blocks of the stage-1 tile loop with their true dependencies and nothing
      // else; per block: scores of the next block (2 MFMAs), two projection MFMAs, 16
      // exponentials of the previous scores, 8 packs, four 4x4x4 denominator MFMAs, two P.V
      // MFMAs.  acc[0] and acc[3] alternate as the score registers, acc[1] is the projection
      // accumulator, acc[2] the output accumulator.
      // (the score operands are weights of an earlier block only so that no product is loop-invariant)
      auto block = [&](const f32x16& sc, f32x16& nx, const bf16x8& qin, bf16x8& qout) __attribute__((always_inline)) {
        const f32x16 z = {0};
        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qin, z, 0, 0, 0);
        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, qin, nx, 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[1], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[1], 0, 0, 0);
        union { bf16x8 v; uint32_t w[4]; } p0, p1;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          f32x2 f = {__builtin_amdgcn_exp2f(sc[i]), __builtin_amdgcn_exp2f(sc[i + 1])};
          const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
          if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
        }
        const i16x4 a4 = {short(0x3F80), short(0x3F80), short(0x3F80), short(0x3F80)};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t w0 = k < 2 ? p0.w[2 * k] : p1.w[2 * k - 4], w1 = k < 2 ? p0.w[2 * k + 1] : p1.w[2 * k - 3];
          const i16x4 b4 = {short(w0), short(w0 >> 16), short(w1), short(w1 >> 16)};
          small[0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a4, b4, small[0], 0, 0, 0);
        }
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p0.v, acc[2], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, p1.v, acc[2], 0, 0, 0);
        qout = p1.v;
      };
      block(acc[0], acc[3], qa, qb);
      block(acc[3], acc[0], qb, qa);
    }
    if constexpr (MODE >= VISTA_CAL_TILE_BODY_NOSMALL && MODE <= VISTA_CAL_TILE_BODY_LOOSE) {
      // The same two query blocks with one ingredient taken out or one dependency loosened:
      //   NOSMALL  no 4x4x4 denominator MFMAs;   NOPROJ  no projection MFMAs;
      //   LOOSE    the same instructions, but the exponentials work on registers of their own
      //            (not on the scores the MFMAs just produced) and the P.V and denominator
      //            MFMAs take the packs made one block earlier.
      constexpr bool SMALL = MODE != VISTA_CAL_TILE_BODY_NOSMALL;
      constexpr bool PROJ = MODE != VISTA_CAL_TILE_BODY_NOPROJ;
      constexpr bool LOOSE = MODE == VISTA_CAL_TILE_BODY_LOOSE;
      auto block = [&](f32x16& sc, f32x16& nx, const bf16x8& qin, bf16x8& qout, uint32_t* pin, uint32_t* pout) __attribute__((always_inline)) {
        const f32x16 z = {0};
        if constexpr (LOOSE) {
          nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qin, nx, 0, 0, 0);
        } else {
          nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qin, z, 0, 0, 0);
        }
        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, qin, nx, 0, 0, 0);
        if constexpr (PROJ) {
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[1], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[1], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          float e0, e1;
          if constexpr (LOOSE) {
            e0 = v[i] = __builtin_amdgcn_exp2f(v[i]);
            e1 = v[i + 1] = __builtin_amdgcn_exp2f(v[i + 1]);
          } else {
            e0 = __builtin_amdgcn_exp2f(sc[i]);
            e1 = __builtin_amdgcn_exp2f(sc[i + 1]);
          }
          f32x2 f = {e0, e1};
          pout[i / 2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
        }
        const uint32_t* pu = LOOSE ? pin : pout;
        if constexpr (SMALL) {
          const i16x4 a4 = {short(0x3F80), short(0x3F80), short(0x3F80), short(0x3F80)};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const i16x4 b4 = {short(pu[2 * k]), short(pu[2 * k] >> 16), short(pu[2 * k + 1]), short(pu[2 * k + 1] >> 16)};
            small[k & 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a4, b4, small[k & 1], 0, 0, 0);
          }
        }
        union { bf16x8 v; uint32_t w[4]; } p0, p1;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          p0.w[k] = pu[k];
          p1.w[k] = pu[4 + k];
        }
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p0.v, acc[2], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, p1.v, acc[2], 0, 0, 0);
        qout = p1.v;
      };
      block(acc[0], acc[3], qa, qb, packed2, packed);
      block(acc[3], acc[0], qb, qa, packed, packed2);
    }
    if constexpr (MODE >= VISTA_CAL_TILE_BODY_LDS && MODE <= VISTA_CAL_TILE_BODY_LDS_BAR_PUB) {
      // The two query blocks again, now with the traffic the kernel has around them:
      //   LDS          the projection MFMAs take both operands from LDS (4 ds_read_b128 per block)
      //                and the second P.V MFMA takes its A operand from LDS (1 per block);
      //   LDS_BAR      plus one LDS-only workgroup barrier every four blocks (a tile);
      //   LDS_BAR_PUB  plus, per tile, the publication of a projected tile: 8 packs of the
      //                projection accumulator and two ds_write_b128.
      constexpr bool BAR = MODE >= VISTA_CAL_TILE_BODY_LDS_BAR;
      constexpr bool PUB = MODE == VISTA_CAL_TILE_BODY_LDS_BAR_PUB;
      __shared__ uint4 lbuf[(10 + 2 * 16) * 64];   // ten operand slabs of 1 KB read by every wave + two per wave slot for publishing
      const int lane = threadIdx.x & 63, slot = threadIdx.x >> 6;
      uint4* mine = lbuf + lane;
      uint4* pub = lbuf + (10 + 2 * slot) * 64 + lane;
      if (it == 0) {
        for (int k = slot; k < 10; k += blockDim.x >> 6) mine[k * 64] = make_uint4(0x3F803F80u, 0x3F003F00u, 0x3E803E80u, 0x3F803F80u);
        __syncthreads();
      }
      auto block = [&](const f32x16& sc, f32x16& nx, const bf16x8& qin, bf16x8& qout, int half) __attribute__((always_inline)) {
        const f32x16 z = {0};
        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qin, z, 0, 0, 0);
        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, qin, nx, 0, 0, 0);
        union U { bf16x8 v; uint4 u; uint32_t w[4]; };
        U x0, w0, x1, w1, vv;
        x0.u = mine[(5 * half + 0) * 64];
        w0.u = mine[(5 * half + 1) * 64];
        x1.u = mine[(5 * half + 2) * 64];
        w1.u = mine[(5 * half + 3) * 64];
        vv.u = mine[(5 * half + 4) * 64];
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0.v, w0.v, acc[1], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1.v, w1.v, acc[1], 0, 0, 0);
        U p0, p1;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          f32x2 f = {__builtin_amdgcn_exp2f(sc[i]), __builtin_amdgcn_exp2f(sc[i + 1])};
          const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
          if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
        }
        const i16x4 a4 = {short(0x3F80), short(0x3F80), short(0x3F80), short(0x3F80)};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t w0_ = k < 2 ? p0.w[2 * k] : p1.w[2 * k - 4], w1_ = k < 2 ? p0.w[2 * k + 1] : p1.w[2 * k - 3];
          const i16x4 b4 = {short(w0_), short(w0_ >> 16), short(w1_), short(w1_ >> 16)};
          small[k & 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a4, b4, small[k & 1], 0, 0, 0);
        }
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p0.v, acc[2], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv.v, p1.v, acc[2], 0, 0, 0);
        qout = p1.v;
      };
      block(acc[0], acc[3], qa, qb, 0);
      block(acc[3], acc[0], qb, qa, 1);
      if (it & 1) {                          // every four blocks: the end of a tile
        if constexpr (PUB) {
          union { uint4 u; uint32_t w[4]; } r0, r1;
#pragma unroll
          for (int i = 0; i < 16; i += 2) {
            f32x2 f = {acc[1][i], acc[1][i + 1]};
            const uint32_t pk = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
            if (i < 8) r0.w[i / 2] = pk; else r1.w[(i - 8) / 2] = pk;
          }
          pub[0] = r0.u;
          pub[64] = r1.u;
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[1][i] = 0.f;
        }
        if constexpr (BAR) {
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
          __builtin_amdgcn_s_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        }
      }
      asm volatile("" ::: "memory");          // the buffer counts as changed: the operand reads stay in the loop
    }
    if constexpr (MODE == VISTA_CAL_MFMA16) {
#pragma unroll
      for (int k = 0; k < 4; ++k) small[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, small[k], 0, 0, 0);
    }
    if constexpr (MODE == VISTA_CAL_MFMA16_ADD32) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        small[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, small[k], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[(8 * k + i) % 16] += seed;
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += v[i] + w[i];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[k][i];
#pragma unroll
    for (int i = 0; i < 4; ++i) s += small[k][i];
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) s += __uint_as_float(packed[i]) + __uint_as_float(packed2[i]);
  if (s == 12345.678f) sink[threadIdx.x] = s;   // never true for the seeds used; keeps the loop alive
}

// LDS operand reads: every lane reads 16 bytes at 16 x lane (the conflict-free pattern of the
// MFMA operand buffers), 16 independent ds_read_b128 per iteration and wave; `mfmas` > 0 adds
// that many independent 32x32x16 MFMAs per iteration to see whether the two overlap.
template <int MFMAS>
__global__ void lds_read_kernel(float* sink, int iters) {
  __shared__ uint4 buf[16 * 64 * 4];        // 64 KB: 16 slabs of 1 KB per wave slot (4 slots, shared beyond)
  for (int i = threadIdx.x; i < 16 * 64 * 4; i += blockDim.x) buf[i] = make_uint4(i, i + 1, i + 2, i + 3);
  __syncthreads();
  const int lane = threadIdx.x & 63, slot = (threadIdx.x >> 6) & 3;
  const uint4* base = buf + slot * 16 * 64 + lane;
  uint4 acc = make_uint4(0, 0, 0, 0);
  f32x16 m[2] = {{0}, {0}};
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(1.0f + i);
    b[i] = (__bf16)(1.0f - i);
  }
  for (int it = 0; it < iters; ++it) {
    uint4 v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = base[k * 64];
    asm volatile("" ::: "memory");          // the buffer counts as changed: the reads stay in the loop
#pragma unroll
    for (int k = 0; k < MFMAS; ++k) m[k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, m[k & 1], 0, 0, 0);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      acc.x ^= v[k].x;
      acc.y ^= v[k].y;
      acc.z ^= v[k].z;
      acc.w ^= v[k].w;
    }
  }
  float s = m[0][0] + m[1][0];
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345679u || s == 12345.678f) sink[threadIdx.x] = 1.f;
}

// Streaming read: grid-stride over 16-byte words, four loads in flight per lane.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, int64_t n16, float* sink) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  uint32_t s = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    s += (a.x ^ a.y ^ a.z ^ a.w) + (b.x ^ b.y ^ b.z ^ b.w) + (c.x ^ c.y ^ c.z ^ c.w) + (d.x ^ d.y ^ d.z ^ d.w);
  }
  for (; i < n16; i += stride) {
    const uint4 a = src[i];
    s += a.x ^ a.y ^ a.z ^ a.w;
  }
  if (s == 0x12345679u) sink[threadIdx.x] = 1.f;
}

template <int MODE>
hipError_t run_issue(int waves_per_simd, int iters, float* sink, hipStream_t s) {
  hipLaunchKernelGGL(issue_kernel<MODE>, dim3(256), dim3(256 * waves_per_simd), 0, s, sink, iters, 1.0f);
  return hipGetLastError();
}

}  // namespace

extern "C" int vista_calibrate_issue(int what, int waves_per_simd, int iters, float* sink, void* hip_stream) {
  if (waves_per_simd < 1 || waves_per_simd > 4 || iters < 1 || !sink) return 1;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  switch (what) {
    case VISTA_CAL_EXP: e = run_issue<VISTA_CAL_EXP>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_ADD: e = run_issue<VISTA_CAL_ADD>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_CVT: e = run_issue<VISTA_CAL_CVT>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_EXP_ADD: e = run_issue<VISTA_CAL_EXP_ADD>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA: e = run_issue<VISTA_CAL_MFMA>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA_ADD16: e = run_issue<VISTA_CAL_MFMA_ADD16>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA_ADD32: e = run_issue<VISTA_CAL_MFMA_ADD32>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA_ADD48: e = run_issue<VISTA_CAL_MFMA_ADD48>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA_ADD64: e = run_issue<VISTA_CAL_MFMA_ADD64>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA_EXP16: e = run_issue<VISTA_CAL_MFMA_EXP16>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA16: e = run_issue<VISTA_CAL_MFMA16>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA16_ADD32: e = run_issue<VISTA_CAL_MFMA16_ADD32>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA_AGPR_ADD32: e = run_issue<VISTA_CAL_MFMA_AGPR_ADD32>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA4: e = run_issue<VISTA_CAL_MFMA4>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_TILE_BODY: e = run_issue<VISTA_CAL_TILE_BODY>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_MFMA4_ADD32: e = run_issue<VISTA_CAL_MFMA4_ADD32>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_TILE_BODY_NOSMALL: e = run_issue<VISTA_CAL_TILE_BODY_NOSMALL>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_TILE_BODY_NOPROJ: e = run_issue<VISTA_CAL_TILE_BODY_NOPROJ>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_TILE_BODY_LOOSE: e = run_issue<VISTA_CAL_TILE_BODY_LOOSE>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_TILE_BODY_LDS: e = run_issue<VISTA_CAL_TILE_BODY_LDS>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_TILE_BODY_LDS_BAR: e = run_issue<VISTA_CAL_TILE_BODY_LDS_BAR>(waves_per_simd, iters, sink, s); break;
    case VISTA_CAL_TILE_BODY_LDS_BAR_PUB: e = run_issue<VISTA_CAL_TILE_BODY_LDS_BAR_PUB>(waves_per_simd, iters, sink, s); break;
    default: return 1;
  }
  return e == hipSuccess ? 0 : 2;
}

extern "C" int vista_calibrate_lds_read(int mfmas, int waves_per_simd, int iters, float* sink, void* hip_stream) {
  if (waves_per_simd < 1 || waves_per_simd > 4 || iters < 1 || !sink) return 1;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (mfmas == 0)
    hipLaunchKernelGGL(lds_read_kernel<0>, dim3(256), dim3(256 * waves_per_simd), 0, s, sink, iters);
  else if (mfmas == 8)
    hipLaunchKernelGGL(lds_read_kernel<8>, dim3(256), dim3(256 * waves_per_simd), 0, s, sink, iters);
  else
    return 1;
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

extern "C" int vista_calibrate_stream_read(const void* src, int64_t bytes, float* sink, void* hip_stream) {
  if (!src || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15) != 0) return 1;
  hipLaunchKernelGGL(stream_read_kernel, dim3(256 * 16), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint4*>(src), bytes / 16, sink);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
