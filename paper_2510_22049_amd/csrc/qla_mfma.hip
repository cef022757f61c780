// Quasi-linear attention, stage 1, on the matrix cores (bf16 MFMA, fp32 accumulate), gfx950.
//
// Sec. 3.2.2 (target-side QLU equation, seeds as targets, history as source):
//     out_h = SiLU(Q_h) SiLU( Z_h ),   Z_h = SiLU(K_h)^T V_h = sum over items of SiLU(k_j)^T v_j.
// The state Z_h is d_h x d_h and additive over items (the block sums of App. B), so the
// history is streamed once: one workgroup per flat segment, one wave per head.  A wave keeps
// its head's 2 x (D x 32) projection weights in registers and, per tile of 32 items,
//   K = X W_k,h and V = X W_v,h           (2 x D/16 MFMAs; the X tile is shared through LDS,
//                                          filled by direct global->LDS loads, three tiles deep)
//   Z += SiLU(K)^T V                      (2 MFMAs: with items on the accumulator rows of both
//                                          projections, SiLU(K) and V already are the A and B
//                                          operands; the contraction runs over the items)
// Nothing is exchanged between waves; the only barrier per tile guards the X ring.  A piece
// (user x segment) ends with one 4 KB record Z_h in row-major fp32; the finishing kernel of
// the plain path sums a user's records in ascending segment order and applies the rest.
#include "common.hpp"

namespace vista {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

namespace {

constexpr int kTile = kTileItems;
constexpr int kRing = 3;

struct QlaParams {
  const uint16_t* X;
  const int64_t* offsets;
  const int* seg_user;
  const uint16_t* Wk;
  const uint16_t* Wv;
  float* partials;    // [slot][head][32][32] fp32
  int B, H;
  int64_t N;
  int seg;
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

__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Register i of a lane in half hf holds row 4 hf + acc_row0(i) of the 32x32 accumulator.
__device__ __forceinline__ constexpr int acc_row0(int i) { return 8 * (i / 4) + (i % 4); }

template <int V>
struct Int { static constexpr int value = V; };

// D = model width, one wave per head (D / 32 waves).
template <int D>
__global__ __launch_bounds__(D * 2, 2) void qla_state_mfma_kernel(QlaParams p) {
  constexpr int NW = D / 32;             // waves = heads
  constexpr int NT = NW * 64;
  constexpr int CH = D / 8;              // 16-byte chunks per row
  constexpr int KS = D / 16;             // k-slices of a projection
  constexpr int CPT = kTile * CH / NT;   // X chunks a thread moves per tile (= 8)
  static_assert(kTile * CH % NT == 0, "tile must split evenly over the workgroup");
  // At D = 256 the weights take half of the register file: scheduling fences keep the compiler from
  // hoisting (and holding) operand reads; at D = 128 there is room and it may interleave freely.
  constexpr bool kFence = D > 128;
  // X tiles, row-major: chunk c of item r sits at position c ^ (r & 15) of the row, so a wave-wide
  // direct load fetches four whole rows (1 KB of contiguous HBM) and the operand reads (lane = item,
  // fixed chunk) still spread over all banks
  __shared__ uint4 xbuf[kRing][CH * 32];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int hf = lane >> 5, l32 = lane & 31;
  const int h = __builtin_amdgcn_readfirstlane(tid >> 6);

  // Weights of this head as B operands: element j of slice ks is W[16 ks + 8 hf + j][32 h + l32].
  // The key weights carry -log2(e): the projection then yields t = -k log2(e) and
  // SiLU(k) = -ln(2) t / (1 + 2^t); the constant is applied once, to the record.
  bf16x8 wk[KS], wv[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    Pack8 a, b;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int64_t at = int64_t(16 * ks + 8 * hf + j) * D + 32 * h + l32;
      a.h[j] = f32_to_bf16_bits(__uint_as_float(uint32_t(p.Wk[at]) << 16) * -kLog2e);
      b.h[j] = p.Wv[at];
    }
    wk[ks] = a.v;
    wv[ks] = b.v;
    __builtin_amdgcn_sched_barrier(0);     // one slice's loads at a time: they all land in registers of their own
  }

  // A workgroup keeps its weights and takes segments blockIdx.x, blockIdx.x + gridDim.x, ...
  // (records are indexed by segment, so the result does not depend on the grid).
  for (int64_t g = blockIdx.x; g * p.seg < p.N; g += gridDim.x) {
  const int64_t seg_begin = g * p.seg;
  const int64_t seg_end = (seg_begin + p.seg < p.N) ? seg_begin + p.seg : p.N;
  TileCursor ca, cf;
  ca.init(p.offsets, p.B, p.seg_user ? __builtin_amdgcn_readfirstlane(p.seg_user[g]) : find_user(p.offsets, p.B, seg_begin),
          seg_begin, seg_end);
  if (!ca.valid) continue;               // only with invalid offsets (whole workgroup)
  cf = ca;

  const int wave = h;
  auto fetch = [&](const TileCursor& c, int xb) __attribute__((always_inline)) {
    const int last = c.rows() - 1;                        // last valid row of the tile
    const char* base = reinterpret_cast<const char*>(p.X) + c.row * (D * 2);
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int slot = k * NT + tid;                      // LDS slot = item * CH + position
      const int r = slot / CH;
      const int rel = r > last ? last : r;                // rows past the piece repeat its last row
      const uint32_t voff = uint32_t(rel) * (D * 2) + uint32_t((slot % CH) ^ (r & 15)) * 16;
      const uint32_t lds_base = uint32_t(reinterpret_cast<uintptr_t>(
          (void __attribute__((address_space(3)))*)(&xbuf[xb][k * NT + wave * 64])));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(lds_base), "v"(voff), "s"(base)
                   : "memory", "m0");
    }
  };
  auto wait_vm = [&](auto n_c) __attribute__((always_inline)) {
    constexpr int n = decltype(n_c)::value;
    __builtin_amdgcn_s_waitcnt((n & 0xF) | ((n >> 4) << 14) | 0x0F70);
  };
  static_assert(2 * CPT < 64, "vmcnt holds six bits");

  f32x16 z = {0};
  auto write_record = [&](int user) __attribute__((always_inline)) {
    float* rec = p.partials + ((g + user) * p.H + h) * 1024;
#pragma unroll
    for (int i = 0; i < 16; ++i) rec[(acc_row0(i) + 4 * hf) * 32 + l32] = z[i] * -0.69314718056f;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
  };

  // prologue: tiles 0, 1, 2 requested; tile 0 landed
  fetch(cf, 0);
  cf.advance(p.offsets, p.B, seg_end);
  fetch(cf, 1);
  cf.advance(p.offsets, p.B, seg_end);
  fetch(cf, 2);
  cf.advance(p.offsets, p.B, seg_end);
  wait_vm(Int<2 * CPT>{});
  lds_barrier();

  int xb = 0;
  bool drain = false;
  for (;;) {
    const bool last_in_piece = ca.tiles_left == 1;
    const int nvl = (last_in_piece ? ca.tail : kTile) - 4 * hf;   // register i is valid iff acc_row0(i) < nvl
    // K first, turned into the A operand right away, then V: one projection accumulator is
    // live at a time (at D = 256 the weights alone take half of the register file).
    Pack8 a0, a1, b0, b1;
    {
      f32x16 ak = {0};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Pack8 x;
        x.u = xbuf[xb][l32 * CH + ((2 * ks + hf) ^ (l32 & 15))];
        ak = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, wk[ks], ak, 0, 0, 0);
        if (kFence && ks % 4 == 3) __builtin_amdgcn_sched_barrier(0);   // keeps later operand reads from being hoisted and held
      }
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float fa = ak[i] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(ak[i]));
        const float fb = ak[i + 1] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(ak[i + 1]));
        const uint32_t pa = cvt_pk_bf16(fa, fb);
        if (i < 8) a0.w[i / 2] = pa; else a1.w[(i - 8) / 2] = pa;
      }
    }
    if (kFence) __builtin_amdgcn_sched_barrier(0);
    {
      f32x16 av = {0};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Pack8 x;
        x.u = xbuf[xb][l32 * CH + ((2 * ks + hf) ^ (l32 & 15))];
        av = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, wv[ks], av, 0, 0, 0);
        if (kFence && ks % 4 == 3) __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const uint32_t pb = cvt_pk_bf16(av[i], av[i + 1]);
        if (i < 8) b0.w[i / 2] = pb; else b1.w[(i - 8) / 2] = pb;
      }
    }
    if (last_in_piece) {
      // Rows past the piece's end count for nothing: their SiLU(k) is cleared.  One wave-uniform
      // branch per tile, taken once per piece, instead of a select per value on every tile.
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const uint32_t keep = (acc_row0(i) < nvl ? 0x0000FFFFu : 0u) | (acc_row0(i + 1) < nvl ? 0xFFFF0000u : 0u);
        if (i < 8) a0.w[i / 2] &= keep; else a1.w[(i - 8) / 2] &= keep;
      }
    }
    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b0.v, z, 0, 0, 0);
    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b1.v, z, 0, 0, 0);

    // tile t+1 has landed (this wave's part); everyone is done with tile t's rows
    if (drain) wait_vm(Int<0>{}); else wait_vm(Int<CPT>{});
    drain = false;
    lds_barrier();
    fetch(cf, xb);                                        // tile t+3 into the slot tile t has vacated
    cf.advance(p.offsets, p.B, seg_end);
    const int done_user = ca.user;
    ca.advance(p.offsets, p.B, seg_end);
    if (last_in_piece) {
      write_record(done_user);
      drain = true;                                       // loads and stores complete out of order with each other
    }
    xb = xb == kRing - 1 ? 0 : xb + 1;
    if (!ca.valid) break;
  }
  wait_vm(Int<0>{});                     // the requests that ran past the segment's end have landed:
  lds_barrier();                         // the ring is free for the next segment
  }
}

// ---------------------------------------------------------------------------------------
// Backward, item pass (App. B.1): for every item of a user and every head
//     dV = SiLU(k) dZs,      dK = (v dZs^T) * SiLU'(k),
// with dZs (d_h x d_h, per user and head) already formed.  Same streaming structure as the
// forward state kernel; here the projections are formed transposed, K^T = W_k,h^T X^T and
// V^T = W_v,h^T X^T (items on the lane index), so that SiLU(K)^T and V^T are B operands as they
// leave the accumulators and both products come out transposed again, one item per lane:
//     dV^T = dZs^T SiLU(K)^T,      dP^T = dZs V^T,      dK^T = dP^T * SiLU'(K)^T.
// The two A operands hold dZs with its contraction index in the accumulators' register order;
// they are reloaded when the stream passes from one user to the next.
template <int D>
__global__ __launch_bounds__(D * 2, 2) void qla_bwd_items_mfma_kernel(QlaParams p, const float* __restrict__ dz,
                                                                      uint16_t* __restrict__ dK,
                                                                      uint16_t* __restrict__ dV) {
  constexpr int NW = D / 32;
  constexpr int NT = NW * 64;
  constexpr int CH = D / 8;
  constexpr int KS = D / 16;
  constexpr int CPT = kTile * CH / NT;
  constexpr bool kFence = D > 128;       // as in the forward kernel
  __shared__ uint4 xbuf[kRing][CH * 32];
  constexpr int kStageRow = 80;                              // bytes between staged rows (64 used)
  __shared__ uint4 stage[NW][2 * 32 * kStageRow / 16];       // per wave: dV^T rows, then dK^T rows

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int hf = lane >> 5, l32 = lane & 31;
  const int h = __builtin_amdgcn_readfirstlane(tid >> 6);

  bf16x8 wk[KS], wv[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    Pack8 a, b;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int64_t at = int64_t(16 * ks + 8 * hf + j) * D + 32 * h + l32;
      a.h[j] = f32_to_bf16_bits(__uint_as_float(uint32_t(p.Wk[at]) << 16) * -kLog2e);   // t = -k log2(e)
      b.h[j] = p.Wv[at];
    }
    wk[ks] = a.v;
    wv[ks] = b.v;
    __builtin_amdgcn_sched_barrier(0);
  }

  const int wave = h;
  auto fetch = [&](const TileCursor& c, int xb) __attribute__((always_inline)) {
    const int last = c.rows() - 1;
    const char* base = reinterpret_cast<const char*>(p.X) + c.row * (D * 2);
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int slot = k * NT + tid;
      const int r = slot / CH;
      const int rel = r > last ? last : r;
      const uint32_t voff = uint32_t(rel) * (D * 2) + uint32_t((slot % CH) ^ (r & 15)) * 16;
      const uint32_t lds_base = uint32_t(reinterpret_cast<uintptr_t>(
          (void __attribute__((address_space(3)))*)(&xbuf[xb][k * NT + wave * 64])));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(lds_base), "v"(voff), "s"(base)
                   : "memory", "m0");
    }
  };
  auto wait_vm = [&](auto n_c) __attribute__((always_inline)) {
    constexpr int n = decltype(n_c)::value;
    __builtin_amdgcn_s_waitcnt((n & 0xF) | ((n >> 4) << 14) | 0x0F70);
  };

  // A operands of the two products for the current user: element j of part q pairs with
  // accumulator register 8 q + j, i.e. with contraction index acc_row0(8 q + j) + 4 hf.
  bf16x8 zt[2], zn[2];      // zt: dZs^T (rows c, contraction a);  zn: dZs (rows a, contraction c)
  auto load_dz = [&](int user) __attribute__((always_inline)) {
    const float* z = dz + (int64_t(user) * p.H + h) * 1024;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      Pack8 t, n;
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        const int r0 = acc_row0(8 * q + j) + 4 * hf, r1 = acc_row0(8 * q + j + 1) + 4 * hf;
        t.w[j / 2] = cvt_pk_bf16(z[r0 * 32 + l32], z[r1 * 32 + l32]);     // dZs^T[c = l32][a = r]
        n.w[j / 2] = cvt_pk_bf16(z[l32 * 32 + r0], z[l32 * 32 + r1]);     // dZs[a = l32][c = r]
      }
      zt[q] = t.v;
      zn[q] = n.v;
    }
  };

  for (int64_t g = blockIdx.x; g * p.seg < p.N; g += gridDim.x) {
    const int64_t seg_begin = g * p.seg;
    const int64_t seg_end = (seg_begin + p.seg < p.N) ? seg_begin + p.seg : p.N;
    TileCursor ca, cf;
    ca.init(p.offsets, p.B, p.seg_user ? __builtin_amdgcn_readfirstlane(p.seg_user[g]) : find_user(p.offsets, p.B, seg_begin),
            seg_begin, seg_end);
    if (!ca.valid) continue;
    cf = ca;
    load_dz(ca.user);

    fetch(cf, 0);
    cf.advance(p.offsets, p.B, seg_end);
    fetch(cf, 1);
    cf.advance(p.offsets, p.B, seg_end);
    fetch(cf, 2);
    cf.advance(p.offsets, p.B, seg_end);
    wait_vm(Int<2 * CPT>{});
    lds_barrier();

    int xb = 0;
    for (;;) {
      const int nvalid = ca.rows();
      Pack8 pk0, pk1, pv0, pv1;       // SiLU(K)^T and V^T as B operands (two halves of the 16 registers)
      float dsilu[16];                // SiLU'(k) of this lane's item, channels in register order
      {
        f32x16 ak = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          Pack8 x;
          x.u = xbuf[xb][l32 * CH + ((2 * ks + hf) ^ (l32 & 15))];
          ak = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wk[ks], x.v, ak, 0, 0, 0);
          if (kFence && ks % 4 == 3) __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          float f[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const float t = ak[i + u];                                  // -k log2(e)
            const float sg = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(t));
            const float k = t * -0.69314718056f;
            f[u] = k * sg;
            dsilu[i + u] = sg * fmaf(k, 1.f - sg, 1.f);
          }
          const uint32_t w = cvt_pk_bf16(f[0], f[1]);
          if (i < 8) pk0.w[i / 2] = w; else pk1.w[(i - 8) / 2] = w;
        }
      }
      if (kFence) __builtin_amdgcn_sched_barrier(0);
      {
        f32x16 av = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          Pack8 x;
          x.u = xbuf[xb][l32 * CH + ((2 * ks + hf) ^ (l32 & 15))];
          av = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[ks], x.v, av, 0, 0, 0);
          if (kFence && ks % 4 == 3) __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const uint32_t w = cvt_pk_bf16(av[i], av[i + 1]);
          if (i < 8) pv0.w[i / 2] = w; else pv1.w[(i - 8) / 2] = w;
        }
      }
      // Both projections have read the tile's rows.  Everything this wave has in flight -- the
      // stores of the previous tile, issued a projection ago, and the requests for the next two
      // tiles -- must be done before the barrier (loads and stores complete out of order with
      // each other, so the count alone cannot tell them apart); then the slot is refilled.
      wait_vm(Int<0>{});
      lds_barrier();
      fetch(cf, xb);
      cf.advance(p.offsets, p.B, seg_end);

      f32x16 gv = {0}, gp = {0};
      gv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zt[0], pk0.v, gv, 0, 0, 0);      // dV^T = dZs^T SiLU(K)^T
      gv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zt[1], pk1.v, gv, 0, 0, 0);
      gp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zn[0], pv0.v, gp, 0, 0, 0);      // dP^T = dZs V^T
      gp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zn[1], pv1.v, gp, 0, 0, 0);
      // lane = item l32 of the tile; register group of four = channels acc_row0(4 q) + 4 hf + 0..3.
      // The wave's two 32 x 32 result tiles pass through its own LDS patch (rows of 64 bytes,
      // 80 apart) so that four lanes store one item's 64 contiguous bytes.
      {
        char* st = reinterpret_cast<char*>(stage[h]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 ov, ok;
          ov.x = cvt_pk_bf16(gv[4 * q], gv[4 * q + 1]);
          ov.y = cvt_pk_bf16(gv[4 * q + 2], gv[4 * q + 3]);
          ok.x = cvt_pk_bf16(gp[4 * q] * dsilu[4 * q], gp[4 * q + 1] * dsilu[4 * q + 1]);
          ok.y = cvt_pk_bf16(gp[4 * q + 2] * dsilu[4 * q + 2], gp[4 * q + 3] * dsilu[4 * q + 3]);
          const int at = l32 * kStageRow + (acc_row0(4 * q) + 4 * hf) * 2;
          *reinterpret_cast<uint2*>(st + at) = ov;
          *reinterpret_cast<uint2*>(st + 32 * kStageRow + at) = ok;
        }
        // (the wave reads back only what it wrote: program order within the wave is enough)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int r = 16 * half + (lane >> 2), c = lane & 3;
          const uint4 ov = *reinterpret_cast<const uint4*>(st + r * kStageRow + 16 * c);
          const uint4 ok = *reinterpret_cast<const uint4*>(st + (32 + r) * kStageRow + 16 * c);
          if (r < nvalid) {
            const int64_t at = (ca.row + r) * D + 32 * h + 8 * c;
            *reinterpret_cast<uint4*>(dV + at) = ov;
            *reinterpret_cast<uint4*>(dK + at) = ok;
          }
        }
      }
      const int prev_user = ca.user;
      ca.advance(p.offsets, p.B, seg_end);
      xb = xb == kRing - 1 ? 0 : xb + 1;
      if (!ca.valid) break;
      if (ca.user != prev_user) load_dz(ca.user);
    }
    wait_vm(Int<0>{});
    lds_barrier();
  }
}

}  // namespace

bool mfma_qla_supported(const vista_summarize_desc& d) {
  return d.dtype == VISTA_BF16 && d.attn == VISTA_ATTN_QLA && ((d.d == 128 && d.H == 4) || (d.d == 256 && d.H == 8));
}

// Streams the history into the state records (slot = segment + user, row-major 32 x 32 fp32).
vista_status mfma_qla_state(const SummarizeArgs& a, float* partials) {
  const vista_summarize_desc& d = a.desc;
  QlaParams p;
  p.X = static_cast<const uint16_t*>(a.X);
  p.offsets = a.offsets;
  p.seg_user = a.seg_user;
  p.Wk = static_cast<const uint16_t*>(a.Wk);
  p.Wv = static_cast<const uint16_t*>(a.Wv);
  p.partials = partials;
  p.B = d.B;
  p.H = d.H;
  p.N = d.total_items;
  p.seg = a.seg;
  // three resident workgroups per compute unit at D = 128 (one at D = 256), each walking its share of the segments
  const int64_t resident = d.d == 128 ? 768 : 256;
  const unsigned blocks = unsigned(a.G < resident ? a.G : resident);
  if (d.d == 128)
    VISTA_LAUNCH(qla_state_mfma_kernel<128>, dim3(blocks), dim3(256), 0, a.stream, p);
  else
    VISTA_LAUNCH(qla_state_mfma_kernel<256>, dim3(blocks), dim3(512), 0, a.stream, p);
  return VISTA_OK;
}

vista_status mfma_qla_backward_items(const SummarizeArgs& a, const float* dz, void* d_keys, void* d_values) {
  const vista_summarize_desc& d = a.desc;
  QlaParams p;
  p.X = static_cast<const uint16_t*>(a.X);
  p.offsets = a.offsets;
  p.seg_user = a.seg_user;
  p.Wk = static_cast<const uint16_t*>(a.Wk);
  p.Wv = static_cast<const uint16_t*>(a.Wv);
  p.partials = nullptr;
  p.B = d.B;
  p.H = d.H;
  p.N = d.total_items;
  p.seg = a.seg;
  const int64_t resident = d.d == 128 ? 512 : 256;
  const unsigned blocks = unsigned(a.G < resident ? a.G : resident);
  if (d.d == 128)
    VISTA_LAUNCH(qla_bwd_items_mfma_kernel<128>, dim3(blocks), dim3(256), 0, a.stream, p, dz,
                 static_cast<uint16_t*>(d_keys), static_cast<uint16_t*>(d_values));
  else
    VISTA_LAUNCH(qla_bwd_items_mfma_kernel<256>, dim3(blocks), dim3(512), 0, a.stream, p, dz,
                 static_cast<uint16_t*>(d_keys), static_cast<uint16_t*>(d_values));
  return VISTA_OK;
}

}  // namespace vista
