// Stage 1 on the matrix cores (bf16 MFMA, fp32 accumulate), gfx950.
//
// One workgroup streams one flat segment of the packed history for HPW heads.
// Each head is served by a pair of waves.  Per tile of 32 items:
//   1. the X tile (32 x D bf16) goes from HBM straight into LDS (direct
//      global->LDS loads, three tiles deep, no stop in registers);
//   2. wave "K" of a pair forms K_h^T = (scale*log2e W_k,h)^T X^T, wave "V" forms
//      V_h = X W_v,h -- eight 32x32x16 MFMAs each for D = 128, weights held in registers
//      (as LDS operands at D = 256) -- and both hand the bf16 result to their partner through LDS;
//   3. each wave owns half of the S queries: for every block of 32 queries
//      S^T = K_h Q_h^T (items x queries), p = 2^(s - m), O^T += V_h^T P^T.
// With items on the MFMA row index and queries on the column index, every lane
// owns one query column: the softmax statistics are per-lane scalars, the
// fp32 score registers turn into the bf16 P operand without any shuffle, and
// the projected K^T / V accumulators already are the next MFMA's A operand.
// The projection of tile t+1 rides along with the attention over tile t, and
// the tiles of all pieces (user x segment) of the segment form one stream.
// Where a pair would leave a wave with more than four query blocks (S = 512) or
// with too few waves per compute unit (D = 256), a head gets four waves instead:
// the K and V waves plus two that only attend, a quarter of the queries each.
//
// Softmax reference.  Scores are kept in base-2 units.  While every score of a
// tile is provably inside [-60, 60] (Cauchy-Schwarz: |q| |k| <= 60) the
// reference maximum stays at the constant 0 and no per-score subtraction or
// maximum is needed; 2^s cannot overflow, underflow or lose relative precision
// there.  A tile that fails the test switches the piece to the usual running
// maximum with rescaling.  Both routes evaluate the same softmax exactly.
//
// Each piece ends with one partial record (O, l, m) per head; merge_mfma_kernel
// combines a user's records in ascending segment order.
#include "common.hpp"

namespace vista {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short i16x4;

constexpr int kTile = kTileItems;    // items per tile
constexpr float kSafeBound2 = 3600.f;  // (60)^2: |q|^2 |k|^2 below this keeps 2^s in range
constexpr int kRecRows = 18;         // 16 O registers + l + m per lane
constexpr int kRecFloats = kRecRows * 64;

struct MfmaSummarizeParams {
  const uint16_t* X;
  const int64_t* offsets;
  const int* seg_user;
  const uint16_t* Q;
  int64_t q_user_stride;
  const uint16_t* Wk;
  const uint16_t* Wv;
  float* partials;
  int B, S, H;
  int64_t N;
  int seg;
  int nhg;        // head groups = H / HPW
  float c;        // scale * log2(e)
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

__device__ __forceinline__ float dot2_self(uint32_t pk, float acc) {
  const bf16x2 v = __builtin_bit_cast(bf16x2, pk);
  return __builtin_amdgcn_fdot2_f32_bf16(v, v, acc, false);
}

// LDS-only workgroup barrier: global loads in flight (the X prefetch) stay in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Register i of a lane in half hf holds row 4 hf + acc_row0(i) of the 32x32 accumulator.
__device__ __forceinline__ constexpr int acc_row0(int i) { return 8 * (i / 4) + (i % 4); }

// One block of 32 queries against one tile of 32 items.  `general` and `masked`
// are wave-uniform; the MFMAs sit on the common path so the accumulators keep
// one register assignment whichever route a tile takes.
__device__ __forceinline__ void attend_block(const bf16x8& kop0, const bf16x8& kop1, const bf16x8& vop0,
                                             const bf16x8& vop1, const bf16x8& q0, const bf16x8& q1,
                                             f32x16& o, float& l, float& m, bool general, bool masked,
                                             int nvl) {
  // nvl = valid items of the tile minus 4 hf: register i is valid iff acc_row0(i) < nvl
  f32x16 s = {0};
  s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop0, q0, s, 0, 0, 0);
  s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop1, q1, s, 0, 0, 0);
  if (general) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (acc_row0(i) >= nvl) s[i] = -INFINITY;
    float tmax = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, s[i]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float mnew = fmaxf(m, tmax);
    const float alpha = __builtin_amdgcn_exp2f(m - mnew);
    l *= alpha;
#pragma unroll
    for (int i = 0; i < 16; ++i) o[i] *= alpha;
    m = mnew;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] -= mnew;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) s[i] = __builtin_amdgcn_exp2f(s[i]);
  if (masked) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if (acc_row0(i) >= nvl) s[i] = 0.f;
  }
  Pack8 p0, p1;
#pragma unroll
  for (int i = 0; i < 16; i += 2) {
    const uint32_t pk = cvt_pk_bf16(s[i], s[i + 1]);
    l = dot2_ones(pk, l);
    if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
  }
  o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop0, p0.v, o, 0, 0, 0);
  o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop1, p1.v, o, 0, 0, 0);
}

template <int V>
struct Int { static constexpr int value = V; };

constexpr int kXBuf = 3;             // ring depth of the X tiles and of the projected tiles in LDS

// Where a projecting wave keeps its 2 x (D x 32) weight operands: in registers at D = 128 (32 of
// them; it saves half of the operand reads of a projection), in LDS at D = 256 (64 would not fit).
__host__ __device__ constexpr bool weights_in_registers(int D) { return D == 128; }

// Shared memory of one workgroup.
template <int D, int HPW>
struct SummarizeLds {
  uint4 xbuf[kXBuf][(D / 8) * 32];    // X tiles: [16-byte chunk][item], filled by direct global->LDS loads
  uint4 kvbuf[kXBuf][HPW][2][2][64];  // projected tiles: [ring slot][head][K|V][half of the 16 registers][lane]
  float knorm[kXBuf][HPW][64];        // squared norm of the scaled key rows (half per lane)
  uint4 wop[weights_in_registers(D) ? 1 : HPW * 2 * (D / 16) * 64];   // projection weights as MFMA operands (D = 256): [head][K|V][k-slice][lane]
};

// Body of one wave; ROLE 0 forms K^T, ROLE 1 forms V, ROLE 2 forms nothing and only attends
// (the third and fourth wave of a head when its queries are spread over four waves: WPH = 4).  The tile loop is
// software-pipelined: while the wave attends over tile t (VALU-heavy) it also
// issues the projection MFMAs of tile t+1, and the X rows of tiles t+2 / t+3 are
// on their way from HBM (registers) into the LDS buffer tile t has vacated.  One
// LDS-only barrier per tile orders the two double-buffered exchanges.
// ATTN selects what is made of a score: VISTA_ATTN_SOFTMAX as described above, or
// VISTA_ATTN_SILU, the pointwise form SiLU(s) v of App. B: no reference maximum, no
// denominator, no norm test; the key weights then carry -scale*log2(e), so a score leaves the
// MFMA as t = -s log2(e) and SiLU(s) = -ln(2) t / (1 + 2^t); the weight handed to the second
// product is t / (1 + 2^t) and the constant joins the 1/L_b of the merge.
template <int D, int NQB, int HPW, int ROLE, int WPH = 2, int ATTN = VISTA_ATTN_SOFTMAX>
__device__ __forceinline__ void summarize_wave(const MfmaSummarizeParams& p, SummarizeLds<D, HPW>& sm,
                                               int64_t g, int h, int hl, int qslot, int64_t seg_begin,
                                               int64_t seg_end) {
  constexpr bool PROJ = ROLE < 2;        // this wave projects
  constexpr bool SILU = ATTN == VISTA_ATTN_SILU;
  constexpr int WR = PROJ ? ROLE : 0;    // its slot in the weight and K/V buffers (unused otherwise)
  constexpr int NT = HPW * WPH * 64;     // threads
  constexpr int CH = D / 8;              // 16-byte chunks per row
  constexpr int KS = D / 16;             // k-slices of the projection
  constexpr int CPT = kTile * CH / NT;   // X chunks a thread moves per tile
  static_assert(kTile * CH % NT == 0, "tile must split evenly over the workgroup");
  static_assert(KS % NQB == 0 || NQB % KS == 0, "projection slices are spread over the query blocks");
  constexpr int KPB = (KS + NQB - 1) / NQB;   // projection k-slices issued per query block

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int hf = lane >> 5;
  const int l32 = lane & 31;

  // Projection weights of this wave's head as MFMA operands, in registers or parked in LDS
  // (each wave reads back only what it wrote).  Element j of slice ks is
  // W[16 ks + 8 hf + j][32 h + l32]; the key weights carry scale*log2(e), so the
  // scores leave the MFMA in base-2 units.
  constexpr bool WREG = weights_in_registers(D);
  bf16x8 wreg[WREG ? KS : 1];
  if constexpr (PROJ) {
    const uint16_t* W = ROLE ? p.Wv : p.Wk;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Pack8 t;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint16_t w = W[(16 * ks + 8 * hf + j) * D + 32 * h + l32];
        t.h[j] = ROLE ? w : f32_to_bf16_bits(__uint_as_float(uint32_t(w) << 16) * p.c);
      }
      if constexpr (WREG) wreg[ks] = t.v; else sm.wop[((hl * 2 + WR) * KS + ks) * 64 + lane] = t.u;
    }
  }

  const int qbase = qslot * (NQB * 32);  // first query of this wave (qslot = ROLE when a head has two waves)
  bf16x8 qop[NQB][2];
  float qmax2 = 0.f;
  auto load_queries = [&](int user) __attribute__((always_inline)) {
    const char* Qb = reinterpret_cast<const char*>(p.Q + p.q_user_stride * user + int64_t(qbase) * D + 32 * h);
    const uint32_t qoff = uint32_t(l32) * (D * 2) + uint32_t(hf) * 8;
    float worst = 0.f;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const char* row = Qb + qb * 32 * D * 2;
      float n2 = 0.f;
#pragma unroll
      for (int part = 0; part < 2; ++part) {
        Pack8 t;
        // dh index of element j: 16 part + 4 hf + 8 (j / 4) + j % 4 -> two runs of four
        const uint2 a = *reinterpret_cast<const uint2*>(row + 32 * part + qoff);
        const uint2 b = *reinterpret_cast<const uint2*>(row + 32 * part + 16 + qoff);
        t.w[0] = a.x; t.w[1] = a.y; t.w[2] = b.x; t.w[3] = b.y;
        qop[qb][part] = t.v;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          float f = __uint_as_float(uint32_t(t.h[j]) << 16);
          n2 = fmaf(f, f, n2);
        }
      }
      n2 += __shfl_xor(n2, 32, 64);
      worst = fmaxf(worst, n2);
    }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) worst = fmaxf(worst, __shfl_xor(worst, off, 64));
    qmax2 = worst;
  };
  if (p.q_user_stride == 0) load_queries(0);

  // ---- the segment as one stream of tiles (TileCursor: scalar state, offsets read through
  // uniform loads).  `ca` names the tile being attended over, `cf` runs three tiles ahead
  // and names the tile whose rows are requested from HBM.
  using Cursor = TileCursor;
  auto cursor_init = [&](Cursor& c) __attribute__((always_inline)) {
    const int first = p.seg_user ? __builtin_amdgcn_readfirstlane(p.seg_user[g]) : find_user(p.offsets, p.B, seg_begin);
    c.init(p.offsets, p.B, first, seg_begin, seg_end);
  };
  auto cursor_advance = [&](Cursor& c) __attribute__((always_inline)) { c.advance(p.offsets, p.B, seg_end); };

  f32x16 o[NQB];
  float l[NQB], m[NQB];
  // plain tiles keep their share of the denominators in lacc (register qb of either accumulator);
  // the general route folds it into l first
  static_assert(NQB <= 4, "one accumulator register per query block");
  f32x4 lacc[2];
  uint2 onesrow[NQB];
#pragma unroll
  for (int r = 0; r < NQB; ++r) {
    const uint32_t w = (lane & 3) == r ? 0x3F803F80u : 0u;
    onesrow[r] = make_uint2(w, w);
  }
  int mode = 0;  // 0 fresh piece, 1 constant reference 0, 2 running maximum
  auto reset_state = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qb][i] = 0.f;
      l[qb] = 0.f;
      m[qb] = 0.f;
    }
    lacc[0] = lacc[1] = f32x4{0.f, 0.f, 0.f, 0.f};
    mode = 0;
  };

  // HBM -> LDS movement of X without a stop in registers (global_load_lds, 16 bytes
  // per lane: lane i of a wave lands at the wave's LDS base + 16 i).  Tile t lives in
  // xbuf[t % 3]; the rows of tile t+3 are requested at the top of tile t into the
  // buffer tile t has vacated and must have landed by the end of tile t+1, so a
  // load has two tile periods.  Rows past the piece are clamped to its last row.
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  auto fetch = [&](const Cursor& c, int xb) __attribute__((always_inline)) {
    const int last = (c.tiles_left == 1 ? c.tail : kTile) - 1;   // last valid row of the tile
    const char* base = reinterpret_cast<const char*>(p.X) + c.row * (D * 2);
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int slot = k * NT + tid;                         // LDS slot = chunk * 32 + item
      int rel = slot & 31;
      if (rel > last) rel = last;
      const uint32_t voff = uint32_t(rel) * (D * 2) + uint32_t(slot >> 5) * 16;
      // Written as assembly so that the completion wait is the explicit vmcnt wait at
      // the end of the next tile, not a conservative one before the next LDS read.
      const uint32_t lds_base = uint32_t(reinterpret_cast<uintptr_t>(
          (void __attribute__((address_space(3)))*)(&sm.xbuf[xb][k * NT + wave * 64])));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(lds_base), "v"(voff), "s"(base)
                   : "memory", "m0");
    }
  };
  // k-slices [ks0, ks1) of this wave's projection of the X tile in xbuf[buf]
  auto project = [&](int buf, int ks0, int ks1, f32x16& acc) __attribute__((always_inline)) {
    if constexpr (PROJ) {
#pragma unroll
      for (int ks = ks0; ks < ks1; ++ks) {
        Pack8 x, w;
        x.u = sm.xbuf[buf][(2 * ks + hf) * 32 + l32];
        if constexpr (WREG) w.v = wreg[ks]; else w.u = sm.wop[((hl * 2 + WR) * KS + ks) * 64 + lane];
        acc = ROLE ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, w.v, acc, 0, 0, 0)
                   : __builtin_amdgcn_mfma_f32_32x32x16_bf16(w.v, x.v, acc, 0, 0, 0);
      }
    }
  };
  // hand the projected tile to the partner wave: bf16 operand halves (+ key norms)
  auto publish = [&](int buf, const f32x16& acc) __attribute__((always_inline)) {
    if constexpr (PROJ) {
      Pack8 r0, r1;
      float n2 = 0.f;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const uint32_t pk = cvt_pk_bf16(acc[i], acc[i + 1]);
        if (ROLE == 0 && !SILU) n2 = dot2_self(pk, n2);
        if (i < 8) r0.w[i / 2] = pk; else r1.w[(i - 8) / 2] = pk;
      }
      sm.kvbuf[buf][hl][WR][0][lane] = r0.u;
      sm.kvbuf[buf][hl][WR][1][lane] = r1.u;
      if (ROLE == 0 && !SILU) sm.knorm[buf][hl][lane] = n2;
    }
  };
  auto unsafe_tile = [&](float kn2) __attribute__((always_inline)) {
    if constexpr (SILU) return false;
    return __builtin_amdgcn_ballot_w64(kn2 * qmax2 > kSafeBound2) != 0;
  };

  Cursor ca, cf;
  cursor_init(ca);
  cf = ca;

  // Common case: a full tile, bounded scores, another tile behind it.  Straight-line
  // code (one scheduling region per tile): two projection MFMAs of the next tile ride
  // along with every query block of this one.
  Pack8 k0, k1, v0, v1;     // K/V operands of the tile being attended over
  float kn2 = 0.f;          // its squared key norm (this lane's item)
  // Operands of tile t+1 (ring slot i1) come out of LDS while tile t is still being worked on,
  // into the registers tile t has just finished with: K (and the norms) once the last scores
  // of the tile are issued, V after its last P.V product.  They were published one tile ago
  // and the barrier at the start of tile t made them visible, so by the next barrier they
  // are in registers and the next tile starts without a round trip to LDS.
  auto read_k = [&](int i1) __attribute__((always_inline)) {
    k0.u = sm.kvbuf[i1][hl][0][0][lane];
    k1.u = sm.kvbuf[i1][hl][0][1][lane];
    if constexpr (!SILU) kn2 = sm.knorm[i1][hl][lane] + sm.knorm[i1][hl][lane ^ 32];
  };
  auto read_v = [&](int i1) __attribute__((always_inline)) {
    v0.u = sm.kvbuf[i1][hl][1][0][lane];
    v1.u = sm.kvbuf[i1][hl][1][1][lane];
  };
  auto fast_tile = [&](int r) __attribute__((always_inline)) {   // r = tile index mod 3
    const int i1 = r == kXBuf - 1 ? 0 : r + 1;
    const int i2 = i1 == kXBuf - 1 ? 0 : i1 + 1;
    f32x16 acc = {0};
    // scores run one query block ahead of the exponentials that consume them
    f32x16 nx = {0};
    nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0.v, qop[0][0], nx, 0, 0, 0);
    nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1.v, qop[0][1], nx, 0, 0, 0);
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      if (qb == NQB - 1) read_k(i1);     // the last scores of this tile are already issued
      const f32x16 sc = nx;
      if (qb + 1 < NQB) {
        const f32x16 z = {0};
        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0.v, qop[qb + 1][0], z, 0, 0, 0);
        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1.v, qop[qb + 1][1], nx, 0, 0, 0);
      }
      if (qb * KPB < KS) project(i2, qb * KPB, qb * KPB + KPB, acc);
      Pack8 p0, p1;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        float ea = __builtin_amdgcn_exp2f(sc[i]), eb = __builtin_amdgcn_exp2f(sc[i + 1]);
        if constexpr (SILU) {
          ea = sc[i] * __builtin_amdgcn_rcpf(1.f + ea);
          eb = sc[i + 1] * __builtin_amdgcn_rcpf(1.f + eb);
        }
        const uint32_t pk = cvt_pk_bf16(ea, eb);
        if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
      }
      // The denominator on the matrix core: a 4x4x4 product (16 blocks, one per four lanes)
      // whose A block has ones in row qb adds a lane's own four packed weights into register
      // qb of that lane -- the lane-local partial sum a chain of adds would form, taken over
      // the bf16 weights the numerator uses.  It issues like one plain vector instruction
      // for four weights; two accumulators take turns so that consecutive products do not
      // wait for each other.
      if constexpr (!SILU) {
        const i16x4 sel = __builtin_bit_cast(i16x4, onesrow[qb]);
#pragma unroll
        for (int part = 0; part < 4; ++part) {
          const uint2 pw = part < 2 ? make_uint2(p0.w[2 * part], p0.w[2 * part + 1])
                                    : make_uint2(p1.w[2 * part - 4], p1.w[2 * part - 3]);
          lacc[part & 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(sel, __builtin_bit_cast(i16x4, pw), lacc[part & 1], 0, 0, 0);
        }
      }
      o[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0.v, p0.v, o[qb], 0, 0, 0);
      o[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1.v, p1.v, o[qb], 0, 0, 0);
    }
    read_v(i1);
    publish(i2, acc);
  };

  // Any tile: ragged tail, scores beyond the bound, last tile of the segment.
  auto slow_tile = [&](int r, int nvalid, bool unsafe) __attribute__((always_inline)) {
    const int i1 = r == kXBuf - 1 ? 0 : r + 1;
    const int i2 = i1 == kXBuf - 1 ? 0 : i1 + 1;
    const int nvl = nvalid - 4 * hf;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      l[qb] += lacc[0][qb] + lacc[1][qb];
      lacc[0][qb] = lacc[1][qb] = 0.f;
    }
    if constexpr (SILU) {
      // pointwise form: scores, weights (rows past the piece's end get weight 0), second product
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        f32x16 sc = {0};
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0.v, qop[qb][0], sc, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1.v, qop[qb][1], sc, 0, 0, 0);
        Pack8 p0, p1;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          float wa = sc[i] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(sc[i]));
          float wb = sc[i + 1] * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(sc[i + 1]));
          if (acc_row0(i) >= nvl) wa = 0.f;
          if (acc_row0(i + 1) >= nvl) wb = 0.f;
          const uint32_t pk = cvt_pk_bf16(wa, wb);
          if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
        }
        o[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0.v, p0.v, o[qb], 0, 0, 0);
        o[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1.v, p1.v, o[qb], 0, 0, 0);
      }
      mode = 1;
    } else {
    const bool general = mode == 2 || unsafe;
    if (mode != 2) {   // the reference so far: nothing (fresh piece) or the constant 0
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) m[qb] = (general && mode == 0) ? -INFINITY : 0.f;
    }
    mode = general ? 2 : 1;
    const bool masked = nvalid < kTile;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
      attend_block(k0.v, k1.v, v0.v, v1.v, qop[qb][0], qop[qb][1], o[qb], l[qb], m[qb], general, masked, nvl);
    }
    read_k(i1);
    read_v(i1);
    // the tile two ahead (past the end of the segment: a repeat of its last tile, never used)
    f32x16 acc = {0};
    project(i2, 0, KS, acc);
    publish(i2, acc);
  };

  // partial record of a finished piece: slot = segment + user
  auto write_partial = [&](int user) __attribute__((always_inline)) {
    const int64_t slot = g + user;
    char* rec = reinterpret_cast<char*>(p.partials +
                                        ((slot * p.H + h) * (p.S / 32) + (qbase / 32)) * kRecFloats);
    const uint32_t lane_off = uint32_t(lane) * 4;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      char* r = rec + size_t(qb) * kRecFloats * 4;       // scalar
#pragma unroll
      for (int i = 0; i < 16; ++i) *reinterpret_cast<float*>(r + i * 256 + lane_off) = o[qb][i];
      *reinterpret_cast<float*>(r + 16 * 256 + lane_off) = l[qb] + __shfl_xor(l[qb], 32, 64);
      *reinterpret_cast<float*>(r + 17 * 256 + lane_off) = (mode == 2) ? m[qb] : 0.f;
    }
  };

  if (!ca.valid) return;               // only with invalid offsets (whole workgroup)
  reset_state();
  if (p.q_user_stride != 0) load_queries(ca.user);

  // Waits until at most `pending` of this wave's newest vector-memory operations
  // are outstanding (s_waitcnt vmcnt only; the other counters are left alone).
  auto wait_vm = [&](auto n_c) __attribute__((always_inline)) {
    constexpr int n = decltype(n_c)::value;
    __builtin_amdgcn_s_waitcnt((n & 0xF) | ((n >> 4) << 14) | 0x0F70);
  };

  // Tile t lives in ring slot t mod 3, as raw rows (xbuf) and, projected, as operands
  // (kvbuf).  While tile t is attended over, tile t+2 is projected and published, the
  // operands of tile t+1 move into registers, the rows of tile t+3 land and those of tile
  // t+4 are requested into the slot whose rows (tile t+1) were projected one tile ago.
  // ---- prologue: tiles 0, 1, 2 requested; 0 and 1 landed, projected and published
  fetch(cf, 0);
  cursor_advance(cf);
  fetch(cf, 1);
  cursor_advance(cf);
  fetch(cf, 2);
  cursor_advance(cf);
  wait_vm(Int<CPT>{});
  lds_barrier();
  {
    f32x16 acc = {0};
    project(0, 0, KS, acc);
    publish(0, acc);
    f32x16 acc1 = {0};
    project(1, 0, KS, acc1);
    publish(1, acc1);
  }
  lds_barrier();              // slot 0's rows are projected by everyone, its operands are visible
  fetch(cf, 0);               // tile 3
  cursor_advance(cf);
  read_k(0);
  read_v(0);
  wait_vm(Int<CPT>{});        // tile 2 has landed

  // One barrier per tile on either route (waves may take different routes: the bound
  // depends on each wave's queries).  Runs of plain tiles (full, bounded scores, not
  // the last of their piece) stay in the inner loop, whose body is straight-line
  // code with the accumulators updated in place; every other tile leaves it, takes
  // the general route and does the piece bookkeeping.
  int r = 0;              // ring slot of the tile being attended over
  bool drain = false;     // other vector-memory traffic (record stores, query loads) is in flight
  // Tile t+3 (requested one tile ago) must have landed before the next barrier; the
  // request just issued for tile t+4 may stay in flight.  Loads complete in order
  // among themselves but not with respect to stores, so after a record write
  // everything is drained once.
  auto end_of_tile = [&]() __attribute__((always_inline)) {
    if (drain) wait_vm(Int<0>{}); else wait_vm(Int<CPT>{});
    drain = false;
    cursor_advance(cf);
  };
  // Start of a tile: the barrier, then the request for tile t+4.
  auto begin_tile = [&]() __attribute__((always_inline)) {
    lds_barrier();
    fetch(cf, r == kXBuf - 1 ? 0 : r + 1);
  };
  // whether the tile whose operands are in registers is a plain one
  bool unsafe = unsafe_tile(kn2);
  auto is_plain = [&]() __attribute__((always_inline)) {
    if constexpr (SILU) return ca.tiles_left != 1;
    return !(ca.tiles_left == 1 || mode == 2 || unsafe);
  };
  bool plain = is_plain();
  for (;;) {
    while (__builtin_expect(plain, 1)) {
      begin_tile();
      mode = 1;
      fast_tile(r);
      end_of_tile();
      --ca.tiles_left;
      ca.row += kTile;
      r = r == kXBuf - 1 ? 0 : r + 1;
      unsafe = unsafe_tile(kn2);
      plain = is_plain();
    }
    begin_tile();
    const bool last_in_piece = ca.tiles_left == 1;
    const int nvalid = last_in_piece ? ca.tail : kTile;
    slow_tile(r, nvalid, unsafe);
    end_of_tile();
    const int done_user = ca.user;
    cursor_advance(ca);
    if (last_in_piece) {
      write_partial(done_user);
      reset_state();
      if (p.q_user_stride != 0 && ca.valid) load_queries(ca.user);
      drain = true;
    }
    r = r == kXBuf - 1 ? 0 : r + 1;
    if (!ca.valid) break;
    unsafe = unsafe_tile(kn2);
    plain = is_plain();
  }
}

template <int D, int NQB, int HPW, int ATTN>
__global__ __launch_bounds__(HPW * 128) void summarize_mfma_kernel(MfmaSummarizeParams p) {
  __shared__ SummarizeLds<D, HPW> sm;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept scalar
  const int hl = wave >> 1;

  // XCD-aware block -> (segment, head group): the head groups of one segment
  // share an XCD (and its L2) because their block ids differ by multiples of 8.
  const int64_t id = blockIdx.x;
  const int64_t grp = id / (8 * p.nhg);
  const int idl = int(id - grp * 8 * p.nhg);
  const int64_t g = grp * 8 + (idl & 7);
  const int hg = idl >> 3;
  const int h = hg * HPW + hl;
  const int64_t seg_begin = g * p.seg;
  if (seg_begin >= p.N) return;          // padding blocks of the last group (whole workgroup)
  const int64_t seg_end = (seg_begin + p.seg < p.N) ? seg_begin + p.seg : p.N;
  // Both roles run the same sequence of barriers; only the MFMA operand order differs.
  if (wave & 1)
    summarize_wave<D, NQB, HPW, 1, 2, ATTN>(p, sm, g, h, hl, 1, seg_begin, seg_end);
  else
    summarize_wave<D, NQB, HPW, 0, 2, ATTN>(p, sm, g, h, hl, 0, seg_begin, seg_end);
}

// Four waves per head (two heads per workgroup): the K and V waves project as above, two more
// waves only attend, each of the four with a quarter of the queries.  With S = 512 this keeps a
// wave at 4 query blocks, i.e. inside 256 vector registers and at two waves per SIMD.  Wave
// w serves head w / 4 in slot (w + 2 (w / 4)) % 4, so that each SIMD (wave id mod 4) gets one
// projecting and one attend-only wave.
template <int D, int NQB, int ATTN>
__global__ __launch_bounds__(512) void summarize_mfma4_kernel(MfmaSummarizeParams p) {
  constexpr int HPW = 2;
  __shared__ SummarizeLds<D, HPW> sm;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int hl = wave >> 2;
  const int slot = (wave + 2 * hl) & 3;
  const int64_t id = blockIdx.x;
  const int64_t grp = id / (8 * p.nhg);
  const int idl = int(id - grp * 8 * p.nhg);
  const int64_t g = grp * 8 + (idl & 7);
  const int hg = idl >> 3;
  const int h = hg * HPW + hl;
  const int64_t seg_begin = g * p.seg;
  if (seg_begin >= p.N) return;          // padding blocks of the last group (whole workgroup)
  const int64_t seg_end = (seg_begin + p.seg < p.N) ? seg_begin + p.seg : p.N;
  if (slot == 0)
    summarize_wave<D, NQB, HPW, 0, 4, ATTN>(p, sm, g, h, hl, 0, seg_begin, seg_end);
  else if (slot == 1)
    summarize_wave<D, NQB, HPW, 1, 4, ATTN>(p, sm, g, h, hl, 1, seg_begin, seg_end);
  else
    summarize_wave<D, NQB, HPW, 2, 4, ATTN>(p, sm, g, h, hl, slot, seg_begin, seg_end);
}

// Merge of a user's partial records, ascending segment order (fixed, so the
// result is bitwise reproducible).  Softmax form: with m the running maximum of the m_c,
// out = sum_c 2^(m_c - m) O_c / sum_c 2^(m_c - m) l_c; the self term (Ks != null) is one more
// record (m = own score, l = 1, O = own value), taken last.  SiLU form: out =
// (-ln 2 sum_c O_c + SiLU(own score) own value) / L_b (the records hold sums of
// t / (1 + 2^t) v with t = -s log2 e).  One block per (user, head, query block), 256 threads:
// wave w owns accumulator registers 4w..4w+3, i.e. channels 8w + 4 hf + 0..3.
template <bool SILU>
__global__ __launch_bounds__(256) void merge_mfma_kernel(const float* __restrict__ partials,
                                                         const int64_t* __restrict__ offsets, int S, int d,
                                                         int H, int seg, int64_t G,
                                                         uint16_t* __restrict__ out, int* status,
                                                         const uint16_t* __restrict__ Q, int64_t q_user_stride,
                                                         const float* __restrict__ Ks,
                                                         const float* __restrict__ Vs, float scale,
                                                         float* __restrict__ out_scales) {
  __shared__ float amax_part[8][32];
  const int nqb = S / 32;
  const int qb = blockIdx.x % nqb, h = (blockIdx.x / nqb) % H, b = blockIdx.x / (nqb * H);
  // without a plan kernel in front (offsets checked on the host) the status word is cleared here
  if (status && qb == 0 && h == 0 && b == 0 && threadIdx.x == 0) *status = VISTA_OK;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int hf = lane >> 5, l32 = lane & 31;
  const int64_t begin = offsets[b], end = offsets[b + 1];
  uint16_t* dst = out + (int64_t(b) * S + qb * 32 + l32) * d + 32 * h + 8 * w + 4 * hf;
  // cache codec (out_scales != null): `out` holds int8 codes, one scale per (token, head)
  int8_t* dst8 = reinterpret_cast<int8_t*>(out) + (int64_t(b) * S + qb * 32 + l32) * d + 32 * h + 8 * w + 4 * hf;
  if (end <= begin) {
    if (out_scales) {
      *reinterpret_cast<uint32_t*>(dst8) = 0u;
      if (w == 0 && hf == 0) out_scales[(int64_t(b) * S + qb * 32 + l32) * H + h] = 0.f;
    } else {
      *reinterpret_cast<uint2*>(dst) = make_uint2(0u, 0u);
    }
    return;
  }
  int64_t g0 = begin / seg, g1 = (end - 1) / seg;
  if (g0 < 0) g0 = 0;
  if (g1 > G - 1) g1 = G - 1;
  // the query's own key and value (self term): score in the units of the records' m
  float s_self = 0.f, vs[4] = {0.f, 0.f, 0.f, 0.f};
  if (Ks) {
    const int i = qb * 32 + l32;
    const uint16_t* q = Q + q_user_stride * b + int64_t(i) * d + 32 * h;
    const int64_t srow = (q_user_stride ? int64_t(b) * S : 0) + i;
    const float* ks = Ks + srow * d + 32 * h;
#pragma unroll 8
    for (int c = 0; c < 32; ++c) s_self = fmaf(__uint_as_float(uint32_t(q[c]) << 16), ks[c], s_self);
    s_self *= scale;
#pragma unroll
    for (int r = 0; r < 4; ++r) vs[r] = Vs[srow * d + 32 * h + 8 * w + 4 * hf + r];
  }
  auto rec = [&](int64_t g) __attribute__((always_inline)) { return partials + (((g + b) * H + h) * nqb + qb) * kRecFloats + lane; };
  // One pass with a running maximum (rescale when it moves); loads are issued kBatch
  // records at a time so a long user is not a chain of dependent round trips.
  constexpr int kBatch = 8;
  float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
  for (int64_t g = g0; g <= g1; g += kBatch) {
    float v[kBatch][6];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const bool on = g + u <= g1;
      const float* r = rec(on ? g + u : g1);
      v[u][0] = on ? r[17 * 64] : -INFINITY;
      v[u][1] = r[16 * 64];
      v[u][2] = r[(4 * w + 0) * 64];
      v[u][3] = r[(4 * w + 1) * 64];
      v[u][4] = r[(4 * w + 2) * 64];
      v[u][5] = r[(4 * w + 3) * 64];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {     // ascending segment order
      if (SILU) {
        const float on = g + u <= g1 ? 1.f : 0.f;
        o0 = fmaf(v[u][2], on, o0);
        o1 = fmaf(v[u][3], on, o1);
        o2 = fmaf(v[u][4], on, o2);
        o3 = fmaf(v[u][5], on, o3);
        continue;
      }
      const float mn = fmaxf(m, v[u][0]);
      const float keep = exp2f(m - mn);       // 0 on the first record (m = -inf), 1 while the maximum stands
      const float wgt = exp2f(v[u][0] - mn);  // 0 for the padding entries
      l = fmaf(v[u][1], wgt, l * keep);
      o0 = fmaf(v[u][2], wgt, o0 * keep);
      o1 = fmaf(v[u][3], wgt, o1 * keep);
      o2 = fmaf(v[u][4], wgt, o2 * keep);
      o3 = fmaf(v[u][5], wgt, o3 * keep);
      m = mn;
    }
  }
  float inv;
  if (SILU) {
    inv = 1.f / float(end - begin);
    const float wself = Ks ? s_self / (1.f + expf(-s_self)) : 0.f;
    o0 = fmaf(o0, -0.69314718056f, wself * vs[0]);
    o1 = fmaf(o1, -0.69314718056f, wself * vs[1]);
    o2 = fmaf(o2, -0.69314718056f, wself * vs[2]);
    o3 = fmaf(o3, -0.69314718056f, wself * vs[3]);
  } else {
    if (Ks) {
      const float mn = fmaxf(m, s_self);
      const float keep = exp2f(m - mn), wgt = exp2f(s_self - mn);
      l = fmaf(l, keep, wgt);
      o0 = fmaf(vs[0], wgt, o0 * keep);
      o1 = fmaf(vs[1], wgt, o1 * keep);
      o2 = fmaf(vs[2], wgt, o2 * keep);
      o3 = fmaf(vs[3], wgt, o3 * keep);
    }
    inv = 1.f / l;
  }
  if (out_scales) {
    // Sec. 3.1's quantisation, fused: the head's 32 channels of a token sit in this block's
    // eight (wave, half) groups of four; their largest magnitude goes through LDS.
    const float y0 = o0 * inv, y1 = o1 * inv, y2 = o2 * inv, y3 = o3 * inv;
    amax_part[2 * w + hf][l32] = fmaxf(fmaxf(fabsf(y0), fabsf(y1)), fmaxf(fabsf(y2), fabsf(y3)));
    __syncthreads();
    float amax = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) amax = fmaxf(amax, amax_part[k][l32]);
    const float q = amax > 0.f ? 127.f / amax : 0.f;
    auto code = [&](float y) __attribute__((always_inline)) {
      return uint32_t(int(fminf(fmaxf(rintf(y * q), -127.f), 127.f))) & 0xFFu;
    };
    *reinterpret_cast<uint32_t*>(dst8) = code(y0) | (code(y1) << 8) | (code(y2) << 16) | (code(y3) << 24);
    if (w == 0 && hf == 0) out_scales[(int64_t(b) * S + qb * 32 + l32) * H + h] = amax > 0.f ? amax / 127.f : 0.f;
    return;
  }
  uint2 pk;
  pk.x = uint32_t(f32_to_bf16_bits(o0 * inv)) | (uint32_t(f32_to_bf16_bits(o1 * inv)) << 16);
  pk.y = uint32_t(f32_to_bf16_bits(o2 * inv)) | (uint32_t(f32_to_bf16_bits(o3 * inv)) << 16);
  *reinterpret_cast<uint2*>(dst) = pk;
}

// ------------------------------------------------------------------ host side

static bool shape_d128(const vista_summarize_desc& d) { return d.d == 128 && d.H == 4; }
static bool shape_d256(const vista_summarize_desc& d) { return d.d == 256 && d.H == 8; }

bool mfma_summarize_supported(const vista_summarize_desc& d) {
  if (d.dtype != VISTA_BF16 || d.attn == VISTA_ATTN_QLA) return false;
  if (!(shape_d128(d) || shape_d256(d))) return false;
  return d.S == 64 || d.S == 128 || d.S == 256 || d.S == 512;
}

static size_t partial_bytes(const vista_summarize_desc& d, int seg) {
  int64_t G = (d.total_items + seg - 1) / seg;
  return size_t(G + d.B) * d.H * (d.S / 32) * kRecFloats * sizeof(float);
}

// [header][seg_user][partial records][K' of the seeds][V' of the seeds]
size_t mfma_summarize_workspace(const vista_summarize_desc& d, int seg) {
  const int64_t G = (d.total_items + seg - 1) / seg;
  return kHeaderBytes + plan_bytes(G) + ((partial_bytes(d, seg) + 255) & ~size_t(255)) + 2 * self_kv_bytes(d);
}

template <int D, int NQB, int ATTN>
static hipError_t launch_main4(const MfmaSummarizeParams& p, int64_t G, hipStream_t s) {
  const int64_t groups = (G + 7) / 8;
  const int64_t blocks = groups * 8 * p.nhg;
  return launch(summarize_mfma4_kernel<D, NQB, ATTN>, dim3(unsigned(blocks)), dim3(512), 0, s, p);
}

template <int D, int NQB, int HPW, int ATTN>
static hipError_t launch_main(const MfmaSummarizeParams& p, int64_t G, hipStream_t s) {
  const int64_t groups = (G + 7) / 8;
  const int64_t blocks = groups * 8 * p.nhg;
  return launch(summarize_mfma_kernel<D, NQB, HPW, ATTN>, dim3(unsigned(blocks)), dim3(HPW * 128), 0, s, p);
}

template <int ATTN>
static hipError_t launch_for_shape(MfmaSummarizeParams& p, const vista_summarize_desc& d, int64_t G,
                                   hipStream_t s) {
  if (shape_d128(d)) {
    p.nhg = 1;
    switch (d.S) {
      case 64: return launch_main<128, 1, 4, ATTN>(p, G, s);
      case 128: return launch_main<128, 2, 4, ATTN>(p, G, s);
      case 256: return launch_main<128, 4, 4, ATTN>(p, G, s);
      default: p.nhg = 2; return launch_main4<128, 4, ATTN>(p, G, s);
    }
  }
  p.nhg = 4;
  switch (d.S) {
    case 64: return launch_main<256, 1, 2, ATTN>(p, G, s);
    case 128: return launch_main4<256, 1, ATTN>(p, G, s);
    case 256: return launch_main4<256, 2, ATTN>(p, G, s);
    default: return launch_main4<256, 4, ATTN>(p, G, s);
  }
}

vista_status mfma_summarize(const SummarizeArgs& a) {
  const vista_summarize_desc& d = a.desc;
  const bool silu = d.attn == VISTA_ATTN_SILU;
  MfmaSummarizeParams p;
  p.X = static_cast<const uint16_t*>(a.X);
  p.offsets = a.offsets;
  p.Q = static_cast<const uint16_t*>(a.Q);
  p.q_user_stride = d.q_user_stride;
  p.Wk = static_cast<const uint16_t*>(a.Wk);
  p.Wv = static_cast<const uint16_t*>(a.Wv);
  p.partials = reinterpret_cast<float*>(a.workspace + kHeaderBytes + plan_bytes(a.G));
  p.seg_user = a.seg_user;

  p.B = d.B;
  p.S = d.S;
  p.H = d.H;
  p.N = d.total_items;
  p.seg = a.seg;
  p.c = silu ? -a.scale_log2 : a.scale_log2;
  float* Ks = nullptr;
  float* Vs = nullptr;
  if (d.flags & VISTA_FLAG_SELF_TERM) {
    Ks = reinterpret_cast<float*>(reinterpret_cast<char*>(p.partials) + ((partial_bytes(d, a.seg) + 255) & ~size_t(255)));
    Vs = Ks + self_kv_bytes(d) / sizeof(float);
    if (launch_self_kv(d, a.Q, a.Wk, a.Wv, Ks, Vs, a.stream) != hipSuccess) return VISTA_ERR_HIP;
  }
  const int64_t merge_blocks = int64_t(d.B) * d.H * (d.S / 32);
  if ((a.G + 7) / 8 * 8 * 4 > 0x7FFFFFFF || merge_blocks > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  if (a.G > 0) {
    const hipError_t e = silu ? launch_for_shape<VISTA_ATTN_SILU>(p, d, a.G, a.stream)
                              : launch_for_shape<VISTA_ATTN_SOFTMAX>(p, d, a.G, a.stream);
    if (e != hipSuccess) return VISTA_ERR_HIP;
  }
  int* status = a.seg_user ? nullptr : reinterpret_cast<int*>(a.workspace);
  if (silu)
    VISTA_LAUNCH(merge_mfma_kernel<true>, dim3(unsigned(merge_blocks)), dim3(256), 0, a.stream, p.partials, a.offsets,
                 d.S, d.d, d.H, a.seg, a.G, static_cast<uint16_t*>(a.out), status, p.Q, d.q_user_stride, Ks, Vs,
                 a.scale_plain, a.out_scales);
  else
    VISTA_LAUNCH(merge_mfma_kernel<false>, dim3(unsigned(merge_blocks)), dim3(256), 0, a.stream, p.partials, a.offsets,
                 d.S, d.d, d.H, a.seg, a.G, static_cast<uint16_t*>(a.out), status, p.Q, d.q_user_stride, Ks, Vs,
                 a.scale_log2, a.out_scales);
  return VISTA_OK;
}

}  // namespace vista
