// Stage 1 on the matrix cores (bf16 MFMA, fp32 accumulate), gfx950.
//
// One workgroup streams one flat segment of the packed history for HPW heads.
// Each head is served by a pair of waves.  Per tile of 32 items:
//   1. the workgroup copies the X tile (32 x D bf16) from HBM into LDS once;
//   2. wave "K" of a pair forms K_h^T = W_k,h^T X^T (scaled by scale*log2 e),
//      wave "V" forms V_h = X W_v,h -- eight 32x32x16 MFMAs each for D = 128 --
//      and both hand the bf16 result to their partner through LDS;
//   3. each wave owns half of the S queries: for every block of 32 queries
//      S^T = K_h Q_h^T (items x queries), p = 2^(s - m), O^T += V_h^T P^T.
// With items on the MFMA row index and queries on the column index, every lane
// owns one query column: the softmax statistics are per-lane scalars, the
// fp32 score registers turn into the bf16 P operand without any shuffle, and
// the projected K^T / V accumulators already are the next MFMA's A operand.
//
// Softmax reference.  Scores are kept in base-2 units.  While every score of a
// tile is provably inside [-60, 60] (Cauchy-Schwarz: |q| |k| <= 60) the
// reference maximum stays at the constant 0 and no per-score subtraction or
// maximum is needed; 2^s cannot overflow, underflow or lose relative precision
// there.  A tile that fails the test switches the piece to the usual running
// maximum with rescaling.  Both routes evaluate the same softmax exactly.
//
// Each piece (segment x user) ends with one partial record (O, l, m) per head;
// merge_mfma_kernel combines a user's records in ascending segment order.
#include "common.hpp"

namespace vista {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kTile = 32;            // items per tile
constexpr float kSafeBound2 = 3600.f;  // (60)^2: |q|^2 |k|^2 below this keeps 2^s in range
constexpr int kRecRows = 18;         // 16 O registers + l + m per lane
constexpr int kRecFloats = kRecRows * 64;

struct MfmaSummarizeParams {
  const uint16_t* X;
  const int64_t* offsets;
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

// Shared memory of one workgroup.
template <int D, int HPW>
struct SummarizeLds {
  uint4 xbuf[2][(D / 8) * 33];        // X tile: [16-byte chunk][item + pad]
  uint4 kvbuf[2][HPW][2][2][64];      // [buffer][head][K|V][half of the 16 registers][lane]
  float knorm[2][HPW][64];            // squared norm of the scaled key rows (half per lane)
};

// Body of one wave; ROLE 0 forms K^T, ROLE 1 forms V.  The tile loop is
// software-pipelined: while the wave attends over tile t (VALU-heavy) it also
// issues the projection MFMAs of tile t+1, and the X rows of tiles t+2 / t+3
// are on their way from HBM (registers) into the other LDS buffer.  One
// LDS-only barrier per tile orders the two double-buffered exchanges.
template <int D, int NQB, int HPW, int ROLE>
__device__ __forceinline__ void summarize_wave(const MfmaSummarizeParams& p, SummarizeLds<D, HPW>& sm,
                                               int64_t g, int h, int hl, int64_t seg_begin, int64_t seg_end) {
  constexpr int NT = HPW * 128;          // threads
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

  // Projection weights of this wave's head, resident as MFMA operands:
  // element j of slice ks is W[16 ks + 8 hf + j][32 h + l32].
  bf16x8 wreg[KS];
  {
    const uint16_t* W = ROLE ? p.Wv : p.Wk;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      Pack8 t;
#pragma unroll
      for (int j = 0; j < 8; ++j) t.h[j] = W[(16 * ks + 8 * hf + j) * D + 32 * h + l32];
      wreg[ks] = t.v;
    }
  }

  const int qbase = ROLE * (NQB * 32);   // first query of this wave
  bf16x8 qop[NQB][2];
  float qmax2 = 0.f;
  auto load_queries = [&](int user) {
    const uint16_t* Qb = p.Q + p.q_user_stride * user;
    float worst = 0.f;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const uint16_t* row = Qb + int64_t(qbase + qb * 32 + l32) * D + 32 * h;
      float n2 = 0.f;
#pragma unroll
      for (int part = 0; part < 2; ++part) {
        Pack8 t;
        // dh index of element j: 16 part + 4 hf + 8 (j / 4) + j % 4 -> two runs of four
        const uint2 a = *reinterpret_cast<const uint2*>(row + 16 * part + 4 * hf);
        const uint2 b = *reinterpret_cast<const uint2*>(row + 16 * part + 4 * hf + 8);
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

  int user = find_user(p.offsets, p.B, seg_begin);
  int64_t pos = seg_begin;
  Piece pc;
  while (next_piece(p.offsets, p.B, seg_end, user, pos, pc)) {
    if (p.q_user_stride != 0) load_queries(pc.user);
    const int ntiles = int((pc.end - pc.begin + kTile - 1) / kTile);

    f32x16 o[NQB];
    float l[NQB], m[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qb][i] = 0.f;
      l[qb] = 0.f;
      m[qb] = 0.f;
    }
    int mode = 0;  // 0 fresh, 1 constant reference 0, 2 running maximum

    // HBM -> registers -> LDS movement of X; two register sets alternate so a
    // load has two tile periods to land.
    uint4 xra[CPT], xrb[CPT];
    auto fetch = [&](int t, uint4 (&xr)[CPT]) {
      if (t >= ntiles) return;
      const int64_t r0 = pc.begin + int64_t(t) * kTile;
#pragma unroll
      for (int k = 0; k < CPT; ++k) {
        const int cid = tid + k * NT;
        int64_t row = r0 + cid / CH;
        if (row > pc.end - 1) row = pc.end - 1;
        xr[k] = *reinterpret_cast<const uint4*>(p.X + row * D + (cid % CH) * 8);
      }
    };
    auto stash = [&](int t, int buf, const uint4 (&xr)[CPT]) {
      if (t >= ntiles) return;
#pragma unroll
      for (int k = 0; k < CPT; ++k) {
        const int cid = tid + k * NT;
        sm.xbuf[buf][(cid % CH) * 33 + cid / CH] = xr[k];
      }
    };
    // k-slices [ks0, ks1) of this wave's projection of the X tile in xbuf[buf]
    auto project = [&](int buf, int ks0, int ks1, f32x16& acc) {
#pragma unroll
      for (int ks = ks0; ks < ks1; ++ks) {
        Pack8 x;
        x.u = sm.xbuf[buf][(2 * ks + hf) * 33 + l32];
        acc = ROLE ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.v, wreg[ks], acc, 0, 0, 0)
                   : __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[ks], x.v, acc, 0, 0, 0);
      }
    };
    // hand the projected tile to the partner wave: bf16 operand halves (+ key norms)
    auto publish = [&](int buf, const f32x16& acc) {
      Pack8 r0, r1;
      float n2 = 0.f;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float a = ROLE ? acc[i] : acc[i] * p.c, b = ROLE ? acc[i + 1] : acc[i + 1] * p.c;
        if (ROLE == 0) n2 = fmaf(a, a, fmaf(b, b, n2));
        const uint32_t pk = cvt_pk_bf16(a, b);
        if (i < 8) r0.w[i / 2] = pk; else r1.w[(i - 8) / 2] = pk;
      }
      sm.kvbuf[buf][hl][ROLE][0][lane] = r0.u;
      sm.kvbuf[buf][hl][ROLE][1][lane] = r1.u;
      if (ROLE == 0) sm.knorm[buf][hl][lane] = n2;
    };
    // attention over tile t (operands in kvbuf[buf]) with the projection of tile t+1 woven in
    auto tile = [&](int t, int buf) {
      Pack8 k0, k1, v0, v1;
      k0.u = sm.kvbuf[buf][hl][0][0][lane];
      k1.u = sm.kvbuf[buf][hl][0][1][lane];
      v0.u = sm.kvbuf[buf][hl][1][0][lane];
      v1.u = sm.kvbuf[buf][hl][1][1][lane];
      const float kn2 = sm.knorm[buf][hl][lane] + sm.knorm[buf][hl][lane ^ 32];
      const bool unsafe = __builtin_amdgcn_ballot_w64(kn2 * qmax2 > kSafeBound2) != 0;
      const int64_t left = pc.end - (pc.begin + int64_t(t) * kTile);
      const int nvalid = left < kTile ? int(left) : kTile;
      const int nvl = nvalid - 4 * hf;
      const bool general = unsafe || mode == 2;
      if (general && mode == 0) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) m[qb] = -INFINITY;
      }
      mode = general ? 2 : 1;
      const bool masked = nvalid < kTile;
      const bool more = t + 1 < ntiles;
      f32x16 acc = {0};
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        attend_block(k0.v, k1.v, v0.v, v1.v, qop[qb][0], qop[qb][1], o[qb], l[qb], m[qb], general, masked, nvl);
        if (more && qb * KPB < KS) project(buf ^ 1, qb * KPB, qb * KPB + KPB, acc);
      }
      if (more) publish(buf ^ 1, acc);
    };

    lds_barrier();   // every wave is done with the previous piece's buffers
    fetch(0, xra);
    fetch(1, xrb);
    stash(0, 0, xra);
    fetch(2, xra);
    lds_barrier();
    {
      f32x16 acc = {0};
      project(0, 0, KS, acc);
      publish(0, acc);
    }
    stash(1, 1, xrb);
    fetch(3, xrb);

    for (int t = 0; t < ntiles; t += 2) {
      lds_barrier();
      tile(t, 0);
      stash(t + 2, 0, xra);
      fetch(t + 4, xra);
      if (t + 1 < ntiles) {
        lds_barrier();
        tile(t + 1, 1);
        stash(t + 3, 1, xrb);
        fetch(t + 5, xrb);
      }
    }

    // ---- partial record of this piece: slot = segment + user
    const int64_t slot = g + pc.user;
    float* rec = p.partials + ((slot * p.H + h) * (p.S / 32) + (qbase / 32)) * kRecFloats;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      float* r = rec + qb * kRecFloats + lane;
#pragma unroll
      for (int i = 0; i < 16; ++i) r[i * 64] = o[qb][i];
      r[16 * 64] = l[qb] + __shfl_xor(l[qb], 32, 64);
      r[17 * 64] = m[qb];
    }
  }
}

template <int D, int NQB, int HPW>
__global__ __launch_bounds__(HPW * 128, (HPW == 1 ? 2 : 1)) void summarize_mfma_kernel(MfmaSummarizeParams p) {
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
    summarize_wave<D, NQB, HPW, 1>(p, sm, g, h, hl, seg_begin, seg_end);
  else
    summarize_wave<D, NQB, HPW, 0>(p, sm, g, h, hl, seg_begin, seg_end);
}

// Merge of a user's partial records, ascending segment order (fixed, so the
// result is bitwise reproducible):  m = max m_c, w_c = 2^(m_c - m),
// out = sum_c w_c O_c / sum_c w_c l_c.   grid (S/32, H, B), 256 threads: wave w
// owns accumulator registers 4w..4w+3, i.e. channels 8w + 4 hf + 0..3.
__global__ __launch_bounds__(256) void merge_mfma_kernel(const float* __restrict__ partials,
                                                         const int64_t* __restrict__ offsets, int S, int d,
                                                         int H, int seg, int64_t G,
                                                         uint16_t* __restrict__ out) {
  const int qb = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int hf = lane >> 5, l32 = lane & 31;
  const int64_t begin = offsets[b], end = offsets[b + 1];
  uint16_t* dst = out + (int64_t(b) * S + qb * 32 + l32) * d + 32 * h + 8 * w + 4 * hf;
  if (end <= begin) {
    *reinterpret_cast<uint2*>(dst) = make_uint2(0u, 0u);
    return;
  }
  int64_t g0 = begin / seg, g1 = (end - 1) / seg;
  if (g0 < 0) g0 = 0;
  if (g1 > G - 1) g1 = G - 1;
  const int nqb = S / 32;
  auto rec = [&](int64_t g) { return partials + (((g + b) * H + h) * nqb + qb) * kRecFloats + lane; };
  float m = -INFINITY;
  for (int64_t g = g0; g <= g1; ++g) m = fmaxf(m, rec(g)[17 * 64]);
  float l = 0.f, o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
  for (int64_t g = g0; g <= g1; ++g) {
    const float* r = rec(g);
    const float wgt = exp2f(r[17 * 64] - m);
    l = fmaf(r[16 * 64], wgt, l);
    o0 = fmaf(r[(4 * w + 0) * 64], wgt, o0);
    o1 = fmaf(r[(4 * w + 1) * 64], wgt, o1);
    o2 = fmaf(r[(4 * w + 2) * 64], wgt, o2);
    o3 = fmaf(r[(4 * w + 3) * 64], wgt, o3);
  }
  const float inv = 1.f / l;
  uint2 pk;
  pk.x = uint32_t(f32_to_bf16_bits(o0 * inv)) | (uint32_t(f32_to_bf16_bits(o1 * inv)) << 16);
  pk.y = uint32_t(f32_to_bf16_bits(o2 * inv)) | (uint32_t(f32_to_bf16_bits(o3 * inv)) << 16);
  *reinterpret_cast<uint2*>(dst) = pk;
}

// ------------------------------------------------------------------ host side

static bool shape_d128(const vista_summarize_desc& d) { return d.d == 128 && d.H == 4; }
static bool shape_d256(const vista_summarize_desc& d) { return d.d == 256 && d.H == 8; }

bool mfma_summarize_supported(const vista_summarize_desc& d) {
  if (d.dtype != VISTA_BF16) return false;
  if (!(shape_d128(d) || shape_d256(d))) return false;
  return d.S == 64 || d.S == 128 || d.S == 256 || d.S == 512;
}

static size_t partial_bytes(const vista_summarize_desc& d, int seg) {
  int64_t G = (d.total_items + seg - 1) / seg;
  return size_t(G + d.B) * d.H * (d.S / 32) * kRecFloats * sizeof(float);
}

size_t mfma_summarize_workspace(const vista_summarize_desc& d, int seg) {
  return kHeaderBytes + ((partial_bytes(d, seg) + 255) & ~size_t(255));
}

template <int D, int NQB, int HPW>
static void launch_main(const MfmaSummarizeParams& p, int64_t G, hipStream_t s) {
  const int64_t groups = (G + 7) / 8;
  const int64_t blocks = groups * 8 * p.nhg;
  hipLaunchKernelGGL((summarize_mfma_kernel<D, NQB, HPW>), dim3(unsigned(blocks)), dim3(HPW * 128), 0, s, p);
}

vista_status mfma_summarize(const SummarizeArgs& a) {
  const vista_summarize_desc& d = a.desc;
  MfmaSummarizeParams p;
  p.X = static_cast<const uint16_t*>(a.X);
  p.offsets = a.offsets;
  p.Q = static_cast<const uint16_t*>(a.Q);
  p.q_user_stride = d.q_user_stride;
  p.Wk = static_cast<const uint16_t*>(a.Wk);
  p.Wv = static_cast<const uint16_t*>(a.Wv);
  p.partials = reinterpret_cast<float*>(a.workspace + kHeaderBytes);
  p.B = d.B;
  p.S = d.S;
  p.H = d.H;
  p.N = d.total_items;
  p.seg = a.seg;
  p.c = a.scale_log2;
  if (a.G > 0) {
    if ((a.G + 7) / 8 * 8 * 4 > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
    if (shape_d128(d)) {
      p.nhg = 1;
      switch (d.S) {
        case 64: launch_main<128, 1, 4>(p, a.G, a.stream); break;
        case 128: launch_main<128, 2, 4>(p, a.G, a.stream); break;
        case 256:
#ifdef EXP_HPW1
          p.nhg = 4;
          launch_main<128, 4, 1>(p, a.G, a.stream);
#else
          launch_main<128, 4, 4>(p, a.G, a.stream);
#endif
          break;
        default:
          p.nhg = 2;
          launch_main<128, 8, 2>(p, a.G, a.stream);
          break;
      }
    } else {
      p.nhg = 4;
      switch (d.S) {
        case 64: launch_main<256, 1, 2>(p, a.G, a.stream); break;
        case 128: launch_main<256, 2, 2>(p, a.G, a.stream); break;
        case 256: launch_main<256, 4, 2>(p, a.G, a.stream); break;
        default: launch_main<256, 8, 2>(p, a.G, a.stream); break;
      }
    }
    VISTA_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(merge_mfma_kernel, dim3(d.S / 32, d.H, d.B), dim3(256), 0, a.stream, p.partials, a.offsets,
                     d.S, d.d, d.H, a.seg, a.G, static_cast<uint16_t*>(a.out));
  VISTA_LAUNCH_CHECK();
  return VISTA_OK;
}

}  // namespace vista
