// Stage 2 on the matrix cores (bf16 MFMA, fp32 accumulate), gfx950.
//
// One workgroup (4 waves) serves one user and two heads; a round scores 64
// candidates: wave (head h, half c) takes the 32 candidates of half c for
// head h.  Several workgroups share a compute unit (three at S = 256), so one
// group's operand set-up hides behind the others' rounds.  The user's S summary tokens of a head are resident twice: as the K
// operand of S^T = K Q^T (keys x candidates) in each wave's registers, and,
// transposed, as the V operand of O^T = V^T P^T in LDS, shared by the head's two
// waves.  The transposed copy is made by the matrix core itself (K block times
// a 0/1 selector matrix lands in the accumulator layout, which is the A-operand
// layout of the second product).
//
// HBM traffic is fully coalesced and never touches vector registers on the way
// in.  The user's S x 128 B slab of summaries is brought in by one burst of
// direct global->LDS loads (each 8 lanes fetch the two heads' 128 bytes of a row) into the region
// that will hold the V operands; every wave lifts its K operands out of it, and
// after a barrier the region is overwritten with the V operands.  Candidates
// arrive the same way, but each wave fetches only its own 32 rows x 64 B of the
// next round while it computes this one, writes its results over them, and
// stores them one round later, so the round loop needs no barrier at all.  Slab
// and parts keep their 16-byte chunks at a position XOR-ed with row bits, so
// row-wise fills and column-wise operand accesses are free of bank conflicts.
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
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short i16x4;

namespace {

constexpr float kSafeBound2 = 3600.f;
constexpr int kRound = 64;                 // candidates per round

struct AttendParams {
  const uint16_t* cand;
  const uint16_t* summ;     // bf16 summaries, or null when they come as codes
  const int8_t* codes;      // int8 summaries [B, S, d] ...
  const float* scales;      // ... and their scales [B, S, H]
  int self_term;            // candidates also attend to themselves (Eq. 3)
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

constexpr int kHeads = 2;                  // heads per workgroup
constexpr int kWaves = 2 * kHeads;         // waves per workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int kRowChunks = 4 * kHeads;     // 16-byte chunks of a workgroup's slice of a row
// Buffers per wave (a deeper queue of parts buys nothing: a round outlasts the memory latency).
constexpr int part_buffers(int) { return 2; }

template <int NKB, int NB>
struct AttendLds {
  uint4 part[kWaves][NB][128];            // per wave, NB buffers: its 32 candidates x 64 B of a round, overwritten by
                                     // their outputs; row r, chunk c at [r * 4 + (c ^ ((r >> 2) & 3))]
  union {
    uint4 vop[NKB][kHeads][2][64];   // V operands: [key block][head][half of the 16 registers][lane]
    uint4 slab[NKB * 32 * kRowChunks];   // before that: the raw summaries: row r, chunk c at [r * 8 + (c ^ ((r >> 1) & 7))]
  };
};

template <int V>
struct Int { static constexpr int value = V; };

// NKB = S / 32 key blocks.
template <int NKB>
__global__ __launch_bounds__(kThreads, (NKB <= 6 || NKB == 8) ? 3 : 2) void attend_mfma_kernel(AttendParams p) {
  constexpr int NB = part_buffers(NKB);
  __shared__ AttendLds<NKB, NB> sm;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hl = wave >> 1;            // head within the group of two
  const int half = wave & 1;           // which 32 candidates of a round
  const int hf = lane >> 5, l32 = lane & 31;
  const int hgroups = p.H / kHeads;
  // XCD-aware block -> (user, chunk, head group): block ids that differ by a multiple of 8 share an
  // XCD and its L2, so the head groups of one (user, chunk) are placed 8 ids apart -- they read
  // neighbouring halves of the same rows (of the same 128-byte lines when the summaries are int8).
  const int64_t units = int64_t(p.B) * p.chunks;
  const int64_t grp = blockIdx.x / (8 * hgroups);
  const int idl = int(blockIdx.x - grp * (8 * hgroups));
  const int64_t unit = grp * 8 + (idl & 7);
  if (unit >= units) return;             // padding blocks of the last group (whole workgroup)
  const int hg = idl >> 3;
  const int chunk = int(unit % p.chunks);
  const int b = int(unit / p.chunks);
  const int row_bytes = p.d * 2;
  const int slice = hg * (64 * kHeads);   // byte offset of this head group's channels inside a row

  const int nrounds_total = (p.C + kRound - 1) / kRound;
  const int r0 = chunk * p.rounds_per_wg;
  int r1 = r0 + p.rounds_per_wg;
  if (r1 > nrounds_total) r1 = nrounds_total;
  if (r0 >= r1) return;                // whole workgroup
  const char* Tb = reinterpret_cast<const char*>(p.cand) + int64_t(b) * p.C * row_bytes + slice;
  char* Ob = reinterpret_cast<char*>(p.out) + int64_t(b) * p.C * row_bytes + slice;
  const char* Yb = reinterpret_cast<const char*>(p.summ) + int64_t(b) * p.S * row_bytes + slice;

  // Direct global->LDS load of 64 x 16 bytes: lane l lands at dst + 16 l.
  auto dma = [&](const uint4* dst, const char* base, uint32_t voff) __attribute__((always_inline)) {
    const uint32_t lds_base =
        uint32_t(reinterpret_cast<uintptr_t>((void __attribute__((address_space(3)))*)(dst)));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(base)
                 : "memory", "m0");
  };
  // Waits until at most n of this wave's newest vector-memory operations are outstanding.
  auto wait_vm = [&](auto n_c) __attribute__((always_inline)) {
    constexpr int n = decltype(n_c)::value;
    __builtin_amdgcn_s_waitcnt((n & 0xF) | ((n >> 4) << 14) | 0x0F70);
  };
  // A wave moves its own part of a round and nobody else touches it, so the round loop
  // needs no barrier.  Fill: two loads per lane; lane l of instruction i fills chunk
  // q = 64 i + l of the part, i.e. row q / 4, and fetches that row's chunk
  // (q % 4) ^ ((row >> 2) % 4) of the head's 64 bytes.  Rows past C are clamped.
  auto fill = [&](int round, int tb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = i * 64 + lane;
      const int row = q >> 2;
      int cand = round * kRound + 32 * half + row;
      if (cand > p.C - 1) cand = p.C - 1;
      dma(&sm.part[wave][tb][i * 64], Tb,
          uint32_t(cand) * uint32_t(row_bytes) + uint32_t(64 * hl + ((q & 3) ^ ((row >> 2) & 3)) * 16));
    }
  };
  // Store of a finished part, 64 contiguous bytes per row (rows past C are skipped).
  auto drain = [&](int round, int tb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = i * 64 + lane;
      const int row = q >> 2;
      const int cand = round * kRound + 32 * half + row;
      const uint4 v = sm.part[wave][tb][q];
      if (cand < p.C)
        *reinterpret_cast<uint4*>(Ob + int64_t(cand) * row_bytes + 64 * hl + ((q & 3) ^ ((row >> 2) & 3)) * 16) = v;
    }
  };

  // ---- the slab of summaries and the first candidate tile are requested together
  if (p.codes == nullptr) {
#pragma unroll
    for (int i = 0; i < NKB; ++i) {
      const int j = (i * kWaves + wave) * 64 + lane;    // slab chunk: row j / 8
      const int row = j / kRowChunks;                   // < 32 NKB = S
      dma(&sm.slab[(i * kWaves + wave) * 64], Yb,
          uint32_t(row) * uint32_t(row_bytes) + uint32_t(((j & (kRowChunks - 1)) ^ ((row >> 1) & (kRowChunks - 1))) * 16));
    }
  } else {
    // Quantized summaries (Sec. 3.1): 16 codes of a row at a time are turned into code * scale,
    // rounded to bf16 and put where the raw rows would have landed.  A thread takes quarter
    // q of the two heads' 64 codes of a row; its scale is that of head q / 2.
    const int8_t* Cb = p.codes + int64_t(b) * p.S * p.d + hg * (32 * kHeads);
    const float* Sb = p.scales + int64_t(b) * p.S * p.H + hg * kHeads;
    for (int j = tid; j < NKB * 32 * 4; j += kThreads) {
      const int row = j >> 2, q = j & 3;
      const uint4 raw = *reinterpret_cast<const uint4*>(Cb + int64_t(row) * p.d + 16 * q);
      const float sc = Sb[int64_t(row) * p.H + (q >> 1)];
      // code + 128 is an unsigned byte (flip the sign bit); it converts exactly and
      // (byte - 128) * scale is one fused multiply-add
      const uint32_t w[4] = {raw.x ^ 0x80808080u, raw.y ^ 0x80808080u, raw.z ^ 0x80808080u, raw.w ^ 0x80808080u};
      const float off = -128.f * sc;
      uint32_t pk[8];
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float a = fmaf(float((w[e / 4] >> (8 * (e % 4))) & 0xFFu), sc, off);
        const float c2 = fmaf(float((w[e / 4] >> (8 * (e % 4) + 8)) & 0xFFu), sc, off);
        pk[e / 2] = cvt_pk_bf16(a, c2);
      }
      const int sw = (row >> 1) & (kRowChunks - 1);
      sm.slab[row * kRowChunks + ((2 * q) ^ sw)] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
      sm.slab[row * kRowChunks + ((2 * q + 1) ^ sw)] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
    }
  }
  // the first NB-1 rounds' parts (a round past the end repeats the last one: the count of
  // loads in flight stays a constant)
#pragma unroll
  for (int i = 0; i < NB - 1; ++i) fill(r0 + i < r1 ? r0 + i : r1 - 1, i);
  wait_vm(Int<2 * (NB - 1)>{});                // the slab has landed (the parts may be on their way)
  lds_barrier();

  // ---- resident operands of this (user, head): K in registers (both waves of the head),
  //      V through the selector MFMA into LDS (each wave builds half of the key blocks)
  bf16x8 kop[NKB][2];
  float kmax2 = 0.f;
  {
    // K operands of all key blocks; they carry the score scale (one extra bf16 rounding of
    // scale*log2e*k)
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      const int row = kb * 32 + l32;
      float n2 = 0.f;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        Pack8 k, s;
        k.u = sm.slab[row * kRowChunks + ((4 * hl + 2 * ks + hf) ^ ((row >> 1) & (kRowChunks - 1)))];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float a = bf16_lo(k.w[w]), c2 = bf16_hi(k.w[w]);
          n2 = fmaf(a, a, fmaf(c2, c2, n2));
          s.w[w] = cvt_pk_bf16(a * p.c, c2 * p.c);
        }
        kop[kb][ks] = s.v;
      }
      n2 += __shfl_xor(n2, 32, 64);
      kmax2 = fmaxf(kmax2, n2);
    }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) kmax2 = fmaxf(kmax2, __shfl_xor(kmax2, off, 64));
    kmax2 *= p.c * p.c;

    // V operands: (K block) x (selector) reproduces the block in accumulator layout.  Block
    // kb of both heads goes exactly where the raw rows of block kb were, so only a
    // block's own readers have to be done before it is written: up to four blocks per wave
    // are converted in registers, then a barrier, then their stores.
    Pack8 sel[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < 8; ++j) sel[ks].h[j] = (l32 == 16 * ks + 8 * hf + j) ? 0x3F80 : 0;
    constexpr int NV = (NKB + 1) / 2;            // key blocks whose V operand this wave builds: kb = 2 j + half
#pragma unroll
    for (int j0 = 0; j0 < NV; j0 += 4) {
      Pack8 vnew[4][2];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int kb = 2 * (j0 + jj) + half;
        if (j0 + jj < NV && kb < NKB) {
          const int row = kb * 32 + l32;
          Pack8 k0, k1;
          k0.u = sm.slab[row * kRowChunks + ((4 * hl + hf) ^ ((row >> 1) & (kRowChunks - 1)))];
          k1.u = sm.slab[row * kRowChunks + ((4 * hl + 2 + hf) ^ ((row >> 1) & (kRowChunks - 1)))];
          f32x16 t = {0};
          t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0.v, sel[0].v, t, 0, 0, 0);
          t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1.v, sel[1].v, t, 0, 0, 0);
#pragma unroll
          for (int i = 0; i < 8; i += 2) {
            vnew[jj][0].w[i / 2] = cvt_pk_bf16(t[i], t[i + 1]);
            vnew[jj][1].w[i / 2] = cvt_pk_bf16(t[8 + i], t[8 + i + 1]);
          }
        }
      }
      lds_barrier();                             // every reader of these blocks' raw rows is done
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int kb = 2 * (j0 + jj) + half;
        if (j0 + jj < NV && kb < NKB) {
          sm.vop[kb][hl][0][lane] = vnew[jj][0].u;
          sm.vop[kb][hl][1][lane] = vnew[jj][1].u;
        }
      }
    }
  }

  // operand position of this lane inside its part: row l32, chunk 2 ks + hf
  const int osw = (l32 >> 2) & 3;
  // A operand of the denominator products: ones in row 0 of every 4x4 block
  const uint32_t onesw = (lane & 3) == 0 ? 0x3F803F80u : 0u;
  const uint2 onesrow = make_uint2(onesw, onesw);
  lds_barrier();                                 // the V operands of all key blocks are in place

  // Round r lives in buffer (r - r0) mod NB.  Its part was requested NB-1 rounds ago; loads
  // complete in order among themselves (stores are not ordered with them), so it has landed
  // once no more operations are outstanding than the loads requested after it.
  int cur = 0;
  for (int r = r0; r < r1; ++r) {
    const int ahead = r1 - 1 - r;                // rounds after this one
    if (NB >= 4 && ahead >= 2) wait_vm(Int<4>{});
    else if (NB >= 3 && ahead >= 1) wait_vm(Int<2>{});
    else wait_vm(Int<0>{});
    const int prev = cur == 0 ? NB - 1 : cur - 1;
    if (r > r0) {
      drain(r - 1, prev);                        // reads the previous round's buffer into registers, then stores
      __builtin_amdgcn_s_waitcnt(0xC07F);        // lgkmcnt(0): those reads are done before the buffer is refilled
    }
    if (r + NB - 1 < r1) fill(r + NB - 1, prev);

    Pack8 c0, c1;
    c0.u = sm.part[wave][cur][l32 * 4 + (hf ^ osw)];
    c1.u = sm.part[wave][cur][l32 * 4 + ((2 + hf) ^ osw)];
    float qn2 = 0.f;                             // squared norm of the candidate's head slice (packed dot products)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const bf16x2 a = __builtin_bit_cast(bf16x2, c0.w[w]), b2 = __builtin_bit_cast(bf16x2, c1.w[w]);
      qn2 = __builtin_amdgcn_fdot2_f32_bf16(a, a, qn2, false);
      qn2 = __builtin_amdgcn_fdot2_f32_bf16(b2, b2, qn2, false);
    }
    qn2 += __shfl_xor(qn2, 32, 64);
    // (with the self term the candidate's own score c |q|^2 must stay in range as well)
    const bool general = __builtin_amdgcn_ballot_w64(qn2 * kmax2 > kSafeBound2 || (p.self_term && qn2 * p.c > 60.f)) != 0;
    float mrun = 0.f;          // reference maximum the weights were taken against
    // Key blocks stream through: 32 keys x 32 candidates of scores at a time.  The common
    // route is straight-line code over all key blocks (one scheduling region), the scores
    // of a block computed while the previous block's exponentials run.
    f32x16 o = {0};
    float lsum;
    if (!general) {
      // The denominator on the matrix core: a 4x4x4 product (16 blocks, one per four lanes) whose
      // A block has ones in its first row adds a lane's own four packed weights into register 0
      // of that lane.  It issues like one plain vector instruction for four weights (a chain of
      // adds takes four) and sums the bf16 weights the numerator uses; two accumulators take turns.
      f32x4 lacc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
      f32x16 nx = {0};
      nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[0][0], c0.v, nx, 0, 0, 0);
      nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[0][1], c1.v, nx, 0, 0, 0);
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
        const f32x16 sc = nx;
        if (kb + 1 < NKB) {
          const f32x16 z = {0};
          nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kb + 1][0], c0.v, z, 0, 0, 0);
          nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kb + 1][1], c1.v, nx, 0, 0, 0);
        }
        Pack8 v0, v1;
        v0.u = sm.vop[kb][hl][0][lane];
        v1.u = sm.vop[kb][hl][1][lane];
        Pack8 p0, p1;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const uint32_t pk = cvt_pk_bf16(__builtin_amdgcn_exp2f(sc[i]), __builtin_amdgcn_exp2f(sc[i + 1]));
          if (i < 8) p0.w[i / 2] = pk; else p1.w[(i - 8) / 2] = pk;
        }
#pragma unroll
        for (int part = 0; part < 4; ++part) {
          const uint2 pw = part < 2 ? make_uint2(p0.w[2 * part], p0.w[2 * part + 1])
                                    : make_uint2(p1.w[2 * part - 4], p1.w[2 * part - 3]);
          lacc[part & 1] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(i16x4, onesrow),
                                                                  __builtin_bit_cast(i16x4, pw), lacc[part & 1], 0, 0, 0);
        }
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v0.v, p0.v, o, 0, 0, 0);
        o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v1.v, p1.v, o, 0, 0, 0);
      }
      lsum = lacc[0][0] + lacc[1][0];
      lsum += __shfl_xor(lsum, 32, 64);
    } else {
      float l[4] = {0.f, 0.f, 0.f, 0.f};
      float m = -INFINITY;
#pragma unroll 1
      for (int kb = 0; kb < NKB; ++kb) {
        f32x16 sc = {0};
        Pack8 ka, kb2;
        // dynamic key-block index: the operands are picked out of the registers by selects
        ka.v = kop[0][0]; kb2.v = kop[0][1];
#pragma unroll
        for (int t = 1; t < NKB; ++t)
          if (t == kb) { ka.v = kop[t][0]; kb2.v = kop[t][1]; }
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, c0.v, sc, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb2.v, c1.v, sc, 0, 0, 0);
        Pack8 v0, v1;
        v0.u = sm.vop[kb][hl][0][lane];
        v1.u = sm.vop[kb][hl][1][lane];
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
      lsum = (l[0] + l[1]) + (l[2] + l[3]);
      lsum += __shfl_xor(lsum, 32, 64);
      mrun = m;
    }
    if (p.self_term) {
      // one more key and value: the candidate itself (no projections in this stage), score c |q|^2
      const float s_self = p.c * qn2;
      float ps;
      if (general) {
        const float mn = fmaxf(mrun, s_self);
        const float alpha = __builtin_amdgcn_exp2f(mrun - mn);
        lsum *= alpha;
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i] *= alpha;
        ps = __builtin_amdgcn_exp2f(s_self - mn);
      } else {
        ps = __builtin_amdgcn_exp2f(s_self);
      }
      lsum += ps;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint2 own = reinterpret_cast<const uint2*>(&sm.part[wave][cur][l32 * 4 + (g ^ osw)])[hf];
        o[4 * g] = fmaf(ps, bf16_lo(own.x), o[4 * g]);
        o[4 * g + 1] = fmaf(ps, bf16_hi(own.x), o[4 * g + 1]);
        o[4 * g + 2] = fmaf(ps, bf16_lo(own.y), o[4 * g + 2]);
        o[4 * g + 3] = fmaf(ps, bf16_hi(own.y), o[4 * g + 3]);
      }
    }
    const float inv = __builtin_amdgcn_rcpf(lsum);
    // register group g holds channels 8 g + 4 hf + 0..3 of the head: 8 bytes at chunk 4 hl + g, half hf.
    // The results go where this wave's own operands were (nobody else reads those chunks).
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 pk;
      pk.x = cvt_pk_bf16(o[4 * g] * inv, o[4 * g + 1] * inv);
      pk.y = cvt_pk_bf16(o[4 * g + 2] * inv, o[4 * g + 3] * inv);
      reinterpret_cast<uint2*>(&sm.part[wave][cur][l32 * 4 + (g ^ osw)])[hf] = pk;
    }
    asm volatile("" ::: "memory");   // the 8-byte stores above are read back as 16-byte chunks by the next drain
    cur = cur == NB - 1 ? 0 : cur + 1;
  }
  __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0): this wave's last results are in its buffer
  drain(r1 - 1, cur == 0 ? NB - 1 : cur - 1);
}

template <int NKB>
hipError_t launch_attend(const AttendParams& p, hipStream_t s) {
  const int64_t units = int64_t(p.B) * p.chunks;
  const unsigned blocks = unsigned((units + 7) / 8 * 8 * (p.H / kHeads));
  return launch(attend_mfma_kernel<NKB>, dim3(blocks), dim3(kThreads), 0, s, p);
}

}  // namespace

bool mfma_target_attend_supported(const vista_attend_desc& d) {
  return d.dtype == VISTA_BF16 && d.d == 32 * d.H && d.H % kHeads == 0 && d.S % 32 == 0 && (d.S <= 256 || (d.S % 64 == 0 && d.S <= 512)) &&
         int64_t(d.C) * d.d * 2 < (int64_t(1) << 32);
}

vista_status mfma_target_attend(const vista_attend_desc& d, float scale_log2, const void* cand,
                                const void* summ, const int8_t* codes, const float* scales, void* out,
                                hipStream_t s) {
  AttendParams p;
  p.cand = static_cast<const uint16_t*>(cand);
  p.summ = static_cast<const uint16_t*>(summ);
  p.codes = codes;
  p.scales = scales;
  p.self_term = (d.flags & VISTA_FLAG_SELF_TERM) ? 1 : 0;
  p.out = static_cast<uint16_t*>(out);
  p.B = d.B; p.C = d.C; p.S = d.S; p.d = d.d; p.H = d.H;
  p.c = scale_log2;
  // Rounds per workgroup: long enough to amortise the operand set-up (about two rounds'
  // worth of work), short enough to give the chip two turns of workgroups (256 compute
  // units x three resident groups, two beyond S = 256).
  const int nrounds = (d.C + kRound - 1) / kRound;
  const int64_t groups = int64_t(d.B) * (d.H / kHeads);
  int per = 8;
  const int nkb = d.S / 32;
  const int64_t want = 256 * 2 * ((nkb <= 6 || nkb == 8) ? 3 : 2);
  while (per > 2 && groups * ((nrounds + per - 1) / per) < want) per >>= 1;
  p.rounds_per_wg = per;
  p.chunks = (nrounds + per - 1) / per;
  if ((int64_t(d.B) * p.chunks + 7) / 8 * 8 * (d.H / kHeads) > 0x7FFFFFFF) return VISTA_ERR_UNSUPPORTED;
  hipError_t e;
  switch (nkb) {
    case 1: e = launch_attend<1>(p, s); break;
    case 2: e = launch_attend<2>(p, s); break;
    case 3: e = launch_attend<3>(p, s); break;
    case 4: e = launch_attend<4>(p, s); break;
    case 5: e = launch_attend<5>(p, s); break;
    case 6: e = launch_attend<6>(p, s); break;
    case 7: e = launch_attend<7>(p, s); break;
    case 8: e = launch_attend<8>(p, s); break;
    case 10: e = launch_attend<10>(p, s); break;
    case 12: e = launch_attend<12>(p, s); break;
    case 14: e = launch_attend<14>(p, s); break;
    case 16: e = launch_attend<16>(p, s); break;
    default: return VISTA_ERR_UNSUPPORTED;
  }
  return e == hipSuccess ? VISTA_OK : VISTA_ERR_HIP;
}

}  // namespace vista
