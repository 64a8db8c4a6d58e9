// Epilogues of the GEMM core: what happens to a lane's 4x4x16 accumulators.
// A lane owns rows m_lane + 16*mi + v (64 consecutive) and columns n_lane + ni (4 consecutive).
#pragma once
#include "gemm_core.hpp"
#include "launch.hpp"

namespace ffn24 {

// Sums two 16-bit fields over the wave (each field's total must stay below 65536) and has lane 0 add them to slot
// `slot` of quantities ka and kb.
__device__ __forceinline__ void tele_add2(unsigned long long* tele, uint32_t packed, int ka, int kb, int slot) {
#pragma unroll
  for (int sft = 1; sft < 64; sft <<= 1) packed += (uint32_t)__shfl_xor((int)packed, sft, 64);
  if ((threadIdx.x & 63) == 0) {
    atomicAdd(tele + tele_index(ka, slot), (unsigned long long)(packed & 0xFFFFu));
    if (kb >= 0) atomicAdd(tele + tele_index(kb, slot), (unsigned long long)(packed >> 16));
  }
}

// A per-feature fp32 vector (bias, weight scale) over the lane's 64 features m_lane .. m_lane + 63, loaded once with
// 16-byte loads and shared by the lane's 4 tokens; `fill` everywhere if the vector is absent.
struct LaneVec64 {
  f32x4 v[16];
  __device__ __forceinline__ void load(const float* p, int m_lane, float fill) {
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = f32x4{fill, fill, fill, fill};
    if (p) {
#pragma unroll
      for (int i = 0; i < 16; i++) v[i] = *reinterpret_cast<const f32x4*>(p + m_lane + 4 * i);
    }
  }
  __device__ __forceinline__ float at(int i) const { return v[i >> 2][i & 3]; }   // feature m_lane + i
};

// The lane's 64 entries m_lane .. m_lane + 63 of a row map, loaded with 16-byte loads (the map and m_lane are 16-byte aligned).
struct LaneIdx64 {
  i32x4 v[16];
  __device__ __forceinline__ void load(const int* p, int m_lane) {
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = *reinterpret_cast<const i32x4*>(p + m_lane + 4 * i);
  }
  __device__ __forceinline__ int at(int i) const { return v[i >> 2][i & 3]; }
};

// What the backward epilogues read back of the forward's saved activation, for the lane's 4 tokens x 64 features, requested in one
// go before any arithmetic or store: a load placed inside the loops is followed by stores through pointers the compiler must assume
// may alias, so each one waited out a full memory round trip by itself (16 of them in the 2:4 epilogue, 32 in the dense one -- the
// latter had made the dense dH kernel 0.4 ms slower than the GEMM alone).
// 2:4: one 64-byte piece of kept values + 8 metadata bytes per token (bf16 panel form).
struct LaneSaved24 {
  u32x4 h[4][4];   // [ni][mi]: the kept values of groups 4 mi .. 4 mi + 3
  u32x2 mt[4];
  __device__ __forceinline__ void load(const __bf16* Hc, const uint8_t* meta, int F, int m_lane, int n_lane) {
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      size_t piece = a24_piece(n_lane + ni, m_lane >> 6, F >> 6);
      mt[ni] = *reinterpret_cast<const u32x2*>(meta + piece * 8);
#pragma unroll
      for (int mi = 0; mi < 4; mi++) h[ni][mi] = *reinterpret_cast<const u32x4*>(Hc + piece * 32 + 8 * mi);
    }
  }
};
// dense: the bf16 activation in dense panel form (64-byte pieces of 32 features), 16 features per (mi, ni).
struct LaneSavedDense {
  u32x4 h[4][4][2];   // [mi][ni][q]: features 16 mi + 8 q .. + 7 of token ni
  __device__ __forceinline__ void load(const __bf16* H, int F, int m_lane, int n_lane) {
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int ni = 0; ni < 4; ni++) {
        int f = m_lane + 16 * mi;
        const __bf16* p = H + a24_piece(n_lane + ni, f >> 5, F >> 5) * 32 + (f & 31);
        h[mi][ni][0] = *reinterpret_cast<const u32x4*>(p);
        h[mi][ni][1] = *reinterpret_cast<const u32x4*>(p + 8);
      }
  }
};

// C[m][n], n contiguous: 4 consecutive columns per lane and row -> one 8-byte store per row.
struct EpiRowMajor {
  struct Args { __bf16* C; int ldc; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        u32x2 o;
        o[0] = pack_bf16x2(acc[mi][0][v], acc[mi][1][v]);
        o[1] = pack_bf16x2(acc[mi][2][v], acc[mi][3][v]);
        *reinterpret_cast<u32x2*>(e.C + (size_t)(m_lane + 16 * mi + v) * e.ldc + n_lane) = o;
      }
  }
};

// Transposing store of a wave's 128 (m) x 128 (n) part of the tile, out[n][m] with m contiguous, through LDS.  A lane owns 64
// consecutive m of 4 columns n, i.e. whole 128-byte runs of 4 output rows, but one store instruction of the wave would put 64
// 16-byte pieces into 64 different lines (32 instructions, 2048 line transactions a wave; on the short-K weight-gradient GEMMs that
// alone made the transposing kernels 15 % slower than the row-major ones).  So the packed pieces first go to a wave-private 32
// KiB image [n][m] in the operand ring, which is free by then (row n, 16-byte piece c at piece position c ^ ((n >> 2) & 15), so
// that the 16 lanes an LDS instruction serves together hit 16 different positions both ways), and leave as 32 instructions that
// write 4 rows x 256 contiguous bytes each: 8 lines an instruction.
struct ColMajorStage {
  static constexpr int WAVE_BYTES = 128 * 256;
  // piece `c` (0..15: m_local / 8) of row 4 rho + ni
  static __device__ __forceinline__ void put(char* wbuf, int rho, int ni, int c, u32x4 v) {
    *reinterpret_cast<u32x4*>(wbuf + (4 * rho + ni) * 256 + ((c ^ (rho & 15)) << 4)) = v;
  }
  // out = the wave's corner &C[n_wave][m_wave]
  static __device__ __forceinline__ void flush(const char* wbuf, __bf16* out, int ldc) {
    const int lane = threadIdx.x & 63, c = lane & 15, sub = lane >> 4;
#pragma unroll
    for (int j = 0; j < 32; j++) {
      const int r = 4 * j + sub;
      u32x4 v = *reinterpret_cast<const u32x4*>(wbuf + r * 256 + ((c ^ (j & 15)) << 4));
      *reinterpret_cast<u32x4*>(out + (size_t)r * ldc + 8 * c) = v;
    }
  }
};

// C stored transposed, out[n][m] with m contiguous (staged through LDS, see ColMajorStage; wbuf = the wave's 32 KiB).
struct EpiColMajor {
  static constexpr bool STAGED = true;
  struct Args { __bf16* C; int ldc; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane, char* wbuf) {
    const int lane = threadIdx.x & 63, rho = lane & 31, h = lane >> 5;
#pragma unroll
    for (int ni = 0; ni < 4; ni++)
#pragma unroll
      for (int mi = 0; mi < 4; mi++)
#pragma unroll
        for (int q = 0; q < 2; q++) {
          u32x4 o;
#pragma unroll
          for (int d = 0; d < 4; d++) o[d] = pack_bf16x2(acc[mi][ni][8 * q + 2 * d], acc[mi][ni][8 * q + 2 * d + 1]);
          ColMajorStage::put(wbuf, rho, ni, 8 * h + 2 * mi + q, o);
        }
    ColMajorStage::flush(wbuf, e.C + (size_t)(n_lane - 4 * rho) * e.ldc + (m_lane - 64 * h), e.ldc);
  }
};

// Dense FFN up-projection epilogue (Sec. 1, Squared ReLU): rows m are features, columns n are tokens;
// H[t][f] = bf16( max(0, acc + b1[f])^2 ), stored as the [T][F] operand of the down-projection; if Ht is given the
// same values are also stored as the [F][T] operand of the weight-gradient GEMM that reduces over tokens.  Both in
// the dense panel form of gemm_core.hpp (64-byte pieces of 32 k), like every A operand the library makes for itself.
// STATS: also counts the non-zero stored activations of the launch into tele (may be NULL), the sparsity level the
// dense path reports while 2:4 is still switched off (Sec. 2, last paragraph: the dense warm-up).
template <bool STATS>
struct EpiRelu2T {
  struct Args { __bf16* H; __bf16* Ht; const float* b1; int F; int T; unsigned long long* tele; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    uint32_t nonzero = 0u;   // of this lane's 256 activations
    LaneVec64 lb;
    lb.load(e.b1, m_lane, 0.f);
#pragma unroll
    for (int mi = 0; mi < 4; mi++) {
#pragma unroll
      for (int ni = 0; ni < 4; ni++) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          float r = fmaxf(acc[mi][ni][v] + lb.at(16 * mi + v), 0.f);
          acc[mi][ni][v] = r * r;
        }
        int f = m_lane + 16 * mi;
        __bf16* row = e.H + a24_piece(n_lane + ni, f >> 5, e.F >> 5) * 32 + (f & 31);
#pragma unroll
        for (int q = 0; q < 2; q++) {
          u32x4 o;
#pragma unroll
          for (int d = 0; d < 4; d++) {
            o[d] = pack_bf16x2(acc[mi][ni][8 * q + 2 * d], acc[mi][ni][8 * q + 2 * d + 1]);
            if constexpr (STATS) nonzero += min(o[d] & 0xFFFFu, 1u) + min(o[d] >> 16, 1u);
          }
          *reinterpret_cast<u32x4*>(row + 8 * q) = o;
        }
      }
      if (e.Ht) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          u32x2 o;
          o[0] = pack_bf16x2(acc[mi][0][v], acc[mi][1][v]);
          o[1] = pack_bf16x2(acc[mi][2][v], acc[mi][3][v]);
          *reinterpret_cast<u32x2*>(e.Ht + a24_piece(m_lane + 16 * mi + v, n_lane >> 5, e.T >> 5) * 32 + (n_lane & 31)) = o;
        }
      }
    }
    if constexpr (STATS) {
      if (e.tele) tele_add2(e.tele, nonzero, TELE_NONZERO, -1, blockIdx.x + (threadIdx.x >> 6));
    }
  }
};
using EpiRelu2 = EpiRelu2T<false>;

// Per-feature non-zero counts of the activation epilogues (Sec. 2, "Optimization 1": the column-level sparsity the first GEMM's
// epilogue can compute for free).  A lane counts its 4 tokens in 8-bit fields, 4 features per register: the packed pair of
// features 16 mi + 2 d and + 1 goes to fields (2 d) % 4 and (2 d + 1) % 4 of register 4 mi + d / 2.
__device__ __forceinline__ void nnz_count(uint32_t (&cnt)[16], uint32_t hpk, int mi, int d) {
  uint32_t lo = min(hpk & 0xFFFFu, 1u), hi = min(hpk >> 16, 1u);
  cnt[4 * mi + (d >> 1)] += (lo << (16 * (d & 1))) + (hi << (16 * (d & 1) + 8));
}
// The 32 lanes that hold the same 64 features add their fields up with a butterfly (<= 128 per field); lane r then adds the
// totals of features r and r + 32 to nnz [F] with atomics (the caller zeroes it).
__device__ __forceinline__ void nnz_flush(uint32_t (&cnt)[16], uint32_t* nnz, int m_lane) {
  int lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 16; i++)
#pragma unroll
    for (int sft = 1; sft < 32; sft <<= 1) cnt[i] += (uint32_t)__shfl_xor((int)cnt[i], sft, 64);
  int r = lane & 31;
  uint32_t w0 = 0u, w1 = 0u;
#pragma unroll
  for (int i = 0; i < 8; i++) {
    w0 = (r >> 2) == i ? cnt[i] : w0;
    w1 = (r >> 2) == i ? cnt[8 + i] : w1;
  }
  uint32_t c0 = (w0 >> (8 * (r & 3))) & 0xFFu, c1 = (w1 >> (8 * (r & 3))) & 0xFFu;
  if (c0) atomicAdd(nnz + m_lane + r, c0);
  if (c1) atomicAdd(nnz + m_lane + 32 + r, c1);
}

// Fused up-projection epilogue of the 2:4 FFN (Sec. 2: activation, then sparsification, in one pass):
// h = bf16(max(0, acc + b1)^2); of every 4 consecutive features of a token keep the 2 largest
// (ties -> lower index); write the kept pair and its metadata nibble.  The 4 members of a group are the
// accumulator registers 4a..4a+3 of one MFMA tile, so the pick needs no cross-lane traffic.
//   Hc, meta: the compressed activation [T][F/2] + [T][F/8] in panel form (gemm_core.hpp): a lane's 64 features of
//   one token are exactly one piece, 64 bytes of kept values (position order) + 8 metadata bytes (nibble
//   i0 | i1<<2, even group low).
//   Hdbg [T][F]    optional, row-major: the rounded activation before pruning (parity checks)
//   nnz  [F] optional: per-feature count of non-zero activations before pruning (Sec. 2, "Optimization 1": the
//   column-level sparsity the first GEMM's epilogue can compute for free), accumulated with atomics; the caller
//   zeroes it.  A lane counts its 4 tokens in 8-bit fields (4 features per register), the 32 lanes that hold the
//   same 64 features add their fields up with a butterfly, and each lane then adds two features' totals.
//   tele optional (STATS only): the launch's totals of non-zero activations before pruning and of non-zero kept values
//   (Sec. 2, first paragraph: the share of non-zeros that 2:4 drops), one pair of atomics per wave.
template <bool STATS>
struct EpiPrune24T {
  struct Args { __bf16* Hc; uint8_t* meta; __bf16* Hdbg; const float* b1; int F; uint32_t* nnz; unsigned long long* tele; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    uint32_t cnt[16];
    uint32_t kept = 0u;   // non-zero values among the lane's 128 stored ones
#pragma unroll
    for (int i = 0; i < 16; i++) cnt[i] = 0u;
    LaneVec64 lb;
    lb.load(e.b1, m_lane, 0.f);
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      size_t t = (size_t)(n_lane + ni);
      uint32_t vals[16];
      uint32_t nib[2] = {0u, 0u};
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        uint32_t hpk[8];
#pragma unroll
        for (int d = 0; d < 8; d++) {
          float b0 = lb.at(16 * mi + 2 * d), b1v = lb.at(16 * mi + 2 * d + 1);
          float r0 = fmaxf(acc[mi][ni][2 * d] + b0, 0.f);
          float r1 = fmaxf(acc[mi][ni][2 * d + 1] + b1v, 0.f);
          hpk[d] = pack_bf16x2(r0 * r0, r1 * r1);
          if constexpr (STATS) nnz_count(cnt, hpk[d], mi, d);
        }
        if (e.Hdbg) {
          __bf16* row = e.Hdbg + t * e.F + m_lane + 16 * mi;
          *reinterpret_cast<u32x4*>(row) = u32x4{hpk[0], hpk[1], hpk[2], hpk[3]};
          *reinterpret_cast<u32x4*>(row + 8) = u32x4{hpk[4], hpk[5], hpk[6], hpk[7]};
        }
#pragma unroll
        for (int a = 0; a < 4; a++) {
          // h >= 0, so the storage word is its own magnitude
          uint32_t pair;
          uint32_t n4 = pick24_packed(hpk[2 * a], hpk[2 * a + 1], pair);
          int gi = 4 * mi + a;
          vals[gi] = pair;
          nib[gi >> 3] |= n4 << (4 * (gi & 7));
          if constexpr (STATS) kept += min(pair & 0xFFFFu, 1u) + min(pair >> 16, 1u);
        }
      }
      size_t piece = a24_piece((int)t, m_lane >> 6, e.F >> 6);
      __bf16* hrow = e.Hc + piece * 32;
#pragma unroll
      for (int q = 0; q < 4; q++)
        *reinterpret_cast<u32x4*>(hrow + 8 * q) = u32x4{vals[4 * q], vals[4 * q + 1], vals[4 * q + 2], vals[4 * q + 3]};
      *reinterpret_cast<u32x2*>(e.meta + piece * 8) = u32x2{nib[0], nib[1]};
    }
    if constexpr (STATS) {
      if (e.tele) {
        // the lane's own non-zero count is the sum of its fields (at most 4 each); with the kept count, over the wave
        uint32_t tot = 0u;
#pragma unroll
        for (int i = 0; i < 16; i++) tot += (cnt[i] & 0xFFu) + ((cnt[i] >> 8) & 0xFFu) + ((cnt[i] >> 16) & 0xFFu) + (cnt[i] >> 24);
        tele_add2(e.tele, tot | (kept << 16), TELE_NONZERO, TELE_KEPT_TOK, blockIdx.x + (threadIdx.x >> 6));
      }
    }
    if constexpr (STATS) if (e.nnz) nnz_flush(cnt, e.nnz, m_lane);
  }
};
using EpiPrune24 = EpiPrune24T<false>;   // without the statistic (a compile-time switch: the plain kernel carries no trace of it)

// C[map[m]][n], n contiguous: the rows of the result are scattered through a row map (the split weight-gradient
// GEMMs work on a permutation of the hidden features and write each row back to its feature).
struct EpiRowMajorMapped {
  struct Args { __bf16* C; int ldc; const int* rowmap; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneIdx64 rows;
    rows.load(e.rowmap, m_lane);
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        u32x2 o;
        o[0] = pack_bf16x2(acc[mi][0][v], acc[mi][1][v]);
        o[1] = pack_bf16x2(acc[mi][2][v], acc[mi][3][v]);
        *reinterpret_cast<u32x2*>(e.C + (size_t)rows.at(16 * mi + v) * e.ldc + n_lane) = o;
      }
  }
};

// Dense backward, pointwise part: rows m are features, columns n are tokens; acc = dH[t][f];
// dZ[t][f] = bf16( acc * 2 sqrt(H[t][f]) )  (derivative of max(0,z)^2 is 2 max(0,z) = 2 sqrt(h)).
// Stored as a [T][F] operand and, for the weight-gradient GEMM that reduces over tokens, also as an [F][T] operand;
// H, dZ and dZt are all in dense panel form.
struct EpiDRelu {
  struct Args { const __bf16* H; __bf16* dZ; __bf16* dZt; int F; int T; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneSavedDense sv;
    sv.load(e.H, e.F, m_lane, n_lane);
#pragma unroll
    for (int mi = 0; mi < 4; mi++) {
#pragma unroll
      for (int ni = 0; ni < 4; ni++) {
        int f = m_lane + 16 * mi;
        size_t o = a24_piece(n_lane + ni, f >> 5, e.F >> 5) * 32 + (f & 31);
#pragma unroll
        for (int q = 0; q < 2; q++) {
          const u32x4 h = sv.h[mi][ni][q];
          u32x4 r;
#pragma unroll
          for (int d = 0; d < 4; d++) {
            float g0 = 2.f * __builtin_amdgcn_sqrtf(bf16_lo_to_f32(h[d]));
            float g1 = 2.f * __builtin_amdgcn_sqrtf(bf16_hi_to_f32(h[d]));
            acc[mi][ni][8 * q + 2 * d] *= g0;
            acc[mi][ni][8 * q + 2 * d + 1] *= g1;
            r[d] = pack_bf16x2(acc[mi][ni][8 * q + 2 * d], acc[mi][ni][8 * q + 2 * d + 1]);
          }
          *reinterpret_cast<u32x4*>(e.dZ + o + 8 * q) = r;
        }
      }
      if (e.dZt) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          u32x2 o;
          o[0] = pack_bf16x2(acc[mi][0][v], acc[mi][1][v]);
          o[1] = pack_bf16x2(acc[mi][2][v], acc[mi][3][v]);
          *reinterpret_cast<u32x2*>(e.dZt + a24_piece(m_lane + 16 * mi + v, n_lane >> 5, e.T >> 5) * 32 + (n_lane & 31)) = o;
        }
      }
    }
  }
};

// 2:4 backward, pointwise part (Fig. 4 caption; Sec. 2, last paragraph): acc = dH[t][f]; on the positions
// the forward kept, dZ = dH * 2 sqrt(h); elsewhere dZ = 0 and nothing is stored.  Output is compressed with
// the forward's metadata: dZc [T][F/2].  Hc, meta and dZc are in panel form: one piece per lane and token.
struct EpiDGather {
  struct Args { const __bf16* Hc; const uint8_t* meta; __bf16* dZc; int F; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneSaved24 sv;
    sv.load(e.Hc, e.meta, e.F, m_lane, n_lane);
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      size_t t = (size_t)(n_lane + ni);
      size_t piece = a24_piece((int)t, m_lane >> 6, e.F >> 6);
      const u32x2 mt = sv.mt[ni];
      __bf16* zrow = e.dZc + piece * 32;
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        const u32x4 h = sv.h[ni][mi];
        u32x4 z;
#pragma unroll
        for (int a = 0; a < 4; a++) {
          int gi = 4 * mi + a;
          uint32_t n4 = (mt[gi >> 3] >> (4 * (gi & 7))) & 15u;
          uint32_t i0 = n4 & 3u, i1 = n4 >> 2;
          float x0 = acc[mi][ni][4 * a], x1 = acc[mi][ni][4 * a + 1], x2 = acc[mi][ni][4 * a + 2], x3 = acc[mi][ni][4 * a + 3];
          float s0 = i0 == 0 ? x0 : (i0 == 1 ? x1 : x2);
          float s1 = i1 == 3 ? x3 : (i1 == 2 ? x2 : x1);
          float g0 = 2.f * __builtin_amdgcn_sqrtf(bf16_lo_to_f32(h[a]));
          float g1 = 2.f * __builtin_amdgcn_sqrtf(bf16_hi_to_f32(h[a]));
          z[a] = pack_bf16x2(s0 * g0, s1 * g1);
        }
        *reinterpret_cast<u32x4*>(zrow + 8 * mi) = z;
      }
    }
  }
};

// ------------------------------------------------------------------------------------------------
// fp8 (e4m3) forward: per-tensor scales; order of Sec. 2: activation, sparsification, then FP8 quantisation
// ------------------------------------------------------------------------------------------------

// Saturating round-to-nearest-even conversion of two floats to e4m3 (the conversion instruction alone turns values
// beyond the format's largest finite number, 448, into NaN codes).
__device__ __forceinline__ uint32_t cvt_e4m3x2(float lo, float hi, uint32_t old, bool high_half) {
  lo = __builtin_fminf(__builtin_fmaxf(lo, -448.f), 448.f);
  hi = __builtin_fminf(__builtin_fmaxf(hi, -448.f), 448.f);
  return high_half ? (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(lo, hi, (int)old, true)
                   : (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(lo, hi, (int)old, false);
}

// fp8 up-projection: z = zscale * acc + b1 (zscale = sx * sw1); h = bf16(max(0, z)^2); the keep-2-of-4 pick is made on
// the bf16 words exactly as in EpiPrune24; the kept values are then quantised, e4m3(h / sh).
//   Hc8, meta: panel form of the fp8 operand: piece = 64 stored bytes + 16 metadata bytes for 128 features of a token;
//   a lane's 64 features are one half of a piece.
//   Hc16, meta16 (optional, a training context): the kept values before quantisation, bf16, with their metadata, in the
//   bf16 panel form -- what the backward takes the activation's derivative from (the e4m3 code of h keeps 4
//   significant bits, too few for 2 sqrt(h)).
struct EpiPrune24F8 {
  struct Args { uint8_t* Hc8; uint8_t* meta; __bf16* Hdbg; const float* b1; int F; float zscale; float sh; __bf16* Hc16; uint8_t* meta16; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneVec64 lb;
    lb.load(e.b1, m_lane, 0.f);
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      size_t t = (size_t)(n_lane + ni);
      uint32_t q8[8];
      uint32_t nib[2] = {0u, 0u};
      size_t piece16 = a24_piece((int)t, m_lane >> 6, e.F >> 6);
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        uint32_t hpk[8];
#pragma unroll
        for (int d = 0; d < 8; d++) {
          float b0 = lb.at(16 * mi + 2 * d), b1v = lb.at(16 * mi + 2 * d + 1);
          float r0 = fmaxf(acc[mi][ni][2 * d] * e.zscale + b0, 0.f);
          float r1 = fmaxf(acc[mi][ni][2 * d + 1] * e.zscale + b1v, 0.f);
          hpk[d] = pack_bf16x2(r0 * r0, r1 * r1);
        }
        if (e.Hdbg) {
          __bf16* row = e.Hdbg + t * e.F + m_lane + 16 * mi;
          *reinterpret_cast<u32x4*>(row) = u32x4{hpk[0], hpk[1], hpk[2], hpk[3]};
          *reinterpret_cast<u32x4*>(row + 8) = u32x4{hpk[4], hpk[5], hpk[6], hpk[7]};
        }
        uint32_t pairs[4];
#pragma unroll
        for (int a = 0; a < 4; a++) {
          uint32_t pair;
          uint32_t n4 = pick24_packed(hpk[2 * a], hpk[2 * a + 1], pair);
          pairs[a] = pair;
          int gi = 4 * mi + a;
          float v0 = bf16_lo_to_f32(pair) / e.sh;
          float v1 = bf16_hi_to_f32(pair) / e.sh;
          // group gi's two stored bytes are bytes 2 gi, 2 gi + 1 of the lane's 32
          q8[gi >> 1] = cvt_e4m3x2(v0, v1, (gi & 1) ? q8[gi >> 1] : 0u, (gi & 1) != 0);
          nib[gi >> 3] |= n4 << (4 * (gi & 7));
        }
        if (e.Hc16) *reinterpret_cast<u32x4*>(e.Hc16 + piece16 * 32 + 8 * mi) = u32x4{pairs[0], pairs[1], pairs[2], pairs[3]};
      }
      size_t piece = a24_piece((int)t, m_lane >> 7, e.F >> 7);
      int half = (m_lane >> 6) & 1;
      uint8_t* hrow = e.Hc8 + piece * 64 + 32 * half;
      *reinterpret_cast<u32x4*>(hrow) = u32x4{q8[0], q8[1], q8[2], q8[3]};
      *reinterpret_cast<u32x4*>(hrow + 16) = u32x4{q8[4], q8[5], q8[6], q8[7]};
      *reinterpret_cast<u32x2*>(e.meta + piece * 16 + 8 * half) = u32x2{nib[0], nib[1]};
      if (e.Hc16) *reinterpret_cast<u32x2*>(e.meta16 + piece16 * 8) = u32x2{nib[0], nib[1]};
    }
  }
};

// fp8 backward, pointwise part (the abstract's FP8 backward pass; Sec. 2's fused backward pointwise step with its FP8
// scaling): acc = (W2_8 . dY8) for a lane's 64 features x 4 tokens; dH = scale * acc (scale = sdy * sw2); on the
// positions the forward kept dZ = dH * 2 sqrt(h) with h the bf16 kept value the forward saved (Hc16, meta16: bf16 panel
// form); the result is quantised, e4m3(dZ / sdz) (saturating), and stored compressed with the forward's metadata in
// the fp8 panel form (the operand of the sparse dX GEMM).
struct EpiDGatherF8 {
  struct Args { const __bf16* Hc16; const uint8_t* meta16; uint8_t* dZc8; int F; float scale; float sdz; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneSaved24 sv;
    sv.load(e.Hc16, e.meta16, e.F, m_lane, n_lane);
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      size_t t = (size_t)(n_lane + ni);
      const u32x2 mt = sv.mt[ni];
      uint32_t q8[8];
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        const u32x4 h = sv.h[ni][mi];
#pragma unroll
        for (int a = 0; a < 4; a++) {
          int gi = 4 * mi + a;
          uint32_t n4 = (mt[gi >> 3] >> (4 * (gi & 7))) & 15u;
          uint32_t i0 = n4 & 3u, i1 = n4 >> 2;
          float x0 = acc[mi][ni][4 * a], x1 = acc[mi][ni][4 * a + 1], x2 = acc[mi][ni][4 * a + 2], x3 = acc[mi][ni][4 * a + 3];
          float s0 = i0 == 0 ? x0 : (i0 == 1 ? x1 : x2);
          float s1 = i1 == 3 ? x3 : (i1 == 2 ? x2 : x1);
          float g0 = 2.f * __builtin_amdgcn_sqrtf(bf16_lo_to_f32(h[a]));
          float g1 = 2.f * __builtin_amdgcn_sqrtf(bf16_hi_to_f32(h[a]));
          float v0 = (s0 * e.scale * g0) / e.sdz, v1 = (s1 * e.scale * g1) / e.sdz;
          q8[gi >> 1] = cvt_e4m3x2(v0, v1, (gi & 1) ? q8[gi >> 1] : 0u, (gi & 1) != 0);
        }
      }
      size_t piece = a24_piece((int)t, m_lane >> 7, e.F >> 7);
      uint8_t* zrow = e.dZc8 + piece * 64 + 32 * ((m_lane >> 6) & 1);
      *reinterpret_cast<u32x4*>(zrow) = u32x4{q8[0], q8[1], q8[2], q8[3]};
      *reinterpret_cast<u32x4*>(zrow + 16) = u32x4{q8[4], q8[5], q8[6], q8[7]};
    }
  }
};

// out[n][m] = bf16(scale * acc), m contiguous: the transposing store of EpiColMajor with a scale (fp8 dW1).
struct EpiColMajorScaled {
  static constexpr bool STAGED = true;
  struct Args { __bf16* C; int ldc; float scale; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane, char* wbuf) {
    const int lane = threadIdx.x & 63, rho = lane & 31, h = lane >> 5;
#pragma unroll
    for (int ni = 0; ni < 4; ni++)
#pragma unroll
      for (int mi = 0; mi < 4; mi++)
#pragma unroll
        for (int q = 0; q < 2; q++) {
          u32x4 o;
#pragma unroll
          for (int d = 0; d < 4; d++) o[d] = pack_bf16x2(acc[mi][ni][8 * q + 2 * d] * e.scale, acc[mi][ni][8 * q + 2 * d + 1] * e.scale);
          ColMajorStage::put(wbuf, rho, ni, 8 * h + 2 * mi + q, o);
        }
    ColMajorStage::flush(wbuf, e.C + (size_t)(n_lane - 4 * rho) * e.ldc + (m_lane - 64 * h), e.ldc);
  }
};

// fp8 up-projection with ROW-WISE scaling (the paper's precision recipe, Sec. 2: "FP8 rowwise scaling"): the
// activation operand carries one scale per token, the weight one per output channel:
//   z = sx[t] sw1[f] acc + b1[f];  h = bf16(max(0, z)^2);  keep-2-of-4 as in EpiPrune24.
// The kept values cannot be quantised here -- their scale is the maximum of the whole token row, which spans many
// block tiles -- so they are written as bf16 in the bf16 panel form (Hc, meta), and every lane raises rowmax[t] (bf16
// word of the largest activation, non-negative, so integer order = value order) with one atomic per token.
// A streaming kernel then quantises with sh[t] = rowmax[t] / 448 (k_stream.hip).
// STATS: also the per-feature non-zero counts of the activation before pruning, into nnz [F] (as in EpiPrune24T).
template <bool STATS>
struct EpiPrune24RwT {
  struct Args { __bf16* Hc; uint8_t* meta; __bf16* Hdbg; const float* b1; int F; const float* sx; const float* sw1; uint32_t* rowmax; uint32_t* nnz; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    uint32_t cnt[16];
#pragma unroll
    for (int i = 0; i < 16; i++) cnt[i] = 0u;
    LaneVec64 lb, lw;
    lb.load(e.b1, m_lane, 0.f);
    lw.load(e.sw1, m_lane, 1.f);
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      size_t t = (size_t)(n_lane + ni);
      const float sxt = e.sx[t];
      uint32_t vals[16];
      uint32_t nib[2] = {0u, 0u};
      uint32_t mx = 0u;
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        uint32_t hpk[8];
#pragma unroll
        for (int d = 0; d < 8; d++) {
          float b0 = lb.at(16 * mi + 2 * d), b1v = lb.at(16 * mi + 2 * d + 1);
          float r0 = fmaxf(acc[mi][ni][2 * d] * (sxt * lw.at(16 * mi + 2 * d)) + b0, 0.f);
          float r1 = fmaxf(acc[mi][ni][2 * d + 1] * (sxt * lw.at(16 * mi + 2 * d + 1)) + b1v, 0.f);
          hpk[d] = pack_bf16x2(r0 * r0, r1 * r1);
          mx = max(mx, max(hpk[d] & 0xFFFFu, hpk[d] >> 16));
          if constexpr (STATS) nnz_count(cnt, hpk[d], mi, d);
        }
        if (e.Hdbg) {
          __bf16* row = e.Hdbg + t * e.F + m_lane + 16 * mi;
          *reinterpret_cast<u32x4*>(row) = u32x4{hpk[0], hpk[1], hpk[2], hpk[3]};
          *reinterpret_cast<u32x4*>(row + 8) = u32x4{hpk[4], hpk[5], hpk[6], hpk[7]};
        }
#pragma unroll
        for (int a = 0; a < 4; a++) {
          uint32_t pair;
          uint32_t n4 = pick24_packed(hpk[2 * a], hpk[2 * a + 1], pair);
          int gi = 4 * mi + a;
          vals[gi] = pair;
          nib[gi >> 3] |= n4 << (4 * (gi & 7));
        }
      }
      size_t piece = a24_piece((int)t, m_lane >> 6, e.F >> 6);
      __bf16* hrow = e.Hc + piece * 32;
#pragma unroll
      for (int q = 0; q < 4; q++)
        *reinterpret_cast<u32x4*>(hrow + 8 * q) = u32x4{vals[4 * q], vals[4 * q + 1], vals[4 * q + 2], vals[4 * q + 3]};
      *reinterpret_cast<u32x2*>(e.meta + piece * 8) = u32x2{nib[0], nib[1]};
      if (mx) atomicMax(e.rowmax + t, mx);
    }
    if constexpr (STATS) nnz_flush(cnt, e.nnz, m_lane);
  }
};
using EpiPrune24Rw = EpiPrune24RwT<false>;

// Dense fp8 up-projection with ROW-WISE scaling (the baseline the paper's forward benchmark compares with: all FP8 GEMMs of
// both sides use row-wise scales): z = sx[t] sw1[f] acc + b1[f];  h = bf16(max(0, z)^2), every one of them stored, as the
// bf16 [T][F] operand in dense panel form (64-byte pieces of 32 k); rowmax[t] is raised to the row's largest word.  A
// streaming kernel then quantises each row with sh[t] = rowmax[t] / 448.
// Ht16 (optional, a training context): the same values once more as the bf16 [F][T] operand (dense panel form, K = T) that the
// backward quantises per hidden feature for its dW2 GEMM.
struct EpiRelu2Rw {
  struct Args { __bf16* H16; const float* b1; int F; const float* sx; const float* sw1; uint32_t* rowmax; __bf16* Ht16; int T; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneVec64 lb, lw;
    lb.load(e.b1, m_lane, 0.f);
    lw.load(e.sw1, m_lane, 1.f);
    uint32_t mx[4] = {0u, 0u, 0u, 0u};
    float sxt[4];
#pragma unroll
    for (int ni = 0; ni < 4; ni++) sxt[ni] = e.sx[n_lane + ni];
#pragma unroll
    for (int mi = 0; mi < 4; mi++) {
#pragma unroll
      for (int ni = 0; ni < 4; ni++) {
        const int t = n_lane + ni;
        int f = m_lane + 16 * mi;
        __bf16* row = e.H16 + a24_piece(t, f >> 5, e.F >> 5) * 32 + (f & 31);
#pragma unroll
        for (int q = 0; q < 2; q++) {
          u32x4 o;
#pragma unroll
          for (int d = 0; d < 4; d++) {
            int i = 16 * mi + 8 * q + 2 * d;
            float r0 = fmaxf(acc[mi][ni][8 * q + 2 * d] * (sxt[ni] * lw.at(i)) + lb.at(i), 0.f);
            float r1 = fmaxf(acc[mi][ni][8 * q + 2 * d + 1] * (sxt[ni] * lw.at(i + 1)) + lb.at(i + 1), 0.f);
            acc[mi][ni][8 * q + 2 * d] = r0 * r0;
            acc[mi][ni][8 * q + 2 * d + 1] = r1 * r1;
            o[d] = pack_bf16x2(r0 * r0, r1 * r1);
            mx[ni] = max(mx[ni], max(o[d] & 0xFFFFu, o[d] >> 16));
          }
          *reinterpret_cast<u32x4*>(row + 8 * q) = o;
        }
      }
      if (e.Ht16) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          u32x2 o;
          o[0] = pack_bf16x2(acc[mi][0][v], acc[mi][1][v]);
          o[1] = pack_bf16x2(acc[mi][2][v], acc[mi][3][v]);
          *reinterpret_cast<u32x2*>(e.Ht16 + a24_piece(m_lane + 16 * mi + v, n_lane >> 5, e.T >> 5) * 32 + (n_lane & 31)) = o;
        }
      }
    }
#pragma unroll
    for (int ni = 0; ni < 4; ni++) if (mx[ni]) atomicMax(e.rowmax + n_lane + ni, mx[ni]);
  }
};

// Dense fp8 backward with ROW-WISE scaling, pointwise part: dH = rs[f] cs[t] acc (rs = the scale of each hidden feature's row of W2,
// cs = the scale of each token's row of dY);  dZ = bf16(dH * 2 sqrt(h)), h the bf16 activation the dense forward kept (H16, dense
// bf16 panel form), at every position.  Stored in bf16 twice, as the [T][F] and the [F][T] operand (dense panel forms) that
// streaming kernels then quantise per token and per hidden feature; rowmax[t] is raised to the largest magnitude word of the row.
struct EpiDReluRw {
  struct Args { const __bf16* H16; __bf16* dZ16; __bf16* dZt16; int F; int T; const float* rs; const float* cs; uint32_t* rowmax; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneVec64 lr;
    lr.load(e.rs, m_lane, 1.f);
    uint32_t mx[4] = {0u, 0u, 0u, 0u};
    float cs[4];
#pragma unroll
    for (int ni = 0; ni < 4; ni++) cs[ni] = e.cs[n_lane + ni];
    LaneSavedDense sv;
    sv.load(e.H16, e.F, m_lane, n_lane);
#pragma unroll
    for (int mi = 0; mi < 4; mi++) {
#pragma unroll
      for (int ni = 0; ni < 4; ni++) {
        int f = m_lane + 16 * mi;
        size_t o = a24_piece(n_lane + ni, f >> 5, e.F >> 5) * 32 + (f & 31);
#pragma unroll
        for (int q = 0; q < 2; q++) {
          const u32x4 h = sv.h[mi][ni][q];
          u32x4 r;
#pragma unroll
          for (int d = 0; d < 4; d++) {
            int i = 16 * mi + 8 * q + 2 * d;
            float g0 = 2.f * __builtin_amdgcn_sqrtf(bf16_lo_to_f32(h[d]));
            float g1 = 2.f * __builtin_amdgcn_sqrtf(bf16_hi_to_f32(h[d]));
            acc[mi][ni][8 * q + 2 * d] *= (cs[ni] * lr.at(i)) * g0;
            acc[mi][ni][8 * q + 2 * d + 1] *= (cs[ni] * lr.at(i + 1)) * g1;
            r[d] = pack_bf16x2(acc[mi][ni][8 * q + 2 * d], acc[mi][ni][8 * q + 2 * d + 1]);
            mx[ni] = max(mx[ni], max(r[d] & 0x7FFFu, (r[d] >> 16) & 0x7FFFu));
          }
          *reinterpret_cast<u32x4*>(e.dZ16 + o + 8 * q) = r;
        }
      }
#pragma unroll
      for (int v = 0; v < 16; v++) {
        u32x2 o;
        o[0] = pack_bf16x2(acc[mi][0][v], acc[mi][1][v]);
        o[1] = pack_bf16x2(acc[mi][2][v], acc[mi][3][v]);
        *reinterpret_cast<u32x2*>(e.dZt16 + a24_piece(m_lane + 16 * mi + v, n_lane >> 5, e.T >> 5) * 32 + (n_lane & 31)) = o;
      }
    }
#pragma unroll
    for (int ni = 0; ni < 4; ni++) if (mx[ni]) atomicMax(e.rowmax + n_lane + ni, mx[ni]);
  }
};

// C[m][n] = bf16(acc * rs[m] * cs[n]), n contiguous (row-wise-scaled fp8 down-projection: rs = sh per token, cs = sw2).
struct EpiRowMajorRowCol {
  struct Args { __bf16* C; int ldc; const float* rs; const float* cs; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    const f32x4 cs = *reinterpret_cast<const f32x4*>(e.cs + n_lane);
    LaneVec64 lr;                                  // the lane's 64 row scales: 16 loads of 16 bytes, not 64 of 4
    lr.load(e.rs, m_lane, 1.f);
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const float r = lr.at(16 * mi + v);
        u32x2 o;
        o[0] = pack_bf16x2(acc[mi][0][v] * r * cs[0], acc[mi][1][v] * r * cs[1]);
        o[1] = pack_bf16x2(acc[mi][2][v] * r * cs[2], acc[mi][3][v] * r * cs[3]);
        *reinterpret_cast<u32x2*>(e.C + (size_t)(m_lane + 16 * mi + v) * e.ldc + n_lane) = o;
      }
  }
};

// C[rowmap[m]][n] = bf16(acc * rs[m] * cs[n]): the split weight-gradient GEMMs of the row-wise fp8 backward (rows are positions
// of the permuted feature space, rs their scales in that order; each row goes back to its feature).
struct EpiRowMajorRowColMapped {
  struct Args { __bf16* C; int ldc; const float* rs; const float* cs; const int* rowmap; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    const f32x4 cs = *reinterpret_cast<const f32x4*>(e.cs + n_lane);
    LaneVec64 lr;
    lr.load(e.rs, m_lane, 1.f);
    LaneIdx64 rows;
    rows.load(e.rowmap, m_lane);
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const float r = lr.at(16 * mi + v);
        u32x2 o;
        o[0] = pack_bf16x2(acc[mi][0][v] * r * cs[0], acc[mi][1][v] * r * cs[1]);
        o[1] = pack_bf16x2(acc[mi][2][v] * r * cs[2], acc[mi][3][v] * r * cs[3]);
        *reinterpret_cast<u32x2*>(e.C + (size_t)rows.at(16 * mi + v) * e.ldc + n_lane) = o;
      }
  }
};

// C stored transposed, out[n][m] = bf16(acc * rs[m] * cs[n]) with m contiguous (row-wise-scaled fp8 dW1 GEMM: rs = the scale of
// each hidden feature's row of the transposed dZ operand, cs = the scale of each model dimension's row of the transposed X).
struct EpiColMajorRowCol {
  static constexpr bool STAGED = true;
  struct Args { __bf16* C; int ldc; const float* rs; const float* cs; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane, char* wbuf) {
    const int lane = threadIdx.x & 63, rho = lane & 31, h = lane >> 5;
    LaneVec64 lr;
    lr.load(e.rs, m_lane, 1.f);
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      const float cs = e.cs[n_lane + ni];
#pragma unroll
      for (int mi = 0; mi < 4; mi++)
#pragma unroll
        for (int q = 0; q < 2; q++) {
          u32x4 o;
#pragma unroll
          for (int d = 0; d < 4; d++) {
            int i = 16 * mi + 8 * q + 2 * d;
            o[d] = pack_bf16x2(acc[mi][ni][8 * q + 2 * d] * lr.at(i) * cs, acc[mi][ni][8 * q + 2 * d + 1] * lr.at(i + 1) * cs);
          }
          ColMajorStage::put(wbuf, rho, ni, 8 * h + 2 * mi + q, o);
        }
    }
    ColMajorStage::flush(wbuf, e.C + (size_t)(n_lane - 4 * rho) * e.ldc + (m_lane - 64 * h), e.ldc);
  }
};

// fp8 backward with ROW-WISE scaling, pointwise part (Sec. 2: the fused backward pointwise step with its FP8 scaling; the
// precision recipe of the paper's benchmarks scales every FP8 GEMM row-wise): acc = (W2_8r . dY8r) for a lane's 64 features x
// 4 tokens; dH = rs[f] cs[t] acc (rs = the scale of each hidden feature's row of W2, cs = the scale of each token's row of dY);
// on the positions the forward kept dZ = dH * 2 sqrt(h), h the bf16 kept value the forward saved (Hc16, meta16: bf16 panel form).
// Like the activation in the row-wise forward, dZ cannot be quantised here -- the scale of a token row spans many block tiles
// -- so it is written as bf16, compressed with the forward's metadata (dZc16, bf16 panel form), and every lane raises
// rowmax[t] to the largest magnitude word of its part of the row; a streaming kernel then quantises with rowmax[t] / 448.
struct EpiDGatherRw {
  struct Args { const __bf16* Hc16; const uint8_t* meta16; __bf16* dZc16; int F; const float* rs; const float* cs; uint32_t* rowmax; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneVec64 lr;
    lr.load(e.rs, m_lane, 1.f);
    LaneSaved24 sv;
    sv.load(e.Hc16, e.meta16, e.F, m_lane, n_lane);
    float csv[4];
#pragma unroll
    for (int ni = 0; ni < 4; ni++) csv[ni] = e.cs[n_lane + ni];
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      size_t t = (size_t)(n_lane + ni);
      const float cs = csv[ni];
      size_t piece = a24_piece((int)t, m_lane >> 6, e.F >> 6);
      const u32x2 mt = sv.mt[ni];
      __bf16* zrow = e.dZc16 + piece * 32;
      uint32_t mx = 0u;
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        const u32x4 h = sv.h[ni][mi];
        u32x4 z;
#pragma unroll
        for (int a = 0; a < 4; a++) {
          int gi = 4 * mi + a;
          uint32_t n4 = (mt[gi >> 3] >> (4 * (gi & 7))) & 15u;
          uint32_t i0 = n4 & 3u, i1 = n4 >> 2;
          float x0 = acc[mi][ni][4 * a] * (cs * lr.at(16 * mi + 4 * a)), x1 = acc[mi][ni][4 * a + 1] * (cs * lr.at(16 * mi + 4 * a + 1));
          float x2 = acc[mi][ni][4 * a + 2] * (cs * lr.at(16 * mi + 4 * a + 2)), x3 = acc[mi][ni][4 * a + 3] * (cs * lr.at(16 * mi + 4 * a + 3));
          float s0 = i0 == 0 ? x0 : (i0 == 1 ? x1 : x2);
          float s1 = i1 == 3 ? x3 : (i1 == 2 ? x2 : x1);
          float g0 = 2.f * __builtin_amdgcn_sqrtf(bf16_lo_to_f32(h[a]));
          float g1 = 2.f * __builtin_amdgcn_sqrtf(bf16_hi_to_f32(h[a]));
          z[a] = pack_bf16x2(s0 * g0, s1 * g1);
          mx = max(mx, max(z[a] & 0x7FFFu, (z[a] >> 16) & 0x7FFFu));
        }
        *reinterpret_cast<u32x4*>(zrow + 8 * mi) = z;
      }
      if (mx) atomicMax(e.rowmax + t, mx);
    }
  }
};

// fp8 dense up-projection (baseline): H8[t][f] = e4m3( bf16(max(0, zscale acc + b1)^2) / sh ), the [T][F] byte operand
// of the dense down-projection, in dense panel form (64-byte pieces of 64 k).
// H16, H8t (optional, a training context): the activation before quantisation as bf16 [T][F] (dense bf16 panel form; the
// backward takes the derivative from it) and the codes once more as the [F][T] operand of the weight-gradient GEMM that
// reduces over tokens (dense fp8 panel form).
struct EpiRelu2F8 {
  struct Args { uint8_t* H8; const float* b1; int F; float zscale; float sh; __bf16* H16; uint8_t* H8t; int T; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    LaneVec64 lb;
    lb.load(e.b1, m_lane, 0.f);
    uint32_t qs[4][16];   // the lane's codes: [token][4 features per word]
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      uint8_t* row = e.H8 + a24_piece(n_lane + ni, m_lane >> 6, e.F >> 6) * 64;   // a lane's 64 features: one piece
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        uint32_t q[4], hp[8];
#pragma unroll
        for (int d = 0; d < 8; d++) {
          float b0 = lb.at(16 * mi + 2 * d), b1v = lb.at(16 * mi + 2 * d + 1);
          float r0 = fmaxf(acc[mi][ni][2 * d] * e.zscale + b0, 0.f);
          float r1 = fmaxf(acc[mi][ni][2 * d + 1] * e.zscale + b1v, 0.f);
          hp[d] = pack_bf16x2(r0 * r0, r1 * r1);
          q[d >> 1] = cvt_e4m3x2(bf16_lo_to_f32(hp[d]) / e.sh, bf16_hi_to_f32(hp[d]) / e.sh, (d & 1) ? q[d >> 1] : 0u, (d & 1) != 0);
        }
        *reinterpret_cast<u32x4*>(row + 16 * mi) = u32x4{q[0], q[1], q[2], q[3]};
        if (e.H16) {
          int f = m_lane + 16 * mi;
          __bf16* r16 = e.H16 + a24_piece(n_lane + ni, f >> 5, e.F >> 5) * 32 + (f & 31);
          *reinterpret_cast<u32x4*>(r16) = u32x4{hp[0], hp[1], hp[2], hp[3]};
          *reinterpret_cast<u32x4*>(r16 + 8) = u32x4{hp[4], hp[5], hp[6], hp[7]};
        }
#pragma unroll
        for (int d = 0; d < 4; d++) qs[ni][4 * mi + d] = q[d];
      }
    }
    if (e.H8t) {
      // feature m_lane + 4 w + b: its codes of the lane's 4 consecutive tokens -> one 4-byte store
#pragma unroll
      for (int w = 0; w < 16; w++)
#pragma unroll
        for (int b = 0; b < 4; b++) {
          uint32_t o = ((qs[0][w] >> (8 * b)) & 0xFFu) | (((qs[1][w] >> (8 * b)) & 0xFFu) << 8) | (((qs[2][w] >> (8 * b)) & 0xFFu) << 16) |
                       (((qs[3][w] >> (8 * b)) & 0xFFu) << 24);
          *reinterpret_cast<uint32_t*>(e.H8t + a24_piece(m_lane + 4 * w + b, n_lane >> 6, e.T >> 6) * 64 + (n_lane & 63)) = o;
        }
    }
  }
};

// Dense fp8 backward, pointwise part: acc = (W2_8 . dY8) for a lane's 64 features x 4 tokens; dZ = scale * acc * 2 sqrt(h) with h
// the bf16 activation the dense forward saved (H16, dense bf16 panel form); stored as e4m3(dZ / sdz) twice: the [T][F]
// operand of the dX GEMM and the [F][T] operand of the dW1 GEMM (dense fp8 panel forms).
struct EpiDReluF8 {
  struct Args { const __bf16* H16; uint8_t* dZ8; uint8_t* dZ8t; int F; int T; float scale; float sdz; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
    uint32_t qs[4][16];
    LaneSavedDense sv;
    sv.load(e.H16, e.F, m_lane, n_lane);
#pragma unroll
    for (int ni = 0; ni < 4; ni++) {
      uint8_t* row = e.dZ8 + a24_piece(n_lane + ni, m_lane >> 6, e.F >> 6) * 64;
#pragma unroll
      for (int mi = 0; mi < 4; mi++) {
        uint32_t q[4];
#pragma unroll
        for (int hq = 0; hq < 2; hq++) {
          const u32x4 h = sv.h[mi][ni][hq];
#pragma unroll
          for (int d = 0; d < 4; d++) {
            float g0 = 2.f * __builtin_amdgcn_sqrtf(bf16_lo_to_f32(h[d]));
            float g1 = 2.f * __builtin_amdgcn_sqrtf(bf16_hi_to_f32(h[d]));
            float v0 = (acc[mi][ni][8 * hq + 2 * d] * e.scale * g0) / e.sdz, v1 = (acc[mi][ni][8 * hq + 2 * d + 1] * e.scale * g1) / e.sdz;
            int dd = 4 * hq + d;
            q[dd >> 1] = cvt_e4m3x2(v0, v1, (dd & 1) ? q[dd >> 1] : 0u, (dd & 1) != 0);
          }
        }
        *reinterpret_cast<u32x4*>(row + 16 * mi) = u32x4{q[0], q[1], q[2], q[3]};
#pragma unroll
        for (int d = 0; d < 4; d++) qs[ni][4 * mi + d] = q[d];
      }
    }
#pragma unroll
    for (int w = 0; w < 16; w++)
#pragma unroll
      for (int b = 0; b < 4; b++) {
        uint32_t o = ((qs[0][w] >> (8 * b)) & 0xFFu) | (((qs[1][w] >> (8 * b)) & 0xFFu) << 8) | (((qs[2][w] >> (8 * b)) & 0xFFu) << 16) |
                     (((qs[3][w] >> (8 * b)) & 0xFFu) << 24);
        *reinterpret_cast<uint32_t*>(e.dZ8t + a24_piece(m_lane + 4 * w + b, n_lane >> 6, e.T >> 6) * 64 + (n_lane & 63)) = o;
      }
  }
};

// C[m][n] = bf16(scale * acc), n contiguous (fp8 down-projection: scale = sh * sw2).
struct EpiRowMajorScaled {
  struct Args { __bf16* C; int ldc; float scale; };
  static __device__ __forceinline__ void run(const Args& e, f32x16 (&acc)[4][4], int m_lane, int n_lane) {
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        u32x2 o;
        o[0] = pack_bf16x2(acc[mi][0][v] * e.scale, acc[mi][1][v] * e.scale);
        o[1] = pack_bf16x2(acc[mi][2][v] * e.scale, acc[mi][3][v] * e.scale);
        *reinterpret_cast<u32x2*>(e.C + (size_t)(m_lane + 16 * mi + v) * e.ldc + n_lane) = o;
      }
  }
};

}  // namespace ffn24
