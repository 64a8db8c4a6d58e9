// MFMA / sparse-MFMA GEMM core for gfx950 (CDNA4), bf16 operands, fp32 accumulation.
//
// One kernel template computes C[m][n] = sum_k A[m][k] * B[n][k] on a 256x256 block tile with four
// wavefronts (2x2), each owning a 128x128 wave tile = 4x4 MFMA tiles of 32x32 (256 accumulator
// registers per lane).  Operands are staged through LDS in K-contiguous rows, double buffered, one
// barrier per 64-wide K stage; the global loads of stage k+1 are in flight while stage k is computed.
//
//   A operand modes:  A_KC  dense, stored [M][K]            (K contiguous)
//                     A_MC  dense, stored [K][M]            (M contiguous; transposed in registers on the way to LDS)
//                     A_SP  2:4-compressed [M][K/2] + metadata [M][K/8]; runs on v_smfmac_f32_32x32x32_bf16
//   B operand modes:  B_KC  stored [N][K],  B_NC  stored [K][N]
//
// 2:4 operand (Sec. 1 of the paper, "Hardware-accelerated (2:4) sparsity"; Fig. 2): of every 4 consecutive
// K entries of a row only two are stored, with a 2-bit position each.  The metadata byte layout used
// throughout (nibble i0 | i1<<2 per group, even group in the low nibble) is exactly the index word the
// sparse MFMA consumes: a lane's 8 stored values of one instruction take 16 consecutive metadata bits,
// selected from a 32-bit register by the instruction's ABID field.
//
// Lane layouts of the matrix instructions (measured on gfx950 with one-hot operands):
//   dense 32x32x16:  A lane l holds row l%32, k = 8*(l/32)..+7;  B lane l holds column l%32, same k;
//                    C register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
//   sparse 32x32x32: A lane l holds row l%32 and the 8 stored values of dense k 16*(l/32)..+15;
//                    B lane l holds column l%32, registers 0..7 = k 8*(l/32)..+7, registers 8..15 = k 16+8*(l/32)..+7.
//
// Row remapping.  Which global row sits in which MFMA-tile row is free, so it is chosen to make every
// lane's accumulators contiguous in memory:  wave-tile row 64*hc + 16*mi + v belongs to lane half hc,
// M-tile mi, accumulator register v (64 consecutive rows per lane, in groups of 4 that never straddle
// lanes -- the 2:4 groups of the fused prune epilogue);  wave-tile column 4*c + ni belongs to lane
// column c, N-tile ni (4 consecutive columns per lane).  The permutation is applied once, when a tile
// is written to LDS, so fragment reads stay linear.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <utility>

namespace ffn24 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int TILE_M = 256, TILE_N = 256, TILE_K = 64, GEMM_THREADS = 256;

enum { A_KC = 0, A_MC = 1, A_SP = 2 };
enum { B_KC = 0, B_NC = 1 };

struct GemmArgs {
  const void* A;         // see modes above
  const uint8_t* Ameta;  // A_SP only
  const void* B;
  int M, N, K;           // K is the dense reduction length
};

// LDS bytes per stage for each operand form
constexpr int LDS_DENSE = 256 * 128;     // 256 rows x 64 k x 2 B
constexpr int LDS_COMP = 256 * 64;       // 256 rows x 32 stored values x 2 B
constexpr int LDS_META = 256 * 8;        // 256 rows x 8 metadata bytes
constexpr int lds_stage_bytes(int amode) { return (amode == A_SP ? LDS_COMP + LDS_META : LDS_DENSE) + LDS_DENSE; }
constexpr int lds_total_bytes(int amode) { return 2 * lds_stage_bytes(amode); }

// block-tile row index (0..255) -> LDS row, M side and N side
__device__ __forceinline__ int perm_m(int g) {
  int wm = g & 127;
  return (g & 128) | (((wm >> 4) & 3) << 5) | (((wm >> 2) & 3) << 3) | (((wm >> 6) & 1) << 2) | (wm & 3);
}
__device__ __forceinline__ int perm_n(int g) {
  int wn = g & 127;
  return (g & 128) | ((wn & 3) << 5) | (wn >> 2);
}
// 16-byte chunk swizzles: conflict-free for 8 and for 16 consecutive rows reading the same logical chunk
__device__ __forceinline__ int swz8(int p) { return (p ^ (p >> 3)) & 7; }          // 128-byte rows
__device__ __forceinline__ int swz4(int p) { return ((p >> 1) ^ (p >> 3)) & 3; }   // 64-byte rows

// ------------------------------------------------------------------------------------------------
// global -> register -> LDS stagers
// ------------------------------------------------------------------------------------------------

// dense, K contiguous in memory: tile = 256 rows x 64 k.  Thread t: chunk t%8 of rows t/8 + 32 j.
template <bool MSIDE>
struct StageKC {
  u32x4 r[8];
  const char* g;
  size_t jstride;  // bytes between rows 32 apart
  int off[8];
  __device__ __forceinline__ void init(const void* base, int row0, int K, int tid) {
    int chunk = tid & 7, row = tid >> 3;
    g = static_cast<const char*>(base) + ((size_t)(row0 + row) * K + chunk * 8) * 2;
    jstride = (size_t)32 * K * 2;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      int p = MSIDE ? perm_m(row + 32 * j) : perm_n(row + 32 * j);
      off[j] = p * 128 + ((chunk ^ swz8(p)) << 4);
    }
  }
  static constexpr int NLOAD = 8, NSTORE = 8;
  template <int J> __device__ __forceinline__ void load1(int kt) {
    r[J] = *reinterpret_cast<const u32x4*>(g + (size_t)kt * (TILE_K * 2) + J * jstride);
  }
  template <int J> __device__ __forceinline__ void store1(char* lds) { *reinterpret_cast<u32x4*>(lds + off[J]) = r[J]; }
  __device__ __forceinline__ void load(int kt) {
    const char* p = g + (size_t)kt * (TILE_K * 2);
#pragma unroll
    for (int j = 0; j < 8; j++) r[j] = *reinterpret_cast<const u32x4*>(p + j * jstride);
  }
  __device__ __forceinline__ void store(char* lds) {
#pragma unroll
    for (int j = 0; j < 8; j++) *reinterpret_cast<u32x4*>(lds + off[j]) = r[j];
  }
};

// dense, M (or N) contiguous in memory: stored [K][ld].  Thread t owns the 8(k) x 8(mn) block
// kb = t%8, nb = t/8, loads its 8 rows of 16 bytes and transposes them in registers.
template <bool MSIDE>
struct StageMC {
  u32x4 r[8];
  const char* g;
  size_t kstride;  // bytes between consecutive k rows
  int off[8];
  __device__ __forceinline__ void init(const void* base, int col0, int ld, int tid) {
    int kb = tid & 7, nb = tid >> 3;
    g = static_cast<const char*>(base) + ((size_t)(8 * kb) * ld + col0 + 8 * nb) * 2;
    kstride = (size_t)ld * 2;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      int p = MSIDE ? perm_m(8 * nb + j) : perm_n(8 * nb + j);
      off[j] = p * 128 + ((kb ^ swz8(p)) << 4);
    }
  }
  static constexpr int NLOAD = 8, NSTORE = 8;
  template <int I> __device__ __forceinline__ void load1(int kt) {
    r[I] = *reinterpret_cast<const u32x4*>(g + ((size_t)kt * TILE_K + I) * kstride);
  }
  // column J of the 8x8 block: dword d = (r[2d] half J, r[2d+1] half J) -- an 8x8 transpose of 16-bit elements
  template <int J> __device__ __forceinline__ void store1(char* lds) {
    u32x4 o;
#pragma unroll
    for (int d = 0; d < 4; d++) {
      uint32_t lo = r[2 * d][J >> 1], hi = r[2 * d + 1][J >> 1];
      o[d] = (J & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
    }
    *reinterpret_cast<u32x4*>(lds + off[J]) = o;
  }
  __device__ __forceinline__ void load(int kt) {
    load1<0>(kt); load1<1>(kt); load1<2>(kt); load1<3>(kt); load1<4>(kt); load1<5>(kt); load1<6>(kt); load1<7>(kt);
  }
  __device__ __forceinline__ void store(char* lds) {
    store1<0>(lds); store1<1>(lds); store1<2>(lds); store1<3>(lds); store1<4>(lds); store1<5>(lds); store1<6>(lds); store1<7>(lds);
  }
};

// 2:4-compressed A: values [M][K/2] (64 bytes per row and stage), metadata [M][K/8] (8 bytes per row and stage)
struct StageSP {
  u32x4 r[4];
  u32x2 m;
  const char* g;
  const char* gm;
  size_t jstride;
  int off[4];
  int moff;
  __device__ __forceinline__ void init(const void* vals, const uint8_t* meta, int row0, int K, int tid) {
    int chunk = tid & 3, row = tid >> 2;
    g = static_cast<const char*>(vals) + ((size_t)(row0 + row) * (K / 2) + chunk * 8) * 2;
    jstride = (size_t)64 * (K / 2) * 2;
    gm = reinterpret_cast<const char*>(meta) + (size_t)(row0 + tid) * (K / 8);
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int p = perm_m(row + 64 * j);
      off[j] = p * 64 + ((chunk ^ swz4(p)) << 4);
    }
    moff = LDS_COMP + perm_m(tid) * 8;
  }
  static constexpr int NLOAD = 5, NSTORE = 5;
  template <int J> __device__ __forceinline__ void load1(int kt) {
    if constexpr (J < 4) r[J] = *reinterpret_cast<const u32x4*>(g + (size_t)kt * (TILE_K / 2 * 2) + J * jstride);
    else m = *reinterpret_cast<const u32x2*>(gm + (size_t)kt * (TILE_K / 8));
  }
  template <int J> __device__ __forceinline__ void store1(char* lds) {
    if constexpr (J < 4) *reinterpret_cast<u32x4*>(lds + off[J]) = r[J];
    else *reinterpret_cast<u32x2*>(lds + moff) = m;
  }
  __device__ __forceinline__ void load(int kt) { load1<0>(kt); load1<1>(kt); load1<2>(kt); load1<3>(kt); load1<4>(kt); }
  __device__ __forceinline__ void store(char* lds) { store1<0>(lds); store1<1>(lds); store1<2>(lds); store1<3>(lds); store1<4>(lds); }
};

template <int AMODE> struct AStager;
template <> struct AStager<A_KC> : StageKC<true> {
  __device__ __forceinline__ void setup(const GemmArgs& a, int m0, int tid) { init(a.A, m0, a.K, tid); }
};
template <> struct AStager<A_MC> : StageMC<true> {
  __device__ __forceinline__ void setup(const GemmArgs& a, int m0, int tid) { init(a.A, m0, a.M, tid); }
};
template <> struct AStager<A_SP> : StageSP {
  __device__ __forceinline__ void setup(const GemmArgs& a, int m0, int tid) { init(a.A, a.Ameta, m0, a.K, tid); }
};
template <int BMODE> struct BStager;
template <> struct BStager<B_KC> : StageKC<false> {
  __device__ __forceinline__ void setup(const GemmArgs& a, int n0, int tid) { init(a.B, n0, a.K, tid); }
};
template <> struct BStager<B_NC> : StageMC<false> {
  __device__ __forceinline__ void setup(const GemmArgs& a, int n0, int tid) { init(a.B, n0, a.N, tid); }
};

// ------------------------------------------------------------------------------------------------
// per-stage compute
// ------------------------------------------------------------------------------------------------

struct LaneCtx {
  int rho, h;      // lane & 31, lane >> 5
  int wy, wx;      // wave row / column inside the block tile
  int a_row_off;   // byte offset of LDS row (wy*128 + rho) for 128-byte rows
  int b_row_off;   // same for the B tile
  int fsw;         // swz8 of the lane's row with mi = 0
};

// compile-time loop: f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N-1>)
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) { (f(std::integral_constant<int, Is>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// Nothing may be moved across this point by the instruction scheduler.  The main loop is written as a sequence of
// slots {one matrix op + the memory ops that ride on it}, fenced from each other, so the issue order is the source order.
#define FFN24_FENCE() __builtin_amdgcn_sched_barrier(0)

// MFMA fragments of one K step.  Dense: 16-wide step, 4 A + 4 B fragments of 8 bf16.
struct FragD {
  bf16x8 a[4], b[4];
};

// fragment I of K step s: I < 4 -> a[I], else b[I-4]
template <int I>
__device__ __forceinline__ void load_frag_dense1(const char* sA, const char* sB, const LaneCtx& L, int s, FragD& f) {
  int c = 2 * s + L.h;
  constexpr int i = I & 3;
  int sw = L.fsw ^ ((i & 1) << 2);
  if constexpr (I < 4) f.a[i] = *reinterpret_cast<const bf16x8*>(sA + L.a_row_off + i * (32 * 128) + ((c ^ sw) << 4));
  else f.b[i] = *reinterpret_cast<const bf16x8*>(sB + L.b_row_off + i * (32 * 128) + ((c ^ sw) << 4));
}

template <int M>
__device__ __forceinline__ void mfma_dense1(const FragD& f, f32x16 (&acc)[4][4]) {
  constexpr int mi = M >> 2, ni = M & 3;
  acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mi], f.b[ni], acc[mi][ni], 0, 0, 0);
}

// Sparse: the stage's K window of 64 = four 16-wide windows w.  Instruction S (0,1) gives lane half q the window
// 2q+S, so a lane's two instructions use 32 consecutive stored-value bytes and one 32-bit metadata word (ABID = S
// picks the half).  B lane half h then needs, for instruction S, the 8-k chunks 2S+h (registers 0..7) and 4+2S+h
// (registers 8..15).
struct FragS {
  bf16x8 a[4];
  bf16x8 blo[4], bhi[4];
};

template <int I>
__device__ __forceinline__ void load_idx_sparse1(const char* sA, const LaneCtx& L, uint32_t (&idx)[4]) {
  int p = L.wy * 128 + L.rho;
  idx[I] = *reinterpret_cast<const uint32_t*>(sA + LDS_COMP + (p + 32 * I) * 8 + 4 * L.h);
}

// fragment I of instruction S: I < 4 -> a[I]; 4..7 -> low half of b[I-4]; 8..11 -> high half of b[I-8]
template <int S, int I>
__device__ __forceinline__ void load_frag_sparse1(const char* sAc, const char* sB, const LaneCtx& L, FragS& f) {
  constexpr int i = I & 3;
  if constexpr (I < 4) {
    int p = L.wy * 128 + L.rho;
    int w = 2 * L.h + S;
    f.a[i] = *reinterpret_cast<const bf16x8*>(sAc + p * 64 + i * (32 * 64) + ((w ^ swz4(p)) << 4));
  } else {
    int sw = L.fsw ^ ((i & 1) << 2);
    const char* row = sB + L.b_row_off + i * (32 * 128);
    if constexpr (I < 8) f.blo[i] = *reinterpret_cast<const bf16x8*>(row + (((2 * S + L.h) ^ sw) << 4));
    else f.bhi[i] = *reinterpret_cast<const bf16x8*>(row + (((4 + 2 * S + L.h) ^ sw) << 4));
  }
}

template <int S, int M>
__device__ __forceinline__ void mfma_sparse1(const FragS& f, const uint32_t (&idx)[4], f32x16 (&acc)[4][4]) {
  constexpr int mi = M >> 2, ni = M & 3;
  bf16x16 b = __builtin_shufflevector(f.blo[ni], f.bhi[ni], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
  acc[mi][ni] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[mi], b, acc[mi][ni], (int)idx[mi], 0, S);
}

// global load / LDS store number J of the stage: A's ops first, then B's
template <int J, class SA, class SB>
__device__ __forceinline__ void gload1(SA& sa, SB& sb, int kt) {
  if constexpr (J < SA::NLOAD) sa.template load1<J>(kt);
  else if constexpr (J < SA::NLOAD + SB::NLOAD) sb.template load1<J - SA::NLOAD>(kt);
}
template <int J, class SA, class SB>
__device__ __forceinline__ void lstore1(SA& sa, SB& sb, char* ldsA, char* ldsB) {
  if constexpr (J < SA::NSTORE) sa.template store1<J>(ldsA);
  else if constexpr (J < SA::NSTORE + SB::NSTORE) sb.template store1<J - SA::NSTORE>(ldsB);
}

// ------------------------------------------------------------------------------------------------
// the kernel
// ------------------------------------------------------------------------------------------------

// tile id -> (tile_m, tile_n).  Consecutive workgroup ids go round-robin over the 8 XCDs (each with its own L2),
// so ids are first regrouped so that each XCD works on a contiguous run of tiles, then walked in bands of
// 8 tile-rows so that a band's A rows and the B columns it sweeps stay L2-resident.
__device__ __forceinline__ void tile_coords(int ntm, int ntn, int& tm, int& tn) {
  int nb = ntm * ntn;
  int pid = blockIdx.x;
  if ((nb & 7) == 0) pid = (pid & 7) * (nb >> 3) + (pid >> 3);
  const int GROUP = 8;
  int per_group = GROUP * ntn;
  int gid = pid / per_group;
  int first = gid * GROUP;
  int gsz = min(ntm - first, GROUP);
  int in = pid - gid * per_group;
  tm = first + in % gsz;
  tn = in / gsz;
}

// Epilogue concept:  struct E { struct Args {...}; static __device__ void run(const Args&, acc, m_lane, n_lane); }
//   m_lane = global row of acc[0][*][0] for this lane (its 64 rows are m_lane + 16*mi + v),
//   n_lane = global column of acc[*][0][*] (its 4 columns are n_lane + ni).
template <int AMODE, int BMODE, class Epi>
__global__ void __launch_bounds__(GEMM_THREADS) gemm_kernel(GemmArgs g, typename Epi::Args ea) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int STAGE = lds_stage_bytes(AMODE);
  constexpr int A_BYTES = (AMODE == A_SP) ? LDS_COMP + LDS_META : LDS_DENSE;

  int tid = threadIdx.x;
  int lane = tid & 63, wave = tid >> 6;
  int tm, tn;
  tile_coords(g.M / TILE_M, g.N / TILE_N, tm, tn);
  int m0 = tm * TILE_M, n0 = tn * TILE_N;

  LaneCtx L;
  L.rho = lane & 31; L.h = lane >> 5; L.wy = wave >> 1; L.wx = wave & 1;
  L.a_row_off = (L.wy * 128 + L.rho) * 128;
  L.b_row_off = (L.wx * 128 + L.rho) * 128;
  L.fsw = (L.rho & 7) ^ (L.rho >> 3);

  AStager<AMODE> sa;
  BStager<BMODE> sb;
  sa.setup(g, m0, tid);
  sb.setup(g, n0, tid);

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;
  // Pin the accumulators to the accumulation register file: an empty asm with an AGPR constraint gives their
  // live ranges the AGPR class, so the 256 arch VGPRs stay free for fragments, prefetch and addresses.
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) asm volatile("" : "+a"(acc[i][j]));

  int nk = g.K / TILE_K;
  sa.load(0);
  sb.load(0);
  sa.store(smem);
  sb.store(smem + A_BYTES);
  __syncthreads();

  // Software pipeline, written slot by slot (one matrix op per slot, fenced).  Per stage: the global loads of the
  // next stage ride on the first matrix ops; the fragments of K step s+1 are read from LDS under the matrix ops of
  // step s; under the first half of the last step the next stage is written to the other LDS buffer; then the one
  // barrier of the stage; under the second half of the last step the first fragments of the next stage are read.
  constexpr int NL = AStager<AMODE>::NLOAD + BStager<BMODE>::NLOAD;
  constexpr int NS = AStager<AMODE>::NSTORE + BStager<BMODE>::NSTORE;
  if constexpr (AMODE == A_SP) {
    FragS f0, f1;
    uint32_t idx[4];
    static_for<4>([&](auto I) { load_idx_sparse1<I>(smem, L, idx); });
    static_for<12>([&](auto I) { load_frag_sparse1<0, I>(smem, smem + A_BYTES, L, f0); });
    auto stage = [&](int kt, auto has_next) {
      constexpr bool more = decltype(has_next)::value;
      const char* cur = smem + (kt & 1) * STAGE;
      char* nxt = smem + ((kt + 1) & 1) * STAGE;
      uint32_t idx_n[4] = {0u, 0u, 0u, 0u};
      FFN24_FENCE();
      static_for<16>([&](auto M) {
        mfma_sparse1<0, M>(f0, idx, acc);
        if constexpr (more) gload1<M>(sa, sb, kt + 1);
        if constexpr (M < 12) load_frag_sparse1<1, M>(cur, cur + A_BYTES, L, f1);
        FFN24_FENCE();
      });
      static_for<8>([&](auto M) {
        mfma_sparse1<1, M>(f1, idx, acc);
        if constexpr (more) {
          lstore1<2 * M>(sa, sb, nxt, nxt + A_BYTES);
          lstore1<2 * M + 1>(sa, sb, nxt, nxt + A_BYTES);
        }
        FFN24_FENCE();
      });
      if constexpr (more) __syncthreads();
      FFN24_FENCE();
      static_for<8>([&](auto M) {
        mfma_sparse1<1, M + 8>(f1, idx, acc);
        if constexpr (more) {
          if constexpr (M < 4) load_idx_sparse1<M>(nxt, L, idx_n);
          if constexpr (M < 6) {
            load_frag_sparse1<0, 2 * M>(nxt, nxt + A_BYTES, L, f0);
            load_frag_sparse1<0, 2 * M + 1>(nxt, nxt + A_BYTES, L, f0);
          }
        }
        FFN24_FENCE();
      });
#pragma unroll
      for (int i = 0; i < 4; i++) idx[i] = idx_n[i];
    };
    for (int kt = 0; kt < nk - 1; kt++) stage(kt, std::true_type{});
    stage(nk - 1, std::false_type{});
  } else {
    static_assert(NL == 16 && NS == 16, "dense stages issue one global load per slot of step 0");
    FragD f0, f1;
    static_for<8>([&](auto I) { load_frag_dense1<I>(smem, smem + A_BYTES, L, 0, f0); });
    auto stage = [&](int kt, auto has_next) {
      constexpr bool more = decltype(has_next)::value;
      const char* cur = smem + (kt & 1) * STAGE;
      char* nxt = smem + ((kt + 1) & 1) * STAGE;
      FFN24_FENCE();
      static_for<16>([&](auto M) {
        mfma_dense1<M>(f0, acc);
        if constexpr (more) gload1<M>(sa, sb, kt + 1);
        if constexpr (M < 8) load_frag_dense1<M>(cur, cur + A_BYTES, L, 1, f1);
        FFN24_FENCE();
      });
      static_for<16>([&](auto M) {
        mfma_dense1<M>(f1, acc);
        if constexpr (M < 8) load_frag_dense1<M>(cur, cur + A_BYTES, L, 2, f0);
        FFN24_FENCE();
      });
      static_for<16>([&](auto M) {
        mfma_dense1<M>(f0, acc);
        if constexpr (M < 8) load_frag_dense1<M>(cur, cur + A_BYTES, L, 3, f1);
        FFN24_FENCE();
      });
      static_for<8>([&](auto M) {
        mfma_dense1<M>(f1, acc);
        if constexpr (more) {
          lstore1<2 * M>(sa, sb, nxt, nxt + A_BYTES);
          lstore1<2 * M + 1>(sa, sb, nxt, nxt + A_BYTES);
        }
        FFN24_FENCE();
      });
      if constexpr (more) __syncthreads();
      FFN24_FENCE();
      static_for<8>([&](auto M) {
        mfma_dense1<M + 8>(f1, acc);
        if constexpr (more) load_frag_dense1<M>(nxt, nxt + A_BYTES, L, 0, f0);
        FFN24_FENCE();
      });
    };
    for (int kt = 0; kt < nk - 1; kt++) stage(kt, std::true_type{});
    stage(nk - 1, std::false_type{});
  }
  int m_lane = m0 + L.wy * 128 + 64 * L.h;
  int n_lane = n0 + L.wx * 128 + 4 * L.rho;
  Epi::run(ea, acc, m_lane, n_lane);
}

// ------------------------------------------------------------------------------------------------
// small device helpers shared by the epilogues
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = (__bf16)lo;   // round-to-nearest-even
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf16_lo_to_f32(uint32_t pk) { return __builtin_bit_cast(float, pk << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t pk) { return __builtin_bit_cast(float, pk & 0xFFFF0000u); }

// Keep-2-of-4 on four storage words (Sec. 2 of the paper: keep the two largest magnitudes of each block of 4;
// ties go to the lower index).  k_i = (magnitude << 2) | (3 - i) makes all four keys distinct and orders them
// by (magnitude, then lower index first), so the two largest keys are the picks.
// Returns the nibble i0 | i1<<2 and the two kept keys ordered by position (key_first has the lower index).
__device__ __forceinline__ uint32_t pick24_keys(uint32_t k0, uint32_t k1, uint32_t k2, uint32_t k3,
                                                uint32_t& key_first, uint32_t& key_second) {
  uint32_t a = max(k0, k1), b = min(k0, k1), c = max(k2, k3), d = min(k2, k3);
  uint32_t top = max(a, c);
  uint32_t e = max(b, d);
  uint32_t second = max(min(a, c), min(max(a, c), e));         // median of (a, c, e) = second largest of the four
  uint32_t ct = top & 3u, cs = second & 3u;                    // 3 - index
  bool top_first = ct > cs;                                    // larger complement = lower index
  key_first = top_first ? top : second;
  key_second = top_first ? second : top;
  uint32_t cmax = max(ct, cs), cmin = min(ct, cs);
  return (cmax | (cmin << 2)) ^ 15u;
}

}  // namespace ffn24
