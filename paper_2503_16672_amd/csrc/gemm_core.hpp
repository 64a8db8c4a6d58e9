// MFMA / sparse-MFMA GEMM core for gfx950 (CDNA4), bf16 operands, fp32 accumulation.
//
// One kernel template computes C[m][n] = sum_k A[m][k] * B[n][k]; both operands are K-contiguous in memory
// (operands that are not are transposed once by a streaming kernel, see k_stream.hip).  Block tile 256x256, four
// wavefronts (2x2), each owning a 128x128 wave tile = 4x4 MFMA tiles of 32x32: 256 accumulator registers per lane,
// pinned to the AGPR file.
//
//   A dense  : [M][K]                         -> v_mfma_f32_32x32x16_bf16
//   A sparse : 2:4-compressed [M][K/2] + metadata [M][K/8] -> v_smfmac_f32_32x32x32_bf16
//   B        : [N][K]
//
// 2:4 operand (Sec. 1 of the paper, "Hardware-accelerated (2:4) sparsity"; Fig. 2): of every 4 consecutive K entries
// of a row only two are stored, with a 2-bit position each.  The metadata byte layout used throughout (nibble
// i0 | i1<<2 per group, even group in the low nibble) is exactly the index word the sparse MFMA consumes: a lane's
// 8 stored values of one instruction take 16 consecutive metadata bits, selected from a 32-bit register by ABID.
//
// Panel form of a 2:4 operand.  The compressed operands that the library produces for itself (never the ones a
// caller hands in) are stored by pieces: piece (r, kp) = the 32 stored values (64 bytes) and the 8 metadata bytes of
// row r for the dense k range [64 kp, 64 kp + 64), at piece index ((r / 256) * (K / 64) + kp) * 256 + r % 256.
// The 256 rows x 64 k that a block tile consumes per stage are then one contiguous 16 KiB (+ 2 KiB) run, fetched as
// full 128-byte lines, instead of 256 pieces of 64 (8) bytes that are a whole matrix row apart.  Measured: the
// sparse GEMM is bound by its global->LDS stream, and the 8-byte metadata pieces alone cost it 17 %.
//
// A dense A operand can be in panel form too: piece (r, kp) = the 32 k (64 bytes) [32 kp, 32 kp + 32) of row r,
// same piece index with K / 32 panels per row (the weight copies the library makes for itself).
//
// Data movement.  Global memory goes straight to LDS (global_load_lds_dwordx4: no VGPR staging, no LDS store
// instructions) into a ring of stage buffers, 2-3 stages ahead of the math, so that L2/HBM latency is covered:
//   dense : stage = 32 k  (A 16 KiB + B 16 KiB), ring of 4  -> 128 KiB of the CU's 160 KiB LDS
//   sparse: stage = 64 k  (A 16 KiB stored values + 2 KiB metadata + B 32 KiB), ring of 3 -> 150 KiB
// A wave-level DMA instruction fills 1 KiB of LDS in lane order, so the swizzled, row-permuted LDS layout is
// produced by choosing which global 16 bytes each lane fetches.
//
// Schedule of one stage (two K steps of 16 matrix ops each), written slot by slot with scheduling fences:
//   step 0: matrix ops; the LDS fragment reads of step 1 ride on them
//   wait for the next stage's DMA, one workgroup barrier
//   step 1: matrix ops; the DMA of the stage that reuses this buffer and the fragment reads of the next stage's
//           step 0 ride on them -- the DMA instructions on every other slot only, and for the sparse stage (14 a wave) half
//           of them on the even slots of the NEXT stage's step 0 (see dma_on_step1 below)
//
// Lane layouts of the matrix instructions (measured on gfx950 with one-hot operands):
//   dense 32x32x16:  A lane l holds row l%32, k = 8*(l/32)..+7;  B lane l holds column l%32, same k;
//                    C register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
//   sparse 32x32x32: A lane l holds row l%32 and the 8 stored values of dense k 16*(l/32)..+15;
//                    B lane l holds column l%32, registers 0..7 = k 8*(l/32)..+7, registers 8..15 = k 16+8*(l/32)..+7.
//
// Row remapping.  Which global row sits in which MFMA-tile row is free, so it is chosen to make every lane's
// accumulators contiguous in memory:  wave-tile row 64*hc + 16*mi + v belongs to lane half hc, M-tile mi,
// accumulator register v (64 consecutive rows per lane, in groups of 4 that never straddle lanes -- the 2:4 groups of
// the fused prune epilogue);  wave-tile column 4*c + ni belongs to lane column c, N-tile ni (4 consecutive columns
// per lane).  The permutation is applied when a tile is brought into LDS, so fragment reads stay linear.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <utility>
#include "launch.hpp"

namespace ffn24 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(1))) const char glb_char;

constexpr int TILE_M = 256, TILE_N = 256, GEMM_THREADS = 256;
constexpr int GEMM_K_MULTIPLE = 64;   // K must be a multiple of this for both kernels

struct GemmArgs {
  const void* A;         // dense [M][K] or stored values [M][K/2]
  const uint8_t* Ameta;  // sparse only: [M][K/8]
  const void* B;         // [N][K]
  int M, N, K;           // K is the dense reduction length
  int a_panel;           // A (and its metadata) is in panel form (see above) instead of row-major
  const int* b_rowmap;   // optional: row n of B is taken from memory row b_rowmap[n] (token permutation, gathered by the DMA)
  int b_panel;           // B is in the B panel form (below) instead of row-major; not together with b_rowmap
  unsigned long long* clk;   // optional (profiling): workgroup i < CLK_SLOTS stores its own {shader-clock ticks, 100 MHz ticks} at 2 i
};

// Measurement variants of the GEMM core (bit mask; 0 = the product).  They exist so that what bounds the main loop can be
// measured with this very code -- the same DMA plan, LDS image, fragment reads and schedule -- with one ingredient taken
// out; they compute nothing useful.  Only the probe entry points of the library instantiate them.
constexpr int PROBE_NO_DMA = 1;      // no global->LDS DMA is issued (the matrix ops run on whatever the LDS holds)
constexpr int PROBE_NO_MFMA = 2;     // no matrix ops
constexpr int PROBE_NO_FRAG = 4;     // no LDS fragment reads
constexpr int PROBE_K_WRAP = 8;      // the K stages walk round the first 8 stages of the operands: every line is an L2 hit
// other tile walks (the product's is a 4 x 2 grid of 8 x 4 patches), to measure what the walk does to time and to L2 fills:
constexpr int PROBE_WALK_BANDS = 16;   // bands of 8 tile-rows, each XCD a contiguous run of tiles (the fallback walk, always)
constexpr int PROBE_WALK_8x1 = 32;     // the 8 patches of a round side by side along M
constexpr int PROBE_PATCH_4x8 = 64;    // per-XCD patches of 4 x 8 tiles
constexpr int PROBE_PATCH_16x2 = 128;  // per-XCD patches of 16 x 2 tiles
constexpr int PROBE_UNPACED = 256;     // a stage's DMA instructions on consecutive matrix-op slots of its second K step
constexpr int PROBE_PERSIST = 1024;    // one workgroup per CU walks the tiles id, id + grid, ...; the next tile's first stages are asked for
                                       // before the epilogue of the present one
constexpr int PROBE_FILL_LESS = 512;   // sparse: the last 3 of a wave's 14 DMA instructions of every stage are left out -- 38 KiB a stage
                                       // instead of 50, about the bytes per matrix op of a 384 x 256 tile (what a taller tile could gain)

// B panel form: the dense panel form (64-byte pieces, a24_piece) whose rows are, inside every block of 256, stored in the
// order the block tile keeps them in LDS: position q of a block holds row unperm_n(q), i.e. row n sits at b_panel_pos(n).
// A stage of a block tile's B operand is then one (sparse: two) contiguous 16 KiB run(s), and every DMA instruction
// reads whole 128-byte lines.  Used for every B operand the library makes itself (re-arranged weights, transposed
// activations); a caller's row-major B (spmm24; X and dY) is read as it is.
__host__ __device__ __forceinline__ int b_panel_pos(int n) { return (n & ~255) | ((n & 3) << 5) | ((n >> 2) & 31) | (n & 128); }

// piece index of row r, 64-k panel kp, for an operand with `npanels` = K / 64 panels per row
__host__ __device__ __forceinline__ size_t a24_piece(int r, int kp, int npanels) {
  return ((size_t)(r >> 8) * npanels + kp) * 256 + (r & 255);
}

// Stage geometry.  Everything is laid out in bytes, and an fp8 kernel has exactly the byte geometry of its bf16
// counterpart with twice the k per byte: the LDS tiles, swizzles, DMA plan and fragment addresses are shared.
template <bool SPARSE, bool F8 = false>
struct Geo {
  static constexpr int ESIZE = F8 ? 1 : 2;
  static constexpr int BK = (SPARSE ? 128 : 64) / ESIZE;  // dense k per stage (B rows of 128 / 64 bytes)
  static constexpr int A_BYTES = 256 * 64;               // 64-byte rows: dense k, or the stored values of twice as many k
  static constexpr int META_ROW = SPARSE ? (F8 ? 16 : 8) : 0;   // metadata bytes per row and stage (4 bits per group of 4 k)
  static constexpr int META_BYTES = 256 * META_ROW;
  static constexpr int B_ROW = SPARSE ? 128 : 64;
  static constexpr int B_BYTES = 256 * B_ROW;
  static constexpr int META_OFF = A_BYTES;
  static constexpr int B_OFF = A_BYTES + META_BYTES;
  static constexpr int STAGE = A_BYTES + META_BYTES + B_BYTES;
  static constexpr int NB = SPARSE ? 3 : 4;              // ring depth
  static constexpr int LDS_TOTAL = NB * STAGE;
  static constexpr int NM = SPARSE ? (F8 ? 1 : 2) : 0;   // metadata DMA instructions per wave and stage
  static constexpr int NDMA = SPARSE ? 4 + NM + 8 : 4 + 4;  // DMA instructions per wave and stage
};

// LDS row -> row of the 256-row block tile (inverse of the permutation described above)
__device__ __forceinline__ int unperm_m(int p) {
  return (p & 128) | (((p >> 2) & 1) << 6) | (((p >> 5) & 3) << 4) | (((p >> 3) & 3) << 2) | (p & 3);
}
__device__ __forceinline__ int unperm_n(int p) { return (p & 128) | ((p & 31) << 2) | ((p >> 5) & 3); }
// 16-byte chunk swizzles.  A 16-byte-per-lane LDS read of a wavefront is served 16 lanes per clock, and the lanes
// that share a clock are not consecutive: {0-3, 20-23} and {4-7, 16-19} each pair up with {8-11, 28-31} or
// {12-15, 24-27} (likewise +32); they must hit 16 different 16-byte slots of the 256-byte bank row (measured on
// gfx950 with a read-throughput probe: both swizzles run at the rate of a linear read).
__device__ __forceinline__ int swz8(int p) { return (p ^ (p >> 3)) & 7; }          // 128-byte rows
__device__ __forceinline__ int swz4(int p) { return ((p >> 2) & 1) | ((((p >> 1) ^ (p >> 3)) & 1) << 1); }   // 64-byte rows

// compile-time loop: f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N-1>)
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) { (f(std::integral_constant<int, Is>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// Nothing may be moved across this point by the instruction scheduler.  The main loop is written as a sequence of
// slots {one matrix op + the memory ops that ride on it}, fenced from each other, so the issue order is the source order.
#define FFN24_FENCE() __builtin_amdgcn_sched_barrier(0)

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt = bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }   // vmcnt(63) expcnt(7) lgkmcnt(0)

// ------------------------------------------------------------------------------------------------
// global -> LDS DMA plan of one wave
// ------------------------------------------------------------------------------------------------
template <bool SPARSE, bool F8 = false, int PROBE = 0>
struct Dma {
  using G = Geo<SPARSE, F8>;
  const char* a;      // block's first A row (uniform)
  const char* am;     // metadata
  const char* b;
  uint32_t va[4], vm[2], vb[SPARSE ? 8 : 4];   // per-lane byte offsets from the uniform bases
  uint32_t a_stage, m_stage, b_stage;          // bytes from one stage to the next in the A values / metadata / B stream
  int wave;

  __device__ __forceinline__ void init(const GemmArgs& g, int m0, int n0, int tid) {
    int lane = tid & 63;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t b_row = (uint32_t)g.K * G::ESIZE;                 // bytes per B row in memory
    const uint32_t a_row = SPARSE ? b_row / 2 : b_row;               // bytes per A row (stored values only if sparse)
    a = static_cast<const char*>(g.A) + (size_t)m0 * a_row;
    b = static_cast<const char*>(g.B) + (g.b_rowmap ? (size_t)0 : (size_t)n0 * b_row);
    am = SPARSE ? reinterpret_cast<const char*>(g.Ameta) + (size_t)m0 * (g.K / 8) : nullptr;
    // a block tile's 256 rows occupy the same byte range in both forms; only the order of the pieces inside differs
    const bool panel = g.a_panel != 0;
    const uint32_t a_pitch = panel ? 64u : a_row, m_pitch = panel ? (uint32_t)G::META_ROW : (uint32_t)(g.K / 8);
    a_stage = panel ? 256u * 64u : 64u;
    m_stage = panel ? 256u * G::META_ROW : (uint32_t)G::META_ROW;
    const bool bp = g.b_panel != 0;
    b_stage = bp ? 256u * (uint32_t)G::B_ROW : (uint32_t)G::B_ROW;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int p = 64 * wave + 16 * j + (lane >> 2);
      int c = (lane & 3) ^ swz4(p);
      va[j] = (uint32_t)unperm_m(p) * a_pitch + c * 16;
      if constexpr (!SPARSE) {
        if (bp) vb[j] = (uint32_t)p * 64u + c * 16;     // LDS row p is piece p of the block's 16 KiB run
        else vb[j] = (g.b_rowmap ? (uint32_t)g.b_rowmap[n0 + unperm_n(p)] : (uint32_t)unperm_n(p)) * b_row + c * 16;
      }
    }
    if constexpr (SPARSE) {
#pragma unroll
      for (int j = 0; j < 8; j++) {
        int p = 64 * wave + 8 * j + (lane >> 3);
        int c = (lane & 7) ^ swz8(p);
        // panel: the row's 128 bytes are two 64-byte pieces in consecutive 16 KiB runs
        if (bp) vb[j] = (uint32_t)(c >> 2) * (256u * 64u) + (uint32_t)p * 64u + (c & 3) * 16;
        else vb[j] = (g.b_rowmap ? (uint32_t)g.b_rowmap[n0 + unperm_n(p)] : (uint32_t)unperm_n(p)) * b_row + c * 16;
      }
      if constexpr (F8) {
        vm[0] = (uint32_t)unperm_m(64 * wave + lane) * m_pitch;      // one row's 16 metadata bytes per lane
        vm[1] = 0;
      } else {
#pragma unroll
        for (int j = 0; j < 2; j++) {
          int d = 64 * (2 * wave + j) + lane;
          vm[j] = (uint32_t)unperm_m(d >> 1) * m_pitch + 4 * (d & 1);
        }
      }
    }
  }

  // DMA instruction J of stage kt into the stage buffer at `buf` (uniform LDS pointer)
  template <int J>
  __device__ __forceinline__ void issue(int kt, char* buf) const {
    if constexpr ((PROBE & PROBE_NO_DMA) != 0) return;
    if constexpr ((PROBE & PROBE_K_WRAP) != 0) kt &= 7;
    // The stage's uniform base goes through an opaque scalar register pair, so that the compiler keeps it apart from the
    // lane's 32-bit offset and picks the instruction's scalar-base + 32-bit-offset form: no 64-bit vector add per
    // instruction, one address register per instruction instead of two.
    if constexpr (J < 4) {
      __builtin_amdgcn_global_load_lds((glb_char*)(sbase(a, kt, a_stage) + voff(va[J])), (lds_char*)(buf + (4 * wave + J) * 1024), 16, 0, 0);
    } else if constexpr (!SPARSE) {
      constexpr int j = J - 4;
      __builtin_amdgcn_global_load_lds((glb_char*)(sbase(b, kt, b_stage) + voff(vb[j])), (lds_char*)(buf + G::B_OFF + (4 * wave + j) * 1024), 16, 0, 0);
    } else if constexpr (J < 4 + G::NM) {
      constexpr int j = J - 4;
      if constexpr (F8)
        __builtin_amdgcn_global_load_lds((glb_char*)(sbase(am, kt, m_stage) + voff(vm[0])), (lds_char*)(buf + G::META_OFF + wave * 1024), 16, 0, 0);
      else
        __builtin_amdgcn_global_load_lds((glb_char*)(sbase(am, kt, m_stage) + voff(vm[j])), (lds_char*)(buf + G::META_OFF + (2 * wave + j) * 256), 4, 0, 0);
    } else {
      constexpr int j = J - 4 - G::NM;
      __builtin_amdgcn_global_load_lds((glb_char*)(sbase(b, kt, b_stage) + voff(vb[j])), (lds_char*)(buf + G::B_OFF + (8 * wave + j) * 1024), 16, 0, 0);
    }
  }
  static __device__ __forceinline__ const char* sbase(const char* base, int kt, uint32_t stage) {
    const char* p = base + (size_t)kt * stage;
    asm volatile("" : "+s"(p));
    return p;
  }
  // (the offset is made opaque at the point of use too: hoisted out of the loop, its zero-extension would be out of the
  // instruction selector's sight and the 64-bit form would come back)
  static __device__ __forceinline__ uint32_t voff(uint32_t o) {
    asm volatile("" : "+v"(o));
    return o;
  }
};

// ------------------------------------------------------------------------------------------------
// fragments and matrix ops
// ------------------------------------------------------------------------------------------------
struct LaneCtx {
  int rho, h;       // lane & 31, lane >> 5
  int wy, wx;       // wave row / column inside the block tile
  int a_row64;      // byte offset of LDS row (wy*128 + rho) with 64-byte rows
  int b_row64;      // (wx*128 + rho) * 64
  int b_row128;     // (wx*128 + rho) * 128
  int sw4;          // swz4 of the lane's row (the same for all four 32-row tiles)
  int sw8;          // swz8 of the lane's B row for even ni (odd ni: ^4)
};

// Dense: K step S (0,1) of the 32-wide stage; fragment I < 4 -> a[I], else b[I-4]
struct FragD {
  bf16x8 a[4], b[4];
};
template <int S, int I, int PROBE = 0>
__device__ __forceinline__ void load_frag_dense1(const char* buf, const LaneCtx& L, FragD& f) {
  if constexpr ((PROBE & PROBE_NO_FRAG) != 0) return;
  constexpr int i = I & 3;
  int c = ((2 * S + L.h) ^ L.sw4) << 4;
  if constexpr (I < 4) f.a[i] = *reinterpret_cast<const bf16x8*>(buf + L.a_row64 + i * (32 * 64) + c);
  else f.b[i] = *reinterpret_cast<const bf16x8*>(buf + Geo<false>::B_OFF + L.b_row64 + i * (32 * 64) + c);
}
template <int M, int PROBE = 0>
__device__ __forceinline__ void mfma_dense1(const FragD& f, f32x16 (&acc)[4][4]) {
  if constexpr ((PROBE & PROBE_NO_MFMA) != 0) return;
  constexpr int mi = M >> 2, ni = M & 3;
  acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mi], f.b[ni], acc[mi][ni], 0, 0, 0);
}
// fp8 e4m3, v_mfma_f32_32x32x64_f8f6f4: 32 operand bytes per lane, paired byte by byte between A and B (measured:
// any assignment of the 64 k to (lane half, byte) works if both operands use the same one).  The two 16-byte
// fragments of a stage (S = 0 and S = 1 above) are exactly one such operand, so a 64-byte-row stage is one K step.
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ i32x8 cat16(const bf16x8& lo, const bf16x8& hi) {
  i32x4 l = __builtin_bit_cast(i32x4, lo), h = __builtin_bit_cast(i32x4, hi);
  return __builtin_shufflevector(l, h, 0, 1, 2, 3, 4, 5, 6, 7);
}
template <int M, int PROBE = 0>
__device__ __forceinline__ void mfma_dense_f8(const FragD& f0, const FragD& f1, f32x16 (&acc)[4][4]) {
  if constexpr ((PROBE & PROBE_NO_MFMA) != 0) return;
  constexpr int mi = M >> 2, ni = M & 3;
  // Written as inline assembly with the accumulator tied in place: through the builtin the compiler gives this
  // instruction a destination different from its accumulator input, which with all 256 accumulation registers in
  // use spills accumulators to scratch memory on every op.  Default modifiers = both operands e4m3, unscaled.
  // No software wait states are needed here: consecutive ops use different accumulators, and the same one is only
  // touched again 16 ops later.
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0"
               : "+a"(acc[mi][ni])
               : "v"(cat16(f0.a[mi], f1.a[mi])), "v"(cat16(f0.b[ni], f1.b[ni])));
}

// Sparse: the stage's K window of 64 = four 16-wide windows w.  Instruction S (0,1) gives lane half q the window
// 2q+S, so a lane's two instructions use 32 consecutive stored-value bytes and one 32-bit metadata word (ABID = S
// picks the half).  B lane half h then needs, for instruction S, the 8-k chunks 2S+h (registers 0..7) and 4+2S+h
// (registers 8..15).
struct FragS {
  bf16x8 a[4];
  bf16x8 blo[4], bhi[4];
};
// Metadata of a lane for the stage's two instructions: bf16 one 32-bit word (16 bits per instruction, picked by
// ABID); fp8 (twice the groups per stored byte) two words, one per instruction.
template <bool F8> struct IdxWords { uint32_t w[F8 ? 2 : 1]; };
template <bool F8, int I>
__device__ __forceinline__ void load_idx_sparse1(const char* buf, const LaneCtx& L, IdxWords<F8> (&idx)[4]) {
  const char* p = buf + Geo<true, F8>::META_OFF + (L.wy * 128 + L.rho + 32 * I) * Geo<true, F8>::META_ROW;
  if constexpr (F8) {
    u32x2 v = *reinterpret_cast<const u32x2*>(p + 8 * L.h);
    idx[I].w[0] = v[0]; idx[I].w[1] = v[1];
  } else {
    idx[I].w[0] = *reinterpret_cast<const uint32_t*>(p + 4 * L.h);
  }
}
// fragment I of instruction S: I < 4 -> a[I]; 4..7 -> low half of b[I-4]; 8..11 -> high half of b[I-8]
template <bool F8, int S, int I, int PROBE = 0>
__device__ __forceinline__ void load_frag_sparse1(const char* buf, const LaneCtx& L, FragS& f) {
  if constexpr ((PROBE & PROBE_NO_FRAG) != 0) return;
  constexpr int i = I & 3;
  if constexpr (I < 4) {
    f.a[i] = *reinterpret_cast<const bf16x8*>(buf + L.a_row64 + i * (32 * 64) + (((2 * L.h + S) ^ L.sw4) << 4));
  } else {
    int sw = L.sw8 ^ ((i & 1) << 2);
    const char* row = buf + Geo<true, F8>::B_OFF + L.b_row128 + i * (32 * 128);
    if constexpr (I < 8) f.blo[i] = *reinterpret_cast<const bf16x8*>(row + (((2 * S + L.h) ^ sw) << 4));
    else f.bhi[i] = *reinterpret_cast<const bf16x8*>(row + (((4 + 2 * S + L.h) ^ sw) << 4));
  }
}
// fp8: v_smfmac_f32_32x32x64_fp8_fp8 has, byte for byte, the operand layout of the bf16 instruction (measured): A 16
// stored bytes of the lane half's window, B the two 16-byte chunks, and a full 32-bit index word per instruction.
template <bool F8, int S, int M, int PROBE = 0>
__device__ __forceinline__ void mfma_sparse1(const FragS& f, const IdxWords<F8> (&idx)[4], f32x16 (&acc)[4][4]) {
  if constexpr ((PROBE & PROBE_NO_MFMA) != 0) return;
  constexpr int mi = M >> 2, ni = M & 3;
  if constexpr (F8) {
    acc[mi][ni] = __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(__builtin_bit_cast(i32x4, f.a[mi]), cat16(f.blo[ni], f.bhi[ni]), acc[mi][ni],
                                                               (int)idx[mi].w[S], 0, 0);
  } else {
    bf16x16 b = __builtin_shufflevector(f.blo[ni], f.bhi[ni], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
    acc[mi][ni] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(f.a[mi], b, acc[mi][ni], (int)idx[mi].w[0], 0, S);
  }
}

// ------------------------------------------------------------------------------------------------
// the kernel
// ------------------------------------------------------------------------------------------------

// tile id -> (tile_m, tile_n).  Consecutive workgroup ids go round-robin over the 8 XCDs (each with its own L2) and an
// XCD hands its ids to its 32 CUs in order, so 256 consecutive ids are one "round" of the chip: XCD x runs ids
// x, x + 8, ... of it.  A round is laid out as a 4 x 2 grid of per-XCD patches of 8 x 4 tiles (32 tile-rows x 8
// tile-columns in all): inside a patch the 8 + 4 operand panels are shared through the XCD's L2, and XCDs that sit in
// the same grid row (column) read the same A (B) panels at the same time, so that what one of them brings in from HBM
// the others find in the memory-side cache.  Measured against one 8 x 4 patch per XCD with all XCDs side by side
// along M (every round then streams the whole A operand): 3.5 % on the sparse GEMMs, nothing on the dense ones.
// Tile-rows beyond the last whole round (ntm not a multiple of 32: the sparse part of a split weight gradient) and shapes whose
// tile-columns the grid does not divide fall back to bands of 8 tile-rows, each XCD a contiguous run of tiles.
template <int PROBE = 0>
__device__ __forceinline__ void tile_coords(int ntm, int ntn, int pid, int& tm, int& tn) {
  // XCD grid, patch shape; GX * GY = 8 XCDs, PM * PN = 32 CUs
  constexpr int GX = (PROBE & PROBE_WALK_8x1) ? 8 : 4, GY = 8 / GX;
  constexpr int PM = (PROBE & PROBE_PATCH_4x8) ? 4 : ((PROBE & PROBE_PATCH_16x2) ? 16 : 8), PN = 32 / PM;
  int tm0 = 0;   // tile-rows [0, tm0) are walked in rounds, the rest in bands
  if (!(PROBE & PROBE_WALK_BANDS) && ntn % (PN * GY) == 0) tm0 = ntm - ntm % (PM * GX);
  if (pid < tm0 * ntn) {
    const int xcd = pid & 7, idx = pid >> 3;
    const int round = idx >> 5, j = idx & 31;
    const int rounds_n = ntn / (PN * GY);
    tm = ((round / rounds_n) * GX + (xcd % GX)) * PM + (j % PM);
    tn = ((round % rounds_n) * GY + (xcd / GX)) * PN + (j / PM);
    return;
  }
  pid -= tm0 * ntn;   // a multiple of 256: the low three bits are still the XCD
  ntm -= tm0;
  int nb = ntm * ntn;
  if ((nb & 7) == 0) pid = (pid & 7) * (nb >> 3) + (pid >> 3);
  const int GROUP = 8;
  int per_group = GROUP * ntn;
  int gid = pid / per_group;
  int first = gid * GROUP;
  int gsz = min(ntm - first, GROUP);
  int in = pid - gid * per_group;
  tm = tm0 + first + in % gsz;
  tn = in / gsz;
}

// an epilogue that declares `static constexpr bool STAGED` takes a fifth argument: 32 KiB of LDS private to the wave
template <class E, class = void> struct epi_is_staged : std::false_type {};
template <class E> struct epi_is_staged<E, std::void_t<decltype(E::STAGED)>> : std::true_type {};

// Epilogue concept:  struct E { struct Args {...}; static __device__ void run(const Args&, acc, m_lane, n_lane); }
//   m_lane = global row of acc[0][*][0] for this lane (its 64 rows are m_lane + 16*mi + v),
//   n_lane = global column of acc[*][0][*] (its 4 columns are n_lane + ni).
// One block tile of one GEMM: tile number `pid` of g (workgroup-uniform), LDS ring at `smem`.
// Pacing of the DMA issue.  The four waves run in step, one per SIMD, and share one address unit that takes about
// 14 cycles per 16-byte-a-lane DMA instruction; a matrix-op slot is 32 cycles.  When every wave hands over a DMA
// instruction on every slot, the unit is oversubscribed (4 x 14 > 32), the waves stall in the issue and their matrix
// pipes idle: measured per K step, the step that carries 14 DMA instructions on consecutive slots takes 1200 cycles
// instead of 512.  So the instructions ride on every other slot only.  Dense (8 a stage): the even slots of the second
// K step.  Sparse (13 or 14 a stage): the first half on the even slots of the second K step, the rest on the even slots of
// the NEXT stage's first K step, still into the buffer that the stage before freed -- one stage buffer is therefore
// half filled across a stage boundary, which costs nothing because the ring keeps NB - 2 whole stages in flight anyway.
// dma_on_step1 / dma_on_step0: which DMA instruction rides on slot M of that K step (-1: none).
template <int NDMA, bool SPREAD, bool PACED>
constexpr int dma_on_step1(int M) {
  constexpr int H1 = SPREAD ? NDMA / 2 : NDMA;
  if (!PACED || 2 * H1 > 16) return M < H1 ? M : -1;
  return (M % 2 == 0 && M / 2 < H1) ? M / 2 : -1;
}
template <int NDMA, bool SPREAD, bool PACED>
constexpr int dma_on_step0(int M) {
  constexpr int H1 = SPREAD ? NDMA / 2 : NDMA;
  if (!SPREAD) return -1;
  return (M % 2 == 0 && M / 2 < NDMA - H1) ? H1 + M / 2 : -1;
}

template <bool SPARSE, class Epi, bool F8 = false, int PROBE = 0>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const typename Epi::Args& ea, char* smem, int pid, int pid_end = 0, int pid_step = 0) {
  using G = Geo<SPARSE, F8>;
  constexpr int NB = G::NB, NDMA = G::NDMA - ((SPARSE && (PROBE & PROBE_FILL_LESS)) ? 3 : 0);
  constexpr bool PERSIST = (PROBE & PROBE_PERSIST) != 0;

  int tid = threadIdx.x;
  int lane = tid & 63, wave = tid >> 6;
  int tm, tn;
  tile_coords<PROBE>(g.M / TILE_M, g.N / TILE_N, pid, tm, tn);
  int m0 = tm * TILE_M, n0 = tn * TILE_N;

  LaneCtx L;
  L.rho = lane & 31; L.h = lane >> 5; L.wy = wave >> 1; L.wx = wave & 1;
  L.a_row64 = (L.wy * 128 + L.rho) * 64;
  L.b_row64 = (L.wx * 128 + L.rho) * 64;
  L.b_row128 = (L.wx * 128 + L.rho) * 128;
  L.sw4 = swz4(L.rho);
  L.sw8 = (L.rho & 7) ^ (L.rho >> 3);

  Dma<SPARSE, F8, PROBE> dma;
  dma.init(g, m0, n0, tid);

  const int nk = g.K / G::BK;
  // prologue: stages 0 .. min(NB, nk)-1 into their ring slots; wait for stage 0 only
  const int npro = nk < NB ? nk : NB;
  for (int s = 0; s < npro; s++) static_for<NDMA>([&](auto J) { dma.template issue<J>(s, smem + s * G::STAGE); });
  bool first = true;

  for (;;) {   // one pass per tile (PERSIST: several tiles per workgroup)
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;
  // Pin the accumulators to the accumulation register file: an empty asm with an AGPR constraint gives their
  // live ranges the AGPR class, so the 256 arch VGPRs stay free for fragments and addresses.
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) asm volatile("" : "+a"(acc[i][j]));

  // a later tile's prologue went out before the previous epilogue, whose stores count in the same counter and complete in no
  // fixed order with the loads: wait for all of it
  if (first && npro == NB) wait_vmcnt<(NB - 1) * NDMA>(); else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  FFN24_FENCE();

  // MODE 0: steady state -- after the barrier the stage kt+NB is issued into the buffer this stage frees
  // MODE 1: tail -- nothing left to issue, wait for everything outstanding before the barrier
  // MODE 2: last stage -- no barrier, no next fragments
  if constexpr (SPARSE) {
    FragS f0, f1;
    IdxWords<F8> idx[4];
    static_for<4>([&](auto I) { load_idx_sparse1<F8, I>(smem, L, idx); });
    static_for<12>([&](auto I) { load_frag_sparse1<F8, 0, I, PROBE>(smem, L, f0); });
    // sparse: spread the DMA of a stage over two K steps (see dma_on_step1) when there is a steady state at all
    constexpr bool PACED = (PROBE & PROBE_UNPACED) == 0;
    auto stage = [&](int kt, char* cur, char* nxt, char* prv, auto mode, auto spread) {
      constexpr int MODE = decltype(mode)::value;
      constexpr bool SPREAD0 = decltype(spread)::value != 0;   // this stage's first K step carries the rest of stage kt-1+NB
      IdxWords<F8> idx_n[4] = {};
      FFN24_FENCE();
      static_for<16>([&](auto M) {
        mfma_sparse1<F8, 0, M, PROBE>(f0, idx, acc);
        constexpr int J0 = dma_on_step0<NDMA, PACED, PACED>(M);
        if constexpr (SPREAD0 && J0 >= 0) dma.template issue<(J0 >= 0 ? J0 : 0)>(kt - 1 + NB, prv);
        if constexpr (M < 12) load_frag_sparse1<F8, 1, M, PROBE>(cur, L, f1);
        FFN24_FENCE();
      });
      if constexpr (MODE != 2) {
        // stage kt+1 must have landed; behind it in issue order are the NB - 2 stages kt+2 .. kt+NB-1, all of them whole
        // (the rest of stage kt-1+NB went out just above)
        if constexpr (MODE == 0) wait_vmcnt<(NB - 2) * NDMA>(); else wait_vmcnt<0>();
        wait_lgkmcnt0();
        __builtin_amdgcn_s_barrier();
      }
      FFN24_FENCE();
      static_for<16>([&](auto M) {
        mfma_sparse1<F8, 1, M, PROBE>(f1, idx, acc);
        constexpr int J1 = dma_on_step1<NDMA, PACED, PACED>(M);
        if constexpr (MODE == 0 && J1 >= 0) dma.template issue<(J1 >= 0 ? J1 : 0)>(kt + NB, cur);
        if constexpr (MODE != 2) {
          if constexpr (M < 4) load_idx_sparse1<F8, M>(nxt, L, idx_n);
          if constexpr (M < 12) load_frag_sparse1<F8, 0, M, PROBE>(nxt, L, f0);
        }
        FFN24_FENCE();
      });
#pragma unroll
      for (int i = 0; i < 4; i++) idx[i] = idx_n[i];
    };
    int slot = 0;
    auto advance = [&](int kt, auto mode, auto spread) {
      int ns = slot + 1 == NB ? 0 : slot + 1;
      int ps = slot == 0 ? NB - 1 : slot - 1;
      stage(kt, smem + slot * G::STAGE, smem + ns * G::STAGE, smem + ps * G::STAGE, mode, spread);
      slot = ns;
    };
    using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>; using I2 = std::integral_constant<int, 2>;
    using SP = std::integral_constant<int, PACED ? 1 : 0>;
    int kt = 0;
    if (nk > NB) {
      // stage 0 issues the first half of stage NB; stages 1 .. nk-NB each issue the rest of what the stage before began,
      // and all but the last of them the first half of their own
      advance(kt, I0{}, I0{}); kt++;
      for (; kt < nk - NB; kt++) advance(kt, I0{}, SP{});
      if constexpr (PACED) { advance(kt, I1{}, I1{}); kt++; }
    }
    for (; kt < nk - 1; kt++) advance(kt, I1{}, I0{});
    advance(kt, I2{}, I0{});
  } else if constexpr (F8) {
    // Dense fp8: a stage is ONE K step of 16 matrix ops (64 cycles each).  The fragments of the whole next stage and
    // the DMA of the stage that reuses this stage's buffer (its fragments are already in registers) ride on them;
    // one barrier at the end of the stage.  Two fragment sets alternate.
    FragD fr[2][2];
    static_for<8>([&](auto I) { load_frag_dense1<0, I, PROBE>(smem, L, fr[0][0]); });
    static_for<8>([&](auto I) { load_frag_dense1<1, I, PROBE>(smem, L, fr[0][1]); });
    auto stage = [&](int kt, char* cur, char* nxt, auto par, auto mode) {
      constexpr int P = decltype(par)::value, MODE = decltype(mode)::value;
      FFN24_FENCE();
      static_for<16>([&](auto M) {
        mfma_dense_f8<M, PROBE>(fr[P][0], fr[P][1], acc);
        if constexpr (MODE == 0 && M < NDMA) dma.template issue<M>(kt + NB, cur);
        if constexpr (MODE != 2) {
          if constexpr (M < 8) load_frag_dense1<0, M, PROBE>(nxt, L, fr[P ^ 1][0]);
          else load_frag_dense1<1, M - 8, PROBE>(nxt, L, fr[P ^ 1][1]);
        }
        FFN24_FENCE();
      });
      if constexpr (MODE != 2) {
        // the next stage reads fragments of stage kt+2 from the first op on: it must have landed, everywhere
        if constexpr (MODE == 0) wait_vmcnt<(NB - 2) * NDMA>(); else wait_vmcnt<0>();
        wait_lgkmcnt0();
        __builtin_amdgcn_s_barrier();
      }
      FFN24_FENCE();
    };
    // the loop above reads stage 1 during stage 0: the prologue's wait covered stage 0 only
    if (npro == NB) wait_vmcnt<(NB - 2) * NDMA>(); else wait_vmcnt<0>();
    wait_lgkmcnt0();
    __builtin_amdgcn_s_barrier();
    FFN24_FENCE();
    // The two fragment sets alternate by stage parity.  The stage count is even (K is a multiple of 128 here), so
    // the stages are walked in pairs, straight-line: a parity branch inside the loop makes the compiler shuffle the
    // 256 accumulation registers between its two arms.
    int slot = 0;
    auto advance = [&](int kt, auto par, auto mode) {
      int ns = slot + 1 == NB ? 0 : slot + 1;
      stage(kt, smem + slot * G::STAGE, smem + ns * G::STAGE, par, mode);
      slot = ns;
    };
    using P0 = std::integral_constant<int, 0>; using P1 = std::integral_constant<int, 1>;
    using M0 = std::integral_constant<int, 0>; using M1 = std::integral_constant<int, 1>; using M2 = std::integral_constant<int, 2>;
    int kt = 0;
    for (; kt < nk - NB; kt += 2) { advance(kt, P0{}, M0{}); advance(kt + 1, P1{}, M0{}); }
    if (nk >= NB) { advance(kt, P0{}, M1{}); advance(kt + 1, P1{}, M1{}); kt += 2; }
    advance(kt, P0{}, M1{});
    advance(kt + 1, P1{}, M2{});
  } else {
    FragD f0, f1;
    static_for<8>([&](auto I) { load_frag_dense1<0, I, PROBE>(smem, L, f0); });
    auto stage = [&](int kt, char* cur, char* nxt, auto mode) {
      constexpr int MODE = decltype(mode)::value;
      FFN24_FENCE();
      static_for<16>([&](auto M) {
        mfma_dense1<M, PROBE>(f0, acc);
        if constexpr (M < 8) load_frag_dense1<1, M, PROBE>(cur, L, f1);
        FFN24_FENCE();
      });
      if constexpr (MODE != 2) {
        if constexpr (MODE == 0) wait_vmcnt<(NB - 2) * NDMA>(); else wait_vmcnt<0>();
        wait_lgkmcnt0();
        __builtin_amdgcn_s_barrier();
      }
      FFN24_FENCE();
      static_for<16>([&](auto M) {
        mfma_dense1<M, PROBE>(f1, acc);
        constexpr int J1 = dma_on_step1<NDMA, false, (PROBE & PROBE_UNPACED) == 0>(M);
        if constexpr (MODE == 0 && J1 >= 0) dma.template issue<(J1 >= 0 ? J1 : 0)>(kt + NB, cur);
        if constexpr (MODE != 2 && M < 8) load_frag_dense1<0, M, PROBE>(nxt, L, f0);
        FFN24_FENCE();
      });
    };
    int slot = 0;
    auto advance = [&](int kt, auto mode) {
      int ns = slot + 1 == NB ? 0 : slot + 1;
      stage(kt, smem + slot * G::STAGE, smem + ns * G::STAGE, mode);
      slot = ns;
    };
    int kt = 0;
    for (; kt < nk - NB; kt++) advance(kt, std::integral_constant<int, 0>{});
    for (; kt < nk - 1; kt++) advance(kt, std::integral_constant<int, 1>{});
    advance(kt, std::integral_constant<int, 2>{});
  }

  if constexpr (F8 && !SPARSE) {
    // the dense fp8 ops are inline assembly, which the compiler's hazard handling does not see: let the last ones
    // (16 passes each) drain before the epilogue reads the accumulators
    asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15" ::: "memory");
    // and tie the accumulators to a point after the wait (volatile statements keep their order), so that no read of
    // them can be scheduled above it
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) asm volatile("" : "+a"(acc[i][j]));
  }
  int m_lane = m0 + L.wy * 128 + 64 * L.h;
  int n_lane = n0 + L.wx * 128 + 4 * L.rho;
  if constexpr (PERSIST) {
    pid += pid_step;
    const bool more = pid < pid_end;
    if (more) {
      // every wave has read its last fragments: the ring is free for the next tile's first stages, which then land while
      // the epilogue runs
      __builtin_amdgcn_s_barrier();
      tile_coords<PROBE>(g.M / TILE_M, g.N / TILE_N, pid, tm, tn);
      m0 = tm * TILE_M; n0 = tn * TILE_N;
      dma.init(g, m0, n0, tid);
      for (int s = 0; s < npro; s++) static_for<NDMA>([&](auto J) { dma.template issue<J>(s, smem + s * G::STAGE); });
    }
    Epi::run(ea, acc, m_lane, n_lane);
    if (!more) break;
    first = false;
  } else {
    if constexpr (epi_is_staged<Epi>::value) {
      // the epilogue stages its stores through the operand ring: every wave must have read its last fragments first
      static_assert(G::LDS_TOTAL >= GEMM_THREADS / 64 * 128 * 256, "a 32 KiB staging area per wave");
      __builtin_amdgcn_s_barrier();
      Epi::run(ea, acc, m_lane, n_lane, smem + wave * (128 * 256));
    } else {
      Epi::run(ea, acc, m_lane, n_lane);
    }
    break;
  }
  }   // tiles
}

// Clock sample of a workgroup (profiling only): ticks of the shader clock and of the constant 100 MHz clock between its
// first and last instruction; their ratio is the clock the kernel really ran at (it drops well below the nominal 2.4 GHz
// under matrix load).
struct ClkSample {
  unsigned long long t0, r0;
  __device__ __forceinline__ void begin(const GemmArgs& g) {
    if (g.clk) { t0 = __builtin_amdgcn_s_memtime(); r0 = __builtin_amdgcn_s_memrealtime(); }
  }
  __device__ __forceinline__ void end(const GemmArgs& g) {
    if (g.clk && blockIdx.x < CLK_SLOTS) {
      unsigned long long t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
      if (threadIdx.x == 0) { g.clk[2 * blockIdx.x] = t1 - t0; g.clk[2 * blockIdx.x + 1] = r1 - r0; }
    }
  }
};

template <bool SPARSE, class Epi, bool F8 = false, int PROBE = 0>
__global__ void __launch_bounds__(GEMM_THREADS) gemm_kernel(GemmArgs g, typename Epi::Args ea) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  ClkSample cs;
  cs.begin(g);
  gemm_tile<SPARSE, Epi, F8, PROBE>(g, ea, smem, blockIdx.x, (g.M / TILE_M) * (g.N / TILE_N), gridDim.x);
  cs.end(g);
}

// Two GEMMs in one launch: the first `nd_tiles` workgroups compute the tiles of a dense GEMM gd, the others those of
// a sparse GEMM gs (same epilogue type, separate arguments).  The split weight-gradient GEMMs use it (Sec. 2,
// "Optimization 1": a 2:4 GEMM over most hidden features plus a dense one over the few that are not sparse enough):
// alone, the small dense GEMM would occupy a fraction of the CUs for as long as a full round of tiles.  The dense
// tiles, which take longer, come first.
template <class Epi, bool F8 = false>
__global__ void __launch_bounds__(GEMM_THREADS) gemm_pair_kernel(GemmArgs gd, typename Epi::Args ead, int nd_tiles,
                                                                  GemmArgs gs, typename Epi::Args eas) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int pid = blockIdx.x;
  ClkSample cs;
  cs.begin(gs);
  if (pid < nd_tiles) gemm_tile<false, Epi, F8>(gd, ead, smem, pid);
  else gemm_tile<true, Epi, F8>(gs, eas, smem, pid - nd_tiles);
  cs.end(gs);
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

// The same pick for a group of non-negative values that arrive packed, lo = h0 | h1 << 16 and hi = h2 | h3 << 16 (the
// activation epilogues): with the value in the upper half, key_i = h_i << 16 | (3 - i) takes one instruction each, and
// the kept pair, in position order, is one byte permute of the two winning keys.
__device__ __forceinline__ uint32_t pick24_packed(uint32_t lo, uint32_t hi, uint32_t& pair) {
  uint32_t k0 = (lo << 16) | 3u, k1 = (lo & 0xFFFF0000u) | 2u, k2 = (hi << 16) | 1u, k3 = hi & 0xFFFF0000u;
  uint32_t a = max(k0, k1), b = min(k0, k1), c = max(k2, k3), d = min(k2, k3);
  uint32_t top = max(a, c);
  uint32_t e = max(b, d);
  uint32_t second = max(min(a, c), min(max(a, c), e));
  uint32_t ct = top & 3u, cs = second & 3u;
  bool top_first = ct > cs;
  uint32_t kf = top_first ? top : second, ks = top_first ? second : top;
  pair = __builtin_amdgcn_perm(ks, kf, 0x07060302u);           // kf's upper half below ks's upper half
  uint32_t cmax = max(ct, cs), cmin = min(ct, cs);
  return (cmax | (cmin << 2)) ^ 15u;
}

}  // namespace ffn24
