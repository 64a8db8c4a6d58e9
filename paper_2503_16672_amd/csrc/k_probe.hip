// Measurement probes: what the matrix pipes, the operand stream and the memory deliver on this chip, measured with the
// library's own code.  Nothing on the product path calls them; bench.py --probe prints their results, and the figures
// the design notes quote for "what the hardware can do" come from here.
//   probe_mfma_rate  register-resident matrix-op loops (no memory traffic at all)
//   probe_gemm       the GEMM core with ingredients removed (gemm_core.hpp, PROBE_*)
//   probe_copy       a plain streaming copy (the HBM rate a simple kernel reaches; also the known-size kernel that
//                    calibrates the profiler's HBM byte counters)
// They allocate their own buffers and synchronise with their own work: diagnostics, not serving code.
#include <algorithm>
#include <vector>
#include "launch_impl.hpp"

namespace ffn24 {

namespace {

struct DevBuf {
  void* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  int alloc(size_t n) { return hipMalloc(&p, n) == hipSuccess ? 0 : 1; }
};

__device__ __forceinline__ uint32_t xorshift(uint32_t& x) { x ^= x << 13; x ^= x >> 17; x ^= x << 5; return x; }

// KIND 0 dense bf16 32x32x16, 1 sparse bf16 32x32x32, 2 dense fp8 32x32x64, 3 sparse fp8 32x32x64.
// 16 independent accumulators per wave, exactly the GEMM core's register tile; operands are pseudo-random finite values
// (the clock the chip settles at under matrix load depends on how much the operand bits toggle).
template <int KIND>
__global__ void __launch_bounds__(256) mfma_rate_kernel(int iters, unsigned long long* out, float* sink, uint32_t seed) {
  uint32_t x = (threadIdx.x + blockIdx.x * 256u) * 2654435761u + seed;
  bf16x8 a[4], b[4], b2[4];
  i32x8 a8[4], b8[4];
  int idx[4];
  for (int i = 0; i < 4; i++) {
    for (int j = 0; j < 4; j++) {
      // bf16 pairs in (-2, 2) without zeros, infinities or NaNs; fp8 bytes with the NaN codes masked out
      reinterpret_cast<uint32_t*>(&a[i])[j] = 0x3C003C00u | (xorshift(x) & 0x83FF83FFu);
      reinterpret_cast<uint32_t*>(&b[i])[j] = 0x3C003C00u | (xorshift(x) & 0x83FF83FFu);
      reinterpret_cast<uint32_t*>(&b2[i])[j] = 0x3C003C00u | (xorshift(x) & 0x83FF83FFu);
    }
    for (int j = 0; j < 8; j++) { a8[i][j] = (int)(xorshift(x) & 0x77777777u); b8[i][j] = (int)(xorshift(x) & 0x77777777u); }
    const uint32_t codes[6] = {0x4, 0x8, 0xC, 0x9, 0xD, 0xE};   // the six legal 2:4 index nibbles
    uint32_t w = 0;
    for (int q = 0; q < 8; q++) w |= codes[xorshift(x) % 6] << (4 * q);
    idx[i] = (int)w;
  }
  f32x16 acc[4][4];
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < 4; j++)
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;
  // (the dense fp8 op is inline assembly on the accumulation registers, as in the GEMM core; the builtins place their
  // accumulators themselves)
  __syncthreads();
  unsigned long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int mi = 0; mi < 4; mi++)
#pragma unroll
      for (int ni = 0; ni < 4; ni++) {
        if constexpr (KIND == 0) acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
        if constexpr (KIND == 1) {
          bf16x16 bb = __builtin_shufflevector(b[ni], b2[ni], 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[mi], bb, acc[mi][ni], idx[mi], 0, 0);
        }
        if constexpr (KIND == 2) asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0" : "+a"(acc[mi][ni]) : "v"(a8[mi]), "v"(b8[ni]));
        if constexpr (KIND == 3)
          acc[mi][ni] = __builtin_amdgcn_smfmac_f32_32x32x64_fp8_fp8(__builtin_bit_cast(i32x4, a[mi]), b8[ni], acc[mi][ni], idx[mi], 0, 0);
      }
  }
  if constexpr (KIND == 2) {
    asm volatile("s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15\n s_nop 15" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) asm volatile("" : "+a"(acc[i][j]));
  }
  unsigned long long t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float s = 0.f;
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < 4; j++)
      for (int v = 0; v < 16; v++) s += acc[i][j][v];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive
  if ((threadIdx.x & 63) == 0) {
    int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    out[2 * w] = t1 - t0;
    out[2 * w + 1] = r1 - r0;
  }
}

// pseudo-random operand fill: mode 0 bf16 pairs in (-2, 2), mode 1 metadata words of legal nibbles
__global__ void __launch_bounds__(256) probe_fill_kernel(uint32_t* p, size_t n, uint32_t seed, int mode) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) {
    uint32_t x = (uint32_t)i * 2654435761u + seed;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    if (mode == 0) {
      p[i] = 0x3C003C00u | (x & 0x83FF83FFu);
    } else {
      const uint32_t codes[6] = {0x4, 0x8, 0xC, 0x9, 0xD, 0xE};
      uint32_t w = 0;
      for (int b = 0; b < 8; b++) w |= codes[(x >> (3 * b)) % 6] << (4 * b);
      p[i] = w;
    }
  }
}

// The fastest plain copy found on this chip: one 16-byte piece per work item, as many workgroups as that takes, loads and
// stores with the non-temporal hint (6.0-6.5 TB/s read + written; a grid-stride loop over 8192 workgroups: 4.5-4.7).
__global__ void __launch_bounds__(256) probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

double median_of(std::vector<float>& v) {
  std::sort(v.begin(), v.end());
  return v[v.size() / 2];
}

template <bool SPARSE, int PROBE>
int run_gemm_variant(const GemmArgs& g, __bf16* C, int reps, double* ms_median, double* mhz) {
  DevBuf clk;
  if (clk.alloc(16 * CLK_SLOTS)) return 1;
  if (hipMemset(clk.p, 0, 16 * CLK_SLOTS) != hipSuccess) return 1;
  EpiRowMajor::Args ea{C, g.N};
  std::vector<hipEvent_t> ev(reps + 1);
  for (auto& e : ev) if (hipEventCreate(&e) != hipSuccess) return 1;
  tl_gemm_clk = static_cast<unsigned long long*>(clk.p);
  int rc = 0;
  for (int i = 0; i < 3 && !rc; i++) rc = launch_gemm<SPARSE, EpiRowMajor, false, PROBE>(g, ea, nullptr);
  if (!rc) rc = hipEventRecord(ev[0], nullptr) != hipSuccess;
  for (int i = 0; i < reps && !rc; i++) {
    rc = launch_gemm<SPARSE, EpiRowMajor, false, PROBE>(g, ea, nullptr);
    if (!rc) rc = hipEventRecord(ev[i + 1], nullptr) != hipSuccess;
  }
  tl_gemm_clk = nullptr;
  if (!rc) rc = hipEventSynchronize(ev[reps]) != hipSuccess;
  std::vector<float> ms(reps, 0.f);
  for (int i = 0; i < reps && !rc; i++) rc = hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]) != hipSuccess;
  for (auto& e : ev) (void)hipEventDestroy(e);
  if (rc) return 1;
  *ms_median = median_of(ms);
  unsigned long long h[2 * CLK_SLOTS];
  if (hipMemcpy(h, clk.p, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return 1;
  double t = 0, r = 0;
  const int nb = std::min(CLK_SLOTS, (g.M / TILE_M) * (g.N / TILE_N));
  for (int i = 0; i < nb; i++) { t += (double)h[2 * i]; r += (double)h[2 * i + 1]; }
  *mhz = r > 0 ? 100.0 * t / r : 0.0;
  return 0;
}

}  // namespace

int probe_mfma_rate(int kind, int iters, double* cycles_per_op, double* mhz, double* tflops_dense_equivalent) {
  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 1;
  const int blocks = prop.multiProcessorCount;   // one workgroup of 4 waves per CU: one wave per SIMD
  DevBuf out, sink;
  if (out.alloc((size_t)blocks * 4 * 16) || sink.alloc(64)) return 1;
  auto launch = [&](int n, uint32_t seed) {
    auto* o = static_cast<unsigned long long*>(out.p);
    auto* sk = static_cast<float*>(sink.p);
    switch (kind) {
      case 0: hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(blocks), dim3(256), 0, nullptr, n, o, sk, seed); break;
      case 1: hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(blocks), dim3(256), 0, nullptr, n, o, sk, seed); break;
      case 2: hipLaunchKernelGGL(mfma_rate_kernel<2>, dim3(blocks), dim3(256), 0, nullptr, n, o, sk, seed); break;
      default: hipLaunchKernelGGL(mfma_rate_kernel<3>, dim3(blocks), dim3(256), 0, nullptr, n, o, sk, seed); break;
    }
  };
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
  launch(200, 1u);   // warm-up: clocks and code in place
  (void)hipEventRecord(e0, nullptr);
  launch(iters, 7u);
  (void)hipEventRecord(e1, nullptr);
  int rc = hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess;
  float ms = 0.f;
  if (!rc) rc = hipEventElapsedTime(&ms, e0, e1) != hipSuccess;
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  std::vector<unsigned long long> h((size_t)blocks * 8);
  if (!rc) rc = hipMemcpy(h.data(), out.p, h.size() * 8, hipMemcpyDeviceToHost) != hipSuccess;
  if (rc) return 1;
  double t = 0, r = 0;
  for (size_t i = 0; i < h.size(); i += 2) { t += (double)h[i]; r += (double)h[i + 1]; }
  const double ops = (double)iters * 16;
  *cycles_per_op = t / (h.size() / 2) / ops;
  *mhz = 100.0 * t / r;
  const double flops_per_op = kind == 0 ? 2.0 * 32 * 32 * 16 : (kind == 1 ? 2.0 * 32 * 32 * 32 : 2.0 * 32 * 32 * 64);
  *tflops_dense_equivalent = flops_per_op * ops * blocks * 4 / (ms * 1e-3) / 1e12;
  return 0;
}

int probe_gemm(int sparse, int variant, int M, int N, int K, int reps, double* ms_median, double* mhz) {
  DevBuf A, meta, B, C;
  const size_t ab = (size_t)M * K * 2, bb = (size_t)N * K * 2;
  if (A.alloc(ab) || meta.alloc((size_t)M * K / 8) || B.alloc(bb) || C.alloc((size_t)M * N * 2)) return 1;
  hipLaunchKernelGGL(probe_fill_kernel, dim3(4096), dim3(256), 0, nullptr, static_cast<uint32_t*>(A.p), ab / 4, 1u, 0);
  hipLaunchKernelGGL(probe_fill_kernel, dim3(4096), dim3(256), 0, nullptr, static_cast<uint32_t*>(B.p), bb / 4, 2u, 0);
  hipLaunchKernelGGL(probe_fill_kernel, dim3(4096), dim3(256), 0, nullptr, static_cast<uint32_t*>(meta.p), (size_t)M * K / 32, 3u, 1);
  if (hipGetLastError() != hipSuccess) return 1;
  // panel-form operands, like every operand the library makes for itself (random data has no layout, so any buffer is one)
  GemmArgs g{A.p, sparse ? static_cast<const uint8_t*>(meta.p) : nullptr, B.p, M, N, K, 1, nullptr, 1};
  __bf16* c = static_cast<__bf16*>(C.p);
  constexpr int MF = PROBE_NO_MFMA | PROBE_NO_FRAG, DF = PROBE_NO_DMA | PROBE_NO_FRAG, WMF = PROBE_K_WRAP | MF;
#define FFN24_PROBE_CASE(V) \
  case V: return sparse ? run_gemm_variant<true, V>(g, c, reps, ms_median, mhz) : run_gemm_variant<false, V>(g, c, reps, ms_median, mhz);
  switch (variant) {
    FFN24_PROBE_CASE(0)
    FFN24_PROBE_CASE(PROBE_NO_DMA)
    FFN24_PROBE_CASE(PROBE_NO_FRAG)
    FFN24_PROBE_CASE(MF)
    FFN24_PROBE_CASE(DF)
    FFN24_PROBE_CASE(PROBE_K_WRAP)
    FFN24_PROBE_CASE(WMF)
    FFN24_PROBE_CASE(PROBE_WALK_BANDS)
    FFN24_PROBE_CASE(PROBE_WALK_8x1)
    FFN24_PROBE_CASE(PROBE_PATCH_4x8)
    FFN24_PROBE_CASE(PROBE_PATCH_16x2)
    FFN24_PROBE_CASE(PROBE_UNPACED)
    FFN24_PROBE_CASE(PROBE_FILL_LESS)
    FFN24_PROBE_CASE(PROBE_PERSIST)
    default: return 2;
  }
#undef FFN24_PROBE_CASE
}

int probe_copy(size_t bytes, int reps, double* ms_median) {
  DevBuf src, dst;
  if (src.alloc(bytes) || dst.alloc(bytes)) return 1;
  if (hipMemset(src.p, 1, bytes) != hipSuccess) return 1;
  const size_t n = bytes / 16;
  std::vector<hipEvent_t> ev(reps + 1);
  for (auto& e : ev) if (hipEventCreate(&e) != hipSuccess) return 1;
  auto launch = [&]() { hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, nullptr, static_cast<const u32x4*>(src.p), static_cast<u32x4*>(dst.p), n); };
  launch();
  (void)hipEventRecord(ev[0], nullptr);
  for (int i = 0; i < reps; i++) { launch(); (void)hipEventRecord(ev[i + 1], nullptr); }
  int rc = hipEventSynchronize(ev[reps]) != hipSuccess || hipGetLastError() != hipSuccess;
  std::vector<float> ms(reps, 0.f);
  for (int i = 0; i < reps && !rc; i++) rc = hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]) != hipSuccess;
  for (auto& e : ev) (void)hipEventDestroy(e);
  if (rc) return 1;
  *ms_median = median_of(ms);
  return 0;
}

}  // namespace ffn24
