// Included by the k_*.hip translation units that instantiate the GEMM kernel.
#pragma once
#include "epilogues.hpp"
#include "launch.hpp"

namespace ffn24 {

template <bool SPARSE, class Epi, bool F8 = false, int PROBE = 0>
static int launch_gemm(const GemmArgs& g_in, const typename Epi::Args& ea, hipStream_t s) {
  GemmArgs g = g_in;
  g.clk = tl_gemm_clk;
  auto kern = gemm_kernel<SPARSE, Epi, F8, PROBE>;
  constexpr int lds = Geo<SPARSE, F8>::LDS_TOTAL;
  static std::atomic<bool> configured[MAX_DEVICES] = {};
  if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, configured)) return rc;
  int nblocks = (g.M / TILE_M) * (g.N / TILE_N);
  if constexpr ((PROBE & PROBE_PERSIST) != 0) nblocks = nblocks < PERSIST_WORKGROUPS ? nblocks : PERSIST_WORKGROUPS;
  hipLaunchKernelGGL(kern, dim3(nblocks), dim3(GEMM_THREADS), lds, s, g, ea);
  return (int)hipGetLastError();
}

// dense GEMM gd and sparse GEMM gs in one launch (gemm_pair_kernel)
template <class Epi, bool F8 = false>
static int launch_gemm_pair(const GemmArgs& gd, const typename Epi::Args& ead, const GemmArgs& gs_in, const typename Epi::Args& eas, hipStream_t s) {
  GemmArgs gs = gs_in;
  gs.clk = tl_gemm_clk;
  auto kern = gemm_pair_kernel<Epi, F8>;
  constexpr int lds = Geo<true, F8>::LDS_TOTAL > Geo<false, F8>::LDS_TOTAL ? Geo<true, F8>::LDS_TOTAL : Geo<false, F8>::LDS_TOTAL;
  static std::atomic<bool> configured[MAX_DEVICES] = {};
  if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, configured)) return rc;
  int nd_tiles = (gd.M / TILE_M) * (gd.N / TILE_N), ns_tiles = (gs.M / TILE_M) * (gs.N / TILE_N);
  hipLaunchKernelGGL(kern, dim3(nd_tiles + ns_tiles), dim3(GEMM_THREADS), lds, s, gd, ead, nd_tiles, gs, eas);
  return (int)hipGetLastError();
}

}  // namespace ffn24
