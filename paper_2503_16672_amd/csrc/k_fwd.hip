// Forward kernels of the 2:4 FFN: fused up-projection (dense MFMA + ReLU^2 + keep-2-of-4) and the
// sparse-MFMA down-projection.
#include "launch_impl.hpp"

namespace ffn24 {

int launch_up_prune24(const void* W1, const void* X, const float* b1, int T, int D, int F,
                      void* Hc, uint8_t* meta, void* Hdbg, hipStream_t s) {
  GemmArgs g{W1, nullptr, X, F, T, D};
  EpiPrune24::Args ea{static_cast<__bf16*>(Hc), meta, static_cast<__bf16*>(Hdbg), b1, F};
  return launch_gemm<A_MC, B_KC, EpiPrune24>(g, ea, s);
}

int launch_sp_rowmajor(const void* vals, const uint8_t* meta, const void* B, int b_kc, int M, int N, int K, void* C, hipStream_t s) {
  GemmArgs g{vals, meta, B, M, N, K};
  EpiRowMajor::Args ea{static_cast<__bf16*>(C), N};
  return b_kc ? launch_gemm<A_SP, B_KC, EpiRowMajor>(g, ea, s) : launch_gemm<A_SP, B_NC, EpiRowMajor>(g, ea, s);
}

}  // namespace ffn24
