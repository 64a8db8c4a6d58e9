// Forward kernels of the 2:4 FFN: fused up-projection (dense MFMA + ReLU^2 + keep-2-of-4) and the
// sparse-MFMA GEMM with a row-major result (down-projection, dX, dW2).
#include "launch_impl.hpp"

namespace ffn24 {

int launch_up_prune24(const void* W1t, const void* X, const float* b1, int T, int D, int F,
                      void* Hc, uint8_t* meta, void* Hdbg, uint32_t* nnz, unsigned long long* tele, const int* token_map, hipStream_t s) {
  GemmArgs g{W1t, nullptr, X, F, T, D, 1, token_map};
  EpiPrune24::Args ea{static_cast<__bf16*>(Hc), meta, static_cast<__bf16*>(Hdbg), b1, F, nullptr, nullptr};
  if (nnz || tele) {
    EpiPrune24T<true>::Args eas{static_cast<__bf16*>(Hc), meta, static_cast<__bf16*>(Hdbg), b1, F, nnz, tele};
    return launch_gemm<false, EpiPrune24T<true>>(g, eas, s);
  }
  return launch_gemm<false, EpiPrune24>(g, ea, s);
}

int launch_sp_rowmajor(const void* vals, const uint8_t* meta, int a_panel, const void* B, int b_panel, int M, int N, int K, void* C, hipStream_t s) {
  GemmArgs g{vals, meta, B, M, N, K, a_panel, nullptr, b_panel};
  EpiRowMajor::Args ea{static_cast<__bf16*>(C), N};
  return launch_gemm<true, EpiRowMajor>(g, ea, s);
}

int launch_sp_rowmajor_mapped(const void* vals, const uint8_t* meta, int a_panel, const void* B, int b_panel, int M, int N, int K, void* C,
                              const int* rowmap, hipStream_t s) {
  GemmArgs g{vals, meta, B, M, N, K, a_panel, nullptr, b_panel};
  EpiRowMajorMapped::Args ea{static_cast<__bf16*>(C), N, rowmap};
  return launch_gemm<true, EpiRowMajorMapped>(g, ea, s);
}

}  // namespace ffn24
