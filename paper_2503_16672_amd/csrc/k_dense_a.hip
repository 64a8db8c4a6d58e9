// Dense Squared-ReLU FFN baseline, part 1: up-projection with ReLU^2, down-projection, dH with the derivative.
#include "launch_impl.hpp"

namespace ffn24 {

int launch_up_relu2(const void* W1, const void* X, const float* b1, int T, int D, int F, void* H, hipStream_t s) {
  GemmArgs g{W1, nullptr, X, F, T, D};
  EpiRelu2::Args ea{static_cast<__bf16*>(H), b1, F};
  return launch_gemm<A_MC, B_KC, EpiRelu2>(g, ea, s);
}

int launch_kc_nc_rowmajor(const void* A, const void* B, int M, int N, int K, void* C, hipStream_t s) {
  GemmArgs g{A, nullptr, B, M, N, K};
  EpiRowMajor::Args ea{static_cast<__bf16*>(C), N};
  return launch_gemm<A_KC, B_NC, EpiRowMajor>(g, ea, s);
}

int launch_dh_drelu(const void* W2, const void* dY, const void* H, int T, int D, int F, void* dZ, hipStream_t s) {
  GemmArgs g{W2, nullptr, dY, F, T, D};
  EpiDRelu::Args ea{static_cast<const __bf16*>(H), static_cast<__bf16*>(dZ), F};
  return launch_gemm<A_KC, B_KC, EpiDRelu>(g, ea, s);
}

}  // namespace ffn24
