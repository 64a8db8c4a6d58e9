// Dense Squared-ReLU FFN baseline, part 2: the plain dense GEMMs (down-projection, dX, dW2, dW1).
#include "launch_impl.hpp"

namespace ffn24 {

int launch_dense_rowmajor(const void* A, int a_panel, const void* B, int b_panel, int M, int N, int K, void* C, hipStream_t s) {
  GemmArgs g{A, nullptr, B, M, N, K, a_panel, nullptr, b_panel};
  EpiRowMajor::Args ea{static_cast<__bf16*>(C), N};
  return launch_gemm<false, EpiRowMajor>(g, ea, s);
}

int launch_dense_colmajor(const void* A, int a_panel, const void* B, int b_panel, int M, int N, int K, void* Ct, hipStream_t s) {
  GemmArgs g{A, nullptr, B, M, N, K, a_panel, nullptr, b_panel};
  EpiColMajor::Args ea{static_cast<__bf16*>(Ct), M};
  return launch_gemm<false, EpiColMajor>(g, ea, s);
}

}  // namespace ffn24
