// Dense Squared-ReLU FFN baseline, part 2: dX and the two weight-gradient GEMMs.
#include "launch_impl.hpp"

namespace ffn24 {

int launch_kc_kc_rowmajor(const void* A, const void* B, int M, int N, int K, void* C, hipStream_t s) {
  GemmArgs g{A, nullptr, B, M, N, K};
  EpiRowMajor::Args ea{static_cast<__bf16*>(C), N};
  return launch_gemm<A_KC, B_KC, EpiRowMajor>(g, ea, s);
}

int launch_mc_nc_rowmajor(const void* A, const void* B, int M, int N, int K, void* C, hipStream_t s) {
  GemmArgs g{A, nullptr, B, M, N, K};
  EpiRowMajor::Args ea{static_cast<__bf16*>(C), N};
  return launch_gemm<A_MC, B_NC, EpiRowMajor>(g, ea, s);
}

int launch_mc_nc_colmajor(const void* A, const void* B, int M, int N, int K, void* Ct, hipStream_t s) {
  GemmArgs g{A, nullptr, B, M, N, K};
  EpiColMajor::Args ea{static_cast<__bf16*>(Ct), M};
  return launch_gemm<A_MC, B_NC, EpiColMajor>(g, ea, s);
}

}  // namespace ffn24
