// Backward kernels of the 2:4 FFN that are not shared with the forward.
#include "launch_impl.hpp"

namespace ffn24 {

int launch_dh_gather(const void* W2, const void* dY, const void* Hc, const uint8_t* meta, int T, int D, int F, void* dZc,
                     const int* token_map, hipStream_t s) {
  GemmArgs g{W2, nullptr, dY, F, T, D, 1, token_map};
  EpiDGather::Args ea{static_cast<const __bf16*>(Hc), meta, static_cast<__bf16*>(dZc), F};
  return launch_gemm<false, EpiDGather>(g, ea, s);
}

int launch_sp_colmajor(const void* vals, const uint8_t* meta, int a_panel, const void* B, int b_panel, int M, int N, int K, void* Ct, hipStream_t s) {
  GemmArgs g{vals, meta, B, M, N, K, a_panel, nullptr, b_panel};
  EpiColMajor::Args ea{static_cast<__bf16*>(Ct), M};
  return launch_gemm<true, EpiColMajor>(g, ea, s);
}

// split weight gradient: rows [0, ns) of the permuted feature space from the sparse GEMM over (vals, meta), rows
// [ns, ns + nd) from the dense GEMM over Ad, both against the same B, in one launch; row m goes to C[rowmap[m]][*]
int launch_split_wgrad(const void* vals, const uint8_t* meta, int ns, const void* Ad, int nd, const void* B, int N, int K,
                       void* C, int ldc, const int* rowmap, hipStream_t s) {
  GemmArgs gs{vals, meta, B, ns, N, K, 1, nullptr, 1};
  GemmArgs gd{Ad, nullptr, B, nd, N, K, 1, nullptr, 1};
  EpiRowMajorMapped::Args eas{static_cast<__bf16*>(C), ldc, rowmap};
  EpiRowMajorMapped::Args ead{static_cast<__bf16*>(C), ldc, rowmap + ns};
  return launch_gemm_pair<EpiRowMajorMapped>(gd, ead, gs, eas, s);
}

}  // namespace ffn24
