// Dense Squared-ReLU FFN baseline, part 1: up-projection with ReLU^2 and dH with the derivative.
#include "launch_impl.hpp"

namespace ffn24 {

int launch_up_relu2(const void* W1t, const void* X, const float* b1, int T, int D, int F, void* H, void* Ht, unsigned long long* tele, hipStream_t s) {
  GemmArgs g{W1t, nullptr, X, F, T, D, 1};
  if (tele) {
    EpiRelu2T<true>::Args eas{static_cast<__bf16*>(H), static_cast<__bf16*>(Ht), b1, F, T, tele};
    return launch_gemm<false, EpiRelu2T<true>>(g, eas, s);
  }
  EpiRelu2::Args ea{static_cast<__bf16*>(H), static_cast<__bf16*>(Ht), b1, F, T, nullptr};
  return launch_gemm<false, EpiRelu2>(g, ea, s);
}

int launch_dh_drelu(const void* W2, const void* dY, const void* H, int T, int D, int F, void* dZ, void* dZt, hipStream_t s) {
  GemmArgs g{W2, nullptr, dY, F, T, D, 1};
  EpiDRelu::Args ea{static_cast<const __bf16*>(H), static_cast<__bf16*>(dZ), static_cast<__bf16*>(dZt), F, T};
  return launch_gemm<false, EpiDRelu>(g, ea, s);
}

}  // namespace ffn24
