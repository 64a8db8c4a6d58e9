// fp8 (e4m3) forward kernels: dense-MFMA up-projection with the fused activation + 2:4 + quantisation epilogue, the
// sparse-MFMA down-projection, and the dense fp8 baseline.
// The up-projection and dH GEMMs take their B operand (X8, dY8) in the B panel form: a stage of the dense fp8 loop reads 64
// bytes of every row, half a line when the rows lie 'D' bytes apart, and that costs 5 % (2:4 up-projection) to 11 % (a dense
// GEMM) of the kernel; the copy is a pass over T * D bytes (0.03 ms at T = D = 8192), with the rows of a token permutation
// gathered on the way.
#include "launch_impl.hpp"

namespace ffn24 {

int launch_up_prune24_f8(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, float zscale, float sh,
                         void* Hc8, uint8_t* meta, void* Hdbg, void* Hc16, uint8_t* meta16, hipStream_t s) {
  GemmArgs g{W1t8, nullptr, X8, F, T, D, 1, nullptr, 1};
  EpiPrune24F8::Args ea{static_cast<uint8_t*>(Hc8), meta, static_cast<__bf16*>(Hdbg), b1, F, zscale, sh, static_cast<__bf16*>(Hc16), meta16};
  return launch_gemm<false, EpiPrune24F8, true>(g, ea, s);
}

int launch_up_relu2_f8(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, float zscale, float sh, void* H8, void* H16, void* H8t,
                       hipStream_t s) {
  GemmArgs g{W1t8, nullptr, X8, F, T, D, 1, nullptr, 1};
  EpiRelu2F8::Args ea{static_cast<uint8_t*>(H8), b1, F, zscale, sh, static_cast<__bf16*>(H16), static_cast<uint8_t*>(H8t), T};
  return launch_gemm<false, EpiRelu2F8, true>(g, ea, s);
}

int launch_sp_rowmajor_f8(const void* vals8, const uint8_t* meta, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* C, hipStream_t s) {
  GemmArgs g{vals8, meta, B8, M, N, K, a_panel, nullptr, b_panel};
  EpiRowMajorScaled::Args ea{static_cast<__bf16*>(C), N, scale};
  return launch_gemm<true, EpiRowMajorScaled, true>(g, ea, s);
}

int launch_dense_rowmajor_f8(const void* A8, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* C, hipStream_t s) {
  GemmArgs g{A8, nullptr, B8, M, N, K, a_panel, nullptr, b_panel};
  EpiRowMajorScaled::Args ea{static_cast<__bf16*>(C), N, scale};
  return launch_gemm<false, EpiRowMajorScaled, true>(g, ea, s);
}

// fp8 backward: dH GEMM (A = W2 itself [F][D] in dense panel form, B = dY8 [T][D]) with the pointwise part fused, and the
// sparse GEMM with the transposing store (dW1)
int launch_dh_gather_f8(const void* W2p8, const void* dY8, const void* Hc16, const uint8_t* meta16, int T, int D, int F, float scale, float sdz,
                        void* dZc8, hipStream_t s) {
  GemmArgs g{W2p8, nullptr, dY8, F, T, D, 1, nullptr, 1};
  EpiDGatherF8::Args ea{static_cast<const __bf16*>(Hc16), meta16, static_cast<uint8_t*>(dZc8), F, scale, sdz};
  return launch_gemm<false, EpiDGatherF8, true>(g, ea, s);
}

int launch_sp_colmajor_f8(const void* vals8, const uint8_t* meta, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* Ct,
                          hipStream_t s) {
  GemmArgs g{vals8, meta, B8, M, N, K, a_panel, nullptr, b_panel};
  EpiColMajorScaled::Args ea{static_cast<__bf16*>(Ct), M, scale};
  return launch_gemm<true, EpiColMajorScaled, true>(g, ea, s);
}

int launch_dh_drelu_f8(const void* W2p8, const void* dY8, const void* H16, int T, int D, int F, float scale, float sdz, void* dZ8, void* dZ8t,
                       hipStream_t s) {
  GemmArgs g{W2p8, nullptr, dY8, F, T, D, 1, nullptr, 1};
  EpiDReluF8::Args ea{static_cast<const __bf16*>(H16), static_cast<uint8_t*>(dZ8), static_cast<uint8_t*>(dZ8t), F, T, scale, sdz};
  return launch_gemm<false, EpiDReluF8, true>(g, ea, s);
}

int launch_dense_colmajor_f8(const void* A8, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* Ct, hipStream_t s) {
  GemmArgs g{A8, nullptr, B8, M, N, K, a_panel, nullptr, b_panel};
  EpiColMajorScaled::Args ea{static_cast<__bf16*>(Ct), M, scale};
  return launch_gemm<false, EpiColMajorScaled, true>(g, ea, s);
}

// row-wise-scaled variants (scales per token for the activation operand, per output channel for the weight)
int launch_up_prune24_f8_rowwise(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, const float* sx, const float* sw1,
                                 void* Hc16, uint8_t* meta16, void* Hdbg, uint32_t* rowmax, uint32_t* nnz, hipStream_t s) {
  GemmArgs g{W1t8, nullptr, X8, F, T, D, 1, nullptr, 1};
  EpiPrune24Rw::Args ea{static_cast<__bf16*>(Hc16), meta16, static_cast<__bf16*>(Hdbg), b1, F, sx, sw1, rowmax, nnz};
  if (nnz) {
    EpiPrune24RwT<true>::Args eas{static_cast<__bf16*>(Hc16), meta16, static_cast<__bf16*>(Hdbg), b1, F, sx, sw1, rowmax, nnz};
    return launch_gemm<false, EpiPrune24RwT<true>, true>(g, eas, s);
  }
  return launch_gemm<false, EpiPrune24Rw, true>(g, ea, s);
}

int launch_sp_rowmajor_f8_rowwise_mapped(const void* vals8, const uint8_t* meta, const void* B8, int b_panel, int M, int N, int K, const float* rs, const float* cs,
                                         void* C, const int* rowmap, hipStream_t s) {
  GemmArgs g{vals8, meta, B8, M, N, K, 1, nullptr, b_panel};
  EpiRowMajorRowColMapped::Args ea{static_cast<__bf16*>(C), N, rs, cs, rowmap};
  return launch_gemm<true, EpiRowMajorRowColMapped, true>(g, ea, s);
}

int launch_split_wgrad_f8_rowwise(const void* vals8, const uint8_t* meta, int ns, const void* Ad8, int nd, const void* B8, int N, int K,
                                  const float* rs, const float* cs, void* C, int ldc, const int* rowmap, hipStream_t s) {
  GemmArgs gs{vals8, meta, B8, ns, N, K, 1, nullptr, 1};
  GemmArgs gd{Ad8, nullptr, B8, nd, N, K, 1, nullptr, 1};
  EpiRowMajorRowColMapped::Args eas{static_cast<__bf16*>(C), ldc, rs, cs, rowmap};
  EpiRowMajorRowColMapped::Args ead{static_cast<__bf16*>(C), ldc, rs + ns, cs, rowmap + ns};
  return launch_gemm_pair<EpiRowMajorRowColMapped, true>(gd, ead, gs, eas, s);
}

int launch_up_relu2_f8_rowwise(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, const float* sx, const float* sw1,
                               void* H16, uint32_t* rowmax, void* Ht16, hipStream_t s) {
  GemmArgs g{W1t8, nullptr, X8, F, T, D, 1, nullptr, 1};
  EpiRelu2Rw::Args ea{static_cast<__bf16*>(H16), b1, F, sx, sw1, rowmax, static_cast<__bf16*>(Ht16), T};
  return launch_gemm<false, EpiRelu2Rw, true>(g, ea, s);
}

int launch_dense_rowmajor_f8_rowwise(const void* A8, const void* B8, int b_panel, int M, int N, int K, const float* rs, const float* cs, void* C, hipStream_t s) {
  GemmArgs g{A8, nullptr, B8, M, N, K, 1, nullptr, b_panel};
  EpiRowMajorRowCol::Args ea{static_cast<__bf16*>(C), N, rs, cs};
  return launch_gemm<false, EpiRowMajorRowCol, true>(g, ea, s);
}

int launch_sp_rowmajor_f8_rowwise(const void* vals8, const uint8_t* meta, const void* B8, int b_panel, int M, int N, int K, const float* rs, const float* cs,
                                  void* C, hipStream_t s) {
  GemmArgs g{vals8, meta, B8, M, N, K, 1, nullptr, b_panel};
  EpiRowMajorRowCol::Args ea{static_cast<__bf16*>(C), N, rs, cs};
  return launch_gemm<true, EpiRowMajorRowCol, true>(g, ea, s);
}

// row-wise-scaled backward: the dH GEMM with the pointwise part fused (bf16 compressed dZ + row maxima out), and the sparse GEMM
// with the transposing store and a scale per row and per column (dW1)
int launch_dh_gather_f8_rowwise(const void* W2rp8, const void* dY8r, const void* Hc16, const uint8_t* meta16, int T, int D, int F,
                                const float* sw2_f, const float* sdy_t, void* dZc16, uint32_t* rowmax, hipStream_t s) {
  GemmArgs g{W2rp8, nullptr, dY8r, F, T, D, 1, nullptr, 1};
  EpiDGatherRw::Args ea{static_cast<const __bf16*>(Hc16), meta16, static_cast<__bf16*>(dZc16), F, sw2_f, sdy_t, rowmax};
  return launch_gemm<false, EpiDGatherRw, true>(g, ea, s);
}

int launch_sp_colmajor_f8_rowwise(const void* vals8, const uint8_t* meta, const void* B8, int M, int N, int K, const float* rs, const float* cs,
                                  void* Ct, hipStream_t s) {
  GemmArgs g{vals8, meta, B8, M, N, K, 1, nullptr, 1};
  EpiColMajorRowCol::Args ea{static_cast<__bf16*>(Ct), M, rs, cs};
  return launch_gemm<true, EpiColMajorRowCol, true>(g, ea, s);
}

// dense row-wise-scaled backward: the dH GEMM with the pointwise part fused (bf16 dZ as [T][F] and [F][T], row maxima), and the
// dense GEMM with the transposing store scaled per row and per column
int launch_dh_drelu_f8_rowwise(const void* W2rp8, const void* dY8r, const void* H16, int T, int D, int F, const float* sw2_f, const float* sdy_t,
                               void* dZ16, void* dZt16, uint32_t* rowmax, hipStream_t s) {
  GemmArgs g{W2rp8, nullptr, dY8r, F, T, D, 1, nullptr, 1};
  EpiDReluRw::Args ea{static_cast<const __bf16*>(H16), static_cast<__bf16*>(dZ16), static_cast<__bf16*>(dZt16), F, T, sw2_f, sdy_t, rowmax};
  return launch_gemm<false, EpiDReluRw, true>(g, ea, s);
}

int launch_dense_colmajor_f8_rowwise(const void* A8, const void* B8, int M, int N, int K, const float* rs, const float* cs, void* Ct, hipStream_t s) {
  GemmArgs g{A8, nullptr, B8, M, N, K, 1, nullptr, 1};
  EpiColMajorRowCol::Args ea{static_cast<__bf16*>(Ct), M, rs, cs};
  return launch_gemm<false, EpiColMajorRowCol, true>(g, ea, s);
}

}  // namespace ffn24
