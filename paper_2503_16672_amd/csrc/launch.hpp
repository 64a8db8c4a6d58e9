// Host-side launch helper for the GEMM core and the list of launchers each translation unit provides.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ffn24 {

struct GemmArgs;

// Plain-pointer launchers (definitions spread over k_*.hip so they compile in parallel).
// All return a hipError_t cast to int (0 = success); shapes must already be validated by the caller:
// M % 256 == 0, N % 256 == 0, K % 64 == 0, 16-byte aligned pointers.

// up-projection, rows = features: A = W1 [D][F] (feature-contiguous), B = X [T][D]
int launch_up_prune24(const void* W1, const void* X, const float* b1, int T, int D, int F,
                      void* Hc, uint8_t* meta, void* Hdbg, hipStream_t s);
int launch_up_relu2(const void* W1, const void* X, const float* b1, int T, int D, int F, void* H, hipStream_t s);
// C[M][N] = A24[M][K] * B ; B stored [K][N] (b_kc = 0) or [N][K] (b_kc = 1)
int launch_sp_rowmajor(const void* vals, const uint8_t* meta, const void* B, int b_kc, int M, int N, int K, void* C, hipStream_t s);
// out[N][M] = (A24[M][K] * B[K][N])^T
int launch_sp_nc_colmajor(const void* vals, const uint8_t* meta, const void* B, int M, int N, int K, void* Ct, hipStream_t s);
// dH = dY W2^T with rows = features: A = W2 [F][D], B = dY [T][D]; pointwise part fused
int launch_dh_gather(const void* W2, const void* dY, const void* Hc, const uint8_t* meta, int T, int D, int F, void* dZc, hipStream_t s);
int launch_dh_drelu(const void* W2, const void* dY, const void* H, int T, int D, int F, void* dZ, hipStream_t s);
// dense GEMMs
int launch_kc_nc_rowmajor(const void* A, const void* B, int M, int N, int K, void* C, hipStream_t s);   // A [M][K], B [K][N]
int launch_kc_kc_rowmajor(const void* A, const void* B, int M, int N, int K, void* C, hipStream_t s);   // A [M][K], B [N][K]
int launch_mc_nc_rowmajor(const void* A, const void* B, int M, int N, int K, void* C, hipStream_t s);   // A [K][M], B [K][N]
int launch_mc_nc_colmajor(const void* A, const void* B, int M, int N, int K, void* Ct, hipStream_t s);  // out [N][M]
// streaming kernels
int launch_sparsify24(const void* H, int64_t rows, int64_t cols, void* vals, uint8_t* meta, hipStream_t s);
int launch_featurewise24(const void* Hc, const uint8_t* meta, const void* dZc, int T, int F,
                         void* Hc_t, uint8_t* meta_t, void* dZc_t, hipStream_t s);

}  // namespace ffn24
