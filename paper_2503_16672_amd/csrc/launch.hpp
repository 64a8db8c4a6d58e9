// Host-side launchers each translation unit provides (definitions spread over k_*.hip so they compile in parallel).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

namespace ffn24 {

// Opts a kernel in to `bytes` of dynamic LDS (more than 64 KiB needs it), once per device; `done` holds one flag per
// device and belongs to the call site.  Threads that race here all make the same idempotent runtime call; the flag
// only saves repeating it on later launches.
constexpr int MAX_DEVICES = 64;
inline int ensure_dynamic_lds(const void* kern, int bytes, std::atomic<bool> (&done)[MAX_DEVICES]) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= MAX_DEVICES) return (int)hipErrorInvalidDevice;
  if (!done[dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return (int)e;
    done[dev].store(true, std::memory_order_release);
  }
  return 0;
}

// Where the GEMM launches of the calling thread store their clock samples (gemm_core.hpp, GemmArgs::clk): set by the
// C-ABI layer around a launch when the context profiles, NULL otherwise.
inline thread_local unsigned long long* tl_gemm_clk = nullptr;
constexpr int CLK_SLOTS = 64;
constexpr int PERSIST_WORKGROUPS = 256;   // one per CU of the chip (gfx950: 256 CUs; a 256 x 256 tile's registers and LDS fill a CU)   // workgroups of a launch that store a clock sample (a pair of 64-bit counts each)

// Telemetry counters (the sparsity level of the activation and what 2:4 keeps of it): TELE_SLOTS 64-bit slots per
// quantity, each in a 128-byte line of its own and summed when read, so that the atomics of a launch spread over many
// lines instead of queueing on one.  Slot s of quantity k is word tele_index(k, s).
constexpr int TELE_SLOTS = 64, TELE_STRIDE = 16;
enum { TELE_NONZERO = 0, TELE_KEPT_TOK = 1, TELE_KEPT_FEAT = 2, TELE_KINDS = 3 };
constexpr int TELE_WORDS = TELE_KINDS * TELE_SLOTS * TELE_STRIDE;   // 64-bit words in the buffer
__host__ __device__ constexpr int tele_index(int kind, int slot) { return (kind * TELE_SLOTS + (slot & (TELE_SLOTS - 1))) * TELE_STRIDE; }

// All return a hipError_t cast to int (0 = success); shapes must already be validated by the caller:
// M % 256 == 0, N % 256 == 0, K % 64 == 0, 16-byte aligned pointers.  Every GEMM operand is K-contiguous.

// up-projection with rows = hidden features: A = W1^T [F][D] in dense panel form, B = X [T][D]
// nnz (may be NULL): [F] per-feature non-zero counts, accumulated with atomics (zeroed by the caller)
// token_map (may be NULL, also below): column n of the GEMM (position n inside the FFN) is token token_map[n] of X / dY
// tele (may be NULL, also below): the telemetry slots (TELE_KINDS x TELE_SLOTS 64-bit counters, epilogues.hpp) the
// launch adds its counts to
int launch_up_prune24(const void* W1t, const void* X, const float* b1, int T, int D, int F,
                      void* Hc, uint8_t* meta, void* Hdbg, uint32_t* nnz, unsigned long long* tele, const int* token_map, hipStream_t s);
int launch_up_relu2(const void* W1t, const void* X, const float* b1, int T, int D, int F, void* H, void* Ht, unsigned long long* tele, hipStream_t s);
// C[M][N] = A24[M][K] * B[N][K]^T; a_panel: (vals, meta) are in panel form instead of row-major;
// b_panel (also below): B is in the B panel form of gemm_core.hpp instead of row-major
int launch_sp_rowmajor(const void* vals, const uint8_t* meta, int a_panel, const void* B, int b_panel, int M, int N, int K, void* C, hipStream_t s);
// out[N][M] = (A24[M][K] * B[N][K]^T)^T
int launch_sp_colmajor(const void* vals, const uint8_t* meta, int a_panel, const void* B, int b_panel, int M, int N, int K, void* Ct, hipStream_t s);
// dH = dY W2^T with rows = hidden features: A = W2 [F][D] in dense panel form, B = dY [T][D]; pointwise part fused
int launch_dh_gather(const void* W2, const void* dY, const void* Hc, const uint8_t* meta, int T, int D, int F, void* dZc,
                     const int* token_map, hipStream_t s);
// C[rowmap[m]][N] = (A24 * B^T)[m][N]: the result rows go back to their tokens
int launch_sp_rowmajor_mapped(const void* vals, const uint8_t* meta, int a_panel, const void* B, int b_panel, int M, int N, int K, void* C,
                              const int* rowmap, hipStream_t s);
int launch_dh_drelu(const void* W2, const void* dY, const void* H, int T, int D, int F, void* dZ, void* dZt, hipStream_t s);
// split weight gradient (operands in panel form): rows [0, ns) from the sparse GEMM over (vals, meta) [ns][K], rows
// [ns, ns + nd) from the dense GEMM over Ad [nd][K], both against B [N][K] (B panel form), one launch; row m goes to C[rowmap[m]][*]
int launch_split_wgrad(const void* vals, const uint8_t* meta, int ns, const void* Ad, int nd, const void* B, int N, int K,
                       void* C, int ldc, const int* rowmap, hipStream_t s);
// feature partition for the split (one workgroup): the n_dense features with the largest counts (ties: lower index)
// become rows [F - n_dense, F) of the split operands, the others rows [0, F - n_dense), both in ascending feature order
// (max_count: an upper bound of every count, the number of tokens)
int launch_split_partition(const uint32_t* nnz, int F, int n_dense, int max_count, int* row_of_feat, int* feat_of_row, hipStream_t s);
// feature-wise re-compression with the split: sparse features as in launch_featurewise24 (panel form, row = row_of_feat),
// dense features as plain [n_dense][T] rows of H24 and dZ24 in dense panel form; hmax, zmax (may be NULL, zeroed by the caller):
// the largest stored magnitude word of every output row, sparse rows [0, n_sparse) first, then the dense ones
int launch_featurewise24_split(const void* Hc, const uint8_t* meta, const void* dZc, int T, int F, const int* row_of_feat, int n_sparse,
                               void* Hc_t, uint8_t* meta_t, void* dZc_t, void* Hdn_t, void* dZdn_t, unsigned long long* tele,
                               uint32_t* hmax, uint32_t* zmax, hipStream_t s);
// dense GEMMs: A [M][K] (a_panel: in dense panel form), B [N][K]
int launch_dense_rowmajor(const void* A, int a_panel, const void* B, int b_panel, int M, int N, int K, void* C, hipStream_t s);
int launch_dense_colmajor(const void* A, int a_panel, const void* B, int b_panel, int M, int N, int K, void* Ct, hipStream_t s);
// fp8 e4m3 forward (per-tensor scales).  W1t8 [F][D] in dense panel form (64-byte pieces = 64 k), X8 [T][D];
// compressed activation in the fp8 panel form (64 stored bytes + 16 metadata bytes per 128 k); bf16 results.
// Hc16, meta16 (may be NULL): also the kept values before quantisation (bf16) and their metadata, in the bf16 panel form
int launch_up_prune24_f8(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, float zscale, float sh,
                         void* Hc8, uint8_t* meta, void* Hdbg, void* Hc16, uint8_t* meta16, hipStream_t s);
// fp8 backward.  dH GEMM with rows = hidden features: A = W2 itself [F][D] e4m3 in dense panel form, B = dY8 [T][D];
// dZc8 = e4m3(scale * acc * 2 sqrt(h) / sdz) on the kept positions (fp8 panel form), h from (Hc16, meta16)
int launch_dh_gather_f8(const void* W2p8, const void* dY8, const void* Hc16, const uint8_t* meta16, int T, int D, int F, float scale, float sdz,
                        void* dZc8, hipStream_t s);
// out[N][M] = bf16(scale * (A24 . B^T))^T, e4m3 operands
int launch_sp_colmajor_f8(const void* vals8, const uint8_t* meta, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* Ct,
                          hipStream_t s);
// feature-wise re-compression of the fp8 operands (all in the fp8 panel form): T, F multiples of 128
int launch_featurewise24_f8(const void* Hc8, const uint8_t* meta, const void* dZc8, int T, int F, void* Hc8_t, uint8_t* meta_t, void* dZc8_t, hipStream_t s);
// H16, H8t (may be NULL): also the activation as bf16 [T][F] (dense bf16 panel form) and the codes transposed, [F][T] (dense fp8 panel form)
int launch_up_relu2_f8(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, float zscale, float sh, void* H8, void* H16, void* H8t,
                       hipStream_t s);
// dense fp8 backward: dH GEMM with dZ8 = e4m3(scale * acc * 2 sqrt(h) / sdz) stored as [T][F] and [F][T]; transposing dense GEMM
int launch_dh_drelu_f8(const void* W2p8, const void* dY8, const void* H16, int T, int D, int F, float scale, float sdz, void* dZ8, void* dZ8t,
                       hipStream_t s);
int launch_dense_colmajor_f8(const void* A8, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* Ct, hipStream_t s);
int launch_sp_rowmajor_f8(const void* vals8, const uint8_t* meta, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* C, hipStream_t s);
int launch_dense_rowmajor_f8(const void* A8, int a_panel, const void* B8, int b_panel, int M, int N, int K, float scale, void* C, hipStream_t s);
// row-wise-scaled fp8 forward: sx [T], sw1 [F], sw2 [N]; the up-projection writes bf16 kept values (bf16 panel form)
// and raises rowmax [T] (bf16 words; zeroed by the caller); quantise_rows turns them into the fp8 panel form with
// sh[t] = rowmax[t] / 448 (1 for an all-zero row), which it also writes out; nnz (may be NULL) as in launch_up_prune24
int launch_up_prune24_f8_rowwise(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, const float* sx, const float* sw1,
                                 void* Hc16, uint8_t* meta16, void* Hdbg, uint32_t* rowmax, uint32_t* nnz, hipStream_t s);
// split weight gradient of the row-wise fp8 backward (operands e4m3 in panel form): as launch_split_wgrad, with the result row m
// scaled by rs[m] (scales in row order of the permuted feature space, sparse rows first) and column n by cs[n]
int launch_split_wgrad_f8_rowwise(const void* vals8, const uint8_t* meta, int ns, const void* Ad8, int nd, const void* B8, int N, int K,
                                  const float* rs, const float* cs, void* C, int ldc, const int* rowmap, hipStream_t s);
// the dense row-wise-scaled baseline: up-projection writing every activation as bf16 (dense panel form) and raising rowmax;
// quantise_rows_dense turns them into e4m3 (dense fp8 panel form) with sh[t] = rowmax[t] / 448; dense GEMM with sh[t] sw2[n]
// (Ht16, may be NULL: the activation once more as the bf16 [F][T] operand, dense panel form)
int launch_up_relu2_f8_rowwise(const void* W1t8, const void* X8, const float* b1, int T, int D, int F, const float* sx, const float* sw1,
                               void* H16, uint32_t* rowmax, void* Ht16, hipStream_t s);
// dense row-wise-scaled backward: dH GEMM with the derivative fused, bf16 dZ out as [T][F] and [F][T] (dense panel forms) and
// rowmax[t]; per-row maxima of a bf16 dense-panel matrix (rmax zeroed by the caller); dense GEMM with the transposing store and a
// scale per row and per column
int launch_dh_drelu_f8_rowwise(const void* W2rp8, const void* dY8r, const void* H16, int T, int D, int F, const float* sw2_f, const float* sdy_t,
                               void* dZ16, void* dZt16, uint32_t* rowmax, hipStream_t s);
int launch_rowmax_dense(const void* X16, int R, int C, uint32_t* rmax, hipStream_t s);
int launch_dense_colmajor_f8_rowwise(const void* A8, const void* B8, int M, int N, int K, const float* rs, const float* cs, void* Ct, hipStream_t s);
int launch_quantise_rows_dense(const void* H16, const uint32_t* rowmax, int T, int F, void* H8, float* sh, hipStream_t s);
int launch_dense_rowmajor_f8_rowwise(const void* A8, const void* B8, int b_panel, int M, int N, int K, const float* rs, const float* cs, void* C, hipStream_t s);
int launch_quantise_rows(const void* Hc16, const uint8_t* meta16, const uint32_t* rowmax, int T, int F, void* Hc8, uint8_t* meta8, float* sh, hipStream_t s);
int launch_sp_rowmajor_f8_rowwise(const void* vals8, const uint8_t* meta, const void* B8, int b_panel, int M, int N, int K, const float* rs, const float* cs,
                                  void* C, hipStream_t s);
// the same with result row m stored as row rowmap[m] (token permutation: the rows go back to their tokens; rs stays in row order)
int launch_sp_rowmajor_f8_rowwise_mapped(const void* vals8, const uint8_t* meta, const void* B8, int b_panel, int M, int N, int K, const float* rs, const float* cs,
                                         void* C, const int* rowmap, hipStream_t s);
// row-wise-scaled fp8 backward: dH GEMM (A = W2 quantised per hidden feature, dense fp8 panel form; B = dY quantised per token)
// with the derivative and the gather fused: bf16 compressed dZ (bf16 panel form) and rowmax[t] = largest magnitude word of a row;
// the sparse GEMM with the transposing store scaled per row and per column
int launch_dh_gather_f8_rowwise(const void* W2rp8, const void* dY8r, const void* Hc16, const uint8_t* meta16, int T, int D, int F,
                                const float* sw2_f, const float* sdy_t, void* dZc16, uint32_t* rowmax, hipStream_t s);
int launch_sp_colmajor_f8_rowwise(const void* vals8, const uint8_t* meta, const void* B8, int M, int N, int K, const float* rs, const float* cs,
                                  void* Ct, hipStream_t s);
// feature-wise kernel on bf16 panel-form operands that also raises hmax[f], zmax[f] (zeroed by the caller) to the largest
// stored magnitude word of each output row
int launch_featurewise24_rowmax(const void* Hc, const uint8_t* meta, const void* dZc, int T, int F, void* Hc_t, uint8_t* meta_t, void* dZc_t,
                                uint32_t* hmax, uint32_t* zmax, hipStream_t s);
// byte matrix [R][C] (C % 64 == 0, R % 256 == 0) -> dense fp8 panel form, or the B panel form if b_form
int launch_panelise8(const void* in, int R, int C, void* out, int b_form, hipStream_t s);
// the same with row r taken from memory row in_rowmap[r] (may be NULL)
int launch_panelise8_rows(const void* in, int R, int C, void* out, int b_form, const int* in_rowmap, hipStream_t s);
// bf16 X [R][C] (C % 8 == 0) -> e4m3 codes [R][C] and one scale per row (axis 1, scales [R]) or per column (axis 0, scales [C]; the
// buffer also holds the column maxima while the call runs)
int launch_quantise_bf16(const void* X, int64_t R, int64_t C, int axis, void* codes, float* scales, hipStream_t s);
// streaming kernels
// p[0..n) = 0 (a kernel, not a memset node)
int launch_zero32(uint32_t* p, size_t n, hipStream_t s);
int launch_sparsify24(const void* H, int64_t rows, int64_t cols, void* vals, uint8_t* meta, hipStream_t s);
// bf16 in, pick on the bf16 words, kept values quantised to e4m3(kept / scale); cols % 8 == 0
int launch_sparsify24_quant(const void* H, int64_t rows, int64_t cols, float scale, void* vals8, uint8_t* meta, hipStream_t s);
// e4m3 in and out, pick on the code bytes; cols % 16 == 0
int launch_sparsify24_bytes(const void* H8, int64_t rows, int64_t cols, void* vals8, uint8_t* meta, hipStream_t s);
// panel: inputs and outputs are in panel form (the library's own buffers) instead of row-major
int launch_featurewise24(const void* Hc, const uint8_t* meta, const void* dZc, int T, int F,
                         void* Hc_t, uint8_t* meta_t, void* dZc_t, int panel, unsigned long long* tele, hipStream_t s);
// out[0] = elements, out[1..3] = the sums of the telemetry slots (non-zero, kept token-wise, kept feature-wise), out[4] = path
int launch_tele_sum(const unsigned long long* tele, long long elements, long long path, long long* out, hipStream_t s);
// panel form -> row-major copy of a compressed operand: rows x npanels pieces of `piece_bytes` (64 values / 8 or 16 metadata)
int launch_unpanel(const void* src, int rows, int npanels, int piece_bytes, void* dst, hipStream_t s);
// in [R][C] -> out [C][R] (R % 64 == 0, C % 128 == 0); out_form: 0 row-major, 1 dense panel form (A operands), 2 B panel form
// (gemm_core.hpp; both then need C % 256 == 0);
// in_panel (may be NULL): also a panel-form copy of `in` itself (then R % 256 == 0), in the B form if in_panel_b
// in_rowmap (may be NULL): row r of the input is taken from memory row in_rowmap[r]
int launch_transpose(const void* in, int R, int C, void* out, int out_form, void* in_panel, int in_panel_b, const int* in_rowmap, hipStream_t s);
// the same for 1-byte elements (fp8): in [R][C] -> out [C][R] (R % 64 == 0, C % 256 == 0); panel forms: 64-byte pieces of 64 k
// in_panel (may be NULL): also a panel-form copy of `in` itself (R % 256 == 0, C % 64 == 0), in the B form if in_panel_b
int launch_transpose8(const void* in, int R, int C, void* out, int out_form, void* in_panel, int in_panel_b, hipStream_t s);
// the same without the panel copy, input row r taken from memory row in_rowmap[r] (may be NULL)
int launch_transpose8_rows(const void* in, int R, int C, void* out, int out_form, const int* in_rowmap, hipStream_t s);
// dst[i] = src[map[i]], i < n
int launch_gather_f32(const float* src, const int* map, int n, float* dst, hipStream_t s);

// ------------------------------------------------------------------------------------------------
// measurement probes (k_probe.hip); they allocate their own buffers and wait for their own work
// ------------------------------------------------------------------------------------------------
// Register-resident matrix-op loop, one wave per SIMD on every CU, random operands: cycles per op and wave (shader-clock
// ticks), the clock it ran at, and the chip-wide rate.  kind: 0 dense bf16 32x32x16, 1 sparse bf16 32x32x32,
// 2 dense fp8 32x32x64, 3 sparse fp8 32x32x64.
int probe_mfma_rate(int kind, int iters, double* cycles_per_op, double* mhz, double* tflops_dense_equivalent);
// The GEMM core on pseudo-random panel-form operands with ingredients taken out (`variant` = mask of PROBE_* in
// gemm_core.hpp; supported: 0, NO_DMA, NO_FRAG, NO_MFMA | NO_FRAG, NO_DMA | NO_FRAG, K_WRAP, K_WRAP | NO_MFMA | NO_FRAG):
// median kernel duration over `reps` launches and the clock it ran at.
int probe_gemm(int sparse, int variant, int M, int N, int K, int reps, double* ms_median, double* mhz);
// Plain device-to-device copy kernel of `bytes` bytes (16 per work item): GB/s read + written.
int probe_copy(size_t bytes, int reps, double* ms_median);

}  // namespace ffn24
