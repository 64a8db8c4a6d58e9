// Streaming (HBM-bound) kernels: the standalone 2:4 compression of an activation matrix, the feature-wise
// (along-token) re-compression the weight-gradient GEMMs need, and the bf16 matrix transpose that brings a GEMM
// operand into K-contiguous form.
#include "epilogues.hpp"
#include "launch.hpp"

namespace ffn24 {

// Streaming accesses: every byte these kernels touch is read or written once, so loads and stores carry the non-temporal
// hint (measured on a plain copy: 6.0-6.5 TB/s with it, 5.6-6.1 without).
template <class T> __device__ __forceinline__ T ld_stream(const T* p) { return __builtin_nontemporal_load(p); }
template <class T> __device__ __forceinline__ void st_stream(T* p, T v) { __builtin_nontemporal_store(v, p); }

// key of a bf16 storage word at position i of its group: ((magnitude << 2) | (3 - i)) << 1 | sign.
// The sign rides in the lowest bit, below the position, so it never takes part in the ordering.
__device__ __forceinline__ uint32_t key_of(uint32_t w, uint32_t i) { return ((((w & 0x7FFFu) << 2) | (3u - i)) << 1) | (w >> 15); }
__device__ __forceinline__ uint32_t word_of(uint32_t key) { return (key >> 3) | ((key & 1u) << 15); }

// pick on keys that carry the sign bit: strip it for the position arithmetic of pick24_keys
__device__ __forceinline__ uint32_t pick24_words(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, uint32_t& pair) {
  uint32_t k0 = key_of(w0, 0), k1 = key_of(w1, 1), k2 = key_of(w2, 2), k3 = key_of(w3, 3);
  uint32_t a = max(k0, k1), b = min(k0, k1), c = max(k2, k3), d = min(k2, k3);
  uint32_t top = max(a, c);
  uint32_t e = max(b, d);
  uint32_t second = max(min(a, c), min(max(a, c), e));
  uint32_t ct = (top >> 1) & 3u, cs = (second >> 1) & 3u;
  bool top_first = ct > cs;
  uint32_t kf = top_first ? top : second, ks = top_first ? second : top;
  pair = word_of(kf) | (word_of(ks) << 16);
  uint32_t cmax = max(ct, cs), cmin = min(ct, cs);
  return (cmax | (cmin << 2)) ^ 15u;
}

// Standalone sparsify24 (Sec. 2 of the paper, first paragraph): each thread takes 8 consecutive elements
// (two groups): one 16-byte load, one 8-byte store of kept values, one metadata byte.  The matrix is
// processed as a flat array, which is valid because cols % 8 == 0.
__global__ void __launch_bounds__(256) sparsify24_kernel(const u32x4* __restrict__ in, int64_t n_oct,
                                                         u32x2* __restrict__ vals, uint8_t* __restrict__ meta) {
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < n_oct; o += stride) {
    u32x4 v = ld_stream(in + o);
    uint32_t p0, p1;
    uint32_t n0 = pick24_words(v[0] & 0xFFFFu, v[0] >> 16, v[1] & 0xFFFFu, v[1] >> 16, p0);
    uint32_t n1 = pick24_words(v[2] & 0xFFFFu, v[2] >> 16, v[3] & 0xFFFFu, v[3] >> 16, p1);
    st_stream(vals + o, u32x2{p0, p1});
    st_stream(meta + o, (uint8_t)(n0 | (n1 << 4)));
  }
}

// Standalone activation-side kernel of Sec. 2 (sparsification and FP8 quantisation in one pass): the pick is made on the
// bf16 words exactly as above, the two kept values of each group are then quantised, e4m3(kept / scale), saturating.
// Per work item 8 elements: one 16-byte load, 4 code bytes, one metadata byte (2.625 bytes per element in all).
__global__ void __launch_bounds__(256) sparsify24_quant_kernel(const u32x4* __restrict__ in, int64_t n_oct, float scale,
                                                               uint32_t* __restrict__ vals8, uint8_t* __restrict__ meta) {
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < n_oct; o += stride) {
    u32x4 v = ld_stream(in + o);
    uint32_t p0, p1;
    uint32_t n0 = pick24_words(v[0] & 0xFFFFu, v[0] >> 16, v[1] & 0xFFFFu, v[1] >> 16, p0);
    uint32_t n1 = pick24_words(v[2] & 0xFFFFu, v[2] >> 16, v[3] & 0xFFFFu, v[3] >> 16, p1);
    uint32_t q = cvt_e4m3x2(bf16_lo_to_f32(p0) / scale, bf16_hi_to_f32(p0) / scale, 0u, false);
    q = cvt_e4m3x2(bf16_lo_to_f32(p1) / scale, bf16_hi_to_f32(p1) / scale, q, true);
    st_stream(vals8 + o, q);
    st_stream(meta + o, (uint8_t)(n0 | (n1 << 4)));
  }
}

// 2:4 compression of a tensor that already is e4m3: the pick on the code bytes (sign cleared, as integers; ties -> lower
// index).  A work item takes 16 bytes (four groups) and writes 8 code bytes and 2 metadata bytes.
__global__ void __launch_bounds__(256) sparsify24_bytes_kernel(const u32x4* __restrict__ in, int64_t n16,
                                                               u32x2* __restrict__ vals8, uint16_t* __restrict__ meta) {
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < n16; o += stride) {
    u32x4 v = ld_stream(in + o);
    uint32_t out[2] = {0u, 0u}, m = 0u;
#pragma unroll
    for (int g = 0; g < 4; g++) {
      uint32_t w = v[g];
      uint32_t b0 = w & 0xFFu, b1 = (w >> 8) & 0xFFu, b2 = (w >> 16) & 0xFFu, b3 = w >> 24;
      uint32_t k0 = ((b0 & 0x7Fu) << 2) | 3u, k1 = ((b1 & 0x7Fu) << 2) | 2u, k2 = ((b2 & 0x7Fu) << 2) | 1u, k3 = (b3 & 0x7Fu) << 2;
      uint32_t kf, ks;
      uint32_t nib = pick24_keys(k0, k1, k2, k3, kf, ks);
      uint32_t i0 = nib & 3u, i1 = nib >> 2;
      uint32_t a = (w >> (8 * i0)) & 0xFFu, b = (w >> (8 * i1)) & 0xFFu;
      out[g >> 1] |= (a | (b << 8)) << (16 * (g & 1));
      m |= nib << (4 * g);
    }
    st_stream(vals8 + o, u32x2{out[0], out[1]});
    st_stream(meta + o, (uint16_t)m);
  }
}

int launch_sparsify24_quant(const void* H, int64_t rows, int64_t cols, float scale, void* vals8, uint8_t* meta, hipStream_t s) {
  int64_t n_oct = rows * cols / 8;
  if (n_oct == 0) return 0;
  int64_t blocks = (n_oct + 255) / 256;
  if (blocks > 0x7FFFFFFF) blocks = 0x7FFFFFFF;   // one work item per thread: the fastest shape for a streaming kernel here
  hipLaunchKernelGGL(sparsify24_quant_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4*>(H), n_oct, scale,
                     static_cast<uint32_t*>(vals8), meta);
  return (int)hipGetLastError();
}

int launch_sparsify24_bytes(const void* H8, int64_t rows, int64_t cols, void* vals8, uint8_t* meta, hipStream_t s) {
  int64_t n16 = rows * cols / 16;
  if (n16 == 0) return 0;
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > 0x7FFFFFFF) blocks = 0x7FFFFFFF;   // one work item per thread: the fastest shape for a streaming kernel here
  hipLaunchKernelGGL(sparsify24_bytes_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4*>(H8), n16,
                     static_cast<u32x2*>(vals8), reinterpret_cast<uint16_t*>(meta));
  return (int)hipGetLastError();
}

int launch_sparsify24(const void* H, int64_t rows, int64_t cols, void* vals, uint8_t* meta, hipStream_t s) {
  int64_t n_oct = rows * cols / 8;
  if (n_oct == 0) return 0;
  int64_t blocks = (n_oct + 255) / 256;
  if (blocks > 0x7FFFFFFF) blocks = 0x7FFFFFFF;   // one work item per thread: the fastest shape for a streaming kernel here
  hipLaunchKernelGGL(sparsify24_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4*>(H), n_oct,
                     static_cast<u32x2*>(vals), meta);
  return (int)hipGetLastError();
}

// Feature-wise 2:4 on top of the token-wise mask (Sec. 2, last paragraph; Fig. 2c).
// Input: token-wise compressed Hc [T][F/2] + meta [T][F/8], and optionally dZc [T][F/2] with the same metadata.
// Output: for every feature, groups of 4 consecutive tokens of the pruned activation keep their top-2:
//   Hc_t [F][T/2], meta_t [F][T/8], and dZc_t [F][T/2] = dZ at the positions picked for H.
// One workgroup handles 64 tokens x 64 features: decompress into LDS, then each work item takes one feature
// and 8 consecutive tokens (two groups).  PANEL: inputs and outputs are in the panel form of gemm_core.hpp (the
// workgroup's input is then one contiguous 4 KiB run per tensor and it writes one contiguous 4 KiB run; 128-token tiles, with
// twice the LDS per workgroup and half the workgroups per CU, ran at 5.0 instead of 5.9 TB/s); otherwise
// row-major, where a feature row's outputs are written 64 bytes at a time.
constexpr int FW_TOK = 64, FW_FEAT = 64, FW_LD = FW_FEAT + 2;

// SPLIT (Sec. 2, "Optimization 1"; panel form only): feature f becomes row row_of_feat[f] of the outputs; rows below
// n_sparse are 2:4-compressed along tokens as above, the others -- the least sparse features -- are written out
// uncompressed, as rows [row - n_sparse] of the dense operands Hdn_t, dZdn_t [n_dense][T] (dense panel form).
template <bool PANEL, bool SPLIT = false>
__global__ void __launch_bounds__(256) featurewise24_kernel(const uint16_t* __restrict__ Hc, const uint8_t* __restrict__ meta,
                                                            const uint16_t* __restrict__ dZc, int T, int F,
                                                            uint16_t* __restrict__ Hc_t, uint8_t* __restrict__ meta_t,
                                                            uint16_t* __restrict__ dZc_t, const int* __restrict__ row_of_feat,
                                                            int n_sparse, uint16_t* __restrict__ Hdn_t, uint16_t* __restrict__ dZdn_t,
                                                            unsigned long long* __restrict__ tele, uint32_t* __restrict__ hmax,
                                                            uint32_t* __restrict__ zmax) {
  __shared__ uint16_t sH[FW_TOK * FW_LD];
  __shared__ uint16_t sZ[FW_TOK * FW_LD];
  int f0 = blockIdx.x * FW_FEAT, t0 = blockIdx.y * FW_TOK;
  int tid = threadIdx.x;
  bool has_z = dZc != nullptr;
#pragma unroll
  for (int i = 0; i < FW_TOK / 64; i++) {
    int item = tid + 256 * i;
    int tok = item >> 2, ch = item & 3;
    int t = t0 + tok;
    size_t vo, mo;   // offsets of this item's 8 stored values (in elements) and of its 2 metadata bytes
    if constexpr (PANEL) {
      size_t piece = a24_piece(t, f0 >> 6, F >> 6);
      vo = piece * 32 + 8 * ch;
      mo = piece * 8 + 2 * ch;
    } else {
      vo = (size_t)t * (F / 2) + f0 / 2 + 8 * ch;
      mo = (size_t)t * (F / 8) + f0 / 8 + 2 * ch;
    }
    u32x4 hv = ld_stream(reinterpret_cast<const u32x4*>(Hc + vo));
    u32x4 zv = {0u, 0u, 0u, 0u};
    if (has_z) zv = ld_stream(reinterpret_cast<const u32x4*>(dZc + vo));
    uint32_t m16 = ld_stream(reinterpret_cast<const uint16_t*>(meta + mo));
#pragma unroll
    for (int g = 0; g < 4; g++) {
      uint32_t nib = (m16 >> (4 * g)) & 15u;
      uint32_t i0 = nib & 3u, i1 = nib >> 2;
      uint32_t h_lo = hv[g] & 0xFFFFu, h_hi = hv[g] >> 16, z_lo = zv[g] & 0xFFFFu, z_hi = zv[g] >> 16;
      uint32_t hw[4], zw[4];
#pragma unroll
      for (uint32_t j = 0; j < 4; j++) {
        hw[j] = (i0 == j) ? h_lo : ((i1 == j) ? h_hi : 0u);
        zw[j] = (i0 == j) ? z_lo : ((i1 == j) ? z_hi : 0u);
      }
      int o = tok * FW_LD + 16 * ch + 4 * g;   // even: 4-byte aligned
      *reinterpret_cast<uint32_t*>(&sH[o]) = hw[0] | (hw[1] << 16);
      *reinterpret_cast<uint32_t*>(&sH[o + 2]) = hw[2] | (hw[3] << 16);
      *reinterpret_cast<uint32_t*>(&sZ[o]) = zw[0] | (zw[1] << 16);
      *reinterpret_cast<uint32_t*>(&sZ[o + 2]) = zw[2] | (zw[3] << 16);
    }
  }
  __syncthreads();
  uint32_t kept = 0u;   // non-zero activations this work item writes out (at most 32)
#pragma unroll
  for (int i = 0; i < FW_TOK / 32; i++) {
    int item = tid + 256 * i;
    int oct, f;
    if constexpr (PANEL) { oct = (item & 7) | ((item >> 9) << 3); f = (item >> 3) & 63; }
    else { oct = item % (FW_TOK / 8); f = item / (FW_TOK / 8); }
    uint32_t h[8], z[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
      h[j] = sH[(8 * oct + j) * FW_LD + f];
      z[j] = sZ[(8 * oct + j) * FW_LD + f];
    }
    int orow = f0 + f;
    if constexpr (SPLIT) {
      orow = row_of_feat[f0 + f];
      if (orow >= n_sparse) {   // dense feature: its 8 tokens as they are (already token-wise pruned)
        size_t o = a24_piece(orow - n_sparse, (t0 + 8 * oct) >> 5, T >> 5) * 32 + ((t0 + 8 * oct) & 31);
        *reinterpret_cast<u32x4*>(Hdn_t + o) = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        if (has_z) *reinterpret_cast<u32x4*>(dZdn_t + o) = u32x4{z[0] | (z[1] << 16), z[2] | (z[3] << 16), z[4] | (z[5] << 16), z[6] | (z[7] << 16)};
#pragma unroll
        for (int j = 0; j < 8; j++) kept += min(h[j], 1u);
        if (hmax) {   // as below: the eight work items of a feature are neighbouring lanes and take this branch together
          uint32_t mh = 0u, mz = 0u;
#pragma unroll
          for (int j = 0; j < 8; j++) { mh = max(mh, h[j]); mz = max(mz, z[j] & 0x7FFFu); }
#pragma unroll
          for (int sft = 1; sft < 8; sft <<= 1) {
            mh = max(mh, (uint32_t)__shfl_xor((int)mh, sft, 64));
            mz = max(mz, (uint32_t)__shfl_xor((int)mz, sft, 64));
          }
          if ((tid & 7) == 0) {
            if (mh) atomicMax(hmax + orow, mh);
            if (mz && has_z) atomicMax(zmax + orow, mz);
          }
        }
        continue;
      }
    }
    uint32_t hp[2], zp[2], nb[2];
#pragma unroll
    for (int g = 0; g < 2; g++) {
      nb[g] = pick24_words(h[4 * g], h[4 * g + 1], h[4 * g + 2], h[4 * g + 3], hp[g]);
      uint32_t i0 = nb[g] & 3u, i1 = nb[g] >> 2;
      uint32_t za = i0 == 0 ? z[4 * g] : (i0 == 1 ? z[4 * g + 1] : z[4 * g + 2]);
      uint32_t zb = i1 == 3 ? z[4 * g + 3] : (i1 == 2 ? z[4 * g + 2] : z[4 * g + 1]);
      zp[g] = za | (zb << 16);
    }
    size_t vo, mo;
    if constexpr (PANEL) {
      size_t piece = a24_piece(orow, (t0 + 8 * oct) >> 6, T >> 6);
      vo = piece * 32 + 4 * (oct & 7);
      mo = piece * 8 + (oct & 7);
    } else {
      size_t frow = (size_t)(f0 + f);
      vo = frow * (T / 2) + (t0 + 8 * oct) / 2;
      mo = frow * (T / 8) + t0 / 8 + oct;
    }
    st_stream(reinterpret_cast<u32x2*>(Hc_t + vo), u32x2{hp[0], hp[1]});
    if (has_z) st_stream(reinterpret_cast<u32x2*>(dZc_t + vo), u32x2{zp[0], zp[1]});
    st_stream(meta_t + mo, (uint8_t)(nb[0] | (nb[1] << 4)));
    if (hmax) {
      // largest stored magnitude word of this feature's row, for a row-wise quantisation that follows (the eight work items of
      // a feature are neighbouring lanes: one atomic per feature, tensor and workgroup)
      static_assert(FW_TOK == 64, "the eight items of a feature are the lanes tid & 7");
      uint32_t mh = max(max(hp[0] & 0xFFFFu, hp[0] >> 16), max(hp[1] & 0xFFFFu, hp[1] >> 16));
      uint32_t mz = max(max(zp[0] & 0x7FFFu, (zp[0] >> 16) & 0x7FFFu), max(zp[1] & 0x7FFFu, (zp[1] >> 16) & 0x7FFFu));
#pragma unroll
      for (int sft = 1; sft < 8; sft <<= 1) {
        mh = max(mh, (uint32_t)__shfl_xor((int)mh, sft, 64));
        mz = max(mz, (uint32_t)__shfl_xor((int)mz, sft, 64));
      }
      if ((tid & 7) == 0) {
        if (mh) atomicMax(hmax + orow, mh);
        if (mz && has_z) atomicMax(zmax + orow, mz);
      }
    }
    kept += min(hp[0] & 0xFFFFu, 1u) + min(hp[0] >> 16, 1u) + min(hp[1] & 0xFFFFu, 1u) + min(hp[1] >> 16, 1u);
  }
  // what the weight-gradient GEMMs still see of the activation (Sec. 2: the second, feature-wise drop): one atomic
  // per workgroup (tele is a kernel argument, so the barrier is reached by all or none)
  if (tele) {
    __shared__ uint32_t s_kept[4];
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) kept += (uint32_t)__shfl_xor((int)kept, sft, 64);
    if ((tid & 63) == 0) s_kept[tid >> 6] = kept;
    __syncthreads();
    if (tid == 0)
      atomicAdd(tele + tele_index(TELE_KEPT_FEAT, blockIdx.x + 5 * blockIdx.y),
                (unsigned long long)(s_kept[0] + s_kept[1] + s_kept[2] + s_kept[3]));
  }
}

// out[0] = elements, out[1 + k] = the sum of the slots of quantity k, out[4] = path: what a telemetry snapshot holds
__global__ void __launch_bounds__(64) tele_sum_kernel(const unsigned long long* __restrict__ tele, long long elements, long long path,
                                                      long long* __restrict__ out) {
  int k = threadIdx.x;
  if (k < TELE_KINDS) {
    unsigned long long sum = 0;
    for (int i = 0; i < TELE_SLOTS; i++) sum += tele[tele_index(k, i)];
    out[1 + k] = (long long)sum;
  }
  if (k == TELE_KINDS) { out[0] = elements; out[1 + TELE_KINDS] = path; }
}

int launch_tele_sum(const unsigned long long* tele, long long elements, long long path, long long* out, hipStream_t s) {
  hipLaunchKernelGGL(tele_sum_kernel, dim3(1), dim3(64), 0, s, tele, elements, path, out);
  return (int)hipGetLastError();
}

int launch_featurewise24(const void* Hc, const uint8_t* meta, const void* dZc, int T, int F,
                         void* Hc_t, uint8_t* meta_t, void* dZc_t, int panel, unsigned long long* tele, hipStream_t s) {
  dim3 grid(F / FW_FEAT, T / FW_TOK);
  auto kern = panel ? featurewise24_kernel<true> : featurewise24_kernel<false>;
  hipLaunchKernelGGL(kern, grid, dim3(256), 0, s, static_cast<const uint16_t*>(Hc), meta,
                     static_cast<const uint16_t*>(dZc), T, F, static_cast<uint16_t*>(Hc_t), meta_t, static_cast<uint16_t*>(dZc_t),
                     nullptr, 0, nullptr, nullptr, tele, nullptr, nullptr);
  return (int)hipGetLastError();
}

// the same (panel form) with the largest stored magnitude word of every output row: hmax, zmax [F], zeroed by the caller
int launch_featurewise24_rowmax(const void* Hc, const uint8_t* meta, const void* dZc, int T, int F, void* Hc_t, uint8_t* meta_t, void* dZc_t,
                                uint32_t* hmax, uint32_t* zmax, hipStream_t s) {
  dim3 grid(F / FW_FEAT, T / FW_TOK);
  hipLaunchKernelGGL(featurewise24_kernel<true>, grid, dim3(256), 0, s, static_cast<const uint16_t*>(Hc), meta,
                     static_cast<const uint16_t*>(dZc), T, F, static_cast<uint16_t*>(Hc_t), meta_t, static_cast<uint16_t*>(dZc_t),
                     nullptr, 0, nullptr, nullptr, nullptr, hmax, zmax);
  return (int)hipGetLastError();
}

int launch_featurewise24_split(const void* Hc, const uint8_t* meta, const void* dZc, int T, int F, const int* row_of_feat, int n_sparse,
                               void* Hc_t, uint8_t* meta_t, void* dZc_t, void* Hdn_t, void* dZdn_t, unsigned long long* tele,
                               uint32_t* hmax, uint32_t* zmax, hipStream_t s) {
  dim3 grid(F / FW_FEAT, T / FW_TOK);
  hipLaunchKernelGGL((featurewise24_kernel<true, true>), grid, dim3(256), 0, s, static_cast<const uint16_t*>(Hc), meta,
                     static_cast<const uint16_t*>(dZc), T, F, static_cast<uint16_t*>(Hc_t), meta_t, static_cast<uint16_t*>(dZc_t),
                     row_of_feat, n_sparse, static_cast<uint16_t*>(Hdn_t), static_cast<uint16_t*>(dZdn_t), tele, hmax, zmax);
  return (int)hipGetLastError();
}

// Feature partition of the split weight-gradient GEMMs (Sec. 2, "Optimization 1", where the paper sorts the features by their statistic).
// Only the set matters, so no sort: the threshold count c* = the smallest c with #{nnz > c} <= n_dense is found by
// bisection over the counts (which sit in LDS); every feature above it is dense, and of those equal to it the first
// (n_dense - #above) by index.  Sparse features become rows 0 .. F - n_dense - 1, dense ones the rows after, both in
// ascending feature order.  One workgroup of 1024; F <= 2^20 (beyond 32768 features the counts stay in global memory).
// In LDS count f sits at word f + f / 32: the ranking passes give every thread a run of consecutive features, and without the
// padding the lanes' runs would start a multiple of 32 words apart, all in two banks.  The rows are first written over the counts
// in LDS and leave in feature order, so that the stores to row_of_feat are whole lines and those to feat_of_row nearly so.
constexpr int PART_LDS_FEATS = 32768;
__device__ __forceinline__ int part_slot(int f) { return f + (f >> 5); }

template <bool IN_LDS>
__global__ void __launch_bounds__(1024) split_partition_kernel(const uint32_t* __restrict__ nnz_g, int F, int n_dense, uint32_t max_count,
                                                               int* __restrict__ row_of_feat, int* __restrict__ feat_of_row) {
  extern __shared__ uint32_t s_nnz[];                // F counts if they fit
  __shared__ int s_part[16];
  __shared__ int s_total;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr bool in_lds = IN_LDS;
  if (in_lds) for (int f = tid; f < F; f += 1024) s_nnz[part_slot(f)] = nnz_g[f];
  __syncthreads();
  auto nnz = [&](int f) { return in_lds ? s_nnz[part_slot(f)] : nnz_g[f]; };
  // block-wide sum, and exclusive prefix over threads, of one int per thread (wave shuffles + 16 partials in LDS)
  auto block_scan = [&](int v, int& total) {
    int incl = v;
#pragma unroll
    for (int st = 1; st < 64; st <<= 1) {
      int o = __shfl_up(incl, st, 64);
      if (lane >= st) incl += o;
    }
    if (lane == 63) s_part[wave] = incl;
    __syncthreads();
    if (tid == 0) {
      int run = 0;
      for (int w = 0; w < 16; w++) { int x = s_part[w]; s_part[w] = run; run += x; }
      s_total = run;
    }
    __syncthreads();
    int excl = s_part[wave] + incl - v;
    total = s_total;
    __syncthreads();
    return excl;
  };
  // block-wide sum alone (the bisection needs no prefix): wave shuffles, 16 partials in LDS that every thread adds up itself
  auto block_sum = [&](int v) {
#pragma unroll
    for (int st = 1; st < 64; st <<= 1) v += __shfl_xor(v, st, 64);
    if (lane == 0) s_part[wave] = v;
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int w = 0; w < 16; w++) total += s_part[w];
    __syncthreads();
    return total;
  };
  // bisection: invariant #{nnz > hi} <= n_dense and (lo == -1 or #{nnz > lo} > n_dense); strided accesses here
  int lo = -1, hi = (int)max_count;              // no count exceeds max_count (the number of tokens, at most 2^20)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    int c = 0;
    for (int f = tid; f < F; f += 1024) c += (int)nnz(f) > mid;
    if (block_sum(c) <= n_dense) hi = mid; else lo = mid;
  }
  const uint32_t cstar = (uint32_t)hi;
  // consecutive features per thread from here on, so that ranks follow the feature index
  const int per = (F + 1023) / 1024;
  const int f_lo = min(tid * per, F), f_hi = min(f_lo + per, F);
  int above = 0, equal = 0;
  for (int f = f_lo; f < f_hi; f++) { above += nnz(f) > cstar; equal += nnz(f) == cstar; }
  int n_above, n_equal;
  block_scan(above, n_above);
  const int take_eq = n_dense - n_above;             // how many of the features equal to c* become dense (by index)
  const int eq_before = block_scan(equal, n_equal);
  int dense_here = 0;
  {
    int e = eq_before;
    for (int f = f_lo; f < f_hi; f++) {
      bool d = nnz(f) > cstar || (nnz(f) == cstar && e < take_eq);
      e += nnz(f) == cstar;
      dense_here += d;
    }
  }
  int n_d;
  const int d_before = block_scan(dense_here, n_d);
  const int n_sparse = F - n_dense;
  int e = eq_before, dpos = d_before;
  for (int f = f_lo; f < f_hi; f++) {
    bool d = nnz(f) > cstar || (nnz(f) == cstar && e < take_eq);
    e += nnz(f) == cstar;
    int row = d ? n_sparse + dpos : f - dpos;
    dpos += d;
    if (in_lds) s_nnz[part_slot(f)] = (uint32_t)row;   // the thread's own slot: its count is not needed again
    else { row_of_feat[f] = row; feat_of_row[row] = f; }
  }
  if (in_lds) {
    __syncthreads();
    for (int f = tid; f < F; f += 1024) {
      int row = (int)s_nnz[part_slot(f)];
      row_of_feat[f] = row;
      feat_of_row[row] = f;
    }
  }
}

int launch_split_partition(const uint32_t* nnz, int F, int n_dense, int max_count, int* row_of_feat, int* feat_of_row, hipStream_t s) {
  static std::atomic<bool> configured[MAX_DEVICES] = {};
  if (F > PART_LDS_FEATS) {
    hipLaunchKernelGGL(split_partition_kernel<false>, dim3(1), dim3(1024), 0, s, nnz, F, n_dense, (uint32_t)max_count, row_of_feat, feat_of_row);
    return (int)hipGetLastError();
  }
  if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(split_partition_kernel<true>), 4 * (PART_LDS_FEATS + PART_LDS_FEATS / 32), configured)) return rc;
  hipLaunchKernelGGL(split_partition_kernel<true>, dim3(1), dim3(1024), 4 * ((size_t)F + (size_t)F / 32), s, nnz, F, n_dense, (uint32_t)max_count,
                     row_of_feat, feat_of_row);
  return (int)hipGetLastError();
}

// Panel form -> row-major.  The operand has `rows` rows and `npanels` pieces of PIECE bytes per row (64: stored
// values, 8 / 16: bf16 / fp8 metadata); each work item moves 8 bytes.
template <int PIECE>
__global__ void __launch_bounds__(256) unpanel_kernel(const u32x2* __restrict__ src, int rows, int npanels, u32x2* __restrict__ dst) {
  constexpr int W = PIECE / 8;                       // 8-byte words per piece
  size_t n = (size_t)rows * npanels * W;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    size_t pc = i / W;                               // row-major piece number: r * npanels + kp
    int w = (int)(i % W);
    int r = (int)(pc / npanels), kp = (int)(pc % npanels);
    dst[i] = src[a24_piece(r, kp, npanels) * W + w];
  }
}

// Clears n 32-bit words.  A kernel rather than a memset node, so that a caller may record the sequence into a HIP graph.
__global__ void __launch_bounds__(256) zero32_kernel(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

int launch_zero32(uint32_t* p, size_t n, hipStream_t s) {
  if (n == 0) return 0;
  size_t blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(zero32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n);
  return (int)hipGetLastError();
}

int launch_unpanel(const void* src, int rows, int npanels, int piece_bytes, void* dst, hipStream_t s) {
  size_t n = (size_t)rows * npanels * (piece_bytes / 8);
  size_t blocks = (n + 255) / 256;
  if (blocks > 0x7FFFFFFF) blocks = 0x7FFFFFFF;   // one work item per thread: the fastest shape for a streaming kernel here
  auto kern = piece_bytes == 64 ? unpanel_kernel<64> : (piece_bytes == 16 ? unpanel_kernel<16> : unpanel_kernel<8>);
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x2*>(src), rows, npanels, static_cast<u32x2*>(dst));
  return (int)hipGetLastError();
}

// out[c][r] = in[r][c] for a bf16 matrix [R][C], R a multiple of 64 and C of 128.  One workgroup per tile of 64 rows x 128
// columns: a work item reads 16 bytes of each of 2 consecutive rows (a row's 256 bytes are read by 16 neighbouring work items),
// pairs the rows' elements column by column with byte permutes, and writes 8 dwords -- 2 elements along r of 8 transposed rows --
// into an LDS image [c][r] (pitch 33 dwords; a row's dwords are rotated by 4 for the second 64 columns, which spreads a wave's
// writes over all banks); then 16 bytes of a transposed row per work item go out: 128 rows x 128 bytes.  (One 64 x 64 tile per
// workgroup with element-wise LDS scatter, the first version, moved 4.3-4.9 TB/s.)
// OUT_FORM: 0 row-major; 1 the dense panel form of gemm_core.hpp (64-byte pieces of 32 k, K = R), as A operands take it;
// 2 the B panel form (the same with the rows of every block of 256 in LDS order).
// in_panel (optional): a copy of the input itself in panel form (K = C), made in the same pass; in_panel_b: in the B form.
// in_rowmap (optional): input row r is read from memory row in_rowmap[r] (token permutation).
constexpr int TR_COLS = 128, TR_LDW = 33;

template <int OUT_FORM>
__global__ void __launch_bounds__(256) transpose_kernel(const uint16_t* __restrict__ in, int R, int C, uint16_t* __restrict__ out,
                                                        uint16_t* __restrict__ in_panel, int in_panel_b, const int* __restrict__ in_rowmap) {
  __shared__ uint32_t sT[TR_COLS * TR_LDW];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * TR_COLS;
  const int tid = threadIdx.x;
  const int ch = tid & 15;                   // 16-byte chunk of a row segment: columns 8 ch .. 8 ch + 7 of the tile
  const int rot = ch >> 3;                   // (c >> 6) of every column this work item holds
  u32x4 v[2][2];
#pragma unroll
  for (int pass = 0; pass < 2; pass++)
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int r = r0 + 2 * ((tid >> 4) + 16 * pass) + i;
      const size_t src_row = in_rowmap ? (size_t)in_rowmap[r] : (size_t)r;
      v[pass][i] = ld_stream(reinterpret_cast<const u32x4*>(in + src_row * C + c0 + 8 * ch));
    }
#pragma unroll
  for (int pass = 0; pass < 2; pass++) {
    const int rp = (tid >> 4) + 16 * pass;   // pair of rows 2 rp, 2 rp + 1 of the tile
    if (in_panel) {
      const int c = c0 + 8 * ch;
#pragma unroll
      for (int i = 0; i < 2; i++) {
        const int r = r0 + 2 * rp + i;
        const int prow = in_panel_b ? b_panel_pos(r) : r;
        st_stream(reinterpret_cast<u32x4*>(in_panel + a24_piece(prow, c >> 5, C >> 5) * 32 + (c & 31)), v[pass][i]);
      }
    }
    uint32_t* dst = sT + ((rp + 4 * rot) & 31);
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const int c = 8 * ch + 2 * g;
      dst[c * TR_LDW] = __builtin_amdgcn_perm(v[pass][1][g], v[pass][0][g], 0x05040100u);         // column c: rows 2 rp, 2 rp + 1
      dst[(c + 1) * TR_LDW] = __builtin_amdgcn_perm(v[pass][1][g], v[pass][0][g], 0x07060302u);   // column c + 1
    }
  }
  __syncthreads();
  const int q = tid & 7;                     // 16-byte chunk of a transposed row: 8 of the tile's 64 rows r
#pragma unroll
  for (int p = 0; p < TR_COLS / 32; p++) {
    const int c = (tid >> 3) + 32 * p;       // transposed row
    const uint32_t* src = sT + c * TR_LDW + 4 * ((q + (c >> 6)) & 7);
    u32x4 o = {src[0], src[1], src[2], src[3]};
    const int r = r0 + 8 * q;
    if constexpr (OUT_FORM == 1) st_stream(reinterpret_cast<u32x4*>(out + a24_piece(c0 + c, r >> 5, R >> 5) * 32 + (r & 31)), o);
    else if constexpr (OUT_FORM == 2) st_stream(reinterpret_cast<u32x4*>(out + a24_piece(b_panel_pos(c0 + c), r >> 5, R >> 5) * 32 + (r & 31)), o);
    else st_stream(reinterpret_cast<u32x4*>(out + (size_t)(c0 + c) * R + r), o);
  }
}

int launch_transpose(const void* in, int R, int C, void* out, int out_form, void* in_panel, int in_panel_b, const int* in_rowmap, hipStream_t s) {
  dim3 grid(C / TR_COLS, R / 64);
  auto kern = out_form == 2 ? transpose_kernel<2> : (out_form == 1 ? transpose_kernel<1> : transpose_kernel<0>);
  hipLaunchKernelGGL(kern, grid, dim3(256), 0, s, static_cast<const uint16_t*>(in), R, C, static_cast<uint16_t*>(out),
                     static_cast<uint16_t*>(in_panel), in_panel_b, in_rowmap);
  return (int)hipGetLastError();
}

// Byte-matrix transpose (fp8 operands): out[c][r] = in[r][c], in [R][C], R a multiple of 64 and C of 256.  One workgroup per
// tile of 64 rows x 256 columns: a work item reads 16 bytes of each of 4 consecutive rows (a row's 256 bytes are read by 16
// neighbouring work items), transposes its four 4 x 4 byte blocks in registers with byte permutes, and writes 16 dwords -- 4
// bytes along r of 16 transposed rows -- into an LDS image [c][r] (pitch 68 bytes; a row's 16 dwords are rotated by 4 for every 64
// columns, which spreads a wave's writes over all banks); then 16 bytes of a transposed row per work item go out: 256 rows x
// 64 bytes, one contiguous 16 KiB run in the panel forms.  (One 64 x 64 tile per workgroup with byte-wise LDS scatter, the
// first version, moved 3.8 TB/s.)  OUT_FORM: 0 row-major, 1 dense panel form (64-byte pieces of 64 k, K = R), 2 the B panel form.
// in_panel (optional): a copy of the input itself in panel form (K = C, 64-byte pieces), made in the same pass; in the
// B form if in_panel_b.  in_rowmap (optional): input row r is read from memory row in_rowmap[r] (token permutation).
constexpr int T8_COLS = 256, T8_LD = 68;

template <int OUT_FORM>
__global__ void __launch_bounds__(256) transpose8_kernel(const uint8_t* __restrict__ in, int R, int C, uint8_t* __restrict__ out,
                                                         uint8_t* __restrict__ in_panel, int in_panel_b, const int* __restrict__ in_rowmap) {
  __shared__ __attribute__((aligned(16))) uint8_t sT[T8_COLS * T8_LD];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * T8_COLS;
  const int tid = threadIdx.x;
  const int ch = tid & 15, rq = tid >> 4;    // 16-byte column chunk of the tile; group of 4 rows
  u32x4 v[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int r = r0 + 4 * rq + i;
    const size_t src_row = in_rowmap ? (size_t)in_rowmap[r] : (size_t)r;
    v[i] = ld_stream(reinterpret_cast<const u32x4*>(in + src_row * C + c0 + 16 * ch));
  }
  if (in_panel) {
    const int c = c0 + 16 * ch;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int r = r0 + 4 * rq + i;
      const int prow = in_panel_b ? b_panel_pos(r) : r;
      st_stream(reinterpret_cast<u32x4*>(in_panel + a24_piece(prow, c >> 6, C >> 6) * 64 + (c & 63)), v[i]);
    }
  }
  const int rot = ch >> 2;                   // (c >> 6) & 3 of every column this work item holds
  uint32_t* dst = reinterpret_cast<uint32_t*>(sT) + ((rq + 4 * rot) & 15);
#pragma unroll
  for (int g = 0; g < 4; g++) {
    // rows i = 0..3, bytes j = 0..3 of column group g  ->  for every j the bytes of rows 0..3
    const uint32_t lo01 = __builtin_amdgcn_perm(v[1][g], v[0][g], 0x05010400u), hi01 = __builtin_amdgcn_perm(v[1][g], v[0][g], 0x07030602u);
    const uint32_t lo23 = __builtin_amdgcn_perm(v[3][g], v[2][g], 0x05010400u), hi23 = __builtin_amdgcn_perm(v[3][g], v[2][g], 0x07030602u);
    const int c = 16 * ch + 4 * g;
    dst[(c + 0) * (T8_LD / 4)] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
    dst[(c + 1) * (T8_LD / 4)] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
    dst[(c + 2) * (T8_LD / 4)] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
    dst[(c + 3) * (T8_LD / 4)] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
  }
  __syncthreads();
  const int q = tid & 3;                     // 16-byte chunk of a transposed row (16 of the tile's 64 rows r)
#pragma unroll
  for (int p = 0; p < T8_COLS / 64; p++) {
    const int c = (tid >> 2) + 64 * p;       // transposed row; (c >> 6) & 3 == p
    const uint32_t* src = reinterpret_cast<const uint32_t*>(sT) + c * (T8_LD / 4) + 4 * ((q + p) & 3);
    u32x4 o = {src[0], src[1], src[2], src[3]};
    const int r = r0 + 16 * q;
    if constexpr (OUT_FORM == 1) st_stream(reinterpret_cast<u32x4*>(out + a24_piece(c0 + c, r >> 6, R >> 6) * 64 + (r & 63)), o);
    else if constexpr (OUT_FORM == 2) st_stream(reinterpret_cast<u32x4*>(out + a24_piece(b_panel_pos(c0 + c), r >> 6, R >> 6) * 64 + (r & 63)), o);
    else st_stream(reinterpret_cast<u32x4*>(out + (size_t)(c0 + c) * R + r), o);
  }
}

int launch_transpose8(const void* in, int R, int C, void* out, int out_form, void* in_panel, int in_panel_b, hipStream_t s) {
  dim3 grid(C / T8_COLS, R / 64);
  auto kern = out_form == 2 ? transpose8_kernel<2> : (out_form == 1 ? transpose8_kernel<1> : transpose8_kernel<0>);
  hipLaunchKernelGGL(kern, grid, dim3(256), 0, s, static_cast<const uint8_t*>(in), R, C, static_cast<uint8_t*>(out),
                     static_cast<uint8_t*>(in_panel), in_panel_b, static_cast<const int*>(nullptr));
  return (int)hipGetLastError();
}

int launch_transpose8_rows(const void* in, int R, int C, void* out, int out_form, const int* in_rowmap, hipStream_t s) {
  dim3 grid(C / T8_COLS, R / 64);
  auto kern = out_form == 2 ? transpose8_kernel<2> : (out_form == 1 ? transpose8_kernel<1> : transpose8_kernel<0>);
  hipLaunchKernelGGL(kern, grid, dim3(256), 0, s, static_cast<const uint8_t*>(in), R, C, static_cast<uint8_t*>(out),
                     static_cast<uint8_t*>(nullptr), 0, in_rowmap);
  return (int)hipGetLastError();
}

// dst[i] = src[map[i]]: a per-token scale vector brought into the order of a token permutation
__global__ void __launch_bounds__(256) gather_f32_kernel(const float* __restrict__ src, const int* __restrict__ map, int n, float* __restrict__ dst) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[map[i]];
}

int launch_gather_f32(const float* src, const int* map, int n, float* dst, hipStream_t s) {
  hipLaunchKernelGGL(gather_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, map, n, dst);
  return (int)hipGetLastError();
}

// A byte matrix [R][C] (row-major, C a multiple of 64) copied into the dense fp8 panel form (64-byte pieces of 64 k, K = C) as
// A operands take it, or, b_form, into the B panel form (rows of every block of 256 in LDS order).  16 bytes per work item.
// in_rowmap (optional): row r is taken from memory row in_rowmap[r] (token permutation).
__global__ void __launch_bounds__(256) panelise8_kernel(const u32x4* __restrict__ in, int R, int C, uint8_t* __restrict__ out, int b_form,
                                                        const int* __restrict__ in_rowmap) {
  const int per_row = C >> 4;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)R * per_row) return;
  int r = (int)(i / per_row), cq = (int)(i % per_row), c = cq << 4;
  int prow = b_form ? b_panel_pos(r) : r;
  size_t src = in_rowmap ? (size_t)in_rowmap[r] * per_row + cq : i;
  st_stream(reinterpret_cast<u32x4*>(out + a24_piece(prow, c >> 6, C >> 6) * 64 + (c & 63)), ld_stream(in + src));
}

int launch_panelise8_rows(const void* in, int R, int C, void* out, int b_form, const int* in_rowmap, hipStream_t s) {
  size_t n = (size_t)R * (C >> 4);
  hipLaunchKernelGGL(panelise8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, static_cast<const u32x4*>(in), R, C,
                     static_cast<uint8_t*>(out), b_form, in_rowmap);
  return (int)hipGetLastError();
}

int launch_panelise8(const void* in, int R, int C, void* out, int b_form, hipStream_t s) {
  return launch_panelise8_rows(in, R, C, out, b_form, nullptr, s);
}

// Feature-wise 2:4 on top of the token-wise mask for the fp8 operands (Sec. 2, last paragraph; the FP8 side of the fused
// backward pointwise step).  Everything is in the fp8 panel form: input pieces = 128 hidden features of one token (64
// stored e4m3 bytes + 16 metadata bytes), output pieces = 128 tokens of one feature.  The picks are made on the stored
// codes of the activation (sign bit cleared, as integers; ties -> lower token); dZ is gathered at the same positions.
// One workgroup handles 128 tokens x 128 features: it reads 128 consecutive input pieces of each tensor (8 KiB + 2 KiB
// runs), spreads them out in LDS, and every work item then takes one feature and 16 consecutive tokens (four groups):
// 8 stored bytes and 2 metadata bytes of an output piece.
constexpr int FW8_TOK = 128, FW8_FEAT = 128, FW8_LD = FW8_FEAT + 4;

__device__ __forceinline__ uint32_t pick24_codes(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, uint32_t& i0, uint32_t& i1) {
  // keys ((magnitude << 2) | (3 - i)): distinct, ordered by (magnitude, then lower index first)
  uint32_t k0 = ((w0 & 0x7Fu) << 2) | 3u, k1 = ((w1 & 0x7Fu) << 2) | 2u, k2 = ((w2 & 0x7Fu) << 2) | 1u, k3 = (w3 & 0x7Fu) << 2;
  uint32_t kf, ks;
  uint32_t nib = pick24_keys(k0, k1, k2, k3, kf, ks);
  i0 = nib & 3u; i1 = nib >> 2;
  return nib;
}

__global__ void __launch_bounds__(256) featurewise24_f8_kernel(const uint8_t* __restrict__ Hc8, const uint8_t* __restrict__ meta,
                                                               const uint8_t* __restrict__ dZc8, int T, int F,
                                                               uint8_t* __restrict__ Hc8_t, uint8_t* __restrict__ meta_t,
                                                               uint8_t* __restrict__ dZc8_t) {
  __shared__ __attribute__((aligned(16))) uint8_t sH[FW8_TOK * FW8_LD];
  __shared__ __attribute__((aligned(16))) uint8_t sZ[FW8_TOK * FW8_LD];
  const int f0 = blockIdx.x * FW8_FEAT, t0 = blockIdx.y * FW8_TOK;
  const int tid = threadIdx.x;
  const bool has_z = dZc8 != nullptr;
#pragma unroll
  for (int i = 0; i < 2; i++) {
    int item = tid + 256 * i;
    int tok = item >> 2, ch = item & 3;              // 16 stored bytes = 8 groups = 32 features
    size_t piece = a24_piece(t0 + tok, f0 >> 7, F >> 7);
    u32x4 hv = ld_stream(reinterpret_cast<const u32x4*>(Hc8 + piece * 64 + 16 * ch));
    u32x4 zv = {0u, 0u, 0u, 0u};
    if (has_z) zv = ld_stream(reinterpret_cast<const u32x4*>(dZc8 + piece * 64 + 16 * ch));
    uint32_t m32 = ld_stream(reinterpret_cast<const uint32_t*>(meta + piece * 16 + 4 * ch));
#pragma unroll
    for (int g = 0; g < 8; g++) {
      uint32_t nib = (m32 >> (4 * g)) & 15u;
      uint32_t i0 = nib & 3u, i1 = nib >> 2;
      uint32_t hb = (hv[g >> 1] >> (16 * (g & 1))) & 0xFFFFu, zb = (zv[g >> 1] >> (16 * (g & 1))) & 0xFFFFu;
      // the group's four bytes as one word: kept byte 0 at position i0, kept byte 1 at position i1
      uint32_t hw = ((hb & 0xFFu) << (8 * i0)) | ((hb >> 8) << (8 * i1));
      uint32_t zw = ((zb & 0xFFu) << (8 * i0)) | ((zb >> 8) << (8 * i1));
      int o = tok * FW8_LD + 32 * ch + 4 * g;         // a multiple of 4
      *reinterpret_cast<uint32_t*>(&sH[o]) = hw;
      *reinterpret_cast<uint32_t*>(&sZ[o]) = zw;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int item = tid + 256 * i;
    int c = item & 7, f = item >> 3;                   // 16 tokens 16 c .. 16 c + 15 of feature f0 + f
    uint32_t hq[2] = {0u, 0u}, zq[2] = {0u, 0u}, mq = 0u;
#pragma unroll
    for (int g = 0; g < 4; g++) {
      uint32_t h[4], z[4];
#pragma unroll
      for (int j = 0; j < 4; j++) {
        h[j] = sH[(16 * c + 4 * g + j) * FW8_LD + f];
        z[j] = sZ[(16 * c + 4 * g + j) * FW8_LD + f];
      }
      uint32_t i0, i1;
      uint32_t nib = pick24_codes(h[0], h[1], h[2], h[3], i0, i1);
      uint32_t ha = i0 == 0 ? h[0] : (i0 == 1 ? h[1] : h[2]), hb = i1 == 3 ? h[3] : (i1 == 2 ? h[2] : h[1]);
      uint32_t za = i0 == 0 ? z[0] : (i0 == 1 ? z[1] : z[2]), zb = i1 == 3 ? z[3] : (i1 == 2 ? z[2] : z[1]);
      hq[g >> 1] |= (ha | (hb << 8)) << (16 * (g & 1));
      zq[g >> 1] |= (za | (zb << 8)) << (16 * (g & 1));
      mq |= nib << (4 * g);
    }
    size_t piece = a24_piece(f0 + f, t0 >> 7, T >> 7);
    st_stream(reinterpret_cast<u32x2*>(Hc8_t + piece * 64 + 8 * c), u32x2{hq[0], hq[1]});
    if (has_z) st_stream(reinterpret_cast<u32x2*>(dZc8_t + piece * 64 + 8 * c), u32x2{zq[0], zq[1]});
    st_stream(reinterpret_cast<uint16_t*>(meta_t + piece * 16 + 2 * c), (uint16_t)mq);
  }
}

int launch_featurewise24_f8(const void* Hc8, const uint8_t* meta, const void* dZc8, int T, int F, void* Hc8_t, uint8_t* meta_t, void* dZc8_t, hipStream_t s) {
  dim3 grid(F / FW8_FEAT, T / FW8_TOK);
  hipLaunchKernelGGL(featurewise24_f8_kernel, grid, dim3(256), 0, s, static_cast<const uint8_t*>(Hc8), meta, static_cast<const uint8_t*>(dZc8),
                     T, F, static_cast<uint8_t*>(Hc8_t), meta_t, static_cast<uint8_t*>(dZc8_t));
  return (int)hipGetLastError();
}

// Row-wise fp8 quantisation of the compressed activation (Sec. 2 describes one kernel for activation, sparsification
// and FP8 quantisation; here only the last step is left to a kernel of its own, because the scale of a token row,
// sh[t] = (largest activation of the row) / 448, is known only once the whole row exists).
// Input: bf16 kept values + metadata in the bf16 panel form (64-byte / 8-byte pieces per 64 features);
// output: e4m3 codes + metadata in the fp8 panel form (64-byte / 16-byte pieces per 128 features), and sh [T].
// One work item per (token, 128 features): two input pieces -> one output piece.
__global__ void __launch_bounds__(256) quantise_rows_kernel(const u32x4* __restrict__ Hc16, const u32x2* __restrict__ meta16,
                                                            const uint32_t* __restrict__ rowmax, int T, int F,
                                                            u32x4* __restrict__ Hc8, u32x4* __restrict__ meta8, float* __restrict__ sh) {
  const int np8 = F >> 7;                                 // output pieces per token
  size_t n = (size_t)T * np8;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    // item order = output piece order: ((t / 256) * np8 + j) * 256 + t % 256
    int tl = (int)(i & 255);
    size_t blk = i >> 8;
    int j = (int)(blk % np8), t = (int)(blk / np8) * 256 + tl;
    float mxv = __builtin_bit_cast(float, rowmax[t] << 16);
    float s = mxv > 0.f ? mxv / 448.f : 1.f;
    if (j == 0) sh[t] = s;
    u32x4 out[4];
    u32x2 mo[2];
#pragma unroll
    for (int hlf = 0; hlf < 2; hlf++) {
      size_t pin = a24_piece(t, 2 * j + hlf, F >> 6);
      mo[hlf] = meta16[pin];
#pragma unroll
      for (int c = 0; c < 4; c++) {
        u32x4 v = Hc16[pin * 4 + c];                      // 8 bf16 values -> 8 codes = 2 dwords
        uint32_t q0 = cvt_e4m3x2(bf16_lo_to_f32(v[0]) / s, bf16_hi_to_f32(v[0]) / s, 0u, false);
        q0 = cvt_e4m3x2(bf16_lo_to_f32(v[1]) / s, bf16_hi_to_f32(v[1]) / s, q0, true);
        uint32_t q1 = cvt_e4m3x2(bf16_lo_to_f32(v[2]) / s, bf16_hi_to_f32(v[2]) / s, 0u, false);
        q1 = cvt_e4m3x2(bf16_lo_to_f32(v[3]) / s, bf16_hi_to_f32(v[3]) / s, q1, true);
        out[2 * hlf + (c >> 1)][2 * (c & 1)] = q0;
        out[2 * hlf + (c >> 1)][2 * (c & 1) + 1] = q1;
      }
    }
#pragma unroll
    for (int c = 0; c < 4; c++) Hc8[i * 4 + c] = out[c];
    meta8[i] = u32x4{mo[0][0], mo[0][1], mo[1][0], mo[1][1]};
  }
}

// The same for the dense baseline: bf16 [T][F] in dense panel form (64-byte pieces of 32 features) -> e4m3 [T][F] in the
// dense fp8 panel form (64-byte pieces of 64 features).  One work item per (token, 64 features).
__global__ void __launch_bounds__(256) quantise_rows_dense_kernel(const u32x4* __restrict__ H16, const uint32_t* __restrict__ rowmax,
                                                                  int T, int F, u32x4* __restrict__ H8, float* __restrict__ sh) {
  const int np8 = F >> 6;                                 // output pieces per token
  size_t n = (size_t)T * np8;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    int tl = (int)(i & 255);
    size_t blk = i >> 8;
    int j = (int)(blk % np8), t = (int)(blk / np8) * 256 + tl;
    float mxv = __builtin_bit_cast(float, rowmax[t] << 16);
    float s = mxv > 0.f ? mxv / 448.f : 1.f;
    if (j == 0) sh[t] = s;
#pragma unroll
    for (int hlf = 0; hlf < 2; hlf++) {
      size_t pin = a24_piece(t, 2 * j + hlf, F >> 5);
#pragma unroll
      for (int c = 0; c < 2; c++) {                       // 16 bf16 values -> 16 codes
        u32x4 v0 = H16[pin * 4 + 2 * c], v1 = H16[pin * 4 + 2 * c + 1];
        u32x4 o;
#pragma unroll
        for (int d = 0; d < 2; d++) {
          uint32_t q = cvt_e4m3x2(bf16_lo_to_f32(v0[2 * d]) / s, bf16_hi_to_f32(v0[2 * d]) / s, 0u, false);
          o[d] = cvt_e4m3x2(bf16_lo_to_f32(v0[2 * d + 1]) / s, bf16_hi_to_f32(v0[2 * d + 1]) / s, q, true);
          q = cvt_e4m3x2(bf16_lo_to_f32(v1[2 * d]) / s, bf16_hi_to_f32(v1[2 * d]) / s, 0u, false);
          o[2 + d] = cvt_e4m3x2(bf16_lo_to_f32(v1[2 * d + 1]) / s, bf16_hi_to_f32(v1[2 * d + 1]) / s, q, true);
        }
        H8[i * 4 + 2 * hlf + c] = o;
      }
    }
  }
}

// Largest magnitude word of every row of a bf16 matrix [R][C] in dense panel form (64-byte pieces of 32 k): rmax[r] is raised
// with an atomic (the caller zeroes it).  A workgroup takes one block of 256 rows (one row per work item, so its loads of a
// panel are one contiguous 16 KiB run) and a slice of the panels.
constexpr int ROWMAX_SLICES = 32;
__global__ void __launch_bounds__(256) rowmax_dense_kernel(const u32x4* __restrict__ X16, int R, int C, uint32_t* __restrict__ rmax) {
  const int np = C >> 5;
  const int per = (np + ROWMAX_SLICES - 1) / ROWMAX_SLICES;
  const int k0 = blockIdx.y * per, k1 = min(np, k0 + per);
  const size_t base = (size_t)blockIdx.x * np * 256 + threadIdx.x;
  uint32_t m = 0u;
  for (int kp = k0; kp < k1; kp++) {
    const u32x4* p = X16 + (base + (size_t)kp * 256) * 4;
#pragma unroll
    for (int c = 0; c < 4; c++) {
      u32x4 v = ld_stream(p + c);
#pragma unroll
      for (int d = 0; d < 4; d++) m = max(m, max(v[d] & 0x7FFFu, (v[d] >> 16) & 0x7FFFu));
    }
  }
  if (m) atomicMax(rmax + blockIdx.x * 256 + threadIdx.x, m);
}

int launch_rowmax_dense(const void* X16, int R, int C, uint32_t* rmax, hipStream_t s) {
  hipLaunchKernelGGL(rowmax_dense_kernel, dim3(R / 256, ROWMAX_SLICES), dim3(256), 0, s, static_cast<const u32x4*>(X16), R, C, rmax);
  return (int)hipGetLastError();
}

int launch_quantise_rows_dense(const void* H16, const uint32_t* rowmax, int T, int F, void* H8, float* sh, hipStream_t s) {
  size_t n = (size_t)T * (F >> 6);
  size_t blocks = (n + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;   // (here the grid-stride walk with plain accesses is the faster shape: 4.8 against 3.0 TB/s)
  hipLaunchKernelGGL(quantise_rows_dense_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4*>(H16), rowmax, T, F,
                     static_cast<u32x4*>(H8), sh);
  return (int)hipGetLastError();
}

int launch_quantise_rows(const void* Hc16, const uint8_t* meta16, const uint32_t* rowmax, int T, int F, void* Hc8, uint8_t* meta8, float* sh,
                         hipStream_t s) {
  size_t n = (size_t)T * (F >> 7);
  size_t blocks = (n + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(quantise_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const u32x4*>(Hc16),
                     reinterpret_cast<const u32x2*>(meta16), rowmax, T, F, static_cast<u32x4*>(Hc8), reinterpret_cast<u32x4*>(meta8), sh);
  return (int)hipGetLastError();
}

// Row-wise / column-wise e4m3 quantisation of a bf16 matrix X [R][C] (the operands a caller hands to the row-wise-scaled
// GEMMs; Sec. 2 of the paper: FP8 row-wise scaling).  scale = (largest magnitude of the row or column) / 448, 1 if that is
// zero; codes = e4m3(x / scale), row-major [R][C].
// Per row: one wave per row, two passes over the row (the second one finds it in the caches).
__global__ void __launch_bounds__(256) quantise_bf16_rows_kernel(const u32x4* __restrict__ X, int64_t R, int C8, u32x2* __restrict__ codes,
                                                                 float* __restrict__ scales) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= R) return;
  const u32x4* row = X + r * C8;
  uint32_t m = 0u;
  for (int c = lane; c < C8; c += 64) {
    u32x4 v = row[c];
#pragma unroll
    for (int d = 0; d < 4; d++) m = max(m, max(v[d] & 0x7FFFu, (v[d] >> 16) & 0x7FFFu));
  }
#pragma unroll
  for (int sft = 1; sft < 64; sft <<= 1) m = max(m, (uint32_t)__shfl_xor((int)m, sft, 64));
  const float mx = __builtin_bit_cast(float, m << 16);
  const float s = mx > 0.f ? mx / 448.f : 1.f;
  if (lane == 0) scales[r] = s;
  u32x2* out = codes + r * C8;
  for (int c = lane; c < C8; c += 64) {
    u32x4 v = row[c];
    uint32_t q0 = cvt_e4m3x2(bf16_lo_to_f32(v[0]) / s, bf16_hi_to_f32(v[0]) / s, 0u, false);
    q0 = cvt_e4m3x2(bf16_lo_to_f32(v[1]) / s, bf16_hi_to_f32(v[1]) / s, q0, true);
    uint32_t q1 = cvt_e4m3x2(bf16_lo_to_f32(v[2]) / s, bf16_hi_to_f32(v[2]) / s, 0u, false);
    q1 = cvt_e4m3x2(bf16_lo_to_f32(v[3]) / s, bf16_hi_to_f32(v[3]) / s, q1, true);
    st_stream(out + c, u32x2{q0, q1});
  }
}

// Per column, step 1: cmax[c] (zeroed by the caller) is raised to the largest magnitude word of column c.  A work item takes 8
// consecutive columns of a slab of QC_ROWS rows.
constexpr int QC_ROWS = 64;
__global__ void __launch_bounds__(256) colmax_bf16_kernel(const u32x4* __restrict__ X, int64_t R, int C8, uint32_t* __restrict__ cmax) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C8) return;
  const int64_t r0 = (int64_t)blockIdx.y * QC_ROWS, r1 = r0 + QC_ROWS < R ? r0 + QC_ROWS : R;
  uint32_t m[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
  for (int64_t r = r0; r < r1; r++) {
    u32x4 v = ld_stream(X + r * C8 + c);
#pragma unroll
    for (int d = 0; d < 4; d++) { m[2 * d] = max(m[2 * d], v[d] & 0x7FFFu); m[2 * d + 1] = max(m[2 * d + 1], (v[d] >> 16) & 0x7FFFu); }
  }
#pragma unroll
  for (int j = 0; j < 8; j++) if (m[j]) atomicMax(cmax + 8 * c + j, m[j]);
}
// step 2: codes with the scales taken from the column maxima
__global__ void __launch_bounds__(256) quantise_bf16_cols_kernel(const u32x4* __restrict__ X, int64_t R, int C8, const u32x4* __restrict__ cmax,
                                                                 u32x2* __restrict__ codes) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C8) return;
  const int64_t r0 = (int64_t)blockIdx.y * QC_ROWS, r1 = r0 + QC_ROWS < R ? r0 + QC_ROWS : R;
  float s[8];
  u32x4 ma = cmax[2 * c], mb = cmax[2 * c + 1];
#pragma unroll
  for (int j = 0; j < 8; j++) {
    float mx = __builtin_bit_cast(float, (j < 4 ? ma[j] : mb[j - 4]) << 16);
    s[j] = mx > 0.f ? mx / 448.f : 1.f;
  }
  for (int64_t r = r0; r < r1; r++) {
    u32x4 v = ld_stream(X + r * C8 + c);
    uint32_t q0 = cvt_e4m3x2(bf16_lo_to_f32(v[0]) / s[0], bf16_hi_to_f32(v[0]) / s[1], 0u, false);
    q0 = cvt_e4m3x2(bf16_lo_to_f32(v[1]) / s[2], bf16_hi_to_f32(v[1]) / s[3], q0, true);
    uint32_t q1 = cvt_e4m3x2(bf16_lo_to_f32(v[2]) / s[4], bf16_hi_to_f32(v[2]) / s[5], 0u, false);
    q1 = cvt_e4m3x2(bf16_lo_to_f32(v[3]) / s[6], bf16_hi_to_f32(v[3]) / s[7], q1, true);
    st_stream(codes + r * C8 + c, u32x2{q0, q1});
  }
}
// step 3: the column maxima (bf16 words) become the scales, in place
__global__ void __launch_bounds__(256) scales_from_max_kernel(uint32_t* __restrict__ cmax, int C) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const float mx = __builtin_bit_cast(float, cmax[c] << 16);
  cmax[c] = __builtin_bit_cast(uint32_t, mx > 0.f ? mx / 448.f : 1.f);
}

int launch_quantise_bf16(const void* X, int64_t R, int64_t C, int axis, void* codes, float* scales, hipStream_t s) {
  const int C8 = (int)(C / 8);
  if (axis == 1) {
    hipLaunchKernelGGL(quantise_bf16_rows_kernel, dim3((unsigned)((R + 3) / 4)), dim3(256), 0, s, static_cast<const u32x4*>(X), R, C8,
                       static_cast<u32x2*>(codes), scales);
    return (int)hipGetLastError();
  }
  uint32_t* cmax = reinterpret_cast<uint32_t*>(scales);
  if (int rc = launch_zero32(cmax, (size_t)C, s)) return rc;
  dim3 grid((unsigned)((C8 + 255) / 256), (unsigned)((R + QC_ROWS - 1) / QC_ROWS));
  hipLaunchKernelGGL(colmax_bf16_kernel, grid, dim3(256), 0, s, static_cast<const u32x4*>(X), R, C8, cmax);
  hipLaunchKernelGGL(quantise_bf16_cols_kernel, grid, dim3(256), 0, s, static_cast<const u32x4*>(X), R, C8, reinterpret_cast<const u32x4*>(cmax),
                     static_cast<u32x2*>(codes));
  hipLaunchKernelGGL(scales_from_max_kernel, dim3((unsigned)((C + 255) / 256)), dim3(256), 0, s, cmax, (int)C);
  return (int)hipGetLastError();
}

}  // namespace ffn24
