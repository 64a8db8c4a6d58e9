// C ABI of libffn24.so: argument checks, the context's workspace, and the kernel sequences.
#include <hip/hip_runtime.h>
#include <new>
#include "../../include/ffn24.h"
#include "launch.hpp"

using namespace ffn24;

namespace {
constexpr int NUM_KERNELS = 22;   // K_QUANT is shared by the 2:4 and the dense row-wise quantisation kernels
enum { K_UP = 0, K_DOWN, K_DH, K_DX, K_FW, K_DW2, K_DW1, KD_UP, KD_DOWN, KD_DH, KD_DX, KD_DW2, KD_DW1, K_TR_W, K_TR_ACT, K_PART, K_TR_DW1, K_QUANT, K_QUANT_DZ, K_QUANT_T, K_PANEL_W, K_PANEL_X };

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Intermediate tensors of ffn24_fwd_static.  One copy per GPU that loads this library, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress: the address kernels and copies use is the one that
// call returns for the current device (scratch_base below), never the name itself.
static __device__ __align__(256) unsigned char scratch[FFN24_STATIC_SCRATCH_BYTES];
unsigned char* scratch_dev[MAX_DEVICES];
std::atomic<bool> scratch_known[MAX_DEVICES];

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
int scratch_base(unsigned char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return FFN24_ERR_HIP;
  if (dev < 0 || dev >= MAX_DEVICES) return FFN24_ERR_HIP;
  if (!scratch_known[dev].load(std::memory_order_acquire)) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return FFN24_ERR_HIP; }
    scratch_dev[dev] = static_cast<unsigned char*>(p);   // threads that race here store the same address
    scratch_known[dev].store(true, std::memory_order_release);
  }
  *out = scratch_dev[dev];
  return FFN24_OK;
}
}  // namespace

struct ffn24_ctx {
  int64_t T, D, F;
  int flags;
  int device;
  int f8;                      // element type FFN24_FP8_E4M3 (forward only)
  float sx, sw1, sh, sw2;      // per-tensor scales of the fp8 path
  float sdy, sdz;              // fp8 backward: scale of the incoming gradient dY8 and of the stored dZ8
  int* perm; int perm_on;      // token permutation (FFN24_PERMUTE): device copy, and whether one is set
  // row-wise-scaled fp8 forward (FFN24_ROWWISE): caller's scale vectors, and the library's intermediate tensors
  const float *rsx, *rsw1, *rsw2;
  void* Hc16; uint8_t* meta16; uint32_t* rowmax; float* rsh;
  void* Hd16;                  // dense row-wise baseline: every activation as bf16 before quantisation
  // row-wise-scaled fp8 backward (FFN24_ROWWISE | FFN24_TRAINING): bf16 compressed dZ and the bf16 transposed operands before
  // their quantisation, the largest magnitude word of each of their rows, the scales derived from those, and the caller's
  // backward-side weight codes in panel form
  void* dZc16; void* Hct16; void* dZct16; uint8_t* meta_t16;
  uint32_t* rowmax_dz; uint32_t* hmax; uint32_t* zmax;
  float* sdz_t; float* sh_f; float* sdz_f;
  void* W2rp; void* W1cp;
  void* dZd16; void* Hdt16; void* dZdt16;   // dense row-wise backward: bf16 dZ [T][F], and the activation and dZ as [F][T]
  // workspace (device)
  void* Hc; uint8_t* meta; void* dZc; void* Hc_t; uint8_t* meta_t; void* dZc_t; void* Hdbg; void* Hd; void* dZd;
  void* W1t; void* W2t; void* Xt; void* dYt; void* Hd_t; void* dZd_t;   // K-contiguous copies of GEMM operands
  void* W2p;   // W2 itself in dense panel form (A operand of the dH GEMMs)
  void* W1p;   // W1 itself in B panel form (B operand of the dX GEMMs)
  // split weight gradients (FFN24_SPLIT)
  uint32_t* nnz; int* row_of_feat; int* feat_of_row; void* Hdn_t; void* dZdn_t; void* dW1t;
  void* Xp8; void* dYp8;         // fp8: X8 and dY8 in B panel form (rows in FFN order), what the up-projection and dH GEMMs read
  float* sx_p; float* sdy_p;     // row-wise fp8 with a token permutation: the caller's per-token scales of X and dY in FFN order
  void* Hdn8_t; void* dZdn8_t;   // row-wise fp8 split: the dense features' rows as e4m3 (Hdn_t, dZdn_t hold them in bf16 first)
  int n_dense;
  // telemetry (FFN24_TELEMETRY): device slots the kernels add to, their sums, and two pinned host snapshots that the
  // forward and the backward fill in turn (an event each tells when a snapshot has landed)
  unsigned long long* tele; long long* tele_sum; long long* tele_host;
  hipEvent_t tele_ev[2];
  int tele_seq;                 // snapshots enqueued so far
  long long tele_last[5]; int tele_have;   // the newest snapshot that was seen complete
  // forward state the backward calls read: the caller's X of the last forward, and which path ran it (the two paths
  // share the weight workspace, so a forward of one invalidates the saved state of the other)
  const void* X;
  int have_fwd24, have_fwd_dense;
  int prepared;                 // ffn24_prepare_weights: the workspace holds the re-arranged weights of that call
  // profiling
  int profiling;
  hipEvent_t ev[NUM_KERNELS][2];
  int ev_valid[NUM_KERNELS];
  unsigned long long* clk;      // clock samples of the GEMM kernels, CLK_SLOTS pairs per kernel id (gemm_core.hpp)
};

namespace {

struct Timed {
  ffn24_ctx* c; int k; hipStream_t s;
  Timed(ffn24_ctx* c_, int k_, hipStream_t s_) : c(c_), k(k_), s(s_) {
    if (c->profiling) { (void)hipEventRecord(c->ev[k][0], s); tl_gemm_clk = c->clk + (size_t)k * 2 * CLK_SLOTS; }
  }
  int done(int rc) {
    if (c->profiling) { (void)hipEventRecord(c->ev[k][1], s); c->ev_valid[k] = (rc == 0); tl_gemm_clk = nullptr; }
    return rc;
  }
};

int free_all(ffn24_ctx* c) {
  int bad = 0;
  void* bufs[] = {c->Hc, c->meta, c->dZc, c->Hc_t, c->meta_t, c->dZc_t, c->Hdbg, c->Hd, c->dZd,
                  c->W1t, c->W2t, c->Xt, c->dYt, c->Hd_t, c->dZd_t, c->W2p, c->W1p,
                  c->nnz, c->row_of_feat, c->feat_of_row, c->Hdn_t, c->dZdn_t, c->dW1t, c->Hc16, c->meta16, c->rowmax, c->rsh, c->perm, c->Hd16,
                  c->dZc16, c->Hct16, c->dZct16, c->meta_t16, c->rowmax_dz, c->hmax, c->zmax, c->sdz_t, c->sh_f, c->sdz_f, c->W2rp, c->W1cp,
                  c->dZd16, c->Hdt16, c->dZdt16, c->Hdn8_t, c->dZdn8_t, c->sx_p, c->sdy_p, c->Xp8, c->dYp8};
  for (void* b : bufs) if (b && hipFree(b) != hipSuccess) bad = 1;
  if (c->clk && hipFree(c->clk) != hipSuccess) bad = 1;
  if (c->tele && hipFree(c->tele) != hipSuccess) bad = 1;
  if (c->tele_sum && hipFree(c->tele_sum) != hipSuccess) bad = 1;
  if (c->tele_host && hipHostFree(c->tele_host) != hipSuccess) bad = 1;
  for (int j = 0; j < 2; j++) if (c->tele_ev[j]) (void)hipEventDestroy(c->tele_ev[j]);
  for (int k = 0; k < NUM_KERNELS; k++) for (int j = 0; j < 2; j++) if (c->ev[k][j]) (void)hipEventDestroy(c->ev[k][j]);
  return bad;
}

// the context's buffers live on the device that was current at ffn24_ctx_create
int check_device(const ffn24_ctx* c) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return FFN24_ERR_HIP;
  return dev == c->device ? FFN24_OK : FFN24_ERR_STATE;
}

// Telemetry snapshot: sum the slots, copy the five numbers to the next pinned host slot, mark it with an event.
int tele_snapshot(ffn24_ctx* c, long long path, hipStream_t s) {
  if (launch_tele_sum(c->tele, (long long)c->T * (long long)c->F, path, c->tele_sum, s)) return FFN24_ERR_HIP;
  const int slot = c->tele_seq & 1;
  if (hipMemcpyAsync(c->tele_host + 5 * slot, c->tele_sum, 8 * 5, hipMemcpyDeviceToHost, s) != hipSuccess) return FFN24_ERR_HIP;
  if (hipEventRecord(c->tele_ev[slot], s) != hipSuccess) return FFN24_ERR_HIP;
  c->tele_seq++;
  return FFN24_OK;
}

// The weight pass: W1 -> W1^T in dense panel form (A operand of the up-projection), W2 -> W2^T in B panel form (B
// operand of the down-projection) and, when the context trains, W2 itself in panel form (A operand of the dH GEMM)
// and W1 itself in B panel form (B operand of the dX GEMM) -- not in a row-wise fp8 context, whose backward takes the
// caller's differently quantised weight codes instead (W1p, W2p are NULL there).
int weight_pass(ffn24_ctx* c, const void* W1, const void* W2, hipStream_t s) {
  int D = (int)c->D, F = (int)c->F;
  Timed t(c, K_TR_W, s);
  int rc1;
  if (c->f8) {
    rc1 = launch_transpose8(W1, D, F, c->W1t, 1, c->W1p, 1, s);
    if (!rc1) rc1 = launch_transpose8(W2, F, D, c->W2t, 2, c->W2p, 0, s);
  } else {
    rc1 = launch_transpose(W1, D, F, c->W1t, 1, c->W1p, 1, nullptr, s);
    if (!rc1) rc1 = launch_transpose(W2, F, D, c->W2t, 2, c->W2p, 0, nullptr, s);
  }
  return t.done(rc1) ? FFN24_ERR_HIP : FFN24_OK;
}

// Weights of a forward call: both given (run the weight pass; prepared copies are gone after it), or both NULL (use
// the copies ffn24_prepare_weights left).
int resolve_weights(ffn24_ctx* c, const void* W1, const void* W2, hipStream_t s) {
  if (!W1 && !W2) return c->prepared ? FFN24_OK : FFN24_ERR_STATE;
  if (!W1 || !W2) return FFN24_ERR_NULL;
  if (misaligned(W1) || misaligned(W2)) return FFN24_ERR_ALIGN;
  c->prepared = 0;
  return weight_pass(c, W1, W2, s);
}

int check_ptrs(std::initializer_list<const void*> ps) {
  for (const void* p : ps) if (!p) return FFN24_ERR_NULL;
  for (const void* p : ps) if (misaligned(p)) return FFN24_ERR_ALIGN;
  return FFN24_OK;
}

}  // namespace

extern "C" {

const char* ffn24_strerror(int code) {
  switch (code) {
    case FFN24_OK: return "ok";
    case FFN24_ERR_NULL: return "a required pointer is NULL";
    case FFN24_ERR_SHAPE: return "a size violates the divisibility rules of the call";
    case FFN24_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    case FFN24_ERR_DTYPE: return "element type not supported";
    case FFN24_ERR_STATE: return "wrong call order, missing context flag, or the context belongs to another device";
    case FFN24_ERR_HIP: return "HIP runtime error";
    case FFN24_ERR_NOTREADY: return "no telemetry snapshot has completed yet";
    case FFN24_ERR_SCRATCH: return "the call's intermediate tensors do not fit the library's static scratch buffer";
    default: return "unknown ffn24 error code";
  }
}

int ffn24_ctx_create(ffn24_ctx** out, int64_t T, int64_t D, int64_t F, ffn24_dtype dtype, int flags) {
  if (!out) return FFN24_ERR_NULL;
  if (dtype != FFN24_BF16 && dtype != FFN24_FP8_E4M3) return FFN24_ERR_DTYPE;
  const bool f8 = dtype == FFN24_FP8_E4M3;
  if (f8 && (flags & FFN24_SPLIT) && !(flags & FFN24_ROWWISE)) return FFN24_ERR_DTYPE;                      // fp8: the split needs the row-wise recipe
  if ((flags & FFN24_SPLIT) && !(flags & FFN24_TRAINING)) return FFN24_ERR_STATE;
  if ((flags & FFN24_ROWWISE) && !f8) return FFN24_ERR_DTYPE;
  if ((flags & FFN24_PERMUTE) && f8 && !(flags & FFN24_ROWWISE)) return FFN24_ERR_DTYPE;                    // fp8: the permutation too
  if ((flags & FFN24_TELEMETRY) && f8) return FFN24_ERR_DTYPE;
  // the DMA gathers permuted rows with 32-bit byte offsets from the tensor base
  if ((flags & FFN24_PERMUTE) && (uint64_t)T * (uint64_t)D * (f8 ? 1u : 2u) >= (1ull << 32)) return FFN24_ERR_SHAPE;
  if (T <= 0 || D <= 0 || F <= 0 || T % 256 || D % 256 || F % 256) return FFN24_ERR_SHAPE;
  if (T > (1 << 20) || D > (1 << 20) || F > (1 << 20)) return FFN24_ERR_SHAPE;
  ffn24_ctx* c = new (std::nothrow) ffn24_ctx();
  if (!c) return FFN24_ERR_HIP;
  c->T = T; c->D = D; c->F = F; c->flags = flags; c->f8 = f8;
  c->sx = c->sw1 = c->sh = c->sw2 = c->sdy = c->sdz = 1.f;
  if (hipGetDevice(&c->device) != hipSuccess) { delete c; return FFN24_ERR_HIP; }
  const size_t es = f8 ? 1 : 2;   // bytes per stored element
  size_t tf = (size_t)T * (size_t)F, df = (size_t)D * (size_t)F, td = (size_t)T * (size_t)D;
  bool ok = hipMalloc(&c->Hc, tf * es / 2) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->meta), tf / 8) == hipSuccess &&
            hipMalloc(&c->W1t, es * df) == hipSuccess && hipMalloc(&c->W2t, es * df) == hipSuccess;
  if (ok && (flags & FFN24_TRAINING))
    ok = hipMalloc(&c->dZc, tf * es / 2) == hipSuccess && hipMalloc(&c->Hc_t, tf * es / 2) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->meta_t), tf / 8) == hipSuccess && hipMalloc(&c->dZc_t, tf * es / 2) == hipSuccess &&
         hipMalloc(&c->Xt, es * td) == hipSuccess && hipMalloc(&c->dYt, es * td) == hipSuccess;
  if (ok && (flags & FFN24_TRAINING) && !(flags & FFN24_ROWWISE))
    ok = hipMalloc(&c->W2p, es * df) == hipSuccess && hipMalloc(&c->W1p, es * df) == hipSuccess;
  if (ok && f8) ok = hipMalloc(&c->Xp8, td) == hipSuccess;
  if (ok && f8 && (flags & FFN24_TRAINING)) ok = hipMalloc(&c->dYp8, td) == hipSuccess;
  // an fp8 training context also keeps the kept activations before quantisation (bf16) for the backward's derivative
  if (ok && f8 && (flags & FFN24_TRAINING))
    ok = hipMalloc(&c->Hc16, tf) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->meta16), tf / 8) == hipSuccess;
  if (ok && (flags & FFN24_TELEMETRY)) {
    ok = hipMalloc(reinterpret_cast<void**>(&c->tele), 8 * TELE_WORDS) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->tele_sum), 8 * 5) == hipSuccess &&
         hipHostMalloc(reinterpret_cast<void**>(&c->tele_host), 8 * 5 * 2, hipHostMallocDefault) == hipSuccess;
    for (int j = 0; ok && j < 2; j++) ok = hipEventCreateWithFlags(&c->tele_ev[j], hipEventDisableTiming) == hipSuccess;
  }
  if (ok && (flags & FFN24_SPLIT))
    ok = hipMalloc(reinterpret_cast<void**>(&c->nnz), 4 * (size_t)F) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->row_of_feat), 4 * (size_t)F) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->feat_of_row), 4 * (size_t)F) == hipSuccess &&
         hipMalloc(&c->Hdn_t, tf / 2) == hipSuccess && hipMalloc(&c->dZdn_t, tf / 2) == hipSuccess &&   // up to F/4 dense rows
         hipMalloc(&c->dW1t, 2 * df) == hipSuccess;
  if (ok && f8 && (flags & FFN24_SPLIT)) ok = hipMalloc(&c->Hdn8_t, tf / 4) == hipSuccess && hipMalloc(&c->dZdn8_t, tf / 4) == hipSuccess;
  if (ok && (flags & FFN24_PERMUTE)) ok = hipMalloc(reinterpret_cast<void**>(&c->perm), 4 * (size_t)T) == hipSuccess;
  if (ok && (flags & FFN24_PERMUTE) && f8)
    ok = hipMalloc(reinterpret_cast<void**>(&c->sx_p), 4 * (size_t)T) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->sdy_p), 4 * (size_t)T) == hipSuccess;
  if (ok && (flags & FFN24_ROWWISE) && !c->Hc16)
    ok = hipMalloc(&c->Hc16, tf) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->meta16), tf / 8) == hipSuccess;
  if (ok && (flags & FFN24_ROWWISE))
    ok = hipMalloc(reinterpret_cast<void**>(&c->rowmax), 4 * (size_t)T) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->rsh), 4 * (size_t)T) == hipSuccess;
  if (ok && (flags & FFN24_ROWWISE) && (flags & FFN24_TRAINING))
    ok = hipMalloc(&c->dZc16, tf) == hipSuccess && hipMalloc(&c->Hct16, tf) == hipSuccess && hipMalloc(&c->dZct16, tf) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->meta_t16), tf / 8) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->rowmax_dz), 4 * (size_t)T) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->hmax), 4 * (size_t)F) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->zmax), 4 * (size_t)F) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->sdz_t), 4 * (size_t)T) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->sh_f), 4 * (size_t)F) == hipSuccess && hipMalloc(reinterpret_cast<void**>(&c->sdz_f), 4 * (size_t)F) == hipSuccess &&
         hipMalloc(&c->W2rp, df) == hipSuccess;
  if (ok && (flags & FFN24_ROWWISE) && (flags & FFN24_TRAINING) && (flags & FFN24_DENSE))   // (W1cp: only the dense dX GEMM wants W1_8c in panel form)
    ok = hipMalloc(&c->W1cp, df) == hipSuccess && hipMalloc(&c->dZd16, 2 * tf) == hipSuccess && hipMalloc(&c->Hdt16, 2 * tf) == hipSuccess && hipMalloc(&c->dZdt16, 2 * tf) == hipSuccess;
  if (ok && (flags & FFN24_DENSE)) ok = hipMalloc(&c->Hd, es * tf) == hipSuccess;
  if (ok && (flags & FFN24_DENSE) && (flags & FFN24_ROWWISE)) ok = hipMalloc(&c->Hd16, 2 * tf) == hipSuccess;
  if (ok && (flags & FFN24_DENSE) && (flags & FFN24_TRAINING))
    ok = hipMalloc(&c->dZd, es * tf) == hipSuccess && hipMalloc(&c->Hd_t, es * tf) == hipSuccess && hipMalloc(&c->dZd_t, es * tf) == hipSuccess;
  if (ok && f8 && (flags & FFN24_DENSE) && (flags & FFN24_TRAINING) && !c->Hd16) ok = hipMalloc(&c->Hd16, 2 * tf) == hipSuccess;
  if (ok && (flags & FFN24_DEBUG_DUMP_H)) ok = hipMalloc(&c->Hdbg, 2 * tf) == hipSuccess;
  for (int k = 0; ok && k < NUM_KERNELS; k++)
    for (int j = 0; ok && j < 2; j++) ok = hipEventCreate(&c->ev[k][j]) == hipSuccess;
  if (ok) ok = hipMalloc(reinterpret_cast<void**>(&c->clk), (size_t)NUM_KERNELS * 2 * CLK_SLOTS * 8) == hipSuccess &&
               hipMemset(c->clk, 0, (size_t)NUM_KERNELS * 2 * CLK_SLOTS * 8) == hipSuccess;
  if (!ok) { (void)hipGetLastError(); free_all(c); delete c; return FFN24_ERR_HIP; }
  *out = c;
  return FFN24_OK;
}

int ffn24_ctx_destroy(ffn24_ctx* c) {
  if (!c) return FFN24_OK;
  int bad = free_all(c);
  delete c;
  return bad ? FFN24_ERR_HIP : FFN24_OK;
}

int ffn24_set_scales(ffn24_ctx* c, float sx, float sw1, float sh, float sw2) {
  if (!c) return FFN24_ERR_NULL;
  if (!c->f8) return FFN24_ERR_DTYPE;
  if (!(sx > 0.f) || !(sw1 > 0.f) || !(sh > 0.f) || !(sw2 > 0.f)) return FFN24_ERR_SHAPE;
  c->sx = sx; c->sw1 = sw1; c->sh = sh; c->sw2 = sw2;
  return FFN24_OK;
}

int ffn24_set_bwd_scales(ffn24_ctx* c, float sdy, float sdz) {
  if (!c) return FFN24_ERR_NULL;
  if (!c->f8) return FFN24_ERR_DTYPE;
  if (!(c->flags & FFN24_TRAINING)) return FFN24_ERR_STATE;
  if (!(sdy > 0.f) || !(sdz > 0.f)) return FFN24_ERR_SHAPE;
  c->sdy = sdy; c->sdz = sdz;
  return FFN24_OK;
}

int ffn24_set_row_scales(ffn24_ctx* c, const float* sx, const float* sw1, const float* sw2) {
  if (!c) return FFN24_ERR_NULL;
  if (!(c->flags & FFN24_ROWWISE)) return FFN24_ERR_STATE;
  if (!sx || !sw1 || !sw2) return FFN24_ERR_NULL;
  if (misaligned(sx) || misaligned(sw1) || misaligned(sw2)) return FFN24_ERR_ALIGN;
  c->rsx = sx; c->rsw1 = sw1; c->rsw2 = sw2;
  return FFN24_OK;
}

int ffn24_set_token_permutation(ffn24_ctx* c, const int32_t* perm_host) {
  if (!c) return FFN24_ERR_NULL;
  if (!(c->flags & FFN24_PERMUTE)) return FFN24_ERR_STATE;
  c->have_fwd24 = 0;
  if (!perm_host) { c->perm_on = 0; return FFN24_OK; }
  if (int rc = check_device(c)) return rc;
  // validated on the host: every index in range and used exactly once (the kernels gather and scatter rows with it)
  const int64_t T = c->T;
  uint8_t* seen = new (std::nothrow) uint8_t[(size_t)T]();
  if (!seen) return FFN24_ERR_HIP;
  bool ok = true;
  for (int64_t i = 0; i < T && ok; i++) {
    int32_t v = perm_host[i];
    ok = v >= 0 && v < T && !seen[v];
    if (ok) seen[v] = 1;
  }
  delete[] seen;
  if (!ok) return FFN24_ERR_SHAPE;
  // synchronous copy: a set-up call, and no stream may still be reading the old permutation
  if (hipDeviceSynchronize() != hipSuccess) return FFN24_ERR_HIP;
  if (hipMemcpy(c->perm, perm_host, 4 * (size_t)T, hipMemcpyHostToDevice) != hipSuccess) return FFN24_ERR_HIP;
  c->perm_on = 1;
  return FFN24_OK;
}

int ffn24_set_split(ffn24_ctx* c, int64_t n_dense) {
  if (!c) return FFN24_ERR_NULL;
  if (!(c->flags & FFN24_SPLIT)) return FFN24_ERR_STATE;
  if (n_dense < 0 || n_dense % 256 || n_dense > c->F / 4) return FFN24_ERR_SHAPE;
  c->n_dense = (int)n_dense;
  c->have_fwd24 = 0;   // the statistics of an earlier forward do not belong to this setting
  return FFN24_OK;
}

int ffn24_prepare_weights(ffn24_ctx* c, const void* W1, const void* W2, void* stream) {
  if (!c) return FFN24_ERR_NULL;
  int rc = check_device(c);
  if (rc) return rc;
  rc = check_ptrs({W1, W2});
  if (rc) return rc;
  c->prepared = 0;
  c->have_fwd24 = c->have_fwd_dense = 0;
  if ((rc = weight_pass(c, W1, W2, static_cast<hipStream_t>(stream)))) return rc;
  c->prepared = 1;
  return FFN24_OK;
}

int ffn24_get_telemetry(ffn24_ctx* c, int64_t* counts, int wait) {
  if (!c || !counts) return FFN24_ERR_NULL;
  if (!(c->flags & FFN24_TELEMETRY)) return FFN24_ERR_STATE;
  // newest snapshot first, then the one before it (its host slot is not written again before a further call enqueues)
  for (int back = 1; back <= 2 && back <= c->tele_seq; back++) {
    const int slot = (c->tele_seq - back) & 1;
    hipError_t e = (wait && back == 1) ? hipEventSynchronize(c->tele_ev[slot]) : hipEventQuery(c->tele_ev[slot]);
    if (e == hipSuccess) {
      for (int i = 0; i < 5; i++) c->tele_last[i] = c->tele_host[5 * slot + i];
      c->tele_have = 1;
      break;
    }
    if (e != hipErrorNotReady) { (void)hipGetLastError(); return FFN24_ERR_HIP; }
  }
  (void)hipGetLastError();   // a pending event leaves hipErrorNotReady behind
  if (!c->tele_have) return FFN24_ERR_NOTREADY;
  for (int i = 0; i < 5; i++) counts[i] = (int64_t)c->tele_last[i];
  return FFN24_OK;
}

int ffn24_policy_use_sparse(ffn24_ctx* c, double min_sparsity, int* use_sparse) {
  if (!c || !use_sparse) return FFN24_ERR_NULL;
  if (!(min_sparsity >= 0.0 && min_sparsity <= 1.0)) return FFN24_ERR_SHAPE;
  int64_t n[5];
  int rc = ffn24_get_telemetry(c, n, 0);
  if (rc == FFN24_ERR_NOTREADY) { *use_sparse = 0; return FFN24_OK; }   // nothing measured yet: stay dense
  if (rc) return rc;
  *use_sparse = (1.0 - (double)n[1] / (double)n[0]) >= min_sparsity;
  return FFN24_OK;
}

int ffn24_set_profiling(ffn24_ctx* c, int on) {
  if (!c) return FFN24_ERR_NULL;
  c->profiling = on != 0;
  return FFN24_OK;
}

int ffn24_kernel_ms(ffn24_ctx* c, int k, float* ms) {
  if (!c || !ms) return FFN24_ERR_NULL;
  if (k < 0 || k >= NUM_KERNELS) return FFN24_ERR_SHAPE;
  if (!c->ev_valid[k]) return FFN24_ERR_STATE;
  if (hipEventSynchronize(c->ev[k][1]) != hipSuccess) return FFN24_ERR_HIP;
  if (hipEventElapsedTime(ms, c->ev[k][0], c->ev[k][1]) != hipSuccess) return FFN24_ERR_HIP;
  return FFN24_OK;
}

int ffn24_kernel_mhz(ffn24_ctx* c, int k, float* mhz) {
  if (!c || !mhz) return FFN24_ERR_NULL;
  if (k < 0 || k >= NUM_KERNELS) return FFN24_ERR_SHAPE;
  if (!c->ev_valid[k]) return FFN24_ERR_STATE;
  if (hipEventSynchronize(c->ev[k][1]) != hipSuccess) return FFN24_ERR_HIP;
  unsigned long long h[2 * CLK_SLOTS];
  if (hipMemcpy(h, c->clk + (size_t)k * 2 * CLK_SLOTS, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return FFN24_ERR_HIP;
  double t = 0, r = 0;
  for (int i = 0; i < CLK_SLOTS; i++) { t += (double)h[2 * i]; r += (double)h[2 * i + 1]; }
  if (r <= 0) return FFN24_ERR_STATE;   // not a GEMM kernel: nothing samples the clock there
  *mhz = (float)(100.0 * t / r);
  return FFN24_OK;
}

int ffn24_probe_mfma_rate(int kind, int iters, double* cycles_per_op, double* mhz, double* tflops_dense_equivalent) {
  if (!cycles_per_op || !mhz || !tflops_dense_equivalent) return FFN24_ERR_NULL;
  if (kind < 0 || kind > 3 || iters < 1 || iters > (1 << 22)) return FFN24_ERR_SHAPE;
  return probe_mfma_rate(kind, iters, cycles_per_op, mhz, tflops_dense_equivalent) ? FFN24_ERR_HIP : FFN24_OK;
}

int ffn24_probe_gemm(int sparse, int variant, int64_t M, int64_t N, int64_t K, int reps, double* ms_median, double* mhz) {
  if (!ms_median || !mhz) return FFN24_ERR_NULL;
  if (M <= 0 || N <= 0 || K < 512 || M % 256 || N % 256 || K % 128 || M > (1 << 16) || N > (1 << 16) || K > (1 << 16) || reps < 1 || reps > 1000)
    return FFN24_ERR_SHAPE;
  int rc = probe_gemm(sparse != 0, variant, (int)M, (int)N, (int)K, reps, ms_median, mhz);
  return rc == 2 ? FFN24_ERR_SHAPE : (rc ? FFN24_ERR_HIP : FFN24_OK);
}

int ffn24_probe_copy(int64_t bytes, int reps, double* ms_median) {
  if (!ms_median) return FFN24_ERR_NULL;
  if (bytes < 4096 || bytes % 4096 || bytes > ((int64_t)16 << 30) || reps < 1 || reps > 1000) return FFN24_ERR_SHAPE;
  return probe_copy((size_t)bytes, reps, ms_median) ? FFN24_ERR_HIP : FFN24_OK;
}

int ffn24_saved_bytes(ffn24_ctx* c, int which, int64_t* nbytes) {
  if (!c || !nbytes) return FFN24_ERR_NULL;
  int64_t tf = c->T * c->F;
  const int64_t es = c->f8 ? 1 : 2;
  switch (which) {
    case 0: case 2: case 3: case 5: *nbytes = tf * es / 2; break;
    case 1: case 4: *nbytes = tf / 8; break;
    case 6: *nbytes = 2 * tf; break;
    case 7: case 8: *nbytes = es * tf; break;
    case 9: case 10: *nbytes = 4 * c->F; break;
    case 11: *nbytes = 4 * c->T; break;
    case 12: case 16: *nbytes = tf; break;
    case 13: *nbytes = 4 * c->T; break;
    case 14: case 15: *nbytes = 4 * c->F; break;
    case 17: *nbytes = 2 * tf; break;
    case 18: case 19: *nbytes = tf; break;
    case 20: case 21: *nbytes = es * tf / 4; break;
    default: return FFN24_ERR_SHAPE;
  }
  return FFN24_OK;
}

int ffn24_copy_saved(ffn24_ctx* c, int which, void* dst, int64_t dst_bytes, void* stream) {
  if (!c || !dst) return FFN24_ERR_NULL;
  if (misaligned(dst)) return FFN24_ERR_ALIGN;
  int64_t need = 0;
  int rc = check_device(c);
  if (rc) return rc;
  rc = ffn24_saved_bytes(c, which, &need);
  if (rc) return rc;
  if (dst_bytes != need) return FFN24_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int T = (int)c->T, F = (int)c->F;
  const void* src = nullptr;
  int rows = 0, K = 0, piece = 0;   // piece != 0: the buffer is in panel form
  switch (which) {
    case 0: src = c->Hc; rows = T; K = F; piece = 64; break;
    case 1: src = c->meta; rows = T; K = F; piece = 8; break;
    case 2: src = c->dZc; rows = T; K = F; piece = 64; break;
    case 3: src = c->Hc_t; rows = F; K = T; piece = 64; break;
    case 4: src = c->meta_t; rows = F; K = T; piece = 8; break;
    case 5: src = c->dZc_t; rows = F; K = T; piece = 64; break;
    case 6: src = c->Hdbg; break;
    case 7: src = c->Hd; break;
    case 8: src = c->dZd; break;
    case 9: src = c->nnz; break;
    case 10: src = c->feat_of_row; break;
    case 11: src = c->rsh; break;
    case 13: src = c->sdz_t; break;
    case 14: src = c->sh_f; break;
    case 15: src = c->sdz_f; break;
    case 16: src = c->dZc16; break;
    case 17: src = c->dZd16; break;
    case 18: src = c->Hd_t; break;
    case 19: src = c->dZd_t; break;
    case 20: src = c->f8 ? c->Hdn8_t : c->Hdn_t; break;
    case 21: src = c->f8 ? c->dZdn8_t : c->dZdn_t; break;
    default: src = c->Hc16; break;
  }
  if (!src) return FFN24_ERR_STATE;
  if (which == 17)   // the dense row-wise backward's bf16 dZ [T][F]: dense bf16 panel form (64-byte pieces of 32 k)
    return launch_unpanel(src, T, F / 32, 64, dst, s) ? FFN24_ERR_HIP : FFN24_OK;
  if (which == 18 || which == 19) {   // the dense fp8 backward's transposed operands [F][T]: dense fp8 panel form (64-byte pieces of 64 k)
    if (!c->f8) return FFN24_ERR_STATE;
    return launch_unpanel(src, F, T / 64, 64, dst, s) ? FFN24_ERR_HIP : FFN24_OK;
  }
  if (which == 20 || which == 21)   // the split's dense feature rows [F/4][T] (the first n_dense are valid): dense panel form
    return launch_unpanel(src, F / 4, c->f8 ? T / 64 : T / 32, 64, dst, s) ? FFN24_ERR_HIP : FFN24_OK;
  if (which == 12 || which == 16)   // bf16 kept values of an fp8 context: bf16 panel form (64-byte pieces of 64 k)
    return launch_unpanel(src, T, F / 64, 64, dst, s) ? FFN24_ERR_HIP : FFN24_OK;
  if (which >= 9) return hipMemcpyAsync(dst, src, (size_t)need, hipMemcpyDeviceToDevice, s) == hipSuccess ? FFN24_OK : FFN24_ERR_HIP;
  if (which >= 7)   // the dense baseline's H and dZ: dense panel form, 64-byte pieces of 32 (fp8: 64) k
    return launch_unpanel(src, T, c->f8 ? F / 64 : F / 32, 64, dst, s) ? FFN24_ERR_HIP : FFN24_OK;
  if (piece) {
    // a piece covers 64 k (bf16) or 128 k (fp8, whose metadata pieces are twice as long)
    const int npanels = c->f8 ? K / 128 : K / 64;
    if (c->f8 && piece == 8) piece = 16;
    return launch_unpanel(src, rows, npanels, piece, dst, s) ? FFN24_ERR_HIP : FFN24_OK;
  }
  return hipMemcpyAsync(dst, src, (size_t)need, hipMemcpyDeviceToDevice, s) == hipSuccess ? FFN24_OK : FFN24_ERR_HIP;
}

int sparsify24(const void* H, int64_t rows, int64_t cols, ffn24_dtype dtype, void* values, uint8_t* meta, void* stream) {
  if (dtype != FFN24_BF16 && dtype != FFN24_FP8_E4M3) return FFN24_ERR_DTYPE;
  const bool f8 = dtype == FFN24_FP8_E4M3;
  if (rows < 0 || cols < 0 || cols % (f8 ? 16 : 8)) return FFN24_ERR_SHAPE;
  if (rows == 0 || cols == 0) return FFN24_OK;
  if (rows > (INT64_MAX / 2) / cols) return FFN24_ERR_SHAPE;
  if (!H || !values || !meta) return FFN24_ERR_NULL;
  if (misaligned(H) || misaligned(values) || (f8 && misaligned(meta))) return FFN24_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (f8) return launch_sparsify24_bytes(H, rows, cols, values, meta, s) ? FFN24_ERR_HIP : FFN24_OK;
  return launch_sparsify24(H, rows, cols, values, meta, s) ? FFN24_ERR_HIP : FFN24_OK;
}

int quantise_e4m3(const void* X, int64_t rows, int64_t cols, int axis, void* codes, float* scales, void* stream) {
  if (axis != 0 && axis != 1) return FFN24_ERR_SHAPE;
  if (rows < 0 || cols < 0 || cols % 8 || rows > ((int64_t)1 << 24) || cols > ((int64_t)1 << 24)) return FFN24_ERR_SHAPE;
  if (rows == 0 || cols == 0) return FFN24_OK;
  if (!X || !codes || !scales) return FFN24_ERR_NULL;
  if (misaligned(X) || misaligned(codes) || misaligned(scales)) return FFN24_ERR_ALIGN;
  return launch_quantise_bf16(X, rows, cols, axis, codes, scales, static_cast<hipStream_t>(stream)) ? FFN24_ERR_HIP : FFN24_OK;
}

int sparsify24_quantise(const void* H, int64_t rows, int64_t cols, float scale, void* values8, uint8_t* meta, void* stream) {
  if (rows < 0 || cols < 0 || cols % 8) return FFN24_ERR_SHAPE;
  if (!(scale > 0.f)) return FFN24_ERR_SHAPE;
  if (rows == 0 || cols == 0) return FFN24_OK;
  if (rows > (INT64_MAX / 2) / cols) return FFN24_ERR_SHAPE;
  if (!H || !values8 || !meta) return FFN24_ERR_NULL;
  if (misaligned(H) || misaligned(values8)) return FFN24_ERR_ALIGN;
  return launch_sparsify24_quant(H, rows, cols, scale, values8, meta, static_cast<hipStream_t>(stream)) ? FFN24_ERR_HIP : FFN24_OK;
}

int sparsify24_featurewise(const void* Hc, const uint8_t* meta, const void* dZc, int64_t T, int64_t F,
                           void* Hc_t, uint8_t* meta_t, void* dZc_t, void* stream) {
  if (T <= 0 || F <= 0 || T % 128 || F % 64 || T > (1 << 20) || F > (1 << 20)) return FFN24_ERR_SHAPE;
  if (!Hc || !meta || !Hc_t || !meta_t) return FFN24_ERR_NULL;
  if ((dZc == nullptr) != (dZc_t == nullptr)) return FFN24_ERR_NULL;
  if (misaligned(Hc) || misaligned(meta) || misaligned(Hc_t) || misaligned(meta_t) || misaligned(dZc) || misaligned(dZc_t))
    return FFN24_ERR_ALIGN;
  return launch_featurewise24(Hc, meta, dZc, (int)T, (int)F, Hc_t, meta_t, dZc_t, 0, nullptr, static_cast<hipStream_t>(stream)) ? FFN24_ERR_HIP : FFN24_OK;
}

int spmm24(const void* values, const uint8_t* meta, const void* Bt, int64_t M, int64_t N, int64_t K, void* C, void* stream) {
  if (M <= 0 || N <= 0 || K <= 0 || M % 256 || N % 256 || K % 64 || M > (1 << 20) || N > (1 << 20) || K > (1 << 20)) return FFN24_ERR_SHAPE;
  int rc = check_ptrs({values, meta, Bt, C});
  if (rc) return rc;
  return launch_sp_rowmajor(values, meta, 0, Bt, 0, (int)M, (int)N, (int)K, C, static_cast<hipStream_t>(stream)) ? FFN24_ERR_HIP : FFN24_OK;
}

int ffn24_fwd(ffn24_ctx* c, const void* X, const void* W1, const float* b1, const void* W2, void* Y, void* stream) {
  if (!c) return FFN24_ERR_NULL;
  int rc = check_device(c);
  if (rc) return rc;
  rc = check_ptrs({X, Y});
  if (rc) return rc;
  if (b1 && misaligned(b1)) return FFN24_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int T = (int)c->T, D = (int)c->D, F = (int)c->F;
  c->have_fwd24 = c->have_fwd_dense = 0;
  if (c->f8 && (c->flags & FFN24_ROWWISE) && !c->rsx) return FFN24_ERR_STATE;
  if ((rc = resolve_weights(c, W1, W2, s))) return rc;
  if (c->f8 && (c->flags & FFN24_ROWWISE)) {
    // row-wise scaling: up-projection (bf16 kept values + row maxima), row-wise quantisation, scaled sparse GEMM
    if (launch_zero32(c->rowmax, (size_t)T, s)) return FFN24_ERR_HIP;
    uint32_t* nnz = (c->flags & FFN24_SPLIT) && c->n_dense > 0 ? c->nnz : nullptr;
    if (nnz && launch_zero32(nnz, (size_t)F, s)) return FFN24_ERR_HIP;
    // token permutation: position p inside the FFN holds token perm[p] -- its row of X8 is gathered by the pass that brings X8
    // into panel form, its scale by a small kernel; everything in between lives in FFN order, and Y's rows go back to their tokens
    const int* perm = c->perm_on ? c->perm : nullptr;
    const float* sx = c->rsx;
    if (perm) { if (launch_gather_f32(c->rsx, perm, T, c->sx_p, s)) return FFN24_ERR_HIP; sx = c->sx_p; }
    { Timed t(c, K_PANEL_X, s); if (t.done(launch_panelise8_rows(X, T, D, c->Xp8, 1, perm, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_UP, s);
      if (t.done(launch_up_prune24_f8_rowwise(c->W1t, c->Xp8, b1, T, D, F, sx, c->rsw1, c->Hc16, c->meta16, c->Hdbg, c->rowmax, nnz, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_QUANT, s);
      if (t.done(launch_quantise_rows(c->Hc16, c->meta16, c->rowmax, T, F, c->Hc, c->meta, c->rsh, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DOWN, s);
      int rc1 = perm ? launch_sp_rowmajor_f8_rowwise_mapped(c->Hc, c->meta, c->W2t, 1, T, D, F, c->rsh, c->rsw2, Y, perm, s)
                     : launch_sp_rowmajor_f8_rowwise(c->Hc, c->meta, c->W2t, 1, T, D, F, c->rsh, c->rsw2, Y, s);
      if (t.done(rc1)) return FFN24_ERR_HIP; }
    if (c->flags & FFN24_TRAINING) { c->X = X; c->have_fwd24 = 1; }
    return FFN24_OK;
  }
  if (c->f8) {
    const bool train = (c->flags & FFN24_TRAINING) != 0;
    { Timed t(c, K_PANEL_X, s); if (t.done(launch_panelise8(X, T, D, c->Xp8, 1, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_UP, s);
      if (t.done(launch_up_prune24_f8(c->W1t, c->Xp8, b1, T, D, F, c->sx * c->sw1, c->sh, c->Hc, c->meta, c->Hdbg, train ? c->Hc16 : nullptr,
                                      train ? c->meta16 : nullptr, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DOWN, s);
      if (t.done(launch_sp_rowmajor_f8(c->Hc, c->meta, 1, c->W2t, 1, T, D, F, c->sh * c->sw2, Y, s))) return FFN24_ERR_HIP; }
    if (train) { c->X = X; c->have_fwd24 = 1; }
    return FFN24_OK;
  }
  uint32_t* nnz = (c->flags & FFN24_SPLIT) && c->n_dense > 0 ? c->nnz : nullptr;
  if (nnz && launch_zero32(nnz, (size_t)F, s)) return FFN24_ERR_HIP;
  if (c->tele && launch_zero32(reinterpret_cast<uint32_t*>(c->tele), 2 * TELE_WORDS, s)) return FFN24_ERR_HIP;
  const int* perm = c->perm_on ? c->perm : nullptr;   // position p inside the FFN holds token perm[p]
  { Timed t(c, K_UP, s);   if (t.done(launch_up_prune24(c->W1t, X, b1, T, D, F, c->Hc, c->meta, c->Hdbg, nnz, c->tele, perm, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_DOWN, s);
    int rc1 = perm ? launch_sp_rowmajor_mapped(c->Hc, c->meta, 1, c->W2t, 1, T, D, F, Y, perm, s) : launch_sp_rowmajor(c->Hc, c->meta, 1, c->W2t, 1, T, D, F, Y, s);
    if (t.done(rc1)) return FFN24_ERR_HIP; }
  if (c->tele && (rc = tele_snapshot(c, 1, s))) return rc;
  c->X = X; c->have_fwd24 = 1;
  return FFN24_OK;
}

int64_t ffn24_static_scratch_needed(int64_t T, int64_t D, int64_t F) {
  if (T <= 0 || D <= 0 || F <= 0 || T > (1 << 20) || D > (1 << 20) || F > (1 << 20)) return -1;
  // compressed activation (kept values + metadata) and the two re-arranged weights; every part a multiple of 256 bytes
  return T * F + T * F / 8 + 2 * (2 * D * F);
}

int ffn24_fwd_static(const void* X, const void* W1, const float* b1, const void* W2, void* Y, int64_t T, int64_t D, int64_t F, void* stream) {
  if (T <= 0 || D <= 0 || F <= 0 || T % 256 || D % 256 || F % 256 || T > (1 << 20) || D > (1 << 20) || F > (1 << 20)) return FFN24_ERR_SHAPE;
  if (ffn24_static_scratch_needed(T, D, F) > (int64_t)FFN24_STATIC_SCRATCH_BYTES) return FFN24_ERR_SCRATCH;
  int rc = check_ptrs({X, W1, W2, Y});
  if (rc) return rc;
  if (b1 && misaligned(b1)) return FFN24_ERR_ALIGN;
  unsigned char* base = nullptr;
  if ((rc = scratch_base(&base))) return rc;
  // carve-up of the scratch buffer: Hc [T][F/2] bf16 | meta [T][F/8] | W1^T [F][D] bf16 | W2^T [D][F] bf16 (panel forms).
  // Every byte a kernel below reads from it has been written by an earlier kernel of this same call, so nothing has to
  // start at zero and what a previous call left behind is never seen.
  const size_t tf = (size_t)T * (size_t)F, df = (size_t)D * (size_t)F;
  unsigned char* Hc = base;
  uint8_t* meta = base + tf;
  unsigned char* W1t = base + tf + tf / 8;
  unsigned char* W2t = W1t + 2 * df;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int Ti = (int)T, Di = (int)D, Fi = (int)F;
  if (launch_transpose(W1, Di, Fi, W1t, 1, nullptr, 0, nullptr, s)) return FFN24_ERR_HIP;
  if (launch_transpose(W2, Fi, Di, W2t, 2, nullptr, 0, nullptr, s)) return FFN24_ERR_HIP;
  if (launch_up_prune24(W1t, X, b1, Ti, Di, Fi, Hc, meta, nullptr, nullptr, nullptr, nullptr, s)) return FFN24_ERR_HIP;
  if (launch_sp_rowmajor(Hc, meta, 1, W2t, 1, Ti, Di, Fi, Y, s)) return FFN24_ERR_HIP;
  return FFN24_OK;
}

int ffn24_bwd_rowwise(ffn24_ctx* c, const ffn24_rowwise_bwd_operands* op, void* dX, void* dW1, void* dW2, void* stream) {
  if (!c || !op) return FFN24_ERR_NULL;
  if (!c->f8 || !(c->flags & FFN24_ROWWISE) || !(c->flags & FFN24_TRAINING) || !c->have_fwd24) return FFN24_ERR_STATE;
  int rc = check_device(c);
  if (rc) return rc;
  rc = check_ptrs({op->dY8r, op->sdy_t, op->dY8c, op->sdy_d, op->X8c, op->sx_d, op->W2_8r, op->sw2_f, op->W1_8c, op->sw1_d, dX, dW1, dW2});
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int T = (int)c->T, D = (int)c->D, F = (int)c->F;
  // the caller's W2 codes (quantised per hidden feature) into the panel form the dH GEMM streams its A operand in; W1 (quantised
  // per model dimension) is the B operand of the sparse dX GEMM, whose stages take a whole 128-byte line of every row: it is read
  // where it lies (measured: no slower than from a panel-form copy, and the copy costs 0.1 ms)
  // dY8r likewise (the B operand of the dense dH GEMM, 64 bytes of every row a stage), with the rows of a token permutation gathered
  const int* perm = c->perm_on ? c->perm : nullptr;
  { Timed t(c, K_PANEL_W, s);
    int rc1 = launch_panelise8(op->W2_8r, F, D, c->W2rp, 0, s);
    if (t.done(rc1 ? rc1 : launch_panelise8_rows(op->dY8r, T, D, c->dYp8, 1, perm, s))) return FFN24_ERR_HIP; }
  if (launch_zero32(c->rowmax_dz, (size_t)T, s) || launch_zero32(c->hmax, (size_t)F, s) || launch_zero32(c->zmax, (size_t)F, s)) return FFN24_ERR_HIP;
  const float* sdy_t = op->sdy_t;                     // as in the forward: the scales of the gathered rows, and dX's rows scattered back
  if (perm) { if (launch_gather_f32(op->sdy_t, perm, T, c->sdy_p, s)) return FFN24_ERR_HIP; sdy_t = c->sdy_p; }
  { Timed t(c, K_DH, s);
    if (t.done(launch_dh_gather_f8_rowwise(c->W2rp, c->dYp8, c->Hc16, c->meta16, T, D, F, op->sw2_f, sdy_t, c->dZc16, c->rowmax_dz, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_QUANT_DZ, s);
    if (t.done(launch_quantise_rows(c->dZc16, c->meta16, c->rowmax_dz, T, F, c->dZc, c->meta, c->sdz_t, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_DX, s);
    int rc1 = perm ? launch_sp_rowmajor_f8_rowwise_mapped(c->dZc, c->meta, op->W1_8c, 0, T, D, F, c->sdz_t, op->sw1_d, dX, perm, s)
                   : launch_sp_rowmajor_f8_rowwise(c->dZc, c->meta, op->W1_8c, 0, T, D, F, c->sdz_t, op->sw1_d, dX, s);
    if (t.done(rc1)) return FFN24_ERR_HIP; }
  if ((c->flags & FFN24_SPLIT) && c->n_dense > 0) {
    // Sec. 2, "Optimization 1" on the row-wise recipe: the n_dense least sparse features keep the token-wise mask only; every
    // row of the permuted feature space (sparse rows first) gets its own scale, the sparse rows are quantised in compressed form,
    // the dense ones as plain rows, and each weight gradient is one launch of a sparse and a dense fp8 GEMM
    const int nd = c->n_dense, ns = F - nd;
    { Timed t(c, K_PART, s); if (t.done(launch_split_partition(c->nnz, F, nd, T, c->row_of_feat, c->feat_of_row, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_FW, s);
      if (t.done(launch_featurewise24_split(c->Hc16, c->meta16, c->dZc16, T, F, c->row_of_feat, ns, c->Hct16, c->meta_t16, c->dZct16, c->Hdn_t, c->dZdn_t,
                                            nullptr, c->hmax, c->zmax, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_QUANT_T, s);
      int rc1 = launch_quantise_rows(c->Hct16, c->meta_t16, c->hmax, ns, T, c->Hc_t, c->meta_t, c->sh_f, s);
      if (!rc1) rc1 = launch_quantise_rows(c->dZct16, c->meta_t16, c->zmax, ns, T, c->dZc_t, c->meta_t, c->sdz_f, s);
      if (!rc1) rc1 = launch_quantise_rows_dense(c->Hdn_t, c->hmax + ns, nd, T, c->Hdn8_t, c->sh_f + ns, s);
      if (t.done(rc1 ? rc1 : launch_quantise_rows_dense(c->dZdn_t, c->zmax + ns, nd, T, c->dZdn8_t, c->sdz_f + ns, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_TR_ACT, s);
      int rc1 = launch_transpose8_rows(op->dY8c, T, D, c->dYt, 2, perm, s);
      if (t.done(rc1 ? rc1 : launch_transpose8_rows(op->X8c, T, D, c->Xt, 2, perm, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DW2, s);
      if (t.done(launch_split_wgrad_f8_rowwise(c->Hc_t, c->meta_t, ns, c->Hdn8_t, nd, c->dYt, D, T, c->sh_f, op->sdy_d, dW2, D, c->feat_of_row, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DW1, s);
      if (t.done(launch_split_wgrad_f8_rowwise(c->dZc_t, c->meta_t, ns, c->dZdn8_t, nd, c->Xt, D, T, c->sdz_f, op->sx_d, c->dW1t, D, c->feat_of_row, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_TR_DW1, s); if (t.done(launch_transpose(c->dW1t, F, D, dW1, 0, nullptr, 0, nullptr, s))) return FFN24_ERR_HIP; }
    return FFN24_OK;
  }
  { Timed t(c, K_FW, s);
    if (t.done(launch_featurewise24_rowmax(c->Hc16, c->meta16, c->dZc16, T, F, c->Hct16, c->meta_t16, c->dZct16, c->hmax, c->zmax, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_QUANT_T, s);
    int rc1 = launch_quantise_rows(c->Hct16, c->meta_t16, c->hmax, F, T, c->Hc_t, c->meta_t, c->sh_f, s);
    if (t.done(rc1 ? rc1 : launch_quantise_rows(c->dZct16, c->meta_t16, c->zmax, F, T, c->dZc_t, c->meta_t, c->sdz_f, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_TR_ACT, s);
    int rc1 = launch_transpose8_rows(op->dY8c, T, D, c->dYt, 2, perm, s);
    if (t.done(rc1 ? rc1 : launch_transpose8_rows(op->X8c, T, D, c->Xt, 2, perm, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_DW2, s);
    if (t.done(launch_sp_rowmajor_f8_rowwise(c->Hc_t, c->meta_t, c->dYt, 1, F, D, T, c->sh_f, op->sdy_d, dW2, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_DW1, s);
    if (t.done(launch_sp_colmajor_f8_rowwise(c->dZc_t, c->meta_t, c->Xt, F, D, T, c->sdz_f, op->sx_d, dW1, s))) return FFN24_ERR_HIP; }
  return FFN24_OK;
}

int ffn24_bwd(ffn24_ctx* c, const void* dY, void* dX, void* dW1, void* dW2, void* stream) {
  if (!c) return FFN24_ERR_NULL;
  if (!(c->flags & FFN24_TRAINING) || !c->have_fwd24) return FFN24_ERR_STATE;
  if (c->flags & FFN24_ROWWISE) return FFN24_ERR_STATE;   // a row-wise context takes ffn24_bwd_rowwise
  int rc = check_device(c);
  if (rc) return rc;
  rc = check_ptrs({dY, dX, dW1, dW2});
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int T = (int)c->T, D = (int)c->D, F = (int)c->F;
  if (c->f8) {
    // fp8 backward (per-tensor scales): every GEMM operand is e4m3, the gradients come out in bf16
    { Timed t(c, K_TR_ACT, s);   // dY^T for the dW2 GEMM first: the same pass leaves dY8 in panel form for the dH GEMM
      int rc1 = launch_transpose8(dY, T, D, c->dYt, 2, c->dYp8, 1, s);
      if (t.done(rc1 ? rc1 : launch_transpose8(c->X, T, D, c->Xt, 2, nullptr, 0, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DH, s);
      if (t.done(launch_dh_gather_f8(c->W2p, c->dYp8, c->Hc16, c->meta16, T, D, F, c->sdy * c->sw2, c->sdz, c->dZc, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DX, s);
      if (t.done(launch_sp_rowmajor_f8(c->dZc, c->meta, 1, c->W1p, 1, T, D, F, c->sdz * c->sw1, dX, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_FW, s);
      if (t.done(launch_featurewise24_f8(c->Hc, c->meta, c->dZc, T, F, c->Hc_t, c->meta_t, c->dZc_t, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DW2, s);
      if (t.done(launch_sp_rowmajor_f8(c->Hc_t, c->meta_t, 1, c->dYt, 1, F, D, T, c->sh * c->sdy, dW2, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DW1, s);
      if (t.done(launch_sp_colmajor_f8(c->dZc_t, c->meta_t, 1, c->Xt, 1, F, D, T, c->sdz * c->sx, dW1, s))) return FFN24_ERR_HIP; }
    return FFN24_OK;
  }
  const int* perm = c->perm_on ? c->perm : nullptr;   // position p inside the FFN holds token perm[p]
  // the forward's two counts stay; the feature-wise one belongs to this backward
  if (c->tele && launch_zero32(reinterpret_cast<uint32_t*>(c->tele + tele_index(TELE_KEPT_FEAT, 0)), 2 * TELE_SLOTS * TELE_STRIDE, s)) return FFN24_ERR_HIP;
  { Timed t(c, K_DH, s);  if (t.done(launch_dh_gather(c->W2p, dY, c->Hc, c->meta, T, D, F, c->dZc, perm, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_DX, s);
    int rc1 = perm ? launch_sp_rowmajor_mapped(c->dZc, c->meta, 1, c->W1p, 1, T, D, F, dX, perm, s) : launch_sp_rowmajor(c->dZc, c->meta, 1, c->W1p, 1, T, D, F, dX, s);
    if (t.done(rc1)) return FFN24_ERR_HIP; }
  const bool split = (c->flags & FFN24_SPLIT) && c->n_dense > 0;
  if (split) {
    // Sec. 2, "Optimization 1": the n_dense least sparse features are kept out of the feature-wise 2:4; their rows
    // of both weight gradients come from dense GEMMs, all others from the sparse ones
    const int nd = c->n_dense, ns = F - nd;
    { Timed t(c, K_PART, s); if (t.done(launch_split_partition(c->nnz, F, nd, T, c->row_of_feat, c->feat_of_row, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_FW, s);
      if (t.done(launch_featurewise24_split(c->Hc, c->meta, c->dZc, T, F, c->row_of_feat, ns, c->Hc_t, c->meta_t, c->dZc_t, c->Hdn_t, c->dZdn_t, c->tele, nullptr, nullptr, s)))
        return FFN24_ERR_HIP; }
    if (c->tele && (rc = tele_snapshot(c, 1, s))) return rc;
    { Timed t(c, K_TR_ACT, s);
      int rc1 = launch_transpose(dY, T, D, c->dYt, 2, nullptr, 0, perm, s);
      if (t.done(rc1 ? rc1 : launch_transpose(c->X, T, D, c->Xt, 2, nullptr, 0, perm, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DW2, s); if (t.done(launch_split_wgrad(c->Hc_t, c->meta_t, ns, c->Hdn_t, nd, c->dYt, D, T, dW2, D, c->feat_of_row, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_DW1, s); if (t.done(launch_split_wgrad(c->dZc_t, c->meta_t, ns, c->dZdn_t, nd, c->Xt, D, T, c->dW1t, D, c->feat_of_row, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_TR_DW1, s); if (t.done(launch_transpose(c->dW1t, F, D, dW1, 0, nullptr, 0, nullptr, s))) return FFN24_ERR_HIP; }
    return FFN24_OK;
  }
  { Timed t(c, K_FW, s);  if (t.done(launch_featurewise24(c->Hc, c->meta, c->dZc, T, F, c->Hc_t, c->meta_t, c->dZc_t, 1, c->tele, s))) return FFN24_ERR_HIP; }
  if (c->tele && (rc = tele_snapshot(c, 1, s))) return rc;
  { Timed t(c, K_TR_ACT, s);
    int rc1 = launch_transpose(dY, T, D, c->dYt, 2, nullptr, 0, perm, s);
    if (t.done(rc1 ? rc1 : launch_transpose(c->X, T, D, c->Xt, 2, nullptr, 0, perm, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_DW2, s); if (t.done(launch_sp_rowmajor(c->Hc_t, c->meta_t, 1, c->dYt, 1, F, D, T, dW2, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_DW1, s); if (t.done(launch_sp_colmajor(c->dZc_t, c->meta_t, 1, c->Xt, 1, F, D, T, dW1, s))) return FFN24_ERR_HIP; }
  return FFN24_OK;
}

int ffn_fwd(ffn24_ctx* c, const void* X, const void* W1, const float* b1, const void* W2, void* Y, void* stream) {
  if (!c) return FFN24_ERR_NULL;
  if (!(c->flags & FFN24_DENSE)) return FFN24_ERR_STATE;
  int rc = check_device(c);
  if (rc) return rc;
  rc = check_ptrs({X, Y});
  if (rc) return rc;
  if (b1 && misaligned(b1)) return FFN24_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int T = (int)c->T, D = (int)c->D, F = (int)c->F;
  c->have_fwd24 = c->have_fwd_dense = 0;
  if (c->f8 && (c->flags & FFN24_ROWWISE) && !c->rsx) return FFN24_ERR_STATE;
  if ((rc = resolve_weights(c, W1, W2, s))) return rc;
  if (c->f8 && (c->flags & FFN24_ROWWISE)) {
    // dense baseline with row-wise scales: up-projection (bf16 activations + row maxima), row-wise quantisation, dense GEMM
    if (launch_zero32(c->rowmax, (size_t)T, s)) return FFN24_ERR_HIP;
    { Timed t(c, K_PANEL_X, s); if (t.done(launch_panelise8(X, T, D, c->Xp8, 1, s))) return FFN24_ERR_HIP; }
    { Timed t(c, KD_UP, s);
      if (t.done(launch_up_relu2_f8_rowwise(c->W1t, c->Xp8, b1, T, D, F, c->rsx, c->rsw1, c->Hd16, c->rowmax, c->Hdt16, s))) return FFN24_ERR_HIP; }
    { Timed t(c, K_QUANT, s);
      if (t.done(launch_quantise_rows_dense(c->Hd16, c->rowmax, T, F, c->Hd, c->rsh, s))) return FFN24_ERR_HIP; }
    { Timed t(c, KD_DOWN, s);
      if (t.done(launch_dense_rowmajor_f8_rowwise(c->Hd, c->W2t, 1, T, D, F, c->rsh, c->rsw2, Y, s))) return FFN24_ERR_HIP; }
    if (c->flags & FFN24_TRAINING) { c->X = X; c->have_fwd_dense = 1; }
    return FFN24_OK;
  }
  if (c->f8) {
    const bool train = (c->flags & FFN24_TRAINING) != 0;
    { Timed t(c, K_PANEL_X, s); if (t.done(launch_panelise8(X, T, D, c->Xp8, 1, s))) return FFN24_ERR_HIP; }
    { Timed t(c, KD_UP, s);
      if (t.done(launch_up_relu2_f8(c->W1t, c->Xp8, b1, T, D, F, c->sx * c->sw1, c->sh, c->Hd, train ? c->Hd16 : nullptr, train ? c->Hd_t : nullptr, s)))
        return FFN24_ERR_HIP; }
    { Timed t(c, KD_DOWN, s);
      if (t.done(launch_dense_rowmajor_f8(c->Hd, 1, c->W2t, 1, T, D, F, c->sh * c->sw2, Y, s))) return FFN24_ERR_HIP; }
    if (train) { c->X = X; c->have_fwd_dense = 1; }
    return FFN24_OK;
  }
  if (c->tele && launch_zero32(reinterpret_cast<uint32_t*>(c->tele), 2 * TELE_WORDS, s)) return FFN24_ERR_HIP;
  { Timed t(c, KD_UP, s);   if (t.done(launch_up_relu2(c->W1t, X, b1, T, D, F, c->Hd, c->Hd_t, c->tele, s))) return FFN24_ERR_HIP; }
  { Timed t(c, KD_DOWN, s); if (t.done(launch_dense_rowmajor(c->Hd, 1, c->W2t, 1, T, D, F, Y, s))) return FFN24_ERR_HIP; }
  if (c->tele && (rc = tele_snapshot(c, 0, s))) return rc;
  c->X = X; c->have_fwd_dense = 1;
  return FFN24_OK;
}

int ffn_bwd_rowwise(ffn24_ctx* c, const ffn24_rowwise_bwd_operands* op, void* dX, void* dW1, void* dW2, void* stream) {
  if (!c || !op) return FFN24_ERR_NULL;
  if (!c->f8 || !(c->flags & FFN24_ROWWISE) || !(c->flags & FFN24_TRAINING) || !(c->flags & FFN24_DENSE) || !c->have_fwd_dense) return FFN24_ERR_STATE;
  int rc = check_device(c);
  if (rc) return rc;
  rc = check_ptrs({op->dY8r, op->sdy_t, op->dY8c, op->sdy_d, op->X8c, op->sx_d, op->W2_8r, op->sw2_f, op->W1_8c, op->sw1_d, dX, dW1, dW2});
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int T = (int)c->T, D = (int)c->D, F = (int)c->F;
  { Timed t(c, K_PANEL_W, s);
    int rc1 = launch_panelise8(op->W2_8r, F, D, c->W2rp, 0, s);
    if (!rc1) rc1 = launch_panelise8(op->W1_8c, D, F, c->W1cp, 1, s);      // (the dense dX GEMM does lose with its B operand row-major: 1.28 -> 1.43 ms)
    if (t.done(rc1 ? rc1 : launch_panelise8(op->dY8r, T, D, c->dYp8, 1, s))) return FFN24_ERR_HIP; }
  if (launch_zero32(c->rowmax_dz, (size_t)T, s) || launch_zero32(c->hmax, (size_t)F, s) || launch_zero32(c->zmax, (size_t)F, s)) return FFN24_ERR_HIP;
  { Timed t(c, KD_DH, s);
    if (t.done(launch_dh_drelu_f8_rowwise(c->W2rp, c->dYp8, c->Hd16, T, D, F, op->sw2_f, op->sdy_t, c->dZd16, c->dZdt16, c->rowmax_dz, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_QUANT_DZ, s);
    if (t.done(launch_quantise_rows_dense(c->dZd16, c->rowmax_dz, T, F, c->dZd, c->sdz_t, s))) return FFN24_ERR_HIP; }
  { Timed t(c, KD_DX, s);
    if (t.done(launch_dense_rowmajor_f8_rowwise(c->dZd, c->W1cp, 1, T, D, F, c->sdz_t, op->sw1_d, dX, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_QUANT_T, s);      // per-feature maxima of the two transposed bf16 operands, then their quantisation
    int rc1 = launch_rowmax_dense(c->Hdt16, F, T, c->hmax, s);
    if (!rc1) rc1 = launch_rowmax_dense(c->dZdt16, F, T, c->zmax, s);
    if (!rc1) rc1 = launch_quantise_rows_dense(c->Hdt16, c->hmax, F, T, c->Hd_t, c->sh_f, s);
    if (t.done(rc1 ? rc1 : launch_quantise_rows_dense(c->dZdt16, c->zmax, F, T, c->dZd_t, c->sdz_f, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_TR_ACT, s);
    int rc1 = launch_transpose8(op->dY8c, T, D, c->dYt, 2, nullptr, 0, s);
    if (t.done(rc1 ? rc1 : launch_transpose8(op->X8c, T, D, c->Xt, 2, nullptr, 0, s))) return FFN24_ERR_HIP; }
  { Timed t(c, KD_DW2, s);
    if (t.done(launch_dense_rowmajor_f8_rowwise(c->Hd_t, c->dYt, 1, F, D, T, c->sh_f, op->sdy_d, dW2, s))) return FFN24_ERR_HIP; }
  { Timed t(c, KD_DW1, s);
    if (t.done(launch_dense_colmajor_f8_rowwise(c->dZd_t, c->Xt, F, D, T, c->sdz_f, op->sx_d, dW1, s))) return FFN24_ERR_HIP; }
  return FFN24_OK;
}

int ffn_bwd(ffn24_ctx* c, const void* dY, void* dX, void* dW1, void* dW2, void* stream) {
  if (!c) return FFN24_ERR_NULL;
  if (!(c->flags & FFN24_DENSE) || !(c->flags & FFN24_TRAINING) || !c->have_fwd_dense) return FFN24_ERR_STATE;
  if (c->flags & FFN24_ROWWISE) return FFN24_ERR_STATE;   // a row-wise context takes ffn_bwd_rowwise
  int rc = check_device(c);
  if (rc) return rc;
  rc = check_ptrs({dY, dX, dW1, dW2});
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int T = (int)c->T, D = (int)c->D, F = (int)c->F;
  if (c->f8) {
    { Timed t(c, K_TR_ACT, s);
      int rc1 = launch_transpose8(dY, T, D, c->dYt, 2, c->dYp8, 1, s);
      if (t.done(rc1 ? rc1 : launch_transpose8(c->X, T, D, c->Xt, 2, nullptr, 0, s))) return FFN24_ERR_HIP; }
    { Timed t(c, KD_DH, s);
      if (t.done(launch_dh_drelu_f8(c->W2p, c->dYp8, c->Hd16, T, D, F, c->sdy * c->sw2, c->sdz, c->dZd, c->dZd_t, s))) return FFN24_ERR_HIP; }
    { Timed t(c, KD_DX, s);
      if (t.done(launch_dense_rowmajor_f8(c->dZd, 1, c->W1p, 1, T, D, F, c->sdz * c->sw1, dX, s))) return FFN24_ERR_HIP; }
    { Timed t(c, KD_DW2, s);
      if (t.done(launch_dense_rowmajor_f8(c->Hd_t, 1, c->dYt, 1, F, D, T, c->sh * c->sdy, dW2, s))) return FFN24_ERR_HIP; }
    { Timed t(c, KD_DW1, s);
      if (t.done(launch_dense_colmajor_f8(c->dZd_t, 1, c->Xt, 1, F, D, T, c->sdz * c->sx, dW1, s))) return FFN24_ERR_HIP; }
    return FFN24_OK;
  }
  { Timed t(c, KD_DH, s);  if (t.done(launch_dh_drelu(c->W2p, dY, c->Hd, T, D, F, c->dZd, c->dZd_t, s))) return FFN24_ERR_HIP; }
  { Timed t(c, KD_DX, s);  if (t.done(launch_dense_rowmajor(c->dZd, 1, c->W1p, 1, T, D, F, dX, s))) return FFN24_ERR_HIP; }
  { Timed t(c, K_TR_ACT, s);
    int rc1 = launch_transpose(dY, T, D, c->dYt, 2, nullptr, 0, nullptr, s);
    if (t.done(rc1 ? rc1 : launch_transpose(c->X, T, D, c->Xt, 2, nullptr, 0, nullptr, s))) return FFN24_ERR_HIP; }
  { Timed t(c, KD_DW2, s); if (t.done(launch_dense_rowmajor(c->Hd_t, 1, c->dYt, 1, F, D, T, dW2, s))) return FFN24_ERR_HIP; }
  { Timed t(c, KD_DW1, s); if (t.done(launch_dense_colmajor(c->dZd_t, 1, c->Xt, 1, F, D, T, dW1, s))) return FFN24_ERR_HIP; }
  return FFN24_OK;
}

}  // extern "C"
