// C-ABI entry points that enqueue GPU work: the GEMM call, the forced-variant call and the event-timing core of
// the tuning run.  Validation, selection and legality are host code in mdg_dispatch.cpp; the kernels live in
// mdg_direct.hip, mdg_tiled.hip, mdg_skinny.hip and mdg_indirect.hip.
#include <atomic>
#include <mutex>

#include "mdg_internal.h"

namespace mdg {

// ---- scratch memory of the allocation-free entry point --------------------------------------------------
// A file-scope device array stands in for the registered workspace (split-K partial sums).  Every GPU the
// library runs on holds its own copy at its own address until the process ends; the name below is only a
// host-side handle, the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) float scratch[MDG_STATIC_SCRATCH_BYTES / sizeof(float)];

constexpr int kMaxDevices = 64;
static std::atomic<float*> g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call on that device).
static int scratch_on_current_device(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MDG_ERR_LAUNCH;
  float* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (p == nullptr) {
      void* sym = nullptr;
      if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || sym == nullptr) {
        (void)hipGetLastError();
        return MDG_ERR_LAUNCH;
      }
      p = static_cast<float*>(sym);
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return MDG_OK;
}

static int run_variant(const VariantEntry& e, const GemmArgs& g) {
  switch (e.desc.family) {
    case MDG_FAMILY_DIRECT: return launch_direct(e.cfg, g);
    case MDG_FAMILY_TILED: return launch_tiled(e.cfg, e.desc.split_k, g);
    case MDG_FAMILY_SKINNY: return launch_skinny(e.cfg, e.desc.split_k, g);
    case MDG_FAMILY_INDIRECT: return launch_indirect(e.cfg, e.desc.tile_m, e.desc.tile_n, e.desc.tile_k, g);
  }
  return MDG_ERR_BAD_VARIANT;
}

// Degenerate problems never reach a GEMM kernel.
static inline bool handled_without_gemm(const GemmArgs& g, int* status) {
  if (g.M == 0 || g.N == 0) {
    *status = MDG_OK;
    return true;
  }
  if (g.K == 0 || g.alpha == 0.f) {
    *status = launch_scale_c(g);
    return true;
  }
  return false;
}

static int dispatch(const GemmArgs& g, SelectorKind sel) {
  int st;
  if (handled_without_gemm(g, &st)) return st;
  return run_variant(variant_table(nullptr)[choose_variant(g, sel)], g);
}

}  // namespace mdg

using namespace mdg;

extern "C" {

int mdg_sgemm(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha, const float* A,
              int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc, void* stream) {
  GemmArgs g;
  float* ws;
  size_t ws_bytes;
  registered_workspace(&ws, &ws_bytes);
  int st = canonicalise(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, ws, ws_bytes, &g);
  if (st != MDG_OK) return st;
  return dispatch(g, SEL_TREE);
}

int mdg_sgemm_variant(int variant, int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                      const float* A, int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc,
                      void* stream) {
  if (variant < 0 || variant >= variant_count()) return MDG_ERR_BAD_VARIANT;
  GemmArgs g;
  float* ws;
  size_t ws_bytes;
  registered_workspace(&ws, &ws_bytes);
  int st = canonicalise(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, ws, ws_bytes, &g);
  if (st != MDG_OK) return st;
  if (handled_without_gemm(g, &st)) return st;
  const VariantEntry& e = variant_table(nullptr)[variant];
  if (workspace_need(e, g.tA, g.tB, g.M, g.N, g.K) > g.ws_bytes) return MDG_ERR_WORKSPACE;
  if (!legal(e, g)) return MDG_ERR_ILLEGAL_VARIANT;
  return run_variant(e, g);
}

int mdg_sgemm_static_scratch(int layout, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha,
                             const float* A, int64_t lda, const float* B, int64_t ldb, float beta, float* C,
                             int64_t ldc, void* stream) {
  GemmArgs g;
  // choose as mdg_sgemm would with a workspace that is never too small ...
  int st = canonicalise(layout, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream, nullptr,
                        ~(size_t)0, &g);
  if (st != MDG_OK) return st;
  if (handled_without_gemm(g, &st)) return st;
  const VariantEntry& e = variant_table(nullptr)[choose_variant(g, SEL_TREE)];
  // ... and refuse, before anything is enqueued, what does not fit the static array
  const size_t need = workspace_need(e, g.tA, g.tB, g.M, g.N, g.K);
  if (need > (size_t)MDG_STATIC_SCRATCH_BYTES) return MDG_ERR_SCRATCH_LIMIT;
  g.ws_bytes = 0;
  if (need > 0) {
    st = scratch_on_current_device(&g.ws);
    if (st != MDG_OK) return st;
    g.ws_bytes = MDG_STATIC_SCRATCH_BYTES;
  }
  return run_variant(e, g);
}

int mdg_time_calls(int variant, int transA, int transB, int64_t M, int64_t N, int64_t K, float alpha, const float* A,
                   int64_t lda, const float* B, int64_t ldb, float beta, float* C, int64_t ldc, int n_sets,
                   int64_t a_set_stride, int64_t b_set_stride, int64_t c_set_stride, int warmup, int reps, int spans,
                   float* ms_per_call, void* stream) {
  if (variant < -2 || variant >= variant_count()) return MDG_ERR_BAD_VARIANT;
  if (!ms_per_call || n_sets < 1 || reps < 1 || spans < 1 || warmup < 0) return MDG_ERR_NULL;
  GemmArgs g0;
  float* ws;
  size_t ws_bytes;
  registered_workspace(&ws, &ws_bytes);
  int st = canonicalise(MDG_COL_MAJOR, transA ? MDG_TRANS : MDG_NO_TRANS, transB ? MDG_TRANS : MDG_NO_TRANS, M, N, K,
                        alpha, A, lda, B, ldb, beta, C, ldc, stream, ws, ws_bytes, &g0);
  if (st != MDG_OK) return st;
  const VariantEntry* e = variant >= 0 ? &variant_table(nullptr)[variant] : nullptr;
  if (e) {
    if (workspace_need(*e, g0.tA, g0.tB, g0.M, g0.N, g0.K) > g0.ws_bytes) return MDG_ERR_WORKSPACE;
    if (!legal(*e, g0)) return MDG_ERR_ILLEGAL_VARIANT;
  }
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t ev0, ev1;
  if (hipEventCreate(&ev0) != hipSuccess) return MDG_ERR_LAUNCH;
  if (hipEventCreate(&ev1) != hipSuccess) {
    (void)hipEventDestroy(ev0);
    return MDG_ERR_LAUNCH;
  }
  int set = 0;
  auto one_call = [&]() -> int {
    GemmArgs g = g0;
    g.A = A + (int64_t)set * a_set_stride;
    g.B = B + (int64_t)set * b_set_stride;
    g.C = C + (int64_t)set * c_set_stride;
    set = (set + 1 == n_sets) ? 0 : set + 1;
    int r;
    if (handled_without_gemm(g, &r)) return r;
    if (e) return run_variant(*e, g);
    return dispatch(g, variant == -1 ? SEL_TREE : SEL_DEFAULT);
  };
  st = MDG_OK;
  for (int i = 0; i < warmup && st == MDG_OK; ++i) st = one_call();
  for (int sp = 0; sp < spans && st == MDG_OK; ++sp) {
    if (hipEventRecord(ev0, s) != hipSuccess) st = MDG_ERR_LAUNCH;
    for (int i = 0; i < reps && st == MDG_OK; ++i) st = one_call();
    if (st == MDG_OK && hipEventRecord(ev1, s) != hipSuccess) st = MDG_ERR_LAUNCH;
    if (st == MDG_OK && hipEventSynchronize(ev1) != hipSuccess) st = MDG_ERR_LAUNCH;
    float ms = 0.f;
    if (st == MDG_OK && hipEventElapsedTime(&ms, ev0, ev1) != hipSuccess) st = MDG_ERR_LAUNCH;
    ms_per_call[sp] = ms / (float)reps;
  }
  (void)hipStreamSynchronize(s);
  (void)hipEventDestroy(ev0);
  (void)hipEventDestroy(ev1);
  return st;
}

}  // extern "C"
