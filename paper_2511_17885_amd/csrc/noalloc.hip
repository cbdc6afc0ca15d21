// fmoe_permute_noalloc: the permutation by expert for callers that cannot allocate or bring a
// workspace (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// Same kernels as fmoe_permute; their scratch (in-block ranks per routed slot, per-block expert
// counts) lives in a file-scope device array instead of a caller-provided workspace.
//
// The array's name is only a host-side handle: the device address comes from hipGetSymbolAddress,
// looked up once per GPU with that GPU current (every GPU that loads the library holds its own copy
// of the array at its own address) and kept in g_scratch_ptr; host code passes that pointer, never
// the array's name, to the kernels.

#include <mutex>

#include "common.h"

namespace {

constexpr int NA_MAX_TOKENS = 65536;              // kept positions per call
constexpr int NA_MAX_ROWS = 1 << 20;              // kept positions x Kmax per call
constexpr size_t NA_RANK_BYTES = (size_t)NA_MAX_ROWS * 4;
constexpr size_t NA_BLK_BYTES = (size_t)(NA_MAX_TOKENS / FMOE_PERM_BLOCK) * FMOE_MAX_EXPERTS * 4;
constexpr int NA_MAX_DEVICES = 64;

static __device__ __align__(256) unsigned char scratch[NA_RANK_BYTES + NA_BLK_BYTES];   // 4.25 MiB per GPU

std::mutex g_mu;
void* g_scratch_ptr[NA_MAX_DEVICES] = {};

// Device address of `scratch` on GPU `device` (looked up on the first call for that GPU).
int scratch_on_device(int device, void** out) {
  if (device < 0 || device >= NA_MAX_DEVICES)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED, "fmoe_permute_noalloc: device %d outside 0..%d", device, NA_MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_scratch_ptr[device] == nullptr) {
    int current = -1;
    FMOE_HIP_CHECK(hipGetDevice(&current));
    if (current != device) FMOE_HIP_CHECK(hipSetDevice(device));
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (current != device) (void)hipSetDevice(current);
    if (e != hipSuccess || p == nullptr)
      return fmoe_fail(FMOE_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d failed: %s", device, hipGetErrorString(e));
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return FMOE_OK;
}

}  // namespace

extern "C" int fmoe_permute_noalloc(fmoe_ctx* ctx, const int32_t* topk_idx, const int32_t* kept_idx, int32_t n_kept,
                                    const int32_t* n_kept_dev, int32_t* expert_offsets, int32_t* perm_src,
                                    int32_t* inv_perm, void* stream) {
  if (!ctx) return fmoe_fail(FMOE_ERR_NULL_PTR, "ctx is NULL");
  if (n_kept < 0) return fmoe_fail(FMOE_ERR_INVALID_ARG, "fmoe_permute_noalloc: n_kept %d is negative", n_kept);
  if (n_kept > NA_MAX_TOKENS || (long long)n_kept * ctx->kmax > NA_MAX_ROWS)
    return fmoe_fail(FMOE_ERR_UNSUPPORTED,
                     "fmoe_permute_noalloc: %d kept positions x Kmax %d exceed the static scratch (at most %d positions "
                     "and %d routed slots per call); use fmoe_permute with a workspace",
                     n_kept, ctx->kmax, NA_MAX_TOKENS, NA_MAX_ROWS);
  if (!expert_offsets) return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_permute_noalloc: expert_offsets is NULL");
  if (n_kept > 0 && ctx->kmax > 0 && (!topk_idx || !perm_src || !inv_perm))
    return fmoe_fail(FMOE_ERR_NULL_PTR, "fmoe_permute_noalloc: topk_idx / perm_src / inv_perm is NULL");
  void* base = nullptr;
  const int rc = scratch_on_device(ctx->device, &base);
  if (rc != FMOE_OK) return rc;
  // the two arrays the permutation kernels use; every entry they read in a call is written earlier in
  // the same call, so nothing has to be cleared between calls
  fmoe_ws_layout L{};
  L.slot_rank = 0;
  L.blk_count = NA_RANK_BYTES;
  L.total = NA_RANK_BYTES + NA_BLK_BYTES;
  return launch_permute(ctx, topk_idx, kept_idx, n_kept, n_kept_dev, expert_offsets, perm_src, inv_perm, base, L,
                        false, static_cast<hipStream_t>(stream));
}
