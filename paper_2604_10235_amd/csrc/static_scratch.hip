// codecomp_compress_static: the fused score -> select -> gather call for callers that can neither allocate
// device memory nor bring a workspace (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc).  The kernels are those of codecomp_compress; what that call takes through its workspace
// argument (row statistics of the segments, row normalisers, raw attention mass, the two-stage membership
// mask) lives here in one file-scope device array per GPU.
#include <atomic>

#include "plan.h"

namespace codecomp {

static_assert(CODECOMP_STATIC_SCRATCH_BYTES % 256 == 0, "scratch size");
// Zero-initialised device memory that every GPU the library runs on holds until the process ends.
static __device__ __align__(256) unsigned char scratch[CODECOMP_STATIC_SCRATCH_BYTES];

// `scratch` above is, in host code, only a handle for the runtime; the array's address on a GPU comes from
// hipGetSymbolAddress with that GPU current, and every GPU has its own copy at its own address.
constexpr int kScratchDevices = 64;
static std::atomic<void*> scratch_ptr[kScratchDevices];   // null = not asked yet

static int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipError_t e = hipGetDevice(&dev)) return (int)e;
  if (dev < 0 || dev >= kScratchDevices) return CODECOMP_EINVAL_SHAPE;
  void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) return (int)e;
    if (!ptr || ((uintptr_t)ptr & 255) != 0) return CODECOMP_EINVAL_WORKSPACE;
    scratch_ptr[dev].store(ptr, std::memory_order_release);     // two threads asking at once store the same address
  }
  *out = ptr;
  return CODECOMP_OK;
}

}  // namespace codecomp

using namespace codecomp;

extern "C" int codecomp_compress_static(const void* q_obs, const void* k, const void* v, const float* prior,
                                        const codecomp_params* params, float* scores, int32_t* idx, void* k_out,
                                        void* v_out, void* hip_stream) {
  if (!q_obs || !k || !v || !prior || !params || !scores || !idx || !k_out || !v_out) return CODECOMP_EINVAL_NULL;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  const uintptr_t ptrs[] = {(uintptr_t)q_obs, (uintptr_t)k, (uintptr_t)v, (uintptr_t)k_out, (uintptr_t)v_out};
  for (uintptr_t p : ptrs)
    if (p & 15) return CODECOMP_EINVAL_SHAPE;
  if (pl.ws_bytes > (size_t)CODECOMP_STATIC_SCRATCH_BYTES) return CODECOMP_EINVAL_WORKSPACE;   // too large for the array
  void* ws = nullptr;
  if (int rc = scratch_of_current_device(&ws)) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  if (int rc = launch_score(pl, q_obs, k, prior, scores, ws, s)) return rc;
  if (pl.select_mode == CODECOMP_SELECT_TWO_STAGE) {
    if (int rc = launch_select_two_stage(pl, scores, prior, idx, ws, s)) return rc;
  } else {
    if (int rc = launch_select(pl, scores, idx, ws, s)) return rc;
  }
  return launch_gather(pl, k, v, idx, k_out, v_out, s);
}
