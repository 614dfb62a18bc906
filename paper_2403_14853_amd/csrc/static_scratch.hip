// isp_spmm_static_scratch: SpMM for callers that cannot allocate.
//
// isp_spmm keeps the partial sums of the hub-row segments in the workspace the caller handed to
// isp_csr_build.  This variant runs the same kernels with those partial rows in a fixed array in the
// library's own device image instead: no buffer besides X and Y is taken from the caller or from an
// allocator, and the call itself makes no HIP allocation (nor does isp_spmm; the difference is where the
// scratch lives).  The array exists once per GPU, for every handle and every call.
#include <mutex>
#include "isp_internal.h"

// Partial-sum rows (ISP_PARTIAL_TILE floats each) one call may use: 32,768 rows = 32 MiB per device, held
// from the first use of the library on that device until the process ends.
#define ISP_STATIC_SCRATCH_ROWS 32768
// (No attribute such as `used` here: the compiler gives this internal-linkage array a global symbol in the
// device image because host code takes its address below, and that symbol is what the runtime looks up; with
// `used` the symbol stays local and the lookup aborts the process.)
static __device__ __align__(256) float scratch[(size_t)ISP_STATIC_SCRATCH_ROWS * ISP_PARTIAL_TILE];

namespace {
constexpr int MAX_DEV = 64;
// Device address of `scratch` on each device (every GPU holds its own copy of the array at its own
// address); the array's name is only a host-side stand-in and is never passed to a kernel.
float* g_scratch_ptr[MAX_DEV] = {};
std::mutex g_scratch_mu;

// Looked up once per device, with that device current.
isp_status scratch_address(int device, float** out) {
  if (device < 0 || device >= MAX_DEV) return isp_fail(ISP_EUNSUPPORTED, "device ordinal %d is beyond %d", device, MAX_DEV - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    ISP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return isp_fail(ISP_EHIP, "hipGetSymbolAddress returned a null address for the static scratch");
    g_scratch_ptr[device] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[device];
  return ISP_OK;
}
}  // namespace

extern "C" isp_status isp_spmm_static_scratch(const isp_csr_t* A, const float* X, int64_t ldx, int32_t d, float* Y,
                                              int64_t ldy, void* stream) {
  if (!A) return isp_fail(ISP_EINVAL, "handle is NULL");
  isp_status st;
  if ((st = isp_check_device(A)) != ISP_OK) return st;  // (the handle's device is the current one from here on)
  if ((st = isp_check_dense(X, ldx, d, A->v.nnz > 0 ? A->v.n_cols : 0, "X")) != ISP_OK) return st;
  if ((st = isp_check_dense(Y, ldy, d, A->v.n_rows, "Y")) != ISP_OK) return st;
  // partial rows a launch may touch: one per hub-row segment, or one per piece where the handle has the
  // packed SpMM layout (large matrices with many columns)
  const int n_partial = A->has_packed && A->info.spmm_pieces > A->v.n_seg ? A->info.spmm_pieces : A->v.n_seg;
  if (n_partial > ISP_STATIC_SCRATCH_ROWS)
    return isp_fail(ISP_EUNSUPPORTED, "the handle needs %d partial rows (hub-row segments / row pieces); the static "
                    "scratch holds %d (use isp_spmm, whose scratch is the build workspace)", n_partial,
                    ISP_STATIC_SCRATCH_ROWS);
  float* ptr = nullptr;
  if ((st = scratch_address(A->device, &ptr)) != ISP_OK) return st;
  // The same handle with its partial rows redirected.  Every partial row a launch reads was written by that
  // launch's segments before (segment kernel, then fix-up, in stream order), so nothing has to start at zero
  // and whatever an earlier call left in the array is never read.
  isp_csr view = *A;
  view.v.partials = ptr;
  view.vp.partials = ptr;
  return isp_spmm_launch(&view, X, ldx, d, Y, ldy, (hipStream_t)stream);
}
