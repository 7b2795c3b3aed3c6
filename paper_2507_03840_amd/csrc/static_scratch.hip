// egnn_radial_weights_static: the radial weights (S3) for callers that cannot allocate.
//
// egnn_radial_weights needs a caller-provided workspace for the power-of-two scalings and the half-precision pieces
// of alpha * W_r2 (egnn_radial_ws_bytes: 384 bytes per output column).  Here that buffer is a file-scope device
// array, one copy per GPU, held until the process ends.  Its device address is looked up once per device
// (egnn_static_scratch_prepare, called by egnn_create and again lazily by the entry point) and kept; every later use
// of the memory goes through that pointer.  Nothing in this file allocates or frees device memory.
//
// Every byte of the array that the kernels read for a given shape is written earlier in the same call (the scalings
// by half_scales_kernel, rows 0 .. P*channels-1 of the pieces by split_w2_half_kernel); the loader wave of
// radial_weights_kernel may copy rows past P*channels when that is not a multiple of 32, which here are stale rows of
// an earlier, larger call -- their products land in columns the kernel never stores.  Nothing has to start at zero.
// All calls on one GPU share the array: two calls that overlap in time on one GPU (two streams, two threads) race.
#include <mutex>
#include "egnn_internal.h"

// largest supported shape: 42 paths x 128 channels, 384 bytes per column
#define EGNN_STATIC_SCRATCH_BYTES (384 * 42 * 128)
#define EGNN_STATIC_MAX_DEVICES 64

static __device__ __align__(256) unsigned char scratch[EGNN_STATIC_SCRATCH_BYTES];

static std::mutex g_scratch_lock;
static void* g_scratch_ptr[EGNN_STATIC_MAX_DEVICES];   // per device: address of that GPU's copy of `scratch`

// Looks up the array's address on the current device (once per device).  Returns it, or nullptr with *err set.
static void* scratch_of_current_device(hipError_t* err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= EGNN_STATIC_MAX_DEVICES)) e = hipErrorInvalidDevice;
  if (e != hipSuccess) { *err = e; return nullptr; }
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { *err = e != hipSuccess ? e : hipErrorInvalidSymbol; return nullptr; }
    g_scratch_ptr[dev] = p;
  }
  *err = hipSuccess;
  return g_scratch_ptr[dev];
}

// Called by egnn_create so that the look-up happens at set-up, outside any stream capture.  Without a GPU (host-only
// use of the library) it does nothing; the entry point then reports the error when it is called.
void egnn_static_scratch_prepare() {
  hipError_t e;
  if (!scratch_of_current_device(&e)) (void)hipGetLastError();
}

extern "C" int egnn_radial_weights_static(egnn_ctx* ctx, int which, const float* rhat_d, int64_t n_edges,
                                          const float* W_r1, const float* W_r2, float* w, void* stream) {
  if (!ctx) return EGNN_EINVAL;
  if (which < 0 || which > 1 || n_edges < 0 || !W_r1 || !W_r2 || (n_edges > 0 && (!rhat_d || !w)))
    return egnn_fail(ctx, EGNN_EINVAL, "radial_weights_static: bad argument");
  if (egnn_radial_ws_bytes(ctx, which) > (size_t)EGNN_STATIC_SCRATCH_BYTES)
    return egnn_fail(ctx, EGNN_EWS, "radial_weights_static: paths x channels exceeds the built-in scratch (42 x 128 columns)");
  if (n_edges == 0) return EGNN_OK;   // nothing to write; rhat_d and w may be NULL
  hipError_t e;
  void* ptr = scratch_of_current_device(&e);
  if (!ptr) return egnn_check_hip(ctx, e, "radial_weights_static: address of the built-in scratch");
  return egnn_launch_radial(ctx, which, rhat_d, n_edges, W_r1, W_r2, w, ptr, (hipStream_t)stream);
}
