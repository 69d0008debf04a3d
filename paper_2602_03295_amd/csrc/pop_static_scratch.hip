// pop_op_gemm_splitk_static: the split-K projection for callers that cannot allocate device memory (code
// under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  It is pop_op_gemm_splitk
// with the scratch for the fp32 partial products taken from a fixed array in this library's device image
// instead of from the caller; the kernels are the same ones and receive the array's address as the scratch
// pointer, exactly as they receive the caller's buffer in pop_op_gemm_splitk.
//
// The array exists once per GPU (every device that loads the library holds its own copy at its own
// address until the process ends).  The name `scratch` is only a host-side stand-in for it: host code
// never passes it to a kernel or a runtime call.  The device address is looked up once per device with
// hipGetSymbolAddress and kept; everything below uses that pointer.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <mutex>

#include "../../include/pop_ops.h"
#include "pop_kernels.h"

namespace {

constexpr size_t kStaticScratchBytes = POP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once looked up

// Address of this device's copy of the array (the current device must be the one the stream belongs to).
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

pop_status fail(pop_status st, const char* msg) { return (pop_status)pop::record_error(st, msg); }

}  // namespace

extern "C" {

size_t pop_static_scratch_bytes(void) { return kStaticScratchBytes; }

pop_status pop_op_gemm_splitk_static(const void* A, int64_t lda, const void* W, int64_t ldw, void* out, int64_t ldc,
                                     int32_t M, int32_t N, int32_t K, int32_t epilogue, pop_stream stream) {
  if (!A || !W || !out) return fail(POP_EINVAL, "NULL pointer");
  if (M < 0 || N < 0 || K < 1) return fail(POP_EINVAL, "bad sizes");
  if (epilogue != 0 && epilogue != 1 && epilogue != 3) return fail(POP_EINVAL, "this epilogue cannot be split");
  if (K % 8 || lda % 8 || ldw % 8 || ldc % 4 || lda < K || ldw < K || ldc < N)
    return fail(POP_ESHAPE, "K, lda, ldw must be multiples of 8 (ldc of 4) and strides must cover the rows");
  if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(out)) & 15)
    return fail(POP_EALIGN, "pointer not 16-byte aligned");
  // the deepest split writes 8 parts of fp32 [M, N]
  if ((unsigned long long)M * (unsigned long long)N * 32ull > kStaticScratchBytes) {
    char msg[200];
    snprintf(msg, sizeof msg,
             "M x N = %d x %d needs %llu bytes of scratch, the built-in array has %zu (M * N <= %zu); use "
             "pop_op_gemm_splitk with a buffer of your own",
             M, N, (unsigned long long)M * N * 32ull, kStaticScratchBytes, kStaticScratchBytes / 32);
    return fail(POP_ENOSPACE, msg);
  }
  void* ptr = nullptr;
  if (hipError_t e = static_scratch(&ptr); e != hipSuccess) {
    char msg[200];
    snprintf(msg, sizeof msg, "hipGetSymbolAddress of the built-in scratch array failed: %s", hipGetErrorString(e));
    return fail(POP_EHIP, msg);
  }
  pop::GemmArgs g{};
  g.A = (const pop::bf16_t*)A; g.lda = lda; g.W = (const pop::bf16_t*)W; g.ldw = ldw; g.out = out; g.ldc = ldc;
  g.M = M; g.N = N; g.K = K; g.epilogue = epilogue; g.batch = 1;
  // Every part of a split writes its whole [M, N] partial product before the second kernel reads it, so
  // nothing in the array has to be cleared between calls; what an earlier call left behind is never read.
  g.splitk_ws = (float*)ptr; g.splitk_ws_bytes = kStaticScratchBytes;
  hipError_t e = pop::launch_gemm(g, reinterpret_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue) return fail(POP_ESHAPE, "operand too large or misaligned for the GEMM kernel");
  if (e != hipSuccess) {
    char msg[200];
    snprintf(msg, sizeof msg, "GEMM launch failed: %s", hipGetErrorString(e));
    return fail(POP_EHIP, msg);
  }
  return POP_OK;
}

}  // extern "C"
