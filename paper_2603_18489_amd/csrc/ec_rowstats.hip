// The vocabulary reduction of Eq. 1 as a call of its own: logits already on the device ->
// per row (argmax token, confidence, entropy, max logit).  Same kernels as the denoising step
// uses for a materialised logits matrix.
#include <cstdio>
#include <mutex>
#include <string>

#include "ec_internal.h"

using namespace ec;

namespace {

constexpr int kRowsMax = EC_MAX_BLOCK;   // rows of one call
constexpr int kVocabMax = 163840;        // as ec_init

int rs_fail(int code, const std::string& msg) {
  set_global_error(msg.c_str());
  return code;
}

int check_args(const float* logits, int rows, int vocab, size_t ld, float* stats) {
  if (!logits || !stats) return rs_fail(EC_ERR_ARG, "logits and stats must not be NULL");
  if (rows < 0 || rows > kRowsMax) return rs_fail(EC_ERR_ARG, "rows must be in [0, EC_MAX_BLOCK]");
  if (vocab < 2 || vocab > kVocabMax) return rs_fail(EC_ERR_ARG, "vocab must be in [2, 163840]");
  if (ld < (size_t)vocab) return rs_fail(EC_ERR_ARG, "row stride smaller than vocab");
  if (((uintptr_t)stats) % 16) return rs_fail(EC_ERR_ARG, "stats must be 16-byte aligned");
  return EC_OK;
}

int run(const float* logits, int rows, int vocab, size_t ld, float* stats, float4* partials,
        hipStream_t s) {
  if (rows == 0) return EC_OK;
  launch_vocab_reduce(logits, rows, vocab, ld, partials, s);
  launch_row_stats(partials, vocab_reduce_parts(vocab), rows, (float4*)stats, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return rs_fail(EC_ERR_HIP, std::string("row statistics kernels: ") + hipGetErrorString(e));
  return EC_OK;
}

// ---- scratch of the call that allocates nothing --------------------------------------------
// Room for the partial tuples of the largest call: EC_MAX_BLOCK rows x 80 parts (vocabularies up
// to 163840) x 16 bytes = 160 KiB.  Every GPU the library runs on holds its own copy of the array
// at its own address until the process ends.  `scratch` is only the host-side handle of the
// symbol: the device address comes from hipGetSymbolAddress, once per device.
constexpr int kScratchParts = 80;
constexpr size_t kScratchTuples = (size_t)kRowsMax * kScratchParts;
static __device__ __align__(256) float4 scratch[kScratchTuples];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float4* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on the first call there)
int scratch_of_current_device(float4** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return rs_fail(EC_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return rs_fail(EC_ERR_HIP, "device index out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return rs_fail(EC_ERR_HIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = (float4*)p;
  }
  *out = g_scratch_ptr[dev];
  return EC_OK;
}

}  // namespace

extern "C" {

size_t ec_row_entropy_workspace_bytes(int32_t rows, int32_t vocab) {
  if (rows < 0 || rows > kRowsMax || vocab < 2 || vocab > kVocabMax) return 0;
  const size_t n = (size_t)(rows > 0 ? rows : 1) * vocab_reduce_parts(vocab) * sizeof(float4);
  return (n + 255) / 256 * 256;
}

int ec_row_entropy(const float* logits, int32_t rows, int32_t vocab, size_t ld, float* stats,
                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_args(logits, rows, vocab, ld, stats);
  if (rc != EC_OK) return rc;
  if (!workspace || ((uintptr_t)workspace) % 256)
    return rs_fail(EC_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  if (workspace_bytes < ec_row_entropy_workspace_bytes(rows, vocab))
    return rs_fail(EC_ERR_WORKSPACE, "workspace smaller than ec_row_entropy_workspace_bytes()");
  return run(logits, rows, vocab, ld, stats, (float4*)workspace, (hipStream_t)hip_stream);
}

int ec_row_entropy_noalloc(const float* logits, int32_t rows, int32_t vocab, size_t ld,
                           float* stats, void* hip_stream) {
  int rc = check_args(logits, rows, vocab, ld, stats);
  if (rc != EC_OK) return rc;
  if ((size_t)rows * vocab_reduce_parts(vocab) > kScratchTuples)
    return rs_fail(EC_ERR_ARG, "rows x vocabulary parts exceed the library's static scratch");
  float4* part = nullptr;
  rc = scratch_of_current_device(&part);
  if (rc != EC_OK) return rc;
  return run(logits, rows, vocab, ld, stats, part, (hipStream_t)hip_stream);
}

}  // extern "C"
