// The vocabulary reduction of Eq. 1 as a call of its own: logits already on the device ->
// per row (argmax token, confidence, entropy, max logit).  Same kernels as the denoising step
// uses for a materialised logits matrix.
#include <cstdio>
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

}  // extern "C"
