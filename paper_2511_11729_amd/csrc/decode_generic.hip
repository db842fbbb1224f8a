// fp32-storage decode path (placeholder until the generic kernels land).
#include "ctx.h"
namespace harli {
harli_status decode_step_f32(harli_ctx*, const harli_decode_batch*, hipStream_t) {
  return fail(HARLI_ERR_STATE, "decode_step: fp32 storage is not implemented yet");
}
}  // namespace harli
