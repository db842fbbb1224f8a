// LoRA finetune unit (placeholder until the MFMA kernels land).
#include "ctx.h"
using namespace harli;
namespace harli {
void free_finetune_state(harli_ctx*) {}
}
extern "C" harli_status harli_lora_attach(harli_ctx*, const harli_lora_cfg*, void* const*, void* const*) {
  return fail(HARLI_ERR_STATE, "lora_attach: not implemented yet");
}
extern "C" harli_status harli_lora_fwd(harli_ctx*, int32_t, const float*, float*, int32_t, int32_t, harli_saved**, void*) {
  return fail(HARLI_ERR_STATE, "lora_fwd: not implemented yet");
}
extern "C" harli_status harli_lora_bwd(harli_ctx*, int32_t, const float*, float*, harli_saved*, float* const*, float* const*, void*) {
  return fail(HARLI_ERR_STATE, "lora_bwd: not implemented yet");
}
extern "C" harli_status harli_saved_release(harli_ctx*, harli_saved*, void*) {
  return fail(HARLI_ERR_STATE, "saved_release: not implemented yet");
}
extern "C" harli_status harli_saved_bytes(const harli_ctx*, int32_t, int32_t, size_t*) {
  return fail(HARLI_ERR_STATE, "saved_bytes: not implemented yet");
}
