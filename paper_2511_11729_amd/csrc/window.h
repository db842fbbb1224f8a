// Window-based residency of the finetune task's frozen weights (Harli Sec. 4.3): the library's finetune-private
// copies live in pinned host memory, a few device slots taken from the unified pool hold the copies about to be
// used, and a copy stream refills a slot as soon as the layer that used it has been enqueued.
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

struct harli_ctx;

namespace harli {
// Called by the finetune entry points around the work of one layer.  acquire makes `st` wait for the layer's copy
// (forward: W, backward: W^T), loading it on demand when absent, and points the layer's weight table at the slot;
// release records the end of use on `st` and starts the refill of the slot.  Both are no-ops without a window.
harli_status window_acquire(harli_ctx* c, int layer, bool backward, hipStream_t st);
harli_status window_release(harli_ctx* c, int layer, bool backward, hipStream_t st);
void free_window_state(harli_ctx* c);
void detach_layers(harli_ctx* c);  // clears every layer's finetune weight table (they point into slots under a window)
}  // namespace harli
