// Internal helpers shared by the host-side translation units of libharli.
#pragma once
#include <cstdarg>
#include <cstddef>
#include <cstdint>

#include "harli.h"

namespace harli {

// Records a thread-local message retrievable through harli_last_error() and returns `s`.
harli_status fail(harli_status s, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Returns 1 when the event has completed, 0 when it is still pending, -1 on error.
// Provided by the HIP side of the library (or a stub in host-only test builds).
int event_done(void* hip_event);
void event_destroy(void* hip_event);

// Geometry of the KV grid, handed to the decode kernels by value.
struct KvGeom {
  unsigned long long small_pool_bytes, chunk_bytes, block_bytes, page_bytes, row_bytes;
  int pages_per_block, page_tokens, n_layers, n_pages_total;
};

}  // namespace harli

// Accessors the compute side uses without seeing the pool's internals.
extern "C" {
void* harli_pool_slab(const harli_pool* p);
size_t harli_pool_slab_bytes(const harli_pool* p);
void harli_pool_geom(const harli_pool* p, harli::KvGeom* g);
}
