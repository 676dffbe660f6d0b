// Entry points shared by the translation units of the library, not part of the public ABI.
#pragma once

#include "../../include/orthdion.h"

#ifdef __cplusplus
extern "C" {
#endif

// orthdion_step with a switch: with allow_second_stream = 0 every kernel is enqueued on `stream`
// itself and no stream or event is ever created (orthdion_step_static promises to allocate
// nothing, host-side runtime objects included).
int orthdion_step_impl(orthdion_handle h, void* const* X, const void* const* G, float* const* M, float* const* Q,
                       void* workspace, size_t workspace_bytes, void* stream, int allow_second_stream);

#ifdef __cplusplus
}
#endif
