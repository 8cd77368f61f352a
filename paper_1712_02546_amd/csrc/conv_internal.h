// Calls shared between the translation units of libconvslice.so; not part of the C ABI.
#pragma once
#include <stddef.h>

#include "../../include/convslice.h"

namespace cs_internal {

// conv_fwd / conv_bwd_weight for the layer driver.  With input_ready != 0 the call skips the re-layout of the
// shared input x: the workspace must be the one a call on another slice of the same layer, pass and dtype has
// just used on the same stream (the input's work copy sits at the same place for every slice).
int conv_fwd_shared(const conv_desc_t* desc, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
                    void* hip_stream, int input_ready);
int conv_bwd_weight_shared(const conv_desc_t* desc, const void* x, const void* dy, void* dw, void* ws, size_t ws_bytes,
                           void* hip_stream, int input_ready);

}  // namespace cs_internal
