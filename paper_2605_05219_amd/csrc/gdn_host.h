// Host-side helpers shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace gdn {

// Copies `bytes` from `src` into a pinned staging buffer the library owns and enqueues its upload
// to the device address `dst` on `stream`.  The buffers form a ring of eight: waits (on the host)
// until the upload eight calls back has left the buffer.  Returns GDN_OK or a GDN_ERR_HIP code.
int32_t upload_plan(const void* src, size_t bytes, void* dst, hipStream_t stream);

}  // namespace gdn
