// Measurement aid (vocabtrim_measure.h): a plain streaming read of a buffer, for the benchmark.  Not part of the
// method's path.
#include "vocabtrim.h"
#include "vocabtrim_measure.h"

#include <hip/hip_runtime.h>

#include "vt_step.h"

extern "C" int vt_stream_read_reference(const void *p, size_t bytes, uint32_t *sink, void *stream) {
    if (p == nullptr || sink == nullptr) return VT_ERR_NULL;
    if (bytes == 0 || (bytes & 15) != 0) return VT_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(p) & 15) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3) != 0) return VT_ERR_ALIGN;
    (void)hipGetLastError();
    vt::launch_stream_read(p, bytes, sink, static_cast<hipStream_t>(stream));
    return hipGetLastError() == hipSuccess ? VT_OK : VT_ERR_DEVICE;
}
