// Matrix-core compress path (bf16) -- placeholder until the kernels land.
#include "kvc_internal.h"
namespace kvc {
bool fast_compress_supported(const kvc_shape &) { return false; }
size_t fast_compress_ws_bytes(const kvc_shape &) { return 0; }
kvc_status fast_compress(const CompressCall &) { return KVC_ERR_UNSUPPORTED; }
}  // namespace kvc
