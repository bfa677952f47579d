// Matrix-core decode path (bf16, head_dim 128) -- placeholder until the kernels land.
#include "kvc_internal.h"
namespace kvc {
bool fast_decode_supported(const kvc_shape &) { return false; }
size_t fast_decode_ws_bytes(const kvc_shape &, int32_t) { return 0; }
kvc_status fast_decode(const DecodeCall &) { return KVC_ERR_UNSUPPORTED; }
}  // namespace kvc
