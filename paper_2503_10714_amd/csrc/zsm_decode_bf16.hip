// Decode-step instantiations for bf16 token slots.
#include "zsm_decode.hpp"

namespace zsm {
hipError_t launch_decode_bf16(const DecodeArgs& a, hipStream_t stream) { return launch_decode_t<bf16_t>(a, stream); }
size_t decode_lds_bf16(int D, int G, int nz) { return decode_lds_t<bf16_t>(D, G, nz); }
hipError_t launch_decode_pooled_bf16(const DecodeArgs& a, hipStream_t stream) { return launch_decode_pooled_t<bf16_t>(a, stream); }
int decode_pool_share_heads_bf16(int D, int nz) { return decode_pool_share_heads_t<bf16_t>(D, nz); }
}  // namespace zsm
