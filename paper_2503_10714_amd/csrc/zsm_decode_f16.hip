// Decode-step instantiations for f16 token slots.
#include "zsm_decode.hpp"

namespace zsm {
hipError_t launch_decode_f16(const DecodeArgs& a, hipStream_t stream) { return launch_decode_t<f16_t>(a, stream); }
size_t decode_lds_f16(int D, int G, int nz) { return decode_lds_t<f16_t>(D, G, nz); }
hipError_t launch_decode_pooled_f16(const DecodeArgs& a, hipStream_t stream) { return launch_decode_pooled_t<f16_t>(a, stream); }
int decode_pool_share_heads_f16(int D, int nz) { return decode_pool_share_heads_t<f16_t>(D, nz); }
}  // namespace zsm
