// Decode-step instantiations for f32 token slots.
#include "zsm_decode.hpp"

namespace zsm {
hipError_t launch_decode_f32(const DecodeArgs& a, hipStream_t stream) { return launch_decode_t<float>(a, stream); }
size_t decode_lds_f32(int D, int G, int nz) { return decode_lds_t<float>(D, G, nz); }
hipError_t launch_decode_pooled_f32(const DecodeArgs& a, hipStream_t stream) { return launch_decode_pooled_t<float>(a, stream); }
int decode_pool_share_heads_f32(int D, int nz) { return decode_pool_share_heads_t<float>(D, nz); }
}  // namespace zsm
