// bf16 instantiations (v_mfma_f32_32x32x16_bf16, fp32 accumulation)
#include "dn_launch.hpp"
namespace dn {
DN_INSTANTIATE(bf16, 128, 128)
DN_INSTANTIATE(bf16, 64, 64)
DN_INSTANTIATE(bf16, 64, 128)
DN_INSTANTIATE(bf16, 128, 64)
} // namespace dn
