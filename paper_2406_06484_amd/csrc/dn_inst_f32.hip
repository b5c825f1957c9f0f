// fp32 instantiations (fp32 MFMA, v_mfma_f32_32x32x2_f32)
#include "dn_launch.hpp"
namespace dn {
DN_INSTANTIATE(float, 64, 64)
DN_INSTANTIATE(float, 32, 64)
DN_INSTANTIATE(float, 64, 32)
} // namespace dn
