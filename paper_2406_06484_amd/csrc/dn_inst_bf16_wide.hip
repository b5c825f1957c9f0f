// bf16 instantiation for d_k = d_v = 256: scans with 32 state columns per workgroup, the backward's chunk
// kernel in its streaming form (dn_chunk_wide.hpp); plain, gated and fused-prologue variants
#include "dn_launch.hpp"
namespace dn {
DN_INSTANTIATE(bf16, 256, 256)
} // namespace dn
