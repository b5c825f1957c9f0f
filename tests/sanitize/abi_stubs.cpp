// Stand-ins for the kernel launch sequences, so that the C ABI's host layer (argument validation, workspace plan,
// dispatch) can be built for the host alone and run under AddressSanitizer / UndefinedBehaviorSanitizer without a GPU
// (tests/test_sanitizers_host.py).  Every stand-in records that it was reached and touches no pointer.
#include "../../paper_2406_06484_amd/csrc/dn_host.hpp"

int g_stub_calls = 0;

namespace dn {
template <typename T, int DK, int DV> int run_fwd(const Problem &, const Ptrs &) { ++g_stub_calls; return 0; }
template <typename T, int DK, int DV> int run_bwd(const Problem &, const Ptrs &) { ++g_stub_calls; return 0; }
template <typename T, int DK, int DV> size_t max_lds_bytes() { return 1024; }
int run_recurrent_fwd(int, int, const RecArgs &, hipStream_t) { ++g_stub_calls; return 0; }

typedef __bf16 bf16_t;
#define STUB(E, T, DK, DV)                                              \
    template int run_fwd<T, DK, DV>(const Problem &, const Ptrs &);   \
    template int run_bwd<T, DK, DV>(const Problem &, const Ptrs &);   \
    template size_t max_lds_bytes<T, DK, DV>();
DN_FOR_EACH_IMPL(STUB)
} // namespace dn
