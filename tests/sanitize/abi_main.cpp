// Calls the C ABI's host layer (built for the host alone, kernel launches replaced by stand-ins) under
// AddressSanitizer / UndefinedBehaviorSanitizer: every status code of the validation path, the workspace plans of
// dense, packed, segmented, gated and fused shapes, and the host copy of cu_seqlens read to its last entry from an
// exactly-sized allocation.  Device pointers are fakes that nothing dereferences.  Without a GPU the calls that pass
// validation end at the device query (DN_ERR_LAUNCH); with one they reach the stand-ins.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/deltanet.h"

extern int g_stub_calls;

#define EXPECT(cond)                                                          \
    do {                                                                      \
        if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

static dn_shape shape(int B, int L, int H, int dk, int dv, dn_dtype dt) {
    dn_shape s;
    memset(&s, 0, sizeof(s));
    s.B = B; s.L = L; s.H = H; s.d_k = dk; s.d_v = dv; s.chunk = 64; s.dtype = dt;
    return s;
}

int main() {
    void *fake = (void *)0x1000, *odd = (void *)0x1004;
    size_t bytes = 0;
    dn_shape s = shape(2, 256, 4, 128, 128, DN_BF16);
    EXPECT(deltanet_workspace_bytes(&s, 1, &bytes) == DN_OK && bytes > 0);
    EXPECT(deltanet_workspace_bytes(nullptr, 1, &bytes) == DN_ERR_NULL);
    EXPECT(deltanet_workspace_bytes(&s, 1, nullptr) == DN_ERR_NULL);
    dn_shape bad = s; bad.H = 0;
    EXPECT(deltanet_workspace_bytes(&bad, 1, &bytes) == DN_ERR_SHAPE);
    bad = s; bad.d_k = 96;
    EXPECT(deltanet_workspace_bytes(&bad, 1, &bytes) == DN_ERR_UNSUPPORTED);
    bad = s; bad.L = 1 << 30; bad.B = 64;
    EXPECT(deltanet_workspace_bytes(&bad, 1, &bytes) == DN_ERR_SHAPE);
    // few long chains: the segmented plan
    dn_shape lng = shape(1, 32768, 16, 128, 128, DN_BF16);
    EXPECT(deltanet_workspace_bytes(&lng, 1, &bytes) == DN_OK && bytes > 0);
    EXPECT(deltanet_gated_workspace_bytes(&s, 1, &bytes) == DN_OK);
    EXPECT(deltanet_fused_workspace_bytes(&s, 1, &bytes) == DN_OK);
    // packed: the host copy is read up to entry num_seqs, from an allocation of exactly that size
    for (int n : {0, 1, 7, 1000}) {
        int32_t *cu = (int32_t *)malloc(sizeof(int32_t) * (n + 1));
        for (int i = 0; i <= n; ++i) cu[i] = (int32_t)((long long)512 * i / (n ? n : 1));
        cu[n] = n ? 512 : 0;
        dn_shape p = shape(1, n ? 512 : 0, 2, 64, 64, DN_F32);
        p.cu_seqlens = (const int32_t *)fake; p.cu_seqlens_host = cu; p.num_seqs = n;
        EXPECT(deltanet_workspace_bytes(&p, 1, &bytes) == DN_OK);
        if (n >= 7) {
            cu[3] = cu[2] - 1;
            EXPECT(deltanet_workspace_bytes(&p, 1, &bytes) == DN_ERR_CUSEQLENS);
        }
        free(cu);
    }
    // argument checks of the passes, before any device call
    EXPECT(deltanet_fwd(&s, nullptr, fake, fake, fake, nullptr, fake, nullptr, fake, (size_t)1 << 40, nullptr) == DN_ERR_NULL);
    EXPECT(deltanet_fwd(&s, odd, fake, fake, fake, nullptr, fake, nullptr, fake, (size_t)1 << 40, nullptr) == DN_ERR_ALIGN);
    EXPECT(deltanet_fwd(&s, fake, fake, fake, fake, nullptr, fake, nullptr, fake, 16, nullptr) == DN_ERR_WORKSPACE);
    EXPECT(deltanet_bwd(&s, fake, fake, fake, fake, nullptr, fake, nullptr, fake, fake, fake, nullptr, nullptr, fake, (size_t)1 << 40,
                        nullptr) == DN_ERR_NULL);
    EXPECT(deltanet_bwd(&s, fake, fake, fake, fake, nullptr, fake, nullptr, fake, fake, fake, (float *)fake, nullptr, fake, 16,
                        nullptr) == DN_ERR_WORKSPACE);
    // a call that passes validation: ends at the device query without a GPU, at the stand-in with one
    const int rc = deltanet_fwd(&s, fake, fake, fake, fake, nullptr, fake, nullptr, fake, (size_t)1 << 40, nullptr);
    EXPECT(rc == DN_OK || rc == DN_ERR_LAUNCH);
    EXPECT((rc == DN_OK) == (g_stub_calls == 1));
    const int rb = deltanet_bwd(&s, fake, fake, fake, fake, nullptr, fake, nullptr, fake, fake, fake, (float *)fake, nullptr, fake,
                                (size_t)1 << 40, nullptr);
    EXPECT(rb == rc);
    const int rr = deltanet_recurrent_fwd(&s, fake, fake, fake, fake, nullptr, fake, nullptr, nullptr);
    EXPECT(rr == DN_OK); // (the token-serial pass asks the device nothing before its launch)
    for (int code = 0; code >= -8; --code) EXPECT(deltanet_status_string(code) != nullptr && deltanet_status_string(code)[0]);
    printf("C ABI host layer under sanitizers: ok (device reached: %s)\n", rc == DN_OK ? "yes" : "no");
    return 0;
}
