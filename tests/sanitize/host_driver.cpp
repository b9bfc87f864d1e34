// Host-side sanitizer driver for the library's argument checks and planner
// (tests/test_sanitizers_cpu.py links this file against a build of the library whose host code
// is instrumented with -fsanitize=address,undefined and runs it without a GPU).  Every call
// here returns before the first HIP call: the planner, the workspace query, and the rejection
// paths of the entry points, driven with extreme shapes.  Pointers are fake and never
// dereferenced by the library on these paths.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/la.h"
#include "../../paper_2405_17381_amd/csrc/la_debug.h"

static int fails = 0;
#define EXPECT(cond) do { if (!(cond)) { std::fprintf(stderr, "host driver: %s failed (line %d)\n", #cond, __LINE__); ++fails; } } while (0)

int main()
{
    void *P = (void *)(uintptr_t)4096;
    std::vector<float> lam(LA_MAX_HEADS, 0.5f);
    const int Bs[] = {1, 2, 31, 300, 65535};
    const int Hs[] = {1, 7, 16, 256};
    const int ns[] = {1, 31, 32, 63, 64, 65, 2048, 65536, 1000003, LA_MAX_SEQ_LEN};
    for (int B : Bs) for (int H : Hs) for (int n : ns) for (int d : {64, 128}) for (int dt : {0, 1}) {
        int tile = 0, L = 0, S = 0;
        const int rc = la_plan(B, H, n, d, (la_dtype)dt, &tile, &L, &S);
        if (rc != LA_OK) continue;                               // B * H beyond the grid limit
        EXPECT(tile > 0 && L > 0 && S > 0 && L % tile == 0);
        EXPECT((long long)(S - 1) * L < n && (long long)S * L >= n);
        const size_t f = la_workspace_bytes(B, H, n, d, (la_dtype)dt, 0), b = la_workspace_bytes(B, H, n, d, (la_dtype)dt, 1);
        EXPECT(b == 2 * f);
        EXPECT(f == (S > 1 ? (size_t)B * H * S * d * d * 4 : 0));
    }
    for (long lseg : {1L, 64L, 100L, 1L << 40}) {
        EXPECT(la_debug_set("lseg", lseg) == LA_OK);
        int tile = 0, L = 0, S = 0;
        EXPECT(la_plan(1, 2, 100000, 128, LA_BF16, &tile, &L, &S) == LA_OK && L % 64 == 0 && S >= 1);
    }
    EXPECT(la_debug_set("lseg", 0) == LA_OK);
    EXPECT(la_debug_set("nonsense", 1) == LA_ERR_NULL && la_debug_get("nonsense") == -1);
    // rejections (all before any HIP call)
    EXPECT(la_fwd(P, P, P, lam.data(), P, 1, 1, LA_MAX_SEQ_LEN, 64, LA_BF16, nullptr, 0, nullptr) == LA_ERR_WORKSPACE);
    EXPECT(la_fwd(P, P, P, lam.data(), P, 1, 1, 8, 96, LA_BF16, nullptr, 0, nullptr) == LA_ERR_SHAPE);
    EXPECT(la_fwd(P, P, P, lam.data(), P, 1, 257, 8, 64, LA_BF16, nullptr, 0, nullptr) == LA_ERR_SHAPE);
    EXPECT(la_fwd(P, P, P, lam.data(), P, 1, 1, -5, 64, LA_BF16, nullptr, 0, nullptr) == LA_ERR_SHAPE);
    EXPECT(la_fwd(nullptr, P, P, lam.data(), P, 1, 1, 8, 64, LA_BF16, nullptr, 0, nullptr) == LA_ERR_NULL);
    EXPECT(la_bwd(P, P, P, lam.data(), P, P, P, (char *)P + 2, 1, 1, 8, 64, LA_F32, nullptr, 0, nullptr) == LA_ERR_ALIGN);
    lam[3] = 1.5f;
    EXPECT(la_fwd(P, P, P, lam.data(), P, 1, 8, 8, 64, LA_BF16, nullptr, 0, nullptr) == LA_ERR_LAMBDA);
    lam[3] = 0.5f;
    EXPECT(la_fwd_static(P, P, P, lam.data(), P, 1, 1, 8, 32, LA_BF16, nullptr) == LA_ERR_SHAPE);
    EXPECT(la_decode_step(P, P, P, lam.data(), nullptr, P, 1, 1, 64, LA_BF16, nullptr) == LA_ERR_NULL);
    la_layout bad = {8, 8, 32}, good = {1 << 20, 1 << 10, 128};
    EXPECT(la_fwd_strided(P, P, P, lam.data(), P, &bad, &good, 1, 2, 8, 64, LA_BF16, nullptr, 0, nullptr) == LA_ERR_SHAPE);
    EXPECT(la_lrpe_workspace_bytes(2, 3, 300, 64) == (size_t)2 * 3 * 3 * 64 * 4);
    for (int st = 1; st >= -9; --st) EXPECT(la_strerror(st) != nullptr);
    if (fails) return 1;
    std::printf("host sanitizer driver: ok\n");
    return 0;
}
