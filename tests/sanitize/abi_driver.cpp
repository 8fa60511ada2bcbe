// Calls the host side of libfsd's C ABI that needs no GPU (planning, and every argument error, which
// is found before anything is launched) in a build whose host code carries AddressSanitizer and
// UndefinedBehaviorSanitizer.  Built and run by tests/test_sanitizers.py from csrc/fsd_kernels.hip.
#include <cmath>
#include <cstdint>
#include <cstdio>

#include "fsd.h"

int main() {
    int bad = 0;
    auto expect = [&](int got, int want, const char* what) {
        if (got != want) { std::printf("%s: status %d, expected %d\n", what, got, want); ++bad; }
    };
    void* fake = reinterpret_cast<void*>(0x1000);   // never dereferenced: every call below fails validation first
    const int32_t* itok = static_cast<const int32_t*>(fake);
    int32_t* iout = static_cast<int32_t*>(fake);
    const size_t big = size_t(1) << 40;
    for (int B : {1, 3, 64, 65535})
        for (int rows : {1, 8, 60, 2048})
            for (int V : {1, 7, 32000, 128256, 256000, 524288})
                for (int dt : {FSD_F32, FSD_BF16}) {
                    if (static_cast<long>(B) * rows >= (1L << 24)) continue;
                    if (fsd_workspace_bytes(B, rows, V, dt) == 0) { std::printf("no plan for %d %d %d %d\n", B, rows, V, dt); ++bad; }
                }
    if (fsd_workspace_bytes(0, 1, 1, FSD_F32) != 0 || fsd_workspace_bytes(1, 1, 524289, FSD_BF16) != 0 ||
        fsd_workspace_bytes(1, 1, 1, 9) != 0 || fsd_workspace_bytes(65535, 2048, 8, FSD_F32) != 0) ++bad;
    if (fsd_calibrate_workspace_bytes(4, 8) == 0 || fsd_calibrate_workspace_bytes(0, 8) != 0) ++bad;
    for (int s = 1; s >= -9; --s) (void)fsd_status_string(s);
    expect(fsd_verify_chain(nullptr, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_NULL, "chain null");
    expect(fsd_verify_chain(fake, fake, itok, 0, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_SHAPE, "chain B");
    expect(fsd_verify_chain(fake, fake, itok, 2, 4, 100, 7, FSD_DIV_JS, 0.1f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_DTYPE, "chain dtype");
    expect(fsd_verify_chain(fake, fake, itok, 2, 4, 100, FSD_F32, 5, 0.1f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_DIV, "chain div");
    expect(fsd_verify_chain(fake, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, NAN, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_SHAPE, "chain T");
    expect(fsd_verify_chain(fake, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, 3, 0, 0, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_MODE, "chain mode");
    expect(fsd_verify_chain(fake, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, fake, 16, nullptr), FSD_ERR_WORKSPACE, "chain workspace");
    expect(fsd_verify_chain(fake, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, reinterpret_cast<void*>(0x1010), big, nullptr), FSD_ERR_WORKSPACE, "chain alignment");
    expect(fsd_verify_chain_static(fake, fake, itok, 256, 16, 151936, FSD_F32, FSD_DIV_JS, 0.3f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, nullptr), FSD_ERR_TOO_LARGE, "static too large");
    expect(fsd_verify_chain_static(nullptr, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, 0.3f, FSD_SAMPLE, 0, 0, iout, iout, nullptr, nullptr, nullptr), FSD_ERR_NULL, "static null");
    expect(fsd_verify_tree(fake, fake, itok, nullptr, 1, 4, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, 0, 0, 0, iout, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_NULL, "tree parent");
    expect(fsd_verify_tree(fake, fake, itok, itok, 1, 4, 0, 100, FSD_F32, FSD_DIV_JS, 0.1f, 0, 0, 0, iout, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_SHAPE, "tree depth");
    expect(sd_verify_chain(fake, fake, itok, 2, 4, 100, FSD_BF16, 2, 0, 0, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_MODE, "sd mode");
    expect(sd_verify_tree(fake, fake, itok, itok, 1, 4, 4, 100, FSD_BF16, 0, 0, 0, iout, nullptr, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_NULL, "sd tree path");
    expect(rfsd_verify_chain(fake, fake, itok, 2, 4, 100, FSD_BF16, -1, 0.1f, 0, 0, 0, iout, iout, nullptr, nullptr, nullptr, fake, big, nullptr), FSD_ERR_DIV, "rfsd div");
    expect(fsd_verify_chain_warped(fake, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, 0, 0, 0, 0.0f, 0, 1.0f, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_SHAPE, "warped temperature");
    expect(fsd_verify_chain_warped(fake, fake, itok, 2, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, 0, 0, 0, 1.0f, -1, 1.0f, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_SHAPE, "warped top_k");
    expect(fsd_verify_tree_warped(fake, fake, itok, itok, 1, 4, 4, 100, FSD_F32, FSD_DIV_JS, 0.1f, 0, 0, 0, 1.0f, 0, 0.0f, iout, iout, iout, nullptr, nullptr, fake, big, nullptr), FSD_ERR_SHAPE, "tree warped top_p");
    expect(fsd_calibrate_threshold(nullptr, 2, 4, 0.5f, static_cast<float*>(fake), nullptr, fake, big, nullptr), FSD_ERR_NULL, "calibrate null");
    expect(fsd_calibrate_threshold(static_cast<const float*>(fake), 2, 4, 0.0f, static_cast<float*>(fake), nullptr, fake, big, nullptr), FSD_ERR_SHAPE, "calibrate fraction");
    expect(fsd_calibrate_threshold(static_cast<const float*>(fake), 2, 4, 0.5f, static_cast<float*>(fake), nullptr, fake, 8, nullptr), FSD_ERR_WORKSPACE, "calibrate workspace");
    expect(fsd_debug_set_shape(3, 4), FSD_ERR_SHAPE, "shape hook");
    expect(fsd_debug_set_shape(0, 0), FSD_OK, "shape hook reset");
    std::printf("abi sanitizer driver: %d unexpected results\n", bad);
    return bad ? 1 : 0;
}
