// Host-only self-test of the C ABI's argument validation (wht_validate.h): every status code, the
// width rules, the order in which violations are reported.  Built with a host compiler, without
// HIP, so that it can run under AddressSanitizer / UndefinedBehaviorSanitizer on the CPU.
#include <cstdio>
#include <cstdlib>

#include "wht_validate.h"

using namespace wht;

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main() {
    alignas(16) static unsigned char buf[64];
    void* ok = buf;
    void* off4 = buf + 4;
    float* fok = reinterpret_cast<float*>(buf);
    float* foff = reinterpret_cast<float*>(buf + 4);
    Width w{};

    // widths: powers of two 32 .. 16384 (float32: .. 8192), 12 * 2^m 768 .. 12288 for bfloat16 only
    for (int l = 0; l <= 20; ++l) {
        const int32_t d = 1 << l;
        const int want_bf = (d >= WHT_MIN_D && d <= WHT_MAX_D) ? WHT_OK : WHT_ERR_BAD_DIM;
        const int want_f32 = (d >= WHT_MIN_D && d <= WHT_MAX_D_F32) ? WHT_OK : WHT_ERR_BAD_DIM;
        EXPECT(check_dims(5, d, WHT_DTYPE_BF16, &w) == want_bf);
        if (want_bf == WHT_OK) EXPECT(w.logd == l && !w.twelve);
        EXPECT(check_dims(5, d, WHT_DTYPE_F32, &w) == want_f32);
    }
    for (int m = 0; m <= 14; ++m) {
        const int32_t d = 12 * (1 << m);
        const int want = (d >= WHT_MIN_D_TWELVE && d <= WHT_MAX_D_TWELVE) ? WHT_OK : WHT_ERR_BAD_DIM;
        EXPECT(check_dims(1, d, WHT_DTYPE_BF16, &w) == want);
        if (want == WHT_OK) EXPECT(w.twelve && w.logd == m + 4);
        EXPECT(check_dims(1, d, WHT_DTYPE_F32, &w) == WHT_ERR_BAD_DIM);
    }
    const int32_t odd[] = {0, -1, -4096, 3, 100, 96, 1000, 1536 + 12, 3 * 4096 + 1, 2147483647, -2147483647 - 1};
    for (int32_t d : odd) EXPECT(check_dims(1, d, WHT_DTYPE_BF16, &w) == WHT_ERR_BAD_DIM);
    EXPECT(check_dims(-1, 1024, WHT_DTYPE_BF16, &w) == WHT_ERR_BAD_DIM);
    EXPECT(check_dims(0, 1024, WHT_DTYPE_BF16, &w) == WHT_OK);
    EXPECT(check_dims(1, 1024, 2, &w) == WHT_ERR_BAD_DTYPE);
    EXPECT(check_dims(1, 1024, -1, &w) == WHT_ERR_BAD_DTYPE);
    EXPECT(check_dims(-1, 100, 7, &w) == WHT_ERR_BAD_DTYPE);            // dtype is reported first

    // forward: NULL before dimensions before alignment
    EXPECT(validate_forward(ok, fok, fok, nullptr, false, ok, nullptr, false, 4, 256, WHT_DTYPE_F32, &w) == WHT_OK);
    EXPECT(validate_forward(nullptr, fok, fok, nullptr, false, ok, nullptr, false, 4, 100, 9, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_forward(ok, nullptr, fok, nullptr, false, ok, nullptr, false, 4, 256, 0, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_forward(ok, fok, nullptr, nullptr, false, ok, nullptr, false, 4, 256, 0, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_forward(ok, fok, fok, nullptr, false, nullptr, nullptr, false, 4, 256, 0, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_forward(ok, fok, fok, nullptr, true, ok, nullptr, false, 4, 256, 0, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_forward(ok, fok, fok, ok, true, ok, nullptr, true, 4, 256, 0, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_forward(off4, fok, fok, nullptr, false, ok, nullptr, false, 4, 100, 0, &w) == WHT_ERR_BAD_DIM);
    EXPECT(validate_forward(off4, fok, fok, nullptr, false, ok, nullptr, false, 4, 256, 0, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_forward(ok, foff, fok, nullptr, false, ok, nullptr, false, 4, 256, 0, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_forward(ok, fok, foff, nullptr, false, ok, nullptr, false, 4, 256, 0, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_forward(ok, fok, fok, nullptr, false, off4, nullptr, false, 4, 256, 0, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_forward(ok, fok, fok, off4, true, ok, nullptr, false, 4, 256, 0, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_forward(ok, fok, fok, ok, true, ok, foff, true, 4, 256, 0, &w) == WHT_OK);      // sumsq: 4 bytes
    EXPECT(validate_forward(ok, fok, fok, ok, true, ok, reinterpret_cast<float*>(buf + 2), true, 4, 256, 0, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_forward(ok, fok, fok, off4, false, ok, nullptr, false, 4, 256, 0, &w) == WHT_OK);  // unused resid ignored

    // backward: which outputs may be left out
    EXPECT(validate_backward(ok, ok, fok, ok, fok, fok, 4, 1024, WHT_DTYPE_BF16, &w) == WHT_OK);
    EXPECT(validate_backward(ok, nullptr, fok, ok, nullptr, nullptr, 4, 1024, 1, &w) == WHT_OK);     // dx only: x unused
    EXPECT(validate_backward(ok, ok, fok, nullptr, fok, fok, 4, 1024, 1, &w) == WHT_OK);             // sums only
    EXPECT(validate_backward(ok, ok, fok, nullptr, nullptr, nullptr, 4, 1024, 1, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_backward(ok, ok, fok, ok, fok, nullptr, 4, 1024, 1, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_backward(ok, ok, fok, ok, nullptr, fok, 4, 1024, 1, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_backward(ok, nullptr, fok, ok, fok, fok, 4, 1024, 1, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_backward(nullptr, ok, fok, ok, fok, fok, 4, 1024, 1, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_backward(ok, ok, nullptr, ok, fok, fok, 4, 1024, 1, &w) == WHT_ERR_NULL_PTR);
    EXPECT(validate_backward(ok, ok, fok, ok, fok, fok, 4, 1024, 7, &w) == WHT_ERR_BAD_DTYPE);
    EXPECT(validate_backward(ok, ok, fok, ok, fok, fok, 4, 16384, WHT_DTYPE_F32, &w) == WHT_ERR_BAD_DIM);
    EXPECT(validate_backward(off4, ok, fok, ok, fok, fok, 4, 1024, 1, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_backward(ok, off4, fok, ok, fok, fok, 4, 1024, 1, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_backward(ok, ok, foff, ok, fok, fok, 4, 1024, 1, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_backward(ok, ok, fok, off4, fok, fok, 4, 1024, 1, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_backward(ok, ok, fok, ok, foff, fok, 4, 1024, 1, &w) == WHT_ERR_MISALIGNED);
    EXPECT(validate_backward(ok, ok, fok, ok, fok, foff, 4, 1024, 1, &w) == WHT_ERR_MISALIGNED);

    // workspace
    EXPECT(validate_workspace(ok, 64, 64) == WHT_OK);
    EXPECT(validate_workspace(ok, 63, 64) == WHT_ERR_WORKSPACE);
    EXPECT(validate_workspace(nullptr, 1 << 20, 64) == WHT_ERR_WORKSPACE);
    EXPECT(validate_workspace(off4, 64, 64) == WHT_ERR_MISALIGNED);

    // log2_exact never shifts out of range
    EXPECT(log2_exact(1) == 0 && log2_exact(1 << 30) == 30 && log2_exact(0) == -1 && log2_exact(-8) == -1);

    std::printf(failures ? "validate_selftest: %d failure(s)\n" : "validate_selftest: ok\n", failures);
    return failures ? 1 : 0;
}
