/* Test helper: binary16 -> binary32 through the x86 F16C hardware converter
 * (VCVTPH2PS).  An implementation of the IEEE widening that is independent of
 * the oracle's arithmetic; used only to pin the oracle. */
#include <immintrin.h>
#include <stdint.h>
#include <string.h>

void f16c_widen(const uint16_t *h, uint32_t *out, int64_t n)
{
    for (int64_t k = 0; k < n; ++k) {
        __m128i v = _mm_cvtsi32_si128((int)h[k]);
        __m128 f = _mm_cvtph_ps(v);
        float x = _mm_cvtss_f32(f);
        memcpy(&out[k], &x, 4);
    }
}
