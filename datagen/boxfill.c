/* Seeded payload of an axis-aligned box of one logical tensor, row-major in global axis order.
 * Pure input generation: coordinates -> global linear index -> pattern word.  No layout or
 * routing arithmetic.  Used to synthesize the buffers that non-resident peers would send. */
#include <stdint.h>

#include "pattern.h"

void vps_pattern_fill_box(uint64_t seed, uint32_t kind, uint32_t tensor, const int32_t* shape,
                          const int32_t* lo, const int32_t* ext, void* out)
{
    const int64_t rows = (int64_t)ext[0] * ext[1] * ext[2];
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t c2 = lo[2] + (int32_t)(r % ext[2]);
        const int32_t c1 = lo[1] + (int32_t)((r / ext[2]) % ext[1]);
        const int32_t c0 = lo[0] + (int32_t)(r / ((int64_t)ext[2] * ext[1]));
        const uint64_t base = (((uint64_t)c0 * (uint64_t)shape[1] + (uint64_t)c1) * (uint64_t)shape[2] +
                               (uint64_t)c2) * (uint64_t)shape[3] + (uint64_t)lo[3];
        for (int32_t k = 0; k < ext[3]; ++k) {
            const uint32_t w = vps_pattern_word(seed, kind, tensor, base + (uint64_t)k);
            const uint64_t o = (uint64_t)r * (uint64_t)ext[3] + (uint64_t)k;
            if (kind == 0) ((uint16_t*)out)[o] = (uint16_t)w; else ((uint32_t*)out)[o] = w;
        }
    }
}
