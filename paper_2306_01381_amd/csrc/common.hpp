// Internal helpers shared by the translation units of libadaqp (host side only, plus a few wave intrinsics).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaqp.h"

namespace adaqp {

// Records the text of a failed HIP call for adaqp_last_hip_error() and maps it to ADAQP_EHIP.
int note_hip_error(hipError_t err, const char *what);

#define ADAQP_HIP_TRY(expr)                                              \
    do {                                                                 \
        hipError_t adaqp_err__ = (expr);                                 \
        if (adaqp_err__ != hipSuccess) return ::adaqp::note_hip_error(adaqp_err__, #expr); \
    } while (0)

inline bool valid_bits(int b) { return b == 2 || b == 4 || b == 8; }

inline bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kBlock = 256;          // threads per workgroup used by every kernel here (4 waves)
constexpr int kWavesPerBlock = kBlock / kWave;

}  // namespace adaqp
