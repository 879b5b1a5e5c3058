// Activation of hidden layers, shared by the kernels that can produce one: ReLU, then (training with
// p > 0) the dropout keep mask times 1 / (1 - p).  sigma of Section 4.1's layer rule is taken as ReLU.
// The mask is a pure integer function of (key, element index), so any implementation of the same
// mixer reproduces it bit for bit:  keep(e) = [ (mix64(key + e * 0x9E3779B97F4A7C15) >> 32) >= threshold ].
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace gcn {

enum ActKind { kActNone = 0, kActRelu = 1 };

struct Activation {
    int kind;                 // kActNone / kActRelu
    int width;                // true row width d_l: element index = row * width + column
    uint32_t drop_threshold;  // 0 = keep everything
    float keep_scale;
    uint64_t drop_key;
};

__device__ inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ inline float activate(float v, const Activation &a, int64_t row, int c) {
    if (a.kind == kActRelu) {
        v = v > 0.0f ? v : 0.0f;
        if (a.drop_threshold != 0u) {
            const uint64_t e = (uint64_t)row * (uint64_t)a.width + (uint64_t)c;
            const uint64_t h = mix64(a.drop_key + e * 0x9E3779B97F4A7C15ull);
            v = ((uint32_t)(h >> 32) >= a.drop_threshold) ? v * a.keep_scale : 0.0f;
        }
    }
    return v;
}

}  // namespace gcn
