// Weights as instruction literals (paper, Section 3.4: the code of a network is written for that network, not
// assembled from general layers; here it is also completed for one weight set).
//
// On this chip a vector multiply-add whose weight sits in a scalar register issues at half the rate of one whose
// weight is a 32-bit literal in the instruction.  Kernels with wave-uniform weights are therefore compiled a second
// time, into a code object of their own, with every weight replaced by a distinct placeholder constant; the build
// records where each placeholder ended up in the code.  At run time the host copies the code object, writes a weight
// set over the placeholders and loads the result as a module.  Contexts with equal weights on one device share it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cnnc {

// Placeholder of weight i: a float in [0.5, 0.75) with scattered mantissa bits, so that it is never one of the
// inline constants of the instruction set (those carry no literal), never equal to another placeholder, and has no
// regularity a compiler could turn into arithmetic on the index.
constexpr uint32_t literal_placeholder_bits(int i) { return 0x3F000001u + (((uint32_t)(i + 1) * 2654435761u) >> 10); }
constexpr int kMaxLiteralWeights = 4096;
constexpr bool literal_placeholders_distinct(int n)
{
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < i; ++j)
            if (literal_placeholder_bits(i) == literal_placeholder_bits(j)) return false;
    return true;
}

// What a kernel body indexes instead of a weight pointer.
struct LiteralWeights {
    __device__ constexpr float operator[](int i) const { return __builtin_bit_cast(float, literal_placeholder_bits(i)); }
};

// The same for weights BASE, BASE + 1, ... of the literal array (a layer inside a larger set of literals).
template <int BASE>
struct LiteralWeightsAt {
    __device__ constexpr float operator[](int i) const { return __builtin_bit_cast(float, literal_placeholder_bits(BASE + i)); }
};

#ifndef CNNC_LITERAL_DEVICE_ONLY
// A code object with placeholders, as the build embeds it: the image, and (byte offset, weight index) of every literal.
struct LiteralImage {
    const unsigned char *image;
    size_t size;
    const uint32_t (*patch)[2];
    size_t n_patch;
    int n_weights;
};

struct LiteralModule;
// The module of `img` completed with `weights` (img.n_weights floats) on the current device; nullptr when the image
// is empty or the module does not load (the caller then keeps to its kernels with weights in memory).
LiteralModule *literal_acquire(const LiteralImage &img, const float *weights);
void literal_release(LiteralModule *m);
hipFunction_t literal_function(LiteralModule *m, const char *name);
#endif

}  // namespace cnnc
