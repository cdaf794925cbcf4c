// The measurement operator as the kernels and their launchers see it (plain data, no device code).
#pragma once
#include <stdint.h>

namespace csk {

struct OpDesc {
    uint32_t k0, k1;      // seed halves
    uint32_t stream;
    int ens;              // 0 Gaussian, 1 Rademacher, 2 subsampled randomised Hadamard
    int m, n;
    float scale;          // 1/sqrt(m)
    int nbits;            // Hadamard ensemble: the transform has 2^nbits >= max(n, 2) points
};

}  // namespace csk
