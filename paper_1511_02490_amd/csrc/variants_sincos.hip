// Variants: the sin/cos stencil under the local-memory tile, and the marching kernels (sin/cos, 5x5 weighted sum).
#include "variants.h"

void register_sincos(std::vector<Variant> &r) {
    reg_blockings<sk::OpSinCos, STENCIL_SINCOS, sk::HaloD, 4>(r);
    reg_blockings<sk::OpSinCos, STENCIL_SINCOS, sk::HaloC<1, 5, 3, 0>, 4>(r);
    reg_march<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<2, 2, 2, 2>>(r);
    reg_march<sk::OpSinCos, STENCIL_SINCOS, sk::HaloC<1, 5, 3, 0>>(r);
}
