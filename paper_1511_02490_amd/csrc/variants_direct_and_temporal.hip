// Variants: the direct kernels and the local-memory temporal kernels.
#include "variants.h"

void register_direct_and_temporal(std::vector<Variant> &r) {
    reg_direct<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_direct<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<2, 2, 2, 2>, 4>(r);
    reg_direct<sk::OpHeat, STENCIL_HEAT, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_temporal<sk::OpHeat, STENCIL_HEAT, 1>(r);
    reg_temporal<sk::OpHeat, STENCIL_HEAT, 2>(r);
    reg_temporal<sk::OpHeat, STENCIL_HEAT, 4>(r);
    reg_temporal<sk::OpHeat, STENCIL_HEAT, 8>(r);
    reg_temporal<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, 1>(r);
    reg_temporal<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, 2>(r);
    reg_temporal<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, 4>(r);
    reg_temporal<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, 8>(r);
    reg_direct<sk::OpSobel, STENCIL_SOBEL, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_direct<sk::OpNms, STENCIL_NMS, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_life_temporal<1>(r);
    reg_life_temporal<2>(r);
    reg_life_temporal<4>(r);
    reg_life_temporal<8>(r);
    reg_life_direct<1>(r);
    reg_life_direct<2>(r);
    reg_life_direct<4>(r);
    reg_life_direct<8>(r);
}
