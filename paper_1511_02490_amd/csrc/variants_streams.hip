// Variants: the register-streaming temporal kernels (heat, 3x3 weighted sum).
#include "variants.h"

void register_streams(std::vector<Variant> &r) {
    reg_stream<sk::OpHeat, STENCIL_HEAT>(r);
    reg_stream<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM>(r);
}
