// Variants: heat, Life, sobel and nms under the local-memory tile, and the threshold kernel.
#include "variants.h"

void register_unit_region_tiles(std::vector<Variant> &r) {
    reg_blockings<sk::OpHeat, STENCIL_HEAT, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_blockings<sk::OpLife, STENCIL_LIFE, sk::HaloC<1, 1, 1, 1>, 16>(r);
    reg_blockings<sk::OpSobel, STENCIL_SOBEL, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_blockings<sk::OpNms, STENCIL_NMS, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_threshold<1, 1>(r);
    reg_threshold<2, 1>(r);
    reg_threshold<1, 4>(r);
    reg_threshold<2, 4>(r);
    reg_threshold<4, 4>(r);
}
