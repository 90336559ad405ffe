// Variants: weighted sums under the local-memory tile (fp32 with run-time and compile-time regions, fp64, int32,
// bytes in / floats out).
#include "variants.h"

void register_weighted_sum_tiles(std::vector<Variant> &r) {
    reg_blockings<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloD, 4>(r);
    reg_blockings<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_blockings<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<2, 2, 2, 2>, 4>(r);
    // the template's other element types (Section 3.3): 16-byte vectors are two doubles or four ints
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloD, 1, 1>(r);
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloD, 1, 2>(r);
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloD, 2, 2>(r);
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloD, 4, 2>(r);
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloC<1, 1, 1, 1>, 2, 2>(r);
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloC<1, 1, 1, 1>, 4, 2>(r);
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloC<2, 2, 2, 2>, 2, 2>(r);
    reg_borders<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloC<2, 2, 2, 2>, 4, 2>(r);
    reg_direct<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloC<1, 1, 1, 1>, 2>(r);
    reg_direct<sk::OpWeightedSumF64, STENCIL_WEIGHTED_SUM_F64, sk::HaloC<2, 2, 2, 2>, 2>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloD, 1, 1>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloD, 1, 4>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloD, 2, 4>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloD, 4, 4>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloC<1, 1, 1, 1>, 2, 4>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloC<1, 1, 1, 1>, 4, 4>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloC<2, 2, 2, 2>, 2, 4>(r);
    reg_borders<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloC<2, 2, 2, 2>, 4, 4>(r);
    reg_direct<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloC<1, 1, 1, 1>, 4>(r);
    reg_direct<sk::OpWeightedSumI32, STENCIL_WEIGHTED_SUM_I32, sk::HaloC<2, 2, 2, 2>, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloD, 1, 1>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloD, 4, 1>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloD, 1, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloD, 2, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloD, 4, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloC<1, 1, 1, 1>, 2, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloC<1, 1, 1, 1>, 4, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloC<2, 2, 2, 2>, 2, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloC<2, 2, 2, 2>, 4, 4>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloD, 1, 16>(r);
    reg_borders<sk::OpWeightedSumU8, STENCIL_WEIGHTED_SUM_U8, sk::HaloD, 2, 16>(r);
}
