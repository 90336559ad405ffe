// Variants: weighted sums with the wider symmetric border regions (Table 2's gaussian goes up to 10) as compile-time
// regions: 7x7 and 9x9 under every mapping, 11x11 marched.
#include "variants.h"

void register_wide_regions(std::vector<Variant> &r) {
    reg_borders<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<3, 3, 3, 3>, 1, 1>(r);
    reg_borders<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<3, 3, 3, 3>, 2, 4>(r);
    reg_borders<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<3, 3, 3, 3>, 4, 4>(r);
    reg_borders<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<4, 4, 4, 4>, 1, 1>(r);
    reg_borders<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<4, 4, 4, 4>, 2, 4>(r);
    reg_borders<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<4, 4, 4, 4>, 4, 4>(r);
    reg_direct<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<3, 3, 3, 3>, 4>(r);
    reg_direct<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<4, 4, 4, 4>, 4>(r);
    reg_march<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<3, 3, 3, 3>>(r);
    reg_march<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<4, 4, 4, 4>>(r);
    reg_march<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloC<5, 5, 5, 5>>(r);
}
