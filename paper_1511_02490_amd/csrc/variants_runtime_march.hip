// Variants: the marching kernel for weighted sums whose border region is only given at run time (the synthetic
// template's asymmetric regions, Section 3.3): any region within N2 S2 E4 W4, and any within N5 S5 E4 W4.  A scenario
// takes the kernel with the fewest rows that holds its region.
#include "variants.h"

void register_runtime_march(std::vector<Variant> &r) {
    reg_march_masked<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloM<2, 2, 4, 4>>(r);
    reg_march_masked<sk::OpWeightedSum, STENCIL_WEIGHTED_SUM, sk::HaloM<5, 5, 4, 4>>(r);
}
