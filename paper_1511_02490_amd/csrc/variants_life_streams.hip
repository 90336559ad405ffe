// Variants: Game of Life in registers.
#include "variants.h"

void register_life_streams(std::vector<Variant> &r) {
    reg_life_stream<1>(r);
    reg_life_stream<2>(r);
    reg_life_stream<4>(r);
}
