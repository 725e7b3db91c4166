// k_product for rows on the grid {-s, 0, +s} (one binary16 scale per row).
#include "qmoe_product.h"

namespace qmoe {

qmoe_status launch_product_sym(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s)
{
    return launch_product_for<0>(a, p, run, s);
}

}  // namespace qmoe
