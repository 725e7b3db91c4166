// k_product for rows on the asymmetric grid {w_min, 0, w_max} (a bf16 pair per row).
#include "qmoe_product.h"

namespace qmoe {

qmoe_status launch_product_asym(const ProductArgs &a, const ProductPlan &p, bool run, hipStream_t s)
{
    return launch_product_for<1>(a, p, run, s);
}

}  // namespace qmoe
