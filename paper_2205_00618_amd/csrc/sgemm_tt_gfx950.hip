// The sgemm kernels for both operands stored transposed: see sgemm_variants.hpp.
#include "sgemm_variants.hpp"

namespace lsmi {
LSMI_DEFINE_SGEMM_TABLE(sgemm_table_tt, true, true, "_tt")
}  // namespace lsmi
