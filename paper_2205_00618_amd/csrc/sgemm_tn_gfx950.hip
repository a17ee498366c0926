// The sgemm kernels for A stored transposed (K x M): see sgemm_variants.hpp.
#include "sgemm_variants.hpp"

namespace lsmi {
LSMI_DEFINE_SGEMM_TABLE(sgemm_table_tn, true, false, "_tn")
}  // namespace lsmi
