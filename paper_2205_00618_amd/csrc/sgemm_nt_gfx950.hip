// The sgemm kernels for B stored transposed (N x K): see sgemm_variants.hpp.
#include "sgemm_variants.hpp"

namespace lsmi {
LSMI_DEFINE_SGEMM_TABLE(sgemm_table_nt, false, true, "_nt")
}  // namespace lsmi
