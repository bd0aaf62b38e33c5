// bf16-input kernel variants of the weight gradient (see dw_impl.hpp)
#include "dw_impl.hpp"

namespace surgeon {
template int run_dw<uint16_t>(const DwPlan&, const surgeon_layer_desc*, const void*, const uint64_t*, const void*, float*, void*,
                        hipStream_t, float*, double*);
}  // namespace surgeon
