// Specialisations of the register-resident product kernel for the 2:8 pattern.
#include <type_traits>
#include "conv_lds.h"
namespace crisp {
CRISP_INSTANTIATE_NM(2, 8)
}  // namespace crisp
