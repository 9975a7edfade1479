// Specialisations of the register-resident product kernel for the 8:8 pattern.
#include <type_traits>
#include "conv_lds.h"
namespace crisp {
CRISP_INSTANTIATE_NM(8, 8)
}  // namespace crisp
