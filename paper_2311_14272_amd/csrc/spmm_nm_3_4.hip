// Specialisations of the register-resident product kernel for the 3:4 pattern.
#include <type_traits>
#include "conv_lds.h"
namespace crisp {
CRISP_INSTANTIATE_NM(3, 4)
}  // namespace crisp
