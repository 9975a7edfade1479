// Specialisations of the register-resident product kernel for the 4:4 pattern.
#include <type_traits>
#include "conv_lds.h"
namespace crisp {
CRISP_INSTANTIATE_NM(4, 4)
}  // namespace crisp
