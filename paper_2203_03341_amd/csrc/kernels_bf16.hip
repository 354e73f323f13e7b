// Compiles one group of the kernels listed in kernel_list.hpp.
#define ECGEMM_INSTANTIATE_BF16
#include "kernel_list.hpp"
