// Compiles one group of the kernels listed in kernel_list.hpp.
#define ECGEMM_INSTANTIATE_COMPARE_B
#include "kernel_list.hpp"
