// The persistent kernel for blocks of up to 64 rows.
#include "la_stack.h"

namespace la {
template int launch_stack_kernel<4>(const StackArgs &, int, hipStream_t);
template int prepare_stack_kernel<4>(int, int);
}  // namespace la
