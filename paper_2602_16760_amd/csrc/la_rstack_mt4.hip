// The register-streaming persistent kernel (la_rstack.h) for blocks of 49..64 rows (4 row tiles).
#include "la_rstack.h"
namespace la {
namespace rs {
template int launch_rstack_kernel<4, 4>(const StackArgs &, int, hipStream_t);
template int prepare_rstack_kernel<4, 4>(int, int);
}
}  // namespace la
