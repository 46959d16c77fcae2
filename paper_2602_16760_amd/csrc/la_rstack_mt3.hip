// The register-streaming persistent kernel (la_rstack.h) for blocks of 33..48 rows (3 row tiles).
#include "la_rstack.h"
namespace la {
namespace rs {
template int launch_rstack_kernel<3, 4>(const StackArgs &, int, hipStream_t);
template int prepare_rstack_kernel<3, 4>(int, int);
}
}  // namespace la
