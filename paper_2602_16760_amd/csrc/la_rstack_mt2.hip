// The register-streaming persistent kernel (la_rstack.h) for blocks of 17..32 rows (2 row tiles).
#include "la_rstack.h"
namespace la {
namespace rs {
template int launch_rstack_kernel<2, 4>(const StackArgs &, int, hipStream_t);
template int prepare_rstack_kernel<2, 4>(int, int);
}
}  // namespace la
