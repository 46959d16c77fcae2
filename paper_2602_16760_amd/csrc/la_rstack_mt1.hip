// The register-streaming persistent kernel (la_rstack.h) for blocks of 1..16 rows (1 row tile).
#include "la_rstack.h"
namespace la {
namespace rs {
template int launch_rstack_kernel<1, 4>(const StackArgs &, int, hipStream_t);
template int prepare_rstack_kernel<1, 4>(int, int);
}
}  // namespace la
