// Stand-ins for the device side of the library in the host-only build that the sanitizer check links
// (build.py --sanitize): everything that would enqueue a kernel reports "not supported".
#include <hip/hip_runtime_api.h>

#include "internal.h"

namespace sc {

int static_scratch(void**) { return (int)hipErrorNotSupported; }
int launch_tile_kernel(int, int, int, int, const KernelArgs&, int, int, int, void*) { return (int)hipErrorNotSupported; }
int launch_lds_read_probe(void*, int, int, void*, long long*) { return (int)hipErrorNotSupported; }
int launch_copy_probe(void*, const void*, long long, void*) { return (int)hipErrorNotSupported; }

}  // namespace sc
