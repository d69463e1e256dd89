// Stand-ins for the device side of libgqsa in a host-only build of the library (the
// sanitizer build of paper_2412_17560_amd/build.py): everything that would touch the GPU
// answers GQSA_ERR_HIP, so that the packer, the image builders and the C boundary can run
// under AddressSanitizer and UndefinedBehaviorSanitizer on a machine without a GPU.
// Never linked into libgqsa.so itself.
#include "gqsa_bench.h"
#include "gqsa_internal.hpp"

namespace gqsa {

gqsa_status_t device_upload(gqsa_matrix*, void*) { return GQSA_ERR_HIP; }
gqsa_status_t pack_on_device(const float*, const float*, gqsa_matrix*, void*) { return GQSA_ERR_HIP; }
void device_release(gqsa_matrix*) {}
gqsa_status_t device_gemv(gqsa_matrix* const*, int, const void*, void* const*, int, void*, void*) { return GQSA_ERR_HIP; }
gqsa_status_t device_gemv_static(gqsa_matrix*, const void*, void*, int, void*) { return GQSA_ERR_HIP; }
bool stream_is_capturing(void*) { return false; }
gqsa_status_t panels_upload(gqsa_matrix*) { return GQSA_ERR_HIP; }
void panels_release(gqsa_matrix*) {}
gqsa_status_t panels_gemm(const gqsa_matrix* const*, int, const void*, void* const*, int, void*) { return GQSA_ERR_HIP; }

}  // namespace gqsa

extern "C" {

gqsa_status_t gqsa_dense_f16_gemv(const void*, const void*, void*, int64_t, int64_t, int, void*) { return GQSA_ERR_HIP; }
gqsa_status_t gqsa_launch_floor(int, int, void*, void*) { return GQSA_ERR_HIP; }
gqsa_status_t gqsa_copy(void*, const void*, size_t, void*) { return GQSA_ERR_HIP; }
int gqsa_stream_read_workgroups(void) { return 0; }
gqsa_status_t gqsa_stream_read(const void*, size_t, void*, void*) { return GQSA_ERR_HIP; }

}  // extern "C"
