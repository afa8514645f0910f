// Matrix-core kernels for the sparse-kernel convolution operators (placeholder:
// nothing is routed here yet).
#include "dsk_internal.h"

namespace dsk {

size_t conv_ws_bytes(int, const ConvShape &, dsk_dtype) { return 0; }
bool conv_mfma_supported(int, const ConvShape &, dsk_dtype, dsk_dtype) { return false; }
int launch_conv_fwd_mfma(const void *, const float *, const float *, void *, const ConvShape &, dsk_dtype,
                         dsk_dtype, int, void *, hipStream_t) { return DSK_EDTYPE; }
int launch_conv_bwd_data_mfma(const void *, const float *, void *, const ConvShape &, dsk_dtype, dsk_dtype,
                              void *, hipStream_t) { return DSK_EDTYPE; }
int launch_conv_bwd_weight_mfma(const void *, const void *, float *, float *, const ConvShape &, dsk_dtype,
                                void *, hipStream_t) { return DSK_EDTYPE; }

} // namespace dsk
