// Launchers private to the convolution translation units.
#pragma once
#include "anr_kernels.h"

namespace anr {

hipError_t launch_conv2d_direct(const ConvArgs& a, hipStream_t stream);
hipError_t launch_dwconv_direct(const ConvArgs& a, hipStream_t stream);

// Implicit-GEMM MFMA convolution.  Returns false in *taken when the geometry is
// outside what the kernel supports or the route rules it out (the caller then uses the
// general kernel).
hipError_t launch_conv2d_igemm(const ConvArgs& a, hipStream_t stream, bool* taken);

// Whether launch_conv2d_igemm would take the problem (same selection, nothing launched).
bool conv2d_igemm_takes(const ConvArgs& a);

// General implicit-GEMM convolution with gathered operands and optional split-K over a
// workspace.  *taken false: extents beyond its 32-bit offsets (the direct kernel runs then).
// *ws_fault as in launch_conv2d.
hipError_t launch_conv2d_gather(const ConvArgs& a, hipStream_t stream, bool* taken, int* ws_fault);
size_t conv2d_gather_workspace_bytes(const ConvArgs& a);

// Streaming kernel for pointwise layers with few channels (conv_pointwise_kernel.h); same contract.
hipError_t launch_conv2d_pointwise(const ConvArgs& a, hipStream_t stream, bool* taken);

// What a launch would do, for introspection (nothing is launched).
struct ConvRoute {
    int kernel;          // 1 patch-staging, 2 taps, 3 bigtaps, 4 gather, 5 direct, 6 pointwise stream (the public ANR_CONV_KERNEL_* values)
    int tile_m, tile_n, ksplit, wave_groups, work_groups;
    size_t workspace_bytes;
};
bool describe_conv2d_igemm(const ConvArgs& a, ConvRoute* r);
bool describe_conv2d_gather(const ConvArgs& a, ConvRoute* r);
bool describe_conv2d_pointwise(const ConvArgs& a, ConvRoute* r);
void describe_conv2d(const ConvArgs& a, ConvRoute* r);

// Register-sliding 3x3 / stride 1 / pad 1 depthwise kernel; same contract.
hipError_t launch_dwconv3x3(const ConvArgs& a, hipStream_t stream, bool* taken);

}  // namespace anr
