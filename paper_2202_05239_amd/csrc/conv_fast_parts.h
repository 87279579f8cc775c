// Entry points of the files that instantiate the tile variants of the LDS-direct dense kernel.
#pragma once

#include "f8_host.h"

namespace f8 {

// Launch tile variant `variant` (one of the variants the part holds; -1 otherwise).  ev is the
// width in bytes (16 or 4) of the epilogue's global accesses.
int launch_conv_fast_part0(int variant, const ConvParams &p, int ev, hipStream_t stream);
int launch_conv_fast_part1(int variant, const ConvParams &p, int ev, hipStream_t stream);
int launch_conv_fast_part2(int variant, const ConvParams &p, int ev, hipStream_t stream);
int launch_conv_fast_part3(int variant, const ConvParams &p, int ev, hipStream_t stream);
int launch_conv_fast_part4(int variant, const ConvParams &p, int ev, hipStream_t stream);
int launch_conv_fast_part5(int variant, const ConvParams &p, int ev, hipStream_t stream);
int launch_conv_fast_part6(int variant, const ConvParams &p, int ev, hipStream_t stream);

}  // namespace f8
