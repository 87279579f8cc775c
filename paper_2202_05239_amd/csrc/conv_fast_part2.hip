// Tile variants 8, 9, 10, 11 of the LDS-direct dense kernel (conv_fast_kernel.h).
#include "conv_fast_kernel.h"
#include "conv_fast_parts.h"

namespace f8 {

int launch_conv_fast_part2(int variant, const ConvParams &p, int ev, hipStream_t stream) {
  switch (variant) {
    case 8: return p.K <= 64 ? launch_fast_tile<128, 64, 2, 2, 64, 1, 6>(p, ev, stream) : -1;
    case 9: return p.K <= 128 ? launch_fast_tile<128, 64, 2, 2, 128, 1, 5>(p, ev, stream) : -1;
    case 10: return p.K <= 64 ? launch_fast_tile<128, 128, 2, 2, 64, 1, 4>(p, ev, stream) : -1;
    case 11: return launch_fast_tile<128, 256, 2, 2, 64, 2, 2>(p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
