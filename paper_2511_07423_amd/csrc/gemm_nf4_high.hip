// Instantiations of the projection GEMM tile (gemm_tile.h): 256 columns, 160 .. 272 rows.
#include "gemm_tile.h"

hipError_t launch_proj_nf4_high(int mt, const GemmArgs& g, hipStream_t s) {
  switch (mt) {
    case 10: return launch_proj<10, 4>(g, s);
    case 11: return launch_proj<11, 4>(g, s);
    case 12: return launch_proj<12, 4>(g, s);
    case 13: return launch_proj<13, 4>(g, s);
    case 14: return launch_proj<14, 4>(g, s);
    case 15: return launch_proj<15, 4>(g, s);
    case 16: return launch_proj<16, 4>(g, s);
    case 17: return launch_proj<17, 4>(g, s);
    default: return hipErrorInvalidValue;
  }
}
