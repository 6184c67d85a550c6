// Instantiations of the projection GEMM tile (gemm_tile.h) with two MFMA K steps per stage (BK = 64): the short
// tiles whose three stages of 128-byte rows fit the LDS -- 128 columns x 16 .. 144 rows, 256 columns x 16 .. 80 rows.
#include "gemm_tile.h"

hipError_t launch_proj_k64(int mt, int nf, const GemmArgs& g, hipStream_t s) {
  if (nf == 2) {
    switch (mt) {
      case 1: return launch_proj<1, 2, 2>(g, s);
      case 2: return launch_proj<2, 2, 2>(g, s);
      case 3: return launch_proj<3, 2, 2>(g, s);
      case 4: return launch_proj<4, 2, 2>(g, s);
      case 5: return launch_proj<5, 2, 2>(g, s);
      case 6: return launch_proj<6, 2, 2>(g, s);
      case 7: return launch_proj<7, 2, 2>(g, s);
      case 8: return launch_proj<8, 2, 2>(g, s);
      case 9: return launch_proj<9, 2, 2>(g, s);
      default: return hipErrorInvalidValue;
    }
  }
  if (nf == 4) {
    switch (mt) {
      case 1: return launch_proj<1, 4, 2>(g, s);
      case 2: return launch_proj<2, 4, 2>(g, s);
      case 3: return launch_proj<3, 4, 2>(g, s);
      case 4: return launch_proj<4, 4, 2>(g, s);
      case 5: return launch_proj<5, 4, 2>(g, s);
      default: return hipErrorInvalidValue;
    }
  }
  return hipErrorInvalidValue;
}
