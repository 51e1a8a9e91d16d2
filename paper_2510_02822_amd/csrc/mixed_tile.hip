// One tile shape of the mixed GEMM / implicit-GEMM kernel: the four instantiations (linear or convolution,
// 4-bit weights from the packed codes or from the expanded copy).  Built once per shape with -DFQ_TILE=i.
#include "mixed_kernel.h"

#ifndef FQ_TILE
#error "compile with -DFQ_TILE=<0..14>"
#endif

namespace flexiq {

// waves along M, waves along N, 32x32 fragments per wave along M and N; then the measured cycles of one
// K-step of a block alone on its CU, the relative growth per co-resident block, the epilogue cycles, and the extra
// cycles of a K-step that lowers its activations.
#if FQ_TILE == 0
TileShape tile_shape_0() { return make_shape<2, 2, 4, 4>(1200.0, 0.00, 9000.0, 415.0); }  // 256 x 256
#elif FQ_TILE == 1
TileShape tile_shape_1() { return make_shape<1, 4, 7, 2>(1060.0, 0.00, 6500.0, 400.0); }  // 224 x 256
#elif FQ_TILE == 2
TileShape tile_shape_2() { return make_shape<2, 2, 3, 4>(950.0, 0.00, 7600.0, 350.0); }  // 192 x 256
#elif FQ_TILE == 3
TileShape tile_shape_3() { return make_shape<1, 4, 5, 2>(860.0, 0.00, 5300.0, 365.0); }   // 160 x 256
#elif FQ_TILE == 4
TileShape tile_shape_4() { return make_shape<2, 2, 2, 4>(720.0, 0.00, 6400.0, 275.0); }   // 128 x 256
#elif FQ_TILE == 5
TileShape tile_shape_5() { return make_shape<2, 2, 2, 2>(640.0, 0.33, 2800.0, 245.0); }   // 128 x 128
#elif FQ_TILE == 6
TileShape tile_shape_6() { return make_shape<2, 2, 1, 2>(580.0, 0.37, 1500.0, 200.0); }   //  64 x 128
#elif FQ_TILE == 7
TileShape tile_shape_7() { return make_shape<2, 2, 1, 1>(465.0, 0.45, 900.0, 150.0); }     //  64 x  64
#elif FQ_TILE == 8
TileShape tile_shape_8() { return make_shape<2, 4, 4, 2>(1240.0, 0.00, 8400.0, 310.0); }   // 256 x 256, eight waves
#elif FQ_TILE == 9
TileShape tile_shape_9() { return make_shape<2, 4, 3, 2>(945.0, 0.00, 4000.0, 340.0); }   // 192 x 256, eight waves
#elif FQ_TILE == 10
TileShape tile_shape_10() { return make_shape<1, 8, 5, 1>(835.0, 0.00, 2900.0, 405.0); }   // 160 x 256, eight waves
#elif FQ_TILE == 11
TileShape tile_shape_11() { return make_shape<1, 8, 7, 1>(1125.0, 0.00, 4800.0, 260.0); }  // 224 x 256, eight waves
#elif FQ_TILE == 12
TileShape tile_shape_12() { return make_shape<2, 4, 5, 2>(1500.0, 0.0, 6000.0, 420.0); }   // 320 x 256, eight waves
#elif FQ_TILE == 13
TileShape tile_shape_13() { return make_shape<1, 8, 3, 1>(770.0, 0.0, 2500.0, 245.0); }    //  96 x 256, eight waves
#elif FQ_TILE == 14
TileShape tile_shape_14() { return make_shape<4, 1, 1, 2>(530.0, 0.45, 7000.0, 286.0); }   // 128 x  64 (layers with at most 64 output channels)
#else
#error "FQ_TILE out of range"
#endif

}  // namespace flexiq
