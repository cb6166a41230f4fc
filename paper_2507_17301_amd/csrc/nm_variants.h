// The kernel variant space: the knobs the per-layer tuner chooses from, the
// counterpart of the paper's tile-size / LMUL template parameters (section 3.3).
//   BP  pixels per workgroup           WP  wavefronts along the pixel axis
//   NJ  16-channel row blocks per wavefront
//   CK  im2col rows per LDS chunk      SPC k-steps (4 kept columns each) per chunk
//   VEC 1: chunks are channel runs of one tap fetched 16 bytes at a time
//       0: chunks are cut on the flat k axis, fetched element-wise (Cin % 4 != 0)
#pragma once

// X(BP, WP, NJ)
#define NM_SHAPES(X) \
    X(128, 1, 2) X(128, 1, 4) X(128, 2, 4) X(128, 2, 2) X(256, 2, 2) X(256, 4, 4) \
    X(64, 1, 2) X(64, 1, 4) X(64, 1, 1)

// Y(BP, WP, NJ, CK, SPC, VEC)
#define NM_VEC_CHUNKS(Y, BP, WP, NJ)                                              \
    Y(BP, WP, NJ, 32, 2, 1) Y(BP, WP, NJ, 32, 4, 1) Y(BP, WP, NJ, 32, 8, 1)       \
    Y(BP, WP, NJ, 64, 2, 1) Y(BP, WP, NJ, 64, 4, 1) Y(BP, WP, NJ, 64, 8, 1)

#define NM_SCALAR_VARIANTS(Y) Y(256, 4, 4, 32, 8, 0) Y(128, 2, 2, 32, 8, 0) Y(64, 1, 1, 32, 8, 0)
