// The kernel variant space: the knobs the per-layer tuner chooses from, the
// counterpart of the paper's tile-size / LMUL template parameters (section 3.3).
//   NBLK 16-pixel MFMA blocks per wavefront   WP  wavefronts along the pixel axis
//        (pixels per workgroup BP = 16*NBLK*WP)
//   NJ  16-channel row blocks per wavefront
//   CK  im2col rows per LDS chunk      SPC k-steps (4 kept columns each) per chunk
//   VEC 1: chunks are channel runs of one tap fetched 16 bytes at a time
//       0: chunks are cut on the flat k axis, fetched element-wise (Cin % 4 != 0)
#pragma once

// X(NBLK, WP, NJ)
#define NM_SHAPES(X) \
    X(8, 1, 2) X(8, 1, 4) X(4, 2, 4) X(4, 2, 2) X(8, 2, 2) X(4, 4, 4) \
    X(4, 1, 2) X(4, 1, 4) X(4, 1, 1)                                  \
    X(1, 4, 1) X(1, 4, 2) X(2, 1, 1) X(2, 1, 2) X(2, 2, 1) X(2, 2, 2) \
    X(3, 1, 1) X(3, 1, 2) X(5, 1, 1) X(6, 1, 1) X(6, 1, 2) X(7, 1, 1) \
    X(7, 1, 2) X(7, 2, 1) X(8, 1, 1) X(10, 1, 1) X(12, 1, 1)          \
    X(13, 1, 1) X(13, 1, 2) X(14, 1, 1) X(16, 1, 1) X(16, 1, 2)

// Y(NBLK, WP, NJ, CK, SPC, VEC)
#define NM_VEC_CHUNKS(Y, NB, WP, NJ)                                              \
    Y(NB, WP, NJ, 32, 2, 1) Y(NB, WP, NJ, 32, 4, 1) Y(NB, WP, NJ, 32, 8, 1)       \
    Y(NB, WP, NJ, 64, 2, 1) Y(NB, WP, NJ, 64, 4, 1) Y(NB, WP, NJ, 64, 8, 1)

// fp32 kernel with a per-(tile, chunk) number of k-steps: for kept sets that are not
// spread evenly over the chunks (group size M larger than a chunk).  SPC = CK / 4 is
// the width of the operand table, not the work done.
// X(NBLK, WP, NJ)
#define NMVAR_SHAPES(X)                                                             \
    X(2, 1, 1) X(3, 1, 1) X(4, 1, 1) X(5, 1, 1) X(6, 1, 1) X(7, 1, 1) X(8, 1, 1)    \
    X(10, 1, 1) X(13, 1, 1) X(2, 1, 2) X(4, 1, 2) X(8, 1, 2) X(2, 2, 1) X(4, 2, 2)
// Y(NBLK, WP, NJ, CK, SPC)
#define NMVAR_CHUNKS(Y, NB, WP, NJ) Y(NB, WP, NJ, 32, 8) Y(NB, WP, NJ, 64, 16)

#define NM_SCALAR_VARIANTS(Y) Y(4, 4, 4, 32, 8, 0) Y(4, 2, 2, 32, 8, 0) Y(4, 1, 1, 32, 8, 0)

// bf16 matrix-core kernel (bf16 activations, bf16-rounded weights):
//   SHARE row blocks of one column tile are fed from the same gathered operand (2 for T = 32)
//   a k-step is 32 kept columns; CK channels per chunk hold SPC k-steps
// X(NBLK, WP, NJ, SHARE)
#define NM16_SHAPES(X)                                                              \
    X(8, 1, 2, 1) X(8, 1, 1, 1) X(4, 1, 2, 1) X(4, 1, 1, 1) X(4, 2, 2, 1) X(2, 1, 2, 1) \
    X(2, 1, 1, 1) X(5, 1, 1, 1) X(6, 1, 1, 1) X(12, 1, 1, 1) X(16, 1, 1, 1)            \
    X(8, 1, 2, 2) X(4, 1, 2, 2) X(4, 2, 2, 2) X(2, 1, 2, 2) X(4, 1, 4, 2)
// Y(NBLK, WP, NJ, SHARE, CK, SPC)
#define NM16_CHUNKS(Y, NB, WP, NJ, SH)                                              \
    Y(NB, WP, NJ, SH, 32, 1) Y(NB, WP, NJ, SH, 64, 1) Y(NB, WP, NJ, SH, 128, 1)     \
    Y(NB, WP, NJ, SH, 64, 2) Y(NB, WP, NJ, SH, 128, 2) Y(NB, WP, NJ, SH, 256, 1)

// bf16 kernels that contract the dense strip without a gather: the sparse
// matrix instruction (SP = 1: N <= 2 kept of every aligned 4 columns) or the
// dense one on zero-filled weights (SP = 0).  A chunk is CK channels of one tap.
// X(NBLK, WP, NJ)
#define NMSP_SHAPES(X)                                                          \
    X(4, 1, 2) X(4, 1, 4) X(2, 1, 2) X(2, 1, 4) X(4, 2, 2) X(4, 2, 4) X(8, 1, 2) \
    X(8, 1, 1) X(4, 1, 1) X(2, 1, 1) X(2, 2, 2) X(6, 1, 2) X(3, 1, 2) X(2, 2, 4)
// Y(NBLK, WP, NJ, CK, SP)
#define NMSP_CHUNKS(Y, NB, WP, NJ)                                   \
    Y(NB, WP, NJ, 64, 1) Y(NB, WP, NJ, 128, 1) Y(NB, WP, NJ, 256, 1) \
    Y(NB, WP, NJ, 64, 0) Y(NB, WP, NJ, 128, 0) Y(NB, WP, NJ, 256, 0)

// The same kernels with four producer wavefronts that issue the loads (512 threads).
// X(NBLK, WP, NJ)
#define NMSPW_SHAPES(X) X(8, 1, 2) X(4, 1, 2) X(4, 2, 4) X(4, 1, 4) X(4, 2, 2) X(6, 1, 2) X(2, 1, 2) X(2, 2, 4)
// Y(NBLK, WP, NJ, CK, SP)
#define NMSPW_CHUNKS(Y, NB, WP, NJ)                                  \
    Y(NB, WP, NJ, 64, 1) Y(NB, WP, NJ, 128, 1) Y(NB, WP, NJ, 256, 1) \
    Y(NB, WP, NJ, 64, 0) Y(NB, WP, NJ, 128, 0) Y(NB, WP, NJ, 256, 0)

// Producer wavefronts, and the weights loaded straight into the contracting wavefronts'
// registers (the LDS stages hold the strip alone).
// X(NBLK, WP, NJ)
#define NMSPR_SHAPES(X) X(4, 2, 4) X(8, 1, 2) X(4, 1, 4) X(2, 2, 4) X(8, 2, 4) X(4, 2, 2) X(8, 1, 4) X(6, 1, 2)
// Y(NBLK, WP, NJ, CK, SP)
#define NMSPR_CHUNKS(Y, NB, WP, NJ)             \
    Y(NB, WP, NJ, 64, 1) Y(NB, WP, NJ, 128, 1) \
    Y(NB, WP, NJ, 64, 0) Y(NB, WP, NJ, 128, 0)

// bf16 kernel for layers with very few input channels (contiguous kernel-row
// runs, one chunk of KS 64-element k-steps).
// X(NBLK, WP, NJ)
#define NMRUN_SHAPES(X) \
    X(4, 1, 1) X(8, 1, 1) X(2, 1, 1) X(2, 2, 2) X(4, 2, 2) X(2, 4, 4) X(4, 4, 4) X(1, 4, 4) X(3, 4, 4) X(7, 1, 1)
// Y(NBLK, WP, NJ, KS)
#define NMRUN_CHUNKS(Y, NB, WP, NJ) Y(NB, WP, NJ, 1) Y(NB, WP, NJ, 2) Y(NB, WP, NJ, 3) Y(NB, WP, NJ, 4)

// fp8 through the staged kernel of the gather-free bf16 form (LDS ring, optional producer
// wavefronts and register-held weights): CK E4M3 channels of one tap per chunk.
// X(NBLK, WP, NJ)
#define NMF8S_SHAPES(X) X(8, 1, 2) X(4, 1, 2) X(4, 1, 1) X(6, 1, 2) X(4, 2, 2) X(8, 1, 4) X(4, 2, 4) X(4, 1, 4) X(2, 1, 2)
// Y(NBLK, WP, NJ, CK)
#define NMF8S_CHUNKS(Y, NB, WP, NJ) Y(NB, WP, NJ, 64) Y(NB, WP, NJ, 128) Y(NB, WP, NJ, 256)

// fp8 (E4M3 activations and weights, bf16 output): both operands streamed from global memory
// into registers, 64-channel k-steps.
// X(NBLK, WP, NJ)
#define NMF8_SHAPES(X) \
    X(4, 1, 4) X(4, 2, 4) X(4, 4, 4) X(2, 1, 4) X(2, 2, 4) X(2, 4, 4) X(4, 1, 2) X(4, 2, 2) X(8, 1, 2) X(8, 2, 2)
