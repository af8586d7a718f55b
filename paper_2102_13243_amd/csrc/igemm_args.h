// Arguments shared by the implicit-GEMM convolution kernels (see igemm.hip for the GEMM view).
#pragma once
#include "s4tf_internal.h"

namespace s4tf {

enum { PASS_FWD = 0, PASS_DGRAD = 1, PASS_WGRAD = 2 };
constexpr int NT = 256;      // threads per block: 4 wavefronts
constexpr int NUM_XCD = 8;   // workgroup ids are dealt round-robin to the 8 XCDs

struct Args {
  ConvGeom g;
  const void* a;
  const void* b;
  void* out;
  const float* bias;
  int Mg, Ng, Kg;
  int act, accumulate, simple;
  int scatter2;                     // dgrad of a 1x1 / stride 2 / no padding layer run over the pixels of dy
  int nk, nk_per_split;
  long long split_stride;
  int tiles_m, tiles_n, tiles_per_xcd;
  uint32_t a_bytes, b_bytes;        // sizes of the tensors behind a and b
  uint32_t magicQ, magicP;          // x / Q and x / P by multiply-high (output pixel index -> n,p,q)
  int shiftQ, shiftP;
  uint32_t magicW, magicH;          // x / W and x / H (input pixel index -> n,h,w)
  int shiftW, shiftH;
};


// bf16 fast path: operands go from global memory straight into LDS (igemm_dma.hip)
bool igemm_dma_geom_ok(int pass, const ConvGeom& g);                     // shape only
bool igemm_dma_ok(int pass, const ConvGeom& g, const Args& a);            // shape and pointer alignment
void igemm_dma_tile(int pass, int Mg, int Ng, int splits, int& BM, int& BN);  // the tile igemm_dma_launch picks
int igemm_dma_launch(int pass, Args& a, int splits, hipStream_t st);

}  // namespace s4tf
