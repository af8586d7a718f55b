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
  float* stats;       // forward only, optional: per-column partial sums of the stored outputs, see igemm_fwd
  int stats_rows;     // set by the launcher: output rows per partial sum
  int Mg, Ng, Kg;
  int act, accumulate, simple;
  // dgrad with accumulate, fast bf16 path only: what is added to the result, if not the old contents of out.
  // acc_src: a tensor shaped like out; acc_bits (optional): one byte per 16-byte chunk of it, bit e set = element
  // e of the chunk counts (the activation bits a BatchNorm's forward pass leaves, see bn_fwd), else it adds 0.
  const void* acc_src;
  const unsigned char* acc_bits;
  int scatter2;                     // dgrad of a 1x1 / stride 2 / no padding layer run over the pixels of dy
  // dgrad of a strided layer with a filter wider than its stride, one launch per parity class (ph, pw):
  // rows are the input pixels (stride*hc + ph, stride*wc + pw), 0 <= hc < Hc, 0 <= wc < Wc, and k runs over
  // the taps r = r0, r0 + stride, ..., s = s0, s0 + stride, ... only (the others never meet such a pixel)
  int cls, ph, pw, r0, s0, Hc, Wc;
  uint32_t magicWc, magicHc;
  int shiftWc, shiftHc;
  // the classes of one launch: slot c holds class 2*ph + pw = 3 - c and takes the workgroups cls_end[c-1] .. cls_end[c]-1; the
  // kernel copies its class's entries into the fields above (and into Mg, nk, tiles_m)
  int cls_end[4], cls_Mg[4], cls_nk[4], cls_tiles_m[4];
  int cls_r0[2], cls_s0[2], cls_Hc[2], cls_Wc[2], cls_shiftHc[2], cls_shiftWc[2];
  uint32_t cls_magicHc[2], cls_magicWc[2];
  int nk, nk_per_split, splits;
  long long split_stride;
  int tiles_m, tiles_n;
  uint32_t a_bytes, b_bytes;        // sizes of the tensors behind a and b
  uint32_t magicQ, magicP;          // x / Q and x / P by multiply-high (output pixel index -> n,p,q)
  int shiftQ, shiftP;
  uint32_t magicW, magicH;          // x / W and x / H (input pixel index -> n,h,w)
  int shiftW, shiftH;
  uint32_t magicC, magicK, magicS;  // x / C, x / K, x / S (k index -> tap and channel; element-wise loaders)
  int shiftC, shiftK, shiftS;
};

// x / d for 0 <= x < 2^31 with the host-computed (magic, shift) of d (magic_div in igemm.hip)
__device__ inline int div_magic(int x, uint32_t magic, int shift) {
  return (int)((__umulhi((uint32_t)x, magic) + (uint32_t)x) >> shift);
}


// Workgroup -> (output tile, split of the reduction axis).  Workgroup ids are dealt round-robin to the
// XCDs, each with an L2 of its own.  The (split, tile) pairs, split-major, are cut into one contiguous
// run per XCD: neighbours in a run share an operand row-block or, across tiles of one split, the same
// slice of both operands, and every XCD gets the same number of workgroups (to within one), also when
// there are fewer tiles than XCDs.  (Dealing whole splits to the XCDs, as an earlier version did, left
// some XCDs with one workgroup more than their CUs hold at once: with 5 tiles x 102 splits six XCDs got
// 65 workgroups for 64 slots, and the one straggler doubled the kernel's duration.)
__device__ inline bool block_to_tile(const Args& a, int bid, int& logical, int& split) {
  const int x = bid % NUM_XCD, j = bid / NUM_XCD;
  const int tiles = a.tiles_m * a.tiles_n;
  const int units = tiles * a.splits, per_xcd = (units + NUM_XCD - 1) / NUM_XCD;
  const int u = x * per_xcd + j;
  split = u / tiles;
  logical = u - split * tiles;
  return j < per_xcd && u < units;
}
__device__ inline bool block_to_tile(const Args& a, int& logical, int& split) {
  return block_to_tile(a, (int)blockIdx.x, logical, split);
}
inline unsigned grid_blocks(const Args& a) {
  const int tiles = a.tiles_m * a.tiles_n;
  return (unsigned)(NUM_XCD * ((tiles * a.splits + NUM_XCD - 1) / NUM_XCD));
}

// bf16 fast path: operands go from global memory straight into LDS (igemm_dma.hip)
bool igemm_dma_geom_ok(int pass, const ConvGeom& g);                     // shape only
bool igemm_dma_ok(int pass, const ConvGeom& g, const Args& a);            // shape and pointer alignment
void igemm_dma_tile(int pass, int Mg, int Ng, int splits, int& BM, int& BN);  // the tile igemm_dma_launch picks
int igemm_dma_launch(int pass, Args& a, int splits, hipStream_t st);

}  // namespace s4tf
