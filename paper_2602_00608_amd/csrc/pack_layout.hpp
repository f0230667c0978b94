// Packed weight layout shared by the pack kernel and both convolution kernels.
//
// The logical tensor W[co][ci][tap] is cut into fragments of 32 output channels
// x 16 input channels per tap.  A fragment is stored as 512 consecutive
// elements in the lane order of the 32x32x16 MFMA B operand: lane = co%32 +
// 32*((ci%16)/8) holds the 8 elements ci%8 = 0..7.  Fragments are ordered
// [tap][ci/16][co/32].  C_in is padded to a multiple of 16 and C_out to a
// multiple of 32 with zeros.
#pragma once
#include <stddef.h>

namespace wmdec {

__host__ __device__ inline int packed_cin_blocks(int cin) { return (cin + 15) / 16; }
__host__ __device__ inline int packed_cout_blocks(int cout) { return (cout + 31) / 32; }
__host__ __device__ inline size_t packed_elems(int taps, int cout, int cin) {
  return (size_t)taps * packed_cin_blocks(cin) * packed_cout_blocks(cout) * 512;
}
__host__ __device__ inline size_t packed_index(int tap, int co, int ci, int cin_blocks, int cout_blocks) {
  const size_t blk = ((size_t)tap * cin_blocks + (ci >> 4)) * cout_blocks + (co >> 5);
  return blk * 512 + (size_t)(((co & 31) + 32 * ((ci & 15) >> 3)) * 8 + (ci & 7));
}

}  // namespace wmdec
