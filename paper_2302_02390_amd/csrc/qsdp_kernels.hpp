// Kernels of the QSDP codec for gfx950.
//
// Two families share the element arithmetic of qsdp_device.hpp:
//   * wave kernels: a bucket is owned by an aligned group of G lanes of one wave and its values
//     never leave registers: one pass over HBM, no barrier (LDS only stages the packed codes so
//     that they are written with 16-byte stores). The bucket is cut into R rows
//     of 4*G elements; lane l of the group holds elements (r*G + l)*4 .. +3 of every row r, so
//     each load/store instruction of a wave touches whole contiguous 16*G-byte segments.
//     Bucket size B = 4*G*R, R even. A Philox block (8 elements) and a packed code chunk
//     (8 codes = BITS bytes) span the lane pair (l even, l+1) of one row: for each row pair
//     (2c, 2c+1) the even lane owns the block/chunk of row 2c and the odd lane that of row
//     2c+1, and the pair swaps halves with one DPP quad permute. A wave handles 64/G buckets
//     at a time, one wave per such group (waves stride only past 2^20 workgroups); a short last
//     bucket takes a guarded element-wise path of the same kernel. Buckets larger than one
//     wave's tile are shared by the W waves of a workgroup (B = 4*G*R*W, G = 64): each wave
//     owns a contiguous 1/W of the bucket and the waves combine their min/max through LDS.
//   * block kernel: one 256-thread workgroup per bucket, staged in LDS; any bucket size, any
//     bits. Used for the bucket sizes the wave kernels are not instantiated for (several times
//     slower: the values make a round trip through LDS and the codes are packed bit by bit).
// The modes and parameters are in qsdp_params.hpp, the two encoder families in qsdp_wave_kernel.hpp and
// qsdp_block_kernel.hpp, the decoders and the element-wise decode-and-sum in qsdp_decoders.hpp, the
// level fit in qsdp_fit_kernel.hpp.
#pragma once

#include "qsdp_params.hpp"
#include "qsdp_wave_kernel.hpp"
#include "qsdp_block_kernel.hpp"
#include "qsdp_decoders.hpp"
#include "qsdp_fit_kernel.hpp"
