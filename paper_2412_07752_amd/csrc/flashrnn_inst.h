// Instantiation lists of the persistent kernels.  Included by one translation unit per
// (cell, I/O dtype) with FRNN_CELL, FRNN_G and FRNN_BF16 defined.
//
// Shapes (KT = k-steps per wave, 32 contraction elements per bf16 step, 4 per f32 step):
//   one workgroup per group:   units D <= 32 / 64 / 128 / 192 (bf16) or 16 / 32 / 64 / 128 (f32)
//   several workgroups:        D up to 1024 (bf16) / 256 (f32) inside one XCD, optionally 4 contraction slices;
//                              D up to 2688 (bf16) spread over all XCDs: one block of 16 units and 4 contraction slices
//                              per workgroup, one wave per SIMD with up to 336 registers of R
#pragma once
#include "flashrnn_host.h"
#include "flashrnn_kernels.h"
#include "flashrnn_tile_kernels.h"
#include "flashrnn_recompute.h"

namespace flashrnn {

#define FRNN_F(KT, KS, BT, MULTI, MAXW, EB) \
    {FRNN_CELL, FRNN_BF16, 0, KT, KS, BT, MULTI, MAXW, EB, 0, 0, (const void*)&fwd_kernel<FRNN_CELL, (FRNN_BF16 != 0), KT, KS, BT, (MULTI != 0), MAXW, EB>},
#define FRNN_B(KT, KS, BT, MULTI, MAXW, EB) \
    {FRNN_CELL, FRNN_BF16, 1, (KT) * FRNN_G, KS, BT, MULTI, MAXW, EB, 0, 0, (const void*)&bwd_kernel<FRNN_CELL, (FRNN_BF16 != 0), (KT) * FRNN_G, KS, BT, (MULTI != 0), MAXW, EB>},
// forward and backward share the shape list: the backward contraction axis is G times longer
#define FRNN_FB(KT, KS, BT, MULTI, MAXW) FRNN_F(KT, KS, BT, MULTI, MAXW, 1) FRNN_B(KT, KS, BT, MULTI, MAXW, 1)
// small batch tiles (bf16, one workgroup per group): forward from the dedicated tile kernel
#define FRNN_FT(KT, BT, MAXW) \
    {FRNN_CELL, FRNN_BF16, 0, KT, 1, BT, 0, MAXW, 1, 1, 0, (const void*)&fwd_tile_kernel<FRNN_CELL, KT, BT, MAXW>},
// ... backward with the contraction split over EBK waves per set of EBK unit blocks; one kernel for heads of exactly
// KT * 32 units (compile-time LDS layout) and one for the sizes below (two kernels, not two paths in one: the backward
// kernel sits at the register limit of its launch bound, and a spill in either path would disqualify both)
#define FRNN_BTL(KT, EBK, BT, MAXW) \
    {FRNN_CELL, FRNN_BF16, 1, (KT) * FRNN_G, 1, BT, 0, MAXW, EBK, 1, 1, (const void*)&bwd_tile_kernel<FRNN_CELL, (KT) * FRNN_G / (EBK), EBK, BT, MAXW, true>}, \
    {FRNN_CELL, FRNN_BF16, 1, (KT) * FRNN_G, 1, BT, 0, MAXW, EBK, 1, 0, (const void*)&bwd_tile_kernel<FRNN_CELL, (KT) * FRNN_G / (EBK), EBK, BT, MAXW, false>},
// ... and, for heads of up to 128 units, two more that request their inputs six steps ahead through registers
// (taken when they will come from HBM; KernelEntry::exact = 2: heads of exactly 32, 64 or 128 units, 3: the sizes below)
#define FRNN_BTLD(KT, EBK, BT, MAXW) \
    {FRNN_CELL, FRNN_BF16, 1, (KT) * FRNN_G, 1, BT, 0, MAXW, EBK, 1, 2, (const void*)&bwd_tile_kernel<FRNN_CELL, (KT) * FRNN_G / (EBK), EBK, BT, MAXW, true, true>}, \
    {FRNN_CELL, FRNN_BF16, 1, (KT) * FRNN_G, 1, BT, 0, MAXW, EBK, 1, 3, (const void*)&bwd_tile_kernel<FRNN_CELL, (KT) * FRNN_G / (EBK), EBK, BT, MAXW, false, true>},
#define FRNN_TILE(KT, EBK, BT, MAXW) FRNN_FT(KT, BT, MAXW) FRNN_B(KT, 1, BT, 0, MAXW, 1) FRNN_BTL(KT, EBK, BT, MAXW)
// the largest heads: one block of 16 units per workgroup, 4 contraction slices, one wave per SIMD
#define FRNN_FL(KT, BT) FRNN_F(KT, 4, BT, 1, 4, 1)
#define FRNN_BL(KT, BT) FRNN_B(KT, 4, BT, 1, 4, 1)
// EB blocks of 16 units per wave (fewer, fatter waves: the operand is read from LDS once per wave)
#define FRNN_FBE(KT, BT, MAXW, EB) FRNN_F(KT, 1, BT, 0, MAXW, EB) FRNN_B(KT, 1, BT, 0, MAXW, EB)

static const KernelEntry kEntries[] = {
#if FRNN_BF16
    FRNN_FB(1, 1, 16, 0, 4) FRNN_TILE(1, 1, 8, 4) FRNN_TILE(1, 1, 4, 4) FRNN_BTLD(1, 1, 8, 4) FRNN_BTLD(1, 1, 4, 4)
    FRNN_FB(2, 1, 16, 0, 4) FRNN_TILE(2, 2, 8, 4) FRNN_TILE(2, 2, 4, 4) FRNN_BTL(2, 1, 8, 4) FRNN_BTL(2, 1, 4, 4) FRNN_BTLD(2, 1, 8, 4) FRNN_BTLD(2, 1, 4, 4)
    FRNN_FB(4, 1, 16, 0, 8) FRNN_TILE(4, 2, 8, 8) FRNN_TILE(4, 2, 4, 8) FRNN_BTL(4, 1, 8, 8) FRNN_BTL(4, 1, 4, 8) FRNN_BTL(4, 4, 8, 8) FRNN_BTL(4, 4, 4, 8) FRNN_BTLD(4, 1, 8, 8) FRNN_BTLD(4, 1, 4, 8)
    FRNN_FB(6, 1, 16, 0, 12) FRNN_TILE(6, 3, 8, 12) FRNN_TILE(6, 3, 4, 12) FRNN_BTL(6, 1, 8, 12) FRNN_BTL(6, 1, 4, 12)
    FRNN_FBE(4, 16, 4, 2) FRNN_FBE(4, 8, 4, 2) FRNN_FBE(4, 4, 4, 2)
    FRNN_FBE(6, 16, 4, 3) FRNN_FBE(6, 8, 4, 3) FRNN_FBE(6, 4, 4, 3)
#define FRNN_MULTI_SHAPES(BT) \
    FRNN_FB(2, 1, BT, 1, 4) FRNN_FB(4, 1, BT, 1, 4) FRNN_FB(6, 1, BT, 1, 4) FRNN_FB(1, 4, BT, 1, 4) \
    FRNN_FB(8, 1, BT, 1, 8) FRNN_FB(12, 1, BT, 1, 4) FRNN_FB(16, 1, BT, 1, 4) FRNN_FB(24, 1, BT, 1, 4) \
    FRNN_FB(6, 4, BT, 1, 8) FRNN_FB(8, 4, BT, 1, 8)
    // a head split over workgroups, for batch tiles of 16, 8 and 4 rows (small tiles: more groups, less to exchange)
    FRNN_MULTI_SHAPES(16) FRNN_MULTI_SHAPES(8) FRNN_MULTI_SHAPES(4)
#undef FRNN_MULTI_SHAPES
    // heads of 1040 .. 2688 units: contraction lengths 1280, 1536, 2048, 2560, 2688.  Forward with all 16 rows of a
    // batch tile where the registers allow, backward (whose point-wise phase holds more values per row) with 8 or 4;
    // the planner takes the largest tile whose kernel neither spills nor overflows the LDS.
    FRNN_FL(10, 16) FRNN_FL(12, 16) FRNN_FL(16, 16) FRNN_FL(20, 16) FRNN_FL(21, 16)
    FRNN_FL(10, 4) FRNN_FL(12, 4) FRNN_FL(16, 4) FRNN_FL(20, 4) FRNN_FL(21, 4)
    FRNN_BL(10, 8) FRNN_BL(12, 8) FRNN_BL(16, 8) FRNN_BL(20, 8) FRNN_BL(21, 8)
    FRNN_BL(10, 4) FRNN_BL(12, 4) FRNN_BL(16, 4) FRNN_BL(20, 4) FRNN_BL(21, 4)
#else
    FRNN_FB(4, 1, 16, 0, 4) FRNN_FB(8, 1, 16, 0, 4) FRNN_FB(16, 1, 16, 0, 4) FRNN_FB(32, 1, 16, 0, 8)
    // small batches: tiles of 4 and 8 rows (a quarter / half of the point-wise work and of the lane-wise traffic per workgroup)
    FRNN_FB(4, 1, 8, 0, 4) FRNN_FB(8, 1, 8, 0, 4) FRNN_FB(16, 1, 8, 0, 4) FRNN_FB(32, 1, 8, 0, 8)
    FRNN_FB(4, 1, 4, 0, 4) FRNN_FB(8, 1, 4, 0, 4) FRNN_FB(16, 1, 4, 0, 4) FRNN_FB(32, 1, 4, 0, 8)
    FRNN_FB(16, 1, 16, 1, 4) FRNN_FB(32, 1, 16, 1, 4) FRNN_FB(48, 1, 16, 1, 4) FRNN_FB(64, 1, 16, 1, 4)
    FRNN_FB(8, 4, 16, 1, 4)
#endif
};

inline KernelTable make_table() {
    return KernelTable{kEntries, (int)(sizeof(kEntries) / sizeof(kEntries[0])), (const void*)&recompute_records_kernel<FRNN_CELL, (FRNN_BF16 != 0)>};
}

#undef FRNN_F
#undef FRNN_B
#undef FRNN_FB
#undef FRNN_FBE
#undef FRNN_FL
#undef FRNN_BL
#undef FRNN_FT
#undef FRNN_BTL
#undef FRNN_BTLD
#undef FRNN_TILE

}  // namespace flashrnn
