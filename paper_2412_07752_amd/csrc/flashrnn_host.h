// Host-side declarations shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace flashrnn {

struct KernelParams;

// One compiled instantiation of the persistent forward or backward kernel.
struct KernelEntry {
    int cell, bf16, bwd;
    int KT;     // MFMA k-steps per wave
    int KS;     // contraction slices per workgroup
    int BT;     // valid batch slots per tile (16, 8, 4)
    int multi;  // several workgroups per group
    int maxw;   // launch bound in waves
    int eb;     // blocks of 16 units per wave
    int tile;   // 0: generic kernel, 1: staged tile kernel (bf16, one workgroup per group, BT < 16)
    int exact;  // 1: only for heads of exactly the kernel's contraction length (compile-time LDS layout); 2: such a kernel that
                // fetches its inputs six steps ahead (for inputs that come from HBM); 3: the same for the sizes below
    const void* fn;
};

struct KernelTable {
    const KernelEntry* entries;
    int count;
    const void* recompute;   // recompute_records_kernel of this (cell, I/O dtype)
};

// tables defined in flashrnn_inst_*.hip
KernelTable table_lstm_bf16();
KernelTable table_lstm_f32();
KernelTable table_gru_bf16();
KernelTable table_gru_f32();
KernelTable table_slstm_bf16();
KernelTable table_slstm_f32();
KernelTable table_elman_bf16();
KernelTable table_elman_f32();
KernelTable table_gru4_bf16();
KernelTable table_gru4_f32();

int dr_split_k(bool bf16, int T, int B, int NH, int D, int G);
hipError_t launch_dr_gemm(bool bf16, const float* states, const void* dWx, const void* dgn, float* part, float* dR, int T, int B,
                          int NH, int D, int G, int S, bool gru, float* db_part, bool db_from_gemm, float* db, hipStream_t stream);
hipError_t launch_sum_slices(const float* part, float* out, size_t count, int NS, size_t stride, hipStream_t stream);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);
hipError_t launch_pack_r(bool bf16, bool bwd, const void* R, void* out, int NH, int D, int G, int DK, int* err, hipStream_t stream);

}  // namespace flashrnn
