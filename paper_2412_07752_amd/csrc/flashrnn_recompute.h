// Backward pass without a saved-values buffer: the values the forward pass would have written out for the backward pass
// (Alg. 1, "write out gates for backward pass") are formed again from Wx, R, b and the stored states, a window of time
// steps at a time.  Every h_{t-1} is in `states`, so inside a window nothing is sequential: the pre-activations
//     g_t = Wx_t + R^T h_{t-1} + b            (Sec. 3, eq. (1))
// of all steps of the window are one dense contraction per head, [G*D gate columns] x [window steps * batch rows] over D,
// and the point-wise function (App. A) applied to (g_t, s_{t-1}) gives the same record the forward kernel stores.
// The persistent backward kernel then runs over the window as usual, with the gradients of the carried states handed
// from window to window.
//
// Tile of one workgroup (4 waves): 64 units x all G gates x 64 columns (a column = one (step, batch row) pair); a wave owns
// 16 units and, like the forward kernel, all gates of them, so that its G accumulators of a column tile hold the G
// pre-activations of a (unit, column) pair in the same lane and the point-wise function runs in registers.
// R[n][d][g][e] has the contraction index d as its slow axis and the units contiguous: its tile goes to LDS as it is and
// the A operands are read with the transposing LDS load (bf16) or element-wise (f32); h is converted to the I/O dtype and
// laid out [column][d].
#pragma once
#include "flashrnn_kernels.h"

namespace flashrnn {

struct RecomputeParams {
    const void* Wx;        // [T,B,G,NH,D] io, already advanced to the window's first step
    const void* R;         // [NH,D,G,D] io (the caller's layout, no packed copy)
    const void* bias;      // [NH,G,D] io
    const float* states;   // [.,S,B,NH,D], already advanced: slot 0 = states before the window's first step
    void* cache;           // OUT [steps,B,NH,D,RS] io: records of the window
    int steps, B, NH, D;
};

template <int CELL, bool BF16>
__global__ __launch_bounds__(256) void recompute_records_kernel(const RecomputeParams p) {
    using CT = CellTraits<CELL>;
    using OP = Operand<BF16>;
    constexpr int G = CT::G, S = CT::S, NC = CT::NC, RS = CT::RS;
    constexpr int ESZ = BF16 ? 2 : 4;
    constexpr int UB = 64, CB = 64, KR = 32;            // units, columns per workgroup; contraction rows per round
    constexpr int NCT = CB / 16;                         // column tiles per wave
    constexpr int PR = G * UB + (BF16 ? 16 : 8);         // LDS row pitch of the R tile (elements): see the dR GEMM for the bf16 choice
    constexpr int PH = KR + (BF16 ? 8 : 4);              // LDS row pitch of the h tile (elements)
    __shared__ __align__(16) char ldsR[KR * PR * ESZ];
    __shared__ __align__(16) char ldsH[CB * PH * ESZ];
    const int B = p.B, NH = p.NH, D = p.D;
    const int n = blockIdx.z, u0 = blockIdx.y * UB, col0 = blockIdx.x * CB;
    const int ncols = p.steps * B;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int c = lane & 15, quad = lane >> 4;
    const size_t HD = (size_t)NH * D;

    f32x4 acc[G][NCT];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int j = 0; j < NCT; ++j) acc[g][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- loader roles (16-byte chunks).  R tile: KR rows x G gates x UB units; h tile: CB columns x KR contraction elements (f32 in memory).
    constexpr int EPC = 16 / ESZ;                        // elements per chunk of the I/O dtype
    constexpr int R_CH = KR * G * UB / EPC, LR = (R_CH + 255) / 256;
    constexpr int H_CH = CB * KR / 4, LH = H_CH / 256;   // chunks of 4 floats
    static_assert(H_CH % 256 == 0, "h loader tiling");
    for (int kb = 0; kb < D; kb += KR) {
        __syncthreads();   // the previous round's operands have been read
#pragma unroll
        for (int x = 0; x < LR; ++x) {
            const int ch = tid + x * 256;
            if (ch < R_CH) {
                const int row = ch / (G * UB / EPC), rem = ch % (G * UB / EPC), g = rem / (UB / EPC), ue = (rem % (UB / EPC)) * EPC;
                const int k = kb + row, e = u0 + ue;
                i32x4 v = i32x4{0, 0, 0, 0};
                if (k < D && e < D) v = *(const i32x4*)((const char*)p.R + ((((size_t)n * D + k) * G + g) * D + e) * ESZ);
                *(i32x4*)(ldsR + ((size_t)row * PR + g * UB + ue) * ESZ) = v;
            }
        }
#pragma unroll
        for (int x = 0; x < LH; ++x) {
            const int ch = tid + x * 256, col = ch / (KR / 4), k4 = (ch % (KR / 4)) * 4;
            const int m = col0 + col, k = kb + k4;
            f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
            if (m < ncols && k < D) {
                const int r = m / B, b = m - r * B;
                v = *(const f32x4*)(p.states + ((size_t)r * S * B + b) * HD + (size_t)n * D + k);   // state 0 = h, the slot before step r
            }
            if constexpr (BF16) *(i32x2*)(ldsH + ((size_t)col * PH + k4) * 2) = i32x2{(int)pack_bf16x2(v[0], v[1]), (int)pack_bf16x2(v[2], v[3])};
            else *(f32x4*)(ldsH + ((size_t)col * PH + k4) * 4) = v;
        }
        __syncthreads();
        if (u0 + w * 16 < D) {   // (a wave beyond the head's units only helps loading)
            if constexpr (BF16) {
                // quad q's 8 contraction elements of a round: rows 4q..4q+3 and 16+4q..16+4q+3, in both operands
                typedef short s16x4 __attribute__((ext_vector_type(4)));
                typedef short s16x8 __attribute__((ext_vector_type(8)));
                typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                const uint16_t* rt = (const uint16_t*)ldsR;
                const int tr_row = 4 * quad + (c >> 2), tr_col = 4 * (c & 3);
                bf16x8 hB[NCT];
#pragma unroll
                for (int j = 0; j < NCT; ++j) {
                    const char* hp = ldsH + ((size_t)(j * 16 + c) * PH) * 2;
                    const i32x2 lo = *(const i32x2*)(hp + (4 * quad) * 2), hi = *(const i32x2*)(hp + (16 + 4 * quad) * 2);
                    hB[j] = __builtin_bit_cast(bf16x8, i32x4{lo[0], lo[1], hi[0], hi[1]});
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const int cg = g * UB + w * 16 + tr_col;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(rt + tr_row * PR + cg));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(rt + (16 + tr_row) * PR + cg));
                    const bf16x8 a = __builtin_bit_cast(bf16x8, s16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
#pragma unroll
                    for (int j = 0; j < NCT; ++j) acc[g][j] = OP::mfma(a, hB[j], acc[g][j]);
                }
            } else {
#pragma unroll
                for (int kk = 0; kk < KR / 4; ++kk) {
                    float hB[NCT];
#pragma unroll
                    for (int j = 0; j < NCT; ++j) hB[j] = *(const float*)(ldsH + ((size_t)(j * 16 + c) * PH + kk * 4 + quad) * 4);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const float a = *(const float*)(ldsR + ((size_t)(kk * 4 + quad) * PR + g * UB + w * 16 + c) * 4);
#pragma unroll
                        for (int j = 0; j < NCT; ++j) acc[g][j] = OP::mfma(a, hB[j], acc[g][j]);
                    }
                }
            }
        }
    }
    // ---- point-wise function per (unit, column) pair: lane holds column c of each column tile and units 4 quad .. 4 quad + 3
    const int e0 = u0 + w * 16 + 4 * quad;
    if (e0 >= D) return;
    float bias[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) load_io<BF16, 4>(p.bias, ((size_t)n * G + g) * D + e0, bias[g]);
    constexpr uint32_t REC = RS * ESZ;
#pragma unroll
    for (int j = 0; j < NCT; ++j) {
        const int m = col0 + j * 16 + c;
        if (m >= ncols) continue;
        const int r = m / B, b = m - r * B;
        float wx[G][4], st[S][4];
#pragma unroll
        for (int g = 0; g < G; ++g) load_io<BF16, 4>(p.Wx, (((size_t)m * G + g) * NH + n) * D + e0, wx[g]);
#pragma unroll
        for (int s = 0; s < S; ++s) load_f32<4>(p.states, (((size_t)r * S + s) * B + b) * HD + (size_t)n * D + e0, st[s]);
        const rsrc_t rs_c = make_rsrc((char*)p.cache + (((size_t)m * NH + n) * D + e0) * REC);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float wxi[G], ybi[G], sti[S], cvi[NC];
#pragma unroll
            for (int g = 0; g < G; ++g) { wxi[g] = wx[g][i]; ybi[g] = acc[g][j][i] + bias[g][i]; }
#pragma unroll
            for (int s = 0; s < S; ++s) sti[s] = st[s][i];
            Cell<CELL, BF16>::fwd(wxi, ybi, sti, cvi);
            store_record<BF16, RS, NC>(rs_c, (uint32_t)i * REC, 0, cvi);
        }
    }
}

}  // namespace flashrnn
