// Backward pass without a saved-values buffer: the values the forward pass would have written out for the backward pass
// (Alg. 1, "write out gates for backward pass") are formed again from Wx, R, b and the stored states, a window of time
// steps at a time.  Every h_{t-1} is in `states`, so inside a window nothing is sequential: the pre-activations
//     g_t = Wx_t + R^T h_{t-1} + b            (Sec. 3, eq. (1))
// of all steps of the window are one dense contraction per head, [G*D gate columns] x [window steps * batch rows] over D,
// and the point-wise function (App. A) applied to (g_t, s_{t-1}) gives the same record the forward kernel stores.
// The persistent backward kernel then runs over the window as usual, with the gradients of the carried states handed
// from window to window.
//
// Tile of one workgroup (4 waves): 64 units x all G gates x 128 columns (a column = one (step, batch row) pair); a wave owns
// 16 units and, like the forward kernel, all gates of them, so that its G accumulators of a column tile hold the G
// pre-activations of a (unit, column) pair in the same lane and the point-wise function runs in registers.
// R[n][d][g][e] has the contraction index d as its slow axis and the units contiguous: its tile goes to LDS as it is and
// the A operands are read with the transposing LDS load (bf16) or element-wise (f32); h is converted to the I/O dtype and
// laid out [column][d].
#pragma once
#include "flashrnn_kernels.h"

namespace flashrnn {

constexpr int kRecomputeCols = 128;   // columns (step, batch row) per workgroup

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
    constexpr int UB = 64, CB = kRecomputeCols, KR = 32;   // units, columns per workgroup; contraction rows per round
    constexpr int NCT = CB / 16;                         // column tiles per wave
    constexpr int PR = G * UB + (BF16 ? 16 : 8);         // LDS row pitch of the R tile (elements): see the dR GEMM for the bf16 choice
    constexpr int PH = KR + (BF16 ? 8 : 4);              // LDS row pitch of the h tile (elements)
    // LDS: the operand tiles of the contraction (two buffers each: one barrier per round), and behind the contraction, in the
    // same memory, the staging tiles of the point-wise phase: inputs, states and records of 16 columns at a time.
    constexpr uint32_t REC = RS * ESZ;
    constexpr uint32_t kTileR = KR * PR * ESZ, kTileH = CB * PH * ESZ;
    constexpr uint32_t PWX = G * UB * ESZ + 32, PST = S * UB * 4 + 64, PRC = UB * REC + 16;   // pitches per column of the staging tiles (bytes)
    constexpr uint32_t kMain = 2 * kTileR + 2 * kTileH, kStage = 16 * (PWX + PST + PRC);
    __shared__ __align__(16) char lds_all[kMain > kStage ? kMain : kStage];
    auto ldsR = [&](int b2) { return lds_all + (uint32_t)b2 * kTileR; };
    auto ldsH = [&](int b2) { return lds_all + 2 * kTileR + (uint32_t)b2 * kTileH; };
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

    // ---- loader roles (16-byte chunks), fixed per thread; a round's chunks wait in registers while the round before is
    // multiplied (the loads of round r+1 are issued before the MFMAs of round r).
    // R tile: KR rows x G gates x UB units; h tile: CB columns x KR contraction elements (f32 in memory).
    constexpr int EPC = 16 / ESZ;                        // elements per chunk of the I/O dtype
    constexpr int R_CH = KR * G * UB / EPC, LR = (R_CH + 255) / 256;
    constexpr int H_CH = CB * KR / 4, LH = H_CH / 256;   // chunks of 4 floats
    static_assert(H_CH % 256 == 0, "h loader tiling");
    const char* r_src[LR];
    uint32_t r_lds[LR];
    int r_row[LR];
    bool r_ok[LR];
#pragma unroll
    for (int x = 0; x < LR; ++x) {
        const int ch = tid + x * 256;
        const int row = ch / (G * UB / EPC), rem = ch % (G * UB / EPC), g = rem / (UB / EPC), ue = (rem % (UB / EPC)) * EPC;
        r_row[x] = row;
        r_ok[x] = ch < R_CH && u0 + ue < D;
        r_src[x] = (const char*)p.R + ((((size_t)n * D + row) * G + g) * D + u0 + ue) * ESZ;   // + kb * G * D * ESZ per round
        r_lds[x] = (uint32_t)(((size_t)row * PR + g * UB + ue) * ESZ);
    }
    const float* h_src[LH];
    uint32_t h_lds[LH];
    int h_k[LH];
    bool h_ok[LH];
#pragma unroll
    for (int x = 0; x < LH; ++x) {
        const int ch = tid + x * 256, col = ch / (KR / 4), k4 = (ch % (KR / 4)) * 4;
        const int m = col0 + col;
        const int r = m / B, b = m - r * B;
        h_k[x] = k4;
        h_ok[x] = m < ncols;
        h_src[x] = p.states + ((size_t)(h_ok[x] ? r : 0) * S * B + (h_ok[x] ? b : 0)) * HD + (size_t)n * D + k4;   // state 0 = h, the slot before step r
        h_lds[x] = (uint32_t)(((size_t)col * PH + k4) * ESZ);
    }
    i32x4 rr[LR];
    f32x4 hr[LH];
    auto load_round = [&](int kb) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < LR; ++x) {
            rr[x] = i32x4{0, 0, 0, 0};
            if (r_ok[x] && kb + r_row[x] < D) rr[x] = *(const i32x4*)(r_src[x] + (size_t)kb * G * D * ESZ);
        }
#pragma unroll
        for (int x = 0; x < LH; ++x) {
            hr[x] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (h_ok[x] && kb + h_k[x] < D) hr[x] = *(const f32x4*)(h_src[x] + kb);
        }
    };
    auto park_round = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int x = 0; x < LR; ++x)
            if (tid + x * 256 < R_CH) *(i32x4*)(ldsR(buf) + r_lds[x]) = rr[x];
#pragma unroll
        for (int x = 0; x < LH; ++x) {
            if constexpr (BF16) *(i32x2*)(ldsH(buf) + h_lds[x]) = i32x2{(int)pack_bf16x2(hr[x][0], hr[x][1]), (int)pack_bf16x2(hr[x][2], hr[x][3])};
            else *(f32x4*)(ldsH(buf) + h_lds[x]) = hr[x];
        }
    };
    load_round(0);
    int buf = 0;
    for (int kb = 0; kb < D; kb += KR, buf ^= 1) {
        park_round(buf);   // (the buffer was last read two rounds ago: the barrier of the round before lies in between)
        __syncthreads();
        if (kb + KR < D) load_round(kb + KR);
        if (u0 + w * 16 < D) {   // (a wave beyond the head's units only helps loading)
            if constexpr (BF16) {
                // quad q's 8 contraction elements of a round: rows 4q..4q+3 and 16+4q..16+4q+3, in both operands
                typedef short s16x4 __attribute__((ext_vector_type(4)));
                typedef short s16x8 __attribute__((ext_vector_type(8)));
                typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                const uint16_t* rt = (const uint16_t*)ldsR(buf);
                const int tr_row = 4 * quad + (c >> 2), tr_col = 4 * (c & 3);
                bf16x8 hB[NCT];
#pragma unroll
                for (int j = 0; j < NCT; ++j) {
                    const char* hp = ldsH(buf) + ((size_t)(j * 16 + c) * PH) * 2;
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
                    for (int j = 0; j < NCT; ++j) hB[j] = *(const float*)(ldsH(buf) + ((size_t)(j * 16 + c) * PH + kk * 4 + quad) * 4);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const float a = *(const float*)(ldsR(buf) + ((size_t)(kk * 4 + quad) * PR + g * UB + w * 16 + c) * 4);
#pragma unroll
                        for (int j = 0; j < NCT; ++j) acc[g][j] = OP::mfma(a, hB[j], acc[g][j]);
                    }
                }
            }
        }
    }
    // ---- point-wise function per (unit, column) pair: lane holds column c of each column tile and units 4 quad .. 4 quad + 3.
    // In memory the units of a column are contiguous and the columns far apart: lanes that fetched their own four units of
    // their own column touched 16 cache lines per instruction for 32 bytes each (the kernel ran at a tenth of the memory
    // bandwidth).  So the workgroup moves whole rows: for 16 columns at a time the inputs Wx, the states and, on the way out, the
    // records go through LDS tiles, 16 bytes per thread and instruction, rows of 128 bytes and more.
    __syncthreads();   // the operand tiles are done with: their memory holds the staging tiles from here on
    char* const wx_t = lds_all;
    char* const st_t = lds_all + 16 * PWX;
    char* const rc_t = st_t + 16 * PST;
    const int ul = w * 16 + 4 * quad, e0 = u0 + ul;
    float bias[G][4];
    if (e0 < D) {
#pragma unroll
        for (int g = 0; g < G; ++g) load_io<BF16, 4>(p.bias, ((size_t)n * G + g) * D + e0, bias[g]);
    }
    // chunk roles of the three tiles (fixed per thread; the column advances by 16 per tile)
    constexpr int CWX = UB * ESZ / 16, NWX = 16 * G * CWX, LWX = (NWX + 255) / 256;   // chunks per (column, gate) row
    constexpr int CST = UB * 4 / 16, NST = 16 * S * CST, LST = (NST + 255) / 256;
    constexpr int CRC = UB * REC / 16, NRC = 16 * CRC, LRC = (NRC + 255) / 256;
    static_assert((UB * REC) % 16 == 0, "record rows are whole chunks");
    const int adv_q = 16 / B, adv_r = 16 % B;
    auto col_of = [&](int cc, int& r, int& b) { const int m = col0 + cc; r = m / B; b = m - r * B; };
    int wx_cc[LWX], st_cc[LST], st_r[LST], st_b[LST], rc_cc[LRC];
    uint32_t wx_in[LWX], wx_l[LWX], st_in[LST], st_l[LST], rc_in[LRC], rc_l[LRC];   // byte offset inside a column's row / in the tile
    bool wx_u[LWX], st_u[LST], rc_u[LRC];                                          // the chunk's units exist
#pragma unroll
    for (int x = 0; x < LWX; ++x) {
        const int ch = tid + x * 256, row = ch / CWX, part = ch % CWX, cc = row / G, g = row % G;
        wx_cc[x] = cc;
        wx_u[x] = ch < NWX && u0 + part * (16 / ESZ) < D;
        wx_in[x] = (uint32_t)(((size_t)g * NH * D + u0) * ESZ) + part * 16;   // + ((m * G) * NH + n) * D * ESZ
        wx_l[x] = cc * PWX + (g * UB) * ESZ + part * 16;
    }
#pragma unroll
    for (int x = 0; x < LST; ++x) {
        const int ch = tid + x * 256, row = ch / CST, part = ch % CST, cc = row / S, s2 = row % S;
        st_cc[x] = cc;
        col_of(cc, st_r[x], st_b[x]);
        st_u[x] = ch < NST && u0 + part * 4 < D;
        st_in[x] = (uint32_t)s2;                                              // state index; the address is formed per tile
        st_l[x] = cc * PST + (s2 * UB) * 4 + part * 16;
        st_in[x] |= (uint32_t)part << 8;
    }
#pragma unroll
    for (int x = 0; x < LRC; ++x) {
        const int ch = tid + x * 256, cc = ch / CRC, part = ch % CRC;
        rc_cc[x] = cc;
        rc_u[x] = ch < NRC && u0 + (part * 16) / (int)REC < D;
        rc_in[x] = part * 16;
        rc_l[x] = cc * PRC + part * 16;
    }
#pragma unroll
    for (int j = 0; j < NCT; ++j) {
        const int mbase = col0 + j * 16;
        // ---- inputs and states of the 16 columns into their tiles
#pragma unroll
        for (int x = 0; x < LWX; ++x) {
            const int m = mbase + wx_cc[x];
            i32x4 v = i32x4{0, 0, 0, 0};
            if (wx_u[x] && m < ncols) v = *(const i32x4*)((const char*)p.Wx + (((size_t)m * G) * NH + n) * D * ESZ + wx_in[x]);
            if (tid + x * 256 < NWX) *(i32x4*)(wx_t + wx_l[x]) = v;
        }
#pragma unroll
        for (int x = 0; x < LST; ++x) {
            const int m = mbase + st_cc[x], s2 = (int)(st_in[x] & 0xFF), part = (int)(st_in[x] >> 8);
            i32x4 v = i32x4{0, 0, 0, 0};
            if (st_u[x] && m < ncols)
                v = *(const i32x4*)(p.states + (((size_t)st_r[x] * S + s2) * B + st_b[x]) * HD + (size_t)n * D + u0 + part * 4);
            if (tid + x * 256 < NST) *(i32x4*)(st_t + st_l[x]) = v;
            st_b[x] += adv_r; st_r[x] += adv_q;                                // the next tile's column: 16 further
            if (st_b[x] >= B) { st_b[x] -= B; st_r[x] += 1; }
        }
        __syncthreads();
        // ---- this lane's four (unit, column) pairs
        if (e0 < D) {
            float wx[G][4], st[S][4];
#pragma unroll
            for (int g = 0; g < G; ++g) load_io<BF16, 4>(wx_t + c * PWX + (g * UB + ul) * ESZ, 0, wx[g]);
#pragma unroll
            for (int s2 = 0; s2 < S; ++s2) load_f32<4>((const float*)(st_t + c * PST + (s2 * UB + ul) * 4), 0, st[s2]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float wxi[G], ybi[G], sti[S], cvi[NC];
#pragma unroll
                for (int g = 0; g < G; ++g) { wxi[g] = wx[g][i]; ybi[g] = acc[g][j][i] + bias[g][i]; }
#pragma unroll
                for (int s2 = 0; s2 < S; ++s2) sti[s2] = st[s2][i];
                Cell<CELL, BF16>::fwd(wxi, ybi, sti, cvi);
                constexpr int NW = BF16 ? (RS + 1) / 2 : RS;
                uint32_t wd[NW];
                pack_record<BF16, RS, NC>(cvi, wd);
                char* dst = rc_t + c * PRC + (ul + i) * REC;
                if constexpr (REC == 2) *(uint16_t*)dst = (uint16_t)(wd[0] & 0xFFFFu);
                else {
#pragma unroll
                    for (int q2 = 0; q2 < NW; ++q2) ((uint32_t*)dst)[q2] = wd[q2];
                }
            }
        }
        __syncthreads();
        // ---- the records of the 16 columns out, row by row
#pragma unroll
        for (int x = 0; x < LRC; ++x) {
            const int m = mbase + rc_cc[x];
            if (tid + x * 256 < NRC && rc_u[x] && m < ncols)
                *(i32x4*)((char*)p.cache + (((size_t)m * NH + n) * D + u0) * REC + rc_in[x]) = *(const i32x4*)(rc_t + rc_l[x]);
        }
        // (the next tile's loads write wx_t / st_t, which every lane has read before the barrier above; rc_t is written
        // again only behind the next tile's first barrier)
    }
}

}  // namespace flashrnn
