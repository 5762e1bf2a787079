// Shared device-side definitions of the persistent forward / backward kernels (gfx950 only).
//
// Tiling vocabulary (paper App. B uses E/W/B/L per axis; ours, chosen for CDNA4):
//   - a *group* is one (head, batch tile); a batch tile holds BT <= 16 rows;
//   - a group is served by P workgroups ("members"), each owning U = 16*NWU consecutive units of
//     the head and ALL gates of those units (the gate axis is never split, so the point-wise
//     function stays in registers);
//   - inside a workgroup a wave owns 16 units (one MFMA tile row block per gate) and, when KS > 1,
//     one of KS slices of the contraction axis; partial sums of the KS slices meet in LDS;
//   - one MFMA tile is [16 units] x [16 batch slots]: the recurrent weights are the A operand (kept
//     in registers for all T steps, paper Sec. 5.2), h_{t-1} (or the gate gradients) is the B operand.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

namespace flashrnn {

enum : int { CELL_LSTM = 0, CELL_GRU = 1, CELL_SLSTM = 2, CELL_ELMAN = 3, CELL_GRU4 = 4 };
// cells whose Jacobian needs h_{t-1} itself (the z gate mixes it into h_t)
constexpr bool cell_uses_h_prev(int cell) { return cell == CELL_GRU || cell == CELL_GRU4; }

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(2 * sizeof(int)))) int i32x2;

template <int CELL> struct CellTraits;
template <> struct CellTraits<CELL_LSTM> { static constexpr int G = 4, S = 2, NC = 4, RS = 4; };
template <> struct CellTraits<CELL_GRU> { static constexpr int G = 3, S = 1, NC = 4, RS = 4; };
template <> struct CellTraits<CELL_SLSTM> { static constexpr int G = 4, S = 4, NC = 5, RS = 8; };
template <> struct CellTraits<CELL_ELMAN> { static constexpr int G = 1, S = 1, NC = 1, RS = 1; };
template <> struct CellTraits<CELL_GRU4> { static constexpr int G = 4, S = 1, NC = 4, RS = 4; };
// NC = values per (t, batch row, unit) the forward pass saves for the backward pass:
//   LSTM  sig(i), sig(f), tanh(z), sig(o)
//   GRU   sig(r), sig(z), tanh(candidate), yn = R_n h + b_n
//   sLSTM input weight exp(i - m_t), forget weight exp(log sig(f) + m_{t-1} - m_t), tanh(z), sig(o), sig(-f)
//   Elman h_t
//   GRU4  sig(z), sig(r), tanh(n + sig(r) tanh(g)), tanh(g)
// They form one record of RS >= NC elements of the I/O dtype per (t, batch row, head, unit): cache[T][B][NH][D][RS].
// RS = NC except for the sLSTM, whose five values are padded to eight: a bf16 record is then one aligned 16-byte access
// in HBM and in the LDS images (8 bytes for the four-value cells, 2 for Elman; twice that with f32 I/O).  A 12-byte
// sLSTM record was measured: its unaligned accesses cost the staged backward kernel 5 % (three 4-byte LDS reads) to 12 %
// (one 12-byte read) at D = 192, and neither sLSTM workload is bound by HBM traffic.  One record is one store in the
// forward pass and one load in the backward pass.
__host__ __device__ constexpr int record_slots(int cell) { return cell == CELL_SLSTM ? 8 : cell == CELL_ELMAN ? 1 : 4; }

// Row pitch (bytes) of an LDS row image whose rows hold `row_bytes` of data: padded so that
// consecutive rows start 16 banks (64 bytes) apart modulo the 64 banks, which keeps the 4-rows x
// 16-units access pattern of a wave free of bank conflicts.
__host__ __device__ inline uint32_t lds_row_pitch(uint32_t row_bytes) {
    const uint32_t dw = row_bytes / 4;
    return (dw + (16u + 64u - dw % 64u) % 64u) * 4u;
}

// LDS layout of the forward tile kernel (bf16 I/O, one workgroup per group, BT < 16), shared by the kernel
// and by the host code that sizes the dynamic LDS.  NT threads; every thread moves NCH 16-byte chunks
// of each image per step, threads without a real chunk own a private pad chunk behind the image.
struct TileLds {
    uint32_t hp;                              // operand row pitch (bytes), buf = BT * hp
    uint32_t rp_io, rp_st;                    // image row pitches: bf16 rows, f32 rows
    uint32_t in_bytes, in_pitch;              // inputs Wx (BT*G rows)
    uint32_t st_bytes, st_pitch;              // f32 state rows
    uint32_t total_fwd;
};
__host__ __device__ inline uint32_t div_up(uint32_t a, uint32_t b) { return (a + b - 1) / b; }
__host__ __device__ inline TileLds tile_lds(int BT, int G, int S, int D, int NT, int k_bytes_fwd) {
    TileLds L;
    const uint32_t nt16 = (uint32_t)NT * 16;
    L.rp_io = lds_row_pitch((uint32_t)D * 2);
    L.rp_st = lds_row_pitch((uint32_t)D * 4);
    L.in_bytes = (uint32_t)BT * G * L.rp_io;
    L.in_pitch = L.in_bytes + div_up((uint32_t)BT * G * (D / 8), NT) * nt16;
    L.st_bytes = (uint32_t)BT * S * L.rp_st;
    L.st_pitch = L.st_bytes + div_up((uint32_t)BT * S * (D / 4), NT) * nt16;
    L.hp = lds_row_pitch((uint32_t)k_bytes_fwd);
    L.total_fwd = 2 * BT * L.hp + 2 * L.in_pitch + 2 * L.st_pitch;
    return L;
}

// LDS layout of the backward tile kernel (bf16 I/O, one workgroup per group, BT < 16, NT = 4 * D threads).
// The input images are filled by loads that write LDS directly: a wave's 64 chunks of 16 bytes land
// back to back, so these images are plain arrays of chunks (no row padding), each rounded up to whole waves.
struct TileLdsBwd {
    uint32_t hp;                 // operand (gate-gradient) row pitch, buf = BT * hp, two buffers
    uint32_t rp_io;              // row pitch of the output image (bf16 rows)
    uint32_t red_off;            // partial sums of the contraction slices
    uint32_t in_off, in_pitch;   // two input images: records | state rows | dh rows
    uint32_t st_off, dh_off;     // ... offsets of the state rows and the dh rows inside an input image
    uint32_t out_off, out_pitch; // two output images: BT * GO bf16 rows
    uint32_t total;
};
__host__ __device__ inline uint32_t round_up(uint32_t a, uint32_t b) { return (a + b - 1) / b * b; }
__host__ __device__ inline TileLdsBwd tile_lds_bwd(int BT, int GO, int NSB, int D, int k_bytes, int EBK, int rec_bytes) {
    TileLdsBwd L;
    const uint32_t NT = 4u * (uint32_t)D, PP = (uint32_t)BT / 4u;
    L.hp = lds_row_pitch((uint32_t)k_bytes);
    L.rp_io = lds_row_pitch((uint32_t)D * 2);
    L.red_off = 2u * BT * L.hp;
    const uint32_t red_bytes = EBK > 1 ? (NT / 64u) * EBK * 64u * PP * 4u : 0u;
    L.in_off = L.red_off + red_bytes;
    L.st_off = round_up((uint32_t)BT * D * (uint32_t)rec_bytes, 1024u);
    L.dh_off = L.st_off + round_up((uint32_t)BT * NSB * D * 4u, 1024u);
    L.in_pitch = L.dh_off + round_up((uint32_t)BT * D * 2u, 1024u);
    L.out_off = L.in_off + 2u * L.in_pitch;
    L.out_pitch = (uint32_t)BT * GO * L.rp_io;
    L.total = L.out_off + 2u * L.out_pitch;
    return L;
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Cache policy bits of the raw buffer intrinsics on gfx942/gfx950.
constexpr int kAuxAgent = 16;  // sc1: coherent at agent scope (misses the CU's vector L1)

// per-phase clock sums of a trace build: [workgroup][kTraceWaves][kTracePhases]
constexpr int kTracePhases = 8, kTraceWaves = 16;

struct KernelParams {
    const void* Wx;        // fwd: [T,B,G,NH,D] io
    const void* R;         // [NH,D,G,D] io
    const void* bias;      // [NH,G,D] io
    const float* states0;  // fwd: [S,B,NH,D] or null
    float* states;         // [T+1,S,B,NH,D]
    void* cache;           // [T,B,NH,D,RS] io dtype (RS = record_slots(cell)), may be null in fwd
    const void* dH;        // bwd: [T,B,NH,D] io
    const float* dlast;    // bwd: [S,B,NH,D] or null
    void* dWx;             // bwd: [T,B,G,NH,D] io
    void* dgn;             // bwd, GRU: recurrent-side gradient of gate n, [T,B,NH,D] io
    float* dstates0;       // bwd: [S,B,NH,D]
    float* db_part;        // bwd: [B,NH,G,D] per-batch-row partial sums of db
    uint32_t* exch;        // cross-CU exchange buffer (stamped words)
    int* err;              // error word
    int T, B, NH, D;
    int P;                 // workgroups per group
    int NWU;               // unit waves per workgroup (each 16 units)
    int NG;                // groups in total: NH * batch tiles; group id = tile * NH + head
    int GPAR;              // groups processed concurrently; a workgroup set loops over NG / GPAR of them
    int spin_limit;
    int db_accumulate;     // bwd: add this launch's per-row db sums to what db_part holds (windowed backward pass)
    int spread;            // several workgroups per group: 0 = a group's members share an XCD, 1 = they are spread over all XCDs
    unsigned long long* trace;   // per-phase clock sums [workgroup][16 waves][8 phases] (trace builds only), or null
    float clip;            // bwd: bound of the recurrent gradient term per value (+inf = not clipped, 0 = cut)
};

// ---------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t u16) { return __builtin_bit_cast(float, u16 << 16); }

// f32 -> bf16, round to nearest even: one v_cvt_pk_bf16_f32 on gfx950
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Point-wise math in two flavours: FAST (bf16 I/O: hardware exp2/log2/rcp, ~1e-6 relative) and
// accurate (f32 I/O: library functions, needed for 1e-5 agreement with the fp64 oracle).
template <bool FAST> __device__ __forceinline__ float sigm(float x) {
    if constexpr (FAST) return fast_rcp(1.0f + fast_exp2(-kLog2e * x));
    else return 1.0f / (1.0f + expf(-x));
}
template <bool FAST> __device__ __forceinline__ float tanh_(float x) {
    if constexpr (FAST) return 1.0f - 2.0f * fast_rcp(1.0f + fast_exp2((2.0f * kLog2e) * x));
    else return tanhf(x);
}
template <bool FAST> __device__ __forceinline__ float exp_(float x) {
    if constexpr (FAST) return fast_exp2(kLog2e * x);
    else return expf(x);
}

// DPP row shift right by N lanes inside each row of 16 lanes, written only to the lanes of the
// banks in BANKS (bank k = lanes 4k..4k+3 of every row); other lanes keep `old`.
template <int N, int BANKS> __device__ __forceinline__ float dpp_row_shr(float old, float src) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, src),
                                                                 0x110 + N, 0xF, BANKS, false));
}

// MFMA output of one [16 units] x [16 batch slots] tile: lane (c = lane%16, q = lane/16) holds batch
// slot c and units 4q..4q+3.  With fewer than 16 valid batch slots the idle lanes take over part of
// the units of the busy ones, so that the point-wise work is spread over all 64 lanes:
//   BT = 16: PP = 4 pairs per lane, unit offset 4q + i
//   BT = 8 : lanes c >= 8 take units 4q+2, 4q+3 of batch slot c-8;       PP = 2, offset 4q + 2(c/8) + i
//   BT = 4 : lanes c in [4k, 4k+4) take unit 4q+k of batch slot c%4;     PP = 1, offset 4q + c/4
template <int BT> __device__ __forceinline__ void compact_tile(f32x4& a) {
    if constexpr (BT == 8) {
        a[0] = dpp_row_shr<8, 0xC>(a[0], a[2]);
        a[1] = dpp_row_shr<8, 0xC>(a[1], a[3]);
    } else if constexpr (BT == 4) {
        a[0] = dpp_row_shr<4, 0x2>(a[0], a[1]);
        a[0] = dpp_row_shr<8, 0x4>(a[0], a[2]);
        a[0] = dpp_row_shr<12, 0x8>(a[0], a[3]);
    }
}

// The inverse of compact_tile for one value per pair: the lanes c < BT of a row collect the four consecutive
// units 4q..4q+3 of their batch slot from the lanes that computed them (valid in those lanes only).
template <int BT, int PP> __device__ __forceinline__ void expand_tile(const float (&v)[PP], float (&out)[4]) {
    auto shl = [](float x, auto n) {   // lane i takes the value of lane i + n of its row
        constexpr int N = decltype(n)::value;
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x100 + N, 0xF, 0xF, false));
    };
    if constexpr (BT == 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = v[i];
    } else if constexpr (BT == 8) {
        out[0] = v[0]; out[1] = v[1];
        out[2] = shl(v[0], std::integral_constant<int, 8>{});
        out[3] = shl(v[1], std::integral_constant<int, 8>{});
    } else {
        out[0] = v[0];
        out[1] = shl(v[0], std::integral_constant<int, 4>{});
        out[2] = shl(v[0], std::integral_constant<int, 8>{});
        out[3] = shl(v[0], std::integral_constant<int, 12>{});
    }
}

// typed I/O of PP consecutive elements (io dtype bf16 or f32), PP in {1, 2, 4}
template <bool BF16, int PP> __device__ __forceinline__ void load_io(const void* base, size_t idx, float (&out)[PP]) {
    if constexpr (BF16) {
        const uint16_t* p = (const uint16_t*)base + idx;
        if constexpr (PP == 4) {
            uint2 v = *(const uint2*)p;
            out[0] = bf16_bits_to_f32(v.x & 0xFFFFu); out[1] = __builtin_bit_cast(float, v.x & 0xFFFF0000u);
            out[2] = bf16_bits_to_f32(v.y & 0xFFFFu); out[3] = __builtin_bit_cast(float, v.y & 0xFFFF0000u);
        } else if constexpr (PP == 2) {
            uint32_t v = *(const uint32_t*)p;
            out[0] = bf16_bits_to_f32(v & 0xFFFFu); out[1] = __builtin_bit_cast(float, v & 0xFFFF0000u);
        } else {
            out[0] = bf16_bits_to_f32(*p);
        }
    } else {
        const float* p = (const float*)base + idx;
        if constexpr (PP == 4) { float4 v = *(const float4*)p; out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w; }
        else if constexpr (PP == 2) { float2 v = *(const float2*)p; out[0] = v.x; out[1] = v.y; }
        else out[0] = *p;
    }
}

template <bool BF16, int PP> __device__ __forceinline__ void store_io(void* base, size_t idx, const float (&v)[PP]) {
    if constexpr (BF16) {
        uint16_t* p = (uint16_t*)base + idx;
        if constexpr (PP == 4) {
            uint2 o;
            o.x = pack_bf16x2(v[0], v[1]);
            o.y = pack_bf16x2(v[2], v[3]);
            *(uint2*)p = o;
        } else if constexpr (PP == 2) {
            *(uint32_t*)p = pack_bf16x2(v[0], v[1]);
        } else {
            *p = (uint16_t)f32_to_bf16_bits(v[0]);
        }
    } else {
        float* p = (float*)base + idx;
        if constexpr (PP == 4) *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
        else if constexpr (PP == 2) *(float2*)p = make_float2(v[0], v[1]);
        else *p = v[0];
    }
}

// Per-step streams go through buffer instructions: a resource built from a uniform pointer (advanced
// per step on the scalar unit), a loop-invariant 32-bit lane offset and a scalar offset.  No vector
// address arithmetic and no 64-bit pointer registers in the time loop.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* p) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, 0x7FFFFFFF, 0x00020000);
}
template <bool BF16, int PP> __device__ __forceinline__ void load_io_r(rsrc_t r, uint32_t voff, uint32_t soff, float (&out)[PP]) {
    if constexpr (BF16) {
        if constexpr (PP == 4) {
            const i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
            out[0] = bf16_bits_to_f32((uint32_t)v[0] & 0xFFFFu); out[1] = __builtin_bit_cast(float, (uint32_t)v[0] & 0xFFFF0000u);
            out[2] = bf16_bits_to_f32((uint32_t)v[1] & 0xFFFFu); out[3] = __builtin_bit_cast(float, (uint32_t)v[1] & 0xFFFF0000u);
        } else if constexpr (PP == 2) {
            const uint32_t v = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
            out[0] = bf16_bits_to_f32(v & 0xFFFFu); out[1] = __builtin_bit_cast(float, v & 0xFFFF0000u);
        } else {
            out[0] = bf16_bits_to_f32((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0));
        }
    } else {
        if constexpr (PP == 4) {
            const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
            out[0] = v[0]; out[1] = v[1]; out[2] = v[2]; out[3] = v[3];
        } else if constexpr (PP == 2) {
            const i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
            const int a = v[0], b = v[1];
            out[0] = __builtin_bit_cast(float, a); out[1] = __builtin_bit_cast(float, b);
        } else {
            out[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
        }
    }
}
template <bool BF16, int PP> __device__ __forceinline__ void store_io_r(rsrc_t r, uint32_t voff, uint32_t soff, const float (&v)[PP]) {
    if constexpr (BF16) {
        if constexpr (PP == 4) __builtin_amdgcn_raw_buffer_store_b64(i32x2{(int)pack_bf16x2(v[0], v[1]), (int)pack_bf16x2(v[2], v[3])}, r, voff, soff, 0);
        else if constexpr (PP == 2) __builtin_amdgcn_raw_buffer_store_b32(pack_bf16x2(v[0], v[1]), r, voff, soff, 0);
        else __builtin_amdgcn_raw_buffer_store_b16((unsigned short)f32_to_bf16_bits(v[0]), r, voff, soff, 0);
    } else {
        if constexpr (PP == 4) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i32x4, f32x4{v[0], v[1], v[2], v[3]}), r, voff, soff, 0);
        else if constexpr (PP == 2) __builtin_amdgcn_raw_buffer_store_b64(i32x2{__builtin_bit_cast(int, v[0]), __builtin_bit_cast(int, v[1])}, r, voff, soff, 0);
        else __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v[0]), r, voff, soff, 0);
    }
}

// 16 bytes per lane from global memory straight into LDS, without passing through registers: lane l's
// chunk lands at lds + 16 * l (lds is wave-uniform), read from byte offset voff of resource r (out of
// range: zeros land).  Completion counts in vmcnt like any load.  The host pass only needs the declaration.
__device__ __forceinline__ void load_chunk_to_lds(rsrc_t r, char* lds, uint32_t voff) {
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(3))) char lds_char;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_char*)lds, 16, voff, 0, 0, 0);
#else
    (void)r; (void)lds; (void)voff;
#endif
}

// One saved-values record (NC values, padded with zeros to RS slots) at byte offset voff + soff of resource r:
// RS elements of the I/O dtype, moved by the widest instructions that tile its 2 .. 32 bytes.
typedef __attribute__((__vector_size__(3 * sizeof(int)))) int i32x3;
template <int NW> struct RecordWords { uint32_t w[NW]; };   // a record as 32-bit words (NW = 0: one 16-bit element in w0)
template <bool BF16, int RS, int NC> __device__ __forceinline__ void pack_record(const float (&v)[NC], uint32_t (&w)[(BF16 ? (RS + 1) / 2 : RS)]) {
    float x[RS + 1];
#pragma unroll
    for (int j = 0; j < RS + 1; ++j) x[j] = j < NC ? v[j] : 0.0f;
    if constexpr (BF16) {
#pragma unroll
        for (int j = 0; j < (RS + 1) / 2; ++j) w[j] = pack_bf16x2(x[2 * j], x[2 * j + 1]);
    } else {
#pragma unroll
        for (int j = 0; j < RS; ++j) w[j] = __builtin_bit_cast(uint32_t, x[j]);
    }
}
template <bool BF16, int RS, int NC> __device__ __forceinline__ void unpack_words(const uint32_t (&w)[(BF16 ? (RS + 1) / 2 : RS)], float (&v)[NC]) {
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        if constexpr (BF16) v[j] = (j & 1) ? __builtin_bit_cast(float, w[j / 2] & 0xFFFF0000u) : bf16_bits_to_f32(w[j / 2] & 0xFFFFu);
        else v[j] = __builtin_bit_cast(float, w[j]);
    }
}
template <bool BF16, int RS, int NC> __device__ __forceinline__ void store_record(rsrc_t r, uint32_t voff, uint32_t soff, const float (&v)[NC]) {
    constexpr int NW = BF16 ? (RS + 1) / 2 : RS;
    uint32_t w[NW];
    pack_record<BF16, RS, NC>(v, w);
    if constexpr (BF16 && RS == 1) __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(w[0] & 0xFFFFu), r, voff, soff, 0);
    else if constexpr (NW == 1) __builtin_amdgcn_raw_buffer_store_b32(w[0], r, voff, soff, 0);
    else if constexpr (NW == 2) __builtin_amdgcn_raw_buffer_store_b64(i32x2{(int)w[0], (int)w[1]}, r, voff, soff, 0);
    else if constexpr (NW == 3) __builtin_amdgcn_raw_buffer_store_b96(i32x3{(int)w[0], (int)w[1], (int)w[2]}, r, voff, soff, 0);
    else if constexpr (NW == 4) __builtin_amdgcn_raw_buffer_store_b128(i32x4{(int)w[0], (int)w[1], (int)w[2], (int)w[3]}, r, voff, soff, 0);
    else {
        static_assert(NW == 8, "record sizes: 1, 2, 3, 4 or 8 dwords");
        __builtin_amdgcn_raw_buffer_store_b128(i32x4{(int)w[0], (int)w[1], (int)w[2], (int)w[3]}, r, voff, soff, 0);
        __builtin_amdgcn_raw_buffer_store_b128(i32x4{(int)w[4], (int)w[5], (int)w[6], (int)w[7]}, r, voff + 16, soff, 0);
    }
}
template <bool BF16, int RS, int NC> __device__ __forceinline__ void load_record(rsrc_t r, uint32_t voff, uint32_t soff, float (&v)[NC]) {
    constexpr int NW = BF16 ? (RS + 1) / 2 : RS;
    uint32_t w[NW];
    if constexpr (BF16 && RS == 1) w[0] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    else if constexpr (NW == 1) w[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
    else if constexpr (NW == 2) { const i32x2 x = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0); w[0] = (uint32_t)x[0]; w[1] = (uint32_t)x[1]; }
    else if constexpr (NW == 3) { const i32x3 x = __builtin_amdgcn_raw_buffer_load_b96(r, voff, soff, 0); w[0] = (uint32_t)x[0]; w[1] = (uint32_t)x[1]; w[2] = (uint32_t)x[2]; }
    else if constexpr (NW == 4) { const i32x4 x = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0); w[0] = (uint32_t)x[0]; w[1] = (uint32_t)x[1]; w[2] = (uint32_t)x[2]; w[3] = (uint32_t)x[3]; }
    else {
        static_assert(NW == 8, "record sizes: 1, 2, 3, 4 or 8 dwords");
        const i32x4 x = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
        const i32x4 y = __builtin_amdgcn_raw_buffer_load_b128(r, voff + 16, soff, 0);
        w[0] = (uint32_t)x[0]; w[1] = (uint32_t)x[1]; w[2] = (uint32_t)x[2]; w[3] = (uint32_t)x[3];
        w[4] = (uint32_t)y[0]; w[5] = (uint32_t)y[1]; w[6] = (uint32_t)y[2]; w[7] = (uint32_t)y[3];
    }
    unpack_words<BF16, RS, NC>(w, v);
}
// a bf16 record out of an LDS image (4-byte aligned, 2-byte aligned for the one-element record)
template <int RS, int NC> __device__ __forceinline__ void take_record_lds(const char* p, float (&v)[NC]) {
    constexpr int NW = (RS + 1) / 2;
    uint32_t w[NW];
    typedef int i32x2_a4 __attribute__((ext_vector_type(2), aligned(4)));
    typedef int i32x3_a4 __attribute__((ext_vector_type(3), aligned(4)));
    if constexpr (RS == 1) w[0] = *(const uint16_t*)p;
    else if constexpr (NW == 2) { const i32x2_a4 x = *(const i32x2_a4*)p; w[0] = (uint32_t)x.x; w[1] = (uint32_t)x.y; }
    else if constexpr (NW == 3) { const i32x3_a4 x = *(const i32x3_a4*)p; w[0] = (uint32_t)x.x; w[1] = (uint32_t)x.y; w[2] = (uint32_t)x.z; }
    else if constexpr (NW == 4) { const i32x4 x = *(const i32x4*)p; w[0] = (uint32_t)x[0]; w[1] = (uint32_t)x[1]; w[2] = (uint32_t)x[2]; w[3] = (uint32_t)x[3]; }
    else {
#pragma unroll
        for (int j = 0; j < NW; ++j) w[j] = ((const uint32_t*)p)[j];
    }
    unpack_words<true, RS, NC>(w, v);
}

template <int PP> __device__ __forceinline__ void load_f32(const float* base, size_t idx, float (&out)[PP]) {
    load_io<false, PP>(base, idx, out);
}
template <int PP> __device__ __forceinline__ void store_f32(float* base, size_t idx, const float (&v)[PP]) {
    store_io<false, PP>(base, idx, v);
}

// Operand type of one MFMA k-step: 8 bf16 (v_mfma_f32_16x16x32_bf16) or one float (v_mfma_f32_16x16x4_f32).
template <bool BF16> struct Operand;
template <> struct Operand<true> {
    using type = bf16x8;
    static constexpr int KPL = 8;   // contraction elements per lane per k-step
    static constexpr int KSTEP = 32;
    static __device__ __forceinline__ f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Operand<false> {
    using type = float;
    static constexpr int KPL = 1;
    static constexpr int KSTEP = 4;
    static __device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
};

// Contraction index held by (k-step kt, lane quad q, element j) of a wave whose slice starts at k0.
// The assignment is free as long as both MFMA operands use the same one; this one makes the KPL*KT
// elements of a lane... (bf16) 8 consecutive per k-step, (f32) KT consecutive per lane.
template <bool BF16, int KT> __device__ __forceinline__ int k_index(int k0, int kt, int q, int j) {
    if constexpr (BF16) return k0 + kt * 32 + q * 8 + j;
    else return k0 + q * KT + kt;
}

}  // namespace flashrnn
