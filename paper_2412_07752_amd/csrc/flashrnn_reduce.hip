// Weight-gradient reduction after the backward time loop (paper Sec. 4 eq. (6)-(7)):
//     dR[n,d,g,e] = sum_{t,b} h_{t-1}[b,n,d] * dg_t[b,g,n,e]        db[n,g,e] = sum_{t,b} dg_t[b,g,n,e]
// dR is one GEMM per head with the (t,b) axis contracted: M = D, N = G*D, K = T*B.  It is the one
// dense, MFMA-bound contraction of the method and runs outside the sequential loop.  Both operands
// have the contraction axis as their slow memory axis, so tiles are transposed through LDS.
// Split-K partial sums are written separately and added in a fixed order (no float atomics).
#include <type_traits>
#include "flashrnn_common.h"
#include "flashrnn_host.h"

namespace flashrnn {

constexpr int TM = 64;    // d rows per workgroup
constexpr int TN = 128;   // (g,e) columns per workgroup
constexpr int TK = 32;    // contraction rows per LDS round

// LDS tiles hold the operands transposed: [row or column][k], bf16 pairs packed along k (BF16) or floats.
template <bool BF16>
__global__ __launch_bounds__(256) void dr_gemm_kernel(const float* __restrict__ states, const void* __restrict__ dWx,
                                                      const void* __restrict__ dgn, float* __restrict__ out, int T, int B, int NH,
                                                      int D, int G, int S, int SK, int gru) {
    constexpr int PITCH = BF16 ? (TK + 8) : (TK + 4);  // elements per LDS row
    constexpr int ESZ = BF16 ? 2 : 4;
    __shared__ __align__(16) char ldsA[TM * PITCH * ESZ];
    __shared__ __align__(16) char ldsB[TN * PITCH * ESZ];
    const int GD = G * D;
    const int tiles_n = (GD + TN - 1) / TN, tiles_m = (D + TM - 1) / TM;
    // Workgroup i runs on XCD i % 8.  All tiles of one (head, K slice) share their operand rows, so they
    // get block indices that are equal modulo 8 and re-read those rows from one L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, tiles = tiles_n * tiles_m;
    const int combo = (slot / tiles) * 8 + xcd, tile = slot % tiles;
    if (combo >= SK * NH) return;
    const int tn = tile % tiles_n, tm = tile / tiles_n;
    const int sk = combo % SK;
    const int n = combo / SK;
    const int K = T * B;
    const int kchunk = ((K + SK - 1) / SK + TK - 1) / TK * TK;
    const int kbeg = sk * kchunk, kend = min(K, kbeg + kchunk);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int c = lane & 15, quad = lane >> 4;
    const int wm = w >> 1, wn = w & 1;  // wave tile: rows [32 wm, +32), columns [64 wn, +64)

    f32x4 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // loader roles: A: thread -> k pair (2 rows) x 4 consecutive d;  B: thread -> k pair x 8 consecutive columns
    // (the 16 k pairs run over the lanes of a 16-lane group: their transposed LDS writes then fall into 16 consecutive banks)
    const int a_kp = tid & 15, a_d = (tid >> 4) * 4;        // 16 k pairs x 16 column groups
    const int b_kp = tid & 15, b_j = (tid >> 4) * 8;        // 16 k pairs x 16 column groups of 8
    const int d_glob = tm * TM + a_d;
    const int j_glob = tn * TN + b_j;
    const bool a_ok = d_glob < D, b_ok = j_glob < GD;
    const int bg = b_ok ? j_glob / D : 0, be = b_ok ? j_glob % D : 0;
    const bool b_from_dgn = gru && bg == 2;

    // Raw tile rows in registers (unconditional loads from clamped addresses, zeroed when they are used),
    // so that the loads of round i+1 are in flight while round i's tiles go through LDS and the matrix cores.
    constexpr int BW = BF16 ? 1 : 2;   // 16-byte words of a B row segment of 8 elements
    const char* b_base = (const char*)(b_from_dgn ? dgn : dWx);
    const size_t b_row = b_from_dgn ? (size_t)NH * D : (size_t)G * NH * D;
    const size_t b_off = b_from_dgn ? (size_t)n * D + be : ((size_t)bg * NH + n) * D + be;
    f32x4 ra[2];
    i32x4 rb[2][BW];
    bool oka[2], okb[2];
    // running position of this thread's two rows: contraction index k = (tt, b) and the element offsets of the row in the
    // states (A operand) and in dWx / the candidate-gradient buffer (B operand), advanced per round without divisions
    int kk_[2], bb_[2];
    size_t offA[2], offB[2];
    const size_t HD = (size_t)NH * D;
    const int adv_q = TK / B, adv_r = TK % B;   // a round advances adv_q whole time steps + adv_r batch rows
    const size_t incA0 = (size_t)TK * HD + (size_t)adv_q * (size_t)(S - 1) * B * HD, incA1 = incA0 + (size_t)(S - 1) * B * HD;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int k = kbeg + a_kp * 2 + r, tt = k / B;
        kk_[r] = k;
        bb_[r] = k - tt * B;
        offA[r] = ((size_t)tt * S * B + bb_[r]) * HD + (size_t)n * D + d_glob;   // row = h_{tt}: the state before step tt + 1
        offB[r] = (size_t)k * b_row + b_off;
    }
    auto load_tiles = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            oka[r] = a_ok && kk_[r] < kend;
            okb[r] = b_ok && kk_[r] < kend;
            ra[r] = *(const f32x4*)(states + (oka[r] ? offA[r] : 0));
            const char* src = b_base + (okb[r] ? offB[r] : 0) * ESZ;
#pragma unroll
            for (int x = 0; x < BW; ++x) rb[r][x] = *(const i32x4*)(src + 16 * x);
            kk_[r] += TK;
            offB[r] += (size_t)TK * b_row;
            int bb = bb_[r] + adv_r;
            const bool wrap = bb >= B;
            bb_[r] = wrap ? bb - B : bb;
            offA[r] += wrap ? incA1 : incA0;
        }
    };
    load_tiles();
    for (int kb = kbeg; kb < kend; kb += TK) {
        __syncthreads();  // previous round's reads are done
        {
            f32x4 a0 = ra[0], a1 = ra[1];
            if (!oka[0]) a0 = f32x4{0.f, 0.f, 0.f, 0.f};
            if (!oka[1]) a1 = f32x4{0.f, 0.f, 0.f, 0.f};
            i32x4 b0[BW], b1[BW];
#pragma unroll
            for (int x = 0; x < BW; ++x) {
                b0[x] = okb[0] ? rb[0][x] : i32x4{0, 0, 0, 0};
                b1[x] = okb[1] ? rb[1][x] : i32x4{0, 0, 0, 0};
            }
            if constexpr (BF16) {   // pairs along k: low half from row 2*kp, high half from row 2*kp + 1
#pragma unroll
                for (int i = 0; i < 4; ++i) *(uint32_t*)(ldsA + ((a_d + i) * PITCH + a_kp * 2) * 2) = pack_bf16x2(a0[i], a1[i]);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t x0 = (uint32_t)b0[0][i >> 1], x1 = (uint32_t)b1[0][i >> 1];
                    const uint32_t v = (i & 1) ? ((x1 & 0xFFFF0000u) | (x0 >> 16)) : ((x1 << 16) | (x0 & 0xFFFFu));
                    *(uint32_t*)(ldsB + ((b_j + i) * PITCH + b_kp * 2) * 2) = v;
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) *(float2*)(ldsA + ((a_d + i) * PITCH + a_kp * 2) * 4) = make_float2(a0[i], a1[i]);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const f32x4 y0 = __builtin_bit_cast(f32x4, b0[i >> 2]), y1 = __builtin_bit_cast(f32x4, b1[i >> 2]);
                    *(float2*)(ldsB + ((b_j + i) * PITCH + b_kp * 2) * 4) = make_float2(y0[i & 3], y1[i & 3]);
                }
            }
        }
        __syncthreads();
        if (kb + TK < kend) load_tiles();
        if constexpr (BF16) {
            bf16x8 af[2], bf[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *(const bf16x8*)(ldsA + ((wm * 32 + i * 16 + c) * PITCH + quad * 8) * 2);
#pragma unroll
            for (int j = 0; j < 4; ++j) bf[j] = *(const bf16x8*)(ldsB + ((wn * 64 + j * 16 + c) * PITCH + quad * 8) * 2);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        } else {
#pragma unroll
            for (int kk = 0; kk < TK / 4; ++kk) {
                float af[2], bf[4];
#pragma unroll
                for (int i = 0; i < 2; ++i) af[i] = *(const float*)(ldsA + ((wm * 32 + i * 16 + c) * PITCH + kk * 4 + quad) * 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) bf[j] = *(const float*)(ldsB + ((wn * 64 + j * 16 + c) * PITCH + kk * 4 + quad) * 4);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
        }
    }
    // ---- store: lane holds column c and rows 4*quad + r of each 16x16 tile
    float* dst = out + ((size_t)sk * NH + n) * (size_t)D * GD;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = tn * TN + wn * 64 + j * 16 + c;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = tm * TM + wm * 32 + i * 16 + quad * 4 + r;
                if (row < D && col < GD) dst[(size_t)row * GD + col] = acc[i][j][r];
            }
        }
}

// bf16 operands without any hand transposition.  Both operands have the contraction index (t, b) as their slow memory
// axis; the tiles go to LDS as they are, [contraction row][column], 16 bytes at a time (h converted from f32 on the way),
// and the matrix-core operands -- 8 contraction elements per lane -- are read with the transposing LDS load of gfx950
// (ds_read_b64_tr_b16: the 16 lanes of a quad read 4 rows x 16 columns and each lane gets the 4 rows of its column).
// Quad q's 8 elements are the rows 4q..4q+3 and 16+4q..16+4q+3 of a round of 32 rows (any assignment of rows to lanes is
// right as long as both operands use the same one): one load then touches 16 consecutive rows, which a row pitch of
// (width + 16 elements) spreads over all 64 banks twice, the minimum for its 512 bytes.
// Tile: (16 FM WM) x (16 FN WN) outputs per workgroup of WM x WN waves, 32 contraction rows per round, two LDS buffers
// (one barrier per round), the next round's global loads in flight during the MFMAs.
// DB: the kernel also sums the gate gradients over (t, b) -- the bias gradient, db[n][g][e] = sum_{t,b} dg_t[b][n][g][e]
// (Sec. 4): the waves that hold the first 16 output rows of a column block multiply a 16 x 32 block of ones onto every B operand
// they read anyway, one more MFMA per round and column block and no further memory traffic.  One row of that product per
// contraction slice goes to dbp[sk][n][g*D + e].  (Used with the staged backward kernels, which have neither the
// registers to keep those sums while their MFMAs run nor the LDS bandwidth to park them.)
// DEPTH: rounds of global loads in flight (register sets).  A round of the small tiles is a few hundred clocks of work
// against a load latency of a microsecond: two sets in flight nearly halve the time of a short contraction.
template <int FM, int FN, int WM, int WN, bool DB, int DEPTH>
__global__ __launch_bounds__(WM * WN * 64) void dr_gemm_tr_kernel(const float* __restrict__ states, const void* __restrict__ dWx,
                                                                 const void* __restrict__ dgn, float* __restrict__ out, float* __restrict__ dbp,
                                                                 int T, int B, int NH, int D, int G, int S, int SK, int gru) {
    constexpr int TMW = 16 * FM * WM, TNW = 16 * FN * WN, NT = 64 * WM * WN;
    constexpr int PA = TMW + 16, PB = TNW + 16;                   // LDS row pitches in bf16 elements
    constexpr int LA = TK * TMW / 4 / NT, LB = TK * TNW / 8 / NT;   // 16-byte global chunks per thread and round
    static_assert(TK == 32 && LA >= 1 && LB >= 1 && (TK * TMW / 4) % NT == 0 && (TK * TNW / 8) % NT == 0, "loader tiling");
    __shared__ __align__(16) uint16_t ldsA[2][TK * PA];
    __shared__ __align__(16) uint16_t ldsB[2][TK * PB];
    const int GD = G * D;
    const int tiles_n = (GD + TNW - 1) / TNW, tiles_m = (D + TMW - 1) / TMW;
    // Workgroup i runs on XCD i % 8.  All tiles of one (head, K slice) share their operand rows, so they get block indices
    // that are equal modulo 8 and re-read those rows from one L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, tiles = tiles_n * tiles_m;
    const int combo = (slot / tiles) * 8 + xcd, tile = slot % tiles;
    if (combo >= SK * NH) return;
    const int tn = tile % tiles_n, tm = tile / tiles_n;
    const int sk = combo % SK, n = combo / SK;
    const int K = T * B;
    const int kchunk = ((K + SK - 1) / SK + TK - 1) / TK * TK;
    const int kbeg = sk * kchunk, kend = min(K, kbeg + kchunk);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int c = lane & 15, quad = lane >> 4;
    const int wm = w / WN, wn = w % WN;

    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 accdb[DB ? FN : 1];
    const bool do_db = DB && tm == 0 && wm == 0;
#pragma unroll
    for (int j = 0; j < (DB ? FN : 1); ++j) accdb[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- loader roles.  A chunk = 4 consecutive d of one contraction row (f32), B chunk = 8 consecutive columns (bf16).
    // Chunk x of a thread: row ra_row[x] of the round, fixed column; the row's position k = (tt, b) is advanced per round
    // without divisions (a round is TK rows = adv_q time steps + adv_r batch rows).
    constexpr int CA = TMW / 4, CB = TNW / 8;   // chunks per tile row
    const size_t HD = (size_t)NH * D;
    const int adv_q = TK / B, adv_r = TK % B;
    const size_t incA0 = (size_t)TK * HD + (size_t)adv_q * (size_t)(S - 1) * B * HD, incA1 = incA0 + (size_t)(S - 1) * B * HD;
    int a_row[LA], a_col[LA], a_bb[LA];
    size_t a_off[LA];
    bool a_ok[LA];
#pragma unroll
    for (int x = 0; x < LA; ++x) {
        const int ch = tid + x * NT;
        a_row[x] = ch / CA;
        a_col[x] = (ch % CA) * 4;
        const int d_glob = tm * TMW + a_col[x];
        a_ok[x] = d_glob < D;
        const int k = kbeg + a_row[x], tt = k / B;
        a_bb[x] = k - tt * B;
        a_off[x] = ((size_t)tt * S * B + a_bb[x]) * HD + (size_t)n * D + (a_ok[x] ? d_glob : 0);   // row = h_{tt}: the state before step tt + 1
    }
    int b_row[LB], b_col[LB];
    size_t b_off[LB], b_rowstride[LB];
    const char* b_base[LB];
    bool b_ok[LB];
#pragma unroll
    for (int x = 0; x < LB; ++x) {
        const int ch = tid + x * NT;
        b_row[x] = ch / CB;
        b_col[x] = (ch % CB) * 8;
        const int j_glob = tn * TNW + b_col[x];
        b_ok[x] = j_glob < GD;
        const int bg = b_ok[x] ? j_glob / D : 0, be = b_ok[x] ? j_glob % D : 0;
        const bool from_dgn = gru && bg == 2;
        b_base[x] = (const char*)(from_dgn ? dgn : dWx);
        b_rowstride[x] = from_dgn ? (size_t)NH * D : (size_t)G * NH * D;
        b_off[x] = (size_t)(kbeg + b_row[x]) * b_rowstride[x] + (from_dgn ? (size_t)n * D + be : ((size_t)bg * NH + n) * D + be);
    }
    f32x4 ra[DEPTH][LA];
    i32x4 rb[DEPTH][LB];
    int kround = kbeg;   // first contraction row of the round the next load fetches
    auto load_tiles = [&](auto set_c) __attribute__((always_inline)) {
        constexpr int SET = decltype(set_c)::value;
#pragma unroll
        for (int x = 0; x < LA; ++x) {
            const bool ok = a_ok[x] && kround + a_row[x] < kend;
            ra[SET][x] = *(const f32x4*)(states + (ok ? a_off[x] : 0));
            if (!ok) ra[SET][x] = f32x4{0.f, 0.f, 0.f, 0.f};
            int bb = a_bb[x] + adv_r;
            const bool wrap = bb >= B;
            a_bb[x] = wrap ? bb - B : bb;
            a_off[x] += wrap ? incA1 : incA0;
        }
#pragma unroll
        for (int x = 0; x < LB; ++x) {
            const bool ok = b_ok[x] && kround + b_row[x] < kend;
            rb[SET][x] = *(const i32x4*)(b_base[x] + (ok ? b_off[x] : 0) * 2);
            if (!ok) rb[SET][x] = i32x4{0, 0, 0, 0};
            b_off[x] += (size_t)TK * b_rowstride[x];
        }
        kround += TK;
    };
    auto park_tiles = [&](auto set_c, int buf) __attribute__((always_inline)) {
        constexpr int SET = decltype(set_c)::value;
#pragma unroll
        for (int x = 0; x < LA; ++x)
            *(i32x2*)(&ldsA[buf][a_row[x] * PA + a_col[x]]) =
                i32x2{(int)pack_bf16x2(ra[SET][x][0], ra[SET][x][1]), (int)pack_bf16x2(ra[SET][x][2], ra[SET][x][3])};
#pragma unroll
        for (int x = 0; x < LB; ++x) *(i32x4*)(&ldsB[buf][b_row[x] * PB + b_col[x]]) = rb[SET][x];
    };
    // this lane's part of a transposing load: row 4 quad + c / 4 (+ 16 for the second half), columns 4 (c % 4) .. + 3 of a 16-column block
    const int tr_row = 4 * quad + (c >> 2), tr_col = 4 * (c & 3);
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    auto operand = [&](const uint16_t* tile, int pitch, int col0) __attribute__((always_inline)) -> bf16x8 {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + tr_row * pitch + col0 + tr_col));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + (16 + tr_row) * pitch + col0 + tr_col));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    };

    using set0 = std::integral_constant<int, 0>;
    using set1 = std::integral_constant<int, DEPTH - 1>;
    // one round: the register set `set` goes to LDS buffer buf, is refilled with the round DEPTH rounds ahead, and the MFMAs run
    auto round = [&](auto set_c, int kb, int buf) __attribute__((always_inline)) {
        park_tiles(set_c, buf);       // (the buffer was last read two rounds ago: the barrier of the previous round lies in between)
        __syncthreads();
        if (kb + DEPTH * TK < kend) load_tiles(set_c);
        bf16x8 af[FM], bfr[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) af[i] = operand(ldsA[buf], PA, (wm * FM + i) * 16);
#pragma unroll
        for (int j = 0; j < FN; ++j) bfr[j] = operand(ldsB[buf], PB, (wn * FN + j) * 16);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        if constexpr (DB) {
            if (do_db) {
                typedef short s16x8 __attribute__((ext_vector_type(8)));
                constexpr short one = 0x3F80;   // bf16 1.0
                const bf16x8 ones = __builtin_bit_cast(bf16x8, s16x8{one, one, one, one, one, one, one, one});
#pragma unroll
                for (int j = 0; j < FN; ++j) accdb[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, bfr[j], accdb[j], 0, 0, 0);
            }
        }
    };
    load_tiles(set0{});
    if constexpr (DEPTH == 2) {
        if (kbeg + TK < kend) load_tiles(set1{});
        int kb = kbeg;
        for (; kb + TK < kend; kb += 2 * TK) {
            round(set0{}, kb, 0);
            round(set1{}, kb + TK, 1);
        }
        if (kb < kend) round(set0{}, kb, 0);
    } else {
        int buf = 0;
        for (int kb = kbeg; kb < kend; kb += TK, buf ^= 1) round(set0{}, kb, buf);
    }
    if constexpr (DB) {
        if (do_db && quad == 0) {   // every row of the product holds the column sums: row 0 is in the lanes of quad 0
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = tn * TNW + (wn * FN + j) * 16 + c;
                if (col < GD) dbp[((size_t)sk * NH + n) * GD + col] = accdb[j][0];
            }
        }
    }
    // ---- store: lane holds column c and rows 4*quad + r of each 16x16 tile
    float* dst = out + ((size_t)sk * NH + n) * (size_t)D * GD;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = tn * TNW + (wn * FN + j) * 16 + c;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = tm * TMW + (wm * FM + i) * 16 + quad * 4 + r;
                if (row < D && col < GD) dst[(size_t)row * GD + col] = acc[i][j][r];
            }
        }
}

// out[j] = sum_{s < NS} part[s * stride + j], added in index order
__global__ void sum_slices_kernel(const float* __restrict__ part, float* __restrict__ out, size_t count, int NS, size_t stride) {
    const size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= count) return;
    float a = 0.f;
    for (int s = 0; s < NS; ++s) a += part[(size_t)s * stride + j];
    out[j] = a;
}

// the two reductions that end the backward pass, in one launch: elements [0, count1) and [count1, count1 + count2);
// four consecutive elements per thread (all counts and strides here are multiples of 4: D is a multiple of 16)
__global__ void sum_slices2_kernel(const float* __restrict__ part1, float* __restrict__ out1, size_t count1, int NS1, size_t stride1,
                                   const float* __restrict__ part2, float* __restrict__ out2, size_t count2, int NS2, size_t stride2) {
    size_t j = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    const float* part = part1;
    float* out = out1;
    int NS = NS1;
    size_t stride = stride1;
    if (j >= count1) {
        j -= count1;
        if (j >= count2) return;
        part = part2; out = out2; NS = NS2; stride = stride2;
    }
    f32x4 a = f32x4{0.f, 0.f, 0.f, 0.f};
    int s = 0;
    for (; s + 8 <= NS; s += 8) {   // eight loads in flight, added in index order
        f32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *(const f32x4*)(part + (size_t)(s + u) * stride + j);
#pragma unroll
        for (int u = 0; u < 8; ++u) a += v[u];
    }
    for (; s < NS; ++s) a += *(const f32x4*)(part + (size_t)s * stride + j);
    *(f32x4*)(out + j) = a;
}

__global__ void fill_zero_kernel(uint32_t* __restrict__ p, size_t count) {
    const size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < count) p[j] = 0u;
}

// Packed copies of R for the persistent kernels (made once per call, R is read once per launch):
//   forward   Rt[n][g][e][k] = R[n][k][g][e]   (k = previous-state index, padded with zeros to DK)
//   backward  Rb[n][d][k]    = R[n][d][k]       (k = gate * D + unit,    padded with zeros to DK)
// The same launch clears the error word of the persistent kernel that follows (the forward one also the backward
// kernels' word next to it; the backward one leaves the forward word alone, so a forward timeout stays visible).
template <typename T>
__global__ void pack_r_fwd_kernel(const T* __restrict__ R, T* __restrict__ out, int NH, int D, int G, int DK, int* __restrict__ err) {
    const size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j == 0) { err[0] = 0; err[1] = 0; }   // a forward call starts a new forward / backward pair: both error words
    const size_t total = (size_t)NH * G * D * DK;
    if (j >= total) return;
    const int k = (int)(j % DK);
    size_t r = j / DK;
    const int e = (int)(r % D); r /= D;
    const int g = (int)(r % G);
    const int n = (int)(r / G);
    out[j] = k < D ? R[(((size_t)n * D + k) * G + g) * D + e] : T(0);
}
template <typename T>
__global__ void pack_r_bwd_kernel(const T* __restrict__ R, T* __restrict__ out, int NH, int D, int G, int DK, int* __restrict__ err) {
    const size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j == 0) *err = 0;
    const size_t total = (size_t)NH * D * DK;
    if (j >= total) return;
    const int k = (int)(j % DK);
    const size_t row = j / DK;  // n * D + d
    out[j] = k < G * D ? R[row * (size_t)(G * D) + k] : T(0);
}

hipError_t launch_pack_r(bool bf16, bool bwd, const void* R, void* out, int NH, int D, int G, int DK, int* err, hipStream_t stream) {
    const size_t total = bwd ? (size_t)NH * D * DK : (size_t)NH * G * D * DK;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (bf16) {
        if (bwd) hipLaunchKernelGGL(pack_r_bwd_kernel<uint16_t>, grid, block, 0, stream, (const uint16_t*)R, (uint16_t*)out, NH, D, G, DK, err);
        else hipLaunchKernelGGL(pack_r_fwd_kernel<uint16_t>, grid, block, 0, stream, (const uint16_t*)R, (uint16_t*)out, NH, D, G, DK, err);
    } else {
        if (bwd) hipLaunchKernelGGL(pack_r_bwd_kernel<float>, grid, block, 0, stream, (const float*)R, (float*)out, NH, D, G, DK, err);
        else hipLaunchKernelGGL(pack_r_fwd_kernel<float>, grid, block, 0, stream, (const float*)R, (float*)out, NH, D, G, DK, err);
    }
    return hipGetLastError();
}

// Output tile of the bf16 GEMM.  A larger tile moves fewer operand bytes through L2 and LDS per flop (the 128 x 256 tile,
// with 64 x 64 outputs per wave, spends more time on its LDS operand reads than on its MFMAs; 256 x 256 with 64 x 128 per
// wave halves them) but needs a large problem: with few output tiles it would take so many contraction slices to fill
// the chip that writing and adding the partial results costs more than it saves (measured: the 128 x 256 tile is slower
// than 64 x 128 on 4 heads x 192 and 8 x 128 units, 28 % faster on 8 x 256; 256 x 256 another 28 % faster there).
// The 256-row tile is taken only where it pads the unit axis no more than the 128-row one.
enum DrTile { kDrSmall = 0, kDrWide = 1, kDrSquare = 2 };
static DrTile dr_tile(bool bf16, int NH, int D, int G) {
    if (!bf16) return kDrSmall;
    const int n256 = (G * D + 255) / 256;
    // (heads of at most 192 units run the staged backward kernels, whose bias gradient comes from this GEMM: the extra
    // accumulators do not fit the registers of the square tile)
    if (D > 192 && (D + 255) / 256 * 2 == (D + 127) / 128 && NH * ((D + 255) / 256) * n256 >= 32) return kDrSquare;
    if (NH * ((D + 127) / 128) * n256 >= 64) return kDrWide;
    return kDrSmall;
}
static int dr_tiles(DrTile t, int NH, int D, int G) {
    const int tm = t == kDrSquare ? 256 : t == kDrWide ? 128 : TM, tn = t == kDrSmall ? TN : 256;
    return NH * ((D + tm - 1) / tm) * ((G * D + tn - 1) / tn);
}

int dr_split_k(bool bf16, int T, int B, int NH, int D, int G) {
    const int K = T * B;
    int sk = 1;
    const DrTile t = dr_tile(bf16, NH, D, G);
    const int tiles = dr_tiles(t, NH, D, G), want = t == kDrSquare ? 256 : 512;   // (the square tile's workgroups fill a CU each)
    while (tiles * sk < want && K / (sk * 2) >= 4 * TK && sk < 64) sk *= 2;
    return sk;
}

// db_from_gemm: db_part is written here, one row of sums per contraction slice (bf16 only); otherwise it holds the
// persistent kernel's per-batch-row sums.
hipError_t launch_dr_gemm(bool bf16, const float* states, const void* dWx, const void* dgn, float* part, float* dR, int T, int B,
                          int NH, int D, int G, int S, bool gru, float* db_part, bool db_from_gemm, float* db, hipStream_t stream) {
    const int SK = dr_split_k(bf16, T, B, NH, D, G);
    const int GD = G * D;
    float* target = SK == 1 ? dR : part;
    const DrTile t = dr_tile(bf16, NH, D, G);
    const int grid = (NH * SK + 7) / 8 * 8 * (dr_tiles(t, NH, D, G) / NH);   // (head, K slice) padded to the 8 XCDs
    if (db_from_gemm && (!bf16 || t == kDrSquare)) return hipErrorInvalidValue;
    if (t == kDrSquare)
        hipLaunchKernelGGL((dr_gemm_tr_kernel<4, 8, 4, 2, false, 1>), dim3(grid), dim3(512), 0, stream, states, dWx, dgn, target, db_part, T, B, NH, D, G, S, SK, gru ? 1 : 0);
    else if (t == kDrWide && db_from_gemm)
        hipLaunchKernelGGL((dr_gemm_tr_kernel<4, 4, 2, 4, true, 2>), dim3(grid), dim3(512), 0, stream, states, dWx, dgn, target, db_part, T, B, NH, D, G, S, SK, gru ? 1 : 0);
    else if (t == kDrWide)
        hipLaunchKernelGGL((dr_gemm_tr_kernel<4, 4, 2, 4, false, 2>), dim3(grid), dim3(512), 0, stream, states, dWx, dgn, target, db_part, T, B, NH, D, G, S, SK, gru ? 1 : 0);
    else if (bf16 && db_from_gemm)
        hipLaunchKernelGGL((dr_gemm_tr_kernel<2, 4, 2, 2, true, 2>), dim3(grid), dim3(256), 0, stream, states, dWx, dgn, target, db_part, T, B, NH, D, G, S, SK, gru ? 1 : 0);
    else if (bf16)
        hipLaunchKernelGGL((dr_gemm_tr_kernel<2, 4, 2, 2, false, 2>), dim3(grid), dim3(256), 0, stream, states, dWx, dgn, target, db_part, T, B, NH, D, G, S, SK, gru ? 1 : 0);
    else
        hipLaunchKernelGGL(dr_gemm_kernel<false>, dim3(grid), dim3(256), 0, stream, states, dWx, dgn, target, T, B, NH, D, G, S, SK, gru ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // split-K partial sums of dR (if any) and the per-row partial sums of db, each added in index order
    const size_t count = SK > 1 ? (size_t)NH * D * GD : 0, nb = (size_t)NH * GD;
    hipLaunchKernelGGL(sum_slices2_kernel, dim3((unsigned)(((count + nb) / 4 + 255) / 256)), dim3(256), 0, stream, part, dR, count, SK, (size_t)NH * D * GD,
                       (const float*)db_part, db, nb, db_from_gemm ? SK : B, nb);
    e = hipGetLastError();
    return e;
}

hipError_t launch_sum_slices(const float* part, float* out, size_t count, int NS, size_t stride, hipStream_t stream) {
    hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, part, out, count, NS, stride);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream) {
    const size_t count = bytes / 4;
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, (uint32_t*)p, count);
    return hipGetLastError();
}

}  // namespace flashrnn
