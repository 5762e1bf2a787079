// Persistent kernels for the case that carries the headline workload: bf16 I/O, one workgroup per
// group, batch tiles of 4 or 8 rows (BT < 16), one block of 16 units per wave.
//
// The matrix pipe of each SIMD is busy for about 1150 cycles per step here (three waves share it), the
// point-wise function of a wave takes a few hundred.  Everything that is not on the dependency chain
//     h_{t-1} in LDS -> MFMA chain -> point-wise -> h_t in LDS -> barrier
// is issued between the MFMAs of a wave's chain:
//   - global traffic goes through LDS images and moves as one 16-byte chunk per thread (a lane holds
//     only one or two values per row, and the CU's memory pipeline needs about 16 cycles per narrow
//     scattered instruction: 13 of them per wave and step would cost more than the MFMAs);
//   - forward: the point-wise phase writes the outputs of step t to their image, from where they leave
//     for HBM during the chain of step t+1; the inputs of step t+1 are fetched during the chain of step t.
// Image rows are padded (lds_row_pitch) so that a wave's 4-rows x 16-units accesses hit 64 distinct banks.
#pragma once
#include <type_traits>

#include "flashrnn_kernels.h"

namespace flashrnn {

__device__ __forceinline__ void pin_order() { __builtin_amdgcn_sched_barrier(0); }

// =============================================================================================
// forward
// =============================================================================================
// LDS: [2] operand rows | [2] input image (BT*G bf16 rows) | [2] output image (BT*S f32 rows, then
// BT*D saved-values records); sizes from tile_lds().
// EXACT: the head has exactly KT * 32 units (the usual case: 32, 64, 128, 192).  Every LDS pitch and image size is then a
// compile-time constant, and with the step's parity a compile-time constant as well (the time loop is unrolled by two) the
// LDS addresses of a step are a lane-constant register plus an immediate offset: a dozen vector adds per wave and step
// less in a loop that is bound by the issue of vector instructions.
template <int CELL, int KT, int BT, int MAXW, bool EXACT>
__device__ __forceinline__ void fwd_tile_body(const KernelParams& p) {
    using CT = CellTraits<CELL>;
    using OP = Operand<true>;
    constexpr int G = CT::G, S = CT::S, NC = CT::NC;
    constexpr int PP = BT / 4;
    constexpr int ESZ = 2;
    constexpr int DK = KT * 32;
    constexpr int NCH_IN = (BT * G + 31) / 32, NCH_ST = (BT * S + 15) / 16;
    constexpr uint32_t kDrop = 0x80000000u;
    constexpr uint32_t REC = CT::RS * ESZ;
    static_assert(BT == 4 || BT == 8, "batch tiles of 4 or 8 rows");

    extern __shared__ __align__(16) char smem[];
    const int gid = blockIdx.x;
    if (gid >= p.NG) return;
    const int D = EXACT ? DK : p.D;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, tid = threadIdx.x, NT = 4 * D;   // one wave per block of 16 units
    stagger_waves(w);
    const LaneMap<BT> lm(lane);
    const int T = p.T, B = p.B, NH = p.NH;
    const int n = gid % NH, q = gid / NH;
    const int e_wave = w * 16, e0 = e_wave + lm.uoff;

    const uint32_t HD = (uint32_t)NH * D;
    const size_t wx_step = (size_t)B * G * HD * ESZ, st_step = (size_t)S * B * HD * 4, c_step = (size_t)B * HD * REC;
    const uint32_t st_state = (uint32_t)B * HD * 4;
    const TileLds L = tile_lds(BT, G, S, D, NT, DK * 2);
    const uint32_t BUF = BT * L.hp, OUT_PITCH = L.st_pitch;
    const uint32_t tid16 = (uint32_t)tid * 16, NT16 = (uint32_t)NT * 16;
    char* hbuf = smem;
    char* in_img = smem + 2 * BUF;
    char* out_img = in_img + 2 * L.in_pitch;

    // ---- R fragments and bias: resident for all T steps.  p.R is the caller's R[n][k][g][e] (no packed copy: a packing
    // kernel in front of this one costs its own run time plus a launch gap, together a few percent of a short sequence).
    // The MFMA A operand of lane (c, quad) is R[k = kt*32 + quad*8 .. +7][g][e_wave + c]: eight values a row pitch apart in
    // memory.  Each wave moves its [32 k] x [16 units] tile of a (gate, k-step) pair to LDS as it lies (two 16-byte
    // pieces per row) and reads it back with the transposing LDS load, which hands every lane four consecutive rows of
    // its column.  The error words of the call are cleared here as well (the kernels of this file never wait on another
    // workgroup, they never set them).
    bf16x8 Rf[G][KT];
    float bias[G][PP];
    if (gid == 0 && tid == 0) { p.err[0] = 0; p.err[1] = 0; }
    {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        char* tile = smem + (uint32_t)w * 1024;                       // this wave's [32][16] bf16 tile
        const int row = lane >> 1, half = lane & 1;
        const char* src = (const char*)p.R + ((((size_t)n * D + row) * G) * D + e_wave + half * 8) * ESZ;
        const uint32_t wr = (uint32_t)row * 32 + half * 16;
        const uint32_t rd = (uint32_t)(lm.quad * 8 + (lm.c >> 2)) * 32 + (lm.c & 3) * 8;
        i32x4 raw[G][KT];   // all loads in flight at once; a fragment takes the registers of the rows it was made from
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                raw[g][kt] = i32x4{0, 0, 0, 0};
                if (kt * 32 + row < D) raw[g][kt] = *(const i32x4*)(src + ((size_t)kt * 32 * G + g) * D * ESZ);
            }
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                // (a wave's LDS operations run in the order it issues them and the tile is its own: no barrier, only the compiler is held)
                asm volatile("" ::: "memory");
                *(i32x4*)(tile + wr) = raw[g][kt];
                asm volatile("" ::: "memory");
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + rd));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + rd + 4 * 32));
                Rf[g][kt] = __builtin_bit_cast(bf16x8, s16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
            }
            load_io<true, PP>(p.bias, ((size_t)n * G + g) * D + e0, bias[g]);
        }
        __syncthreads();   // the tiles lie where the operand rows and images are set up next
    }

    const int bb_raw = q * BT + lm.bslot;
    const bool row_valid = bb_raw < B;
    const int bb = row_valid ? bb_raw : B - 1;
    const char* wx_g = (const char*)p.Wx + (size_t)n * D * ESZ;
    char* st_g = (char*)p.states + (size_t)n * D * 4;
    char* c_g = (char*)p.cache + (size_t)n * D * REC;
    const uint32_t voff_st = ((uint32_t)bb * HD + e0) * 4;

    // ---- chunk roles: global byte offset (out of range = nothing to move) and LDS offset inside the image
    uint32_t cin_g[NCH_IN], cin_l[NCH_IN], cst_g[NCH_ST], cst_l[NCH_ST];
    {
        const uint32_t cpr_io = (uint32_t)D / 8, cpr_st = (uint32_t)D / 4;
#pragma unroll
        for (int k2 = 0; k2 < NCH_IN; ++k2) {
            const uint32_t idx = tid + k2 * NT, row = idx / cpr_io, ch = idx % cpr_io, brow = q * BT + row / G, g = row % G;
            const bool in = row < (uint32_t)BT * G;
            cin_g[k2] = (in && brow < (uint32_t)B) ? ((brow * G + g) * HD) * ESZ + ch * 16 : kDrop;
            // (image rows in the order gate, slot: the rows that one instruction reads -- one gate, all slots -- are then one
            // pitch apart, 16 banks; in memory order, slot * G + gate, they would be G pitches apart: the same banks for G = 4)
            cin_l[k2] = in ? (g * BT + row / G) * L.rp_io + ch * 16 : L.in_bytes + tid16 + k2 * NT16;
        }
#pragma unroll
        for (int k2 = 0; k2 < NCH_ST; ++k2) {
            const uint32_t idx = tid + k2 * NT, row = idx / cpr_st, ch = idx % cpr_st, s = row / BT, brow = q * BT + row % BT;
            const bool in = row < (uint32_t)BT * S;
            cst_g[k2] = (in && brow < (uint32_t)B) ? s * st_state + (brow * HD) * 4 + ch * 16 : kDrop;
            cst_l[k2] = in ? row * L.rp_st + ch * 16 : L.st_bytes + tid16 + k2 * NT16;
        }
    }
    // this lane's places: inputs row = g*BT + slot, states row = s*BT + slot; the saved-values records (16 bytes per
    // lane, 256 contiguous bytes per batch row and wave) go to HBM straight from the lanes
    const uint32_t l_in = (uint32_t)lm.bslot * L.rp_io + e0 * ESZ;
    const uint32_t l_st = (uint32_t)lm.bslot * L.rp_st + e0 * 4;
    const uint32_t voff_c = (row_valid && p.cache != nullptr) ? ((uint32_t)bb * HD + e0) * REC : kDrop;
    const uint32_t lds_row = (uint32_t)lm.bslot * L.hp;

    constexpr bool kLongChain = KT >= 6;   // (see below: how far ahead the inputs are fetched)
    // ---- initial states: slot 0 is written directly (once)
    float st[S][PP];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        if (p.states0 != nullptr) load_io_r<false, PP>(make_rsrc((const char*)p.states0 + (size_t)n * D * 4), voff_st, s * st_state, st[s]);
        else
#pragma unroll
            for (int i = 0; i < PP; ++i) st[s][i] = 0.0f;
        store_io_r<false, PP>(make_rsrc(st_g), row_valid ? voff_st : kDrop, s * st_state, st[s]);
    }
    for (uint32_t j = tid; j < 2 * BUF / 4; j += NT) ((uint32_t*)hbuf)[j] = 0u;
    __syncthreads();
    write_operand_lds<true, PP>(hbuf + lds_row, e0, st[0]);
    if (T > 0) {
        const rsrc_t rs1 = make_rsrc(wx_g);
#pragma unroll
        for (int k2 = 0; k2 < NCH_IN; ++k2) *(i32x4*)(in_img + L.in_pitch + cin_l[k2]) = __builtin_amdgcn_raw_buffer_load_b128(rs1, cin_g[k2], 0, 0);
    }
    __syncthreads();
    // With a short chain a step is shorter than the HBM latency under load (0.4 us against 1 us and more once most CUs
    // stream): the inputs are fetched four steps ahead there, in four register sets of one chunk per thread (Wx_j travels
    // in set j mod 4: requested at the top of step j - 4, parked in its image at the end of step j - 1), one step ahead with a
    // long chain.  Requests beyond the last step fetch the last step's inputs again.
    i32x4 pre[4][NCH_IN];
    if constexpr (!kLongChain) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int k2 = 0; k2 < NCH_IN; ++k2) pre[j][k2] = i32x4{0, 0, 0, 0};
        if (T > 0) {   // (with T = 0 there is no Wx to touch)
#pragma unroll
            for (int j = 2; j <= 4; ++j) {   // Wx_2, Wx_3, Wx_4: slots 1, 2, 3
                const rsrc_t rsj = make_rsrc(wx_g + (size_t)(j - 1 < T ? j - 1 : T - 1) * wx_step);
#pragma unroll
                for (int k2 = 0; k2 < NCH_IN; ++k2) pre[j & 3][k2] = __builtin_amdgcn_raw_buffer_load_b128(rsj, cin_g[k2], 0, 0);
                // Each request is followed by at least as many stores as a step issues behind its own, all of them out of range (the
                // memory pipeline drops them).  The compiler waits for a request by counting the memory operations issued
                // after it, and where two paths meet -- this prologue and the loop's back edge, at the loop's head -- it
                // takes the smaller count: without the padding three of the four steps of the loop waited for requests only
                // one and two steps old (wait counts 5, 7, 9, 11 instead of 11 four times).
#pragma unroll
                for (int x = 0; x < NCH_ST + 2 * PP; ++x) __builtin_amdgcn_raw_buffer_store_b128(i32x4{0, 0, 0, 0}, rsj, kDrop, 0, 0);
            }
        }
    }

    // move the image of the states after step j to HBM (slot j)
    auto copy_out_load = [&](int parity, i32x4 (&vs)[NCH_ST]) {
        const char* img = out_img + parity * OUT_PITCH;
#pragma unroll
        for (int k2 = 0; k2 < NCH_ST; ++k2) vs[k2] = *(const i32x4*)(img + cst_l[k2]);
    };
    // The three streams of a step advance by whole time steps: their bases are carried as pointers (a product of the
    // step index and a 64-bit stride per stream and step is a dozen scalar instructions).
    // Long chain: one register set, Wx_{t+2} requested at the tail of step t and parked a third into step t+1 -- or, with the
    // step's parity a compile-time constant (EXACT), two sets that alternate: Wx_{t+3} requested at the tail of step t into the
    // set that Wx_{t+1} has just left, parked a third into step t+2 (1.6 steps of lead instead of 0.6: with a hundred and more
    // CUs streaming the latency of HBM exceeds a step).
    constexpr bool kTwoSets = kLongChain && EXACT;
    constexpr int kFirstAhead = kLongChain ? (kTwoSets ? 3 : 2) : 4;   // slot of the first request made inside the time loop (slot 2 = Wx_3)
    const char* wx_ptr = wx_g + (size_t)(kFirstAhead < T ? kFirstAhead : (T > 0 ? T - 1 : 0)) * wx_step;   // Wx of the step fetched next
    // Long chain: Wx_{t+1} is requested at the end of step t-1, AHEAD of that step's stores in the wave's memory queue.  A
    // wave's vector memory operations retire in order: a load issued behind the stores of the step before could not be
    // waited for without waiting for their acknowledgements as well, which tied the step to the write latency of the
    // memory system (sequences whose buffers outgrow the last-level cache ran 15 % slower per step, the LSTM 25 %).
    i32x4 pre_next[NCH_IN];
    if constexpr (kLongChain) {
        // (behind each request of the prologue the stores that follow a request in the time loop, dropped ones: see the short chain)
        auto dropped_stores = [&](const rsrc_t rs, const int count) {
            for (int x = 0; x < count; ++x) __builtin_amdgcn_raw_buffer_store_b128(i32x4{0, 0, 0, 0}, rs, kDrop, 0, 0);
        };
#pragma unroll
        for (int k2 = 0; k2 < NCH_IN; ++k2) pre_next[k2] = pre[0][k2] = pre[1][k2] = i32x4{0, 0, 0, 0};
        if (T > 0) {
            const rsrc_t rs2 = make_rsrc(wx_g + (size_t)(T > 1 ? 1 : 0) * wx_step);
            if constexpr (kTwoSets) {   // Wx_2 travels in set 0, Wx_3 in set 1
                const rsrc_t rs3 = make_rsrc(wx_g + (size_t)(T > 2 ? 2 : T - 1) * wx_step);
#pragma unroll
                for (int k2 = 0; k2 < NCH_IN; ++k2) pre[0][k2] = __builtin_amdgcn_raw_buffer_load_b128(rs2, cin_g[k2], 0, 0);
                dropped_stores(rs2, 2 * PP + NCH_ST);
#pragma unroll
                for (int k2 = 0; k2 < NCH_IN; ++k2) pre[1][k2] = __builtin_amdgcn_raw_buffer_load_b128(rs3, cin_g[k2], 0, 0);
                dropped_stores(rs3, 2 * PP);
            } else {
#pragma unroll
                for (int k2 = 0; k2 < NCH_IN; ++k2) pre_next[k2] = __builtin_amdgcn_raw_buffer_load_b128(rs2, cin_g[k2], 0, 0);
                dropped_stores(rs2, 2 * PP);
            }
        }
    }
    // Short chain (kDefer): the states after step t go to their image at the top of step t+1 (they are still in registers
    // there, and every LDS write behind the point-wise function is on the step's tail: 12 x 64 forward 0.361 -> 0.327 ms per
    // 1024 steps), are read back as 16-byte chunks at the top of step t+2 and leave for HBM during that step's chain.  With
    // a long chain the writes would land between the MFMAs, where the LDS is busy with operand reads (4 x 192: +3 %): there
    // they stay at the end of step t, and the chunks leave during step t+1.
    constexpr bool kDefer = !kLongChain;
    char* st_ptr = st_g;   // state slot t-2 (kDefer) or t-1 of step t (slot 0 is written directly, not through the image)
    char* c_ptr = c_g;     // saved values of the current step (kDefer: of the step before, whose records leave at the top of this one)
    // (the saved values too, for heads of up to 64 units -- kDeferRec: 12 x 64 with 64 rows forward 0.388 -> 0.360 ms per 1024
    // steps; with eight waves the GRU lost 5 % by it and the LSTM gained 3: left at the end of the step there)
    constexpr bool kDeferRec = kDefer && MAXW <= 4;
    float cv_keep[PP][CT::NC];   // kDeferRec: the saved values of the step before
#pragma unroll
    for (int i = 0; i < PP; ++i)
#pragma unroll
        for (int c2 = 0; c2 < CT::NC; ++c2) cv_keep[i][c2] = 0.0f;
    auto copy_out_store = [&](int j, const i32x4 (&vs)[NCH_ST]) {
        const uint32_t none = j < 1 ? kDrop : 0u;
        const rsrc_t rs_st = make_rsrc(st_ptr);
#pragma unroll
        for (int k2 = 0; k2 < NCH_ST; ++k2) __builtin_amdgcn_raw_buffer_store_b128(vs[k2], rs_st, cst_g[k2] | none, 0, 0);
    };
    // (trace builds: clocks per wave between 0 the barrier and the top of a step | 2 the top and the issue of the chain's
    // last MFMA | 3 that and the barrier: compaction, point-wise function, LDS writes)
    FRNN_TRACE_BEGIN();
    // one time step; PH = t & 3 as a compile-time constant where it selects a register set (short chain), PAR = t & 1
    auto step = [&](auto ph_c, const int t) {
        constexpr int PH = decltype(ph_c)::value;
        constexpr int PAR = PH & 1;
        // parity of the step: a compile-time constant where the loop is unrolled by two (always with a short chain, where it
        // selects a register set; with a long chain only for EXACT heads: with run-time pitches the two sets of addresses
        // would not fit the registers)
        const int par = (EXACT || !kLongChain) ? PAR : (t & 1);
        FRNN_TRACE_MARK(0);
        // The MFMA chain of the step, k-step by k-step, and the work off the dependency chain: this step's inputs out of
        // their image, the state rows of the previous step on their way to HBM, the next step's inputs into their image
        // (the sched barriers keep the compiler from bunching it all up in front).  With a long chain (KT >= 6) that
        // work sits between the k-steps; with a short one all LDS reads go out together at the top of the step (one
        // latency) and the next inputs are parked at its end, where they have had time to arrive (measured both ways).
        bf16x8 hB[KT];
        const char* hrow = hbuf + (par ^ 1) * BUF + lds_row;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) hB[kt] = *(const bf16x8*)(hrow + (size_t)(kt * 32 + lm.quad * 8) * 2);
        i32x4 vs[NCH_ST];
        float wx[G][PP];
        auto side_reads = [&]() {
            const char* im = in_img + par * L.in_pitch + l_in;
#pragma unroll
            for (int g = 0; g < G; ++g) load_io<true, PP>(im + (uint32_t)g * BT * L.rp_io, 0, wx[g]);
            if constexpr (kDefer) {
                if constexpr (kDeferRec) {   // the saved values of step t-1 leave here as well: packing and storing them is off the tail too
                    const rsrc_t rs_prev = make_rsrc(c_ptr);
                    c_ptr += t >= 2 ? c_step : 0;
#pragma unroll
                    for (int i = 0; i < PP; ++i) store_record<true, CT::RS, NC>(rs_prev, (voff_c + i * REC) | (t < 2 ? kDrop : 0u), 0, cv_keep[i]);
                }
#pragma unroll
                for (int s = 0; s < S; ++s) store_io<false, PP>(out_img + (par ^ 1) * OUT_PITCH + l_st + (uint32_t)s * BT * L.rp_st, 0, st[s]);   // states after step t-1
                copy_out_load(par, vs);                                                                                                       // states after step t-2
            } else {
                copy_out_load(par ^ 1, vs);   // states after step t-1
            }
#pragma unroll
            for (int g = 0; g < G; ++g)     // the bias joins the inputs here, off the step's tail (GRU's candidate bias
#pragma unroll                      // belongs to the recurrent term that sig(r) multiplies: it stays with y)
                for (int i = 0; i < PP; ++i)
                    if (!(CELL == CELL_GRU && g == 2)) wx[g][i] += bias[g][i];
        };
        if constexpr (!kLongChain) side_reads();
        if constexpr (!kLongChain) {
            const int ahead = t + 3;   // slot of Wx_{t+4} (the last steps fetch the last slot again)
            const rsrc_t rsn = make_rsrc(wx_ptr);
            wx_ptr += ahead < T - 1 ? wx_step : 0;
#pragma unroll
            for (int k2 = 0; k2 < NCH_IN; ++k2) pre[PH][k2] = __builtin_amdgcn_raw_buffer_load_b128(rsn, cin_g[k2], 0, 0);
        }
        pin_order();
        f32x4 acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = OP::mfma(Rf[g][0], hB[0], f32x4{0.f, 0.f, 0.f, 0.f});
        pin_order();
        if constexpr (!kLongChain) {
            copy_out_store(kDefer ? t - 2 : t - 1, vs);
            pin_order();
#pragma unroll
            for (int kt = 1; kt < (KT < 3 ? KT : 3); ++kt)
#pragma unroll
                for (int g = 0; g < G; ++g) acc[g] = OP::mfma(Rf[g][kt], hB[kt], acc[g]);
        } else {
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = OP::mfma(Rf[g][1], hB[1], acc[g]);
            pin_order();
            side_reads();
            pin_order();
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = OP::mfma(Rf[g][2], hB[2], acc[g]);
            pin_order();
            copy_out_store(kDefer ? t - 2 : t - 1, vs);
            pin_order();
            char* im = in_img + (par ^ 1) * L.in_pitch;
#pragma unroll
            for (int k2 = 0; k2 < NCH_IN; ++k2) *(i32x4*)(im + cin_l[k2]) = kTwoSets ? pre[PAR ^ 1][k2] : pre_next[k2];
        }
        pin_order();
#pragma unroll
        for (int kt = 3; kt < KT; ++kt)
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = OP::mfma(Rf[g][kt], hB[kt], acc[g]);
        FRNN_TRACE_MARK(2);
        // (short chain: Wx_{t+1}, requested three steps ago, goes to its image here, in the shadow of the last MFMAs, not behind the
        // point-wise function, where every instruction is on the step's tail; Wx_{t+2} .. Wx_{t+4} stay in flight)
        if constexpr (!kLongChain) {
            char* im = in_img + (par ^ 1) * L.in_pitch;
#pragma unroll
            for (int k2 = 0; k2 < NCH_IN; ++k2) *(i32x4*)(im + cin_l[k2]) = pre[(PH + 1) & 3][k2];
        }
        pin_order();
        // ---- point-wise function; the step's outputs go to their image (they leave for HBM during the next step)
#pragma unroll
        for (int g = 0; g < G; ++g) compact_tile<BT>(acc[g]);
        if constexpr (kLongChain) {   // Wx_{t+2}: slot t + 1, or with two sets Wx_{t+3} (the last steps fetch the last slot again)
            const rsrc_t rsn = make_rsrc(wx_ptr);
            wx_ptr += t + (kTwoSets ? 2 : 1) < T - 1 ? wx_step : 0;
#pragma unroll
            for (int k2 = 0; k2 < NCH_IN; ++k2) {
                if constexpr (kTwoSets) pre[PAR ^ 1][k2] = __builtin_amdgcn_raw_buffer_load_b128(rsn, cin_g[k2], 0, 0);
                else pre_next[k2] = __builtin_amdgcn_raw_buffer_load_b128(rsn, cin_g[k2], 0, 0);
            }
        }
        const rsrc_t rs_c = make_rsrc(c_ptr);
        if constexpr (!kDeferRec) c_ptr += c_step;
        st_ptr += (!kDefer || t >= 2) ? st_step : 0;
#pragma unroll
        for (int i = 0; i < PP; ++i) {
            float wxi[G], ybi[G], sti[S], cvi[NC];
#pragma unroll
            for (int g = 0; g < G; ++g) { wxi[g] = wx[g][i]; ybi[g] = (CELL == CELL_GRU && g == 2) ? acc[g][i] + bias[g][i] : acc[g][i]; }
#pragma unroll
            for (int s = 0; s < S; ++s) sti[s] = st[s][i];
            Cell<CELL, true>::fwd(wxi, ybi, sti, cvi);
#pragma unroll
            for (int s = 0; s < S; ++s) st[s][i] = sti[s];
            if constexpr (kDeferRec) {
#pragma unroll
                for (int c2 = 0; c2 < NC; ++c2) cv_keep[i][c2] = cvi[c2];
            } else {
                store_record<true, CT::RS, NC>(rs_c, voff_c + i * REC, 0, cvi);
            }
        }
        write_operand_lds<true, PP>(hbuf + par * BUF + lds_row, e0, st[0]);
        if constexpr (!kDefer) {
#pragma unroll
            for (int s = 0; s < S; ++s) store_io<false, PP>(out_img + par * OUT_PITCH + l_st + (uint32_t)s * BT * L.rp_st, 0, st[s]);
        }
#ifdef FLASHRNN_TRACE
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#endif
        FRNN_TRACE_MARK(3);
        __syncthreads();
    };
    using ph0 = std::integral_constant<int, 0>;
    using ph1 = std::integral_constant<int, 1>;
    using ph2 = std::integral_constant<int, 2>;
    using ph3 = std::integral_constant<int, 3>;
    if constexpr (kLongChain && !EXACT) {
        for (int t = 1; t <= T; ++t) step(ph0{}, t);
    } else if constexpr (kLongChain) {
        int t = 1;
        for (; t + 1 <= T; t += 2) {
            step(ph1{}, t);
            step(ph0{}, t + 1);
        }
        if (t <= T) step(ph1{}, t);
    } else {
        int t = 1;
        for (; t + 3 <= T; t += 4) {
            step(ph1{}, t);
            step(ph2{}, t + 1);
            step(ph3{}, t + 2);
            step(ph0{}, t + 3);
        }
        if (t <= T) step(ph1{}, t);
        if (t + 1 <= T) step(ph2{}, t + 1);
        if (t + 2 <= T) step(ph3{}, t + 2);
    }
    // ---- drain: the states after step T are in their image -- or (kDefer) those after step T-1, and those after step T still in registers
    if (T > 0) {
        i32x4 vs[NCH_ST];
        if constexpr (kDefer) {
            if constexpr (kDeferRec) {
                const rsrc_t rs_last = make_rsrc(c_g + (size_t)(T - 1) * c_step);   // the saved values of step T
#pragma unroll
                for (int i = 0; i < PP; ++i) store_record<true, CT::RS, NC>(rs_last, voff_c + i * REC, 0, cv_keep[i]);
            }
#pragma unroll
            for (int s = 0; s < S; ++s) store_io<false, PP>(out_img + (T & 1) * OUT_PITCH + l_st + (uint32_t)s * BT * L.rp_st, 0, st[s]);
            st_ptr = st_g + (size_t)(T - 1) * st_step;
            copy_out_load((T & 1) ^ 1, vs);
            copy_out_store(T - 1, vs);
            __syncthreads();
            st_ptr += st_step;
        }
        copy_out_load(T & 1, vs);
        copy_out_store(T, vs);
    }
    FRNN_TRACE_END(p);
}

template <int CELL, int KT, int BT, int MAXW>
__global__ __launch_bounds__(MAXW * 64) void fwd_tile_kernel(const KernelParams p) {
    if (p.D == KT * 32) fwd_tile_body<CELL, KT, BT, MAXW, true>(p);
    else fwd_tile_body<CELL, KT, BT, MAXW, false>(p);
}

// =============================================================================================
// backward, one block of 16 units per wave, contraction split over EBK waves
// =============================================================================================
// A step of the backward pass is the chain
//     point-wise Jacobians of step t -> dg_t in LDS -> barrier -> MFMA chain R dg_t -> dh_{t-1}.
// The contraction axis (G * D gate gradients) is G times longer than in the forward pass; if every wave
// read all of it from LDS, the LDS would bound the step.  Here waves come in sets of EBK: a set owns EBK
// blocks of units, and each of its waves contracts all of the set's blocks over one of EBK slices of the
// axis (the same number of MFMAs and R registers per wave, 1/EBK of the operand reads).  The partial sums
// go through LDS; wave w then runs the point-wise function of block w.
// Global traffic moves as 16-byte chunks through LDS images, off the chain: the inputs of step t-2 are
// fetched while step t's MFMAs run, by loads that write their image in LDS directly (no registers are
// held across the HBM latency), and are read into registers during step t-1's MFMAs; dWx_t leaves
// during step t's MFMAs.
// EXACT: as in the forward kernel (the head has exactly KTW * EBK * 32 / G units: compile-time LDS pitches, and a
// compile-time step parity with the time loop unrolled by two).
// 1 KB pieces of an input image of the backward kernel (records | state rows | dh rows, each part rounded up to whole
// pieces as in tile_lds_bwd) per wave of a head of D units
constexpr int deep_pieces_per_wave(int BT, int D, int rec_bytes, int nsb) {
    const int pieces = (BT * D * rec_bytes + 1023) / 1024 + (BT * nsb * D * 4 + 1023) / 1024 + (BT * D * 2 + 1023) / 1024;
    return (pieces + D / 16 - 1) / (D / 16);
}

template <int CELL, int KTW, int EBK, int BT, int MAXW, bool EXACT, bool DEEP = false>
__global__ __launch_bounds__(MAXW * 64) void bwd_tile_kernel(const KernelParams p) {
    using CT = CellTraits<CELL>;
    using OP = Operand<true>;
    constexpr int G = CT::G, S = CT::S, NC = CT::NC;
    constexpr int PP = BT / 4;
    constexpr int ESZ = 2;
    constexpr int KT = KTW * EBK, DK = KT * 32;
    constexpr int NSB = CELL == CELL_SLSTM ? 2 : CELL == CELL_ELMAN ? 0 : 1;   // state rows the Jacobian needs per time level ...
    constexpr int SB0 = cell_uses_h_prev(CELL) ? 0 : 1;   // ... starting at this state
    constexpr int GO = CELL == CELL_GRU ? G + 1 : G;  // output rows per batch row: dWx (+ the recurrent-side candidate gradient)
    // accumulators per block: independent MFMAs in flight.  A wave that has its SIMD to itself (heads of up to 64 units) issues
    // an MFMA every 16 clocks, so two chains keep dependent ones 32 apart, which a 4-pass MFMA allows; four chains cost eight
    // more additions and eight more register moves per step there (12 x 64 backward: -6 %).  With two waves per SIMD four measured 1 % better.
    constexpr int NA = EBK == 1 ? (MAXW <= 4 ? 2 : 4) : (EBK == 2 ? 2 : 1);
    constexpr uint32_t kDrop = 0x80000000u;
    constexpr uint32_t REC = CT::RS * ESZ;
    static_assert(BT == 4 || BT == 8, "batch tiles of 4 or 8 rows");
    static_assert(BT * NSB <= 16 && BT * GO <= 32, "one chunk per thread and image");

    extern __shared__ __align__(16) char smem[];
    const int gid = blockIdx.x;
    if (gid >= p.NG) return;
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), tid = threadIdx.x;
    const int tg = w / EBK, ks = w % EBK;
    const LaneMap<BT> lm(lane);
    const int D = EXACT ? DK / G : p.D;
    const int T = p.T, B = p.B, NH = p.NH;
    const int NT = 4 * D;
    const int n = gid % NH, q = gid / NH;
    const int e0 = w * 16 + lm.uoff;                 // this lane's units in the point-wise phase: block w

    const uint32_t HD = (uint32_t)NH * D;
    const size_t wx_step = (size_t)B * G * HD * ESZ, st_step = (size_t)S * B * HD * 4, c_step = (size_t)B * HD * REC;
    const size_t dh_step = (size_t)B * HD * ESZ;
    const uint32_t st_state = (uint32_t)B * HD * 4;
    const TileLdsBwd L = tile_lds_bwd(BT, GO, NSB, D, DK * 2, EBK, REC);
    const uint32_t BUF = BT * L.hp;
    char* gbuf = smem;
    float* red = (float*)(smem + L.red_off);
    char* in_img = smem + L.in_off;
    char* out_img = smem + L.out_off;

    // ---- R fragments: blocks tg*EBK + j, contraction slice ks
    bf16x8 Rf[EBK][KTW];
#pragma unroll
    for (int j = 0; j < EBK; ++j) {
        const size_t rrow = ((size_t)n * D + (tg * EBK + j) * 16 + lm.c) * DK + (size_t)ks * KTW * 32;
#pragma unroll
        for (int kt = 0; kt < KTW; ++kt) Rf[j][kt] = *(const bf16x8*)((const uint16_t*)p.R + rrow + kt * 32 + lm.quad * 8);
    }

    const int bb_raw = q * BT + lm.bslot;
    const bool row_valid = bb_raw < B;
    const int bb = row_valid ? bb_raw : B - 1;
    const char* c_g = (const char*)p.cache + (size_t)n * D * REC;
    const char* st_g = (const char*)p.states + (size_t)n * D * 4;
    const char* dh_g = (const char*)p.dH + (size_t)n * D * ESZ;
    char* dwx_g = (char*)p.dWx + (size_t)n * D * ESZ;
    char* dgn_g = (char*)p.dgn + (size_t)n * D * ESZ;
    const uint32_t voff_st = ((uint32_t)bb * HD + e0) * 4;

    // ---- chunk roles: global byte offsets (out of range = nothing to move)
    constexpr int NCC = (BT * (int)REC + 63) / 64;   // record chunks per thread: BT rows of D records, NT = 4 D threads
    uint32_t cc_g[NCC], cst_g, cdh_g, cout_g, cout_n, cout_l;
    bool out_real, cout_img, c_wave[NCC];
    const uint32_t cpr_io = (uint32_t)D / 8;
    const bool st_wave = (uint32_t)w * 64 < (uint32_t)BT * NSB * (D / 4), dh_wave = (uint32_t)w * 64 < (uint32_t)BT * cpr_io;
    // The input images are plain arrays of rows whose pitch (D records, D floats, D bf16) is a multiple of 256 bytes for the
    // larger heads: the rows of the batch slots would fall on the same LDS banks, and a wave reads 4 (8) of them with one
    // instruction.  So the chunks of slot r's row are stored rotated by 4 r chunks (64 r bytes, modulo the row): a thread's
    // slot in the image is fixed by the loads that write LDS directly, which global chunk it fetches is free.
    auto rotated = [](uint32_t ch, uint32_t slot, uint32_t cpr) { return (ch + (4u * slot) % cpr) % cpr; };          // row position of chunk ch
    auto unrotated = [](uint32_t pos, uint32_t slot, uint32_t cpr) { return (pos + cpr - (4u * slot) % cpr) % cpr; }; // chunk at row position pos
    const uint32_t cpr_c = (uint32_t)D * REC / 16, cpr_st = (uint32_t)D / 4;
    {
        const uint32_t nch_c = (uint32_t)BT * cpr_c;
#pragma unroll
        for (int k2 = 0; k2 < NCC; ++k2) {   // records: a row of the image is the D records of one batch row
            const uint32_t idx = tid + k2 * NT, row = idx / cpr_c, ch = unrotated(idx % cpr_c, row, cpr_c), brow = q * BT + row;
            cc_g[k2] = (idx < nch_c && brow < (uint32_t)B) ? (brow * HD) * REC + ch * 16 : kDrop;
            c_wave[k2] = (uint32_t)w * 64 + k2 * NT < nch_c;   // (a wave beyond the image must not land zeros behind it)
        }
        {   // state rows: row = state * BT + slot
            const uint32_t row = tid / cpr_st, ch = unrotated(tid % cpr_st, row % BT, cpr_st), sidx = row / BT, brow = q * BT + row % BT;
            cst_g = (row < (uint32_t)BT * NSB && brow < (uint32_t)B) ? (SB0 + sidx) * st_state + (brow * HD) * 4 + ch * 16 : kDrop;
        }
        {   // dh rows: row = slot
            const uint32_t row = tid / cpr_io, ch = unrotated(tid % cpr_io, row, cpr_io), brow = q * BT + row;
            cdh_g = (row < (uint32_t)BT && brow < (uint32_t)B) ? (brow * HD) * ESZ + ch * 16 : kDrop;
        }
        {   // output rows: row = slot * GO + g; g < G goes to dWx, g == G to the candidate-gradient buffer
            const uint32_t row = tid / cpr_io, ch = tid % cpr_io, g = row % GO, brow = q * BT + row / GO;
            const bool in = row < (uint32_t)BT * GO && brow < (uint32_t)B;
            cout_g = (in && g < (uint32_t)G) ? ((brow * G + g) * HD) * ESZ + ch * 16 : kDrop;
            cout_n = (in && g == (uint32_t)G) ? (brow * HD) * ESZ + ch * 16 : kDrop;
            // Where the input-side gate gradients equal the recurrent-side ones, the rows written for the MFMA operand are
            // the output rows as well.  That is every gate of every cell but the GRU's candidate, whose input-side gradient
            // alone goes through an image of its own (one row per batch row; the recurrent-side one is the operand's).
            const uint32_t og = g == (uint32_t)G ? 2u : g;   // gate segment of the operand row
            cout_img = CELL == CELL_GRU && g == 2;
            cout_l = cout_img ? (row / GO) * L.rp_io + ch * 16 : (row / GO) * L.hp + og * (uint32_t)D * ESZ + ch * 16;
            out_real = row < (uint32_t)BT * GO;
        }
    }
    // DEEP: the same image filled through registers, by loads that every wave issues in the same number every step (the
    // compiler counts the memory operations behind a request to wait for it: see request below).  Either every wave issues
    // the loads of all three kinds, those of a wave without chunks of a kind out of range and dropped (NCC + 2 per wave
    // and step), or -- kPieces: where the image, a run of 1 KB pieces of 64 chunks, has no more pieces than the
    // workgroup has waves (heads of exactly 64 or 128 units, 4-row tiles, every cell but the sLSTM) -- wave w moves piece w:
    // one load per wave and step, at most one of them dropped.  (With two pieces per wave the first way measured faster.)
    constexpr bool kPieces = EXACT && DEEP && deep_pieces_per_wave(BT, DK / G, (int)REC, NSB) == 1;
    constexpr int NSL = kPieces ? 1 : NCC + 2;
    int sl_kind[NSL];        // 0 records, 1 state rows, 2 dh rows, 3 none (wave-uniform)
    uint32_t sl_g[NSL];      // global byte offset of this lane's chunk of the piece
    uint32_t sl_l[NSL];      // LDS byte offset of the piece inside the image
    if constexpr (kPieces) {
        const uint32_t NW = (uint32_t)D / 16;
#pragma unroll
        for (int j = 0; j < NSL; ++j) {
            const uint32_t off = ((uint32_t)w + j * NW) * 1024u;
            sl_l[j] = off;
            sl_kind[j] = off < L.st_off ? 0 : (off < L.dh_off ? 1 : (off < L.in_pitch ? 2 : 3));
            const uint32_t idx = (off - (sl_kind[j] == 1 ? L.st_off : (sl_kind[j] == 2 ? L.dh_off : 0u))) / 16 + lane;
            uint32_t g = kDrop;
            if (sl_kind[j] == 0) {
                const uint32_t row = idx / cpr_c, ch = unrotated(idx % cpr_c, row, cpr_c), brow = q * BT + row;
                if (idx < (uint32_t)BT * cpr_c && brow < (uint32_t)B) g = (brow * HD) * REC + ch * 16;
            } else if (sl_kind[j] == 1) {
                const uint32_t row = idx / cpr_st, ch = unrotated(idx % cpr_st, row % BT, cpr_st), sidx = row / BT, brow = q * BT + row % BT;
                if (row < (uint32_t)BT * NSB && brow < (uint32_t)B) g = (SB0 + sidx) * st_state + (brow * HD) * 4 + ch * 16;
            } else if (sl_kind[j] == 2) {
                const uint32_t row = idx / cpr_io, ch = unrotated(idx % cpr_io, row, cpr_io), brow = q * BT + row;
                if (row < (uint32_t)BT && brow < (uint32_t)B) g = (brow * HD) * ESZ + ch * 16;
            }
            sl_g[j] = g;
        }
    }
    // this lane's places in the images
    // (byte o of slot r's row lies in the chunk at row position rotated(o / 16); a lane's PP values of a state or of dh share
    // a chunk, its PP records need not)
    auto in_row = [&](uint32_t o, uint32_t cpr) { return rotated(o / 16, (uint32_t)lm.bslot, cpr) * 16 + o % 16; };
    uint32_t l_c[PP];
#pragma unroll
    for (int i = 0; i < PP; ++i) l_c[i] = (uint32_t)lm.bslot * D * REC + in_row((e0 + i) * REC, cpr_c);
    const uint32_t l_st = L.st_off + (uint32_t)lm.bslot * D * 4 + in_row(e0 * 4, cpr_st);
    const uint32_t l_dh = L.dh_off + (uint32_t)lm.bslot * D * ESZ + in_row(e0 * ESZ, cpr_io);
    const uint32_t l_out = (uint32_t)lm.bslot * L.rp_io + e0 * ESZ;
    const uint32_t lds_row = (uint32_t)lm.bslot * L.hp;

    // carried state gradients; ds[0] is the part of dh_t that came through R and the direct path
    float ds[S][PP];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        if (p.dlast != nullptr && !(CELL == CELL_SLSTM && s == 3))
            load_io_r<false, PP>(make_rsrc((const char*)p.dlast + (size_t)n * D * 4), voff_st, s * st_state, ds[s]);
        else
#pragma unroll
            for (int i = 0; i < PP; ++i) ds[s][i] = 0.0f;
    }

    for (uint32_t j = tid; j < 2 * BUF / 4; j += NT) ((uint32_t*)gbuf)[j] = 0u;

    // the image of the inputs of step j: global -> LDS (each wave's 64 chunks back to back), LDS -> this lane's values
    // (the steps are fetched in the order T, T-1, ..., 1: the three streams' bases are carried as pointers, and so are
    // those of the outputs -- a product of the step index and a 64-bit stride per stream and step is a dozen scalar
    // instructions)
    const ptrdiff_t back = T > 0 ? T - 1 : 0;
    const char* fc_ptr = c_g + back * (ptrdiff_t)c_step;
    const char* fst_ptr = st_g + back * (ptrdiff_t)st_step;
    const char* fdh_ptr = dh_g + back * (ptrdiff_t)dh_step;
    char* dwx_ptr = dwx_g + back * (ptrdiff_t)wx_step;
    char* dgn_ptr = dgn_g + back * (ptrdiff_t)dh_step;
    // (DEEP: every step requests, also the last ones, whose requests have no step left to serve: the pointers stop at step 1,
    // whose inputs are then fetched again)
    int fleft = T;   // steps not yet fetched or requested
    auto advance = [&]() {
        if constexpr (DEEP) {
            const bool more = fleft > 1;
            fc_ptr -= more ? c_step : 0; fst_ptr -= more ? st_step : 0; fdh_ptr -= more ? dh_step : 0;
            fleft -= more ? 1 : 0;
        } else {
            fc_ptr -= c_step; fst_ptr -= st_step; fdh_ptr -= dh_step;
        }
    };
    auto fetch = [&](const int parity) {
        const rsrc_t rc = make_rsrc(fc_ptr), rst = make_rsrc(fst_ptr), rdh = make_rsrc(fdh_ptr);
        advance();
        char* img = in_img + parity * L.in_pitch + (uint32_t)w * 1024;
#pragma unroll
        for (int k2 = 0; k2 < NCC; ++k2)
            if (c_wave[k2]) load_chunk_to_lds(rc, img + (uint32_t)k2 * NT * 16, cc_g[k2]);
        if (st_wave) load_chunk_to_lds(rst, img + L.st_off, cst_g);
        if (dh_wave) load_chunk_to_lds(rdh, img + L.dh_off, cdh_g);
    };
    // DEEP (a kernel of its own for heads of up to 128 units, steps of 0.4 to 0.6 us; the host takes it when the inputs exceed the
    // last-level cache and will come from HBM): the same chunks through registers instead, requested SIX steps before their
    // step and written into the image four steps later.  With the loads that write LDS directly the request can only go out
    // once its image is free, two steps before the data is used -- less than the latency of HBM, which these short steps then
    // wait for (12 x 64, B = 16: 0.40 us per step up to T = 512, 0.54 us from T = 1024 on; through registers 0.48 us).  While
    // the inputs still come from the cache the direct loads are the faster way (0.40 against 0.44 us).  Four register sets
    // take turns by the step index modulo 4 (the time loop of these kernels is unrolled by four).  Both ways in one kernel, chosen
    // by a flag, measured slower than either: where the branches join the compiler waits for the requests just issued.
    static_assert(!DEEP || MAXW <= 8, "the deep fetch: heads of up to 128 units");
    constexpr bool kRegFetch = DEEP;
    struct Held { i32x4 v[NSL]; };
    Held held[4];   // the chunks of the steps t = T, T-1, T-2, T-3 modulo 4
    // (Every wave issues NSL loads, every step.  The compiler waits for a request by counting the memory operations issued
    // after it; a load or a request under a condition makes it count the path with the fewest, and the wait for a request four
    // steps old becomes a wait for the one of the step before.)
    auto request = [&](Held& h) {
        if constexpr (kPieces) {
#pragma unroll
            for (int j = 0; j < NSL; ++j) {
                const char* base = sl_kind[j] == 0 ? fc_ptr : (sl_kind[j] == 1 ? fst_ptr : fdh_ptr);
                h.v[j] = __builtin_amdgcn_raw_buffer_load_b128(make_rsrc(base), sl_g[j], 0, 0);
            }
        } else {
            const rsrc_t rc = make_rsrc(fc_ptr), rst = make_rsrc(fst_ptr), rdh = make_rsrc(fdh_ptr);
            // (eight waves: the dropped loads -- 17 of 24 per step at 128 units -- cost more issue slots than the exact counts
            // bring; there only the waves that have chunks of a kind request them, as the direct loads do)
            constexpr bool kAllWaves = MAXW <= 4;
#pragma unroll
            for (int k2 = 0; k2 < NCC; ++k2)
                if (kAllWaves || c_wave[k2]) h.v[k2] = __builtin_amdgcn_raw_buffer_load_b128(rc, cc_g[k2], 0, 0);
            if (kAllWaves || st_wave) h.v[NCC] = __builtin_amdgcn_raw_buffer_load_b128(rst, cst_g, 0, 0);
            if (kAllWaves || dh_wave) h.v[NCC + 1] = __builtin_amdgcn_raw_buffer_load_b128(rdh, cdh_g, 0, 0);
        }
        advance();
    };
    auto park = [&](const Held& h, const int parity) {   // (the places the direct loads would have written)
        char* img = in_img + parity * L.in_pitch + (uint32_t)lane * 16;
        if constexpr (kPieces) {
#pragma unroll
            for (int j = 0; j < NSL; ++j)
                if (sl_kind[j] != 3) *(i32x4*)(img + sl_l[j]) = h.v[j];
        } else {
            img += (uint32_t)w * 1024;
#pragma unroll
            for (int k2 = 0; k2 < NCC; ++k2)
                if (c_wave[k2]) *(i32x4*)(img + (uint32_t)k2 * NT * 16) = h.v[k2];
            if (st_wave) *(i32x4*)(img + L.st_off) = h.v[NCC];
            if (dh_wave) *(i32x4*)(img + L.dh_off) = h.v[NCC + 1];
        }
    };
    float cv[NC][PP], sc[S][PP], sp[S][PP], dh_ext[PP];
    auto take = [&](const int parity) {
        const char* img = in_img + parity * L.in_pitch;
#pragma unroll
        for (int i = 0; i < PP; ++i) {
            float rec[NC];
            take_record_lds<CT::RS, NC>(img + l_c[i], rec);
#pragma unroll
            for (int c2 = 0; c2 < NC; ++c2) cv[c2][i] = rec[c2];
        }
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (s >= SB0 && s < SB0 + NSB) load_io<false, PP>(img + l_st + (uint32_t)(s - SB0) * BT * D * 4, 0, sp[s]);
            else
#pragma unroll
                for (int i = 0; i < PP; ++i) sp[s][i] = 1.0f;
        }
        load_io<true, PP>(img + l_dh, 0, dh_ext);
    };

    // The factors of the Jacobian that do not depend on dh_t are formed as soon as the step's saved values and states
    // are in registers (in the shadow of the previous step's MFMAs), which leaves a few multiply-adds for the point-wise
    // phase, where all waves compete for the VALU.
    //   sLSTM kc = {o/n, o c/n^2, ig (1 - z^2), fg sig(-f), (c/n) o (1 - o)}
    //   LSTM  kc = {o (1 - tanh^2 c), z i (1 - i), c_prev f (1 - f), i (1 - z^2), tanh(c) o (1 - o)}
    //   GRU   kc = {(1 - z)(1 - cand^2), (h_prev - cand) z (1 - z), kc0 yn r (1 - r), kc0 r}
    constexpr bool kPre = CELL == CELL_LSTM || CELL == CELL_SLSTM || CELL == CELL_GRU;
    float kc[5][PP];
    auto precompute = [&]() {
#pragma unroll
        for (int i = 0; i < PP; ++i) {
            if constexpr (CELL == CELL_SLSTM) {
                const float inv = fast_rcp(sc[2][i]), q = sc[1][i] * inv, o = cv[3][i], z = cv[2][i], oi = o * inv;
                kc[0][i] = oi;
                kc[1][i] = oi * q;
                kc[2][i] = cv[0][i] * (1.0f - z * z);
                kc[3][i] = cv[1][i] * cv[4][i];
                kc[4][i] = q * o * (1.0f - o);
            } else if constexpr (CELL == CELL_LSTM) {
                const float ig = cv[0][i], f = cv[1][i], z = cv[2][i], o = cv[3][i], tc = tanh_<true>(sc[1][i]);
                kc[0][i] = o * (1.0f - tc * tc);
                kc[1][i] = z * ig * (1.0f - ig);
                kc[2][i] = sp[1][i] * f * (1.0f - f);
                kc[3][i] = ig * (1.0f - z * z);
                kc[4][i] = tc * o * (1.0f - o);
            } else if constexpr (CELL == CELL_GRU) {
                const float r = cv[0][i], z = cv[1][i], cand = cv[2][i], yn = cv[3][i];
                kc[0][i] = (1.0f - z) * (1.0f - cand * cand);
                kc[1][i] = (sp[0][i] - cand) * z * (1.0f - z);
                kc[2][i] = kc[0][i] * yn * r * (1.0f - r);
                kc[3][i] = kc[0][i] * r;
            }
        }
    };
    // ---- prologue: images of steps T and T-1, this lane's inputs of step T, the states after step T
#pragma unroll
    for (int s = 0; s < S; ++s) {
        if (!cell_uses_h_prev(CELL) && s >= SB0 && s < SB0 + NSB && T > 0)
            load_io_r<false, PP>(make_rsrc(st_g + (size_t)T * st_step), voff_st, s * st_state, sc[s]);
        else
#pragma unroll
            for (int i = 0; i < PP; ++i) sc[s][i] = 1.0f;
    }
    // (DEEP: images and register sets take turns by the distance T - t from the first step, not by t: the first step
    // then has phase 0 whatever T is, and the time loop needs no steps peeled off in front of it)
    auto par_of = [&](const int t) { return DEEP ? ((T - t) & 1) : (t & 1); };
    if (T > 0) {
        fetch(par_of(T));
        if (T > 1) fetch(par_of(T - 1));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    if constexpr (kRegFetch) {
        if (T > 0) {   // steps T-2 .. T-5 into the sets 2, 3, 0, 1
#pragma unroll
            for (int j = 2; j <= 5; ++j) {
                request(held[j & 3]);
                // (as many dropped stores behind each request as a step issues at most: the wait counts at the head of the time
                // loop are the smaller of what this prologue and the loop's back edge leave behind)
                __builtin_amdgcn_raw_buffer_store_b128(i32x4{0, 0, 0, 0}, make_rsrc(dwx_g), kDrop, 0, 0);
                __builtin_amdgcn_raw_buffer_store_b128(i32x4{0, 0, 0, 0}, make_rsrc(dwx_g), kDrop, 0, 0);
            }
        }
    }
    __syncthreads();
    if (T > 0) { take(par_of(T)); precompute(); }

    // (the bias gradient, the sum of dg over time and batch rows, is formed by the dR GEMM, which reads every dg anyway:
    // this kernel has neither the registers to keep the sums while its MFMAs run nor LDS bandwidth to spare for them)
    // one time step; PH = (T - t) & 3 (DEEP) or t & 1 as a compile-time constant where the loop is unrolled by four or two
    constexpr bool kUnroll = true;
    auto step = [&](auto ph_c, const int t) {
        const int par = ((EXACT || DEEP) && kUnroll) ? (decltype(ph_c)::value & 1) : (t & 1);
        // ---- point-wise Jacobians of step t
        {
            float dwx[G][PP], dg[G][PP];
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                float cvi[NC], sci[S], spi[S], dsi[S], dwxi[G], dgi[G];
#pragma unroll
                for (int c2 = 0; c2 < NC; ++c2) cvi[c2] = cv[c2][i];
#pragma unroll
                for (int s = 0; s < S; ++s) { sci[s] = sc[s][i]; spi[s] = sp[s][i]; dsi[s] = ds[s][i]; }
                dsi[0] += dh_ext[i];
                if constexpr (kPre) {
                    const float dh = dsi[0];
                    if constexpr (CELL == CELL_SLSTM) {
                        const float dc = fmaf(dh, kc[0][i], dsi[1]), dn = fmaf(-dh, kc[1][i], dsi[2]);
                        dgi[0] = fmaf(dc, cvi[2], dn) * cvi[0];
                        dgi[1] = fmaf(dc, spi[1], dn * spi[2]) * kc[3][i];
                        dgi[2] = dc * kc[2][i];
                        dgi[3] = dh * kc[4][i];
                        dsi[0] = 0.0f; dsi[1] = dc * cvi[1]; dsi[2] = dn * cvi[1]; dsi[3] = 0.0f;
                    } else if constexpr (CELL == CELL_LSTM) {
                        const float dc = fmaf(dh, kc[0][i], dsi[1]);
                        dgi[0] = dc * kc[1][i];
                        dgi[1] = dc * kc[2][i];
                        dgi[2] = dc * kc[3][i];
                        dgi[3] = dh * kc[4][i];
                        dsi[0] = 0.0f; dsi[1] = dc * cvi[1];
                    } else {   // GRU: the input side sees d(pre-tanh) in gate n, the recurrent side d(yn)
                        dgi[0] = dh * kc[2][i];
                        dgi[1] = dh * kc[1][i];
                        dgi[2] = dh * kc[3][i];
                        dsi[0] = dh * cvi[1];   // direct path h_{t-1} -> h_t
                    }
#pragma unroll
                    for (int g = 0; g < G; ++g) dwxi[g] = dgi[g];
                    if constexpr (CELL == CELL_GRU) dwxi[2] = dh * kc[0][i];
                } else {
                    Cell<CELL, true>::bwd(cvi, sci, spi, dsi, dwxi, dgi);
                }
#pragma unroll
                for (int s = 0; s < S; ++s) ds[s][i] = dsi[s];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    dwx[g][i] = dwxi[g];
                    dg[g][i] = dgi[g];
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                write_operand_lds<true, PP>(gbuf + par * BUF + lds_row, g * D + e0, dg[g]);
            }
            if constexpr (CELL == CELL_GRU) store_io<true, PP>(out_img + par * L.out_pitch + l_out, 0, dwx[2]);
            if constexpr (!cell_uses_h_prev(CELL)) {
#pragma unroll
                for (int s = SB0; s < SB0 + NSB; ++s)
#pragma unroll
                    for (int i = 0; i < PP; ++i) sc[s][i] = sp[s][i];
            }
        }
        // the chunks fetched during the previous step are in LDS once only that step's stores are younger;
        // they are read after this barrier
        if constexpr (!kRegFetch) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(CELL == CELL_GRU ? 2 : 1) : "memory");
        __syncthreads();
        // ---- dh_{t-1} += R dg_t; in the shadow of the chain: fetch step t-2, dWx_t out, step t-1's values
        // The operand is read in chunks of KC k-steps, one chunk ahead of the MFMAs that use it.
        constexpr int KC = 4, NCK = (KTW + KC - 1) / KC;
        bf16x8 gB[NCK][KC];
        const char* grow = gbuf + par * BUF + lds_row + (size_t)(ks * KTW * 32 + lm.quad * 8) * 2;
        // Only the lanes of the BT valid batch columns read: the backward step is bound by the LDS (busy 62 % of the
        // step, nearly half of it these reads), and an LDS read costs bandwidth per active lane.  The other lanes' registers
        // keep whatever they held -- a column of the B operand only reaches the same column of the result, and the
        // columns c >= BT of a result are never used; the empty asm statements stand for "any value" (without them
        // the compiler would give the idle lanes a defined value, one move per register and chunk).
        auto read_chunk = [&](int c) {
            i32x4 raw[KC];
#pragma unroll
            for (int k = 0; k < KC; ++k) asm volatile("" : "=v"(raw[k]));
            if (lm.c < BT) {
#pragma unroll
                for (int k = 0; k < KC; ++k)
                    if (c * KC + k < KTW) raw[k] = *(const i32x4*)(grow + (size_t)(c * KC + k) * 64);
            }
#pragma unroll
            for (int k = 0; k < KC; ++k) gB[c][k] = __builtin_bit_cast(bf16x8, raw[k]);
        };
        read_chunk(0);
        if constexpr (kRegFetch) {
            // step t-2's chunks (requested four steps ago) into the image that step t's have left; then the request for step t-6
            // (both also in the last steps, where nobody reads what they bring: no condition, see request)
            constexpr int PH = decltype(ph_c)::value, SET = (PH + 2) & 3;
            park(held[SET], PH & 1);
            request(held[SET]);
        } else {
            if (t > 2) fetch(par);
        }
        pin_order();
        f32x4 acc[EBK][NA];
#pragma unroll
        for (int j = 0; j < EBK; ++j)
#pragma unroll
            for (int a = 0; a < NA; ++a) acc[j][a] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NCK; ++c) {
#pragma unroll
            for (int k = 0; k < KC; ++k)
                if (c * KC + k < KTW) {
#pragma unroll
                    for (int j = 0; j < EBK; ++j) acc[j][(c * KC + k) % NA] = OP::mfma(Rf[j][c * KC + k], gB[c][k], acc[j][(c * KC + k) % NA]);
                }
            pin_order();
            if (c + 1 < NCK) read_chunk(c + 1);
            if (c == 0) {   // dWx_t out of its image and on its way, step t-1's values out of theirs
                i32x4 o = i32x4{0, 0, 0, 0};
                if (out_real) o = *(const i32x4*)(((CELL == CELL_GRU && cout_img) ? out_img + par * L.out_pitch : gbuf + par * BUF) + cout_l);
                if (t > 1) { take(par ^ 1); precompute(); }
                pin_order();
                __builtin_amdgcn_raw_buffer_store_b128(o, make_rsrc(dwx_ptr), cout_g, 0, 0);
                dwx_ptr -= wx_step;
                if constexpr (CELL == CELL_GRU) {
                    __builtin_amdgcn_raw_buffer_store_b128(o, make_rsrc(dgn_ptr), cout_n, 0, 0);
                    dgn_ptr -= dh_step;
                }
            }
            pin_order();
        }
        float part[EBK][PP];
#pragma unroll
        for (int j = 0; j < EBK; ++j) {
            f32x4 a = acc[j][0];
#pragma unroll
            for (int x = 1; x < NA; ++x) a += acc[j][x];
            compact_tile<BT>(a);
#pragma unroll
            for (int i = 0; i < PP; ++i) part[j][i] = a[i];
        }
        if constexpr (EBK > 1) {
#pragma unroll
            for (int j = 0; j < EBK; ++j)   // partial sum of block tg*EBK + j from slice ks
                store_io<false, PP>(red, ((size_t)((tg * EBK + j) * EBK + ks) * 64 + lane) * PP, part[j]);
            __syncthreads();
            float rec[PP];   // R dg_t of this lane's pairs, summed over the slices
#pragma unroll
            for (int i = 0; i < PP; ++i) rec[i] = 0.0f;
#pragma unroll
            for (int x = 0; x < EBK; ++x) {
                float v[PP];
                load_io<false, PP>(red, ((size_t)(w * EBK + x) * 64 + lane) * PP, v);
#pragma unroll
                for (int i = 0; i < PP; ++i) rec[i] += v[i];
            }
#pragma unroll
            for (int i = 0; i < PP; ++i) ds[0][i] += fminf(fmaxf(rec[i], -p.clip), p.clip);   // (Sec. 4.1 clip; +inf = off)
        } else {
#pragma unroll
            for (int i = 0; i < PP; ++i) ds[0][i] += fminf(fmaxf(part[0][i], -p.clip), p.clip);
        }
    };
    using ph0 = std::integral_constant<int, 0>;
    using ph1 = std::integral_constant<int, 1>;
    using ph2 = std::integral_constant<int, 2>;
    using ph3 = std::integral_constant<int, 3>;
    if constexpr (DEEP && kUnroll) {
        int t = T;
        for (; t >= 4; t -= 4) {
            step(ph0{}, t);
            step(ph1{}, t - 1);
            step(ph2{}, t - 2);
            step(ph3{}, t - 3);
        }
        if (t >= 1) step(ph0{}, t);
        if (t >= 2) step(ph1{}, t - 1);
        if (t >= 3) step(ph2{}, t - 2);
    } else if constexpr (EXACT && kUnroll) {
        int t = T;
        if (t & 1) { step(ph1{}, t); --t; }
        for (; t >= 2; t -= 2) {
            step(ph0{}, t);
            step(ph1{}, t - 1);
        }
    } else {
        for (int t = T; t >= 1; --t) step(ph0{}, t);
    }
    // ---- gradients w.r.t. the initial states
    if (row_valid) {
#pragma unroll
        for (int s = 0; s < S; ++s)
            store_io_r<false, PP>(make_rsrc((char*)p.dstates0 + (size_t)n * D * 4), voff_st, s * st_state, ds[s]);
    }
}

}  // namespace flashrnn
