// Persistent forward and backward kernels of the RNN time-step loop (gfx950, wave64, MFMA).
//
// Forward (paper Sec. 3 eq. (1)-(2), Alg. 1): per step  y = R^T h_{t-1}  on the matrix cores, then
// g = Wx_t + y + b and the cell's point-wise function in registers; states and the values the
// backward pass needs go to HBM; the new h goes to LDS (one CU per group) or to a stamped exchange
// buffer in global memory (several CUs per group) and is the next step's MFMA operand.
// Backward (paper Sec. 4 eq. (3)-(4)): per step the point-wise Jacobians give the gate gradients dg_t,
// which are streamed out as dWx, handed to the other waves like h in the forward pass, and contracted
// with the same resident R along its gate/unit axis to give dh_{t-1}.
#pragma once
#include "flashrnn_common.h"

namespace flashrnn {

// ---------------------------------------------------------------------------------------------
// point-wise functions (paper App. A); gate order i,f,z,o (LSTM, sLSTM) and r,z,n (GRU); Elman has one gate
// ---------------------------------------------------------------------------------------------
template <int CELL, bool FAST> struct Cell;

template <bool FAST> struct Cell<CELL_LSTM, FAST> {
    // st = {h, c}; wx = input pre-activations, yb = R^T h + b
    static __device__ __forceinline__ void fwd(const float (&wx)[4], const float (&yb)[4], float (&st)[2], float (&cv)[4]) {
        const float i = sigm<FAST>(wx[0] + yb[0]), f = sigm<FAST>(wx[1] + yb[1]);
        const float z = tanh_<FAST>(wx[2] + yb[2]), o = sigm<FAST>(wx[3] + yb[3]);
        const float c = f * st[1] + i * z;
        st[1] = c;
        st[0] = o * tanh_<FAST>(c);
        cv[0] = i; cv[1] = f; cv[2] = z; cv[3] = o;
    }
    // sc = states after the step (h unused), sp = states before the step;
    // ds = carried gradients {dh (total incl. external), dc}; on return ds = point-wise carries
    // (ds[0] = direct h path, zero here); dwx = input-side, dg = recurrent-side gate gradients.
    static __device__ __forceinline__ void bwd(const float (&cv)[4], const float (&sc)[2], const float (&sp)[2], float (&ds)[2],
                                               float (&dwx)[4], float (&dg)[4]) {
        const float i = cv[0], f = cv[1], z = cv[2], o = cv[3];
        const float tc = tanh_<FAST>(sc[1]);
        const float dh = ds[0];
        const float dc = ds[1] + dh * o * (1.0f - tc * tc);
        dg[0] = dc * z * i * (1.0f - i);
        dg[1] = dc * sp[1] * f * (1.0f - f);
        dg[2] = dc * i * (1.0f - z * z);
        dg[3] = dh * tc * o * (1.0f - o);
        dwx[0] = dg[0]; dwx[1] = dg[1]; dwx[2] = dg[2]; dwx[3] = dg[3];
        ds[1] = dc * f;
        ds[0] = 0.0f;
    }
};

template <bool FAST> struct Cell<CELL_SLSTM, FAST> {
    // st = {h, c, n, m}
    static __device__ __forceinline__ void fwd(const float (&wx)[4], const float (&yb)[4], float (&st)[4], float (&cv)[5]) {
        const float pi = wx[0] + yb[0], pf = wx[1] + yb[1];
        float lf, sf;  // log sig(pf), sig(-pf)
        if constexpr (FAST) {
            // log sig(f) = min(f, 0) - log(1 + exp(-|f|)): no product that could underflow for large |f|
            const float t = fast_exp2(-kLog2e * fabsf(pf));
            const float r = fast_rcp(1.0f + t);
            sf = pf >= 0.0f ? t * r : r;
            lf = fmaf(kLn2, fast_log2(r), fminf(pf, 0.0f));
        } else {
            lf = pf >= 0.0f ? -log1pf(expf(-pf)) : pf - log1pf(expf(pf));
            sf = 1.0f / (1.0f + expf(pf));
        }
        const float a = lf + st[3];
        const float m = fmaxf(a, pi);
        const float fg = exp_<FAST>(a - m), ig = exp_<FAST>(pi - m);
        const float z = tanh_<FAST>(wx[2] + yb[2]), o = sigm<FAST>(wx[3] + yb[3]);
        const float c = fg * st[1] + ig * z;
        const float n = fg * st[2] + ig;
        st[1] = c; st[2] = n; st[3] = m;
        if constexpr (FAST) st[0] = o * c * fast_rcp(n);
        else st[0] = o * c / n;
        cv[0] = ig; cv[1] = fg; cv[2] = z; cv[3] = o; cv[4] = sf;
    }
    // ds = {dh, dc, dn, -}; the stabilizer carries no gradient
    static __device__ __forceinline__ void bwd(const float (&cv)[5], const float (&sc)[4], const float (&sp)[4], float (&ds)[4],
                                               float (&dwx)[4], float (&dg)[4]) {
        const float ig = cv[0], fg = cv[1], z = cv[2], o = cv[3], sf = cv[4];
        const float dh = ds[0];
        float inv;
        if constexpr (FAST) inv = fast_rcp(sc[2]);
        else inv = 1.0f / sc[2];
        const float ho = dh * o * inv;        // dh * o / n_t
        const float q = sc[1] * inv;          // c_t / n_t
        const float dc = ds[1] + ho;
        const float dn = ds[2] - ho * q;
        dg[0] = (dc * z + dn) * ig;
        dg[1] = (dc * sp[1] + dn * sp[2]) * fg * sf;
        dg[2] = dc * ig * (1.0f - z * z);
        dg[3] = dh * q * o * (1.0f - o);
        dwx[0] = dg[0]; dwx[1] = dg[1]; dwx[2] = dg[2]; dwx[3] = dg[3];
        ds[1] = dc * fg; ds[2] = dn * fg; ds[3] = 0.0f;
        ds[0] = 0.0f;
    }
};

template <bool FAST> struct Cell<CELL_GRU, FAST> {
    // st = {h}; gate n: yb[2] = R_n h + b_n is multiplied by sig(r) before it meets the input
    static __device__ __forceinline__ void fwd(const float (&wx)[3], const float (&yb)[3], float (&st)[1], float (&cv)[4]) {
        const float r = sigm<FAST>(wx[0] + yb[0]), z = sigm<FAST>(wx[1] + yb[1]);
        const float yn = yb[2];
        const float cand = tanh_<FAST>(wx[2] + r * yn);
        st[0] = z * st[0] + (1.0f - z) * cand;
        cv[0] = r; cv[1] = z; cv[2] = cand; cv[3] = yn;
    }
    static __device__ __forceinline__ void bwd(const float (&cv)[4], const float (&sc)[1], const float (&sp)[1], float (&ds)[1],
                                               float (&dwx)[3], float (&dg)[3]) {
        const float r = cv[0], z = cv[1], cand = cv[2], yn = cv[3];
        const float dh = ds[0];
        const float dpre = dh * (1.0f - z) * (1.0f - cand * cand);
        const float dz = dh * (sp[0] - cand) * z * (1.0f - z);
        const float dr = dpre * yn * r * (1.0f - r);
        dwx[0] = dr; dwx[1] = dz; dwx[2] = dpre;
        dg[0] = dr; dg[1] = dz; dg[2] = dpre * r;
        ds[0] = dh * z;  // direct path h_{t-1} -> h_t
        (void)sc;
    }
};

template <bool FAST> struct Cell<CELL_GRU4, FAST> {
    // the GRU as App. A prints it; gates z, r, n, g (all full pre-activations); st = {h}
    static __device__ __forceinline__ void fwd(const float (&wx)[4], const float (&yb)[4], float (&st)[1], float (&cv)[4]) {
        const float z = sigm<FAST>(wx[0] + yb[0]), r = sigm<FAST>(wx[1] + yb[1]);
        const float tg = tanh_<FAST>(wx[3] + yb[3]);
        const float cand = tanh_<FAST>(wx[2] + yb[2] + r * tg);
        st[0] = z * st[0] + (1.0f - z) * cand;
        cv[0] = z; cv[1] = r; cv[2] = cand; cv[3] = tg;
    }
    static __device__ __forceinline__ void bwd(const float (&cv)[4], const float (&sc)[1], const float (&sp)[1], float (&ds)[1],
                                               float (&dwx)[4], float (&dg)[4]) {
        const float z = cv[0], r = cv[1], cand = cv[2], tg = cv[3];
        const float dh = ds[0];
        const float dpre = dh * (1.0f - z) * (1.0f - cand * cand);
        dg[0] = dh * (sp[0] - cand) * z * (1.0f - z);
        dg[1] = dpre * tg * r * (1.0f - r);
        dg[2] = dpre;
        dg[3] = dpre * r * (1.0f - tg * tg);
        dwx[0] = dg[0]; dwx[1] = dg[1]; dwx[2] = dg[2]; dwx[3] = dg[3];
        ds[0] = dh * z;  // direct path h_{t-1} -> h_t
        (void)sc;
    }
};

template <bool FAST> struct Cell<CELL_ELMAN, FAST> {
    // st = {h}: h_t = tanh(x_t + R h_{t-1} + b)
    static __device__ __forceinline__ void fwd(const float (&wx)[1], const float (&yb)[1], float (&st)[1], float (&cv)[1]) {
        st[0] = tanh_<FAST>(wx[0] + yb[0]);
        cv[0] = st[0];
    }
    static __device__ __forceinline__ void bwd(const float (&cv)[1], const float (&sc)[1], const float (&sp)[1], float (&ds)[1],
                                               float (&dwx)[1], float (&dg)[1]) {
        dg[0] = ds[0] * (1.0f - cv[0] * cv[0]);
        dwx[0] = dg[0];
        ds[0] = 0.0f;   // h_{t-1} enters the step only through R
        (void)sc; (void)sp;
    }
};

// Forces prefetched values to be complete (and converted) at this point of the program.  Vector
// memory operations retire in order, so a wait placed later would also wait for the stores issued
// in between; placing it before them keeps the store latency off the per-step critical path.
template <int N, int M> __device__ __forceinline__ void pin(float (&v)[N][M]) {
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int j = 0; j < M; ++j) asm volatile("" : "+v"(v[i][j]) : : "memory");
}
template <int N> __device__ __forceinline__ void pin(float (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(v[i]) : : "memory");
}

// Per-phase clock stamps of a time step (a library built with -DFLASHRNN_TRACE; no code otherwise).  Every wave adds up, per
// phase, the shader clocks between consecutive marks; at the end of the kernel lane 0 of each wave writes its sums to
// p.trace[workgroup][wave][phase].  Phases of the kernels whose groups span several workgroups:
//   forward   0 issue of the input prefetch | 1 barrier (all waves have read the old rows) | 7 first round trip of the poll
//             (everything the wave has in flight retires first) | 2 further rounds until the partners' h_{t-1} is complete,
//             payloads into LDS | 3 barrier | 4 operand reads + MFMA chain + slice sums | 5 point-wise + publish h_t
//             | 6 stores of states / saved values and the wait for the prefetched inputs
//   backward  0 issue of the loads of step t-1, point-wise Jacobians of step t, publish dg_t, dWx stores | 1 barrier | 7 first
//             round trip of the poll | 2 further rounds until the partners' dg_t is complete, payloads into LDS | 3 barrier | 4 operand reads + MFMA chain + slice sums | 5 wait for
//             the prefetched inputs
#ifdef FLASHRNN_TRACE
#define FRNN_TRACE_BEGIN() unsigned long long tr_acc[kTracePhases] = {0, 0, 0, 0, 0, 0, 0, 0}; unsigned long long tr_t = __builtin_amdgcn_s_memtime(), tr_first = 0;
#define FRNN_TRACE_MARK(i) { __builtin_amdgcn_sched_barrier(0); const unsigned long long tr_n = __builtin_amdgcn_s_memtime(); \
                             tr_acc[i] += tr_n - tr_t; tr_t = tr_n; __builtin_amdgcn_sched_barrier(0); }
#define FRNN_TRACE_FIRST (&tr_first)
// the time up to `tr_first` (taken inside the phase) goes to phase a, the rest to phase b
#define FRNN_TRACE_SPLIT(a, b) { __builtin_amdgcn_sched_barrier(0); const unsigned long long tr_n = __builtin_amdgcn_s_memtime(); \
                                 if (tr_first > tr_t && tr_first <= tr_n) { tr_acc[a] += tr_first - tr_t; tr_acc[b] += tr_n - tr_first; } else tr_acc[b] += tr_n - tr_t; \
                                 tr_t = tr_n; tr_first = 0; __builtin_amdgcn_sched_barrier(0); }
#define FRNN_TRACE_RESET() { __builtin_amdgcn_sched_barrier(0); tr_t = __builtin_amdgcn_s_memtime(); __builtin_amdgcn_sched_barrier(0); }
#define FRNN_TRACE_END(p) if ((p).trace != nullptr && (threadIdx.x & 63) == 0 && (threadIdx.x >> 6) < kTraceWaves) { \
        for (int tr_j = 0; tr_j < kTracePhases; ++tr_j) (p).trace[((size_t)blockIdx.x * kTraceWaves + (threadIdx.x >> 6)) * kTracePhases + tr_j] = tr_acc[tr_j]; }
#else
#define FRNN_TRACE_BEGIN()
#define FRNN_TRACE_FIRST nullptr
#define FRNN_TRACE_SPLIT(a, b)
#define FRNN_TRACE_MARK(i)
#define FRNN_TRACE_RESET()
#define FRNN_TRACE_END(p)
#endif

// ---------------------------------------------------------------------------------------------
// common per-lane geometry
// ---------------------------------------------------------------------------------------------
template <int BT> struct LaneMap {
    static constexpr int PP = BT / 4;  // (unit, batch row) pairs per lane and tile
    int c, quad, bslot, uoff;
    __device__ __forceinline__ LaneMap(int lane) {
        c = lane & 15;
        quad = lane >> 4;
        if constexpr (BT == 16) { bslot = c; uoff = 4 * quad; }
        else if constexpr (BT == 8) { bslot = c & 7; uoff = 4 * quad + 2 * (c >> 3); }
        else { bslot = c & 3; uoff = 4 * quad + (c >> 2); }
    }
};

// group / member of a workgroup.  With several workgroups per group the members of a group get
// block indices that are equal modulo 8: the hardware hands consecutive workgroups to the 8 XCDs in
// turn, so a group's members share one XCD and its L2.
// A head too large for the registers of one XCD's CUs is spread over all of them (p.spread): consecutive block
// indices, hence all eight XCDs in turn, serve one group; the exchange then goes through memory at agent scope.
struct BlockMap {
    int member, gpar;
    bool active;
    __device__ __forceinline__ BlockMap(const KernelParams& p, bool multi) {
        const int L = blockIdx.x;
        if (multi && p.spread) {
            member = L % p.P;
            gpar = L / p.P;
        } else if (multi) {
            const int xcd = L & 7, slot = L >> 3;
            member = slot % p.P;
            gpar = (slot / p.P) * 8 + xcd;
        } else {
            member = 0;
            gpar = L;
        }
        active = gpar < p.GPAR;
    }
};

// Waves that share a SIMD (wave w runs on SIMD w % 4) get different issue priorities, so that after the
// per-step barrier the first wave of a SIMD takes the matrix pipe first and its point-wise phase overlaps the
// next wave's MFMA chain.  (The hardware already tends to serve the oldest wave first: measured, the
// priorities change the step time by less than 1 %; they are kept because they make that order explicit.)
__device__ __forceinline__ void stagger_waves(int w) {
    const int slot = w >> 2;
    if (slot == 0) __builtin_amdgcn_s_setprio(3);
    else if (slot == 1) __builtin_amdgcn_s_setprio(2);
    else if (slot == 2) __builtin_amdgcn_s_setprio(1);
    else __builtin_amdgcn_s_setprio(0);
}

// ---------------------------------------------------------------------------------------------
// operand hand-over between waves: LDS (one workgroup per group) or stamped words in global memory
// ---------------------------------------------------------------------------------------------
// Exchange word = 8 bytes {payload, stamp}: payload is two bf16 or one float.  A consumer polls the
// words it needs until every stamp equals the one it expects; a word is written by one aligned
// 8- or 16-byte store, so payload and stamp always arrive together and no fence is needed.  Stores and
// loads carry the agent-scope cache policy.  Two buffers alternate; writing round r+1 requires having
// read round r from every member, which implies every member has finished reading round r-1.
// The operand rows of a group (`rows` of them, cpr chunks of 16 bytes = two stamped
// words per row, rows xrow bytes apart from byte offset goff of rs) are polled once, NT threads taking consecutive
// chunks, and their payloads go to LDS rows (lds_pitch bytes apart, plain element order).  The waves then read
// their MFMA operands from LDS like the one-workgroup kernels do (every wave polling every row in L2 itself
// measured 1.2x to 1.5x slower at D = 256 and 768).  The loads are marked volatile: every round goes to memory again.
// Returns false on a timeout (the error word is set; the caller stops waiting from then on).
// Everything about a thread's chunks that does not change from step to step is formed once per kernel (Poller): the
// global and LDS offsets of its first NB chunks and how many of them its wave really has.  A step then only supplies the
// (uniform) offset of the buffer in use as the scalar offset of the loads.  Forming the offsets inside the time loop --
// sixteen integer divisions and a hundred more instructions per thread and step -- cost more than the hand-over itself
// (measured: 2000 of 7500 clocks per step at D = 256).
struct Poller {
    static constexpr int NBP = 2;  // chunks per thread whose offsets are kept for the whole kernel (the usual shapes need no more)
    static constexpr int NB = 8;   // chunks per thread and round beyond those (a round costs one L2 round trip: few rounds)
    static constexpr uint32_t kDrop = 0x80000000u;
    uint32_t voff[NBP], loff[NBP];  // first round: byte offset inside the group's rows (kDrop = no chunk), LDS offset
    int nb;                         // chunks of this wave in the first round
    uint32_t total, cpr, xrow, lds_pitch, tid, NT;
    uint32_t row, c, dq, dr;        // position of chunk tid + NBP * NT and the step to the chunk NT further on
    __device__ __forceinline__ Poller(uint32_t tid_, uint32_t NT_, uint32_t rows, uint32_t cpr_, uint32_t xrow_, uint32_t lds_pitch_)
        : total(rows * cpr_), cpr(cpr_), xrow(xrow_), lds_pitch(lds_pitch_), tid(tid_), NT(NT_) {
        row = tid / cpr; c = tid % cpr; dq = NT / cpr; dr = NT % cpr;
#pragma unroll
        for (int j = 0; j < NBP; ++j) place(tid + (uint32_t)j * NT, voff[j], loff[j]);
        const uint32_t wave_first = tid & ~63u;
        nb = wave_first >= total ? 0 : (int)min((uint32_t)NBP, (total - wave_first + NT - 1) / NT);
    }
    // offsets of chunk idx (the running position is at idx) and the advance to chunk idx + NT
    __device__ __forceinline__ void place(uint32_t idx, uint32_t& vo, uint32_t& lo) {
        vo = idx < total ? row * xrow + c * 16u : kDrop;
        lo = row * lds_pitch + c * 8u;
        row += dq;
        c += dr;
        if (c >= cpr) { c -= cpr; ++row; }
    }
    // one set of up to N chunks: poll until every stamp is there, then move the payloads to LDS
    template <int N>
    __device__ __forceinline__ bool round(__amdgpu_buffer_rsrc_t rs, uint32_t goff, const uint32_t (&vo)[N], const uint32_t (&lo)[N], int n, char* lds,
                                          uint32_t stamp, int spin_limit, int* err, unsigned long long* first_round) const {
        constexpr int kAuxPoll = (int)(0x80000000u | (unsigned)kAuxAgent);
        i32x4 raw[N];
        bool good = true;
        for (int spins = 0;; ++spins) {
            // (a load whose lanes are all out of range still costs its issue slot in the memory pipeline: only the n real ones)
#pragma unroll
            for (int j = 0; j < N; ++j)
                if (j < n) raw[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, vo[j], goff, kAuxPoll);
            bool ok = true;
#pragma unroll
            for (int j = 0; j < N; ++j)
                if (j < n) ok = ok && (vo[j] == kDrop || ((uint32_t)raw[j][1] == stamp && (uint32_t)raw[j][3] == stamp));
#ifdef FLASHRNN_TRACE
            if (first_round != nullptr && spins == 0) { asm volatile("" : : "v"(ok) : "memory"); *first_round = __builtin_amdgcn_s_memtime(); }
#else
            (void)first_round;
#endif
            if (__all((int)ok)) break;
            if (spins > spin_limit) {
                __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                good = false;
                break;
            }
            if ((spins & 255) == 255 && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { good = false; break; }
        }
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j < n && vo[j] != kDrop) *(i32x2*)(lds + lo[j]) = i32x2{raw[j][0], raw[j][2]};
        return good;
    }
    // goff: byte offset of the group's rows in the buffer in use (uniform).  Returns false on a timeout.
    __device__ __forceinline__ bool poll(__amdgpu_buffer_rsrc_t rs, uint32_t goff, char* lds, uint32_t stamp, int spin_limit, int* err,
                                         unsigned long long* first_round = nullptr) const {
        if (spin_limit < 0) {   // host-forced failure (tests of the error path): give up without looking
            __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        bool good = round<NBP>(rs, goff, voff, loff, nb, lds, stamp, spin_limit, err, first_round);
        if (total > NT * NBP) {   // long rows: further sets, their offsets formed on the way
            Poller run = *this;
            for (uint32_t base = NT * NBP; base < total && good; base += NT * NB) {
                uint32_t vo[NB], lo[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j) run.place(base + tid + (uint32_t)j * NT, vo[j], lo[j]);
                good = round<NB>(rs, goff, vo, lo, NB, lds, stamp, spin_limit, err, nullptr);
            }
        }
        return good;
    }
};

// write PP = 4 consecutive operand elements of one row as stamped words.  far = the group's workgroups sit on several
// XCDs: the store must go through to memory (agent scope).  Inside one XCD the L2 is the point of coherence and an
// ordinary store reaches it (the vector L1 writes through); it is acknowledged by the L2, not by memory, which matters
// because a wave's memory operations retire in order: the next poll's first answer waits for this store's acknowledgement
// (measured: 0.9 us per step with the write-through store).
template <bool BF16>
__device__ __forceinline__ void publish4(__amdgpu_buffer_rsrc_t rs, uint32_t row_off, int k, const float (&v)[4], uint32_t stamp, bool far) {
    if constexpr (BF16) {
        const i32x4 w = {(int)pack_bf16x2(v[0], v[1]), (int)stamp, (int)pack_bf16x2(v[2], v[3]), (int)stamp};
        if (far) __builtin_amdgcn_raw_buffer_store_b128(w, rs, row_off + k * 4, 0, kAuxAgent);
        else __builtin_amdgcn_raw_buffer_store_b128(w, rs, row_off + k * 4, 0, 0);
    } else {
        const i32x4 w0 = {__builtin_bit_cast(int, v[0]), (int)stamp, __builtin_bit_cast(int, v[1]), (int)stamp};
        const i32x4 w1 = {__builtin_bit_cast(int, v[2]), (int)stamp, __builtin_bit_cast(int, v[3]), (int)stamp};
        if (far) {
            __builtin_amdgcn_raw_buffer_store_b128(w0, rs, row_off + k * 8, 0, kAuxAgent);
            __builtin_amdgcn_raw_buffer_store_b128(w1, rs, row_off + k * 8 + 16, 0, kAuxAgent);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(w0, rs, row_off + k * 8, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(w1, rs, row_off + k * 8 + 16, 0, 0);
        }
    }
}

// A wave publishes its 16 units of the group's BT rows: with BT < 16 the lanes c < BT collect the four consecutive
// units 4q..4q+3 of their batch row first (every lane holds fewer values there), the other lanes' stores are dropped.
template <bool BF16, int BT, int PP>
__device__ __forceinline__ void publish_tile(__amdgpu_buffer_rsrc_t rs, uint32_t group_off, uint32_t xrow, const LaneMap<BT>& lm, int k_wave,
                                             const float (&v)[PP], uint32_t stamp, bool far) {
    float v4[4];
    expand_tile<BT, PP>(v, v4);
    const uint32_t row_off = lm.c < BT ? group_off + (uint32_t)lm.c * xrow : 0x80000000u;
    publish4<BF16>(rs, row_off, k_wave + 4 * lm.quad, v4, stamp, far);
}

// KC consecutive k-steps (64 bytes apart) of the B operand, read by the lanes of the valid batch columns only, under one
// execution mask.  The other lanes' registers keep whatever they held: a column of the B operand only reaches the same
// column of the result, and the columns c >= BT of a result are never used (the empty asm statements stand for "any
// value": without them the compiler would give the idle lanes a defined value, one move per register).  An LDS read costs
// bandwidth per active lane, and the backward step of a split group, whose waves read all G * D gate gradients, is bound by the LDS.
template <int BT, int KC, bool MASKED> __device__ __forceinline__ void lds_operand_chunk(const char* p, int c, bf16x8 (&out)[KC]) {
    if constexpr (BT == 16 || !MASKED) {
#pragma unroll
        for (int j = 0; j < KC; ++j) out[j] = *(const bf16x8*)(p + j * 64);
    } else {
        i32x4 raw[KC];
#pragma unroll
        for (int j = 0; j < KC; ++j) asm volatile("" : "=v"(raw[j]));
        if (c < BT) {
#pragma unroll
            for (int j = 0; j < KC; ++j) raw[j] = *(const i32x4*)(p + j * 64);
        }
#pragma unroll
        for (int j = 0; j < KC; ++j) out[j] = __builtin_bit_cast(bf16x8, raw[j]);
    }
}

// LDS operand row: element type bf16 (as uint16) or float
template <bool BF16, int KT>
__device__ __forceinline__ void read_operand_lds(const char* row, int k0, int quad, typename Operand<BF16>::type (&hB)[KT]) {
    if constexpr (BF16) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) hB[kt] = *(const bf16x8*)(row + (size_t)(k0 + kt * 32 + quad * 8) * 2);
    } else {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) hB[kt] = *(const float*)(row + (size_t)(k0 + quad * KT + kt) * 4);
    }
}

template <bool BF16, int PP> __device__ __forceinline__ void write_operand_lds(char* row, int k, const float (&v)[PP]) {
    if constexpr (BF16) {
        if constexpr (PP == 4) {
            uint2 o;
            o.x = pack_bf16x2(v[0], v[1]);
            o.y = pack_bf16x2(v[2], v[3]);
            *(uint2*)(row + k * 2) = o;
        } else if constexpr (PP == 2) {
            *(uint32_t*)(row + k * 2) = pack_bf16x2(v[0], v[1]);
        } else {
            *(uint16_t*)(row + k * 2) = (uint16_t)f32_to_bf16_bits(v[0]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < PP; ++i) *(float*)(row + (k + i) * 4) = v[i];
    }
}

// partial sums of the KS contraction slices meet in LDS: slices 1.. write, slice 0 adds.  A lane's four values of a tile
// travel as one 16-byte access (64 lanes x 16 bytes back to back: no bank conflicts, a quarter of the LDS instructions).
// Only the lanes of the BT valid batch columns take part (the others' sums are never used, and LDS traffic costs per active lane).
template <int NT, int KS, int BT>
__device__ __forceinline__ void reduce_slices(float* red, int parity, int ks, int wu, int NWU, int lane, f32x4 (&acc)[NT]) {
    if constexpr (KS > 1) {
        const bool valid = BT == 16 || (lane & 15) < BT;
        if (ks > 0 && valid) {
#pragma unroll
            for (int g = 0; g < NT; ++g)
                *(f32x4*)(red + (((((size_t)(parity * (KS - 1) + ks - 1) * NWU + wu) * NT + g) * 64 + lane) * 4)) = acc[g];
        }
        __syncthreads();
        if (ks == 0 && valid) {
#pragma unroll
            for (int s = 1; s < KS; ++s)
#pragma unroll
                for (int g = 0; g < NT; ++g)
                    acc[g] += *(const f32x4*)(red + (((((size_t)(parity * (KS - 1) + s - 1) * NWU + wu) * NT + g) * 64 + lane) * 4));
        }
    }
}

// =============================================================================================
// forward
// =============================================================================================
// CELL, BF16 (I/O dtype), KT k-steps per wave, KS contraction slices, BT valid batch slots per tile,
// MULTI several workgroups per group, MAXW launch bound in waves.
// p.R is the packed forward copy of R: Rt[n][g][e][k], k < DK = KT*KS*KSTEP, zero beyond D.
// The launch guarantees P * NWU * 16 == D and DK >= D (operand rows and packed R are zero beyond D).
// Global addresses are formed as (uniform base advanced per step on the scalar unit) + (32-bit lane offset).
template <bool BF16> constexpr int poll_chunk(int KT) {
    if (!BF16) return 8;
    if (KT <= 6) return KT;
    return KT % 6 == 0 ? 6 : KT % 4 == 0 ? 4 : KT % 3 == 0 ? 3 : KT % 2 == 0 ? 2 : 1;
}

// EB = blocks of 16 units per wave: the wave reads the operand h once and uses it for all of them.
template <int CELL, bool BF16, int KT, int KS, int BT, bool MULTI, int MAXW, int EB = 1>
__global__ __launch_bounds__(MAXW * 64) void fwd_kernel(const KernelParams p) {
    using CT = CellTraits<CELL>;
    using OP = Operand<BF16>;
    using op_t = typename OP::type;
    constexpr int G = CT::G, S = CT::S, NC = CT::NC;
    constexpr int PP = BT / 4;
    constexpr int ESZ = BF16 ? 2 : 4;               // element size of the I/O dtype and of LDS operand rows
    constexpr int DK = KT * KS * OP::KSTEP;         // padded contraction length
    constexpr int HP = DK + (BF16 ? 8 : 4);         // LDS row pitch in elements
    constexpr int BUF = BT * HP * ESZ;              // bytes of one LDS operand buffer
    constexpr int KC = poll_chunk<BF16>(KT);
    static_assert(KS == 1 || MULTI, "contraction slices are only used with several workgroups per group");
    static_assert(!MULTI || KT % KC == 0, "poll chunks must tile the k-steps");
    static_assert(EB == 1 || !MULTI, "several unit blocks per wave only with one workgroup per group");

    extern __shared__ __align__(16) char smem[];
    const BlockMap bm(p, MULTI);
    if (!bm.active) return;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wu = w % p.NWU, ks = w / p.NWU;
    stagger_waves(w);
    const LaneMap<BT> lm(lane);
    const int T = p.T, B = p.B, NH = p.NH, D = p.D;
    const int e_wave = (bm.member * p.NWU + wu) * 16 * EB;  // first unit of this wave
    const int e0 = e_wave + lm.uoff;                    // first unit of this lane's pairs
    const int k0 = ks * KT * OP::KSTEP;

    char* hbuf = smem;                                          // !MULTI: [2][BT][HP] operand rows
    float* red = (float*)(smem + (MULTI ? BUF : 0));            // MULTI: one operand buffer [BT][HP], then (KS > 1) the partial sums
    __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(p.exch, 0, 0x7FFFFFFF, 0x00020000);
    constexpr uint32_t XROW = DK * (BF16 ? 4 : 8);             // bytes per exchange row
    const uint32_t xgroup = (uint32_t)bm.gpar * BT * XROW;     // this group's BT rows inside one buffer
    const uint32_t xbuf = (uint32_t)p.GPAR * BT * XROW;        // bytes per buffer
    bool failed = false;
    const Poller poller(MULTI ? threadIdx.x : 0u, MULTI ? blockDim.x : 64u, MULTI ? BT : 0, (uint32_t)p.D * (BF16 ? 4 : 8) / 16, XROW, HP * ESZ);
    FRNN_TRACE_BEGIN();

    // uniform strides in bytes
    const uint32_t HD = (uint32_t)NH * D;
    const size_t wx_step = (size_t)B * G * HD * ESZ;
    const uint32_t wx_gate = HD * ESZ;
    const size_t st_step = (size_t)S * B * HD * 4;
    const uint32_t st_state = (uint32_t)B * HD * 4;
    constexpr uint32_t REC = CT::RS * ESZ;                      // bytes of one saved-values record
    const size_t c_step = (size_t)B * HD * REC;
    // LDS lane offsets inside one operand buffer
    const uint32_t lds_rd = (uint32_t)lm.bslot * HP * ESZ;     // row this lane reads as the B operand column
    const uint32_t lds_wr = (uint32_t)lm.bslot * HP * ESZ;     // row this lane writes its new h into

    int iter = 0;
    for (int gid = bm.gpar; gid < p.NG; gid += p.GPAR, ++iter) {
        const int n = gid % NH, q = gid / NH;
        // ---- load once per group: R fragments (A operand: row = unit e_wave + c) and bias; they stay
        // in registers for all T steps
        op_t Rf[EB][G][KT];
        float bias[EB][G][PP];
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const size_t rrow = (((size_t)n * G + g) * D + e_wave + 16 * eb + lm.c) * DK;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                if constexpr (BF16) Rf[eb][g][kt] = *(const bf16x8*)((const uint16_t*)p.R + rrow + k_index<BF16, KT>(k0, kt, lm.quad, 0));
                else Rf[eb][g][kt] = ((const float*)p.R)[rrow + k_index<BF16, KT>(k0, kt, lm.quad, 0)];
            }
            load_io<BF16, PP>(p.bias, ((size_t)n * G + g) * D + e0 + 16 * eb, bias[eb][g]);
        }

        const int bb_raw = q * BT + lm.bslot;
        const bool row_valid = bb_raw < B;
        const int bb = row_valid ? bb_raw : B - 1;
        const bool lane_ok = row_valid && ks == 0;
        // per-group uniform bases and per-lane offsets
        const char* wx_g = (const char*)p.Wx + (size_t)n * D * ESZ;
        char* st_g = (char*)p.states + (size_t)n * D * 4;
        char* c_g = (char*)p.cache + (size_t)n * D * REC;
        constexpr uint32_t kDrop = 0x80000000u;  // beyond every resource's range: the access is dropped
        const uint32_t voff_wx = ((uint32_t)bb * G * HD + e0) * ESZ;
        const uint32_t voff_st = ((uint32_t)bb * HD + e0) * 4;
        const uint32_t soff_st = lane_ok ? voff_st : kDrop;
        const uint32_t soff_c = (lane_ok && p.cache != nullptr) ? ((uint32_t)bb * HD + e0) * REC : kDrop;

        // ---- initial states
        float st[EB][S][PP];
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (p.states0 != nullptr) load_io_r<false, PP>(make_rsrc((const char*)p.states0 + (size_t)n * D * 4), voff_st + eb * 64, s * st_state, st[eb][s]);
            else
#pragma unroll
                for (int i = 0; i < PP; ++i) st[eb][s][i] = 0.0f;
            store_io_r<false, PP>(make_rsrc(st_g), soff_st + eb * 64, s * st_state, st[eb][s]);
        }
        if constexpr (MULTI) {   // the polled rows fill the first D elements; the padding up to DK stays zero
            __syncthreads();
            for (int j = threadIdx.x; j < BUF / 4; j += blockDim.x) ((uint32_t*)hbuf)[j] = 0u;
        }
        if constexpr (!MULTI) {
            __syncthreads();  // the previous group is done with the operand rows
            for (int j = threadIdx.x; j < 2 * BUF / 4; j += blockDim.x) ((uint32_t*)hbuf)[j] = 0u;
            __syncthreads();
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) write_operand_lds<BF16, PP>(hbuf + lds_wr, e0 + 16 * eb, st[eb][0]);
            __syncthreads();
        } else {
            if (ks == 0 && T > 0) {
                const uint32_t cnt = (uint32_t)iter * (uint32_t)T;
                publish_tile<BF16, BT, PP>(xr, (cnt & 1u) * xbuf + xgroup, XROW, lm, e_wave, st[0][0], cnt + 1u, p.spread != 0);
            }
        }

        // input pre-activations are fetched one step ahead
        float wx[EB][G][PP];
        if (T > 0) {
#pragma unroll
            for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int g = 0; g < G; ++g) load_io_r<BF16, PP>(make_rsrc(wx_g), voff_wx + eb * 16 * ESZ, g * wx_gate, wx[eb][g]);
        }

        FRNN_TRACE_RESET();
        for (int t = 1; t <= T; ++t) {
            // ---- prefetch the inputs of step t + 1 (clamped at the end).  A wave's vector memory operations retire in
            // order: with several workgroups per group the loads are issued behind the poll for h_{t-1}, not in front of it
            // (the poll's first answer would otherwise wait for these to come back from HBM: measured 1.2 us per step)
            float wxn[EB][G][PP];
            auto prefetch_inputs = [&]() {
                const rsrc_t rsn = make_rsrc(wx_g + (size_t)(t < T ? t : T - 1) * wx_step);
#pragma unroll
                for (int eb = 0; eb < EB; ++eb)
#pragma unroll
                for (int g = 0; g < G; ++g) load_io_r<BF16, PP>(rsn, voff_wx + eb * 16 * ESZ, g * wx_gate, wxn[eb][g]);
            };
            if constexpr (!MULTI) prefetch_inputs();
            // ---- recurrent product y = R^T h_{t-1} on the matrix cores
            f32x4 accs[EB][G];
#pragma unroll
            for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int g = 0; g < G; ++g) accs[eb][g] = f32x4{0.f, 0.f, 0.f, 0.f};
            f32x4 (&acc)[G] = accs[0];
            if constexpr (!MULTI) {
                op_t hB[KT];
                read_operand_lds<BF16, KT>(hbuf + ((t - 1) & 1) * BUF + lds_rd, k0, lm.quad, hB);
#pragma unroll
                for (int eb = 0; eb < EB; ++eb)
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int g = 0; g < G; ++g) accs[eb][g] = OP::mfma(Rf[eb][g][kt], hB[kt], accs[eb][g]);
            } else {
                // h_{t-1} of the whole group: polled once per workgroup into LDS, then read like in the one-workgroup case
                const uint32_t cnt = (uint32_t)iter * (uint32_t)T + (uint32_t)(t - 1);
                FRNN_TRACE_MARK(0);
                __syncthreads();   // every wave has read the previous step's rows
                FRNN_TRACE_MARK(1);
                if (!failed) failed = !poller.poll(xr, (cnt & 1u) * xbuf + xgroup, hbuf, cnt + 1u, p.spin_limit, p.err, FRNN_TRACE_FIRST);
                FRNN_TRACE_SPLIT(7, 2);
                __syncthreads();
                FRNN_TRACE_MARK(3);
                prefetch_inputs();
#pragma unroll
                for (int kc = 0; kc < KT; kc += KC) {
                    op_t hB[KC];
                    if constexpr (BF16) {
                        // (forward: worth it from 8 k-steps per wave on; with shorter rows the LDS is not what bounds the step)
                        lds_operand_chunk<BT, KC, (KT >= 8)>(hbuf + lds_rd + (size_t)(k0 + kc * 32 + lm.quad * 8) * 2, lm.c, hB);
                    } else {
#pragma unroll
                        for (int j = 0; j < KC; ++j) hB[j] = *(const float*)(hbuf + lds_rd + (size_t)(k0 + lm.quad * KT + kc + j) * 4);
                    }
#pragma unroll
                    for (int j = 0; j < KC; ++j)
#pragma unroll
                        for (int g = 0; g < G; ++g) acc[g] = OP::mfma(Rf[0][g][kc + j], hB[j], acc[g]);
                }
            }
            reduce_slices<G, KS, BT>(red, t & 1, ks, wu, p.NWU, lane, acc);
#ifdef FLASHRNN_TRACE
            if constexpr (MULTI) { asm volatile("" : "+v"(acc[0]), "+v"(acc[G - 1]) : : "memory"); FRNN_TRACE_MARK(4); }
#endif

            if (KS == 1 || ks == 0) {
                float cvs[EB][NC][PP];
#pragma unroll
                for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
                    for (int g = 0; g < G; ++g) compact_tile<BT>(accs[eb][g]);
#pragma unroll
                    for (int i = 0; i < PP; ++i) {
                        float wxi[G], ybi[G], sti[S], cvi[NC];
#pragma unroll
                        for (int g = 0; g < G; ++g) { wxi[g] = wx[eb][g][i]; ybi[g] = accs[eb][g][i] + bias[eb][g][i]; }
#pragma unroll
                        for (int s = 0; s < S; ++s) sti[s] = st[eb][s][i];
                        Cell<CELL, BF16>::fwd(wxi, ybi, sti, cvi);
#pragma unroll
                        for (int s = 0; s < S; ++s) st[eb][s][i] = sti[s];
#pragma unroll
                        for (int c2 = 0; c2 < NC; ++c2) cvs[eb][c2][i] = cvi[c2];
                    }
                    // ---- hand the new h to the other waves as soon as it exists
                    if constexpr (!MULTI) {
                        write_operand_lds<BF16, PP>(hbuf + (t & 1) * BUF + lds_wr, e0 + 16 * eb, st[eb][0]);
                    } else {
                        // (the last step has nobody to hand its h to: its stores are issued all the same, out of range and dropped.
                        // Under a condition the compiler could no longer count this store among the memory operations behind the
                        // input prefetch, and the wait for the prefetched inputs below would wait for its acknowledgement as well.)
                        const uint32_t cnt = (uint32_t)iter * (uint32_t)T + (uint32_t)t;
                        publish_tile<BF16, BT, PP>(xr, t < T ? (cnt & 1u) * xbuf + xgroup : 0x80000000u, XROW, lm, e_wave, st[0][0], cnt + 1u, p.spread != 0);
                    }
                }
                if constexpr (MULTI) FRNN_TRACE_MARK(5);
                // stores of lanes without a valid row (and of the saved values in a forward-only call) carry
                // an out-of-range offset and are dropped by the buffer bounds check: no branch, so the
                // wait for the prefetched inputs at the end of the step does not have to cover them
                {
                    const rsrc_t rs_st = make_rsrc(st_g + (size_t)t * st_step);
                    const rsrc_t rs_c = make_rsrc(c_g + (size_t)(t - 1) * c_step);
#pragma unroll
                    for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
                        for (int s = 0; s < S; ++s) store_io_r<false, PP>(rs_st, soff_st + eb * 64, s * st_state, st[eb][s]);
#pragma unroll
                        for (int i = 0; i < PP; ++i) {
                            float rec[NC];
#pragma unroll
                            for (int c2 = 0; c2 < NC; ++c2) rec[c2] = cvs[eb][c2][i];
                            store_record<BF16, CT::RS, NC>(rs_c, soff_c + (eb * 16 + i) * REC, 0, rec);
                        }
                    }
                }
            }
#pragma unroll
            for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int i = 0; i < PP; ++i) wx[eb][g][i] = wxn[eb][g][i];
            if constexpr (!MULTI) __syncthreads();
#ifdef FLASHRNN_TRACE
            if constexpr (MULTI) { pin(wx[0]); FRNN_TRACE_MARK(6); }
#endif
        }
    }
    FRNN_TRACE_END(p);
}

// =============================================================================================
// backward
// =============================================================================================
// Wave owns 16 previous-state indices d (= its 16 units) and one of KS slices of the contraction
// axis k = gate * D + unit (length G*D, padded to DK = KT*KS*KSTEP).  KT counts k-steps per wave.
// p.R is the packed backward copy of R: Rb[n][d][k], k < DK, zero beyond G*D.
// The launch guarantees P * NWU * 16 == D, and with MULTI also DK == G*D.
template <int CELL, bool BF16, int KT, int KS, int BT, bool MULTI, int MAXW, int EB = 1>
__global__ __launch_bounds__(MAXW * 64) void bwd_kernel(const KernelParams p) {
    using CT = CellTraits<CELL>;
    using OP = Operand<BF16>;
    using op_t = typename OP::type;
    constexpr int G = CT::G, S = CT::S, NC = CT::NC;
    constexpr int PP = BT / 4;
    constexpr int ESZ = BF16 ? 2 : 4;
    constexpr int DK = KT * KS * OP::KSTEP;
    constexpr int HP = DK + (BF16 ? 8 : 4);
    constexpr int BUF = BT * HP * ESZ;
    constexpr int KC = poll_chunk<BF16>(KT);
    static_assert(KS == 1 || MULTI, "contraction slices are only used with several workgroups per group");
    static_assert(!MULTI || KT % KC == 0, "poll chunks must tile the k-steps");
    static_assert(EB == 1 || !MULTI, "several unit blocks per wave only with one workgroup per group");

    extern __shared__ __align__(16) char smem[];
    const BlockMap bm(p, MULTI);
    if (!bm.active) return;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int wu = w % p.NWU, ks = w / p.NWU;
    stagger_waves(w);
    const LaneMap<BT> lm(lane);
    const int T = p.T, B = p.B, NH = p.NH, D = p.D;
    const int e_wave = (bm.member * p.NWU + wu) * 16 * EB;
    const int e0 = e_wave + lm.uoff;
    const int k0 = ks * KT * OP::KSTEP;

    char* gbuf = smem;          // !MULTI: [2][BT][HP] gate-gradient rows
    float* red = (float*)(smem + (MULTI ? BUF : 0));  // MULTI: one operand buffer [16][HP], then (KS > 1) the partial sums
    __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(p.exch, 0, 0x7FFFFFFF, 0x00020000);
    constexpr uint32_t XROW = DK * (BF16 ? 4 : 8);
    const uint32_t xgroup = (uint32_t)bm.gpar * BT * XROW;
    const uint32_t xbuf = (uint32_t)p.GPAR * BT * XROW;
    bool failed = false;
    const Poller poller(MULTI ? threadIdx.x : 0u, MULTI ? blockDim.x : 64u, MULTI ? BT : 0, (uint32_t)(G * p.D) * (BF16 ? 4 : 8) / 16, XROW, HP * ESZ);
    FRNN_TRACE_BEGIN();

    const uint32_t HD = (uint32_t)NH * D;
    const size_t wx_step = (size_t)B * G * HD * ESZ;
    const uint32_t wx_gate = HD * ESZ;
    const size_t st_step = (size_t)S * B * HD * 4;
    const uint32_t st_state = (uint32_t)B * HD * 4;
    constexpr uint32_t REC = CT::RS * ESZ;                      // bytes of one saved-values record
    const size_t c_step = (size_t)B * HD * REC;
    const size_t dh_step = (size_t)B * HD * ESZ;
    const uint32_t lds_row = (uint32_t)lm.bslot * HP * ESZ;

    int iter = 0;
    for (int gid = bm.gpar; gid < p.NG; gid += p.GPAR, ++iter) {
        const int n = gid % NH, q = gid / NH;
        // ---- load once per group: R fragments, A operand row = previous-state index d = e_wave + c
        op_t Rf[EB][KT];
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) {
            const size_t rrow = ((size_t)n * D + e_wave + 16 * eb + lm.c) * DK;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                if constexpr (BF16) Rf[eb][kt] = *(const bf16x8*)((const uint16_t*)p.R + rrow + k_index<BF16, KT>(k0, kt, lm.quad, 0));
                else Rf[eb][kt] = ((const float*)p.R)[rrow + k_index<BF16, KT>(k0, kt, lm.quad, 0)];
            }
        }
        const int bb_raw = q * BT + lm.bslot;
        const bool row_valid = bb_raw < B;
        const int bb = row_valid ? bb_raw : B - 1;
        const bool lane_ok = row_valid && ks == 0;
        const char* c_g = (const char*)p.cache + (size_t)n * D * REC;
        const char* st_g = (const char*)p.states + (size_t)n * D * 4;
        const char* dh_g = (const char*)p.dH + (size_t)n * D * ESZ;
        char* dwx_g = (char*)p.dWx + (size_t)n * D * ESZ;
        char* dgn_g = (char*)p.dgn + (size_t)n * D * ESZ;
        constexpr uint32_t kDrop = 0x80000000u;  // beyond every resource's range: the access is dropped
        const uint32_t voff_st = ((uint32_t)bb * HD + e0) * 4;
        const uint32_t voff_c = ((uint32_t)bb * HD + e0) * REC;
        const uint32_t voff_dh = ((uint32_t)bb * HD + e0) * ESZ;
        const uint32_t soff_wx = lane_ok ? ((uint32_t)bb * G * HD + e0) * ESZ : kDrop;
        const uint32_t soff_dh = lane_ok ? voff_dh : kDrop;

        // With several workgroups per group the polled rows in LDS are the complete dg_t of the group's batch rows -- which,
        // for every cell but the GRU, is dWx_t as well: the group's threads move them out as 16-byte chunks (each thread
        // at most NBO of them, fixed for the group) instead of every lane storing four 2-byte values of its own.
        constexpr bool kOutRows = MULTI && CELL != CELL_GRU;
        constexpr int NBO = BF16 ? 2 : 4;
        uint32_t out_g[NBO], out_l[NBO];   // byte offset inside a step's dWx (dropped if there is no chunk), byte offset in the LDS rows
        if constexpr (kOutRows) {
            const uint32_t EPC = 16 / ESZ, cpg = (uint32_t)D / EPC, cprow = (uint32_t)G * cpg, total = (uint32_t)BT * cprow;
            const uint32_t TG = (uint32_t)p.P * blockDim.x;
#pragma unroll
            for (int j = 0; j < NBO; ++j) {
                const uint32_t ci = (uint32_t)bm.member * blockDim.x + threadIdx.x + (uint32_t)j * TG;
                const uint32_t r = ci / cprow, rem = ci % cprow, g2 = rem / cpg, ch = rem % cpg, brow = (uint32_t)q * BT + r;
                const bool ok = ci < total && brow < (uint32_t)B;
                out_g[j] = ok ? ((brow * G + g2) * HD) * ESZ + ch * 16 : 0x80000000u;
                out_l[j] = ok ? r * (uint32_t)(HP * ESZ) + rem * 16 : 0u;
            }
        }

        // carried state gradients; ds[0] is the part of dh_t that came through R and the direct path
        float ds[EB][S][PP];
        float dbacc[EB][G][PP];
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (p.dlast != nullptr && !(CELL == CELL_SLSTM && s == 3))
                load_io_r<false, PP>(make_rsrc((const char*)p.dlast + (size_t)n * D * 4), voff_st + eb * 64, s * st_state, ds[eb][s]);
            else
#pragma unroll
                for (int i = 0; i < PP; ++i) ds[eb][s][i] = 0.0f;
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < PP; ++i) dbacc[eb][g][i] = 0.0f;
        }

        {   // operand rows start from zero (with MULTI one buffer: the polled rows fill the first G*D elements)
            __syncthreads();
            for (int j = threadIdx.x; j < (MULTI ? 1 : 2) * BUF / 4; j += blockDim.x) ((uint32_t*)gbuf)[j] = 0u;
            __syncthreads();
        }

        // inputs of a step: saved values, the states the cell's Jacobian needs, external dh
        float cv[EB][NC][PP], sc[EB][S][PP], sp[EB][S][PP], dh_ext[EB][PP];
        // The streams move by whole time steps: their bases are carried as pointers (a product of the step index and a 64-bit
        // stride per stream and step is a dozen scalar instructions, in a step that is one chain of dependent instructions:
        // measured 3 % of the step on sLSTM heads of 256 units, 10 % on GRU heads).  The three input
        // streams point at the step that is loaded next; `more` = a further (earlier) step follows, else step 1 is loaded again.
        // (Kernels with contraction slices, and those with three waves per SIMD, have no register to spare: they keep forming the bases from the step
        // index, whose temporaries are short-lived.)
        constexpr bool kRunning = KS == 1 && MAXW < 12;
        const int t_last = T > 0 ? T - 1 : 0;
        const char* c_run = c_g + (size_t)t_last * c_step;      // saved values of that step
        const char* st_run = st_g + (size_t)t_last * st_step;   // states before it (the states after it: one step further on)
        const char* dh_run = dh_g + (size_t)t_last * dh_step;
        char* dwx_run = dwx_g + (size_t)t_last * wx_step;       // dWx (and the GRU's candidate-gate gradient) of the current step
        char* dgn_run = dgn_g + (size_t)t_last * dh_step;
        auto load_step = [&](int t, bool more, float (&cv_)[EB][NC][PP], float (&sc_)[EB][S][PP], float (&sp_)[EB][S][PP], float (&dh_)[EB][PP]) {
            const rsrc_t c_t = make_rsrc(kRunning ? c_run : c_g + (size_t)(t - 1) * c_step);
            const rsrc_t st_p = make_rsrc(kRunning ? st_run : st_g + (size_t)(t - 1) * st_step);
            const rsrc_t dh_t = make_rsrc(kRunning ? dh_run : dh_g + (size_t)(t - 1) * dh_step);
            // the states after the step: one step further on -- as a uniform offset on the same base where the bases are carried
            const rsrc_t st_t = kRunning ? st_p : make_rsrc(st_g + (size_t)t * st_step);
            const uint32_t st_after = kRunning ? (uint32_t)st_step : 0u;
            if constexpr (kRunning) {
                c_run -= more ? c_step : 0;
                st_run -= more ? st_step : 0;
                dh_run -= more ? dh_step : 0;
            }
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                float rec[NC];
                load_record<BF16, CT::RS, NC>(c_t, voff_c + (eb * 16 + i) * REC, 0, rec);
#pragma unroll
                for (int c2 = 0; c2 < NC; ++c2) cv_[eb][c2][i] = rec[c2];
            }
#pragma unroll
            for (int s = 0; s < S; ++s) {
                if (!cell_uses_h_prev(CELL) && s > 0 && s < 3) load_io_r<false, PP>(st_t, voff_st + eb * 64, s * st_state + st_after, sc_[eb][s]);
                else
#pragma unroll
                    for (int i = 0; i < PP; ++i) sc_[eb][s][i] = 1.0f;
                if (cell_uses_h_prev(CELL) ? (s == 0) : (s > 0 && s < 3)) load_io_r<false, PP>(st_p, voff_st + eb * 64, s * st_state, sp_[eb][s]);
                else
#pragma unroll
                    for (int i = 0; i < PP; ++i) sp_[eb][s][i] = 1.0f;
            }
            load_io_r<BF16, PP>(dh_t, voff_dh + eb * 16 * ESZ, 0, dh_[eb]);
            }
        };
        if ((KS == 1 || ks == 0) && T > 0) load_step(T, T > 1, cv, sc, sp, dh_ext);

        FRNN_TRACE_RESET();
        for (int t = T; t >= 1; --t) {
            float cvn[EB][NC][PP], scn[EB][S][PP], spn[EB][S][PP], dhn[EB][PP];
            if (KS == 1 || ks == 0) {
                // ---- prefetch the inputs of the next (earlier) step; they are pinned after the MFMA phase
                // (with several workgroups per group they are issued behind the poll for dg_t: see the forward kernel)
                if constexpr (!MULTI) load_step(t > 1 ? t - 1 : 1, t > 2, cvn, scn, spn, dhn);
                // ---- point-wise Jacobians
                const rsrc_t dwx_t = make_rsrc(kRunning ? dwx_run : dwx_g + (size_t)(t - 1) * wx_step);
#pragma unroll
                for (int eb = 0; eb < EB; ++eb) {
                    float dwx[G][PP], dg[G][PP];
#pragma unroll
                    for (int i = 0; i < PP; ++i) {
                        float cvi[NC], sci[S], spi[S], dsi[S], dwxi[G], dgi[G];
#pragma unroll
                        for (int c2 = 0; c2 < NC; ++c2) cvi[c2] = cv[eb][c2][i];
#pragma unroll
                        for (int s = 0; s < S; ++s) { sci[s] = sc[eb][s][i]; spi[s] = sp[eb][s][i]; dsi[s] = ds[eb][s][i]; }
                        dsi[0] += dh_ext[eb][i];
                        Cell<CELL, BF16>::bwd(cvi, sci, spi, dsi, dwxi, dgi);
#pragma unroll
                        for (int s = 0; s < S; ++s) ds[eb][s][i] = dsi[s];
#pragma unroll
                        for (int g2 = 0; g2 < G; ++g2) { dwx[g2][i] = dwxi[g2]; dg[g2][i] = dgi[g2]; dbacc[eb][g2][i] += dgi[g2]; }
                    }
                    // ---- hand dg_t to the other waves, then stream out dWx
                    if constexpr (!MULTI) {
#pragma unroll
                        for (int g2 = 0; g2 < G; ++g2)
                            write_operand_lds<BF16, PP>(gbuf + (t & 1) * BUF + lds_row, g2 * D + e0 + 16 * eb, dg[g2]);
                    } else {
                        const uint32_t cnt = (uint32_t)iter * (uint32_t)T + (uint32_t)(T - t);
#pragma unroll
                        for (int g2 = 0; g2 < G; ++g2)
                            publish_tile<BF16, BT, PP>(xr, (cnt & 1u) * xbuf + xgroup, XROW, lm, g2 * D + e_wave, dg[g2], cnt + 1u, p.spread != 0);
                    }
                    if constexpr (!kOutRows) {
#pragma unroll
                        for (int g2 = 0; g2 < G; ++g2) store_io_r<BF16, PP>(dwx_t, soff_wx + eb * 16 * ESZ, g2 * wx_gate, dwx[g2]);
                    }
                    if constexpr (CELL == CELL_GRU)
                        store_io_r<BF16, PP>(make_rsrc(kRunning ? dgn_run : dgn_g + (size_t)(t - 1) * dh_step), soff_dh + eb * 16 * ESZ, 0, dg[2]);
                }
            }
            // ---- dh_{t-1} += R dg_t on the matrix cores; NA accumulators per unit block break the dependent chain
            constexpr int NA = EB == 1 ? 4 : 2;
            f32x4 a4[EB][NA];
#pragma unroll
            for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int j = 0; j < NA; ++j) a4[eb][j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (!MULTI) {
                __syncthreads();
                op_t gB[KT];
                read_operand_lds<BF16, KT>(gbuf + (t & 1) * BUF + lds_row, k0, lm.quad, gB);
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int eb = 0; eb < EB; ++eb) a4[eb][kt % NA] = OP::mfma(Rf[eb][kt], gB[kt], a4[eb][kt % NA]);
            } else {
                // dg_t of the whole group: polled once per workgroup into LDS, then read like in the one-workgroup case
                const uint32_t cnt = (uint32_t)iter * (uint32_t)T + (uint32_t)(T - t);
                FRNN_TRACE_MARK(0);
                __syncthreads();   // every wave has read the previous step's rows
                FRNN_TRACE_MARK(1);
                if (!failed) failed = !poller.poll(xr, (cnt & 1u) * xbuf + xgroup, gbuf, cnt + 1u, p.spin_limit, p.err, FRNN_TRACE_FIRST);
                FRNN_TRACE_SPLIT(7, 2);
                __syncthreads();
                FRNN_TRACE_MARK(3);
                if (KS == 1 || ks == 0) load_step(t > 1 ? t - 1 : 1, t > 2, cvn, scn, spn, dhn);
                i32x4 out_v[NBO];
                if constexpr (kOutRows) {
#pragma unroll
                    for (int j = 0; j < NBO; ++j) out_v[j] = *(const i32x4*)(gbuf + out_l[j]);
                }
#pragma unroll
                for (int kc = 0; kc < KT; kc += KC) {
                    op_t gB[KC];
                    if constexpr (BF16) {
                        lds_operand_chunk<BT, KC, true>(gbuf + lds_row + (size_t)(k0 + kc * 32 + lm.quad * 8) * 2, lm.c, gB);
                    } else {
#pragma unroll
                        for (int j = 0; j < KC; ++j) gB[j] = *(const float*)(gbuf + lds_row + (size_t)(k0 + lm.quad * KT + kc + j) * 4);
                    }
#pragma unroll
                    for (int j = 0; j < KC; ++j) a4[0][(kc + j) % NA] = OP::mfma(Rf[0][kc + j], gB[j], a4[0][(kc + j) % NA]);
                }
                if constexpr (kOutRows) {
                    const rsrc_t dwx_rows = make_rsrc(kRunning ? dwx_run : dwx_g + (size_t)(t - 1) * wx_step);
#pragma unroll
                    for (int j = 0; j < NBO; ++j) __builtin_amdgcn_raw_buffer_store_b128(out_v[j], dwx_rows, out_g[j], 0, 0);
                }
            }
            f32x4 accs[EB][1];
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) {
                if constexpr (NA == 4) accs[eb][0] = (a4[eb][0] + a4[eb][1]) + (a4[eb][2] + a4[eb][3]);
                else accs[eb][0] = a4[eb][0] + a4[eb][1];
            }
            reduce_slices<1, KS, BT>(red, t & 1, ks, wu, p.NWU, lane, accs[0]);
#ifdef FLASHRNN_TRACE
            if constexpr (MULTI) { asm volatile("" : "+v"(accs[0][0]) : : "memory"); FRNN_TRACE_MARK(4); }
#endif
            if (KS == 1 || ks == 0) {
#pragma unroll
                for (int eb = 0; eb < EB; ++eb) {
                    compact_tile<BT>(accs[eb][0]);
#pragma unroll
                    for (int i = 0; i < PP; ++i) ds[eb][0][i] += fminf(fmaxf(accs[eb][0][i], -p.clip), p.clip);   // (Sec. 4.1 clip; +inf = off)
                }
                // wait for the prefetched inputs here, where only this step's stores are younger
#pragma unroll
                for (int eb = 0; eb < EB; ++eb) { pin(cvn[eb]); pin(scn[eb]); pin(spn[eb]); pin(dhn[eb]); }
#pragma unroll
                for (int eb = 0; eb < EB; ++eb)
#pragma unroll
                for (int i = 0; i < PP; ++i) {
#pragma unroll
                    for (int c2 = 0; c2 < NC; ++c2) cv[eb][c2][i] = cvn[eb][c2][i];
#pragma unroll
                    for (int s = 0; s < S; ++s) { sc[eb][s][i] = scn[eb][s][i]; sp[eb][s][i] = spn[eb][s][i]; }
                    dh_ext[eb][i] = dhn[eb][i];
                }
            }
            if constexpr (kRunning) {
                dwx_run -= wx_step;
                dgn_run -= dh_step;
            }
            if constexpr (MULTI) FRNN_TRACE_MARK(5);
        }
        // ---- gradients w.r.t. the initial states, per-row partial sums of db
        if (lane_ok) {
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
                for (int s = 0; s < S; ++s)
                    store_io_r<false, PP>(make_rsrc((char*)p.dstates0 + (size_t)n * D * 4), voff_st + eb * 64, s * st_state, ds[eb][s]);
#pragma unroll
                for (int g2 = 0; g2 < G; ++g2) {
                    const size_t at = (((size_t)bb * NH + n) * G + g2) * D + e0 + 16 * eb;
                    if (p.db_accumulate) {   // a later window of a windowed backward pass: on top of the windows before it
                        float prev[PP];
                        load_f32<PP>(p.db_part, at, prev);
#pragma unroll
                        for (int i = 0; i < PP; ++i) dbacc[eb][g2][i] += prev[i];
                    }
                    store_f32<PP>(p.db_part, at, dbacc[eb][g2]);
                }
            }
        }
    }
    FRNN_TRACE_END(p);
}

}  // namespace flashrnn
