// C ABI of the library (see include/flashrnn.h): argument checks, launch planning, workspace carving
// and the launches.  No device memory is allocated here.
#include "flashrnn.h"

#include <hip/hip_ext.h>

#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <map>
#include <set>

#include "flashrnn_common.h"
#include "flashrnn_host.h"
#include "flashrnn_recompute.h"

using namespace flashrnn;

namespace {

constexpr int kXcds = 8;            // accelerator dies a workgroup index cycles through
constexpr size_t kAlign = 256;

inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline int num_states(int cell) { return cell == FLASHRNN_LSTM ? 2 : cell == FLASHRNN_GRU ? 1 : cell == FLASHRNN_SLSTM ? 4 : cell == FLASHRNN_ELMAN ? 1 : cell == FLASHRNN_GRU4 ? 1 : -1; }
inline int num_gates(int cell) { return cell == FLASHRNN_LSTM ? 4 : cell == FLASHRNN_GRU ? 3 : cell == FLASHRNN_SLSTM ? 4 : cell == FLASHRNN_ELMAN ? 1 : cell == FLASHRNN_GRU4 ? 4 : -1; }
inline int num_cached(int cell) { return cell == FLASHRNN_SLSTM ? 5 : 4; }
inline size_t io_size(int dt) { return dt == FLASHRNN_BF16 ? 2 : 4; }

// The planner's override variables (FLASHRNN_MULTI, _BT, ...) and FLASHRNN_SPIN_LIMIT exist for the tests that force
// every kernel family onto small shapes.  They are looked at only when FLASHRNN_PLAN_OVERRIDES=1 was in the
// environment at the library's first call; otherwise no call touches the environment.
bool overrides_enabled() {
    static const bool on = [] {
        const char* v = getenv("FLASHRNN_PLAN_OVERRIDES");
        return v && *v == '1';
    }();
    return on;
}
int env_int(const char* name, int dflt) {
    if (!overrides_enabled()) return dflt;
    const char* v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

int device_cus() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
        else cus = 256;  // MI355X
    }
    return cus;
}

KernelTable table_for(int cell, int dt) {
    const bool bf = dt == FLASHRNN_BF16;
    switch (cell) {
        case FLASHRNN_LSTM: return bf ? table_lstm_bf16() : table_lstm_f32();
        case FLASHRNN_GRU: return bf ? table_gru_bf16() : table_gru_f32();
        case FLASHRNN_ELMAN: return bf ? table_elman_bf16() : table_elman_f32();
        case FLASHRNN_GRU4: return bf ? table_gru4_bf16() : table_gru4_f32();
        default: return bf ? table_slstm_bf16() : table_slstm_f32();
    }
}

struct Plan {
    const KernelEntry* e = nullptr;
    int NWU = 0, P = 0, NG = 0, GPAR = 0, grid = 0, block = 0, DK = 0, spread = 0;
    size_t smem = 0, exch_bytes = 0, rpack_bytes = 0;
};

int validate(const flashrnn_desc_t* d) {
    if (!d) return FLASHRNN_ERR_NULL;
    if (num_states(d->cell) < 0 || (d->io_dtype != FLASHRNN_F32 && d->io_dtype != FLASHRNN_BF16)) return FLASHRNN_ERR_SHAPE;
    if (d->T < 0 || d->B <= 0 || d->NH <= 0 || d->D <= 0) return FLASHRNN_ERR_SHAPE;
    if (d->recurrent_grad_clip != d->recurrent_grad_clip) return FLASHRNN_ERR_SHAPE;   // NaN
    if (d->D % 16 != 0) return FLASHRNN_ERR_UNSUPPORTED;
    // The kernels address one time step's slab of every tensor with 32-bit byte offsets below 2^31 (offsets from
    // 2^31 on mean "drop this access"): the largest slabs are the states (S f32 values per unit), the inputs (G values)
    // and the saved-values records.
    const unsigned long long units = (unsigned long long)d->B * d->NH * d->D, e = io_size(d->io_dtype);
    const unsigned long long slab_max = 0x7FFFFFFFull;
    if (units * num_states(d->cell) * 4 > slab_max || units * num_gates(d->cell) * e > slab_max || units * record_slots(d->cell) * e > slab_max)
        return FLASHRNN_ERR_UNSUPPORTED;
    return FLASHRNN_OK;
}

constexpr size_t kLdsBytes = 160 * 1024;   // LDS of one CU
constexpr int kTraceGrid = 512;            // workgroups whose per-phase clock sums a trace build keeps
constexpr size_t kTraceBytes = (size_t)kTraceGrid * kTraceWaves * kTracePhases * 8;

// true if the kernel keeps part of its registers in scratch memory (known once a device is there)
bool kernel_spills(const void* fn) {
    static std::mutex mu;
    static std::map<const void*, bool> seen;
    std::lock_guard<std::mutex> lock(mu);
    auto it = seen.find(fn);
    if (it != seen.end()) return it->second;
    hipFuncAttributes attr;
    bool spills = false;
    if (hipFuncGetAttributes(&attr, fn) == hipSuccess) spills = attr.localSizeBytes > 0;
    else (void)hipGetLastError();
    seen[fn] = spills;
    return spills;
}

// Launch plan.  One workgroup per group whenever the head's R fits one CU's registers with 16 units
// per wave (no cross-CU traffic at all); then small batch tiles spread the point-wise work over more
// CUs.  Otherwise a group is split over P workgroups of one XCD that exchange h / dg every step.
// mode 0: forward call that saves its values, 1: backward call, 2: forward call that saves nothing.
int make_plan(const flashrnn_desc_t* d, int mode, Plan* out) {
    const int bwd = mode == 1 ? 1 : 0;
    const int G = num_gates(d->cell);
    const bool bf = d->io_dtype == FLASHRNN_BF16;
    const int kstep = bf ? 32 : 4;
    const int kdim = bwd ? G * d->D : d->D;
    const int units16 = d->D / 16;
    const KernelTable tab = table_for(d->cell, d->io_dtype);
    const int cus = device_cus();
    const int force_multi = env_int("FLASHRNN_MULTI", -1);   // 1: always split groups, 0: never, 2: always spread over all XCDs
    const int force_bt = env_int("FLASHRNN_BT", 0);
    const int force_nwu = env_int("FLASHRNN_NWU", 0);
    const int force_ks = env_int("FLASHRNN_KS", 0);
    const int force_gpar = env_int("FLASHRNN_GPAR", 0);
    const int force_ebk = env_int("FLASHRNN_EBK", 0);        // contraction slices of the backward tile kernel
    const int force_kind = env_int("FLASHRNN_KIND", -1);     // kernel family (KernelEntry::tile)
    const int force_eb = env_int("FLASHRNN_EB", 0);          // blocks of 16 units per wave (one workgroup per group)      // groups in flight when groups are split (testing the group loop)
    Plan pl;
    // What the backward pass reads and writes per (t, row, unit): saved values, states, dH, dWx.  Beyond the last-level cache
    // (256 MB; the forward pass has just written most of it) its inputs come from HBM, and small heads take the kernels that fetch deeper.
    const double bwd_bytes = ((double)record_slots(d->cell) * io_size(d->io_dtype) + (double)num_states(d->cell) * 4 + (double)(1 + G) * io_size(d->io_dtype)) *
                             (double)d->T * d->B * d->NH * d->D;
    // (measured at 12 x 64, T = 1024: up to 165 MB -- LSTM with 8 rows, sLSTM with 5 -- the direct loads are 10 % faster, from
    // 184 MB on -- LSTM with 9 rows -- the deep fetch is)
    const int deep_mode = bwd ? env_int("FLASHRNN_DEEP_FETCH", bwd_bytes > 172.0 * 1024 * 1024 ? 1 : 0) : 0;   // (2: also where the rules below exclude it)
    const bool deep = deep_mode != 0;

    if (force_multi < 1) {
        // Every (batch tile, kernel) pair that can run the shape gets a cost: rounds of workgroups over the CUs
        // times a relative time per step.  The relative times are measured ones (D = 192 and 128, MI355X): the
        // staged tile kernels run a step of 4 rows in 1.0, of 8 rows in 1.45 to 2.7 (below); the generic kernels, whose
        // lanes access global memory themselves, need about 1.8 / 3.0 / 6.0 for 4 / 8 / 16 rows.  A kernel that
        // spills registers or whose images do not fit the LDS is not a candidate.
        const KernelEntry* best = nullptr;
        double best_cost = 0.0;
        size_t best_smem = 0;
        for (int i = 0; i < tab.count; ++i) {
            const KernelEntry& e = tab.entries[i];
            if (e.bwd != bwd || e.multi || e.KS != 1) continue;
            if (force_bt && e.BT != force_bt) continue;
            if (e.KT * kstep < kdim || units16 % e.eb != 0 || e.maxw * (e.tile == 1 ? 1 : e.eb) < units16) continue;
            if (force_eb ? e.eb != force_eb : false) continue;
            if (force_kind >= 0 && e.tile != force_kind) continue;
            if (force_ebk && bwd && e.tile == 1 && e.eb != force_ebk) continue;
            const int dk = e.KT * kstep, nw = e.tile == 1 ? units16 : units16 / e.eb;
            const bool exact_only = e.exact == 1 || e.exact == 2;
            if (exact_only && dk != kdim) continue;
            if (e.exact >= 2 && !deep) continue;
            // (heads of 128 units: the deeper fetch pays only once half of the CUs stream -- GRU 8 x 128 with 64 rows backward
            // -6 %, LSTM 6 x 128 with 128 rows -5 %, with 16 rows +10 %)
            if (e.exact >= 2 && deep_mode != 2 && e.maxw > 4 && d->NH * ((d->B + e.BT - 1) / e.BT) < cus / 2) continue;
            // (three and more workgroups per CU: they hide each other's latency and the call runs at the bandwidth of HBM; the
            // direct loads are then 4 to 9 % faster -- 12 x 64 with 512 rows, 24 x 32 with 256)
            if (e.exact >= 2 && deep_mode != 2 && d->NH * ((d->B + e.BT - 1) / e.BT) > 2 * cus) continue;
            size_t smem = (size_t)2 * e.BT * (dk + (bf ? 8 : 4)) * (bf ? 2 : 4);
            if (e.tile == 1 && bwd) {
                const int nsb = d->cell == FLASHRNN_SLSTM ? 2 : d->cell == FLASHRNN_ELMAN ? 0 : 1, go = d->cell == FLASHRNN_GRU ? G + 1 : G;
                smem = tile_lds_bwd(e.BT, go, nsb, d->D, dk * 2, e.eb, record_slots(d->cell) * 2).total;
            } else if (e.tile == 1) {
                smem = tile_lds(e.BT, G, num_states(d->cell), d->D, 64 * nw, dk * 2).total_fwd;
            }
            if (smem > kLdsBytes) continue;
            if (e.tile == 1 && kernel_spills(e.fn)) continue;
            const int ng = d->NH * ((d->B + e.BT - 1) / e.BT);
            // Rounds of workgroups over the CUs.  Small staged workgroups (4 rows, at most 4 waves) share a CU, two and three at a
            // time, and overlap each other's waits: with more groups than CUs their time grows by 0.62 per CU-load of groups, not by
            // whole rounds (forward 12 x 64: 1.38 of a single round's time at 1.125 groups per CU, 1.55 at 1.5, 2.6 at 3).
            const double per_cu = (double)ng / cus;
            const double rounds = (e.tile == 1 && e.BT == 4 && nw <= 4 && ng > cus) ? 0.7 + 0.62 * per_cu : (double)((ng + cus - 1) / cus);
            // (8-row staged tiles, measured at 12 x 64 with 96 to 256 rows: backward 1.3 of a 4-row step, forward 1.65 --
            // 1.25 when the call saves nothing and writes a third of the bytes: 1.48 in one round, 1.12 per round in two --, the
            // sLSTM's forward step, whose point-wise function is the longest, 2.7)
            const double rel8 = bwd ? 1.3 : (d->cell == FLASHRNN_SLSTM ? 2.7 : (mode == 2 ? 1.25 : 1.65));
            double rel = e.tile == 1 ? (e.BT == 4 ? 1.0 : rel8) : (e.BT == 4 ? 1.8 : e.BT == 8 ? 3.0 : 6.0);
            // the backward tile kernel splits the contraction over its waves only when the operand reads are
            // many (k-steps x waves); otherwise the second barrier costs more than it saves
            if (e.tile == 1 && bwd && ((e.eb > 1) != (e.KT * units16 >= 256))) rel *= 1.05;
            if (e.tile == 0) rel *= 1.0 + 0.05 * (e.eb - 1);       // thin waves overlap better
            rel *= 1.0 + 0.02 * (dk - kdim) / (double)kstep;       // padded k-steps are wasted MFMAs
            if (exact_only) rel *= 0.99;                           // compile-time LDS layout: fewer address instructions
            if (e.exact >= 2) rel *= 0.9;                          // (only a candidate when the inputs come from HBM: -10 % there)
            const double cost = rounds * rel;
            if (!best || cost < best_cost) { best = &e; best_cost = cost; best_smem = smem; }
        }
        if (best) {
            pl.e = best;
            pl.NWU = best->tile == 1 ? units16 : units16 / best->eb;   // the tile kernels run one wave per block of 16 units
            pl.P = 1;
            pl.NG = d->NH * ((d->B + best->BT - 1) / best->BT);
            pl.GPAR = pl.NG;
            pl.grid = pl.NG;
            pl.block = 64 * pl.NWU;
            pl.DK = best->KT * kstep;
            pl.smem = best_smem;
            pl.exch_bytes = 0;
        }
    }
    if (!pl.e && force_multi != 0 && force_multi != 2) {
        // Batch tiles of 16, 8 or 4 rows here too.  A smaller tile means more groups (each with its own workgroups, on its
        // own XCD when there are few) and proportionally less to exchange and less point-wise work per workgroup; the
        // smallest tile whose groups all run at once is taken, else the largest (fewest rounds over the groups).
        const int want_ks = force_ks ? force_ks : (d->D >= 512 ? 4 : 1);
        const int bts[3] = {4, 8, 16};
        for (int pass = 0; pass < 2 && !pl.e; ++pass) {
            for (int bi = 0; bi < 3 && !pl.e; ++bi) {
                const int BT = pass == 0 ? bts[bi] : bts[2 - bi];
                if (force_bt && BT != force_bt) continue;
                // workgroups of one launch per XCD: all members of a group must be resident at once, at most one per CU
                // where a workgroup takes all registers of its CU.  (A head of 1024 units asks for every CU of an XCD, in both
                // directions: with two CUs kept back the backward pass of such a head fell to one group of 16 rows at 13 us a step.)
                int cap = cus / kXcds;
                const int NG = d->NH * ((d->B + BT - 1) / BT);
                const KernelEntry* best = nullptr;
                for (int spills_ok = 0; spills_ok < 2 && !best; ++spills_ok)   // a kernel that keeps registers in scratch memory only as a last resort
                for (int i = 0; i < tab.count; ++i) {
                    const KernelEntry& e = tab.entries[i];
                    const int dk = e.KT * e.KS * kstep;
                    if (e.bwd != bwd || !e.multi || e.BT != BT || dk < kdim) continue;
                    if (e.maxw == 4 && e.KS == 4 && e.KT * (bwd ? 1 : G) >= 40) continue;   // the shapes of the spread placement
                    if (!spills_ok && kernel_spills(e.fn)) continue;
                    // least padding of the contraction axis first, then the wanted number of slices, then the most waves
                    const int bdk = best ? best->KT * best->KS * kstep : 0;
                    const bool want = e.KS == want_ks, bwant = best && best->KS == want_ks;
                    if (!best || dk < bdk || (dk == bdk && (want > bwant || (want == bwant && e.maxw > best->maxw)))) best = &e;
                }
                if (!best) continue;
                const int nwu_max = best->maxw / best->KS;
                // most workgroups per group (shortest MFMA and point-wise phase per step) that still lets
                // every group run at once; fall back to looping over groups
                const int slots = (NG + kXcds - 1) / kXcds;       // groups per XCD if all run at once
                int chosen = 0;
                // (at least four waves per workgroup where the shape allows: the workgroup polls the group's rows
                // together, and with fewer threads that takes more rounds - measured on D = 256 and 768)
                const int nwu_min = 4 / best->KS > 1 ? 4 / best->KS : 1;
                // Forward: the most workgroups per group that fit (shortest MFMA and point-wise phase; its rows are short to poll).
                // Backward: the fewest -- its exchanged rows are G times longer, and a workgroup with more threads strips them
                // in fewer rounds (measured at D = 256: forward 1.27 / 1.36 / 1.74 ms with 8 / 4 / 2 workgroups per group,
                // backward 2.70 / 2.88 / 2.38 ms).
                for (int p2 = 0; p2 < 2 && !chosen; ++p2) {
                    const int lo = p2 == 0 ? nwu_min : 1;
                    for (int step = 0; step <= nwu_max - lo; ++step) {
                        const int nwu = bwd && !force_nwu ? nwu_max - step : lo + step;
                        if (units16 % nwu) continue;
                        const int P = units16 / nwu;
                        if (force_nwu ? nwu == force_nwu : P * slots <= cap) { chosen = nwu; break; }
                    }
                }
                int gpar = NG;
                if (!chosen && pass == 0 && !force_bt) continue;      // not all groups at once with this tile: try a larger one
                if (!chosen) {
                    // even the fewest workgroups per group do not fit all groups: loop over groups
                    for (int nwu = nwu_max; nwu >= 1 && !chosen; --nwu)
                        if (units16 % nwu == 0 && units16 / nwu <= cap) chosen = nwu;
                    if (!chosen && units16 % nwu_max == 0 && units16 / nwu_max <= cus / kXcds) {
                        // the largest heads need every CU of an XCD for one group (no margin: should a CU be taken, the
                        // waits run into their spin limit and the call reports a timeout)
                        chosen = nwu_max;
                        cap = cus / kXcds;
                    }
                    if (chosen) gpar = kXcds * (cap / (units16 / chosen));
                    if (gpar > NG) gpar = NG;
                }
                if (chosen && force_gpar > 0 && force_gpar < gpar) gpar = force_gpar;
                if (chosen) {
                    pl.e = best;
                    pl.NWU = chosen;
                    pl.P = units16 / chosen;
                    pl.NG = NG;
                    pl.GPAR = gpar;
                    pl.grid = (gpar + kXcds - 1) / kXcds * pl.P * kXcds;
                    pl.block = 64 * chosen * best->KS;
                    pl.DK = best->KT * best->KS * kstep;
                    const int nt = bwd ? 1 : G;
                    // one buffer of BT operand rows (polled once per workgroup and step), then the partial sums of the slices
                    pl.smem = (size_t)BT * (pl.DK + (bf ? 8 : 4)) * (bf ? 2 : 4) + (best->KS > 1 ? (size_t)2 * (best->KS - 1) * chosen * nt * 4 * 64 * 4 : 16);
                    pl.exch_bytes = (size_t)2 * gpar * BT * pl.DK * (bf ? 4 : 8);
                }
            }
        }
    }
    if (!pl.e && force_multi != 0 && bf) {
        // Heads beyond what the CUs of one XCD can hold (D > 1024): the group is spread over the CUs of all XCDs, one
        // block of 16 units and 4 contraction slices per workgroup (one wave per SIMD, up to 336 registers of R each),
        // and h / dg cross the XCDs through memory.  The largest batch tile whose kernel neither spills registers nor
        // overflows the LDS; as many groups at once as fit the chip, the rest in turn.  (No CUs are kept back: a head of 2048
        // units takes 128 of them, and two of its groups side by side halve the backward pass.)
        const int budget = cus;
        const int bts[3] = {16, 8, 4};
        for (int spills_ok = 0; spills_ok < 2 && !pl.e; ++spills_ok)   // (a kernel with a few registers in scratch memory only if no tile is free of them)
        for (int bi = 0; bi < 3 && !pl.e; ++bi) {
            const int BT = bts[bi];
            if (force_bt && BT != force_bt) continue;
            const KernelEntry* best = nullptr;
            for (int i = 0; i < tab.count; ++i) {
                const KernelEntry& e = tab.entries[i];
                const int dk = e.KT * e.KS * kstep;
                if (e.bwd != bwd || !e.multi || e.BT != BT || e.KS != 4 || e.maxw != 4 || dk < kdim) continue;
                if (!best || dk < best->KT * best->KS * kstep) best = &e;
            }
            if (!best || units16 > budget) continue;
            const int dk = best->KT * best->KS * kstep, nt = bwd ? 1 : G;
            const size_t smem = (size_t)BT * (dk + 8) * 2 + (size_t)2 * 3 * nt * 4 * 64 * 4;
            if (smem > kLdsBytes || (!spills_ok && kernel_spills(best->fn))) continue;
            const int NG = d->NH * ((d->B + BT - 1) / BT);
            int gpar = budget / units16;
            if (gpar > NG) gpar = NG;
            if (force_gpar > 0 && force_gpar < gpar) gpar = force_gpar;
            pl.e = best;
            pl.NWU = 1;
            pl.P = units16;
            pl.NG = NG;
            pl.GPAR = gpar;
            pl.grid = gpar * pl.P;
            pl.block = 64 * 4;
            pl.DK = dk;
            pl.smem = smem;
            pl.exch_bytes = (size_t)2 * gpar * BT * dk * 4;
            pl.spread = 1;
        }
    }
    if (!pl.e) return FLASHRNN_ERR_UNSUPPORTED;
    pl.rpack_bytes = (bwd ? (size_t)d->NH * d->D * pl.DK : (size_t)d->NH * G * d->D * pl.DK) * io_size(d->io_dtype);
    *out = pl;
    return FLASHRNN_OK;
}

struct Workspace {
    size_t err_off, exch_off, rpack_off, dgn_off, dbpart_off, drpart_off, trace_off, total;
    size_t fwd_total;   // bytes a forward call touches: error words, exchange buffers, the forward copy of R
};

int carve_uncached(const flashrnn_desc_t* d, Workspace* w, Plan* pf, Plan* pb, Plan* pfn) {
    int rc = make_plan(d, 0, pf);
    if (rc != FLASHRNN_OK) return rc;
    rc = make_plan(d, 1, pb);
    if (rc != FLASHRNN_OK) return rc;
    // A forward call that saves nothing may take another batch tile of the staged kernels (they use no workspace beyond the
    // error words, so the layout below does not depend on it); everywhere else it runs the plan of the saving call.
    if (make_plan(d, 2, pfn) != FLASHRNN_OK || pfn->e->tile == 0 || pf->e->tile == 0) *pfn = *pf;
    const int G = num_gates(d->cell);
    size_t off = 0;
    w->err_off = off; off += kAlign;   // word 0: forward kernels, word 1: backward kernels
    w->exch_off = off; off += align_up(pf->exch_bytes > pb->exch_bytes ? pf->exch_bytes : pb->exch_bytes);
    w->rpack_off = off; off += align_up(pf->rpack_bytes > pb->rpack_bytes ? pf->rpack_bytes : pb->rpack_bytes);
    w->fwd_total = w->rpack_off + align_up(pf->rpack_bytes);
    w->dgn_off = off; off += align_up(d->cell == FLASHRNN_GRU ? (size_t)d->T * d->B * d->NH * d->D * io_size(d->io_dtype) : 0);
    const int sk = dr_split_k(d->io_dtype == FLASHRNN_BF16, d->T, d->B, d->NH, d->D, G);
    // partial sums of db: one row per batch row (from the persistent kernel) or per contraction slice (from the dR GEMM)
    w->dbpart_off = off; off += align_up((size_t)(d->B > sk ? d->B : sk) * d->NH * G * d->D * 4);
    w->drpart_off = off;
    off += align_up(sk > 1 ? (size_t)sk * d->NH * d->D * G * d->D * 4 : 0);
    w->trace_off = off;
#ifdef FLASHRNN_TRACE
    off += 2 * kTraceBytes;   // forward, backward
#endif
    w->total = off;
    return FLASHRNN_OK;
}

// Plans and workspace layout of a descriptor.  A thread that calls with the same descriptor again (the usual case:
// forward, backward, forward, ...) gets the last answer back instead of planning anew; the answer depends on the
// descriptor and the device only (and on the override variables, which switch this memo off).
int carve(const flashrnn_desc_t* d, Workspace* w, Plan* pf, Plan* pb, Plan* pfn = nullptr) {
    struct Memo { bool valid = false; flashrnn_desc_t d; int dev; int rc; Workspace w; Plan pf, pb, pfn; };
    static thread_local Memo memo;
    int dev = -1;
    (void)hipGetDevice(&dev);
    flashrnn_desc_t key = *d;
    key.recurrent_grad_clip = 0.0f;   // does not enter the plan
    if (!overrides_enabled() && memo.valid && memo.dev == dev && memcmp(&memo.d, &key, sizeof(key)) == 0) {
        *w = memo.w; *pf = memo.pf; *pb = memo.pb;
        if (pfn) *pfn = memo.pfn;
        return memo.rc;
    }
    Plan nosave;
    const int rc = carve_uncached(d, w, pf, pb, &nosave);
    memo.valid = true; memo.d = key; memo.dev = dev; memo.rc = rc; memo.w = *w; memo.pf = *pf; memo.pb = *pb; memo.pfn = nosave;
    if (pfn) *pfn = nosave;
    return rc;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

int prepare_kernel(const Plan& pl) {
    static std::mutex mu;
    static std::set<const void*> done;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count(pl.e->fn)) return FLASHRNN_OK;
    if (hipFuncSetAttribute(pl.e->fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) {
        (void)hipGetLastError();
        if (pl.smem > 64 * 1024) return FLASHRNN_ERR_LAUNCH;
    }
    done.insert(pl.e->fn);
    return FLASHRNN_OK;
}

// optional bracketing of the persistent kernels with HIP events (flashrnn_profile_*)
constexpr int kProfSlots = 256;
struct Profile {
    int stride = 0;            // 0 = off; n = every n-th call per direction carries events
    int seen[2] = {0, 0};
    int count[2] = {0, 0};
    hipEvent_t ev[2][kProfSlots][2] = {};
};
Profile g_prof;
std::mutex g_prof_mu;

int launch_persistent(const Plan& pl, KernelParams& kp, hipStream_t stream) {
    if (prepare_kernel(pl) != FLASHRNN_OK) return FLASHRNN_ERR_LAUNCH;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_prof_mu);
        const int dir = pl.e->bwd;
        if (g_prof.stride > 0 && g_prof.seen[dir]++ % g_prof.stride == 0 && g_prof.count[dir] < kProfSlots) {
            const int i = g_prof.count[dir]++;
            for (int j = 0; j < 2; ++j)
                if (!g_prof.ev[dir][i][j] && hipEventCreate(&g_prof.ev[dir][i][j]) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
            e0 = g_prof.ev[dir][i][0];
            e1 = g_prof.ev[dir][i][1];
        }
    }
    kp.P = pl.P;
    kp.NWU = pl.NWU;
    kp.NG = pl.NG;
    kp.GPAR = pl.GPAR;
    kp.spread = pl.spread;
    kp.spin_limit = env_int("FLASHRNN_SPIN_LIMIT", 1 << 21);
    void* args[] = {&kp};
    if (e0 && e1) {
        // the two events ride on the kernel's own dispatch (start and end time stamps of that dispatch): no extra commands
        // in the stream, so the measurement does not slow the step down
        if (hipExtLaunchKernel(pl.e->fn, dim3(pl.grid), dim3(pl.block), args, pl.smem, stream, e0, e1, 0) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
    } else if (hipLaunchKernel(pl.e->fn, dim3(pl.grid), dim3(pl.block), args, pl.smem, stream) != hipSuccess) {
        return FLASHRNN_ERR_LAUNCH;
    }
    return FLASHRNN_OK;
}

// Scratch memory of flashrnn_fwd_static_scratch: one array per GPU, part of the loaded code object (no allocation call
// ever).  Host code must not use the array's name as an address: the device address is looked up once per device, with
// that device current, and kept.
constexpr size_t kStaticScratchBytes = (size_t)FLASHRNN_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

void* static_scratch_ptr() {
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return nullptr; }
        ptrs[dev] = ptr;
    }
    return ptrs[dev];
}

// Forward call on the workspace `workspace`; ws_limit > 0: the workspace is the library's own array of that size and
// only the part a forward call touches has to fit.
int fwd_impl(const flashrnn_desc_t* d, const void* Wx, const void* R, const void* b, const void* states0, void* states,
             void* gate_cache, void* workspace, size_t ws_limit, void* hip_stream) {
    int rc = validate(d);
    if (rc != FLASHRNN_OK) return rc;
    if (!R || !b || !states || (d->T > 0 && !Wx)) return FLASHRNN_ERR_NULL;
    if (!aligned16(Wx) || !aligned16(R) || !aligned16(b) || !aligned16(states0) || !aligned16(states) || !aligned16(gate_cache))
        return FLASHRNN_ERR_UNSUPPORTED;
    Workspace w;
    Plan pf, pb, pfn;
    rc = carve(d, &w, &pf, &pb, &pfn);
    if (rc != FLASHRNN_OK) return rc;
    if (!gate_cache) pf = pfn;
    if (!workspace || ((uintptr_t)workspace & (kAlign - 1))) return FLASHRNN_ERR_WORKSPACE;
    if (ws_limit && w.fwd_total > ws_limit) return FLASHRNN_ERR_SCRATCH;
    hipStream_t stream = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const int G = num_gates(d->cell);
    // the exchange words start from zero stamps (a fill kernel, not a memset: the call may be captured into a graph);
    // both error words are cleared by the packing kernel
    if (pf.exch_bytes && launch_fill_zero(ws + w.exch_off, align_up(pf.exch_bytes), stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
    // (the staged forward kernels read R as it is and clear the error words themselves)
    const bool r_in_place = pf.e->tile != 0;
    if (!r_in_place && launch_pack_r(d->io_dtype == FLASHRNN_BF16, false, R, ws + w.rpack_off, d->NH, d->D, G, pf.DK, (int*)(ws + w.err_off), stream) != hipSuccess)
        return FLASHRNN_ERR_LAUNCH;
    KernelParams kp;
    memset(&kp, 0, sizeof(kp));
    kp.Wx = Wx; kp.R = r_in_place ? R : (const void*)(ws + w.rpack_off); kp.bias = b; kp.states0 = (const float*)states0; kp.states = (float*)states;
    kp.cache = gate_cache;
    kp.exch = (uint32_t*)(ws + w.exch_off);
    kp.err = (int*)(ws + w.err_off);
    kp.T = d->T; kp.B = d->B; kp.NH = d->NH; kp.D = d->D;
#ifdef FLASHRNN_TRACE
    if (!ws_limit && pf.grid <= kTraceGrid) {
        kp.trace = (unsigned long long*)(ws + w.trace_off);
        if (launch_fill_zero(kp.trace, kTraceBytes, stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
    }
#endif
    return launch_persistent(pf, kp, stream);
}

// Workspace of flashrnn_bwd_recompute behind the ordinary one: the records of one window of time steps and two buffers
// for the state gradients carried from window to window.  The window holds as many steps as fit 64 MiB (at least one):
// small enough to stay in the last-level cache between the kernel that writes it and the one that reads it.
struct RecomputeLayout { size_t window_off, carry_off, total; int window; };
RecomputeLayout recompute_layout(const flashrnn_desc_t* d, size_t base_total) {
    RecomputeLayout rl;
    const size_t units = (size_t)d->B * d->NH * d->D;
    const size_t rec_step = units * record_slots(d->cell) * io_size(d->io_dtype);
    long long steps = (long long)((64ull << 20) / (rec_step ? rec_step : 1));
    const int forced = env_int("FLASHRNN_RECOMPUTE_STEPS", 0);   // (test hook: windows of this many steps)
    if (forced > 0) steps = forced;
    if (steps < 1) steps = 1;
    if (steps > d->T) steps = d->T > 0 ? d->T : 1;
    rl.window = (int)steps;
    rl.window_off = base_total;
    rl.carry_off = rl.window_off + align_up((size_t)steps * rec_step);
    rl.total = rl.carry_off + 2 * align_up((size_t)num_states(d->cell) * units * 4);
    return rl;
}

// Backward call.  Wx == nullptr: the saved values come from gate_cache (flashrnn_bwd).  Otherwise (flashrnn_bwd_recompute)
// they are formed again, a window of time steps at a time, into the window buffer behind the ordinary workspace, and the
// persistent kernel runs window by window from the last step to the first, the gradients of the carried states going from
// one launch to the next through two buffers in the workspace.
int bwd_impl(const flashrnn_desc_t* d, const void* Wx, const void* R, const void* b, const void* states, const void* gate_cache,
             const void* dH, const void* dstates_last, void* dWx, void* dR, void* db, void* dstates0, void* workspace, void* hip_stream) {
    int rc = validate(d);
    if (rc != FLASHRNN_OK) return rc;
    const bool recompute = Wx != nullptr;
    if (!R || !states || !dR || !db || !dstates0 || (d->T > 0 && ((!recompute && !gate_cache) || !dH || !dWx)) || (recompute && !b)) return FLASHRNN_ERR_NULL;
    if (!aligned16(R) || !aligned16(states) || !aligned16(gate_cache) || !aligned16(dH) || !aligned16(dstates_last) ||
        !aligned16(dWx) || !aligned16(dR) || !aligned16(db) || !aligned16(dstates0) || !aligned16(Wx) || !aligned16(b))
        return FLASHRNN_ERR_UNSUPPORTED;
    Workspace w;
    Plan pf, pb;
    rc = carve(d, &w, &pf, &pb);
    if (rc != FLASHRNN_OK) return rc;
    if (!workspace || ((uintptr_t)workspace & (kAlign - 1))) return FLASHRNN_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const int G = num_gates(d->cell), S = num_states(d->cell);
    const bool bf = d->io_dtype == FLASHRNN_BF16;
    const size_t esz = io_size(d->io_dtype);
    // The backward copy of R is R itself, padded along (gate, unit) to the kernel's contraction length: without padding
    // and without cross-CU waits (whose error word the packing kernel clears) the kernel reads R where it is.
    const bool r_in_place = !pb.e->multi && pb.DK == G * d->D;
    if (!r_in_place && launch_pack_r(bf, true, R, ws + w.rpack_off, d->NH, d->D, G, pb.DK, (int*)(ws + w.err_off) + 1, stream) != hipSuccess)
        return FLASHRNN_ERR_LAUNCH;
    const size_t units = (size_t)d->B * d->NH * d->D;
    const size_t st_step = (size_t)S * units * 4, io_step = units * esz, rec_step = units * record_slots(d->cell) * esz;
    const RecomputeLayout rl = recompute_layout(d, w.total);
    const int window = recompute ? rl.window : (d->T > 0 ? d->T : 1);
    // windows from the last step to the first; [r0, r1) are 0-based step indices (step r turns states[r] into states[r + 1])
    for (int r1 = d->T; r1 > 0 || (r1 == 0 && d->T == 0); r1 -= window) {
        const int r0 = r1 - window > 0 ? r1 - window : 0, steps = r1 - r0;
        const bool first = r1 == d->T, last = r0 == 0;
        const void* cache = gate_cache;
        if (recompute && steps > 0) {
            RecomputeParams rp;
            rp.Wx = (const char*)Wx + (size_t)r0 * G * io_step; rp.R = R; rp.bias = b;
            rp.states = (const float*)((const char*)states + (size_t)r0 * st_step);
            rp.cache = ws + rl.window_off; rp.steps = steps; rp.B = d->B; rp.NH = d->NH; rp.D = d->D;
            void* args[] = {&rp};
            const dim3 grid((unsigned)((steps * d->B + kRecomputeCols - 1) / kRecomputeCols), (unsigned)((d->D + 63) / 64), (unsigned)d->NH);
            if (hipLaunchKernel(table_for(d->cell, d->io_dtype).recompute, grid, dim3(256), args, 0, stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
            cache = ws + rl.window_off;
        } else if (!recompute) {
            cache = gate_cache;
        }
        if (pb.exch_bytes && launch_fill_zero(ws + w.exch_off, align_up(pb.exch_bytes), stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
        KernelParams kp;
        memset(&kp, 0, sizeof(kp));
        kp.R = r_in_place ? R : (const void*)(ws + w.rpack_off);
        kp.states = (float*)((char*)const_cast<void*>(states) + (size_t)r0 * st_step);
        kp.cache = const_cast<void*>(cache);
        kp.dH = (const char*)dH + (size_t)r0 * io_step;
        kp.dWx = (char*)dWx + (size_t)r0 * G * io_step;
        kp.dgn = ws + w.dgn_off + (size_t)r0 * io_step;
        // carried state gradients: in from the caller (first launch) or from the window after this one, out to the caller
        // (last launch) or to the window before this one; the two carry buffers alternate
        const int flip = ((d->T - r1) / window) & 1;
        kp.dlast = first ? (const float*)dstates_last : (const float*)(ws + rl.carry_off + (size_t)(flip ^ 1) * align_up((size_t)S * units * 4));
        kp.dstates0 = last ? (float*)dstates0 : (float*)(ws + rl.carry_off + (size_t)flip * align_up((size_t)S * units * 4));
        kp.db_accumulate = first ? 0 : 1;
        kp.clip = d->recurrent_grad_clip > 0.0f ? d->recurrent_grad_clip : d->recurrent_grad_clip < 0.0f ? 0.0f : __builtin_inff();
        kp.db_part = (float*)(ws + w.dbpart_off);
        kp.exch = (uint32_t*)(ws + w.exch_off);
        kp.err = (int*)(ws + w.err_off) + 1;   // the forward call's word stays as it is: flashrnn_check reports both
        kp.T = steps; kp.B = d->B; kp.NH = d->NH; kp.D = d->D;
#ifdef FLASHRNN_TRACE
        if (pb.grid <= kTraceGrid && first) {
            kp.trace = (unsigned long long*)(ws + w.trace_off + kTraceBytes);
            if (launch_fill_zero(kp.trace, kTraceBytes, stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
        }
#endif
        rc = launch_persistent(pb, kp, stream);
        if (rc != FLASHRNN_OK) return rc;
        if (d->T == 0) break;
    }
    (void)rec_step;
    // db: sum of the per-row partial sums in row order; dR: GEMM over (t, b)
    // (the staged kernels leave db to the GEMM, which reads every gate gradient anyway)
    const size_t nb = (size_t)d->NH * G * d->D;
    const bool db_from_gemm = pb.e->tile != 0;
    if (d->T == 0) {
        if (db_from_gemm) {
            if (launch_fill_zero(db, nb * 4, stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
        } else if (launch_sum_slices((const float*)(ws + w.dbpart_off), (float*)db, nb, d->B, nb, stream) != hipSuccess) {
            return FLASHRNN_ERR_LAUNCH;
        }
        if (launch_fill_zero(dR, (size_t)d->NH * d->D * G * d->D * 4, stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
        return FLASHRNN_OK;
    }
    if (launch_dr_gemm(bf, (const float*)states, dWx, ws + w.dgn_off, (float*)(ws + w.drpart_off), (float*)dR, d->T, d->B, d->NH, d->D,
                       G, S, d->cell == FLASHRNN_GRU, (float*)(ws + w.dbpart_off), db_from_gemm, (float*)db, stream) != hipSuccess)
        return FLASHRNN_ERR_LAUNCH;
    return FLASHRNN_OK;
}

}  // namespace

extern "C" {

int flashrnn_num_states(int cell) { return num_states(cell); }
int flashrnn_num_gates(int cell) { return num_gates(cell); }

size_t flashrnn_gate_cache_bytes(const flashrnn_desc_t* d) {
    if (validate(d) != FLASHRNN_OK) return 0;
    return (size_t)d->T * d->B * d->NH * d->D * record_slots(d->cell) * io_size(d->io_dtype);
}

size_t flashrnn_workspace_bytes(const flashrnn_desc_t* d) {
    if (validate(d) != FLASHRNN_OK) return 0;
    Workspace w;
    Plan pf, pb;
    if (carve(d, &w, &pf, &pb) != FLASHRNN_OK) return 0;
    return w.total;
}

namespace {
// The plan a call runs: which = 0 forward call that saves its values, 1 backward call, 2 forward call that saves nothing.
int plan_of_call(const flashrnn_desc_t* d, int which, Plan* pl) {
    if (which < 0 || which > 2) return FLASHRNN_ERR_SHAPE;
    Workspace w;
    Plan pf, pb, pfn;
    const int rc = carve(d, &w, &pf, &pb, &pfn);
    if (rc != FLASHRNN_OK) return rc;
    *pl = which == 0 ? pf : (which == 1 ? pb : pfn);
    return FLASHRNN_OK;
}
}  // namespace

int flashrnn_plan(const flashrnn_desc_t* d, int backward, int* workgroups, int* cus_per_head, int* waves_per_wg) {
    int rc = validate(d);
    if (rc != FLASHRNN_OK) return rc;
    Plan pl;
    rc = plan_of_call(d, backward, &pl);
    if (rc != FLASHRNN_OK) return rc;
    if (workgroups) *workgroups = (pl.GPAR < pl.NG ? pl.GPAR : pl.NG) * pl.P;
    if (cus_per_head) *cus_per_head = pl.P * ((d->B + pl.e->BT - 1) / pl.e->BT);
    if (waves_per_wg) *waves_per_wg = pl.block / 64;
    return FLASHRNN_OK;
}

int flashrnn_plan_kernel(const flashrnn_desc_t* d, int backward, int* staged, int* batch_tile, int* split) {
    int rc = validate(d);
    if (rc != FLASHRNN_OK) return rc;
    Plan pl;
    rc = plan_of_call(d, backward, &pl);
    if (rc != FLASHRNN_OK) return rc;
    if (staged) *staged = pl.e->tile != 0 ? (pl.e->exact >= 2 ? 2 : 1) : 0;
    if (batch_tile) *batch_tile = pl.e->BT;
    if (split) *split = pl.P;
    return FLASHRNN_OK;
}

int flashrnn_fwd(const flashrnn_desc_t* d, const void* Wx, const void* R, const void* b, const void* states0, void* states,
                 void* gate_cache, void* workspace, void* hip_stream) {
    return fwd_impl(d, Wx, R, b, states0, states, gate_cache, workspace, 0, hip_stream);
}

int flashrnn_fwd_static_scratch(const flashrnn_desc_t* d, const void* Wx, const void* R, const void* b, const void* states0,
                                void* states, void* gate_cache, void* hip_stream) {
    const int rc = validate(d);   // argument errors are reported without touching a device
    if (rc != FLASHRNN_OK) return rc;
    void* ws = static_scratch_ptr();
    if (!ws) return FLASHRNN_ERR_LAUNCH;
    return fwd_impl(d, Wx, R, b, states0, states, gate_cache, ws, kStaticScratchBytes, hip_stream);
}

int flashrnn_bwd(const flashrnn_desc_t* d, const void* R, const void* b, const void* states, const void* gate_cache,
                 const void* dH, const void* dstates_last, void* dWx, void* dR, void* db, void* dstates0, void* workspace,
                 void* hip_stream) {
    return bwd_impl(d, nullptr, R, b, states, gate_cache, dH, dstates_last, dWx, dR, db, dstates0, workspace, hip_stream);
}

int flashrnn_bwd_recompute(const flashrnn_desc_t* d, const void* Wx, const void* R, const void* b, const void* states, const void* dH,
                           const void* dstates_last, void* dWx, void* dR, void* db, void* dstates0, void* workspace, void* hip_stream) {
    if (d && validate(d) == FLASHRNN_OK && d->T > 0 && !Wx) return FLASHRNN_ERR_NULL;
    alignas(16) static const char kNoInputs[16] = {0};   // T = 0: nothing to recompute; any non-null, aligned pointer selects the windowed path
    return bwd_impl(d, Wx ? Wx : (d && d->T == 0 ? (const void*)kNoInputs : nullptr), R, b, states, nullptr, dH, dstates_last, dWx, dR, db, dstates0,
                    workspace, hip_stream);
}

size_t flashrnn_recompute_workspace_bytes(const flashrnn_desc_t* d) {
    if (validate(d) != FLASHRNN_OK) return 0;
    Workspace w;
    Plan pf, pb;
    if (carve(d, &w, &pf, &pb) != FLASHRNN_OK) return 0;
    return recompute_layout(d, w.total).total;
}

int flashrnn_check(const flashrnn_desc_t* d, const void* workspace, void* hip_stream) {
    if (!workspace) return FLASHRNN_OK;
    if (workspace == FLASHRNN_STATIC_SCRATCH) {
        workspace = static_scratch_ptr();
        if (!workspace) return FLASHRNN_ERR_LAUNCH;
    }
    int flags[2] = {0, 0};
    hipStream_t stream = (hipStream_t)hip_stream;
    bool fwd_waits = true, bwd_waits = true;
    {   // plans without cross-CU waits cannot time out and do not maintain their error word
        Workspace w;
        Plan pf, pb;
        if (d && validate(d) == FLASHRNN_OK && carve(d, &w, &pf, &pb) == FLASHRNN_OK) { fwd_waits = pf.e->multi; bwd_waits = pb.e->multi; }
        if (!fwd_waits && !bwd_waits) return hipStreamSynchronize(stream) == hipSuccess ? FLASHRNN_OK : FLASHRNN_ERR_LAUNCH;
    }
    if (hipMemcpyAsync(flags, workspace, sizeof(flags), hipMemcpyDeviceToHost, stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
    if (hipStreamSynchronize(stream) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
    return ((fwd_waits && flags[0] != 0) || (bwd_waits && flags[1] != 0)) ? FLASHRNN_ERR_TIMEOUT : FLASHRNN_OK;
}

int flashrnn_trace_phases(const flashrnn_desc_t* d, const void* workspace, int backward, double* clocks, int* waves, void* hip_stream) {
#ifdef FLASHRNN_TRACE
    int rc = validate(d);
    if (rc != FLASHRNN_OK) return rc;
    if (!workspace || !clocks) return FLASHRNN_ERR_NULL;
    Workspace w;
    Plan pf, pb;
    rc = carve(d, &w, &pf, &pb);
    if (rc != FLASHRNN_OK) return rc;
    static unsigned long long host[kTraceGrid * kTraceWaves * kTracePhases];
    hipStream_t stream = (hipStream_t)hip_stream;
    if (hipMemcpyAsync(host, (const char*)workspace + w.trace_off + (backward ? kTraceBytes : 0), kTraceBytes, hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return FLASHRNN_ERR_LAUNCH;
    // mean over the waves that recorded anything
    double sum[kTracePhases] = {0};
    int n = 0;
    for (int i = 0; i < kTraceGrid * kTraceWaves; ++i) {
        unsigned long long tot = 0;
        for (int j = 0; j < kTracePhases; ++j) tot += host[(size_t)i * kTracePhases + j];
        if (tot == 0) continue;
        for (int j = 0; j < kTracePhases; ++j) sum[j] += (double)host[(size_t)i * kTracePhases + j];
        ++n;
    }
    for (int j = 0; j < kTracePhases; ++j) clocks[j] = n ? sum[j] / n : 0.0;
    if (waves) *waves = n;
    return FLASHRNN_OK;
#else
    (void)d; (void)workspace; (void)backward; (void)clocks; (void)waves; (void)hip_stream;
    return FLASHRNN_ERR_UNSUPPORTED;
#endif
}

int flashrnn_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    g_prof.stride = on > 0 ? on : 0;
    g_prof.seen[0] = g_prof.seen[1] = 0;
    g_prof.count[0] = g_prof.count[1] = 0;
    return FLASHRNN_OK;
}

int flashrnn_profile_kernel_ms(int backward, float* mean_ms, int* launches) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    const int dir = backward ? 1 : 0;
    double sum = 0.0;
    for (int i = 0; i < g_prof.count[dir]; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.ev[dir][i][1]) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
        if (hipEventElapsedTime(&ms, g_prof.ev[dir][i][0], g_prof.ev[dir][i][1]) != hipSuccess) return FLASHRNN_ERR_LAUNCH;
        sum += ms;
    }
    if (mean_ms) *mean_ms = g_prof.count[dir] ? (float)(sum / g_prof.count[dir]) : 0.f;
    if (launches) *launches = g_prof.count[dir];
    return FLASHRNN_OK;
}

const char* flashrnn_status_string(int status) {
    switch (status) {
        case FLASHRNN_OK: return "ok";
        case FLASHRNN_ERR_NULL: return "a required pointer is NULL";
        case FLASHRNN_ERR_SHAPE: return "invalid shape, cell or dtype";
        case FLASHRNN_ERR_UNSUPPORTED: return "unsupported head size, alignment or dtype combination";
        case FLASHRNN_ERR_WORKSPACE: return "workspace missing or not 256-byte aligned";
        case FLASHRNN_ERR_LAUNCH: return "a HIP call failed";
        case FLASHRNN_ERR_TIMEOUT: return "a cross-CU wait ran into its spin limit";
        case FLASHRNN_ERR_SCRATCH: return "the problem needs more scratch memory than the library's static array holds";
        default: return "unknown status";
    }
}

}  // extern "C"
