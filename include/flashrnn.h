/*
 * flashrnn.h -- C ABI of the MI355X (gfx950) FlashRNN time-step loop.
 *
 * One library, two compute entry points: flashrnn_fwd runs the strictly sequential, head-wise
 * block-diagonal recurrence for all T steps in one persistent kernel, flashrnn_bwd runs
 * back-propagation through time and the weight-gradient reduction.
 *
 * Conventions for every function below
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never allocates or
 *     frees device memory and keeps no state between calls that a result depends on (it remembers the
 *     launch plan of the last descriptor per thread, and which kernels it has prepared).
 *   - Calls are asynchronous on the HIP stream passed as `hip_stream` (a hipStream_t cast to void*,
 *     NULL = the default stream).  Buffers must stay valid until the stream has drained.
 *   - All tensors are dense, row major, in the layouts written next to each argument.
 *   - Return value: FLASHRNN_OK (0) or a negative flashrnn_status_t.  Nothing is thrown.
 *   - Calls that share a workspace must not overlap in time.
 *   - flashrnn_fwd and flashrnn_bwd record only kernel launches on the stream (no allocation, no memset, no
 *     synchronization): after one ordinary call with the same descriptor (kernel attributes are set on first use)
 *     they may be captured into a HIP graph and replayed.
 *
 * Index names:  T time steps, B batch, NH heads, D units per head, G gates, S states.
 *   Gate order on the G axis:  LSTM, sLSTM: i, f, z, o     GRU: r, z, n     Elman: one gate     GRU4: z, r, n, g
 *   State order on the S axis: LSTM: h, c     GRU, GRU4: h     sLSTM: h, c, n, m     Elman: h   (paper App. A)
 *   GRU is the three-gate cell (candidate bias inside the r-product); GRU4 is the cell exactly as App. A prints it:
 *   h_t = sig(z) h_{t-1} + (1 - sig(z)) tanh(n + sig(r) tanh(g)), all four gates full pre-activations.
 */
#ifndef FLASHRNN_H
#define FLASHRNN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FLASHRNN_LSTM = 0, FLASHRNN_GRU = 1, FLASHRNN_SLSTM = 2, FLASHRNN_ELMAN = 3, FLASHRNN_GRU4 = 4 } flashrnn_cell_t;
typedef enum { FLASHRNN_F32 = 0, FLASHRNN_BF16 = 1 } flashrnn_dtype_t;

typedef enum {
    FLASHRNN_OK = 0,
    FLASHRNN_ERR_NULL = -1,        /* a required pointer is NULL                                   */
    FLASHRNN_ERR_SHAPE = -2,       /* T < 0, or B, NH, D <= 0, or unknown cell / dtype             */
    FLASHRNN_ERR_UNSUPPORTED = -3, /* D not a multiple of 16 or above 2688 (bf16) / 256 (f32), a time step of more than
                                      2 GiB in one tensor, or a misaligned pointer */
    FLASHRNN_ERR_WORKSPACE = -4,   /* workspace missing or misaligned (needs 256-byte alignment)   */
    FLASHRNN_ERR_LAUNCH = -5,      /* a HIP call failed                                            */
    FLASHRNN_ERR_TIMEOUT = -6,     /* a cross-CU wait gave up (reported by flashrnn_check)         */
    FLASHRNN_ERR_SCRATCH = -7      /* flashrnn_fwd_static_scratch: the problem needs more than FLASHRNN_STATIC_SCRATCH_BYTES */
} flashrnn_status_t;

/*
 * Problem description.  io_dtype is the type of Wx, R, b, dH and dWx (bf16 or f32).  States, dR, db
 * and dstates0 are always f32.  With bf16 I/O the recurrent product runs on the bf16 matrix cores
 * with f32 accumulation and h (forward) / the gate gradients (backward) are rounded to bf16 as
 * its operand; with f32 I/O it runs on the f32 matrix cores.
 */
typedef struct {
    int cell;     /* flashrnn_cell_t  */
    int T, B, NH, D;
    int io_dtype; /* flashrnn_dtype_t */
    /* Backward pass only (paper Sec. 4.1): clipping of the term of dh_{t-1} that contains the recurrent matrix,
     * R^T dg_t, value by value after each time step.  0 = off, c > 0 clips to [-c, c], any negative value cuts
     * the term to zero (no gradient flows through R between steps; dR and db still see every step). */
    float recurrent_grad_clip;
} flashrnn_desc_t;

/* Number of states / gates of a cell (paper App. A): LSTM 2 / 4, GRU 1 / 3, sLSTM 4 / 4, Elman 1 / 1, GRU4 1 / 4; -1 if unknown. */
int flashrnn_num_states(int cell);
int flashrnn_num_gates(int cell);

/*
 * Size in bytes of the opaque buffer the forward pass fills for the backward pass (the "gates
 * written out for the backward pass" of Alg. 1), and of the scratch workspace both passes need
 * (cross-CU exchange buffers and flags, GRU recurrent-side gate gradients, split-K partial sums).
 * Both return 0 for an invalid descriptor.  The workspace content need not be preserved between
 * calls; it must be 256-byte aligned.
 */
size_t flashrnn_gate_cache_bytes(const flashrnn_desc_t* desc);
size_t flashrnn_workspace_bytes(const flashrnn_desc_t* desc);

/*
 * Forward pass (paper Sec. 3 eq. (1)-(2), Alg. 1):
 *     g_t = Wx_t + R s0_{t-1} + b ;   s_t = P(s_{t-1}, g_t)      for t = 1..T, every head and batch row.
 *   Wx       [T,B,G,NH,D] io_dtype  input pre-activations (the input projection W x is the caller's)
 *   R        [NH,D,G,D]   io_dtype  recurrent weights; first D = previous-state index (contracted),
 *                                   last D = unit the gate belongs to
 *   b        [NH,G,D]     io_dtype  bias
 *   states0  [S,B,NH,D]   f32       initial states, or NULL for zeros
 *   states   [T+1,S,B,NH,D] f32     OUT: slot 0 = initial states, slot t = states after step t
 *   gate_cache  flashrnn_gate_cache_bytes() bytes, OUT, or NULL for a forward-only call
 *   workspace   flashrnn_workspace_bytes() bytes (may be NULL when that size is 0)
 */
int flashrnn_fwd(const flashrnn_desc_t* desc, const void* Wx, const void* R, const void* b, const void* states0,
                 void* states, void* gate_cache, void* workspace, void* hip_stream);

/*
 * flashrnn_fwd for callers that can neither allocate device memory nor hand a workspace over (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without `workspace`, same kernels,
 * same results bit for bit.  The scratch memory (error words, cross-CU exchange buffers, the packed copy of R) is a
 * static array of FLASHRNN_STATIC_SCRATCH_BYTES inside the library's code object; every GPU the library runs on holds
 * its own copy until the process ends.  The call allocates nothing and frees nothing.
 *   - A problem whose forward scratch does not fit returns FLASHRNN_ERR_SCRATCH (nothing is launched); every one of
 *     the five benchmark shapes fits (the largest, one head of 768 units, needs 4.6 MiB + exchange buffers).
 *   - All calls on one GPU share that GPU's array, on whatever stream: calls that overlap in time race.  The array
 *     keeps the last call's content; what a call needs cleared (exchange stamps, error words) it clears itself.
 *   - Timeouts of split plans: flashrnn_check(desc, FLASHRNN_STATIC_SCRATCH, stream).
 */
#define FLASHRNN_STATIC_SCRATCH_BYTES (16u << 20)
int flashrnn_fwd_static_scratch(const flashrnn_desc_t* desc, const void* Wx, const void* R, const void* b,
                                const void* states0, void* states, void* gate_cache, void* hip_stream);

/*
 * Backward pass, BPTT (paper Sec. 4 eq. (3)-(7)), with L depending on h_1..h_T through dH and on the
 * final states through dstates_last:
 *     dg_t = dP/dg ds_t ;  ds_{t-1} = dP/ds ds_t (+ R^T dg_t on the hidden state) ;
 *     dWx_t = dg_t ;  db = sum_t dg_t ;  dR = sum_t s0_{t-1} (x) dg_t
 *   R, b        as in the forward call
 *   states      [T+1,S,B,NH,D] f32  the forward call's output
 *   gate_cache  the forward call's output
 *   dH          [T,B,NH,D] io_dtype gradient w.r.t. h_1..h_T (slot t-1 belongs to h_t)
 *   dstates_last [S,B,NH,D] f32     gradient w.r.t. the final states, or NULL for zeros
 *                                   (the sLSTM stabilizer slot is ignored: m carries no gradient)
 *   dWx         [T,B,G,NH,D] io_dtype OUT
 *   dR          [NH,D,G,D] f32      OUT
 *   db          [NH,G,D]   f32      OUT
 *   dstates0    [S,B,NH,D] f32      OUT (sLSTM stabilizer slot = 0)
 * For the GRU, gate n's input-side gradient (dWx) and recurrent-side gradient (used for dR, db and
 * dh_{t-1}) differ by the factor sig(r); the library keeps the latter in the workspace.
 */
int flashrnn_bwd(const flashrnn_desc_t* desc, const void* R, const void* b, const void* states,
                 const void* gate_cache, const void* dH, const void* dstates_last, void* dWx, void* dR, void* db,
                 void* dstates0, void* workspace, void* hip_stream);

/*
 * flashrnn_bwd without the buffer of saved values (Alg. 1 "write out gates for backward pass"; App. F: the memory of
 * back-propagation through time): call flashrnn_fwd with gate_cache = NULL, keep only `states`, and pass the inputs Wx again
 * here.  The values the backward pass needs are formed again from Wx, R, b and the states, a window of time steps at a
 * time -- inside a window all h_{t-1} are known, so its pre-activations are one dense contraction per head -- and the
 * persistent backward kernel runs window by window from the last step to the first.  Same outputs as flashrnn_bwd
 * within rounding (the saved values are rounded to the I/O dtype either way).
 *   Wx          [T,B,G,NH,D] io_dtype  the forward call's inputs
 *   workspace   flashrnn_recompute_workspace_bytes() bytes: the ordinary workspace, the records of one window (as many
 *               steps as fit 64 MiB) and two buffers for the state gradients carried between windows
 *   all other arguments as in flashrnn_bwd
 */
size_t flashrnn_recompute_workspace_bytes(const flashrnn_desc_t* desc);
int flashrnn_bwd_recompute(const flashrnn_desc_t* desc, const void* Wx, const void* R, const void* b, const void* states,
                           const void* dH, const void* dstates_last, void* dWx, void* dR, void* db, void* dstates0,
                           void* workspace, void* hip_stream);

/*
 * Reads the error words the kernels of the last forward and the last backward call on this workspace left behind
 * (synchronizes the stream).  A plan that splits a head over several CUs waits for its partners with a bounded poll
 * (2^21 polls); if a wait gives up, every kernel still runs to its end, flashrnn_fwd / flashrnn_bwd have long returned
 * FLASHRNN_OK, and the results are invalid: on such plans (flashrnn_plan_kernel: *split > 1) call this after every
 * forward / backward pair at the latest.  The forward call's word survives the backward call that follows it (a new
 * forward call clears both), so one check after the backward call sees a timeout of either.  flashrnn_bwd on a workspace
 * that no flashrnn_fwd call has used yet: zero its first 256 bytes first.
 * Returns FLASHRNN_OK, FLASHRNN_ERR_TIMEOUT, or FLASHRNN_ERR_LAUNCH.  workspace may be NULL (returns OK) or
 * FLASHRNN_STATIC_SCRATCH (the array flashrnn_fwd_static_scratch works in, on the current device).  A shape whose plans
 * never wait across CUs (one workgroup per group) cannot time out: the call then only synchronizes the stream.
 * Test hooks: with FLASHRNN_PLAN_OVERRIDES=1 in the environment when the library is first called, the variables
 * FLASHRNN_SPIN_LIMIT (a negative value makes every wait give up at once, which exercises this error path without
 * hanging anything), FLASHRNN_MULTI, _BT, _NWU, _KS, _GPAR, _EB, _EBK, _KIND (single choices of the launch planner,
 * to force every kernel family onto small shapes) and FLASHRNN_RECOMPUTE_STEPS (window length of flashrnn_bwd_recompute)
 * are read on every call; without it the environment is never read.
 */
#define FLASHRNN_STATIC_SCRATCH ((const void*)(size_t)1)
int flashrnn_check(const flashrnn_desc_t* desc, const void* workspace, void* hip_stream);

/*
 * Launch plan the library would use for `desc`, for reporting: number of workgroups (= CUs kept
 * busy) of the forward / backward persistent kernel, workgroups that share one head, waves per
 * workgroup.  backward = 0: the forward call that saves its values (gate_cache given), 1: the backward call, 2: the
 * forward call that saves nothing (it may take another batch tile; other values: FLASHRNN_ERR_SHAPE).  Any out pointer
 * may be NULL.  Returns a status.
 */
int flashrnn_plan(const flashrnn_desc_t* desc, int backward, int* workgroups, int* cus_per_head, int* waves_per_wg);

/*
 * Which kernel family that plan uses, for reports and regression tests: *staged = 1 for the kernels that move
 * global traffic as 16-byte chunks through LDS images (small batch tiles, bf16), 2 for the variant of those that requests
 * its inputs six steps ahead (backward pass of heads of up to 128 units whose inputs exceed the last-level cache; test
 * hook FLASHRNN_DEEP_FETCH = 1 / 0 allows it whatever the size of the inputs / forbids it, 2 takes it also where the planner's
 * rules on the number of workgroups exclude it), 0 for the kernels whose lanes access global memory themselves; *batch_tile = rows of a batch tile (16, 8 or 4); *split = workgroups per group
 * (> 1: the head is split over CUs that exchange h / dg every step).  Any out pointer may be NULL.
 */
int flashrnn_plan_kernel(const flashrnn_desc_t* desc, int backward, int* staged, int* batch_tile, int* split);

/*
 * Measurement aid (the only state the library keeps; meant for benchmarks, not thread-hot paths).
 * flashrnn_profile_enable(n), n > 0: every n-th flashrnn_fwd / flashrnn_bwd call (the first one included) attaches a
 * start and a stop HIP event to the dispatch of its persistent time-loop kernel on the call's stream (up to 256 calls
 * per direction; later calls are not recorded); n <= 0 switches it off.  A dispatch that carries events starts a few
 * microseconds later than one that does not (measured: 5 us per dispatch), hence the stride.  The call also resets
 * the record.
 * flashrnn_profile_kernel_ms waits for the recorded events and returns the mean duration in
 * milliseconds of the forward (backward = 0) or backward (backward = 1) persistent kernel and the
 * number of launches recorded.
 */
int flashrnn_profile_enable(int on);
int flashrnn_profile_kernel_ms(int backward, float* mean_ms, int* launches);

/*
 * Measurement aid of a library built with -DFLASHRNN_TRACE (python -m paper_2412_07752_amd.build --trace builds it as
 * libflashrnn_trace.so); the ordinary library returns FLASHRNN_ERR_UNSUPPORTED.  In a trace build the persistent kernels
 * of plans that split a head over several workgroups stamp the shader clock between the phases of every time step
 * (Alg. 1: wait for the other workgroups' part of the state, matrix product, point-wise function, stores).  After a
 * forward (backward = 0) or backward (backward = 1) call on `workspace` this returns, per phase, the clocks a wave spent
 * in it over the whole call, averaged over the *waves recorded.  clocks holds 8 values; the phases are listed where the
 * kernels define them (csrc/flashrnn_kernels.h).  Synchronizes the stream.
 */
int flashrnn_trace_phases(const flashrnn_desc_t* desc, const void* workspace, int backward, double* clocks, int* waves,
                          void* hip_stream);

const char* flashrnn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FLASHRNN_H */
