/*
 * ckpt_dp.h - C ABI of the batched activation-checkpoint dynamic program for AMD
 * MI355X (gfx950).
 *
 * The library fills, for B independent chains of L stages, the table
 *     C_BP(s, t, m),  1 <= s <= t <= L,  m = 0..M
 * of the paper's Theorem (Section "Activation Checkpoint Solver / Modeling"): the
 * optimal time of a persistent schedule that back-propagates through stages s..t
 * with m memory slots, together with the candidate that attains it, and turns one
 * chain's recorded candidates into the operation sequence of Table 1.  The planner
 * of Section "Integrate Two Solvers" re-solves the chain for every candidate
 * intra-op plan, hence the batch.
 *
 * Conventions
 *   - Stages are numbered 1..L, activations and gradients 0..L, as in the paper.
 *   - All values are int32.  Times are arbitrary ticks, sizes are memory slots.
 *     u_f / u_b already include the communication times of Table 2, o_f / o_b the
 *     communication overheads.
 *   - Infinity is CKPT_INF = 2^30.  A cell holds min(CKPT_INF, exact value); an
 *     infeasible operand makes a candidate infeasible; a negative memory argument
 *     is infeasible.
 *   - Candidates of cell (s, t): k = s is C_all (keep abar^s; the only candidate
 *     when s == t), k = s' in s+1..t is C_ck(s, s', t, m) (checkpoint a^{s-1}, run
 *     forward to a^{s'-1}).  The recorded candidate is the smallest k that attains
 *     the minimum, 0 when the cell is infeasible.
 *   - m counts everything resident while s..t is processed except the segment's
 *     input a^{s-1}; delta^t is counted.  The whole chain under a device budget of
 *     M_total slots is cell (1, L, M_total - omega_a^0).
 *
 * Table layout (device memory, owned by the caller)
 *   cost : int32  [B][ckpt_table_rows(L)][ckpt_row_pitch(M)]
 *   arg  : uint8  [B][ckpt_table_rows(L)][ckpt_row_pitch(M)]
 *   Row ckpt_row_index(L, s, t) of a chain holds cell (s, t) for m = 0..M in
 *   columns 0..M; columns M+1..pitch-1 are padding with unspecified contents.
 *   Rows are ordered by s, then t:  index = (s-1)*L - (s-1)*(s-2)/2 + (t-s).
 *
 * Ownership and threading: every buffer belongs to the caller and must stay valid
 * until the work enqueued on the stream has finished.  The library's only state is the
 * last HIP error code and, per device, three helper streams with five events (see
 * ckpt_init) on which ckpt_solve_batched runs up to three quarters of a large batch,
 * forked from and joined back into the caller's stream.  A solve with
 * ckpt_solve_opts_t.groups = 1 touches none of it.  Calls from several threads and on
 * different streams with disjoint buffers are safe; the enqueueing of split solves is
 * serialised per device.
 *
 * Errors: every function that can fail returns CKPT_OK (0) or a negative code and
 * never throws or aborts.  Argument errors are reported before anything is
 * enqueued.
 */
#ifndef CKPT_DP_H
#define CKPT_DP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CKPT_INF (1 << 30)
#define CKPT_MAX_L 254 /* the recorded candidate is one byte; 0 means infeasible */

enum {
    CKPT_OK = 0,
    CKPT_E_ARG = -1,        /* null pointer, L < 1, M < 0, B < 1, s/t/m out of range */
    CKPT_E_LIMIT = -2,      /* L > CKPT_MAX_L, rows*pitch >= 2^30 elements per chain, B > 65535 */
    CKPT_E_INFEASIBLE = -3, /* ckpt_schedule: the requested cell is infeasible */
    CKPT_E_SMALLBUF = -4,   /* ckpt_schedule: ops_cap too small (2L-1 .. L(L+1)/2+L operations) */
    CKPT_E_HIP = -5,        /* a HIP call failed; see ckpt_last_hip_error() */
    CKPT_E_INPUT = -6,      /* ckpt_check_inputs: some chain violates the value preconditions */
    CKPT_E_CORRUPT = -7,    /* the arg table or operation list is not one this library wrote */
    CKPT_E_NOTREADY = -8,   /* helper streams are missing and cannot be created now (stream capture) */
    CKPT_E_INTERNAL = -9    /* ckpt_check_inputs: a bounded wait between work-groups expired; tables incomplete */
};

/*
 * Chain descriptors: DEVICE pointers, chain-major, int32.  Stage k of chain b is
 * element [b*L + (k-1)] of the [B][L] arrays; activation / gradient i is element
 * [b*(L+1) + i] of the [B][L+1] arrays.
 * Preconditions on values (checked on the device, see ckpt_check_inputs): all >= 0;
 * sum of u_f of a chain < 2^30 and every u_b < 2^30; every size and overhead
 * <= 2^28; omega_abar^k >= omega_a^k for every stage (abar^k contains a^k: without it
 * the Theorem is not the optimum over persistent schedules).  Costs that reach 2^30
 * saturate to CKPT_INF exactly as defined above.
 */
typedef struct ckpt_chains {
    const int32_t* uf;     /* [B][L]   u_f^k + u_fcomm^k            (Tables 1, 2) */
    const int32_t* ub;     /* [B][L]   u_b^k + u_bcomm^k                          */
    const int32_t* wa;     /* [B][L+1] omega_a^0..L                               */
    const int32_t* wabar;  /* [B][L]   omega_abar^1..L                            */
    const int32_t* wdelta; /* [B][L+1] omega_delta^0..L, or NULL: same as wa      */
    const int32_t* of;     /* [B][L]   o_f^k + o_fcomm^k, or NULL: zeros          */
    const int32_t* ob;     /* [B][L]   o_b^k + o_bcomm^k, or NULL: zeros          */
} ckpt_chains_t;

/* One operation of Table 1. */
enum { CKPT_OP_F_ALL = 0, CKPT_OP_F_CK = 1, CKPT_OP_F_NULL = 2, CKPT_OP_B = 3 };
typedef struct ckpt_op {
    uint8_t kind;  /* CKPT_OP_* */
    uint8_t stage; /* 1..L */
} ckpt_op_t;

/* Elements per table row: M+1 rounded up to a multiple of 64.  0 if M < 0. */
size_t ckpt_row_pitch(int M);
/* Rows per chain: L(L+1)/2.  0 if L < 1. */
size_t ckpt_table_rows(int L);
/* Row of cell (s, t), 1 <= s <= t <= L; -1 otherwise. */
long ckpt_row_index(int L, int s, int t);
/* Elements of the whole cost (or arg) table: B * rows * pitch.  0 on bad arguments. */
size_t ckpt_table_elems(int L, int M, int B);
/* Bytes of device workspace ckpt_solve_batched needs.  0 on bad arguments. */
size_t ckpt_workspace_bytes(int L, int M, int B);

/*
 * Set-up for one device (device < 0: the current one): creates the helper streams and events
 * of the batch split and sets the kernel attributes a solve needs.  Idempotent and
 * thread-safe; what it creates lives until the process ends.  ckpt_solve_batched does the
 * same on its first large solve on a device, except when its stream is being captured into
 * a HIP graph (nothing is created behind a capture: the solve then runs unsplit); call
 * ckpt_init first to capture split solves.
 * Returns CKPT_OK, CKPT_E_LIMIT (device >= 64) or CKPT_E_HIP.
 */
int ckpt_init(int device);

/*
 * Fill cost and arg for all B chains (Theorem, all three displays: the recurrence,
 * C_ck / C_all, and the thresholds m_null / m_all).
 *   chains    host pointer to a struct of DEVICE pointers (read during the call
 *             only; the arrays it names are read by the enqueued kernels)
 *   stream    a hipStream_t (NULL = the default stream); the call only enqueues
 *             work and returns, it does not synchronise and allocates no device
 *             memory; it may be captured into a HIP graph
 *   cost, arg DEVICE tables laid out as above, 256-byte aligned
 *   workspace DEVICE memory of ckpt_workspace_bytes(L, M, B) bytes, 256-byte
 *             aligned; holds per-chain prefix sums, thresholds and input flags
 * Returns CKPT_OK, CKPT_E_ARG, CKPT_E_LIMIT or CKPT_E_HIP.
 */
int ckpt_solve_batched(const ckpt_chains_t* chains, int L, int M, int B, void* stream,
                       int32_t* cost, uint8_t* arg, void* workspace);

/*
 * The same fill with the schedule under the caller's control.  The tables do not depend on
 * any of these choices, bit for bit.
 *   groups        0: automatic (a large batch is cut into up to four groups of chains that run
 *                 on four streams).  1: everything on `stream`; no helper stream, event or
 *                 lock of the library is touched.  2..4: that many groups (at most B), also on
 *                 small batches.
 *   side_streams  caller-owned hipStream_t for groups 2, 3, 4, or all NULL: the library's
 *                 helper streams.  The fork and join events are the library's in both cases.
 *   list_split    0: automatic.  1, 2 or 4: waves that share one chunk's list of splits in
 *                 every launch of the block-product kernel.
 *   row_launches  0: the rows of all tiles of a block diagonal are finished by one launch whose
 *                 work-groups wait for each other's rows.  1: one launch per row of the tiles.
 *   stagger       1: half of the groups start their first block product when the first group has
 *                 finished its own (an experiment: the phases of the groups then alternate).
 *   frontier      0: automatic.  1: always run the kernel that computes the exact feasibility
 *                 frontier.  2: never (the fill then prunes with the weaker bound
 *                 min(m_all, m_null) only).
 *   spin_limit    0: default.  > 0: polls after which a wait of one work-group for another gives up.
 *                 < 0: every such wait gives up at once -- for tests of the failure path: the
 *                 kernels still end normally, the tables are incomplete and ckpt_check_inputs
 *                 returns CKPT_E_INTERNAL.
 *   reserved      zeros
 * opts == NULL is ckpt_solve_batched.  Returns as ckpt_solve_batched, plus CKPT_E_NOTREADY
 * when groups > 1 is requested while `stream` is being captured and ckpt_init has not run.
 */
typedef struct ckpt_solve_opts {
    int groups;
    void* side_streams[3];
    int list_split;
    int row_launches;
    int stagger;
    int frontier;
    int spin_limit;
    int reserved[3];
} ckpt_solve_opts_t;
int ckpt_solve_batched_opts(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                            uint8_t* arg, void* workspace, const ckpt_solve_opts_t* opts);

/*
 * ckpt_solve_batched for callers that cannot allocate or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a
 * fixed array of CKPT_NOALLOC_MAX_WORKSPACE bytes inside the library's device code, one copy
 * per GPU, held until the process ends.  The call allocates nothing and creates nothing (the
 * batch is split over the helper streams only if ckpt_init has made them); its very first
 * use on a device resolves the array's address, so call ckpt_init once beforehand if that
 * first use would fall inside a stream capture.  Every call on one GPU uses the same array:
 * calls that overlap in time on one GPU race -- serialise them (one stream, or events).
 * The tables are those of ckpt_solve_batched, bit for bit.  ckpt_check_inputs with
 * workspace = NULL reads the flags of the most recent such solve on the current device.
 * Returns as ckpt_solve_batched, plus CKPT_E_LIMIT when ckpt_workspace_bytes(L, M, B) exceeds
 * CKPT_NOALLOC_MAX_WORKSPACE.
 */
#define CKPT_NOALLOC_MAX_WORKSPACE (16u << 20)
int ckpt_solve_batched_noalloc(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                               uint8_t* arg);

/*
 * Measurement aid: the same fill as ckpt_solve_batched on one stream, with a HIP event recorded
 * after every kernel launch.  The call waits for the stream, then adds the elapsed time between
 * consecutive events to the kernel kind launched in between (so a kind's time includes the
 * idle gap before each of its launches).
 *   kind_ms, kind_launches   HOST arrays of CKPT_N_KERNEL_KINDS entries, overwritten
 *   kind_bytes               HOST array of 2 * CKPT_N_KERNEL_KINDS doubles or NULL.  If given, the
 *                            fill runs a second time, untimed, and every wave of the two fill
 *                            kernels adds up what it asks the memory system for: entry 2k = bytes
 *                            of table loads of kind k (256 per wave and load), entry 2k + 1 =
 *                            bytes stored (320 per wave and cell: cost and candidate number).
 *                            Work that the feasibility tests skip is not counted.
 * Creates and destroys events and a small device buffer (allocates); not for latency-critical
 * callers.  Returns as ckpt_solve_batched.
 */
enum { CKPT_K_PRECOMPUTE = 0, CKPT_K_FRONTIER = 1, CKPT_K_GEMM = 2, CKPT_K_ROW = 3, CKPT_N_KERNEL_KINDS = 4 };
int ckpt_solve_profiled(const ckpt_chains_t* chains, int L, int M, int B, void* stream, int32_t* cost,
                        uint8_t* arg, void* workspace, float* kind_ms, int* kind_launches, double* kind_bytes);
/* Name of a kernel kind as it appears in a rocprofv3 kernel trace; NULL if out of range. */
const char* ckpt_kernel_name(int kind);

/*
 * After ckpt_solve_batched on the same stream (workspace = the one it was given; NULL = the
 * static one of ckpt_solve_batched_noalloc): wait for the stream and copy the
 * per-chain input flags (0 = chain met the value preconditions) into flags_host[B]
 * (HOST memory).  Returns CKPT_OK, CKPT_E_INPUT if any flag is nonzero (the
 * tables of such a chain are unspecified, all memory accesses stayed in bounds),
 * CKPT_E_ARG, CKPT_E_HIP, or CKPT_E_INTERNAL if a work-group of the fill gave up waiting for
 * another one (never seen; every such wait is bounded so that the kernels always end).
 * Bits: 1 negative value, 2 time too large, 4 size too large,
 * 8 some omega_abar^k below its omega_a^k (the tables of such a chain follow the printed
 * formulas, which are then no longer the optimum over persistent schedules).
 */
int ckpt_check_inputs(const void* workspace, int L, int M, int B, void* stream, int32_t* flags_host);

/*
 * Rebuild the operation sequence that realises C_BP(s, t, m_budget) of ONE chain
 * from its recorded candidates (C_ck / C_all of the Theorem read backwards; the
 * operations are those of Table 1).
 *   arg_host  HOST copy of that chain's arg table [rows][pitch]
 *   wa, wabar HOST arrays of that chain: omega_a^0..L [L+1], omega_abar^1..L [L]
 *   m_budget  memory for the segment, its input not counted; values above M read column M
 *             (as in ckpt_schedule_batched and ckpt_select_plan), negative values are an error
 *   ops_out   HOST array of ops_cap operations, written in execution order
 * Returns the number of operations (>= 2), or CKPT_E_ARG, CKPT_E_LIMIT,
 * CKPT_E_INFEASIBLE, CKPT_E_SMALLBUF, CKPT_E_CORRUPT.  Runs on the host only.
 */
int ckpt_schedule(const uint8_t* arg_host, const int32_t* wa, const int32_t* wabar, int L, int M,
                  int s, int t, int m_budget, ckpt_op_t* ops_out, int ops_cap);

/*
 * Activation-checkpoint block index of every stage (Section "Code generation": every node is
 * annotated with the index of its checkpoint block, and the nodes of one index are packaged
 * into one function that is wrapped in the framework's checkpoint call, which keeps the
 * block's input and recomputes its inside during the backward phase).  Read off an
 * operation list of the WHOLE chain (s = 1, t = L) as ckpt_schedule writes it: a stage's
 * annotation comes from its first forward operation -- F_ck^j opens a new block (only its
 * input is kept), F_null^j continues the block of stage j-1, F_all^j keeps abar^j and lies in
 * no block.  Later forwards of a stage are the recomputation and change nothing.
 *   ops, n_ops       HOST operation list
 *   block_of_stage   HOST out [L]: block number 0, 1, ... in chain order, -1 = in no block
 * Returns the number of blocks, or CKPT_E_ARG, CKPT_E_LIMIT, CKPT_E_CORRUPT (not the list of
 * a whole chain).  Runs on the host only.
 */
int ckpt_block_indices(const ckpt_op_t* ops, int n_ops, int L, int32_t* block_of_stage);

/*
 * Planner-side steps around the table fill (Section "Integrate Two Solvers": the planner
 * solves one chain per candidate intra-op plan and keeps the plan with the shortest total
 * time).  All three only enqueue work on `stream` and allocate nothing.
 */

/*
 * Plan selection: out[0] = the chain b with the smallest C_BP(1, L, m_b), the smallest b
 * on ties, -1 if no chain is feasible; out[1] = that cost (CKPT_INF if none).
 *   cost      DEVICE cost table filled by ckpt_solve_batched
 *   m_budget  DEVICE int32 [B]: memory for the whole chain of plan b, input a^0 already
 *             subtracted; values above M read column M, negative values are infeasible
 *   out       DEVICE int32 [2]
 * Returns CKPT_OK, CKPT_E_ARG, CKPT_E_LIMIT or CKPT_E_HIP.
 */
int ckpt_select_plan(const int32_t* cost, int L, int M, int B, const int32_t* m_budget, void* stream,
                     int32_t* out);

/*
 * Memory discretisation (the step the paper inherits from Rotor without describing it):
 * the byte budget of chain b is cut into M equal slots and every size is rounded up,
 *     slots = min(2^31 - 1, ceil(bytes * M / budget_bytes[b])),   exact integer arithmetic.
 *   bytes_*      DEVICE int64, shapes as the int32 arrays of ckpt_chains_t; bytes_wdelta,
 *                bytes_of, bytes_ob may be NULL (then the matching output is not written)
 *   budget_bytes DEVICE int64 [B], each > 0
 *   out          host struct of DEVICE int32 output pointers (uf, ub are ignored)
 * Preconditions (not checked): 0 <= bytes < 2^42, M <= 2^20, budget > 0.
 * Returns CKPT_OK, CKPT_E_ARG, CKPT_E_LIMIT or CKPT_E_HIP.
 */
int ckpt_discretize(const int64_t* bytes_wa, const int64_t* bytes_wabar, const int64_t* bytes_wdelta,
                    const int64_t* bytes_of, const int64_t* bytes_ob, const int64_t* budget_bytes, int L,
                    int M, int B, void* stream, const ckpt_chains_t* out);

/*
 * Memory budgets of the planner's loop (Section "Integrate Two Solvers": budgets (1+alpha)^n
 * for n = 0..9), scaled by a base budget, with alpha = alpha_num / alpha_den:
 *     budgets[n] = floor(base_budget * (1 + alpha)^n),  n = 0..count-1,  exact.
 * Host function, host output.  Returns CKPT_OK; CKPT_E_ARG (base_budget <= 0, alpha_num < 0,
 * alpha_den <= 0, count < 1, NULL); CKPT_E_LIMIT (count > CKPT_MAX_SWEEP, a budget above
 * 2^63 - 1, or base * (den + num)^n resp. den^n beyond 128 bits).
 */
#define CKPT_MAX_SWEEP 16
int ckpt_budget_sweep(int64_t base_budget, int alpha_num, int alpha_den, int count, int64_t* budgets);

/*
 * ckpt_discretize of ONE profile under every budget of ckpt_budget_sweep: chain n of the
 * output holds the profile's sizes in slots of budgets[n] / M bytes, so that the `count`
 * chains can go to ckpt_solve_batched as one batch.
 *   bytes_*      DEVICE int64 arrays of one chain ([L+1] resp. [L]); optional ones may be NULL
 *   budgets_out  DEVICE int64 [count] or NULL: the budgets used
 *   out          host struct of DEVICE int32 output pointers shaped for B = count chains
 * Preconditions and limits as for ckpt_discretize and ckpt_budget_sweep.
 * Returns CKPT_OK, CKPT_E_ARG, CKPT_E_LIMIT or CKPT_E_HIP.
 */
int ckpt_discretize_sweep(const int64_t* bytes_wa, const int64_t* bytes_wabar, const int64_t* bytes_wdelta,
                          const int64_t* bytes_of, const int64_t* bytes_ob, int64_t base_budget, int alpha_num,
                          int alpha_den, int count, int L, int M, void* stream, int64_t* budgets_out,
                          const ckpt_chains_t* out);

/*
 * ckpt_schedule for every chain at once, on the device: chain b is walked from cell
 * (1, L, min(m_budget[b], M)).
 *   arg        DEVICE arg table; wa, wabar DEVICE arrays of ckpt_chains_t shape
 *   ops        DEVICE [B][ops_cap]; ops_cap >= L(L+1)/2 + L always suffices
 *   n_ops      DEVICE int32 [B]: number of operations of chain b, or CKPT_E_INFEASIBLE,
 *              CKPT_E_SMALLBUF, CKPT_E_CORRUPT, CKPT_E_ARG (negative budget) for that chain
 *   workspace  DEVICE memory of ckpt_schedule_workspace_bytes(L, B) bytes
 * Returns CKPT_OK, CKPT_E_ARG, CKPT_E_LIMIT or CKPT_E_HIP.
 */
int ckpt_schedule_batched(const uint8_t* arg, const int32_t* wa, const int32_t* wabar, int L, int M, int B,
                          const int32_t* m_budget, void* stream, ckpt_op_t* ops, int ops_cap, int32_t* n_ops,
                          void* workspace);
/* Bytes of DEVICE workspace (16-byte aligned) ckpt_schedule_batched needs: the walk stacks. */
size_t ckpt_schedule_workspace_bytes(int L, int B);

/*
 * ckpt_block_indices for every chain at once, on the device, from the output of
 * ckpt_schedule_batched.
 *   ops, ops_cap, n_ops   DEVICE, as written by ckpt_schedule_batched
 *   block_of_stage        DEVICE int32 [B][L]; all -1 for a chain without a valid list
 *   n_blocks              DEVICE int32 [B]: number of blocks of chain b; n_ops[b] itself if that
 *                         is negative; CKPT_E_ARG if n_ops[b] > ops_cap; CKPT_E_CORRUPT if the
 *                         list is not that of a whole chain
 * Returns CKPT_OK, CKPT_E_ARG, CKPT_E_LIMIT or CKPT_E_HIP.
 */
int ckpt_block_indices_batched(const ckpt_op_t* ops, int ops_cap, const int32_t* n_ops, int L, int B, void* stream,
                               int32_t* block_of_stage, int32_t* n_blocks);

/*
 * Self-check of operation lists on the device: the list of every chain is executed over
 * stages 1..L under the memory model of Table 1 ("List of Operations") -- F_all^j and F_ck^j
 * read a^{j-1} (on its own or inside abar^{j-1}), keep it and add abar^j resp. a^j; F_null^j
 * reads a^{j-1} on its own, adds a^j and drops a^{j-1}; B^j reads delta^j, abar^j and a^{j-1},
 * adds delta^{j-1} and drops delta^j, abar^j and an a^{j-1} held on its own -- counted the way
 * the Theorem's thresholds count: a^0 is free, delta^L is resident from the start, a forward
 * operation needs room for its output and o_f^j while it runs, B^j needs o_b^j and does not
 * count its output while it runs.  A list realises cell (1, L, m) of the cost table exactly
 * when time_out equals the cell's cost and peak_out <= m.
 *   chains     host struct of DEVICE pointers, as for ckpt_solve_batched (values >= 0)
 *   ops, ops_cap, n_ops   DEVICE, as written by ckpt_schedule_batched
 *   time_out   DEVICE int64 [B]: sum of u_f / u_b over the list, -1 unless status is CKPT_OK
 *   peak_out   DEVICE int64 [B]: largest memory need over the list, -1 unless status is CKPT_OK
 *   status     DEVICE int32 [B]: CKPT_OK; CKPT_E_CORRUPT for a list that cannot be executed (an
 *              operand that is not resident, a tensor computed while it is resident, an unknown
 *              operation or stage) or that ends without delta^0; CKPT_E_ARG if n_ops[b] >
 *              ops_cap; n_ops[b] itself if that is negative (the chain is skipped)
 * Returns CKPT_OK, CKPT_E_ARG, CKPT_E_LIMIT or CKPT_E_HIP.
 */
int ckpt_simulate_batched(const ckpt_chains_t* chains, int L, int B, const ckpt_op_t* ops, int ops_cap,
                          const int32_t* n_ops, void* stream, int64_t* time_out, int64_t* peak_out,
                          int32_t* status);

/*
 * Network linearisation on the host (Sections "Linearization", "Common Node" and the
 * algorithm of "Full Set of Linearization Rules"): cuts a computation DAG into the node
 * groups that become the stages of a chain.
 *   n, child_ptr[n+1], child_idx   HOST CSR adjacency; nodes are numbered in topological
 *                                  order (every child index is larger than its parent's)
 *   flags[n]                       HOST CKPT_NODE_* bit sets
 *   group_of_node[n]               HOST out: group index 0.., -1 for placeholders
 *   is_common[n]                   HOST out: 1 if the node is a common node (seeded, or its
 *                                  operation is non-differentiable, or all its parents are common)
 * A node that is neither placeholder nor common keeps dependencies outstanding until the last
 * of its non-placeholder children has been appended.  A node ends a group when, once it has
 * been appended, no earlier node has a dependency outstanding and none of its own children is
 * an in-place or communication operation.  Nodes left after the last cut form a final group.
 * Returns the number of groups, or CKPT_E_ARG (bad pointers, edges that are not forward).
 */
enum {
    CKPT_NODE_PLACEHOLDER = 1, /* network input or output */
    CKPT_NODE_COMMON_SEED = 2, /* non-differentiable input, e.g. an attention mask */
    CKPT_NODE_NON_DIFF = 4,    /* non-differentiable operation, e.g. getattr, getitem */
    CKPT_NODE_IN_PLACE = 8,    /* in-place operation: stays with its parent */
    CKPT_NODE_COMM = 16        /* communication operation: stays with its parent */
};
int ckpt_linearize(int n, const int32_t* child_ptr, const int32_t* child_idx, const uint8_t* flags,
                   int32_t* group_of_node, uint8_t* is_common);

/* hipError_t of the most recent failed HIP call made by this library (0 if none). */
int ckpt_last_hip_error(void);
/* Static description of a CKPT_* code. */
const char* ckpt_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CKPT_DP_H */
