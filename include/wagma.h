/*
 * libwagma — the per-iteration hot path of WAGMA-SGD (wait-avoiding group
 * model averaging, arXiv 2005.00124) for P model replicas that live as P rows
 * in the HBM of one AMD MI355X (gfx950).
 *
 * One call of wagma_step() is one iteration t of Algorithm 2, lines 6-17, for
 * all P processes at once:
 *   lines 6-7   local update  m' = mu*m + g,  W' = W - lr*m'   (heavy-ball SGD)
 *   lines 9-14  group model average over the groups of Algorithm 1, with the
 *               stale rule (W_sum + W')/(S+1) for late processes, whose
 *               contribution to W_sum is their send buffer ("pub")
 *   lines 15-16 global average over all P when (t+1) mod tau == 0
 *   Section 4   (execution snapshot): the send buffer is refreshed with W'.
 *
 * Conventions common to all entry points
 *   - Plain C ABI.  "device" pointers are HIP device memory on the GPU that was
 *     current when the context was created; "host" pointers are ordinary host
 *     memory.  The library never takes ownership of a caller's buffer.
 *   - Every function returns WAGMA_OK (0) or a negative error code; nothing is
 *     thrown, nothing aborts, and on error no caller buffer has been modified.
 *   - A context is not thread-safe; different contexts are independent.
 *   - Layout of w, g, m, pub: P rows of ld floats (row-major, row p at
 *     base + p*ld), fp32, base 16-byte aligned, ld = wagma_row_stride(ctx)
 *     (a multiple of 4, >= n).  Columns [0, n) carry the model.  Columns
 *     [n, ld) are padding: the library may read them and may overwrite columns
 *     [n, 4*ceil(n/4)) with unspecified values; it never lets padding
 *     influence columns [0, n).  The four arrays must be four different pieces
 *     of memory: arrays whose P*ld-float extents overlap are WAGMA_EINVAL.
 *     Any 16-byte aligned base is correct; the step is fastest when the arrays
 *     begin on 64 KiB boundaries (device allocations of this size do) and the
 *     row stride is the one wagma_create chose (a multiple of 64 KiB for
 *     n >= 2^18): off such boundaries up to 15 % of the bandwidth is lost.
 */
#ifndef WAGMA_H
#define WAGMA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define WAGMA_OK 0
#define WAGMA_EINVAL (-1) /* bad argument: P or S not a power of two, S > P, n < 1,
                             tau < 0, NULL or misaligned pointer, negative iter, ... */
#define WAGMA_EHIP (-2)   /* a HIP runtime call failed; see wagma_last_hip_error() */
#define WAGMA_ENOMEM (-3) /* a host or device allocation failed */

#define WAGMA_MAX_P 1024 /* largest supported number of processes */

typedef struct wagma_ctx wagma_ctx; /* opaque; owned by the library */

/*
 * Create a context for P processes in groups of S on models of n parameters,
 * with a global average every tau iterations (Algorithm 2, inputs; P and S
 * powers of two with S <= P as Section 3.3 assumes).
 *   out  host pointer that receives the context.
 *   P    1 <= P <= WAGMA_MAX_P, power of two.      S  1 <= S <= P, power of two.
 *   n    1 <= n <= 2^31.     tau  >= 0; 0 = never average globally, 1 = every iteration.
 * Builds the group-schedule table (Algorithm 1 for every distinct iteration
 * residue) with a kernel on the current device, keeps it in device memory and
 * mirrors it on the host.  Synchronises the device once.  Chooses the row
 * stride ld.
 */
int wagma_create(wagma_ctx** out, int P, int S, int64_t n, int tau);

/* Frees the tables and the context.  Does not touch caller buffers.  The
 * caller must have synchronised every stream that still runs a wagma_step of
 * this context.  NULL is accepted. */
int wagma_destroy(wagma_ctx* ctx);

/* Row stride ld in floats chosen by wagma_create (>= n, multiple of 4), or a
 * negative error code.  The caller allocates P*ld floats per buffer. */
int64_t wagma_row_stride(const wagma_ctx* ctx);

/* Override the row stride (before the first step): ld >= 4*ceil(n/4), ld % 4 == 0.  While arrays
 * of wagma_alloc_buffers exist, a stride above the one they were sized for is WAGMA_EINVAL. */
int wagma_set_row_stride(wagma_ctx* ctx, int64_t ld);

/*
 * The paper's family of variants (Section 4, the paragraph on the four parameters tau, alpha,
 * beta, S; Section 6.2, the four ablation experiments) is reached through the arguments:
 *   wait-avoiding group allreduce (alpha)      a stale_mask with late processes
 *   plain group allreduce (beta)               stale_mask = NULL
 *   local SGD with period tau (ablation 1)     S = 1
 *   global model averaging every step          tau = 1   (or S = P: ablation 3)
 *   smaller groups (ablation 4)                S
 *   no periodic synchronisation                tau = 0
 *   fixed groups (ablation 2)                  wagma_set_grouping(ctx, WAGMA_GROUPING_FIXED):
 *       every group iteration uses the groups of iteration 0 instead of Algorithm 1's
 *       rotation; global iterations are unchanged.
 */
#define WAGMA_GROUPING_DYNAMIC 0 /* Algorithm 1 (default) */
#define WAGMA_GROUPING_FIXED 1   /* the groups of iteration 0, always */
int wagma_set_grouping(wagma_ctx* ctx, int mode);

/* Number of distinct group schedules: the schedule of iteration t equals that
 * of iteration t + period.  period = G / gcd(g, G) with G = log2 P, g = log2 S
 * (the starting phase of Algorithm 1, line 3, is (t*g) mod G). */
int wagma_schedule_period(const wagma_ctx* ctx);

/*
 * Group schedule of iteration iter (Algorithm 1; iter is the paper's 0-based t).
 *   dev_table   host pointer receiving a DEVICE pointer to P int32, or NULL.
 *   host_table  host pointer receiving a HOST pointer to the same P int32, or NULL.
 * Entry k*S + e is the rank of member e of group k.  Groups are listed by
 * ascending smallest member; member e differs from the smallest member in the
 * phase bits selected by the binary digits of e (digit r <-> phase r of
 * Algorithm 1), so e and e^1 exchange in the first butterfly phase.
 * For an iteration that ends in the global average ((iter+1) mod tau == 0) the
 * table is the single group 0..P-1.
 * Both pointers stay valid until wagma_destroy and must not be written.
 */
int wagma_group_schedule(const wagma_ctx* ctx, int64_t iter,
                         const int32_t** dev_table, const int32_t** host_table);

/* 1 if iteration iter ends in the global average, 0 if in group averages,
 * negative on error (Algorithm 2, line 8). */
int wagma_is_global_iteration(const wagma_ctx* ctx, int64_t iter);

/*
 * One iteration of Algorithm 2 (lines 6-17) for all P processes, enqueued on
 * `stream`; returns without waiting for the GPU.
 *   w     device, in/out  P x ld   models W_t -> W_{t+1}
 *   g     device, in      P x ld   local gradients G_t (never written)
 *   m     device, in/out  P x ld   momentum state
 *   pub   device, in/out  P x ld   send buffers: read for late processes (their
 *                                  contribution to the group sum), then set to W'_t.
 *                                  Must be initialised (e.g. to W_0) before the first
 *                                  step in which a process is late.
 *   stale_mask  host, ceil(P/64) words; bit p of the mask set = process p is late
 *               in this iteration.  NULL = nobody is late.  Read before the call
 *               returns; ignored in a global iteration (Section 4: all processes
 *               contribute equally aged models at the synchronisation point).
 *   lr, mu      learning rate and momentum coefficient.
 *   iter        the paper's 0-based t; selects the groups and group/global.
 *               Calls may come in any order of iter: the context keeps no
 *               iteration state, so resuming is passing the right iter.
 *   stream      a hipStream_t (NULL = the default stream).
 * Arithmetic is IEEE fp32: both update lines are one fused multiply-add each,
 * the group (or global) sum is a balanced pairwise tree over the member order
 * of wagma_group_schedule, 1/S and 1/P are exact, 1/(S+1) is a true division.
 * No allocation, no host<->device copy and no synchronisation happen here.
 */
int wagma_step(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub,
               const uint64_t* stale_mask, float lr, float mu, int64_t iter,
               void* stream);

/*
 * Per-tensor layout.  Training frameworks keep a model as a list of tensors (the ResNet-50 of
 * Section 6.2 has 161, each replica its own set), not as one flat row.  A plan describes
 * where they are; wagma_step_tensors then does exactly what wagma_step does (same arithmetic,
 * same order, same results) on that layout.
 *   T       number of tensors per replica, >= 1.
 *   sizes   host, T entries: floats in tensor k; their sum must be the n of wagma_create.
 *   w, g, m, pub   host arrays of P*T DEVICE pointers; entry p*T + k is tensor k of process p.
 *           Every pointer 16-byte aligned; tensors must not overlap one another.  Sizes need
 *           not be multiples of 4: nothing beyond a tensor's last element is read or written.
 * wagma_tensors_create copies the tables to the device (allocation, copy and synchronisation
 * happen here, none in the step); the plan refers to ctx and to the tensors, which must stay
 * where they are while the plan is used.  Destroy the plan before its context.
 * Any placement of the tensors gives the same results; wagma_tensors_create recognises by
 * itself what makes the step faster:
 *   - tensors that follow one another without a gap, in every array of every process (views into
 *     one buffer per process), count as one tensor: a model that is views into P rows, back to
 *     back, runs at the rate of wagma_step;
 *   - where the P replicas of a tensor lie equally far apart, by the same distance in w, g, m
 *     and pub (a parameter stacked to [P, ...], views into P rows), the step computes every
 *     address from one table entry per 4 KiB tile; else it reads the tensors' pointers from a
 *     table laid out by the places of the group schedule (the same rate for groups of up to 8,
 *     a few per cent less for larger ones);
 *   - large tensors that begin at the same address modulo 64 KiB in every process and array
 *     (a distance between replicas that is a multiple of 64 KiB, or allocations of their own).
 */
typedef struct wagma_tensors wagma_tensors;
int wagma_tensors_create(wagma_ctx* ctx, wagma_tensors** out, int T, const int64_t* sizes,
                         float* const* w, const float* const* g, float* const* m, float* const* pub);
int wagma_tensors_destroy(wagma_tensors* plan);
/* One iteration of Algorithm 2 (lines 6-17) on the tensors of `plan`; stale_mask, lr, mu, iter
 * and stream as for wagma_step.  Launch only: no allocation, copy or synchronisation. */
int wagma_step_tensors(wagma_ctx* ctx, const wagma_tensors* plan, const uint64_t* stale_mask,
                       float lr, float mu, int64_t iter, void* stream);

/*
 * Lateness deeper than one iteration.  The execution snapshot of Section 4 shows a straggler
 * whose send buffer is taken by a group allreduce while it is still computing; Assumption 1
 * (item 3) lets that go on for up to tau iterations.  In wagma_step_lag a process is in one of
 * three states in a group iteration:
 *   in time          bit clear in both masks: Algorithm 2 lines 6-7 and 9-11;
 *   late             bit set in late_mask: it contributes its send buffer, ends its local step
 *                    afterwards and averages the group's sum with its W' (lines 12-13), exactly
 *                    the stale_mask of wagma_step;
 *   still computing  bit set in busy_mask (late_mask is then not looked at for it): it
 *                    contributes its send buffer once more and nothing else of it is read or
 *                    written: no gradient, no local step, send buffer not refreshed; the sum it
 *                    would find in its receive buffer is overwritten by a later one.
 * A global iteration ((iter+1) mod tau == 0) waits for everybody: both masks are ignored.
 * late_mask, busy_mask: host, ceil(P/64) words each, bit p = process p, either may be NULL
 * (nobody), consumed before the call returns.  With busy_mask NULL or empty the call is
 * wagma_step.  All other arguments, errors and the absence of allocation, copies and
 * synchronisation as for wagma_step and wagma_step_tensors.
 */
int wagma_step_lag(wagma_ctx* ctx, float* w, const float* g, float* m, float* pub,
                   const uint64_t* late_mask, const uint64_t* busy_mask, float lr, float mu,
                   int64_t iter, void* stream);
int wagma_step_tensors_lag(wagma_ctx* ctx, const wagma_tensors* plan, const uint64_t* late_mask,
                           const uint64_t* busy_mask, float lr, float mu, int64_t iter, void* stream);

/*
 * wagma_step for callers that cannot allocate device memory or keep a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The one piece of device
 * memory the step's kernels use beyond the caller's arrays, the group-schedule table that
 * wagma_create allocates, lives here in a static device array of WAGMA_STATIC_TABLE_BYTES that
 * each GPU the library runs on holds until the process ends.  The call writes the table for
 * (P, S) into that array with a kernel on `stream` and then launches the same step kernel as
 * wagma_step on `stream`: same arithmetic, same results.  It allocates nothing, copies nothing
 * and does not synchronise.
 *   P, S, n, tau   as for wagma_create (P <= WAGMA_MAX_P is what the array holds; beyond it,
 *                  and for every other bad size, WAGMA_EINVAL before anything is launched).
 *   ld             row stride in floats (multiple of 4, >= 4*ceil(n/4)), or 0 for the stride
 *                  wagma_create would choose for this n.
 *   w, g, m, pub, stale_mask, lr, mu, iter, stream   as for wagma_step, on the current device.
 * Every call on one GPU shares that GPU's array: calls that may overlap on one GPU (different
 * streams, or graphs replayed concurrently) race on it unless they use the same P and S.
 */
#define WAGMA_STATIC_TABLE_BYTES 45056 /* 11 * WAGMA_MAX_P int32: (log2 P + 1) schedules of P ranks */
int wagma_step_static(int P, int S, int64_t n, int tau, int64_t ld, float* w, const float* g,
                      float* m, float* pub, const uint64_t* stale_mask, float lr, float mu,
                      int64_t iter, void* stream);

/*
 * Seeded lateness model (not from the paper, whose lateness is physical; its
 * simulation delays random ranks, Section 6.2): process p is late in iteration
 * iter iff the upper 32 bits of a 64-bit hash of (seed, iter, p) are below
 * `threshold` = floor(q * 2^32).  Integer arithmetic only.
 *   mask_words  host, out, ceil(P/64) words in the layout wagma_step takes.
 */
int wagma_stale_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter,
                     uint32_t threshold, uint64_t* mask_words);

/*
 * Two more lateness models, both integer-only and reproducible, in the layout wagma_step takes.
 *
 * wagma_straggler_mask: exactly `count` randomly selected processes are late in iteration iter,
 * as the image-classification experiment injects its delays (Section 6.2 selects two processes
 * per training step).  0 <= count <= P.
 *
 * wagma_clock_mask: every process draws a step time shaped like the reinforcement-learning
 * workload of Section 6.4 (1.7 s to 43.5 s, median below 2 s: nine steps in sixteen take
 * 1.7-2 s, the others one of 16 geometrically spaced times from 2 s to 43.5 s).  The process that
 * finishes first is the activator of Section 3.2 and is never late; any other process is late
 * iff it finishes more than tolerance_ms after it.  step_ms (host, P entries, may be NULL)
 * receives the step times in milliseconds.
 */
int wagma_straggler_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, int count,
                         uint64_t* mask_words);
int wagma_clock_mask(const wagma_ctx* ctx, uint64_t seed, int64_t iter, uint32_t tolerance_ms,
                     uint64_t* mask_words, uint32_t* step_ms);

/*
 * The two masks of wagma_step_lag for iteration iter when nobody waits for anybody between two
 * global iterations (Section 3.2): every process runs its local steps back to back with the step
 * times of wagma_clock_mask (a step begun for the group allreduce of iteration k takes the time
 * the process draws in iteration k); the first process to end a step begun for an allreduce
 * activates it, the allreduce reads the models tolerance_ms later, and who arrived by then takes
 * the average and goes on from that moment.  A process that ends a step after an allreduce has
 * read and before the next one reads is late in that iteration and begins its next step at
 * once; one that is still computing when the next one reads is busy.  The clocks restart after
 * every global iteration, where everybody waits (both masks are empty there); a context with
 * tau == 0 restarts them every `window` iterations (window >= 1; ignored when tau > 0), so that
 * no send buffer is older than that (Assumption 1, item 3).
 *   tolerance_ms  below 1700 (the shortest step), else WAGMA_EINVAL.
 *   late_words, busy_words   host, out, ceil(P/64) words each; no process is in both.
 * Integer only and reproducible; host work proportional to P times the iterations since the
 * clocks restarted.
 */
int wagma_lag_masks(const wagma_ctx* ctx, uint64_t seed, int64_t iter, int window,
                    uint32_t tolerance_ms, uint64_t* late_words, uint64_t* busy_words);

/*
 * Optional allocator for the four P x ld arrays (device memory, contents unspecified).  A caller
 * may always bring its own buffers instead; results never depend on where the arrays lie.
 * On MI355X the HBM falls into three regions of about 96 GiB (selected by the top physical
 * address bits).  Where the four arrays lie among them decides a few per cent of the step's
 * bandwidth, and differently for its kernels: the one that holds a group of up to 8 rows in
 * registers is fastest on arrays that all lie in one region, the one for larger groups where w,
 * m and pub lie in three.  Regions cannot be queried, so the allocator finds them by timing a
 * small write kernel on pairs of memory blocks, and places the arrays in one of these ways:
 *   WAGMA_PLACE_CHUNKS  every array is built, through the virtual memory API, from 1 GiB
 *                       chunks after one of three patterns, whichever the step runs fastest
 *                       on: w, g and m from one region and pub (written, hardly ever read)
 *                       from another; all chunks of all arrays from one region; or so that
 *                       at every column w, m and pub lie in three regions and g lies with w;
 *   WAGMA_PLACE_ARRAYS  whole arrays: w, m, pub in three regions, g in that of w (regions
 *                       found with the probe);
 *   WAGMA_PLACE_SEARCH  up to eight candidate arrays spread over the free memory, and a
 *                       descent over which of them plays which role, judged by the time of
 *                       the step kernel itself (no assumption about regions);
 *   WAGMA_PLACE_PLAIN   four ordinary allocations.
 * On a GPU whose memory is untouched ordinary allocations lie in one region; on one that has
 * been in use they are mixed over the regions, and arrays built from chunks bring back what
 * that costs (0.80 -> 0.81 of the peak bandwidth on a 26 GB problem) or more.  By default
 * (WAGMA_PLACE_AUTO) PLAIN and the three forms of CHUNKS are each timed with the step kernels,
 * in this order, and a later one replaces what is kept if it is 0.5 % faster.
 * On the arrays it hands out the call also measures which way of dealing the column tiles out to
 * the chip's eight dies and to the wavefronts of a workgroup is fastest for steps on these
 * arrays, and the context uses that one whenever a step is given exactly these four arrays
 * (results do not depend on it; a caller's own arrays get a fixed choice).
 * Arrays under 1 GiB get plain allocations.  The call takes from a fraction of a second to
 * some twenty seconds, may hold most of the free memory while it searches, synchronises the
 * device and runs kernels on the default stream.  One set of buffers per context: a second
 * call before wagma_free_buffers is WAGMA_EINVAL.  wagma_destroy frees buffers that are still
 * allocated; free them (or destroy the context) only when no step is running on them.
 */
int wagma_alloc_buffers(wagma_ctx* ctx, float** w, float** g, float** m, float** pub);
int wagma_free_buffers(wagma_ctx* ctx);
/* What the last wagma_alloc_buffers found (any pointer may be NULL): the WAGMA_PLACE_* it ended
 * with, memory blocks examined, how many regions w, m, pub are spread over (1..3, 0 = not
 * known), whether g
 * lies with w (1/0), and the probe's write rate in GB/s inside one region and across two
 * (0 = unknown). */
int wagma_placement_info(const wagma_ctx* ctx, int* mode, int* candidates, int* regions, int* g_with_w,
                         double* same_gbs, double* split_gbs);

/* Options; the defaults are the measured best on MI355X.  Results do not depend on them. */
#define WAGMA_OPT_NONTEMPORAL 2  /* 0/1: non-temporal hint on loads and stores (default: 1
                                    unless the four arrays fit in 256 MB together)     */
#define WAGMA_OPT_PLACEMENT 9    /* how wagma_alloc_buffers places the arrays: WAGMA_PLACE_*  */
#define WAGMA_PLACE_PLAIN 0      /* four ordinary allocations                                  */
#define WAGMA_PLACE_ARRAYS 1     /* whole arrays in different HBM regions                      */
#define WAGMA_PLACE_CHUNKS 2     /* arrays built from 1 GiB chunks of chosen regions (three patterns) */
#define WAGMA_PLACE_AUTO 3       /* default: PLAIN and the patterns of CHUNKS are timed with the
                                    step kernel and the fastest is kept                      */
#define WAGMA_PLACE_SEARCH 4     /* candidate arrays spread over the free memory; which one
                                    becomes w, g, m, pub is decided by timing the step kernel */
int wagma_set_option(wagma_ctx* ctx, int option, int64_t value);

/* Text for an error code (static storage). */
const char* wagma_strerror(int code);

/* The hipError_t (as int) of the last failed HIP call in this thread, 0 if none. */
int wagma_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* WAGMA_H */
