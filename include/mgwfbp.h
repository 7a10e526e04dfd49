/*
 * mgwfbp.h - C ABI of the MI355X merged-gradient reduction library (libmgwfbp.so).
 *
 * The library implements, for one GPU's share of a data-parallel S-SGD job, the data
 * path behind MG-WFBP (Shi, Chu, Li, "MG-WFBP: Efficient Data Communication for
 * Distributed Synchronous SGD Algorithms"):
 *
 *   plan    which consecutive layers send their gradients as one message
 *           (Section III, Eq. 19-23; Section IV, Theorem 1 and Algorithm 1);
 *   pack    the layer buffer of Algorithm 2: the gradients of a group laid end to end in
 *           arrival order of the backward pass (Definition 1, Condition 3 / Eq. 16);
 *   reduce  the arithmetic of the all-reduce: sum over the N workers, times 1/N (Eq. 2);
 *   unpack  the averaged values back into per-layer tensors, optionally with the weight
 *           update of Algorithm 2 (W = W - eta * grad, Eq. 1-2) extended by a momentum
 *           buffer.
 *
 * Conventions
 *   - Layers are 0-based in every array: index 0 is the paper's layer 1.  The backward pass
 *     visits index L-1 first.  Groups are numbered in communication order: group 0 holds
 *     the highest layers and is ready first.
 *   - All gradients, weights and momentum buffers are fp32 (Section V).  Message sizes in
 *     the cost model are bytes: a layer of p parameters is a 4p-byte message.
 *   - The N workers' gradients are N replicas resident in this GPU's memory.
 *   - "host" / "device" is stated for every pointer.  The caller owns every tensor, the
 *     workspace and the stream.  The library owns the plan handle and the small device
 *     tables created by mgwfbp_bind; mgwfbp_plan_destroy frees both.
 *   - Every function returns a status code and never throws or aborts.  On failure
 *     mgwfbp_last_error() describes the reason (thread-local, library-owned string).
 *   - Device work is enqueued on the caller's HIP stream and is asynchronous; the caller
 *     synchronises.  A launch failure is reported as MGWFBP_EHIP.
 *   - Reduction arithmetic is fixed: acc = x_0; acc = acc + x_g for g = 1..N-1 in fp32
 *     (round to nearest even, no fused multiply-add), result = acc * (1.0f / N).
 *     Update arithmetic: v = mu*v + g; w = w - lr*v, each operation rounded separately.
 *     Pack and unpack are bit copies.
 *   - A plan handle must not be used from two threads at once.
 *   - Launches read the plan's device tables while they run: wait for the streams they were
 *     enqueued on before calling mgwfbp_bind again or mgwfbp_plan_destroy.
 *   - mgwfbp_bind places the plan's tables on the current device; later launches must be made
 *     with that device current (MGWFBP_ESTATE otherwise).
 */
#ifndef MGWFBP_H
#define MGWFBP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mgwfbp_plan_s mgwfbp_plan_t; /* opaque */

enum {
    MGWFBP_OK = 0,
    MGWFBP_EINVAL = -1, /* bad argument (null pointer, L < 1, N < 1, p = 0, negative or NaN time ...) */
    MGWFBP_ENOMEM = -2, /* host or device allocation failed */
    MGWFBP_EHIP = -3,   /* a HIP runtime call failed */
    MGWFBP_ESTATE = -4  /* call not valid in the handle's state (e.g. launch before bind) */
};

enum {
    MGWFBP_MODE_OPTIMAL = 0,      /* exact minimum of Eq. 19-23 by an O(L^2) dynamic program   */
    MGWFBP_MODE_PAPER_GREEDY = 1, /* the rule of Theorem 1 / Algorithm 1                        */
    MGWFBP_MODE_WFBP = 2,         /* no merging: every layer is its own group (Section II-C)    */
    MGWFBP_MODE_SINGLE = 3        /* all layers in one group (the single-message scheme of Sec. I) */
};

/* Tuning keys for mgwfbp_plan_set_option (before mgwfbp_bind). */
enum {
    MGWFBP_OPT_TILE_ELEMS = 1,  /* elements of one layer handled by one workgroup; multiple of 1024, <= 8192 */
    MGWFBP_OPT_SMALL_ELEMS = 2, /* layers shorter than this share gather tiles (default 64)         */
    MGWFBP_OPT_NONTEMPORAL = 3, /* 1: streaming (non-temporal) loads and stores; 0: plain            */
    MGWFBP_OPT_PACE = 4,        /* pause between two loads of a wave, units of ~64 clocks, 0..16;
                                   -1 (default): chosen per launch from its size and N           */
    MGWFBP_OPT_LONG_TILES = 5,  /* tile length of the whole-plan fused reduce pass (only next to
                                   tile_elems = 4096).  -1 (default): the length among 4096, 5120,
                                   6144, 7168, 8192 that fills the chip's batches of workgroups best
                                   for this plan's size; 0: tile_elems; 1 or 8192, 5120, 6144, 7168:
                                   that length                                                     */
    MGWFBP_OPT_PAD_ELEMS = 6,   /* layout of the merged buffers.  0 (default): the layers of a group
                                   follow each other without padding, as the cost model counts them
                                   (Condition 3).  4, 8, 16 or 32: every layer starts on a multiple of
                                   that many elements (4: a 16-byte boundary, so that every copy is
                                   128 bits wide whatever the layer lengths; 32: a 128-byte boundary,
                                   so that both sides of every copy are aligned to whole memory
                                   lines); the padding elements after a layer are written as zeros by
                                   pack and mgwfbp_pack_reduce and skipped by unpack.  offset_in_group,
                                   group_elems, workspace and merged-buffer sizes follow the layout;
                                   the predicted times do not change                               */
    MGWFBP_OPT_UPDATE_WGS_PER_CU = 7, /* workgroups of the update kernel (mgwfbp_step without
                                   workspace) one compute unit may hold.  -1 (default): chosen per
                                   launch so that its batches of resident workgroups fill well;
                                   0: whatever the kernel's registers allow (14; 12 for N = 16);
                                   8, 9, 10, 11: that many.  Results do not depend on it            */
    MGWFBP_OPT_GATED_WGS_PER_CU = 8, /* workgroups per compute unit in mgwfbp_gated_launch, which
                                   stay for the whole launch: -1 (default) four fewer than a unit
                                   holds, or 1 .. 15 (never more than two fewer than it holds):
                                   the rest is room for the kernels that produce the gradients     */
    MGWFBP_OPT_GATED_CUS = 9        /* compute units the stream of mgwfbp_gated_launch may use, when
                                   the caller made it with a compute-unit mask
                                   (hipExtStreamCreateWithCUMask) so that the other units stay
                                   free for kernels that need whole SIMDs: the grid is sized for
                                   that many units.  0 (default): all of the device              */
};

/*
 * Merge planning (Algorithm 1's inputs: a, b, L, N, p; t_b and t_f stand for T_b and T_f,
 * which the paper derives from benchmarks of the first iterations).
 *
 *   L              number of learnable layers, 1 .. 2^20.  The exact planner stops growing a
 *                  message once no longer one can win, which makes it near-linear while the net
 *                  has compute-bound stretches (0.2 s for 2^20 layers); a net that is
 *                  communication-bound throughout costs the full O(L^2): 0.1 s at 10^4 layers,
 *                  about 10 s at 10^5.  The other modes are linear.
 *   p_elems        host [L]   parameters per layer, each >= 1, at most 2^40 in total
 *   tb_ms          host [L]   backward time of each layer, finite and >= 0
 *   tf_ms          forward time (a pure offset of the timeline), finite and >= 0
 *   a_ms, b_ms_per_byte       all-reduce cost T_ar(M) = a + b*M (Eq. 9), finite and >= 0
 *   N              number of workers (>= 1); only used for the 1/N scale
 *   mode           MGWFBP_MODE_*
 *   out            receives a new handle; free with mgwfbp_plan_destroy
 *
 * The predicted iteration time follows Eq. 6-8 with Conditions 1-3 for merged layers.
 * Ties between equally good plans are broken towards smaller groups (Theorem 1's
 * inequality is strict).
 */
int mgwfbp_plan(int32_t L, const uint64_t *p_elems, const double *tb_ms, double tf_ms,
                double a_ms, double b_ms_per_byte, int32_t N, int32_t mode, mgwfbp_plan_t **out);

/*
 * Same, but with the merged-gradient set M given by the caller (Eq. 22):
 *   merged  host [L] bytes; merged[l] != 0 means layer l (0-based, l >= 1) sends its gradients
 *           together with layer l-1.  merged[0] must be 0.
 */
int mgwfbp_plan_explicit(int32_t L, const uint64_t *p_elems, const double *tb_ms, double tf_ms,
                         double a_ms, double b_ms_per_byte, int32_t N, const uint8_t *merged,
                         mgwfbp_plan_t **out);

/*
 * Read a plan back: the merged-gradient set M of Eq. 22 as groups, and where each layer sits in
 * its group's merged message (Condition 3 / Eq. 16: a merged layer's parameters are appended to
 * those of the layer below it).  Every out-pointer is a host pointer and may be NULL.
 *   n_groups         number of groups
 *   group_of_layer   [L]  group id of each layer
 *   offset_in_group  [L]  element offset of the layer inside its group's merged buffer
 *                         (arrival order: the highest layer of a group has offset 0)
 *   group_elems      [n_groups]  total elements of each group's merged buffer (no padding
 *                         unless MGWFBP_OPT_PAD_ELEMS is set)
 *   t_iter_ms        predicted iteration time of this plan
 *   t_iter_wfbp_ms   predicted iteration time without merging
 */
int mgwfbp_plan_info(const mgwfbp_plan_t *plan, int32_t *n_groups, int32_t *group_of_layer,
                     uint64_t *offset_in_group, uint64_t *group_elems, double *t_iter_ms,
                     double *t_iter_wfbp_ms);

/*
 * Predicted timeline of the plan (Eq. 6-8): host arrays, any may be NULL.
 *   mu_b          [L]         when each layer's gradients are ready (tau_b + t_b)
 *   group_start   [n_groups]  tau_c of each group's message
 *   group_finish  [n_groups]  tau_c + T_ar of each group's message
 */
int mgwfbp_plan_timeline(const mgwfbp_plan_t *plan, double *mu_b, double *group_start,
                         double *group_finish);

/* Set a tuning option (MGWFBP_OPT_*).  Only before mgwfbp_bind; MGWFBP_ESTATE afterwards. */
int mgwfbp_plan_set_option(mgwfbp_plan_t *plan, int32_t key, int64_t value);

/*
 * Host-only view of the segment and tile tables the kernels would run with under the plan's
 * current options (the tile table of Section IV's layer buffer, cut for the GPU).  Needs no
 * device and no binding: every tensor is taken to be 16-byte aligned.
 *   segments  host [segments_cap][MGWFBP_LAYOUT_SEGMENT_COLS] out or NULL: layer, elements, offset in the plan-wide
 *             merged order (elements), group -- in communication order
 *   tiles     host [tiles_cap][MGWFBP_LAYOUT_TILE_COLS] out or NULL: first segment, segment count, start, elements,
 *             list, tile length, padding.
 *             segment count 1: `start` is the element offset inside that segment; more than
 *             one: the tile gathers whole short segments and `start` is its offset in the
 *             plan-wide merged order.
 *             list 0: the per-group lists (group after group); list 1: the second copy used
 *             by whole-plan launches; list 2 or 3 (when built): the whole plan in longer
 *             tiles (MGWFBP_OPT_LONG_TILES), 2 if the fused reduce pass uses it by default,
 *             3 if only mgwfbp_tune may select it; list 4: the whole plan group after group in
 *             communication order (mgwfbp_gated_launch), in tiles of 1024 or (long plans) 4096
 *             elements whatever tile_elems is, groups of up to 64 Ki elements in tiles of 512.
 *             tile length: elements of a full tile in that list (a group launched alone is
 *             cut into shorter tiles than the whole plan when it would otherwise give too
 *             few workgroups).
 *             padding: padding elements of the merged order that follow the tile and belong
 *             to it (MGWFBP_OPT_PAD_ELEMS; a gather tile's `elements` already include the
 *             padding between and after its layers).
 *   n_segments, n_tiles   out or NULL: the counts (call with NULL arrays to size them)
 */
enum { MGWFBP_LAYOUT_SEGMENT_COLS = 4, MGWFBP_LAYOUT_TILE_COLS = 7 }; /* row widths of the two arrays */
int mgwfbp_plan_layout(const mgwfbp_plan_t *plan, uint64_t *n_segments, uint64_t *segments,
                       size_t segments_cap, uint64_t *n_tiles, uint64_t *tiles, size_t tiles_cap);

/*
 * Attach the per-layer tensors Algorithm 2 works on -- every worker's gradients (the layers it
 * pushes into the queue), the averaged gradient and the weights of its update line, plus the
 * momentum buffers -- and upload the segment, tile and pointer tables (once; the pointers are
 * not re-read from host memory afterwards).  A second call replaces the binding.
 *   grads  host array [N*L] of device pointers, worker-major: grads[g*L + l] is worker g's
 *          gradient of layer l, p_elems[l] floats, 4-byte aligned (16-byte alignment of
 *          every pointer of a layer enables 128-bit accesses for that layer)
 *   out    host array [L] of device pointers receiving the averaged gradients, or NULL.
 *          out[l] may be the same pointer as grads[0*L + l] (in place); any other overlap
 *          between buffers is undefined.
 *   w, v   host arrays [L] of device pointers (weights, momentum buffers), both or neither.
 * The current HIP device at the time of the call owns the tables.
 */
int mgwfbp_bind(mgwfbp_plan_t *plan, const float *const *grads, float *const *out,
                float *const *w, float *const *v);

/*
 * Optional, after mgwfbp_bind: time the whole-plan fused reduce pass (mgwfbp_pack_reduce_unpack
 * with group = -1 and no workspace) under a handful of launch shapes -- tile list, pause
 * between loads, workgroups per compute unit -- on the bound tensors, and keep the fastest for
 * later whole-plan launches of this plan (also for mgwfbp_pack_reduce).  How well a launch
 * fills the chip depends on its size in ways the built-in rules only approximate; the result
 * is the same whatever shape is chosen.  Runs the pass up to about 500 times on `hip_stream`
 * (fewer when a launch is long: about 2 ms of launches per candidate, 4 to 32 of them) and
 * waits for it; out[] ends up holding the reduced gradients.  out[] must be bound and must not alias
 * a gradient tensor (the pass is repeated).  A new mgwfbp_bind discards the choice.
 *   chosen      out or NULL: index of the winning candidate (0 = the built-in rules)
 *   chosen_ms   out or NULL: its time per launch in milliseconds
 */
int mgwfbp_tune(mgwfbp_plan_t *plan, void *hip_stream, int32_t *chosen, double *chosen_ms);

/*
 * Workspace size in bytes for the materialised path on `group` (-1 = all groups at once):
 * N packed replica buffers followed by one reduced buffer, each rounded up to 256 bytes.
 */
int mgwfbp_workspace_bytes(const mgwfbp_plan_t *plan, int32_t group, size_t *bytes);

/*
 * What Algorithm 2's communication thread does with one merged group: the layer buffer `lb` of
 * the group's gradients, the all-reduce of it -- whose arithmetic is Eq. 2's average over the N
 * workers -- and the averaged gradients back in per-layer form.
 * Pack + N-way reduce + unpack of one group (or all groups when group = -1) into out[].
 *   workspace == NULL : one fused pass that never materialises the merged buffers.
 *   workspace != NULL : device pointer, 256-byte aligned, at least mgwfbp_workspace_bytes;
 *                       runs pack, reduce and unpack as three kernels through it.
 *   hip_stream        : a hipStream_t (NULL = the default stream).
 * Requires out[] to be bound.
 */
int mgwfbp_pack_reduce_unpack(mgwfbp_plan_t *plan, int32_t group, void *workspace,
                              size_t workspace_bytes, void *hip_stream);

/*
 * Same reduction fused with Algorithm 2's update line W = W - eta * grad (Eq. 1 with the
 * averaged gradient of Eq. 2), extended by a momentum buffer: v = momentum*v + avg;
 * w = w - lr*v on the bound w[], v[]; momentum = 0 is the paper's update exactly.  The averaged
 * gradient is also written to out[] when out[] is bound.
 */
int mgwfbp_step(mgwfbp_plan_t *plan, int32_t group, float lr, float momentum, void *workspace,
                size_t workspace_bytes, void *hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): mgwfbp_pack_reduce_unpack through pack, reduce and
 * unpack kernels with the workspace in a device array that is part of the library's own code
 * object, MGWFBP_STATIC_WORKSPACE_BYTES long.  The call allocates nothing and frees nothing,
 * on the host's heap or on the device, and makes no runtime query on a device the plan was
 * bound on (mgwfbp_bind looks the array's address up; on any other device the first call does).
 *   group        as for mgwfbp_pack_reduce_unpack (-1 = all groups at once)
 *   hip_stream   a hipStream_t (NULL = the default stream)
 * Results are those of mgwfbp_pack_reduce_unpack with a workspace, bit for bit.
 * MGWFBP_EINVAL when mgwfbp_workspace_bytes(plan, group) exceeds the array; the other errors of
 * mgwfbp_pack_reduce_unpack apply.  Every device the library runs on holds one copy of the
 * array until the process ends, and all calls on a device share it: calls that overlap in time
 * on one device (two streams, two threads, two plans) race on it; calls on one stream are safe.
 * Nothing in it needs clearing between calls: every element that is read is written earlier by
 * the same call.
 */
#define MGWFBP_STATIC_WORKSPACE_BYTES (64u * 1024u * 1024u)
int mgwfbp_pack_reduce_unpack_static(mgwfbp_plan_t *plan, int32_t group, void *hip_stream);

/* The three materialised steps on their own (workspace layout as above, required). */
int mgwfbp_pack(mgwfbp_plan_t *plan, int32_t group, void *workspace, size_t workspace_bytes,
                void *hip_stream);
int mgwfbp_reduce(mgwfbp_plan_t *plan, int32_t group, void *workspace, size_t workspace_bytes,
                  void *hip_stream);
int mgwfbp_unpack(mgwfbp_plan_t *plan, int32_t group, void *workspace, size_t workspace_bytes,
                  void *hip_stream);

/*
 * The two halves of the path as a real transport would call them (Algorithm 2 with the
 * all-reduce in between): N + 1 and 2 (5 with the update) units of traffic instead of the
 * 3N + 3 of the three materialised steps.
 *   mgwfbp_pack_reduce    reads the N workers' layers of the group and writes the group's
 *                         merged buffer already reduced: merged[j] = (1/N) sum_g x_g[j], packed
 *                         in arrival order without padding (this GPU's share of the all-reduce
 *                         arithmetic applied to the layer buffer).
 *   mgwfbp_unpack_update  scatters a merged buffer back to out[] (update = 0) or applies
 *                         v = momentum*v + merged; w = w - lr*v on w[], v[] and also writes
 *                         out[] when bound (update != 0).
 *   merged  device pointer, 256-byte aligned, at least 4 * (elements of the group, or of the
 *           whole plan for group = -1) bytes.
 */
int mgwfbp_pack_reduce(mgwfbp_plan_t *plan, int32_t group, void *merged, size_t merged_bytes,
                       void *hip_stream);
int mgwfbp_unpack_update(mgwfbp_plan_t *plan, int32_t group, const void *merged,
                         size_t merged_bytes, int32_t update, float lr, float momentum,
                         void *hip_stream);

/*
 * Fit the all-reduce cost model T_ar(M) = a + b*M (Eq. 9) to measured (message size, time)
 * pairs by ordinary least squares, the way Section V-A obtains a and b from benchmarks.
 *   n            number of measurements (>= 2, with at least two distinct sizes)
 *   bytes, ms    host [n]
 *   a_ms, b_ms_per_byte   out.  The fitted intercept is clamped at 0 (a negative start-up time
 *                has no meaning in the model); the slope is then refitted through the origin.
 */
int mgwfbp_fit_cost(int32_t n, const double *bytes, const double *ms, double *a_ms,
                    double *b_ms_per_byte);

/*
 * (a, b) of Table II for an all-reduce algorithm on N workers:
 *   algorithm  0 binary tree, 1 recursive doubling, 2 recursive halving and doubling, 3 ring
 *   alpha_ms, beta_ms_per_byte, gamma_ms_per_byte   latency, per-byte transfer, per-byte sum
 */
int mgwfbp_table2_cost(int32_t algorithm, int32_t N, double alpha_ms, double beta_ms_per_byte,
                       double gamma_ms_per_byte, double *a_ms, double *b_ms_per_byte);

/*
 * Predicted weak-scaling curve (the trace-based simulation of Section V-C): for each worker
 * count the all-reduce cost (a, b) follows Table II, the layers are planned in `mode`, and the
 * iteration time follows Eq. 8.  Speedup over one worker is Eq. 4: N * (t_f + t_b) / t_iter.
 *   tb_ms, tf_ms   the per-layer backward trace and forward time of ONE worker (host [L])
 *   algorithm      Table II row, as for mgwfbp_table2_cost
 *   n_workers      host [n_points] worker counts (each >= 1)
 *   t_iter_ms, speedup   host [n_points] out, either may be NULL
 */
int mgwfbp_scaling_curve(int32_t L, const uint64_t *p_elems, const double *tb_ms, double tf_ms,
                         int32_t algorithm, double alpha_ms, double beta_ms_per_byte,
                         double gamma_ms_per_byte, int32_t n_points, const int32_t *n_workers,
                         int32_t mode, double *t_iter_ms, double *speedup);

/*
 * One iteration of Algorithm 2 (MG-WFBP S-SGD) on two HIP streams, driven by events.
 *
 * The computation thread of Algorithm 2 is played by `compute_stream`: a stand-in backward
 * pass from layer L-1 down to layer 0, one kernel per group that occupies one wave until the
 * backward pass has reached the end of the group's lowest layer (an absolute deadline: the sum
 * of tb_ms so far after time zero, read from the device clock) and touches no gradient memory
 * (only the moment a group's lowest layer is done matters to the communication side).  The
 * communication thread is played by `comm_stream`: the reduction of group k
 * (mgwfbp_pack_reduce_unpack or, with update != 0, mgwfbp_step, fused form) is enqueued behind an event recorded when the group's lowest
 * layer has finished its backward kernel, which is the start rule of Eq. 7 / Condition 2;
 * groups follow each other in communication order.  The call blocks until both streams are
 * idle and reports the measured timeline, in milliseconds from the start of the backward pass:
 *   tb_ms           host [L] or NULL (NULL = the backward times the plan was made with)
 *   group_ready_ms  host [n_groups] out or NULL: when the backward pass of group k's lowest
 *                   layer ended (mu_b of that layer)
 *   group_start_ms  host [n_groups] out or NULL: when group k's kernel could start (tau_c)
 *   group_finish_ms host [n_groups] out or NULL
 *   t_iter_ms       out or NULL: end of the last group
 * Per-group timestamps cost a timed event record each (a few microseconds of stream time);
 * pass NULL for the three arrays to run the schedule with only the events it needs.
 * Streams: hipStream_t handles at default priority; NULL = the default stream (using one
 * stream for both serialises everything).  Creates and destroys HIP events internally.
 * Time zero and the end of the last group are device-clock values kept in two words owned by
 * the plan: two calls on the same plan must not run at the same time.
 */
int mgwfbp_run_iteration(mgwfbp_plan_t *plan, const double *tb_ms, int32_t update, float lr,
                         float momentum, void *compute_stream, void *comm_stream,
                         double *group_ready_ms, double *group_start_ms,
                         double *group_finish_ms, double *t_iter_ms);

/*
 * mgwfbp_run_iteration with several communication streams: group k is enqueued on
 * comm_streams[k mod n_comm_streams], so consecutive groups may overlap (one group's ramp-up
 * hides the previous group's drain; they touch disjoint tensors).  Each group still waits for
 * its own gradients (Condition 2); what is given up is the serial channel of Eq. 7, which is a
 * property of a network, not of one GPU's memory.  n_comm_streams = 1 is mgwfbp_run_iteration.
 *   comm_streams    host array [n_comm_streams] of different hipStream_t handles, 1 .. 8 of
 *                   them, default priority.  Results do not depend on their number.
 * With more than one stream group_start_ms[k] >= group_finish_ms[k-1] no longer holds;
 * t_iter_ms is the end of the last group to finish.
 */
int mgwfbp_run_iteration_streams(mgwfbp_plan_t *plan, const double *tb_ms, int32_t update, float lr,
                                 float momentum, void *compute_stream, void *const *comm_streams,
                                 int32_t n_comm_streams, double *group_ready_ms,
                                 double *group_start_ms, double *group_finish_ms, double *t_iter_ms);

/*
 * Algorithm 2's communication thread as ONE launch.  A kernel launch per group costs a few
 * microseconds however little the group holds, which is the start-up term a of this
 * "transport"; here the whole plan is a single launch whose workgroups take the tiles in
 * arrival order (group 0 first) and, before each tile, wait until the tile's group has arrived:
 * the plan keeps one arrival counter per group in device memory, and a tile runs once its
 * group's counter has reached the `arrival` number of the launch (counters only grow; use 1, 2,
 * 3, ... for successive iterations; they start at 0 after mgwfbp_bind).
 *   mgwfbp_gated_launch   enqueues the launch on `hip_stream` (reduction into out[], or with
 *                         update != 0 the update of w[], v[]; fused form, results as
 *                         mgwfbp_pack_reduce_unpack / mgwfbp_step with group = -1).  It starts
 *                         at once and waits on the device.  Every wait is bounded: a workgroup
 *                         that has waited about give_up_ms (0 < give_up_ms <= 60000; counted in
 *                         looks at the counter, each a microsecond or more) for a group sets a
 *                         give-up word and ends, the others end at their next look at it, so the
 *                         launch always drains; tiles not yet run are then left undone.
 *   mgwfbp_gated_signal   enqueues, behind the work already in `hip_stream`, a small kernel that
 *                         stores `arrival` to the group's counter: call it on the stream that
 *                         produces the group's gradients, after the kernel that writes the lowest
 *                         layer (the end of that kernel is what makes the gradients visible to the
 *                         launch, which reads them past its own caches).  That stream must not be
 *                         the one the launch is on, nor wait for it.
 *   mgwfbp_gated_gave_up  after the launch's stream has been waited for: *gave_up = 1 if the
 *                         last launch gave up.
 *   mgwfbp_gated_workgroups  how many workgroups the launch would use now, and how many of them a
 *                         compute unit holds at most (either pointer may be NULL; 0 workgroups:
 *                         the device holds too few of them).
 * By default the launch holds four workgroups per compute unit fewer than the unit can take of
 * this kernel (16; 14 with update != 0), another number with MGWFBP_OPT_GATED_WGS_PER_CU (never
 * less than two free), so that the kernels that produce gradients and bump counters find room
 * on the chip while it waits; each workgroup walks its share of the tiles.  The default leaves
 * room for kernels with workgroups of 256 lanes and moderate register use.  A kernel that needs
 * whole SIMDs (a matrix-core GEMM using every register) is not placed while the launch has
 * workgroups on every compute unit, and a host call that synchronises the device blocks behind
 * it: the launch then gives up after give_up_ms.  One gated launch per plan at a time.
 *
 * For a backward pass made of such kernels the launch can be confined to part of the chip:
 *   mgwfbp_confined_stream_create   a stream (default priority) whose kernels run on the first
 *                         n_compute_units of the current device only (a multiple of 32 below the
 *                         device's count; the runtime's compute-unit mask).  Every such stream
 *                         takes a hardware queue of its own: make one, not many.
 *   mgwfbp_confined_stream_destroy  releases it (the caller has waited for its work).
 * With MGWFBP_OPT_GATED_CUS set to the same number before mgwfbp_bind, mgwfbp_gated_launch on that
 * stream sizes its grid for those units and leaves the others untouched: kernels that need whole
 * SIMDs then run beside it, on the rest of the chip, and the launch streams at the rate its
 * units reach (half of an MI355X: about 0.65 of the whole chip's).
 *
 * The signalling kernels must be able to run WHILE the launch is running.  The runtime serves its
 * streams from a few hardware queues (four by default), and two streams that share a queue run
 * their kernels one after the other: the signals would then sit behind the launch that waits for
 * them, and the launch would give up.
 *   mgwfbp_streams_side_by_side  *side_by_side = 1 if a kernel on stream_a runs while a kernel on
 *                         stream_b is still running, 0 if not (also for stream_a == stream_b).  It
 *                         finds out with a handshake of two tiny kernels (the waiting one ends by
 *                         itself after 2 ms), blocks until both streams are idle, and remembers in
 *                         the plan the pairs that passed (until mgwfbp_bind is called again; a
 *                         stream that is destroyed and created anew has to be checked anew).  The
 *                         plan must be bound.  Take another stream when a pair fails: most pairs
 *                         pass.
 *
 * mgwfbp_run_iteration_gated is mgwfbp_run_iteration in this form: the stand-in backward pass on
 * `compute_stream` signals each group's arrival, `comm_stream` (a different stream) holds the one
 * launch.  It first checks the pair as mgwfbp_streams_side_by_side(compute, comm) does and returns
 * MGWFBP_ESTATE, with nothing run, if the pair fails.  It blocks until both streams are idle,
 * reports the time from the start of the backward pass to the end of the launch, and returns
 * MGWFBP_ESTATE if the launch gave up.  Like several communication streams, this form does not
 * serialise the groups (Eq. 7's channel); it keeps Condition 2.
 */
int mgwfbp_gated_launch(mgwfbp_plan_t *plan, int32_t update, float lr, float momentum, uint32_t arrival,
                        double give_up_ms, void *hip_stream);
int mgwfbp_gated_signal(mgwfbp_plan_t *plan, int32_t group, uint32_t arrival, void *hip_stream);
int mgwfbp_gated_gave_up(mgwfbp_plan_t *plan, int32_t *gave_up);
int mgwfbp_gated_workgroups(mgwfbp_plan_t *plan, int32_t update, uint32_t *workgroups, uint32_t *per_compute_unit);
int mgwfbp_confined_stream_create(uint32_t n_compute_units, void **hip_stream);
int mgwfbp_confined_stream_destroy(void *hip_stream);
int mgwfbp_streams_side_by_side(mgwfbp_plan_t *plan, void *stream_a, void *stream_b, int32_t *side_by_side);
int mgwfbp_run_iteration_gated(mgwfbp_plan_t *plan, const double *tb_ms, int32_t update, float lr,
                               float momentum, void *compute_stream, void *comm_stream,
                               double give_up_ms, double *t_iter_ms);

/*
 * The same iteration captured once into a HIP graph and replayed: one graph launch per
 * iteration instead of several runtime calls per group, for loops in which the schedule
 * (plan, backward times, update parameters, bound tensors) does not change.
 *   mgwfbp_iteration_capture  records the stand-ins, the per-group dependencies and the group
 *       launches of mgwfbp_run_iteration from two different non-default streams (used only
 *       to express the fork and join; nothing runs during capture).  lr and momentum are
 *       frozen into the graph.  The tensors bound to the plan are referenced, not copied:
 *       replays see their current contents.
 *   mgwfbp_iteration_replay   launches the graph on `hip_stream`.  t_iter_ms == NULL: returns
 *       at once (asynchronous).  Otherwise waits for the stream and reports the time from the
 *       start of the backward pass to the end of the last group, read from the device clock.
 *   mgwfbp_iteration_destroy  frees the graph.  After a new mgwfbp_bind, or once the plan has
 *       been destroyed, the graph is stale: replay then returns MGWFBP_ESTATE (the handle itself
 *       stays valid until it is destroyed).  Replays of one plan must not overlap.
 */
typedef struct mgwfbp_iteration_s mgwfbp_iteration_t; /* opaque */
int mgwfbp_iteration_capture(mgwfbp_plan_t *plan, const double *tb_ms, int32_t update, float lr,
                             float momentum, void *compute_stream, void *comm_stream,
                             mgwfbp_iteration_t **out);
int mgwfbp_iteration_replay(mgwfbp_iteration_t *iteration, void *hip_stream, double *t_iter_ms);
void mgwfbp_iteration_destroy(mgwfbp_iteration_t *iteration);

void mgwfbp_plan_destroy(mgwfbp_plan_t *plan);

const char *mgwfbp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MGWFBP_H */
