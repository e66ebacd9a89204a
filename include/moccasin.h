/*
 * moccasin.h -- C ABI of libmoccasin_hip.so: batched evaluation of candidate
 * assignments to the retention-interval model of Moccasin (arXiv 2304.14463)
 * on one AMD MI355X (gfx950).
 *
 * Model (paper, Section 2 and Section 2.1).  A compute DAG G = (V, E) has n
 * nodes; node v has a duration w_v and an output size m_v; the memory budget
 * is M.  Every node may be computed up to C times; copy i of node v is a
 * retention interval with variables a (active flag), s (start = the event at
 * which v is computed) and e (end = last event at which its output is kept).
 * A candidate is one assignment to all n*C copies.
 *
 * Conventions of this library
 *   - copy index k = v*C + i (the copies of a node are adjacent), T = n*C;
 *   - positions are 0-based: the paper's event t in D = {1..sum C_v} (the
 *     display after Eq. (8)) is position t-1 in [0, T);
 *   - a batch of B candidates is three row-major [B][T] arrays: int32 starts,
 *     int32 ends, uint8 active (non-zero = active);
 *   - a copy is "live" iff it is active and 0 <= s <= e <= T-1.  An inactive
 *     copy is ignored by every constraint (Section 2.1, first paragraph).  An
 *     active copy that is not live is counted once as a violation of
 *     Eq. (2)/(8), is ignored by Eq. (3)-(6), and still counts in Eq. (1).
 *
 * What is computed per candidate (moc_result)
 *   duration   = sum over active copies of w_v                       Eq. (1)
 *   peak       = max over positions t of the summed m_v of the live
 *                copies with s <= t <= e (closed intervals)           Eq. (4)
 *   violations = number of violated constraint instances:
 *                  active copies that are not live                    Eq. (2), (8)
 *                + nodes whose copy 0 is inactive                     Eq. (7)
 *                + live copies that end after the next live copy of
 *                  the same node starts                               Eq. (3)
 *                + sum over positions of (live starts there - 1)+     Eq. (6)
 *                + pairs (edge (u,v), live copy i of v) for which no
 *                  live copy j of u has s_u^j + 1 <= s_v^i <= e_u^j   Eq. (5)
 *   feasible   = (violations == 0 && peak <= M)
 * The budget never adds to `violations`; its slack is peak - M.
 *
 * Memory and ownership.  Graph arrays are HOST pointers, read during
 * moc_graph_upload only.  Candidate and result arrays are DEVICE pointers
 * owned by the caller and must stay valid until the work queued on the stream
 * has finished.  Evaluation calls allocate nothing and are asynchronous on
 * the given HIP stream.  The device that was current at upload must be
 * current at every later call with that graph.
 *
 * Concurrency.  A graph handle may be used from several host threads and
 * streams at once.  The handle owns 16 sets of device-side work counters for
 * moc_eval_batch; a set belongs to a stream (launches on one stream follow
 * each other and share it), every launch leaves its set at zero.  The first 16
 * distinct streams used with a handle get a set each; launches on any further
 * stream are split statically over the workgroups instead, which touches no
 * counters and gives the same results, up to a third slower on small graphs.
 * A launch that is aborted (device reset) leaves the handle unusable: free it
 * and upload the graph again.
 *
 * Errors.  Every function that returns int returns MOC_OK (0) or a negative
 * code.  Arguments are checked before anything is queued: with MOC_EINVAL,
 * MOC_EDEVICE or MOC_EOVERFLOW nothing has been queued on the stream.  MOC_EHIP
 * reports a failed HIP runtime call; from the calls that queue several kernels
 * (moc_search_cuts, moc_search_moves) the kernels queued before the failing
 * one still run.  Contents of a candidate are never an error: bad values are
 * violations.
 */
#ifndef MOCCASIN_H
#define MOCCASIN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOC_OK          0
#define MOC_EINVAL    (-1)  /* bad argument: null pointer, size out of range, index out of range, misaligned */
#define MOC_EOVERFLOW (-2)  /* C * sum(size) or C * sum(dur) >= 2^31, or T too large for the LDS layout */
#define MOC_ENOMEM    (-3)  /* host or device allocation failed */
#define MOC_EHIP      (-4)  /* a HIP runtime call failed; see moc_last_hip_error() */
#define MOC_EDEVICE   (-5)  /* the graph's device is not the current device */

/* Largest T = n*C an uploaded graph may have: the per-candidate working set
 * (memory-delta array, one record of packed intervals per node, start bitmap)
 * lives in the 160 KB LDS of one compute unit.  The bound is reached with
 * C = 1; with more copies per node the records take more room (about 16200
 * for C = 3, 14900 for C = 4).  moc_graph_upload returns MOC_EOVERFLOW for a
 * graph that does not fit. */
#define MOC_MAX_T 19455

typedef struct moc_graph moc_graph; /* opaque; owns device copies of the graph */

typedef struct {
  int64_t peak;       /* Eq. (4) left-hand side, maximised over positions */
  int64_t duration;   /* Eq. (1) */
  int32_t violations; /* violated instances of Eq. (2),(3),(5),(6),(7),(8) */
  int32_t feasible;   /* 1 iff violations == 0 and peak <= M */
} moc_result;         /* 24 bytes */

typedef struct {
  int32_t violations; /* -1 if the move is not applicable */
  int32_t peak;       /* -1 if the move is not applicable */
} moc_move_score;

typedef struct {
  int32_t violations; /* as moc_result.violations */
  int32_t peak;       /* as moc_result.peak (below 2^31 for any uploaded graph) */
  int64_t duration;   /* as moc_result.duration: the base's, minus or plus w_v */
} moc_toggle_score;   /* 16 bytes */

typedef moc_toggle_score moc_cut_score; /* violations = peak = -1, duration = 0: not applicable */

typedef struct {
  int32_t status;     /* 1 a valid sequence, 0 decoded but not valid, -1 not decodable */
  int32_t length;     /* number of steps = active copies; 0 when status == -1 */
  int64_t peak;       /* the sequence's own peak footprint; 0 unless status == 1 */
  int64_t duration;   /* summed duration of its steps; 0 unless status == 1 */
} moc_decode_result;  /* 24 bytes */

typedef struct {
  int32_t move;       /* index of the best move, -1 if no move is applicable */
  int32_t violations; /* 0 when move == -1 */
  int64_t peak;       /* 0 when move == -1 */
} moc_best_move;

/*
 * Upload a problem instance (Section 1, problem statement; Section 2.1: w_v and
 * m_v are known).
 *   n        number of nodes, >= 1
 *   in_ptr   host, [n+1], CSR offsets by in-edges: the predecessors u of v
 *            (edges (u,v) in E) are in_idx[in_ptr[v] .. in_ptr[v+1]); in_ptr[0] = 0,
 *            non-decreasing
 *   in_idx   host, [m = in_ptr[n]], each in [0, n)
 *   size     host, [n], m_v >= 0
 *   dur      host, [n], w_v >= 0
 *   budget   M
 *   C        copies per node (the paper's C_v, uniform), >= 1
 *   out      receives the handle; release with moc_graph_free
 * Acyclicity is not required and not checked (evaluation is defined on any
 * digraph).  Duplicate in-edges are kept and counted as separate instances.
 * Errors: MOC_EINVAL, MOC_EOVERFLOW (sums, or n*C > MOC_MAX_T), MOC_ENOMEM, MOC_EHIP.
 */
int moc_graph_upload(int32_t n, const int32_t* in_ptr, const int32_t* in_idx, const int32_t* size,
                     const int32_t* dur, int64_t budget, int32_t C, moc_graph** out);

/* Sizes of an uploaded graph; any output pointer may be NULL. */
int moc_graph_info(const moc_graph* g, int32_t* n, int32_t* m, int32_t* C, int32_t* T);

/*
 * Evaluate B candidates (Eq. (1)-(8) as listed above).
 *   starts, ends   device, int32 [B][T]
 *   active         device, uint8 [B][T]
 *   out            device, moc_result [B], 8-byte aligned
 *   hip_stream     a hipStream_t (NULL = the default stream)
 * starts/ends must be 4-byte aligned.  The C copies of a node are read as one
 * vector when the arrays allow it (C = 2: starts/ends 8-byte and active 2-byte
 * aligned; C = 4: 16-byte and 4-byte), otherwise element by element (slower,
 * same results).  B == 0 is a no-op.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EHIP.
 */
int moc_eval_batch(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                   const uint8_t* active, moc_result* out, void* hip_stream);

/*
 * moc_eval_batch for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same results, same kernels; the work counters of the launch are
 * not the handle's (device memory allocated at upload) but one fixed set of
 * 4160 bytes inside the library's device image, which each GPU the library
 * runs on holds until the process ends.  The call queues a kernel that clears
 * them, then the evaluation; it calls no hipMalloc, hipFree or other
 * allocating routine (what the kernels need to know of the device was asked
 * for when the graph was uploaded).
 *   B   at most MOC_NOALLOC_MAX_B (one launch: the counters count candidates
 *       in 32 bits); MOC_EOVERFLOW beyond that.  Longer batches: several calls
 *       on one stream.
 * All calls on a GPU share that one set of counters, whatever graph handle
 * and stream they use: two such calls whose kernels overlap on one GPU race
 * (candidates skipped or evaluated twice, result rows left unwritten).  Issue
 * them on one stream, or order them with events.  They do not interfere with
 * moc_eval_batch.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW, MOC_EHIP.
 */
#define MOC_NOALLOC_MAX_B 2147483648ll /* 2^31 */
int moc_eval_batch_noalloc(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                           const uint8_t* active, moc_result* out, void* hip_stream);

/*
 * Give an uploaded graph the topological order that the stage-restricted
 * domain of Section 2.3 is built on.
 *   order   host, [n]: order[j] = the node with place j; a permutation of the
 *           nodes in which every edge (u, v) has u before v
 * May be called again with another order (synchronises the device first); not
 * while another thread evaluates with this handle.
 * Errors: MOC_EINVAL (not a permutation, or not topological), MOC_EDEVICE,
 * MOC_ENOMEM, MOC_EHIP.
 */
int moc_graph_set_order(moc_graph* g, const int32_t* order);

/*
 * Evaluate B candidates in the stage-restricted domain (Section 2.3,
 * "Complexity Reduction by Enforcing an Initial Topological Ordering").
 * Positions are 0-based in [0, n(n+1)/2): stage j = 0..n-1 holds the j + 1
 * positions j(j+1)/2 .. j(j+1)/2 + j (the paper's events, shifted by one).  A
 * node with place k in the order of moc_graph_set_order may be computed only
 * at slot k of a stage, i.e. at a position j(j+1)/2 + k with j >= k, and its
 * first copy only at slot k of stage k (the paper's fixed s_v^1 = k'(k'+1)/2
 * for the k'-th node, 1-based).  An active copy whose start is not such a
 * position is outside its domain: like a position outside [0, T) in
 * moc_eval_batch it counts as one violation of Eq. (8), is used by no other
 * constraint and still counts in Eq. (1).  Ends may be any position of the
 * domain.  Everything else, and the result, is as for moc_eval_batch with
 * n(n+1)/2 positions in place of T; Eq. (6) is kept as it is there (here only
 * copies of one node can share an event).
 *   starts, ends   device, int32 [B][T] (T = n*C values per candidate)
 *   active         device, uint8 [B][T]
 *   out            device, moc_result [B], 8-byte aligned
 * This call keeps 3.5 words per copy and one per node in LDS: T <= about
 * 10000.  B == 0 is a no-op.
 * Errors: MOC_EINVAL (also: no order set), MOC_EDEVICE, MOC_EOVERFLOW (T too
 * large for this call), MOC_EHIP.
 */
int moc_eval_batch_staged(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                          const uint8_t* active, moc_result* out, void* hip_stream);

/*
 * Score every single-field move of B base candidates.  Not part of the paper:
 * it is the neighbourhood a local search over the variables of Section 2.1
 * would scan.  Move index q = ((k*2 + field)*2R + d): copy k, field 0 = start,
 * 1 = end, displacement delta = d-R for d < R and d-R+1 otherwise (delta runs
 * over -R..-1, +1..+R).  A move is not applicable when copy k is inactive or
 * the moved field would leave [0, T): its score is (-1, -1).  Otherwise its
 * score is the (violations, peak) that moc_eval_batch returns for the
 * candidate with that one field changed; the duration does not change.
 *   R           radius, 1 <= R <= 32
 *   out_moves   device, moc_move_score [B][T*4R], or NULL
 *   out_best    device, moc_best_move [B], or NULL: the applicable move that
 *               minimises (violations, max(peak, M), peak, q) lexicographically
 *               (max(peak, M) is the Phase-1 objective of Section 2.4)
 * At least one of out_moves / out_best must be given; both 8-byte aligned.
 * This call keeps 4.6 words per copy in LDS: T <= about 8800.  A graph with an
 * edge (v,v) is not accepted.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW (T too large for this call), MOC_EHIP.
 */
int moc_eval_neighbours(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                        const uint8_t* active, int32_t R, moc_move_score* out_moves,
                        moc_best_move* out_best, void* hip_stream);

/*
 * Score every candidate that differs from a base in one active flag.  Not part
 * of the paper: these are the moves of a local search over the variables of
 * Section 2.1 that change the objective, Eq. (1) -- dropping a copy saves its
 * node's duration, activating a spare copy (at the start and end it already
 * carries) costs it.  Entry [b][k] is what moc_eval_batch returns for base b
 * with active[k] flipped and everything else unchanged.
 *   out   device, moc_toggle_score [B][T], 8-byte aligned
 * This call keeps 4.7 words per copy in LDS: T <= about 8800.  A graph with an
 * edge (v,v) is not accepted.  B == 0 is a no-op.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW (T too large for this call), MOC_EHIP.
 */
int moc_eval_toggles(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                     const uint8_t* active, moc_toggle_score* out, void* hip_stream);

/*
 * Score every cut-and-recompute move of B base candidates: keep a producer's
 * output only as long as its earlier uses need it and compute it again just
 * before a later use.  Not part of the paper as a procedure; it is the edit
 * that trades duration, Eq. (1), for memory, Eq. (4), within the variables of
 * Section 2.1.  Move index q = x*C + i: in-edge x = (u, v) in the order of
 * in_idx, copy i of the consumer v.  With t the start of that copy (which must
 * be live):
 *   k   the live copy of u with s_k < t <= e_k that starts last (the lowest
 *       index among equal starts),
 *   j   the lowest copy of u that is not active,
 *   p   the last position in (s_k, t) at which no live copy starts and every
 *       predecessor w of u has a live copy with s_w < p <= e_w (so that the
 *       new computation finds its inputs, Eq. (5)),
 *   e'  the last start in (s_k, p) of a live copy of any consumer of u, s_k if
 *       there is none;
 * the move sets copy k to [s_k, e'] and copy j to active, [p, e_k].  It is not
 * applicable (score -1, -1, 0) if the consumer copy is not live or k, j or p
 * does not exist.  Otherwise entry [b][q] is what moc_eval_batch returns for
 * the edited candidate (the duration is the base's plus w_u).
 *   out_moves   device, moc_cut_score [B][m*C], or NULL
 *   out_best    device, moc_best_move [B], or NULL: the applicable move that
 *               minimises (violations, peak, n_at, q) lexicographically, n_at
 *               being the number of positions at which the edited candidate's
 *               memory still reaches the base's peak (0 when the peak falls):
 *               among moves that leave the peak where it is, the one that
 *               clears most of the positions that attain it; move = -1 and
 *               zeros if none is applicable (always so when m == 0)
 * At least one of out_moves / out_best must be given; both 8-byte aligned.
 * LDS use and limits as moc_eval_toggles.  A graph with an edge (v,v) is not
 * accepted.  B == 0 is a no-op.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW (T too large for this call), MOC_EHIP.
 */
int moc_eval_cuts(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                  const uint8_t* active, moc_cut_score* out_moves, moc_best_move* out_best,
                  void* hip_stream);

/*
 * moc_eval_cuts with the other rule for where the recomputation goes: instead
 * of waiting at a position where every input of the producer u is still held,
 *   p   is the last position in (s_k, t) at which no live copy starts and every
 *       predecessor w of u either is held (a live copy with s_w < p <= e_w) or
 *       has a live copy that ends before p;
 * and for every predecessor that is not held at p, its live copy with the
 * largest end below p (the highest index among equals) is kept until p (its
 * end becomes p): small inputs are carried across the stretch on which the
 * large output is dropped.  k, j, e' and the edit of u's copies are as for
 * moc_eval_cuts, and so are the move index, the outputs, the order of the best
 * move, the limits and the errors.  Where all inputs are held at the last free
 * position the two calls describe the same move.
 */
int moc_eval_cuts_keep(const moc_graph* g, int64_t B, const int32_t* starts, const int32_t* ends,
                       const uint8_t* active, moc_cut_score* out_moves, moc_best_move* out_best,
                       void* hip_stream);

/*
 * Greedy descent by cut-and-recompute moves, every candidate on its own: the
 * memory-reducing half of a local search in the spirit of Phase 1 of
 * Section 2.4, which minimises max(peak, M).  Repeats max_steps times: find the
 * best move as moc_eval_cuts does; apply it in place if it lowers
 * (violations, max(peak, M)) lexicographically against the candidate as it
 * stands or, with both unchanged and the peak above M, leaves fewer positions
 * at the peak.  A candidate whose best move does neither stays as it is from
 * then on.
 *   starts, ends, active   device, [B][T], edited in place
 *   max_steps              >= 0
 *   work_best              device, moc_best_move [B], 8-byte aligned: workspace
 *                          (holds the last step's choice on return)
 *   out_steps              device, int32 [B]: number of moves applied
 * Queues 2 * max_steps + 1 kernels on the stream and returns; allocates
 * nothing.  Limits as moc_eval_cuts; B <= 2^31 - 1.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW, MOC_EHIP.
 */
int moc_search_cuts(const moc_graph* g, int64_t B, int32_t* starts, int32_t* ends, uint8_t* active,
                    int32_t max_steps, moc_best_move* work_best, int32_t* out_steps, void* hip_stream);

/*
 * Local search in the two phases of Section 2.4, every candidate on its own.
 * Phase 1 (towards the budget; the paper's Phase 1 minimises max(peak, M)):
 * max_cuts steps as in moc_search_cuts, with the moves of moc_eval_cuts_keep.
 * Phase 2 (the paper's Phase 2 minimises the duration, Eq. (1), from a solution
 * within the budget): max_merges times, the merge moves of the candidate are
 * written out as candidates of their own, evaluated by moc_eval_batch, and the
 * best one is applied in place.  A merge move exists for every live copy c that
 * has a live copy of its node below it (lower copy index); it switches c off
 * and keeps the nearest such copy until the later of the two ends: the node is
 * computed once less and its output held across the gap.  Only the first K
 * merge moves of a candidate, in order of the copy index, are looked at in a
 * step; the one applied is, among those whose result is feasible (no violation
 * and peak <= M), the one with the lowest duration, then the lowest peak, then
 * the lowest copy index.  A candidate with no feasible merge stays as it is.
 *   starts, ends, active   device, [B][T], edited in place
 *   K                      >= 1, merge moves per candidate and step
 *   work_best              device, moc_best_move [B], 8-byte aligned
 *   work_starts, work_ends device, int32 [B*K][T]      workspaces of Phase 2
 *   work_active            device, uint8 [B*K][T]      (may be NULL when
 *   work_list              device, int32 [B*K]          max_merges == 0)
 *   work_results           device, moc_result [B*K], 8-byte aligned
 *   out_cuts, out_merges   device, int32 [B]: moves applied in each phase
 * Queues 2 * max_cuts + 4 * max_merges + 2 kernels and returns; allocates
 * nothing.  Limits as moc_eval_cuts; B * K <= 2^31 - 1.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW, MOC_EHIP.
 */
int moc_search_two_phase(const moc_graph* g, int64_t B, int32_t* starts, int32_t* ends, uint8_t* active,
                         int32_t max_cuts, int32_t max_merges, int32_t K, moc_best_move* work_best,
                         int32_t* work_starts, int32_t* work_ends, uint8_t* work_active, int32_t* work_list,
                         moc_result* work_results, int32_t* out_cuts, int32_t* out_merges, void* hip_stream);

/*
 * Greedy descent by single-field moves, every candidate on its own: the moves
 * of moc_eval_neighbours, which cost no duration (they re-time computations
 * and retentions).  Repeats max_steps times: evaluate the candidate, find its
 * best move as moc_eval_neighbours does, and apply it in place if it lowers
 * (violations, max(peak, M), peak) lexicographically.  A candidate whose best
 * move does not stays as it is from then on.
 *   starts, ends    device, [B][T], edited in place; active is only read
 *   R               radius of the moves, 1 <= R <= 32
 *   work_results    device, moc_result [B], 8-byte aligned: workspace
 *   work_best       device, moc_best_move [B], 8-byte aligned: workspace
 *   out_steps       device, int32 [B]: number of moves applied
 * Queues 3 * max_steps + 1 kernels on the stream and returns; allocates
 * nothing.  Limits as moc_eval_neighbours; B <= 2^31 - 1.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW, MOC_EHIP.
 */
int moc_search_moves(const moc_graph* g, int64_t B, int32_t* starts, int32_t* ends, const uint8_t* active,
                     int32_t R, int32_t max_steps, moc_result* work_results, moc_best_move* work_best,
                     int32_t* out_steps, void* hip_stream);

/*
 * Turn B candidates into the rematerialisation sequences they stand for and
 * cost each sequence on its own terms (Section 2: the start of an active
 * interval is the event at which its node is computed; Section 1, problem
 * statement: validity, total duration and peak footprint of a sequence).
 * Only starts and active flags are read.  The steps of a candidate are its
 * active copies in order of their starts.  If an active copy starts outside
 * [0, T) or two active copies share a start (Eq. (8), Eq. (6)) there is no such
 * order: status -1.  The sequence is valid (status 1) when every node occurs
 * and every predecessor of a step's node has been computed at an earlier step;
 * otherwise status 0.  For a valid sequence, each use is served by the most
 * recent earlier computation of the producer, an output is held from the step
 * that computes it through the last step it serves (its own if none), and
 * peak is the largest summed size held at any step.  A candidate without
 * violations decodes to a valid sequence of the same duration whose peak is
 * not above the candidate's (ends may keep outputs longer than needed).
 *   out       device, moc_decode_result [B], 8-byte aligned
 *   out_seq   device, int32 [B][T], or NULL: the node of every step in order,
 *             then -1 up to T (all -1 when status == -1); 4-byte aligned
 * This call keeps 2.5 words per copy in LDS: T <= about 16000.  Edges (v,v) are
 * accepted (the first computation of such a node finds nothing to read: status
 * 0).  B == 0 is a no-op.
 * Errors: MOC_EINVAL, MOC_EDEVICE, MOC_EOVERFLOW (T too large for this call), MOC_EHIP.
 */
int moc_decode_batch(const moc_graph* g, int64_t B, const int32_t* starts, const uint8_t* active,
                     moc_decode_result* out, int32_t* out_seq, void* hip_stream);

/* Release a graph (synchronises its device first).  NULL is a no-op. */
void moc_graph_free(moc_graph* g);

/* Static description of an error code. */
const char* moc_strerror(int code);

/* hipError_t value of the last failed HIP call on this thread (0 if none). */
int moc_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOCCASIN_H */
