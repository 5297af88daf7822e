/*
 * hop.h -- C ABI of the MI355X chunked N-way reduce library.
 *
 * The library implements, on one GPU, the reduce path of Hoplite
 * (arXiv 2002.05814): Reduce(target, num_objects, sources, op) of Table 1,
 * scheduled by the dynamic d-ary tree of section 3.4.2, pipelined in chunks
 * as in section 3.3, tolerant of failing participants as in section 3.5.2,
 * plus the broadcast of section 3.4.1 and the reduce-then-broadcast allreduce
 * of section 3.4.3.
 *
 * Conventions shared by every call
 *   - "device pointer" = address in the memory of the current HIP device;
 *     "host pointer"   = ordinary process memory.
 *   - Objects are immutable (section 3.3): the library never writes a source
 *     object and never frees caller memory. Destinations must not overlap any
 *     source nor each other.
 *   - Device buffers (sources, destinations) must be 16-byte aligned.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and return without waiting for the GPU, like the
 *     paper's Reduce, which returns a future. Host arrays passed in are read
 *     before the call returns and may be reused at once.
 *   - Return value: a hop_status_t. Negative = error, nothing usable was
 *     written. No C++ exception crosses this boundary.
 *   - Thread safety: different sessions / calls may run on different host
 *     threads; one session must be driven from one thread at a time.
 */
#ifndef HOP_H
#define HOP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reduce operations of Table 1 ("sum, min, max"). */
typedef enum { HOP_SUM = 0, HOP_MIN = 1, HOP_MAX = 2 } hop_op_t;

/* Element types. The paper reduces 32-bit floats (section 5.1); bf16 and
 * int32 are additions. bf16 is widened exactly to binary32, combined in
 * binary32 and rounded to nearest-even once when stored; int32 sum wraps
 * modulo 2^32. */
typedef enum { HOP_F32 = 0, HOP_BF16 = 1, HOP_I32 = 2 } hop_dtype_t;

typedef enum {
    HOP_OK = 0,
    HOP_PARTIAL = 1,            /* fewer than k objects survived; all survivors were reduced */
    HOP_ERR_INVALID = -1,       /* bad argument (see each call)                              */
    HOP_ERR_ALIGN = -2,         /* a device buffer is not 16-byte aligned                    */
    HOP_ERR_NO_SURVIVOR = -3,   /* no object survived: there is nothing to reduce            */
    HOP_ERR_DEVICE = -4,        /* a HIP call failed                                         */
    HOP_ERR_NOMEM = -5,         /* host or device allocation failed                          */
    HOP_ERR_DEPTH = -6,         /* the tree needs more partial results in flight than the
                                   kernels hold in registers (see HOP_MAX_DEPTH)             */
    HOP_ERR_TOO_LARGE = -7,     /* the call needs more device scratch than it may take: than
                                   the library's static array holds (hop_reduce_noalloc) or
                                   than the caller's workspace (hop_session_set_workspace)   */
    HOP_ERR_CAPTURE = -8        /* the stream is being captured into a graph and the call
                                   would need memory from the library's caches (a staged
                                   program of more than 128 steps, a table too long for the
                                   kernel arguments, saved accumulators), which a replay of
                                   the graph would find
                                   rewritten: use hop_reduce_noalloc, or a session with
                                   hop_session_set_workspace                                 */
} hop_status_t;

/* Most partial results that can be live at once while one element's tree
 * expression is evaluated. A child subtree that is not a first child and has
 * more than one node is evaluated into a partial result of its own while its
 * parent's partial waits; the depth is 1 + the deepest nesting of such
 * subtrees. A chain (d = 1) and a star need 1, a complete binary tree on k
 * nodes about log2(k) - 1. */
#define HOP_MAX_DEPTH 16

typedef struct {
    int32_t k_eff;          /* objects folded into the result                         */
    int32_t n_failed_seen;  /* failure notifications the scheduler acted on           */
    int32_t n_replaced;     /* failed tree positions refilled by a waiting object     */
    int32_t degree_used;    /* tree degree actually used (matters for tree_degree 0)  */
    int64_t chunks_redone;  /* repair work: chunks relaunched after a failure, each
                               counted once per source object read again             */
    int32_t n_launches;     /* reduce kernels enqueued                                */
    int32_t stack_depth;    /* partial results live at once (<= HOP_MAX_DEPTH)        */
    int64_t chunk_steps;    /* work actually enqueued: sum over launches of chunks x
                               program steps (= source chunks read), repairs included */
    int64_t chunk_stores;   /* sum over launches of chunks whose result or accumulators
                               were written                                           */
    int64_t partial_loads;  /* sum over launches of chunks x kept partial results read
                               (4 bytes per element each), see hop_session_set_retention */
    int64_t partial_stores; /* sum over launches of chunks x partial results kept      */
} hop_info_t;

/*
 * hop_reduce -- Reduce of Table 1 with the tree schedule of section 3.4.2
 * and the failure handling of section 3.5.2, over objects already resident
 * in device memory.
 *
 *   dst          device pointer, object_bytes bytes; receives the result.
 *   objs         host array of n device pointers, each object_bytes bytes.
 *   n            number of source objects (the paper's source list), >= 1.
 *   object_bytes size of every object; a multiple of the element size; may
 *                be 0 (nothing is launched).
 *   ready_order  host array, a permutation of 0..n-1: the order in which the
 *                objects become ready (arrive). NULL = 0,1,..,n-1.
 *   k            num_objects: how many objects to reduce, 1 <= k <= n. The
 *                first k arrivals take the k tree positions by generalised
 *                in-order traversal (first child, node, other children).
 *   op, dtype    see above.
 *   chunk_bytes  pipelining block (section 3.3; the paper uses 4 MB): the unit
 *                of readiness, scheduling, failure and repair. > 0 and a
 *                multiple of 16.
 *   tree_degree  d >= 1 (1 = chain, >= k-1 = star); 0 lets the library choose
 *                among {1, 2, k} with the cost model of section 3.4.2 (Eq. 1).
 *   fail_mask    host array of n entries or NULL (nobody fails).
 *                fail_mask[i] < 0: object i is healthy. fail_mask[i] = c >= 0:
 *                object i delivers exactly c chunks and then fails; c = 0 means
 *                it never becomes ready; c >= number of chunks means it
 *                completed, i.e. healthy. All participants stream their chunks
 *                side by side, so a participant that fails after c chunks is
 *                noticed when chunks 0..c-1 of the output have already been
 *                produced with its data: those chunks are produced again
 *                without it, from the kept partial results of the subtrees it
 *                was not in where there are any (see
 *                hop_session_set_retention). The failed position goes to the
 *                next ready object not yet in the tree, else stays empty.
 *   stream       hipStream_t.
 *   info         host pointer or NULL; filled before return.
 *
 * Result: for every element, the tree-ordered op over the objects finally in
 * the tree = the first k ready objects that did not fail. HOP_PARTIAL when
 * fewer than k survive (the paper would wait for reconstruction instead).
 * Errors: HOP_ERR_INVALID for n < 1, k < 1, k > n, a non-permutation
 * ready_order, bad op/dtype, object_bytes not a multiple of the element size,
 * chunk_bytes 0 or not a multiple of 16, tree_degree < 0, NULL dst/objs;
 * HOP_ERR_ALIGN; HOP_ERR_NO_SURVIVOR; HOP_ERR_DEPTH; HOP_ERR_DEVICE/NOMEM.
 */
int hop_reduce(void *dst, const void *const *objs, int n, size_t object_bytes,
               const int32_t *ready_order, int k, hop_op_t op, hop_dtype_t dtype,
               size_t chunk_bytes, int tree_degree, const int64_t *fail_mask,
               void *stream, hop_info_t *info);

/*
 * hop_reduce_noalloc -- hop_reduce for callers that cannot allocate device
 * memory: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc. Same arguments, same result bits, same status codes as
 * hop_reduce, but the call allocates and frees nothing on the device and
 * calls no allocating library routine: whatever device scratch the kernels
 * need (programs of more than 128 steps; long chain tables, partial results
 * and sub-programs of a reduce over many small objects) lives in one static
 * device array of hop_noalloc_scratch_bytes() bytes (8 MiB) that every GPU
 * the library runs on holds until the process ends, and programs and tables
 * reach it through kernel arguments instead of a staging buffer.
 *   - A call whose program alone does not fit (about 500 000 inputs) returns
 *     HOP_ERR_TOO_LARGE and enqueues nothing. A many-small-objects call
 *     whose partial results do not fit is evaluated by one program instead
 *     (slower, same bits).
 *   - All calls on one GPU share that GPU's array, which keeps the last
 *     call's contents; nothing in it has to start at zero (every partial
 *     result is written before it is read). Calls on the same stream are
 *     ordered by the stream. Calls that overlap on one GPU (different
 *     streams, or host threads on different streams) race on the array:
 *     the caller must serialise them.
 *   - hop_reduce's repair of a mid-stream failure works as in hop_reduce.
 */
int hop_reduce_noalloc(void *dst, const void *const *objs, int n, size_t object_bytes,
                       const int32_t *ready_order, int k, hop_op_t op, hop_dtype_t dtype,
                       size_t chunk_bytes, int tree_degree, const int64_t *fail_mask,
                       void *stream, hop_info_t *info);

/* Size in bytes of the static device array behind hop_reduce_noalloc. */
size_t hop_noalloc_scratch_bytes(void);

/*
 * hop_broadcast -- section 3.4.1: every receiver ends with a byte-identical
 * copy of the object, moved chunk by chunk.
 *   dsts   host array of n_dst device pointers (object_bytes each); n_dst >= 0.
 *   src    device pointer, object_bytes bytes.
 * The source is fetched from device memory once and written to every
 * destination (with several destinations it is re-read per destination from
 * the on-chip caches).
 * Errors: HOP_ERR_INVALID (n_dst < 0, NULL table or entry, chunk_bytes 0 or
 * not a multiple of 16, destinations overlapping the source or each other),
 * HOP_ERR_ALIGN, HOP_ERR_DEVICE/NOMEM.
 */
int hop_broadcast(void *const *dsts, int n_dst, const void *src, size_t object_bytes,
                  size_t chunk_bytes, void *stream);

/*
 * Receiver-driven broadcast, event by event (sections 3.4.1 and 3.5.1).
 * hop_broadcast above is the case where all receivers are known at once; here
 * receivers join one after the other and the library plays the object
 * directory: a joining receiver is given ONE sender, an idle complete copy if
 * there is one, else an idle partial copy (a receiver still receiving);
 * a copy serves one receiver at a time and is listed again when its transfer
 * ends, so the broadcast tree forms from the arrival order and data flows
 * chunk by chunk through chains of partial copies. If a copy fails, the
 * receiver it was serving asks again and resumes from the chunks it already
 * has, never from a copy that (transitively) fetches from itself.
 * Time is explicit: nothing moves until hop_bcast_step, which lets every
 * transfer advance by at most max_chunks chunks (0 = as far as its sender
 * has), senders before their receivers. On one GPU every "transfer" is a
 * chunk-range copy between two device buffers on `stream`.
 *
 *   hop_bcast_begin        src = device pointer of the original copy, or NULL
 *                          for a host-only session that only records copies.
 *   hop_bcast_source_ready the original has chunks [0, c) (its Put may still be
 *                          in progress); begins at 0.
 *   hop_bcast_join         a receiver arrives with its device buffer dst
 *                          (ignored in host-only sessions). Returns its copy id
 *                          (>= 1; the original is copy 0) or a negative status;
 *                          *sender (may be NULL) = the copy it was given, -1 if
 *                          every copy is busy (it asks again at each step).
 *   hop_bcast_fail         copy `copy` is lost.
 *   hop_bcast_sender       the copy that `copy` currently fetches from, or -1.
 *   hop_bcast_finish       steps until nothing moves any more, fills info and
 *                          the log of copies (both may be NULL), frees the
 *                          session. HOP_OK if every surviving receiver is
 *                          complete, HOP_PARTIAL otherwise.
 */
typedef struct hop_bcast hop_bcast_t;
typedef struct { int32_t from, to; int64_t chunk_begin, chunk_end; } hop_bcast_copy_t;
typedef struct {
    int32_t n_receivers;    /* receivers that joined                                   */
    int32_t n_failed;       /* copies reported lost                                    */
    int32_t n_resumed;      /* transfers taken up again from another sender            */
    int32_t n_complete;     /* surviving receivers that hold the whole object          */
    int64_t chunks_copied;  /* chunk transfers performed (no chunk is sent twice to the
                               same receiver)                                          */
} hop_bcast_info_t;

int hop_bcast_begin(hop_bcast_t **b, const void *src, size_t object_bytes, size_t chunk_bytes, void *stream);
int hop_bcast_source_ready(hop_bcast_t *b, int64_t chunks_ready_total);
int hop_bcast_join(hop_bcast_t *b, void *dst, int *sender);
int hop_bcast_fail(hop_bcast_t *b, int copy);
int hop_bcast_step(hop_bcast_t *b, int64_t max_chunks);
int hop_bcast_sender(hop_bcast_t *b, int copy);
int hop_bcast_finish(hop_bcast_t *b, hop_bcast_info_t *info, hop_bcast_copy_t *log, int log_capacity, int *n_log);

/*
 * hop_allreduce -- section 3.4.3: Reduce followed by Broadcast, composed
 * chunk by chunk (section 3.3): each finished result chunk goes to all n_dst
 * destinations. Arguments as hop_reduce / hop_broadcast; n_dst >= 1. Every
 * destination receives the same bits hop_reduce would have produced.
 */
int hop_allreduce(void *const *dsts, int n_dst, const void *const *objs, int n,
                  size_t object_bytes, const int32_t *ready_order, int k, hop_op_t op,
                  hop_dtype_t dtype, size_t chunk_bytes, int tree_degree,
                  const int64_t *fail_mask, void *stream, hop_info_t *info);

/*
 * Event-level form of Reduce: the caller reports, as they happen, which
 * chunks of which object have become ready and which participants failed;
 * the scheduler assigns tree positions in arrival order (section 3.4.2),
 * launches the reduce of every output chunk whose inputs are all present, and
 * repairs after failures (section 3.5.2). hop_reduce is a replay of these
 * calls.
 */
typedef struct hop_session hop_session_t;

/* Opens a session. Arguments as hop_reduce. *s is set on HOP_OK. */
int hop_session_begin(hop_session_t **s, void *dst, const void *const *objs, int n,
                      size_t object_bytes, int k, hop_op_t op, hop_dtype_t dtype,
                      size_t chunk_bytes, int tree_degree, void *stream);

/* Object obj now has chunks 0..chunks_ready_total-1 ready (monotone; the first
 * call for an object is its arrival and fixes its tree position or puts it
 * among the waiting objects; 0 announces an object that has no data yet).
 * Launches every output chunk that became complete. HOP_ERR_INVALID for an
 * unknown object, a count that decreases or exceeds the number of chunks, or
 * an object already reported failed. */
int hop_session_ready(hop_session_t *s, int obj, int64_t chunks_ready_total);

/* The same notification for data that is still being produced on the GPU: the
 * chunks are ready once `event` (a hipEvent_t recorded on the producer's
 * stream, passed as void*; NULL = ready now) has completed. The session's
 * stream is made to wait for the event before any work enqueued from now on,
 * so no host synchronisation is needed between a producer (a copy landing a
 * chunk, a kernel computing an object, another session's output) and the
 * reduce: the event plays the part of the paper's readiness notification
 * (section 3.3). The event may be re-recorded or destroyed after the call
 * returns. Host-only sessions ignore it. */
int hop_session_ready_after(hop_session_t *s, int obj, int64_t chunks_ready_total, void *event);

/* Participant obj failed. If all its chunks were already ready the object is
 * complete and the call changes nothing. Otherwise it leaves the tree: output
 * chunks already produced with its data are scheduled again, its position
 * goes to the next waiting object (else stays empty). */
int hop_session_fail(hop_session_t *s, int obj);

/* Scheduling policy. min_steps = 0 (default): an output chunk is produced by one
 * launch once all its inputs are present (least traffic). min_steps = m >= 1:
 * a chunk also advances whenever at least m further steps of its program have
 * become runnable, its accumulators being saved in device scratch in between
 * (4 bytes per element and live level), so that work overlaps the wait for
 * late participants and little is left to do when the last one arrives
 * (section 3.4.2: progress with a subset of the objects). Results are
 * bit-identical in both modes. */
int hop_session_set_eager(hop_session_t *s, int min_steps);

/* Refinement of the eager policy (min_steps >= 1): a chunk advances part of
 * the way only if the stream has already executed everything this session
 * enqueued before. Participants that arrive faster than the GPU works are then
 * folded together into fewer, longer launches (in the limit the default
 * policy's single launch); participants that arrive with gaps are worked off
 * in the gaps. The number of launches then depends on timing; the result does
 * not. Host-only sessions count as always idle. */
int hop_session_set_adaptive(hop_session_t *s, int on);

/* Keeping partial results for the repair of failures (section 3.5.2: when a
 * participant fails, the partial results that do not contain its object are
 * kept and only its ancestors in the tree start over). on != 0 (default): a
 * launch that produces output chunks while some participant in the tree is
 * still streaming - and so can still fail - also stores, in device scratch of
 * the library (4 bytes per element and subtree), the partial result of every
 * subtree with more than one node rooted at one level of the tree: one to
 * four levels below the root, the level for which a repair reads least on
 * average over who fails (level 1 for the wide trees, level 2 for a binary
 * tree on 32). After a failure (or a late arrival into an empty position)
 * the chunks already produced are repaired by a launch that reads the kept
 * partials of the untouched subtrees and re-reads only the objects of the
 * subtree that changed and those above the kept level. Launches made when
 * nobody can fail any more (every launch of a call whose participants all
 * complete) keep nothing and cost nothing extra; launches that keep partials
 * move 10-20 % more bytes and take about as much longer. Nothing is kept
 * either for launches over less than 8 MiB per object, for chains and stars
 * (no subtrees), when every level has more than 16 subtrees or kept arrays
 * beyond a quarter of what the launch reads or 16 GiB, or in
 * hop_reduce_noalloc. on = 0: never keep; a repair reads every object
 * of the chunk again. Results are bit-identical either way. */
int hop_session_set_retention(hop_session_t *s, int on);

/* A workspace of the caller's for this session: from now on every byte of
 * device scratch the session needs - staged programs and program segments,
 * the saved accumulators of the eager policy, the kept partial results of
 * failure repair - is taken from [device_memory, device_memory + bytes) and
 * the session allocates nothing, neither on the device nor in pinned host
 * memory (programs reach the workspace through kernel arguments), so its calls
 * never block on an allocation and can be captured into a HIP graph.
 * device_memory: device pointer, 256-byte aligned, owned by the caller, not to
 * be touched until the stream has executed the session's work (and, for a
 * captured graph, as long as the graph is replayed). Call it right after
 * hop_session_begin: HOP_ERR_INVALID once the session has staged anything.
 * hop_workspace_bytes gives the size of the object-sized arrays (saved
 * accumulators, kept partials); on top of that every launch of the eager policy
 * stages its program segment (16 bytes per step, rounded up to 256) and nothing
 * is given back before the session ends, so add that for the launches expected.
 * An event call that runs out of workspace returns HOP_ERR_TOO_LARGE (kept
 * partial results that do not fit are simply not kept). */
int hop_session_set_workspace(hop_session_t *s, void *device_memory, size_t bytes);

/* Number of leading output chunks that are final in dst as far as the work
 * enqueued so far goes (a later failure can take chunks back). This is what a
 * downstream consumer on the same stream may read, e.g. a second session that
 * takes dst as one of its sources (composed Reduce, section 3.4.2):
 * hop_session_ready(next, obj, hop_session_chunks_final(s)). */
int64_t hop_session_chunks_final(hop_session_t *s);

/* Ends the session: participants that have not delivered every chunk are
 * treated as failed, remaining work is enqueued, info (may be NULL) is
 * filled, the session is freed. Returns HOP_OK / HOP_PARTIAL or an error
 * (the session is freed in every case). */
int hop_session_finish(hop_session_t *s, hop_info_t *info);

/*
 * Host-only view of the schedule, for inspection and tests: runs the same
 * scheduler as hop_reduce on the same arguments but enqueues nothing on any
 * device (no pointer is dereferenced; objects are named by index).
 *
 * Launch l works on output chunks [chunk_begin, chunk_end) by evaluating steps
 * [step_begin, step_end) of the program entries[entry_begin, entry_end) for
 * each element (hop_reduce always runs whole programs: step_begin = 0, final):
 *   SET  : acc[level] = x            (x = the element of object `obj`)
 *   else : acc[level] = acc[level] (op) x
 *   then n_fold times: acc[level-1] = acc[level-1] (op) acc[level]; --level
 * and storing acc[0]. Launches must be applied in order (a later launch may
 * overwrite chunks of an earlier one: that is failure repair).
 * Kept partial results (hop_session_set_retention): there are up to 16 arrays
 * kept[q] of accumulator-typed values, indexed like the object's elements. A
 * step with obj = -(1 + q) takes x from kept[q] instead of an object. A step
 * with save = q >= 0 stops its folds when they have come down to save_level,
 * stores kept[q] = acc[save_level] for the launch's chunks, and then performs
 * the remaining folds.
 * Returns the status hop_reduce would return; *n_launches / *n_entries hold
 * the counts needed (also when they exceed the capacities, in which case
 * the arrays are filled up to capacity).
 */
typedef struct {
    int32_t obj;            /* >= 0: object; -(1 + q): kept partial result q (see below)            */
    uint8_t level;
    uint8_t set;
    uint16_t n_fold;
    int16_t save;           /* -1, or q: this step also stores kept partial q (see below)          */
    uint8_t save_level;
    uint8_t reserved;
} hop_plan_entry_t;
typedef struct {
    int64_t chunk_begin, chunk_end;   /* output chunks the launch works on                            */
    int32_t entry_begin, entry_end;   /* the program in force: entries[entry_begin, entry_end)         */
    int32_t step_begin, step_end;     /* steps of that program the launch runs (0 .. program length)   */
    int32_t final;                    /* 1: stores the result; 0: saves live_after accumulator levels  */
    int32_t live_before, live_after;  /* accumulator levels restored before / saved after the steps    */
    int32_t reserved;
} hop_plan_launch_t;

int hop_plan_reduce(int n, size_t object_bytes, const int32_t *ready_order, int k,
                    hop_dtype_t dtype, size_t chunk_bytes, int tree_degree,
                    const int64_t *fail_mask, hop_info_t *info,
                    hop_plan_launch_t *launches, int launch_capacity, int *n_launches,
                    hop_plan_entry_t *entries, int entry_capacity, int *n_entries);

/* The same for the event-level form: a session that enqueues nothing. Drive it
 * with hop_session_ready / _fail / _set_eager, then collect the record (and
 * free the session) with hop_plan_session_finish. */
int hop_plan_session_begin(hop_session_t **s, int n, size_t object_bytes, int k, hop_dtype_t dtype,
                           size_t chunk_bytes, int tree_degree);
int hop_plan_session_finish(hop_session_t *s, hop_info_t *info,
                            hop_plan_launch_t *launches, int launch_capacity, int *n_launches,
                            hop_plan_entry_t *entries, int entry_capacity, int *n_entries);

/*
 * Host-only view of how a long program is cut for launches that cover few
 * tiles (many small objects). A run is a stretch of steps that starts a partial
 * above level 0 and ends where it is folded away: a non-first-child subtree, an
 * independent sub-expression. While the program has at least want_steps steps,
 * every outermost run of min_run..max_run steps becomes a sub-program of its
 * own (levels counted from the run's level); in the program it came from it is
 * replaced by one step with obj = -(1 + g) naming the partial of sub-program g.
 * What is left is cut again by the same rule until it is short or nothing
 * more can be cut. sub_pass[g] is the pass in which sub-program g must run: it
 * reads only objects and partials of earlier passes; the top program runs last.
 * sub_begin receives n_subs + 1 offsets into sub_entries (capacity counts
 * entries of sub_begin; sub_pass needs one less). Counts are always returned;
 * arrays are filled up to capacity. Returns HOP_OK if anything was cut,
 * HOP_PARTIAL if the program stays whole.
 */
int hop_plan_split(const hop_plan_entry_t *entries, int n_entries, int want_steps, int min_run, int max_run,
                   hop_plan_entry_t *top, int top_capacity, int *n_top,
                   hop_plan_entry_t *sub_entries, int sub_capacity, int *n_sub_entries,
                   int32_t *sub_begin, int32_t *sub_pass, int sub_table_capacity, int *n_subs, int *n_passes);

/*
 * Host-only view of the one-launch form of a long program over small objects:
 * the program as chains. A chain is a left fold, item 0 (op) item 1 (op) ...
 * in that order, of objects (item >= 0) and of the values of other chains
 * (item = -(1 + g)); the last chain's value is the program's result. Every
 * accumulator level of the program is one such fold (the steps that combine
 * into it and the values folded down into it, in program order - the
 * arithmetic of section 3.4.2's tree, unchanged). A chain is cut where it
 * first needs a value that is ready later than all it holds so far, if it
 * holds at least min_cut items by then: the front becomes a chain of its own.
 * A chain that reaches max_items (>= 2) items is cut the same way.
 * chain_pass[g] = 0 if chain g reads objects only, else 1 + the largest pass
 * among the chains it reads; the chains of one pass are independent, and one
 * workgroup evaluates them side by side, their values held in LDS.
 * chain_begin receives n_chains + 1 offsets into items (table_capacity counts
 * entries of chain_begin; chain_pass needs one less). Counts are always
 * returned, arrays filled up to capacity. HOP_OK, or HOP_PARTIAL if the
 * program has no such form (one object, or it reads kept partial results).
 */
int hop_plan_chains(const hop_plan_entry_t *entries, int n_entries, int min_cut, int max_items,
                    int32_t *items, int item_capacity, int *n_items,
                    int32_t *chain_begin, int32_t *chain_pass, int table_capacity, int *n_chains, int *n_passes);

/* node_of_slot[t] (k entries) = level-order index of the tree node that the
 * t-th arrival takes in the complete d-ary tree on k nodes. */
int hop_plan_slots(int k, int tree_degree, int32_t *node_of_slot);

/* Degree the library would choose for tree_degree = 0: argmin over {1, 2, k}
 * (the candidates of the paper's runtime, section 4) of T(d) of Eq. 1
 * (section 3.4.2) with per-level latency latency_s and bandwidth
 * bytes_per_s. Candidates within 2 % of the best predicted time count as
 * equal; among equals the tree that needs the fewest accumulator levels wins
 * (a chain and a star need one), then the smaller degree. Non-positive
 * values select the constants measured by the last hop_calibrate of this
 * process, or, if there was none, typical MI355X figures (3 us, 6.5 TB/s). */
int hop_pick_degree(int k, size_t object_bytes, double latency_s, double bytes_per_s);

/* Measures the two constants of Eq. 1 on the current device, as section 4 of
 * the paper does on its cluster: latency_s = what one more dependent launch of
 * the smallest reduce costs (the price of a tree level that is a launch of its
 * own), bytes_per_s = the rate at which the reduce kernel streams objects in
 * (four 64 MiB objects). Takes under a millisecond of GPU time on a stream of
 * its own, allocates 320 MiB of device memory and frees it again, waits for the
 * result. The values are kept per device and used by every later
 * tree_degree = 0 call there; the first such call on a device calibrates by
 * itself (and so blocks once) unless its stream is being captured into a
 * graph. Either pointer may be NULL. On one GPU the degree changes neither the
 * bytes moved nor the number of launches of the default policy, only the
 * association order and the number of accumulator levels, so the choice
 * matters little for speed (measured: under 1 % for fp32 and int32); for floats
 * it decides the result's bits, which therefore can differ between devices
 * and library versions when tree_degree is 0. Pass an explicit degree where
 * bit-reproducibility matters. */
int hop_calibrate(double *latency_s, double *bytes_per_s);

/* Upper bound, in bytes, of the device memory the library takes from its
 * cached workspaces for ONE hop_reduce / hop_allreduce call or one session of
 * this shape (arguments as hop_reduce; n_dst = destinations, 1 for a plain
 * reduce; tree_degree 0 = the degree the library would pick now). Counted:
 *   - the staged program (16 bytes per step when there are more than 128) and
 *     the table of the other n_dst - 1 destinations when there are more than
 *     64 of them (shorter programs and tables ride in the kernel arguments),
 *     in blocks of 256 KiB (the same number of bytes of pinned host memory
 *     goes with them);
 *   - for a call over 48 or more inputs of at most 768 KiB each: the table of
 *     the one-launch form of its program (192 bytes per chain, fewer chains
 *     than inputs);
 *   - for a call over 128 or more inputs of at most 768 KiB each (bf16:
 *     512 KiB, and its partial results are 4-byte accumulators): the partial
 *     results and records of its sub-programs (at most 256 MiB; a cut that
 *     would need more is not made);
 *   - HOP_WS_EAGER (sessions with hop_session_set_eager(s, m >= 1)): the saved
 *     accumulators, 4 bytes per element and accumulator level of the tree;
 *   - HOP_WS_FAILURES (participants may fail mid-stream; objects of 8 MiB or more):
 *     the kept partial results, 4 bytes per element and subtree below the
 *     root (hop_session_set_retention).
 * The memory is allocated on first use, cached by the library (idle buffers
 * above 8 GiB in total are freed) and freed by hop_shutdown; calls that find
 * nothing cached allocate, and so can block. Returns 0 for invalid arguments.
 * hop_reduce_noalloc takes none of this: see hop_noalloc_scratch_bytes. */
#define HOP_WS_EAGER 1
#define HOP_WS_FAILURES 2
size_t hop_workspace_bytes(int n, int k, size_t object_bytes, size_t chunk_bytes, int tree_degree,
                           hop_dtype_t dtype, int n_dst, int policy);

/* Frees the cached workspaces of the calling process (optional; for leak checks). */
int hop_shutdown(void);

const char *hop_strerror(int status);

/* Static string naming the launch shape the kernels were built with (vectors
 * per lane, unroll, workgroup size, cache policy). Measurements taken with
 * hardware counters are only valid for the shape they were taken on. */
const char *hop_kernel_config(void);

#ifdef __cplusplus
}
#endif
#endif /* HOP_H */
