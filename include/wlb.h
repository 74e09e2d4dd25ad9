/*
 * wlb.h -- C ABI of the MI355X (gfx950) WLB-LLM hot path.
 *
 * Four groups of calls:
 *   wlb_pack        workload-aware variable-length packing (host, integers)
 *   wlb_shard*      context-parallel sharding maps          (host, integers)
 *   wlb_attn_plan   tile schedule for the attention kernels (device, integers)
 *   wlb_attn_fwd / wlb_attn_bwd   document-masked causal attention (device, bf16 MFMA)
 *
 * Conventions
 *   - Every call returns a wlb_status; WLB_OK is 0.  No exception crosses the
 *     boundary.  wlb_last_error() returns a thread-local, NUL-terminated text for
 *     the last non-OK status returned on the calling thread.
 *   - The caller owns every buffer.  "host" pointers are ordinary host memory;
 *     "device" pointers are HIP device memory on the current device.  The library
 *     keeps no device memory of its own: scratch lives in the caller's workspace,
 *     sized by wlb_attn_workspace_size().
 *   - Host calls are synchronous.  Device calls only enqueue work on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and return; they
 *     never synchronise and never allocate.  They issue kernel launches only (no
 *     memset, no copy), so a caller may capture them into a HIP graph and replay it.
 *     Calls that share a workspace must be ordered on their stream(s): the schedule,
 *     partial results and per-row scratch in it are rewritten by every call.
 *   - Token indices and offsets are int32 (T < 2^31); pair counts and costs are 64-bit.
 *   - bf16 tensors are passed as void* to 2-byte elements, row-major, token-major:
 *     Q, O, dO, dQ are [n_q][hq][head_dim]; K, V, dK, dV are [t_kv][hkv][head_dim];
 *     LSE is float [hq][n_q].
 */
#ifndef WLB_H
#define WLB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WLB_OK = 0,
    WLB_ERR_INVALID_ARG = 1,      /* null pointer, non-positive length, rank out of range, ... */
    WLB_ERR_BUFFER_TOO_SMALL = 2, /* workspace smaller than wlb_attn_workspace_size() asks for */
    WLB_ERR_UNSUPPORTED = 3,      /* head_dim other than 64 or 128, sizes beyond the int32 range, a tensor near 4 GiB */
    WLB_ERR_HIP = 4               /* a HIP runtime call failed; text in wlb_last_error() */
} wlb_status;

const char* wlb_last_error(void);

/* ------------------------------------------------------------------------------------------
 * Packing -- the greedy core of Algorithm 1 (paper Section 4.3), with the workload model of
 * Equation 2 (Section 4.1): a micro-batch's workload is the sum over its documents of
 * W_a(d) + W_l(d), attention quadratic and everything else linear in the document length
 * (Sections 3.2 and 4.1):  cost(d) = cost_a*d*d + cost_b*d  in unsigned 64-bit integers.
 *
 * Documents are taken longest first (stable: equal lengths keep arrival order).  Each goes
 * to the micro-batch with the least workload if its token count stays <= l_max, else to the
 * micro-batch with the fewest tokens if it fits there, else it is left over (assign = -1)
 * for the caller to carry into the next iteration.  Ties go to the lowest micro-batch index.
 *
 *   doc_len   host, [n_docs], each > 0
 *   assign    host, [n_docs], out: micro-batch id in [0, n_microbatch) or -1
 *   mb_len    host, [n_microbatch], out: tokens per micro-batch
 *   mb_cost   host, [n_microbatch], out: workload per micro-batch
 * Errors: INVALID_ARG for null pointers (n_docs == 0 is allowed), n_microbatch < 1,
 * l_max < 1, a document length <= 0, or cost_a/cost_b so large that a full micro-batch
 * (cost_a*l_max^2 + cost_b*l_max) would not fit in 64 bits.
 */
wlb_status wlb_pack(const int32_t* doc_len, int64_t n_docs,
                    int32_t n_microbatch, int64_t l_max,
                    uint64_t cost_a, uint64_t cost_b,
                    int32_t* assign, int64_t* mb_len, uint64_t* mb_cost);

/* ------------------------------------------------------------------------------------------
 * Exact solution of Equation 2 (Section 4.1) for small inputs, by branch and bound: every
 * document in exactly one micro-batch, every micro-batch at most l_max tokens, the largest
 * micro-batch cost (cost as in wlb_pack) minimal.  The paper solves this with an ILP solver
 * and reports it too slow for training (Section 4.1, Table 2); here it measures how far the
 * greedy of wlb_pack is from the optimum on small instances.  Host, synchronous.
 * node_limit > 0 bounds the search (nodes visited); *proven = 1 when the search finished, 0 when
 * the limit cut it short (the result is then the best assignment found).  Outputs as wlb_pack,
 * without -1 entries.  Errors: INVALID_ARG (null pointers, n_docs or n_microbatch outside
 * 1..64, a length outside (0, l_max], cost overflow, no feasible assignment found).
 */
wlb_status wlb_pack_optimal(const int32_t* doc_len, int64_t n_docs, int32_t n_microbatch, int64_t l_max,
                            uint64_t cost_a, uint64_t cost_b, int64_t node_limit, int32_t* assign,
                            int64_t* mb_len, uint64_t* mb_cost, uint64_t* optimal_cost, int32_t* proven);

/* ------------------------------------------------------------------------------------------
 * Streaming packer -- the whole of Algorithm 1 (Section 4.3) including the outlier delay of
 * Section 4.2, one step per global batch.  The packer object lives in host memory and carries
 * the algorithm's state between steps: the left-over documents and the FIFO waiting queues.
 *
 * thresholds[0] < ... < thresholds[n_queues-1] are the queue bounds L_1..L_n: a document of
 * length >= L_1 is an outlier and waits in queue i with L_i <= length < L_{i+1} (the last
 * queue is open-ended).  In a step, after the batch is read, every queue holding at least
 * n_microbatch documents releases its n_microbatch oldest ones (queues in index order).  The
 * pending set -- previous left-overs, then this batch's ordinary documents in arrival order,
 * then the released outliers -- is sorted by length (stable) and packed exactly as wlb_pack
 * does; what fits nowhere is carried over.  n_queues == 0 gives the plain streaming packer.
 *
 * wlb_packer_create: host; *out receives the object (free it with wlb_packer_destroy).
 * wlb_packer_step:   host; doc_len/doc_id [n_docs] describe the arriving batch (ids are opaque
 *   to the library).  Outputs, in placement order (longest first): out_doc_id, out_doc_len,
 *   out_mb [capacity]; *n_out = documents placed; mb_len, mb_cost [n_microbatch].
 *   capacity must be >= wlb_packer_pending() total + n_docs (everything that could be placed).
 * wlb_packer_pending: host; documents carried over and documents waiting in queues.
 * Errors: INVALID_ARG (null pointers, non-increasing thresholds, a length <= 0 or > l_max, the
 * cost overflow rule of wlb_pack), BUFFER_TOO_SMALL (capacity).  A failed step changes nothing.
 */
typedef struct wlb_packer wlb_packer;

wlb_status wlb_packer_create(int32_t n_microbatch, int64_t l_max, uint64_t cost_a, uint64_t cost_b,
                             const int64_t* thresholds, int32_t n_queues, wlb_packer** out);
void wlb_packer_destroy(wlb_packer* packer);
wlb_status wlb_packer_step(wlb_packer* packer, const int32_t* doc_len, const int64_t* doc_id, int64_t n_docs,
                           int64_t* out_doc_id, int32_t* out_doc_len, int32_t* out_mb, int64_t capacity,
                           int64_t* n_out, int64_t* mb_len, uint64_t* mb_cost);
wlb_status wlb_packer_pending(const wlb_packer* packer, int64_t* n_left_over, int64_t* n_queued);

/* ------------------------------------------------------------------------------------------
 * Sharding maps (paper Section 3.1 for per-sequence, Section 5.1 for per-document).
 *
 * WLB_SHARD_PER_SEQ: the packed sequence is cut into 2*cp equal chunks; rank r owns chunks
 * r and 2*cp-1-r.  Needs 2*cp | T.
 * WLB_SHARD_PER_DOC_PADDED: every document is cut into 2*cp chunks of c = ceil(L/(2*cp))
 * positions; rank r owns chunks r and 2*cp-1-r of every document; positions >= L are padding
 * and appear as slots with q_idx = -1, so every rank has the same number of slots.
 * WLB_SHARD_PER_DOC_NOPAD (Section 5.1, "Avoid Padding"): the first 2*cp*floor(L/(2*cp)) tokens of
 * a document are sharded as above without padding; its last L mod 2*cp tokens are dealt to the
 * ranks round-robin by one counter that runs on across documents (remaining token number t of
 * the sequence goes to rank t mod cp).  No slot is padding; when 2*cp | T every rank gets T/cp
 * slots, otherwise the counts differ by at most one.  A rank's slots stay document-major: front
 * chunk, back chunk, then its remaining tokens of that document.
 * cp == 1 is the identity map (no padding) in every mode.
 *
 * A rank's slots are ordered document-major, front chunk before back chunk.  A segment is a
 * maximal run of slots from one chunk and one document.
 *
 * wlb_shard_size: host; writes the slot count n_q and segment count n_seg for `rank`.
 * wlb_shard: host; all outputs are caller-allocated host arrays:
 *   q_idx        [n_q]      global token index of each local slot, -1 = padding slot
 *   cu_seqlens_q [n_seg+1]  slot offsets of the segments
 *   seg_k_begin  [n_seg]    first key a segment's rows may see (= its document's start)
 *   seg_k_end    [n_seg]    one past the last key the segment's last real row may see
 *                           (= seg_k_begin when the segment has no real row)
 *   cu_seqlens_k [n_docs+1] document offsets in the packed sequence
 *   useful_pairs            this rank's count of in-document causal (query,key) pairs
 * Any output pointer except q_idx may be NULL to skip it.
 * Errors: INVALID_ARG for null doc_len/q_idx, n_docs < 1, cp < 1, rank outside [0,cp),
 * unknown mode, a length <= 0, per-sequence mode with T not divisible by 2*cp;
 * UNSUPPORTED when T (or the padded slot count) does not fit in int32.
 */
enum { WLB_SHARD_PER_DOC_PADDED = 0, WLB_SHARD_PER_SEQ = 1, WLB_SHARD_PER_DOC_NOPAD = 2 };

wlb_status wlb_shard_size(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t rank,
                          int32_t mode, int64_t* n_q, int64_t* n_seg);

wlb_status wlb_shard(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t rank, int32_t mode,
                     int32_t* q_idx, int32_t* cu_seqlens_q, int32_t* seg_k_begin,
                     int32_t* seg_k_end, int32_t* cu_seqlens_k, int64_t* useful_pairs);

/* ------------------------------------------------------------------------------------------
 * Attention on one context-parallel rank's rows (paper Sections 1 and 3.2 for the mask:
 * a token attends only to earlier-or-equal tokens of its own document; Section 2.1 for the
 * data flow: local Q rows against the gathered K/V of the whole packed sequence, K/V
 * gradients leaving the rank as partial sums).
 *
 * The mask is defined per row from q_idx and cu_seqlens_k alone: a row whose global token
 * index g lies in document [s, e) sees keys s..g inclusive.  Rows with q_idx = -1 are
 * padding: their Q/dO content is ignored, O and dQ are written as 0, LSE as -inf, and they
 * add nothing to dK/dV.  Softmax is over scale * <q, k>; LSE is the natural log of the sum
 * of exponentials of the scaled scores.  Query head h uses KV head h / (hq/hkv).
 */
typedef struct {
    int32_t n_q;       /* local query slots (rows of Q/O), >= 1                        */
    int32_t t_kv;      /* tokens in the packed sequence (rows of K/V), >= 1           */
    int32_t n_docs;    /* documents; cu_seqlens_k has n_docs+1 entries, last == t_kv  */
    int32_t hq;        /* query heads                                                 */
    int32_t hkv;       /* KV heads, hq % hkv == 0                                     */
    int32_t head_dim;  /* 64 or 128                                                   */
    float   scale;     /* softmax scale, finite and > 0                               */
    int32_t flags;     /* WLB_ATTN_* bits                                             */
    /* In-document causal (row, key) pairs these rows see, per head -- wlb_shard's useful_pairs for this rank -- or
     * 0 if not known.  It never changes a result: the host only uses it to choose between the two work schedules
     * of the forward and dQ kernels from the real amount of work; without it the choice rests on the mean document
     * length (the host does not see the mask), which misjudges a long document among many tiny ones. */
    int64_t visible_pairs;
} wlb_attn_desc;

enum {
    /* The workspace already holds the schedule that wlb_attn_plan (or an earlier
     * wlb_attn_fwd/bwd without this flag) built for this same desc, q_idx and cu_seqlens_k:
     * skip rebuilding it.  The mask is the same for every layer and for forward and
     * backward, so one schedule serves them all. */
    WLB_ATTN_REUSE_PLAN = 1,
    /* Measurement aids for wlb_attn_bwd, so that one kernel can be timed or profiled alone:
     * reuse the delta the previous backward call left in this workspace; do not run the dQ
     * kernel (dq is left untouched); do not run the dK/dV kernel (dk, dv left untouched). */
    WLB_ATTN_BWD_SKIP_DELTA = 2,
    WLB_ATTN_BWD_SKIP_DQ = 4,
    WLB_ATTN_BWD_SKIP_DKV = 8,
    /* The forward and dQ kernels have two work schedules (see wlb_plan_layout: row_gangs); the
     * library picks one from the shape.  These flags force one of them (tests, measurements). */
    WLB_ATTN_SCHEDULE_GANGS = 32,
    WLB_ATTN_SCHEDULE_ITEMS = 64,
    /* In the one-workgroup-per-item schedule, query tiles whose rows see only a short run of keys
     * (documents of a few dozen tokens: the short-chunk case of Section 5.2) go to kernels that
     * keep that run of K/V in LDS for all query heads of a KV head.  This flag sends every tile
     * through the general kernels instead (tests, measurements). */
    WLB_ATTN_NO_SHORT_PATH = 128
};

/* Bytes of device workspace needed (256-byte aligned pointer expected).  The forward needs
 * fwd_bytes, the backward bwd_bytes >= fwd_bytes; the schedule sits at the start of the
 * workspace in both, so one buffer of bwd_bytes serves plan, forward and backward. */
wlb_status wlb_attn_workspace_size(const wlb_attn_desc* desc, size_t* fwd_bytes, size_t* bwd_bytes);

/* Builds the tile schedule into the workspace (device, asynchronous): per-row key
 * intervals, per-row-group key hulls and fully-visible ranges (so kernels skip cross-document
 * tiles and mask only partial ones), the query-tile and key-tile work lists, both ordered
 * longest first.  Called implicitly by wlb_attn_fwd / wlb_attn_bwd unless WLB_ATTN_REUSE_PLAN
 * is set.  q_idx [n_q] and cu_seqlens_k [n_docs+1] are device pointers.
 * Entries of q_idx must be -1 or in [0, t_kv); others are treated as padding. */
wlb_status wlb_attn_plan(const wlb_attn_desc* desc, const int32_t* q_idx, const int32_t* cu_seqlens_k,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Where the schedule's arrays sit inside the workspace (byte offsets; for inspection and
 * tests).  Row arrays have n_q entries; group arrays n_groups entries of 4 int32
 * {k_lo, k_hi, max_lo, min_hi} per group of group_rows consecutive slots; the work lists are
 * permutations of the query-tile / key-tile indices, heaviest first. */
typedef struct {
    int32_t group_rows, n_groups;
    int32_t fwd_tile_rows, n_fwd_tiles;
    int32_t bwd_key_tile, n_key_tiles;
    size_t  off_row_lo, off_row_hi;      /* int32 [n_q]: visible keys are [lo, hi); pads: lo > hi */
    size_t  off_group;                   /* int32 [n_groups][4] */
    size_t  off_group_real;              /* int32 [n_groups]: real (non-padding, in-range) rows in the group */
    size_t  off_fwd_order;               /* int32 [n_fwd_tiles] */
    size_t  off_fwd_cost;                /* int32 [n_fwd_tiles]: key tiles each query tile visits */
    size_t  off_key_order;               /* int32 [n_key_tiles] */
    size_t  off_key_range;               /* int32 [n_key_tiles][2]: first, one-past-last group that can see the tile */
    /* dK/dV work items: a key tile whose work (groups in its range x query heads of a KV head) exceeds
       a threshold is split by heads into 2, 4 or 8 items that write fp32 partial results; tiles are
       ordered by item cost, heaviest first (off_key_order), and a tile's items are consecutive */
    int32_t dkv_max_items, dkv_max_partials;   /* upper bounds used for the launch and the workspace */
    size_t  off_key_ways;                /* int32 [n_key_tiles]: items per (key tile, KV head), by key tile */
    size_t  off_key_item_base;           /* int32 [n_key_tiles + 1]: first item of the tile of order rank r */
    size_t  off_key_slot_base;           /* int32 [n_key_tiles + 1]: first partial slot of the tile of rank r */
    size_t  off_dkv_counters;            /* int32 [8]: dK/dV items handed out per XCD list; zero between launches */
    /* forward / dQ work: the query tiles in order, each repeated for every KV head, form one line of
       work measured in key tiles (plus a fixed per-tile cost); row_gangs gangs of hq/hkv workgroups
       take consecutive shares of it (the first half of the gangs, whose workgroups run faster, a
       somewhat larger one), so a tile cut by a share's end is finished by the next gang and the
       parts are merged from fp32 partial results */
    int32_t row_gangs;
    int32_t uses_gangs;                  /* 1: forward and dQ of this desc (its flags included) run the gang schedule */
    size_t  off_fwd_prefix;              /* int64 [n_fwd_tiles + 1]: cost of the query tiles before order rank r */
    /* short-hull path: per block of 32 slots the hull {k_lo, k_hi} of the keys its real rows see (k_hi <= k_lo:
       no real row), and per query tile whether each of its blocks' hulls fits the short-hull kernels' LDS window */
    int32_t n_blocks32;
    size_t  off_block_hull;              /* int32 [n_blocks32][2] */
    size_t  off_tile_short;              /* int32 [n_fwd_tiles]: 1 = short-hull tile */
    /* diagnostics of the gang schedule: each workgroup of the forward (k = 0) and dQ (k = 1) gang kernels leaves
       the GPU's constant-rate real-time counter (100 MHz) at its start and at its end, so that a caller can see
       how evenly the gangs finish: uint64 [2][row_gangs * hq / hkv][2], workgroup index as launched */
    size_t  off_gang_clock;
    size_t  plan_bytes;
} wlb_plan_layout;

wlb_status wlb_attn_plan_layout(const wlb_attn_desc* desc, wlb_plan_layout* layout);

/* Weights of the gang schedule's shares (host call, process-wide, takes effect with the next forward / backward
 * call; set it while no call is being issued on another thread).  The gangs of a forward (kernel = 0) or dQ
 * (kernel = 1) launch take shares of the work proportional to weights[half * 8 + xcd]: half = 0 for the first
 * n_gangs / 2 gangs of the launch, 1 for the others; gang g runs on XCD g % 8.  The defaults give the first half
 * a larger share (its workgroups are the older wavefronts of their SIMDs and advance faster) and treat the XCDs
 * alike; the XCDs of one GPU differ in speed by several percent (which ones are slow differs from GPU to GPU),
 * so a caller may measure them -- run its own problem, or any with WLB_ATTN_SCHEDULE_GANGS, read the gangs'
 * clocks at off_gang_clock, and scale the weights of each XCD by mean end time / that XCD's end time; two or
 * three rounds settle.  Weights change where query tiles are cut, i.e. the rounding of the
 * results, never their definition; with fixed weights results stay reproducible bit for bit.
 * weights: host, 16 values in [1, 10^6], or NULL to restore the defaults.  Errors: INVALID_ARG. */
wlb_status wlb_attn_set_gang_weights(int32_t kernel, const int32_t* weights);

/* The weights in force for `kernel` (the defaults if none were set): weights_out: host, 16 values, layout as above.
 * Errors: INVALID_ARG. */
wlb_status wlb_attn_get_gang_weights(int32_t kernel, int32_t* weights_out);

/* Forward.  Device pointers: q [n_q][hq][D], k, v [t_kv][hkv][D] (bf16), q_idx, cu_seqlens_k;
 * outputs o [n_q][hq][D] bf16 and lse [hq][n_q] float are overwritten.
 * Errors: INVALID_ARG (null pointer, bad desc), UNSUPPORTED (head_dim; Q or K of 4 GiB or more,
 * counting 128 rows past the end: the kernels address tensors with 32-bit offsets), BUFFER_TOO_SMALL,
 * HIP (launch failure).  Argument errors are found before anything is enqueued; after a HIP
 * error the stream may already hold the kernels launched before the failing one (the schedule's,
 * unless WLB_ATTN_REUSE_PLAN is set), and the outputs and the workspace are undefined. */
wlb_status wlb_attn_fwd(const wlb_attn_desc* desc, const void* q, const void* k, const void* v,
                        const int32_t* q_idx, const int32_t* cu_seqlens_k,
                        void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same forward as
 * wlb_attn_fwd with its scratch -- the schedule tables -- in a fixed device array of
 * WLB_ATTN_FWD_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process
 * ends) instead of a caller's workspace.  The call allocates nothing and launches the same kernels;
 * it always uses the one-workgroup-per-(query tile, head) schedule, which leaves no partial results.
 * Arguments as wlb_attn_fwd.  flags: WLB_ATTN_REUSE_PLAN means the array still holds the schedule
 * that the previous wlb_attn_fwd_static call on this GPU built for the same desc, q_idx and
 * cu_seqlens_k (every layer of a model shares one mask); WLB_ATTN_SCHEDULE_ITEMS is implied; any
 * other flag is INVALID_ARG.  Nothing in the array has to start at zero: each call without
 * WLB_ATTN_REUSE_PLAN rewrites every table it reads.
 * Limit: UNSUPPORTED when the schedule of (n_q, t_kv) is larger than the array -- it holds about
 * 8.2 bytes per query row and 0.2 bytes per key, so e.g. n_q = t_kv = 131072 (1.1 MiB) fits and
 * n_q above about 240000 does not.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race on it and must be ordered by the caller.  The first call on a GPU looks up the
 * array's address (no allocation); make that call outside graph capture. */
#define WLB_ATTN_FWD_STATIC_SCRATCH_BYTES (2u << 20)
wlb_status wlb_attn_fwd_static(const wlb_attn_desc* desc, const void* q, const void* k, const void* v,
                               const int32_t* q_idx, const int32_t* cu_seqlens_k,
                               void* o, float* lse, void* stream);

/* Backward.  Takes the forward's o and lse plus d_o [n_q][hq][D]; overwrites dq [n_q][hq][D],
 * dk and dv [t_kv][hkv][D] (bf16) with THIS call's rows' contribution (a CP rank's partial;
 * keys no local row can see get 0).  Deterministic: no atomics. */
wlb_status wlb_attn_bwd(const wlb_attn_desc* desc, const void* q, const void* k, const void* v,
                        const void* o, const float* lse, const void* d_o,
                        const int32_t* q_idx, const int32_t* cu_seqlens_k,
                        void* dq, void* dk, void* dv,
                        void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Adaptive sharding selection (Section 5.3): predict the attention forward+backward latency of a
 * micro-batch under per-sequence and under per-document sharding and pick the faster one.
 * Per segment of the sharding map (a rank's run of slots inside one chunk of one document; shape
 * Q_len = slots, KV_len = keys its last row sees): operations = padded pairs * 14 * head_dim * hq,
 * where the rows are cut into tiles of tile_q rows and a tile ending at local row e counts
 * tile_q * roundup(KV_len - Q_len + e, tile_k) pairs; rate = bilinear interpolation of the profiled
 * TFLOP/s table in (Q_len, KV_len), clamped at the grid edges; latency = operations / rate.  A
 * rank's latency is the sum over its segments, a sharding's latency the maximum over ranks.
 * The table comes from profiling this library's kernels offline; all pointers are host memory.
 *
 * wlb_predict_latency: rank_latency [cp] (seconds) for `mode` (a WLB_SHARD_* value).
 * wlb_select_sharding: *mode = WLB_SHARD_PER_DOC_PADDED if its latency is strictly lower, else
 *   WLB_SHARD_PER_SEQ; the two predicted latencies are returned as well.
 * Errors: INVALID_ARG (null pointers, grids not strictly increasing, non-positive rates, and
 * every error of wlb_shard for the same documents / cp / mode).
 */
typedef struct {
    int32_t n_q, n_kv;          /* grid sizes */
    const int32_t* q_len;       /* [n_q]  strictly increasing */
    const int32_t* kv_len;      /* [n_kv] strictly increasing */
    const double* tflops;       /* [n_q][n_kv] achieved TFLOP/s (executed operations / time) */
    int32_t tile_q, tile_k;     /* the kernel's tile: rows per query tile, keys per key tile */
} wlb_kernel_profile;

wlb_status wlb_predict_latency(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t mode, int32_t hq,
                               int32_t head_dim, const wlb_kernel_profile* profile, double* rank_latency);
wlb_status wlb_select_sharding(const int32_t* doc_len, int64_t n_docs, int32_t cp, int32_t hq, int32_t head_dim,
                               const wlb_kernel_profile* profile, int32_t* mode, double* latency_per_seq,
                               double* latency_per_doc);

/* ------------------------------------------------------------------------------------------
 * Measurement aid (not part of the method): one launch of a kernel that issues only dense
 * 32x32x16 bf16 MFMAs on register operands, to measure the MFMA rate the GPU sustains.  The
 * attention kernels are MFMA bound on long documents (Section 5.2 quotes kernel efficiency as
 * achieved TFLOPs); on MI355X the sustained rate depends on the operand values, so
 * random_operands selects all-ones (0) or pseudo-random values in [-1, 1) (1).
 * sink: device, >= 4 bytes, never written in practice.  *flops (host) receives the floating-point
 * operations the launch performs; the caller times the launch on `stream`.  Asynchronous.
 * Errors: INVALID_ARG (null pointer, n_iter outside [1, 2^20]), HIP (launch failure).
 */
wlb_status wlb_calib_mfma(int32_t random_operands, int32_t n_iter, float* sink, double* flops, void* stream);

/* Measurement aid (not part of the method): one launch of a kernel that only adds 64 x 128 fp32 tiles into
 * `buf` with device-scope atomic adds, one workgroup per compute unit, n_iter tiles each -- the traffic a
 * single-kernel backward (Section 6.4 measures forward+backward) would produce for dQ.  shared = 0: every
 * addition of a launch goes to a tile no other workgroup touches at that time (tiles are taken round-robin
 * from buf); shared = 1: the workgroups walk the same few tiles.  buf: device, buf_bytes >= 32 KiB, holds
 * floats that the launch increments.  *bytes_added (host) receives the bytes of fp32 data added; the caller
 * times the launch on `stream`.  Asynchronous.  Errors: INVALID_ARG, HIP. */
wlb_status wlb_calib_atomic_add(int32_t shared, int32_t n_iter, float* buf, size_t buf_bytes, double* bytes_added,
                                void* stream);

#ifdef __cplusplus
}
#endif
#endif /* WLB_H */
