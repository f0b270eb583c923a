/*
 * ep.h -- C ABI of the MI355X expert-parallel dispatch/combine library.
 *
 * One rank's share of MoE dispatch and combine, as the paper's C API states it
 * (Sec. III-B, Table II: CreateGroup / CreateHandle / Dispatch / Combine /
 * HandleGetNumRecvTokens and their Destroy calls), on one GPU: the receive
 * windows of all R ranks are plain regions of this GPU's memory.
 *
 * Conventions (Sec. III-A): every function returns an ep_result_t and never
 * throws; work is enqueued asynchronously on the stream passed in; resources are
 * created and destroyed explicitly; the caller owns every tensor it passes
 * ("pre-allocated receive buffers", Sec. III-B) and must keep it alive until the
 * stream work that uses it has finished.  No entry point takes a PyTorch type.
 *
 * All `data` pointers in ep_tensor_t are DEVICE pointers (or pinned host memory
 * mapped into the device address space) unless a comment says "host".
 * Pointers to config / info / result structs are HOST pointers.
 */
#ifndef EP_MI355X_H
#define EP_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EP_API __attribute__((visibility("default")))

typedef struct ep_group_s *ep_group_t;   /* long-lived: configuration, buffers (Sec. III-C) */
typedef struct ep_handle_s *ep_handle_t; /* one routing decision (Sec. III-C)               */
typedef void *ep_stream_t;               /* a hipStream_t; NULL = the default stream         */

typedef enum {
    EP_SUCCESS = 0,
    EP_ERR_INVALID_ARG = 1,     /* bad pointer, shape, stride, dtype, tag or config value      */
    EP_ERR_INVALID_ROUTING = 2, /* reported by queries when expert ids outside [0,E) were seen */
    EP_ERR_OVERFLOW = 3,        /* rows did not fit the output tensor given to dispatch        */
    EP_ERR_UNSUPPORTED = 4,     /* e.g. send_only != 0, dtype other than bf16                  */
    EP_ERR_BUSY = 5,            /* group destroyed while handles are alive                     */
    EP_ERR_HIP = 6,             /* a HIP runtime call failed                                   */
    EP_ERR_NOMEM = 7,
    EP_ERR_TIMEOUT = 8          /* ep_complete waited for counters that were never published   */
} ep_result_t;

/* Algorithm mode, fixed at group creation (Sec. III-D).  It selects the output
 * layout of dispatch (Sec. III-E "Tensor Layouts"):
 *   EP_MODE_LL  3-D expert-major [E, C, H]: C slots per (expert, source rank)
 *               sub-region; an entry whose slot would be >= C is dropped.
 *   EP_MODE_HT  2-D concatenated [rows, H] with per-expert counts marking the
 *               boundaries; rows of expert e start at expert_offset[e].           */
enum { EP_MODE_LL = 0, EP_MODE_HT = 1 };

/* How dispatch moves rows (Sec. IV-B send phase vs. Sec. IV-D layout optimisation):
 *   EP_PATH_DIRECT      one row copy per (token, selected expert).
 *   EP_PATH_RANK_DEDUP  a token is sent once per destination rank into that
 *                       rank's staging window with its routing vector in the
 *                       message header; the receiving side fans it out to the
 *                       local experts.  Same final windows, bit for bit.          */
enum { EP_PATH_DIRECT = 0, EP_PATH_RANK_DEDUP = 1 };

/* Order in which the direct dispatch walks its work (a tuning knob: every order writes
 * the same bytes to the same places).
 *   EP_ORDER_TOKEN        token by token: a row is read once and stored to its
 *                         destinations.  Insensitive to what the caches hold.  Default.
 *   EP_ORDER_DESTINATION  in the order of the destination rows, for inputs of at least
 *                         8192 routed entries (smaller ones use the token order): rows
 *                         that end up next to each other are written close in time,
 *                         which the memory system rewards.  A read pass over the tokens
 *                         (in pieces of at most 64 MiB) precedes the copy so that the
 *                         copy finds them in the memory-side cache (ep_layout_prefetch
 *                         can do that reading in the shadow of the layout kernels).
 *   EP_ORDER_DESTINATION_RESIDENT  the same without the read pass: for callers whose
 *                         tokens were produced or read just before the call and are at
 *                         most a fraction of the 256 MiB memory-side cache.  When the
 *                         tokens are not resident this order is the slowest of the three. */
enum { EP_ORDER_TOKEN = 0, EP_ORDER_DESTINATION = 1, EP_ORDER_DESTINATION_RESIDENT = 2 };

enum { EP_DTYPE_BF16 = 0, EP_DTYPE_F32 = 1, EP_DTYPE_I32 = 2, EP_DTYPE_U8 = 3,
       EP_DTYPE_FP8_E4M3 = 4 /* OCP E4M3: 1-4-3 bits, bias 7, max 448, no infinity */ };

/* Tensor roles (Sec. III-E, Table IV).  The last three are this library's own. */
enum {
    EP_TAG_NONE = 0,
    EP_TAG_TOKENS = 1,                     /* token data, input or output                 */
    EP_TAG_TOPK_IDX = 2,                   /* int32 [T, K] expert ids, -1 = not routed    */
    EP_TAG_TOPK_WEIGHTS = 3,               /* f32 [T, K] gate weights / f32 [rows] output */
    EP_TAG_SCALES = 4,                     /* f32 [rows, H/128] FP8 scales (dispatch output) */
    EP_TAG_RECV_EXPERT_COUNTER_DEVICE = 5, /* int32 [E] rows placed per expert            */
    EP_TAG_RECV_EXPERT_COUNTER_HOST = 6,   /* same, pinned host memory mapped to device   */
    EP_TAG_TOKENS_PER_EXPERTS = 7,         /* same as RECV_EXPERT_COUNTER_DEVICE          */
    EP_TAG_RECV_SRC_TOKEN = 8,             /* int32 [rows] source token index of each row */
    EP_TAG_EXPERT_BASE = 9,                /* int32 [E], see ep_layout                    */
    EP_TAG_EXPERT_TOKENS = 10              /* expert outputs, shaped like dispatch's TOKENS
                                              output (input of ep_combine_backward)       */
};

/* N-d tensor descriptor (Sec. III-E): shape and strides in ELEMENTS, innermost
 * stride must be 1; rows of bf16 token tensors must start on 16-byte boundaries
 * (data % 16 == 0 and every outer stride % 8 == 0). */
typedef struct {
    void *data;
    int32_t ndim;
    int32_t dtype;
    int32_t tag;
    int32_t reserved;
    int64_t shape[4];
    int64_t stride[4];
} ep_tensor_t;

/* Group configuration (Sec. III-C "MoE Group").  `size` must be sizeof(ep_group_config_t). */
typedef struct {
    uint32_t size;
    int32_t num_ranks;           /* R >= 1                                                 */
    int32_t my_rank;             /* in [0, R)                                              */
    int32_t num_experts;         /* E, multiple of R, <= 1024; expert e lives on rank e/(E/R)
                                    (block-wise placement, Sec. IV-A)                      */
    int32_t hidden;              /* H, bf16 elements per token; 2H must be a multiple of 16 */
    int32_t top_k;               /* K in [1, 64]                                           */
    int32_t max_tokens_per_rank; /* B: upper bound on T of any ep_layout call              */
    int32_t dtype;               /* EP_DTYPE_BF16                                          */
    int32_t mode;                /* EP_MODE_LL / EP_MODE_HT                                */
    int32_t slots_per_subregion; /* C for EP_MODE_LL; 0 = max_tokens_per_rank (Sec. IV-B:
                                    each sub-region holds B slots)                         */
    int32_t dispatch_path;       /* EP_PATH_DIRECT / EP_PATH_RANK_DEDUP                    */
    int32_t max_handles;         /* handle slabs allocated up front; 0 = 2; more are
                                    allocated on demand                                    */
    int32_t staged_buffers;      /* 0: send_only calls are refused; 1 or 2: buffer sets for
                                    staged execution (2 = double buffering, Sec. IV-B): each
                                    set holds the coordination counters, a (t,k)-indexed
                                    combine staging of B*K rows and, on the once-per-rank
                                    path, its own staging windows                          */
    int32_t ranks_per_node;      /* 0 or >= R: combine sums in flat k order; otherwise ranks
                                    d with equal d / ranks_per_node form a node and combine
                                    sums per node first, then across nodes (the HT
                                    "hierarchical" reduction of Sec. III-D / V-A)          */
    int32_t dispatch_order;      /* EP_ORDER_TOKEN / EP_ORDER_DESTINATION /
                                    EP_ORDER_DESTINATION_RESIDENT (EP_PATH_DIRECT only)     */
    int32_t quantize_ahead;      /* 0, or 1 (needs EP_ORDER_DESTINATION, EP_PATH_DIRECT and
                                    H % 128 == 0): ep_layout_prefetch does not only read the
                                    announced tokens, it also quantises them to FP8 -- the
                                    format of the quantising ep_dispatch -- into a staging
                                    copy kept with the handle (max_tokens_per_rank *
                                    (H + H/32) bytes per handle), on the compute units the
                                    layout leaves idle.  The handle's first ep_dispatch, when
                                    it is a quantising one of that tensor (same address and
                                    row stride), copies the staged rows in destination order
                                    instead of quantising in token order: same codes, same
                                    scales.  The tokens must not change between the two
                                    calls; every later dispatch quantises for itself.  Inputs too small for the destination order are
                                    quantised by the dispatch as usual.  (Sec. I: dispatch
                                    may quantise; Sec. IV-C: work next to the send.)       */
} ep_group_config_t;

/* Allocator callbacks (Sec. III-C): when given, every device allocation of the
 * group goes through them.  Return 0 on success; the memory must be device memory
 * aligned to 256 bytes (ep_group_create / ep_layout fail with EP_ERR_INVALID_ARG
 * otherwise and hand the block back through the free callback). */
typedef int (*ep_alloc_fn)(void **ptr, size_t bytes);
typedef int (*ep_free_fn)(void *ptr);

typedef struct {
    int32_t num_ranks, my_rank, num_experts, experts_per_rank, hidden, top_k;
    int32_t max_tokens_per_rank, mode, slots_per_subregion, dispatch_path;
    int64_t row_bytes;            /* 2H                                                    */
    int64_t msg_header_bytes;     /* staging message header: 4 + 8K rounded up to 16       */
    int64_t msg_bytes;            /* header + 2H                                           */
    int64_t staging_slots;        /* message slots in the staging windows (0 if DIRECT)    */
    void *staging;                /* device pointer to the staging windows (borrowed)      */
    /* Communication-buffer footprints of Sec. IV-D for this configuration, in bytes,
     * with slot size P = 2H: per-expert sub-regions 2*E*B*P versus the optimised
     * scheme R*B*P (dispatch) + B*K*P (combine). */
    int64_t footprint_per_expert_bytes;
    int64_t footprint_optimised_bytes;
    int32_t live_handles;
    int32_t staged_buffers;
    /* per buffer set (borrowed device pointers, NULL when absent): staging windows,
     * coordination counters int32 [E dispatch | R once-per-rank | E combine], and the
     * combine staging bf16 [B*K, H] */
    void *staging_sets[2];
    void *signals[2];
    void *combine_staging[2];
    /* Staging slot s occupies bytes [s * msg_stride, (s+1) * msg_stride) of a staging window
     * set; its message (msg_bytes: header, then token data) starts msg_lead bytes in, which
     * puts the token data on a 256-byte boundary.  The other bytes of a slot are never
     * written. */
    int64_t msg_stride;
    int64_t msg_lead;
    /* Padded windows with EP_ORDER_DESTINATION*: rows kept and rows cut by the capacity in the
     * most recent layout of the group that has FINISHED on the device (0, 0 before the first,
     * and for every other kind of group).  The layout kernel leaves the pair in host memory
     * and ep_dispatch reads it as a hint, without waiting for anything: when more than a
     * third of the routed entries were cut, it walks the tokens instead of the destination
     * rows (the rows that survive then sit in a few long runs, which the token walk copies
     * faster).  Both walks write the same bytes; the hint changes time only. */
    int32_t hint_rows_kept;
    int32_t hint_rows_dropped;
} ep_group_info_t;

/* Result of a layout, host-side copy of the totals plus borrowed DEVICE pointers
 * to the arrays held by the handle (valid until ep_handle_destroy). */
typedef struct {
    int32_t num_tokens;      /* T of this layout                                           */
    int32_t status;          /* bit 0: ids outside [0,E) seen; bit 1: entries dropped for
                                capacity; bit 2: a dispatch found rows beyond its output;
                                bit 3: a bounded device-side wait ran out (ep_complete waiting
                                for counters, or the workgroups of a layout for each other).
                                Bits 2 and 3 stay set for the lifetime of the handle once a
                                call has raised them                                       */
    int64_t rows_kept;       /* routed entries that own a destination row                  */
    int64_t rows_dropped;    /* entries cut by the LL capacity C                           */
    int64_t entries_masked;  /* topk_idx == -1                                             */
    int64_t entries_invalid; /* other ids outside [0, E)                                   */
    int64_t entries_sorted;  /* rows_kept + rows_dropped                                   */
    int64_t rank_messages;   /* (token, destination rank) pairs                            */
    int64_t rows_end;        /* one past the highest destination row = expert_offset[E]    */
    const int32_t *expert_count;     /* [E]   demand per expert                            */
    const int32_t *expert_kept;      /* [E]   rows placed per expert                       */
    const int32_t *expert_offset;    /* [E+1] first row of each expert                     */
    const int32_t *rank_pair_count;  /* [R]   entries per destination rank                 */
    const int32_t *rank_token_count; /* [R]   tokens per destination rank, each once       */
    const int32_t *rank_offset;      /* [R+1] first staging slot of each destination rank  */
    const int32_t *slot;             /* [T,K] index among entries naming the same expert   */
    const int32_t *dst_row;          /* [T,K] destination row, -1 if none                  */
    const int32_t *rank_row;         /* [T,K] staging slot for the first k naming a rank   */
    const int32_t *sorted_token;     /* [entries_sorted] token of each entry in (expert,
                                        slot) order                                        */
    const int32_t *sorted_k;         /* [entries_sorted] its k                             */
    const int32_t *sorted_row;       /* [entries_sorted] its destination row or -1         */
    const int32_t *entry_rank;       /* [T,K] destination rank of the entry, -1 = not routed */
} ep_layout_info_t;

EP_API const char *ep_error_string(ep_result_t code);

/* Library version, major*10000 + minor*100 + patch. */
EP_API int32_t ep_version(void);

/* Identifies the sources and compiler flags this library was built from (16 hex digits
 * computed by the build script; "unknown" for a build that bypassed it).  Benchmarks print
 * it so that a number can be tied to the code that produced it. */
EP_API const char *ep_build_id(void);

/*
 * Diagnostic: how ep_layout would cut `num_entries` = T*K routing entries into wave-chunks
 * (64 * passes consecutive entries per wavefront).  Host-only, no GPU needed.
 * Errors: EP_ERR_INVALID_ARG (NULL pointers, negative count).
 */
EP_API ep_result_t ep_layout_plan(int64_t num_entries, int32_t *passes, int32_t *wave_chunks);

/* Diagnostic: how the direct dispatch of a group configured like `cfg` would walk an input
 * of `num_tokens` tokens, `prefetched_rows` of which ep_layout_prefetch has already read.
 * Pure host arithmetic (no device is touched); the same function plans the real launches. */
typedef struct {
    int32_t run_order;          /* 1: destination order; 0: token order, the rest is 0       */
    int32_t group;              /* wave-chunks of the layout per block                       */
    int32_t blocks;             /* blocks the input is cut into                              */
    int32_t block_entries;      /* routed entries per block                                  */
    int32_t splits;             /* workgroups that share the run of one (block, expert)      */
    int32_t slice_units;        /* 16-byte units of a row per slice (8 slices per row)       */
    int32_t threads_per_piece;  /* threads that copy one row piece                           */
    int32_t blocks_per_launch;  /* blocks per copy launch                                    */
    int32_t launches;           /* copy launches                                             */
    int32_t read_passes;        /* token read passes (at most one per copy launch)           */
} ep_dispatch_plan_t;
EP_API ep_result_t ep_dispatch_plan(const ep_group_config_t *cfg, int64_t num_tokens, int64_t prefetched_rows,
                             ep_dispatch_plan_t *plan);

/* Diagnostic: how ep_combine of a group configured like `cfg` would cut `num_tokens` tokens into
 * wavefronts on a GPU of `compute_units` compute units (0 = unknown).  A wavefront reduces one
 * 1 KiB segment of a token row, two adjacent ones in long launches, or -- rows of 14 336 bytes
 * (Sec. IV-B) whose tokens fill whole rounds of the GPU's resident wavefronts -- the whole row.
 * Pure host arithmetic; the same function plans the real launches with the device's count.
 * Errors: EP_ERR_INVALID_ARG. */
typedef struct {
    int32_t segments_per_wavefront; /* 1, 2 or 14                                             */
    int32_t whole_row;              /* 1: one wavefront per token                             */
    int64_t workgroups;             /* workgroups of 4 wavefronts in the launch               */
} ep_combine_plan_t;
EP_API ep_result_t ep_combine_plan(const ep_group_config_t *cfg, int64_t num_tokens, int32_t compute_units,
                            ep_combine_plan_t *plan);

/*
 * Measurement aid, not part of the paper's API: a plain streaming copy of `bytes`
 * (multiple of 16; dst and src 16-byte aligned DEVICE pointers, not overlapping)
 * with the same 16-byte-per-lane accesses the row kernels use.  It is what the
 * hardware byte counters and "achievable copy bandwidth" are calibrated against.
 * Errors: EP_ERR_INVALID_ARG, EP_ERR_HIP.
 */
EP_API ep_result_t ep_calibration_copy(void *dst, const void *src, size_t bytes, ep_stream_t stream);

/*
 * Measurement aids like ep_calibration_copy, for the two directions on their own: dispatch
 * mostly writes (K rows written per token read) and combine mostly reads, so each is
 * bounded by what the memory sustains in that direction, which differs from the mixed copy.
 * ep_calibration_fill writes `bytes` (multiple of 16) of the bf16 value 1.0 to the 16-byte
 * aligned DEVICE pointer dst.  ep_calibration_read reads `bytes` from the 16-byte aligned
 * DEVICE pointer src and folds them into a checksum; `sink` is a DEVICE pointer to 4
 * writable bytes that the kernel writes only when a lane's checksum equals one fixed
 * constant (it exists so that the reads cannot be optimised away; its content means nothing).
 * Errors: EP_ERR_INVALID_ARG, EP_ERR_HIP.
 */
EP_API ep_result_t ep_calibration_fill(void *dst, size_t bytes, ep_stream_t stream);
EP_API ep_result_t ep_calibration_read(const void *src, size_t bytes, void *sink, ep_stream_t stream);

/*
 * ep_group_create -- Table II "ncclEpCreateGroup" without the communicator.
 * Validates cfg, computes the window geometry and allocates (through alloc_fn or
 * hipMalloc) the handle slabs and, for EP_PATH_RANK_DEDUP, the staging windows:
 * R*B message slots in LL mode, B*min(R,K) in HT mode.  Host-synchronous; may be
 * called on any thread with the target device current.
 * Errors: EP_ERR_INVALID_ARG (NULL pointers, size mismatch, E % R != 0, 2H % 16
 * != 0, limits exceeded), EP_ERR_UNSUPPORTED (dtype), EP_ERR_NOMEM, EP_ERR_HIP.
 */
EP_API ep_result_t ep_group_create(ep_group_t *group, const ep_group_config_t *cfg, ep_stream_t stream,
                            ep_alloc_fn alloc_fn, ep_free_fn free_fn);

/* Table II "ncclEpGroupDestroy".  Fails with EP_ERR_BUSY while handles are alive.
 * Before freeing it waits (on the host) for `stream` and for the streams the last calls of
 * the group's destroyed handles were given. */
EP_API ep_result_t ep_group_destroy(ep_group_t group, ep_stream_t stream);

/* Geometry and footprints of a group (host struct filled synchronously). */
EP_API ep_result_t ep_group_query(ep_group_t group, ep_group_info_t *info);

/*
 * ep_layout -- Table II "ncclEpCreateHandle": captures one routing decision.
 * topk_idx: int32 [T, K], tag EP_TAG_TOPK_IDX, T <= max_tokens_per_rank, entries in
 * [0, E) or -1.  Runs on `stream`: per-expert and per-destination-rank counts,
 * prefix offsets, and the stable slot map -- slot(t,k) = number of entries before
 * (t,k) in flattened t*K+k order that name the same expert, i.e. the "next unused
 * index" of Sec. IV-B made deterministic: (source rank, token index) order.
 * expert_base (optional, may be NULL): int32 [E] device array, HT mode only; row
 * at which this source's rows of expert e start in the receiver's tensor (what the
 * handle-time metadata exchange of Sec. III-C would deliver).  NULL = exclusive
 * prefix sum of this source's own counts.
 * The handle is read-only afterwards and may serve any number of dispatch/combine
 * calls (forward and backward reuse, Sec. III-C).  Takes a slab from the group's
 * pool; allocates only if the pool is exhausted.
 * Errors: EP_ERR_INVALID_ARG, EP_ERR_NOMEM, EP_ERR_HIP.  Bad expert ids are found
 * on the device and reported by ep_handle_query.
 */
EP_API ep_result_t ep_layout(ep_handle_t *handle, ep_group_t group, const ep_tensor_t *topk_idx,
                      const ep_tensor_t *expert_base, ep_stream_t stream);

/*
 * ep_layout with a hint: `tokens` is the bf16 [T, H] tensor (tag EP_TAG_TOKENS, rows on
 * 16-byte boundaries) that the caller is going to hand to ep_dispatch next.  The layout
 * kernels keep only a few compute units busy; for a group whose dispatch_order is
 * EP_ORDER_DESTINATION and an input of at least 8192 routed entries, the same launch
 * therefore also reads the tokens (the first 64 MiB of them) into the memory-side cache
 * on the idle units, and the first ep_dispatch of the handle, when it is given the same
 * tensor (data pointer and row stride), leaves out its own read pass over those rows.  In every other case the
 * hint is ignored.  The handle, its arrays and all results are those of ep_layout.
 */
EP_API ep_result_t ep_layout_prefetch(ep_handle_t *handle, ep_group_t group, const ep_tensor_t *topk_idx,
                               const ep_tensor_t *expert_base, const ep_tensor_t *tokens,
                               ep_stream_t stream);

/* Output arrays of ep_layout_static: DEVICE pointers to int32 arrays the caller owns.
 * `size` must be sizeof(ep_layout_arrays_t).  Meanings as in ep_layout_info_t. */
typedef struct {
    uint32_t size;
    uint32_t reserved;
    int32_t *totals;           /* [16] required: rows_kept, rows_dropped, entries_masked,
                                  entries_invalid, entries_sorted, rank_messages, status,
                                  rows_end, then 8 unused words                            */
    int32_t *expert_count;     /* [E]   required                                           */
    int32_t *expert_kept;      /* [E]   required                                           */
    int32_t *expert_offset;    /* [E+1] required                                           */
    int32_t *rank_pair_count;  /* [R]   required                                           */
    int32_t *rank_token_count; /* [R]   required                                           */
    int32_t *rank_offset;      /* [R+1] required                                           */
    int32_t *dst_row;          /* [T,K] required when T > 0                                */
    int32_t *slot;             /* [T,K] optional (NULL = not wanted)                       */
    int32_t *rank_row;         /* [T,K] optional                                           */
    int32_t *entry_rank;       /* [T,K] optional                                           */
    int32_t *sorted_token;     /* [T*K] optional; the three sorted arrays come together    */
    int32_t *sorted_k;         /* [T*K]                                                    */
    int32_t *sorted_row;       /* [T*K]                                                    */
} ep_layout_arrays_t;

/*
 * ep_layout_static -- ep_layout for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  It creates no group and
 * no handle and calls no allocating routine, on the host or on the device: the
 * configuration comes in as the plain struct (validated like ep_group_create does; only
 * num_ranks, num_experts, top_k, max_tokens_per_rank, mode and slots_per_subregion matter
 * here), the results go to arrays the caller passes in `out`, and the kernels' own working
 * memory -- the per-chunk bin sums ep_layout keeps in its handle -- is a fixed array of
 * 2.1 MB inside the library image, one copy per GPU, held until the process ends.  That array
 * is sized for the limits of ep_group_create (1024 experts, hence at most 2050 bins,
 * 256 chunks, 2^28 entries); a configuration beyond them is refused with
 * EP_ERR_INVALID_ARG.
 * Same kernels, same results as ep_layout, array for array (ep_handle_query of an ep_layout
 * handle is what `out` is compared with).  All calls on one GPU share the one scratch
 * array: calls that may overlap in time on one GPU (different streams, or different
 * threads) race and must be serialised by the caller; calls on one stream are safe.  The array
 * is zero when the library is loaded and every launch leaves it ready for the next one.
 * topk_idx and expert_base as for ep_layout.  Errors: EP_ERR_INVALID_ARG,
 * EP_ERR_UNSUPPORTED, EP_ERR_HIP.
 */
EP_API ep_result_t ep_layout_static(const ep_group_config_t *cfg, const ep_tensor_t *topk_idx,
                                    const ep_tensor_t *expert_base, const ep_layout_arrays_t *out,
                                    ep_stream_t stream);

/* Synchronises the handle's last stream and fills `info`.  Returns
 * EP_ERR_INVALID_ROUTING if bad expert ids were seen and EP_ERR_OVERFLOW if a
 * dispatch ran out of output rows (info is filled in both cases); capacity drops
 * in LL mode are reported in info->status / rows_dropped only. */
EP_API ep_result_t ep_handle_query(ep_handle_t handle, ep_layout_info_t *info);

/* Table II "ncclEpHandleGetNumRecvTokens": rows this source places in the
 * receivers' tensors (rows_kept).  Synchronises like ep_handle_query. */
EP_API ep_result_t ep_handle_get_num_recv_tokens(ep_handle_t handle, int64_t *num);

/* Table II "ncclEpHandleDestroy".  Host-only and immediate: the handle's device arrays return
 * to the group's pool and the next ep_layout may take them.  Work of this handle that is still
 * queued stays safe: the library remembers the stream of the handle's last call, and a later
 * ep_layout on another stream first makes that stream wait (on the device, through an event)
 * for everything queued there; a later ep_layout on the same stream is ordered by the stream.
 * What the caller must see to: calls of one handle on several streams must have been ordered
 * among themselves so that the last call's stream comes after the others (as data dependencies
 * between dispatch and combine require anyway).  A staged call that was never completed is
 * abandoned: its coordination counters are cleared on the stream of its send phase. */
EP_API ep_result_t ep_handle_destroy(ep_handle_t handle);

/*
 * ep_dispatch -- Table II "ncclEpDispatch" (Sec. III-B; data movement of Sec. IV-B/C,
 * or Sec. IV-D when the group was created with EP_PATH_RANK_DEDUP).
 * inputs (by tag):  TOKENS x [T, H] bf16 (required);
 *                   TOPK_WEIGHTS w [T, K] f32 (optional, forwarded per row);
 *                   TOPK_IDX [T, K] int32, the tensor the handle was built from
 *                     (required for EP_PATH_RANK_DEDUP: it fills the message headers).
 * outputs (by tag): TOKENS (required) -- HT: [rows_cap, H]; LL: [E, C, H], possibly a
 *                     strided view of a larger receiver tensor [E, R*C, H];
 *                   TOPK_WEIGHTS recv_w [rows_cap] f32 (optional; LL: [E*C]);
 *                   RECV_SRC_TOKEN recv_src [rows_cap] int32 (optional);
 *                   RECV_EXPERT_COUNTER_DEVICE / _HOST / TOKENS_PER_EXPERTS [E] int32
 *                     (optional): rows placed per expert.
 * For every (t,k) with dst_row >= 0: recv_x[dst_row] = x[t] (byte copy),
 * recv_w[dst_row] = w[t,k] (1.0 when no TOPK_WEIGHTS input is given: absent weights mean a
 * plain sum, Sec. III-B), recv_src[dst_row] = t.  Rows not named by the layout are
 * left untouched.  A row index >= rows_cap is skipped and flagged (status bit 2).
 * send_only = 1 (staged execution, Sec. III-B; needs staged_buffers > 0, else
 * EP_ERR_UNSUPPORTED; a handle can have one staged call pending, else EP_ERR_BUSY): only
 * the send phase runs -- rows (or once-per-rank messages) are written and the
 * coordination counters are raised to count + 1 (Sec. IV-B) -- and the call is finished
 * by ep_complete, which also delivers the per-expert counter output.  The output
 * tensors must stay valid until then.
 * Quantising dispatch (Sec. I "in-kernel quantization", Sec. IV-B payload: H bytes of FP8
 * plus H/128 float scales per row): give the TOKENS output the dtype EP_DTYPE_FP8_E4M3
 * (same shape rules, one byte per element, outer strides multiples of 16) together with a
 * SCALES output f32 [rows_cap, H/128] (contiguous; LL: rows_cap = E*C).  Requires
 * H % 128 == 0 and EP_PATH_DIRECT.  Per token and group of 128 channels:
 * amax = max|x|; scales[row, g] = amax / 448; q = e4m3(f32(x) * (448 / amax)), float32
 * operations, round to nearest even, magnitudes above 448 saturate; amax == 0 gives scale 1.
 * The quantising dispatch walks the tokens whatever the group's dispatch_order, except in a
 * group with quantize_ahead, after an ep_layout_prefetch that announced the same tokens.
 * EP_PATH_RANK_DEDUP runs three steps on the stream -- send to the group's staging
 * windows, receiver-side ranking of the header entries, fan-out -- and produces the
 * same outputs; dispatches of one group must then not overlap (they share the
 * staging windows).  An expert_base given to ep_layout must stay valid until then.
 */
EP_API ep_result_t ep_dispatch(ep_handle_t handle, const ep_tensor_t *inputs, int32_t num_inputs,
                        const ep_tensor_t *outputs, int32_t num_outputs, int32_t send_only,
                        ep_stream_t stream);

/*
 * ep_combine -- Table II "ncclEpCombine" (Sec. III-B; reduction of Sec. IV-B/C
 * "Combine/recv", addressing of Sec. IV-D).
 * inputs:  TOKENS y with exactly the shape rules of dispatch's TOKENS output
 *          (Sec. III-E: combine input = dispatch output); TOPK_WEIGHTS w [T, K] f32
 *          (optional; absent = plain sum).
 * outputs: TOKENS out [T, H] bf16.
 * out[t,h] = bf16_rne( sum over k = 0..K-1 in that order of w[t,k] * f32(y[dst_row[t,k], h]) )
 * with float32 multiply and float32 add, each rounded to nearest even; entries
 * without a destination row contribute nothing.  With ranks_per_node set (see the group
 * configuration) the same products are summed per node in ascending k and the node sums
 * are then added in ascending node order, still in float32 with one final rounding.
 * send_only = 1: the expert side packs the rows into the group's staging at slot
 * t*K + k (Sec. IV-D) and raises the combine counters to 1; ep_complete waits for them
 * and reduces from the staging into `out` (same arithmetic, same result).
 */
EP_API ep_result_t ep_combine(ep_handle_t handle, const ep_tensor_t *inputs, int32_t num_inputs,
                       const ep_tensor_t *outputs, int32_t num_outputs, int32_t send_only,
                       ep_stream_t stream);

/*
 * ep_layout_dispatch -- ep_layout (Table II "ncclEpCreateHandle") and ep_dispatch of the
 * tokens it was made for, in one call.  In the paper's low-latency kernels the token count
 * runs next to the send (Sec. IV-C); here an input of at most 1024 routed entries on the
 * direct path with bf16 rows is laid out and dispatched by ONE kernel launch: every
 * workgroup derives the layout from the few KB of ids in its own LDS and copies its share
 * of the rows, one workgroup also writes the handle's arrays.  Any other input runs the two
 * calls one after the other (the layout with the tokens announced, as ep_layout_prefetch
 * does).  Arguments, outputs, results and errors are those of ep_layout and ep_dispatch
 * (send_only = 0); on an error no handle is returned.
 */
EP_API ep_result_t ep_layout_dispatch(ep_handle_t *handle, ep_group_t group, const ep_tensor_t *topk_idx,
                                      const ep_tensor_t *expert_base, const ep_tensor_t *inputs,
                                      int32_t num_inputs, const ep_tensor_t *outputs, int32_t num_outputs,
                                      ep_stream_t stream);

/*
 * ep_combine_backward -- the backward pass of ep_combine with the handle of the forward pass
 * (Sec. III-C: a handle serves forward and backward; Sec. III-F training pattern, where the
 * backward of combine is a dispatch of the gradients).  For out[t] = sum_k w[t,k] * y[row(t,k)]
 * and g the gradient with respect to out:
 * inputs:  TOKENS g [T, H] bf16 (required); TOPK_WEIGHTS w [T, K] f32 (optional, absent = 1);
 *          EXPERT_TOKENS y with the shape rules of dispatch's TOKENS output (optional; needed for
 *          the weight gradient).
 * outputs: TOKENS grad_y, shaped like y / like dispatch's TOKENS output (required):
 *            grad_y[row(t,k), h] = bf16_rne( w[t,k] * f32(g[t,h]) ), other rows untouched;
 *          TOPK_WEIGHTS grad_w [T, K] f32 (given exactly when y is):
 *            grad_w[t,k] = sum over h of f32(y[row(t,k), h]) * f32(g[t,h]) in float32, in a fixed
 *            order (per thread of a 256-thread workgroup over its 16-byte units, a fixed tree over
 *            the lanes, the four waves in order); 0 for an entry without a row.
 * The backward pass of ep_dispatch needs no call of its own: it is ep_combine without weights.
 * Errors: EP_ERR_INVALID_ARG, EP_ERR_UNSUPPORTED, EP_ERR_HIP.
 */
EP_API ep_result_t ep_combine_backward(ep_handle_t handle, const ep_tensor_t *inputs, int32_t num_inputs,
                                       const ep_tensor_t *outputs, int32_t num_outputs, ep_stream_t stream);

/* Options of ep_complete.  `size` must be sizeof(ep_complete_config_t). */
typedef struct {
    uint32_t size;
    int32_t spin_limit; /* polls per counter before giving up; 0 = 1 << 20 */
} ep_complete_config_t;

/*
 * ep_complete -- Table II "ncclEpComplete": the receive phase of the staged call pending
 * on `handle` (Sec. III-B, Sec. IV-B receive phase).  Enqueues on `stream` (which may
 * differ from the stream of the send phase) a bounded wait until every coordination
 * counter of the call is non-zero, takes the counts from them, clears them, and then
 *   dispatch, direct path:   writes the per-expert counter output given to ep_dispatch;
 *   dispatch, once per rank: ranks the header entries of the staged messages and fans
 *                            them out to the expert rows;
 *   combine:                 reduces from the (t,k)-indexed staging into `out`.
 * cfg may be NULL.  Errors: EP_ERR_INVALID_ARG (no pending call, bad cfg), EP_ERR_HIP.
 * A wait that runs out sets status bit 3; ep_handle_query then returns EP_ERR_TIMEOUT
 * and counts of counters that never arrived read as 0.
 */
EP_API ep_result_t ep_complete(ep_handle_t handle, const ep_complete_config_t *cfg, ep_stream_t stream);

/* Clears every coordination counter of the group (e.g. after an abandoned staged call). */
EP_API ep_result_t ep_group_reset_signals(ep_group_t group, ep_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* EP_MI355X_H */
