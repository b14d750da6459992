/* vps.h - C ABI of the MI355X Virtual Parameter Space state-transition engine.
 *
 * The library implements the data path of a parallelism switch as described in the DynaTrain
 * paper: every training-state tensor exists once in a global logical coordinate space (the
 * VPS, Section 4.1); a parallel configuration P maps each rank to a region of that space
 * (F_P, Section 4.1); a switch from configuration A to B is the set of intersections between
 * source and destination regions (Section 4.2.1), including ZeRO flat-buffer shards mapped
 * back into the same space (Section 4.2.2); outgoing slices are packed into one contiguous
 * buffer per peer, exchanged, and unpacked into the new local layout (Algorithm 1, PackData and
 * UnpackData; Section 4.3 "Memory-Aware Contiguous Buffer").
 *
 * All mapping, planning and copying runs in HIP kernels on the current device.  The library
 * never allocates payload memory: state buffers, send/receive buffers and scratch are owned
 * by the caller (device memory), and must stay alive until the stream has executed the work.
 * Its own tables (piece, box, descriptor and tile tables) come from a process-wide pool of
 * device blocks on the device that is current at the call; a process uses the library with
 * one device current throughout (handles made on one device are not usable on another).
 * Calls are thread-safe on distinct handles; a plan may be used by one thread at a time.
 *
 * Conventions
 *   state kinds     0 = bf16 parameters (2-byte words), 1 = fp32 master weights,
 *                   2 = fp32 Adam m, 3 = fp32 Adam v (4-byte words).  Payload is opaque.
 *   local buffers   every rank has 8 buffers, index = group*4 + kind; group 0 = dense
 *                   tensors, group 1 = expert tensors.  Empty buffers have 0 bytes.
 *   flat layout     per (rank, group) the local tensor shards are concatenated in tensor-id
 *                   order without gaps and the tail is padded to a multiple of 8*D elements
 *                   (D = data-parallel group size).  Kind 0 holds the whole padded buffer;
 *                   kinds 1..3 hold the rank's 1/D range when zero_stage = 1.
 *   ranks           ep_placement 0: rank = tp + TP*(ddp + DDP*pp), ddp = ep + EP*edp, DDP = EP*DP.
 *                   ep_placement 1: rank = tp + TP*(dp + DP*pp) for dense tensors; for expert
 *                   tensors the position q = tp + TP*dp inside the stage gives ep = q mod EP and
 *                   the expert data-parallel index q div EP (see vps_parallel_desc).
 *   limits          at most 32768 ranks per configuration and 2^24 logical tensors; fewer than
 *                   2^31 pieces, boxes and tiles per table (VPS_ERR_OOM beyond); an all-ranks
 *                   plan keeps a src x dst byte matrix and is refused above 2^26 rank pairs;
 *                   tensor axes are 31-bit, offsets and strides 64-bit.
 *   return values   0 on success, a negative vps_status otherwise; vps_last_error() returns
 *                   a thread-local message.  Functions never throw.  On error no device work
 *                   has been enqueued.
 *   synchronisation which calls wait for the device, and how often:
 *                   vps_describe_config          never (one kernel on the null stream)
 *                   vps_plan_intersections[_ex]  once, for the counts and byte totals the host
 *                                                needs; twice when the tile table has to be
 *                                                built after that wait (the first plan of a
 *                                                (model, configurations, rank, flags, tile size)
 *                                                combination in the process; later plans of the
 *                                                same combination size the table from the first
 *                                                one's counts) and for plans above
 *                                                VPS_OPT_SMALL_PLAN_BOXES boxes
 *                   vps_pack, vps_unpack, vps_apply_transition[_static|_staged], vps_plain_*
 *                                                never
 *                   vps_stage_exchange, vps_plan_classify_collectives
 *                                                their stream, once or twice
 *                   vps_plan_get_boxes, vps_plan_peer_segment, vps_config_buffer_bytes,
 *                   vps_config_num_pieces, vps_config_get_pieces
 *                                                once, on first use (they fetch or build
 *                                                tables that planning itself does not need)
 *                   other queries                never
 *                   vps_plan_destroy, vps_stage_plan_destroy
 *                                                the streams the plan was used on (its tables
 *                                                go back to the pool)
 */
#ifndef VPS_H
#define VPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum vps_status {
    VPS_OK = 0,
    VPS_ERR_INVALID_ARG = -1,
    VPS_ERR_INDIVISIBLE = -2,      /* a parallel degree does not divide the axis it shards */
    VPS_ERR_RANK_RANGE = -3,
    VPS_ERR_MODEL_MISMATCH = -4,   /* the two configurations describe different models */
    VPS_ERR_SCRATCH_TOO_SMALL = -5,
    VPS_ERR_OOM = -6,
    VPS_ERR_HIP = -7               /* a HIP call failed (no device, launch error, ...) */
} vps_status;

enum { VPS_FAMILY_GPT = 0, VPS_FAMILY_GQA = 1, VPS_FAMILY_MOE = 2 };
enum { VPS_NUM_KINDS = 4, VPS_NUM_BUFFERS = 8 };

/* Model shape.  The tensor inventory follows from the family:
 *   GPT  per layer ln1.w ln1.b qkv.w qkv.b proj.w proj.b ln2.w ln2.b fc1.w fc1.b fc2.w fc2.b
 *   GQA  per layer in_norm qkv.w o.w post_norm gate_up.w down.w
 *   MOE  per layer in_norm qkv.w q_norm k_norm o.w post_norm router.w, then per expert
 *        gate_up.w down.w
 * preceded by the word embedding and followed by the final norm(s) and the output layer.
 * Tensor ids ascend in that order. */
typedef struct vps_model_desc {
    int32_t family, layers, hidden, q_heads, kv_heads, head_dim, ffn, vocab, experts, expert_ffn;
} vps_model_desc;

/* Parallel configuration.  With ep_placement = 0 the world size is tp*pp*dp*ep, dp is the
 * data-parallel degree of the expert group and dense tensors are replicated over dp*ep ranks. */
typedef struct vps_parallel_desc {
    int32_t tp, pp, dp, ep;
    int32_t zero_stage;    /* 0 or 1 */
    int32_t gpus_per_node; /* used by the replica source rule */
    int32_t qkv_layout;    /* 0 interleaved per kv group, 1 blocked [all Q | all K | all V] */
    int32_t expert_layout; /* 0 row-major, 1 transposed storage (gate_up as (h,2,f), down as (f,h)) */
    int32_t flat_order;    /* 0 ascending tensor id, 1 descending */
    int32_t ep_placement;  /* 0: EP and expert-DP form a grid beside TP: world = tp*pp*dp*ep, experts
                              are TP-sharded like the dense MLP, dp = expert data-parallel degree.
                              1: EP is carved out of the tp*dp ranks of a pipeline stage (the form
                              of the paper's (TP, PP, DP, EP) MoE tuples): world = tp*pp*dp, position
                              q = tp + tp_degree*dp_index in the stage has ep = q mod EP and expert
                              data-parallel index q div EP; experts are not TP-sharded; ep must
                              divide tp*dp */
} vps_parallel_desc;

typedef struct vps_config vps_config; /* a configuration mapped onto the VPS (device tables) */
typedef struct vps_plan vps_plan;     /* the routing plan of one transition (device tables) */

/* One piece of a rank's region: an axis-aligned box of one logical tensor that is stored as a
 * strided block of one local buffer (Section 4.1, sub-VPS: resident regions with their local
 * partition attributes). */
typedef struct vps_piece {
    int32_t tensor, rank, kind, buf;
    int32_t lo[4], ext[4]; /* box in global coordinates (4-D, leading axes of extent 1) */
    int64_t off;           /* element offset of the lo corner in the local buffer */
    int64_t stride[4];     /* elements per unit step along each global axis */
} vps_piece;

/* One routed sub-box: the intersection of a source piece with a destination piece for which
 * the source rank is the selected owner (Section 4.2.1; a retain entry when src_rank ==
 * dst_rank).  send_pos/recv_pos are byte offsets of its payload (row-major in global axis
 * order, 16-byte aligned) in the source rank's send buffer and the destination rank's
 * receive buffer; both are UINT64_MAX for retained boxes or non-resident sides. */
typedef struct vps_box {
    int32_t tensor, kind, src_rank, dst_rank, src_buf, dst_buf;
    int32_t lo[4], ext[4];
    int64_t src_off, dst_off;             /* element offsets of the lo corner */
    int64_t src_stride[4], dst_stride[4]; /* element strides per global axis */
    uint64_t send_pos, recv_pos;
} vps_box;

typedef struct vps_plan_stats_t {
    int64_t num_boxes, num_retain_boxes, num_send_boxes, num_recv_boxes;
    int64_t num_pack_tiles, num_unpack_tiles, num_retain_tiles;
    int64_t num_peers_out, num_peers_in; /* single-rank plans; 0 otherwise */
    double plan_ms;                      /* host wall time of vps_plan_intersections */
} vps_plan_stats_t;

/* F_P (Section 4.1, Section 4.2.2): map configuration `par` of `model` onto the VPS.
 * rank = -1 maps every rank (needed for planning); rank >= 0 keeps only that rank's pieces.
 * Both descriptors are caller-owned host structs, copied on entry.  *out is library-owned;
 * release with vps_config_destroy.  The tables are filled by a kernel queued on the null
 * stream; the call does not wait for it (planning orders itself after it).
 * Errors: VPS_ERR_INVALID_ARG (null pointers, non-positive sizes), VPS_ERR_INDIVISIBLE,
 * VPS_ERR_RANK_RANGE, VPS_ERR_HIP. */
int vps_describe_config(const vps_model_desc* model, const vps_parallel_desc* par, int32_t rank,
                        vps_config** out);

/* Section 4.2.1 / 4.2.2: intersect the source and destination regions and resolve every
 * destination element to exactly one source rank.  rank >= 0 plans the share of one rank (its
 * retained, outgoing and incoming boxes; the rank index is used on both sides and must be
 * < max(world_src, world_dst)); rank = -1 plans all ranks (all virtual ranks resident).
 * Source rule for replicated data: the destination rank itself if it is an owner, else the
 * owners on its node if any, else all owners; ascending; index = destination data-parallel
 * index modulo count.  `stream` (hipStream_t) orders the device work; the call waits for it
 * once or twice before returning (see "synchronisation" above).  Both configs must have been described with rank = -1 for the same model
 * (VPS_ERR_MODEL_MISMATCH otherwise).  *out is library-owned (vps_plan_destroy). */
int vps_plan_intersections(const vps_config* src, const vps_config* dst, int32_t rank,
                           void* stream, vps_plan** out);

/* Same, with flags.
 * VPS_PLAN_ROUTES_ONLY builds the routed boxes, their order and the byte counts but no copy
 * descriptors and no tile table: for planning many ranks whose buffers are not resident (queries
 * work; vps_pack / vps_unpack / vps_apply_transition return VPS_ERR_INVALID_ARG).
 * VPS_PLAN_THROUGH_BUFFERS treats a rank as its own peer: the data that stays on a rank (T_retain
 * of Section 4.2.1) is packed into the rank's own segment of the send buffer and unpacked from
 * there instead of being copied directly, so that pack and unpack each run over the whole share
 * (a measurement mode; the destination bits are the same).  retain_total is then 0 and the
 * rank's own segment counts in send_total / recv_total and in vps_plan_peer_segment.
 * vps_apply_transition on a single-rank plan reads the rank's own segment out of the send region
 * (two launches); with vps_pack / vps_unpack the caller moves that segment from the send buffer
 * to the receive buffer like any peer's.  vps_stage_exchange refuses such a plan. */
enum { VPS_PLAN_ROUTES_ONLY = 1, VPS_PLAN_THROUGH_BUFFERS = 2 };
int vps_plan_intersections_ex(const vps_config* src, const vps_config* dst, int32_t rank,
                              uint32_t flags, void* stream, vps_plan** out);

/* Algorithm 1, PackData: copy every outgoing sub-box of `rank` from its old local
 * buffers into its send buffer.  src_bufs: host array of 8 device pointers (entries of empty
 * buffers may be NULL).  send_buf: device, >= send_total bytes (vps_plan_buffer_bytes), 16-byte
 * aligned.  Peer segments are laid out in ascending peer order; inside a segment boxes are
 * ordered by (kind 1,2,3,0; tensor id; lo corner), each row-major, each starting at a multiple
 * of 16 bytes; pad bytes are not written.  rank must be the planned rank, or any source rank for
 * an all-ranks plan. */
int vps_pack(const vps_plan* plan, int32_t rank, const void* const* src_bufs, void* send_buf,
             void* stream);

/* Algorithm 1, UnpackData: copy every incoming sub-box of `rank` from its receive
 * buffer (same layout rules, segments in ascending source-rank order) into the new local
 * buffers.  dst_bufs: host array of 8 device pointers.  Padding elements of dst are never
 * written. */
int vps_unpack(const vps_plan* plan, int32_t rank, const void* recv_buf, void* const* dst_bufs,
               void* stream);

/* Algorithm 1, the body of ExecuteSwitch for the resident ranks, in one call: retained boxes are copied
 * old-local -> new-local directly, outgoing boxes are packed, incoming ones unpacked.
 *   single-rank plan: rank = planned rank; src_bufs/dst_bufs are 8 pointers each; scratch holds
 *     [send buffer | receive buffer] at the offsets reported by vps_plan_buffer_bytes.  The
 *     peers are not resident, so the receive part must already hold the peers' packed data.
 *   all-ranks plan: rank = -1; src_bufs is [world_src][8], dst_bufs is [world_dst][8]; scratch
 *     holds every rank's send buffer and the exchange is done by reading the peer's segment
 *     in place.
 * VPS_ERR_SCRATCH_TOO_SMALL if scratch_bytes < scratch_needed.  A source buffer must not be
 * passed as a destination buffer as well (checked for equal pointers only: VPS_ERR_INVALID_ARG).
 * Calls on a single-rank plan are re-entrant; calls on an all-ranks plan share one device-side
 * pointer table, so they must not overlap on different streams.  The call enqueues kernels only
 * (no allocation, no memset, no copy engine, no synchronisation), so it may be captured into a
 * HIP graph; the same holds for vps_pack and vps_unpack. */
int vps_apply_transition(const vps_plan* plan, int32_t rank, const void* const* src_bufs,
                         void* const* dst_bufs, void* scratch, uint64_t scratch_bytes,
                         void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): vps_apply_transition for an all-ranks plan with the
 * staging area (every rank's send buffer) in a device array that is part of the library image
 * instead of a caller-owned scratch.  The call allocates nothing on the device and frees nothing;
 * it enqueues the same kernels as vps_apply_transition(plan, -1, ...).
 *   plan       an all-ranks plan (VPS_ERR_INVALID_ARG for a single-rank plan: its receive buffer
 *              is filled by the caller and cannot be library memory)
 *   src_bufs   host array [world_src][8] of device pointers, dst_bufs [world_dst][8]
 *   limit      scratch_needed of the plan (vps_plan_buffer_bytes, rank = -1) must not exceed
 *              VPS_STATIC_SCRATCH_BYTES: VPS_ERR_SCRATCH_TOO_SMALL otherwise, nothing enqueued
 * Every GPU that the library runs on holds its own copy of the array until the process ends.  All
 * calls on one GPU share that GPU's array, which keeps the previous call's contents (nothing in it
 * needs clearing: pack writes every byte that unpack reads): calls that overlap on one GPU, on any
 * streams, race and must be serialised by the caller. */
#define VPS_STATIC_SCRATCH_BYTES (128ull << 20)
int vps_apply_transition_static(const vps_plan* plan, const void* const* src_bufs,
                                void* const* dst_bufs, void* stream);
uint64_t vps_static_scratch_bytes(void); /* VPS_STATIC_SCRATCH_BYTES of the loaded library */

/* ---- staged exchange among resident ranks ----
 * Algorithm 1 (MemoryAwareChunk and the step loop) and Section 4.3 "Asynchronous Deadlock-Free
 * Communication", for an all-ranks plan.  Steps s = 1 .. 2^ceil(log2 N) - 1 (N = the larger
 * world): in step s rank i is paired with rank i XOR s; the pair is skipped when the peer does
 * not exist or no data flows.  cost(s) = max over ranks of the bytes the rank sends plus the
 * bytes it receives in step s (alignment pad included).  Steps are taken in ascending order; a
 * step joins the current stage unless the stage would then exceed budget_bytes_per_rank, in
 * which case the stage is closed first.  Steps without traffic belong to no stage, no empty
 * stage is emitted, and a step that alone exceeds the budget forms a stage of its own.
 * Every stage is executed as pack -> exchange (each send segment is copied to the peer's
 * receive segment) -> unpack, all stages reusing one scratch area of scratch_needed bytes;
 * retained boxes are copied once, first.  The plan must outlive the stage plan. */
typedef struct vps_stage_plan vps_stage_plan;
int vps_stage_exchange(const vps_plan* plan, uint64_t budget_bytes_per_rank, void* stream,
                       vps_stage_plan** out);
int vps_stage_info(const vps_stage_plan* sp, int32_t* num_steps, int32_t* num_stages,
                   uint64_t* scratch_needed);
/* stage_of_step[s] (-1: no traffic) and step_cost[s] for s = 0 .. num_steps (entry 0 unused). */
int vps_stage_steps(const vps_stage_plan* sp, int32_t* stage_of_step, uint64_t* step_cost,
                    int32_t max_entries);
/* src_bufs is [world_src][8], dst_bufs is [world_dst][8] (host arrays of device pointers).
 * VPS_ERR_SCRATCH_TOO_SMALL if scratch_bytes < scratch_needed. */
int vps_apply_transition_staged(const vps_stage_plan* sp, const void* const* src_bufs,
                                void* const* dst_bufs, void* scratch, uint64_t scratch_bytes,
                                void* stream);
void vps_stage_plan_destroy(vps_stage_plan* sp);

/* ---- collective intent ----
 * Algorithm 1 (OptimizePrimitives) and Section 4.3 "Communication Primitive Optimization": group
 * the routed boxes that leave their rank by logical tensor and state kind and infer which
 * collective the group amounts to from the number of distinct sources and destinations and from
 * the slices: identical slices from one source to several destinations are a broadcast; slices
 * from one source to several destinations that tile one contiguous range of the flattened
 * tensor are a scatter; such slices from several sources to one destination a gather; all else
 * stays point-to-point.  A slice is one routed box; it is contiguous when it is a single range of
 * the row-major flattening of the unsharded tensor.  classes[tensor*4 + kind] receives the code;
 * src must be the source configuration the plan was made from.  Runs on the device, synchronises
 * the stream. */
enum { VPS_COLL_NONE = 0, VPS_COLL_P2P = 1, VPS_COLL_BROADCAST = 2, VPS_COLL_SCATTER = 3, VPS_COLL_GATHER = 4 };
int vps_plan_classify_collectives(const vps_plan* plan, const vps_config* src, void* stream,
                                  int32_t* classes, int64_t max_entries);

/* ---- queries (host side, no device work unless stated) ---- */
int vps_config_world(const vps_config* cfg, int32_t* world);
int vps_config_num_buffers(const vps_config* cfg, int32_t rank, int32_t* n); /* always VPS_NUM_BUFFERS */
int vps_config_num_tensors(const vps_config* cfg, int32_t* n);
int vps_config_buffer_bytes(const vps_config* cfg, int32_t rank, int32_t buf, uint64_t* bytes);
int vps_config_num_pieces(const vps_config* cfg, int64_t* n);
/* Copies up to `max` pieces (ordered by tensor, kind, tp, dp index) to host memory. */
int vps_config_get_pieces(const vps_config* cfg, vps_piece* out, int64_t max);

/* Payload bytes (without alignment pad) that src_rank sends to dst_rank (retained volume when
 * equal).  Pairs outside a single-rank plan report 0. */
int vps_plan_pair_bytes(const vps_plan* plan, int32_t src_rank, int32_t dst_rank, uint64_t* bytes);
/* As seen from `rank`: payload bytes it sends to and receives from `peer`. */
int vps_plan_peer_bytes(const vps_plan* plan, int32_t rank, int32_t peer, uint64_t* send,
                        uint64_t* recv);
/* Buffer sizes of `rank` including alignment pad: send buffer, receive buffer, retained payload
 * and the scratch size for vps_apply_transition (rank = -1: the all-ranks scratch).
 * recv_offset_in_scratch is where the receive part starts for single-rank plans. */
int vps_plan_buffer_bytes(const vps_plan* plan, int32_t rank, uint64_t* send_total,
                          uint64_t* recv_total, uint64_t* retain_total, uint64_t* scratch_needed,
                          uint64_t* recv_offset_in_scratch);
/* Byte range of the segment src_rank -> dst_rank inside the sender's send buffer and the
 * receiver's receive buffer (bytes includes alignment pad between boxes). */
int vps_plan_peer_segment(const vps_plan* plan, int32_t src_rank, int32_t dst_rank,
                          uint64_t* send_off, uint64_t* recv_off, uint64_t* bytes);
int vps_plan_num_boxes(const vps_plan* plan, int64_t* n);
int vps_plan_get_boxes(const vps_plan* plan, vps_box* out, int64_t max);
int vps_plan_stats(const vps_plan* plan, vps_plan_stats_t* out);

void vps_config_destroy(vps_config* cfg);
void vps_plan_destroy(vps_plan* plan);
const char* vps_last_error(void);

/* Settings for benchmarks and tests; they apply to plans created afterwards (launch settings to
 * launches made afterwards) and may be changed from any thread.
 *   VPS_OPT_TILE_BYTES        target payload bytes per workgroup tile: a power of two between
 *                             4 KiB and 1 MiB, default 8 KiB (vps_set_tile_bytes sets the same)
 *   VPS_OPT_SMALL_PLAN_BOXES  plans with at most this many boxes (1 .. 65536, default 8192) are
 *                             ordered by counting in one launch; larger ones pair by pair or by
 *                             a radix sort (see VPS_OPT_PAIR_ORDER_WORK)
 *   VPS_OPT_XPOSE_SHAPE       super-block shape of transposed boxes, sa | sb << 16 (1 .. 64 each);
 *                             0 = chosen per box from the row pitches (default)
 *   VPS_OPT_XCD_RUN           consecutive tiles handed to one XCD (0 = round-robin, default 64)
 *   VPS_OPT_PAIR_ORDER_WORK   larger all-ranks plans are ordered pair by pair (source rank x
 *                             destination rank) by counting as long as the sum over the pairs of
 *                             the squared number of their boxes stays below 2^value (default 32,
 *                             at most 40), and by a radix sort otherwise; 0 = always the sort */
enum { VPS_OPT_TILE_BYTES = 0, VPS_OPT_SMALL_PLAN_BOXES = 1, VPS_OPT_XPOSE_SHAPE = 2, VPS_OPT_XCD_RUN = 3,
       VPS_OPT_PAIR_ORDER_WORK = 4 };
int vps_set_option(int32_t option, uint32_t value);
int vps_set_tile_bytes(uint32_t bytes);

/* Measurement aid, not part of the paper's method: a plain contiguous device-to-device copy of
 * `bytes` bytes in the copy engine's launch shape (one workgroup per 8 KiB, the same XCD-aware
 * block order, 16-byte nontemporal loads and stores) without any table.  Its rate is the
 * practical ceiling the descriptor-driven copies are compared with.  dst, src: device, 16-byte
 * aligned, not overlapping; bytes a multiple of 16 (VPS_ERR_INVALID_ARG otherwise).
 * Asynchronous on `stream`. */
int vps_plain_copy(void* dst, const void* src, uint64_t bytes, void* stream);
/* The two halves of that copy alone, in the same launch shape: read `bytes` bytes from src (the
 * loads feed a value that is stored to `sink`, 4 bytes of device memory, only if it equals a
 * sentinel), or fill `bytes` bytes at dst with the byte 0xA5.  Same argument rules. */
int vps_plain_read(const void* src, uint64_t bytes, void* sink, void* stream);
int vps_plain_fill(void* dst, uint64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VPS_H */
