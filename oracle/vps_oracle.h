/* CPU oracle for the Virtual Parameter Space state transition (DynaTrain, Sections 4.1-4.3).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, per-element, obviously-correct definition of
 * what a strategy transition must produce.  It has no box logic, no tiling and no fusion, and
 * shares no code with the HIP library.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.
 *
 * The method reaches an exact result (Section 6, convergence study: resharding is exact), so
 * the oracle is the plain definition:
 *
 *   for destination configuration B, rank j, every buffer b and every non-padding local
 *   offset o:  (t, c) = coord_B(j, b, o);  dst_j[b][o] = src_i[b'][o'] for the source
 *   (i, b', o') chosen among owners_A(kind(b), t, c).
 *
 * Every configuration P is described by two mutually inverse per-element maps
 * (Section 4.1, F_P and the sub-VPS): coord_P (local slot -> logical element) and owners_P
 * (logical element -> every local slot that stores it).  ZeRO flat-buffer shards are handled
 * by the same two maps (Section 4.2.2: a flat offset is a position in the flattened
 * parameter order, evenly cut across the data-parallel group).
 *
 * Parity pins (tests/test_oracle_*.py): inverse property by brute force, replica counts,
 * an independent assemble-then-slice reshard in numpy, identity and round-trip transitions,
 * closed-form byte counts, the Figure 4 worked example, parameter counts.
 * parity unpinned by the paper: the replica source rule (orc_select_source), the placement of
 * EP inside TP x DP (ep_placement = 1) and the order of elements inside a per-peer buffer
 * (orc_piece_key, orc_recv_payload) are conventions of this repository; the paper only says that
 * the source is chosen by proximity (Section 4.3), prints (TP, PP, DP, EP) tuples without a
 * placement, and says that slices are packed per peer.  They are checked against examples
 * evaluated by hand (tests/golden/declared_readings.txt) and against a second, box-based
 * formulation in numpy.
 */
#ifndef VPS_ORACLE_H
#define VPS_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_FAMILY_GPT = 0, ORC_FAMILY_GQA = 1, ORC_FAMILY_MOE = 2 };
enum { ORC_NKIND = 4, ORC_NBUF = 8 }; /* buffer index = group*4 + kind; group 0 dense, 1 expert */

typedef struct {
    int32_t family, layers, hidden, q_heads, kv_heads, head_dim, ffn, vocab, experts, expert_ffn;
} orc_model;

typedef struct {
    int32_t tp, pp, dp, ep;
    int32_t zero;          /* 0: fp32 kinds replicated over the DP group; 1: sharded by flat offset */
    int32_t gpus_per_node;
    int32_t qkv_layout;    /* 0 interleaved, 1 blocked [Q|K|V] */
    int32_t expert_layout; /* 0 row-major, 1 transposed storage */
    int32_t flat_order;    /* 0 ascending tensor id, 1 descending */
    int32_t ep_placement;  /* 0: world = tp*pp*dp*ep, experts TP-sharded, dp = expert data-parallel
                              degree; 1: EP carved out of the tp*dp ranks of a stage (world =
                              tp*pp*dp), experts not TP-sharded, expert dp = tp*dp/ep */
} orc_parallel;

typedef struct orc_config orc_config;

/* Returns NULL and writes a message into err when a degree does not divide its axis. */
orc_config* orc_config_create(const orc_model* m, const orc_parallel* p, char* err, int errlen);
void orc_config_destroy(orc_config* c);

int32_t orc_world(const orc_config* c);
int32_t orc_num_tensors(const orc_config* c);
/* shape[4] (leading 1s), info[4] = {tp_axis (-1 = replicated), group, layer (-1 pre, L post), expert} */
void orc_tensor_info(const orc_config* c, int32_t t, int32_t* shape, int32_t* info);
uint64_t orc_tensor_numel(const orc_config* c, int32_t t);
uint64_t orc_total_params(const orc_config* c);

/* rank -> {tp, dense dp index, pp, ep, expert dp index, expert tp index} */
void orc_rank_coords(const orc_config* c, int32_t rank, int32_t* out6);

/* Element counts of local buffer `buf` of `rank`: allocated size and non-padding part. */
uint64_t orc_buffer_elems(const orc_config* c, int32_t rank, int32_t buf);
uint64_t orc_payload_elems(const orc_config* c, int32_t rank, int32_t buf);

/* coord_P: returns 1 and fills (tensor, coord[4]) for a stored element, 0 for padding,
 * -1 when off is outside the buffer. */
int orc_coord(const orc_config* c, int32_t rank, int32_t buf, uint64_t off, int32_t* tensor,
              int32_t* coord);
/* owners_P: every (rank, buffer, offset) that stores element (kind, tensor, coord).
 * Returns the count (ascending rank order); writes at most `max` entries. */
int orc_owners(const orc_config* c, int32_t kind, int32_t tensor, const int32_t* coord, int max,
               int32_t* ranks, int32_t* bufs, uint64_t* offs);
/* Row-major linear index of coord in the unsharded logical tensor. */
uint64_t orc_linear(const orc_config* c, int32_t tensor, const int32_t* coord);

/* Source chosen for destination rank j among owners_A (retain if j owns it, else same-node
 * owners if any, else all; ascending; index = destination data-parallel index mod count).
 * Returns 1 on success. */
int orc_select_source(const orc_config* a, const orc_config* b, int32_t j, int32_t kind,
                      int32_t tensor, const int32_t* coord, int32_t* rank, int32_t* buf,
                      uint64_t* off);

/* Fill out[0..n) (16-bit words for kind 0, 32-bit otherwise) with the pattern of the elements
 * stored at offsets [off0, off0+n) of the buffer.  Padding slots get pad_word. */
int orc_fill(const orc_config* c, int32_t rank, int32_t buf, uint64_t seed, uint64_t rank_salt,
             uint64_t off0, uint64_t n, void* out, uint32_t pad_word);

/* Expected destination content of offsets [off0, off0+n) after A -> B when every source rank i
 * was filled by orc_fill(a, i, ..., seed, rank_salt).  Padding slots get pad_word. */
int orc_expected(const orc_config* a, const orc_config* b, int32_t j, int32_t buf, uint64_t seed,
                 uint64_t rank_salt, uint64_t off0, uint64_t n, void* out, uint32_t pad_word);

/* The transition itself on host memory: src_bufs[rank*8+buf] are the source ranks' buffers
 * (may be NULL for ranks that are never chosen).  Writes dst[0..n) for offsets
 * [off0, off0+n) of (j, buf); padding slots are left untouched.  Returns 0, or -1 if a needed
 * source buffer is NULL. */
int orc_transition(const orc_config* a, const orc_config* b, int32_t j, int32_t buf,
                   const void* const* src_bufs, uint64_t off0, uint64_t n, void* dst);

/* Bytes that destination rank j takes from every source rank: from_bytes[world_A] (the entry of
 * j itself is the retained volume).  Counts offsets [off0, off0+n) of every buffer in
 * buf_mask (bit b = buffer b); n == 0 means the whole buffer. */
int orc_route_bytes(const orc_config* a, const orc_config* b, int32_t j, uint32_t buf_mask,
                    uint64_t* from_bytes);

/* Bytes that source rank i sends to every destination rank: to_bytes[world_B] (entry i =
 * retained).  Walks i's source buffers; for sharded kinds every element has one slot, for
 * replicated ones each replica is asked whether it is the chosen source. */
int orc_send_bytes(const orc_config* a, const orc_config* b, int32_t i, uint32_t buf_mask,
                   uint64_t* to_bytes);

/* Validate a list of sub-boxes produced by some planner, element by element.
 * Box k: ints[k*16 + 0..15] = {kind, tensor, src_rank, dst_rank, src_buf, dst_buf, lo[4], ext[4],
 * 0, 0}; offs[k*10 + 0..9] = {src_off, dst_off, src_stride[4], dst_stride[4]} (elements).
 * For every element of the box (or `samples` pseudo-random ones plus the corners when
 * samples > 0) checks that the source slot is an owner under A, the destination slot is the
 * owner under B, and the source rank is the selected one.  Returns the number of violations
 * (0 = valid); first_bad receives the index of the first offending box or -1. */
int64_t orc_check_boxes(const orc_config* a, const orc_config* b, const int32_t* ints,
                        const int64_t* offs, int64_t nboxes, int32_t samples, int64_t* first_bad);

/* The piece (see vps_oracle.c, "per-peer buffers") of the element stored at (rank, buf, off):
 * out3 = {storage block, level, parent unit}.  Two stored elements of one (rank, buffer, tensor)
 * belong to the same piece iff the three numbers agree.  Returns 1, 0 for padding, < 0 on error. */
int orc_piece_key(const orc_config* c, int32_t rank, int32_t buf, uint64_t off, int64_t* out3);

/* Algorithm 1, PackData / Section 4.3: the receive buffer of destination rank j as its source
 * ranks must have packed it, i.e. the segments i -> j in ascending i, which are also the
 * pieces of the senders' send buffers.  Every element comes from the pattern of its selected
 * source (orc_fill with the same seed and rank_salt); pad bytes between boxes are pad_byte.
 * seg_off[0..world_A] receives the byte offset of every source's segment (seg_off[world_A] =
 * total).  through != 0 also routes the data that stays on rank j through its own segment.
 * Returns the number of bytes, or < 0 (-3: cap too small). */
int64_t orc_recv_payload(const orc_config* a, const orc_config* b, int32_t j, int through,
                         uint64_t seed, uint64_t rank_salt, uint8_t pad_byte, void* out,
                         uint64_t cap, uint64_t* seg_off);

int orc_num_threads(void);
void orc_set_num_threads(int n);

#ifdef __cplusplus
}
#endif
#endif
