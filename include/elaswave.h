/*
 * elaswave.h -- C ABI of the MI355X (gfx950) reshard + snapshot/checksum library.
 *
 * The library implements the data-parallel hot path of ElasWave's parameter
 * recovery (arXiv 2510.00606): re-partitioning one DP group's flat ZeRO state
 * from an old DP degree to a new one under the interleaved ZeRO assignment
 * (Sec. 6.3), driven by the Live Remap transfer plan (Sec. 5.2), plus the
 * per-step in-memory snapshot (Sec. 5.1) with per-block checksums for the
 * "online verification" the abstract names.
 *
 * Conventions
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory of the current device.  Pointer ARRAYS (old_shards,
 *     snapshots, new_shards) are host arrays whose entries are device pointers.
 *   - All offsets and lengths in plans are in ELEMENTS, so one plan serves the
 *     bf16 parameter array and the fp32 master / Adam m / Adam v arrays.
 *   - Ranks: "old rank" indexes the DP group before the event (0..old_dp-1),
 *     "new rank" after it (0..new_dp-1).  Survivors keep their relative order
 *     and are renumbered densely from 0; joiners follow; if new_dp is smaller
 *     than the number of survivors the highest survivors only give data away.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Kernel-launching calls enqueue work and return; the caller synchronises.
 *   - Every call returns EW_OK (0) or a negative error code.  Nothing throws,
 *     aborts or falls back to the CPU.  On error output arguments are untouched.
 *   - The caller owns every device buffer it passes.  The library owns only the
 *     plan object (host) and, after ew_plan_upload, its device tables.
 */
#ifndef ELASWAVE_H
#define ELASWAVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EW_MAX_DP 64u            /* alive_mask is 64 bits wide                              */
#define EW_GRANULE 8u            /* elements; piece boundaries inside a unit are multiples  */
#define EW_CKSUM_BLOCK (1u << 20) /* bytes covered by one checksum record                   */

enum {
  EW_OK = 0,
  EW_EINVAL = -1,          /* bad argument (zero degree, degree > 64, chunk 0, mask bits above
                              old_dp, non-monotone unit boundaries, elem_size not 2 or 4, NULL
                              where data is needed, plan not uploaded)                          */
  EW_EUNRECOVERABLE = -2,  /* no survivor, or a failed rank whose ring predecessor failed too */
  EW_ENOMEM = -3,          /* host or device allocation failed                                 */
  EW_EHIP = -4,            /* HIP runtime error; text of the last one via ew_strerror(EW_EHIP) */
  EW_EINFEASIBLE = -5,     /* ew_partition_layers: no partition fits the stages' memory caps   */
  EW_ETOOBIG = -6          /* ew_snapshot_noalloc: nbytes above EW_NOALLOC_MAX_BYTES           */
};

typedef struct ew_plan_s ew_plan_t; /* opaque */

/* One checksum record: wrapping sum and XOR of a block's little-endian u64 words. */
typedef struct {
  uint64_t sum;
  uint64_t xr;
} ew_cksum_t;

#define EW_SEG_SNAPSHOT 1u /* source is the snapshot of src_owner's shard (src_owner failed)   */
#define EW_SEG_LOCAL 2u    /* holder's new rank == dst_rank: bypasses the staging arena        */
#define EW_NO_STAGE (~(uint64_t)0)

/* One entry of the transfer plan: an element-exact cell fragment of the overlap
 * matrix M_overlap (Sec. 5.2 step 2, Fig. 7b). 40 bytes. */
typedef struct {
  uint64_t src_off;   /* offset inside src_owner's OLD shard (live or snapshot copy)           */
  uint64_t dst_off;   /* offset inside dst_rank's NEW shard                                    */
  uint64_t stage_off; /* offset inside the staging arena; EW_NO_STAGE for LOCAL segments       */
  uint64_t len;       /* elements, > 0                                                         */
  uint16_t src_owner; /* old rank whose partition the data belongs to                          */
  uint16_t holder;    /* old rank that serves it: src_owner if alive, else (src_owner-1) mod old_dp
                         (worker i keeps the snapshot of worker (i+1) mod n, Sec. 5.1)          */
  uint16_t dst_rank;  /* new rank                                                              */
  uint16_t flags;     /* EW_SEG_*                                                              */
} ew_seg_t;

/* ---- Live Remap steps 1+2: integrity check and transfer plan (Sec. 5.2) -------------------
 * Layout (Sec. 6.3, Fig. 10b): the flat state of `numel` elements is cut into units (the
 * paper's layers) of `chunk` elements, the last one short; every unit of L elements is split
 * uniformly over D ranks at b_j = min(L, 8*floor(j*ceil(L/8)/D)); rank j's shard is its piece
 * of every unit, in unit order.  The plan intersects, unit by unit, what each surviving
 * holder has (its own piece, plus its ring successor's piece from the snapshot if that
 * successor failed) with the new layout's pieces.
 * alive_mask: bit j set = old rank j survived.  *out receives a new plan (host memory) to be
 * released with ew_plan_free.  Synchronous, no GPU work. */
int ew_plan(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, uint64_t numel, uint64_t chunk,
            ew_plan_t **out);

/* Same, with explicit unit boundaries (host array of n_units+1 ascending values,
 * unit_starts[0] = 0, unit_starts[n_units] = numel; empty units allowed). */
int ew_plan_bounds(uint32_t old_dp, uint32_t new_dp, uint64_t alive_mask, uint64_t n_units,
                   const uint64_t *unit_starts, ew_plan_t **out);

/* ---- Layer migration between two pipeline stages of equal DP degree (Sec. 6.3, Fig. 10) ------
 * The last n_move units (layers) of stage S become the first units of stage S+1.  Both stages
 * use the same ZeRO assignment:
 *   EW_ASSIGN_INTERLEAVED  every unit is split uniformly over the dp ranks of the stage that
 *                          holds it; rank j's shard is its piece of every unit (Fig. 10b);
 *   EW_ASSIGN_CONTIGUOUS   a stage's units form one flat array cut into dp contiguous blocks of
 *                          (about) equal size, block r belonging to rank r (Fig. 10a).
 * The plan has 2*dp old and 2*dp new ranks: ranks 0..dp-1 are stage S, dp..2dp-1 stage S+1, all
 * alive.  It is executed by ew_pack / ew_unpack like any other plan (pointer arrays of 2*dp
 * entries); ew_plan_pair_len(h, k) is the traffic matrix: under the interleaved assignment only
 * the dp pairs (j, dp + j) are non-empty and sum to the moved state, under the contiguous one
 * both stages also re-compact ((dp-1)/2 of the moved state per stage when a small layer moves).
 * src/dst_unit_starts: host arrays of n_units+1 ascending boundaries starting at 0.
 * EW_EINVAL: unknown assignment, dp = 0, 2*dp > 64, n_move > n_src_units, bad boundaries. */
#define EW_ASSIGN_INTERLEAVED 0u
#define EW_ASSIGN_CONTIGUOUS 1u
int ew_plan_migrate(uint32_t assignment, uint32_t dp, uint64_t n_src_units, const uint64_t *src_unit_starts,
                    uint64_t n_dst_units, const uint64_t *dst_unit_starts, uint64_t n_move, ew_plan_t **out);

/* ---- Which layers sit on which stage: minimax layer partition (Sec. 4.2, Eq. 2-3, Alg. 1) ------
 * Cuts layers 0..n_layers-1 into n_stages non-empty contiguous blocks, block p on stage p, so that
 * every block's memory fits its stage and the largest per-stage mini-step time is minimal.  The
 * result says which boundary layers have to move between adjacent stages (ew_plan_migrate).
 * t:   host [n_stages][n_layers][n_layers], t[p][a][b] = mini-step time of stage p hosting layers
 *      a..b (entries with a > b are ignored);
 * mem: host [n_layers][n_layers], mem[a][b] = memory of layers a..b on one stage; cap: host [n_stages].
 * out_bounds: host [n_stages-1], out_bounds[p] = number of layers on stages 0..p (stage p hosts
 * layers out_bounds[p-1] .. out_bounds[p]-1); *out_cost = the optimal worst-stage time.  Among
 * optimal partitions the one found by scanning split points upward is returned.
 * EW_EINFEASIBLE if no partition fits; EW_EINVAL for zero sizes, more stages than layers, NULLs. */
int ew_partition_layers(uint32_t n_layers, uint32_t n_stages, const double *t, const double *mem,
                        const double *cap, uint32_t *out_bounds, double *out_cost);

/* Frees host and device tables.  Work enqueued with this plan must have completed. */
void ew_plan_free(ew_plan_t *plan);

/* Plan queries (host, constant time).  Segments are ordered by unit, then by element. */
uint64_t ew_plan_numel(const ew_plan_t *plan);
uint32_t ew_plan_old_dp(const ew_plan_t *plan);
uint32_t ew_plan_new_dp(const ew_plan_t *plan);
uint64_t ew_plan_num_segs(const ew_plan_t *plan);
/* The explicit segment table (ew_plan_num_segs entries), expanded from the plan's run-length
 * form on the first call and cached; borrowed, valid until ew_plan_free; NULL if out of memory.
 * The hot path never needs it: it is for inspection and tests. */
const ew_seg_t *ew_plan_segs(const ew_plan_t *plan);
/* Runs of consecutive equal-length units the plan is stored as (2 for a uniform chunk). */
uint64_t ew_plan_num_runs(const ew_plan_t *plan);
uint64_t ew_plan_old_shard_len(const ew_plan_t *plan, uint32_t old_rank); /* elements         */
uint64_t ew_plan_new_shard_len(const ew_plan_t *plan, uint32_t new_rank); /* elements         */
int32_t ew_plan_new_rank_of(const ew_plan_t *plan, uint32_t old_rank); /* -1: failed/leaving */
int32_t ew_plan_holder_of(const ew_plan_t *plan, uint32_t old_rank);   /* rank serving its data */
uint64_t ew_plan_stage_len(const ew_plan_t *plan);                     /* arena size, elements */
/* Message of pair (holder -> new rank) inside the arena; messages are contiguous and laid
 * out sorted by (dst_rank, holder).  Length 0 for pairs that exchange nothing. */
uint64_t ew_plan_pair_len(const ew_plan_t *plan, uint32_t holder, uint32_t dst_rank);
uint64_t ew_plan_pair_off(const ew_plan_t *plan, uint32_t holder, uint32_t dst_rank);
uint64_t ew_plan_remote_elems(const ew_plan_t *plan); /* == stage_len                        */
/* Workgroup-sized copy tiles of ew_pack (which = 0) / ew_unpack (which = 1) for elem_size. */
uint64_t ew_plan_num_tiles(const ew_plan_t *plan, int which, uint32_t elem_size);

/* Host-side view of the copy tiles, decoded by the same routine the kernels use (inspection and
 * tests; no GPU needed).  src_buf: 0..63 = live shard of that old rank, 64..127 = snapshot of
 * that owner, 128 = staging arena.  dst_buf: 0..63 = new shard of that rank, 64 = arena. */
typedef struct {
  uint64_t src_off; /* elements */
  uint64_t dst_off; /* elements */
  uint32_t len;     /* elements */
  uint16_t src_buf;
  uint16_t dst_buf;
} ew_tile_t;
/* Writes tiles [first, first+count) of the table for `which` (0 pack, 1 unpack, 2 direct), cut at
 * tile_elems elements with cut points on multiples of align_elems in the destination (0: no
 * alignment), into out[] (host) and the table's tile count into *total (may be NULL). */
int ew_plan_tiles(const ew_plan_t *plan, int which, uint32_t tile_elems, uint32_t align_elems, uint64_t first,
                  uint64_t count, ew_tile_t *out, uint64_t *total);

/* Which tile of a launch of n_workgroups tiles workgroup `workgroup` copies (the routine the tile
 * kernels use, on the host: inspection and tests).  Consecutive workgroup ids go round-robin to the
 * GPU's 8 XCDs, each with an L2 of its own; with group > 1, inside every block of 8*group workgroups
 * XCD x takes the `group` consecutive tiles x*group .. x*group+group-1, so that each XCD streams
 * through runs of the destination instead of every eighth tile (the knob "xcd_group_kib" divided
 * by the tile size is the group the kernels use).  group 0 or 1, and a trailing partial block: identity. */
uint64_t ew_tile_of_workgroup(uint64_t workgroup, uint64_t n_workgroups, uint32_t group);

/* Builds the copy-tile tables (segments cut into pieces of at most tile_elems elements;
 * 0 = library default, 4 KiB worth of elements) for both element sizes and uploads them to the
 * current device on `stream` (a few hundred KiB for a uniform chunk).  Must precede ew_pack /
 * ew_unpack, which return EW_EINVAL when another device is current than the one the tables
 * were uploaded to.  Calling it again replaces the tables (previous work must be done).
 * The copy is asynchronous on `stream`: calls that use the plan must be ordered after it, i.e. be
 * issued on the same stream, or on another one only after `stream` has been synchronised (or after
 * an event recorded on it behind this call has been waited for).
 * EW_EINVAL if a table would exceed 2^31-1 tiles. */
int ew_plan_upload(ew_plan_t *plan, uint32_t tile_elems, void *stream);

/* ---- Live Remap step 3, send side: gather into per-destination messages -------------------
 * For every non-LOCAL segment copies len elements from the holder's live shard
 * (old_shards[holder]) or from the snapshot of the failed owner (snapshots[src_owner]) to
 * stage[stage_off ...].  old_shards / snapshots: host arrays of old_dp device pointers;
 * entries the plan never reads may be NULL (failed ranks' live shards are never read).
 * stage: device, ew_plan_stage_len()*elem_size bytes.  elem_size: 2 (bf16) or 4 (fp32).
 * All buffers should be 16-byte aligned for full speed; any alignment is handled correctly. */
int ew_pack(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots,
            void *stage, uint32_t elem_size, void *stream);

/* ---- Live Remap step 3 receive side + step 4: build the new shards ------------------------
 * Non-LOCAL segments: stage -> new_shards[dst_rank][dst_off...].  LOCAL segments (diagonal of
 * M_overlap): old shard or locally held snapshot -> new shard directly.  Every element of
 * every new shard is written exactly once.  new_shards: host array of new_dp device pointers,
 * each ew_plan_new_shard_len()*elem_size bytes. */
int ew_unpack(const ew_plan_t *plan, const void *stage, const void *const *old_shards,
              const void *const *snapshots, void *const *new_shards, uint32_t elem_size,
              void *stream);

/* ---- Unpack fused with the fresh snapshot of the new layout ---------------------------------
 * Same result as ew_unpack followed, for every new rank k, by ew_snapshot(new_shards[k],
 * new_snapshots[k], new_len[k]*elem_size, new_cksums[k]) -- the snapshot that makes the next
 * failure recoverable (ring placement, Sec. 5.1) and verifiable (abstract) -- but every element is
 * read once: it is stored to the new shard and to its snapshot copy and folded into the checksum
 * of the new shard's 1 MiB block it lands in.  new_snapshots, new_cksums: host arrays of new_dp
 * device pointers (buffers of new_len[k]*elem_size bytes / ceil(that / 2^20) records, records
 * overwritten).  Uses the library's scratch array like ew_snapshot, and like it has a slower form
 * that needs no scratch (every workgroup adds its tile to the records with atomics) for a stream
 * under graph capture that can get no region; see ew_snapshot for the rules.
 * EW_EINVAL if the plan was uploaded with tiles above 1 MiB.
 * Speed: the call streams from three places at once (sources, new shards, snapshot copies).  The
 * MI355X's 288 GiB of HBM behave as three regions of 96 GiB of physical memory, and streams that
 * share a region slow each other down: 6.2 TB/s with all three in one region, 6.55-6.65 with the
 * two written buffers in different ones.  Physical addresses are not visible to a program, so
 * where these long-lived buffers matter, allocate a few candidates for the snapshot copies (and
 * for the new shards), time one call on each and keep the best. */
int ew_unpack_snapshot(const ew_plan_t *plan, const void *stage, const void *const *old_shards,
                       const void *const *snapshots, void *const *new_shards, void *const *new_snapshots,
                       ew_cksum_t *const *new_cksums, uint32_t elem_size, void *stream);

/* ---- Live Remap steps 3 and 4 without the arena ------------------------------------------------
 * Where holders and destinations share one address space -- all ranks in one GPU's memory as here,
 * or load/store-mapped peers -- a destination can pull every segment straight from the holder's
 * live shard or snapshot (the two kinds of pull that Fig. 7a's caption names: from a survivor's
 * device memory and from the snapshot a survivor keeps of its failed neighbour) and
 * the pair messages need not be materialised: new_shards as after ew_pack + ew_unpack, 28 B per
 * element of traffic less for every remote element.  ew_reshard_snapshot adds the snapshot copies
 * and checksums of the new shards exactly as ew_unpack_snapshot does.  Arguments, errors and
 * scratch use as for ew_unpack / ew_unpack_snapshot, minus `stage`. */
int ew_reshard(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots,
               void *const *new_shards, uint32_t elem_size, void *stream);
int ew_reshard_snapshot(const ew_plan_t *plan, const void *const *old_shards, const void *const *snapshots,
                        void *const *new_shards, void *const *new_snapshots, ew_cksum_t *const *new_cksums,
                        uint32_t elem_size, void *stream);

/* ---- Per-step snapshot (Sec. 5.1) with block checksums ------------------------------------
 * dst[0..nbytes) = src[0..nbytes); cksums[b] = (wrapping u64 sum, XOR) of the little-endian
 * 64-bit words of bytes [b*2^20, min((b+1)*2^20, nbytes)), a trailing partial word being
 * zero-padded.  src, dst, cksums: device; cksums has ceil(nbytes / 2^20) records and is
 * overwritten.  src and dst must not overlap.  nbytes = 0 is a no-op.
 * Never allocates device memory: per-workgroup partial checksums go through a fixed scratch array
 * inside the library (128 MiB per device, 4 regions).  A stream keeps the region it used last; when
 * more than 4 streams take turns, the least recently used region changes hands and the new stream
 * is made to wait (on the device, not the host) for that region's last use.  Calls may be issued
 * from several host threads, also on one stream; calls on different streams are enqueued side by
 * side.  Buffers that are not 16-byte aligned use a slower kernel that needs no scratch.
 * Graph capture: a capturing stream can use a region it already owns (run the calls once on it
 * before capturing) or one that no stream has used yet.  A region that a captured graph uses stays
 * with the capturing stream (the graph's replays are invisible to the library) until
 * ew_scratch_release: replay such a graph on the stream it was captured on, or ordered after that
 * stream's other calls.  One region per device always stays outside graphs, so at most 3 streams
 * per device capture with scratch; a capture that can get no region (a fourth capturing stream, or
 * one whose warm-up region went to another stream meanwhile) records the slower scratch-free
 * kernels instead, with the same results. */
int ew_snapshot(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *cksums, void *stream);

/* Tells the library that every graph captured on `stream` (on the current device) has been
 * destroyed and its replays are complete: the scratch regions those graphs used may change hands
 * again.  Harmless when there is nothing to release. */
int ew_scratch_release(void *stream);

/* ---- ew_snapshot for callers that cannot allocate ----------------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid allocation: same
 * arguments and results as ew_snapshot, but the call touches no allocator of any kind -- no
 * hipMalloc / hipFree, no event or lock creation, no scratch lease.  Its checksum slots live in a
 * second fixed device array of 16 MiB (sized for one 16-byte slot per KiB of input) that every GPU the
 * library runs on holds until the process ends; the array's address is looked up on the first call
 * on each device (make that call outside a capture).
 * nbytes above EW_NOALLOC_MAX_BYTES (1 GiB: more than one fp32 array of a 7B-stage rank shard)
 * returns EW_ETOOBIG and does nothing.  All calls on one GPU share the array: calls that may run at
 * the same time on one GPU (different streams) race on it and must be serialised by the caller;
 * calls on one stream are safe back to back.  Nothing in the array needs clearing between calls. */
#define EW_NOALLOC_MAX_BYTES ((uint64_t)1 << 30)
int ew_snapshot_noalloc(const void *src, void *dst, uint64_t nbytes, ew_cksum_t *cksums, void *stream);

/* ---- Integrity check of stored bytes (Live Remap step 1) ----------------------------------
 * Recomputes the block checksums of buf into got[] (device, ceil(nbytes/2^20) records,
 * overwritten) and compares them with expect[] (device).  *n_bad (device) receives the number
 * of differing blocks; the first min(*n_bad, cap) of them are listed in ascending order in
 * bad_blocks[] (device) with diffs[i] = (got.sum - expect.sum mod 2^64, got.xr ^ expect.xr)
 * (device, cap records).  bad_blocks/diffs may be NULL when cap = 0. */
int ew_verify(const void *buf, uint64_t nbytes, const ew_cksum_t *expect, ew_cksum_t *got,
              uint64_t *n_bad, uint64_t *bad_blocks, ew_cksum_t *diffs, uint64_t cap,
              void *stream);

/* What a bad block's differences say about the damage (host, pure arithmetic).  One flipped bit
 * at byte offset o, bit b of a buffer changes exactly one 64-bit word of block o >> 20 by
 * +-2^(8*(o mod 8) + b): the xor difference is one-hot and the sum difference is plus or minus the
 * same value mod 2^64.  Returns 1 if *diff (one record of ew_verify's diffs[], copied to the host)
 * has that form and then writes the bit lane 8*(o mod 8) + b (0..63) to *lane and +1 (the bit
 * reads 1 now and was 0 when the checksum was taken) or -1 to *direction; returns 0 otherwise
 * (several bits, or none).  In lane 63 both directions give the same differences: +1 is reported.
 * Which word of the block was hit cannot be told from (sum, xor). */
int ew_single_bit_flip(const ew_cksum_t *diff, uint32_t *lane, int32_t *direction);

/* ---- Gradient-shipping snapshot (Sec. 5.1, Fig. 6) --------------------------------------------
 * The paper keeps worker i's snapshot of worker (i+1)'s optimizer partition current without copying
 * the Adam state every step: worker i+1 ships the GRADIENT shard of its partition (device to device,
 * then device to host on worker i) and worker i's host CPU replays the optimizer update on the
 * snapshot in host memory.  The replay reproduces the owner's update bit for bit because both run
 * the same sequence of single fp32 operations (no fused multiply-add, correctly rounded divide and
 * square root):  m <- beta1*m + (1-beta1)*g;  v <- beta2*v + (1-beta2)*(g*g);
 * w <- w - lr*((m*bias1)/(sqrt(v*bias2) + eps) + weight_decay*w);  p <- bf16(w), nearest even. */
typedef struct {
  float lr, beta1, beta2;
  float omb1, omb2;   /* 1-beta1, 1-beta2, rounded once from float64 */
  float eps, wd;
  float bias1, bias2; /* 1/(1-beta1^t), 1/(1-beta2^t), rounded once from float64 */
} ew_adam_t;
/* Fills *out for optimizer step `step` (1-based).  EW_EINVAL for step 0 or betas outside [0, 1). */
int ew_adam_hyper(float lr, float beta1, float beta2, float eps, float weight_decay, uint64_t step, ew_adam_t *out);
/* The owner's step on its live shard: p_bf16, w, m, v (device, n elements each; updated in place),
 * grad (device, n elements of grad_elem_size 4 = fp32 or 2 = bf16).  Enqueued on `stream`. */
int ew_adam_step(void *p_bf16, float *w, float *m, float *v, const void *grad, uint32_t grad_elem_size, uint64_t n,
                 const ew_adam_t *h, void *stream);
/* The same update on a snapshot in HOST memory (all pointers host), split over n_threads host
 * threads (0 = all hardware threads).  Synchronous.  This runs on the CPU by the paper's design; it
 * is not a fallback for anything. */
int ew_adam_replay_host(void *p_bf16, float *w, float *m, float *v, const void *grad, uint32_t grad_elem_size,
                        uint64_t n, const ew_adam_t *h, uint32_t n_threads);
/* Ships a gradient shard: grad_dev -> peer_dev (device to device; NULL skips the hop) -> host_buf
 * (device to host; pinned host memory keeps it asynchronous; NULL skips it), on `stream`. */
int ew_grad_ship(const void *grad_dev, void *peer_dev, void *host_buf, uint64_t nbytes, void *stream);
/* Block checksums (as ew_snapshot's) of a HOST buffer into cksums (host), over n_threads threads:
 * upload them and run ew_verify on the live device shard to check a host snapshot against it. */
int ew_checksum_host(const void *buf, uint64_t nbytes, ew_cksum_t *cksums, uint32_t n_threads);

/* Plain device copy dst[0..nbytes) = src[0..nbytes) with the access pattern of the copy tiles
 * (one 128-bit vector per lane) and nothing else: the yardstick that benchmarks quote
 * the other kernels against and that profiler byte counters are calibrated with.  Not part of
 * the paper's method.  src, dst: device, 16-byte aligned, non-overlapping; nbytes a multiple of
 * 16 and at most (2^31-1) KiB, else EW_EINVAL. */
int ew_memcpy(const void *src, void *dst, uint64_t nbytes, void *stream);

/* Launch-shape knobs for benchmarking sweeps (process-wide; each is read and written atomically,
 * so setting one while other threads launch is safe; defaults are the tuned ones).  Names: "tile_bytes", "tile_elems", "tile_align_bytes", "cksum_sub_bytes",
 * "cksum_wgs_per_cu", "cksum_mode" (-1 = default: slot kernel + fold for ew_snapshot, atomic kernel
 * for ew_verify; 0 / 1 force the slot / atomic kernel for both), "snapshot_wave_min_bytes"
 * (ew_snapshot uses one-wave workgroups from this size on, 256-lane ones below; default: never),
 * "snapshot_xcd_group_kib" (ew_snapshot's chunks go to the XCDs in runs of this many KiB; default 128),
 * "fused_wgs_per_cu", "verify_wgs_per_cu", "adam_wgs_per_cu" (workgroups resident per CU for the
 * kernels of ew_unpack_snapshot, ew_verify and ew_adam_step; 0 = all that fit; defaults 0, 4, 10),
 * "verify_large_min_bytes", "verify_large_sub_bytes", "verify_large_wgs_per_cu" (from the first size on,
 * ew_verify reads in sub-blocks of up to the second size -- halved, down to 128 KiB, until every resident
 * workgroup gets five -- with the third number of workgroups per CU, instead of "cksum_sub_bytes" and
 * "verify_wgs_per_cu": fewer, longer streams; defaults 256 MiB, 512 KiB, 2),
 * "adam_xcd_group" (ew_adam_step's 256-element workgroups go to the XCDs in runs of this many; default 256),
 * "xcd_group_kib" (the tile kernels hand each of the 8 XCDs runs of consecutive tiles of this many
 * KiB instead of dealing tiles out one by one; 0 = one by one; default 2048),
 * "fused_mode" (0 = default; 1 forces the scratch-free form of ew_unpack_snapshot),
 * "fused_pass_tiles" (ew_unpack_snapshot cuts its tile kernel into launches of at most this many tiles;
 * 0 = one launch per scratch region; default 262144),
 * "fold_tiles_per_lane" (tiles each lane of ew_unpack_snapshot's fold kernel walks; 0 = default, 2),
 * "scratch_max_concurrent" (read-only statistic: the most calls that ever held a scratch region at
 * the same time; setting it to 0 resets it).
 * Returns EW_EINVAL for an unknown name or an out-of-range value. */
int ew_set_param(const char *name, int64_t value);
int64_t ew_get_param(const char *name);

const char *ew_strerror(int code);
const char *ew_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ELASWAVE_H */
