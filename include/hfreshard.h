/*
 * hfreshard — train <-> generation weight resharding of the HybridFlow
 * 3D-HybridEngine (arXiv 2409.19256, Section 5) on one MI355X (gfx950).
 *
 * All simulated ranks live in two device buffers of one process:
 *   train_buf : the N = p*t*d training shards (Megatron layout, fused QKV and
 *               fused gate/up), rank regions concatenated in rank order;
 *   gen_buf   : the generation partitions (separate q/k/v/gate/up) of the
 *               "materialised" ranks, concatenated in the order they were given.
 * The paper's all-gather inside each micro-DP group (Section 5.2 step 1,
 * Section 5.4) becomes a list of strided copy descriptors executed by one HIP
 * kernel; the re-partition for training (Section 5.2 step 4) is the inverse list.
 *
 * Conventions
 *   - plain C ABI, no exceptions cross it; every function that can fail returns
 *     0 (HF_OK) or a negative hf_status; hf_last_error() gives a thread-local text.
 *   - threads: queries and the execution entry points take a const plan and may run
 *     concurrently on one plan from several host threads (each on a stream of its own, on
 *     buffers the caller keeps apart); hf_plan_set_param, hf_debug_restrict_kinds and
 *     hf_plan_destroy need the plan for themselves.  hf_reshard_execute_static shares one
 *     staging array per GPU (see there).
 *   - "device pointer" = memory of the HIP device that was current when the plan
 *     was built; "host pointer" = ordinary process memory.
 *   - sizes and offsets are in BYTES unless a name says otherwise; weights are
 *     opaque 16-bit words (bf16), row-major [out, in].
 *   - byte layout of a rank region (both buffers): tensors in table order, each
 *     start rounded up to 256 B, region size rounded up to 4096 B.
 *     training order : embed (first stage) | per layer ln1 qkv o ln2 gate_up down |
 *                      lnf head (last stage)
 *     generation order: embed (first gen stage) | per layer ln1 q k v o ln2 gate up
 *                      down | lnf head (last gen stage)
 *     fused qkv [(n_q+2 n_kv)/t*hd, h]: per local KV group: its n_q/n_kv query
 *     heads, then its key head, then its value head.  fused gate_up [2F/t, h]: the
 *     rank's gate rows, then its up rows.
 */
#ifndef HFRESHARD_H
#define HFRESHARD_H

#include <stddef.h>
#include <stdint.h>

#if defined(HF_BUILD)
#define HF_API __attribute__((visibility("default")))
#else
#define HF_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HF_OK = 0,
  HF_EINVAL = -1, /* null pointer, non-positive size, elem_bytes != 2, tied embedding,
                     misaligned buffer, wrong direction, plan without device copy   */
  HF_EDIVIS = -2, /* t%t_g, p%p_g, L%p, L%p_g, V%t, F%t, n_q%n_kv, n_kv%t or n_kv%t_g != 0 */
  HF_ERANGE = -3, /* rank out of range or listed twice; index past the end; a size that
                     does not fit the descriptor fields                              */
  HF_ENOMEM = -4, /* host or device allocation failed while building the plan        */
  HF_EHIP = -5    /* HIP runtime error (no device, launch failure)                   */
} hf_status;

/* Model shape: a Llama-style decoder (RMSNorm vectors, GQA attention, SwiGLU MLP,
 * untied embedding / LM head).  The paper evaluates Llama 7B-70B (Section 8.1). */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  int32_t elem_bytes; /* must be 2 */
  int32_t tied_embed; /* must be 0 */
} hf_model_desc;

/* Training 3D-parallel sizes p-t-d (Section 5.1).  Rank r = dp*p*t + pp*t + tp:
 * TP and PP groups are consecutive ranks, DP groups are at stride p*t (Section 5.3). */
typedef struct {
  int32_t pp, tp, dp;
} hf_train_layout;

/* hf_gen_layout.flags */
#define HF_SKIP_OWN 0x0u         /* default: a rank's own pieces are resident in its
                                    generation buffer and are never copied (Section 5.3,
                                    zero redundancy; Section 5.4: only remote parameters
                                    are collected)                                       */
#define HF_COPY_OWN 0x1u         /* execute also copies the own pieces                  */
#define HF_GROUPING_VANILLA 0x2u /* HybridFlow-V grouping (Section 5.3, Figure 8(a)):
                                    consecutive ranks form generation TP/PP groups      */
#define HF_PLAN_HOST_ONLY 0x4u   /* build no device copy of the plan: every query works,
                                    execute/back/install return HF_EINVAL.  For hosts
                                    without a GPU.                                      */
#define HF_PLAN_OFFLOAD 0x8u     /* also build (and upload) the work lists of
                                    hf_offload_remote / hf_reload_remote                */
#define HF_GATHER_FROM_GEN 0x10u /* hf_reshard_execute reads every peer's piece from that
                                    peer's GENERATION buffer (where it is resident as the
                                    peer's own piece) instead of train_buf: the weights
                                    then exist once per rank, inside gen_buf, as in the
                                    paper (Section 5.3: the training weights are a sub-part
                                    of the generation weights; Section 5.4).  train_buf is
                                    not touched by execute and may be NULL there; the
                                    descriptors of direction 0 carry src_off relative to
                                    gen_buf.  Needs the HybridFlow grouping, HF_SKIP_OWN,
                                    and every member of the micro-DP group of a materialised
                                    rank materialised too (HF_EINVAL otherwise).            */

/* Generation sizes p_g-t_g (Section 5.1); the micro-DP size is derived,
 * d_g = p*t/(p_g*t_g).  mat_ranks (host pointer, copied) lists the ranks whose
 * generation buffer exists in gen_buf, in buffer order; NULL means all N ranks. */
typedef struct {
  int32_t pp, tp;
  uint32_t flags;
  const int32_t *mat_ranks;
  int32_t n_mat;
} hf_gen_layout;

typedef struct hf_plan hf_plan; /* opaque; owned by the library */

/* tensor ids (hf_desc.tensor_id is the id on the GENERATION side) */
enum {
  HF_T_EMBED = 0, HF_T_LN1, HF_T_QKV, HF_T_O, HF_T_LN2, HF_T_GATE_UP, HF_T_DOWN, HF_T_LNF, HF_T_HEAD,
  HF_G_EMBED = 16, HF_G_LN1, HF_G_Q, HF_G_K, HF_G_V, HF_G_O, HF_G_LN2, HF_G_GATE, HF_G_UP, HF_G_DOWN,
  HF_G_LNF, HF_G_HEAD
};

/* hf_desc.kind */
enum {
  HF_COL = 0,          /* column-parallel: concatenate along dim 0 (embed, head)       */
  HF_ROW = 1,          /* row-parallel: concatenate along dim 1 (o, down)              */
  HF_REPL = 2,         /* replicated vector (norms)                                    */
  HF_QKV_DEINT = 3,    /* fused qkv <-> separate q / k / v                              */
  HF_GATEUP_DEINT = 4  /* fused gate_up <-> separate gate / up                          */
};

/* hf_desc.flags */
#define HF_DESC_OWN 0x1u     /* source rank == destination rank                         */
#define HF_DESC_ALIGN16 0x10u /* widest vector that divides every offset, stride, size  */
#define HF_DESC_ALIGN8 0x20u
#define HF_DESC_ALIGN4 0x40u
#define HF_DESC_ALIGN2 0x80u

/* One strided copy: n_blocks x rows x row_bytes.
 * byte (b, r, i) of the source, at src_off + b*src_block_stride + r*src_row_stride + i,
 * goes to dst_off + b*dst_block_stride + r*dst_row_stride + i.  For the direction
 * train->gen src_off is relative to train_buf and dst_off to gen_buf; for gen->train
 * the other way round. */
typedef struct {
  int32_t src_rank, dst_rank, tensor_id, layer; /* layer = -1 for embed / lnf / head */
  uint32_t kind, flags;
  uint64_t src_off, dst_off;
  uint32_t n_blocks, rows, row_bytes, _pad;
  uint64_t src_block_stride, dst_block_stride, src_row_stride, dst_row_stride;
} hf_desc;

/* One tensor of one rank region. */
typedef struct {
  int32_t tensor_id, layer;
  uint32_t rows, cols;   /* elements */
  uint64_t offset;       /* bytes from the base of train_buf / gen_buf */
  int32_t tp_index;      /* TP index of the slice (training) or generation TP index;
                            0 for replicated tensors */
  int32_t replicated;    /* 1 for norm vectors */
} hf_tensor_info;

/* One unit of device work (what a workgroup copies at a time): rows x row_bytes with
 * byte strides; produced from the descriptors by the planner's tiler. */
typedef struct {
  uint64_t src_off, dst_off; /* dst_off: the first destination                          */
  uint32_t rows, row_bytes;
  uint32_t src_row_stride, dst_row_stride;
  uint32_t vec_bytes;    /* 16, 8, 4 or 2: widest access that is aligned everywhere */
  uint32_t n_dst;        /* Multicast: the source tile is read once and written to
                            n_dst destinations with the same row stride (one training
                            piece wanted by several ranks of a micro-DP group).  0 = a
                            load-only tile: loaded and stored nowhere (dst_off unused)   */
  uint32_t dst_list;     /* n_dst > 1: position of destinations 2..n_dst in the plan's list
                            of extra destination offsets (see hf_plan_get_tile_dst).
                            n_dst == 0: 0 = the rows are loaded like those of a copy tile;
                            c > 0 (= rows, at most HF_MAX_PREFETCH_CHUNKS) = chunked form:
                            the rows are c source chunks that c later copy tiles read, and
                            the workgroup with part number k loads part k of EVERY chunk
                            (the bytes the workgroups with part number k of those copy
                            tiles will want; same workgroup index mod 8 = same XCD)      */
  uint32_t _pad;
} hf_tile;

#define HF_MAX_PREFETCH_CHUNKS 8

#define HF_DIR_TRAIN_TO_GEN 0
#define HF_DIR_GEN_TO_TRAIN 1
#define HF_DIR_OFFLOAD 2 /* gen_buf -> packed host image of the remote pieces */
#define HF_DIR_RELOAD 3  /* packed host image -> gen_buf                      */
#define HF_BUF_TRAIN 0
#define HF_BUF_GEN 1

/* ---- plan -------------------------------------------------------------------
 * hf_reshard_plan: host work only plus one upload of the tile lists to the current
 * HIP device (unless HF_PLAN_HOST_ONLY).  Builds rank coordinates (Section 5.3),
 * tensor tables, and the copy descriptors of step 1 and step 4 (Section 5.2).  All
 * argument structs are host pointers and are copied.  *out receives the plan; the
 * caller releases it with hf_plan_destroy (which frees the device copy). */
HF_API int hf_reshard_plan(const hf_model_desc *model, const hf_train_layout *train, const hf_gen_layout *gen,
                    hf_plan **out);
HF_API void hf_plan_destroy(hf_plan *plan);

/* ---- execution ----------------------------------------------------------------
 * train_buf / gen_buf: DEVICE pointers, 256-byte aligned, at least
 * hf_plan_train_bytes / hf_plan_gen_bytes long, not overlapping; they may be two
 * offsets into one allocation.  hip_stream: a hipStream_t (NULL = default stream).
 * The calls enqueue one kernel launch on that stream (a few for work lists beyond
 * 16.7 million workgroups, see HF_PARAM_MAX_WGS_PER_LAUNCH) and return; they never
 * allocate, synchronise or touch host copies of the buffers.  Padding between tensors is never
 * written.
 *
 * hf_reshard_execute (Section 5.2 step 1; Section 5.4): fills the generation buffers
 *   of the materialised ranks from the training shards of their micro-DP groups.
 *   Under HF_SKIP_OWN the own pieces are left alone (they must already be resident,
 *   see hf_reshard_install_own); under HF_COPY_OWN they are copied too.
 * hf_reshard_back (Section 5.2 step 4): rewrites the training shard of every
 *   materialised rank from that rank's own generation buffer.  HF_EINVAL for a plan
 *   with HF_GROUPING_VANILLA, where the training shard is not inside the generation
 *   buffer (Section 5.3) and has to be kept besides it instead.
 * hf_reshard_install_own: copies only the own pieces train_buf[r] -> gen_buf[r]: what
 *   makes HF_SKIP_OWN's residency assumption true.
 *
 * Freshness contract.  train_buf and gen_buf are separate memory, so under HF_SKIP_OWN
 * the own pieces inside gen_buf[r] are as old as the last hf_reshard_install_own (or the
 * last write of the caller through the own view, hf_plan_get_own_view, which is where a
 * trainer that updates the weights in place inside the generation buffer keeps them).  A
 * caller that updates train_buf instead must refresh the own pieces after every update:
 * either hf_reshard_execute + hf_reshard_install_own on a HF_SKIP_OWN plan, or one
 * hf_reshard_execute on a HF_COPY_OWN plan (one launch, every byte of every generation
 * buffer rewritten).  hf_reshard_execute alone on a HF_SKIP_OWN plan moves exactly the
 * bytes the paper's all-gather moves between GPUs (Section 5.4) and nothing else.  With
 * HF_GATHER_FROM_GEN there is no second copy to go stale: the peers' pieces are gathered
 * from the owners' generation buffers, which is where such a trainer keeps the weights. */
HF_API int hf_reshard_execute(const hf_plan *plan, const void *train_buf, void *gen_buf, void *hip_stream);
HF_API int hf_reshard_back(const hf_plan *plan, void *train_buf, const void *gen_buf, void *hip_stream);
HF_API int hf_reshard_install_own(const hf_plan *plan, const void *train_buf, void *gen_buf, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture set-up,
 * tight serving loops, harnesses that forbid hipMalloc): hf_reshard_execute with the work
 * list staged in a static device array of the library instead of a hipMalloc'ed copy owned by
 * the plan.  The plan may therefore be built with HF_PLAN_HOST_ONLY (no device memory is ever
 * allocated for it); train_buf / gen_buf and the result are as for hf_reshard_execute.
 * The call copies the plan's current train->gen work list into the array on hip_stream (only
 * if the array does not already hold it) and enqueues the same kernel; it calls no
 * hipMalloc / hipFree and does not synchronise.  HF_ERANGE if the work list is larger than
 * HF_STATIC_SCRATCH_BYTES (about 349 000 tiles: the Llama-7B transition fits, the larger
 * ones need a larger HF_PARAM_TILE_BYTES).  Every GPU holds one such array until the process
 * ends, and every call on a GPU uses it: calls that overlap on one GPU (different streams,
 * different plans) race; calls on one stream, or separated by synchronisation, do not. */
#define HF_STATIC_SCRATCH_BYTES (16u << 20)
HF_API int hf_reshard_execute_static(const hf_plan *plan, const void *train_buf, void *gen_buf, void *hip_stream);

/* Section 5.2 step 3: all-gather of the generation results inside each micro-DP group.
 * resp_in  (DEVICE, 256-byte aligned): N slots of slot_bytes; slot r holds the results
 *          (prompt + response token ids, any 4-byte-multiple payload) that rank r's
 *          generation replica produced for its micro-batch.
 * resp_out (DEVICE, 256-byte aligned, not overlapping resp_in): N * d_g slots; after the
 *          call, slots r*d_g .. r*d_g+d_g-1 hold the results of the d_g members of rank r's
 *          micro-DP group in the order of their micro-DP index (member j = the rank
 *          hf_plan_micro_dp_peer(plan, r, j)), i.e. every rank of a training replica ends up
 *          with the whole batch of its micro-DP group, ready for the training stage.
 * slot_bytes: > 0, multiple of 4; may change from call to call (the group table is part of
 * the plan, nothing is allocated or uploaded here).  One kernel launch on hip_stream. */
HF_API int hf_gather_responses(const hf_plan *plan, const void *resp_in, void *resp_out, size_t slot_bytes,
                        void *hip_stream);
/* rank with micro-DP index j (0 <= j < d_g) in the micro-DP group of `rank`; -1 if out of range */
HF_API int hf_plan_micro_dp_peer(const hf_plan *plan, int rank, int j);

/* ---- offload / reload of the remote pieces (Section 7, "Implementation": the weights of
 * the generation stage are kept in a buffer of their own, moved to host memory while the
 * model trains and brought back in the transition).  What leaves the GPU is exactly what
 * the transition gathered: the pieces of the d_g-1 micro-DP peers in every materialised
 * generation buffer; the own pieces (the training shard, Section 5.3) stay.
 * host_buf: PINNED host memory that the device can address (hipHostMalloc; torch's
 *   pin_memory), 256-byte aligned, at least hf_plan_remote_bytes long.  Packed image: for
 *   every materialised rank in buffer order (part starts rounded up to 4096 B; see
 *   hf_plan_remote_rank_offset), for every generation tensor in table order that has
 *   remote elements (tensor parts rounded up to 256 B): its remote elements in row-major
 *   order.  Bytes between the parts are never written.
 * Both calls need a plan built with HF_PLAN_OFFLOAD; they enqueue one kernel on hip_stream
 * that reads / writes host_buf across the host link, and never allocate or synchronise.
 * hf_offload_remote leaves gen_buf as it is (the caller may then reuse the remote parts);
 * hf_reload_remote writes only remote pieces: own pieces and padding are left alone.
 * HF_EINVAL if host_buf is not pinned host memory. */
HF_API int hf_offload_remote(const hf_plan *plan, const void *gen_buf, void *host_buf, void *hip_stream);
HF_API int hf_reload_remote(const hf_plan *plan, const void *host_buf, void *gen_buf, void *hip_stream);
HF_API size_t hf_plan_remote_bytes(const hf_plan *plan);                /* size of the packed image */
HF_API size_t hf_plan_remote_rank_offset(const hf_plan *plan, int rank); /* (size_t)-1 if not mat.  */

/* Host-side check of a caller's buffers against the plan, for set-up code (not needed on
 * the hot path): HF_EINVAL if a pointer is null or not 256-byte aligned, if the ranges
 * overlap, or if train_len / gen_len (bytes the caller owns from the pointers on) are
 * smaller than hf_plan_train_bytes / hf_plan_gen_bytes.  With a device plan the ranges
 * must also lie inside device allocations of the HIP runtime (HF_ERANGE otherwise).
 * train_buf may be null (train_len is then ignored) for a HF_GATHER_FROM_GEN plan. */
HF_API int hf_plan_check_buffers(const hf_plan *plan, const void *train_buf, size_t train_len, const void *gen_buf,
                          size_t gen_len);

/* Plain 16-byte grid-stride copy of `bytes` (multiple of 16) from src to dst (DEVICE
 * pointers, 16-byte aligned, not overlapping) on hip_stream: a kernel of known traffic,
 * for calibrating hardware counters and for measuring the copy ceiling of a box.
 * dst == NULL: only reads src; src == NULL: only writes dst (a constant pattern).  Not
 * part of the paper's method. */
HF_API int hf_calib_copy(const void *src, void *dst, size_t bytes, void *hip_stream);
/* One read, n_dst writes: `bytes` of src go to dst, dst + dst_stride, ..., n_dst places
 * (1 <= n_dst <= 8; DEVICE pointers, 256-byte aligned; bytes a multiple of 8192;
 * dst_stride >= bytes, multiple of 256; nothing overlaps).  The traffic mix of a
 * transition in which every training piece is wanted by n_dst ranks, without any of its
 * geometry: the ceiling such a mix can reach on a box.
 * method HF_FANOUT_REGISTERS: every workgroup loads its part once and stores it n_dst times
 *   (block_bytes ignored);
 * HF_FANOUT_CACHE_BLOCKED: a block of block_bytes (multiple of 64 KiB) of the source is
 *   copied to the first place, then the same block to the second, ... (re-reads served by
 *   L2), like the library's cache-blocked work list;
 * HF_FANOUT_PREFETCHED: a block is first loaded by workgroups that store nothing, then
 *   loaded again (from L2) and stored n_dst times, like the library's prefetched list.
 * wg_bytes: bytes per workgroup, 1024 (one wavefront), 4096 or 8192.  src == NULL: only the
 * n_dst writes (of a constant pattern); dst == NULL: only the read (both: method
 * HF_FANOUT_REGISTERS only).  Not part of the paper's method. */
enum { HF_FANOUT_REGISTERS = 0, HF_FANOUT_CACHE_BLOCKED = 1, HF_FANOUT_PREFETCHED = 2 };
HF_API int hf_calib_fanout(const void *src, void *dst, size_t bytes, int n_dst, size_t dst_stride, int method,
                    size_t block_bytes, int wg_bytes, void *hip_stream);

/* ---- tuning (host; takes effect on the next launch) -----------------------------
 * HF_PARAM_TILE_BYTES, HF_PARAM_MC_BLOCK_BYTES, HF_PARAM_PREFETCH_BLOCK_BYTES, HF_PARAM_PREFETCH_MERGE
 * and HF_PARAM_ROW_INTERLEAVE re-tile and re-upload; HF_PARAM_MULTICAST uploads the work list of
 * the new mode and frees the old one (they allocate; not for the hot path).  Only the work lists of the current mode are resident on the device. */
enum {
  HF_PARAM_TILE_BYTES = 0,   /* bytes of work per tile, 4096 .. 4 MiB, multiple of 4096   */
  HF_PARAM_GRID_WGS = 1,     /* workgroups of the persistent kernels, 1 .. 65536          */
  HF_PARAM_VARIANT = 2,      /* HF_VARIANT_*                                              */
  HF_PARAM_MULTICAST = 3,    /* HF_MULTICAST_*: how train->gen serves a training piece that
                                several ranks of a micro-DP group want.  Same result in
                                every mode; the modes differ in HBM reads and in speed.
                                Default (and HF_MULTICAST_AUTO): chosen from the fan-out of
                                the list, i.e. bytes written per distinct byte read, as
                                measured: about 2 -> REGISTERS, 3 and more -> PREFETCHED
                                (re-chosen when the list is rebuilt;
                                hf_plan_get_param returns the mode in force).  When no piece
                                of the plan has more than one destination (e.g. only one
                                rank per micro-DP group is materialised) every mode runs
                                as HF_MULTICAST_OFF, and hf_plan_get_param says so.      */
  HF_PARAM_CACHE_POLICY = 4, /* -1 (default): chosen by the library (0 for one-to-one
                                streaming lists, 5 for the cache-blocked and the prefetched
                                list, 4 for the register-multicast list); 0 = non-temporal loads and
                                system-scope streaming stores; bit 0 = plain loads,
                                bit 1 = plain stores, 4 / 5 = compiler non-temporal stores
                                with non-temporal / plain loads (not for
                                HF_VARIANT_LDS_STAGED)                                   */
  HF_PARAM_PART_BYTES = 5,   /* HF_VARIANT_PARTS: payload bytes per workgroup: a power of two
                                from 4096 to 32768 (1024 to 8192 with 64-lane workgroups;
                                values outside the range are clamped), or 0 (default) =
                                automatic: 8192 for the cache-blocked train->gen list,
                                1024 for every other list                                */
  HF_PARAM_MC_BLOCK_BYTES = 6, /* HF_MULTICAST_CACHE_BLOCKED: source bytes per block,
                                1 MiB .. 1 GiB, default 2 MiB (re-tiles and re-uploads)  */
  HF_PARAM_MAX_WGS_PER_LAUNCH = 8, /* HF_VARIANT_PARTS / ONE_WG_PER_TILE: a work list that needs
                                more workgroups goes out in several launches of at most this
                                many 256-lane workgroups (four times as many 64-lane ones),
                                in list order; 1024 .. 16777215 (default: a HIP grid holds
                                fewer than 2^32 threads)                                  */
  HF_PARAM_WG_THREADS = 9,   /* HF_VARIANT_PARTS: lanes per workgroup: 256, 64, or 0 (default) =
                                automatic: 256 for the cache-blocked train->gen list, 64
                                (one wavefront) for every other list                     */
  HF_PARAM_PREFETCH_BLOCK_BYTES = 12, /* HF_MULTICAST_PREFETCHED: source bytes per block, 1 MiB ..
                                64 MiB, default 6 MiB: the eight 4 MiB L2s must hold a block
                                until its copies are done (re-tiles and re-uploads)        */
  HF_PARAM_PREFETCH_MERGE = 13, /* HF_MULTICAST_PREFETCHED: up to this many copy tiles that follow
                                one another in the source share one chunked load-only tile, whose
                                wavefronts then have that many loads in flight; 1 ..
                                HF_MAX_PREFETCH_CHUNKS, or 0 (default) = the library's choice
                                (2, as measured) (re-tiles and re-uploads)                 */
  HF_PARAM_ROW_INTERLEAVE = 11, /* 1 (default): the tiles of the column stripes that several
                                training ranks contribute to one row-parallel generation
                                tensor (o, down) go out round-robin, so that a destination
                                row is completed while it is open; 0: stripe after stripe
                                (re-tiles and re-uploads)                                 */
  HF_PARAM_OFFLOAD_WGS = 10  /* persistent workgroups of hf_offload_remote / hf_reload_remote,
                                1 .. 4096.  Default 8: measured, that many keep the host link
                                as busy as the runtime's copy engine does, while a reshard on
                                another stream runs at its own speed; hundreds of workgroups
                                gain nothing on the link and their queued host writes slow
                                every other kernel's memory traffic by orders of magnitude */
};
enum {
  HF_MULTICAST_AUTO = -1,     /* hf_plan_set_param only: back to the library's choice     */
  HF_MULTICAST_OFF = 0,       /* one read per destination, destination-major order        */
  HF_MULTICAST_REGISTERS = 1, /* a workgroup loads a tile once and stores it to every
                                 destination                                             */
  HF_MULTICAST_CACHE_BLOCKED = 2, /* one destination per workgroup, work ordered so
                                 that a block of source is copied to destination 1, then
                                 the same block to destination 2, ...; the re-reads are
                                 served by L2 instead of HBM                             */
  HF_MULTICAST_PREFETCHED = 3 /* as HF_MULTICAST_REGISTERS, but every block of
                                 HF_PARAM_PREFETCH_BLOCK_BYTES of source is first touched
                                 by workgroups that only load it (tiles with n_dst == 0),
                                 so that the workgroups that store it to all destinations
                                 find it in L2 and spend their life on stores          */
};
enum {
  HF_VARIANT_PERSISTENT = 0, /* persistent workgroups stride over the tile list, direct
                                global->register->global 16-byte accesses               */
  HF_VARIANT_ONE_WG_PER_TILE = 1, /* same copy loop, one workgroup per tile             */
  HF_VARIANT_LDS_STAGED = 2, /* persistent, tile staged through LDS                     */
  HF_VARIANT_WAVE_PERSISTENT = 3, /* persistent, every WAVEFRONT strides over the tile
                                list on its own (wavefront-level dispatch)              */
  HF_VARIANT_PARTS = 4       /* one short-lived workgroup per HF_PARAM_PART_BYTES of every
                                tile, handed out in order by the hardware dispatcher    */
};
HF_API int hf_plan_set_param(hf_plan *plan, int param, int64_t value);
HF_API int64_t hf_plan_get_param(const hf_plan *plan, int param);

/* ---- profiling aid, NOT for production ---------------------------------------------
 * Restricts the plan to the descriptors of some kinds: bit k of kind_mask set = kind k
 * (HF_COL .. HF_GATEUP_DEINT) takes part; 31 = all (the state of a new plan).  Serves to
 * time one tensor kind at a time.  While the mask is not 31, execute / back / install_own
 * copy ONLY those kinds, hf_plan_bytes_moved / hf_plan_unique_src_bytes count only them
 * and hf_plan_validate fails.  Re-tiles and re-uploads (allocates). */
HF_API int hf_debug_restrict_kinds(hf_plan *plan, int kind_mask);

/* ---- queries (host only, no device work) --------------------------------------- */
HF_API size_t hf_plan_train_bytes(const hf_plan *plan);              /* required size of train_buf */
HF_API size_t hf_plan_gen_bytes(const hf_plan *plan);                /* required size of gen_buf   */
HF_API int hf_plan_num_ranks(const hf_plan *plan);                   /* N = p*t*d                  */
HF_API int hf_plan_num_mat(const hf_plan *plan);
HF_API int hf_plan_mat_rank(const hf_plan *plan, int i);             /* i-th materialised rank, -1 */
HF_API size_t hf_plan_rank_train_offset(const hf_plan *plan, int rank); /* (size_t)-1 on bad rank  */
HF_API size_t hf_plan_rank_gen_offset(const hf_plan *plan, int rank);   /* (size_t)-1 if not mat.  */
/* out[6] = dp, pp, tp, gpp, gtp, micro-DP index (Section 5.3) */
HF_API int hf_plan_rank_coords(const hf_plan *plan, int rank, int32_t out[6]);
HF_API int hf_plan_micro_dp_size(const hf_plan *plan);               /* d_g (Section 5.1)          */
HF_API size_t hf_plan_num_tensors(const hf_plan *plan, int which_buf, int rank);
HF_API int hf_plan_get_tensor(const hf_plan *plan, int which_buf, int rank, size_t i, hf_tensor_info *out);
/* copy descriptors that execute (direction 0) / back (direction 1) / offload (2: src_off
 * in gen_buf, dst_off in the host image) / reload (3: the other way round) perform */
HF_API size_t hf_plan_num_desc(const hf_plan *plan, int direction);
HF_API int hf_plan_get_desc(const hf_plan *plan, int direction, size_t i, hf_desc *out);
HF_API size_t hf_plan_bytes_moved(const hf_plan *plan, int direction); /* sum n_blocks*rows*row_bytes */
/* bytes of distinct source addresses those descriptors read (a training shard read by
 * several generation ranks counts once) */
HF_API size_t hf_plan_unique_src_bytes(const hf_plan *plan, int direction);
/* own view: where the pieces of rank's own training shard sit in its generation
 * buffer (src_off in train_buf, dst_off in gen_buf); the zero-redundancy overlap */
HF_API size_t hf_plan_num_own_view(const hf_plan *plan, int rank);
HF_API int hf_plan_get_own_view(const hf_plan *plan, int rank, size_t i, hf_desc *out);
/* device work list of a direction (0..3), in launch order (for host-side checking) */
HF_API size_t hf_plan_num_tiles(const hf_plan *plan, int direction);
HF_API int hf_plan_get_tile(const hf_plan *plan, int direction, size_t i, hf_tile *out);
/* k-th destination offset (0 <= k < n_dst) of tile i */
HF_API int hf_plan_get_tile_dst(const hf_plan *plan, int direction, size_t i, uint32_t k, uint64_t *out);
/* full consistency check of the plan on the host: destinations pairwise disjoint and
 * inside tensor payloads, sources inside tensor payloads, tiles cover the descriptors
 * exactly.  O(bytes/row) time: meant for tests, not for the hot path. */
HF_API int hf_plan_validate(const hf_plan *plan);

HF_API const char *hf_last_error(void);
HF_API const char *hf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HFRESHARD_H */
