/* chunkflow.h -- C ABI of the layerwise-offloaded DiT block path for one MI355X (gfx950).
 *
 * What the library does: runs one GPU's Ulysses share of a diffusion-transformer block
 * forward (App. B block designs; Sec. 2.1 for the Ulysses split) while that block's bf16
 * weights are streamed from pinned host memory in fixed-size chunks on a copy stream
 * (Sec. 2.2 layerwise offloading loop; Sec. 3.2 chunked prefetch with pause/resume at chunk
 * boundaries; Sec. 3.3 chunk-granular partial residency).
 *
 * Conventions
 *   - Every function returns 0 on success or a negative cf_status; cf_last_error() gives text.
 *   - Pointers named `host_*` are host memory, everything inside cf_block_io is DEVICE memory.
 *   - The caller owns all host blobs and all device tensors it passes in.  The library owns its
 *     context, its events, the two staging slots, the per-block resident buffers and (when the
 *     pause/resume worker is enabled) one host thread.  Nothing is freed behind the caller's back.
 *   - Streams are hipStream_t handles passed as void*.  Calls only enqueue work unless stated.
 *     Calls that block the host until the GPU is idle: cf_sync, cf_destroy, set_resident_fraction,
 *     cf_set_contention, cf_checksum_block, cf_op_checksum, cf_read_block, cf_kernel_times.
 *     Calls that may block the host for a bounded time, to keep it at most one block forward ahead of
 *     the GPU: chunked_prefetch_begin (whenever it has chunks to copy) and dit_block_fwd (while
 *     emulated collectives are enabled); each waits for the block forward issued two forwards earlier.
 *     The prefetch worker of pause/resume mode is a host thread of the library's own; it never blocks
 *     the caller except inside dit_block_fwd, which waits until the worker has enqueued the chunk a
 *     layer needs.
 *   - bf16 tensors are uint16_t bit patterns.  The residual stream (x in, y out) is fp32.
 *   - A context is not thread-safe; use it from one host thread.
 */
#ifndef CHUNKFLOW_H
#define CHUNKFLOW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cf_ctx cf_ctx;

typedef enum {
    CF_OK = 0,
    CF_ERR_ARG = -1,         /* bad argument (shape, alignment, range, null pointer)            */
    CF_ERR_STATE = -2,       /* call order violated (wait before begin, slot still in use, ...) */
    CF_ERR_HIP = -3,         /* a HIP runtime call failed; text has hipGetErrorString           */
    CF_ERR_NOMEM = -4,       /* device or host allocation failed                                */
    CF_ERR_UNSUPPORTED = -5  /* valid request this build does not implement                     */
} cf_status;

/* Block designs of App. B. */
typedef enum {
    CF_SINGLE_STREAM = 0,    /* MM-DiT single-stream: fused linear_1 (QKV + MLP-up), linear_2    */
    CF_DIT_CROSS = 1,        /* DiT: self-attention, cross-attention to text, MLP                */
    CF_DOUBLE_STREAM = 2     /* MM-DiT double-stream: per-stream weights, joint attention        */
} cf_block_kind;

/* Shape of one rank's share.  n_local = n_total / sp_degree tokens go through the linear
 * layers; attention covers all n_total tokens for heads [sp_rank*H/P, (sp_rank+1)*H/P).
 * Tokens split contiguously per stream; for CF_DOUBLE_STREAM the joint order is text then image
 * and the local rows are this rank's n_txt_local text rows followed by its image rows. */
typedef struct {
    int32_t kind;            /* cf_block_kind */
    int32_t n_blocks;
    int32_t d;               /* hidden size, multiple of 256, <= 4096 */
    int32_t n_heads;         /* H; d == n_heads * head_dim */
    int32_t head_dim;        /* 64 or 128 */
    int32_t f;               /* MLP width, multiple of 64 */
    int32_t n_total;         /* N */
    int32_t sp_degree;       /* P; divides n_heads, n_total (and n_txt_total) */
    int32_t sp_rank;
    int32_t n_txt_total;     /* text tokens leading the joint sequence (double-stream and mixed models), else 0 */
    int32_t l_ctx;           /* CF_DIT_CROSS: context length, else 0 */
    int32_t qk_rmsnorm;      /* per-head RMSNorm on q and k (learned weight, eps 1e-6) */
    int32_t gelu_erf;        /* MLP activation: 0 = tanh approximation of GELU, 1 = x * Phi(x) with erf */
    int32_t batch;           /* B of App. B: independent samples per forward, each with its own timestep  */
                             /*   embedding; 0 or 1 = one sample.  Linear layers run on B * n_local rows,  */
                             /*   attention per sample; the weights are fetched once for the whole batch   */
    uint64_t chunk_bytes;    /* C of Sec. 3.2; multiple of 256 */
} cf_model_desc;

/* One tensor of the block's weight blob: bf16 [rows, cols] row-major at byte `offset`
 * (256-byte aligned).  Linear weights are [out_features, in_features]. */
typedef struct {
    char name[32];
    uint64_t offset;
    uint32_t rows, cols;
} cf_tensor_slot;

/* Device buffers of one block invocation.  Peer buffers stand in for what the two Ulysses
 * exchanges around attention deliver; send buffers receive what this rank would have sent.
 * With sp_degree == 1 all peer/send pointers are ignored.  Send pointers may be NULL.
 * With batch = B > 1 every tensor below except the rotary tables gains a leading dimension B
 * (sample after sample, dense: x is [B, n_local, d], temb [B, d], peer_q [B, H/P, N - n_local, hd],
 * ...); the residual streams alone may be strided between samples (x_sample_stride). */
typedef struct {
    const float* x;              /* [n_local, d] (double-stream: the image rows) residual stream in */
    const float* x_txt;          /* double-stream: [n_txt_local, d] */
    const float* temb;           /* [d] timestep embedding */
    const uint16_t* ctx;         /* DiT: [l_ctx, d] bf16 text context */
    const uint16_t* peer_q;      /* [H/P, N - n_local, hd] q of remote tokens, this rank's heads */
    const uint16_t* peer_k;
    const uint16_t* peer_v;
    const uint16_t* peer_attn;   /* [n_local, H - H/P, hd] attention output of the other heads */
    const float* rope_cos;       /* optional rotary position tables [n_local, hd/2] for this rank's rows */
    const float* rope_sin;       /*   (text rows first): after the per-head norm, every head's q and k  */
                                 /*   pairs (2i, 2i+1) are rotated by angle i of the row; both or neither; */
                                 /*   peer_q / peer_k arrive rotated; not applied to cross-attention     */
    float* y;                    /* [n_local, d] (double-stream: image rows) residual stream out */
    float* y_txt;                /* double-stream: [n_txt_local, d] */
    uint16_t* send_q;            /* [H - H/P, n_local, hd] */
    uint16_t* send_k;
    uint16_t* send_v;
    uint16_t* send_attn;         /* [H/P, N - n_local, hd] */
    void* workspace;             /* >= cf_workspace_bytes, 256-byte aligned */
    uint64_t workspace_bytes;
    int64_t x_sample_stride;     /* batch > 1: elements from one sample's x (and y) to the next; 0 = dense.      */
    int64_t x_txt_sample_stride; /*   same for x_txt / y_txt.  With both set to n_local * d, x_txt = buf and     */
                                 /*   x = buf + n_txt_local * d view one [B, n_local, d] buffer of text-then-    */
                                 /*   image rows, the layout single-stream blocks of a mixed model take as x     */
} cf_block_io;

typedef struct {
    uint64_t h2d_bytes;          /* bytes copied by chunked_prefetch_begin since the last reset   */
    uint64_t h2d_chunks;
    uint64_t resident_bytes;     /* per block (mixed-kind model: mean over its blocks, rounded down) */
    uint64_t blob_bytes;
    uint64_t weight_memory_bytes;/* device bytes held for weights: resident buffers + 2 slots     */
    uint64_t comm_bytes_h2d;     /* emulated collective traffic                                   */
    uint64_t comm_bytes_d2h;
    uint64_t pauses;             /* chunk launches that were made to wait for a collective        */
    uint64_t model_resident_bytes;/* resident bytes summed over all blocks                          */
    uint64_t model_blob_bytes;   /* blob bytes summed over all blocks                              */
    uint64_t blocks_one_wait;    /* block forwards that waited once for all their chunks (see below) */
} cf_stats_t;

/* Per-kernel timing collected while profiling is on (cf_set_profiling). */
typedef struct {
    char name[32];
    uint64_t launches;
    double total_ms;             /* sum of hipEvent-measured durations */
    double flops;                /* algorithmic FLOPs summed over those launches (0 if n/a) */
    double bytes;                /* algorithmic HBM bytes summed over those launches (0 if n/a) */
} cf_kernel_time;

/* What the overlap model needs to know about the machine (Sec. 3.1: eta_c * P_peak and
 * eta_p * BW enter only through these measured figures). */
typedef struct {
    double t_comp_ms[3];         /* compute time of one block of each cf_block_kind, everything resident */
    double link_gbs;             /* achieved host-to-device rate of chunk copies, 1e9 bytes/s            */
    double chunk_overhead_us;    /* fixed cost per chunk copy (launch + event), 0 if unknown             */
} cf_machine_t;

typedef struct {
    double step_ms;              /* predicted steady-state step time                                      */
    double compute_ms;           /* sum of the blocks' compute times                                      */
    double exposed_ms;           /* step_ms - compute_ms: prefetch time the compute could not hide        */
    uint64_t weight_memory_bytes;/* resident parts of all blocks + two staging slots (Sec. 3.3)           */
    uint64_t h2d_bytes_per_step;
    double resident_fraction;    /* byte fraction actually resident for the requested r                   */
} cf_sim_result;

typedef struct {
    uint64_t chunk_bytes;
    double r;
    int32_t feasible;            /* 1 if the choice meets the constraint, 0 if nothing did (closest given) */
    cf_sim_result sim;
} cf_tune_choice;

/* ---- context and layout (Sec. 3.2: a layer's parameters are partitioned into fixed-size chunks).
 * cf_create validates the description and plans blob layout and chunking; it touches no GPU. */
int cf_create(const cf_model_desc* desc, cf_ctx** out);
int cf_destroy(cf_ctx* ctx);                                   /* syncs, frees everything it owns */
const char* cf_last_error(const cf_ctx* ctx);                  /* ctx may be NULL: last create error */
int cf_blob_bytes(const cf_ctx* ctx, uint64_t* out);            /* of block 0; every block's in a one-kind model */
int cf_n_chunks(const cf_ctx* ctx, int32_t* out);
/* tensors in blob order; *n is capacity on entry, count on return (call with out=NULL to query) */
int cf_blob_layout(const cf_ctx* ctx, cf_tensor_slot* out, int32_t* n);
int cf_workspace_bytes(const cf_ctx* ctx, uint64_t* out);      /* enough for every kind in the model */
/* A model that mixes block kinds (App. B: MMDiT = double-stream blocks followed by single-stream
 * blocks over the concatenated text+image sequence): kinds[b] is the cf_block_kind of block b,
 * n must equal n_blocks.  Call right after cf_create, before any block is registered.  Each kind
 * has its own blob layout and chunk count (same chunk_bytes); the two staging slots are sized for
 * the kind with the most streamed bytes; set_resident_fraction keeps the leading
 * round(r * n_chunks(kind)) chunks of every block.  With n_txt_total > 0 a single-stream block's
 * rows are this rank's text rows followed by its image rows, at the joint positions the
 * double-stream blocks use, so x_txt/x of one kind and x of the other can alias one buffer. */
int cf_set_block_kinds(cf_ctx* ctx, const int32_t* kinds, int32_t n);
int cf_block_kind_of(const cf_ctx* ctx, int32_t block, int32_t* out);
int cf_blob_bytes_of(const cf_ctx* ctx, int32_t block, uint64_t* out);
int cf_n_chunks_of(const cf_ctx* ctx, int32_t block, int32_t* out);
int cf_blob_layout_of(const cf_ctx* ctx, int32_t block, cf_tensor_slot* out, int32_t* n);
/* Host-only view of how dit_block_fwd cuts weight matrix `tensor` into panels of output features
 * when the first n_resident_chunks chunks are resident (Sec. 3.2/3.3): panel i covers rows
 * [row0[i], row1[i]) and may run once chunk wait_chunk[i] has landed (-1: no streamed chunk
 * needed).  m_rows = the tokens the layer is applied to: panels are whole 256-feature tiles,
 * as many of the landed ones as fill the launch's rounds of workgroups (a poorly filled remainder
 * stays with the next panel); m_rows = 0 plans the modulation matrix-vector product, whose
 * panels are multiples of 8 rows.  The last panel ends with the matrix.  *n: capacity / count;
 * pass NULL arrays to query the count. */
int cf_plan_panels(const cf_ctx* ctx, const char* tensor, int32_t m_rows, int32_t n_resident_chunks,
                   int32_t* row0, int32_t* row1, int32_t* wait_chunk, int32_t* n);

/* ---- overlap model at chunk granularity and the memory-latency dial (Sec. 3.1-3.3; host only).
 * cf_simulate walks the copy stream and the compute stream of the scheduler chunk by chunk for the
 * context's model, chunk size and block kinds: chunks of block i+1 are copied back to back while
 * block i computes (after block i-1 released the slot), and the part of a block's compute that a
 * chunk's bytes enable starts when the chunk has landed; the first round(r * n_chunks) chunks of
 * every block are resident.  With one chunk per block and r = 0 the result is the sum over blocks
 * of max(T_comp, T_pref) (Eq. 1-3).  Emulated collectives are not modelled.
 * cf_tune evaluates chunk_candidates x {0, 1/r_steps, ..., 1} and returns, under a memory budget
 * (step_target_ms = 0), the fastest point that fits, or, under a step-time target
 * (memory_budget_bytes = 0), the point with the least weight memory that meets it.  Exactly one of
 * the two constraints must be given. */
int cf_simulate(const cf_ctx* ctx, double r, const cf_machine_t* machine, cf_sim_result* out);
int cf_tune(const cf_ctx* ctx, const cf_machine_t* machine, const uint64_t* chunk_candidates, int32_t n_candidates,
            int32_t r_steps, uint64_t memory_budget_bytes, double step_target_ms, cf_tune_choice* out);

/* ---- weights (Sec. 2.2: all layers are placed in pinned host memory at initialisation).
 * host_blob must be pinned (hipHostMalloc), hold exactly cf_blob_bytes and outlive the context. */
int cf_register_block(cf_ctx* ctx, int32_t block, const void* host_blob, uint64_t bytes);

/* ---- Sec. 3.3 partial parameter residency: keep floor(r*n_chunks + 0.5) leading chunks of every
 * block permanently in HBM and prefetch only the rest.  r=0 is full offload, r=1 no offload.
 * Synchronises the device, re-plans, uploads the resident chunks; *actual (optional) receives
 * resident_bytes / blob_bytes.  r outside [0,1] is CF_ERR_ARG. */
int set_resident_fraction(cf_ctx* ctx, double r, double* actual);

/* ---- Sec. 2.2 step 3 + Sec. 3.2: start the asynchronous chunk-by-chunk prefetch of `block`
 * into one of the two staging slots (they alternate per call) on copy_stream.  The copy first
 * waits (on the GPU) for the slot's previous tenant to finish computing.  CF_ERR_STATE if that
 * tenant was prefetched but its dit_block_fwd has not been issued yet.
 * copy_stream and the compute stream must run concurrently: HIP multiplexes streams onto a few
 * hardware queues (4 by default), in creation order, and two streams that land on the same queue
 * execute one after the other -- the prefetch then hides behind nothing.  A process that creates
 * many streams should create these two back to back, or reuse one pair.
 * Host wait: before enqueueing, the call waits (hipEventSynchronize) for the block forward that last
 * used the OTHER slot, i.e. the forward issued two forwards ago, so that the host never runs more than
 * one block ahead of the GPU; with everything resident it returns at once. */
int chunked_prefetch_begin(cf_ctx* ctx, int32_t block, void* copy_stream);

/* ---- Sec. 2.2 step 1, at chunk granularity: make compute_stream wait (on the GPU) until chunk
 * `chunk` of `block` (and all earlier ones) has landed; chunk = -1 means the whole block.
 * Resident chunks need no wait.  CF_ERR_STATE if the block's prefetch was never begun. */
int chunked_prefetch_wait(cf_ctx* ctx, int32_t block, int32_t chunk, void* compute_stream);

/* ---- Sec. 2.2 step 2: enqueue the forward pass of `block` on compute_stream.  Each kernel that
 * reads weights is preceded by the wait for the last chunk it needs, and the GEMMs are launched
 * as panels of output features per chunk, so compute starts before the whole layer has landed.
 * Marks the staging slot reusable when the block's last kernel finishes (step 4); a forward that
 * returns an error after it began enqueueing releases the slot as well, behind what it enqueued.
 * Host waits: in pause/resume mode, for the worker thread to have enqueued each chunk a layer is about
 * to wait for; while emulated collectives are enabled, for the forward issued two forwards earlier. */
int dit_block_fwd(cf_ctx* ctx, int32_t block, const cf_block_io* io, void* compute_stream);

/* ---- Sec. 3.2 pause/resume.  cf_set_contention enables, per block forward, four emulated
 * collectives (q,k,v before attention, o after), each moving `bytes_per_collective` split half
 * host->device / half device->host on comm_stream through host_pinned / a device buffer the
 * library owns; the compute stream waits for each.  comm_stream NULL disables.
 * pause_resume = 0: chunk copies are enqueued by chunked_prefetch_begin as without collectives.
 * pause_resume = 1 or 2: a prefetch worker thread enqueues the chunks, keeping that many copies ahead
 * of the link (1: a chunk is enqueued when the one before it has landed, so a collective never waits
 * for more than the chunk on the link, the bound of Sec. 3.2; 2: one more copy queued behind it, which
 * closes the gap between copies and doubles the bound).  Before each chunk the worker looks at the
 * oldest unfinished collective: if the compute stream has reached it (GPU time, not host enqueue time),
 * the copy stream is made to wait for that collective's completion event -- once per collective;
 * cf_stats().pauses counts these.  Blocks the host until the GPU is idle (it changes streams' roles). */
int cf_set_contention(cf_ctx* ctx, void* comm_stream, void* host_pinned, uint64_t host_bytes,
                      uint64_t bytes_per_collective, int32_t pause_resume);
/* The same two hooks for a caller that issues its own collective on comm_stream between them. */
int cf_comm_begin(cf_ctx* ctx, void* comm_stream, void* compute_stream);
int cf_comm_end(cf_ctx* ctx, void* comm_stream, void* compute_stream);

/* ---- integrity: 64-bit checksum of every chunk of `block` as it currently sits in HBM (resident
 * buffer or staging slot); host_out[n_chunks].  Waits for the block's prefetch, then blocks the
 * host until done.  Word i of the blob (little-endian 64-bit, i from the blob start) contributes
 * splitmix64_finalise(word XOR (i+1)*0x9E3779B97F4A7C15), summed modulo 2^64. */
int cf_checksum_block(cf_ctx* ctx, int32_t block, uint64_t* host_out, void* stream);
/* copy the device image of `block` back to host_out[blob_bytes] (for byte-exact comparison) */
int cf_read_block(cf_ctx* ctx, int32_t block, void* host_out, void* stream);

/* Per-chunk consumer waits pay off while the link is the bottleneck; once a block kind's prefetch is
 * hidden (Sec. 3.1: its weights had landed before the block started, observed on the previous block of
 * that kind) a wait per chunk only costs stream bubbles and splits the layers into panels for nothing.
 * With adaptive waits on (the default) such a block waits once, for its last chunk, as the plain
 * layerwise loop of Sec. 2.2 does, and goes back to per-chunk waits as soon as a prefetch is seen to
 * land late.  Results do not depend on the mode.  Not used together with the pause/resume worker. */
int cf_set_adaptive_waits(cf_ctx* ctx, int32_t on);
int cf_stats(cf_ctx* ctx, cf_stats_t* out);
int cf_stats_reset(cf_ctx* ctx);
/* Profiling puts a hipEvent pair around every kernel launch and around every wait of the compute
 * stream on a chunk event ("prefetch_stall": the exposed prefetch of Sec. 4.3's breakdown) or on a
 * collective's completion ("collective_wait"); cf_kernel_times returns one record per name. */
int cf_set_profiling(cf_ctx* ctx, int32_t on);
int cf_kernel_times(cf_ctx* ctx, cf_kernel_time* out, int32_t* n);   /* syncs; *n capacity/count */
int cf_kernel_times_reset(cf_ctx* ctx);
int cf_sync(cf_ctx* ctx);                                      /* hipDeviceSynchronize */

/* ---- integrity of any device byte range (same definition as cf_checksum_block) */
/* checksum of a device byte range (definition above); host_out[1]; blocks the host. */
int cf_op_checksum(const void* data, uint64_t bytes, uint64_t first_word, uint64_t* host_out, void* stream);
/* The same checksum for callers that cannot allocate device memory or block: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  `data` (device, 8-byte aligned,
 * `bytes` a multiple of 8) is reduced into *dev_out (DEVICE memory, one uint64_t, caller-owned); the call
 * only enqueues two kernels on `stream` and returns.  No hipMalloc/hipFree, no host synchronisation.
 * The per-workgroup partial sums live in a fixed 256 KiB array inside the library image (one copy per
 * GPU, held until the process ends), which bounds a call to 1 GiB (2^30 bytes): larger `bytes` is
 * CF_ERR_ARG, as are NULL or misaligned pointers; nothing is launched then.  bytes = 0 stores 0.
 * All calls on one GPU share that array: two calls whose kernels may overlap (different streams
 * without an ordering between them) race; calls on one stream, or ordered by events, are safe. */
int cf_op_checksum_noalloc(const void* data, uint64_t bytes, uint64_t first_word, uint64_t* dev_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CHUNKFLOW_H */
