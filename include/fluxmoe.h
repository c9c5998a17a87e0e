/*
 * fluxmoe.h - C ABI of the MI355X expert-materialization library (libfluxmoe.so).
 *
 * The library implements the per-layer hot path of expert paging (paper Sec. 3 "Expert
 * paging"): routed-expert weights live in a losslessly compressed pool (Sec. 4.2
 * "Compressed GPU backend": Huffman code over the BF16 exponent bits, sign and mantissa
 * unchanged), are materialized on demand into reusable staging slots (Sec. 4.1
 * "PagedTensor": reusable physical blocks, contents updated by materialization), and are
 * then consumed by the expert FFN.  Ordering between the two follows the PagedTensor
 * synchronization protocol (Alg. 1: write-after-read and read-after-write events).
 *
 * Conventions
 *   - plain C, no exceptions cross the boundary; every call returns a fluxmoe_status
 *     (0 = OK, negative = error) and leaves a text in fluxmoe_last_error() (thread local).
 *   - "host" pointers are ordinary process memory, "pinned" is page-locked host memory
 *     (hipHostMalloc), "device" is HBM of the current HIP device.  All large buffers are
 *     allocated and owned by the caller and must outlive every enqueued operation; the
 *     context owns only small host metadata, a small pinned command ring and HIP events.
 *   - `stream` arguments are hipStream_t values passed as void* (NULL = default stream).
 *     Calls that take a stream only enqueue work and return.
 *   - arguments are validated on the host before anything is enqueued; on error nothing
 *     is enqueued.  Kernels never write outside the bound slot arenas, the page table,
 *     `out` and the bound workspace, whatever the compressed pool contains.
 *   - hidden and ffn must be multiples of 8, hidden * ffn under 2^30; block_bytes must be 4096.
 *
 * Compressed block (block_bytes bytes, independently decodable; this build's container,
 * the paper prints none):
 *     +0   u32 n            elements in the block (positive multiple of 64)
 *     +4   u32 e0           index of the block's first element inside its tensor
 *     +8   u16 sub_bits[64] bit length of each of the 64 sub-streams
 *     +136 u8  sm[n]        raw sign|mantissa byte of every element (sign in bit 7)
 *     +136+n                64 sub-streams back to back, then zero padding
 *   element m of the block belongs to sub-stream (m >> 3) & 63; stream bit k is bit k & 31
 *   of little-endian u32 word k >> 5; codes are canonical (sorted by length, then symbol)
 *   and written first (most significant) code bit first.
 * Layer blob: blocks of the down tensors (type 2) of experts 0..E-1, then of the fused
 * gate/up tensors (type 1) of experts 0..E-1; a tensor's blocks are contiguous.
 */
#ifndef FLUXMOE_H
#define FLUXMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fluxmoe_ctx fluxmoe_ctx;

typedef enum {
    FLUXMOE_OK = 0,
    FLUXMOE_EINVAL = -1,   /* bad argument */
    FLUXMOE_ENOMEM = -2,   /* a caller-provided buffer is too small / host allocation failed */
    FLUXMOE_ECORRUPT = -3, /* compressed pool fails validation */
    FLUXMOE_ERANGE = -4,   /* layer / expert / slot index out of range */
    FLUXMOE_EHIP = -5,     /* a HIP runtime call failed (text has the HIP error) */
    FLUXMOE_ESTATE = -6    /* call made in the wrong state (layer not encoded / not bound) */
} fluxmoe_status;

/* Homogeneous MoE model (Sec. 3: N layers, L routed experts of one architecture). */
typedef struct {
    uint32_t n_layers;     /* N pageable MoE layers */
    uint32_t n_experts;    /* L routed experts per layer */
    uint32_t hidden;       /* H */
    uint32_t ffn;          /* F, per-expert intermediate size */
    uint32_t block_bytes;  /* compressed block size; 4096 */
    uint32_t max_code_len; /* Huffman length limit, 8..12 (0 = 12) */
    uint32_t n_slots;      /* staging budget in experts (slots per arena) */
    uint32_t flags;        /* reserved, 0 */
} fluxmoe_desc;

typedef struct {
    uint64_t sigma1;            /* bytes of one fused gate/up tensor [2][H][F] (type 1) */
    uint64_t sigma2;            /* bytes of one down tensor [F][H] (type 2); sigma1 = 2 sigma2 */
    uint64_t slots13_bytes;     /* n_slots * sigma1 */
    uint64_t slots2_bytes;      /* n_slots * sigma2 */
    uint64_t page_table_bytes;  /* int32 [n_layers][n_experts] */
    uint64_t layer_blob_bound;  /* upper bound of one layer's compressed blob */
    uint64_t pool_workspace_bytes; /* device workspace needed by materialize (tables, commands) */
} fluxmoe_sizes;

typedef struct {
    uint64_t n_blocks;          /* blocks in the layer blob */
    uint64_t payload_bits[2];   /* sum of code lengths over all elements: [0] type 1, [1] type 2 */
    uint64_t elements[2];       /* elements per type over all experts */
} fluxmoe_layer_info;

/* Text of the last error on this thread ("" if none).  Never NULL. */
const char* fluxmoe_last_error(void);

/* Create / destroy a context.  Host only; no HIP call is made until a bind call. */
int fluxmoe_create(const fluxmoe_desc* desc, fluxmoe_ctx** out_ctx);
int fluxmoe_destroy(fluxmoe_ctx* ctx);

int fluxmoe_query_sizes(const fluxmoe_ctx* ctx, fluxmoe_sizes* out);

/* Device workspace bytes fluxmoe_expert_ffn needs for T tokens with K experts each
 * (shared_expert != 0 adds the always-on shared expert's rows). */
uint64_t fluxmoe_ffn_workspace_bytes(const fluxmoe_ctx* ctx, uint32_t T, uint32_t K,
                                     int shared_expert);

/*
 * Offline compression of one layer's routed experts (Sec. 4.2 "Compressed GPU backend": only the
 * exponent field is entropy coded, ahead of serving; sign and mantissa are stored as they are).  CPU only,
 * deterministic (independent of n_threads).
 *   w13  host, BF16 bit patterns [n_experts][2][hidden][ffn]  (gate, then up; y = x W)
 *   w2   host, BF16 bit patterns [n_experts][ffn][hidden]
 *   dst  host (may be pinned), receives the layer blob; dst_cap in bytes
 *   dst_used receives the blob size (a multiple of block_bytes)
 * One code table per tensor type over all experts of the layer; metadata (code lengths,
 * block ranges of every tensor) is kept in ctx.  ENOMEM if dst_cap is too small.
 */
int fluxmoe_encode_pool(fluxmoe_ctx* ctx, uint32_t layer, const uint16_t* w13,
                        const uint16_t* w2, void* dst, size_t dst_cap, size_t* dst_used,
                        int n_threads);

/* Metadata of an encoded layer (host). type: 1 = fused gate/up, 2 = down. */
int fluxmoe_layer_info_get(const fluxmoe_ctx* ctx, uint32_t layer, fluxmoe_layer_info* out);
int fluxmoe_code_lengths(const fluxmoe_ctx* ctx, uint32_t layer, int type, uint8_t out_lens[256]);
int fluxmoe_tensor_blocks(const fluxmoe_ctx* ctx, uint32_t layer, int type, uint32_t expert,
                          uint64_t* first_block, uint64_t* n_blocks);
/* first element index of every block of one tensor: out[n_blocks + 1] (last = tensor size) */
int fluxmoe_tensor_first_elems(const fluxmoe_ctx* ctx, uint32_t layer, int type, uint32_t expert,
                               uint32_t* out, size_t out_cap);

/*
 * Bind caller-owned device memory.
 *   slots13  device, n_slots * sigma1 bytes, 256-byte aligned: type-1 staging slots
 *   slots2   device, n_slots * sigma2 bytes, 256-byte aligned: type-2 staging slots
 *   workspace device, 256-byte aligned; at least pool_workspace_bytes; whatever lies
 *            beyond that is what fluxmoe_expert_ffn may use (see fluxmoe_ffn_workspace_bytes)
 * The type-d tensor of the expert mapped to slot s lives at slots_d + s * sigma_d (the
 * PagedTensor address formula of Sec. 4.1 with the layer term replaced by the page table).
 */
int fluxmoe_bind_arenas(fluxmoe_ctx* ctx, void* slots13, void* slots2, void* workspace,
                        size_t workspace_bytes);

/*
 * Bind one encoded layer's blob, split between the two tiers of Sec. 4.2 ("Memory hierarchy
 * model"): blocks [0, n_host_blocks) of the blob are read from `host_blocks` (pinned host
 * memory, block 0 first), blocks [n_host_blocks, n_blocks) from `hbm_blocks` (device; its
 * first byte is block n_host_blocks).  Either part may be empty (pointer then ignored).
 * Validates every block header against the encoder's metadata when the blob is host
 * readable (check_host_copy: optional host pointer to the whole blob, may be NULL) ->
 * ECORRUPT.  Uploads the layer's decode tables into the workspace (synchronous).
 */
int fluxmoe_bind_layer(fluxmoe_ctx* ctx, uint32_t layer, const void* hbm_blocks,
                       uint64_t n_host_blocks, const void* host_blocks,
                       const void* check_host_copy);

/*
 * Move one whole tensor of a bound layer to another backing copy (Sec. 4.3 "Runtime
 * adaptation": tensor-level offloading and restoration between compressed GPU memory and
 * pinned host memory, inside a running engine).  From this call on fluxmoe_materialize reads
 * the type-`type` tensor of `expert` from `blocks`:
 *   FLUXMOE_TIER_HBM       device memory, the tensor's compressed blocks;
 *   FLUXMOE_TIER_HOST      pinned host memory, the tensor's compressed blocks (fetched by DMA into
 *                          the staging buffer, then decoded like device-resident ones);
 *   FLUXMOE_TIER_HOST_RAW  pinned host memory, the tensor's dense BF16 bytes (the CPU offload
 *                          backend as Sec. 4.2 states it: weights in pinned host memory, moved by
 *                          asynchronous DMA).  Fetched into the staging buffer like the
 *                          compressed host tier and copied from there into the slot; nothing is
 *                          decoded.  The staging buffer must hold the dense bytes.
 * For the first two, `blocks` holds the tensor's blocks exactly as fluxmoe_encode_pool wrote them
 * (fluxmoe_tensor_blocks gives their range in the layer blob).  16-byte aligned in every case.
 * Host state only, nothing is enqueued: work enqueued
 * earlier still reads the previous copy, which the caller may free once that work has
 * completed (Sec. 4.3: the retired copy is freed after the events complete).  A host-tier
 * fetch of this layer issued before the call is forgotten.
 */
#define FLUXMOE_TIER_HBM 0
#define FLUXMOE_TIER_HOST 1
#define FLUXMOE_TIER_HOST_RAW 2
int fluxmoe_set_tensor_backing(fluxmoe_ctx* ctx, uint32_t layer, int type, uint32_t expert,
                               int tier, const void* blocks);

/* Bind the device staging buffer host-tier blocks are copied into before decoding
 * (two halves, used alternately by consecutive layers).  Needed only if some layer has
 * n_host_blocks > 0. */
int fluxmoe_bind_staging(fluxmoe_ctx* ctx, void* staging, size_t staging_bytes);

/* Enqueue: set every entry of the device page table to -1 and forget all slot ownership. */
int fluxmoe_reset_page_table(fluxmoe_ctx* ctx, int32_t* page_table, void* stream);

/*
 * Host-tier fetch (Sec. 4.2 "CPU offload backend": asynchronous DMA from pinned host
 * memory, overlapped with inference).  Enqueues on copy_stream the hipMemcpyAsync of every
 * host-tier block the listed experts of `layer` need into the staging half of that layer,
 * after waiting (on the device) for the last decode that read that half and for the copies
 * of the previous fetch into it (which may have been issued on another stream).  Layer l uses half
 * l & 1 and the half keeps the blocks until the next fetch into it, so one fetch can serve
 * several fluxmoe_materialize calls (waves) of that layer over subsets of the listed experts;
 * each of them waits for these copies.  Issue the fetch for layer l + 2 only after the last
 * fluxmoe_materialize of layer l has been issued.  Optional: if the experts a materialize needs
 * are not staged, it issues the copies on its own stream.
 */
int fluxmoe_prefetch_host(fluxmoe_ctx* ctx, uint32_t layer, const int32_t* expert_ids,
                          uint32_t n, void* copy_stream);

/*
 * Materialize experts of one layer into staging slots (Sec. 3 "Expert paging": a layer's experts
 * become resident only for the time the layer is scheduled; Alg. 1 MaterializeLayer).
 *   expert_ids host, n distinct ids in [0, n_experts)
 *   dst_slots  host, n distinct slots in [0, n_slots)
 *   page_table device int32 [n_layers][n_experts]; the same table on every call
 * Enqueued on `stream`: wait for the last expert-FFN call that read any of the target
 * slots (write-after-read), [wait for the layer's host-tier copies], decode + paged
 * scatter, page-table update, record the layer's load event.  After that event, for each
 * i: slot dst_slots[i] holds exactly the original bytes of both tensors of expert_ids[i],
 * page_table[layer][expert_ids[i]] = dst_slots[i], the entry of whichever (layer, expert)
 * owned that slot before is -1; nothing else changes.  n = 0 is valid and enqueues nothing.
 */
int fluxmoe_materialize(fluxmoe_ctx* ctx, uint32_t layer, const int32_t* expert_ids,
                        uint32_t n, int32_t* page_table, const int32_t* dst_slots,
                        void* stream);

/*
 * fluxmoe_materialize with the two tensor types decoded on two streams, the stream layout of the paper's
 * loading path (Sec. 5 "Expert memory backends" and Sec. 6.3 Exp#3: separate streams for the fused
 * gate/up tensors and the down tensors, the latency of a layer counted from issue until both types are
 * ready).  Waits, command upload and the type-1 launch go to `stream`, the type-2 launch to
 * `stream_type2` after them; `stream` then waits for the type-2 launch and records the layer's load
 * event, so everything that holds after fluxmoe_materialize's event holds after this one.  The caller
 * must not reuse `stream_type2` for work that has to precede this call.  stream_type2 == stream is
 * fluxmoe_materialize.
 */
int fluxmoe_materialize_two_streams(fluxmoe_ctx* ctx, uint32_t layer, const int32_t* expert_ids,
                                    uint32_t n, int32_t* page_table, const int32_t* dst_slots,
                                    void* stream, void* stream_type2);

/*
 * Release experts of one layer (Sec. 3 "Expert paging": once a layer's MoE block has run, the
 * forward proxy gives that layer's expert set back): enqueue page_table[layer][e] = -1 for the
 * listed experts that are mapped; their slots become free for reuse (a later materialize into
 * them still waits for the FFN that last read them).  expert_ids NULL with n = 0 releases every
 * expert of the layer.  Slot contents are not touched.
 * Stream contract: the update is enqueued on `stream` after waiting (on the device) for the
 * layer's last fluxmoe_expert_ffn and last fluxmoe_materialize, whatever streams those ran on;
 * a later fluxmoe_materialize or fluxmoe_expert_ffn of the same layer waits for the release.
 * Calls of one kind for one layer (two materializes, two releases) must be ordered by the
 * caller: same stream, or the caller's own events.
 */
int fluxmoe_release(fluxmoe_ctx* ctx, uint32_t layer, const int32_t* expert_ids, uint32_t n,
                    int32_t* page_table, void* stream);

/* fluxmoe_expert_ffn flags */
#define FLUXMOE_FFN_ACCUMULATE 1u    /* out += result instead of out = result */
#define FLUXMOE_FFN_SKIP_UNMAPPED 2u /* ignore (token, k) pairs whose expert is not mapped
                                        (a wave of a slot budget smaller than the union);
                                        without it such a pair sets the device error flag */

/*
 * Routed SwiGLU expert FFN over the materialized slots (Alg. 1 ForwardPass: wait for the
 * layer's load event, launch, record the inference event).
 *   tokens   device BF16 [T][hidden]
 *   topk_ids device int32 [T][K], topk_w device float [T][K]
 *   page_table device int32 [n_layers][n_experts] (expert -> slot, -1 = not resident)
 *   out      device float [T][hidden]
 * out_t = sum_k topk_w[t][k] * ( (silu(x_t W1_e) * (x_t W3_e)) W2_e ),  e = topk_ids[t][k];
 * BF16 inputs, FP32 accumulation, the SwiGLU product rounded to BF16 before the second
 * product.  Deterministic (fixed summation order).  T = 0 is valid.
 * Limits (the kernels address activations and one expert matrix with 32-bit byte offsets):
 * T <= 65535 and T * hidden * 2 bytes under 4 GiB here (EINVAL, nothing enqueued); hidden * ffn * 2
 * bytes under 2 GiB is checked by fluxmoe_create.
 */
int fluxmoe_expert_ffn(fluxmoe_ctx* ctx, uint32_t layer, const uint16_t* tokens, uint32_t T,
                       const int32_t* topk_ids, const float* topk_w, uint32_t K,
                       const int32_t* page_table, float* out, uint32_t flags, void* stream);

/*
 * fluxmoe_expert_ffn for callers that cannot allocate or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same result, same
 * event protocol, but the FFN scratch (pair order, tile list, the SwiGLU product h, split-K partials)
 * lives in a static device array of FLUXMOE_STATIC_SCRATCH_BYTES bytes that is part of the loaded
 * library (every GPU the library runs on holds its own copy until the process ends) instead of the
 * bound workspace.  The call itself allocates nothing and frees nothing; the array's device address
 * is resolved by fluxmoe_bind_arenas, which must have run on the current device.
 *   ENOMEM  T, K need more scratch than FLUXMOE_STATIC_SCRATCH_BYTES (fluxmoe_ffn_workspace_bytes
 *           gives the need); nothing is enqueued
 *   ESTATE  the current device is not the one fluxmoe_bind_arenas ran on
 * Every call on a GPU shares that GPU's array, whatever the context: calls that overlap on one GPU
 * (two streams, two contexts, two threads) race on it and must be ordered by the caller.  Nothing
 * in the array has to start at zero: every call rewrites each part before reading it.
 */
#define FLUXMOE_STATIC_SCRATCH_BYTES (32ull << 20)
int fluxmoe_expert_ffn_static(fluxmoe_ctx* ctx, uint32_t layer, const uint16_t* tokens, uint32_t T,
                              const int32_t* topk_ids, const float* topk_w, uint32_t K,
                              const int32_t* page_table, float* out, uint32_t flags, void* stream);

/*
 * The shared expert of a layer (Sec. 3 excludes shared experts from the routed set; Sec. 4.2
 * keeps their weights uncompressed and GPU resident): the same SwiGLU FFN applied to every
 * token with gate 1, on dense weights the caller keeps resident.
 *   w13 device BF16 [2][hidden][ffn], w2 device BF16 [ffn][hidden], 16-byte aligned
 *   tokens device BF16 [T][hidden]; out device float [T][hidden]
 *   flags: 0 or FLUXMOE_FFN_ACCUMULATE (out += result, e.g. after fluxmoe_expert_ffn)
 * Uses the bound workspace (fluxmoe_ffn_workspace_bytes with shared_expert != 0) and the
 * stream's order only; it takes no part in the slot event protocol.
 */
int fluxmoe_shared_expert_ffn(fluxmoe_ctx* ctx, const uint16_t* w13, const uint16_t* w2,
                              const uint16_t* tokens, uint32_t T, float* out, uint32_t flags,
                              void* stream);

/*
 * Budget-aware residency planner (Sec. 4.3, Alg. 2).  Host logic only; one planner per rank.
 * Every decoding iteration the serving loop reports the remaining batch B_rem, the active
 * batch B_act, the measured forward latency tau_fwd and the measured materialization time of
 * every MoE layer (any one time unit).  Every control_interval iterations with B_act > 0 the
 * planner forms
 *     tau_eff = (B_rem / B_act) tau_fwd,  tau_load = sum_l tau_load_layer[l],
 *     rho = tau_eff / tau_load  (+inf when tau_load = 0)
 * and takes one reclamation step if rho > 1 and B_act < B_rem, reverses the latest step if
 * rho < theta, and otherwise keeps the state.  Reclamation first turns uncompressed-resident
 * layers into pageable ones (one per step, largest index first), then offloads expert
 * tensors to the host: ceil(AG L_r) down-projection tensors per step, and once none is left
 * ceil(AG L_r / 2) fused gate/up tensors, each taken from the pageable layer with the smallest
 * host-assigned volume (ties: larger layer index), largest expert index first.  The moves of a
 * step are returned for the caller to carry out (fluxmoe_set_tensor_backing).
 */
typedef struct fluxmoe_planner fluxmoe_planner;

typedef struct {
    uint32_t n_layers;              /* MoE layers of this rank */
    uint32_t experts_per_rank;      /* L_r */
    uint32_t control_interval;      /* CI in decoding iterations (0 = 16) */
    uint32_t reserved;              /* 0 */
    double theta;                   /* restoration threshold in (0, 1] (0 = 0.9) */
    double adjustment_granularity;  /* AG in (0, 1] (0 = 0.25) */
} fluxmoe_planner_desc;

typedef struct {
    uint32_t layer;
    uint32_t expert;                /* rank-local expert index (0 for a layer move) */
    int32_t type;                   /* 1 fused gate/up, 2 down; 0 = the layer changes class */
    int32_t to_host;                /* tensor: 1 to pinned host, 0 back to compressed GPU memory;
                                       layer: 1 becomes pageable, 0 becomes uncompressed-resident */
} fluxmoe_planner_move;

#define FLUXMOE_PLAN_KEEP 0
#define FLUXMOE_PLAN_RECLAIM 1
#define FLUXMOE_PLAN_RESTORE (-1)
#define FLUXMOE_PLAN_SKIP 2         /* not a control iteration, or B_act = 0 */
#define FLUXMOE_PLAN_DONE 3         /* B_rem = 0: the run is over */

typedef struct {
    int32_t action;
    uint32_t n_moves;
    double rho, tau_eff, tau_load;  /* NaN unless the control rule ran */
} fluxmoe_planner_decision;

/* uncompressed: host, n_layers flags (non-zero = the layer starts uncompressed-resident), or
 * NULL for all pageable.  All tensors start GPU-backed. */
int fluxmoe_planner_create(const fluxmoe_planner_desc* desc, const uint8_t* uncompressed,
                           fluxmoe_planner** out);
int fluxmoe_planner_destroy(fluxmoe_planner* p);
/* Largest number of moves one step can return; `moves` must hold at least that many. */
uint32_t fluxmoe_planner_max_moves(const fluxmoe_planner* p);
/* One decoding iteration of Alg. 2.  tau_load_layer: host, n_layers values (NULL = all 0). */
int fluxmoe_planner_tick(fluxmoe_planner* p, uint64_t B_rem, uint64_t B_act, double tau_fwd,
                         const double* tau_load_layer, fluxmoe_planner_decision* out,
                         fluxmoe_planner_move* moves, size_t moves_cap);
/* One reclamation / restoration step regardless of the control rule (n_moves 0 = nothing left). */
int fluxmoe_planner_reclaim(fluxmoe_planner* p, fluxmoe_planner_move* moves, size_t moves_cap,
                            uint32_t* n_moves);
int fluxmoe_planner_restore(fluxmoe_planner* p, fluxmoe_planner_move* moves, size_t moves_cap,
                            uint32_t* n_moves);
/* layer_pageable: n_layers flags; on_host: [n_layers][experts_per_rank][2] flags, last index
 * 0 = type 1, 1 = type 2.  Either may be NULL. */
int fluxmoe_planner_state(const fluxmoe_planner* p, uint8_t* layer_pageable, uint8_t* on_host);

/*
 * PagedTensor on the device's virtual memory management (Sec. 4.1).  For tensor type d the
 * layer group is A_d = L sigma_d bytes, padded to S_d = alignUp(A_d, g) for the allocation
 * granularity g; a virtual range of N S_d bytes at v0_d is reserved and the type-d tensor of
 * expert e in layer i (both 0-based here) has the stable address
 *     v0_d + i S_d + e sigma_d.
 * A pageable layer's range is mapped onto reusable block F_{i mod 2} (all pageable layers of one
 * parity share one physical block), an uncompressed-resident layer's range onto a dedicated
 * block.  Physical memory is (|U| + 2) (S_1 + S_2) bytes, of which
 *     M_pad = (|U| + 2) sum_d (S_d - A_d)
 * is padding.  Kernels read the tensors through these addresses with no translation of their
 * own.  reusable_window[d] is one more view of the two reusable blocks, F_0 at +0 and F_1 at
 * +S_d: when S_d = A_d for both types it can be bound as the slot arenas of a context with
 * n_slots = 2 L (fluxmoe_bind_arenas), and materializing expert e of layer i into slot
 * (i mod 2) L + e then fills exactly the bytes that layer i's own addresses show.
 */
typedef struct fluxmoe_paged_tensor fluxmoe_paged_tensor;

typedef struct {
    uint64_t granularity;          /* g */
    uint64_t A[2], S[2];           /* [0] type 1, [1] type 2 */
    uint64_t v0[2];                /* device virtual addresses (0 from fluxmoe_paged_tensor_layout) */
    uint64_t reusable_window[2];   /* device virtual addresses (0 from fluxmoe_paged_tensor_layout) */
    uint64_t virtual_bytes;        /* N (S_1 + S_2) */
    uint64_t physical_bytes;       /* (|U| + 2) (S_1 + S_2) */
    uint64_t pad_bytes;            /* M_pad */
    uint32_t n_uncompressed, n_pageable;
} fluxmoe_paged_tensor_info;

/* The arithmetic alone (host, no device needed): sizes for a granularity and |U|. */
int fluxmoe_paged_tensor_layout(const fluxmoe_desc* desc, uint64_t granularity,
                                uint32_t n_uncompressed, fluxmoe_paged_tensor_info* out);
/* Reserve, create and map on the current device (only n_layers, n_experts, hidden, ffn of desc
 * are used).  uncompressed: host, n_layers flags, or NULL for all pageable.  Block contents are
 * undefined until written.  EHIP if the device lacks virtual memory management. */
int fluxmoe_paged_tensor_create(const fluxmoe_desc* desc, const uint8_t* uncompressed,
                                fluxmoe_paged_tensor** out);
/* Unmaps and frees everything; no kernel may still be using the addresses. */
int fluxmoe_paged_tensor_destroy(fluxmoe_paged_tensor* p);
int fluxmoe_paged_tensor_info_get(const fluxmoe_paged_tensor* p, fluxmoe_paged_tensor_info* out);
int fluxmoe_paged_tensor_address(const fluxmoe_paged_tensor* p, uint32_t layer, int type,
                                 uint32_t expert, void** out);
/* Residency change of one layer (Sec. 4.1: mappings change only when a layer changes residency
 * class, never on materialization): remap its
 * ranges to a new dedicated block (contents undefined) or back to its reusable block (the
 * dedicated block is released).  Synchronises the device first; addresses do not change. */
int fluxmoe_paged_tensor_set_class(fluxmoe_paged_tensor* p, uint32_t layer, int uncompressed);

/*
 * Bandwidth-balanced tier split (Sec. 4.2 "Memory hierarchy model").  With the two backends
 * materializing their shares of a layer concurrently at effective rates beta_gpu and beta_cpu
 * (any one unit, in dense BF16 bytes per time), both finish together when the host share is
 *     x_bw = beta_cpu / (beta_gpu + beta_cpu).
 * It is realised with whole tensors: ceil(3 L_r x_bw) down-projection tensors (a layer is
 * 3 L_r down-projection volumes), so the realised share exceeds x_bw by less than 1/(3 L_r).
 * If that count exceeds L_r (x_bw > 1/3) the remainder is taken as fused tensors, two volumes
 * each, rounded upward.  Host only; output pointers may be NULL.
 */
int fluxmoe_balanced_split(double beta_gpu, double beta_cpu, uint32_t experts_per_rank,
                           double* x_bw, uint32_t* n_down, uint32_t* n_fused);

/* Synchronous: read and clear the device error word (0 = none; bit 0 a block failed
 * validation during decode and was skipped, bit 1 an unmapped expert was routed to). */
int fluxmoe_device_errors(fluxmoe_ctx* ctx, uint32_t* out_flags);

/* ------------------------------------------------------------------------------------------
 * Measurement section.  Nothing below is part of the hot path or needed to use it: these entry
 * points exist for benchmarks, counter calibration and tests of the launch plan.
 * ------------------------------------------------------------------------------------------ */

/*
 * The launch plan fluxmoe_expert_ffn takes for T tokens with K experts each (host only; for tests
 * and reports): rows per tile of the grouped products (16..128 = weight-streaming kernels, 256 =
 * LDS-tiled MFMA kernels) and the number of K splits of the second product.  The plan depends on the
 * shapes, on T * K / n_experts and on the CU count of the device (256 until a bind call has
 * queried it).
 */
int fluxmoe_ffn_plan(const fluxmoe_ctx* ctx, uint32_t T, uint32_t K, uint32_t* rows_per_tile,
                     uint32_t* k_splits);

/*
 * Measurement aid: a plain device-to-device copy of `bytes` bytes (multiple of 16, both
 * pointers 16-byte aligned) with the same streaming 16-byte accesses the decode kernel
 * uses, on n_workgroups workgroups of 256 lanes.  Gives the achievable HBM rate on the box
 * and a known-traffic kernel for calibrating hardware counters.  Needs no context.
 */
int fluxmoe_stream_copy(void* dst, const void* src, uint64_t bytes, uint32_t n_workgroups,
                        void* stream);

/*
 * Measurement aid: the memory traffic of the materialization kernel without its work, in the same
 * launch shape (workgroups of waves_per_workgroup = 4, 8 or 16 wavefronts, blocks_per_wave blocks to
 * each wavefront; order 0 deals the blocks round-robin over all wavefronts of the launch as the
 * materialization kernel does, order 1 gives a workgroup consecutive blocks which its wavefronts
 * pass over side by side, order 2 gives every wavefront consecutive blocks).  `src` (device, 128-byte aligned) is read
 * as src_bytes / 4096 blocks of 4096 bytes, each by one wavefront with streaming 16-byte loads;
 * for every block the wavefront then writes out_bytes_small bytes (three blocks of every eight:
 * out_bytes_small + 128; a multiple of 128 in [128, 16384]) to `dst` (device, 128-byte aligned),
 * block after block without gaps, in pieces of 1 KiB with streaming 16-byte stores whose data
 * depend on the loads.  *bytes_written (may be NULL) receives the bytes written; FLUXMOE_EINVAL
 * if dst_bytes is less than that, nothing is enqueued then.  Timed by the caller with the ratio
 * of a pool (4096 / out bytes = compressed / dense), it gives what HBM delivers to this access
 * pattern on the box: the ceiling of the decode kernel short of changing the container.
 * Needs no context.
 */
int fluxmoe_stream_mix(void* dst, uint64_t dst_bytes, const void* src, uint64_t src_bytes,
                       uint32_t out_bytes_small, uint32_t waves_per_workgroup, uint32_t blocks_per_wave,
                       uint32_t order, uint64_t* bytes_written, void* stream);

/*
 * Measurement aid: n_workgroups workgroups of four wavefronts each issue iters x 16 independent
 * v_mfma_f32_32x32x16_bf16 (32768 flops each) on operands taken once from `operands` (device, 64 KiB
 * of BF16 values, 16-byte aligned) and no memory traffic in the loop; `out` (device, n_workgroups *
 * 256 floats) receives sums that keep the work alive.  Timed by the caller, it gives the rate the
 * matrix cores sustain for that operand content (the chip's clock depends on it).  Needs no context.
 */
int fluxmoe_mfma_probe(const void* operands, float* out, uint32_t n_workgroups, uint32_t iters,
                       void* stream);

/*
 * Kernel timing for benchmarks.  While enabled, every kernel the library launches is
 * bracketed by HIP events on its own stream.  fluxmoe_profile_collect waits for them, adds
 * the elapsed milliseconds and launch counts per kind and forgets them:
 *   kind 0 decode + paged scatter, 1 token grouping, 2 gate/up product + SwiGLU,
 *   3 down product, 4 gated combine.
 * on: 0 = off, 1 = every kind, FLUXMOE_PROFILE_ONLY(mask) = only the kinds whose bit is set in
 * mask (an event between two kernels costs a few microseconds of idle device time; a benchmark
 * that times whole steps brackets only the kernel it reports).
 */
#define FLUXMOE_PROFILE_KINDS 5
#define FLUXMOE_PROFILE_ONLY(mask) (0x100 | ((mask) & 0x1F))
int fluxmoe_profile_enable(fluxmoe_ctx* ctx, int on);
int fluxmoe_profile_collect(fluxmoe_ctx* ctx, double out_ms[FLUXMOE_PROFILE_KINDS],
                            uint32_t out_count[FLUXMOE_PROFILE_KINDS]);

#ifdef __cplusplus
}
#endif
#endif /* FLUXMOE_H */
