/*
 * tessera.h - C ABI of the MI355X (gfx950) decoder-layer kernel library.
 *
 * The paper schedules the kernels of one LLM forward iteration, one by one,
 * across GPUs (kernel-granularity disaggregation, Sec. 3).  It treats those
 * kernels as opaque framework kernels with declared read and write buffers
 * (Sec. 3.1) and characterises them only by regime: skinny matrix products are
 * HBM-bandwidth-bound, tiled prefill attention is compute-bound (Sec. 2.3).
 * This library IS that kernel set for one decoder layer, one entry point per
 * kernel, plus the whole-layer call and the pipelined micro-batch step with
 * boundary-activation copies on a side stream (Sec. 3.3, "Disaggregated kernel
 * execution" and "Pipelined request processing").
 *
 * Conventions that hold for every entry point unless stated otherwise:
 *   - All tensor pointers are DEVICE pointers (HIP global memory) unless the
 *     parameter comment says "host".  Integer index arrays are device int32.
 *   - ts_bf16 is the raw 16-bit pattern of a bfloat16.  Tensors are row-major,
 *     innermost dimension contiguous, no padding.
 *   - Every device pointer must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise, allocate or free device
 *     memory.  The caller owns every buffer and keeps it alive (and does not
 *     overwrite inputs) until the enqueued work has finished.
 *   - Accumulation is fp32; results are rounded once (nearest-even) to bf16.
 *   - Return value: TS_OK or a negative TS_ERR_* code.  Argument, shape and
 *     workspace checks run before the first HIP call (so they work on a host
 *     without a GPU), and a call they reject has enqueued nothing.  A
 *     TS_ERR_HIP raised by the runtime in the middle of a call that launches
 *     several kernels (ts_layer_forward, ts_pipeline_step, the split-K and
 *     split-KV paths) leaves the earlier launches enqueued; output and
 *     workspace contents are then undefined.  ts_last_error() gives a
 *     thread-local detail string for the last failing call on this thread.
 *   - Output buffers must not alias inputs except where a parameter is
 *     documented as in/out.
 */
#ifndef TESSERA_H_
#define TESSERA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default) /* the library is built with hidden visibility */
#endif

typedef uint16_t ts_bf16;

#define TS_OK 0
#define TS_ERR_INVALID_ARG (-1)       /* null pointer, non-positive size, nq % nkv != 0, misaligned pointer */
#define TS_ERR_UNSUPPORTED_SHAPE (-2) /* valid but outside what the kernels cover (see each call) */
#define TS_ERR_WORKSPACE (-3)         /* workspace / staging buffer too small or missing */
#define TS_ERR_HIP (-4)               /* a HIP runtime call failed; see ts_last_error() */

#define TS_MODE_DECODE 0
#define TS_MODE_PREFILL 1

/* Text for a status code (static storage). */
const char* ts_strerror(int code);
/* Detail of the last error raised on the calling thread (thread-local storage, never NULL). */
const char* ts_last_error(void);
/* Library version string (static storage). */
const char* ts_version(void);

/* ---------------------------------------------------------------------------
 * Per-kernel latency profile (the t_{k,g} table the policy planner of Sec. 3.2
 * is fed with, measured per launch).  Between ts_profile_begin and
 * ts_profile_end every kernel the calling thread launches through this library
 * is bracketed by two of the caller's events, recorded on the launch stream:
 * events[2*i] before launch i, events[2*i+1] after it; names[i] receives a
 * pointer to a static kernel-family name.  events: HOST array of 2*max_launches
 * hipEvent_t created with timing enabled; names: HOST array of max_launches
 * pointers.  Launches beyond max_launches are not recorded.  ts_profile_end
 * returns the number of recorded launches (>= 0) and deactivates the profile;
 * the caller synchronises and reads elapsed times itself.
 */
int ts_profile_begin(void** events, const char** names, int max_launches);
int ts_profile_end(void);

/* ---------------------------------------------------------------------------
 * RMSNorm: y[t,i] = x[t,i] * rsqrt(mean_j x[t,j]^2 + eps) * gamma[i].
 * One of the small memory-bound kernels of the layer (Sec. 2.3 regime split).
 * x, y: [T,H]; gamma: [H].  y may alias x.  Requires H % 8 == 0, H <= 32768.
 * T == 0 is a no-op.
 */
int ts_rmsnorm(const ts_bf16* x, const ts_bf16* gamma, ts_bf16* y, int T, int H, float eps, void* stream);

/* ---------------------------------------------------------------------------
 * Dense projection C = A * W^T (+ residual): the layer's QKV, O, gate|up and
 * down products.  With few rows this is the paper's bandwidth-bound
 * matrix-vector regime (weights streamed once from HBM); with thousands of
 * rows it is the compute-bound regime (Sec. 2.3).
 * A: [M,K]; W: [N,K]; residual: [M,N] or NULL; C: [M,N].  C may alias residual.
 * Requires K % 8 == 0 and N % 2 == 0.  M == 0 is a no-op.
 * ws: scratch of at least ts_gemm_workspace_bytes(M,N,K) bytes (may be NULL
 * when that is 0).  Contents of ws are undefined afterwards.
 */
size_t ts_gemm_workspace_bytes(int M, int N, int K);
int ts_gemm_bf16(const ts_bf16* A, const ts_bf16* W, const ts_bf16* residual, ts_bf16* C,
                 int M, int N, int K, void* ws, size_t ws_bytes, void* stream);
/* Same product with an fp32 result (router logits of the MoE layer). No residual. */
int ts_gemm_bf16_f32out(const ts_bf16* A, const ts_bf16* W, float* C,
                        int M, int N, int K, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Rotary embedding (rotate-half pairing (i, i + d/2), theta_i = base^(-2i/d),
 * angle = pos * theta_i) applied in place to q and k, followed by the KV-cache
 * append: the cache is the buffer written in one iteration and read by later
 * ones (cross-iteration dependency, Sec. 3.1), and the appended rows are the
 * "delta" that would be replicated between GPUs (Sec. 4, memory management).
 * q: [T,nq,d] in/out with row stride `q_stride` elements between tokens;
 * k: [T,nkv,d] in/out, v: [T,nkv,d] in, both with row stride `kv_stride`.
 *   (strides let q,k,v live inside one [T,(nq+2nkv)d] projection output.)
 * pos: [T] position of each token; seq_id: [T] cache row of each token (may be
 * NULL when kcache is NULL).  cos_sin: optional fp32 table [table_len, d]
 * (row p = cos(p*theta_0..d/2-1) then sin(...)), built by ts_rope_table; when
 * NULL the angles are evaluated in fp64 inside the kernel.
 * kcache, vcache: [B,nkv,Lcap,d] or both NULL to skip the append.  Rotated k and
 * v of token t go to cache[seq_id[t], :, pos[t], :].
 * Requires d % 16 == 0, d <= 256, strides % 8 == 0.  Positions outside
 * [0,Lcap) (or [0,table_len) with a table) are the caller's error; tokens with
 * such positions are skipped for the append and rotated with the fp64 path.
 */
int ts_rope(ts_bf16* q, ts_bf16* k, const ts_bf16* v, int q_stride, int kv_stride,
            const int32_t* pos, const int32_t* seq_id, const float* cos_sin, int table_len,
            ts_bf16* kcache, ts_bf16* vcache, int T, int nq, int nkv, int d, int Lcap,
            float base, void* stream);
/* Host helper: fill a HOST buffer table[table_len*d] with the fp32 cos|sin table (fp64 evaluation). */
int ts_rope_table(float* table_host, int table_len, int d, float base);

/* ---------------------------------------------------------------------------
 * Decode attention over the contiguous KV cache: the large bandwidth-bound
 * kernel of a decode iteration (K and V are each read once).
 * For sequence b and query head h (kv head h / (nq/nkv)), over keys
 * j in [0, seq_lens[b]):  out = softmax_j(scale * <q, K_j>) . V
 * q, out: [B,nq,d]; kcache, vcache: [B,nkv,Lcap,d]; seq_lens: [B] (number of
 * keys attended, the just-appended token included; 0 gives a zero row).
 * Requires d == 64 or d == 128, nq/nkv <= 16, seq_lens[b] <= Lcap.
 * ws: at least ts_attention_decode_workspace_bytes(B,nq,nkv,d,Lcap) bytes (fp32 partial results of
 * the split over keys and, for long caches, one arrival counter per (sequence, kv head), which
 * the call clears itself); contents undefined afterwards.  The split is derived on the device from
 * seq_lens (no host synchronisation); the result does not depend on the order in which workgroups
 * finish.
 */
size_t ts_attention_decode_workspace_bytes(int B, int nq, int nkv, int d, int Lcap);
int ts_attention_decode(const ts_bf16* q, const ts_bf16* kcache, const ts_bf16* vcache,
                        const int32_t* seq_lens, ts_bf16* out, int B, int nq, int nkv, int d,
                        int Lcap, float scale, void* ws, size_t ws_bytes, void* stream);

/* The same call for callers that cannot allocate or carry a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the split-KV partials live in a device array that is part
 * of the library image, ts_attention_decode_static_limit() bytes (16 MiB) on every GPU the library runs on, held
 * until the process ends.  Same kernels and bit-identical results to ts_attention_decode (what must start at
 * zero in the array, the arrival counters, is cleared by a kernel of the call).  Shapes whose
 * partials (ts_attention_decode_workspace_bytes) exceed the limit are rejected with TS_ERR_WORKSPACE before
 * anything is enqueued.  The call allocates and frees nothing.  All calls on one GPU share that GPU's array:
 * calls that may run at the same time on one GPU (different streams) race and must be ordered by the caller. */
size_t ts_attention_decode_static_limit(void);
int ts_attention_decode_static(const ts_bf16* q, const ts_bf16* kcache, const ts_bf16* vcache,
                               const int32_t* seq_lens, ts_bf16* out, int B, int nq, int nkv, int d,
                               int Lcap, float scale, void* stream);

/* ---------------------------------------------------------------------------
 * Prefill attention over packed fresh sequences: the compute-bound tiled
 * kernel (Sec. 2.3).  Token at in-sequence index i attends keys j <= i of its
 * own sequence when `causal` != 0, all keys of its sequence otherwise.
 * q: [T,nq,d] row stride q_stride; k, v: [T,nkv,d] row stride kv_stride;
 * cu_seqlens: [S+1] device int32, sequence s owns rows cu[s]..cu[s+1]-1, cu[S] <= T;
 * out: [T,nq,d] dense.  max_seqlen: host-known upper bound on any sequence
 * length (sizes the grid).  Requires d == 64 or d == 128.
 */
int ts_attention_prefill(const ts_bf16* q, const ts_bf16* k, const ts_bf16* v, int q_stride,
                         int kv_stride, const int32_t* cu_seqlens, ts_bf16* out, int S, int T,
                         int max_seqlen, int nq, int nkv, int d, float scale, int causal,
                         void* stream);

/* ---------------------------------------------------------------------------
 * SwiGLU: out[t,f] = silu(gate_up[t,f]) * gate_up[t,F+f], silu(z) = z/(1+exp(-z)).
 * gate_up: [T,2F] = [gate | up]; out: [T,F].  Requires F % 8 == 0.
 */
int ts_swiglu(const ts_bf16* gate_up, ts_bf16* out, int T, int F, void* stream);

/* ---------------------------------------------------------------------------
 * MoE routing from fp32 logits[T,E]: per token the k largest logits (ties to
 * the lower expert index, slots in descending-logit order), weights = softmax
 * over the k selected logits, per-expert counts, exclusive offsets[E+1], and
 * perm[T*k]: flat assignment ids a = t*k+s grouped by expert, ascending inside
 * each expert (deterministic).  Integer outputs are exact.
 * Requires 1 <= k <= E <= 64, T*k <= 2^20.
 */
int ts_moe_route(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w,
                 int32_t* counts, int32_t* offsets, int32_t* perm, void* stream);

/* ---------------------------------------------------------------------------
 * Grouped expert projection: for expert e and grouped row r in
 * [offsets[e], offsets[e+1]):  C[r,:] = A[src(r),:] * W[e]^T, with
 * src(r) = row_map[r] / row_div when row_map != NULL (gather; pass perm and
 * row_div = k to read token rows), else src(r) = r.
 * A: [*,K]; W: [E,N,K]; offsets: [E+1] device; C: [rows,N] where rows is the
 * host-known total offsets[E].  All E weight matrices are streamed from HBM
 * once per call when every expert has at most 128 rows (bandwidth-bound).
 * Requires K % 8 == 0, N % 2 == 0.  No workspace.
 */
int ts_moe_gemm(const ts_bf16* A, const int32_t* row_map, int row_div, const ts_bf16* W,
                const int32_t* offsets, ts_bf16* C, int rows, int E, int N, int K, void* stream);

/* out[t,:] = residual[t,:] + sum_s topk_w[t,s] * y[r(t,s),:], perm[r(t,s)] = t*k+s.
 * y: [T*k,H] grouped order; perm: [T*k]; topk_w: [T,k] fp32; residual: [T,H] or NULL; out: [T,H].
 * scratch_inv: device int32[T*k] scratch (inverse permutation), contents undefined afterwards.
 * Requires H % 8 == 0.
 */
int ts_moe_combine(const ts_bf16* y, const int32_t* perm, const float* topk_w,
                   const ts_bf16* residual, ts_bf16* out, int32_t* scratch_inv, int T, int k, int H,
                   void* stream);

/* ---------------------------------------------------------------------------
 * Whole decoder layer on one stream, no host synchronisation inside:
 *   rmsnorm -> QKV -> rope + KV append -> attention -> O (+x) -> rmsnorm ->
 *   dense:  gate|up -> swiglu -> down (+x2)
 *   MoE:    router logits -> route -> grouped gate|up -> swiglu -> grouped down -> combine (+x2)
 * Every arrow is a separate kernel with a materialised buffer between, because
 * those buffers are the edges the method may cut between GPUs (Sec. 3.1, 3.3).
 */
typedef struct ts_layer_desc {
  int32_t H, nq, nkv, d, F;
  int32_t E, k;          /* E == 0: dense MLP */
  int32_t Lcap;          /* positions per cache row */
  int32_t mode;          /* TS_MODE_DECODE | TS_MODE_PREFILL */
  float eps, rope_base;
} ts_layer_desc;

typedef struct ts_layer_weights {
  const ts_bf16* gamma1;    /* [H] */
  const ts_bf16* w_qkv;     /* [(nq+2nkv)d, H], rows = q heads, then k heads, then v heads */
  const ts_bf16* w_o;       /* [H, nq*d] */
  const ts_bf16* gamma2;    /* [H] */
  const ts_bf16* w_router;  /* [E,H] (MoE) or NULL */
  const ts_bf16* w_gate_up; /* [2F,H] = [gate rows | up rows]; MoE: [E,2F,H] */
  const ts_bf16* w_down;    /* [H,F]; MoE: [E,H,F] */
  const float* rope_cos_sin;/* optional device table [rope_table_len, d] or NULL */
  int32_t rope_table_len;
} ts_layer_weights;

typedef struct ts_layer_io {
  const ts_bf16* x;          /* [T,H] */
  ts_bf16* out;              /* [T,H] */
  const int32_t* pos;        /* [T] */
  const int32_t* seq_id;     /* [T] */
  const int32_t* seq_lens;   /* decode: [B] keys attended after the append */
  const int32_t* cu_seqlens; /* prefill: [B+1] */
  ts_bf16* kcache;           /* [Bcache,nkv,Lcap,d], in/out */
  ts_bf16* vcache;
  int32_t T, B;
  int32_t max_seqlen;        /* prefill: host-known bound on a sequence's token count */
} ts_layer_io;

/* Kernel-boundary buffers of the layer, in kernel order.  Dense layers have
 * TS_NB_DENSE of them, MoE layers TS_NB_MOE. */
enum {
  TS_B_H1 = 0, TS_B_QKV = 1, TS_B_ATTN = 2, TS_B_X2 = 3, TS_B_H2 = 4,
  TS_B_GATE_UP = 5, TS_B_ACT = 6,
  TS_B_OUT_DENSE = 7, TS_NB_DENSE = 8,
  TS_B_Y_MOE = 7, TS_B_OUT_MOE = 8, TS_NB_MOE = 9
};

/* Bytes of workspace ts_layer_forward needs for T tokens / B sequences (0 on invalid desc). */
size_t ts_layer_workspace_bytes(const ts_layer_desc* desc, int T, int B);
/* Where boundary `index` lives: byte offset inside the workspace (or (size_t)-1 for the last
 * boundary, which is io->out) and its size in bytes.  Host-only arithmetic. */
int ts_layer_boundary(const ts_layer_desc* desc, int T, int B, int index, size_t* ws_offset,
                      size_t* bytes);
/* Where the MoE routing outputs live inside the workspace (host-only arithmetic):
 * offsets of logits f32[T,E], topk_idx i32[T,k], topk_w f32[T,k], counts i32[E], offsets i32[E+1], perm i32[T*k]. */
int ts_layer_moe_buffers(const ts_layer_desc* desc, int T, int B, size_t ws_offsets[6]);
/* The byte ranges that node `node` of the layer (the group of kernels that ends at kernel boundary `node`, see
 * ts_layer_node_name) reads and writes when ts_layer_forward runs it: the hand-declared counterpart of the
 * [min, max] range the paper's kernel analyzer derives per memory instruction (Sec. 3.1, "Memory access
 * analysis"), and what ts_layer_ddg feeds to the dependency analysis.  An access names one of the layer's five
 * buffers and a byte range inside it: offset, extent (the hull) and the bytes really touched inside the hull;
 * iter_advance as in ts_access.  kind: TS_ACC_READ, TS_ACC_WRITE, or TS_ACC_PRIVATE for scratch that the node
 * writes and reads back itself (split-K and split-KV partials, arrival counters, the inverse permutation of the
 * MoE combine): it carries nothing between nodes and its contents are undefined afterwards.  Decode: kv_len =
 * keys each sequence attends, the appended one included (the declaration assumes equal lengths; the append is
 * one row per sequence and kv head at position kv_len - 1).  Prefill ignores kv_len.  Weights are never written
 * and are left out.  HOST-only arithmetic; `out` is a host array of max_accesses entries; if more are needed,
 * *n_accesses is the number and TS_ERR_WORKSPACE is returned with nothing written.
 * A GPU test fills everything outside the declared write ranges with a pattern and everything the layer does
 * not produce itself with NaNs and checks that the kernels stay inside these declarations. */
#define TS_BUF_WORKSPACE 0
#define TS_BUF_X 1
#define TS_BUF_OUT 2
#define TS_BUF_KCACHE 3
#define TS_BUF_VCACHE 4
#define TS_ACC_READ 0
#define TS_ACC_WRITE 1
#define TS_ACC_PRIVATE 2
typedef struct ts_layer_access {
  int32_t buffer, kind;
  uint64_t offset, extent, bytes;
  int64_t iter_advance;
} ts_layer_access;
int ts_layer_node_accesses(const ts_layer_desc* desc, int T, int B, int kv_len, int node, ts_layer_access* out,
                           int max_accesses, int* n_accesses);
/* Enqueues the whole layer on `stream` and returns; kernels only: no allocation, no memset, no copy-engine
 * command, no host synchronisation, so the call may be recorded into a HIP graph by stream capture and
 * replayed (sizes, pointers and sequence lengths are those of the capture; the lengths are read from
 * device memory at run time). */
int ts_layer_forward(const ts_layer_desc* desc, const ts_layer_weights* w, const ts_layer_io* io,
                     void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Pipelined micro-batch step (Sec. 3.3): micro-batch i runs the layer on
 * compute stream i % 2; after every flagged kernel boundary an event is
 * recorded and, on the copy stream, the boundary tensor is packed into the
 * micro-batch's contiguous staging slot and copied to pinned host memory (the
 * stand-in for the `send` on a cut edge).  Compute streams never wait for the
 * copy stream except before a workspace slot is reused by a later micro-batch.
 *
 * ts_pipeline owns only HIP events (created by the first step, so creating and
 * destroying a pipeline needs no GPU).  boundary_mask bit i selects boundary i.
 * Layout: ts_pipeline_boundary_layout gives, for the flagged boundaries in
 * kernel order, byte offsets inside one micro-batch slot (offsets[n] = slot
 * bytes).  Slot i of dev_staging / pinned_host starts at i * slot_stride where
 * slot_stride = offsets[n] rounded up to 256.
 * dev_staging: device, >= n_mb*slot_stride bytes.  pinned_host: HOST pinned
 * memory of the same size that the device can address (hipHostMalloc, or a
 * torch tensor created with pin_memory): the pack kernel stores to it
 * directly, no copy-engine command is issued.  ws: device, at least two workspace slots of
 * ts_pipeline_workspace_slot_bytes(desc, Ts, Bs, n_mb) bytes each: the largest, over the micro-batches, of
 * ts_layer_workspace_bytes(desc, T_i, B_i) rounded up to 256 (that size is NOT monotone in T or B, so the
 * plan of the largest micro-batch is not enough; TS_ERR_WORKSPACE otherwise).  The step uses as many
 * workspace slots of that size as ws_bytes holds (at most n_mb): micro-batch i works in slot i % nslot and
 * waits, before it starts, for the transfers and the kernels of the micro-batch that used the slot before
 * it, in this step or the previous one, whichever streams those ran on.  With n_mb slots no micro-batch
 * waits for a transfer of its own step.
 * All micro-batches must flag the same boundaries; their T may differ (the
 * layout is computed for each T; slot_stride uses the largest).
 * copy_mode: TS_PIPE_COPY_SIDE_STREAM sends every flagged boundary as soon as its kernel is enqueued (one
 * event per boundary, carried by the kernel that completes it); TS_PIPE_COPY_SERIALISED runs the pack kernels on the compute
 * stream itself (the no-overlap reference); TS_PIPE_COPY_COALESCED sends on the side stream at four
 * points of the layer (after RoPE, after the second norm, after SwiGLU, at the end), each send carrying
 * the flagged boundaries produced since the previous one: half the events and pack launches, same bytes in
 * the same slots.
 * TS_PIPE_COPY_COALESCED_HALVES sends twice per layer (after the attention half, i.e. once x2 exists, and
 * at the end; a send carries at most four tensors, so a layer with more than eight boundaries sends a third
 * time): a quarter of the events.  A boundary then leaves up to half a layer after it was produced, which
 * costs a consumer on another GPU latency, not throughput.
 * The call returns after enqueueing; steps may be enqueued back to back (each waits for the transfers of
 * the previous one that still read its workspace slot); the caller synchronises the streams before it
 * reads the slots or frees the buffers.
 */
#define TS_PIPE_COPY_SIDE_STREAM 0
#define TS_PIPE_COPY_SERIALISED 1
#define TS_PIPE_COPY_COALESCED 2
#define TS_PIPE_COPY_COALESCED_HALVES 3
typedef struct ts_pipeline ts_pipeline;
int ts_pipeline_create(const ts_layer_desc* desc, int max_micro_batches, ts_pipeline** out);
void ts_pipeline_destroy(ts_pipeline* p);
int ts_pipeline_boundary_layout(const ts_layer_desc* desc, int T, int B, uint64_t boundary_mask,
                                size_t* offsets /* host, [n+1] */, int* n_boundaries);
size_t ts_pipeline_slot_stride(const ts_layer_desc* desc, int T, int B, uint64_t boundary_mask);
/* Bytes of one workspace slot of ts_pipeline_step for micro-batches of Ts[i] tokens / Bs[i] sequences (HOST
 * arrays of n_mb entries); 0 on invalid arguments.  Host-only arithmetic. */
size_t ts_pipeline_workspace_slot_bytes(const ts_layer_desc* desc, const int32_t* Ts, const int32_t* Bs, int n_mb);
/* Background replication of the KV-cache delta (Sec. 4: buffers with a cross-iteration dependency keep a
 * replica per GPU and the rows written in an iteration are propagated asynchronously, apart from the
 * dependency transfers).  Once set, every ts_pipeline_step also packs, for each micro-batch i, the K and V
 * rows its tokens append to the cache into slot i of dev_slots and host_slots (device memory and
 * device-addressable pinned host memory, slot stride ts_pipeline_kv_delta_stride(desc, Tmax), layout
 * [T][K row of nkv*d | V row of nkv*d] bf16, keys already rotated) with a small kernel on delta_stream,
 * which the compute streams wait for only before the workspace slot is reused.  All streams here have
 * the default priority.  Passing dev_slots = host_slots = NULL switches it off.  `bytes` is the size of
 * each of the two buffers; ts_pipeline_step checks it against n_mb * stride. */
size_t ts_pipeline_kv_delta_stride(const ts_layer_desc* desc, int T);
int ts_pipeline_set_kv_delta(ts_pipeline* p, void* delta_stream, void* dev_slots, void* host_slots,
                             size_t bytes);
/* Slower link (Sec. 5, sensitivity of the method to the interconnect bandwidth: 200 down to 25 Gbps): from the
 * next step on every boundary tensor is stored `factor` times to its pinned-host slot, so the bytes that
 * cross the host link are multiplied and the link looks `factor` times slower to the step; slot contents and
 * everything on the device are unchanged.  factor in [1,64], 1 = off (default).  Host; TS_ERR_INVALID_ARG
 * otherwise.  The KV delta stream is not affected. */
int ts_pipeline_set_link_slowdown(ts_pipeline* p, int factor);
int ts_pipeline_step(ts_pipeline* p, const ts_layer_weights* w, const ts_layer_io* mb, int n_mb,
                     void* compute_streams[2], void* copy_stream, uint64_t boundary_mask,
                     int copy_mode, void* dev_staging, void* pinned_host,
                     size_t staging_bytes, void* ws, size_t ws_bytes);

/* ---------------------------------------------------------------------------
 * Kernel analyzer: data-dependency graph (Sec. 3.1, "Data dependency analysis").
 * HOST-only: every pointer below is host memory, nothing touches the GPU.
 *
 * A kernel is described by the byte ranges it reads and writes.  An access is
 * the hull [addr, addr + extent) of what the kernel touches in one buffer plus
 * the number of bytes it really touches inside it (bytes <= extent; a strided
 * or indexed access has bytes < extent).  iter_advance is the number of bytes
 * the range moves forward from one iteration to the next (0 for ordinary
 * buffers; one cache position for the append of a decode step).
 *
 * ts_ddg_build visits the kernels in execution order for two consecutive
 * iterations, keeping for every byte its last writer.  A read adds an edge from
 * the most recent writer of each part of its range (read-after-write only; a
 * kernel reads before it writes and never depends on itself); the bytes on the
 * edge are min(overlap, bytes written, bytes read), summed over the buffers
 * shared by the two kernels.  Edges found in the second iteration whose writer
 * ran in the first have cross_iteration = 1.
 * Output: edges[0..*n_edges), intra-iteration edges first, each group sorted by
 * (src, dst).  If more than max_edges exist, *n_edges is the number needed and
 * TS_ERR_WORKSPACE is returned with nothing written to edges.
 */
typedef struct ts_access {
  uint64_t addr, extent, bytes;
  int64_t iter_advance;
} ts_access;
typedef struct ts_kernel_io {
  const ts_access* reads;
  const ts_access* writes;
  int32_t n_reads, n_writes;
} ts_kernel_io;
typedef struct ts_ddg_edge {
  int32_t src, dst;          /* kernel indices, src is the writer */
  uint64_t bytes;
  int32_t cross_iteration;   /* 1: the value comes from the previous iteration */
  int32_t reserved;
} ts_ddg_edge;
int ts_ddg_build(const ts_kernel_io* kernels, int n_kernels, ts_ddg_edge* edges, int max_edges,
                 int* n_edges);

/* The dependency graph of n_layers decoder layers of `desc` at T tokens / B
 * sequences, built by ts_ddg_build from the buffers ts_layer_forward really
 * uses (workspace offsets of the kernel boundaries, the routing tables of a MoE
 * layer, the residual input, the KV caches).  A node is the group of kernels
 * that ends at one kernel boundary, so node (layer * NB + i) produces boundary
 * i of that layer (NB = TS_NB_DENSE or TS_NB_MOE); ts_layer_node_name names it.
 * Decode: the cache append is modelled row by row with iter_advance = one
 * position, kv_len = keys each sequence attends (>= 1), so the cache shows up
 * as a cross-iteration edge carrying one iteration's new K/V rows.  Prefill:
 * attention reads K/V from the projection output and kv_len is ignored.
 * Weights are never written and are left out.  Same output rules as ts_ddg_build.
 */
int ts_layer_ddg(const ts_layer_desc* desc, int T, int B, int kv_len, int n_layers,
                 ts_ddg_edge* edges, int max_edges, int* n_edges);
const char* ts_layer_node_name(const ts_layer_desc* desc, int node_in_layer);
/* boundary_mask for ts_pipeline_step from a placement of one layer's nodes:
 * placement[i] is the GPU of node i, placement[NB] the GPU that consumes the
 * layer's output.  Bit i is set when some consumer of boundary i sits on
 * another GPU than its producer.  TS_ERR_UNSUPPORTED_SHAPE if the placement
 * separates kernels that exchange data outside the kernel boundaries (the
 * routing tables of a MoE layer). */
int ts_layer_cut_mask(const ts_layer_desc* desc, const int32_t* placement, uint64_t* boundary_mask);

/* ---------------------------------------------------------------------------
 * Policy planner (Sec. 3.2).  HOST-only.
 * Chooses placement[k] in [0, n_gpus) for every kernel so as to minimise
 *   TS_PLAN_THROUGHPUT:  max_g max(T_g, M_g)      (the slowest pipeline stage)
 *   TS_PLAN_LATENCY:     sum_g T_g + sum_g M_g    (every kernel and every cut edge once)
 * with T_g = sum of t[k][g] over kernels placed on g and M_g = sum over edges
 * (i, j) with j on g and i on u != g of lat[u][g] + bytes / bw[u][g].
 * t: [n_kernels][n_gpus] seconds; bw: [n_gpus][n_gpus] bytes/s; lat: same
 * shape, seconds (diagonals ignored; both may be NULL when n_gpus == 1).
 * Edges must satisfy src < dst; edges with cross_iteration != 0 are ignored
 * (such buffers are replicated and their deltas shipped in the background).
 * The latency objective is solved exactly.  The throughput objective is solved
 * by branch and bound, exactly unless more than node_limit search nodes are
 * needed (node_limit <= 0: 5e7); then the best placement found is returned and
 * *proved_optimal = 0.  T_g, M_g (each [n_gpus]) and proved_optimal may be NULL.
 * Ties between optimal placements are broken arbitrarily.
 */
#define TS_PLAN_THROUGHPUT 0
#define TS_PLAN_LATENCY 1
typedef struct ts_plan_problem {
  int32_t n_kernels, n_gpus, n_edges, reserved;
  const double* t;
  const ts_ddg_edge* edges;
  const double* bw;
  const double* lat;
} ts_plan_problem;
int ts_plan_policy(const ts_plan_problem* problem, int objective, int64_t node_limit,
                   int32_t* placement, double* value, double* T_g, double* M_g,
                   int* proved_optimal);
/* The same search with a stopping rule and its certificate.  It stops as soon as the placement found is within
 * rel_gap (relative, in [0, 1); 0 = never) of a lower bound of the optimum that needs no search (the one
 * ts_plan_lower_bound returns), which proves the placement optimal to that tolerance; the paper's solver call
 * has the same kind of gap (Sec. 3.2, Sec. 5.4: about 500 kernels in 20 ms, 1500 in under a second).  Before and
 * after the branch and bound a two-GPU throughput placement is balanced by moving whole classes of equal kernels
 * (a decoder stack repeats a handful of shapes; Sec. 5.4 notes the same redundancy).
 * *status: 2 = proved optimal (search finished), 1 = within rel_gap of *lower_bound, 0 = stopped by node_limit
 * (the placement is valid and (value - *lower_bound) / value bounds its distance from the optimum).
 * lower_bound and status may be NULL. */
int ts_plan_policy_bounded(const ts_plan_problem* problem, int objective, int64_t node_limit, double rel_gap,
                           int32_t* placement, double* value, double* T_g, double* M_g, double* lower_bound,
                           int* status);
/* A lower bound of the optimum of `objective` that needs no search: the sum over kernels of their fastest
 * time for the latency objective; for the throughput objective the larger of that sum divided by the number
 * of GPUs and, with two GPUs, the makespan of the best fractional split of the kernels without communication.
 * (value - bound) / value bounds the optimality gap of a ts_plan_policy result that was stopped by its
 * node limit. */
int ts_plan_lower_bound(const ts_plan_problem* problem, int objective, double* lower_bound);

/* ---------------------------------------------------------------------------
 * Online monitor (Sec. 3.4).  HOST-only, O(1) state, not thread-safe.
 * Time is cut into windows [n W, (n+1) W).  ts_monitor_record reports one
 * finished request: its completion time (seconds on any monotonic clock that
 * starts at 0), its end-to-end latency, the latency of each of its kernel
 * groups (the kernels between two consecutive communication operations) and
 * its communication time; execution latency = sum of the groups + comm.
 * Completion times may arrive in any order inside the open window but never
 * in a window that has already closed (TS_ERR_INVALID_ARG).
 * When a window closes with at least one completion, ratio = (mean request
 * latency) / (mean execution latency); ratio > beta selects
 * TS_PLAN_THROUGHPUT, otherwise TS_PLAN_LATENCY.  Empty windows keep the policy.
 * ts_monitor_advance closes every window that ended at or before now_s and
 * reports the policy in effect, the number of windows closed and of policy
 * switches so far, and the ratio of the last non-empty window (NaN before the
 * first); any of the four outputs may be NULL.  The paper's defaults are
 * window_s = 0.3 and beta = 1.5 (Sec. 5.4).
 */
typedef struct ts_monitor ts_monitor;
int ts_monitor_create(double window_s, double beta, int initial_policy, ts_monitor** out);
void ts_monitor_destroy(ts_monitor* m);
int ts_monitor_record(ts_monitor* m, double t_complete_s, double request_latency_s,
                      const double* group_latency_s, int n_groups, double comm_s);
int ts_monitor_advance(ts_monitor* m, double now_s, int* policy, int64_t* windows_closed,
                       int64_t* n_switches, double* last_ratio);
#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* TESSERA_H_ */
