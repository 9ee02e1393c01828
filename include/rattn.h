/*
 * rattn.h - C ABI of librattn: the RAttention token-mixing layer on one MI355X (gfx950).
 *
 * The layer (paper Sec. 3.1-3.2) maps shared q/k/v to
 *     o_t = RMS_s(x^s_t) + RMS_r(x^r_t)
 * where x^s is sliding-window softmax attention over the last `window` keys (Sec. 2.1)
 * and x^r = phi(q_t) S_{t-window} is residual linear attention over every older key
 * (Eq. 4), S_t = sum_{s<=t} phi(k_s)^T v_s, phi = softmax over the head features, with
 * group-query sharing of k/v (Sec. 3.1) and separate per-head RMS gains (Sec. 3.2).
 *
 * Conventions
 *  - Positions are 0-based.  `window` = W >= 1 counts the keys the softmax branch sees
 *    INCLUDING the current one: query t attends keys max(0,t-W+1)..t and the linear
 *    branch covers keys 0..t-W.  The paper's symbol is w = W-1.  W >= T leaves the
 *    linear branch empty (its output and RMS are exactly 0) = causal attention.
 *  - Layer tensors are contiguous [B, T, H, D], D fastest.  Query head h reads KV head
 *    h / (Hq/Hkv).  D is 64 or 128.  The matrix-core kernels take bf16 tensors with
 *    window >= 8 and T >= 128: D = 128 in place (of a T that is no multiple of 128 only the
 *    last, partial 128-row tile of every sequence goes through zero-padded buffers in the
 *    workspace), D = 64 through copies widened to 128 features that live in the workspace;
 *    every other shape (fp32, T < 128, tiny windows) runs on the general (vector-ALU) kernels.
 *  - dtype is the element type of q,k,v,o,dO,dq,dk,dv (and of the decode ring buffers).
 *    Accumulators, softmax/RMS statistics and gains are fp32.  Linear-attention states are
 *    accumulated in fp32; the decode, prefill-export and general kernels also keep them in
 *    fp32, while the matrix-core layer kernels (bf16, D = 128) store each per-128-key chunk
 *    state once as a bf16 matrix-core operand (a carried-in fp32 state of rattn_prefill_chunk
 *    is rounded the same way where it enters those kernels).
 *  - Every pointer is a DEVICE pointer unless stated otherwise.  The caller owns all
 *    buffers; the library never allocates, frees or synchronises.  All work is enqueued
 *    on `stream` (a hipStream_t passed as void*; NULL = the default stream).  Outputs are
 *    overwritten, never accumulated into.
 *  - Errors: every call returns a rattn_status; arguments are validated on the host
 *    before anything is launched, so a failed call has launched nothing.
 *    rattn_last_error() returns a thread-local human-readable detail string.
 *  - Results are deterministic for fixed inputs and parameters (no floating-point atomics).
 */
#ifndef RATTN_H
#define RATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RATTN_OK = 0,
  RATTN_ERR_INVALID_ARG = -1,   /* NULL pointer, non-positive size, Hq % Hkv != 0, eps <= 0 ... */
  RATTN_ERR_UNSUPPORTED = -2,   /* D not in {64,128}, unknown dtype                             */
  RATTN_ERR_WORKSPACE = -3,     /* workspace_bytes smaller than rattn_workspace_bytes reports   */
  RATTN_ERR_HIP = -4            /* a HIP launch failed; detail in rattn_last_error()            */
} rattn_status;

typedef enum { RATTN_F32 = 0, RATTN_BF16 = 1 } rattn_dtype;

/* Feature map phi of the linear branch, applied to every q and k row over its D features.  The layer uses the
 * softmax map (Sec. 3.1, "Parameterization"); the other two are the alternatives of the ablation (Sec. 4.5):
 * ReLU = max(x, 0) per feature, identity = x.  Zero-initialised parameter structs select the softmax map.
 * With the identity map only calls with save_for_bwd = 0 use the matrix-core kernels: a training step (forward that
 * saves + backward) runs on the general kernels, because its backward is not accurate enough with bf16 operands. */
typedef enum { RATTN_PHI_SOFTMAX = 0, RATTN_PHI_RELU = 1, RATTN_PHI_IDENTITY = 2 } rattn_feature_map;

typedef struct {
  int32_t B, T, Hq, Hkv, D;
  int32_t window;        /* W >= 1 (see conventions)                                                   */
  int32_t chunk;         /* linear-branch chunk size C of Eqs. 2-3 (0 = library chooses); the result does not
                            depend on it beyond rounding.  General kernels: any value; matrix-core kernels:
                            64 or 128 keys per chunk product (other values mean 128)                   */
  int32_t dtype;         /* rattn_dtype                                                                */
  float softmax_scale;   /* multiplies q.k in the softmax branch only (the paper's formula is 1.0)     */
  float rms_eps;         /* > 0                                                                        */
  int32_t save_for_bwd;  /* rattn_fwd also fills `saved` (needed by rattn_bwd)                         */
  int32_t feature_map;   /* rattn_feature_map                                                          */
  int32_t kernel_path;   /* rattn_kernel_path: 0 = the library chooses (matrix-core kernels where the
                            shape allows); RATTN_PATH_GENERAL forces the general kernels (a second,
                            independent implementation used by tests).  It changes what `saved` holds:
                            rattn_fwd and rattn_bwd of one step must be given the same value           */
  int32_t state_policy;  /* rattn_state_policy: what rattn_fwd keeps of the linear-branch chunk states for
                            rattn_bwd (matrix-core kernels; ignored by the general kernels, which always rebuild).
                            Same value in both calls: it changes what `saved` holds                           */
} rattn_params;

typedef enum { RATTN_PATH_AUTO = 0, RATTN_PATH_GENERAL = 1 } rattn_kernel_path;

/* The paper's kernel stores chunk states only every m-th chunk and recomputes the others to save accelerator memory,
 * "storing more leads to faster backward passes ... at a higher memory cost" (Sec. 3.2, Fig. 3); it searches over m and
 * the chunk size C.  Here the same trade is selectable: KEEP stores every chunk state (one per 128 keys, bf16) in
 * `saved` so that backward reads them (m = 1); KEEP_EVERY_2ND / _4TH store states 0, m, 2m, ... and backward forms only
 * the chunk products that lead to the states in between, continuing from the stored ones (m = 2, 4); REBUILD stores
 * none and backward builds all of them again from k and v.  The chunk size of the state-building kernels is the `chunk`
 * parameter: 64 selects 64-key chunk products (two per state), anything else 128-key products. */
typedef enum {
  RATTN_STATES_KEEP = 0,
  RATTN_STATES_REBUILD = 1,
  RATTN_STATES_KEEP_EVERY_2ND = 2,
  RATTN_STATES_KEEP_EVERY_4TH = 4
} rattn_state_policy;

/* Sizes in bytes of the scratch `workspace` rattn_fwd / rattn_bwd need and of the opaque
 * `saved` buffer rattn_fwd fills for rattn_bwd.  Any of the three out pointers (HOST) may
 * be NULL.  Sizes depend on every field of *p except save_for_bwd. */
rattn_status rattn_workspace_bytes(const rattn_params* p, size_t* fwd_bytes, size_t* bwd_bytes,
                                   size_t* saved_bytes);

/* Forward of the layer (Sec. 2.1 softmax branch, Eqs. 2-4 linear branch in chunkwise form
 * with phi computed in-kernel, Sec. 3.2 combination).
 *   q [B,T,Hq,D]; k,v [B,T,Hkv,D]; o [B,T,Hq,D]
 *   gamma_swa, gamma_rla: fp32 [Hq,D] RMS gains of the two branches, NULL = all ones
 *   saved: opaque, saved_bytes large, written iff p->save_for_bwd (else may be NULL);
 *          holds the pre-norm branch outputs, the softmax / RMS row statistics and, on the
 *          matrix-core path, the linear-branch chunk states
 *   workspace: fwd_bytes of scratch (16-byte aligned), contents undefined on return */
rattn_status rattn_fwd(const rattn_params* p, const void* q, const void* k, const void* v,
                       const float* gamma_swa, const float* gamma_rla, void* o, void* saved,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the layer: gradients of sum(o * dO) w.r.t. q, k, v and the gains.
 * Derived from Sec. 2.1, Eq. 4 and Sec. 3.2 (the linear-branch state gradients are the
 * reverse-time counterpart of Eqs. 2-3).
 *   saved: as written by rattn_fwd with the same params (incl. kernel_path) and inputs
 *   dq [B,T,Hq,D]; dk,dv [B,T,Hkv,D] (summed over the query heads of each group)
 *   dgamma_swa, dgamma_rla: fp32 [Hq,D], each may be NULL (then not computed) */
rattn_status rattn_bwd(const rattn_params* p, const void* q, const void* k, const void* v,
                       const float* gamma_swa, const float* gamma_rla, const void* saved,
                       const void* dO, void* dq, void* dk, void* dv, float* dgamma_swa,
                       float* dgamma_rla, void* workspace, size_t workspace_bytes, void* stream);

/* rattn_fwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and errors as rattn_fwd
 * (bit-identical output: the same kernels run), but the scratch memory is a buffer of RATTN_STATIC_SCRATCH_BYTES
 * that lives inside the library's device image (one copy per GPU, held until the process ends); the call itself
 * allocates and frees nothing.  Shapes whose forward workspace (rattn_workspace_bytes: fwd_bytes) exceeds that
 * size are rejected with RATTN_ERR_WORKSPACE before anything is launched.  The first call on a device looks the
 * buffer's address up once (make that call outside graph capture).  All calls on one GPU share the buffer:
 * calls that may overlap on the same GPU (different streams, different threads) race and must be serialised
 * by the caller; its contents are undefined between calls. */
#define RATTN_STATIC_SCRATCH_BYTES ((size_t)96 << 20)
rattn_status rattn_fwd_static(const rattn_params* p, const void* q, const void* k, const void* v,
                              const float* gamma_swa, const float* gamma_rla, void* o, void* saved,
                              void* stream);

typedef struct {
  int32_t N;             /* sequences in the batch                                   */
  int32_t Hq, Hkv, D;
  int32_t window;        /* W >= 1: ring capacity in tokens                          */
  int32_t dtype;         /* of q, k_new, v_new, rings, o                             */
  float softmax_scale;
  float rms_eps;
  int32_t feature_map;   /* rattn_feature_map, as in rattn_params                    */
} rattn_decode_params;

/* One generated token per sequence with constant memory (Sec. 2.1: a cache of the last W
 * keys; Sec. 2.2: a fixed D x D state; Eq. 4).  For sequence n with pos[n] = p:
 *   1. if p >= W the key/value leaving the window (token p-W, stored in slot p % W) is
 *      folded into the state: state += phi(k_old)^T v_old;
 *   2. slot p % W of the rings is overwritten with (k_new, v_new);
 *   3. x^s = softmax attention of each query head over the min(p+1, W) valid slots,
 *      x^r = phi(q) state, o = RMS_s(x^s) + RMS_r(x^r).
 *   q [N,Hq,D]; k_new,v_new [N,Hkv,D]; pos int32 [N] (device), 0-based index of the new
 *   token, >= 0; k_ring,v_ring [N,Hkv,W,D] updated in place, token s lives in slot s % W;
 *   state fp32 [N,Hkv,D,D] (row = feature of phi(k), column = value feature), updated in
 *   place; o [N,Hq,D].  No workspace. */
rattn_status rattn_decode_step(const rattn_decode_params* p, const void* q, const void* k_new,
                               const void* v_new, const int32_t* pos, void* k_ring, void* v_ring,
                               float* state, const float* gamma_swa, const float* gamma_rla,
                               void* o, void* stream);

/* Prefill -> decode hand-over (Sec. 2.1: the window cache; Sec. 2.2 and Eq. 4: the lagged state).  From the keys
 * and values of a prompt of T tokens (k, v [B,T,Hkv,D] as in rattn_fwd; Hq, chunk, softmax_scale, rms_eps,
 * save_for_bwd of *p are not used but must be valid) it fills what rattn_decode_step with pos = T expects for
 * the N = B sequences:
 *   k_ring, v_ring [B,Hkv,W,D]: token s in slot s % W for s in [max(0, T-W), T); other slots are left untouched;
 *   state fp32 [B,Hkv,D,D] = sum over s < T-W of phi(k_s)^T v_s (row = feature, column = value), zero if T <= W,
 *   summed in a fixed order (deterministic).
 * workspace: rattn_prefill_export_workspace_bytes() bytes of scratch (may be 0 => NULL allowed). */
rattn_status rattn_prefill_export_workspace_bytes(const rattn_params* p, size_t* bytes);
rattn_status rattn_prefill_export(const rattn_params* p, const void* k, const void* v, void* k_ring,
                                  void* v_ring, float* state, void* workspace, size_t workspace_bytes,
                                  void* stream);

/* Chunked prefill (Sec. 2.1: the window cache; Sec. 2.2 and Eq. 4: the state carried between chunks).  The layer's
 * forward for tokens pos0 .. pos0 + T - 1 of B sequences whose first pos0 tokens (pos0 >= 0, HOST value, the same
 * for every sequence) are present only as rings and state, i.e. as rattn_prefill_export / rattn_prefill_chunk /
 * rattn_decode_step leave them at position pos0.  The result equals rows pos0 .. pos0 + T - 1 of rattn_fwd over the
 * whole sequence.
 *   p: B, T (= tokens in this chunk), Hq, Hkv, D, window, chunk, dtype, softmax_scale, rms_eps as for rattn_fwd;
 *      save_for_bwd is ignored
 *   q [B,T,Hq,D]; k,v [B,T,Hkv,D]: the chunk; o [B,T,Hq,D]
 *   k_ring, v_ring [B,Hkv,W,D], state fp32 [B,Hkv,D,D]: read (rings: the last min(pos0, W) tokens; state: only if
 *      pos0 > W, before that it is zero by definition and the buffer's contents are ignored) and updated in place
 *      to position pos0 + T (slots of tokens that stay in the window are left as they are)
 *   workspace: rattn_prefill_chunk_workspace_bytes(p, pos0) bytes of scratch, 16-byte aligned.
 * The matrix-core kernels are used when dtype = bf16, D = 128, window >= 8 and min(pos0, W) + T >= 128; any other
 * shape runs on the general kernels. */
rattn_status rattn_prefill_chunk_workspace_bytes(const rattn_params* p, int32_t pos0, size_t* bytes);
rattn_status rattn_prefill_chunk(const rattn_params* p, int32_t pos0, const void* q, const void* k, const void* v,
                                 const float* gamma_swa, const float* gamma_rla, void* k_ring, void* v_ring,
                                 float* state, void* o, void* workspace, size_t workspace_bytes, void* stream);

/* Closed forms of the paper's inference analysis (Sec. 4.4), evaluated on the HOST: nothing is launched, every
 * argument is a host value and the result is written to *out (HOST).
 *
 * rattn_cache_bytes: bytes of decode cache one sequence holds in a stack of `layers` token-mixing layers of which
 * every `global_every`-th is global attention (0 = none) and the others are local with `window` keys: a global
 * layer keeps ctx tokens, a local one min(ctx, window) tokens, each token 2 * Hkv * D * elem_bytes (key and value),
 * and a local layer with `with_state` != 0 also one fp32 D x D state per KV head (Sec. 2.2).
 *
 * rattn_step_time_model: T_step = batch * cache_bytes / bandwidth + max(2 * batch * param_count / flops,
 * param_bytes / bandwidth), in seconds (bandwidth in bytes/s, flops in FLOP/s).
 * Both return RATTN_ERR_INVALID_ARG for NULL out, negative sizes or non-positive rates. */
rattn_status rattn_cache_bytes(int32_t layers, int32_t global_every, int64_t ctx, int64_t window, int32_t with_state,
                               int32_t Hkv, int32_t D, int32_t elem_bytes, double* out);
rattn_status rattn_step_time_model(double batch, double cache_bytes, double param_count, double param_bytes,
                                   double bandwidth, double flops, double* out);

/* Per-kernel timing (tracing aid; off by default).  While enabled, every kernel the library
 * launches is bracketed by a pair of HIP events recorded on the launch stream.  rattn_profile_enable(1)
 * creates a fixed pool of RATTN_PROFILE_MAX_RECORDS event pairs (the only allocation; the layer calls
 * themselves never allocate); records pile up until rattn_profile_reset(), launches beyond the pool
 * are not recorded.  rattn_profile_get waits for record `idx` to finish and returns
 * its kernel name (library-owned HOST string) and duration in milliseconds; it returns
 * RATTN_ERR_INVALID_ARG for an index outside [0, rattn_profile_count()).  Not thread-safe. */
#define RATTN_PROFILE_MAX_RECORDS 16384
void rattn_profile_enable(int on);
void rattn_profile_reset(void);
int rattn_profile_count(void);
rattn_status rattn_profile_get(int idx, const char** name, float* ms);

/* Machine probe for benchmarks: enqueues a kernel of `blocks` work-groups (256 threads) in which every wave issues
 * 16 * iters bf16 matrix-core instructions (v_mfma_f32_32x32x16_bf16) and nothing else; *flops (HOST, may be NULL)
 * receives the floating-point operations issued.  The caller times the stream.  sink: >= 16 bytes of device
 * memory (never written in practice).  A measurement aid, not an operation of the paper: the benchmark reports
 * the rate this loop sustains next to the published matrix-core peak. */
rattn_status rattn_probe_mfma(void* sink, int iters, int blocks, double* flops, void* stream);

/* Static description of a status code. */
const char* rattn_status_string(rattn_status s);
/* Detail of the last failure on the calling thread ("" if none). HOST string, library-owned. */
const char* rattn_last_error(void);
/* Library version, e.g. "0.1". */
const char* rattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RATTN_H */
