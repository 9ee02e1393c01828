// Host-side declarations shared by the C ABI (api.hip) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace rattn {

// per-kernel event timing (see rattn_profile_* in rattn.h); no-ops while profiling is off
void prof_begin(const char* name, hipStream_t st);
void prof_end(hipStream_t st);
struct ProfScope {
  hipStream_t st;
  ProfScope(const char* name, hipStream_t s) : st(s) { prof_begin(name, s); }
  ~ProfScope() { prof_end(st); }
};

// feature map of the linear branch (values of rattn_feature_map)
enum { PHI_SOFTMAX = 0, PHI_RELU = 1, PHI_IDENTITY = 2 };

struct LayerDims {
  int B, T, Hq, Hkv, D, W, C, G;
  int Dv;   // features of a head that carry data: D, or 64 when the matrix-core kernels run a head size of 64
            // on rows zero-padded to D = 128 (the RMS norms and the softmax feature map then cover Dv features)
  int chunk_req;  // the caller's `chunk` parameter as given (0 = unspecified); C above is what the general kernels use
  int nst;  // number of chunk states per (batch, kv head): ceil(max(T-W,0) / C)
  float scale, eps;
  int phi;  // feature map of the linear branch: PHI_SOFTMAX (Sec. 3.1), PHI_RELU, PHI_IDENTITY (Sec. 4.5 ablation)
};

// views into the opaque `saved` buffer: pre-norm branch outputs ([B,T,Hq,D]; the I/O dtype on the MFMA path, fp32
// on the general path: the backward through the second RMS norm projects the upstream gradient off x^r, and where
// the state has very low rank - the first rows past the window - rounding x^r to bf16 leaves an error that the
// state multiplies back up) and the
// row statistics (fp32, [B,Hq,T]): log-sum-exp of the softmax branch and the two RMS reciprocals; on the MFMA
// path also the linear-branch chunk states (bf16, transposed), so that backward does not rebuild them
struct SavedPtrs {
  void* xs;
  void* xr;
  float* lse;
  float* rs;
  float* rr;
  void* states;  // null on the general path
  bool f32;      // x^s, x^r are stored as fp32 whatever the tensor dtype
  int state_stride;  // `states` holds every chunk state (0 or 1) or states 0, m, 2m, ... only (m = 2, 4): the
                     // forward then works on the full set in its workspace and backward rebuilds the states in
                     // between from the stored ones (Sec. 3.2: store every m-th state, recompute the others)
};

struct GenericBwdWs {
  float* states;   // [B,Hkv,nst,D,D]
  float* rstates;  // [B,Hkv,nst,D,D]
  float* dxs;      // [B,T,Hq,D]
  float* dxr;      // [B,T,Hq,D]
  float* delta;    // [B,Hq,T]
  float* dgpart;   // [2,RB,Hq,D]
  int RB;
};

void generic_fwd(const LayerDims& dm, int dtype, const void* q, const void* k, const void* v, const float* gs,
                 const float* gr, void* o, const SavedPtrs& sv, float* states, hipStream_t st);
void generic_bwd(const LayerDims& dm, int dtype, const void* q, const void* k, const void* v, const float* gs,
                 const float* gr, const SavedPtrs& sv, const void* dO, void* dq, void* dk, void* dv, float* dgs,
                 float* dgr, const GenericBwdWs& ws, hipStream_t st);

// compile-time feature-map variant (FM_* in mfma.hpp) the matrix-core kernels use for these dimensions
inline int feature_map_variant(const LayerDims& dm) {
  if (dm.phi == PHI_RELU) return 1;
  if (dm.phi == PHI_IDENTITY) return 2;
  return dm.Dv == 64 ? 3 : 0;
}

// Ragged sequence lengths on the matrix-core kernels (bf16, D = 128): the kernels work in 128-row tiles over the
// length rounded up (LayerDims::T), the caller's tensors hold Tc rows per sequence.  Tiles below 128 * (Tc / 128) are
// read and written in place; the last, partial tile of every sequence goes through [B,128,H,128] buffers that the host
// layer fills (inputs, zero past row Tc) before and copies back (results, rows below Tc) after the kernels.  The saved
// and workspace tensors are laid out for the rounded-up length.  Null where a function takes a RaggedTails*: every
// tensor holds LayerDims::T rows itself.
struct RaggedTails {
  int Tc;
  const void *q, *k, *v, *dO;   // dO: backward only
  void *o;                      // forward only
  void *dq, *dk, *dv;           // backward only
};

// MFMA forward path (bf16, D = 128, T % 128 == 0, any W >= 8)
struct FastFwdPlan {
  int W;        // window the tiles and states are laid out for: min(W, T) rounded up to a multiple of 64
  int gap;      // that minus the true window (0..63): masks and the reach of the intra-chunk part
  int base;     // key position of state 0 (0 or 64); state i sits at base + 128*i
  int nstf;     // number of states per (batch, kv head) = query tiles that have a linear branch
  int ckeys;    // keys per chunk-local product (64 or 128): the chunk size C of Eqs. 2-3 on this path
  int nchunks;  // chunk-local products needed to build them
  size_t u_bytes, state_bytes;
};
bool fast_fwd_supported(const LayerDims& dm, int dtype);
FastFwdPlan fast_fwd_plan(const LayerDims& dm);
// qt0 > 0: only query tiles qt0 .. T/128-1 are computed, and q, o and the saved tensors hold just those rows
// ([B, T - 128 qt0, Hq, D]); k, v always hold all T rows.  state0 (fp32 [B,Hkv,D(feature),D(value)], may be NULL): a
// linear-branch state that precedes key 0 and is added to every chunk state; tiles whose chunk starts before key 0
// do not see it, so the caller uses it only when no computed tile is of that kind.
void fast_fwd(const LayerDims& dm, const void* q, const void* k, const void* v, const float* gs, const float* gr,
              void* o, const SavedPtrs& sv, float* U, void* states, hipStream_t st, int qt0 = 0,
              const float* state0 = nullptr, const RaggedTails* tails = nullptr);

// linear-branch chunk states for the MFMA paths (bf16 [d][f] per state, fp32 scratch U per chunk)
// With m > 1: `subset_out` (forward) also receives states 0, m, 2m, ...; `restart` (backward) holds those states from
// the forward pass: only the chunk products that lead to a state in between are formed, and the scan restarts from
// every stored state.
void rla_forward_states(const LayerDims& dm, const FastFwdPlan& pl, const void* k, const void* v, float* U,
                        void* states, hipStream_t st, const float* state0 = nullptr,
                        const RaggedTails* tails = nullptr, void* subset_out = nullptr, const void* restart = nullptr,
                        int m = 1);
// MFMA backward path (same shape class as the MFMA forward)
struct FastBwdPlan {
  FastFwdPlan fwd;
  int nk;  // key tiles that have a linear branch = number of reverse states
  int nrchunks;  // reverse-time chunk-local products
  int RB;  // row blocks of the prep kernel (dgamma partials)
  size_t u_bytes, rstate_bytes;
};
struct FastBwdWs {
  void *dxs, *dxr;       // bf16 [B,T,Hq,128]
  float* delta;          // [B,Hq,T]
  float* U;              // chunk scratch
  void *states, *rstates;
  float* dgpart;         // [2,RB,Hq,128]
};
FastBwdPlan fast_bwd_plan(const LayerDims& dm);
// reverse-time states R_i = sum over t' >= 128(i+1) and over the group's heads of phi(q_{t'+W})^T dxr_{t'+W},
// i in [0, nk), nk = ceil((T-W)/128); stored transposed [d][f] bf16.  U needs (nk-1) chunks.
void rla_reverse_states(const LayerDims& dm, const FastBwdPlan& pl, const void* q, const void* dxr, float* U,
                        void* rstates, hipStream_t st, const RaggedTails* tails = nullptr);
void fast_bwd(const LayerDims& dm, const void* q, const void* k, const void* v, const float* gs, const float* gr,
              const SavedPtrs& sv, const void* dO, void* dq, void* dk, void* dv, float* dgs, float* dgr,
              const FastBwdWs& ws, hipStream_t st, const RaggedTails* tails = nullptr);

// prefill -> decode hand-over: rings of the last min(T, W) tokens and the state of all keys before them
struct ExportPlan {
  int Tp;        // keys folded into the state (T - W, or 0)
  int nseg;      // key segments with their own partial state
  int seg_len;   // keys per segment (multiple of the staging batch)
  size_t partial_bytes;
};
ExportPlan export_plan(const LayerDims& dm);
// Row s of k / v is token tok0 + s of its sequence (ring slots); with `accumulate` the keys that fall out of the
// window are added to what `state` already holds.
void prefill_export(const LayerDims& dm, int dtype, const void* k, const void* v, void* k_ring, void* v_ring,
                    float* state, float* partial, hipStream_t st, int tok0 = 0, bool accumulate = false);

// chunked prefill (see chunk_kernels.hip): dmc describes the concatenated sequence of R ring rows + Tc new rows
void chunk_concat(const LayerDims& dmc, int dtype, int Tc, int R, int pos0, const void* q, const void* k, const void* v,
                  const void* k_ring, const void* v_ring, void* qc, void* kc, void* vc, hipStream_t st);
void chunk_copy_out(const LayerDims& dmc, int dtype, int Tc, int R, const void* oc, void* o, hipStream_t st);
// Ls: rows per sequence of the saved tensors (> R + Tc when the forward ran on a zero-padded copy)
void chunk_fixup(const LayerDims& dmc, int dtype, int Tc, int R, int Ls, const void* qc, const SavedPtrs& sv,
                 const float* state, const float* gs, const float* gr, void* o, hipStream_t st);

// [B,T,H,head] <-> [B,Tp,H,head_padded] with zeros at t >= T and past `head_bytes` of every head row (both sizes
// multiples of 16 bytes)
void pad_rows(const void* src, void* dst, int B, int T, int Tp, int H, size_t head_bytes, size_t head_bytes_padded,
              hipStream_t st);
void unpad_rows(const void* src, void* dst, int B, int T, int Tp, int H, size_t head_bytes, size_t head_bytes_padded,
                hipStream_t st);

// rows 128 * (T / 128) .. of up to four [B,T,H,128] bf16 tensors <-> their [B,128,H,128] tail buffers (RaggedTails):
// gather fills the buffers (zero from row T on), scatter copies the rows below T back.  n tensors, H[i] heads each.
void gather_tails(int n, const void* const* src, void* const* tail, const int* H, int B, int T, hipStream_t st);
void scatter_tails(int n, const void* const* tail, void* const* dst, const int* H, int B, int T, hipStream_t st);

// launches the matrix-core probe loop; returns the FLOPs it issues
double probe_mfma(float* sink, int iters, int blocks, hipStream_t st);

struct DecodeDims {
  int N, Hq, Hkv, D, W, G;
  float scale, eps;
  int phi;  // as LayerDims::phi
};
void decode_step(const DecodeDims& dd, int dtype, const void* q, const void* k_new, const void* v_new,
                 const int32_t* pos, void* k_ring, void* v_ring, float* state, const float* gs, const float* gr,
                 void* o, hipStream_t st);

}  // namespace rattn
