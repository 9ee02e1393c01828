// C ABI of librattn: argument validation, workspace layout, path selection, launches.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kernels.hpp"
#include "rattn.h"

namespace rattn {
namespace {
// Event pairs come from a pool created by rattn_profile_enable(1): recording inside the layer calls allocates nothing.
struct ProfRec { const char* name; hipEvent_t a, b; };
bool g_prof_on = false;
ProfRec g_pool[RATTN_PROFILE_MAX_RECORDS];
int g_pool_size = 0;   // event pairs that exist
int g_prof_count = 0;  // records in use
bool g_prof_open = false;
}  // namespace
void prof_begin(const char* name, hipStream_t st) {
  g_prof_open = false;
  if (!g_prof_on || g_prof_count >= g_pool_size) return;
  ProfRec& r = g_pool[g_prof_count];
  r.name = name;
  if (hipEventRecord(r.a, st) != hipSuccess) return;  // tracing aid: the launch itself is not affected
  ++g_prof_count;
  g_prof_open = true;
}
void prof_end(hipStream_t st) {
  if (!g_prof_on || !g_prof_open) return;
  (void)hipEventRecord(g_pool[g_prof_count - 1].b, st);
  g_prof_open = false;
}
}  // namespace rattn

namespace {

thread_local char g_err[512] = "";

rattn_status fail(rattn_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Sequence lengths from this size on run on the matrix-core kernels (bf16) whether or not they are a multiple of
// the 128-row tile: with D = 128 in place, only the last partial tile of every sequence goes through zero-padded
// buffers; with D = 64 through zero-padded copies of the whole tensors.  Shorter ones (less than one tile) stay on
// the general kernels.
constexpr int PAD_MIN_T = 128;

struct Layout {
  rattn::LayerDims dm;
  rattn::LayerDims dmf;  // what the matrix-core kernels see: dm with T rounded up to 128 when `pad`
  bool pad;
  bool pad_d;                                             // head size 64 widened to 128 (implies pad)
  bool tails;                                             // pad without pad_d: the pf_* / pb_* areas hold the last
                                                          // 128-row tile of every sequence only (RaggedTails)
  size_t pf_q, pf_k, pf_v, pf_o, pf_gs, pf_gr;            // padded copies, forward workspace (gains only if pad_d)
  size_t pb_q, pb_k, pb_v, pb_dO, pb_dq, pb_dk, pb_dv;    // padded copies, backward workspace
  size_t pb_gs, pb_gr, pb_dgs, pb_dgr;                    // padded gains and gain gradients (pad_d)
  size_t esize;
  // saved
  size_t sv_xs, sv_xr, sv_lse, sv_rs, sv_rr, sv_states, saved_bytes;
  int state_stride;   // chunk states kept in `saved`: 0 = none, 1 = all, m = every m-th
  // generic forward / backward workspace
  size_t gf_states, gen_fwd_bytes;
  size_t gb_states, gb_rstates, gb_dxs, gb_dxr, gb_delta, gb_dgpart, gen_bwd_bytes;
  int RB;
  // MFMA forward workspace
  bool fast_fwd;
  size_t ff_u, ff_states, fast_fwd_bytes;
  size_t fb_dxs, fb_dxr, fb_delta, fb_u, fb_states, fb_rstates, fb_dgpart, fast_bwd_bytes;
  size_t fwd_bytes, bwd_bytes;
};

rattn_status make_layout(const rattn_params* p, Layout* L) {
  if (!p) return fail(RATTN_ERR_INVALID_ARG, "params is NULL");
  if (p->B < 1 || p->T < 1 || p->Hq < 1 || p->Hkv < 1)
    return fail(RATTN_ERR_INVALID_ARG, "B, T, Hq, Hkv must be >= 1 (got %d, %d, %d, %d)", p->B, p->T, p->Hq, p->Hkv);
  if (p->Hq % p->Hkv != 0)
    return fail(RATTN_ERR_INVALID_ARG, "Hq (%d) must be a multiple of Hkv (%d)", p->Hq, p->Hkv);
  if (p->B > 65535 || p->Hq > 65535)
    return fail(RATTN_ERR_UNSUPPORTED, "B and Hq must be <= 65535 (got %d, %d)", p->B, p->Hq);
  if (p->D != 64 && p->D != 128) return fail(RATTN_ERR_UNSUPPORTED, "head_dim D must be 64 or 128 (got %d)", p->D);
  if (p->window < 1) return fail(RATTN_ERR_INVALID_ARG, "window must be >= 1 (got %d)", p->window);
  if (p->chunk < 0) return fail(RATTN_ERR_INVALID_ARG, "chunk must be >= 0 (got %d)", p->chunk);
  if (p->dtype != RATTN_F32 && p->dtype != RATTN_BF16) return fail(RATTN_ERR_UNSUPPORTED, "unknown dtype %d", p->dtype);
  if (p->feature_map < RATTN_PHI_SOFTMAX || p->feature_map > RATTN_PHI_IDENTITY)
    return fail(RATTN_ERR_UNSUPPORTED, "unknown feature_map %d", p->feature_map);
  if (p->kernel_path != RATTN_PATH_AUTO && p->kernel_path != RATTN_PATH_GENERAL)
    return fail(RATTN_ERR_UNSUPPORTED, "unknown kernel_path %d", p->kernel_path);
  if (p->state_policy != RATTN_STATES_KEEP && p->state_policy != RATTN_STATES_REBUILD &&
      p->state_policy != RATTN_STATES_KEEP_EVERY_2ND && p->state_policy != RATTN_STATES_KEEP_EVERY_4TH)
    return fail(RATTN_ERR_UNSUPPORTED, "unknown state_policy %d", p->state_policy);
  if (!(p->rms_eps > 0.f)) return fail(RATTN_ERR_INVALID_ARG, "rms_eps must be > 0");
  if (!(p->softmax_scale == p->softmax_scale) || p->softmax_scale == 0.f)
    return fail(RATTN_ERR_INVALID_ARG, "softmax_scale must be a non-zero number");
  if ((long long)p->B * p->T >= (1ll << 31) / 4 || (long long)p->B * p->T * p->Hq * p->D >= (1ll << 40))
    return fail(RATTN_ERR_UNSUPPORTED, "tensor too large for 32-bit row indexing");

  rattn::LayerDims& dm = L->dm;
  dm.B = p->B; dm.T = p->T; dm.Hq = p->Hq; dm.Hkv = p->Hkv; dm.D = p->D;
  dm.W = p->window; dm.G = p->Hq / p->Hkv;
  dm.C = p->chunk > 0 ? p->chunk : 64;
  dm.chunk_req = p->chunk;
  const int Tp = p->T > p->window ? p->T - p->window : 0;
  dm.nst = Tp > 0 ? (Tp - 1) / dm.C + 1 : 0;
  dm.scale = p->softmax_scale; dm.eps = p->rms_eps; dm.phi = p->feature_map;
  L->esize = p->dtype == RATTN_F32 ? 4 : 2;

  // What the matrix-core kernels would see: the sequence length rounded up to whole 128-row tiles (ragged lengths from
  // PAD_MIN_T on: tail buffers) and a head size of 64 widened to 128 (zero-padded copies in the workspace)
  dm.Dv = dm.D;
  L->dmf = dm;
  const bool ragged = dm.T % 128 != 0;
  L->pad_d = p->dtype == RATTN_BF16 && dm.D == 64 && (!ragged || dm.T >= PAD_MIN_T);
  L->pad = p->dtype == RATTN_BF16 && ((dm.D == 128 && ragged && dm.T >= PAD_MIN_T) || L->pad_d);
  if (L->pad) L->dmf.T = (dm.T + 127) / 128 * 128;
  if (L->pad_d) L->dmf.D = 128;
  const rattn::LayerDims& dmf = L->dmf;
  // Identity feature map: only calls that keep nothing for a backward pass (inference, prefill) run on the matrix
  // cores.  Its backward with bf16 operands is not accurate enough: on the first rows past the window the state has
  // rank 1, 2, ..., d x^r is orthogonal to the few value rows x^r is made of, and with features of size ~1 (not ~1/D
  // as after the softmax map) the 2^-9 that rounding leaves of that cancellation reaches single dq elements at
  // 0.1 .. 2 times the gradient's RMS (GPU and the CPU model of the roundings agree on every such case).
  const bool identity_training = dm.phi == rattn::PHI_IDENTITY && p->save_for_bwd;
  L->fast_fwd = p->kernel_path != RATTN_PATH_GENERAL && !identity_training && rattn::fast_fwd_supported(dmf, p->dtype);
  if (!L->fast_fwd) { L->pad = L->pad_d = false; L->dmf = dm; }
  L->tails = L->pad && !L->pad_d;
  // `saved` is sized for the padded length
  const size_t nq = (size_t)dm.B * dm.T * dm.Hq * dm.D;
  const size_t nrow = (size_t)dm.B * dm.Hq * dm.T;
  const size_t nq_f = (size_t)dmf.B * dmf.T * dmf.Hq * dmf.D, nkv_f = (size_t)dmf.B * dmf.T * dmf.Hkv * dmf.D;
  const size_t nrow_f = (size_t)dmf.B * dmf.Hq * dmf.T;
  size_t off = 0;
  // pre-norm branch outputs: tensor dtype for the matrix-core kernels, fp32 for the general kernels
  const size_t sv_esize = L->fast_fwd ? L->esize : 4;
  L->sv_xs = off; off += align_up(nq_f * sv_esize);
  L->sv_xr = off; off += align_up(nq_f * sv_esize);
  L->sv_lse = off; off += align_up(nrow_f * 4);
  L->sv_rs = off; off += align_up(nrow_f * 4);
  L->sv_rr = off; off += align_up(nrow_f * 4);
  L->sv_states = off;
  L->state_stride = !L->fast_fwd || p->state_policy == RATTN_STATES_REBUILD ? 0
                    : p->state_policy == RATTN_STATES_KEEP ? 1 : p->state_policy;
  if (L->state_stride > 0) {
    const int nstf = rattn::fast_fwd_plan(dmf).nstf;
    off += align_up((size_t)dmf.B * dmf.Hkv * ((nstf + L->state_stride - 1) / L->state_stride) * 128 * 128 * 2);
  }
  L->saved_bytes = off;

  const size_t nstate = (size_t)dm.B * dm.Hkv * dm.nst * dm.D * dm.D;
  L->gf_states = 0;
  L->gen_fwd_bytes = align_up(nstate * 4);

  const long long rows = (long long)dm.B * dm.T;
  L->RB = (int)(rows / 4 < 1 ? 1 : (rows / 4 > 256 ? 256 : rows / 4));
  off = 0;
  L->gb_states = off; off += align_up(nstate * 4);
  L->gb_rstates = off; off += align_up(nstate * 4);
  L->gb_dxs = off; off += align_up(nq * 4);
  L->gb_dxr = off; off += align_up(nq * 4);
  L->gb_delta = off; off += align_up(nrow * 4);
  L->gb_dgpart = off; off += align_up((size_t)2 * L->RB * dm.Hq * dm.D * 4);
  L->gen_bwd_bytes = off;

  L->ff_u = L->ff_states = L->fast_fwd_bytes = 0;
  if (L->fast_fwd) {
    const rattn::FastFwdPlan pl = rattn::fast_fwd_plan(dmf);
    off = 0;
    L->ff_u = off; off += align_up(pl.u_bytes);
    L->ff_states = off; off += align_up(pl.state_bytes);
    // padded copies of whole tensors, or of the last tile of every sequence
    const size_t cq = L->tails ? (size_t)dmf.B * 128 * dmf.Hq * 128 * 2 : nq_f * 2;
    const size_t ckv = L->tails ? (size_t)dmf.B * 128 * dmf.Hkv * 128 * 2 : nkv_f * 2;
    if (L->pad) {
      L->pf_q = off; off += align_up(cq);
      L->pf_k = off; off += align_up(ckv);
      L->pf_v = off; off += align_up(ckv);
      L->pf_o = off; off += align_up(cq);
      L->pf_gs = off; off += align_up((size_t)dmf.Hq * 128 * 4);
      L->pf_gr = off; off += align_up((size_t)dmf.Hq * 128 * 4);
    }
    L->fast_fwd_bytes = off;
  }
  L->fast_bwd_bytes = 0;
  if (L->fast_fwd) {
    const rattn::FastBwdPlan bp = rattn::fast_bwd_plan(dmf);
    off = 0;
    L->fb_dxs = off; off += align_up(nq_f * 2);
    L->fb_dxr = off; off += align_up(nq_f * 2);
    L->fb_delta = off; off += align_up(nrow_f * 8);  // delta, then log-sum-exp in log2 units
    L->fb_u = off; off += align_up(bp.u_bytes);
    L->fb_states = off; off += align_up(bp.fwd.state_bytes);
    L->fb_rstates = off; off += align_up(bp.rstate_bytes);
    L->fb_dgpart = off; off += align_up((size_t)2 * bp.RB * dmf.Hq * dmf.D * 4);
    const size_t cq = L->tails ? (size_t)dmf.B * 128 * dmf.Hq * 128 * 2 : nq_f * 2;
    const size_t ckv = L->tails ? (size_t)dmf.B * 128 * dmf.Hkv * 128 * 2 : nkv_f * 2;
    if (L->pad) {
      L->pb_q = off; off += align_up(cq);
      L->pb_k = off; off += align_up(ckv);
      L->pb_v = off; off += align_up(ckv);
      L->pb_dO = off; off += align_up(cq);
      L->pb_dq = off; off += align_up(cq);
      L->pb_dk = off; off += align_up(ckv);
      L->pb_dv = off; off += align_up(ckv);
      L->pb_gs = off; off += align_up((size_t)dmf.Hq * 128 * 4);
      L->pb_gr = off; off += align_up((size_t)dmf.Hq * 128 * 4);
      L->pb_dgs = off; off += align_up((size_t)dmf.Hq * 128 * 4);
      L->pb_dgr = off; off += align_up((size_t)dmf.Hq * 128 * 4);
    }
    L->fast_bwd_bytes = off;
  }
  L->fwd_bytes = L->fast_fwd ? L->fast_fwd_bytes : L->gen_fwd_bytes;
  L->bwd_bytes = L->fast_fwd ? L->fast_bwd_bytes : L->gen_bwd_bytes;
  return RATTN_OK;
}

rattn::SavedPtrs saved_views(const Layout& L, void* saved) {
  rattn::SavedPtrs sv = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, !L.fast_fwd, 0};
  if (saved) {
    char* s = (char*)saved;
    sv.xs = s + L.sv_xs; sv.xr = s + L.sv_xr;
    sv.lse = (float*)(s + L.sv_lse); sv.rs = (float*)(s + L.sv_rs); sv.rr = (float*)(s + L.sv_rr);
    if (L.state_stride > 0) { sv.states = s + L.sv_states; sv.state_stride = L.state_stride; }
  }
  return sv;
}

// chunked prefill: the forward runs over R ring rows + the chunk's T rows
struct ChunkLayout {
  rattn_params p2;
  Layout L2;
  int R;
  size_t kc, vc, qc, oc, saved, fwdws, partial, bytes;
};

rattn_status make_chunk_layout(const rattn_params* p, int32_t pos0, ChunkLayout* C) {
  Layout L;
  rattn_status s = make_layout(p, &L);
  if (s != RATTN_OK) return s;
  if (pos0 < 0) return fail(RATTN_ERR_INVALID_ARG, "pos0 must be >= 0 (got %d)", pos0);
  if ((long long)pos0 + p->T >= (1ll << 31)) return fail(RATTN_ERR_UNSUPPORTED, "pos0 + T must stay below 2^31");
  C->R = pos0 < p->window ? pos0 : p->window;
  C->p2 = *p;
  C->p2.T = C->R + p->T;
  C->p2.save_for_bwd = 1;
  // chunked prefill reads the forward's saved tensors in the caller's head size: a head size of 64, which the
  // matrix-core kernels would run on widened copies, stays on the general kernels here
  if (p->D == 64) C->p2.kernel_path = RATTN_PATH_GENERAL;
  s = make_layout(&C->p2, &C->L2);
  if (s != RATTN_OK) return s;
  const rattn::LayerDims& dm = C->L2.dm;
  const size_t nkv = (size_t)dm.B * dm.T * dm.Hkv * dm.D * C->L2.esize, nq = (size_t)dm.B * dm.T * dm.Hq * dm.D * C->L2.esize;
  size_t off = 0;
  C->kc = off; off += align_up(nkv);
  C->vc = off; off += align_up(nkv);
  C->qc = off; off += align_up(nq);
  C->oc = off; off += align_up(nq);
  C->saved = off; off += align_up(C->L2.saved_bytes);
  C->fwdws = off; off += align_up(C->L2.fwd_bytes);
  C->partial = off; off += align_up(rattn::export_plan(dm).partial_bytes);
  C->bytes = off;
  return RATTN_OK;
}

rattn_status check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(RATTN_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return RATTN_OK;
}

}  // namespace

extern "C" {

const char* rattn_status_string(rattn_status s) {
  switch (s) {
    case RATTN_OK: return "ok";
    case RATTN_ERR_INVALID_ARG: return "invalid argument";
    case RATTN_ERR_UNSUPPORTED: return "unsupported configuration";
    case RATTN_ERR_WORKSPACE: return "workspace too small";
    case RATTN_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* rattn_last_error(void) { return g_err; }

void rattn_profile_reset(void) {
  rattn::g_prof_count = 0;
  rattn::g_prof_open = false;
}
void rattn_profile_enable(int on) {
  rattn_profile_reset();
  if (on) {  // fill the event pool once; the layer calls only record into it
    while (rattn::g_pool_size < RATTN_PROFILE_MAX_RECORDS) {
      rattn::ProfRec& r = rattn::g_pool[rattn::g_pool_size];
      if (hipEventCreate(&r.a) != hipSuccess) break;
      if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); break; }
      ++rattn::g_pool_size;
    }
  }
  rattn::g_prof_on = on != 0;
}
int rattn_profile_count(void) { return rattn::g_prof_count; }
rattn_status rattn_profile_get(int idx, const char** name, float* ms) {
  if (idx < 0 || idx >= rattn::g_prof_count) return fail(RATTN_ERR_INVALID_ARG, "profile index %d out of range", idx);
  const auto& r = rattn::g_pool[idx];
  if (hipEventSynchronize(r.b) != hipSuccess) return fail(RATTN_ERR_HIP, "hipEventSynchronize failed");
  float t = 0.f;
  if (hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) return fail(RATTN_ERR_HIP, "hipEventElapsedTime failed");
  if (name) *name = r.name;
  if (ms) *ms = t;
  return RATTN_OK;
}
const char* rattn_version(void) { return "0.1"; }

rattn_status rattn_workspace_bytes(const rattn_params* p, size_t* fwd_bytes, size_t* bwd_bytes, size_t* saved_bytes) {
  if (!p) return fail(RATTN_ERR_INVALID_ARG, "params is NULL");
  // sizes do not depend on save_for_bwd: `saved` and the backward scratch are those of a call that saves, the
  // forward scratch covers both kinds of call (they differ only where the kernel family depends on it)
  rattn_params q = *p;
  Layout L;
  q.save_for_bwd = 1;
  rattn_status s = make_layout(&q, &L);
  if (s != RATTN_OK) return s;
  size_t fwd = L.fwd_bytes;
  Layout L0;
  q.save_for_bwd = 0;
  s = make_layout(&q, &L0);
  if (s != RATTN_OK) return s;
  if (L0.fwd_bytes > fwd) fwd = L0.fwd_bytes;
  if (fwd_bytes) *fwd_bytes = fwd;
  if (bwd_bytes) *bwd_bytes = L.bwd_bytes;
  if (saved_bytes) *saved_bytes = L.saved_bytes;
  return RATTN_OK;
}

rattn_status rattn_fwd(const rattn_params* p, const void* q, const void* k, const void* v, const float* gamma_swa,
                       const float* gamma_rla, void* o, void* saved, void* workspace, size_t workspace_bytes,
                       void* stream) {
  Layout L;
  rattn_status s = make_layout(p, &L);
  if (s != RATTN_OK) return s;
  if (!q || !k || !v || !o) return fail(RATTN_ERR_INVALID_ARG, "q, k, v, o must be non-NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(saved) || !aligned16(workspace))
    return fail(RATTN_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  if (p->save_for_bwd && !saved) return fail(RATTN_ERR_INVALID_ARG, "save_for_bwd set but saved is NULL");
  if (L.fwd_bytes > 0 && (!workspace || workspace_bytes < L.fwd_bytes))
    return fail(RATTN_ERR_WORKSPACE, "forward needs %zu workspace bytes, got %zu", L.fwd_bytes, workspace_bytes);
  hipStream_t st = (hipStream_t)stream;
  rattn::SavedPtrs sv = saved_views(L, p->save_for_bwd ? saved : nullptr);
  if (L.fast_fwd) {
    char* w = (char*)workspace;
    const void *qf = q, *kf = k, *vf = v;
    void* of = o;
    const float *gsf = gamma_swa, *grf = gamma_rla;
    const size_t hb = (size_t)L.dm.D * 2, hbp = (size_t)L.dmf.D * 2;  // bytes of one head row, caller's and padded
    if (L.tails) {
      const void* src[3] = {q, k, v};
      void* tl[3] = {w + L.pf_q, w + L.pf_k, w + L.pf_v};
      const int Hs[3] = {L.dm.Hq, L.dm.Hkv, L.dm.Hkv};
      rattn::gather_tails(3, src, tl, Hs, L.dm.B, L.dm.T, st);
      rattn::RaggedTails rt = {L.dm.T, tl[0], tl[1], tl[2], nullptr, w + L.pf_o, nullptr, nullptr, nullptr};
      rattn::fast_fwd(L.dmf, q, k, v, gamma_swa, gamma_rla, o, sv, (float*)(w + L.ff_u),
                      sv.states && sv.state_stride <= 1 ? sv.states : (void*)(w + L.ff_states), st, 0, nullptr, &rt);
      const void* otl[1] = {w + L.pf_o};
      void* odst[1] = {o};
      rattn::scatter_tails(1, otl, odst, Hs, L.dm.B, L.dm.T, st);
      return check_launch("rattn_fwd");
    }
    if (L.pad) {
      rattn::pad_rows(q, w + L.pf_q, L.dm.B, L.dm.T, L.dmf.T, L.dm.Hq, hb, hbp, st);
      rattn::pad_rows(k, w + L.pf_k, L.dm.B, L.dm.T, L.dmf.T, L.dm.Hkv, hb, hbp, st);
      rattn::pad_rows(v, w + L.pf_v, L.dm.B, L.dm.T, L.dmf.T, L.dm.Hkv, hb, hbp, st);
      qf = w + L.pf_q; kf = w + L.pf_k; vf = w + L.pf_v; of = w + L.pf_o;
      if (L.pad_d) {  // gains are [Hq, 64] fp32: widened to [Hq, 128] (the padding features of x are zero)
        if (gamma_swa) { rattn::pad_rows(gamma_swa, w + L.pf_gs, 1, L.dm.Hq, L.dm.Hq, 1, 256, 512, st); gsf = (const float*)(w + L.pf_gs); }
        if (gamma_rla) { rattn::pad_rows(gamma_rla, w + L.pf_gr, 1, L.dm.Hq, L.dm.Hq, 1, 256, 512, st); grf = (const float*)(w + L.pf_gr); }
      }
    }
    rattn::fast_fwd(L.dmf, qf, kf, vf, gsf, grf, of, sv, (float*)(w + L.ff_u),
                    sv.states && sv.state_stride <= 1 ? sv.states : (void*)(w + L.ff_states), st);
    if (L.pad) rattn::unpad_rows(of, o, L.dm.B, L.dm.T, L.dmf.T, L.dm.Hq, hb, hbp, st);
  } else
    rattn::generic_fwd(L.dm, p->dtype, q, k, v, gamma_swa, gamma_rla, o, sv, (float*)((char*)workspace + L.gf_states), st);
  return check_launch("rattn_fwd");
}

// ---- rattn_fwd_static: the forward with its scratch memory inside the library's device image
// BEGIN-STATIC-ENTRY
namespace {
// One copy per GPU that loads this library, alive until the process ends.  In host code the array's name is only
// a handle for hipGetSymbolAddress; the kernels get the looked-up device address like any other workspace.
static __device__ __align__(256) unsigned char scratch[RATTN_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};  // device address of `scratch`, per device, looked up once
}  // namespace

rattn_status rattn_fwd_static(const rattn_params* p, const void* q, const void* k, const void* v,
                              const float* gamma_swa, const float* gamma_rla, void* o, void* saved, void* stream) {
  Layout L;
  rattn_status s = make_layout(p, &L);
  if (s != RATTN_OK) return s;
  if (L.fwd_bytes > RATTN_STATIC_SCRATCH_BYTES)
    return fail(RATTN_ERR_WORKSPACE, "rattn_fwd_static: this shape needs %zu bytes of forward scratch, the built-in buffer "
                "holds %zu; use rattn_fwd with a caller-provided workspace", L.fwd_bytes, (size_t)RATTN_STATIC_SCRATCH_BYTES);
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
    return fail(RATTN_ERR_HIP, "rattn_fwd_static: no current HIP device (or device index >= %d)", MAX_DEVICES);
  void* ws = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!ws) {  // first call on this device (every thread that gets here looks up the same address)
    const hipError_t e = hipGetSymbolAddress(&ws, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ws)
      return fail(RATTN_ERR_HIP, "rattn_fwd_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
    __atomic_store_n(&g_scratch_ptr[dev], ws, __ATOMIC_RELEASE);
  }
  // Every part of the scratch that the forward kernels read is written earlier in the same call (chunk products,
  // then the scanned states, and - for ragged lengths or a head size of 64 - the zero-padded copies), so nothing has
  // to be cleared.
  return rattn_fwd(p, q, k, v, gamma_swa, gamma_rla, o, saved, ws, RATTN_STATIC_SCRATCH_BYTES, stream);
}
// END-STATIC-ENTRY

rattn_status rattn_bwd(const rattn_params* p, const void* q, const void* k, const void* v, const float* gamma_swa,
                       const float* gamma_rla, const void* saved, const void* dO, void* dq, void* dk, void* dv,
                       float* dgamma_swa, float* dgamma_rla, void* workspace, size_t workspace_bytes, void* stream) {
  if (!p) return fail(RATTN_ERR_INVALID_ARG, "params is NULL");
  rattn_params pb = *p;
  pb.save_for_bwd = 1;   // `saved` comes from a forward call that saved, whatever this copy of the parameters says
  p = &pb;
  Layout L;
  rattn_status s = make_layout(p, &L);
  if (s != RATTN_OK) return s;
  if (!q || !k || !v || !saved || !dO || !dq || !dk || !dv)
    return fail(RATTN_ERR_INVALID_ARG, "q, k, v, saved, dO, dq, dk, dv must be non-NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(saved) || !aligned16(dO) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv) || !aligned16(workspace))
    return fail(RATTN_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  if (!workspace || workspace_bytes < L.bwd_bytes)
    return fail(RATTN_ERR_WORKSPACE, "backward needs %zu workspace bytes, got %zu", L.bwd_bytes, workspace_bytes);
  hipStream_t st = (hipStream_t)stream;
  rattn::SavedPtrs sv = saved_views(L, const_cast<void*>(saved));
  char* w = (char*)workspace;
  if (L.fast_fwd) {
    rattn::FastBwdWs fw;
    fw.dxs = w + L.fb_dxs; fw.dxr = w + L.fb_dxr; fw.delta = (float*)(w + L.fb_delta); fw.U = (float*)(w + L.fb_u);
    fw.states = w + L.fb_states; fw.rstates = w + L.fb_rstates; fw.dgpart = (float*)(w + L.fb_dgpart);
    const size_t hb = (size_t)L.dm.D * 2, hbp = (size_t)L.dmf.D * 2;  // bytes of one head row, caller's and padded
    if (L.tails) {
      const void* src[4] = {q, k, v, dO};
      void* tl[4] = {w + L.pb_q, w + L.pb_k, w + L.pb_v, w + L.pb_dO};
      const int Hs[4] = {L.dm.Hq, L.dm.Hkv, L.dm.Hkv, L.dm.Hq};
      rattn::gather_tails(4, src, tl, Hs, L.dm.B, L.dm.T, st);
      rattn::RaggedTails rt = {L.dm.T, tl[0], tl[1], tl[2], tl[3], nullptr, w + L.pb_dq, w + L.pb_dk, w + L.pb_dv};
      rattn::fast_bwd(L.dmf, q, k, v, gamma_swa, gamma_rla, sv, dO, dq, dk, dv, dgamma_swa, dgamma_rla, fw, st, &rt);
      const void* gtl[3] = {w + L.pb_dq, w + L.pb_dk, w + L.pb_dv};
      void* gdst[3] = {dq, dk, dv};
      rattn::scatter_tails(3, gtl, gdst, Hs, L.dm.B, L.dm.T, st);
    } else if (L.pad) {
      const int B = L.dm.B, T = L.dm.T, Tp = L.dmf.T, Hq = L.dm.Hq, Hkv = L.dm.Hkv;
      rattn::pad_rows(q, w + L.pb_q, B, T, Tp, Hq, hb, hbp, st);
      rattn::pad_rows(k, w + L.pb_k, B, T, Tp, Hkv, hb, hbp, st);
      rattn::pad_rows(v, w + L.pb_v, B, T, Tp, Hkv, hb, hbp, st);
      rattn::pad_rows(dO, w + L.pb_dO, B, T, Tp, Hq, hb, hbp, st);
      const float *gsf = gamma_swa, *grf = gamma_rla;
      float *dgs = dgamma_swa, *dgr = dgamma_rla;
      if (L.pad_d) {  // gains and gain gradients are [Hq, 64] fp32 for the caller, [Hq, 128] for the kernels
        if (gamma_swa) { rattn::pad_rows(gamma_swa, w + L.pb_gs, 1, Hq, Hq, 1, 256, 512, st); gsf = (const float*)(w + L.pb_gs); }
        if (gamma_rla) { rattn::pad_rows(gamma_rla, w + L.pb_gr, 1, Hq, Hq, 1, 256, 512, st); grf = (const float*)(w + L.pb_gr); }
        if (dgamma_swa) dgs = (float*)(w + L.pb_dgs);
        if (dgamma_rla) dgr = (float*)(w + L.pb_dgr);
      }
      rattn::fast_bwd(L.dmf, w + L.pb_q, w + L.pb_k, w + L.pb_v, gsf, grf, sv, w + L.pb_dO, w + L.pb_dq,
                      w + L.pb_dk, w + L.pb_dv, dgs, dgr, fw, st);
      rattn::unpad_rows(w + L.pb_dq, dq, B, T, Tp, Hq, hb, hbp, st);
      rattn::unpad_rows(w + L.pb_dk, dk, B, T, Tp, Hkv, hb, hbp, st);
      rattn::unpad_rows(w + L.pb_dv, dv, B, T, Tp, Hkv, hb, hbp, st);
      if (L.pad_d && dgamma_swa) rattn::unpad_rows(dgs, dgamma_swa, 1, Hq, Hq, 1, 256, 512, st);
      if (L.pad_d && dgamma_rla) rattn::unpad_rows(dgr, dgamma_rla, 1, Hq, Hq, 1, 256, 512, st);
    } else {
      rattn::fast_bwd(L.dm, q, k, v, gamma_swa, gamma_rla, sv, dO, dq, dk, dv, dgamma_swa, dgamma_rla, fw, st);
    }
    return check_launch("rattn_bwd");
  }
  rattn::GenericBwdWs ws;
  ws.states = (float*)(w + L.gb_states); ws.rstates = (float*)(w + L.gb_rstates);
  ws.dxs = (float*)(w + L.gb_dxs); ws.dxr = (float*)(w + L.gb_dxr);
  ws.delta = (float*)(w + L.gb_delta); ws.dgpart = (float*)(w + L.gb_dgpart);
  ws.RB = L.RB;
  rattn::generic_bwd(L.dm, p->dtype, q, k, v, gamma_swa, gamma_rla, sv, dO, dq, dk, dv, dgamma_swa, dgamma_rla, ws, st);
  return check_launch("rattn_bwd");
}

rattn_status rattn_decode_step(const rattn_decode_params* p, const void* q, const void* k_new, const void* v_new,
                               const int32_t* pos, void* k_ring, void* v_ring, float* state, const float* gamma_swa,
                               const float* gamma_rla, void* o, void* stream) {
  if (!p) return fail(RATTN_ERR_INVALID_ARG, "params is NULL");
  if (p->N < 1 || p->Hq < 1 || p->Hkv < 1)
    return fail(RATTN_ERR_INVALID_ARG, "N, Hq, Hkv must be >= 1 (got %d, %d, %d)", p->N, p->Hq, p->Hkv);
  if (p->Hq % p->Hkv != 0)
    return fail(RATTN_ERR_INVALID_ARG, "Hq (%d) must be a multiple of Hkv (%d)", p->Hq, p->Hkv);
  if (p->D != 64 && p->D != 128) return fail(RATTN_ERR_UNSUPPORTED, "head_dim D must be 64 or 128 (got %d)", p->D);
  if (p->window < 1) return fail(RATTN_ERR_INVALID_ARG, "window must be >= 1 (got %d)", p->window);
  if (p->dtype != RATTN_F32 && p->dtype != RATTN_BF16) return fail(RATTN_ERR_UNSUPPORTED, "unknown dtype %d", p->dtype);
  if (p->feature_map < RATTN_PHI_SOFTMAX || p->feature_map > RATTN_PHI_IDENTITY)
    return fail(RATTN_ERR_UNSUPPORTED, "unknown feature_map %d", p->feature_map);
  if (!(p->rms_eps > 0.f)) return fail(RATTN_ERR_INVALID_ARG, "rms_eps must be > 0");
  if (!(p->softmax_scale == p->softmax_scale) || p->softmax_scale == 0.f)
    return fail(RATTN_ERR_INVALID_ARG, "softmax_scale must be a non-zero number");
  if (p->N > 65535) return fail(RATTN_ERR_UNSUPPORTED, "N must be <= 65535 (got %d)", p->N);
  if ((long long)p->N * p->Hkv * p->window * p->D >= (1ll << 40))
    return fail(RATTN_ERR_UNSUPPORTED, "ring buffers too large");
  if (!q || !k_new || !v_new || !pos || !k_ring || !v_ring || !state || !o)
    return fail(RATTN_ERR_INVALID_ARG, "q, k_new, v_new, pos, k_ring, v_ring, state, o must be non-NULL");
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(k_ring) || !aligned16(v_ring) ||
      !aligned16(state) || !aligned16(o))
    return fail(RATTN_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  rattn::DecodeDims dd;
  dd.N = p->N; dd.Hq = p->Hq; dd.Hkv = p->Hkv; dd.D = p->D; dd.W = p->window; dd.G = p->Hq / p->Hkv;
  dd.scale = p->softmax_scale; dd.eps = p->rms_eps; dd.phi = p->feature_map;
  rattn::decode_step(dd, p->dtype, q, k_new, v_new, pos, k_ring, v_ring, state, gamma_swa, gamma_rla, o,
                     (hipStream_t)stream);
  return check_launch("rattn_decode_step");
}

rattn_status rattn_prefill_export_workspace_bytes(const rattn_params* p, size_t* bytes) {
  Layout L;
  rattn_status s = make_layout(p, &L);
  if (s != RATTN_OK) return s;
  if (bytes) *bytes = align_up(rattn::export_plan(L.dm).partial_bytes);
  return RATTN_OK;
}

rattn_status rattn_prefill_export(const rattn_params* p, const void* k, const void* v, void* k_ring, void* v_ring,
                                  float* state, void* workspace, size_t workspace_bytes, void* stream) {
  Layout L;
  rattn_status s = make_layout(p, &L);
  if (s != RATTN_OK) return s;
  if (!k || !v || !k_ring || !v_ring || !state) return fail(RATTN_ERR_INVALID_ARG, "k, v, k_ring, v_ring, state must be non-NULL");
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_ring) || !aligned16(v_ring) || !aligned16(state) ||
      !aligned16(workspace))
    return fail(RATTN_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  const size_t need = align_up(rattn::export_plan(L.dm).partial_bytes);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(RATTN_ERR_WORKSPACE, "prefill export needs %zu workspace bytes, got %zu", need, workspace_bytes);
  rattn::prefill_export(L.dm, p->dtype, k, v, k_ring, v_ring, state, (float*)workspace, (hipStream_t)stream);
  return check_launch("rattn_prefill_export");
}

rattn_status rattn_prefill_chunk_workspace_bytes(const rattn_params* p, int32_t pos0, size_t* bytes) {
  ChunkLayout C;
  rattn_status s = make_chunk_layout(p, pos0, &C);
  if (s != RATTN_OK) return s;
  if (bytes) *bytes = C.bytes;
  return RATTN_OK;
}

rattn_status rattn_prefill_chunk(const rattn_params* p, int32_t pos0, const void* q, const void* k, const void* v,
                                 const float* gamma_swa, const float* gamma_rla, void* k_ring, void* v_ring,
                                 float* state, void* o, void* workspace, size_t workspace_bytes, void* stream) {
  ChunkLayout C;
  rattn_status s = make_chunk_layout(p, pos0, &C);
  if (s != RATTN_OK) return s;
  if (!q || !k || !v || !o || !k_ring || !v_ring || !state)
    return fail(RATTN_ERR_INVALID_ARG, "q, k, v, o, k_ring, v_ring, state must be non-NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(k_ring) || !aligned16(v_ring) ||
      !aligned16(state) || !aligned16(workspace))
    return fail(RATTN_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  if (!workspace || workspace_bytes < C.bytes)
    return fail(RATTN_ERR_WORKSPACE, "chunked prefill needs %zu workspace bytes, got %zu", C.bytes, workspace_bytes);
  hipStream_t st = (hipStream_t)stream;
  char* w = (char*)workspace;
  const rattn::LayerDims& dm = C.L2.dm;
  // keys before the ring exist only once more than `window` tokens have been seen; until then the state is zero
  // by definition and what the caller's buffer holds is not read
  const bool carried = pos0 > p->window;
  // Direct route on the matrix-core kernels: ring and chunk are whole 128-row tiles, so the forward computes the
  // chunk's query tiles only, straight from q into o, and (window a multiple of 128: every such tile reads a chunk
  // state) the carried state enters as the initial value of the state scan.  Only K and V are gathered.
  if (C.L2.fast_fwd && !C.L2.pad && C.R % 128 == 0 && (!carried || p->window % 128 == 0)) {
    rattn::chunk_concat(dm, p->dtype, p->T, C.R, pos0, nullptr, k, v, k_ring, v_ring, nullptr, w + C.kc, w + C.vc, st);
    rattn::SavedPtrs none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, false, 0};
    rattn::fast_fwd(dm, q, w + C.kc, w + C.vc, gamma_swa, gamma_rla, o, none, (float*)(w + C.fwdws + C.L2.ff_u),
                    w + C.fwdws + C.L2.ff_states, st, C.R / 128, carried ? state : nullptr);
    rattn::prefill_export(dm, p->dtype, w + C.kc, w + C.vc, k_ring, v_ring, state, (float*)(w + C.partial), st,
                          pos0 - C.R, carried);
    return check_launch("rattn_prefill_chunk");
  }
  rattn::chunk_concat(dm, p->dtype, p->T, C.R, pos0, q, k, v, k_ring, v_ring, w + C.qc, w + C.kc, w + C.vc, st);
  s = check_launch("rattn_prefill_chunk (gather)");
  if (s != RATTN_OK) return s;
  s = rattn_fwd(&C.p2, w + C.qc, w + C.kc, w + C.vc, gamma_swa, gamma_rla, w + C.oc, w + C.saved, w + C.fwdws,
                C.L2.fwd_bytes, stream);
  if (s != RATTN_OK) return s;
  if (carried)
    rattn::chunk_fixup(dm, p->dtype, p->T, C.R, C.L2.fast_fwd ? C.L2.dmf.T : dm.T, w + C.qc,
                       saved_views(C.L2, w + C.saved), state, gamma_swa, gamma_rla, o, st);
  else
    rattn::chunk_copy_out(dm, p->dtype, p->T, C.R, w + C.oc, o, st);
  rattn::prefill_export(dm, p->dtype, w + C.kc, w + C.vc, k_ring, v_ring, state, (float*)(w + C.partial), st,
                        pos0 - C.R, carried);
  return check_launch("rattn_prefill_chunk");
}

rattn_status rattn_cache_bytes(int32_t layers, int32_t global_every, int64_t ctx, int64_t window, int32_t with_state,
                               int32_t Hkv, int32_t D, int32_t elem_bytes, double* out) {
  if (!out) return fail(RATTN_ERR_INVALID_ARG, "out is NULL");
  if (layers < 0 || global_every < 0 || ctx < 0 || window < 0 || Hkv < 1 || D < 1 || elem_bytes < 1)
    return fail(RATTN_ERR_INVALID_ARG, "sizes must be non-negative (Hkv, D, elem_bytes positive)");
  const int n_glob = global_every > 0 ? layers / global_every : 0;
  const int n_loc = layers - n_glob;
  const double tok = 2.0 * Hkv * D * elem_bytes;
  const double loc_tokens = (double)(ctx < window ? ctx : window);
  const double st = with_state ? (double)Hkv * D * D * 4.0 : 0.0;
  *out = n_glob * (double)ctx * tok + n_loc * (loc_tokens * tok + st);
  return RATTN_OK;
}

rattn_status rattn_step_time_model(double batch, double cache_bytes, double param_count, double param_bytes,
                                   double bandwidth, double flops, double* out) {
  if (!out) return fail(RATTN_ERR_INVALID_ARG, "out is NULL");
  if (!(batch >= 0.0) || !(cache_bytes >= 0.0) || !(param_count >= 0.0) || !(param_bytes >= 0.0))
    return fail(RATTN_ERR_INVALID_ARG, "batch, cache_bytes, param_count, param_bytes must be >= 0");
  if (!(bandwidth > 0.0) || !(flops > 0.0)) return fail(RATTN_ERR_INVALID_ARG, "bandwidth and flops must be > 0");
  const double compute = 2.0 * batch * param_count / flops, weights = param_bytes / bandwidth;
  *out = batch * cache_bytes / bandwidth + (compute > weights ? compute : weights);
  return RATTN_OK;
}

rattn_status rattn_probe_mfma(void* sink, int iters, int blocks, double* flops, void* stream) {
  if (!sink || !aligned16(sink)) return fail(RATTN_ERR_INVALID_ARG, "sink must be a 16-byte aligned device pointer");
  if (iters < 1 || iters > (1 << 24) || blocks < 1 || blocks > (1 << 20))
    return fail(RATTN_ERR_INVALID_ARG, "iters must be in [1, 2^24] and blocks in [1, 2^20] (got %d, %d)", iters, blocks);
  const double f = rattn::probe_mfma((float*)sink, iters, blocks, (hipStream_t)stream);
  if (flops) *flops = f;
  return check_launch("rattn_probe_mfma");
}

}  // extern "C"
