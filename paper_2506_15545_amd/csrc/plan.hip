// Shape planning shared by the C ABI and the kernel launchers: which shapes the matrix-core kernels take, how many
// chunk states a call needs and how large its scratch areas are.  Host arithmetic only (nothing here touches a
// device), so this file is also part of the CPU build of the host layer that runs under the sanitizers.
#include "kernels.hpp"

namespace rattn {

// dm: the dimensions the kernels would see, i.e. after any zero-padding of the sequence length to whole tiles and of
// a head size of 64 to 128 (dm.D = 128, dm.Dv = 64)
bool fast_fwd_supported(const LayerDims& dm, int dtype) {
  if (dtype != 1 || dm.D != 128 || dm.T % 128 != 0) return false;
  if (!(dm.scale > 0.f)) return false;
  // Windows below 8 keys stay on the general path: their softmax rows are close to one-hot, so the backward's
  // dS = P (dP - delta) is a near-cancellation (exact for W = 1) that bf16 operands turn into rounding noise
  // above the gradient tolerance (measured: worst element 4 % of RMS at W = 2, 3 % at W = 4, 2.5 % from W = 8 on)
  if (dm.W < 8) return false;
  return true;
}

FastFwdPlan fast_fwd_plan(const LayerDims& dm) {
  FastFwdPlan p;
  const int wt = dm.W >= dm.T ? dm.T : dm.W;
  p.W = (wt + 63) / 64 * 64;
  p.gap = p.W - wt;
  p.base = p.W % 128;
  p.nstf = dm.T / 128 - (p.W + 127) / 128;
  if (p.nstf < 0) p.nstf = 0;
  // chunk-local products of `ckeys` keys each (128 unless the caller asks for `chunk` = 64); with 128 and states at the 64
  // alignment the first product covers the 64 keys in front of state 0
  p.ckeys = dm.chunk_req == 64 ? 64 : 128;
  p.nchunks = p.nstf > 0 ? (p.nstf - 1) * (128 / p.ckeys) + (p.base > 0 ? 1 : 0) : 0;
  p.u_bytes = (size_t)dm.B * dm.Hkv * p.nchunks * 16384 * 4;
  p.state_bytes = (size_t)dm.B * dm.Hkv * p.nstf * 16384 * 2;
  return p;
}

FastBwdPlan fast_bwd_plan(const LayerDims& dm) {
  FastBwdPlan p;
  p.fwd = fast_fwd_plan(dm);
  const int Tp = dm.T - p.fwd.W;
  p.nk = Tp > 0 ? (Tp + 127) / 128 : 0;
  // reverse-time chunk products: query rows t' in [128, Tp) in pieces of ckeys
  p.nrchunks = Tp > 128 ? (Tp - 128 + p.fwd.ckeys - 1) / p.fwd.ckeys : 0;
  const int nch = p.fwd.nchunks > p.nrchunks ? p.fwd.nchunks : p.nrchunks;
  p.u_bytes = (size_t)dm.B * dm.Hkv * (nch > 0 ? nch : 0) * 16384 * 4;
  p.rstate_bytes = (size_t)dm.B * dm.Hkv * p.nk * 16384 * 2;
  p.RB = 4 * (dm.T / 128) * dm.B;  // one gain-gradient partial per wave of the dq kernel
  return p;
}

ExportPlan export_plan(const LayerDims& dm) {
  ExportPlan pl;
  pl.Tp = dm.T > dm.W ? dm.T - dm.W : 0;
  const int kb = 256 / (dm.D / 8);
  int nseg = (pl.Tp + 4 * kb - 1) / (4 * kb);  // at least four key batches per segment
  if (nseg > 64) nseg = 64;
  pl.nseg = nseg;
  pl.seg_len = nseg > 0 ? ((pl.Tp + nseg - 1) / nseg + kb - 1) / kb * kb : 0;
  pl.partial_bytes = (size_t)dm.B * dm.Hkv * nseg * dm.D * dm.D * sizeof(float);
  return pl;
}

}  // namespace rattn
