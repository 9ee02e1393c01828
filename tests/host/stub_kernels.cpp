// Stand-ins for the kernel translation units, so that the host layer of the library (argument validation, workspace
// layout, path selection: csrc/api.hip) can be built for the CPU alone and run under AddressSanitizer and
// UndefinedBehaviorSanitizer.  The shape planning is the library's own (csrc/plan.hip is part of that build); every
// launcher here records that it was called and touches no memory.
#include "kernels.hpp"

namespace rattn {

int g_stub_launches = 0;

void generic_fwd(const LayerDims&, int, const void*, const void*, const void*, const float*, const float*, void*,
                 const SavedPtrs&, float*, hipStream_t) { ++g_stub_launches; }
void generic_bwd(const LayerDims&, int, const void*, const void*, const void*, const float*, const float*,
                 const SavedPtrs&, const void*, void*, void*, void*, float*, float*, const GenericBwdWs&, hipStream_t) {
  ++g_stub_launches;
}
void fast_fwd(const LayerDims&, const void*, const void*, const void*, const float*, const float*, void*,
              const SavedPtrs&, float*, void*, hipStream_t, int, const float*, const RaggedTails*) { ++g_stub_launches; }
void rla_forward_states(const LayerDims&, const FastFwdPlan&, const void*, const void*, float*, void*, hipStream_t,
                        const float*, const RaggedTails*, void*, const void*, int) { ++g_stub_launches; }
void rla_reverse_states(const LayerDims&, const FastBwdPlan&, const void*, const void*, float*, void*, hipStream_t,
                        const RaggedTails*) { ++g_stub_launches; }
void fast_bwd(const LayerDims&, const void*, const void*, const void*, const float*, const float*, const SavedPtrs&,
              const void*, void*, void*, void*, float*, float*, const FastBwdWs&, hipStream_t, const RaggedTails*) {
  ++g_stub_launches;
}
void prefill_export(const LayerDims&, int, const void*, const void*, void*, void*, float*, float*, hipStream_t, int,
                    bool) { ++g_stub_launches; }
void chunk_concat(const LayerDims&, int, int, int, int, const void*, const void*, const void*, const void*, const void*,
                  void*, void*, void*, hipStream_t) { ++g_stub_launches; }
void chunk_copy_out(const LayerDims&, int, int, int, const void*, void*, hipStream_t) { ++g_stub_launches; }
void chunk_fixup(const LayerDims&, int, int, int, int, const void*, const SavedPtrs&, const float*, const float*,
                 const float*, void*, hipStream_t) { ++g_stub_launches; }
void pad_rows(const void*, void*, int, int, int, int, size_t, size_t, hipStream_t) { ++g_stub_launches; }
void unpad_rows(const void*, void*, int, int, int, int, size_t, size_t, hipStream_t) { ++g_stub_launches; }
void gather_tails(int, const void* const*, void* const*, const int*, int, int, hipStream_t) { ++g_stub_launches; }
void scatter_tails(int, const void* const*, void* const*, const int*, int, int, hipStream_t) { ++g_stub_launches; }
double probe_mfma(float*, int iters, int blocks, hipStream_t) { ++g_stub_launches; return 16.0 * iters * blocks * 4 * 32768.0; }
void decode_step(const DecodeDims&, int, const void*, const void*, const void*, const int32_t*, void*, void*, float*,
                 const float*, const float*, void*, hipStream_t) { ++g_stub_launches; }

}  // namespace rattn
