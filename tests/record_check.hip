// Host-side access to the record format and the fixed-point product of the sorted backward pass
// (csrc/bwd_record.hpp), so that tests can check their rounding without a GPU.
#include <stdint.h>

#include "bwd_record.hpp"

namespace {
template <typename IT, int F>
void roundtrip(uint32_t n, const uint32_t* la, const uint32_t* k, const float* wf0, const float* wrow,
               const float* g, int dense, int smooth, uint32_t cmask, uint32_t xmask, double scale, uint32_t* words,
               uint32_t* out_la, uint32_t* out_lb, float* out_wlo, float* out_wup, double* out_G) {
  using Rec = hg::Record<IT, F>;
  for (uint32_t i = 0; i < n; ++i) {
    IT gi[F];
    for (int f = 0; f < F; ++f) gi[f] = (IT)g[(uint64_t)i * F + f];
    const typename Rec::Stored r = Rec::make(la[i], k[i], wf0[i], wrow[i], gi, smooth != 0);
    *words = Rec::kWords;
    double G[F];
    bool first;
    Rec::unpack_scaled(r, dense != 0, cmask, xmask, scale, out_la[i], out_lb[i], out_wlo[i], out_wup[i], first, G);
    if (first != (k[i] == 15u)) out_la[i] = 0xffffffffu;  // would show in the caller's comparison
    for (int f = 0; f < F; ++f) out_G[(uint64_t)i * F + f] = G[f];
  }
}
}  // namespace

// n records made from (la, k, wf0, wrow, g[F]) and read back as the accumulate pass reads them
// (k = 15: the pair lies in the first voxel along dimension 0; out_wlo / out_wup: the pair's two weights,
// final ones in the first-voxel form when smooth != 0, else before any smoothstep).
// half != 0: dL/dy is fp16 (g is rounded to it first).  Returns 0, or 1 for an F that does not exist.
extern "C" int record_roundtrip(uint32_t n, uint32_t F, int half, const uint32_t* la, const uint32_t* k,
                                const float* wf0, const float* wrow, const float* g, int dense, int smooth, uint32_t cmask,
                                uint32_t xmask, double scale, uint32_t* words, uint32_t* out_la, uint32_t* out_lb,
                                float* out_wlo, float* out_wup, double* out_G) {
#define HG_RT(IT, FF) \
  roundtrip<IT, FF>(n, la, k, wf0, wrow, g, dense, smooth, cmask, xmask, scale, words, out_la, out_lb, out_wlo, out_wup, out_G)
  switch (F) {
    case 1: half ? HG_RT(_Float16, 1) : HG_RT(float, 1); return 0;
    case 2: half ? HG_RT(_Float16, 2) : HG_RT(float, 2); return 0;
    case 4: half ? HG_RT(_Float16, 4) : HG_RT(float, 4); return 0;
    case 8: half ? HG_RT(_Float16, 8) : HG_RT(float, 8); return 0;
    default: return 1;
  }
#undef HG_RT
}

extern "C" void fixed_products(uint32_t n, const float* w, const double* G, long long* out) {
  for (uint32_t i = 0; i < n; ++i) out[i] = (long long)hg::fixed_product(w[i], G[i]);
}
