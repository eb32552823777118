// Counter-based random numbers for dropout: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw,
// "Parallel random numbers: as easy as 1, 2, 3", SC'11).  A mask element is a pure function of
// (seed, site, position), so the forward kernel and every backward kernel regenerate the same
// decision in whatever order and lane layout suits them, and nothing is stored.
//
// Conventions (the paper's Transformer workloads train with dropout -- the primitive appears in the
// Sequential listing of Section 4.2 -- but the paper fixes no generator):
//   key = (seed mod 2^32, seed div 2^32); one call with counter (c0, c1, c2, c3) yields four words;
//   the element with column index n uses word n mod 4 of the call with c0 = n div 4;
//   kept iff word >= thr, thr = min(2^32 - 1, floor(p * 2^32)) computed by the host in double;
//   kept elements are multiplied by scale = 1 / (1 - p).
//   Attention probabilities (site 1): c1 = query, c0 = key div 4, c2 = 1, c3 = b * H + h.
//   Hidden states (site 2 = attention projection output, 3 = feed-forward activation output,
//   4 = second feed-forward linear output): c1 = row (b * T + t), c0 = column div 4, c2 = site, c3 = 0.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace fl {

struct DropSpec {
  uint32_t k0 = 0, k1 = 0;  // key
  uint32_t thr = 0;         // 0 = dropout off
  uint32_t site = 0;        // c2
  float scale = 1.f;
};

// Fills a DropSpec on the host.  p in [0, 1); p == 0 switches dropout off.
inline DropSpec make_drop_spec(float p, uint64_t seed, uint32_t site) {
  DropSpec d;
  if (!(p > 0.f)) return d;
  double t = (double)p * 4294967296.0;
  d.thr = t >= 4294967295.0 ? 4294967295u : (uint32_t)t;  // floor: t >= 0
  d.k0 = (uint32_t)(seed & 0xFFFFFFFFu);
  d.k1 = (uint32_t)(seed >> 32);
  d.site = site;
  d.scale = (float)(1.0 / (1.0 - (double)p));
  return d;
}

#if defined(__HIPCC__)
__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return make_uint4(c0, c1, c2, c3);
}

// Multipliers (0 or scale) of the four elements with columns 4*c0 .. 4*c0+3 of row c1.
__device__ __forceinline__ void drop_keep4(const DropSpec &d, uint32_t c0, uint32_t c1, uint32_t c3, float (&m)[4]) {
  const uint4 w = philox4x32_10(c0, c1, d.site, c3, d.k0, d.k1);
  m[0] = w.x >= d.thr ? d.scale : 0.f;
  m[1] = w.y >= d.thr ? d.scale : 0.f;
  m[2] = w.z >= d.thr ? d.scale : 0.f;
  m[3] = w.w >= d.thr ? d.scale : 0.f;
}
// Multiplier of the single element (row c1, column n).
__device__ __forceinline__ float drop_keep1(const DropSpec &d, uint32_t n, uint32_t c1, uint32_t c3) {
  const uint4 w = philox4x32_10(n >> 2, c1, d.site, c3, d.k0, d.k1);
  const uint32_t v = (n & 3) == 0 ? w.x : ((n & 3) == 1 ? w.y : ((n & 3) == 2 ? w.z : w.w));
  return v >= d.thr ? d.scale : 0.f;
}
#endif

}  // namespace fl
