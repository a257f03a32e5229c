// Host side of the GELU epilogue (out_kind 3): the feed-forward activation of a transformer layer
// (the BERT-base workload of Section 4.1) followed by the affine 4-bit activation quantizer,
//   g = GELU(y) = y * Phi(y)  evaluated in float64 and rounded to fp32 once,
//   code = clamp(rint(g * inv_s) + z, 0, 15).
// A kernel cannot afford a float64 erf per output value, and does not need one: as a function of the
// fp32 pre-activation y the code is piecewise constant with at most 30 break points -- GELU falls
// from 0 to its minimum (about -0.17 at y* = -0.7518) and rises from there, and rounding keeps
// either branch monotone.  This file finds the break points exactly, by bisection over the fp32
// number line with the definition above; the kernels then only compare y with them.
#include <cmath>
#include <cstring>

#include "rmsmp_internal.h"

namespace rmsmp {
namespace {

// fp32 <-> a signed integer key that orders like the float (64 bits wide: the distance between two
// keys does not fit 32)
inline int64_t key_of(float f) {
  int32_t i;
  std::memcpy(&i, &f, 4);
  return i < 0 ? -(int64_t)(i & 0x7fffffff) : (int64_t)i;
}
inline float float_of(int64_t k) {
  const uint32_t i = k < 0 ? 0x80000000u | (uint32_t)(-k) : (uint32_t)k;
  float f;
  std::memcpy(&f, &i, 4);
  return f;
}

inline float gelu_f32(float y) {
  const double x = (double)y;
  return (float)(0.5 * x * erfc(-x / sqrt(2.0)));
}

inline int code_of(float y, float inv_s, int z) {
  const float t = gelu_f32(y) * inv_s;
  float c = rintf(t) + (float)z;
  c = c < 0.0f ? 0.0f : c > 15.0f ? 15.0f : c;
  return (int)c;
}

// what the kernel starts its search from on the rising branch: the code y itself would get
inline int guess_of(float y, float inv_s, int z) {
  const float yp = y > 0.0f ? y : 0.0f;
  float t = yp * inv_s;
  t = t < 15.0f ? t : 15.0f;
  int g = (int)rintf(t) + z;
  return g > 15 ? 15 : g;
}

}  // namespace

// The split point between the branches: the fp32 number nearest to the minimum of y * Phi(y).
// Within one fp32 step of the true minimum GELU varies by less than 1e-14, far below fp32
// resolution, so both branches are monotone in fp32 on their side of it.
static const float kGeluSplit = -0.7517916f;
static const float kFar = 3.0e38f;

void gelu_table(float inv_s, int32_t z, GeluTable* t) {
  t->y_split = kGeluSplit;
  const int64_t k_split = key_of(kGeluSplit), k_hi = key_of(kFar), k_lo = key_of(-kFar);
  // ---- rising branch, y >= split: rise[c] = smallest y with code >= c (-inf: every y, +inf: none)
  const int c_split = code_of(kGeluSplit, inv_s, z), c_top = code_of(kFar, inv_s, z);
  for (int c = 0; c < 16; ++c) {
    if (c <= c_split) {
      t->rise[c] = -INFINITY;
    } else if (c > c_top) {
      t->rise[c] = INFINITY;
    } else {
      int64_t lo = k_split, hi = k_hi;  // code(lo) < c <= code(hi)
      while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (code_of(float_of(mid), inv_s, z) >= c) hi = mid; else lo = mid;
      }
      t->rise[c] = float_of(hi);
    }
  }
  // how far the first guess can lie above the code: checked right below every break point
  // (between break points the code stands still and the guess only grows with y) and at the top
  int d = guess_of(kGeluSplit, inv_s, z) - c_split;
  for (int c = c_split + 1; c <= c_top; ++c) {
    const int g = guess_of(float_of(key_of(t->rise[c]) - 1), inv_s, z) - (c - 1);
    d = g > d ? g : d;
  }
  { const int g = guess_of(kFar, inv_s, z) - c_top; d = g > d ? g : d; }
  t->fix_steps = d < 0 ? 0 : d;
  // ---- falling branch, y < split: code = fall_base + #{ j : y <= fall[j] }
  const int64_t k_below = k_split - 1;
  const int c_below = code_of(float_of(k_below), inv_s, z), c_far = code_of(-kFar, inv_s, z);
  t->fall_base = c_below;
  t->n_fall = 0;
  for (int j = 0; j < 16; ++j) t->fall[j] = -INFINITY;
  for (int c = c_below + 1; c <= c_far; ++c) {
    int64_t lo = k_lo, hi = k_below;  // code(lo) >= c > code(hi): largest y with code >= c
    while (hi - lo > 1) {
      const int64_t mid = lo + (hi - lo) / 2;
      if (code_of(float_of(mid), inv_s, z) >= c) lo = mid; else hi = mid;
    }
    t->fall[t->n_fall++] = float_of(lo);
  }
}

}  // namespace rmsmp
