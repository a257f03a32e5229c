// Host side of rmsmp_pack_weights: row-wise quantization (Section 3.1.1, 3.1.2), grouping of
// rows by storage class, nibble packing and the tile layout the GEMM kernels read.
#include <algorithm>
#include <cfenv>
#include <cmath>
#include <cstring>
#include <numeric>

#include "rmsmp_internal.h"

namespace rmsmp {
namespace {

inline uint32_t float_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return u;
}

// w/alpha limited to [-1, 1] (the clip of Section 3.1.1).
inline float clipped_ratio(float w, float alpha) {
  if (w > alpha) return 1.0f;
  if (w < -alpha) return -1.0f;
  return w / alpha;
}

// Fixed-m code (Eq. 1-2): the integer q in [-Q, Q] whose level alpha*q/Q is nearest to w.
inline int fixed_code(float x, int Q) { return (int)std::nearbyintf(x * (float)Q); }

// PoT-4 (Eq. 3-4) on the clipped ratio x: returns sign * 2^(6-k), k = 0..6, or 0.
// round(log2 |x|) is read off the float's own fields: with |x| = 1.f * 2^e the logarithm
// rounds up exactly when 1.f > sqrt(2), i.e. when the 23 fraction bits exceed those of the
// largest float below sqrt(2) (0x3504F3).  No libm call, no rounding issue.
inline int pot4_int(float x) {
  const uint32_t u = float_bits(x) & 0x7fffffffu;
  if (u <= 0x3c000000u) return 0;  // |x| <= 2^-7: below half of the smallest level
  int e = (int)(u >> 23) - 127;
  if ((u & 0x7fffffu) > 0x3504f3u) e += 1;
  e = std::min(0, std::max(-6, e));
  const int mag = 1 << (6 + e);
  return (float_bits(x) >> 31) ? -mag : mag;
}

// 4-bit PoT code: bit 3 = sign, bits 2..0 = c with magnitude 2^(c-1), c = 0 for the zero level.
inline uint8_t pot4_nibble(int v) {
  if (v == 0) return 0;
  int mag = v < 0 ? -v : v, c = 1;
  while ((1 << (c - 1)) != mag) ++c;
  return (uint8_t)((v < 0 ? 8 : 0) | c);
}
inline int pot4_value(uint8_t nib) {
  const int c = nib & 7;
  if (c == 0) return 0;
  const int mag = 1 << (c - 1);
  return (nib & 8) ? -mag : mag;
}

// Build the two 8-byte tables with which two v_perm_b32 and one XOR turn a nibble n into the
// byte D[n]:   D[n] = perm(T1, n) ^ perm(T2, n ^ 8).
// v_perm_b32 returns table byte s for selector s < 8; for the other selectors it returns a
// constant: 8..11 -> 0x00/0xff by the sign of table byte 1/3/5/7, 12 -> 0x00, 13..15 -> 0xff.
// Each nibble hits a real entry in one table and a constant in the other; the constants are
// folded into the entries here.
void build_perm_tables(const int8_t D[16], uint32_t out[4]) {
  uint8_t T1[8], T2[8];
  auto sgn = [](uint8_t b) -> uint8_t { return (b & 0x80) ? 0xff : 0x00; };
  // selectors 12..15 in the other table give 0x00, 0xff, 0xff, 0xff
  const uint8_t c_hi[4] = {0x00, 0xff, 0xff, 0xff};
  for (int j = 0; j < 4; ++j) {
    T1[4 + j] = (uint8_t)D[4 + j] ^ c_hi[j];
    T2[4 + j] = (uint8_t)D[12 + j] ^ c_hi[j];
  }
  // selectors 8..11 in the other table give sign(byte 1), sign(byte 3), sign(byte 5), sign(byte 7)
  T1[2] = (uint8_t)D[2] ^ sgn(T2[5]);
  T1[3] = (uint8_t)D[3] ^ sgn(T2[7]);
  T2[2] = (uint8_t)D[10] ^ sgn(T1[5]);
  T2[3] = (uint8_t)D[11] ^ sgn(T1[7]);
  T2[1] = (uint8_t)D[9] ^ sgn(T1[3]);
  T1[1] = (uint8_t)D[1] ^ sgn(T2[3]);
  T1[0] = (uint8_t)D[0] ^ sgn(T2[1]);
  T2[0] = (uint8_t)D[8] ^ sgn(T1[1]);
  auto word = [](const uint8_t* b) {
    return (uint32_t)b[0] | ((uint32_t)b[1] << 8) | ((uint32_t)b[2] << 16) | ((uint32_t)b[3] << 24);
  };
  out[0] = word(T1);      // T1 bytes 0..3
  out[1] = word(T1 + 4);  // T1 bytes 4..7
  out[2] = word(T2);
  out[3] = word(T2 + 4);
}

}  // namespace

rmsmp_status ratio_counts(int64_t M, int32_t a, int32_t b, int32_t c, int64_t counts[3]) {
  if (M < 0 || a < 0 || b < 0 || c < 0 || a + b + c != 100 || !counts) return RMSMP_EINVAL;
  // round-half-to-even of M*pct/100 in integers
  auto share = [M](int pct) -> int64_t {
    const int64_t num = M * pct, q = num / 100, r = num % 100;
    if (r > 50 || (r == 50 && (q & 1))) return q + 1;
    return q;
  };
  int64_t n8 = share(c);
  if (c > 0 && n8 < 1 && M > 0) n8 = 1;
  int64_t np = (b == 0) ? M - n8 : share(a);
  if (np + n8 > M) np = M - n8;
  counts[RMSMP_FIXED4] = M - n8 - np;
  counts[RMSMP_POT4] = np;
  counts[RMSMP_FIXED8] = n8;
  return RMSMP_OK;
}

rmsmp_status assign_by_variance(const float* W, int64_t M, int64_t K, int64_t n_pot4, uint8_t* scheme) {
  if (!W || !scheme || M < 1 || K < 1 || n_pot4 < 0) return RMSMP_EINVAL;
  std::vector<std::pair<double, int64_t>> v;
  v.reserve((size_t)M);
  for (int64_t r = 0; r < M; ++r) {
    if (scheme[r] == RMSMP_FIXED8) continue;
    if (scheme[r] > RMSMP_FIXED8) return RMSMP_EINVAL;
    const float* w = W + r * K;
    double s = 0.0;
    for (int64_t k = 0; k < K; ++k) s += w[k];
    const double mean = s / (double)K;
    double q = 0.0;
    for (int64_t k = 0; k < K; ++k) q += ((double)w[k] - mean) * ((double)w[k] - mean);
    v.emplace_back(q / (double)K, r);
  }
  std::sort(v.begin(), v.end());
  for (size_t i = 0; i < v.size(); ++i)
    scheme[v[i].second] = ((int64_t)i < n_pot4) ? (uint8_t)RMSMP_POT4 : (uint8_t)RMSMP_FIXED4;
  return RMSMP_OK;
}

rmsmp_status pack_host(const float* W, int64_t M, int64_t K, const uint8_t* scheme, const float* alpha_in,
                       int32_t taps, const int32_t* in_perm, HostPacked* hp, std::string* err, uint32_t flags) {
  if (!W || !scheme || !hp) {
    *err = "pack_weights: NULL argument";
    return RMSMP_EINVAL;
  }
  if (M < 1 || K < 1 || taps < 1 || K % taps != 0) {
    *err = "pack_weights: need M >= 1, K >= 1, taps >= 1 and K % taps == 0";
    return RMSMP_ESHAPE;
  }
  if (std::fegetround() != FE_TONEAREST) {
    *err = "pack_weights: floating-point rounding mode must be round-to-nearest";
    return RMSMP_EINVAL;
  }
  const int64_t C = K / taps;
  hp->M = M;
  hp->K = K;
  hp->C = C;
  hp->taps = taps;
  // filter-row layout for small-channel square filters (see KLayout)
  int64_t kw_side = 0;
  while (kw_side * kw_side < taps) ++kw_side;
  const bool rows_layout = taps > 1 && C <= 4 && kw_side * kw_side == taps && kw_side <= 8;
  hp->k_layout = rows_layout ? K_FILTER_ROWS : K_TAP_CHANNEL;
  const int64_t Kint = rows_layout ? kw_side * KSTEP : K;
  hp->Kpad = (Kint + KPAD_UNIT - 1) / KPAD_UNIT * KPAD_UNIT;
  hp->nks = hp->Kpad / KSTEP;

  // internal K order -> original (channel, tap) index; -1 where the internal axis is padding
  hp->kmap.assign((size_t)hp->Kpad, -1);
  {
    std::vector<char> seen((size_t)C, 0);
    for (int64_t j = 0; j < C; ++j) {
      const int64_t c = in_perm ? in_perm[j] : j;
      if (c < 0 || c >= C || seen[(size_t)c]) {
        *err = "pack_weights: in_perm is not a permutation of the input channels";
        return RMSMP_EINVAL;
      }
      seen[(size_t)c] = 1;
      for (int64_t t = 0; t < taps; ++t) {
        const int64_t kint = rows_layout ? (t / kw_side) * KSTEP + (t % kw_side) * 4 + j : t * C + j;
        hp->kmap[(size_t)kint] = (int32_t)(c * taps + t);
      }
    }
  }

  // 1. quantize every row (original K order), keep integer levels
  std::vector<int8_t> wint((size_t)M * (size_t)K);
  hp->rowscale.resize((size_t)M);
  hp->rowsum.resize((size_t)M);
  hp->scheme.assign(scheme, scheme + M);
  hp->counts[0] = hp->counts[1] = hp->counts[2] = 0;
  for (int64_t r = 0; r < M; ++r) {
    if (scheme[r] > RMSMP_FIXED8) {
      *err = "pack_weights: scheme code out of range at row " + std::to_string(r);
      return RMSMP_EINVAL;
    }
    const float* w = W + r * K;
    // a NaN or infinite weight has no level: refused whether or not the caller supplies alpha
    float wmax = 0.0f;
    bool finite = true;
    for (int64_t k = 0; k < K; ++k) {
      finite = finite && std::isfinite(w[k]);
      wmax = std::max(wmax, std::fabs(w[k]));
    }
    if (!finite) {
      *err = "pack_weights: non-finite weight in row " + std::to_string(r);
      return RMSMP_EINVAL;
    }
    float alpha;
    if (alpha_in) {
      alpha = alpha_in[r];
      if (!(alpha > 0.0f) || !std::isfinite(alpha)) {
        *err = "pack_weights: alpha must be positive and finite (row " + std::to_string(r) + ")";
        return RMSMP_EINVAL;
      }
    } else {
      alpha = wmax == 0.0f ? 1.0f : wmax;
    }
    hp->counts[scheme[r]] += 1;
    int8_t* q = wint.data() + r * K;
    int64_t sum = 0;
    if (scheme[r] == RMSMP_POT4) {
      hp->rowscale[(size_t)r] = alpha * 0.015625f;
      for (int64_t k = 0; k < K; ++k) {
        q[k] = (int8_t)pot4_int(clipped_ratio(w[k], alpha));
        sum += q[k];
      }
    } else {
      const int Q = scheme[r] == RMSMP_FIXED4 ? 7 : 127;
      hp->rowscale[(size_t)r] = alpha / (float)Q;
      for (int64_t k = 0; k < K; ++k) {
        q[k] = (int8_t)fixed_code(clipped_ratio(w[k], alpha), Q);
        sum += q[k];
      }
    }
    hp->rowsum[(size_t)r] = (int32_t)sum;
  }

  // 2. storage class per row.  Fixed-4 rows decode by mask/shift, PoT-4 rows through the byte
  // table, Fixed-8 rows are stored as bytes.  A class whose row count is not a multiple of the
  // tile height hands its last (count % TILE_M) rows to the next, more general class when one
  // follows: a Fixed-4 row decodes fine through a table and any 4-bit row fits a byte.  Levels
  // and scales do not change, and the layer needs ceil(M / TILE_M) tiles instead of up to two more.
  // Every class then starts at a multiple of TILE_M in grouped order (two grouped rows share
  // one byte of the 4-bit output, so class boundaries must at least be even).
  // With RMSMP_PACK_POT_AS_INT8 the PoT-4 rows are stored decoded, one byte per level: the same
  // levels and scales, twice the bytes, and nothing to decode in the kernels' K loops.
  const bool pot_bytes = (flags & RMSMP_PACK_POT_AS_INT8) != 0;
  std::vector<int32_t> cls((size_t)M);
  for (int64_t r = 0; r < M; ++r)
    cls[(size_t)r] = scheme[r] == RMSMP_FIXED4 ? TILE_NIB_SHIFT : (scheme[r] == RMSMP_POT4 && !pot_bytes) ? TILE_NIB_LUT : TILE_I8;
  int64_t n_cls[3] = {hp->counts[0], pot_bytes ? 0 : hp->counts[1], hp->counts[2] + (pot_bytes ? hp->counts[1] : 0)};
  for (int c = 0; c < 2; ++c) {
    int64_t spill = n_cls[c] % TILE_M;
    if (spill == 0) continue;
    bool later = false;
    for (int c2 = c + 1; c2 < 3; ++c2) later = later || n_cls[c2] > 0;
    if (!later) continue;  // nothing follows: the last tile of this class is padded instead
    const int next = c + 1;
    for (int64_t r = M - 1; r >= 0 && spill > 0; --r)
      if (cls[(size_t)r] == c) {
        cls[(size_t)r] = next;
        --spill;
        n_cls[c] -= 1;
        n_cls[next] += 1;
      }
  }

  // 3. grouped order and tiles
  hp->perm.clear();
  hp->tiles.clear();
  for (int c = 0; c < 3; ++c) {
    const int64_t g_begin = (int64_t)hp->perm.size();
    for (int64_t r = 0; r < M; ++r)
      if (cls[(size_t)r] == c) hp->perm.push_back((int32_t)r);
    const int64_t n = (int64_t)hp->perm.size() - g_begin;
    for (int64_t t = 0; t * TILE_M < n; ++t) {
      TileDesc td{};
      td.kind = c;
      td.g0 = (int32_t)(g_begin + t * TILE_M);
      td.nvalid = (int32_t)std::min<int64_t>(TILE_M, n - t * TILE_M);
      hp->tiles.push_back(td);
    }
  }
  const int64_t n_tiles = (int64_t)hp->tiles.size();
  const int64_t Mpad = n_tiles * TILE_M;
  hp->p_rowscale.assign((size_t)Mpad, 0.0f);
  hp->p_rowsum.assign((size_t)Mpad, 0);
  hp->p_orig.assign((size_t)Mpad, -1);
  hp->p_gpos.assign((size_t)Mpad, -1);
  hp->p_lut.assign((size_t)Mpad * 4, 0u);
  hp->p_meta.assign((size_t)Mpad * 4, 0);
  for (int64_t p = 0; p < Mpad; ++p) hp->p_meta[(size_t)p * 4 + 2] = hp->p_meta[(size_t)p * 4 + 3] = -1;

  int64_t off = 0;
  for (auto& td : hp->tiles) {
    td.blob_off = off;
    off += hp->nks * LANES * (td.kind == TILE_I8 ? 16 : 8);
  }
  hp->blob.assign((size_t)off, 0);

  // 4. fill tables and blob.  MFMA row i of a tile carries grouped offset tile_row_goff(i).
  for (int64_t t = 0; t < n_tiles; ++t) {
    const TileDesc& td = hp->tiles[(size_t)t];
    for (int i = 0; i < TILE_M; ++i) {
      const int goff = tile_row_goff(i);
      if (goff >= td.nvalid) continue;
      const int64_t p = t * TILE_M + goff;
      const int64_t g = td.g0 + goff;
      const int64_t orig = hp->perm[(size_t)g];
      hp->p_orig[(size_t)p] = (int32_t)orig;
      hp->p_gpos[(size_t)p] = (int32_t)g;
      hp->p_rowscale[(size_t)p] = hp->rowscale[(size_t)orig];
      hp->p_rowsum[(size_t)p] = hp->rowsum[(size_t)orig];
      {
        int32_t* m = &hp->p_meta[(size_t)p * 4];
        std::memcpy(&m[0], &hp->rowscale[(size_t)orig], 4);
        m[1] = hp->rowsum[(size_t)orig];
        m[2] = (int32_t)orig;
        m[3] = (int32_t)g;
      }
      const bool pot = scheme[orig] == RMSMP_POT4;
      if (td.kind == TILE_NIB_LUT) {
        int8_t D[16];
        for (int n = 0; n < 16; ++n) D[n] = pot ? (int8_t)pot4_value((uint8_t)n) : (int8_t)(n < 8 ? n : n - 16);
        build_perm_tables(D, &hp->p_lut[(size_t)p * 4]);
      }
      const int8_t* q = wint.data() + orig * K;
      for (int64_t ks = 0; ks < hp->nks; ++ks)
        for (int kb = 0; kb < 2; ++kb) {
          const int lane = kb * TILE_M + i;
          int8_t v[16];
          for (int e = 0; e < 16; ++e) {
            const int64_t kk = ks * KSTEP + kb * 16 + e;
            v[e] = hp->kmap[(size_t)kk] >= 0 ? q[hp->kmap[(size_t)kk]] : (int8_t)0;
          }
          if (td.kind == TILE_I8) {
            uint8_t* dst = hp->blob.data() + td.blob_off + (ks * LANES + lane) * 16;
            for (int s = 0; s < 16; ++s) dst[s] = (uint8_t)v[kSlot[s]];
          } else {
            uint8_t* dst = hp->blob.data() + td.blob_off + (ks * LANES + lane) * 8;
            for (int b = 0; b < 8; ++b) {
              uint8_t lo, hi;
              if (pot) {
                lo = pot4_nibble(v[2 * b]);
                hi = pot4_nibble(v[2 * b + 1]);
              } else {
                lo = (uint8_t)v[2 * b] & 0xf;
                hi = (uint8_t)v[2 * b + 1] & 0xf;
              }
              dst[b] = (uint8_t)(lo | (hi << 4));
            }
          }
        }
    }
  }
  return RMSMP_OK;
}

// Software model of v_perm_b32 for one selector byte over the 8-byte pool {hi, lo}.
static uint8_t perm_byte(uint32_t hi, uint32_t lo, uint8_t sel) {
  const uint64_t pool = ((uint64_t)hi << 32) | lo;
  if (sel >= 13) return 0xff;
  if (sel == 12) return 0x00;
  if (sel >= 8) return ((pool >> (8 * (2 * (sel - 8) + 1) + 7)) & 1) ? 0xff : 0x00;
  return (uint8_t)(pool >> (8 * sel));
}

// Nibble -> byte exactly as the kernel does it: two table look-ups and an xor.
static int8_t lut_decode(const uint32_t* T, uint8_t nib) {
  return (int8_t)(perm_byte(T[1], T[0], nib) ^ perm_byte(T[3], T[2], (uint8_t)(nib ^ 8)));
}

void unpack_host(const HostPacked& hp, const uint8_t* blob, int8_t* wint) {
  const int64_t K = hp.K;
  for (size_t t = 0; t < hp.tiles.size(); ++t) {
    const TileDesc& td = hp.tiles[t];
    for (int i = 0; i < TILE_M; ++i) {
      const int goff = tile_row_goff(i);
      if (goff >= td.nvalid) continue;
      const int64_t orig = hp.perm[(size_t)(td.g0 + goff)];
      for (int64_t ks = 0; ks < hp.nks; ++ks)
        for (int kb = 0; kb < 2; ++kb) {
          const int lane = kb * TILE_M + i;
          int8_t v[16];
          if (td.kind == TILE_I8) {
            const uint8_t* src = blob + td.blob_off + (ks * LANES + lane) * 16;
            for (int s = 0; s < 16; ++s) v[kSlot[s]] = (int8_t)src[s];
          } else {
            const uint8_t* src = blob + td.blob_off + (ks * LANES + lane) * 8;
            for (int b = 0; b < 8; ++b) {
              const uint8_t lo = src[b] & 0xf, hi = src[b] >> 4;
              if (td.kind == TILE_NIB_LUT) {
                const uint32_t* T = &hp.p_lut[((size_t)t * TILE_M + goff) * 4];
                v[2 * b] = lut_decode(T, lo);
                v[2 * b + 1] = lut_decode(T, hi);
              } else {
                v[2 * b] = (int8_t)(lo < 8 ? lo : lo - 16);
                v[2 * b + 1] = (int8_t)(hi < 8 ? hi : hi - 16);
              }
            }
          }
          for (int e = 0; e < 16; ++e) {
            const int64_t kk = ks * KSTEP + kb * 16 + e;
            if (hp.kmap[(size_t)kk] >= 0) wint[orig * K + hp.kmap[(size_t)kk]] = v[e];
          }
        }
    }
  }
}

}  // namespace rmsmp
