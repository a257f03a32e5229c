// Host side of the wide LDS-resident kernel: which layers it takes, how the four waves of a
// work-group are shared out, and the dispatch to the per-family launchers (patch_wide_inst.hip).
#include <hip/hip_runtime.h>

#include <cmath>

#include "patch_wide.h"

namespace rmsmp {

#ifndef RMSMP_WIDE_FAMILIES  // (a tuning build may restrict the families it links)
#define RMSMP_WIDE_FAMILIES(X) X(9, 2) X(9, 4) X(9, 8) X(9, 16) X(1, 2) X(1, 4) X(1, 8) X(1, 16) X(1, 24)
#endif
#ifndef RMSMP_WIDE_DEEP_FAMILIES  // channel counts (in K steps) a deep 1x1 layer / GEMM is staged in parts of
#define RMSMP_WIDE_DEEP_FAMILIES(X) X(16) X(24)
#endif
#define RMSMP_WIDE_DECL(TP, CP) int launch_wide_##TP##_##CP(const WidePlan& p, hipStream_t s);
RMSMP_WIDE_FAMILIES(RMSMP_WIDE_DECL)
#undef RMSMP_WIDE_DECL
#define RMSMP_WIDE_DECL(CP) int launch_wide_deep_##CP(const WidePlan& p, hipStream_t s);
RMSMP_WIDE_DEEP_FAMILIES(RMSMP_WIDE_DECL)
#undef RMSMP_WIDE_DECL

#ifndef RMSMP_WIDE_PAIR_FAMILIES  // channel counts / 32 the two-layer launch exists for
#define RMSMP_WIDE_PAIR_FAMILIES(X) X(2) X(4) X(8)
#endif
#define RMSMP_WIDE_DECL(CP) int launch_wide_pair_##CP(const WidePlan& pa, const WidePlan& pb, hipStream_t s);
RMSMP_WIDE_PAIR_FAMILIES(RMSMP_WIDE_DECL)
#undef RMSMP_WIDE_DECL

static uint32_t wide_div_magic(int64_t d) {
  return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + (uint64_t)d - 1) / (uint64_t)d);
}


// One candidate split of the four waves; fills the plan when the layer fits it.
// cc: channels staged at a time (all of them, or a part of a deep 1x1 layer / GEMM).
static bool wide_plan_mode(const GemmArgs& a, int cc, int xb, int ks, int nwt, int ms, WidePlan* plan) {
  const bool known = (ks == 2 && nwt == 1 && ms == 2 && (xb == 2 || xb == 4)) ||
                     (xb == 4 && ((ks == 4 && nwt == 1 && ms == 1) || (ks == 2 && nwt == 2 && ms == 1) ||
                                 (ks == 1 && nwt == 4 && ms == 1) || (ks == 1 && nwt == 1 && ms == 4))) ||
                     (xb == 2 && ((ks == 2 && nwt == 2 && ms == 1) || (ks == 4 && nwt == 1 && ms == 1) ||
                                 (ks == 1 && nwt == 1 && ms == 4) || (ks == 1 && nwt == 4 && ms == 1)));
  if (!known) return false;
  if (a.ep.out_kind == 3 && !wide_has_gelu(a.d.KH * a.d.KW, xb)) return false;
  const int cpt = cc / KSTEP;
  if (cpt % ks != 0 || a.d.KH * a.d.KW * (cpt / ks) < 2) return false;
  const int64_t S = a.d.stride;
  const int64_t row_extra = S * ((int64_t)a.d.W - a.OW);
  const int64_t img_extra = (int64_t)a.d.W * ((int64_t)a.d.H - S * a.OH);
  const int64_t hw = (int64_t)a.OH * a.OW, in_px = (int64_t)a.d.B * a.d.H * a.d.W;
  const int rs = cc + 16;
  const int64_t bn = (int64_t)32 * xb * nwt;
  // widest run of flattened input pixels a tile of bn output pixels touches
  const int64_t rows_crossed = (bn + a.OW - 1) / a.OW + 1, imgs_crossed = (bn + hw - 1) / hw + 1;
  const bool gather = a.d.KH * a.d.KW == 1 && a.d.stride > 1;
  const int64_t span = gather ? bn : (bn - 1) * S + 1 + (int64_t)(a.d.KH - 1) * a.d.W + (a.d.KW - 1) + rows_crossed * row_extra +
                       imgs_crossed * (img_extra > 0 ? img_extra : 0);
  // 32-bit pixel arithmetic and exact one-multiply division in the kernel
  if ((a.N + bn) * hw >= ((int64_t)1 << 32) || in_px * (a.d.C / 2) >= ((int64_t)1 << 31) || in_px * (a.d.C / 2) < 16) return false;
  if (in_px + span >= ((int64_t)1 << 31) / rs) return false;
  // 24-bit multiplications in the kernel's pixel index arithmetic
  if (in_px + span >= ((int64_t)1 << 23) || a.N + bn >= ((int64_t)1 << 23) || hw >= ((int64_t)1 << 23)) return false;
  // image sides, stride and padding travel packed in the kernels' leading arguments
  if (a.d.H >= 65536 || a.d.W >= 65536 || a.OH >= 65536 || a.OW >= 65536 || a.d.stride >= 256 || a.d.pad >= 256) return false;
  // 24-bit LDS address arithmetic
  const size_t need = (size_t)(span + 1) * rs;  // patch + zero-point row
  const size_t xch = (size_t)pw_xch_bytes(xb, ks, ks * nwt * ms);
  const size_t lds = PHASE_LDS_BYTES + (size_t)ms * PW_META_BYTES + (need > xch ? need : xch);
  if (lds > 160 * 1024) return false;
  const int n_pairs = (a.w.n_tiles + 1) / 2;
  const int64_t gx = (a.N + bn - 1) / bn;
  const int gy = (n_pairs + ms - 1) / ms;
  if ((gx + 7) / 8 * 8 * gy > 0x7fffffff) return false;
  plan->a = a;
  plan->g.gx = (int)gx;
  plan->g.gy = gy;
  plan->g.row_stride = rs;
  plan->g.patch_rows = (int)span;
  plan->g.gather = gather ? 1 : 0;
  plan->g.nchunk = a.d.C / cc;
  plan->g.pix_bytes = a.d.C / 2;
  plan->cpt = cpt;
  plan->g.magic_hw = wide_div_magic(hw);
  plan->g.magic_ow = wide_div_magic(a.OW);
  plan->lds = lds;
  plan->blocks = (unsigned)((gx + 7) / 8 * 8 * gy);
  plan->xb = xb;
  plan->ks = ks;
  plan->nwt = nwt;
  plan->ms = ms;
  return true;
}

// Channel counts (in K steps of 32) the kernel is instantiated for.
static bool wide_cpt_supported(int taps, int cpt) {
  if (taps == 9) return cpt == 2 || cpt == 4 || cpt == 8 || cpt == 16;
  return cpt == 2 || cpt == 4 || cpt == 8 || cpt == 16 || cpt == 24;
}

// Whether the layer is one the kernel takes at all.  *a_out: the layer as a convolution (a plain
// GEMM becomes a 1x1 convolution over N single-pixel images); *cc_out: channels staged at a time.
static bool wide_layer_fits(const GemmArgs& a0, GemmArgs* a_out, int* cc_out) {
  if (a0.ep.act_bits != 4) return false;
  GemmArgs& a = *a_out;
  a = a0;
  if (!a.conv) {
    if (a.K % (2 * KSTEP) != 0 || a.K > 64 * 768 || a.N >= ((int64_t)1 << 30)) return false;
    a.conv = 1;
    a.d = rmsmp_conv_desc{(int32_t)a.N, (int32_t)a.K, 1, 1, 1, 1, 1, 0};
    a.OH = a.OW = 1;
    // A K that no 1x1 family takes, neither whole nor in parts, but that is nine times a channel
    // count of the 3x3 families (576, 1152: the lowered matrices of 3x3 layers): the same numbers
    // are a 3x3 convolution without padding over N images of 3x3 pixels -- column n of X is image
    // n, K index (tap, channel) -- which is the order a plain GEMM's weights are stored in.
    const int64_t c9 = a.K / 9;
    const bool as_1x1 = wide_cpt_supported(1, (int)(a.K / KSTEP)) || a.K % 768 == 0 || a.K % 512 == 0;
    if (!as_1x1 && a.K % 9 == 0 && c9 % KSTEP == 0 && wide_cpt_supported(9, (int)(c9 / KSTEP)) && a.N * 9 < ((int64_t)1 << 31)) {
      a.d = rmsmp_conv_desc{(int32_t)a.N, (int32_t)c9, 3, 3, 3, 3, 1, 0};
    }
  }
  const int taps = a.d.KH * a.d.KW;
  if (!(taps == 1 || (a.d.KH == 3 && a.d.KW == 3))) return false;
  // a strided 1x1 layer stages only the pixels it uses (one per output pixel); padding would need
  // out-of-image pixels there
  if (taps == 1 && a.d.stride > 1 && a.d.pad != 0) return false;
  // Channels staged at a time: all of them when the kernel exists for that count; a 1x1 layer of
  // stride 1 (a GEMM) with more takes them in equal parts, the largest part the kernel exists for.
  if (a.d.C % KSTEP != 0) return false;
  int cc = a.d.C;
  if (!wide_cpt_supported(taps, cc / KSTEP)) {
    if (!(taps == 1 && a.d.stride == 1)) return false;
    cc = 0;
    for (int c : {768, 512})
      if (a.d.C % c == 0 && a.d.C / c <= 64) {
        cc = c;
        break;
      }
    if (cc == 0) return false;
  }
  const int cpt = cc / KSTEP, nchunk = a.d.C / cc;
  if (a.w.nks != taps * cpt * nchunk) return false;
  // The flattened input index of tap (0,0) must grow with the output pixel number, also across
  // output rows and images, so that a tile's pixels lie in one contiguous run of the input.
  const int64_t S = a.d.stride;
  const int64_t row_extra = S * ((int64_t)a.d.W - a.OW);
  const int64_t img_extra = (int64_t)a.d.W * ((int64_t)a.d.H - S * a.OH);
  if (row_extra < 0 || row_extra + img_extra < 0) return false;
  *cc_out = cc;
  return true;
}

static bool wide_kernel_applies(const GemmArgs& a0, WidePlan* plan) {
  GemmArgs a;
  int cc = 0;
  if (!wide_layer_fits(a0, &a, &cc)) return false;
  const int taps = a.d.KH * a.d.KW;
  const int cpt = cc / KSTEP, nchunk = a.d.C / cc;
  const int n_pairs = (a.w.n_tiles + 1) / 2;
  // How the four waves are shared out: the candidate with the lowest estimated time wins.  The
  // estimate is a per-work-group critical path (cycles; the constants started from per-phase clock
  // stamps and were then fitted to the measured launch times of every candidate on the ResNet-18 and
  // BERT-base layer shapes on an MI355X) times the number of rounds the grid needs: prologue (a fixed part plus the
  // patch's way through LDS), K loop (cycles per MFMA depend on how many MFMAs share a decoded
  // weight fragment), partial-sum exchange (LDS traffic), epilogue (per finished 32x32 block).
  // Work-groups that share a compute unit overlap everything except their K loops' MFMAs.
  struct Mode { int xb, ks, nwt, ms; };
  const Mode modes[] = {{4, 1, 1, 4}, {4, 1, 4, 1}, {4, 2, 2, 1}, {4, 4, 1, 1}, {4, 2, 1, 2}, {2, 2, 2, 1}, {2, 4, 1, 1}, {2, 1, 1, 4}, {2, 1, 4, 1}, {2, 2, 1, 2}};
  WidePlan best;
  double best_cost = 0;
  bool have = false;
  for (const Mode& m : modes) {
    if (m.ms > 1 && n_pairs < m.ms) continue;
    WidePlan p;
    if (!wide_plan_mode(a, cc, m.xb, m.ks, m.nwt, m.ms, &p)) continue;
    const double wgs = (double)p.g.gx * p.g.gy;
    const double steps = (double)taps * cpt * nchunk / m.ks;
    const double mfmas = steps * 2 * m.xb;
    const double kloop = mfmas * (m.xb == 4 ? 36.3 : 49.7);
    // (every further part of the channels is staged like the first, between two barriers)
    const double prologue = 818.0 + (double)p.g.patch_rows * p.g.row_stride / 17.6 + (nchunk - 1) * (1500.0 + (double)p.g.patch_rows * p.g.row_stride / 17.6);
    const double exchange = m.ks == 1 ? 0.0 : (double)pw_xch_bytes(m.xb, m.ks, m.ks * m.nwt * m.ms) / 26.3;
    const double epilogue = 1520.0 + 665.0 * (2.0 * m.xb / m.ks);
    const double t_wg = prologue + kloop + exchange + epilogue;
    const int by_lds = (int)((160 * 1024) / p.lds), by_regs = (m.xb == 4 || nchunk > 1) ? 2 : 3;
    const int k_max = by_lds < by_regs ? by_lds : by_regs;
    const double per_cu = wgs / 256.0;
    // what one more work-group on the same compute unit adds: its MFMAs (the matrix pipe is
    // shared) and about a third of everything else; with 64 pixels per wave the vector ALU is the
    // shared bottleneck throughout, and little of the rest overlaps
    const double extra = m.xb == 4 ? mfmas * 28.5 + 0.264 * (t_wg - kloop) : mfmas * 46.7 + 0.434 * (t_wg - kloop);
    // the busiest compute units get n work-groups (a few stragglers beyond a whole number do not
    // count): whole rounds of k_max sharing the unit, then the rest
    const int n = per_cu < 1.0 ? 1 : (int)ceil(per_cu - 0.15);
    const int full = n / k_max, rest = n % k_max;
    const double cost = full * (t_wg + (k_max - 1) * extra) + (rest > 0 ? t_wg + (rest - 1) * extra : 0.0);
    if (!have || cost < best_cost) {
      best = p;
      best_cost = cost;
      have = true;
    }
  }
  if (!have) return false;
  *plan = best;
  return true;
}

static int launch_wide(const WidePlan& p, hipStream_t s) {
  const int taps = p.a.d.KH * p.a.d.KW;
  const int cpt = p.cpt;
  if (p.g.nchunk > 1) {
#define RMSMP_WIDE_CASE(CP) \
  if (taps == 1 && cpt == CP) return launch_wide_deep_##CP(p, s);
    RMSMP_WIDE_DEEP_FAMILIES(RMSMP_WIDE_CASE)
#undef RMSMP_WIDE_CASE
    return (int)hipErrorInvalidValue;
  }
#define RMSMP_WIDE_CASE(TP, CP) \
  if (taps == TP && cpt == CP) return launch_wide_##TP##_##CP(p, s);
  RMSMP_WIDE_FAMILIES(RMSMP_WIDE_CASE)
#undef RMSMP_WIDE_CASE
  return (int)hipErrorInvalidValue;
}

// Launches the wide kernel when the layer fits it; *applied says whether it did.
int try_launch_wide(const GemmArgs& a, void* stream, bool* applied) {
  WidePlan plan;
  *applied = wide_kernel_applies(a, &plan);
  const int* forced = forced_split();
  if (*applied && forced[0] > 0) {
    WidePlan p2;
    if (wide_plan_mode(plan.a, plan.cpt * KSTEP, forced[0], forced[1], forced[2], forced[3], &p2)) plan = p2;
  }
  if (!*applied) return 0;
  DispatchRecord& rec = last_dispatch();
  rec.kernel = 5;
  rec.xb = plan.xb, rec.ks = plan.ks, rec.nwt = plan.nwt, rec.ms = plan.ms;
  return launch_wide(plan, (hipStream_t)stream);
}

// Two layers on the same input as one launch (see conv_wide_pair_kernel): a 3x3 layer and a 1x1
// layer with the same 64, 128 or 256 input channels, both with 4-bit activations, neither with
// the GELU epilogue, each fitting the split the pair kernel is built with.  *applied says whether
// the launch happened; if not, the caller launches the layers one after the other.
int try_launch_wide_pair(const GemmArgs& a0, const GemmArgs& b0, void* stream, bool* applied) {
  *applied = false;
  GemmArgs a, b;
  int cca = 0, ccb = 0;
  if (a0.X != b0.X || !a0.conv || !b0.conv) return 0;
  if (a0.ep.out_kind == 3 || b0.ep.out_kind == 3) return 0;
  if (!wide_layer_fits(a0, &a, &cca) || !wide_layer_fits(b0, &b, &ccb)) return 0;
  if (a.d.KH * a.d.KW != 9 || b.d.KH * b.d.KW != 1) return 0;
  if (a.d.C != b.d.C || cca != a.d.C || ccb != b.d.C) return 0;
  const int cpt = a.d.C / KSTEP;
  if (cpt != 2 && cpt != 4 && cpt != 8) return 0;
  const WidePairSplit sp = wide_pair_split(cpt);
  if ((a.w.n_tiles + 1) / 2 < sp.ma || (b.w.n_tiles + 1) / 2 < sp.mb) return 0;
  WidePlan pa, pb;
  if (!wide_plan_mode(a, cca, sp.xa, sp.ka, sp.na, sp.ma, &pa) || !wide_plan_mode(b, ccb, sp.xb, sp.kb, sp.nb, sp.mb, &pb)) return 0;
  if ((uint64_t)pa.blocks + pb.blocks > 0x7fffffffu) return 0;
  *applied = true;
  DispatchRecord& rec = last_dispatch();
  rec.kernel = 6;
  rec.xb = 0, rec.ks = 0, rec.nwt = 0, rec.ms = 0;
#define RMSMP_WIDE_CASE(CP) \
  if (cpt == CP) return launch_wide_pair_##CP(pa, pb, (hipStream_t)stream);
  RMSMP_WIDE_PAIR_FAMILIES(RMSMP_WIDE_CASE)
#undef RMSMP_WIDE_CASE
  return (int)hipErrorInvalidValue;
}

}  // namespace rmsmp
