// Launch-shape selection of the register-resident inner loop (Algorithm 4, inner
// `for t`; kernel in inner_reg_impl.hpp): how many waves share a chain and how
// many 16-bit strips of z a lane owns.
#include "inner_args.hpp"

namespace halp {

int launch_inner_reg_b8(const InArgs& a, int nw, int upl, int R, bool packed, hipStream_t s);
int launch_inner_reg_b16(const InArgs& a, int nw, int upl, int R, hipStream_t s);
int launch_inner_reg_helped_b8(const InArgs& a, int nw, int upl, int R, hipStream_t s);
int launch_inner_reg_helped_b16(const InArgs& a, int nw, int upl, int R, hipStream_t s);
int launch_inner_reg_lone_b8(const InArgs& a, int upl, int R, bool pair, hipStream_t s);

namespace {

struct Shape {
  int nw, upl;
};

bool launchable(Shape sh) {
  if (sh.upl != 1 && sh.upl != 2 && sh.upl != 4 && sh.upl != 8) return false;
  if (sh.nw == 1 || sh.nw == 2 || sh.nw == 4) return true;
  return (sh.nw == 8 || sh.nw == 16) && sh.upl >= 4;
}

// `want_nw` waves per chain if the strips can be spread that thin, else as many
// strips per lane as it takes (at most 8, then more waves)
Shape pick_shape(const halp_params& p, int want_nw) {
  const int ct = 16 / p.b;
  const int U = (p.d + ct - 1) / ct;
  int nw = want_nw < 1 ? 1 : (want_nw > 16 ? 16 : want_nw);
  while (nw > 1 && (nw / 2) * 64 >= U) nw /= 2;  // no wave without a strip
  auto strips = [&](int w) {
    const int upl = (U + 64 * w - 1) / (64 * w);
    int u2 = 1;
    while (u2 < upl) u2 *= 2;
    return u2;
  };
  int upl = strips(nw);
  while (upl > 8 && nw < 16) {
    nw *= 2;
    upl = strips(nw);
  }
  if ((nw == 8 || nw == 16) && upl < 4) upl = 4;  // only wide lanes are built for 8 / 16 waves
  return Shape{nw, upl};
}

// the form with a helper wave beside every chain wave exists for these shapes
bool helped_shape(Shape sh) { return (sh.nw == 2 || sh.nw == 4) && sh.upl <= 2; }

// Chains per CU up to which that form pays, by chain waves (measured at d = 512, b = 8, epochs of
// 16384 steps: four chain waves win up to 2 chains per CU -- 3.0 ms at 256 chains, 3.7 at 512,
// where one wave per chain takes 5.5 -- two chain waves up to 5 per CU -- 4.2 ms at 576 chains,
// 6.0 at 1280 against 4.8 and 7.6 -- beyond that one wave per chain and no helpers)
constexpr int kHelpedChainsPerCu4 = 2, kHelpedChainsPerCu2 = 5;

// Strips per lane of the form with one chain wave and its helpers on the other SIMDs (8 bits,
// rows up to 1024 coordinates), or 0 if the shape does not fit it.  A helper reads fragments
// of one or two strips: every fragment that starts inside the row must end inside it.
int lone_strips(const halp_handle& h) {
  const halp_params& p = h.p;
  if (p.b != 8 || p.B != 1 || p.K != 1) return 0;
  const int U = (p.d + 1) / 2;
  const int upl = U <= 128 ? 2 : (U <= 256 ? 4 : (U <= 512 ? 8 : 0));
  if (upl == 0) return 0;
  const int sph = upl == 8 ? 2 : 1;  // strips of the widest fragment a helper reads
  if ((int64_t)((U + sph - 1) / sph) * sph * 2 > h.buf.ldxq) return 0;
  return upl;
}

// Where the library takes that form by itself: rows of 129 .. 512 coordinates (two or four strips
// per lane) up to two chains per CU, wider rows up to one.  Measured per epoch of 16384 steps at d = 512 (ms):
// 128 chains 2.57 against 2.91 for four chain waves with helpers, 256: 2.66 / 3.00, 384: 3.19 /
// 3.67, 512: 3.26 / 3.69; 768: 5.95 against 4.27 for the library's choice there, 1024: 6.43 / 5.15.
// d = 256 at 256 chains: 2.10 against 2.91.  d = 1024: 3.97 against 3.79 (the single wave issues
// ~9 instructions per strip and step); up to 128 coordinates one wave without helpers is faster.
// Rows of 513 .. 1024 coordinates (eight strips per lane) gain little -- 3.76 against 3.80 ms at 256
// chains, 22.4 against 22.8 ms for the single chain of 100000 steps, logistic 5.56 against 5.80 -- and only
// with a CU per chain.
bool lone_pays(const halp_handle& h, int upl) {
  if (h.p.d <= 128) return false;
  const int64_t per_cu = upl <= 4 ? 2 : 1;
  return (int64_t)h.p.R <= per_cu * h.num_cus;
}

// waves per chain: use the chip's SIMDs when chains are few, one wave per chain
// when they are many
int auto_waves(const halp_handle& h) {
  if (h.inner_waves > 0) return h.inner_waves;
  if (h.inner_helpers != 2) {
    const int64_t R = h.p.R, cus = h.num_cus;
    if (R <= kHelpedChainsPerCu4 * cus) {
      const Shape sh = pick_shape(h.p, 4);
      if (sh.nw == 4 && helped_shape(sh)) return 4;
    }
    if (R <= kHelpedChainsPerCu2 * cus) {
      const Shape sh = pick_shape(h.p, 2);
      if (sh.nw == 2 && helped_shape(sh)) return 2;
    }
  }
  const int64_t simds = 4 * (int64_t)h.num_cus;
  int nw = 1;
  while (nw < 4 && (int64_t)h.p.R * nw * 2 <= simds) nw *= 2;
  return nw;
}

}  // namespace

int inner_reg_supported(const halp_params& p) {
  if (p.B != 1 || p.K != 1) return HALP_ERR_UNSUPPORTED;
  if (p.loss != HALP_LOSS_SQUARED && p.loss != HALP_LOSS_LOGISTIC) return HALP_ERR_UNSUPPORTED;
  if (p.b == 8 && p.d > 131071) return HALP_ERR_UNSUPPORTED;  // int32 dot product stays exact
  const Shape sh = pick_shape(p, 16);
  return sh.upl <= 8 ? HALP_OK : HALP_ERR_UNSUPPORTED;
}

int launch_inner_reg(const halp_handle& h, uint32_t epoch, hipStream_t s) {
  const halp_params& p = h.p;
  int rc = inner_reg_supported(p);
  if (rc != HALP_OK) return rc;
  const InArgs a = make_inner_args(h, epoch);
  // 8 bits, at most one chain per CU: one chain wave with all of z, helpers on the other SIMDs
  const int lone_upl = lone_strips(h);
  if (lone_upl > 0 && (h.inner_helpers == 3 || (h.inner_helpers == 0 && h.inner_waves == 0 && lone_pays(h, lone_upl))))
    return launch_inner_reg_lone_b8(a, lone_upl, p.R, (int64_t)p.R > (int64_t)h.num_cus, s);  // more chains than CUs: the build that fits twice
  if (h.inner_helpers == 3) return HALP_ERR_UNSUPPORTED;
  Shape sh = pick_shape(p, auto_waves(h));
  const int ct = 16 / p.b;
  const int U = (p.d + ct - 1) / ct;
  // a lane reads whole fragments of 2*UPL bytes: the last one must lie inside the row, and
  // 16-byte fragments want 16-byte aligned rows
  const int64_t row_bytes = h.buf.ldxq * (p.b / 8);
  const bool base16 = (reinterpret_cast<uintptr_t>(h.buf.Xq) % 16) == 0 && row_bytes % 16 == 0;
  while (sh.upl > 1 && ((int64_t)((U + sh.upl - 1) / sh.upl) * sh.upl * 2 > row_bytes ||
                        (sh.upl == 8 && !base16))) {
    if (sh.nw >= 16) return HALP_ERR_UNSUPPORTED;
    sh.nw *= 2;  // spread the strips over more waves instead
    sh.upl /= 2;
  }
  if (!launchable(sh)) return HALP_ERR_UNSUPPORTED;
  // Few chains, two or four waves each: a helper wave beside every chain wave takes whatever
  // does not depend on z off the step's dependent chain.  Worth it while a CU holds a few chains.
  const bool helped_built = helped_shape(sh);
  if (helped_built &&
      (h.inner_helpers == 1 || (h.inner_helpers == 0 && (int64_t)p.R <= (int64_t)kHelpedChainsPerCu2 * h.num_cus)))
    return p.b == 8 ? launch_inner_reg_helped_b8(a, sh.nw, sh.upl, p.R, s)
                    : launch_inner_reg_helped_b16(a, sh.nw, sh.upl, p.R, s);
  // 8 bits, one wave per chain: the packed form once every SIMD holds two chains or more (its
  // steps issue fewer instructions but take longer alone), or as HALP_OPT_INNER_PACKED says
  const bool many = (int64_t)p.R >= 8 * (int64_t)h.num_cus;
  const bool packed = p.b == 8 && sh.nw == 1 && (h.inner_packed == 1 || (h.inner_packed == 0 && many));
  return p.b == 8 ? launch_inner_reg_b8(a, sh.nw, sh.upl, p.R, packed, s)
                  : launch_inner_reg_b16(a, sh.nw, sh.upl, p.R, s);
}

}  // namespace halp
