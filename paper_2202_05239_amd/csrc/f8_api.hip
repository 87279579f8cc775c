// C-ABI entry points of the single-layer calls: validation on the host, then launches.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <unordered_map>

#include "f8_host.h"

namespace f8 {

namespace {
struct TuningName { const char *name; const char *env; std::atomic<int> Tuning::*field; };
const TuningName kTuningNames[] = {
    {"conv_variant", "F8_CONV_VARIANT", &Tuning::conv_variant}, {"conv_ws", "F8_CONV_WS", &Tuning::conv_ws},
    {"conv_ws_min", "F8_CONV_WS_MIN", &Tuning::conv_ws_min},
    {"pw_ws", "F8_PW_WS", &Tuning::pw_ws},                       {"pw_small", "F8_PW_SMALL", &Tuning::pw_small},
    {"xcd_remap", "F8_XCD_REMAP", &Tuning::xcd_remap},           {"stem_pool", "F8_STEM_POOL", &Tuning::stem_pool},
    {"conv_tail", "F8_CONV_TAIL", &Tuning::conv_tail},         {"conv_img", "F8_CONV_IMG", &Tuning::conv_img},
    {"pw_wide", "F8_PW_WIDE", &Tuning::pw_wide},                 {"conv_img_min", "F8_CONV_IMG_MIN", &Tuning::conv_img_min},
    {"pw_mid", "F8_PW_MID", &Tuning::pw_mid},
};
}  // namespace

Tuning &tuning() {
  // the environment is read here, once, the first time any switch is looked at
  static Tuning *t = [] {
    Tuning *n = new Tuning();
    for (const TuningName &k : kTuningNames)
      if (const char *e = getenv(k.env)) (n->*(k.field)).store(atoi(e));
    return n;
  }();
  return *t;
}

f8_status check_quant(const f8_quant *q, bool allow_res) {
  if (!q) return F8_ERR_NULL;
  if (q->x_type != F8_U8 && q->x_type != F8_S8) return F8_ERR_DTYPE;
  if (q->y_type != F8_U8 && q->y_type != F8_S8 && q->y_type != F8_S32) return F8_ERR_DTYPE;
  if (q->res) {
    if (!allow_res) return F8_ERR_UNSUPPORTED;
    if (q->res_type != F8_U8 && q->res_type != F8_S8 && q->res_type != F8_S32) return F8_ERR_DTYPE;
    const int d = q->fl_x + q->fl_w - q->fl_res;
    if (d < -24 || d > 24) return F8_ERR_FL;
  }
  if (q->y_type != F8_S32) {
    const int s = q->fl_x + q->fl_w - q->fl_y;
    if (s < -8 || s > 24) return F8_ERR_FL;
    if (q->clip_lo > q->clip_hi) return F8_ERR_CLIP;
    if (q->y_type == F8_U8 && (q->clip_lo < 0 || q->clip_hi > 255)) return F8_ERR_CLIP;
    if (q->y_type == F8_S8 && (q->clip_lo < -127 || q->clip_hi > 127)) return F8_ERR_CLIP;
  }
  return F8_OK;
}

f8_status check_requant2(const f8_quant &q, const f8_requant2 *q2) {
  if (!q2) return F8_ERR_NULL;
  if (q.y_type == F8_S32) return F8_ERR_DTYPE;
  if (q2->y_type != F8_U8 && q2->y_type != F8_S8) return F8_ERR_DTYPE;
  const int s = q.fl_x + q.fl_w - q2->fl_y;
  if (s < -8 || s > 24) return F8_ERR_FL;
  if (q2->clip_lo > q2->clip_hi) return F8_ERR_CLIP;
  if (q2->y_type == F8_U8 && (q2->clip_lo < 0 || q2->clip_hi > 255)) return F8_ERR_CLIP;
  if (q2->y_type == F8_S8 && (q2->clip_lo < -127 || q2->clip_hi > 127)) return F8_ERR_CLIP;
  return F8_OK;
}

f8_status check_geom(Geom &g, bool depthwise) {
  if (g.B < 0 || g.H < 1 || g.W < 1 || g.Cin < 1 || g.Cout < 0 || g.R < 1 || g.S < 1 || g.sh < 1 ||
      g.sw < 1 || g.ph < 0 || g.pw < 0)
    return F8_ERR_SHAPE;
  if (depthwise && g.Cout != g.Cin) return F8_ERR_SHAPE;
  const long long K = (long long)g.R * g.S * (depthwise ? 1 : g.Cin);
  if (K > 65536) return F8_ERR_SHAPE;
  g.P = out_extent(g.H, g.ph, g.R, g.sh);
  g.Q = out_extent(g.W, g.pw, g.S, g.sw);
  const long long lim = 0x7fffffffLL;
  const long long xb = (long long)g.B * g.H * g.W;
  const long long yb = (long long)g.B * g.P * g.Q;
  if (xb > lim || xb * g.Cin > lim || yb > lim || yb * g.Cout > lim) return F8_ERR_UNSUPPORTED;
  return F8_OK;
}

f8_status check_align(const int32_t *bias, const void *y, const f8_quant &q, const void *res) {
  if (reinterpret_cast<uintptr_t>(bias) & 3) return F8_ERR_ALIGN;
  if (q.y_type == F8_S32 && (reinterpret_cast<uintptr_t>(y) & 3)) return F8_ERR_ALIGN;
  if (res && q.res_type == F8_S32 && (reinterpret_cast<uintptr_t>(res) & 3)) return F8_ERR_ALIGN;
  return F8_OK;
}

static int widest_vec(int C, const void *a, const void *b) {
  const uintptr_t bits = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | (uintptr_t)C;
  if ((bits & 15) == 0) return 16;
  if ((bits & 3) == 0) return 4;
  return 1;
}

// The 3x3 64 -> 64 layers have a kernel of their own (weights in registers, input patch in LDS).
static bool use_conv_ws(const void *x, const int8_t *w, const void *y, const void *res, const Geom &g,
                        const f8_quant &q, const void *y2) {
  if (!tuning().conv_ws.load(std::memory_order_relaxed) || res || y2 || q.y_type == F8_S32) return false;
  // measured against the general kernel: 10-15 % ahead at 800 blocks (the single 3x3 layer at batch 32),
  // 20-30 % ahead once every workgroup walks over several tiles
  const int granule = g.Cin == 64 ? 128 : 64;       // pixels
  if ((long long)g.B * ((g.H * g.W + granule - 1) / granule) < tuning().conv_ws_min.load(std::memory_order_relaxed)) return false;
  return conv_ws_applicable(g.Cin, g.Cout, g.R, g.S, g.sh, g.sw, g.ph, g.pw, g.H, g.W, q.fl_x + q.fl_w - q.fl_y, x, w, y);
}

// So do the 1x1 64 -> 256 layers (weights in registers, every wave streams pixels on its own).
static bool use_pw_ws(const void *x, const int8_t *w, const void *y, const void *res, const Geom &g,
                      const f8_quant &q, const void *y2) {
  if (!tuning().pw_ws.load(std::memory_order_relaxed) || y2 || q.y_type == F8_S32 || (res && q.res_type == F8_S32)) return false;
  // it pays once every workgroup walks over several blocks of pixels
  if ((long long)g.B * g.H * g.W < 131072) return false;
  return pw_ws_applicable(g.Cin, g.Cout, g.R, g.S, g.sh, g.sw, g.ph, g.pw, q.fl_x + q.fl_w - q.fl_y, x, w, y, res);
}

// The 1x1 128 -> 512 layers (the closing layers of the second ResNet stage): with the 512 -> 128 layer behind
// them in the same launch, or (switch at 2) on their own.
static bool use_pw_mid(const void *x, const int8_t *w, const void *y, const void *res, const Geom &g,
                       const f8_quant &q, const void *y2, bool with_tail) {
  const int level = tuning().pw_mid.load(std::memory_order_relaxed);
  if (level < (with_tail ? 1 : 2) || y2 || q.y_type == F8_S32 || (res && q.res_type == F8_S32)) return false;
  // it pays once every workgroup walks over several pairs of blocks
  if ((long long)g.B * g.H * g.W < 65536) return false;
  return pw_mid_applicable(g.Cin, g.Cout, g.R, g.S, g.sh, g.sw, g.ph, g.pw, q.fl_x + q.fl_w - q.fl_y, x, w, y, res);
}

// And the 1x1 layers with 256 or 512 input channels and at least as many output channels per workgroup
// as its four waves hold weights for (the closing layers of the third and fourth ResNet stage).
static bool use_pw_wide(const void *x, const int8_t *w, const void *y, const void *res, const Geom &g,
                        const f8_quant &q, const void *y2) {
  if (!tuning().pw_wide.load(std::memory_order_relaxed) || y2 || q.y_type == F8_S32 || (res && q.res_type == F8_S32)) return false;
  // it pays once every workgroup walks over several blocks of 32 pixels: blocks x channel slices >= 4 x 512
  if ((g.Cin != 256 && g.Cin != 512) || (long long)g.B * g.H * g.W / 32 * (g.Cout / (4 * (16384 / g.Cin))) < 2048) return false;
  return pw_wide_applicable(g.Cin, g.Cout, g.R, g.S, g.sh, g.sw, g.ph, g.pw, q.fl_x + q.fl_w - q.fl_y, x, w, y, res);
}

// And the 1x1 layers with 16 or 32 input and 96 / 144 / 192 output channels (MobileNetV2's first expand layers).
static bool use_pw_small(const void *x, const int8_t *w, const void *y, const void *res, const Geom &g,
                         const f8_quant &q, const void *y2) {
  if (!tuning().pw_small.load(std::memory_order_relaxed) || res || y2 || q.y_type == F8_S32) return false;
  if ((long long)g.B * g.H * g.W < 65536) return false;
  return pw_small_applicable(g.Cin, g.Cout, g.R, g.S, g.sh, g.sw, g.ph, g.pw, q.fl_x + q.fl_w - q.fl_y, x, w, y);
}

f8_status enqueue_conv(const void *x, const int8_t *w, const int32_t *acc0, const void *zero, void *y,
                       const void *res, const Geom &g, const f8_quant &q, hipStream_t stream,
                       const f8_requant2 *q2, void *y2, const ConvTail *tail) {
  if (!tail && use_pw_small(x, w, y, res, g, q, (q2 && y2) ? y2 : nullptr) && (reinterpret_cast<uintptr_t>(acc0) & 15) == 0) {
    PwSmallParams sp;
    sp.x = static_cast<const uint8_t *>(x);
    sp.w = w;
    sp.acc0 = acc0;
    sp.y = static_cast<uint8_t *>(y);
    sp.M = (long long)g.B * g.H * g.W;
    sp.C = g.Cin; sp.N = g.Cout;
    sp.shift = q.fl_x + q.fl_w - q.fl_y; sp.lo = q.clip_lo; sp.hi = q.clip_hi;
    sp.x_xor = q.x_type == F8_U8 ? 0x80808080u : 0u;
    return launch_pw_small(sp, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
  }
  const bool pw_ws = use_pw_ws(x, w, y, res, g, q, (q2 && y2) ? y2 : nullptr) && (reinterpret_cast<uintptr_t>(acc0) & 15) == 0;
  const bool pw_mid = use_pw_mid(x, w, y, res, g, q, (q2 && y2) ? y2 : nullptr, tail != nullptr) && (reinterpret_cast<uintptr_t>(acc0) & 15) == 0;
  if (pw_mid && (!tail || (tail->Cout == 128 && tail->q.y_type != F8_S32))) {
    PwMidParams pp;
    pp.t_w = nullptr; pp.t_acc0 = nullptr; pp.t_y = nullptr;
    pp.t_shift = pp.t_lo = pp.t_hi = 0; pp.t_xor = 0;
    if (tail) {
      pp.t_w = tail->w; pp.t_acc0 = tail->acc0; pp.t_y = static_cast<uint8_t *>(tail->y);
      pp.t_shift = tail->q.fl_x + tail->q.fl_w - tail->q.fl_y;
      pp.t_lo = tail->q.clip_lo; pp.t_hi = tail->q.clip_hi;
      pp.t_xor = tail->q.x_type == F8_U8 ? 0x80808080u : 0u;
    }
    pp.x = static_cast<const uint8_t *>(x);
    pp.w = w;
    pp.acc0 = acc0;
    pp.res = static_cast<const uint8_t *>(res);
    pp.y = static_cast<uint8_t *>(y);
    pp.M = (long long)g.B * g.H * g.W;
    pp.shift = q.fl_x + q.fl_w - q.fl_y; pp.lo = q.clip_lo; pp.hi = q.clip_hi;
    pp.res_signed = q.res_type == F8_S8;
    pp.res_d = res ? q.fl_x + q.fl_w - q.fl_res : 0;
    pp.x_xor = q.x_type == F8_U8 ? 0x80808080u : 0u;
    return launch_pw_mid(pp, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
  }
  if (tail && !(pw_ws && (tail->Cout == 64 || tail->Cout == 128) && tail->q.y_type != F8_S32)) return F8_ERR_UNSUPPORTED;
  if (pw_ws) {
    PwWsParams pp;
    pp.t_w = nullptr; pp.t_acc0 = nullptr; pp.t_y = nullptr;
    pp.t_n = pp.t_shift = pp.t_lo = pp.t_hi = 0; pp.t_xor = 0;
    if (tail) {
      pp.t_w = tail->w; pp.t_acc0 = tail->acc0; pp.t_y = static_cast<uint8_t *>(tail->y); pp.t_n = tail->Cout;
      pp.t_shift = tail->q.fl_x + tail->q.fl_w - tail->q.fl_y;
      pp.t_lo = tail->q.clip_lo; pp.t_hi = tail->q.clip_hi;
      pp.t_xor = tail->q.x_type == F8_U8 ? 0x80808080u : 0u;
    }
    pp.x = static_cast<const uint8_t *>(x);
    pp.w = w;
    pp.acc0 = acc0;
    pp.res = static_cast<const uint8_t *>(res);
    pp.y = static_cast<uint8_t *>(y);
    pp.M = (long long)g.B * g.H * g.W;
    pp.shift = q.fl_x + q.fl_w - q.fl_y; pp.lo = q.clip_lo; pp.hi = q.clip_hi;
    pp.res_signed = q.res_type == F8_S8;
    pp.res_d = res ? q.fl_x + q.fl_w - q.fl_res : 0;
    pp.x_xor = q.x_type == F8_U8 ? 0x80808080u : 0u;
    return launch_pw_ws(pp, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
  }
  if (use_pw_wide(x, w, y, res, g, q, (q2 && y2) ? y2 : nullptr) && (reinterpret_cast<uintptr_t>(acc0) & 15) == 0) {
    PwWideParams pp;
    pp.x = static_cast<const uint8_t *>(x);
    pp.w = w;
    pp.acc0 = acc0;
    pp.res = static_cast<const uint8_t *>(res);
    pp.y = static_cast<uint8_t *>(y);
    pp.M = (long long)g.B * g.H * g.W;
    pp.K = g.Cin; pp.N = g.Cout;
    pp.shift = q.fl_x + q.fl_w - q.fl_y; pp.lo = q.clip_lo; pp.hi = q.clip_hi;
    pp.res_signed = q.res_type == F8_S8;
    pp.res_d = res ? q.fl_x + q.fl_w - q.fl_res : 0;
    pp.x_xor = q.x_type == F8_U8 ? 0x80808080u : 0u;
    return launch_pw_wide(pp, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
  }
  if (use_conv_ws(x, w, y, res, g, q, (q2 && y2) ? y2 : nullptr) && (reinterpret_cast<uintptr_t>(acc0) & 15) == 0) {
    ConvWsParams wp;
    wp.x = static_cast<const uint8_t *>(x);
    wp.w = w;
    wp.acc0 = acc0;
    wp.y = static_cast<uint8_t *>(y);
    wp.B = g.B; wp.H = g.H; wp.W = g.W; wp.C = g.Cin;
    wp.shift = q.fl_x + q.fl_w - q.fl_y; wp.lo = q.clip_lo; wp.hi = q.clip_hi;
    wp.x_xor = q.x_type == F8_U8 ? 0x80808080u : 0u;
    wp.tiles_per_image = wp.ntiles = wp.nrows = wp.pitch = wp.nchunks = 0;
    return launch_conv_ws(wp, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
  }
  ConvParams p;
  p.y2 = nullptr;
  p.shift2 = p.lo2 = p.hi2 = p.add2 = 0;
  if (q2 && y2) {
    p.y2 = y2;
    p.shift2 = q.fl_x + q.fl_w - q2->fl_y;
    p.lo2 = q2->clip_lo; p.hi2 = q2->clip_hi;
    p.add2 = (p.shift2 > 0 ? (1 << (p.shift2 - 1)) : 0) - rounding_addend(q);
  }
  p.zero = static_cast<const uint8_t *>(zero);
  {
    const uintptr_t xa = reinterpret_cast<uintptr_t>(x), za = reinterpret_cast<uintptr_t>(zero);
    const uintptr_t lo = xa < za ? xa : za;
    const unsigned long long xbytes = (unsigned long long)g.B * g.H * g.W * g.Cin;
    p.lo_base = reinterpret_cast<const uint8_t *>(lo);
    p.x_delta = (uint32_t)(xa - lo);
    p.z_delta = (uint32_t)(za - lo);
    p.near = (xa - lo) + xbytes + 64 < 0x7fffffffULL && (za - lo) + 64 < 0x7fffffffULL;
  }
  p.x = static_cast<const uint8_t *>(x);
  p.w = w;
  p.acc0 = acc0;
  p.y = y;
  p.res = res;
  p.B = g.B; p.H = g.H; p.W = g.W; p.C = g.Cin; p.N = g.Cout; p.R = g.R; p.S = g.S;
  p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.P = g.P; p.Q = g.Q;
  p.M = g.B * g.P * g.Q;
  p.K = g.R * g.S * g.Cin;
  p.xor_mask = q.x_type == F8_U8 ? 0x80808080u : 0u;
  p.shift = q.y_type == F8_S32 ? 0 : q.fl_x + q.fl_w - q.fl_y;
  p.lo = q.clip_lo; p.hi = q.clip_hi;
  p.y_type = q.y_type;
  p.res_type = q.res_type;
  p.res_d = q.fl_x + q.fl_w - q.fl_res;
  const int vec = widest_vec(g.Cin, x, w);
  p.fd_pq = FastDiv((uint32_t)(g.P * g.Q));
  p.fd_q = FastDiv((uint32_t)g.Q);
  p.fd_c = FastDiv((uint32_t)g.Cin);
  p.fd_cpt = FastDiv((uint32_t)((g.Cin & 63) == 0 ? g.Cin / 64 : 1));
  p.fd_cpt2 = FastDiv((uint32_t)((g.Cin & 127) == 0 ? g.Cin / 128 : 1));
  p.remap = tuning().xcd_remap.load(std::memory_order_relaxed) != 0;
  p.gemm = g.R == 1 && g.S == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0;
  p.fd_s = FastDiv((uint32_t)g.S);
  p.tap_rep = 0;
  if (g.R * g.S <= 32)
    for (int r = 0; r < g.R; ++r) p.tap_rep |= 1u << (r * g.S);
  if (p.M == 0 || p.N == 0) return F8_OK;
  if (conv_fast_applicable(p)) return launch_conv_fast(p, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
  return launch_conv_igemm(p, vec, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
}

bool conv_reads_narrow_rows(const Geom &g, const f8_quant &q, bool has_res) {
  return use_pw_small(nullptr, nullptr, nullptr, has_res ? &g : nullptr, g, q, nullptr);
}

bool conv_tail_ok(const Geom &g, const f8_quant &q, int Cout2) {
  if (g.Cin == 128) return Cout2 == 128 && use_pw_mid(nullptr, nullptr, nullptr, nullptr, g, q, nullptr, true);
  return (Cout2 == 64 || Cout2 == 128) && use_pw_ws(nullptr, nullptr, nullptr, nullptr, g, q, nullptr);
}

const char *conv_kernel_name(const Geom &g, const f8_quant &q, bool has_res) {
  if (use_pw_small(nullptr, nullptr, nullptr, has_res ? &g : nullptr, g, q, nullptr)) {
    if (g.Cout == 16) return "pw1x1_small<32x16>";
    if (g.Cout == 64) return "pw1x1_small<32x64>";
    static const char *const names[3][3] = {{"pw1x1_small<16x96>", "pw1x1_small<16x144>", "pw1x1_small<16x192>"},
                                            {"pw1x1_small<24x96>", "pw1x1_small<24x144>", "pw1x1_small<24x192>"},
                                            {"pw1x1_small<32x96>", "pw1x1_small<32x144>", "pw1x1_small<32x192>"}};
    return names[g.Cin == 16 ? 0 : (g.Cin == 24 ? 1 : 2)][g.Cout == 96 ? 0 : (g.Cout == 144 ? 1 : 2)];
  }
  if (!(has_res && q.res_type == F8_S32) && use_pw_ws(nullptr, nullptr, nullptr, nullptr, g, q, nullptr)) return "pw1x1_ws<64x256>";
  if (!(has_res && q.res_type == F8_S32) && use_pw_mid(nullptr, nullptr, nullptr, nullptr, g, q, nullptr, false)) return "pw1x1_mid<128x512>";
  if (!(has_res && q.res_type == F8_S32) && use_pw_wide(nullptr, nullptr, nullptr, nullptr, g, q, nullptr))
    return g.Cin == 256 ? "pw1x1_wide<256>" : "pw1x1_wide<512>";
  if (use_conv_ws(nullptr, nullptr, nullptr, has_res ? &g : nullptr, g, q, nullptr)) return g.Cin == 64 ? "conv3x3_ws<64x64>" : "conv3x3_ws<128x128>";
  ConvParams p;
  p.x = nullptr; p.w = nullptr; p.y = nullptr; p.res = has_res ? &p : nullptr;   // aligned stand-ins
  p.y2 = nullptr; p.shift2 = 0;
  p.near = 1;
  p.C = g.Cin; p.N = g.Cout; p.y_type = q.y_type; p.res_type = q.res_type;
  p.H = g.H; p.W = g.W; p.R = g.R; p.S = g.S; p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
  p.P = g.P; p.Q = g.Q;
  p.M = (g.B > 0 ? g.B : 1) * g.P * g.Q;
  p.K = g.R * g.S * g.Cin;
  if (conv_fast_applicable(p)) return conv_fast_variant_name(conv_fast_variant(p));
  return conv_variant_name(conv_variant(g.Cout));
}

f8_status enqueue_fold(const int8_t *w, const int32_t *bias, int32_t *acc0, const Geom &g,
                       const f8_quant &q, hipStream_t stream) {
  const int rc = launch_fold_acc0(w, bias, acc0, g.Cout, (int)acc0_padded(g.Cout), g.R * g.S * g.Cin,
                                  q.x_type == F8_U8, rounding_addend(q), stream);
  return rc == 0 ? F8_OK : F8_ERR_DEVICE;
}

static DwParams dw_params(const void *x, const int8_t *w, const int32_t *bias, void *y, const void *res,
                          const Geom &g, const f8_quant &q) {
  DwParams p;
  p.x = static_cast<const uint8_t *>(x);
  p.w = w; p.bias = bias; p.y = y; p.res = res;
  p.B = g.B; p.H = g.H; p.W = g.W; p.C = g.Cin; p.R = g.R; p.S = g.S;
  p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.P = g.P; p.Q = g.Q;
  p.x_type = q.x_type; p.y_type = q.y_type; p.res_type = q.res_type;
  p.res_d = q.fl_x + q.fl_w - q.fl_res;
  p.shift = q.y_type == F8_S32 ? 0 : q.fl_x + q.fl_w - q.fl_y;
  p.rnd = rounding_addend(q);
  p.lo = q.clip_lo; p.hi = q.clip_hi;
  return p;
}

f8_status enqueue_dwconv(const void *x, const int8_t *w, const int32_t *bias, void *y, const void *res,
                         const Geom &g, const f8_quant &q, hipStream_t stream) {
  const DwParams p = dw_params(x, w, bias, y, res, g, q);
  uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) |
                   reinterpret_cast<uintptr_t>(y) | (uintptr_t)g.Cin;
  if (res && q.res_type != F8_S32) bits |= reinterpret_cast<uintptr_t>(res);
  return launch_dwconv(p, (bits & 3) == 0, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
}

f8_status enqueue_maxpool(const void *x, void *y, const Geom &g, int dtype, hipStream_t stream) {
  PoolParams p;
  p.x = static_cast<const uint8_t *>(x);
  p.y = static_cast<uint8_t *>(y);
  p.B = g.B; p.H = g.H; p.W = g.W; p.C = g.Cin; p.R = g.R; p.S = g.S;
  p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.P = g.P; p.Q = g.Q;
  p.type = dtype;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) | (uintptr_t)g.Cin;
  return launch_maxpool(p, (bits & 3) == 0, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
}

f8_status enqueue_gpool(const void *x, void *y, const Geom &g, const f8_quant &q, hipStream_t stream) {
  const DwParams p = dw_params(x, nullptr, nullptr, y, nullptr, g, q);
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) | (uintptr_t)g.Cin;
  return launch_gpool(p, (bits & 3) == 0, stream) == 0 ? F8_OK : F8_ERR_DEVICE;
}

// ---- per-stream scratch for the folded accumulator start values ------------------------
namespace {
struct Scratch { int32_t *ptr; size_t ints; };
// Held from the look-up of a stream's buffer until both kernels of the call (the fold that
// writes the buffer and the layer that reads it) are enqueued, so that two host threads
// calling on one stream cannot interleave their folds and layers.
std::mutex g_mu;
std::unordered_map<uint64_t, Scratch> g_scratch;   // key: device id, stream handle

// Caller holds g_mu.
int32_t *scratch_for(hipStream_t stream, size_t ints) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return nullptr;
  const uint64_t key = (reinterpret_cast<uint64_t>(stream) << 4) ^ (uint64_t)dev;
  Scratch &s = g_scratch[key];
  if (s.ints < ints) {
    // Growing: work already queued on this stream may still read the old buffer.
    if (s.ptr) {
      if (hipStreamSynchronize(stream) != hipSuccess) return nullptr;
      (void)hipFree(s.ptr);
      s.ptr = nullptr; s.ints = 0;
    }
    size_t want = ints < 16384 ? 16384 : ints;
    if (hipMalloc(reinterpret_cast<void **>(&s.ptr), want * sizeof(int32_t)) != hipSuccess) {
      s.ptr = nullptr;
      return nullptr;
    }
    // the first 64 ints stay zero for the life of the buffer (the kernels' page of zeros)
    if (hipMemset(s.ptr, 0, 64 * sizeof(int32_t)) != hipSuccess) {
      (void)hipFree(s.ptr);
      s.ptr = nullptr;
      return nullptr;
    }
    s.ints = want;
  }
  return s.ptr;
}

// Fold + layer of one single-layer dense call on the stream's own scratch.
f8_status dense_on_stream_scratch(const void *x, const int8_t *w, const int32_t *bias, void *y, const Geom &g,
                                  const f8_quant &q, hipStream_t s, const f8_requant2 *q2, void *y2) {
  std::lock_guard<std::mutex> lock(g_mu);
  int32_t *scratch = scratch_for(s, 64 + acc0_padded(g.Cout));
  if (!scratch) return F8_ERR_DEVICE;
  int32_t *acc0 = scratch + 64;
  const f8_status st = enqueue_fold(w, bias, acc0, g, q, s);
  if (st != F8_OK) return st;
  return enqueue_conv(x, w, acc0, scratch, y, q.res, g, q, s, q2, y2);
}

// ---- scratch of the entry point that allocates nothing ----------------------------------
// 64 ints that are never written (static storage starts as zeros: the kernels' page of zeros)
// followed by the folded start values of one call.  Every device the library's code object is
// loaded on holds its own copy at its own address; host code uses the per-device address from
// hipGetSymbolAddress, never the array's name.
constexpr int kStaticMaxCout = F8_NOALLOC_MAX_COUT;
__device__ __align__(256) int32_t scratch[64 + kStaticMaxCout];

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
int32_t *g_static_ptr[kMaxDevices] = {};

// Address of this device's copy of `scratch` (looked up once per device, with that device current).
int32_t *static_scratch() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_static_ptr[dev] = static_cast<int32_t *>(ptr);
  }
  return g_static_ptr[dev];
}
}  // namespace

}  // namespace f8

using namespace f8;

extern "C" {

f8_status f8_conv2d_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y, int B, int H, int W,
                          int Cin, int Cout, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                          const f8_quant *q, void *stream) {
  if (!x || !w || !y) return F8_ERR_NULL;
  f8_status st = check_quant(q, true);
  if (st != F8_OK) return st;
  Geom g{B, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, 0, 0};
  st = check_geom(g, false);
  if (st != F8_OK) return st;
  st = check_align(bias, y, *q, q->res);
  if (st != F8_OK) return st;
  if (q->res == y) return F8_ERR_UNSUPPORTED;
  if ((long long)g.B * g.P * g.Q * g.Cout == 0) return F8_OK;
  return dense_on_stream_scratch(x, w, bias, y, g, *q, static_cast<hipStream_t>(stream), nullptr, nullptr);
}

size_t f8_conv_workspace_bytes(int Cout) { return Cout < 0 ? 0 : (64 + acc0_padded(Cout)) * sizeof(int32_t); }

f8_status f8_conv2d_fixed_ws(const void *x, const int8_t *w, const int32_t *bias, void *y, int B, int H, int W, int Cin,
                             int Cout, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w, const f8_quant *q,
                             void *workspace, size_t workspace_bytes, void *stream) {
  if (!x || !w || !y || !workspace) return F8_ERR_NULL;
  f8_status st = check_quant(q, true);
  if (st != F8_OK) return st;
  Geom g{B, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, 0, 0};
  st = check_geom(g, false);
  if (st != F8_OK) return st;
  st = check_align(bias, y, *q, q->res);
  if (st != F8_OK) return st;
  if (q->res == y) return F8_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return F8_ERR_ALIGN;
  if (workspace_bytes < f8_conv_workspace_bytes(Cout)) return F8_ERR_SHAPE;
  if ((long long)g.B * g.P * g.Q * g.Cout == 0) return F8_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the first 256 bytes are the kernels' page of zeros (cleared by a kernel, so the call can be captured),
  // the folded start values follow
  int32_t *base = static_cast<int32_t *>(workspace);
  if (launch_fold_acc0(nullptr, nullptr, base, 0, 64, 0, 0, 0, s) != 0) return F8_ERR_DEVICE;
  int32_t *acc0 = base + 64;
  st = enqueue_fold(w, bias, acc0, g, *q, s);
  if (st != F8_OK) return st;
  return enqueue_conv(x, w, acc0, base, y, q->res, g, *q, s);
}

f8_status f8_conv2d_fixed_noalloc(const void *x, const int8_t *w, const int32_t *bias, void *y, int B, int H, int W,
                                  int Cin, int Cout, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                                  const f8_quant *q, void *stream) {
  if (!x || !w || !y) return F8_ERR_NULL;
  f8_status st = check_quant(q, true);
  if (st != F8_OK) return st;
  Geom g{B, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, 0, 0};
  st = check_geom(g, false);
  if (st != F8_OK) return st;
  st = check_align(bias, y, *q, q->res);
  if (st != F8_OK) return st;
  if (q->res == y) return F8_ERR_UNSUPPORTED;
  if (Cout > kStaticMaxCout || acc0_padded(Cout) > (size_t)kStaticMaxCout) return F8_ERR_UNSUPPORTED;
  if ((long long)g.B * g.P * g.Q * g.Cout == 0) return F8_OK;
  int32_t *base = static_scratch();
  if (!base) return F8_ERR_DEVICE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t *acc0 = base + 64;
  st = enqueue_fold(w, bias, acc0, g, *q, s);
  if (st != F8_OK) return st;
  return enqueue_conv(x, w, acc0, base, y, q->res, g, *q, s);
}

f8_status f8_conv2d_fixed_dual(const void *x, const int8_t *w, const int32_t *bias, void *y, void *y2, int B, int H,
                               int W, int Cin, int Cout, int R, int S, int stride_h, int stride_w, int pad_h,
                               int pad_w, const f8_quant *q, const f8_requant2 *q2, void *stream) {
  if (!x || !w || !y || !y2) return F8_ERR_NULL;
  f8_status st = check_quant(q, true);
  if (st != F8_OK) return st;
  st = check_requant2(*q, q2);
  if (st != F8_OK) return st;
  Geom g{B, H, W, Cin, Cout, R, S, stride_h, stride_w, pad_h, pad_w, 0, 0};
  st = check_geom(g, false);
  if (st != F8_OK) return st;
  st = check_align(bias, y, *q, q->res);
  if (st != F8_OK) return st;
  if (q->res == y || q->res == y2 || y == y2) return F8_ERR_UNSUPPORTED;
  if ((long long)g.B * g.P * g.Q * g.Cout == 0) return F8_OK;
  return dense_on_stream_scratch(x, w, bias, y, g, *q, static_cast<hipStream_t>(stream), q2, y2);
}

f8_status f8_gemm_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y, int M, int K, int N,
                        const f8_quant *q, void *stream) {
  if (M < 0 || K < 1 || N < 0) return (x && w && y) ? F8_ERR_SHAPE : F8_ERR_NULL;
  // A GEMM is the 1x1 convolution of a 1 x M image with K channels.
  return f8_conv2d_fixed(x, w, bias, y, 1, 1, M > 0 ? M : 1, K, M > 0 ? N : 0, 1, 1, 1, 1, 0, 0, q, stream);
}

f8_status f8_dwconv_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y, int B, int H, int W,
                          int C, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w,
                          const f8_quant *q, void *stream) {
  if (!x || !w || !y) return F8_ERR_NULL;
  f8_status st = check_quant(q, true);
  if (st != F8_OK) return st;
  Geom g{B, H, W, C, C, R, S, stride_h, stride_w, pad_h, pad_w, 0, 0};
  st = check_geom(g, true);
  if (st != F8_OK) return st;
  st = check_align(bias, y, *q, q->res);
  if (st != F8_OK) return st;
  if (q->res == y) return F8_ERR_UNSUPPORTED;
  if ((long long)g.B * g.P * g.Q * g.Cout == 0) return F8_OK;
  return enqueue_dwconv(x, w, bias, y, q->res, g, *q, static_cast<hipStream_t>(stream));
}

f8_status f8_maxpool(const void *x, void *y, int B, int H, int W, int C, int R, int S, int stride_h,
                     int stride_w, int pad_h, int pad_w, int dtype, void *stream) {
  if (!x || !y) return F8_ERR_NULL;
  if (dtype != F8_U8 && dtype != F8_S8) return F8_ERR_DTYPE;
  Geom g{B, H, W, C, C, R, S, stride_h, stride_w, pad_h, pad_w, 0, 0};
  f8_status st = check_geom(g, true);
  if (st != F8_OK) return st;
  if (pad_h >= R || pad_w >= S) return F8_ERR_SHAPE;
  if ((long long)g.B * g.P * g.Q * g.Cout == 0) return F8_OK;
  return enqueue_maxpool(x, y, g, dtype, static_cast<hipStream_t>(stream));
}

f8_status f8_global_pool_fixed(const void *x, void *y, int B, int H, int W, int C, const f8_quant *q,
                               void *stream) {
  if (!x || !y) return F8_ERR_NULL;
  f8_status st = check_quant(q, false);
  if (st != F8_OK) return st;
  if (B < 0 || H < 1 || W < 1 || C < 1 || (long long)H * W > 65536) return F8_ERR_SHAPE;
  Geom g{B, H, W, C, C, H, W, 1, 1, 0, 0, 1, 1};
  if ((long long)B * H * W * C > 0x7fffffffLL) return F8_ERR_UNSUPPORTED;
  st = check_align(nullptr, y, *q, nullptr);
  if (st != F8_OK) return st;
  if (B == 0) return F8_OK;
  return enqueue_gpool(x, y, g, *q, static_cast<hipStream_t>(stream));
}

int32_t f8_clip_from_alpha(double alpha, int fl_y, int is_signed) {
  const int top = is_signed ? 127 : 255;
  if (!(alpha > 0.0)) return 0;
  double v = alpha;
  for (int i = 0; i < fl_y; ++i) v *= 2.0;
  for (int i = 0; i > fl_y; --i) v *= 0.5;
  if (v >= (double)top) return top;
  const int32_t r = (int32_t)(v + 0.5);    // v >= 0: truncation of v + 1/2 is round half up
  return r > top ? top : r;
}

const char *f8_status_str(f8_status s) {
  switch (s) {
    case F8_OK: return "ok";
    case F8_ERR_NULL: return "null pointer";
    case F8_ERR_SHAPE: return "bad shape";
    case F8_ERR_FL: return "fractional lengths give a shift outside the supported range";
    case F8_ERR_CLIP: return "clip bounds outside the output type's range";
    case F8_ERR_DTYPE: return "type code not allowed for this operand";
    case F8_ERR_ACC_OVERFLOW: return "accumulator overflow";
    case F8_ERR_ALIGN: return "int32 operand is not 4-byte aligned";
    case F8_ERR_UNSUPPORTED: return "unsupported configuration";
    case F8_ERR_DEVICE: return "HIP runtime error";
    case F8_ERR_STATE: return "chain not prepared for this workspace";
  }
  return "unknown status";
}

void f8_release_scratch(void) {
  std::lock_guard<std::mutex> lock(g_mu);
  for (auto &kv : g_scratch)
    if (kv.second.ptr) (void)hipFree(kv.second.ptr);
  g_scratch.clear();
}

f8_status f8_copy_bytes(const void *src, void *dst, size_t bytes, void *stream) {
  if (!src || !dst) return F8_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst) | bytes) & 15) return F8_ERR_ALIGN;
  return launch_copy(src, dst, bytes, static_cast<hipStream_t>(stream)) == 0 ? F8_OK : F8_ERR_DEVICE;
}

int f8_tuning_set(const char *name, int value) {
  if (!name) return -1;
  for (const TuningName &k : kTuningNames)
    if (strcmp(name, k.name) == 0) {
      (tuning().*(k.field)).store(value);
      return 0;
    }
  return -1;
}

int f8_tuning_get(const char *name) {
  if (!name) return -1;
  for (const TuningName &k : kTuningNames)
    if (strcmp(name, k.name) == 0) return (tuning().*(k.field)).load();
  return -1;
}

int f8_abi_version(void) { return 3; }

}  // extern "C"
