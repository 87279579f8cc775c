// Layer-chain runner: a whole fixed-point network forward as a fixed sequence of launches.
//
// The chain owns only host-side book-keeping.  Activations and the per-layer constants
// live in a caller-provided device workspace whose layout is
//   [ constants: acc0 vector (and re-laid-out stem weights) of every dense layer ][ arena ]
// Every tensor's size is linear in the batch, so the arena is planned once per image
// (first-fit over tensor lifetimes, offsets in multiples of 256 bytes) and scaled by the
// batch at run time.
//
// Stem re-layout.  A dense layer with at most 4 input channels (the 7x7/2 ImageNet stem)
// is run on a re-laid-out copy of its operands: the input gets an explicit zero border
// and 4 channels, each window row is padded to a multiple of 4 taps with zero weights.
// The sums are unchanged (only zero products are added), windows are never clipped, and
// 16 contiguous bytes hold four whole taps, which is what the fast kernel's loads need.
// A dense layer whose input channel count is above 4 and not a multiple of 16 (24 in the
// first MobileNetV2 blocks) is run on a copy of its input and weights with the channels
// padded with zeros to the next multiple of 16, for the same reason.
//
// Stem + pool.  The ImageNet stem (7x7 stride-2 convolution of a 3-channel image to 64 unsigned
// channels) followed by a 3x3 stride-2 pad-1 max pool that is its only reader runs as one kernel
// on the re-laid-out operands; the tensor between the two then gets no memory.  (Not when every
// tensor is to be kept; F8_STEM_POOL=0, read when the chain is created, turns it off: tuning aid.)
//
// Block fusion.  Three consecutive layers that form an inverted-residual block (1x1 dense,
// 3x3 depthwise stride 1 pad 1, 1x1 dense, optional shortcut from the block input) whose two
// intermediate tensors have no other reader run as one kernel that keeps the intermediates on
// chip; those tensors then get no memory.  Opt-in (f8_chain_set_fusion(c, 1)): measured on
// MI355X it beats the three kernels on a single block at batch 64 but not on whole MobileNetV2
// forwards, where it is bound by the vector ALU and, late in the network, by too few tiles.
// Never used with keep_all (every tensor inspectable).
#include <algorithm>
#include <new>
#include <vector>

#include "block_fused.h"
#include "stem_pool.h"
#include "conv_img.h"
#include "f8_host.h"

using namespace f8;

namespace {

struct Tensor {
  int h = 0, w = 0, c = 0;
  int type = -1;
  int fl = 0;
  bool fl_known = false;
  int producer = -2;        // -2: not defined, -1: network input, else layer index
  int last_use = -1;        // last layer index that reads it
  size_t bytes_per_image = 0;
  size_t offset_per_image = 0;
  bool external = false;    // input x or final output
};

struct Stem {
  bool on = false;
  int Cp = 4;                       // channels after the re-layout: 4 (stem) or a multiple of 16
  int Sp = 0, Hp = 0, Wp = 0;       // stem: padded window width, padded image extent
  size_t w_off = 0;                 // re-laid-out weights: byte offset in the constants region
  size_t x_off_per_image = 0;       // re-laid-out input: arena offset per image
  size_t x_bytes_per_image = 0;
  int pool = 0;                     // 1: this layer also does the max pool that follows; 2: that (absorbed) pool
};

// Role of a layer in a fused block, and where the block's re-laid-out constants live.
struct Fused {
  int role = 0;                     // 0 ordinary layer, 1 first layer of a fused block, 2 absorbed
  int K1 = 0, CH = 0, NB2 = 0;
  size_t w1p = 0, w2p = 0, wdp = 0, acc1 = 0, accd = 0, acc2 = 0;   // byte offsets in the constants region
};

size_t elem_size(int type) { return type == F8_S32 ? 4 : 1; }
size_t round256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

struct f8_chain {
  std::vector<f8_layer_desc> layers;
  std::vector<Geom> geom;              // per layer, B filled at run time
  std::vector<Stem> stem;              // per layer
  std::vector<Fused> fused;            // per layer
  bool fusion = false;
  bool use_fusion() const { return fusion && !keep_all; }
  bool stem_pool = true;
  int pool_role(size_t i) const { return stem_pool && !keep_all ? stem[i].pool : 0; }
  // A dense layer and the 1x1 layer that reads its output in one launch: tail[i] = 1 for the first,
  // 2 for the 1x1 layer behind it, tail_peer[i] = the other layer of the pair (candidates; both
  // tensors are still written).  Whether the kernel that can do this is chosen depends on the batch.
  std::vector<int> tail, tail_peer;    // per layer
  bool conv_tail = true;
  // 3x3 layers the image-stationary kernel can take: byte offset of their weights in fragment order
  // in the constants region (0: not such a layer).
  std::vector<size_t> img_w_off;       // per layer
  bool conv_img = true;
  int conv_img_min = 96;
  bool img_role(size_t i, int batch) const {
    return conv_img && img_w_off[i] != 0 && !(use_fusion() && fused[i].role != 0) &&
           conv_img_units(layers[i].Cin, batch, geom[i].H) >= conv_img_min;
  }
  bool tail_in_fused_block(size_t i) const {
    const size_t a = tail[i] == 1 ? i : (size_t)tail_peer[i], b = tail[i] == 1 ? (size_t)tail_peer[i] : i;
    return use_fusion() && (fused[a].role != 0 || fused[b].role != 0);
  }
  int tail_role(size_t i, int batch) const {
    if (!conv_tail || tail[i] == 0 || tail_in_fused_block(i)) return 0;
    const size_t head = tail[i] == 1 ? i : (size_t)tail_peer[i], behind = tail[i] == 1 ? (size_t)tail_peer[i] : i;
    Geom g = geom[head];
    g.B = batch;
    return conv_tail_ok(g, layers[head].q, layers[behind].Cout) ? tail[i] : 0;
  }
  std::vector<Tensor> tensors;
  std::vector<size_t> acc0_off;        // per layer: byte offset in the constants region
  size_t const_bytes = 0;
  size_t arena_per_image = 0;
  bool keep_all = false;
  bool planned = false;
  int last_tensor = 0;
  void *prepared_ws = nullptr;
  int prepared_batch = -1;

  void plan() {
    struct Block { size_t off, size; };
    std::vector<Block> free_list;      // sorted by offset
    size_t top = 0;
    auto alloc = [&](size_t size) -> size_t {
      for (size_t i = 0; i < free_list.size(); ++i) {
        if (free_list[i].size >= size) {
          const size_t off = free_list[i].off;
          free_list[i].off += size;
          free_list[i].size -= size;
          if (free_list[i].size == 0) free_list.erase(free_list.begin() + i);
          return off;
        }
      }
      // extend the arena, reusing a free tail if there is one
      if (!free_list.empty() && free_list.back().off + free_list.back().size == top) {
        const size_t off = free_list.back().off;
        free_list.pop_back();
        top = off + size;
        return off;
      }
      const size_t off = top;
      top += size;
      return off;
    };
    auto release = [&](size_t off, size_t size) {
      Block b{off, size};
      auto it = std::lower_bound(free_list.begin(), free_list.end(), b,
                                 [](const Block &a, const Block &c) { return a.off < c.off; });
      it = free_list.insert(it, b);
      const size_t i = it - free_list.begin();
      if (i + 1 < free_list.size() && free_list[i].off + free_list[i].size == free_list[i + 1].off) {
        free_list[i].size += free_list[i + 1].size;
        free_list.erase(free_list.begin() + i + 1);
      }
      if (i > 0 && free_list[i - 1].off + free_list[i - 1].size == free_list[i].off) {
        free_list[i - 1].size += free_list[i].size;
        free_list.erase(free_list.begin() + i);
      }
    };
    // tail candidates as the planner sees them: any batch, but not inside a fused block
    auto tail_plan = [&](size_t li) { return tail[li] == 0 || tail_in_fused_block(li) ? 0 : tail[li]; };
    for (size_t li = 0; li < layers.size(); ++li) {
      if (pool_role(li) == 2) continue;
      if (pool_role(li) == 1) {
        // one kernel: re-laid-out input in, the pool's output out
        stem[li].x_off_per_image = alloc(round256(stem[li].x_bytes_per_image));
        Tensor &d = tensors[layers[li + 1].dst];
        if (!d.external) d.offset_per_image = alloc(round256(d.bytes_per_image));
        release(stem[li].x_off_per_image, round256(stem[li].x_bytes_per_image));
        Tensor &t = tensors[layers[li].src];
        if (!t.external && t.last_use == (int)li) release(t.offset_per_image, round256(t.bytes_per_image));
        continue;
      }
      if (use_fusion() && fused[li].role == 2) continue;
      if (use_fusion() && fused[li].role == 1) {
        // one kernel: reads the block input, writes the third layer's output
        Tensor &d = tensors[layers[li + 2].dst];
        if (!d.external) d.offset_per_image = alloc(round256(d.bytes_per_image));
        Tensor &t = tensors[layers[li].src];
        if (!t.external && t.last_use <= (int)li + 2) release(t.offset_per_image, round256(t.bytes_per_image));
        continue;
      }
      if (stem[li].on) stem[li].x_off_per_image = alloc(round256(stem[li].x_bytes_per_image));
      Tensor &d = tensors[layers[li].dst];
      // (the output of a 1x1 layer that may run inside the previous launch got its place there)
      if (!d.external && tail_plan(li) != 2) d.offset_per_image = alloc(round256(d.bytes_per_image));
      if (tail_plan(li) == 1) {
        // written by this launch too: must not share memory with what this layer reads
        Tensor &dt = tensors[layers[tail_peer[li]].dst];
        if (!dt.external) dt.offset_per_image = alloc(round256(dt.bytes_per_image));
      }
      if (layers[li].dst2 > 0) {
        Tensor &d2 = tensors[layers[li].dst2];
        d2.offset_per_image = alloc(round256(d2.bytes_per_image));
        // never read: give the space back once this layer has run
        if (!keep_all && d2.last_use < 0) release(d2.offset_per_image, round256(d2.bytes_per_image));
      }
      if (keep_all) continue;
      if (stem[li].on) release(stem[li].x_off_per_image, round256(stem[li].x_bytes_per_image));
      const int ids[2] = {layers[li].src, layers[li].res};
      for (int k = 0; k < 2; ++k) {
        if (ids[k] < 0) continue;
        if (k == 1 && ids[1] == ids[0]) continue;
        Tensor &t = tensors[ids[k]];
        if (!t.external && t.last_use == (int)li) release(t.offset_per_image, round256(t.bytes_per_image));
      }
    }
    arena_per_image = top;
    planned = true;
  }

  // Two halves of a batch can run side by side (f8_chain_set_streams): the second half's tensors lie
  // behind the first half's, arena_shift bytes into the arena, while its layers are enqueued.
  size_t arena_shift = 0;
  int n_streams = 1;
  hipStream_t side_stream = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  uint8_t *arena(void *workspace) const { return static_cast<uint8_t *>(workspace) + const_bytes + arena_shift; }

  void *tensor_ptr(int id, const void *x, void *out, void *workspace, int batch) const {
    if (id == 0) return const_cast<void *>(x);
    if (id == last_tensor) return out;
    return arena(workspace) + tensors[id].offset_per_image * (size_t)batch;
  }

  // Geometry and operands of dense layer i as the kernel sees them (after the stem re-layout).
  Geom conv_geom(size_t i, int batch) const {
    Geom g = geom[i];
    g.B = batch;
    if (stem[i].on && stem[i].Cp == 4) {
      g.H = stem[i].Hp; g.W = stem[i].Wp; g.Cin = 4; g.S = stem[i].Sp; g.ph = 0; g.pw = 0;
    } else if (stem[i].on) {
      g.Cin = stem[i].Cp;
    }
    return g;
  }
  const int8_t *conv_weights(size_t i, void *workspace) const {
    if (!stem[i].on) return layers[i].w;
    return reinterpret_cast<const int8_t *>(static_cast<uint8_t *>(workspace) + stem[i].w_off);
  }

  // A dense layer whose channel count is not a multiple of 16 normally runs on a zero-padded copy;
  // not when the kernel for few input channels takes it at this batch (its weights 16-byte aligned,
  // its tensors in the arena).
  bool narrow_rows(size_t i, int batch) const {
    const f8_layer_desc &L = layers[i];
    if (!stem[i].on || stem[i].Cp == 4 || L.op != F8_OP_CONV || L.dst2 > 0 || (reinterpret_cast<uintptr_t>(L.w) & 15)) return false;
    if (tensors[L.src].external || tensors[L.dst].external) return false;
    Geom g = geom[i];
    g.B = batch;
    return conv_reads_narrow_rows(g, L.q, L.res >= 0);
  }

  // Parameters of the fused block that starts at layer i.
  BlockParams block_params(size_t i, const void *x, void *out, void *workspace, int batch) const {
    const f8_layer_desc &L0 = layers[i], &L1 = layers[i + 1], &L2 = layers[i + 2];
    const Fused &f = fused[i];
    uint8_t *cb = static_cast<uint8_t *>(workspace);
    BlockParams p;
    p.x = static_cast<const uint8_t *>(tensor_ptr(L0.src, x, out, workspace, batch));
    p.y = tensor_ptr(L2.dst, x, out, workspace, batch);
    p.w1p = reinterpret_cast<const int8_t *>(cb + f.w1p);
    p.w2p = reinterpret_cast<const int8_t *>(cb + f.w2p);
    p.wdp = reinterpret_cast<const int8_t *>(cb + f.wdp);
    p.acc1 = reinterpret_cast<const int32_t *>(cb + f.acc1);
    p.accd = reinterpret_cast<const int32_t *>(cb + f.accd);
    p.acc2 = reinterpret_cast<const int32_t *>(cb + f.acc2);
    p.B = batch; p.H = geom[i].H; p.W = geom[i].W;
    p.Cin = L0.Cin; p.Ce = L0.Cout; p.Cout = L2.Cout;
    p.K1 = f.K1; p.CH = f.CH; p.NB2 = f.NB2;
    block_fused_tiling(p);
    p.x_xor = L0.q.x_type == F8_U8 ? 0x80808080u : 0u;
    const int eb = L0.q.y_type == F8_U8 ? 128 : 0, db = L1.q.y_type == F8_U8 ? 128 : 0;
    p.sh1 = L0.q.fl_x + L0.q.fl_w - L0.q.fl_y; p.lo1 = L0.q.clip_lo - eb; p.hi1 = L0.q.clip_hi - eb;
    p.e_zero = eb ? 0x80808080u : 0u;
    p.shd = L1.q.fl_x + L1.q.fl_w - L1.q.fl_y; p.lod = L1.q.clip_lo - db; p.hid = L1.q.clip_hi - db;
    p.sh2 = L2.q.fl_x + L2.q.fl_w - L2.q.fl_y; p.lo2 = L2.q.clip_lo; p.hi2 = L2.q.clip_hi;
    p.has_res = L2.res >= 0;
    p.res_signed = L2.q.res_type == F8_S8;
    p.res_d = L2.q.fl_x + L2.q.fl_w - L2.q.fl_res;
    return p;
  }

  f8_status launch_layer(size_t i, const void *x, void *out, void *workspace, int batch, hipStream_t s) const {
    const f8_layer_desc &L = layers[i];
    Geom g = geom[i];
    g.B = batch;
    if (pool_role(i) == 2) return F8_OK;
    if (pool_role(i) == 1) {
      const void *src = tensor_ptr(L.src, x, out, workspace, batch);
      void *xp = arena(workspace) + stem[i].x_off_per_image * (size_t)batch;
      if (launch_pad_input(src, xp, batch, g.H, g.W, g.Cin, stem[i].Hp, stem[i].Wp, g.ph, g.pw, s,
                           L.q.x_type == F8_U8 ? 0x80808080u : 0u) != 0)
        return F8_ERR_DEVICE;
      StemPoolParams sp;
      sp.xp = static_cast<const uint8_t *>(xp);
      sp.wp = conv_weights(i, workspace);
      sp.acc0 = reinterpret_cast<const int32_t *>(static_cast<uint8_t *>(workspace) + acc0_off[i]);
      sp.y = static_cast<uint8_t *>(tensor_ptr(layers[i + 1].dst, x, out, workspace, batch));
      sp.B = batch; sp.Hp = stem[i].Hp; sp.Wp = stem[i].Wp;
      sp.P = g.P; sp.Q = g.Q; sp.PP = geom[i + 1].P; sp.QP = geom[i + 1].Q;
      sp.shift = L.q.fl_x + L.q.fl_w - L.q.fl_y; sp.lo = L.q.clip_lo; sp.hi = L.q.clip_hi;
      sp.ntiles = 0;
      return launch_stem_pool(sp, s) == 0 ? F8_OK : F8_ERR_DEVICE;
    }
    if (use_fusion() && fused[i].role == 2) return F8_OK;
    if (use_fusion() && fused[i].role == 1) {
      const BlockParams bp = block_params(i, x, out, workspace, batch);
      return launch_block_fused(bp, s) == 0 ? F8_OK : F8_ERR_DEVICE;
    }
    if (tail_role(i, batch) == 2) return F8_OK;
    const void *src = tensor_ptr(L.src, x, out, workspace, batch);
    void *dst = tensor_ptr(L.dst, x, out, workspace, batch);
    const void *res = L.res >= 0 ? tensor_ptr(L.res, x, out, workspace, batch) : nullptr;
    switch (L.op) {
      case F8_OP_CONV: {
        const int32_t *acc0 = reinterpret_cast<const int32_t *>(static_cast<uint8_t *>(workspace) + acc0_off[i]);
        if (img_role(i, batch) && conv_img_applicable(L.Cin, L.Cout, L.R, L.S, L.stride_h, L.stride_w, L.pad_h, L.pad_w, g.H, g.W,
                                               L.q.fl_x + L.q.fl_w - L.q.fl_y, src, dst)) {
          ConvImgParams ip;
          ip.x = static_cast<const uint8_t *>(src);
          ip.wf = reinterpret_cast<const int8_t *>(static_cast<uint8_t *>(workspace) + img_w_off[i]);
          ip.acc0 = acc0;
          ip.y = static_cast<uint8_t *>(dst);
          ip.B = batch; ip.H = g.H; ip.W = g.W; ip.C = L.Cin;
          ip.shift = L.q.fl_x + L.q.fl_w - L.q.fl_y; ip.lo = L.q.clip_lo; ip.hi = L.q.clip_hi;
          ip.x_xor = L.q.x_type == F8_U8 ? 0x80808080u : 0u;
          return launch_conv_img(ip, s) == 0 ? F8_OK : F8_ERR_DEVICE;
        }
        if (narrow_rows(i, batch)) {
          // the kernel for few input channels reads the 24-channel rows and weights as they are
          return enqueue_conv(src, L.w, acc0, workspace, dst, res, g, L.q, s);
        }
        if (stem[i].on) {
          void *xp = arena(workspace) + stem[i].x_off_per_image * (size_t)batch;
          const int e = stem[i].Cp == 4
                            ? launch_pad_input(src, xp, batch, g.H, g.W, g.Cin, stem[i].Hp, stem[i].Wp, g.ph, g.pw, s)
                            : launch_pad_rows(src, xp, (long long)batch * g.H * g.W, g.Cin, stem[i].Cp, s);
          if (e != 0) return F8_ERR_DEVICE;
          src = xp;
        }
        void *dst2 = L.dst2 > 0 ? tensor_ptr(L.dst2, x, out, workspace, batch) : nullptr;
        ConvTail ct;
        const bool with_tail = tail_role(i, batch) == 1;
        if (with_tail) {
          const f8_layer_desc &T = layers[tail_peer[i]];
          ct.w = T.w;
          ct.acc0 = reinterpret_cast<const int32_t *>(static_cast<uint8_t *>(workspace) + acc0_off[tail_peer[i]]);
          ct.y = tensor_ptr(T.dst, x, out, workspace, batch);
          ct.Cout = T.Cout;
          ct.q = T.q;
        }
        return enqueue_conv(src, conv_weights(i, workspace), acc0, workspace, dst, res, conv_geom(i, batch), L.q, s,
                            dst2 ? &L.q2 : nullptr, dst2, with_tail ? &ct : nullptr);
      }
      case F8_OP_DWCONV: return enqueue_dwconv(src, L.w, L.bias, dst, res, g, L.q, s);
      case F8_OP_MAXPOOL: return enqueue_maxpool(src, dst, g, L.q.x_type, s);
      default: return enqueue_gpool(src, dst, g, L.q, s);
    }
  }
};

extern "C" {

f8_status f8_chain_create(const f8_layer_desc *layers, int n_layers, int in_h, int in_w, int in_c,
                          int in_type, f8_chain **out) {
  if (!layers || !out) return F8_ERR_NULL;
  *out = nullptr;
  if (n_layers < 1 || in_h < 1 || in_w < 1 || in_c < 1) return F8_ERR_SHAPE;
  if (in_type != F8_U8 && in_type != F8_S8) return F8_ERR_DTYPE;
  f8_chain *c = new (std::nothrow) f8_chain();
  if (!c) return F8_ERR_DEVICE;
  f8_status st = F8_OK;
  int max_id = 0;
  for (int i = 0; i < n_layers; ++i) {
    if (layers[i].dst < 1 || layers[i].src < 0 || layers[i].res < -1) { st = F8_ERR_SHAPE; break; }
    max_id = std::max(max_id, std::max(layers[i].dst, std::max(layers[i].src, layers[i].res)));
    max_id = std::max(max_id, (int)layers[i].dst2);
  }
  if (st == F8_OK && max_id > 16 * n_layers + 16) st = F8_ERR_SHAPE;
  if (st != F8_OK) { delete c; return st; }
  c->const_bytes = 256;                // the workspace starts with a block of zeros
  c->tensors.resize(max_id + 1);
  Tensor &t0 = c->tensors[0];
  t0.h = in_h; t0.w = in_w; t0.c = in_c; t0.type = in_type; t0.producer = -1; t0.external = true;
  t0.bytes_per_image = (size_t)in_h * in_w * in_c;

  for (int i = 0; i < n_layers && st == F8_OK; ++i) {
    f8_layer_desc L = layers[i];
    L.q.res = nullptr;
    if (L.dst2 <= 0) L.dst2 = -1;
    Tensor &s = c->tensors[L.src];
    if (s.producer == -2) { st = F8_ERR_SHAPE; break; }           // read before written
    if (c->tensors[L.dst].producer != -2) { st = F8_ERR_SHAPE; break; }   // written twice
    if (L.op < F8_OP_CONV || L.op > F8_OP_GPOOL) { st = F8_ERR_UNSUPPORTED; break; }
    if (L.Cin != s.c || L.q.x_type != s.type) { st = F8_ERR_SHAPE; break; }
    if (s.fl_known && s.fl != L.q.fl_x) { st = F8_ERR_FL; break; }
    s.fl = L.q.fl_x; s.fl_known = true;
    Geom g{1, s.h, s.w, L.Cin, L.Cout, L.R, L.S, L.stride_h, L.stride_w, L.pad_h, L.pad_w, 0, 0};
    Tensor d;
    d.producer = i;
    if (L.op == F8_OP_MAXPOOL) {
      if (L.Cout != L.Cin || L.res >= 0) { st = F8_ERR_SHAPE; break; }
      st = check_geom(g, true);
      if (st != F8_OK) break;
      if (L.pad_h >= L.R || L.pad_w >= L.S) { st = F8_ERR_SHAPE; break; }
      d.type = s.type; d.fl = s.fl; d.fl_known = true;
    } else {
      if (L.op == F8_OP_GPOOL) {
        if (L.Cout != L.Cin || L.res >= 0 || (long long)s.h * s.w > 65536) { st = F8_ERR_SHAPE; break; }
        g.R = s.h; g.S = s.w; g.sh = g.sw = 1; g.ph = g.pw = 0; g.P = g.Q = 1;
        L.R = s.h; L.S = s.w;
      } else {
        if (!L.w) { st = F8_ERR_NULL; break; }
        st = check_geom(g, L.op == F8_OP_DWCONV);
        if (st != F8_OK) break;
      }
      // a dummy non-null residual pointer lets check_quant vet the residual fields
      f8_quant qq = L.q;
      if (L.res >= 0) qq.res = &qq;
      st = check_quant(&qq, L.op != F8_OP_GPOOL);
      if (st != F8_OK) break;
      if (reinterpret_cast<uintptr_t>(L.bias) & 3) { st = F8_ERR_ALIGN; break; }
      d.type = L.q.y_type;
      d.fl = L.q.y_type == F8_S32 ? L.q.fl_x + L.q.fl_w : L.q.fl_y;
      d.fl_known = true;
    }
    if (g.P < 1 || g.Q < 1) { st = F8_ERR_SHAPE; break; }
    d.h = g.P; d.w = g.Q; d.c = L.Cout;
    d.bytes_per_image = (size_t)d.h * d.w * d.c * elem_size(d.type);
    if (L.res >= 0) {
      const Tensor &r = c->tensors[L.res];
      if (r.producer == -2 || L.res == L.dst) { st = F8_ERR_SHAPE; break; }
      if (r.h != d.h || r.w != d.w || r.c != d.c || r.type != L.q.res_type) { st = F8_ERR_SHAPE; break; }
      if (r.fl_known && r.fl != L.q.fl_res) { st = F8_ERR_FL; break; }
      c->tensors[L.res].fl = L.q.fl_res; c->tensors[L.res].fl_known = true;
      c->tensors[L.res].last_use = i;
    }
    if (L.dst2 > 0) {
      // a second format of the same result for a sibling consumer
      if (L.op != F8_OP_CONV || L.dst2 == L.dst || L.dst2 == L.src || L.dst2 == L.res ||
          c->tensors[L.dst2].producer != -2) { st = F8_ERR_SHAPE; break; }
      st = check_requant2(L.q, &L.q2);
      if (st != F8_OK) break;
      Tensor d2 = d;
      d2.type = L.q2.y_type; d2.fl = L.q2.fl_y;
      d2.bytes_per_image = (size_t)d2.h * d2.w * d2.c;
      c->tensors[L.dst2] = d2;
    }
    s.last_use = i;
    c->tensors[L.dst] = d;
    c->layers.push_back(L);
    c->geom.push_back(g);
    c->acc0_off.push_back(c->const_bytes);
    Stem sm;
    if (L.op == F8_OP_CONV) {
      c->const_bytes += acc0_padded(L.Cout) * sizeof(int32_t);
      if (L.Cin <= 4 && L.q.y_type != F8_S32 && (L.Cout & 3) == 0) {
        sm.on = true;
        sm.Sp = (L.S + 3) / 4 * 4;
        sm.Hp = (g.P - 1) * g.sh + g.R;
        // whole 16-byte groups of pixels per row, and two pixels no window reaches at the end of a row (the
        // fused stem fetches some rows 8 bytes off the 16-byte grid)
        sm.Wp = ((g.Q - 1) * g.sw + sm.Sp + 2 + 3) / 4 * 4;
        sm.x_bytes_per_image = (size_t)sm.Hp * sm.Wp * 4;
        sm.w_off = c->const_bytes;
        c->const_bytes += round256((size_t)L.Cout * g.R * sm.Sp * 4);
      } else if (L.Cin > 4 && (L.Cin & 15) != 0 && L.q.y_type != F8_S32 && (L.Cout & 3) == 0) {
        sm.on = true;
        sm.Cp = (L.Cin + 15) / 16 * 16;
        sm.x_bytes_per_image = (size_t)g.H * g.W * sm.Cp;
        sm.w_off = c->const_bytes;
        c->const_bytes += round256((size_t)L.Cout * g.R * g.S * sm.Cp);
      }
    }
    size_t img_off = 0;
    if (L.op == F8_OP_CONV && !sm.on && L.res < 0 && L.dst2 <= 0 && L.q.y_type != F8_S32 &&
        (reinterpret_cast<uintptr_t>(L.w) & 15) == 0 &&
        conv_img_applicable(L.Cin, L.Cout, L.R, L.S, L.stride_h, L.stride_w, L.pad_h, L.pad_w, g.H, g.W,
                            L.q.fl_x + L.q.fl_w - L.q.fl_y, nullptr, nullptr)) {
      img_off = c->const_bytes;
      c->const_bytes += round256(conv_img_weight_bytes(L.Cin));
    }
    c->img_w_off.push_back(img_off);
    c->stem.push_back(sm);
    c->fused.push_back(Fused());
    c->tail.push_back(0);
    c->tail_peer.push_back(-1);
  }
  if (st != F8_OK) { delete c; return st; }
  c->last_tensor = c->layers.back().dst;
  c->tensors[c->last_tensor].external = true;
  c->stem_pool = tuning().stem_pool.load() != 0;
  c->conv_img = tuning().conv_img.load() != 0;
  c->conv_img_min = tuning().conv_img_min.load();
  // a stem whose only reader is a 3x3 stride-2 pad-1 max pool: both in one kernel
  for (size_t i = 0; i + 1 < c->layers.size(); ++i) {
    const f8_layer_desc &L = c->layers[i], &M = c->layers[i + 1];
    const Stem &sm = c->stem[i];
    if (L.op != F8_OP_CONV || !sm.on || sm.Cp != 4 || L.Cin != 3 || L.res >= 0 || L.dst2 > 0) continue;
    if (!stem_pool_applicable(L.Cout, L.R, L.S, L.stride_h, L.stride_w, L.pad_h, L.pad_w, sm.Sp)) continue;
    if (L.q.y_type != F8_U8 || L.q.clip_lo < 0 || L.q.fl_x + L.q.fl_w - L.q.fl_y < 0) continue;
    if (M.op != F8_OP_MAXPOOL || M.src != L.dst || M.R != 3 || M.S != 3 || M.stride_h != 2 || M.stride_w != 2 ||
        M.pad_h != 1 || M.pad_w != 1)
      continue;
    if (c->tensors[L.dst].last_use != (int)i + 1 || L.dst == c->last_tensor) continue;
    c->stem[i].pool = 1;
    c->stem[i + 1].pool = 2;
  }
  c->conv_tail = tuning().conv_tail.load() != 0;      // tuning aid
  // a 1x1 64 -> 256 layer and a 1x1 layer of 64 or 128 channels that reads it, or a 1x1 128 -> 512 layer and
  // a 1x1 layer of 128 channels that reads it (the hand-over between two bottleneck blocks): the second can run on each block of the first one's output while it is in LDS.
  // It is the next layer, or the one after it when the layer between them takes no part in a pair (the
  // shortcut projection of a new stage).  Every tensor involved lives in the arena (aligned); weights
  // must be 16-byte aligned.
  for (size_t i = 0; i + 1 < c->layers.size(); ++i) {
    const f8_layer_desc &L = c->layers[i];
    if (c->tail[i] != 0 || c->stem[i].pool != 0 || c->stem[i].on) continue;
    if (L.op != F8_OP_CONV || L.dst2 > 0) continue;
    const bool head64 = L.Cin == 64 && L.Cout == 256, head128 = L.Cin == 128 && L.Cout == 512;
    if (!(head64 || head128) || L.R != 1 || L.S != 1 || L.stride_h != 1 || L.stride_w != 1 || L.pad_h != 0 || L.pad_w != 0) continue;
    if (L.q.y_type == F8_S32 || (L.res >= 0 && L.q.res_type == F8_S32) || L.q.fl_x + L.q.fl_w - L.q.fl_y < 0) continue;
    for (size_t j = i + 1; j <= i + 2 && j < c->layers.size(); ++j) {
      const f8_layer_desc &T = c->layers[j];
      if (c->tail[j] != 0 || c->stem[j].on || c->stem[j].pool != 0) break;
      const bool fits = T.op == F8_OP_CONV && T.src == L.dst && T.dst2 <= 0 && T.res < 0 && (T.Cout == 128 || (head64 && T.Cout == 64)) &&
                        T.R == 1 && T.S == 1 && T.stride_h == 1 && T.stride_w == 1 && T.pad_h == 0 && T.pad_w == 0 &&
                        T.q.y_type != F8_S32 && T.q.fl_x + T.q.fl_w - T.q.fl_y >= 0 &&
                        ((reinterpret_cast<uintptr_t>(L.w) | reinterpret_cast<uintptr_t>(T.w)) & 15) == 0;
      const int ids[4] = {L.src, L.res, L.dst, T.dst};
      bool arena_only = true;
      for (int id : ids) arena_only = arena_only && (id < 0 || !c->tensors[id].external);
      if (fits && arena_only) {
        c->tail[i] = 1; c->tail_peer[i] = (int)j;
        c->tail[j] = 2; c->tail_peer[j] = (int)i;
        break;
      }
    }
  }
  // inverted-residual blocks that can run as one kernel
  for (size_t i = 0; i + 2 < c->layers.size(); ++i) {
    const f8_layer_desc &L0 = c->layers[i], &L1 = c->layers[i + 1], &L2 = c->layers[i + 2];
    const Geom &g1 = c->geom[i + 1];
    auto pointwise = [](const f8_layer_desc &L) {
      return L.op == F8_OP_CONV && L.R == 1 && L.S == 1 && L.stride_h == 1 && L.stride_w == 1 && L.pad_h == 0 &&
             L.pad_w == 0 && L.q.y_type != F8_S32 && L.q.fl_x + L.q.fl_w - L.q.fl_y >= 0;
    };
    if (c->fused[i].role != 0 || !pointwise(L0) || !pointwise(L2) || L0.res >= 0) continue;
    if (L0.dst2 > 0 || L1.dst2 > 0 || L2.dst2 > 0) continue;
    if (L1.op != F8_OP_DWCONV || g1.R != 3 || g1.S != 3 || g1.sh != 1 || g1.sw != 1 || g1.ph != 1 || g1.pw != 1 ||
        L1.res >= 0 || L1.q.y_type == F8_S32 || L1.q.fl_x + L1.q.fl_w - L1.q.fl_y < 0)
      continue;
    if (L1.src != L0.dst || L2.src != L1.dst) continue;
    if (c->tensors[L0.dst].last_use != (int)i + 1 || c->tensors[L1.dst].last_use != (int)i + 2) continue;
    if (L0.dst == c->last_tensor || L1.dst == c->last_tensor) continue;
    if (L2.res >= 0 && (L2.res != L0.src || L0.Cin != L2.Cout || L2.q.res_type == F8_S32)) continue;
    if ((L0.Cin & 3) || (L0.Cout & 3) || (L2.Cout & 3) || L0.Cin > BLOCK_MAX_CIN || L2.Cout > BLOCK_MAX_COUT) continue;
    Fused &f = c->fused[i];
    f.role = 1;
    c->fused[i + 1].role = c->fused[i + 2].role = 2;
    f.K1 = (L0.Cin + 31) / 32 * 32;
    f.CH = (L0.Cout + 31) / 32;
    f.NB2 = (L2.Cout + 31) / 32;
    auto take = [&](size_t bytes) { const size_t off = c->const_bytes; c->const_bytes += round256(bytes); return off; };
    f.w1p = take((size_t)f.CH * 32 * f.K1);
    f.w2p = take((size_t)f.CH * f.NB2 * 1024);
    f.wdp = take((size_t)f.CH * 288);
    f.acc1 = take((size_t)f.CH * 32 * sizeof(int32_t));
    f.accd = take((size_t)f.CH * 32 * sizeof(int32_t));
    f.acc2 = take((size_t)f.NB2 * 32 * sizeof(int32_t));
    i += 2;
  }
  c->const_bytes = round256(c->const_bytes);
  *out = c;
  return F8_OK;
}

f8_status f8_chain_set_keep_all(f8_chain *c, int keep_all) {
  if (!c) return F8_ERR_NULL;
  c->keep_all = keep_all != 0;
  c->planned = false;
  c->prepared_ws = nullptr;
  return F8_OK;
}

f8_status f8_chain_set_fusion(f8_chain *c, int fusion) {
  if (!c) return F8_ERR_NULL;
  c->fusion = fusion != 0;
  c->planned = false;
  c->prepared_ws = nullptr;
  return F8_OK;
}

f8_status f8_chain_workspace_bytes(const f8_chain *cc, int batch, size_t *bytes) {
  if (!cc || !bytes) return F8_ERR_NULL;
  if (batch < 0) return F8_ERR_SHAPE;
  f8_chain *c = const_cast<f8_chain *>(cc);
  if (!c->planned) c->plan();
  // every tensor must stay addressable with 32-bit element counts
  for (const Tensor &t : c->tensors)
    if (t.producer != -2 && (long long)t.bytes_per_image / (long long)elem_size(t.type) * batch > 0x7fffffffLL)
      return F8_ERR_UNSUPPORTED;
  for (const Stem &sm : c->stem)
    if (sm.on && (long long)sm.x_bytes_per_image * batch > 0x7fffffffLL) return F8_ERR_UNSUPPORTED;
  *bytes = c->const_bytes + c->arena_per_image * (size_t)batch + 256;
  return F8_OK;
}

f8_status f8_chain_prepare(f8_chain *c, void *workspace, int batch, void *stream) {
  if (!c || !workspace) return F8_ERR_NULL;
  if (batch < 0) return F8_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return F8_ERR_ALIGN;
  if (!c->planned) c->plan();
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (hipMemsetAsync(workspace, 0, 256, s) != hipSuccess) return F8_ERR_DEVICE;
  for (size_t i = 0; i < c->layers.size(); ++i) {
    const f8_layer_desc &L = c->layers[i];
    if (L.op != F8_OP_CONV) continue;
    if (c->stem[i].on) {
      void *wp = static_cast<uint8_t *>(workspace) + c->stem[i].w_off;
      const int e = c->stem[i].Cp == 4
                        ? launch_repack_weights(L.w, wp, L.Cout, L.R, L.S, L.Cin, c->stem[i].Sp, s)
                        : launch_pad_rows(L.w, wp, (long long)L.Cout * L.R * L.S, L.Cin, c->stem[i].Cp, s);
      if (e != 0) return F8_ERR_DEVICE;
    }
    int32_t *acc0 = reinterpret_cast<int32_t *>(static_cast<uint8_t *>(workspace) + c->acc0_off[i]);
    const f8_status st = enqueue_fold(c->conv_weights(i, workspace), L.bias, acc0, c->conv_geom(i, 1), L.q, s);
    if (st != F8_OK) return st;
    if (c->img_w_off[i] != 0 &&
        launch_conv_img_weights(L.w, reinterpret_cast<int8_t *>(static_cast<uint8_t *>(workspace) + c->img_w_off[i]), L.Cin, s) != 0)
      return F8_ERR_DEVICE;
  }
  for (size_t i = 0; i < c->layers.size(); ++i) {
    const Fused &f = c->fused[i];
    if (f.role != 1) continue;
    const f8_layer_desc &L0 = c->layers[i], &L1 = c->layers[i + 1], &L2 = c->layers[i + 2];
    uint8_t *cb = static_cast<uint8_t *>(workspace);
    int e = launch_block_pack_w1(L0.w, reinterpret_cast<int8_t *>(cb + f.w1p), L0.Cout, L0.Cin, f.CH, f.K1, s);
    if (e == 0) e = launch_block_pack_w2(L2.w, reinterpret_cast<int8_t *>(cb + f.w2p), L2.Cout, L0.Cout, f.NB2, f.CH, s);
    if (e == 0) e = launch_block_pack_wd(L1.w, reinterpret_cast<int8_t *>(cb + f.wdp), L0.Cout, f.CH, s);
    // start values; an unsigned intermediate is kept minus 128 (see BlockParams)
    const int eb = L0.q.y_type == F8_U8 ? 128 : 0, db = L1.q.y_type == F8_U8 ? 128 : 0;
    const int sh1 = L0.q.fl_x + L0.q.fl_w - L0.q.fl_y, shd = L1.q.fl_x + L1.q.fl_w - L1.q.fl_y;
    if (e == 0) e = launch_fold_acc0(L0.w, L0.bias, reinterpret_cast<int32_t *>(cb + f.acc1), L0.Cout, f.CH * 32, L0.Cin,
                                     L0.q.x_type == F8_U8, rounding_addend(L0.q) - (eb << sh1), s);
    if (e == 0) e = launch_block_fold_dw(L1.w, L1.bias, reinterpret_cast<int32_t *>(cb + f.accd), L0.Cout, f.CH * 32,
                                         rounding_addend(L1.q) - (db << shd), eb, s);
    if (e == 0) e = launch_fold_acc0(L2.w, L2.bias, reinterpret_cast<int32_t *>(cb + f.acc2), L2.Cout, f.NB2 * 32, L0.Cout,
                                     L2.q.x_type == F8_U8, rounding_addend(L2.q), s);
    if (e != 0) return F8_ERR_DEVICE;
  }
  c->prepared_ws = workspace;
  c->prepared_batch = batch;
  return F8_OK;
}

f8_status f8_chain_run(f8_chain *c, const void *x, void *out, void *workspace, int batch, void *stream) {
  if (!c || !x || !out || !workspace) return F8_ERR_NULL;
  if (batch < 0) return F8_ERR_SHAPE;
  if (c->prepared_ws != workspace || c->prepared_batch != batch) return F8_ERR_STATE;
  if (c->tensors[c->last_tensor].type == F8_S32 && (reinterpret_cast<uintptr_t>(out) & 3)) return F8_ERR_ALIGN;
  if (batch == 0) return F8_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (c->n_streams == 2 && !c->keep_all && batch >= 2) {
    // first half of the images on the caller's stream, second half on the chain's own stream, which
    // starts behind everything already queued on the caller's stream and is waited for at the end
    const int b0 = batch / 2, b1 = batch - b0;
    const Tensor &tin = c->tensors[0], &tout = c->tensors[c->last_tensor];
    const void *x1 = static_cast<const uint8_t *>(x) + tin.bytes_per_image * (size_t)b0;
    void *out1 = static_cast<uint8_t *>(out) + tout.bytes_per_image * (size_t)b0;
    if (hipEventRecord(c->ev_fork, s) != hipSuccess || hipStreamWaitEvent(c->side_stream, c->ev_fork, 0) != hipSuccess)
      return F8_ERR_DEVICE;
    f8_status st = F8_OK;
    for (size_t i = 0; i < c->layers.size() && st == F8_OK; ++i) {
      c->arena_shift = 0;
      st = c->launch_layer(i, x, out, workspace, b0, s);
      if (st != F8_OK) break;
      c->arena_shift = c->arena_per_image * (size_t)b0;
      st = c->launch_layer(i, x1, out1, workspace, b1, c->side_stream);
    }
    c->arena_shift = 0;
    // join even after a failed launch, so that a capture in progress is left in a consistent state
    if (hipEventRecord(c->ev_join, c->side_stream) != hipSuccess || hipStreamWaitEvent(s, c->ev_join, 0) != hipSuccess)
      return F8_ERR_DEVICE;
    return st;
  }
  for (size_t i = 0; i < c->layers.size(); ++i) {
    const f8_status st = c->launch_layer(i, x, out, workspace, batch, s);
    if (st != F8_OK) return st;
  }
  return F8_OK;
}

f8_status f8_chain_set_streams(f8_chain *c, int n_streams) {
  if (!c) return F8_ERR_NULL;
  if (n_streams != 1 && n_streams != 2) return F8_ERR_UNSUPPORTED;
  if (n_streams == 2 && !c->side_stream) {
    if (hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking) != hipSuccess) { c->side_stream = nullptr; return F8_ERR_DEVICE; }
    if (hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess)
      return F8_ERR_DEVICE;
  }
  c->n_streams = n_streams;
  return F8_OK;
}

f8_status f8_chain_tensor(const f8_chain *c, int id, void *workspace, int batch, void **ptr, int *h, int *w,
                          int *ch, int *dtype, int *live_at_end) {
  if (!c) return F8_ERR_NULL;
  if (id < 0 || id >= (int)c->tensors.size() || c->tensors[id].producer == -2) return F8_ERR_SHAPE;
  if (!c->planned) const_cast<f8_chain *>(c)->plan();
  const Tensor &t = c->tensors[id];
  // tensors inside a fused block are never materialised
  const bool elided = (t.producer >= 0 && c->pool_role((size_t)t.producer) == 1) ||
                      (c->use_fusion() && t.producer >= 0 && c->fused[t.producer].role != 0 &&
                       !(c->fused[t.producer].role == 2 && t.producer >= 2 && c->fused[t.producer - 2].role == 1));
  // (with two streams the two halves of a tensor lie apart: not reported)
  const bool halves = c->n_streams == 2 && !c->keep_all && batch >= 2;
  if (ptr) *ptr = (t.external || !workspace || elided || halves) ? nullptr : c->tensor_ptr(id, nullptr, nullptr, workspace, batch);
  if (h) *h = t.h;
  if (w) *w = t.w;
  if (ch) *ch = t.c;
  if (dtype) *dtype = t.type;
  if (live_at_end) {
    int live = elided ? 0 : 1;
    if (!c->keep_all && !t.external && !elided) {
      // overwritten if something allocated after this tensor's last use overlaps it
      const size_t a0 = t.offset_per_image, a1 = a0 + round256(t.bytes_per_image);
      for (size_t j = 0; j < c->tensors.size() && live; ++j) {
        const Tensor &o = c->tensors[j];
        if ((int)j == id || o.external || o.producer == -2 || o.producer <= t.last_use ||
            o.producer <= t.producer)
          continue;
        const size_t b0 = o.offset_per_image, b1 = b0 + round256(o.bytes_per_image);
        if (a0 < b1 && b0 < a1) live = 0;
      }
      for (size_t j = 0; j < c->stem.size() && live; ++j) {
        const Stem &sm = c->stem[j];
        if (!sm.on || (int)j <= t.last_use || (int)j <= t.producer) continue;
        const size_t b0 = sm.x_off_per_image, b1 = b0 + round256(sm.x_bytes_per_image);
        if (a0 < b1 && b0 < a1) live = 0;
      }
    }
    *live_at_end = live;
  }
  return F8_OK;
}

void f8_chain_destroy(f8_chain *c) {
  if (!c) return;
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
  delete c;
}

// ---- measurement aids ---------------------------------------------------------------------

int f8_chain_num_layers(const f8_chain *c) { return c ? (int)c->layers.size() : 0; }

f8_status f8_chain_layer_info(const f8_chain *c, int layer, int batch, char *kernel_name, int name_len,
                              double *alg_ops, double *alg_bytes) {
  if (!c) return F8_ERR_NULL;
  if (layer < 0 || layer >= (int)c->layers.size() || batch < 0) return F8_ERR_SHAPE;
  const f8_layer_desc &L = c->layers[layer];
  const Geom &g = c->geom[layer];
  const char *name = "?";
  double ops = 0.0;
  if (c->pool_role((size_t)layer) != 0) {
    // stem and pool are accounted to the stem: image in, pooled tensor out, weights
    const bool first = c->pool_role((size_t)layer) == 1;
    const char *fname = first ? "stem_pool_fused" : "(fused)";
    if (kernel_name && name_len > 0) {
      int i = 0;
      for (; fname[i] && i < name_len - 1; ++i) kernel_name[i] = fname[i];
      kernel_name[i] = 0;
    }
    const Geom &gp = c->geom[first ? layer + 1 : layer];
    if (alg_ops) *alg_ops = first ? 2.0 * batch * g.P * g.Q * (double)g.R * g.S * g.Cin * g.Cout : 0.0;
    if (alg_bytes)
      *alg_bytes = first ? (double)batch * g.H * g.W * g.Cin + (double)batch * gp.P * gp.Q * g.Cout +
                               (double)g.R * g.S * g.Cin * g.Cout + 4.0 * g.Cout
                         : 0.0;
    return F8_OK;
  }
  if (c->use_fusion() && c->fused[layer].role != 0) {
    // the whole block is accounted to its first layer: block input + output (+ shortcut read
    // from the same input), all weights
    double fo = 0.0, fb = 0.0;
    const char *fname = "(fused)";
    if (c->fused[layer].role == 1) {
      const f8_layer_desc &L1 = c->layers[layer + 1], &L2 = c->layers[layer + 2];
      const double px = (double)batch * g.H * g.W;
      fo = 2.0 * px * ((double)L.Cin * L.Cout + 9.0 * L1.Cout + (double)L2.Cin * L2.Cout);
      fb = px * (L.Cin + L2.Cout) + (double)L.Cin * L.Cout + 9.0 * L1.Cout + (double)L2.Cin * L2.Cout +
           4.0 * (L.Cout + L1.Cout + L2.Cout);
      fname = "block_fused";
    }
    if (kernel_name && name_len > 0) {
      int i = 0;
      for (; fname[i] && i < name_len - 1; ++i) kernel_name[i] = fname[i];
      kernel_name[i] = 0;
    }
    if (alg_ops) *alg_ops = fo;
    if (alg_bytes) *alg_bytes = fb;
    return F8_OK;
  }
  if (c->tail_role((size_t)layer, batch) == 2) {
    // accounted to the layer in front, whose launch computes this one
    const char *fname = "(fused)";
    if (kernel_name && name_len > 0) {
      int i = 0;
      for (; fname[i] && i < name_len - 1; ++i) kernel_name[i] = fname[i];
      kernel_name[i] = 0;
    }
    if (alg_ops) *alg_ops = 0.0;
    if (alg_bytes) *alg_bytes = 0.0;
    return F8_OK;
  }
  const bool with_tail = c->tail_role((size_t)layer, batch) == 1;
  const double M = (double)batch * g.P * g.Q;
  // input pixels a strided window actually touches
  const double rows = g.sh >= g.R ? (double)g.P * g.R : (double)std::min(g.H, (g.P - 1) * g.sh + g.R);
  const double cols = g.sw >= g.S ? (double)g.Q * g.S : (double)std::min(g.W, (g.Q - 1) * g.sw + g.S);
  double bytes = (double)batch * rows * cols * g.Cin + M * g.Cout * (double)elem_size(c->tensors[L.dst].type);
  if (L.res >= 0) bytes += M * g.Cout * (double)elem_size(c->tensors[L.res].type);
  if (L.dst2 > 0) bytes += M * g.Cout;
  switch (L.op) {
    case F8_OP_CONV: {
      Geom gk = c->narrow_rows((size_t)layer, batch) ? g : c->conv_geom(layer, batch);
      gk.B = batch;
      gk.P = g.P; gk.Q = g.Q;
      name = c->img_role((size_t)layer, batch)
                 ? (L.Cin == 256 ? "conv3x3_img<256x256>" : "conv3x3_img<128x128>")
                 : conv_kernel_name(gk, L.q, L.res >= 0);
      ops = 2.0 * M * g.R * g.S * g.Cin * g.Cout;
      bytes += (double)g.R * g.S * g.Cin * g.Cout + 4.0 * g.Cout;
      if (with_tail) {
        // plus the 1x1 layer behind it: its output and weights; its input never leaves the chip
        const f8_layer_desc &T = c->layers[c->tail_peer[layer]];
        name = L.Cin == 128 ? "pw1x1_mid<128x512>+1x1<128>" : (T.Cout == 64 ? "pw1x1_ws<64x256>+1x1<64>" : "pw1x1_ws<64x256>+1x1<128>");
        ops += 2.0 * M * (double)T.Cin * T.Cout;
        bytes += M * T.Cout + (double)T.Cin * T.Cout + 4.0 * T.Cout;
      }
      break;
    }
    case F8_OP_DWCONV:
      name = (g.R == 3 && g.S == 3 && g.sh == g.sw && (g.sh == 1 || g.sh == 2) && g.Cin % 4 == 0 && L.res < 0 &&
              c->tensors[L.dst].type != F8_S32 && L.q.fl_x + L.q.fl_w - L.q.fl_y >= 0)
                 ? (g.sh == 1 ? "dwconv3x3<s1>" : "dwconv3x3<s2>")
                 : "dwconv_generic";
      ops = 2.0 * M * g.R * g.S * g.Cout;
      bytes += (double)g.R * g.S * g.Cout + 4.0 * g.Cout;
      break;
    case F8_OP_MAXPOOL: name = "maxpool"; break;
    default: name = "gpool"; break;
  }
  if (kernel_name && name_len > 0) {
    int i = 0;
    for (; name[i] && i < name_len - 1; ++i) kernel_name[i] = name[i];
    kernel_name[i] = 0;
  }
  if (alg_ops) *alg_ops = ops;
  if (alg_bytes) *alg_bytes = bytes;
  return F8_OK;
}

f8_status f8_chain_profile(f8_chain *c, const void *x, void *out, void *workspace, int batch, void *stream,
                           int repeats, float *layer_ms) {
  if (!c || !x || !out || !workspace || !layer_ms) return F8_ERR_NULL;
  if (batch < 1 || repeats < 1) return F8_ERR_SHAPE;
  if (c->prepared_ws != workspace || c->prepared_batch != batch) return F8_ERR_STATE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t n = c->layers.size();
  // Two passes per repeat, events after every layer: pass A launches each layer once, pass B
  // launches it 1 + EXTRA times back to back (a layer never writes what it reads, so the
  // relaunches recompute the same bytes).  (B - A) / EXTRA is the duration of one launch in a
  // busy stream; the cost of the event pair itself, a few microseconds, cancels.
  constexpr int EXTRA = 4;
  const size_t per = 2 * (n + 1);
  std::vector<hipEvent_t> ev(repeats * per);
  for (auto &e : ev)
    if (hipEventCreate(&e) != hipSuccess) return F8_ERR_DEVICE;
  f8_status st = F8_OK;
  for (int r = 0; r < repeats && st == F8_OK; ++r) {
    for (int pass = 0; pass < 2 && st == F8_OK; ++pass) {
      hipEvent_t *e = &ev[r * per + pass * (n + 1)];
      (void)hipEventRecord(e[0], s);
      for (size_t i = 0; i < n && st == F8_OK; ++i) {
        for (int k = 0; k < (pass ? 1 + EXTRA : 1) && st == F8_OK; ++k) st = c->launch_layer(i, x, out, workspace, batch, s);
        (void)hipEventRecord(e[i + 1], s);
      }
    }
  }
  if (hipStreamSynchronize(s) != hipSuccess) st = F8_ERR_DEVICE;
  if (st == F8_OK) {
    for (size_t i = 0; i < n; ++i) {
      double a_sum = 0.0, b_sum = 0.0;
      for (int r = 0; r < repeats; ++r) {
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, ev[r * per + i], ev[r * per + i + 1]);
        a_sum += ms;
        (void)hipEventElapsedTime(&ms, ev[r * per + (n + 1) + i], ev[r * per + (n + 1) + i + 1]);
        b_sum += ms;
      }
      const double one = (b_sum - a_sum) / (EXTRA * (double)repeats);
      layer_ms[i] = (float)(one > 0.0 ? one : b_sum / ((1 + EXTRA) * (double)repeats));
    }
  }
  for (auto &e : ev) (void)hipEventDestroy(e);
  return st;
}

}  // extern "C"
