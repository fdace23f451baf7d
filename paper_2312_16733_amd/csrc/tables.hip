// Architecture validation and the layout of the weight blob / statistics row (host only).
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "host.h"

namespace sna {

static thread_local char g_err[512] = "";

sna_status fail(sna_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}
const char* last_error_text() { return g_err; }

static int out_size(int h, int k, int stride) { return (h + 2 * (k / 2) - k) / stride + 1; }

namespace {
struct Builder {
  ArchTables* t;
  int64_t off = 0;
  void tensor(const std::string& name, int kind, int dtype, int d0, int d1, int d2, int d3) {
    sna_tensor_info ti;
    memset(&ti, 0, sizeof(ti));
    snprintf(ti.name, SNA_NAME_LEN, "%s", name.c_str());
    ti.kind = kind;
    ti.dtype = dtype;
    ti.dims[0] = d0; ti.dims[1] = d1; ti.dims[2] = d2; ti.dims[3] = d3;
    ti.c_pad = kind == 0 ? d3 : (kind == 1 ? d2 : (kind == 2 ? d1 : d0));
    // conv weights of a bf16 family store their input channels padded to a multiple of 8 (zeros),
    // so that a 3-channel stem runs on the MFMA path over channel-padded inputs
    if (kind == 0 && dtype == SNA_DTYPE_BF16) ti.c_pad = (d3 + 7) / 8 * 8;
    const int64_t elems = kind == 0 ? (int64_t)d0 * d1 * d2 * ti.c_pad : (int64_t)d0 * d1 * d2 * d3;
    ti.bytes = elems * (dtype == SNA_DTYPE_BF16 ? 2 : 4);
    ti.offset = off;
    off += (ti.bytes + 255) / 256 * 256;
    t->tidx[name] = (int)t->tensors.size();
    t->tensors.push_back(ti);
  }
  void conv(const std::string& n, int k, int r, int c) { tensor(n, 0, t->arch.dtype, k, r, r, c); }
  void dw(const std::string& n, int r, int c) { tensor(n, 1, t->arch.dtype, r, r, c, 1); }
  void linear(const std::string& n, int k, int c) { tensor(n, 2, t->arch.dtype, k, c, 1, 1); }
  void vec(const std::string& n, int c) { tensor(n, 3, SNA_DTYPE_FP32, c, 1, 1, 1); }
  void norm(const std::string& name, int c) {
    sna_norm_info ni;
    memset(&ni, 0, sizeof(ni));
    snprintf(ni.name, SNA_NAME_LEN, "%s", name.c_str());
    ni.channels = c;
    ni.offset = (int32_t)t->row_len;
    t->row_len += c;
    t->nidx[name] = (int)t->norms.size();
    t->norms.push_back(ni);
  }
};
std::string blk(int s, int j) { return "s" + std::to_string(s) + ".b" + std::to_string(j) + "."; }
}  // namespace

sna_status build_tables(const sna_arch_desc* a, ArchTables* t) {
  if (!a || !t) return fail(SNA_E_NULL, "arch is NULL");
  t->arch = *a;
  t->tensors.clear(); t->norms.clear(); t->tidx.clear(); t->nidx.clear();
  t->row_len = 0;
  if (a->dtype != SNA_DTYPE_FP32 && a->dtype != SNA_DTYPE_BF16) return fail(SNA_E_ARCH, "bad dtype %d", a->dtype);
  t->esz = a->dtype == SNA_DTYPE_BF16 ? 2 : 4;
  if (a->n_classes < 1) return fail(SNA_E_ARCH, "n_classes < 1");
  Builder b{t};
  const int fam = a->family;
  if (fam == SNA_FAMILY_TINY || fam == SNA_FAMILY_RESNET || fam == SNA_FAMILY_MBV3) {
    if (a->n_stages < 1 || a->n_stages > SNA_MAX_STAGES) return fail(SNA_E_ARCH, "n_stages %d", a->n_stages);
    if (a->in_ch < 1 || a->in_ch > 8) return fail(SNA_E_ARCH, "in_ch %d", a->in_ch);
    if (a->stem_ch < 8 || a->stem_ch % 8) return fail(SNA_E_ARCH, "stem_ch %d", a->stem_ch);
    if (a->max_res < 8 || a->max_res > 1024) return fail(SNA_E_ARCH, "max_res %d", a->max_res);
    for (int s = 0; s < a->n_stages; ++s) {
      if (a->stage_ch[s] < 8 || a->stage_ch[s] % 8) return fail(SNA_E_ARCH, "stage_ch[%d]=%d", s, a->stage_ch[s]);
      if (a->stage_max_depth[s] < 1 || a->stage_max_depth[s] > SNA_MAX_DEPTH)
        return fail(SNA_E_ARCH, "stage_max_depth[%d]=%d", s, a->stage_max_depth[s]);
      if (fam != SNA_FAMILY_TINY && a->stage_stride[s] != 1 && a->stage_stride[s] != 2)
        return fail(SNA_E_ARCH, "stage_stride[%d]=%d", s, a->stage_stride[s]);
      if (fam != SNA_FAMILY_TINY)
        for (int j = 0; j < a->stage_max_depth[s]; ++j)
          if (a->block_max_mid[s][j] < 8 || a->block_max_mid[s][j] % 8)
            return fail(SNA_E_ARCH, "block_max_mid[%d][%d]=%d", s, j, a->block_max_mid[s][j]);
    }
  }
  int64_t per = 0;
  auto upd = [&](int64_t v) { if (v > per) per = v; };
  if (fam == SNA_FAMILY_TINY) {
    if (a->dtype != SNA_DTYPE_FP32) return fail(SNA_E_ARCH, "TINY family is fp32");
    b.conv("stem.w", a->stem_ch, 3, a->in_ch);
    b.norm("stem.sn", a->stem_ch);
    int prev = a->stem_ch, h = a->max_res;
    upd((int64_t)h * h * a->stem_ch);
    for (int s = 0; s < a->n_stages; ++s) {
      const int c = a->stage_ch[s];
      h = out_size(h, 3, 2);
      upd((int64_t)h * h * c);
      for (int j = 0; j < a->stage_max_depth[s]; ++j) {
        b.conv(blk(s, j) + "w", c, 3, j == 0 ? prev : c);
        b.norm(blk(s, j) + "sn", c);
      }
      prev = c;
    }
    b.linear("head.w", a->n_classes, prev);
    b.vec("head.b", a->n_classes);
    t->in_elems_max = (int64_t)a->max_res * a->max_res * (a->dtype == SNA_DTYPE_BF16 ? 8 : a->in_ch);
    t->small_elems = prev + a->n_classes;
  } else if (fam == SNA_FAMILY_RESNET) {
    if (a->dtype != SNA_DTYPE_BF16) return fail(SNA_E_ARCH, "RESNET family is bf16");
    b.conv("stem.w", a->stem_ch, 7, a->in_ch);
    b.norm("stem.sn", a->stem_ch);
    int prev = a->stem_ch;
    int h = out_size(a->max_res, 7, 2);
    upd((int64_t)h * h * a->stem_ch);
    h = out_size(h, 3, 2);
    for (int s = 0; s < a->n_stages; ++s) {
      const int c = a->stage_ch[s];
      const int ho = out_size(h, 3, a->stage_stride[s]);
      for (int j = 0; j < a->stage_max_depth[s]; ++j) {
        const int m = a->block_max_mid[s][j], cin = j == 0 ? prev : c;
        const std::string p = blk(s, j);
        b.conv(p + "conv1.w", m, 1, cin); b.norm(p + "sn1", m);
        b.conv(p + "conv2.w", m, 3, m);   b.norm(p + "sn2", m);
        b.conv(p + "conv3.w", c, 1, m);   b.norm(p + "sn3", c);
        if (j == 0) { b.conv(p + "short.w", c, 1, cin); b.norm(p + "sn_short", c); }
        upd((int64_t)h * h * (m > cin ? m : cin));
        upd((int64_t)ho * ho * (m > c ? m : c));
      }
      h = ho; prev = c;
    }
    b.linear("head.w", a->n_classes, prev);
    b.vec("head.b", a->n_classes);
    t->in_elems_max = (int64_t)a->max_res * a->max_res * (a->dtype == SNA_DTYPE_BF16 ? 8 : a->in_ch);
    t->small_elems = prev + a->n_classes;
  } else if (fam == SNA_FAMILY_MBV3) {
    if (a->dtype != SNA_DTYPE_BF16) return fail(SNA_E_ARCH, "MBV3 family is bf16");
    if (a->tail_ch < 8 || a->tail_ch % 8 || a->fc_ch < 8 || a->fc_ch % 8) return fail(SNA_E_ARCH, "tail/fc");
    const int c0 = a->stem_ch;
    b.conv("stem.w", c0, 3, a->in_ch); b.norm("stem.sn", c0);
    b.dw("first.dw.w", 3, c0); b.norm("first.sn1", c0);
    b.conv("first.pw.w", c0, 1, c0); b.norm("first.sn2", c0);
    int prev = c0, h = out_size(a->max_res, 3, 2);
    upd((int64_t)h * h * c0);
    int64_t small = 0;
    for (int s = 0; s < a->n_stages; ++s) {
      const int c = a->stage_ch[s];
      const int ho = out_size(h, 3, a->stage_stride[s]);
      for (int j = 0; j < a->stage_max_depth[s]; ++j) {
        const int m = a->block_max_mid[s][j], q = a->block_max_aux[s][j], cin = j == 0 ? prev : c;
        const std::string p = blk(s, j);
        b.conv(p + "expand.w", m, 1, cin); b.norm(p + "sn1", m);
        b.dw(p + "dw.w", 7, m); b.norm(p + "sn2", m);
        if (a->stage_se[s]) {
          if (q < 8 || q % 8) return fail(SNA_E_ARCH, "block_max_aux[%d][%d]=%d", s, j, q);
          b.linear(p + "se.fc1.w", q, m); b.vec(p + "se.fc1.b", q);
          b.linear(p + "se.fc2.w", m, q); b.vec(p + "se.fc2.b", m);
        }
        b.conv(p + "project.w", c, 1, m); b.norm(p + "sn3", c);
        upd((int64_t)(j == 0 ? h : ho) * (j == 0 ? h : ho) * m);
        upd((int64_t)ho * ho * (m > c ? m : c));
        if (a->stage_se[s]) {                        // pool partial sums of the depthwise blocks, then the gate's hidden layer
          if (m / 8 > 256) return fail(SNA_E_ARCH, "block_max_mid[%d][%d]=%d: squeeze-excite layers take at most 2048 channels", s, j, m);
          const int64_t need = (int64_t)depthwise_pool_blocks(ho, ho, m) * m + q;
          if (need > small) small = need;
        }
      }
      h = ho; prev = c;
    }
    b.conv("tail.w", a->tail_ch, 1, prev); b.norm("tail.sn", a->tail_ch);
    upd((int64_t)h * h * a->tail_ch);
    b.linear("fc1.w", a->fc_ch, a->tail_ch); b.vec("fc1.b", a->fc_ch);
    b.linear("head.w", a->n_classes, a->fc_ch); b.vec("head.b", a->n_classes);
    t->in_elems_max = (int64_t)a->max_res * a->max_res * (a->dtype == SNA_DTYPE_BF16 ? 8 : a->in_ch);
    const int64_t head_small = (int64_t)a->tail_ch + a->fc_ch + a->n_classes;
    t->small_elems = small > head_small ? small : head_small;
  } else if (fam == SNA_FAMILY_TRANSFORMER) {
    if (a->dtype != SNA_DTYPE_BF16) return fail(SNA_E_ARCH, "TRANSFORMER family is bf16");
    if (a->head_dim != 64) return fail(SNA_E_ARCH, "head_dim must be 64");
    if (a->hidden < 8 || a->hidden % 8 || a->n_heads < 1 || a->ffn < 8 || a->ffn % 8 ||
        a->max_layers < 1 || a->max_layers > SNA_MAX_DEPTH || a->seq_len < 1 || a->seq_len > 128)
      return fail(SNA_E_ARCH, "transformer shape");
    const int hd = a->hidden, at = a->n_heads * a->head_dim;
    for (int i = 0; i < a->max_layers; ++i) {
      const std::string p = "l" + std::to_string(i) + ".";
      for (const char* nm : {"q", "k", "v"}) { b.linear(p + nm + ".w", at, hd); b.vec(p + nm + ".b", at); }
      b.linear(p + "o.w", hd, at); b.vec(p + "o.b", hd);
      b.vec(p + "ln1.g", hd); b.vec(p + "ln1.b", hd);
      b.linear(p + "ffn1.w", a->ffn, hd); b.vec(p + "ffn1.b", a->ffn);
      b.linear(p + "ffn2.w", hd, a->ffn); b.vec(p + "ffn2.b", hd);
      b.vec(p + "ln2.g", hd); b.vec(p + "ln2.b", hd);
    }
    b.linear("head.w", a->n_classes, hd); b.vec("head.b", a->n_classes);
    int mx = hd > at ? hd : at; mx = mx > a->ffn ? mx : a->ffn;
    per = (int64_t)a->seq_len * mx;
    t->in_elems_max = (int64_t)a->seq_len * hd;
    t->small_elems = a->n_classes;
  } else {
    return fail(SNA_E_ARCH, "unknown family %d", fam);
  }
  t->weight_bytes = b.off;
  t->per_image_elems = (per + 127) / 128 * 128;
  return SNA_OK;
}

}  // namespace sna
