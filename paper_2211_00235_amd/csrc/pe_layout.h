// Host-only: dims checks, flat parameter layout, ctx (saved activation) layout.
#pragma once
#include <string.h>
#include <vector>
#include "../../include/pe.h"

struct AttnP { long long ln_g, ln_b, ln_z_g, ln_z_b, w_bias, w_q, w_k, w_v, w_g, b_g, w_o, b_o; };
struct TransP { long long ln_g, ln_b, w1, b1, w2, b2; };
struct OpmP { long long ln_g, ln_b, w_a, b_a, w_b, b_b, w_o, b_o; };
struct TriMulP {
  long long ln_in_g, ln_in_b, w_ap, b_ap, w_ag, b_ag, w_bp, b_bp, w_bg, b_bg, w_g, b_g, ln_out_g, ln_out_b, w_o, b_o;
};
struct ParamLayout {
  AttnP row, col, tas, tae;
  TransP mtrans, ptrans;
  OpmP opm;
  TriMulP tmo, tmi;
  long long total;
  std::vector<pe_param_entry> entries;
};

inline int pe_check_dims_impl(const pe_dims* d) {
  if (!d) return PE_ERR_NULL;
  if (d->s < 1 || d->r < 1) return PE_ERR_DIMS;
  if (d->dtype != PE_F32 && d->dtype != PE_BF16) return PE_ERR_DIMS;
  if (d->n_trans < 1 || d->h_msa < 1 || d->h_pair < 1) return PE_ERR_DIMS;
  if (d->h_msa > 8 || d->h_pair > 8) return PE_ERR_DIMS;                 // bias projection keeps <= 8 heads in registers
  int ch[] = {d->c_m, d->c_z, d->h_msa * d->d_msa, d->h_pair * d->d_pair, d->c_tri, d->c_opm};
  for (int c : ch)
    if (c < 8 || c % 8 || c > 1024) return PE_ERR_DIMS;
  if (d->c_z > 256) return PE_ERR_DIMS;                                  // fused LayerNorm + bias projection: one chunk per lane
  if (d->c_tri > 192) return PE_ERR_DIMS;                                // channel-major LayerNorm tile in 64 KB of LDS
  if ((long long)d->n_trans * d->c_m > 4096 || (long long)d->n_trans * d->c_z > 4096) return PE_ERR_DIMS;
  if (d->d_msa % 8 || d->d_msa > 32 || d->d_pair % 8 || d->d_pair > 32) return PE_ERR_DIMS;
  if (d->col_global != 0 && d->col_global != 1) return PE_ERR_DIMS;
  if (d->variant < PE_VARIANT_PARALLEL || d->variant > PE_VARIANT_MULTIMER) return PE_ERR_DIMS;
  if (!(d->ln_eps > 0.0f) || !(d->opm_eps > 0.0f)) return PE_ERR_DIMS;
  if ((long long)d->r * d->r * 4 * d->h_pair * d->d_pair >= (1LL << 40)) return PE_ERR_DIMS;
  return PE_OK;
}

struct ParamBuilder {
  ParamLayout& L;
  long long off = 0;
  explicit ParamBuilder(ParamLayout& l) : L(l) {}
  long long add(const char* pre, const char* nm, int a, int b, int kind) {
    pe_param_entry e;
    memset(&e, 0, sizeof(e));
    snprintf(e.name, sizeof(e.name), "%s.%s", pre, nm);
    e.offset = off;
    e.ndim = b ? 2 : 1;
    e.shape[0] = a;
    e.shape[1] = b;
    e.fan_in = (kind == 0) ? a : 0;
    e.kind = kind;
    L.entries.push_back(e);
    long long o = off;
    off += (long long)a * (b ? b : 1);
    return o;
  }
};

inline void build_attn(ParamBuilder& B, AttnP& p, const char* pre, int c_in, int h, int d, int c_bias, bool is_row,
                       bool global_kv) {
  int hd = h * d;
  memset(&p, 0xff, sizeof(p));
  if (is_row) {
    p.ln_g = B.add(pre, "ln_m.g", c_in, 0, 1);
    p.ln_b = B.add(pre, "ln_m.b", c_in, 0, 2);
    p.ln_z_g = B.add(pre, "ln_z.g", c_bias, 0, 1);
    p.ln_z_b = B.add(pre, "ln_z.b", c_bias, 0, 2);
  } else {
    p.ln_g = B.add(pre, "ln.g", c_in, 0, 1);
    p.ln_b = B.add(pre, "ln.b", c_in, 0, 2);
  }
  if (c_bias) p.w_bias = B.add(pre, "w_bias", c_bias, h, 0);
  int kv = global_kv ? d : hd;
  p.w_q = B.add(pre, "w_q", c_in, hd, 0);
  p.w_k = B.add(pre, "w_k", c_in, kv, 0);
  p.w_v = B.add(pre, "w_v", c_in, kv, 0);
  p.w_g = B.add(pre, "w_g", c_in, hd, 0);
  p.b_g = B.add(pre, "b_g", hd, 0, 3);
  p.w_o = B.add(pre, "w_o", hd, c_in, 0);
  p.b_o = B.add(pre, "b_o", c_in, 0, 3);
}
inline void build_trans(ParamBuilder& B, TransP& p, const char* pre, int c, int n) {
  p.ln_g = B.add(pre, "ln.g", c, 0, 1);
  p.ln_b = B.add(pre, "ln.b", c, 0, 2);
  p.w1 = B.add(pre, "w1", c, n * c, 0);
  p.b1 = B.add(pre, "b1", n * c, 0, 3);
  p.w2 = B.add(pre, "w2", n * c, c, 0);
  p.b2 = B.add(pre, "b2", c, 0, 3);
}
inline void build_trimul(ParamBuilder& B, TriMulP& p, const char* pre, int cz, int ct) {
  p.ln_in_g = B.add(pre, "ln_in.g", cz, 0, 1);
  p.ln_in_b = B.add(pre, "ln_in.b", cz, 0, 2);
  p.w_ap = B.add(pre, "w_ap", cz, ct, 0); p.b_ap = B.add(pre, "b_ap", ct, 0, 3);
  p.w_ag = B.add(pre, "w_ag", cz, ct, 0); p.b_ag = B.add(pre, "b_ag", ct, 0, 3);
  p.w_bp = B.add(pre, "w_bp", cz, ct, 0); p.b_bp = B.add(pre, "b_bp", ct, 0, 3);
  p.w_bg = B.add(pre, "w_bg", cz, ct, 0); p.b_bg = B.add(pre, "b_bg", ct, 0, 3);
  p.w_g = B.add(pre, "w_g", cz, cz, 0); p.b_g = B.add(pre, "b_g", cz, 0, 3);
  p.ln_out_g = B.add(pre, "ln_out.g", ct, 0, 1);
  p.ln_out_b = B.add(pre, "ln_out.b", ct, 0, 2);
  p.w_o = B.add(pre, "w_o", ct, cz, 0); p.b_o = B.add(pre, "b_o", cz, 0, 3);
}

inline void build_param_layout(const pe_dims& d, ParamLayout& L) {
  L.entries.clear();
  ParamBuilder B(L);
  build_attn(B, L.row, "row", d.c_m, d.h_msa, d.d_msa, d.c_z, true, false);
  build_attn(B, L.col, "col", d.c_m, d.h_msa, d.d_msa, 0, false, d.col_global != 0);
  build_trans(B, L.mtrans, "mtrans", d.c_m, d.n_trans);
  L.opm.ln_g = B.add("opm", "ln.g", d.c_m, 0, 1);
  L.opm.ln_b = B.add("opm", "ln.b", d.c_m, 0, 2);
  L.opm.w_a = B.add("opm", "w_a", d.c_m, d.c_opm, 0); L.opm.b_a = B.add("opm", "b_a", d.c_opm, 0, 3);
  L.opm.w_b = B.add("opm", "w_b", d.c_m, d.c_opm, 0); L.opm.b_b = B.add("opm", "b_b", d.c_opm, 0, 3);
  L.opm.w_o = B.add("opm", "w_o", d.c_opm * d.c_opm, d.c_z, 0); L.opm.b_o = B.add("opm", "b_o", d.c_z, 0, 3);
  build_trimul(B, L.tmo, "tmo", d.c_z, d.c_tri);
  build_trimul(B, L.tmi, "tmi", d.c_z, d.c_tri);
  build_attn(B, L.tas, "tas", d.c_z, d.h_pair, d.d_pair, d.c_z, false, false);
  build_attn(B, L.tae, "tae", d.c_z, d.h_pair, d.d_pair, d.c_z, false, false);
  build_trans(B, L.ptrans, "ptrans", d.c_z, d.n_trans);
  L.total = B.off;
}
