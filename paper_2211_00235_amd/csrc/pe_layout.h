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

// why != nullptr receives a static string that names the violated limit
inline int pe_check_dims_impl(const pe_dims* d, const char** why = nullptr) {
  const char* dummy;
  if (!why) why = &dummy;
  *why = "";
  if (!d) { *why = "dims is NULL"; return PE_ERR_NULL; }
#define PE_DIM_REQUIRE(cond, text) do { if (!(cond)) { *why = text; return PE_ERR_DIMS; } } while (0)
  PE_DIM_REQUIRE(d->s >= 1 && d->r >= 1, "s and r must be >= 1");
  PE_DIM_REQUIRE(d->dtype == PE_F32 || d->dtype == PE_BF16, "dtype must be PE_F32 or PE_BF16");
  PE_DIM_REQUIRE(d->n_trans >= 1 && d->h_msa >= 1 && d->h_pair >= 1, "n_trans, h_msa and h_pair must be >= 1");
  // the fused LayerNorm + bias projection keeps at most 8 heads in registers
  PE_DIM_REQUIRE(d->h_msa <= 8 && d->h_pair <= 8, "h_msa and h_pair must be <= 8");
  int ch[] = {d->c_m, d->c_z, d->h_msa * d->d_msa, d->h_pair * d->d_pair, d->c_tri, d->c_opm};
  for (int c : ch)
    PE_DIM_REQUIRE(c >= 8 && c % 8 == 0 && c <= 1024,
                   "c_m, c_z, h_msa*d_msa, h_pair*d_pair, c_tri and c_opm must be multiples of 8 in [8, 1024]");
  PE_DIM_REQUIRE(d->c_z <= 256, "c_z must be <= 256");        // fused LayerNorm + bias projection: one chunk per lane
  PE_DIM_REQUIRE(d->c_tri <= 192, "c_tri must be <= 192");    // channel-major LayerNorm tile in 64 KB of LDS
  PE_DIM_REQUIRE((long long)d->n_trans * d->c_m <= 4096 && (long long)d->n_trans * d->c_z <= 4096,
                 "n_trans*c_m and n_trans*c_z must be <= 4096");
  PE_DIM_REQUIRE(d->d_msa % 8 == 0 && d->d_msa <= 32 && d->d_pair % 8 == 0 && d->d_pair <= 32,
                 "d_msa and d_pair must be 8, 16, 24 or 32");
  PE_DIM_REQUIRE(d->col_global == 0 || d->col_global == 1, "col_global must be 0 or 1");
  PE_DIM_REQUIRE(d->variant >= PE_VARIANT_PARALLEL && d->variant <= PE_VARIANT_MULTIMER, "variant must be one of PE_VARIANT_*");
  PE_DIM_REQUIRE(d->ln_eps > 0.0f && d->opm_eps > 0.0f, "ln_eps and opm_eps must be > 0");
  // GEMM row counts and the attention planes are 32-bit in the kernels
  PE_DIM_REQUIRE((long long)d->s * d->r < (1LL << 31) && (long long)d->r * d->r < (1LL << 31), "s*r and r*r must be < 2^31");
  PE_DIM_REQUIRE((long long)d->r * d->r * 4 * d->h_pair * d->d_pair < (1LL << 40), "r*r*4*h_pair*d_pair must be < 2^40");
#undef PE_DIM_REQUIRE
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
