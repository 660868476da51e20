// Tiled MFMA GEMM for gfx950 used by every linear layer (forward, dX, dW), by the
// triangle-multiplication contraction and by the outer-product-mean contractions.
//
//   C[b][m][n] = epilogue( sum_k A[b][m][k] * B[b][n][k] )
//
// Both operands are addressed as (row x, contraction k) through a two-level
// index map, so that plain matrices, transposed matrices, channel-major tensors
// and the [(i,p),(j,q)] outer-product layout are all reachable without copies:
//   addr(x,k) = (x / x_in) * x_outer + (x % x_in) * x_stride
//             + (k / k_in) * k_outer + (k % k_in) * k_stride
// An operand is either "k-contiguous" (k_stride == 1, 16-byte loads along k) or
// "x-contiguous" (x_stride == 1, 16-byte loads along x, transposed in registers
// on the way into LDS).  LDS always holds k-contiguous rows, which is what the
// 32x32 MFMA operand fragments want.
//
// Workgroup: 256 threads = 4 waves in a 2x2 grid; block tile 128x128; each wave
// owns 64x64 = 2x2 MFMA tiles (64 accumulator VGPRs).  Next k-tile is prefetched
// into registers while the current one is consumed from LDS.
#pragma once
#include <stdlib.h>
#include <string.h>
#include <type_traits>
#include "pe_common.h"

struct Operand {
  const void* ptr;
  long long batch_stride;
  int x_in; long long x_outer, x_stride;
  int k_in; long long k_outer, k_stride;
};

static inline Operand op_plain(const void* p, long long ld /*row stride, k contiguous*/, long long batch = 0) {
  Operand o; o.ptr = p; o.batch_stride = batch;
  o.x_in = 1 << 30; o.x_outer = 0; o.x_stride = ld;
  o.k_in = 1 << 30; o.k_outer = 0; o.k_stride = 1;
  return o;
}
// operand stored [k][x] (x contiguous): contraction index strided by ld
static inline Operand op_trans(const void* p, long long ld, long long batch = 0) {
  Operand o; o.ptr = p; o.batch_stride = batch;
  o.x_in = 1 << 30; o.x_outer = 0; o.x_stride = 1;
  o.k_in = 1 << 30; o.k_outer = 0; o.k_stride = ld;
  return o;
}

struct GemmShape {
  int M, N, K, batch;
  int k_chunk;  // > 0: split-K; batch index selects the k range [b*k_chunk, min(K,(b+1)*k_chunk))
  int unit_n;   // block mapping: 0 = an XCD owns (batch, m-tile) units, 1 = (batch, n-tile) units (set by the launcher)
};

// 8 consecutive storage elements <-> 8 floats (one or two 16-byte accesses)
template <typename T> PE_DEV void load8(const T* p, float (&v)[8]);
template <> PE_DEV void load8<bf16>(const bf16* p, float (&v)[8]) {
  bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int e = 0; e < 8; e++) v[e] = (float)t[e];
}
template <> PE_DEV void load8<float>(const float* p, float (&v)[8]) {
  f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int e = 0; e < 4; e++) { v[e] = a[e]; v[4 + e] = b[e]; }
}
template <typename T> PE_DEV void store8(T* p, const float (&v)[8]);
template <> PE_DEV void store8<bf16>(bf16* p, const float (&v)[8]) {
  bf16x8 t;
#pragma unroll
  for (int e = 0; e < 8; e++) t[e] = (bf16)v[e];
  *reinterpret_cast<bf16x8*>(p) = t;
}
template <> PE_DEV void store8<float>(float* p, const float (&v)[8]) {
  f32x4 a, b;
#pragma unroll
  for (int e = 0; e < 4; e++) { a[e] = v[e]; b[e] = v[4 + e]; }
  *reinterpret_cast<f32x4*>(p) = a;
  *reinterpret_cast<f32x4*>(p + 4) = b;
}

// 8 consecutive storage elements as loaded (one or two 16-byte registers groups), converted when they are used:
// a load issued early costs 4 registers (bf16) until then instead of 8
template <typename T> struct Raw8;
template <> struct Raw8<bf16> {
  bf16x8 v;
  PE_DEV void ld(const bf16* p) { v = *reinterpret_cast<const bf16x8*>(p); }
  PE_DEV void zero() {
#pragma unroll
    for (int e = 0; e < 8; e++) v[e] = (bf16)0.0f;
  }
  PE_DEV void get(float (&f)[8]) const {
#pragma unroll
    for (int e = 0; e < 8; e++) f[e] = (float)v[e];
  }
};
template <> struct Raw8<float> {
  f32x4 lo, hi;
  PE_DEV void ld(const float* p) { lo = *reinterpret_cast<const f32x4*>(p); hi = *reinterpret_cast<const f32x4*>(p + 4); }
  PE_DEV void zero() { lo = f32x4{0.0f, 0.0f, 0.0f, 0.0f}; hi = lo; }
  PE_DEV void get(float (&f)[8]) const {
#pragma unroll
    for (int e = 0; e < 4; e++) { f[e] = lo[e]; f[4 + e] = hi[e]; }
  }
};

// ---------------------------------------------------------------------------
// Epilogues
// ---------------------------------------------------------------------------
// Compile-time feature sets of the vector epilogue: a kernel instantiated with mask F keeps the
// code (and the run-time checks) of the features in F only; EF_ALL is the fully general kernel.
enum : int { EF_BIASN = 1, EF_BIASM = 2, EF_ACT = 4, EF_RELUMASK = 8, EF_AUX = 16, EF_MUL = 32, EF_ROWSCALE = 64,
             EF_SCALE2D = 128, EF_RES = 256, EF_ACC = 512, EF_OM2 = 1024, EF_ON2 = 2048, EF_ALPHA = 4096,
             EF_ALL = 8191 };

template <typename T> struct EpiGeneric {
  static constexpr bool HAS_COLSUM = false;
  static constexpr bool TM_GATE = false;
  T* out; long long out_batch;
  int om_in; long long om_outer, om_stride;
  int on_in; long long on_outer, on_stride;
  const float* bias_n; int bn_begin;     // v += bias_n[n] for n >= bn_begin
  const float* bias_m;
  float alpha;
  int act;                       // 0 none, 1 relu, 2 sigmoid
  const T* relu_mask; long long ld_rm;   // v *= (relu_mask[m][n] > 0)
  // The same decisions as one bit per element, 8 columns per byte (bit e of byte [m][n / 8] <-> column n + e):
  // bits_out is written by a ReLU epilogue (act == 1; vector epilogue only, the host makes sure it is taken),
  // bits_in replaces relu_mask where the activation itself is not needed - an eighth of a byte instead of an element
  unsigned char* bits_out; const unsigned char* bits_in; long long ld_bits;   // ld_bits: bytes per row
  T* aux; long long ld_aux;              // aux[m][n] = v (after bias/act, before mul)
  const T* mul; long long ld_mul;        // v *= mul[m][n]
  const float* rowscale;                 // v *= rowscale[m]
  const float* scale2d; int s2_mdiv, s2_ndiv, s2_ld;  // v *= scale2d[(m/mdiv)*ld + n/ndiv]
  const T* res; long long ld_res;        // v += res[m][n]
  int accumulate;                        // v += out (read-modify-write)

  // Per-row and per-column parts of the addressing are computed once per row / column.
  struct Row { long long o; long long s2; };
  struct Col { long long o; int s2; };
  PE_DEV Row row(int b, int m) const {
    Row r;
    r.o = (long long)b * out_batch +
          ((om_in >= (1 << 30)) ? (long long)m * om_stride
                                : (long long)(m / om_in) * om_outer + (long long)(m % om_in) * om_stride);
    r.s2 = scale2d ? (long long)(m / s2_mdiv) * s2_ld : 0;
    return r;
  }
  PE_DEV Col col(int n) const {
    Col c;
    c.o = (on_in >= (1 << 30)) ? (long long)n * on_stride
                               : (long long)(n / on_in) * on_outer + (long long)(n % on_in) * on_stride;
    c.s2 = scale2d ? n / s2_ndiv : 0;
    return c;
  }
  PE_DEV void operator()(int m, int n, const Row& r, const Col& c, float v) const {
    v *= alpha;
    if (bias_n && n >= bn_begin) v += bias_n[n];
    if (bias_m) v += bias_m[m];
    if (act == 1) v = fmaxf(v, 0.0f);
    else if (act == 2) v = sigmoidf_(v);
    if (bits_in) v = ((bits_in[(long long)m * ld_bits + (n >> 3)] >> (n & 7)) & 1) ? v : 0.0f;
    else if (relu_mask) v = (to_f(relu_mask[(long long)m * ld_rm + n]) > 0.0f) ? v : 0.0f;
    if (aux) aux[(long long)m * ld_aux + n] = from_f<T>(v);
    if (mul) v *= to_f(mul[(long long)m * ld_mul + n]);
    if (rowscale) v *= rowscale[m];
    if (scale2d) v *= scale2d[r.s2 + c.s2];
    if (res) v += to_f(res[(long long)m * ld_res + n]);
    long long o = r.o + c.o;
    if (accumulate) v += to_f(out[o]);
    out[o] = from_f<T>(v);
  }
  // Vector epilogue: 8 consecutive columns n..n+7 of row m at once (host checked vec_ok).  The
  // column part (offset, bias values) is the same for every row a thread handles: ColV.
  int features() const {
    int f = 0;
    if (bias_n) f |= EF_BIASN;
    if (bias_m) f |= EF_BIASM;
    if (act) f |= EF_ACT;
    if (relu_mask || bits_in) f |= EF_RELUMASK;
    if (aux) f |= EF_AUX;
    if (mul) f |= EF_MUL;
    if (rowscale) f |= EF_ROWSCALE;
    if (scale2d) f |= EF_SCALE2D;
    if (res) f |= EF_RES;
    if (accumulate) f |= EF_ACC;
    if (om_in < (1 << 30)) f |= EF_OM2;
    if (on_in < (1 << 30)) f |= EF_ON2;
    if (alpha != 1.0f) f |= EF_ALPHA;
    return f;
  }
  struct ColV { long long o; int s2; float bn[8]; };
  template <int F> PE_DEV void colv(int n, ColV& c) const {
    c.o = ((F & EF_ON2) && on_in < (1 << 30))
              ? (long long)((unsigned)n / (unsigned)on_in) * on_outer + (long long)((unsigned)n % (unsigned)on_in) * on_stride
              : (long long)n * on_stride;
    c.s2 = ((F & EF_SCALE2D) && scale2d) ? n / s2_ndiv : 0;
    const bool hb = (F & EF_BIASN) && bias_n && n >= bn_begin;
#pragma unroll
    for (int e = 0; e < 8; e++) c.bn[e] = hb ? bias_n[n + e] : 0.0f;
  }
  // The epilogue of one (row, 8 columns) group in two steps: pre8 issues every load the feature set needs (raw, not
  // converted), apply8 does the arithmetic and the stores.  A kernel that calls pre8 for several rows before the
  // first apply8 has all their loads in flight at once; behind a store the compiler cannot move a later row's
  // loads up by itself (the pointers may alias).  vec8 = pre8 + apply8.
  struct Pre8 { Raw8<T> rm, mu, rs, ac; unsigned bits; float bm, sc; };
  template <int F> PE_DEV long long out_off(int b, int m, const ColV& c) const {
    long long ro = (long long)b * out_batch;
    if ((F & EF_OM2) && om_in < (1 << 30))
      ro += (long long)((unsigned)m / (unsigned)om_in) * om_outer + (long long)((unsigned)m % (unsigned)om_in) * om_stride;
    else
      ro += (long long)m * om_stride;
    return ro + c.o;
  }
  template <int F> PE_DEV void pre8(int b, int m, int n, const ColV& c, Pre8& p) const {
    if ((F & EF_BIASM) && bias_m) p.bm = bias_m[m];
    if ((F & EF_RELUMASK) && bits_in) p.bits = bits_in[(long long)m * ld_bits + (n >> 3)];
    else if ((F & EF_RELUMASK) && relu_mask) p.rm.ld(relu_mask + (long long)m * ld_rm + n);
    if ((F & EF_MUL) && mul) p.mu.ld(mul + (long long)m * ld_mul + n);
    if (F & (EF_ROWSCALE | EF_SCALE2D)) {
      float sc = ((F & EF_ROWSCALE) && rowscale) ? rowscale[m] : 1.0f;
      if ((F & EF_SCALE2D) && scale2d) sc *= scale2d[(long long)(m / s2_mdiv) * s2_ld + c.s2];
      p.sc = sc;
    }
    if ((F & EF_RES) && res) p.rs.ld(res + (long long)m * ld_res + n);
    if ((F & EF_ACC) && accumulate) p.ac.ld(out + out_off<F>(b, m, c));
  }
  template <int F> PE_DEV void apply8(int b, int m, int n, const ColV& c, float (&v)[8], const Pre8& p) const {
    if ((F & EF_ALPHA) && alpha != 1.0f) {
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] *= alpha;
    }
    if (F & EF_BIASN) {
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] += c.bn[e];
    }
    if ((F & EF_BIASM) && bias_m) {
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] += p.bm;
    }
    if (F & EF_ACT) {
      if (act == 1) {
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = fmaxf(v[e], 0.0f);
        if (bits_out) {
          unsigned bb = 0;
#pragma unroll
          for (int e = 0; e < 8; e++) bb |= (to_f(from_f<T>(v[e])) > 0.0f ? 1u : 0u) << e;   // the decision of the STORED value
          bits_out[(long long)m * ld_bits + (n >> 3)] = (unsigned char)bb;
        }
      } else if (act == 2) {
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = sigmoidf_(v[e]);
      }
    }
    float t[8];
    if ((F & EF_RELUMASK) && bits_in) {
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] = ((p.bits >> e) & 1u) ? v[e] : 0.0f;
    } else if ((F & EF_RELUMASK) && relu_mask) {
      p.rm.get(t);
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] = (t[e] > 0.0f) ? v[e] : 0.0f;
    }
    if ((F & EF_AUX) && aux) store8<T>(aux + (long long)m * ld_aux + n, v);
    if ((F & EF_MUL) && mul) {
      p.mu.get(t);
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] *= t[e];
    }
    if (F & (EF_ROWSCALE | EF_SCALE2D)) {
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] *= p.sc;
    }
    if ((F & EF_RES) && res) {
      p.rs.get(t);
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] += t[e];
    }
    if ((F & EF_ACC) && accumulate) {
      p.ac.get(t);
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] += t[e];
    }
    store8<T>(out + out_off<F>(b, m, c), v);
  }
  template <int F> PE_DEV void vec8(int b, int m, int n, const ColV& c, float (&v)[8]) const {
    Pre8 p;
    pre8<F>(b, m, n, c, p);
    apply8<F>(b, m, n, c, v, p);
  }
  bool vec_ok(int N) const {
    auto a8 = [](long long x) { return x % 8 == 0; };
    auto p16 = [](const void* p) { return ((uintptr_t)p) % 16 == 0; };
    if (N % 8) return false;
    if (on_stride != 1 || !(on_in >= (1 << 30) || on_in % 8 == 0) || !a8(on_outer)) return false;
    if (!a8(om_stride) || !a8(om_outer) || !a8(out_batch) || !p16(out)) return false;
    if (bias_n && bn_begin % 8) return false;
    if (relu_mask && (!a8(ld_rm) || !p16(relu_mask))) return false;
    if (aux && (!a8(ld_aux) || !p16(aux))) return false;
    if (mul && (!a8(ld_mul) || !p16(mul))) return false;
    if (res && (!a8(ld_res) || !p16(res))) return false;
    if (scale2d && s2_ndiv % 8) return false;
    return true;
  }
};

template <typename T> static inline EpiGeneric<T> epi_plain(void* out, long long ldc) {
  EpiGeneric<T> e;
  memset(&e, 0, sizeof(e));
  e.out = (T*)out; e.out_batch = 0;
  e.om_in = 1 << 30; e.om_outer = 0; e.om_stride = ldc;
  e.on_in = 1 << 30; e.on_outer = 0; e.on_stride = 1;
  e.alpha = 1.0f; e.s2_mdiv = 1; e.s2_ndiv = 1;
  return e;
}

// fp32 partial sums of a split-K GEMM: part[b][m][n]
struct EpiPartial {
  static constexpr bool HAS_COLSUM = true;
  static constexpr bool TM_GATE = false;
  float* out; long long mn; int ldn;
  float* colsum;   // nullable: [batch][N] sums over k of the B operand (bias gradients ride on the dW GEMM)
  struct Row { long long o; };
  struct Col { long long o; };
  PE_DEV Row row(int b, int m) const { return Row{(long long)b * mn + (long long)m * ldn}; }
  PE_DEV Col col(int n) const { return Col{(long long)n}; }
  PE_DEV void operator()(int, int, const Row& r, const Col& c, float v) const { out[r.o + c.o] = v; }
  struct ColV {};
  int features() const { return 0; }
  template <int F> PE_DEV void colv(int, ColV&) const {}
  template <int F> PE_DEV void vec8(int b, int m, int n, const ColV&, float (&v)[8]) const {
    store8<float>(out + (long long)b * mn + (long long)m * ldn + n, v);
  }
  struct Pre8 {};
  template <int F> PE_DEV void pre8(int, int, int, const ColV&, Pre8&) const {}
  template <int F> PE_DEV void apply8(int b, int m, int n, const ColV& c, float (&v)[8], const Pre8&) const { vec8<F>(b, m, n, c, v); }
  bool vec_ok(int N) const { return N % 8 == 0 && ldn % 8 == 0 && mn % 8 == 0 && ((uintptr_t)out) % 16 == 0; }
};

// ---------------------------------------------------------------------------
// Kernel
// ---------------------------------------------------------------------------
// Epilogue of the GEMM that produces the cotangent of the gated attention output (dog = dY W_o^T): instead
// of storing dog it finishes the attention backward's first step on the tile, for head-major tensors
// (element (h, position, c) at h*plane + position*dh + c):
//   dO = dog * sigmoid(g)  (stored),  dg = dog * o * s(1-s) -> gate slot of dqkvg,  D[b][h][p] = sum_c dO * o.
// Vector epilogue only (a lane holds 8 consecutive channels of one head; the dh/8 lanes of a head are
// neighbours and always active together); the host falls back to a plain GEMM + a pass of its own otherwise.
template <typename T> struct EpiAttnPre {
  static constexpr bool HAS_COLSUM = false;
  static constexpr bool TM_GATE = false;
  const T* gate;       // gate pre-activation plane group: qkvg + 3*H*plane
  const T* o;
  T* dO;
  T* dgate;            // dqkvg + 3*H*plane
  float* D;            // [B][H][L]
  long long plane;
  int H, dh, L;
  int tr, inner;       // tr = 1: GEMM row m = p*inner + b (else m = b*L + p)
  struct Row { long long o; };
  struct Col { long long o; };
  PE_DEV Row row(int, int) const { return Row{0}; }
  PE_DEV Col col(int) const { return Col{0}; }
  PE_DEV void operator()(int, int, const Row&, const Col&, float) const {}   // element-wise path: never launched
  int features() const { return 0; }
  bool vec_ok(int N) const {
    return N % 8 == 0 && dh % 8 == 0 && (dh == 8 || dh == 16 || dh == 32) && plane % 8 == 0 &&
           ((uintptr_t)gate) % 16 == 0 && ((uintptr_t)o) % 16 == 0 && ((uintptr_t)dO) % 16 == 0 && ((uintptr_t)dgate) % 16 == 0;
  }
  struct ColV { int h, c; };
  template <int F> PE_DEV void colv(int n, ColV& cv) const {
    cv.h = (int)((unsigned)n / (unsigned)dh);
    cv.c = (int)((unsigned)n % (unsigned)dh);
  }
  // (loading gate and o in pre8, ahead of the LDS staging, measured slower here: +10 us over a step's four launches)
  struct Pre8 { long long idx; int b, pp; };
  template <int F> PE_DEV void pre8(int, int m, int, const ColV& cv, Pre8& p) const {
    if (tr) { p.pp = (int)((unsigned)m / (unsigned)inner); p.b = (int)((unsigned)m % (unsigned)inner); }
    else { p.b = (int)((unsigned)m / (unsigned)L); p.pp = (int)((unsigned)m % (unsigned)L); }
    p.idx = (long long)cv.h * plane + ((long long)p.b * L + p.pp) * dh + cv.c;
  }
  template <int F> PE_DEV void vec8(int b_, int m, int n, const ColV& cv, float (&v)[8]) const {
    Pre8 p;
    pre8<F>(b_, m, n, cv, p);
    apply8<F>(b_, m, n, cv, v, p);
  }
  template <int F> PE_DEV void apply8(int, int, int, const ColV& cv, float (&v)[8], const Pre8& p) const {
    const int b = p.b, pp = p.pp;
    const long long idx = p.idx;
    float gv[8], ov[8], dov[8], dgv[8];
    load8<T>(gate + idx, gv);
    load8<T>(o + idx, ov);
    float Dsum = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const float sg = sigmoidf_(gv[e]);
      dov[e] = to_f(from_f<T>(v[e] * sg));
      dgv[e] = v[e] * ov[e] * sg * (1.0f - sg);
      Dsum += dov[e] * ov[e];
    }
    store8<T>(dO + idx, dov);
    store8<T>(dgate + idx, dgv);
    if (dh >= 16) Dsum += __shfl_xor(Dsum, 1, 64);
    if (dh >= 32) Dsum += __shfl_xor(Dsum, 2, 64);
    if (cv.c == 0) D[((long long)b * H + cv.h) * L + pp] = Dsum;
  }
};

// Epilogue of the triangle multiplication's projection GEMM with the gating folded in (Section "Evoformer",
// triangle multiplicative update: a = mask * sigmoid(gate a) * projection a, b likewise).  The GEMM computes the
// channel-major projections out[row][position] from a weight copy whose rows come in 64-row strips: 32 projection
// rows, then the 32 gate rows of the same channels (a-side strips first, then the b-side).  A wave's 64 x 64
// accumulator block is one strip, so projection and gate of a (channel, position) sit in the same lane and register
// index of its two row halves: the gated value is formed in registers from the two values as they are stored
// (rounded to the storage type, so the result equals that of a separate gating pass over the stored tensor), and
// three 32 x 64 tiles leave the wave: projection and gate pre-activation (proj_t, rows in the order
// [a proj | a gate | b proj | b gate] that the backward pass reads) and the gated operand (a_t or b_t).
// Only the vector path of gemm_kernel (k-contiguous aligned operands) has this epilogue; the host checks.
template <typename T> struct EpiTmGate {
  static constexpr bool HAS_COLSUM = false;
  static constexpr bool TM_GATE = true;
  T* proj_t; T* a_t; T* b_t;
  const float* bias;     // [4 ct] in the order of proj_t's rows
  const float* mask;     // [Mz]
  int ct; long long Mz;
  struct Row { long long o; };
  struct Col { long long o; };
  PE_DEV Row row(int, int) const { return Row{0}; }
  PE_DEV Col col(int) const { return Col{0}; }
  PE_DEV void operator()(int, int, const Row&, const Col&, float) const {}   // element-wise path: never launched
  struct ColV {};
  struct Pre8 {};
  int features() const { return 0; }
  template <int F> PE_DEV void colv(int, ColV&) const {}
  template <int F> PE_DEV void pre8(int, int, int, const ColV&, Pre8&) const {}
  template <int F> PE_DEV void apply8(int, int, int, const ColV&, float (&)[8], const Pre8&) const {}
  template <int F> PE_DEV void vec8(int, int, int, const ColV&, float (&)[8]) const {}
  bool vec_ok(int N) const {
    auto p16 = [](const void* p) { return ((uintptr_t)p) % 16 == 0; };
    return N % 8 == 0 && Mz % 8 == 0 && ct % 32 == 0 && p16(proj_t) && p16(a_t) && p16(b_t);
  }
};

// Epilogue of the triangle multiplication's backward contractions with the gating backward folded in.  The batched
// GEMM (batch index = channel) produces the cotangent d of the gated operand a (side 0) or b (side 1) at pair
// position m * r + n; with p and g the stored projection and gate pre-activation at that (channel, position),
//   d' = round(d) * mask,   dproj = d' * sigmoid(g),   dgate = d' * p * sigmoid(g) * (1 - sigmoid(g)),
// written to the projection and gate rows of dproj_t ([a proj | a gate | b proj | b gate] x ct rows of Mz).  d is
// rounded to the storage type first, so the results equal those of a separate pass over a stored d.
template <typename T> struct EpiTmGateBwd {
  static constexpr bool HAS_COLSUM = false;
  static constexpr bool TM_GATE = false;
  const T* proj_t; const float* mask; T* dproj_t;
  int ct, r, side; long long Mz;
  struct Row { long long o; };
  struct Col { long long o; };
  PE_DEV Row row(int, int) const { return Row{0}; }
  PE_DEV Col col(int) const { return Col{0}; }
  PE_DEV void operator()(int, int, const Row&, const Col&, float) const {}   // element-wise path: never launched
  struct ColV {};
  int features() const { return 0; }
  template <int F> PE_DEV void colv(int, ColV&) const {}
  struct Pre8 { Raw8<T> p, g; Raw8<float> mk; };
  template <int F> PE_DEV void pre8(int b, int m, int n, const ColV&, Pre8& q) const {
    const long long pos = (long long)m * r + n;
    q.p.ld(proj_t + ((long long)(side * 2) * ct + b) * Mz + pos);
    q.g.ld(proj_t + ((long long)(side * 2 + 1) * ct + b) * Mz + pos);
    q.mk.ld(mask + pos);
  }
  template <int F> PE_DEV void apply8(int b, int m, int n, const ColV&, float (&v)[8], const Pre8& q) const {
    const long long pos = (long long)m * r + n;
    float pv[8], gv[8], mk[8], o0[8], o1[8];
    q.p.get(pv); q.g.get(gv); q.mk.get(mk);
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const float s = sigmoidf_(gv[e]);
      const float dd = to_f(from_f<T>(v[e])) * mk[e];
      o0[e] = dd * s;
      o1[e] = dd * pv[e] * s * (1.0f - s);
    }
    store8<T>(dproj_t + ((long long)(side * 2) * ct + b) * Mz + pos, o0);
    store8<T>(dproj_t + ((long long)(side * 2 + 1) * ct + b) * Mz + pos, o1);
  }
  template <int F> PE_DEV void vec8(int b, int m, int n, const ColV& c, float (&v)[8]) const {
    Pre8 q;
    pre8<F>(b, m, n, c, q);
    apply8<F>(b, m, n, c, v, q);
  }
  bool vec_ok(int N) const {
    auto p16 = [](const void* p) { return ((uintptr_t)p) % 16 == 0; };
    return N % 8 == 0 && r % 8 == 0 && Mz % 8 == 0 && p16(proj_t) && p16(dproj_t) && p16(mask);
  }
};

template <typename T> struct GemmCfg {
  static constexpr int VEC = Vec16<T>::N;
  static constexpr int BM = 128, BN = 128;
  static constexpr int BK = 8 * VEC;        // 64 (bf16) or 32 (fp32): 128-byte rows
  static constexpr int LDSS = BK + VEC;     // +16 bytes: conflict-free 16-byte fragment reads
  // LDS element offset of (row, 16-byte chunk c of the row, element w inside the chunk).  For a tile
  // filled by the transposing store of an x-contiguous operand (SW = true) the chunk index is
  // XOR-swizzled with the row's 8-row group, so that this store (8 rows apart per lane) does not hit
  // one bank pair 16 times.  A tile of a k-contiguous operand is stored row by row and keeps the plain
  // layout, in which the 16 rows that a fragment read touches at once fall on 16 different bank
  // groups (row stride 144 bytes); with the swizzle rows 8..15 would land on the groups of rows 0..7
  // (counters: 45 % of the LDS cycles of the k-contiguous GEMMs were bank-conflict cycles).
  template <bool SW> static PE_DEV int off(int row, int c, int w) {
    return SW ? row * LDSS + ((c ^ ((row >> 3) & 7)) * VEC) + w : row * LDSS + c * VEC + w;
  }
};

// element-wise (unaligned) variant of one 16-byte vector load: elements e = 0..VEC-1 along k (KC) or x
template <typename T, bool KC>
PE_DEV typename Vec16<T>::type gemm_load_slow(const T* base, const Operand& op, int x, int X, int k, int kend) {
  constexpr int VEC = Vec16<T>::N;
  typename Vec16<T>::type v;
#pragma unroll
  for (int e = 0; e < VEC; e++) {
    int xx = KC ? x : x + e, kk = KC ? k + e : k;
    float f = 0.0f;
    if (xx < X && kk < kend) {
      long long a = (long long)(xx / op.x_in) * op.x_outer + (long long)(xx % op.x_in) * op.x_stride +
                    (long long)(kk / op.k_in) * op.k_outer + (long long)(kk % op.k_in) * op.k_stride;
      f = to_f(base[a]);
    }
    v[e] = from_f<T>(f);
  }
  return v;
}

// Per-thread row part of the tile addressing, computed once before the k loop.
template <typename T, bool KC> struct RowAddr {
  long long a[KC ? 4 : 1];
  bool ok[KC ? 4 : 1];
  int x[KC ? 4 : 1];
  PE_DEV void init(const Operand& op, int x0, int X, int tid) {
    constexpr int VEC = Vec16<T>::N;
    if (KC) {
#pragma unroll
      for (int i = 0; i < (KC ? 4 : 1); i++) {
        int xx = x0 + (tid >> 3) + 32 * i;
        x[i] = xx;
        ok[i] = xx < X;
        int xc = ok[i] ? xx : 0;
        a[i] = (op.x_in >= (1 << 30)) ? (long long)xc * op.x_stride
                                      : (long long)((unsigned)xc / (unsigned)op.x_in) * op.x_outer +
                                            (long long)((unsigned)xc % (unsigned)op.x_in) * op.x_stride;
      }
    } else {
      constexpr int XB = 128 / VEC;
      int xx = x0 + (tid % XB) * VEC;
      x[0] = xx;
      ok[0] = xx < X;
      int xc = ok[0] ? xx : 0;
      a[0] = (op.x_in >= (1 << 30)) ? (long long)xc
                                    : (long long)((unsigned)xc / (unsigned)op.x_in) * op.x_outer +
                                          (long long)((unsigned)xc % (unsigned)op.x_in);
    }
  }
};
PE_DEV long long gemm_kaddr(const Operand& op, int k) {
  return (op.k_in >= (1 << 30)) ? (long long)k * op.k_stride
                                : (long long)((unsigned)k / (unsigned)op.k_in) * op.k_outer +
                                      (long long)((unsigned)k % (unsigned)op.k_in) * op.k_stride;
}

template <typename T, bool KC, bool AL>
PE_DEV void gemm_load_tile(typename Vec16<T>::type (&regs)[4], const T* base, const Operand& op, const RowAddr<T, KC>& ra,
                           int X, int k0, int kend, int tid) {
  constexpr int VEC = Vec16<T>::N;
  typedef typename Vec16<T>::type V;
  if (!AL) {
    if (KC) {
      int kv = tid & 7;
#pragma unroll
      for (int i = 0; i < 4; i++) regs[i] = gemm_load_slow<T, true>(base, op, ra.x[i], X, k0 + kv * VEC, kend);
    } else {
      int kb = tid / (128 / VEC);
#pragma unroll
      for (int j = 0; j < 4; j++) regs[j] = gemm_load_slow<T, false>(base, op, ra.x[0], X, k0 + kb * 4 + j, kend);
    }
    return;
  }
  if (KC) {
    // thread loads 4 vectors: row = tid/8 + 32*i, k-vector kv = tid%8
    int k = k0 + (tid & 7) * VEC;
    long long ka = gemm_kaddr(op, k);
    bool kok = k < kend;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      V v;
#pragma unroll
      for (int e = 0; e < VEC; e++) v[e] = from_f<T>(0.0f);
      if (kok && ra.ok[i]) v = *reinterpret_cast<const V*>(base + ra.a[i] + ka);
      regs[i] = v;
    }
  } else {
    // micro-block: VEC rows (x) by 4 contraction steps; 4 loads of VEC elements along x
    int kb = tid / (128 / VEC);
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int k = k0 + kb * 4 + j;
      V v;
#pragma unroll
      for (int e = 0; e < VEC; e++) v[e] = from_f<T>(0.0f);
      if (ra.ok[0] && k < kend) v = *reinterpret_cast<const V*>(base + ra.a[0] + gemm_kaddr(op, k));
      regs[j] = v;
    }
  }
}

template <typename T, bool KC>
PE_DEV void gemm_store_tile(const typename Vec16<T>::type (&regs)[4], T* lds, int tid) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int LDSS = GemmCfg<T>::LDSS;
  typedef typename Vec16<T>::type V;
  if (KC) {
    int kv = tid & 7;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int row = (tid >> 3) + 32 * i;
      *reinterpret_cast<V*>(lds + GemmCfg<T>::template off<false>(row, kv, 0)) = regs[i];
    }
  } else {
    constexpr int XB = 128 / VEC;
    int xb = tid % XB, kb = tid / XB;
    typedef T V4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int e = 0; e < VEC; e++) {
      V4 w;
      w[0] = regs[0][e]; w[1] = regs[1][e]; w[2] = regs[2][e]; w[3] = regs[3][e];
      *reinterpret_cast<V4*>(lds + GemmCfg<T>::template off<true>(xb * VEC + e, (kb * 4) / VEC, (kb * 4) % VEC)) = w;
    }
  }
}

template <typename T, bool A_KC, bool B_KC, bool AL, bool VE, class Epi, int F = EF_ALL>
__global__ __launch_bounds__(256) void gemm_kernel(Operand A, Operand B, GemmShape sh, Epi epi) {
  typedef GemmCfg<T> C;
  typedef Mma<T> MM;
  typedef typename Vec16<T>::type V;
  __shared__ __attribute__((aligned(16))) T lds_all[(C::BM + C::BN) * C::LDSS];   // 36 KB
  T* lds_a = lds_all;
  T* lds_b = lds_all + C::BM * C::LDSS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  // XCD-aware mapping: workgroup w runs on XCD w % 8.  All column tiles of one (batch, m-tile)
  // unit go to the same XCD so that its L2 serves the shared A rows; when there are too few
  // such units to balance 8 XCDs the roles of m and n are swapped (unit_n).
  const int NTm = (sh.M + C::BM - 1) / C::BM, NTn = (sh.N + C::BN - 1) / C::BN;
  const int xcd = blockIdx.x & 7, jq = blockIdx.x >> 3;
  const int NTu = sh.unit_n ? NTn : NTm, NTi = sh.unit_n ? NTm : NTn;
  const int unit = xcd + 8 * (jq / NTi);
  if (unit >= NTu * sh.batch) return;
  const int b = unit / NTu;
  const int tu = (unit % NTu) * C::BM, ti = (jq % NTi) * C::BM;
  static_assert(C::BM == C::BN, "square block tile");
  const int m0 = sh.unit_n ? ti : tu, n0 = sh.unit_n ? tu : ti;

  int kbeg = 0, kend = sh.K;
  const T* pa = (const T*)A.ptr;
  const T* pb = (const T*)B.ptr;
  if (sh.k_chunk > 0) {
    kbeg = b * sh.k_chunk;
    kend = min(sh.K, kbeg + sh.k_chunk);
  } else {
    pa += (long long)b * A.batch_stride;
    pb += (long long)b * B.batch_stride;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.0f;
  // column sums of B: for every (batch, n-tile) one of the m-tile workgroups adds up its B tiles
  bool do_cs = false;
  float cs = 0.0f;
  if constexpr (Epi::HAS_COLSUM) do_cs = epi.colsum != nullptr && tid < C::BN && (m0 / C::BM) == (n0 / C::BN + b) % NTm;

  V ra[4], rb[4];
  RowAddr<T, A_KC> rowa;
  RowAddr<T, B_KC> rowb;
  rowa.init(A, m0, sh.M, tid);
  rowb.init(B, n0, sh.N, tid);
  if (kbeg < kend) {
    gemm_load_tile<T, A_KC, AL>(ra, pa, A, rowa, sh.M, kbeg, kend, tid);
    gemm_load_tile<T, B_KC, AL>(rb, pb, B, rowb, sh.N, kbeg, kend, tid);
  }
  for (int k0 = kbeg; k0 < kend; k0 += C::BK) {
    __syncthreads();  // previous tile fully consumed
    gemm_store_tile<T, A_KC>(ra, lds_a, tid);
    gemm_store_tile<T, B_KC>(rb, lds_b, tid);
    __syncthreads();
    if (k0 + C::BK < kend) {
      gemm_load_tile<T, A_KC, AL>(ra, pa, A, rowa, sh.M, k0 + C::BK, kend, tid);
      gemm_load_tile<T, B_KC, AL>(rb, pb, B, rowb, sh.N, k0 + C::BK, kend, tid);
    }
    if constexpr (Epi::HAS_COLSUM) {
      if (do_cs) {
#pragma unroll
        for (int ch = 0; ch < C::BK / C::VEC; ch++) {
          V v = *reinterpret_cast<const V*>(lds_b + C::template off<!B_KC>(tid, ch, 0));
#pragma unroll
          for (int e = 0; e < C::VEC; e++) cs += to_f(v[e]);
        }
      }
    }
#pragma unroll
    for (int kk = 0; kk < C::BK / MM::KSTEP; kk++) {
      typename MM::frag af[2], bf[2];
#pragma unroll
      for (int t = 0; t < 2; t++) {
        const int eo = kk * MM::KSTEP + g * MM::KP;
        af[t] = MM::load(lds_a + C::template off<!A_KC>(wm * 64 + t * 32 + l32, eo / C::VEC, eo % C::VEC));
        bf[t] = MM::load(lds_b + C::template off<!B_KC>(wn * 64 + t * 32 + l32, eo / C::VEC, eo % C::VEC));
      }
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) MM::mma(acc[i][j], af[i], bf[j]);
    }
  }

  if constexpr (Epi::HAS_COLSUM) {
    if (do_cs && n0 + tid < sh.N) epi.colsum[(long long)b * sh.N + n0 + tid] = cs;
  }
  if (VE) {
    // Coalesced epilogue without workgroup barriers: every wave passes its own 64x64 accumulator
    // tile through a private LDS region, 32 rows at a time, and then handles 8 consecutive
    // columns of one row per lane (16-byte loads / stores of every epilogue operand).  LDS
    // operations of one wave execute in order, so the wave only needs the compiler to keep
    // the write and read phases apart.
    constexpr int WS = 64 + 4;
    static_assert(4 * 32 * WS * sizeof(float) <= (C::BM + C::BN) * C::LDSS * sizeof(T), "stage tiles must fit");
    float* stage = reinterpret_cast<float*>(lds_all) + wave * 32 * WS;
    const int c8 = (lane & 7) * 8, n = n0 + wn * 64 + c8;
    if constexpr (Epi::TM_GATE) {
      // the wave's 64 rows are one strip: rows 0..31 projection, 32..63 gate of channels ch0..ch0+31 of one side
      const int strip = (m0 >> 6) + wm, nside = epi.ct >> 5;
      const int side = strip / nside, ch0 = (strip % nside) * 32;
      float mk[2];
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const int col = n0 + wn * 64 + j * 32 + l32;
        mk[j] = col < sh.N ? epi.mask[col] : 0.0f;
      }
#pragma unroll
      for (int a = 0; a < 16; a++) {
        const int ch = ch0 + acc_row(g, a);
        const float bp = epi.bias[(side * 2) * epi.ct + ch], bg = epi.bias[(side * 2 + 1) * epi.ct + ch];
#pragma unroll
        for (int j = 0; j < 2; j++) {
          acc[0][j][a] = to_f(from_f<T>(acc[0][j][a] + bp));   // as stored
          acc[1][j][a] = to_f(from_f<T>(acc[1][j][a] + bg));
        }
      }
      __syncthreads();   // all waves are done with the operand tiles
#pragma unroll
      for (int rnd = 0; rnd < 3; rnd++) {
        if (rnd == 2) {
#pragma unroll
          for (int j = 0; j < 2; j++)
#pragma unroll
            for (int a = 0; a < 16; a++) acc[0][j][a] = mk[j] * sigmoidf_(acc[1][j][a]) * acc[0][j][a];
        }
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
          for (int a = 0; a < 16; a++) stage[acc_row(g, a) * WS + j * 32 + l32] = (rnd == 1) ? acc[1][j][a] : acc[0][j][a];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        T* dst = rnd == 2 ? (side ? epi.b_t : epi.a_t) : epi.proj_t + (long long)(side * 2 + rnd) * epi.ct * epi.Mz;
#pragma unroll
        for (int it = 0; it < 4; it++) {
          const int row = (lane >> 3) + it * 8;
          if (n < sh.N) {
            float vals[8];
            f32x4 lo = *reinterpret_cast<const f32x4*>(stage + row * WS + c8);
            f32x4 hi = *reinterpret_cast<const f32x4*>(stage + row * WS + c8 + 4);
#pragma unroll
            for (int e = 0; e < 4; e++) { vals[e] = lo[e]; vals[4 + e] = hi[e]; }
            store8<T>(dst + (long long)(ch0 + row) * epi.Mz + n, vals);
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
      return;
    }
    typename Epi::ColV cv;
    if (n < sh.N) epi.template colv<F>(n, cv);
    __syncthreads();   // all waves are done with the operand tiles
#pragma unroll
    for (int i = 0; i < 2; i++) {
      // the loads of the group's four rows are issued before its accumulators go through LDS, all in flight together
      // (not in the general kernel, which would go beyond 168 registers: three workgroups per CU)
      constexpr bool PF = F != EF_ALL || !std::is_same<Epi, EpiGeneric<T>>::value;
      typename Epi::Pre8 pre[4];
#pragma unroll
      for (int it = 0; it < 4; it++) {
        const int m = m0 + wm * 64 + i * 32 + (lane >> 3) + it * 8;
        if (PF && m < sh.M && n < sh.N) epi.template pre8<F>(b, m, n, cv, pre[it]);
      }
#pragma unroll
      for (int j = 0; j < 2; j++)
#pragma unroll
        for (int a = 0; a < 16; a++) stage[acc_row(g, a) * WS + j * 32 + l32] = acc[i][j][a];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 4; it++) {
        const int row = (lane >> 3) + it * 8;
        const int m = m0 + wm * 64 + i * 32 + row;
        if (m < sh.M && n < sh.N) {
          float vals[8];
          f32x4 lo = *reinterpret_cast<const f32x4*>(stage + row * WS + c8);
          f32x4 hi = *reinterpret_cast<const f32x4*>(stage + row * WS + c8 + 4);
#pragma unroll
          for (int e = 0; e < 4; e++) { vals[e] = lo[e]; vals[4 + e] = hi[e]; }
          if constexpr (PF) epi.template apply8<F>(b, m, n, cv, vals, pre[it]);
          else epi.template vec8<F>(b, m, n, cv, vals);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    return;
  }
  typename Epi::Col cols[2];
  int ncol[2];
#pragma unroll
  for (int j = 0; j < 2; j++) {
    ncol[j] = n0 + wn * 64 + j * 32 + l32;
    cols[j] = epi.col(ncol[j] < sh.N ? ncol[j] : 0);
  }
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int a = 0; a < 16; a++) {
      int m = m0 + wm * 64 + i * 32 + acc_row(g, a);
      if (m < sh.M) {
        typename Epi::Row r = epi.row(b, m);
#pragma unroll
        for (int j = 0; j < 2; j++)
          if (ncol[j] < sh.N) epi(m, ncol[j], r, cols[j], acc[i][j][a]);
      }
    }
}

// Second stage of a split-K GEMM with a full epilogue: sums the fp32 partials part[s][m][n]
// in a fixed order and applies the epilogue to 8 consecutive columns per thread.
template <typename T>
__global__ __launch_bounds__(256) void gemm_finish_kernel(const float* part, int nsplit, int M, int N, EpiGeneric<T> epi) {
  const long long v = (long long)blockIdx.x * 256 + threadIdx.x;
  const int n8 = N / 8;
  if (v >= (long long)M * n8) return;
  const int m = v / n8, n = (v % n8) * 8;
  const long long mn = (long long)M * N;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int s = 0; s < nsplit; s++) {
    float t[8];
    load8<float>(part + s * mn + (long long)m * N + n, t);
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] += t[e];
  }
  typename EpiGeneric<T>::ColV cv;
  epi.template colv<EF_ALL>(n, cv);
  epi.template vec8<EF_ALL>(0, m, n, cv, acc);
}

// ---------------------------------------------------------------------------
// Host launcher.  Returns 0 or a negative code when an operand violates the
// vector-alignment rules (nothing is launched then).
// ---------------------------------------------------------------------------
template <typename T> static inline bool gemm_operand_ok(const Operand& o, bool kc, int X, const GemmShape& sh) {
  const int VEC = Vec16<T>::N;
  if (((uintptr_t)o.ptr) % 16) return false;
  if (o.batch_stride % VEC) return false;
  if (kc) {
    if (o.k_stride != 1) return false;
    if (o.k_in % VEC && o.k_in < sh.K) return false;
    if (sh.K % VEC) return false;
    if (o.x_outer % VEC || (o.x_stride % VEC)) return false;
    if (o.k_outer % VEC) return false;
    if (sh.k_chunk > 0 && sh.k_chunk % GemmCfg<T>::BK) return false;
  } else {
    if (o.x_stride != 1) return false;
    if (o.x_in % VEC && o.x_in < X) return false;
    if (X % VEC) return false;
    if (o.x_outer % VEC || o.k_outer % VEC || o.k_stride % VEC) return false;
  }
  return true;
}

// ---------------------------------------------------------------------------
// Narrow-output variant (N <= 128, k-contiguous aligned operands, vector epilogue, no batch):
// 64 x 128 block tile, wave w owns all 64 rows of columns [32w, 32w+32).  A 128-row tile would
// give such a GEMM only M/128 workgroups (2 per CU at M = 65536), too few to overlap one
// workgroup's loads with another's arithmetic and stores; this one doubles them and needs ~100
// registers.
// ---------------------------------------------------------------------------
template <typename T, class Epi, int F>
__global__ __launch_bounds__(256) void gemm64_kernel(Operand A, Operand B, GemmShape sh, Epi epi) {
  typedef GemmCfg<T> C;
  typedef Mma<T> MM;
  typedef typename Vec16<T>::type V;
  constexpr int BM = 64;
  __shared__ __attribute__((aligned(16))) T lds_all[(BM + C::BN) * C::LDSS];   // 27 KB
  T* lds_a = lds_all;
  T* lds_b = lds_all + BM * C::LDSS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int m0 = blockIdx.x * BM;
  const T* pa = (const T*)A.ptr;
  const T* pb = (const T*)B.ptr;

  f32x16 acc[2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[i][e] = 0.0f;

  // per-thread addressing: k-vector kv = tid % 8, rows tid / 8 + 32 i (2 rows of A, 4 of B)
  const int kv = tid & 7;
  long long aa[2];
  bool aok[2];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int m = m0 + (tid >> 3) + 32 * i;
    aok[i] = m < sh.M;
    const int mc = aok[i] ? m : 0;
    aa[i] = (A.x_in >= (1 << 30)) ? (long long)mc * A.x_stride
                                  : (long long)((unsigned)mc / (unsigned)A.x_in) * A.x_outer +
                                        (long long)((unsigned)mc % (unsigned)A.x_in) * A.x_stride;
  }
  RowAddr<T, true> rowb;
  rowb.init(B, 0, sh.N, tid);
  V ra[2], rb[4];
  auto load_a = [&](int k0) {
    const int k = k0 + kv * C::VEC;
    const long long ka = gemm_kaddr(A, k);
#pragma unroll
    for (int i = 0; i < 2; i++) {
      V v;
#pragma unroll
      for (int e = 0; e < C::VEC; e++) v[e] = from_f<T>(0.0f);
      // the tile spans every output column, so these rows have no second reader: non-temporal
      if (k < sh.K && aok[i]) v = __builtin_nontemporal_load(reinterpret_cast<const V*>(pa + aa[i] + ka));
      ra[i] = v;
    }
  };
  load_a(0);
  gemm_load_tile<T, true, true>(rb, pb, B, rowb, sh.N, 0, sh.K, tid);
  for (int k0 = 0; k0 < sh.K; k0 += C::BK) {
    __syncthreads();  // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < 2; i++) *reinterpret_cast<V*>(lds_a + C::template off<false>((tid >> 3) + 32 * i, kv, 0)) = ra[i];
    gemm_store_tile<T, true>(rb, lds_b, tid);
    __syncthreads();
    if (k0 + C::BK < sh.K) {
      load_a(k0 + C::BK);
      gemm_load_tile<T, true, true>(rb, pb, B, rowb, sh.N, k0 + C::BK, sh.K, tid);
    }
#pragma unroll
    for (int kk = 0; kk < C::BK / MM::KSTEP; kk++) {
      const int eo = kk * MM::KSTEP + g * MM::KP;
      typename MM::frag bf = MM::load(lds_b + C::template off<false>(wave * 32 + l32, eo / C::VEC, eo % C::VEC));
#pragma unroll
      for (int t = 0; t < 2; t++)
        MM::mma(acc[t], MM::load(lds_a + C::template off<false>(t * 32 + l32, eo / C::VEC, eo % C::VEC)), bf);
    }
  }

  // wave-private staging of the 32 x 32 sub-tiles, then 8 consecutive columns per lane
  constexpr int WS = 32 + 4;
  static_assert(4 * 32 * WS * sizeof(float) <= (BM + C::BN) * C::LDSS * sizeof(T), "stage tiles must fit");
  float* stage = reinterpret_cast<float*>(lds_all) + wave * 32 * WS;
  const int c8 = (lane & 3) * 8, n = wave * 32 + c8;
  typename Epi::ColV cv;
  if (n < sh.N) epi.template colv<F>(n, cv);
  // every load of the epilogue is issued before the accumulators go through LDS, all rows in flight together
  typename Epi::Pre8 pre[4];
#pragma unroll
  for (int q = 0; q < 4; q++) {
    const int m = m0 + (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2);
    if (m < sh.M && n < sh.N) epi.template pre8<F>(0, m, n, cv, pre[q]);
  }
  __syncthreads();   // all waves are done with the operand tiles
#pragma unroll
  for (int i = 0; i < 2; i++) {
#pragma unroll
    for (int a = 0; a < 16; a++) stage[acc_row(g, a) * WS + l32] = acc[i][a];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int it = 0; it < 2; it++) {
      const int row = (lane >> 2) + it * 16;
      const int m = m0 + i * 32 + row;
      if (m < sh.M && n < sh.N) {
        float vals[8];
        f32x4 lo = *reinterpret_cast<const f32x4*>(stage + row * WS + c8);
        f32x4 hi = *reinterpret_cast<const f32x4*>(stage + row * WS + c8 + 4);
#pragma unroll
        for (int e = 0; e < 4; e++) { vals[e] = lo[e]; vals[4 + e] = hi[e]; }
        epi.template apply8<F>(0, m, n, cv, vals, pre[i * 2 + it]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

// ---------------------------------------------------------------------------
// Row-complete variant of the narrow-output kernel: N == 128 == the channel count of a LayerNorm, so the 64 x 128
// tile of a workgroup holds whole rows and the LayerNorm work that would follow the GEMM as a pass of its own is
// done on the tile (row sums: four lanes of a wave by shuffles, the four waves through LDS).
//   MODE 1 (forward): the generic epilogue finishes and stores the output row (the new residual stream), then
//     y = LayerNorm(stored row) with the NEXT sub-operation's gain / offset, and the row's (mean, 1/std).
//   MODE 2 (backward): the GEMM value (+ prev) is the cotangent dy of a LayerNorm output; the kernel stores
//     gout = gin + LayerNorm-backward(dy; x, stats, gain) and the workgroup's column sums of dy * xhat and dy
//     (partial[blockIdx.x][2 * 128 (+ 128 H)], summed over the workgroups by the ordered partial reduction).
//     HB = 4 or 8 (heads, padded): the pair-bias path of a triangle attention rides along (see RowLn).
// ---------------------------------------------------------------------------
template <typename T> struct RowLn {
  const float* gamma; const float* beta;   // MODE 1: gain and offset; MODE 2: gain only
  T* y; float* stats; float eps;           // MODE 1 outputs: y[M][128], stats[M][2]
  const T* prev;                           // MODE 2: nullable, added to the GEMM value (an earlier GEMM's share of dy)
  const T* x; const float* stats_in;       // MODE 2: LayerNorm input and its saved (mean, 1/std)
  const T* gin; T* gout; float* partial;   // MODE 2: gin nullable; gout may alias gin
  const T* gin2;                           // MODE 2: nullable second addend of gout (same shape as gin)
  // MODE 2 with HB > 0: the LayerNorm output also feeds a pair-bias projection b[h][row] = sum_c y[row][c] w_bias[c][h]
  // (triangle attention); its cotangent db[h][row] (fp32, [H][db_ld]) adds sum_h db[h][row] w_bias[c][h] to dy, and
  // the workgroup's partial gets 128 * H more entries: sum over its rows of y[row][c] db[h][row] at 2 * 128 + c * H + h
  const float* db; long long db_ld; const float* w_bias; int H;
  // db_r > 0: db is not [H][db_ld] in row order but the attention kernels' tiled sum (fp32 values in the query-per-lane
  // chunk order of T, db_ld elements per head): row m is pair position (q, k) = (m / db_r, m % db_r), or (k, q) when
  // db_transposed
  int db_r, db_transposed;
  // MODE 1 with HB > 0: that projection itself, bias_out[h][row] = sum_c y[row][c] w_bias[c][h] (fp32, [H][M]), and a
  // second copy of the row statistics (nullable) where the bias path's backward kernel looks for them
  float* bias_out; float* stats2;
};

// (asking for three waves per SIMD, which the variant with the bias path misses at 174 registers, makes the pair
// stack 0.7 % faster alone and the two-stream step 0.4 % slower: not asked for)
template <typename T, int F, int MODE, int HB = 0, bool G2 = false>
__global__ __launch_bounds__(256) void gemm64r_kernel(Operand A, Operand B, GemmShape sh, EpiGeneric<T> epi, RowLn<T> ln) {
  typedef GemmCfg<T> C;
  typedef Mma<T> MM;
  typedef typename Vec16<T>::type V;
  constexpr int BM = 64, CH = 128;
  __shared__ __attribute__((aligned(16))) T lds_all[(BM + C::BN) * C::LDSS];   // 27 KB
  __shared__ __attribute__((aligned(16))) float wbl[HB > 0 ? HB * CH : 4];      // w_bias as [h][c], zero beyond H
  if constexpr (HB > 0) {
    for (int i = threadIdx.x; i < HB * CH; i += 256) {
      const int hh = i / CH, c = i % CH;
      wbl[i] = hh < ln.H ? ln.w_bias[c * ln.H + hh] : 0.0f;
    }
  }
  T* lds_a = lds_all;
  T* lds_b = lds_all + BM * C::LDSS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int m0 = blockIdx.x * BM;
  const T* pa = (const T*)A.ptr;
  const T* pb = (const T*)B.ptr;

  f32x16 acc[2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int e = 0; e < 16; e++) acc[i][e] = 0.0f;

  const int kv = tid & 7;
  long long aa[2];
  bool aok[2];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int m = m0 + (tid >> 3) + 32 * i;
    aok[i] = m < sh.M;
    const int mc = aok[i] ? m : 0;
    aa[i] = (A.x_in >= (1 << 30)) ? (long long)mc * A.x_stride
                                  : (long long)((unsigned)mc / (unsigned)A.x_in) * A.x_outer +
                                        (long long)((unsigned)mc % (unsigned)A.x_in) * A.x_stride;
  }
  RowAddr<T, true> rowb;
  rowb.init(B, 0, sh.N, tid);
  V ra[2], rb[4];
  auto load_a = [&](int k0) {
    const int k = k0 + kv * C::VEC;
    const long long ka = gemm_kaddr(A, k);
#pragma unroll
    for (int i = 0; i < 2; i++) {
      V v;
#pragma unroll
      for (int e = 0; e < C::VEC; e++) v[e] = from_f<T>(0.0f);
      if (k < sh.K && aok[i]) v = *reinterpret_cast<const V*>(pa + aa[i] + ka);
      ra[i] = v;
    }
  };
  load_a(0);
  gemm_load_tile<T, true, true>(rb, pb, B, rowb, sh.N, 0, sh.K, tid);
  for (int k0 = 0; k0 < sh.K; k0 += C::BK) {
    __syncthreads();  // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < 2; i++) *reinterpret_cast<V*>(lds_a + C::template off<false>((tid >> 3) + 32 * i, kv, 0)) = ra[i];
    gemm_store_tile<T, true>(rb, lds_b, tid);
    __syncthreads();
    if (k0 + C::BK < sh.K) {
      load_a(k0 + C::BK);
      gemm_load_tile<T, true, true>(rb, pb, B, rowb, sh.N, k0 + C::BK, sh.K, tid);
    }
#pragma unroll
    for (int kk = 0; kk < C::BK / MM::KSTEP; kk++) {
      const int eo = kk * MM::KSTEP + g * MM::KP;
      typename MM::frag bf = MM::load(lds_b + C::template off<false>(wave * 32 + l32, eo / C::VEC, eo % C::VEC));
#pragma unroll
      for (int t = 0; t < 2; t++)
        MM::mma(acc[t], MM::load(lds_a + C::template off<false>(t * 32 + l32, eo / C::VEC, eo % C::VEC)), bf);
    }
  }

  // wave-private staging of the 32 x 32 sub-tiles; lane -> 8 consecutive columns of the rows
  // rloc(q) = 32 (q / 2) + 16 (q % 2) + lane / 4, q = 0..3
  constexpr int WS = 32 + 4;
  static_assert((4 * 32 * WS + 4 * BM * 2) * sizeof(float) <= (BM + C::BN) * C::LDSS * sizeof(T), "stage tiles and row sums must fit");
  float* stage = reinterpret_cast<float*>(lds_all) + wave * 32 * WS;
  float* rowred = reinterpret_cast<float*>(lds_all) + 4 * 32 * WS;   // [wave][row][2]
  const int c8 = (lane & 3) * 8, n = wave * 32 + c8;
  float vals[4][8];
  // every global load of the epilogue is issued here, before the accumulators go through LDS (raw registers)
  float gm[8];
#pragma unroll
  for (int e = 0; e < 8; e++) gm[e] = ln.gamma[n + e];
  typename EpiGeneric<T>::ColV cv;
  typename EpiGeneric<T>::Pre8 pre[MODE == 1 ? 4 : 1];
  Raw8<T> xr[MODE == 2 ? 4 : 1], pr[MODE == 2 ? 4 : 1], gr[MODE == 2 ? 4 : 1], g2[G2 ? 4 : 1];   // G2: the kernel takes gin2
  float mean[MODE == 2 ? 4 : 1], rstd[MODE == 2 ? 4 : 1];
  float dbv[HB > 0 ? 4 : 1][HB > 0 ? HB : 1];
  if constexpr (MODE == 1) {
    epi.template colv<F>(n, cv);
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int m = m0 + (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2);
      if (m < sh.M) epi.template pre8<F>(0, m, n, cv, pre[q]);
    }
  } else {
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int m = m0 + (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2);
      xr[q].zero(); pr[q].zero(); gr[q].zero();
      if constexpr (G2) g2[q].zero();
      mean[q] = 0.0f; rstd[q] = 0.0f;
      if constexpr (HB > 0) {
#pragma unroll
        for (int hh = 0; hh < HB; hh++) dbv[q][hh] = 0.0f;
        if (m < sh.M) {
          long long off = m;
          if (ln.db_r > 0) {   // gather from the tiled sum: element e of lane (query, g) of key tile kq >> 5 holds key offset 8 (e / 4) + 4 g + e % 4
            const int a0 = (int)((unsigned)m / (unsigned)ln.db_r), a1 = (int)((unsigned)m % (unsigned)ln.db_r);
            const int qq = ln.db_transposed ? a1 : a0, kq = ln.db_transposed ? a0 : a1;
            const int o = kq & 31, gg = (o >> 2) & 1, ee = ((o >> 3) << 2) | (o & 3);
            off = bias_chunk_off<T>(kq >> 5, ee / BiasChunk<T>::CH, gg, qq, ln.db_r) + ee % BiasChunk<T>::CH;
          }
#pragma unroll
          for (int hh = 0; hh < HB; hh++)
            if (hh < ln.H) dbv[q][hh] = ln.db[(long long)hh * ln.db_ld + off];
        }
      }
      if (m < sh.M) {
        xr[q].ld(ln.x + (long long)m * CH + n);
        if (ln.prev) pr[q].ld(ln.prev + (long long)m * CH + n);
        if (ln.gin) gr[q].ld(ln.gin + (long long)m * CH + n);
        if constexpr (G2) g2[q].ld(ln.gin2 + (long long)m * CH + n);
        mean[q] = ln.stats_in[(long long)m * 2];
        rstd[q] = ln.stats_in[(long long)m * 2 + 1];
      }
    }
  }
  __syncthreads();   // all waves are done with the operand tiles
#pragma unroll
  for (int i = 0; i < 2; i++) {
#pragma unroll
    for (int a = 0; a < 16; a++) stage[acc_row(g, a) * WS + l32] = acc[i][a];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int it = 0; it < 2; it++) {
      const int row = (lane >> 2) + it * 16;
      f32x4 lo = *reinterpret_cast<const f32x4*>(stage + row * WS + c8);
      f32x4 hi = *reinterpret_cast<const f32x4*>(stage + row * WS + c8 + 4);
#pragma unroll
      for (int e = 0; e < 4; e++) { vals[i * 2 + it][e] = lo[e]; vals[i * 2 + it][4 + e] = hi[e]; }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  auto quad_sum = [](float v) { v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); return v; };
  auto row_total = [&](int rloc, int j) {
    return (rowred[(0 * BM + rloc) * 2 + j] + rowred[(1 * BM + rloc) * 2 + j]) + (rowred[(2 * BM + rloc) * 2 + j] + rowred[(3 * BM + rloc) * 2 + j]);
  };
  if constexpr (MODE == 1) {
    float mu[4];
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int rloc = (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2), m = m0 + rloc;
      float s = 0.0f;
      if (m < sh.M) {
        epi.template apply8<F>(0, m, n, cv, vals[q], pre[q]);
#pragma unroll
        for (int e = 0; e < 8; e++) { vals[q][e] = to_f(from_f<T>(vals[q][e])); s += vals[q][e]; }   // the stored row
      }
      s = quad_sum(s);
      if ((lane & 3) == 0) rowred[(wave * BM + rloc) * 2] = s;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int rloc = (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2);
      mu[q] = row_total(rloc, 0) * (1.0f / CH);
      float s = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; e++) { const float t = vals[q][e] - mu[q]; s += t * t; }
      s = quad_sum(s);
      if ((lane & 3) == 0) rowred[(wave * BM + rloc) * 2 + 1] = s;
    }
    __syncthreads();
    float bt[8];
#pragma unroll
    for (int e = 0; e < 8; e++) bt[e] = ln.beta[n + e];
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int rloc = (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2), m = m0 + rloc;
      if (m < sh.M) {
        const float rstd = rsqrtf(row_total(rloc, 1) * (1.0f / CH) + ln.eps);
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (vals[q][e] - mu[q]) * rstd * gm[e] + bt[e];
        store8<T>(ln.y + (long long)m * CH + n, o);
        if (wave == 0 && (lane & 3) == 0) {
          ln.stats[(long long)m * 2] = mu[q]; ln.stats[(long long)m * 2 + 1] = rstd;
          if (HB > 0 && ln.stats2) { ln.stats2[(long long)m * 2] = mu[q]; ln.stats2[(long long)m * 2 + 1] = rstd; }
        }
        if constexpr (HB > 0) {   // this lane's share of the row's bias projection (the staging area is free by now)
          float* brd = reinterpret_cast<float*>(lds_all);   // [wave][row][HB]
#pragma unroll
          for (int hh = 0; hh < HB; hh++) {
            const f32x4 w0 = *reinterpret_cast<const f32x4*>(wbl + hh * CH + n);
            const f32x4 w1 = *reinterpret_cast<const f32x4*>(wbl + hh * CH + n + 4);
            float t = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; e++) t += o[e] * w0[e] + o[4 + e] * w1[e];
            t = quad_sum(t);
            if ((lane & 3) == 0) brd[(wave * BM + rloc) * HB + hh] = t;
          }
        }
      }
    }
    if constexpr (HB > 0) {
      static_assert(4 * BM * HB <= 4 * 32 * WS, "bias row sums must fit in the staging area");
      const float* brd = reinterpret_cast<const float*>(lds_all);
      __syncthreads();
      const int row = tid & 63, m = m0 + row;
      if (m < sh.M) {
#pragma unroll
        for (int hh = tid >> 6; hh < HB; hh += 4)
          if (hh < ln.H)
            ln.bias_out[(long long)hh * sh.M + m] = (brd[(0 * BM + row) * HB + hh] + brd[(1 * BM + row) * HB + hh]) +
                                                    (brd[(2 * BM + row) * HB + hh] + brd[(3 * BM + row) * HB + hh]);
      }
    }
  } else {
    float dgs[8], dbs[8];   // xhat is recomputed from the raw row in the second step instead of kept (32 registers)
#pragma unroll
    for (int e = 0; e < 8; e++) { dgs[e] = 0.0f; dbs[e] = 0.0f; }
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int rloc = (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2), m = m0 + rloc;
      float s1 = 0.0f, s2 = 0.0f;
      if (m < sh.M) {
        float xv[8], pv[8];
        xr[q].get(xv);
        pr[q].get(pv);
        if constexpr (HB > 0) {
#pragma unroll
          for (int hh = 0; hh < HB; hh++) {
            const f32x4 w0 = *reinterpret_cast<const f32x4*>(wbl + hh * CH + n);
            const f32x4 w1 = *reinterpret_cast<const f32x4*>(wbl + hh * CH + n + 4);
#pragma unroll
            for (int e = 0; e < 4; e++) { pv[e] += dbv[q][hh] * w0[e]; pv[4 + e] += dbv[q][hh] * w1[e]; }
          }
        }
#pragma unroll
        for (int e = 0; e < 8; e++) {
          const float dv = vals[q][e] + pv[e];
          const float xh = (xv[e] - mean[q]) * rstd[q];
          const float dx = dv * gm[e];
          dgs[e] += dv * xh;
          dbs[e] += dv;
          s1 += dx;
          s2 += dx * xh;
          vals[q][e] = dx;
        }
      }
      s1 = quad_sum(s1);
      s2 = quad_sum(s2);
      if ((lane & 3) == 0) { rowred[(wave * BM + rloc) * 2] = s1; rowred[(wave * BM + rloc) * 2 + 1] = s2; }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const int rloc = (q >> 1) * 32 + (q & 1) * 16 + (lane >> 2), m = m0 + rloc;
      if (m < sh.M) {
        const float s1 = row_total(rloc, 0) * (1.0f / CH), s2 = row_total(rloc, 1) * (1.0f / CH);
        float o[8], xv[8];
        gr[q].get(o);
        if constexpr (G2) {
          float o2[8];
          g2[q].get(o2);
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] += o2[e];
        }
        xr[q].get(xv);
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] += (vals[q][e] - s1 - (xv[e] - mean[q]) * rstd[q] * s2) * rstd[q];
        store8<T>(ln.gout + (long long)m * CH + n, o);
      }
    }
    // column sums over the workgroup's 64 rows: the 16 lanes of a wave with the same columns, rows in a fixed order
#pragma unroll
    for (int e = 0; e < 8; e++) {
#pragma unroll
      for (int o = 4; o < 64; o <<= 1) { dgs[e] += __shfl_xor(dgs[e], o, 64); dbs[e] += __shfl_xor(dbs[e], o, 64); }
    }
    const int plen = 2 * CH + (HB > 0 ? CH * ln.H : 0);
    float* pp = ln.partial + (long long)blockIdx.x * plen;
    if (lane < 4) {
      store8<float>(pp + n, dgs);
      store8<float>(pp + CH + n, dbs);
    }
    if constexpr (HB > 0) {
      // bias weight: sum over the 64 rows of y[row][c] db[h][row], 32 rows at a time through LDS (y in fp32 where the
      // accumulator staging was): thread -> channel c = tid % 128 and HB / 2 heads, rows in order
      constexpr int YL = CH + 4, HH2 = HB / 2;
      static_assert(32 * YL + 32 * HB <= 4 * 32 * WS, "y tile and db rows must fit in the staging area");
      float* ytile = reinterpret_cast<float*>(lds_all);
      float* dbl = ytile + 32 * YL;
      float bt[8], accw[HH2];
#pragma unroll
      for (int e = 0; e < 8; e++) bt[e] = ln.beta[n + e];
#pragma unroll
      for (int j = 0; j < HH2; j++) accw[j] = 0.0f;
      const int cc = tid & 127, h0 = (tid >> 7) * HH2;
#pragma unroll
      for (int half = 0; half < 2; half++) {
        __syncthreads();   // half 0: every wave is past its row-sum reads; half 1: the first half's tile has been read
#pragma unroll
        for (int qq = 0; qq < 2; qq++) {
          const int q = half * 2 + qq, lr = qq * 16 + (lane >> 2), m = m0 + half * 32 + lr;
          float xv[8], yv[8];
          xr[q].get(xv);
#pragma unroll
          for (int e = 0; e < 8; e++) yv[e] = (m < sh.M) ? (xv[e] - mean[q]) * rstd[q] * gm[e] + bt[e] : 0.0f;
          *reinterpret_cast<f32x4*>(ytile + lr * YL + n) = f32x4{yv[0], yv[1], yv[2], yv[3]};
          *reinterpret_cast<f32x4*>(ytile + lr * YL + n + 4) = f32x4{yv[4], yv[5], yv[6], yv[7]};
          if (wave == 0 && (lane & 3) == 0) {
#pragma unroll
            for (int hh = 0; hh < HB; hh++) dbl[lr * HB + hh] = dbv[q][hh];
          }
        }
        __syncthreads();
        for (int row = 0; row < 32; row++) {
          const float yv = ytile[row * YL + cc];
#pragma unroll
          for (int j = 0; j < HH2; j++) accw[j] += yv * dbl[row * HB + h0 + j];
        }
      }
#pragma unroll
      for (int j = 0; j < HH2; j++)
        if (h0 + j < ln.H) pp[2 * CH + cc * ln.H + h0 + j] = accw[j];
    }
  }
}

// ---------------------------------------------------------------------------
// The LayerNorm-backward epilogue (MODE 2 of gemm64r_kernel) for 256 channels (the MSA representation): 64 x 256
// tile, wave w owns all 64 rows of columns [64 w, 64 w + 64) as 2 x 2 MFMA tiles.  The epilogue goes through the two
// 32-row halves one after the other (rows are independent), so that only one half's values, raw loads and row
// statistics are live at a time; a lane holds 8 consecutive columns of four rows per half, a row's sums come from
// eight lanes and four waves.  Without the earlier share of dy, the bias path and the second addend.
// The forward counterpart (output projection + next LayerNorm on such tiles) was built and measured: the MSA stack
// alone 9 us faster, the two-stream step 18 us slower (64-row tiles take in 25 % more operand bytes per flop than
// the 128 x 128 kernel they replace, and the forward GEMMs are the ones that run at its full rate): not kept.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gemm64w_kernel(Operand A, Operand B, GemmShape sh, RowLn<T> ln) {
  typedef GemmCfg<T> C;
  typedef Mma<T> MM;
  typedef typename Vec16<T>::type V;
  constexpr int BM = 64, CH = 256;
  __shared__ __attribute__((aligned(16))) T lds_all[(BM + CH) * C::LDSS];   // 45 KB
  T* lds_a = lds_all;
  T* lds_b = lds_all + BM * C::LDSS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int m0 = blockIdx.x * BM;
  const T* pa = (const T*)A.ptr;
  const T* pb = (const T*)B.ptr;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.0f;

  const int kv = tid & 7;
  long long aa[2];
  bool aok[2];
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int m = m0 + (tid >> 3) + 32 * i;
    aok[i] = m < sh.M;
    const int mc = aok[i] ? m : 0;
    aa[i] = (A.x_in >= (1 << 30)) ? (long long)mc * A.x_stride
                                  : (long long)((unsigned)mc / (unsigned)A.x_in) * A.x_outer +
                                        (long long)((unsigned)mc % (unsigned)A.x_in) * A.x_stride;
  }
  RowAddr<T, true> rowb0, rowb1;
  rowb0.init(B, 0, sh.N, tid);
  rowb1.init(B, 128, sh.N, tid);
  V ra[2], rb0[4], rb1[4];
  auto load_a = [&](int k0) {
    const int k = k0 + kv * C::VEC;
    const long long ka = gemm_kaddr(A, k);
#pragma unroll
    for (int i = 0; i < 2; i++) {
      V v;
#pragma unroll
      for (int e = 0; e < C::VEC; e++) v[e] = from_f<T>(0.0f);
      if (k < sh.K && aok[i]) v = *reinterpret_cast<const V*>(pa + aa[i] + ka);
      ra[i] = v;
    }
  };
  load_a(0);
  gemm_load_tile<T, true, true>(rb0, pb, B, rowb0, sh.N, 0, sh.K, tid);
  gemm_load_tile<T, true, true>(rb1, pb, B, rowb1, sh.N, 0, sh.K, tid);
  for (int k0 = 0; k0 < sh.K; k0 += C::BK) {
    __syncthreads();  // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < 2; i++) *reinterpret_cast<V*>(lds_a + C::template off<false>((tid >> 3) + 32 * i, kv, 0)) = ra[i];
    gemm_store_tile<T, true>(rb0, lds_b, tid);
    gemm_store_tile<T, true>(rb1, lds_b + 128 * C::LDSS, tid);
    __syncthreads();
    if (k0 + C::BK < sh.K) {
      load_a(k0 + C::BK);
      gemm_load_tile<T, true, true>(rb0, pb, B, rowb0, sh.N, k0 + C::BK, sh.K, tid);
      gemm_load_tile<T, true, true>(rb1, pb, B, rowb1, sh.N, k0 + C::BK, sh.K, tid);
    }
#pragma unroll
    for (int kk = 0; kk < C::BK / MM::KSTEP; kk++) {
      const int eo = kk * MM::KSTEP + g * MM::KP;
      typename MM::frag af[2], bf[2];
#pragma unroll
      for (int t = 0; t < 2; t++) {
        af[t] = MM::load(lds_a + C::template off<false>(t * 32 + l32, eo / C::VEC, eo % C::VEC));
        bf[t] = MM::load(lds_b + C::template off<false>(wave * 64 + t * 32 + l32, eo / C::VEC, eo % C::VEC));
      }
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) MM::mma(acc[i][j], af[i], bf[j]);
    }
  }

  constexpr int WS = 64 + 4;
  static_assert((4 * 32 * WS + 2 * 4 * 32 * 2) * sizeof(float) <= (BM + CH) * C::LDSS * sizeof(T), "stage tiles and row sums must fit");
  float* stage = reinterpret_cast<float*>(lds_all) + wave * 32 * WS;
  float* rowred_all = reinterpret_cast<float*>(lds_all) + 4 * 32 * WS;   // [half][wave][row][2]
  const int c8 = (lane & 7) * 8, n = wave * 64 + c8;
  auto oct_sum = [](float v) { v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64); return v; };
  float gm[8];
#pragma unroll
  for (int e = 0; e < 8; e++) gm[e] = ln.gamma[n + e];
  float dgs[8], dbs[8];
#pragma unroll
  for (int e = 0; e < 8; e++) { dgs[e] = 0.0f; dbs[e] = 0.0f; }
  __syncthreads();   // all waves are done with the operand tiles
#pragma unroll
  for (int i = 0; i < 2; i++) {
    float* rowred = rowred_all + i * 4 * 32 * 2;
    auto row_total = [&](int r, int j) {
      return (rowred[(0 * 32 + r) * 2 + j] + rowred[(1 * 32 + r) * 2 + j]) + (rowred[(2 * 32 + r) * 2 + j] + rowred[(3 * 32 + r) * 2 + j]);
    };
    // the half's global loads first, then its accumulators through LDS
    Raw8<T> xr[4], gr[4];
    float mean[4], rstd[4];
#pragma unroll
    for (int it = 0; it < 4; it++) {
      const int m = m0 + i * 32 + (lane >> 3) + it * 8;
      xr[it].zero(); gr[it].zero();
      mean[it] = 0.0f; rstd[it] = 0.0f;
      if (m < sh.M) {
        xr[it].ld(ln.x + (long long)m * CH + n);
        if (ln.gin) gr[it].ld(ln.gin + (long long)m * CH + n);
        mean[it] = ln.stats_in[(long long)m * 2];
        rstd[it] = ln.stats_in[(long long)m * 2 + 1];
      }
    }
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int a = 0; a < 16; a++) stage[acc_row(g, a) * WS + j * 32 + l32] = acc[i][j][a];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float vals[4][8];
#pragma unroll
    for (int it = 0; it < 4; it++) {
      const int row = (lane >> 3) + it * 8;
      f32x4 lo = *reinterpret_cast<const f32x4*>(stage + row * WS + c8);
      f32x4 hi = *reinterpret_cast<const f32x4*>(stage + row * WS + c8 + 4);
#pragma unroll
      for (int e = 0; e < 4; e++) { vals[it][e] = lo[e]; vals[it][4 + e] = hi[e]; }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    {
#pragma unroll
      for (int it = 0; it < 4; it++) {
        const int r = (lane >> 3) + it * 8, m = m0 + i * 32 + r;
        float s1 = 0.0f, s2 = 0.0f;
        if (m < sh.M) {
          float xv[8];
          xr[it].get(xv);
#pragma unroll
          for (int e = 0; e < 8; e++) {
            const float dv = vals[it][e];
            const float xh = (xv[e] - mean[it]) * rstd[it];
            const float dx = dv * gm[e];
            dgs[e] += dv * xh;
            dbs[e] += dv;
            s1 += dx;
            s2 += dx * xh;
            vals[it][e] = dx;
          }
        }
        s1 = oct_sum(s1);
        s2 = oct_sum(s2);
        if ((lane & 7) == 0) { rowred[(wave * 32 + r) * 2] = s1; rowred[(wave * 32 + r) * 2 + 1] = s2; }
      }
      __syncthreads();
#pragma unroll
      for (int it = 0; it < 4; it++) {
        const int r = (lane >> 3) + it * 8, m = m0 + i * 32 + r;
        if (m < sh.M) {
          const float s1 = row_total(r, 0) * (1.0f / CH), s2 = row_total(r, 1) * (1.0f / CH);
          float o[8], xv[8];
          gr[it].get(o);
          xr[it].get(xv);
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] += (vals[it][e] - s1 - (xv[e] - mean[it]) * rstd[it] * s2) * rstd[it];
          store8<T>(ln.gout + (long long)m * CH + n, o);
        }
      }
    }
  }
  {
    // column sums over the workgroup's 64 rows: the 8 lanes of a wave with the same columns
#pragma unroll
    for (int e = 0; e < 8; e++) {
#pragma unroll
      for (int o = 8; o < 64; o <<= 1) { dgs[e] += __shfl_xor(dgs[e], o, 64); dbs[e] += __shfl_xor(dbs[e], o, 64); }
    }
    if (lane < 8) {
      float* pp = ln.partial + (long long)blockIdx.x * 2 * CH;
      store8<float>(pp + n, dgs);
      store8<float>(pp + CH + n, dbs);
    }
  }
}

// feature mask of the kernel instantiation that the last launch_gemm call of this host thread took (EF_ALL = the
// general kernel); read by the caller to label the launch with the exact kernel symbol
static thread_local int g_gemm_last_features = EF_ALL;

// launches the row-complete kernel when its conditions hold (N == 128, k-contiguous aligned operands, the vector
// epilogue, one of the feature sets below); false: nothing was launched and the caller takes the separate kernels
template <typename T, int MODE>
static inline bool launch_gemm64r(hipStream_t st, const Operand& A, const Operand& B, const GemmShape& sh, const EpiGeneric<T>& epi,
                                  const RowLn<T>& ln, bool launch = true) {
  if ((sh.N != 128 && sh.N != 256) || sh.M <= 0 || sh.batch != 1 || sh.k_chunk != 0) return false;
  if (A.k_stride != 1 || B.k_stride != 1) return false;
  if (!gemm_operand_ok<T>(A, true, sh.M, sh) || !gemm_operand_ok<T>(B, true, sh.N, sh)) return false;
  auto p16 = [](const void* p) { return ((uintptr_t)p) % 16 == 0; };
  dim3 grid((unsigned)((sh.M + 63) / 64)), block(256);
  if (sh.N == 256) {   // the 256-channel kernel: LayerNorm backward only, without the options
    if constexpr (MODE == 1) {
      return false;
    } else {
      if (ln.prev || ln.db || ln.gin2) return false;
      if (!p16(ln.x) || !p16(ln.gout) || (ln.gin && !p16(ln.gin)) || !p16(ln.partial)) return false;
      if (!launch) return true;
      hipLaunchKernelGGL((gemm64w_kernel<T>), grid, block, 0, st, A, B, sh, ln);
      g_gemm_last_features = 0;
      return true;
    }
  }
  if constexpr (MODE == 1) {
    if (!epi.vec_ok(sh.N) || !p16(ln.y)) return false;
    const int f = epi.features();
    if (ln.bias_out && (ln.H < 1 || ln.H > 8 || !ln.w_bias)) return false;
    if (!launch) return (f & ~(EF_BIASN | EF_AUX | EF_MUL | EF_RES)) == 0;
#define PE_GEMM64R_SPEC(S)                                                                                             \
    if ((f & ~(S)) == 0) {                                                                                             \
      if (!ln.bias_out) hipLaunchKernelGGL((gemm64r_kernel<T, (S), 1, 0>), grid, block, 0, st, A, B, sh, epi, ln);     \
      else if (ln.H <= 4) hipLaunchKernelGGL((gemm64r_kernel<T, (S), 1, 4>), grid, block, 0, st, A, B, sh, epi, ln);   \
      else hipLaunchKernelGGL((gemm64r_kernel<T, (S), 1, 8>), grid, block, 0, st, A, B, sh, epi, ln);                  \
      g_gemm_last_features = (S);                                                                                      \
      return true;                                                                                                     \
    }
    PE_GEMM64R_SPEC(EF_BIASN | EF_RES)
    PE_GEMM64R_SPEC(EF_BIASN | EF_AUX | EF_MUL | EF_RES)
#undef PE_GEMM64R_SPEC
    return false;
  } else {
    if (!p16(ln.x) || !p16(ln.gout) || (ln.gin && !p16(ln.gin)) || (ln.gin2 && !p16(ln.gin2)) || (ln.prev && !p16(ln.prev)) || !p16(ln.partial)) return false;
    if (ln.db && (ln.H < 1 || ln.H > 8 || !ln.w_bias || !ln.beta)) return false;
    if (ln.gin2 && ln.db) return false;   // no instantiation with both
    if (!launch) return true;
    if (ln.gin2) hipLaunchKernelGGL((gemm64r_kernel<T, 0, 2, 0, true>), grid, block, 0, st, A, B, sh, epi, ln);
    else if (!ln.db) hipLaunchKernelGGL((gemm64r_kernel<T, 0, 2, 0>), grid, block, 0, st, A, B, sh, epi, ln);
    else if (ln.H <= 4) hipLaunchKernelGGL((gemm64r_kernel<T, 0, 2, 4>), grid, block, 0, st, A, B, sh, epi, ln);
    else hipLaunchKernelGGL((gemm64r_kernel<T, 0, 2, 8>), grid, block, 0, st, A, B, sh, epi, ln);
    g_gemm_last_features = 0;
    return true;
  }
}

// ---------------------------------------------------------------------------
// Parameter-gradient variant (bf16, both operands x-contiguous and 16-byte aligned, fp32 partials):
//   part[b][m][n] = sum over the k range of split b of A[k][m] * B[k][n]
// The operand tiles stay in their memory order in LDS ([k][x], 16-byte stores, no register
// transpose).  The MFMA fragments (8 consecutive k of one row per lane) are gathered with eight
// 32-bit reads per pair of MFMA row blocks: lane l reads the rows (2l, 2l+1) of its wave's 64-row
// strip at eight k and splits the halves, so MFMA row block i of a wave covers the strip's rows
// 2r + i (r = 0..31) instead of 32 consecutive ones; the accumulator mapping below follows.
// Rows k and k+8 are read by the two lane halves at once: the 16-byte chunk index of a row is
// XOR-ed with 8 when (k / 8) is odd, which puts them on disjoint banks.
// KG wave groups (4 waves each) take alternate k-tiles of the workgroup's range, each with its own
// tiles in LDS and its own register prefetch, which doubles the bytes in flight per CU without a
// second set of partials; the groups' accumulators are added through LDS at the end.
// ---------------------------------------------------------------------------
// partial sums are read back by the deferred reduction at the end of the backward pass, long after the L2 has
// turned over: written non-temporally, they do not displace the lines the neighbouring kernels share
PE_DEV void dw_store_partial(float* p, f32x2 v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x2*>(p)); }
struct XAddr {   // per-thread x part of the tile addressing: 8 consecutive x, 4 consecutive k per tile
  long long a; bool ok;
  PE_DEV void init(const Operand& op, int x0, int X, int xb) {
    const int xx = x0 + xb * 8;
    ok = xx < X;
    const int xc = ok ? xx : 0;
    a = (op.x_in >= (1 << 30)) ? (long long)xc
                               : (long long)((unsigned)xc / (unsigned)op.x_in) * op.x_outer + (long long)((unsigned)xc % (unsigned)op.x_in);
  }
};
PE_DEV void dwx_load(bf16x8 (&regs)[4], const bf16* base, const Operand& op, const XAddr& xa, int k, int kend) {
  // k, k+1, k+2, k+3 through the two-level map: one division for the first, steps for the rest
  unsigned q = 0, r = (unsigned)k;
  const bool two = op.k_in < (1 << 30);
  if (two) { q = (unsigned)k / (unsigned)op.k_in; r = (unsigned)k % (unsigned)op.k_in; }
#pragma unroll
  for (int j = 0; j < 4; j++) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; e++) v[e] = (bf16)0.0f;
    if (xa.ok && k + j < kend) v = *reinterpret_cast<const bf16x8*>(base + xa.a + (long long)q * op.k_outer + (long long)r * op.k_stride);
    regs[j] = v;
    r++;
    if (two && r == (unsigned)op.k_in) { r = 0; q++; }
  }
}

template <int KG>
__global__ __launch_bounds__(256 * KG) void gemm_dwx_kernel(Operand A, Operand B, GemmShape sh, EpiPartial epi) {
  constexpr int BM = 128, BK = 64;
  constexpr int TILE = BK * 128;                       // elements of one operand tile (16 KB)
  extern __shared__ __attribute__((aligned(16))) bf16 lds_all[];   // KG * 2 * TILE elements (32 KB per group)
  const int kg = threadIdx.x >> 8, tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  bf16* lds_a = lds_all + kg * 2 * TILE;
  bf16* lds_b = lds_a + TILE;

  // same XCD-aware workgroup -> (batch, m-tile, n-tile) mapping as gemm_kernel
  const int NTm = (sh.M + BM - 1) / BM, NTn = (sh.N + BM - 1) / BM;
  const int xcd = blockIdx.x & 7, jq = blockIdx.x >> 3;
  const int NTu = sh.unit_n ? NTn : NTm, NTi = sh.unit_n ? NTm : NTn;
  const int unit = xcd + 8 * (jq / NTi);
  if (unit >= NTu * sh.batch) return;
  const int b = unit / NTu;
  const int tu = (unit % NTu) * BM, ti = (jq % NTi) * BM;
  const int m0 = sh.unit_n ? ti : tu, n0 = sh.unit_n ? tu : ti;

  int kbeg = 0, kend = sh.K;
  const bf16* pa = (const bf16*)A.ptr;
  const bf16* pb = (const bf16*)B.ptr;
  if (sh.k_chunk > 0) {
    kbeg = b * sh.k_chunk;
    kend = min(sh.K, kbeg + sh.k_chunk);
  } else {
    pa += (long long)b * A.batch_stride;
    pb += (long long)b * B.batch_stride;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.0f;

  // loader role: 8 x (chunk xb) at k rows 4 kb .. 4 kb + 3 of the tile
  const int xb = tid & 15, kb = tid >> 4;
  XAddr xa, xbb;
  xa.init(A, m0, sh.M, xb);
  xbb.init(B, n0, sh.N, xb);
  const int st_off = kb * 4 * 128 + ((xb ^ (((kb >> 1) & 1) << 3)) * 8);
  // column sums of B (bias gradients): one m-tile workgroup per (batch, n-tile) adds up what it loads
  const bool do_cs = epi.colsum != nullptr && (m0 / BM) == (n0 / BM + b) % NTm;
  float cs[8];
#pragma unroll
  for (int e = 0; e < 8; e++) cs[e] = 0.0f;

  // fragment role: 32-bit words (rows 2 l32, 2 l32 + 1 of the wave's strip) at k = 16 kk + 8 g + e
  const uint32_t* fa = reinterpret_cast<const uint32_t*>(lds_a) + (((wm * 64 + 2 * l32) ^ (g * 64)) >> 1) + g * 8 * 64;
  const uint32_t* fb = reinterpret_cast<const uint32_t*>(lds_b) + (((wn * 64 + 2 * l32) ^ (g * 64)) >> 1) + g * 8 * 64;

  bf16x8 ra[4], rb[4];
  const int nt = (kend - kbeg + BK - 1) / BK;          // k-tiles of this workgroup
  const int nit = (nt + KG - 1) / KG;                  // lock-step iterations (group kg takes tile it*KG + kg)
  if (nit > 0) {
    const int k0 = kbeg + kg * BK + kb * 4;
    dwx_load(ra, pa, A, xa, k0, kend);
    dwx_load(rb, pb, B, xbb, k0, kend);
  }
  for (int it = 0; it < nit; it++) {
    __syncthreads();  // previous tile fully consumed
#pragma unroll
    for (int j = 0; j < 4; j++) {
      *reinterpret_cast<bf16x8*>(lds_a + st_off + j * 128) = ra[j];
      *reinterpret_cast<bf16x8*>(lds_b + st_off + j * 128) = rb[j];
    }
    if (do_cs) {
#pragma unroll
      for (int j = 0; j < 4; j++)
#pragma unroll
        for (int e = 0; e < 8; e++) cs[e] += (float)rb[j][e];
    }
    __syncthreads();
    if (it + 1 < nit) {
      const int k0 = kbeg + ((it + 1) * KG + kg) * BK + kb * 4;
      dwx_load(ra, pa, A, xa, k0, kend);
      dwx_load(rb, pb, B, xbb, k0, kend);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; kk++) {
      uint32_t wa[8], wb[8];
#pragma unroll
      for (int e = 0; e < 8; e++) {
        wa[e] = fa[(kk * 16 + e) * 64];
        wb[e] = fb[(kk * 16 + e) * 64];
      }
      union { uint32_t u[4]; bf16x8 v; } a0, a1, b0, b1;
#pragma unroll
      for (int j = 0; j < 4; j++) {
        // byte permute of {first operand, second operand}: selectors 0..3 take bytes of the second, 4..7 of the
        // first: low halves (rows 2l) -> 0x05040100, high halves (rows 2l + 1) -> 0x07060302
        a0.u[j] = __builtin_amdgcn_perm(wa[2 * j + 1], wa[2 * j], 0x05040100u);
        a1.u[j] = __builtin_amdgcn_perm(wa[2 * j + 1], wa[2 * j], 0x07060302u);
        b0.u[j] = __builtin_amdgcn_perm(wb[2 * j + 1], wb[2 * j], 0x05040100u);
        b1.u[j] = __builtin_amdgcn_perm(wb[2 * j + 1], wb[2 * j], 0x07060302u);
      }
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b0.v, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b1.v, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b0.v, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b1.v, acc[1][1], 0, 0, 0);
    }
  }

  float* lds_f = reinterpret_cast<float*>(lds_all);
  if (epi.colsum != nullptr) {   // uniform over the workgroup
    __syncthreads();
    if (do_cs) {
#pragma unroll
      for (int e = 0; e < 8; e++) lds_f[(kg * 16 + kb) * 128 + xb * 8 + e] = cs[e];
    }
    __syncthreads();
    if (do_cs && threadIdx.x < 128 && n0 + (int)threadIdx.x < sh.N) {
      float s = 0.0f;
      for (int r = 0; r < 16 * KG; r++) s += lds_f[r * 128 + threadIdx.x];
      epi.colsum[(long long)b * sh.N + n0 + threadIdx.x] = s;
    }
  }
  // accumulator element (i, j, a) of lane (l32, g): row 2 acc_row(g, a) + i, column 2 l32 + j of the wave's 64 x 64
#pragma unroll 1
  for (int og = 1; og < KG; og++) {   // group og hands its 128 x 128 tile to group 0 (64 KB at the start of LDS)
    __syncthreads();
    if (kg == og) {
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int a = 0; a < 16; a++) {
          f32x2 v; v[0] = acc[i][0][a]; v[1] = acc[i][1][a];
          *reinterpret_cast<f32x2*>(lds_f + (wm * 64 + 2 * acc_row(g, a) + i) * 128 + wn * 64 + 2 * l32) = v;
        }
    }
    __syncthreads();
    if (kg == 0) {
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int a = 0; a < 16; a++) {
          f32x2 o = *reinterpret_cast<const f32x2*>(lds_f + (wm * 64 + 2 * acc_row(g, a) + i) * 128 + wn * 64 + 2 * l32);
          acc[i][0][a] += o[0]; acc[i][1][a] += o[1];
        }
    }
  }
  if (kg != 0) return;
  const int n = n0 + wn * 64 + 2 * l32;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int a = 0; a < 16; a++) {
      const int rloc = wm * 64 + 2 * acc_row(g, a) + i;
      const int m = m0 + rloc;
      f32x2 v; v[0] = acc[i][0][a]; v[1] = acc[i][1][a];
      if (m < sh.M && n < sh.N) dw_store_partial(epi.out + (long long)b * epi.mn + (long long)m * epi.ldn + n, v);
    }
}

// ---------------------------------------------------------------------------
// Pipelined parameter-gradient kernel: the arithmetic, LDS layout, fragment gather and accumulator mapping of
// gemm_dwx_kernel<1>, with S k-tiles in flight per workgroup instead of one.  Every thread keeps a ring of S
// register tiles (S x 8 loads of 16 bytes): in step t it stores ring slot t % S to the LDS buffer t % 2, re-issues
// the slot's loads for tile t + S, passes ONE barrier and multiplies from that buffer; the next store to the
// same buffer comes two steps later, behind the barrier in between, so it cannot overtake a reader.  All
// loads are unconditional (the host sends only shapes made of full tiles whose k-tiles do not straddle a group
// of the two-level k map), so nothing but the consuming LDS store waits for them.  A workgroup owns a CU's
// registers here anyway (256 workgroups on 256 CUs), and a k-step costs its memory latency, not its 16 MFMAs:
// more bytes in flight is what shortens it.
// ---------------------------------------------------------------------------
PE_DEV void dwp_load(bf16x8 (&regs)[4], const bf16* base, const Operand& op, long long xa, int k) {
  long long ka;
  if (op.k_in >= (1 << 30)) ka = (long long)k * op.k_stride;
  else ka = (long long)((unsigned)k / (unsigned)op.k_in) * op.k_outer + (long long)((unsigned)k % (unsigned)op.k_in) * op.k_stride;
  const bf16* p = base + xa + ka;
#pragma unroll
  for (int j = 0; j < 4; j++) regs[j] = *reinterpret_cast<const bf16x8*>(p + (long long)j * op.k_stride);
}

template <int S>
__global__ __launch_bounds__(256) void gemm_dwp_kernel(Operand A, Operand B, GemmShape sh, EpiPartial epi) {
  static_assert(S == 2 || S == 4, "ring depth: even (the LDS buffer of a ring slot must not change between rounds)");
  constexpr int BM = 128, BK = 64;
  constexpr int TILE = BK * 128;                       // elements of one operand tile (16 KB)
  extern __shared__ __attribute__((aligned(16))) bf16 lds_all[];   // 2 buffers x (A tile, B tile) = 64 KB
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;

  // same XCD-aware workgroup -> (batch, m-tile, n-tile) mapping as gemm_kernel
  const int NTm = sh.M / BM, NTn = sh.N / BM;
  const int xcd = blockIdx.x & 7, jq = blockIdx.x >> 3;
  const int NTu = sh.unit_n ? NTn : NTm, NTi = sh.unit_n ? NTm : NTn;
  const int unit = xcd + 8 * (jq / NTi);
  if (unit >= NTu * sh.batch) return;
  const int b = unit / NTu;
  const int tu = (unit % NTu) * BM, ti = (jq % NTi) * BM;
  const int m0 = sh.unit_n ? ti : tu, n0 = sh.unit_n ? tu : ti;
  const int kbeg = b * sh.k_chunk, kend = min(sh.K, kbeg + sh.k_chunk);
  const bf16* pa = (const bf16*)A.ptr;
  const bf16* pb = (const bf16*)B.ptr;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.0f;

  // loader role: 8 x (chunk xb) at k rows 4 kb .. 4 kb + 3 of the tile
  const int xb = tid & 15, kb = tid >> 4;
  XAddr xa, xbb;
  xa.init(A, m0, sh.M, xb);
  xbb.init(B, n0, sh.N, xb);
  const int st_off = kb * 4 * 128 + ((xb ^ (((kb >> 1) & 1) << 3)) * 8);
  const bool do_cs = epi.colsum != nullptr && (m0 / BM) == (n0 / BM + b) % NTm;
  float cs[8];
#pragma unroll
  for (int e = 0; e < 8; e++) cs[e] = 0.0f;
  // fragment role (word offsets inside an operand tile): rows 2 l32, 2 l32 + 1 of the wave's strip at k = 16 kk + 8 g + e
  const int fa_off = (((wm * 64 + 2 * l32) ^ (g * 64)) >> 1) + g * 8 * 64;
  const int fb_off = (((wn * 64 + 2 * l32) ^ (g * 64)) >> 1) + g * 8 * 64;

  bf16x8 ra[S][4], rb[S][4];
  const int nt = (kend - kbeg) / BK;                   // a multiple of S
#pragma unroll
  for (int j = 0; j < S; j++) {
    dwp_load(ra[j], pa, A, xa.a, kbeg + j * BK + kb * 4);
    dwp_load(rb[j], pb, B, xbb.a, kbeg + j * BK + kb * 4);
  }
  auto step = [&](auto jc, int t, bool reload) {
    constexpr int j = decltype(jc)::value;
    bf16* la = lds_all + (j & 1) * 2 * TILE;
    bf16* lb = la + TILE;
#pragma unroll
    for (int q = 0; q < 4; q++) {
      *reinterpret_cast<bf16x8*>(la + st_off + q * 128) = ra[j][q];
      *reinterpret_cast<bf16x8*>(lb + st_off + q * 128) = rb[j][q];
    }
    if (do_cs) {
#pragma unroll
      for (int q = 0; q < 4; q++)
#pragma unroll
        for (int e = 0; e < 8; e++) cs[e] += (float)rb[j][q][e];
    }
    if (reload) {   // uniform over the workgroup
      dwp_load(ra[j], pa, A, xa.a, kbeg + (t + S) * BK + kb * 4);
      dwp_load(rb[j], pb, B, xbb.a, kbeg + (t + S) * BK + kb * 4);
    }
    __syncthreads();
    const uint32_t* fa = reinterpret_cast<const uint32_t*>(la) + fa_off;
    const uint32_t* fb = reinterpret_cast<const uint32_t*>(lb) + fb_off;
#pragma unroll
    for (int kk = 0; kk < BK / 16; kk++) {
      uint32_t wa[8], wb[8];
#pragma unroll
      for (int e = 0; e < 8; e++) {
        wa[e] = fa[(kk * 16 + e) * 64];
        wb[e] = fb[(kk * 16 + e) * 64];
      }
      union { uint32_t u[4]; bf16x8 v; } a0, a1, b0, b1;
#pragma unroll
      for (int q = 0; q < 4; q++) {
        a0.u[q] = __builtin_amdgcn_perm(wa[2 * q + 1], wa[2 * q], 0x05040100u);
        a1.u[q] = __builtin_amdgcn_perm(wa[2 * q + 1], wa[2 * q], 0x07060302u);
        b0.u[q] = __builtin_amdgcn_perm(wb[2 * q + 1], wb[2 * q], 0x05040100u);
        b1.u[q] = __builtin_amdgcn_perm(wb[2 * q + 1], wb[2 * q], 0x07060302u);
      }
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b0.v, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0.v, b1.v, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b0.v, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1.v, b1.v, acc[1][1], 0, 0, 0);
    }
  };
  int t = 0;
  for (; t + S < nt; t += S) {     // rounds whose reloads stay inside the k range
    step(std::integral_constant<int, 0>{}, t, true);
    step(std::integral_constant<int, 1>{}, t + 1, true);
    if constexpr (S == 4) {
      step(std::integral_constant<int, 2>{}, t + 2, true);
      step(std::integral_constant<int, 3>{}, t + 3, true);
    }
  }
  // last round: nothing left to load
  step(std::integral_constant<int, 0>{}, t, false);
  step(std::integral_constant<int, 1>{}, t + 1, false);
  if constexpr (S == 4) {
    step(std::integral_constant<int, 2>{}, t + 2, false);
    step(std::integral_constant<int, 3>{}, t + 3, false);
  }

  if (epi.colsum != nullptr) {   // uniform over the workgroup
    float* lds_f = reinterpret_cast<float*>(lds_all);
    __syncthreads();
    if (do_cs) {
#pragma unroll
      for (int e = 0; e < 8; e++) lds_f[kb * 128 + xb * 8 + e] = cs[e];
    }
    __syncthreads();
    if (do_cs && tid < 128) {
      float s = 0.0f;
      for (int r = 0; r < 16; r++) s += lds_f[r * 128 + tid];
      epi.colsum[(long long)b * sh.N + n0 + tid] = s;
    }
  }
  // accumulator element (i, j, a) of lane (l32, g): row 2 acc_row(g, a) + i, column 2 l32 + j of the wave's 64 x 64
  const int n = n0 + wn * 64 + 2 * l32;
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int a = 0; a < 16; a++) {
      const int m = m0 + wm * 64 + 2 * acc_row(g, a) + i;
      f32x2 v; v[0] = acc[i][0][a]; v[1] = acc[i][1][a];
      dw_store_partial(epi.out + (long long)b * epi.mn + (long long)m * epi.ldn + n, v);
    }
}

// ring depth of the pipelined kernel for a shape (0: the shape is not made of full tiles, take another kernel).
// What bounds these kernels is the rate at which a CU takes in tile bytes (about 25 GB/s per CU, L2 hits
// included: 256 x 1024 x 32768 loads 256 MiB of tiles for 80 MiB of operands and takes 40 us, 128 MiB take 23 us,
// 64 MiB 14 us, whatever the prefetch depth or the number of wave groups), so more depth buys nothing.
static inline int dwp_depth(const Operand& A, const Operand& B, const GemmShape& sh) {
  if (sh.k_chunk <= 0 || sh.M % 128 || sh.N % 128 || sh.K % 64 || sh.k_chunk % 64) return 0;
  auto kmap_ok = [](const Operand& o) { return o.k_in >= (1 << 30) || o.k_in % 64 == 0; };
  if (!kmap_ok(A) || !kmap_ok(B)) return 0;
  const int last = sh.K - (sh.batch - 1) * sh.k_chunk;       // length of the last split
  if (last <= 0 || last > sh.k_chunk) return 0;
  if (sh.k_chunk % 128 == 0 && last % 128 == 0) return 2;   // a ring of 4 measured no faster (same 40 us at 256 x 1024 x 32768)
  return 0;
}

// Two wave groups: measured 15 - 27 % faster than one on the block's parameter-gradient shapes when the
// kernel has the chip to itself; three are no faster (and need more than 64 KB of LDS), four spill at
// 128 registers.  Next to another branch's kernels on a second stream the extra resident waves cost
// more than they win (the step is 1.3 % slower), so the caller asks for two groups only when nothing
// else runs beside the call and for one group otherwise (0.4 % faster there than the register-transposing
// kernel: no bank conflicts, fewer instructions).
constexpr int DWX_GROUPS = 2;
static inline int launch_dwx(hipStream_t st, dim3 grid, int groups, const Operand& A, const Operand& B, const GemmShape& sh, const EpiPartial& epi,
                             int* depth_used = nullptr) {
  constexpr unsigned bytes = DWX_GROUPS * 32768u;
  // A call that has the chip to itself takes the pipelined kernel where the shape allows it (one wave group, two
  // k-tiles in flight: as fast there as two wave groups, 1.3 % on the one-stream step, and it sums the k-tiles in
  // the order of gemm_dwx_kernel<1>, so its results are bit-identical to a two-stream call's).  Beside another
  // branch's kernels it does not pay (two-stream step 2.685 -> 2.695 ms): the one-group kernel stays there.
  const int depth = groups == 2 ? dwp_depth(A, B, sh) : 0;
  if (depth_used) *depth_used = depth;
  if (depth == 2) { hipLaunchKernelGGL((gemm_dwp_kernel<2>), grid, dim3(256), 65536u, st, A, B, sh, epi); return hipGetLastError() == hipSuccess ? 0 : -2; }
  static_assert(bytes <= 65536u, "more dynamic LDS than the default limit: raise hipFuncAttributeMaxDynamicSharedMemorySize first");
  if (groups == 1) hipLaunchKernelGGL((gemm_dwx_kernel<1>), grid, dim3(256), 32768u, st, A, B, sh, epi);
  else hipLaunchKernelGGL((gemm_dwx_kernel<DWX_GROUPS>), grid, dim3(256 * DWX_GROUPS), bytes, st, A, B, sh, epi);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

// the narrow-output kernel for the feature sets that occur with N <= 128 (else: not taken)
template <typename T, class Epi>
static inline bool launch_gemm64(hipStream_t st, const Operand& A, const Operand& B, const GemmShape& sh, const Epi& epi) {
  if constexpr (Epi::HAS_COLSUM || Epi::TM_GATE) {
    return false;   // split-K partials, gated projection: not for this kernel (and no instantiations for those epilogues)
  } else {
  const int f = epi.features();
  dim3 grid((unsigned)((sh.M + 63) / 64)), block(256);
  if constexpr (!std::is_same<Epi, EpiGeneric<T>>::value) {   // no feature sets: one instantiation
    hipLaunchKernelGGL((gemm64_kernel<T, Epi, 0>), grid, block, 0, st, A, B, sh, epi);
    g_gemm_last_features = 0;
    return true;
  } else {
#define PE_GEMM64_SPEC(S)                                                                         \
  if ((f & ~(S)) == 0) {                                                                          \
    hipLaunchKernelGGL((gemm64_kernel<T, Epi, (S)>), grid, block, 0, st, A, B, sh, epi);           \
    g_gemm_last_features = (S);                                                                   \
    return true;                                                                                  \
  }
  PE_GEMM64_SPEC(0)
  PE_GEMM64_SPEC(EF_BIASN | EF_RES)
  PE_GEMM64_SPEC(EF_BIASN | EF_ACT)
  PE_GEMM64_SPEC(EF_ACC | EF_BIASM)
  PE_GEMM64_SPEC(EF_OM2 | EF_ON2 | EF_BIASN)
  PE_GEMM64_SPEC(EF_BIASN | EF_AUX | EF_MUL | EF_RES)
  PE_GEMM64_SPEC(EF_BIASN | EF_ROWSCALE)
#undef PE_GEMM64_SPEC
  return false;
  }
  }
}

// Feature sets with a kernel of their own (k-contiguous operands, vector epilogue): a launch takes
// the first one that covers what its epilogue uses, else the general kernel.
template <typename T, class Epi>
static inline bool launch_gemm_spec(hipStream_t st, dim3 grid, const Operand& A, const Operand& B, const GemmShape& sh,
                                    const Epi& epi) {
  if constexpr (Epi::HAS_COLSUM) {
    return false;   // split-K partials: one kernel
  } else if constexpr (!std::is_same<Epi, EpiGeneric<T>>::value) {
    // the special-purpose epilogues have no feature sets: one instantiation
    hipLaunchKernelGGL((gemm_kernel<T, true, true, true, true, Epi, 0>), grid, dim3(256), 0, st, A, B, sh, epi);
    g_gemm_last_features = 0;
    return true;
  } else {
  const int f = epi.features();
  dim3 block(256);
#define PE_GEMM_SPEC(S)                                                                                     \
  if ((f & ~(S)) == 0) {                                                                                    \
    hipLaunchKernelGGL((gemm_kernel<T, true, true, true, true, Epi, (S)>), grid, block, 0, st, A, B, sh, epi); \
    g_gemm_last_features = (S);                                                                             \
    return true;                                                                                            \
  }
  PE_GEMM_SPEC(0)
  PE_GEMM_SPEC(EF_BIASN)
  PE_GEMM_SPEC(EF_BIASN | EF_RES)
  PE_GEMM_SPEC(EF_BIASN | EF_ACT)
  PE_GEMM_SPEC(EF_RELUMASK)
  PE_GEMM_SPEC(EF_OM2 | EF_ON2 | EF_BIASN)
  PE_GEMM_SPEC(EF_ACC | EF_BIASM)
  PE_GEMM_SPEC(EF_BIASN | EF_ROWSCALE)
  PE_GEMM_SPEC(EF_BIASN | EF_AUX | EF_MUL | EF_RES)
  PE_GEMM_SPEC(EF_OM2 | EF_ON2 | EF_ROWSCALE)
#undef PE_GEMM_SPEC
  return false;
  }
}

template <typename T, bool AL, bool VE, class Epi>
static inline void launch_gemm_al(hipStream_t st, dim3 grid, const Operand& A, bool a_kc, const Operand& B, bool b_kc,
                                  const GemmShape& sh, const Epi& epi) {
  dim3 block(256);
  if (AL && VE && a_kc && b_kc && launch_gemm_spec<T, Epi>(st, grid, A, B, sh, epi)) return;
  if constexpr (AL && VE && std::is_same<Epi, EpiGeneric<T>>::value) {
    // the other operand layouts occur with two feature sets only (the triangle contractions: none; the
    // outer product: the 2-D scale): lean kernels for those
    const int f = epi.features();
#define PE_GEMM_SPEC_L(S)                                                                                              \
    if ((f & ~(S)) == 0) {                                                                                             \
      if (a_kc && !b_kc) hipLaunchKernelGGL((gemm_kernel<T, true, false, true, true, Epi, (S)>), grid, block, 0, st, A, B, sh, epi);       \
      else if (!a_kc && b_kc) hipLaunchKernelGGL((gemm_kernel<T, false, true, true, true, Epi, (S)>), grid, block, 0, st, A, B, sh, epi);  \
      else hipLaunchKernelGGL((gemm_kernel<T, false, false, true, true, Epi, (S)>), grid, block, 0, st, A, B, sh, epi);                    \
      g_gemm_last_features = (S);                                                                                      \
      return;                                                                                                          \
    }
    if (!(a_kc && b_kc)) {
      PE_GEMM_SPEC_L(0)
      PE_GEMM_SPEC_L(EF_SCALE2D)
    }
#undef PE_GEMM_SPEC_L
  }
  if (a_kc && b_kc) hipLaunchKernelGGL((gemm_kernel<T, true, true, AL, VE, Epi>), grid, block, 0, st, A, B, sh, epi);
  else if (a_kc && !b_kc) hipLaunchKernelGGL((gemm_kernel<T, true, false, AL, VE, Epi>), grid, block, 0, st, A, B, sh, epi);
  else if (!a_kc && b_kc) hipLaunchKernelGGL((gemm_kernel<T, false, true, AL, VE, Epi>), grid, block, 0, st, A, B, sh, epi);
  else hipLaunchKernelGGL((gemm_kernel<T, false, false, AL, VE, Epi>), grid, block, 0, st, A, B, sh, epi);
}

// Operands that break the 16-byte vector rules (odd leading dimensions) take the
// element-wise loader and the per-element epilogue: same tiles, same arithmetic, slower.
template <typename T, class Epi>
static inline int launch_gemm(hipStream_t st, const Operand& A, bool a_kc, const Operand& B, bool b_kc,
                              const GemmShape& shape, const Epi& epi, bool* used_vec = nullptr, bool* used_narrow = nullptr,
                              int wave_groups = 0, int* dwp_depth_used = nullptr) {
  GemmShape sh = shape;
  g_gemm_last_features = EF_ALL;
  if (sh.M <= 0 || sh.N <= 0 || sh.batch <= 0) return 0;
  if (a_kc ? A.k_stride != 1 : A.x_stride != 1) return -1;
  if (b_kc ? B.k_stride != 1 : B.x_stride != 1) return -1;
  if (sh.k_chunk > 0 && sh.k_chunk % GemmCfg<T>::BK) return -1;
  bool al = gemm_operand_ok<T>(A, a_kc, sh.M, sh) && gemm_operand_ok<T>(B, b_kc, sh.N, sh);
  bool ve = al && epi.vec_ok(sh.N);
  if (used_vec) *used_vec = ve;
  const int NTm_ = (sh.M + 127) / 128, NTn_ = (sh.N + 127) / 128;
  // units over m-tiles unless units over n-tiles leave fewer idle slots on the 8 XCDs
  const long long um = (long long)NTm_ * sh.batch, un = (long long)NTn_ * sh.batch;
  const long long gm_ = 8 * ((um + 7) / 8) * NTn_, gn_ = 8 * ((un + 7) / 8) * NTm_;
  sh.unit_n = gn_ < gm_ ? 1 : 0;
  dim3 grid((unsigned)(sh.unit_n ? gn_ : gm_));
  // narrow outputs of tall GEMMs: 64-row tiles (twice the workgroups)
  const bool narrow = ve && a_kc && b_kc && sh.batch == 1 && sh.k_chunk == 0 && sh.N <= 128 && sh.M >= 128 * 256;
  if (used_narrow) *used_narrow = false;
  if (narrow && launch_gemm64<T, Epi>(st, A, B, sh, epi)) {
    if (used_narrow) *used_narrow = true;
    return hipGetLastError() == hipSuccess ? 0 : -2;
  }
  if constexpr (std::is_same<Epi, EpiPartial>::value && std::is_same<T, bf16>::value) {
    // parameter gradients from two x-contiguous operands: the kernel that keeps the tiles in memory order,
    // with wave_groups (1 or 2) wave groups (*used_narrow reports that it was taken)
    if (wave_groups && ve && !a_kc && !b_kc) {
      if (used_narrow) *used_narrow = true;
      return launch_dwx(st, grid, wave_groups, A, B, sh, epi, dwp_depth_used);
    }
  }
  if (ve) launch_gemm_al<T, true, true, Epi>(st, grid, A, a_kc, B, b_kc, sh, epi);
  else if (al) launch_gemm_al<T, true, false, Epi>(st, grid, A, a_kc, B, b_kc, sh, epi);
  else launch_gemm_al<T, false, false, Epi>(st, grid, A, a_kc, B, b_kc, sh, epi);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
