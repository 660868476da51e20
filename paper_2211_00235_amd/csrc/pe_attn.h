// Gated multi-head attention with optional pair bias and key mask: forward and backward.
//
// Used four ways by the block: MSA row attention (bias from the pair representation),
// MSA column attention (no bias, strided sequence axis), triangle attention around the
// starting node and around the ending node (strided axes + transposed bias).
//
// Data layout: HEAD-MAJOR.  q, k, v and the gate pre-activation live in one tensor `qkvg` of
// 4*H planes [B*L][d]; element (which w, head h, batch b, position p, channel c) is at
//   qkvg + (w*H + h)*plane + (b*L + p)*d + c,      plane = B*L*d.
// o / og / dO / dog are H planes of the same shape.  A head's K, V, Q tile is therefore one
// contiguous run of memory (64 positions x 64 bytes at d = 32) whatever axis the attention runs
// along; the producing / consuming GEMMs reach this layout through their two-level index maps.
// (With channel-last [B*L][4*H*d] rows a head's 64-byte slice sits alone in its 128-byte line:
// measured HBM fetch of the forward kernel was 2.5x its algorithmic bytes.)
//
// Kernel design (gfx950): every wave owns 32 queries (or 32 keys in the dK/dV kernel) and
// computes TRANSPOSED score tiles S^T = K Q^T with v_mfma 32x32, so that a query is a
// lane (column) and its keys are spread over the lane's 16 accumulator elements and the
// partner lane (lane ^ 32).  Row max / row sum then need one cross-lane exchange, the
// per-query softmax state is one scalar per lane, and the probability tile can be fed
// straight back as an MFMA operand (the contraction index is permuted consistently on
// both operands; the other operand is read from a transposed LDS copy of V / K / Q / dO).
// Online softmax over key tiles of 64; K row-major and V transposed are staged in LDS.
#pragma once
#include "pe_common.h"
#include "pe_elem.h"

struct AttnArgs {
  const void* qkvg; long long plane;    // plane = B*L*d elements
  int B, L, H, d;
  // pair bias, multiplied by log2 e, storage type, in the two layouts that bias_tile_kernel writes (nullptr: no bias):
  const void* biasQ;                 // [H][key tile][chunk][g][query][CH]: read by the query-per-lane kernels
  const void* biasK;                 // [H][query tile][chunk][g][key][CH]: read by the key-per-lane kernel
  const float* mask; long long mask_bs, mask_ks;   // key mask value at mask[b*mask_bs + j*mask_ks]
  void* o; void* og;                 // forward outputs (o ungated, og = sigmoid(g) * o)
  float* lse;                        // [B][H][L]
  float scale;                       // 1/sqrt(d)
  // backward
  const void* dog;                   // cotangent of og
  void* dO;                          // scratch: cotangent of o (written by pre kernel)
  float* D;                          // [B][H][L] rowsum(dO * o)
  void* dqkvg;                       // same layout as qkvg
  void* dS;                          // [ceil(B/2)][H] planes in the layout of biasQ (storage type), biased attention only
};

// XCD-aware decode of the 1-D grid of the three tile kernels: workgroup w runs on XCD w % 8, and all
// 128-position tiles of one (batch, head) unit go to the same XCD, so that its L2 serves the K / V
// (Q / dO in the dK/dV kernel) reads of the unit's second and later tiles; heads cycle fastest over the
// units, so an XCD also sees only H / 8 (or one) of the bias planes.
struct AttnWg { int tile, h, b; bool ok; };
PE_DEV AttnWg attn_decode_wg(const AttnArgs& a) {
  const int nt = (a.L + 127) / 128;
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int u = (j / nt) * 8 + xcd;
  AttnWg r;
  r.tile = j % nt;
  r.ok = u < a.B * a.H;
  r.h = u % a.H;
  r.b = u / a.H;
  return r;
}
static inline unsigned attn_grid_size(long long B, int H, long long L) {
  const long long nt = (L + 127) / 128, units = B * H;
  return (unsigned)(8 * ((units + 7) / 8) * nt);
}

template <typename T> struct AttnCfg {
  static constexpr int VEC = Vec16<T>::N;
  static constexpr int KT = 64;                                   // positions staged per iteration
  static constexpr int RM = (sizeof(T) == 2) ? 40 : 36;           // row-major LDS row stride (elements), d padded <= 32
  static constexpr int TS = KT + 4;                               // transposed LDS row stride
};

PE_DEV int round_up_i(int a, int b) { return (a + b - 1) / b * b; }

// Stage `KT` rows (positions pos0..pos0+KT-1) of one [d]-vector per row into LDS, as a
// row-major copy (stride RM, columns d..DP-1 zero filled) and/or a transposed copy
// (rows = channel, stride TS).  Rows beyond L are zero.
template <typename T>
PE_DEV void attn_stage(const T* src /* at (w, h, b, position 0, 0) */, int seq_stride, int pos0, int L, int d, int DP,
                       T* lds_rm, T* lds_t, int tid, int nthreads) {
  typedef AttnCfg<T> C;
  typedef typename Vec16<T>::type V;
  const int vpr = DP / C::VEC;
  for (int idx = tid; idx < C::KT * vpr; idx += nthreads) {
    int row = idx / vpr, dd0 = (idx % vpr) * C::VEC;
    V v;
#pragma unroll
    for (int e = 0; e < C::VEC; e++) v[e] = from_f<T>(0.0f);
    int pos = pos0 + row;
    if (pos < L && dd0 < d) v = *reinterpret_cast<const V*>(src + pos * seq_stride + dd0);
    if (lds_rm) *reinterpret_cast<V*>(lds_rm + row * C::RM + dd0) = v;
    if (lds_t) {
#pragma unroll
      for (int e = 0; e < C::VEC; e++) lds_t[(dd0 + e) * C::TS + row] = v[e];
    }
  }
}

// The same staging in two halves, so that the global loads of the next tile can be in flight while
// the current one is being used: `load` fills up to two 16-byte vectors per thread (zero beyond L / d),
// `store` writes them to the row-major and / or transposed LDS copies.
template <typename T> struct AttnStageRegs { typename Vec16<T>::type v[2]; };
template <typename T>
PE_DEV void attn_stage_load(const T* src, int seq_stride, int pos0, int L, int d, int DP, AttnStageRegs<T>& r, int tid) {
  typedef AttnCfg<T> C;
  typedef typename Vec16<T>::type V;
  const int vpr = DP / C::VEC;
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int idx = tid + i * 256;
    V v;
#pragma unroll
    for (int e = 0; e < C::VEC; e++) v[e] = from_f<T>(0.0f);
    const int row = idx / vpr, dd0 = (idx % vpr) * C::VEC;
    const int pos = pos0 + row;
    if (idx < C::KT * vpr && pos < L && dd0 < d) v = *reinterpret_cast<const V*>(src + pos * seq_stride + dd0);
    r.v[i] = v;
  }
}
template <typename T>
PE_DEV void attn_stage_store(const AttnStageRegs<T>& r, int DP, T* lds_rm, T* lds_t, int tid) {
  typedef AttnCfg<T> C;
  typedef typename Vec16<T>::type V;
  const int vpr = DP / C::VEC;
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const int idx = tid + i * 256;
    if (idx < C::KT * vpr) {
      const int row = idx / vpr, dd0 = (idx % vpr) * C::VEC;
      if (lds_rm) *reinterpret_cast<V*>(lds_rm + row * C::RM + dd0) = r.v[i];
      if (lds_t) {
#pragma unroll
        for (int e = 0; e < C::VEC; e++) lds_t[(dd0 + e) * C::TS + row] = r.v[i][e];
      }
    }
  }
}

// accumulator elements [u*KP, u*KP+KP) of a 32x32 tile as an MFMA operand fragment
template <typename T> PE_DEV typename Mma<T>::frag acc_to_frag(const f32x16& acc, int u);
template <> PE_DEV Mma<bf16>::frag acc_to_frag<bf16>(const f32x16& acc, int u) {
  bf16x8 f;
#pragma unroll
  for (int t = 0; t < 8; t++) f[t] = (bf16)acc[u * 8 + t];
  return f;
}
template <> PE_DEV Mma<float>::frag acc_to_frag<float>(const f32x16& acc, int u) { return acc[u]; }

// matching fragment of the other operand from a transposed LDS tile: row pointer `rowp`
// points at element [row = lane%32][tile_base]; contraction slots follow acc_row(g, a).
template <typename T> PE_DEV typename Mma<T>::frag lds_tfrag(const T* rowp, int g, int u);
template <> PE_DEV Mma<bf16>::frag lds_tfrag<bf16>(const bf16* rowp, int g, int u) {
  bf16x4 lo = *reinterpret_cast<const bf16x4*>(rowp + 16 * u + 4 * g);
  bf16x4 hi = *reinterpret_cast<const bf16x4*>(rowp + 16 * u + 8 + 4 * g);
  bf16x8 f;
  f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3];
  f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3];
  return f;
}
template <> PE_DEV Mma<float>::frag lds_tfrag<float>(const float* rowp, int g, int u) {
  return rowp[8 * (u >> 2) + 4 * g + (u & 3)];
}

// operand fragment straight from global memory: row `p` (nullptr = out of range), channels
// [kk*KSTEP + g*KP, +KP), zero beyond d
template <typename T> PE_DEV typename Mma<T>::frag gl_frag(const T* p, int kk, int g, int d) {
  typedef Mma<T> MM;
  int c0 = kk * MM::KSTEP + g * MM::KP;
  if (p == nullptr || c0 >= d) return MM::zero();
  return MM::load(p + c0);
}

// Softmax is evaluated in the base-2 domain: t = q' k + bias', p = 2^(t - m), where q' = q * log2 e / sqrt(d) comes out
// of the projection GEMM already scaled (its prepared weight copy carries the factor) and bias' = bias * log2 e is what
// bias_tile_kernel stores.  A logit costs the vector unit no multiply-add and no conversion:
//   * the bias tile is added by the matrix unit, as I x bias with an identity A operand (bf16; the 32-bit path adds it
//     with 16 vector adds), and is loaded in exactly the B-operand order, so it needs no conversion;
//   * the additive 0 / -inf key mask is applied only to 32-key tiles that hold a masked or padded key (one flag per
//     tile, decided when the tile is staged);
//   * in the dK / dV kernel, where -lse and -D of a tile's queries sit in LDS in accumulator order, they are the C
//     operands of the S and dP products.
// These kernels are bound by the length of a workgroup's life (memory round trips and dependent stages in a row at 3-4
// waves per SIMD), not by any one unit: measured on MI355X, halving the vector instructions per logit changed the
// forward kernel by 2 %, taking the exponentials out by 3 %, while its loads and stores add their full time to the
// arithmetic's.  What helps is fewer round trips in a row (K / V staged 256 keys at a time in the forward kernel) and
// registers kept at the 128 that four waves per SIMD allow.
#define PE_LOG2E 1.4426950408889634f
#define PE_LN2 0.6931471805599453f
// raw v_exp_f32 (2^x; results below the normal range flush to zero, which is what softmax wants)
PE_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T> PE_DEV f32x16 mma_c(typename Mma<T>::frag a, typename Mma<T>::frag b, const f32x16& c);
template <> PE_DEV f32x16 mma_c<bf16>(bf16x8 a, bf16x8 b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
template <> PE_DEV f32x16 mma_c<float>(float a, float b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
PE_DEV f32x16 splat16(float v) {
  f32x16 r;
#pragma unroll
  for (int e = 0; e < 16; e++) r[e] = v;
  return r;
}

// Bias values of one 32x32 tile for the lane that owns position `col` (clamped to L-1 by the caller) of the lane axis,
// from the chunk-ordered plane of its head (bias_tile_kernel).  bf16: chunk c of lane group g holds positions
// 16 c + 8 g + 0..7 of the other axis, i.e. the B operand of MFMA step c; fp32: accumulator order.  16-byte loads; a half
// wave's 32 lanes read 512 contiguous bytes per load.
template <typename T> struct BiasTile;
template <> struct BiasTile<bf16> { bf16x8 v[2]; };
template <> struct BiasTile<float> { float v[16]; };
PE_DEV void attn_load_bias(const bf16* plane, int L, int tile, int col, int g, BiasTile<bf16>& b) {
#pragma unroll
  for (int c = 0; c < 2; c++) b.v[c] = *reinterpret_cast<const bf16x8*>(plane + bias_chunk_off<bf16>(tile, c, g, col, L));
}
PE_DEV void attn_load_bias(const float* plane, int L, int tile, int col, int g, BiasTile<float>& b) {
#pragma unroll
  for (int c = 0; c < 4; c++) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(plane + bias_chunk_off<float>(tile, c, g, col, L));
#pragma unroll
    for (int r = 0; r < 4; r++) b.v[c * 4 + r] = v[r];
  }
}
// identity A operand: lane (row l32, group g) of step c holds [16 c + 8 g + t == l32], t = 0..7
template <typename T> struct IdFrag;
template <> struct IdFrag<bf16> {
  bf16x8 f[2];
  PE_DEV void init(int l32, int g) {
#pragma unroll
    for (int c = 0; c < 2; c++)
#pragma unroll
      for (int t = 0; t < 8; t++) f[c][t] = (bf16)((16 * c + 8 * g + t == l32) ? 1.0f : 0.0f);
  }
};
template <> struct IdFrag<float> { PE_DEV void init(int, int) {} };
PE_DEV void attn_add_bias(f32x16& acc, const BiasTile<bf16>& b, const IdFrag<bf16>& id) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(id.f[0], b.v[0], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(id.f[1], b.v[1], acc, 0, 0, 0);
}
PE_DEV void attn_add_bias(f32x16& acc, const BiasTile<float>& b, const IdFrag<float>&) {
#pragma unroll
  for (int e = 0; e < 16; e++) acc[e] += b.v[e];
}
// additive key mask of one tile in accumulator order (rows of the tile = keys)
PE_DEV void attn_add_row_mask(f32x16& acc, const float* lds_madd_tile, int g) {
#pragma unroll
  for (int q4 = 0; q4 < 4; q4++) {
    const f32x4 ma = *reinterpret_cast<const f32x4*>(lds_madd_tile + 8 * q4 + 4 * g);
#pragma unroll
    for (int r = 0; r < 4; r++) acc[q4 * 4 + r] += ma[r];
  }
}
// Key mask of the 64 staged keys: lds_madd = 0 / -inf per key, lds_flag[t] = 1 when tile t holds a masked or padded
// key.  Called by threads 0..63 (one wave) with their key's mask value (0 beyond L).
PE_DEV void attn_stage_mask(float mk, float* lds_madd, int* lds_flag, int t64) {
  const bool masked = !(mk > 0.0f);
  lds_madd[t64] = masked ? -INFINITY : 0.0f;
  const unsigned long long bal = __ballot(masked);
  if (t64 == 0) { lds_flag[0] = (bal & 0xffffffffull) != 0; lds_flag[1] = (bal >> 32) != 0; }
}
// a lane's 16 elements of a score tile (dS) stored in the same chunk order
template <typename T> PE_DEV void attn_store_tile16(T* plane, int L, int tile, int col, int g, const float (&v)[16]);
template <> PE_DEV void attn_store_tile16<float>(float* plane, int L, int tile, int col, int g, const float (&v)[16]) {
#pragma unroll
  for (int c = 0; c < 4; c++) {
    float t[4];
#pragma unroll
    for (int r = 0; r < 4; r++) t[r] = v[c * 4 + r];
    store4<float>(plane + bias_chunk_off<float>(tile, c, g, col, L), t);
  }
}
template <> PE_DEV void attn_store_tile16<bf16>(bf16* plane, int L, int tile, int col, int g, const float (&v)[16]) {
#pragma unroll
  for (int c = 0; c < 2; c++) {
    float t[8];
#pragma unroll
    for (int r = 0; r < 8; r++) t[r] = v[c * 8 + r];
    bf16x8 o;   // non-temporal: read once, by the reduction over the batch axis
#pragma unroll
    for (int r = 0; r < 8; r++) o[r] = (bf16)t[r];
    __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(plane + bias_chunk_off<bf16>(tile, c, g, col, L)));
  }
}
// number of 32-position tiles of an axis of length L
PE_DEV int attn_tiles32(int L) { return (L + 31) >> 5; }

// ---------------------------------------------------------------------------
// Forward
// grid attn_grid_size(B, H, L), 256 threads; wave w owns queries q0 = tile*128 + 32*w
// ---------------------------------------------------------------------------
// The running maximum is a REFERENCE m_ref that follows the true maximum only when it has to.  The first tile in which a
// query meets a finite logit sets m_ref to that tile's maximum (so a query with a single valid key gets the
// probability 1 and its value row back exactly); after that the probabilities 2^(t - m_ref) <= 2^TAU are used as they
// are, and only when a lane's tile maximum is more than TAU above m_ref the wave re-bases (accumulators and sum times
// 2^(old - new)).  The result o = acc / l and lse = (m_ref + log2 l) ln 2 do not depend on the reference.
#define ATTN_TAU 8.0f
// Forward: K and V are staged a CHUNK of up to 256 keys at a time: all loads of the chunk are issued at once and waited
// for once (with 64-key tiles a workgroup paid one memory round trip per tile, four to six in a row), and the waves then
// run through its tiles without a barrier.  38 KB of LDS per workgroup, four workgroups per CU.
template <typename T> struct AttnChunk {
  static constexpr int CH = (sizeof(T) == 2) ? 256 : 128;          // keys per chunk
  static constexpr int TS = CH + 4;                                // transposed row stride
  static constexpr int NV = CH * (32 / Vec16<T>::N) / 256;         // 16-byte vectors per thread and tensor (4)
};
// all vectors of one [CH keys][d] chunk for this thread: vector idx = tid + 256 i <-> (row idx / vpr, channels
// (idx % vpr) VEC ..) with vpr = 32 / VEC vector slots per row whatever d is (slots beyond d stay zero)
template <typename T>
PE_DEV void attn_chunk_load(const T* src, int pos0, int L, int d, typename Vec16<T>::type (&r)[AttnChunk<T>::NV], int tid) {
  typedef typename Vec16<T>::type V;
  constexpr int VEC = Vec16<T>::N;
  constexpr int vpr = 32 / VEC;
#pragma unroll
  for (int i = 0; i < AttnChunk<T>::NV; i++) {
    const int idx = tid + i * 256;
    V v;
#pragma unroll
    for (int e = 0; e < VEC; e++) v[e] = from_f<T>(0.0f);
    const int row = idx / vpr, dd0 = (idx % vpr) * VEC;
    const int pos = pos0 + row;
    if (pos < L && dd0 < d) v = *reinterpret_cast<const V*>(src + (long long)pos * d + dd0);
    r[i] = v;
  }
}
template <typename T>
PE_DEV void attn_chunk_store(const typename Vec16<T>::type (&r)[AttnChunk<T>::NV], int DP, T* lds_rm, T* lds_t, int tid) {
  typedef typename Vec16<T>::type V;
  constexpr int VEC = Vec16<T>::N;
  constexpr int vpr = 32 / VEC;
#pragma unroll
  for (int i = 0; i < AttnChunk<T>::NV; i++) {
    const int idx = tid + i * 256;
    const int row = idx / vpr, dd0 = (idx % vpr) * VEC;
    if (dd0 < DP) {
      if (lds_rm) *reinterpret_cast<V*>(lds_rm + row * AttnCfg<T>::RM + dd0) = r[i];
      if (lds_t) {
#pragma unroll
        for (int e = 0; e < VEC; e++) lds_t[(dd0 + e) * AttnChunk<T>::TS + row] = r[i][e];
      }
    }
  }
}

#ifndef PE_FWD_WAVES
#define PE_FWD_WAVES 4
#endif
template <typename T, bool HAS_BIAS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PE_FWD_WAVES, PE_FWD_WAVES))) void attn_fwd_kernel(AttnArgs a) {
  typedef AttnCfg<T> C;
  typedef Mma<T> MM;
  typedef AttnChunk<T> K;
  typedef typename Vec16<T>::type V;
  __shared__ __attribute__((aligned(16))) T lds_k[K::CH * C::RM];
  __shared__ __attribute__((aligned(16))) T lds_vt[32 * K::TS];
  __shared__ __attribute__((aligned(16))) float lds_madd[K::CH];   // 0 for a valid key, -inf for a masked one
  __shared__ int lds_flag[K::CH / 32];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const AttnWg wg = attn_decode_wg(a);
  if (!wg.ok) return;
  const int h = wg.h, b = wg.b;
  const int L = a.L, d = a.d;
  const int DP = round_up_i(d, MM::KSTEP);
  const int NKK = DP / MM::KSTEP;
  const int qi = wg.tile * 128 + wave * 32 + l32;       // this lane's query
  const bool qok = qi < L;
  const long long HP = (long long)a.H * a.plane;            // distance between the q, k, v, gate groups
  const T* base = (const T*)a.qkvg + h * a.plane + (long long)b * L * d;
  const T* qrow = qok ? base + qi * d : nullptr;

  constexpr int MAXKK = 32 / MM::KSTEP;   // 2 (bf16) or 16 (fp32): d <= 32
  typename MM::frag qf[MAXKK];
  f32x16 oacc = splat16(0.0f);
  float m_ref = 0.0f, l_part = 0.0f;     // l_part: this lane's keys only; the two halves of a query are added at the end
  bool seen = false;                     // a finite logit has been seen
  constexpr bool has_bias = HAS_BIAS;
  const T* bplane = has_bias ? (const T*)a.biasQ + (long long)h * attn_tiles32(L) * L * 32 : nullptr;
  const int bcolq = min(qi, L - 1);
  IdFrag<T> idf;
  idf.init(l32, g);

  for (int c0 = 0; c0 < L; c0 += K::CH) {
    {
      V rk[K::NV], rv[K::NV];
      if (c0 > 0) __syncthreads();
      attn_chunk_load<T>(base + HP, c0, L, d, rk, tid);
      attn_chunk_load<T>(base + 2 * HP, c0, L, d, rv, tid);
      const int j = c0 + tid;
      const float mk = (tid < K::CH && j < L) ? a.mask[(long long)b * a.mask_bs + (long long)j * a.mask_ks] : 0.0f;
      if (c0 == 0) {
#pragma unroll
        for (int kk = 0; kk < MAXKK; kk++)
          if (kk < NKK) qf[kk] = gl_frag<T>(qrow, kk, g, d);
      }
      attn_chunk_store<T>(rk, DP, lds_k, (T*)nullptr, tid);
      attn_chunk_store<T>(rv, DP, (T*)nullptr, lds_vt, tid);
      if (tid < K::CH) attn_stage_mask(mk, lds_madd + 64 * wave, lds_flag + 2 * wave, lane);
      __syncthreads();
    }
    const int jend = min(K::CH, L - c0);
    BiasTile<T> bt;
    if (has_bias) attn_load_bias(bplane, L, c0 >> 5, bcolq, g, bt);
    for (int js = 0; js < jend; js += 32) {
      const int masked = __builtin_amdgcn_readfirstlane(lds_flag[js >> 5]);
      // base-2 logits for (query = lane, keys = acc rows)
      f32x16 sacc = splat16(0.0f);
#pragma unroll
      for (int kk = 0; kk < MAXKK; kk++)
        if (kk < NKK) MM::mma(sacc, MM::load(lds_k + (js + l32) * C::RM + kk * MM::KSTEP + g * MM::KP), qf[kk]);
      if (has_bias) {
        attn_add_bias(sacc, bt, idf);
        attn_load_bias(bplane, L, min(((c0 + js) >> 5) + 1, attn_tiles32(L) - 1), bcolq, g, bt);   // next tile's bias
      }
      if (masked) attn_add_row_mask(sacc, lds_madd + js, g);
      float tmax = sacc[0];
#pragma unroll
      for (int e = 1; e < 16; e++) tmax = fmaxf(tmax, sacc[e]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      // re-base when the tile's maximum is more than TAU above the reference, and at the first finite logit
      const bool finite = tmax > -INFINITY;
      const bool rebase = tmax > m_ref + ATTN_TAU || (!seen && finite);
      seen = seen || finite;
      if (__any(rebase)) {
        const float m_new = rebase ? tmax : m_ref;
        const float corr = fast_exp2(m_ref - m_new);
        m_ref = m_new;
        l_part *= corr;
#pragma unroll
        for (int e = 0; e < 16; e++) oacc[e] *= corr;
      }
      float psum = 0.0f;
#pragma unroll
      for (int e = 0; e < 16; e++) {
        float p = fast_exp2(sacc[e] - m_ref);
        sacc[e] = p;
        psum += p;
      }
      l_part += psum;
      // O^T[dd, i] += sum_j V^T[dd, j] P^T[j, i]
      const T* vrow = lds_vt + l32 * K::TS + js;
#pragma unroll
      for (int u = 0; u < 32 / MM::KSTEP; u++) MM::mma(oacc, lds_tfrag<T>(vrow, g, u), acc_to_frag<T>(sacc, u));
    }
  }
  const float l_run = l_part + __shfl_xor(l_part, 32, 64);
  if (!qok) return;
  float inv = (l_run > 0.0f) ? 1.0f / l_run : 0.0f;
  if (g == 0) a.lse[((long long)b * a.H + h) * L + qi] = (l_run > 0.0f) ? (m_ref + log2f(l_run)) * PE_LN2 : 0.0f;
  const long long orow = h * a.plane + ((long long)b * L + qi) * d;
  T* po = (T*)a.o + orow;
  T* pog = (T*)a.og + orow;
  const T* pg = qrow + 3 * HP;
#pragma unroll
  for (int q4 = 0; q4 < 4; q4++) {
    int dd = 8 * q4 + 4 * g;
    if (dd < d) {
      float gv[4], ov[4], ogv[4];
      load4<T>(pg + dd, gv);
#pragma unroll
      for (int r = 0; r < 4; r++) {
        ov[r] = oacc[q4 * 4 + r] * inv;
        ogv[r] = ov[r] * sigmoidf_(gv[r]);
      }
      store4<T>(po + dd, ov);
      store4<T>(pog + dd, ogv);
    }
  }
}

// ---------------------------------------------------------------------------
// Backward, step 0: dO = dog * sigmoid(g); dg = dog * o * s(1-s) -> dqkvg gate slot;
// D = sum_c dO * o.  One thread per (b, p, h).
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_pre_kernel(AttnArgs a) {
  // 8 lanes per (h, b, p): lane `sub` owns channels [4*sub, 4*sub+4); consecutive groups walk
  // consecutive positions of one head plane (contiguous memory)
  long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int sub = gid & 7;
  long long idx = gid >> 3;
  const long long M = (long long)a.B * a.L;
  long long total = M * a.H;
  const bool ok = idx < total;
  if (!ok) idx = total - 1;
  const int h = idx / M;
  const long long plin = idx % M;
  const int b = plin / a.L, p = plin % a.L;
  const int d = a.d;
  long long qoff = (3LL * a.H + h) * a.plane + plin * d;
  long long ooff = h * a.plane + plin * d;
  float Dsum = 0.0f;
  const int c0 = sub * 4;
  if (ok && c0 < d) {
    float gv[4], ov[4], dv[4], dov[4], dgv[4];
    load4<T>((const T*)a.qkvg + qoff + c0, gv);
    load4<T>((const T*)a.o + ooff + c0, ov);
    load4<T>((const T*)a.dog + ooff + c0, dv);
#pragma unroll
    for (int e = 0; e < 4; e++) {
      float sg = sigmoidf_(gv[e]);
      dov[e] = to_f(from_f<T>(dv[e] * sg));
      dgv[e] = dv[e] * ov[e] * sg * (1.0f - sg);
      Dsum += dov[e] * ov[e];
    }
    store4<T>((T*)a.dO + ooff + c0, dov);
    store4<T>((T*)a.dqkvg + qoff + c0, dgv);
  }
  Dsum += __shfl_xor(Dsum, 4, 64);
  Dsum += __shfl_xor(Dsum, 2, 64);
  Dsum += __shfl_xor(Dsum, 1, 64);
  if (ok && sub == 0) a.D[((long long)b * a.H + h) * a.L + p] = Dsum;
}

// ---------------------------------------------------------------------------
// Backward, dQ (+ dS for the bias gradient).  Same tiling as the forward kernel.
// ---------------------------------------------------------------------------
// Capped at 128 registers (4 waves per SIMD instead of 3 at the 138 the compiler would take; three
// dwords spill): measured 85 -> 77 us per biased attention at L = 256.
template <typename T, bool HAS_BIAS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void attn_bwd_dq_kernel(AttnArgs a) {
  typedef AttnCfg<T> C;
  typedef Mma<T> MM;
  __shared__ __attribute__((aligned(16))) T lds_k[C::KT * C::RM];
  __shared__ __attribute__((aligned(16))) T lds_kt[32 * C::TS];
  __shared__ __attribute__((aligned(16))) T lds_v[C::KT * C::RM];
  __shared__ __attribute__((aligned(16))) float lds_madd[C::KT];
  __shared__ int lds_flag[2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const AttnWg wg = attn_decode_wg(a);
  if (!wg.ok) return;
  const int h = wg.h, b = wg.b;
  const int L = a.L, d = a.d;
  const int DP = round_up_i(d, MM::KSTEP);
  const int NKK = DP / MM::KSTEP;
  const int qi = wg.tile * 128 + wave * 32 + l32;
  const bool qok = qi < L;
  const long long HP = (long long)a.H * a.plane;
  const T* base = (const T*)a.qkvg + h * a.plane + (long long)b * L * d;
  const T* qrow = qok ? base + qi * d : nullptr;
  const long long orow = h * a.plane + ((long long)b * L + qi) * d;
  const T* dorow = qok ? (const T*)a.dO + orow : nullptr;

  constexpr int MAXKK = 32 / MM::KSTEP;
  typename MM::frag qf[MAXKK], dof[MAXKK];
#pragma unroll
  for (int kk = 0; kk < MAXKK; kk++)
    if (kk < NKK) {
      qf[kk] = gl_frag<T>(qrow, kk, g, d);
      dof[kk] = gl_frag<T>(dorow, kk, g, d);
    }
  const long long sidx = ((long long)b * a.H + h) * L + qi;
  const float lse2 = qok ? a.lse[sidx] * PE_LOG2E : 0.0f;
  const float Di = qok ? a.D[sidx] : 0.0f;
  constexpr bool has_bias = HAS_BIAS;
  const T* bplane = has_bias ? (const T*)a.biasQ + (long long)h * attn_tiles32(L) * L * 32 : nullptr;
  const int bcolq = min(qi, L - 1);
  // dS plane of this (b, h) in the layout of biasQ
  T* dsplane = a.dS ? (T*)a.dS + ((long long)b * a.H + h) * attn_tiles32(L) * L * 32 : nullptr;
  IdFrag<T> idf;
  idf.init(l32, g);

  f32x16 dq;
#pragma unroll
  for (int e = 0; e < 16; e++) dq[e] = 0.0f;

  for (int j0 = 0; j0 < L; j0 += C::KT) {
    __syncthreads();
    attn_stage<T>(base + HP, d, j0, L, d, DP, lds_k, lds_kt, tid, 256);
    attn_stage<T>(base + 2 * HP, d, j0, L, d, DP, lds_v, (T*)nullptr, tid, 256);
    if (tid < C::KT) {
      const int j = j0 + tid;
      attn_stage_mask((j < L) ? a.mask[(long long)b * a.mask_bs + (long long)j * a.mask_ks] : 0.0f, lds_madd, lds_flag, tid);
    }
    __syncthreads();
#pragma unroll
    for (int jt = 0; jt < C::KT / 32; jt++) {
      const int kt0 = j0 + jt * 32;
      if (kt0 >= L) break;
      BiasTile<T> bt;
      if (has_bias) attn_load_bias(bplane, L, kt0 >> 5, bcolq, g, bt);
      const int masked = __builtin_amdgcn_readfirstlane(lds_flag[jt]);
      const int off0 = (jt * 32 + l32) * C::RM + g * MM::KP;
      f32x16 sacc = splat16(0.0f), pacc = splat16(0.0f);
#pragma unroll
      for (int kk = 0; kk < MAXKK; kk++)
        if (kk < NKK) {
          MM::mma(sacc, MM::load(lds_k + off0 + kk * MM::KSTEP), qf[kk]);      // S^T = K Q^T
          MM::mma(pacc, MM::load(lds_v + off0 + kk * MM::KSTEP), dof[kk]);     // dP^T = V dO^T
        }
      if (has_bias) attn_add_bias(sacc, bt, idf);
      if (masked) attn_add_row_mask(sacc, lds_madd + jt * 32, g);
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[e] = fast_exp2(sacc[e] - lse2) * (pacc[e] - Di);     // dS = P (dP - D)
      if (dsplane && qok) {
        float v16[16];
#pragma unroll
        for (int e = 0; e < 16; e++) v16[e] = sacc[e];
        attn_store_tile16<T>(dsplane, L, kt0 >> 5, qi, g, v16);
      }
      const T* krow = lds_kt + l32 * C::TS + jt * 32;
#pragma unroll
      for (int u = 0; u < 32 / MM::KSTEP; u++) MM::mma(dq, lds_tfrag<T>(krow, g, u), acc_to_frag<T>(sacc, u));
    }
  }
  if (!qok) return;
  T* pdq = (T*)a.dqkvg + orow;
#pragma unroll
  for (int q4 = 0; q4 < 4; q4++) {
    int dd = 8 * q4 + 4 * g;
    if (dd < d) {
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; r++) v[r] = dq[q4 * 4 + r] * a.scale;
      store4<T>(pdq + dd, v);
    }
  }
}

// ---------------------------------------------------------------------------
// Backward, dQ for TWO batch rows per workgroup (biased attention only).  Waves 0-3 work on batch row
// 2u, waves 4-7 on row 2u+1 of the same head and query tile, each group exactly as attn_bwd_dq_kernel
// with its own LDS tiles.  The bias gradient is a sum over the batch axis, so the two groups add their
// dS tiles before the write: the upper group passes each 32x32 tile through LDS (two buffers, one
// workgroup barrier per tile), the lower group adds its own and stores dS^T[u][h][key][query].  That
// halves the dS traffic and the input of the reduction that follows.  With an odd B the last
// workgroup's upper group runs on row B-1 again and contributes nothing.
// ---------------------------------------------------------------------------
#ifndef PE_DQ2_WAVES
#define PE_DQ2_WAVES 4
#endif
template <typename T>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(PE_DQ2_WAVES, PE_DQ2_WAVES))) void attn_bwd_dq2_kernel(AttnArgs a) {
  typedef AttnCfg<T> C;
  typedef Mma<T> MM;
  __shared__ __attribute__((aligned(16))) T lds_k2[2][C::KT * C::RM];
  __shared__ __attribute__((aligned(16))) T lds_kt2[2][32 * C::TS];
  __shared__ __attribute__((aligned(16))) T lds_v2[2][C::KT * C::RM];
  __shared__ __attribute__((aligned(16))) float lds_madd2[2][C::KT];
  __shared__ int lds_flag2[2][2];
  __shared__ __attribute__((aligned(16))) float lds_x[2][4][16][64];   // [buffer][wave of the upper group][element][lane]

  const int tid = threadIdx.x, lane = tid & 63, wave8 = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const int grp = wave8 >> 2, wave = wave8 & 3, tg = tid & 255;
  // XCD-aware decode as in attn_decode_wg, over (pair of batch rows, head) units
  const int nt = (a.L + 127) / 128, Bp = (a.B + 1) / 2;
  const int xcd = blockIdx.x & 7, jq = blockIdx.x >> 3;
  const int u = (jq / nt) * 8 + xcd;
  if (u >= Bp * a.H) return;
  const int tile = jq % nt, h = u % a.H, bp = u / a.H;
  const bool bvalid = 2 * bp + grp < a.B;
  const int b = bvalid ? 2 * bp + grp : a.B - 1;
  T* lds_k = lds_k2[grp];
  T* lds_kt = lds_kt2[grp];
  T* lds_v = lds_v2[grp];
  float* lds_madd = lds_madd2[grp];
  int* lds_flag = lds_flag2[grp];

  const int L = a.L, d = a.d;
  const int DP = round_up_i(d, MM::KSTEP);
  const int NKK = DP / MM::KSTEP;
  const int qi = tile * 128 + wave * 32 + l32;
  const bool qok = qi < L;
  const long long HP = (long long)a.H * a.plane;
  const T* base = (const T*)a.qkvg + h * a.plane + (long long)b * L * d;
  const T* qrow = qok ? base + qi * d : nullptr;
  const long long orow = h * a.plane + ((long long)b * L + qi) * d;
  const T* dorow = qok ? (const T*)a.dO + orow : nullptr;

  constexpr int MAXKK = 32 / MM::KSTEP;
  typename MM::frag qf[MAXKK], dof[MAXKK];
#pragma unroll
  for (int kk = 0; kk < MAXKK; kk++)
    if (kk < NKK) {
      qf[kk] = gl_frag<T>(qrow, kk, g, d);
      dof[kk] = gl_frag<T>(dorow, kk, g, d);
    }
  const long long sidx = ((long long)b * a.H + h) * L + qi;
  const float lse2 = qok ? a.lse[sidx] * PE_LOG2E : 0.0f;
  const float Di = qok ? a.D[sidx] : 0.0f;
  const T* bplane = (const T*)a.biasQ + (long long)h * attn_tiles32(L) * L * 32;
  const int bcolq = min(qi, L - 1);
  T* dsplane = (T*)a.dS + ((long long)bp * a.H + h) * attn_tiles32(L) * L * 32;   // summed pair of rows, accumulator order
  IdFrag<T> idf;
  idf.init(l32, g);

  f32x16 dq;
#pragma unroll
  for (int e = 0; e < 16; e++) dq[e] = 0.0f;

  int xb = 0;   // exchange buffer of the current tile
  for (int j0 = 0; j0 < L; j0 += C::KT) {
    __syncthreads();
    attn_stage<T>(base + HP, d, j0, L, d, DP, lds_k, lds_kt, tg, 256);
    attn_stage<T>(base + 2 * HP, d, j0, L, d, DP, lds_v, (T*)nullptr, tg, 256);
    if (tg < C::KT) {
      const int j = j0 + tg;
      attn_stage_mask((j < L) ? a.mask[(long long)b * a.mask_bs + (long long)j * a.mask_ks] : 0.0f, lds_madd, lds_flag, tg);
    }
    __syncthreads();
#pragma unroll
    for (int jt = 0; jt < C::KT / 32; jt++) {
      const int kt0 = j0 + jt * 32;
      if (kt0 >= L) break;   // uniform over the workgroup
      BiasTile<T> bt;
      attn_load_bias(bplane, L, kt0 >> 5, bcolq, g, bt);
      const int masked = __builtin_amdgcn_readfirstlane(lds_flag[jt]);
      const int off0 = (jt * 32 + l32) * C::RM + g * MM::KP;
      f32x16 sacc = splat16(0.0f), pacc = splat16(0.0f);
#pragma unroll
      for (int kk = 0; kk < MAXKK; kk++)
        if (kk < NKK) {
          MM::mma(sacc, MM::load(lds_k + off0 + kk * MM::KSTEP), qf[kk]);      // S^T = K Q^T
          MM::mma(pacc, MM::load(lds_v + off0 + kk * MM::KSTEP), dof[kk]);     // dP^T = V dO^T
        }
      attn_add_bias(sacc, bt, idf);
      if (masked) attn_add_row_mask(sacc, lds_madd + jt * 32, g);
#pragma unroll
      for (int e = 0; e < 16; e++) sacc[e] = fast_exp2(sacc[e] - lse2) * (pacc[e] - Di);     // dS = P (dP - D)
      // the upper group hands its dS tile over; the lower group adds its own and writes the sum
      if (grp == 1) {
#pragma unroll
        for (int e = 0; e < 16; e++) lds_x[xb][wave][e][lane] = bvalid ? sacc[e] : 0.0f;
      }
      __syncthreads();
      if (grp == 0 && qok) {   // 16-byte stores; a half wave's lanes write 512 contiguous bytes each
        float v16[16];
#pragma unroll
        for (int e = 0; e < 16; e++) v16[e] = sacc[e] + lds_x[xb][wave][e][lane];
        attn_store_tile16<T>(dsplane, L, kt0 >> 5, qi, g, v16);
      }
      xb ^= 1;
      const T* krow = lds_kt + l32 * C::TS + jt * 32;
#pragma unroll
      for (int uu = 0; uu < 32 / MM::KSTEP; uu++) MM::mma(dq, lds_tfrag<T>(krow, g, uu), acc_to_frag<T>(sacc, uu));
    }
  }
  if (!qok || !bvalid) return;
  T* pdq = (T*)a.dqkvg + orow;
#pragma unroll
  for (int q4 = 0; q4 < 4; q4++) {
    int dd = 8 * q4 + 4 * g;
    if (dd < d) {
      float v[4];
#pragma unroll
      for (int r = 0; r < 4; r++) v[r] = dq[q4 * 4 + r] * a.scale;
      store4<T>(pdq + dd, v);
    }
  }
}

// ---------------------------------------------------------------------------
// Backward, dK and dV.  Wave w owns keys k0 = tile*128 + 32*w (a key is a lane);
// loops over query tiles staged in LDS (row-major and transposed copies of Q and dO).
// ---------------------------------------------------------------------------
#ifndef PE_DKV_WAVES
#define PE_DKV_WAVES 3
#endif
template <typename T, bool HAS_BIAS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PE_DKV_WAVES, PE_DKV_WAVES))) void attn_bwd_dkv_kernel(AttnArgs a) {
  typedef AttnCfg<T> C;
  typedef Mma<T> MM;
  __shared__ __attribute__((aligned(16))) T lds_q[C::KT * C::RM];
  __shared__ __attribute__((aligned(16))) T lds_qt[32 * C::TS];
  __shared__ __attribute__((aligned(16))) T lds_do[C::KT * C::RM];
  __shared__ __attribute__((aligned(16))) T lds_dot[32 * C::TS];
  __shared__ __attribute__((aligned(16))) float lds_lse[C::KT];   // minus the base-2 log-sum-exp, -inf beyond L
  __shared__ __attribute__((aligned(16))) float lds_D[C::KT];     // minus D

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const AttnWg wg = attn_decode_wg(a);
  if (!wg.ok) return;
  const int h = wg.h, b = wg.b;
  const int L = a.L, d = a.d;
  const int DP = round_up_i(d, MM::KSTEP);
  const int NKK = DP / MM::KSTEP;
  const int kj = wg.tile * 128 + wave * 32 + l32;       // this lane's key
  const bool kok = kj < L;
  const long long HP = (long long)a.H * a.plane;
  const T* base = (const T*)a.qkvg + h * a.plane + (long long)b * L * d;
  const T* krow = kok ? base + HP + kj * d : nullptr;
  const T* vrow = kok ? base + 2 * HP + kj * d : nullptr;
  const T* dobase = (const T*)a.dO + h * a.plane + (long long)b * L * d;

  constexpr int MAXKK = 32 / MM::KSTEP;
  typename MM::frag kf[MAXKK], vf[MAXKK];
#pragma unroll
  for (int kk = 0; kk < MAXKK; kk++)
    if (kk < NKK) {
      kf[kk] = gl_frag<T>(krow, kk, g, d);
      vf[kk] = gl_frag<T>(vrow, kk, g, d);
    }
  const float mk = kok ? a.mask[(long long)b * a.mask_bs + (long long)kj * a.mask_ks] : 0.0f;
  const float madd = (mk > 0.0f) ? 0.0f : -INFINITY;
  const bool wave_masked = __any(!(mk > 0.0f));          // some key of this wave is masked or padded
  constexpr bool has_bias = HAS_BIAS;
  const T* bplane = has_bias ? (const T*)a.biasK + (long long)h * attn_tiles32(L) * L * 32 : nullptr;
  const int bcolk = min(kj, L - 1);
  IdFrag<T> idf;
  idf.init(l32, g);

  f32x16 dk, dv;
#pragma unroll
  for (int e = 0; e < 16; e++) { dk[e] = 0.0f; dv[e] = 0.0f; }

  // Q, dO, -lse and -D of the next 64 queries are loaded into registers while the current ones are used; the bias
  // one 32-query tile ahead of its use
  AttnStageRegs<T> rq, rdo;
  float r_lse = 0.0f, r_D = 0.0f;
  auto prefetch = [&](int i0) {
    attn_stage_load<T>(base, d, i0, L, d, DP, rq, tid);
    attn_stage_load<T>(dobase, d, i0, L, d, DP, rdo, tid);
    const int i = i0 + tid;
    const bool ok = tid < C::KT && i < L;
    const long long sidx = ((long long)b * a.H + h) * L + (ok ? i : 0);
    r_lse = ok ? -a.lse[sidx] * PE_LOG2E : -INFINITY;
    r_D = ok ? -a.D[sidx] : 0.0f;
  };
  prefetch(0);
  const int ntile = attn_tiles32(L);
  BiasTile<T> bt;                       // refilled for the next 32-query tile as soon as its MFMAs have taken it
  if (has_bias) attn_load_bias(bplane, L, 0, bcolk, g, bt);
  for (int i0 = 0; i0 < L; i0 += C::KT) {
    __syncthreads();
    attn_stage_store<T>(rq, DP, lds_q, lds_qt, tid);
    attn_stage_store<T>(rdo, DP, lds_do, lds_dot, tid);
    if (tid < C::KT) { lds_lse[tid] = r_lse; lds_D[tid] = r_D; }
    __syncthreads();
    if (i0 + C::KT < L) prefetch(i0 + C::KT);
#pragma unroll
    for (int it = 0; it < C::KT / 32; it++) {
      if (i0 + it * 32 >= L) break;
      // C operands: -lse and -D of the tile's queries in accumulator order
      f32x16 sacc, pacc;
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const f32x4 ls = *reinterpret_cast<const f32x4*>(lds_lse + it * 32 + 8 * q4 + 4 * g);
        const f32x4 Dr = *reinterpret_cast<const f32x4*>(lds_D + it * 32 + 8 * q4 + 4 * g);
#pragma unroll
        for (int r = 0; r < 4; r++) { sacc[q4 * 4 + r] = ls[r]; pacc[q4 * 4 + r] = Dr[r]; }
      }
#pragma unroll
      for (int kk = 0; kk < MAXKK; kk++)
        if (kk < NKK) {
          int off = (it * 32 + l32) * C::RM + kk * MM::KSTEP + g * MM::KP;
          MM::mma(sacc, MM::load(lds_q + off), kf[kk]);      // S - lse = Q K^T - lse   (rows queries, col = key lane)
          MM::mma(pacc, MM::load(lds_do + off), vf[kk]);     // dP - D = dO V^T - D
        }
      if (has_bias) {
        attn_add_bias(sacc, bt, idf);
        attn_load_bias(bplane, L, min((i0 >> 5) + it + 1, ntile - 1), bcolk, g, bt);
      }
      if (wave_masked) {
#pragma unroll
        for (int e = 0; e < 16; e++) sacc[e] += madd;
      }
      f32x16 pv;
#pragma unroll
      for (int e = 0; e < 16; e++) {
        const float p = fast_exp2(sacc[e]);
        pv[e] = p;
        sacc[e] = p * pacc[e];                                // dS = P (dP - D)
      }
      const T* dotrow = lds_dot + l32 * C::TS + it * 32;
      const T* qtrow = lds_qt + l32 * C::TS + it * 32;
#pragma unroll
      for (int u = 0; u < 32 / MM::KSTEP; u++) {
        MM::mma(dv, lds_tfrag<T>(dotrow, g, u), acc_to_frag<T>(pv, u));     // dV^T += dO^T P
        MM::mma(dk, lds_tfrag<T>(qtrow, g, u), acc_to_frag<T>(sacc, u));    // dK^T += Q^T dS
      }
    }
  }
  if (!kok) return;
  T* pdk = (T*)a.dqkvg + HP + h * a.plane + ((long long)b * L + kj) * d;
  T* pdv = pdk + HP;
#pragma unroll
  for (int q4 = 0; q4 < 4; q4++) {
    int dd = 8 * q4 + 4 * g;
    if (dd < d) {
      float v1[4], v2[4];
#pragma unroll
      for (int r = 0; r < 4; r++) { v1[r] = dk[q4 * 4 + r] * PE_LN2; v2[r] = dv[q4 * 4 + r]; }   // q' = q scale log2 e
      store4<T>(pdk + dd, v1);
      store4<T>(pdv + dd, v2);
    }
  }
}

// The same reduction with 8 consecutive outputs per thread (16-byte loads for bf16) and eight loads in
// flight: 64 output groups x 4 batch lanes per workgroup.  Needs hll % 8 == 0 and 16-byte aligned buffers.
template <typename T>
__global__ __launch_bounds__(256) void attn_dbias_reduce8_kernel(const T* dS, float* dbias, int B, long long hll) {
  __shared__ float red[3][64][8];
  const int x = threadIdx.x & 63, y = threadIdx.x >> 6;
  const long long idx = ((long long)blockIdx.x * 64 + x) * 8;
  float s[8];
#pragma unroll
  for (int e = 0; e < 8; e++) s[e] = 0.0f;
  if (idx < hll) {
    for (int b = y; b < B; b += 32) {
      float v[8][8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int bb = b + 4 * u;
        if (bb < B) ld8_once<T>(dS + (long long)bb * hll + idx, v[u]);
        else {
#pragma unroll
          for (int e = 0; e < 8; e++) v[u][e] = 0.0f;
        }
      }
#pragma unroll
      for (int e = 0; e < 8; e++)
        s[e] += ((v[0][e] + v[1][e]) + (v[2][e] + v[3][e])) + ((v[4][e] + v[5][e]) + (v[6][e] + v[7][e]));
    }
  }
  if (y != 0) {
#pragma unroll
    for (int e = 0; e < 8; e++) red[y - 1][x][e] = s[e];
  }
  __syncthreads();
  if (y != 0 || idx >= hll) return;
#pragma unroll
  for (int k = 0; k < 3; k++)
#pragma unroll
    for (int e = 0; e < 8; e++) s[e] += red[k][x][e];
  st8<float>(dbias + idx, s);
}

// dbiasT[h][j][i] = sum_b dS[b][h][j][i]  (elementwise over the trailing [H][L][L] block)
// 256 threads = 64 groups of 4 consecutive outputs x 4 batch lanes; 8- / 16-byte loads
template <typename T>
__global__ __launch_bounds__(256) void attn_dbias_reduce_kernel(const T* dS, float* dbias, int B, long long hll) {
  __shared__ float red[256][4];
  const int x = threadIdx.x & 63, y = threadIdx.x >> 6;
  const long long idx = ((long long)blockIdx.x * 64 + x) * 4;
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (idx < hll) {
    if ((hll & 3) == 0) {
      for (int b = y; b < B; b += 16) {      // 4 independent loads in flight
        float v[4][4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
          int bb = b + 4 * u;
          if (bb < B) load4<T>(dS + (long long)bb * hll + idx, v[u]);
          else { v[u][0] = v[u][1] = v[u][2] = v[u][3] = 0.0f; }
        }
#pragma unroll
        for (int e = 0; e < 4; e++) s[e] += (v[0][e] + v[1][e]) + (v[2][e] + v[3][e]);
      }
    } else {
      for (int b = y; b < B; b += 4)
        for (int e = 0; e < 4; e++)
          if (idx + e < hll) s[e] += to_f(dS[(long long)b * hll + idx + e]);
    }
  }
  red[threadIdx.x][0] = s[0]; red[threadIdx.x][1] = s[1]; red[threadIdx.x][2] = s[2]; red[threadIdx.x][3] = s[3];
  __syncthreads();
  if (y != 0 || idx >= hll) return;
  for (int k = 1; k < 4; k++)
    for (int e = 0; e < 4; e++) s[e] += red[k * 64 + x][e];
  for (int e = 0; e < 4; e++)
    if (idx + e < hll) dbias[idx + e] = s[e];
}
