// Global column attention of the extra-MSA blocks: one mask-averaged query per (residue,
// head), single-head keys and values, attention over the sequence axis.
//
// Projections live in one tensor proj[s][r][Wg], Wg = 2*H*d + 2*d, row layout
// [ q (H*d) | k (d) | v (d) | gate (H*d) ].  Per residue the work is tiny (H*s logits,
// d = 8), so these are plain-ALU / HBM-bound kernels: one workgroup per residue, three
// passes over the sequence axis (max, sum, output) that recompute the d-wide dot products
// instead of storing logits.  H <= 8, d <= 8.
#pragma once
#include "pe_common.h"
#include "pe_elem.h"

constexpr int GC_MAXH = 8, GC_MAXD = 8;

struct GcolArgs {
  const void* proj; void* dproj;    // [s][r][Wg] storage type
  const float* mask;                // msa_mask[s][r]
  float* qbar;                      // [r][H*d]
  float* den;                       // [r]   sum_s mask + 1e-10
  float* p;                         // [r][H][s] attention weights
  float* o;                         // [r][H*d]
  void* og;                         // [s][r][H*d] storage type, sigmoid(gate) * o
  const void* dog;                  // cotangent of og
  float* dO;                        // [r][H*d]  sum_s dog * sigmoid(gate)
  float* dqbar;                     // [r][H*d]
  int s, r, H, d;
  float scale;
  float* part;                      // [chunks][r][H*d] partial sums over sequence chunks (qmean: numerators; gate_bwd: dO)
  float* partm;                     // [chunks][r] partial mask sums (qmean)
  int chunks;                       // sequence chunks of gc_chunk_len(H*d) positions
};
// sequence positions per workgroup of the two reductions over s (up to four per sequence lane, 16-byte loads)
static inline int gc_chunk_len(int HD) { return 32 * (256 / HD); }

// d (<= 8) consecutive channels of one (sequence, residue) row -> float[8] (zero beyond d)
template <typename T> PE_DEV void gc_load_row(const T* p, int d, float (&v)[GC_MAXD]) {
  if (d == GC_MAXD) { ld8<T>(p, v); return; }   // 16 / 32 bytes, aligned: row offsets are multiples of 8 channels
#pragma unroll
  for (int c = 0; c < GC_MAXD; c++) v[c] = c < d ? to_f(p[c]) : 0.0f;
}

PE_DEV float block_reduce_sum(float v, float* red /*[4]*/) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}
PE_DEV float block_reduce_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// qbar[i][hd] = sum_s mask[s][i] q[s][i][hd] / den[i], in two stages: grid (r, chunks), block = 256 = (HD / 8) column
// groups x sequence lanes; a workgroup sums one chunk of gc_chunk_len(HD) sequence positions of one residue (up to four
// independent 16-byte loads in flight per thread) into part / partm, gcol_qmean_fin_kernel adds the chunks in order.
// (One workgroup per residue walking the whole sequence axis ran at 0.2 TB/s: 256 workgroups, each a chain of
// dependent load rounds; 2-byte loads, one column per thread, at 0.8 TB/s.)
template <typename T>
__global__ __launch_bounds__(256) void gcol_qmean_kernel(GcolArgs a) {
  // a thread owns 8 consecutive (head, channel) columns (one 16-byte load in the storage type) of up to four sequence
  // positions of the chunk; TPP threads cover a position, SL sequence lanes a workgroup
  __shared__ float red[256][8], redm[256];
  const int i = blockIdx.x, ch = blockIdx.y, HD = a.H * a.d, Wg = 2 * HD + 2 * a.d;
  const int TPP = HD / 8, SL = 256 / TPP, hd0 = ((int)threadIdx.x % TPP) * 8, sl = threadIdx.x / TPP;
  const int len = 32 * (256 / HD), tbeg = ch * len, tend = min(a.s, tbeg + len);   // the chunk of gc_chunk_len(HD) positions
  float acc[8], msum = 0.0f;
#pragma unroll
  for (int e = 0; e < 8; e++) acc[e] = 0.0f;
  if (sl < SL) {
    float mk[4], qv[4][8];
#pragma unroll
    for (int u = 0; u < 4; u++) {   // all loads first (4 SL >= len for every H*d), then the arithmetic
      const int t = tbeg + sl + u * SL;
      const bool ok = t < tend;
      const long long pos = (long long)(ok ? t : tbeg) * a.r + i;
      mk[u] = ok ? a.mask[pos] : 0.0f;
      ld8<T>((const T*)a.proj + pos * Wg + hd0, qv[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      if (tbeg + sl + u * SL < tend) {
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] += mk[u] * qv[u][e];
        msum += mk[u];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; e++) red[threadIdx.x][e] = acc[e];
  redm[threadIdx.x] = msum;
  __syncthreads();
  if (sl == 0) {
    for (int k = 1; k < SL; k++) {
#pragma unroll
      for (int e = 0; e < 8; e++) acc[e] += red[k * TPP + (int)threadIdx.x][e];
      msum += redm[k * TPP + (int)threadIdx.x];
    }
    st8<float>(a.part + ((long long)ch * a.r + i) * HD + hd0, acc);
    if (hd0 == 0) a.partm[(long long)ch * a.r + i] = msum;
  }
}
// grid = ceil(r * HD / 256)
__global__ __launch_bounds__(256) void gcol_qmean_fin_kernel(GcolArgs a) {
  const int HD = a.H * a.d;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)a.r * HD) return;
  const int i = (int)(idx / HD);
  float acc = 0.0f, msum = 0.0f;
  for (int c = 0; c < a.chunks; c++) {
    acc += a.part[(long long)c * a.r * HD + idx];
    msum += a.partm[(long long)c * a.r + i];
  }
  const float den = msum + 1e-10f;
  a.qbar[idx] = acc / den;
  if (idx % HD == 0) a.den[i] = den;
}

// softmax over the sequence axis and weighted value sum; grid = r, block = 256.
// Every pass walks the sequence axis 4 positions per thread at a time: the 4 (k, v) rows and
// masks are loaded first (one 16-byte load per row when d = 8), then used; all per-head arrays
// have compile-time bounds (H <= 8, d <= 8 with guards) and live in registers.
constexpr int GC_U = 4;
template <typename T>
__global__ __launch_bounds__(256) void gcol_attn_fwd_kernel(GcolArgs a) {
  __shared__ float qb[GC_MAXH * GC_MAXD], red[4], ored[4][GC_MAXH * GC_MAXD];
  const int i = blockIdx.x, H = a.H, d = a.d, HD = H * d, Wg = 2 * HD + 2 * d;
  if (threadIdx.x < GC_MAXH * GC_MAXD) {
    const int h = threadIdx.x / GC_MAXD, c = threadIdx.x % GC_MAXD;
    qb[threadIdx.x] = (h < H && c < d) ? a.qbar[(long long)i * HD + h * d + c] * a.scale : 0.0f;   // scaled query, padded
  }
  __syncthreads();
  float q[GC_MAXH][GC_MAXD];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++)
#pragma unroll
    for (int c = 0; c < GC_MAXD; c++) q[h][c] = qb[h * GC_MAXD + c];
  const T* kbase = (const T*)a.proj + (long long)i * Wg + HD;
  const long long tstride = (long long)a.r * Wg;
  float mx[GC_MAXH], sm[GC_MAXH];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++) { mx[h] = -INFINITY; sm[h] = 0.0f; }
  // pass 1: max over valid keys
  for (int t0 = threadIdx.x; t0 < a.s; t0 += 256 * GC_U) {
    float kv[GC_U][GC_MAXD], mk[GC_U];
#pragma unroll
    for (int u = 0; u < GC_U; u++) {
      const int t = t0 + 256 * u;
      const bool ok = t < a.s;
      mk[u] = ok ? a.mask[(long long)t * a.r + i] : 0.0f;
      gc_load_row<T>(kbase + (ok ? t : 0) * tstride, d, kv[u]);
    }
#pragma unroll
    for (int u = 0; u < GC_U; u++)
      if (mk[u] > 0.0f) {
#pragma unroll
        for (int h = 0; h < GC_MAXH; h++) {
          float l = 0.0f;
#pragma unroll
          for (int c = 0; c < GC_MAXD; c++) l += q[h][c] * kv[u][c];
          mx[h] = fmaxf(mx[h], l);
        }
      }
  }
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++) {
    mx[h] = block_reduce_max(mx[h], red);
    if (mx[h] == -INFINITY) mx[h] = 0.0f;
  }
  // pass 2: sum of exponentials
  for (int t0 = threadIdx.x; t0 < a.s; t0 += 256 * GC_U) {
    float kv[GC_U][GC_MAXD], mk[GC_U];
#pragma unroll
    for (int u = 0; u < GC_U; u++) {
      const int t = t0 + 256 * u;
      const bool ok = t < a.s;
      mk[u] = ok ? a.mask[(long long)t * a.r + i] : 0.0f;
      gc_load_row<T>(kbase + (ok ? t : 0) * tstride, d, kv[u]);
    }
#pragma unroll
    for (int u = 0; u < GC_U; u++)
      if (mk[u] > 0.0f) {
#pragma unroll
        for (int h = 0; h < GC_MAXH; h++) {
          float l = 0.0f;
#pragma unroll
          for (int c = 0; c < GC_MAXD; c++) l += q[h][c] * kv[u][c];
          sm[h] += __expf(l - mx[h]);
        }
      }
  }
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++) sm[h] = block_reduce_sum(sm[h], red);
  // pass 3: weights and output
  float oacc[GC_MAXH][GC_MAXD];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++)
#pragma unroll
    for (int c = 0; c < GC_MAXD; c++) oacc[h][c] = 0.0f;
  for (int t0 = threadIdx.x; t0 < a.s; t0 += 256 * GC_U) {
    float kv[GC_U][GC_MAXD], vv[GC_U][GC_MAXD], mk[GC_U];
#pragma unroll
    for (int u = 0; u < GC_U; u++) {
      const int t = t0 + 256 * u;
      const bool ok = t < a.s;
      mk[u] = ok ? a.mask[(long long)t * a.r + i] : 0.0f;
      const T* row = kbase + (ok ? t : 0) * tstride;
      gc_load_row<T>(row, d, kv[u]);
      gc_load_row<T>(row + d, d, vv[u]);
    }
#pragma unroll
    for (int u = 0; u < GC_U; u++) {
      const int t = t0 + 256 * u;
      if (t < a.s) {
#pragma unroll
        for (int h = 0; h < GC_MAXH; h++) {
          if (h < H) {
            float l = 0.0f;
#pragma unroll
            for (int c = 0; c < GC_MAXD; c++) l += q[h][c] * kv[u][c];
            float pw = (mk[u] > 0.0f && sm[h] > 0.0f) ? __expf(l - mx[h]) / sm[h] : 0.0f;
            a.p[((long long)i * H + h) * a.s + t] = pw;
#pragma unroll
            for (int c = 0; c < GC_MAXD; c++) oacc[h][c] += pw * vv[u][c];
          }
        }
      }
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++)
#pragma unroll
    for (int c = 0; c < GC_MAXD; c++) {
      float v = wave_sum(oacc[h][c]);
      if (lane == 0) ored[wave][h * GC_MAXD + c] = v;
    }
  __syncthreads();
  if (threadIdx.x < HD) {
    int h = threadIdx.x / d, c = threadIdx.x % d, k = h * GC_MAXD + c;
    a.o[(long long)i * HD + threadIdx.x] = ored[0][k] + ored[1][k] + ored[2][k] + ored[3][k];
  }
}

// og[t][i][hd] = sigmoid(gate[t][i][hd]) * o[i][hd]
template <typename T>
__global__ void gcol_gate_fwd_kernel(GcolArgs a) {
  const int HD = a.H * a.d, Wg = 2 * HD + 2 * a.d;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  long long total = (long long)a.s * a.r * HD;
  if (idx >= total) return;
  int hd = idx % HD;
  long long pos = idx / HD;
  int i = pos % a.r;
  float g = to_f(((const T*)a.proj)[pos * Wg + HD + 2 * a.d + hd]);
  ((T*)a.og)[idx] = from_f<T>(sigmoidf_(g) * a.o[(long long)i * HD + hd]);
}

// the same with 8 consecutive channels per thread (16-byte accesses): needs (H*d) % 8 == 0 and d % 4 == 0
template <typename T>
__global__ __launch_bounds__(256) void gcol_gate_fwd8_kernel(GcolArgs a) {
  const int HD = a.H * a.d, Wg = 2 * HD + 2 * a.d, HD8 = HD >> 3;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)a.s * a.r * HD8) return;
  const int hd0 = (int)(idx % HD8) * 8;
  const long long pos = idx / HD8;
  const int i = (int)(pos % a.r);
  float g[8], o[8];
  ld8<T>((const T*)a.proj + pos * Wg + HD + 2 * a.d + hd0, g);
  ld8<float>(a.o + (long long)i * HD + hd0, o);
#pragma unroll
  for (int e = 0; e < 8; e++) o[e] *= sigmoidf_(g[e]);
  st8<T>((T*)a.og + pos * HD + hd0, o);
}

// dO[i][hd] = sum_t dog * sigmoid(g);  dgate = dog * o * s(1-s) -> dproj gate slot.  Two stages like the mean query:
// grid (r, chunks) writes the chunk sums to part, gcol_sum_chunks_kernel adds them in order.
template <typename T>
__global__ __launch_bounds__(256) void gcol_gate_bwd_kernel(GcolArgs a) {
  // a thread owns 8 consecutive (head, channel) columns (16-byte accesses in the storage type; H*d is a multiple of 8)
  // of up to four sequence positions of the chunk; TPP threads cover a position, SL sequence lanes a workgroup
  __shared__ float red[256][8];
  const int i = blockIdx.x, ch = blockIdx.y, HD = a.H * a.d, Wg = 2 * HD + 2 * a.d;
  const int TPP = HD / 8, SL = 256 / TPP, hd0 = ((int)threadIdx.x % TPP) * 8, sl = threadIdx.x / TPP;
  const int len = 32 * (256 / HD), tbeg = ch * len, tend = min(a.s, tbeg + len);   // the chunk of gc_chunk_len(HD) positions
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; e++) acc[e] = 0.0f;
  if (sl < SL) {
    float ov[8], gv[4][8], dv[4][8];
    ld8<float>(a.o + (long long)i * HD + hd0, ov);
#pragma unroll
    for (int u = 0; u < 4; u++) {   // all loads first (4 SL >= len for every H*d), then the arithmetic
      const int t = tbeg + sl + u * SL;
      const long long pos = (long long)(t < tend ? t : tbeg) * a.r + i;
      ld8<T>((const T*)a.proj + pos * Wg + HD + 2 * a.d + hd0, gv[u]);
      ld8<T>((const T*)a.dog + pos * HD + hd0, dv[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int t = tbeg + sl + u * SL;
      if (t < tend) {
        const long long pos = (long long)t * a.r + i;
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
          const float sg = sigmoidf_(gv[u][e]);
          acc[e] += dv[u][e] * sg;
          o[e] = dv[u][e] * ov[e] * sg * (1.0f - sg);
        }
        st8<T>((T*)a.dproj + pos * Wg + HD + 2 * a.d + hd0, o);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; e++) red[threadIdx.x][e] = acc[e];
  __syncthreads();
  if (sl == 0) {
    for (int k = 1; k < SL; k++)
#pragma unroll
      for (int e = 0; e < 8; e++) acc[e] += red[k * TPP + (int)threadIdx.x][e];
    st8<float>(a.part + ((long long)ch * a.r + i) * HD + hd0, acc);
  }
}
// out[idx] = sum_c part[c][idx], idx < n;  grid = ceil(n / 256)
__global__ __launch_bounds__(256) void gcol_sum_chunks_kernel(const float* part, float* out, int chunks, long long n) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  float acc = 0.0f;
  for (int c = 0; c < chunks; c++) acc += part[(long long)c * n + idx];
  out[idx] = acc;
}

// softmax backward per residue: dk, dv -> dproj; dqbar.  grid = r, block = 256; same batching
// and register-resident per-head arrays as the forward kernel
template <typename T>
__global__ __launch_bounds__(256) void gcol_attn_bwd_kernel(GcolArgs a) {
  __shared__ float qb[GC_MAXH * GC_MAXD], dob[GC_MAXH * GC_MAXD], red[4], qred[4][GC_MAXH * GC_MAXD];
  const int i = blockIdx.x, H = a.H, d = a.d, HD = H * d, Wg = 2 * HD + 2 * d;
  if (threadIdx.x < GC_MAXH * GC_MAXD) {
    const int h = threadIdx.x / GC_MAXD, c = threadIdx.x % GC_MAXD;
    const bool in = h < H && c < d;
    qb[threadIdx.x] = in ? a.qbar[(long long)i * HD + h * d + c] : 0.0f;
    dob[threadIdx.x] = in ? a.dO[(long long)i * HD + h * d + c] : 0.0f;
  }
  __syncthreads();
  float q[GC_MAXH][GC_MAXD], dov[GC_MAXH][GC_MAXD];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++)
#pragma unroll
    for (int c = 0; c < GC_MAXD; c++) { q[h][c] = qb[h * GC_MAXD + c]; dov[h][c] = dob[h * GC_MAXD + c]; }
  const T* kbase = (const T*)a.proj + (long long)i * Wg + HD;
  T* dkbase = (T*)a.dproj + (long long)i * Wg + HD;
  const long long tstride = (long long)a.r * Wg;
  float D[GC_MAXH];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++) D[h] = 0.0f;
  for (int t0 = threadIdx.x; t0 < a.s; t0 += 256 * GC_U) {
    float vv[GC_U][GC_MAXD], pw[GC_U][GC_MAXH];
#pragma unroll
    for (int u = 0; u < GC_U; u++) {
      const int t = t0 + 256 * u;
      const bool ok = t < a.s;
      gc_load_row<T>(kbase + (ok ? t : 0) * tstride + d, d, vv[u]);
#pragma unroll
      for (int h = 0; h < GC_MAXH; h++) pw[u][h] = (ok && h < H) ? a.p[((long long)i * H + h) * a.s + t] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < GC_U; u++)
#pragma unroll
      for (int h = 0; h < GC_MAXH; h++) {
        float dp = 0.0f;
#pragma unroll
        for (int c = 0; c < GC_MAXD; c++) dp += dov[h][c] * vv[u][c];
        D[h] += pw[u][h] * dp;
      }
  }
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++) D[h] = block_reduce_sum(D[h], red);
  float dq[GC_MAXH][GC_MAXD];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++)
#pragma unroll
    for (int c = 0; c < GC_MAXD; c++) dq[h][c] = 0.0f;
  for (int t0 = threadIdx.x; t0 < a.s; t0 += 256 * GC_U) {
    float kv[GC_U][GC_MAXD], vv[GC_U][GC_MAXD], pw[GC_U][GC_MAXH];
#pragma unroll
    for (int u = 0; u < GC_U; u++) {
      const int t = t0 + 256 * u;
      const bool ok = t < a.s;
      const T* row = kbase + (ok ? t : 0) * tstride;
      gc_load_row<T>(row, d, kv[u]);
      gc_load_row<T>(row + d, d, vv[u]);
#pragma unroll
      for (int h = 0; h < GC_MAXH; h++) pw[u][h] = (ok && h < H) ? a.p[((long long)i * H + h) * a.s + t] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < GC_U; u++) {
      const int t = t0 + 256 * u;
      if (t < a.s) {
        float dk[GC_MAXD], dv[GC_MAXD];
#pragma unroll
        for (int c = 0; c < GC_MAXD; c++) { dk[c] = 0.0f; dv[c] = 0.0f; }
#pragma unroll
        for (int h = 0; h < GC_MAXH; h++) {
          float dp = 0.0f;
#pragma unroll
          for (int c = 0; c < GC_MAXD; c++) dp += dov[h][c] * vv[u][c];
          const float dl = pw[u][h] * (dp - D[h]);
#pragma unroll
          for (int c = 0; c < GC_MAXD; c++) {
            dq[h][c] += dl * kv[u][c];
            dk[c] += dl * q[h][c];
            dv[c] += pw[u][h] * dov[h][c];
          }
        }
        T* orow = dkbase + t * tstride;
        if (d == GC_MAXD) {
          float o1[8], o2[8];
#pragma unroll
          for (int c = 0; c < GC_MAXD; c++) { o1[c] = dk[c] * a.scale; o2[c] = dv[c]; }
          st8<T>(orow, o1);
          st8<T>(orow + d, o2);
        } else {
#pragma unroll
          for (int c = 0; c < GC_MAXD; c++)
            if (c < d) { orow[c] = from_f<T>(dk[c] * a.scale); orow[d + c] = from_f<T>(dv[c]); }
        }
      }
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++)
#pragma unroll
    for (int c = 0; c < GC_MAXD; c++) {
      float v = wave_sum(dq[h][c]);
      if (lane == 0) qred[wave][h * GC_MAXD + c] = v;
    }
  __syncthreads();
  if (threadIdx.x < HD) {
    int h = threadIdx.x / d, c = threadIdx.x % d, k = h * GC_MAXD + c;
    a.dqbar[(long long)i * HD + threadIdx.x] = (qred[0][k] + qred[1][k] + qred[2][k] + qred[3][k]) * a.scale;
  }
}

// dq[t][i][hd] = mask[t][i] * dqbar[i][hd] / den[i] -> dproj q slot
template <typename T>
__global__ void gcol_dq_kernel(GcolArgs a) {
  const int HD = a.H * a.d, Wg = 2 * HD + 2 * a.d;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  long long total = (long long)a.s * a.r * HD;
  if (idx >= total) return;
  int hd = idx % HD;
  long long pos = idx / HD;
  int i = pos % a.r;
  ((T*)a.dproj)[pos * Wg + hd] = from_f<T>(a.mask[pos] * a.dqbar[(long long)i * HD + hd] / a.den[i]);
}

// the same with 8 consecutive channels per thread (16-byte stores): needs (H*d) % 8 == 0 and d % 4 == 0
template <typename T>
__global__ __launch_bounds__(256) void gcol_dq8_kernel(GcolArgs a) {
  const int HD = a.H * a.d, Wg = 2 * HD + 2 * a.d, HD8 = HD >> 3;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)a.s * a.r * HD8) return;
  const int hd0 = (int)(idx % HD8) * 8;
  const long long pos = idx / HD8;
  const int i = (int)(pos % a.r);
  float v[8];
  ld8<float>(a.dqbar + (long long)i * HD + hd0, v);
  const float f = a.mask[pos], den = a.den[i];
#pragma unroll
  for (int e = 0; e < 8; e++) v[e] = f * v[e] / den;
  st8<T>((T*)a.dproj + pos * Wg + hd0, v);
}
