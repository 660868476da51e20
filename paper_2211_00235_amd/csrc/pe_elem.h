// HBM-bound kernels of the block: LayerNorm (forward / backward, channel-last and
// channel-major), the pair-bias projection fused with its LayerNorm, gating of the
// triangle-multiplication projections, reductions for parameter gradients, parameter
// preparation (fp32 -> storage type, transposed copies).
//
// Row-wise kernels give one row to one 64-lane wave: lane l holds channels
// c = (ch*64 + l)*4 + 0..3 for ch < NCH (8- or 16-byte loads), row statistics are wave
// reductions, per-channel parameter-gradient partial sums stay in registers over the
// wave's rows and are written once per workgroup as fp32 partials; a second small
// kernel reduces the partials in a fixed order (deterministic, no atomics).
#pragma once
#include "pe_common.h"

constexpr int LN_NCH = 4;          // channels <= 64*4*LN_NCH = 1024
constexpr int LN_MAX_WG = 2048;    // workgroups (x4 waves) of the row-wise backward kernels

template <typename T> PE_DEV void load4(const T* p, float (&v)[4]);
template <> PE_DEV void load4<float>(const float* p, float (&v)[4]) {
  f32x4 t = *reinterpret_cast<const f32x4*>(p);
  v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
}
template <> PE_DEV void load4<bf16>(const bf16* p, float (&v)[4]) {
  bf16x4 t = *reinterpret_cast<const bf16x4*>(p);
  v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
}
template <typename T> PE_DEV void store4(T* p, const float (&v)[4]);
template <> PE_DEV void store4<float>(float* p, const float (&v)[4]) {
  f32x4 t; t[0] = v[0]; t[1] = v[1]; t[2] = v[2]; t[3] = v[3];
  *reinterpret_cast<f32x4*>(p) = t;
}
template <> PE_DEV void store4<bf16>(bf16* p, const float (&v)[4]) {
  bf16x4 t; t[0] = (bf16)v[0]; t[1] = (bf16)v[1]; t[2] = (bf16)v[2]; t[3] = (bf16)v[3];
  *reinterpret_cast<bf16x4*>(p) = t;
}

// ---------------------------------------------------------------------------
// LayerNorm forward, channel-last: y = (x - mu) * rstd * gamma + beta; stats = (mu, rstd)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* x, const float* gamma, const float* beta, T* y,
                                                     float* stats, long long M, int C, float eps) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float gm[LN_NCH][4], bt[LN_NCH][4];
#pragma unroll
  for (int ch = 0; ch < LN_NCH; ch++) {
    int c = (ch * 64 + lane) * 4;
#pragma unroll
    for (int e = 0; e < 4; e++) { gm[ch][e] = (c < C) ? gamma[c + e] : 0.0f; bt[ch][e] = (c < C) ? beta[c + e] : 0.0f; }
  }
  for (long long row = (long long)blockIdx.x * 4 + wave; row < M; row += (long long)gridDim.x * 4) {
    float v[LN_NCH][4];
    float s = 0.0f;
#pragma unroll
    for (int ch = 0; ch < LN_NCH; ch++) {
      int c = (ch * 64 + lane) * 4;
      if (c < C) load4<T>(x + row * C + c, v[ch]);
      else { v[ch][0] = v[ch][1] = v[ch][2] = v[ch][3] = 0.0f; }
      s += v[ch][0] + v[ch][1] + v[ch][2] + v[ch][3];
    }
    float mu = wave_sum(s) / C;
    float q = 0.0f;
#pragma unroll
    for (int ch = 0; ch < LN_NCH; ch++) {
      int c = (ch * 64 + lane) * 4;
      if (c < C) {
#pragma unroll
        for (int e = 0; e < 4; e++) { float t = v[ch][e] - mu; q += t * t; }
      }
    }
    float rstd = rsqrtf(wave_sum(q) / C + eps);
#pragma unroll
    for (int ch = 0; ch < LN_NCH; ch++) {
      int c = (ch * 64 + lane) * 4;
      if (c < C) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; e++) o[e] = (v[ch][e] - mu) * rstd * gm[ch][e] + bt[ch][e];
        store4<T>(y + row * C + c, o);
      }
    }
    if (lane == 0) { stats[row * 2] = mu; stats[row * 2 + 1] = rstd; }
  }
}

// ---------------------------------------------------------------------------
// LayerNorm backward, channel-last.
//   dx = (dxh - mean(dxh) - xh * mean(dxh * xh)) * rstd,  dxh = dy * gamma
//   gout = (gin ? gin : 0) + dx;  partial[wg][0:C] = sum dy*xh, partial[wg][C:2C] = sum dy
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const T* dy, const T* x, const float* stats, const float* gamma,
                                                     const T* gin, T* gout, float* partial, long long M, int C) {
  __shared__ float red[4][2 * 64 * 4 * LN_NCH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float gm[LN_NCH][4], dgs[LN_NCH][4], dbs[LN_NCH][4];
#pragma unroll
  for (int ch = 0; ch < LN_NCH; ch++) {
    int c = (ch * 64 + lane) * 4;
#pragma unroll
    for (int e = 0; e < 4; e++) { gm[ch][e] = (c < C) ? gamma[c + e] : 0.0f; dgs[ch][e] = 0.0f; dbs[ch][e] = 0.0f; }
  }
  for (long long row = (long long)blockIdx.x * 4 + wave; row < M; row += (long long)gridDim.x * 4) {
    float mu = stats[row * 2], rstd = stats[row * 2 + 1];
    float xh[LN_NCH][4], dxh[LN_NCH][4];
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int ch = 0; ch < LN_NCH; ch++) {
      int c = (ch * 64 + lane) * 4;
      if (c < C) {
        float xv[4], dv[4];
        load4<T>(x + row * C + c, xv);
        load4<T>(dy + row * C + c, dv);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          xh[ch][e] = (xv[e] - mu) * rstd;
          dxh[ch][e] = dv[e] * gm[ch][e];
          dgs[ch][e] += dv[e] * xh[ch][e];
          dbs[ch][e] += dv[e];
          s1 += dxh[ch][e];
          s2 += dxh[ch][e] * xh[ch][e];
        }
      }
    }
    s1 = wave_sum(s1) / C;
    s2 = wave_sum(s2) / C;
#pragma unroll
    for (int ch = 0; ch < LN_NCH; ch++) {
      int c = (ch * 64 + lane) * 4;
      if (c < C) {
        float o[4];
        if (gin) load4<T>(gin + row * C + c, o);
        else { o[0] = o[1] = o[2] = o[3] = 0.0f; }
#pragma unroll
        for (int e = 0; e < 4; e++) o[e] += (dxh[ch][e] - s1 - xh[ch][e] * s2) * rstd;
        store4<T>(gout + row * C + c, o);
      }
    }
  }
  // cross-wave reduction of the parameter-gradient partials
#pragma unroll
  for (int ch = 0; ch < LN_NCH; ch++)
#pragma unroll
    for (int e = 0; e < 4; e++) {
      int c = (ch * 64 + lane) * 4 + e;
      red[wave][c] = dgs[ch][e];
      red[wave][64 * 4 * LN_NCH + c] = dbs[ch][e];
    }
  __syncthreads();
  for (int c = threadIdx.x; c < C; c += 256) {
    float a = 0.0f, b = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; w++) { a += red[w][c]; b += red[w][64 * 4 * LN_NCH + c]; }
    partial[(long long)blockIdx.x * 2 * C + c] = a;
    partial[(long long)blockIdx.x * 2 * C + C + c] = b;
  }
}

// ---------------------------------------------------------------------------
// Fast LayerNorm path for C = 8 * LPR channels (LPR = lanes per row, a power of two <= 64):
// a wave handles 64 / LPR rows at once, every lane owns 8 consecutive channels (one 16-byte
// load for bf16), row statistics are reductions over LPR lanes.  Twice to eight times more
// bytes in flight per wave than the generic kernels above, which stay as the fallback.
// ---------------------------------------------------------------------------
template <typename T> PE_DEV void ld8(const T* p, float (&v)[8]) {
  float a[4], b[4];
  load4<T>(p, a);
  load4<T>(p + 4, b);
#pragma unroll
  for (int e = 0; e < 4; e++) { v[e] = a[e]; v[4 + e] = b[e]; }
}
template <> PE_DEV void ld8<bf16>(const bf16* p, float (&v)[8]) {
  bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int e = 0; e < 8; e++) v[e] = (float)t[e];
}
// the same for data that is read once (the inputs of the reductions over splits and over the batch axis):
// non-temporal, the lines are not kept in L2 for a second reader that never comes
template <typename T> PE_DEV void ld8_once(const T* p, float (&v)[8]) { ld8<T>(p, v); }
template <> PE_DEV void ld8_once<bf16>(const bf16* p, float (&v)[8]) {
  bf16x8 t = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p));
#pragma unroll
  for (int e = 0; e < 8; e++) v[e] = (float)t[e];
}
PE_DEV f32x4 ld4f_once(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p)); }
template <typename T> PE_DEV void st8(T* p, const float (&v)[8]) {
  float a[4] = {v[0], v[1], v[2], v[3]}, b[4] = {v[4], v[5], v[6], v[7]};
  store4<T>(p, a);
  store4<T>(p + 4, b);
}
template <> PE_DEV void st8<bf16>(bf16* p, const float (&v)[8]) {
  bf16x8 t;
#pragma unroll
  for (int e = 0; e < 8; e++) t[e] = (bf16)v[e];
  *reinterpret_cast<bf16x8*>(p) = t;
}
template <int LPR> PE_DEV float group_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T, int LPR>
__global__ __launch_bounds__(256) void ln_fwd_fast_kernel(const T* x, const float* gamma, const float* beta, T* y,
                                                          float* stats, long long M, float eps) {
  constexpr int C = 8 * LPR, RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rw = lane / LPR, c0 = sub * 8;
  float gm[8], bt[8];
#pragma unroll
  for (int e = 0; e < 8; e++) { gm[e] = gamma[c0 + e]; bt[e] = beta[c0 + e]; }
  // two row groups per wave and iteration (rows r and r + RPW): both loads are issued before the first
  // reduction starts, which doubles the bytes a wave has in flight
  const long long stride = (long long)gridDim.x * 8 * RPW;
  for (long long row = ((long long)blockIdx.x * 4 + wave) * 2 * RPW + rw; row < M + rw; row += stride) {
    // row - rw < M for the whole wave: shuffles stay convergent
    long long rr[2] = {row, row + RPW};
    bool ok[2];
    float v[2][8];
#pragma unroll
    for (int u = 0; u < 2; u++) {
      ok[u] = rr[u] < M;
      if (ok[u]) ld8<T>(x + rr[u] * C + c0, v[u]);
      else {
#pragma unroll
        for (int e = 0; e < 8; e++) v[u][e] = 0.0f;
      }
    }
#pragma unroll
    for (int u = 0; u < 2; u++) {
      float s = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; e++) s += v[u][e];
      float mu = group_sum<LPR>(s) * (1.0f / C);
      float q = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; e++) { float t = v[u][e] - mu; q += t * t; }
      float rstd = rsqrtf(group_sum<LPR>(q) * (1.0f / C) + eps);
      if (ok[u]) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (v[u][e] - mu) * rstd * gm[e] + bt[e];
        st8<T>(y + rr[u] * C + c0, o);
        if (sub == 0) { stats[rr[u] * 2] = mu; stats[rr[u] * 2 + 1] = rstd; }
      }
    }
  }
}

template <typename T, int LPR>
__global__ __launch_bounds__(256) void ln_bwd_fast_kernel(const T* dy, const T* x, const float* stats, const float* gamma,
                                                          const T* gin, T* gout, float* partial, long long M) {
  constexpr int C = 8 * LPR, RPW = 64 / LPR;
  __shared__ float red[4][2 * C];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rw = lane / LPR, c0 = sub * 8;
  float gm[8], dgs[8], dbs[8];
#pragma unroll
  for (int e = 0; e < 8; e++) { gm[e] = gamma[c0 + e]; dgs[e] = 0.0f; dbs[e] = 0.0f; }
  const long long stride = (long long)gridDim.x * 4 * RPW;
  for (long long row = ((long long)blockIdx.x * 4 + wave) * RPW + rw; row < M + rw; row += stride) {
    const bool ok = row < M;
    float xv[8], dv[8], xh[8], dxh[8];
    float mu = 0.0f, rstd = 0.0f;
    if (ok) {
      ld8<T>(x + row * C + c0, xv);
      ld8<T>(dy + row * C + c0, dv);
      mu = stats[row * 2];
      rstd = stats[row * 2 + 1];
    } else {
#pragma unroll
      for (int e = 0; e < 8; e++) { xv[e] = 0.0f; dv[e] = 0.0f; }
    }
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      xh[e] = (xv[e] - mu) * rstd;
      dxh[e] = dv[e] * gm[e];
      dgs[e] += dv[e] * xh[e];
      dbs[e] += dv[e];
      s1 += dxh[e];
      s2 += dxh[e] * xh[e];
    }
    s1 = group_sum<LPR>(s1) * (1.0f / C);
    s2 = group_sum<LPR>(s2) * (1.0f / C);
    if (ok) {
      float o[8];
      if (gin) ld8<T>(gin + row * C + c0, o);
      else {
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = 0.0f;
      }
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] += (dxh[e] - s1 - xh[e] * s2) * rstd;
      st8<T>(gout + row * C + c0, o);
    }
  }
  // rows of a wave hold the same channels in lanes sub, sub + LPR, ...: fold them, then fold the waves
#pragma unroll
  for (int e = 0; e < 8; e++) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) { dgs[e] += __shfl_xor(dgs[e], o, 64); dbs[e] += __shfl_xor(dbs[e], o, 64); }
  }
  if (rw == 0) {
#pragma unroll
    for (int e = 0; e < 8; e++) { red[wave][c0 + e] = dgs[e]; red[wave][C + c0 + e] = dbs[e]; }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < 2 * C; c += 256)
    partial[(long long)blockIdx.x * 2 * C + c] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
}

// ---------------------------------------------------------------------------
// LayerNorm over channels of a CHANNEL-MAJOR tensor x_t[C][M] (triangle-multiplication
// contraction output), producing channel-last y[M][C].  A workgroup handles 64
// consecutive positions: thread (p = tid%64, part = tid/64) walks channels part, part+4, ..
// (coalesced along positions), tile transposed through LDS for the channel-last store.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ln_cmajor_fwd_kernel(const T* xt, const float* gamma, const float* beta, T* y,
                                                            float* stats, long long M, int C, float eps) {
  extern __shared__ float tile[];   // [64][C+1]
  __shared__ float rs[4][64], rq[4][64];
  const int p = threadIdx.x & 63, part = threadIdx.x >> 6;
  const long long m0 = (long long)blockIdx.x * 64;
  const long long m = m0 + p;
  float s = 0.0f;
  for (int c = part; c < C; c += 4) {
    float v = (m < M) ? to_f(xt[(long long)c * M + m]) : 0.0f;
    tile[p * (C + 1) + c] = v;
    s += v;
  }
  rs[part][p] = s;
  __syncthreads();
  float mu = (rs[0][p] + rs[1][p] + rs[2][p] + rs[3][p]) / C;
  float q = 0.0f;
  for (int c = part; c < C; c += 4) { float t = tile[p * (C + 1) + c] - mu; q += t * t; }
  rq[part][p] = q;
  __syncthreads();
  float rstd = rsqrtf((rq[0][p] + rq[1][p] + rq[2][p] + rq[3][p]) / C + eps);
  if (part == 0 && m < M) { stats[m * 2] = mu; stats[m * 2 + 1] = rstd; }
  // channel-last store: thread t handles channel c = t % C.. for rows
  for (int idx = threadIdx.x; idx < 64 * C; idx += 256) {
    int pp = idx / C, c = idx % C;
    long long mm = m0 + pp;
    if (mm < M) {
      float mu2 = (rs[0][pp] + rs[1][pp] + rs[2][pp] + rs[3][pp]) / C;
      float rstd2 = rsqrtf((rq[0][pp] + rq[1][pp] + rq[2][pp] + rq[3][pp]) / C + eps);
      y[mm * C + c] = from_f<T>((tile[pp * (C + 1) + c] - mu2) * rstd2 * gamma[c] + beta[c]);
    }
  }
}

// backward: dy[M][C] channel-last, x_t[C][M] channel-major, -> dx_t[C][M]; partial[wg][2C]
template <typename T>
__global__ __launch_bounds__(256) void ln_cmajor_bwd_kernel(const T* dy, const T* xt, const float* stats,
                                                            const float* gamma, T* dxt, float* partial, long long M,
                                                            int C) {
  extern __shared__ float tile[];   // dy tile [64][C+1]
  __shared__ float r1[4][64], r2[4][64];
  const int p = threadIdx.x & 63, part = threadIdx.x >> 6;
  const long long m0 = (long long)blockIdx.x * 64;
  const long long m = m0 + p;
  for (int idx = threadIdx.x; idx < 64 * C; idx += 256) {
    int pp = idx / C, c = idx % C;
    long long mm = m0 + pp;
    tile[pp * (C + 1) + c] = (mm < M) ? to_f(dy[mm * C + c]) : 0.0f;
  }
  __syncthreads();
  float mu = (m < M) ? stats[m * 2] : 0.0f, rstd = (m < M) ? stats[m * 2 + 1] : 0.0f;
  float s1 = 0.0f, s2 = 0.0f;
  for (int c = part; c < C; c += 4) {
    float xh = (m < M) ? (to_f(xt[(long long)c * M + m]) - mu) * rstd : 0.0f;
    float dxh = tile[p * (C + 1) + c] * gamma[c];
    s1 += dxh;
    s2 += dxh * xh;
  }
  r1[part][p] = s1;
  r2[part][p] = s2;
  __syncthreads();
  s1 = (r1[0][p] + r1[1][p] + r1[2][p] + r1[3][p]) / C;
  s2 = (r2[0][p] + r2[1][p] + r2[2][p] + r2[3][p]) / C;
  for (int c = part; c < C; c += 4) {
    float xh = (m < M) ? (to_f(xt[(long long)c * M + m]) - mu) * rstd : 0.0f;
    float dv = tile[p * (C + 1) + c];
    float dxh = dv * gamma[c];
    if (m < M) dxt[(long long)c * M + m] = from_f<T>((dxh - s1 - xh * s2) * rstd);
    // per-channel partials over the 64 positions: wave reduction (a wave = one `part`)
    float a = wave_sum(dv * xh), b = wave_sum(dv);
    if (p == 0) {
      partial[(long long)blockIdx.x * 2 * C + c] = a;
      partial[(long long)blockIdx.x * 2 * C + C + c] = b;
    }
  }
}

// Fast forms for M % 4 == 0 and C % 8 == 0: thread (pl = tid%16, cl = tid/16) moves 4
// consecutive positions of channel cl, cl+16, .. per load (8 / 16 bytes per lane, 128 / 256
// bytes per 16 lanes); the channel-last side moves 8 channels per lane.
// NIT = ceil(C / 16), the number of channels a thread walks, as a compile-time constant: the loops
// are unrolled, all of a thread's loads are issued before the first use (a loop with a run-time
// trip count waits for memory once per channel) and the backward pass keeps x in registers.
template <typename T, int NIT>
__global__ __launch_bounds__(256) void ln_cmajor_fwd_fast_kernel(const T* xt, const float* gamma, const float* beta,
                                                                 T* y, float* stats, long long M, int C, float eps) {
  extern __shared__ float tile[];   // [64][C+1]
  __shared__ float rs[16][65], smu[64], srstd[64];
  const int pl = threadIdx.x & 15, cl = threadIdx.x >> 4, ld = C + 1;
  const long long m0 = (long long)blockIdx.x * 64, mb = m0 + 4 * pl;
  const bool ok = mb < M;
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  float xv[NIT][4];
#pragma unroll
  for (int it = 0; it < NIT; it++) {
    const int c = cl + 16 * it;
#pragma unroll
    for (int k = 0; k < 4; k++) xv[it][k] = 0.0f;
    if (ok && c < C) load4<T>(xt + (long long)c * M + mb, xv[it]);
  }
#pragma unroll
  for (int it = 0; it < NIT; it++) {
    const int c = cl + 16 * it;
    if (c < C) {
#pragma unroll
      for (int k = 0; k < 4; k++) { tile[(4 * pl + k) * ld + c] = xv[it][k]; s[k] += xv[it][k]; }
    }
  }
#pragma unroll
  for (int k = 0; k < 4; k++) rs[cl][4 * pl + k] = s[k];
  __syncthreads();
  if (threadIdx.x < 64) {
    float t = 0.0f;
#pragma unroll
    for (int k = 0; k < 16; k++) t += rs[k][threadIdx.x];
    smu[threadIdx.x] = t / C;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; k++) s[k] = 0.0f;
#pragma unroll
  for (int it = 0; it < NIT; it++) {
    const int c = cl + 16 * it;
    if (c < C) {
#pragma unroll
      for (int k = 0; k < 4; k++) { float t = xv[it][k] - smu[4 * pl + k]; s[k] += t * t; }
    }
  }
#pragma unroll
  for (int k = 0; k < 4; k++) rs[cl][4 * pl + k] = s[k];
  __syncthreads();
  if (threadIdx.x < 64) {
    float t = 0.0f;
#pragma unroll
    for (int k = 0; k < 16; k++) t += rs[k][threadIdx.x];
    float rstd = rsqrtf(t / C + eps);
    srstd[threadIdx.x] = rstd;
    long long m = m0 + threadIdx.x;
    if (m < M) { stats[m * 2] = smu[threadIdx.x]; stats[m * 2 + 1] = rstd; }
  }
  __syncthreads();
  const int C8 = C >> 3;
  for (int idx = threadIdx.x; idx < 64 * C8; idx += 256) {
    const int pp = idx / C8, c0 = (idx - pp * C8) * 8;
    const long long mm = m0 + pp;
    if (mm < M) {
      const float mu = smu[pp], rstd = srstd[pp];
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = (tile[pp * ld + c0 + e] - mu) * rstd * gamma[c0 + e] + beta[c0 + e];
      st8<T>(y + mm * C + c0, o);
    }
  }
}

template <typename T, int NIT>
__global__ __launch_bounds__(256) void ln_cmajor_bwd_fast_kernel(const T* dy, const T* xt, const float* stats,
                                                                 const float* gamma, T* dxt, float* partial,
                                                                 long long M, int C) {
  extern __shared__ float tile[];   // dy tile [64][C+1]
  __shared__ float r1[16][65], r2[16][65], t1[64], t2[64];
  const int pl = threadIdx.x & 15, cl = threadIdx.x >> 4, ld = C + 1;
  const long long m0 = (long long)blockIdx.x * 64, mb = m0 + 4 * pl;
  const bool ok = mb < M;
  const int C8 = C >> 3;
  // x of this thread's channels (kept for both passes) and the LayerNorm statistics
  float xv[NIT][4], gv[NIT];
#pragma unroll
  for (int it = 0; it < NIT; it++) {
    const int c = cl + 16 * it;
#pragma unroll
    for (int k = 0; k < 4; k++) xv[it][k] = 0.0f;
    if (ok && c < C) load4<T>(xt + (long long)c * M + mb, xv[it]);
    gv[it] = c < C ? gamma[c] : 0.0f;
  }
  float mu[4], rstd[4];
#pragma unroll
  for (int k = 0; k < 4; k++) {
    mu[k] = ok ? stats[(mb + k) * 2] : 0.0f;
    rstd[k] = ok ? stats[(mb + k) * 2 + 1] : 0.0f;
  }
  for (int idx = threadIdx.x; idx < 64 * C8; idx += 256) {
    const int pp = idx / C8, c0 = (idx - pp * C8) * 8;
    const long long mm = m0 + pp;
    float v[8];
    if (mm < M) ld8<T>(dy + mm * C + c0, v);
    else {
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] = 0.0f;
    }
#pragma unroll
    for (int e = 0; e < 8; e++) tile[pp * ld + c0 + e] = v[e];
  }
  __syncthreads();
  float s1[4] = {0.0f, 0.0f, 0.0f, 0.0f}, s2[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  float dv[NIT][4];
#pragma unroll
  for (int it = 0; it < NIT; it++) {
    const int c = cl + 16 * it;
#pragma unroll
    for (int k = 0; k < 4; k++) {
      xv[it][k] = (xv[it][k] - mu[k]) * rstd[k];          // x-hat from here on
      dv[it][k] = c < C ? tile[(4 * pl + k) * ld + c] : 0.0f;
      float dxh = dv[it][k] * gv[it];
      s1[k] += dxh;
      s2[k] += dxh * xv[it][k];
    }
  }
#pragma unroll
  for (int k = 0; k < 4; k++) { r1[cl][4 * pl + k] = s1[k]; r2[cl][4 * pl + k] = s2[k]; }
  __syncthreads();
  if (threadIdx.x < 64) {
    float a = 0.0f, b = 0.0f;
#pragma unroll
    for (int k = 0; k < 16; k++) { a += r1[k][threadIdx.x]; b += r2[k][threadIdx.x]; }
    t1[threadIdx.x] = a / C;
    t2[threadIdx.x] = b / C;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; k++) { s1[k] = t1[4 * pl + k]; s2[k] = t2[4 * pl + k]; }
#pragma unroll
  for (int it = 0; it < NIT; it++) {
    const int c = cl + 16 * it;
    float o[4], a = 0.0f, b = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; k++) {
      o[k] = (dv[it][k] * gv[it] - s1[k] - xv[it][k] * s2[k]) * rstd[k];
      a += dv[it][k] * xv[it][k];
      b += dv[it][k];
    }
    if (ok && c < C) store4<T>(dxt + (long long)c * M + mb, o);
    // per-channel partials over the 64 positions: the 16 lanes sharing cl
    a = group_sum<16>(a);
    b = group_sum<16>(b);
    if (pl == 0 && c < C) {
      partial[(long long)blockIdx.x * 2 * C + c] = a;
      partial[(long long)blockIdx.x * 2 * C + C + c] = b;
    }
  }
}

// ---------------------------------------------------------------------------
// Channel-major LayerNorm, bf16, C = 8 * LPR channels (64 or 128): the variants that move 256-byte runs.
// A workgroup handles 128 consecutive positions.  The channel-major side is read / written in 16-byte vectors of 8
// positions (16 lanes cover one channel's 256-byte run; the 64-position kernels above move 128-byte runs and reach
// 1.6 - 2.5 TB/s) and transposed through an LDS tile [position][channel] whose 8-channel groups are XOR-swizzled
// with (position / 8): the scalar transposing accesses of a wave and the 16-byte row accesses are both free of
// bank conflicts.  Per position the arithmetic is that of the channel-last kernels (LPR lanes per position, 8
// channels each).  All loads of a workgroup are issued before the first wait.  Needs M % 8 == 0.
// ---------------------------------------------------------------------------
template <int LPR> struct LnCmT {
  static constexpr int C = 8 * LPR, PT = 128, PV = PT / 8, NV = C * PV / 256, RPI = 256 / LPR, NIT = PT / RPI;
  // element offset of (position p, channel c) in the tile
  static PE_DEV int off(int p, int c) { return p * C + ((((c >> 3) ^ (p >> 3)) & (LPR - 1)) << 3) + (c & 7); }
};
template <int LPR>
PE_DEV void lncm_load_tile(const bf16* xt, long long M, long long m0, bf16x8 (&xr)[LnCmT<LPR>::NV]) {
  typedef LnCmT<LPR> K;
#pragma unroll
  for (int i = 0; i < K::NV; i++) {
    const int idx = threadIdx.x + 256 * i, pv = idx % K::PV, ch = idx / K::PV;
    const long long pos = m0 + 8 * pv;
    bf16x8 v;
#pragma unroll
    for (int k = 0; k < 8; k++) v[k] = (bf16)0.0f;
    if (pos < M) v = *reinterpret_cast<const bf16x8*>(xt + (long long)ch * M + pos);
    xr[i] = v;
  }
}
template <int LPR>
PE_DEV void lncm_store_tile(const bf16x8 (&xr)[LnCmT<LPR>::NV], bf16* tile) {
  typedef LnCmT<LPR> K;
#pragma unroll
  for (int i = 0; i < K::NV; i++) {
    const int idx = threadIdx.x + 256 * i, pv = idx % K::PV, ch = idx / K::PV;
#pragma unroll
    for (int k = 0; k < 8; k++) tile[K::off(8 * pv + k, ch)] = xr[i][k];
  }
}

template <int LPR>
__global__ __launch_bounds__(256) void ln_cmajor_fwd_t_kernel(const bf16* xt, const float* gamma, const float* beta,
                                                              bf16* y, float* stats, long long M, float eps) {
  typedef LnCmT<LPR> K;
  constexpr int C = K::C;
  __shared__ __attribute__((aligned(16))) bf16 tile[K::PT * C];
  const long long m0 = (long long)blockIdx.x * K::PT;
  const int sub = threadIdx.x % LPR, rr = threadIdx.x / LPR, c0 = sub * 8;
  bf16x8 xr[K::NV];
  lncm_load_tile<LPR>(xt, M, m0, xr);
  float gm[8], bt[8];
#pragma unroll
  for (int e = 0; e < 8; e++) { gm[e] = gamma[c0 + e]; bt[e] = beta[c0 + e]; }
  lncm_store_tile<LPR>(xr, tile);
  __syncthreads();
#pragma unroll
  for (int it = 0; it < K::NIT; it++) {
    const int p = it * K::RPI + rr;
    const long long row = m0 + p;
    const bf16x8 xb = *reinterpret_cast<const bf16x8*>(tile + K::off(p, c0));
    float xv[8], s = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; e++) { xv[e] = (float)xb[e]; s += xv[e]; }
    const float mu = group_sum<LPR>(s) * (1.0f / C);
    float q = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; e++) { const float t = xv[e] - mu; q += t * t; }
    const float rstd = rsqrtf(group_sum<LPR>(q) * (1.0f / C) + eps);
    if (row < M) {
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = (xv[e] - mu) * rstd * gm[e] + bt[e];
      st8<bf16>(y + row * C + c0, o);
      if (sub == 0) { stats[row * 2] = mu; stats[row * 2 + 1] = rstd; }
    }
  }
}

template <int LPR>
__global__ __launch_bounds__(256) void ln_cmajor_bwd_t_kernel(const bf16* dy, const bf16* xt, const float* stats,
                                                              const float* gamma, bf16* dxt, float* partial, long long M) {
  typedef LnCmT<LPR> K;
  constexpr int C = K::C;
  __shared__ __attribute__((aligned(16))) bf16 tile[K::PT * C];
  __shared__ float red[4][2 * C];
  const long long m0 = (long long)blockIdx.x * K::PT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = threadIdx.x % LPR, rr = threadIdx.x / LPR, c0 = sub * 8;
  bf16x8 xr[K::NV];
  lncm_load_tile<LPR>(xt, M, m0, xr);
  // cotangent rows and statistics of this thread's positions: requested before the tile is waited for
  bf16x8 dyr[K::NIT];
  float mu[K::NIT], rstd[K::NIT];
#pragma unroll
  for (int it = 0; it < K::NIT; it++) {
    const long long row = m0 + it * K::RPI + rr;
    const bool ok = row < M;
#pragma unroll
    for (int k = 0; k < 8; k++) dyr[it][k] = (bf16)0.0f;
    if (ok) dyr[it] = *reinterpret_cast<const bf16x8*>(dy + row * C + c0);
    mu[it] = ok ? stats[row * 2] : 0.0f;
    rstd[it] = ok ? stats[row * 2 + 1] : 0.0f;
  }
  float gm[8], dgs[8], dbs[8];
#pragma unroll
  for (int e = 0; e < 8; e++) { gm[e] = gamma[c0 + e]; dgs[e] = 0.0f; dbs[e] = 0.0f; }
  lncm_store_tile<LPR>(xr, tile);
  __syncthreads();
#pragma unroll
  for (int it = 0; it < K::NIT; it++) {
    const int p = it * K::RPI + rr;
    bf16* slot = tile + K::off(p, c0);
    const bf16x8 xb = *reinterpret_cast<const bf16x8*>(slot);
    float xh[8], dxh[8], s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const float dv = (float)dyr[it][e];
      xh[e] = ((float)xb[e] - mu[it]) * rstd[it];
      dxh[e] = dv * gm[e];
      dgs[e] += dv * xh[e];
      dbs[e] += dv;
      s1 += dxh[e];
      s2 += dxh[e] * xh[e];
    }
    s1 = group_sum<LPR>(s1) * (1.0f / C);
    s2 = group_sum<LPR>(s2) * (1.0f / C);
    bf16x8 ob;
#pragma unroll
    for (int e = 0; e < 8; e++) ob[e] = (bf16)((dxh[e] - s1 - xh[e] * s2) * rstd[it]);
    *reinterpret_cast<bf16x8*>(slot) = ob;     // the slot belongs to this thread alone
  }
  __syncthreads();
  // transposed copy out: 8 positions of one channel per 16-byte store
#pragma unroll
  for (int i = 0; i < K::NV; i++) {
    const int idx = threadIdx.x + 256 * i, pv = idx % K::PV, ch = idx / K::PV;
    const long long pos = m0 + 8 * pv;
    bf16x8 v;
#pragma unroll
    for (int k = 0; k < 8; k++) v[k] = tile[K::off(8 * pv + k, ch)];
    if (pos < M) *reinterpret_cast<bf16x8*>(dxt + (long long)ch * M + pos) = v;
  }
  // gain / offset partials of the workgroup: positions of a wave hold the same channels in lanes sub, sub + LPR, ...
#pragma unroll
  for (int e = 0; e < 8; e++) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) { dgs[e] += __shfl_xor(dgs[e], o, 64); dbs[e] += __shfl_xor(dbs[e], o, 64); }
  }
  if (lane < LPR) {
#pragma unroll
    for (int e = 0; e < 8; e++) { red[wave][c0 + e] = dgs[e]; red[wave][C + c0 + e] = dbs[e]; }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < 2 * C; c += 256)
    partial[(long long)blockIdx.x * 2 * C + c] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
}

// ---------------------------------------------------------------------------
// Pair-bias projection fused with its LayerNorm: bias[h][i][j] = (LN(z_ij) W)_h
// (transposed: bias[h][j][i]); biasT holds the other orientation multiplied by log2(e),
// the form the base-2 softmax of the query-per-lane attention kernels reads.  C <= 256 (one 4-channel chunk per lane).
// ---------------------------------------------------------------------------
constexpr int BIAS_MAXH = 8;
template <typename T>
__global__ __launch_bounds__(256) void ln_bias_fwd_kernel(const T* z, const float* gamma, const float* beta,
                                                          const float* w /*[C][H]*/, float* bias, float* biasT,
                                                          float* stats, int r, int C, int H, float eps, int transposed) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane * 4;
  float gm[4], bt[4], wv[4][BIAS_MAXH];
#pragma unroll
  for (int e = 0; e < 4; e++) {
    gm[e] = (c < C) ? gamma[c + e] : 0.0f;
    bt[e] = (c < C) ? beta[c + e] : 0.0f;
#pragma unroll
    for (int h = 0; h < BIAS_MAXH; h++) wv[e][h] = (c < C && h < H) ? w[(c + e) * H + h] : 0.0f;
  }
  const long long M = (long long)r * r;
  for (long long row = (long long)blockIdx.x * 4 + wave; row < M; row += (long long)gridDim.x * 4) {
    float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (c < C) load4<T>(z + row * C + c, v);
    float mu = wave_sum(v[0] + v[1] + v[2] + v[3]) / C;
    float q = 0.0f;
    if (c < C) {
#pragma unroll
      for (int e = 0; e < 4; e++) { float t = v[e] - mu; q += t * t; }
    }
    float rstd = rsqrtf(wave_sum(q) / C + eps);
    float y[4];
#pragma unroll
    for (int e = 0; e < 4; e++) y[e] = (c < C) ? (v[e] - mu) * rstd * gm[e] + bt[e] : 0.0f;
    int i = row / r, j = row % r;
    long long o = transposed ? ((long long)j * r + i) : row;
    long long oT = transposed ? row : ((long long)j * r + i);
#pragma unroll
    for (int h = 0; h < BIAS_MAXH; h++) {
      if (h < H) {
        float t = y[0] * wv[0][h] + y[1] * wv[1][h] + y[2] * wv[2][h] + y[3] * wv[3][h];
        t = wave_sum(t);
        if (lane == 0) { bias[(long long)h * M + o] = t; biasT[(long long)h * M + oT] = t * 1.4426950408889634f; }
      }
    }
    if (lane == 0) { stats[row * 2] = mu; stats[row * 2 + 1] = rstd; }
  }
}

// backward: dy_c = sum_h dbias[h][row] W[c][h]; LayerNorm backward -> gout = gin + dz;
// partial[wg] = [ dgamma (C) | dbeta (C) | dW (C*H) ]
template <typename T>
__global__ __launch_bounds__(256) void ln_bias_bwd_kernel(const float* dbias, const T* z, const float* stats,
                                                          const float* gamma, const float* beta, const float* w,
                                                          const T* gin, T* gout, float* partial, int r, int C, int H,
                                                          int transposed) {
  __shared__ float red[4][256 * (2 + BIAS_MAXH)];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane * 4;
  float gm[4], bt[4], wv[4][BIAS_MAXH], dgs[4], dbs[4], dws[4][BIAS_MAXH];
#pragma unroll
  for (int e = 0; e < 4; e++) {
    gm[e] = (c < C) ? gamma[c + e] : 0.0f;
    bt[e] = (c < C) ? beta[c + e] : 0.0f;
    dgs[e] = 0.0f; dbs[e] = 0.0f;
#pragma unroll
    for (int h = 0; h < BIAS_MAXH; h++) { wv[e][h] = (c < C && h < H) ? w[(c + e) * H + h] : 0.0f; dws[e][h] = 0.0f; }
  }
  const long long M = (long long)r * r;
  for (long long row = (long long)blockIdx.x * 4 + wave; row < M; row += (long long)gridDim.x * 4) {
    float mu = stats[row * 2], rstd = stats[row * 2 + 1];
    int i = row / r, j = row % r;
    long long o = transposed ? ((long long)j * r + i) : row;
    float db[BIAS_MAXH];
#pragma unroll
    for (int h = 0; h < BIAS_MAXH; h++) db[h] = (h < H) ? dbias[(long long)h * M + o] : 0.0f;
    float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (c < C) load4<T>(z + row * C + c, v);
    float xh[4], dxh[4];
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; e++) {
      xh[e] = (c < C) ? (v[e] - mu) * rstd : 0.0f;
      float y = xh[e] * gm[e] + bt[e];
      float dy = 0.0f;
#pragma unroll
      for (int h = 0; h < BIAS_MAXH; h++) { dy += db[h] * wv[e][h]; dws[e][h] += y * db[h]; }
      dxh[e] = dy * gm[e];
      dgs[e] += dy * xh[e];
      dbs[e] += dy;
      s1 += dxh[e];
      s2 += dxh[e] * xh[e];
    }
    s1 = wave_sum(s1) / C;
    s2 = wave_sum(s2) / C;
    if (c < C) {
      float ov[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (gin) load4<T>(gin + row * C + c, ov);
#pragma unroll
      for (int e = 0; e < 4; e++) ov[e] += (dxh[e] - s1 - xh[e] * s2) * rstd;
      store4<T>(gout + row * C + c, ov);
    }
  }
#pragma unroll
  for (int e = 0; e < 4; e++) {
    red[wave][c + e] = dgs[e];
    red[wave][256 + c + e] = dbs[e];
#pragma unroll
    for (int h = 0; h < BIAS_MAXH; h++) red[wave][512 + (c + e) * BIAS_MAXH + h] = dws[e][h];
  }
  __syncthreads();
  float* pp = partial + (long long)blockIdx.x * (2 * C + C * H);
  for (int t = threadIdx.x; t < C; t += 256) {
    pp[t] = red[0][t] + red[1][t] + red[2][t] + red[3][t];
    pp[C + t] = red[0][256 + t] + red[1][256 + t] + red[2][256 + t] + red[3][256 + t];
  }
  for (int t = threadIdx.x; t < C * H; t += 256) {
    int cc = t / H, h = t % H;
    int k = 512 + cc * BIAS_MAXH + h;
    pp[2 * C + t] = red[0][k] + red[1][k] + red[2][k] + red[3][k];
  }
}

// Fast variants for C = 8 * LPR (LPR <= 32): 64 / LPR rows per wave, 8 channels per lane.
// w (and the per-lane slices of it) go through LDS: sw[sub] holds the 8 x HH weights of lane
// group `sub`, rows padded by 4 floats so that the 16-byte reads of neighbouring lanes hit
// different banks.  HH = 4 or 8 is the compile-time head count (H <= HH).
template <int LPR, int HH>
PE_DEV void bias_stage_w(const float* w, int H, float (*sw)[8 * HH + 4], int sub, float (&wv)[8][HH]) {
  for (int idx = threadIdx.x; idx < 8 * LPR * HH; idx += 256) {
    const int c = idx / HH, h = idx % HH;
    sw[c >> 3][(c & 7) * HH + h] = (h < H) ? w[c * H + h] : 0.0f;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 8; e++)
#pragma unroll
    for (int h = 0; h < HH; h++) wv[e][h] = sw[sub][e * HH + h];
}

constexpr int LNB_UN = 4;   // rows per lane group and step (the 16-byte stores below assume 4)
template <typename T, int LPR, int HH>
__global__ __launch_bounds__(256) void ln_bias_fwd_fast_kernel(const T* z, const float* gamma, const float* beta,
                                                               const float* w, float* direct, float direct_scale,
                                                               float* stats, int r, int H, float eps) {
  // writes direct[h][row] = (LN(z_row) W)_h * direct_scale in row order (coalesced); the other
  // orientation is produced by bias_transpose_kernel
  constexpr int C = 8 * LPR, RPW = 64 / LPR;
  __shared__ float sw[LPR][8 * HH + 4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rw = lane / LPR, c0 = sub * 8;
  float gm[8], bt[8], wv[8][HH];
#pragma unroll
  for (int e = 0; e < 8; e++) { gm[e] = gamma[c0 + e]; bt[e] = beta[c0 + e]; }
  bias_stage_w<LPR, HH>(w, H, sw, sub, wv);
  const long long M = (long long)r * r;
  // A lane group handles LNB_UN = 4 CONSECUTIVE rows per step (loads of all four issued before the first is used), so
  // that its lane 0 writes the four rows' value of a head with one 16-byte store and their statistics with two: with
  // one row per step the outputs left as 4-byte stores, one per row and head, and those bounded the kernel.
  const long long wg_rows = 4LL * RPW * LNB_UN, stride = (long long)gridDim.x * wg_rows;
  for (long long base = (long long)blockIdx.x * wg_rows + (wave * RPW + rw) * LNB_UN; base < M + (wave * RPW + rw) * LNB_UN; base += stride) {
    typename Vec16<T>::type raw[LNB_UN][sizeof(T) == 2 ? 1 : 2];
#pragma unroll
    for (int u = 0; u < LNB_UN; u++) {
      const long long row = base + u;
      const T* src = z + (row < M ? row : 0) * C + c0;
#pragma unroll
      for (int q = 0; q < (sizeof(T) == 2 ? 1 : 2); q++) raw[u][q] = *reinterpret_cast<const typename Vec16<T>::type*>(src + q * Vec16<T>::N);
    }
    float outv[HH][LNB_UN], st[2 * LNB_UN];
#pragma unroll
    for (int u = 0; u < LNB_UN; u++) {
      const bool ok = base + u < M;
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] = ok ? to_f<T>(raw[u][e / Vec16<T>::N][e % Vec16<T>::N]) : 0.0f;
      float s = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; e++) s += v[e];
      float mu = group_sum<LPR>(s) * (1.0f / C);
      float q = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; e++) { float t = v[e] - mu; q += t * t; }
      float rstd = rsqrtf(group_sum<LPR>(q) * (1.0f / C) + eps);
      float y[8];
#pragma unroll
      for (int e = 0; e < 8; e++) y[e] = (v[e] - mu) * rstd * gm[e] + bt[e];
#pragma unroll
      for (int h = 0; h < HH; h++) {
        float t = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; e++) t += y[e] * wv[e][h];
        outv[h][u] = group_sum<LPR>(t) * direct_scale;
      }
      st[2 * u] = mu; st[2 * u + 1] = rstd;
    }
    if (sub == 0 && base < M) {
      if (base + LNB_UN <= M && (M & 3) == 0) {      // rows base .. base+3 exist and the stores are 16-byte aligned
#pragma unroll
        for (int h = 0; h < HH; h++)
          if (h < H) store4<float>(direct + (long long)h * M + base, outv[h]);
        float s0[4] = {st[0], st[1], st[2], st[3]}, s1[4] = {st[4], st[5], st[6], st[7]};
        store4<float>(stats + base * 2, s0);
        store4<float>(stats + base * 2 + 4, s1);
      } else {
#pragma unroll
        for (int u = 0; u < LNB_UN; u++)
          if (base + u < M) {
#pragma unroll
            for (int h = 0; h < HH; h++)
              if (h < H) direct[(long long)h * M + base + u] = outv[h][u];
            stats[(base + u) * 2] = st[2 * u]; stats[(base + u) * 2 + 1] = st[2 * u + 1];
          }
      }
    }
  }
}

// Copies of the pair bias for the attention kernels, in the storage type and in "lane chunk" order.
// direct[h][.][.] (r x r per head, fp32) holds value(query q, key k) at [q][k] (transposed == 0) or at [k][q]
// (transposed == 1).  Lane (position p, g) of a 32 x 32 score tile holds the 16 elements whose other-axis
// offsets are acc_row(g, e) = 8 (e / 4) + 4 g + e % 4.  With CH = 16 bytes / sizeof(T) elements per chunk
// (4 fp32, 8 bf16) the copies are stored as
//   biasQ[h][key tile][chunk c][g][query][CH]   element i of chunk c: e = c CH + i   (kernels with a query per lane)
//   biasK[h][query tile][chunk c][g][key][CH]                                          (the kernel with a key per lane)
// both multiplied by f.  A lane then reads its 16 values with 16 / CH loads of 16 bytes, and the 32 lanes of a
// half wave read 512 contiguous bytes per load - instead of sixteen 4-byte loads with a row multiplication each
// (whose address arithmetic was about a sixth of the attention kernels' vector instructions) - and, in bf16, half
// the bytes: every workgroup of an attention kernel reads its whole 128 x L bias slab, 268 MB per launch in fp32
// at the row-attention shape, which is what the forward kernel was waiting for.  The tile axis is padded to a
// multiple of 32 positions with zeros (padded keys are masked, padded queries never stored).
// grid (NT, NT, H) with NT = ceil(r / 32): blockIdx.x = key tile, blockIdx.y = query tile.
template <typename T> struct BiasChunk { static constexpr int CH = 16 / sizeof(T), NC = 16 / CH; };
// offset (in elements) of chunk c of lane (position p of L, g) of tile t inside one head's plane
template <typename T> PE_DEV long long bias_chunk_off(int t, int c, int g, int p, int L) {
  return ((((long long)t * BiasChunk<T>::NC + c) * 2 + g) * L + p) * BiasChunk<T>::CH;
}
// position inside the 32-wide tile of the other axis that element i of chunk c of lane group g holds in the BIAS planes:
// bf16 planes are in MFMA B-operand order (the attention kernels add the tile as identity x bias), fp32 planes in
// accumulator order (added element by element).  dS planes are in accumulator order for both types.
template <typename T> PE_DEV int bias_slot(int c, int g, int i);
template <> PE_DEV int bias_slot<bf16>(int c, int g, int i) { return 16 * c + 8 * g + i; }
template <> PE_DEV int bias_slot<float>(int c, int g, int i) { return 8 * c + 4 * g + i; }
template <typename T>
__global__ __launch_bounds__(256) void bias_tile_kernel(const float* direct, T* biasQ, T* biasK, int r, int transposed, float f) {
  constexpr int CH = BiasChunk<T>::CH, NC = BiasChunk<T>::NC;
  __shared__ float tile[32][33];   // tile[query - q0][key - k0]
  const int h = blockIdx.z, q0 = blockIdx.y * 32, k0 = blockIdx.x * 32, NT = gridDim.x;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const long long base = (long long)h * r * r, plane = (long long)NT * 32 * r;
  for (int a = ty; a < 32; a += 8) {   // coalesced along the fast axis of the direct plane
    if (!transposed) {
      const int q = q0 + a, k = k0 + tx;
      tile[a][tx] = (q < r && k < r) ? direct[base + (long long)q * r + k] * f : 0.0f;
    } else {
      const int k = k0 + a, q = q0 + tx;
      tile[tx][a] = (q < r && k < r) ? direct[base + (long long)k * r + q] * f : 0.0f;
    }
  }
  __syncthreads();
  // thread (tx, ty): position tx of the lane axis; (c, g) = the ty-th chunk
  if (ty < 2 * NC) {
    const int c = ty >> 1, g = ty & 1;
    float vq[CH], vk[CH];
#pragma unroll
    for (int i = 0; i < CH; i++) {
      const int o = bias_slot<T>(c, g, i);
      vq[i] = tile[tx][o];
      vk[i] = tile[o][tx];
    }
    if (q0 + tx < r) {
      T* p = biasQ + h * plane + bias_chunk_off<T>(blockIdx.x, c, g, q0 + tx, r);
#pragma unroll
      for (int i = 0; i < CH; i++) p[i] = from_f<T>(vq[i]);
    }
    if (k0 + tx < r) {
      T* p = biasK + h * plane + bias_chunk_off<T>(blockIdx.y, c, g, k0 + tx, r);
#pragma unroll
      for (int i = 0; i < CH; i++) p[i] = from_f<T>(vk[i]);
    }
  }
}

// Bias gradient (fp32 sums in the query-per-lane chunk order of storage type T) back to pair-row order:
//   d bias(q, k) -> rows[h][q r + k]  (transposed == 0: the bias of (q, k) was read from pair position (q, k)) or
//   rows[h][k r + q] (transposed == 1).  Same grid as above.
template <typename T>
__global__ __launch_bounds__(256) void bias_untile_kernel(const float* tiled, float* rows, int r, int transposed) {
  constexpr int CH = BiasChunk<T>::CH, NC = BiasChunk<T>::NC;
  __shared__ float tile[32][33];   // tile[query - q0][key - k0]
  const int h = blockIdx.z, q0 = blockIdx.y * 32, k0 = blockIdx.x * 32, NT = gridDim.x;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const long long plane = (long long)NT * 32 * r;
  if (ty < 2 * NC) {
    const int c = ty >> 1, g = ty & 1;
    const float* p = tiled + h * plane + bias_chunk_off<T>(blockIdx.x, c, g, min(q0 + tx, r - 1), r);
#pragma unroll
    for (int i = 0; i < CH; i++) {
      const int e = c * CH + i, o = 8 * (e >> 2) + 4 * g + (e & 3);
      tile[tx][o] = (q0 + tx < r) ? p[i] : 0.0f;
    }
  }
  __syncthreads();
  const long long base = (long long)h * r * r;
  for (int a = ty; a < 32; a += 8) {
    if (!transposed) {
      const int q = q0 + a, k = k0 + tx;
      if (q < r && k < r) rows[base + (long long)q * r + k] = tile[a][tx];
    } else {
      const int k = k0 + a, q = q0 + tx;
      if (q < r && k < r) rows[base + (long long)k * r + q] = tile[tx][a];
    }
  }
}

template <typename T, int LPR, int HH>
__global__ __launch_bounds__(256) void ln_bias_bwd_fast_kernel(const float* dbias /*[H][M], pair-row order*/, const T* z,
                                                               const float* stats, const float* gamma,
                                                               const float* beta, const float* w, const T* gin, T* gout,
                                                               float* partial, int r, int H) {
  constexpr int C = 8 * LPR, RPW = 64 / LPR;
  __shared__ float red[4][C * (2 + HH)];
  __shared__ float sw[LPR][8 * HH + 4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPR, rw = lane / LPR, c0 = sub * 8;
  float gm[8], bt[8], wv[8][HH], dgs[8], dbs[8], dws[8][HH];
#pragma unroll
  for (int e = 0; e < 8; e++) {
    gm[e] = gamma[c0 + e];
    bt[e] = beta[c0 + e];
    dgs[e] = 0.0f; dbs[e] = 0.0f;
#pragma unroll
    for (int h = 0; h < HH; h++) dws[e][h] = 0.0f;
  }
  bias_stage_w<LPR, HH>(w, H, sw, sub, wv);
  const long long M = (long long)r * r;
  const long long stride = (long long)gridDim.x * 4 * RPW;
  for (long long row = ((long long)blockIdx.x * 4 + wave) * RPW + rw; row < M + rw; row += stride) {
    const bool ok = row < M;
    float db[HH];
#pragma unroll
    for (int h = 0; h < HH; h++) db[h] = (ok && h < H) ? dbias[(long long)h * M + row] : 0.0f;
    float v[8];
    float mu = 0.0f, rstd = 0.0f;
    if (ok) { ld8<T>(z + row * C + c0, v); mu = stats[row * 2]; rstd = stats[row * 2 + 1]; }
    else {
#pragma unroll
      for (int e = 0; e < 8; e++) v[e] = 0.0f;
    }
    float xh[8], dxh[8];
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      xh[e] = (v[e] - mu) * rstd;
      float y = xh[e] * gm[e] + bt[e];
      float dy = 0.0f;
#pragma unroll
      for (int h = 0; h < HH; h++) { dy += db[h] * wv[e][h]; dws[e][h] += y * db[h]; }
      dxh[e] = dy * gm[e];
      dgs[e] += dy * xh[e];
      dbs[e] += dy;
      s1 += dxh[e];
      s2 += dxh[e] * xh[e];
    }
    s1 = group_sum<LPR>(s1) * (1.0f / C);
    s2 = group_sum<LPR>(s2) * (1.0f / C);
    if (ok) {
      float ov[8];
      if (gin) ld8<T>(gin + row * C + c0, ov);
      else {
#pragma unroll
        for (int e = 0; e < 8; e++) ov[e] = 0.0f;
      }
#pragma unroll
      for (int e = 0; e < 8; e++) ov[e] += (dxh[e] - s1 - xh[e] * s2) * rstd;
      st8<T>(gout + row * C + c0, ov);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; e++) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      dgs[e] += __shfl_xor(dgs[e], o, 64);
      dbs[e] += __shfl_xor(dbs[e], o, 64);
#pragma unroll
      for (int h = 0; h < HH; h++) dws[e][h] += __shfl_xor(dws[e][h], o, 64);
    }
  }
  if (rw == 0) {
#pragma unroll
    for (int e = 0; e < 8; e++) {
      red[wave][c0 + e] = dgs[e];
      red[wave][C + c0 + e] = dbs[e];
#pragma unroll
      for (int h = 0; h < HH; h++) red[wave][2 * C + (c0 + e) * HH + h] = dws[e][h];
    }
  }
  __syncthreads();
  float* pp = partial + (long long)blockIdx.x * (2 * C + C * H);
  for (int t = threadIdx.x; t < 2 * C; t += 256) pp[t] = red[0][t] + red[1][t] + red[2][t] + red[3][t];
  for (int t = threadIdx.x; t < C * H; t += 256) {
    int k = 2 * C + (t / H) * HH + (t % H);
    pp[2 * C + t] = red[0][k] + red[1][k] + red[2][k] + red[3][k];
  }
}

// ---------------------------------------------------------------------------
// Reductions for parameter gradients
// ---------------------------------------------------------------------------
// dst[seg] += sum_s part[s][idx]; the [rows][cols] result is scattered by column segments
struct ReduceSeg { int n_begin, n_count; long long dst_off; int dst_ld; };
struct ReduceArgs {
  const float* part; int nsplit; long long stride;   // partial s at part + s*stride
  int rows, cols;
  int nseg; ReduceSeg seg[5];
  float* dst;
  int ylanes;
  int vec;   // 1 or 4 outputs per thread
};
// 256 threads = X outputs x Y split lanes (Y = a.ylanes in {1, 4, 16}, X = 256 / Y); fixed
// summation order (deterministic).  Up to REDUCE_BATCH independent reductions per launch
// (blockIdx.y selects one); their destinations must not overlap.
constexpr int REDUCE_BATCH = 16;   // 16 descriptors of 176 bytes: within the 4 KB of kernel arguments
// first[k] = first workgroup of reduction k (first[n] = grid size): every workgroup has work
struct ReduceBatch { ReduceArgs a[REDUCE_BATCH]; int first[REDUCE_BATCH + 1]; int n; };
__global__ __launch_bounds__(256) void reduce_partials_kernel(ReduceBatch rb) {
  __shared__ float red[256][4];
  int which = 0;
#pragma unroll
  for (int k = 1; k < REDUCE_BATCH; k++)
    if (k < rb.n && (int)blockIdx.x >= rb.first[k]) which = k;
  const ReduceArgs& a = rb.a[which];
  const int blk = blockIdx.x - rb.first[which];
  const int Y = a.ylanes, X = 256 / Y, V = a.vec;   // V = 4: every thread owns 4 consecutive outputs (16-byte loads)
  const long long total = (long long)a.rows * a.cols;
  if ((long long)blk * X * V >= total) return;
  const int x = threadIdx.x % X, y = threadIdx.x / X;
  const long long idx = ((long long)blk * X + x) * V;
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  // the lane that will write the result fetches the destination's current value first, so that this load is
  // in flight together with the partials instead of after the workgroup's barrier
  float* dst = nullptr;
  f32x4 cur = {0.0f, 0.0f, 0.0f, 0.0f};
  if (y == 0 && idx < total) {
    // a 4-group never straddles a row or a segment (the host checks the multiples of 4)
    const int m = idx / a.cols, n = idx % a.cols;
    for (int q = 0; q < a.nseg; q++) {
      const ReduceSeg& g = a.seg[q];
      if (n >= g.n_begin && n < g.n_begin + g.n_count) {
        dst = a.dst + g.dst_off + (long long)m * g.dst_ld + (n - g.n_begin);
        break;
      }
    }
    if (dst) {
      if (V == 4) cur = *reinterpret_cast<const f32x4*>(dst);   // host checked: 16-byte aligned destination groups
      else cur[0] = dst[0];
    }
  }
  if (idx < total) {
    // several independent loads in flight per thread; the sum order is a fixed function of (nsplit, Y, V)
    if (V == 4) {
      int k = y;
      for (; k + 4 * Y < a.nsplit; k += 8 * Y) {   // more than four splits left for this lane: eight loads in flight
        f32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
          int kk = k + u * Y;
          if (kk < a.nsplit) v[u] = ld4f_once(a.part + (long long)kk * a.stride + idx);
          else v[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
#pragma unroll
        for (int e = 0; e < 4; e++) s[e] += ((v[0][e] + v[1][e]) + (v[2][e] + v[3][e])) + ((v[4][e] + v[5][e]) + (v[6][e] + v[7][e]));
      }
      for (; k < a.nsplit; k += 4 * Y) {
        f32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
          int kk = k + u * Y;
          if (kk < a.nsplit) v[u] = ld4f_once(a.part + (long long)kk * a.stride + idx);
          else v[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
#pragma unroll
        for (int e = 0; e < 4; e++) s[e] += (v[0][e] + v[1][e]) + (v[2][e] + v[3][e]);
      }
    } else {
      for (int k = y; k < a.nsplit; k += 8 * Y) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
          int kk = k + u * Y;
          v[u] = (kk < a.nsplit) ? a.part[(long long)kk * a.stride + idx] : 0.0f;
        }
        s[0] += ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
      }
    }
  }
  if (Y > 1) {
#pragma unroll
    for (int e = 0; e < 4; e++) red[threadIdx.x][e] = s[e];
    __syncthreads();
    if (y != 0) return;
    for (int k = 1; k < Y; k++)
#pragma unroll
      for (int e = 0; e < 4; e++) s[e] += red[k * X + x][e];
  }
  if (idx >= total || !dst) return;
  if (V == 4) {
#pragma unroll
    for (int e = 0; e < 4; e++) cur[e] += s[e];
    *reinterpret_cast<f32x4*>(dst) = cur;
  } else {
    dst[0] = cur[0] + s[0];
  }
}

// ---------------------------------------------------------------------------
// Parameter preparation: dst[r*ld_r + c*ld_c] = T(src[r*cols + c])
// ---------------------------------------------------------------------------
// copy = scale * source; c_blk > 0: column c of the source goes to destination column (c / c_blk) * c_blk_to + c % c_blk
// (blocks of c_blk columns spread c_blk_to apart: the interleaved projection / gate rows of the triangle multiplication)
// ld_r < 0: a plain fp32 copy of `cols` values into the fp32 region (dst_off counts floats there) instead of the storage-type region
struct PrepDesc { long long src_off, dst_off; int rows, cols; long long ld_r, ld_c; float scale; int c_blk, c_blk_to; };
constexpr int PREP_MAX = 64;   // descriptors per launch (3 KB of kernel arguments)
struct PrepBatch { PrepDesc d[PREP_MAX]; int n; };
template <typename T>
__global__ __launch_bounds__(256) void prep_params_kernel(const float* params, T* dst, float* fdst, PrepBatch pb) {
  // 32 x 32 tiles; a transposed destination (ld_r == 1) goes through LDS so that reads and
  // writes both run along the contiguous index
  __shared__ float tile[32][33];
  const PrepDesc& d = pb.d[blockIdx.y];
  if (d.ld_r < 0) {   // fp32 copy (biases that a GEMM epilogue reads as one vector)
    for (int c = blockIdx.x * 256 + threadIdx.x; c < d.cols; c += gridDim.x * 256) fdst[d.dst_off + c] = params[d.src_off + c];
    return;
  }
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int ntr = (d.rows + 31) / 32, ntc = (d.cols + 31) / 32;
  const bool transposed = d.ld_r == 1 && d.ld_c != 1;
  const float* src = params + d.src_off;
  T* out = dst + d.dst_off;
  for (int t = blockIdx.x; t < ntr * ntc; t += gridDim.x) {
    const int r0 = (t / ntc) * 32, c0 = (t % ntc) * 32;
    if (transposed) {
      for (int k = ty; k < 32; k += 8) {
        const int r = r0 + k, c = c0 + tx;
        tile[k][tx] = (r < d.rows && c < d.cols) ? src[(long long)r * d.cols + c] * d.scale : 0.0f;
      }
      __syncthreads();
      for (int k = ty; k < 32; k += 8) {
        const int c = c0 + k, r = r0 + tx;
        const int cd = d.c_blk > 0 ? (c / d.c_blk) * d.c_blk_to + c % d.c_blk : c;
        if (r < d.rows && c < d.cols) out[r + cd * d.ld_c] = from_f<T>(tile[tx][k]);
      }
      __syncthreads();
    } else {
      for (int k = ty; k < 32; k += 8) {
        const int r = r0 + k, c = c0 + tx;
        const int cd = d.c_blk > 0 ? (c / d.c_blk) * d.c_blk_to + c % d.c_blk : c;
        if (r < d.rows && c < d.cols) out[r * d.ld_r + cd * d.ld_c] = from_f<T>(src[(long long)r * d.cols + c] * d.scale);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Triangle multiplication gating (channel-major tensors [c][M]):
//   proj_t rows: [0,ct) a-projection, [ct,2ct) a-gate, [2ct,3ct) b-projection, [3ct,4ct) b-gate
//   a = mask * sigmoid(ag) * ap,  b likewise
// ---------------------------------------------------------------------------
template <typename T>
__global__ void tm_gate_fwd_kernel(const T* proj_t, const float* mask, T* a_t, T* b_t, int ct, long long M) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)ct * M) return;
  long long m = idx % M;
  int c = idx / M;
  float mk = mask[m];
  float ap = to_f(proj_t[(long long)c * M + m]), ag = to_f(proj_t[(long long)(ct + c) * M + m]);
  float bp = to_f(proj_t[(long long)(2 * ct + c) * M + m]), bg = to_f(proj_t[(long long)(3 * ct + c) * M + m]);
  a_t[idx] = from_f<T>(mk * sigmoidf_(ag) * ap);
  b_t[idx] = from_f<T>(mk * sigmoidf_(bg) * bp);
}
template <typename T>
__global__ void tm_gate_bwd_kernel(const T* proj_t, const float* mask, const T* da_t, const T* db_t, T* dproj_t, int ct,
                                   long long M) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)ct * M) return;
  long long m = idx % M;
  int c = idx / M;
  float mk = mask[m];
  float ap = to_f(proj_t[(long long)c * M + m]), sa = sigmoidf_(to_f(proj_t[(long long)(ct + c) * M + m]));
  float bp = to_f(proj_t[(long long)(2 * ct + c) * M + m]), sb = sigmoidf_(to_f(proj_t[(long long)(3 * ct + c) * M + m]));
  float da = to_f(da_t[idx]) * mk, db = to_f(db_t[idx]) * mk;
  dproj_t[(long long)c * M + m] = from_f<T>(da * sa);
  dproj_t[(long long)(ct + c) * M + m] = from_f<T>(da * ap * sa * (1.0f - sa));
  dproj_t[(long long)(2 * ct + c) * M + m] = from_f<T>(db * sb);
  dproj_t[(long long)(3 * ct + c) * M + m] = from_f<T>(db * bp * sb * (1.0f - sb));
}
// output gate backward: du = G * g, dgraw = G * u * g * (1 - g)
template <typename T>
__global__ void tm_out_bwd_kernel(const T* G, const T* g, const T* u, T* du, T* dgraw, long long n) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  float gv = to_f(g[idx]), Gv = to_f(G[idx]), uv = to_f(u[idx]);
  du[idx] = from_f<T>(Gv * gv);
  dgraw[idx] = from_f<T>(Gv * uv * gv * (1.0f - gv));
}

// The same three kernels and the two-operand add with 8 consecutive elements per thread (16-byte
// accesses for bf16); the host takes them when the row length (M, or n) is a multiple of 8 and the
// buffers are 16-byte aligned: an eighth of the waves for the same bytes.
template <typename T>
__global__ __launch_bounds__(256) void tm_gate_fwd8_kernel(const T* proj_t, const float* mask, T* a_t, T* b_t, int ct, long long M) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (idx >= (long long)ct * M) return;
  const long long m = idx % M;
  const int c = idx / M;
  float mk[8], ap[8], ag[8], bp[8], bg[8], a[8], b[8];
  ld8<float>(mask + m, mk);
  ld8<T>(proj_t + (long long)c * M + m, ap);
  ld8<T>(proj_t + (long long)(ct + c) * M + m, ag);
  ld8<T>(proj_t + (long long)(2 * ct + c) * M + m, bp);
  ld8<T>(proj_t + (long long)(3 * ct + c) * M + m, bg);
#pragma unroll
  for (int e = 0; e < 8; e++) {
    a[e] = mk[e] * sigmoidf_(ag[e]) * ap[e];
    b[e] = mk[e] * sigmoidf_(bg[e]) * bp[e];
  }
  st8<T>(a_t + idx, a);
  st8<T>(b_t + idx, b);
}
template <typename T>
__global__ __launch_bounds__(256) void tm_gate_bwd8_kernel(const T* proj_t, const float* mask, const T* da_t, const T* db_t, T* dproj_t,
                                                           int ct, long long M) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (idx >= (long long)ct * M) return;
  const long long m = idx % M;
  const int c = idx / M;
  float mk[8], ap[8], sa[8], bp[8], sb[8], da[8], db[8], o0[8], o1[8], o2[8], o3[8];
  ld8<float>(mask + m, mk);
  ld8<T>(proj_t + (long long)c * M + m, ap);
  ld8<T>(proj_t + (long long)(ct + c) * M + m, sa);
  ld8<T>(proj_t + (long long)(2 * ct + c) * M + m, bp);
  ld8<T>(proj_t + (long long)(3 * ct + c) * M + m, sb);
  ld8<T>(da_t + idx, da);
  ld8<T>(db_t + idx, db);
#pragma unroll
  for (int e = 0; e < 8; e++) {
    const float s_a = sigmoidf_(sa[e]), s_b = sigmoidf_(sb[e]);
    const float d_a = da[e] * mk[e], d_b = db[e] * mk[e];
    o0[e] = d_a * s_a;
    o1[e] = d_a * ap[e] * s_a * (1.0f - s_a);
    o2[e] = d_b * s_b;
    o3[e] = d_b * bp[e] * s_b * (1.0f - s_b);
  }
  st8<T>(dproj_t + (long long)c * M + m, o0);
  st8<T>(dproj_t + (long long)(ct + c) * M + m, o1);
  st8<T>(dproj_t + (long long)(2 * ct + c) * M + m, o2);
  st8<T>(dproj_t + (long long)(3 * ct + c) * M + m, o3);
}
template <typename T>
__global__ __launch_bounds__(256) void tm_out_bwd8_kernel(const T* G, const T* g, const T* u, T* du, T* dgraw, long long n) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (idx >= n) return;
  float gv[8], Gv[8], uv[8], o0[8], o1[8];
  ld8<T>(g + idx, gv);
  ld8<T>(G + idx, Gv);
  ld8<T>(u + idx, uv);
#pragma unroll
  for (int e = 0; e < 8; e++) {
    o0[e] = Gv[e] * gv[e];
    o1[e] = Gv[e] * uv[e] * gv[e] * (1.0f - gv[e]);
  }
  st8<T>(du + idx, o0);
  st8<T>(dgraw + idx, o1);
}
template <typename T>
__global__ __launch_bounds__(256) void add2x8_kernel(const T* a, const T* b, T* out, long long n) {
  const long long idx = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (idx >= n) return;
  float x[8], y[8];
  ld8<T>(a + idx, x);
  ld8<T>(b + idx, y);
#pragma unroll
  for (int e = 0; e < 8; e++) x[e] += y[e];
  st8<T>(out + idx, x);
}
// ---------------------------------------------------------------------------
// Outer product mean normaliser: inv_norm[i][j] = 1 / (eps + sum_s mask[s][i] mask[s][j])
// ---------------------------------------------------------------------------
__global__ void opm_norm_kernel(const float* mask, float* inv_norm, int s, int r, float eps) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)r * r) return;
  int i = idx / r, j = idx % r;
  float acc = 0.0f;   // 0/1 products: any summation order gives the same (exact) count
  int t = 0;
  for (; t + 32 <= s; t += 32) {   // 64 independent loads in flight per thread: the loop is a chain of memory round trips
    float a[32], b[32];
#pragma unroll
    for (int u = 0; u < 32; u++) { a[u] = mask[(long long)(t + u) * r + i]; b[u] = mask[(long long)(t + u) * r + j]; }
#pragma unroll
    for (int u = 0; u < 32; u++) acc += a[u] * b[u];
  }
  for (; t < s; t++) acc += mask[(long long)t * r + i] * mask[(long long)t * r + j];
  inv_norm[idx] = 1.0f / (eps + acc);
}

// zero n 16-byte words (buffers are 256-byte multiples)
__global__ void zero_bytes16_kernel(uint4* p, long long n) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) p[idx] = make_uint4(0u, 0u, 0u, 0u);
}
template <typename T>
__global__ void add2_kernel(const T* a, const T* b, T* out, long long n) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) out[idx] = from_f<T>(to_f(a[idx]) + to_f(b[idx]));
}
// rows of y[M][N] (row stride ld) scaled by a per-row fp32 factor, in place
template <typename T>
__global__ void rowscale_kernel(T* y, const float* scale, long long M, int N, long long ld) {
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= M * N) return;
  long long m = idx / N;
  int n = idx % N;
  y[m * ld + n] = from_f<T>(to_f(y[m * ld + n]) * scale[m]);
}
