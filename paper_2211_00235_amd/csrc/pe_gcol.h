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
};

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

// qbar[i][hd] = sum_s mask[s][i] q[s][i][hd] / den[i];  grid = r, block = 256 = HD x (256/HD) sequence lanes
template <typename T>
__global__ __launch_bounds__(256) void gcol_qmean_kernel(GcolArgs a) {
  __shared__ float red[256], redm[256];
  const int i = blockIdx.x, HD = a.H * a.d, Wg = 2 * HD + 2 * a.d;
  const int SL = 256 / HD, hd = threadIdx.x % HD, sl = threadIdx.x / HD;
  const T* q = (const T*)a.proj + (long long)i * Wg + hd;
  float acc = 0.0f, msum = 0.0f;
  if (sl < SL)
    for (int t = sl; t < a.s; t += SL) {
      float mk = a.mask[(long long)t * a.r + i];
      acc += mk * to_f(q[(long long)t * a.r * Wg]);
      msum += mk;
    }
  red[threadIdx.x] = acc;
  redm[threadIdx.x] = msum;
  __syncthreads();
  if (sl == 0) {
    for (int k = 1; k < SL; k++) { acc += red[k * HD + hd]; msum += redm[k * HD + hd]; }
    float den = msum + 1e-10f;
    a.qbar[(long long)i * HD + hd] = acc / den;
    if (hd == 0) a.den[i] = den;
  }
}

// softmax over the sequence axis and weighted value sum; grid = r, block = 256
template <typename T>
__global__ __launch_bounds__(256) void gcol_attn_fwd_kernel(GcolArgs a) {
  __shared__ float qb[GC_MAXH * GC_MAXD], red[4], ored[4][GC_MAXH * GC_MAXD];
  const int i = blockIdx.x, H = a.H, d = a.d, HD = H * d, Wg = 2 * HD + 2 * d;
  if (threadIdx.x < HD) qb[threadIdx.x] = a.qbar[(long long)i * HD + threadIdx.x];
  __syncthreads();
  const T* kbase = (const T*)a.proj + (long long)i * Wg + HD;
  const long long tstride = (long long)a.r * Wg;
  float mx[GC_MAXH], sm[GC_MAXH];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++) { mx[h] = -INFINITY; sm[h] = 0.0f; }
  // pass 1: max over valid keys
  for (int t = threadIdx.x; t < a.s; t += 256) {
    if (a.mask[(long long)t * a.r + i] > 0.0f) {
      float kv[GC_MAXD];
      for (int c = 0; c < d; c++) kv[c] = to_f(kbase[t * tstride + c]);
      for (int h = 0; h < H; h++) {
        float l = 0.0f;
        for (int c = 0; c < d; c++) l += qb[h * d + c] * kv[c];
        mx[h] = fmaxf(mx[h], l * a.scale);
      }
    }
  }
  for (int h = 0; h < H; h++) {
    mx[h] = block_reduce_max(mx[h], red);
    if (mx[h] == -INFINITY) mx[h] = 0.0f;
  }
  // pass 2: sum of exponentials
  for (int t = threadIdx.x; t < a.s; t += 256) {
    if (a.mask[(long long)t * a.r + i] > 0.0f) {
      float kv[GC_MAXD];
      for (int c = 0; c < d; c++) kv[c] = to_f(kbase[t * tstride + c]);
      for (int h = 0; h < H; h++) {
        float l = 0.0f;
        for (int c = 0; c < d; c++) l += qb[h * d + c] * kv[c];
        sm[h] += __expf(l * a.scale - mx[h]);
      }
    }
  }
  for (int h = 0; h < H; h++) sm[h] = block_reduce_sum(sm[h], red);
  // pass 3: weights and output
  float oacc[GC_MAXH * GC_MAXD];
#pragma unroll
  for (int e = 0; e < GC_MAXH * GC_MAXD; e++) oacc[e] = 0.0f;
  for (int t = threadIdx.x; t < a.s; t += 256) {
    bool valid = a.mask[(long long)t * a.r + i] > 0.0f;
    float kv[GC_MAXD], vv[GC_MAXD];
    for (int c = 0; c < d; c++) { kv[c] = to_f(kbase[t * tstride + c]); vv[c] = to_f(kbase[t * tstride + d + c]); }
    for (int h = 0; h < H; h++) {
      float l = 0.0f;
      for (int c = 0; c < d; c++) l += qb[h * d + c] * kv[c];
      float pw = (valid && sm[h] > 0.0f) ? __expf(l * a.scale - mx[h]) / sm[h] : 0.0f;
      a.p[((long long)i * H + h) * a.s + t] = pw;
      for (int c = 0; c < d; c++) oacc[h * GC_MAXD + c] += pw * vv[c];
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int h = 0; h < H; h++)
    for (int c = 0; c < d; c++) {
      float v = wave_sum(oacc[h * GC_MAXD + c]);
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

// dO[i][hd] = sum_t dog * sigmoid(g);  dgate = dog * o * s(1-s) -> dproj gate slot.  grid = r
template <typename T>
__global__ __launch_bounds__(256) void gcol_gate_bwd_kernel(GcolArgs a) {
  __shared__ float red[256];
  const int i = blockIdx.x, HD = a.H * a.d, Wg = 2 * HD + 2 * a.d;
  const int SL = 256 / HD, hd = threadIdx.x % HD, sl = threadIdx.x / HD;
  const float ov = a.o[(long long)i * HD + hd];
  float acc = 0.0f;
  if (sl < SL)
    for (int t = sl; t < a.s; t += SL) {
      long long pos = (long long)t * a.r + i;
      float g = to_f(((const T*)a.proj)[pos * Wg + HD + 2 * a.d + hd]);
      float sg = sigmoidf_(g);
      float dv = to_f(((const T*)a.dog)[pos * HD + hd]);
      acc += dv * sg;
      ((T*)a.dproj)[pos * Wg + HD + 2 * a.d + hd] = from_f<T>(dv * ov * sg * (1.0f - sg));
    }
  red[threadIdx.x] = acc;
  __syncthreads();
  if (sl == 0) {
    for (int k = 1; k < SL; k++) acc += red[k * HD + hd];
    a.dO[(long long)i * HD + hd] = acc;
  }
}

// softmax backward per residue: dk, dv -> dproj; dqbar.  grid = r, block = 256
template <typename T>
__global__ __launch_bounds__(256) void gcol_attn_bwd_kernel(GcolArgs a) {
  __shared__ float qb[GC_MAXH * GC_MAXD], dob[GC_MAXH * GC_MAXD], red[4], qred[4][GC_MAXH * GC_MAXD];
  const int i = blockIdx.x, H = a.H, d = a.d, HD = H * d, Wg = 2 * HD + 2 * d;
  if (threadIdx.x < HD) {
    qb[threadIdx.x] = a.qbar[(long long)i * HD + threadIdx.x];
    dob[threadIdx.x] = a.dO[(long long)i * HD + threadIdx.x];
  }
  __syncthreads();
  const T* kbase = (const T*)a.proj + (long long)i * Wg + HD;
  T* dkbase = (T*)a.dproj + (long long)i * Wg + HD;
  const long long tstride = (long long)a.r * Wg;
  float D[GC_MAXH];
#pragma unroll
  for (int h = 0; h < GC_MAXH; h++) D[h] = 0.0f;
  for (int t = threadIdx.x; t < a.s; t += 256) {
    float vv[GC_MAXD];
    for (int c = 0; c < d; c++) vv[c] = to_f(kbase[t * tstride + d + c]);
    for (int h = 0; h < H; h++) {
      float dp = 0.0f;
      for (int c = 0; c < d; c++) dp += dob[h * d + c] * vv[c];
      D[h] += a.p[((long long)i * H + h) * a.s + t] * dp;
    }
  }
  for (int h = 0; h < H; h++) D[h] = block_reduce_sum(D[h], red);
  float dq[GC_MAXH * GC_MAXD];
#pragma unroll
  for (int e = 0; e < GC_MAXH * GC_MAXD; e++) dq[e] = 0.0f;
  for (int t = threadIdx.x; t < a.s; t += 256) {
    float kv[GC_MAXD], vv[GC_MAXD], dk[GC_MAXD], dv[GC_MAXD];
    for (int c = 0; c < d; c++) {
      kv[c] = to_f(kbase[t * tstride + c]);
      vv[c] = to_f(kbase[t * tstride + d + c]);
      dk[c] = 0.0f; dv[c] = 0.0f;
    }
    for (int h = 0; h < H; h++) {
      float pw = a.p[((long long)i * H + h) * a.s + t];
      float dp = 0.0f;
      for (int c = 0; c < d; c++) dp += dob[h * d + c] * vv[c];
      float dl = pw * (dp - D[h]);
      for (int c = 0; c < d; c++) {
        dq[h * GC_MAXD + c] += dl * kv[c];
        dk[c] += dl * qb[h * d + c];
        dv[c] += pw * dob[h * d + c];
      }
    }
    for (int c = 0; c < d; c++) {
      dkbase[t * tstride + c] = from_f<T>(dk[c] * a.scale);
      dkbase[t * tstride + d + c] = from_f<T>(dv[c]);
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int h = 0; h < H; h++)
    for (int c = 0; c < d; c++) {
      float v = wave_sum(dq[h * GC_MAXD + c]);
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
