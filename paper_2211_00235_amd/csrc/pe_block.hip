// Parallel Evoformer block: host orchestration and the C ABI (see include/pe.h).
//
// The MSA branch (+ outer product mean) is enqueued on stream_msa and the pair branch on
// stream_pair; the only cross-stream edges are the ones the paper's Branch Parallelism
// section lists: forward, the pair branch's result is needed by the final outer-product
// projection (which adds it); backward, the outer-product-mean backward reads the pair
// output cotangent (an input) and the row-attention-bias gradient is added to the pair
// branch's gradient of the input pair representation at the very end.
#include <stdio.h>
#include <functional>
#include <mutex>
#include <string>
#include <vector>

#include "pe_attn.h"
#include "pe_elem.h"
#include "pe_gcol.h"
#include "pe_gemm.h"
#include "pe_layout.h"

// Scratch of pe_block_fwd_static: one array per device, held from the load of the library's code object
// until the process ends.  Host code never uses the array's name as an address: pe_create looks the
// device address up once per device and every later use goes through that pointer.
#define PE_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
// No kernel names the array (kernels get its address as an argument).  It stays in the code object, under a symbol
// the loader can find, because host code names it in hipGetSymbolAddress; an explicit `used` attribute would
// keep it as a local symbol instead, which the runtime cannot look up.
static __device__ __align__(256) unsigned char scratch[PE_STATIC_SCRATCH_BYTES];
#define PE_MAX_DEVICES 64
static void* g_scratch_ptr[PE_MAX_DEVICES];
static std::mutex g_scratch_mutex;

struct ProfRec { const char* label; std::string kern; double flops, bytes; hipEvent_t e0, e1; };
struct pe_handle {
  int device;                       // device that was current in pe_create
  void* static_scratch;             // that device's copy of `scratch`
  hipEvent_t ev[6];
  int branches;
  int sync_debug;
  int timing;                       // PE_OPT_KERNEL_TIMING
  int side_streams;                 // PE_OPT_SIDE_STREAMS
  int stack_keep;                   // PE_OPT_STACK_KEEP_CTX
  int stack_overlap;                // PE_OPT_STACK_OVERLAP
  hipStream_t side[2];              // side stream of the MSA branch / of the pair branch
  hipEvent_t side_ev[32];           // ring of fork/join events
  int side_ev_next;
  std::vector<ProfRec> recs;        // one per timed launch since the last collect
  std::vector<hipEvent_t> ev_pool;  // reusable timing events
  std::string last_error;
};

// ---------------------------------------------------------------------------
// bump allocators
// ---------------------------------------------------------------------------
// Base "address" of the dry runs that size the workspace and list the ctx entries: the same carving code runs
// there without memory behind it.  Not null (offsets added to a null pointer are undefined behaviour, which the
// sanitizer build of the host code reports), far from anything mapped, never dereferenced.
static char* const kDryBase = reinterpret_cast<char*>((uintptr_t)1 << 44);
struct Arena {
  char* base = nullptr;
  size_t off = 0, high = 0;
  void* alloc(size_t bytes) {
    size_t o = (off + 255) & ~(size_t)255;
    off = o + bytes;
    if (off > high) high = off;
    return base + o;
  }
  size_t mark() const { return off; }
  void release(size_t m) { off = m; }
};

struct Carver {   // fixed layouts (ctx, prepared weights); optionally records entries
  char* base;
  size_t off = 0;
  std::vector<pe_ctx_entry>* rec = nullptr;
  template <typename U> U* take(const char* name, long long count, int dtype_tag) {
    size_t o = (off + 255) & ~(size_t)255;
    off = o + (size_t)count * sizeof(U);
    if (rec && name) {
      pe_ctx_entry e;
      memset(&e, 0, sizeof(e));
      snprintf(e.name, sizeof(e.name), "%s", name);
      e.offset_bytes = (long long)o;
      e.count = count;
      e.dtype = dtype_tag;
      rec->push_back(e);
    }
    return reinterpret_cast<U*>(base + o);
  }
};

// direct: the pair bias as projected, fp32 [H][r * r] in pair-row order (scratch between the projection and the two
// tiled copies; in the ctx so that the previous sub-operation's epilogue can write it)
template <typename T> struct AttnCtx { T* xhat; float* stats; T* qkvg; T* bias; T* biasT; float* zstats; float* lse; T* o; T* og; float* direct; };
template <typename T> struct TransCtx { T* xhat; float* stats; T* h; unsigned char* hbits; };   // hbits: [M][nC / 8], bit = (h > 0)
template <typename T> struct TriMulCtx { T* zhat; float* stats; T* proj_t; T* a_t; T* b_t; T* g; T* x_t; float* stats_out; T* xhat; T* u; };
template <typename T> struct OpmCtx { T* mhat; float* stats; T* a; T* b; float* inv_norm; T* O; };
template <typename T> struct GlobCtx { T* xhat; float* stats; T* proj; float* qbar; float* den; float* p; float* o; T* og; };
template <typename T> struct Ctx {
  AttnCtx<T> row, col, tas, tae;
  TransCtx<T> mt, pt;
  TriMulCtx<T> tmo, tmi;
  OpmCtx<T> opm;
  GlobCtx<T> gcol;
  T *m1, *m2, *m3, *z0, *z1, *z2, *z3, *z4, *z5;   // z0 = pair input + outer product mean (variants 1, 2)
};

template <typename T> struct AttnW { T *wt_qkvg, *wn_qkvg, *wt_o, *wn_o; };
template <typename T> struct TransW { T *wt_1, *wn_1, *wt_2, *wn_2; };
template <typename T> struct OpmW { T *wt_ab, *wn_ab, *wt_o, *wn_o; };
// wt_pi: the rows of wt_p in 64-row strips of 32 projection rows followed by the 32 gate rows of the same channels
// (a-side strips, then b-side), nullptr unless c_tri is a multiple of 32
template <typename T> struct TriMulW { T *wt_p, *wn_p, *wt_g, *wn_g, *wt_o, *wn_o; float* bias_p; T* wt_pi; };
template <typename T> struct GlobW { T *wt_proj, *wn_proj, *wt_o, *wn_o; };
template <typename T> struct PrepW {
  AttnW<T> row, col, tas, tae;
  TransW<T> mt, pt;
  OpmW<T> opm;
  TriMulW<T> tmo, tmi;
  GlobW<T> gcol;
};

template <typename T> constexpr int dtype_tag() { return sizeof(T) == 2 ? PE_BF16 : PE_F32; }

template <typename T> static void carve_attn_ctx(Carver& cv, AttnCtx<T>& a, const char* pre, long long M, int C, int HD,
                                                 int H, long long B, long long L, bool has_bias, long long Mz) {
  char nm[32];
  auto N = [&](const char* s) { snprintf(nm, sizeof(nm), "%s.%s", pre, s); return nm; };
  a.xhat = cv.take<T>(N("xhat"), M * C, dtype_tag<T>());
  a.stats = cv.take<float>(N("stats"), M * 2, PE_F32);
  a.qkvg = cv.take<T>(N("qkvg"), M * 4 * HD, dtype_tag<T>());
  // pair bias x log2 e, storage type, in the two lane-chunk layouts the attention kernels read (bias_tile_kernel):
  // a key per lane ("bias") and a query per lane ("biasT"); the tile axis is padded to a multiple of 32
  const long long btile = (long long)H * ((L + 31) / 32) * L * 32;
  a.bias = has_bias ? cv.take<T>(N("bias"), btile, dtype_tag<T>()) : nullptr;
  a.biasT = has_bias ? cv.take<T>(N("biasT"), btile, dtype_tag<T>()) : nullptr;
  a.zstats = has_bias ? cv.take<float>(N("zstats"), Mz * 2, PE_F32) : nullptr;
  a.direct = has_bias ? cv.take<float>(nullptr, (long long)H * Mz, 0) : nullptr;   // not listed in the ctx table
  a.lse = cv.take<float>(N("lse"), B * H * L, PE_F32);
  a.o = cv.take<T>(N("o"), M * HD, dtype_tag<T>());
  a.og = cv.take<T>(N("og"), M * HD, dtype_tag<T>());
}
// The ReLU decisions of a transition are also kept as bits when the first GEMM is sure to take the vector epilogue
// (8 consecutive columns per lane): channel counts that are multiples of 8 (ctx and arenas are 256-byte aligned)
static bool trans_bits_ok(int C, int n) { return C % 8 == 0 && (n * C) % 8 == 0; }
template <typename T> static void carve_trans_ctx(Carver& cv, TransCtx<T>& a, const char* pre, long long M, int C, int n) {
  char nm[32];
  auto N = [&](const char* s) { snprintf(nm, sizeof(nm), "%s.%s", pre, s); return nm; };
  a.xhat = cv.take<T>(N("xhat"), M * C, dtype_tag<T>());
  a.stats = cv.take<float>(N("stats"), M * 2, PE_F32);
  a.h = cv.take<T>(N("h"), M * n * C, dtype_tag<T>());
  a.hbits = trans_bits_ok(C, n) ? cv.take<unsigned char>(nullptr, M * ((n * C) / 8), 0) : nullptr;   // not listed in the ctx table
}
template <typename T> static void carve_trimul_ctx(Carver& cv, TriMulCtx<T>& a, const char* pre, long long Mz, int cz, int ct) {
  char nm[32];
  auto N = [&](const char* s) { snprintf(nm, sizeof(nm), "%s.%s", pre, s); return nm; };
  a.zhat = cv.take<T>(N("zhat"), Mz * cz, dtype_tag<T>());
  a.stats = cv.take<float>(N("stats"), Mz * 2, PE_F32);
  a.proj_t = cv.take<T>(N("proj_t"), Mz * 4 * ct, dtype_tag<T>());
  a.a_t = cv.take<T>(N("a_t"), Mz * ct, dtype_tag<T>());
  a.b_t = cv.take<T>(N("b_t"), Mz * ct, dtype_tag<T>());
  a.g = cv.take<T>(N("g"), Mz * cz, dtype_tag<T>());
  a.x_t = cv.take<T>(N("x_t"), Mz * ct, dtype_tag<T>());
  a.stats_out = cv.take<float>(N("stats_out"), Mz * 2, PE_F32);
  a.xhat = cv.take<T>(N("xhat"), Mz * ct, dtype_tag<T>());
  a.u = cv.take<T>(N("u"), Mz * cz, dtype_tag<T>());
}

template <typename T> static size_t carve_ctx(char* base, const pe_dims& d, Ctx<T>& C, std::vector<pe_ctx_entry>* rec) {
  Carver cv;
  cv.base = base;
  cv.rec = rec;
  const long long s = d.s, r = d.r, Mm = s * r, Mz = r * r;
  const int HDm = d.h_msa * d.d_msa, HDz = d.h_pair * d.d_pair;
  carve_attn_ctx<T>(cv, C.row, "row", Mm, d.c_m, HDm, d.h_msa, s, r, true, Mz);
  C.m1 = cv.take<T>("m1", Mm * d.c_m, dtype_tag<T>());
  if (d.col_global) {
    const long long Wg = 2LL * HDm + 2 * d.d_msa;
    C.gcol.xhat = cv.take<T>("col.xhat", Mm * d.c_m, dtype_tag<T>());
    C.gcol.stats = cv.take<float>("col.stats", Mm * 2, PE_F32);
    C.gcol.proj = cv.take<T>("col.proj", Mm * Wg, dtype_tag<T>());
    C.gcol.qbar = cv.take<float>("col.qbar", r * HDm, PE_F32);
    C.gcol.den = cv.take<float>("col.den", r, PE_F32);
    C.gcol.p = cv.take<float>("col.p", r * d.h_msa * s, PE_F32);
    C.gcol.o = cv.take<float>("col.o", r * HDm, PE_F32);
    C.gcol.og = cv.take<T>("col.og", Mm * HDm, dtype_tag<T>());
    memset(&C.col, 0, sizeof(C.col));
  } else {
    carve_attn_ctx<T>(cv, C.col, "col", Mm, d.c_m, HDm, d.h_msa, r, s, false, Mz);
  }
  C.m2 = cv.take<T>("m2", Mm * d.c_m, dtype_tag<T>());
  carve_trans_ctx<T>(cv, C.mt, "mtrans", Mm, d.c_m, d.n_trans);
  C.m3 = cv.take<T>("m3", Mm * d.c_m, dtype_tag<T>());
  C.opm.mhat = cv.take<T>("opm.mhat", Mm * d.c_m, dtype_tag<T>());
  C.opm.stats = cv.take<float>("opm.stats", Mm * 2, PE_F32);
  C.opm.a = cv.take<T>("opm.a", 2 * Mm * d.c_opm, dtype_tag<T>());
  C.opm.b = C.opm.a + Mm * d.c_opm;
  C.opm.inv_norm = cv.take<float>("opm.inv_norm", Mz, PE_F32);
  C.opm.O = cv.take<T>("opm.O", Mz * d.c_opm * d.c_opm, dtype_tag<T>());
  carve_trimul_ctx<T>(cv, C.tmo, "tmo", Mz, d.c_z, d.c_tri);
  C.z0 = d.variant != PE_VARIANT_PARALLEL ? cv.take<T>("z0", Mz * d.c_z, dtype_tag<T>()) : nullptr;
  C.z1 = cv.take<T>("z1", Mz * d.c_z, dtype_tag<T>());
  carve_trimul_ctx<T>(cv, C.tmi, "tmi", Mz, d.c_z, d.c_tri);
  C.z2 = cv.take<T>("z2", Mz * d.c_z, dtype_tag<T>());
  carve_attn_ctx<T>(cv, C.tas, "tas", Mz, d.c_z, HDz, d.h_pair, r, r, true, Mz);
  C.z3 = cv.take<T>("z3", Mz * d.c_z, dtype_tag<T>());
  carve_attn_ctx<T>(cv, C.tae, "tae", Mz, d.c_z, HDz, d.h_pair, r, r, true, Mz);
  C.z4 = cv.take<T>("z4", Mz * d.c_z, dtype_tag<T>());
  carve_trans_ctx<T>(cv, C.pt, "ptrans", Mz, d.c_z, d.n_trans);
  C.z5 = cv.take<T>("z5", Mz * d.c_z, dtype_tag<T>());
  return (cv.off + 255) & ~(size_t)255;
}

// ---------------------------------------------------------------------------
// prepared weights
// ---------------------------------------------------------------------------
struct PrepList {
  std::vector<PrepDesc> t;   // storage-type destinations (offsets in elements from the T region)
  std::vector<PrepDesc> f;   // fp32 destinations
};
template <typename T> struct PrepCarver {
  T* tbase; float* fbase;
  long long toff = 0, foff = 0;
  PrepList* list;
  // weight W[in][out] at params offset src -> transposed copy [out][in] placed at row block `row0` of a [*, in] matrix
  T* region(long long count) { long long o = (toff + 127) & ~127LL; toff = o + count; return tbase + o; }
  float* fregion(long long count) { long long o = (foff + 63) & ~63LL; foff = o + count; return fbase + o; }
  void add(T* dst, long long src, int rows, int cols, long long ld_r, long long ld_c, float scale = 1.0f, int c_blk = 0, int c_blk_to = 0) {
    PrepDesc p; p.src_off = src; p.dst_off = dst - tbase; p.rows = rows; p.cols = cols; p.ld_r = ld_r; p.ld_c = ld_c;
    p.scale = scale; p.c_blk = c_blk; p.c_blk_to = c_blk_to;
    list->t.push_back(p);
  }
  void addf(float* dst, long long src, int n) {
    PrepDesc p; p.src_off = src; p.dst_off = dst - fbase; p.rows = 1; p.cols = n; p.ld_r = -1; p.ld_c = 1; p.scale = 1.0f;
    p.c_blk = 0; p.c_blk_to = 0;
    list->f.push_back(p);
  }
};

// The forward copy of the query weights carries log2 e / sqrt(d): the attention kernels take q' = q log2 e / sqrt(d)
// from the projection and work on base-2 logits q' k without a scale of their own (Section "Evoformer", gated
// self-attention: logits q k / sqrt(d) + bias).  The copy that the backward GEMM uses is unscaled: the dq kernel returns
// the gradient with respect to the unscaled q.
template <typename T> static void prep_attn(PrepCarver<T>& pc, AttnW<T>& w, const AttnP& p, int C, int HD, int dh) {
  const float qscale = 1.4426950408889634f / sqrtf((float)dh);
  w.wt_qkvg = pc.region((long long)4 * HD * C);
  w.wn_qkvg = pc.region((long long)4 * HD * C);
  w.wt_o = pc.region((long long)HD * C);
  w.wn_o = pc.region((long long)HD * C);
  const long long src[4] = {p.w_q, p.w_k, p.w_v, p.w_g};
  for (int k = 0; k < 4; k++) {
    pc.add(w.wt_qkvg + (long long)k * HD * C, src[k], C, HD, 1, C, k == 0 ? qscale : 1.0f);   // [out][in]
    pc.add(w.wn_qkvg + (long long)k * HD, src[k], C, HD, 4 * HD, 1);  // [in][4HD]
  }
  pc.add(w.wt_o, p.w_o, HD, C, 1, HD);   // [C][HD]
  pc.add(w.wn_o, p.w_o, HD, C, C, 1);    // [HD][C]
}
template <typename T> static void prep_trans(PrepCarver<T>& pc, TransW<T>& w, const TransP& p, int C, int n) {
  long long nc = (long long)n * C;
  w.wt_1 = pc.region(nc * C); w.wn_1 = pc.region(nc * C); w.wt_2 = pc.region(nc * C); w.wn_2 = pc.region(nc * C);
  pc.add(w.wt_1, p.w1, C, (int)nc, 1, C);      // [nC][C]
  pc.add(w.wn_1, p.w1, C, (int)nc, nc, 1);     // [C][nC]
  pc.add(w.wt_2, p.w2, (int)nc, C, 1, nc);     // [C][nC]
  pc.add(w.wn_2, p.w2, (int)nc, C, C, 1);      // [nC][C]
}
template <typename T> static void prep_trimul(PrepCarver<T>& pc, TriMulW<T>& w, const TriMulP& p, int cz, int ct) {
  w.wt_p = pc.region((long long)4 * ct * cz); w.wn_p = pc.region((long long)4 * ct * cz);
  w.wt_g = pc.region((long long)cz * cz); w.wn_g = pc.region((long long)cz * cz);
  w.wt_o = pc.region((long long)cz * ct); w.wn_o = pc.region((long long)cz * ct);
  w.bias_p = pc.fregion(4 * ct);
  const long long src[4] = {p.w_ap, p.w_ag, p.w_bp, p.w_bg};
  const long long bsrc[4] = {p.b_ap, p.b_ag, p.b_bp, p.b_bg};
  for (int k = 0; k < 4; k++) {
    pc.add(w.wt_p + (long long)k * ct * cz, src[k], cz, ct, 1, cz);   // [4ct][cz]
    pc.add(w.wn_p + (long long)k * ct, src[k], cz, ct, 4 * ct, 1);    // [cz][4ct]
    pc.addf(w.bias_p + k * ct, bsrc[k], ct);
  }
  w.wt_pi = nullptr;
  if (ct % 32 == 0) {
    w.wt_pi = pc.region((long long)4 * ct * cz);
    for (int k = 0; k < 4; k++)   // group k = 2 side + i: strip (side, block j) holds rows [i * 32, i * 32 + 32) of block j
      pc.add(w.wt_pi + ((long long)(k >> 1) * (ct / 32) * 64 + (k & 1) * 32) * cz, src[k], cz, ct, 1, cz, 1.0f, 32, 64);
  }
  pc.add(w.wt_g, p.w_g, cz, cz, 1, cz);
  pc.add(w.wn_g, p.w_g, cz, cz, cz, 1);
  pc.add(w.wt_o, p.w_o, ct, cz, 1, ct);   // [cz][ct]
  pc.add(w.wn_o, p.w_o, ct, cz, cz, 1);   // [ct][cz]
}

// ---------------------------------------------------------------------------
// Runner: one block, one storage type
// ---------------------------------------------------------------------------
// out = a + b, element-wise; 8 elements per thread when the size and the pointers allow 16-byte accesses
template <typename T> static void launch_add2(hipStream_t st, const T* a, const T* b, T* out, long long n) {
  auto al = [](const void* q) { return ((uintptr_t)q) % 16 == 0; };
  if (n % 8 == 0 && al(a) && al(b) && al(out))
    hipLaunchKernelGGL(add2x8_kernel<T>, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, st, a, b, out, n);
  else
    hipLaunchKernelGGL(add2_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a, b, out, n);
}

template <typename T> struct Runner {
  pe_handle* h;
  pe_dims d;
  ParamLayout PL;
  bool dry = false;
  int err = 0;
  const float* params = nullptr;
  float* dparams = nullptr;
  const T* msa_in = nullptr; const T* pair_in = nullptr;
  const float* msa_mask = nullptr; const float* pair_mask = nullptr;
  hipStream_t sm = nullptr, sp = nullptr;
  Ctx<T> C;
  PrepW<T> W;
  PrepList prep_msa, prep_pair;
  T* prep_tbase_m = nullptr; float* prep_fbase_m = nullptr;
  T* prep_tbase_p = nullptr; float* prep_fbase_p = nullptr;
  Arena am, ap;   // work arenas of the two branches (stack discipline, one frame per sub-operation)
  Arena pm, pp;   // partial sums of the parameter gradients: kept until the end of the backward pass
  long long Mm, Mz;
  int HDm, HDz;

  void init(const pe_dims& dd) {
    d = dd;
    build_param_layout(d, PL);
    Mm = (long long)d.s * d.r;
    Mz = (long long)d.r * d.r;
    HDm = d.h_msa * d.d_msa;
    HDz = d.h_pair * d.d_pair;
  }
  // e: the failing call's code when the caller has it (hipGetLastError clears the error it returns)
  void fail(const char* what, hipError_t e = hipSuccess) {
    if (!err) {
      err = PE_ERR_HIP;
      if (e == hipSuccess) e = hipGetLastError();
      if (h) h->last_error = std::string(what) + ": " + hipGetErrorString(e);
    }
  }
  void check(const char* what) {
    if (dry || err) return;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { fail(what, e); return; }
    if (h && h->sync_debug) {
      e = hipDeviceSynchronize();
      if (e != hipSuccess) fail(what, e);
    }
  }

  hipEvent_t prof_event() {
    hipEvent_t e;
    if (!h->ev_pool.empty()) { e = h->ev_pool.back(); h->ev_pool.pop_back(); return e; }
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  hipEvent_t prof_e0 = nullptr;
  void prof_begin(hipStream_t st) {
    if (dry || err || !h || !h->timing) return;
    prof_e0 = prof_event();
    if (prof_e0) (void)hipEventRecord(prof_e0, st);
  }
  void prof_end(hipStream_t st, const char* label, const char* kern, double flops, double bytes) {
    if (dry || err || !h || !h->timing || !prof_e0) return;
    hipEvent_t e1 = prof_event();
    if (e1) {
      (void)hipEventRecord(e1, st);
      h->recs.push_back(ProfRec{label, kern, flops, bytes, prof_e0, e1});
    }
    prof_e0 = nullptr;
  }
#define PE_LAUNCH(label, flops, bytes, st, kern, grid, block, lds, ...)     \
  do {                                                                      \
    prof_begin(st);                                                         \
    hipLaunchKernelGGL(kern, grid, block, lds, st, __VA_ARGS__);            \
    prof_end(st, label, #kern, (double)(flops), (double)(bytes));           \
    check(label);                                                           \
  } while (0)

  // ---- prepared weights: returns bytes used -------------------------------
  size_t carve_prep(char* base) {
    size_t off = 0;
    auto region = [&](size_t bytes) { size_t o = (off + 255) & ~(size_t)255; off = o + bytes; return base + o; };
    // sizes: generous upper bounds (2 copies of every weight + padding)
    size_t tbytes = (size_t)(2 * PL.total + 128 * 64 + 2LL * 4 * d.c_tri * d.c_z) * sizeof(T);   // + the interleaved projection weights
    size_t fbytes = (size_t)(16 * d.c_tri + 1024) * sizeof(float);
    prep_tbase_m = (T*)region(tbytes); prep_fbase_m = (float*)region(fbytes);
    prep_tbase_p = (T*)region(tbytes); prep_fbase_p = (float*)region(fbytes);
    prep_msa.t.clear(); prep_msa.f.clear(); prep_pair.t.clear(); prep_pair.f.clear();
    PrepCarver<T> pm{prep_tbase_m, prep_fbase_m, 0, 0, &prep_msa};
    prep_attn<T>(pm, W.row, PL.row, d.c_m, HDm, d.d_msa);
    if (!d.col_global) prep_attn<T>(pm, W.col, PL.col, d.c_m, HDm, d.d_msa);
    else {
      const int C_ = d.c_m, dd = d.d_msa, Wg = 2 * HDm + 2 * dd;
      W.gcol.wt_proj = pm.region((long long)Wg * C_); W.gcol.wn_proj = pm.region((long long)Wg * C_);
      W.gcol.wt_o = pm.region((long long)HDm * C_); W.gcol.wn_o = pm.region((long long)HDm * C_);
      const long long src[4] = {PL.col.w_q, PL.col.w_k, PL.col.w_v, PL.col.w_g};
      const int wd[4] = {HDm, dd, dd, HDm}, c0[4] = {0, HDm, HDm + dd, HDm + 2 * dd};
      for (int k = 0; k < 4; k++) {
        pm.add(W.gcol.wt_proj + (long long)c0[k] * C_, src[k], C_, wd[k], 1, C_);   // [Wg][C]
        pm.add(W.gcol.wn_proj + c0[k], src[k], C_, wd[k], Wg, 1);                    // [C][Wg]
      }
      pm.add(W.gcol.wt_o, PL.col.w_o, HDm, C_, 1, HDm);
      pm.add(W.gcol.wn_o, PL.col.w_o, HDm, C_, C_, 1);
    }
    prep_trans<T>(pm, W.mt, PL.mtrans, d.c_m, d.n_trans);
    {
      int co = d.c_opm, cm = d.c_m, cz = d.c_z;
      W.opm.wt_ab = pm.region((long long)2 * co * cm); W.opm.wn_ab = pm.region((long long)2 * co * cm);
      W.opm.wt_o = pm.region((long long)co * co * cz); W.opm.wn_o = pm.region((long long)co * co * cz);
      pm.add(W.opm.wt_ab, PL.opm.w_a, cm, co, 1, cm);
      pm.add(W.opm.wt_ab + (long long)co * cm, PL.opm.w_b, cm, co, 1, cm);
      pm.add(W.opm.wn_ab, PL.opm.w_a, cm, co, 2 * co, 1);
      pm.add(W.opm.wn_ab + co, PL.opm.w_b, cm, co, 2 * co, 1);
      pm.add(W.opm.wt_o, PL.opm.w_o, co * co, cz, 1, (long long)co * co);   // [cz][co*co]
      pm.add(W.opm.wn_o, PL.opm.w_o, co * co, cz, cz, 1);                   // [co*co][cz]
    }
    PrepCarver<T> pp{prep_tbase_p, prep_fbase_p, 0, 0, &prep_pair};
    prep_trimul<T>(pp, W.tmo, PL.tmo, d.c_z, d.c_tri);
    prep_trimul<T>(pp, W.tmi, PL.tmi, d.c_z, d.c_tri);
    prep_attn<T>(pp, W.tas, PL.tas, d.c_z, HDz, d.d_pair);
    prep_attn<T>(pp, W.tae, PL.tae, d.c_z, HDz, d.d_pair);
    prep_trans<T>(pp, W.pt, PL.ptrans, d.c_z, d.n_trans);
    if ((size_t)pm.toff * sizeof(T) > tbytes || (size_t)pp.toff * sizeof(T) > tbytes || (size_t)pm.foff * sizeof(float) > fbytes ||
        (size_t)pp.foff * sizeof(float) > fbytes) {
      err = PE_ERR_DIMS;
      if (h) h->last_error = "prepared weights exceed their region";
    }
    return (off + 255) & ~(size_t)255;
  }
  // one launch per PREP_MAX descriptors; the storage-type copies and the fp32 copies of a branch go together
  void run_prep_list(hipStream_t st, const std::vector<PrepDesc>& vt, const std::vector<PrepDesc>& vf, T* tbase, float* fbase) {
    std::vector<PrepDesc> v(vt);
    v.insert(v.end(), vf.begin(), vf.end());
    for (size_t i = 0; i < v.size(); i += PREP_MAX) {
      PrepBatch pb;
      pb.n = (int)std::min((size_t)PREP_MAX, v.size() - i);
      for (int k = 0; k < pb.n; k++) pb.d[k] = v[i + k];
      dim3 grid(64, pb.n);
      double bytes = 0;
      for (int k = 0; k < pb.n; k++) bytes += (double)pb.d[k].rows * pb.d[k].cols * (4 + (pb.d[k].ld_r < 0 ? 4 : sizeof(T)));
      PE_LAUNCH("prep_params", 0, bytes, st, prep_params_kernel<T>, grid, dim3(256), 0, params, tbase, fbase, pb);
    }
  }
  void run_prep(bool msa_side) {
    if (dry) return;
    if (msa_side) run_prep_list(sm, prep_msa.t, prep_msa.f, prep_tbase_m, prep_fbase_m);
    else run_prep_list(sp, prep_pair.t, prep_pair.f, prep_tbase_p, prep_fbase_p);
  }

  // ---- kernel wrappers -----------------------------------------------------
  const float* P(long long off) const { return params + off; }

  static int ln_lpr(int Cc) {   // lanes per row of the fast LayerNorm kernels, 0 = generic kernel
    for (int l = 2; l <= 64; l <<= 1)
      if (Cc == 8 * l) return l;
    return 0;
  }
  // LayerNorm of the NEXT sub-operation, done by the row-complete epilogue of this sub-operation's last GEMM
  // (gemm_out): nxt is set by the caller of a sub-operation, ln_done_y names the LayerNorm output that a fused
  // launch has already written, and k_ln_fwd skips the launch for exactly that output.
  // w_bias_off / H / direct / zstats: the next sub-operation is a triangle attention whose pair bias is projected
  // from that LayerNorm output (direct == nullptr: no such projection)
  struct NextLn { long long g_off, b_off; T* y; float* stats; bool on; long long w_bias_off; int H; float* direct; float* zstats; };
  NextLn nxt{0, 0, nullptr, nullptr, false, 0, 0, nullptr, nullptr};
  // (one slot per branch is pending at most: the host alternates between the two branches' sub-operations)
  const T* ln_done_y[4] = {nullptr, nullptr, nullptr, nullptr};
  void ln_done_set(const T* y) {
    for (int i = 0; i < 4; i++)
      if (!ln_done_y[i]) { ln_done_y[i] = y; return; }
    ln_done_y[0] = y;
  }
  bool ln_done_take(const T* y) {
    for (int i = 0; i < 4; i++)
      if (ln_done_y[i] == y && y) { ln_done_y[i] = nullptr; return true; }
    return false;
  }
  const float* bias_done_direct = nullptr;
  void prof_cancel() {
    if (prof_e0 && h) h->ev_pool.push_back(prof_e0);
    prof_e0 = nullptr;
  }
  void k_ln_fwd(hipStream_t st, const T* x, long long g_off, long long b_off, T* y, float* stats, long long M, int Cc) {
    if (dry || err) return;
    if (ln_done_take(y)) return;
    const int lpr = ln_lpr(Cc);
    const double bytes = 2.0 * M * Cc * sizeof(T);
    if (lpr) {
      const int rpw = 64 / lpr;
      int grid = (int)std::min<long long>((M + 8 * rpw - 1) / (8 * rpw), 8192);   // a workgroup takes 8 rpw rows per iteration
#define PE_LN_FWD(L) PE_LAUNCH("ln_fwd", 0, bytes, st, (ln_fwd_fast_kernel<T, L>), dim3(grid), dim3(256), 0, x, P(g_off), P(b_off), y, stats, M, d.ln_eps)
      switch (lpr) {
        case 2: PE_LN_FWD(2); break;   case 4: PE_LN_FWD(4); break;   case 8: PE_LN_FWD(8); break;
        case 16: PE_LN_FWD(16); break; case 32: PE_LN_FWD(32); break; default: PE_LN_FWD(64); break;
      }
#undef PE_LN_FWD
      return;
    }
    int grid = (int)std::min<long long>((M + 3) / 4, 4096);
    PE_LAUNCH("ln_fwd", 0, bytes, st, ln_fwd_kernel<T>, dim3(grid), dim3(256), 0, x, P(g_off), P(b_off), y, stats, M, Cc, d.ln_eps);
  }
  // Side streams: parameter-gradient work (dW GEMMs, bias column sums, partial reductions) is off
  // the critical path of the backward pass and its kernels have small grids, so it runs on a
  // second stream per branch, forked from / joined to the branch's stream with events.  A join
  // happens before any buffer the side stream reads is overwritten or released.
  static bool al16(const void* q) { return ((uintptr_t)q) % 16 == 0; }
  // true when no other branch's kernels run beside this call's: both branches on one stream, one branch only,
  // or the AlphaFold2 ordering (MSA stack, outer product mean, pair stack: serial by its data flow)
  // wave groups of the parameter-gradient GEMM: two when the call has the chip to itself, one beside another branch
  int dw_groups() const { return alone() ? 2 : 1; }
  bool alone() const { return sm == sp || (h && h->branches != 3) || d.variant == PE_VARIANT_AF2; }
  bool side_dirty[2] = {false, false};
  int side_idx(hipStream_t st) const { return (st == sp && sp != sm) ? 1 : 0; }
  bool side_on() const { return !dry && h && h->side_streams; }
  hipStream_t side_of(hipStream_t st) { return side_on() ? h->side[side_idx(st)] : st; }
  hipEvent_t next_side_event() { hipEvent_t e = h->side_ev[h->side_ev_next]; h->side_ev_next = (h->side_ev_next + 1) & 31; return e; }
  void fork_side(hipStream_t st) {      // side stream waits for everything queued on st so far
    if (!side_on() || err) return;
    hipEvent_t e = next_side_event();
    if (hipEventRecord(e, st) != hipSuccess || hipStreamWaitEvent(h->side[side_idx(st)], e, 0) != hipSuccess) fail("fork_side");
    side_dirty[side_idx(st)] = true;
  }
  void join_side(hipStream_t st) {      // st waits for the side stream
    if (!side_on() || err || !side_dirty[side_idx(st)]) return;
    hipEvent_t e = next_side_event();
    if (hipEventRecord(e, h->side[side_idx(st)]) != hipSuccess || hipStreamWaitEvent(st, e, 0) != hipSuccess) fail("join_side");
    side_dirty[side_idx(st)] = false;
  }

  // Reductions of fp32 partials into d_params are queued per branch and launched at the end of the
  // backward pass, REDUCE_BATCH per kernel (flush_all): one launch then reads 100 MB and more, while the
  // two or three reductions of a single sub-operation are a launch too small to get near the memory
  // rate.  The partial buffers therefore come from arenas of their own (pm, pp), which are only reset by
  // flush_all.  Two reductions of one sub-operation that add to the same parameters (the z LayerNorm of a
  // biased attention gets one from the q/k/v path and one from the bias path) go into different phases,
  // which are launched one after the other.
  std::vector<ReduceArgs> pend[2][2];
  int phase[2] = {0, 0};
  int bidx(const Arena& ar) const { return &ar == &ap ? 1 : 0; }
  Arena& part_arena(const Arena& ar) { return &ar == &ap ? pp : pm; }
  void next_phase(const Arena& ar) { phase[bidx(ar)] = 1; }
  void end_subop(const Arena& ar) { phase[bidx(ar)] = 0; }
  void reduce_to(const Arena& ar, const float* part, int nsplit, long long stride, int rows, int cols, int nseg,
                 const ReduceSeg* segs) {
    if (dry || err) return;
    ReduceArgs ra;
    ra.part = part; ra.nsplit = nsplit; ra.stride = stride; ra.rows = rows; ra.cols = cols; ra.nseg = nseg;
    for (int i = 0; i < nseg; i++) ra.seg[i] = segs[i];
    ra.dst = dparams;
    long long total = (long long)rows * cols;
    // split lanes per output: 4 up to 256 splits (a wave then reads 1 KB runs of every partial, each thread
    // up to 64 splits with eight loads in flight), 16 beyond.  Measured on the two-stream step: 64 lanes
    // (64-byte runs, twice the bytes fetched) -> 16 lanes -0.6 %, 16 -> 4 lanes for 17..256 splits -0.5 %.
    ra.ylanes = nsplit > 256 ? 16 : (nsplit > 4 ? 4 : 1);
    bool v4 = total >= 4096 && cols % 4 == 0 && stride % 4 == 0 && ((uintptr_t)part) % 16 == 0;
    v4 = v4 && ((uintptr_t)dparams) % 16 == 0;
    for (int i = 0; i < nseg; i++)
      v4 = v4 && segs[i].n_begin % 4 == 0 && segs[i].n_count % 4 == 0 && segs[i].dst_off % 4 == 0 && segs[i].dst_ld % 4 == 0;
    ra.vec = v4 ? 4 : 1;
    pend[bidx(ar)][phase[bidx(ar)]].push_back(ra);
  }
  void launch_reductions(const std::vector<ReduceArgs>& pending, size_t begin, size_t end, hipStream_t st) {
    for (size_t i = begin; i < end; i += REDUCE_BATCH) {
      ReduceBatch rb;
      rb.n = (int)std::min((size_t)REDUCE_BATCH, end - i);
      long long nblocks = 0;
      double bytes = 0;
      for (int k = 0; k < REDUCE_BATCH; k++) {
        rb.a[k] = pending[i + (k < rb.n ? k : 0)];
        rb.first[k] = (int)nblocks;
        if (k < rb.n) {
          long long total = (long long)rb.a[k].rows * rb.a[k].cols;
          int X = 256 / rb.a[k].ylanes * rb.a[k].vec;
          nblocks += (total + X - 1) / X;
          bytes += 4.0 * total * (rb.a[k].nsplit + 2);
        }
      }
      rb.first[REDUCE_BATCH] = (int)nblocks;
      PE_LAUNCH("reduce_partials", 0, bytes, st, reduce_partials_kernel, dim3((unsigned)nblocks), dim3(256), 0, rb);
    }
  }
  // launches every queued reduction of the branch that works in `ar` on that branch's stream and releases the
  // branch's partial buffers.  early_st != nullptr: the reductions queued before mark_early(ar) was called go to
  // early_st instead (the caller has made early_st wait for the kernels that wrote their partials).
  size_t early_n[2][2] = {{0, 0}, {0, 0}};
  void mark_early(const Arena& ar) { const int bi = bidx(ar); early_n[bi][0] = pend[bi][0].size(); early_n[bi][1] = pend[bi][1].size(); }
  void flush_all(const Arena& ar, hipStream_t main_st, hipStream_t early_st = nullptr) {
    const int bi = bidx(ar);
    part_arena(ar).release(0);
    if (dry || err) { pend[bi][0].clear(); pend[bi][1].clear(); phase[bi] = 0; early_n[bi][0] = early_n[bi][1] = 0; return; }
    if (early_st) {
      for (int ph = 0; ph < 2; ph++) launch_reductions(pend[bi][ph], 0, std::min(early_n[bi][ph], pend[bi][ph].size()), early_st);
    }
    fork_side(main_st);
    hipStream_t st = side_of(main_st);
    for (int ph = 0; ph < 2; ph++) {
      const size_t from = early_st ? std::min(early_n[bi][ph], pend[bi][ph].size()) : 0;
      launch_reductions(pend[bi][ph], from, pend[bi][ph].size(), st);
      pend[bi][ph].clear();
    }
    phase[bi] = 0;
    early_n[bi][0] = early_n[bi][1] = 0;
    join_side(main_st);
  }
  void k_ln_bwd(hipStream_t st, Arena& ar, const T* dy, const T* x, const float* stats, long long g_off, long long b_off,
                const T* gin, T* gout, long long M, int Cc) {
    const int lpr = ln_lpr(Cc);
    const int rpw = lpr ? 64 / lpr : 1;
    int grid = (int)std::min<long long>((M + 4 * rpw - 1) / (4 * rpw), LN_MAX_WG);
    float* part = (float*)part_arena(ar).alloc((size_t)grid * 2 * Cc * sizeof(float));
    if (!dry && !err) {
      join_side(st);   // gout may alias a buffer the side stream is still reading
      const double bytes = (gin ? 4.0 : 3.0) * M * Cc * sizeof(T);
      if (lpr) {
#define PE_LN_BWD(L) PE_LAUNCH("ln_bwd", 0, bytes, st, (ln_bwd_fast_kernel<T, L>), dim3(grid), dim3(256), 0, dy, x, stats, P(g_off), gin, gout, part, M)
        switch (lpr) {
          case 2: PE_LN_BWD(2); break;   case 4: PE_LN_BWD(4); break;   case 8: PE_LN_BWD(8); break;
          case 16: PE_LN_BWD(16); break; case 32: PE_LN_BWD(32); break; default: PE_LN_BWD(64); break;
        }
#undef PE_LN_BWD
      } else {
        PE_LAUNCH("ln_bwd", 0, bytes, st, ln_bwd_kernel<T>, dim3(grid), dim3(256), 0, dy, x, stats, P(g_off), gin, gout, part, M, Cc);
      }
      ReduceSeg sg[2] = {{0, Cc, g_off, 0}, {Cc, Cc, b_off, 0}};
      reduce_to(ar, part, grid, 2LL * Cc, 1, 2 * Cc, 2, sg);
    }
  }
  void gemm(hipStream_t st, const Operand& A, bool akc, const Operand& B, bool bkc, int M, int N, int K, int batch,
            const EpiGeneric<T>& e, const char* what, Arena* split_arena = nullptr) {
    // A grid too small to fill the chip with a long contraction: split K, fp32 partials,
    // fixed-order finish kernel that applies the epilogue.
    const int tiles = ((M + 127) / 128) * ((N + 127) / 128);
    const int BK = GemmCfg<T>::BK;
    if (split_arena && batch == 1 && tiles <= 96 && K >= 16 * BK && N % 8 == 0) {
      int want = std::max(2, 256 / tiles);
      long long kc = ((K + want - 1) / want + BK - 1) / BK * BK;
      int nsplit = (int)((K + kc - 1) / kc);
      float* part = (float*)split_arena->alloc((size_t)nsplit * M * N * sizeof(float));
      if (dry || err) return;
      if (!e.vec_ok(N)) { err = PE_ERR_DIMS; if (h) h->last_error = std::string("split-K epilogue alignment: ") + what; return; }
      GemmShape sh{M, N, K, nsplit, (int)kc};
      EpiPartial ep{part, (long long)M * N, N};
      prof_begin(st);
      bool al = false, dwx = false;
      int depth = 0;
      int rc = launch_gemm<T, EpiPartial>(st, A, akc, B, bkc, sh, ep, &al, &dwx, dw_groups(), &depth);
      char kn[64];
      if (dwx && depth) snprintf(kn, sizeof(kn), "gemm_dwp_kernel<%d>", depth);
      else if (dwx) snprintf(kn, sizeof(kn), "gemm_dwx_kernel<%d>", dw_groups());
      else snprintf(kn, sizeof(kn), "gemm_kernel<%s,%s,%s,EpiPartial>", akc ? "kc" : "xc", bkc ? "kc" : "xc", al ? "vec" : "elem");
      prof_end(st, what, kn, 2.0 * M * N * K, ((double)M * K + (double)N * K) * sizeof(T));
      if (rc == -1) { err = PE_ERR_DIMS; if (h) h->last_error = std::string("gemm operand alignment: ") + what; return; }
      check(what);
      long long nv = (long long)M * (N / 8);
      PE_LAUNCH("gemm_finish", 0, 4.0 * nsplit * M * N, st, gemm_finish_kernel<T>, dim3((unsigned)((nv + 255) / 256)), dim3(256), 0,
                part, nsplit, M, N, e);
      return;
    }
    if (dry || err) return;
    GemmShape sh{M, N, K, batch, 0};
    prof_begin(st);
    bool al = false, narrow = false;
    int rc = launch_gemm<T, EpiGeneric<T>>(st, A, akc, B, bkc, sh, e, &al, &narrow);
    if (e.bits_out && !al && rc == 0) {   // the per-element epilogue cannot write the bit mask
      err = PE_ERR_DIMS;
      if (h) h->last_error = std::string("ReLU bit mask without the vector epilogue: ") + what;
    }
    // the exact instantiation (operand layouts, epilogue path, feature mask F; F = 8191 is the general kernel)
    char kn[64];
    if (narrow) snprintf(kn, sizeof(kn), "gemm64_kernel<EpiGeneric,F=%d>", g_gemm_last_features);
    else snprintf(kn, sizeof(kn), "gemm_kernel<%s,%s,%s,EpiGeneric,F=%d>", akc ? "kc" : "xc", bkc ? "kc" : "xc", al ? "vec" : "elem",
                  g_gemm_last_features);
    prof_end(st, what, kn, 2.0 * M * N * K * batch, ((double)M * K + (double)N * K + (double)M * N) * batch * sizeof(T));
    if (rc == -1) { err = PE_ERR_DIMS; if (h) h->last_error = std::string("gemm operand alignment: ") + what; return; }
    check(what);
  }
  // last GEMM of a sub-operation (output projection + residual): where the row-complete kernel applies it also
  // writes the next sub-operation's LayerNorm (nxt), else the plain GEMM
  void gemm_out(hipStream_t st, const Operand& A, const Operand& B, int M, int N, int K, const EpiGeneric<T>& e, const char* what) {
    const bool want = nxt.on;
    nxt.on = false;
    if (want && !dry && !err) {
      RowLn<T> ln;
      memset(&ln, 0, sizeof(ln));
      ln.gamma = P(nxt.g_off); ln.beta = P(nxt.b_off); ln.y = nxt.y; ln.stats = nxt.stats; ln.eps = d.ln_eps;
      if (nxt.direct) { ln.bias_out = nxt.direct; ln.stats2 = nxt.zstats; ln.w_bias = P(nxt.w_bias_off); ln.H = nxt.H; }
      GemmShape sh{M, N, K, 1, 0, 0};
      prof_begin(st);
      if (launch_gemm64r<T, 1>(st, A, B, sh, e, ln)) {
        char kn[64];
        snprintf(kn, sizeof(kn), "gemm64r_kernel<F=%d,MODE=1,HB=%d>", g_gemm_last_features, nxt.direct ? (nxt.H <= 4 ? 4 : 8) : 0);
        prof_end(st, what, kn, 2.0 * M * N * K, ((double)M * K + (double)N * K + 2.0 * M * N) * sizeof(T));
        check(what);
        ln_done_set(nxt.y);
        if (nxt.direct) bias_done_direct = nxt.direct;
        return;
      }
      prof_cancel();
    }
    gemm(st, A, true, B, true, M, N, K, 1, e, what);
  }
  // dy = A . B^T (+ the earlier share already in dxh when acc) is the cotangent of a LayerNorm output:
  //   gout = gin + LayerNorm-backward(dy; x, stats, gain),  gain / offset gradients queued for reduction.
  // Where the row-complete kernel applies this is the GEMM's epilogue (dy never reaches memory), else the GEMM
  // into dxh followed by the LayerNorm backward kernel.
  // bias_db != nullptr: the same LayerNorm output also feeds a pair-bias projection with weight w_bias [Cc][bias_H]
  // whose cotangent is bias_db [bias_H][M] (triangle attention); the fused launch then covers that path as well
  // (returns true), otherwise the caller runs the bias path's own kernel (returns false).
  // fin_add != nullptr (set by the block's backward around the LAST sub-operation of the pair stack): the fused
  // launch writes fin_out = gin + fin_add + (gradient through the LayerNorm) instead of gout and sets fin_done; the
  // stream first waits for fin_from (the stream that produced fin_add).
  // bias_tiled_r > 0 (set by the attention backward around its call): bias_db is the tiled sum as the reduction over the
  // batch axis left it (plane = elements per head), not the row-order copy
  int bias_tiled_r = 0, bias_tiled_transposed = 0;
  long long bias_tiled_plane = 0;
  const T* fin_add = nullptr;
  T* fin_out = nullptr;
  bool fin_done = false;
  hipStream_t fin_from = nullptr;
  hipEvent_t fin_ev = nullptr;
  bool gemm_ln_bwd(hipStream_t st, Arena& ar, const Operand& A, const Operand& B, long long M, int Cc, int K, T* dxh, bool acc,
                   const T* x, const float* stats, long long g_off, long long b_off, const T* gin, T* gout, const char* what,
                   const float* bias_db = nullptr, long long w_bias_off = 0, int bias_H = 0, bool probe = false) {
    if (probe) {   // would the fused launch (with the bias path) be taken?  nothing is allocated or launched
      if (dry || err || Cc != 128 || !bias_db) return false;
      RowLn<T> ln;
      memset(&ln, 0, sizeof(ln));
      ln.gamma = P(g_off); ln.beta = P(b_off); ln.prev = acc ? dxh : nullptr; ln.x = x; ln.stats_in = stats; ln.gin = gin; ln.gout = gout;
      ln.partial = reinterpret_cast<float*>((uintptr_t)256); ln.db = bias_db; ln.db_ld = M; ln.w_bias = P(w_bias_off); ln.H = bias_H;
      GemmShape sh{(int)M, Cc, K, 1, 0, 0};
      return launch_gemm64r<T, 2>(st, A, B, sh, epi_plain<T>(dxh, Cc), ln, false);
    }
    const long long gridf = (M + 63) / 64;
    const int plen = 2 * Cc + (bias_db ? Cc * bias_H : 0);
    // sized by bias_H whether or not the bias path is taken: the planning pass must not depend on pointer values
    float* part = (Cc == 128 || Cc == 256) ? (float*)part_arena(ar).alloc((size_t)gridf * (2 * Cc + Cc * bias_H) * sizeof(float)) : nullptr;
    if (part && !dry && !err) {
      RowLn<T> ln;
      memset(&ln, 0, sizeof(ln));
      ln.gamma = P(g_off); ln.prev = acc ? dxh : nullptr; ln.x = x; ln.stats_in = stats; ln.gin = gin; ln.gout = gout; ln.partial = part;
      if (bias_db) {
        ln.beta = P(b_off); ln.db = bias_db; ln.db_ld = M; ln.w_bias = P(w_bias_off); ln.H = bias_H;
        if (bias_tiled_r > 0) { ln.db_r = bias_tiled_r; ln.db_transposed = bias_tiled_transposed; ln.db_ld = bias_tiled_plane; }
      }
      const bool fin = fin_add != nullptr && fin_out != nullptr && ((uintptr_t)fin_add) % 16 == 0 && ((uintptr_t)fin_out) % 16 == 0;
      if (fin) {
        if (fin_ev && fin_from != st &&
            (hipEventRecord(fin_ev, fin_from) != hipSuccess || hipStreamWaitEvent(st, fin_ev, 0) != hipSuccess)) fail("final add: stream wait");
        ln.gin2 = fin_add; ln.gout = fin_out;
      }
      EpiGeneric<T> e = epi_plain<T>(dxh, Cc);
      GemmShape sh{(int)M, Cc, K, 1, 0, 0};
      join_side(st);   // gout may alias a buffer the side stream is still reading
      prof_begin(st);
      if (launch_gemm64r<T, 2>(st, A, B, sh, e, ln)) {
        char kn[64];
        if (Cc == 256) snprintf(kn, sizeof(kn), "gemm64w_kernel<F=0,MODE=2>");
        else snprintf(kn, sizeof(kn), "gemm64r_kernel<F=0,MODE=2,HB=%d,G2=%d>", bias_db ? (bias_H <= 4 ? 4 : 8) : 0, fin ? 1 : 0);
        prof_end(st, what, kn, 2.0 * M * Cc * K,
                 ((double)M * K + (double)Cc * K + (gin ? 3.0 : 2.0) * M * Cc + (acc ? 1.0 : 0.0) * M * Cc) * sizeof(T));
        check(what);
        ReduceSeg sg[3] = {{0, Cc, g_off, 0}, {Cc, Cc, b_off, 0}, {2 * Cc, Cc * bias_H, w_bias_off, 0}};
        reduce_to(ar, part, (int)gridf, plen, 1, plen, bias_db ? 3 : 2, sg);
        if (fin) fin_done = true;
        return bias_db != nullptr;
      }
      prof_cancel();
    }
    EpiGeneric<T> e = epi_plain<T>(dxh, Cc);
    e.accumulate = acc ? 1 : 0;
    gemm(st, A, true, B, true, (int)M, Cc, K, 1, e, what);
    k_ln_bwd(st, ar, dxh, x, stats, g_off, b_off, gin, gout, M, Cc);
    return false;
  }
  // dW[rows][cols] += sum_k X(row,k) * Y(col,k), K huge: split-K partials + ordered reduce into dparams
  // ncs > 0: additionally dparams[cs[i].dst_off + j] += sum_k Y(cs[i].n_begin + j, k) (bias gradients)
  void gemm_dw(hipStream_t st, Arena& ar, const Operand& X, bool xkc, const Operand& Y, bool ykc, int rows, int cols,
               long long K, int nseg, const ReduceSeg* segs, const char* what, int ncs = 0, const ReduceSeg* cs = nullptr) {
    int tiles = ((rows + 127) / 128) * ((cols + 127) / 128);
    int want = std::max(1, 256 / tiles);
    const int BK = GemmCfg<T>::BK;
    long long kc = (K + want - 1) / want;
    kc = (kc + BK - 1) / BK * BK;
    int nsplit = (int)((K + kc - 1) / kc);
    float* part = (float*)part_arena(ar).alloc((size_t)nsplit * rows * cols * sizeof(float));
    float* cs_part = ncs ? (float*)part_arena(ar).alloc((size_t)nsplit * cols * sizeof(float)) : nullptr;
    if (!dry && !err) {
      fork_side(st);
      st = side_of(st);
      GemmShape sh{rows, cols, (int)K, nsplit, (int)kc};
      EpiPartial ep{part, (long long)rows * cols, cols, cs_part};
      prof_begin(st);
      bool al = false, dwx = false;
      int depth = 0;
      int rc = launch_gemm<T, EpiPartial>(st, X, xkc, Y, ykc, sh, ep, &al, &dwx, dw_groups(), &depth);
      char kn[64];
      if (dwx && depth) snprintf(kn, sizeof(kn), "gemm_dwp_kernel<%d>", depth);
      else if (dwx) snprintf(kn, sizeof(kn), "gemm_dwx_kernel<%d>", dw_groups());
      else snprintf(kn, sizeof(kn), "gemm_kernel<%s,%s,%s,EpiPartial>", xkc ? "kc" : "xc", ykc ? "kc" : "xc", al ? "vec" : "elem");
      prof_end(st, what, kn, 2.0 * rows * cols * K, ((double)rows * K + (double)cols * K) * sizeof(T));
      if (rc == -1) { err = PE_ERR_DIMS; if (h) h->last_error = std::string("gemm_dw operand alignment: ") + what; }
      else check(what);
      reduce_to(ar, part, nsplit, (long long)rows * cols, rows, cols, nseg, segs);
      if (ncs) reduce_to(ar, cs_part, nsplit, cols, 1, cols, ncs, cs);
    }
  }

  // ---- sub-operations: forward ---------------------------------------------
  // tr = 0: GEMM row m is already the head-plane position b*L + p (row attention, starting node);
  // tr = 1: m = p*B' + b with B' = inner (the attention runs along the slow axis: column attention,
  // ending node), so the plane position is (m % inner)*L + m / inner.
  struct AttnGeom { long long B, L; int tr; long long inner, mask_bs, mask_ks; const float* mask; int bias_transposed;
                    const char *l_fwd, *l_dq, *l_dkv; };
  // head-major addressing of the per-head tensors through the GEMM index maps (dh = head dim)
  static void plane_rows(const AttnGeom& g, int dh, int& in, long long& outer, long long& stride) {
    if (g.tr) { in = (int)g.inner; outer = dh; stride = g.L * dh; }
    else { in = 1 << 30; outer = 0; stride = dh; }
  }
  Operand op_heads_rows(const void* ptr, const AttnGeom& g, int dh, long long plane) const {   // rows = positions, k = (head, c)
    Operand o; o.ptr = ptr; o.batch_stride = 0;
    plane_rows(g, dh, o.x_in, o.x_outer, o.x_stride);
    o.k_in = dh; o.k_outer = plane; o.k_stride = 1;
    return o;
  }
  Operand op_heads_cols(const void* ptr, const AttnGeom& g, int dh, long long plane) const {   // rows = (head, c), k = positions
    Operand o; o.ptr = ptr; o.batch_stride = 0;
    o.x_in = dh; o.x_outer = plane; o.x_stride = 1;
    plane_rows(g, dh, o.k_in, o.k_outer, o.k_stride);
    return o;
  }
  void epi_heads(EpiGeneric<T>& e, const AttnGeom& g, int dh, long long plane) const {
    plane_rows(g, dh, e.om_in, e.om_outer, e.om_stride);
    e.on_in = dh; e.on_outer = plane; e.on_stride = 1;
  }

  // first part of an attention sub-operation: LayerNorm of its input and the fused q / k / v / gate projection.
  // It reads nothing but x, so the trunk can enqueue it for the NEXT block's row attention as soon as this
  // block's MSA representation is final (see stack_impl).
  void attn_sub_fwd_pre(hipStream_t st, const AttnP& p, const AttnW<T>& w, AttnCtx<T>& c, const T* x, long long M, int Cc,
                        int H, int dh, const AttnGeom& g) {
    const int HD = H * dh;
    k_ln_fwd(st, x, p.ln_g, p.ln_b, c.xhat, c.stats, M, Cc);
    EpiGeneric<T> e = epi_plain<T>(c.qkvg, 4 * HD);
    epi_heads(e, g, dh, M * dh);
    e.bias_n = P(p.b_g) - 3 * HD;   // only columns >= 3HD carry a bias (see bn_begin)
    e.bn_begin = 3 * HD;
    gemm(st, op_plain(c.xhat, Cc), true, op_plain(w.wt_qkvg, Cc), true, (int)M, 4 * HD, Cc, 1, e, "attn qkvg");
  }
  void attn_sub_fwd(hipStream_t st, Arena& ar, const AttnP& p, const AttnW<T>& w, AttnCtx<T>& c, const T* x, T* xout,
                    long long M, int Cc, int H, int dh, const AttnGeom& g, const T* bias_src, long long bias_ln_g,
                    long long bias_ln_b, bool pre_done = false) {
    const int HD = H * dh;
    if (!pre_done) attn_sub_fwd_pre(st, p, w, c, x, M, Cc, H, dh, g);
    if (c.bias) {
      // bias projection fused with its LayerNorm into a plain [h][pair row] plane (scratch), then the two tiled
      // copies that the attention kernels read
      size_t mkb = ar.mark();
      float* direct = c.direct;
      float* unused = nullptr;
      const int lpr = ln_lpr(d.c_z);
      const bool fast = lpr && lpr <= 32;
      if (!fast) unused = (float*)ar.alloc((size_t)H * Mz * sizeof(float));
      if (!dry && !err) {
        const double fl = 2.0 * Mz * d.c_z * H, by = 1.0 * Mz * d.c_z * sizeof(T) + 4.0 * Mz * H;
        int transposed = g.bias_transposed;
        if (bias_done_direct == direct) {
          bias_done_direct = nullptr;   // projected (in pair-row order) by the previous sub-operation's last GEMM
        } else if (fast) {
          const int rpw = 64 / lpr;
          int grid = (int)std::min<long long>((Mz + 4 * rpw * LNB_UN - 1) / (4 * rpw * LNB_UN), 2048);
#define PE_LNB_FWD(L, HH) PE_LAUNCH("ln_bias_fwd", fl, by, st, (ln_bias_fwd_fast_kernel<T, L, HH>), dim3(grid), dim3(256), 0, bias_src, P(bias_ln_g), P(bias_ln_b), P(p.w_bias), direct, 1.0f, c.zstats, d.r, H, d.ln_eps)
#define PE_LNB_FWD_H(L) do { if (H <= 4) PE_LNB_FWD(L, 4); else PE_LNB_FWD(L, 8); } while (0)
          switch (lpr) {
            case 2: PE_LNB_FWD_H(2); break; case 4: PE_LNB_FWD_H(4); break; case 8: PE_LNB_FWD_H(8); break;
            case 16: PE_LNB_FWD_H(16); break; default: PE_LNB_FWD_H(32); break;
          }
#undef PE_LNB_FWD_H
#undef PE_LNB_FWD
        } else {
          // the general kernel writes [h][query][key] itself (and a second orientation that is not used here)
          int grid = (int)std::min<long long>((Mz + 3) / 4, 4096);
          PE_LAUNCH("ln_bias_fwd", fl, by, st, ln_bias_fwd_kernel<T>, dim3(grid), dim3(256), 0, bias_src, P(bias_ln_g), P(bias_ln_b),
                    P(p.w_bias), direct, unused, c.zstats, d.r, d.c_z, H, d.ln_eps, g.bias_transposed);
          transposed = 0;
        }
        const int NT = (d.r + 31) / 32;
        PE_LAUNCH("bias_tile", 0, (4.0 + 2.0 * sizeof(T)) * H * Mz, st, bias_tile_kernel<T>, dim3(NT, NT, H), dim3(256), 0, direct, c.biasT,
                  c.bias, d.r, transposed, 1.4426950408889634f);
      }
      ar.release(mkb);
    }
    if (!dry && !err) {
      AttnArgs a;
      memset(&a, 0, sizeof(a));
      a.qkvg = c.qkvg; a.plane = M * dh;
      a.B = (int)g.B; a.L = (int)g.L; a.H = H; a.d = dh;
      a.biasK = c.bias; a.biasQ = c.biasT; a.mask = g.mask; a.mask_bs = g.mask_bs; a.mask_ks = g.mask_ks;
      a.o = c.o; a.og = c.og; a.lse = c.lse; a.scale = 1.0f / sqrtf((float)dh);
      dim3 grid(attn_grid_size(g.B, H, g.L));
      if (c.bias) PE_LAUNCH(g.l_fwd, 4.0 * g.B * H * g.L * g.L * dh, (5.0 * M * HD + 1.0 * M * HD) * sizeof(T) + (c.bias ? 4.0 * H * g.L * g.L : 0.0), st, (attn_fwd_kernel<T, true>), grid, dim3(256), 0, a);
      else PE_LAUNCH(g.l_fwd, 4.0 * g.B * H * g.L * g.L * dh, (5.0 * M * HD + 1.0 * M * HD) * sizeof(T) + (c.bias ? 4.0 * H * g.L * g.L : 0.0), st, (attn_fwd_kernel<T, false>), grid, dim3(256), 0, a);
    }
    {
      EpiGeneric<T> e = epi_plain<T>(xout, Cc);
      e.bias_n = P(p.b_o);
      e.res = x; e.ld_res = Cc;
      gemm_out(st, op_heads_rows(c.og, g, dh, M * dh), op_plain(w.wt_o, HD), (int)M, Cc, HD, e, "attn out");
    }
  }

  // ---- global column attention (extra-MSA blocks) ---------------------------
  GcolArgs gcol_args(const GlobCtx<T>& c) const {
    GcolArgs a;
    memset(&a, 0, sizeof(a));
    a.proj = c.proj; a.mask = msa_mask; a.qbar = c.qbar; a.den = c.den; a.p = c.p; a.o = c.o; a.og = c.og;
    a.s = d.s; a.r = d.r; a.H = d.h_msa; a.d = d.d_msa; a.scale = 1.0f / sqrtf((float)d.d_msa);
    return a;
  }
  void gcol_sub_fwd(hipStream_t st, Arena& ar, const T* x, T* xout) {
    const AttnP& p = PL.col;
    GlobCtx<T>& c = C.gcol;
    const int Cc = d.c_m, HD = HDm, dd = d.d_msa, Wg = 2 * HD + 2 * dd;
    k_ln_fwd(st, x, p.ln_g, p.ln_b, c.xhat, c.stats, Mm, Cc);
    {
      EpiGeneric<T> e = epi_plain<T>(c.proj, Wg);
      e.bias_n = P(p.b_g) - (HD + 2 * dd);
      e.bn_begin = HD + 2 * dd;
      gemm(st, op_plain(c.xhat, Cc), true, op_plain(W.gcol.wt_proj, Cc), true, (int)Mm, Wg, Cc, 1, e, "gcol proj");
    }
    size_t mk = ar.mark();
    const int chunks = (d.s + gc_chunk_len(HD) - 1) / gc_chunk_len(HD);
    float* part = (float*)ar.alloc((size_t)chunks * d.r * HD * sizeof(float));
    float* partm = (float*)ar.alloc((size_t)chunks * d.r * sizeof(float));
    if (!dry && !err) {
      GcolArgs a = gcol_args(c);
      a.part = part; a.partm = partm; a.chunks = chunks;
      PE_LAUNCH("gcol_qmean", 0, (double)Mm * HD * sizeof(T), st, gcol_qmean_kernel<T>, dim3(d.r, chunks), dim3(256), 0, a);
      PE_LAUNCH("gcol_qmean_fin", 0, 4.0 * chunks * d.r * HD, st, gcol_qmean_fin_kernel, dim3((unsigned)(((long long)d.r * HD + 255) / 256)), dim3(256), 0, a);
      PE_LAUNCH("gcol_attn_fwd", 6.0 * Mm * HD, 3.0 * Mm * 2 * dd * sizeof(T), st, gcol_attn_fwd_kernel<T>, dim3(d.r), dim3(256), 0, a);
      long long n = Mm * HD;
      if (HD % 8 == 0 && dd % 4 == 0)
        PE_LAUNCH("gcol_gate_fwd", 0, 2.0 * n * sizeof(T), st, gcol_gate_fwd8_kernel<T>, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, a);
      else
        PE_LAUNCH("gcol_gate_fwd", 0, 2.0 * n * sizeof(T), st, gcol_gate_fwd_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, a);
    }
    ar.release(mk);
    {
      EpiGeneric<T> e = epi_plain<T>(xout, Cc);
      e.bias_n = P(p.b_o);
      e.res = x; e.ld_res = Cc;
      gemm(st, op_plain(c.og, HD), true, op_plain(W.gcol.wt_o, HD), true, (int)Mm, Cc, HD, 1, e, "gcol out");
    }
  }
  void gcol_sub_bwd(hipStream_t st, Arena& ar, const T* x, T* g) {
    const AttnP& p = PL.col;
    const GlobCtx<T>& c = C.gcol;
    size_t mk = ar.mark();
    const int Cc = d.c_m, HD = HDm, dd = d.d_msa, Wg = 2 * HD + 2 * dd;
    T* dog = (T*)ar.alloc((size_t)Mm * HD * sizeof(T));
    T* dproj = (T*)ar.alloc((size_t)Mm * Wg * sizeof(T));
    float* dO = (float*)ar.alloc((size_t)d.r * HD * sizeof(float));
    float* dqbar = (float*)ar.alloc((size_t)d.r * HD * sizeof(float));
    T* dxh = (T*)ar.alloc((size_t)Mm * Cc * sizeof(T));
    const int chunks = (d.s + gc_chunk_len(HD) - 1) / gc_chunk_len(HD);
    float* part = (float*)ar.alloc((size_t)chunks * d.r * HD * sizeof(float));
    { ReduceSeg sg[1] = {{0, Cc, p.w_o, Cc}}, cb = {0, Cc, p.b_o, 0};
      gemm_dw(st, ar, op_trans(c.og, HD), false, op_trans(g, Cc), false, HD, Cc, Mm, 1, sg, "gcol dWo", 1, &cb); }
    { EpiGeneric<T> e = epi_plain<T>(dog, HD);
      gemm(st, op_plain(g, Cc), true, op_plain(W.gcol.wn_o, Cc), true, (int)Mm, HD, Cc, 1, e, "gcol dog"); }
    if (!dry && !err) {
      GcolArgs a = gcol_args(c);
      a.dproj = dproj; a.dog = dog; a.dO = dO; a.dqbar = dqbar;
      long long n = Mm * HD;
      a.part = part; a.chunks = chunks;
      PE_LAUNCH("gcol_gate_bwd", 0, 3.0 * n * sizeof(T), st, gcol_gate_bwd_kernel<T>, dim3(d.r, chunks), dim3(256), 0, a);
      PE_LAUNCH("gcol_sum_chunks", 0, 4.0 * chunks * d.r * HD, st, gcol_sum_chunks_kernel, dim3((unsigned)(((long long)d.r * HD + 255) / 256)), dim3(256), 0,
                (const float*)part, dO, chunks, (long long)d.r * HD);
      PE_LAUNCH("gcol_attn_bwd", 12.0 * Mm * HD, 4.0 * Mm * 2 * dd * sizeof(T), st, gcol_attn_bwd_kernel<T>, dim3(d.r), dim3(256), 0, a);
      if (HD % 8 == 0 && dd % 4 == 0)
        PE_LAUNCH("gcol_dq", 0, 1.0 * n * sizeof(T), st, gcol_dq8_kernel<T>, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, a);
      else
        PE_LAUNCH("gcol_dq", 0, 1.0 * n * sizeof(T), st, gcol_dq_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, a);
    }
    { ReduceSeg sg[4] = {{0, HD, p.w_q, HD}, {HD, dd, p.w_k, dd}, {HD + dd, dd, p.w_v, dd}, {HD + 2 * dd, HD, p.w_g, HD}};
      ReduceSeg cb = {HD + 2 * dd, HD, p.b_g, 0};
      gemm_dw(st, ar, op_trans(c.xhat, Cc), false, op_trans(dproj, Wg), false, Cc, Wg, Mm, 4, sg, "gcol dWproj", 1, &cb); }
    { EpiGeneric<T> e = epi_plain<T>(dxh, Cc);
      gemm(st, op_plain(dproj, Wg), true, op_plain(W.gcol.wn_proj, Wg), true, (int)Mm, Cc, Wg, 1, e, "gcol dxhat"); }
    k_ln_bwd(st, ar, dxh, x, c.stats, p.ln_g, p.ln_b, g, g, Mm, Cc);
    end_subop(ar);
    ar.release(mk);
  }

  void trans_sub_fwd(hipStream_t st, const TransP& p, const TransW<T>& w, TransCtx<T>& c, const T* x, T* xout, long long M,
                     int Cc) {
    const int nC = d.n_trans * Cc;
    k_ln_fwd(st, x, p.ln_g, p.ln_b, c.xhat, c.stats, M, Cc);
    {
      EpiGeneric<T> e = epi_plain<T>(c.h, nC);
      e.bias_n = P(p.b1); e.act = 1;
      if (c.hbits) { e.bits_out = c.hbits; e.ld_bits = nC / 8; }
      gemm(st, op_plain(c.xhat, Cc), true, op_plain(w.wt_1, Cc), true, (int)M, nC, Cc, 1, e, "trans 1");
    }
    {
      EpiGeneric<T> e = epi_plain<T>(xout, Cc);
      e.bias_n = P(p.b2); e.res = x; e.ld_res = Cc;
      gemm_out(st, op_plain(c.h, nC), op_plain(w.wt_2, nC), (int)M, Cc, nC, e, "trans 2");
    }
  }

  void trimul_sub_fwd(hipStream_t st, const TriMulP& p, const TriMulW<T>& w, TriMulCtx<T>& c, const T* z, T* zout,
                      bool outgoing) {
    const int cz = d.c_z, ct = d.c_tri, r = d.r;
    k_ln_fwd(st, z, p.ln_in_g, p.ln_in_b, c.zhat, c.stats, Mz, cz);
    bool gated = false;   // projection, gate pre-activation and gated operands from one kernel
    if (!dry && !err && w.wt_pi) {
      EpiTmGate<T> eg;
      eg.proj_t = c.proj_t; eg.a_t = c.a_t; eg.b_t = c.b_t; eg.bias = w.bias_p; eg.mask = pair_mask; eg.ct = ct; eg.Mz = Mz;
      const Operand A = op_plain(w.wt_pi, cz), B = op_plain(c.zhat, cz);
      GemmShape sh{4 * ct, (int)Mz, cz, 1, 0, 0};
      if (eg.vec_ok((int)Mz) && gemm_operand_ok<T>(A, true, 4 * ct, sh) && gemm_operand_ok<T>(B, true, (int)Mz, sh)) {
        prof_begin(st);
        int rc = launch_gemm<T, EpiTmGate<T>>(st, A, true, B, true, sh, eg);
        prof_end(st, "trimul proj+gate", "gemm_kernel<kc,kc,vec,EpiTmGate>", 2.0 * 4 * ct * Mz * cz,
                 ((double)4 * ct * cz + (double)Mz * cz + 6.0 * ct * Mz) * sizeof(T));
        if (rc == -1) { err = PE_ERR_DIMS; if (h) h->last_error = "gemm operand alignment: trimul proj+gate"; }
        else check("trimul proj+gate");
        gated = true;
      }
    }
    if (!gated) {  // channel-major projections: proj_t[4ct][Mz] = W_p^T[4ct][cz] . zhat^T
      EpiGeneric<T> e = epi_plain<T>(c.proj_t, Mz);
      e.bias_m = w.bias_p;
      gemm(st, op_plain(w.wt_p, cz), true, op_plain(c.zhat, cz), true, 4 * ct, (int)Mz, cz, 1, e, "trimul proj");
    }
    if (!dry && !err && !gated) {
      long long n = (long long)ct * Mz;
      if (Mz % 8 == 0 && al16(c.proj_t) && al16(pair_mask) && al16(c.a_t) && al16(c.b_t))
        PE_LAUNCH("tm_gate_fwd", 0, 6.0 * n * sizeof(T), st, tm_gate_fwd8_kernel<T>, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, c.proj_t,
                  pair_mask, c.a_t, c.b_t, ct, Mz);
      else
        PE_LAUNCH("tm_gate_fwd", 0, 6.0 * n * sizeof(T), st, tm_gate_fwd_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c.proj_t, pair_mask,
                  c.a_t, c.b_t, ct, Mz);
    }
    {  // per-channel contraction over the third residue
      EpiGeneric<T> e = epi_plain<T>(c.x_t, r);
      e.out_batch = Mz;
      if (outgoing) gemm(st, op_plain(c.a_t, r, Mz), true, op_plain(c.b_t, r, Mz), true, r, r, r, ct, e, "trimul out");
      else gemm(st, op_trans(c.a_t, r, Mz), false, op_trans(c.b_t, r, Mz), false, r, r, r, ct, e, "trimul in");
    }
    bool lnc_t = false;   // bf16, 64 or 128 channels: the kernels that move 256-byte runs
    if constexpr (std::is_same<T, bf16>::value)
      lnc_t = (ct == 64 || ct == 128) && Mz % 8 == 0 && al16(c.x_t) && al16(c.xhat);
    if (!dry && !err && lnc_t) {
      if constexpr (std::is_same<T, bf16>::value) {
        const unsigned g128 = (unsigned)((Mz + 127) / 128);
        if (ct == 128)
          PE_LAUNCH("ln_cmajor_fwd", 0, 2.0 * Mz * ct * sizeof(T), st, ln_cmajor_fwd_t_kernel<16>, dim3(g128), dim3(256), 0, c.x_t, P(p.ln_out_g),
                    P(p.ln_out_b), c.xhat, c.stats_out, Mz, d.ln_eps);
        else
          PE_LAUNCH("ln_cmajor_fwd", 0, 2.0 * Mz * ct * sizeof(T), st, ln_cmajor_fwd_t_kernel<8>, dim3(g128), dim3(256), 0, c.x_t, P(p.ln_out_g),
                    P(p.ln_out_b), c.xhat, c.stats_out, Mz, d.ln_eps);
      }
    }
    if (!dry && !err && !lnc_t) {
      size_t lds = (size_t)64 * (ct + 1) * sizeof(float);
#define PE_LNC_FWD(N) PE_LAUNCH("ln_cmajor_fwd", 0, 2.0 * Mz * ct * sizeof(T), st, (ln_cmajor_fwd_fast_kernel<T, N>), dim3((unsigned)((Mz + 63) / 64)), dim3(256), lds, c.x_t, P(p.ln_out_g), P(p.ln_out_b), c.xhat, c.stats_out, Mz, ct, d.ln_eps)
      if (Mz % 4 == 0 && ct % 8 == 0) {
        const int nit = (ct + 15) / 16;   // c_tri <= 192
        if (nit <= 2) PE_LNC_FWD(2); else if (nit <= 4) PE_LNC_FWD(4); else if (nit <= 8) PE_LNC_FWD(8); else PE_LNC_FWD(12);
      }
#undef PE_LNC_FWD
      else
        PE_LAUNCH("ln_cmajor_fwd", 0, 2.0 * Mz * ct * sizeof(T), st, ln_cmajor_fwd_kernel<T>, dim3((unsigned)((Mz + 63) / 64)), dim3(256), lds, c.x_t,
                  P(p.ln_out_g), P(p.ln_out_b), c.xhat, c.stats_out, Mz, ct, d.ln_eps);
    }
    {
      EpiGeneric<T> e = epi_plain<T>(c.g, cz);
      e.bias_n = P(p.b_g); e.act = 2;
      gemm(st, op_plain(c.zhat, cz), true, op_plain(w.wt_g, cz), true, (int)Mz, cz, cz, 1, e, "trimul gate");
    }
    {
      EpiGeneric<T> e = epi_plain<T>(zout, cz);
      e.bias_n = P(p.b_o);
      e.aux = c.u; e.ld_aux = cz;
      e.mul = c.g; e.ld_mul = cz;
      e.res = z; e.ld_res = cz;
      gemm_out(st, op_plain(c.xhat, ct), op_plain(w.wt_o, ct), (int)Mz, cz, ct, e, "trimul outproj");
    }
  }

  AttnGeom geom_row() const { return AttnGeom{d.s, d.r, 0, 0, d.r, 1, msa_mask, 0,
                                               "attn_fwd row", "attn_dq row", "attn_dkv row"}; }
  AttnGeom geom_col() const { return AttnGeom{d.r, d.s, 1, d.r, 1, d.r, msa_mask, 0,
                                               "attn_fwd col", "attn_dq col", "attn_dkv col"}; }
  AttnGeom geom_tas() const { return AttnGeom{d.r, d.r, 0, 0, d.r, 1, pair_mask, 0,
                                               "attn_fwd tas", "attn_dq tas", "attn_dkv tas"}; }
  AttnGeom geom_tae() const { return AttnGeom{d.r, d.r, 1, d.r, 1, d.r, pair_mask, 1,
                                               "attn_fwd tae", "attn_dq tae", "attn_dkv tae"}; }

  // MSA stack: row attention (bias read from bias_pair), column attention, transition.  Steps can
  // be enqueued one at a time so that the host alternates between the two streams (a stream whose
  // kernels are enqueued late starts late: the host needs ~10 us per launch).
  static constexpr int MSA_STEPS = 3, PAIR_STEPS = 5;
  static_assert(MSA_STEPS <= PAIR_STEPS - 2, "the backward pass enqueues every MSA step before the last pair step");
  // set by the trunk when the previous block's call has already enqueued this block's MSA-side weight preparation
  // and the first part of its row attention (fwd_row_pre) on stream_msa
  bool row_pre_done = false;
  void fwd_row_pre() {
    run_prep(true);
    attn_sub_fwd_pre(sm, PL.row, W.row, C.row, msa_in, Mm, d.c_m, d.h_msa, d.d_msa, geom_row());
  }
  void fwd_msa_step(int i, const T* bias_pair, T* msa_out) {
    if (i == 0) {
      attn_sub_fwd(sm, am, PL.row, W.row, C.row, msa_in, C.m1, Mm, d.c_m, d.h_msa, d.d_msa, geom_row(), bias_pair,
                   PL.row.ln_z_g, PL.row.ln_z_b, row_pre_done);
    } else if (i == 1) {
      if (d.col_global) gcol_sub_fwd(sm, am, C.m1, C.m2);
      else attn_sub_fwd(sm, am, PL.col, W.col, C.col, C.m1, C.m2, Mm, d.c_m, d.h_msa, d.d_msa, geom_col(), nullptr, 0, 0);
    } else {
      trans_sub_fwd(sm, PL.mtrans, W.mt, C.mt, C.m2, C.m3, Mm, d.c_m);
      if (!dry && !err && msa_out) {
        if (hipMemcpyAsync(msa_out, C.m3, (size_t)Mm * d.c_m * sizeof(T), hipMemcpyDeviceToDevice, sm) != hipSuccess)
          fail("copy msa_out");
      }
    }
  }
  void fwd_msa_stack(const T* bias_pair, T* msa_out) {
    for (int i = 0; i < MSA_STEPS; i++) fwd_msa_step(i, bias_pair, msa_out);
  }
  // outer product mean of x, up to its output projection
  void fwd_opm_outer(const T* x) {
    const int co = d.c_opm, r = d.r;
    const long long Wd = (long long)r * co;
    k_ln_fwd(sm, x, PL.opm.ln_g, PL.opm.ln_b, C.opm.mhat, C.opm.stats, Mm, d.c_m);
    for (int k = 0; k < 2; k++) {
      EpiGeneric<T> e = epi_plain<T>(k ? C.opm.b : C.opm.a, co);
      e.bias_n = P(k ? PL.opm.b_b : PL.opm.b_a);
      e.rowscale = msa_mask;
      gemm(sm, op_plain(C.opm.mhat, d.c_m), true, op_plain(W.opm.wt_ab + (long long)k * co * d.c_m, d.c_m), true, (int)Mm,
           co, d.c_m, 1, e, "opm ab");
    }
    if (!dry && !err) {
      PE_LAUNCH("opm_norm", 2.0 * Mz * d.s, 4.0 * (Mz + Mm), sm, opm_norm_kernel, dim3((unsigned)((Mz + 255) / 256)), dim3(256), 0, msa_mask, C.opm.inv_norm,
                         d.s, r, d.opm_eps);
    }
    {
      EpiGeneric<T> e = epi_plain<T>(C.opm.O, Wd);
      e.scale2d = C.opm.inv_norm; e.s2_mdiv = co; e.s2_ndiv = co; e.s2_ld = r;
      gemm(sm, op_trans(C.opm.a, Wd), false, op_trans(C.opm.b, Wd), false, (int)Wd, (int)Wd, d.s, 1, e, "opm outer");
    }
  }
  // Parallel block, MSA branch: the stack, then the outer product mean of its output up to the
  // projection (which needs the pair branch's result)
  void fwd_msa(T* msa_out) {
    run_prep(true);
    fwd_msa_stack(pair_in, msa_out);
    fwd_opm_outer(C.m3);
  }
  // output projection of the outer product mean, added to z5 (a pair representation)
  void fwd_opm_project(T* pair_out, const T* z5) {
    const int co = d.c_opm, r = d.r;
    const long long Wd = (long long)r * co;
    Operand A;
    A.ptr = C.opm.O; A.batch_stride = 0;
    A.x_in = r; A.x_outer = (long long)co * Wd; A.x_stride = co;
    A.k_in = co; A.k_outer = Wd; A.k_stride = 1;
    EpiGeneric<T> e = epi_plain<T>(pair_out, d.c_z);
    e.bias_n = P(PL.opm.b_o);
    e.res = z5; e.ld_res = d.c_z;
    gemm(sm, A, true, op_plain(W.opm.wt_o, (long long)co * co), true, (int)Mz, d.c_z, co * co, 1, e, "opm project");
  }
  void fwd_pair() {
    run_prep(false);
    fwd_pair_stack(pair_in, C.z5);
  }
  void fwd_pair_step(int i, const T* z_in, T* z_out) {
    // the LayerNorm that opens the next pair sub-operation rides on this one's output projection
    switch (i) {
      case 0: nxt = NextLn{PL.tmi.ln_in_g, PL.tmi.ln_in_b, C.tmi.zhat, C.tmi.stats, true, 0, 0, nullptr, nullptr}; break;
      case 1: nxt = NextLn{PL.tas.ln_g, PL.tas.ln_b, C.tas.xhat, C.tas.stats, true, PL.tas.w_bias, d.h_pair, C.tas.direct, C.tas.zstats}; break;
      case 2: nxt = NextLn{PL.tae.ln_g, PL.tae.ln_b, C.tae.xhat, C.tae.stats, true, PL.tae.w_bias, d.h_pair, C.tae.direct, C.tae.zstats}; break;
      case 3: nxt = NextLn{PL.ptrans.ln_g, PL.ptrans.ln_b, C.pt.xhat, C.pt.stats, true, 0, 0, nullptr, nullptr}; break;
      default: nxt.on = false; break;
    }
    switch (i) {
      case 0: trimul_sub_fwd(sp, PL.tmo, W.tmo, C.tmo, z_in, C.z1, true); break;
      case 1: trimul_sub_fwd(sp, PL.tmi, W.tmi, C.tmi, C.z1, C.z2, false); break;
      case 2: attn_sub_fwd(sp, ap, PL.tas, W.tas, C.tas, C.z2, C.z3, Mz, d.c_z, d.h_pair, d.d_pair, geom_tas(), C.z2,
                           PL.tas.ln_g, PL.tas.ln_b); break;
      case 3: attn_sub_fwd(sp, ap, PL.tae, W.tae, C.tae, C.z3, C.z4, Mz, d.c_z, d.h_pair, d.d_pair, geom_tae(), C.z3,
                           PL.tae.ln_g, PL.tae.ln_b); break;
      default: trans_sub_fwd(sp, PL.ptrans, W.pt, C.pt, C.z4, z_out, Mz, d.c_z); break;
    }
    nxt.on = false;
  }
  void fwd_pair_stack(const T* z_in, T* z_out) {
    for (int i = 0; i < PAIR_STEPS; i++) fwd_pair_step(i, z_in, z_out);
  }

  // ---- sub-operations: backward --------------------------------------------
  // g: running gradient w.r.t. the sub-op's output (and, after the call, its input) [M][C]
  // g = gin + (gradient through the transition); gin defaults to g (in place)
  void trans_sub_bwd(hipStream_t st, Arena& ar, const TransP& p, const TransW<T>& w, const TransCtx<T>& c, const T* x, T* g,
                     long long M, int Cc, const T* gin = nullptr) {
    if (!gin) gin = g;
    size_t mk = ar.mark();
    const int nC = d.n_trans * Cc;
    T* dh = (T*)ar.alloc((size_t)M * nC * sizeof(T));
    T* dxh = (T*)ar.alloc((size_t)M * Cc * sizeof(T));
    { ReduceSeg sg[1] = {{0, Cc, p.w2, Cc}}, cb = {0, Cc, p.b2, 0};
      gemm_dw(st, ar, op_trans(c.h, nC), false, op_trans(gin, Cc), false, nC, Cc, M, 1, sg, "trans dW2", 1, &cb); }
    { EpiGeneric<T> e = epi_plain<T>(dh, nC);
      if (c.hbits) { e.bits_in = c.hbits; e.ld_bits = nC / 8; }     // 1 bit instead of 16 per hidden unit
      else { e.relu_mask = c.h; e.ld_rm = nC; }
      gemm(st, op_plain(gin, Cc), true, op_plain(w.wn_2, Cc), true, (int)M, nC, Cc, 1, e, "trans dh"); }
    { ReduceSeg sg[1] = {{0, nC, p.w1, nC}}, cb = {0, nC, p.b1, 0};
      gemm_dw(st, ar, op_trans(c.xhat, Cc), false, op_trans(dh, nC), false, Cc, nC, M, 1, sg, "trans dW1", 1, &cb); }
    gemm_ln_bwd(st, ar, op_plain(dh, nC), op_plain(w.wn_1, nC), M, Cc, nC, dxh, false, x, c.stats, p.ln_g, p.ln_b, gin, g, "trans dxhat");
    end_subop(ar);
    ar.release(mk);
  }

  // bias_gout: where the gradient through the pair bias goes (gin added when not null)
  void attn_sub_bwd(hipStream_t st, Arena& ar, const AttnP& p, const AttnW<T>& w, const AttnCtx<T>& c, const T* x, T* g,
                    long long M, int Cc, int H, int dh, const AttnGeom& gm, const T* bias_src, long long bias_ln_g,
                    long long bias_ln_b, const T* bias_gin, T* bias_gout) {
    size_t mk = ar.mark();
    const int HD = H * dh;
    T* dog = (T*)ar.alloc((size_t)M * HD * sizeof(T));
    T* dO = (T*)ar.alloc((size_t)M * HD * sizeof(T));
    T* dqkvg = (T*)ar.alloc((size_t)M * 4 * HD * sizeof(T));
    float* Dv = (float*)ar.alloc((size_t)gm.B * H * gm.L * sizeof(float));
    T* dxh = (T*)ar.alloc((size_t)M * Cc * sizeof(T));
    T* dS = nullptr;
    float* dbias = nullptr;
    float* dbias_rows = nullptr;
    const long long btile = (long long)H * ((gm.L + 31) / 32) * gm.L * 32;   // elements of one [H] set of chunk-ordered planes
    if (c.bias) {
      dS = (T*)ar.alloc((size_t)((gm.B + 1) / 2) * btile * sizeof(T));
      dbias = (float*)ar.alloc((size_t)btile * sizeof(float));
      dbias_rows = (float*)ar.alloc((size_t)H * Mz * sizeof(float));   // dbias in pair-row order
    }
    // triangle attention: the bias is projected from the same LayerNorm output as q / k / v / gate and its gradient
    // goes into the same running gradient, so the two LayerNorm backward passes are one (on the sum of the cotangents)
    bool bias_gather = false;
    const bool bias_same_ln = c.bias && bias_src == x && bias_ln_g == p.ln_g && bias_ln_b == p.ln_b && bias_gin == g && bias_gout == g &&
                              M == Mz && Cc == d.c_z;
    { ReduceSeg sg[1] = {{0, Cc, p.w_o, Cc}}, cb = {0, Cc, p.b_o, 0};
      gemm_dw(st, ar, op_heads_cols(c.og, gm, dh, M * dh), false, op_trans(g, Cc), false, HD, Cc, M, 1, sg, "attn dWo", 1, &cb); }
    // dog = g W_o^T; its epilogue turns dog into dO, the gate gradient and D (no dog tensor, no pass of its
    // own) whenever the vector epilogue applies
    bool pre_fused = false;
    {
      EpiAttnPre<T> ep;
      ep.gate = c.qkvg + 3LL * H * M * dh; ep.o = c.o; ep.dO = dO; ep.dgate = dqkvg + 3LL * H * M * dh; ep.D = Dv;
      ep.plane = M * dh; ep.H = H; ep.dh = dh; ep.L = (int)gm.L; ep.tr = gm.tr; ep.inner = (int)gm.inner;
      const Operand A = op_plain(g, Cc), B = op_plain(w.wn_o, Cc);
      GemmShape sh{(int)M, HD, Cc, 1, 0};
      pre_fused = ep.vec_ok(HD) && gemm_operand_ok<T>(A, true, (int)M, sh) && gemm_operand_ok<T>(B, true, HD, sh);
      if (pre_fused && !dry && !err) {
        prof_begin(st);
        bool al = false, narrow = false;
        int rc = launch_gemm<T, EpiAttnPre<T>>(st, A, true, B, true, sh, ep, &al, &narrow);
        prof_end(st, "attn dog+pre", narrow ? "gemm64_kernel<EpiAttnPre>" : "gemm_kernel<kc,kc,vec,EpiAttnPre>", 2.0 * M * HD * Cc,
                 ((double)M * Cc + (double)HD * Cc + 4.0 * M * HD) * sizeof(T));
        if (rc == -1) { err = PE_ERR_DIMS; if (h) h->last_error = "gemm operand alignment: attn dog"; }
        else check("attn dog+pre");
      }
    }
    if (!pre_fused) {
      EpiGeneric<T> e = epi_plain<T>(dog, HD);
      epi_heads(e, gm, dh, M * dh);
      gemm(st, op_plain(g, Cc), true, op_plain(w.wn_o, Cc), true, (int)M, HD, Cc, 1, e, "attn dog");
    }
    if (!dry && !err) {
      AttnArgs a;
      memset(&a, 0, sizeof(a));
      a.qkvg = c.qkvg; a.plane = M * dh;
      a.B = (int)gm.B; a.L = (int)gm.L; a.H = H; a.d = dh;
      a.biasK = c.bias; a.biasQ = c.biasT; a.mask = gm.mask; a.mask_bs = gm.mask_bs; a.mask_ks = gm.mask_ks;
      a.o = c.o; a.og = c.og; a.lse = c.lse; a.scale = 1.0f / sqrtf((float)dh);
      a.dog = dog; a.dO = dO; a.D = Dv; a.dqkvg = dqkvg; a.dS = dS;
      long long tot = gm.B * gm.L * H;
      if (!pre_fused)
        PE_LAUNCH("attn_bwd_pre", 0, 5.0 * M * HD * sizeof(T), st, attn_bwd_pre_kernel<T>, dim3((unsigned)((tot * 8 + 255) / 256)), dim3(256), 0, a);
      dim3 grid(attn_grid_size(gm.B, H, gm.L));
      // biased attention: two batch rows per workgroup, their dS tiles summed before the write
      const long long Bds = c.bias ? (gm.B + 1) / 2 : gm.B;
      if (c.bias) PE_LAUNCH(gm.l_dq, 6.0 * gm.B * H * gm.L * gm.L * dh, 5.0 * M * HD * sizeof(T) + 1.0 * Bds * H * gm.L * gm.L * sizeof(T), st, (attn_bwd_dq2_kernel<T>), dim3(attn_grid_size(Bds, H, gm.L)), dim3(512), 0, a);
      else PE_LAUNCH(gm.l_dq, 6.0 * gm.B * H * gm.L * gm.L * dh, 5.0 * M * HD * sizeof(T) + (c.bias ? 1.0 * gm.B * H * gm.L * gm.L * sizeof(T) : 0.0), st, (attn_bwd_dq_kernel<T, false>), grid, dim3(256), 0, a);
      if (c.bias) PE_LAUNCH(gm.l_dkv, 8.0 * gm.B * H * gm.L * gm.L * dh, 6.0 * M * HD * sizeof(T), st, (attn_bwd_dkv_kernel<T, true>), grid, dim3(256), 0, a);
      else PE_LAUNCH(gm.l_dkv, 8.0 * gm.B * H * gm.L * gm.L * dh, 6.0 * M * HD * sizeof(T), st, (attn_bwd_dkv_kernel<T, false>), grid, dim3(256), 0, a);
      if (c.bias) {
        const long long hll = btile;
        if (hll % 8 == 0 && al16(dS) && al16(dbias))
          PE_LAUNCH("attn_dbias_reduce", 0, 1.0 * Bds * hll * sizeof(T) + 4.0 * hll, st, attn_dbias_reduce8_kernel<T>, dim3((unsigned)((hll / 8 + 63) / 64)), dim3(256), 0,
                    dS, dbias, (int)Bds, hll);
        else
          PE_LAUNCH("attn_dbias_reduce", 0, 1.0 * Bds * hll * sizeof(T) + 4.0 * hll, st, attn_dbias_reduce_kernel<T>, dim3((unsigned)((hll + 255) / 256)), dim3(256), 0, dS, dbias,
                    (int)Bds, hll);
        // dbias is in the chunk order of the query-per-lane bias copy; the fused LayerNorm-backward epilogue gathers from
        // it directly, the kernel of the bias path wants it in pair-row order
        bias_gather = bias_same_ln && gemm_ln_bwd(st, ar, op_heads_rows(dqkvg, gm, dh, M * dh), op_plain(w.wn_qkvg, 4 * HD), M, Cc, 4 * HD, dxh,
                                                  false, x, c.stats, p.ln_g, p.ln_b, g, g, "attn dxhat", dbias, p.w_bias, H, true);
        if (!bias_gather) {
          const int NT = (d.r + 31) / 32;
          PE_LAUNCH("bias_untile", 0, 8.0 * H * Mz, st, bias_untile_kernel<T>, dim3(NT, NT, H), dim3(256), 0, dbias, dbias_rows, d.r,
                    gm.bias_transposed);
        }
      }
    }
    { ReduceSeg sg[4] = {{0, HD, p.w_q, HD}, {HD, HD, p.w_k, HD}, {2 * HD, HD, p.w_v, HD}, {3 * HD, HD, p.w_g, HD}};
      ReduceSeg cb = {3 * HD, HD, p.b_g, 0};
      gemm_dw(st, ar, op_trans(c.xhat, Cc), false, op_heads_cols(dqkvg, gm, dh, M * dh), false, Cc, 4 * HD, M, 4, sg, "attn dWqkvg", 1, &cb); }
    if (bias_gather) { bias_tiled_r = d.r; bias_tiled_transposed = gm.bias_transposed; bias_tiled_plane = btile / H; }
    const bool bias_done = gemm_ln_bwd(st, ar, op_heads_rows(dqkvg, gm, dh, M * dh), op_plain(w.wn_qkvg, 4 * HD), M, Cc, 4 * HD, dxh, false, x,
                                       c.stats, p.ln_g, p.ln_b, g, g, "attn dxhat",
                                       bias_same_ln ? (bias_gather ? dbias : dbias_rows) : nullptr, p.w_bias, c.bias ? H : 0);
    bias_tiled_r = 0;
    if (bias_gather && !bias_done && !err) fail("attn dxhat: the fused launch was announced but not taken");
    next_phase(ar);   // the bias path below adds to the same LayerNorm parameters: a later launch
    if (c.bias && bias_done) end_subop(ar);
    if (c.bias && !bias_done) {
      const int cz = d.c_z;
      const int lpr = (ln_lpr(cz) && ln_lpr(cz) <= 32) ? ln_lpr(cz) : 0;
      const int rpw = lpr ? 64 / lpr : 1;
      int grid = (int)std::min<long long>((Mz + 4 * rpw - 1) / (4 * rpw), 1024);
      int plen = 2 * cz + cz * H;
      float* part = (float*)part_arena(ar).alloc((size_t)grid * plen * sizeof(float));
      if (!dry && !err) {
        const double fl = 4.0 * Mz * cz * H, by = (bias_gin ? 3.0 : 2.0) * Mz * cz * sizeof(T) + 4.0 * Mz * H;
        if (lpr) {
#define PE_LNB_BWD(L, HH) PE_LAUNCH("ln_bias_bwd", fl, by, st, (ln_bias_bwd_fast_kernel<T, L, HH>), dim3(grid), dim3(256), 0, dbias_rows, bias_src, c.zstats, P(bias_ln_g), P(bias_ln_b), P(p.w_bias), bias_gin, bias_gout, part, d.r, H)
#define PE_LNB_BWD_H(L) do { if (H <= 4) PE_LNB_BWD(L, 4); else PE_LNB_BWD(L, 8); } while (0)
          switch (lpr) {
            case 2: PE_LNB_BWD_H(2); break; case 4: PE_LNB_BWD_H(4); break; case 8: PE_LNB_BWD_H(8); break;
            case 16: PE_LNB_BWD_H(16); break; default: PE_LNB_BWD_H(32); break;
          }
#undef PE_LNB_BWD_H
#undef PE_LNB_BWD
        } else {
          PE_LAUNCH("ln_bias_bwd", fl, by, st, ln_bias_bwd_kernel<T>, dim3(grid), dim3(256), 0, dbias_rows, bias_src, c.zstats,
                    P(bias_ln_g), P(bias_ln_b), P(p.w_bias), bias_gin, bias_gout, part, d.r, cz, H, 0);
        }
        ReduceSeg sg[3] = {{0, cz, bias_ln_g, 0}, {cz, cz, bias_ln_b, 0}, {2 * cz, cz * H, p.w_bias, 0}};
        reduce_to(ar, part, grid, plen, 1, plen, 3, sg);
      }
      end_subop(ar);
    }
    ar.release(mk);
  }

  void trimul_sub_bwd(hipStream_t st, Arena& ar, const TriMulP& p, const TriMulW<T>& w, const TriMulCtx<T>& c, const T* z,
                      T* g, bool outgoing) {
    size_t mk = ar.mark();
    const int cz = d.c_z, ct = d.c_tri, r = d.r;
    T* du = (T*)ar.alloc((size_t)Mz * cz * sizeof(T));
    T* dgraw = (T*)ar.alloc((size_t)Mz * cz * sizeof(T));
    T* dxh_o = (T*)ar.alloc((size_t)Mz * ct * sizeof(T));
    T* dx_t = (T*)ar.alloc((size_t)Mz * ct * sizeof(T));
    T* da_t = (T*)ar.alloc((size_t)Mz * ct * sizeof(T));
    T* db_t = (T*)ar.alloc((size_t)Mz * ct * sizeof(T));
    T* dproj_t = (T*)ar.alloc((size_t)Mz * 4 * ct * sizeof(T));
    T* dzh = (T*)ar.alloc((size_t)Mz * cz * sizeof(T));
    if (!dry && !err) {
      long long n = Mz * cz;
      if (n % 8 == 0 && al16(g) && al16(c.g) && al16(c.u) && al16(du) && al16(dgraw))
        PE_LAUNCH("tm_out_bwd", 0, 5.0 * n * sizeof(T), st, tm_out_bwd8_kernel<T>, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, g, c.g, c.u, du, dgraw, n);
      else
        PE_LAUNCH("tm_out_bwd", 0, 5.0 * n * sizeof(T), st, tm_out_bwd_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, g, c.g, c.u, du, dgraw, n);
    }
    { ReduceSeg sg[1] = {{0, cz, p.w_o, cz}}, cb = {0, cz, p.b_o, 0};
      gemm_dw(st, ar, op_trans(c.xhat, ct), false, op_trans(du, cz), false, ct, cz, Mz, 1, sg, "trimul dWo", 1, &cb); }
    { EpiGeneric<T> e = epi_plain<T>(dxh_o, ct);
      gemm(st, op_plain(du, cz), true, op_plain(w.wn_o, cz), true, (int)Mz, ct, cz, 1, e, "trimul dxhat_o"); }
    {  // LayerNorm (channel-major input) backward
      bool lnc_t = false;   // bf16, 64 or 128 channels: the kernel that moves 256-byte runs (128 positions per workgroup)
      if constexpr (std::is_same<T, bf16>::value)
        lnc_t = (ct == 64 || ct == 128) && Mz % 8 == 0 && al16(c.x_t) && al16(dxh_o) && al16(dx_t);
      int grid = lnc_t ? (int)((Mz + 127) / 128) : (int)((Mz + 63) / 64);
      float* part = (float*)part_arena(ar).alloc((size_t)grid * 2 * ct * sizeof(float));
      if (!dry && !err && lnc_t) {
        if constexpr (std::is_same<T, bf16>::value) {
          if (ct == 128)
            PE_LAUNCH("ln_cmajor_bwd", 0, 3.0 * Mz * ct * sizeof(T), st, ln_cmajor_bwd_t_kernel<16>, dim3(grid), dim3(256), 0, dxh_o, c.x_t, c.stats_out,
                      P(p.ln_out_g), dx_t, part, Mz);
          else
            PE_LAUNCH("ln_cmajor_bwd", 0, 3.0 * Mz * ct * sizeof(T), st, ln_cmajor_bwd_t_kernel<8>, dim3(grid), dim3(256), 0, dxh_o, c.x_t, c.stats_out,
                      P(p.ln_out_g), dx_t, part, Mz);
          ReduceSeg sg[2] = {{0, ct, p.ln_out_g, 0}, {ct, ct, p.ln_out_b, 0}};
          reduce_to(ar, part, grid, 2LL * ct, 1, 2 * ct, 2, sg);
        }
      }
      if (!dry && !err && !lnc_t) {
        size_t lds = (size_t)64 * (ct + 1) * sizeof(float);
#define PE_LNC_BWD(N) PE_LAUNCH("ln_cmajor_bwd", 0, 3.0 * Mz * ct * sizeof(T), st, (ln_cmajor_bwd_fast_kernel<T, N>), dim3(grid), dim3(256), lds, dxh_o, c.x_t, c.stats_out, P(p.ln_out_g), dx_t, part, Mz, ct)
        if (Mz % 4 == 0 && ct % 8 == 0) {
          const int nit = (ct + 15) / 16;   // c_tri <= 192
          if (nit <= 2) PE_LNC_BWD(2); else if (nit <= 4) PE_LNC_BWD(4); else if (nit <= 8) PE_LNC_BWD(8); else PE_LNC_BWD(12);
        }
#undef PE_LNC_BWD
        else
          PE_LAUNCH("ln_cmajor_bwd", 0, 3.0 * Mz * ct * sizeof(T), st, ln_cmajor_bwd_kernel<T>, dim3(grid), dim3(256), lds, dxh_o, c.x_t, c.stats_out,
                    P(p.ln_out_g), dx_t, part, Mz, ct);
        ReduceSeg sg[2] = {{0, ct, p.ln_out_g, 0}, {ct, ct, p.ln_out_b, 0}};
        reduce_to(ar, part, grid, 2LL * ct, 1, 2 * ct, 2, sg);
      }
    }
    // contraction backward, per channel; where the vector path applies the gating backward is the epilogue of these
    // GEMMs (da_t / db_t are never stored), else they are followed by the gating kernel
    bool gate_fused = false;
    {
      Operand A1, B1, A2, B2;
      bool a1k, b1k, a2k, b2k;
      if (outgoing) {
        A1 = op_plain(dx_t, r, Mz); a1k = true; B1 = op_trans(c.b_t, r, Mz); b1k = false;
        A2 = op_trans(dx_t, r, Mz); a2k = false; B2 = op_trans(c.a_t, r, Mz); b2k = false;
      } else {
        A1 = op_plain(c.b_t, r, Mz); a1k = true; B1 = op_plain(dx_t, r, Mz); b1k = true;
        A2 = op_plain(c.a_t, r, Mz); a2k = true; B2 = op_trans(dx_t, r, Mz); b2k = false;
      }
      EpiTmGateBwd<T> ga;
      ga.proj_t = c.proj_t; ga.mask = pair_mask; ga.dproj_t = dproj_t; ga.ct = ct; ga.r = r; ga.side = 0; ga.Mz = Mz;
      EpiTmGateBwd<T> gb = ga;
      gb.side = 1;
      GemmShape sh{r, r, r, ct, 0, 0};
      if (!dry && !err && ga.vec_ok(r) && gemm_operand_ok<T>(A1, a1k, r, sh) && gemm_operand_ok<T>(B1, b1k, r, sh) &&
          gemm_operand_ok<T>(A2, a2k, r, sh) && gemm_operand_ok<T>(B2, b2k, r, sh)) {
        gate_fused = true;
        const double fl = 2.0 * r * r * r * ct, by = (2.0 * r * r + 5.0 * r * r) * ct * sizeof(T);
        prof_begin(st);
        int rc = launch_gemm<T, EpiTmGateBwd<T>>(st, A1, a1k, B1, b1k, sh, ga);
        prof_end(st, "trimul da+gate", a1k && b1k ? "gemm_kernel<kc,kc,vec,EpiTmGateBwd>" : "gemm_kernel<kc,xc,vec,EpiTmGateBwd>", fl, by);
        if (rc == -1) { err = PE_ERR_DIMS; if (h) h->last_error = "gemm operand alignment: trimul da+gate"; }
        else check("trimul da+gate");
        if (!err) {
          prof_begin(st);
          rc = launch_gemm<T, EpiTmGateBwd<T>>(st, A2, a2k, B2, b2k, sh, gb);
          prof_end(st, "trimul db+gate", a2k ? "gemm_kernel<kc,xc,vec,EpiTmGateBwd>" : "gemm_kernel<xc,xc,vec,EpiTmGateBwd>", fl, by);
          if (rc == -1) { err = PE_ERR_DIMS; if (h) h->last_error = "gemm operand alignment: trimul db+gate"; }
          else check("trimul db+gate");
        }
      }
    }
    if (!gate_fused) {
      EpiGeneric<T> ea = epi_plain<T>(da_t, r); ea.out_batch = Mz;
      EpiGeneric<T> eb = epi_plain<T>(db_t, r); eb.out_batch = Mz;
      if (outgoing) {
        // da[i,k] = sum_j dx[i,j] b[j,k];  db[j,k] = sum_i dx[i,j] a[i,k]
        gemm(st, op_plain(dx_t, r, Mz), true, op_trans(c.b_t, r, Mz), false, r, r, r, ct, ea, "trimul da");
        gemm(st, op_trans(dx_t, r, Mz), false, op_trans(c.a_t, r, Mz), false, r, r, r, ct, eb, "trimul db");
      } else {
        // da[k,i] = sum_j b[k,j] dx[i,j];  db[k,j] = sum_i a[k,i] dx[i,j]
        gemm(st, op_plain(c.b_t, r, Mz), true, op_plain(dx_t, r, Mz), true, r, r, r, ct, ea, "trimul da");
        gemm(st, op_plain(c.a_t, r, Mz), true, op_trans(dx_t, r, Mz), false, r, r, r, ct, eb, "trimul db");
      }
    }
    if (!dry && !err && !gate_fused) {
      long long n = (long long)ct * Mz;
      if (Mz % 8 == 0 && al16(c.proj_t) && al16(pair_mask) && al16(da_t) && al16(db_t) && al16(dproj_t))
        PE_LAUNCH("tm_gate_bwd", 0, 10.0 * n * sizeof(T), st, tm_gate_bwd8_kernel<T>, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, c.proj_t,
                  pair_mask, da_t, db_t, dproj_t, ct, Mz);
      else
        PE_LAUNCH("tm_gate_bwd", 0, 10.0 * n * sizeof(T), st, tm_gate_bwd_kernel<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c.proj_t, pair_mask,
                  da_t, db_t, dproj_t, ct, Mz);
    }
    { ReduceSeg sg[4] = {{0, ct, p.w_ap, ct}, {ct, ct, p.w_ag, ct}, {2 * ct, ct, p.w_bp, ct}, {3 * ct, ct, p.w_bg, ct}};
      ReduceSeg cb[4] = {{0, ct, p.b_ap, 0}, {ct, ct, p.b_ag, 0}, {2 * ct, ct, p.b_bp, 0}, {3 * ct, ct, p.b_bg, 0}};
      gemm_dw(st, ar, op_trans(c.zhat, cz), false, op_plain(dproj_t, Mz), true, cz, 4 * ct, Mz, 4, sg, "trimul dWp", 4, cb); }
    { ReduceSeg sg[1] = {{0, cz, p.w_g, cz}}, cb = {0, cz, p.b_g, 0};
      gemm_dw(st, ar, op_trans(c.zhat, cz), false, op_trans(dgraw, cz), false, cz, cz, Mz, 1, sg, "trimul dWg", 1, &cb); }
    { EpiGeneric<T> e = epi_plain<T>(dzh, cz);
      gemm(st, op_trans(dproj_t, Mz), false, op_plain(w.wn_p, 4 * ct), true, (int)Mz, cz, 4 * ct, 1, e, "trimul dzhat p"); }
    gemm_ln_bwd(st, ar, op_plain(dgraw, cz), op_plain(w.wn_g, cz), Mz, cz, cz, dzh, true, z, c.stats, p.ln_in_g, p.ln_in_b, g, g,
                "trimul dzhat g");
    end_subop(ar);
    ar.release(mk);
  }

  // MSA side backward.  gm_out receives d_msa_in; dz_bias receives the row-attention-bias
  // term of d_pair_in.
  void bwd_msa(const T* d_msa_out, const T* d_pair_out, T* gm, T* dz_bias) {
    bwd_opm(d_pair_out, C.m3, d_msa_out, gm);
    bwd_msa_stack(gm, pair_in, dz_bias);
  }
  // outer product mean backward: dz = cotangent of its output, x = the MSA tensor it read;
  // gout = gin + gradient w.r.t. x
  void bwd_opm(const T* d_pair_out, const T* x, const T* gin, T* gout) {
    const int co = d.c_opm, r = d.r, cm = d.c_m, cz = d.c_z;
    const long long Wd = (long long)r * co;
    {
      size_t mk = am.mark();
      T* dOs = (T*)am.alloc((size_t)Wd * Wd * sizeof(T));
      T* dab = (T*)am.alloc((size_t)2 * Mm * co * sizeof(T));
      T* dmh = (T*)am.alloc((size_t)Mm * cm * sizeof(T));
      {
        Operand X;   // rows (p,q), contraction (i,j) over O[(i,p),(j,q)]
        X.ptr = C.opm.O; X.batch_stride = 0;
        X.x_in = co; X.x_outer = Wd; X.x_stride = 1;
        X.k_in = r; X.k_outer = (long long)co * Wd; X.k_stride = co;
        ReduceSeg sg[1] = {{0, cz, PL.opm.w_o, cz}}, cb = {0, cz, PL.opm.b_o, 0};
        gemm_dw(sm, am, X, false, op_trans(d_pair_out, cz), false, co * co, cz, Mz, 1, sg, "opm dWo", 1, &cb);
      }
      {
        EpiGeneric<T> e = epi_plain<T>(dOs, Wd);
        e.om_in = r; e.om_outer = (long long)co * Wd; e.om_stride = co;
        e.on_in = co; e.on_outer = Wd; e.on_stride = 1;
        e.rowscale = C.opm.inv_norm;
        gemm(sm, op_plain(d_pair_out, cz), true, op_plain(W.opm.wn_o, cz), true, (int)Mz, co * co, cz, 1, e, "opm dO");
      }
      {
        EpiGeneric<T> e = epi_plain<T>(dab, Wd);
        e.scale2d = msa_mask; e.s2_mdiv = 1; e.s2_ndiv = co; e.s2_ld = r;
        gemm(sm, op_plain(C.opm.b, Wd), true, op_plain(dOs, Wd), true, d.s, (int)Wd, (int)Wd, 1, e, "opm da", &am);
        EpiGeneric<T> e2 = e;
        e2.out = dab + Mm * co;
        gemm(sm, op_plain(C.opm.a, Wd), true, op_trans(dOs, Wd), false, d.s, (int)Wd, (int)Wd, 1, e2, "opm db", &am);
      }
      {
        Operand Y;   // rows n = (which, c), contraction over MSA positions
        Y.ptr = dab; Y.batch_stride = 0;
        Y.x_in = co; Y.x_outer = Mm * co; Y.x_stride = 1;
        Y.k_in = 1 << 30; Y.k_outer = 0; Y.k_stride = co;
        ReduceSeg sg[2] = {{0, co, PL.opm.w_a, co}, {co, co, PL.opm.w_b, co}};
        ReduceSeg cb[2] = {{0, co, PL.opm.b_a, 0}, {co, co, PL.opm.b_b, 0}};
        gemm_dw(sm, am, op_trans(C.opm.mhat, cm), false, Y, false, cm, 2 * co, Mm, 2, sg, "opm dWab", 2, cb);
      }
      {
        Operand A;   // [Mm][2co] view of the two gradient halves
        A.ptr = dab; A.batch_stride = 0;
        A.x_in = 1 << 30; A.x_outer = 0; A.x_stride = co;
        A.k_in = co; A.k_outer = Mm * co; A.k_stride = 1;
        gemm_ln_bwd(sm, am, A, op_plain(W.opm.wn_ab, 2 * co), Mm, cm, 2 * co, dmh, false, x, C.opm.stats, PL.opm.ln_g, PL.opm.ln_b, gin,
                    gout, "opm dmhat");
      }
      end_subop(am);
      am.release(mk);
    }
  }
  // MSA stack backward, in place on gm; dz_bias receives the gradient through the row-attention bias
  void bwd_msa_step(int i, T* gm, const T* bias_pair, T* dz_bias) {
    const int cm = d.c_m;
    if (i == 0) {
      trans_sub_bwd(sm, am, PL.mtrans, W.mt, C.mt, C.m2, gm, Mm, cm);
    } else if (i == 1) {
      if (d.col_global) gcol_sub_bwd(sm, am, C.m1, gm);
      else attn_sub_bwd(sm, am, PL.col, W.col, C.col, C.m1, gm, Mm, cm, d.h_msa, d.d_msa, geom_col(), nullptr, 0, 0, nullptr, nullptr);
    } else {
      attn_sub_bwd(sm, am, PL.row, W.row, C.row, msa_in, gm, Mm, cm, d.h_msa, d.d_msa, geom_row(), bias_pair, PL.row.ln_z_g,
                   PL.row.ln_z_b, nullptr, dz_bias);
    }
  }
  void bwd_msa_stack(T* gm, const T* bias_pair, T* dz_bias) {
    for (int i = 0; i < MSA_STEPS; i++) bwd_msa_step(i, gm, bias_pair, dz_bias);
  }
  void bwd_pair(const T* d_pair_out, T* gz) { bwd_pair_stack(d_pair_out, gz, pair_in); }
  void bwd_pair_step(int i, const T* d_pair_out, T* gz, const T* z_in) {
    switch (i) {
      case 0:
        // the running pair gradient gz starts as the output cotangent: read in place, no copy
        trans_sub_bwd(sp, ap, PL.ptrans, W.pt, C.pt, C.z4, gz, Mz, d.c_z, d_pair_out);
        break;
      case 1: attn_sub_bwd(sp, ap, PL.tae, W.tae, C.tae, C.z3, gz, Mz, d.c_z, d.h_pair, d.d_pair, geom_tae(), C.z3,
                           PL.tae.ln_g, PL.tae.ln_b, gz, gz); break;
      case 2: attn_sub_bwd(sp, ap, PL.tas, W.tas, C.tas, C.z2, gz, Mz, d.c_z, d.h_pair, d.d_pair, geom_tas(), C.z2,
                           PL.tas.ln_g, PL.tas.ln_b, gz, gz); break;
      case 3: trimul_sub_bwd(sp, ap, PL.tmi, W.tmi, C.tmi, C.z1, gz, false); break;
      default: trimul_sub_bwd(sp, ap, PL.tmo, W.tmo, C.tmo, z_in, gz, true); break;
    }
  }
  void bwd_pair_stack(const T* d_pair_out, T* gz, const T* z_in) {
    for (int i = 0; i < PAIR_STEPS; i++) bwd_pair_step(i, d_pair_out, gz, z_in);
  }

  // The two stacks side by side, enqueued alternately (pair first: it is the longer one).
  // with_opm: the outer product mean of the MSA stack's output follows the stack on stream_msa.
  void fwd_stacks(bool do_m, bool do_p, const T* bias_pair, const T* z_in, T* msa_out, T* z_out, bool with_opm) {
    for (int i = 0; i < PAIR_STEPS; i++) {
      if (do_p) fwd_pair_step(i, z_in, z_out);
      if (do_m && i < MSA_STEPS) fwd_msa_step(i, bias_pair, msa_out);
      if (do_m && i == MSA_STEPS && with_opm) fwd_opm_outer(C.m3);
    }
  }
  void bwd_stacks(bool do_m, bool do_p, const T* d_pair_out, T* gz, const T* z_in, T* gm, const T* bias_pair, T* dz_bias) {
    for (int i = 0; i < PAIR_STEPS; i++) {
      if (do_p) bwd_pair_step(i, d_pair_out, gz, z_in);
      if (do_m && i < MSA_STEPS) bwd_msa_step(i, gm, bias_pair, dz_bias);
    }
  }
};

// ---------------------------------------------------------------------------
// Plans: workspace layout = [MSA arena | pair arena | internal ctx]; a ctx (the caller's or the
// internal one) = [saved activations | prepared weights], so that a backward pass that gets the
// forward's ctx does not convert the parameters again
// ---------------------------------------------------------------------------
struct Plan {
  size_t prep_bytes, arena_m, arena_p, part_m, part_p, ctx_bytes;
  size_t ctx_total() const { return ctx_bytes + prep_bytes; }
  size_t arenas() const { return arena_m + arena_p + part_m + part_p; }
  size_t total(bool with_ctx) const { return arenas() + (with_ctx ? ctx_total() : 0) + 1024; }
};

template <typename T> static Plan make_plan(const pe_dims& d) {
  Runner<T> R;
  R.h = nullptr;
  R.init(d);
  R.dry = true;
  Plan pl;
  R.am.base = R.ap.base = R.pm.base = R.pp.base = kDryBase;
  R.params = reinterpret_cast<const float*>(kDryBase);
  R.dparams = reinterpret_cast<float*>(kDryBase);
  R.msa_in = reinterpret_cast<const T*>(kDryBase);
  R.pair_in = reinterpret_cast<const T*>(kDryBase);
  R.msa_mask = R.pair_mask = reinterpret_cast<const float*>(kDryBase);
  pl.ctx_bytes = carve_ctx<T>(kDryBase, d, R.C, nullptr);
  pl.prep_bytes = R.carve_prep(kDryBase);
  // forward needs z5-independent scratch only from ctx; backward uses the arenas
  R.fwd_msa(nullptr);
  R.fwd_opm_project(nullptr, nullptr);
  R.fwd_pair();
  T* gm = (T*)R.am.alloc((size_t)R.Mm * d.c_m * sizeof(T));
  T* dzb = (T*)R.am.alloc((size_t)R.Mz * d.c_z * sizeof(T));
  R.bwd_msa(nullptr, nullptr, gm, dzb);
  T* gz = (T*)R.ap.alloc((size_t)R.Mz * d.c_z * sizeof(T));
  R.bwd_pair(nullptr, gz);
  pl.arena_m = (R.am.high + 255) & ~(size_t)255;
  pl.arena_p = (R.ap.high + 255) & ~(size_t)255;
  pl.part_m = (R.pm.high + 255) & ~(size_t)255;
  pl.part_p = (R.pp.high + 255) & ~(size_t)255;
  return pl;
}
static Plan plan_for(const pe_dims& d) { return d.dtype == PE_BF16 ? make_plan<bf16>(d) : make_plan<float>(d); }

template <typename T> static void setup_runner(Runner<T>& R, pe_handle* h, const pe_dims& d, const Plan& pl, char* ws,
                                               char* ctx, hipStream_t sm, hipStream_t sp) {
  R.h = h;
  R.init(d);
  R.sm = sm;
  R.sp = sp;
  R.am.base = ws;
  R.ap.base = ws + pl.arena_m;
  R.pm.base = ws + pl.arena_m + pl.arena_p;
  R.pp.base = R.pm.base + pl.part_m;
  char* cbase = ctx ? ctx : ws + pl.arenas();
  carve_ctx<T>(cbase, d, R.C, nullptr);
  R.carve_prep(cbase + pl.ctx_bytes);
}

static bool hip_ok(pe_handle* h, hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  if (h) h->last_error = std::string(what) + ": " + hipGetErrorString(e);
  return false;
}

// `to` waits for everything queued on `from` so far
static bool ev_link(pe_handle* h, int e, hipStream_t from, hipStream_t to) {
  if (from == to) return true;
  return hip_ok(h, hipEventRecord(h->ev[e], from), "event record") && hip_ok(h, hipStreamWaitEvent(to, h->ev[e], 0), "stream wait");
}

// Forward schedule of one block (Figure 1).  At entry stream_pair has been forked from stream_msa.
// msa_out / pair_out may be null (recompute inside the backward pass: only ctx is needed).  On
// return every forward kernel is ordered before later work on BOTH streams.
// early_next (nullable): called when everything of this block that stream_msa can do before it has to wait for
// the pair branch is enqueued; the trunk uses it to enqueue the first kernels of the next block there
template <typename T>
static int run_forward(Runner<T>& R, pe_handle* h, const pe_dims& d, T* msa_out, T* pair_out,
                       const std::function<int()>* early_next = nullptr) {
  hipStream_t sm = R.sm, sp = R.sp;
  const bool do_m = h->branches & 1, do_p = h->branches & 2;
  if (d.variant == PE_VARIANT_PARALLEL) {
    if (do_p) R.run_prep(false);
    if (do_m && !R.row_pre_done) R.run_prep(true);
    R.fwd_stacks(do_m, do_p, R.pair_in, R.pair_in, msa_out, R.C.z5, true);
    if (early_next && *early_next) { int rc = (*early_next)(); if (rc) return rc; }
    if (do_p && !ev_link(h, 1, sp, sm)) return PE_ERR_HIP;
    if (pair_out) {
      if (do_m && do_p) R.fwd_opm_project(pair_out, R.C.z5);
      else if (do_p && !R.err) {
        if (!hip_ok(h, hipMemcpyAsync(pair_out, R.C.z5, (size_t)R.Mz * d.c_z * sizeof(T), hipMemcpyDeviceToDevice, sm),
                    "copy pair_out")) return PE_ERR_HIP;
      }
    }
    if (!ev_link(h, 2, sm, sp)) return PE_ERR_HIP;
    return R.err;
  }
  R.run_prep(true);
  R.run_prep(false);
  T* z_out = pair_out ? pair_out : R.C.z5;
  if (d.variant == PE_VARIANT_AF2) {
    // MSA stack -> outer product mean of its output added to the pair input -> pair stack
    R.fwd_msa_stack(R.pair_in, msa_out);
    R.fwd_opm_outer(R.C.m3);
    R.fwd_opm_project(R.C.z0, R.pair_in);
    if (!ev_link(h, 1, sm, sp)) return PE_ERR_HIP;
    R.fwd_pair_stack(R.C.z0, z_out);
    if (!ev_link(h, 2, sp, sm)) return PE_ERR_HIP;
  } else {
    // outer product mean of the input MSA added to the pair input, then the two stacks side by side
    R.fwd_opm_outer(R.msa_in);
    R.fwd_opm_project(R.C.z0, R.pair_in);
    if (!ev_link(h, 1, sm, sp)) return PE_ERR_HIP;
    R.fwd_stacks(true, true, R.C.z0, R.C.z0, msa_out, z_out, false);
    if (!ev_link(h, 2, sp, sm)) return PE_ERR_HIP;
    if (!ev_link(h, 3, sm, sp)) return PE_ERR_HIP;
  }
  return R.err;
}

template <typename T>
static int block_fwd_impl(pe_handle* h, const pe_dims& d, const void* msa_in, const void* pair_in, const float* msa_mask,
                          const float* pair_mask, const float* params, void* msa_out, void* pair_out, void* ctx,
                          void* workspace, size_t wbytes, hipStream_t sm, hipStream_t sp, bool row_pre_done = false,
                          const std::function<int()>* early_next = nullptr) {
  Plan pl = plan_for(d);
  if (wbytes < pl.total(ctx == nullptr)) return PE_ERR_WORKSPACE;
  if (d.variant != PE_VARIANT_PARALLEL && h->branches != 3) return PE_ERR_ARG;
  Runner<T> R;
  setup_runner<T>(R, h, d, pl, (char*)workspace, (char*)ctx, sm, sp);
  R.params = params;
  R.msa_in = (const T*)msa_in; R.pair_in = (const T*)pair_in;
  R.msa_mask = msa_mask; R.pair_mask = pair_mask;
  R.row_pre_done = row_pre_done;
  if (!ev_link(h, 0, sm, sp)) return PE_ERR_HIP;
  return run_forward<T>(R, h, d, (T*)msa_out, (T*)pair_out, early_next);
}

// The part of a block's forward that depends on its MSA input alone (weights of the MSA branch into their
// storage form, LayerNorm and q / k / v / gate projection of the row attention), enqueued on stream_msa.  ctx
// is the block's own (kept) ctx: nothing of it is shared with the block that is still running.
template <typename T>
static int block_fwd_row_pre(pe_handle* h, const pe_dims& d, const void* msa_in, const float* msa_mask, const float* params,
                             void* ctx, void* workspace, hipStream_t sm, hipStream_t sp) {
  Plan pl = plan_for(d);
  Runner<T> R;
  setup_runner<T>(R, h, d, pl, (char*)workspace, (char*)ctx, sm, sp);
  R.params = params;
  R.msa_in = (const T*)msa_in;
  R.msa_mask = msa_mask;
  R.fwd_row_pre();
  return R.err;
}

template <typename T>
static int block_bwd_impl(pe_handle* h, const pe_dims& d, const void* msa_in, const void* pair_in, const float* msa_mask,
                          const float* pair_mask, const float* params, const void* d_msa_out, const void* d_pair_out,
                          void* d_msa_in, void* d_pair_in, float* d_params, const void* ctx, void* workspace,
                          size_t wbytes, hipStream_t sm, hipStream_t sp) {
  Plan pl = plan_for(d);
  if (wbytes < pl.total(ctx == nullptr)) return PE_ERR_WORKSPACE;
  if (d.variant != PE_VARIANT_PARALLEL && h->branches != 3) return PE_ERR_ARG;
  const bool do_m = h->branches & 1, do_p = h->branches & 2;
  Runner<T> R;
  setup_runner<T>(R, h, d, pl, (char*)workspace, (char*)ctx, sm, sp);
  R.params = params; R.dparams = d_params;
  R.msa_in = (const T*)msa_in; R.pair_in = (const T*)pair_in;
  R.msa_mask = msa_mask; R.pair_mask = pair_mask;
  if (!ev_link(h, 0, sm, sp)) return PE_ERR_HIP;
  if (ctx == nullptr) {   // recompute the forward into the internal ctx (else: ctx also holds the prepared weights)
    if (d.variant == PE_VARIANT_PARALLEL) {
      if (do_p) R.run_prep(false);
      if (do_m) R.run_prep(true);
      R.fwd_stacks(do_m, do_p, R.pair_in, R.pair_in, nullptr, R.C.z5, true);   // the projection is not needed here
    } else {
      int rc = run_forward<T>(R, h, d, nullptr, nullptr);
      if (rc) return rc;
    }
  }
  const long long n = R.Mz * d.c_z;
  T* dzb = (T*)R.am.alloc((size_t)n * sizeof(T));
  T* gz = (T*)R.ap.alloc((size_t)n * sizeof(T));
  T* gm = (T*)d_msa_in;
  if (d.variant == PE_VARIANT_PARALLEL) {
    if (do_p) R.bwd_pair_step(0, (const T*)d_pair_out, gz, R.pair_in);
    if (do_m) R.bwd_opm((const T*)d_pair_out, R.C.m3, (const T*)d_msa_out, gm);
    // The MSA branch finishes first.  The reductions of all pair sub-operations but the last are therefore handed
    // to stream_msa (after its own), which waits for the event recorded here: they then run beside the pair
    // branch's last sub-operation instead of after it.
    const bool hand_over = do_m && do_p && sm != sp && !h->side_streams;
    for (int i = 1; i < Runner<T>::PAIR_STEPS; i++) {
      // the last pair sub-operation's last kernel also adds the row-attention-bias term and writes d_pair_in
      // (every MSA-side step is enqueued by then: the MSA stack has fewer steps)
      if (do_p && do_m && i == Runner<T>::PAIR_STEPS - 1) {
        R.fin_add = dzb; R.fin_out = (T*)d_pair_in; R.fin_from = sm; R.fin_ev = h->ev[1];
      }
      if (do_p) R.bwd_pair_step(i, (const T*)d_pair_out, gz, R.pair_in);
      R.fin_add = nullptr;
      if (hand_over && i == Runner<T>::PAIR_STEPS - 2) {
        R.mark_early(R.ap);
        if (!R.err && !hip_ok(h, hipEventRecord(h->ev[4], sp), "event record")) return PE_ERR_HIP;
      }
      if (do_m && i - 1 < Runner<T>::MSA_STEPS) R.bwd_msa_step(i - 1, gm, R.pair_in, dzb);
    }
    if (do_m && !R.fin_done && !ev_link(h, 1, sm, sp)) return PE_ERR_HIP;
    if (!R.err) {
      if (do_m && do_p) {
        if (!R.fin_done) {
          launch_add2<T>(sp, gz, dzb, (T*)d_pair_in, n);
          R.check("add d_pair_in");
        }
      } else if (do_p) {
        if (!hip_ok(h, hipMemcpyAsync(d_pair_in, gz, (size_t)n * sizeof(T), hipMemcpyDeviceToDevice, sp), "copy")) return PE_ERR_HIP;
      } else if (do_m) {
        if (!hip_ok(h, hipMemcpyAsync(d_pair_in, dzb, (size_t)n * sizeof(T), hipMemcpyDeviceToDevice, sp), "copy")) return PE_ERR_HIP;
      }
    }
    // the queued parameter-gradient reductions of both branches, each on its own stream; then both streams wait
    // for each other
    R.flush_all(R.am, sm);
    if (hand_over && !R.err && !hip_ok(h, hipStreamWaitEvent(sm, h->ev[4], 0), "stream wait")) return PE_ERR_HIP;
    R.flush_all(R.ap, sp, hand_over ? sm : nullptr);
    if (!ev_link(h, 2, sp, sm)) return PE_ERR_HIP;
    if (!ev_link(h, 3, sm, sp)) return PE_ERR_HIP;
    return R.err;
  }
  if (d.variant == PE_VARIANT_AF2) {
    // pair stack -> outer product mean (cotangent = the pair stack's input gradient) -> MSA stack
    R.bwd_pair_stack((const T*)d_pair_out, gz, R.C.z0);
    if (!ev_link(h, 1, sp, sm)) return PE_ERR_HIP;
    R.bwd_opm(gz, R.C.m3, (const T*)d_msa_out, gm);
    R.bwd_msa_stack(gm, R.pair_in, dzb);
    if (!R.err) {
      launch_add2<T>(sm, gz, dzb, (T*)d_pair_in, n);
      R.check("add d_pair_in");
    }
  } else {
    // both stacks side by side; their two gradients w.r.t. (pair input + outer product mean) are
    // summed, and that sum is also the cotangent of the outer product mean of the input MSA
    if (!R.err && !hip_ok(h, hipMemcpyAsync(gm, d_msa_out, (size_t)R.Mm * d.c_m * sizeof(T), hipMemcpyDeviceToDevice, sm), "copy"))
      return PE_ERR_HIP;
    R.bwd_stacks(true, true, (const T*)d_pair_out, gz, R.C.z0, gm, R.C.z0, dzb);
    if (!ev_link(h, 1, sp, sm)) return PE_ERR_HIP;
    if (!R.err) {
      launch_add2<T>(sm, gz, dzb, (T*)d_pair_in, n);
      R.check("add d_pair_in");
    }
    R.bwd_opm((const T*)d_pair_in, R.msa_in, gm, gm);
  }
  R.flush_all(R.ap, sp);
  R.flush_all(R.am, sm);
  if (!ev_link(h, 3, sp, sm)) return PE_ERR_HIP;
  if (!ev_link(h, 2, sm, sp)) return PE_ERR_HIP;
  return R.err;
}


// ---------------------------------------------------------------------------
// Stack (trunk): saved block inputs + recompute in the backward pass
// ---------------------------------------------------------------------------
struct StackPlan {
  size_t E;
  size_t n_pair, n_msa, n_extra;        // bytes of one pair / msa / extra-msa tensor
  size_t off_pair_saved, off_msa_saved, off_extra_saved, off_pp, off_block, block_bytes, total;
  bool keep;                            // every block's ctx is kept: nothing is recomputed
  size_t off_ctx, ctx_e, ctx_m;         // kept ctx slots: n_extra of ctx_e bytes, then n_main of ctx_m bytes
};
static size_t al256(size_t v) { return (v + 255) & ~(size_t)255; }
static int make_stack_plan(int n_extra, const pe_dims* ex, int n_main, const pe_dims* mn, bool keep, StackPlan& sp) {
  if (n_extra < 0 || n_main < 0 || n_extra + n_main < 1) return PE_ERR_ARG;
  if ((n_extra && !ex) || (n_main && !mn)) return PE_ERR_NULL;
  if (n_extra && pe_check_dims(ex)) return PE_ERR_DIMS;
  if (n_main && pe_check_dims(mn)) return PE_ERR_DIMS;
  if (n_extra && n_main && (ex->r != mn->r || ex->c_z != mn->c_z || ex->dtype != mn->dtype)) return PE_ERR_DIMS;
  const pe_dims* any = n_main ? mn : ex;
  sp.E = any->dtype == PE_BF16 ? 2 : 4;
  sp.n_pair = al256((size_t)any->r * any->r * any->c_z * sp.E);
  sp.n_msa = n_main ? al256((size_t)mn->s * mn->r * mn->c_m * sp.E) : 0;
  sp.n_extra = n_extra ? al256((size_t)ex->s * ex->r * ex->c_m * sp.E) : 0;
  int nb = n_extra + n_main;
  size_t off = 0;
  sp.off_pair_saved = off; off += sp.n_pair * (size_t)(nb - 1);
  sp.off_msa_saved = off; off += sp.n_msa * (size_t)(n_main > 0 ? n_main - 1 : 0);
  sp.off_extra_saved = off; off += sp.n_extra * (size_t)n_extra;     // slot n_extra-1 = dropped final output
  sp.off_pp = off; off += 2 * (sp.n_pair + sp.n_msa + sp.n_extra);   // ping-pong cotangents
  sp.keep = keep;
  Plan pe_ = n_extra ? plan_for(*ex) : Plan{0, 0, 0, 0}, pm_ = n_main ? plan_for(*mn) : Plan{0, 0, 0, 0};
  sp.ctx_e = al256(pe_.ctx_total());
  sp.ctx_m = al256(pm_.ctx_total());
  sp.off_ctx = off;
  if (keep) off += sp.ctx_e * (size_t)n_extra + sp.ctx_m * (size_t)n_main;
  sp.off_block = off;
  size_t be = n_extra ? pe_.total(!keep) : 0, bm = n_main ? pm_.total(!keep) : 0;
  sp.block_bytes = al256(be > bm ? be : bm);
  sp.total = off + sp.block_bytes;
  return PE_OK;
}

template <typename T>
static int stack_impl(pe_handle* h, int n_extra, const pe_dims* ex, int n_main, const pe_dims* mn, const StackPlan& sp,
                      const void* extra_msa_in, const void* msa_in, const void* pair_in, const float* extra_mask,
                      const float* msa_mask, const float* pair_mask, const float* params, const void* d_msa_out,
                      const void* d_pair_out, void* msa_out, void* pair_out, void* d_extra_msa_in, void* d_msa_in,
                      void* d_pair_in, float* d_params, char* ws, hipStream_t sm, hipStream_t sp_) {
  const int nb = n_extra + n_main;
  const long long pe_n = n_extra ? pe_param_count(ex) : 0, pm_n = n_main ? pe_param_count(mn) : 0;
  char* blockws = ws + sp.off_block;
  auto pair_slot = [&](int b) -> char* { return ws + sp.off_pair_saved + sp.n_pair * (size_t)(b - 1); };   // input of block b>=1
  auto x_in = [&](int b) -> const void* {
    if (b < n_extra) return b == 0 ? extra_msa_in : (const void*)(ws + sp.off_extra_saved + sp.n_extra * (size_t)(b - 1));
    int k = b - n_extra;
    return k == 0 ? msa_in : (const void*)(ws + sp.off_msa_saved + sp.n_msa * (size_t)(k - 1));
  };
  auto z_in = [&](int b) -> const void* { return b == 0 ? pair_in : (const void*)pair_slot(b); };
  auto poff = [&](int b) -> long long { return b < n_extra ? pe_n * b : pe_n * n_extra + pm_n * (b - n_extra); };
  auto ctx_of = [&](int b) -> char* {
    if (!sp.keep) return nullptr;
    return ws + sp.off_ctx + (b < n_extra ? sp.ctx_e * (size_t)b : sp.ctx_e * (size_t)n_extra + sp.ctx_m * (size_t)(b - n_extra));
  };
  // forward.  Cross-block overlap: a block's MSA representation is final before its outer product mean and before
  // the pair branch has finished, and the next block's row attention needs the new pair representation only for
  // its bias.  So, when every block has a ctx of its own (PE_OPT_STACK_KEEP_CTX) and the branches run on two
  // streams, the next block's MSA-side weight preparation, LayerNorm and q / k / v / gate projection are enqueued
  // on stream_msa right after this block's outer product, in the time that stream would otherwise spend waiting
  // for the pair branch.  The same kernels run on the same data, so results are bit-identical.
  const bool overlap_blocks = sp.keep && h->stack_overlap && sm != sp_;
  bool pre_done = false;
  for (int b = 0; b < nb; b++) {
    const bool is_e = b < n_extra;
    const pe_dims& d = is_e ? *ex : *mn;
    void* xo;
    if (is_e) xo = ws + sp.off_extra_saved + sp.n_extra * (size_t)b;
    else xo = (b == nb - 1) ? msa_out : (void*)(ws + sp.off_msa_saved + sp.n_msa * (size_t)(b - n_extra));
    void* zo = (b == nb - 1) ? pair_out : (void*)pair_slot(b + 1);
    const bool chain = overlap_blocks && b + 1 < nb && d.variant == PE_VARIANT_PARALLEL &&
                       (b + 1 < n_extra ? ex : mn)->variant == PE_VARIANT_PARALLEL;
    std::function<int()> early = [&, b]() -> int {
      const bool ne = b + 1 < n_extra;
      return block_fwd_row_pre<T>(h, ne ? *ex : *mn, x_in(b + 1), ne ? extra_mask : msa_mask, params + poff(b + 1),
                                  ctx_of(b + 1), blockws, sm, sp_);
    };
    int rc = block_fwd_impl<T>(h, d, x_in(b), z_in(b), is_e ? extra_mask : msa_mask, pair_mask, params + poff(b), xo, zo,
                               ctx_of(b), blockws, sp.block_bytes, sm, sp_, pre_done, chain ? &early : nullptr);
    if (rc) return rc;
    pre_done = chain;
  }
  // backward
  char* pp = ws + sp.off_pp;
  char* dz_pp[2] = {pp, pp + sp.n_pair};
  char* dm_pp[2] = {pp + 2 * sp.n_pair, pp + 2 * sp.n_pair + sp.n_msa};
  char* de_pp[2] = {pp + 2 * sp.n_pair + 2 * sp.n_msa, pp + 2 * sp.n_pair + 2 * sp.n_msa + sp.n_extra};
  const void* dz = d_pair_out;
  const void* dm = d_msa_out;
  const void* de = nullptr;
  if (n_extra) {
    // a fill kernel, not hipMemsetAsync: the call may be captured into a HIP graph by the caller
    // the slot that the last extra block does NOT write (it writes de_pp[(n_extra - 1) & 1], or d_extra_msa_in)
    char* zero_slot = de_pp[n_extra & 1];
    hipLaunchKernelGGL(zero_bytes16_kernel, dim3((unsigned)((sp.n_extra / 16 + 255) / 256)), dim3(256), 0, sm,
                       (uint4*)zero_slot, (long long)(sp.n_extra / 16));
    if (!hip_ok(h, hipGetLastError(), "zero fill")) return PE_ERR_HIP;
    de = zero_slot;
  }
  for (int b = nb - 1; b >= 0; b--) {
    const bool is_e = b < n_extra;
    const pe_dims& d = is_e ? *ex : *mn;
    void* dz_in = (b == 0) ? d_pair_in : (void*)dz_pp[b & 1];
    void* dx_in;
    if (is_e) dx_in = (b == 0) ? d_extra_msa_in : (void*)de_pp[b & 1];
    else dx_in = (b == n_extra) ? d_msa_in : (void*)dm_pp[b & 1];
    int rc = block_bwd_impl<T>(h, d, x_in(b), z_in(b), is_e ? extra_mask : msa_mask, pair_mask, params + poff(b),
                               is_e ? de : dm, dz, dx_in, dz_in, d_params + poff(b), ctx_of(b), blockws, sp.block_bytes, sm,
                               sp_);
    if (rc) return rc;
    dz = dz_in;
    if (is_e) de = dx_in; else dm = dx_in;
  }
  return PE_OK;
}

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
static bool overlap(const void* a, size_t na, const void* b, size_t nb) {
  const char* x = (const char*)a; const char* y = (const char*)b;
  return x < y + nb && y < x + na;
}
// a buffer of a call: written = the call writes it (outputs, ctx of the forward, workspace)
struct Region { const void* p; size_t n; bool written; };
// true when two buffers overlap of which at least one is written (null and empty buffers are skipped)
static bool any_alias(const Region* r, int n) {
  for (int i = 0; i < n; i++)
    for (int j = i + 1; j < n; j++)
      if ((r[i].written || r[j].written) && r[i].p && r[j].p && r[i].n && r[j].n && overlap(r[i].p, r[i].n, r[j].p, r[j].n))
        return true;
  return false;
}

extern "C" {

int pe_destroy(pe_handle* h);

int pe_create(pe_handle** out) {
  if (!out) return PE_ERR_NULL;
  pe_handle* h = new pe_handle();
  {
    // Device address of `scratch` on the current device, looked up on the first pe_create per device.
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= PE_MAX_DEVICES)) e = hipErrorInvalidDevice;
    if (e == hipSuccess) {
      std::lock_guard<std::mutex> lock(g_scratch_mutex);
      if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e == hipSuccess && !p) e = hipErrorInvalidSymbol;
        if (e == hipSuccess) g_scratch_ptr[dev] = p;
      }
      if (e == hipSuccess) { h->device = dev; h->static_scratch = g_scratch_ptr[dev]; }
    }
    if (e != hipSuccess) {
      (void)hipGetLastError();
      delete h;
      return PE_ERR_HIP;
    }
  }
  h->branches = 3;
  h->sync_debug = 0;
  h->timing = 0;
  h->side_streams = 0;
  h->stack_keep = 0;
  h->stack_overlap = 0;
  h->side[0] = h->side[1] = nullptr;
  h->side_ev_next = 0;
  for (int i = 0; i < 32; i++) h->side_ev[i] = nullptr;
  for (int i = 0; i < 6; i++) {
    if (hipEventCreateWithFlags(&h->ev[i], hipEventDisableTiming) != hipSuccess) {
      for (int j = 0; j < i; j++) (void)hipEventDestroy(h->ev[j]);
      delete h;
      return PE_ERR_HIP;
    }
  }
  *out = h;
  return PE_OK;
}
int pe_destroy(pe_handle* h) {
  if (!h) return PE_ERR_NULL;
  for (int i = 0; i < 6; i++) (void)hipEventDestroy(h->ev[i]);
  for (auto& r : h->recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  for (auto e : h->ev_pool) (void)hipEventDestroy(e);
  for (int i = 0; i < 2; i++) if (h->side[i]) (void)hipStreamDestroy(h->side[i]);
  for (int i = 0; i < 32; i++) if (h->side_ev[i]) (void)hipEventDestroy(h->side_ev[i]);
  delete h;
  return PE_OK;
}
int pe_set_option(pe_handle* h, int option, int value) {
  if (!h) return PE_ERR_NULL;
  if (option == PE_OPT_BRANCHES) { if (value < 1 || value > 3) return PE_ERR_ARG; h->branches = value; return PE_OK; }
  if (option == PE_OPT_SYNC_DEBUG) { h->sync_debug = value ? 1 : 0; return PE_OK; }
  if (option == PE_OPT_KERNEL_TIMING) { h->timing = value ? 1 : 0; return PE_OK; }
  if (option == PE_OPT_STACK_KEEP_CTX) { h->stack_keep = value ? 1 : 0; return PE_OK; }
  if (option == PE_OPT_STACK_OVERLAP) { h->stack_overlap = value ? 1 : 0; return PE_OK; }
  if (option == PE_OPT_SIDE_STREAMS) {
    // Created on first use only: every extra stream competes for the process's few hardware
    // queues (4 by default), and two streams that share a queue serialise.
    if (value && !h->side[0]) {
      for (int i = 0; i < 2; i++)
        if (hipStreamCreateWithFlags(&h->side[i], hipStreamNonBlocking) != hipSuccess) return PE_ERR_HIP;
      for (int i = 0; i < 32; i++)
        if (hipEventCreateWithFlags(&h->side_ev[i], hipEventDisableTiming) != hipSuccess) return PE_ERR_HIP;
    }
    h->side_streams = value ? 1 : 0;
    return PE_OK;
  }
  return PE_ERR_ARG;
}
static int check_dims_why(const pe_dims* d, const char** why) {
  int rc = pe_check_dims_impl(d, why);
  if (rc) return rc;
  if (d->col_global && (d->d_msa > GC_MAXD || d->h_msa > GC_MAXH)) {
    *why = "global column attention needs d_msa <= 8 and h_msa <= 8";
    return PE_ERR_DIMS;
  }
  return PE_OK;
}
int pe_check_dims(const pe_dims* d) {
  const char* why;
  return check_dims_why(d, &why);
}
const char* pe_dims_error(const pe_dims* d) {
  const char* why = "";
  (void)check_dims_why(d, &why);
  return why;
}
long long pe_param_count(const pe_dims* d) {
  if (pe_check_dims_impl(d)) return -1;
  ParamLayout L;
  build_param_layout(*d, L);
  return L.total;
}
int pe_param_table(const pe_dims* d, pe_param_entry* out, int cap) {
  int rc = pe_check_dims_impl(d);
  if (rc) return rc;
  ParamLayout L;
  build_param_layout(*d, L);
  int n = (int)L.entries.size();
  if (out) {
    if (cap < n) return PE_ERR_ARG;
    for (int i = 0; i < n; i++) out[i] = L.entries[i];
  }
  return n;
}
int pe_ctx_table(const pe_dims* d, pe_ctx_entry* out, int cap) {
  int rc = pe_check_dims(d);
  if (rc) return rc;
  std::vector<pe_ctx_entry> rec;
  if (d->dtype == PE_BF16) { Ctx<bf16> c; carve_ctx<bf16>(kDryBase, *d, c, &rec); }
  else { Ctx<float> c; carve_ctx<float>(kDryBase, *d, c, &rec); }
  int n = (int)rec.size();
  if (out) {
    if (cap < n) return PE_ERR_ARG;
    for (int i = 0; i < n; i++) out[i] = rec[i];
  }
  return n;
}
size_t pe_ctx_bytes(const pe_dims* d) {
  if (pe_check_dims(d)) return 0;
  return plan_for(*d).ctx_total();
}
size_t pe_workspace_bytes(const pe_dims* d, int with_ctx) {
  if (pe_check_dims(d)) return 0;
  return plan_for(*d).total(with_ctx != 0);
}

int pe_block_fwd(pe_handle* h, const pe_dims* dims, const void* msa_in, const void* pair_in, const float* msa_mask,
                 const float* pair_mask, const float* params, void* msa_out, void* pair_out, void* ctx, void* workspace,
                 size_t workspace_bytes, void* stream_msa, void* stream_pair) {
  if (!h || !dims || !msa_in || !pair_in || !msa_mask || !pair_mask || !params || !msa_out || !pair_out || !workspace)
    return PE_ERR_NULL;
  int rc = pe_check_dims(dims);
  if (rc) return rc;
  size_t E = dims->dtype == PE_BF16 ? 2 : 4;
  size_t nm = (size_t)dims->s * dims->r * dims->c_m * E, nz = (size_t)dims->r * dims->r * dims->c_z * E;
  {
    const Plan pl = plan_for(*dims);
    const Region rg[] = {{msa_in, nm, false}, {pair_in, nz, false}, {msa_mask, (size_t)dims->s * dims->r * 4, false},
                         {pair_mask, (size_t)dims->r * dims->r * 4, false}, {params, (size_t)pe_param_count(dims) * 4, false},
                         {msa_out, nm, true}, {pair_out, nz, true}, {ctx, ctx ? pl.ctx_total() : 0, true},
                         {workspace, pl.total(ctx == nullptr), true}};
    if (any_alias(rg, (int)(sizeof(rg) / sizeof(rg[0])))) return PE_ERR_ALIAS;
  }
  if (((uintptr_t)workspace) % 256 || (ctx && ((uintptr_t)ctx) % 256)) return PE_ERR_ARG;
  if (dims->dtype == PE_BF16)
    return block_fwd_impl<bf16>(h, *dims, msa_in, pair_in, msa_mask, pair_mask, params, msa_out, pair_out, ctx, workspace,
                                workspace_bytes, (hipStream_t)stream_msa, (hipStream_t)stream_pair);
  return block_fwd_impl<float>(h, *dims, msa_in, pair_in, msa_mask, pair_mask, params, msa_out, pair_out, ctx, workspace,
                               workspace_bytes, (hipStream_t)stream_msa, (hipStream_t)stream_pair);
}

size_t pe_static_scratch_bytes(void) { return PE_STATIC_SCRATCH_BYTES; }

int pe_block_fwd_static(pe_handle* h, const pe_dims* dims, const void* msa_in, const void* pair_in, const float* msa_mask,
                        const float* pair_mask, const float* params, void* msa_out, void* pair_out, void* stream_msa,
                        void* stream_pair) {
  if (!h || !dims) return PE_ERR_NULL;
  int rc = pe_check_dims(dims);
  if (rc) return rc;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != h->device) {
    h->last_error = "pe_block_fwd_static: the handle belongs to another device than the current one";
    return PE_ERR_ARG;
  }
  const size_t need = plan_for(*dims).total(true);
  if (need > PE_STATIC_SCRATCH_BYTES) {
    char msg[160];
    snprintf(msg, sizeof(msg), "pe_block_fwd_static: these dims need %zu bytes of scratch, the static array holds %zu",
             need, (size_t)PE_STATIC_SCRATCH_BYTES);
    h->last_error = msg;
    return PE_ERR_WORKSPACE;
  }
  // nothing in the scratch has to start at zero: every kernel writes what it later reads
  return pe_block_fwd(h, dims, msa_in, pair_in, msa_mask, pair_mask, params, msa_out, pair_out, nullptr, h->static_scratch,
                      PE_STATIC_SCRATCH_BYTES, stream_msa, stream_pair);
}

int pe_block_bwd(pe_handle* h, const pe_dims* dims, const void* msa_in, const void* pair_in, const float* msa_mask,
                 const float* pair_mask, const float* params, const void* d_msa_out, const void* d_pair_out,
                 void* d_msa_in, void* d_pair_in, float* d_params, const void* ctx, void* workspace,
                 size_t workspace_bytes, void* stream_msa, void* stream_pair) {
  if (!h || !dims || !msa_in || !pair_in || !msa_mask || !pair_mask || !params || !d_msa_out || !d_pair_out ||
      !d_msa_in || !d_pair_in || !d_params || !workspace)
    return PE_ERR_NULL;
  int rc = pe_check_dims(dims);
  if (rc) return rc;
  size_t E = dims->dtype == PE_BF16 ? 2 : 4;
  size_t nm = (size_t)dims->s * dims->r * dims->c_m * E, nz = (size_t)dims->r * dims->r * dims->c_z * E;
  {
    const Plan pl = plan_for(*dims);
    const size_t np = (size_t)pe_param_count(dims) * 4;
    const Region rg[] = {{msa_in, nm, false}, {pair_in, nz, false}, {msa_mask, (size_t)dims->s * dims->r * 4, false},
                         {pair_mask, (size_t)dims->r * dims->r * 4, false}, {params, np, false},
                         {d_msa_out, nm, false}, {d_pair_out, nz, false}, {ctx, ctx ? pl.ctx_total() : 0, false},
                         {d_msa_in, nm, true}, {d_pair_in, nz, true}, {d_params, np, true},
                         {workspace, pl.total(ctx == nullptr), true}};
    if (any_alias(rg, (int)(sizeof(rg) / sizeof(rg[0])))) return PE_ERR_ALIAS;
  }
  if (((uintptr_t)workspace) % 256 || (ctx && ((uintptr_t)ctx) % 256)) return PE_ERR_ARG;
  if (dims->dtype == PE_BF16)
    return block_bwd_impl<bf16>(h, *dims, msa_in, pair_in, msa_mask, pair_mask, params, d_msa_out, d_pair_out, d_msa_in,
                                d_pair_in, d_params, ctx, workspace, workspace_bytes, (hipStream_t)stream_msa,
                                (hipStream_t)stream_pair);
  return block_bwd_impl<float>(h, *dims, msa_in, pair_in, msa_mask, pair_mask, params, d_msa_out, d_pair_out, d_msa_in,
                               d_pair_in, d_params, ctx, workspace, workspace_bytes, (hipStream_t)stream_msa,
                               (hipStream_t)stream_pair);
}

size_t pe_stack_workspace_bytes(int n_extra, const pe_dims* extra, int n_main, const pe_dims* main_) {
  StackPlan sp;
  if (make_stack_plan(n_extra, extra, n_main, main_, false, sp)) return 0;
  return sp.total;
}
size_t pe_stack_workspace_bytes_keep(int n_extra, const pe_dims* extra, int n_main, const pe_dims* main_) {
  StackPlan sp;
  if (make_stack_plan(n_extra, extra, n_main, main_, true, sp)) return 0;
  return sp.total;
}

int pe_stack_fwd_bwd(pe_handle* h, int n_extra, const pe_dims* extra, int n_main, const pe_dims* main_,
                     const void* extra_msa_in, const void* msa_in, const void* pair_in, const float* extra_msa_mask,
                     const float* msa_mask, const float* pair_mask, const float* params, const void* d_msa_out,
                     const void* d_pair_out, void* msa_out, void* pair_out, void* d_extra_msa_in, void* d_msa_in,
                     void* d_pair_in, float* d_params, void* workspace, size_t workspace_bytes, void* stream_msa,
                     void* stream_pair) {
  if (!h || !pair_in || !pair_mask || !params || !d_pair_out || !pair_out || !d_pair_in || !d_params || !workspace)
    return PE_ERR_NULL;
  if (h->branches != 3) {   // a block with one branch switched off leaves an output unwritten that the next block reads
    h->last_error = "pe_stack_fwd_bwd needs both branches (PE_OPT_BRANCHES = 3)";
    return PE_ERR_ARG;
  }
  StackPlan sp;
  int rc = make_stack_plan(n_extra, extra, n_main, main_, h->stack_keep != 0, sp);
  if (rc) return rc;
  if (n_extra && (!extra_msa_in || !extra_msa_mask || !d_extra_msa_in)) return PE_ERR_NULL;
  if (n_main && (!msa_in || !msa_mask || !d_msa_out || !msa_out || !d_msa_in)) return PE_ERR_NULL;
  if (((uintptr_t)workspace) % 256) return PE_ERR_ARG;
  if (workspace_bytes < sp.total) return PE_ERR_WORKSPACE;
  {
    const size_t np = (size_t)((n_extra ? pe_param_count(extra) * n_extra : 0) + (n_main ? pe_param_count(main_) * n_main : 0)) * 4;
    const size_t nem = n_extra ? (size_t)extra->s * extra->r * 4 : 0, nmm = n_main ? (size_t)main_->s * main_->r * 4 : 0;
    const pe_dims* any = n_main ? main_ : extra;
    // exact tensor sizes (the plan's are rounded up to its 256-byte slots)
    const size_t ze = n_extra ? (size_t)extra->s * extra->r * extra->c_m * sp.E : 0;
    const size_t zm = n_main ? (size_t)main_->s * main_->r * main_->c_m * sp.E : 0;
    const size_t zz = (size_t)any->r * any->r * any->c_z * sp.E;
    const Region rg[] = {{extra_msa_in, ze, false}, {msa_in, zm, false}, {pair_in, zz, false},
                         {extra_msa_mask, nem, false}, {msa_mask, nmm, false}, {pair_mask, (size_t)any->r * any->r * 4, false},
                         {params, np, false}, {d_msa_out, zm, false}, {d_pair_out, zz, false},
                         {msa_out, zm, true}, {pair_out, zz, true}, {d_extra_msa_in, ze, true},
                         {d_msa_in, zm, true}, {d_pair_in, zz, true}, {d_params, np, true},
                         {workspace, sp.total, true}};
    if (any_alias(rg, (int)(sizeof(rg) / sizeof(rg[0])))) return PE_ERR_ALIAS;
  }
  const int dt = n_main ? main_->dtype : extra->dtype;
  if (dt == PE_BF16)
    return stack_impl<bf16>(h, n_extra, extra, n_main, main_, sp, extra_msa_in, msa_in, pair_in, extra_msa_mask, msa_mask,
                            pair_mask, params, d_msa_out, d_pair_out, msa_out, pair_out, d_extra_msa_in, d_msa_in,
                            d_pair_in, d_params, (char*)workspace, (hipStream_t)stream_msa, (hipStream_t)stream_pair);
  return stack_impl<float>(h, n_extra, extra, n_main, main_, sp, extra_msa_in, msa_in, pair_in, extra_msa_mask, msa_mask,
                           pair_mask, params, d_msa_out, d_pair_out, msa_out, pair_out, d_extra_msa_in, d_msa_in,
                           d_pair_in, d_params, (char*)workspace, (hipStream_t)stream_msa, (hipStream_t)stream_pair);
}

int pe_timing_collect(pe_handle* h, pe_timing_entry* out, int cap) {
  if (!h) return PE_ERR_NULL;
  if (hipDeviceSynchronize() != hipSuccess) { h->last_error = "timing: device synchronize failed"; return PE_ERR_HIP; }
  std::vector<pe_timing_entry> agg;
  for (auto& r : h->recs) {
    float ms = 0.0f;
    (void)hipEventElapsedTime(&ms, r.e0, r.e1);
    size_t k = 0;
    for (; k < agg.size(); k++)
      if (!strncmp(agg[k].name, r.label, sizeof(agg[k].name) - 1) &&
          !strncmp(agg[k].kernel, r.kern.c_str(), sizeof(agg[k].kernel) - 1)) break;
    if (k == agg.size()) {
      pe_timing_entry e;
      memset(&e, 0, sizeof(e));
      snprintf(e.name, sizeof(e.name), "%s", r.label);
      snprintf(e.kernel, sizeof(e.kernel), "%s", r.kern.c_str());
      agg.push_back(e);
    }
    agg[k].launches += 1;
    agg[k].total_ms += ms;
    agg[k].flops += r.flops;
    agg[k].bytes += r.bytes;
  }
  int n = (int)agg.size();
  if (!out) return n;               // query only: records are kept
  if (cap < n) return PE_ERR_ARG;
  for (int i = 0; i < n; i++) out[i] = agg[i];
  for (auto& r : h->recs) { h->ev_pool.push_back(r.e0); h->ev_pool.push_back(r.e1); }
  h->recs.clear();
  return n;
}

const char* pe_strerror(int code) {
  switch (code) {
    case PE_OK: return "ok";
    case PE_ERR_NULL: return "required pointer is NULL";
    case PE_ERR_DIMS: return "unsupported dims";
    case PE_ERR_WORKSPACE: return "workspace too small";
    case PE_ERR_ALIAS: return "output aliases an input or another output";
    case PE_ERR_HIP: return "HIP error (see pe_last_error)";
    case PE_ERR_ARG: return "bad argument";
    default: return "unknown error";
  }
}
const char* pe_last_error(pe_handle* h) { return h ? h->last_error.c_str() : ""; }

}  // extern "C"
