// Host-only exercise of the C ABI for a sanitizer build (address + undefined behaviour): every entry point that
// needs no GPU - dims validation and its messages, the parameter and ctx tables, the dry-run plans behind the
// size queries (single block, stack with and without kept activations), argument validation of the compute
// calls that returns before any HIP call - over the workload shapes, ragged shapes and the limits of pe_dims.
// Built and run by tests/test_abi.py::test_host_paths_under_sanitizers; prints "ok <checks>" on success.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <vector>
#include "../../include/pe.h"

static int checks = 0;
#define REQUIRE(c) do { checks++; if (!(c)) { fprintf(stderr, "FAILED line %d: %s\n", __LINE__, #c); exit(1); } } while (0)

static pe_dims dims(int s, int r, int cm, int cz, int hm, int dm, int hp, int dp, int ct, int co, int n, int glob, int dt, int var) {
  pe_dims d;
  memset(&d, 0, sizeof(d));
  d.s = s; d.r = r; d.c_m = cm; d.c_z = cz; d.h_msa = hm; d.d_msa = dm; d.h_pair = hp; d.d_pair = dp;
  d.c_tri = ct; d.c_opm = co; d.n_trans = n; d.col_global = glob; d.dtype = dt; d.ln_eps = 1e-5f; d.opm_eps = 1e-3f;
  d.variant = var;
  return d;
}

static void exercise(const pe_dims& d) {
  REQUIRE(pe_check_dims(&d) == PE_OK);
  REQUIRE(strlen(pe_dims_error(&d)) == 0);
  const long long np = pe_param_count(&d);
  REQUIRE(np > 0);
  const int nt = pe_param_table(&d, nullptr, 0);
  REQUIRE(nt > 0);
  std::vector<pe_param_entry> tab(nt);
  REQUIRE(pe_param_table(&d, tab.data(), nt) == nt);
  REQUIRE(pe_param_table(&d, tab.data(), nt - 1) == PE_ERR_ARG);
  long long end = 0;
  for (const pe_param_entry& e : tab) {
    REQUIRE(e.offset == end);                                   // entries are contiguous and in order
    end += (long long)e.shape[0] * (e.ndim == 2 ? e.shape[1] : 1);
    REQUIRE(memchr(e.name, 0, sizeof(e.name)) != nullptr);      // names are terminated
  }
  REQUIRE(end == np);
  const int nc = pe_ctx_table(&d, nullptr, 0);
  REQUIRE(nc > 0);
  std::vector<pe_ctx_entry> ctab(nc);
  REQUIRE(pe_ctx_table(&d, ctab.data(), nc) == nc);
  const size_t cb = pe_ctx_bytes(&d);
  for (const pe_ctx_entry& e : ctab) {
    REQUIRE(e.offset_bytes % 256 == 0);
    REQUIRE((size_t)e.offset_bytes + (size_t)e.count * (e.dtype == PE_BF16 ? 2 : 4) <= cb);
  }
  const size_t w0 = pe_workspace_bytes(&d, 0), w1 = pe_workspace_bytes(&d, 1);
  REQUIRE(w0 > 0 && w1 >= w0 + cb);
  for (int ne = 0; ne <= 2; ne++)
    for (int nm = (ne ? 0 : 1); nm <= 3; nm += 2) {
      pe_dims e = d;
      e.col_global = 1; e.d_msa = 8; e.h_msa = 4; e.c_m = 64; e.s = d.s + 3;
      const size_t a = pe_stack_workspace_bytes(ne, &e, nm, &d), b = pe_stack_workspace_bytes_keep(ne, &e, nm, &d);
      REQUIRE(a > 0 && b >= a);
    }
}

int main() {
  // the workload shapes, the tiny test shape, ragged and degenerate shapes, both storage types, the three orderings
  const pe_dims shapes[] = {
      dims(8, 16, 32, 16, 4, 8, 2, 8, 16, 8, 4, 0, PE_F32, 0),
      dims(128, 256, 256, 128, 8, 32, 4, 32, 128, 32, 4, 0, PE_BF16, 0),
      dims(1024, 256, 64, 128, 8, 8, 4, 32, 128, 32, 4, 1, PE_BF16, 0),
      dims(512, 384, 256, 128, 8, 32, 4, 32, 128, 32, 4, 0, PE_BF16, 1),
      dims(5120, 384, 64, 128, 8, 8, 4, 32, 128, 32, 4, 1, PE_BF16, 0),
      dims(37, 150, 64, 32, 2, 16, 4, 8, 24, 16, 2, 0, PE_F32, 2),
      dims(1, 1, 8, 8, 1, 8, 1, 8, 8, 8, 1, 0, PE_F32, 0),
      dims(3, 7, 1024, 256, 8, 32, 8, 32, 192, 1024, 4, 0, PE_BF16, 0),
  };
  for (const pe_dims& d : shapes) exercise(d);

  // every limit of pe_dims: rejected, with a message, and the size queries return 0 instead of planning
  pe_dims ok = shapes[1];
  struct { int pe_dims::*field; int bad; } cases[] = {
      {&pe_dims::s, 0}, {&pe_dims::r, -1}, {&pe_dims::c_m, 250}, {&pe_dims::c_m, 2048}, {&pe_dims::c_z, 512},
      {&pe_dims::h_msa, 9}, {&pe_dims::d_msa, 12}, {&pe_dims::d_pair, 64}, {&pe_dims::c_tri, 200}, {&pe_dims::c_opm, 4},
      {&pe_dims::n_trans, 0}, {&pe_dims::n_trans, 64}, {&pe_dims::col_global, 2}, {&pe_dims::dtype, 5}, {&pe_dims::variant, 3},
  };
  for (auto& c : cases) {
    pe_dims d = ok;
    d.*(c.field) = c.bad;
    REQUIRE(pe_check_dims(&d) == PE_ERR_DIMS);
    REQUIRE(strlen(pe_dims_error(&d)) > 0);
    REQUIRE(pe_param_count(&d) == -1 || pe_workspace_bytes(&d, 1) == 0);
    REQUIRE(pe_workspace_bytes(&d, 1) == 0 && pe_ctx_bytes(&d) == 0);
    REQUIRE(pe_stack_workspace_bytes(0, nullptr, 2, &d) == 0);
  }
  { pe_dims d = ok; d.s = 70000; d.r = 40000; REQUIRE(pe_check_dims(&d) == PE_ERR_DIMS); }
  { pe_dims d = ok; d.ln_eps = 0.0f; REQUIRE(pe_check_dims(&d) == PE_ERR_DIMS); }
  REQUIRE(pe_check_dims(nullptr) == PE_ERR_NULL);
  REQUIRE(pe_stack_workspace_bytes(0, nullptr, 0, nullptr) == 0);
  REQUIRE(pe_stack_workspace_bytes(-1, &ok, 1, &ok) == 0);

  // compute calls: argument validation that returns before any HIP call
  REQUIRE(pe_block_fwd(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr) == PE_ERR_NULL);
  REQUIRE(pe_block_bwd(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr) == PE_ERR_NULL);
  REQUIRE(pe_block_fwd_static(nullptr, &ok, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == PE_ERR_NULL);
  REQUIRE(pe_stack_fwd_bwd(nullptr, 0, nullptr, 1, &ok, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, nullptr) == PE_ERR_NULL);
  REQUIRE(pe_set_option(nullptr, PE_OPT_BRANCHES, 3) == PE_ERR_NULL);
  REQUIRE(pe_timing_collect(nullptr, nullptr, 0) == PE_ERR_NULL);
  REQUIRE(pe_destroy(nullptr) == PE_ERR_NULL);
  REQUIRE(pe_static_scratch_bytes() == (size_t)32 << 20);
  for (int code = 0; code >= -7; code--) REQUIRE(strlen(pe_strerror(code)) > 0);
  REQUIRE(strlen(pe_last_error(nullptr)) == 0);
  printf("ok %d\n", checks);
  return 0;
}
