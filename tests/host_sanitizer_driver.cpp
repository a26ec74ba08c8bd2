// Host-side exercise of liblsw's C ABI for an AddressSanitizer + UndefinedBehaviorSanitizer build of the HOST code
// (tests/test_host_sanitizers.py compiles lsw_api.cpp with the sanitizers and links this driver against it).
// Everything here returns before any device work: routers, term lists, work decomposition, argument validation.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <vector>

#include "lsw.h"
#include "lsw_tuning.h"

#define EXPECT(cond)                                                         \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                          \
    }                                                                        \
  } while (0)

int main() {
  // router: every k, ties, extremes, bad arguments
  for (int E : {1, 2, 8, 16, 4096}) {
    std::vector<float> logits(static_cast<size_t>(E));
    for (int i = 0; i < E; ++i) logits[size_t(i)] = std::sin(0.37f * float(i)) * 3.0f;
    for (int k = 0; k <= (E < 8 ? E : 8); ++k) {
      std::vector<int32_t> ids(size_t(k) + 1, -7);
      std::vector<float> gates(size_t(k) + 1, -7.0f);
      EXPECT(lsw_route(logits.data(), E, k, ids.data(), gates.data()) == LSW_OK);
      double sum = 0;
      for (int c = 0; c < k; ++c) { EXPECT(ids[size_t(c)] >= 0 && ids[size_t(c)] < E); sum += gates[size_t(c)]; }
      EXPECT(k == 0 || std::fabs(sum - 1.0) < 1e-5);
      EXPECT(ids[size_t(k)] == -7 && gates[size_t(k)] == -7.0f);       // nothing written past k entries
    }
  }
  {
    float l[4] = {1e30f, -1e30f, 1e30f, 0.0f};
    int32_t ids[2];
    float g[2];
    EXPECT(lsw_route(l, 4, 2, ids, g) == LSW_OK && ids[0] == 0 && ids[1] == 2);
    l[1] = std::numeric_limits<float>::quiet_NaN();
    EXPECT(lsw_route(l, 4, 2, ids, g) == LSW_ERR_ARG);
    EXPECT(lsw_route(nullptr, 4, 2, ids, g) == LSW_ERR_ARG);
    EXPECT(lsw_route(l, 4, 5, ids, g) == LSW_ERR_ARG);
    EXPECT(lsw_last_error()[0] != 0);
  }
  // term lists at the largest sizes, full overlap, no overlap, bad lists
  {
    int32_t a[LSW_MAX_K], b[LSW_MAX_K], out_ids[2 * LSW_MAX_K + 1];
    float ga[LSW_MAX_K], gb[LSW_MAX_K], out_c[2 * LSW_MAX_K + 1];
    for (int i = 0; i < LSW_MAX_K; ++i) { a[i] = i; b[i] = LSW_MAX_K + i; ga[i] = 0.125f; gb[i] = 0.125f; }
    int32_t n = -1;
    out_ids[2 * LSW_MAX_K] = -9;
    EXPECT(lsw_build_terms(a, ga, LSW_MAX_K, b, gb, LSW_MAX_K, 64, 2.0f, out_ids, out_c, &n) == LSW_OK && n == 2 * LSW_MAX_K);
    EXPECT(out_ids[2 * LSW_MAX_K] == -9);
    EXPECT(lsw_build_terms(a, ga, LSW_MAX_K, a, ga, LSW_MAX_K, 64, 2.0f, out_ids, out_c, &n) == LSW_OK && n == 0);
    EXPECT(lsw_build_terms(a, ga, LSW_MAX_K + 1, nullptr, nullptr, 0, 64, 1.0f, out_ids, out_c, &n) == LSW_ERR_ARG);
    a[3] = 64;
    EXPECT(lsw_build_terms(a, ga, LSW_MAX_K, nullptr, nullptr, 0, 64, 1.0f, out_ids, out_c, &n) == LSW_ERR_ARG);
    EXPECT(lsw_build_terms(nullptr, nullptr, 0, nullptr, nullptr, 0, 64, 1.0f, nullptr, nullptr, &n) == LSW_OK && n == 0);
    EXPECT(lsw_build_terms(nullptr, nullptr, 0, nullptr, nullptr, 0, 64, 1.0f, nullptr, nullptr, nullptr) == LSW_ERR_ARG);
  }
  // work decomposition: every item of a ragged stack decodes inside its matrix; sizes near the 32-bit limit are refused
  {
    const int32_t out[4] = {37, 4096, 1, 11008}, in[4] = {264, 11008, 8, 4096};
    const int64_t n = lsw_worklist_size(out, in, 4, 128, 1024);
    EXPECT(n > 0);
    int64_t cells = 0;
    for (int64_t it = 0; it < n; ++it) {
      int32_t lin, r0, nr, c0, nc;
      EXPECT(lsw_worklist_item(out, in, 4, 128, 1024, it, &lin, &r0, &nr, &c0, &nc) == LSW_OK);
      EXPECT(lin >= 0 && lin < 4 && r0 >= 0 && nr > 0 && r0 + nr <= out[lin] && c0 >= 0 && nc > 0 && c0 + nc <= in[lin]);
      cells += int64_t(nr) * nc;
    }
    int64_t want = 0;
    for (int p = 0; p < 4; ++p) want += int64_t(out[p]) * in[p];
    EXPECT(cells == want);
    int32_t lin, r0, nr, c0, nc;
    EXPECT(lsw_worklist_item(out, in, 4, 128, 1024, n, &lin, &r0, &nr, &c0, &nc) == LSW_ERR_ARG);
    EXPECT(lsw_worklist_item(out, in, 4, 128, 1024, -1, &lin, &r0, &nr, &c0, &nc) == LSW_ERR_ARG);
    const int32_t big_out[1] = {2147483647}, big_in[1] = {2147483640};
    EXPECT(lsw_worklist_size(big_out, big_in, 1, 1, 1) > 0);          // 64-bit count
    EXPECT(lsw_worklist_item(big_out, big_in, 1, 1, 1, 0, &lin, &r0, &nr, &c0, &nc) == LSW_ERR_SHAPE);
    EXPECT(lsw_worklist_size(out, in, 0, 128, 1024) == -1);
  }
  // creation is validated before any device is touched; null contexts fail cleanly everywhere
  {
    lsw_linear L{reinterpret_cast<void*>(0x1000), reinterpret_cast<void*>(0x2000), reinterpret_cast<void*>(0x3000), 64, 64, 0, 0};
    lsw_ctx* ctx = reinterpret_cast<lsw_ctx*>(0x1);
    EXPECT(lsw_create_adapters(&L, 1, 0, 8, 1.0f, &ctx) == LSW_ERR_ARG && ctx == nullptr);
    EXPECT(lsw_create_adapters_ex(&L, 1, 8, 4, 1.0f, LSW_FACTOR_BF16, &ctx) == LSW_ERR_SHAPE);
    EXPECT(lsw_create_adapters_ex(&L, 1, 8, 8, 1.0f, 5, &ctx) == LSW_ERR_ARG);
    L.in = 12;
    EXPECT(lsw_create_adapters(&L, 1, 8, 8, 1.0f, &ctx) == LSW_ERR_SHAPE);
    L.in = 64;
    L.ld = 56;                 // a leading dimension below in, and one that leaves rows misaligned
    EXPECT(lsw_create_adapters(&L, 1, 8, 8, 1.0f, &ctx) == LSW_ERR_SHAPE);
    L.ld = 68;
    EXPECT(lsw_create_adapters(&L, 1, 8, 8, 1.0f, &ctx) == LSW_ERR_SHAPE);
    L.ld = 1 << 24;            // 64 rows rounded up to 128 x 2^24 x 2 bytes: beyond 2 GiB because of the pitch alone
    EXPECT(lsw_create_adapters(&L, 1, 8, 8, 1.0f, &ctx) == LSW_ERR_SHAPE);
    L.ld = 0;
    L.out = 40000000;          // 40e6 x 64 x 2 bytes: above 2 GiB
    EXPECT(lsw_create_adapters(&L, 1, 8, 8, 1.0f, &ctx) == LSW_ERR_SHAPE);
    EXPECT(lsw_create_adapters(&L, 1, 8, 8, 1.0f, nullptr) == LSW_ERR_ARG);
    int32_t k = 0, flags = 0;
    EXPECT(lsw_switch(nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_switch_dev(nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_rebase(nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_set_base(nullptr, nullptr, 0) == LSW_ERR_ARG);
    EXPECT(lsw_drop_subset_tables(nullptr) == LSW_ERR_ARG);
    { int32_t rr[2] = {300, 5}, cc[2] = {520, 264}, m, r0, c0, nc; int64_t nx;
      EXPECT(lsw_flat_item(rr, cc, 2, 16, 3, -1, &m, &r0, &c0, &nc, &nx) == LSW_OK);
      EXPECT(lsw_flat_item(rr, cc, 2, 12, 3, -1, &m, &r0, &c0, &nc, &nx) == LSW_ERR_ARG);
      EXPECT(lsw_flat_item(rr, cc, 2, 16, 3, -1, nullptr, &r0, &c0, &nc, &nx) == LSW_ERR_ARG); }
    { double ns = 0; EXPECT(lsw_probe_matrix_loop(0, 1, 0, 0, &ns) == LSW_ERR_ARG); EXPECT(lsw_probe_matrix_loop(1, 1, 3, 0, &ns) == LSW_ERR_ARG);
      EXPECT(lsw_probe_matrix_loop(1, 1, 0, 0, nullptr) == LSW_ERR_ARG); }
    EXPECT(lsw_enable_adapter_path(nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_adapter_forward(nullptr, 0, nullptr, 1, nullptr, nullptr, 0, nullptr, nullptr, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_adapter_workspace_bytes(nullptr, 0, 1) == -1);
    EXPECT(lsw_adapter_layer_workspace_bytes(nullptr, 0, 1) == -1);
    EXPECT(lsw_adapter_forward_layer(nullptr, 0, nullptr, 1, nullptr, nullptr, 0, nullptr, nullptr, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_adapter_forward_static(nullptr, 0, nullptr, 1, nullptr, nullptr, 0, nullptr, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_route_batch_dev(nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_get_state(nullptr, 0, nullptr, nullptr, &k) == LSW_ERR_ARG);
    EXPECT(lsw_dev_status(nullptr, &flags) == LSW_ERR_ARG);
    EXPECT(lsw_gemv_bf16(nullptr, nullptr, nullptr, 1, 8, nullptr) == LSW_ERR_ARG);
    EXPECT(lsw_query(nullptr, LSW_Q_N_LINEARS) == -1);
    lsw_destroy(nullptr);
  }
  std::puts("host sanitizer driver OK");
  return 0;
}
