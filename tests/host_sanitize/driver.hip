// Host-side exercise of the C ABI for a sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer on the host
// code only; no kernel is launched and no GPU is needed).  Linked with csrc/api.hip alone: the kernel launchers
// are stubbed here, every call below stops on the host before it would reach one.  Mirrors tests/test_host_api.py
// and adds ap_set_weights for every compiled channel pair, whose operand-table builders index a dozen arrays.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "ap_internal.h"

namespace ap {
#define AP_STUB { return hipErrorUnknown; }
hipError_t launch_predict(const Shape&, int, int, const float*, const float*, int, int, int, float*, float*, hipStream_t) AP_STUB
hipError_t launch_predict_interior(const Shape&, int, int, const float*, const float*, int, int, float*, hipStream_t) AP_STUB
hipError_t launch_predict_columns(const Shape&, int, int, const float*, const float*, int, int, int, float*, float*, hipStream_t) AP_STUB
hipError_t launch_predict_inc(const Shape&, int, int, const float*, const float*, int, int, int, float*, float*, hipStream_t) AP_STUB
hipError_t launch_select(const Shape&, int, int, const float*, int, int32_t*, int32_t*, hipStream_t) AP_STUB
hipError_t launch_sparse_decode(const Shape&, int, int, const void*, const void*, const void*, int, const int32_t*,
                                const int32_t*, float*, float*, size_t, float*, hipStream_t) AP_STUB
hipError_t launch_calibrate(const Shape&, const void*, const void*, int, float*, float*, hipStream_t) AP_STUB
hipError_t launch_refresh_selection(const Shape&, int, int, int32_t*, int32_t*, hipStream_t) AP_STUB
int prefetch_state_stride(const Shape& s) { return 3 * s.k + 4; }
hipError_t launch_gather_blocks(const Shape&, const void*, const void*, int, int, const int32_t*, const int32_t*, void*,
                                void*, int32_t*, int32_t*, hipStream_t) AP_STUB
hipError_t launch_append_row(const Shape&, const void*, const void*, int, const int32_t*, const int32_t*, void*, void*,
                             hipStream_t) AP_STUB
hipError_t launch_stream_read(const void*, size_t, void*, int, hipStream_t) AP_STUB
hipError_t launch_stream_copy(const void*, size_t, void*, int, hipStream_t) AP_STUB
hipError_t launch_push_row(const Shape&, float*, int, const float*, hipStream_t) AP_STUB
hipError_t static_scratch(float**, size_t*) AP_STUB
}  // namespace ap

static int failures = 0;
#define CHECK(cond)                                                     \
  do {                                                                  \
    if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static ap_config base_cfg() {
  ap_config c;
  c.n_inst = 8; c.g = 4; c.head_dim = 128; c.block = 16; c.hist_len = 64; c.t_cap = 32768 + 256; c.k_blocks = 64;
  c.n_sink = 4; c.n_local = 4; c.c1 = 8; c.c2 = 8; c.kv_dtype = AP_BF16; c.flags = 0;
  return c;
}

int main() {
  ap_ctx* ctx = nullptr;
  ap_config c = base_cfg();
  CHECK(ap_create(nullptr, &ctx) == AP_ERR_ARG);
  CHECK(ap_create(&c, nullptr) == AP_ERR_ARG);
  struct Bad { int field, value, code; };
  // field: 0 n_inst, 1 t_cap, 2 n_sink, 3 hist_len, 4 block, 5 g, 6 head_dim, 7 c2, 8 kv_dtype, 9 k_blocks
  const Bad bad[] = {{0, 0, AP_ERR_ARG}, {1, 1000, AP_ERR_ARG}, {2, 80, AP_ERR_ARG}, {3, 0, AP_ERR_ARG},
                     {4, 12, AP_ERR_UNSUPPORTED}, {5, 3, AP_ERR_UNSUPPORTED}, {6, 96, AP_ERR_UNSUPPORTED},
                     {7, 16, AP_ERR_UNSUPPORTED}, {8, 7, AP_ERR_UNSUPPORTED}, {9, 20000, AP_ERR_UNSUPPORTED},
                     {3, 300, AP_ERR_UNSUPPORTED}, {0, 70000, AP_ERR_UNSUPPORTED}};
  for (const Bad& b : bad) {
    ap_config x = base_cfg();
    int32_t* f[] = {&x.n_inst, &x.t_cap, &x.n_sink, &x.hist_len, &x.block, &x.g, &x.head_dim, &x.c2, &x.kv_dtype, &x.k_blocks};
    *f[b.field] = b.value;
    ap_ctx* y = nullptr;
    CHECK(ap_create(&x, &y) == b.code && y == nullptr);
  }
  // every compiled channel pair and a few shapes: create, size queries, the weight re-packing (it fails at the
  // device allocation without a GPU, after all host tables are built), destroy
  const int pairs[3][2] = {{4, 4}, {8, 8}, {16, 32}};
  for (const auto& pr : pairs)
    for (int H : {1, 5, 64, 256})
      for (int n_inst : {1, 128, 2048}) {
        ap_config x = base_cfg();
        x.c1 = pr[0]; x.c2 = pr[1]; x.hist_len = H; x.n_inst = n_inst;
        ap_ctx* y = nullptr;
        CHECK(ap_create(&x, &y) == AP_OK && y != nullptr);
        if (y == nullptr) continue;
        CHECK(ap_workspace_bytes(y) > 0 && ap_workspace_bytes(y) % 16 == 0);
        CHECK(ap_hist_slots(y) == H + 1 && ap_nb_cap(y) == x.t_cap / x.block);
        CHECK(ap_prefetch_state_bytes(y) == (size_t)n_inst * (3 * 64 + 4) * 4);
        CHECK(ap_score_offset(y) == 0.0);
        const size_t n = 9 * (size_t)x.c1 + x.c1 + 9 * (size_t)x.c1 * x.c2 + 2 * x.c2 + 1;
        std::vector<float> blob(n);
        for (size_t i = 0; i < n; ++i) blob[i] = 0.01f * (float)((int)(i * 2654435761u % 201) - 100);
        CHECK(ap_set_weights(y, blob.data(), n - 1, nullptr) == AP_ERR_ARG);
        const int rc = ap_set_weights(y, blob.data(), n, nullptr);
        CHECK(rc == AP_ERR_HIP || rc == AP_OK);          // no GPU here: the device allocation fails
        CHECK(ap_destroy(y) == AP_OK);
      }
  CHECK(ap_create(&c, &ctx) == AP_OK);
  void* ok = reinterpret_cast<void*>(4096);               // a fake, aligned, non-null address
  void* odd = reinterpret_cast<void*>(4100);
  float* fok = static_cast<float*>(ok);
  int32_t* iok = static_cast<int32_t*>(ok);
  CHECK(ap_predict(ctx, nullptr, 0, 100, fok, ok, nullptr) == AP_ERR_ARG);
  CHECK(ap_predict(ctx, static_cast<float*>(odd), 0, 100, fok, ok, nullptr) == AP_ERR_ALIGN);
  CHECK(ap_predict(ctx, fok, 0, 100, fok, ok, nullptr) == AP_ERR_STATE);
  CHECK(ap_select_topk(ctx, fok, 0, iok, iok, ok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_select_topk(ctx, fok, 1000000, iok, iok, ok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_sparse_decode(ctx, ok, ok, ok, 0, iok, iok, fok, fok, ok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_sparse_decode_noalloc(ctx, ok, ok, ok, 100000000, iok, iok, fok, fok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_calibrate(ctx, ok, nullptr, 5, fok, ok, nullptr) == AP_ERR_ARG);
  CHECK(ap_calibrate(ctx, ok, ok, 5, fok, ok, nullptr) == AP_ERR_ARG);           // not device-readable memory
  CHECK(ap_update_history(ctx, fok, -1, fok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_step(ctx, fok, 0, ok, ok, ok, 5, fok, iok, iok, fok, fok, 0, ok, nullptr) == AP_ERR_STATE);
  CHECK(ap_predict_incremental(ctx, fok, 0, 100, 100, 9, fok, fok, ok, nullptr) == AP_ERR_STATE);
  CHECK(ap_refresh_selection(ctx, 10, 5, iok, iok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_refresh_selection(ctx, 5, 10, nullptr, iok, nullptr) == AP_ERR_ARG);
  CHECK(ap_prefetch_blocks(ctx, ok, ok, 10, 0, iok, iok, ok, ok, iok, iok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_prefetch_blocks(ctx, ok, ok, 10, 5, iok, iok, ok, ok, iok, iok, nullptr) == AP_ERR_ARG);
  CHECK(ap_append_kv(ctx, ok, ok, -1, iok, iok, ok, ok, nullptr) == AP_ERR_RANGE);
  CHECK(ap_offload_begin(ctx, fok, 0, ok, ok, 5, iok, iok, fok, fok, ok, ok, iok, iok, ok, nullptr, nullptr) == AP_ERR_STATE);
  CHECK(ap_offload_step(ctx, fok, 0, ok, ok, ok, ok, ok, 5, 0, fok, iok, iok, fok, fok, 1, ok, ok, iok, iok, fok, ok,
                        nullptr, nullptr) == AP_ERR_STATE);
  CHECK(ap_set_block_table(ctx, iok, 0) == AP_ERR_ARG);
  CHECK(ap_set_block_table(ctx, iok, 10) == AP_OK);
  CHECK(ap_set_block_table(ctx, nullptr, 0) == AP_OK);
  CHECK(ap_stream_read(nullptr, 64, ok, 1, nullptr) == AP_ERR_ARG);
  for (int code = 0; code > -8; --code) CHECK(ap_strerror(code) != nullptr);
  CHECK(ap_destroy(ctx) == AP_OK);
  CHECK(ap_destroy(nullptr) == AP_ERR_ARG);
  std::printf(failures ? "host sanitizer driver: %d checks failed\n" : "host sanitizer driver: all checks passed\n", failures);
  return failures ? 1 : 0;
}
