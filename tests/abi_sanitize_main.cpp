// Driver for a host-sanitizer build of the library's argument checks (CPU only, no GPU work):
// oea_api.hip compiled with AddressSanitizer + UndefinedBehaviorSanitizer on the host side and
// linked against stand-ins for the kernel launchers, which the calls below never reach: every
// call here is refused by an argument check.  Prints "abi sanitize: ok".
#include <cstdio>
#include <cstring>

#include "oea_internal.h"

namespace oea {  // stand-ins: reaching one of them means a check let a bad call through
static hipError_t reached(const char* what) {
  std::printf("abi sanitize: launcher reached: %s\n", what);
  return hipErrorUnknown;
}
hipError_t launch_ws_prepare(uint32_t*, size_t, hipStream_t) { return reached("ws_prepare"); }
hipError_t launch_route(const float*, const uint8_t*, int, int, int, int, int, RouteOut, hipStream_t) { return reached("route"); }
hipError_t launch_router_and_route(const void*, const void*, const float*, const uint8_t*, int, int, int, int, int,
                                   oea_dtype, float*, float*, size_t, uint32_t*, RouteOut, const RouteGeneralArgs*,
                                   hipStream_t) {
  return reached("router_and_route");
}
hipError_t launch_route_general(const float*, const uint8_t*, int, int, int, const RouteGeneralArgs&, int32_t*, RouteOut,
                                hipStream_t) {
  return reached("route_general");
}
hipError_t launch_expert_gate_up(const void*, const void*, const void*, void*, int, int, int, int, int, oea_dtype,
                                 Grouping, bool, hipStream_t) {
  return reached("gate_up");
}
hipError_t launch_expert_down(const void*, const void*, float*, int, int, int, int, int, oea_dtype, Grouping, bool,
                              bool, hipStream_t) {
  return reached("down");
}
hipError_t try_launch_fused(const void*, const void*, const void*, const void*, const void*, const float*,
                            const uint8_t*, float*, float*, void*, RouteOut, uint32_t*, int, int, int, int, int, int,
                            oea_dtype, hipStream_t, uint32_t, bool, float*, const RouteGeneralArgs*) {
  return reached("fused");
}
hipError_t try_launch_stage_kernels(int, const void*, const void*, const void*, void*, float*, int, int, int, int, int,
                                    oea_dtype, Grouping, bool, hipStream_t) {
  return reached("stage_kernels");
}
hipError_t try_launch_dense_stage(int, const void*, const void*, const void*, void*, float*, int, int, int, int, int,
                                  oea_dtype, Grouping, bool, hipStream_t) {
  return reached("dense_stage");
}
hipError_t launch_combine(const float*, const int32_t*, const int32_t*, float*, int, int, int, hipStream_t) {
  return reached("combine");
}
hipError_t launch_read_probe(const void*, size_t, uint32_t*, hipStream_t) { return reached("read_probe"); }
}  // namespace oea

static int failures = 0;
#define EXPECT(call, want)                                                          \
  do {                                                                              \
    const int got_ = (call);                                                        \
    if (got_ != (want)) {                                                           \
      std::printf("abi sanitize: %s returned %d, expected %d\n", #call, got_, want); \
      ++failures;                                                                   \
    }                                                                               \
  } while (0)

int main() {
  void* const P = reinterpret_cast<void*>(0x10000);  // aligned, never dereferenced
  void* const Q = reinterpret_cast<void*>(0x10002);  // misaligned
  float* const F = static_cast<float*>(P);
  int32_t* const I32 = static_cast<int32_t*>(P);
  for (int code = 1; code >= -12; --code)
    if (!oea_status_string(code) || !std::strlen(oea_status_string(code))) ++failures;
  // sizes at and beyond every limit: no overflow in the size arithmetic
  if (oea_workspace_bytes(OEA_MAX_B, OEA_MAX_D, OEA_MAX_N, OEA_MAX_D, OEA_MAX_K) == 0) ++failures;
  EXPECT((int)oea_workspace_bytes(0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff), 0);
  EXPECT((int)oea_workspace_bytes(-1, 8, 8, 8, 1), 0);
  EXPECT(oea_workspace_init(nullptr, 1 << 20, nullptr), OEA_ERR_NULL);
  EXPECT(oea_workspace_init(Q, 1 << 20, nullptr), OEA_ERR_ALIGN);
  EXPECT(oea_workspace_init(P, 16, nullptr), OEA_ERR_WORKSPACE);
  EXPECT(oea_workspace_check(nullptr, 1 << 20, nullptr), OEA_ERR_NULL);
  EXPECT(oea_workspace_check(P, 16, nullptr), OEA_ERR_WORKSPACE);
  EXPECT(oea_route(nullptr, 16, 128, 8, 3, I32, F, I32, I32, I32, nullptr), OEA_ERR_NULL);
  EXPECT(oea_route(F, 0, 128, 8, 3, I32, F, I32, I32, I32, nullptr), OEA_ERR_SHAPE);
  EXPECT(oea_route(F, 16, 0x7fffffff, 8, 3, I32, F, I32, I32, I32, nullptr), OEA_ERR_SHAPE);
  EXPECT(oea_route(F, 16, 128, 8, 9, I32, F, I32, I32, I32, nullptr), OEA_ERR_K);
  EXPECT(oea_route(F, 16, 128, -2147483647 - 1, 1, I32, F, I32, I32, I32, nullptr), OEA_ERR_K);
  EXPECT(oea_route_batched(F, nullptr, 0, 16, 128, 8, 3, I32, F, I32, I32, I32, nullptr), OEA_ERR_SHAPE);
  EXPECT(oea_route_batched(F, nullptr, 0x7fffffff, 16, 128, 8, 3, I32, F, I32, I32, I32, nullptr), OEA_ERR_SHAPE);
  EXPECT(oea_route_general(F, nullptr, 16, 128, 3, 0.0, 8, 128, I32, F, I32, nullptr, I32, I32, nullptr), OEA_ERR_K);
  EXPECT(oea_route_general(F, nullptr, 16, 128, 3, 0.5, 0x7fffffff, 128, I32, F, I32, nullptr, I32, I32, nullptr), OEA_ERR_K);
  EXPECT(oea_route_general(F, nullptr, 16, 128, 3, 0.5, 8, 0, I32, F, I32, nullptr, I32, I32, nullptr), OEA_ERR_K);
  const size_t big = (size_t)1 << 40;
  EXPECT(moe_decode(nullptr, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, P, big, nullptr), OEA_ERR_NULL);
  EXPECT(moe_decode(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, nullptr, big, nullptr), OEA_ERR_NULL);
  EXPECT(moe_decode(P, P, P, P, P, F, 16, 2052, 128, 768, 8, 3, OEA_BF16, P, big, nullptr), OEA_ERR_SHAPE);
  EXPECT(moe_decode(P, P, P, P, P, F, 16, 0x7ffffff8, 128, 0x7ffffff8, 8, 3, OEA_BF16, P, big, nullptr), OEA_ERR_SHAPE);
  EXPECT(moe_decode(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 0, OEA_BF16, P, big, nullptr), OEA_ERR_K);
  EXPECT(moe_decode(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, 5, P, big, nullptr), OEA_ERR_DTYPE);
  EXPECT(moe_decode(Q, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, P, big, nullptr), OEA_ERR_ALIGN);
  EXPECT(moe_decode(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, Q, big, nullptr), OEA_ERR_ALIGN);
  EXPECT(moe_decode(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, P, 1024, nullptr), OEA_ERR_WORKSPACE);
  oea_decode_ex ex;
  std::memset(&ex, 0, sizeof ex);
  EXPECT(moe_decode_ex(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, P, 1024, nullptr, &ex), OEA_ERR_WORKSPACE);
  ex.deterministic = 1;  // needs the larger workspace
  EXPECT(moe_decode_ex(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, P, oea_workspace_bytes(16, 2048, 128, 768, 8),
                       nullptr, &ex),
         OEA_ERR_WORKSPACE);
  if (oea_workspace_bytes_deterministic(16, 2048, 128, 768, 8) !=
      oea_workspace_bytes(16, 2048, 128, 768, 8) + (size_t)16 * 8 * 2048 * 4)
    ++failures;
  EXPECT(moe_decode_static(P, P, P, P, P, F, 128, 4096, 128, 1536, 8, 3, OEA_BF16, nullptr, &ex), OEA_ERR_LIMIT);
  ex.deterministic = 0;
  oea_test_opts opts;
  std::memset(&opts, 0, sizeof opts);
  opts.kernel_path = 7;
  EXPECT(moe_decode_test(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, P, big, nullptr, &ex, &opts), OEA_ERR_SHAPE);
  opts.kernel_path = -1;
  EXPECT(moe_decode_test(P, P, P, P, P, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, P, big, nullptr, nullptr, &opts), OEA_ERR_SHAPE);
  EXPECT(moe_decode_static(P, P, P, P, nullptr, F, 16, 2048, 128, 768, 8, 3, OEA_BF16, nullptr, nullptr), OEA_ERR_NULL);
  EXPECT(moe_decode_static(P, P, P, P, P, F, 1024, 4096, 128, 1536, 8, 3, OEA_BF16, nullptr, nullptr), OEA_ERR_LIMIT);
  EXPECT(moe_decode_static(P, P, P, P, P, F, 1024, 8192, 512, 8192, 32, 32, OEA_BF16, nullptr, &ex), OEA_ERR_LIMIT);
  EXPECT(oea_read_probe(nullptr, 1 << 20, nullptr, nullptr), OEA_ERR_NULL);
  EXPECT(oea_read_probe(P, 100, nullptr, nullptr), OEA_ERR_SHAPE);
  if (failures) {
    std::printf("abi sanitize: FAILED (%d)\n", failures);
    return 1;
  }
  std::printf("abi sanitize: ok\n");
  return 0;
}
