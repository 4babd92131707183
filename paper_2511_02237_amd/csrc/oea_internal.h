// Internal declarations shared by the translation units of liboea (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "oea.h"
#include "oea_testing.h"

namespace oea {

// Control words at the start of a workspace (see WsLayout::ctrl).  oea_workspace_init writes the
// magic word; the layer kernels look at it before they wait for anybody, so a workspace that was
// never prepared (or was overwritten) makes them return at once instead of spinning.
constexpr int kCtrlErrWord = 3;    // set by a workgroup whose bounded wait ran out
constexpr int kCtrlMagicWord = 4;  // kWsMagic on a prepared workspace
constexpr uint32_t kWsMagic = 0x4F454131u;
// Large batches route in several kernels over many workgroups; between them the union bit mask of
// Phase 1 and the number of pairs per expert live in control words that are otherwise unused (the
// first of these kernels clears them).
constexpr int kCtrlWideUnion = 5120;  // [16]  bit e % 32 of word e / 32: expert e is in the union
constexpr int kCtrlWideCount = 5152;  // counter of expert e at word e * wide_count_stride(N): atomics on one
                                      // 128-byte line execute one after the other, so the counters are spread out
constexpr int kCtrlWideCountWords = 9216 - kCtrlWideCount;
__host__ __device__ inline int wide_count_stride(int N) {
  const int s = kCtrlWideCountWords / (N > 0 ? N : 1);
  return s > 32 ? 32 : (s < 1 ? 1 : s);
}

// State that is looked up or set once per DEVICE (a process may drive several): indexed by the
// HIP device id of the calling thread's current device.
constexpr int kMaxDevices = 64;
struct PerDevice {
  std::atomic<int> v[kMaxDevices];  // zero-initialised for objects of static storage duration
};
// Current device and its number of compute units (cached per device).  Returns false if HIP fails.
bool current_device(int* dev, int* cus);
// hipFuncSetAttribute(max dynamic LDS) for `kern` on the current device, once per device (`done`
// belongs to that kernel); *dev_out receives the device id.
inline hipError_t ensure_dynamic_lds(const void* kern, int bytes, PerDevice& done, int* dev_out = nullptr) {
  int dev = 0, cus = 0;
  if (!current_device(&dev, &cus)) return hipErrorInvalidDevice;
  if (dev_out) *dev_out = dev;
  if (done.v[dev].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.v[dev].store(bytes, std::memory_order_relaxed);
  return e;
}

// Carving of the caller's workspace.  All offsets are multiples of 256 bytes.
struct WsLayout {
  size_t ctrl;         // uint32[1024 + 8192 + 768].  [9216..) is the fused kernel's load-balancing state (speed
                       // weights of the workgroups, adapted from call to call); [4] holds kWsMagic; the rest is zero
                       // between calls: [0] arrival counter of the router kernel, [3] error flag, [32], [64] and
                       // [256 + 32 i] grid-barrier words of the fused kernel, [1024..) its per-expert completion
                       // counters, one 128-byte line each; [5120..9216) union mask and pair counts of the
                       // several-kernel routing of large batches (kCtrlWideUnion, kCtrlWideCount)
  size_t logits;       // float [B,N]
  size_t expert_idx;   // int32 [B,k]
  size_t gate_w;       // float [B,k]
  size_t n_sel;        // int32 [B]
  size_t active_list;  // int32 [N]
  size_t n_active;     // int32 [1]
  size_t grp_off;      // int32 [N+1]  CSR offsets, indexed by position in active_list
  size_t grp_tok;      // int32 [B*k]  token of each (expert, token) pair, grouped by expert
  size_t grp_gw;       // float [B*k]  gate weight of that pair
  size_t h;            // storage type [B*k, I]  hidden activations of each pair
  size_t grp_pos;      // int32 [B*k]  position of (token, slot) in the grouped pair order, -1 for an unused slot
  size_t total;        // bytes without the area below (what oea_workspace_bytes reports)
  size_t y;            // float [B*k, d]  deterministic combine only: weighted down-projection of each pair
  size_t total_with_y; // what oea_workspace_bytes_deterministic reports
};

WsLayout ws_layout(int B, int d, int N, int I, int k, int elem_bytes);

// Device-side view of the routing results that the expert kernels consume.
struct Grouping {
  const int32_t* active_list;
  const int32_t* n_active;
  const int32_t* grp_off;
  const int32_t* grp_tok;
  const float* grp_gw;
};

struct RouteOut {
  int32_t* expert_idx;
  float* gate_w;
  int32_t* n_sel;
  int32_t* active_list;
  int32_t* n_active;
  int32_t* grp_off;  // may be nullptr (routing-only entry point)
  int32_t* grp_tok;  // may be nullptr
  float* grp_gw;     // may be nullptr
  int32_t* grp_pos;  // may be nullptr: [B*k] position of each (token, slot) in the grouped order
};

// parameters of the general OEA routing (Algorithm 2) beyond k0: top-p threshold, cap, rank window
struct RouteGeneralArgs {
  double p;
  int k_max;
  int max_p;
};

// launchers (each returns the hipError_t of the launch)
// zero the control words and write the magic word (a kernel, not a memset: captures stay valid)
hipError_t launch_ws_prepare(uint32_t* ctrl, size_t n_words, hipStream_t s);
// L independent positions: logits [L,B,N]; every output has a leading dimension L
hipError_t launch_route(const float* logits, const uint8_t* token_mask, int L, int B, int N, int k, int k0,
                        RouteOut o, hipStream_t s);
hipError_t launch_router_and_route(const void* x, const void* w_router, const float* bias,
                                   const uint8_t* token_mask, int B, int d, int N, int k, int k0,
                                   oea_dtype dt, float* logits, float* to_zero, size_t n_zero, uint32_t* counter,
                                   RouteOut o, const RouteGeneralArgs* general, hipStream_t s);
hipError_t launch_route_general(const float* logits, const uint8_t* token_mask, int B, int N, int k0,
                                const RouteGeneralArgs& ga, int32_t* n_base, RouteOut o, hipStream_t s);
// generic_only: skip the streaming kernels with fixed shares (test aid)
hipError_t launch_expert_gate_up(const void* x, const void* w_gate, const void* w_up, void* h, int B,
                                 int d, int N, int I, int k, oea_dtype dt, Grouping g, bool generic_only,
                                 hipStream_t s);
// per_pair: `out` is the [B*k, d] buffer of the deterministic combine; pair p adds its weighted result to row p
hipError_t launch_expert_down(const void* h, const void* w_down, float* out, int B, int d, int N, int I,
                              int k, oea_dtype dt, Grouping g, bool generic_only, bool per_pair, hipStream_t s);
// out[t, :] = sum over the slots of token t, in slot order, of y[grp_pos[t, slot], :]  (Eq. 1 in a fixed order)
hipError_t launch_combine(const float* y, const int32_t* grp_pos, const int32_t* n_sel, float* out, int B, int d,
                          int k, hipStream_t s);

// whole layer in one persistent kernel; hipErrorNotSupported if the shape is not one it is built for
hipError_t try_launch_fused(const void* x, const void* w_router, const void* w_gate, const void* w_up,
                            const void* w_down, const float* bias, const uint8_t* token_mask, float* out,
                            float* logits, void* h, RouteOut ro, uint32_t* ctrl, int B, int d, int N, int I,
                            int k, int k0, oea_dtype dt, hipStream_t s, uint32_t spin_limit = 0,
                            bool cooperative = false, float* y_per_pair = nullptr,
                            const RouteGeneralArgs* general = nullptr);

// one expert stage (0 gate/up, 1 down) with the fused kernel's stage code, for larger batches
hipError_t try_launch_stage_kernels(int stage, const void* vec, const void* wa, const void* wb, void* h_out,
                                    float* out, int B, int d, int N, int I, int k, oea_dtype dt, Grouping g,
                                    bool per_pair, hipStream_t s);

// one expert stage (0 gate/up, 1 down) on the matrix cores, for batches in which experts serve many tokens
hipError_t try_launch_dense_stage(int stage, const void* vec, const void* wa, const void* wb, void* h_out,
                                  float* out, int B, int d, int N, int I, int k, oea_dtype dt, Grouping g,
                                  bool per_pair, hipStream_t s);

hipError_t launch_read_probe(const void* buf, size_t bytes, uint32_t* sink, hipStream_t s);
size_t route_lds_bytes(int B, int N);

}  // namespace oea
