// C ABI of liboea: argument checks, workspace carving, kernel enqueue.  See include/oea.h.
#include <hip/hip_runtime.h>

#include <mutex>

#include "oea_internal.h"

namespace oea {

static size_t align256(size_t v) { return (v + 255) & ~size_t(255); }
// control words at the start of a workspace (zeroed by init): 1024 barrier/flag words, then one
// 128-byte line per expert for the completion counters (128 experts) and as many unused lines
static constexpr size_t kCtrlWords = 1024 + 2 * 128 * 32 + 3 * 256;  // see WsLayout::ctrl

WsLayout ws_layout(int B, int d, int N, int I, int k, int elem_bytes) {
  WsLayout w{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = align256(off + bytes);
    return at;
  };
  const size_t P = (size_t)B * k;
  w.ctrl = take(kCtrlWords * sizeof(uint32_t));
  w.logits = take((size_t)B * N * sizeof(float));
  w.expert_idx = take(P * sizeof(int32_t));
  w.gate_w = take(P * sizeof(float));
  w.n_sel = take((size_t)B * sizeof(int32_t));
  w.active_list = take((size_t)N * sizeof(int32_t));
  w.n_active = take(sizeof(int32_t));
  w.grp_off = take((size_t)(N + 1) * sizeof(int32_t));
  w.grp_tok = take(P * sizeof(int32_t));
  w.grp_gw = take(P * sizeof(float));
  w.h = take(P * (size_t)I * elem_bytes);
  w.grp_pos = take(P * sizeof(int32_t));
  w.total = off;
  w.y = take(P * (size_t)d * sizeof(float));
  w.total_with_y = off;
  return w;
}

static int check_route_sizes(int B, int N, int k, int k0) {
  if (B < 1 || B > OEA_MAX_B || N < 1 || N > OEA_MAX_N) return OEA_ERR_SHAPE;
  if (k0 < 1 || k0 > k || k > N || k > OEA_MAX_K) return OEA_ERR_K;
  return OEA_OK;
}

// batches above this run their expert stages on the matrix cores (three-kernel path)
static constexpr int kDenseFromBatch = 128;

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace oea

using namespace oea;

extern "C" const char* oea_status_string(int status) {
  switch (status) {
    case OEA_OK: return "ok";
    case OEA_ERR_NULL: return "a required pointer is NULL";
    case OEA_ERR_SHAPE: return "shape out of range (B, N, d or I)";
    case OEA_ERR_K: return "need 1 <= k0 <= k <= min(N, OEA_MAX_K)";
    case OEA_ERR_ALIGN: return "pointer not 16-byte aligned";
    case OEA_ERR_WORKSPACE: return "workspace too small";
    case OEA_ERR_DTYPE: return "unknown dtype";
    case OEA_ERR_HIP: return "HIP runtime error";
    case OEA_ERR_TIMEOUT: return "a bounded wait inside a kernel gave up";
    case OEA_ERR_LIMIT: return "sizes need more scratch than the allocation-free entry point has built in";
    case OEA_ERR_WORKSPACE_STATE: return "workspace not prepared by oea_workspace_init (or overwritten since)";
    default: return "unknown status";
  }
}

static int elem_bytes_of(int dt) { return dt == OEA_F32 ? 4 : dt == OEA_BF16 ? 2 : 0; }

static int check_decode_sizes(int B, int d, int N, int I, int k, int k0, int dt) {
  const int eb = elem_bytes_of(dt);
  if (eb == 0) return OEA_ERR_DTYPE;
  int rc = check_route_sizes(B, N, k, k0);
  if (rc != OEA_OK) return rc;
  // fp32 rows are twice as many 16-byte granules: half the bf16 limit
  const int max_dim = dt == OEA_F32 ? OEA_MAX_D / 2 : OEA_MAX_D;
  if (d < 8 || I < 8 || (d % 8) != 0 || (I % 8) != 0 || d > max_dim || I > max_dim) return OEA_ERR_SHAPE;
  return OEA_OK;
}

extern "C" size_t oea_workspace_bytes(int B, int d, int N, int I, int k) {
  if (B < 1 || B > OEA_MAX_B || N < 1 || N > OEA_MAX_N || k < 1 || k > OEA_MAX_K || d < 1 || I < 1 ||
      d > OEA_MAX_D || I > OEA_MAX_D)
    return 0;
  return ws_layout(B, d, N, I, k, 4).total;  // sized for the wider storage type
}

extern "C" size_t oea_workspace_bytes_deterministic(int B, int d, int N, int I, int k) {
  if (oea_workspace_bytes(B, d, N, I, k) == 0) return 0;
  return ws_layout(B, d, N, I, k, 4).total_with_y;
}

extern "C" int oea_read_probe(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf) return OEA_ERR_NULL;
  if (!aligned16(buf)) return OEA_ERR_ALIGN;
  if (bytes < (size_t)1 << 20) return OEA_ERR_SHAPE;
  hipError_t e = launch_read_probe(buf, bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OEA_OK : OEA_ERR_HIP;
}

extern "C" int oea_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return OEA_ERR_NULL;
  if (!aligned16(workspace)) return OEA_ERR_ALIGN;
  if (workspace_bytes < oea::kCtrlWords * sizeof(uint32_t)) return OEA_ERR_WORKSPACE;
  hipError_t e =
      launch_ws_prepare(static_cast<uint32_t*>(workspace), oea::kCtrlWords, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OEA_OK : OEA_ERR_HIP;
}

extern "C" int oea_workspace_check(const void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace) return OEA_ERR_NULL;
  if (!aligned16(workspace)) return OEA_ERR_ALIGN;
  if (workspace_bytes < oea::kCtrlWords * sizeof(uint32_t)) return OEA_ERR_WORKSPACE;
  static_assert(oea::kCtrlMagicWord == oea::kCtrlErrWord + 1, "the two words are read with one copy");
  uint32_t words[2] = {0, 0};  // error flag (set by a workgroup whose wait ran out), magic word
  if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return OEA_ERR_HIP;
  if (hipMemcpy(words, static_cast<const uint32_t*>(workspace) + oea::kCtrlErrWord, sizeof(words),
                hipMemcpyDeviceToHost) != hipSuccess)
    return OEA_ERR_HIP;
  if (words[1] != oea::kWsMagic) return OEA_ERR_WORKSPACE_STATE;
  return words[0] ? OEA_ERR_TIMEOUT : OEA_OK;
}

extern "C" int oea_route(const float* router_logits, int B, int N, int k, int k0, int32_t* expert_idx,
                         float* gate_w, int32_t* n_sel, int32_t* active_list, int32_t* n_active,
                         void* stream) {
  if (!router_logits || !expert_idx || !gate_w || !n_sel || !active_list || !n_active) return OEA_ERR_NULL;
  int rc = check_route_sizes(B, N, k, k0);
  if (rc != OEA_OK) return rc;
  RouteOut o{expert_idx, gate_w, n_sel, active_list, n_active, nullptr, nullptr, nullptr};
  hipError_t e = launch_route(router_logits, nullptr, 1, B, N, k, k0, o, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OEA_OK : OEA_ERR_HIP;
}

extern "C" int oea_route_batched(const float* router_logits, const uint8_t* token_mask, int L, int B, int N, int k,
                                 int k0, int32_t* expert_idx, float* gate_w, int32_t* n_sel, int32_t* active_list,
                                 int32_t* n_active, void* stream) {
  if (!router_logits || !expert_idx || !gate_w || !n_sel || !active_list || !n_active) return OEA_ERR_NULL;
  if (L < 1 || L > OEA_MAX_POSITIONS) return OEA_ERR_SHAPE;
  int rc = check_route_sizes(B, N, k, k0);
  if (rc != OEA_OK) return rc;
  RouteOut o{expert_idx, gate_w, n_sel, active_list, n_active, nullptr, nullptr, nullptr};
  hipError_t e = launch_route(router_logits, token_mask, L, B, N, k, k0, o, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OEA_OK : OEA_ERR_HIP;
}

extern "C" int oea_route_general(const float* router_logits, const uint8_t* token_mask, int B, int N, int k0,
                                 double p, int k_max, int max_p, int32_t* expert_idx, float* gate_w,
                                 int32_t* n_sel, int32_t* n_base, int32_t* active_list, int32_t* n_active,
                                 void* stream) {
  if (!router_logits || !expert_idx || !gate_w || !n_sel || !active_list || !n_active) return OEA_ERR_NULL;
  if (B < 1 || B > OEA_MAX_B || N < 1 || N > OEA_MAX_N) return OEA_ERR_SHAPE;
  const int kw = k0 > k_max ? k0 : k_max;
  if (k0 < 1 || k0 > N || k_max < 1 || k_max > N || kw > OEA_MAX_K || max_p < 1 || max_p > N || !(p > 0.0) ||
      p > 1.0)
    return OEA_ERR_K;
  RouteOut o{expert_idx, gate_w, n_sel, active_list, n_active, nullptr, nullptr, nullptr};
  const oea::RouteGeneralArgs ga{p, k_max, max_p};
  hipError_t e = launch_route_general(router_logits, token_mask, B, N, k0, ga, n_base, o,
                                      static_cast<hipStream_t>(stream));
  return e == hipSuccess ? OEA_OK : OEA_ERR_HIP;
}

// Argument checks shared by the layer entry points (everything but the workspace).
static int check_decode_args(const void* x, const void* W_router, const void* W_gate, const void* W_up,
                             const void* W_down, const float* out, int B, int d, int N, int I, int k, int k0,
                             int dt) {
  if (!x || !W_router || !W_gate || !W_up || !W_down || !out) return OEA_ERR_NULL;
  int rc = check_decode_sizes(B, d, N, I, k, k0, dt);
  if (rc != OEA_OK) return rc;
  if (!aligned16(x) || !aligned16(W_router) || !aligned16(W_gate) || !aligned16(W_up) || !aligned16(W_down) ||
      !aligned16(out))
    return OEA_ERR_ALIGN;
  return OEA_OK;
}

// The extras' numeric fields: a negative or NaN top_p and a negative max_p mean nothing.
static int check_extras(const oea_decode_ex* ex) {
  if (!ex) return OEA_OK;
  if (!(ex->top_p >= 0.0) || ex->max_p < 0) return OEA_ERR_K;
  return OEA_OK;
}

// workspace bytes a call needs: more with the deterministic combine
static size_t workspace_need(int B, int d, int N, int I, int k, const oea_decode_ex* ex) {
  return ex && ex->deterministic ? oea_workspace_bytes_deterministic(B, d, N, I, k) : oea_workspace_bytes(B, d, N, I, k);
}

// The layer on a checked workspace: carve it, enqueue the kernels and the taps.
static int decode_enqueue(const void* x, const void* W_router, const void* W_gate, const void* W_up,
                          const void* W_down, float* out, int B, int d, int N, int I, int k, int k0, int dt_checked,
                          void* workspace, void* stream, const oea_decode_ex* ex,
                          const oea_test_opts* opts = nullptr) {
  const oea_dtype dt = dt_checked == OEA_F32 ? OEA_F32 : OEA_BF16;  // check_decode_args has seen it
  const int path = opts ? opts->kernel_path : 0;
  if (path < 0 || path > 4) return OEA_ERR_SHAPE;
  const WsLayout w = ws_layout(B, d, N, I, k, elem_bytes_of(dt));
  char* ws = static_cast<char*>(workspace);
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* logits = reinterpret_cast<float*>(ws + w.logits);
  RouteOut ro{reinterpret_cast<int32_t*>(ws + w.expert_idx), reinterpret_cast<float*>(ws + w.gate_w),
              reinterpret_cast<int32_t*>(ws + w.n_sel),      reinterpret_cast<int32_t*>(ws + w.active_list),
              reinterpret_cast<int32_t*>(ws + w.n_active),   reinterpret_cast<int32_t*>(ws + w.grp_off),
              reinterpret_cast<int32_t*>(ws + w.grp_tok),    reinterpret_cast<float*>(ws + w.grp_gw),
              reinterpret_cast<int32_t*>(ws + w.grp_pos)};
  // deterministic combine: the down stage adds each pair's weighted result into a row of its own
  // (zeroed first; a single add per element, so the order of the adds cannot matter), and a last
  // kernel sums the rows of every token in slot order
  float* const y = ex && ex->deterministic ? reinterpret_cast<float*>(ws + w.y) : nullptr;
  Grouping g{ro.active_list, ro.n_active, ro.grp_off, ro.grp_tok, ro.grp_gw};
  void* h = ws + w.h;

  hipEvent_t* ev = opts && opts->h_kernel_events ? reinterpret_cast<hipEvent_t*>(opts->h_kernel_events) : nullptr;
  auto mark = [&](int i) { return !ev || hipEventRecord(ev[i], s) == hipSuccess; };

  // general OEA (Algorithm 2) only if the extras ask for it; k is then k_max
  oea::RouteGeneralArgs ga{1.0, k, N};
  if (ex && ex->top_p > 0.0 && ex->top_p < 1.0) ga.p = ex->top_p;
  if (ex && ex->max_p > 0 && ex->max_p < N) ga.max_p = ex->max_p;
  const bool general = ga.p < 1.0 || ga.max_p < N;

  if (!mark(0)) return OEA_ERR_HIP;
  hipError_t e = hipErrorNotSupported;
  if (path == 0)
    e = try_launch_fused(x, W_router, W_gate, W_up, W_down, ex ? ex->router_bias : nullptr,
                         ex ? ex->token_mask : nullptr, out, logits, h, ro,
                         reinterpret_cast<uint32_t*>(ws + w.ctrl), B, d, N, I, k, k0, dt, s,
                         opts ? opts->spin_limit : 0u, ex && ex->cooperative != 0, y, general ? &ga : nullptr);
  if (e == hipSuccess) {  // one kernel: the inner event pairs collapse onto its end
    for (int i = 1; i < 6; ++i)
      if (!mark(i)) return OEA_ERR_HIP;
  } else if (e != hipErrorNotSupported) {
    return OEA_ERR_HIP;
  } else {
    e = launch_router_and_route(x, W_router, ex ? ex->router_bias : nullptr, ex ? ex->token_mask : nullptr, B, d,
                                N, k, k0, dt, logits, y ? y : out, y ? (size_t)B * k * d : (size_t)B * d,
                                reinterpret_cast<uint32_t*>(ws + w.ctrl), ro, general ? &ga : nullptr, s);
    if (e != hipSuccess || !mark(1) || !mark(2)) return OEA_ERR_HIP;
    const bool stage_kernels = path == 0 || path == 3;
    const bool generic_only = path == 1;
    // matrix cores once an expert serves many tokens: above the single kernel's batch range
    const bool dense = path == 4 || (path == 0 && B > kDenseFromBatch);
    e = dense ? try_launch_dense_stage(0, x, W_gate, W_up, h, nullptr, B, d, N, I, k, dt, g, false, s)
              : hipErrorNotSupported;
    if (e == hipErrorNotSupported && stage_kernels)
      e = try_launch_stage_kernels(0, x, W_gate, W_up, h, nullptr, B, d, N, I, k, dt, g, false, s);
    if (e == hipErrorNotSupported) e = launch_expert_gate_up(x, W_gate, W_up, h, B, d, N, I, k, dt, g, generic_only, s);
    if (e != hipSuccess || !mark(3) || !mark(4)) return OEA_ERR_HIP;
    e = dense ? try_launch_dense_stage(1, h, W_down, nullptr, nullptr, y ? y : out, B, d, N, I, k, dt, g, y != nullptr, s)
              : hipErrorNotSupported;
    if (e == hipErrorNotSupported && stage_kernels)
      e = try_launch_stage_kernels(1, h, W_down, nullptr, nullptr, y ? y : out, B, d, N, I, k, dt, g, y != nullptr, s);
    if (e == hipErrorNotSupported)
      e = launch_expert_down(h, W_down, y ? y : out, B, d, N, I, k, dt, g, generic_only, y != nullptr, s);
    if (e != hipSuccess || !mark(5)) return OEA_ERR_HIP;
  }
  if (y && launch_combine(y, ro.grp_pos, ro.n_sel, out, B, d, k, s) != hipSuccess) return OEA_ERR_HIP;

  if (ex) {  // taps: device-to-device copies in stream order
    const size_t P = (size_t)B * k;
    struct { void* dst; const void* src; size_t bytes; } taps[] = {
        {ex->logits_out, logits, (size_t)B * N * sizeof(float)},
        {ex->expert_idx_out, ro.expert_idx, P * sizeof(int32_t)},
        {ex->gate_w_out, ro.gate_w, P * sizeof(float)},
        {ex->n_sel_out, ro.n_sel, (size_t)B * sizeof(int32_t)},
        {ex->active_list_out, ro.active_list, (size_t)N * sizeof(int32_t)},
        {ex->n_active_out, ro.n_active, sizeof(int32_t)},
    };
    for (auto& t : taps)
      if (t.dst && hipMemcpyAsync(t.dst, t.src, t.bytes, hipMemcpyDeviceToDevice, s) != hipSuccess)
        return OEA_ERR_HIP;
  }
  return OEA_OK;
}

extern "C" int moe_decode_ex(const void* x, const void* W_router, const void* W_gate, const void* W_up,
                             const void* W_down, float* out, int B, int d, int N, int I, int k, int k0,
                             int dt, void* workspace, size_t workspace_bytes, void* stream,
                             const oea_decode_ex* ex) {
  if (!workspace) return OEA_ERR_NULL;
  int rc = check_decode_args(x, W_router, W_gate, W_up, W_down, out, B, d, N, I, k, k0, dt);
  if (rc != OEA_OK) return rc;
  if (!aligned16(workspace)) return OEA_ERR_ALIGN;
  if ((rc = check_extras(ex)) != OEA_OK) return rc;
  if (workspace_bytes < workspace_need(B, d, N, I, k, ex)) return OEA_ERR_WORKSPACE;
  return decode_enqueue(x, W_router, W_gate, W_up, W_down, out, B, d, N, I, k, k0, dt, workspace, stream, ex);
}

extern "C" int moe_decode_test(const void* x, const void* W_router, const void* W_gate, const void* W_up,
                               const void* W_down, float* out, int B, int d, int N, int I, int k, int k0,
                               int dt, void* workspace, size_t workspace_bytes, void* stream,
                               const oea_decode_ex* ex, const oea_test_opts* opts) {
  if (!workspace) return OEA_ERR_NULL;
  int rc = check_decode_args(x, W_router, W_gate, W_up, W_down, out, B, d, N, I, k, k0, dt);
  if (rc != OEA_OK) return rc;
  if (!aligned16(workspace)) return OEA_ERR_ALIGN;
  if ((rc = check_extras(ex)) != OEA_OK) return rc;
  if (workspace_bytes < workspace_need(B, d, N, I, k, ex)) return OEA_ERR_WORKSPACE;
  return decode_enqueue(x, W_router, W_gate, W_up, W_down, out, B, d, N, I, k, k0, dt, workspace, stream, ex, opts);
}

extern "C" int moe_decode(const void* x, const void* W_router, const void* W_gate, const void* W_up,
                          const void* W_down, float* out, int B, int d, int N, int I, int k, int k0,
                          int dt, void* workspace, size_t workspace_bytes, void* stream) {
  return moe_decode_ex(x, W_router, W_gate, W_up, W_down, out, B, d, N, I, k, k0, dt, workspace,
                       workspace_bytes, stream, nullptr);
}

// ---------------------------------------------------------------------------------------------
// moe_decode_static: the layer for callers that cannot allocate device memory.  The workspace
// that moe_decode takes as an argument (control words, logits, routing result, hidden vectors) is
// a file-scope device array instead; every GPU the library runs on holds its own copy of it at
// its own address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the address that call returns, kept per device, is what the kernels get.
static __device__ __align__(256) unsigned char scratch[OEA_STATIC_SCRATCH_BYTES];

namespace {
struct StaticScratch {
  void* ptr = nullptr;    // device address of `scratch` on this device
  bool prepared = false;  // its control words have been cleared by a kernel on some stream
};
StaticScratch g_static[oea::kMaxDevices];
std::mutex g_static_mutex;
}  // namespace

extern "C" int moe_decode_static(const void* x, const void* W_router, const void* W_gate, const void* W_up,
                                 const void* W_down, float* out, int B, int d, int N, int I, int k, int k0,
                                 int dt, void* stream, const oea_decode_ex* ex) {
  int rc = check_decode_args(x, W_router, W_gate, W_up, W_down, out, B, d, N, I, k, k0, dt);
  if (rc != OEA_OK) return rc;
  if ((rc = check_extras(ex)) != OEA_OK) return rc;
  const size_t need = workspace_need(B, d, N, I, k, ex);
  if (need == 0 || need > (size_t)OEA_STATIC_SCRATCH_BYTES) return OEA_ERR_LIMIT;  // before any HIP call
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return OEA_ERR_HIP;
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticScratch& st = g_static[dev];
    if (!st.ptr) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return OEA_ERR_HIP;
      st.ptr = p;
    }
    if (!st.prepared) {
      // first call on this device: clear the control words with a kernel on the caller's stream,
      // ahead of the layer (what oea_workspace_init does for a caller-owned workspace).  Under
      // capture that kernel would only be recorded, not run: refuse.
      hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
      if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &cs) == hipSuccess && cs != hipStreamCaptureStatusNone)
        return OEA_ERR_HIP;
      if (launch_ws_prepare(static_cast<uint32_t*>(st.ptr), oea::kCtrlWords, static_cast<hipStream_t>(stream)) !=
          hipSuccess)
        return OEA_ERR_HIP;
      st.prepared = true;
    }
    ws = st.ptr;
  }
  return decode_enqueue(x, W_router, W_gate, W_up, W_down, out, B, d, N, I, k, k0, dt, ws, stream, ex);
}
