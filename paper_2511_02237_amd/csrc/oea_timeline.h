// Optional phase timeline of the layer kernels.  The product build compiles every OEA_TL(slot) to
// nothing.  A build with -DOEA_TIMELINE keeps, for every workgroup, the 100 MHz wall clock at which
// its thread 0 passed each stamp of the LAST kernel launched, in a device array of the library's
// own (no caller buffer is touched), and exports oea_timeline_read to copy it to the host.
#pragma once
#ifdef OEA_TIMELINE
namespace oea {
namespace {
constexpr int kTlSlots = 24;
constexpr int kTlWgs = 256;
__device__ unsigned long long g_timeline[kTlSlots * kTlWgs];
}  // namespace
}  // namespace oea
#define OEA_TL(slot_)                                                                       \
  do {                                                                                      \
    if (threadIdx.x == 0 && blockIdx.x < oea::kTlWgs)                                       \
      oea::g_timeline[(slot_) * oea::kTlWgs + blockIdx.x] = wall_clock64();                 \
  } while (0)
// record a value instead of the clock (the row cuts of the workgroup)
#define OEA_TL_VAL(slot_, v_)                                                               \
  do {                                                                                      \
    if (threadIdx.x == 0 && blockIdx.x < oea::kTlWgs)                                       \
      oea::g_timeline[(slot_) * oea::kTlWgs + blockIdx.x] = (unsigned long long)(v_);       \
  } while (0)
// wait for this wavefront's outstanding memory operations, then stamp (measures their drain)
#define OEA_TL_DRAINED(slot_)                          \
  do {                                                 \
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   \
    OEA_TL(slot_);                                     \
  } while (0)
#else
#define OEA_TL(slot_) \
  do {                \
  } while (0)
#define OEA_TL_VAL(slot_, v_) \
  do {                        \
  } while (0)
#define OEA_TL_DRAINED(slot_) \
  do {                        \
  } while (0)
#endif

// Stamps of the single-kernel layer (moe_fused_kernel):
//   0 kernel entered                1 logits stored, x staged       2 grid barrier passed
//   3 candidate keys in registers   4 Phase 1 done, union complete  5 Phase 2 and weights done
//   6 CSR offsets done              7 routing and row cuts done (gate/up stage begins)
//   8 gate/up rows streamed, results written   9 completion announced
//  10 first down tiles requested   11 hidden vectors of own experts complete   12 ... staged in LDS
//  13 down rows streamed, adds into out issued   14 those adds drained
//  16..19 values: first and end row of the workgroup in the gate/up stage, then in the down stage
