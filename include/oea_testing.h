/*
 * oea_testing.h - test and measurement aids of liboea.  Not part of the product interface
 * (include/oea.h): nothing here is needed to run the layer, and a serving stack should not
 * depend on it.  Same conventions as oea.h (device pointers, caller-owned buffers, stream as
 * void*, negative oea_status on error).
 */
#ifndef OEA_TESTING_H_
#define OEA_TESTING_H_

#include "oea.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-call switches for moe_decode_test; a zeroed struct changes nothing. */
typedef struct {
  int32_t kernel_path;    /* which expert-FFN kernels this call uses:
                               0 = automatic: the single fused kernel for the shapes and batch sizes
                                   it is built for, else three kernels (router + routing, gate/up,
                                   down) with the best expert kernels that apply
                               1 = three kernels, generic expert kernels only (any shape, any batch)
                               2 = three kernels, streaming expert kernels with fixed shares when
                                   the token vectors fit in LDS, else generic ones
                               3 = three kernels, the fused kernel's stage code as expert kernels
                                   where the shape allows
                               4 = three kernels, expert stages on the matrix cores where the shape
                                   allows (bf16; the automatic choice uses them above B = 128) */
  uint32_t spin_limit;    /* polls after which a wait inside the single kernel gives up
                             (0 = the default, about a second); 1 forces every wait to give up */
  void **h_kernel_events; /* HOST array of 6 hipEvent_t created by the caller, or NULL: recorded on
                             the stream before/after the router+routing kernel [0],[1], the gate/up
                             kernel [2],[3] and the down kernel [4],[5] (the single kernel: [0] before,
                             [1]..[5] after it) */
} oea_test_opts;

/*
 * moe_decode_ex (oea.h) with the switches above; ex and opts may each be NULL.
 * Errors as moe_decode_ex, and OEA_ERR_SHAPE for a kernel_path outside 0..4.
 */
int moe_decode_test(const void *x, const void *W_router, const void *W_gate, const void *W_up,
                    const void *W_down, float *out, int B, int d, int N, int I, int k, int k0,
                    int dt, void *workspace, size_t workspace_bytes, void *stream,
                    const oea_decode_ex *ex, const oea_test_opts *opts);

/*
 * Measurement aid: enqueue a kernel that reads `bytes` bytes (>= 1 MiB) at `buf` once, with the
 * access pattern the expert kernels stream weights with, and discards them.  Timing it over memory
 * that is not in any cache gives the practical read ceiling of the device, the yardstick next to
 * the published HBM peak.  `sink` (4 bytes of device memory, may be NULL) is never written in practice.
 */
int oea_read_probe(const void *buf, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* OEA_TESTING_H_ */
