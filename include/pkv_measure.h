/*
 * pkv_measure.h -- test and measurement aids of libpkv.  Nothing here is part
 * of the method (arXiv 2406.02069) or needed in production; benchmarks and
 * tests include it next to pkv.h.
 */
#ifndef PKV_MEASURE_H_
#define PKV_MEASURE_H_

#include "pkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Switches in pkv_layer_desc.flags (per call, taken from the first
 * descriptor of a multi-layer call; all descriptors must agree).
 */
typedef enum {
  /* score with the per-layer streaming kernels (K read twice) even where the
     register-resident kernel would serve the shape: lets tests run both */
  PKV_FLAG_STREAM_SCORING = 1,
  /* exchange the softmax statistics through the arrival counter where the
     tagged exchange would be used (units of 4 parts or more) */
  PKV_FLAG_COUNTER_EXCHANGE = 2,
  /* every bounded wait between workgroups gives up at once: forces, from the
     host, the outcome a caller sees when the resident kernel's workgroups
     cannot be resident together (count_out = -1); every kernel still exits
     normally */
  PKV_FLAG_NO_WAIT = 4,
  PKV_FLAG_ALL = 7
} pkv_flags;

/*
 * Measurement aid (no part of the method): pkv_compress_layers (lse NULL)
 * or pkv_compress_layers_lse (lse given), compact (paged NULL) or paged
 * output (paged and block_tables given; K_out / V_out are then the page
 * pools), with the caller's HIP events recorded around the kernels, so that
 * a benchmark can attribute device time to each kernel without a profiler.
 *
 * events     HOST array of n_events hipEvent_t handles created by the caller
 *            with timing enabled.  events[0] is recorded on `stream` before
 *            the first kernel, events[i] after the i-th kernel launched.
 * kernel_ids HOST int32[n_events - 1], written: kernel_ids[i-1] is the
 *            pkv_kernel_id of the kernel between events[i-1] and events[i].
 * n_used     HOST int32, written: number of events recorded (kernels + 1).
 * The call does not synchronise; the caller synchronises the stream and
 * reads hipEventElapsedTime(events[i-1], events[i]).
 * Errors: as pkv_compress_layers; n_events too small for the launch
 * sequence (5 kernels per layer + 1) -> PKV_ERR_INVALID_ARG.
 */
typedef enum {
  PKV_KERNEL_SCORE_STATS = 0, /* sweep 1 over K: per-row softmax statistics */
  PKV_KERNEL_SCORE_FINALIZE = 1,
  PKV_KERNEL_SCORE_ACCUM = 2, /* sweep 2 over K: per-key window scores      */
  PKV_KERNEL_POOL_SELECT = 3,
  PKV_KERNEL_GATHER = 4,
  PKV_KERNEL_SCORE_RESIDENT = 5 /* both sweeps, K held in registers (all layers) */
} pkv_kernel_id;

int pkv_compress_layers_profiled(
    int32_t L, const pkv_layer_desc* descs, const void* const* Q_win,
    const void* const* K, const void* const* V, const float* const* lse,
    const int32_t* seq_lens, const pkv_paged_desc* paged,
    const int32_t* const* block_tables,
    void* const* K_out, void* const* V_out, int32_t* const* idx_out,
    int32_t* const* count_out, float* const* scores_out, void* workspace,
    size_t workspace_bytes, void* stream, void* const* events,
    int32_t n_events, int32_t* kernel_ids, int32_t* n_used);

/*
 * Measurement aid (no part of the method): streams `bytes` bytes starting at
 * `buf` from memory once, with 16-byte loads by a grid that fills the chip,
 * and discards them.  Timed by the caller (events or a synchronised clock), it
 * gives the read bandwidth this device reaches on a plain scan: the measured
 * ceiling beside the published peak in the roofline of the scoring kernel.
 *
 * buf    DEVICE pointer, 16-byte aligned, readable for `bytes` bytes.
 * bytes  multiple of 16, > 0.
 * sink   DEVICE uint32, written only if a checksum of the data takes one
 *        particular value (it keeps the loads alive); contents meaningless.
 * stream hipStream_t as void*.  Asynchronous; never allocates.
 * Returns PKV_OK, PKV_ERR_INVALID_ARG (null / misaligned / size) or
 * PKV_ERR_HIP.
 */
int pkv_probe_read(const void* buf, size_t bytes, uint32_t* sink,
                   void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PKV_MEASURE_H_ */
