/*
 * cq_measure.h -- measurement hooks of libcq (not part of the method's call surface in cq.h): the layer with
 * per-stage timing, the device facts and the two yardsticks (streaming read, bare matrix-core loop) that
 * bench.py reports next to the nominal peaks.  Same conventions as cq.h.
 */
#ifndef CQ_MEASURE_H_
#define CQ_MEASURE_H_

#include "cq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement variant of cq_moe_forward: same launches, with HIP events recorded on `stream` at the
 * stage boundaries.  It waits for the last event (so, unlike cq_moe_forward, it synchronises the
 * host) and writes the elapsed milliseconds of the CQ_N_STAGES stages to stage_ms (host memory):
 * [0] rotate+quantize, [1] route+permute, [2] gate/up product, [3] down product, [4] combine.
 */
#define CQ_N_STAGES 5
cq_status cq_moe_forward_timed(const cq_layer* L, const float* X, int T, float* Y,
                               void* workspace, size_t workspace_bytes, cq_stream stream,
                               float* stage_ms);

/* Device facts used for rooflines: writes CU count, max clock (kHz), memory clock (kHz), memory
 * bus width (bits), LDS bytes per workgroup. Returns CQ_ERR_HIP when no device is present. */
cq_status cq_device_info(int* cu_count, int* clock_khz, int* mem_clock_khz, int* bus_bits, int* lds_bytes);

/* Streaming read of `bytes` bytes (16-byte multiples) used to measure the achievable HBM read ceiling next
 * to the nominal one, with the access pattern of the product kernel's index stream: one workgroup of 8
 * wavefronts per contiguous 512 KiB, contiguous KiB per wavefront load, non-temporal, 8 loads in flight per
 * wavefront.  sink[0..3] exists to keep the loads alive (written only for one XOR value in 2^32). */
cq_status cq_stream_read(const void* src, size_t bytes, uint32_t* sink, cq_stream stream);

/* Bare matrix-core loop used to measure the achievable dense bf16 MFMA ceiling next to the nominal
 * one: `workgroups` workgroups of 4 wavefronts, each wavefront issuing iters x 16 independent
 * v_mfma_f32_32x32x16_bf16 (32768 flops each) on register operands.  sink[workgroups * 256] f32
 * receives one value per thread (keeps the loop alive).  Flops = workgroups * 4 * iters * 16 * 32768. */
cq_status cq_mfma_loop(int workgroups, int iters, float* sink, cq_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CQ_MEASURE_H_ */
