/*
 * dta_probe.h - C ABI of libdta_probe.so: two measurement kernels used by the
 * benchmark to put a measured ceiling beside the published peak that the
 * attention kernels are priced against.  They are not part of the method and
 * not part of libdta.so.  Status codes are those of dta.h.
 */
#ifndef DTA_PROBE_H_
#define DTA_PROBE_H_

#include <stddef.h>
#include <stdint.h>

#include "dta.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * dta_probe_mfma_bf16 - measurement helper, not part of the method: enqueues a
 * kernel that does nothing but bf16 matrix-core products (the instruction and
 * block shape of the attention kernels, register operands, no memory traffic)
 * so that a caller who times it gets the rate the matrix pipes of this GPU
 * sustain under its power limit, the practical ceiling beside the published
 * peak that the roofline of the attention kernels is priced against.
 *
 * n_blocks blocks of 256 threads, `iters` iterations of 16 products per wave.
 * out   [n_blocks * 256] fp32, device: written (keeps the work observable).
 * ticks [2 * n_blocks] uint64, device: per block, the shader-clock cycles and
 *       the constant-rate wall-clock ticks the loop took; their ratio times
 *       the wall-clock rate gives the shader clock during the run.
 * *flop (host, may be NULL) receives the floating-point operations of the
 * launch: n_blocks * 4 waves * iters * 16 * (2*32*32*16).
 * *wall_clock_khz (host, may be NULL) receives the rate of the wall-clock
 * counter on the current device.
 * Asynchronous on hip_stream; allocates nothing.  INVALID_ARG for null buffers,
 * n_blocks outside [1, 2^20] or iters outside [1, 2^24].
 */
int dta_probe_mfma_bf16(int32_t n_blocks, int32_t iters, float* out, uint64_t* ticks, void* hip_stream,
                        int64_t* flop, int32_t* wall_clock_khz);

/*
 * dta_probe_overlap - measurement helper, not part of the method: how much of
 * the vector-ALU work of one wave does the hardware hide behind the matrix
 * products of ANOTHER wave on the same SIMD?  Enqueues n_blocks blocks of 8
 * waves (two per SIMD): waves 0-3 do mfma_iters x 16 bf16 matrix products, waves
 * 4-7 do valu_iters x 64 v_exp_f32, all on registers.  The caller times three
 * launches (valu_iters = 0, mfma_iters = 0, both); `both` between max and sum of
 * the other two says how far any schedule of the attention kernels, whose time
 * is products plus exponentials, can go.
 * out [n_blocks * 512] fp32, device: written.  Asynchronous on hip_stream;
 * allocates nothing.  INVALID_ARG for a null buffer, n_blocks outside [1, 2^20]
 * or an iteration count outside [0, 2^24].
 */
int dta_probe_overlap(int32_t n_blocks, int32_t mfma_iters, int32_t valu_iters, float* out,
                      void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DTA_PROBE_H_ */
