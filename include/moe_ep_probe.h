/*
 * moe_ep_probe.h -- measurement aid of the benchmark, NOT part of the layer's library: a caller of
 * the layer links libmoe_ep.so (moe_ep.h) and never needs this.  Built as libmoe_ep_probe.so.
 */
#ifndef MOE_EP_PROBE_H
#define MOE_EP_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * What `device` sustains right now.  *mfma_tflops and *mfma_ghz: rate and shader clock of a
 * register-only v_mfma_f32_32x32x16_bf16 loop on all compute units (no LDS, no memory traffic;
 * operands are standard-normal bf16 values, or all zeros when zero_operands != 0 -- the part trades
 * clock for matrix-pipe activity under its power limit, so the two differ); *copy_gbs: bytes read
 * plus bytes written per second by a device-to-device copy of 512 MiB (twice the memory-side
 * cache).  Allocates and frees the copy's two buffers (1 GiB together) and a few KiB of operands,
 * runs on the default stream and returns when done (about 0.1 s).  Returns 0, -1 on NULL outputs
 * or a negative device, -3 if a HIP call fails.
 */
int moe_ep_probe_device(int32_t device, int32_t zero_operands, double *mfma_tflops, double *mfma_ghz,
                        double *copy_gbs);

#ifdef __cplusplus
}
#endif
#endif /* MOE_EP_PROBE_H */
