/*
 * xy_probe.h -- measurement helpers of the attention meta-kernel library for MI355X (gfx950).
 *
 * Instruments, not part of the attention path: small kernels that show what this GPU reaches on the two resources
 * the path is priced against (a plain streaming read of HBM, back-to-back bf16 MFMAs), and what the instructions
 * between the MFMAs of a lone wavefront cost, which is what the placement of the vector work in the wide units of
 * xy_attn_run is derived from.  bench.py prints their results next to the path's own figures.
 * Status codes and conventions as in xy_attn.h.
 */
#ifndef XY_PROBE_H
#define XY_PROBE_H

#include "xy_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Each enqueues one launch on hip_stream and returns; time them with events.
 *   xy_probe_stream_read: every byte of src[0 .. bytes) (device, 16-byte aligned, bytes a multiple of
 *     16) is read once with 16-byte loads by a grid that fills the chip; sink (device, >= 4 bytes) receives
 *     a checksum so the loads cannot be dropped.
 *   xy_probe_mfma: 2048 wavefronts (two per SIMD) issue iters x 16 independent
 *     v_mfma_f32_32x32x16_bf16 each: 2048 * iters * 16 * 32768 FLOPs; sink (device, >= 4 bytes) as above.
 * Errors: XY_ERR_ARG, XY_ERR_HIP. */
int xy_probe_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream);
/* The same read with the non-temporal hint on every load (data that is read once), which is how the
 * bandwidth-bound units of xy_attn_run fetch K and V. */
int xy_probe_stream_read_once(const void* src, size_t bytes, void* sink, void* hip_stream);
int xy_probe_mfma(int32_t iters, void* sink, void* hip_stream);

/* What the instructions between the MFMAs of a lone wavefront cost (the wide units run one wavefront per SIMD).
 * 256 workgroups of four wavefronts, one per SIMD, each issue iters x 32 v_mfma_f32_32x32x16_bf16 (1024 cycles
 * of the matrix pipe per 32) with, between them:
 *   XY_MIX_NONE        nothing
 *   XY_MIX_EVEN_4      four v_fma_f32 behind every MFMA
 *   XY_MIX_UNEVEN_8_0  the same eight per pair, all behind the first MFMA of the pair
 *   XY_MIX_DOT2        one v_dot2c_f32_bf16 behind every MFMA
 *   XY_MIX_SCALAR_2    three v_fma_f32 and two s_add_u32 behind every MFMA
 *   XY_MIX_ATTENTION   one v_exp_f32, two v_fma_f32 and (three times of four) a 16-byte LDS read per lane
 * cycles (device, 8-byte aligned, 1024 x uint64) receives, per wavefront, the shader-clock ticks of the whole
 * loop; divide by iters.  sink (device, >= 4 bytes) as above.  Errors: XY_ERR_ARG (unknown mix too), XY_ERR_HIP. */
enum { XY_MIX_NONE = 0, XY_MIX_EVEN_4 = 1, XY_MIX_UNEVEN_8_0 = 2, XY_MIX_DOT2 = 3, XY_MIX_SCALAR_2 = 4,
       XY_MIX_ATTENTION = 5 };
int xy_probe_issue_mix(int32_t mix, int32_t iters, void* cycles, void* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XY_PROBE_H */
