/*
 * libhaflo_peak: the roofline denominators of the Paillier operator path,
 * measured on the part itself. Not part of the operator library; nothing in
 * libhaflo calls it. Each function enqueues one kernel on `stream` (a
 * hipStream_t) and returns 0, -1 for a bad argument, -4 for a HIP error; the
 * caller times the launch (bench_peak.py does, with HIP events).
 *
 * The operators' bound is the issue rate of the 32x32+64-bit integer
 * multiply-add (paper Section 4.2: modular exponentiation dominates); the
 * fixed-point encoders and decoders (paper Table 2, "Encoding" / "Decoding")
 * are bound by HBM traffic.
 */
#ifndef HAFLO_PEAK_H
#define HAFLO_PEAK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Instruction streams without memory traffic: every lane runs
 * haflo_peak_streams() independent dependency chains of `iters` iterations. */
enum haflo_peak_alu_kind {
  HAFLO_PEAK_MAD_U64_U32 = 0, /* one v_mad_u64_u32 per chain and iteration (the shipped limb product) */
  HAFLO_PEAK_MUL_LO_HI = 1,   /* one v_mul_lo_u32, one v_mul_hi_u32 and one add (32-bit limbs without a fused add) */
  HAFLO_PEAK_MUL_U24 = 2,     /* one v_mad_u32_u24 (24-bit limbs) */
  HAFLO_PEAK_FMA_F64 = 3,     /* one FP64 fused multiply-add (limbs in doubles) */
  HAFLO_PEAK_ADD_U32 = 4      /* one 32-bit add: a plain full-rate VALU instruction, for reference */
};
int haflo_peak_streams(void);
/* blocks: 256-lane workgroups; d_out: device, blocks * 256 uint32 (written once per lane). */
int haflo_peak_alu(int kind, int blocks, int iters, uint32_t* d_out, void* stream);

/* Plain HBM kernels, 16 bytes per lane and access, grid-stride over `bytes`
 * (a multiple of 16). FILL writes d_dst; COPY reads d_src and writes d_dst;
 * READ reads d_src (d_dst: at least 4 bytes, practically never written). */
enum haflo_peak_hbm_kind { HAFLO_PEAK_FILL = 0, HAFLO_PEAK_COPY = 1, HAFLO_PEAK_READ = 2 };
int haflo_peak_hbm(int kind, int blocks, void* d_dst, const void* d_src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HAFLO_PEAK_H */
