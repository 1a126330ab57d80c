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

/* Alternative limb widths for the Montgomery product, timed against the shipped
 * 29-bit core: one big integer per lane, `iters` dependent products
 * x <- x * y / R mod n (x <- x^2 / R for the squaring kind) per lane, R = 2 to the
 * power (limbs * limb_bits). Every array is in the variant's own radix, least
 * significant limb first: `limbs` uint32 per element for the integer kinds,
 * `limbs` doubles (each an integer below 2^23) for HAFLO_LIMBS_23_FMA64; d_x, d_y,
 * d_out hold `count` elements, d_n one (odd, below R / 2^10). n0inv = -1/n modulo
 * 2^limb_bits. Operand limbs below 2^limb_bits, values below 2n; results are
 * below 2n, limbs slightly above 2^limb_bits allowed (29-bit kinds), and are to
 * be reduced modulo n by the caller. */
enum haflo_peak_limb_kind {
  HAFLO_LIMBS_29_MAD64 = 0,        /* the shipped core: v_mad_u64_u32 into 64-bit columns, 18 limbs */
  HAFLO_LIMBS_29_MAD64_SQUARE = 1, /* its squaring, which leaves out the symmetric half (d_y unused) */
  HAFLO_LIMBS_24_MUL24 = 2,        /* v_mul_u32_u24 + v_mul_hi_u32_u24 per limb product, 22 limbs */
  HAFLO_LIMBS_23_FMA64 = 3         /* one FP64 FMA per limb product, 23 limbs held in doubles */
};
int haflo_peak_limbs(int kind, uint32_t* limbs, uint32_t* limb_bits);
int haflo_peak_montmul_chain(int kind, const void* d_x, const void* d_y, const void* d_n, uint64_t n0inv, int iters,
                             void* d_out, size_t count, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HAFLO_PEAK_H */
