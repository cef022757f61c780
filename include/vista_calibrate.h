/*
 * libvista_calibrate -- calibration kernels of the benchmark (not part of the
 * product path and not linked into libvista.so).  They measure what one MI355X
 * sustains with the instructions the hot kernels are made of, so that every
 * roofline figure the benchmark prints can be reproduced: the achievable bf16
 * MFMA rate (and with it the shader clock under load), the achievable HBM read
 * bandwidth, and the vector-ALU issue-port cost of the softmax's instructions.
 * Both calls only enqueue one kernel on the given stream and return 0 on
 * success, 1 for bad arguments, 2 when the launch failed.  The caller times them.
 */
#ifndef VISTA_CALIBRATE_H
#define VISTA_CALIBRATE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Loop bodies of vista_calibrate_issue; the counts are per wave and iteration. */
enum {
  VISTA_CAL_EXP = 0,          /* 16 v_exp_f32                                            */
  VISTA_CAL_ADD = 1,          /* 16 v_add_f32                                            */
  VISTA_CAL_CVT = 2,          /* 8 v_cvt_pk_bf16_f32 (+ 8 v_add_f32 that feed them)      */
  VISTA_CAL_EXP_ADD = 3,      /* 16 v_exp_f32 + 16 independent v_add_f32                 */
  VISTA_CAL_MFMA = 4,         /* 4 independent v_mfma_f32_32x32x16_bf16                  */
  VISTA_CAL_MFMA_ADD16 = 5,   /* 4 MFMAs + 16 v_add_f32                                  */
  VISTA_CAL_MFMA_ADD32 = 6,   /* 4 MFMAs + 32 v_add_f32                                  */
  VISTA_CAL_MFMA_ADD48 = 7,   /* 4 MFMAs + 48 v_add_f32                                  */
  VISTA_CAL_MFMA_ADD64 = 8,   /* 4 MFMAs + 64 v_add_f32                                  */
  VISTA_CAL_MFMA_EXP16 = 9,   /* 4 MFMAs + 16 v_exp_f32                                  */
  VISTA_CAL_MFMA16 = 10,      /* 4 independent v_mfma_f32_16x16x32_bf16                  */
  VISTA_CAL_MFMA16_ADD32 = 11,/* 4 small MFMAs + 32 v_add_f32                            */
  VISTA_CAL_MFMA_AGPR_ADD32 = 12, /* as MFMA_ADD32 with the accumulators in AGPRs        */
  VISTA_CAL_MFMA4 = 13,       /* 16 v_mfma_f32_4x4x4_16b_bf16 on four accumulators       */
  VISTA_CAL_MFMA4_ADD32 = 14, /* 16 of those + 32 v_add_f32                              */
  VISTA_CAL_TILE_BODY = 15,   /* two query blocks of the stage-1 tile loop, registers only; per
                                 block 6 MFMAs, 16 v_exp_f32, 8 v_cvt_pk_bf16_f32, 4 4x4x4 MFMAs */
  VISTA_CAL_TILE_BODY_NOSMALL = 16, /* the same without the 4x4x4 MFMAs                       */
  VISTA_CAL_TILE_BODY_NOPROJ = 17,  /* the same without the two projection MFMAs per block    */
  VISTA_CAL_TILE_BODY_LOOSE = 18,   /* the same instructions with the MFMA -> v_exp_f32 dependency
                                       removed and the pack -> MFMA dependency one block long */
  VISTA_CAL_TILE_BODY_LDS = 19,     /* TILE_BODY with five MFMA operands per block read from LDS
                                       (ds_read_b128), as the kernel's projection and P.V have    */
  VISTA_CAL_TILE_BODY_LDS_BAR = 20, /* ... plus an LDS-only workgroup barrier every four blocks   */
  VISTA_CAL_TILE_BODY_LDS_BAR_PUB = 21 /* ... plus 8 packs and two ds_write_b128 every four blocks */
};

/*
 * One workgroup per compute unit (256), waves_per_simd (1..4) x 4 waves each;
 * every wave runs `iters` iterations of loop body `what`.  sink: device, >= 1024
 * floats, never written in practice.
 */
int vista_calibrate_issue(int what, int waves_per_simd, int iters, float* sink, void* hip_stream);

/*
 * LDS operand reads: every wave issues 16 independent ds_read_b128 per iteration
 * (lane i reads 16 bytes at 16 i of a 1 KB slab: the conflict-free pattern of the MFMA
 * operand buffers), plus `mfmas` (0 or 8) independent 32x32x16 MFMAs per iteration.
 */
int vista_calibrate_lds_read(int mfmas, int waves_per_simd, int iters, float* sink, void* hip_stream);

/* Reads `bytes` (multiple of 16) from device pointer src (16-byte aligned) once. */
int vista_calibrate_stream_read(const void* src, int64_t bytes, float* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* VISTA_CALIBRATE_H */
