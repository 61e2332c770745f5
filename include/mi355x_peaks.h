/*
 * Published peak rates of one MI355X (gfx950, 256 compute units in 8 XCDs, 2.4 GHz), the
 * denominators of every roofline fraction this repository reports.  Dense figures (AMD's headline
 * matrix numbers with 2:1 structured sparsity are twice these and are never used).  bench.py reads
 * this file; the probes in hgrn2.h (hgrn2_probe_copy, hgrn2_probe_mfma) measure what the same
 * machine sustains for a plain copy and for a loop of nothing but matrix instructions.
 */
#ifndef MI355X_PEAKS_H
#define MI355X_PEAKS_H

#define MI355X_HBM_GBPS             8000.0   /* HBM3E, 288 GB */
#define MI355X_MFMA_BF16_TFLOPS     2500.0   /* dense bf16 / fp16 matrix */
#define MI355X_MFMA_FP8_TFLOPS      5000.0
#define MI355X_MFMA_FP32_TFLOPS      157.3   /* fp32 matrix = fp32 vector */
#define MI355X_VALU_FP32_TFLOPS      157.3
#define MI355X_FP64_TFLOPS            78.6
#define MI355X_COMPUTE_UNITS           256
#define MI355X_CLOCK_GHZ               2.4
#define MI355X_LDS_KB_PER_CU           160
#define MI355X_INFINITY_CACHE_MB       256

#endif /* MI355X_PEAKS_H */
