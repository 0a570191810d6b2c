/*
 * libfa2_probe -- a measurement aid beside libfa2: the matrix-core roof of the machine as it is, measured.
 *
 * The published MI355X peak (2516.6 TFLOP/s dense fp16/bf16) assumes the 2.4 GHz engine clock; under load the
 * clock depends on the operand data.  fa2_probe_mfma runs nothing but v_mfma_f32_32x32x16 on operands the caller
 * supplies (constants, or the N(0,1) values of the attention workloads) and reports the clock it ran at, so that the
 * attention kernel's TFLOP/s can also be read against a roof measured on the same box with the same kind of data.
 * Not part of the attention path; plain C ABI, device pointers, allocates nothing.
 */
#ifndef FA2_PROBE_H_
#define FA2_PROBE_H_

#ifdef __cplusplus
extern "C" {
#endif

enum {
  FA2_PROBE_WORKGROUPS = 512,           /* 2 per CU, 4 wavefronts each: two wavefronts per SIMD               */
  FA2_PROBE_MFMA_PER_ITER = 16,         /* MFMAs per wavefront and loop iteration                             */
  FA2_PROBE_OPERAND_BYTES = 256 * 4 * 2 * 16 /* operands: per thread of a workgroup 4 A and 4 B fragments of 16 B */
};

/*
 * fa2_probe_mfma -- enqueue one launch of FA2_PROBE_WORKGROUPS workgroups in which every wavefront issues
 * iters * FA2_PROBE_MFMA_PER_ITER independent-enough MFMAs (4 accumulators) on operands held in registers.
 *
 *  operands  in   device, FA2_PROBE_OPERAND_BYTES bytes of 16-bit values of `dtype` (FA2_FP16 = 0 / FA2_BF16 = 1 as in
 *                 fa2.h), 16-byte aligned; thread t of every workgroup uses bytes [128 t, 128 t + 128).
 *  ticks     out  device, 4 x 64-bit: engine-clock counter at start and end, then the constant 100 MHz counter at
 *                 start and end, read by one wavefront (clock in MHz = 100 * (t1 - t0) / (t3 - t2)).  8-byte aligned.
 *  sink      out  device, FA2_PROBE_WORKGROUPS * 256 floats (keeps the MFMAs alive); 4-byte aligned.
 *  iters          loop iterations, >= 1.
 *  stream         hipStream_t as void*.
 *
 * FLOPs of the launch: FA2_PROBE_WORKGROUPS * 4 * iters * FA2_PROBE_MFMA_PER_ITER * 32768; the caller times it.
 * Returns 0, -1 (bad argument) or -3 (launch refused), as the codes of fa2.h.
 */
int fa2_probe_mfma(const void* operands, unsigned long long* ticks, float* sink, int dtype, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FA2_PROBE_H_ */
