/*
 * calidrop_probes.h - machine probes used by the benchmark (libcalidrop_probes.so).
 *
 * Not part of the CaliDrop path: plain kernels that show what the GPU at hand reaches on a
 * streaming read, on a dense bf16 matrix-core loop and on matrix and vector instructions issued together, so that roofline fractions can be quoted
 * against measured ceilings next to the published peaks.  Device pointers, caller-owned; the
 * calls enqueue one kernel on `stream` (a hipStream_t, NULL = default) and return 0, or -1 on
 * bad arguments or a failed launch.  The caller times them (events on the same stream).
 */
#ifndef CALIDROP_PROBES_H
#define CALIDROP_PROBES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reads `bytes` bytes at `buf` once (16 bytes per lane, `blocks` workgroups of 256 threads, each
 * on its own contiguous slice).  bytes must be a multiple of 16 * blocks; `out`: blocks uint32. */
int calidrop_probe_stream_read(const void* buf, uint64_t bytes, int32_t blocks, void* out, void* stream);

/* The same read issued as non-temporal loads (the hint for data that is not read again soon). */
int calidrop_probe_stream_read_nt(const void* buf, uint64_t bytes, int32_t blocks, void* out, void* stream);

/* The same read requested the way a matrix-operand fragment load requests 256-byte rows: 16 rows x
 * 64 bytes per wave instruction (what a link that moves small requests badly shows).  bytes must be
 * a multiple of 32768 * blocks. */
int calidrop_probe_stream_read_pieces(const void* buf, uint64_t bytes, int32_t blocks, void* out, void* stream);

/* A non-temporal streaming read of blocks * stages * 16 KiB from `src` with full-line stores mixed
 * in: `rows` x 256 bytes per workgroup and stage into `dst` (rows * blocks * stages * 256 bytes;
 * rows = 0: the read alone, dst unused).  `out`: blocks uint32. */
int calidrop_probe_stream_read_store(const void* src, void* dst, int32_t blocks, int32_t stages, int32_t rows, void* out,
                                     void* stream);

/* `blocks` workgroups of 4 waves; every wave executes iters * 8 independent-chain
 * v_mfma_f32_16x16x32_bf16 instructions (16384 flop each) and nothing else.  `out`: blocks * 256
 * floats.  Total flop = blocks * 4 * iters * 8 * 16384. */
int calidrop_probe_mfma_loop(void* out, int32_t blocks, int32_t iters, void* stream);

/* Matrix and ordinary vector instructions side by side: `blocks` workgroups of 4 waves (1024 puts 4
 * waves on every SIMD), every wave runs iters rounds of 16 v_mfma_f32_16x16x32_bf16 (`matrix` != 0)
 * with valu_per_pair / 2 independent vector instructions behind each (valu_per_pair: 0 or 8; fused
 * multiply-adds, or exp2 when `use_exp` != 0).  Timing the three launches (matrix only, vector
 * only, both) shows how much of the vector work issues in the shadow of the matrix pipe.  `out`:
 * blocks * 256 floats. */
int calidrop_probe_mfma_valu(void* out, int32_t blocks, int32_t iters, int32_t matrix, int32_t valu_per_pair,
                             int32_t use_exp, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CALIDROP_PROBES_H */
