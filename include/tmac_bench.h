/*
 * tmac_bench.h -- measurement helpers that ship beside the LUT mpGEMM library in a library of
 * their own (libtmac_bench.so).  They take no part in the mpGEMM path and are not part of its ABI:
 * a plain streaming-read kernel and a probe of the LDS lookup rate, the two ceilings the benchmark
 * prints next to the lookup kernels, and a probe of the issue rate of the vector instructions the
 * register-table lookups consist of.
 */
#ifndef TMAC_BENCH_H_
#define TMAC_BENCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Return codes: 0 ok, 1 invalid argument, 2 unsupported, 4 HIP error while enqueuing. */

/* Reads `bytes` bytes from src_dev with 16-byte loads, `per_thread` (1, 4 or 8) loads in flight per
 * lane, optionally non-temporal; sink_dev needs 256 writable bytes.  Enqueues on `stream`. */
int tmac_bench_stream_read(const void* src_dev, size_t bytes, void* sink_dev, int32_t per_thread,
                           int32_t nontemporal, void* stream);

/* `workgroups` workgroups of 256 lanes each hold 32 KB of tables in LDS and issue `rounds` x 16
 * reads of 16 bytes per lane at data-dependent offsets, with the address arithmetic of the batched
 * lookup kernels and no other work; sink_dev needs 256 writable bytes. */
int tmac_bench_lds_lookup_probe(int32_t workgroups, int32_t rounds, void* sink_dev, void* stream);

/* `workgroups` workgroups of 256 lanes (workgroups / 256 wavefronts per SIMD on a 256-CU chip) run
 * `iters` x 64 vector instructions of one kind per lane on eight independent registers (kind 0:
 * v_and_b32, 1: v_perm_b32, 2: v_dot2c_f32_f16), or, kind 3, `iters` x 8 times the 17-instruction
 * lookup sequence of one index dword of the register-table kernel; sink_dev needs 256 writable
 * bytes. */
int tmac_bench_valu_rate_probe(int32_t kind, int32_t workgroups, int32_t iters, void* sink_dev, void* stream);

/* A kernel that does nothing, one wavefront: the cost of a launch. */
int tmac_bench_empty_kernel(void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TMAC_BENCH_H_ */
