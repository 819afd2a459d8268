/*
 * vattn_bench.h - measurement probes that ship in libvattn.so but are NOT part of the method's interface
 * (vattn.h): micro-benchmarks that price the hardware the attention kernels run on, used by bench.py and
 * vmm_report.py only.  Same conventions as vattn.h: extern "C", int return (0 / -1), vattn_last_error().
 */
#ifndef VATTN_BENCH_H
#define VATTN_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per-call latency of the HIP virtual-memory API at one page-group size (the analogue of Table 3 of
 * the paper): creates, maps, touches and tears down `count` page-groups of `bytes` each on `device`
 * and writes average microseconds per call to out_us[0..8] (host, 12 values):
 *   0 hipMemAddressReserve   1 hipMemCreate   2 hipMemMap   3 hipMemSetAccess (one page-group per call)
 *   4 hipMemSetAccess, ONE call over all page-groups freshly mapped again (total)   5 hipMemUnmap   6 hipMemRelease
 *   7 hipMemAddressFree      8 a kernel writing every mapped byte once (total).
 * out_us[9..11] count instead of time: memory mappings of the process (lines of /proc/self/maps) added per
 * hipMemCreate, added per hipMemMap, given back per hipMemUnmap - what the library's mapping budget rests on.
 * Needs no context.  `bytes` must be a multiple of the allocation granularity. */
int vattn_vmm_microbench(int device, int64_t bytes, int count, double* out_us /*host*/);

/* Matrix-pipe micro-benchmark for the roofline of the prefill kernel (the bf16 contractions of Eq. 2): two
 * waves per SIMD on every CU run `rounds` rounds of four independent v_mfma_f32_32x32x16_bf16 with operands
 * held in registers.  normal_operands = 0: all-zero operands (the chip keeps its full clock); 1: N(0,1)
 * operands, the value distribution of the workloads here (the chip lowers its clock to hold its power limit).
 * Further bits of the same argument add, per matrix instruction, the other work an attention inner loop does beside
 * it, so that its cost under the power limit can be read off: 2 = the A operand is read from LDS (16 bytes per lane
 * and instruction, fetched a round ahead), 4 = three independent fp32 multiply-adds, 8 = one exp2; values 0 .. 15.
 * out[0] = dense TFLOP/s over the launch, out[1] = shader clock in MHz seen inside the kernel.  Needs no
 * context; allocates and frees a few KiB of device memory; synchronises the device. */
int vattn_mfma_microbench(int device, int normal_operands, int rounds, double* out /*host, 2 values*/);

/* Streaming-read micro-benchmark for the roofline of the decode kernel (which reads every K/V byte once, Sec. 7.2
 * calls it memory-bound): one workgroup of four waves per CU reads its contiguous share of a `bytes`-sized buffer
 * with 16-byte non-temporal loads, 16 per lane in flight - the decode kernel's launch shape and load pattern
 * without its arithmetic.  *out_gbs = best of three launches, GB/s.  Needs no context; allocates and frees the
 * buffer (64 MiB .. 64 GiB); synchronises the device. */
int vattn_stream_microbench(int device, int64_t bytes, double* out_gbs /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* VATTN_BENCH_H */
