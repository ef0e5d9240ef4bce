/*
 * smat_bench.h -- measurement entry points of the MI355X (gfx950) blocked SpMM library.
 *
 * Not part of the method's interface (that is smat.h): the reduced kernels of the paper's
 * optimisation-step comparison, and six probe kernels that measure what the device delivers
 * for the access patterns the SpMM kernels are made of.  Conventions as in smat.h.
 */
#ifndef SMAT_BENCH_H
#define SMAT_BENCH_H

#include "smat.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Ablation (Performance model section, figure of measured against modelled time; Implementation
 * section, optimisation steps B and T): the same product from the canonical BCSR arrays of the
 * handle (rowPtr, col, 256 values per block) with fewer of the optimisations, to be timed next
 * to smat_spmm.  fp16 / bf16 handles only; one wavefront per (block row, 16 columns of C), no
 * pipelining.
 *   level 0   every block of the grid is visited and its presence looked up in a dense block
 *             map (no BCSR iteration), scalar multiply-adds in fp32
 *   level 1   "B": iteration over the stored blocks through rowPtr / col, scalar multiply-adds
 *   level 2   "B + T": the same iteration, one MFMA 16x16x16 per stored block
 * smat_ablation_bytes   bytes of DEVICE memory smat_ablation_bind needs (the block values in
 *                       canonical layout, 512 bytes per stored block, plus the block map when
 *                       the block grid has at most 2^26 entries; without it level 0 is refused)
 * smat_ablation_bind    fills that area (256-byte aligned, caller-owned, alive until
 *                       smat_destroy); the handle must already be bound with smat_bind_device,
 *                       whose rowPtr / col / permutation copies the kernels share; synchronises
 * smat_ablation_spmm    arguments as smat_spmm; only enqueues
 */
smat_status_t smat_ablation_bytes(const smat_handle_t *h, size_t *bytes);
smat_status_t smat_ablation_bind(smat_handle_t *h, void *dev_area, size_t bytes, void *stream);
smat_status_t smat_ablation_spmm(const smat_handle_t *h, int level, const void *dB, int64_t ldb,
                                 void *dC, int64_t ldc, int64_t N, void *stream);

/*
 * Probes: six kernels that measure what the device delivers for the access patterns the SpMM
 * kernels are made of (bench.py --probes times them and prints the rates next to the
 * rooflines).  They compute nothing of the method.  All pointers DEVICE, calls only enqueue.
 *
 *   smat_probe_read    reads `bytes` (a multiple of 8 KiB is read) from dev_buf once, streaming
 *   smat_probe_read_window  `waves` wavefronts (a multiple of 4) each read the first window_bytes (a
 *                      multiple of 8 KiB, at most 1 GiB) of dev_buf once, every wave beginning at
 *                      another place and wrapping round: with a window that fits an XCD's L2
 *                      this is the rate at which the L2s feed the L1s (waves * window_bytes moved)
 *   smat_probe_gather  `waves` wavefronts each fetch `packs` groups of 32 rows named by dev_idx
 *                      (uint32[waves * packs * 32], row numbers into a table of row_bytes-byte
 *                      rows): 16 lanes x bytes_per_lane (8 or 16) bytes from the start of
 *                      every row, eight row loads in flight per lane as in the SpMM kernel
 *   smat_probe_pieces  every lane of `waves` wavefronts fetches `per_lane` pieces of
 *                      bytes_per_lane (2, 4, 8 or 16) bytes, one from the start of each row named
 *                      by dev_idx (uint32[waves * per_lane * 64], row numbers into a table of
 *                      row_bytes-byte rows; row_bytes a multiple of bytes_per_lane; per_lane a
 *                      multiple of 4): the fetch of the SpMM kernel at N = 1, 2, 4, 8, 16,
 *                      where a lane loads the whole piece of the row of B of one entry
 *   smat_probe_mfma    workgroups x 4 waves issue iters x 16 MFMA 16x16x32 (fp16) each on
 *                      register operands: 2 * 16*16*32 flop per instruction and wave
 *   smat_probe_tile_step  workgroups x 8 waves run `steps` (a multiple of 3) steps of the 16-bit tile
 *                      kernel's loop on data that stays in the L1 (dev_buf, at least 1 MiB, read only):
 *                      per wave and step 32 MFMA 16x16x32 with four byte permutes per operand, plus the
 *                      parts named by the bits of `parts`: 1 = four 1 KiB loads of block values into a
 *                      register ring, 2 = eight 16-byte LDS reads of the panel, 4 = the barrier, 8 = two
 *                      1 KiB loads straight into LDS, 16 = the loads issued together behind the barrier
 *                      instead of between the groups of matrix instructions, 32 = right operands by
 *                      transposing LDS reads one group of columns ahead instead of part 2 and the
 *                      permutes.  Built for parts = 0, 1, 2, 3, 6, 7, 12, 14, 15, 31, 32, 36, 37, 45;
 *                      2 * 16*16*32 * 32 flop per wave and step
 *   dev_sink           4 bytes the kernels may write (they never do for the probe's data)
 */
smat_status_t smat_probe_read(const void *dev_buf, size_t bytes, void *dev_sink, void *stream);
smat_status_t smat_probe_read_window(const void *dev_buf, size_t window_bytes, int waves, void *dev_sink,
                                     void *stream);
smat_status_t smat_probe_gather(const void *dev_table, uint32_t row_bytes, const uint32_t *dev_idx, int waves,
                                int packs, int bytes_per_lane, void *dev_sink, void *stream);
smat_status_t smat_probe_pieces(const void *dev_table, uint32_t row_bytes, const uint32_t *dev_idx, int waves,
                                int per_lane, int bytes_per_lane, void *dev_sink, void *stream);
smat_status_t smat_probe_tile_step(int workgroups, int steps, int parts, const void *dev_buf, size_t bytes,
                                   void *dev_sink, void *stream);
smat_status_t smat_probe_mfma(int workgroups, int iters, void *dev_sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SMAT_BENCH_H */
