/* taw_diag.h -- measurement probes of the library: what the part sustains, against which the kernels'
 * rates are read.  Not part of the hot path: every call here runs a short synthetic kernel, WAITS for it
 * (the only calls of the library that synchronise with the host) and returns the measured figures in host
 * memory.  bench.py --workload diag prints them; profiles/mfma_ceiling.md records a run.
 *
 * Why they exist.  The layer's roofline is the dense bf16 matrix rate (Experimental Setup of the paper trains in
 * 16-bit precision; the target of this build is quoted against the 2.5 PFLOP/s figure).  On real operands that
 * rate is not reachable: the part lowers its clock under the power the matrix cores draw.  These probes put the
 * sustained figures on record: a loop of nothing but MFMAs, the same loop with the LDS fragment reads and the
 * global->LDS loads a GEMM tile needs, the LDS read rate, and the rate of fp32 atomic adds (which decides
 * whether an attention backward that accumulates dQ with atomics can pay).
 *
 * Same conventions as taw.h: int status, no exceptions, device pointers 16-byte aligned, host pointers for results. */
#ifndef TAW_DIAG_H
#define TAW_DIAG_H

#include "taw.h"

#ifdef __cplusplus
extern "C" {
#endif

enum {
  TAW_DIAG_MFMA_RANDOM = 0,       /* v_mfma_f32_32x32x16_bf16 back to back, operands in registers, random bf16 values */
  TAW_DIAG_MFMA_ZERO = 1,         /* the same on all-zero operands (no switching activity: the clock stays up) */
  TAW_DIAG_MFMA_LDS = 2,          /* + one LDS fragment read (ds_read_b128) per two MFMAs, the ratio of a 128x128 wavefront tile */
  TAW_DIAG_MFMA_LDS_LOADS = 3     /* + one direct global->LDS load (16 bytes per lane) per four MFMAs, the ratio of a 256x256x64 tile step */
};

typedef struct {
  double tflops;      /* 2 * 32 * 32 * 16 flops per MFMA, all 256 compute units x 4 wavefronts */
  double clock_ghz;   /* shader clock inside the loop: core-clock ticks over wall-clock ticks */
  double mfma_busy;   /* 32 cycles per MFMA over the cycles the loop took: 1.0 = the matrix pipe never idles */
  double ms;          /* duration of the launch */
} taw_diag_rate;

/* kind: TAW_DIAG_MFMA_*.  iters: loop trips of 16 MFMAs per wavefront (>= 1; 20000 gives about 10 ms).
 * src / src_bytes: a device buffer the loads of TAW_DIAG_MFMA_LDS_LOADS stream from (>= 1 MiB, a multiple of
 * 64 KiB; ignored by the other kinds, may be NULL there).  Synchronises with the host. */
int taw_diag_mfma_loop(int32_t kind, int32_t iters, const void* src, size_t src_bytes, taw_diag_rate* out);

/* LDS read rate of one compute unit, bytes per core clock: instr 0 = ds_read_b128, 1 = ds_read_b64,
 * 2 = ds_read_b64_tr_b16; waves = 4 or 8 wavefronts per compute unit, conflict-free addresses. */
int taw_diag_lds_read_rate(int32_t instr, int32_t waves, double* bytes_per_clock_per_cu, double* clock_ghz);

/* Rate of dQ-tile updates in the access pattern of a key-stationary attention backward: every workgroup walks down
 * the query rows of its head from its key block's diagonal on and updates a [32 x 128] fp32 tile per step (rows of
 * 128 contiguous bytes per half wavefront).  mode 0: no-return fp32 atomic adds; 1: plain stores; 2: load, add, store
 * (what a private slot allows).  buf: S * n_heads * 128 floats (overwritten).  *updates_per_s counts 4-byte elements. */
int taw_diag_dq_update_rate(float* buf, int32_t S, int32_t n_heads, int32_t mode, double* updates_per_s, double* ms);

/* What a vector store costs a SIMD that is otherwise issuing MFMAs (the question behind the attention backward that
 * hands dS from one kernel to the other through memory): 256 workgroups of `waves` (4 or 8) wavefronts, each running
 * 20000 trips of {`mfmas` (16 or 64) MFMAs, then `stores` (0, 1, 2 or 4) non-temporal stores of one contiguous KiB}.
 * buf: device, taw_diag_store_cost_bytes() bytes (128 MiB: a 64 KiB window per wavefront), overwritten.
 * *ns_per_trip: duration of the launch over the trips.  The difference to stores = 0 is what the stores cost. */
size_t taw_diag_store_cost_bytes(void);
int taw_diag_store_cost(void* buf, size_t buf_bytes, int32_t waves, int32_t mfmas, int32_t stores, double* ns_per_trip);

/* Host only: the layout of the dS matrix that the default attention backward hands from its dK/dV kernel to its dQ
 * kernel, for sequence length S (1 .. 2^20), as the kernels compute it.  nqt = ceil(S / 256) blocks of query rows.
 * *pair_bytes: bytes per (batch, head).  unit_offsets[]: byte offset of every 2 KiB unit, in the order block ib, 32-row
 * group s = 0..7, key group g = 0 .. 8 (ib + 1) - 1: 32 nqt (nqt + 1) entries.  slots[(2 tt + hh) * 32 + kk]: the 16-byte
 * slot (0..127) inside a unit that lane (key kk, lane half hh) of the writer gives its piece tt.  rows[p]: the query row
 * (0..31 of its group) at position p = 16 hh + 8 tt + e of a key's 32 values.  All host pointers. */
int taw_diag_attn_ds_layout(int32_t S, int64_t* pair_bytes, int64_t* unit_offsets, int32_t* slots, int32_t* rows);

/* How vector instructions issue beside MFMAs on one SIMD: core-clock cycles per slot of {one MFMA + nvalu vector instructions}.
 * mode 0: one wavefront per SIMD runs both; mode 1: two wavefronts per SIMD, each runs both; mode 2: two wavefronts per SIMD,
 * one issues only the MFMAs, the other only the vector instructions.  kind 0: v_fma_f32, 1: v_exp_f32.  nvalu: 0, 2, 4 or 8.
 * *cycles_mfma_wave: per slot, seen by a wavefront that issues MFMAs (32 = the matrix pipe never idles with one such
 * wavefront per SIMD, 64 with two); *cycles_valu_wave: the same for the last wavefront (the vector-only one in mode 2).
 * What the attention kernels' design rests on: a lone wavefront issues about one vector instruction per 5 cycles, two
 * wavefronts of a SIMD issue theirs side by side. */
int taw_diag_issue_rate(int32_t mode, int32_t kind, int32_t nvalu, double* cycles_mfma_wave, double* cycles_valu_wave);

/* The order in which the GEMM kernels' grid walks its 256 x 256 output tiles, evaluated on the host (no GPU call):
 * workgroup id b of a grid of tiles_m x tiles_n tiles computes tile (tile_rows[b], tile_cols[b]).  Host arrays of
 * tiles_m * tiles_n int32 each.  Ids b and b + 8 k run on one XCD, ids of one block of 256 at about the same time;
 * the tests check that the map is a bijection for ragged grids and count the operand panels such a block shares. */
int taw_diag_gemm_tile_order(int32_t tiles_m, int32_t tiles_n, int32_t* tile_rows, int32_t* tile_cols);

#ifdef __cplusplus
}
#endif
#endif /* TAW_DIAG_H */
