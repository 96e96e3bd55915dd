/*
 * probe.h -- C ABI of libattn_probe_gfx950.so: measurement aids used by the benchmark only
 * (no attention arithmetic, nothing from the paper; not part of the attention library).
 * Return values: 0 = ok, 1 = NULL pointer, 2 = bad argument, 5 = launch failed.  Device pointers,
 * work enqueued on `stream` (hipStream_t as void*), no allocation, no synchronisation.
 */
#ifndef PAPER_2510_04212_PROBE_H
#define PAPER_2510_04212_PROBE_H
#ifdef __cplusplus
extern "C" {
#endif

/*
 * `workgroups` work-groups of 4 waves, each wave issuing 4 * iters independent
 * v_mfma_f32_32x32x16_bf16 instructions on register operands.  `out` is a DEVICE array of
 * 4 + 2 * workgroups int64, 16-byte aligned: out[4 + 2g] = shader-clock cycles and out[5 + 2g] =
 * ticks of the constant 100 MHz counter that the first wave of work-group g spent in its loop
 * (out[0], out[1] repeat work-group 0; out[2], out[3] are scratch).  cycles / (ticks / 1e8) is the
 * shader clock that CU ran at; the caller times the launch to get the instruction rate.
 * 1 <= workgroups <= 65536, 1 <= iters <= 2^22.
 */
int attn_probe_matrix_clock(long long* out, int workgroups, int iters, void* stream);

/*
 * The same kind of aid for the LDS: `workgroups` work-groups of 4 waves, each wave issuing
 * 16 * iters conflict-free LDS reads and nothing else; kind 0: ds_read_b128 (1 KB per instruction,
 * one matrix-instruction operand fragment), kind 1: ds_read_b64_tr_b16 (the transposing read,
 * 512 bytes per instruction).  out[0], out[1] (DEVICE, 4 x int64, 16-byte aligned): shader-clock
 * cycles and 100 MHz ticks of the first wave's loop.  With one work-group per CU,
 * 4 waves * 16 * iters * bytes-per-instruction / out[0] is the LDS read bandwidth of a CU in bytes
 * per clock.
 */
int attn_probe_lds_clock(long long* out, int kind, int workgroups, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif
