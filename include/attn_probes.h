/* attn_probes.h -- C ABI of libattn_probes.so: measurement probes for MI355X (gfx950).
 *
 * Not part of the attention library (include/attn.h, libattn.so): these entry points exist to measure
 * the rates of the machine's units in the access and instruction patterns the attention kernels use,
 * so that the kernels' fractions of peak can be put in proportion.  Only tests and profiles call them.
 * Every entry point enqueues one kernel on `stream` (a hipStream_t, NULL = default stream) and
 * returns the amount of work enqueued (> 0) or a negative code; the caller times it on the stream.
 * All pointers are DEVICE pointers owned by the caller.
 */
#ifndef ATTN_PROBES_H
#define ATTN_PROBES_H

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ATTN_PROBE_EINVAL = -1,       /* null pointer or non-positive count */
    ATTN_PROBE_EUNSUPPORTED = -2, /* a variant that is not built */
    ATTN_PROBE_ELAUNCH = -3       /* the HIP runtime refused the launch */
};

/* Rate of 2^x evaluations (paper Sec. 3.1.3): a pure-ALU kernel of ATTN_EXP2_RATE_BLOCKS x 256
 * threads, each doing 8 x iters evaluations with the polynomial emulation of the given degree (3, 4,
 * 5) or the hardware instruction (0), writing one float per thread to out (ATTN_EXP2_RATE_BLOCKS *
 * 256 floats).  Returns the number of evaluations. */
enum { ATTN_EXP2_RATE_BLOCKS = 2048 };
long long attn_exp2_rate(float* out, int degree, int iters, void* stream);
/* The same kernel with the section's partial emulation: of the 8 evaluations per thread and
 * iteration, emulated_of_8 (0, 1, 2, 4 or 8; the paper emulates 10-25 % of a row) go through the
 * degree-3 polynomial and the rest through the hardware instruction. */
long long attn_exp2_rate_partial(float* out, int emulated_of_8, int iters, void* stream);

/* Matrix-core ceiling: a kernel of ATTN_MFMA_RATE_BLOCKS x 512 threads (two waves per SIMD on 256
 * CUs) that issues nothing but v_mfma_f32_32x32x16_bf16 on register operands, 32 x iters per wave,
 * with constant operands (random_operands = 0) or N(0,1)-like ones (!= 0: the data the attention
 * workloads of paper Sec. 5 use).  out: ATTN_MFMA_RATE_BLOCKS * 512 floats.  Returns the FLOPs. */
enum { ATTN_MFMA_RATE_BLOCKS = 256 };
long long attn_mfma_rate(float* out, int random_operands, int iters, void* stream);

/* LDS read rate in the kernels' two access patterns: ATTN_LDS_RATE_BLOCKS blocks of 256 threads (2
 * resident per CU) read a swizzled 64 x 128 tile of 16-bit elements over and over, pattern 0 with
 * ds_read_b128 as the MFMA A-operand fragments are read, pattern 1 with ds_read_b64_tr_b16 as the
 * transposed fragments are; one float per thread to out (ATTN_LDS_RATE_BLOCKS * 256 floats).
 * Returns the number of bytes read from LDS. */
#define ATTN_LDS_RATE_BLOCKS 512
long long attn_lds_rate(float* out, int pattern, int iters, void* stream);

/* What the instructions that accompany an MFMA cost a wave that is alone on its SIMD (the situation of
 * the attention kernels that run one wave per SIMD): ATTN_PROBE_WAVE_ISSUE_BLOCKS blocks of 4 waves
 * loop over steps of {1 MFMA, nv vector instructions, nb ds_read_b128, ntr pairs of
 * ds_read_b64_tr_b16 feeding the MFMA `ring` steps later, one global->LDS copy every `dma` steps}.
 * attn_probe_wave_issue_configs() is the number of built variants; variant `config` stores its
 * (nv, nb, ntr, dma, ring) in describe5 (host pointer, may be NULL) and, if out (256 *
 * ATTN_PROBE_WAVE_ISSUE_BLOCKS floats, also the source of the copies) and clk (2 long long: shader
 * cycles and 100 MHz ticks of the loop in one wave) are given, enqueues it.  Returns the number of
 * steps per wave. */
enum { ATTN_PROBE_WAVE_ISSUE_BLOCKS = 256 };
int attn_probe_wave_issue_configs(void);
long long attn_probe_wave_issue(int config, int* describe5, float* out, long long* clk, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif
