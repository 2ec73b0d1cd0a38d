/*
 * cryptogen_bench.h -- measurement support of the library, kept apart from the
 * evaluator interface in cryptogen.h: per-launch timing with HIP events and the
 * micro-benchmark of the modular multiply.  Nothing here is needed to evaluate
 * on ciphertexts.
 */
#ifndef CRYPTOGEN_BENCH_H
#define CRYPTOGEN_BENCH_H

#include "cryptogen.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Benchmark support: between cg_profile_begin and cg_profile_end every kernel
 * launch of this context is bracketed by a pair of HIP events on the stream it is
 * launched on.  cg_profile_end waits for the recorded events and returns, per
 * kernel class, the number of launches, their summed duration, their summed
 * algorithmic bytes (distinct inputs read once plus outputs written once) and the
 * rows (transforms) or batch units (pointwise kernels) they processed.
 * At most max_launches launches are recorded (later ones run untimed).  Not
 * thread-safe; do not use around graph capture. */
typedef struct {
    uint32_t kernel_id;   /* see cg_kernel_name */
    uint32_t launches;
    double total_ms;
    double algo_bytes;
    double work_items;    /* residue rows worked through by transform launches; batch units for pointwise ones */
} cg_kernel_stat;
int cg_profile_begin(cg_ctx *ctx, uint32_t max_launches);
int cg_profile_end(cg_ctx *ctx, cg_kernel_stat *stats_host, uint32_t cap, uint32_t *n_out_host);
const char *cg_kernel_name(uint32_t kernel_id);

/* Micro-benchmark of the modular multiply used by every kernel (evidence for
 * the arithmetic choice): runs `iters` dependent modular multiplications per
 * lane on n_lanes lanes with kind 0 = FP64 FMA quotient estimate,
 * 1 = 64-bit Barrett on 32-bit integer multiplies; results go to out_dev
 * (uint64[n_lanes]) and are identical for both kinds. */
int cg_bench_modmul(cg_ctx *ctx, void *stream, int kind, uint32_t n_lanes, uint32_t iters,
                    uint64_t *out_dev);

/* Micro-benchmark of the wave-local exchange between two transform stages that pair elements 32
 * lanes apart (evidence for keeping that exchange in LDS): n_blocks workgroups of 1024 threads,
 * every lane holding 16 doubles, run `iters` exchanges of 8 doubles per lane with kind 0 = through
 * the wave's region of LDS, 1 = v_permlane32_swap on the 32-bit halves.  out_dev: double[n_blocks *
 * 1024], one checksum per lane, identical for both kinds. */
int cg_bench_exchange(cg_ctx *ctx, void *stream, int kind, uint32_t n_blocks, uint32_t iters,
                      double *out_dev);

#ifdef __cplusplus
}
#endif
#endif /* CRYPTOGEN_BENCH_H */
