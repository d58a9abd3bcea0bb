/*
 * he_issue_rates.h -- C ABI of the small measurement library that backs the integer-ALU peak used in the
 * rooflines of bench.py: register-only loops of one vector instruction (or of one modular butterfly in a given
 * instruction selection), timed with HIP events on the given GPU.  No inputs, no state; for benchmarks only.
 */
#ifndef HE_ISSUE_RATES_H
#define HE_ISSUE_RATES_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
/* Number of measurements and the name of measurement i ("v_add_u32", "butterfly forward, min-based", ...). */
uint32_t he_issue_rates_count(void);
const char* he_issue_rates_name(uint32_t i);
/* Vector instructions of one wave64 per measured unit (1 for single instructions, 10 or 11 for butterflies). */
uint32_t he_issue_rates_instructions(uint32_t i);
/* Runs every measurement on GPU `device` (synchronous, allocates 4 MiB for the duration of the call).
   ns_per_unit_host[i]: nanoseconds one SIMD needs per unit (instruction or butterfly) of one wave64 with 8 waves
   resident per SIMD = kernel time * number of SIMDs (n_simd_host, 4 per compute unit) / units issued.
   Returns 0, or the hipError_t that stopped it. */
int he_issue_rates_run(int device, double* ns_per_unit_host, uint32_t* n_simd_host);
#ifdef __cplusplus
}
#endif
#endif
