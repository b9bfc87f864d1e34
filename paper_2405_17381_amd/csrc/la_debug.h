/*
 * Test and tuning switches of libla.so.  NOT part of the public interface (include/la.h):
 * only the test-suite, the benchmark's A/B legs and tuning scripts call these.
 *
 * The switches are process-wide and all start at 0 (= the library's own choice).  The
 * library never reads the environment, so la_workspace_bytes / la_plan and the launch that
 * follows them always agree unless a switch is changed in between.  Do not change a switch
 * while another thread is inside a library call.
 *
 *   "lseg"           > 0: segment length in tokens (rounded up to the tile length) instead
 *                    of the planner's choice
 *   "no_pair"        != 0: the dK and dV scans of the backward pass run as two launches
 *                    instead of one XCD-paired launch
 *   "no_decay_skip"  != 0: the segment-state pre-pass reads every block, also those whose
 *                    decay weight is below its cut-off
 *   "f32_plain"      != 0: fp32 at d = 128 runs the plain FMA kernel instead of the
 *                    matrix-core one
 *   "ablate"         1..4: measurement-only variants of the direct-to-LDS block scan that
 *                    leave work out (1: no result stores, 2: loads and barriers only,
 *                    3: arithmetic only, 4: loads, barriers and stores without arithmetic);
 *                    their results are wrong by design
 *   "staged_prepass" != 0: bf16 runs the register-staged segment-state pre-pass
 *                    instead of the direct-to-LDS one
 *   "prepass_groups" 1, 2: the direct-to-LDS pre-pass at d = 128 runs with that many groups of four waves per
 *                    workgroup instead of four (each group takes every G-th block of the segment;
 *                    the sums differ in rounding order between group counts)
 *   "no_trio"        != 0: la_bwd runs its direct-to-LDS block scans as a dQ launch followed by a
 *                    paired dK / dV launch instead of one launch of three roles
 *   "wide_slices"    != 0: la_fwd_wide always runs accumulated scans over d_v-wide slices, also where
 *                    the single kernel with the non-square state applies
 *   "store_policy"   2: the direct-to-LDS block scan stores its results with ordinary instead
 *                    of non-temporal stores
 *   "staged_scan"    != 0: bf16 runs the register-staged block scan (64-row
 *                    blocks) instead of the direct-to-LDS one (32-row blocks)
 *
 * la_debug_set returns LA_OK, or LA_ERR_NULL for an unknown name; la_debug_get returns the
 * value, or -1 for an unknown name.
 */
#ifndef LA_DEBUG_H
#define LA_DEBUG_H
#ifdef __cplusplus
extern "C" {
#endif
int la_debug_set(const char *name, long value);
long la_debug_get(const char *name);
/*
 * Measurement aid for the benchmark's matrix-core denominator: launches `workgroups`
 * workgroups of four waves that each issue 4 * iters v_mfma_f32_32x32x16_bf16 from registers
 * only (2 * 32 * 32 * 16 flops each).  `sink` is a DEVICE pointer to one float that is never
 * written in practice.  The caller times the launch.  Returns an la_status.
 */
int la_debug_mfma_rate(int workgroups, int iters, float *sink, void *hip_stream);
#ifdef __cplusplus
}
#endif
#endif
