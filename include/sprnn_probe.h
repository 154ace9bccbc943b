/*
 * sprnn_probe — device microbenchmarks behind the roofline that bench.py states for the persistent
 * sparse recurrent step (libsprnn_probe.so).  Measurement tools only: nothing in libsprnn depends on
 * them.  All functions return 0 on success, a negative value on a HIP error or a bad argument, and
 * synchronise with the device before returning.  They allocate and free their own scratch memory.
 *
 * The step time of the method is bounded by (paper, Section 3.3: "overall performance is limited by
 * shared memory throughput"; Section 4.2: cross-block synchronisation costs memory round trips)
 *     T_step >= nnz * gather_bytes / LDS_bandwidth  +  hand-off latency  +  |h| / fill_bandwidth
 * and the three device constants in that bound are what this library measures.
 */
#ifndef SPRNN_PROBE_H_
#define SPRNN_PROBE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Conflict-free LDS gather rate: every lane of `workgroups` x `threads` issues `width_bytes`-wide
 * (4, 8 or 16) reads at lane-contiguous addresses.  *bytes_per_second is the aggregate over all
 * workgroups (one per CU when workgroups <= number of CUs).  pattern 0 = conflict free,
 * 1 = uniformly random columns (what an unordered sparse row produces).
 */
int sprnn_probe_lds_gather(int device, int workgroups, int threads, int width_bytes, int pattern,
                           double* bytes_per_second);

/*
 * The same measurement with the caller's own read pattern: offsets (host) holds 16 x `threads` byte offsets into a 64 KB
 * LDS array, offsets[k * threads + t] = address of thread t's k-th read (multiples of width_bytes, below 65536).  Every
 * thread issues its 16 reads over and over; *bytes_per_second counts width_bytes per read.  bare = 1
 * leaves everything but the reads out of the loop, so that the LDS alone bounds it (the default loop also adds the
 * values up, which costs about as many issue cycles as conflict-free reads take).  Used to check the model of which lanes
 * the LDS serves together (and hence which column orders collide) against packed weight images.
 */
int sprnn_probe_lds_gather_offsets(int device, int workgroups, int threads, int width_bytes, int bare, const uint32_t* offsets,
                                   double* bytes_per_second);

/*
 * One-way producer-store -> consumer-observes latency between two workgroups, by ping-pong on two
 * agent-coherent flags.  `same_xcd` = 1 picks two workgroups on one XCD, 0 two on different XCDs
 * (workgroups are dealt round-robin over the XCDs).  *nanoseconds = round trip / 2;
 * xcc[0], xcc[1] receive the XCC ids the two workgroups actually ran on.
 */
int sprnn_probe_handoff(int device, int same_xcd, int rounds, double* nanoseconds, int xcc[2]);

/*
 * Rate at which one workgroup of `threads` lanes copies `bytes` (multiple of 16) of agent-coherent
 * global memory into its LDS with 16-byte loads, `workgroups` of them reading the same bytes at the
 * same time (the "load" stage of Section 3.3).  *seconds_per_copy is the time of one whole copy.
 */
int sprnn_probe_fill(int device, int workgroups, int threads, int bytes, int rounds, double* seconds_per_copy);

#ifdef __cplusplus
}
#endif
#endif /* SPRNN_PROBE_H_ */
