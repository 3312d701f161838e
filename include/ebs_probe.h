/*
 * Measurement probes of libebs: they do not implement any step of the method;
 * they measure what the hardware sustains for the two resources the method's
 * kernels are bound by, so that roofline fractions can also be quoted against
 * measured (not only published) peaks.  Same conventions as ebs.h: device
 * pointers owned by the caller, asynchronous on `stream`, negative ebs_status
 * on argument errors.
 */
#ifndef EBS_PROBE_H
#define EBS_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Integer-ALU probe for the inner body of Eq. 2 (Sec. 3): every lane executes
 * trips*4*32 pairs of bitwise AND + accumulating bitcount on registers only.
 *   seed : in,  device, at least 264 uint32 (any values)
 *   sink : out, device, blocks*256 uint32 (keeps the work observable)
 * ebs_probe_and_bcnt_pairs() returns the number of lane-level pairs one launch
 * executes; one pair is 32 binary multiply-accumulates.
 */
int ebs_probe_and_bcnt(const uint32_t *seed, uint32_t *sink, int blocks, int trips, void *stream);
long long ebs_probe_and_bcnt_pairs(int blocks, int trips);

/*
 * HBM probe: copies `bytes` (multiple of 16) from src to dst with 16-byte
 * accesses; src == NULL makes it a pure fill (write-only traffic).
 */
int ebs_probe_copy(const void *src, void *dst, size_t bytes, int blocks, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EBS_PROBE_H */
