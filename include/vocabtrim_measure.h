/*
 * vocabtrim_measure.h -- a measurement aid exported by libvocabtrim.so beside the
 * C ABI of vocabtrim.h.  NOT part of the method and not needed by any caller of
 * the draft step: the benchmark uses it to time what merely streaming a trimmed
 * head's bytes costs on the device.
 */
#ifndef VOCABTRIM_MEASURE_H_
#define VOCABTRIM_MEASURE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------
 * Measurement reference (not part of the method): reads `bytes` bytes at `p`
 * once, in the launch and load shape of the small-n draft step (*sink is
 * written only if a lane's fold of its words hits one fixed value, which keeps
 * the loads alive at no cost).  Its duration is what the device needs to merely
 * stream the bytes a draft step has to stream; the benchmark reports it next
 * to the step.
 *   p      device, 16-byte aligned;  bytes > 0, a multiple of 16
 *   sink   [1] uint32, device
 * ---------------------------------------------------------------------- */
int vt_stream_read_reference(const void *p, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* VOCABTRIM_MEASURE_H_ */
