/*
 * wsvd_test.h - entry points of libwsvd.so that are NOT part of the product boundary: hooks for tests, tuning and
 * profiling.  Nothing here is needed to use the library (see wsvd.h for that); the calls exist so that measurements and
 * tests can reach into it through plain C symbols.
 */
#ifndef WSVD_TEST_H
#define WSVD_TEST_H

#include "wsvd.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * In-kernel timeline (profiling build only: the library compiled with -DWSVD_TIMELINE, `python -m
 * paper_2604_02570_amd.build --timeline` -> libwsvd_timeline.so).  The decode-attention kernels then write the chip-wide
 * 100 MHz wall clock at marked points: int64 buf[(workgroup * 16 + wave) * 16 + slot], workgroup = linear id of the
 * launch grid, written by lane 0 of each wavefront.  dev_ptr: DEVICE buffer, 16-byte aligned, owned by the caller, at
 * least workgroups * 2048 bytes (a smaller buffer switches the stamps of that launch off); NULL detaches.  Slots of the
 * decode attention: 0 kernel entry, 1 first loads issued, 2 factors staged, 3 query limbs ready, 4 first tile consumed,
 * 5 last tile consumed, 6 wave's partial result written, 7 workgroup barrier passed, 8 output stored.
 * The product build returns WSVD_E_UNSUPPORTED.
 */
wsvd_status wsvd_timeline_set_buffer(wsvd_ctx *ctx, void *dev_ptr, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* WSVD_TEST_H */
