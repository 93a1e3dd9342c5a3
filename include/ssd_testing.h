/*
 * ssd_testing.h -- test-only entry points of libssd_hip.so.
 *
 * The library chooses by itself which kernel family runs a prefill, how a prompt is
 * cut into segments and whether outputs and states stream past the caches.  Tests
 * and tuning runs need to force those choices (to reach every code path at small
 * sizes, to compare both cache policies bit for bit); these calls do that.  The
 * settings are process-wide and not synchronised: set them from one thread while no
 * call of the library is in flight, and reset them afterwards.  Nothing in the
 * library reads the environment.  Workspace sizes (ssd_prefill_workspace_bytes,
 * ssd_prefill_varlen_workspace_bytes) do not depend on any knob.
 */
#ifndef SSD_TESTING_H_
#define SSD_TESTING_H_

#include "ssd.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SSD_KNOB_FORCE_GENERIC = 0, /* 1: every prefill runs on the generic fp32 kernels; 0: default */
  SSD_KNOB_SEG_CHUNKS = 1,    /* k > 0: k chunks per segment in the MFMA prefill; 0: library's choice */
  SSD_KNOB_SEG_BLOCKS = 2,    /* k > 0: k 64-token blocks per segment (when SEG_CHUNKS is 0); 0: default */
  SSD_KNOB_SEG_PARTS = 3,     /* k > 0: pieces per segment in the states-only pass, if k divides the
                                 segment length and the state slots suffice; 0: default */
  SSD_KNOB_Y_STREAM = 4,      /* 0 / 1: ordinary / non-temporal stores of y in the full scan; -1: default */
  SSD_KNOB_DECODE_STREAM = 5, /* 0 / 1: ordinary / non-temporal accesses to the decode state; -1: default */
  SSD_KNOB_FORCE_MFMA_F32 = 6, /* 1: fp32 io runs on the fp32 MFMA kernel whenever the shape is eligible (headdim
                                 a multiple of 32, dstate a multiple of 8 up to 128), also where the library
                                 expects the generic kernels to be faster; 0: default */
  SSD_KNOB_F32_SEGMENTS = 7,   /* k > 0: the fp32 MFMA kernel cuts every sequence into k time segments (at most
                                 one per 64-token block); 0: library's choice */
  SSD_KNOB_FOLD_MAX_SLOTS = 8  /* k >= 0: a plain batch whose chain over segment-state slots, (segments - 1) x
                                 pieces, is at most k long runs no separate pass over those states -- every
                                 segment of the full scan sums the slots before it as it loads them; 0: never.
                                 Default 3.  Reset with ssd_testing_reset_knobs */
} ssd_knob;

/* Sets one knob.  Errors: SSD_ERR_SHAPE for an unknown knob. */
SSD_API ssd_status ssd_testing_set_knob(int32_t knob, int32_t value);

/* All knobs back to the library's own choices. */
SSD_API void ssd_testing_reset_knobs(void);

/* How ssd_prefill would run a shape under the current knobs (host arithmetic only: no GPU call, nothing
 * launched).  plan[0]: kernel family, 0 generic fp32 kernels, 1 bf16 MFMA, 2 fp32 MFMA.  For the bf16
 * MFMA family (per state slice of 128 columns): plan[1] 64-token blocks per segment, plan[2] segments
 * per sequence, plan[3] pieces per segment in the states-only pass, plan[4] 1 if the full scan sums the
 * chain over segment states itself and no separate pass runs (h0_aliases_final_state != 0: as for a call
 * whose h0 and final_state share memory, which rules that out).  For the fp32 MFMA family: plan[5] time
 * segments per sequence.  The other entries are zero.
 * Errors: SSD_ERR_NULL; the shape errors of ssd_prefill. */
SSD_API ssd_status ssd_testing_prefill_plan(const ssd_shape *shape, int32_t h0_aliases_final_state,
                                            int32_t plan[8]);

#ifdef __cplusplus
}
#endif
#endif /* SSD_TESTING_H_ */
