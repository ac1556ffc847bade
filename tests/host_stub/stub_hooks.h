// Hooks of the recording stubs (stub_launches.cpp) for the host-logic test driver.
#pragma once
#include <stdint.h>

enum { STUB_MAX_SEGS = 384 };

typedef struct {
    int gated;                      // the launch belongs to an enqueued, stoppable sequence
    int nseg;                       // > 0: row ranges below; 0: units [u0, u0+nu) of the device list
    uint32_t u0, nu;
    int max_rows;
    uint32_t row0[STUB_MAX_SEGS];
    uint16_t rows[STUB_MAX_SEGS];
    uint16_t expert[STUB_MAX_SEGS];
} StubLaunch;

#ifdef __cplusplus
extern "C" {
#endif
void stub_set_counts(const int32_t *cnt, int n);      /* queue lengths [E][2] the next moe_permute reports */
void stub_reset_launches(void);
int stub_n_launches(void);
const StubLaunch *stub_launch(int i);
void stub_complete_first(int n);                       /* the next reports mark ranges [0,n) complete; -1 = all */
#ifdef __cplusplus
}
#endif
