/*
 * libpoly measurement hooks -- NOT part of the method and outside the "allocates nothing" contract of poly.h:
 * poly_profile_begin creates host-side HIP events for the launches it records.
 */
#ifndef POLY_PROFILE_H
#define POLY_PROFILE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per-stage kernel timing for measurement harnesses.  Between
 * poly_profile_begin and poly_profile_end every kernel the library launches carries a start/stop
 * event pair stamped by the runtime with the dispatch's own begin and end, and poly_profile_end
 * (which synchronises the device) returns, per stage, the number of launches and the sum of their
 * execution times in milliseconds.  `max_launches` bounds the number of recorded launches (host
 * events are created for them); launches beyond it run untimed.  Process-wide, not thread-safe.
 */
enum {
    POLY_STAGE_SELECT = 0, /* Alg. 2 kernel */
    POLY_STAGE_GEMM = 1,   /* base linears with fused expand and epilogue (patch embedding included) */
    POLY_STAGE_SHRINK = 2, /* x A_k */
    POLY_STAGE_ATTN = 3,
    POLY_STAGE_NORM = 4,   /* LayerNorm */
    POLY_STAGE_OTHER = 5,  /* CSR check, patch gathering, class token, heads, merge */
    POLY_STAGE_COUNT = 6
};

typedef struct poly_profile {
    int32_t launches[POLY_STAGE_COUNT];
    float ms[POLY_STAGE_COUNT];
    int32_t dropped; /* recorded launches whose events could not be read */
} poly_profile;

int poly_profile_begin(int max_launches);
int poly_profile_end(poly_profile *out); /* host struct */

#ifdef __cplusplus
}
#endif
#endif /* POLY_PROFILE_H */
