/*
 * taser_profile.h - optional per-kernel timing of the library declared in
 * taser.h, for benchmarks and tuning; no part of the mini-batch generation path.
 */
#ifndef TASER_PROFILE_H
#define TASER_PROFILE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------------------
 * Per-kernel timing. Between taser_profile_begin and
 * taser_profile_end every kernel the library launches (from the thread that
 * began the session; one session at a time) is bracketed by two HIP events on
 * the stream it runs on. taser_profile_end waits for those events and fills
 * `out` (host, caller-allocated, max_entries structs) with one entry per
 * distinct kernel: its name (static storage), number of launches and summed
 * device time in milliseconds; *num_entries receives the number of entries.
 * At most 65536 launches are recorded per session; later ones are not timed.
 * taser_profile_begin_only(kernel_name) starts a session that brackets only the
 * kernel of that name (as reported by an earlier session; NULL or "" = all):
 * every event pair costs a few microseconds of stream time, which matters when
 * the whole pass is being timed as well.
 * ------------------------------------------------------------------------- */
typedef struct taser_kernel_time {
    const char* name;
    int64_t launches;
    double total_ms;
} taser_kernel_time;

int taser_profile_begin(void);
int taser_profile_begin_only(const char* kernel_name);
int taser_profile_end(taser_kernel_time* out, int32_t max_entries, int32_t* num_entries);

#ifdef __cplusplus
}
#endif
#endif /* TASER_PROFILE_H */
