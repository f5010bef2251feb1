/*
 * mustdrop_bench.h -- benchmarking aid of the MustDrop library; not part of the method and not
 * needed to use it (the stage entry points are declared in mustdrop.h).
 *
 * Per-kernel timing with HIP events.  Between mustdrop_profile_start() and mustdrop_profile_stop()
 * every kernel the library launches carries an event pair that receives the begin and end timestamps
 * of that dispatch on its stream (what a kernel trace reports; marker events around a launch would add
 * their own few microseconds).  While switched on, the library creates two HIP events per launch and
 * keeps them in a process-wide list: this is the one place where it holds state and creates runtime
 * objects on behalf of the caller.  Switched off (the default) a launch costs one load of a flag.
 * _stop waits for the events, destroys them and reports, per distinct kernel name, the summed
 * milliseconds and the number of launches: names is a host array of cap*64 chars, total_ms / calls
 * host arrays of cap entries, *n_out the number of names filled.  Host pointers.  Not thread-safe;
 * do not use while another thread is inside the library, and never under stream capture.
 */
#ifndef MUSTDROP_BENCH_H
#define MUSTDROP_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

int mustdrop_profile_start(void);
int mustdrop_profile_stop(char* names, float* total_ms, int* calls, int cap, int* n_out);

#ifdef __cplusplus
}
#endif
#endif /* MUSTDROP_BENCH_H */
