/*
 * disco_bench.h -- measurement hooks of libdisco for benchmarks; not part of the product boundary (disco.h).
 */
#ifndef DISCO_BENCH_H
#define DISCO_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

/* Brackets, with two HIP events on the launch stream, the MLP-input GEMM (gate/up + SwiGLU, or W1 + GELU) of
 * layer `layer` in every forward or prompt pass of a model that has more than `layer` layers (layer < 0
 * switches the probe off; launch mode 1 has no such launch and takes no bracket).  disco_probe_read_ms
 * returns the elapsed time of the most recent bracket (the caller has synchronised the stream) or a
 * negative value if none was taken.  The dominant kernel's roofline figure of bench.py comes from here
 * (Sec. 2 of the paper: the target forward is where the time goes).  Process-wide state guarded by a
 * mutex; one stream at a time.                                                                          */
int disco_probe_enable(int layer);
float disco_probe_read_ms(void);

/* Testing aid for the failure path of launches that wait inside (the QKV projection + attention launch of launch
 * mode 0): polls before such a wait gives up, sets the workspace's abort word and lets the launch finish with
 * unusable data (default 2^20, about a second).  A negative value makes every such wait give up at once, so the
 * failure path (NaN logits, -1 from the arg-max and loop-finish kernels, DISCO_EHIP from disco_iterate) can be
 * exercised with kernels that still run to their end.  After a failure the workspace has to be initialised again
 * (disco_workspace_init).  Returns the previous value.  Process-wide.                                     */
int disco_set_wait_limit(int polls);

#ifdef __cplusplus
}
#endif
#endif /* DISCO_BENCH_H */
