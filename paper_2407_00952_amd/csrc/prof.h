// Optional timing of kernel launches with HIP events on the launch stream (measurement hook, not part of
// the method).  A launcher brackets its launch with prof_begin / prof_end, naming the kind of kernel and
// the algorithmic work of the launch (flop for the matrix-core kinds, bytes for the HBM-bound kinds).
#pragma once
#include <hip/hip_runtime.h>

enum { PK_GEMM = 0, PK_LN_FWD, PK_LN_BWD, PK_LORA_GRAD, PK_SGD, PK_ATTN_FWD, PK_ATTN_BWD, PK_FEDAVG, PK_COUNT };

bool prof_begin(int kind, hipStream_t st);               // true if this launch is being recorded
void prof_end(bool recording, int kind, double work, hipStream_t st);
int prof_enable(unsigned mask);                          // bit k = record kind k; resets what was recorded
int prof_read(int kind, double *ms, double *work, int *launches);   // blocks until the events have happened
// Shader clock under load: while the GEMM kind is being recorded, the 4-wave GEMM kernel stores the shader
// clock counter and the 100 MHz reference counter at its start and end into the four words this returns (device
// memory of the library's own, null when nothing is recorded); prof_read_clock turns them into MHz.
unsigned long long *prof_clock_words(bool recording);
int prof_read_clock(double *mhz, int *samples);
