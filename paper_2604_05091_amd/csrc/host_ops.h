// Host-side arithmetic of the library: the Adam update, the fp32 -> bf16 conversion of the
// streamed weight copy, rotary tables and a small fork-join helper.  CPU only.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <functional>

namespace mt {

int host_threads();
// Runs fn(begin, end) over [0, n) split into contiguous chunks on host_threads() threads.
void parallel_for(size_t n, size_t min_chunk, const std::function<void(size_t, size_t)> &fn);

void host_f32_to_bf16(uint16_t *out, const float *in, size_t n);
void host_adam(float *p, const float *g, float *m, float *v, uint16_t *shadow, size_t n, float lr, float beta1,
               float beta2, float eps, float wd, int64_t step);
void host_zero(void *p, size_t bytes);  // multi-threaded first touch
void rope_table(float *cs, float *sn, int T, int hd, double base);

}  // namespace mt
