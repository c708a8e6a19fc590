// Table of rotary angles by position for the decode over a cache whose keys carry no position
// encoding (Sec. 3.3 "Positional Encoding": the positions that count are those within the cache, so
// they change whenever entries are dropped and cannot be baked into the stored keys).
//     table[pos][0][i] = cos(pos * base^(-2i/d)),  table[pos][1][i] = sin(pos * base^(-2i/d)),  i < d/2
// Built once per (base, d) in double precision and rounded to fp32; the decode kernels read rows of it.
#include "common.h"

namespace sepattn {

namespace {

constexpr int kTableThreads = 256;

__global__ __launch_bounds__(kTableThreads) void rope_table_kernel(int n_pos, int d, double log2_base,
                                                                  float *__restrict__ table) {
    const int h = d / 2;
    const long item = (long)blockIdx.x * kTableThreads + threadIdx.x;
    if (item >= (long)n_pos * h) return;
    const int pos = (int)(item / h), i = (int)(item % h);
    const double theta = exp2(-(2.0 * i / d) * log2_base);
    double sn, cs;
    sincos((double)pos * theta, &sn, &cs);
    table[(long)pos * d + i] = (float)cs;
    table[(long)pos * d + h + i] = (float)sn;
}

}  // namespace

int launch_rope_table(int n_pos, int d, double base, float *table, hipStream_t st) {
    const long items = (long)n_pos * (d / 2);
    const long blocks = (items + kTableThreads - 1) / kTableThreads;
    if (blocks > 0x7FFFFFFFL) return SEPATTN_ERR_SHAPE;
    ProfScope prof(SEPATTN_K_ROPE_TABLE, st);
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)blocks), dim3(kTableThreads), 0, st, n_pos, d, log2(base), table);
    return launch_status();
}

}  // namespace sepattn
