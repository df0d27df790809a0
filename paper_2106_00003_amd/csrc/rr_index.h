// Circle-method indexing shared by host and device code of the library.
//
// Section 3 / Figure 1 of the paper: the dimension sequence of block k+1 (k = 0..n-2) is
// obtained from (0, 1, ..., n-1) by holding element 0 and shifting the other n-1 elements
// cyclically k times, the last element moving to position 1 each time.  Written in closed
// form, the label at position q of that sequence is
//
//     seq_k[0] = 0,      seq_k[q] = 1 + ((q - 1 - k) mod (n - 1))   for q = 1..n-1,
//
// and arc p of the block joins positions p and n-1-p, i.e. the p-th position from each end.
// The prototype described in the paper's Section 3 derives (i, j) on the device from the step
// number in the same spirit; nothing but n, k and p is needed.
#pragma once

#if defined(__HIPCC__)
#define RR_HD __host__ __device__
#else
#define RR_HD
#endif

// Label held at position q (0 <= q < n) of the dimension sequence of block k+1 (0 <= k <= n-2).
RR_HD inline int rr_label(int n, int k, int q)
{
    if (q == 0) return 0;
    int v = q - 1 - k;          // in [-(n-2), n-2]
    if (v < 0) v += n - 1;
    return 1 + v;
}
