// Dealing the units of a decode-attention call to the workers of the persistent grid
// (internal to the library: included by lamina_attn.hip for device and host code, and by the
// host-only check of these functions in the tests).
#ifndef LAMINA_SHARES_H
#define LAMINA_SHARES_H

#if defined(__HIPCC__)
#define LAMINA_HD __host__ __device__
#else
#define LAMINA_HD
#endif

// Dealing U units to n workers in contiguous shares.  `skew` = 0: as evenly as whole units
// allow.  Balanced mode uses skew = kParitySkew: even-numbered work-groups take (64 + skew) / 64
// of an even share and odd-numbered ones (64 - skew) / 64.  Work-groups go round-robin to the
// eight accelerator dies, and on every chip measured the odd dies stream 7-14 % slower than the
// even ones; with equal shares the even dies run dry while the odd ones still have a twelfth of
// their work, and the call's last tenth runs at half the memory rate.  Measured with the skew
// swept 0 / 2 / 4 / 6 on one chip (512 work-groups): workload 5 takes 374 / 367 / 362 / 367 us,
// workload 7 378 / 374 / 371 / 376 us, workload 3 85.2 / 84.4 / 84.3 / 84.8 us.  With a skew,
// worker j starts at unit floor(U * c(j) / c(n)), c(j) = 64 j + skew * (j odd).
// The main pass and the host-side accounting both use these two functions.
// (U never exceeds 2^30 -- checked at creation -- and c(n) < 2^17, so 64-bit products are exact.)
constexpr int kParitySkew = 4;
// The skew pays once a share is long enough for the dies' different speeds to show; a short
// call is still filling the memory pipeline for a good part of its time, which the dies do
// alike.  Measured with 256 work-groups, units per work-group / skew 0, 2, 4: 16 (8 requests x
// 8 kv heads x 8192 tokens) 52.1 / 49.6 / - us; 21 (20 x 8 x 4096) 61.7 / 61.3 / - us; 28
// (workload 3) - / 82.7 / 83.1 us; 32 (4 x 8 x 32768) - / 87.7 / 87.0 us; 41 (20 x 8 x 8192)
// - / 109.1 / 110.5 us; beyond that the full skew.  Half the skew from 12 units per
// work-group, all of it from 48.  (Below two units per work-group it has to be zero in any
// case: the merge pass relies on every work-group between a row's first and last piece holding
// a piece of it.)
LAMINA_HD inline int share_skew(bool balanced, unsigned U, unsigned n)
{
    if (!balanced || U < 12u * n)
        return 0;
    return U >= 48u * n ? kParitySkew : kParitySkew / 2;
}
LAMINA_HD inline unsigned share_begin(unsigned U, unsigned n, unsigned j, int skew)
{
    if (skew == 0) {
        // the first U % n workers take U / n + 1 units, the others U / n: with fewer units than
        // workers the workers that get one are the first U, without gaps
        const unsigned q = U / n, rem = U % n;
        return j * q + (j < rem ? j : rem);
    }
    const unsigned long long cj = 64ull * j + (unsigned long long)skew * (j & 1u);
    const unsigned long long cn = 64ull * n + (unsigned long long)skew * (n & 1u);
    return (unsigned)((unsigned long long)U * cj / cn);
}
// The worker whose share holds unit u (u < U): the largest j with share_begin(j) <= u.
LAMINA_HD inline int share_owner(unsigned U, unsigned n, unsigned u, int skew)
{
    if (skew == 0) {
        const unsigned q = U / n, rem = U % n;
        if (u < rem * (q + 1))
            return (int)(u / (q + 1));
        return (int)(rem + (u - rem * (q + 1)) / q);      // q >= 1 here: u >= rem * (q + 1)
    }
    long long j = (long long)((unsigned long long)u * n / U);              // a step or two off
    if (j > (long long)n - 1)
        j = (long long)n - 1;
    while (j > 0 && share_begin(U, n, (unsigned)j, skew) > u)
        --j;
    while (j + 1 < (long long)n && share_begin(U, n, (unsigned)j + 1, skew) <= u)
        ++j;
    return (int)j;
}

#endif  // LAMINA_SHARES_H
