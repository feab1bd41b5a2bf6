/*
 * Sanitizer driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY (tests/test_oracle_pins.py builds it with
 * -fsanitize=address,undefined and runs it): the oracle's C code is included whole and run on small inputs that
 * reach its corners -- all three storage types, both metrics, empty lists, skipped and out-of-range probe places,
 * fewer candidates than k, nprobe = nlist -- so that an out-of-bounds access, a use after free or undefined
 * arithmetic in it stops the run.  It checks two invariants on the way (whole search with nprobe = nlist equals
 * the exhaustive search; every reported id lies in a probed list) and prints "oracle sanitize ok".
 */
#include "ivf_oracle.c"

#include <stdio.h>

static unsigned long long rng_state = 88172645463325252ULL;
static double rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 - 0.5;
}

static uint16_t to_bf16(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16); }
/* float -> binary16 for values of ordinary magnitude (round to nearest even; inputs here are in [-0.5, 0.5]) */
static uint16_t to_half(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    int exp = (int)((u >> 23) & 0xff) - 127 + 15;
    uint32_t man = u & 0x7fffffu;
    if (exp <= 0) return (uint16_t)sign;                        /* tiny: flushed, fine for this driver */
    uint32_t h = sign | ((uint32_t)exp << 10) | (man >> 13);
    if ((man & 0x1fffu) > 0x1000u || ((man & 0x1fffu) == 0x1000u && (h & 1u))) h++;
    return (uint16_t)h;
}

int main(void)
{
    enum { NLIST = 7, N = 61, D = 24, NQ = 9, K = 12 };
    const int64_t off[NLIST + 1] = {0, 5, 5, 20, 21, 40, 40, 61};      /* lists 1 and 5 are empty */
    float cent[NLIST * D], q[NQ * D], xf[N * D];
    uint16_t xh[N * D], xb[N * D];
    int64_t ids[N];
    for (int i = 0; i < NLIST * D; i++) cent[i] = (float)rnd();
    for (int i = 0; i < NQ * D; i++) q[i] = (float)rnd();
    for (int i = 0; i < N * D; i++) { xf[i] = (float)rnd(); xh[i] = to_half(xf[i]); xb[i] = to_bf16(xf[i]); }
    for (int i = 0; i < N; i++) ids[i] = 1000 + (i * 37) % N;
    const void *tabs[3] = {xf, xh, xb};
    for (int dtype = 0; dtype < 3; dtype++) {
        for (int metric = 0; metric < 2; metric++) {
            int32_t probe[NQ * NLIST];
            double psc[NQ * NLIST], s1[NQ * K], s2[NQ * K];
            int64_t i1[NQ * K], i2[NQ * K];
            if (oracle_ivf_search(q, NQ, D, cent, off, NLIST, tabs[dtype], dtype, ids, NLIST, K, metric, probe, i1, s1)) return 1;
            if (oracle_bruteforce(q, NQ, D, tabs[dtype], dtype, ids, N, K, metric, i2, s2)) return 2;
            if (memcmp(i1, i2, sizeof i1) || memcmp(s1, s2, sizeof s1)) { printf("nprobe = nlist differs from exhaustive\n"); return 3; }
            /* three places per query: one skipped, one out of range (skipped), one real; k exceeds a list's size */
            if (oracle_coarse(q, NQ, cent, NLIST, D, metric, 3, probe, psc)) return 4;
            for (int qi = 0; qi < NQ; qi++) { probe[qi * 3 + 1] = -1; if (qi & 1) probe[qi * 3 + 2] = NLIST + 5; }
            if (oracle_scan(q, NQ, D, off, NLIST, tabs[dtype], dtype, ids, probe, 3, K, metric, i1, s1)) return 5;
            for (int qi = 0; qi < NQ; qi++)
                for (int j = 0; j < K; j++) {
                    const int64_t id = i1[qi * K + j];
                    if (id < 0) continue;
                    int found = 0;
                    for (int p = 0; p < 3; p++) {
                        const int l = probe[qi * 3 + p];
                        if (l < 0 || l >= NLIST) continue;
                        for (int64_t r = off[l]; r < off[l + 1]; r++) found |= ids[r] == id;
                    }
                    if (!found) { printf("id outside the probed lists\n"); return 6; }
                }
            int64_t qi_[4] = {0, 3, 8, 8}, ri_[4] = {0, 60, 20, 5};
            double ps[4];
            if (oracle_pair_scores(q, D, tabs[dtype], dtype, metric, qi_, ri_, 4, ps)) return 7;
        }
    }
    oracle_set_threads(1);
    if (oracle_num_threads() < 1) return 8;
    printf("oracle sanitize ok\n");
    return 0;
}
