/*
 * Seeded synthetic inputs: And-Inverter Graphs and Gaussian tensors.
 *
 * This file is INPUT code only. It is the one piece both the CPU oracle's
 * tests and the GPU path's tests/bench call, and it contains none of the
 * method's arithmetic (no levels-by-Eq.-1, no cones, no attention): it only
 * draws random graphs and random numbers.
 *
 * The graphs stand in for the circuit AIGs the paper evaluates on (ITC99,
 * EPFL, OpenABC-D, Section "Dataset Statistic"), which are not available:
 * node in-degree is 0 (primary input) or 2 (AND), inverters sit on edges.
 *
 * RNG: counter based. value(seed, stream, i) is a pure function, so every
 * draw can be reproduced independently and in parallel.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* 64-bit finaliser of the splitmix64 generator (Steele, Lea, Flood 2014). */
static inline uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

/* value(seed, stream, i): two rounds of the finaliser over a Weyl sequence. */
uint64_t dg4s_rand(uint64_t seed, uint64_t stream, uint64_t i)
{
    uint64_t a = mix64(seed + 0x9E3779B97F4A7C15ull * (stream + 1));
    return mix64(a ^ mix64(0x9E3779B97F4A7C15ull * (i + 1) + 0xD1B54A32D192ED03ull * stream));
}

/* uniform integer in [0, n), n >= 1: multiply-shift, no rejection. */
static inline uint64_t rand_below(uint64_t r, uint64_t n)
{
    return (uint64_t)(((unsigned __int128)r * n) >> 64);
}

/* uniform double in [0,1) with 53 bits. */
static inline double rand_unit(uint64_t r) { return (double)(r >> 11) * 0x1.0p-53; }

/* float -> nearest bfloat16 (ties to even), returned as a float. Input format
 * conversion only: bf16 configs feed values that are exactly representable. */
static inline float round_to_bf16(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return f;           /* inf / nan */
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return f;
}

/*
 * count standard normals * scale, by Box-Muller in double on counters
 * (2i, 2i+1) of the stream, cast to float, optionally rounded to bf16.
 */
void dg4s_normal(uint64_t seed, uint64_t stream, int64_t count, double scale,
                 int32_t to_bf16, float* out)
{
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        double u1 = 1.0 - rand_unit(dg4s_rand(seed, stream, 2 * (uint64_t)i));     /* (0,1] */
        double u2 = rand_unit(dg4s_rand(seed, stream, 2 * (uint64_t)i + 1));
        float z = (float)(scale * sqrt(-2.0 * log(u1)) * cos(two_pi * u2));
        out[i] = to_bf16 ? round_to_bf16(z) : z;
    }
}

/*
 * Synthetic AIG. Nodes 0..n_pi-1 are primary inputs; AND j has id n_pi + j and
 * two distinct fanins among earlier ids. Edges are emitted by destination,
 * fanin 0 then fanin 1: edge 2j and 2j+1 end in AND j.
 *
 *   window   size W of the "recent nodes" window (in creation order)
 *   p_window probability that a fanin is drawn from the window rather than
 *            uniformly from all earlier nodes. 1.0 = windowed generator:
 *            the pair is drawn without replacement from the last
 *            min(W, id) nodes.
 *   level_cap 0: no depth control. >0: each AND first draws a target level
 *            t ~ U{1..cap}; a fanin candidate is accepted only if its own
 *            assigned level is < t (primary inputs have level 0). After
 *            MAX_TRIES rejected draws the fanin falls back to a uniformly
 *            drawn primary input. The AND's assigned level is t; the
 *            assigned levels are returned in level_hint (a valid topological
 *            levelling, in general NOT the longest-path level).
 *
 * Streams: 1 fanin choices, 2 inverter flags, 3 target levels.
 * Returns 0, or -1 on bad arguments.
 */
#define MAX_TRIES 24
#define DRAWS_PER_NODE 128   /* counters reserved per AND on stream 1 */

int dg4s_aig(uint64_t seed, int64_t n_pi, int64_t n_and, int64_t window,
             double p_window, int32_t level_cap,
             int32_t* edge_src, int32_t* edge_dst, uint8_t* edge_inv,
             int32_t* level_hint /* [n_pi+n_and] or NULL */)
{
    if (n_pi < 2 || n_and < 0 || window < 2 || n_pi + n_and > 0x3FFFFFFF) return -1;
    if (level_cap > 0 && !level_hint) return -1;
    if (level_hint) memset(level_hint, 0, sizeof(int32_t) * (size_t)(n_pi + n_and));

    for (int64_t j = 0; j < n_and; ++j) {
        const int64_t id = n_pi + j;                 /* earlier nodes: 0..id-1 */
        const int64_t m = id < window ? id : window; /* window = ids id-m..id-1 */
        uint64_t ctr = (uint64_t)j * DRAWS_PER_NODE;
        int64_t f[2];

        if (level_cap <= 0 && p_window >= 1.0) {
            int64_t a = (int64_t)rand_below(dg4s_rand(seed, 1, ctr++), (uint64_t)m);
            int64_t b = (int64_t)rand_below(dg4s_rand(seed, 1, ctr++), (uint64_t)(m - 1));
            if (b >= a) ++b;
            f[0] = id - m + a; f[1] = id - m + b;
        } else {
            int32_t t = 0;
            if (level_cap > 0)
                t = 1 + (int32_t)rand_below(dg4s_rand(seed, 3, (uint64_t)j), (uint64_t)level_cap);
            for (int k = 0; k < 2; ++k) {
                int64_t pick = -1;
                for (int tries = 0; tries < MAX_TRIES && pick < 0; ++tries) {
                    int in_window = rand_unit(dg4s_rand(seed, 1, ctr++)) < p_window;
                    uint64_t r = dg4s_rand(seed, 1, ctr++);
                    int64_t c = in_window ? id - m + (int64_t)rand_below(r, (uint64_t)m)
                                          : (int64_t)rand_below(r, (uint64_t)id);
                    if (k == 1 && c == f[0]) continue;
                    if (level_cap > 0 && level_hint[c] >= t) continue;
                    pick = c;
                }
                if (pick < 0) {                      /* fall back to a primary input */
                    if (level_cap <= 0) {            /* only duplicates were rejected */
                        pick = (f[0] + 1) % id;
                    } else {
                        int64_t c = (int64_t)rand_below(dg4s_rand(seed, 1, ctr++), (uint64_t)n_pi);
                        if (k == 1 && c == f[0]) c = (c + 1) % n_pi;
                        pick = c;
                    }
                }
                f[k] = pick;
            }
            if (level_cap > 0) level_hint[id] = t;
        }
        for (int k = 0; k < 2; ++k) {
            edge_src[2 * j + k] = (int32_t)f[k];
            edge_dst[2 * j + k] = (int32_t)id;
            edge_inv[2 * j + k] = (uint8_t)(dg4s_rand(seed, 2, 2 * (uint64_t)j + k) >> 63);
        }
    }
    return 0;
}
