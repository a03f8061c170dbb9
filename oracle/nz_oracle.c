/*
 * nz_oracle.c -- plain CPU oracle for the multi-rail allreduce arithmetic.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product library may include, link
 * or call this file; it exists so that tests, the smoke check and the CPU
 * baseline leg of the benchmark have an independent statement of what the
 * GPU path must compute.  It shares no code, header, table or helper with the
 * HIP sources.
 *
 * What it states (Nezha, arXiv 2405.17870):
 *   - Sec. 3.4 / 3.5 / 4.2: the Load Balancer hands every member network one
 *     contiguous (ptr, data_length) slice of the message; the slices'
 *     proportions alpha sum to one (Sec. 4.3, text under Eq. 5).
 *   - Sec. 2.1.1, Eq. 1: a ring allreduce over N workers moves
 *     2(N-1) * M/N per worker: N-1 reduce-scatter steps and N-1 allgather
 *     steps over N pieces of the message.
 *   - Sec. 4.2: the "data aggregation (computation)" phase is the elementwise
 *     sum of the workers' gradients; every worker ends with the same sums.
 *   - Sec. 3.2: a rail's slice is staged from the user buffer (UnboundBuffer)
 *     into a contiguous per-rail Buffer and the result is returned.
 *
 * Everything is written as the definition or as the literal step sequence:
 * no blocking, no vectorisation, no reordering.  Floating-point definitional
 * sums are taken in fp64, left to right over the node index.
 *
 * Every function here is pinned by tests/test_oracle_*.py against closed
 * forms, brute force, hand-worked cases and library routines.  For the data
 * allocation scheme (Sec. 4.3) the oracle holds the definitions -- Eq. 4,
 * Eq. 5, the minimum of Eq. 5 over the shares, the threshold of Eq. 6 -- and
 * one subgradient reading of Eq. 7 / Eq. 8 (orc_balance_iterate); the
 * library's own iteration is judged against the definitions.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#include <math.h>

#define ORC_OK 0
#define ORC_BAD 1

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2, ORC_I32 = 3 };

static int elem_bytes_of(int dtype)
{
    switch (dtype) {
    case ORC_F32: return 4;
    case ORC_I32: return 4;
    case ORC_BF16: return 2;
    case ORC_F16: return 2;
    default: return 0;
    }
}

/* ---------------------------------------------------------------------- */
/* 16-bit float formats (IEEE binary16 and bfloat16), by their definitions */
/* ---------------------------------------------------------------------- */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* bfloat16 is the upper half of a binary32: widening appends 16 zero bits. */
float orc_bf16_to_f32(uint16_t h) { return bits_f32((uint32_t)h << 16); }

/* binary32 -> bfloat16, round to nearest, ties to even; NaN stays a quiet NaN. */
uint16_t orc_f32_to_bf16(float f)
{
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)            /* NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t low = u & 0xffffu;                      /* the 16 dropped bits   */
    uint32_t top = u >> 16;
    if (low > 0x8000u || (low == 0x8000u && (top & 1u)))
        top += 1u;              /* carries into the exponent (and to Inf) correctly */
    return (uint16_t)top;
}

/* IEEE binary16 -> binary32 (exact). */
float orc_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    int exp = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ffu;
    if (exp == 0x1f)
        return bits_f32(sign | 0x7f800000u | (man << 13));
    if (exp == 0) {
        /* zero or subnormal: value = man * 2^-24 */
        float v = ldexpf((float)man, -24);
        return sign ? -v : v;
    }
    return bits_f32(sign | ((uint32_t)(exp - 15 + 127) << 23) | (man << 13));
}

/* binary32 -> IEEE binary16, round to nearest, ties to even. */
uint16_t orc_f32_to_f16(float f)
{
    uint32_t u = f32_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u)
        return (uint16_t)(sign | 0x7e00u | ((a >> 13) & 0x3ffu));   /* quiet NaN */
    if (a == 0x7f800000u)
        return (uint16_t)(sign | 0x7c00u);
    /* |f| as an exact multiple of 2^-24 would overflow for large values, so
       split by magnitude. */
    float af = bits_f32(a);
    if (af >= 65520.0f)                   /* rounds to infinity (max half 65504, ulp 32) */
        return (uint16_t)(sign | 0x7c00u);
    if (af < 6.103515625e-05f) {          /* below 2^-14: subnormal half, spacing 2^-24 */
        /* nearbyintf in the default rounding mode is round-half-even; the
           scaling by 2^24 is exact. */
        float q = nearbyintf(ldexpf(af, 24));
        return (uint16_t)(sign | (uint16_t)q);     /* q == 1024 lands on the smallest normal */
    }
    int e = (int)(a >> 23) - 127;                  /* -14 .. 15 */
    uint32_t man = a & 0x7fffffu;
    uint32_t keep = man >> 13;
    uint32_t low = man & 0x1fffu;
    uint32_t h = ((uint32_t)(e + 15) << 10) | keep;
    if (low > 0x1000u || (low == 0x1000u && (keep & 1u)))
        h += 1u;                                   /* may carry into the exponent */
    return (uint16_t)(sign | h);
}

/* ---------------------------------------------------------------------- */
/* Rail partition (Sec. 3.5 Load Balancer, Sec. 4.3 proportions)           */
/* ---------------------------------------------------------------------- */

/*
 * Split [0, n) into n_rails contiguous ranges, in rail order, with lengths
 * proportional to the integer weights w[].  Every interior boundary is the
 * proportional point n * (w_0 + ... + w_{k-1}) / W rounded DOWN to a
 * multiple of align_elems; b[0] = 0 and b[n_rails] = n, so the last rail
 * takes whatever the rounding leaves.  A rail of weight zero is given nothing
 * (that is how "all data on the best rail", Eq. 4, and a failed rail,
 * Sec. 4.4, are expressed): once the weights before a boundary already add
 * up to W, that boundary is n itself, so the remainder goes to the last rail
 * of non-zero weight.
 */
int orc_rail_partition(uint64_t n, uint64_t align_elems, const uint32_t *w,
                       uint32_t n_rails, uint64_t *b)
{
    if (!w || !b || n_rails == 0 || align_elems == 0) return ORC_BAD;
    uint64_t W = 0;
    for (uint32_t k = 0; k < n_rails; ++k) W += w[k];
    if (W == 0) return ORC_BAD;
    b[0] = 0;
    uint64_t P = 0;
    for (uint32_t k = 1; k < n_rails; ++k) {
        P += w[k - 1];
        if (P == W) { b[k] = n; continue; }
        unsigned __int128 num = (unsigned __int128)n * P;
        unsigned __int128 den = (unsigned __int128)W * align_elems;
        b[k] = (uint64_t)(num / den) * align_elems;
    }
    b[n_rails] = n;
    return ORC_OK;
}

/* ---------------------------------------------------------------------- */
/* Ring segments (Eq. 1: N pieces of M/N)                                  */
/* ---------------------------------------------------------------------- */

/*
 * Cut every rail range [b[k], b[k+1]) into n_nodes consecutive segments whose
 * lengths differ by at most one element, the longer ones first.
 * seg is [n_rails][n_nodes + 1]: segment j of rail k is
 * [seg[k][j], seg[k][j+1]).
 */
int orc_segment_map(const uint64_t *b, uint32_t n_rails, uint32_t n_nodes,
                    uint64_t *seg)
{
    if (!b || !seg || n_rails == 0 || n_nodes == 0) return ORC_BAD;
    for (uint32_t k = 0; k < n_rails; ++k) {
        if (b[k + 1] < b[k]) return ORC_BAD;
        uint64_t L = b[k + 1] - b[k];
        uint64_t q = L / n_nodes, r = L % n_nodes;
        uint64_t *row = seg + (size_t)k * (n_nodes + 1);
        row[0] = b[k];
        for (uint32_t j = 0; j < n_nodes; ++j)
            row[j + 1] = row[j] + q + (j < r ? 1u : 0u);
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------- */
/* Definitional allreduce: out[x] = sum over nodes of in[i][x] (Sec. 4.2)  */
/* ---------------------------------------------------------------------- */

/*
 * Floating-point inputs: each element is widened exactly to fp64 and the N
 * values are added left to right in fp64.  sum[x] receives the total and
 * abssum[x] (may be NULL) the sum of magnitudes, which scales the tolerance.
 */
int orc_sum_float(int dtype, const void *const *in, uint32_t n_nodes,
                  uint64_t n, double *sum, double *abssum)
{
    if (!in || !sum || n_nodes == 0) return ORC_BAD;
    if (dtype != ORC_F32 && dtype != ORC_BF16 && dtype != ORC_F16) return ORC_BAD;
#pragma omp parallel for schedule(static)
    for (uint64_t x = 0; x < n; ++x) {
        double s = 0.0, a = 0.0;
        for (uint32_t i = 0; i < n_nodes; ++i) {
            double v;
            if (dtype == ORC_F32)
                v = (double)((const float *)in[i])[x];
            else if (dtype == ORC_BF16)
                v = (double)orc_bf16_to_f32(((const uint16_t *)in[i])[x]);
            else
                v = (double)orc_f16_to_f32(((const uint16_t *)in[i])[x]);
            if (i == 0) s = v; else s += v;    /* no "+0.0" in front: keeps -0 */
            a += fabs(v);
        }
        sum[x] = s;
        if (abssum) abssum[x] = a;
    }
    return ORC_OK;
}

/* int32 inputs: two's-complement wrapping sum (computed in uint32). */
int orc_sum_i32(const void *const *in, uint32_t n_nodes, uint64_t n, int32_t *out)
{
    if (!in || !out || n_nodes == 0) return ORC_BAD;
#pragma omp parallel for schedule(static)
    for (uint64_t x = 0; x < n; ++x) {
        uint32_t s = 0;
        for (uint32_t i = 0; i < n_nodes; ++i)
            s += ((const uint32_t *)in[i])[x];
        out[x] = (int32_t)s;
    }
    return ORC_OK;
}

/*
 * The value a 16-bit-float output must be compared with: the fp64 sum rounded
 * once to fp32 (the accumulator precision) and then once to the storage type.
 */
int orc_round_to_storage(int dtype, const double *sum, uint64_t n, void *out)
{
    if (!sum || !out) return ORC_BAD;
    for (uint64_t x = 0; x < n; ++x) {
        float f = (float)sum[x];
        if (dtype == ORC_F32) ((float *)out)[x] = f;
        else if (dtype == ORC_BF16) ((uint16_t *)out)[x] = orc_f32_to_bf16(f);
        else if (dtype == ORC_F16) ((uint16_t *)out)[x] = orc_f32_to_f16(f);
        else return ORC_BAD;
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------- */
/* Step-by-step ring allreduce (Eq. 1)                                     */
/* ---------------------------------------------------------------------- */

static void add_into(int dtype, void *dst, const void *src, uint64_t off, uint64_t len)
{
    /* dst[off..off+len) = storage( fp32(src) + fp32(dst) ); the received
       partial is the left operand.  int32 wraps. */
    for (uint64_t x = off; x < off + len; ++x) {
        switch (dtype) {
        case ORC_F32: {
            volatile float s = ((const float *)src)[x] + ((float *)dst)[x];
            ((float *)dst)[x] = s;
            break;
        }
        case ORC_I32:
            ((uint32_t *)dst)[x] = ((const uint32_t *)src)[x] + ((uint32_t *)dst)[x];
            break;
        case ORC_BF16: {
            volatile float s = orc_bf16_to_f32(((const uint16_t *)src)[x]) +
                               orc_bf16_to_f32(((uint16_t *)dst)[x]);
            ((uint16_t *)dst)[x] = orc_f32_to_bf16(s);
            break;
        }
        case ORC_F16: {
            volatile float s = orc_f16_to_f32(((const uint16_t *)src)[x]) +
                               orc_f16_to_f32(((uint16_t *)dst)[x]);
            ((uint16_t *)dst)[x] = orc_f32_to_f16(s);
            break;
        }
        }
    }
}

/* The N-1 reduce-scatter steps (receive-and-add) over every rail. */
static void ring_reduce_scatter(int dtype, int e, void *const *buf, uint32_t N,
                                const uint64_t *seg, uint32_t n_rails, uint64_t *sent_bytes)
{
    for (uint32_t s = 0; s + 1 < N; ++s) {
        for (uint32_t k = 0; k < n_rails; ++k) {
            const uint64_t *row = seg + (size_t)k * (N + 1);
            for (uint32_t r = 0; r < N; ++r) {
                uint32_t j = (r + N - s) % N;
                uint32_t d = (r + 1) % N;
                uint64_t off = row[j], len = row[j + 1] - row[j];
                add_into(dtype, buf[d], buf[r], off, len);
                if (sent_bytes) sent_bytes[r] += len * (uint64_t)e;
            }
        }
    }
}

/* The N-1 allgather steps (receive-and-overwrite) over every rail. */
static void ring_allgather(int e, void *const *buf, uint32_t N, const uint64_t *seg,
                           uint32_t n_rails, uint64_t *sent_bytes)
{
    for (uint32_t s = 0; s + 1 < N; ++s) {
        for (uint32_t k = 0; k < n_rails; ++k) {
            const uint64_t *row = seg + (size_t)k * (N + 1);
            for (uint32_t r = 0; r < N; ++r) {
                uint32_t j = (r + 1 + N - s) % N;
                uint32_t d = (r + 1) % N;
                uint64_t off = row[j], len = row[j + 1] - row[j];
                memcpy((char *)buf[d] + off * e, (const char *)buf[r] + off * e, len * e);
                if (sent_bytes) sent_bytes[r] += len * (uint64_t)e;
            }
        }
    }
}

/*
 * Literal emulation of a ring allreduce run independently on every rail.
 *
 * buf[i] is node i's private buffer of n elements; on entry it holds node i's
 * gradients, on exit the allreduced result.  Node r always sends to node
 * (r+1) mod N.  In reduce-scatter step s (s = 0 .. N-2) it sends segment
 * (r - s) mod N of every rail and the receiver adds it into its own copy,
 * storing the partial in the storage type; after the last such step node r
 * holds the complete segment (r + 1) mod N.  In allgather step s it sends
 * segment (r + 1 - s) mod N and the receiver overwrites its copy.
 *
 * All sends of one step happen "at once": a step's sends are taken from the
 * state at the start of the step.  No segment is both sent and received by
 * one node in the same step, so processing the nodes one after another is
 * the same thing.
 *
 * stop_after_reduce_scatter != 0 returns after the first N-1 steps.
 * sent_bytes[i] (may be NULL) is incremented by what node i puts on the wire.
 */
int orc_ring_allreduce(int dtype, void *const *buf, uint32_t n_nodes, uint64_t n,
                       const uint64_t *seg, uint32_t n_rails,
                       int stop_after_reduce_scatter, uint64_t *sent_bytes)
{
    int e = elem_bytes_of(dtype);
    if (!buf || !seg || n_nodes == 0 || n_rails == 0 || e == 0) return ORC_BAD;
    (void)n;
    ring_reduce_scatter(dtype, e, buf, n_nodes, seg, n_rails, sent_bytes);
    if (!stop_after_reduce_scatter)
        ring_allgather(e, buf, n_nodes, seg, n_rails, sent_bytes);
    return ORC_OK;
}

/*
 * The allgather half on its own: on entry node r's buffer holds valid data in
 * segment (r + 1) mod N of every rail (what the reduce-scatter leaves it
 * owning); on exit every buffer holds every segment.  N - 1 steps, node r
 * sending segment (r + 1 - s) mod N to node (r + 1) mod N in step s.
 */
int orc_ring_allgather(int dtype, void *const *buf, uint32_t n_nodes, uint64_t n,
                       const uint64_t *seg, uint32_t n_rails, uint64_t *sent_bytes)
{
    int e = elem_bytes_of(dtype);
    if (!buf || !seg || n_nodes == 0 || n_rails == 0 || e == 0) return ORC_BAD;
    (void)n;
    ring_allgather(e, buf, n_nodes, seg, n_rails, sent_bytes);
    return ORC_OK;
}

/*
 * Ring allreduce with every segment transfer cut into pieces of at most
 * chunk_elems elements, sent one after another (the "Ring_Chunked" variant
 * the evaluation section mentions: large packets are split and their
 * transmission pipelined).  Within a step, piece c of every (rail, node) is
 * moved before piece c + 1.  The arithmetic per element is that of the plain
 * ring.  messages[i] (may be NULL) counts the non-empty pieces node i sends.
 */
int orc_ring_allreduce_chunked(int dtype, void *const *buf, uint32_t n_nodes, uint64_t n,
                               const uint64_t *seg, uint32_t n_rails, uint64_t chunk_elems,
                               uint64_t *sent_bytes, uint64_t *messages)
{
    int e = elem_bytes_of(dtype);
    if (!buf || !seg || n_nodes == 0 || n_rails == 0 || e == 0 || chunk_elems == 0) return ORC_BAD;
    (void)n;
    const uint32_t N = n_nodes;
    uint64_t longest = 0;
    for (uint32_t k = 0; k < n_rails; ++k)
        for (uint32_t j = 0; j < N; ++j) {
            uint64_t len = seg[(size_t)k * (N + 1) + j + 1] - seg[(size_t)k * (N + 1) + j];
            if (len > longest) longest = len;
        }
    const uint64_t n_chunks = (longest + chunk_elems - 1) / chunk_elems;
    for (int phase = 0; phase < 2; ++phase) {
        for (uint32_t s = 0; s + 1 < N; ++s) {
            for (uint64_t c = 0; c < n_chunks; ++c) {
                for (uint32_t k = 0; k < n_rails; ++k) {
                    const uint64_t *row = seg + (size_t)k * (N + 1);
                    for (uint32_t r = 0; r < N; ++r) {
                        uint32_t j = phase == 0 ? (r + N - s) % N : (r + 1 + N - s) % N;
                        uint32_t d = (r + 1) % N;
                        uint64_t len = row[j + 1] - row[j];
                        uint64_t lo = c * chunk_elems;
                        if (lo >= len) continue;
                        uint64_t piece = len - lo < chunk_elems ? len - lo : chunk_elems;
                        uint64_t off = row[j] + lo;
                        if (phase == 0)
                            add_into(dtype, buf[d], buf[r], off, piece);
                        else
                            memcpy((char *)buf[d] + off * e, (const char *)buf[r] + off * e, piece * e);
                        if (sent_bytes) sent_bytes[r] += piece * (uint64_t)e;
                        if (messages) messages[r] += 1;
                    }
                }
            }
        }
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------- */
/* Fault tolerance (Sec. 4.4)                                              */
/* ---------------------------------------------------------------------- */

/*
 * The member network that takes over a failed rail's (ptr, data_length): the
 * surviving rail that was allocated the most data (the paper takes the rail
 * handling more data to be the more performant one); among equals the lowest
 * index.  alive[k] != 0 marks a surviving rail.  Returns ORC_BAD if none
 * survives.
 */
int orc_failover_target(const uint64_t *b, uint32_t n_rails, const uint8_t *alive, uint32_t *target)
{
    if (!b || !alive || !target || n_rails == 0) return ORC_BAD;
    int found = 0;
    uint64_t best_len = 0;
    for (uint32_t k = 0; k < n_rails; ++k) {
        if (!alive[k]) continue;
        uint64_t len = b[k + 1] - b[k];
        if (!found || len > best_len) { found = 1; best_len = len; *target = k; }
    }
    return found ? ORC_OK : ORC_BAD;
}

/* ---------------------------------------------------------------------- */
/* Pack / unpack (Sec. 3.2: UnboundBuffer <-> per-rail Buffer)             */
/* ---------------------------------------------------------------------- */

/*
 * Concatenate the listed segments of one rail, in list order and without
 * padding, from node_buf into send_buf.  Returns the byte count through
 * packed_bytes.  seg is the table of orc_segment_map.
 */
int orc_pack(const void *node_buf, const uint64_t *seg, uint32_t n_nodes,
             uint32_t rail, const uint32_t *seg_ids, uint32_t n_segs,
             uint32_t elem_bytes, void *send_buf, uint64_t *packed_bytes)
{
    if (!node_buf || !seg || !send_buf || (!seg_ids && n_segs)) return ORC_BAD;
    const uint64_t *row = seg + (size_t)rail * (n_nodes + 1);
    uint64_t pos = 0;
    for (uint32_t i = 0; i < n_segs; ++i) {
        uint32_t j = seg_ids[i];
        if (j >= n_nodes) return ORC_BAD;
        uint64_t bytes = (row[j + 1] - row[j]) * elem_bytes;
        memcpy((char *)send_buf + pos, (const char *)node_buf + row[j] * elem_bytes, bytes);
        pos += bytes;
    }
    if (packed_bytes) *packed_bytes = pos;
    return ORC_OK;
}

/* Inverse of orc_pack: scatter send_buf back into the listed segments. */
int orc_unpack(const void *send_buf, const uint64_t *seg, uint32_t n_nodes,
               uint32_t rail, const uint32_t *seg_ids, uint32_t n_segs,
               uint32_t elem_bytes, void *node_buf)
{
    if (!node_buf || !seg || !send_buf || (!seg_ids && n_segs)) return ORC_BAD;
    const uint64_t *row = seg + (size_t)rail * (n_nodes + 1);
    uint64_t pos = 0;
    for (uint32_t i = 0; i < n_segs; ++i) {
        uint32_t j = seg_ids[i];
        if (j >= n_nodes) return ORC_BAD;
        uint64_t bytes = (row[j + 1] - row[j]) * elem_bytes;
        memcpy((char *)node_buf + row[j] * elem_bytes, (const char *)send_buf + pos, bytes);
        pos += bytes;
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------- */
/* Data allocation scheme (Sec. 4.3, Eq. 4-8)                              */
/* ---------------------------------------------------------------------- */

/*
 * Rail i is modelled by its startup latency t_setup[i] (seconds) and its
 * effective bandwidth bw[i] (bytes per second); S is the message size.
 *
 * Eq. 4: cold start, all data on the best single rail.
 */
double orc_t_cold(uint32_t n_rails, const double *t_setup, const double *bw, double S,
                  uint32_t *best)
{
    double t = 0.0;
    for (uint32_t i = 0; i < n_rails; ++i) {
        double ti = t_setup[i] + S / bw[i];
        if (i == 0 || ti < t) { t = ti; if (best) *best = i; }
    }
    return t;
}

/*
 * Eq. 5: hot start, rail i carries the share alpha[i]; the allreduce ends
 * when the slowest rail ends.  A rail that is given nothing (alpha = 0) does
 * not take part, so its startup latency does not count.
 */
double orc_t_hot(uint32_t n_rails, const double *t_setup, const double *bw, double S,
                 const double *alpha, uint32_t *slowest)
{
    double t = 0.0;
    int any = 0;
    for (uint32_t i = 0; i < n_rails; ++i) {
        if (!(alpha[i] > 0.0)) continue;
        double ti = t_setup[i] + alpha[i] * S / bw[i];
        if (!any || ti > t) { t = ti; any = 1; if (slowest) *slowest = i; }
    }
    return t;
}

/*
 * The Load Balancer's iteration.
 *   Eq. 8: starting shares from the rails' latencies T_i under a uniform
 *          allocation, alpha_i = (T - T_i) / (T (R - 1)) with T = sum T_i and
 *          R the number of member networks (with that reading the shares sum
 *          to one).
 *   Eq. 7: alpha <- alpha - eta * dT_hot/dalpha.  T_hot is a maximum, so the
 *          derivative is S / bw on the slowest rail and zero elsewhere: the
 *          step takes share away from the slowest rail.  eta is taken relative
 *          to the derivative's size: in step k the slowest rail gives up
 *          0.25 / sqrt(k + 1) of the message, but never more than half of
 *          what it has; what it gives up is spread evenly over the other
 *          rails that take part, which keeps the shares summing to one.  A
 *          rail whose share falls below 2^-21 (less than one unit of the
 *          data-length table) is given nothing from then on and sits out.
 *          The best shares seen are kept, as any subgradient iteration must
 *          to settle.
 * Returns the best T_hot found; alpha receives its shares.
 */
double orc_balance_iterate(uint32_t n_rails, const double *t_setup, const double *bw, double S,
                           uint32_t iterations, double *alpha)
{
    if (n_rails == 0 || n_rails > 64) return -1.0;
    double a[64], best_a[64];
    const uint32_t R = n_rails;
    if (R == 1) { alpha[0] = 1.0; return t_setup[0] + S / bw[0]; }
    double T = 0.0, Ti[64];
    for (uint32_t i = 0; i < R; ++i) {
        Ti[i] = t_setup[i] + (S / R) / bw[i];
        T += Ti[i];
    }
    for (uint32_t i = 0; i < R; ++i) a[i] = (T - Ti[i]) / (T * (double)(R - 1));
    double best_t = orc_t_hot(R, t_setup, bw, S, a, NULL);
    for (uint32_t i = 0; i < R; ++i) best_a[i] = a[i];
    const double floor_share = 1.0 / 2097152.0;
    for (uint32_t k = 0; k < iterations; ++k) {
        uint32_t worst = 0, taking_part = 0;
        (void)orc_t_hot(R, t_setup, bw, S, a, &worst);
        for (uint32_t i = 0; i < R; ++i) taking_part += a[i] > 0.0;
        if (taking_part < 2) break;
        double give = 0.25 / sqrt((double)k + 1.0);
        if (give > 0.5 * a[worst]) give = 0.5 * a[worst];
        if (a[worst] - give < floor_share) { give = a[worst]; taking_part -= 1; }
        a[worst] -= give;
        if (a[worst] < 0.0 || give == 0.0) a[worst] = 0.0;
        uint32_t others = a[worst] > 0.0 ? taking_part - 1 : taking_part;
        for (uint32_t i = 0; i < R; ++i)
            if (i != worst && a[i] > 0.0) a[i] += give / (double)others;
        double t = orc_t_hot(R, t_setup, bw, S, a, NULL);
        if (t < best_t) { best_t = t; for (uint32_t i = 0; i < R; ++i) best_a[i] = a[i]; }
    }
    for (uint32_t i = 0; i < R; ++i) alpha[i] = best_a[i];
    return best_t;
}

/*
 * The definition the iteration aims at: the smallest value Eq. 5 can take
 * over all shares alpha >= 0 that sum to one (rails given nothing sit out),
 * found without any step rule.
 *
 * If the allreduce is to end by time T, rail i can carry at most
 * (T - T_setup_i) * B_i bytes (nothing if T <= T_setup_i).  The capacity
 *   cap(T) = sum_i max(0, (T - T_setup_i) * B_i)
 * grows with T, and S bytes can be finished by time T exactly when
 * cap(T) >= S.  The minimum of Eq. 5 is therefore the T with cap(T) = S,
 * located here by plain bisection; the shares that reach it give each rail
 * what it can carry by then, alpha_i = max(0, (T - T_setup_i) * B_i) / S.
 * Returns T; alpha (may be NULL) receives the shares.  S > 0.
 */
static double capacity_by(uint32_t n_rails, const double *t_setup, const double *bw, double T)
{
    double cap = 0.0;
    for (uint32_t i = 0; i < n_rails; ++i)
        if (T > t_setup[i]) cap += (T - t_setup[i]) * bw[i];
    return cap;
}

double orc_balance_optimum(uint32_t n_rails, const double *t_setup, const double *bw, double S,
                           double *alpha)
{
    if (n_rails == 0 || !(S > 0.0)) return -1.0;
    /* cap(lo) = 0 < S at the smallest startup latency; the best single rail's
     * finishing time (Eq. 4) is certainly enough. */
    double lo = t_setup[0];
    for (uint32_t i = 1; i < n_rails; ++i)
        if (t_setup[i] < lo) lo = t_setup[i];
    double hi = orc_t_cold(n_rails, t_setup, bw, S, NULL);
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (capacity_by(n_rails, t_setup, bw, mid) < S) lo = mid; else hi = mid;
    }
    if (alpha)
        for (uint32_t i = 0; i < n_rails; ++i)
            alpha[i] = hi > t_setup[i] ? (hi - t_setup[i]) * bw[i] / S : 0.0;
    return hi;
}

/*
 * Eq. 6: the message size at which cold start (Eq. 4) and hot start with its
 * best shares (the minimum of Eq. 5) take the same time.  Sharing can never
 * be slower than the best single rail, so T_cold(S) - T_hot(S) is zero up to
 * the threshold and positive beyond it; the threshold is the largest S at
 * which the two are still equal.  Bisection on S.  "Equal" means a relative
 * difference of at most 1e-12 (the accuracy of the inner bisection).
 * Returns HUGE_VAL when no size up to 1e30 bytes makes sharing pay (a single
 * rail).
 */
static int sharing_pays(uint32_t n_rails, const double *t_setup, const double *bw, double S)
{
    double cold = orc_t_cold(n_rails, t_setup, bw, S, NULL);
    double hot = orc_balance_optimum(n_rails, t_setup, bw, S, NULL);
    return cold - hot > 1e-12 * cold;
}

double orc_threshold(uint32_t n_rails, const double *t_setup, const double *bw)
{
    if (n_rails == 0) return -1.0;
    double hi = 1.0;
    while (!sharing_pays(n_rails, t_setup, bw, hi)) {
        hi *= 2.0;
        if (hi > 1e30) return HUGE_VAL;
    }
    double lo = 0.0;   /* at S -> 0 everything goes to the rail that starts first */
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (mid <= 0.0) break;
        if (sharing_pays(n_rails, t_setup, bw, mid)) hi = mid; else lo = mid;
    }
    return lo;
}

/* ---------------------------------------------------------------------- */
/* Network efficiency and the efficiency ratio (Sec. 2.1.2 Eq. 2,          */
/* Sec. 2.2.1 Eq. 3)                                                       */
/* ---------------------------------------------------------------------- */

/*
 * Eq. 2: efficiency of one network on a message of S bytes,
 *   delta = T_theoretical / T_actual = 1 / (1 + T_setup / (S / B)),
 * with T_theoretical = S / B the transmission time without overheads.
 * S must be positive.
 */
double orc_net_efficiency(double t_setup, double bw, double S)
{
    double t_theoretical = S / bw;
    return 1.0 / (1.0 + t_setup / t_theoretical);
}

/*
 * Eq. 3: real-time efficiency ratio of networks i and j that carry S_i and
 * S_j bytes of one message,
 *   rho = (S_i * delta_i / That_i) / (S_j * delta_j / That_j),
 * delta from Eq. 2 at the network's own volume and That = S / B its ideal
 * transmission time: numerator and denominator are the two networks'
 * throughputs at that moment.  S_i, S_j must be positive.
 */
double orc_efficiency_ratio(double t_setup_i, double bw_i, double S_i,
                            double t_setup_j, double bw_j, double S_j)
{
    double num = S_i * orc_net_efficiency(t_setup_i, bw_i, S_i) / (S_i / bw_i);
    double den = S_j * orc_net_efficiency(t_setup_j, bw_j, S_j) / (S_j / bw_j);
    return num / den;
}

#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
/* Number of host threads the definitional sums use from now on (timing aid; no arithmetic). */
void orc_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int orc_threads(void) { return 1; }
void orc_set_threads(int n) { (void)n; }
#endif
