/*
 * r2_oracle.c -- CPU oracle for the resilient ring all-reduce hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * statement of what the hot path computes.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the product library never
 * does, and the two share no code, headers, tables or helpers.
 *
 * What is modelled (R2CCL paper):
 *   - Sec. 2.1 "GPU Cluster & Collective Communication": a collective's data
 *     is partitioned over channels, each bound to one NIC of the server.
 *   - Sec. 5.1 "R2CCL Load Balancing", paragraph R2CCL-Balance: when a NIC
 *     fails, its share of the server's data D_i is spread over the healthy
 *     NICs in proportion to their available bandwidth; paragraph "Overhead
 *     Analysis": the volumes themselves do not change.
 *   - Sec. 5.2 "Standard AllReduce algorithms": ring all-reduce is a
 *     reduce-scatter over all ranks followed by an all-gather.
 *   - Sec. 4.3 Technique II: send buffers are NIC-registered DMA (staging)
 *     buffers and progress is chunk-granular.
 *   - Appendix C (failure scope table): at least one healthy NIC must remain.
 *
 * Floating point: fp32 adds in the ring's fixed order; bf16 values are
 * widened to fp32, added, and rounded to nearest-even back to bf16 after
 * every hop (the wire and the buffers are bf16).  The paper states no
 * precision; this reading is fixed by the build's problem statement.
 *
 * Build: gcc -O2 -fno-fast-math -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    R2O_OK = 0,
    R2O_INVALID = -1,
    R2O_NO_HEALTHY_CHANNEL = -2,
    R2O_CAPACITY = -4,
    R2O_NOMEM = -6
};

enum { R2O_F32 = 0, R2O_BF16 = 1 };
enum { R2O_OP_SUM = 0, R2O_OP_COPY = 1, R2O_OP_SUM_FORWARD = 2 };
enum { R2O_PHASE_RS = 1, R2O_PHASE_AG = 2 };

#define R2O_MAX_CHANNELS 64

typedef struct {
    uint64_t t_start;        /* first transmission index this state applies to */
    uint64_t fail_mask;      /* bit c set = channel c is down                  */
    const uint32_t *weights; /* C bandwidth weights                            */
} r2o_epoch;

/* ------------------------------------------------------------------ */
/* bf16 <-> fp32 (IEEE round-to-nearest-even on the 16 dropped bits)   */
/* ------------------------------------------------------------------ */

float r2o_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

uint16_t r2o_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) /* NaN: keep sign, force quiet bit */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t kept_lsb = (u >> 16) & 1u;
    u += 0x7fffu + kept_lsb; /* ties go to the even kept mantissa */
    return (uint16_t)(u >> 16);
}

static size_t elem_size(int dtype) { return dtype == R2O_F32 ? 4 : 2; }

/* ------------------------------------------------------------------ */
/* Partition of one chunk over the channels (Sec. 5.1, R2CCL-Balance)  */
/* ------------------------------------------------------------------ */
/*
 * Healthy channels share `bytes` in proportion to their weights; a failed
 * channel gets nothing.  The paper gives the rule only in words, so the
 * rounding is fixed here: channel c starts at the cumulative share of the
 * channels before it, floored to whole alignment units,
 *     off[c] = align * floor(U * P_c / W),  U = floor(bytes/align),
 *     P_c = sum of effective weights before c,  W = their total,
 * and once every unit of weight has been passed (P_c == W) at `bytes`, so
 * the sub-alignment tail lands on the last healthy channel.
 * off has C+1 entries; slice c is bytes [off[c], off[c+1]).
 */
int r2o_partition(const uint32_t *weights, uint64_t fail_mask, uint32_t C,
                  uint64_t bytes, uint32_t align, uint64_t *off)
{
    if (!weights || !off || C == 0 || C > R2O_MAX_CHANNELS || align == 0)
        return R2O_INVALID;

    uint64_t e[R2O_MAX_CHANNELS];
    unsigned __int128 W = 0;
    for (uint32_t c = 0; c < C; ++c) {
        e[c] = ((fail_mask >> c) & 1u) ? 0u : weights[c];
        W += e[c];
    }
    if (W == 0) {
        for (uint32_t c = 0; c <= C; ++c) off[c] = 0;
        return R2O_NO_HEALTHY_CHANNEL;
    }
    uint64_t U = bytes / align;
    unsigned __int128 P = 0;
    for (uint32_t c = 0; c < C; ++c) {
        if (P == W)
            off[c] = bytes;
        else
            off[c] = (uint64_t)align * (uint64_t)(((unsigned __int128)U * P) / W);
        P += e[c];
    }
    off[C] = bytes;
    return R2O_OK;
}

/* ------------------------------------------------------------------ */
/* In-flight failover plan (Sec. 4.3 live migration + Sec. 5.1 shares)  */
/* ------------------------------------------------------------------ */
/*
 * A chunk was staged with table `off` while the channels of mask_before were
 * down.  During the transmission the channels of mask_after (a superset) are
 * down.  The data stays where it is: every NIC is registered on every stage
 * buffer and send buffers stay intact until completion (Sec. 4.3, Techniques
 * I and II), so only the carrier changes.  The slice of each newly failed
 * channel f, bytes [0, len_f) of stage buffer f, is shared out over the
 * channels still healthy, in proportion to their bandwidth (Sec. 5.1), by the
 * same cumulative-floor rule as the partition itself.
 * plan: C rows of C+1 cut points; row f is relative to the start of slice f,
 * NIC c carries bytes [plan[f][c], plan[f][c+1]) of buffer f.  Rows of channels
 * that did not newly fail are all zero.
 */
int r2o_rollback_plan(const uint64_t *off, const uint32_t *weights, uint64_t mask_before,
                      uint64_t mask_after, uint32_t C, uint32_t align, uint64_t *plan)
{
    if (!off || !weights || !plan || C == 0 || C > R2O_MAX_CHANNELS || align == 0)
        return R2O_INVALID;
    if ((mask_before & ~mask_after) != 0) return R2O_INVALID; /* a recovery is not a rollback */
    int rc = R2O_OK;
    for (uint32_t f = 0; f < C; ++f) {
        uint64_t *row = plan + (uint64_t)f * (C + 1);
        for (uint32_t c = 0; c <= C; ++c) row[c] = 0;
        int newly = ((mask_after >> f) & 1u) && !((mask_before >> f) & 1u);
        uint64_t len = off[f + 1] - off[f];
        if (!newly || len == 0) continue;
        int r = r2o_partition(weights, mask_after, C, len, align, row);
        if (r != R2O_OK) rc = r;
    }
    return rc;
}

/* ------------------------------------------------------------------ */
/* One fused reduce-copy on one chunk (Sec. 2.1 kernels; Sec. 4.3      */
/* staging buffers)                                                    */
/* ------------------------------------------------------------------ */
/*
 * incoming = the concatenation of the peer's stage slices (slice c is packed
 * at offset 0 of channel buffer c and has length in_off[c+1]-in_off[c]).
 *   in_stage == NULL : nothing arrives; v = local          (copy-send)
 *   op == SUM        : v = incoming + local
 *   op == COPY       : v = incoming
 * If something arrived, local <- v.  If out_stage != NULL, v is cut by
 * out_off and slice c is written at offset 0 of out_stage[c].
 *   op == SUM_FORWARD: local <- incoming + local as for SUM, but what is
 *                      staged onward is `incoming` itself (the relay step of
 *                      the broadcast in Sec. 5.2, R2CCL-AllReduce stage 2).
 * cap = capacity in bytes of every stage buffer.
 */
int r2o_reduce_copy(void *local, uint64_t bytes, int dtype, int op,
                    const void *const *in_stage, const uint64_t *in_off,
                    void *const *out_stage, const uint64_t *out_off,
                    uint32_t C, uint64_t cap)
{
    size_t es = elem_size(dtype);
    if (!local || bytes % es != 0 || C == 0 || C > R2O_MAX_CHANNELS)
        return R2O_INVALID;
    if ((in_stage && !in_off) || (out_stage && !out_off)) return R2O_INVALID;
    if (bytes == 0) return R2O_OK;

    uint8_t *v = (uint8_t *)malloc(bytes);
    if (!v) return R2O_NOMEM;
    uint8_t *relay = NULL; /* the untouched incoming data, for SUM_FORWARD */
    if (op == R2O_OP_SUM_FORWARD) {
        if (!in_stage || !out_stage) { free(v); return R2O_INVALID; }
        relay = (uint8_t *)malloc(bytes);
        if (!relay) { free(v); return R2O_NOMEM; }
    }

    if (in_stage) {
        if (in_off[0] != 0 || in_off[C] != bytes) { free(v); free(relay); return R2O_INVALID; }
        for (uint32_t c = 0; c < C; ++c) {
            if (in_off[c + 1] < in_off[c]) { free(v); free(relay); return R2O_INVALID; }
            uint64_t len = in_off[c + 1] - in_off[c];
            if (len > cap) { free(v); free(relay); return R2O_CAPACITY; }
            if (len) memcpy(v + in_off[c], in_stage[c], len);
        }
        if (relay) memcpy(relay, v, bytes);
        if (op == R2O_OP_SUM || op == R2O_OP_SUM_FORWARD) {
            int64_t n = (int64_t)(bytes / es);
            if (dtype == R2O_F32) {
                float *inc = (float *)v;
                const float *loc = (const float *)local;
#pragma omp parallel for schedule(static)
                for (int64_t i = 0; i < n; ++i) inc[i] = inc[i] + loc[i];
            } else {
                uint16_t *inc = (uint16_t *)v;
                const uint16_t *loc = (const uint16_t *)local;
#pragma omp parallel for schedule(static)
                for (int64_t i = 0; i < n; ++i)
                    inc[i] = r2o_f32_to_bf16(r2o_bf16_to_f32(inc[i]) +
                                             r2o_bf16_to_f32(loc[i]));
            }
        }
        memcpy(local, v, bytes);
    } else {
        memcpy(v, local, bytes);
    }

    if (out_stage) {
        if (out_off[0] != 0 || out_off[C] != bytes) { free(v); free(relay); return R2O_INVALID; }
        for (uint32_t c = 0; c < C; ++c) {
            if (out_off[c + 1] < out_off[c]) { free(v); free(relay); return R2O_INVALID; }
            uint64_t len = out_off[c + 1] - out_off[c];
            if (len > cap) { free(v); free(relay); return R2O_CAPACITY; }
            if (len) memcpy(out_stage[c], (relay ? relay : v) + out_off[c], len);
        }
    }
    free(v);
    free(relay);
    return R2O_OK;
}

/* ------------------------------------------------------------------ */
/* Ring schedule helpers (Sec. 5.2: reduce-scatter, then all-gather)   */
/* ------------------------------------------------------------------ */

/* fused steps per slab */
uint32_t r2o_num_steps(uint32_t R, int phases)
{
    return phases == (R2O_PHASE_RS | R2O_PHASE_AG) ? 2 * R - 1 : R;
}

/* transmissions (stage writes) per rank per slab */
uint32_t r2o_num_transmissions(uint32_t R, int phases)
{
    return r2o_num_steps(R, phases) - 1;
}

static const r2o_epoch *epoch_at(const r2o_epoch *ep, uint32_t n, uint64_t t)
{
    const r2o_epoch *cur = &ep[0];
    for (uint32_t i = 0; i < n; ++i)
        if (ep[i].t_start <= t) cur = &ep[i];
    return cur;
}

static int check_epochs(const r2o_epoch *ep, uint32_t n)
{
    if (!ep || n == 0 || ep[0].t_start != 0) return R2O_INVALID;
    for (uint32_t i = 0; i < n; ++i) {
        if (!ep[i].weights) return R2O_INVALID;
        if (i && ep[i].t_start <= ep[i - 1].t_start) return R2O_INVALID;
    }
    return R2O_OK;
}

/* ------------------------------------------------------------------ */
/* The ring, step by step, with explicit per-rank buffers and stages   */
/* ------------------------------------------------------------------ */
/*
 * bufs[r]: N elements, updated in place.  The buffer is S slabs; a slab is R
 * ring chunks of E = N/(S*R) elements.  Ranks form a ring: r receives from
 * r-1 and sends to r+1.
 *
 * Per slab, fused step j = 0 .. J-1 (J = 2R-1 for all-reduce, R for a single
 * phase).  Rank r works on ring chunk (r - j) mod R  [all-gather alone:
 * (r + 1 - j) mod R, i.e. it starts from the chunk a reduce-scatter leaves
 * fully reduced on r].
 *   j = 0             : copy-send (stage <- local)
 *   reduce-scatter j  : local <- incoming + local, staged onward
 *   all-gather j      : local <- incoming, staged onward
 *   j = J-1           : local is updated, nothing is staged
 * "incoming" is what rank r-1 staged at step j-1.  A stage write at step j of
 * slab l is transmission t = l*(J-1) + j; the channel state (weights, mask)
 * of the epoch in force at t decides the partition of that chunk, and the
 * reader uses the writer's table.  Every rank sees the same channel state
 * (they stand for one server's NIC pool).
 *
 * stage: [2 parities][R][S][C] buffers of cap bytes each; transmission at
 * step j uses parity j&1.  offsets_log (optional): [S*(J-1)][C+1].
 */
int r2o_ring_sim(void *const *bufs, uint32_t R, uint64_t N, int dtype,
                 uint32_t S, uint32_t C, uint32_t align,
                 const r2o_epoch *epochs, uint32_t n_epochs, int phases,
                 uint8_t *stage, uint64_t cap, uint64_t *offsets_log)
{
    if (!bufs || R < 2 || S == 0 || C == 0 || C > R2O_MAX_CHANNELS || !stage)
        return R2O_INVALID;
    if (phases != R2O_PHASE_RS && phases != R2O_PHASE_AG &&
        phases != (R2O_PHASE_RS | R2O_PHASE_AG))
        return R2O_INVALID;
    if (N % ((uint64_t)S * R) != 0) return R2O_INVALID;
    int rc = check_epochs(epochs, n_epochs);
    if (rc) return rc;

    size_t es = elem_size(dtype);
    uint64_t E = N / ((uint64_t)S * R);
    uint64_t chunk_bytes = E * es;
    if (align == 0 || align % es != 0) return R2O_INVALID;
    uint32_t J = r2o_num_steps(R, phases);
    uint32_t T_slab = J - 1;

    /* every state that will be used must leave a healthy channel */
    for (uint64_t t = 0; t < (uint64_t)S * T_slab; ++t) {
        const r2o_epoch *ep = epoch_at(epochs, n_epochs, t);
        uint64_t tmp[R2O_MAX_CHANNELS + 1];
        rc = r2o_partition(ep->weights, ep->fail_mask, C, chunk_bytes, align, tmp);
        if (rc) return rc;
        if (offsets_log) memcpy(offsets_log + t * (C + 1), tmp, (C + 1) * 8);
    }

#define STAGE_PTR(par, r, l, c) \
    (stage + ((((uint64_t)(par) * R + (r)) * S + (l)) * C + (c)) * cap)

    for (uint32_t l = 0; l < S; ++l) {
        for (uint32_t j = 0; j < J; ++j) {
            int has_in = j > 0;
            int has_out = j < J - 1;
            int op;
            if (phases == R2O_PHASE_AG) op = R2O_OP_COPY;
            else if (phases == R2O_PHASE_RS) op = R2O_OP_SUM;
            else op = (j <= R - 1) ? R2O_OP_SUM : R2O_OP_COPY;

            uint64_t in_off[R2O_MAX_CHANNELS + 1], out_off[R2O_MAX_CHANNELS + 1];
            if (has_in) {
                const r2o_epoch *ep = epoch_at(epochs, n_epochs, (uint64_t)l * T_slab + j - 1);
                r2o_partition(ep->weights, ep->fail_mask, C, chunk_bytes, align, in_off);
            }
            if (has_out) {
                const r2o_epoch *ep = epoch_at(epochs, n_epochs, (uint64_t)l * T_slab + j);
                r2o_partition(ep->weights, ep->fail_mask, C, chunk_bytes, align, out_off);
            }
            for (uint32_t r = 0; r < R; ++r) {
                uint32_t start = (phases == R2O_PHASE_AG) ? r + 1 : r;
                uint32_t c = (start + 2 * R - j) % R; /* j <= 2R-2 */
                uint8_t *local = (uint8_t *)bufs[r] + ((uint64_t)l * R + c) * chunk_bytes;
                uint32_t peer = (r + R - 1) % R;
                const void *inp[R2O_MAX_CHANNELS];
                void *outp[R2O_MAX_CHANNELS];
                for (uint32_t k = 0; k < C; ++k) {
                    inp[k] = has_in ? STAGE_PTR((j - 1) & 1, peer, l, k) : NULL;
                    outp[k] = STAGE_PTR(j & 1, r, l, k);
                }
                rc = r2o_reduce_copy(local, chunk_bytes, dtype, op,
                                     has_in ? inp : NULL, in_off,
                                     has_out ? outp : NULL, out_off, C, cap);
                if (rc) return rc;
            }
        }
    }
#undef STAGE_PTR
    return R2O_OK;
}

/* ------------------------------------------------------------------ */
/* The result by its plain definition (no ring, no stages)             */
/* ------------------------------------------------------------------ */
/*
 * in[r] are the R original rank buffers, out[r] receives what rank r must
 * hold afterwards.  For ring chunk c (of any slab), element i:
 *   all-reduce : every rank holds  fold_{k=0..R-1} x_{(c+k) mod R}[i]
 *   reduce-scatter only: rank r holds the partial fold over
 *                k = 0 .. (r - c) mod R   (rank c keeps x_c; rank c-1 has all)
 *   all-gather only: every rank holds what rank (c-1) mod R had at chunk c
 * fold = left-to-right sum starting from x_c, rounded to the buffer type
 * after every addition.
 */
int r2o_expected(const void *const *in, uint32_t R, uint64_t N, int dtype,
                 uint32_t S, int phases, void *const *out)
{
    if (!in || !out || R < 2 || S == 0) return R2O_INVALID;
    if (phases != R2O_PHASE_RS && phases != R2O_PHASE_AG &&
        phases != (R2O_PHASE_RS | R2O_PHASE_AG))
        return R2O_INVALID;
    if (N % ((uint64_t)S * R) != 0) return R2O_INVALID;
    uint64_t E = N / ((uint64_t)S * R);

    for (uint32_t r = 0; r < R; ++r) {
        for (uint32_t l = 0; l < S; ++l) {
            for (uint32_t c = 0; c < R; ++c) {
                uint64_t base = ((uint64_t)l * R + c) * E;
                if (phases == R2O_PHASE_AG) {
                    uint32_t owner = (c + R - 1) % R;
                    size_t es = elem_size(dtype);
                    memcpy((uint8_t *)out[r] + base * es,
                           (const uint8_t *)in[owner] + base * es, E * es);
                    continue;
                }
                uint32_t terms = (phases == R2O_PHASE_RS) ? ((r + R - c) % R) + 1 : R;
                if (dtype == R2O_F32) {
                    float *o = (float *)out[r] + base;
#pragma omp parallel for schedule(static)
                    for (int64_t i = 0; i < (int64_t)E; ++i) {
                        float acc = ((const float *)in[c])[base + i];
                        for (uint32_t k = 1; k < terms; ++k)
                            acc = acc + ((const float *)in[(c + k) % R])[base + i];
                        o[i] = acc;
                    }
                } else {
                    uint16_t *o = (uint16_t *)out[r] + base;
#pragma omp parallel for schedule(static)
                    for (int64_t i = 0; i < (int64_t)E; ++i) {
                        uint16_t acc = ((const uint16_t *)in[c])[base + i];
                        for (uint32_t k = 1; k < terms; ++k) {
                            uint16_t x = ((const uint16_t *)in[(c + k) % R])[base + i];
                            acc = r2o_f32_to_bf16(r2o_bf16_to_f32(acc) + r2o_bf16_to_f32(x));
                        }
                        o[i] = acc;
                    }
                }
            }
        }
    }
    return R2O_OK;
}

/* number of OpenMP threads the loops above will use (1 if built without) */
#ifdef _OPENMP
#include <omp.h>
int r2o_threads(void) { return omp_get_max_threads(); }
void r2o_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int r2o_threads(void) { return 1; }
void r2o_set_threads(int n) { (void)n; }
#endif
