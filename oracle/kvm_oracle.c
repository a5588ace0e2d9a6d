/*
 * kvm_oracle.c — plain CPU reference for the KV-cache management pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * checked against; nothing in the product path may call it.  It shares no code
 * with the GPU library: formats (bf16/fp16 decoding, the K unit layout, the
 * state bits) are restated here from their definitions.
 *
 * Everything is written as the defining formula, in double precision, with no
 * blocking or reordering beyond "for each row, for each query, for each
 * token".  The only parallelism is an OpenMP loop over rows in the scorer.
 *
 * What each function follows:
 *   kvm_ref_size            section 3.1, Eq. 3 (per-layer bytes) and Eq. 4 / the
 *                           max-batch formula that follows it; head weights of section 3.4
 *   kvm_ref_score_step      Eq. 1 (softmax(q k^T / sqrt(d))) summed per token block;
 *                           group maximum of section 3.4
 *   kvm_ref_ema_update      section 3.4 (EMA importance, head weights) times the
 *                           posterior mean of Eq. 5
 *   kvm_ref_ema_update_ex   the same with the two refinements section 3.4 names: the
 *                           importance decays with positional distance, and per-head
 *                           multipliers chosen by the transition type (sections 3.4, 3.7)
 *   kvm_ref_beta_update     section 3.3, Eq. 5 and the update rule after it
 *   kvm_ref_beta_blend_update
 *                           section 3.3, last two paragraphs: confidence that saturates
 *                           with the number of observations, empirical frequency over a
 *                           sliding window, blend weighted by the confidence
 *   kvm_ref_select_victims  section 3.4 (the smallest head-weighted importance goes first),
 *                           as a full sort
 *   kvm_ref_span_update     section 3.5: per-layer prefetch window from the observed
 *                           attention span
 *   kvm_ref_prefetch_keys   section 3.5: candidates inside the positional window around the
 *                           decode position, ranked with the reuse estimate of section 3.3
 *   kvm_ref_pack / unpack   section 3.2 (tier 0 <-> tier 1 moves), as memcpy
 *   kvm_ref_exchange        the same as an in-place trade with a slot-addressed host tier
 *   kvm_ref_sha256, kvm_ref_hash_units, kvm_ref_dedup_insert / release
 *                           section 3.6: content addressing by SHA-256 (FIPS 180-4), store with
 *                           reference counts
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (paper tables, closed forms, library routines, brute force); none is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK      0
#define REF_EINVAL (-1)

enum { ST_RESIDENT = 1, ST_ON_HOST = 2, ST_PROTECTED = 4, ST_SCORED = 8, ST_SHARED = 16 };

/* ---------------------------------------------------------------- formats */

/* bfloat16: the upper 16 bits of an IEEE binary32. */
static double bf16_to_double(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double fp16_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);                 /* subnormal: frac * 2^-10 * 2^-14 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

static double elem_to_double(const uint16_t* p, int dtype) {
    return dtype == 0 ? bf16_to_double(*p) : fp16_to_double(*p);
}

/* Exposed so that the decoders can be checked exhaustively against a library. */
double kvm_ref_decode(uint16_t bits, int dtype) { return elem_to_double(&bits, dtype); }

/* Index of (token t, channel c) inside a K unit laid out as
 * [dim/8][block_tokens][8]. */
static size_t k_elem_index(int t, int c, int block_tokens) {
    return (size_t)(c / 8) * (size_t)block_tokens * 8 + (size_t)t * 8 + (size_t)(c % 8);
}

/* ----------------------------------------------------------------- sizing */

typedef struct {
    int32_t n_layers, n_q_heads, n_kv_heads, head_dim, d_latent, d_rope;
    int32_t bits_per_elem, block_tokens, head_divisor;
} ref_model_t;

typedef struct {
    int32_t  arch, group_size;
    uint64_t bytes_per_token_layer, bytes_per_token, bytes_per_seq, max_batch;
    uint32_t units_per_block, unit_k_bytes, unit_v_bytes;
    uint32_t head_weight;
    uint64_t pool_units;
} ref_sizing_t;

int kvm_ref_size(const ref_model_t* m, uint64_t n_max, uint64_t mem_target, ref_sizing_t* o) {
    if (!m || !o) return REF_EINVAL;
    if (m->n_layers <= 0 || m->block_tokens <= 0 || m->head_divisor <= 0) return REF_EINVAL;
    if (m->bits_per_elem != 4 && m->bits_per_elem != 8 && m->bits_per_elem != 16 &&
        m->bits_per_elem != 32)
        return REF_EINVAL;
    memset(o, 0, sizeof *o);
    uint64_t bits_tok_layer;      /* B(1) in bits */
    uint64_t k_channels, v_channels, heads;
    if (m->d_latent > 0) {                                   /* MLA */
        if (m->d_rope < 0 || m->n_q_heads <= 0) return REF_EINVAL;
        o->arch = 3;
        o->group_size = m->n_q_heads;
        k_channels = (uint64_t)m->d_latent + (uint64_t)m->d_rope;
        v_channels = 0;
        heads = 1;
        bits_tok_layer = k_channels * (uint64_t)m->bits_per_elem;
    } else {
        if (m->n_q_heads <= 0 || m->n_kv_heads <= 0 || m->head_dim <= 0) return REF_EINVAL;
        if (m->n_q_heads % m->n_kv_heads) return REF_EINVAL;
        if (m->n_kv_heads % m->head_divisor) return REF_EINVAL;
        if (m->n_q_heads == m->n_kv_heads) o->arch = 0;      /* MHA */
        else if (m->n_kv_heads == 1)       o->arch = 2;      /* MQA */
        else                               o->arch = 1;      /* GQA */
        o->group_size = m->n_q_heads / m->n_kv_heads;
        heads = (uint64_t)(m->n_kv_heads / m->head_divisor);
        k_channels = v_channels = (uint64_t)m->head_dim;
        bits_tok_layer = 2 * heads * (uint64_t)m->head_dim * (uint64_t)m->bits_per_elem;
    }
    if (bits_tok_layer % 8) return REF_EINVAL;
    uint64_t unit_k_bits = (uint64_t)m->block_tokens * k_channels * (uint64_t)m->bits_per_elem;
    uint64_t unit_v_bits = (uint64_t)m->block_tokens * v_channels * (uint64_t)m->bits_per_elem;
    if (unit_k_bits % 8 || unit_v_bits % 8) return REF_EINVAL;
    o->bytes_per_token_layer = bits_tok_layer / 8;
    o->bytes_per_token = o->bytes_per_token_layer * (uint64_t)m->n_layers;
    o->bytes_per_seq = o->bytes_per_token * n_max;
    o->max_batch = o->bytes_per_seq ? mem_target / o->bytes_per_seq : 0;
    o->units_per_block = (uint32_t)((uint64_t)m->n_layers * heads);
    o->unit_k_bytes = (uint32_t)(unit_k_bits / 8);
    o->unit_v_bytes = (uint32_t)(unit_v_bits / 8);
    o->pool_units = mem_target / ((uint64_t)o->unit_k_bytes + o->unit_v_bytes);
    /* Head weights, section 3.4: uniform for MHA, proportional to the group size for grouped
     * heads (GQA, and MQA as the group of all query heads); the MLA matrix has a single head. */
    switch (o->arch) {
        case 0: o->head_weight = 1; break;
        case 1: o->head_weight = (uint32_t)(m->n_q_heads / m->n_kv_heads); break;
        case 2: o->head_weight = (uint32_t)m->n_q_heads; break;
        default: o->head_weight = 1; break;
    }
    return REF_OK;
}

/* ---------------------------------------------------------------- scoring */

/* mass_q (optional, may be NULL): per-query block masses in double,
 * mass_q[uid * g + j]; written for the same units as mass. */
int kvm_ref_score_step(const uint16_t* k_pool, uint64_t n_slots, int dim, int dtype, int block_tokens,
                       int n_rows, int g, int64_t n_uids,
                       const int32_t* row_ntok, const int64_t* row_off, const int64_t* row_q_off,
                       const uint8_t* row_active, const int32_t* slot_tbl,
                       const uint16_t* q, double softmax_scale, int agg,
                       float* mass, double* mass_q) {
    if (!k_pool || !row_ntok || !row_off || !row_q_off || !slot_tbl || !q || !mass) return REF_EINVAL;
    if (dim <= 0 || dim % 8 || g <= 0 || block_tokens <= 0 || (agg != 0 && agg != 1)) return REF_EINVAL;
    const size_t unit_elems = (size_t)block_tokens * (size_t)dim;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(|:bad)
    for (int r = 0; r < n_rows; ++r) {
        if (row_active && !row_active[r]) continue;
        const int n = row_ntok[r];
        if (n <= 0) continue;
        const int nb = (n + block_tokens - 1) / block_tokens;
        if (row_off[r] < 0 || row_off[r] + nb > n_uids) { bad = 1; continue; }
        double* z = (double*)malloc(sizeof(double) * (size_t)n);
        double* mb = (double*)malloc(sizeof(double) * (size_t)nb * (size_t)g);
        for (int j = 0; j < g; ++j) {
            const uint16_t* qj = q + row_q_off[r] + (int64_t)j * dim;
            /* logits of the resident tokens */
            double zmax = -INFINITY;
            for (int t = 0; t < n; ++t) {
                const int b = t / block_tokens;
                const int32_t slot = slot_tbl[row_off[r] + b];
                if (slot < 0) continue;
                if ((uint64_t)slot >= n_slots) { bad = 1; continue; }
                const uint16_t* unit = k_pool + (size_t)slot * unit_elems;
                double dot = 0.0;
                for (int c = 0; c < dim; ++c)
                    dot += elem_to_double(qj + c, dtype) *
                           elem_to_double(unit + k_elem_index(t % block_tokens, c, block_tokens), dtype);
                z[t] = softmax_scale * dot;
                if (z[t] > zmax) zmax = z[t];
            }
            /* softmax normaliser over the resident tokens */
            double Z = 0.0;
            for (int t = 0; t < n; ++t) {
                const int32_t slot = slot_tbl[row_off[r] + t / block_tokens];
                if (slot < 0 || (uint64_t)slot >= n_slots) continue;
                Z += exp(z[t] - zmax);
            }
            /* mass per block */
            for (int b = 0; b < nb; ++b) {
                double s = 0.0;
                const int32_t slot = slot_tbl[row_off[r] + b];
                if (slot >= 0 && (uint64_t)slot < n_slots) {
                    for (int t = b * block_tokens; t < n && t < (b + 1) * block_tokens; ++t)
                        s += exp(z[t] - zmax);
                    s /= Z;
                }
                mb[(size_t)b * g + j] = s;
            }
        }
        for (int b = 0; b < nb; ++b) {
            const int64_t uid = row_off[r] + b;
            const int32_t slot = slot_tbl[uid];
            if (slot < 0 || (uint64_t)slot >= n_slots) continue;
            double a = (agg == 0) ? -INFINITY : 0.0;
            for (int j = 0; j < g; ++j) {
                const double v = mb[(size_t)b * g + j];
                if (agg == 0) { if (v > a) a = v; } else a += v;
                if (mass_q) mass_q[uid * g + j] = v;
            }
            if (agg == 1) a /= (double)g;
            mass[uid] = (float)a;
        }
        free(z);
        free(mb);
    }
    return bad ? REF_EINVAL : REF_OK;
}

/* ------------------------------------------------------------------- beta */

int kvm_ref_beta_update(const uint8_t* ev_pair, const uint8_t* ev_outcome, int64_t n_events,
                        uint32_t* hits, uint32_t* misses, double alpha0, double beta0,
                        float* p_hat, uint32_t* n_bad) {
    if (n_events < 0 || !hits || !misses || !p_hat) return REF_EINVAL;
    if (n_events > 0 && (!ev_pair || !ev_outcome)) return REF_EINVAL;
    if (!(alpha0 > 0.0) || !(beta0 > 0.0)) return REF_EINVAL;
    for (int64_t e = 0; e < n_events; ++e) {
        if (ev_pair[e] >= 16 || ev_outcome[e] > 1) { if (n_bad) ++*n_bad; continue; }
        if (ev_outcome[e]) hits[ev_pair[e]] += 1; else misses[ev_pair[e]] += 1;
    }
    for (int i = 0; i < 16; ++i) {
        const double a = alpha0 + (double)hits[i];
        const double b = beta0 + (double)misses[i];
        p_hat[i] = (float)(a / (a + b));
    }
    return REF_OK;
}

/* Section 3.3, after Eq. 5: the estimate used for decisions blends the posterior
 * mean with the hit frequency among the last `window` observations of the pair;
 * the weight of the posterior is a confidence that grows towards 1 with the
 * number of observations.  The paper gives neither formula; the reading taken:
 *   n      = hits + misses of the pair (all observations so far)
 *   conf   = n / (n + kappa)                  (0 when n + kappa == 0)
 *   f      = (1-outcomes among the last min(n_pushed, window) observations) / their number,
 *            or the posterior mean when the window holds nothing yet
 *   blend  = conf * posterior + (1 - conf) * f
 * The window is a ring per pair: win[pair * window + i] holds 0 or 1, any other value
 * marks a place never written; win_head[pair] is the next place to write.
 * Events are taken in array order; malformed events are skipped as in
 * kvm_ref_beta_update and touch neither the counters nor the window. */
int kvm_ref_beta_blend_update(const uint8_t* ev_pair, const uint8_t* ev_outcome, int64_t n_events,
                              uint32_t* hits, uint32_t* misses, double alpha0, double beta0,
                              uint8_t* win, uint32_t* win_head, int window, double kappa,
                              float* p_hat, float* conf, float* p_blend, uint32_t* n_bad) {
    if (n_events < 0 || !hits || !misses || !p_hat || !conf || !p_blend || !win || !win_head) return REF_EINVAL;
    if (n_events > 0 && (!ev_pair || !ev_outcome)) return REF_EINVAL;
    if (!(alpha0 > 0.0) || !(beta0 > 0.0) || window <= 0 || !(kappa >= 0.0)) return REF_EINVAL;
    for (int i = 0; i < 16; ++i)
        if (win_head[i] >= (uint32_t)window) return REF_EINVAL;
    for (int64_t e = 0; e < n_events; ++e) {
        const int p = ev_pair[e], o = ev_outcome[e];
        if (p >= 16 || o > 1) { if (n_bad) ++*n_bad; continue; }
        if (o) hits[p] += 1; else misses[p] += 1;
        win[(size_t)p * window + win_head[p]] = (uint8_t)o;
        win_head[p] = (win_head[p] + 1) % (uint32_t)window;
    }
    for (int i = 0; i < 16; ++i) {
        const double a = alpha0 + (double)hits[i];
        const double b = beta0 + (double)misses[i];
        const double post = a / (a + b);
        const double n = (double)hits[i] + (double)misses[i];
        const double c = (n + kappa > 0.0) ? n / (n + kappa) : 0.0;
        long ones = 0, seen = 0;
        for (int j = 0; j < window; ++j) {
            const uint8_t v = win[(size_t)i * window + j];
            if (v <= 1) { ++seen; ones += v; }
        }
        const double f = seen ? (double)ones / (double)seen : post;
        p_hat[i] = (float)post;
        conf[i] = (float)c;
        p_blend[i] = (float)(c * post + (1.0 - c) * f);
    }
    return REF_OK;
}

/* -------------------------------------------------------- EMA + priority */

int kvm_ref_ema_update(int n_rows, int block_tokens, int64_t n_uids,
                       const int32_t* row_ntok, const int64_t* row_off, const uint8_t* row_active,
                       const float* mass, double decay, const float* row_weight,
                       const uint8_t* pair, const float* p_hat,
                       uint8_t* state, float* S, float* prio) {
    if (!row_ntok || !row_off || !mass || !row_weight || !pair || !p_hat || !state || !S || !prio)
        return REF_EINVAL;
    if (!(decay >= 0.0 && decay <= 1.0) || block_tokens <= 0) return REF_EINVAL;
    for (int r = 0; r < n_rows; ++r) {
        const int n = row_ntok[r];
        const int nb = n > 0 ? (n + block_tokens - 1) / block_tokens : 0;
        if (nb && (row_off[r] < 0 || row_off[r] + nb > n_uids)) return REF_EINVAL;
        const int active = row_active ? row_active[r] != 0 : 1;
        for (int b = 0; b < nb; ++b) {
            const int64_t uid = row_off[r] + b;
            if (active && (state[uid] & ST_RESIDENT)) {
                const double x = (double)mass[uid];
                if (!(state[uid] & ST_SCORED)) {
                    S[uid] = (float)x;
                    state[uid] |= ST_SCORED;
                } else {
                    S[uid] = (float)(decay * (double)S[uid] + (1.0 - decay) * x);
                }
            }
            if (state[uid] & ST_SCORED)
                prio[uid] = (float)((double)row_weight[r] * (double)S[uid] * (double)p_hat[pair[uid] & 15]);
            else
                prio[uid] = INFINITY;
        }
    }
    return REF_OK;
}

/* Section 3.4 says that the EMA also decays with positional distance and that per-head
 * multipliers are applied during task transitions (section 3.7, item 2) without giving
 * either formula.  The reading taken:
 *   distance d of block b in a row of nb blocks = nb - 1 - b (blocks behind the decode
 *   position, which lies in the row's last block);
 *   the observation fed to the EMA is x = pos_decay^d * mass            (pos_decay in (0, 1]);
 *   multiplier of row r = head_mult[t * n_heads + row_head[r]] where t = seq_transition[row_seq[r]]
 *   is the transition type (0..3) its sequence is going through, or 1 when t > 3 (no
 *   transition) or when head_mult is NULL;
 *   prio = row_weight * multiplier * S * p_hat[pair].
 * With pos_decay = 1 and no multipliers this is kvm_ref_ema_update. */
int kvm_ref_ema_update_ex(int n_rows, int block_tokens, int64_t n_uids,
                          const int32_t* row_ntok, const int64_t* row_off, const uint8_t* row_active,
                          const float* mass, double decay, double pos_decay, const float* row_weight,
                          const int32_t* row_seq, const int32_t* row_head, const uint8_t* seq_transition,
                          int n_seq, const float* head_mult, int n_heads,
                          const uint8_t* pair, const float* p_hat,
                          uint8_t* state, float* S, float* prio) {
    if (!row_ntok || !row_off || !mass || !row_weight || !pair || !p_hat || !state || !S || !prio)
        return REF_EINVAL;
    if (!(decay >= 0.0 && decay <= 1.0) || !(pos_decay > 0.0 && pos_decay <= 1.0) || block_tokens <= 0)
        return REF_EINVAL;
    if (head_mult && (!row_seq || !row_head || !seq_transition || n_seq <= 0 || n_heads <= 0)) return REF_EINVAL;
    for (int r = 0; r < n_rows; ++r) {
        const int n = row_ntok[r];
        const int nb = n > 0 ? (n + block_tokens - 1) / block_tokens : 0;
        if (nb && (row_off[r] < 0 || row_off[r] + nb > n_uids)) return REF_EINVAL;
        const int active = row_active ? row_active[r] != 0 : 1;
        double mult = 1.0;
        if (head_mult) {
            if (row_seq[r] < 0 || row_seq[r] >= n_seq || row_head[r] < 0 || row_head[r] >= n_heads) return REF_EINVAL;
            const int t = seq_transition[row_seq[r]];
            if (t <= 3) mult = (double)head_mult[(size_t)t * n_heads + row_head[r]];
        }
        for (int b = 0; b < nb; ++b) {
            const int64_t uid = row_off[r] + b;
            if (active && (state[uid] & ST_RESIDENT)) {
                const double x = pow(pos_decay, (double)(nb - 1 - b)) * (double)mass[uid];
                if (!(state[uid] & ST_SCORED)) {
                    S[uid] = (float)x;
                    state[uid] |= ST_SCORED;
                } else {
                    S[uid] = (float)(decay * (double)S[uid] + (1.0 - decay) * x);
                }
            }
            if (state[uid] & ST_SCORED)
                prio[uid] = (float)((double)row_weight[r] * mult * (double)S[uid] * (double)p_hat[pair[uid] & 15]);
            else
                prio[uid] = INFINITY;
        }
    }
    return REF_OK;
}

/* ----------------------------------------------------------------- select */

typedef struct { float prio; int64_t uid; } cand_t;

static int cand_cmp(const void* a, const void* b) {
    const cand_t* x = (const cand_t*)a;
    const cand_t* y = (const cand_t*)b;
    if (x->prio < y->prio) return -1;
    if (x->prio > y->prio) return 1;
    return (x->uid > y->uid) - (x->uid < y->uid);
}

static int i64_cmp(const void* a, const void* b) {
    const int64_t x = *(const int64_t*)a, y = *(const int64_t*)b;
    return (x > y) - (x < y);
}

int kvm_ref_select_victims(const float* prio, const uint8_t* state, int64_t n_uids,
                           int64_t k_or_neg1, int64_t budget_units,
                           int64_t* victims, int64_t victims_cap, int64_t* n_victims) {
    if (!prio || !state || !victims || !n_victims || n_uids < 0 || k_or_neg1 < -1 ||
        budget_units < 0 || victims_cap < 0)
        return REF_EINVAL;
    cand_t* c = (cand_t*)malloc(sizeof(cand_t) * (size_t)(n_uids ? n_uids : 1));
    int64_t n_el = 0, n_res = 0;
    for (int64_t u = 0; u < n_uids; ++u) {
        if (state[u] & ST_RESIDENT) ++n_res;
        if ((state[u] & ST_RESIDENT) && !(state[u] & (ST_PROTECTED | ST_SHARED)) && (state[u] & ST_SCORED)) {
            float p = prio[u];
            if (isnan(p)) p = INFINITY;      /* NaN ranks last */
            c[n_el].prio = p;                /* -0 == +0 under float comparison */
            c[n_el].uid = u;
            ++n_el;
        }
    }
    int64_t k = k_or_neg1 >= 0 ? k_or_neg1 : (n_res > budget_units ? n_res - budget_units : 0);
    if (k > n_el) k = n_el;
    if (k > victims_cap) k = victims_cap;
    qsort(c, (size_t)n_el, sizeof(cand_t), cand_cmp);
    for (int64_t i = 0; i < k; ++i) victims[i] = c[i].uid;
    qsort(victims, (size_t)k, sizeof(int64_t), i64_cmp);
    *n_victims = k;
    free(c);
    return REF_OK;
}

/* ---------------------------------------------- position-aware prefetching */

/* Section 3.5: the prefetch window follows the attention pattern a layer is observed to have,
 * narrow for layers that attend locally, wide for layers that attend globally.  No
 * formula is given.  The reading taken: the attention span of a row is the smallest
 * number s >= 1 of trailing blocks (counted back from the row's last block, blocks not
 * in HBM counting as distance but contributing nothing) whose masses hold at least
 * theta = theta_num / theta_den of the row's total mass this step; a layer's window is
 * block_tokens * ceil(mean span of its rows), clamped to [w_min, w_max] tokens.
 * So that the integer decision is the same on every implementation, masses enter as
 * fixed point: Q(m) = floor(m * 2^32) for m in (0, 1], 0 for anything else (NaN
 * included), clamped at 1 (a unit's mass is a softmax share, so it cannot exceed 1; the
 * clamp keeps the 64-bit sums exact for any row length); the comparison with theta is
 * made on exact 128-bit products.
 * span_sum / span_cnt accumulate over calls (the caller resets or ages them);
 * layer_window[l] is rewritten for layers with span_cnt > 0 and left alone otherwise. */
int kvm_ref_span_update(int n_rows, int block_tokens, int64_t n_uids,
                        const int32_t* row_ntok, const int64_t* row_off, const uint8_t* row_active,
                        const int32_t* row_layer, int n_layers, const float* mass, const uint8_t* state,
                        uint32_t theta_num, uint32_t theta_den, uint64_t* span_sum, uint32_t* span_cnt,
                        int32_t w_min, int32_t w_max, int32_t* layer_window) {
    if (!row_ntok || !row_off || !row_layer || !mass || !state || !span_sum || !span_cnt || !layer_window)
        return REF_EINVAL;
    if (block_tokens <= 0 || n_layers <= 0 || theta_den == 0 || theta_num > theta_den || theta_den > 65536 ||
        w_min < 0 || w_max < w_min)
        return REF_EINVAL;
    for (int r = 0; r < n_rows; ++r) {
        const int n = row_ntok[r];
        const int nb = n > 0 ? (n + block_tokens - 1) / block_tokens : 0;
        if (nb && (row_off[r] < 0 || row_off[r] + nb > n_uids)) return REF_EINVAL;
        if (row_layer[r] < 0 || row_layer[r] >= n_layers) return REF_EINVAL;
        if (row_active && !row_active[r]) continue;
        uint64_t total = 0;
        for (int b = 0; b < nb; ++b) {
            const int64_t uid = row_off[r] + b;
            const float m = mass[uid];
            uint64_t qv = 0;
            if ((state[uid] & ST_RESIDENT) && m > 0.0f) qv = (uint64_t)((double)(m < 1.0f ? m : 1.0f) * 4294967296.0);
            total += qv;
        }
        if (total == 0) continue;
        uint64_t acc = 0;
        int span = nb;
        for (int s = 1; s <= nb; ++s) {
            const int64_t uid = row_off[r] + (nb - s);
            const float m = mass[uid];
            if ((state[uid] & ST_RESIDENT) && m > 0.0f) acc += (uint64_t)((double)(m < 1.0f ? m : 1.0f) * 4294967296.0);
            if ((unsigned __int128)acc * theta_den >= (unsigned __int128)theta_num * total) { span = s; break; }
        }
        span_sum[row_layer[r]] += (uint64_t)span;
        span_cnt[row_layer[r]] += 1;
    }
    for (int l = 0; l < n_layers; ++l) {
        if (!span_cnt[l]) continue;
        const uint64_t mean_up = (span_sum[l] + span_cnt[l] - 1) / span_cnt[l];
        uint64_t w = mean_up * (uint64_t)block_tokens;
        if (w < (uint64_t)w_min) w = (uint64_t)w_min;
        if (w > (uint64_t)w_max) w = (uint64_t)w_max;
        layer_window[l] = (int32_t)w;
    }
    return REF_OK;
}

/* Section 3.5: while a request decodes at position n, the blocks most likely to be
 * needed next are those within a window w of n; they are promoted from the lower tier
 * ahead of use, together with the reuse estimate of section 3.3.  The text gives the
 * window once as [n - w, n] and once as [n, n + w]; positions after n hold no keys yet
 * during decoding, so the reading taken is [n - w, n].  For row r with decode position
 * n = row_pos[r] (tokens; negative = the row asks for nothing) and w = layer_window[row_layer[r]]:
 *   block b is a candidate iff it is on the host and not in HBM and its tokens
 *   [B b, B b + B - 1] meet [n - w, n]  (B = block_tokens);
 *   key = 1 - p_est[pair] * pos_decay^(floor(n / B) - b)      (lower = fetch sooner);
 *   cand = RESIDENT | SCORED for candidates (the pattern kvm_ref_select_victims admits), 0
 *   otherwise, and key = +inf for non-candidates.
 * The list itself is then the k lowest (key, uid) by kvm_ref_select_victims(key, cand, k). */
int kvm_ref_prefetch_keys(int n_rows, int block_tokens, int64_t n_uids,
                          const int32_t* row_ntok, const int64_t* row_off, const int32_t* row_layer,
                          const int32_t* row_pos, const int32_t* layer_window, int n_layers,
                          const uint8_t* state, const uint8_t* pair, const float* p_est, double pos_decay,
                          float* key, uint8_t* cand) {
    if (!row_ntok || !row_off || !row_layer || !row_pos || !layer_window || !state || !pair || !p_est || !key || !cand)
        return REF_EINVAL;
    if (block_tokens <= 0 || n_layers <= 0 || !(pos_decay > 0.0 && pos_decay <= 1.0)) return REF_EINVAL;
    for (int r = 0; r < n_rows; ++r) {
        const int nt = row_ntok[r];
        const int nb = nt > 0 ? (nt + block_tokens - 1) / block_tokens : 0;
        if (nb && (row_off[r] < 0 || row_off[r] + nb > n_uids)) return REF_EINVAL;
        if (row_layer[r] < 0 || row_layer[r] >= n_layers) return REF_EINVAL;
        const int64_t n = row_pos[r];
        const int64_t w = layer_window[row_layer[r]];
        for (int b = 0; b < nb; ++b) {
            const int64_t uid = row_off[r] + b;
            const int64_t first = (int64_t)b * block_tokens, last = first + block_tokens - 1;
            const int on_host = (state[uid] & ST_ON_HOST) && !(state[uid] & ST_RESIDENT);
            if (n >= 0 && w >= 0 && on_host && last >= n - w && first <= n) {
                const double dist = (double)(n / block_tokens - b);
                key[uid] = (float)(1.0 - (double)p_est[pair[uid] & 15] * pow(pos_decay, dist));
                cand[uid] = ST_RESIDENT | ST_SCORED;
            } else {
                key[uid] = INFINITY;
                cand[uid] = 0;
            }
        }
    }
    return REF_OK;
}

/* ---------------------------------------------------------- pack / unpack */
/* A unit that shares its frame with others (ST_SHARED, kvm_ref_dedup_share) is refused by pack
 * and as the outgoing half of an exchange, like a unit that is not in HBM: its frame must not
 * be handed out while others read it.  The victim selection never names such a unit. */

int kvm_ref_pack(const uint8_t* k_pool, const uint8_t* v_pool, uint64_t n_slots,
                 uint32_t unit_k_bytes, uint32_t unit_v_bytes,
                 int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                 const int64_t* uids, int64_t n, const int32_t* host_slots,
                 int32_t* freed_slots, uint8_t* staging, uint32_t* n_bad) {
    if (!k_pool || (unit_v_bytes && !v_pool) || !slot_tbl || !state || n < 0) return REF_EINVAL;
    if (n > 0 && (!uids || !host_slots || !freed_slots || !staging)) return REF_EINVAL;
    const size_t rec = (size_t)unit_k_bytes + unit_v_bytes;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t uid = uids[i];
        int32_t slot = -1;
        if (uid >= 0 && uid < n_uids && (state[uid] & ST_RESIDENT) && !(state[uid] & ST_SHARED)) slot = slot_tbl[uid];
        if (slot < 0 || (uint64_t)slot >= n_slots) {
            freed_slots[i] = -1;
            if (n_bad) ++*n_bad;
            continue;
        }
        memcpy(staging + (size_t)i * rec, k_pool + (size_t)slot * unit_k_bytes, unit_k_bytes);
        if (unit_v_bytes)
            memcpy(staging + (size_t)i * rec + unit_k_bytes, v_pool + (size_t)slot * unit_v_bytes,
                   unit_v_bytes);
        freed_slots[i] = slot;
        slot_tbl[uid] = -1 - host_slots[i];
        state[uid] = (uint8_t)((state[uid] & ~ST_RESIDENT) | ST_ON_HOST);
    }
    return REF_OK;
}

int kvm_ref_unpack(uint8_t* k_pool, uint8_t* v_pool, uint64_t n_slots,
                   uint32_t unit_k_bytes, uint32_t unit_v_bytes,
                   int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                   const int64_t* uids, int64_t n, const int32_t* dst_slots,
                   const uint8_t* staging, uint32_t* n_bad) {
    if (!k_pool || (unit_v_bytes && !v_pool) || !slot_tbl || !state || n < 0) return REF_EINVAL;
    if (n > 0 && (!uids || !dst_slots || !staging)) return REF_EINVAL;
    const size_t rec = (size_t)unit_k_bytes + unit_v_bytes;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t uid = uids[i];
        const int32_t slot = dst_slots[i];
        if (uid < 0 || uid >= n_uids || (state[uid] & ST_RESIDENT) || slot < 0 ||
            (uint64_t)slot >= n_slots) {
            if (n_bad) ++*n_bad;
            continue;
        }
        memcpy(k_pool + (size_t)slot * unit_k_bytes, staging + (size_t)i * rec, unit_k_bytes);
        if (unit_v_bytes)
            memcpy(v_pool + (size_t)slot * unit_v_bytes, staging + (size_t)i * rec + unit_k_bytes,
                   unit_v_bytes);
        slot_tbl[uid] = slot;
        state[uid] = (uint8_t)((state[uid] & ~ST_ON_HOST) | ST_RESIDENT);
    }
    return REF_OK;
}

/* The trade of section 3.2 (demote one unit, promote another) against a host tier that is
 * addressed by slot: the frame of out_uids[i] and the tier record of in_uids[i] swap
 * contents, the table entries and state bits follow.  Written with a temporary copy. */
int kvm_ref_exchange(uint8_t* k_pool, uint8_t* v_pool, uint64_t n_slots,
                     uint32_t unit_k_bytes, uint32_t unit_v_bytes,
                     int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                     const int64_t* out_uids, const int64_t* in_uids, int64_t n,
                     uint8_t* tier, uint64_t tier_slots, uint32_t* n_bad) {
    if (!k_pool || (unit_v_bytes && !v_pool) || !slot_tbl || !state || n < 0) return REF_EINVAL;
    if (n > 0 && (!out_uids || !in_uids || !tier)) return REF_EINVAL;
    const size_t rec = (size_t)unit_k_bytes + unit_v_bytes;
    uint8_t* tmp = (uint8_t*)malloc(rec ? rec : 1);
    if (!tmp) return REF_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t uo = out_uids[i], ui = in_uids[i];
        int ok = uo >= 0 && uo < n_uids && ui >= 0 && ui < n_uids && uo != ui;
        ok = ok && (state[uo] & ST_RESIDENT) && !(state[uo] & ST_SHARED) && slot_tbl[uo] >= 0 &&
             (uint64_t)slot_tbl[uo] < n_slots;
        ok = ok && (state[ui] & ST_ON_HOST) && !(state[ui] & ST_RESIDENT) && slot_tbl[ui] < 0 &&
             (uint64_t)(-1 - (int64_t)slot_tbl[ui]) < tier_slots;
        if (!ok) { if (n_bad) ++*n_bad; continue; }
        const int32_t frame = slot_tbl[uo];
        const int64_t host = -1 - (int64_t)slot_tbl[ui];
        uint8_t* r = tier + (size_t)host * rec;
        memcpy(tmp, r, rec);                                               /* record coming in  */
        memcpy(r, k_pool + (size_t)frame * unit_k_bytes, unit_k_bytes);    /* frame going out   */
        if (unit_v_bytes) memcpy(r + unit_k_bytes, v_pool + (size_t)frame * unit_v_bytes, unit_v_bytes);
        memcpy(k_pool + (size_t)frame * unit_k_bytes, tmp, unit_k_bytes);
        if (unit_v_bytes) memcpy(v_pool + (size_t)frame * unit_v_bytes, tmp + unit_k_bytes, unit_v_bytes);
        slot_tbl[uo] = (int32_t)(-1 - host);
        state[uo] = (uint8_t)((state[uo] & ~ST_RESIDENT) | ST_ON_HOST);
        slot_tbl[ui] = frame;
        state[ui] = (uint8_t)((state[ui] & ~ST_ON_HOST) | ST_RESIDENT);
    }
    free(tmp);
    return REF_OK;
}

/* --------------------------------------------- content-addressed dedup */

/* SHA-256 as FIPS 180-4 defines it.  The round constants and the initial hash value are
 * derived here from their definition (section 4.2.2: first 32 bits of the fractional parts
 * of the cube roots of the first 64 primes; section 5.3.3: of the square roots of the first
 * 8 primes) with exact integer arithmetic, not typed in. */
static uint32_t sha_k[64], sha_h0[8];
static int sha_ready = 0;

static uint64_t int_root(unsigned __int128 x, int r) {      /* floor(x^(1/r)), r = 2 or 3 */
    uint64_t lo = 0, hi = (uint64_t)1 << 40;
    while (hi - lo > 1) {
        const uint64_t mid = lo + (hi - lo) / 2;
        unsigned __int128 p = (unsigned __int128)mid * mid;
        if (r == 3) p *= mid;
        if (p <= x) lo = mid; else hi = mid;
    }
    return lo;
}

static void sha_init(void) {
    int found = 0;
    for (int c = 2; found < 64; ++c) {
        int prime = 1;
        for (int d = 2; d * d <= c; ++d) if (c % d == 0) { prime = 0; break; }
        if (!prime) continue;
        /* floor(c^(1/3) * 2^32) = floor((c * 2^96)^(1/3)); its low 32 bits are the fraction's first 32 bits */
        sha_k[found] = (uint32_t)int_root((unsigned __int128)c << 96, 3);
        if (found < 8) sha_h0[found] = (uint32_t)int_root((unsigned __int128)c << 64, 2);
        ++found;
    }
    sha_ready = 1;
}

static uint32_t rotr32(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

static void sha_block(uint32_t h[8], const uint8_t* blk) {
    uint32_t w[64];
    for (int t = 0; t < 16; ++t)
        w[t] = ((uint32_t)blk[4 * t] << 24) | ((uint32_t)blk[4 * t + 1] << 16) | ((uint32_t)blk[4 * t + 2] << 8) | blk[4 * t + 3];
    for (int t = 16; t < 64; ++t) {
        const uint32_t s0 = rotr32(w[t - 15], 7) ^ rotr32(w[t - 15], 18) ^ (w[t - 15] >> 3);
        const uint32_t s1 = rotr32(w[t - 2], 17) ^ rotr32(w[t - 2], 19) ^ (w[t - 2] >> 10);
        w[t] = s1 + w[t - 7] + s0 + w[t - 16];
    }
    uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], hh = h[7];
    for (int t = 0; t < 64; ++t) {
        const uint32_t S1 = rotr32(e, 6) ^ rotr32(e, 11) ^ rotr32(e, 25);
        const uint32_t ch = (e & f) ^ (~e & g);
        const uint32_t t1 = hh + S1 + ch + sha_k[t] + w[t];
        const uint32_t S0 = rotr32(a, 2) ^ rotr32(a, 13) ^ rotr32(a, 22);
        const uint32_t maj = (a & b) ^ (a & c) ^ (b & c);
        const uint32_t t2 = S0 + maj;
        hh = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    h[0] += a; h[1] += b; h[2] += c; h[3] += d; h[4] += e; h[5] += f; h[6] += g; h[7] += hh;
}

/* Digest of msg_a followed by msg_b (either may be empty). */
static void sha256_two(const uint8_t* a, size_t na, const uint8_t* b, size_t nb, uint8_t out[32]) {
    if (!sha_ready) sha_init();
    uint32_t h[8];
    memcpy(h, sha_h0, sizeof h);
    uint8_t buf[64];
    size_t fill = 0;
    const uint64_t total = (uint64_t)na + nb;
    for (size_t i = 0; i < na + nb; ++i) {
        buf[fill++] = i < na ? a[i] : b[i - na];
        if (fill == 64) { sha_block(h, buf); fill = 0; }
    }
    buf[fill++] = 0x80;                                      /* padding: 1 bit, zeros, 64-bit length */
    if (fill > 56) { while (fill < 64) buf[fill++] = 0; sha_block(h, buf); fill = 0; }
    while (fill < 56) buf[fill++] = 0;
    for (int i = 0; i < 8; ++i) buf[56 + i] = (uint8_t)((total * 8) >> (56 - 8 * i));
    sha_block(h, buf);
    for (int i = 0; i < 8; ++i) {
        out[4 * i] = (uint8_t)(h[i] >> 24); out[4 * i + 1] = (uint8_t)(h[i] >> 16);
        out[4 * i + 2] = (uint8_t)(h[i] >> 8); out[4 * i + 3] = (uint8_t)h[i];
    }
}

int kvm_ref_sha256(const uint8_t* msg, uint64_t len, uint8_t* out) {
    if ((!msg && len) || !out) return REF_EINVAL;
    sha256_two(msg, (size_t)len, NULL, 0, out);
    return REF_OK;
}

/* Section 3.6: blocks are indexed by the SHA-256 of their content.  The content of a unit is
 * its record: K frame followed by V frame.  Units that are not in HBM (or malformed uids) get
 * an all-zero digest and are counted in *n_bad. */
int kvm_ref_hash_units(const uint8_t* k_pool, const uint8_t* v_pool, uint64_t n_slots,
                       uint32_t unit_k_bytes, uint32_t unit_v_bytes,
                       const int32_t* slot_tbl, const uint8_t* state, int64_t n_uids,
                       const int64_t* uids, int64_t n, uint8_t* digests, uint32_t* n_bad) {
    if (!k_pool || (unit_v_bytes && !v_pool) || !slot_tbl || !state || n < 0) return REF_EINVAL;
    if (n > 0 && (!uids || !digests)) return REF_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t uid = uids[i];
        if (uid < 0 || uid >= n_uids || !(state[uid] & ST_RESIDENT) || slot_tbl[uid] < 0 ||
            (uint64_t)slot_tbl[uid] >= n_slots) {
            memset(digests + 32 * i, 0, 32);
            if (n_bad) ++*n_bad;
            continue;
        }
        const size_t slot = (size_t)slot_tbl[uid];
        sha256_two(k_pool + slot * unit_k_bytes, unit_k_bytes,
                   unit_v_bytes ? v_pool + slot * unit_v_bytes : NULL, unit_v_bytes, digests + 32 * i);
    }
    return REF_OK;
}

/* Section 3.6: content store with reference counts; a digest that is already there gains a
 * reference and the block is not duplicated.  The store here is a plain list searched
 * from the front: entry e holds a digest, the uid that first brought it (the canonical
 * copy) and the number of references.  Items are taken in list order, so within one call
 * the first occurrence of a new digest becomes canonical.  An entry whose count has dropped
 * to zero (kvm_ref_dedup_release) is revived by the next insert of its digest, which becomes
 * the new canonical copy.  canon_out[i] = canonical uid of item i (== uids[i] when item i is
 * not a duplicate).  Returns REF_EINVAL when the list is full. */
int kvm_ref_dedup_insert(uint8_t* st_digest, int64_t* st_canon, uint32_t* st_refs, int64_t* st_n, int64_t st_cap,
                         const uint8_t* digests, const int64_t* uids, int64_t n, int64_t* canon_out) {
    if (!st_digest || !st_canon || !st_refs || !st_n || n < 0 || (n > 0 && (!digests || !uids || !canon_out)))
        return REF_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        int64_t e = 0;
        while (e < *st_n && memcmp(st_digest + 32 * e, digests + 32 * i, 32) != 0) ++e;
        if (e == *st_n) {
            if (*st_n >= st_cap) return REF_EINVAL;
            memcpy(st_digest + 32 * e, digests + 32 * i, 32);
            st_canon[e] = uids[i];
            st_refs[e] = 1;
            ++*st_n;
        } else if (st_refs[e] == 0) {
            st_canon[e] = uids[i];
            st_refs[e] = 1;
        } else {
            st_refs[e] += 1;
        }
        canon_out[i] = st_canon[e];
    }
    return REF_OK;
}

/* One reference less for each digest in the list (unknown digests and counts already at zero
 * are counted in *n_bad). */
int kvm_ref_dedup_release(const uint8_t* st_digest, uint32_t* st_refs, int64_t st_n,
                          const uint8_t* digests, int64_t n, uint32_t* n_bad) {
    if (!st_digest || !st_refs || n < 0 || (n > 0 && !digests)) return REF_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        int64_t e = 0;
        while (e < st_n && memcmp(st_digest + 32 * e, digests + 32 * i, 32) != 0) ++e;
        if (e == st_n || st_refs[e] == 0) { if (n_bad) ++*n_bad; continue; }
        st_refs[e] -= 1;
    }
    return REF_OK;
}

/* Frames shared by units of equal content (section 3.6: a block whose content the pool already
 * holds is referenced instead of being stored again).  Items in list order; canon[i] is what
 * kvm_ref_dedup_insert reported for uids[i].  Item i with canon[i] != uids[i] whose two units are
 * in range, RESIDENT and not PROTECTED (content still being written), whose duplicate is not
 * SHARED already (others may read its frame) and whose frames are inside the pool and differ:
 * the duplicate gives up its frame (freed[i]) and reads the canonical unit's from now on
 * (slot_tbl[uid] = slot_tbl[canon]); both units get SHARED, which keeps them out of the victim
 * selection and makes pack and exchange refuse them, so a frame that several units read is never
 * handed out again; frame_refs[frame] = number of units reading it (2 after the first sharing,
 * one more for each further duplicate; 0 for frames that are not shared).  Every other item:
 * freed[i] = -1; a uid or canonical uid outside [0, n_uids) is counted in *n_bad. */
int kvm_ref_dedup_share(int32_t* slot_tbl, uint8_t* state, int64_t n_uids, uint64_t n_slots,
                        const int64_t* uids, const int64_t* canon, int64_t n, uint32_t* frame_refs,
                        int32_t* freed, uint32_t* n_bad) {
    if (!slot_tbl || !state || !frame_refs || n < 0 || (n > 0 && (!uids || !canon || !freed))) return REF_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t u = uids[i], c = canon[i];
        freed[i] = -1;
        if (u < 0 || u >= n_uids || c < 0 || c >= n_uids) { if (n_bad) ++*n_bad; continue; }
        if (u == c) continue;
        if (!(state[u] & ST_RESIDENT) || !(state[c] & ST_RESIDENT)) continue;
        if ((state[u] & (ST_PROTECTED | ST_SHARED)) || (state[c] & ST_PROTECTED)) continue;
        const int32_t fu = slot_tbl[u], fc = slot_tbl[c];
        if (fu < 0 || (uint64_t)fu >= n_slots || fc < 0 || (uint64_t)fc >= n_slots || fu == fc) continue;
        slot_tbl[u] = fc;
        freed[i] = fu;
        state[u] |= ST_SHARED;
        state[c] |= ST_SHARED;
        frame_refs[fc] += frame_refs[fc] == 0 ? 2u : 1u;
    }
    return REF_OK;
}

/* A unit gets a frame of its own again (before it may be evicted, or before its content is
 * written to).  Item i with uids[i] in range, RESIDENT and SHARED, its frame and new_frames[i]
 * inside the pool: the bytes it reads are copied to frame new_frames[i], slot_tbl[uid] =
 * new_frames[i], SHARED is cleared, frame_refs[old frame] -= 1 (a unit left as the only reader
 * of a frame keeps SHARED until it is unshared itself); when the count reaches 0 the old frame
 * is free: freed[i] = old frame, otherwise -1.  Every other item: freed[i] = new_frames[i] (the
 * frame comes back unused); out-of-range uids and frames are counted in *n_bad. */
int kvm_ref_dedup_unshare(uint8_t* k_pool, uint8_t* v_pool, uint64_t n_slots, uint32_t unit_k_bytes,
                          uint32_t unit_v_bytes, int32_t* slot_tbl, uint8_t* state, int64_t n_uids,
                          const int64_t* uids, const int32_t* new_frames, int64_t n, uint32_t* frame_refs,
                          int32_t* freed, uint32_t* n_bad) {
    if (!k_pool || (unit_v_bytes && !v_pool) || !slot_tbl || !state || !frame_refs || n < 0) return REF_EINVAL;
    if (n > 0 && (!uids || !new_frames || !freed)) return REF_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t u = uids[i];
        const int32_t nf = new_frames[i];
        freed[i] = nf;
        if (u < 0 || u >= n_uids || nf < 0 || (uint64_t)nf >= n_slots) { if (n_bad) ++*n_bad; continue; }
        if (!(state[u] & ST_RESIDENT) || !(state[u] & ST_SHARED)) continue;
        const int32_t f = slot_tbl[u];
        if (f < 0 || (uint64_t)f >= n_slots || f == nf || frame_refs[f] == 0) continue;
        memcpy(k_pool + (size_t)nf * unit_k_bytes, k_pool + (size_t)f * unit_k_bytes, unit_k_bytes);
        if (unit_v_bytes) memcpy(v_pool + (size_t)nf * unit_v_bytes, v_pool + (size_t)f * unit_v_bytes, unit_v_bytes);
        slot_tbl[u] = nf;
        state[u] &= (uint8_t)~ST_SHARED;
        frame_refs[f] -= 1;
        freed[i] = frame_refs[f] == 0 ? f : -1;
    }
    return REF_OK;
}

/* Number of OpenMP threads the scorer will use (for reporting). */
int kvm_ref_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sets that number (timing on one core and on all of them); returns what is in force. */
int kvm_ref_set_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}
