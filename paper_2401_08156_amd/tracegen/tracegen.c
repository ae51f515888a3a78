/*
 * Seeded synthetic alloc/free trace generators.
 *
 * The paper's allocation streams come from fine-tuning real LLMs with
 * recomputation, offloading and LoRA (Sec. 2.3, Sec. 5.1, Table 2).  Those
 * runs cannot be reproduced offline, so these generators emit streams with the
 * same structure: layer-periodic transformer activations with recomputation,
 * out-of-order transient staging buffers, long-lived frozen weights plus many
 * small adapter tensors.  Nothing here knows anything about an allocator
 * policy: the output is only a sequence of (ALLOC size slot) / (FREE slot)
 * events, consumed unchanged by every replay implementation.
 *
 * Event word (u64):  bits 0-30  size in 512-byte units (ALLOC only)
 *                    bit  31    kind: 0 = ALLOC, 1 = FREE
 *                    bits 32-63 slot (handle chosen by the generator: always
 *                               the lowest slot not currently bound)
 *
 * Random numbers: splitmix64 (Steele, Lea, Flood 2014; Vigna's public-domain
 * formulation), one independent stream per (seed, trace index).
 * "Log-uniform" sizes are drawn integer-only as octave-uniform: pick the
 * octave e uniformly, then 2^e + (r mod 2^e), rounded up to 512 bytes.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <pthread.h>

#define UNIT 512ull
#define KIND_FREE (1ull << 31)

typedef struct {
    uint64_t s;
} rng_t;

static uint64_t rng_next(rng_t *r)
{
    uint64_t z = (r->s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static void rng_seed(rng_t *r, uint64_t seed, uint64_t trace)
{
    r->s = seed * 0xD1342543DE82EF95ull + trace * 0x2545F4914F6CDD1Dull + 1;
    (void)rng_next(r);
    (void)rng_next(r);
}

/* octave-uniform size in bytes over [2^lo, 2^hi), rounded up to 512 B */
static uint64_t draw_octave(rng_t *r, unsigned lo, unsigned hi)
{
    uint64_t a = rng_next(r);
    unsigned e = lo + (unsigned)(a % (hi - lo));
    uint64_t b = rng_next(r);
    uint64_t v = (1ull << e) + (b & ((1ull << e) - 1));
    return (v + UNIT - 1) / UNIT * UNIT;
}

/* ---- event sink with lowest-free-slot handle assignment ---------------- */

typedef struct {
    uint64_t *out;
    uint32_t n, cap;          /* events written / wanted                    */
    uint32_t *heap;           /* min-heap of released slots                 */
    uint32_t heap_n, heap_cap;
    uint32_t next_slot;       /* slots >= next_slot were never used         */
    uint32_t max_slot_used;
} sink_t;

static int sink_full(const sink_t *s) { return s->n >= s->cap; }

static void heap_push(sink_t *s, uint32_t v)
{
    if (s->heap_n == s->heap_cap) {
        s->heap_cap = s->heap_cap ? 2 * s->heap_cap : 256;
        s->heap = (uint32_t *)realloc(s->heap, s->heap_cap * sizeof(uint32_t));
    }
    uint32_t i = s->heap_n++;
    while (i > 0) {
        uint32_t p = (i - 1) / 2;
        if (s->heap[p] <= v) break;
        s->heap[i] = s->heap[p];
        i = p;
    }
    s->heap[i] = v;
}

static uint32_t heap_pop(sink_t *s)
{
    uint32_t top = s->heap[0];
    uint32_t v = s->heap[--s->heap_n];
    uint32_t i = 0;
    for (;;) {
        uint32_t c = 2 * i + 1;
        if (c >= s->heap_n) break;
        if (c + 1 < s->heap_n && s->heap[c + 1] < s->heap[c]) c++;
        if (s->heap[c] >= v) break;
        s->heap[i] = s->heap[c];
        i = c;
    }
    if (s->heap_n) s->heap[i] = v;
    return top;
}

#define NO_SLOT 0xFFFFFFFFu

/* emit ALLOC of `bytes`; returns the slot, or NO_SLOT once the row is full */
static uint32_t ev_alloc(sink_t *s, uint64_t bytes)
{
    if (sink_full(s)) return NO_SLOT;
    uint32_t slot = s->heap_n ? heap_pop(s) : s->next_slot++;
    if (slot > s->max_slot_used) s->max_slot_used = slot;
    uint64_t units = (bytes + UNIT - 1) / UNIT;
    s->out[s->n++] = ((uint64_t)slot << 32) | units;
    return slot;
}

static void ev_free(sink_t *s, uint32_t slot)
{
    if (slot == NO_SLOT || sink_full(s)) return;
    s->out[s->n++] = ((uint64_t)slot << 32) | KIND_FREE;
    heap_push(s, slot);
}

/* ---- config 1: random alloc/free ---------------------------------------- */

static void gen_random(sink_t *s, rng_t *r)
{
    uint32_t *live = (uint32_t *)malloc((size_t)(s->cap + 1) * sizeof(uint32_t));
    uint32_t n_live = 0;
    while (!sink_full(s)) {
        uint64_t a = rng_next(r);
        uint32_t lo = (uint32_t)a, hi = (uint32_t)(a >> 32);
        if (n_live > 0 && lo < 1932735283u /* floor(0.45 * 2^32) */) {
            uint32_t k = hi % n_live;
            ev_free(s, live[k]);
            live[k] = live[--n_live];
        } else {
            live[n_live++] = ev_alloc(s, draw_octave(r, 9, 26)); /* 512 B .. 64 MiB */
        }
    }
    free(live);
}

/* ---- transformer step with activation recomputation --------------------- */

typedef struct {
    unsigned layers;          /* L                                           */
    uint64_t hidden;          /* h                                           */
    uint64_t micro_batch;     /* b                                           */
    int staging;              /* config 3: transient offload buffers         */
    int lora;                 /* config 4: frozen weights + adapters         */
    int periodic;             /* every step has the same sequence length     */
} model_t;

#define MAX_PENDING 4096
typedef struct {
    uint64_t due[MAX_PENDING];
    uint32_t slot[MAX_PENDING];
    uint32_t n;
} pending_t;

typedef struct {
    sink_t *s;
    rng_t *r;
    const model_t *m;
    pending_t *pend;          /* NULL unless staging                         */
} ctx_t;

/* staging buffers (offloading): before a base event, release what is due,
 * then with probability 1/8 allocate a 256 MiB - 2 GiB buffer whose release
 * is scheduled 1 + Geometric(0.1) events later. */
static void staging_tick(ctx_t *c)
{
    pending_t *p = c->pend;
    if (!p) return;
    uint64_t now = c->s->n;
    for (;;) {                      /* oldest due first, then insertion order */
        uint32_t best = NO_SLOT;
        for (uint32_t i = 0; i < p->n; i++)
            if (p->due[i] <= now && (best == NO_SLOT || p->due[i] < p->due[best])) best = i;
        if (best == NO_SLOT) break;
        ev_free(c->s, p->slot[best]);
        for (uint32_t i = best; i + 1 < p->n; i++) {
            p->due[i] = p->due[i + 1];
            p->slot[i] = p->slot[i + 1];
        }
        p->n--;
    }
    uint64_t a = rng_next(c->r);
    if ((a & 7) == 0 && p->n < MAX_PENDING && !sink_full(c->s)) {
        uint64_t bytes = draw_octave(c->r, 28, 31);
        uint32_t lag = 1;
        for (int t = 0; t < 256; t++) {
            if ((uint32_t)rng_next(c->r) < 429496729u /* floor(0.1 * 2^32) */) break;
            lag++;
        }
        uint32_t slot = ev_alloc(c->s, bytes);
        p->due[p->n] = (uint64_t)c->s->n + lag;
        p->slot[p->n] = slot;
        p->n++;
    }
}

static uint32_t A(ctx_t *c, uint64_t bytes)
{
    staging_tick(c);
    return ev_alloc(c->s, bytes);
}

static void F(ctx_t *c, uint32_t slot)
{
    staging_tick(c);
    ev_free(c->s, slot);
}

#define MAX_LAYERS 64
#define ADAPT_PER_LAYER 8

static void gen_transformer(sink_t *s, rng_t *r, const model_t *m)
{
    pending_t *pend = NULL;
    if (m->staging) {
        pend = (pending_t *)malloc(sizeof(pending_t));
        pend->n = 0;
    }
    ctx_t c = { s, r, m, pend };
    const unsigned L = m->layers;
    uint32_t ckpt[MAX_LAYERS];
    uint32_t *grads = NULL;
    uint64_t rank = 0, adapter_bytes = 0;

    if (m->lora) {
        /* long-lived state: frozen weight blocks, then the adapter tensors */
        for (int i = 0; i < 128; i++) (void)A(&c, draw_octave(r, 25, 29)); /* 32 - 512 MiB */
        rank = 8ull << (rng_next(r) & 3);                                 /* 8,16,32,64   */
        adapter_bytes = rank * 4096 * 4;                                  /* fp32         */
        for (unsigned i = 0; i < L * ADAPT_PER_LAYER; i++) (void)A(&c, adapter_bytes);
        grads = (uint32_t *)malloc(sizeof(uint32_t) * L * ADAPT_PER_LAYER);
    }

    while (!sink_full(s)) {
        uint64_t seq = 1024 + 256 * (rng_next(r) % 13);        /* 1024 .. 4096 */
        if (m->periodic) seq = 2048;                           /* strictly periodic variant */
        uint64_t T1 = m->micro_batch * seq * m->hidden * 2;    /* [b,s,h] bf16 */
        uint64_t T4 = 4 * T1;                                  /* [b,s,4h]     */
        uint64_t Ta = m->micro_batch * seq * rank * 2;         /* [b,s,rank]   */
        uint32_t out_prev = NO_SLOT;
        uint32_t act[4] = { NO_SLOT, NO_SLOT, NO_SLOT, NO_SLOT };

        /* forward: keep one checkpoint per layer, drop the rest */
        for (unsigned l = 0; l < L && !sink_full(s); l++) {
            ckpt[l] = A(&c, T1);
            if (m->lora) { act[0] = A(&c, Ta); act[1] = A(&c, Ta); }
            uint32_t mid = A(&c, T4);
            if (m->lora) { act[2] = A(&c, Ta); act[3] = A(&c, Ta); }
            uint32_t out = A(&c, T1);
            if (m->lora) F(&c, act[0]);
            F(&c, mid);
            if (m->lora) { F(&c, act[1]); F(&c, act[2]); F(&c, act[3]); }
            if (out_prev != NO_SLOT) F(&c, out_prev);
            out_prev = out;
        }
        /* backward: recompute each layer's activations, newest layer first */
        uint32_t g1_next = out_prev;
        unsigned n_grads = 0;
        for (unsigned l = L; l-- > 0 && !sink_full(s);) {
            uint32_t r1 = A(&c, T1);
            if (m->lora) { act[0] = A(&c, Ta); act[1] = A(&c, Ta); }
            uint32_t r4 = A(&c, T4);
            if (m->lora) { act[2] = A(&c, Ta); act[3] = A(&c, Ta); }
            uint32_t g4 = A(&c, T4);
            uint32_t g1 = A(&c, T1);
            if (m->lora)
                for (int j = 0; j < ADAPT_PER_LAYER; j++) grads[n_grads++] = A(&c, adapter_bytes);
            F(&c, r4);
            if (m->lora) { F(&c, act[3]); F(&c, act[2]); }
            F(&c, g4);
            F(&c, r1);
            if (m->lora) { F(&c, act[1]); F(&c, act[0]); }
            F(&c, g1_next);
            F(&c, ckpt[l]);
            g1_next = g1;
        }
        F(&c, g1_next);
        /* optimizer phase: adapter gradients released in allocation order */
        for (unsigned i = 0; i < n_grads && !sink_full(s); i++) F(&c, grads[i]);
    }
    free(grads);
    free(pend);
}

/* ---- ZeRO-3 data parallelism over N devices (Sec. 2.4, Sec. 5.3.2) -------- */

/*
 * One rank's stream under parameter / gradient / optimizer-state partitioning
 * with LoRA and recomputation.  Persistent tensors are the rank's 1/N shards,
 * so they shrink as N grows; before a layer runs (forward, and again for the
 * recomputing backward) its four weight matrices are gathered into transient
 * full-size buffers, the next layer's being fetched one layer ahead, and are
 * released when the layer is done.  Adapter gradients are produced full-size
 * and reduced into a kept 1/N shard.  With N = 1 nothing is gathered.
 */
static uint64_t shard(uint64_t bytes, uint64_t n) { return (bytes + n - 1) / n; }

static void gather_layer(ctx_t *c, const uint64_t w[4], uint32_t buf[4])
{
    for (int k = 0; k < 4; k++) buf[k] = A(c, w[k]);
}

static void release_layer(ctx_t *c, uint32_t buf[4])
{
    for (int k = 0; k < 4; k++) { F(c, buf[k]); buf[k] = NO_SLOT; }
}

static void gen_zero3(sink_t *s, rng_t *r, const model_t *m, uint64_t world)
{
    ctx_t c = { s, r, m, NULL };
    const unsigned L = m->layers;
    const uint64_t h = m->hidden;
    const uint64_t w[4] = { 3 * h * h * 2, h * h * 2, 4 * h * h * 2, 4 * h * h * 2 };  /* qkv, proj, up, down; 2 B */
    const uint64_t rank = 8ull << (rng_next(r) & 3);
    const uint64_t adapter = rank * h * 4;                                        /* fp32 */
    uint32_t ckpt[MAX_LAYERS];
    uint32_t *grads = (uint32_t *)malloc(sizeof(uint32_t) * L * ADAPT_PER_LAYER);

    /* persistent: frozen weight shards, then adapter shards with two optimizer moments each */
    for (unsigned l = 0; l < L; l++)
        for (int k = 0; k < 4; k++) (void)A(&c, shard(w[k], world));
    for (unsigned i = 0; i < L * ADAPT_PER_LAYER * 3; i++) (void)A(&c, shard(adapter, world));

    while (!sink_full(s)) {
        uint64_t seq = 1024 + 256 * (rng_next(r) % 13);
        uint64_t T1 = m->micro_batch * seq * h * 2, T4 = 4 * T1;
        uint32_t cur[4] = { NO_SLOT, NO_SLOT, NO_SLOT, NO_SLOT }, nxt[4] = { NO_SLOT, NO_SLOT, NO_SLOT, NO_SLOT };
        uint32_t out_prev = NO_SLOT;

        if (world > 1) gather_layer(&c, w, cur);
        for (unsigned l = 0; l < L && !sink_full(s); l++) {
            ckpt[l] = A(&c, T1);
            if (world > 1 && l + 1 < L) gather_layer(&c, w, nxt);
            uint32_t mid = A(&c, T4);
            uint32_t out = A(&c, T1);
            F(&c, mid);
            if (out_prev != NO_SLOT) F(&c, out_prev);
            out_prev = out;
            if (world > 1) { release_layer(&c, cur); memcpy(cur, nxt, sizeof cur); }
        }
        uint32_t g1_next = out_prev;
        unsigned n_grads = 0;
        if (world > 1) gather_layer(&c, w, cur);
        for (unsigned l = L; l-- > 0 && !sink_full(s);) {
            uint32_t r1 = A(&c, T1);
            if (world > 1 && l > 0) gather_layer(&c, w, nxt);
            uint32_t r4 = A(&c, T4);
            uint32_t g4 = A(&c, T4);
            uint32_t g1 = A(&c, T1);
            for (int j = 0; j < ADAPT_PER_LAYER; j++) {
                uint32_t full = A(&c, adapter);
                if (world > 1) {
                    grads[n_grads++] = A(&c, shard(adapter, world));
                    F(&c, full);
                } else {
                    grads[n_grads++] = full;
                }
            }
            F(&c, r4);
            F(&c, g4);
            F(&c, r1);
            F(&c, g1_next);
            F(&c, ckpt[l]);
            g1_next = g1;
            if (world > 1) { release_layer(&c, cur); memcpy(cur, nxt, sizeof cur); }
        }
        F(&c, g1_next);
        for (unsigned i = 0; i < n_grads && !sink_full(s); i++) F(&c, grads[i]);
    }
    free(grads);
}

/* ---- public entry -------------------------------------------------------- */

static const model_t MODEL_RECOMPUTE = { 32, 4096, 4, 0, 0, 0 };
static const model_t MODEL_OFFLOAD   = { 40, 5120, 4, 1, 0, 0 };
static const model_t MODEL_LORA      = { 32, 4096, 4, 0, 1, 0 };

static uint32_t gen_one(int config, uint64_t seed, uint64_t trace, uint64_t *row, uint32_t n_events)
{
    sink_t s;
    memset(&s, 0, sizeof s);
    s.out = row;
    s.cap = n_events;
    rng_t r;
    rng_seed(&r, seed, trace);
    int kind = config % 10;
    if (config == 5) kind = 2 + (int)(trace % 3);
    model_t m = MODEL_RECOMPUTE;
    switch (kind) {
    case 1: gen_random(&s, &r); break;
    case 2: m = MODEL_RECOMPUTE; break;
    case 3: m = MODEL_OFFLOAD; break;
    case 4: m = MODEL_LORA; break;
    case 6: gen_zero3(&s, &r, &MODEL_RECOMPUTE, 1ull << (trace % 5)); break;   /* 1, 2, 4, 8, 16 devices */
    default: break;
    }
    if (kind >= 2 && kind <= 4) {
        m.periodic = config >= 10;          /* 12, 13, 14: the same recipes with a fixed sequence length */
        gen_transformer(&s, &r, &m);
    }
    free(s.heap);
    return s.max_slot_used + 1;
}

typedef struct {
    int config;
    uint64_t seed;
    uint32_t t0, t1, first_trace, trace_stride, n_events;
    uint64_t *events;
    uint32_t max_slots;
} job_t;

static void *worker(void *arg)
{
    job_t *j = (job_t *)arg;
    for (uint32_t t = j->t0; t < j->t1; t++) {
        uint32_t m = gen_one(j->config, j->seed, (uint64_t)j->first_trace + (uint64_t)t * j->trace_stride,
                             j->events + (size_t)t * j->n_events, j->n_events);
        if (m > j->max_slots) j->max_slots = m;
    }
    return NULL;
}

/*
 * Fill events[n_traces][n_events] (host memory, row-major) for traces
 * first_trace, first_trace + trace_stride, ... of configuration `config`
 * (1 random, 2 recompute, 3 offload, 4 LoRA, 5 even mixture of 2/3/4;
 * 6: one rank of ZeRO-3 over 2^(trace mod 5) devices;
 * 12, 13, 14: recipes 2, 3, 4 with the same sequence length in every step).
 * Returns the number of slots needed (1 + the largest slot used), or 0 on a
 * bad argument.  Every row holds exactly n_events events.
 */
uint32_t tracegen_fill(int config, uint64_t seed, uint32_t first_trace, uint32_t trace_stride,
                       uint32_t n_traces, uint32_t n_events, uint64_t *events, int n_threads)
{
    if (!((config >= 1 && config <= 6) || (config >= 12 && config <= 14)) || !events || n_events == 0 || trace_stride == 0)
        return 0;
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 64) n_threads = 64;
    if ((uint32_t)n_threads > n_traces) n_threads = (int)(n_traces ? n_traces : 1);
    job_t jobs[64];
    pthread_t th[64];
    for (int i = 0; i < n_threads; i++) {
        jobs[i].config = config;
        jobs[i].seed = seed;
        jobs[i].t0 = (uint32_t)((uint64_t)n_traces * i / n_threads);
        jobs[i].t1 = (uint32_t)((uint64_t)n_traces * (i + 1) / n_threads);
        jobs[i].first_trace = first_trace;
        jobs[i].trace_stride = trace_stride;
        jobs[i].n_events = n_events;
        jobs[i].events = events;
        jobs[i].max_slots = 0;
    }
    for (int i = 1; i < n_threads; i++) pthread_create(&th[i], NULL, worker, &jobs[i]);
    worker(&jobs[0]);
    uint32_t m = jobs[0].max_slots;
    for (int i = 1; i < n_threads; i++) {
        pthread_join(th[i], NULL);
        if (jobs[i].max_slots > m) m = jobs[i].max_slots;
    }
    return m;
}
