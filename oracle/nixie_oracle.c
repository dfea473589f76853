/*
 * nixie_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what one context-switch
 * swap computes.  Ordinary host arrays stand in for GPU memory.  Only the
 * tests, the smoke check and the bench's cpu_baseline leg may call this; the
 * GPU library shares no source, header, table or helper with it.
 *
 * What the swap computes (paper, "Hierarchical Memory": every chunk has exactly
 * one copy in the hierarchy and moves between tiers as a whole; "Overview" and
 * "Speeding Up Context Switches": when B is scheduled its chunks go to GPU
 * memory while A's are evicted to CPU memory):
 *
 *     for every outgoing allocation i:  host_i[0..bytes_i) = dev_i[0..bytes_i)
 *     for every incoming allocation j:  dev_j[0..bytes_j)  = host_j[0..bytes_j)
 *
 * o_switch_direct is that definition.  o_switch_staged reaches the same state
 * through a pinned staging ring of bounded size, one step at a time in a
 * seeded random order, and checks the invariants the problem fixes while it
 * goes (every byte moved exactly once, nothing written outside an allocation,
 * a slot free before it is used and staged bytes never above the ring size --
 * both recounted from the slot table after every step, so that a planted
 * mistake in the slot choice or in a direction's share trips them -- and the
 * ring empty at the end).
 *
 * o_switch_staged with in_place = 1 is the in-place switch: the incoming
 * allocations may reuse GPU memory of the outgoing ones, and a GPU byte is
 * only overwritten after its old content has been staged out.  The direct
 * definition covers it unchanged because it evicts everything first.
 *
 * Pins: final state against numpy slicing (a library copy), per-byte copy
 * counts on tiny inputs, red zones checked by the caller, order independence
 * over seeds, planted faults that each check must catch.  The 64-bit hash
 * (o_hash64) is this build's own definition: pinned by the published
 * splitmix64 output sequence for seed 0 (which fixes mix64), by algebraic
 * properties, and by an independent big-integer Python evaluation.
 */
#define _GNU_SOURCE
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <pthread.h>
#include <time.h>

typedef struct {
    uint8_t *dev;   /* stand-in for the device allocation */
    uint8_t *host;  /* pageable host backing */
    uint64_t bytes;
} o_alloc;

/* ---- result definition ------------------------------------------------- */

void o_switch_direct(const o_alloc *out, uint64_t n_out,
                     const o_alloc *in, uint64_t n_in)
{
    for (uint64_t i = 0; i < n_out; i++)
        memcpy(out[i].host, out[i].dev, out[i].bytes);
    for (uint64_t j = 0; j < n_in; j++)
        memcpy(in[j].dev, in[j].host, in[j].bytes);
}

/* ---- 64-bit per-allocation hash ---------------------------------------- */
/* H(b[0..n)) = mix64(n) + sum_k mix64(w_k + G*(k+1))  (mod 2^64),
 * w_k = k-th little-endian 8-byte word of b, the last one zero-padded,
 * mix64 = the output function of splitmix64, G its increment. */

#define O_G 0x9E3779B97F4A7C15ULL

uint64_t o_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

uint64_t o_hash64(const uint8_t *b, uint64_t n)
{
    uint64_t h = o_mix64(n);
    uint64_t nwords = (n + 7) / 8;
    for (uint64_t k = 0; k < nwords; k++) {
        uint64_t w = 0;
        for (int j = 0; j < 8; j++) {
            uint64_t idx = 8 * k + (uint64_t)j;
            if (idx < n)
                w |= (uint64_t)b[idx] << (8 * j);
        }
        h += o_mix64(w + O_G * (k + 1));
    }
    return h;
}

/* hashes of the side that holds the data: which = 0 -> dev, 1 -> host */
void o_hash_table(const o_alloc *t, uint64_t n, int which, uint64_t *hash_out)
{
    for (uint64_t i = 0; i < n; i++)
        hash_out[i] = o_hash64(which ? t[i].host : t[i].dev, t[i].bytes);
}

/* ---- staged form ------------------------------------------------------- */

typedef struct { uint64_t alloc, off, len, slot_off; } o_piece;
typedef struct { uint64_t first, count, bytes; } o_chunk;

typedef struct {
    o_piece *pieces; uint64_t n_pieces;
    o_chunk *chunks; uint64_t n_chunks;
} o_cut;

/* Walk the allocations in table order and cut them into pieces of at most S
 * bytes.  pack = 0: a chunk never mixes allocations.  pack = 1: the next
 * piece continues in the current chunk until it holds S bytes. */
static int cut_table(const o_alloc *t, uint64_t n, uint64_t S, int pack, o_cut *c)
{
    uint64_t max_pieces = 0;
    for (uint64_t i = 0; i < n; i++)
        max_pieces += t[i].bytes / S + 2;
    c->pieces = (o_piece *)calloc(max_pieces + 1, sizeof(o_piece));
    c->chunks = (o_chunk *)calloc(max_pieces + 1, sizeof(o_chunk));
    if (!c->pieces || !c->chunks)
        return -1;
    c->n_pieces = 0;
    c->n_chunks = 0;
    uint64_t fill = 0;
    int open = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint64_t off = 0;
        if (!pack)
            open = 0;
        while (off < t[i].bytes) {
            if (!open || fill == S) {
                c->chunks[c->n_chunks].first = c->n_pieces;
                c->chunks[c->n_chunks].count = 0;
                c->chunks[c->n_chunks].bytes = 0;
                c->n_chunks++;
                fill = 0;
                open = 1;
            }
            uint64_t take = S - fill;
            if (take > t[i].bytes - off)
                take = t[i].bytes - off;
            o_piece *p = &c->pieces[c->n_pieces++];
            p->alloc = i; p->off = off; p->len = take; p->slot_off = fill;
            o_chunk *ch = &c->chunks[c->n_chunks - 1];
            ch->count++;
            ch->bytes += take;
            fill += take;
            off += take;
        }
    }
    return 0;
}

static uint64_t rng_next(uint64_t *s)
{
    *s += O_G;
    return o_mix64(*s);
}

static void shuffle(uint64_t *v, uint64_t n, uint64_t *rng)
{
    for (uint64_t i = n; i > 1; i--) {
        uint64_t j = rng_next(rng) % i;
        uint64_t t = v[i - 1]; v[i - 1] = v[j]; v[j] = t;
    }
}

typedef struct {
    uint64_t hwm_staged_bytes;   /* most payload bytes ever held in the ring  */
    uint64_t final_staged_bytes; /* must be 0                                 */
    uint64_t n_out_chunks, n_in_chunks;
    uint64_t bytes_out, bytes_in;
    uint64_t count_errors;       /* bytes whose copy count != 1 (check_bytes) */
    uint64_t steps;
} o_report;

enum {
    O_OK = 0, O_EINVAL = -1, O_ENOMEM = -2, O_ESLOT_BUSY = -3,
    O_EBUDGET = -4, O_ECOUNT = -5, O_ERANGE = -6, O_ELEFTOVER = -7
};

/* planted mistakes, for the tests that show the checks bite */
enum {
    O_FAULT_NONE = 0, O_FAULT_DROP_CHUNK = 1, O_FAULT_SHORT_PIECE = 2,
    O_FAULT_SLOT_SHIFT = 3, O_FAULT_DOUBLE_COPY = 4, O_FAULT_OVERRUN = 5,
    O_FAULT_WRONG_DIRECTION = 6, O_FAULT_IGNORE_ALIAS = 7,
    O_FAULT_REUSE_BUSY_SLOT = 8,   /* a chunk is staged into a slot that still holds another one      */
    O_FAULT_OVERCOMMIT = 9         /* a direction believes it owns one slot more than the ring gives it */
};

typedef struct {
    const o_alloc *t; uint64_t n; o_cut cut;
    uint64_t *order; uint64_t next;          /* seeded chunk order          */
    int64_t *slot_chunk; uint64_t n_slots;   /* -1 = free, else staged chunk */
    uint64_t granted_slots;                  /* slots of the ring this direction really owns */
    uint8_t *ring;                           /* this direction's sub-ring   */
    uint8_t **stage_cnt, **dest_cnt;         /* per-byte copy counts or NULL */
    uint8_t **gone;                          /* out only, in-place mode: byte has left the GPU */
    int to_host;                             /* 1 = out (dev->host)          */
    uint64_t done;
} o_dir;

static int dir_init(o_dir *d, const o_alloc *t, uint64_t n, uint64_t S, int pack,
                    uint64_t n_slots, uint8_t *ring, int to_host, int check_bytes,
                    uint64_t *rng)
{
    memset(d, 0, sizeof(*d));
    d->t = t; d->n = n; d->n_slots = n_slots; d->ring = ring; d->to_host = to_host;
    d->granted_slots = n_slots;
    if (cut_table(t, n, S, pack, &d->cut))
        return O_ENOMEM;
    d->order = (uint64_t *)malloc((d->cut.n_chunks + 1) * sizeof(uint64_t));
    d->slot_chunk = (int64_t *)malloc((n_slots + 2) * sizeof(int64_t));
    if (!d->order || !d->slot_chunk)
        return O_ENOMEM;
    for (uint64_t k = 0; k < d->cut.n_chunks; k++)
        d->order[k] = k;
    shuffle(d->order, d->cut.n_chunks, rng);
    for (uint64_t s = 0; s < n_slots + 2; s++)
        d->slot_chunk[s] = -1;
    if (check_bytes) {
        d->stage_cnt = (uint8_t **)calloc(n + 1, sizeof(uint8_t *));
        d->dest_cnt = (uint8_t **)calloc(n + 1, sizeof(uint8_t *));
        if (!d->stage_cnt || !d->dest_cnt)
            return O_ENOMEM;
        for (uint64_t i = 0; i < n; i++) {
            d->stage_cnt[i] = (uint8_t *)calloc(t[i].bytes + 1, 1);
            d->dest_cnt[i] = (uint8_t *)calloc(t[i].bytes + 1, 1);
            if (!d->stage_cnt[i] || !d->dest_cnt[i])
                return O_ENOMEM;
        }
    }
    return O_OK;
}

static void dir_free(o_dir *d)
{
    if (d->stage_cnt)
        for (uint64_t i = 0; i < d->n; i++) { free(d->stage_cnt[i]); free(d->dest_cnt[i]); }
    if (d->gone)
        for (uint64_t i = 0; i < d->n; i++) free(d->gone[i]);
    free(d->gone);
    free(d->stage_cnt); free(d->dest_cnt);
    free(d->order); free(d->slot_chunk);
    free(d->cut.pieces); free(d->cut.chunks);
}

static int count_free(const o_dir *d)
{
    int c = 0;
    for (uint64_t s = 0; s < d->n_slots; s++) c += d->slot_chunk[s] < 0;
    return c;
}

static uint64_t pick_slot(const o_dir *d, int want_free, uint64_t *rng)
{
    uint64_t cand = 0, n = 0;
    for (uint64_t s = 0; s < d->n_slots; s++)
        n += (d->slot_chunk[s] < 0) == (want_free != 0);
    uint64_t r = rng_next(rng) % n;
    for (uint64_t s = 0; s < d->n_slots; s++)
        if ((d->slot_chunk[s] < 0) == (want_free != 0)) {
            if (r == 0) { cand = s; break; }
            r--;
        }
    return cand;
}

/* The two invariants of the staging tier, recounted from the slot table after every step and
 * independently of how the step chose its slot:
 *   - a slot is free before it is used: every chunk that has been staged and not yet delivered
 *     must still sit in a slot (a chunk staged over a live one makes the live one vanish), and
 *     no chunk sits in two slots;
 *   - pinned bytes never above ring_bytes: every occupied slot is one the ring really gave to its
 *     direction, and the payload held by all occupied slots fits the ring.
 * running = the step loop's own byte count, which must agree with the recount. */
static int audit_ring(const o_dir *d, uint64_t slot_bytes, uint64_t ring_bytes, uint64_t running)
{
    uint64_t held = 0, extent = 0;
    for (int x = 0; x < 2; x++) {
        uint64_t occupied = 0;
        for (uint64_t s = 0; s < d[x].n_slots; s++) {
            if (d[x].slot_chunk[s] < 0) continue;
            occupied++;
            if (s >= d[x].granted_slots) return O_EBUDGET;          /* memory beyond this direction's share */
            held += d[x].cut.chunks[d[x].slot_chunk[s]].bytes;
            for (uint64_t r = s + 1; r < d[x].n_slots; r++)
                if (d[x].slot_chunk[r] == d[x].slot_chunk[s]) return O_ESLOT_BUSY;
        }
        if (d[x].next - d[x].done != occupied) return O_ESLOT_BUSY;  /* a staged chunk was overwritten */
        extent += d[x].granted_slots * slot_bytes;
    }
    if (held != running) return O_ECOUNT;
    if (held > ring_bytes || extent > ring_bytes) return O_EBUDGET;
    return O_OK;
}

/* In-place switch (the incoming application reuses GPU memory the outgoing one gives up; paper,
 * "Maintaining consistent virtual memory addresses" and the premise that both sets do not fit):
 * a GPU byte may only be overwritten once its old content has been staged out.  True if every
 * byte that chunk k of the incoming direction would write has already left the GPU. */
static int scatter_allowed(const o_dir *in, const o_dir *out, uint64_t k)
{
    const o_chunk *ch = &in->cut.chunks[k];
    for (uint64_t q = ch->first; q < ch->first + ch->count; q++) {
        const o_piece *p = &in->cut.pieces[q];
        uintptr_t a = (uintptr_t)in->t[p->alloc].dev + p->off, b = a + p->len;
        for (uint64_t i = 0; i < out->n; i++) {
            uintptr_t lo = (uintptr_t)out->t[i].dev, hi = lo + out->t[i].bytes;
            uintptr_t x0 = a > lo ? a : lo, x1 = b < hi ? b : hi;
            for (uintptr_t x = x0; x < x1; x++)
                if (!out->gone[i][x - lo]) return 0;
        }
    }
    return 1;
}

/*
 * One bidirectional switch through a ring of ring_bytes cut into slots of
 * slot_bytes; the first n_out_slots slots serve the outgoing direction (the
 * window reserved for the evicted application, "Speeding Up Context
 * Switches"), the rest the incoming one.  Steps are taken one at a time in an
 * order drawn from seed.  Returns O_OK or the first violated invariant.
 */
int o_switch_staged(const o_alloc *out, uint64_t n_out,
                    const o_alloc *in, uint64_t n_in,
                    uint64_t ring_bytes, uint64_t slot_bytes, uint64_t n_out_slots,
                    int pack, uint64_t seed, int check_bytes, int fault, int in_place,
                    o_report *rep)
{
    o_report local;
    if (!rep) rep = &local;
    memset(rep, 0, sizeof(*rep));
    if (slot_bytes == 0 || ring_bytes < slot_bytes)
        return O_EINVAL;
    uint64_t n_slots = ring_bytes / slot_bytes;
    uint64_t tot_out = 0, tot_in = 0;
    for (uint64_t i = 0; i < n_out; i++) tot_out += out[i].bytes;
    for (uint64_t j = 0; j < n_in; j++) tot_in += in[j].bytes;
    if (tot_out == 0) n_out_slots = 0;
    if (tot_in == 0) n_out_slots = n_slots;
    if (n_out_slots > n_slots) return O_EINVAL;
    if (tot_out && n_out_slots == 0) return O_EINVAL;
    if (tot_in && n_out_slots == n_slots) return O_EINVAL;

    /* the pinned budget; one slot of slack behind it so that a planted overcommit is caught by the
     * audit, not by the allocator */
    uint8_t *ring = (uint8_t *)malloc(ring_bytes + slot_bytes);
    if (!ring) return O_ENOMEM;
    uint64_t rng = seed;
    o_dir d[2];
    int rc = dir_init(&d[0], out, n_out, slot_bytes, pack, n_out_slots, ring, 1, check_bytes, &rng);
    if (rc == O_OK)
        rc = dir_init(&d[1], in, n_in, slot_bytes, pack, n_slots - n_out_slots,
                      ring + n_out_slots * slot_bytes, 0, check_bytes, &rng);
    rep->n_out_chunks = d[0].cut.n_chunks;
    rep->n_in_chunks = d[1].cut.n_chunks;
    if (rc == O_OK && in_place) {
        d[0].gone = (uint8_t **)calloc(n_out + 1, sizeof(uint8_t *));
        if (!d[0].gone) rc = O_ENOMEM;
        for (uint64_t i = 0; rc == O_OK && i < n_out; i++)
            if (!(d[0].gone[i] = (uint8_t *)calloc(out[i].bytes + 1, 1))) rc = O_ENOMEM;
    }
    uint64_t staged = 0;
    int fault_armed = fault;
    if (rc == O_OK && fault == O_FAULT_OVERCOMMIT)   /* the last direction in the ring counts one slot too many */
        d[tot_in ? 1 : 0].n_slots++;

    while (rc == O_OK) {
        /* feasible steps: 0 stage-out (GPU->ring), 1 drain (ring->host),
         *                 2 fill (host->ring),     3 scatter (ring->GPU) */
        int feas[4], nf = 0;
        int64_t ok_slot[4096];   /* staged incoming slots whose chunk may be scattered now */
        uint64_t n_ok = 0;
        for (int x = 0; x < 2; x++) {
            if (d[x].next < d[x].cut.n_chunks && count_free(&d[x]) > 0) feas[nf++] = 2 * x;
            if (x == 0 || !in_place || fault == O_FAULT_IGNORE_ALIAS) {
                if ((uint64_t)count_free(&d[x]) < d[x].n_slots) feas[nf++] = 2 * x + 1;
            } else {
                for (uint64_t s = 0; s < d[1].n_slots && n_ok < 4096; s++)
                    if (d[1].slot_chunk[s] >= 0 && scatter_allowed(&d[1], &d[0], (uint64_t)d[1].slot_chunk[s]))
                        ok_slot[n_ok++] = (int64_t)s;
                if (n_ok) feas[nf++] = 3;
            }
        }
        if (nf == 0) break;
        int step = feas[rng_next(&rng) % (uint64_t)nf];
        o_dir *D = &d[step / 2];
        int stage_in = (step % 2) == 0;
        rep->steps++;
        if (stage_in) {
            uint64_t s = pick_slot(D, 1, &rng);
            if (fault_armed == O_FAULT_REUSE_BUSY_SLOT && (uint64_t)count_free(D) < D->n_slots) {
                s = pick_slot(D, 0, &rng);
                fault_armed = 0;
            }
            if (fault_armed == O_FAULT_OVERCOMMIT && D->n_slots > D->granted_slots) {
                s = D->granted_slots;
                fault_armed = 0;
            }
            uint64_t k = D->order[D->next++];
            const o_chunk *ch = &D->cut.chunks[k];
            for (uint64_t q = ch->first; q < ch->first + ch->count; q++) {
                const o_piece *p = &D->cut.pieces[q];
                const o_alloc *a = &D->t[p->alloc];
                if (p->off + p->len > a->bytes || p->slot_off + p->len > slot_bytes) { rc = O_ERANGE; break; }
                const uint8_t *src = (D->to_host ? a->dev : a->host) + p->off;
                if (fault_armed == O_FAULT_WRONG_DIRECTION) { src = (D->to_host ? a->host : a->dev) + p->off; }
                memcpy(D->ring + s * slot_bytes + p->slot_off, src, p->len);
                if (D->stage_cnt)
                    for (uint64_t b = 0; b < p->len; b++) D->stage_cnt[p->alloc][p->off + b]++;
                if (D->gone)
                    for (uint64_t b = 0; b < p->len; b++) D->gone[p->alloc][p->off + b] = 1;
            }
            if (fault_armed == O_FAULT_WRONG_DIRECTION) fault_armed = 0;
            D->slot_chunk[s] = (int64_t)k;
            staged += ch->bytes;
            if (staged > rep->hwm_staged_bytes) rep->hwm_staged_bytes = staged;
        } else {
            uint64_t s = n_ok && step == 3 ? (uint64_t)ok_slot[rng_next(&rng) % n_ok] : pick_slot(D, 0, &rng);
            uint64_t k = (uint64_t)D->slot_chunk[s];
            const o_chunk *ch = &D->cut.chunks[k];
            int drop = 0;
            if (fault_armed == O_FAULT_DROP_CHUNK) { drop = 1; fault_armed = 0; }
            for (uint64_t q = ch->first; q < ch->first + ch->count && !drop; q++) {
                const o_piece *p = &D->cut.pieces[q];
                const o_alloc *a = &D->t[p->alloc];
                uint64_t len = p->len, shift = 0;
                if (fault_armed == O_FAULT_SHORT_PIECE && len > 0) { len--; fault_armed = 0; }
                if (fault_armed == O_FAULT_OVERRUN) { len++; fault_armed = 0; }
                if (fault_armed == O_FAULT_SLOT_SHIFT && p->slot_off + p->len < slot_bytes) { shift = 1; fault_armed = 0; }
                uint8_t *dst = (D->to_host ? a->host : a->dev) + p->off;
                memcpy(dst, D->ring + s * slot_bytes + p->slot_off + shift, len);
                if (D->dest_cnt)
                    for (uint64_t b = 0; b < len && p->off + b < a->bytes; b++) D->dest_cnt[p->alloc][p->off + b]++;
                if (fault_armed == O_FAULT_DOUBLE_COPY) {
                    memcpy(dst, D->ring + s * slot_bytes + p->slot_off, len);
                    if (D->dest_cnt)
                        for (uint64_t b = 0; b < len; b++) D->dest_cnt[p->alloc][p->off + b]++;
                    fault_armed = 0;
                }
            }
            D->slot_chunk[s] = -1;
            staged -= ch->bytes;
            D->done++;
            if (D->to_host) rep->bytes_out += ch->bytes; else rep->bytes_in += ch->bytes;
        }
        if (rc == O_OK) rc = audit_ring(d, slot_bytes, ring_bytes, staged);
    }

    if (rc == O_OK) {
        rep->final_staged_bytes = staged;
        if (staged != 0 || d[0].done != d[0].cut.n_chunks || d[1].done != d[1].cut.n_chunks)
            rc = O_ELEFTOVER;
    }
    if (rc == O_OK && check_bytes) {
        for (int x = 0; x < 2; x++)
            for (uint64_t i = 0; i < d[x].n; i++)
                for (uint64_t b = 0; b < d[x].t[i].bytes; b++)
                    if (d[x].stage_cnt[i][b] != 1 || d[x].dest_cnt[i][b] != 1)
                        rep->count_errors++;
        if (rep->count_errors) rc = O_ECOUNT;
    }
    dir_free(&d[0]);
    dir_free(&d[1]);
    free(ring);
    return rc;
}

/* ---- timed, multi-threaded staged form (reported CPU baseline) ---------- */
/* T threads per direction.  Thread t of a direction owns slot t of that
 * direction's sub-ring and moves chunks t, t+T, t+2T, ... through it:
 * source -> slot -> destination.  Same cut as above (pack = 1). */

typedef struct {
    const o_alloc *t; const o_cut *cut; uint8_t *slot; uint64_t first, stride; int to_host;
} mt_arg;

static void *mt_worker(void *vp)
{
    mt_arg *a = (mt_arg *)vp;
    for (uint64_t k = a->first; k < a->cut->n_chunks; k += a->stride) {
        const o_chunk *ch = &a->cut->chunks[k];
        for (uint64_t q = ch->first; q < ch->first + ch->count; q++) {
            const o_piece *p = &a->cut->pieces[q];
            const o_alloc *al = &a->t[p->alloc];
            memcpy(a->slot + p->slot_off, (a->to_host ? al->dev : al->host) + p->off, p->len);
        }
        for (uint64_t q = ch->first; q < ch->first + ch->count; q++) {
            const o_piece *p = &a->cut->pieces[q];
            const o_alloc *al = &a->t[p->alloc];
            memcpy((a->to_host ? al->host : al->dev) + p->off, a->slot + p->slot_off, p->len);
        }
    }
    return NULL;
}

int o_switch_staged_mt(const o_alloc *out, uint64_t n_out, const o_alloc *in, uint64_t n_in,
                       uint64_t ring_bytes, uint64_t slot_bytes, int threads_per_dir,
                       double *seconds)
{
    if (threads_per_dir < 1 || slot_bytes == 0 ||
        (uint64_t)(2 * threads_per_dir) * slot_bytes > ring_bytes)
        return O_EINVAL;
    uint8_t *ring = (uint8_t *)malloc(ring_bytes);
    if (!ring) return O_ENOMEM;
    memset(ring, 0, ring_bytes);
    o_cut cut[2];
    if (cut_table(out, n_out, slot_bytes, 1, &cut[0]) || cut_table(in, n_in, slot_bytes, 1, &cut[1])) {
        free(ring);
        return O_ENOMEM;
    }
    int T = threads_per_dir;
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * 2 * (size_t)T);
    mt_arg *args = (mt_arg *)malloc(sizeof(mt_arg) * 2 * (size_t)T);
    struct timespec t0, t1;
    clock_gettime(CLOCK_MONOTONIC, &t0);
    for (int x = 0; x < 2; x++)
        for (int t = 0; t < T; t++) {
            mt_arg *a = &args[x * T + t];
            a->t = x ? in : out; a->cut = &cut[x]; a->to_host = !x;
            a->slot = ring + (uint64_t)(x * T + t) * slot_bytes;
            a->first = (uint64_t)t; a->stride = (uint64_t)T;
            pthread_create(&th[x * T + t], NULL, mt_worker, a);
        }
    for (int i = 0; i < 2 * T; i++)
        pthread_join(th[i], NULL);
    clock_gettime(CLOCK_MONOTONIC, &t1);
    if (seconds)
        *seconds = (double)(t1.tv_sec - t0.tv_sec) + 1e-9 * (double)(t1.tv_nsec - t0.tv_nsec);
    free(th); free(args); free(ring);
    free(cut[0].pieces); free(cut[0].chunks); free(cut[1].pieces); free(cut[1].chunks);
    return O_OK;
}
