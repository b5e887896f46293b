/*
 * lmc_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded CPU statement of what the KV-cache chunk path
 * computes.  It exists so that the GPU library can be checked against something
 * that can be verified by eye.  Nothing in the product may include, link, import
 * or call this file; only tests, the smoke check and the benchmark's CPU-baseline
 * leg do.  It shares no header, helper or constant with the GPU library: the
 * geometry struct below is declared here a second time on purpose.
 *
 * What is modelled (paper section 5.1, "Configurable Chunk Size", and the store /
 * retrieve workflows of section 4):
 *   - the engine keeps KV cache in small pages, one page = BS tokens of one layer;
 *   - the cache layer groups the pages of CT (default 256) consecutive tokens, over
 *     all layers and both K and V, into one contiguous chunk;
 *   - store   = copy the scattered pages into a contiguous chunk buffer, then move
 *               that buffer as a whole to CPU memory;
 *   - retrieve = move whole chunks back and split them into (fresh) pages;
 *   - a token processor decides which chunks are new (store) and how many leading
 *     chunks of a prompt are already present (retrieve).
 *
 * The paper fixes none of the layouts, the hash or the slot mapping.  The readings
 * taken here (each a choice where the paper is silent) are:
 *   pages : per layer l a base pointer; a run of D*e bytes for (plane p, block b,
 *           in-block offset o, head h) starts at
 *             layer[l] + p*plane_stride + b*block_stride + o*token_stride + h*head_stride
 *   chunk : [L][P][CT][H][D] elements, dense, layer-major
 *   slot  : one int64 per token, slot = b*BS + o; a negative slot means "no page":
 *           gather writes zeros for it, scatter writes nothing for it
 *   hash  : FNV-1a 64 over LE64(previous hash) followed by the chunk's CT tokens as
 *           LE32, chained from a seed; only full chunks are hashed
 *   pool  : fixed-size slots of one chunk each, lowest free slot first
 *   evict : off by default (a full pool refuses new chunks); when switched on, least
 *           recently used with the tail of a request going before its head (see the
 *           comment at orc_store_set_evict)
 *
 * Parity pins (tests/test_oracle_*.py): coordinate stamping closed form, identity
 * mapping == memcpy, store/retrieve round trip, untouched-byte sentinel, brute force
 * over every injective mapping on a tiny shape, numpy take / indexed assignment as a
 * library third opinion, published FNV-1a vectors, the prefix property of the chain,
 * a model check of the store against a dict of bytes, and for eviction the textbook
 * LRU cache (ordered dict) in the one-chunk-per-call case, a hand-worked sequence and
 * invariants on random sequences.  The paper prints no
 * values for this path, so parity against printed values is unpinned; the pins
 * above fix the definitions taken.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    ORC_OK = 0,
    ORC_INVAL = -1,
    ORC_NOMEM = -2,
    ORC_MISS = -3,
    ORC_BADSLOT = -4,
    ORC_BUSY = -6
};

typedef struct {
    int32_t L;   /* layers */
    int32_t P;   /* planes: 2 = K and V, 1 = one latent */
    int32_t H;   /* KV heads */
    int32_t D;   /* head dim, elements */
    int32_t e;   /* bytes per element */
    int32_t BS;  /* tokens per page (block) */
    int32_t NB;  /* blocks in the engine's pool */
    int32_t CT;  /* tokens per chunk */
    int64_t plane_stride, block_stride, token_stride, head_stride; /* bytes */
} orc_geom_t;

int64_t orc_chunk_bytes(const orc_geom_t *g)
{
    return (int64_t)g->L * g->P * g->CT * g->H * g->D * g->e;
}

/* byte offset inside a chunk of the run (l, p, t, h) */
static int64_t chunk_off(const orc_geom_t *g, int l, int p, int t, int h)
{
    int64_t run = (int64_t)g->D * g->e;
    return ((((int64_t)l * g->P + p) * g->CT + t) * g->H + h) * run;
}

/* byte offset inside layer l's allocation of the run (p, b, o, h) */
static int64_t page_off(const orc_geom_t *g, int p, int64_t b, int64_t o, int h)
{
    return (int64_t)p * g->plane_stride + b * g->block_stride + o * g->token_stride +
           (int64_t)h * g->head_stride;
}

/* every slot is either negative (skip) or below NB*BS */
int orc_check_slots(const orc_geom_t *g, const int64_t *slot, int64_t n)
{
    int64_t limit = (int64_t)g->NB * g->BS;
    for (int64_t i = 0; i < n; i++)
        if (slot[i] >= limit) return ORC_BADSLOT;
    return ORC_OK;
}

/* Store direction, one chunk: pages -> contiguous chunk (section 5.1). */
int orc_gather_chunk(const orc_geom_t *g, const uint8_t *const *layers, const int64_t *slot,
                     uint8_t *chunk)
{
    size_t run = (size_t)g->D * g->e;
    if (orc_check_slots(g, slot, g->CT) != ORC_OK) return ORC_BADSLOT;
    for (int l = 0; l < g->L; l++)
        for (int p = 0; p < g->P; p++)
            for (int t = 0; t < g->CT; t++)
                for (int h = 0; h < g->H; h++) {
                    uint8_t *dst = chunk + chunk_off(g, l, p, t, h);
                    int64_t s = slot[t];
                    if (s < 0) {
                        memset(dst, 0, run);
                    } else {
                        memcpy(dst, layers[l] + page_off(g, p, s / g->BS, s % g->BS, h), run);
                    }
                }
    return ORC_OK;
}

/* Retrieve direction, one chunk: contiguous chunk -> pages (section 5.1).
 * Tokens are taken in order, so for a repeated slot the last token wins. */
int orc_scatter_chunk(const orc_geom_t *g, const uint8_t *chunk, const int64_t *slot,
                      uint8_t *const *layers)
{
    size_t run = (size_t)g->D * g->e;
    if (orc_check_slots(g, slot, g->CT) != ORC_OK) return ORC_BADSLOT;
    for (int l = 0; l < g->L; l++)
        for (int p = 0; p < g->P; p++)
            for (int t = 0; t < g->CT; t++)
                for (int h = 0; h < g->H; h++) {
                    int64_t s = slot[t];
                    if (s < 0) continue;
                    memcpy(layers[l] + page_off(g, p, s / g->BS, s % g->BS, h),
                           chunk + chunk_off(g, l, p, t, h), run);
                }
    return ORC_OK;
}

/* ---- chunk identity: chained FNV-1a 64 (token processor, section 4) ---- */

uint64_t orc_fnv1a64(const uint8_t *bytes, int64_t n)
{
    uint64_t h = 0xcbf29ce484222325ULL;
    for (int64_t i = 0; i < n; i++) {
        h ^= bytes[i];
        h *= 0x100000001b3ULL;
    }
    return h;
}

/* hashes_out[i] identifies tokens[0 .. (i+1)*CT): it depends on every earlier chunk.
 * Returns the number of full chunks; a tail shorter than CT is ignored. */
int64_t orc_hash_chunks(uint64_t seed, int32_t CT, const int32_t *tokens, int64_t n_tokens,
                        uint64_t *hashes_out)
{
    int64_t n_chunks = n_tokens / CT;
    size_t len = 8 + 4 * (size_t)CT;
    uint8_t *msg = (uint8_t *)malloc(len);
    uint64_t prev = seed;
    for (int64_t i = 0; i < n_chunks; i++) {
        for (int k = 0; k < 8; k++) msg[k] = (uint8_t)(prev >> (8 * k));
        for (int t = 0; t < CT; t++) {
            uint32_t v = (uint32_t)tokens[i * CT + t];
            for (int k = 0; k < 4; k++) msg[8 + 4 * t + k] = (uint8_t)(v >> (8 * k));
        }
        prev = orc_fnv1a64(msg, (int64_t)len);
        hashes_out[i] = prev;
    }
    free(msg);
    return n_chunks;
}

/* ---- the CPU-memory chunk store: pool + index (storage manager, section 4) ---- */

typedef struct {
    orc_geom_t g;
    int64_t n_slots;
    int64_t chunk_bytes;
    uint8_t *pool;      /* n_slots * chunk_bytes */
    uint8_t *used;      /* per slot: 0 free, 1 holds a chunk */
    uint64_t *key;      /* per slot: the chunk's hash when used */
    int32_t *pins;      /* per slot: pin count */
    int32_t *refs;      /* per slot: transfers that are reading the chunk's bytes in place */
    /* optional eviction (off unless orc_store_set_evict): recency of use per slot.
     * Every store or retrieve call takes the next call number; a chunk it uses gets
     * (that number, its position in the call's chunk list). */
    int evict;
    uint64_t calls;      /* number of the latest store / retrieve call */
    uint64_t *use_call;  /* per slot: number of the last call that used the chunk */
    int64_t *use_pos;    /* per slot: first position of the chunk in that call */
    uint64_t *evicted;   /* hashes evicted since the log was last drained */
    int64_t n_evicted, cap_evicted;
} orc_store_t;

orc_store_t *orc_store_new(const orc_geom_t *g, int64_t n_slots)
{
    orc_store_t *s = (orc_store_t *)calloc(1, sizeof *s);
    if (!s) return NULL;
    s->g = *g;
    s->n_slots = n_slots;
    s->chunk_bytes = orc_chunk_bytes(g);
    s->pool = (uint8_t *)calloc((size_t)n_slots, (size_t)s->chunk_bytes);
    s->used = (uint8_t *)calloc((size_t)n_slots, 1);
    s->key = (uint64_t *)calloc((size_t)n_slots, sizeof(uint64_t));
    s->pins = (int32_t *)calloc((size_t)n_slots, sizeof(int32_t));
    s->refs = (int32_t *)calloc((size_t)n_slots, sizeof(int32_t));
    s->use_call = (uint64_t *)calloc((size_t)n_slots, sizeof(uint64_t));
    s->use_pos = (int64_t *)calloc((size_t)n_slots, sizeof(int64_t));
    return s;
}

void orc_store_free(orc_store_t *s)
{
    if (!s) return;
    free(s->pool); free(s->used); free(s->key); free(s->pins); free(s->refs);
    free(s->use_call); free(s->use_pos); free(s->evicted); free(s);
}

/* slot holding hash h, or -1 */
int64_t orc_store_find(const orc_store_t *s, uint64_t h)
{
    for (int64_t i = 0; i < s->n_slots; i++)
        if (s->used[i] && s->key[i] == h) return i;
    return -1;
}

const uint8_t *orc_store_slot_ptr(const orc_store_t *s, int64_t slot)
{
    return s->pool + slot * s->chunk_bytes;
}

int64_t orc_store_used(const orc_store_t *s)
{
    int64_t n = 0;
    for (int64_t i = 0; i < s->n_slots; i++) n += s->used[i];
    return n;
}

/* number of leading hashes that are all present: a later isolated hit does not count */
int64_t orc_lookup(const orc_store_t *s, const uint64_t *hashes, int64_t n)
{
    int64_t k = 0;
    while (k < n && orc_store_find(s, hashes[k]) >= 0) k++;
    return k;
}

/* ---- eviction (the paper says that instances store and evict, sections 4.2 and 7,
 * but names no policy; the reading taken here is least recently used, refined for
 * prefix caches) ----
 *
 * Recency: a chunk used by call number c at position i of the call's chunk list is
 * "(c, i)".  Chunk A is older than chunk B if A's call is earlier, or, within one call,
 * if A's position is LATER: the tail of a request goes before its head, because a
 * lookup counts only the leading run of present chunks, so a request that lost its
 * tail still hits on what remains while one that lost its head hits on nothing.
 * The victim is the oldest chunk that is not pinned and was not used by the call that
 * needs the room (a call never evicts what it is itself storing or has just found). */
void orc_store_set_evict(orc_store_t *s, int on) { s->evict = on; }

/* writes up to cap evicted hashes, oldest eviction first, and forgets them */
int64_t orc_store_drain_evicted(orc_store_t *s, uint64_t *out, int64_t cap)
{
    int64_t n = s->n_evicted < cap ? s->n_evicted : cap;
    for (int64_t i = 0; i < n; i++) out[i] = s->evicted[i];
    for (int64_t i = n; i < s->n_evicted; i++) s->evicted[i - n] = s->evicted[i];
    s->n_evicted -= n;
    return n;
}

static int64_t pick_victim(const orc_store_t *s)
{
    int64_t v = -1;
    for (int64_t f = 0; f < s->n_slots; f++) {
        if (!s->used[f] || s->pins[f] > 0 || s->refs[f] > 0 || s->use_call[f] == s->calls) continue;
        if (v < 0 || s->use_call[f] < s->use_call[v] ||
            (s->use_call[f] == s->use_call[v] && s->use_pos[f] > s->use_pos[v]))
            v = f;
    }
    return v;
}

static void evict_slot(orc_store_t *s, int64_t v)
{
    if (s->n_evicted == s->cap_evicted) {
        s->cap_evicted = s->cap_evicted ? 2 * s->cap_evicted : 64;
        s->evicted = (uint64_t *)realloc(s->evicted, (size_t)s->cap_evicted * sizeof(uint64_t));
    }
    s->evicted[s->n_evicted++] = s->key[v];
    s->used[v] = 0;
}

/* the chunks of the current call that are present get this call's number ... */
static void mark_call(orc_store_t *s, const uint64_t *hashes, int64_t n)
{
    for (int64_t i = 0; i < n; i++) {
        int64_t f = orc_store_find(s, hashes[i]);
        if (f >= 0) s->use_call[f] = s->calls;
    }
}

/* ... and, when the call ends, their first position in it */
static void mark_positions(orc_store_t *s, const uint64_t *hashes, int64_t n)
{
    for (int64_t i = n - 1; i >= 0; i--) {
        int64_t f = orc_store_find(s, hashes[i]);
        if (f >= 0) s->use_pos[f] = i;
    }
}

/* Store chunks in order.  A chunk already present is left as it is (only new tokens
 * are stored, section 4 "Store").  A new chunk takes the lowest free slot.  With no
 * free slot, and with eviction on, the oldest evictable chunk gives up its slot; if
 * there is none, or eviction is off, the call stops with ORC_NOMEM and everything
 * stored before stays.  n_new_out counts chunks actually written. */
int orc_store(orc_store_t *s, const uint8_t *const *layers, const int64_t *slot_mapping,
              const uint64_t *hashes, int64_t n_chunks, int64_t *n_new_out)
{
    int64_t n_new = 0;
    int rc = ORC_OK;
    if (n_new_out) *n_new_out = 0;
    if (orc_check_slots(&s->g, slot_mapping, n_chunks * s->g.CT) != ORC_OK) return ORC_BADSLOT;
    s->calls++;
    mark_call(s, hashes, n_chunks);   /* what the call finds present is safe from it */
    for (int64_t i = 0; i < n_chunks; i++) {
        if (orc_store_find(s, hashes[i]) >= 0) continue;
        int64_t f = 0;
        while (f < s->n_slots && s->used[f]) f++;
        if (f == s->n_slots && s->evict) {
            f = pick_victim(s);
            if (f >= 0) evict_slot(s, f); else f = s->n_slots;
        }
        if (f == s->n_slots) {
            rc = ORC_NOMEM;
            break;
        }
        orc_gather_chunk(&s->g, layers, slot_mapping + i * s->g.CT, s->pool + f * s->chunk_bytes);
        s->used[f] = 1;
        s->key[f] = hashes[i];
        s->pins[f] = 0;
        s->refs[f] = 0;
        s->use_call[f] = s->calls;
        n_new++;
    }
    mark_positions(s, hashes, n_chunks);
    if (n_new_out) *n_new_out = n_new;
    return rc;
}

static void scatter_all(const orc_store_t *s, const uint64_t *hashes, int64_t n_chunks,
                        const int64_t *slot_mapping, uint8_t *const *layers)
{
    for (int64_t i = 0; i < n_chunks; i++) {
        int64_t f = orc_store_find(s, hashes[i]);
        orc_scatter_chunk(&s->g, s->pool + f * s->chunk_bytes, slot_mapping + i * s->g.CT, layers);
    }
}

/* All chunks must be present, else ORC_MISS and no page byte changes (and no chunk
 * counts as used). */
int orc_retrieve(orc_store_t *s, const uint64_t *hashes, int64_t n_chunks,
                 const int64_t *slot_mapping, uint8_t *const *layers)
{
    if (orc_check_slots(&s->g, slot_mapping, n_chunks * s->g.CT) != ORC_OK) return ORC_BADSLOT;
    for (int64_t i = 0; i < n_chunks; i++)
        if (orc_store_find(s, hashes[i]) < 0) return ORC_MISS;
    scatter_all(s, hashes, n_chunks, slot_mapping, layers);
    s->calls++;
    mark_call(s, hashes, n_chunks);
    mark_positions(s, hashes, n_chunks);
    return ORC_OK;
}

/* Many requests at once: request r owns chunks [off[r], off[r+1]) of hashes and of the
 * slot mapping.  One missing chunk anywhere means nothing is written.  For recency the
 * batch is one call and a chunk's position is its place in the concatenated list. */
int orc_retrieve_batch(orc_store_t *s, int64_t n_req, const int64_t *req_chunk_offsets,
                       const uint64_t *hashes, const int64_t *slot_mapping,
                       uint8_t *const *layers)
{
    int64_t total = req_chunk_offsets[n_req];
    if (orc_check_slots(&s->g, slot_mapping, total * s->g.CT) != ORC_OK) return ORC_BADSLOT;
    for (int64_t i = 0; i < total; i++)
        if (orc_store_find(s, hashes[i]) < 0) return ORC_MISS;
    for (int64_t r = 0; r < n_req; r++) {
        int64_t a = req_chunk_offsets[r], b = req_chunk_offsets[r + 1];
        scatter_all(s, hashes + a, b - a, slot_mapping + a * s->g.CT, layers);
    }
    s->calls++;
    mark_call(s, hashes, total);
    mark_positions(s, hashes, total);
    return ORC_OK;
}

/* pin / unpin / clear: local forms of the controller verbs (section 7, Table 3).
 * pin: every hash must be present, else ORC_MISS and no count changes.
 * unpin: every hash must be present (else ORC_MISS) and hold enough pins (else
 *        ORC_INVAL); on either error no count changes.
 * clear: absent hashes are ignored; a pinned one makes the call ORC_BUSY and nothing
 *        is removed. */
int orc_pin(orc_store_t *s, const uint64_t *hashes, int64_t n)
{
    for (int64_t i = 0; i < n; i++)
        if (orc_store_find(s, hashes[i]) < 0) return ORC_MISS;
    for (int64_t i = 0; i < n; i++) s->pins[orc_store_find(s, hashes[i])]++;
    return ORC_OK;
}

int orc_unpin(orc_store_t *s, const uint64_t *hashes, int64_t n)
{
    for (int64_t i = 0; i < n; i++)
        if (orc_store_find(s, hashes[i]) < 0) return ORC_MISS;
    /* a hash listed k times needs a count of at least k */
    for (int64_t i = 0; i < n; i++) {
        int64_t times = 0;
        for (int64_t j = 0; j < n; j++) times += (hashes[j] == hashes[i]);
        if (s->pins[orc_store_find(s, hashes[i])] < times) return ORC_INVAL;
    }
    for (int64_t i = 0; i < n; i++) s->pins[orc_store_find(s, hashes[i])]--;
    return ORC_OK;
}

int orc_clear(orc_store_t *s, const uint64_t *hashes, int64_t n)
{
    for (int64_t i = 0; i < n; i++) {
        int64_t f = orc_store_find(s, hashes[i]);
        if (f >= 0 && (s->pins[f] > 0 || s->refs[f] > 0)) return ORC_BUSY;
    }
    for (int64_t i = 0; i < n; i++) {
        int64_t f = orc_store_find(s, hashes[i]);
        if (f >= 0) s->used[f] = 0;
    }
    return ORC_OK;
}

/* The reference counter of section 5.3 "Zero-Copy Operations": a transfer that sends a
 * chunk somewhere else (a write to disk, to a remote store, ...) does not copy it first;
 * it raises the chunk's counter, reads the bytes where they are, and lowers the counter
 * when it completes.  Several transfers of the same chunk at once, e.g. to two
 * destinations, each hold their own count.  While the counter is above zero the chunk
 * keeps its slot: clear answers ORC_BUSY (above) and eviction passes it over.
 * acquire: ORC_MISS if the chunk is absent.  release: ORC_MISS if absent, ORC_INVAL if
 * the counter is already zero. */
int orc_acquire(orc_store_t *s, uint64_t h)
{
    int64_t f = orc_store_find(s, h);
    if (f < 0) return ORC_MISS;
    s->refs[f]++;
    return ORC_OK;
}

int orc_release(orc_store_t *s, uint64_t h)
{
    int64_t f = orc_store_find(s, h);
    if (f < 0) return ORC_MISS;
    if (s->refs[f] == 0) return ORC_INVAL;
    s->refs[f]--;
    return ORC_OK;
}

int32_t orc_refs(const orc_store_t *s, uint64_t h)
{
    int64_t f = orc_store_find(s, h);
    return f < 0 ? -1 : s->refs[f];
}
