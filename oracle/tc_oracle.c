/*
 * CPU oracle for paged-KV offload / upload.  TEST INFRASTRUCTURE ONLY.
 *
 * Nothing in the product library may include, link or call this file; only the
 * test-suite, the smoke check and the benchmark's CPU-baseline leg use it.  It
 * shares no code with the HIP path: the index arithmetic below is written out
 * on its own, single-threaded, with one memcpy per page.
 *
 * What it defines (paper Sec. 6.3 "CPU Migration Infrastructure": KV migrates
 * between GPU blocks and CPU blocks, the pool owns the GPU<->CPU block mapping
 * and puts the GPU mapping back on upload; Sec. 7.6: a block holds block_size
 * tokens of every layer's K and V, e.g. 48 layers x {K,V} x 8 heads x 128 x
 * 16 tokens x 2 B = 3 MiB; Table 2: the Temporal Scheduler works at block
 * granularity).  The paper fixes no memory layout, so the layouts are this
 * build's reading:
 *
 *   planes      P = 2 * L                     plane p = 2*layer + kv (kv 0 = K, 1 = V)
 *   device pool pool[p][block][byte]          P x NB x pb bytes, plane-major
 *   scales      scales[s][block]              S x NB 32-bit words, S in {0, 1, P}
 *   host record rec = roundup256(P*pb + 4*S)  one contiguous record per moved block:
 *               [page 0 | page 1 | ... | page P-1 | S scale words | zero pad]
 *
 *   offload:  host[j*rec + p*pb + b]        = pool[(p*NB + ids[j])*pb + b]
 *             word(host, j*rec + P*pb)[s]   = scales[s*NB + ids[j]]
 *             pad bytes of the record       = 0
 *   upload:   the inverse copy with new_ids (pad ignored), then
 *             table_row[i] = new_ids[i]  for i < n
 *
 * Bytes are opaque: no value is interpreted, so NaN payloads and -0 survive.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define TCO_OK 0
#define TCO_BAD_ID (-1)
#define TCO_BAD_SHAPE (-2)

static int shape_ok(uint32_t L, uint64_t NB, uint64_t pb, uint32_t S)
{
    if (L == 0 || NB == 0 || pb == 0) return 0;
    if (S != 0 && S != 1 && S != 2 * L) return 0;
    return 1;
}

/* Host bytes per moved block (Sec. 7.6 size formula, plus this layout's scale words and pad). */
uint64_t tco_record_bytes(uint32_t L, uint64_t pb, uint32_t S)
{
    uint64_t raw = (uint64_t)2 * L * pb + (uint64_t)4 * S;
    return (raw + 255u) / 256u * 256u;
}

/* Bytes of one page: block_size tokens x kv heads x head_dim x element bytes (Sec. 7.6). */
uint64_t tco_page_bytes(uint32_t block_size, uint32_t kv_heads, uint32_t head_dim, uint32_t elem_bytes)
{
    return (uint64_t)block_size * kv_heads * head_dim * elem_bytes;
}

/* Blocks that hold `tokens` tokens: 1 024..5 120 tokens = 64..320 blocks of 16 (Sec. 7.6). */
uint64_t tco_blocks_for_tokens(uint64_t tokens, uint32_t block_size)
{
    return (tokens + block_size - 1) / block_size;
}

int tco_offload(const uint8_t *pool, const uint32_t *scales,
                uint32_t L, uint64_t NB, uint64_t pb, uint32_t S,
                const int32_t *ids, uint64_t n, uint8_t *host)
{
    if (!shape_ok(L, NB, pb, S)) return TCO_BAD_SHAPE;
    const uint64_t P = (uint64_t)2 * L;
    const uint64_t rec = tco_record_bytes(L, pb, S);
    for (uint64_t j = 0; j < n; ++j)
        if (ids[j] < 0 || (uint64_t)ids[j] >= NB) return TCO_BAD_ID;

    for (uint64_t j = 0; j < n; ++j) {
        const uint64_t blk = (uint64_t)ids[j];
        uint8_t *record = host + j * rec;
        for (uint64_t p = 0; p < P; ++p)
            memcpy(record + p * pb, pool + (p * NB + blk) * pb, pb);
        uint64_t at = P * pb;
        for (uint32_t s = 0; s < S; ++s) {
            uint32_t w = scales[(uint64_t)s * NB + blk];
            memcpy(record + at, &w, 4);
            at += 4;
        }
        while (at < rec) record[at++] = 0;
    }
    return TCO_OK;
}

int tco_upload(const uint8_t *host,
               uint32_t L, uint64_t NB, uint64_t pb, uint32_t S,
               const int32_t *new_ids, uint64_t n,
               uint8_t *pool, uint32_t *scales, int32_t *table_row)
{
    if (!shape_ok(L, NB, pb, S)) return TCO_BAD_SHAPE;
    const uint64_t P = (uint64_t)2 * L;
    const uint64_t rec = tco_record_bytes(L, pb, S);
    for (uint64_t i = 0; i < n; ++i)
        if (new_ids[i] < 0 || (uint64_t)new_ids[i] >= NB) return TCO_BAD_ID;

    for (uint64_t i = 0; i < n; ++i) {
        const uint64_t blk = (uint64_t)new_ids[i];
        const uint8_t *record = host + i * rec;
        for (uint64_t p = 0; p < P; ++p)
            memcpy(pool + (p * NB + blk) * pb, record + p * pb, pb);
        for (uint32_t s = 0; s < S; ++s) {
            uint32_t w;
            memcpy(&w, record + P * pb + (uint64_t)4 * s, 4);
            scales[(uint64_t)s * NB + blk] = w;
        }
    }
    if (table_row)
        for (uint64_t i = 0; i < n; ++i) table_row[i] = new_ids[i];
    return TCO_OK;
}

/*
 * Bytes of logical token t of one agent in plane (layer, kv), read through the
 * agent's block table: block table[t / block_size], slot t % block_size, each
 * slot pb / block_size bytes ([block_size][kv_heads][head_dim] inside a page).
 * Used to state that a table rewritten by an upload still addresses the same logical tokens.
 */
int tco_read_token(const uint8_t *pool, uint32_t L, uint64_t NB, uint64_t pb,
                   uint32_t block_size, const int32_t *table, uint64_t t,
                   uint32_t layer, uint32_t kv, uint8_t *out)
{
    if (!shape_ok(L, NB, pb, 0) || block_size == 0 || pb % block_size) return TCO_BAD_SHAPE;
    if (layer >= L || kv > 1) return TCO_BAD_SHAPE;
    const int32_t id = table[t / block_size];
    if (id < 0 || (uint64_t)id >= NB) return TCO_BAD_ID;
    const uint64_t tok = pb / block_size;
    const uint64_t p = (uint64_t)2 * layer + kv;
    memcpy(out, pool + (p * NB + (uint64_t)id) * pb + (t % block_size) * tok, tok);
    return TCO_OK;
}
