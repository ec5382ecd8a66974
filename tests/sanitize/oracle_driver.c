/*
 * Sanitizer driver for the CPU oracle: built together with oracle/zipccl_oracle.c under
 * -fsanitize=address,undefined and run by tests/test_sanitizers.py.  It exercises the encoder, the decoder
 * (good, corrupt and truncated streams) and the decode-and-reduce on host buffers that are exactly as large as
 * the interface promises, so that any access outside them, any misaligned or overflowing arithmetic aborts the run.
 * Exit status 0 = every check passed and no sanitizer report.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint64_t zo_slot_cap(uint64_t n, int dtype, uint32_t G);
int zo_build_table(double sigma, uint8_t dec[8]);
int zo_slot_offsets(uint64_t n_elems, int dtype, uint32_t G, uint32_t n_chunks, const uint64_t* chunk_elems, uint64_t* slot_off);
int zo_compress(const void* in, uint64_t n_elems, int dtype, uint32_t G, uint32_t n_chunks, const uint64_t* chunk_elems,
                const uint8_t dec[8], void* out, uint64_t out_capacity, uint64_t* chunk_bytes);
int zo_decompress(const void* comp, uint64_t comp_capacity, void* out, uint64_t n_elems, int dtype, uint32_t n_chunks,
                  const uint64_t* chunk_elems);
int zo_decompress_reduce(const void* comp, uint64_t comp_capacity, void* out, uint64_t n, int dtype, uint32_t n_peers,
                         int out_dtype, void* scratch, float* acc);

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); exit(1); } } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 16);
}

/* round trip of n elements in the given split; buffers sized exactly */
static void round_trip(const void* data, uint64_t n, int dtype, uint32_t G, uint32_t n_chunks, const uint64_t* ce, double sigma)
{
    const size_t es = dtype == 0 ? 2 : 4;
    uint8_t dec[8];
    CHECK(zo_build_table(sigma, dec) == 0);
    uint64_t* off = malloc((n_chunks + 1) * sizeof *off);
    uint64_t* cb = malloc(n_chunks * sizeof *cb);
    CHECK(zo_slot_offsets(n, dtype, G, n_chunks, ce, off) == 0);
    uint8_t* comp = malloc(off[n_chunks] ? off[n_chunks] : 1);
    CHECK(zo_compress(data, n, dtype, G, n_chunks, ce, dec, comp, off[n_chunks], cb) == 0);
    CHECK(zo_compress(data, n, dtype, G, n_chunks, ce, dec, comp, off[n_chunks] - 1, cb) == 3);   /* one byte short */
    uint8_t* back = malloc(n ? n * es : 1);
    CHECK(zo_decompress(comp, off[n_chunks], back, n, dtype, n_chunks, ce) == 0);
    CHECK(memcmp(back, data, n * es) == 0);
    /* what a collective transmits for the last chunk is enough to decode it: capacity cut to its chunk_bytes */
    CHECK(zo_decompress(comp, off[n_chunks - 1] + cb[n_chunks - 1], back, n, dtype, n_chunks, ce) == 0);
    /* truncated anywhere, and with any single header byte of the first slot damaged: an error code or (for bytes
       the format does not define) a clean decode, never an access outside the buffers */
    for (uint64_t cut = 0; cut < off[n_chunks]; cut += 1 + off[n_chunks] / 97) {
        uint8_t* part = malloc(cut ? cut : 1);
        memcpy(part, comp, cut);
        (void)zo_decompress(part, cut, back, n, dtype, n_chunks, ce);
        free(part);
    }
    for (int b = 0; b < 128; ++b) {
        const uint8_t keep = comp[b];
        comp[b] ^= (uint8_t)(1u << (b & 7));
        (void)zo_decompress(comp, off[n_chunks], back, n, dtype, n_chunks, ce);
        comp[b] = 0xFF;
        (void)zo_decompress(comp, off[n_chunks], back, n, dtype, n_chunks, ce);
        comp[b] = keep;
    }
    /* damaged bytes anywhere in the buffer (headers of later slots, sections, index, lists) */
    if (n) {
        for (int k = 0; k < 300; ++k) {
            const uint64_t at = rnd() % off[n_chunks];
            const uint8_t keep = comp[at];
            comp[at] ^= (uint8_t)(1u + rnd() % 255);
            (void)zo_decompress(comp, off[n_chunks], back, n, dtype, n_chunks, ce);
            comp[at] = keep;
        }
    }
    free(back); free(comp); free(cb); free(off);
}

int main(void)
{
    /* every bf16 pattern, as one tensor, for two group sizes and an odd split */
    uint16_t* all = malloc(65536 * 2);
    for (uint32_t i = 0; i < 65536; ++i) all[i] = (uint16_t)i;
    round_trip(all, 65536, 0, 512, 1, NULL, 1.0);
    round_trip(all, 65536, 0, 8, 4, NULL, 0.02);
    const uint64_t ragged[6] = {0, 1, 511, 8193, 0, 65536 - 1 - 511 - 8193};
    round_trip(all, 65536, 0, 512, 6, ragged, 1e-4);
    round_trip(all, 0, 0, 512, 1, NULL, 1.0);                       /* nothing */
    round_trip(all, 7, 0, 1, 1, NULL, 1.0);                         /* G = 1 */

    /* random fp32 bit patterns */
    uint32_t* w = malloc(30011 * 4);
    for (int i = 0; i < 30011; ++i) w[i] = rnd() ^ (rnd() << 16);
    const uint64_t split3[3] = {10000, 1, 20010};
    round_trip(w, 30011, 1, 512, 3, split3, 0.5);

    /* argument errors */
    uint8_t dec[8], small[64];
    CHECK(zo_build_table(0.0, dec) == 1 && zo_build_table(-1.0, dec) == 1);
    CHECK(zo_build_table(1e-300, dec) == 0 && dec[1] == 1);
    CHECK(zo_build_table(1e300, dec) == 0 && dec[7] == 254);
    CHECK(zo_compress(all, 10, 7, 512, 1, NULL, dec, small, sizeof small, NULL) == 2);
    CHECK(zo_compress(all, 10, 0, 512, 3, NULL, dec, small, sizeof small, NULL) == 1);
    CHECK(zo_decompress(small, 0, all, 0, 0, 1, NULL) != 0);

    /* decode-and-reduce of three peers, both output types, exact-size buffers; then a damaged second slot */
    const uint64_t n = 5000;
    uint8_t d2[8];
    CHECK(zo_build_table(1.0, d2) == 0);
    const uint64_t cap1 = zo_slot_cap(n, 0, 512);
    uint8_t* rb = malloc(3 * cap1);
    CHECK(zo_compress(all + 100, 3 * n, 0, 512, 3, NULL, d2, rb, 3 * cap1, NULL) == 0);
    uint32_t* sums = malloc(n * 4);
    uint16_t* sums16 = malloc(n * 2);
    uint16_t* scratch = malloc(n * 2);
    float* acc = malloc(n * 4);
    CHECK(zo_decompress_reduce(rb, 3 * cap1, sums, n, 0, 3, 1, scratch, acc) == 0);
    CHECK(zo_decompress_reduce(rb, 3 * cap1, sums16, n, 0, 3, 0, scratch, acc) == 0);
    rb[cap1] ^= 1;
    CHECK(zo_decompress_reduce(rb, 3 * cap1, sums, n, 0, 3, 1, scratch, acc) == 4);
    CHECK(zo_decompress_reduce(rb, 2 * cap1, sums, n, 0, 3, 1, scratch, acc) != 0);      /* third slot not there */
    free(acc); free(scratch); free(sums16); free(sums); free(rb); free(w); free(all);
    puts("oracle sanitizer driver: ok");
    return 0;
}
