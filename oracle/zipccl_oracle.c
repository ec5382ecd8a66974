/*
 * zipccl_oracle.c -- plain, slow, scalar CPU reference for the ZipCCL exponent-coding
 * format (paper section 4, "Communication-Aware Lossless Compression and Decompression").
 *
 * THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or helper with the
 * HIP library; the product path never routes through it.
 *
 * What it computes (one element at a time, in element order, no blocking or fusion):
 *   - zo_build_table : section 4.1, Eq.2 and Eq.5 -- the 7-exponent window for a
 *     zero-mean Gaussian of standard deviation sigma.
 *   - zo_compress    : section 4 (second paragraph) -- split every value into
 *     sign+mantissa (kept verbatim) and exponent; exponents inside the window become a
 *     3-bit code 1..7, all others code 0 plus the raw exponent appended to the
 *     zero-point list; section 4.2.1 -- the code is stored as three 1-bit planes and every
 *     peer chunk is padded to 128 bytes; section 4.2.3 -- a per-group prefix count of
 *     zero-points is stored so a decoder can find each group's zero-points.
 *   - zo_decompress  : section 4 (third paragraph) -- the inverse.
 *   - zo_decompress_reduce : section 3.3 and section 5.2 -- the device half of the zipped
 *     Reduce-Scatter: decode the slices received from every peer and sum them locally in FP32
 *     (the paper fixes FP32 for the local reduction of BF16 traffic), in peer order.
 *
 * The byte-level layout (where the paper is silent) is the one fixed for this build:
 * little-endian; per chunk a slot of
 *   HDR(128) | SM pad(n) | [LO pad(2n), fp32 only] | P0 | P1 | P2 (each pad(ceil(n/8)))
 *   | IDX pad(4*ceil(n/G)) | ESC (pad(n_esc) used, pad(n) reserved)
 * with pad(x) = x rounded up to 128.  Parity of the layout choices themselves is
 * "unpinned by the paper"; they are pinned by the hand-worked example and the
 * brute-force / independent-decoder tests.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ZO_OK 0
#define ZO_ERR_ARG 1
#define ZO_ERR_DTYPE 2
#define ZO_ERR_SMALL 3
#define ZO_ERR_CORRUPT 4

#define ZO_BF16 0
#define ZO_FP32 1

static uint64_t zo_pad(uint64_t x) { return (x + 127u) / 128u * 128u; }
static uint64_t zo_ceil_div(uint64_t a, uint64_t b) { return (a + b - 1u) / b; }

static void put32(uint8_t* p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static void put64(uint8_t* p, uint64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static uint32_t get32(const uint8_t* p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }
static uint64_t get64(const uint8_t* p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return v; }

/* Eq.2: probability that |w|, w ~ N(0, sigma^2), lies in [2^x, 2^(x+7)). */
double zo_pwin(double sigma, int x)
{
    const double s = sigma * sqrt(2.0);
    return erf(ldexp(1.0, x + 7) / s) - erf(ldexp(1.0, x) / s);
}

/* Eq.5: continuous optimum of the window base for a given sigma. */
double zo_xopt(double sigma)
{
    return log2(sigma) + 0.5 * log2(14.0 * log(2.0) / 16383.0);
}

/*
 * Section 4.1.  The paper treats x as continuous and does not say how to discretise:
 * take the better of floor/ceil of Eq.5 under Eq.2, the lower one on a tie.
 * dec[0] is unused (code 0 is the zero-point flag); dec[1..7] are biased exponents.
 */
int zo_build_table(double sigma, uint8_t dec[8])
{
    if (!(sigma > 0.0) || isinf(sigma) || isnan(sigma)) return ZO_ERR_ARG;
    const double xo = zo_xopt(sigma);
    int xl = (int)floor(xo), xh = (int)ceil(xo);
    int x = (zo_pwin(sigma, xh) > zo_pwin(sigma, xl)) ? xh : xl;
    int e0 = x + 127;
    if (e0 < 1) e0 = 1;
    if (e0 > 248) e0 = 248;
    dec[0] = 0;
    for (int k = 1; k <= 7; ++k) dec[k] = (uint8_t)(e0 + k - 1);
    return ZO_OK;
}

static int elem_size(int dtype) { return dtype == ZO_BF16 ? 2 : dtype == ZO_FP32 ? 4 : 0; }

/* Slot capacity of a chunk of n elements: every section padded to 128 B. */
uint64_t zo_slot_cap(uint64_t n, int dtype, uint32_t G)
{
    uint64_t c = 128 + zo_pad(n);
    if (dtype == ZO_FP32) c += zo_pad(2 * n);
    c += 3 * zo_pad(zo_ceil_div(n, 8));
    c += zo_pad(4 * zo_ceil_div(n, G));
    c += zo_pad(n);
    return c;
}

/* Bytes a collective would transmit for the chunk: everything but the unused ESC reserve. */
uint64_t zo_chunk_bytes(uint64_t n, uint64_t n_esc, int dtype, uint32_t G)
{
    return zo_slot_cap(n, dtype, G) - zo_pad(n) + zo_pad(n_esc);
}

/* chunk_elems == NULL means an equal split (n_elems must divide). slot_off has n_chunks+1 entries. */
int zo_slot_offsets(uint64_t n_elems, int dtype, uint32_t G, uint32_t n_chunks,
                    const uint64_t* chunk_elems, uint64_t* slot_off)
{
    if (!elem_size(dtype)) return ZO_ERR_DTYPE;
    if (n_chunks == 0 || G == 0) return ZO_ERR_ARG;
    uint64_t total = 0, off = 0;
    if (!chunk_elems && n_elems % n_chunks) return ZO_ERR_ARG;
    for (uint32_t c = 0; c < n_chunks; ++c) {
        uint64_t n = chunk_elems ? chunk_elems[c] : n_elems / n_chunks;
        slot_off[c] = off;
        off += zo_slot_cap(n, dtype, G);
        total += n;
    }
    slot_off[n_chunks] = off;
    return total == n_elems ? ZO_OK : ZO_ERR_ARG;
}

/* Compress one chunk of n elements into its slot; returns n_esc through *n_esc_out. */
static void compress_chunk(const uint8_t* in, uint64_t n, int dtype, uint32_t G,
                           const uint8_t dec[8], uint8_t* slot, uint64_t* n_esc_out)
{
    const uint64_t cap = zo_slot_cap(n, dtype, G);
    const uint64_t plane_sz = zo_pad(zo_ceil_div(n, 8));
    uint8_t* hdr = slot;
    uint8_t* sm = hdr + 128;
    uint8_t* lo = sm + zo_pad(n);
    uint8_t* p0 = lo + (dtype == ZO_FP32 ? zo_pad(2 * n) : 0);
    uint8_t* p1 = p0 + plane_sz;
    uint8_t* p2 = p1 + plane_sz;
    uint8_t* idx = p2 + plane_sz;
    uint8_t* esc = idx + zo_pad(4 * zo_ceil_div(n, G));

    /* exponent -> code table from dec[] */
    uint8_t enc[256];
    memset(enc, 0, sizeof enc);
    for (int k = 1; k <= 7; ++k) enc[dec[k]] = (uint8_t)k;

    /* all static sections (and so all their padding) start as zero */
    memset(slot, 0, (size_t)(cap - zo_pad(n)));

    uint64_t n_esc = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i % G == 0) put32(idx + 4 * (i / G), (uint32_t)n_esc); /* zero-points before this group */
        uint32_t hi16;
        if (dtype == ZO_BF16) {
            hi16 = (uint32_t)in[2 * i] | ((uint32_t)in[2 * i + 1] << 8);
        } else {
            hi16 = (uint32_t)in[4 * i + 2] | ((uint32_t)in[4 * i + 3] << 8);
            lo[2 * i] = in[4 * i];
            lo[2 * i + 1] = in[4 * i + 1];
        }
        const uint32_t sign = (hi16 >> 15) & 1u, E = (hi16 >> 7) & 0xFFu, mant = hi16 & 0x7Fu;
        sm[i] = (uint8_t)((sign << 7) | mant);
        const uint32_t code = enc[E];
        p0[i >> 3] |= (uint8_t)(((code >> 0) & 1u) << (i & 7));
        p1[i >> 3] |= (uint8_t)(((code >> 1) & 1u) << (i & 7));
        p2[i >> 3] |= (uint8_t)(((code >> 2) & 1u) << (i & 7));
        if (code == 0) esc[n_esc++] = (uint8_t)E;
    }
    for (uint64_t j = n_esc; j < zo_pad(n_esc); ++j) esc[j] = 0;

    memcpy(hdr, "ZPCL", 4);
    put32(hdr + 4, 1u);
    put32(hdr + 8, (uint32_t)dtype);
    put32(hdr + 12, G);
    put64(hdr + 16, n);
    put64(hdr + 24, n_esc);
    put64(hdr + 32, zo_chunk_bytes(n, n_esc, dtype, G));
    memcpy(hdr + 40, dec, 8);
    *n_esc_out = n_esc;
}

/*
 * Compress n_elems values (host pointers) into n_chunks independent slots.
 * chunk_bytes (n_chunks entries, may be NULL) receives the transmitted size of each chunk.
 */
int zo_compress(const void* in, uint64_t n_elems, int dtype, uint32_t G, uint32_t n_chunks,
                const uint64_t* chunk_elems, const uint8_t dec[8],
                void* out, uint64_t out_capacity, uint64_t* chunk_bytes)
{
    const int es = elem_size(dtype);
    if (!es) return ZO_ERR_DTYPE;
    if (n_chunks == 0 || G == 0 || !dec || !out || (!in && n_elems)) return ZO_ERR_ARG;
    for (int a = 1; a <= 7; ++a)
        for (int b = a + 1; b <= 7; ++b)
            if (dec[a] == dec[b]) return ZO_ERR_ARG;
    if (!chunk_elems && n_elems % n_chunks) return ZO_ERR_ARG;
    uint64_t total = 0, need = 0;
    for (uint32_t c = 0; c < n_chunks; ++c) {
        uint64_t n = chunk_elems ? chunk_elems[c] : n_elems / n_chunks;
        if (n > 0xFFFFFFFFull) return ZO_ERR_ARG; /* IDX entries are u32 */
        total += n;
        need += zo_slot_cap(n, dtype, G);
    }
    if (total != n_elems) return ZO_ERR_ARG;
    if (need > out_capacity) return ZO_ERR_SMALL;

    const uint8_t* src = (const uint8_t*)in;
    uint8_t* dst = (uint8_t*)out;
    for (uint32_t c = 0; c < n_chunks; ++c) {
        uint64_t n = chunk_elems ? chunk_elems[c] : n_elems / n_chunks;
        uint64_t n_esc = 0;
        compress_chunk(src, n, dtype, G, dec, dst, &n_esc);
        if (chunk_bytes) chunk_bytes[c] = zo_chunk_bytes(n, n_esc, dtype, G);
        src += n * (uint64_t)es;
        dst += zo_slot_cap(n, dtype, G);
    }
    return ZO_OK;
}

/* Decode one slot.  avail = bytes of the slot that may be read. */
static int decompress_chunk(const uint8_t* slot, uint64_t avail, uint64_t n, int dtype, uint8_t* out)
{
    if (avail < 128) return ZO_ERR_CORRUPT;
    if (memcmp(slot, "ZPCL", 4) != 0 || get32(slot + 4) != 1u) return ZO_ERR_CORRUPT;
    if (get32(slot + 8) != (uint32_t)dtype) return ZO_ERR_CORRUPT;
    const uint32_t G = get32(slot + 12);
    if (G == 0 || get64(slot + 16) != n) return ZO_ERR_CORRUPT;
    const uint64_t n_esc = get64(slot + 24);
    if (n_esc > n) return ZO_ERR_CORRUPT;
    const uint64_t cbytes = zo_chunk_bytes(n, n_esc, dtype, G);
    if (get64(slot + 32) != cbytes || cbytes > avail) return ZO_ERR_CORRUPT;
    uint8_t dec[8];
    memcpy(dec, slot + 40, 8);

    const uint64_t plane_sz = zo_pad(zo_ceil_div(n, 8));
    const uint8_t* sm = slot + 128;
    const uint8_t* lo = sm + zo_pad(n);
    const uint8_t* p0 = lo + (dtype == ZO_FP32 ? zo_pad(2 * n) : 0);
    const uint8_t* p1 = p0 + plane_sz;
    const uint8_t* p2 = p1 + plane_sz;
    const uint8_t* idx = p2 + plane_sz;
    const uint8_t* esc = idx + zo_pad(4 * zo_ceil_div(n, G));

    uint64_t running = 0; /* zero-points seen so far in the chunk */
    uint64_t base = 0, rank = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (i % G == 0) {
            base = get32(idx + 4 * (i / G));
            rank = 0;
            if (base != running) return ZO_ERR_CORRUPT; /* index must be the exclusive prefix */
        }
        const uint32_t code = ((p0[i >> 3] >> (i & 7)) & 1u) | (((p1[i >> 3] >> (i & 7)) & 1u) << 1) |
                              (((p2[i >> 3] >> (i & 7)) & 1u) << 2);
        uint32_t E;
        if (code) {
            E = dec[code];
        } else {
            if (base + rank >= n_esc) return ZO_ERR_CORRUPT;
            E = esc[base + rank];
            ++rank;
            ++running;
        }
        const uint32_t hi16 = ((uint32_t)(sm[i] & 0x80u) << 8) | (E << 7) | (sm[i] & 0x7Fu);
        if (dtype == ZO_BF16) {
            out[2 * i] = (uint8_t)hi16;
            out[2 * i + 1] = (uint8_t)(hi16 >> 8);
        } else {
            out[4 * i] = lo[2 * i];
            out[4 * i + 1] = lo[2 * i + 1];
            out[4 * i + 2] = (uint8_t)hi16;
            out[4 * i + 3] = (uint8_t)(hi16 >> 8);
        }
    }
    return running == n_esc ? ZO_OK : ZO_ERR_CORRUPT;
}

/*
 * Decompress n_chunks slots laid out back to back at their a-priori offsets.
 * G is read from each header (the slot offsets use the G of the first header).
 */
int zo_decompress(const void* comp, uint64_t comp_capacity, void* out, uint64_t n_elems, int dtype,
                  uint32_t n_chunks, const uint64_t* chunk_elems)
{
    const int es = elem_size(dtype);
    if (!es) return ZO_ERR_DTYPE;
    if (n_chunks == 0 || !comp || (!out && n_elems)) return ZO_ERR_ARG;
    if (!chunk_elems && n_elems % n_chunks) return ZO_ERR_ARG;
    uint64_t total = 0;
    for (uint32_t c = 0; c < n_chunks; ++c) total += chunk_elems ? chunk_elems[c] : n_elems / n_chunks;
    if (total != n_elems) return ZO_ERR_ARG;
    if (comp_capacity < 128) return ZO_ERR_CORRUPT;
    const uint32_t G = get32((const uint8_t*)comp + 12);
    if (G == 0) return ZO_ERR_CORRUPT;

    const uint8_t* src = (const uint8_t*)comp;
    uint8_t* dst = (uint8_t*)out;
    uint64_t off = 0;
    for (uint32_t c = 0; c < n_chunks; ++c) {
        uint64_t n = chunk_elems ? chunk_elems[c] : n_elems / n_chunks;
        if (off > comp_capacity) return ZO_ERR_CORRUPT;
        int rc = decompress_chunk(src + off, comp_capacity - off, n, dtype, dst);
        if (rc != ZO_OK) return rc;
        off += zo_slot_cap(n, dtype, G);
        dst += n * (uint64_t)es;
    }
    return ZO_OK;
}

/* fp32 bits (not a NaN: the caller has replaced those) -> bf16, round to nearest even */
static uint16_t f32_bits_to_bf16_rne(uint32_t u)
{
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/*
 * Section 3.3 / 5.2: local reduction after a zipped All-to-All.  comp holds n_peers slots of n
 * elements each, back to back at their a-priori offsets (what a rank's receive buffer looks
 * like).  The paper says "in FP32" and nothing more; the definition taken here:
 *   acc = -0.0f;  for p = 0 .. n_peers-1 (slot order):  acc = acc + x_p[i]   (FP32, round to nearest even)
 * -0 is the identity of FP32 addition for everything that is not a NaN (-0 + x = x, signed zeros
 * included), so out[i] = ((x_0[i] + x_1[i]) + x_2[i]) + ... and a single peer is widened exactly.
 * IEEE 754 leaves open which payload and sign a NaN result carries (the NaN that Inf - Inf produces
 * differs in sign between x86 and CDNA), so a sum that is a NaN is stored as the one quiet NaN
 * 0x7FC00000: the result is then the same bits on every machine.
 * bf16 inputs are widened exactly.  out_dtype ZO_FP32 writes the sums, ZO_BF16 the sums rounded to
 * nearest even (the NaN becomes 0x7FC0).  scratch holds one decoded slice (n elements of the input dtype).
 */
int zo_decompress_reduce(const void* comp, uint64_t comp_capacity, void* out, uint64_t n, int dtype,
                         uint32_t n_peers, int out_dtype, void* scratch, float* acc)
{
    const int es = elem_size(dtype);
    if (!es) return ZO_ERR_DTYPE;
    if (out_dtype != ZO_BF16 && out_dtype != ZO_FP32) return ZO_ERR_DTYPE;
    if (n_peers == 0 || !comp || (n && (!out || !scratch || !acc))) return ZO_ERR_ARG;
    if (comp_capacity < 128) return ZO_ERR_CORRUPT;
    const uint32_t G = get32((const uint8_t*)comp + 12);
    if (G == 0) return ZO_ERR_CORRUPT;
    const uint64_t cap = zo_slot_cap(n, dtype, G);
    for (uint32_t p = 0; p < n_peers; ++p) {
        const uint64_t off = (uint64_t)p * cap;
        if (off > comp_capacity) return ZO_ERR_CORRUPT;
        int rc = decompress_chunk((const uint8_t*)comp + off, comp_capacity - off, n, dtype, (uint8_t*)scratch);
        if (rc != ZO_OK) return rc;
        for (uint64_t i = 0; i < n; ++i) {
            uint32_t bits;
            if (dtype == ZO_BF16) bits = (uint32_t)((const uint16_t*)scratch)[i] << 16;
            else bits = ((const uint32_t*)scratch)[i];
            float x;
            memcpy(&x, &bits, 4);
            if (p == 0) acc[i] = -0.0f;
            acc[i] = acc[i] + x;
        }
    }
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t bits;
        memcpy(&bits, &acc[i], 4);
        if (isnan(acc[i])) bits = 0x7FC00000u;
        if (out_dtype == ZO_FP32) ((uint32_t*)out)[i] = bits;
        else ((uint16_t*)out)[i] = f32_bits_to_bf16_rne(bits);
    }
    return ZO_OK;
}
