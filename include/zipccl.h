/*
 * zipccl.h -- C ABI of libzipccl.so: lossless exponent coding of bf16 / fp32 communication
 * tensors on one MI355X (gfx950), after "ZipCCL" section 4.
 *
 * Conventions (all entry points):
 *   - `d_` pointers are DEVICE pointers, everything else is a HOST pointer.
 *   - The caller owns every buffer.  The library allocates nothing, frees nothing and keeps
 *     no pointer past the call.  Host arrays are read before the call returns.
 *   - compress / decompress are asynchronous on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream); they never synchronise with the host.
 *   - The return value covers argument and launch errors only.  Data-dependent problems
 *     (a corrupt stream) are reported through a device status word.
 *   - The device of the calling thread's current HIP context is used.
 *
 * Compressed layout, little-endian.  The output holds one SLOT per chunk; slot c starts at
 * slot_off[c] (a multiple of 128, known before compression from the element counts alone:
 * section 4.2.1's 128-byte peer padding), so a collective can send and decode every peer
 * slice on its own.  With pad(x) = x rounded up to 128 and a chunk of n elements:
 *
 *   HDR  128 B          "ZPCL", version u32 = 1, dtype u32, G u32, n u64, n_esc u64,
 *                       chunk_bytes u64, dec[8] (dec[0] = 0), then bytes 48..127 reserved: written
 *                       as zero, ignored when decoding
 *   SM   pad(n)         byte i = sign << 7 | 7 mantissa bits of the high 16-bit word
 *                       (section 4: sign and mantissa kept verbatim at a fixed stride)
 *   LO   pad(2n)        fp32 only: u16 i = low 16 bits of the word
 *   P0,P1,P2  pad(ceil(n/8)) each
 *                       plane k, byte i >> 3, bit i & 7 = bit k of code_i (section 4.2.1:
 *                       the 3-bit code stored as three 1-bit arrays)
 *   IDX  pad(4 ceil(n/G))  u32 g = zero-points among elements [0, g G) of this chunk
 *                       (section 4.2.3's stored prefix count; G = ZIPCCL_GROUP = 512)
 *   ESC  pad(n_esc) used, pad(n) reserved
 *                       byte j = raw exponent of the j-th zero-point, in element order
 *
 *   code_i = E - dec[1] + 1 when dec[1] <= E <= dec[7], else 0 (a "zero-point", section 4).
 *   Padding, and plane bits / IDX entries past n, are zero.
 *   chunk_bytes = HDR..IDX (the "static part", size independent of the data) + pad(n_esc)
 *   (the "dynamic part") = what a collective transmits for the chunk.
 */
#ifndef ZIPCCL_H
#define ZIPCCL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZIPCCL_GROUP 512u        /* elements per IDX entry: one wave64 x 8 values per lane */
#define ZIPCCL_ALIGN 128u        /* alignment of every slot and section */
#define ZIPCCL_MAX_CHUNK_ELEMS 0xFFFFFFFFull /* IDX entries are u32 */
#define ZIPCCL_STATIC_SCRATCH_BYTES (32u << 20) /* the library's own workspace, per GPU: zipccl_compress_static */
#define ZIPCCL_MAX_SAMPLE_STRIDE 4096u /* largest sample_stride of zipccl_estimate_chunk_tables_sampled */

typedef enum { ZIPCCL_BF16 = 0, ZIPCCL_FP32 = 1 } zipccl_dtype_t;

typedef enum {
    ZIPCCL_OK = 0,
    ZIPCCL_ERR_INVALID_ARG = 1,       /* null pointer, misaligned buffer, bad chunk split, bad table */
    ZIPCCL_ERR_UNSUPPORTED_DTYPE = 2,
    ZIPCCL_ERR_BUFFER_TOO_SMALL = 3,  /* out_capacity / workspace_bytes / comp_capacity too small */
    ZIPCCL_ERR_CORRUPT = 4,           /* device status word only: header or index inconsistent */
    ZIPCCL_ERR_DEVICE = 5             /* a HIP call failed (launch error) */
} zipccl_status_t;

/* dec[0] is unused (code 0 flags a zero-point); dec[1..7] are the biased exponents of codes
 * 1..7 and must be consecutive ascending values with 1 <= dec[1] <= 249 (the Gaussian model
 * always yields such a window). */
typedef struct { uint8_t dec[8]; } zipccl_table_t;

/*
 * Code-table builder (section 4.1).  Host only, pure.  For a zero-mean Gaussian of standard
 * deviation sigma, Eq.5 gives the continuous optimum of the window base
 * x_opt = log2(sigma) + 0.5 log2(14 ln2 / 16383); the better of floor/ceil(x_opt) under the
 * coverage of Eq.2 is taken (lower on a tie) and clamped so that dec[1] = x + 127 lies in
 * [1, 248].  The same table serves bf16 and fp32 (same exponent field).
 * Errors: sigma <= 0, NaN or Inf, or out == NULL -> ZIPCCL_ERR_INVALID_ARG.
 */
zipccl_status_t zipccl_build_table(double sigma, zipccl_dtype_t dt, zipccl_table_t* out);

/*
 * Chunk split used by every call below: chunk_elems (host, n_chunks entries) gives the
 * element count of each peer chunk, in order, and must sum to n_elems; NULL means an equal
 * split and requires n_elems % n_chunks == 0.  A chunk may be empty (header-only slot).
 * Each chunk holds at most ZIPCCL_MAX_CHUNK_ELEMS elements.
 */

/* Bytes needed for the compressed buffer in the worst case (every value a zero-point) =
 * slot_off[n_chunks].  Returns 0 on invalid arguments. */
size_t zipccl_max_compressed_size(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                  const uint64_t* chunk_elems);

/* slot_off (host, n_chunks + 1 entries): byte offset of every slot, and the total. */
zipccl_status_t zipccl_chunk_slot_offsets(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                          const uint64_t* chunk_elems, uint64_t* slot_off);

/*
 * Static / dynamic split of every slot (section 3.2, second All-to-All design; section 4: only the
 * zero-point list has a data-dependent size).  static_bytes (host, n_chunks entries) receives the
 * size of HDR..IDX of each chunk, known before compression.  A collective sends
 * [slot_off[c], slot_off[c] + static_bytes[c]) first, then exchanges chunk_bytes (one u64 per
 * peer, written by zipccl_compress), then sends the dynamic part
 * [slot_off[c] + static_bytes[c], slot_off[c] + chunk_bytes[c]); the receiver places both at
 * the same offsets of its own slot and decodes.
 */
zipccl_status_t zipccl_chunk_static_bytes(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                          const uint64_t* chunk_elems, uint64_t* static_bytes);

/* Bytes of device scratch for zipccl_compress.  With zipccl_compress_workspace_size bytes
 * (about one byte per element) compress reads the input once: zero-point exponents are parked
 * in the scratch until the per-chunk prefix of section 4.2.3 is known.  With less, but at least
 * zipccl_compress_min_workspace_size bytes (8 bytes per 8192 elements), it reads the input twice
 * (count, prefix, emit): workspace_bytes alone selects the form, call by call, and both write the same bytes.
 * Both return 0 on invalid arguments. */
size_t zipccl_compress_workspace_size(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                      const uint64_t* chunk_elems);
size_t zipccl_compress_min_workspace_size(size_t n_elems, zipccl_dtype_t dt, uint32_t n_chunks,
                                          const uint64_t* chunk_elems);

/*
 * Compress (section 4, second paragraph; kernel steps of section 4.2).
 *   d_in            device, n_elems values of dtype dt, aligned to the element size
 *                   (whole tiles of 8192 values take the vector path wherever the chunk starts)
 *   table           host, from zipccl_build_table
 *   d_out           device, 128-byte aligned, out_capacity >= zipccl_max_compressed_size(...)
 *   d_chunk_bytes   device, n_chunks u64, may be NULL: bytes to transmit for each chunk
 *   d_workspace     device, 16-byte aligned, workspace_bytes >= zipccl_compress_min_workspace_size(...)
 *                   (see above for what more buys); contents are overwritten
 * Every byte of [slot_off[c], slot_off[c] + chunk_bytes[c]) is written; the rest of a slot is
 * left untouched.  No kernel waits on another workgroup.  Calls that may overlap in time need
 * different workspaces.
 */
zipccl_status_t zipccl_compress(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                uint32_t n_chunks, const uint64_t* chunk_elems,
                                const zipccl_table_t* table,
                                void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes,
                                void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * zipccl_compress for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * bytes as zipccl_compress, minus the workspace: that is a fixed array of ZIPCCL_STATIC_SCRATCH_BYTES
 * (32 MiB) inside the library's device code, one copy on every GPU the library runs on, held until the process
 * ends.  The call makes no hipMalloc, hipFree or other allocating device call.
 *   - Up to about 33.5 million values (zipccl_compress_workspace_size(...) <= 32 MiB) the input is read once;
 *     above that twice (the form zipccl_compress takes with its minimum workspace).
 *   - A call whose zipccl_compress_min_workspace_size(...) exceeds 32 MiB (more than about 4.19 million tiles
 *     of 8192 values) returns ZIPCCL_ERR_BUFFER_TOO_SMALL and launches nothing.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap in time on the same GPU (different
 *     streams, different threads) race and must be ordered by the caller.  Nothing in the array needs to be
 *     cleared between calls, and nothing of a call's result stays in it.
 *   - The first call on each GPU looks up the array's device address (hipGetSymbolAddress); make that call
 *     outside a stream capture.
 */
zipccl_status_t zipccl_compress_static(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                       uint32_t n_chunks, const uint64_t* chunk_elems,
                                       const zipccl_table_t* table,
                                       void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes, void* stream);

/*
 * Table from the data (section 4.1, last sentence: sigma of the tensor by torch.std, i.e. the
 * unbiased sample standard deviation), computed and kept on the device so that no host
 * round trip sits between estimate and compress.  One pass over the tensor in FP64, then the
 * window by Eq.5 / Eq.2 exactly as zipccl_build_table does.  A sigma that is not a positive
 * finite number (constant tensor, NaN/Inf in the data, fewer than two values) selects the
 * lowest window (dec[1] = 1).
 *   d_in         device, n_elems values of dt, aligned to the element size
 *   d_table      device, 8-byte aligned: receives the table
 *   d_sigma      device double, 8-byte aligned, may be NULL: receives sigma (NaN if undefined)
 *   d_workspace  device, 8-byte aligned, >= zipccl_estimate_workspace_size() bytes
 * zipccl_compress_device_table is zipccl_compress with the table read from device memory
 * (as written by zipccl_estimate_table earlier on the same stream).
 */
size_t zipccl_estimate_workspace_size(void);
zipccl_status_t zipccl_estimate_table(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                      zipccl_table_t* d_table, double* d_sigma,
                                      void* d_workspace, size_t workspace_bytes, void* stream);
/*
 * The same with a sigma that a few large entries cannot move.  Section 4.1 derives the window for a
 * zero-mean Gaussian; activations with outlier channels, or a parameter shard that also holds LayerNorm
 * gains, inflate the sample standard deviation many times over and push the window off the bulk of the
 * values.  For w ~ N(0, sigma^2) the median of |w| is sigma * Phi^-1(3/4), so
 *     sigma = median(|w|) / 0.6744897501960817,
 * the median taken over the 15-bit magnitudes of the values' high 16-bit words (the bf16 value; the bf16
 * prefix of an fp32 value), as integers: rank floor((K - 1) / 2) of the K magnitudes that are neither zero
 * nor Inf/NaN.  K = 0 selects the lowest window (sigma NaN).  The window then follows from Eq.5 / Eq.2 as in
 * zipccl_build_table.  One pass over the tensor; the result is exact (a count) whatever the order of work.
 *   d_workspace  device, 8-byte aligned, >= zipccl_estimate_robust_workspace_size() bytes (256 KiB);
 *                contents are overwritten
 * n_elems must be below 2^40.  Other arguments as for zipccl_estimate_table.
 */
size_t zipccl_estimate_robust_workspace_size(void);
zipccl_status_t zipccl_estimate_table_robust(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             zipccl_table_t* d_table, double* d_sigma,
                                             void* d_workspace, size_t workspace_bytes, void* stream);
/*
 * One table per peer chunk.  Section 4.1 takes sigma per layer; the chunks of one collective call may hold
 * different layers, experts or peers' contributions whose scales differ by orders of magnitude, and every chunk
 * header carries its own table anyway (the decoders read it per slot).  zipccl_estimate_chunk_tables is
 * zipccl_estimate_table_robust applied to every chunk of the split on its own, in one pass over the tensor;
 * zipccl_compress_chunk_tables is zipccl_compress with chunk c coded by d_tables[c].
 *   d_tables     device, 8-byte aligned, n_chunks tables (written by the estimate, read by the compress)
 *   d_sigmas     device, n_chunks doubles, may be NULL
 *   d_workspace  of the estimate: 8-byte aligned, >= zipccl_estimate_chunk_tables_workspace_size(n_chunks)
 *                bytes (256 KiB per chunk); contents are overwritten
 * Chunk split and all other arguments as for zipccl_compress.
 */
size_t zipccl_estimate_chunk_tables_workspace_size(uint32_t n_chunks);
zipccl_status_t zipccl_estimate_chunk_tables(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             uint32_t n_chunks, const uint64_t* chunk_elems,
                                             zipccl_table_t* d_tables, double* d_sigmas,
                                             void* d_workspace, size_t workspace_bytes, void* stream);
/*
 * The same tables from a sample of every chunk (section 4.1 takes sigma of the whole tensor; the window base it
 * fixes is one integer, and one part in sample_stride of the values fixes the same integer unless sigma sits
 * within the sampling error, a few parts in ten thousand for 2^20 sampled values, of a window boundary) at
 * 1 / sample_stride of the memory traffic.  The sample consists of whole groups of 512 consecutive values, one
 * from every block of sample_stride consecutive groups of a chunk (groups count from the chunk's first value),
 * at position ((k * 2654435761 mod 2^32) >> 16) mod sample_stride inside block k; a block's group that lies
 * past the chunk's end adds nothing, a last group cut short adds the values it has.  The estimate is then the
 * one of zipccl_estimate_table_robust over the sampled values.
 *   sample_stride   a power of two in [1, ZIPCCL_MAX_SAMPLE_STRIDE]; 1 = zipccl_estimate_chunk_tables
 * Everything else, the workspace included, as for zipccl_estimate_chunk_tables (n_chunks = 1 for one table
 * for the whole tensor, of up to ZIPCCL_MAX_CHUNK_ELEMS values).
 */
zipccl_status_t zipccl_estimate_chunk_tables_sampled(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                                     uint32_t n_chunks, const uint64_t* chunk_elems,
                                                     uint32_t sample_stride,
                                                     zipccl_table_t* d_tables, double* d_sigmas,
                                                     void* d_workspace, size_t workspace_bytes, void* stream);
zipccl_status_t zipccl_compress_chunk_tables(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             uint32_t n_chunks, const uint64_t* chunk_elems,
                                             const zipccl_table_t* d_tables,
                                             void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes,
                                             void* d_workspace, size_t workspace_bytes, void* stream);
zipccl_status_t zipccl_compress_device_table(const void* d_in, size_t n_elems, zipccl_dtype_t dt,
                                             uint32_t n_chunks, const uint64_t* chunk_elems,
                                             const zipccl_table_t* d_table,
                                             void* d_out, size_t out_capacity, uint64_t* d_chunk_bytes,
                                             void* d_workspace, size_t workspace_bytes, void* stream);

/*
 * Decompress (section 4, third paragraph): code != 0 -> exponent from the table in the chunk
 * header, code == 0 -> next exponent of the zero-point list, found through IDX; recombined
 * with the stored sign and mantissa bits.
 *   d_comp          device, 128-byte aligned; slots at the a-priori offsets for this split
 *                   (a peer decodes one received slice with n_chunks = 1); comp_capacity is
 *                   the number of readable bytes and must cover the static part of every slot;
 *                   the kernel checks that each slot's zero-point list also fits
 *   d_out           device, n_elems values of dtype dt, aligned to the element size
 *   d_status        device u32, may be NULL: OR-ed with ZIPCCL_ERR_CORRUPT if a header does not
 *                   match (magic, version, dtype, G, n, sizes, a table that is not a window with
 *                   dec[0] = 0) or an index leaves the list;
 *                   the caller zeroes it.  Values of a corrupt chunk are unspecified, but no
 *                   read or write leaves the caller's buffers.
 */
zipccl_status_t zipccl_decompress(const void* d_comp, size_t comp_capacity,
                                  void* d_out, size_t n_elems, zipccl_dtype_t dt,
                                  uint32_t n_chunks, const uint64_t* chunk_elems,
                                  uint32_t* d_status, void* stream);

/*
 * Decompress and reduce: the local half of the zipped Reduce-Scatter (section 3.3; section 5.2
 * fixes FP32 for the local reduction of BF16 traffic).  d_comp holds the n_peers slots a rank has
 * received for its shard, back to back at the a-priori offsets of an equal split (slot p at
 * p * zipccl_max_compressed_size(n_elems, dt, 1, NULL)), n_elems values each; every slot may carry
 * its own table.  acc = -0.0f, then acc = acc + x_p[i] for every slot p in slot order, in FP32 with round to
 * nearest even: -0 is the identity of that addition for everything that is not a NaN, so
 * out[i] = ((x_0[i] + x_1[i]) + x_2[i]) + ... and a single slot is widened exactly (signed zeros, subnormals
 * and infinities included).  A sum that is a NaN is stored as the quiet NaN 0x7FC00000 whatever produced it
 * (IEEE 754 leaves payload and sign of a NaN result open), so the result is reproducible bit for bit.
 *   d_out    device, n_elems values of out_dt: ZIPCCL_FP32 = the sums, ZIPCCL_BF16 = the sums
 *            rounded to nearest even (the NaN becomes 0x7FC0); aligned to its element size
 *   d_status as in zipccl_decompress; a corrupt slot is left out of the sum
 * comp_capacity must cover the static part of every slot; 1 <= n_peers <= 1024.
 * Asynchronous on `stream`.
 */
zipccl_status_t zipccl_decompress_reduce(const void* d_comp, size_t comp_capacity, void* d_out, size_t n_elems,
                                         zipccl_dtype_t dt, uint32_t n_peers, zipccl_dtype_t out_dt,
                                         uint32_t* d_status, void* stream);

/*
 * Adaptive switcher for Reduce-Scatter (section 5.2).  Host only, pure.  Linear cost models
 *   T_RS(d)  = alpha_rs  + beta_rs  * d                  (Eq.6, native Reduce-Scatter)
 *   T_A2A(d) = alpha_a2a + beta_a2a * e * s * d          (Eq.7, zipped All-to-All + local reduce)
 * with d the data size in bytes, alpha in seconds, beta in seconds per byte, e the compression
 * factor of the zipped All-to-All (compressed / original bytes: 1 / compression ratio) and s the
 * precision scale factor (0.5 when the native collective moves a format twice as wide).
 * zipccl_switch_prefers_zipped returns 1 when T_A2A(d) < T_RS(d), 0 otherwise, -1 on bad
 * arguments (null model, negative or non-finite inputs); t_rs / t_a2a (nullable) receive the times.
 * zipccl_fit_link_model is the profiling step: ordinary least squares of t = alpha + beta d over
 * k >= 2 measured (d, t) pairs with at least two distinct sizes.
 */
typedef struct { double alpha_rs, beta_rs, alpha_a2a, beta_a2a; } zipccl_link_model_t;
int zipccl_switch_prefers_zipped(const zipccl_link_model_t* m, double d_bytes, double e, double s,
                                 double* t_rs, double* t_a2a);
zipccl_status_t zipccl_fit_link_model(const double* d_bytes, const double* t_seconds, size_t k,
                                      double* alpha, double* beta);

const char* zipccl_status_string(zipccl_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* ZIPCCL_H */
