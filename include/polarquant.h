/*
 * polarquant.h -- C ABI of libpolarquant: the PolarQuant KV-cache hot path
 * (random preconditioning, recursive polar transform, per-level angle
 * quantisation, attention computed on the packed codes) for one MI355X GPU.
 *
 * Configuration (Section 4.1 of the PolarQuant paper, "Practical
 * Implementation"): head dimension d = 128, L = 4 polar levels, 4 bits per
 * level-1 angle, 2 bits per angle of levels 2..4, one binary16 radius per
 * block of 16 rotated coordinates: 46 code bytes + 16 radius bytes = 62 bytes
 * per vector (3.875 bits per coordinate).
 *
 * Conventions
 *   - Every function returns a pq_status and never throws or aborts.
 *   - "device" pointers are HIP device memory owned by the caller and must be
 *     16-byte aligned (PQ_EALIGN otherwise); "host" pointers are ordinary
 *     memory.  The library allocates device memory only for the constants of
 *     a pq_ctx (< 1 MB per device, on the first call that uses that device).
 *   - Kernels are enqueued on the caller's hipStream_t (passed as void*; NULL
 *     is the default stream).  The library does not synchronise the stream and
 *     records no memset or copy nodes, so its calls can be captured into a HIP
 *     graph -- with one exception, stated where it is declared:
 *     pq_fit_codebooks(_deep) copy their histograms to the host and wait.
 *   - A pq_ctx is configured (pq_set_codebooks, pq_set_recursion_depth,
 *     pq_set_upper_codebooks) before its first launch; from then on it is
 *     immutable and may be shared by threads.
 *   - Block norms: the stored radius is a binary16 number; a block whose norm
 *     exceeds the format's range is stored with the largest finite radius,
 *     65504 (its direction is kept).  Everything computed from a cache of finite
 *     inputs is finite.
 *
 * Cache layout ("tiles")
 *   A cache holds keys or values of n_heads head planes.  Each plane is an
 *   array of pool_tokens token slots, pool_tokens a multiple of 64.  64
 *   consecutive slots form a tile: PQ_TILE_CODE_BYTES (2944) code bytes in
 *   the codes buffer and PQ_TILE_RADII (512) binary16 radii in the radii
 *   buffer, i.e. exactly 62 bytes per token.
 *     codes: uint8_t [n_heads][pool_tokens/64][2944]
 *     radii: uint16_t[n_heads][pool_tokens/64][512]
 *   Inside a tile the 46 code bits of a block are stored as the table
 *   indices the attention kernel gathers with (four 10-bit quarter indices
 *   and one 6-bit block index), in per-lane bit strings spread over planes
 *   that a 64-lane wavefront reads with full-width coalesced loads; keys
 *   (PQ_KEY: one token per lane) and values (PQ_VALUE: one half-block of 16
 *   tokens per lane) use different in-tile orders because the score and the
 *   weighted-sum contractions consume them differently.  The exact bit
 *   positions are specified at the top of csrc/pq_layout.h;
 *   pq_export_canonical converts tiles to the order-independent canonical
 *   62-byte records.
 *   A sequence must start on a tile boundary (seq_start % 64 == 0).
 */
#ifndef POLARQUANT_H
#define POLARQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pq_ctx pq_ctx; /* opaque: S, codebooks, device constant tables */

typedef enum { PQ_F32 = 0, PQ_BF16 = 1 } pq_dtype;
typedef enum { PQ_KEY = 0, PQ_VALUE = 1 } pq_kind;
typedef enum {
    PQ_OK = 0,
    PQ_EINVAL = -1,       /* null pointer, bad size, bad enum */
    PQ_EUNSUPPORTED = -2, /* d != 128, more than 16 query heads per kv head, ... */
    PQ_EALIGN = -3,       /* device pointer or stride not 16-byte aligned */
    PQ_EHIP = -4,         /* a HIP runtime call failed (no device, launch error) */
    PQ_ENOMEM = -5,       /* host or device allocation failed, workspace too small */
    PQ_ESCRATCH = -6,     /* pq_attn_decode_polar_static: the problem needs more than PQ_STATIC_SCRATCH_BYTES */
    PQ_ENOTREADY = -7     /* pq_attn_decode_polar_static: pq_prepare_device has not run for this context and device */
} pq_status;

#define PQ_D 128               /* head dimension */
#define PQ_LEVELS 4            /* polar levels */
#define PQ_BLOCK 16            /* coordinates per stored radius */
#define PQ_RECORD_BYTES 62     /* canonical record: 46 code bytes + 8 binary16 radii */
#define PQ_TILE_TOKENS 64
#define PQ_TILE_CODE_BYTES 2944
#define PQ_TILE_RADII 512

const char *pq_status_string(pq_status s);

/* ---------------------------------------------------------------------------
 * Preconditioner and codebooks (Section 3.2 footnote and Section 4.1: one
 * random rotation S shared by keys, values, layers and heads; Algorithm 1
 * line 3 / Eq. 3 with the "offline" codebook: the optimal 1-D quantiser of the
 * closed-form angle density of Lemma 2, shared by every prompt).
 *
 * d must be 128 (PQ_EUNSUPPORTED otherwise).  If S_rowmajor_f64 (host, d*d
 * doubles, S[i][j] at i*d+j, used as y = x * S) is not NULL it is taken
 * verbatim after checking ||S^T S - I||_max <= 1e-10 (PQ_EINVAL otherwise);
 * if NULL, S is generated on the host in double precision from `seed`:
 * a Gaussian matrix from a counter-based generator (splitmix64 finaliser +
 * Box-Muller), whose columns are orthonormalised in order (modified
 * Gram-Schmidt, every projection pass done twice): the Q factor of its QR
 * factorisation with a positive diagonal of R.  Codebooks are computed on the
 * host in double precision.
 * No device is touched; *out receives the context (caller frees it with
 * pq_destroy).
 * ------------------------------------------------------------------------- */
pq_status pq_init_preconditioner(pq_ctx **out, int d, uint64_t seed, const double *S_rowmajor_f64);

/* The same with a structured preconditioner: S = D H / sqrt(d), H the Sylvester
 * Hadamard matrix H[i][j] = (-1)^popcount(i & j), D a diagonal of random signs
 * drawn from seed (Section 1 names random Hadamard matrices as preconditioners
 * of this kind).  Everything else (codebooks, layout, kernels) is unchanged;
 * because all entries of such an S are +-1/sqrt(d), pq_encode_kv rotates with
 * one exact bf16 term instead of three.  Any S passed to pq_init_preconditioner
 * whose entries all have that magnitude takes the same path.
 * The products of single vectors with such an S -- the query rotation, the key
 * and value of pq_append_kv / pq_decode_step_polar, the un-rotation of the
 * attention output -- run as a fast Walsh-Hadamard transform (d log2 d additions
 * in one wavefront, S is not read); so does any S given to pq_init_preconditioner
 * that is exactly a sign diagonal times the Sylvester matrix over sqrt(d). */
pq_status pq_init_preconditioner_hadamard(pq_ctx **out, int d, uint64_t seed);

/* How the kernels multiply by this context's S: 0 = general matrix (three bf16
 * terms in pq_encode_kv, dense products elsewhere), 1 = all entries +-1/sqrt(d)
 * (one term in pq_encode_kv), 2 = D H / sqrt(d) with the Sylvester H (one term,
 * and the single-vector products by fast Walsh-Hadamard transform).  -1 if ctx is
 * NULL. */
int pq_preconditioner_structure(const pq_ctx *ctx);

/* Replaces the codebooks of a context that has not launched anything yet (PQ_EINVAL
 * afterwards: the tables are already on a device) -- the place where codebooks fitted
 * to a prompt's own angles (Section 4.1, online variant) come in, and with S = I the
 * un-preconditioned variant.  cb (host): 28 centroids in radians, level 1 first (16 in
 * [0, 2 pi)), then 4 each for levels 2, 3, 4 (in [0, pi/2)), strictly increasing per
 * level.  Cell boundaries are the midpoints of neighbouring centroids (procedure Quant:
 * nearest centroid, linear distance, no wrap-around at level 1).  PQ_EUNSUPPORTED if two
 * level-1 boundaries are closer than about 0.02 rad.  Encode, append, DeQuant and the
 * attention kernels all follow the new codebooks; encoding is somewhat slower than with
 * the analytic ones (level 1 no longer has equal cells). */
pq_status pq_set_codebooks(pq_ctx *ctx, const double *cb);

/* Online codebook construction (Section 4.1; line 3 of Algorithm 1 fitted to the input
 * instead of the analytic densities): the vectors x (device, layout and strides as for
 * pq_encode_kv, keys and values alike) are rotated with the context's S, their angles
 * are counted on the GPU into fine per-level histograms (8192 bins over [0, 2 pi) at
 * level 1, 2048 over [0, pi/2] above; bins uniform in v / (u + v) of a node's two inputs,
 * 4.9e-4 to 9.8e-4 rad wide), and `iterations` k-means rounds -- nearest centroid, then
 * centroid := mean of its cell -- run on the histograms from cb_init (host, 28
 * centroids; NULL: the context's current codebooks).  The paper seeds k-means++ at
 * random; a fixed seed codebook makes the result a function of the data.  cb_out
 * (host): 28 centroids, ready for pq_set_codebooks on a fresh context.  workspace
 * (device): pq_fit_workspace_bytes() bytes.  This call copies the histograms
 * to the host and WAITS for the stream (it cannot be captured into a graph);
 * pq_fit_count_angles and pq_fit_cluster below are its two halves for callers
 * that place the wait themselves.  x, ld_token, ld_head aligned as for
 * pq_encode_kv (PQ_EALIGN).  PQ_EUNSUPPORTED beyond 2^26 vectors per call. */
pq_status pq_fit_codebooks(const pq_ctx *ctx, const void *x, pq_dtype xt, int64_t n_tokens, int n_heads,
                           int64_t ld_token, int64_t ld_head, const double *cb_init, int iterations,
                           double *cb_out, void *workspace, size_t workspace_bytes, void *hip_stream);
size_t pq_fit_workspace_bytes(void);

/* The two halves of pq_fit_codebooks(_deep).
 * pq_fit_count_angles: clears the histograms in workspace (device) with a kernel of
 * its own and counts the angles of x into them (for a depth-7 context also those of
 * levels 5..7); enqueued on the stream, returns at once, no memset or copy nodes.
 * pq_fit_cluster: host only; hist (host) is a copy of those pq_fit_workspace_bytes()
 * bytes, taken after the stream has reached that point; the k-means rounds of Section
 * 4.1 on the bins from cb_init / cbt_init (NULL: the context's codebooks) ->
 * cb_out (28), cbt_out ([3][8]; required for a depth-7 context, ignored otherwise). */
pq_status pq_fit_count_angles(const pq_ctx *ctx, const void *x, pq_dtype xt, int64_t n_tokens, int n_heads,
                              int64_t ld_token, int64_t ld_head, void *workspace, size_t workspace_bytes,
                              void *hip_stream);
pq_status pq_fit_cluster(const pq_ctx *ctx, const uint32_t *hist, const double *cb_init, const double *cbt_init,
                         int iterations, double *cb_out, double *cbt_out);

/* The same for a depth-7 context (PQ_EINVAL otherwise): the angles of levels 5, 6, 7 -- 4 + 2 + 1
 * per vector, formed from the 8 block radii -- are counted as well ((pi/2) / 2048 bins) and
 * clustered from cbt_init (host, [3][8] as for pq_set_upper_codebooks; NULL: the context's
 * current ones) with the bit widths of the context.  cbt_out (host): [3][8], ready for
 * pq_set_upper_codebooks on a fresh context; cb_out as above.  Same workspace. */
pq_status pq_fit_codebooks_deep(const pq_ctx *ctx, const void *x, pq_dtype xt, int64_t n_tokens, int n_heads,
                                int64_t ld_token, int64_t ld_head, const double *cb_init, const double *cbt_init,
                                int iterations, double *cb_out, double *cbt_out, void *workspace,
                                size_t workspace_bytes, void *hip_stream);

/* Full-depth recursion (Definition 1 and procedure Polar of Algorithm 1 run to level
 * log2 d = 7; memory count of Section 4: one floating-point radius per vector plus the
 * angle codes; remark after Theorem 1: the codebook size of a level is free).
 * depth 4 (the default) is Section 4.1's truncation.  depth 7: the recursion continues
 * over the 8 block radii of a vector with 4 + 2 + 1 more angles (levels 5, 6, 7), coded
 * with upper_bits[0..2] (host) bits each, 1..3, 4 b5 + 2 b6 + b7 <= 16 (PQ_EUNSUPPORTED
 * beyond); their codebooks are the optimal quantisers of Lemma 2's densities for those
 * levels.  Levels 1..4 keep Section 4.1's widths (4, 2, 2, 2) and the context's codebooks.
 * A vector then takes 46 code bytes + one 32-bit word (binary16 radius and the upper
 * codes) = 50 bytes (3.125 bits per coordinate); other depths: PQ_EUNSUPPORTED.
 * The cache layout changes with it: the radii buffer of a cache holds
 * pq_radii_halves_per_tile(ctx) halves per tile (512 at depth 4; 128 at depth 7: word
 * tau of a tile = radius << 16 | upper codes, level-5 codes lowest), canonical records
 * have pq_record_bytes(ctx) bytes (62; 50 = bytes 0..45 as before, the 16-bit code word
 * little endian, the radius little endian).  Like pq_set_codebooks this must precede the
 * first launch with the context (PQ_EINVAL afterwards).  At depth 7 pq_encode_kv,
 * pq_append_kv(_pair), pq_decode_kv, pq_export_canonical and every attention entry
 * point follow the new format; pq_set_codebooks (levels 1..4) combines with it, and
 * pq_set_upper_codebooks replaces the codebooks of levels 5..7. */
pq_status pq_set_recursion_depth(pq_ctx *ctx, int depth, const int *upper_bits);
/* Replaces the codebooks of levels 5, 6, 7 of a depth-7 context (Algorithm 1 takes a
 * codebook per level as input; Section 4.1's online variant fits them to the data): cbt
 * (host) [3][8] doubles, row l-5 holds the 2^bits(l) centroids of level l in (0, pi/2),
 * strictly increasing, the rest of the row ignored.  Cell boundaries are the midpoints
 * of neighbouring centroids.  After pq_set_recursion_depth(ctx, 7, ...) and before the
 * first launch with the context (PQ_EINVAL otherwise). */
pq_status pq_set_upper_codebooks(pq_ctx *ctx, const double *cbt);
int pq_recursion_depth(const pq_ctx *ctx);
int pq_radii_halves_per_tile(const pq_ctx *ctx);
int pq_record_bytes(const pq_ctx *ctx);
/* level in 5..7 of a depth-7 context (PQ_EINVAL otherwise): its bit width, 2^bits
 * centroids, 2^bits + 1 boundaries; any output may be NULL. */
pq_status pq_get_upper_codebook(const pq_ctx *ctx, int level, int *bits, double *centroids, double *boundaries);

/* Copies S (d*d doubles, row-major, S[i][j] at i*d+j) to host memory S_out. */
pq_status pq_get_preconditioner(const pq_ctx *ctx, double *S_out);

/* level in 1..4.  centroids: K doubles (K = 16 for level 1, 4 otherwise);
 * boundaries: K+1 doubles (lower end, K-1 inner boundaries, upper end).
 * Either output may be NULL. */
pq_status pq_get_codebook(const pq_ctx *ctx, int level, double *centroids, double *boundaries);

void pq_destroy(pq_ctx *ctx);

/* ---------------------------------------------------------------------------
 * Encode (Algorithm 1 lines 2 and 4, procedures Polar and Quant, with the
 * settings of Section 4.1): for every vector y = x * S, a depth-4 polar
 * transform of each block of 16 coordinates, every angle replaced by the
 * index of its nearest centroid, the block radius rounded to binary16, the
 * result bit-packed into the tile layout of `kind`.
 *
 * x (device): element (t, h, k) at x[t*ld_token + h*ld_head + k], k < 128,
 *   t < n_tokens, h < n_heads; dtype xt; ld_token and ld_head in elements,
 *   multiples of 8 (bf16) or 4 (f32) so that every row is 16-byte aligned.
 * Token t of head h is written to slot dst_token0 + t of head plane h of the
 * cache (codes, radii) whose planes hold pool_tokens slots.  Slots of a tile
 * outside [dst_token0, dst_token0 + n_tokens) keep their contents.
 * Two calls that write into the same tile must not overlap in time.
 * n_tokens == 0 is a no-op (pointers are not examined).
 * ------------------------------------------------------------------------- */
pq_status pq_encode_kv(const pq_ctx *ctx, const void *x, pq_dtype xt, pq_kind kind,
                       int64_t n_tokens, int n_heads, int64_t ld_token, int64_t ld_head,
                       uint8_t *codes, uint16_t *radii, int64_t pool_tokens,
                       int64_t dst_token0, void *hip_stream);

/* Keys and values of the same tokens in one launch: exactly pq_encode_kv(xk, PQ_KEY, ...) followed by
 * pq_encode_kv(xv, PQ_VALUE, ...) with the same n_tokens, n_heads, strides, pool size and first slot
 * (Algorithm 1 applied to both streams of the cache of Section 4), bit for bit.  Half of the
 * workgroups take the key tiles, half the value tiles: one dispatch, S staged once per CU, twice the
 * tiles per wavefront -- noticeably faster than two calls when a call covers only a few tiles per CU
 * (a 32k-token prompt of 8 kv heads).  Arguments and errors as for pq_encode_kv. */
pq_status pq_encode_kv_pair(const pq_ctx *ctx, const void *xk, const void *xv, pq_dtype xt,
                            int64_t n_tokens, int n_heads, int64_t ld_token, int64_t ld_head,
                            uint8_t *k_codes, uint16_t *k_radii, uint8_t *v_codes, uint16_t *v_radii,
                            int64_t pool_tokens, int64_t dst_token0, void *hip_stream);

/* Decode-time append: one new token per sequence.  x (device): [n_seq][n_heads][128]
 * contiguous; sequence b's vectors go to slot dst_token[b] (device array of
 * n_seq int64) of every head plane.  Same arithmetic as pq_encode_kv. */
pq_status pq_append_kv(const pq_ctx *ctx, const void *x, pq_dtype xt, pq_kind kind,
                       int n_seq, int n_heads, uint8_t *codes, uint16_t *radii,
                       int64_t pool_tokens, const int64_t *dst_token, void *hip_stream);

/* The same for the key and the value vectors of the new tokens in one launch
 * (a decode step appends both): xk, xv (device) [n_seq][n_heads][128] contiguous,
 * same dtype; both caches have pool_tokens slots per head plane and the vectors
 * of sequence b go to slot dst_token[b] of either.  Results are identical to two
 * pq_append_kv calls. */
pq_status pq_append_kv_pair(const pq_ctx *ctx, const void *xk, const void *xv, pq_dtype xt,
                            int n_seq, int n_heads, uint8_t *k_codes, uint16_t *k_radii,
                            uint8_t *v_codes, uint16_t *v_radii, int64_t pool_tokens,
                            const int64_t *dst_token, void *hip_stream);

/* ---------------------------------------------------------------------------
 * DeQuant (Algorithm 1, procedure DeQuant): slots [token0, token0+n_tokens)
 * of every head plane are rebuilt top-down from the stored radius with the
 * cos / sin of the code centroids.  rotated == 0 applies the trailing
 * multiplication by S^T (the procedure as printed); rotated != 0 stops
 * before it and returns r^(0), the vector in the rotated domain.
 * out (device): element (t, h, k) at out[t*ld_token + h*ld_head + k].
 * ------------------------------------------------------------------------- */
pq_status pq_decode_kv(const pq_ctx *ctx, pq_kind kind, const uint8_t *codes, const uint16_t *radii,
                       int64_t pool_tokens, int64_t token0, int64_t n_tokens, int n_heads,
                       void *out, pq_dtype ot, int64_t ld_token, int64_t ld_head,
                       int rotated, void *hip_stream);

/* Tiles -> canonical records (device to device): rec[h][t][62] for slots
 * [token0, token0+n_tokens) of each head plane.  Canonical record: bytes
 * 0..31 the 64 level-1 codes in coordinate order, two per byte, earlier code
 * in the high nibble; bytes 32..39 / 40..43 / 44..45 the level-2 / 3 / 4
 * codes, four per byte, earlier code in the higher bits; bytes 46..61 the 8
 * binary16 radii in block order, little endian. */
pq_status pq_export_canonical(const pq_ctx *ctx, pq_kind kind, const uint8_t *codes,
                              const uint16_t *radii, int64_t pool_tokens, int64_t token0,
                              int64_t n_tokens, int n_heads, uint8_t *rec, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Decode attention on the packed cache (Eq. 5: softmax(Khat q / sqrt(d))
 * Vhat with Khat, Vhat the DeQuant of the cached codes), one query token per
 * sequence, grouped-query heads.  Because S is a rotation, the kernels work
 * in the rotated domain: q is multiplied by S once, keys and values are
 * rebuilt from their codes without the trailing S^T, and the weighted value
 * sum is multiplied by S^T once at the end.
 *
 * q (device): [B][Hq][128] bf16.  out (device): [B][Hq][128] of out_dtype
 * (PQ_BF16, rounded to nearest even, or PQ_F32).  k_* / v_*: caches written by
 * pq_encode_kv with PQ_KEY / PQ_VALUE, Hkv head planes of pool_tokens slots.
 * Sequence b owns slots [seq_start[b], seq_start[b] + ctx_len[b]) of every
 * plane (seq_start, ctx_len: device arrays of B entries; seq_start[b] % 64
 * == 0; the tile holding the last token must lie inside the pool).  The
 * query attends to all ctx_len[b] cached tokens (its own key/value are
 * appended before the call).  Query head h reads KV head h / (Hq/Hkv);
 * Hq must be a multiple of Hkv and Hq/Hkv at most 16.  ctx_len[b] == 0 gives a zero output row.
 * max_ctx (host) bounds every ctx_len[b]; it sizes the workspace; at most
 * 2^26 tokens, and B * Hkv * ceil(max_ctx / 64) must stay below 2^31 - 4096
 * (PQ_EUNSUPPORTED beyond).  The context lengths themselves are only read on
 * the device: the work is split there into equal shares of 64-token tiles
 * per wavefront, whatever the mix of lengths, so a ragged batch costs what
 * its total number of cached tokens costs.
 * workspace (device): at least pq_attn_workspace_bytes(B, Hq, Hkv, max_ctx)
 * bytes, PQ_ENOMEM otherwise; contents need not be preserved between calls.
 * ------------------------------------------------------------------------- */
pq_status pq_attn_decode_polar(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                               const uint8_t *k_codes, const uint16_t *k_radii,
                               const uint8_t *v_codes, const uint16_t *v_radii,
                               const int64_t *seq_start, const int32_t *ctx_len,
                               int B, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                               float softmax_scale, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

size_t pq_attn_workspace_bytes(int B, int Hq, int Hkv, int64_t max_ctx);

/* ---------------------------------------------------------------------------
 * pq_attn_decode_polar for callers that cannot allocate device memory or hand
 * over a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and bit-identical results,
 * but the workspace is a device array inside the library of
 * PQ_STATIC_SCRATCH_BYTES bytes (held by every GPU the library runs on until the
 * process ends).  The call itself allocates nothing and frees nothing:
 *   - a problem whose workspace (pq_attn_workspace_bytes) exceeds the array is
 *     refused with PQ_ESCRATCH before anything is launched;
 *   - the context's constants must already be on the current device, which
 *     pq_prepare_device(ctx) does once (it allocates; so does the first
 *     pq_encode_kv or attention call with the context on that device):
 *     PQ_ENOTREADY otherwise.
 * Every call on a GPU uses that GPU's one array, and the array keeps the last
 * call's contents (nothing in it has to start at zero: the work plan and every
 * partial result are written before they are read).  Calls that overlap in time
 * on one GPU -- two streams, two threads -- race on it; calls ordered on one
 * stream do not.
 * ------------------------------------------------------------------------- */
#define PQ_STATIC_SCRATCH_BYTES (16u << 20)
size_t pq_static_scratch_bytes(void);
pq_status pq_prepare_device(const pq_ctx *ctx);
pq_status pq_attn_decode_polar_static(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                                      const uint8_t *k_codes, const uint16_t *k_radii,
                                      const uint8_t *v_codes, const uint16_t *v_radii,
                                      const int64_t *seq_start, const int32_t *ctx_len,
                                      int B, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                                      float softmax_scale, void *hip_stream);

/* The same for M query tokens per sequence at once (several draft tokens of a
 * speculative step, or a chunk of a prompt): q, out (device): [B][M][Hq][128].  The
 * M tokens are the M newest of the sequence and their keys and values are already in
 * the cache (ctx_len counts them): query token m attends to the first
 * ctx_len[b] - (M-1-m) cached tokens, i.e. up to and including its own (causal order,
 * Eq. 4-5 with K_{:i}).  The keys and values are rebuilt once per kv head for all
 * M * (Hq/Hkv) query rows, which is what makes this cheaper than M separate calls.
 * M * (Hq/Hkv) <= 16, else PQ_EUNSUPPORTED.  workspace: pq_attn_mq_workspace_bytes. */
pq_status pq_attn_decode_polar_mq(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                                  const uint8_t *k_codes, const uint16_t *k_radii,
                                  const uint8_t *v_codes, const uint16_t *v_radii,
                                  const int64_t *seq_start, const int32_t *ctx_len,
                                  int B, int M, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                                  float softmax_scale, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

size_t pq_attn_mq_workspace_bytes(int B, int M, int Hq, int Hkv, int64_t max_ctx);

/* One whole decode step (Algorithm 1 on the newest token of every sequence, then
 * Eq. 5 on the cache that now holds it): pq_append_kv_pair(xk, xv -> dst_token)
 * followed by pq_attn_decode_polar, with identical results; the appends and the
 * rotation of q share one launch.  xk, xv (device): [B][Hkv][128] contiguous of
 * dtype xt; dst_token (device): B slots, normally seq_start[b] + ctx_len[b] - 1
 * with ctx_len already counting the new token.  The caches are written (the
 * appended slots) and read.  All other arguments as for pq_attn_decode_polar. */
pq_status pq_decode_step_polar(const pq_ctx *ctx, const void *xk, const void *xv, pq_dtype xt,
                               const int64_t *dst_token, const void *q, void *out, pq_dtype out_dtype,
                               uint8_t *k_codes, uint16_t *k_radii, uint8_t *v_codes, uint16_t *v_radii,
                               const int64_t *seq_start, const int32_t *ctx_len,
                               int B, int Hq, int Hkv, int64_t pool_tokens, int64_t max_ctx,
                               float softmax_scale, void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/* ---------------------------------------------------------------------------
 * Decode attention over a quantised prefix plus an unquantised recent window
 * (Section 5.3: the keys and values streamed in during generation are kept in
 * 16 bits, only the prompt's are quantised): one softmax over the DeQuant of
 * sequence b's ctx_len[b] cached tokens (Eq. 5) and its win_len[b] window
 * tokens, taken as given.  win_k, win_v (device): bf16 [B][Hkv][win_cap][128]
 * contiguous; win_len (device): B entries, clamped to [0, win_cap]; the order
 * of the window tokens does not matter.  All other arguments as for
 * pq_attn_decode_polar (ctx_len counts the quantised tokens only); workspace:
 * at least pq_attn_hybrid_workspace_bytes(B, Hq, Hkv, max_ctx, win_cap) bytes.
 * A sequence with neither prefix nor window gives a zero output row.
 * Hq/Hkv at most 16.
 * ------------------------------------------------------------------------- */
pq_status pq_attn_decode_hybrid(const pq_ctx *ctx, const void *q, void *out, pq_dtype out_dtype,
                                const uint8_t *k_codes, const uint16_t *k_radii,
                                const uint8_t *v_codes, const uint16_t *v_radii,
                                const int64_t *seq_start, const int32_t *ctx_len,
                                const void *win_k, const void *win_v, const int32_t *win_len,
                                int64_t win_cap, int B, int Hq, int Hkv, int64_t pool_tokens,
                                int64_t max_ctx, float softmax_scale, void *workspace,
                                size_t workspace_bytes, void *hip_stream);

size_t pq_attn_hybrid_workspace_bytes(int B, int Hq, int Hkv, int64_t max_ctx, int64_t win_cap);

/* ---------------------------------------------------------------------------
 * The general format: recursion depths 4 to 7 with other bit widths than
 * Section 4.1's (Definition 1 recurses to log2 d; the remark after Theorem 1
 * leaves the codebook size of each level free).  A plain path next to the tuned
 * one: records in the canonical general layout, one after another, read through
 * a generic bit reader by simple fp32 kernels (one wavefront per vector, or per
 * (sequence, query head) in attention); not tuned.
 *   format: depth in 4..7; bits[l-1] bits for the angles of level l:
 *           level 1: 3 or 4; levels 2-4: 2 or 3; levels 5-7 (up to depth): 1, 2 or 3.
 *   record: the codes of level 1 (64, in coordinate order), then level 2 (32), ...,
 *           each bits[l-1] wide, in one little-endian bit stream (bit p of the
 *           stream is bit p & 7 of byte p >> 3) padded to a whole byte, then the
 *           128 >> depth radii r^(depth) as little-endian binary16 (saturating at
 *           65504).  pq_general_record_bytes gives its size (0: format refused).
 *   cbg (host): the centroids of levels 1..depth one after another, level l holding
 *           2^bits[l-1] ascending entries (level 1 in [0, 2 pi], others in [0, pi/2]);
 *           cell boundaries are midpoints (procedure Quant).  pq_general_codebooks
 *           writes the Lloyd-Max codebooks of Lemma 2's densities (level 1: equal
 *           cells) into cbg[pq_general_codebook_entries(f)].
 * All of them use the context's S only.  x: device, n_vectors rows of 128 values
 * (PQ_BF16 or PQ_F32), row r at element r * ld_vector.  records: device,
 * [n_vectors][record bytes].  pq_general_decode: out device fp32 [n_vectors][128];
 * rotated != 0 stops before the trailing S^T of procedure DeQuant.
 * pq_general_attn_decode: Eq. 5 for one bf16 query per sequence (q device
 * [B][Hq][128]) on records [Hkv][pool_tokens][record bytes], sequence b owning
 * tokens [seq_start[b], seq_start[b] + ctx_len[b]) of every head plane (device
 * arrays; a range outside the pool or an empty one gives a zero row), out device
 * fp32 [B][Hq][128].  No workspace, nothing allocated, launches only.
 * ------------------------------------------------------------------------- */
typedef struct pq_general_format {
    int depth;
    int bits[7];
} pq_general_format;

size_t pq_general_record_bytes(const pq_general_format *f);
int pq_general_codebook_entries(const pq_general_format *f);
pq_status pq_general_codebooks(const pq_general_format *f, double *cbg);
pq_status pq_general_encode(const pq_ctx *ctx, const pq_general_format *f, const double *cbg, const void *x,
                            pq_dtype xt, int64_t n_vectors, int64_t ld_vector, uint8_t *records, void *hip_stream);
pq_status pq_general_decode(const pq_ctx *ctx, const pq_general_format *f, const double *cbg, const uint8_t *records,
                            int64_t n_vectors, int rotated, float *out, void *hip_stream);
pq_status pq_general_attn_decode(const pq_ctx *ctx, const pq_general_format *f, const double *cbg, const void *q,
                                 float *out, const uint8_t *k_records, const uint8_t *v_records,
                                 const int64_t *seq_start, const int32_t *ctx_len, int B, int Hq, int Hkv,
                                 int64_t pool_tokens, float softmax_scale, void *hip_stream);

/* ---------------------------------------------------------------------------
 * Optional timing of the two dominant kernels (the attention partial kernel
 * and the encode kernel) with HIP events recorded on the launch stream,
 * for benchmarks: pq_profile_begin(max_launches) creates the events and turns
 * recording on (at most max_launches launches of each kernel are timed);
 * pq_profile_end waits for the recorded events, returns the summed kernel
 * time in milliseconds and the number of timed launches per kernel (any
 * output may be NULL) and turns recording off.  Process-wide, not per ctx.
 * ------------------------------------------------------------------------- */
pq_status pq_profile_begin(int max_launches);
/* The same, timing only every `every`-th launch of each kernel (the two event records around a launch
 * cost a few microseconds of stream time: sampling keeps a timed loop close to its untimed speed). */
pq_status pq_profile_begin_sampled(int max_launches, int every);
pq_status pq_profile_end(double *attn_ms, int *attn_launches, double *encode_ms, int *encode_launches);

/* Name of the dominant kernel of the last pq_attn_decode_polar / pq_encode_kv
 * launch configuration (for matching profiler output); static strings. */
const char *pq_kernel_name_attn(void);
const char *pq_kernel_name_encode(void);

#ifdef __cplusplus
}
#endif
#endif /* POLARQUANT_H */
