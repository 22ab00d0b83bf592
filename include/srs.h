/*
 * srs.h -- C ABI of the MI355X (gfx950) hot path of lossless sparse weight synchronisation.
 *
 * Two operations, as the paper states the problem:
 *
 *   extract (Trainer side)  -- the changed-index set I = { i : W[i] != W_prev[i] } (Alg. 1, the
 *       line that forms I_t; Sec. 3.1 "Compute indices"), with "!=" taken on the 16-bit pattern so
 *       that the receiver can be bit-identical (goal G1), together with the values V = W[I], I as
 *       int32 and V as BF16 (Alg. 2, the line that forms V), in ascending index order (Sec. 3.3
 *       relies on sorted indices), one (I, V) payload per fixed-size bucket (the unit that is sent:
 *       Fig. 2 caption, Sec. 2 on bucketing).  The same pass brings the snapshot W_prev up to date.
 *
 *   apply (Rollout side)    -- the in-place scatter W[I] <- V (Alg. 3, the scatter line; Sec. 3.2
 *       calls it a fused kernel), after which W equals the Trainer's weights bit for bit.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller (the library never frees or keeps
 *     it past the call's completion on the stream).  Arrays of descriptors (srs_tensor_pair[],
 *     srs_tensor[], numel[]) are HOST arrays, read before the call returns.
 *   - Weights are 16-bit patterns (BF16; FP16 works unchanged).  No arithmetic is done on them.
 *     Base pointers need 2-byte alignment only; 16-byte alignment takes the fast path.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call is
 *     asynchronous on it and does no host synchronisation, except where stated.
 *   - Payload layout: bucket b owns the slots I[b*cap .. b*cap+cap) and V[b*cap .. b*cap+cap).
 *     counts[b] is always the TRUE number of changed elements of bucket b.  If it exceeds cap only
 *     the first cap pairs (ascending) are stored and the SRS_FLAG_OVERFLOW device flag is raised;
 *     the snapshot is refreshed all the same, and the caller sends that bucket as a dense copy of
 *     the new weights (the full-copy route of Sec. 3.4 for dense parameters).  Slots at and beyond
 *     counts[b] are left untouched.
 *   - Return value: SRS_OK (0) or a negative srs_error.  Argument errors (SRS_ERR_INVALID,
 *     SRS_ERR_TOO_LARGE) are found before anything is launched or copied.  SRS_ERR_HIP reports a
 *     failed runtime call (allocation, copy, launch); calls that issue several kernels (the encoded
 *     applies, the value coder, every extract with its clearing kernel) may then have launched the
 *     earlier ones, so the outputs of such a call are undefined.  Device-side conditions (overflow,
 *     bad index, look-back time-out) are reported through srs_status().
 *   - A context serialises its own scratch memory: use one context per stream, and do not run
 *     two calls on the same context concurrently.  A plan caches the device copy of the last pointer
 *     arrays it was called with (one for extract-side pairs, one for apply-side weights) and is
 *     updated by the calls that take it: one host thread at a time per plan, and calls that pass
 *     DIFFERENT pointer arrays to one plan must be ordered on one stream (the array of a later call
 *     replaces the earlier one in stream order).  Callers that alternate between pointer sets keep
 *     one plan per set.
 *   - Weights of a call may not overlap each other or the payload buffers.
 *   - A context belongs to the device it was created on; every call works on that device whatever device is
 *     current in the calling thread, and leaves the caller's current device as it found it.
 */
#ifndef SRS_H
#define SRS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SRS_OK = 0,
    SRS_ERR_INVALID = -1,     /* null pointer, zero bucket size or capacity, size beyond int32 indexing */
    SRS_ERR_HIP = -2,         /* a HIP runtime call failed (allocation, copy, launch) */
    SRS_ERR_NOMEM = -3,       /* host allocation failed */
    SRS_ERR_NO_DEVICE = -4,   /* no usable GPU / wrong architecture */
    SRS_ERR_TOO_LARGE = -5    /* srs_extract_noalloc: the input needs more scratch than the library's static array holds */
} srs_error;

/* device flags reported by srs_status() */
#define SRS_FLAG_OVERFLOW  1u  /* extract: some bucket had more than cap changed elements */
#define SRS_FLAG_BAD_INDEX 2u  /* apply: an index lay outside its bucket's span and was skipped */
#define SRS_FLAG_TIMEOUT   4u  /* extract: a tile gave up waiting for its predecessors (payload invalid) */

/* options for srs_set_option() */
#define SRS_OPT_SPIN_LIMIT 1   /* max polls of a predecessor tile before SRS_FLAG_TIMEOUT (default 1<<24) */
#define SRS_OPT_TILE_ELEMS 2   /* elements per extract tile: 4096, 8192, 16384 or 32768 (default; tuning; affects
                                  plans created afterwards) */
#define SRS_OPT_REFRESH_GROUP 3 /* snapshot refresh: 8 (default) = a full tile of 16-byte-aligned weights rewrites
                                  every 128-byte run of the snapshot that holds a change (a whole line when the tensor
                                  starts on a 128-byte boundary, which is where the gain comes from), from the
                                  new weights (unchanged elements get the value they have), other tiles store element
                                  by element; 0 = a store per changed element everywhere.  Same result; tuning.
                                  Applies to the extract calls of every element width and to the fused cast. */
#define SRS_OPT_INTERLEAVE 4   /* buckets whose tiles are interleaved over consecutive workgroups, 1..4096
                                  (default 64; tuning; affects plans created afterwards) */
#define SRS_OPT_SNAPSHOT 5     /* what srs_extract / srs_extract_multi do with the snapshot:
                                  0 (default) refresh it in place, so that old_snapshot == new_w afterwards;
                                  1 leave it untouched: the caller rotates buffers instead, i.e. new_w IS the
                                  snapshot of the next call and the Trainer's next cast writes into the buffer
                                  that held old_snapshot (same two resident BF16 copies, no scattered stores
                                  into the weights; Alg. 1's W_prev without the clone).  Payload identical.
                                  This mode measures best with SRS_OPT_INTERLEAVE = 256;
                                  2 refresh it in a second pass: the scan leaves it untouched as under 1, then the
                                  same call scatters the payload into it (and copies a bucket whole whose payload
                                  overflowed cap), so that old_snapshot == new_w afterwards exactly as under 0.
                                  Payload, counts and flags identical.  Keeping the stores out of the read stream
                                  pays when few elements change (at one-byte width and 0.07 % changed: 10.4 against
                                  11.8 ms on a 30.5 G-element list, both with SRS_OPT_INTERLEAVE = 256; at 16 bits and 0.1 %: 3.5 % faster; from 0.3 %
                                  up the default is faster).  Ignored, like 1, by the fused-cast and cumulative calls. */

typedef struct srs_ctx srs_ctx;    /* per-stream scratch: tile status words, per-bucket ticket counters, flag word */
typedef struct srs_plan srs_plan;  /* immutable bucket / segment / tile tables of one tensor list */

/* Context.  srs_create selects `device`, allocates a few KiB of device scratch and synchronises.
 * The tile-status and ticket arrays grow on demand inside srs_extract* (that one call then allocates
 * and synchronises the device; later calls of the same or smaller size do not). */
int srs_create(srs_ctx **out, int device);
int srs_destroy(srs_ctx *ctx);                       /* synchronises the device, frees scratch */
int srs_set_option(srs_ctx *ctx, int option, uint64_t value);
const char *srs_strerror(int err);
int srs_version(void);

/* Waits for `stream`, copies the device flag word to *flags (host pointer) and clears it. */
int srs_status(srs_ctx *ctx, uint32_t *flags, void *stream);

/*
 * Single tensor (Alg. 1 / Alg. 2 for one parameter).  old_snapshot (in/out) and new_w are n 16-bit
 * elements.  Bucket b covers the flat range [b*bucket_elems, min(n, (b+1)*bucket_elems)).
 * I[nb*cap] receives tensor-flat indices i (the per-tensor int32 index of Alg. 2), V[nb*cap] the
 * patterns new_w[i], counts[nb] the per-bucket counts; nb = ceil(n / bucket_elems).  On completion
 * old_snapshot equals new_w bitwise.  n and bucket_elems must be below 2^31 (int32 indices,
 * Sec. 3.2); n == 0 is SRS_OK and writes nothing.
 */
int srs_extract(srs_ctx *ctx, void *old_snapshot, const void *new_w, uint64_t n, uint64_t bucket_elems,
                int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream);

/*
 * srs_extract for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same payload, same snapshot refresh, same flags as srs_extract, but the
 * tile status words and ticket counters live in a static device array of the library (9 MiB per GPU, held until
 * the process ends) instead of the context's growable scratch, so the call never allocates, frees or
 * synchronises, whatever its size.  Limits: at most 2^20 tiles (a bucket has ceil(bucket_elems / SRS_OPT_TILE_ELEMS)
 * tiles: with buckets of at least one default tile of 32768 elements every n below 2^31 fits) and at most 2^18 buckets; beyond either the call returns
 * SRS_ERR_TOO_LARGE and launches nothing.  Every context on one GPU shares that GPU's array: two such calls that
 * overlap in time on one GPU (different streams or different contexts) race; order them on one stream.  The
 * array keeps the previous call's contents; a small kernel at the head of each call clears what the call uses.
 */
int srs_extract_noalloc(srs_ctx *ctx, void *old_snapshot, const void *new_w, uint64_t n, uint64_t bucket_elems,
                        int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream);

/*
 * Single tensor scatter (Alg. 3): weights[I[b*cap+r]] <- V[b*cap+r] for r < min(counts[b], cap).
 * counts is read on the device.  An index outside bucket b's span is skipped and raises
 * SRS_FLAG_BAD_INDEX; nothing is ever written out of bounds.  Duplicate indices are a caller
 * error (extract never produces them): one of the values wins.
 */
int srs_apply(srs_ctx *ctx, void *weights, uint64_t n, uint64_t bucket_elems,
              const int32_t *I, const uint16_t *V, const uint32_t *counts, uint64_t cap, void *stream);

/*
 * Tensor lists.  The tensors are laid end to end in list order, without padding, and that packed
 * space is cut into buckets of bucket_elems (the last one short); a tensor may straddle buckets and
 * a bucket may hold many tensors.  Indices are positions INSIDE the bucket (packed position minus
 * b*bucket_elems), because packed positions of a 30 B-element model do not fit int32; with the
 * plan's segment table they map one-to-one to Alg. 2's per-tensor flat indices.
 * The pointer arrays are host arrays of plan-many entries, read during the call; a tensor that has elements needs
 * every pointer the call uses, aligned to its element size (else SRS_ERR_INVALID); the entries of a tensor without
 * elements are ignored.
 */
typedef struct { void *old_snapshot; const void *new_w; } srs_tensor_pair;   /* extract side */
typedef struct { void *weights; } srs_tensor;                                 /* apply side   */

/* Builds the tables on the host and uploads them (allocates; synchronises).  numel[k] < 2^31. */
int srs_plan_create(srs_ctx *ctx, const uint64_t *numel, uint32_t ntensors, uint64_t bucket_elems,
                    srs_plan **out);
int srs_plan_info(const srs_plan *plan, uint64_t *total_elems, uint32_t *nbuckets, uint32_t *nsegments,
                  uint32_t *ntiles);
int srs_plan_destroy(srs_plan *plan);

/* Host only (touches no device): the tables srs_plan_create builds, for inspection and tests.  All output
 * pointers are HOST arrays and may be NULL; call once with NULL arrays to get the sizes.
 *   tiles[4*ntiles]     : tensor, first element inside the tensor, first element inside the bucket, length
 *   segs[4*nsegments]   : first element inside the bucket, length, tensor, first element inside the tensor
 *   seg_begin[nb+1], bucket_first[nb+1] : first segment / first tile of each bucket
 *   wg_bucket[ntiles]   : the bucket that extract's workgroup i serves
 * tile_elems and interleave as in SRS_OPT_TILE_ELEMS / SRS_OPT_INTERLEAVE. */
int srs_plan_layout(const uint64_t *numel, uint32_t ntensors, uint64_t bucket_elems, uint32_t tile_elems,
                    uint32_t interleave, uint32_t *nbuckets, uint32_t *nsegments, uint32_t *ntiles, uint32_t *tiles,
                    uint32_t *segs, uint32_t *seg_begin, uint32_t *bucket_first, uint32_t *wg_bucket);

/* t[ntensors] (host array) gives the device pointers of each tensor, in plan order.  The library
 * keeps a device copy and re-uploads it (hipMemcpyAsync on `stream`) only when a pointer changed. */
int srs_extract_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t,
                      int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream);
int srs_apply_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t,
                    const int32_t *I, const uint16_t *V, const uint32_t *counts, uint64_t cap, void *stream);

/*
 * Per-tensor view of a list payload.  Alg. 2's message is, per parameter tensor, (name, I, V) with I the int32
 * indices into that tensor's flattened elements; the list calls store positions inside the bucket.  This call
 * gives the former from the latter: for r < min(counts[b], cap), tensor_id[b*cap + r] = the list position k of
 * the tensor that holds the pair and tensor_idx[b*cap + r] = its flat index inside tensor k (device arrays laid
 * out like I; other slots are left alone).  Within a bucket the pairs of one tensor are contiguous and ascending,
 * tensors in list order.  A position outside its bucket raises SRS_FLAG_BAD_INDEX and its slot is left alone.
 */
int srs_tensor_indices(srs_ctx *ctx, srs_plan *plan, const int32_t *I, const uint32_t *counts, uint64_t cap,
                       uint32_t *tensor_id, int32_t *tensor_idx, void *stream);

/*
 * One-byte elements.  The changed-element density is measured at BF16, FP16 and FP8 synchronisation precision
 * (Sec. 2.1); Alg. 1-3 compare and move opaque patterns and do not depend on their width.  FP16 weights go
 * through the 16-bit calls above unchanged.  These four calls are the same operations on 8-bit patterns (FP8 in
 * either of its formats, or any other one-byte type): old_snapshot / new_w / weights hold n (or numel[k]) bytes,
 * V is uint8_t[nb*cap]; indices, counts, capacity rule, flags, snapshot semantics (SRS_OPT_SNAPSHOT included) and
 * error behaviour are those of the 16-bit calls.  No alignment is required (16-byte aligned tensors take the
 * vector path).  A plan serves both widths.  Restrictions: SRS_OPT_TILE_ELEMS 4096 is rejected with
 * SRS_ERR_INVALID (a one-byte tile is at least 8192 elements).  The fused cast, the cumulative set, the index coding of an
 * existing payload (srs_encode_indices reads I only) and the routing work as they stand or do not apply; an
 * encoded apply and a value coder for one-byte values are not provided.
 */
int srs_extract_u8(srs_ctx *ctx, void *old_snapshot, const void *new_w, uint64_t n, uint64_t bucket_elems,
                   int32_t *I, uint8_t *V, uint32_t *counts, uint64_t cap, void *stream);
int srs_apply_u8(srs_ctx *ctx, void *weights, uint64_t n, uint64_t bucket_elems,
                 const int32_t *I, const uint8_t *V, const uint32_t *counts, uint64_t cap, void *stream);
int srs_extract_multi_u8(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t,
                         int32_t *I, uint8_t *V, uint32_t *counts, uint64_t cap, void *stream);
int srs_apply_multi_u8(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t,
                       const int32_t *I, const uint8_t *V, const uint32_t *counts, uint64_t cap, void *stream);

/*
 * Fused cast + diff.  The Trainer's hook sits where the FP32 master weights are cast and copied into the BF16
 * model parameters (Alg. 1: CastAndCopy, then I_t = { i : W[i] != W_prev[i] }; Sec. 3.4 "Trainer").  These
 * calls do both at once, so that no snapshot W_prev exists: for every element r = round_BF16(master[i]);
 * if r differs bitwise from weights[i] the pair (i, r) is emitted; weights[i] <- r.  `weights` holds the old
 * model parameters on entry and the new ones on completion; the payload is exactly what srs_extract(old =
 * weights before, new = round_BF16(master)) would give, with the same layout, capacity rule and flags.
 * round_BF16 rounds the binary32 value to the nearest BF16, ties to even; a NaN becomes 0x7FC0.
 * master: device pointer(s) to FP32 data, 4-byte aligned (16-byte alignment of both buffers takes the vector
 * path).  In the list form t[k].old_snapshot is tensor k's BF16 model parameters and t[k].new_w its FP32
 * master weights.
 */
int srs_extract_cast(srs_ctx *ctx, void *weights, const float *master, uint64_t n, uint64_t bucket_elems,
                     int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream);
int srs_extract_cast_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t,
                           int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream);

/*
 * Cumulative changed-index set: Alg. 1 as printed.  Between two synchronisations the Trainer takes T optimizer
 * steps; after each cast it forms I_t = { i : W[i] != W_prev[i] } and accumulates I_cum <- I_cum U I_t; at the
 * synchronisation Alg. 2 sends V = W[I_cum] with the CURRENT values.  I_cum is a superset of the exact delta
 * (an element that changed and changed back stays in it), which costs payload but not correctness: the receiver
 * ends bit-identical.  No snapshot of the last synchronised state is kept in this mode.
 *
 * The set is a device bitmap over the packed positions g of the plan's tensor list: bit (g & 31) of 32-bit word
 * g >> 5, srs_bitmap_words(total) words, cleared by the caller (e.g. hipMemsetAsync) after each synchronisation.
 *   srs_mark_multi       bitmap |= (t[k].new_w != t[k].old_snapshot), both BF16: one step, two versions at hand.
 *   srs_cast_mark_multi  the Trainer's own step without the clone: t[k].old_snapshot is the BF16 model parameters
 *                        (in/out), t[k].new_w the FP32 master weights; parameters <- round_BF16(master) and every
 *                        element whose pattern changed is marked.
 *   srs_extract_marked_multi  the payload of the marked positions, ascending per bucket, with the current values
 *                        of t[k].weights; layout, capacity rule and flags as srs_extract_multi.  Only the bitmap
 *                        and the marked elements are read (a gather), not the whole weight set.
 */
uint64_t srs_bitmap_words(uint64_t total_elems);
int srs_mark_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t, uint32_t *bitmap, void *stream);
int srs_cast_mark_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t, uint32_t *bitmap, void *stream);
int srs_extract_marked_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t, const uint32_t *bitmap,
                             int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream);

/*
 * Lossless index coding (Sec. 3.3, "Index delta encoding"): the indices of a payload are sorted, so their
 * first differences (with a zero prepended) are stored instead; when every difference of a bucket is below
 * 2^15 they fit 16 bits (b_i = 2 B instead of 4 B), otherwise the bucket keeps its 32-bit indices.
 *
 * srs_encode_indices reads an extract payload (I, counts; same layout and cap) and writes, per bucket b,
 *   D[b*cap + r]   = (pos[r] - pos[r-1]) mod 2^16, pos[-1] = 0, where pos = I - b*base_stride is the position
 *                    inside the bucket (base_stride = 0 for list payloads, bucket_elems for single-tensor ones),
 *   max_gap[b]     = the bucket's largest difference (0 if empty): D is exact iff max_gap[b] < 32768,
 *   anchors[b*nchunk + k] = pos[k*2048] for every started chunk of 2048 pairs, nchunk = ceil(cap/2048)
 *                    (srs_anchor_count(nbuckets, cap) entries; redundant metadata of 4 B per 2048 pairs that
 *                    lets the receiver decode chunks independently).
 * A bucket is then sent as (D, V) at 4 B per pair, or as (I, V) at 6 B per pair when max_gap[b] >= 32768.
 * Indices that do not ascend raise SRS_FLAG_BAD_INDEX and force that bucket to 32-bit transport.
 *
 * srs_apply_encoded / srs_apply_multi_encoded are srs_apply / srs_apply_multi for such payloads: buckets with
 * max_gap[b] < 32768 are decoded from D (running sums from the chunk's anchor) and scattered in one kernel,
 * the others are scattered from I_wide (only their slots of I_wide are read).  All arrays are device pointers.
 */
uint64_t srs_anchor_count(uint32_t nbuckets, uint64_t cap);
int srs_encode_indices(srs_ctx *ctx, const int32_t *I, const uint32_t *counts, uint32_t nbuckets, uint64_t cap,
                       uint64_t base_stride, uint16_t *D, uint32_t *max_gap, int32_t *anchors, void *stream);
int srs_apply_encoded(srs_ctx *ctx, void *weights, uint64_t n, uint64_t bucket_elems, const uint16_t *D,
                      const int32_t *I_wide, const uint16_t *V, const uint32_t *counts, const uint32_t *max_gap,
                      const int32_t *anchors, uint64_t cap, void *stream);
int srs_apply_multi_encoded(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t, const uint16_t *D,
                            const int32_t *I_wide, const uint16_t *V, const uint32_t *counts, const uint32_t *max_gap,
                            const int32_t *anchors, uint64_t cap, void *stream);

/*
 * Lossless value coding (Sec. 3.3, "Value entropy coding"): the BF16 values of a payload cluster in a few binades,
 * so the value stream compresses under a standard entropy coder; the paper names none and reports that the stream
 * shrinks to 0.60-0.70 of its size.  The coder here is a static Huffman code on the part of a value that carries
 * the redundancy: each value is split into its high byte (sign, upper seven exponent bits) and its low byte (lowest
 * exponent bit, mantissa); low bytes are kept as they are, the high bytes of one bucket are coded with a code built
 * from that bucket's own histogram.
 *
 * Code construction (fixed, so that independent implementations agree bit for bit):
 *   1. hist[s] over the high bytes of the bucket's min(counts[b], cap) values.
 *   2. Huffman lengths: repeatedly merge the two live nodes of smallest weight, ties to the smaller id; leaves have
 *      id = symbol, the k-th merged node id 256 + k.  A lone symbol gets length 1, an absent one length 0.
 *   3. While some length exceeds 12: every non-zero weight w becomes (w + 1) / 2 and step 2 is repeated.
 *   4. Canonical codes as in DEFLATE: symbols ordered by (length, symbol) take consecutive code values.
 * Stream layout per bucket, chunks of 2048 values, nchunk = srs_value_chunks(cap):
 *   lens[b*256 + s]                       code lengths (the code follows from them)
 *   low[b*cap + r]                        low bytes
 *   bits[(b*nchunk + k)*768 ...]          chunk k's code bits, most significant code bit first, bit i of the chunk =
 *                                         bit (i & 31) of word i >> 5; chunk_words[b*nchunk + k] words are used
 *                                         (0 for a chunk without values); words beyond that are unspecified
 *   sub[(b*nchunk + k)*32 + j]            bit position inside the chunk where its value j*64 starts
 * Wire size of a bucket = 256 + count + 4*sum(chunk_words) + 64 per started chunk bytes, against 2*count raw.
 * srs_decode_values is the inverse (V_out[b*cap + r] for r < min(counts[b], cap)); a stream that does not decode
 * under its own table raises SRS_FLAG_BAD_INDEX.  All pointers are device pointers; asynchronous on `stream`
 * (the first encode at a larger bucket count grows a small scratch array: allocation + synchronisation).
 */
uint64_t srs_value_chunks(uint64_t cap);
int srs_encode_values(srs_ctx *ctx, const uint16_t *V, const uint32_t *counts, uint32_t nbuckets, uint64_t cap,
                      uint8_t *lens, uint8_t *low, uint32_t *bits, uint32_t *chunk_words, uint16_t *sub, void *stream);
int srs_decode_values(srs_ctx *ctx, const uint8_t *lens, const uint8_t *low, const uint32_t *bits,
                      const uint32_t *chunk_words, const uint16_t *sub, const uint32_t *counts, uint32_t nbuckets,
                      uint64_t cap, uint16_t *V_out, void *stream);

/*
 * Density routing (Sec. 3.4, WeightUpdater): parameters that are highly sparse take the (I, V) route, those
 * that change on nearly every element are sent as a full copy.  The unit here is the bucket and the rule is
 * the break-even of the cost model, Eq. (1): bucket b of len_b elements goes dense when
 *     counts[b] > cap      (it overflowed its slot)      or
 *     counts[b] * bytes_per_pair >= 2 * len_b            (6 B per pair with int32 indices, 4 B with 16-bit
 *                                                         differences: break-even density 1/3 resp. 1/2).
 * srs_route reads counts[nbuckets] and writes route_slot[b] (-1 = sparse, else the bucket's place s among the
 * dense buckets, in bucket order), dense_bucket[s] = b, sparse_counts[b] (= counts[b] for sparse buckets, 0 for
 * dense ones: pass it to srs_apply* in place of counts and the dense buckets are skipped there) and *n_dense.
 * At most max_dense buckets go dense; a further candidate stays sparse, truncated to cap, and raises
 * SRS_FLAG_OVERFLOW.  All pointers are device pointers; one small kernel, asynchronous.
 *
 * srs_pack_dense_multi gathers the new weights (t[k].new_w) of the dense buckets into dense[s*bucket_elems ..),
 * the message body of the full-copy route; srs_unpack_dense_multi writes such bodies into the resident
 * weights.  Both read dense_bucket and n_dense on the device (max_dense bounds the launch).
 */
int srs_route(srs_ctx *ctx, const uint32_t *counts, uint32_t nbuckets, uint64_t bucket_elems, uint64_t total_elems,
              uint64_t cap, uint32_t bytes_per_pair, uint32_t max_dense, int32_t *route_slot, uint32_t *sparse_counts,
              int32_t *dense_bucket, uint32_t *n_dense, void *stream);
int srs_pack_dense_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t, const int32_t *dense_bucket,
                         const uint32_t *n_dense, uint32_t max_dense, uint16_t *dense, void *stream);
int srs_unpack_dense_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t, const int32_t *dense_bucket,
                           const uint32_t *n_dense, uint32_t max_dense, const uint16_t *dense, void *stream);

/*
 * Measurement aid (not part of the method): reads `bytes` bytes from each of a and b with the same
 * 16-byte streaming loads (non-temporal hint) and launch shape as extract and writes one word per workgroup to `sink`
 * (at least srs_stream_probe_sink_words(bytes) uint32).  Gives the box's achievable two-stream read
 * bandwidth, the practical ceiling for extract.  a, b 16-byte aligned; bytes a multiple of 16.
 */
int srs_stream_probe(srs_ctx *ctx, const void *a, const void *b, uint64_t bytes, uint32_t *sink, void *stream);
uint64_t srs_stream_probe_sink_words(uint64_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* SRS_H */
