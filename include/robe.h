/*
 * robe.h - C ABI of the MI355X (gfx950) ROBE-Z embedding library.
 *
 * ROBE ("Random Offset Block Embedding Array", arXiv 2108.02191) replaces all
 * embedding tables of a recommendation model by ONE circular array M of m
 * floats.  The d-element embedding of token x of table e is the
 * concatenation of d/Z blocks of Z consecutive array elements (wrapping past
 * the end), block c starting at a universally hashed offset h(e,x,c); each
 * element may be multiplied by a hashed sign g(e,x,i).  Gradients flow back
 * by a signed sum into the same array.
 *
 * Equation numbers below count the paper's displayed equations in order:
 *   Eq. 1  ROBE-D forward            (Section 3.1)
 *   Eq. 2  h, idx and g for ROBE-D   (Section 3.1)
 *   Eq. 3  backward pass             (Section 3.1)
 *   Eq. 4  ROBE-Z forward            (Section 3.2)
 *   Eq. 5  h and idx for ROBE-Z      (Section 3.2)
 *
 * General rules of this interface
 *   - Plain C: pointers and sizes only.  "device" pointers are HIP device
 *     memory of the current device, "host" pointers are ordinary memory.
 *   - The caller owns every buffer.  The library allocates nothing, frees
 *     nothing and never synchronises: all GPU work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream) and the
 *     call returns at once.  Buffers must stay valid until that work is done.
 *   - Every function returns ROBE_OK (0) or a negative error code and never
 *     aborts.  robe_last_error() gives the text of the calling thread's most
 *     recent failure.  Arguments are validated on the host before anything is
 *     launched; a failed call launches nothing.
 *   - Calls that launch kernels take a `const robe_options_t *options`; NULL means
 *     the defaults (every field zero).  Options are read during the call only and
 *     are the only thing besides the arguments that a call depends on: the library
 *     keeps no process-wide settings and reads no environment variables.
 *   - Token ids are int64 and are read as unsigned 64-bit integers in the hash
 *     formulas (a negative id is the integer id + 2^64).  No cardinality is
 *     needed: hashing accepts any id.
 *   - Index conventions are 0-based: table id e = feature column, element
 *     i in [0,d), chunk c = i / Z, position in chunk j = i mod Z.
 *   - Layouts: single-hot ids `indices[batch][n_features]`; bags in (b,f)
 *     row-major order, bag k = b*n_features + f, CSR `offsets[batch*n_features+1]`,
 *     non-decreasing with offsets[0] = 0 and offsets[last] = n_indices,
 *     `indices[n_indices]`;
 *     `out` / `grad_out` are `[batch][n_features][d]` float32, row-major.
 */
#ifndef ROBE_H
#define ROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROBE_OK       0
#define ROBE_EINVAL  (-1)  /* bad argument: null pointer, bad shape, value out of range */
#define ROBE_EHIP    (-2)  /* a HIP runtime call or kernel launch failed                 */

#define ROBE_PRIME 2147483647u /* P = 2^31 - 1, the prime modulus of Eq. 2 / Eq. 5 */

/*
 * One ROBE-Z instance (Eq. 5 and the text under it; g from Eq. 2).
 * Plain data, owned by the caller, copied by value into kernel arguments.
 *   m          array length in floats, 1 <= m <= 2^31 - 1
 *   d, Z       embedding size and block size, Z >= 1, Z <= m, and either Z divides d
 *              or d divides Z (Section 3.3: r = Z/d consecutive tokens of a table share a
 *              block; then idx(e,x,i) = (h(e, x / r, 0) + (x mod r)*d + i) mod m)
 *   use_sign   0: g == +1 everywhere; non-zero: g as in Eq. 2
 *   P          must be ROBE_PRIME
 *   Ah,Bh,Ch   multipliers of h in [1, P-1];  Dh additive constant in [0, P-1]
 *   Ag,Bg,Cg   multipliers of g in [1, P-1];  Dg additive constant in [0, P-1]
 *
 *   h(e,x,c)   = ((Ah*e + Bh*x + Ch*c + Dh) mod P) mod m
 *   idx(e,x,i) = (h(e,x,i / Z) + i mod Z) mod m
 *   g(e,x,i)   = 2*(((Ag*e + Bg*x + Cg*i + Dg) mod P) mod 2) - 1
 * all evaluated over the integers.
 */
typedef struct robe_hash_t {
    uint64_t m;
    uint32_t d, Z;
    uint32_t use_sign;
    uint32_t P;
    uint32_t Ah, Bh, Ch, Dh;
    uint32_t Ag, Bg, Cg, Dg;
} robe_hash_t;

/*
 * Per-call choices.  All-zero is "let the library decide" for every field; a value the field does
 * not define makes the call fail with ROBE_EINVAL.  Apart from `reproducible` they exist for
 * measurements and for tests that must reach every kernel variant; results are the same to
 * rounding whatever is chosen.
 *
 *   reproducible   1: run-to-run reproducible backward.  Eq. 3 sums float32 terms in an order the
 *                  paper does not fix; with float atomics that order, and so the last bits of the
 *                  result, change from run to run.  With this set, robe_backward, robe_backward_mixed
 *                  and robe_backward_adagrad take the route that has no float atomic (blocks sorted by
 *                  destination region, one workgroup per region) and add every slice's blocks in a
 *                  canonical order: the same call on the same inputs on the same device gives the same
 *                  bits every time.  It costs a few per cent on large problems, more on small ones, and
 *                  the larger workspace (pass the same options to the workspace query).  A shape or
 *                  size that route cannot take (see robe_backward) fails with ROBE_EINVAL rather than
 *                  giving up reproducibility.  Forward and the update rules are reproducible always.
 *   backward_route ROBE_ROUTE_AUTO, or a request for one scatter strategy: _DIRECT (one float atomic
 *                  per element), _COMBINE (tokens sorted, repeated tokens summed, atomics once per
 *                  distinct token) or _REGIONS (no float atomics).  A request that the shape or size
 *                  cannot follow falls back to _DIRECT (the workspace query then reports 0 bytes);
 *                  `reproducible` overrides it.
 *   fused_route    how robe_backward_adagrad runs: ROBE_ROUTE_AUTO, _REGIONS (scatter and update in
 *                  one pass) or _TWO_STEP (scatter into a gradient array in the workspace, then the
 *                  update kernel).
 *   fwd_elems, fwd_strided / bwd_elems, bwd_strided
 *                  lane layout of the gather / direct-scatter kernels: elements per lane (1, 2 or 4;
 *                  also 3, 6, 8 when strided; d / elems must be a power of two <= 64), owned as
 *                  consecutive elements of one chunk (strided = 0) or as elements lane + k * lanes
 *                  (strided = 1).  elems = -1 selects the shape-generic kernel, 0 the default.
 *   tile_lookups   lookups per wavefront tile of the single-hot kernels (a multiple of 64 / lanes, <= 64)
 *   row_order      ROBE_ROWS_AUTO, _MEMORY (rows in memory order), _BY_TABLE (table by table, one
 *                  eighth of that order per XCD, when the launch is large enough to matter) or
 *                  _BY_TABLE_ALWAYS
 *   tile_combine   direct single-hot scatter: 0 by size, 1 never, 2 always combine the duplicates of
 *                  every tile of 64 lookups before the atomics
 *   region_shift   log2 of the region size in floats for ROBE_ROUTE_REGIONS, 10..15
 *   key_bits       most significant bits of the 31-bit token key that the sort looks at, 8..31
 *                  (with Z > d the key is an array offset below m: at most ceil(log2 m) bits)
 *   region_records 0 by size, 1: ROBE_ROUTE_REGIONS writes a region-sorted copy of the block records,
 *                  2: the region workgroups look their blocks up in the sorted token list instead
 *   probe_kernel, probe_begin, probe_end
 *                  a measurement aid.  With probe_kernel = ROBE_PROBE_* and two hipEvent_t handles,
 *                  a backward call records probe_begin on the stream just before the named kernel of
 *                  the sorted routes and probe_end just after it, so that a benchmark can time that one
 *                  kernel inside the call (calls that do not launch it record neither).
 *                  ROBE_PROBE_NONE (0) or NULL events: nothing is recorded.
 */
typedef struct robe_options_t {
    int32_t reproducible;
    int32_t backward_route;
    int32_t fused_route;
    int32_t fwd_elems, fwd_strided;
    int32_t bwd_elems, bwd_strided;
    int32_t tile_lookups;
    int32_t row_order;
    int32_t tile_combine;
    int32_t region_shift;
    int32_t key_bits;
    int32_t region_records;
    int32_t probe_kernel;
    int32_t reserved[2];      /* must be zero */
    void *probe_begin, *probe_end;
} robe_options_t;

#define ROBE_PROBE_NONE     0
#define ROBE_PROBE_COMBINE  1   /* the kernel that sums the rows of repeated tokens (both sorted routes) */
#define ROBE_PROBE_REDUCE   2   /* the per-region reduce kernel of ROBE_ROUTE_REGIONS                    */
#define ROBE_PROBE_SORT     3   /* the radix sort passes, first count kernel to last scatter kernel      */

#define ROBE_ROUTE_AUTO      0
#define ROBE_ROUTE_DIRECT    1
#define ROBE_ROUTE_COMBINE   2
#define ROBE_ROUTE_REGIONS   3
#define ROBE_ROUTE_TWO_STEP  4

#define ROBE_ROWS_AUTO             0
#define ROBE_ROWS_MEMORY           1
#define ROBE_ROWS_BY_TABLE         2
#define ROBE_ROWS_BY_TABLE_ALWAYS  3

/*
 * Draw the hash coefficients from a seed (host only; Section 3.2: "randomly
 * chosen values").  The stream is SplitMix64 (Steele, Lea, Flood 2014) started
 * at state `seed`; eight successive outputs r give, in this order,
 * Ah,Bh,Ch = 1 + r mod (P-1), Dh = r mod P, Ag,Bg,Cg = 1 + r mod (P-1),
 * Dg = r mod P.  `out` (host) receives the complete struct.
 * Errors: ROBE_EINVAL for out == NULL or shapes that violate the rules above.
 */
int robe_init_hash(uint64_t seed, uint64_t m, uint32_t d, uint32_t Z, int use_sign, robe_hash_t *out);

/*
 * Testing aid: the integer maps alone (Eq. 5 for h, Eq. 2 for g).
 *   indices      device int64[n]; lookup k belongs to table k mod n_features
 *   out_offsets  device int64[n * d/Z] or NULL:  out_offsets[k*(d/Z) + c] = h(e,x,c);
 *                for Z > d: int64[n], out_offsets[k] = idx(e,x,0)
 *   out_signs    device int8 [n * d]   or NULL:  out_signs[k*d + i] = g(e,x,i)
 * Errors: ROBE_EINVAL (null hash/indices with n > 0, n < 0, n_features < 1,
 * invalid hash); ROBE_EHIP on launch failure.  n == 0 is a no-op.
 */
int robe_offsets(const robe_hash_t *hash, const int64_t *indices, int64_t n, int32_t n_features,
                 int64_t *out_offsets, int8_t *out_signs, void *stream);

/*
 * Forward lookup (Eq. 4 with idx from Eq. 5, E = G o P).
 *   array      device float[m], read only
 *   indices    device int64[n_indices]
 *   offsets    NULL: single-hot, n_indices must equal batch*n_features and
 *                    out[k][i] = g(f,x_k,i) * array[idx(f,x_k,i)]   (a copy with an exact sign flip)
 *              device int64[batch*n_features + 1]: bag-sum,
 *                    out[k][i] = sum over t in [offsets[k], offsets[k+1]) of g(f,x_t,i) * array[idx(f,x_t,i)],
 *                    duplicates counted each time, empty bag -> +0.0, summed in
 *                    float32 in token order.  Bag bounds are clamped to
 *                    [0, n_indices] on the device, so a malformed CSR cannot
 *                    read outside `indices`.
 *   out        device float[batch][n_features][d], fully overwritten
 *   options    NULL or host robe_options_t (fwd_elems, fwd_strided, tile_lookups, row_order are read)
 * Errors: ROBE_EINVAL, ROBE_EHIP.  batch == 0 is a no-op.
 */
int robe_forward(const robe_hash_t *hash, const float *array,
                 const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                 int64_t batch, int32_t n_features, float *out,
                 const robe_options_t *options, void *stream);

/*
 * Bytes of device workspace robe_backward needs for this problem size and these options, for
 * either kind of input (single-hot or bags), written to *bytes (host); 0 when none is needed
 * (small problems scatter directly).  Host arithmetic only: no device is touched.
 * Errors: ROBE_EINVAL (bad hash, sizes or options, bytes == NULL; options->reproducible set for a
 * shape or size that has no reproducible route); *bytes is 0 then.
 */
int robe_workspace_bytes(const robe_hash_t *hash, int64_t batch, int32_t n_features, int64_t n_indices,
                         const robe_options_t *options, size_t *bytes);

/*
 * Backward scatter-add (Eq. 3):
 *   grad_array[j] += sum over (k, t, i) with idx(f,x_t,i) == j of g(f,x_t,i) * grad_out[k][i]
 * where every token t of bag k receives row k of grad_out (single-hot: one
 * token per row).  Accumulates onto the caller's grad_array (device float[m]);
 * the order of the float32 additions is not fixed, so results agree with an
 * exact sum only to rounding.  Small scatters issue one float atomic per
 * element (ROBE_ROUTE_DIRECT).  Larger ones first combine the gradient rows of repeated tokens
 * (sort by the token part of the hash, run-wise sums) and issue the atomics
 * once per run (ROBE_ROUTE_COMBINE); the largest (arrays of 2^26 slots or more with 2^21 tokens or
 * more) then collect the blocks by destination region and sum each region in LDS,
 * with no float atomic at all (ROBE_ROUTE_REGIONS; the route of the reproducible option).  The
 * sorted routes need the workspace, rows and n_indices below 2^31 - 1 and d <= 512 (with Z > d,
 * Section 3.3, tokens are sorted by the array offset of their d slots instead of the token hash);
 * ROBE_ROUTE_REGIONS also needs d / Z and the lane group to be powers of two, at most 2^30 array
 * slots, and a region size (2^10 .. 2^15 floats, at least 2 Z) that leaves the array's last region
 * either full or at least Z floats long.
 * With a CSR that is not non-decreasing, bag bounds
 * are clamped to [0, n_indices] so nothing outside the buffers is touched, but
 * which tokens such bags hold is unspecified here.  Every route records kernels
 * only on the stream (no fill or copy operations, no synchronisation), so the
 * call may be captured into a HIP graph.
 *   workspace  device buffer of at least robe_workspace_bytes(...) bytes (same options),
 *              256-byte aligned, contents undefined before and after; may be
 *              NULL when that size is 0
 * Errors: ROBE_EINVAL (also: workspace too small), ROBE_EHIP.
 */
int robe_backward(const robe_hash_t *hash, const float *grad_out,
                  const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                  int64_t batch, int32_t n_features, float *grad_array,
                  void *workspace, size_t workspace_bytes,
                  const robe_options_t *options, void *stream);

/*
 * robe_backward for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, result
 * and routes as robe_backward, but the workspace is a buffer built into the library: a fixed
 * robe_noalloc_max_workspace_bytes() = 32 MiB of device memory per GPU, present from the moment the
 * library is loaded until the process ends.  The call allocates and frees nothing (no hipMalloc, no
 * library routine that allocates); its first use on a device looks the buffer's address up once.
 * A problem whose workspace (robe_workspace_bytes with the same options) exceeds the buffer fails with
 * ROBE_EINVAL and launches nothing; problems that scatter directly need no workspace and have no
 * size limit.  The buffer holds nothing between calls that a call relies on.  All calls on one GPU
 * share it: two such calls that overlap in time on one GPU (different streams, or different threads)
 * race and give wrong results - order them on one stream or with events.
 * Errors: as robe_backward, plus ROBE_EHIP if the buffer's address cannot be obtained.
 */
size_t robe_noalloc_max_workspace_bytes(void);
int robe_backward_noalloc(const robe_hash_t *hash, const float *grad_out,
                          const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                          int64_t batch, int32_t n_features, float *grad_array,
                          const robe_options_t *options, void *stream);

/*
 * Sparse Adagrad step on the touched slots (Duchi, Hazan, Singer 2011; the
 * optimizer is named by the workload, not by the paper).  For every j with
 * grad_array[j] != 0, in float32 with each operation rounded on its own:
 *   state[j] += grad_array[j]^2
 *   array[j] -= lr * grad_array[j] / (sqrt(state[j]) + eps)
 *   grad_array[j] = 0
 * Slots with a zero gradient are left bit-for-bit unchanged, which is what a
 * dense Adagrad step does to them too.  All three are device float[m].
 * Errors: ROBE_EINVAL (null pointers, eps <= 0, non-finite lr/eps), ROBE_EHIP.
 */
int robe_adagrad_update(const robe_hash_t *hash, float *array, float *state, float *grad_array,
                        float lr, float eps, void *stream);

/*
 * Sparse SGD step on the touched slots, the rule the paper trains DLRM with
 * (Appendix, hyper-parameter table: SGD, learning rate 1.0).  For every j with
 * grad_array[j] != 0, in float32 with each operation rounded on its own:
 *   array[j] -= lr * grad_array[j]
 *   grad_array[j] = 0
 * Slots with a zero gradient are left bit-for-bit unchanged.  Both are device float[m].
 * Errors: ROBE_EINVAL (null pointers, non-finite lr), ROBE_EHIP.
 */
int robe_sgd_update(const robe_hash_t *hash, float *array, float *grad_array, float lr, void *stream);

/*
 * Fused training step: backward scatter-add (Eq. 3) and the Adagrad update in one pass, for a
 * gradient array that would otherwise start from zero.  The result is that of
 *   robe_backward(..., grad_array = zeros, ...) followed by robe_adagrad_update(array, state, grad_array)
 * to the same rounding caveats, but on large arrays the gradient never exists in device memory:
 * the blocks are collected by destination region, every region of the array is summed in LDS by the
 * one workgroup that owns it, and that workgroup updates array and state directly.  Slots that
 * receive no gradient are left bit-for-bit unchanged, and regions that receive none are not read.
 *   array, state   device float[m], updated in place
 *   workspace      device buffer of at least robe_fused_workspace_bytes(...) bytes (same options),
 *                  256-byte aligned (it holds the sort buffers, the summed rows of repeated tokens and
 *                  the block records; for problems too small or shapes too odd for the sorted path it
 *                  holds a gradient array instead and the two steps run one after the other)
 * robe_fused_workspace_bytes is host arithmetic like robe_workspace_bytes and fails the same way.
 * Errors: ROBE_EINVAL (null pointers, eps <= 0, non-finite lr/eps, workspace too small), ROBE_EHIP.
 * Like robe_backward it records kernels only and may be captured into a HIP graph.
 */
int robe_fused_workspace_bytes(const robe_hash_t *hash, int64_t batch, int32_t n_features, int64_t n_indices,
                               const robe_options_t *options, size_t *bytes);
int robe_backward_adagrad(const robe_hash_t *hash, const float *grad_out,
                          const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                          int64_t batch, int32_t n_features, float *array, float *state,
                          float lr, float eps, void *workspace, size_t workspace_bytes,
                          const robe_options_t *options, void *stream);

/*
 * The same with the SGD rule of robe_sgd_update (the rule the paper trains DLRM with, Appendix,
 * hyper-parameter table): array[j] -= lr * (sum of Eq. 3 for slot j), in float32 with the product and
 * the difference rounded on their own, for every slot that receives a gradient; the others are left
 * bit-for-bit unchanged.  Routes, workspace (robe_fused_workspace_bytes, same options) and errors as
 * robe_backward_adagrad; there is no state.
 */
int robe_backward_sgd(const robe_hash_t *hash, const float *grad_out,
                      const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                      int64_t batch, int32_t n_features, float *array, float lr,
                      void *workspace, size_t workspace_bytes,
                      const robe_options_t *options, void *stream);

/*
 * Tables of different embedding dimensions sharing the one array (Section 3.2, "Multiple embedding
 * tables": all tables, even with varying dimensions, share the array; the table id is an argument of
 * h and g).  Table f has dimension dims[f], a positive multiple of Z or a divisor of it; its
 * embedding is Eq. 4 / Eq. 5 with d = dims[f] (for a divisor: Section 3.3, Z / dims[f] consecutive
 * tokens of the table share a block; hash->d is not used).  A sample's row is the concatenation of
 * its tables' embeddings: out and grad_out are device float[batch][D], D = dims[0] + ... +
 * dims[n_features-1], table f at column dims[0] + ... + dims[f-1].  indices / offsets / n_indices /
 * batch are as in robe_forward; dims is a HOST array of n_features entries, read during the call only.
 * robe_forward_mixed makes one launch per run of consecutive tables of equal dimension.
 * robe_backward_mixed accumulates onto grad_array like robe_backward.  Large scatters (the size rule
 * of robe_backward on the average dimension; every dimension a multiple of Z, the largest at most
 * 512, batch * D below 2^32) sort the tokens of all tables once and combine repeated tokens before
 * the atomics (ROBE_ROUTE_COMBINE; two tokens are the same when key and table agree), or, when
 * ROBE_ROUTE_REGIONS or options->reproducible asks for it, take the region route with no float
 * atomics (same conditions as robe_backward, on the largest dimension); anything else is one direct
 * scatter per run of equal dimensions.  With options->reproducible a shape the region route cannot
 * take (a table narrower than the block among them) fails with ROBE_EINVAL.
 * robe_backward_adagrad_mixed is robe_backward_adagrad for such tables: the fused region route where
 * the plan has one (by default on arrays of 2^26 slots or more), else the scatter into a gradient
 * array at the front of the workspace followed by the update kernel.  Otherwise follow
 * robe_backward_mixed with robe_adagrad_update / robe_sgd_update.
 *   workspace  device buffer of at least robe_mixed_workspace_bytes(...) bytes
 *              (robe_fused_mixed_workspace_bytes for the fused call; same dims and options),
 *              256-byte aligned; may be NULL when that size is 0
 * Errors: ROBE_EINVAL (also: a dims entry that is zero or neither a multiple nor a divisor of Z;
 * workspace too small), ROBE_EHIP.
 */
int robe_forward_mixed(const robe_hash_t *hash, const uint32_t *dims, const float *array,
                       const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                       int64_t batch, int32_t n_features, float *out,
                       const robe_options_t *options, void *stream);
int robe_mixed_workspace_bytes(const robe_hash_t *hash, const uint32_t *dims, int64_t batch, int32_t n_features,
                               int64_t n_indices, const robe_options_t *options, size_t *bytes);
int robe_backward_mixed(const robe_hash_t *hash, const uint32_t *dims, const float *grad_out,
                        const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                        int64_t batch, int32_t n_features, float *grad_array,
                        void *workspace, size_t workspace_bytes,
                        const robe_options_t *options, void *stream);
int robe_fused_mixed_workspace_bytes(const robe_hash_t *hash, const uint32_t *dims, int64_t batch, int32_t n_features,
                                     int64_t n_indices, const robe_options_t *options, size_t *bytes);
int robe_backward_adagrad_mixed(const robe_hash_t *hash, const uint32_t *dims, const float *grad_out,
                                const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                                int64_t batch, int32_t n_features, float *array, float *state,
                                float lr, float eps, void *workspace, size_t workspace_bytes,
                                const robe_options_t *options, void *stream);

/*
 * Low-precision array (Section 2 notes that quantisation can be applied together with the method;
 * it fixes no format).  The array is stored as bfloat16 bit patterns, uint16_t[m]: the upper half of
 * the float32 pattern.  robe_array_to_bf16 converts a float32 device array (round to nearest, ties
 * to even; NaN stays NaN) - post-hoc quantisation of a trained array; dst may not overlap src.
 * robe_forward_bf16 is robe_forward on such an array: every element read is widened exactly (16 zero
 * bits appended), sign, bag-sum and output are float32 as before, so a single-hot lookup returns
 * exactly the stored values.  Half the array bytes per lookup; training keeps the float32 array.
 * Errors: ROBE_EINVAL, ROBE_EHIP.
 */
int robe_array_to_bf16(const float *src, uint16_t *dst, uint64_t n, void *stream);
int robe_forward_bf16(const robe_hash_t *hash, const uint16_t *array,
                      const int64_t *indices, const int64_t *offsets, int64_t n_indices,
                      int64_t batch, int32_t n_features, float *out,
                      const robe_options_t *options, void *stream);

/*
 * The stable radix sort the backward pass sorts its tokens with, on its own (a testing aid, like
 * robe_offsets, and usable as a primitive): n pairs of 32-bit keys and values are sorted by key bits
 * [lo_bit, hi_bit) in ascending order, pairs with equal bits keeping their input order.  Eight bits
 * per pass, ping-pong between the two pairs of device buffers; both are overwritten, and
 * *result_in_b (host) says whether the sorted pairs ended in (keys_b, vals_b) or (keys_a, vals_a).
 *   workspace  device buffer of robe_sort_workspace_bytes(n) bytes, 256-byte aligned
 * Errors: ROBE_EINVAL, ROBE_EHIP.  Records kernels only: it may be captured into a HIP graph.
 */
size_t robe_sort_workspace_bytes(uint64_t n);
int robe_sort_pairs(uint32_t *keys_a, uint32_t *vals_a, uint32_t *keys_b, uint32_t *vals_b, uint64_t n,
                    uint32_t lo_bit, uint32_t hi_bit, void *workspace, size_t workspace_bytes, int *result_in_b,
                    void *stream);

/* Text of the calling thread's most recent error ("" if none).  Never NULL. */
const char *robe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ROBE_H */
