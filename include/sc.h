/*
 * sc.h — C ABI of the MI355X (gfx950) sparse 3-D convolution path.
 *
 * The three steps are the ones the paper gives for every sparse-convolution operator
 * (Section III-C: location table, offset table, result):
 *
 *     sc_hash_build   location table: coordinate -> input row        (Section III-C.1)
 *     (sc_hash_rebuild: the same into a table that is already initialised, without refilling it)
 *     sc_kmap_build   offset table / rulebook of (in,out) pairs       (Section III-C.2, III-B, III-D)
 *     sc_conv_fwd     out[o] = sum_k sum_{(i,o) in M_k} in[i] . W[k]   (Algorithm 2, Section III-C.3)
 *
 * Data model (Section II-A, Fig. 2; Section III-A): a sparse tensor is an index array of
 * int32 rows (batch, x, y, z), rows distinct, plus a feature array with one row of C channels
 * per index row.  Plain arrays in, plain arrays out; no framework types cross this boundary.
 *
 * Conventions
 *   - Every pointer named d_* is DEVICE memory owned by the caller, 16-byte aligned, and only
 *     borrowed for the duration of the stream work the call enqueues.  Pointers named h_* are
 *     host memory.  The library allocates nothing on the device (the measurement aids at the
 *     end of this file aside).  State it keeps between calls: per device, which kernels have
 *     been granted their large LDS allocation (set on first use), its number of compute units
 *     (asked once) and the address of the array behind sc_kmap_build_noalloc; process-wide, the samples of the optional timing aid.
 *     None of it changes results.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All calls except
 *     sc_counts_read (and sc_profile_read) are asynchronous on that stream and never synchronise.
 *   - Every function returns an int status: SC_OK or a negative SC_E* code.  Argument errors
 *     are detected on the host before anything is enqueued.  Data-dependent errors (duplicate
 *     or out-of-domain coordinates, table overflow) are latched by the kernels into
 *     sc_counts.status on the device and reported by sc_counts_read.
 *   - Coordinate domain: 0 <= b <= SC_BATCH_MAX, 0 <= x, y, z <= SC_COORD_MAX (8 + 3 x 16 bits
 *     of a 64-bit key whose top byte holds the epoch of the build).  1 <= n <= SC_N_MAX rows
 *     (n = 0 is accepted and yields empty results).  Neighbour probes that leave the domain
 *     simply miss; nothing wraps.
 *   - Kernel offsets d in {0..K-1}^3 are numbered k = dX*K^2 + dY*K + dZ (Section III-B eq. 5).
 *     A pair (in = i, out = o) belongs to offset k iff p_i = q_o*stride + d_k - pad, batch
 *     equal, with pad = (K-1)/2 for submanifold layers and 0 for strided ones (the direction
 *     is the one the offset-table figure of Section III-C shows: column 8 of a 3x3 row holds
 *     the (+1,+1) neighbour).
 *   - Weights are [K^3][C_in][C_out], row-major (one C_in x C_out matrix per offset).
 *     Algorithm 2 indexes them [C_out][K^3][C_in]; that is a relabelling of the same numbers.
 */
#ifndef SC_H_
#define SC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define SC_OK        0
#define SC_EINVAL   (-1)   /* bad argument: null / misaligned pointer, unsupported K, stride, mode, dtype, channels */
#define SC_ERANGE   (-2)   /* a coordinate lies outside the key domain */
#define SC_EDUP     (-3)   /* the same coordinate appears twice in the input */
#define SC_ECAP     (-4)   /* a caller-provided buffer is too small */
#define SC_EHIP     (-5)   /* the HIP runtime reported an error */
#define SC_EFULL    (-6)   /* hash table overflow (cannot happen with a table sized by sc_hash_bytes) */

/* layer kinds */
#define SC_SUBM      0     /* submanifold: outputs = inputs, stride 1, K odd (Section II-B) */
#define SC_STRIDED   1     /* "normal" down-sampling sparse convolution (Section III-B, III-D) */
#define SC_INVERSE   2     /* inverse (up-sampling) convolution (Section III-E); maps come from sc_kmap_transpose */

/* element types of features and weights */
#define SC_F32       0
#define SC_F16       1
#define SC_BF16      2

#define SC_COORD_MAX 65534
#define SC_BATCH_MAX 255
#define SC_HASH_EPOCH_MAX 254      /* epochs of sc_hash_rebuild: 1..254 */
#define SC_N_MAX     67108864LL   /* 2^26 rows: kernel-map entries pack (row, 6-bit slot) in 32 bits */
#define SC_K_MAX     7            /* K^3 <= 343 */

/* Data-dependent results, kept on the device until the caller asks for them. */
typedef struct sc_counts {
    int64_t n_in;              /* rows given to sc_hash_build / sc_kmap_build */
    int64_t n_out;             /* output rows of the last sc_kmap_build */
    int64_t n_pairs;           /* P: (in,out) pairs over all offsets (filled by sc_counts_read) */
    int32_t per_offset[343];   /* pairs per offset k (filled by sc_counts_read) */
    int32_t status;            /* 0, or the first SC_E* a kernel latched */
} sc_counts;

/* ---- location table (Section III-C.1; the paper offers a dense array or a hash table, this
 * library uses an open-addressing hash table keyed on the packed (b,x,y,z); sc_grid_* below is
 * the dense array) ------------------------------------------------------------------------- */

/* Bytes of the table for n keys: 16 bytes per slot plus a 256-byte header.  The capacity is a
 * power of two, at least 1024 slots and at least 8n (load factor <= 1/8); small tables are made
 * sparser still - up to 32 slots per key while the table stays within 2^22 slots (64 MiB) -
 * because shorter probe chains save round trips and a table of that size can be built again
 * without being refilled (sc_hash_rebuild). */
size_t sc_hash_bytes(int64_t n);

/* Build the table coordinate -> row index over d_coords [n][4] (b,x,y,z).  Also resets
 * *d_counts (n_in = n, everything else 0).  Latches SC_ERANGE / SC_EDUP into d_counts->status.
 * d_table: table_bytes >= sc_hash_bytes(n) bytes, fully overwritten (one pass that fills every
 * slot, then the inserts). */
int sc_hash_build(const int32_t* d_coords, int64_t n,
                  void* d_table, size_t table_bytes,
                  sc_counts* d_counts, void* stream);

/* Build again into a table that sc_hash_build has initialised, without the filling pass: stored
 * keys carry the epoch of their build, and whatever another epoch left in a slot counts as
 * free.  `epoch` is any value in 1..SC_HASH_EPOCH_MAX not used on this table since its last
 * sc_hash_build (a counter; call sc_hash_build again when it runs out).  table_bytes >=
 * sc_hash_bytes(n) as for sc_hash_build.  n may change from build to build: the table keeps
 * the capacity it was last filled with, and a build of more than a quarter of that many rows
 * is refused with SC_ECAP.  Resets *d_counts like sc_hash_build.  SC_ERANGE / SC_EDUP /
 * SC_ECAP of such a build are kept in the table's header and latched into d_counts->status by
 * the next sc_kmap_build that is given this table; sc_hash_lookup alone does not report them
 * (a duplicated coordinate maps to one of its rows, a coordinate outside the domain is
 * absent).  Tables above 64 MiB are filled all the same, with the capacity for n (measured
 * faster there: the fill leaves the table in the last-level cache for the probes that
 * follow), and then report like sc_hash_build.
 * A captured HIP graph replays its arguments, the epoch among them: capture sc_hash_build, not
 * this call, for a table that is rebuilt on every replay.
 * SC_EINVAL if epoch is outside 1..SC_HASH_EPOCH_MAX. */
int sc_hash_rebuild(const int32_t* d_coords, int64_t n,
                    void* d_table, size_t table_bytes, int epoch,
                    sc_counts* d_counts, void* stream);

/* ---- dense location table (Section III-C.1 offers both forms: a "large array" indexed by the
 * linearised coordinate, eq. 6, which the paper prefers when the domain is confined, or a hash
 * table; this is the array, as an alternative to sc_hash_build for submanifold layers) -------
 *
 * The table covers the box 0 <= b < B, 0 <= x < X, 0 <= y < Y, 0 <= z < Z with one 8-byte cell
 * per site (z runs fastest).  A cell holds a row index and the `epoch` of the build that wrote
 * it; look-ups only accept cells of the epoch they are given.  The caller clears the array once
 * (sc_grid_clear) and then passes a fresh epoch >= 1 to every sc_grid_build - any value it has
 * not used on this array since the last clear, e.g. a counter - so a build costs one scatter of
 * n cells: no fill before it, no clean-up after it.  Clear again before the counter wraps. */

#define SC_GRID_CELLS_MAX 8589934592LL   /* 2^33 sites = 64 GiB of cells */

/* Bytes of the array for the box, 0 if a side is < 1 or > SC_COORD_MAX + 1 or the box has more
 * than SC_GRID_CELLS_MAX sites. */
size_t sc_grid_bytes(int32_t B, int32_t X, int32_t Y, int32_t Z);

/* Zero the array (all cells unoccupied for every epoch >= 1). */
int sc_grid_clear(void* d_grid, size_t grid_bytes, int32_t B, int32_t X, int32_t Y, int32_t Z, void* stream);

/* Scatter the n rows of d_coords [n][4] into the array under `epoch` (plain stores, as in the
 * paper's table kernel).  Also resets *d_counts (n_in = n, everything else 0).  Nothing is
 * checked here: a coordinate outside the box, or two rows with one coordinate, are found by
 * sc_kmap_build_grid, which latches SC_ERANGE / SC_EDUP into d_counts->status.  Returns
 * SC_EINVAL for epoch 0. */
int sc_grid_build(const int32_t* d_coords, int64_t n,
                  void* d_grid, size_t grid_bytes, int32_t B, int32_t X, int32_t Y, int32_t Z,
                  uint32_t epoch, sc_counts* d_counts, void* stream);

/* d_rows[i] = row index of d_query[i] in the build of `epoch`, or -1. */
int sc_grid_lookup(const void* d_grid, int32_t B, int32_t X, int32_t Y, int32_t Z, uint32_t epoch,
                   const int32_t* d_query, int64_t n_query, int32_t* d_rows, void* stream);

/* ---- offset table / kernel map (Section III-C.2 for submanifold layers: probe the K^3
 * neighbours of every active site in the location table; Section III-B eq. 1-5 and
 * Section III-D for strided layers: cell index floor(p/s), in-cell offset, distinct output
 * cells counted and numbered) ------------------------------------------------------------- */

/* Upper bound on output rows for n inputs: n for SC_SUBM; n * ceil(K/stride)^3 for SC_STRIDED
 * (an input p belongs to every cell q with p = q*stride + d, d in [0,K)^3: one cell when
 * K == stride, up to ceil(K/stride)^3 otherwise); for SC_INVERSE the n fine rows themselves.
 * -1 if the combination is not supported (see sc_kmap_build) or the bound exceeds SC_N_MAX. */
int64_t sc_out_bound(int64_t n, int K, int stride, int mode);

/* Bytes of the kernel-map blob and of the scratch buffer sc_kmap_build needs (0 = unsupported). */
size_t sc_kmap_bytes(int64_t n, int K, int stride, int mode);
size_t sc_kmap_scratch_bytes(int64_t n, int K, int stride, int mode);

/* Build the kernel map.
 *   d_table       table built by sc_hash_build / sc_hash_rebuild over the same d_coords (required
 *                 for SC_SUBM).
 *                 SC_STRIDED layers do not look anything up in it (Section III-D builds the
 *                 output side only): pass NULL and the build is self-contained - it then also
 *                 resets *d_counts the way sc_hash_build does (n_in = n, status 0); pass the
 *                 table of a preceding sc_hash_build / sc_hash_rebuild and *d_counts is left as
 *                 that call set it (plus what a rebuild left in the table header), including
 *                 SC_EDUP, which only those two can detect
 *   mode          SC_SUBM (stride must be 1, K odd, K <= SC_K_MAX) or SC_STRIDED (2 <= K <=
 *                 SC_K_MAX, 1 <= stride <= K, no padding: input p pairs with output cell q at
 *                 offset d iff p = q*stride + d; K == stride <= 4 is the down-sampling layer of
 *                 Section III-B / III-D and has its own faster build)
 *   d_out_coords  [sc_out_bound][4]; receives the output coordinates.  SC_SUBM: may be NULL
 *                 (outputs are the inputs, same order).  SC_STRIDED: required; output o is the
 *                 o-th distinct cell in order of first occurrence (input rows ascending, then
 *                 offsets ascending), so the result does not depend on thread timing.
 *   d_kmap        opaque blob, kmap_bytes >= sc_kmap_bytes(...).  It holds the offset table of
 *                 Section III-C.2 (for every output row and offset the paired input row or -1),
 *                 tile-major: 64 consecutive output rows per tile, offset-major inside a tile,
 *                 plus one bit per (16-row group, offset) that tells whether the group has any
 *                 neighbour there.  Read it with sc_kmap_export; feed it to sc_conv_fwd (any
 *                 number of times: layers that share coordinates share the map).
 *   d_scratch     scratch_bytes >= sc_kmap_scratch_bytes(...); contents undefined afterwards.
 *   d_counts      n_out is written here (device side); errors are latched into status. */
int sc_kmap_build(const int32_t* d_coords, int64_t n,
                  const void* d_table,
                  int K, int stride, int mode,
                  int32_t* d_out_coords,
                  void* d_kmap, size_t kmap_bytes,
                  void* d_scratch, size_t scratch_bytes,
                  sc_counts* d_counts, void* stream);

/* sc_kmap_build for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same build with the scratch buffer
 * taken from a fixed array inside the library (SC_NOALLOC_SCRATCH_BYTES of device memory per GPU
 * the library runs on, held until the process ends) instead of d_scratch.  Every other argument,
 * the results and the errors are those of sc_kmap_build; the call itself allocates nothing.
 * SC_ECAP if sc_kmap_scratch_bytes(n, K, stride, mode) exceeds SC_NOALLOC_SCRATCH_BYTES (K ==
 * stride layers: up to 65,536 input rows; submanifold layers need no scratch and are never
 * refused for it).  All calls on one GPU share that one array: calls that overlap in time on the
 * same GPU (different streams or host threads) race; calls on one stream are safe, and a call
 * does not depend on what an earlier one left in the array. */
#define SC_NOALLOC_SCRATCH_BYTES (16 << 20)
int sc_kmap_build_noalloc(const int32_t* d_coords, int64_t n,
                          const void* d_table,
                          int K, int stride, int mode,
                          int32_t* d_out_coords,
                          void* d_kmap, size_t kmap_bytes,
                          sc_counts* d_counts, void* stream);

/* The submanifold kernel map (mode SC_SUBM, stride 1, K odd) from a dense location table built by
 * sc_grid_build(d_coords, n, ..., epoch): same blob, same meaning of every other argument as in
 * sc_kmap_build; needs no scratch buffer.  Every row reads its own cell: a row outside the box
 * latches SC_ERANGE, a cell that names another row (two rows, one coordinate) latches SC_EDUP. */
int sc_kmap_build_grid(const int32_t* d_coords, int64_t n,
                       const void* d_grid, size_t grid_bytes, int32_t B, int32_t X, int32_t Y, int32_t Z,
                       uint32_t epoch, int K,
                       void* d_kmap, size_t kmap_bytes,
                       sc_counts* d_counts, void* stream);

/* Inverse (up-sampling) layer, Section III-E: every row of the fine set finds its parent in the
 * coarse set and its place in the kernel, and receives parent_features . W[place].  The pairs are
 * those of the strided layer that made the coarse set, with input and output swapped, so the map
 * is made from that layer's map:
 *   d_kmap, n, K, stride   the strided layer's map and the arguments it was built with
 *   d_counts               the counts block of that build (n_out is read on the device)
 *   d_kmap_inv             receives the inverse map, kmap_inv_bytes >= sc_kmap_bytes(n, K,
 *                          stride, SC_INVERSE); must not alias d_kmap
 * Use it with sc_conv_fwd(mode = SC_INVERSE): d_feat_in has one row per coarse cell, d_feat_out
 * one row per fine row (n of them), W[k] is applied to the pair whose fine row sits at in-cell
 * offset k.  sc_counts_read / sc_kmap_export accept the inverse map with mode = SC_INVERSE. */
int sc_kmap_transpose(const void* d_kmap, int64_t n, int K, int stride,
                      const sc_counts* d_counts,
                      void* d_kmap_inv, size_t kmap_inv_bytes, void* stream);

/* ---- compute (Algorithm 2; Section III-C.3) ---------------------------------------------- */

/* Workspace sc_conv_fwd may use for the given layer (weights re-laid out as MFMA operand tiles
 * when they do not fit in LDS as a whole); 0 for fp32 layers. */
size_t sc_conv_workspace_bytes(int K, int C_in, int C_out, int dtype_in);

/* d_feat_out[o][:] = sum over offsets k and pairs (i,o) of d_feat_in[i][:] . d_weight[k]
 *   n_map       the n the kernel map was built with (rows of d_feat_in for SC_SUBM / SC_STRIDED;
 *               rows of d_feat_out for SC_INVERSE)
 *   d_feat_in   [rows][C_in]  of dtype_in
 *   d_weight    [K^3][C_in][C_out] of dtype_in
 *   d_feat_out  [n_out_cap][C_out] of dtype_out; rows [0, n_out) are fully overwritten (a row
 *               with no pair becomes 0), rows >= n_out are left untouched.  n_out is read on
 *               the device from d_counts; n_out_cap >= sc_out_bound(...) is always enough.
 *   d_kmap      blob from sc_kmap_build (or sc_kmap_transpose) for the same (n_map, K, stride)
 *   dtype_in    SC_F32 (fp32 MFMA) or SC_F16 / SC_BF16 (16-bit MFMA, fp32 accumulation)
 *   dtype_out   SC_F32 or the same as dtype_in (one round-to-nearest-even at the end)
 *   channels    SC_F32: any C_in >= 1, 1 <= C_out <= 256.  SC_F16 / SC_BF16: C_in one of 32, 64,
 *               128, 256 and C_out a multiple of 16, 16 <= C_out <= 256.
 *   d_workspace workspace_bytes >= sc_conv_workspace_bytes(...); contents undefined afterwards */
int sc_conv_fwd(const void* d_feat_in, int64_t n_map,
                const void* d_weight,
                void* d_feat_out, int64_t n_out_cap,
                const void* d_kmap, size_t kmap_bytes,
                const sc_counts* d_counts,
                int K, int stride, int mode,
                int C_in, int C_out, int dtype_in, int dtype_out,
                void* d_workspace, size_t workspace_bytes,
                void* stream);

/* The weights of a layer in the form sc_conv_fwd's kernels consume (Algorithm 2 indexes the
 * weights per (offset, input channel, output channel); the matrix cores want them as operand
 * tiles).  sc_conv_fwd re-lays the weights out on every call; a caller whose weights do not change
 * from frame to frame packs them once and calls sc_conv_fwd_packed instead.
 *   sc_conv_packed_bytes   bytes of the packed form (0 for an unsupported K / dtype)
 *   sc_conv_weight_pack    d_weight [K^3][C_in][C_out] of dtype_in -> d_packed (packed_bytes >=
 *                          sc_conv_packed_bytes(...)); asynchronous on `stream`.  The layout is
 *                          private to the library and depends on (K, C_in, C_out, dtype_in); for
 *                          SC_F32 it is a copy.  SC_EINVAL for channel counts sc_conv_fwd rejects.
 *   sc_conv_fwd_packed     sc_conv_fwd with d_packed in place of d_weight and no workspace: same
 *                          arguments otherwise, same results bit for bit. */
size_t sc_conv_packed_bytes(int K, int C_in, int C_out, int dtype_in);
int sc_conv_weight_pack(const void* d_weight, int K, int C_in, int C_out, int dtype_in,
                        void* d_packed, size_t packed_bytes, void* stream);
int sc_conv_fwd_packed(const void* d_feat_in, int64_t n_map,
                       const void* d_packed,
                       void* d_feat_out, int64_t n_out_cap,
                       const void* d_kmap, size_t kmap_bytes,
                       const sc_counts* d_counts,
                       int K, int stride, int mode,
                       int C_in, int C_out, int dtype_in, int dtype_out,
                       void* stream);

/* Fused form of the last two steps for 3x3x3 submanifold layers over a dense location table
 * (Section III-C.2 and III-C.3 in one pass): the convolution looks the 27 neighbours of its rows
 * up in the table built by sc_grid_build(d_coords, n, ..., epoch) itself, so no kernel map is
 * built, stored or read.  Output row i belongs to d_coords row i; d_feat_out [n][C_out] is fully
 * overwritten.  16-bit layers only (dtype_in SC_F16 / SC_BF16), (C_in, C_out) one of (32,32),
 * (64,64), (128,128), (32,64), (64,128); anything else returns SC_EINVAL - use the three calls.
 * Nothing is validated here (no counts block): rows outside the box get only their centre term,
 * repeated coordinates are not noticed; sc_kmap_build_grid is the call that checks. */
int sc_conv_fwd_grid(const void* d_feat_in, const int32_t* d_coords, int64_t n,
                     const void* d_grid, size_t grid_bytes, int32_t B, int32_t X, int32_t Y, int32_t Z,
                     uint32_t epoch,
                     const void* d_weight, void* d_feat_out,
                     int K, int C_in, int C_out, int dtype_in, int dtype_out,
                     void* d_workspace, size_t workspace_bytes, void* stream);

/* The inverse layer of a K == stride layer straight from that layer's own map, without
 * sc_kmap_transpose (Section III-E: the pairs of the down-sampling layer with input and output
 * swapped).  Every fine row has exactly one parent there, so the kernel walks the coarse rows,
 * multiplies each by the W[k] of the offsets it has children at and stores the products at the
 * children's rows: d_feat_fine[i][:] = d_feat_coarse[o][:] . d_weight[k] for the pair (i, o) of
 * offset k.  The result equals sc_kmap_transpose + sc_conv_fwd(SC_INVERSE).
 *   n_map          the n the strided map was built with (= rows of d_feat_fine)
 *   d_feat_coarse  [n_out][C_in] of dtype_in, n_out = d_counts->n_out of that build
 *   d_weight       [K^3][C_in][C_out] of dtype_in
 *   d_feat_fine    [n_map][C_out] of dtype_out, every row overwritten
 *   d_kmap         blob from sc_kmap_build(SC_STRIDED, K, stride = K)
 * K = 2 with (C_in, C_out) one of (32,32), (64,32), (64,64), (128,64), or K = 3 with (32,32);
 * dtype_in SC_F16 / SC_BF16, dtype_out SC_F32 or dtype_in.  SC_EINVAL otherwise (use the
 * transposed map). */
int sc_conv_up_fwd(const void* d_feat_coarse, int64_t n_map,
                   const void* d_weight, void* d_feat_fine,
                   const void* d_kmap, size_t kmap_bytes, const sc_counts* d_counts,
                   int K, int C_in, int C_out, int dtype_in, int dtype_out,
                   void* stream);

/* ---- reading results back ------------------------------------------------------------------ */

/* Fill n_pairs and per_offset from the kernel map (d_kmap may be NULL to skip that), copy the
 * block to h_counts and SYNCHRONISE the stream.  Returns h_counts->status if it is an error,
 * else SC_OK.  (n, K, stride, mode) must be the ones the map was built with. */
int sc_counts_read(sc_counts* d_counts, sc_counts* h_counts,
                   const void* d_kmap, int64_t n, int K, int stride, int mode,
                   void* stream);

/* Rulebook in its plain form, for inspection and tests: pairs grouped by offset,
 * d_pairs_in / d_pairs_out [n_pairs] and d_offset_start [K^3+1] (int32, device memory; pairs of
 * offset k are [offset_start[k], offset_start[k+1])), ordered by output row inside one offset
 * (ballot + prefix-count compaction of the offset table).  h_counts must come from
 * sc_counts_read on the same map (it gives the sizes).  Asynchronous on `stream`. */
int sc_kmap_export(const void* d_kmap, int64_t n, int K, int stride, int mode,
                   const sc_counts* h_counts,
                   int32_t* d_pairs_in, int32_t* d_pairs_out, int32_t* d_offset_start,
                   void* stream);

/* Look up coordinates in a table built by sc_hash_build / sc_hash_rebuild: d_rows[i] = row index
 * of d_query[i], or -1 if absent.  n_table is only range-checked (the table knows its capacity).
 * (Not on the layer's hot path; lets callers and tests read the table.) */
int sc_hash_lookup(const void* d_table, int64_t n_table,
                   const int32_t* d_query, int64_t n_query, int32_t* d_rows, void* stream);

/* Host-side inspection aid: the slot (0 .. capacity-1) at which a table sized for n keys looks for
 * coordinate (b,x,y,z) on its attempt-th try (0 = first); -1 outside the key domain.  Pure
 * arithmetic, no device work; lets tests examine the probe sequence. */
int64_t sc_hash_probe_slot(int32_t b, int32_t x, int32_t y, int32_t z, uint32_t attempt, int64_t n);

const char* sc_strerror(int status);

/* ---- measurement aid (not part of the paper's method) -------------------------------------- */

/* Per-kernel timing for benchmarks.  sc_profile_enable(1) clears earlier samples and makes every
 * later call of this library attach a pair of HIP events to each kernel it launches (stamped with
 * the dispatch's own begin and end times); sc_profile_enable(0) stops that.  sc_profile_read
 * synchronises the device and fills up to max_entries entries (one per kernel that ran: name,
 * number of launches, summed and median duration in ms); it returns the number of entries written
 * or a negative SC_E* code.  `name` points to a static string.  This is process-wide state for
 * single-threaded measurement code (the only state the library keeps besides per-device launch
 * attributes and the array of sc_kmap_build_noalloc); it is off by default. */
typedef struct sc_profile_entry {
    const char* name;
    int64_t launches;
    double total_ms;
    double median_ms;
} sc_profile_entry;
int sc_profile_enable(int enable);
int sc_profile_read(sc_profile_entry* h_entries, int max_entries);

/* Measured counterpart of the published matrix-core peak: runs a short loop of independent
 * 16x16x32 fp16 multiplies with register operands on the current device (default stream,
 * synchronises, allocates a few bytes for the duration of the call) and returns the sustained
 * TFLOP/s in *h_tflops. */
int sc_profile_mfma_peak(double* h_tflops);

#ifdef __cplusplus
}
#endif
#endif /* SC_H_ */
