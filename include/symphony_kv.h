/* symphony_kv.h — C ABI of libsymphony_kv.so
 *
 * The data-parallel hot path behind Symphony's `pred` system call (paper section 4.1) on one
 * MI355X: a KV-cache file system whose files are lists of fixed-size pages of GPU memory
 * (paper section 4.2, "KVFS"), copy-on-write forks of those files, and ONE batched launch
 * that appends the new tokens' K/V rows of many LIPs and computes attention for every new
 * token through the per-file page tables (the batch that the inference scheduler of paper
 * section 4.4 forms from the pending `pred` calls).
 *
 * Conventions
 *  - Every function returns an int status unless stated: 0 = SYM_OK, negative = error.
 *    On an error the host state is unchanged (all-or-nothing): arguments are validated, pool
 *    space is counted and pinned staging memory is reserved before anything is committed.  The
 *    one exception: SYM_EHIP from a kernel launch or from a wait on the device (reported AFTER
 *    the commit) means the device is in an unknown state; the files of the call may then be
 *    longer than their data, and the context should be destroyed.  No exception or abort
 *    crosses this boundary.  sym_strerror() returns the last message of the context.
 *  - "device" pointers are HIP device memory owned by the CALLER (e.g. a torch tensor's
 *    data_ptr()).  The library allocates no device memory, never synchronises `stream`
 *    and enqueues all device work on the `stream` argument (a hipStream_t passed as
 *    void*; NULL = the default stream).  All calls on one context must be issued on one
 *    stream, or be ordered by the caller: the descriptor area of the workspace is reused
 *    from call to call in stream order.
 *  - "host" pointers are ordinary host memory, read (or written) before the call returns.
 *  - One mutex per context makes calls thread-safe; a context created with device = -1
 *    is host-only: file-system state and descriptors work, device calls return SYM_EINVAL.
 *
 * Page layout (internal; parity is defined on outputs and page ids, not on pool bytes):
 *    page = [n_kv_heads][2 (K, V)][row_halves][page_tokens][row_bytes / row_halves],
 *  row_bytes = head_dim * sizeof(element) = 256, row_halves = 2: each 256-byte K or V row
 *  of a token is stored as two 128-byte halves, all first halves of the page's tokens
 *  contiguous, then all second halves, so that 8 consecutive tokens of one half form one
 *  contiguous 1 KiB run = one 64-lane x 16-byte load.
 */
#ifndef SYMPHONY_KV_H
#define SYMPHONY_KV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SYM_OK      0
#define SYM_EINVAL (-1)  /* bad argument / unsupported shape                         */
#define SYM_EBADF  (-2)  /* stale or unknown file handle                             */
#define SYM_ENOSPC (-3)  /* page pool (or workspace) too small for the request       */
#define SYM_ENOENT (-4)
#define SYM_EEXIST (-5)
#define SYM_EBUSY  (-6)  /* same file twice in one batch (stand-in for the write lock
                            of paper section 4.2)                                    */
#define SYM_EHIP   (-7)  /* a HIP runtime call failed                                */

#define SYM_F32  0
#define SYM_BF16 1

typedef struct sym_ctx sym_ctx;   /* opaque; owns host metadata and pinned staging only */
typedef int32_t sym_kv;           /* file handle >= 0; the lowest free slot is reused   */

/* Planner settings.  They decide how a batch is laid over the GPU, never what it computes:
 * every setting gives the same outputs up to the order of floating-point sums (the tests
 * sweep them).  sym_tuning_defaults() fills the values that sym_init uses when
 * sym_config.tuning is NULL; a caller changes the fields it wants and passes the struct.
 * Out-of-range values are clamped to the nearest allowed one.                             */
typedef struct sym_tuning {
  int32_t decode_mfma;     /* ranges of single tokens and short drafts on the matrix cores (1)
                              or on the vector ALUs (0); bf16 only.  Default: 1 when
                              Hq/Hkv = 8, else 0                                          */
  int32_t min_units;       /* smallest piece, in pages, that a long range is cut into;
                              >= 1, default 4                                             */
  int32_t prefill_min;     /* a pred of at least this many new tokens is computed by tiles
                              (bf16); >= 2, default 16                                    */
  int32_t share_min_lips;  /* files of a batch that must share a page-list prefix before
                              the prefix is read once for all of them; 0 = never group,
                              default 4                                                   */
  int32_t share_min_pages; /* shortest shared prefix that is grouped; >= 2, default 8     */
  int32_t tile_rows;       /* query rows of a tile: 256 (default) or 128                  */
  int32_t row_tokens;      /* new tokens of a short draft that share one pass over the file:
                              1 .. 16 / (Hq/Hkv), default the maximum; bf16 only          */
  int32_t range_cost;      /* what the start of a range costs, in pages' worth of work, when
                              work is divided; >= 0, default 3                            */
  int32_t bin_tolerance;   /* whole ranges are packed into workgroups only if the fullest
                              then holds at most this many percent more than the mean;
                              otherwise ranges are cut at equal cost; >= 0, default 3     */
  int32_t bin_waves;       /* wavefronts of a decode workgroup: 8 (default) or 4          */
  int32_t fuse_append;     /* 1 (default): the K/V row of a single new token is written by
                              the wavefront that reads the row's last page; 0: by a launch
                              of its own before attention                                 */
  int32_t mix_lead;        /* a launch that holds tiles and decode workgroups starts with this
                              many percent of its tile workgroups (0..100, default 0) ...  */
  int32_t mix_spread;      /* ... and spreads the decode workgroups evenly among the next this
                              many percent of them (0..100 - mix_lead, default 50); the other
                              tile workgroups follow                                      */
  int32_t share_tiles;     /* shared prefixes are cut by key chunk (at most 8 chunks each) until
                              the batch has about this many tiles; >= 1, default 512 (two
                              workgroups per CU)                                          */
} sym_tuning;

typedef struct sym_config {
  int32_t n_q_heads;       /* Hq; Hq / Hkv must be 1, 2, 4 or 8                           */
  int32_t n_kv_heads;      /* Hkv, divides Hq; query head h reads kv head h / (Hq/Hkv)   */
  int32_t head_dim;        /* D; D * sizeof(element) must be 256 (bf16: 128, f32: 64)    */
  int32_t page_tokens;     /* P = 16                                                     */
  int32_t dtype;           /* SYM_F32 or SYM_BF16: storage type of Q, K, V.  The matrix-core
                              paths (tiles for preds of many tokens and for shared prefixes,
                              rows of several draft tokens) exist for SYM_BF16 only: with
                              SYM_F32 every new token is a row of its own that reads the file */
  int32_t device;          /* HIP device ordinal, or -1 for a host-only context          */
  int64_t n_pages;         /* pages in the pool; page ids are int32, n_pages < 2^27      */
  void*   pool;            /* device, n_pages * sym_page_bytes() bytes, 256-aligned      */
  void*   workspace;       /* device scratch: descriptors + partial results              */
  int64_t workspace_bytes;
  const int32_t* free_order; /* host, optional permutation of [0,n_pages): allocation
                              ranking (the free page of lowest rank is taken first);
                              NULL = identity.  Copied by sym_init.                      */
  float   softmax_scale;   /* 0 = 1/sqrt(D)                                              */
  int32_t decode_waves;    /* wavefront slots the decode kernel is cut into; 0 = auto    */
  int32_t n_layers;        /* attention layers that share the files' page tables; 0 or 1 =
                              one.  The pool then holds n_layers * n_pages pages, layer after
                              layer: page p of layer l is page l * n_pages + p of the pool.   */
  const sym_tuning* tuning;  /* host, optional: planner settings, NULL = the defaults.
                                Copied by sym_init.                                        */
} sym_config;

typedef struct sym_stats {
  int64_t pages_total, pages_free, pages_shared;  /* shared = reference count > 1        */
  int64_t cow_copies, pages_allocated, tokens_appended;
  int64_t pred_batches, kernel_launches;
  int64_t files, handles;
  int64_t host_ns_plan;   /* host time inside sym_pred_batch spent on append planning +
                             descriptor build + staging, summed over calls, nanoseconds    */
  int64_t host_ns_pred;   /* host time of whole sym_pred_batch calls (planning + launches),
                             not counting waits for a staging buffer still in use by the GPU */
  int64_t tokens_moved;      /* tokens copied by sym_kv_extract / sym_kv_merge              */
  int64_t pages_referenced;  /* pages those calls shared with the source instead of copying */
  int64_t pages_offloaded, pages_restored;   /* page copies of sym_kv_offload / sym_kv_restore */
  int64_t host_slots;        /* pinned host slots (pages) the context has created so far      */
  int64_t last_batch_tiles;        /* of the last pred batch planned: matrix-core tiles ...            */
  int64_t last_batch_shared_rows;  /* ... and rows whose shared prefix is read through such tiles      */
} sym_stats;

/* Sizes.  sym_page_bytes: bytes of one page for this shape (0 if unsupported).
 * sym_workspace_bytes: a workspace size sufficient for any batch with at most max_lips
 * files, max_tokens new tokens in total and max_table_entries page-table entries summed
 * over the batch's files (after the append). */
int64_t sym_page_bytes(const sym_config* cfg);
/* The planner settings sym_init uses for this shape when cfg->tuning is NULL (cfg->tuning
 * itself is not read).  SYM_EINVAL for an unsupported shape.                             */
int     sym_tuning_defaults(const sym_config* cfg, sym_tuning* out);
int64_t sym_workspace_bytes(const sym_config* cfg, int64_t max_lips, int64_t max_tokens,
                            int64_t max_table_entries);

int  sym_init(const sym_config* cfg, sym_ctx** out);
void sym_destroy(sym_ctx* ctx);
const char* sym_strerror(sym_ctx* ctx);   /* valid until the next call on ctx */

/* ---- KVFS: the file calls of the paper's Fig. 1 and section 4.2 -------------------- */
/* kv_open: name NULL = new anonymous empty file; otherwise open the file of that name,
 * creating it empty if absent; a second open of a name returns a second handle to the SAME
 * file (files are shared, section 4.2).  Returns a handle >= 0 or a negative status.     */
sym_kv  sym_kv_open(sym_ctx* ctx, const char* name);
/* kv_fork: new anonymous file with a copy of the parent's page list; every page's
 * reference count goes up by one; no tensor is copied, no page allocated, no device work
 * (section 4.2: a fork must not duplicate the tensors).                                  */
sym_kv  sym_kv_fork(sym_ctx* ctx, sym_kv parent);
/* kv_remove: delete the file: every page's count goes down by one, pages reaching zero
 * return to the free set; all handles of the file become invalid (Fig. 1).               */
int     sym_kv_remove(sym_ctx* ctx, sym_kv kv);
/* kv_close: drop this handle.  A named file persists (section 4.2: files outlive a
 * process); an anonymous file with no handle left is removed.                            */
int     sym_kv_close(sym_ctx* ctx, sym_kv kv);
/* Token count of the file (Fig. 1 `.len()`), or a negative status.                       */
int64_t sym_kv_len(sym_ctx* ctx, sym_kv kv);
/* kv_truncate: for n files at once, drop the tokens from new_len[i] on (POSIX-style truncate
 * of a KVFS file, section 4.2: a LIP that verifies draft tokens with a multi-token pred,
 * section 4.1, rolls the rejected ones back).  Host-only: pages no longer needed lose one
 * reference; K/V bytes are not touched.  kv, new_len: host.  All or nothing.              */
int     sym_kv_truncate(sym_ctx* ctx, int32_t n, const sym_kv* kv, const int64_t* new_len);
/* kv_append: the half of pred (section 4.1) that adds the new tokens' tensors to the file, on its own:
 * append n >= 1 token rows.  k, v: device, [n][Hkv][D] in the storage dtype.  Allocates
 * pages as needed; a shared, partly filled last page is first copied (copy-on-write).    */
int     sym_kv_append(sym_ctx* ctx, sym_kv kv, int32_t n, const void* k, const void* v,
                      void* stream);

/* kv_extract, kv_merge (section 4.2: a new file from chosen token indices of an existing one, and
 * a new file that is several existing files joined, e.g. to prune a context).
 * Both make NEW anonymous files; the source files are not modified.
 *   sym_kv_extract: for n_files files at once (one launch): token j of new file i is token
 *     idx[idx_off[i] + j] of src[i], j < idx_off[i+1] - idx_off[i].  src, idx_off [n_files + 1],
 *     idx: host; indices in any order, repeats allowed, each inside its source file (else
 *     SYM_EINVAL); an empty range gives an empty file.  out [n_files]: host, receives the new
 *     handles.  All files or none (SYM_ENOSPC, SYM_EBADF, SYM_EINVAL: nothing changed).
 *   sym_kv_merge: returns the handle (or a negative status) of a new file holding the tokens of
 *     files[0], then files[1], ... (m >= 0 files, host handles; a file may appear more than once).
 * The stored K/V rows move bit for bit (no re-encoding of positions).  A destination page
 * whose tokens are slots 0, 1, 2, ... of one existing page references that page (its count
 * goes up, nothing is copied: an identity extract or a merge of one file is a fork); every
 * other destination page is a fresh page (lowest rank first, in destination order) filled by
 * the copy kernel on `stream`.  In a host-only context only the integer state is built.   */
int     sym_kv_extract(sym_ctx* ctx, int32_t n_files, const sym_kv* src, const int64_t* idx_off,
                       const int64_t* idx, sym_kv* out, void* stream);
sym_kv  sym_kv_merge(sym_ctx* ctx, int32_t m, const sym_kv* files, void* stream);
/* The copy list of the last sym_kv_extract / sym_kv_merge on this context, for inspection:
 * (source, destination) pairs of token slots, each page * P + slot, in destination order.
 * Returns the number of pairs; writes at most cap of them (out may be NULL).             */
int64_t sym_last_moves(sym_ctx* ctx, int32_t* out, int64_t cap);

/* kv_offload, kv_restore (section 4.3: while a thread waits for I/O its KV cache moves from
 * the GPU to CPU memory and is restored when the I/O completes).  kv: host, n distinct handles.
 *   sym_kv_offload: the files start to wait.  A waiting file cannot be read or written (pred,
 *     append, fork, truncate, extract, merge, read: SYM_EBUSY) but can be removed or closed.  A
 *     page leaves the GPU when EVERY reference to it belongs to a waiting file (a page that a
 *     running file still shares stays): it is copied into pinned host memory owned by the
 *     context (host slots, lowest free first, allocated with hipHostMalloc as needed, kept until
 *     sym_destroy), every table entry that referenced it becomes -(slot + 1) (as sym_kv_pages
 *     shows), and the page returns to the free set.  Other pages stay where they are.
 *   sym_kv_restore: the files' waits end.  Every host slot they reference comes back into a
 *     fresh page (lowest rank first, in table order) and EVERY entry that referenced the slot is
 *     rewritten, also those of files that still wait.  SYM_ENOSPC (nothing changed) if the pages
 *     do not fit.
 * Files already (not) waiting, or named twice: SYM_EBUSY.  The copies are one kernel launch per
 * call on `stream`, before the call returns control of the freed pages / slots to the allocator
 * (stream order keeps later writers behind them).  sym_kv_waiting: 1, 0 or a negative status.
 * In a host-only context only the integer state is built.                                 */
int     sym_kv_offload(sym_ctx* ctx, int32_t n, const sym_kv* kv, void* stream);
int     sym_kv_restore(sym_ctx* ctx, int32_t n, const sym_kv* kv, void* stream);
int     sym_kv_waiting(sym_ctx* ctx, sym_kv kv);
/* The page copies of the last sym_kv_offload ((page, host slot) pairs) or sym_kv_restore
 * ((host slot, page) pairs) on this context, for inspection.  Returns the number of pairs. */
int64_t sym_last_swaps(sym_ctx* ctx, int32_t* out, int64_t cap);

/* ---- pred (section 4.1), batched (section 4.4) ------------------------------------- */
/* One launch for n_lips pending pred calls.  LIP b appends n_tokens[b] >= 1 rows to file
 * kv[b] (files distinct, else SYM_EBUSY) and gets one output row per new token: row i of
 * LIP b attends to file tokens 0 .. len_before_b + i (the whole existing file plus the new
 * tokens up to itself).  T = sum n_tokens.  q: device [T][Hq][D]; k_new, v_new: device
 * [T][Hkv][D] (storage dtype, LIPs in batch order); out: device [T][Hq][D] float32.
 * kv, n_tokens: host.  If the pool cannot hold the batch: SYM_ENOSPC, nothing changes.   */
int sym_pred_batch(sym_ctx* ctx, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens,
                   const void* q, const void* k_new, const void* v_new, float* out,
                   void* stream);

/* sym_pred_batch for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same result, same state changes as
 * sym_pred_batch, but the device scratch of the batch (descriptor words, partial results of cut
 * ranges and shared prefixes) is a file-scope device array inside the library instead of the
 * workspace of sym_config, and the call allocates nothing on the way: no device memory, no pinned
 * memory (the staging buffers sym_init made are used as they are), no events (launches of this
 * entry point are not profiled).  The array has sym_static_scratch_bytes() = 64 MiB and lives on
 * every GPU the library has been used on until the process ends; its address on the context's
 * device is looked up once, by sym_init.  Limits, refused with SYM_ENOSPC before anything changes:
 * the descriptor blob of the batch (its upper bound: about 40 words per wavefront slot + 21 per new
 * token + one per page-table entry + about 1000 per LIP at 8 kv heads) must not exceed 1 Mi words,
 * and the partial results this shape needs at least (2 x tokens per row x wavefront slots + 1 slots of
 * G x (head_dim + 2) floats) must fit behind it; with fewer slots than the workspace would have,
 * fewer shared prefixes are read once (results are the same to rounding).  The array is shared by
 * EVERY context and stream on the GPU and keeps the last call's contents (nothing in it has to
 * start at zero: each launch writes every slot it reads): two calls of this entry point that
 * overlap on one GPU, from different streams or contexts, race; order them.                   */
int sym_pred_batch_static(sym_ctx* ctx, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens,
                          const void* q, const void* k_new, const void* v_new, float* out,
                          void* stream);
int64_t sym_static_scratch_bytes(void);

/* pred over the layers of a model (section 4.1: one pred is a forward pass, and every attention
 * layer of it sees the same files, page tables and batch).  In a context with n_layers layers a
 * page id names one page in EVERY layer; the file calls act on all layers at once:
 *   sym_kv_append:  k, v are [n_layers][n][Hkv][D];
 *   sym_kv_extract / sym_kv_merge / sym_kv_offload / sym_kv_restore and the copy-on-write copies
 *     move the rows or pages of every layer (a host slot holds a page's bytes of all layers);
 *   sym_kv_read reads layer 0, sym_kv_read_layer any layer.
 * A batch runs in two steps:
 *   sym_pred_begin:  the host half, once per batch: plans and commits the append of
 *     n_tokens[b] rows to file kv[b] (same rules and errors as sym_pred_batch), builds the batch
 *     descriptor and copies it to the workspace (one small launch on `stream`).
 *   sym_pred_layer:  the device half, once per layer, in any order, on the same stream: appends
 *     this layer's rows k_new, v_new [T][Hkv][D] and computes this layer's attention for q
 *     [T][Hq][D] into out [T][Hq][D] float32, against layer `layer` of the pool: the attention
 *     launch (plain decode batches: this one launch appends the rows as well), preceded by a
 *     launch for page copies and the rows of multi-token LIPs when the batch has any, followed
 *     by the merge of partial results when ranges were divided.
 * Between sym_pred_begin and the last of the n_layers sym_pred_layer calls (or sym_pred_end,
 * which abandons the layers not yet run: their new rows stay unwritten) every call that changes
 * file-system state or reads files is refused with SYM_EBUSY; kv_open, kv_len, kv_pages and
 * the other introspection calls work.  A single-layer context may use either these calls or
 * sym_pred_batch; a context with several layers only these.                               */
int sym_pred_begin(sym_ctx* ctx, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens,
                   void* stream);
int sym_pred_layer(sym_ctx* ctx, int32_t layer, const void* q, const void* k_new,
                   const void* v_new, float* out, void* stream);
int sym_pred_end(sym_ctx* ctx);

/* Kernel-level entry without the allocator: attention only, over page tables the caller
 * supplies.  K/V of every token (new ones included) must already be in the pool.
 * page_table_flat: host int32, LIP b's page ids at [pt_offsets[b], pt_offsets[b+1]);
 * lengths: host int64 [n_lips], tokens of the file INCLUDING this call's n_tokens[b] new
 * ones; row i of LIP b sees lengths[b] - n_tokens[b] + i + 1 tokens.                      */
int sym_pred_batch_raw(sym_ctx* ctx, int32_t n_lips, const int32_t* n_tokens,
                       const int32_t* page_table_flat, const int64_t* pt_offsets,
                       const int64_t* lengths, const void* q, float* out, void* stream);

/* ---- introspection: integer state, compared bit for bit with the oracle's model ----- */
int64_t sym_kv_pages(sym_ctx* ctx, sym_kv kv, int32_t* out, int64_t cap); /* returns count */
int32_t sym_page_refcount(sym_ctx* ctx, int32_t page);                    /* < 0 = error   */
int64_t sym_free_pages(sym_ctx* ctx);
int     sym_get_stats(sym_ctx* ctx, sym_stats* out);

/* The host half of sym_pred_batch alone (usable in a host-only context): plans AND COMMITS
 * the append of the batch (page allocation, copy-on-write decisions) and returns the plan:
 *   cow_out   [3 * cow_cap]  (src page, dst page, slots to copy) per copy, in batch order
 *   slots_out [T]            destination of each new token as page * P + slot
 * *n_cow receives the number of copies.  Either output may be NULL.                      */
int sym_plan_append(sym_ctx* ctx, int32_t n_lips, const sym_kv* kv, const int32_t* n_tokens,
                    int32_t* cow_out, int64_t cow_cap, int32_t* n_cow, int32_t* slots_out);
/* 1 if the last planned batch (sym_plan_append, sym_pred_batch, sym_kv_append) has to run its
 * page copies before its appends, 0 if they may run in any order.  Copies take the slots of a
 * shared, partly filled page below what the copying file sees, appends the slots from what
 * the appending file sees on: disjoint when both see the same, as forks do; after a truncate
 * or an extract a sharer may see less, and once the others have copied and left it appends
 * in place into slots that their copies still read.                                        */
int sym_plan_copies_first(sym_ctx* ctx);

/* The packed descriptor of the attention launch for a batch given by page tables (same
 * arguments as sym_pred_batch_raw), written to host memory for inspection: int32 words.
 * Layout: words[0..47] = header {n_rows, n_waves, n_partials, n_lips, n_tiles, then word
 * offsets of the sections: rows, wave_work, merge, page_table, pt_off, tiles; total words;
 * total units (lo, hi); n_merge; offset of the member list; n_members; n_shared_tiles;
 * [18] workgroups of the tile part of the launch; [20..28] the 9 offsets that cut the tile list
 * into 8 shares of equal cost, one per XCD (workgroup b runs tile b / 8 of share b % 8);
 * [32] n_segs, [33] offset of the segments, [34] n_bins, [35] wavefronts of a bin,
 * [36] offset of the in-bin merge lists (all five 0 when ranges are cut globally, as the
 * matrix-core decode kernel wants: wave_work is then one record per wavefront slot);
 * [37] n_groups, [38] offset of the order table (0 unless the launch holds tiles and bins)},
 * then the sections:
 *   rows      [n_rows][4]   page-table offset, tokens the row's first new token sees, its q/out
 *                           row, and in one word: first page of the row's own range (low 28 bits;
 *                           pages before it belong to a shared prefix) | (new tokens in the
 *                           row - 1) << 28 (a row holds up to 4 consecutive draft tokens of a LIP)
 *   wave_work [n_waves][8]  global cut: row, kv head, page, units, first partial, ids of the
 *                           first three pages of the first range (its first loads need no
 *                           table lookup).  Bins (decode workgroups of [35] wavefronts; wavefront
 *                           w of bin b is record b * [35] + w): first segment, page inside it,
 *                           units, 0, ids of its first three pages, 0: the wavefronts of a bin
 *                           take equal consecutive parts of the bin's segments
 *   segs      [n_segs + 2][8]  (bins) a (row, kv head) range or the part of one that falls
 *                           into a bin: page-table offset, kv head, first page, end page,
 *                           tokens the row sees, q row * Hq + first query head, destination
 *                           (-1: the output rows; else the partial slot of its first piece),
 *                           pool slot (page * 16 + token) that receives the row's new K/V
 *                           row from the wavefront reading the last page (-1: none); two
 *                           spare records end the list
 *   lmerge    [n_bins][32]  (bins) segments of the bin that its wavefronts cut into pieces,
 *                           combined through LDS when the workgroup ends: count, first and
 *                           end segment of the bin, 0, then per cut segment: segment, LDS
 *                           slot of its first piece, wavefront of that piece, pieces
 *   order     [n_groups]    (tiles and bins in one launch) what each group of 8 workgroups
 *                           (one per XCD) runs, in launch order: g >= 0 = tile workgroups
 *                           8g .. 8g + 7, g < 0 = bins 8 * ~g .. 8 * ~g + 7
 *   merge     [n_merge][8]  first partial, pieces, q row * Hq + first query head, then the
 *                           partials of the row's shared prefix: first, stride, count; then the
 *                           distance between the own pieces (tokens in the row); 0
 *   page_table, pt_off [n_lips + 1]   page ids file by file; a member of a shared-prefix group
 *                           that is not the first member of a tile leaves out the common
 *                           pages (nothing reads them through its table) and its offset,
 *                           in rows and in pt_off, is moved back by their number, so that
 *                           entry offset + i is page i for every i from its first own page on
 *   tiles     [n_tiles][12] page-table offset, file length before the call, first q/out row
 *                           (shared: offset into the member list), new tokens (shared: members)
 *                           in the tile, kv head, token offset in the chunk (shared: first
 *                           partial slot), kind (0 prefill chunk, 1 shared prefix), first page,
 *                           end page, 0, 0, 0; ordered share by share
 *   members   [n_members]   q rows of the members of shared-prefix tiles
 * Returns the number of words (or a negative status); writes at most cap words.             */
int64_t sym_build_desc(sym_ctx* ctx, int32_t n_lips, const int32_t* n_tokens,
                       const int32_t* page_table_flat, const int64_t* pt_offsets,
                       const int64_t* lengths, int32_t* words_out, int64_t cap);

/* Test/debug aid: gather tokens [start, start+n) of a file from the pool into contiguous
 * device arrays k_out, v_out [n][Hkv][D] (storage dtype).                                */
int sym_kv_read(sym_ctx* ctx, sym_kv kv, int64_t start, int32_t n, void* k_out, void* v_out,
                void* stream);
int sym_kv_read_layer(sym_ctx* ctx, sym_kv kv, int32_t layer, int64_t start, int32_t n,
                      void* k_out, void* v_out, void* stream);

/* Test hook: the next `count` reservations of pinned staging memory on this context fail with
 * SYM_EHIP (as if the runtime had no pinned memory left).  Every call that changes file-system
 * state reserves its staging memory BEFORE the change, so such a failure must leave page tables,
 * lengths, reference counts and the free set exactly as they were; tests check that.  Works in a
 * host-only context too (whose calls stage nothing but still pass through the reservation).  */
int sym_test_fail_staging(sym_ctx* ctx, int32_t count);

/* ---- inference scheduler: when to fire a batch (section 4.4) ------------------------- */
/* The controller that decides WHEN the pending pred calls go to the GPU as one batch.  The
 * paper states the trade-off (too early wastes the GPU, too late makes threads wait) and that
 * the batch size follows the average call frequency through an arrival model such as a Poisson process; the
 * formulas are this library's: arrival rate lambda = 1 / (exponentially weighted mean gap);
 * service time S(b) = a + c*b fitted to the batches reported with sym_sched_done; target batch
 * b* = lambda*a / (1 - lambda*c) (the fixed point b = lambda*S(b): expected arrivals during one
 * service period), max_batch when lambda*c >= 1.  sym_sched_decide, asked while the GPU is
 * idle, returns how many of the OLDEST pending calls to fire now: all of them (at most
 * max_batch) if there are b* of them, if the oldest has waited max_wait_us, or if the missing
 * ones are not expected before that deadline; otherwise 0 (wait; ask again at the next arrival
 * or at sym_sched_next_deadline).  Times are microseconds on any clock of the caller's.  Host
 * only, no device work; not thread-safe (one scheduler thread owns it).
 *   weight: weight of a new sample in the running means (0 < weight <= 1, e.g. 0.125);
 *   a_us, c_us: service model until measurements arrive.                                   */
typedef struct sym_sched sym_sched;
sym_sched* sym_sched_create(int32_t max_batch, double max_wait_us, double weight, double a_us,
                            double c_us);               /* NULL on a bad argument */
void    sym_sched_destroy(sym_sched* s);
void    sym_sched_arrive(sym_sched* s, double now_us);  /* one pred call became pending   */
int32_t sym_sched_decide(sym_sched* s, double now_us, int gpu_idle);
void    sym_sched_fired(sym_sched* s, int32_t n);       /* the n oldest calls were fired  */
void    sym_sched_done(sym_sched* s, int32_t n, double service_us);   /* that batch took this long */
double  sym_sched_next_deadline(sym_sched* s);          /* +inf when nothing is pending   */
/* Current estimates; any output pointer may be NULL. */
int     sym_sched_state(sym_sched* s, double* rate_per_us, double* target_batch, double* a_us,
                        double* c_us, int64_t* pending);

/* ---- measurement ------------------------------------------------------------------- */
/* Kernel ids for sym_profile_read. */
#define SYM_K_PROLOGUE 0   /* descriptor copy + copy-on-write copies + KV append, one launch */
#define SYM_K_ATTN     1   /* attention over the page tables: decode ranges + MFMA tiles     */
#define SYM_K_MERGE    2   /* merge of the partial results of ranges that were cut           */
#define SYM_K_MOVE     3   /* token copies of sym_kv_extract / sym_kv_merge                  */
#define SYM_K_SWAP     4   /* page copies of sym_kv_offload / sym_kv_restore                 */
#define SYM_K_COUNT    5
/* sym_profile_enable(mask): bit k (k < 8) of mask set = launches of kernel id k are bracketed by
 * HIP events on the launch stream (at most 4096 timed launches are kept per kernel id, later
 * ones are not timed).  For SYM_K_ATTN the two events are attached to the dispatches themselves
 * (start of the first kernel of the attention launch, end of its last): kernel time only; bits 8..23 of mask = stride s (0 or 1: every launch; s > 1: every s-th
 * launch of each kernel id, so that the two event records do not stretch every step); mask 0 = off.
 * sym_profile_read synchronises on the recorded events and returns the summed duration in
 * milliseconds and the number of timed launches of one kernel id, then forgets them.     */
int sym_profile_enable(sym_ctx* ctx, int mask);
int sym_profile_read(sym_ctx* ctx, int kernel_id, double* total_ms, int64_t* launches);

/* Calibration kernels of known traffic: a streaming read of `bytes` bytes (sum written to
 * out8, 8 bytes) and a plain copy dst <- src.  bytes must be a multiple of 16.           */
int sym_calib_read(const void* src, int64_t bytes, void* out8, void* stream);
int sym_calib_copy(void* dst, const void* src, int64_t bytes, void* stream);
/* Calibration of the matrix cores: `blocks` workgroups of 8 wavefronts (two per SIMD, the occupancy of
 * the prefill tile kernel) issue nothing but 32x32x16 bf16 MFMAs on register operands, 16 per
 * iteration and wavefront: blocks * 8 * iters * 16 * 32768 flops.  out: device, blocks * 512
 * floats (one per thread, keeps the work alive).  Timed by the caller; what it sustains is
 * the rate the part delivers under its power limit, below the nominal peak.                */
int sym_calib_mfma(float* out, int32_t blocks, int32_t iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SYMPHONY_KV_H */
