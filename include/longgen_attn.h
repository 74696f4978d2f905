/*
 * longgen_attn.h — C ABI of liblonggen_attn.so
 *
 * Causal sparse attention for the "efficient layers" of the LongGen hybrid
 * model (arxiv 2410.01485): attention-sink + sliding-window attention and
 * blockwise strided sparse attention (paper Section 3.1, paragraph "Different
 * KV-Reduced Attention Strategies"; settings in Section 4.1), as a fused
 * block-skipping kernel for prefill forward and backward (Section 3.2) and a
 * bandwidth-bound decode kernel over the rolling-buffer KV cache (Section 3.2,
 * second paragraph).  Hand-written HIP for gfx950; one GPU.
 *
 * ---------------------------------------------------------------------------
 * THE MASK (integer-only; every entry point uses exactly this predicate)
 * ---------------------------------------------------------------------------
 * i = query position, j = key position, both 0-based in the same index space.
 *   b  = max(block, 1)            granularity of the pattern in tokens
 *   qb = i / b,  kb = j / b       block indices (integer division)
 *   sb = sink / b, wb = window / b   (exact when block > 1: enforced)
 *
 *   live(i,j) :=  j <= i  &&  (  kb < sb                              sink
 *                             || qb - kb < wb                         local window (own block included)
 *                             || (stride > 0 && kb % stride == stride-1)   strided block columns
 *                             )
 *
 * block <= 1, stride == 0  =>  token-exact sink + sliding window:
 *        j <= i && (j < sink || i - j < window)      (exactly `window` keys incl. the query itself)
 * block == 64, sink == 64, window == 2048            the paper's AttnSink setting (Section 4.1)
 * block == 64, stride == 64                          the paper's BlockSparse setting (Section 4.1)
 * The strided columns are ABSOLUTE block indices (the same for every query and
 * every head — Section 3.1 criterion "static access of position"), which is
 * what lets the KV cache keep one block in every `stride` (Section 4.1).
 * The residue (last block of each group of `stride`) is this library's
 * convention; the paper does not state one.
 *
 * ---------------------------------------------------------------------------
 * Conventions common to all calls
 * ---------------------------------------------------------------------------
 * Pointers q/k/v/out/dout/dq/dk/dv/lse/workspace/caches are DEVICE pointers
 * (hipMalloc'ed or PyTorch-owned), 16-byte aligned, dense row-major with the
 * head dimension D innermost and no strides:
 *     prefill  q,out,dout,dq : [B, Hq,  N, D]      k,v,dk,dv : [B, Hkv, N, D]
 *              lse           : [B, Hq,  N]  float32, natural log of the sum of
 *                              exp(scaled scores) over the live keys of a row
 *     decode   q,out : [B, Hq, D]   k_cache,v_cache : [B, Hkv, sink+window, D]
 *              lse   : [B, Hq] float32
 *     (the *_varlen calls pack sequences of different lengths per head: see there)
 * Element type of q/k/v/out/dout/dq/dk/dv/caches is `dtype` (lg_dtype);
 * accumulation and softmax are always float32.
 * GQA: query head hq reads kv head hq / (Hq/Hkv)  (consecutive query heads
 * share a kv head; Llama-2-70B, Section 4.1).  dk/dv of a kv head are the sum
 * over its Hq/Hkv query heads.
 * scale <= 0 selects 1/sqrt(D).
 * Ownership: the caller owns every buffer.  The library allocates nothing,
 * frees nothing, never synchronises, and enqueues all work on `hip_stream`
 * (a hipStream_t passed as void*; NULL = the default stream).  Outputs are
 * fully overwritten.  Scratch memory comes from the caller through `workspace`
 * (size from the matching *_workspace_bytes call; contents need not be
 * initialised and are undefined afterwards).
 * Errors: every call returns an lg_status.  All argument checks run before
 * the first HIP call, so they behave the same on a host without a GPU.
 *   LG_ERR_NULL         a required pointer is NULL (lse may be NULL in fwd and
 *                       decode: then it is not written)
 *   LG_ERR_INVALID_ARG  B,Hq,Hkv,N < 1; N > 2^30; Hq % Hkv != 0; sink < 0; window < 1
 *                       (so every row has at least one live key); block < 0;
 *                       stride < 0; block > 1 with sink % block != 0 or
 *                       window % block != 0; a pointer not 16-byte aligned;
 *                       B*H*N*D beyond 2^40 elements
 *   LG_ERR_UNSUPPORTED  D not in {64, 128}; dtype not in lg_dtype; lg_sparse_attn_decode
 *                       with stride > 0 (use lg_sparse_attn_decode_cache); Hq/Hkv > 16
 *                       in decode
 *   LG_ERR_WORKSPACE    workspace NULL or smaller than *_workspace_bytes
 *   LG_ERR_LAUNCH       the HIP runtime reported an error at launch (no GPU,
 *                       wrong architecture, ...)
 * Any N >= 1 works (ragged tails are masked), not only multiples of a tile.
 */
#ifndef LONGGEN_ATTN_H_
#define LONGGEN_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LG_OK = 0,
  LG_ERR_NULL = 1,
  LG_ERR_INVALID_ARG = 2,
  LG_ERR_UNSUPPORTED = 3,
  LG_ERR_WORKSPACE = 4,
  LG_ERR_LAUNCH = 5
} lg_status;

typedef enum { LG_F32 = 0, LG_BF16 = 1 } lg_dtype;

/* Static, never-freed description of a status code. */
const char* lg_status_str(int status);

/*
 * Prefill forward (Section 3.2, first paragraph: a FlashAttention-style fused
 * kernel that never loads key blocks whose mask is zero).
 *   out[b,hq,i,:] = sum_j P_ij v[b,hk,j,:],  P_ij = exp(scale*<q_i,k_j> - lse_i)
 *   over the keys j with live(i,j);  lse_i = ln sum_j exp(scale*<q_i,k_j>).
 * out has the dtype of q (float32 results rounded to nearest-even for bf16).
 */
int lg_sparse_attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
                       int B, int Hq, int Hkv, int N, int D,
                       int sink, int window, int block, int stride,
                       int dtype, float scale, void* hip_stream);

/*
 * Backward of lg_sparse_attn_fwd (Section 3.2: masked blocks are skipped in the
 * backward step as well; Table 1 counts forward and backward FLOPs).
 * Inputs: q,k,v, the forward's out and lse, and dout = dLoss/dout.
 *   Delta_i = <dout_i, out_i>;   dP_ij = <dout_i, v_j>;   dS_ij = P_ij (dP_ij - Delta_i)
 *   dq_i = scale * sum_j dS_ij k_j;   dk_j = scale * sum_i dS_ij q_i;   dv_j = sum_i P_ij dout_i
 * (sums over live pairs only; dk/dv also summed over the query heads of a kv head).
 * workspace holds per-row values (float32 [B,Hq,N]: Delta on the float32 path; -Delta and
 * -lse / scale on the bf16 path), any float32 partial sums and, on the bf16 path, the counters
 * of the kernels' work queues (cleared by every call).  A workspace belongs to one call at a
 * time: two calls that may overlap (different streams) need a workspace each.  It must be ordinary device memory (hipMalloc /
 * PyTorch): with a strided pattern or Hq > Hkv the bf16 path adds partial dk/dv sums of sink
 * and strided-column keys into it with hardware float atomics; their order is not fixed, so
 * the last bits of those dk/dv rows can differ between runs (a sink + window call with
 * Hq == Hkv uses no atomics and is bit-reproducible).
 */
size_t lg_sparse_attn_bwd_workspace_bytes(int B, int Hq, int Hkv, int N, int D,
                                          int sink, int window, int block, int stride, int dtype);
int lg_sparse_attn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                       const void* dout, void* dq, void* dk, void* dv,
                       void* workspace, size_t workspace_bytes,
                       int B, int Hq, int Hkv, int N, int D,
                       int sink, int window, int block, int stride,
                       int dtype, float scale, void* hip_stream);

/*
 * Measurement aid (benchmarks only): lg_sparse_attn_bwd with each of its three kernels
 * bracketed by HIP events on hip_stream.  Synchronises the stream and writes the kernel
 * durations in milliseconds to the HOST array kernel_ms[3] = {set-up, dq, dk/dv}:
 *   set-up  float32 path: the Delta pre-pass kernel; bf16 path: the kernel that clears the work-queue
 *           counters (a few microseconds: on that path Delta is formed inside the dq kernel)
 *   dq      the dq kernel
 *   dk/dv   the dk/dv kernel and, for strided patterns and GQA, what precedes it: the column-table
 *           kernel, the clearing of the partial sums and the column instance
 * Creates and destroys its events; results are those of lg_sparse_attn_bwd.
 */
int lg_debug_bwd_kernel_ms(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, void* dq, void* dk, void* dv,
                           void* workspace, size_t workspace_bytes,
                           int B, int Hq, int Hkv, int N, int D,
                           int sink, int window, int block, int stride,
                           int dtype, float scale, void* hip_stream, float* kernel_ms);

/*
 * Prefill over a batch of sequences of DIFFERENT lengths, packed without padding (Section 4.3 measures
 * prefilling in a serving setting, where the requests of a batch differ in length; Section 3.2's
 * kernel applied per sequence).  Layout: the sequences lie one after the other along the token axis
 * of every head,
 *     q,out,dout,dq : [Hq,  T, D]      k,v,dk,dv : [Hkv, T, D]      lse : [Hq, T] float32
 * with T = cu_seqlens[num_seqs]; sequence s owns rows cu_seqlens[s] .. cu_seqlens[s+1]-1 of each head.
 * cu_seqlens is a HOST array of num_seqs + 1 non-decreasing offsets starting at 0, read during the
 * call only.  Every sequence is attended on its own, positions counted from its first token:
 * the results of sequence s equal lg_sparse_attn_fwd / lg_sparse_attn_bwd with B = 1 and
 * N = its length on its rows (bit for bit on the paths those calls reproduce bit for bit).
 * Empty sequences are allowed and skipped; when all are empty nothing is enqueued.
 * No work is spent on padding.  The bf16 forward puts up to 128 sequences into one launch (every
 * (sequence, head, 256-row query tile) is a workgroup of the same grid, so short sequences fill the GPU
 * together; each sequence's pattern is cut to its length on the device).  The float32 forward and the
 * backward enqueue one set of launches per sequence, in order, each at the sequence's own length: there
 * the launches of short sequences (under ~64K query rows x heads) do not fill the GPU.
 * The backward workspace is shared by the sequences (size = the largest any of them needs; the
 * remarks on lg_sparse_attn_bwd's workspace apply).
 * Errors, beyond the common ones: LG_ERR_NULL for cu_seqlens == NULL; LG_ERR_INVALID_ARG for
 * num_seqs < 1, cu_seqlens[0] != 0, a decreasing offset, a sequence longer than 2^30, or
 * Hq*T*D beyond 2^40 elements.  *_workspace_bytes returns 0 for invalid arguments.
 */
int lg_sparse_attn_fwd_varlen(const void* q, const void* k, const void* v, void* out, float* lse,
                              const int* cu_seqlens, int num_seqs, int Hq, int Hkv, int D,
                              int sink, int window, int block, int stride,
                              int dtype, float scale, void* hip_stream);
size_t lg_sparse_attn_bwd_varlen_workspace_bytes(const int* cu_seqlens, int num_seqs, int Hq, int Hkv, int D,
                                                 int sink, int window, int block, int stride, int dtype);
int lg_sparse_attn_bwd_varlen(const void* q, const void* k, const void* v, const void* out, const float* lse,
                              const void* dout, void* dq, void* dk, void* dv,
                              void* workspace, size_t workspace_bytes,
                              const int* cu_seqlens, int num_seqs, int Hq, int Hkv, int D,
                              int sink, int window, int block, int stride,
                              int dtype, float scale, void* hip_stream);

/*
 * Decode over the reduced KV cache (Section 3.2, second paragraph: loading the
 * KV cache is the bottleneck; the attention-sink variant keeps the window in a
 * rolling buffer).  One query per (b,hq): the token at position N-1 of a
 * context of N tokens, whose own k/v is already in the cache.
 * Cache slot map: token p lives in slot p when p < sink, otherwise in slot
 * sink + ((p - sink) % window).  The first min(N, sink+window) slots are valid;
 * they hold exactly the keys j with live(N-1, j), so the result equals row N-1
 * of lg_sparse_attn_fwd on the whole context.  stride must be 0 here (a strided pattern
 * needs the retained-block part of the cache: lg_sparse_attn_decode_cache below); with
 * block > 1 the part of the ring that belongs to the block that just left the window is
 * skipped.
 * workspace holds float32 partial results of the split over cache slots.
 */
size_t lg_sparse_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int N, int D,
                                             int sink, int window, int dtype);
int lg_sparse_attn_decode(const void* q, const void* k_cache, const void* v_cache, void* out, float* lse,
                          void* workspace, size_t workspace_bytes,
                          int B, int Hq, int Hkv, int N, int D,
                          int sink, int window, int block, int stride,
                          int dtype, float scale, void* hip_stream);

/*
 * Reduced KV cache for every pattern (Section 3.2: a fixed cache-management rule, no per-step
 * token selection; Section 4.1: the block-sparse variant keeps one block per `stride` blocks,
 * about 2K tokens at 128K).  A cache row [cache_slots, D] of one (b, kv head) is laid out as
 *     [ sink tokens | rolling window of `window` tokens | retained strided blocks ]
 * Token p is stored in slot p when p < sink, otherwise in slot sink + ((p - sink) % window);
 * when its block kb = p / max(block,1) is a strided column (stride > 0 and
 * kb % stride == stride - 1) it is also stored in slot
 * sink + window + (kb / stride) * max(block,1) + p % max(block,1), which is never reused.
 *
 * lg_kv_cache_slots: slots a row needs for contexts of up to n_max tokens
 *   (sink + window when stride == 0); 0 if the arguments are invalid.
 * lg_kv_ring_append: stores the T tokens at positions pos .. pos+T-1.
 *   k_new, v_new : [B, Hkv, T, D] device;  k_cache, v_cache : [B, Hkv, cache_slots, D] device,
 *   updated in place (other slots keep their contents).  The result is what storing the tokens
 *   one by one in position order would give.  T = N, pos = 0 builds the cache after a prefill.
 *   LG_ERR_INVALID_ARG also when T < 1, pos < 0, or cache_slots < lg_kv_cache_slots(pos + T, ...).
 * lg_sparse_attn_decode_cache: decode (as lg_sparse_attn_decode: the query is token N-1, its
 *   own k/v already appended) for any pattern, over caches [B, Hkv, cache_slots, D] with
 *   cache_slots >= lg_kv_cache_slots(N, ...).  Reads the sink slots, the live part of the
 *   rolling window and the retained blocks older than the window, each live key once; equals
 *   row N-1 of lg_sparse_attn_fwd on the whole context.  lg_sparse_attn_decode is this call
 *   with cache_slots = sink + window (stride == 0).
 */
size_t lg_kv_cache_slots(int n_max, int sink, int window, int block, int stride);
int lg_kv_ring_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                      int B, int Hkv, int D, int T, int pos, int cache_slots,
                      int sink, int window, int block, int stride, int dtype, void* hip_stream);
size_t lg_sparse_attn_decode_cache_workspace_bytes(int B, int Hq, int Hkv, int N, int D,
                                                   int sink, int window, int block, int stride, int dtype);
int lg_sparse_attn_decode_cache(const void* q, const void* k_cache, const void* v_cache, void* out,
                                float* lse, void* workspace, size_t workspace_bytes,
                                int B, int Hq, int Hkv, int N, int D,
                                int sink, int window, int block, int stride, int cache_slots,
                                int dtype, float scale, void* hip_stream);
/*
 * lg_sparse_attn_decode_cache for callers that cannot allocate or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the
 * workspace), same kernels and bit-identical results; the partial results of the split over cache
 * slots go to a scratch array of LG_DECODE_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (every GPU the library runs on holds it until the process ends).  Calls no allocating or
 * freeing routine.  The first call on a device looks up the array's device address (make one call
 * before capturing a graph).  LG_ERR_WORKSPACE when the call would need more scratch than the array
 * holds (lg_sparse_attn_decode_cache_workspace_bytes tells; e.g. more than about 16000 (b, query head,
 * split) records at D = 128): use lg_sparse_attn_decode_cache then.  All calls on one GPU share the
 * array: two calls that may overlap in time (different streams) race; calls on one stream do not.
 * Nothing in the array needs clearing between calls (every record is written before it is read).
 */
#define LG_DECODE_STATIC_SCRATCH_BYTES (8u << 20)
int lg_sparse_attn_decode_cache_static(const void* q, const void* k_cache, const void* v_cache, void* out,
                                       float* lse, int B, int Hq, int Hkv, int N, int D,
                                       int sink, int window, int block, int stride, int cache_slots,
                                       int dtype, float scale, void* hip_stream);

/*
 * Serving-style layout (the paper's inference section measures inside a paged-cache serving
 * engine): a paged cache shared by sequences of different lengths.
 *   k_pages, v_pages : [num_pages, Hkv, page_size, D] device; page_size a power of two, 16..4096
 *   page_table       : [B, pages_per_seq] int32 device; entry x of sequence b names the page that
 *                      holds its cache slots [x*page_size, (x+1)*page_size); the slot layout of a
 *                      sequence is the one of lg_kv_ring_append
 *   seq_lens         : [B] int32 device, context length of each sequence (the query is its last
 *                      token); values outside [1, n_max] are clamped
 *   positions        : [B] int32 device, position of the first of the T new tokens per sequence
 * n_max bounds the context lengths: pages_per_seq * page_size >= lg_kv_cache_slots(n_max, ...)
 * is required, and the workspace is sized for it.  Every table entry a sequence can reach must be
 * in [0, num_pages); an entry outside that range is clamped into it on the device (the result of that
 * sequence is then wrong, but nothing outside the pool is read or written).
 * lg_kv_paged_append stores k_new, v_new [B, Hkv, T, D]; a strided-block copy whose slot lies
 * beyond pages_per_seq pages is dropped.
 */
size_t lg_sparse_attn_decode_paged_workspace_bytes(int B, int Hq, int Hkv, int n_max, int D,
                                                   int sink, int window, int block, int stride, int dtype);
int lg_sparse_attn_decode_paged(const void* q, const void* k_pages, const void* v_pages,
                                const int32_t* page_table, const int32_t* seq_lens, void* out, float* lse,
                                void* workspace, size_t workspace_bytes,
                                int B, int Hq, int Hkv, int n_max, int D,
                                int sink, int window, int block, int stride,
                                int page_size, int pages_per_seq, int num_pages,
                                int dtype, float scale, void* hip_stream);
int lg_kv_paged_append(const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                       const int32_t* page_table, const int32_t* positions,
                       int B, int Hkv, int D, int T, int n_max,
                       int sink, int window, int block, int stride,
                       int page_size, int pages_per_seq, int num_pages, int dtype, void* hip_stream);

/*
 * Measurement aid, not a product path: decode over the token-granular cache of
 * lg_sparse_attn_decode with the work split over the HEAD DIMENSION instead of the cache slots,
 * the design the paper describes for its decode kernel (Section 3.2, second paragraph: the loading
 * of the head dimension is split across thread blocks).  Two halves of D, two passes (partial
 * scores through the workspace, then softmax and the V slice).  Same arguments and result as
 * lg_sparse_attn_decode with block <= 1, stride == 0; workspace from the call below.  Exists so
 * that the two splits can be timed against each other on the same inputs.
 */
size_t lg_debug_decode_split_headdim_workspace_bytes(int B, int Hq, int sink, int window);
int lg_debug_decode_split_headdim(const void* q, const void* k_cache, const void* v_cache, void* out, float* lse,
                                  void* workspace, size_t workspace_bytes,
                                  int B, int Hq, int Hkv, int N, int D, int sink, int window,
                                  int dtype, float scale, void* hip_stream);

/*
 * Host-only: the runs of consecutive cache slots a decode step at context length N reads
 * (at most 4; start/len are HOST arrays of 4 entries; *nseg receives the count).  Runs the
 * same source the decode launch uses (no GPU needed).
 */
int lg_debug_decode_segments(int N, int sink, int window, int block, int stride,
                             int* nseg, int32_t* start, int32_t* len);

/*
 * Host-only view of the block-skipping tile scheduler (Section 3.2: the mask is
 * kept in compressed-sparse-row form, O(N) memory; it is static for all heads).
 * Writes, in CSR form, the list of live kernel tiles the device code walks:
 *   transposed == 0: rows are query tiles, columns key tiles (forward, dq);
 *   transposed == 1: rows are key tiles, columns query tiles (dk/dv).
 * tq/tk receive the kernel tile sizes used for `dtype`.  row_ptr has rows+1
 * entries; col_idx/kind have row_ptr[rows] entries; kind is 1 when every
 * (i,j) of the tile is live (no masking needed) and 0 when the predicate must
 * be applied per element.  All output pointers are HOST pointers; cap is the
 * capacity of col_idx/kind in entries and row_cap that of row_ptr; *needed
 * always receives the number of live tiles and *rows the number of rows, and
 * nothing is written past a capacity (call once with cap = 0 to size).
 * Runs the same source the kernels compile (no GPU needed).  The lists are in increasing
 * tile order; the kernels visit the same tiles, some of them in a rotated order (the result of
 * the online softmax and of the gradient sums does not depend on the order).
 */
int lg_debug_tile_map(int N, int sink, int window, int block, int stride, int dtype, int transposed,
                      int* tq, int* tk, int32_t* row_ptr, size_t row_cap,
                      int32_t* col_idx, uint8_t* kind, size_t cap,
                      size_t* rows, size_t* needed);

/*
 * Host-only: the ORDER in which the bf16 kernels visit the live tiles of one row of the tile map
 * (row = query tile for transposed == 0, key tile for transposed == 1).  Patterns without
 * strided columns walk their contiguous run of tiles rotated (see lg_debug_tile_map); for a key
 * tile the window part comes first (rotated), then the column part in increasing order.
 * order: HOST array of cap entries (may be NULL with cap = 0); *count receives the number of
 * tiles.  The set of tiles equals the row of lg_debug_tile_map.
 */
int lg_debug_tile_walk(int N, int sink, int window, int block, int stride, int transposed, int row,
                       int32_t* order, size_t cap, size_t* count);

/*
 * Host-only: the pattern as the kernels hold it for a sequence of n tokens, derived from the pattern made for
 * n_made_for >= n tokens (the packed different-lengths forward makes ONE pattern for a length no sequence
 * exceeds and derives each sequence's own on the device; sink, window and the strided columns are cut to the
 * sequence's length).  fields: HOST array of 9 entries = {n, sink, window, max(block, 1), stride, sink blocks,
 * window blocks, log2(block) or -1, stride - 1 if a power of two else -1}, after the cut.  With
 * n == n_made_for: the pattern made directly for n.  Runs the same source the kernels compile.
 */
int lg_debug_pattern_fields(int n_made_for, int n, int sink, int window, int block, int stride, int32_t* fields);

/*
 * Host-only: the per-lane register mask the bf16 kernels apply on a PARTIAL tile (a tile with live and
 * dead pairs), computed in closed form from the pattern (Section 3.1) instead of evaluating the
 * predicate per element.  Bit r (0..31) of *bits belongs to the entry at offset 4 * half + 8 * (r / 4) + r % 4
 * along the tile (half = 0 or 1: the lane's half of the wave).
 *   transposed == 0: the lane owns query row `fixed`; the tile is keys tile0 .. tile0 + 63
 *                    (forward, dq): bit r = live(fixed, tile0 + offset)
 *   transposed == 1: the lane owns key `fixed`; the tile is query rows tile0 .. tile0 + 63
 *                    (dk/dv): bit r = (tile0 + offset < N) && live(tile0 + offset, fixed)
 * fixed must be in [0, N), tile0 >= 0.  Runs the same source the kernels compile (no GPU needed).
 */
int lg_debug_partial_tile_bits(int N, int sink, int window, int block, int stride, int transposed,
                               int fixed, int tile0, int half, uint32_t* bits);

#ifdef __cplusplus
}
#endif
#endif /* LONGGEN_ATTN_H_ */
