/* ooco.h -- C ABI of the MI355X (gfx950) mixed-batch paged-attention library.
 *
 * The library runs the attention step of a latency-relaxed serving instance: one call covers
 * many offline *decode* requests (one query token each, reading the request's whole KV cache)
 * together with online *prefill chunks* (several query rows with causal attention on top of
 * already-cached context), all over one non-contiguous ("paged") KV pool.
 *   - mixed placement of online/offline prefill and offline decode on one instance:
 *     paper Section 3.2.1; iteration-level batching of requests of different lengths over a
 *     non-contiguous KV pool: Section 2.1; decode = one token per request reading the entire
 *     KV cache, prefill = causal forward over all input tokens, GQA: Section 2.3;
 *     attention as one fused softmax(QK^T)V operator whose scores never reach memory:
 *     Section 3.3.1 and Table 2 (Attention row).
 * ooco_kv_block_copy moves whole KV blocks between pools (swap-out / swap-in of the requests
 * evicted when an online request preempts offline work, Section 3.4.1; local half of KV
 * migration, Section 3.4.3).
 *
 * Everything is plain C: integers, sizes and raw pointers.  Each pointer argument is marked
 * HOST or DEVICE.  The caller owns every buffer it passes; the library neither frees nor
 * keeps them beyond the stream work of the call.  All entry points return an ooco_status;
 * nothing aborts or throws across this boundary.  Calls that launch GPU work are asynchronous
 * on the given HIP stream: inputs must stay alive and unmodified, and outputs must not be
 * read, until the stream has passed the work of the call.
 * A context is not thread-safe, and the GPU work of two calls on one context must not overlap
 * in time: they share the context's workspace (partial results) and arrival counters.  Calls
 * issued to one stream are ordered by it; callers that drive several streams at once use one
 * context per stream.  The host-only functions (ooco_plan_dry_run, ooco_predict_latency and the
 * scheduling rules at the end of this file) keep no state and may be called from any thread.
 *
 * ---------------------------------------------------------------------------------------
 * Data layout (bf16 = upper 16 bits of IEEE binary32; all tensors contiguous)
 *
 *   q, out       [total_q_tokens][Hq][hd]
 *   k_cache      [num_blocks][Hkv][hd/8][BS][8]
 *                element (block b, kv head h, dim d, slot s) at
 *                (((b*Hkv + h)*(hd/8) + d/8)*BS + s)*8 + d%8
 *   v_cache      [num_blocks][Hkv][hd][BS]
 *                element (b, h, d, s) at ((b*Hkv + h)*hd + d)*BS + s
 *   block_tables int32 [num_seqs][max_blocks_per_seq]
 *   seq_lens, ctx_lens int32 [num_seqs];  query_start_loc int32 [num_seqs+1]
 *
 * BS = 16 tokens per block.  Token j of sequence i is in physical block
 * block_tables[i][j / BS], slot j % BS.  One (block, kv head) tile of K and of V is one
 * contiguous 16*hd*2-byte run whose inner order is the operand order of the CDNA4 bf16 MFMA
 * instructions, so that a 64-lane wave fetches it with fully contiguous 8/16-byte loads and
 * feeds the matrix cores without any shuffle.  A block of K (all kv heads) is one contiguous
 * Hkv*16*hd*2-byte run; the same holds for V.
 *
 * Semantics of one sequence i with q_len_i = query_start_loc[i+1] - query_start_loc[i]:
 *   ctx_lens[i] = tokens cached before this step, seq_lens[i] = ctx_lens[i] + q_len_i.
 *   Query row t (0 <= t < q_len_i) sits at position ctx_lens[i] + t and attends keys
 *   0 .. ctx_lens[i] + t (its own key included; the K/V of this step's tokens are already in
 *   the cache).  Query head h uses kv head h / (Hq/Hkv).  q_len_i == 1 is a decode request,
 *   q_len_i > 1 a prefill chunk, q_len_i == 0 contributes nothing.  Cache slots past
 *   seq_lens[i], unreferenced blocks and unused block-table columns are never used as values
 *   (they may hold NaN/Inf or invalid ids).  The ids in the USED columns, block_tables[i][0 ..
 *   ceil(seq_lens[i]/BS) - 1], must lie in [0, num_blocks): the attention kernels read through them
 *   unchecked.
 *   out = softmax(scale * q K^T) V with fp32 accumulation, rounded to bf16 (nearest even).
 */
#ifndef OOCO_H
#define OOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ooco_ctx ooco_ctx; /* opaque; owns only its workspace and plan buffers */

typedef enum {
    OOCO_OK = 0,
    OOCO_EINVAL = -1,   /* bad argument value (null pointer, negative size, bad option) */
    OOCO_ESHAPE = -2,   /* inconsistent shapes / lengths / unsupported head geometry    */
    OOCO_ENOMEM = -3,   /* allocation failed or workspace too small                     */
    OOCO_EHIP = -4      /* a HIP runtime call or kernel launch failed                   */
} ooco_status;

/* Creates a context for one attention-layer geometry on the current HIP device.
 *   num_q_heads % num_kv_heads == 0, group size num_q_heads/num_kv_heads <= 16,
 *   head_dim in {64, 128}, block_size == 16, num_blocks > 0, max_blocks_per_seq > 0.
 *   softmax_scale <= 0 selects 1/sqrt(head_dim).
 *   workspace: DEVICE memory for split-KV partial results, 256-byte aligned, owned by the
 *   caller and alive until ooco_ctx_destroy; NULL lets the library allocate workspace_bytes
 *   itself (0 = a default of 128 MiB) and free it in ooco_ctx_destroy.
 * On failure *out is NULL and ooco_last_error(NULL) describes the reason. */
ooco_status ooco_ctx_create(ooco_ctx **out, int num_q_heads, int num_kv_heads, int head_dim,
                            int block_size, int64_t num_blocks, int max_blocks_per_seq,
                            float softmax_scale, void *workspace /*DEVICE or NULL*/,
                            size_t workspace_bytes);

/* Frees the context and whatever it allocated (never the caller's buffers).  Waits for the work the
 * context has enqueued: the streams its calls were given (up to four different ones are remembered,
 * beyond that the whole device) and its own side stream; those streams must still exist.  NULL is accepted. */
ooco_status ooco_ctx_destroy(ooco_ctx *ctx);

/* Message of the last failure on this context (or, with ctx == NULL, of the calling thread's
 * last failed ooco_ctx_create).  The string is owned by the library and valid until the next
 * call on the same context / thread. */
const char *ooco_last_error(const ooco_ctx *ctx);

/* Options (name, value >= 0).  Unknown name -> OOCO_EINVAL.
 *
 * Decode run layout; these take effect at the next ooco_plan.  The KV blocks of all decode
 * sequences, laid end to end, are streamed in runs, one launched wave per run and kv head.  A run
 * that crosses a sequence boundary, or a sequence that spans several runs, is handled by partial
 * results merged inside the decode kernel.
 *   "decode_segments"     number of static runs (0 = automatic: three waves per compute unit,
 *                         fewer for small batches)
 *   "decode_tail_pct"     share (percent, default 0 = none) of the line that is cut into short
 *                         runs which the waves fetch from a shared counter once their own run is
 *                         done
 *   "decode_tail_blocks"  KV blocks per such run (default 8)
 *   "xcd_weights"         relative lengths of the static runs per XCD (the eight dies of the GPU
 *                         differ by several percent in delivered memory bandwidth): eight bytes,
 *                         XCD 0 in the lowest, each 1..255; static run v then goes to XCD v % 8
 *                         and the number of static runs is rounded down to a multiple of 8.
 *                         0 (default) = equal runs.  Weights must differ by at most 4x; they
 *                         apply only when the static runs average at least 16 KV blocks.
 *   "decode_piece_pad"    what starting a piece is charged when the line is cut into runs, in KV
 *                         blocks: a run that holds the beginnings of n sequences streams n times
 *                         this many blocks less than a run that holds none, so that all waves
 *                         finish together.  Default 3 * 128 / head_dim (a wave needs about 3 us
 *                         from one piece to the first tile of the next); 0 = runs of equal
 *                         block counts; at most 64.
 * Prefill tiles (takes effect at the next ooco_plan):
 *   "prefill_split"       parts a prefill tile's key range is cut into, 1..16 (more is taken as 16); every part is
 *                         a workgroup of its own and the last one to finish merges their partial
 *                         results (held in the workspace).  0 (default) = automatic: split only
 *                         when the batch cannot occupy the compute units, or when a few tiles on a long context
 *                         would run on long after all others, and an estimate of the kernel time improves by at
 *                         least 3 %; in a batch of at most 896 tiles every tile then gets parts by its own number of
 *                         steps (the tile with the most steps k parts, the others as many as keep their parts no
 *                         longer than that tile's), so that a chunk on a short context stays whole beside one on a
 *                         long context.  A tile never gets more parts than it has 64-key steps.
 *   "prefill_sorted"      0/1/2 (default 1): a batch of at most 896 prefill tiles dispatches the tiles of ALL its
 *                         chunks -- the parts of its tiles, if they are split -- by decreasing number of 64-key
 *                         steps (one list entry per tile or part, in the kernel arguments; at most 896 entries);
 *                         0 or more tiles: chunk by chunk, longest sequence first, the later tiles of
 *                         a chunk first, every tile the same number of parts.  A launch of at most two workgroups per compute unit lists the second
 *                         half of its tiles in ascending order, so that the two workgroups that share a unit are
 *                         a long and a short one (2 = never, plain descending order).  Measured on MI355X, 8 chunks of 512 rows on 175..1781 cached tokens:
 *                         the span of the workgroups 94..98 -> 89..92 us.
 * Batches that hold both prefill chunks and decode sequences (take effect at the next ooco_plan):
 *   "mixed_lean"          the register-lean pair of kernels (head_dim 128): prefill workgroups of eight waves
 *                         (256 query columns, at most 176 registers per wave) beside decode waves of 144 registers,
 *                         four per compute unit, so that a SIMD holds two prefill waves and a decode wave at once.
 *                         1 (default) = automatic: when the prefill part gives every compute unit at least one
 *                         eight-wave workgroup and, by the batch's FLOPs and bytes, would by itself take between
 *                         0.30 and 4 times as long as the decode part (a shorter one does not repay the lean
 *                         decode kernel's 3 %, a longer one not the lean prefill kernel's 5 %); 0 = never (the
 *                         stand-alone kernels side by side); 2 = whenever the batch holds both kinds of work.
 *   "prefill_waves"       waves per prefill workgroup: 4 (128 query columns per staged K/V tile), 8 (256), or
 *                         0 (default) = 4, and 8 where "mixed_lean" applies.  Other values -> OOCO_EINVAL.
 *   "mixed_fused"         0 (default) / 1: 1 = both kinds of work in ONE launch of a persistent kernel in which a
 *                         compute unit runs either decode waves or prefill workgroups (with "overlap" on).  Slower
 *                         than the two kernels side by side at every split measured; kept for measurements.
 *   "mixed_dec_cus"       with "mixed_fused": compute units per XCD that decode (the others prefill); 0 (default) =
 *                         from the batch's bytes and FLOPs; 99 = every unit runs both kinds.
 * Immediate options:
 *   "plan_persistent"  0/1 (default 0): 0 = a plan made by ooco_plan serves exactly one ooco_attn_mixed and is
 *                then used up (a later call without a new plan plans by itself from the device arrays), so that
 *                a caller that advances the lengths on the device between steps can never run on a stale
 *                plan; 1 = the plan stays current for every following call with the same num_seqs and
 *                total_q_tokens until the next ooco_plan -- for callers that repeat one batch (benchmarks,
 *                the layers of one iteration, graph replay), who then answer for the device arrays still
 *                matching it
 *   "overlap"    0/1/2 (default 1): in a batch that holds both prefill chunks and decode sequences,
 *                run the prefill kernel on the context's own side stream (default priority)
 *                concurrently with the decode kernel; the call still appears as one unit of work
 *                on the caller's stream (fork and join by events).  1 = unless the plan estimates the two
 *                kernels at under 80 us together (they then run one after the other on the caller's stream:
 *                measured faster there, and the host enqueues the call in 8 us instead of 41); 2 = always;
 *                0 = never
 *   "decode_first"  0/1 (default 1): with "overlap", enqueue the decode kernel before the prefill
 *                kernel (0: the other way round)
 *   "profile"    0/1: every ooco_attn_mixed records HIP events around its two kernels (each on the
 *                stream the kernel runs on) and around the whole call for ooco_profile_read; at most
 *                1024 calls between two reads
 *   "trace"      0/1: see ooco_trace_read
 * Tuning knobs kept for experiments (defaults are the measured best): "decode_nbi" (KV blocks per
 * softmax step of the decode kernel: 1, 2 or 4; 0 = the plan's choice: 1 for head_dim 128 -- 2 for small batches, whose
 * waves are chains of dependent steps --, 2 for head_dim 64), "copy_sort" (block copy: 0 = pairs in the caller's order, 1 = default: copies of 2048 pairs or more are first
 * ordered by destination id on the device, into a buffer of the context that grows on demand -- measured on MI355X,
 * 13,044 blocks into random slots of a staging pool: 332 -> 314 us including the sort, which costs about 30 us and
 * does not pay when the slots are handed out in ascending order anyway (283 us) -- 2 = always),
 * "append_parts" (KV append: workgroups that share one (sequence, KV block) pair,
 * 1..8; 0 = default), "rotate_heads" (0/1: rotate the kv
 * head of a decode wave by its run index, default 1), "copy_variant" (block copy of this context: 10 * 16-byte
 * vectors per thread + 1 for non-temporal accesses, one of 10, 11, 20, 21, 40, 41, 80, 81; 0 = default 41;
 * any other value -> OOCO_EINVAL). */
ooco_status ooco_set_option(ooco_ctx *ctx, const char *name, int64_t value);

/* Waits for the profiled calls made since the last read and returns the summed event-to-event
 * times in milliseconds: ms_sum[0] = prefill kernel, ms_sum[1] = decode kernel, ms_sum[2] = whole call
 * (HOST double[3]), and the number of calls (HOST).  Either pointer may be NULL.  Resets the sums.
 * Profiling changes neither the launch order nor the streams: in a batch with both kinds of work the two
 * kernels still run side by side, each bracketed by events on its own stream, so the times are those of
 * the kernels as they run in the step (they overlap; the whole-call time is not their sum). */
ooco_status ooco_profile_read(ooco_ctx *ctx, double *ms_sum /*HOST*/, int64_t *calls /*HOST*/);

/* The same, and also the event-to-event times of every call: per_call_ms is a HOST double
 * [cap][3] = (prefill kernel ms, decode kernel ms, whole call ms) for the first cap calls since the
 * last read (may be NULL with cap 0). */
ooco_status ooco_profile_read_calls(ooco_ctx *ctx, double *per_call_ms /*HOST*/, int64_t cap,
                                    double *ms_sum /*HOST double[3]*/, int64_t *calls /*HOST*/);

/* Wave-level trace of the decode kernel, for tuning.  With option "trace" = 1 every decode wave of
 * the following ooco_attn_mixed calls stores four device time stamps (constant 100 MHz clock):
 * wave start, first K/V tiles arrived, end of KV streaming, wave end (after partial results and
 * merge).  ooco_trace_read waits for the streams the context's calls were given and copies the stamps of the last
 * traced call:
 *   stamps: HOST uint64 [cap_waves][4], wave index = run * num_kv_heads + kv head;
 *   waves: HOST, receives the number of decode waves of that call.
 * A traced batch WITHOUT decode sequences stores per prefill workgroup instead (workgroup index = (tile in
 * dispatch order * num_kv_heads + kv head) * parts + part): start, XCD * 256 + compute-unit id, phases, end; `waves`
 * then receives the number of prefill workgroups.  `phases` packs four times since the workgroup's start, 16 bits
 * each (units of 10 ns, saturating at 65535), lowest first: tile looked up, first K/V loads sent off, first tiles
 * arrived in LDS, last step done; 0 for a part of a split tile that had no step to work on.
 * Tracing adds waits to the kernel; never leave it on when measuring throughput. */
ooco_status ooco_trace_read(ooco_ctx *ctx, uint64_t *stamps /*HOST*/, int64_t cap_waves, int64_t *waves /*HOST*/);

/* Plans one batch from HOST copies of the length arrays (the serving scheduler knows every
 * request's length on the CPU; Section 3.3.2 / Algorithm 2 reason about them there): classifies
 * sequences into decode (q_len 1) and prefill (q_len > 1), sums their KV blocks and query tiles
 * into two small cumulative arrays and picks the number of decode runs.  Pure host work, no
 * device call: the arrays travel to the GPU inside the kernel arguments of the next
 * ooco_attn_mixed (batches above 960 sequences: one small asynchronous copy on its stream).
 *   h_seq_lens, h_ctx_lens: HOST int32 [num_seqs]; h_query_start_loc: HOST int32 [num_seqs+1].
 * Checks: query_start_loc starts at 0 and is non-decreasing, ctx + q_len == seq_len,
 * 0 <= lengths, ceil(seq_len/BS) <= max_blocks_per_seq -> OOCO_ESHAPE otherwise;
 * OOCO_ENOMEM when the batch exceeds the context's fixed buffers (2^20 / num_kv_heads sequences).
 * A workspace too small for the wanted number of runs silently lowers that number. */
ooco_status ooco_plan(ooco_ctx *ctx, int num_seqs, const int32_t *h_seq_lens /*HOST*/,
                      const int32_t *h_query_start_loc /*HOST*/, const int32_t *h_ctx_lens /*HOST*/);

/* The planner of ooco_plan as a pure HOST function (no context, no device): validates the length
 * arrays exactly as ooco_plan does and lists the work the kernels will derive from the plan for
 * the given geometry, CU count, workspace size and decode run options (every other option at a context's
 * default).  For schedulers that
 * want to know the split of a batch in advance, and for testing the planner without a GPU.
 *   decode_pieces_out: HOST int32 [decode_cap][5] = (seq, blk_begin, blk_end, slot, run): the KV
 *     block range of sequence seq that decode run `run` streams; slot = partial-result slot, or
 *     -1 when the piece covers the whole sequence and writes the output directly
 *   prefill_tiles_out: HOST int32 [prefill_cap][5] = (seq, q_row0, rows, pos0, parts), in the order in which
 *     the tiles (their first parts) are dispatched; a tile holds up to 128 / (num_q_heads/num_kv_heads) query rows
 *     (256 / ... in the eight-wave kernel) and runs once per kv head; parts = workgroups its key range is cut into
 *   counts: HOST int64 [6] = (decode pieces, prefill tiles, static decode runs, partial-result
 *     slots, dynamically fetched tail runs, the most parts a prefill tile's key range is cut into);
 *     runs are numbered static first, then tail
 *   msg: HOST buffer of msg_cap bytes receiving the error text.  Any output pointer may be NULL.
 *   xcd_weights: NULL for equal static runs, else the relative run lengths per XCD that option
 *     "xcd_weights" would set (static run v then belongs to XCD v % 8).
 *   prefill_split: what option "prefill_split" would set (0 = automatic).
 *   decode_piece_pad: what option "decode_piece_pad" would set; negative = the default. */
ooco_status ooco_plan_dry_run(int num_q_heads, int num_kv_heads, int head_dim, int block_size,
                              int max_blocks_per_seq, int num_cus, size_t workspace_bytes,
                              int64_t decode_segments, int64_t decode_tail_pct, int64_t decode_tail_blocks,
                              int num_seqs, const int32_t *h_seq_lens /*HOST*/,
                              const int32_t *h_query_start_loc /*HOST*/, const int32_t *h_ctx_lens /*HOST*/,
                              int32_t *decode_pieces_out /*HOST*/, int64_t decode_cap,
                              int32_t *prefill_tiles_out /*HOST*/, int64_t prefill_cap,
                              int64_t *counts /*HOST*/, char *msg /*HOST*/, size_t msg_cap,
                              const int32_t *xcd_weights /*HOST, 8 values in 1..255, or NULL*/,
                              int64_t prefill_split, int64_t decode_piece_pad);

/* Numbers describing the last plan made, current or used up (any pointer may be NULL): decode runs (waves per kv head),
 * prefill tiles, KV blocks of all decode sequences, bytes of workspace the partial results use,
 * the most parts a prefill tile's key range is cut into (1 = no tile is split). */
ooco_status ooco_plan_info(const ooco_ctx *ctx, int64_t *decode_waves, int64_t *prefill_tiles,
                           int64_t *decode_blocks, int64_t *workspace_used, int64_t *prefill_parts);

/* Names of the kernels the last plan made launches, as rocprofv3 shows them without the argument list, separated
 * by ';' (decode first), e.g. "decode_kernel_lean<128>;prefill_kernel_lean<128>": for matching profiler output
 * with a batch.  names: HOST buffer of cap bytes. */
ooco_status ooco_plan_kernels(const ooco_ctx *ctx, char *names /*HOST*/, size_t cap);

/* The mixed-batch attention step (operation defined at the top of this file).
 *   q, out: DEVICE bf16 [total_q_tokens][Hq][hd]; k_cache, v_cache: DEVICE, read-only here;
 *   block_tables, seq_lens, query_start_loc, ctx_lens: DEVICE int32 (shapes above).
 *   stream: a hipStream_t (NULL = the default stream).
 * If ooco_plan was called for this batch (same num_seqs and total_q_tokens) its work lists are
 * used and the three DEVICE length arrays are trusted to equal the planned HOST copies; the plan is
 * used up by the call unless option "plan_persistent" is set.
 * Without a current plan the call copies the length arrays to the host, waits for that copy
 * (one stream synchronisation) and plans by itself.
 * Launches at most two kernels (decode with its in-kernel merge, and prefill chunks -- on the context's
 * side stream when the batch holds both kinds of work and is not a short one, see option "overlap") and no
 * copies (batches above 960 sequences: one small copy).
 * Writes every row of out (and the context's workspace), nothing else.  num_seqs == 0 or
 * total_q_tokens == 0 returns OOCO_OK without launching anything.
 * Same context + same plan + same inputs give bit-identical output on every call (no
 * floating-point atomics).  One context serves one stream at a time.
 * A planned call enqueues only kernels and event records / waits, so it can be recorded into a HIP
 * graph (stream capture) and replayed; keep "profile" and "trace" off for captured calls.  A plan
 * with a dynamic tail ("decode_tail_pct") is refused on a capturing stream with OOCO_EINVAL (the
 * tail's ticket base is fixed at enqueue time).
 * Errors: OOCO_EINVAL for null pointers / negative sizes, OOCO_ESHAPE when sizes contradict
 * the plan, OOCO_EHIP when a launch fails (message holds hipGetErrorString). */
ooco_status ooco_attn_mixed(ooco_ctx *ctx, const void *q /*DEVICE*/, const void *k_cache /*DEVICE*/,
                            const void *v_cache /*DEVICE*/, const int32_t *block_tables /*DEVICE*/,
                            const int32_t *seq_lens /*DEVICE*/, const int32_t *query_start_loc /*DEVICE*/,
                            const int32_t *ctx_lens /*DEVICE*/, void *out /*DEVICE*/, int num_seqs,
                            int total_q_tokens, void *stream);

/* ooco_attn_mixed for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No context: the geometry (as for ooco_ctx_create) and the HOST copies of the
 * length arrays (as for ooco_plan) come with the call, the plan is made on the stack, and everything the kernels
 * need beyond the caller's tensors -- arrival counters and the partial results of split sequences -- lives in one
 * 16 MiB array that is part of the library's device code (every GPU the library runs on holds its own copy until the
 * process ends).  The call allocates nothing on host or device, creates no stream or event, never synchronises
 * and enqueues at most three kernels on `stream` (a small fill that zeroes the counters it will use, the prefill
 * kernel, the decode kernel; the two attention kernels run one after the other).
 *   Device arguments, shapes and results as for ooco_attn_mixed; default run layout; prefill tiles are never
 *   split along the context.  Limits: num_seqs <= 960, num_seqs * num_kv_heads <= 65536 (-> OOCO_ENOMEM with a
 *   message beyond them); a partial-result area too small for the usual number of decode runs lowers that number.
 *   All calls on one GPU share the array, which keeps the contents of the last call: calls whose GPU work
 *   overlaps in time on one GPU (two streams, two threads) race and give unspecified results.
 *   msg: HOST buffer of msg_cap bytes for the error text (may be NULL).
 * Errors: OOCO_EINVAL (NULL pointers, negative sizes), OOCO_ESHAPE (geometry, inconsistent lengths), OOCO_ENOMEM
 * (limits above), OOCO_EHIP (symbol lookup or launch failed). */
ooco_status ooco_attn_mixed_static(int num_q_heads, int num_kv_heads, int head_dim, int block_size,
                                   int max_blocks_per_seq, float softmax_scale,
                                   const int32_t *h_seq_lens /*HOST*/, const int32_t *h_query_start_loc /*HOST*/,
                                   const int32_t *h_ctx_lens /*HOST*/, const void *q /*DEVICE*/,
                                   const void *k_cache /*DEVICE*/, const void *v_cache /*DEVICE*/,
                                   const int32_t *block_tables /*DEVICE*/, const int32_t *seq_lens /*DEVICE*/,
                                   const int32_t *query_start_loc /*DEVICE*/, const int32_t *ctx_lens /*DEVICE*/,
                                   void *out /*DEVICE*/, int num_seqs, int total_q_tokens, void *stream,
                                   char *msg /*HOST*/, size_t msg_cap);

/* Whole-block copy for preemption eviction / restore:
 *   for p in [0, num_pairs):  k_dst[dst_block_ids[p]] <- k_src[src_block_ids[p]]  (one block =
 *   Hkv*BS*hd bf16, all slots, garbage tail included) and the same for V.  Bit-exact.
 *   k_src, v_src, k_dst, v_dst: DEVICE pools with the cache layout of this context (the
 *   destination pool may be smaller or the same allocation as the source);
 *   src_block_ids, dst_block_ids: DEVICE int64 [num_pairs].
 * dst ids must be pairwise distinct, and when source and destination are the same allocation
 * no dst id may equal any src id; neither is checked (ids live on the device) and violating
 * it gives unspecified block contents.  Ids must lie inside their pools (unchecked).
 * num_pairs == 0 returns OOCO_OK without a launch.  ctx supplies the block geometry.
 * Large copies (option "copy_sort") are carried out in order of destination id: the result is the same, the
 * caller's id lists are not modified; the first such call on a context allocates the buffer for the ordered lists
 * (never on a capturing stream: a captured copy keeps the caller's order). */
ooco_status ooco_kv_block_copy(ooco_ctx *ctx, const void *k_src /*DEVICE*/, const void *v_src /*DEVICE*/,
                               void *k_dst /*DEVICE*/, void *v_dst /*DEVICE*/,
                               const int64_t *src_block_ids /*DEVICE*/,
                               const int64_t *dst_block_ids /*DEVICE*/, int64_t num_pairs, void *stream);

/* KV append, the step that precedes ooco_attn_mixed: the K and V vectors of this step's tokens are
 * written into their paged slots (the paper's KV cache keeps the K/V of every processed token for
 * reuse by later steps, Section 2.1 and 2.3): row query_start_loc[i] + t of k_new / v_new is the
 * token at position ctx_lens[i] + t of sequence i and goes to block
 * block_tables[i][pos / BS], slot pos % BS.  Bit-exact; no other element of the pools changes.
 *   k_new, v_new: DEVICE bf16 [total_q_tokens][Hkv][hd]; k_cache, v_cache: DEVICE pools of this
 *   context's geometry (written); block_tables, query_start_loc, ctx_lens: DEVICE int32 as for
 *   ooco_attn_mixed (seq_lens is not needed).
 * Needs no plan, never synchronises, one kernel on `stream`.  Rows whose position lies beyond the
 * block table, or whose block id lies outside [0, num_blocks), are skipped (ids are otherwise
 * trusted).  num_seqs == 0 or total_q_tokens == 0 returns OOCO_OK without a launch. */
ooco_status ooco_kv_append(ooco_ctx *ctx, const void *k_new /*DEVICE*/, const void *v_new /*DEVICE*/,
                           void *k_cache /*DEVICE*/, void *v_cache /*DEVICE*/, const int32_t *block_tables /*DEVICE*/,
                           const int32_t *query_start_loc /*DEVICE*/, const int32_t *ctx_lens /*DEVICE*/,
                           int num_seqs, int total_q_tokens, void *stream);

/* Roofline latency model of the attention operator (paper Section 3.3: Table 2 gives the operator's
 * FLOPs 4*D_h*S_q*S_kv and bytes 2d*(S_q*D_h + S_kv*D_h*H_kv/H_q) with D_h = H_q*head_dim.  Table 2 as
 * printed shows the head ratio of the KV term as H_q/H_kv; the library uses H_kv/H_q, because the KV
 * tensors have H_kv heads of head_dim values per token, i.e. D_h*H_kv/H_q values (grouped-query attention
 * shrinks the KV cache, Section 2.3).  Equation 1
 * gives its latency max(FLOPs/F_a, bytes/M_a) with separate achievable FLOP rates for prefill and decode
 * attention (Table 3); an iteration's latency is the sum over its operators plus a static overhead).
 * Pure HOST function.  One operator per sequence with q_len > 0 (S_q = q_len, S_kv = ctx_len + q_len;
 * F_ap when q_len > 1, F_ad when q_len == 1); O_p is added once if the batch holds prefill work, O_d
 * once if it holds decode work.  causal_flops != 0 counts only the visible (row, key) pairs,
 * 4*D_h*(S_q*ctx + S_q(S_q+1)/2), instead of Table 2's S_q*S_kv (same for decode operators).
 *   params: environment parameters, fitted from measurements of this library on the target GPU
 *           (FLOP/s, FLOP/s, bytes/s, seconds, seconds)
 *   h_query_start_loc [num_seqs+1], h_ctx_lens [num_seqs]: HOST, as for ooco_plan
 *   out: HOST double[8] = (latency s, prefill operators s, decode operators s, overhead s, FLOPs, bytes,
 *        time of compute-bound operators s, time of memory-bound operators s)
 *   msg: HOST buffer for the error text, may be NULL.
 * Errors: OOCO_EINVAL (NULL pointers, non-positive rates), OOCO_ESHAPE (geometry, negative lengths). */
typedef struct ooco_model_params {
    double F_ap, F_ad, M_a, O_p, O_d;
} ooco_model_params;
ooco_status ooco_predict_latency(const ooco_model_params *params /*HOST*/, int num_q_heads, int num_kv_heads,
                                 int head_dim, int bytes_per_value, int causal_flops, int num_seqs,
                                 const int32_t *h_query_start_loc /*HOST*/, const int32_t *h_ctx_lens /*HOST*/,
                                 double *out /*HOST*/, char *msg /*HOST*/, size_t msg_cap);

/* Mix Decoding Selection (paper Section 3.4.4, Algorithm 2): the requests of the next decode step.  All
 * online requests are kept; offline candidates join while the predicted step latency L(batch) (the
 * attention model above on a decode-only batch: one operator per request, S_q = 1, S_kv = its length,
 * plus O_d) stays within the TPOT bound slo_s: first num_looks candidates are looked at in the given
 * random order (each joins if the batch still fits, else is dropped for this step), then, if candidates
 * remain unlooked and L(batch) < slo_s, the remaining ones are sorted by ascending length (ties by
 * index) and the longest prefix that still fits joins, found by bisection.
 * Pure HOST function.
 *   h_online_lens [num_online], h_offline_lens [num_offline]: HOST int32 request lengths (KV tokens
 *     including the token of this step, >= 1)
 *   h_random_order [num_looks]: HOST int32 indices into the offline candidates, drawn by the caller
 *     (the algorithm's random choice is an input so that runs can be reproduced); an index that
 *     repeats or lies outside [0, num_offline) uses up its look and changes nothing
 *   h_selected [num_offline]: HOST bytes, written 1 for the candidates that join
 *   latency_out: HOST, predicted latency of the chosen batch in seconds (may be NULL)
 * If the online requests alone exceed slo_s they are all kept and no candidate joins. */
ooco_status ooco_mix_decoding_select(const ooco_model_params *params /*HOST*/, int num_q_heads, int num_kv_heads,
                                     int head_dim, int bytes_per_value, double slo_s, int num_online,
                                     const int32_t *h_online_lens /*HOST*/, int num_offline,
                                     const int32_t *h_offline_lens /*HOST*/, int num_looks,
                                     const int32_t *h_random_order /*HOST*/, uint8_t *h_selected /*HOST*/,
                                     double *latency_out /*HOST*/, char *msg /*HOST*/, size_t msg_cap);

/* Offline Request Migration Decision (paper Section 3.4.3, Algorithm 1), the latency-strict node's side:
 * the request length it prefers to pull from a latency-relaxed node.  L is the predictor of
 * ooco_mix_decoding_select; lengths on offer range over [len_min, len_max]; the cache holds
 * capacity_blocks blocks of block_size tokens and a request of length n occupies ceil(n / block_size).
 *   L(batch) >= slo_s, or all_included == 0 (the last mix decoding selection left a request of the
 *     node out): no migration, *pref_out = -1, *branch_out = 0;
 *   batch_size >= bs_sat (compute-saturated; fill the memory): the largest length whose request keeps
 *     L <= slo_s and fits the cache (branch 1; none fits: -1, branch 0);
 *   else, with n = bs_sat - batch_size requests missing to saturation: if n requests of len_min keep
 *     L <= slo_s, the largest length such that n requests of that length do (branch 2; the cache
 *     condition is stated for the saturated case only and applied only there), otherwise len_min,
 *     to make the batch as large as possible (branch 3).
 * Pure HOST function.  h_batch_lens [batch_size]: HOST int32, >= 1.  branch_out may be NULL.
 * Errors: OOCO_EINVAL (NULL pointers, sizes out of range), OOCO_ESHAPE (a length below 1). */
ooco_status ooco_migration_preference(const ooco_model_params *params /*HOST*/, int num_q_heads, int num_kv_heads,
                                      int head_dim, int bytes_per_value, double slo_s, int batch_size,
                                      const int32_t *h_batch_lens /*HOST*/, int all_included, int bs_sat,
                                      int block_size, int64_t capacity_blocks, int32_t len_min, int32_t len_max,
                                      int32_t *pref_out /*HOST*/, int32_t *branch_out /*HOST*/, char *msg /*HOST*/,
                                      size_t msg_cap);

/* The latency-relaxed node's side of the same algorithm: which of its ongoing offline requests
 * (h_relaxed_lens [num_relaxed]) go to the strict node whose batch is h_batch_lens.  They are visited
 * by ascending distance of their length from pref (ties: shorter first, then lower index); a request
 * goes if the strict node's batch with it keeps L <= slo_s and fits its cache, otherwise it is passed
 * over; at most max_migrate go.  h_chosen: HOST int32 [min(max_migrate, num_relaxed)], the indices in
 * the order taken; *num_chosen their number.  Pure HOST function. */
ooco_status ooco_migration_select(const ooco_model_params *params /*HOST*/, int num_q_heads, int num_kv_heads,
                                  int head_dim, int bytes_per_value, double slo_s, int batch_size,
                                  const int32_t *h_batch_lens /*HOST*/, int num_relaxed,
                                  const int32_t *h_relaxed_lens /*HOST*/, int32_t pref, int block_size,
                                  int64_t capacity_blocks, int max_migrate, int32_t *h_chosen /*HOST*/,
                                  int32_t *num_chosen /*HOST*/, char *msg /*HOST*/, size_t msg_cap);

/* Which offline requests a latency-strict node evicts to free need_blocks KV blocks for an online
 * request arriving from its prefill (paper Section 3.4.1): when the node is compute-bound
 * (batch_size >= bs_sat) long requests go first, so that the decode batch stays large; otherwise
 * short ones go first, which keeps the recomputation small.  Requests are taken in that order (ties
 * by index) until their blocks cover the need; then, in the order taken, a request whose blocks the
 * others make unnecessary stays after all.  The blocks of the victims are what a caller hands to
 * ooco_kv_block_copy.
 *   h_victims: HOST int32 [num_offline], indices in the order taken; *num_victims their number;
 *   *enough (may be NULL): 0 when all requests together do not cover the need (then all are listed).
 * Pure HOST function. */
ooco_status ooco_eviction_victims(int num_offline, const int32_t *h_offline_lens /*HOST*/, int64_t need_blocks,
                                  int block_size, int batch_size, int bs_sat, int32_t *h_victims /*HOST*/,
                                  int32_t *num_victims /*HOST*/, int32_t *enough /*HOST*/, char *msg /*HOST*/,
                                  size_t msg_cap);

#ifdef __cplusplus
}
#endif
#endif /* OOCO_H */
