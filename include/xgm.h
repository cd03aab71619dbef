/*
 * xgm: grammar-constrained decoding masks on AMD CDNA4 (gfx950).
 *
 * C ABI of the data-parallel hot path of the structured-generation method of
 * arxiv 2411.15100 ("XGrammar"): a context-free grammar is compiled on the
 * host into a byte-level pushdown automaton (one finite automaton per rule,
 * character edges and rule-reference edges; section 2.2 and Appendix A); once
 * per (grammar, vocabulary) a GPU kernel classifies every vocabulary token at
 * every automaton node as accepted / rejected / context-dependent (the token
 * mask cache of section 3.1); per decoding step a GPU kernel produces each
 * request's next-token bitmask from the cached bitsets and the request's live
 * stacks (section 3.1, Algorithm 1: union over parallel stacks), and another
 * writes -inf into the logits of disallowed tokens (section 2.1).
 *
 * Conventions
 *  - Every function returns 0 (XGM_OK) or a negative xgm_status; a message is
 *    kept per thread and read with xgm_last_error().  No C++ exception leaves
 *    the library.
 *  - Handles are opaque.  Every *_create / *_compile / *_build has a
 *    *_destroy.  A cache keeps its grammar and vocabulary alive by reference
 *    count; a matcher keeps its cache alive.  Immutable handles (vocab,
 *    grammar, cache) may be shared between threads; a matcher may not.
 *  - Pointers named h_* are host memory, d_* are device memory on the current
 *    HIP device.  The caller owns every buffer it passes; the library never
 *    frees or reallocates them.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default
 *    stream).  Calls documented as asynchronous enqueue work on that stream
 *    and return without waiting for it.
 *  - Bitmask layout: row-major int32 [rows, xgm_bitmask_words(V)]; token i is
 *    bit (i & 31) of word (i >> 5), least significant bit first; 1 = allowed;
 *    bits at positions >= V are 0.
 *  - The library needs a gfx950 device for everything except vocabulary and
 *    grammar handling and the matcher's host state; there is no CPU path for
 *    the three kernels.
 */
#ifndef XGM_H
#define XGM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct xgm_vocab xgm_vocab;
typedef struct xgm_grammar xgm_grammar;
typedef struct xgm_cache xgm_cache;
typedef struct xgm_matcher xgm_matcher;
typedef struct xgm_batch xgm_batch;

typedef enum {
  XGM_OK = 0,
  XGM_ERR_BAD_ARG = -1,          /* null pointer, bad size, bad dtype, misaligned buffer */
  XGM_ERR_PARSE = -2,            /* grammar text is malformed */
  XGM_ERR_UNDEFINED_RULE = -3,   /* a referenced rule (or the root) is not defined */
  XGM_ERR_LEFT_RECURSION = -4,   /* a rule can re-enter itself without consuming a byte */
  XGM_ERR_UNPRODUCTIVE = -5,     /* the root rule derives no string */
  XGM_ERR_TOKEN_REJECTED = -6,   /* accept_token: token not allowed; state unchanged */
  XGM_ERR_TERMINATED = -7,       /* accept_token after the stop token */
  XGM_ERR_TOO_MANY_STACKS = -8,  /* more parallel stacks than XGM_MAX_STACKS; state unchanged */
  XGM_ERR_TOO_LARGE = -9,        /* automaton, stack depth or vocabulary beyond a documented limit */
  XGM_ERR_HIP = -10,             /* a HIP runtime call failed, or no device */
  XGM_ERR_INTERNAL = -11
} xgm_status;

typedef enum { XGM_F32 = 0, XGM_BF16 = 1, XGM_F16 = 2 } xgm_dtype;

enum {
  XGM_MAX_STACKS = 64,       /* parallel stacks per matcher */
  XGM_MAX_STACK_DEPTH = 4096,/* frames per stack */
  XGM_MAX_NODES = 32767,     /* automaton nodes per grammar */
  XGM_MAX_VOCAB = 589824,    /* tokens per vocabulary (two bitset rows of a node must fit the LDS of one workgroup) */
  XGM_BATCH_MAX_HISTORY = 63,/* older states a row of an xgm_batch can keep */
  XGM_BATCH_MAX_STACKS = 16, /* parallel stacks per row of an xgm_batch */
  XGM_BATCH_MAX_DEPTH = 128, /* frames per stack in an xgm_batch */
  XGM_BATCH_MAX_ROWS = 1024  /* rows of an xgm_batch */
};

const char* xgm_last_error(void);

/* ceil(V / 32) */
int32_t xgm_bitmask_words(int32_t V);

/* ---------------------------------------------------------------- vocabulary
 * Token i is h_bytes[h_offsets[i] .. h_offsets[i+1]) (host memory, copied).
 * stop_ids are the end-of-generation tokens (section 3 is silent on them; the
 * reading here: a stop token is allowed exactly when the text generated so
 * far is a complete sentence of the grammar).  A token with zero bytes that
 * is not a stop token is never allowed.  The library keeps, on the host and
 * on the device, the tokens sorted by their bytes (section 3.3: neighbours in
 * sorted order share prefixes) next to the id order.
 * Device copies are made lazily by the first xgm_cache_build. */
int xgm_vocab_create(const uint8_t* h_bytes, const int64_t* h_offsets, int32_t V,
                     const int32_t* h_stop_ids, int32_t n_stop, xgm_vocab** out);
void xgm_vocab_destroy(xgm_vocab* v);
int32_t xgm_vocab_size(const xgm_vocab* v);

/* ------------------------------------------------------------------- grammar
 * 1. Compile a grammar (host only).  text is UTF-8 EBNF: `name ::= alt`,
 * alternatives `|`, items "literal" (escapes \" \\ \' \/ \n \t \r \b \f \xHH
 * \uHHHH), classes [a-z] / [^...] over Unicode scalar values, rule names,
 * groups ( ), postfix * + ?, `#` comments.  The result is the automaton of
 * section 2.2 / Appendix A in flattened form: every reachable rule is a
 * minimal deterministic automaton over bytes and rule references; references
 * to rules that can match "" may be skipped, and a rule instance always
 * consumes at least one byte, so that no epsilon cycle exists.
 * Errors: PARSE, UNDEFINED_RULE, LEFT_RECURSION, UNPRODUCTIVE, TOO_LARGE. */
int xgm_grammar_compile(const char* text, size_t len, const char* root_rule, xgm_grammar** out);
void xgm_grammar_destroy(xgm_grammar* g);
int32_t xgm_grammar_num_nodes(const xgm_grammar* g);
int32_t xgm_grammar_num_rules(const xgm_grammar* g);
/* Name of rule r (0 <= r < num_rules), valid while g lives; NULL if out of range. */
const char* xgm_grammar_rule_name(const xgm_grammar* g, int32_t r);
/* Rule index that node n belongs to, or a negative status. */
int32_t xgm_grammar_node_rule(const xgm_grammar* g, int32_t node);
/* A shortest path of symbols leading from the start of the node's rule to the
 * node: values 0..255 are bytes, 256 + r is a reference to rule r.  Writes at
 * most cap symbols to h_out and returns the path length (or a negative
 * status).  This names a node independently of the library's numbering. */
int32_t xgm_grammar_node_path(const xgm_grammar* g, int32_t node, int32_t* h_out, int32_t cap);
/* 1 if the node is accepting in its rule (the rule may end here), else 0. */
int32_t xgm_grammar_node_is_final(const xgm_grammar* g, int32_t node);

/* JSON-schema front end (host only; the schema tasks of section 4.1): writes
 * the grammar text for a JSON schema (UTF-8, len bytes) into h_text (cap
 * bytes, NUL-terminated) and its length without the NUL into *h_len; with
 * cap == 0 only the length is returned.  The root rule is `root`; compile the
 * text with xgm_grammar_compile.  Supported: "type" (a name or a list of names:
 * object, array, string, integer, number, boolean, null); "properties" with
 * "required" - the members of an object appear in the order of "properties",
 * those not listed in "required" may be left out (without "required" all are
 * required), no other members are allowed; "items" with "minItems" /
 * "maxItems" (at most 64); "enum" and "const" of strings, numbers, booleans
 * and null; "anyOf" / "oneOf" (both as a union); `true` and `{}` (any JSON
 * value); annotations are ignored.  Member names and the strings of "enum" /
 * "const" are matched in their shortest JSON spelling (only `"`, `\` and
 * control characters escaped); white space is allowed where JSON allows it.
 * Keywords that would change the language and are not listed here ("pattern",
 * "format", numeric ranges, "$ref", "allOf", "not", "additionalProperties"
 * other than false, ...) are refused: XGM_ERR_PARSE with a message, as for
 * malformed JSON.  XGM_ERR_BAD_ARG if cap is too small (*h_len is still set). */
int xgm_schema_to_grammar(const char* schema_json, size_t len, char* h_text, size_t cap, size_t* h_len);

/* --------------------------------------------------------------------- cache
 * 2. Once per (grammar, vocabulary): build the token mask cache of section
 * 3.1 on the GPU.  For every node n and token t, starting with n alone on the
 * stack: accepted if some path consumes all bytes of t without leaving n's
 * frame downwards; else context-dependent ("uncertain") if some path reaches
 * the end of n's rule while at least one byte remains; else rejected.
 * The context-dependent class is then narrowed with one byte of context, a
 * small form of the context expansion of section 3.2: an exit from n's rule
 * R only counts if the byte that comes next can follow an instance of R in
 * some context (the FOLLOW set of R: what can be consumed at the return node
 * of any reference to R, and, where the referencing rule may end there, what
 * can follow that rule).  A token all of whose exits fail this test is
 * rejected in every context, so it is stored as rejected ("plain-only"
 * context-dependent tokens are counted, and kept with XGM_CACHE_KEEP_PLAIN);
 * final masks are unchanged.
 * The result is kept on the device in the cheapest exact form per node (the
 * adaptive storage of section 3.1, and section 3.2 taken per call site):
 *  - the accepted tokens as a bitset row (every distinct row once) if there
 *    are many, as a list of token ids if there are few;
 *  - the context-dependent tokens resolved ahead of time against what can
 *    lie below: a frame of rule R can only sit on one of the nodes that follow
 *    a reference to R (its contexts).  For every node n with such tokens and
 *    every context r of n's rule there is a list of the tokens whose rest,
 *    after leaving n's frame, is consumed from r without leaving r's frame;
 *    for the tokens that leave r's frame as well, one more list per context
 *    of r's rule, and once more below that (three frames deep).  Tokens that
 *    leave a fourth frame, and tokens whose walk at build time exceeded a
 *    limit, are listed as entries to be walked against the live stack at
 *    fill time.  Lists are cut at every 8192 token ids.
 * The fill call therefore ORs one bitset or list per stack, sets the bits of
 * three short lists, and walks only the rare remainder.
 * Synchronous: returns after the build has finished on hip_stream. */
int xgm_cache_build(xgm_grammar* g, xgm_vocab* v, void* hip_stream, xgm_cache** out);
enum { XGM_CACHE_KEEP_PLAIN = 1, XGM_CACHE_DEPTH_SHIFT = 4, XGM_CACHE_DEPTH_MASK = 0x70 };
/* Same, with flags: XGM_CACHE_KEEP_PLAIN also keeps, per node, the bitsets of
 * the context-dependent tokens and of the plain-only context-dependent tokens
 * (for xgm_cache_copy_node_bits' h_unc and xgm_cache_copy_node_plain).
 * XGM_CACHE_DEPTH(d), d = 1 .. 3: resolve the context-dependent tokens at most d
 * frames deep at build time instead of three (0: the default).  A shallower cache is
 * built faster and is smaller (grammars whose rules are used in many places have long
 * lists at the deeper levels); the tokens that leave more frames than that are walked
 * against the live stack by every fill.  The masks are the same. */
#define XGM_CACHE_DEPTH(d) ((uint32_t)(d) << XGM_CACHE_DEPTH_SHIFT)
int xgm_cache_build_ex(xgm_grammar* g, xgm_vocab* v, void* hip_stream, uint32_t flags, xgm_cache** out);
void xgm_cache_destroy(xgm_cache* c);
int32_t xgm_cache_num_nodes(const xgm_cache* c);
/* Copies node's accepted and context-dependent bitsets (bitmask layout, each
 * xgm_bitmask_words(V) words) to host buffers; either pointer may be NULL.
 * h_unc needs XGM_CACHE_KEEP_PLAIN at build time (XGM_ERR_BAD_ARG otherwise). */
int xgm_cache_copy_node_bits(const xgm_cache* c, int32_t node, int32_t* h_acc, int32_t* h_unc);
/* Number of context-dependent tokens cached for a node (or a negative status). */
int32_t xgm_cache_num_uncertain(const xgm_cache* c, int32_t node);
/* Number of tokens that section 3.1 alone calls context-dependent at the node
 * but that the one-byte context refinement rejects (so: num_uncertain +
 * num_uncertain_plain = size of the class of section 3.1). */
int32_t xgm_cache_num_uncertain_plain(const xgm_cache* c, int32_t node);
/* The bitset of those tokens (needs XGM_CACHE_KEEP_PLAIN at build time). */
int xgm_cache_copy_node_plain(const xgm_cache* c, int32_t node, int32_t* h_plain);
/* Number of (node, token) pairs of the build whose walk exceeded the on-chip
 * bounds and were classified exactly on the host instead (0 for every
 * workload shipped with this repository). */
int64_t xgm_cache_host_classified(const xgm_cache* c);
/* Seconds the GPU spent in the classification kernel during the build, and
 * the number of (node, token) pairs it classified. */
double xgm_cache_build_kernel_seconds(const xgm_cache* c);
/* Seconds the whole xgm_cache_build call took on the host clock (all kernels,
 * the copies of sizes back to the host, allocation; the vocabulary upload only
 * on the first build that uses it). */
double xgm_cache_build_seconds(const xgm_cache* c);
/* The part of those seconds that the classification of section 3.1 took: from the start of the call until
 * every node's accepted and context-dependent tokens lie in id-space bitsets on the device and their
 * per-node statistics on the host (first-byte bitsets, classification kernel, rank -> id permutation with
 * the row statistics, one synchronisation).  The rest of the call resolves the context-dependent tokens
 * per call site (section 3.2) and lays out the lists. */
double xgm_cache_build_classify_seconds(const xgm_cache* c);
/* Test knob: the following builds classify their nodes in batches of `nodes` (rounded down to a multiple of
 * 32, at least 32) instead of all at once; 0 restores the default (as many nodes as 1 GiB of rank-space rows
 * holds: every grammar of this repository in one batch).  The caches built are the same. */
void xgm_debug_set_build_batch_nodes(int32_t nodes);
/* Section 3.1 (storage of the cache): number of distinct accepted bitsets kept (nodes with few accepted
 * tokens keep a list instead and are not counted), and the bytes of device memory the cache holds
 * (bitsets, lists, offsets, table image).  Negative: error. */
int32_t xgm_cache_num_accept_rows(const xgm_cache* c);
int64_t xgm_cache_device_bytes(const xgm_cache* c);
/* Sizes of the cache, into h_out8 (host, 8 values): [0] list keys in all, [1] keys of the first kind
 * (node, context), [2] of the deeper kinds (node, context, context of that context's rule, ...), [3] list entries
 * in all, [4] of them accepted tokens of nodes that keep a list, [5] context-dependent (node, token) pairs
 * the lists were made from, [6] (pair, context) combinations examined at build time, [7] bitset rows. */
int xgm_cache_stats(const xgm_cache* c, int64_t* h_out8);

/* The exact host routine that decides a (node, token) pair whose GPU walk
 * exceeded its limits during xgm_cache_build: 0 rejected, 1 context-dependent,
 * 2 accepted, negative status on error.  Exported so that this slow path can
 * be tested without a device; nothing on the hot path calls it.  4 = context-
 * dependent by section 3.1 alone, rejected by the one-byte context refinement. */
int xgm_debug_classify_host(const xgm_grammar* g, int32_t node, const uint8_t* h_bytes, int32_t n);
/* The token walk of the two GPU kernels, compiled for the host from the same
 * source and run on the flattened tables, for tests without a device.
 * h_stack: depth nodes, bottom first.  build != 0: depth must be 1, result is
 * 0 rejected / 1 context-dependent / 2 accepted / 4 plain-only context-
 * dependent, as in xgm_cache_build;
 * build == 0: result is 2 (token allowed from this stack) or 0.  3 = the walk
 * exceeded its limits (64 frames, 24 alternatives, 4096 steps, 255 bytes).
 * h_steps (may be NULL) receives the number of automaton steps taken. */
int xgm_debug_walk_host(const xgm_grammar* g, const int32_t* h_stack, int32_t depth,
                        const uint8_t* h_bytes, int32_t n, int32_t build, int32_t* h_steps);
/* A frame whose current node is `top` can only sit on one of the nodes that
 * follow a reference to top's rule (directly, or through references in tail
 * position): the contexts of the rule.  Returns the index of `below` among them
 * (what names the stack's token lists in the mask cache), or -1000 if `below`
 * is not one of them (never the case for a stack the matcher produced). */
int32_t xgm_debug_context_index(const xgm_grammar* g, int32_t top, int32_t below);
/* ------------------------------------------------------------------- matcher
 * Per-request state: the set of parallel stacks of section 2.2, each a list of
 * automaton nodes (return nodes below, current node on top).  Host memory. */
int xgm_matcher_create(xgm_cache* c, xgm_matcher** out);
/* A matcher without a cache (host only; v may be NULL if only accept_bytes is
 * used): every call below works except xgm_fill_next_token_bitmask. */
int xgm_matcher_create_host(xgm_grammar* g, xgm_vocab* v, xgm_matcher** out);
void xgm_matcher_destroy(xgm_matcher* m);
int xgm_matcher_reset(xgm_matcher* m);
/* 3. Accept a token: advance every stack over the token's bytes and keep all
 * survivors (section 3: the sampled token updates the stack state).  A stop
 * token terminates the matcher if the text is complete.  Errors:
 * TOKEN_REJECTED / TOO_MANY_STACKS / TOO_LARGE (state unchanged), TERMINATED,
 * BAD_ARG. */
int xgm_matcher_accept_token(xgm_matcher* m, int32_t token_id);
/* Feed raw bytes instead of a token (same semantics and errors). */
int xgm_matcher_accept_bytes(xgm_matcher* m, const uint8_t* h_bytes, int32_t n);
int32_t xgm_matcher_is_terminated(const xgm_matcher* m);
/* 1 if the text accepted so far is a complete sentence. */
int32_t xgm_matcher_can_terminate(const xgm_matcher* m);
int32_t xgm_matcher_num_stacks(const xgm_matcher* m);
/* Depth of stack s and (optionally) its nodes, bottom first, top last. */
int32_t xgm_matcher_stack(const xgm_matcher* m, int32_t s, int32_t* h_nodes, int32_t cap);

/* ---------------------------------------------------------------------- fill
 * 4. Fill the next-token bitmask for a batch (asynchronous).  Row b of
 * d_bitmask ([B, xgm_bitmask_words(V)], device) becomes
 *     OR over the stacks s of ms[b] of
 *        accepted[top(s)]  |  { t context-dependent at top(s) : walking t's
 *                               bytes from s with the full stack survives }
 * plus the stop tokens iff the matcher can terminate; a terminated matcher
 * gets a row with only the stop tokens.  All matchers must share one
 * vocabulary; their grammars may differ.  B <= 65535.  The call packs the
 * stacks (per stack: its frames and which token lists of the cache are its)
 * into pinned staging owned by the library (a ring of 8 slots), enqueues a
 * small kernel that copies them and looks up where those lists lie, and the
 * fill kernel (one workgroup per row and 8192
 * token ids) on hip_stream, and returns.
 * A walk that exceeds the on-chip bounds (64 frames pushed inside one token,
 * 24 pending alternatives, 4096 steps, tokens longer than 255 bytes) is never
 * guessed: the pair is recorded on the device, its bit is left 0, and
 * xgm_fill_overflow_fixup() decides it exactly. */
int xgm_fill_next_token_bitmask(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask,
                                void* hip_stream);
/* 4 + 5 in one launch (asynchronous): fills d_bitmask exactly as
 * xgm_fill_next_token_bitmask does and applies row b of the result to logits
 * row b as xgm_apply_token_bitmask_inplace does (section 2.1): d_logits is
 * [B, V_logits] of dt (device), V_logits >= the vocabulary size (wider columns
 * are masked), row stride row_stride_elems; the base address and the row pitch
 * must be multiples of 16 bytes (XGM_ERR_BAD_ARG otherwise: use the two
 * calls).  A token whose walk exceeded the on-chip limits is left allowed
 * (bit set, logit untouched) by this call; if the counter behind
 * xgm_fill_overflow_count_device() moved, xgm_fill_overflow_fixup() makes the
 * bitmask exact and the caller applies it once more with
 * xgm_apply_token_bitmask_inplace. */
int xgm_fill_and_apply(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* d_logits, xgm_dtype dt,
                       int32_t V_logits, int64_t row_stride_elems, void* hip_stream);
/* For callers that cannot allocate device memory where they call from (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): xgm_fill_next_token_bitmask with its per-call staging in fixed
 * memory.  Same arguments, same result in d_bitmask, same handling of walks
 * over the on-chip limits.  The packed stacks are
 * written into a fixed host array and copied, in stream order, into a fixed
 * array of XGM_STATIC_STAGING_BYTES (1 MiB) that every device holds from the
 * moment the library is loaded until the process ends, where a kernel writes
 * them out in the form the fill kernel reads (both forms lie in the array);
 * the call makes no hipMalloc / hipHostMalloc / hipFree and uses no event.  A
 * batch whose stacks need more than that returns XGM_ERR_TOO_LARGE (nothing is
 * enqueued); batch 128 at a vocabulary of 151936 needs about 110 KiB.  The
 * mask caches of the matchers must have been built before (they were, or the
 * matchers would not exist).  All calls on one device share the array, which
 * keeps the last call's contents: calls whose work overlaps on one device
 * (different streams, or several host threads) race and must be ordered by
 * the caller; calls on one stream are ordered by the stream. */
#define XGM_STATIC_STAGING_BYTES (1 << 20)
int xgm_fill_next_token_bitmask_static(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask,
                                       void* hip_stream);
/* What a fill has to read for this matcher's state, into h_out4 (host, 4
 * values): [0] stacks whose top node keeps its accepted tokens as a bitset row,
 * [1] entries of the stacks' lists of accepted tokens (top nodes that keep a
 * list), [2] of their (node, context) lists, [3] of their deeper per-context
 * lists.  For the byte counts of benchmarks; needs a mask cache. */
int xgm_debug_matcher_fill_work(const xgm_matcher* m, int64_t* h_out4);
/* Instrumentation for benchmarks: the same fill (same result in d_bitmask)
 * with a kernel instantiation that also counts the automaton steps of all
 * walks; synchronous; *h_steps receives the count.  Not for the hot path. */
int xgm_debug_fill_count_steps(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask,
                               void* hip_stream, int64_t* h_steps);
/* Instrumentation for the benchmark: the same fill, with HIP events recorded on
 * hip_stream around its two kernels; waits for them.  h_us2[0] = microseconds
 * of the stack upload kernel, h_us2[1] = of the fill kernel (host array of 2). */
int xgm_debug_fill_timed(xgm_matcher* const* ms, int32_t B, int32_t* d_bitmask, void* hip_stream, float* h_us2);
/* Walks over the on-chip limits, fills from host-side matchers.  Every such
 * fill (either entry point above, the fused one, the static one) records its
 * pairs in one log that these fills share; each record names its fill, and the
 * library keeps what it needs to decide the records of the last 8 fills (their
 * packed stacks, where their masks went, their caches).
 * xgm_fill_overflow_fixup synchronises hip_stream, decides on the host every
 * pair recorded since the previous fixup, whichever of those fills recorded
 * it, and writes the exact bits into that fill's d_bitmask.  Returns the
 * number of pairs decided (>= 0).  Records of fills older than the last 8 can
 * no longer be decided: the call then decides the others and returns
 * XGM_ERR_TOO_LARGE with the counts in the message - never silently.
 * Callers that never see the counter below move may skip the call. */
int xgm_fill_overflow_fixup(void* hip_stream);
/* Device address of the counter of those records (uint32, only ever grows;
 * valid until the process ends): a caller can read it in a kernel of its own
 * or copy it on its stream, without synchronising the device.  NULL if there
 * is no device. */
const uint32_t* xgm_fill_overflow_count_device(void);
/* Total number of pairs recorded so far by all cache builds and fills, of
 * host-side and of device-resident states (synchronises the device to read
 * the counters; for tests and reports). */
int64_t xgm_overflow_total(void);

/* ------------------------------------------- states that live on the device
 * 4b. The matcher states of a fixed batch of requests kept in device memory
 * (section 3.3: the persistent stack and its rollback, here as a ring of
 * states per row in HBM).  The sampled token ids never leave the device: a
 * kernel moves every row's stacks on by its token and writes the row's next
 * state in the layout the fill kernel reads (frames, and where each stack's
 * token lists lie in the mask cache); a fill is then a single launch without
 * any host packing or upload.  Going back k tokens (speculative decoding,
 * section 3.3) re-points a row k states back.  Calls on one batch must be
 * ordered by the caller (one stream, or events).
 *
 * xgm_batch_create: row b starts in the current state of ms[b] (host
 * matchers with mask caches over one vocabulary; they are not referenced
 * afterwards, their caches are).  history: how many older states each row
 * keeps (0 .. XGM_BATCH_MAX_HISTORY).  Device limits per row:
 * XGM_BATCH_MAX_STACKS parallel stacks of XGM_BATCH_MAX_DEPTH frames
 * (XGM_ERR_TOO_MANY_STACKS / XGM_ERR_TOO_LARGE at creation; at run time such
 * a row reports the code in its status and keeps its state, see
 * xgm_batch_get_row / xgm_batch_set_row for the way through the host).
 * B <= XGM_BATCH_MAX_ROWS.  Synchronises hip_stream. */
int xgm_batch_create(xgm_matcher* const* ms, int32_t B, int32_t history, void* hip_stream, xgm_batch** out);
void xgm_batch_destroy(xgm_batch* bt);
int32_t xgm_batch_size(const xgm_batch* bt);
/* Asynchronous.  d_token_ids: [B] device int32; row b accepts token
 * d_token_ids[b] exactly as xgm_matcher_accept_token would (same resulting
 * stacks, in the same order); a negative id leaves the row and its status
 * alone.  Per-row result in the status array: XGM_OK, XGM_ERR_TOKEN_REJECTED,
 * XGM_ERR_TERMINATED, XGM_ERR_BAD_ARG (id >= V), XGM_ERR_TOO_MANY_STACKS or
 * XGM_ERR_TOO_LARGE (device limits, or the walk's limits: 64 frames pushed
 * inside one token, 24 pending alternatives, 4096 steps, 32 end
 * configurations); on any error the row keeps its state.  One kernel launch. */
int xgm_batch_accept_tokens(xgm_batch* bt, const int32_t* d_token_ids, void* hip_stream);
/* Asynchronous.  d_steps: [B] device int32; row b goes back d_steps[b] accepted
 * tokens (<= 0: stays).  More than the row still holds: XGM_ERR_BAD_ARG in its
 * status, state unchanged. */
int xgm_batch_rollback(xgm_batch* bt, const int32_t* d_steps, void* hip_stream);
/* Asynchronous.  d_src_rows: [B] device int32; row b continues from the current
 * state of row d_src_rows[b] (section 3.3: one prefix continued in several
 * ways, as in tree decoding); negative or b itself: the row stays.  All rows
 * take the states as they were before the call.  The new state counts as one
 * accepted token for rollback.  Both rows must use the same mask cache
 * (XGM_ERR_BAD_ARG in the row's status otherwise, also for a row index
 * >= B); the batch must have been created with history >= 1 (XGM_ERR_BAD_ARG
 * from the call otherwise). */
int xgm_batch_fork(xgm_batch* bt, const int32_t* d_src_rows, void* hip_stream);
/* Synchronises hip_stream and copies the per-row status of the last accept /
 * rollback / fork into h_status[B] (host).  Returns the number of rows whose status
 * is not XGM_OK, or a negative status of the call itself. */
int xgm_batch_status(xgm_batch* bt, int32_t* h_status, void* hip_stream);
/* The way through the host for a row that hit a device limit (both
 * synchronise hip_stream): get_row copies the row's current state into the
 * host matcher m (which must belong to the row's mask cache); set_row makes
 * m's state the row's next state (it counts as one accepted token for
 * rollback). */
int xgm_batch_get_row(xgm_batch* bt, int32_t row, xgm_matcher* m, void* hip_stream);
int xgm_batch_set_row(xgm_batch* bt, int32_t row, const xgm_matcher* m, void* hip_stream);
/* As xgm_fill_next_token_bitmask / xgm_fill_and_apply for the batch's current
 * states: one kernel launch, nothing packed or uploaded.  Walks that exceed
 * the on-chip limits are recorded in a log of the batch's own (each record
 * names its fill and the state of its row) and decided by
 * xgm_batch_fill_overflow_fixup(). */
int xgm_batch_fill_next_token_bitmask(xgm_batch* bt, int32_t* d_bitmask, void* hip_stream);
int xgm_batch_fill_and_apply(xgm_batch* bt, int32_t* d_bitmask, void* d_logits, xgm_dtype dt, int32_t V_logits,
                             int64_t row_stride_elems, void* hip_stream);
/* Synchronises hip_stream, then decides on the host every pair that fills of
 * this batch have recorded since the batch's previous fixup and writes the
 * exact bits into the d_bitmask of the fill that recorded it (the last 8
 * fills of the batch are remembered).  A record can only be decided while its
 * row is still in the state that the fill saw: call this before the next
 * accept / rollback / fork / set_row of such a row.  Returns the number of
 * pairs decided (>= 0); if some records could not be decided (their row has
 * moved on, or their fill is more than 8 fills back) the others are decided
 * and XGM_ERR_TOO_LARGE is returned with the counts in the message.  Other
 * batches' and the host-state fills' records are never touched. */
int xgm_batch_fill_overflow_fixup(xgm_batch* bt, void* hip_stream);
/* Device address of the batch's record counter (uint32, only ever grows; valid
 * until xgm_batch_destroy): poll it without synchronising the device. */
const uint32_t* xgm_batch_overflow_count_device(const xgm_batch* bt);
/* Measurement aid for the benchmark (synchronous): dependent 4-byte LDS reads
 * per second of the whole device with two 1024-lane workgroups per compute
 * unit, every lane following a chain through a 32 KB table.  The table
 * lookups of the token walks (section 3.1, 3.3) are reads of this kind, each
 * depending on the one before. */
int xgm_debug_lds_lookup_rate(void* hip_stream, double* h_lookups_per_second);
/* For tests without a device: accept a token with the routine the device uses
 * (a depth-first walk over the flattened tables that writes out every stack
 * the token can end in) instead of the host engine.  Same results and errors
 * as xgm_matcher_accept_token, plus XGM_ERR_TOO_LARGE when the walk's limits
 * are hit. */
int xgm_debug_matcher_accept_token_walk(xgm_matcher* m, int32_t token_id);

/* --------------------------------------------------------------------- apply
 * 5. Apply a bitmask to logits in place (asynchronous; section 2.1).
 * d_logits: [B, V_logits] of dt with row stride row_stride_elems (elements).
 * d_bitmask: [n_rows, xgm_bitmask_words(V_mask)].  If d_row_index is NULL,
 * n_rows must equal B and bitmask row j masks logits row j; otherwise bitmask
 * row j masks logits row d_row_index[j] (device int32, values in [0, B), no
 * duplicates).  For every masked row: logits[i] becomes -inf where bit i is 0
 * or i >= V_mask; every other element keeps its exact bit pattern. */
int xgm_apply_token_bitmask_inplace(void* d_logits, xgm_dtype dt, int32_t B, int32_t V_logits,
                                    int64_t row_stride_elems, const int32_t* d_bitmask,
                                    int32_t V_mask, const int32_t* d_row_index, int32_t n_rows,
                                    void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* XGM_H */
