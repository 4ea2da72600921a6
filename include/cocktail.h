/*
 * cocktail.h - C ABI of the chunk-level KV cache computation of Cocktail
 * (arXiv 2503.23294, Sec. III-C, Algorithm 1) for AMD MI355X (gfx950).
 *
 * The library covers the data-parallel hot path of the paper's second module.
 * Given the bitwidth (FP16 / INT8 / INT4 / INT2) that the chunk-level quantization
 * search (Sec. III-B) chose for every context chunk, it
 *   1. reorders the KV chunks so that every bitwidth class is contiguous in
 *      memory (Alg. 1, prefill loop; Fig. 3),
 *   2. quantizes and packs the INT2, INT4 and INT8 classes (Alg. 1, `quant`),
 *   3. runs single-query decode attention over the classes: logits of the
 *      INT2, INT4 (INT8) and FP16 blocks, one softmax over their concatenation, the
 *      att x V products of the blocks summed (Alg. 1, decode phase).  The concatenation is
 *      never materialised: each worker keeps a partial softmax state
 *      (max, sum, weighted V sum) and the states are merged exactly, which
 *      gives the same result because the softmax-weighted sum does not depend
 *      on the order or grouping of the tokens (Sec. III-C, Eq. 4-5).
 *
 * Conventions
 *   - Every pointer is marked HOST or DEVICE.  The library never allocates,
 *     frees or copies device memory and never synchronises the device (the one
 *     exception, cocktail_decode_check, says so); the GPU entry points only
 *     enqueue kernels on the caller's stream.
 *   - All functions return a cocktail_status; on failure a message is kept in
 *     thread-local storage (cocktail_last_error).  Arguments are validated on
 *     the host before anything is launched.
 *   - class index 0 = INT2, 1 = INT4, 2 = INT8, 3 = FP16: the concatenation order of Alg. 1 (INT2, INT4,
 *     FP16) with INT8, which Sec. I names as a further bitwidth, in its place by precision.
 *
 * Packed cache layout (an encoding defined by this library; the paper does not
 * fix one).  For each class c the K data and the V data live in one device
 * buffer each.  A buffer is a sequence of 64-token blocks ordered by
 * (sequence b, kv head h, block j); sequence b owns ceil(n_{b,c}/64) blocks per
 * head, n_{b,c} being its token count in class c (the FP16 runs of a plan made with
 * cocktail_plan_options::max_seq_lens own more: room for the tokens that may be folded in later, zero blocks
 * until then).  Inside a block:
 *   codes   the row of token i (i = 0..63) is cut into 16-byte pieces; piece p
 *           of token i is at byte (p*64 + i)*16.  Row size: D*bits/8 bytes for
 *           INT2/INT4/INT8, 2*D bytes (raw fp16, channel order) for FP16.
 *           A quantized row is a sequence of little-endian 32-bit words; word k
 *           covers the n = 32/bits channels k*n .. k*n+n-1, channel k*n+2f in
 *           bits [f*bits, f*bits+bits) and channel k*n+2f+1 in bits
 *           [16+f*bits, 16+f*bits+bits).
 *   meta    (quantized classes only) after the codes, at byte 64*rowbytes: for token i
 *           and group g of G consecutive channels, 4 bytes at (i*(D/G)+g)*4 =
 *           fp16 scale, then fp16 zero.  Value of a code: zero + code*scale.
 *   Tokens past n_{b,c} in the last block of a head are zero bytes.
 *   (At head_dim 64 a row is half as long, everything else is the same; group_size is then 32 or 64.)
 *   V in token quads (cocktail_sizes::v_layout == COCKTAIL_V_TOKEN_QUADS; chosen
 *   wherever the matrix kernel runs (Hq/Hkv >= 2 unless the plan is vector-ALU-only or Hq/Hkv > 8 is prime), where a wave serves four query heads of a kv head
 *   with matrix instructions and needs four tokens of a channel side by side):
 *   same block size, piece addressing and meta as above, but the 16-byte piece at
 *   slot sl no longer holds one token.  With n = 16/bits values per half-word,
 *   token i of the block and channel c are found at
 *     h = c / 64, j = (c % 32) / 8, e = 8 * ((c % 64) / 32) + c % 8,
 *     slot sl = 4 * (i / 4) + j, word w = 2 * (e / n) + (i % 4) / 2,
 *     piece (bits / 2) * h + w / 4 (a 64-channel half of a row is bits / 2 pieces), 32-bit word w % 4 of the piece, low (i even)
 *     or high (i odd) half-word, bits [(e % n) * bits, +bits).
 *   K always uses the row form.
 *
 * Quantizer (the paper names `quant` without defining it; this is the reading
 * used): per token, per group of G channels along head_dim, asymmetric min/max.
 * Every step is one IEEE binary32 operation, round-to-nearest-even, unfused:
 *   mn, mx = min, max of the group (zeros of either sign compare equal: a zero minimum or maximum is +0)
 *   scale  = fp16((f32(mx) - f32(mn)) / (2^bits - 1)),  zero = mn
 *   code   = 0 if scale == 0, else
 *            clamp(rint((f32(x) - f32(mn)) * (1.0f / f32(scale))), 0, 2^bits - 1)
 */
#ifndef COCKTAIL_H
#define COCKTAIL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COCKTAIL_NUM_CLASSES 4
#define COCKTAIL_TOKENS_PER_BLOCK 64
#define COCKTAIL_MAX_Q_PER_KV 64
#define COCKTAIL_V_ROWS 0
#define COCKTAIL_V_TOKEN_QUADS 1

typedef enum cocktail_status {
  COCKTAIL_OK = 0,
  COCKTAIL_EINVAL = -1,       /* NULL pointer, non-positive size, bad chunk bit value, ...    */
  COCKTAIL_EUNSUPPORTED = -2, /* valid request this build has no kernel for                    */
  COCKTAIL_EALIGN = -3,       /* a device pointer is not 16-byte aligned                       */
  COCKTAIL_ENOSPACE = -4,     /* plan or workspace buffer smaller than required                */
  COCKTAIL_EHIP = -5,         /* the HIP runtime reported an error at launch                   */
  COCKTAIL_ESTATE = -6        /* cocktail_decode_check: the last decode call did not attend to every token once */
} cocktail_status;

/* Geometry of one attention layer call.  group_size divides head_dim. */
typedef struct cocktail_shape {
  int32_t batch;        /* B  sequences                                        */
  int32_t num_q_heads;  /* Hq query heads, a multiple of num_kv_heads          */
  int32_t num_kv_heads; /* Hkv                                                 */
  int32_t head_dim;     /* D, a multiple of 64 (kernels: 64 and 128)           */
  int32_t chunk_size;   /* C tokens per context chunk (Sec. III-A)             */
  int32_t group_size;   /* G in {32, 64, 128}: channels per scale/zero pair    */
} cocktail_shape;

/* Sizes the caller needs to allocate buffers; filled by cocktail_plan. */
typedef struct cocktail_sizes {
  int64_t total_chunks;                        /* sum_b floor(T_b / C): entries of perm            */
  int64_t class_tokens[COCKTAIL_NUM_CLASSES];  /* sum_b n_{b,c}                                    */
  int64_t class_blocks[COCKTAIL_NUM_CLASSES];  /* 64-token blocks in the K (= V) buffer of class c */
  int64_t class_bytes[COCKTAIL_NUM_CLASSES];   /* bytes of the K buffer, and of the V buffer       */
  int64_t plan_bytes;                          /* bytes of the plan blob                           */
  int64_t workspace_bytes;                     /* bytes of the decode-attention workspace          */
  int64_t packed_bytes;                        /* K+V bytes of codes + scale/zero, padding excluded */
  int32_t num_workers;                         /* workgroups the decode kernel is launched with    */
  int32_t num_partials;                        /* partial softmax states written per call          */
  int32_t num_segments;
  int32_t append_capacity;                     /* tokens per sequence the append buffers can take  */
  int64_t append_bytes;                        /* bytes of the K append buffer, and of the V one   */
  int32_t v_layout;                            /* COCKTAIL_V_ROWS or COCKTAIL_V_TOKEN_QUADS: form of the V blocks */
  int32_t reserved;
} cocktail_sizes;

/* The packed mixed-precision cache of one layer: the six lists of Alg. 1
 * (K_q2, K_q4, K_fp16, V_q2, V_q4, V_fp16), an INT8 pair between the INT4 and the FP16 ones, and the plan
 * that describes them. */
typedef struct cocktail_cache {
  void* k[COCKTAIL_NUM_CLASSES]; /* DEVICE, class_bytes[c] each, 256-byte aligned; may be NULL iff 0 bytes */
  void* v[COCKTAIL_NUM_CLASSES]; /* DEVICE, same sizes                                                     */
  const void* plan_host;         /* HOST   plan blob written by cocktail_plan                              */
  void* plan_dev;                /* DEVICE byte-for-byte copy of the plan blob, 16-byte aligned; also holds
                                    the decode kernel's ticket counters, the only part kernels write
                                    (see cocktail_decode_attention)                                        */
  void* k_app;                   /* DEVICE append_bytes each, 256-byte aligned: K/V rows of the tokens     */
  void* v_app;                   /*        generated during decoding; NULL iff append_capacity == 0         */
  int32_t num_appended;          /* tokens appended so far to every sequence, 0 .. append_capacity (batches
                                    that generate in lockstep); 0 if appended_dev is used                  */
  int32_t reserved;
  int32_t* appended_dev;         /* DEVICE int32 [B], or NULL: tokens appended so far per sequence, for batches
                                    whose sequences stop generating at different steps; read by
                                    cocktail_decode_attention, advanced by cocktail_append_fp16_ragged      */
} cocktail_cache;

/*
 * Host-only planning step (Alg. 1, prefill loop).
 * Computes the stable partition of every sequence's chunks by bitwidth, the token
 * count of every class (the FP16 class also receives the T_b mod C tail tokens,
 * Sec. III-A), the block layout of the packed cache and the static split of the
 * decode work over `num_workers` workgroups.
 *
 *   seq_lens     HOST [B]           context tokens T_b >= 0
 *   chunk_bits   HOST [sum_b N_b]   N_b = floor(T_b / C) values in {2, 4, 8, 16}, sequence after sequence
 *   num_workers  most workgroups the decode kernel may be launched with (> 0), normally
 *                cocktail_default_workers(); a plan never has more workers than 32-token
 *                (head_dim 64: 64-token) units of work, rounded up to a multiple of 64:
 *                sizes->num_workers says how many it has
 *   sizes        HOST out, always written on success
 *   plan_host    HOST out, plan_capacity bytes, or NULL to query sizes only
 *   class_tokens HOST out [B][COCKTAIL_NUM_CLASSES] n_{b,c}, or NULL
 *   perm         HOST out [sum_b N_b]: position j of sequence b's reordered chunk
 *                list holds original chunk perm[off_b + j] (the x_j of Eq. 5), or NULL
 *
 * Errors: EINVAL (NULL, bad shape, bad bit value), ENOSPACE (plan_capacity too small).
 * The plan blob is position independent: copy its plan_bytes bytes to the device
 * unchanged.  The host arrays may be freed on return.
 */
int cocktail_plan(const cocktail_shape* shape, const int32_t* seq_lens, const uint8_t* chunk_bits,
                  int32_t num_workers, cocktail_sizes* sizes, void* plan_host, size_t plan_capacity,
                  int32_t* class_tokens, int32_t* perm);

/* Options of cocktail_plan_ex; zero-initialise, then set what is needed. */
typedef struct cocktail_plan_options {
  int32_t append_capacity; /* >= 0: generated tokens per sequence the cache can take (Sec. III-A keeps their K/V
                              in FP16 behind the context).  They live in two extra buffers
                              (cocktail_cache::k_app, v_app; sizes->append_bytes each): per (sequence, kv head)
                              ceil(append_capacity / 64) blocks in the block layout of the FP16 class, ordered
                              (b, h, block).                                                                  */
  int32_t reproducible;    /* != 0: purely static split of the decode work (no shared pools): calls on the same
                              inputs then agree bit for bit, at some cost in speed                            */
  int32_t vector_alu_only; /* != 0: grouped-query shapes are planned for the kernel that runs one query head per wave
                              on the vector ALU alone (no matrix instructions, V in token rows); every query head
                              then reads the blocks of its kv head by itself                                    */
  int32_t reserved0;       /* must be zero                                                                    */
  const int32_t* max_seq_lens; /* HOST [B] or NULL: the context length every sequence may reach when generated tokens
                              are folded into the packed cache (cocktail_fold_appended; Sec. III-A: they stay FP16).
                              The FP16 run of every (sequence, kv head) is laid out with room for
                              max_seq_lens[b] - seq_lens[b] more tokens (zero blocks after reorder+quantize), so a
                              plan for a longer context with the same max_seq_lens has the same cache layout.
                              max_seq_lens[b] >= seq_lens[b].                                                   */
  int32_t reserved[2];     /* must be zero                                                                    */
} cocktail_plan_options;

/* cocktail_plan with options (NULL = defaults = cocktail_plan). */
int cocktail_plan_ex(const cocktail_shape* shape, const int32_t* seq_lens, const uint8_t* chunk_bits,
                     int32_t num_workers, const cocktail_plan_options* options, cocktail_sizes* sizes,
                     void* plan_host, size_t plan_capacity, int32_t* class_tokens, int32_t* perm);

/* Source layouts accepted by cocktail_reorder_quantize (element = one fp16). */
#define COCKTAIL_SRC_STRIDED 0 /* element (b,h,t,d) at b*stride_b + h*stride_h + t*stride_t + d        */
#define COCKTAIL_SRC_RAGGED 1  /* sequences concatenated; sequence b is [Hkv][T_b] rows of stride_t
                                  elements, starting at (sum_{b'<b} T_b') * Hkv * stride_t              */

/*
 * Prefill side of Alg. 1: gather every chunk into its class (reorder), then
 * quantize and pack the INT2, INT4 and INT8 classes; FP16 chunks and the tail are
 * copied.  One kernel launch handles K and V of all classes.
 *
 *   k_src, v_src  DEVICE fp16, 16-byte aligned, head_dim contiguous; strides in
 *                 elements, multiples of 8
 *   cache         k/v buffers are written completely (padding included), the append
 *                 buffers (if any) are zeroed; num_appended is not read;
 *                 plan_host/plan_dev must come from cocktail_plan for this shape
 *   stream        hipStream_t (NULL = default stream)
 *
 * Inputs must be finite.  Errors: EINVAL, EUNSUPPORTED (head_dim other than 64 or 128),
 * EALIGN, EHIP.  Nothing is launched when an error is returned.
 */
int cocktail_reorder_quantize(const cocktail_shape* shape, const void* k_src, const void* v_src,
                              int32_t src_layout, int64_t stride_b, int64_t stride_h, int64_t stride_t,
                              const cocktail_cache* cache, void* stream);

/*
 * The same prefill step from a paged KV cache, the way serving stacks keep K and V between prefill and
 * decode: two pools of fixed-size pages (one for K, one for V, same geometry) and a page table per
 * sequence.  Token t of sequence b, kv head h, channel d is the fp16 element at
 *     page_table[b * table_stride + t / page_size] * stride_page + h * stride_h + (t % page_size) * stride_t + d
 * of k_pages (v_pages).  Blocks whose 64 tokens lie inside one page are read with one base address, the
 * others row by row; any page_size >= 1 works, multiples of 64 are fastest.
 *
 *   k_pages, v_pages  DEVICE fp16, 16-byte aligned; strides in elements, multiples of 8, stride_t >= head_dim
 *   page_table        DEVICE int32 [B][table_stride]; row b names the ceil(T_b / page_size) pages of sequence b
 *                     in token order; entries behind them are not read.  An entry outside [0, num_pages) is
 *                     not followed: the rows of that page are quantized as zeros.
 *   cache, stream     as cocktail_reorder_quantize
 *
 * Errors: EINVAL (NULL, bad page geometry, a page table row too short for its sequence), EUNSUPPORTED, EALIGN, EHIP.
 */
typedef struct cocktail_paged_source {
  const void* k_pages;
  const void* v_pages;
  const int32_t* page_table;
  int32_t table_stride; /* entries per page table row                      */
  int32_t page_size;    /* tokens per page                                 */
  int32_t num_pages;    /* pages in each pool                              */
  int32_t reserved;     /* must be zero                                    */
  int64_t stride_page, stride_h, stride_t;
} cocktail_paged_source;

int cocktail_reorder_quantize_paged(const cocktail_shape* shape, const cocktail_paged_source* src,
                                    const cocktail_cache* cache, void* stream);

/*
 * Decode side of Alg. 1: out[b,h] = softmax(sm_scale * q[b,h] . K^_b^T) V^_b over
 * all tokens of all classes of sequence b, K^/V^ being the dequantized
 * (or raw fp16) rows of kv head h / (Hq/Hkv).  Two launches: partial states per
 * worker, then the exact merge.  Workers that finish their own share early take
 * further pieces from a pool shared by a few neighbouring workers; the pools are
 * handed out through ticket counters that live in the device copy of the plan.
 * The counters are zero in the blob cocktail_plan writes and every call leaves
 * them zero again, so calls on the same plan_dev must not overlap in time (calls
 * on one stream never do), and a plan_dev whose call was aborted has to be
 * re-uploaded.  A call that breaks this rule is not silently wrong: every partial
 * state records how many tokens it covers, the merge compares their sum with the
 * token count of the sequence, and a (sequence, query head) row that does not add
 * up gets NaN in out and lse and a non-zero status word (cocktail_decode_check);
 * the call after it finds the counters at zero again.  Which worker takes which pool piece differs from call to call, so
 * two calls on the same inputs agree to fp32 summation order, not bit for bit
 * (shapes with Hq/Hkv > 4 use no pools and are reproducible bit for bit, and so is any plan made with
 * cocktail_plan_options::reproducible).  Shapes with Hq = Hkv run one query head per wave on the vector
 * ALU; 2 <= Hq/Hkv <= 8 run four query heads per wave on 4x4x4 matrix instructions (V in token quads), unless
 * the plan asks for the vector ALU only; for larger ratios (up to COCKTAIL_MAX_Q_PER_KV) the query heads of a kv
 * head are cut into equal sets of up to 8 that each read the kv head's blocks (one head per wave if no such set size
 * divides the ratio).
 *
 *   cache      the appended tokens (num_appended of every sequence, or appended_dev[b] of sequence b) are
 *              attended to after the context
 *   q          DEVICE fp16 [B][Hq][D], 16-byte aligned
 *   sm_scale   softmax scale; <= 0 selects 1/sqrt(D)
 *   out        DEVICE fp16 [B][Hq][D]; a sequence with no tokens yields zeros
 *   lse        DEVICE fp32 [B][Hq] natural-log-sum-exp of the scaled logits
 *              (-inf for an empty sequence), or NULL
 *   workspace  DEVICE, workspace_bytes >= sizes.workspace_bytes, 16-byte aligned;
 *              contents need not be initialised and are overwritten (partial states,
 *              then one status word per (sequence, query head)).  Calls that share a
 *              workspace must not overlap in time.
 *
 * The packed K/V data is not modified.  Errors: EINVAL, EUNSUPPORTED (head_dim other than 64 or 128,
 * Hq/Hkv > COCKTAIL_MAX_Q_PER_KV), EALIGN, ENOSPACE, EHIP.
 */
int cocktail_decode_attention(const cocktail_shape* shape, const void* q, const cocktail_cache* cache,
                              float sm_scale, void* out, float* lse, void* workspace,
                              size_t workspace_bytes, void* stream);

/*
 * Measurement aid: cocktail_decode_attention that also records `event_between` (a hipEvent_t created by the
 * caller with timing enabled) on `stream` between its two kernels, so that the partial-state kernel (Alg. 1
 * decode phase, the kernel that streams the cache) and the merge can be timed apart with events on the launch
 * stream.  The record itself sits between the kernels: time whole calls with cocktail_decode_attention.
 * Errors: as cocktail_decode_attention; EINVAL if event_between is NULL; EHIP if the record fails.
 */
int cocktail_decode_attention_marked(const cocktail_shape* shape, const void* q, const cocktail_cache* cache,
                                     float sm_scale, void* out, float* lse, void* workspace, size_t workspace_bytes,
                                     void* stream, void* event_between);

/*
 * cocktail_decode_attention for callers that cannot allocate device memory or hand over a workspace: code
 * that runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same two kernels and same results, but the partial states go to a workspace built into the library: a
 * static device array of COCKTAIL_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds until the
 * process ends.  The call allocates and frees nothing, on the device or through any library.
 *
 * Every call on a GPU shares that GPU's array, so calls that overlap in time on one GPU (two streams, two
 * threads) race; nothing in it has to survive from one call to the next.  The array's address is looked up
 * on the first call on each device (with that device current): make that call outside a graph capture.
 *
 * Errors: as cocktail_decode_attention, and ENOSPACE if the plan's workspace_bytes exceeds
 * COCKTAIL_STATIC_WORKSPACE_BYTES (the five benchmark shapes need 0.1 to 5.2 MB).
 */
#define COCKTAIL_STATIC_WORKSPACE_BYTES (16u << 20)
int cocktail_decode_attention_static(const cocktail_shape* shape, const void* q, const cocktail_cache* cache,
                                     float sm_scale, void* out, float* lse, void* stream);

/*
 * Diagnostic: waits for `stream`, then reads the status words the last decode call on `workspace` left
 * (the only entry point that synchronises and copies).  The softmax of Alg. 1's decode phase runs over the
 * concatenation of all classes, i.e. over every token of the sequence exactly once; the status word
 * of a (sequence, query head) is the number of tokens its partial states covered minus the sequence length.
 *
 *   workspace  DEVICE, the workspace of that call; NULL = the built-in one of cocktail_decode_attention_static
 *
 * Returns COCKTAIL_OK if every word is zero, else COCKTAIL_ESTATE with a message naming the first bad row
 * (see cocktail_decode_attention for the causes).  Other errors: EINVAL, EHIP.
 */
int cocktail_decode_check(const cocktail_shape* shape, const cocktail_cache* cache, const void* workspace,
                          void* stream);

/*
 * Sec. III-A: stores the K/V rows of one generated token per sequence, in FP16, as token `position`
 * (0-based) of the append buffers.  The caller then sets cache->num_appended = position + 1 (or higher)
 * for the following cocktail_decode_attention calls, which attend to the context and to the first
 * num_appended appended tokens of every sequence.
 *
 *   k_new, v_new  DEVICE fp16 [B][Hkv][D], 16-byte aligned
 *   position      0 <= position < append_capacity of the plan
 *
 * One kernel launch.  Errors: EINVAL (no append buffers, position out of range, NULL), EALIGN, EHIP.
 */
int cocktail_append_fp16(const cocktail_shape* shape, const void* k_new, const void* v_new,
                         const cocktail_cache* cache, int32_t position, void* stream);

/*
 * Sec. III-A for a batch whose sequences generate (and stop) independently: for every sequence b with
 * active_dev[b] != 0 the K/V rows of its new token are stored as appended token cache->appended_dev[b] of that
 * sequence, then appended_dev[b] is advanced by one; the rows of the other sequences are ignored.  A sequence
 * whose append buffer is full (appended_dev[b] == append_capacity) is left as it is.  The following
 * cocktail_decode_attention calls attend to the context and to the first appended_dev[b] appended tokens of
 * every sequence.  Counts and flags live on the device, so a decode loop needs no host round trip.
 *
 *   k_new, v_new  DEVICE fp16 [B][Hkv][D], 16-byte aligned
 *   cache         appended_dev must not be NULL (zero it before the first token; cocktail_reorder_quantize
 *                 does not touch it)
 *   active_dev    DEVICE uint8 [B], or NULL = every sequence
 *
 * Two kernel launches (store, then advance the counts).  Errors: EINVAL, EUNSUPPORTED, EALIGN, EHIP.
 */
int cocktail_append_fp16_ragged(const cocktail_shape* shape, const void* k_new, const void* v_new,
                                const cocktail_cache* cache, const uint8_t* active_dev, void* stream);

/*
 * Sec. III-A, for long generations: the tokens appended so far become context.  Their K/V rows move from the
 * append buffers into the packed cache, behind the FP16 rows of their (sequence, kv head) (they stay FP16 and keep
 * their place in the order of the tokens: the FP16 list of Alg. 1 grows at its end, nothing is quantized again), so
 * that the decode work split of a new plan covers them like any other token instead of leaving them to the few
 * workgroups that serve the append buffers.
 *
 *   cache          the cache as it is: plan_host / plan_dev = the plan in use (made with append buffers and with
 *                  cocktail_plan_options::max_seq_lens), class and append buffers, appended_dev or num_appended
 *   new_plan_host  HOST plan of the longer contexts: seq_lens[b] + (tokens appended to sequence b), chunk_bits
 *                  extended by 16 for every chunk the new tokens complete, the same shape and the same
 *                  max_seq_lens, hence the same cache layout (checked)
 *   new_plan_dev   DEVICE copy of new_plan_host, 16-byte aligned, complete before this call runs on `stream`
 *
 * Every sequence is folded completely: new seq_lens[b] - old seq_lens[b] has to be the number of tokens appended
 * to sequence b (checked against num_appended for batches in lockstep; with appended_dev the counts live on the
 * device and are the caller's to match).  Afterwards the caller switches cache->plan_host and cache->plan_dev to
 * the new plan and sets num_appended = 0; appended_dev is cleared by this call.  The workspace of the new plan may
 * be larger than the old one's.
 *
 * One or two kernel launches.  Errors: EINVAL (plans that differ in more than FP16 tokens at the end, counts out of
 * range, NULL), EUNSUPPORTED, EALIGN, EHIP.
 */
int cocktail_fold_appended(const cocktail_shape* shape, const cocktail_cache* cache, const void* new_plan_host,
                           const void* new_plan_dev, void* stream);

/*
 * Chunk-level quantization search (Sec. III-B): scores[i] = cosine similarity of sequence b's query
 * embedding with chunk embedding i (Eq. 1); per sequence T_low = s_min + (s_max - s_min) * alpha and
 * T_high = s_max - (s_max - s_min) * beta (Eq. 2-3); chunk_bits[i] = 2 if scores[i] < T_low, else 16
 * if scores[i] > T_high, else 4 (the comparisons of Alg. 1's prefill loop, in that order).  The
 * embeddings come from the caller's encoder.  Arithmetic: sums in binary64, the score rounded once
 * to binary32 (0 if either vector is zero), thresholds and comparisons in unfused binary32.
 *
 *   chunk_off   DEVICE int32 [B+1]  prefix sum of the chunk counts N_b (chunk_off[B] = total_chunks)
 *   query_emb   DEVICE fp32 [B][E]
 *   chunk_emb   DEVICE fp32 [total_chunks][E], sequence after sequence
 *   alpha, beta in [0, 1] (the paper uses 0.6 and 0.1)
 *   scores      DEVICE fp32 [total_chunks] out
 *   chunk_bits  DEVICE uint8 [total_chunks] out, values 2 / 4 / 16: copy to the host for cocktail_plan
 *
 * Two kernel launches.  Errors: EINVAL, EALIGN, EHIP.
 */
int cocktail_chunk_bitwidths(int32_t batch, int32_t embed_dim, int32_t total_chunks, const int32_t* chunk_off,
                             const float* query_emb, const float* chunk_emb, float alpha, float beta, float* scores,
                             uint8_t* chunk_bits, void* stream);

/*
 * Number of decode workgroups that fills the current HIP device for this shape
 * (compute units x resident waves per unit / waves per workgroup; a workgroup is two waves for
 * 5 <= Hq/Hkv <= 8 and one wave otherwise).  Needs a GPU: EHIP otherwise.
 */
int cocktail_default_workers(const cocktail_shape* shape, int32_t* num_workers);

/*
 * Measurement aid, not a step of the method: enqueues a plain 128-bit streaming read of
 * `buf` (2048 single-wave workgroups, each over one contiguous range), so that a benchmark
 * can report the HBM read rate this GPU reaches with loads alone beside the rate of the
 * decode kernel (whose cost the paper attributes to loading the KV cache, Sec. I).
 *
 *   buf         DEVICE, 16-byte aligned, `bytes` >= 16 MiB readable bytes
 *   sink        DEVICE, 4 bytes the kernel may write
 *   bytes_read  HOST out: bytes the launch reads (`bytes` rounded down to 16 MiB)
 *
 * Errors: EINVAL, EALIGN, EHIP.
 */
int cocktail_stream_read_probe(const void* buf, size_t bytes, void* sink, size_t* bytes_read, void* stream);

/*
 * Diagnostic, not a step of the method.  The quantizer (top of this file) is defined by IEEE binary32
 * divisions; the kernel replaces them by shorter sequences that are exact on the operands that can
 * occur.  This call checks that claim on the device for every such operand: all floats in [0, 131008]
 * for (mx - mn) / 3, / 15 and / 255, and every positive finite fp16 value for 1 / scale.
 *
 *   mismatches  DEVICE uint64 [4] out, 16-byte aligned: operands on which the result differs from the
 *               division, for / 3, / 15, 1 / scale, / 255.  All zero on a correct device.
 *
 * Two kernel launches (about a millisecond).  Errors: EINVAL, EALIGN, EHIP.
 */
int cocktail_selftest_arithmetic(uint64_t* mismatches, void* stream);

/*
 * Debugging aid: value of one field of the plan header (the internal layout of the blob cocktail_plan writes),
 * by the name it has in the library's source, e.g. "off_counters", "num_groups", "class_blocks" (index =
 * class), plus a few constants of the layout ("counter_stride_bytes", "iter_units", "sizeof_worker_rec", ...).
 * Errors: EINVAL (not a plan of this library version, unknown name, index out of range).
 */
int cocktail_plan_field(const void* plan_host, const char* name, int32_t index, int64_t* value);

/* Message of the last failure on the calling thread ("" if none).  Static storage. */
const char* cocktail_last_error(void);

/* Library version, (major << 16) | minor. */
int cocktail_version(void);

#ifdef __cplusplus
}
#endif
#endif /* COCKTAIL_H */
