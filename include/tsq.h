/*
 * tsq.h — C ABI of the MI355X (gfx950) library for two-stage compression of a
 * split-point hidden-state tensor [tokens x hidden] and its exact inverse:
 *
 *   threshold splitting (TS)  — paper Sec. II-C.1, Eq. (ts): elements with
 *       |x| >= tau go, untouched, to a sparse side stream stored in CSR form;
 *   token-wise adaptive bit quantization (TAB-Q) — Sec. II-C.2, Eq. (Proposed)
 *       and Algorithm 1: every token gets its own bit-width from an allowed
 *       set, chosen by descending through the set while a distortion statistic
 *       stays within a budget; magnitudes are quantized with round-half-even
 *       and bit-packed, one sign bit per element;
 *   restore — Eq. (dequnt): unpack, dequantize, put the outliers back.
 *
 * All pointers named d_* are DEVICE pointers on the current HIP device; every
 * other pointer is a HOST pointer.  The library allocates no device memory and never
 * synchronizes the host except where stated.  The state it keeps per device is small: the static
 * workspace of tsq_compress_static, and which stream the last single-pass compress call used.  Two
 * such calls on different streams of one device are ordered one after the other (the later one's
 * stream is made to wait for what the earlier one's stream holds at that moment; an event, no
 * host synchronization): their kernels' workgroups wait for one another and would, sharing the
 * device, keep each other from starting.  Calls on one stream, restore calls and the staged
 * pipeline are not affected.  Calls recorded into a HIP graph are ordered by the graph only: do
 * not replay two graphs that hold single-pass compress calls at the same time on one device.
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *
 * Errors are return codes only (no exceptions, no abort).
 */
#ifndef TSQ_H
#define TSQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TSQ_OK              = 0,
    TSQ_ERR_INVALID_ARG = 1,  /* NULL pointer, zero size, tau/budget/bit set out of domain      */
    TSQ_ERR_UNSUPPORTED = 2,  /* valid request this build cannot run (shape limits below)       */
    TSQ_ERR_CAPACITY    = 3,  /* the outlier side stream did not fit max_outliers               */
    TSQ_ERR_HIP         = 4,  /* a HIP call or kernel launch failed                             */
    TSQ_ERR_FORMAT      = 5,  /* the blob does not carry this library's header / this plan, or
                                 the workspace was not reset for this plan's shape              */
    TSQ_ERR_INTERNAL    = 6,  /* a bounded device-side wait expired, or the workspace still
                                 carries the failure of an earlier call                         */
    TSQ_ERR_NO_MEMORY   = 7   /* a host allocation failed                                       */
} tsq_status;

typedef enum { TSQ_F16 = 0, TSQ_BF16 = 1 } tsq_dtype;

typedef enum {
    TSQ_BUDGET_LSB     = 0,   /* Algorithm 1 as printed: mean |floor(T0/2^k) - T| in code LSBs
                                 of the candidate width, compared with Delta                    */
    TSQ_BUDGET_REL_RMS = 1    /* the same statistic in value units, compared with
                                 budget * RMS of the token's inlier part                        */
} tsq_budget_mode;

typedef enum {
    TSQ_RETURN_LAST_PASSING = 0, /* the last width whose statistic stayed within the budget (the largest
                                    allowed width if the first candidate already exceeds it)      */
    TSQ_RETURN_AS_PRINTED   = 1  /* Algorithm 1's steps in their printed order: the candidate is
                                    quantized, tested, and on failure THAT quantization is returned */
} tsq_return_rule;

typedef enum {
    TSQ_PIPE_AUTO   = 0,      /* the library picks: TSQ_PIPE_FUSED wherever the device can hold
                                 two workgroups of its kernel at once, else TSQ_PIPE_STAGED     */
    TSQ_PIPE_STAGED = 1,      /* row statistics -> device-wide scan -> pack: three launches,
                                 the input is read twice                                        */
    TSQ_PIPE_FUSED  = 2       /* one launch, the input is read once.  Every token is handed out
                                 by ticket counters in the workspace, so whichever workgroups
                                 are running finish the call (none waits for one that has not
                                 started); one workgroup scans the published sizes into the
                                 tokens' places.  Every device-side wait is bounded: if the
                                 workgroup that scans is kept from running for about a second,
                                 the call ends with TSQ_ERR_INTERNAL in the blob's status      */
} tsq_pipeline;

/* Problem statement (Algorithm 1 "Require": T, Q-bar, Delta; Eq. (ts): tau). */
typedef struct {
    uint32_t tokens;        /* T >= 1: rows of the tensor                                       */
    uint32_t hidden;        /* H: row length; this build needs H % 8 == 0 and 8 <= H <= 32768
                               (one workgroup of at most 1024 lanes holds a row, 32 elements
                               per lane)                                                        */
    int32_t  dtype;         /* tsq_dtype of the input and of the restored output                */
    float    tau;           /* TS threshold, 0 < tau < inf                                      */
    uint32_t bit_mask;      /* allowed widths: bit b set <=> b allowed, 2 <= b <= 8, b counts
                               the sign bit (magnitude levels 2^(b-1) - 1)                      */
    float    budget;        /* Delta (LSB mode) or epsilon (REL_RMS mode), >= 0, may be +inf    */
    int32_t  mode;          /* tsq_budget_mode                                                  */
    int32_t  pipeline;      /* tsq_pipeline                                                     */
    uint64_t max_outliers;  /* capacity of the side stream in elements; 0 = tokens*hidden       */
    int32_t  return_rule;   /* tsq_return_rule: which width the descent returns when a candidate
                               exceeds the budget (both give the smallest width if none does)   */
    int32_t  reserved;      /* 0                                                                */
} tsq_config;

typedef struct tsq_plan tsq_plan;   /* opaque, host memory, never written after tsq_plan_create,
                                       usable from any thread, on any device, across calls     */

/*
 * Layout of a compressed blob (device memory, all little-endian, every section
 * 256-byte aligned, offsets in bytes from the blob's start):
 *   header    128 B   magic "TSQ1", version, the plan's parameters, status, nnz, payload_bytes,
 *                     the section offsets and capacities below
 *   bits      u8 [T]      chosen width b_t per token            (Algorithm 1's Q*)
 *   scale     f32[T]      s_t = inlier absmax / (2^(b_t-1) - 1) (Algorithm 1's S*; Z* = 0)
 *   pay_off   u64[T+1]    byte offset of each token's codes inside payload (exclusive scan)
 *   row_ptr   u64[T+1]    CSR row pointers of the outlier stream            (exclusive scan)
 *   payload   bytes       per token a dense LSB-first stream of b_t-bit sign|magnitude codes,
 *                         element j in stream bits [j*b_t, (j+1)*b_t), sign in the field's top
 *                         bit, zero padded to a multiple of 4 bytes; outlier slots hold code 0
 *   out_col   u16[cap]    CSR column indices, ascending inside a token
 *   out_val   u16[cap]    the outliers' raw 16-bit input values (lossless, NaN payloads kept)
 * Bytes past the actual lengths (payload_bytes, nnz) are unspecified.
 */
typedef struct {
    uint64_t blob_bytes;       /* what the caller must allocate for d_blob                      */
    uint64_t workspace_bytes;  /* what the caller must allocate for d_ws                        */
    uint64_t off_bits, off_scale, off_pay_off, off_row_ptr, off_payload, off_out_col, off_out_val;
    uint64_t payload_capacity; /* bytes                                                         */
    uint64_t outlier_capacity; /* elements                                                      */
} tsq_layout;

typedef struct {
    uint64_t nnz;               /* outliers stored                                              */
    uint64_t payload_bytes;     /* sum over tokens of 4*ceil(H*b_t/32)                          */
    uint64_t compressed_bytes;  /* 128 + 5T + 16(T+1) + payload_bytes + 4*nnz                   */
    uint64_t width_hist[9];     /* tokens per width, index = width                              */
    uint32_t status;            /* tsq_status recorded by the device (0 = ok)                   */
    uint32_t reserved;
} tsq_info;

/* Validates cfg and fixes the blob layout.  Host only.  Returns INVALID_ARG / UNSUPPORTED /
 * NO_MEMORY without touching *out on failure.  (How many workgroups a launch gets depends on the
 * device and is looked up at each call for the device current then.) */
tsq_status tsq_plan_create(const tsq_config *cfg, tsq_plan **out);
void       tsq_plan_destroy(tsq_plan *plan);
tsq_status tsq_plan_layout(const tsq_plan *plan, tsq_layout *out);
size_t     tsq_plan_blob_bytes(const tsq_plan *plan);
size_t     tsq_plan_workspace_bytes(const tsq_plan *plan);

/*
 * Puts d_ws into its initial state (enqueues one small kernel on `stream`).
 * Required once after d_ws is allocated, and again after any compress call on
 * it that was aborted or returned TSQ_ERR_INTERNAL through tsq_blob_info; every
 * completed compress call leaves the workspace ready for the next call by
 * itself.  A workspace serves one compress call at a time (calls that overlap
 * on one workspace race), and only plans of one shape (tokens, hidden): the
 * reset records the shape, and a compress call with a plan of another shape (or
 * on a workspace that was never reset) touches nothing in the workspace, stores
 * nothing but a header with status TSQ_ERR_FORMAT, and tsq_blob_info returns that.
 */
tsq_status tsq_workspace_reset(const tsq_plan *plan, void *d_ws, void *stream);

/*
 * TS + TAB-Q (Eq. (ts), Eq. (Proposed), Algorithm 1).
 *   d_in   : tokens*hidden 16-bit values, row-major, 16-byte aligned, read only
 *   d_blob : tsq_plan_blob_bytes() bytes, 256-byte aligned, fully overwritten where specified
 *   d_ws   : tsq_plan_workspace_bytes() bytes, 256-byte aligned, reset as described above
 * Only enqueues work on `stream`; never synchronizes.  Buffers must not overlap.
 * A side stream larger than max_outliers is detected on the device: the blob's
 * status becomes TSQ_ERR_CAPACITY (reported by tsq_blob_info) and the tokens
 * that no longer fit have no outliers stored.
 */
tsq_status tsq_compress(const tsq_plan *plan, const void *d_in, void *d_blob, void *d_ws,
                        void *stream);

/*
 * tsq_compress for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is a static device array inside the library, tsq_static_workspace_bytes() = 4 MiB
 * per GPU the library runs on, held until the process ends.  A plan whose
 * tsq_plan_workspace_bytes() exceeds that (about 200 000 tokens) is refused with
 * TSQ_ERR_UNSUPPORTED before anything is enqueued.  The call allocates and frees nothing, needs no
 * tsq_workspace_reset (it enqueues a small fill kernel ahead of the compress kernels, so any plan
 * may follow any other), and writes the same blob as tsq_compress.  All calls on one GPU share
 * that GPU's array: calls that overlap in time on one GPU (different streams, different threads)
 * race; calls on one stream are safe.  Arguments, asynchrony and errors otherwise as for
 * tsq_compress.
 */
tsq_status tsq_compress_static(const tsq_plan *plan, const void *d_in, void *d_blob, void *stream);
size_t     tsq_static_workspace_bytes(void);

/*
 * tsq_compress, then tsq_blob_info into *info_out: SYNCHRONIZES `stream`.  For callers that want the
 * outcome before going on (the controller of Algorithm 2 needs the compressed size anyway).  With
 * TSQ_PIPE_AUTO, a call whose single pass gave up (status TSQ_ERR_INTERNAL, or TSQ_ERR_FORMAT
 * recorded by the device because of the workspace) is run once more here: the workspace is reset
 * and the staged kernels, which wait for nothing, compress the same input into the same blob.
 * Returns what tsq_blob_info returns for the final blob.
 */
tsq_status tsq_compress_blocking(const tsq_plan *plan, const void *d_in, void *d_blob, void *d_ws,
                                 void *stream, tsq_info *info_out);

/*
 * Restore (Eq. (dequnt)): d_out receives tokens*hidden 16-bit values of the
 * plan's dtype.  Inliers become sign * (code * s_t) rounded to nearest even,
 * outliers their stored bits.  If the blob's header does not match the plan or
 * carries a non-zero status, nothing is written.  Enqueues only.
 */
tsq_status tsq_decompress(const tsq_plan *plan, const void *d_blob, void *d_out, void *stream);

/*
 * The KV-cache form of the two calls above (Sec. II-B: Eq. (bkv_lth_stage) counts the key and
 * value tensors of every layer, Eq. (if_total) with I_kv = 1 sends them; footnote of Sec. II-C.1:
 * the cache goes through the same TS + TAB-Q as the layer output): the plan's `tokens` rows are
 * the rows of tokens / rows_per_tensor separate tensors [rows_per_tensor x hidden], taken in
 * table order, all compressed by ONE launch into ONE blob that is byte for byte what
 * tsq_compress produces for the concatenation of the tensors.
 *   d_in_ptrs / d_out_ptrs : DEVICE array (8-byte aligned) of tokens / rows_per_tensor device
 *                            pointers, each to a row-major, 16-byte aligned tensor; the table
 *                            and the tensors belong to the caller and must stay valid until the
 *                            call has run on `stream`
 *   rows_per_tensor        : >= 1 and a divisor of the plan's tokens, else TSQ_ERR_INVALID_ARG
 * Everything else (workspace, errors, asynchrony) as for tsq_compress / tsq_decompress; a blob
 * written by either form is read by either form.
 */
tsq_status tsq_compress_batch(const tsq_plan *plan, const void *const *d_in_ptrs,
                              uint32_t rows_per_tensor, void *d_blob, void *d_ws, void *stream);
tsq_status tsq_decompress_batch(const tsq_plan *plan, const void *d_blob, void *const *d_out_ptrs,
                                uint32_t rows_per_tensor, void *stream);

/*
 * Symbol statistics for the entropy coder that follows TAB-Q (Sec. II-C.2, last paragraph: the
 * quantized symbols are coded with rANS).  d_hist receives tokens*256 32-bit counts, row-major:
 * entry [t][c] = number of elements of token t whose b_t-bit code (sign in bit b_t-1, magnitude
 * below it, exactly the field stored in the payload) equals c.  A row sums to `hidden`;
 * entries c >= 2^b_t are written as 0; outlier slots carry code 0 and count as such.
 *   d_hist : tokens*256*4 bytes, 4-byte aligned
 * If the blob's header does not match the plan or carries a non-zero status, nothing is written.
 * Enqueues only.
 */
tsq_status tsq_code_histogram(const tsq_plan *plan, const void *d_blob, void *d_hist, void *stream);

/*
 * Entropy coding of the payload (Sec. II-C.2, last paragraph: the symbols TAB-Q produces are coded
 * with rANS).  The paper leaves the coder to a third-party package; the format is this library's:
 * one 12-bit frequency table per width class, built from the pooled code counts (scaled to a sum
 * of 4096, every occurring code at least 1); per token 64 interleaved rANS coders (state in
 * [2^16, 2^32), 16-bit renormalisation), coder l owning the runs of 32 codes l, l + 64, ...; a
 * token's stream is the final states of the coders that own a run (min(64, runs) of them)
 * followed by the 16-bit words in the order the decoder reads them, padded to 4 bytes.
 *
 * Entropy-coded payload ("eblob", device memory, little-endian, offsets from its start in
 * tsq_entropy_layout): 256-byte header | tables u16[7][256] (row b - 2: width b) |
 * stream offsets u64[tokens + 1] (bytes from the start of the streams) | streams.
 *
 * tsq_entropy_encode reads a completed blob and writes d_eblob; only the payload section of the
 * blob is recoded, its other sections (widths, scales, offsets, outliers) travel as they are.
 * tsq_entropy_decode writes the payload section of d_blob back from d_eblob; d_blob must hold the
 * blob's other sections (header, widths, offsets) already.  The restored payload is byte for byte
 * the one that was encoded.
 *   d_eblob : tsq_entropy_blob_bytes() bytes (capacity for the longest possible streams), 256-byte aligned
 *   d_ews   : tsq_entropy_workspace_bytes() bytes, 256-byte aligned, encoder only, needs no reset;
 *             it serves one encode call at a time (calls that overlap on one workspace race)
 * Both calls only enqueue.  If the blob (or, for decode, the eblob) is not this plan's or carries
 * a non-zero status, nothing is written and the eblob's header stays invalid.
 * tsq_entropy_info SYNCHRONIZES `stream`; it returns FORMAT for an eblob that is not this plan's.
 */
typedef struct {
    uint64_t off_tables, off_stream_off, off_streams;
    uint64_t stream_capacity;   /* bytes                                                          */
    uint64_t stream_bytes;      /* bytes of all streams                                           */
    uint64_t coded_bytes;       /* header + tables + offsets + streams: what replaces the payload */
} tsq_entropy_layout;
size_t     tsq_entropy_blob_bytes(const tsq_plan *plan);
size_t     tsq_entropy_workspace_bytes(const tsq_plan *plan);
tsq_status tsq_entropy_encode(const tsq_plan *plan, const void *d_blob, void *d_eblob, void *d_ews, void *stream);
tsq_status tsq_entropy_decode(const tsq_plan *plan, const void *d_eblob, void *d_blob, void *stream);
tsq_status tsq_entropy_info(const tsq_plan *plan, const void *d_eblob, tsq_entropy_layout *host_out, void *stream);

/*
 * Size in bytes of what carries the first k tokens when the codes travel entropy-coded: the blob's
 * header, per-token metadata and CSR entries as in tsq_prefix_bytes, and in place of the codes the
 * coded blob's header, its frequency tables (those of the whole blob: a prefix is coded with them),
 * k + 1 stream offsets and the streams of the first k tokens.  For k = tokens that is
 * tsq_info.compressed_bytes - payload_bytes + tsq_entropy_layout.coded_bytes.  d_eblob must be the
 * coded form of d_blob.  k, n, bytes_out, synchronization and results as for tsq_prefix_bytes
 * (FORMAT also for an eblob that is not this plan's).
 */
tsq_status tsq_entropy_prefix_bytes(const tsq_plan *plan, const void *d_blob, const void *d_eblob,
                                    const uint32_t *k, uint32_t n, uint64_t *bytes_out, void *stream);

/*
 * Reads the blob's header and widths back to the host.  SYNCHRONIZES `stream`.
 * Returns the status stored in the blob (CAPACITY / FORMAT / INTERNAL), FORMAT when
 * the header is not this plan's (host_out->status is 0 then), or OK.
 */
tsq_status tsq_blob_info(const tsq_plan *plan, const void *d_blob, tsq_info *host_out,
                         void *stream);

/*
 * Compressed size in bytes of the first k tokens of a blob, as a blob of k tokens would report it
 * (tsq_info.compressed_bytes: header, 5 bytes and two offsets per token plus the closing pair, the
 * codes before pay_off[k], 4 bytes per outlier before row_ptr[k]): what Algorithm 2 needs when it
 * sends fewer tokens.  k (host) lists n token counts, each <= tokens; k = NULL means k = 0 .. n-1
 * (n <= tokens + 1).  bytes_out (host) receives n sizes.  SYNCHRONIZES `stream`.  Returns as
 * tsq_blob_info does; bytes_out is unspecified unless the result is TSQ_OK.
 */
tsq_status tsq_prefix_bytes(const tsq_plan *plan, const void *d_blob, const uint32_t *k, uint32_t n,
                            uint64_t *bytes_out, void *stream);

/*
 * Link model and early exit (Sec. II-D.2).  HOST-only scalar code, no GPU work; every pointer
 * is a host pointer.  Sizes are in bits, rates in bits per second, times in seconds.
 *
 * tsq_link: bandwidth W in Hz, received SNR gamma, target outage probability epsilon.
 *   outage probability     P_o(R) = 1 - exp(-(2^(R/W) - 1) / gamma)
 *   worst-case latency     L_eps(D_tx; R) = D_tx / R * ceil(ln eps / ln P_o(R))   Eq. (comm_latency)
 *                          (+inf where P_o(R) = 1; at least one transmission; 0 for D_tx = 0)
 *   best rate              Eq. (epsilon_rstar): the rate in [rate_lo, rate_hi] with the smallest
 *                          worst-case delay, i.e. the one that maximises R * ln(1 / P_o(R))
 *                          (Eq. (comm_latency) without its ceiling is proportional to the
 *                          reciprocal of that product; the function g as printed next to
 *                          Eq. (epsilon_rstar) has the rate in the denominator and falls to 0 as the
 *                          link saturates, so it cannot be what is minimised), by search on a
 *                          uniform grid of steps + 1 rates (the first best wins)
 * Invalid arguments (NULL, W <= 0, gamma <= 0, epsilon outside (0,1), rate <= 0, ...) give NaN.
 */
typedef struct {
    double bandwidth_hz;
    double snr;
    double outage;
} tsq_link;
double tsq_link_outage_probability(const tsq_link *link, double rate);
double tsq_link_latency(const tsq_link *link, double bits, double rate);
double tsq_link_best_rate(const tsq_link *link, double rate_lo, double rate_hi, uint32_t steps);

/*
 * One decision of Algorithm 2 (early exit under a delay constraint) for the token count and the
 * layer at hand: keep going if the intermediate output fits the deadline as it is; else send it
 * compressed; else compressed without the KV cache (I_kv = 0); else cut tokens from the end
 * until the deadline holds.  Total latency is L_c(w) + L_eps(size; rate), Eq. (total).
 *   tokens                   : w, tokens of the hidden state so far
 *   compute_latency          : w + 1 entries, L_c(k) for k = 0 .. w tokens (profiled by the caller)
 *   raw_bits                 : B_io of Eq. (if_total) with the cache, uncompressed
 *   compressed_bits_with_kv  : 8 * compressed_bytes of the hidden state's blob plus the cache's
 *   hidden_prefix_bits       : w + 1 entries, compressed size of the first k tokens of the hidden
 *                              state (k = 0 .. w; from the blob's pay_off / row_ptr and the
 *                              21 bytes of metadata per token)
 * Returns INVALID_ARG on NULL pointers or a link / rate / deadline out of domain.
 */
typedef enum {
    TSQ_EXIT_CONTINUE = 0,      /* the uncompressed output meets the deadline: no exit            */
    TSQ_EXIT_COMPRESSED = 1,    /* exit, sending hidden state and cache through TS + TAB-Q        */
    TSQ_EXIT_WITHOUT_KV = 2,    /* exit, sending the compressed hidden state only                 */
    TSQ_EXIT_FEWER_TOKENS = 3   /* exit, sending the first `tokens` tokens of it only             */
} tsq_exit_action;
typedef struct {
    tsq_link link;
    double rate;                /* R*, e.g. from tsq_link_best_rate                               */
    double deadline;            /* D                                                              */
    uint32_t tokens;
    const double *compute_latency;
    double raw_bits;
    double compressed_bits_with_kv;
    const uint64_t *hidden_prefix_bits;
} tsq_exit_input;
typedef struct {
    int32_t action;             /* tsq_exit_action                                                */
    int32_t with_kv;            /* I_kv of what is sent                                           */
    uint32_t tokens;            /* tokens of the hidden state that are sent                       */
    uint32_t reserved;
    double latency;             /* L_t of the decision (above the deadline only if even zero
                                   tokens do not meet it)                                         */
} tsq_exit_decision;
tsq_status tsq_early_exit_decide(const tsq_exit_input *in, tsq_exit_decision *out);

/*
 * Algorithm 2 with its two loops: for w = 1 .. max_tokens (W-bar), for layer = 1 .. layers (L), in
 * the printed order of steps.  The caller's callbacks stand for the forward pass and for the sizes:
 *   compute_latency(w, layer, user)                 L_c after w tokens up to `layer`, seconds
 *   bits(w, layer, with_kv, compressed, keep, user) what would be sent then, in bits: compressed = 0
 *       the raw intermediate output (B_io of Eq. (if_total), cache included iff with_kv); compressed
 *       = 1 the output through TS + TAB-Q with only the first `keep` tokens of the hidden state
 *       (tsq_compress, then tsq_blob_info / tsq_prefix_bytes; cache included iff with_kv)
 * Each (w, layer) is one step; the callbacks are called at every step, so sizes are measured as the
 * tensors grow.  The walk returns at the first exit: TSQ_EXIT_COMPRESSED (the compressed output
 * meets the deadline) or TSQ_EXIT_FEWER_TOKENS (not even without the cache: tokens are cut from the
 * end until it does, or none is left).  When dropping the cache alone brings the latency under the
 * deadline the printed steps do not return: the walk goes on with I_kv = 0.  If no step exits, the
 * result is TSQ_EXIT_COMPLETED with the compressed size of the whole output.  A callback that returns
 * a negative value or NaN ends the walk with INVALID_ARG.
 */
#define TSQ_EXIT_COMPLETED 4       /* all max_tokens x layers steps ran; the output is sent compressed */
typedef double (*tsq_exit_latency_fn)(uint32_t tokens, uint32_t layer, void *user);
typedef double (*tsq_exit_bits_fn)(uint32_t tokens, uint32_t layer, int32_t with_kv, int32_t compressed,
                                   uint32_t keep, void *user);
typedef struct {
    tsq_link link;
    double rate;                /* R*                                                             */
    double deadline;            /* D                                                              */
    uint32_t max_tokens;        /* W-bar                                                          */
    uint32_t layers;            /* L >= 1                                                         */
    tsq_exit_latency_fn compute_latency;
    tsq_exit_bits_fn bits;
    void *user;                 /* passed through to the callbacks                                */
} tsq_exit_walk_input;
typedef struct {
    int32_t action;             /* TSQ_EXIT_COMPRESSED, TSQ_EXIT_FEWER_TOKENS or TSQ_EXIT_COMPLETED */
    int32_t with_kv;            /* I_kv of what is sent                                           */
    uint32_t tokens;            /* w at the exit                                                  */
    uint32_t layer;             /* layer at the exit                                              */
    uint32_t sent_tokens;       /* tokens of the hidden state that are sent (<= tokens)           */
    uint32_t steps;             /* (w, layer) steps taken                                         */
    double latency;             /* L_t of what is sent                                            */
} tsq_exit_walk_result;
tsq_status tsq_early_exit_walk(const tsq_exit_walk_input *in, tsq_exit_walk_result *out);

const char *tsq_status_string(tsq_status s);

#ifdef __cplusplus
}
#endif
#endif /* TSQ_H */
