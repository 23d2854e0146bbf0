// Shared between the host API (tsq_api.hip) and the kernels (tsq_kernels.hip).
// Plain data only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsq {

constexpr uint32_t kMagic   = 0x31515354u;   // "TSQ1", little-endian
constexpr uint32_t kVersion = 1;

constexpr int kRun      = 32;   // elements owned by one lane (a "run")
constexpr int kRunLdsDw = 20;   // dwords one run occupies in LDS: 16 of data + 4 of padding,
                                // so that 8 lanes reading 16 B each hit 32 distinct banks
constexpr int kMaxWaves = 16;   // 1024 threads per workgroup at most
// LDS scratch of the staged row kernels behind the row: four reduce areas (2 dwords per wave
// each) and one scan area
constexpr uint32_t kScratchDw = 4 * 2 * kMaxWaves + kMaxWaves;
constexpr uint32_t kMaxHidden = 32768;
// fused kernel: outliers of one token and wave that fit the wave's LDS stash (a wave with more takes
// a slower path), the largest grid, the ticket classes (one counter line each, kTicketStride
// dwords apart so that no two share a 256-byte line), and its LDS behind the row and the two
// payload images in dwords (four reduce areas, ticket slots; the stashes follow: 2 per wave)
constexpr uint32_t kStashWave = 232;
constexpr uint32_t kFusedGridCap = 4096;
constexpr uint32_t kTicketClasses = 64, kTicketStride = 64;
constexpr uint32_t kFusedScratchDw = 4 * 2 * kMaxWaves + 8;
// words of a workspace's control block
constexpr uint32_t kCtlError = 1, kCtlTokens = 2, kCtlHidden = 3;

// 128-byte header at the start of every blob.
struct BlobHeader {
    uint32_t magic, version, dtype, tokens, hidden, tau_bits, bit_mask, budget_bits, mode, status;
    uint64_t nnz, payload_bytes;
    uint64_t off_bits, off_scale, off_pay_off, off_row_ptr, off_payload, off_out_col, off_out_val;
    uint64_t payload_capacity, outlier_capacity;
};
static_assert(sizeof(BlobHeader) == 128, "blob header must be 128 bytes");

// Entropy-coded payload ("eblob"): 256-byte header | frequency tables u16[7][256] (row b-2: width b) |
// stream offsets u64[T+1] (bytes from the start of the streams) | the tokens' streams.
constexpr uint32_t kEntropyMagic = 0x45515354u;   // "TSQE"
struct EntropyHeader {
    uint32_t magic, version, tokens, hidden;
    uint64_t stream_bytes;                          // sum of the tokens' streams
    uint64_t off_tables, off_stream_off, off_streams, stream_capacity;
    uint64_t reserved[25];
};
static_assert(sizeof(EntropyHeader) == 256, "entropy header must be 256 bytes");
// Sections of the eblob and of the encoder's workspace (bytes), fixed by the plan.
struct EntropyLayout {
    uint64_t off_tables, off_stream_off, off_streams, stream_capacity, eblob_bytes;
    uint64_t ws_pooled;     // u32[kPoolCopies][7][256] code counts per width class (a counting workgroup adds to set id % kPoolCopies)
    uint64_t ws_block;      // u32[ceil(T / kLenBlock)][kBlockStride], word 0 of each: padded stream bytes of the block of kLenBlock tokens
    uint64_t ws_len;        // u32[T] stream bytes per token
    uint64_t ws_slots;      // T slots of slot_bytes: the streams before they are moved together
    uint64_t ws_bytes;
    uint32_t slot_bytes;    // 256 (states) + 2 bytes per element (rounded up to 4): the longest possible stream
    uint32_t pool_groups;   // workgroups of k_code_pool
    uint32_t pool_tokens;   // consecutive tokens each of them counts
    uint32_t pad;
};
constexpr uint32_t kLenBlock = 256;     // tokens per partial sum of stream lengths
constexpr uint32_t kBlockStride = 64;   // 32-bit words from one partial sum to the next: the encoder's waves add to them, and
                                        // adds to one 128-byte line from all over the chip hold up the stores queued behind them
constexpr uint32_t kMaxPoolGroups = 512;    // counting workgroups of 1024 threads: two fit a compute unit, 256 compute units: one round
constexpr uint32_t kPoolCopies = 16;    // sets of pooled counts: 16 times fewer atomic adds per address

// Kernel argument block (passed by value).
struct Params {
    uint32_t tokens, hidden;
    uint32_t runs;          // ceil(hidden / 32): lanes that own data in a row
    uint32_t pieces;        // hidden / 8: 16-byte pieces in a row
    uint32_t dtype;
    uint32_t thr_pk;        // smallest 16-bit magnitude pattern with value >= tau, in both halves
    uint32_t bit_mask;
    uint32_t n_widths;      // number of allowed widths
    uint32_t return_failing;  // Algorithm 1 returns the width that failed the test (1) or the last that passed (0)
    uint64_t widths_pk;     // allowed widths, descending, one per byte (byte 0 = largest)
    double   test_rhs[8];   // Algorithm 1's test for candidate i (descending widths): everything of its right-hand side
                            // that does not depend on the token, computed on the host in the very sequence of binary64
                            // operations that defines the test.  REL_RMS: ((double)budget * (double)Q_i)^2 * (double)H, to be
                            // multiplied by (double)SS0; LSB: (double)budget * (double)H
    float    tau;
    float    budget;
    int32_t  mode;
    uint32_t spin_limit;    // bound on every device-side wait (fused pipeline)
    uint64_t off_bits, off_scale, off_pay_off, off_row_ptr, off_payload, off_out_col, off_out_val;
    uint64_t payload_capacity, outlier_capacity;
    // workspace sections (bytes from d_ws)
    uint64_t ws_cnt;        // u32[T]  outliers per token           (staged)
    uint64_t ws_amax;       // f32[T]  inlier absmax per token      (staged)
    uint64_t ws_sizes;      // u32[T]   published (tag, words, count) of every token   (fused)
    uint64_t ws_prefix;     // u64[T+1] (tag, words before, outliers before) of every token, from the scanner (fused)
    uint64_t ws_tickets;    // u32[kTicketClasses][kTicketStride] per class: epoch << 24 | tickets drawn, waves done (fused)
    uint64_t ws_ctrl;       // u32[64]  at the start of every workspace: word kCtlError = a call on it failed (fused);
                            //          words kCtlTokens, kCtlHidden = the shape it was reset for
    uint32_t fused_classes; // ticket classes in use: min(kTicketClasses, computing workgroups; set per call) (fused)
    uint32_t rows_per_tensor;  // 0: the rows form one contiguous tensor.  Otherwise the data pointer of a
                               // call is a device table of tensor pointers, rows_per_tensor rows each
                               // (set per call from a copy of the plan's block)
};

// Row t of the input / output of a call (see Params::rows_per_tensor).  t must be uniform.
template <typename T16>
__device__ __forceinline__ T16 *row_address(const Params &p, T16 *base, uint32_t t, uint32_t hidden) {
    if (p.rows_per_tensor == 0) return base + (size_t)t * hidden;
    T16 *const *table = reinterpret_cast<T16 *const *>(base);
    const uint32_t k = t / p.rows_per_tensor;
    return table[k] + (size_t)(t - k * p.rows_per_tensor) * hidden;
}

inline __host__ __device__ uint32_t width_at(const Params &p, uint32_t i) {
    return (uint32_t)(p.widths_pk >> (8u * i)) & 0xFFu;
}

// Launch geometry fixed by the plan.
struct Geometry {
    uint32_t block;         // threads per workgroup of unpack = 64 * ceil(runs / 64)
    uint32_t lds_bytes;     // dynamic LDS of the staged row kernels and of unpack
    uint32_t waves;         // waves per workgroup of the compress kernels (an instantiated size >= block / 64)
    uint32_t lds_fused_bytes;  // dynamic LDS of the fused kernel: row, scratch, outlier stash
};

// launchers implemented in tsq_kernels.hip; each returns a hipError_t as int
int launch_row_stats(const Params &p, const Geometry &g, const void *d_in, void *d_blob, void *d_ws,
                     void *stream);
int launch_scan(const Params &p, void *d_blob, void *d_ws, void *stream);
int launch_pack(const Params &p, const Geometry &g, const void *d_in, void *d_blob, void *d_ws,
                void *stream);
int launch_fused(const Params &p, const Geometry &g, uint32_t grid, const void *d_in, void *d_blob,
                 void *d_ws, void *stream);
uint32_t compress_waves(uint32_t runs);
int fused_resident_workgroups(const Params &p, const Geometry &g, uint32_t *out);
int prepare_fused_kernels();
int launch_ws_reset(const Params &p, void *d_ws, void *stream);
int launch_unpack(const Params &p, const Geometry &g, const void *d_blob, void *d_out, void *stream);
int launch_code_hist(const Params &p, const Geometry &g, const void *d_blob, void *d_hist, void *stream);
int launch_code_pool(const Params &p, const Geometry &g, const EntropyLayout &e, const void *d_blob, void *d_counts,
                     void *stream);
int launch_rans_encode(const Params &p, const Geometry &g, const EntropyLayout &e, const void *d_blob, void *d_eblob,
                       void *d_ews, void *stream);
int launch_rans_decode(const Params &p, const EntropyLayout &e, const void *d_eblob, void *d_blob, void *stream);
int launch_plain_copy(void *d_dst, const void *d_src, size_t bytes, void *stream);     // measurement aids
int launch_plain_read(const void *d_src, size_t bytes, void *d_sink, void *stream);
int prepare_kernels();  // raises the dynamic-LDS limit of the row kernels once per process

}  // namespace tsq
