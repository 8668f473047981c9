// Internal declarations shared by the host API and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "shifter.h"

namespace shifter {

constexpr uint32_t TILE = 4096;      // elements per tile of the streaming kernels
constexpr uint32_t BLOCK = 256;      // threads per block (4 wavefronts of 64)
constexpr uint32_t HIST_BINS = 2048; // stride of one histogram slot
constexpr uint32_t MAXK = SHIFTER_MAX_VARIANTS;
constexpr uint32_t SLOTS_PER_PASS = 8;
constexpr uint32_t GATHER_CHUNK = 1024;  // columns of a gather work unit (16 per lane)
constexpr uint32_t GATHER_ROWS = 16;
constexpr uint32_t RECT_ELEMS = 8192;    // floats of a source rectangle staged in LDS by the portfolio rebuild

// Device-side view of one weight tensor.
struct DevTensor {
    uint64_t offset;     // element offset in the weight arena
    uint64_t gbase;      // global index of element 0 (0 if not prunable)
    uint32_t numel;
    uint32_t out_ch, in_ch, khw;
    uint32_t row_len;    // in_ch * khw: elements per filter
    uint32_t kk;         // khw * in_mult: elements per (filter, input channel)
    uint32_t cin;        // in_ch / in_mult: width of the in-group
    uint32_t magic_khw;  // floor(2^32 / khw) + 1 when 1 < khw <= 2 * TILE, else 0
    uint32_t magic_row;  // same for row_len
    uint32_t magic_in;   // same for in_ch
    uint32_t magic_kk, shift_kk;  // any 32-bit x / kk (kk >= 2): see div_u32
    int32_t out_group, in_group;
    uint32_t out_flag_off, in_flag_off;
    uint32_t prunable;
    uint32_t band_rows;   // portfolio rebuild: filters per source rectangle (at most 64)
    uint32_t chunk_ch;    //   in-group channels per source rectangle
    uint32_t src_chunks;  //   rectangles per band of filters: ceil(cin / chunk_ch)
};

struct DevGroup {
    uint32_t width, pinned;
    uint32_t off;        // offset in the per-group arrays
    uint32_t prod_begin, prod_end;  // range in the producer list
    uint32_t pad;
};

struct DevVec {
    uint64_t offset;
    uint32_t len;
    int32_t group;
};

// State of the multi-rank radix select, one entry per requested prune count.
struct SelRank {
    uint64_t rank;     // remaining 1-based rank inside the current prefix; 0: P == 0
    uint64_t n_less;   // weights known to be smaller than every key with this prefix
    uint64_t n_equal;  // weights sharing the prefix
    uint32_t prefix;   // decided high bits of the key, right aligned
    uint32_t slot;     // histogram slot of this prefix in the next round
};

struct SelState {
    SelRank r[MAXK];
    uint32_t slot_prefix[MAXK];
    uint32_t n_slots;
    uint32_t k;
    uint32_t nan_seen;
    uint32_t pad;
};

// State of the single-pass (sample, predict, one pass, finish) selection.
constexpr uint32_t SPEC_SUB = 256;         // split counters / candidate sub-buffers
constexpr uint32_t SPEC_FIN_BLOCKS = 256;  // blocks of the finishing passes
constexpr uint32_t SPEC_LIST_CAP = 65536;  // pairs of the selected round-1 bin
constexpr uint32_t SPEC_SMALL_CAP = 1024;  // pairs of the selected round-2 bin
struct SpecState {
    uint64_t p;          // prune count
    uint64_t r2;         // 1-based rank of the P-th pair inside the selected round-1 bin
    uint64_t less;       // weights below that bin
    uint64_t n_below;    // weights with key < lo
    uint64_t n_inside;   // weights with lo <= key <= hi (the candidates)
    uint32_t lo, hi;     // inclusive key interval of the candidates
    uint32_t mid;        // provisional threshold key of the fused pass, lo <= mid <= hi
    uint32_t sh;         // round-1 bin = (key - lo) >> sh
    uint32_t m_valid;    // sample size
    uint32_t status;     // bit 0: not decided, use the multi-pass select; bit 1: NaN seen
    uint32_t bin, bin_cnt;
    uint32_t list_cnt;
    uint32_t pad;
    shifter_threshold rec;   // copy of the record written to the caller's d_thr (one read-back)
};

// State of the single-pass selection for all prune counts of a portfolio (ranks sorted by
// prune count, zero counts left out).
constexpr uint32_t SPEC_MULTI_MAXK = 32;   // LDS of the fused pass's private counters: 256 B per rank
// What the finish of one rank reads (written by the predict kernel) and what its filter step
// leaves for its last step: one cache line each instead of a line per field.
struct RankIn {
    uint64_t p;
    uint32_t lo, sh;                       // its cluster's interval start; the first histogram's shift (256 bins)
    uint32_t clast, cand_off, cand_cap;    // its cluster's last rank and candidate region
    uint32_t perm;                         // original position of this rank
};
struct RankOut {
    uint64_t r2, less;     // rank of the P-th pair inside the selected bin; weights below that bin
    uint32_t bin, bin_cnt;
    uint32_t fail;         // why the finish gave up (0: it has not)
    uint32_t pad;
};
struct MultiState {
    uint64_t p[MAXK];
    uint32_t perm[MAXK];   // original position of sorted rank k
    uint32_t lo[MAXK], hi[MAXK];   // candidate interval; ranks whose intervals met share one (a cluster)
    uint32_t mid[MAXK];    // predicted threshold key of rank k, lo <= mid <= hi, non-decreasing
    uint32_t clast[MAXK];  // last rank of rank k's cluster: the owner of the cluster's candidate region
    uint32_t cand_off[MAXK], cand_cap[MAXK];   // region of the cluster ending at rank k: first pair, pairs per part
    RankIn rin[MAXK];
    RankOut rout[MAXK];
    uint32_t k, m_valid, status, pad;
};
struct MultiPerm {
    uint32_t v[MAXK];
};

// Conv + BatchNorm fold: element offsets of a tensor's vectors in the vector arena and of
// its folded bias in the bias arena; -1: not present.
struct FoldTensor {
    int64_t gamma, beta, mean, var, bias, out_offset;
};

struct PruneCounts {
    uint64_t p[MAXK];
};

// Device-side rebuild plan (sizes and offsets of the compacted tensors).
struct PlanTensor {
    uint64_t out_off;
    uint32_t o2, c2;     // surviving filters, surviving input channels
    uint32_t numel2;
    uint32_t row2;       // c2 * kk: elements per rebuilt filter
    uint32_t chunks;     // column chunks per row
    uint32_t rb;         // rows per work unit
};

struct PlanVec {
    uint64_t out_off;
    uint32_t len2;
    uint32_t pad;
};

struct PlanHeader {
    uint64_t elems_w, elems_v;
    uint32_t total_units;
    uint32_t status;     // bit 0: capacity exceeded; bit 1: some group collapsed
};

enum KernelId {
    K_SEL_INIT = 0, K_HIST0, K_HIST1, K_HIST2, K_SELECT, K_TIE_COUNT, K_TIE_FINAL,
    K_ZERO_FLAGS, K_MASK_SCAN, K_SCAN, K_PROPAGATE, K_PLAN, K_GATHER,
    K_COPY, K_KERNEL_SCAN, K_FIX_ROUND, K_FOLD_SCALE, K_FOLD_APPLY,
    K_DEFLATE_CHUNK, K_CODEC_SCAN, K_CODEC_PACK, K_INFLATE_CHUNK,
    K_MASK_SCAN_BATCH, K_EXPAND_LEVELS,
    K_SPEC_INIT, K_SPEC_SAMPLE, K_SPEC_PREDICT, K_SPEC_PASS, K_SPEC_FINISH, K_SPEC_FINISH2,
    K_SPEC_FIXUP, K_SPEC_RANK,
    K_COUNT
};
extern const char* const kKernelNames[K_COUNT];

}  // namespace shifter

namespace shifter {
// Device buffers of one portfolio step (shifter_portfolio_begin's arguments, checked).
struct PortfolioBuffers {
    const float* d_w; const float* d_vecs;
    uint32_t k_var, flags;
    shifter_threshold* d_thr;
    float* d_w_sparse; uint64_t w_stride;          // or nullptr
    uint8_t* d_mask; uint64_t mask_stride;         // or nullptr
    uint8_t* d_out_alive; uint8_t* d_in_alive;     // in: or nullptr
    uint8_t* d_group_alive; int32_t* d_index_map; uint32_t* d_keep; uint32_t* d_new_width;
    float* d_w_out; uint64_t cap_w; float* d_vecs_out; uint64_t cap_v;
};
}  // namespace shifter

struct shifter_model {
    std::vector<shifter_tensor_desc> t;
    std::vector<shifter_vec_desc> v;
    std::vector<shifter_group_desc> g;
    shifter_model_info info{};
    std::vector<shifter::DevTensor> dt;
    std::vector<shifter::DevGroup> dg;
    std::vector<shifter::DevVec> dv;
    std::vector<uint32_t> producers;     // tensor indices, grouped by out_group
    std::vector<uint32_t> tile_prefix;   // n_tensors + 1
    std::vector<uint64_t> out_flag_off, in_flag_off, group_off;
    uint32_t n_tiles = 0;
    std::vector<uint32_t> ranked_ids;    // indices of the prunable tensors, in order
    uint32_t n_ranked = 0;
    uint32_t sample_tile_stride = 1;     // every how many tiles the selection samples
    uint32_t sample_size = 0;            // weights in that sample
    uint32_t gather_units_bound = 0;     // gather work units when nothing is removed
    // portfolio rebuild: per tensor prefix sums of its source rectangles, of its row-table
    // entries (bands + 1) and of its column-table entries (src_chunks + 1)
    std::vector<uint32_t> rect_prefix, rowtab_prefix, coltab_prefix;
    bool rect_ok = true;                 // every tensor has kk <= GATHER_CHUNK
    // liveness fixpoint: offset of every tensor's [out_ch][in_ch] block in the kernel
    // index, its size, tiles of that index per tensor (prefix sums), consumers per group
    std::vector<uint64_t> kernel_off;
    uint64_t sum_kernels = 0;
    std::vector<uint32_t> fix_prefix, cons_prefix, consumers;

    // device side, created by the first call that uses the model with a context
    struct Bound {
        shifter_ctx* ctx = nullptr;
        uint64_t ctx_id = 0;                  // that context's id: an address alone may be reused
        int device = 0;
        shifter::DevTensor* tens = nullptr;
        shifter::DevGroup* groups = nullptr;
        shifter::DevVec* vecs = nullptr;
        uint32_t* producers = nullptr;
        uint32_t* tile_prefix = nullptr;
        uint16_t* tile_tensor = nullptr;      // n_tiles: tensor of every tile
        shifter::SelState* sel = nullptr;
        uint32_t* ghist = nullptr;       // MAXK * HIST_BINS
        uint32_t* tile_cnt = nullptr;    // MAXK * n_tiles
        shifter::PlanTensor* plan_t = nullptr;
        shifter::PlanVec* plan_v = nullptr;
        shifter::PlanHeader* plan_h = nullptr;
        uint32_t* out_tile_prefix = nullptr;  // MAXK * (n_tensors + 1)
        uint32_t* rect_prefix = nullptr;      // n_tensors + 1 each
        uint32_t* rowtab_prefix = nullptr;
        uint32_t* coltab_prefix = nullptr;
        uint32_t* rowtab = nullptr;           // MAXK * rowtab_prefix.back()
        uint32_t* coltab = nullptr;           // MAXK * coltab_prefix.back()
        uint32_t* levels = nullptr;           // sum_out_ch + sum_in_ch
        uint64_t* kernel_off = nullptr;       // n_tensors
        uint32_t* fix_prefix = nullptr;       // n_tensors + 1
        uint32_t* cons_prefix = nullptr;      // n_groups + 1
        uint32_t* consumers = nullptr;        // tensor indices, grouped by in_group
        uint8_t* fix_alive = nullptr;         // sum_group_width
        uint8_t* fix_produced = nullptr;      // sum_out_ch
        uint8_t* fix_read = nullptr;          // sum_in_ch
        uint8_t* fix_out_flags = nullptr;     // sum_out_ch
        uint32_t* fix_removed = nullptr;      // FIX_STATE_WORDS: per-round counters of a batch, rounds so far
        shifter::FoldTensor* fold = nullptr;  // n_tensors
        std::vector<shifter::FoldTensor> fold_host;   // the layer table the device holds (empty: none yet)
        float* fold_scale = nullptr;          // sum_out_ch
        shifter::SpecState* spec = nullptr;
        uint32_t* shist = nullptr;            // 65536 sample bins
        uint32_t* spec_cnt = nullptr;         // 2 * SPEC_SUB counters, one 128-byte line each
        uint32_t* partial = nullptr;          // SPEC_FIN_BLOCKS * 256 partial histograms
        uint2* cand = nullptr;                // SPEC_SUB sub-buffers of (key, g) pairs
        uint32_t cand_cap_sb = 0;             // pairs per sub-buffer
        uint2* list = nullptr;                // SPEC_LIST_CAP pairs
        uint32_t* ranked_ids = nullptr;
        shifter::MultiState* multi = nullptr;
        uint32_t* multi_cnt = nullptr;        // (2 * MAXK + 1) * SPEC_SUB counters, 128-byte lines
        uint8_t* multi_tab = nullptr;         // 4096 bucket entries of the K-rank pass
        uint32_t* multi_hist = nullptr;       // MAXK * 256: the clusters' first histograms
        uint64_t* multi_rowsum = nullptr;     // MAXK + 1: totals of the split counters' rows
        uint2* multi_list = nullptr;          // SPEC_MULTI_MAXK * SPEC_LIST_CAP pairs: the ranks' selected bins
        uint32_t* multi_list_cnt = nullptr;   // MAXK
        uint32_t* below = nullptr;            // MAXK * (sum_group_width + n_groups): survivors below a channel
        uint8_t* host_stage = nullptr;        // pinned, for small read-backs
        // pinned mirrors of the one-count selection's state, written by its last kernel: one
        // for calls that wait themselves, one for a deferred call (host and device addresses)
        uint8_t* host_spec = nullptr;
        uint8_t* host_spec_now = nullptr;
        shifter::SpecState* dev_spec = nullptr;
        shifter::SpecState* dev_spec_now = nullptr;
        // pinned mirrors the kernels write themselves (no copy on the stream): the K-rank
        // ranking's status words (MAXK) and records (MAXK), and the packed plans of MAXK variants
        uint8_t* host_multi = nullptr;
        uint32_t* dev_multi_status = nullptr;       // device addresses of the same memory
        shifter_threshold* dev_multi_rec = nullptr;
        uint8_t* host_plan = nullptr;
        uint8_t* dev_plan = nullptr;
        uint32_t* host_width = nullptr;       // n_groups: the fixpoint plan's widths
        uint32_t* dev_width = nullptr;
        size_t host_stage_bytes = 0;
    } b;
};

struct shifter_ctx {
    uint64_t id = 0;       // unique per shifter_create in this process
    int device = 0;
    hipStream_t stream = nullptr;
    uint8_t* static_scratch = nullptr;   // this device's copy of the library's static scratch array
    std::string err;
    bool profiling = false;
    struct Rec { int id; hipEvent_t a, b; };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    uint32_t hist_grid = 2048;
    int select_path = 0;   // 0: single-pass where it applies; 1: multi-pass radix only
    double margin_sigmas = 4.0;   // half-width of the predicted interval, in binomial sigmas
    uint64_t fused_min_bytes = 192ull << 20;   // portfolio_begin: arenas above this take the fused pass
    shifter::SpecState last_spec{};  // outcome of the last single-pass selection
    int last_path = 0;               // 1: single pass decided; 2: multi-pass select ran
    shifter_threshold last_record{};  // record of the last shifter_prune_fused that waited
    uint64_t* d_codec = nullptr;      // codec: [0] stream bytes, [1] status bits, [2], [3] list lengths (device)
    uint64_t* h_codec = nullptr;      // pinned mirror of the first two, written by the call's last kernel
    uint64_t* dev_codec_mirror = nullptr;   //   its device address
    uint32_t* d_codec_list = nullptr; // chunk lists of the instances that take the longer segments
    uint64_t codec_list_cap = 0;      //   its capacity in entries
    bool codec_dirty = true;          // the codec's result words may be non-zero (see codec_begin)
    // a shifter_prune_fused call whose outcome has not been collected yet
    struct Pending {
        bool active = false;
        const shifter_model* model = nullptr;
        const float* d_w = nullptr;
        uint64_t n_prune = 0;
        shifter_threshold* d_thr = nullptr;
        float* d_w_out = nullptr;
        uint8_t* d_mask = nullptr;
        uint8_t* d_out_alive = nullptr;
        uint8_t* d_in_alive = nullptr;
    } pending;
    // a shifter_global_threshold_begin whose outcome has not been collected yet
    struct PendingRank {
        bool active = false;
        const shifter_model* model = nullptr;
        const float* d_w = nullptr;
        shifter::PruneCounts pc{};
        uint32_t k = 0, k_eff = 0;   // counts asked for; counts above zero (single pass)
        shifter_threshold* d_thr = nullptr;
        bool single_pass = false;
    } pending_rank;
    // a shifter_portfolio_begin whose outcome has not been collected yet
    struct PendingPortfolio {
        bool active = false;
        const shifter_model* model = nullptr;
        shifter::PortfolioBuffers buf{};
        shifter::PruneCounts pc{};
        uint32_t k_eff = 0;
        int mode = 0;    // 1: one-count single pass; 2: K-rank single pass; 3: multi-pass select
    } pending_portfolio;
};

namespace shifter {

// Launchers (defined next to their kernels).  All enqueue on ctx->stream.
void launch_select(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                   const PruneCounts& pc, uint32_t k, shifter_threshold* d_thr);
// The tables and scratch the multi-pass select works on: a model's, or the ones laid out in
// the static scratch array for one flat run of weights.
struct SelectTables {
    const DevTensor* tens;
    const uint32_t* tile_prefix;
    uint32_t n_t, n_tiles;
    SelState* sel;
    uint32_t* ghist;      // MAXK * HIST_BINS
    uint32_t* tile_cnt;   // k * n_tiles
};
void launch_select_tables(shifter_ctx* ctx, const SelectTables& tb, const float* d_w,
                          const PruneCounts& pc, uint32_t k, shifter_threshold* d_thr);
// Layout of the static scratch array used by shifter_global_threshold_static (byte offsets
// from its 256-byte aligned start) and the limits that follow from its size.
constexpr uint64_t STATIC_MAX_WEIGHTS = 1ull << 28;       // weights of one flat run
constexpr uint64_t STATIC_MAX_TILE_COUNTS = 1ull << 20;   // K * tiles of the run
constexpr size_t STATIC_OFF_TENSOR = 0;
constexpr size_t STATIC_OFF_PREFIX = 256;
constexpr size_t STATIC_OFF_SEL = 512;
constexpr size_t STATIC_OFF_GHIST = STATIC_OFF_SEL + ((sizeof(SelState) + 255) / 256) * 256;
constexpr size_t STATIC_OFF_TILE_CNT = STATIC_OFF_GHIST + sizeof(uint32_t) * MAXK * HIST_BINS;
constexpr size_t STATIC_SCRATCH_BYTES = STATIC_OFF_TILE_CNT + sizeof(uint32_t) * STATIC_MAX_TILE_COUNTS;
static_assert(sizeof(DevTensor) <= 256, "the one-tensor table fits its slot");
// Writes the one-tensor table of a flat run of n weights (one prunable tensor at offset 0).
void launch_flat_tables(shifter_ctx* ctx, DevTensor* tens, uint32_t* tile_prefix, uint64_t n);
// host_mirror: device address of the pinned SpecState the last kernel leaves the outcome in.
void launch_spec_select(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint64_t p,
                        shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                        uint8_t* d_out_alive, uint8_t* d_in_alive, SpecState* host_mirror);
// Scratch of the K-rank ranking that the sample kernel clears on the way (cnt == nullptr:
// nothing): the split counters' rows in use, the clusters' histograms, the list lengths
// and the finish's per-rank outcome.
struct SampleZero {
    uint32_t* cnt = nullptr;
    uint32_t k = 0;
    uint32_t* ghist = nullptr;
    uint32_t* list_cnt = nullptr;
    RankOut* rout = nullptr;
    uint32_t* extra = nullptr;     // one more array of extra_n words to clear
    uint32_t extra_n = 0;
    // the one-count selection: its state to set up, its split counters and the caller's
    // flag arrays to clear (ss == nullptr: not this call)
    shifter::SpecState* ss = nullptr;
    uint32_t* cnt1 = nullptr;
    uint64_t p = 0;
    uint32_t m_valid = 0;
    uint8_t* fa = nullptr;
    uint8_t* fb = nullptr;
    uint64_t na = 0, nb = 0;
};
void launch_spec_sample(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                        const SampleZero& z = SampleZero());
// Outputs of the fused portfolio pass (steps 1-3 in one read): k_all variants in caller order.
struct FusedBatch {
    uint32_t k_all;
    float* d_w_out;          // or nullptr
    uint64_t w_stride;
    uint8_t* d_mask;         // or nullptr
    uint64_t mask_stride;
    uint8_t* d_out_alive;
    uint8_t* d_in_alive;     // or nullptr
    bool levels_only = false;   // leave the levels unexpanded: the planning launch behind it writes the flags
};
// zero_ptr / zero_n: an array of 32-bit words the ranking's set-up clears on the way (or
// nullptr), for the step that follows it.
void launch_spec_multi(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                       const shifter::PruneCounts& sorted_p, const shifter::MultiPerm& perm,
                       uint32_t k, uint64_t zero_mask, shifter_threshold* d_thr,
                       const FusedBatch* fb, uint32_t* zero_ptr = nullptr, uint32_t zero_n = 0);
constexpr size_t MULTI_MIRROR_REC_OFF = 512;   // records follow the MAXK status words
// The liveness fixpoint enqueues its rounds in batches of FIX_BATCH with no wait inside a
// batch; its state on the device is removed[0 .. FIX_BATCH] and the rounds run so far, and
// (rounds, settled) go to two words of the status mirror behind the MAXK status words.
constexpr uint32_t FIX_BATCH = 4;
constexpr uint32_t FIX_STATE_WORDS = FIX_BATCH + 2;
constexpr uint32_t FIX_MIRROR_WORD = 64;
constexpr uint32_t FIX_ENQUEUED_BATCHES = 4;   // of a call that may not wait
static_assert(MAXK <= FIX_MIRROR_WORD && (FIX_MIRROR_WORD + 2) * 4 <= MULTI_MIRROR_REC_OFF, "mirror layout");
void launch_zero_levels(shifter_ctx* ctx, const shifter_model* m);
void launch_expand_levels(shifter_ctx* ctx, const shifter_model* m, const shifter_threshold* d_thr,
                          uint32_t k_var, uint8_t* d_out_alive, uint8_t* d_in_alive);
void launch_mask_scan(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                      const shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                      uint8_t* d_out_alive, uint8_t* d_in_alive);
void launch_scan(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                 uint8_t* d_out_alive, uint8_t* d_in_alive);
void launch_mask_scan_batch(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                            const shifter_threshold* d_thr, uint32_t k_var, float* d_w_out,
                            uint64_t w_stride, uint8_t* d_mask, uint64_t mask_stride,
                            uint8_t* d_out_alive, uint8_t* d_in_alive);
void launch_propagate(shifter_ctx* ctx, const shifter_model* m, const uint8_t* d_out_alive,
                      uint32_t flags, uint8_t* d_group_alive, int32_t* d_index_map,
                      uint32_t* d_keep, uint32_t* d_new_width, uint32_t k_var);
void launch_compact(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint64_t w_stride,
                    const float* d_vecs, const uint32_t* d_keep,
                    const uint32_t* d_new_width, float* d_w_out, uint64_t cap_w,
                    float* d_vecs_out, uint64_t cap_v, uint32_t k_var,
                    const shifter_threshold* d_thr);
// pos[k] = number of variants that remove fewer weights than variant k (ties by index).
void launch_plan_and_gather(shifter_ctx* ctx, const shifter_model* m, const PortfolioBuffers& a,
                            bool from_levels, const MultiPerm& pos);
// The batched mask pass alone: with_zero clears the level arrays first, with_expand turns
// them into the variants' flag bytes afterwards.
void launch_mask_scan_batch_core(shifter_ctx* ctx, const shifter_model* m, const float* d_w,
                                 const shifter_threshold* d_thr, uint32_t k_var, float* d_w_out,
                                 uint64_t w_stride, uint8_t* d_mask, uint64_t mask_stride);
void launch_copy(shifter_ctx* ctx, const float* src, float* dst, uint64_t n);
void launch_kernel_scan(shifter_ctx* ctx, const shifter_model* m, const float* d_w, uint8_t* d_nz);
void launch_fix_begin(shifter_ctx* ctx, const shifter_model* m);
void launch_fix_batch(shifter_ctx* ctx, const shifter_model* m, const uint8_t* d_nz, uint32_t flags);
void launch_fix_widths(shifter_ctx* ctx, const shifter_model* m, const uint32_t* d_new_width);
// Codec workspace: segment sizes (u32 per chunk) first, then one slot per chunk.
inline uint64_t codec_slots_offset(uint64_t n_chunks) { return (n_chunks * 4u + 255u) & ~(uint64_t)255u; }
int launch_deflate(shifter_ctx* ctx, const uint8_t* d_in, uint64_t n_bytes, uint32_t n_chunks,
                   uint8_t* d_work, uint8_t* d_stream, uint64_t stream_cap, uint64_t* d_seg_off,
                   uint16_t* d_sub_bits, uint64_t* d_sub_marks);
int launch_inflate(shifter_ctx* ctx, const uint8_t* d_stream, uint64_t stream_bytes,
                   const uint64_t* d_seg_off, const uint16_t* d_sub_bits, const uint64_t* d_sub_marks,
                   uint64_t n_bytes, uint32_t n_chunks, uint8_t* d_out);
void launch_fold(shifter_ctx* ctx, const shifter_model* m, const float* d_w, const float* d_vecs,
                 float eps, float* d_w_out, float* d_bias_out);

// Event bracketing for per-kernel timing.
struct ProfileScope {
    shifter_ctx* ctx;
    int idx;
    ProfileScope(shifter_ctx* c, int id);
    ~ProfileScope();
};

}  // namespace shifter
