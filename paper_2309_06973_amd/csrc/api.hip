// Host side of the C ABI: descriptor validation, device tables and scratch, argument
// checks, stream-ordered launches and the small read-backs the ABI documents.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "internal.h"

using namespace shifter;

namespace shifter {
const char* const kKernelNames[K_COUNT] = {
    "sel_init", "hist_round0", "hist_round1", "hist_round2", "select", "tie_count", "tie_final",
    "zero_flags", "mask_scan", "scan", "propagate", "plan", "gather",
    "copy", "kernel_scan", "fix_round", "fold_scale", "fold_apply",
    "deflate_chunk", "codec_scan", "codec_pack", "inflate_chunk",
    "mask_scan_batch", "expand_levels",
    "spec_init", "spec_sample", "spec_predict", "spec_pass", "spec_hist_locate", "spec_filter_rank",
    "spec_fixup", "spec_rank"};

ProfileScope::ProfileScope(shifter_ctx* c, int id) : ctx(c), idx(-1) {
    if (!c->profiling) return;
    hipEvent_t a = nullptr, b = nullptr;
    if (c->pool.size() >= 2) {
        a = c->pool.back(); c->pool.pop_back();
        b = c->pool.back(); c->pool.pop_back();
    } else if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        return;
    }
    (void)hipEventRecord(a, c->stream);
    c->recs.push_back({id, a, b});
    idx = (int)c->recs.size() - 1;
}
ProfileScope::~ProfileScope() {
    if (idx >= 0) (void)hipEventRecord(ctx->recs[idx].b, ctx->stream);
}
}  // namespace shifter

static thread_local std::string g_err;

// Scratch of shifter_global_threshold_static: the tables, histograms and per-tile counts of
// the multi-pass select for one flat run of weights, in a file-scope device array instead
// of allocated memory.  Every device the library runs on holds its own copy at its own
// address; the name below is only a host-side handle for hipGetSymbolAddress, never a
// pointer to pass to a kernel or a copy.
static __device__ __align__(256) uint8_t scratch[shifter::STATIC_SCRATCH_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
static uint8_t* g_static_ptr[STATIC_MAX_DEVICES];   // device address of `scratch`, per device
static std::mutex g_static_mutex;

// Device address of this device's copy of the scratch array, resolved once per device with
// that device current.
static hipError_t static_scratch_address(int device, uint8_t** out) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (device < 0 || device >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    if (!g_static_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_static_ptr[device] = static_cast<uint8_t*>(p);
    }
    *out = g_static_ptr[device];
    return hipSuccess;
}

static int fail(shifter_ctx* ctx, int code, const std::string& msg) {
    g_err = msg;
    if (ctx) ctx->err = msg;
    return code;
}

#define HIP_TRY(ctx, expr)                                                              \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess)                                                           \
            return fail(ctx, e_ == hipErrorOutOfMemory ? SHIFTER_ERR_OOM : SHIFTER_ERR_HIP, \
                        std::string(#expr) + ": " + hipGetErrorString(e_));             \
    } while (0)

extern "C" const char* shifter_last_error(const shifter_ctx* ctx) {
    return ctx ? ctx->err.c_str() : g_err.c_str();
}

static void destroy_codec_objects(shifter_ctx* c) {
    if (c->d_codec) (void)hipFree(c->d_codec);
    if (c->h_codec) (void)hipHostFree(c->h_codec);
    if (c->d_codec_list) (void)hipFree(c->d_codec_list);
}

extern "C" int shifter_create(shifter_ctx** out, int device, void* hip_stream) {
    if (!out) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "shifter_create: out is NULL");
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return fail(nullptr, SHIFTER_ERR_NO_DEVICE, "shifter_create: no HIP device visible");
    }
    if (device < 0 || device >= n)
        return fail(nullptr, SHIFTER_ERR_NO_DEVICE, "shifter_create: device ordinal out of range");
    HIP_TRY(nullptr, hipSetDevice(device));
    shifter_ctx* c = new (std::nothrow) shifter_ctx();
    if (!c) return fail(nullptr, SHIFTER_ERR_OOM, "shifter_create: host allocation failed");
    static std::atomic<uint64_t> next_id{1};
    c->id = next_id.fetch_add(1);
    c->device = device;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    {
        const hipError_t e = static_scratch_address(device, &c->static_scratch);
        if (e != hipSuccess) {
            delete c;
            return fail(nullptr, SHIFTER_ERR_HIP,
                        std::string("shifter_create: hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
        }
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
        c->hist_grid = (uint32_t)prop.multiProcessorCount * 8u;
    // result words of the codec calls (stream size, status): on the device, and a pinned
    // mirror the last kernel of a call writes
    void* mirror_dev = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&c->d_codec), 4 * sizeof(uint64_t)) != hipSuccess ||
        hipHostMalloc(reinterpret_cast<void**>(&c->h_codec), 4 * sizeof(uint64_t),
                      hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess ||
        hipHostGetDevicePointer(&mirror_dev, c->h_codec, 0) != hipSuccess) {
        (void)hipGetLastError();
        destroy_codec_objects(c);
        delete c;
        return fail(nullptr, SHIFTER_ERR_OOM, "shifter_create: allocation failed");
    }
    c->dev_codec_mirror = static_cast<uint64_t*>(mirror_dev);
    memset(c->h_codec, 0, 4 * sizeof(uint64_t));
    *out = c;
    return SHIFTER_OK;
}

static void unbind(shifter_model* m) {
    auto& b = m->b;
    if (!b.ctx) return;
    (void)hipSetDevice(b.device);
    void* ptrs[] = {b.tens, b.groups, b.vecs, b.producers, b.tile_prefix, b.tile_tensor, b.sel,
                    b.ghist, b.tile_cnt, b.plan_t, b.plan_v, b.plan_h,
                    b.out_tile_prefix, b.rect_prefix, b.rowtab_prefix, b.coltab_prefix, b.rowtab,
                    b.coltab, b.kernel_off, b.fix_prefix, b.cons_prefix, b.consumers, b.fix_alive,
                    b.fix_produced, b.fix_read, b.fix_out_flags, b.fix_removed, b.fold,
                    b.fold_scale, b.levels, b.spec, b.shist, b.spec_cnt, b.partial, b.cand, b.list,
                    b.ranked_ids, b.multi, b.multi_cnt, b.multi_tab, b.below, b.multi_hist,
                    b.multi_list, b.multi_list_cnt, b.multi_rowsum};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (b.host_stage) (void)hipHostFree(b.host_stage);
    if (b.host_spec) (void)hipHostFree(b.host_spec);
    if (b.host_spec_now) (void)hipHostFree(b.host_spec_now);
    if (b.host_multi) (void)hipHostFree(b.host_multi);
    if (b.host_plan) (void)hipHostFree(b.host_plan);
    if (b.host_width) (void)hipHostFree(b.host_width);
    b = shifter_model::Bound();
}

extern "C" int shifter_destroy(shifter_ctx* ctx) {
    if (!ctx) return SHIFTER_OK;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& r : ctx->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : ctx->pool) (void)hipEventDestroy(e);
    destroy_codec_objects(ctx);
    delete ctx;
    return SHIFTER_OK;
}

// (magic, shift) with x / d == (((x - mulhi(x, magic)) >> 1) + mulhi(x, magic)) >> shift
// for every 32-bit x, d >= 2 (the round-up method of division by an invariant integer).
static void magic_u32(uint32_t d, uint32_t* magic, uint32_t* shift) {
    uint32_t l = 31;
    while (!(d >> l)) --l;              // floor(log2 d)
    if ((d & (d - 1)) == 0) { *magic = 0; *shift = l - 1; return; }
    uint64_t pm = (1ull << (32 + l)) / d;
    const uint64_t rem = (1ull << (32 + l)) - pm * d;
    pm *= 2;
    if (2 * rem >= d) pm += 1;
    *magic = (uint32_t)(pm + 1);
    *shift = l;
}

static uint32_t magic_for(uint32_t d) {
    if (d <= 1 || d > 2 * TILE) return 0;
    return (uint32_t)((1ull << 32) / d) + 1u;
}

extern "C" int shifter_model_create(const shifter_tensor_desc* tensors, uint32_t n_tensors,
                                    const shifter_vec_desc* vecs, uint32_t n_vecs,
                                    const shifter_group_desc* groups, uint32_t n_groups,
                                    shifter_model** out) {
    if (!out) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "model_create: out is NULL");
    *out = nullptr;
    if (!tensors || !groups || n_tensors == 0 || n_groups == 0 || (n_vecs && !vecs))
        return fail(nullptr, SHIFTER_ERR_INVALID_ARG,
                    "model_create: tensors and groups must be non-empty, non-NULL");
    if (n_tensors > 65535u)
        return fail(nullptr, SHIFTER_ERR_BAD_MODEL, "model_create: more than 65535 tensors");
    char buf[256];
    shifter_model* m = new (std::nothrow) shifter_model();
    if (!m) return fail(nullptr, SHIFTER_ERR_OOM, "model_create: host allocation failed");
    auto bad = [&](const char* what, uint32_t idx) {
        snprintf(buf, sizeof buf, "model_create: %s (index %u)", what, idx);
        delete m;
        return fail(nullptr, SHIFTER_ERR_BAD_MODEL, buf);
    };
    m->t.assign(tensors, tensors + n_tensors);
    m->g.assign(groups, groups + n_groups);
    if (n_vecs) m->v.assign(vecs, vecs + n_vecs);

    uint64_t goff = 0;
    m->dg.resize(n_groups);
    for (uint32_t g = 0; g < n_groups; ++g) {
        if (groups[g].width == 0) return bad("group of width 0", g);
        m->group_off.push_back(goff);
        m->dg[g].width = groups[g].width;
        m->dg[g].pinned = groups[g].pinned ? 1u : 0u;
        m->dg[g].off = (uint32_t)goff;
        goff += groups[g].width;
        if (goff >= (1ull << 32)) return bad("sum of group widths reaches 2^32", g);
    }
    uint64_t gbase = 0, so = 0, si = 0, w_ext = 0, w_el = 0, tiles = 0;
    m->dt.resize(n_tensors);
    std::vector<std::pair<uint64_t, uint64_t>> spans;
    for (uint32_t i = 0; i < n_tensors; ++i) {
        const shifter_tensor_desc& t = tensors[i];
        if (!t.out_ch || !t.in_ch || !t.kh || !t.kw || !t.in_mult) return bad("zero-sized tensor dimension", i);
        if (t.out_group < 0 || (uint32_t)t.out_group >= n_groups || t.in_group < 0 ||
            (uint32_t)t.in_group >= n_groups)
            return bad("tensor group index out of range", i);
        if (groups[t.out_group].width != t.out_ch) return bad("out_ch differs from the width of out_group", i);
        if ((uint64_t)groups[t.in_group].width * t.in_mult != t.in_ch)
            return bad("in_ch differs from width of in_group times in_mult", i);
        const uint64_t khw = (uint64_t)t.kh * t.kw;
        const uint64_t numel = (uint64_t)t.out_ch * t.in_ch * khw;
        if (khw >= (1ull << 32) || numel >= (1ull << 32) - 2 * TILE || khw * t.in_mult >= (1ull << 32))
            return bad("tensor of 2^32 or more elements", i);
        if (t.offset >= (1ull << 62)) return bad("tensor offset beyond 2^62", i);
        DevTensor& d = m->dt[i];
        d.offset = t.offset;
        d.gbase = t.prunable ? gbase : 0;
        d.numel = (uint32_t)numel;
        d.out_ch = t.out_ch;
        d.in_ch = t.in_ch;
        d.khw = (uint32_t)khw;
        d.row_len = (uint32_t)(t.in_ch * khw);
        d.kk = (uint32_t)(khw * t.in_mult);
        d.cin = t.in_ch / t.in_mult;
        d.magic_khw = magic_for(d.khw);
        d.magic_row = magic_for(d.row_len);
        d.magic_in = magic_for(d.in_ch);
        d.magic_kk = d.shift_kk = 0;
        if (d.kk >= 2) magic_u32(d.kk, &d.magic_kk, &d.shift_kk);
        {
            // work units of the gather when nothing is removed (see plan_kernel)
            const uint32_t chunks = (d.row_len + GATHER_CHUNK - 1) / GATHER_CHUNK;
            uint32_t lg = 6;
            while (lg < 10 && (1u << lg) < d.row_len) ++lg;
            const uint32_t rows_par = GATHER_CHUNK >> lg;
            const uint32_t rb = 4u * std::max(rows_par, 4u);
            m->gather_units_bound += chunks * ((t.out_ch + rb - 1) / rb);
            // portfolio rebuild: the source is cut into rectangles of band_rows filters
            // times chunk_ch whole channels (at most GATHER_CHUNK columns), sized to the
            // RECT_ELEMS floats a block stages in LDS (see gather_rect_kernel)
            if (d.kk > GATHER_CHUNK) m->rect_ok = false;
            d.chunk_ch = std::min(d.cin, std::max(1u, GATHER_CHUNK / d.kk));
            d.src_chunks = (d.cin + d.chunk_ch - 1) / d.chunk_ch;
            const uint32_t wp = (d.chunk_ch * d.kk + 127u) & ~127u;
            d.band_rows = std::max(1u, std::min(64u, RECT_ELEMS / std::max(wp, 128u)));
            const uint64_t bands = (t.out_ch + d.band_rows - 1) / d.band_rows;
            if (m->rect_prefix.empty()) {
                m->rect_prefix.push_back(0);
                m->rowtab_prefix.push_back(0);
                m->coltab_prefix.push_back(0);
            }
            // blocks are dealt to the eight XCDs in turn: eight bands side by side, one per
            // XCD, each XCD walking its band chunk by chunk (see gather_rect_kernel)
            const uint64_t rects = (bands + 7) / 8 * 8 * d.src_chunks;
            if (m->rect_prefix.back() + rects >= (1ull << 31) ||
                m->rowtab_prefix.back() + bands + 1 >= (1ull << 31) / MAXK)
                return bad("model too large for 32-bit gather unit indices", i);
            m->rect_prefix.push_back(m->rect_prefix.back() + (uint32_t)rects);
            m->rowtab_prefix.push_back(m->rowtab_prefix.back() + (uint32_t)bands + 1);
            m->coltab_prefix.push_back(m->coltab_prefix.back() + d.src_chunks + 1);
            // kernel-level index of the liveness fixpoint: one byte per (filter, feature),
            // walked in tiles of 16 filters x 1024 features
            m->kernel_off.push_back(m->sum_kernels);
            m->sum_kernels += (uint64_t)t.out_ch * t.in_ch;
            const uint64_t ft = (uint64_t)((t.out_ch + 15) / 16) * ((t.in_ch + 1023) / 1024);
            if (m->fix_prefix.empty()) m->fix_prefix.push_back(0);
            if (m->fix_prefix.back() + ft >= (1ull << 31))
                return bad("model too large for 32-bit kernel-index tiles", i);
            m->fix_prefix.push_back(m->fix_prefix.back() + (uint32_t)ft);
        }
        d.out_group = t.out_group;
        d.in_group = t.in_group;
        d.out_flag_off = (uint32_t)so;
        d.in_flag_off = (uint32_t)si;
        d.prunable = t.prunable ? 1u : 0u;
        m->out_flag_off.push_back(so);
        m->in_flag_off.push_back(si);
        m->tile_prefix.push_back((uint32_t)tiles);
        so += t.out_ch;
        si += t.in_ch;
        if (t.prunable) gbase += numel;
        tiles += (numel + TILE - 1) / TILE;
        w_el += numel;
        w_ext = std::max(w_ext, t.offset + numel);
        spans.push_back({t.offset, t.offset + numel});
        if (so >= (1ull << 32) || si >= (1ull << 32) || tiles >= (1ull << 31))
            return bad("model too large for 32-bit flag or tile indices", i);
        if (gbase >= (1ull << 32) - 1) return bad("prunable weights reach 2^32 - 1 (32-bit global index)", i);
    }
    m->tile_prefix.push_back((uint32_t)tiles);
    m->n_tiles = (uint32_t)tiles;
    if (m->rect_prefix.empty()) {
        m->rect_prefix.push_back(0);
        m->rowtab_prefix.push_back(0);
        m->coltab_prefix.push_back(0);
    }
    if (m->fix_prefix.empty()) m->fix_prefix.push_back(0);
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
        if (spans[i].first < spans[i - 1].second) return bad("tensors overlap in the weight arena", (uint32_t)i);
    for (uint32_t i = 0; i < n_tensors; ++i)
        if (tensors[i].prunable) m->ranked_ids.push_back(i);
    m->n_ranked = (uint32_t)m->ranked_ids.size();
    // the single-pass selection samples one 16-weight sector per 1024 weights of every
    // sample_tile_stride-th tile (see spec_sample_kernel); its size is fixed by the
    // descriptors.  N / 64 samples for models up to 164 M weights; beyond that 40000
    // tiles (2.6 M samples), and from 1.3 G weights on every 8th tile: the candidate
    // interval is about N / sqrt(samples) weights wide, and the finishing passes hold a
    // fixed number of them.
    {
        const uint32_t sampled = std::max(40000u, m->n_tiles / 8u);
        m->sample_tile_stride = (m->n_tiles + sampled - 1) / sampled;   // 1 up to 164 M weights
    }
    for (uint32_t tile = 0, ti = 0; tile < m->n_tiles; tile += m->sample_tile_stride) {
        while (m->tile_prefix[ti + 1] <= tile) ++ti;
        if (!tensors[ti].prunable) continue;
        const uint64_t e0 = (uint64_t)(tile - m->tile_prefix[ti]) * TILE;
        const uint64_t n = std::min<uint64_t>(TILE, m->dt[ti].numel - e0);
        for (uint32_t quarter = 0; quarter < 4; ++quarter) {
            const uint32_t sector = (tile * 37u + quarter * 11u) & 63u;
            for (uint32_t part = 0; part < 4; ++part) {
                const uint64_t j = quarter * 1024u + sector * 16u + part * 4u;
                if (j + 3 < n) m->sample_size += 4;
            }
        }
    }

    uint64_t v_ext = 0, v_el = 0;
    m->dv.resize(n_vecs);
    spans.clear();
    for (uint32_t i = 0; i < n_vecs; ++i) {
        const shifter_vec_desc& v = vecs[i];
        if (v.group < 0 || (uint32_t)v.group >= n_groups) return bad("vector group index out of range", i);
        if (groups[v.group].width != v.len) return bad("vector length differs from the width of its group", i);
        if (v.offset >= (1ull << 62)) return bad("vector offset beyond 2^62", i);
        m->dv[i] = {v.offset, v.len, v.group};
        v_ext = std::max(v_ext, v.offset + v.len);
        v_el += v.len;
        spans.push_back({v.offset, v.offset + v.len});
    }
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
        if (spans[i].first < spans[i - 1].second) return bad("vectors overlap in the vector arena", (uint32_t)i);

    // consumers of each group, in tensor order
    {
        std::vector<uint32_t> at(n_groups + 1, 0);
        for (uint32_t i = 0; i < n_tensors; ++i) ++at[tensors[i].in_group + 1];
        for (uint32_t g = 0; g < n_groups; ++g) at[g + 1] += at[g];
        m->cons_prefix.assign(at.begin(), at.end());
        m->consumers.resize(n_tensors);
        for (uint32_t i = 0; i < n_tensors; ++i) m->consumers[at[tensors[i].in_group]++] = i;
    }
    // producers of each group, in tensor order
    {
        std::vector<uint32_t> at(n_groups + 1, 0);
        for (uint32_t i = 0; i < n_tensors; ++i) ++at[tensors[i].out_group + 1];
        for (uint32_t g = 0; g < n_groups; ++g) at[g + 1] += at[g];
        for (uint32_t g = 0; g < n_groups; ++g) {
            m->dg[g].prod_begin = at[g];
            m->dg[g].prod_end = at[g + 1];
            m->dg[g].pad = 0;
        }
        m->producers.resize(n_tensors);
        for (uint32_t i = 0; i < n_tensors; ++i) m->producers[at[tensors[i].out_group]++] = i;
    }
    shifter_model_info& inf = m->info;
    inf.n_prunable = gbase;
    inf.w_extent = w_ext;
    inf.v_extent = v_ext;
    inf.w_elems = w_el;
    inf.v_elems = v_el;
    inf.sum_out_ch = so;
    inf.sum_in_ch = si;
    inf.sum_group_width = goff;
    inf.n_tensors = n_tensors;
    inf.n_vecs = n_vecs;
    inf.n_groups = n_groups;
    inf.reserved = 0;
    *out = m;
    return SHIFTER_OK;
}

extern "C" int shifter_model_destroy(shifter_model* m) {
    if (!m) return SHIFTER_OK;
    unbind(m);
    delete m;
    return SHIFTER_OK;
}

extern "C" int shifter_model_get_info(const shifter_model* m, shifter_model_info* out) {
    if (!m || !out) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "model_get_info: NULL argument");
    *out = m->info;
    return SHIFTER_OK;
}

extern "C" int shifter_model_get_layout(const shifter_model* m, uint64_t* h_out_flag_off,
                                        uint64_t* h_in_flag_off, uint64_t* h_group_off) {
    if (!m) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "model_get_layout: model is NULL");
    if (h_out_flag_off) std::copy(m->out_flag_off.begin(), m->out_flag_off.end(), h_out_flag_off);
    if (h_in_flag_off) std::copy(m->in_flag_off.begin(), m->in_flag_off.end(), h_in_flag_off);
    if (h_group_off) std::copy(m->group_off.begin(), m->group_off.end(), h_group_off);
    return SHIFTER_OK;
}

template <typename T>
static int upload(shifter_ctx* ctx, T** dptr, const T* src, size_t n) {
    const size_t bytes = std::max<size_t>(n, 1) * sizeof(T);
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(dptr), bytes));
    if (n) HIP_TRY(ctx, hipMemcpy(*dptr, src, n * sizeof(T), hipMemcpyHostToDevice));
    return SHIFTER_OK;
}

static int bind_tables(shifter_ctx* ctx, shifter_model* m);

// Device tables and scratch of a model, created once per (model, context).  A binding that
// fails half way is taken down again, so that a later call starts from nothing.
static int bind(shifter_ctx* ctx, const shifter_model* cm) {
    shifter_model* m = const_cast<shifter_model*>(cm);
    if (m->b.ctx == ctx && m->b.ctx_id == ctx->id) return SHIFTER_OK;
    unbind(m);
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    m->b.ctx = ctx;
    m->b.ctx_id = ctx->id;
    m->b.device = ctx->device;
    const int rc = bind_tables(ctx, m);
    if (rc) unbind(m);
    return rc;
}

static int bind_tables(shifter_ctx* ctx, shifter_model* m) {
    auto& b = m->b;
    int rc;
    const size_t n_t = m->t.size(), n_v = m->v.size();
    if ((rc = upload(ctx, &b.tens, m->dt.data(), n_t))) return rc;
    if ((rc = upload(ctx, &b.groups, m->dg.data(), m->dg.size()))) return rc;
    if ((rc = upload(ctx, &b.vecs, m->dv.data(), n_v))) return rc;
    if ((rc = upload(ctx, &b.producers, m->producers.data(), m->producers.size()))) return rc;
    if ((rc = upload(ctx, &b.tile_prefix, m->tile_prefix.data(), m->tile_prefix.size()))) return rc;
    {
        std::vector<uint16_t> tt(m->n_tiles);
        for (size_t t = 0; t < n_t; ++t)
            for (uint32_t tile = m->tile_prefix[t]; tile < m->tile_prefix[t + 1]; ++tile) tt[tile] = (uint16_t)t;
        if ((rc = upload(ctx, &b.tile_tensor, tt.data(), tt.size()))) return rc;
    }
    if ((rc = upload(ctx, &b.rect_prefix, m->rect_prefix.data(), m->rect_prefix.size()))) return rc;
    if ((rc = upload(ctx, &b.rowtab_prefix, m->rowtab_prefix.data(), m->rowtab_prefix.size()))) return rc;
    if ((rc = upload(ctx, &b.coltab_prefix, m->coltab_prefix.data(), m->coltab_prefix.size()))) return rc;
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.rowtab),
                           sizeof(uint32_t) * MAXK * std::max<size_t>(m->rowtab_prefix.back(), 1)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.coltab),
                           sizeof(uint32_t) * MAXK * std::max<size_t>(m->coltab_prefix.back(), 1)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.sel), sizeof(SelState)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.ghist), sizeof(uint32_t) * MAXK * HIST_BINS));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.tile_cnt),
                           sizeof(uint32_t) * (size_t)MAXK * std::max<uint32_t>(m->n_tiles, 1)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.plan_t), sizeof(PlanTensor) * n_t * MAXK));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.plan_v), sizeof(PlanVec) * std::max<size_t>(n_v, 1) * MAXK));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.plan_h), sizeof(PlanHeader) * MAXK));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.out_tile_prefix), sizeof(uint32_t) * (n_t + 1) * MAXK));
    if ((rc = upload(ctx, &b.kernel_off, m->kernel_off.data(), m->kernel_off.size()))) return rc;
    if ((rc = upload(ctx, &b.fix_prefix, m->fix_prefix.data(), m->fix_prefix.size()))) return rc;
    if ((rc = upload(ctx, &b.cons_prefix, m->cons_prefix.data(), m->cons_prefix.size()))) return rc;
    if ((rc = upload(ctx, &b.consumers, m->consumers.data(), m->consumers.size()))) return rc;
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.fix_alive), std::max<uint64_t>(m->info.sum_group_width, 16)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.fix_produced), std::max<uint64_t>(m->info.sum_out_ch, 16)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.fix_read), std::max<uint64_t>(m->info.sum_in_ch, 16)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.fix_out_flags), std::max<uint64_t>(m->info.sum_out_ch, 16)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.fix_removed), sizeof(uint32_t) * FIX_STATE_WORDS));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.fold), sizeof(FoldTensor) * std::max<size_t>(n_t, 1)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.fold_scale),
                           sizeof(float) * std::max<uint64_t>(m->info.sum_out_ch, 4)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.levels),
                           sizeof(uint32_t) * (m->info.sum_out_ch + m->info.sum_in_ch)));
    if ((rc = upload(ctx, &b.ranked_ids, m->ranked_ids.data(), m->ranked_ids.size()))) return rc;
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.spec), sizeof(SpecState)));
    // every ranking reads the sample histogram and leaves it cleared for the next one
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.shist), sizeof(uint32_t) * 65536));
    HIP_TRY(ctx, hipMemset(b.shist, 0, sizeof(uint32_t) * 65536));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.spec_cnt), sizeof(uint32_t) * 2 * SPEC_SUB * 32));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.partial), sizeof(uint32_t) * SPEC_FIN_BLOCKS * 256));
    // candidate pairs: 1/4 of N in total (a 20-variant portfolio on a mid-size model makes
    // candidates of about a tenth of the weights), at least two tiles per sub-buffer
    b.cand_cap_sb = (uint32_t)std::max<uint64_t>(m->info.n_prunable / 4 / SPEC_SUB, 2 * TILE);
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.cand), sizeof(uint2) * (size_t)b.cand_cap_sb * SPEC_SUB));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.list), sizeof(uint2) * SPEC_LIST_CAP));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.multi), sizeof(MultiState)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.multi_cnt), sizeof(uint32_t) * (2 * MAXK + 1) * SPEC_SUB * 32));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.multi_tab), 4096));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.multi_hist), sizeof(uint32_t) * MAXK * 256));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.multi_list),
                           sizeof(uint2) * (size_t)SPEC_MULTI_MAXK * SPEC_LIST_CAP));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.multi_list_cnt), sizeof(uint32_t) * MAXK));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.multi_rowsum), sizeof(uint64_t) * (MAXK + 1)));
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&b.below),
                           sizeof(uint32_t) * MAXK * (m->info.sum_group_width + m->g.size())));
    b.host_stage_bytes = sizeof(SelState) + sizeof(shifter_threshold) * MAXK +
                         MAXK * (sizeof(PlanHeader) + sizeof(PlanTensor) * n_t + sizeof(PlanVec) * n_v +
                                 sizeof(uint32_t) * m->g.size()) +
                         sizeof(SpecState) + sizeof(MultiState) + 256;
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&b.host_stage), b.host_stage_bytes, hipHostMallocDefault));
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&b.host_spec), sizeof(SpecState),
                               hipHostMallocMapped | hipHostMallocCoherent));
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&b.host_spec_now), sizeof(SpecState),
                               hipHostMallocMapped | hipHostMallocCoherent));
    memset(b.host_spec, 0, sizeof(SpecState));
    memset(b.host_spec_now, 0, sizeof(SpecState));
    {
        void* q = nullptr;
        HIP_TRY(ctx, hipHostGetDevicePointer(&q, b.host_spec, 0));
        b.dev_spec = static_cast<SpecState*>(q);
        HIP_TRY(ctx, hipHostGetDevicePointer(&q, b.host_spec_now, 0));
        b.dev_spec_now = static_cast<SpecState*>(q);
    }
    // mirrors written by kernels: host-coherent pinned memory, addressed through its device pointer
    const size_t plan_stride = sizeof(PlanHeader) + sizeof(PlanTensor) * n_t + sizeof(PlanVec) * n_v;
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&b.host_multi),
                               MULTI_MIRROR_REC_OFF + sizeof(shifter_threshold) * MAXK,
                               hipHostMallocMapped | hipHostMallocCoherent));
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&b.host_plan), plan_stride * MAXK,
                               hipHostMallocMapped | hipHostMallocCoherent));
    memset(b.host_multi, 0, MULTI_MIRROR_REC_OFF + sizeof(shifter_threshold) * MAXK);
    memset(b.host_plan, 0, plan_stride * MAXK);
    void* dp = nullptr;
    HIP_TRY(ctx, hipHostGetDevicePointer(&dp, b.host_multi, 0));
    b.dev_multi_status = reinterpret_cast<uint32_t*>(dp);
    b.dev_multi_rec = reinterpret_cast<shifter_threshold*>(static_cast<uint8_t*>(dp) + MULTI_MIRROR_REC_OFF);
    HIP_TRY(ctx, hipHostGetDevicePointer(&dp, b.host_plan, 0));
    b.dev_plan = static_cast<uint8_t*>(dp);
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&b.host_width),
                               sizeof(uint32_t) * std::max<size_t>(m->g.size(), 1),
                               hipHostMallocMapped | hipHostMallocCoherent));
    memset(b.host_width, 0, sizeof(uint32_t) * std::max<size_t>(m->g.size(), 1));
    HIP_TRY(ctx, hipHostGetDevicePointer(&dp, b.host_width, 0));
    b.dev_width = static_cast<uint32_t*>(dp);
    HIP_TRY(ctx, hipDeviceSynchronize());     // the memsets above are done before any kernel of the model
    return SHIFTER_OK;
}

static int enter(shifter_ctx* ctx, const shifter_model* m, const char* fn) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, std::string(fn) + ": ctx is NULL");
    if (!m) return fail(ctx, SHIFTER_ERR_INVALID_ARG, std::string(fn) + ": model is NULL");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    return bind(ctx, m);
}

static bool misaligned(const void* p, uintptr_t a) {
    return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0;
}

static int after_launch(shifter_ctx* ctx, const char* fn) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(ctx, SHIFTER_ERR_HIP, std::string(fn) + ": launch failed: " + hipGetErrorString(e));
    return SHIFTER_OK;
}

// Waits for the stream and evaluates the outcome the selection's last kernel left in the
// pinned mirror `st`.
static int spec_result_collect(shifter_ctx* ctx, const uint8_t* st, shifter_threshold* h_thr,
                               int* decided) {
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    SpecState ss;
    memcpy(&ss, st, sizeof ss);
    ctx->last_spec = ss;
    ctx->last_path = (ss.status & 1u) ? 2 : 1;
    // a prediction that missed (not a tie overflow) widens the margin of later calls
    if ((ss.status & 1u) && ss.p > 0 && !(ss.n_below < ss.p && ss.p <= ss.n_below + ss.n_inside) &&
        ctx->margin_sigmas < 64.0)
        ctx->margin_sigmas *= 2.0;
    if (ss.status & 2u)
        return fail(ctx, SHIFTER_ERR_NONFINITE, "NaN among the prunable weights");
    *decided = (ss.status & 1u) ? 0 : 1;
    if (*decided) {
        ctx->last_record = ss.rec;
        if (h_thr) *h_thr = ctx->last_record;
    }
    return SHIFTER_OK;
}

static int spec_result(shifter_ctx* ctx, const shifter_model* model, shifter_threshold* h_thr,
                       int* decided) {
    return spec_result_collect(ctx, model->b.host_spec_now, h_thr, decided);
}

// Waits for the stream and evaluates the outcome of the K-rank single pass, which its
// kernels left in the model's pinned mirror: one status word per sorted rank (bit 0: could
// not decide, bit 1: NaN) and the K records.
static int multi_result(shifter_ctx* ctx, const shifter_model* model, uint32_t k_eff, uint32_t K,
                        shifter_threshold* h_thr, int* decided, const char* fn) {
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    const uint32_t* hs = reinterpret_cast<const uint32_t*>(model->b.host_multi);
    uint32_t status = 0;
    for (uint32_t k = 0; k < k_eff; ++k) status |= hs[k];
    if (status & 2u)
        return fail(ctx, SHIFTER_ERR_NONFINITE, std::string(fn) + ": NaN among the prunable weights");
    ctx->last_path = (status & 1u) ? 2 : 1;
    *decided = (status & 1u) ? 0 : 1;
    if (*decided) {
        if (h_thr) memcpy(h_thr, model->b.host_multi + MULTI_MIRROR_REC_OFF, sizeof(shifter_threshold) * K);
    } else if (!(status & 4u) && ctx->margin_sigmas < 64.0) {
        ctx->margin_sigmas *= 2.0;     // a prediction missed: wider intervals from now on
    }
    return SHIFTER_OK;
}

extern "C" int shifter_global_threshold(shifter_ctx* ctx, const shifter_model* model,
                                        const float* d_w, const uint64_t* h_n_prune, uint32_t K,
                                        shifter_threshold* d_thr, shifter_threshold* h_thr) {
    int rc = enter(ctx, model, "global_threshold");
    if (rc) return rc;
    if (!d_w || !h_n_prune || !d_thr)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold: NULL pointer argument");
    if (misaligned(d_w, 16) || misaligned(d_thr, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold: d_w must be 16-byte aligned");
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold: K must be in [1, SHIFTER_MAX_VARIANTS]");
    PruneCounts pc;
    memset(&pc, 0, sizeof pc);
    for (uint32_t k = 0; k < K; ++k) {
        if (h_n_prune[k] > model->info.n_prunable)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold: prune count exceeds N");
        pc.p[k] = h_n_prune[k];
    }
    if (h_thr && K == 1 && ctx->select_path == 0) {
        // single pass; exact when its own check holds, else fall through to the radix select
        launch_spec_select(ctx, model, d_w, pc.p[0], d_thr, nullptr, nullptr, nullptr, nullptr,
                           model->b.dev_spec_now);
        if ((rc = after_launch(ctx, "global_threshold"))) return rc;
        int decided = 0;
        if ((rc = spec_result(ctx, model, h_thr, &decided))) return rc;
        if (decided) return SHIFTER_OK;
    }
    if (h_thr && K > 1 && ctx->select_path == 0) {
        // all counts in a single pass; the counts > 0 sorted ascending, at most
        // SPEC_MULTI_MAXK of them
        PruneCounts sp;
        MultiPerm perm;
        memset(&sp, 0, sizeof sp);
        memset(&perm, 0, sizeof perm);
        uint32_t idx[MAXK], k_eff = 0;
        uint64_t zero_mask = 0;
        for (uint32_t k = 0; k < K; ++k) {
            if (pc.p[k] == 0) zero_mask |= 1ull << k; else idx[k_eff++] = k;
        }
        if (k_eff <= SPEC_MULTI_MAXK) {
            std::stable_sort(idx, idx + k_eff, [&](uint32_t a, uint32_t b) { return pc.p[a] < pc.p[b]; });
            for (uint32_t i = 0; i < k_eff; ++i) { sp.p[i] = pc.p[idx[i]]; perm.v[i] = idx[i]; }
            launch_spec_multi(ctx, model, d_w, sp, perm, k_eff, zero_mask, d_thr, nullptr);
            if ((rc = after_launch(ctx, "global_threshold"))) return rc;
            int decided = 0;
            if ((rc = multi_result(ctx, model, k_eff, K, h_thr, &decided, "global_threshold"))) return rc;
            if (decided) return SHIFTER_OK;
        }
    }
    launch_select(ctx, model, d_w, pc, K, d_thr);
    if ((rc = after_launch(ctx, "global_threshold"))) return rc;
    if (h_thr) {
        uint8_t* st = model->b.host_stage;
        HIP_TRY(ctx, hipMemcpyAsync(st, d_thr, sizeof(shifter_threshold) * K, hipMemcpyDeviceToHost, ctx->stream));
        HIP_TRY(ctx, hipMemcpyAsync(st + sizeof(shifter_threshold) * MAXK, &model->b.sel->nan_seen,
                                    sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        memcpy(h_thr, st, sizeof(shifter_threshold) * K);
        uint32_t nan_seen;
        memcpy(&nan_seen, st + sizeof(shifter_threshold) * MAXK, sizeof nan_seen);
        if (nan_seen)
            return fail(ctx, SHIFTER_ERR_NONFINITE, "global_threshold: NaN among the prunable weights");
    }
    return SHIFTER_OK;
}

extern "C" int shifter_global_threshold_static(shifter_ctx* ctx, const float* d_w, uint64_t n,
                                               const uint64_t* h_n_prune, uint32_t K,
                                               shifter_threshold* d_thr) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "global_threshold_static: ctx is NULL");
    if ((!d_w && n) || !h_n_prune || !d_thr)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_static: NULL pointer argument");
    if (misaligned(d_w, 16) || misaligned(d_thr, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_static: d_w must be 16-byte aligned");
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_static: K must be in [1, SHIFTER_MAX_VARIANTS]");
    const uint64_t n_tiles = (n + TILE - 1) / TILE;
    if (n > STATIC_MAX_WEIGHTS || n_tiles * K > STATIC_MAX_TILE_COUNTS)
        return fail(ctx, SHIFTER_ERR_CAPACITY,
                    "global_threshold_static: " + std::to_string(n) + " weights and " + std::to_string(K) +
                        " prune counts exceed the static scratch (at most " +
                        std::to_string(STATIC_MAX_WEIGHTS) + " weights and K * ceil(n / 4096) <= " +
                        std::to_string(STATIC_MAX_TILE_COUNTS) + ")");
    PruneCounts pc;
    memset(&pc, 0, sizeof pc);
    for (uint32_t k = 0; k < K; ++k) {
        if (h_n_prune[k] > n)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_static: prune count exceeds n");
        pc.p[k] = h_n_prune[k];
    }
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    uint8_t* base = ctx->static_scratch;   // the array's device address, never its name
    DevTensor* tens = reinterpret_cast<DevTensor*>(base + STATIC_OFF_TENSOR);
    uint32_t* prefix = reinterpret_cast<uint32_t*>(base + STATIC_OFF_PREFIX);
    launch_flat_tables(ctx, tens, prefix, n);
    const SelectTables tb{tens, prefix, 1u, (uint32_t)n_tiles,
                          reinterpret_cast<SelState*>(base + STATIC_OFF_SEL),
                          reinterpret_cast<uint32_t*>(base + STATIC_OFF_GHIST),
                          reinterpret_cast<uint32_t*>(base + STATIC_OFF_TILE_CNT)};
    launch_select_tables(ctx, tb, d_w, pc, K, d_thr);
    return after_launch(ctx, "global_threshold_static");
}

// Enqueues the read-back of a ranking's outcome (a status word, then the K records) into
// the model's pinned buffer.
static int rank_result_enqueue(shifter_ctx* ctx, const shifter_model* model, const uint32_t* d_status,
                               const shifter_threshold* d_thr, uint32_t K) {
    uint8_t* st = model->b.host_multi;
    HIP_TRY(ctx, hipMemcpyAsync(st, d_status, sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(st + MULTI_MIRROR_REC_OFF, d_thr, sizeof(shifter_threshold) * K,
                                hipMemcpyDeviceToHost, ctx->stream));
    return SHIFTER_OK;
}

extern "C" int shifter_global_threshold_begin(shifter_ctx* ctx, const shifter_model* model,
                                              const float* d_w, const uint64_t* h_n_prune, uint32_t K,
                                              shifter_threshold* d_thr) {
    int rc = enter(ctx, model, "global_threshold_begin");
    if (rc) return rc;
    if (ctx->pending_rank.active)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "global_threshold_begin: the previous one has not been collected (global_threshold_end)");
    if (!d_w || !h_n_prune || !d_thr)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_begin: NULL pointer argument");
    if (misaligned(d_w, 16) || misaligned(d_thr, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_begin: d_w must be 16-byte aligned");
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_begin: K must be in [1, SHIFTER_MAX_VARIANTS]");
    auto& pr = ctx->pending_rank;
    memset(&pr.pc, 0, sizeof pr.pc);
    for (uint32_t k = 0; k < K; ++k) {
        if (h_n_prune[k] > model->info.n_prunable)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_begin: prune count exceeds N");
        pr.pc.p[k] = h_n_prune[k];
    }
    uint32_t idx[MAXK], k_eff = 0;
    uint64_t zero_mask = 0;
    for (uint32_t k = 0; k < K; ++k) {
        if (pr.pc.p[k] == 0) zero_mask |= 1ull << k; else idx[k_eff++] = k;
    }
    pr.single_pass = ctx->select_path == 0 && k_eff <= SPEC_MULTI_MAXK;
    if (pr.single_pass) {
        PruneCounts sp;
        MultiPerm perm;
        memset(&sp, 0, sizeof sp);
        memset(&perm, 0, sizeof perm);
        std::stable_sort(idx, idx + k_eff, [&](uint32_t a, uint32_t b) { return pr.pc.p[a] < pr.pc.p[b]; });
        for (uint32_t i = 0; i < k_eff; ++i) { sp.p[i] = pr.pc.p[idx[i]]; perm.v[i] = idx[i]; }
        // the kernels leave the outcome in the pinned mirror themselves
        launch_spec_multi(ctx, model, d_w, sp, perm, k_eff, zero_mask, d_thr, nullptr);
        if ((rc = after_launch(ctx, "global_threshold_begin"))) return rc;
        pr.k_eff = k_eff;
    } else {
        launch_select(ctx, model, d_w, pr.pc, K, d_thr);
        if ((rc = after_launch(ctx, "global_threshold_begin"))) return rc;
        if ((rc = rank_result_enqueue(ctx, model, &model->b.sel->nan_seen, d_thr, K))) return rc;
    }
    pr.active = true;
    pr.model = model;
    pr.d_w = d_w;
    pr.k = K;
    pr.d_thr = d_thr;
    return SHIFTER_OK;
}

extern "C" int shifter_global_threshold_end(shifter_ctx* ctx, shifter_threshold* h_thr, int* h_redone) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "global_threshold_end: ctx is NULL");
    auto& pr = ctx->pending_rank;
    if (!pr.active)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "global_threshold_end: nothing to collect");
    pr.active = false;
    if (h_redone) *h_redone = 0;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    const shifter_model* model = pr.model;
    uint8_t* st = model->b.host_multi;
    uint32_t status;
    if (pr.single_pass) {
        int decided = 0;
        int rc = multi_result(ctx, model, pr.k_eff, pr.k, h_thr, &decided, "global_threshold_end");
        if (rc) return rc;
        if (decided) return SHIFTER_OK;
        // the single pass could not decide: the multi-pass select, and the caller repeats
        // what it had enqueued behind the ranking
        launch_select(ctx, model, pr.d_w, pr.pc, pr.k, pr.d_thr);
        if ((rc = after_launch(ctx, "global_threshold_end"))) return rc;
        if ((rc = rank_result_enqueue(ctx, model, &model->b.sel->nan_seen, pr.d_thr, pr.k))) return rc;
        if (h_redone) *h_redone = 1;
    } else {
        ctx->last_path = 2;
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    memcpy(&status, st, sizeof status);
    if (status)
        return fail(ctx, SHIFTER_ERR_NONFINITE, "global_threshold_end: NaN among the prunable weights");
    if (h_thr) memcpy(h_thr, st + MULTI_MIRROR_REC_OFF, sizeof(shifter_threshold) * pr.k);
    return SHIFTER_OK;
}

extern "C" int shifter_apply_mask(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                                  const shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                                  uint8_t* d_out_alive, uint8_t* d_in_alive) {
    int rc = enter(ctx, model, "apply_mask");
    if (rc) return rc;
    if (!d_w || !d_thr || !d_w_out)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "apply_mask: NULL pointer argument");
    if (misaligned(d_w, 16) || misaligned(d_w_out, 16) || misaligned(d_mask, 4) || misaligned(d_thr, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "apply_mask: arenas must be 16-byte aligned, the mask 4-byte aligned");
    if ((d_out_alive == nullptr) != (d_in_alive == nullptr))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "apply_mask: d_out_alive and d_in_alive must both be NULL or both be given");
    launch_mask_scan(ctx, model, d_w, d_thr, d_w_out, d_mask, d_out_alive, d_in_alive);
    return after_launch(ctx, "apply_mask");
}

// The two separate steps, for when the single pass could not decide or is switched off.
static int prune_unfused(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                         uint64_t n_prune, shifter_threshold* d_thr, float* d_w_out, uint8_t* d_mask,
                         uint8_t* d_out_alive, uint8_t* d_in_alive, shifter_threshold* h_thr) {
    const int saved = ctx->select_path;
    ctx->select_path = 1;
    int rc = shifter_global_threshold(ctx, model, d_w, &n_prune, 1, d_thr, nullptr);
    ctx->select_path = saved;
    if (rc) return rc;
    launch_mask_scan(ctx, model, d_w, d_thr, d_w_out, d_mask, d_out_alive, d_in_alive);
    if ((rc = after_launch(ctx, "prune_fused"))) return rc;
    uint8_t* st = model->b.host_stage;
    HIP_TRY(ctx, hipMemcpyAsync(st, d_thr, sizeof(shifter_threshold), hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(st + sizeof(shifter_threshold), &model->b.sel->nan_seen, sizeof(uint32_t),
                                hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    memcpy(&ctx->last_record, st, sizeof(shifter_threshold));
    if (h_thr) *h_thr = ctx->last_record;
    uint32_t nan_seen;
    memcpy(&nan_seen, st + sizeof(shifter_threshold), sizeof nan_seen);
    if (nan_seen) return fail(ctx, SHIFTER_ERR_NONFINITE, "prune_fused: NaN among the prunable weights");
    return SHIFTER_OK;
}

extern "C" int shifter_prune_fused(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                                   uint64_t n_prune, shifter_threshold* d_thr, float* d_w_out,
                                   uint8_t* d_mask, uint8_t* d_out_alive, uint8_t* d_in_alive,
                                   shifter_threshold* h_thr) {
    int rc = enter(ctx, model, "prune_fused");
    if (rc) return rc;
    if (!d_w || !d_thr || !d_w_out || !d_out_alive || !d_in_alive)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused: NULL pointer argument");
    if (d_w == d_w_out)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused: cannot work in place");
    if (misaligned(d_w, 16) || misaligned(d_w_out, 16) || misaligned(d_mask, 4) || misaligned(d_thr, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "prune_fused: arenas must be 16-byte aligned, the mask 4-byte aligned");
    if (n_prune > model->info.n_prunable)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused: prune count exceeds N");
    if (ctx->pending.active)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "prune_fused: the outcome of an earlier deferred call has not been collected");
    if (ctx->select_path == 0) {
        launch_spec_select(ctx, model, d_w, n_prune, d_thr, d_w_out, d_mask, d_out_alive, d_in_alive,
                           h_thr ? model->b.dev_spec_now : model->b.dev_spec);
        if ((rc = after_launch(ctx, "prune_fused"))) return rc;
        if (!h_thr) {
            // deferred: the outcome waits in its pinned mirror and is looked at later
            ctx->pending = {true, model, d_w, n_prune, d_thr, d_w_out, d_mask, d_out_alive, d_in_alive};
            return SHIFTER_OK;
        }
        int decided = 0;
        if ((rc = spec_result(ctx, model, h_thr, &decided))) return rc;
        if (decided) return SHIFTER_OK;
    }
    // the single pass could not decide (or is switched off): rank, then mask and scan
    return prune_unfused(ctx, model, d_w, n_prune, d_thr, d_w_out, d_mask, d_out_alive, d_in_alive, h_thr);
}

extern "C" int shifter_prune_fused_result(shifter_ctx* ctx, shifter_threshold* h_thr, int* h_redone) {
    if (!ctx || !h_redone)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused_result: NULL argument");
    *h_redone = 0;
    if (!ctx->pending.active) {
        // the call was not deferred (or ran the separate steps at once): nothing to collect
        HIP_TRY(ctx, hipSetDevice(ctx->device));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        if (h_thr) *h_thr = ctx->last_record;
        return SHIFTER_OK;
    }
    const shifter_ctx::Pending p = ctx->pending;
    ctx->pending.active = false;
    int rc = enter(ctx, p.model, "prune_fused_result");
    if (rc) return rc;
    int decided = 0;
    if ((rc = spec_result_collect(ctx, p.model->b.host_spec, h_thr, &decided))) return rc;
    if (decided) return SHIFTER_OK;
    *h_redone = 1;
    return prune_unfused(ctx, p.model, p.d_w, p.n_prune, p.d_thr, p.d_w_out, p.d_mask, p.d_out_alive,
                         p.d_in_alive, h_thr);
}

extern "C" int shifter_get_select_stats(const shifter_ctx* ctx, uint64_t* out8) {
    if (!ctx || !out8) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "get_select_stats: NULL argument");
    const SpecState& ss = ctx->last_spec;
    out8[0] = (uint64_t)ctx->last_path;
    out8[1] = ss.p;
    out8[2] = ss.n_below;
    out8[3] = ss.n_inside;
    out8[4] = ss.m_valid;
    out8[5] = ss.lo;
    out8[6] = ss.hi;
    out8[7] = ss.status;
    return SHIFTER_OK;
}

extern "C" int shifter_set_margin_sigmas(shifter_ctx* ctx, double sigmas) {
    if (!ctx || !(sigmas >= 0.0 && sigmas <= 1e6))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "set_margin_sigmas: value out of range");
    ctx->margin_sigmas = sigmas;
    return SHIFTER_OK;
}

extern "C" int shifter_set_select_grid(shifter_ctx* ctx, uint32_t blocks) {
    if (!ctx || blocks == 0 || blocks > 65536)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "set_select_grid: blocks must be in [1, 65536]");
    ctx->hist_grid = blocks;
    return SHIFTER_OK;
}

extern "C" int shifter_set_fused_min_bytes(shifter_ctx* ctx, uint64_t bytes) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "set_fused_min_bytes: ctx is NULL");
    ctx->fused_min_bytes = bytes;
    return SHIFTER_OK;
}

extern "C" int shifter_set_select_path(shifter_ctx* ctx, int path) {
    if (!ctx || path < 0 || path > 1)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "set_select_path: path must be 0 or 1");
    ctx->select_path = path;
    return SHIFTER_OK;
}

extern "C" int shifter_dead_channel_scan(shifter_ctx* ctx, const shifter_model* model,
                                         const float* d_w_sparse, uint8_t* d_out_alive,
                                         uint8_t* d_in_alive) {
    int rc = enter(ctx, model, "dead_channel_scan");
    if (rc) return rc;
    if (!d_w_sparse || !d_out_alive || !d_in_alive)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "dead_channel_scan: NULL pointer argument");
    if (misaligned(d_w_sparse, 16))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "dead_channel_scan: arena must be 16-byte aligned");
    launch_scan(ctx, model, d_w_sparse, d_out_alive, d_in_alive);
    return after_launch(ctx, "dead_channel_scan");
}

extern "C" int shifter_apply_mask_batch(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                                       const shifter_threshold* d_thr, uint32_t K, float* d_w_out,
                                       uint64_t w_stride, uint8_t* d_mask, uint64_t mask_stride,
                                       uint8_t* d_out_alive, uint8_t* d_in_alive) {
    int rc = enter(ctx, model, "apply_mask_batch");
    if (rc) return rc;
    if (!d_w || !d_thr || !d_out_alive)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "apply_mask_batch: NULL pointer argument");
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "apply_mask_batch: K must be in [1, SHIFTER_MAX_VARIANTS]");
    if (misaligned(d_w, 16) || misaligned(d_w_out, 16) || misaligned(d_mask, 4) || misaligned(d_thr, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "apply_mask_batch: arenas must be 16-byte aligned, the masks 4-byte aligned");
    if ((d_w_out && w_stride < model->info.w_extent) || (d_mask && mask_stride < model->info.n_prunable))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "apply_mask_batch: stride smaller than one variant");
    if (d_w_out == d_w)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "apply_mask_batch: cannot work in place");
    launch_mask_scan_batch(ctx, model, d_w, d_thr, K, d_w_out, w_stride, d_mask, mask_stride,
                           d_out_alive, d_in_alive);
    return after_launch(ctx, "apply_mask_batch");
}

extern "C" int shifter_prune_fused_batch(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                                         const uint64_t* h_n_prune, uint32_t K, shifter_threshold* d_thr,
                                         float* d_w_out, uint64_t w_stride, uint8_t* d_mask,
                                         uint64_t mask_stride, uint8_t* d_out_alive,
                                         uint8_t* d_in_alive, shifter_threshold* h_thr) {
    int rc = enter(ctx, model, "prune_fused_batch");
    if (rc) return rc;
    if (!d_w || !h_n_prune || !d_thr || !d_out_alive || !h_thr)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused_batch: NULL pointer argument");
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused_batch: K must be in [1, SHIFTER_MAX_VARIANTS]");
    if (misaligned(d_w, 16) || misaligned(d_w_out, 16) || misaligned(d_mask, 4) || misaligned(d_thr, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "prune_fused_batch: arenas must be 16-byte aligned, the masks 4-byte aligned");
    if ((d_w_out && w_stride < model->info.w_extent) || (d_mask && mask_stride < model->info.n_prunable))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused_batch: stride smaller than one variant");
    if (d_w_out == d_w)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused_batch: cannot work in place");
    PruneCounts pc, sp;
    MultiPerm perm;
    memset(&pc, 0, sizeof pc);
    memset(&sp, 0, sizeof sp);
    memset(&perm, 0, sizeof perm);
    uint32_t idx[MAXK], k_eff = 0;
    uint64_t zero_mask = 0;
    for (uint32_t k = 0; k < K; ++k) {
        if (h_n_prune[k] > model->info.n_prunable)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, "prune_fused_batch: prune count exceeds N");
        pc.p[k] = h_n_prune[k];
        if (pc.p[k] == 0) zero_mask |= 1ull << k; else idx[k_eff++] = k;
    }
    if (ctx->select_path == 0 && k_eff <= SPEC_MULTI_MAXK) {
        std::stable_sort(idx, idx + k_eff, [&](uint32_t a, uint32_t b) { return pc.p[a] < pc.p[b]; });
        for (uint32_t i = 0; i < k_eff; ++i) { sp.p[i] = pc.p[idx[i]]; perm.v[i] = idx[i]; }
        FusedBatch fb{K, d_w_out, w_stride, d_mask, mask_stride, d_out_alive, d_in_alive};
        launch_spec_multi(ctx, model, d_w, sp, perm, k_eff, zero_mask, d_thr, &fb);
        if ((rc = after_launch(ctx, "prune_fused_batch"))) return rc;
        int decided = 0;
        if ((rc = multi_result(ctx, model, k_eff, K, h_thr, &decided, "prune_fused_batch"))) return rc;
        if (decided) return SHIFTER_OK;
    }
    // the single pass could not decide (or is switched off, or too many counts): rank with
    // the multi-pass select, then mask and scan
    const int saved = ctx->select_path;
    ctx->select_path = 1;
    rc = shifter_global_threshold(ctx, model, d_w, h_n_prune, K, d_thr, h_thr);
    ctx->select_path = saved;
    if (rc) return rc;
    return shifter_apply_mask_batch(ctx, model, d_w, d_thr, K, d_w_out, w_stride, d_mask, mask_stride,
                                    d_out_alive, d_in_alive);
}

extern "C" int shifter_propagate_groups_batch(shifter_ctx* ctx, const shifter_model* model,
                                             const uint8_t* d_out_alive, uint32_t K, uint32_t flags,
                                             uint8_t* d_group_alive, int32_t* d_index_map,
                                             uint32_t* d_keep, uint32_t* d_new_width,
                                             uint32_t* h_new_width) {
    int rc = enter(ctx, model, "propagate_groups");
    if (rc) return rc;
    if (!d_out_alive || !d_group_alive || !d_index_map || !d_keep || !d_new_width)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "propagate_groups: NULL pointer argument");
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "propagate_groups: K must be in [1, SHIFTER_MAX_VARIANTS]");
    if (flags & ~SHIFTER_PAPER_FREEZE_RESIDUAL)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "propagate_groups: unknown flag bits");
    launch_propagate(ctx, model, d_out_alive, flags, d_group_alive, d_index_map, d_keep, d_new_width, K);
    if ((rc = after_launch(ctx, "propagate_groups"))) return rc;
    if (h_new_width) {
        const size_t n = model->g.size() * K;
        uint32_t* st = reinterpret_cast<uint32_t*>(model->b.host_stage);
        HIP_TRY(ctx, hipMemcpyAsync(st, d_new_width, sizeof(uint32_t) * n, hipMemcpyDeviceToHost, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        bool collapse = false;
        for (size_t g = 0; g < n; ++g) {
            h_new_width[g] = st[g];
            collapse |= st[g] == 0;
        }
        if (collapse) {
            fail(ctx, SHIFTER_WARN_COLLAPSE, "propagate_groups: a group kept no channel (layer collapse)");
            return SHIFTER_WARN_COLLAPSE;
        }
    }
    return SHIFTER_OK;
}

extern "C" int shifter_propagate_groups(shifter_ctx* ctx, const shifter_model* model,
                                        const uint8_t* d_out_alive, const uint8_t* d_in_alive,
                                        uint32_t flags, uint8_t* d_group_alive,
                                        int32_t* d_index_map, uint32_t* d_keep,
                                        uint32_t* d_new_width, uint32_t* h_new_width) {
    (void)d_in_alive;
    return shifter_propagate_groups_batch(ctx, model, d_out_alive, 1, flags, d_group_alive, d_index_map,
                                          d_keep, d_new_width, h_new_width);
}

extern "C" int shifter_model_get_kernel_layout(const shifter_model* model, uint64_t* h_kernel_off,
                                               uint64_t* h_sum_kernels) {
    if (!model) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "model_get_kernel_layout: model is NULL");
    if (h_kernel_off)
        for (size_t i = 0; i < model->kernel_off.size(); ++i) h_kernel_off[i] = model->kernel_off[i];
    if (h_sum_kernels) *h_sum_kernels = model->sum_kernels;
    return SHIFTER_OK;
}

extern "C" int shifter_kernel_scan(shifter_ctx* ctx, const shifter_model* model, const float* d_w_sparse,
                                   uint8_t* d_kernel_nz) {
    int rc = enter(ctx, model, "kernel_scan");
    if (rc) return rc;
    if (!d_w_sparse || !d_kernel_nz)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "kernel_scan: NULL pointer argument");
    if (misaligned(d_w_sparse, 16))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "kernel_scan: arena must be 16-byte aligned");
    launch_kernel_scan(ctx, model, d_w_sparse, d_kernel_nz);
    return after_launch(ctx, "kernel_scan");
}

extern "C" int shifter_propagate_groups_fixpoint(shifter_ctx* ctx, const shifter_model* model,
                                                 const uint8_t* d_kernel_nz, uint32_t flags,
                                                 uint8_t* d_group_alive, int32_t* d_index_map,
                                                 uint32_t* d_keep, uint32_t* d_new_width,
                                                 uint32_t* h_new_width, uint32_t* h_rounds) {
    int rc = enter(ctx, model, "propagate_groups_fixpoint");
    if (rc) return rc;
    if (!d_kernel_nz || !d_group_alive || !d_index_map || !d_keep || !d_new_width)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "propagate_groups_fixpoint: NULL pointer argument");
    if (flags & ~(uint32_t)(SHIFTER_PAPER_FREEZE_RESIDUAL | SHIFTER_GROUPS_FIXPOINT))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "propagate_groups_fixpoint: unknown flag");
    const auto& b = model->b;
    const bool wait = h_new_width || h_rounds;
    launch_fix_begin(ctx, model);
    // every round that changes something removes at least one channel
    const uint64_t max_rounds = model->info.sum_group_width + 1;
    const volatile uint32_t* mirror = reinterpret_cast<const volatile uint32_t*>(b.host_multi) + FIX_MIRROR_WORD;
    const volatile uint32_t* st = b.host_width;
    const size_t n_g = model->g.size();
    for (uint32_t batch = 0;; ++batch) {
        // a batch of rounds, the flags of what is alive after it, and the plan from them
        launch_fix_batch(ctx, model, d_kernel_nz, flags);
        launch_propagate(ctx, model, b.fix_out_flags, flags & SHIFTER_PAPER_FREEZE_RESIDUAL, d_group_alive,
                         d_index_map, d_keep, d_new_width, 1);
        if ((rc = after_launch(ctx, "propagate_groups_fixpoint"))) return rc;
        if (!wait) {
            // nothing is read back: a fixed number of batches, of which those after the
            // fixpoint cost a few empty launches
            if (batch + 1 == FIX_ENQUEUED_BATCHES) return SHIFTER_OK;
            continue;
        }
        if (h_new_width) launch_fix_widths(ctx, model, d_new_width);
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        if (mirror[1]) break;
        if ((uint64_t)mirror[0] > max_rounds)
            return fail(ctx, SHIFTER_ERR_INTERNAL, "propagate_groups_fixpoint: did not settle");
    }
    if (h_rounds) *h_rounds = mirror[0];
    if (h_new_width) {
        bool collapse = false;
        for (size_t g = 0; g < n_g; ++g) {
            h_new_width[g] = st[g];
            collapse |= st[g] == 0;
        }
        if (collapse) {
            fail(ctx, SHIFTER_WARN_COLLAPSE, "propagate_groups_fixpoint: a group kept no channel (layer collapse)");
            return SHIFTER_WARN_COLLAPSE;
        }
    }
    return SHIFTER_OK;
}

extern "C" int shifter_fixpoint_status(shifter_ctx* ctx, const shifter_model* model, uint32_t* h_rounds,
                                       uint32_t* h_settled) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "fixpoint_status: ctx is NULL");
    if (!model || model->b.ctx != ctx || model->b.ctx_id != ctx->id)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "fixpoint_status: the model has run nothing on this context");
    const volatile uint32_t* mirror =
        reinterpret_cast<const volatile uint32_t*>(model->b.host_multi) + FIX_MIRROR_WORD;
    if (h_rounds) *h_rounds = mirror[0];
    if (h_settled) *h_settled = mirror[1];
    return SHIFTER_OK;
}

extern "C" int shifter_fold_bn(shifter_ctx* ctx, const shifter_model* model,
                               const shifter_fold_desc* h_fold, uint32_t n_fold, float eps,
                               const float* d_w, const float* d_vecs, float* d_w_out,
                               float* d_bias_out, uint64_t cap_bias) {
    int rc = enter(ctx, model, "fold_bn");
    if (rc) return rc;
    if (!d_w || !d_w_out || (n_fold && (!h_fold || !d_vecs || !d_bias_out)))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "fold_bn: NULL pointer argument");
    if (misaligned(d_w, 16) || misaligned(d_w_out, 16) || misaligned(d_vecs, 4) || misaligned(d_bias_out, 4))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "fold_bn: weight arenas must be 16-byte aligned");
    if (!(eps >= 0.0f) || !std::isfinite(eps))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "fold_bn: eps must be finite and not negative");
    const size_t n_t = model->t.size(), n_v = model->v.size();
    std::vector<FoldTensor> tab(n_t, FoldTensor{-1, -1, -1, -1, -1, -1});
    std::vector<std::pair<uint64_t, uint64_t>> spans;
    for (uint32_t i = 0; i < n_fold; ++i) {
        const shifter_fold_desc& f = h_fold[i];
        const std::string at = "fold_bn: entry " + std::to_string(i) + ": ";
        if (f.tensor >= n_t) return fail(ctx, SHIFTER_ERR_INVALID_ARG, at + "tensor index out of range");
        if (tab[f.tensor].out_offset >= 0)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, at + "tensor listed twice");
        const uint32_t out_ch = model->t[f.tensor].out_ch;
        const int32_t bn[4] = {f.gamma, f.beta, f.mean, f.var};
        const bool has_bn = f.gamma >= 0;
        int64_t off[5];
        const int32_t ids[5] = {f.gamma, f.beta, f.mean, f.var, f.bias};
        for (int j = 0; j < 4; ++j)
            if ((bn[j] >= 0) != has_bn)
                return fail(ctx, SHIFTER_ERR_INVALID_ARG, at + "gamma, beta, mean and var go together");
        for (int j = 0; j < 5; ++j) {
            off[j] = -1;
            if (ids[j] < 0) continue;
            if ((size_t)ids[j] >= n_v) return fail(ctx, SHIFTER_ERR_INVALID_ARG, at + "vector index out of range");
            if (model->v[ids[j]].len != out_ch)
                return fail(ctx, SHIFTER_ERR_INVALID_ARG, at + "vector length differs from the tensor's out_ch");
            off[j] = (int64_t)model->v[ids[j]].offset;
        }
        if (f.out_offset > cap_bias || out_ch > cap_bias - f.out_offset)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, at + "bias range exceeds cap_bias");
        spans.push_back({f.out_offset, f.out_offset + out_ch});
        tab[f.tensor] = FoldTensor{off[0], off[1], off[2], off[3], off[4], (int64_t)f.out_offset};
    }
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
        if (spans[i].first < spans[i - 1].second)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, "fold_bn: bias ranges overlap");
    if (n_t == 0) return SHIFTER_OK;
    // the validated table stays on the device: a call with the list of the call before
    // uploads nothing and waits for nothing
    auto& held = const_cast<shifter_model*>(model)->b.fold_host;
    if (held.size() != n_t || memcmp(held.data(), tab.data(), sizeof(FoldTensor) * n_t) != 0) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        HIP_TRY(ctx, hipStreamIsCapturing(ctx->stream, &cap));
        if (cap != hipStreamCaptureStatusNone)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                        "fold_bn: a new layer list needs an upload and a wait, which a capturing stream "
                        "cannot take: call once with this list before the capture");
        // the pinned staging area may still feed an earlier upload: wait before rewriting it
        // (read-backs into it are enqueued behind this upload, so they cannot overtake it)
        held.clear();
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        memcpy(model->b.host_stage, tab.data(), sizeof(FoldTensor) * n_t);
        HIP_TRY(ctx, hipMemcpyAsync(model->b.fold, model->b.host_stage, sizeof(FoldTensor) * n_t,
                                    hipMemcpyHostToDevice, ctx->stream));
        held = tab;
    }
    launch_fold(ctx, model, d_w, d_vecs, eps, d_w_out, d_bias_out);
    return after_launch(ctx, "fold_bn");
}

// The plans of K variants, read from the pinned mirror the planning kernel wrote (the stream
// must have been waited for): descriptors and sizes of the rebuilt tensors and vectors, and
// the status they imply.
static int plan_readout(shifter_ctx* ctx, const shifter_model* model, uint32_t K,
                        shifter_tensor_desc* h_out_tensors, shifter_vec_desc* h_out_vecs,
                        uint64_t* h_elems_w, uint64_t* h_elems_v) {
    const size_t n_t = model->t.size(), n_v = model->v.size();
    const uint8_t* st = model->b.host_plan;
    const size_t stride = sizeof(PlanHeader) + sizeof(PlanTensor) * n_t + sizeof(PlanVec) * n_v;
    auto hh = [&](uint32_t k) { return reinterpret_cast<const PlanHeader*>(st + stride * k); };
    auto ht = [&](uint32_t k) { return reinterpret_cast<const PlanTensor*>(st + stride * k + sizeof(PlanHeader)); };
    auto hv = [&](uint32_t k) {
        return reinterpret_cast<const PlanVec*>(st + stride * k + sizeof(PlanHeader) + sizeof(PlanTensor) * n_t);
    };
    uint32_t status = 0;
    for (uint32_t k = 0; k < K; ++k) {
        status |= hh(k)->status;
        if (h_elems_w) h_elems_w[k] = hh(k)->elems_w;
        if (h_elems_v) h_elems_v[k] = hh(k)->elems_v;
        if (h_out_tensors) {
            for (size_t i = 0; i < n_t; ++i) {
                shifter_tensor_desc d = model->t[i];
                d.offset = ht(k)[i].out_off;
                d.out_ch = ht(k)[i].o2;
                d.in_ch = ht(k)[i].c2 * d.in_mult;
                h_out_tensors[k * n_t + i] = d;
            }
        }
        if (h_out_vecs) {
            for (size_t i = 0; i < n_v; ++i) {
                shifter_vec_desc d = model->v[i];
                d.offset = hv(k)[i].out_off;
                d.len = hv(k)[i].len2;
                h_out_vecs[k * n_v + i] = d;
            }
        }
    }
    if (status & 1u)
        return fail(ctx, SHIFTER_ERR_CAPACITY, "compact: output capacity too small; nothing gathered");
    if (status & 2u) {
        fail(ctx, SHIFTER_WARN_COLLAPSE, "compact: a group kept no channel (layer collapse)");
        return SHIFTER_WARN_COLLAPSE;
    }
    return SHIFTER_OK;
}

// d_thr == NULL: d_w holds K sparse arenas w_stride apart; else d_w is the dense arena
// (w_stride 0) and variant k is masked by d_thr[k] while it is gathered.
static int compact_impl(shifter_ctx* ctx, const shifter_model* model, const float* d_w_sparse,
                        uint64_t w_stride, const shifter_threshold* d_thr, const float* d_vecs,
                        const uint32_t* d_keep, const uint32_t* d_new_width, uint32_t K,
                        float* d_w_out, uint64_t cap_w, float* d_vecs_out, uint64_t cap_v,
                        shifter_tensor_desc* h_out_tensors, shifter_vec_desc* h_out_vecs,
                        uint64_t* h_elems_w, uint64_t* h_elems_v) {
    int rc = enter(ctx, model, "compact");
    if (rc) return rc;
    const size_t n_v = model->v.size();
    if (!d_w_sparse || !d_keep || !d_new_width || !d_w_out || (n_v && (!d_vecs || !d_vecs_out)))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "compact: NULL pointer argument");
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "compact: K must be in [1, SHIFTER_MAX_VARIANTS]");
    if (misaligned(d_w_out, 16) || (K > 1 && (cap_w & 3u)))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "compact: d_w_out must be 16-byte aligned (and cap_w a multiple of 4 in a batch)");
    launch_compact(ctx, model, d_w_sparse, w_stride, d_vecs, d_keep, d_new_width, d_w_out, cap_w,
                   d_vecs_out, cap_v, K, d_thr);
    if ((rc = after_launch(ctx, "compact"))) return rc;
    if (h_out_tensors || h_out_vecs || h_elems_w || h_elems_v) {
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        return plan_readout(ctx, model, K, h_out_tensors, h_out_vecs, h_elems_w, h_elems_v);
    }
    return SHIFTER_OK;
}

// ---- a whole portfolio step behind one call ---------------------------------------------

// The multi-pass ranking and everything behind it for a portfolio step: the path of a step
// whose single pass is switched off, does not apply or could not decide.
// Position of every variant in the order of the cuts: the cut grows strictly with the prune
// count (P = 0 gives cut 0), so it is the position of its count, ties by index - known on
// the host before any record exists.
static MultiPerm cut_positions(const PruneCounts& pc, uint32_t K) {
    MultiPerm pos;
    memset(&pos, 0, sizeof pos);
    for (uint32_t k = 0; k < K; ++k)
        for (uint32_t j = 0; j < K; ++j)
            pos.v[k] += (pc.p[j] < pc.p[k] || (pc.p[j] == pc.p[k] && j < k)) ? 1u : 0u;
    return pos;
}

static int portfolio_radix(shifter_ctx* ctx, const shifter_model* model, const PruneCounts& pc,
                           const PortfolioBuffers& a) {
    int rc;
    launch_select(ctx, model, a.d_w, pc, a.k_var, a.d_thr);
    if ((rc = after_launch(ctx, "portfolio"))) return rc;
    if ((rc = rank_result_enqueue(ctx, model, &model->b.sel->nan_seen, a.d_thr, a.k_var))) return rc;
    launch_zero_levels(ctx, model);
    launch_mask_scan_batch_core(ctx, model, a.d_w, a.d_thr, a.k_var, a.d_w_sparse, a.w_stride, a.d_mask,
                                a.mask_stride);
    launch_plan_and_gather(ctx, model, a, true, cut_positions(pc, a.k_var));
    return after_launch(ctx, "portfolio");
}

extern "C" int shifter_portfolio_begin(shifter_ctx* ctx, const shifter_model* model,
                                       const shifter_portfolio_args* args) {
    int rc = enter(ctx, model, "portfolio_begin");
    if (rc) return rc;
    if (!args) return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_begin: args is NULL");
    if (ctx->pending_portfolio.active || ctx->pending.active || ctx->pending_rank.active)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "portfolio_begin: an earlier deferred call on this context has not been collected");
    const shifter_portfolio_args& g = *args;
    const size_t n_v = model->v.size();
    if (!g.d_w || !g.h_n_prune || !g.d_thr || !g.d_out_alive || !g.d_group_alive || !g.d_index_map ||
        !g.d_keep || !g.d_new_width || !g.d_w_out || (n_v && (!g.d_vecs || !g.d_vecs_out)))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_begin: NULL pointer argument");
    const uint32_t K = g.K;
    if (K == 0 || K > MAXK)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_begin: K must be in [1, SHIFTER_MAX_VARIANTS]");
    if (misaligned(g.d_w, 16) || misaligned(g.d_w_sparse, 16) || misaligned(g.d_mask, 4) ||
        misaligned(g.d_thr, 8) || misaligned(g.d_w_out, 16) || (K > 1 && (g.cap_w & 3u)))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "portfolio_begin: arenas must be 16-byte aligned, masks 4-byte aligned, cap_w a "
                    "multiple of 4 for several variants");
    if ((g.d_w_sparse && K > 1 && g.w_stride < model->info.w_extent) ||
        (g.d_mask && K > 1 && g.mask_stride < model->info.n_prunable))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_begin: stride smaller than one variant");
    if (g.d_w_sparse == g.d_w)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_begin: cannot work in place");
    if (g.flags & ~SHIFTER_PAPER_FREEZE_RESIDUAL)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_begin: unknown flag bits");
    auto& pp = ctx->pending_portfolio;
    memset(&pp.pc, 0, sizeof pp.pc);
    uint32_t idx[MAXK], k_eff = 0;
    uint64_t zero_mask = 0;
    for (uint32_t k = 0; k < K; ++k) {
        if (g.h_n_prune[k] > model->info.n_prunable)
            return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_begin: prune count exceeds N");
        pp.pc.p[k] = g.h_n_prune[k];
        if (pp.pc.p[k] == 0) zero_mask |= 1ull << k; else idx[k_eff++] = k;
    }
    pp.buf = PortfolioBuffers{g.d_w, g.d_vecs, K, g.flags, g.d_thr, g.d_w_sparse, g.w_stride, g.d_mask,
                              g.mask_stride, g.d_out_alive, g.d_in_alive, g.d_group_alive, g.d_index_map,
                              g.d_keep, g.d_new_width, g.d_w_out, g.cap_w, g.d_vecs_out, g.cap_v};
    pp.model = model;
    pp.k_eff = k_eff;
    const auto& b = model->b;
    if (ctx->select_path == 0 && K == 1 && g.d_w_sparse && g.d_in_alive) {
        // one prune count: ranking, sparse arena, mask and flags in a single read
        pp.mode = 1;
        launch_spec_select(ctx, model, g.d_w, pp.pc.p[0], g.d_thr, g.d_w_sparse, g.d_mask, g.d_out_alive,
                           g.d_in_alive, b.dev_spec);
        if ((rc = after_launch(ctx, "portfolio_begin"))) return rc;
        launch_plan_and_gather(ctx, model, pp.buf, false, cut_positions(pp.pc, K));
    } else if (ctx->select_path == 0 && k_eff <= SPEC_MULTI_MAXK) {
        PruneCounts sp;
        MultiPerm perm;
        memset(&sp, 0, sizeof sp);
        memset(&perm, 0, sizeof perm);
        std::stable_sort(idx, idx + k_eff, [&](uint32_t x, uint32_t y) { return pp.pc.p[x] < pp.pc.p[y]; });
        for (uint32_t i = 0; i < k_eff; ++i) { sp.p[i] = pp.pc.p[idx[i]]; perm.v[i] = idx[i]; }
        pp.mode = 2;
        if (model->info.w_extent * 4 > ctx->fused_min_bytes) {
            // an arena beyond the last-level cache: ranking, masks and levels in one read of it
            // (the planning launch expands the levels into the variants' flags on the way)
            FusedBatch fb{K, g.d_w_sparse, g.w_stride, g.d_mask, g.mask_stride, g.d_out_alive, g.d_in_alive, true};
            launch_spec_multi(ctx, model, g.d_w, sp, perm, k_eff, zero_mask, g.d_thr, &fb);
            launch_plan_and_gather(ctx, model, pp.buf, true, cut_positions(pp.pc, K));
        } else {
            // a cache-sized arena: the counting pass, then the mask pass reads it again; the
            // planning launch expands the levels into the variants' flags on the way
            launch_spec_multi(ctx, model, g.d_w, sp, perm, k_eff, zero_mask, g.d_thr, nullptr, b.levels,
                              (uint32_t)(model->info.sum_out_ch + model->info.sum_in_ch));
            launch_mask_scan_batch_core(ctx, model, g.d_w, g.d_thr, K, g.d_w_sparse, g.w_stride, g.d_mask,
                                        g.mask_stride);
            launch_plan_and_gather(ctx, model, pp.buf, true, cut_positions(pp.pc, K));
        }
    } else {
        pp.mode = 3;
        if ((rc = portfolio_radix(ctx, model, pp.pc, pp.buf))) return rc;
    }
    if ((rc = after_launch(ctx, "portfolio_begin"))) return rc;
    pp.active = true;
    return SHIFTER_OK;
}

extern "C" int shifter_portfolio_end(shifter_ctx* ctx, shifter_threshold* h_thr,
                                     shifter_tensor_desc* h_out_tensors, shifter_vec_desc* h_out_vecs,
                                     uint64_t* h_elems_w, uint64_t* h_elems_v) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "portfolio_end: ctx is NULL");
    auto& pp = ctx->pending_portfolio;
    if (!pp.active) return fail(ctx, SHIFTER_ERR_INVALID_ARG, "portfolio_end: nothing to collect");
    pp.active = false;
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    const shifter_model* model = pp.model;
    const uint32_t K = pp.buf.k_var;
    int rc, decided = 0;
    if (pp.mode == 1) {
        if ((rc = spec_result_collect(ctx, model->b.host_spec, h_thr, &decided))) return rc;
    } else if (pp.mode == 2) {
        if ((rc = multi_result(ctx, model, pp.k_eff, K, h_thr, &decided, "portfolio_end"))) return rc;
    }
    if (!decided) {
        if (pp.mode != 3) {
            // the single pass could not decide: the multi-pass select, and every later step again
            if ((rc = portfolio_radix(ctx, model, pp.pc, pp.buf))) return rc;
        }
        ctx->last_path = 2;
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        const uint8_t* st = model->b.host_multi;
        uint32_t nan_seen;
        memcpy(&nan_seen, st, sizeof nan_seen);
        if (nan_seen)
            return fail(ctx, SHIFTER_ERR_NONFINITE, "portfolio_end: NaN among the prunable weights");
        if (h_thr) memcpy(h_thr, st + MULTI_MIRROR_REC_OFF, sizeof(shifter_threshold) * K);
    }
    return plan_readout(ctx, model, K, h_out_tensors, h_out_vecs, h_elems_w, h_elems_v);
}

extern "C" int shifter_compact_batch(shifter_ctx* ctx, const shifter_model* model, const float* d_w_sparse,
                                     uint64_t w_stride, const float* d_vecs, const uint32_t* d_keep,
                                     const uint32_t* d_new_width, uint32_t K, float* d_w_out,
                                     uint64_t cap_w, float* d_vecs_out, uint64_t cap_v,
                                     shifter_tensor_desc* h_out_tensors, shifter_vec_desc* h_out_vecs,
                                     uint64_t* h_elems_w, uint64_t* h_elems_v) {
    return compact_impl(ctx, model, d_w_sparse, w_stride, nullptr, d_vecs, d_keep, d_new_width, K,
                        d_w_out, cap_w, d_vecs_out, cap_v, h_out_tensors, h_out_vecs, h_elems_w,
                        h_elems_v);
}

extern "C" int shifter_compact_batch_masked(shifter_ctx* ctx, const shifter_model* model, const float* d_w,
                                            const shifter_threshold* d_thr, const float* d_vecs,
                                            const uint32_t* d_keep, const uint32_t* d_new_width,
                                            uint32_t K, float* d_w_out, uint64_t cap_w,
                                            float* d_vecs_out, uint64_t cap_v,
                                            shifter_tensor_desc* h_out_tensors,
                                            shifter_vec_desc* h_out_vecs, uint64_t* h_elems_w,
                                            uint64_t* h_elems_v) {
    if (!d_thr) return fail(ctx, SHIFTER_ERR_INVALID_ARG, "compact: d_thr is NULL");
    return compact_impl(ctx, model, d_w, 0, d_thr, d_vecs, d_keep, d_new_width, K, d_w_out, cap_w,
                        d_vecs_out, cap_v, h_out_tensors, h_out_vecs, h_elems_w, h_elems_v);
}

extern "C" int shifter_compact(shifter_ctx* ctx, const shifter_model* model, const float* d_w_sparse,
                               const float* d_vecs, const uint32_t* d_keep,
                               const uint32_t* d_new_width, float* d_w_out, uint64_t cap_w,
                               float* d_vecs_out, uint64_t cap_v,
                               shifter_tensor_desc* h_out_tensors, shifter_vec_desc* h_out_vecs,
                               uint64_t* h_elems_w, uint64_t* h_elems_v) {
    return shifter_compact_batch(ctx, model, d_w_sparse, 0, d_vecs, d_keep, d_new_width, 1, d_w_out, cap_w,
                                 d_vecs_out, cap_v, h_out_tensors, h_out_vecs, h_elems_w, h_elems_v);
}

extern "C" int shifter_profile_enable(shifter_ctx* ctx, int on) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "profile_enable: ctx is NULL");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    ctx->profiling = on != 0;
    return SHIFTER_OK;
}

extern "C" int shifter_profile_read(shifter_ctx* ctx, const char** names, uint32_t* counts,
                                    double* total_ms, uint32_t cap, uint32_t* n_out) {
    if (!ctx || !n_out) return fail(ctx, SHIFTER_ERR_INVALID_ARG, "profile_read: NULL argument");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    uint32_t cnt[K_COUNT] = {0};
    double ms[K_COUNT] = {0};
    for (auto& r : ctx->recs) {
        float t = 0;
        if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) {
            cnt[r.id]++;
            ms[r.id] += t;
        }
        ctx->pool.push_back(r.a);
        ctx->pool.push_back(r.b);
    }
    ctx->recs.clear();
    uint32_t n = 0;
    for (int i = 0; i < K_COUNT; ++i) {
        if (!cnt[i]) continue;
        if (n < cap && names && counts && total_ms) {
            names[n] = kKernelNames[i];
            counts[n] = cnt[i];
            total_ms[n] = ms[i];
        }
        ++n;
    }
    *n_out = n < cap ? n : cap;
    return SHIFTER_OK;
}

static uint64_t codec_chunks(uint64_t n_bytes) {
    return n_bytes == 0 ? 1 : (n_bytes + SHIFTER_CODEC_CHUNK - 1) / SHIFTER_CODEC_CHUNK;
}
static uint64_t codec_work_bytes(uint64_t n_chunks) {
    return codec_slots_offset(n_chunks) + n_chunks * (uint64_t)(SHIFTER_CODEC_CHUNK + 8u);
}

extern "C" int shifter_codec_layout(uint64_t n_bytes, uint64_t* h_n_chunks, uint64_t* h_work_bytes,
                                    uint64_t* h_stream_bound) {
    const uint64_t n_chunks = codec_chunks(n_bytes);
    if (h_n_chunks) *h_n_chunks = n_chunks;
    if (h_work_bytes) *h_work_bytes = codec_work_bytes(n_chunks);
    if (h_stream_bound) *h_stream_bound = n_bytes + 5u * n_chunks;   // every segment stored
    return SHIFTER_OK;
}

static int codec_enter(shifter_ctx* ctx, const char* fn) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, std::string(fn) + ": ctx is NULL");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    return SHIFTER_OK;
}

// Waits for the stream and reads what the call's last kernel wrote to the pinned mirror.
static int codec_result(shifter_ctx* ctx, uint64_t* total, uint64_t* status) {
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    const volatile uint64_t* mirror = ctx->h_codec;
    *total = mirror[0];
    *status = mirror[1];
    return SHIFTER_OK;
}

extern "C" int shifter_deflate(shifter_ctx* ctx, const void* d_in, uint64_t n_bytes, void* d_work,
                               uint64_t work_bytes, uint8_t* d_stream, uint64_t stream_cap,
                               uint64_t* d_seg_off, uint16_t* d_sub_bits, uint64_t* d_sub_marks,
                               uint64_t* h_stream_bytes) {
    int rc = codec_enter(ctx, "deflate");
    if (rc) return rc;
    if ((!d_in && n_bytes) || !d_work || !d_stream || !d_seg_off || !d_sub_bits || !d_sub_marks)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "deflate: NULL pointer argument");
    if (misaligned(d_in, 16) || misaligned(d_work, 256) || misaligned(d_stream, 16) ||
        misaligned(d_seg_off, 8) || misaligned(d_sub_bits, 2) || misaligned(d_sub_marks, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "deflate: input and stream must be 16-byte aligned, the workspace 256-byte aligned");
    const uint64_t n_chunks = codec_chunks(n_bytes);
    if (n_chunks >= (1ull << 31))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "deflate: input too large (2^31 chunks or more)");
    if (work_bytes < codec_work_bytes(n_chunks))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "deflate: workspace too small, needs " + std::to_string(codec_work_bytes(n_chunks)) + " bytes");
    HIP_TRY(ctx, (hipError_t)launch_deflate(ctx, static_cast<const uint8_t*>(d_in), n_bytes, (uint32_t)n_chunks,
                                            static_cast<uint8_t*>(d_work), d_stream, stream_cap, d_seg_off,
                                            d_sub_bits, d_sub_marks));
    if ((rc = after_launch(ctx, "deflate"))) return rc;
    if (!h_stream_bytes) return SHIFTER_OK;
    uint64_t total, status;
    if ((rc = codec_result(ctx, &total, &status))) return rc;
    *h_stream_bytes = total;
    if (status)
        return fail(ctx, SHIFTER_ERR_CAPACITY,
                    "deflate: the stream takes " + std::to_string(total) + " bytes, capacity " +
                        std::to_string(stream_cap));
    return SHIFTER_OK;
}

extern "C" int shifter_inflate(shifter_ctx* ctx, const uint8_t* d_stream, uint64_t stream_bytes,
                               const uint64_t* d_seg_off, const uint16_t* d_sub_bits,
                               const uint64_t* d_sub_marks, uint64_t n_bytes, void* d_out, int wait) {
    int rc = codec_enter(ctx, "inflate");
    if (rc) return rc;
    if (!d_stream || !d_seg_off || !d_sub_bits || !d_sub_marks || (!d_out && n_bytes))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "inflate: NULL pointer argument");
    if (misaligned(d_stream, 16) || misaligned(d_out, 16) || misaligned(d_seg_off, 8) ||
        misaligned(d_sub_bits, 2) || misaligned(d_sub_marks, 8))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "inflate: stream and output must be 16-byte aligned");
    const uint64_t n_chunks = codec_chunks(n_bytes);
    if (n_chunks >= (1ull << 31))
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "inflate: output too large (2^31 chunks or more)");
    if (stream_bytes < 5u * n_chunks)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "inflate: bad stream (shorter than its segments' headers)");
    HIP_TRY(ctx, (hipError_t)launch_inflate(ctx, d_stream, stream_bytes, d_seg_off, d_sub_bits, d_sub_marks,
                                            n_bytes, (uint32_t)n_chunks, static_cast<uint8_t*>(d_out)));
    if ((rc = after_launch(ctx, "inflate"))) return rc;
    if (!wait) return SHIFTER_OK;
    uint64_t total, status;
    if ((rc = codec_result(ctx, &total, &status))) return rc;
    if (status)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG,
                    "inflate: bad stream (segments, offsets and bit counts do not fit together)");
    return SHIFTER_OK;
}

extern "C" int shifter_codec_status(shifter_ctx* ctx, uint64_t* h_stream_bytes, uint32_t* h_bad) {
    if (!ctx) return fail(nullptr, SHIFTER_ERR_INVALID_ARG, "codec_status: ctx is NULL");
    const volatile uint64_t* mirror = ctx->h_codec;
    if (h_stream_bytes) *h_stream_bytes = mirror[0];
    if (h_bad) *h_bad = mirror[1] != 0;
    return SHIFTER_OK;
}

extern "C" int shifter_copy_f32(shifter_ctx* ctx, const float* d_src, float* d_dst, uint64_t n) {
    if (!ctx || !d_src || !d_dst) return fail(ctx, SHIFTER_ERR_INVALID_ARG, "copy_f32: NULL argument");
    if ((reinterpret_cast<uintptr_t>(d_src) | reinterpret_cast<uintptr_t>(d_dst)) & 15u)
        return fail(ctx, SHIFTER_ERR_INVALID_ARG, "copy_f32: pointers must be 16-byte aligned");
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    launch_copy(ctx, d_src, d_dst, n);
    return after_launch(ctx, "copy_f32");
}
