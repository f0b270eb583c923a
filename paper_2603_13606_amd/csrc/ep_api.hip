// C-ABI entry points: group / handle lifetime, argument validation, and the
// translation of tensor descriptors into kernel arguments (Sec. III-A..E).
// Host code only; every step of the data path runs in the kernels of
// ep_layout.hip, ep_dispatch.hip, ep_dedup.hip, ep_combine.hip and ep_staged.hip.
#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "ep_internal.h"

using namespace ep;

namespace {

constexpr int kSlabAlign = 64;  // ints; every device array starts on a 256-byte boundary

struct Slab {
    int32_t* base = nullptr;
    // carved arrays
    int32_t *totals, *expert_count, *expert_kept, *expert_offset, *own_prefix;
    int32_t *rank_pair_count, *rank_token_count, *rank_offset;
    uint32_t* pub;   // per-chunk bin sums of the layout kernel (kMaxChunks rows of W words)
    uint32_t* ctl;   // its generation / arrival words; pub and ctl are zeroed when the slab is made
    int32_t *slot, *dst_row, *rank_row, *sorted_token, *sorted_k, *sorted_row, *entry_rank, *run_start;
    uint8_t* quant;  // FP8 staging copy of the tokens (groups that quantise ahead), or nullptr
    // receiving side of the once-per-rank path (only carved for EP_PATH_RANK_DEDUP)
    int32_t *recv_count, *recv_kept, *recv_dst_row;
    // what the receiving side of a staged call learns from the coordination counters
    int32_t *recv_rank_count, *recv_rank_offset;
    // the stream of the last call of the handle that held the slab before (valid once `used`), and
    // the event through which a layout on another stream waits for the work queued there
    hipStream_t last_stream = nullptr;
    hipEvent_t reuse_event = nullptr;
    bool used = false;
};

}  // namespace

struct ep_group_s {
    ep_group_config_t cfg;
    int L, L_shift, K_shift, W, bits_e, bits_r;
    int C;       // slots per sub-region (LL)
    int64_t slab_ints;
    ep_alloc_fn alloc_fn;
    ep_free_fn free_fn;
    std::mutex mu;
    std::vector<Slab> free_slabs;
    int live_handles = 0;
    int device = 0;
    // staging windows of the once-per-rank path, one per buffer set
    uint8_t* staging[2] = {nullptr, nullptr};
    int64_t staging_slots = 0;
    int64_t hdr_bytes = 0, msg_bytes = 0;   // header and whole message (header + 2H)
    int64_t msg_stride = 0, msg_lead = 0;    // slot pitch, and where the message starts in its slot
    // staged execution: buffer sets (0 = not available), coordination counters
    // [E dispatch | R once-per-rank | E combine] and (t,k)-indexed combine staging per set
    int nsets = 0, next_set = 0;
    int32_t* signals[2] = {nullptr, nullptr};
    uint16_t* comb_stage[2] = {nullptr, nullptr};
    // Padded windows, destination-ordered dispatch: what the capacity kept and cut in the most
    // recent layout that has finished, low word kept, high word dropped, written by the layout
    // kernel into mapped host memory (one 8-byte store).  ep_dispatch reads it as a hint: when
    // most entries were cut, the rows that remain sit in a few long runs and the token walk
    // copies them faster.  Either walk writes the same bytes; a stale hint costs time only.
    int64_t* drop_hint = nullptr;      // host address
    int64_t* drop_hint_dev = nullptr;  // the same word as the kernels address it
    int sig_ints() const { return 2 * cfg.num_experts + cfg.num_ranks; }
    int32_t* sig_dispatch(int set) const { return signals[set]; }
    int32_t* sig_rank(int set) const { return signals[set] + cfg.num_experts; }
    int32_t* sig_combine(int set) const { return signals[set] + cfg.num_experts + cfg.num_ranks; }
};

enum { PENDING_NONE = 0, PENDING_DISPATCH_DIRECT, PENDING_DISPATCH_DEDUP, PENDING_COMBINE };

struct ep_handle_s {
    ep_group_s* group;
    Slab slab;
    int T;
    hipStream_t last_stream;
    const int32_t* expert_base;  // as given to ep_layout (borrowed), or nullptr
    bool has_runs = false;       // the layout filled slab.run_start
    int nwc = 0;                 // wave-chunks of the layout plan
    int chunk_entries = 0;       // entries per wave-chunk
    const void* warm_x = nullptr;  // tokens the layout launch has read into cache (ep_layout_prefetch)
    int64_t warm_stride = 0;
    int warm_rows = 0;
    const void* quant_x = nullptr;  // tokens the layout launch has quantised into slab.quant (all T rows)
    int64_t quant_stride = 0;
    // receive phase of a staged (send_only) call, run by ep_complete
    int pending = PENDING_NONE;
    int pending_set = 0;
    int32_t* pending_recv_count = nullptr;
    DedupRankArgs pending_rank;
    DedupFanoutArgs pending_fanout;
    CombineArgs pending_combine;
};

namespace {

int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

int bits_for(int n) {  // bits needed to write any value in [0, n)
    int b = 0;
    while ((1 << b) < n) ++b;
    return b;
}

ep_result_t dev_alloc(ep_group_s* g, void** p, size_t bytes) {
    if (g->alloc_fn) {
        if (g->alloc_fn(p, bytes) != 0 || !*p) return EP_ERR_NOMEM;
        if ((uintptr_t)*p & 255u) {  // the kernels rely on 256-byte aligned arrays
            g->free_fn(*p);
            *p = nullptr;
            return EP_ERR_INVALID_ARG;
        }
        return EP_SUCCESS;
    }
    hipError_t e = hipMalloc(p, bytes);
    if (e == hipErrorOutOfMemory) return EP_ERR_NOMEM;
    return e == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

void dev_free(ep_group_s* g, void* p) {
    if (!p) return;
    if (g->free_fn) g->free_fn(p);
    else (void)hipFree(p);
}

int64_t carve(int64_t* cursor, int64_t ints) {
    const int64_t at = *cursor;
    *cursor = round_up(at + ints, kSlabAlign);
    return at;
}

// Lays the handle arrays out inside one allocation; with base == nullptr only the size is computed.
int64_t carve_slab(const ep_group_s* g, Slab* s, int32_t* base) {
    const int E = g->cfg.num_experts, R = g->cfg.num_ranks;
    const int64_t nB = (int64_t)g->cfg.max_tokens_per_rank * g->cfg.top_k;
    int64_t cur = 0;
    const int64_t o_tot = carve(&cur, kTotalsWords), o_ec = carve(&cur, E), o_ek = carve(&cur, E);
    const int64_t o_eo = carve(&cur, E + 1), o_op = carve(&cur, E + 1), o_rp = carve(&cur, R);
    const int64_t o_rt = carve(&cur, R), o_ro = carve(&cur, R + 1);
    const int64_t o_h = carve(&cur, (int64_t)kMaxChunks * g->W), o_ctl = carve(&cur, kLayoutCtlWords);
    const bool runs = g->cfg.dispatch_order != EP_ORDER_TOKEN && g->cfg.dispatch_path == EP_PATH_DIRECT;
    const int64_t o_rn = runs ? carve(&cur, (int64_t)(kMaxWaveChunks + 1) * E) : 0;
    const int64_t o_sl = carve(&cur, nB), o_dr = carve(&cur, nB), o_rr = carve(&cur, nB);
    const int64_t o_st = carve(&cur, nB), o_sk = carve(&cur, nB), o_sr = carve(&cur, nB), o_er = carve(&cur, nB);
    const bool dedup = g->cfg.dispatch_path == EP_PATH_RANK_DEDUP;
    const int64_t o_vc = dedup ? carve(&cur, E) : 0, o_vk = dedup ? carve(&cur, E) : 0;
    const int64_t o_vr = dedup ? carve(&cur, g->staging_slots * g->cfg.top_k) : 0;
    const int64_t o_rc = carve(&cur, R), o_rf = carve(&cur, R + 1);
    const bool ahead = g->cfg.quantize_ahead != 0;
    const int64_t o_q = ahead ? carve(&cur, (int64_t)g->cfg.max_tokens_per_rank * quant_row_pitch(g->cfg.hidden) / 4) : 0;
    if (base && s) {
        s->base = base;
        s->totals = base + o_tot; s->expert_count = base + o_ec; s->expert_kept = base + o_ek;
        s->expert_offset = base + o_eo; s->own_prefix = base + o_op; s->rank_pair_count = base + o_rp;
        s->rank_token_count = base + o_rt; s->rank_offset = base + o_ro;
        s->pub = (uint32_t*)(base + o_h); s->ctl = (uint32_t*)(base + o_ctl); s->slot = base + o_sl; s->dst_row = base + o_dr; s->rank_row = base + o_rr;
        s->sorted_token = base + o_st; s->sorted_k = base + o_sk; s->sorted_row = base + o_sr;
        s->entry_rank = base + o_er; s->run_start = runs ? base + o_rn : nullptr;
        s->recv_count = dedup ? base + o_vc : nullptr; s->recv_kept = dedup ? base + o_vk : nullptr;
        s->recv_dst_row = dedup ? base + o_vr : nullptr;
        s->recv_rank_count = base + o_rc; s->recv_rank_offset = base + o_rf;
        s->quant = ahead ? (uint8_t*)(base + o_q) : nullptr;
    }
    return cur;
}

void free_slab(ep_group_s* g, Slab& s) {
    if (s.reuse_event) (void)hipEventDestroy(s.reuse_event);
    dev_free(g, s.base);
}

// A new slab; the words through which the layout workgroups talk to each other must start
// out zero (pub and ctl are adjacent), which a small fill kernel on `stream` sees to.
ep_result_t new_slab(ep_group_s* g, Slab* s, hipStream_t stream) {
    void* p = nullptr;
    ep_result_t r = dev_alloc(g, &p, sizeof(int32_t) * (size_t)g->slab_ints);
    if (r != EP_SUCCESS) return r;
    carve_slab(g, s, (int32_t*)p);
    const int64_t ints = (int32_t*)(s->ctl + kLayoutCtlWords) - (int32_t*)s->pub;
    if (hipEventCreateWithFlags(&s->reuse_event, hipEventDisableTiming) != hipSuccess) {
        s->reuse_event = nullptr;
        dev_free(g, p);
        return EP_ERR_HIP;
    }
    if (launch_clear_counts((int32_t*)s->pub, (int)ints, stream) != hipSuccess) {
        (void)hipStreamSynchronize(stream);  // nothing queued may still write the memory given back below
        free_slab(g, *s);
        return EP_ERR_HIP;
    }
    s->used = false;
    return EP_SUCCESS;
}

const ep_tensor_t* find_tag(const ep_tensor_t* ts, int n, int tag, int tag2 = -1, int tag3 = -1) {
    for (int i = 0; i < n; ++i)
        if (ts[i].tag == tag || ts[i].tag == tag2 || ts[i].tag == tag3) return &ts[i];
    return nullptr;
}

bool has_scales(const ep_tensor_t* ts, int n) {
    for (int i = 0; i < n; ++i)
        if (ts[i].tag == EP_TAG_SCALES) return true;
    return false;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// 2-D [rows, cols] tensor of `dtype`, innermost stride 1.
bool check_2d(const ep_tensor_t* t, int dtype, int64_t rows, int64_t cols, bool rows_exact) {
    if (!t || t->ndim != 2 || t->dtype != dtype) return false;
    if (t->shape[1] != cols || t->stride[1] != 1 || t->stride[0] < cols) return false;
    if (rows_exact ? t->shape[0] != rows : t->shape[0] < rows) return false;
    if (t->shape[0] > 0 && !t->data) return false;
    return true;
}

bool check_1d(const ep_tensor_t* t, int dtype, int64_t n) {
    if (!t || t->ndim != 1 || t->dtype != dtype || t->shape[0] < n || t->stride[0] != 1) return false;
    return t->data != nullptr || t->shape[0] == 0;
}

// Token windows: HT [rows_cap, H]; LL [E, C, H].  Fills a WindowDesc.  Rows must start on
// 16-byte boundaries: outer strides are multiples of `align` elements (8 for bf16, 16 for fp8).
bool window_from_tensor(const ep_group_s* g, const ep_tensor_t* t, WindowDesc* w, int dtype = EP_DTYPE_BF16) {
    const int H = g->cfg.hidden;
    const int align = dtype == EP_DTYPE_BF16 ? 8 : 16;
    if (!t || t->dtype != dtype || !aligned16(t->data)) return false;
    if (g->cfg.mode == EP_MODE_LL) {
        if (t->ndim != 3 || t->shape[0] != g->cfg.num_experts || t->shape[1] != g->C || t->shape[2] != H)
            return false;
        if (t->stride[2] != 1 || t->stride[1] < H || t->stride[1] % align || t->stride[0] % align) return false;
        if (t->stride[0] < 0) return false;
        if (!t->data) return false;
        w->stride0 = t->stride[0];
        w->stride1 = t->stride[1];
        w->rows_cap = (int64_t)g->cfg.num_experts * g->C;
        w->padded = 1;
        w->C = g->C;
    } else {
        if (t->ndim != 2 || t->shape[1] != H || t->stride[1] != 1 || t->stride[0] < H || t->stride[0] % align)
            return false;
        if (t->shape[0] < 0 || t->shape[0] > 0x7fffffffLL) return false;
        if (t->shape[0] > 0 && !t->data) return false;
        w->stride0 = t->stride[0];
        w->stride1 = 0;
        w->rows_cap = t->shape[0];
        w->padded = 0;
        w->C = 1;
    }
    w->base = (uint16_t*)t->data;
    return true;
}

// Checks every field of a group configuration (the rules ep.h states for ep_group_config_t).
ep_result_t validate_config(const ep_group_config_t* cfg) {
    if (!cfg || cfg->size != sizeof(ep_group_config_t)) return EP_ERR_INVALID_ARG;
    const int R = cfg->num_ranks, E = cfg->num_experts, H = cfg->hidden, K = cfg->top_k;
    if (R < 1 || cfg->my_rank < 0 || cfg->my_rank >= R) return EP_ERR_INVALID_ARG;
    if (E < 1 || E > kMaxExperts || E % R != 0) return EP_ERR_INVALID_ARG;
    if (H < 8 || (2 * (int64_t)H) % 16 != 0) return EP_ERR_INVALID_ARG;
    if (K < 1 || K > kMaxTopK) return EP_ERR_INVALID_ARG;
    if (cfg->max_tokens_per_rank < 1 || (int64_t)cfg->max_tokens_per_rank * K > (1 << 28)) return EP_ERR_INVALID_ARG;
    if (cfg->dtype != EP_DTYPE_BF16) return EP_ERR_UNSUPPORTED;
    if (cfg->mode != EP_MODE_LL && cfg->mode != EP_MODE_HT) return EP_ERR_INVALID_ARG;
    if (cfg->dispatch_path != EP_PATH_DIRECT && cfg->dispatch_path != EP_PATH_RANK_DEDUP) return EP_ERR_INVALID_ARG;
    if (cfg->slots_per_subregion < 0 || cfg->max_handles < 0) return EP_ERR_INVALID_ARG;
    if (cfg->staged_buffers < 0 || cfg->staged_buffers > 2) return EP_ERR_INVALID_ARG;
    if (cfg->ranks_per_node < 0) return EP_ERR_INVALID_ARG;
    if (cfg->dispatch_order < EP_ORDER_TOKEN || cfg->dispatch_order > EP_ORDER_DESTINATION_RESIDENT) return EP_ERR_INVALID_ARG;
    if (cfg->quantize_ahead != 0 && cfg->quantize_ahead != 1) return EP_ERR_INVALID_ARG;
    if (cfg->quantize_ahead && (cfg->dispatch_order != EP_ORDER_DESTINATION || cfg->dispatch_path != EP_PATH_DIRECT || H % 128 != 0))
        return EP_ERR_INVALID_ARG;
    const int C = cfg->slots_per_subregion ? cfg->slots_per_subregion : cfg->max_tokens_per_rank;
    if (cfg->mode == EP_MODE_LL && (int64_t)E * C > 0x7fffffffLL) return EP_ERR_INVALID_ARG;
    return EP_SUCCESS;
}

int log2_exact(int v) {  // log2(v) when v is a power of two, else -1
    for (int b = 0; b < 31; ++b)
        if ((1 << b) == v) return b;
    return -1;
}

ep_result_t sync_and_read_totals(ep_handle_s* h, int32_t* tot) {
    if (hipStreamSynchronize(h->last_stream) != hipSuccess) return EP_ERR_HIP;
    if (hipMemcpy(tot, h->slab.totals, sizeof(int32_t) * kTotalsWords, hipMemcpyDeviceToHost) != hipSuccess)
        return EP_ERR_HIP;
    return EP_SUCCESS;
}


// ---- scratch of ep_layout_static: one array per GPU, part of the library image, so the
// entry point never allocates.  It holds what ep_layout keeps in the handle's slab beyond
// the arrays a caller asks for: the per-chunk bin sums through which the layout workgroups
// talk to each other, their generation words, and the per-expert positions in the
// expert-sorted entry list.
constexpr int64_t kStaticPubInts = (int64_t)kMaxChunks * (2 * kMaxExperts + 2);
constexpr int64_t kStaticScratchInts = kStaticPubInts + kSlabAlign + kMaxExperts + 1 + kSlabAlign;
static __device__ __align__(256) int32_t scratch[kStaticScratchInts];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
int32_t* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, once known

// Device address of this GPU's copy of the scratch array (the array's name is only a
// host-side stand-in for it).
ep_result_t static_scratch(int32_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return EP_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return EP_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return EP_ERR_HIP;
        g_scratch_ptr[dev] = (int32_t*)p;
    }
    *out = g_scratch_ptr[dev];
    return EP_SUCCESS;
}

}  // namespace

extern "C" {

const char* ep_error_string(ep_result_t code) {
    switch (code) {
        case EP_SUCCESS: return "success";
        case EP_ERR_INVALID_ARG: return "invalid argument";
        case EP_ERR_INVALID_ROUTING: return "expert ids outside [0, num_experts) in topk_idx";
        case EP_ERR_OVERFLOW: return "destination rows beyond the output tensor";
        case EP_ERR_UNSUPPORTED: return "unsupported feature";
        case EP_ERR_BUSY: return "group still has live handles";
        case EP_ERR_HIP: return "HIP runtime error";
        case EP_ERR_NOMEM: return "out of device memory";
        case EP_ERR_TIMEOUT: return "coordination counters were not published within the spin limit";
    }
    return "unknown error code";
}

int32_t ep_version(void) { return 400; }  // 0.4.0: calibration fill / read and ep_combine_plan added (0.3.0: ep_group_config_t and ep_group_info_t grew)

#ifndef EP_BUILD_ID_STRING
#define EP_BUILD_ID_STRING "unknown"
#endif
// the marker lets build tooling read the id from the file without loading it
static const char kBuildId[] = "EP_BUILD_ID=" EP_BUILD_ID_STRING;
const char* ep_build_id(void) { return kBuildId + sizeof("EP_BUILD_ID=") - 1; }

ep_result_t ep_layout_plan(int64_t num_entries, int32_t* passes, int32_t* wave_chunks) {
    if (!passes || !wave_chunks || num_entries < 0 || num_entries > (1 << 28)) return EP_ERR_INVALID_ARG;
    int p = 0, w = 0;
    plan_layout((int)num_entries, &p, &w);
    *passes = p;
    *wave_chunks = w;
    return EP_SUCCESS;
}

ep_result_t ep_dispatch_plan(const ep_group_config_t* cfg, int64_t num_tokens, int64_t prefetched_rows,
                             ep_dispatch_plan_t* plan) {
    if (!cfg || !plan || cfg->size != sizeof(ep_group_config_t)) return EP_ERR_INVALID_ARG;
    if (num_tokens < 0 || prefetched_rows < 0 || cfg->top_k < 1 || cfg->hidden < 8 || cfg->num_experts < 1 ||
        num_tokens * cfg->top_k > (1 << 28))
        return EP_ERR_INVALID_ARG;
    DispatchPlan d;
    // layouts of more than 1024 entries record the runs whenever the group asks for them
    const bool have_runs = cfg->dispatch_order != EP_ORDER_TOKEN && cfg->dispatch_path == EP_PATH_DIRECT;
    plan_dispatch((int)num_tokens, cfg->top_k, cfg->hidden, cfg->num_experts, cfg->dispatch_order, have_runs,
                  (int)std::min<int64_t>(prefetched_rows, num_tokens), &d);
    plan->run_order = d.run_order; plan->group = d.group; plan->blocks = d.blocks;
    plan->block_entries = d.block_entries; plan->splits = d.splits; plan->slice_units = d.piece;
    plan->threads_per_piece = d.run_order ? 1 << d.tpr_shift : 0;
    plan->blocks_per_launch = d.blocks_per_launch; plan->launches = d.launches; plan->read_passes = d.read_passes;
    return EP_SUCCESS;
}

ep_result_t ep_combine_plan(const ep_group_config_t* cfg, int64_t num_tokens, int32_t compute_units, ep_combine_plan_t* plan) {
    if (!cfg || !plan || cfg->size != sizeof(ep_group_config_t)) return EP_ERR_INVALID_ARG;
    if (num_tokens < 0 || compute_units < 0 || cfg->hidden < 8 || cfg->hidden % 8 || num_tokens > (1 << 28)) return EP_ERR_INVALID_ARG;
    CombinePlan p;
    plan_combine(num_tokens, cfg->hidden, cfg->ranks_per_node, compute_units, &p);
    plan->segments_per_wavefront = p.segments;
    plan->whole_row = p.whole_row;
    plan->workgroups = p.workgroups;
    return EP_SUCCESS;
}

ep_result_t ep_calibration_copy(void* dst, const void* src, size_t bytes, ep_stream_t stream) {
    if (!dst || !src || bytes % 16 || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return EP_ERR_INVALID_ARG;
    return launch_calibration_copy(dst, src, bytes, (hipStream_t)stream) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

ep_result_t ep_calibration_fill(void* dst, size_t bytes, ep_stream_t stream) {
    if (!dst || bytes % 16 || ((uintptr_t)dst & 15u)) return EP_ERR_INVALID_ARG;
    return launch_calibration_fill(dst, bytes, (hipStream_t)stream) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

ep_result_t ep_calibration_read(const void* src, size_t bytes, void* sink, ep_stream_t stream) {
    if (!src || !sink || bytes % 16 || ((uintptr_t)src & 15u) || ((uintptr_t)sink & 3u)) return EP_ERR_INVALID_ARG;
    return launch_calibration_read(src, bytes, (uint32_t*)sink, (hipStream_t)stream) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

ep_result_t ep_group_create(ep_group_t* group, const ep_group_config_t* cfg, ep_stream_t stream,
                            ep_alloc_fn alloc_fn, ep_free_fn free_fn) {
    if (!group || !cfg) return EP_ERR_INVALID_ARG;
    if ((alloc_fn == nullptr) != (free_fn == nullptr)) return EP_ERR_INVALID_ARG;
    if (ep_result_t v = validate_config(cfg); v != EP_SUCCESS) return v;
    const int R = cfg->num_ranks, E = cfg->num_experts, H = cfg->hidden, K = cfg->top_k;
    const int C = cfg->slots_per_subregion ? cfg->slots_per_subregion : cfg->max_tokens_per_rank;

    ep_group_s* g = new (std::nothrow) ep_group_s();
    if (!g) return EP_ERR_NOMEM;
    g->cfg = *cfg;
    g->C = C;
    g->L = E / R;
    g->L_shift = log2_exact(g->L);
    g->K_shift = log2_exact(K);
    g->W = E + 2 + R;
    g->bits_e = bits_for(E);
    g->bits_r = bits_for(R);
    g->alloc_fn = alloc_fn;
    g->free_fn = free_fn;
    g->hdr_bytes = round_up(4 + 8 * (int64_t)K, 16);
    g->msg_bytes = g->hdr_bytes + 2 * (int64_t)H;
    // the token data of a message starts on a 256-byte boundary of its slot
    g->msg_lead = round_up(g->hdr_bytes, 256) - g->hdr_bytes;
    g->msg_stride = round_up(g->msg_lead + g->msg_bytes, 256);
    if (cfg->dispatch_path == EP_PATH_RANK_DEDUP) {
        // LL: B slots per destination rank (Sec. IV-D, O(N*B*P)); HT: a token reaches at
        // most min(R, K) ranks, windows are packed back to back.
        const int64_t B = cfg->max_tokens_per_rank;
        g->staging_slots = cfg->mode == EP_MODE_LL ? (int64_t)R * B : B * (R < K ? R : K);
        if (g->staging_slots * K > (1 << 28)) { delete g; return EP_ERR_INVALID_ARG; }
    }
    g->slab_ints = carve_slab(g, nullptr, nullptr);
    if (hipGetDevice(&g->device) != hipSuccess) { delete g; return EP_ERR_HIP; }
    g->nsets = cfg->staged_buffers;
    auto fail = [&](ep_result_t r) {
        (void)hipStreamSynchronize((hipStream_t)stream);  // fill kernels queued so far write what is freed here
        for (int i = 0; i < 2; ++i) { dev_free(g, g->staging[i]); dev_free(g, g->signals[i]); dev_free(g, g->comb_stage[i]); }
        for (auto& f : g->free_slabs) free_slab(g, f);
        if (g->drop_hint) (void)hipHostFree(g->drop_hint);
        delete g;
        return r;
    };
    if (cfg->mode == EP_MODE_LL && cfg->dispatch_order != EP_ORDER_TOKEN && cfg->dispatch_path == EP_PATH_DIRECT) {
        void *hp = nullptr, *dp = nullptr;
        if (hipHostMalloc(&hp, 64, hipHostMallocMapped) != hipSuccess) return fail(EP_ERR_NOMEM);
        g->drop_hint = (int64_t*)hp;
        *g->drop_hint = 0;
        if (hipHostGetDevicePointer(&dp, hp, 0) != hipSuccess) return fail(EP_ERR_HIP);
        g->drop_hint_dev = (int64_t*)dp;
    }
    const int nstaging = g->staging_slots > 0 ? (g->nsets > 1 ? g->nsets : 1) : 0;
    for (int i = 0; i < nstaging; ++i) {
        void* p = nullptr;
        ep_result_t r = dev_alloc(g, &p, (size_t)(g->staging_slots * g->msg_stride));
        if (r != EP_SUCCESS) return fail(r);
        g->staging[i] = (uint8_t*)p;
    }
    for (int i = 0; i < g->nsets; ++i) {
        void* p = nullptr;
        ep_result_t r = dev_alloc(g, &p, sizeof(int32_t) * (size_t)g->sig_ints());
        if (r != EP_SUCCESS) return fail(r);
        g->signals[i] = (int32_t*)p;
        if (launch_clear_counts(g->signals[i], g->sig_ints(), (hipStream_t)stream) != hipSuccess) return fail(EP_ERR_HIP);
        r = dev_alloc(g, &p, (size_t)cfg->max_tokens_per_rank * K * H * 2);
        if (r != EP_SUCCESS) return fail(r);
        g->comb_stage[i] = (uint16_t*)p;
    }
    if (g->nsets > 0 && hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return fail(EP_ERR_HIP);
    const int nslabs = cfg->max_handles ? cfg->max_handles : 2;
    for (int i = 0; i < nslabs; ++i) {
        Slab s;
        ep_result_t r = new_slab(g, &s, (hipStream_t)stream);
        if (r != EP_SUCCESS) return fail(r);
        g->free_slabs.push_back(s);
    }
    // the slabs were zeroed on `stream`; layouts may come on any stream
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return fail(EP_ERR_HIP);
    *group = g;
    return EP_SUCCESS;
}

ep_result_t ep_group_destroy(ep_group_t g, ep_stream_t stream) {
    if (!g) return EP_ERR_INVALID_ARG;
    {
        std::lock_guard<std::mutex> lk(g->mu);
        if (g->live_handles > 0) return EP_ERR_BUSY;
    }
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return EP_ERR_HIP;
    // work of destroyed handles may still be running on other streams: wait for it, slab by slab (a stream
    // the caller has destroyed in the meantime had to finish its work then; its error is ignored)
    for (auto& s : g->free_slabs) {
        if (s.used && s.last_stream != (hipStream_t)stream && s.reuse_event &&
            hipEventRecord(s.reuse_event, s.last_stream) == hipSuccess)
            (void)hipEventSynchronize(s.reuse_event);
    }
    (void)hipGetLastError();
    for (auto& s : g->free_slabs) free_slab(g, s);
    for (int i = 0; i < 2; ++i) { dev_free(g, g->staging[i]); dev_free(g, g->signals[i]); dev_free(g, g->comb_stage[i]); }
    if (g->drop_hint) (void)hipHostFree(g->drop_hint);
    delete g;
    return EP_SUCCESS;
}

ep_result_t ep_group_query(ep_group_t g, ep_group_info_t* info) {
    if (!g || !info) return EP_ERR_INVALID_ARG;
    const ep_group_config_t& c = g->cfg;
    info->num_ranks = c.num_ranks; info->my_rank = c.my_rank; info->num_experts = c.num_experts;
    info->experts_per_rank = g->L; info->hidden = c.hidden; info->top_k = c.top_k;
    info->max_tokens_per_rank = c.max_tokens_per_rank; info->mode = c.mode;
    info->slots_per_subregion = g->C; info->dispatch_path = c.dispatch_path;
    info->row_bytes = 2 * (int64_t)c.hidden;
    info->msg_header_bytes = g->hdr_bytes;
    info->msg_bytes = g->msg_bytes;
    info->msg_stride = g->msg_stride;
    info->msg_lead = g->msg_lead;
    const int64_t hint = g->drop_hint ? __atomic_load_n(g->drop_hint, __ATOMIC_RELAXED) : 0;
    info->hint_rows_kept = (int32_t)(hint & 0xffffffffLL);
    info->hint_rows_dropped = (int32_t)(hint >> 32);
    info->staging_slots = g->staging_slots;
    info->staging = g->staging[0];
    info->staged_buffers = g->nsets;
    for (int i = 0; i < 2; ++i) {
        info->staging_sets[i] = g->staging[i];
        info->signals[i] = g->signals[i];
        info->combine_staging[i] = g->comb_stage[i];
    }
    const int64_t B = c.max_tokens_per_rank, P = info->row_bytes;
    info->footprint_per_expert_bytes = 2 * (int64_t)c.num_experts * B * P;
    info->footprint_optimised_bytes = (int64_t)c.num_ranks * B * P + B * c.top_k * P;
    {
        std::lock_guard<std::mutex> lk(g->mu);
        info->live_handles = g->live_handles;
    }
    return EP_SUCCESS;
}

ep_result_t ep_layout(ep_handle_t* handle, ep_group_t g, const ep_tensor_t* topk_idx,
                      const ep_tensor_t* expert_base, ep_stream_t stream) {
    return ep_layout_prefetch(handle, g, topk_idx, expert_base, nullptr, stream);
}

// Validates a layout call, takes a slab for the new handle and fills the kernel arguments;
// launches nothing.  On success *handle is live (ep_handle_destroy releases it).
static ep_result_t prepare_layout(ep_handle_t* handle, ep_group_t g, const ep_tensor_t* topk_idx,
                                  const ep_tensor_t* expert_base, const ep_tensor_t* tokens, ep_stream_t stream,
                                  LayoutArgs* args) {
    if (!handle || !g || !topk_idx) return EP_ERR_INVALID_ARG;
    const ep_group_config_t& c = g->cfg;
    if (topk_idx->tag != EP_TAG_TOPK_IDX || topk_idx->ndim != 2 || topk_idx->dtype != EP_DTYPE_I32)
        return EP_ERR_INVALID_ARG;
    const int64_t T = topk_idx->shape[0];
    if (T < 0 || T > c.max_tokens_per_rank) return EP_ERR_INVALID_ARG;
    if (!check_2d(topk_idx, EP_DTYPE_I32, T, c.top_k, true)) return EP_ERR_INVALID_ARG;
    if (expert_base) {
        if (c.mode != EP_MODE_HT) return EP_ERR_INVALID_ARG;
        if (expert_base->tag != EP_TAG_EXPERT_BASE || !check_1d(expert_base, EP_DTYPE_I32, c.num_experts) ||
            !expert_base->data)
            return EP_ERR_INVALID_ARG;
    }
    if (tokens) {
        if (tokens->tag != EP_TAG_TOKENS || !check_2d(tokens, EP_DTYPE_BF16, T, c.hidden, true) ||
            tokens->stride[0] % 8 || !aligned16(tokens->data))
            return EP_ERR_INVALID_ARG;
    }
    ep_handle_s* h = new (std::nothrow) ep_handle_s();
    if (!h) return EP_ERR_NOMEM;
    {
        std::lock_guard<std::mutex> lk(g->mu);
        if (!g->free_slabs.empty()) {
            h->slab = g->free_slabs.back();
            g->free_slabs.pop_back();
        } else {
            ep_result_t r = new_slab(g, &h->slab, (hipStream_t)stream);
            if (r != EP_SUCCESS) { delete h; return r; }
        }
        g->live_handles += 1;
    }
    h->group = g;
    h->T = (int)T;
    h->last_stream = (hipStream_t)stream;
    // The slab may still be read by work of the handle that held it before, queued on another
    // stream: this stream then waits for everything queued there so far (no host wait; work of
    // that handle on the same stream is ordered by the stream itself).
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (h->slab.used && h->slab.last_stream != (hipStream_t)stream &&
        hipStreamIsCapturing((hipStream_t)stream, &capturing) == hipSuccess && capturing == hipStreamCaptureStatusNone) {
        // (a stream under graph capture cannot wait for work outside its graph: there the caller
        // orders the capture after that work)
        if (hipEventRecord(h->slab.reuse_event, h->slab.last_stream) != hipSuccess ||
            hipStreamWaitEvent((hipStream_t)stream, h->slab.reuse_event, 0) != hipSuccess) {
            ep_handle_destroy(h);
            return EP_ERR_HIP;
        }
    }
    h->expert_base = expert_base ? (const int32_t*)expert_base->data : nullptr;

    LayoutArgs a;
    a.topk = (const int32_t*)topk_idx->data;
    a.topk_stride = topk_idx->stride[0];
    a.expert_base = expert_base ? (const int32_t*)expert_base->data : nullptr;
    a.T = (int)T; a.K = c.top_k; a.E = c.num_experts; a.R = c.num_ranks; a.L = g->L; a.L_shift = g->L_shift; a.K_shift = g->K_shift;
    a.padded = c.mode == EP_MODE_LL; a.C = g->C; a.C_rank = c.max_tokens_per_rank;
    a.n = (int)(T * c.top_k);
    plan_layout(a.n, &a.passes, &a.nwc);
    a.W = g->W; a.bits_e = g->bits_e; a.bits_r = g->bits_r;
    const Slab& s = h->slab;
    a.pub = s.pub; a.ctl = s.ctl; a.expert_count = s.expert_count; a.expert_kept = s.expert_kept;
    a.expert_offset = s.expert_offset; a.own_prefix = s.own_prefix; a.rank_pair_count = s.rank_pair_count;
    a.rank_token_count = s.rank_token_count; a.rank_offset = s.rank_offset; a.totals = s.totals;
    a.slot = s.slot; a.dst_row = s.dst_row; a.rank_row = s.rank_row; a.sorted_token = s.sorted_token;
    a.sorted_k = s.sorted_k; a.sorted_row = s.sorted_row;
    a.entry_rank = s.entry_rank;
    // the table of run starts is only wanted by the destination-ordered dispatch
    a.run_start = (c.dispatch_order != EP_ORDER_TOKEN && c.dispatch_path == EP_PATH_DIRECT) ? s.run_start : nullptr;
    a.warm_x = nullptr; a.warm_stride = 0; a.warm_rows = 0; a.warm_units = c.hidden / 8; a.nchunks = 1;
    a.rows_cap = -1; a.recv_count = nullptr;
    a.drop_hint = (a.padded && a.run_start) ? g->drop_hint_dev : nullptr;
    a.quant_out = nullptr; a.quant_pitch = 0;
    h->quant_x = nullptr;
    if (tokens && a.run_start && c.dispatch_order == EP_ORDER_DESTINATION) {
        a.warm_x = (const uint16_t*)tokens->data;
        a.warm_stride = tokens->stride[0];
        const int cached_rows = (int)std::min<int64_t>(T, kWarmBytes / (2 * (int64_t)c.hidden));
        a.warm_rows = c.quantize_ahead ? (int)T : cached_rows;  // a staging copy needs every row
        if (layout_prefetches(a)) {
            h->warm_x = tokens->data; h->warm_stride = a.warm_stride; h->warm_rows = cached_rows;
            if (c.quantize_ahead) {
                a.quant_out = s.quant; a.quant_pitch = quant_row_pitch(c.hidden);
                h->quant_x = tokens->data; h->quant_stride = a.warm_stride;
            }
        } else {
            a.warm_x = nullptr;
        }
    }
    h->has_runs = layout_writes_runs(a);
    h->nwc = a.nwc;
    h->chunk_entries = a.passes * kWave;
    *args = a;
    *handle = h;
    return EP_SUCCESS;
}

ep_result_t ep_layout_prefetch(ep_handle_t* handle, ep_group_t g, const ep_tensor_t* topk_idx,
                               const ep_tensor_t* expert_base, const ep_tensor_t* tokens, ep_stream_t stream) {
    LayoutArgs a;
    ep_handle_t h = nullptr;
    if (ep_result_t r = prepare_layout(&h, g, topk_idx, expert_base, tokens, stream, &a); r != EP_SUCCESS) return r;
    if (launch_layout(a, (hipStream_t)stream) != hipSuccess) {
        ep_handle_destroy(h);
        return EP_ERR_HIP;
    }
    *handle = h;
    return EP_SUCCESS;
}

ep_result_t ep_handle_query(ep_handle_t h, ep_layout_info_t* info) {
    if (!h || !info) return EP_ERR_INVALID_ARG;
    int32_t tot[kTotalsWords];
    ep_result_t r = sync_and_read_totals(h, tot);
    if (r != EP_SUCCESS) return r;
    const Slab& s = h->slab;
    info->num_tokens = h->T;
    info->status = tot[TOT_STATUS];
    info->rows_kept = tot[TOT_KEPT]; info->rows_dropped = tot[TOT_DROPPED];
    info->entries_masked = tot[TOT_MASKED]; info->entries_invalid = tot[TOT_INVALID];
    info->entries_sorted = tot[TOT_SORTED]; info->rank_messages = tot[TOT_MSGS];
    info->rows_end = tot[TOT_ROWS_END];
    info->expert_count = s.expert_count; info->expert_kept = s.expert_kept;
    info->expert_offset = s.expert_offset; info->rank_pair_count = s.rank_pair_count;
    info->rank_token_count = s.rank_token_count; info->rank_offset = s.rank_offset;
    info->slot = s.slot; info->dst_row = s.dst_row; info->rank_row = s.rank_row; info->entry_rank = s.entry_rank;
    info->sorted_token = s.sorted_token; info->sorted_k = s.sorted_k; info->sorted_row = s.sorted_row;
    if (tot[TOT_STATUS] & STATUS_INVALID_IDS) return EP_ERR_INVALID_ROUTING;
    if (tot[TOT_STATUS] & STATUS_OUTPUT_OVERFLOW) return EP_ERR_OVERFLOW;
    if (tot[TOT_STATUS] & STATUS_TIMEOUT) return EP_ERR_TIMEOUT;
    return EP_SUCCESS;
}

ep_result_t ep_handle_get_num_recv_tokens(ep_handle_t h, int64_t* num) {
    if (!h || !num) return EP_ERR_INVALID_ARG;
    int32_t tot[kTotalsWords];
    ep_result_t r = sync_and_read_totals(h, tot);
    if (r != EP_SUCCESS) return r;
    *num = tot[TOT_KEPT];
    return EP_SUCCESS;
}

ep_result_t ep_handle_destroy(ep_handle_t h) {
    if (!h) return EP_ERR_INVALID_ARG;
    ep_group_s* g = h->group;
    ep_result_t r = EP_SUCCESS;
    if (h->pending != PENDING_NONE) {
        // an abandoned staged call: its coordination counters are raised and would be taken for
        // those of the next call that uses the buffer set; clear them behind the send phase
        const ep_group_config_t& c = g->cfg;
        int32_t* sig = h->pending == PENDING_DISPATCH_DIRECT ? g->sig_dispatch(h->pending_set)
                       : h->pending == PENDING_DISPATCH_DEDUP ? g->sig_rank(h->pending_set) : g->sig_combine(h->pending_set);
        const int n = h->pending == PENDING_DISPATCH_DEDUP ? c.num_ranks : c.num_experts;
        if (launch_clear_counts(sig, n, h->last_stream) != hipSuccess) r = EP_ERR_HIP;
    }
    h->slab.last_stream = h->last_stream;
    h->slab.used = true;
    {
        std::lock_guard<std::mutex> lk(g->mu);
        g->free_slabs.push_back(h->slab);
        g->live_handles -= 1;
    }
    delete h;
    return r;
}

// The tensors of a dispatch call, checked against the group and turned into kernel arguments
// (everything but what depends on the handle's bookkeeping).
struct DispatchCall {
    DispatchArgs a;
    bool fp8;
    float* scales;
    const ep_tensor_t* x;
};

static ep_result_t parse_dispatch(ep_group_s* g, int T, const Slab& slab, const ep_tensor_t* inputs, int32_t num_inputs,
                                  const ep_tensor_t* outputs, int32_t num_outputs, DispatchCall* call) {
    if (!inputs || !outputs || num_inputs < 1 || num_outputs < 1) return EP_ERR_INVALID_ARG;
    if (has_scales(inputs, num_inputs)) return EP_ERR_UNSUPPORTED;  // inputs are bf16 tokens
    const ep_group_config_t& c = g->cfg;
    const ep_tensor_t* x = find_tag(inputs, num_inputs, EP_TAG_TOKENS);
    const ep_tensor_t* w = find_tag(inputs, num_inputs, EP_TAG_TOPK_WEIGHTS);
    const ep_tensor_t* rx = find_tag(outputs, num_outputs, EP_TAG_TOKENS);
    const ep_tensor_t* rw = find_tag(outputs, num_outputs, EP_TAG_TOPK_WEIGHTS);
    const ep_tensor_t* rs = find_tag(outputs, num_outputs, EP_TAG_RECV_SRC_TOKEN);
    const ep_tensor_t* rq = find_tag(outputs, num_outputs, EP_TAG_SCALES);
    const ep_tensor_t* rc = find_tag(outputs, num_outputs, EP_TAG_RECV_EXPERT_COUNTER_DEVICE,
                                     EP_TAG_RECV_EXPERT_COUNTER_HOST, EP_TAG_TOKENS_PER_EXPERTS);
    if (!check_2d(x, EP_DTYPE_BF16, T, c.hidden, true) || x->stride[0] % 8 || !aligned16(x->data))
        return EP_ERR_INVALID_ARG;
    if (w && !check_2d(w, EP_DTYPE_F32, T, c.top_k, true)) return EP_ERR_INVALID_ARG;
    // An FP8 output selects the quantising dispatch (Sec. III-E: the tags tell the library
    // which tensors to expect -- FP8 tokens come with a SCALES tensor).
    const bool fp8 = rx && rx->dtype == EP_DTYPE_FP8_E4M3;
    if (fp8 != (rq != nullptr)) return EP_ERR_INVALID_ARG;
    DispatchArgs& a = call->a;
    if (!window_from_tensor(g, rx, &a.win, fp8 ? EP_DTYPE_FP8_E4M3 : EP_DTYPE_BF16)) return EP_ERR_INVALID_ARG;
    if (fp8) {
        if (c.hidden % 128 != 0) return EP_ERR_INVALID_ARG;
        if (c.dispatch_path != EP_PATH_DIRECT) return EP_ERR_UNSUPPORTED;
        if (!check_2d(rq, EP_DTYPE_F32, a.win.rows_cap, c.hidden / 128, false) || rq->stride[0] != c.hidden / 128)
            return EP_ERR_INVALID_ARG;
    }
    if (rw && !check_1d(rw, EP_DTYPE_F32, a.win.rows_cap)) return EP_ERR_INVALID_ARG;
    if (rs && !check_1d(rs, EP_DTYPE_I32, a.win.rows_cap)) return EP_ERR_INVALID_ARG;
    if (rc && !check_1d(rc, EP_DTYPE_I32, c.num_experts)) return EP_ERR_INVALID_ARG;
    a.x = (const uint16_t*)x->data;
    a.x_stride = x->stride[0];
    a.w = w ? (const float*)w->data : nullptr;
    a.w_stride = w ? w->stride[0] : 0;
    a.dst_row = slab.dst_row;
    a.recv_w = rw ? (float*)rw->data : nullptr;
    a.recv_src = rs ? (int32_t*)rs->data : nullptr;
    a.recv_count = rc ? (int32_t*)rc->data : nullptr;
    a.expert_kept = slab.expert_kept;
    a.totals = slab.totals;
    a.T = T; a.K = c.top_k; a.H = c.hidden; a.E = c.num_experts;
    a.sorted_token = slab.sorted_token; a.sorted_k = slab.sorted_k; a.sorted_row = slab.sorted_row;
    a.own_prefix = slab.own_prefix;
    a.run_start = nullptr; a.nwc = 0; a.chunk_entries = 0; a.order = c.dispatch_order; a.prefetched_rows = 0;
    call->fp8 = fp8;
    call->scales = rq ? (float*)rq->data : nullptr;
    call->x = x;
    return EP_SUCCESS;
}

ep_result_t ep_dispatch(ep_handle_t h, const ep_tensor_t* inputs, int32_t num_inputs,
                        const ep_tensor_t* outputs, int32_t num_outputs, int32_t send_only,
                        ep_stream_t stream) {
    if (!h) return EP_ERR_INVALID_ARG;
    if (send_only != 0 && send_only != 1) return EP_ERR_INVALID_ARG;
    ep_group_s* g = h->group;
    if (send_only && g->nsets == 0) return EP_ERR_UNSUPPORTED;
    if (send_only && h->pending != PENDING_NONE) return EP_ERR_BUSY;
    const ep_group_config_t& c = g->cfg;
    DispatchCall call;
    if (ep_result_t r = parse_dispatch(g, h->T, h->slab, inputs, num_inputs, outputs, num_outputs, &call); r != EP_SUCCESS)
        return r;
    DispatchArgs& a = call.a;
    const bool fp8 = call.fp8;
    const ep_tensor_t* x = call.x;
    a.run_start = h->has_runs ? h->slab.run_start : nullptr;
    if (a.run_start && a.win.padded && g->drop_hint) {  // capacity cut most entries last time: walk the tokens
        const int64_t v = __atomic_load_n(g->drop_hint, __ATOMIC_RELAXED);
        const int64_t kept = v & 0xffffffffLL, dropped = v >> 32;
        if (2 * dropped > kept) a.run_start = nullptr;
    }
    a.nwc = h->nwc; a.chunk_entries = h->chunk_entries;
    // the read-ahead of the layout call is good for the dispatch that follows it, once
    a.prefetched_rows = (h->warm_x == x->data && h->warm_stride == x->stride[0]) ? h->warm_rows : 0;
    h->warm_x = nullptr;
    h->warm_rows = 0;
    h->last_stream = (hipStream_t)stream;
    int set = 0;
    if (send_only) {
        std::lock_guard<std::mutex> lk(g->mu);
        set = g->next_set;
        g->next_set = (set + 1) % g->nsets;
    }
    if (fp8 || c.dispatch_path == EP_PATH_DIRECT) {
        // staged: rows go straight to the output windows (they are the receive region), the
        // per-expert counts are delivered by ep_complete from the coordination counters
        int32_t* recv_count = a.recv_count;
        if (send_only) a.recv_count = nullptr;
        // rows the layout call quantised ahead are copied in destination order, by the handle's first dispatch only
        const bool staged = fp8 && h->quant_x == x->data && h->quant_stride == x->stride[0] && dispatch_fp8_staged_possible(a);
        h->quant_x = nullptr;  // whatever this dispatch is, a later one may be given other data at the same address
        hipError_t e = staged ? launch_dispatch_fp8_staged(a, call.scales, h->slab.quant, quant_row_pitch(c.hidden), (hipStream_t)stream)
                       : fp8  ? launch_dispatch_fp8(a, call.scales, (hipStream_t)stream)
                              : launch_dispatch(a, (hipStream_t)stream);
        if (e != hipSuccess) return EP_ERR_HIP;
        if (send_only) {
            if (launch_publish_counts(g->sig_dispatch(set), h->slab.expert_kept, c.num_experts, (hipStream_t)stream) != hipSuccess)
                return EP_ERR_HIP;
            h->pending = PENDING_DISPATCH_DIRECT;
            h->pending_set = set;
            h->pending_recv_count = recv_count;
        }
        return EP_SUCCESS;
    }

    // Once per destination rank: send to the staging windows, rank the header entries on
    // the receiving side, fan out to the expert rows.
    const ep_tensor_t* ti = find_tag(inputs, num_inputs, EP_TAG_TOPK_IDX);
    if (!check_2d(ti, EP_DTYPE_I32, h->T, c.top_k, true)) return EP_ERR_INVALID_ARG;
    const Slab& s = h->slab;
    DedupSendArgs sa;
    sa.x = a.x; sa.x_stride = a.x_stride;
    sa.topk = (const int32_t*)ti->data; sa.topk_stride = ti->stride[0];
    sa.w = a.w; sa.w_stride = a.w_stride;
    sa.rank_row = s.rank_row;
    sa.staging = g->staging[set]; sa.msg_stride = g->msg_stride; sa.msg_lead = g->msg_lead;
    sa.staging_slots = g->staging_slots;
    sa.hdr_units = (int)(g->hdr_bytes / 16);
    sa.totals = s.totals;
    sa.T = h->T; sa.K = c.top_k; sa.H = c.hidden;
    if (launch_dedup_send(sa, (hipStream_t)stream) != hipSuccess) return EP_ERR_HIP;

    DedupRankArgs ra;
    ra.staging = g->staging[set]; ra.msg_stride = g->msg_stride; ra.msg_lead = g->msg_lead;
    ra.staging_slots = g->staging_slots;
    ra.slots_per_rank = c.mode == EP_MODE_LL ? c.max_tokens_per_rank : 0;
    // a staged call lets the receiving side learn the message counts from the counters
    ra.rank_offset = send_only ? s.recv_rank_offset : s.rank_offset;
    ra.rank_count = send_only ? s.recv_rank_count : s.rank_token_count;
    ra.expert_offset = s.expert_offset;
    ra.recv_dst_row = s.recv_dst_row; ra.recv_count = s.recv_count; ra.recv_kept = s.recv_kept;
    ra.K = c.top_k; ra.E = c.num_experts; ra.R = c.num_ranks; ra.L = g->L; ra.L_shift = g->L_shift;
    ra.K_shift = g->K_shift; ra.bits_l = bits_for(g->L);
    ra.padded = c.mode == EP_MODE_LL; ra.C = g->C;

    DedupFanoutArgs fa;
    fa.staging = g->staging[set]; fa.msg_stride = g->msg_stride; fa.msg_lead = g->msg_lead;
    fa.hdr_bytes = g->hdr_bytes;
    fa.staging_slots = g->staging_slots; fa.slots_per_rank = ra.slots_per_rank;
    fa.rank_offset = ra.rank_offset; fa.rank_count = ra.rank_count;
    fa.recv_dst_row = s.recv_dst_row; fa.recv_kept = s.recv_kept;
    fa.win = a.win; fa.recv_w = a.recv_w; fa.recv_src = a.recv_src; fa.recv_count = a.recv_count;
    fa.totals = s.totals;
    fa.K = c.top_k; fa.H = c.hidden; fa.E = c.num_experts; fa.R = c.num_ranks;
    if (send_only) {
        if (launch_publish_counts(g->sig_rank(set), s.rank_token_count, c.num_ranks, (hipStream_t)stream) != hipSuccess)
            return EP_ERR_HIP;
        h->pending = PENDING_DISPATCH_DEDUP;
        h->pending_set = set;
        h->pending_rank = ra;
        h->pending_fanout = fa;
        return EP_SUCCESS;
    }
    if (launch_dedup_rank(ra, (hipStream_t)stream) != hipSuccess) return EP_ERR_HIP;
    return launch_dedup_fanout(fa, (hipStream_t)stream) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

ep_result_t ep_layout_dispatch(ep_handle_t* handle, ep_group_t g, const ep_tensor_t* topk_idx,
                               const ep_tensor_t* expert_base, const ep_tensor_t* inputs, int32_t num_inputs,
                               const ep_tensor_t* outputs, int32_t num_outputs, ep_stream_t stream) {
    if (!handle || !g || !inputs || num_inputs < 1) return EP_ERR_INVALID_ARG;
    LayoutArgs la;
    ep_handle_t h = nullptr;
    // the tokens are announced to the layout, as ep_layout_prefetch would
    const ep_tensor_t* x = find_tag(inputs, num_inputs, EP_TAG_TOKENS);
    if (ep_result_t r = prepare_layout(&h, g, topk_idx, expert_base, x, stream, &la); r != EP_SUCCESS) return r;
    DispatchCall call;
    ep_result_t r = parse_dispatch(g, h->T, h->slab, inputs, num_inputs, outputs, num_outputs, &call);
    if (r == EP_SUCCESS) {
        if (!call.fp8 && g->cfg.dispatch_path == EP_PATH_DIRECT && layout_dispatch_fusable(la, call.a)) {
            h->warm_x = nullptr;
            h->warm_rows = 0;
            if (launch_layout_dispatch(la, call.a, (hipStream_t)stream) != hipSuccess) r = EP_ERR_HIP;
        } else {
            if (launch_layout(la, (hipStream_t)stream) != hipSuccess) r = EP_ERR_HIP;
            else r = ep_dispatch(h, inputs, num_inputs, outputs, num_outputs, 0, stream);
        }
    }
    if (r != EP_SUCCESS) {
        ep_handle_destroy(h);
        return r;
    }
    *handle = h;
    return EP_SUCCESS;
}

ep_result_t ep_complete(ep_handle_t h, const ep_complete_config_t* cfg, ep_stream_t stream) {
    if (!h) return EP_ERR_INVALID_ARG;
    if (cfg && cfg->size != sizeof(ep_complete_config_t)) return EP_ERR_INVALID_ARG;
    if (h->pending == PENDING_NONE) return EP_ERR_INVALID_ARG;
    ep_group_s* g = h->group;
    const ep_group_config_t& c = g->cfg;
    int spin = cfg && cfg->spin_limit > 0 ? cfg->spin_limit : (1 << 20);
    const int set = h->pending_set;
    const int kind = h->pending;
    hipStream_t st = (hipStream_t)stream;
    h->pending = PENDING_NONE;
    h->last_stream = st;
    const Slab& s = h->slab;
    if (kind == PENDING_DISPATCH_DIRECT) {
        return launch_await_counts(g->sig_dispatch(set), c.num_experts, spin, h->pending_recv_count, nullptr,
                                   s.totals, st) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
    }
    if (kind == PENDING_DISPATCH_DEDUP) {
        if (launch_await_counts(g->sig_rank(set), c.num_ranks, spin, s.recv_rank_count, s.recv_rank_offset,
                                s.totals, st) != hipSuccess) return EP_ERR_HIP;
        if (launch_dedup_rank(h->pending_rank, st) != hipSuccess) return EP_ERR_HIP;
        return launch_dedup_fanout(h->pending_fanout, st) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
    }
    if (launch_await_counts(g->sig_combine(set), c.num_experts, spin, nullptr, nullptr, s.totals, st) != hipSuccess)
        return EP_ERR_HIP;
    return launch_combine(h->pending_combine, st) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

ep_result_t ep_group_reset_signals(ep_group_t g, ep_stream_t stream) {
    if (!g) return EP_ERR_INVALID_ARG;
    for (int i = 0; i < g->nsets; ++i)
        if (launch_clear_counts(g->signals[i], g->sig_ints(), (hipStream_t)stream) != hipSuccess) return EP_ERR_HIP;
    return EP_SUCCESS;
}

ep_result_t ep_combine(ep_handle_t h, const ep_tensor_t* inputs, int32_t num_inputs,
                       const ep_tensor_t* outputs, int32_t num_outputs, int32_t send_only,
                       ep_stream_t stream) {
    if (!h || !inputs || !outputs || num_inputs < 1 || num_outputs < 1) return EP_ERR_INVALID_ARG;
    if (send_only != 0 && send_only != 1) return EP_ERR_INVALID_ARG;
    if (has_scales(inputs, num_inputs) || has_scales(outputs, num_outputs)) return EP_ERR_UNSUPPORTED;
    ep_group_s* g = h->group;
    if (send_only && g->nsets == 0) return EP_ERR_UNSUPPORTED;
    if (send_only && h->pending != PENDING_NONE) return EP_ERR_BUSY;
    const ep_group_config_t& c = g->cfg;
    const ep_tensor_t* y = find_tag(inputs, num_inputs, EP_TAG_TOKENS);
    const ep_tensor_t* w = find_tag(inputs, num_inputs, EP_TAG_TOPK_WEIGHTS);
    const ep_tensor_t* out = find_tag(outputs, num_outputs, EP_TAG_TOKENS);
    CombineArgs a;
    if (!window_from_tensor(g, y, &a.win)) return EP_ERR_INVALID_ARG;
    if (w && !check_2d(w, EP_DTYPE_F32, h->T, c.top_k, true)) return EP_ERR_INVALID_ARG;
    if (!check_2d(out, EP_DTYPE_BF16, h->T, c.hidden, true) || out->stride[0] % 8 || !aligned16(out->data))
        return EP_ERR_INVALID_ARG;
    a.w = w ? (const float*)w->data : nullptr;
    a.w_stride = w ? w->stride[0] : 0;
    a.dst_row = h->slab.dst_row;
    a.out = (uint16_t*)out->data;
    a.out_stride = out->stride[0];
    a.T = h->T; a.K = c.top_k; a.H = c.hidden;
    a.staged = 0;
    // two-level order only when it differs from the flat one (more than one node)
    a.ranks_per_node = (c.ranks_per_node > 0 && c.ranks_per_node < c.num_ranks) ? c.ranks_per_node : 0;
    a.nodes = a.ranks_per_node ? (c.num_ranks + a.ranks_per_node - 1) / a.ranks_per_node : 1;
    a.entry_rank = h->slab.entry_rank;
    h->last_stream = (hipStream_t)stream;
    if (!send_only) return launch_combine(a, (hipStream_t)stream) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
    // staged: the expert side packs its rows into the (t,k)-indexed staging and raises the
    // counters; ep_complete reduces from the staging
    int set;
    {
        std::lock_guard<std::mutex> lk(g->mu);
        set = g->next_set;
        g->next_set = (set + 1) % g->nsets;
    }
    if (launch_combine_pack(a, g->comb_stage[set], (hipStream_t)stream) != hipSuccess) return EP_ERR_HIP;
    if (launch_publish_counts(g->sig_combine(set), nullptr, c.num_experts, (hipStream_t)stream) != hipSuccess)
        return EP_ERR_HIP;
    h->pending = PENDING_COMBINE;
    h->pending_set = set;
    h->pending_combine = a;
    h->pending_combine.win.base = g->comb_stage[set];
    h->pending_combine.staged = 1;
    return EP_SUCCESS;
}

ep_result_t ep_layout_static(const ep_group_config_t* cfg, const ep_tensor_t* topk_idx, const ep_tensor_t* expert_base,
                             const ep_layout_arrays_t* out, ep_stream_t stream) {
    if (!topk_idx || !out || out->size != sizeof(ep_layout_arrays_t)) return EP_ERR_INVALID_ARG;
    if (ep_result_t v = validate_config(cfg); v != EP_SUCCESS) return v;
    const ep_group_config_t& c = *cfg;
    if (topk_idx->tag != EP_TAG_TOPK_IDX || topk_idx->ndim != 2 || topk_idx->dtype != EP_DTYPE_I32)
        return EP_ERR_INVALID_ARG;
    const int64_t T = topk_idx->shape[0];
    if (T < 0 || T > c.max_tokens_per_rank) return EP_ERR_INVALID_ARG;
    if (!check_2d(topk_idx, EP_DTYPE_I32, T, c.top_k, true)) return EP_ERR_INVALID_ARG;
    if (expert_base) {
        if (c.mode != EP_MODE_HT) return EP_ERR_INVALID_ARG;
        if (expert_base->tag != EP_TAG_EXPERT_BASE || !check_1d(expert_base, EP_DTYPE_I32, c.num_experts) ||
            !expert_base->data)
            return EP_ERR_INVALID_ARG;
    }
    if (!out->totals || !out->expert_count || !out->expert_kept || !out->expert_offset || !out->rank_pair_count ||
        !out->rank_token_count || !out->rank_offset)
        return EP_ERR_INVALID_ARG;
    if (T > 0 && !out->dst_row) return EP_ERR_INVALID_ARG;
    // the expert-sorted list is three arrays: all of them or none
    const int nsorted = (out->sorted_token != nullptr) + (out->sorted_k != nullptr) + (out->sorted_row != nullptr);
    if (nsorted != 0 && nsorted != 3) return EP_ERR_INVALID_ARG;
    LayoutArgs a;
    a.E = c.num_experts; a.R = c.num_ranks; a.K = c.top_k; a.T = (int)T;
    a.W = a.E + 2 + a.R;
    // the limit of the scratch array: at most kMaxChunks rows of W bin sums
    if ((int64_t)kMaxChunks * a.W > kStaticPubInts) return EP_ERR_INVALID_ARG;
    int32_t* sc = nullptr;
    if (ep_result_t r = static_scratch(&sc); r != EP_SUCCESS) return r;
    a.topk = (const int32_t*)topk_idx->data;
    a.topk_stride = topk_idx->stride[0];
    a.expert_base = expert_base ? (const int32_t*)expert_base->data : nullptr;
    a.L = a.E / a.R; a.L_shift = log2_exact(a.L); a.K_shift = log2_exact(a.K);
    a.padded = c.mode == EP_MODE_LL;
    a.C = c.slots_per_subregion ? c.slots_per_subregion : c.max_tokens_per_rank;
    a.C_rank = c.max_tokens_per_rank;
    a.n = (int)(T * c.top_k);
    plan_layout(a.n, &a.passes, &a.nwc);
    a.bits_e = bits_for(a.E); a.bits_r = bits_for(a.R);
    // the array is zero when the library is loaded, and every launch leaves the words through
    // which its workgroups talk to each other ready for the next one
    a.pub = (uint32_t*)sc;
    a.ctl = (uint32_t*)(sc + kStaticPubInts);
    a.own_prefix = sc + kStaticPubInts + kSlabAlign;
    a.expert_count = out->expert_count; a.expert_kept = out->expert_kept; a.expert_offset = out->expert_offset;
    a.rank_pair_count = out->rank_pair_count; a.rank_token_count = out->rank_token_count;
    a.rank_offset = out->rank_offset; a.totals = out->totals;
    a.slot = out->slot; a.dst_row = out->dst_row; a.rank_row = out->rank_row; a.entry_rank = out->entry_rank;
    a.sorted_token = out->sorted_token; a.sorted_k = out->sorted_k; a.sorted_row = out->sorted_row;
    a.run_start = nullptr; a.drop_hint = nullptr; a.quant_out = nullptr; a.quant_pitch = 0;
    a.warm_x = nullptr; a.warm_stride = 0; a.warm_rows = 0; a.warm_units = c.hidden / 8; a.nchunks = 1;
    a.rows_cap = -1; a.recv_count = nullptr;
    return launch_layout(a, (hipStream_t)stream) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

ep_result_t ep_combine_backward(ep_handle_t h, const ep_tensor_t* inputs, int32_t num_inputs,
                                const ep_tensor_t* outputs, int32_t num_outputs, ep_stream_t stream) {
    if (!h || !inputs || !outputs || num_inputs < 1 || num_outputs < 1) return EP_ERR_INVALID_ARG;
    if (has_scales(inputs, num_inputs) || has_scales(outputs, num_outputs)) return EP_ERR_UNSUPPORTED;
    ep_group_s* g = h->group;
    const ep_group_config_t& c = g->cfg;
    const ep_tensor_t* go = find_tag(inputs, num_inputs, EP_TAG_TOKENS);
    const ep_tensor_t* w = find_tag(inputs, num_inputs, EP_TAG_TOPK_WEIGHTS);
    const ep_tensor_t* y = find_tag(inputs, num_inputs, EP_TAG_EXPERT_TOKENS);
    const ep_tensor_t* gy = find_tag(outputs, num_outputs, EP_TAG_TOKENS);
    const ep_tensor_t* gw = find_tag(outputs, num_outputs, EP_TAG_TOPK_WEIGHTS);
    if (!check_2d(go, EP_DTYPE_BF16, h->T, c.hidden, true) || go->stride[0] % 8 || !aligned16(go->data))
        return EP_ERR_INVALID_ARG;
    if (w && !check_2d(w, EP_DTYPE_F32, h->T, c.top_k, true)) return EP_ERR_INVALID_ARG;
    if ((y != nullptr) != (gw != nullptr)) return EP_ERR_INVALID_ARG;  // the weight gradient needs the expert outputs
    if (gw && !check_2d(gw, EP_DTYPE_F32, h->T, c.top_k, true)) return EP_ERR_INVALID_ARG;
    CombineArgs a;
    WindowDesc gyw;
    if (!window_from_tensor(g, gy, &gyw)) return EP_ERR_INVALID_ARG;
    if (y) {
        if (!window_from_tensor(g, y, &a.win)) return EP_ERR_INVALID_ARG;
        if (a.win.rows_cap != gyw.rows_cap) return EP_ERR_INVALID_ARG;
    } else {
        a.win = gyw;
        a.win.base = nullptr;
    }
    a.w = w ? (const float*)w->data : nullptr;
    a.w_stride = w ? w->stride[0] : 0;
    a.dst_row = h->slab.dst_row;
    a.out = nullptr; a.out_stride = 0;
    a.T = h->T; a.K = c.top_k; a.H = c.hidden;
    a.staged = 0; a.entry_rank = nullptr; a.ranks_per_node = 0; a.nodes = 1;
    h->last_stream = (hipStream_t)stream;
    return launch_combine_backward(a, (const uint16_t*)go->data, go->stride[0], gyw, gw ? (float*)gw->data : nullptr,
                                   gw ? gw->stride[0] : 0, (hipStream_t)stream) == hipSuccess ? EP_SUCCESS : EP_ERR_HIP;
}

}  // extern "C"
