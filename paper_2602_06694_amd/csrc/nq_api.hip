// C ABI of libnq_binlr: host-side packing, layer handles, plans.  See include/nq_binlr.h.
#include <algorithm>
#include <cctype>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "nq_internal.h"

namespace nq {

static thread_local std::string g_last_error;

void set_error(const std::string& msg) { g_last_error = msg; }

int hip_fail(hipError_t e, const char* what, const char* file, int line)
{
    char buf[512];
    snprintf(buf, sizeof buf, "HIP error %d (%s) in %s at %s:%d", (int)e, hipGetErrorString(e), what, file, line);
    set_error(buf);
    return NQ_E_HIP;
}

static int fail(int code, const char* msg)
{
    set_error(msg);
    return code;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// ---- tuning options: one table, filled once from the environment, then only through nq_set_option ----
struct OptEntry { const char* name; bool flag; };
static const OptEntry kOptTable[OPT_COUNT] = {
    {"slab_mb", false}, {"force_w", false}, {"split_steps", false}, {"selfq4_min_steps", false}, {"share_steps", false},
    {"share_min_batch", false}, {"stream_steps", false}, {"schedule_full", false}, {"fuse_max_mb", false},
    {"no_fuse", true}, {"no_selfq", true}, {"no_selfq_c2", true}, {"no_resident", true}, {"no_quant_wave", true},
    {"pf_splits1", false}, {"pf_splits2", false}, {"pf_tg1", false}, {"pf_tg2", false}, {"pf_ks1", false}, {"pf_ks2", false},
    {"pf_verbose", true}, {"exec_spin_limit_us", false}, {"no_small_layer", true}, {"small_layer_kb", false},
    {"dgemm_tile", false}, {"admm_no_overlap", true}, {"two_slice_b8", true},
    {"admm_no_prio", true}, {"admm_product_mode", false}, {"admm_inline_svid", true}, {"admm_no_fused_step", true},
};
static int g_opt[OPT_COUNT];
static std::once_flag g_opt_once;

static void options_from_environment()
{
    for (int i = 0; i < OPT_COUNT; ++i) {
        g_opt[i] = -1;
        std::string env = "NQ_";
        for (const char* c = kOptTable[i].name; *c; ++c) env += (char)toupper((unsigned char)*c);
        const char* v = getenv(env.c_str());
        if (!v || !*v) continue;
        const int x = atoi(v);
        if (kOptTable[i].flag) g_opt[i] = (v[0] == '0' && v[1] == 0) ? 0 : 1;
        else if (x >= 0) g_opt[i] = x;
    }
}

int opt(Opt o)
{
    std::call_once(g_opt_once, options_from_environment);
    return g_opt[o];
}

thread_local LaunchTiming g_launch_timing;

static size_t dtype_size(int dt) { return dt == NQ_F32 ? 4 : 2; }

}  // namespace nq

using namespace nq;

// ---------------------------------------------------------------------------------------------
// Device memory for layers comes from large slabs, not from one hipMalloc per layer: a model is
// hundreds of layers of ~1 MB each, and the streaming kernels run measurably faster when those
// sit back to back in a few big, contiguously mapped allocations (fewer address-translation
// misses) than in hundreds of small ones.  A slab is released when its last layer is destroyed.
// ---------------------------------------------------------------------------------------------
struct Slab {
    char* base;
    size_t size, used;
    int live;          // allocations handed out and not yet released
    int device;
    int kind;          // 0: sign tiles and scales (streamed), 1: per-layer workspaces (small, reused)
    std::vector<std::pair<size_t, size_t>> free_ranges;    // (offset, bytes) of released blocks, sorted by offset, neighbours merged
};
static std::mutex g_slab_mutex;
static std::vector<Slab*> g_slabs;

static size_t slab_bytes()
{
    return (size_t)std::max(1, opt_or(OPT_SLAB_MB, 512)) << 20;
}

// returns hipSuccess and (*out, *owner); the block is 4 KiB aligned.  Released blocks are reused (first
// fit) before a slab grows, so a process that keeps rebuilding layers beside a long-lived one does not
// take a new slab every time.
static hipError_t slab_alloc(size_t bytes, int device, int kind, void** out, Slab** owner)
{
    std::lock_guard<std::mutex> lk(g_slab_mutex);
    bytes = (bytes + 4095) / 4096 * 4096;
    const size_t std_size = kind == 0 ? slab_bytes() : slab_bytes() / 4;
    Slab* s = nullptr;
    if (bytes <= std_size / 4) {
        for (Slab* c : g_slabs) {
            if (c->device != device || c->kind != kind || c->size != std_size) continue;
            for (size_t i = 0; i < c->free_ranges.size(); ++i) {
                if (c->free_ranges[i].second < bytes) continue;
                *out = c->base + c->free_ranges[i].first;
                c->free_ranges[i].first += bytes;
                c->free_ranges[i].second -= bytes;
                if (c->free_ranges[i].second == 0) c->free_ranges.erase(c->free_ranges.begin() + i);
                c->live += 1;
                *owner = c;
                return hipSuccess;
            }
        }
        for (Slab* c : g_slabs)
            if (c->device == device && c->kind == kind && c->size == std_size && c->size - c->used >= bytes) { s = c; break; }
    }
    if (!s) {
        const size_t sz = bytes <= std_size / 4 ? std_size : bytes;     // big requests get a slab of their own
        void* p = nullptr;
        hipError_t e = hipMalloc(&p, sz);
        if (e != hipSuccess) return e;
        s = new Slab{(char*)p, sz, 0, 0, device, kind, {}};
        g_slabs.push_back(s);
    }
    *out = s->base + s->used;
    s->used += bytes;
    s->live += 1;
    *owner = s;
    return hipSuccess;
}

// gives the block [p, p + bytes) back to its slab; the slab itself is freed when its last block goes
static void slab_release(Slab* s, void* p, size_t bytes)
{
    if (!s) return;
    std::lock_guard<std::mutex> lk(g_slab_mutex);
    if (--s->live > 0) {
        bytes = (bytes + 4095) / 4096 * 4096;
        const size_t off = (size_t)((char*)p - s->base);
        auto it = s->free_ranges.begin();
        while (it != s->free_ranges.end() && it->first < off) ++it;
        it = s->free_ranges.insert(it, std::make_pair(off, bytes));
        if (it + 1 != s->free_ranges.end() && it->first + it->second == (it + 1)->first) {      // merge with the next
            it->second += (it + 1)->second;
            s->free_ranges.erase(it + 1);
        }
        if (it != s->free_ranges.begin() && (it - 1)->first + (it - 1)->second == it->first) {  // and with the previous
            (it - 1)->second += it->second;
            it = s->free_ranges.erase(it) - 1;
        }
        if (it->first + it->second == s->used) {                  // the tail of the slab: plain unused space again
            s->used = it->first;
            s->free_ranges.erase(it);
        }
        return;
    }
    (void)hipFree(s->base);
    g_slabs.erase(std::find(g_slabs.begin(), g_slabs.end(), s));
    delete s;
}

extern "C" int nq_debug_slab_count(void)
{
    std::lock_guard<std::mutex> lk(g_slab_mutex);
    return (int)g_slabs.size();
}

// ---------------------------------------------------------------------------------------------
// Carves a DecodeWorkspace for `batch` tokens of a (d_in, r) layer out of `base` (256-byte aligned);
// returns the bytes it takes (base == nullptr: only the size).
static size_t carve_workspace(DecodeWorkspace* w, char* base, int64_t d_in, int64_t r, int batch)
{
    auto al = [](size_t v) { return (v + 255) / 256 * 256; };
    // (+1 KiB: the shared-input kernel stages whole chunks of 8 steps and may read up to 4 steps
    // past the last token's data; what it reads there meets 0 bits only and is never used)
    const size_t bqx_bytes = al((size_t)batch * n_steps(d_in) * 4 * kSlices * 16 + 1024);
    const size_t bqt_bytes = al((size_t)batch * n_steps(r) * 4 * kSlices * 16 + 1024);
    const size_t meta_bytes = al(sizeof(QMeta) * batch);
    const int t_stride = (int)round_up(r, kTileRows);
    const size_t t_bytes = al((size_t)batch * t_stride * 4);
    if (w) {
        char* q = base;
        w->bq_x = (uint8_t*)q; q += bqx_bytes;
        w->bq_t = (uint8_t*)q; q += bqt_bytes;
        w->meta_x = (QMeta*)q; q += meta_bytes;
        w->meta_t = (QMeta*)q; q += meta_bytes;
        w->t = (float*)q;
        w->t_stride = t_stride;
    }
    return bqx_bytes + bqt_bytes + 2 * meta_bytes + t_bytes;
}

struct nq_plan_s {
    int n, batch, device;
    void* alloc;
    QuantDesc* qx;
    StageDesc* s1;
    QuantDesc* qt;
    StageDesc* s2;
    WorkItem* items1;
    WorkItem* items2;
    FusedItem* fitems1;             // the same lists in the form of the fused schedule (empty otherwise)
    FusedItem* fitems2;
    int n_items1, n_items2;
    int w1, w2;                     // schedule of each stage launch (see stage_schedule; kFusedSchedule: no quantisation launch)
    int max_steps1, max_steps2;     // longest reduction of each stage launch
    int max_chunks_x, max_chunks_t; // longest vector of each quantisation launch (picks its block size)
    std::vector<nq_handle> handles;
    hipEvent_t ev[8];               // start / stop of the four launches of a timed run
    bool have_events;
};

// ---------------------------------------------------------------------------------------------
// packing (host)
// ---------------------------------------------------------------------------------------------
extern "C" size_t nq_packed_words(int64_t rows, int64_t cols)
{
    if (rows < 0 || cols < 0) return 0;
    return (size_t)rows * (size_t)((cols + 31) / 32);
}

static inline float half_to_float_host(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31, ex = (h >> 10) & 31u, man = h & 1023u;
    uint32_t bits;
    if (ex == 0) {
        if (man == 0) bits = sign;
        else {                                   // subnormal: value = man * 2^-24
            float f = (float)man * 5.9604644775390625e-8f;
            memcpy(&bits, &f, 4);
            bits |= sign;
        }
    } else if (ex == 31) bits = sign | 0x7F800000u | (man << 13);
    else bits = sign | ((ex + 112u) << 23) | (man << 13);
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

extern "C" int nq_pack_signs(const void* signs, int dtype, int64_t rows, int64_t cols, uint32_t* out_words)
{
    if (!signs || !out_words) return fail(NQ_E_NULL, "nq_pack_signs: NULL pointer");
    if (rows < 1 || cols < 1) return fail(NQ_E_SHAPE, "nq_pack_signs: rows and cols must be >= 1");
    if (dtype != NQ_I8 && dtype != NQ_F32 && dtype != NQ_F16 && dtype != NQ_BF16)
        return fail(NQ_E_INVALID_ARG, "nq_pack_signs: unknown dtype");
    const int64_t wpr = (cols + 31) / 32;
    for (int64_t i = 0; i < rows; ++i) {
        uint32_t* dst = out_words + i * wpr;
        for (int64_t w = 0; w < wpr; ++w) {
            uint32_t word = 0;
            const int64_t k0 = w * 32, k1 = std::min<int64_t>(cols, k0 + 32);
            for (int64_t k = k0; k < k1; ++k) {
                const int64_t idx = i * cols + k;
                bool plus;
                if (dtype == NQ_I8) {
                    int8_t v = ((const int8_t*)signs)[idx];
                    if (v != 1 && v != -1) return fail(NQ_E_INVALID_ARG, "nq_pack_signs: int8 sign is not +-1");
                    plus = v > 0;
                } else {
                    float v;
                    if (dtype == NQ_F32) v = ((const float*)signs)[idx];
                    else if (dtype == NQ_F16) v = half_to_float_host(((const uint16_t*)signs)[idx]);
                    else {
                        uint32_t b = (uint32_t)((const uint16_t*)signs)[idx] << 16;
                        memcpy(&v, &b, 4);
                    }
                    if (std::isnan(v)) return fail(NQ_E_INVALID_ARG, "nq_pack_signs: NaN has no sign");
                    plus = v >= 0.0f;
                }
                if (plus) word |= 1u << (k - k0);
            }
            dst[w] = word;
        }
    }
    return NQ_OK;
}

extern "C" int nq_unpack_signs(const uint32_t* words, int64_t rows, int64_t cols, int8_t* out_pm1)
{
    if (!words || !out_pm1) return fail(NQ_E_NULL, "nq_unpack_signs: NULL pointer");
    if (rows < 1 || cols < 1) return fail(NQ_E_SHAPE, "nq_unpack_signs: rows and cols must be >= 1");
    const int64_t wpr = (cols + 31) / 32;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t k = 0; k < cols; ++k)
            out_pm1[i * cols + k] = ((words[i * wpr + (k >> 5)] >> (k & 31)) & 1u) ? (int8_t)1 : (int8_t)-1;
    return NQ_OK;
}

extern "C" const char* nq_status_string(int status)
{
    switch (status) {
        case NQ_OK: return "ok";
        case NQ_E_INVALID_ARG: return "invalid argument";
        case NQ_E_SHAPE: return "bad shape";
        case NQ_E_ALIGN: return "pointer not 16-byte aligned";
        case NQ_E_NULL: return "null pointer";
        case NQ_E_UNSUPPORTED: return "unsupported";
        case NQ_E_HIP: return "HIP runtime error";
        case NQ_E_TIMEOUT: return "a bounded wait on the device ran into its limit";
        default: return "unknown status";
    }
}

extern "C" const char* nq_last_error_string(void) { return g_last_error.c_str(); }

static int find_option(const char* name)
{
    if (!name) return -1;
    for (int i = 0; i < OPT_COUNT; ++i)
        if (strcmp(name, kOptTable[i].name) == 0) return i;
    return -1;
}

extern "C" int nq_set_option(const char* name, int value)
{
    const int i = find_option(name);
    if (i < 0) return fail(NQ_E_INVALID_ARG, "nq_set_option: unknown option name");
    (void)opt((Opt)i);                                   // the environment is read before the first override, not after it
    g_opt[i] = value < 0 ? -1 : (kOptTable[i].flag ? (value != 0) : value);
    return NQ_OK;
}

extern "C" int nq_get_option(const char* name, int* value)
{
    const int i = find_option(name);
    if (i < 0 || !value) return fail(i < 0 ? NQ_E_INVALID_ARG : NQ_E_NULL, "nq_get_option: unknown option name or NULL pointer");
    *value = opt((Opt)i);
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// handles
// ---------------------------------------------------------------------------------------------
static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static void free_handle(nq_handle h)
{
    if (!h) return;
    slab_release(h->w_slab, h->w_alloc, h->w_bytes);
    slab_release(h->ws_slab, h->ws_alloc, h->ws_bytes);
    if (h->pf_alloc) (void)hipFree(h->pf_alloc);
    if (h->tp_alloc) (void)hipFree(h->tp_alloc);
    if (h->s_mid) (void)hipFree(h->s_mid);
    delete h;
}

static std::mutex g_cache_mutex;
// plans compiled by nq_binlr_forward_many, most recently used first (a decoder block calls it with a
// handful of different lists in turn: q, k, v | o | gate, up | down)
struct CachedPlan {
    std::vector<const void*> key;
    nq_plan plan;
};
static std::vector<CachedPlan> g_plan_cache;
constexpr size_t kPlanCacheSize = 32;
static void drop_cached_plan_locked();

// the inputs are host buffers (from_device = false) or device buffers of the current device
static int create_layer(nq_handle* out, int64_t d_out, int64_t d_in, int64_t r, const uint32_t* U_words,
                        const uint32_t* V_words, const uint16_t* s_out_fp16, const uint16_t* s_in_fp16,
                        int x_dtype, int y_dtype, uint32_t flags, bool from_device)
{
    const hipMemcpyKind kind = from_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    if (!out) return fail(NQ_E_NULL, "nq_binlr_create: out is NULL");
    *out = nullptr;
    if (d_out < 1 || d_in < 1 || r < 1) return fail(NQ_E_SHAPE, "nq_binlr_create: d_out, d_in, r must be >= 1");
    if (d_out > NQ_MAX_DIM || d_in > NQ_MAX_DIM || r > NQ_MAX_DIM)
        return fail(NQ_E_SHAPE, "nq_binlr_create: dimension exceeds NQ_MAX_DIM");
    if (!U_words || !V_words || !s_out_fp16 || !s_in_fp16) return fail(NQ_E_NULL, "nq_binlr_create: NULL input");
    if (x_dtype != NQ_F32 && x_dtype != NQ_F16 && x_dtype != NQ_BF16)
        return fail(NQ_E_INVALID_ARG, "nq_binlr_create: x_dtype must be NQ_F32, NQ_F16 or NQ_BF16");
    if (y_dtype != NQ_F32 && y_dtype != NQ_F16 && y_dtype != NQ_BF16)
        return fail(NQ_E_INVALID_ARG, "nq_binlr_create: y_dtype must be NQ_F32, NQ_F16 or NQ_BF16");
    if (flags & ~(NQ_FLAG_DECODE_VALU | NQ_FLAG_NO_PREFILL)) return fail(NQ_E_INVALID_ARG, "nq_binlr_create: unknown flag");

    nq_handle h = new (std::nothrow) nq_binlr_s();
    if (!h) return fail(NQ_E_HIP, "nq_binlr_create: out of host memory");
    memset(h, 0, sizeof *h);
    h->d_out = d_out; h->d_in = d_in; h->r = r;
    h->x_dtype = x_dtype; h->y_dtype = y_dtype; h->flags = flags;
    hipError_t e = hipGetDevice(&h->device);
    if (e != hipSuccess) { delete h; return hip_fail(e, "hipGetDevice", __FILE__, __LINE__); }

    const int64_t wpr = (r + 31) / 32;
    const size_t vt_bytes = tile_words(r, d_in) * 4, u_bytes = tile_words(d_out, r) * 4;
    const size_t sin_bytes = align_up((size_t)d_in * 2, 256), sout_bytes = align_up((size_t)d_out * 2, 256);
    const size_t w_total = vt_bytes + u_bytes + sin_bytes + sout_bytes;

    // decode workspace
    const size_t ws_total = carve_workspace(nullptr, nullptr, d_in, r, NQ_DECODE_MAX_BATCH);

    uint32_t* d_canon = nullptr;
    const size_t canon_u = (size_t)d_out * wpr * 4, canon_v = (size_t)d_in * wpr * 4;
    int rc = NQ_OK;
#define CREATE_HIP(call)                                                   \
    do {                                                                   \
        hipError_t e__ = (call);                                           \
        if (e__ != hipSuccess) {                                           \
            rc = hip_fail(e__, #call, __FILE__, __LINE__);                 \
            goto done;                                                     \
        }                                                                  \
    } while (0)
    h->w_bytes = w_total;
    h->ws_bytes = ws_total;
    CREATE_HIP(slab_alloc(w_total, h->device, 0, &h->w_alloc, &h->w_slab));
    CREATE_HIP(slab_alloc(ws_total, h->device, 1, &h->ws_alloc, &h->ws_slab));
    CREATE_HIP(hipMalloc((void**)&d_canon, std::max(canon_u, canon_v)));
    {
        char* p = (char*)h->w_alloc;
        h->vt_tiles = (uint32_t*)p; p += vt_bytes;
        h->u_tiles = (uint32_t*)p; p += u_bytes;
        h->s_in = (uint16_t*)p; p += sin_bytes;
        h->s_out = (uint16_t*)p;
        (void)carve_workspace(&h->ws, (char*)h->ws_alloc, d_in, r, NQ_DECODE_MAX_BATCH);
    }
    CREATE_HIP(hipMemset(h->ws_alloc, 0, ws_total));
    CREATE_HIP(hipMemcpy(d_canon, V_words, canon_v, kind));
    rc = launch_repack(d_canon, wpr, true, r, d_in, h->vt_tiles, nullptr);
    if (rc != NQ_OK) goto done;
    CREATE_HIP(hipDeviceSynchronize());
    CREATE_HIP(hipMemcpy(d_canon, U_words, canon_u, kind));
    rc = launch_repack(d_canon, wpr, false, d_out, r, h->u_tiles, nullptr);
    if (rc != NQ_OK) goto done;
    CREATE_HIP(hipMemcpy(h->s_in, s_in_fp16, (size_t)d_in * 2, kind));
    CREATE_HIP(hipMemcpy(h->s_out, s_out_fp16, (size_t)d_out * 2, kind));
    CREATE_HIP(hipDeviceSynchronize());
#undef CREATE_HIP
done:
    if (d_canon) (void)hipFree(d_canon);
    if (rc != NQ_OK) {
        free_handle(h);
        return rc;
    }
    *out = h;
    return NQ_OK;
}

extern "C" int nq_binlr_create(nq_handle* out, int64_t d_out, int64_t d_in, int64_t r, const uint32_t* U_words,
                               const uint32_t* V_words, const uint16_t* s_out_fp16, const uint16_t* s_in_fp16,
                               int x_dtype, int y_dtype, uint32_t flags)
{
    return create_layer(out, d_out, d_in, r, U_words, V_words, s_out_fp16, s_in_fp16, x_dtype, y_dtype, flags, false);
}

extern "C" int nq_binlr_create_from_device(nq_handle* out, int64_t d_out, int64_t d_in, int64_t r,
                                           const uint32_t* d_U_words, const uint32_t* d_V_words,
                                           const uint16_t* d_s_out_fp16, const uint16_t* d_s_in_fp16, int x_dtype,
                                           int y_dtype, uint32_t flags)
{
    return create_layer(out, d_out, d_in, r, d_U_words, d_V_words, d_s_out_fp16, d_s_in_fp16, x_dtype, y_dtype, flags,
                        true);
}

extern "C" int nq_pack_signs_device(const void* d_signs, int dtype, int64_t rows, int64_t cols, uint32_t* d_words,
                                    int32_t* d_invalid, void* stream)
{
    if (!d_signs || !d_words) return fail(NQ_E_NULL, "nq_pack_signs_device: NULL buffer");
    if (rows < 1 || cols < 1) return fail(NQ_E_SHAPE, "nq_pack_signs_device: rows and cols must be >= 1");
    if (rows > 0x7fffffffLL || cols > 65535LL * 256)
        return fail(NQ_E_SHAPE, "nq_pack_signs_device: matrix too large for one launch");
    if (dtype != NQ_I8 && dtype != NQ_F32 && dtype != NQ_F16 && dtype != NQ_BF16)
        return fail(NQ_E_INVALID_ARG, "nq_pack_signs_device: dtype must be NQ_I8, NQ_F32, NQ_F16 or NQ_BF16");
    return launch_pack_signs(d_signs, dtype, rows, cols, d_words, (int*)d_invalid, (hipStream_t)stream);
}

extern "C" int nq_binlr_destroy(nq_handle h)
{
    if (!h) return NQ_OK;
    {
        std::lock_guard<std::mutex> lk(g_cache_mutex);
        drop_cached_plan_locked();
    }
    free_handle(h);
    return NQ_OK;
}

extern "C" size_t nq_binlr_weight_bytes(nq_handle h)
{
    if (!h) return 0;
    return (size_t)(h->r * (h->d_in + h->d_out) + 7) / 8 + 2 * (size_t)(h->d_in + h->d_out) +
           (h->s_mid ? 2 * (size_t)h->r : 0);
}

extern "C" int nq_binlr_set_mid_scale(nq_handle h, const uint16_t* s_mid_fp16)
{
    if (!h) return fail(NQ_E_NULL, "nq_binlr_set_mid_scale: NULL handle");
    {
        std::lock_guard<std::mutex> lk(g_cache_mutex);
        drop_cached_plan_locked();                       // its descriptors hold the old pointer
    }
    NQ_HIP(hipDeviceSynchronize());
    if (!s_mid_fp16) {
        if (h->s_mid) NQ_HIP(hipFree(h->s_mid));
        h->s_mid = nullptr;
        h->mid_exp = 0;
        return NQ_OK;
    }
    float mx = 0.f;
    for (int64_t k = 0; k < h->r; ++k) {
        const float v = half_to_float_host(s_mid_fp16[k]);
        if (!(std::fabs(v) <= 65504.f)) return fail(NQ_E_INVALID_ARG, "nq_binlr_set_mid_scale: non-finite scale");
        mx = std::max(mx, std::fabs(v));
    }
    int e = 0;
    if (mx > 0.f) {
        (void)std::frexp(mx, &e);                          // mx = f 2^e, f in [0.5, 1)  ->  mx <= 2^e
        e = std::max(-8, std::min(16, e));
    }
    const size_t bytes = (size_t)round_up(h->r, kTileRows) * 2;
    if (!h->s_mid) NQ_HIP(hipMalloc((void**)&h->s_mid, bytes));
    NQ_HIP(hipMemset(h->s_mid, 0, bytes));
    NQ_HIP(hipMemcpy(h->s_mid, s_mid_fp16, (size_t)h->r * 2, hipMemcpyHostToDevice));
    h->mid_exp = e;
    return NQ_OK;
}

// grows the dense path's workspace to `need` bytes (never shrinks it)
static int grow_prefill_workspace(nq_handle h, size_t need)
{
    if (need <= h->pf_bytes) return NQ_OK;
    NQ_HIP(hipDeviceSynchronize());
    if (h->pf_alloc) NQ_HIP(hipFree(h->pf_alloc));
    h->pf_alloc = nullptr;
    h->pf_bytes = 0;
    NQ_HIP(hipMalloc(&h->pf_alloc, need));
    h->pf_bytes = need;
    NQ_HIP(hipMemset(h->pf_alloc, 0, need));
    NQ_HIP(hipDeviceSynchronize());
    return NQ_OK;
}

static int ensure_prefill_workspace(nq_handle h, int batch)
{
    return grow_prefill_workspace(h, prefill_workspace_bytes(h->d_out, h->d_in, h->r, batch));
}

extern "C" int nq_binlr_reserve(nq_handle h, int max_batch)
{
    if (!h) return fail(NQ_E_NULL, "nq_binlr_reserve: NULL handle");
    if (max_batch < 1) return fail(NQ_E_INVALID_ARG, "nq_binlr_reserve: max_batch must be >= 1");
    if (max_batch < NQ_PREFILL_MIN_BATCH || (h->flags & (NQ_FLAG_NO_PREFILL | NQ_FLAG_DECODE_VALU))) return NQ_OK;   // decode workspace is fixed
    // The dense path's need is not monotone in the batch: smaller batches split the reduction
    // over more workgroups and keep more partial sums.  It depends on the batch only through its
    // padding to whole 64-token tiles, so the maximum over every padding up to max_batch's is taken.
    size_t need = 0;
    for (int64_t b = 64; ; b += 64) {
        const int bb = (int)std::min<int64_t>(b, max_batch);
        need = std::max(need, prefill_workspace_bytes(h->d_out, h->d_in, h->r, bb));
        if (b >= max_batch) break;
    }
    int rc = grow_prefill_workspace(h, need);
    if (rc != NQ_OK) return rc;
    h->pf_batch = std::max(h->pf_batch, max_batch);
    return NQ_OK;
}

extern "C" int nq_binlr_reserved(nq_handle h, int* max_batch, size_t* workspace_bytes)
{
    if (!h) return fail(NQ_E_NULL, "nq_binlr_reserved: NULL handle");
    if (max_batch) *max_batch = std::max(h->pf_batch, (int)NQ_DECODE_MAX_BATCH);
    if (workspace_bytes) *workspace_bytes = h->pf_bytes;
    return NQ_OK;
}

static QuantDesc make_qx(nq_handle h, const DecodeWorkspace& w, const void* x)
{
    QuantDesc q;
    q.x = x; q.scale = h->s_in; q.bq = w.bq_x; q.meta = w.meta_x;
    q.N = (int)h->d_in; q.n_chunks = (int)n_steps(h->d_in) * 4; q.x_stride = (int)h->d_in; q.dtype = h->x_dtype;
    q.mag_exp = 22;
    return q;
}
static StageDesc make_s1(nq_handle h, const DecodeWorkspace& w)
{
    StageDesc s;
    s.tiles = h->vt_tiles; s.bq = w.bq_x; s.meta = w.meta_x; s.out_scale = nullptr; s.out = w.t;
    s.M = (int)h->r; s.n_steps = (int)n_steps(h->d_in); s.out_stride = w.t_stride; s.out_dtype = NQ_F32;
    return s;
}
static QuantDesc make_qt(nq_handle h, const DecodeWorkspace& w)
{
    QuantDesc q;
    q.x = w.t; q.scale = h->s_mid; q.bq = w.bq_t; q.meta = w.meta_t;
    q.N = (int)h->r; q.n_chunks = (int)n_steps(h->r) * 4; q.x_stride = w.t_stride; q.dtype = NQ_F32;
    q.mag_exp = 22;
    return q;
}
static StageDesc make_s2(nq_handle h, const DecodeWorkspace& w, void* y)
{
    StageDesc s;
    s.tiles = h->u_tiles; s.bq = w.bq_t; s.meta = w.meta_t; s.out_scale = h->s_out; s.out = y;
    s.M = (int)h->d_out; s.n_steps = (int)n_steps(h->r); s.out_stride = (int)h->d_out; s.out_dtype = h->y_dtype;
    return s;
}

// Row blocks chained into one item of the stream kernel for an op with `nst` steps per row block:
// aim at stream_target_steps(batch) steps per wave, but keep at least ~16 items per CU in the launch
// (`total_rb` = row blocks of the whole launch).
static int rbs_per_stream_item(int n_rb, int nst, int total_rb, int batch)
{
    int per = std::max(1, stream_target_steps(batch) / std::max(1, nst));
    per = std::min(per, stream_max_rbs(batch));
    const int want_items = device_cu_count() * 16;
    while (per > 1 && total_rb / per < want_items) per /= 2;
    return std::min(per, std::max(1, n_rb));
}

// one pass of the streaming path for batch <= 8; `unscaled`: without the output scale (z = U t)
// (`w`: the workspace the kernels use -- the layer's own, or one carved out of the static scratch array)
static int decode_once(nq_handle h, const DecodeWorkspace& w, const void* x, void* y, int batch, hipStream_t s,
                       bool unscaled = false)
{
    int rc;
    if (h->flags & NQ_FLAG_DECODE_VALU) {
        rc = launch_valu_gemv(h->vt_tiles, x, h->x_dtype, (int)h->d_in, h->s_in, nullptr, w.t, NQ_F32, w.t_stride,
                              h->r, h->d_in, batch, s);
        if (rc != NQ_OK) return rc;
        return launch_valu_gemv(h->u_tiles, w.t, NQ_F32, w.t_stride, h->s_mid, unscaled ? nullptr : h->s_out, y, h->y_dtype,
                                (int)h->d_out, h->d_out, h->r, batch, s);
    }
    // a small layer on its own: one workgroup runs both stages in one launch, t staying in LDS
    if (small_layer_fits(h, batch)) return launch_small_layer(h, w, x, y, unscaled, s);
    QuantDesc qx = make_qx(h, w, x);
    StageDesc s1 = make_s1(h, w);
    QuantDesc qt = make_qt(h, w);
    StageDesc s2 = make_s2(h, w, y);
    if (unscaled) s2.out_scale = nullptr;
    const int rb1 = (int)n_rowblocks(h->r), rb2 = (int)n_rowblocks(h->d_out);
    const int w1 = stage_schedule(rb1, s1.n_steps, batch), w2 = stage_schedule(rb2, s2.n_steps, batch);
    const int per1 = w1 == 1 ? rbs_per_stream_item(rb1, s1.n_steps, rb1, batch) : 1;
    const int per2 = w2 == 1 ? rbs_per_stream_item(rb2, s2.n_steps, rb2, batch) : 1;
    // a lone layer is bound by launch latency: where the quantised input of a stage fits LDS, the
    // stage quantises it itself (two launches per forward instead of four)
    // (reductions of up to 4096 elements by the waves of the one- or four-wave kernel, longer ones
    // up to 16384 by the 16-wave kernel)
    const bool no_fuse = opt_flag(OPT_NO_FUSE), no_selfq = opt_flag(OPT_NO_SELFQ);
    const int sq1 = no_selfq ? 0 : selfq_width(s1.n_steps, s1.n_steps, batch);
    const int sq2 = no_selfq ? 0 : selfq_width(s2.n_steps, s2.n_steps, batch);
    if (sq1) {
        if ((rc = launch_selfq(nullptr, rb1, qx, s1, sq1, s1.n_steps, s)) != NQ_OK) return rc;
    } else if (!no_fuse && fused_fits(s1.n_steps, batch)) {
        if ((rc = launch_fused(qx, s1, s)) != NQ_OK) return rc;
    } else {
        if ((rc = launch_quantize(nullptr, qx, 1, qx.n_chunks, batch, s)) != NQ_OK) return rc;
        if ((rc = launch_stage(nullptr, s1, nullptr, (rb1 + per1 - 1) / per1, w1, per1, batch, s)) != NQ_OK) return rc;
    }
    if (sq2) return launch_selfq(nullptr, rb2, qt, s2, sq2, s2.n_steps, s);
    if (!no_fuse && fused_fits(s2.n_steps, batch)) return launch_fused(qt, s2, s);
    if ((rc = launch_quantize(nullptr, qt, 1, qt.n_chunks, batch, s)) != NQ_OK) return rc;
    return launch_stage(nullptr, s2, nullptr, (rb2 + per2 - 1) / per2, w2, per2, batch, s);
}

static int check_xy(const char* who, const void* x, const void* y, size_t x_bytes, size_t y_bytes)
{
    char buf[160];
    if (!x || !y) { snprintf(buf, sizeof buf, "%s: x or y is NULL", who); return fail(NQ_E_NULL, buf); }
    if (!aligned16(x) || !aligned16(y)) { snprintf(buf, sizeof buf, "%s: x and y must be 16-byte aligned", who); return fail(NQ_E_ALIGN, buf); }
    const char* xb = (const char*)x; const char* yb = (const char*)y;
    if (xb < yb + y_bytes && yb < xb + x_bytes) { snprintf(buf, sizeof buf, "%s: x and y overlap", who); return fail(NQ_E_INVALID_ARG, buf); }
    return NQ_OK;
}

extern "C" int nq_binlr_forward(nq_handle h, const void* x, void* y, int batch, void* stream)
{
    if (!h) return fail(NQ_E_NULL, "nq_binlr_forward: NULL handle");
    if (batch < 1) return fail(NQ_E_INVALID_ARG, "nq_binlr_forward: batch must be >= 1");
    const size_t xs = dtype_size(h->x_dtype);
    const size_t ys = dtype_size(h->y_dtype);
    int rc = check_xy("nq_binlr_forward", x, y, (size_t)batch * h->d_in * xs, (size_t)batch * h->d_out * ys);
    if (rc != NQ_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (batch <= NQ_DECODE_MAX_BATCH) return decode_once(h, h->ws, x, y, batch, s);
    if (batch >= NQ_PREFILL_MIN_BATCH && !(h->flags & (NQ_FLAG_NO_PREFILL | NQ_FLAG_DECODE_VALU))) {
        if ((rc = ensure_prefill_workspace(h, batch)) != NQ_OK) return rc;
        PrefillArgs a;
        a.vt_tiles = h->vt_tiles; a.u_tiles = h->u_tiles; a.s_in = h->s_in; a.s_out = h->s_out;
        a.s_mid = h->s_mid; a.mid_exp = h->mid_exp;
        a.x = x; a.y = y; a.workspace = h->pf_alloc;
        a.d_out = h->d_out; a.d_in = h->d_in; a.r = h->r; a.batch = batch; a.x_dtype = h->x_dtype; a.y_dtype = h->y_dtype;
        return launch_prefill(a, s);
    }
    // larger batches without the dense path: chunks of 8 through the streaming path (each chunk re-reads the bits)
    for (int b0 = 0; b0 < batch; b0 += NQ_DECODE_MAX_BATCH) {
        int nb = std::min(NQ_DECODE_MAX_BATCH, batch - b0);
        rc = decode_once(h, h->ws, (const char*)x + (size_t)b0 * h->d_in * xs, (char*)y + (size_t)b0 * h->d_out * ys, nb, s);
        if (rc != NQ_OK) return rc;
    }
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// nq_binlr_forward for callers that must not allocate: the kernels' scratch memory (fixed-point
// x' and t, token constants, the intermediate t) is carved out of one file-scope device array
// instead of the layer's workspace.  Every GPU the library runs on holds its own copy of the array
// (at its own address) until the process ends.  The array's name is only a host-side stand-in: its
// device address is looked up once per device and that pointer is what the kernels receive.
// ---------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = NQ_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// the address of the current device's copy of `scratch` (the current device must be `device`)
static int static_scratch(int device, char** out)
{
    if (device < 0 || device >= kMaxDevices) return fail(NQ_E_UNSUPPORTED, "nq_binlr_forward_static: device index beyond 63");
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        NQ_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(NQ_E_HIP, "nq_binlr_forward_static: hipGetSymbolAddress returned no address");
        g_scratch_ptr[device] = p;
    }
    *out = (char*)g_scratch_ptr[device];
    return NQ_OK;
}

extern "C" int nq_binlr_forward_static(nq_handle h, const void* x, void* y, int batch, void* stream)
{
    if (!h) return fail(NQ_E_NULL, "nq_binlr_forward_static: NULL handle");
    if (batch < 1) return fail(NQ_E_INVALID_ARG, "nq_binlr_forward_static: batch must be >= 1");
    if (batch > NQ_DECODE_MAX_BATCH)
        return fail(NQ_E_UNSUPPORTED, "nq_binlr_forward_static: batch must be <= NQ_DECODE_MAX_BATCH (the streaming kernels)");
    int rc = check_xy("nq_binlr_forward_static", x, y, (size_t)batch * h->d_in * dtype_size(h->x_dtype),
                      (size_t)batch * h->d_out * dtype_size(h->y_dtype));
    if (rc != NQ_OK) return rc;
    const size_t need = carve_workspace(nullptr, nullptr, h->d_in, h->r, batch);
    if (need > kStaticScratchBytes) {
        char buf[200];
        snprintf(buf, sizeof buf, "nq_binlr_forward_static: batch %d of this layer needs %zu bytes of scratch, the static array holds %zu",
                 batch, need, kStaticScratchBytes);
        return fail(NQ_E_SHAPE, buf);
    }
    int dev = -1;
    NQ_HIP(hipGetDevice(&dev));
    if (dev != h->device) return fail(NQ_E_INVALID_ARG, "nq_binlr_forward_static: the layer lives on another device than the current one");
    char* base = nullptr;
    if ((rc = static_scratch(dev, &base)) != NQ_OK) return rc;
    // Nothing in the array has to start at zero: every byte a kernel reads from it was written
    // earlier in the same call (the quantiser writes the padding of the fixed-point vectors too; the
    // bytes past the last token that the shared-input kernel may touch only ever meet 0 bits).
    DecodeWorkspace w;
    (void)carve_workspace(&w, base, h->d_in, h->r, batch);
    return decode_once(h, w, x, y, batch, (hipStream_t)stream);
}

extern "C" int nq_binlr_export_words(nq_handle h, uint32_t* U_words, uint32_t* V_words)
{
    if (!h) return fail(NQ_E_NULL, "nq_binlr_export_words: NULL handle");
    const int64_t wpr = (h->r + 31) / 32;
    const size_t canon_u = (size_t)h->d_out * wpr * 4, canon_v = (size_t)h->d_in * wpr * 4;
    uint32_t* d_canon = nullptr;
    NQ_HIP(hipMalloc((void**)&d_canon, std::max(canon_u, canon_v)));
    int rc = NQ_OK;
    hipError_t e = hipSuccess;
    if (V_words) {
        rc = launch_export(h->vt_tiles, wpr, true, h->r, h->d_in, d_canon, nullptr);
        if (rc == NQ_OK && (e = hipMemcpy(V_words, d_canon, canon_v, hipMemcpyDeviceToHost)) != hipSuccess)
            rc = hip_fail(e, "hipMemcpy", __FILE__, __LINE__);
    }
    if (rc == NQ_OK && U_words) {
        rc = launch_export(h->u_tiles, wpr, false, h->d_out, h->r, d_canon, nullptr);
        if (rc == NQ_OK && (e = hipMemcpy(U_words, d_canon, canon_u, hipMemcpyDeviceToHost)) != hipSuccess)
            rc = hip_fail(e, "hipMemcpy", __FILE__, __LINE__);
    }
    (void)hipFree(d_canon);
    return rc;
}

extern "C" int nq_binlr_read_intermediate(nq_handle h, float* t_host, int batch)
{
    if (!h || !t_host) return fail(NQ_E_NULL, "nq_binlr_read_intermediate: NULL pointer");
    if (batch < 1 || batch > NQ_DECODE_MAX_BATCH) return fail(NQ_E_INVALID_ARG, "nq_binlr_read_intermediate: batch must be 1..8");
    NQ_HIP(hipDeviceSynchronize());
    NQ_HIP(hipMemcpy2D(t_host, (size_t)h->r * 4, h->ws.t, (size_t)h->ws.t_stride * 4, (size_t)h->r * 4, batch,
                       hipMemcpyDeviceToHost));
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// plans
// ---------------------------------------------------------------------------------------------
extern "C" int nq_plan_destroy(nq_plan p)
{
    if (!p) return NQ_OK;
    if (p->have_events)
        for (auto& e : p->ev) (void)hipEventDestroy(e);
    if (p->alloc) (void)hipFree(p->alloc);
    delete p;
    return NQ_OK;
}

// every cached plan goes (a handle one of them may use is being destroyed or changed)
static void drop_cached_plan_locked()
{
    if (g_plan_cache.empty()) return;
    (void)hipDeviceSynchronize();
    for (CachedPlan& c : g_plan_cache) nq_plan_destroy(c.plan);
    g_plan_cache.clear();
}

extern "C" int nq_plan_create(nq_plan* out, const nq_handle* hs, const void* const* xs, void* const* ys, int n,
                              int batch)
{
    if (!out) return fail(NQ_E_NULL, "nq_plan_create: out is NULL");
    *out = nullptr;
    if (!hs || !xs || !ys) return fail(NQ_E_NULL, "nq_plan_create: NULL array");
    if (n < 1) return fail(NQ_E_INVALID_ARG, "nq_plan_create: n must be >= 1");
    if (batch < 1) return fail(NQ_E_INVALID_ARG, "nq_plan_create: batch must be >= 1");
    if (batch > NQ_DECODE_MAX_BATCH) return fail(NQ_E_UNSUPPORTED, "nq_plan_create: batch must be <= NQ_DECODE_MAX_BATCH");
    std::vector<nq_handle> sorted(hs, hs + n);
    for (int i = 0; i < n; ++i) {
        if (!hs[i]) return fail(NQ_E_NULL, "nq_plan_create: NULL handle in list");
        if (hs[i]->flags & NQ_FLAG_DECODE_VALU) return fail(NQ_E_UNSUPPORTED, "nq_plan_create: handle uses NQ_FLAG_DECODE_VALU");
        if (hs[i]->device != hs[0]->device) return fail(NQ_E_INVALID_ARG, "nq_plan_create: handles live on different devices");
        int rc = check_xy("nq_plan_create", xs[i], ys[i], (size_t)batch * hs[i]->d_in * dtype_size(hs[i]->x_dtype),
                          (size_t)batch * hs[i]->d_out * dtype_size(hs[i]->y_dtype));
        if (rc != NQ_OK) return rc;
    }
    std::sort(sorted.begin(), sorted.end());
    if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end())
        return fail(NQ_E_INVALID_ARG, "nq_plan_create: a handle appears twice (its workspace would be shared)");

    std::vector<QuantDesc> qx(n), qt(n);
    std::vector<StageDesc> s1(n), s2(n);
    for (int i = 0; i < n; ++i) {
        qx[i] = make_qx(hs[i], hs[i]->ws, xs[i]);
        s1[i] = make_s1(hs[i], hs[i]->ws);
        qt[i] = make_qt(hs[i], hs[i]->ws);
        s2[i] = make_s2(hs[i], hs[i]->ws, ys[i]);
    }
    // one work list per stage launch; its shape follows the schedule the launch will use
    int sched[2], max_steps_of[2] = {0, 0};
    std::vector<WorkItem> lists[2];
    for (int st = 0; st < 2; ++st) {
        const std::vector<StageDesc>& sd = st == 0 ? s1 : s2;
        double sq = 0, sm = 0;
        int total_rb = 0;
        for (int i = 0; i < n; ++i) {
            const int nrb = (int)n_rowblocks(sd[i].M);
            total_rb += nrb;
            sq += (double)nrb * sd[i].n_steps * sd[i].n_steps;     // mean length seen by a streamed tile
            sm += (double)nrb * sd[i].n_steps;
        }
        int w = stage_schedule(total_rb, (int)(sq / sm), batch);
        // A short launch at batch 1 is bound by launch latency, not by bandwidth: the stage then
        // quantises its own input, which saves the quantisation launch -- by the waves of the one- or
        // four-wave kernel where the reductions are short enough for it (measured faster than the
        // 16-wave kernel at every size: 4 layers of 4096x4096 r=1024 11.6 vs 13.0 us, 32 layers 13.8
        // vs 29.5), else by the 16-wave kernel, every workgroup for itself, up to NQ_FUSE_MAX_MB of tiles.
        {
            int max_steps = 0;
            for (int i = 0; i < n; ++i) max_steps = std::max(max_steps, sd[i].n_steps);
            const double tile_mb = sm * (kTileWords * 4) / 1.0e6;
            int min_steps = max_steps;
            for (int i = 0; i < n; ++i) min_steps = std::min(min_steps, sd[i].n_steps);
            const bool full = total_rb >= schedule_full_rowblocks();
            const int sq = full || opt_flag(OPT_NO_SELFQ) ? 0 : selfq_width(max_steps, min_steps, batch);
            if (sq)
                w = sq == 1 ? kSelfqSchedule1 : kSelfqSchedule4;
            else if (batch == 1 && !opt_flag(OPT_NO_FUSE) && fused_fits(max_steps, batch) &&
                     tile_mb <= (double)opt_or(OPT_FUSE_MAX_MB, 24))
                w = kFusedSchedule;
            max_steps_of[st] = max_steps;
            // A launch that fills the chip keeps its schedule, but its waves quantise their own share
            // of the input: no quantisation launch, and the B operand comes out of LDS.
            // batch 6..8, short reductions: the shared-input kernel with the whole input resident in LDS
            if (w == 1 && batch > 5 && max_steps <= 16 && total_rb >= schedule_full_rowblocks() && !opt_flag(OPT_NO_RESIDENT))
                w = kSharedResidentSchedule;
            // (with four waves per row block only where every reduction has 48 steps or more: for shorter
            // ones the split kernel with its quantisation launch measured the same or faster -- 35 steps:
            // 62 against 66 us, 55 steps: 85 against 85 -- and a mixed list, as stage 2 of the 70B stack
            // with its 8-step ranks, 442 + 9 against 476 us)
            if ((w == 1 || (w == 4 && min_steps >= opt_or(OPT_SELFQ4_MIN_STEPS, 48))) && !opt_flag(OPT_NO_SELFQ) && full &&
                selfq_fits(w, max_steps, min_steps, batch))
                w = w == 1 ? kSelfqSchedule1 : kSelfqSchedule4;
        }
        // Option "two_slice_b8": at batch 6..8 the shared-input launches take their input as 16-bit fixed point (the top
        // byte slice stays zero), which puts the eight tokens into ONE group of 16 MFMA columns instead of two.
        if (opt_flag(OPT_TWO_SLICE_B8) && batch >= 6 && (w == kSharedSchedule || w == kSharedResidentSchedule)) {
            w = w == kSharedSchedule ? kSharedSchedule2 : kSharedResidentSchedule2;
            for (int i = 0; i < n; ++i) (st == 0 ? qx : qt)[i].mag_exp = 14;
        }
        sched[st] = w;
        for (int i = 0; i < n; ++i) {
            const int nrb = (int)n_rowblocks(sd[i].M);
            if (is_shared_schedule(w)) {
                // the waves of a workgroup share an op's input: items of kShareWaves x (row blocks per wave) row blocks
                const int group = kShareWaves * shared_per_wave(sd[i].n_steps, batch);
                for (int rb = 0; rb < nrb; rb += group)
                    lists[st].push_back(WorkItem{sd[i].tiles + (size_t)rb * sd[i].n_steps * kTileWords, sd[i].bq,
                                                 sd[i].n_steps, i, rb, std::min(group, nrb - rb)});
                continue;
            }
            const int per = w == 1 ? rbs_per_stream_item(nrb, sd[i].n_steps, total_rb, batch) : 1;
            // runs of `per` row blocks first, then shorter and shorter ones: the sorted list ends in
            // small items, which level out the finishing times of the waves (the hardware hands an
            // idle slot the next item)
            for (int rb = 0; rb < nrb;) {
                const int rem = nrb - rb;
                int c = 1;
                while (c * 3 < rem) c *= 2;                   // smallest power of two >= rem / 3
                c = std::min(std::min(c, per), rem);
                lists[st].push_back(WorkItem{sd[i].tiles + (size_t)rb * sd[i].n_steps * kTileWords, sd[i].bq,
                                             sd[i].n_steps, i, rb, c});
                rb += c;
            }
        }
        // longest items first: the hardware dispatches workgroups in order, so the short ones fill the tail
        std::stable_sort(lists[st].begin(), lists[st].end(), [](const WorkItem& a, const WorkItem& b) {
            return (int64_t)a.n_steps * a.n_rb > (int64_t)b.n_steps * b.n_rb;
        });
        // Workgroup i runs on XCD i % 8, each XCD with its own L2.  Deal the list into 8 queues op by
        // op (an op's items stay together, queues stay sorted) and interleave them, so that all row
        // blocks of a layer read that layer's activation vector through ONE L2 instead of eight.
        {
            constexpr int kXcds = 8;
            std::vector<WorkItem> q[kXcds];
            int lane = -1, last_op = -1;
            size_t load[kXcds] = {0};
            for (const WorkItem& w : lists[st]) {
                if (w.op != last_op) {                       // next op goes to the least loaded queue
                    lane = 0;
                    for (int x = 1; x < kXcds; ++x)
                        if (load[x] < load[lane]) lane = x;
                    last_op = w.op;
                }
                q[lane].push_back(w);
                load[lane] += (size_t)w.n_steps * w.n_rb;
            }
            std::vector<WorkItem> out;
            out.reserve(lists[st].size());
            size_t pos[kXcds] = {0};
            while (out.size() < lists[st].size()) {
                for (int x = 0; x < kXcds; ++x) {
                    if (pos[x] < q[x].size()) out.push_back(q[x][pos[x]++]);
                    else {                                   // queue ran dry: borrow from the fullest one
                        int f = 0;
                        for (int y = 1; y < kXcds; ++y)
                            if (q[y].size() - pos[y] > q[f].size() - pos[f]) f = y;
                        if (pos[f] < q[f].size()) out.push_back(q[f][pos[f]++]);
                    }
                }
            }
            lists[st].swap(out);
        }
    }
    std::vector<WorkItem>& it1 = lists[0];
    std::vector<WorkItem>& it2 = lists[1];

    nq_plan p = new (std::nothrow) nq_plan_s();
    if (!p) return fail(NQ_E_HIP, "nq_plan_create: out of host memory");
    p->n = n; p->batch = batch; p->device = hs[0]->device; p->alloc = nullptr; p->have_events = false;
    p->handles.assign(hs, hs + n);
    p->n_items1 = (int)it1.size(); p->n_items2 = (int)it2.size();
    p->w1 = sched[0]; p->w2 = sched[1];
    p->max_steps1 = max_steps_of[0]; p->max_steps2 = max_steps_of[1];
    p->max_chunks_x = p->max_chunks_t = 0;
    for (int i = 0; i < n; ++i) {
        p->max_chunks_x = std::max(p->max_chunks_x, qx[i].n_chunks);
        p->max_chunks_t = std::max(p->max_chunks_t, qt[i].n_chunks);
    }
    const size_t qb = align_up(sizeof(QuantDesc) * n, 256), sb = align_up(sizeof(StageDesc) * n, 256);
    const size_t i1b = align_up(sizeof(WorkItem) * it1.size(), 256), i2b = align_up(sizeof(WorkItem) * it2.size(), 256);
    // stages on the fused schedule get items that carry their op's descriptors
    std::vector<FusedItem> fit[2];
    for (int st = 0; st < 2; ++st) {
        if (sched[st] != kFusedSchedule && sched[st] != kSelfqSchedule1 && sched[st] != kSelfqSchedule4) continue;
        for (const WorkItem& w : lists[st]) {
            FusedItem f{};
            f.q = st == 0 ? qx[w.op] : qt[w.op];
            f.s = st == 0 ? s1[w.op] : s2[w.op];
            f.rb = w.rb;
            fit[st].push_back(f);
        }
    }
    const size_t f1b = align_up(sizeof(FusedItem) * fit[0].size(), 256), f2b = align_up(sizeof(FusedItem) * fit[1].size(), 256);
    hipError_t e = hipMalloc(&p->alloc, 2 * qb + 2 * sb + i1b + i2b + f1b + f2b);
    if (e != hipSuccess) { delete p; return hip_fail(e, "hipMalloc(plan)", __FILE__, __LINE__); }
    char* c = (char*)p->alloc;
    p->qx = (QuantDesc*)c; c += qb;
    p->qt = (QuantDesc*)c; c += qb;
    p->s1 = (StageDesc*)c; c += sb;
    p->s2 = (StageDesc*)c; c += sb;
    p->items1 = (WorkItem*)c; c += i1b;
    p->items2 = (WorkItem*)c; c += i2b;
    p->fitems1 = (FusedItem*)c; c += f1b;
    p->fitems2 = (FusedItem*)c;
    const struct { void* dst; const void* src; size_t bytes; } copies[] = {
        {p->qx, qx.data(), sizeof(QuantDesc) * n}, {p->qt, qt.data(), sizeof(QuantDesc) * n},
        {p->s1, s1.data(), sizeof(StageDesc) * n}, {p->s2, s2.data(), sizeof(StageDesc) * n},
        {p->items1, it1.data(), sizeof(WorkItem) * it1.size()}, {p->items2, it2.data(), sizeof(WorkItem) * it2.size()},
        {p->fitems1, fit[0].data(), sizeof(FusedItem) * fit[0].size()},
        {p->fitems2, fit[1].data(), sizeof(FusedItem) * fit[1].size()}};
    for (const auto& cp : copies) {
        if (cp.bytes == 0) continue;
        e = hipMemcpy(cp.dst, cp.src, cp.bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) { nq_plan_destroy(p); return hip_fail(e, "hipMemcpy(plan)", __FILE__, __LINE__); }
    }
    *out = p;
    return NQ_OK;
}

static int plan_run(nq_plan p, hipStream_t s, bool timed)
{
    const QuantDesc qdummy{};
    const StageDesc sdummy{};
    int rc;
    // a stage on one of the self-quantising schedules has no quantisation launch
    auto self_quantising = [](int w) { return w == kFusedSchedule || w == kSelfqSchedule1 || w == kSelfqSchedule4; };
    auto run_stage = [&](int w, const StageDesc* sd, const WorkItem* items, const FusedItem* fitems, int n_items,
                         int max_steps) {
        if (w == kFusedSchedule) return launch_fused_list(fitems, n_items, max_steps, s);
        if (w == kSelfqSchedule1 || w == kSelfqSchedule4)
            return launch_selfq(fitems, n_items, qdummy, sdummy, w == kSelfqSchedule1 ? 1 : 4, max_steps, s);
        return launch_stage(sd, sdummy, items, n_items, w, stream_max_rbs(p->batch), p->batch, s);
    };
    // timed: launch k carries the event pair ev[2k], ev[2k + 1], bound to the kernel itself (see LaunchTiming)
    struct Timed {
        Timed(bool on, hipEvent_t a, hipEvent_t b) : on_(on) { if (on) g_launch_timing = LaunchTiming{a, b}; }
        ~Timed() { if (on_) g_launch_timing = LaunchTiming{}; }
        bool on_;
    };
    if (!self_quantising(p->w1)) {
        Timed t(timed, p->ev[0], p->ev[1]);
        if ((rc = launch_quantize(p->qx, qdummy, p->n, p->max_chunks_x, p->batch, s)) != NQ_OK) return rc;
    }
    {
        Timed t(timed, p->ev[2], p->ev[3]);
        if ((rc = run_stage(p->w1, p->s1, p->items1, p->fitems1, p->n_items1, p->max_steps1)) != NQ_OK) return rc;
    }
    if (!self_quantising(p->w2)) {
        Timed t(timed, p->ev[4], p->ev[5]);
        if ((rc = launch_quantize(p->qt, qdummy, p->n, p->max_chunks_t, p->batch, s)) != NQ_OK) return rc;
    }
    {
        Timed t(timed, p->ev[6], p->ev[7]);
        if ((rc = run_stage(p->w2, p->s2, p->items2, p->fitems2, p->n_items2, p->max_steps2)) != NQ_OK) return rc;
    }
    return NQ_OK;
}

extern "C" int nq_plan_schedules(nq_plan p, int w[2])
{
    if (!p || !w) return fail(NQ_E_NULL, "nq_plan_schedules: NULL pointer");
    w[0] = p->w1;
    w[1] = p->w2;
    return NQ_OK;
}

extern "C" int nq_plan_forward(nq_plan p, void* stream)
{
    if (!p) return fail(NQ_E_NULL, "nq_plan_forward: NULL plan");
    return plan_run(p, (hipStream_t)stream, false);
}

extern "C" int nq_plan_forward_timed(nq_plan p, void* stream, float ms[4])
{
    if (!p || !ms) return fail(NQ_E_NULL, "nq_plan_forward_timed: NULL pointer");
    if (!p->have_events) {
        for (auto& e : p->ev) NQ_HIP(hipEventCreate(&e));
        p->have_events = true;
    }
    int rc = plan_run(p, (hipStream_t)stream, true);
    if (rc != NQ_OK) return rc;
    NQ_HIP(hipEventSynchronize(p->ev[7]));
    auto self_quantising = [](int w) { return w == kFusedSchedule || w == kSelfqSchedule1 || w == kSelfqSchedule4; };
    ms[0] = ms[2] = 0.f;
    if (!self_quantising(p->w1)) NQ_HIP(hipEventElapsedTime(&ms[0], p->ev[0], p->ev[1]));
    NQ_HIP(hipEventElapsedTime(&ms[1], p->ev[2], p->ev[3]));
    if (!self_quantising(p->w2)) NQ_HIP(hipEventElapsedTime(&ms[2], p->ev[4], p->ev[5]));
    NQ_HIP(hipEventElapsedTime(&ms[3], p->ev[6], p->ev[7]));
    return NQ_OK;
}

// any batch through the streaming kernels, in passes of up to 8 tokens; `unscaled`: z = U (V^T (s_in (.) x))
static int forward_in_passes(const char* who, nq_handle h, const void* x, void* y, int batch, void* stream, bool unscaled)
{
    char buf[96];
    if (!h) { snprintf(buf, sizeof buf, "%s: NULL handle", who); return fail(NQ_E_NULL, buf); }
    if (batch < 1) { snprintf(buf, sizeof buf, "%s: batch must be >= 1", who); return fail(NQ_E_INVALID_ARG, buf); }
    const size_t xs = dtype_size(h->x_dtype), ys = dtype_size(h->y_dtype);
    int rc = check_xy(who, x, y, (size_t)batch * h->d_in * xs, (size_t)batch * h->d_out * ys);
    if (rc != NQ_OK) return rc;
    for (int b0 = 0; b0 < batch; b0 += NQ_DECODE_MAX_BATCH) {
        const int nb = std::min(NQ_DECODE_MAX_BATCH, batch - b0);
        rc = decode_once(h, h->ws, (const char*)x + (size_t)b0 * h->d_in * xs, (char*)y + (size_t)b0 * h->d_out * ys, nb,
                         (hipStream_t)stream, unscaled);
        if (rc != NQ_OK) return rc;
    }
    return NQ_OK;
}

extern "C" int nq_binlr_forward_unscaled(nq_handle h, const void* x, void* z, int batch, void* stream)
{
    return forward_in_passes("nq_binlr_forward_unscaled", h, x, z, batch, stream, true);
}

extern "C" int nq_binlr_forward_exact(nq_handle h, const void* x, void* y, int batch, void* stream)
{
    return forward_in_passes("nq_binlr_forward_exact", h, x, y, batch, stream, false);
}

// w = [s_in (.)] V (s_mid (.) (U^T (s_out (.) g))) from the resident tiles
static int transposed_forward(const char* who, nq_handle h, const void* g, float* w, int batch, void* stream, bool with_s_in)
{
    char buf[96];
    if (!h) { snprintf(buf, sizeof buf, "%s: NULL handle", who); return fail(NQ_E_NULL, buf); }
    if (batch < 1) { snprintf(buf, sizeof buf, "%s: batch must be >= 1", who); return fail(NQ_E_INVALID_ARG, buf); }
    const size_t gs = dtype_size(h->y_dtype);
    int rc = check_xy(who, g, w, (size_t)batch * h->d_out * gs, (size_t)batch * h->d_in * sizeof(float));
    if (rc != NQ_OK) return rc;
    // workspace for passes of up to 8 tokens: the intermediate u = s_mid (.) U^T (s_out (.) g) [8][r padded], then the
    // partial sums of the larger of the two products
    const int nb_max = NQ_DECODE_MAX_BATCH;
    const size_t r_pad = (size_t)n_steps(h->r) * kTileCols;
    const size_t u_bytes = align_up(nb_max * r_pad * sizeof(float), 256);
    const size_t need = u_bytes + std::max(gemv_t_partial_bytes(h->d_out, h->r, nb_max), gemv_t_partial_bytes(h->r, h->d_in, nb_max));
    if (h->tp_bytes < need) {
        NQ_HIP(hipDeviceSynchronize());
        if (h->tp_alloc) NQ_HIP(hipFree(h->tp_alloc));
        h->tp_alloc = nullptr;
        h->tp_bytes = 0;
        NQ_HIP(hipMalloc(&h->tp_alloc, need));
        h->tp_bytes = need;
    }
    float* u = (float*)h->tp_alloc;
    double* partial = (double*)((char*)h->tp_alloc + u_bytes);
    hipStream_t s = (hipStream_t)stream;
    for (int b0 = 0; b0 < batch; b0 += nb_max) {
        const int nb = std::min(nb_max, batch - b0);
        // u = s_mid (.) U^T (s_out (.) g): the tiles of U ([d_out][r]) read along their columns
        rc = launch_gemv_t(h->u_tiles, h->d_out, h->r, (const char*)g + (size_t)b0 * h->d_out * gs, h->y_dtype, (int)h->d_out, h->s_out,
                           h->s_mid, u, NQ_F32, (int)r_pad, nb, partial, s);
        if (rc != NQ_OK) return rc;
        // w = V u: the tiles of V^T ([r][d_in]) read along their columns
        rc = launch_gemv_t(h->vt_tiles, h->r, h->d_in, u, NQ_F32, (int)r_pad, nullptr, with_s_in ? h->s_in : nullptr,
                           w + (size_t)b0 * h->d_in, NQ_F32, (int)h->d_in, nb, partial, s);
        if (rc != NQ_OK) return rc;
    }
    return NQ_OK;
}

extern "C" int nq_binlr_forward_transposed_unscaled(nq_handle h, const void* g, float* w, int batch, void* stream)
{
    return transposed_forward("nq_binlr_forward_transposed_unscaled", h, g, w, batch, stream, false);
}

extern "C" int nq_binlr_backward_input(nq_handle h, const void* g, float* dx, int batch, void* stream)
{
    return transposed_forward("nq_binlr_backward_input", h, g, dx, batch, stream, true);
}

extern "C" int nq_scale_grad(const void* a, int a_dtype, const void* b, int b_dtype, int batch, int64_t n, float* out,
                             void* stream)
{
    if (!a || !b || !out) return fail(NQ_E_NULL, "nq_scale_grad: NULL pointer");
    if (batch < 1 || n < 1) return fail(NQ_E_INVALID_ARG, "nq_scale_grad: batch and n must be >= 1");
    for (int dt : {a_dtype, b_dtype})
        if (dt != NQ_F32 && dt != NQ_F16 && dt != NQ_BF16) return fail(NQ_E_INVALID_ARG, "nq_scale_grad: dtype must be NQ_F32, NQ_F16 or NQ_BF16");
    return launch_scale_grad(a, a_dtype, b, b_dtype, batch, n, out, (hipStream_t)stream);
}

extern "C" int nq_binlr_forward_many(const nq_handle* hs, const void* const* xs, void* const* ys, int n, int batch,
                                     void* stream)
{
    if (!hs || !xs || !ys) return fail(NQ_E_NULL, "nq_binlr_forward_many: NULL array");
    if (n < 1) return fail(NQ_E_INVALID_ARG, "nq_binlr_forward_many: n must be >= 1");
    std::vector<const void*> key;
    key.reserve(3 * (size_t)n + 2);
    key.push_back((const void*)(intptr_t)n);
    key.push_back((const void*)(intptr_t)batch);
    for (int i = 0; i < n; ++i) { key.push_back(hs[i]); key.push_back(xs[i]); key.push_back(ys[i]); }
    std::lock_guard<std::mutex> lk(g_cache_mutex);
    size_t at = 0;
    while (at < g_plan_cache.size() && g_plan_cache[at].key != key) ++at;
    if (at == g_plan_cache.size()) {
        nq_plan p = nullptr;
        int rc = nq_plan_create(&p, hs, xs, ys, n, batch);
        if (rc != NQ_OK) return rc;
        if (g_plan_cache.size() >= kPlanCacheSize) {          // the least recently used one makes room
            (void)hipDeviceSynchronize();
            nq_plan_destroy(g_plan_cache.back().plan);
            g_plan_cache.pop_back();
        }
        g_plan_cache.push_back(CachedPlan{key, p});
        at = g_plan_cache.size() - 1;
    }
    if (at != 0) std::rotate(g_plan_cache.begin(), g_plan_cache.begin() + at, g_plan_cache.begin() + at + 1);
    return plan_run(g_plan_cache.front().plan, (hipStream_t)stream, false);
}
