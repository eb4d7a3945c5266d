// Host runtime and C ABI of libeeverify (declarations and semantics: include/ee.h).
#include <fcntl.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <climits>
#include <new>
#include <vector>

#include "ee_kernels.hpp"

using namespace ee;

// ------------------------------------------------------------------ errors

static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail(EE_EDEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

extern "C" const char *ee_last_error(void) { return g_err; }

// ------------------------------------------------------------------ objects

struct ee_model {
    ee_model_config cfg;
    int device;
    int nwg;
    size_t lds_budget;           // dynamic LDS bytes each launch asks for
    ModelDev host_md;            // the descriptor the launches carry by value
    // Weight-stream plans and tiled weights per GEMM kind (a launch gets its plan and weights by
    // value): [0] every workgroup streams whole rows of K, [1] K split over groups of workgroups
    // (launches of more than 16 rows; only the kinds where it pays have one, nwg = 0 otherwise).
    // One allocation per kind and variant, layer l (adapters: stored exit l) at w + l * wstride (uint4 units).
    GemmPlan plan[2][G_KINDS];
    const uint4 *w[2][G_KINDS];
    long long wstride[2][G_KINDS];
    std::vector<void *> allocs;  // every device allocation of the model
    const float *g_exit[EE_MAX_EXITS];
    // exit-head adapters (per stored exit): biases of the hidden units and the summed output biases
    const float *ad_bdown[EE_MAX_EXITS];
    const float *ad_bup[EE_MAX_EXITS];
};

struct ee_session {
    const ee_model *m;
    unsigned flags;
    int max_ctx, max_gamma;
    hipStream_t stream;
    hipStream_t run_stream;          // stream the pass this session leads is enqueued on (its own, or the first
                                     // group leader's when a batch runs as several groups)
    hipEvent_t ev_start, ev_final, ev_exit[EE_MAX_EXITS];
    // KV cache
    int n_pages;
    uint16_t *kpool, *vpool;
    int *dev_page_table;
    int *host_page_table;            // pinned mirror
    std::vector<int> free_pages;     // LIFO free list of physical pages
    int pages_used;                  // logical pages mapped
    float2 *rope;
    // device state and staging
    int *dev_state;
    int *dev_drafts;
    int *host_drafts;                // pinned
    float *host_sample;              // pinned staging of a sampled pass: draft distributions, then u, then v (EE_SAMPLING)
    float *dev_sample;               // device copy of the same
    int *dev_sample_out;             // [2 * EE_MAX_ROWS + 1] rows' tokens, keep flags, arrival counter
    int *dev_pf_tokens;
    int *host_pf_tokens;             // pinned
    uint16_t *dev_pf_emb;
    ee_verify_result *result;        // pinned, mapped
    ee_verify_result *dev_result;
    SessDev *dev_sessdev;            // [EE_MAX_BATCH] per-pass session descriptors
    SessDev *host_sessdev;           // pinned staging for them
    Scratch sc;
    int att_items_cap;               // attention work items the partials buffer has room for
    int att_splits_opt;              // EE_OPT_ATT_SPLITS (0: chosen per pass)
    int head_batch;                  // EE_OPT_HEAD_BATCH: exit heads per launch of the LM head
    bool scatter_pages;              // EE_OPT_SCATTER_PAGES
    int flight_row0;                 // first row of this session in the pass in flight
    unsigned long long popped_mask;  // exits of the pass in flight that ee_exit_pop has handed out
    std::vector<hipEvent_t> lt_events;   // EE_TIME_LAUNCHES: event pairs around every launch of the pass
    std::vector<int> lt_codes;           // what each timed launch ran (EE_LAUNCH_* code)
    std::vector<void *> allocs;
    // host mirror of the session state
    int kv_len;
    int pending;
    bool has_pending;
    bool in_flight;                  // a verify pass was enqueued and not yet waited for
    int flight_gamma, flight_exits;
    ee_session *leader;              // session whose stream/events carry the pass in flight
};

// ------------------------------------------------------------------ planning

typedef void (*pass_kernel_t)(PassArgs);

static pass_kernel_t gemm_kernel(int rows)
{
    return rows <= 16 ? ee_gemm_kernel<1> : (rows <= 32 ? ee_gemm_kernel<2> : ee_gemm_kernel<3>);
}

static pass_kernel_t att_kernel(int hd) { return hd == 128 ? ee_att_kernel<128> : ee_att_kernel<64>; }

// n-tiles the busiest workgroup owns
static int plan_max_local(const GemmPlan &p)
{
    int mx = 0;
    for (int g = 0; g < p.nwg; ++g) {
        int nt0, n_local;
        wg_units(p, g, nt0, n_local);
        mx = std::max(mx, n_local);
    }
    return mx;
}

// ksl > 0: K split over groups of 1 << ksl workgroups where the k-tiles divide evenly (otherwise the plan comes back unsplit)
static GemmPlan make_plan(int N, int K, int tpu, int nwg_max, int ksl = 0)
{
    GemmPlan p;
    memset(&p, 0, sizeof p);
    p.N = N;
    p.K = K;
    p.NT = (N + 15) / 16;
    p.NT = (p.NT + tpu - 1) / tpu * tpu;
    p.KT = (K + 31) / 32;
    p.tpu = tpu;
    p.U = p.NT / tpu;
    p.KTs = p.KT;
    if (ksl > 0 && p.KT % (1 << ksl) == 0 && (nwg_max >> ksl) >= 1) {
        p.ksl = ksl;
        p.KTs = p.KT >> ksl;
    }
    // the fewest (groups of) workgroups that do not raise the busiest one's share
    const int groups_max = nwg_max >> p.ksl;
    const int most = (p.U + groups_max - 1) / groups_max;
    p.nwg = std::min(groups_max, (p.U + most - 1) / most) << p.ksl;
    // every wave's sequence has room for the busiest wave's k-steps of every n-tile
    p.steps = wave_ksteps(p.KTs, 0) * plan_max_local(p);
    return p;
}

// LDS map of one GEMM launch with `rows` rows (see StageLds)
static bool plan_lds(const GemmPlan &p, int rows, size_t lds_total, StageLds &ly)
{
    const size_t misc = (MISC_BYTES + 255) / 256 * 256;
    if (lds_total < misc + 4096) return false;
    const size_t avail = (lds_total - misc) / 256 * 256;
    const size_t tile_bytes = (size_t)rows * 128;           // one k-tile of the input: two terms, all rows
    const int KT8 = (p.KTs + SWAVES - 1) / SWAVES * SWAVES;   // the k-tiles one workgroup streams
    memset(&ly, 0, sizeof ly);
    if ((size_t)KT8 * tile_bytes <= avail) {
        ly.kbt = KT8;
        ly.nkb = 1;
        ly.nbuf = 1;
    } else {
        ly.nbuf = 2;
        ly.kbt = (int)(avail / 2 / tile_bytes) / SWAVES * SWAVES;
        if (ly.kbt < SWAVES) return false;
        // blocks of one k-step per wave: a block is read faster than its copy arrives; a third
        // buffer lets the copy run two blocks ahead
        if (ly.kbt == SWAVES && avail / 3 / tile_bytes >= (size_t)SWAVES) ly.nbuf = 3;
        ly.nkb = (p.KTs + ly.kbt - 1) / ly.kbt;
        if (ly.nkb < ly.nbuf) ly.nbuf = std::max(ly.nkb, 1);
    }
    ly.xbuf_bytes = (int)((size_t)ly.kbt * tile_bytes);
    // cross-wave sum: SWAVES partial tiles plus one logits / squares tile per n-tile of a chunk
    int chunk = (int)(avail / ((size_t)rows * 64 * (SWAVES + 1)));
    chunk = std::min(chunk, GROUP_TILES);
    if (p.tpu == 2) chunk &= ~1;
    if (chunk < p.tpu) return false;
    ly.chunk = chunk;
    ly.zbuf_off = (int)((size_t)SWAVES * chunk * rows * 64);
    ly.misc_off = (int)avail;
    return true;
}

template <typename T>
static int dev_alloc(std::vector<void *> &list, T **out, size_t count, bool zero = true)
{
    void *p = nullptr;
    size_t bytes = std::max<size_t>(count * sizeof(T), 256);
    HIP_TRY(hipMalloc(&p, bytes));
    list.push_back(p);
    if (zero) HIP_TRY(hipMemset(p, 0, bytes));
    *out = reinterpret_cast<T *>(p);
    return EE_OK;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ------------------------------------------------------------------ model load

namespace {
struct FileMap {
    void *p = MAP_FAILED;
    size_t n = 0;
    ~FileMap()
    {
        if (p != MAP_FAILED) munmap(p, n);
    }
};
}  // namespace

// concatenates the sources row-wise in a device buffer and writes layer slice `dst` in tile order
static int upload_tiled(const ee_model *m, const GemmPlan &pl, int perm, const uint16_t *const *srcs, int n_src,
                        size_t elems_each, uint16_t *tmp, uint4 *dst)
{
    for (int i = 0; i < n_src; ++i)
        HIP_TRY(hipMemcpy(tmp + (size_t)i * elems_each, srcs[i], elems_each * 2, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(tile_weights_kernel, dim3(pl.nwg), dim3(512), 0, 0, tmp, dst, pl, perm,
                       m->cfg.d_model, m->cfg.head_dim, m->cfg.d_ffn);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipDeviceSynchronize());
    return EE_OK;
}

static int upload_gain(const uint16_t *src, int d, uint16_t *tmp, float *dst)
{
    HIP_TRY(hipMemcpy(tmp, src, (size_t)d * 2, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((d + 255) / 256), dim3(256), 0, 0, tmp, dst, d);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipDeviceSynchronize());
    return EE_OK;
}

// which GEMM kinds get a K-split tile order in models loaded for more than 16 rows, and the splits (ee_tune_k_split)
static unsigned g_ksplit_kinds = (1u << G_O) | (1u << G_DN);
static int g_ksplit_log2 = KSPLIT_LOG2;

extern "C" int ee_tune_k_split(unsigned kind_mask, int log2_splits)
{
    if (log2_splits < 1 || (1 << log2_splits) > SWAVES || kind_mask >= (1u << G_KINDS))
        return fail(EE_EINVAL, "ee_tune_k_split: mask %u, log2 splits %d (mask below %u, 1 <= log2 splits <= 3)", kind_mask, log2_splits, 1u << G_KINDS);
    g_ksplit_kinds = kind_mask;
    g_ksplit_log2 = log2_splits;
    return EE_OK;
}

extern "C" int ee_model_free(ee_model *m)
{
    if (!m) return EE_OK;
    hipSetDevice(m->device);
    for (void *p : m->allocs) hipFree(p);
    delete m;
    return EE_OK;
}

extern "C" int ee_model_load_ex(const char *path, int device, int max_rows, ee_model **out)
{
    if (!path || !out) return fail(EE_EINVAL, "ee_model_load: null argument");
    if (max_rows < 1 || max_rows > EE_MAX_ROWS) return fail(EE_EINVAL, "ee_model_load: max_rows %d not in [1,%d]", max_rows, EE_MAX_ROWS);
    *out = nullptr;
    int fd = open(path, O_RDONLY);
    if (fd < 0) return fail(EE_EIO, "ee_model_load: cannot open %s", path);
    struct stat st;
    if (fstat(fd, &st) != 0) {
        close(fd);
        return fail(EE_EIO, "ee_model_load: cannot stat %s", path);
    }
    FileMap fm;
    fm.n = (size_t)st.st_size;
    if (fm.n < 256) {
        close(fd);
        return fail(EE_EFORMAT, "ee_model_load: %s is shorter than a header", path);
    }
    fm.p = mmap(nullptr, fm.n, PROT_READ, MAP_SHARED, fd, 0);
    close(fd);
    if (fm.p == MAP_FAILED) return fail(EE_EIO, "ee_model_load: cannot map %s", path);
    const uint8_t *b = static_cast<const uint8_t *>(fm.p);
    if (memcmp(b, "EEVMODL1", 8) != 0) return fail(EE_EFORMAT, "ee_model_load: bad magic in %s", path);
    uint32_t u[8];
    memcpy(u, b + 8, sizeof u);
    if (u[0] != 1) return fail(EE_EFORMAT, "ee_model_load: unsupported version %u", u[0]);
    ee_model_config c;
    memset(&c, 0, sizeof c);
    c.n_layers = (int)u[1];
    c.d_model = (int)u[2];
    c.n_heads = (int)u[3];
    c.head_dim = (int)u[4];
    c.d_ffn = (int)u[5];
    c.vocab = (int)u[6];
    c.n_exits = (int)u[7];
    memcpy(&c.rope_base, b + 40, 4);
    memcpy(&c.rms_eps, b + 44, 4);
    if (c.n_layers < 1 || c.n_layers > 4096 || c.d_model < 16 || c.n_heads < 1 || c.d_ffn < 1 || c.vocab < 1 ||
        c.n_exits < 0 || c.n_exits > EE_MAX_EXITS || (long long)c.n_heads * c.head_dim != c.d_model)
        return fail(EE_EFORMAT, "ee_model_load: inconsistent header");
    if (c.head_dim != 64 && c.head_dim != 128)
        return fail(EE_EFORMAT, "ee_model_load: head_dim %d unsupported (64 or 128)", c.head_dim);
    if (c.d_model % 16 != 0 || c.d_ffn % 2 != 0)
        return fail(EE_EFORMAT, "ee_model_load: d_model must be a multiple of 16, d_ffn even");
    uint32_t ex[EE_MAX_EXITS], ad[2];
    static_assert(EE_MAX_EXITS == 40, "the header's exit table has 40 entries");
    memcpy(ex, b + 48, sizeof ex);
    memcpy(ad, b + 208, sizeof ad);
    const int n_ad = (int)ad[0], ad_w = (int)ad[1];
    if ((n_ad == 0) != (ad_w == 0) || n_ad < 0 || n_ad > 64 || ad_w < 0 || ad_w > 4096 || (n_ad * ad_w) % 16 != 0)
        return fail(EE_EFORMAT, "ee_model_load: bad adapter shape %d x %d (the hidden units together must be a multiple of 16)", n_ad, ad_w);
    const size_t A = (size_t)n_ad * (size_t)ad_w;
    c.n_adapters = n_ad;
    c.adapter_width = ad_w;
    for (int i = 0; i < c.n_exits; ++i) {
        c.exit_layers[i] = (int)ex[i];
        if (c.exit_layers[i] < 1 || c.exit_layers[i] >= c.n_layers || (i > 0 && c.exit_layers[i] <= c.exit_layers[i - 1]))
            return fail(EE_EFORMAT, "ee_model_load: bad exit layer list");
    }
    const size_t d = (size_t)c.d_model, F = (size_t)c.d_ffn, V = (size_t)c.vocab;
    // tensor offsets: each tensor starts on a 256-byte boundary, fixed order
    size_t off = 256;
    auto take = [&](size_t elems) -> const uint16_t * {
        off = align_up(off, 256);
        const uint16_t *p = reinterpret_cast<const uint16_t *>(b + off);
        off += elems * 2;
        return p;
    };
    struct LayerSrc {
        const uint16_t *g_attn, *wq, *wk, *wv, *wo, *g_ffn, *wg, *wu, *wd;
    };
    const uint16_t *emb = take(V * d);
    std::vector<LayerSrc> ls((size_t)c.n_layers);
    for (auto &l : ls) {
        l.g_attn = take(d);
        l.wq = take(d * d);
        l.wk = take(d * d);
        l.wv = take(d * d);
        l.wo = take(d * d);
        l.g_ffn = take(d);
        l.wg = take(F * d);
        l.wu = take(F * d);
        l.wd = take(d * F);
    }
    const uint16_t *g_final = take(d);
    const uint16_t *w_lm = take(V * d);
    const uint16_t *g_exit_src[EE_MAX_EXITS];
    for (int i = 0; i < c.n_exits; ++i) g_exit_src[i] = take(d);
    struct AdapterSrc {
        const uint16_t *down, *bdown, *up, *bup;
    };
    std::vector<AdapterSrc> ads((size_t)(A ? c.n_exits : 0));
    for (auto &x : ads) {
        x.down = take(A * d);
        x.bdown = take(A);
        x.up = take(d * A);
        x.bup = take((size_t)n_ad * d);
    }
    if (off > fm.n) return fail(EE_EFORMAT, "ee_model_load: %s is truncated (%zu < %zu bytes)", path, fm.n, off);

    int n_dev = 0;
    HIP_TRY(hipGetDeviceCount(&n_dev));
    if (device < 0 || device >= n_dev) return fail(EE_EINVAL, "ee_model_load: device %d of %d", device, n_dev);
    HIP_TRY(hipSetDevice(device));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, device));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(EE_EDEVICE, "ee_model_load: device %d is %s, this library is built for gfx950 only", device, prop.gcnArchName);

    ee_model *m = new (std::nothrow) ee_model();
    if (!m) return fail(EE_EDEVICE, "out of host memory");
    m->device = device;
    m->nwg = std::min(prop.multiProcessorCount, 256);   // one workgroup per compute unit; the accept step reads at most 256 candidates per row
    c.max_rows = max_rows;
    c.n_workgroups = m->nwg;
    m->cfg = c;
    ModelDev &md = m->host_md;
    memset(&md, 0, sizeof md);
    md.L = c.n_layers;
    md.d = c.d_model;
    md.H = c.n_heads;
    md.hd = c.head_dim;
    md.F = c.d_ffn;
    md.V = c.vocab;
    md.eps = c.rms_eps;
    md.att_scale = (float)(1.0 / sqrt((double)c.head_dim));
    md.Kpad_d = (int)align_up(d, 32);
    md.Kpad_F = (int)align_up(F, 32);
    md.rows_max = max_rows;
    md.A = (int)A;
    md.Kpad_A = (int)align_up(A, 32);
    if (c.d_ffn % 16 != 0) {
        ee_model_free(m);
        return fail(EE_EFORMAT, "ee_model_load: d_ffn must be a multiple of 16");
    }

    // ---- weight-stream plans (independent of the rows) and the LDS block every launch asks for
    size_t lds_cap = prop.sharedMemPerBlock;
    {
        int optin = 0;
        if (hipDeviceGetAttribute(&optin, hipDeviceAttributeSharedMemPerBlockOptin, device) == hipSuccess && optin > 0)
            lds_cap = std::max(lds_cap, (size_t)optin);
    }
    auto plan_of = [&](int kind, int ksl) {
        switch (kind) {
        case G_QKV: return make_plan(3 * c.d_model, c.d_model, 1, m->nwg, ksl);
        case G_O: return make_plan(c.d_model, c.d_model, 1, m->nwg, ksl);
        case G_GU: return make_plan(2 * c.d_ffn, c.d_model, 2, m->nwg, ksl);
        case G_DN: return make_plan(c.d_model, c.d_ffn, 1, m->nwg, ksl);
        case G_HEAD: return make_plan(c.vocab, c.d_model, 1, m->nwg, ksl);
        case G_AD: return make_plan(A ? (int)A : 16, c.d_model, 1, m->nwg, ksl);
        default: return make_plan(c.d_model, A ? (int)A : 32, 1, m->nwg, ksl);
        }
    };
    memset(m->plan, 0, sizeof m->plan);
    memset(m->w, 0, sizeof m->w);
    memset(m->wstride, 0, sizeof m->wstride);
    for (int k = 0; k < G_KINDS; ++k) m->plan[0][k] = plan_of(k, 0);
    if (max_rows > 16) {
        // Launches of more than 16 rows: K split four ways for the projections whose input is as large
        // as, or larger than, a workgroup's share of the weights (see GemmPlan).  Those weights are
        // kept in both tile orders; launches of up to 16 rows keep using the unsplit one.
        const unsigned kinds = g_ksplit_kinds;
        const int ksl = g_ksplit_log2;
        for (int k = 0; k < G_KINDS; ++k)
            if ((kinds >> k) & 1u) {
                const GemmPlan p = plan_of(k, ksl);
                if (p.ksl > 0) m->plan[1][k] = p;
            }
    }
    m->lds_budget = lds_cap / 256 * 256;   // the whole block: more than half of it also keeps a compute unit to one workgroup
    for (int v = 0; v < 2; ++v)
        for (int k = 0; k < G_KINDS; ++k) {
            const GemmPlan &pl = m->plan[v][k];
            if (pl.nwg == 0) continue;
            StageLds ly;
            if (!plan_lds(pl, max_rows, m->lds_budget, ly)) {
                ee_model_free(m);
                return fail(EE_EDEVICE, "ee_model_load: max_rows %d needs more LDS than the device's %zu bytes", max_rows, lds_cap);
            }
            // the kernels' exact small-integer division (div_small) covers the unit arithmetic of this plan
            if ((long long)pl.U * pl.nwg > DIV_SMALL_MAX || pl.N > DIV_SMALL_MAX) {
                ee_model_free(m);
                return fail(EE_EFORMAT, "ee_model_load: a weight matrix with %d rows is beyond what the kernels' index arithmetic covers", pl.N);
            }
            // tile offsets inside a stage are 32-bit byte offsets
            if ((long long)pl.steps * pl.nwg * SWAVES * 1024 >= (1LL << 31)) {
                ee_model_free(m);
                return fail(EE_EFORMAT, "ee_model_load: a weight matrix of %d x %d exceeds the 2 GiB a stage can address", pl.N, pl.K);
            }
            m->wstride[v][k] = (long long)pl.steps * pl.nwg * SWAVES * 64;
        }
    {
        const size_t att = (size_t)WAVES * ATT_ROWS * (c.head_dim + 2) * sizeof(float) + 16;  // wave partials + the "last item of the unit" flag
        const size_t emb = (size_t)max_rows * (((c.d_model + m->nwg - 1) / m->nwg + 3) / 4 + 1) * sizeof(float);
        if (att > m->lds_budget || emb > m->lds_budget) {
            ee_model_free(m);
            return fail(EE_EDEVICE, "ee_model_load: not enough LDS");
        }
        pass_kernel_t ks[6] = {gemm_kernel(16), gemm_kernel(32), gemm_kernel(48), att_kernel(64), att_kernel(128), ee_misc_kernel};
        for (pass_kernel_t k : ks) {
            hipError_t fe = hipFuncSetAttribute(reinterpret_cast<const void *>(k),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)m->lds_budget);
            if (fe != hipSuccess) {
                ee_model_free(m);
                return fail(EE_EDEVICE, "hipFuncSetAttribute(%zu bytes LDS): %s", m->lds_budget, hipGetErrorString(fe));
            }
        }
    }

    int rc = EE_OK;
    uint16_t *tmp = nullptr;
    size_t tmp_elems = std::max({V * d, 3 * d * d, 2 * F * d, A * d});
    void *tmp_raw = nullptr;
    if (hipMalloc(&tmp_raw, tmp_elems * 2) != hipSuccess) {
        ee_model_free(m);
        return fail(EE_EDEVICE, "ee_model_load: cannot allocate the upload buffer");
    }
    tmp = static_cast<uint16_t *>(tmp_raw);

    auto bail = [&](int code) {
        hipFree(tmp_raw);
        ee_model_free(m);
        return code;
    };

    // embedding table stays row-major
    uint16_t *dev_emb = nullptr;
    if ((rc = dev_alloc(m->allocs, &dev_emb, V * d, false)) != EE_OK) return bail(rc);
    if (hipMemcpy(dev_emb, emb, V * d * 2, hipMemcpyHostToDevice) != hipSuccess) return bail(fail(EE_EDEVICE, "upload of the embedding table failed"));
    md.emb = dev_emb;

    // tiled weights: one allocation per GEMM kind and variant, layers at a fixed stride.  Zero-filled: tile slots no wave's
    // sequence reaches (a wave without k-steps, the shorter sequences' tails) are still loaded by the clamped
    // look-ahead and multiplied with zeros, so they must hold finite values.
    float *g_attn = nullptr, *g_ffn = nullptr, *g_final_d = nullptr;
    const size_t Lz = (size_t)c.n_layers;
    uint4 *wdev[2][G_KINDS];
    memset(wdev, 0, sizeof wdev);
    for (int v = 0; v < 2; ++v)
        for (int k = 0; k < G_KINDS; ++k) {
            if (m->plan[v][k].nwg == 0 || ((k == G_AD || k == G_AU) && !A)) continue;
            const size_t slices = k == G_HEAD ? 1 : ((k == G_AD || k == G_AU) ? (size_t)c.n_exits : Lz);
            if ((rc = dev_alloc(m->allocs, &wdev[v][k], std::max<size_t>(slices, 1) * (size_t)m->wstride[v][k], true)) != EE_OK) return bail(rc);
            m->w[v][k] = wdev[v][k];
        }
    // every variant of a kind from the same upload
    auto tile_all = [&](int kind, int perm, const uint16_t *const *srcs, int n_src, size_t elems_each, size_t slice) {
        for (int v = 0; v < 2; ++v) {
            if (!wdev[v][kind]) continue;
            const int r = upload_tiled(m, m->plan[v][kind], perm, srcs, v == 0 ? n_src : 0, elems_each, tmp,
                                       wdev[v][kind] + slice * (size_t)m->wstride[v][kind]);
            if (r != EE_OK) return r;
        }
        return (int)EE_OK;
    };
    if ((rc = dev_alloc(m->allocs, &g_attn, Lz * d, false)) != EE_OK) return bail(rc);
    if ((rc = dev_alloc(m->allocs, &g_ffn, Lz * d, false)) != EE_OK) return bail(rc);
    if ((rc = dev_alloc(m->allocs, &g_final_d, d, false)) != EE_OK) return bail(rc);
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerSrc &s = ls[(size_t)l];
        const uint16_t *qkv[3] = {s.wq, s.wk, s.wv};
        const uint16_t *gu[2] = {s.wg, s.wu};
        const uint16_t *so[1] = {s.wo}, *sd[1] = {s.wd};
        if ((rc = tile_all(G_QKV, PERM_QKV, qkv, 3, d * d, (size_t)l)) != EE_OK) return bail(rc);
        if ((rc = tile_all(G_O, PERM_NONE, so, 1, d * d, (size_t)l)) != EE_OK) return bail(rc);
        if ((rc = tile_all(G_GU, PERM_GU, gu, 2, F * d, (size_t)l)) != EE_OK) return bail(rc);
        if ((rc = tile_all(G_DN, PERM_NONE, sd, 1, d * F, (size_t)l)) != EE_OK) return bail(rc);
        if ((rc = upload_gain(s.g_attn, c.d_model, tmp, g_attn + (size_t)l * d)) != EE_OK) return bail(rc);
        if ((rc = upload_gain(s.g_ffn, c.d_model, tmp, g_ffn + (size_t)l * d)) != EE_OK) return bail(rc);
    }
    {
        const uint16_t *lm[1] = {w_lm};
        if ((rc = tile_all(G_HEAD, PERM_NONE, lm, 1, V * d, 0)) != EE_OK) return bail(rc);
        if ((rc = upload_gain(g_final, c.d_model, tmp, g_final_d)) != EE_OK) return bail(rc);
        for (int i = 0; i < c.n_exits; ++i) {
            float *ge = nullptr;
            if ((rc = dev_alloc(m->allocs, &ge, d, false)) != EE_OK) return bail(rc);
            if ((rc = upload_gain(g_exit_src[i], c.d_model, tmp, ge)) != EE_OK) return bail(rc);
            m->g_exit[i] = ge;
        }
    }
    if (A) {
        // adapters: weights in tile order per stored exit; biases as fp32, the bottlenecks' output biases summed in order
        for (int i = 0; i < c.n_exits; ++i) {
            const uint16_t *sd_[1] = {ads[(size_t)i].down}, *su_[1] = {ads[(size_t)i].up};
            if ((rc = tile_all(G_AD, PERM_NONE, sd_, 1, A * d, (size_t)i)) != EE_OK) return bail(rc);
            if ((rc = tile_all(G_AU, PERM_NONE, su_, 1, d * A, (size_t)i)) != EE_OK) return bail(rc);
            float *bd = nullptr, *bu = nullptr;
            if ((rc = dev_alloc(m->allocs, &bd, A, false)) != EE_OK) return bail(rc);
            if ((rc = dev_alloc(m->allocs, &bu, d, false)) != EE_OK) return bail(rc);
            std::vector<float> hb(std::max(A, d));
            auto bf = [](uint16_t v) {
                uint32_t u32 = (uint32_t)v << 16;
                float f;
                memcpy(&f, &u32, 4);
                return f;
            };
            for (size_t r = 0; r < A; ++r) hb[r] = bf(ads[(size_t)i].bdown[r]);
            if (hipMemcpy(bd, hb.data(), A * 4, hipMemcpyHostToDevice) != hipSuccess) return bail(fail(EE_EDEVICE, "upload of adapter biases failed"));
            for (size_t col = 0; col < d; ++col) {
                float acc = 0.f;
                for (int j = 0; j < n_ad; ++j) acc += bf(ads[(size_t)i].bup[(size_t)j * d + col]);
                hb[col] = acc;
            }
            if (hipMemcpy(bu, hb.data(), d * 4, hipMemcpyHostToDevice) != hipSuccess) return bail(fail(EE_EDEVICE, "upload of adapter biases failed"));
            m->ad_bdown[i] = bd;
            m->ad_bup[i] = bu;
        }
    }
    md.g_attn = g_attn;
    md.g_ffn = g_ffn;
    md.g_final = g_final_d;
    hipFree(tmp_raw);
    tmp_raw = nullptr;
    if (hipDeviceSynchronize() != hipSuccess) return bail(fail(EE_EDEVICE, "device error while loading the model"));
    *out = m;
    return EE_OK;
}

extern "C" int ee_model_load(const char *path, int device, ee_model **out)
{
    return ee_model_load_ex(path, device, 16, out);
}

extern "C" int ee_model_info(const ee_model *m, ee_model_config *out)
{
    if (!m || !out) return fail(EE_EINVAL, "ee_model_info: null argument");
    *out = m->cfg;
    return EE_OK;
}

// ------------------------------------------------------------------ sessions

// Splits of the cache's pages per attention unit: enough items to occupy every compute unit
// (one unit alone pulls a head's cache too slowly), at least one page per split, no more
// than ATT_TILES pages per wave, and no more items than the leader's partials buffer holds.
// Returns 0 when the buffer is too small for the context.
static int attention_splits(const ee_session *lead, int items_cap, int n_sess, int M, int n_pos_max)
{
    const ee_model *m = lead->m;
    const int chunks = (M + ATT_ROWS - 1) / ATT_ROWS;
    const int units = n_sess * m->cfg.n_heads * chunks;
    const int pages = (n_pos_max + KV_PAGE - 1) / KV_PAGE;
    const int forced = (pages + ATT_TILES * WAVES - 1) / (ATT_TILES * WAVES);
    const int cap = std::min(ATT_MAX_SPLITS, items_cap / std::max(units, 1));
    int s = std::min(m->nwg / std::max(units, 1), pages);
    if (lead->att_splits_opt > 0) s = lead->att_splits_opt;
    s = std::max(std::max(1, s), forced);
    if (forced > cap) return 0;
    return std::min(s, cap);
}

extern "C" int ee_session_free(ee_session *s)
{
    if (!s) return EE_OK;
    hipSetDevice(s->m->device);
    if (s->stream) hipStreamSynchronize(s->stream);
    for (void *p : s->allocs) hipFree(p);
    if (s->host_page_table) hipHostFree(s->host_page_table);
    if (s->host_drafts) hipHostFree(s->host_drafts);
    if (s->host_sample) hipHostFree(s->host_sample);
    if (s->host_pf_tokens) hipHostFree(s->host_pf_tokens);
    if (s->result) hipHostFree(s->result);
    if (s->host_sessdev) hipHostFree(s->host_sessdev);
    if (s->ev_start) hipEventDestroy(s->ev_start);
    if (s->ev_final) hipEventDestroy(s->ev_final);
    for (hipEvent_t e : s->ev_exit)
        if (e) hipEventDestroy(e);
    for (hipEvent_t e : s->lt_events) hipEventDestroy(e);
    if (s->stream) hipStreamDestroy(s->stream);
    delete s;
    return EE_OK;
}

extern "C" int ee_session_create(const ee_model *m, int max_ctx, int max_gamma, unsigned flags, ee_session **out)
{
    if (!m || !out) return fail(EE_EINVAL, "ee_session_create: null argument");
    *out = nullptr;
    if (max_gamma < 1 || max_gamma > EE_MAX_M - 1) return fail(EE_EINVAL, "ee_session_create: max_gamma %d not in [1,%d]", max_gamma, EE_MAX_M - 1);
    if (max_gamma + 1 > m->cfg.max_rows) return fail(EE_EINVAL, "ee_session_create: max_gamma+1 exceeds the model's max_rows %d", m->cfg.max_rows);
    // attention keeps at most ATT_TILES pages per wave and ATT_MAX_SPLITS splits per head
    const int ctx_cap = ATT_MAX_SPLITS * ATT_TILES * WAVES * KV_PAGE;
    if (max_ctx < max_gamma + 2 || max_ctx > ctx_cap)
        return fail(EE_EINVAL, "ee_session_create: max_ctx %d out of range (at most %d)", max_ctx, ctx_cap);
    HIP_TRY(hipSetDevice(m->device));
    ee_session *s = new (std::nothrow) ee_session();
    if (!s) return fail(EE_EDEVICE, "out of host memory");
    s->m = m;
    s->flags = flags;
    s->max_ctx = max_ctx;
    s->max_gamma = max_gamma;
    s->leader = s;
    s->head_batch = 1;
    const ee_model_config &c = m->cfg;
    const int rows_max = c.max_rows;
    const size_t d = (size_t)c.d_model;
    int rc = EE_OK;
#define S_TRY(expr)                  \
    do {                             \
        rc = (expr);                 \
        if (rc != EE_OK) {           \
            ee_session_free(s);      \
            return rc;               \
        }                            \
    } while (0)
#define S_HIP(expr)                                                                          \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) {                                                              \
            ee_session_free(s);                                                              \
            return fail(EE_EDEVICE, "%s failed: %s", #expr, hipGetErrorString(e_));          \
        }                                                                                    \
    } while (0)

    S_HIP(hipStreamCreate(&s->stream));
    s->run_stream = s->stream;
    S_HIP(hipEventCreate(&s->ev_start));
    S_HIP(hipEventCreate(&s->ev_final));
    for (int i = 0; i < EE_MAX_EXITS; ++i) S_HIP(hipEventCreate(&s->ev_exit[i]));

    s->n_pages = (max_ctx + KV_PAGE - 1) / KV_PAGE;
    size_t kv_elems = (size_t)c.n_layers * s->n_pages * c.n_heads * KV_PAGE * 2 * c.head_dim;  // hi and lo terms
    S_TRY(dev_alloc(s->allocs, &s->kpool, kv_elems));
    S_TRY(dev_alloc(s->allocs, &s->vpool, kv_elems));
    S_TRY(dev_alloc(s->allocs, &s->dev_page_table, (size_t)s->n_pages));
    S_HIP(hipHostMalloc(reinterpret_cast<void **>(&s->host_page_table), (size_t)s->n_pages * sizeof(int), hipHostMallocDefault));
    memset(s->host_page_table, 0, (size_t)s->n_pages * sizeof(int));
    // LIFO free list: the first logical page gets the highest physical page, so
    // the mapping is never the identity
    for (int p = s->n_pages - 1; p >= 0; --p) s->free_pages.push_back(p);  // handed out in ascending order
    s->pages_used = 0;

    // RoPE table in double on the host: angle = pos * base^(-2j/hd)
    {
        const int half = c.head_dim / 2;
        std::vector<float2> tab((size_t)max_ctx * half);
        for (int j = 0; j < half; ++j) {
            double theta = pow((double)c.rope_base, -2.0 * (double)j / (double)c.head_dim);
            for (int pos = 0; pos < max_ctx; ++pos) {
                double ang = (double)pos * theta;
                tab[(size_t)pos * half + j] = make_float2((float)cos(ang), (float)sin(ang));
            }
        }
        S_TRY(dev_alloc(s->allocs, &s->rope, tab.size(), false));
        S_HIP(hipMemcpy(s->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice));
    }

    S_TRY(dev_alloc(s->allocs, &s->dev_state, 4));
    S_TRY(dev_alloc(s->allocs, &s->dev_drafts, EE_MAX_M));
    S_HIP(hipHostMalloc(reinterpret_cast<void **>(&s->host_drafts), EE_MAX_M * sizeof(int), hipHostMallocDefault));
    S_TRY(dev_alloc(s->allocs, &s->dev_pf_tokens, (size_t)rows_max));
    S_HIP(hipHostMalloc(reinterpret_cast<void **>(&s->host_pf_tokens), (size_t)rows_max * sizeof(int), hipHostMallocDefault));
    S_TRY(dev_alloc(s->allocs, &s->dev_pf_emb, (size_t)rows_max * d));
    S_HIP(hipHostMalloc(reinterpret_cast<void **>(&s->result), sizeof(ee_verify_result), hipHostMallocMapped));
    memset(s->result, 0, sizeof(ee_verify_result));
    S_HIP(hipHostGetDevicePointer(reinterpret_cast<void **>(&s->dev_result), s->result, 0));
    S_TRY(dev_alloc(s->allocs, &s->dev_sessdev, EE_MAX_BATCH));
    S_HIP(hipHostMalloc(reinterpret_cast<void **>(&s->host_sessdev), EE_MAX_BATCH * sizeof(SessDev), hipHostMallocDefault));

    Scratch &sc = s->sc;
    const ModelDev &md = m->host_md;
    S_TRY(dev_alloc(s->allocs, &sc.h, (size_t)rows_max * d));
    S_TRY(dev_alloc(s->allocs, &sc.q, (size_t)rows_max * d));
    S_TRY(dev_alloc(s->allocs, &sc.xn, (size_t)2 * rows_max * md.Kpad_d));
    S_TRY(dev_alloc(s->allocs, &sc.xh, (size_t)2 * rows_max * md.Kpad_d));
    S_TRY(dev_alloc(s->allocs, &sc.attn, (size_t)2 * rows_max * md.Kpad_d));
    S_TRY(dev_alloc(s->allocs, &sc.u, (size_t)2 * rows_max * md.Kpad_F));
    S_TRY(dev_alloc(s->allocs, &sc.xa, (size_t)2 * rows_max * md.Kpad_d));
    S_TRY(dev_alloc(s->allocs, &sc.t, (size_t)2 * rows_max * std::max(md.Kpad_A, 32)));
    S_TRY(dev_alloc(s->allocs, &sc.ss_h, (size_t)m->nwg * rows_max));
    S_TRY(dev_alloc(s->allocs, &sc.ss_a, (size_t)m->nwg * rows_max));
    S_TRY(dev_alloc(s->allocs, &sc.ss_f, (size_t)m->nwg * rows_max));
    {
        // items = units * splits; splits are chosen per pass and clamped to this room.  Units: a
        // batch of sessions with one chunk of rows each, or one session with the rows of a prefill chunk.
        const size_t max_units = (size_t)c.n_heads * std::max<size_t>(EE_MAX_BATCH, (rows_max + ATT_ROWS - 1) / ATT_ROWS);
        const size_t forced = ((size_t)s->n_pages + ATT_TILES * WAVES - 1) / (ATT_TILES * WAVES);
        const size_t max_items = max_units * std::max<size_t>(forced, 2) + (size_t)m->nwg;
        s->att_items_cap = (int)max_items;
        S_TRY(dev_alloc(s->allocs, &sc.att_part, max_items * ATT_ROWS * (c.head_dim + 2)));
        S_TRY(dev_alloc(s->allocs, &sc.att_count, max_units));
        S_TRY(dev_alloc(s->allocs, &sc.head_count, 1));
    }
    if (flags & (EE_KEEP_LOGITS | EE_SAMPLING))
        S_TRY(dev_alloc(s->allocs, &sc.logits, (size_t)(EE_MAX_EXITS + 1) * rows_max * c.vocab));
    if (flags & EE_SAMPLING) {
        // room for the draft distributions of every row a pass led by this session can carry
        const size_t n = (size_t)rows_max * c.vocab + (size_t)EE_MAX_BATCH * (2 * EE_MAX_M + 2);
        S_HIP(hipHostMalloc(reinterpret_cast<void **>(&s->host_sample), n * sizeof(float), hipHostMallocDefault));
        S_TRY(dev_alloc(s->allocs, &s->dev_sample, n));
        S_TRY(dev_alloc(s->allocs, &s->dev_sample_out, 2 * EE_MAX_ROWS + 1));
    }
    {
        // partial tiles of the K-split launches: [split][n-tile][row][16] floats for the largest split kind
        size_t part = 0;
        for (int k = 0; k < G_KINDS; ++k)
            if (m->plan[1][k].nwg > 0) part = std::max(part, ((size_t)m->plan[1][k].NT << m->plan[1][k].ksl) * rows_max * 16);
        if (part) {
            S_TRY(dev_alloc(s->allocs, &sc.part, part));
            S_TRY(dev_alloc(s->allocs, &sc.part_count, (size_t)m->nwg));
        }
    }
    S_TRY(dev_alloc(s->allocs, &sc.cand, (size_t)m->nwg * rows_max));
    S_TRY(dev_alloc(s->allocs, &sc.cand_sum, (size_t)m->nwg * rows_max));
    S_HIP(hipDeviceSynchronize());
#undef S_TRY
#undef S_HIP
    *out = s;
    return EE_OK;
}

// map logical pages so that positions [0, upto) are backed; upload new entries
static int ensure_pages(ee_session *s, int upto, hipStream_t stream)
{
    int need = (upto + KV_PAGE - 1) / KV_PAGE;
    if (need > s->n_pages) return fail(EE_ECAPACITY, "KV cache: %d positions exceed max_ctx %d", upto, s->max_ctx);
    int first_new = s->pages_used;
    while (s->pages_used < need) {
        if (s->free_pages.empty()) return fail(EE_ECAPACITY, "KV cache: out of pages");
        s->host_page_table[s->pages_used++] = s->free_pages.back();
        s->free_pages.pop_back();
    }
    if (s->pages_used > first_new)
        HIP_TRY(hipMemcpyAsync(s->dev_page_table + first_new, s->host_page_table + first_new,
                               (size_t)(s->pages_used - first_new) * sizeof(int), hipMemcpyHostToDevice, stream));
    return EE_OK;
}

static void release_pages(ee_session *s, int keep_positions)
{
    int keep = (keep_positions + KV_PAGE - 1) / KV_PAGE;
    while (s->pages_used > keep) s->free_pages.push_back(s->host_page_table[--s->pages_used]);
}

static void fill_sessdev(SessDev &sd, const ee_session *s)
{
    sd.state = s->dev_state;
    sd.page_table = s->dev_page_table;
    sd.kpool = s->kpool;
    sd.vpool = s->vpool;
    sd.rope = s->rope;
    sd.drafts = s->dev_drafts;
    sd.result = s->dev_result;
    sd.n_pages = s->n_pages;
    sd.kv_len = s->kv_len;
    sd.pending = s->pending;
    // the common case: the session's pages are consecutive (a fresh pool hands them out in
    // ascending order and a rollback returns them in the order that restores it)
    sd.contig_base = s->pages_used > 0 ? s->host_page_table[0] : 0;
    for (int i = 1; i < s->pages_used; ++i)
        if (s->host_page_table[i] != s->host_page_table[0] + i) {
            sd.contig_base = -1;
            break;
        }
}

// host mirror of the kernels' stage list: [EMBED] { QKV ATT O GU DN } x layers [AD AU] [HEAD];
// returns the stage's EE_LAUNCH_* code (for a GEMM stage: its GemmKind), or -1 past the end
static int launch_code(const PassArgs &a, int ph)
{
    const int per_layer = 5;
    int idx = ph - (a.do_embed ? 1 : 0);
    if (idx < 0) return EE_LAUNCH_EMBED;
    const int nl = a.layer_end - a.layer_begin;
    if (idx < per_layer * nl) {
        const int r = idx % per_layer;
        if (r == 0) return EE_LAUNCH_QKV;
        if (r == 1) return EE_LAUNCH_ATT;
        return EE_LAUNCH_O + (r - 2);
    }
    idx -= per_layer * nl;
    if (a.head_kind != HEAD_NONE) {
        const int n_ad = a.adapter ? 2 : 0;
        if (idx < n_ad) return EE_LAUNCH_ADAPTER_DOWN + idx;
        if (idx == n_ad && a.head_stage) return EE_LAUNCH_HEAD;
    }
    return -1;
}

// Enqueues the stages of one segment, one launch each, on the leader's stream.
static int launch_segment(ee_session *lead, PassArgs &a, int adapter_slot)
{
    const ee_model *m = lead->m;
    const int per_layer = 5;
    const int rows = a.rows;
    for (int ph = 0;; ++ph) {
        const int code = launch_code(a, ph);
        if (code < 0) break;
        const bool gemm = code != EE_LAUNCH_EMBED && code != EE_LAUNCH_ATT;
        a.stage = ph;
        a.fuse_accept = (code == EE_LAUNCH_HEAD && !a.sm.on) ? 1 : 0;
        a.rows = code == EE_LAUNCH_HEAD ? a.head_rows : rows;   // the head launch carries the rows of all exits of its group
        pass_kernel_t k = gemm ? gemm_kernel(a.rows) : (code == EE_LAUNCH_ATT ? att_kernel(m->cfg.head_dim) : ee_misc_kernel);
        if (gemm) {  // the stage's plan, LDS map and weights travel with the launch
            static_assert(EE_LAUNCH_QKV == G_QKV && EE_LAUNCH_HEAD == G_HEAD && EE_LAUNCH_ADAPTER_DOWN == G_AD && EE_LAUNCH_ADAPTER_UP == G_AU,
                          "launch codes of GEMM stages are their GemmKind");
            const int idx = ph - (a.do_embed ? 1 : 0);
            const int slice = code == EE_LAUNCH_HEAD ? 0 : (code >= EE_LAUNCH_ADAPTER_DOWN ? adapter_slot : a.layer_begin + idx / per_layer);
            // more than 16 rows: the K-split variant of the kind, where the model has one and the scratch its buffers
            const int v = (a.rows > 16 && m->plan[1][code].nwg > 0 && a.sc.part) ? 1 : 0;
            a.plan0 = m->plan[v][code];
            a.W0 = m->w[v][code] + (size_t)slice * m->wstride[v][code];
            if (!plan_lds(a.plan0, a.rows, m->lds_budget, a.lay)) return fail(EE_EDEVICE, "no LDS layout for %d rows", a.rows);
        }
        const bool timed = (lead->flags & EE_TIME_LAUNCHES) && a.mode == 0;
        if (timed) {
            const size_t i = lead->lt_codes.size();
            while (lead->lt_events.size() < 2 * (i + 1)) {
                hipEvent_t ev;
                HIP_TRY(hipEventCreate(&ev));
                lead->lt_events.push_back(ev);
            }
            lead->lt_codes.push_back(code);
            HIP_TRY(hipEventRecord(lead->lt_events[2 * i], lead->run_stream));
        }
        hipLaunchKernelGGL(k, dim3(m->nwg), dim3(WG_THREADS), m->lds_budget, lead->run_stream, a);
        HIP_TRY(hipGetLastError());
        if (timed) HIP_TRY(hipEventRecord(lead->lt_events[2 * lead->lt_codes.size() - 1], lead->run_stream));
        if (code == EE_LAUNCH_HEAD && a.sm.on) {
            // probabilistic verification: the rows' keep tests and draws, one workgroup per head row,
            // then the accept rule and the publication (in the workgroup that finishes last)
            if (timed) {
                const size_t i = lead->lt_codes.size();
                while (lead->lt_events.size() < 2 * (i + 1)) {
                    hipEvent_t ev;
                    HIP_TRY(hipEventCreate(&ev));
                    lead->lt_events.push_back(ev);
                }
                lead->lt_codes.push_back(EE_LAUNCH_SAMPLE);
                HIP_TRY(hipEventRecord(lead->lt_events[2 * i], lead->run_stream));
            }
            hipLaunchKernelGGL(ee_sample_kernel, dim3(a.head_rows), dim3(WG_THREADS), SAMPLE_LDS_BYTES, lead->run_stream, a);
            HIP_TRY(hipGetLastError());
            if (timed) HIP_TRY(hipEventRecord(lead->lt_events[2 * lead->lt_codes.size() - 1], lead->run_stream));
        }
    }
    a.rows = rows;
    return EE_OK;
}

static void base_args(const ee_session *lead, PassArgs &a)
{
    memset(&a, 0, sizeof a);
    a.mdv = lead->m->host_md;
    a.sc = lead->sc;
    a.nwg = lead->m->nwg;
    a.H = lead->m->host_md.H;
    a.d = lead->m->host_md.d;
    a.Kpad_d = lead->m->host_md.Kpad_d;
    a.att_scale = lead->m->host_md.att_scale;
    a.keep_logits = (lead->flags & EE_KEEP_LOGITS) ? 1 : 0;
}

static int finish_flight(ee_session *s)
{
    if (!s->in_flight) return EE_OK;
    ee_session *lead = s->leader;
    HIP_TRY(hipEventSynchronize(lead->ev_final));
    s->in_flight = false;
    if (s->result->device_status != 0) return fail(EE_EDEVICE, "a device-side wait gave up during the pass; results are invalid");
    if (!(s->flags & EE_NO_AUTOCOMMIT)) {
        s->kv_len += s->result->accept_len + 1;
        s->pending = s->result->next_token;
    }
    return EE_OK;
}

// ------------------------------------------------------------------ prefill

static int set_device_state(ee_session *s, bool set_kv, bool set_pending)
{
    hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(64), 0, s->stream, s->dev_state, s->kv_len, s->pending,
                       set_kv ? 1 : 0, set_pending ? 1 : 0);
    HIP_TRY(hipGetLastError());
    return EE_OK;
}

extern "C" int ee_prefill_embeds(ee_session *s, const uint16_t *emb_bf16, int n_emb, const int32_t *tokens, int n,
                                 unsigned flags, int32_t *first_token)
{
    if (!s) return fail(EE_EINVAL, "ee_prefill: null session");
    if (n_emb < 0 || n < 0 || (n_emb > 0 && !emb_bf16) || (n > 0 && !tokens)) return fail(EE_EINVAL, "ee_prefill: bad arguments");
    const ee_model *m = s->m;
    const ee_model_config &c = m->cfg;
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= c.vocab) return fail(EE_EINVAL, "ee_prefill: token %d at %d outside [0,%d)", tokens[i], i, c.vocab);
    const bool hold = (flags & EE_HOLD_LAST) != 0;
    if (hold && n < 1) return fail(EE_EINVAL, "ee_prefill: EE_HOLD_LAST needs at least one token");
    const int total = n_emb + n - (hold ? 1 : 0);
    if (!hold && total < 1) return fail(EE_EINVAL, "ee_prefill: empty prompt");
    if (total + 1 > s->max_ctx) return fail(EE_ECAPACITY, "ee_prefill: %d rows do not fit max_ctx %d", total, s->max_ctx);
    HIP_TRY(hipSetDevice(m->device));
    int rc = finish_flight(s);
    if (rc != EE_OK && rc != EE_EDEVICE) return rc;
    HIP_TRY(hipStreamSynchronize(s->stream));
    // reset
    s->run_stream = s->stream;
    release_pages(s, 0);
    // all pages are free here: hand them out in ascending order (a fresh session's pages are then
    // consecutive and the kernels skip the table lookup) or, as a test aid, in descending order
    std::sort(s->free_pages.begin(), s->free_pages.end());
    if (!s->scatter_pages) std::reverse(s->free_pages.begin(), s->free_pages.end());
    s->kv_len = 0;
    s->has_pending = false;
    s->leader = s;
    s->flight_gamma = 0;
    s->flight_exits = 0;
    s->result->device_status = 0;
    if ((rc = ensure_pages(s, total + 1, s->stream)) != EE_OK) return rc;

    fill_sessdev(s->host_sessdev[0], s);
    HIP_TRY(hipMemcpyAsync(s->dev_sessdev, s->host_sessdev, sizeof(SessDev), hipMemcpyHostToDevice, s->stream));
    const int chunk = c.max_rows;
    const size_t d = (size_t)c.d_model;
    for (int start = 0; start < total; start += chunk) {
        const int rows = std::min(chunk, total - start);
        HIP_TRY(hipStreamSynchronize(s->stream));  // staging buffers are reused
        for (int i = 0; i < rows; ++i) {
            int r = start + i;
            s->host_pf_tokens[i] = r < n_emb ? -1 : tokens[r - n_emb];
        }
        HIP_TRY(hipMemcpyAsync(s->dev_pf_tokens, s->host_pf_tokens, (size_t)rows * sizeof(int), hipMemcpyHostToDevice, s->stream));
        if (start < n_emb) {
            int ne = std::min(rows, n_emb - start);
            HIP_TRY(hipMemcpyAsync(s->dev_pf_emb, emb_bf16 + (size_t)start * d, (size_t)ne * d * 2, hipMemcpyHostToDevice, s->stream));
        }
        const bool last = (start + rows == total) && !hold;
        PassArgs a;
        base_args(s, a);
        a.n_sess = 1;
        a.M = rows;
        a.rows = rows;
        a.mode = 1;
        a.pf_tokens = s->dev_pf_tokens;
        a.pf_emb = s->dev_pf_emb;
        a.pf_pos0 = start;
        a.layer_begin = 0;
        a.layer_end = c.n_layers;
        a.do_embed = 1;
        a.head_kind = last ? HEAD_PREFILL : HEAD_NONE;
        a.head_idx = 0;
        a.head_gain = m->host_md.g_final;
        a.n_heads = 1;
        a.head_rows = rows;
        a.head_row0 = 0;
        a.head_stage = 1;
        a.att_splits = attention_splits(s, s->att_items_cap, 1, rows, start + rows);
        if (a.att_splits == 0) return fail(EE_ECAPACITY, "ee_prefill: context too long for the session's attention scratch");
        a.sess = s->dev_sessdev;
        a.sess0 = s->host_sessdev[0];
        if ((rc = launch_segment(s, a, 0)) != EE_OK) return rc;
    }
    HIP_TRY(hipStreamSynchronize(s->stream));
    s->kv_len = total;
    if (hold) {
        s->pending = tokens[n - 1];
    } else {
        if (s->result->device_status != 0) return fail(EE_EDEVICE, "a device-side wait gave up during prefill");
        s->pending = s->result->next_token;
        if (first_token) *first_token = s->pending;
    }
    s->has_pending = true;
    if ((rc = set_device_state(s, true, true)) != EE_OK) return rc;
    HIP_TRY(hipStreamSynchronize(s->stream));
    return EE_OK;
}

extern "C" int ee_prefill(ee_session *s, const int32_t *tokens, int n, unsigned flags, int32_t *first_token)
{
    return ee_prefill_embeds(s, nullptr, 0, tokens, n, flags, first_token);
}

// ------------------------------------------------------------------ verify

static int check_exits(const ee_model *m, const int32_t *exit_layers, int n_exits, const float **gains, int *slots)
{
    if (n_exits < 0 || n_exits > EE_MAX_EXITS || (n_exits > 0 && !exit_layers))
        return fail(EE_EINVAL, "ee_verify: n_exits %d not in [0,%d]", n_exits, EE_MAX_EXITS);
    for (int e = 0; e < n_exits; ++e) {
        if (exit_layers[e] < 1 || exit_layers[e] > m->cfg.n_layers - 1)
            return fail(EE_EINVAL, "ee_verify: exit layer %d not in [1,%d]", exit_layers[e], m->cfg.n_layers - 1);
        if (e > 0 && exit_layers[e] <= exit_layers[e - 1]) return fail(EE_EINVAL, "ee_verify: exit layers must increase strictly");
        gains[e] = nullptr;
        for (int i = 0; i < m->cfg.n_exits; ++i)
            if (m->cfg.exit_layers[i] == exit_layers[e]) {
                gains[e] = m->g_exit[i];
                slots[e] = i;
            }
        if (!gains[e]) return fail(EE_EINVAL, "ee_verify: the model stores no exit gain for layer %d", exit_layers[e]);
    }
    return EE_OK;
}

// ------------------------------------------------------------------ static scratch (ee_verify_static)

// Scratch of one single-session pass for callers that must not allocate.  One copy per GPU the
// library is loaded on, held until the process ends.  In host code the array's name is only a
// handle: its device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[EE_STATIC_SCRATCH_BYTES];

constexpr int EE_MAX_DEVICES = 64;
static void *g_scratch_ptr[EE_MAX_DEVICES];   // per device: address of that GPU's copy of `scratch`

static int static_scratch_ptr(int device, unsigned char **out)
{
    if (device < 0 || device >= EE_MAX_DEVICES) return fail(EE_EINVAL, "device %d: at most %d devices", device, EE_MAX_DEVICES);
    if (!g_scratch_ptr[device]) {   // the model's device is current here
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[device] = p;
    }
    *out = static_cast<unsigned char *>(g_scratch_ptr[device]);
    return EE_OK;
}

// fills n 16-byte words with zeros (a kernel, not hipMemsetAsync: callers may be capturing a graph)
__global__ void __launch_bounds__(256) ee_zero_kernel(uint4 *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// Lays the pass's scratch buffers out in the static array (sizes for M rows of this model),
// points a.sc at them, picks the attention splits for that room and enqueues the clearing of
// the part in use: the array keeps the last call's contents, and the padding columns of the GEMM
// inputs and the attention / head counters must start at zero.
static int use_static_scratch(ee_session *lead, PassArgs &a, int M, int n_pos_max)
{
    const ee_model *m = lead->m;
    const ModelDev &md = m->host_md;
    unsigned char *base = nullptr;
    int rc = static_scratch_ptr(m->device, &base);
    if (rc != EE_OK) return rc;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        unsigned char *p = base + off;
        off += align_up(std::max<size_t>(bytes, 16), 256);
        return p;
    };
    const size_t rows = (size_t)M, d = (size_t)md.d;
    Scratch sc;
    memset(&sc, 0, sizeof sc);
    sc.h = reinterpret_cast<float *>(take(rows * d * 4));
    sc.q = reinterpret_cast<float *>(take(rows * d * 4));
    sc.xn = reinterpret_cast<uint16_t *>(take(2 * rows * md.Kpad_d * 2));
    sc.xh = reinterpret_cast<uint16_t *>(take(2 * rows * md.Kpad_d * 2));
    sc.attn = reinterpret_cast<uint16_t *>(take(2 * rows * md.Kpad_d * 2));
    sc.u = reinterpret_cast<uint16_t *>(take(2 * rows * md.Kpad_F * 2));
    sc.xa = reinterpret_cast<uint16_t *>(take(2 * rows * md.Kpad_d * 2));
    sc.t = reinterpret_cast<uint16_t *>(take(2 * rows * std::max(md.Kpad_A, 32) * 2));
    sc.ss_h = reinterpret_cast<float *>(take((size_t)m->nwg * md.rows_max * 4));
    sc.ss_a = reinterpret_cast<float *>(take((size_t)m->nwg * md.rows_max * 4));
    sc.ss_f = reinterpret_cast<float *>(take((size_t)m->nwg * md.rows_max * 4));
    sc.cand = reinterpret_cast<int2 *>(take((size_t)m->nwg * md.rows_max * 8));
    sc.cand_sum = reinterpret_cast<float *>(take((size_t)m->nwg * md.rows_max * 4));
    sc.att_count = reinterpret_cast<int *>(take((size_t)md.H * 4));
    sc.head_count = reinterpret_cast<int *>(take(4));
    sc.logits = lead->sc.logits;   // kept logits are an output of the session, not scratch
    // attention partials: what is left, at most one item per compute unit and split
    const size_t item_bytes = (size_t)ATT_ROWS * (md.hd + 2) * 4;
    if (off + (size_t)md.H * item_bytes > EE_STATIC_SCRATCH_BYTES)
        return fail(EE_ECAPACITY, "ee_verify_static: %d rows of this model need more than the %d bytes of static scratch", M, EE_STATIC_SCRATCH_BYTES);
    const int items_cap = (int)std::min<size_t>((EE_STATIC_SCRATCH_BYTES - off) / item_bytes, (size_t)md.H * ATT_MAX_SPLITS);
    a.att_splits = attention_splits(lead, items_cap, 1, M, n_pos_max);
    if (a.att_splits == 0)
        return fail(EE_ECAPACITY, "ee_verify_static: a context of %d positions needs more than the %d bytes of static scratch", n_pos_max, EE_STATIC_SCRATCH_BYTES);
    sc.att_part = reinterpret_cast<float *>(take((size_t)md.H * a.att_splits * item_bytes));
    a.sc = sc;
    hipLaunchKernelGGL(ee_zero_kernel, dim3(256), dim3(256), 0, lead->run_stream, reinterpret_cast<uint4 *>(base), off / 16);
    HIP_TRY(hipGetLastError());
    return EE_OK;
}

// One pass for all sessions of the call: rows = n_sessions * (gamma + 1) share one stream of the
// weights; the first session leads (its stream, events and scratch carry the pass).
// static_scratch: run the pass on the library's static scratch array instead of the leader's own
// buffers (ee_verify_static); nothing on this path allocates.
static int verify_impl(ee_session *const *sessions, int n_sessions, const int32_t *const *drafts, int gamma,
                       const int32_t *exit_layers, int n_exits, const ee_verify_result **outs, bool static_scratch,
                       const ee_sampling *sp = nullptr)
{
    if (!sessions || !drafts || n_sessions < 1 || n_sessions > EE_MAX_BATCH)
        return fail(EE_EINVAL, "ee_verify: n_sessions %d not in [1,%d]", n_sessions, EE_MAX_BATCH);
    for (int i = 0; i < n_sessions; ++i)
        if (!sessions[i] || !drafts[i]) return fail(EE_EINVAL, "ee_verify: null session or drafts");
    ee_session *lead = sessions[0];
    const ee_model *m = lead->m;
    const ee_model_config &c = m->cfg;
    const int M = gamma + 1;
    if (gamma < 1) return fail(EE_EINVAL, "ee_verify: gamma %d < 1", gamma);
    for (int i = 0; i < n_sessions; ++i) {
        ee_session *s = sessions[i];
        if (s->m != m) return fail(EE_EINVAL, "ee_verify_batch: sessions of different models");
        if (gamma > s->max_gamma) return fail(EE_EINVAL, "ee_verify: gamma %d exceeds the session's max_gamma %d", gamma, s->max_gamma);
        for (int j = 0; j < i; ++j)
            if (sessions[j] == s) return fail(EE_EINVAL, "ee_verify_batch: session listed twice");
        for (int j = 0; j < gamma; ++j)
            if (drafts[i][j] < 0 || drafts[i][j] >= c.vocab)
                return fail(EE_EINVAL, "ee_verify: draft token %d outside [0,%d)", drafts[i][j], c.vocab);
        if (((s->flags ^ lead->flags) & EE_NO_AUTOCOMMIT) != 0)
            return fail(EE_EINVAL, "ee_verify_batch: sessions mix EE_NO_AUTOCOMMIT settings");
    }
    if (n_sessions * M > c.max_rows) return fail(EE_EINVAL, "ee_verify: %d rows exceed the model's max_rows %d", n_sessions * M, c.max_rows);
    if (sp) {   // sp[b]: session b's draft distributions and uniform numbers
        if (static_scratch) return fail(EE_EINVAL, "ee_verify_sampled: not with the static scratch");
        for (int b = 0; b < n_sessions; ++b) {
            const ee_sampling &q = sp[b];
            if (!(sessions[b]->flags & EE_SAMPLING)) return fail(EE_ESTATE, "ee_verify_sampled: session %d was created without EE_SAMPLING", b);
            if (!q.draft_probs || !q.u || !q.v) return fail(EE_EINVAL, "ee_verify_sampled: null draft_probs, u or v");
            if (!(q.temperature > 0.f) || !std::isfinite(q.temperature)) return fail(EE_EINVAL, "ee_verify_sampled: temperature must be positive");
            for (int i = 0; i < gamma; ++i)
                if (!(q.u[i] >= 0.f && q.u[i] < 1.f)) return fail(EE_EINVAL, "ee_verify_sampled: u[%d] not in [0,1)", i);
            for (int i = 0; i <= gamma; ++i)
                if (!(q.v[i] >= 0.f && q.v[i] < 1.f)) return fail(EE_EINVAL, "ee_verify_sampled: v[%d] not in [0,1)", i);
            for (int i = 0; i < gamma; ++i) {   // the drafts' own probabilities; the full rows are the caller's responsibility
                const float px = q.draft_probs[(size_t)i * c.vocab + drafts[b][i]];
                if (!(px >= 0.f && px <= 1.f)) return fail(EE_EINVAL, "ee_verify_sampled: draft_probs[%d][draft] = %g is not a probability", i, (double)px);
            }
        }
    }
    const float *gains[EE_MAX_EXITS];
    int slots[EE_MAX_EXITS];
    int rc = check_exits(m, exit_layers, n_exits, gains, slots);
    if (rc != EE_OK) return rc;
    HIP_TRY(hipSetDevice(m->device));
    int n_pos_max = 0;
    for (int i = 0; i < n_sessions; ++i) {
        ee_session *s = sessions[i];
        if ((rc = finish_flight(s)) != EE_OK) return rc;
        if (!s->has_pending) return fail(EE_ESTATE, "ee_verify: session has no pending token (call ee_prefill first)");
        if (s->kv_len + M > s->max_ctx) return fail(EE_ECAPACITY, "ee_verify: kv_len %d + %d rows exceed max_ctx %d", s->kv_len, M, s->max_ctx);
        n_pos_max = std::max(n_pos_max, s->kv_len + M);
    }
    PassArgs a;
    base_args(lead, a);
    lead->run_stream = lead->stream;
    if (static_scratch) {
        if ((rc = use_static_scratch(lead, a, M, n_pos_max)) != EE_OK) return rc;
    } else {
        a.att_splits = attention_splits(lead, lead->att_items_cap, n_sessions, M, n_pos_max);
        if (a.att_splits == 0)
            return fail(EE_ECAPACITY, "ee_verify_batch: a context of %d positions needs more attention scratch than the first session holds "
                                      "(list the session with the largest max_ctx first)", n_pos_max);
    }
    // everything below is enqueued on the leader's stream; other sessions' own
    // streams are idle here (their last pass has been waited for)
    for (int i = 0; i < n_sessions; ++i) {
        ee_session *s = sessions[i];
        if (s != lead) HIP_TRY(hipStreamSynchronize(s->stream));
        if ((rc = ensure_pages(s, s->kv_len + M, lead->run_stream)) != EE_OK) return rc;
        memcpy(s->host_drafts, drafts[i], (size_t)gamma * sizeof(int));
        HIP_TRY(hipMemcpyAsync(s->dev_drafts, s->host_drafts, (size_t)gamma * sizeof(int), hipMemcpyHostToDevice, lead->run_stream));
        s->result->gamma = gamma;
        s->result->n_exits = n_exits;
        s->result->device_status = 0;
    }
    a.n_sess = n_sessions;
    a.M = M;
    a.rows = n_sessions * M;
    a.mode = 0;
    a.commit = (lead->flags & EE_NO_AUTOCOMMIT) ? 0 : 1;
    if (sp) {
        // [session][gamma][V] distributions, then per session u, v and 1 / temperature (SampleDev)
        const size_t V = (size_t)c.vocab, np = (size_t)n_sessions * gamma * V, blk = 2 * (size_t)gamma + 2;
        for (int b = 0; b < n_sessions; ++b) {
            memcpy(lead->host_sample + (size_t)b * gamma * V, sp[b].draft_probs, (size_t)gamma * V * sizeof(float));
            float *uv = lead->host_sample + np + (size_t)b * blk;
            memcpy(uv, sp[b].u, (size_t)gamma * sizeof(float));
            memcpy(uv + gamma, sp[b].v, (size_t)(gamma + 1) * sizeof(float));
            uv[2 * gamma + 1] = 1.0f / sp[b].temperature;
        }
        HIP_TRY(hipMemcpyAsync(lead->dev_sample, lead->host_sample, (np + (size_t)n_sessions * blk) * sizeof(float), hipMemcpyHostToDevice, lead->run_stream));
        a.sm.probs = lead->dev_sample;
        a.sm.uv = lead->dev_sample + np;
        a.sm.on = 1;
        a.sm.tok = lead->dev_sample_out;
        a.sm.kept = lead->dev_sample_out + EE_MAX_ROWS;
        a.sm.count = lead->dev_sample_out + 2 * EE_MAX_ROWS;
        a.keep_logits = 1;   // the sampling launch reads the head launch's logits
    }
    for (int i = 0; i < n_sessions; ++i) fill_sessdev(lead->host_sessdev[i], sessions[i]);
    HIP_TRY(hipMemcpyAsync(lead->dev_sessdev, lead->host_sessdev, (size_t)n_sessions * sizeof(SessDev),
                           hipMemcpyHostToDevice, lead->run_stream));
    a.sess = lead->dev_sessdev;
    a.sess0 = lead->host_sessdev[0];

    HIP_TRY(hipEventRecord(lead->ev_start, lead->run_stream));
    lead->lt_codes.clear();
    // Exit heads run in groups of up to head_batch consecutive exits: every exit deposits its
    // LM-head input rows when its layer is done, and the last one of the group runs the LM head
    // over the rows of all of them (one stream of W_lm per group), after which the group's results
    // are published together.  head_batch = 1: every exit is published right after its layer.
    const int per_group = std::max(1, std::min(lead->head_batch, c.max_rows / a.rows));
    int layer = 0;
    for (int e = 0; e <= n_exits; ++e) {
        const bool fin = (e == n_exits);
        const int g_first = fin ? e : e / per_group * per_group;             // first exit of e's group
        const int g_size = fin ? 1 : std::min(per_group, n_exits - g_first);
        a.layer_begin = layer;
        a.layer_end = fin ? c.n_layers : exit_layers[e];
        a.do_embed = (e == 0) ? 1 : 0;
        a.head_kind = fin ? HEAD_FINAL : HEAD_EXIT;
        a.head_idx = g_first;
        a.head_gain = fin ? m->host_md.g_final : gains[e];
        a.n_heads = g_size;
        a.head_rows = g_size * a.rows;
        a.head_row0 = (e - g_first) * a.rows;
        a.head_stage = (e - g_first == g_size - 1) ? 1 : 0;
        a.adapter = (!fin && m->host_md.A > 0) ? 1 : 0;
        a.ad_bdown = a.adapter ? m->ad_bdown[slots[e]] : nullptr;
        a.ad_bup = a.adapter ? m->ad_bup[slots[e]] : nullptr;
        if ((rc = launch_segment(lead, a, fin ? 0 : slots[e])) != EE_OK) return rc;
        if (fin) {
            HIP_TRY(hipEventRecord(lead->ev_final, lead->run_stream));
        } else if (a.head_stage) {
            for (int j = g_first; j <= e; ++j) HIP_TRY(hipEventRecord(lead->ev_exit[j], lead->run_stream));
        }
        layer = a.layer_end;
    }
    for (int i = 0; i < n_sessions; ++i) {
        ee_session *s = sessions[i];
        s->in_flight = true;
        s->leader = lead;
        s->flight_gamma = gamma;
        s->flight_exits = n_exits;
        s->flight_row0 = i * M;
        s->popped_mask = 0;
        if (outs) outs[i] = s->result;
    }
    return EE_OK;
}

extern "C" int ee_verify_batch(ee_session *const *sessions, int n_sessions, const int32_t *const *drafts, int gamma,
                               const int32_t *exit_layers, int n_exits, const ee_verify_result **outs)
{
    return verify_impl(sessions, n_sessions, drafts, gamma, exit_layers, n_exits, outs, false);
}

extern "C" int ee_verify(ee_session *s, const int32_t *draft_tokens, int gamma, const int32_t *exit_layers, int n_exits,
                         const ee_verify_result **out)
{
    if (!s) return fail(EE_EINVAL, "ee_verify: null session");
    ee_session *ss[1] = {s};
    const int32_t *dd[1] = {draft_tokens};
    const ee_verify_result *oo[1] = {nullptr};
    int rc = verify_impl(ss, 1, dd, gamma, exit_layers, n_exits, oo, false);
    if (rc == EE_OK && out) *out = oo[0];
    return rc;
}

extern "C" int ee_verify_sampled(ee_session *s, const int32_t *draft_tokens, int gamma, const int32_t *exit_layers, int n_exits,
                                 const ee_sampling *sampling, const ee_verify_result **out)
{
    if (!s) return fail(EE_EINVAL, "ee_verify_sampled: null session");
    if (!sampling) return fail(EE_EINVAL, "ee_verify_sampled: null sampling arguments");
    ee_session *ss[1] = {s};
    const int32_t *dd[1] = {draft_tokens};
    const ee_verify_result *oo[1] = {nullptr};
    int rc = verify_impl(ss, 1, dd, gamma, exit_layers, n_exits, oo, false, sampling);
    if (rc == EE_OK && out) *out = oo[0];
    return rc;
}

extern "C" int ee_verify_sampled_batch(ee_session *const *sessions, int n_sessions, const int32_t *const *drafts, int gamma,
                                       const int32_t *exit_layers, int n_exits, const ee_sampling *samplings,
                                       const ee_verify_result **outs)
{
    if (!samplings) return fail(EE_EINVAL, "ee_verify_sampled_batch: null sampling arguments");
    return verify_impl(sessions, n_sessions, drafts, gamma, exit_layers, n_exits, outs, false, samplings);
}

extern "C" int ee_verify_static(ee_session *s, const int32_t *draft_tokens, int gamma, const int32_t *exit_layers, int n_exits,
                                const ee_verify_result **out)
{
    if (!s) return fail(EE_EINVAL, "ee_verify_static: null session");
    if (s->flags & EE_TIME_LAUNCHES) return fail(EE_ESTATE, "ee_verify_static: not for EE_TIME_LAUNCHES sessions (their event pairs are created on demand)");
    ee_session *ss[1] = {s};
    const int32_t *dd[1] = {draft_tokens};
    const ee_verify_result *oo[1] = {nullptr};
    int rc = verify_impl(ss, 1, dd, gamma, exit_layers, n_exits, oo, true);
    if (rc == EE_OK && out) *out = oo[0];
    return rc;
}

// ------------------------------------------------------------------ waiting

static int exit_event(ee_session *s, int exit_idx, hipEvent_t *ev)
{
    if (!s) return fail(EE_EINVAL, "null session");
    if (s->flight_exits < 0 || exit_idx < 0 || exit_idx >= s->flight_exits)
        return fail(EE_EINVAL, "exit index %d not in [0,%d)", exit_idx, s->flight_exits);
    *ev = s->leader->ev_exit[exit_idx];
    return EE_OK;
}

extern "C" int ee_wait_exit(ee_session *s, int exit_idx)
{
    hipEvent_t ev;
    int rc = exit_event(s, exit_idx, &ev);
    if (rc != EE_OK) return rc;
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_wait_exit: no verify pass was enqueued");
    HIP_TRY(hipEventSynchronize(ev));
    return EE_OK;
}

extern "C" int ee_query_exit(ee_session *s, int exit_idx)
{
    hipEvent_t ev;
    int rc = exit_event(s, exit_idx, &ev);
    if (rc != EE_OK) return rc;
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_query_exit: no verify pass was enqueued");
    hipError_t e = hipEventQuery(ev);
    if (e == hipSuccess) return EE_OK;
    if (e == hipErrorNotReady) return EE_NOT_READY;
    return fail(EE_EDEVICE, "hipEventQuery: %s", hipGetErrorString(e));
}

extern "C" int ee_wait_final(ee_session *s)
{
    if (!s) return fail(EE_EINVAL, "null session");
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_wait_final: no verify pass was enqueued");
    return finish_flight(s);
}

extern "C" int ee_query_final(ee_session *s)
{
    if (!s) return fail(EE_EINVAL, "null session");
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_query_final: no verify pass was enqueued");
    if (!s->in_flight) return EE_OK;
    hipError_t e = hipEventQuery(s->leader->ev_final);
    if (e == hipSuccess) return EE_OK;
    if (e == hipErrorNotReady) return EE_NOT_READY;
    return fail(EE_EDEVICE, "hipEventQuery: %s", hipGetErrorString(e));
}

// ------------------------------------------------------------------ sender queue, latency model

// s^(e) of Alg. 2: the largest confidence among the rows the exit's result consists of
static float exit_score(const ee_verify_result *r, int e)
{
    float sc = 0.f;
    for (int i = 0; i <= r->exit_accept_len[e] && i < EE_MAX_M; ++i) sc = std::max(sc, r->exit_conf[e][i]);
    return sc;
}

extern "C" int ee_exit_pop(ee_session *s, int wait, int *exit_idx, float *score)
{
    if (!s || !exit_idx) return fail(EE_EINVAL, "null argument");
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_exit_pop: no verify pass was enqueued");
    ee_session *lead = s->leader;
    HIP_TRY(hipSetDevice(s->m->device));
    for (;;) {
        if (!s->in_flight || hipEventQuery(lead->ev_final) == hipSuccess) {  // the final result is there: Q_e is reset
            s->popped_mask = ~0ull;
            return EE_DONE;
        }
        int best = -1, first_unpublished = -1;
        float best_sc = -1.f;
        for (int e = 0; e < s->flight_exits; ++e) {
            if (s->popped_mask & (1ull << e)) continue;
            const hipError_t q = hipEventQuery(lead->ev_exit[e]);
            if (q == hipSuccess) {
                const float sc = exit_score(s->result, e);
                if (sc > best_sc) {
                    best_sc = sc;
                    best = e;
                }
            } else if (q == hipErrorNotReady) {
                if (first_unpublished < 0) first_unpublished = e;
            } else {
                return fail(EE_EDEVICE, "hipEventQuery: %s", hipGetErrorString(q));
            }
        }
        if (best >= 0) {
            s->popped_mask |= 1ull << best;
            *exit_idx = best;
            if (score) *score = best_sc;
            return EE_OK;
        }
        if (first_unpublished < 0) return EE_DONE;
        if (!wait) return EE_NOT_READY;
        HIP_TRY(hipEventSynchronize(lead->ev_exit[first_unpublished]));
    }
}

extern "C" int ee_exit_order(ee_session *s, int *order, float *scores)
{
    if (!s || !order) return fail(EE_EINVAL, "null argument");
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_exit_order: no verify pass was enqueued");
    int rc = finish_flight(s);
    if (rc != EE_OK) return rc;
    const int n = s->flight_exits;
    float sc[EE_MAX_EXITS];
    for (int e = 0; e < n; ++e) {
        sc[e] = exit_score(s->result, e);
        order[e] = e;
    }
    std::stable_sort(order, order + n, [&](int a, int b) { return sc[a] > sc[b]; });  // ties: the earlier exit first
    if (scores)
        for (int i = 0; i < n; ++i) scores[i] = sc[order[i]];
    return EE_OK;
}

extern "C" int ee_latency_model(const ee_latency_params *p, ee_latency *out)
{
    if (!p || !out) return fail(EE_EINVAL, "null argument");
    if (!(p->tau > 0.0) || !(p->T_q > 0.0) || p->n < 1 || p->gamma < 1 || !(p->r >= 0.0 && p->r <= 1.0) || p->T_p < 0.0 ||
        p->T_c < 0.0 || p->T_r < 0.0)
        return fail(EE_EINVAL, "ee_latency_model: tau, T_q, n > 0, gamma >= 1, 0 <= r <= 1 and non-negative times are required");
    const double n = (double)p->n, g = (double)p->gamma, rounds = n / p->tau;
    out->ar_ms = 2.0 * p->T_c + n * p->T_q;
    out->sd_ms = rounds * (2.0 * p->T_c + g * p->T_p + p->T_q);
    out->fsd_ms = rounds * (2.0 * p->T_c + p->r * g * p->T_p + (1.0 - p->r) * p->T_r + p->T_q);
    out->ar_ms_per_token = out->ar_ms / n;
    out->sd_ms_per_token = out->sd_ms / n;
    out->fsd_ms_per_token = out->fsd_ms / n;
    out->speedup_ar_to_sd = out->ar_ms / out->sd_ms;
    out->speedup_sd_to_fsd = out->sd_ms / out->fsd_ms;
    out->c = p->T_p / p->T_q;
    out->projected_sd_to_fsd = (g * out->c + 1.0) / (p->r * g * out->c + 1.0);
    return EE_OK;
}

extern "C" int ee_pass_time_ms(ee_session *s, int exit_idx, float *ms)
{
    if (!s || !ms) return fail(EE_EINVAL, "null argument");
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_pass_time_ms: no verify pass was enqueued");
    if (s->in_flight) return fail(EE_ESTATE, "ee_pass_time_ms: the pass has not been waited for");
    if (exit_idx < 0 || exit_idx > s->flight_exits) return fail(EE_EINVAL, "exit index %d not in [0,%d]", exit_idx, s->flight_exits);
    ee_session *lead = s->leader;
    hipEvent_t ev = exit_idx == s->flight_exits ? lead->ev_final : lead->ev_exit[exit_idx];
    HIP_TRY(hipEventElapsedTime(ms, lead->ev_start, ev));
    return EE_OK;
}

// ------------------------------------------------------------------ state

extern "C" int ee_kv_truncate(ee_session *s, int new_len)
{
    if (!s) return fail(EE_EINVAL, "null session");
    HIP_TRY(hipSetDevice(s->m->device));
    int rc = finish_flight(s);
    if (rc != EE_OK) return rc;
    if (new_len < 0 || new_len > s->kv_len) return fail(EE_EINVAL, "ee_kv_truncate: %d not in [0, kv_len=%d]", new_len, s->kv_len);
    s->kv_len = new_len;
    release_pages(s, new_len);
    if ((rc = set_device_state(s, true, false)) != EE_OK) return rc;
    HIP_TRY(hipStreamSynchronize(s->stream));
    return EE_OK;
}

extern "C" int ee_set_pending(ee_session *s, int32_t token)
{
    if (!s) return fail(EE_EINVAL, "null session");
    if (token < 0 || token >= s->m->cfg.vocab) return fail(EE_EINVAL, "ee_set_pending: token %d outside [0,%d)", token, s->m->cfg.vocab);
    HIP_TRY(hipSetDevice(s->m->device));
    int rc = finish_flight(s);
    if (rc != EE_OK) return rc;
    s->pending = token;
    s->has_pending = true;
    if ((rc = set_device_state(s, false, true)) != EE_OK) return rc;
    HIP_TRY(hipStreamSynchronize(s->stream));
    return EE_OK;
}

extern "C" int ee_kv_len(ee_session *s, int *out)
{
    if (!s || !out) return fail(EE_EINVAL, "null argument");
    int rc = finish_flight(s);
    if (rc != EE_OK) return rc;
    *out = s->kv_len;
    return EE_OK;
}

extern "C" int ee_pending(ee_session *s, int32_t *out)
{
    if (!s || !out) return fail(EE_EINVAL, "null argument");
    int rc = finish_flight(s);
    if (rc != EE_OK) return rc;
    if (!s->has_pending) return fail(EE_ESTATE, "ee_pending: no pending token");
    *out = s->pending;
    return EE_OK;
}

extern "C" int ee_debug_logits(ee_session *s, int head_idx, float *out)
{
    if (!s || !out) return fail(EE_EINVAL, "null argument");
    if (s->flight_gamma == 0) return fail(EE_ESTATE, "ee_debug_logits: no verify pass was enqueued");
    ee_session *lead = s->leader;
    if (!(lead->flags & EE_KEEP_LOGITS))
        return fail(EE_ESTATE, "ee_debug_logits: the session that led the pass was created without EE_KEEP_LOGITS");
    if (head_idx < 0 || head_idx > s->flight_exits) return fail(EE_EINVAL, "head index %d not in [0,%d]", head_idx, s->flight_exits);
    HIP_TRY(hipSetDevice(s->m->device));
    HIP_TRY(hipEventSynchronize(lead->ev_final));
    const size_t V = (size_t)s->m->cfg.vocab, rows_max = (size_t)s->m->cfg.max_rows;
    const int M = s->flight_gamma + 1;
    HIP_TRY(hipMemcpy(out, lead->sc.logits + ((size_t)head_idx * rows_max + (size_t)s->flight_row0) * V, (size_t)M * V * sizeof(float),
                      hipMemcpyDeviceToHost));
    return EE_OK;
}

extern "C" int ee_session_option(ee_session *s, int option, int value)
{
    if (!s) return fail(EE_EINVAL, "null session");
    int rc = finish_flight(s);
    if (rc != EE_OK) return rc;
    switch (option) {
    case EE_OPT_ATT_SPLITS:
        if (value < 0 || value > ATT_MAX_SPLITS) return fail(EE_EINVAL, "EE_OPT_ATT_SPLITS: %d not in [0,%d]", value, ATT_MAX_SPLITS);
        s->att_splits_opt = value;
        return EE_OK;
    case EE_OPT_HEAD_BATCH:
        if (value < 1 || value > EE_MAX_EXITS) return fail(EE_EINVAL, "EE_OPT_HEAD_BATCH: %d not in [1,%d]", value, EE_MAX_EXITS);
        s->head_batch = value;
        return EE_OK;
    case EE_OPT_SCATTER_PAGES:
        if (value != 0 && value != 1) return fail(EE_EINVAL, "EE_OPT_SCATTER_PAGES: %d not 0 or 1", value);
        s->scatter_pages = value != 0;
        return EE_OK;
    default:
        return fail(EE_EINVAL, "ee_session_option: unknown option %d", option);
    }
}

// EE_TIME_LAUNCHES sessions: what every launch of the last verify pass ran and how long the
// stream spent between the events recorded right before and right after it.
extern "C" int ee_launch_times(ee_session *s, int32_t *codes, float *ms, int max_launches, int *n_launches)
{
    if (!s || !codes || !ms || !n_launches) return fail(EE_EINVAL, "null argument");
    if (!(s->flags & EE_TIME_LAUNCHES)) return fail(EE_ESTATE, "ee_launch_times: session was created without EE_TIME_LAUNCHES");
    HIP_TRY(hipSetDevice(s->m->device));
    int rc = finish_flight(s);
    if (rc != EE_OK) return rc;
    const int n = std::min((int)s->lt_codes.size(), max_launches);
    for (int i = 0; i < n; ++i) {
        codes[i] = s->lt_codes[i];
        HIP_TRY(hipEventElapsedTime(&ms[i], s->lt_events[2 * i], s->lt_events[2 * i + 1]));
    }
    *n_launches = n;
    return EE_OK;
}

// Measurement aid: `reps` launches of a plain copy kernel (ee_copy_kernel) moving `bytes` bytes
// each between two freshly allocated device buffers.  Profiled with the HBM traffic counters it
// gives the counter reading of a known number of bytes read and written.
extern "C" int ee_debug_copy(int device, size_t bytes, int reps)
{
    HIP_TRY(hipSetDevice(device));
    if (bytes < 16 || reps < 1) return fail(EE_EINVAL, "ee_debug_copy: bytes %zu, reps %d", bytes, reps);
    void *src = nullptr, *dst = nullptr;
    HIP_TRY(hipMalloc(&src, bytes));
    if (hipMalloc(&dst, bytes) != hipSuccess) {
        hipFree(src);
        return fail(EE_EDEVICE, "ee_debug_copy: out of memory");
    }
    hipMemset(src, 0x3C, bytes);
    hipMemset(dst, 0, bytes);
    for (int r = 0; r < reps; ++r)
        hipLaunchKernelGGL(ee_copy_kernel, dim3(4096), dim3(256), 0, 0, static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), bytes / 16);
    hipError_t e = hipDeviceSynchronize();
    hipFree(src);
    hipFree(dst);
    if (e != hipSuccess) return fail(EE_EDEVICE, "ee_debug_copy: %s", hipGetErrorString(e));
    return EE_OK;
}

extern "C" int ee_device_synchronize(int device)
{
    HIP_TRY(hipSetDevice(device));
    HIP_TRY(hipDeviceSynchronize());
    return EE_OK;
}

// ------------------------------------------------------------------ self-check of the MFMA lane layout

// Fills A[16][32] and B[32][16] with small integers, runs one MFMA through the
// lane layout the kernels assume and compares with the plain product.
// Returns EE_OK when every element agrees.
extern "C" int ee_debug_div_small(int device, const int32_t *divisors, int n, long long *mismatches)
{
    if (!divisors || !mismatches || n < 1 || n > 65536) return fail(EE_EINVAL, "ee_debug_div_small: bad argument");
    for (int i = 0; i < n; ++i)
        if (divisors[i] < 1) return fail(EE_EINVAL, "ee_debug_div_small: divisor %d", divisors[i]);
    HIP_TRY(hipSetDevice(device));
    int *dd = nullptr;
    unsigned long long *dbad = nullptr, bad = 0;
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&dd), (size_t)n * sizeof(int)));
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&dbad), sizeof bad));
    HIP_TRY(hipMemcpy(dd, divisors, (size_t)n * sizeof(int), hipMemcpyHostToDevice));
    HIP_TRY(hipMemset(dbad, 0, sizeof bad));
    hipLaunchKernelGGL(div_small_check_kernel, dim3(256, std::min(n, 256)), dim3(256), 0, 0, dd, n, DIV_SMALL_MAX, dbad);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpy(&bad, dbad, sizeof bad, hipMemcpyDeviceToHost));
    hipFree(dd);
    hipFree(dbad);
    *mismatches = (long long)bad;
    return EE_OK;
}

extern "C" int ee_debug_mfma_layout(int device)
{
    HIP_TRY(hipSetDevice(device));
    uint16_t ha[64 * 8], hb[64 * 8];
    float A[16][32], B[32][16];
    for (int i = 0; i < 16; ++i)
        for (int k = 0; k < 32; ++k) A[i][k] = (float)((i * 7 + k * 3) % 13 - 6);
    for (int k = 0; k < 32; ++k)
        for (int j = 0; j < 16; ++j) B[k][j] = (float)((k * 5 + j * 11) % 9 - 4);
    auto bf = [](float f) {
        uint32_t u;
        memcpy(&u, &f, 4);
        return (uint16_t)(u >> 16);  // small integers are exact in bf16
    };
    for (int l = 0; l < 64; ++l)
        for (int e = 0; e < 8; ++e) {
            ha[l * 8 + e] = bf(A[l & 15][(l >> 4) * 8 + e]);
            hb[l * 8 + e] = bf(B[(l >> 4) * 8 + e][l & 15]);
        }
    uint4 *da = nullptr, *db = nullptr;
    float *dout = nullptr;
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&da), sizeof ha));
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&db), sizeof hb));
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&dout), 256 * sizeof(float)));
    HIP_TRY(hipMemcpy(da, ha, sizeof ha, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(db, hb, sizeof hb, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(mfma_layout_probe_kernel, dim3(1), dim3(64), 0, 0, da, db, dout);
    HIP_TRY(hipGetLastError());
    float out[256];
    HIP_TRY(hipMemcpy(out, dout, sizeof out, hipMemcpyDeviceToHost));
    hipFree(da);
    hipFree(db);
    hipFree(dout);
    int bad = 0;
    for (int l = 0; l < 64; ++l)
        for (int r = 0; r < 4; ++r) {
            int i = (l >> 4) * 4 + r, j = l & 15;
            float ref = 0.f;
            for (int k = 0; k < 32; ++k) ref += A[i][k] * B[k][j];
            if (out[l * 4 + r] != ref) ++bad;
        }
    if (bad) return fail(EE_EDEVICE, "MFMA 16x16x32 lane layout differs from the assumed one in %d of 256 elements", bad);

    // v_mfma_f32_16x16x16bf16_1k: the first 16 k of the same matrices, four k per lane
    uint16_t ga[64 * 4], gb[64 * 4];
    for (int l = 0; l < 64; ++l)
        for (int e = 0; e < 4; ++e) {
            ga[l * 4 + e] = bf(A[l & 15][(l >> 4) * 4 + e]);
            gb[l * 4 + e] = bf(B[(l >> 4) * 4 + e][l & 15]);
        }
    uint2 *ea = nullptr, *eb = nullptr;
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&ea), sizeof ga));
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&eb), sizeof gb));
    HIP_TRY(hipMalloc(reinterpret_cast<void **>(&dout), 256 * sizeof(float)));
    HIP_TRY(hipMemcpy(ea, ga, sizeof ga, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(eb, gb, sizeof gb, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(mfma16_layout_probe_kernel, dim3(1), dim3(64), 0, 0, ea, eb, dout);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpy(out, dout, sizeof out, hipMemcpyDeviceToHost));
    hipFree(ea);
    hipFree(eb);
    hipFree(dout);
    bad = 0;
    for (int l = 0; l < 64; ++l)
        for (int r = 0; r < 4; ++r) {
            int i = (l >> 4) * 4 + r, j = l & 15;
            float ref = 0.f;
            for (int k = 0; k < 16; ++k) ref += A[i][k] * B[k][j];
            if (out[l * 4 + r] != ref) ++bad;
        }
    if (bad) return fail(EE_EDEVICE, "MFMA 16x16x16 lane layout differs from the assumed one in %d of 256 elements", bad);
    return EE_OK;
}
