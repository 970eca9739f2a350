// Host side of the engine: arena planning, weight loading, the forward-pass launch sequence
// (skip-mask scheduling: a removed sublayer is simply not launched), prompt pass, the
// draft / verify / accept loop with optional HIP-graph replay, and the C ABI of asd.h.
#include "../../include/asd.h"
#include "asd_attn.h"
#include "asd_common.h"
#include "asd_gemm.h"
#include "asd_misc.h"
#include "asd_pass.h"
#include "asd_prefill.h"
#include "asd_sample.h"

#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <map>
#include <string>
#include <vector>

// Scratch of asd_forward_noalloc: the partial sums, attention partials, counters and argmax candidates of one pass.
// One copy per GPU the library runs on, held until the process ends.  In host code the array's name is only a stand-in
// for the symbol: the address kernels can use comes from hipGetSymbolAddress (scratch_ptr below), once per device.
#define ASD_SCRATCH_BYTES ASD_NOALLOC_SCRATCH_BYTES
static __device__ __align__(256) unsigned char scratch[ASD_SCRATCH_BYTES];

namespace {

thread_local std::string g_create_error;

constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices];      // per device: address of that device's copy of `scratch`

// The current device's scratch address (looked up on the first call per device, with that device current).
hipError_t scratch_ptr(unsigned char** out) {
    int dev = 0;
    hipError_t r = hipGetDevice(&dev);
    if (r != hipSuccess) return r;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        r = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (r != hipSuccess) return r;
        g_scratch_ptr[dev] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

struct GemmCfg { int TN, NW, grid, kmajor, kint; };
struct PfCfg { int NC, KS, PD, NA; };  // prompt GEMM: 16-row chunks per workgroup, K slices, prefetch depth, tiles per wave (0: by balance)

struct Layer {
    char *wqkv, *wo, *wg, *wu, *wd;
    float *g_attn, *g_mlp;
};

struct Profiler {
    std::vector<hipEvent_t> ev;        // pairs
    std::vector<int> cls;
    std::vector<double> bytes;
};

}  // namespace

struct asd_engine {
    asd_config c;
    hipStream_t stream;
    char* arena;
    size_t arena_bytes;
    int es, KE, KBd, KBq, KBf;
    int n_pages, nc_stride, qkv_tiles;
    // weights
    std::vector<Layer> layers;
    char *embed, *lm;
    float* g_final;
    std::vector<uint8_t> have;          // per tensor slot
    // cache
    char* kv;
    size_t kv_layer_bytes;
    int32_t* page_table;
    // workspace
    float *xres, *ssq, *part, *cos_rows, *logits, *o_part, *rope;
    float* ml_part;
    float* qlogits;                     // [16][vocab] draft-model logits of a sampled cycle
    int last_logits_row;                // row of `logits` holding the last prompt row after a prompt pass
    unsigned* arrivals;
    void *xb, *q, *attn_out, *hmid;
    unsigned* counters;
    double* cos_acc;
    AmaxPart* amax_part;
    int32_t *argmax, *tokbuf, *out_tokens;
    DevState* st;
    char* staging;
    size_t staging_bytes;
    // prompt-block workspace
    int32_t* pf_tok;
    float *pf_xres, *pf_raw, *pf_ssq, *pf_rscale, *pf_cos_rows;
    void *pf_xb, *pf_q, *pf_attn_out, *pf_hmid;
    PfCfg pf_qkv, pf_o, pf_gu, pf_down;
    // launch shapes
    GemmCfg g_qkv, g_o, g_gu, g_down, g_lm;
    GemmCfg g_qkv_rows;                 // QKV launch shape of passes of at least QKV_ROWS_MIN rows (same layout, same bits)
    // host state
    int kv_len;
    std::vector<float> acs;
    std::vector<double> acs_sum;         // per sublayer: sum of the prompt rows' cosines
    int acs_rows;
    bool acs_valid;
    DevState* h_st;                     // pinned
    std::map<std::vector<int>, hipGraphExec_t> graphs;
    std::vector<uint8_t> graph_mask;
    unsigned char* scratch = nullptr;   // this device's copy of the static scratch array (asd_forward_noalloc)
    std::string tune;                   // copy of the configuration's debug_tune
    bool sample_mem = false;            // ASD_DBG_SAMPLE_MEM: sampling kernels that re-read memory instead of holding their segments
    bool att_gh1 = false;               // ASD_DBG_ATT_GH1: one query head per attention workgroup also for grouped-query models
    bool force_att_w4 = false;          // ASD_DBG_ATT_W4: always launch the four-waves-per-SIMD attention variant
    bool rs_pow2 = false;               // ASD_DBG_RS_POW2: activation row stride = next power of two
    float graph_T = 0.f;
    uint64_t graph_seed = 0;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};     // phase stamps of a decode cycle: start, drafts done, verification done
    std::string err;
};

namespace {

int fail(asd_engine* e, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (e) e->err = buf; else g_create_error = buf;
    return code;
}

#define CK(e, expr)                                                                              \
    do {                                                                                         \
        hipError_t _r = (expr);                                                                  \
        if (_r != hipSuccess) return fail(e, ASD_E_HIP, "%s: %s", #expr, hipGetErrorString(_r)); \
    } while (0)

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

bool config_ok(const asd_config* c, std::string* why) {
    auto bad = [&](const char* m) { if (why) *why = m; return false; };
    if (!c) return bad("null configuration");
    if (c->dtype != ASD_DT_F32 && c->dtype != ASD_DT_BF16) return bad("dtype must be ASD_DT_F32 or ASD_DT_BF16");
    if (c->n_layers < 1 || c->d_model < 16 || c->n_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 16 || c->d_ffn < 16 ||
        c->vocab < 16 || c->max_seq < 1)
        return bad("non-positive dimension");
    if (c->d_model % 16 || c->d_ffn % 16 || c->vocab % 16) return bad("d_model, d_ffn and vocab must be multiples of 16");
    if (c->n_heads % c->n_kv_heads) return bad("n_heads must be a multiple of n_kv_heads");
    const int hq = c->dtype == ASD_DT_BF16 ? 32 : 16;
    if (c->head_dim % hq) return bad("head_dim must be a multiple of 32 (bf16) or 16 (fp32)");
    if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 32, 64 or 128");
    if (c->page_tokens < 64 || c->page_tokens % 64) return bad("page_tokens must be a positive multiple of 64");
    if (c->max_rows < 1 || c->max_rows > ASD_MAX_ROWS) return bad("max_rows must be in 1..16");
    if (!(c->rms_eps > 0.f) || !(c->rope_theta > 1.f)) return bad("rms_eps must be > 0 and rope_theta > 1");
    if ((long)c->n_layers * 2 > 4096) return bad("too many layers");
    // the decode-attention merge keeps the statistics of at most 64 * ATT_NCL groups of ATT_GROUP keys per head
    static_assert(ASD_MAX_SEQ == 64 * ATT_NCL * ATT_GROUP, "ASD_MAX_SEQ is the attention merge's limit");
    const long pages = ((long)c->max_seq + c->page_tokens - 1) / c->page_tokens;
    if (pages * c->page_tokens > ASD_MAX_SEQ) return bad("max_seq (rounded up to whole pages) exceeds ASD_MAX_SEQ = 65536 positions");
    return true;
}

// Compute units of the current device (what the tile-per-workgroup rule balances over); 256, an MI355X, when no
// device is visible (sizing an arena on a machine without a GPU).
int device_units() {
    static int units = 0;
    if (!units) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) units = n;
        else units = 256;
    }
    return units;
}

// "name=a,b,c,d" entry of the configuration's debug_tune string
int tune_entry(const char* tune, const char* name, int* v, int max_n) {
    if (!tune) return 0;
    const std::string e(tune), key = std::string(name) + "=";
    const size_t pos = (";" + e).find(";" + key);
    if (pos == std::string::npos) return 0;
    int n = 0;
    const char* q = e.c_str() + pos + key.size();
    while (n < max_n) {
        char* end = nullptr;
        const long x = strtol(q, &end, 10);
        if (end == q) break;
        v[n++] = (int)x;
        if (*end != ',') break;
        q = end + 1;
    }
    return n;
}

// Launch shape and weight layout per GEMM class.  Tile-major keeps a tile's K range contiguous; k-major
// keeps the fragments of all tiles for one k-block contiguous (with interleaved k-blocks per wave the
// whole grid then sweeps one contiguous window).  Chosen by measurement on the 7B, 13B and 70B shapes; the
// configuration's debug_tune (development aid) overrides, e.g. "qkv=1,8,1,1;o=1,16,0,0" (TN, NW, k-major, interleave).
GemmCfg pick_cfg(const asd_config& c, int epi, int cls, int tiles, int KB) {
    GemmCfg g{};
    // One tile per workgroup unless two tiles per workgroup leave the busiest compute unit with no more tiles than
    // before (e.g. 320 tiles on 256 units: 2 either way, and the two-tile workgroups stream better: 13B O / down).
    const int units = device_units();
    const int max1 = (tiles + units - 1) / units, max2 = ((tiles + 1) / 2 + units - 1) / units * 2;
    g.TN = (epi == EPI_LM || max2 <= max1) ? 2 : 1;      // (the LM head: two tiles per workgroup at every vocabulary size)
    g.kmajor = (cls == ASD_K_QKV || cls == ASD_K_DOWN || cls == ASD_K_LMHEAD) ? 1 : 0;
    // Long K ranges (KB = KiB of weights per tile), measured on the 70B shape: the output projection (256 KiB per
    // tile, 512 tiles) streams better k-major with one tile per workgroup (24.7 us against 28.7 us), the down
    // projection (896 KiB per tile) better tile-major (73.3 us against 78.1 us); 7B and 13B sit below both limits.
    if (cls == ASD_K_OPROJ && KB >= 256) { g.kmajor = 1; g.TN = 1; }
    if (cls == ASD_K_DOWN && KB >= 512) g.kmajor = 0;
    g.kint = g.kmajor;
    // Waves per workgroup: 8, except where a launch has more workgroups than two rounds of 8-wave workgroups can
    // hold at once and its waves finish far apart (QKV; gate/up with two tile pairs per workgroup): there 4 waves with
    // twice the loads in flight each (the same bytes per workgroup, half the waves to join) measured 1-4 % faster per
    // launch on the 7B, 13B and 70B shapes.
    g.NW = (cls == ASD_K_QKV || (cls == ASD_K_GATEUP && g.TN == 2)) ? 4 : 8;
    static const char* names[ASD_K_COUNT] = {"", "qkv", "", "o", "gu", "down", "lm", ""};       // indexed by kernel class
    int v[4];
    if (tune_entry(c.debug_tune, names[cls], v, 4) == 4) { g.TN = v[0]; g.NW = v[1]; g.kmajor = v[2]; g.kint = v[3]; }
    g.grid = (tiles + g.TN - 1) / g.TN;
    return g;
}

// QKV in passes of several rows.  Every workgroup reads the whole activation vector of every row (as many bytes as its
// weights at 8 rows), and the tiles of one workgroup share those loads: with three tiles per workgroup the 7B QKV
// launch takes 18.5 us at 1, 5, 7 and 9 rows alike, with one tile 17.9 / 18.9 / 19.9 / 21.9 us.  The tiles of a
// workgroup are independent outputs and the waves split K the same way, so the bits do not depend on the choice
// (`test_tiles_per_qkv_workgroup_give_the_same_bits`).  Rule: from QKV_ROWS_MIN rows on, the largest of 3, 2, 1 tiles
// per workgroup that leaves the busiest compute unit with no more tiles than one tile per workgroup does.
#define QKV_ROWS_MIN 5
GemmCfg pick_qkv_rows(const GemmCfg& base, int tiles, const char* tune) {
    GemmCfg g = base;
    int v[4];
    if (tune_entry(tune, "qkv", v, 4) == 4) return g;               // an explicit launch shape holds for every row count
    const int units = device_units();
    auto busiest = [&](int tn) { return ((tiles + tn - 1) / tn + units - 1) / units * tn; };
    for (int tn = 3; tn > base.TN; --tn)
        if (busiest(tn) <= busiest(base.TN)) { g.TN = tn; break; }
    if (tune_entry(tune, "qkv_rows", v, 1) == 1 && v[0] >= 1 && v[0] <= 3) g.TN = v[0];
    g.grid = (tiles + g.TN - 1) / g.TN;
    return g;
}

struct Plan {
    size_t embed, lm, g_final, layer0, layer_stride, wqkv, wo, wg, wu, wd, g_attn, g_mlp;
    size_t kv, kv_layer, page_table;
    size_t xres, ssq, part, cos_rows, logits, o_part, rope, ml_part, arrivals, xb, q, attn_out, hmid, counters, cos_acc, amax_part,
        argmax, tokbuf, out_tokens, st, ops, ops_bytes, staging, staging_bytes, total, qlogits;
    size_t pf_tok, pf_xres, pf_raw, pf_ssq, pf_rscale, pf_cos_rows, pf_xb, pf_q, pf_attn_out, pf_hmid;
    int es, KE, KBd, KBq, KBf, n_pages, nc_stride, qkv_tiles;
    GemmCfg g_qkv, g_o, g_gu, g_down, g_lm;
};

Plan make_plan(const asd_config& c) {
    Plan p{};
    p.es = c.dtype == ASD_DT_BF16 ? 2 : 4;
    p.KE = 16 / p.es;
    const int kblk = 4 * p.KE;
    const int qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
    p.KBd = (c.d_model + kblk - 1) / kblk;
    p.KBq = (qd + kblk - 1) / kblk;
    p.KBf = (c.d_ffn + kblk - 1) / kblk;
    p.n_pages = (c.max_seq + c.page_tokens - 1) / c.page_tokens;
    p.nc_stride = (p.n_pages * c.page_tokens + ATT_GROUP - 1) / ATT_GROUP;
    p.qkv_tiles = (qd + 2 * kvd) / 16;
    p.g_qkv = pick_cfg(c, EPI_QKV, ASD_K_QKV, p.qkv_tiles, p.KBd);
    p.g_o = pick_cfg(c, EPI_RES, ASD_K_OPROJ, c.d_model / 16, p.KBq);
    p.g_gu = pick_cfg(c, EPI_GU, ASD_K_GATEUP, c.d_ffn / 16, p.KBd);
    p.g_down = pick_cfg(c, EPI_RES, ASD_K_DOWN, c.d_model / 16, p.KBf);
    p.g_lm = pick_cfg(c, EPI_LM, ASD_K_LMHEAD, c.vocab / 16, p.KBd);

    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    const size_t frag = 1024;   // bytes of one (tile, k-block)
    p.embed = take((size_t)c.vocab * c.d_model * p.es);
    p.lm = take((size_t)(c.vocab / 16) * p.KBd * frag);
    p.g_final = take((size_t)c.d_model * 4);
    p.layer0 = off;
    p.wqkv = take((size_t)p.qkv_tiles * p.KBd * frag) - p.layer0;
    p.wo = take((size_t)(c.d_model / 16) * p.KBq * frag) - p.layer0;
    p.wg = take((size_t)(c.d_ffn / 16) * p.KBd * frag) - p.layer0;
    p.wu = take((size_t)(c.d_ffn / 16) * p.KBd * frag) - p.layer0;
    p.wd = take((size_t)(c.d_model / 16) * p.KBf * frag) - p.layer0;
    p.g_attn = take((size_t)c.d_model * 4) - p.layer0;
    p.g_mlp = take((size_t)c.d_model * 4) - p.layer0;
    p.layer_stride = off - p.layer0;
    off = p.layer0 + p.layer_stride * c.n_layers;
    p.kv_layer = (size_t)p.n_pages * c.n_kv_heads * 2 * c.page_tokens * c.head_dim * p.es;
    p.kv = take(p.kv_layer * c.n_layers);
    p.page_table = take((size_t)p.n_pages * 4);
    p.xres = take((size_t)ASD_ROWS * c.d_model * 4);
    p.ssq = take(ASD_ROWS * 4);
    int pmax = p.g_o.grid > p.g_down.grid ? p.g_o.grid : p.g_down.grid;
    if (pmax < EMBED_SPLIT) pmax = EMBED_SPLIT;
    p.part = take((size_t)pmax * ASD_ROWS * 2 * 4);
    p.cos_rows = take((size_t)2 * c.n_layers * ASD_ROWS * 4);
    p.logits = take((size_t)ASD_ROWS * c.vocab * 4);
    p.qlogits = take((size_t)ASD_ROWS * c.vocab * 4 + ASD_ROWS * 16);      // + per row: (maximum, Z) of the draft softmax as doubles
    p.o_part = take((size_t)c.n_heads * p.nc_stride * ASD_ROWS * c.head_dim * 4);
    p.rope = take((size_t)p.n_pages * c.page_tokens * (c.head_dim / 2) * 2 * 4);
    p.ml_part = take((size_t)c.n_heads * p.nc_stride * ASD_ROWS * 8);
    p.arrivals = take((size_t)c.n_heads * 4);
    const int NPL = c.dtype == ASD_DT_BF16 ? 2 : 1;     // activation planes
    p.xb = take((size_t)p.KBd * frag * NPL);
    p.q = take((size_t)c.n_heads * c.head_dim * ASD_ROWS * p.es * NPL);
    p.attn_out = take((size_t)p.KBq * frag * NPL);
    p.hmid = take((size_t)p.KBf * frag * NPL);
    p.counters = take(256);
    p.cos_acc = take((size_t)2 * c.n_layers * 8);
    p.amax_part = take((size_t)p.g_lm.grid * ASD_ROWS * sizeof(AmaxPart));
    p.argmax = take(ASD_ROWS * 4);
    p.tokbuf = take(64 * 4);
    p.out_tokens = take((size_t)(p.n_pages * c.page_tokens + 64) * 4);
    p.st = take(sizeof(DevState));
    size_t biggest = (size_t)c.vocab * c.d_model;
    if ((size_t)c.d_ffn * c.d_model > biggest) biggest = (size_t)c.d_ffn * c.d_model;
    if ((size_t)qd * c.d_model > biggest) biggest = (size_t)qd * c.d_model;
    p.staging_bytes = align_up(biggest * p.es + 4096);
    p.staging = take(p.staging_bytes);
    // prompt-block workspace: PF_ROWS rows as PF_CHUNKS chunks of 16
    p.pf_tok = take((size_t)PF_ROWS * 4);
    p.pf_xres = take((size_t)PF_ROWS * c.d_model * 4);
    p.pf_raw = take((size_t)PF_MAX_KSPLIT * PF_ROWS * c.d_model * 4);
    p.pf_ssq = take((size_t)PF_ROWS * 4);
    p.pf_rscale = take((size_t)PF_ROWS * 4);
    p.pf_cos_rows = take((size_t)2 * c.n_layers * PF_ROWS * 4);
    p.pf_xb = take((size_t)PF_CHUNKS * p.KBd * frag * NPL);
    p.pf_q = take((size_t)PF_CHUNKS * p.KBq * frag * NPL);
    p.pf_attn_out = take((size_t)PF_CHUNKS * p.KBq * frag * NPL);
    p.pf_hmid = take((size_t)PF_CHUNKS * p.KBf * frag * NPL);
    p.total = off;
    return p;
}

// ------------------------------------------------------------------ tensor table
struct TensorInfo { int rows, cols; bool norm; bool tiled; };

bool tensor_info(const asd_config& c, int t, TensorInfo* ti) {
    const int qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
    switch (t) {
        case ASD_T_EMBED: *ti = {c.vocab, c.d_model, false, false}; return true;
        case ASD_T_LM_HEAD: *ti = {c.vocab, c.d_model, false, true}; return true;
        case ASD_T_WQ: *ti = {qd, c.d_model, false, true}; return true;
        case ASD_T_WK: case ASD_T_WV: *ti = {kvd, c.d_model, false, true}; return true;
        case ASD_T_WO: *ti = {c.d_model, qd, false, true}; return true;
        case ASD_T_WG: case ASD_T_WU: *ti = {c.d_ffn, c.d_model, false, true}; return true;
        case ASD_T_WD: *ti = {c.d_model, c.d_ffn, false, true}; return true;
        case ASD_T_ATTN_NORM: case ASD_T_MLP_NORM: case ASD_T_FINAL_NORM: *ti = {1, c.d_model, true, false}; return true;
        default: return false;
    }
}
bool tensor_is_global(int t) { return t == ASD_T_EMBED || t == ASD_T_LM_HEAD || t == ASD_T_FINAL_NORM; }
int have_slot(const asd_engine* e, int t, int layer) { return tensor_is_global(t) ? t : 12 + layer * 12 + t; }

// where a tensor lives: base address of its (possibly fused) tile array and how its tiles are laid out
struct TensorLoc { char* base; TileMap tm; };

TileMap make_map(const GemmCfg& g, int total_tiles, int KB, int tile0, int rope_h) {
    TileMap tm;
    tm.ts = g.kmajor ? 1 : KB; tm.ks = g.kmajor ? total_tiles : 1; tm.tile0 = tile0; tm.KB = KB; tm.rope_h = rope_h;
    return tm;
}

TensorLoc tensor_loc(asd_engine* e, int t, int layer) {
    const asd_config& c = e->c;
    const int qd = c.n_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
    const TileMap none{};
    switch (t) {
        case ASD_T_EMBED: return {e->embed, none};
        case ASD_T_FINAL_NORM: return {(char*)e->g_final, none};
        case ASD_T_ATTN_NORM: return {(char*)e->layers[layer].g_attn, none};
        case ASD_T_MLP_NORM: return {(char*)e->layers[layer].g_mlp, none};
        case ASD_T_LM_HEAD: return {e->lm, make_map(e->g_lm, c.vocab / 16, e->KBd, 0, 0)};
        case ASD_T_WQ: return {e->layers[layer].wqkv, make_map(e->g_qkv, e->qkv_tiles, e->KBd, 0, c.head_dim)};
        case ASD_T_WK: return {e->layers[layer].wqkv, make_map(e->g_qkv, e->qkv_tiles, e->KBd, qd / 16, c.head_dim)};
        case ASD_T_WV: return {e->layers[layer].wqkv, make_map(e->g_qkv, e->qkv_tiles, e->KBd, (qd + kvd) / 16, c.head_dim)};
        case ASD_T_WO: return {e->layers[layer].wo, make_map(e->g_o, c.d_model / 16, e->KBq, 0, 0)};
        case ASD_T_WG: return {e->layers[layer].wg, make_map(e->g_gu, c.d_ffn / 16, e->KBd, 0, 0)};
        case ASD_T_WU: return {e->layers[layer].wu, make_map(e->g_gu, c.d_ffn / 16, e->KBd, 0, 0)};
        case ASD_T_WD: return {e->layers[layer].wd, make_map(e->g_down, c.d_model / 16, e->KBf, 0, 0)};
    }
    return {nullptr, none};
}

template <class T> void launch_tile(asd_engine* e, const void* src, void* dst, int N, int K, const TileMap& tm, bool untile) {
    const size_t frags = (size_t)(N / 16) * tm.KB * 64;
    const unsigned grid = (unsigned)((frags + 255) / 256);
    using El = typename T::elem;
    if (untile) untile_weight_kernel<T><<<grid, 256, 0, e->stream>>>((const El*)src, (El*)dst, N, K, tm);
    else tile_weight_kernel<T><<<grid, 256, 0, e->stream>>>((const El*)src, (El*)dst, N, K, tm);
}

// ------------------------------------------------------------------ GEMM dispatch
#ifndef ASD_GEMM_U
#define ASD_GEMM_U 4          // weight fragments in flight per wave and tile
#endif
template <class T, int EPI, int TN, int NW>
void launch_gemm_inst(hipStream_t s, int grid, const GemmArgs& a) {
    // four-wave workgroups keep twice the weight fragments in flight per wave: the same bytes per workgroup
    constexpr int UU = NW == 4 ? 2 * ASD_GEMM_U : ASD_GEMM_U;
    // (the leading arguments: what the first requests need, preloaded into SGPRs; see gemm_kernel)
    const int32_t packed = a.k_interleave | (a.M << 8) | (a.RS << 16);
    const int32_t wts = (int32_t)a.w_tile_stride, wks = (int32_t)a.w_kb_stride;
    if constexpr (T::NP == 2) {          // two-plane activations: passes of at most 8 rows pack both planes into one operand
        if (a.M <= 8) {
            gemm_kernel<T, EPI, TN, NW, UU, true><<<grid, NW * 64, 0, s>>>(a.W, a.X, wts, wks, a.n_tiles, a.KB, packed, 0, a.x_plane, a.W2, a);
            return;
        }
    }
    gemm_kernel<T, EPI, TN, NW, UU, false><<<grid, NW * 64, 0, s>>>(a.W, a.X, wts, wks, a.n_tiles, a.KB, packed, 0, a.x_plane, a.W2, a);
}

template <class T, int EPI>
bool launch_gemm_t(hipStream_t s, const GemmCfg& g, const GemmArgs& a) {
#define CASE(tn, nw) if (g.TN == tn && g.NW == nw) { launch_gemm_inst<T, EPI, tn, nw>(s, g.grid, a); return true; }
    if constexpr (EPI == EPI_QKV) { CASE(1, 4) CASE(1, 8) CASE(1, 16) CASE(2, 4) CASE(2, 8) CASE(3, 4) CASE(3, 8) }
    if constexpr (EPI == EPI_RES) { CASE(1, 4) CASE(1, 8) CASE(1, 16) CASE(2, 4) CASE(2, 8) CASE(2, 16) }
    if constexpr (EPI == EPI_GU) { CASE(1, 4) CASE(1, 8) CASE(2, 4) CASE(2, 8) }
    if constexpr (EPI == EPI_LM) { CASE(1, 4) CASE(1, 8) CASE(2, 4) CASE(2, 8) }
#undef CASE
    return false;
}

template <int EPI> bool launch_gemm(asd_engine* e, const GemmCfg& g, const GemmArgs& a) {
    return e->c.dtype == ASD_DT_BF16 ? launch_gemm_t<BF16, EPI>(e->stream, g, a) : launch_gemm_t<F32, EPI>(e->stream, g, a);
}

int capacity(const asd_engine* e);

static const GemmCfg& qkv_cfg(const asd_engine* e, int M) { return M >= QKV_ROWS_MIN ? e->g_qkv_rows : e->g_qkv; }

// Row stride of the tiled activation buffers of an M-row pass (rows per k-group).  The activation bytes a GEMM
// workgroup reads grow with it, so it is the row count itself, not the next power of two (a 5-row verification
// pass read 8 rows' worth).
static int row_stride(const asd_engine* e, int M) {
    if (e->rs_pow2) { int rs = 1; while (rs < M) rs *= 2; return rs; }
    return M;
}

// Launch shape of the decode attention for a context of nc 64-key chunks (a.M and a.RS are set)
void attn_shape(const asd_engine* e, AttnArgs& a, int nc) {
    a.grid_groups = (nc + ATT_GW - 1) / ATT_GW;
    a.cap_chunks = capacity(e) / ASD_CHUNK;
    // grouped-query models: as many query heads of a KV head per workgroup as the 16 columns hold beside the rows
    a.gh = 1;
    if (!e->att_gh1) while (a.gh * 2 * a.RS <= ASD_ROWS && a.gh * 2 <= e->c.n_heads / e->c.n_kv_heads && (e->c.n_heads / e->c.n_kv_heads) % (a.gh * 2) == 0) a.gh *= 2;
}

template <class T> void launch_attn_t(asd_engine* e, const AttnArgs& a) {
    const int H = e->c.head_dim;
    const int units = e->c.n_heads / a.gh;                    // workgroups per group index
    const int grid = attn_grid(e->c.n_heads, e->c.n_kv_heads, a.grid_groups, a.gh);
    // The first variant holds 512 workgroups at once (two per compute unit) and keeps all of a chunk's loads in flight;
    // the four-waves-per-SIMD variant holds 1024.  It wins only where it takes the whole grid in one round while the
    // first variant would be left with a small second one (measured, 7B: 21.7 against 23.2 us at 544 workgroups);
    // beyond 1024 workgroups both run in rounds and the first is faster per byte (36 against 40 us at 1056,
    // 60 against 69 us at 2080, 110 against 115 us at 4128).
    const long n_wg = (long)a.grid_groups * units;
    const bool many = (n_wg > 512 && n_wg <= 1024) || e->force_att_w4;
    // (the leading arguments: what the first requests need, preloaded into SGPRs; see attn_kernel)
#define ATT_HOT a.q, a.kv, a.page_table, a.q_plane, a.n_h | (a.n_kv << 16), a.M | (a.RS << 8) | (a.gh << 16), a.grid_groups, a.cap_chunks, a.page_tokens, 0
#define ATT(h)                                                                          \
    if (H == h) {                                                                       \
        if (many) attn_kernel_w4<T, h><<<grid, ATT_GW * 64, 0, e->stream>>>(ATT_HOT, a); \
        else attn_kernel<T, h><<<grid, ATT_GW * 64, 0, e->stream>>>(ATT_HOT, a);         \
    }
    ATT(32) ATT(64) ATT(128)
#undef ATT
#undef ATT_HOT
}
void launch_attn(asd_engine* e, const AttnArgs& a) {
    if (e->c.dtype == ASD_DT_BF16) launch_attn_t<BF16>(e, a); else launch_attn_t<F32>(e, a);
}

// ------------------------------------------------------------------ algorithmic bytes
// What one forward pass must read: kept sublayers' weights, the LM head, and the K/V of ctx positions.
void pass_bytes(const asd_engine* e, const uint8_t* mask, int ctx, double* by_class) {
    const asd_config& c = e->c;
    const double es = e->es, qd = (double)c.n_heads * c.head_dim, kvd = (double)c.n_kv_heads * c.head_dim;
    for (int i = 0; i < ASD_K_COUNT; ++i) by_class[i] = 0.0;
    for (int l = 0; l < c.n_layers; ++l) {
        if (!(mask && mask[2 * l])) {
            by_class[ASD_K_QKV] += es * (qd + 2 * kvd) * c.d_model;
            by_class[ASD_K_ATTN] += es * 2 * kvd * ctx;
            by_class[ASD_K_OPROJ] += es * qd * c.d_model;
        }
        if (!(mask && mask[2 * l + 1])) {
            by_class[ASD_K_GATEUP] += es * 2.0 * c.d_ffn * c.d_model;
            by_class[ASD_K_DOWN] += es * (double)c.d_ffn * c.d_model;
        }
    }
    by_class[ASD_K_LMHEAD] = es * (double)c.vocab * c.d_model;
}

// ------------------------------------------------------------------ forward pass (enqueue only)
const float* next_gain(const asd_engine* e, const uint8_t* mask, int after /* sublayer index, -1 = before all */) {
    for (int j = after + 1; j < 2 * e->c.n_layers; ++j)
        if (!(mask && mask[j])) return (j & 1) ? e->layers[j / 2].g_mlp : e->layers[j / 2].g_attn;
    return e->g_final;
}

struct Prof {
    Profiler* p;
    hipStream_t s;
    void begin(int cls, double bytes) {
        if (!p) return;
        hipEvent_t a, b;
        hipEventCreate(&a); hipEventCreate(&b);
        hipEventRecord(a, s);
        p->ev.push_back(a); p->ev.push_back(b); p->cls.push_back(cls); p->bytes.push_back(bytes);
    }
    void end() { if (p) hipEventRecord(p->ev.back(), s); }
};

// Where a pass's results go (the engine's own buffers, or a caller's device buffers) and where its kernels keep what
// they exchange: partial sums, attention partials and their arrival counters, argmax candidates (the engine's arena,
// or the library's static scratch array).
struct PassOut {
    float* logits;       // [rows][vocab]
    int32_t* argmax;     // [16]
    float *ssq, *part, *cos_rows;
    double* cos_acc;
    float *o_part, *ml_part;
    unsigned* arrivals;
    AmaxPart* amax_part;
    int nc_stride;       // groups per head in o_part / ml_part
};
PassOut engine_out(const asd_engine* e) {
    return PassOut{e->logits, e->argmax, e->ssq, e->part, e->cos_rows, e->cos_acc, e->o_part, e->ml_part, e->arrivals, e->amax_part, e->nc_stride};
}

// The steps of one forward pass of M rows (first row at cache position st->pos + pos_off) under a skip mask:
// a removed sublayer contributes no step at all.
void build_pass(asd_engine* e, int M, int pos_off, const uint8_t* mask, int ctx_for_bytes, int nc, const PassOut& out, std::vector<PassOp>& ops) {
    const asd_config& c = e->c;
    double cls_bytes[ASD_K_COUNT];
    pass_bytes(e, nullptr, ctx_for_bytes, cls_bytes);   // full-model totals; per-sublayer figures divide by L
    const double L = c.n_layers;
    const int RS = row_stride(e, M);
    ops.clear();
    auto push = [&](int type, int cls, int grid, double bytes) -> PassOp& {
        PassOp op{};
        op.type = type; op.cls = cls; op.grid = grid; op.bytes = bytes;
        ops.push_back(op);
        return ops.back();
    };
    push(OP_EMBED, ASD_K_EMBED, EMBED_SPLIT * M, 0);

    GemmArgs base{};
    base.M = M; base.RS = RS; base.ssq = out.ssq; base.inv_d = 1.f / (float)c.d_model; base.eps = c.rms_eps;
    base.xres = e->xres; base.xb = e->xb; base.part = out.part; base.d = c.d_model;
    base.st = e->st; base.pos_off = pos_off; base.rope = e->rope; base.page_table = e->page_table;
    base.n_h = c.n_heads; base.n_kv = c.n_kv_heads; base.h = c.head_dim; base.page_tokens = c.page_tokens;
    base.xb_plane = (int64_t)e->KBd * 64 * e->KE; base.hmid_plane = (int64_t)e->KBf * 64 * e->KE;
    base.q_plane = (int64_t)c.n_heads * c.head_dim * ASD_ROWS;
    base.logits = out.logits; base.V = c.vocab; base.amax_part = out.amax_part;
    // the cosine tap still open: partials of the last residual-add step and where its cosine goes
    // (the embedding leaves EMBED_SPLIT partials of ||x||^2 and no cosine to finish)
    int open_P = EMBED_SPLIT, open_sub = -1;
    // a step that reads the normed residual: its input, the producing step's partials, the open cosine tap
    auto consume = [&](GemmArgs& g) {
        g.X = (const u32x4*)e->xb; g.x_plane = (int64_t)e->KBd * 64;
        g.part_in = out.part; g.P_in = open_P;
        if (open_sub >= 0) { g.fin_cos_rows = out.cos_rows + (size_t)open_sub * ASD_ROWS; g.fin_cos_acc = out.cos_acc + open_sub; }
    };
    auto layout = [&](GemmArgs& g, const GemmCfg& cfg, int total_tiles, int KB) {
        g.KB = KB; g.w_tile_stride = cfg.kmajor ? 1 : KB; g.w_kb_stride = cfg.kmajor ? total_tiles : 1; g.k_interleave = cfg.kint;
    };

    for (int l = 0; l < c.n_layers; ++l) {
        const Layer& ly = e->layers[l];
        if (!(mask && mask[2 * l])) {
            GemmArgs a = base;
            a.W = (const u32x4*)ly.wqkv; a.n_tiles = e->qkv_tiles;
            layout(a, e->g_qkv, e->qkv_tiles, e->KBd);
            a.kv = e->kv + (size_t)l * e->kv_layer_bytes;
            a.q = e->q;
            consume(a);
            push(OP_QKV, ASD_K_QKV, qkv_cfg(e, M).grid, cls_bytes[ASD_K_QKV] / L).g = a;

            AttnArgs t{};
            t.q = a.q; t.q_plane = base.q_plane; t.out_plane = (int64_t)e->KBq * 64 * e->KE; t.kv = a.kv;
            t.page_table = e->page_table; t.st = e->st; t.pos_off = pos_off; t.M = M; t.RS = RS;
            t.n_h = c.n_heads; t.n_kv = c.n_kv_heads; t.h = c.head_dim; t.page_tokens = c.page_tokens;
            t.nc_stride = out.nc_stride; t.scale = 1.f / sqrtf((float)c.head_dim);
            t.o_part = out.o_part; t.ml_part = out.ml_part; t.arrivals = out.arrivals;
            t.out = e->attn_out;
            attn_shape(e, t, nc);
            push(OP_ATTN, ASD_K_ATTN, attn_grid(c.n_heads, c.n_kv_heads, t.grid_groups, t.gh), cls_bytes[ASD_K_ATTN] / L).t = t;

            GemmArgs o = base;
            o.W = (const u32x4*)ly.wo; o.X = (const u32x4*)t.out; o.x_plane = (int64_t)e->KBq * 64; o.n_tiles = c.d_model / 16;
            layout(o, e->g_o, c.d_model / 16, e->KBq);
            o.g_next = next_gain(e, mask, 2 * l);
            open_P = e->g_o.grid; open_sub = 2 * l;
            push(OP_OPROJ, ASD_K_OPROJ, e->g_o.grid, cls_bytes[ASD_K_OPROJ] / L).g = o;
        }
        if (!(mask && mask[2 * l + 1])) {
            GemmArgs a = base;
            a.W = (const u32x4*)ly.wg; a.W2 = (const u32x4*)ly.wu;
            a.n_tiles = c.d_ffn / 16; layout(a, e->g_gu, c.d_ffn / 16, e->KBd);
            a.hmid = e->hmid;
            consume(a);
            push(OP_GU, ASD_K_GATEUP, e->g_gu.grid, cls_bytes[ASD_K_GATEUP] / L).g = a;

            GemmArgs dn = base;
            dn.W = (const u32x4*)ly.wd; dn.X = (const u32x4*)a.hmid; dn.x_plane = (int64_t)e->KBf * 64; dn.n_tiles = c.d_model / 16;
            layout(dn, e->g_down, c.d_model / 16, e->KBf);
            dn.g_next = next_gain(e, mask, 2 * l + 1);
            open_P = e->g_down.grid; open_sub = 2 * l + 1;
            push(OP_DOWN, ASD_K_DOWN, e->g_down.grid, cls_bytes[ASD_K_DOWN] / L).g = dn;
        }
    }
    GemmArgs lm = base;
    lm.W = (const u32x4*)e->lm; lm.n_tiles = c.vocab / 16;
    layout(lm, e->g_lm, c.vocab / 16, e->KBd);
    consume(lm);
    push(OP_LM, ASD_K_LMHEAD, e->g_lm.grid, cls_bytes[ASD_K_LMHEAD]).g = lm;
    push(OP_FINISH, ASD_K_FINISH, 1, 0);
}

// Run a pass as one launch per step.
int launch_steps(asd_engine* e, const std::vector<PassOp>& ops, const int32_t* d_tokens, int M, const uint8_t* mask,
                 Profiler* profiler, int fin_mode, int fin_arg, const PassOut& out) {
    const asd_config& c = e->c;
    Prof pr{profiler, e->stream};
    const int RS = row_stride(e, M);
    for (const PassOp& op : ops) {
        pr.begin(op.cls, op.bytes);
        bool ok = true;
        switch (op.type) {
            case OP_EMBED:
                if (c.dtype == ASD_DT_BF16)
                    embed_kernel<BF16><<<dim3(EMBED_SPLIT, M), EMBED_THREADS, 0, e->stream>>>((const uint16_t*)e->embed, d_tokens, c.d_model, c.vocab, e->st,
                        next_gain(e, mask, -1), e->xres, e->xb, (size_t)e->KBd * 64 * e->KE, RS, out.part);
                else
                    embed_kernel<F32><<<dim3(EMBED_SPLIT, M), EMBED_THREADS, 0, e->stream>>>((const float*)e->embed, d_tokens, c.d_model, c.vocab, e->st,
                        next_gain(e, mask, -1), e->xres, e->xb, (size_t)e->KBd * 64 * e->KE, RS, out.part);
                break;
            case OP_QKV: ok = launch_gemm<EPI_QKV>(e, qkv_cfg(e, M), op.g); break;
            case OP_OPROJ: ok = launch_gemm<EPI_RES>(e, e->g_o, op.g); break;
            case OP_DOWN: ok = launch_gemm<EPI_RES>(e, e->g_down, op.g); break;
            case OP_GU: ok = launch_gemm<EPI_GU>(e, e->g_gu, op.g); break;
            case OP_LM: ok = launch_gemm<EPI_LM>(e, e->g_lm, op.g); break;
            case OP_ATTN: launch_attn(e, op.t); break;
            case OP_FINISH:
                finish_kernel<<<1, 64 * M, 0, e->stream>>>((const AmaxCand*)out.amax_part, e->g_lm.grid, M, c.vocab, out.argmax, fin_mode, fin_arg,
                                                           e->st, e->tokbuf, e->out_tokens);
                break;
        }
        pr.end();
        if (!ok) return fail(e, ASD_E_STATE, "no kernel instance for step type %d of this shape", op.type);
    }
    hipError_t r = hipGetLastError();
    if (r != hipSuccess) return fail(e, ASD_E_HIP, "kernel launch: %s", hipGetErrorString(r));
    return ASD_OK;
}

int enqueue_forward(asd_engine* e, const int32_t* d_tokens, int M, int pos_off, const uint8_t* mask, int nc,
                    Profiler* profiler, int ctx_for_bytes, int fin_mode = FIN_NONE, int fin_arg = 0, const PassOut* out_or_null = nullptr) {
    const PassOut out = out_or_null ? *out_or_null : engine_out(e);
    std::vector<PassOp> ops;
    build_pass(e, M, pos_off, mask, ctx_for_bytes, nc, out, ops);
    return launch_steps(e, ops, d_tokens, M, mask, profiler, fin_mode, fin_arg, out);
}

bool weights_ready(asd_engine* e) {
    for (uint8_t h : e->have) if (!h) return false;
    return true;
}

int chunks_for(int last_pos) { return last_pos / ASD_CHUNK + 1; }

// After a synchronisation: did a kernel meet a token id outside the vocabulary, or a row of logits without a finite
// maximum?  (st: a host copy of the decoding state, or NULL to fetch it.)
int check_pass_error(asd_engine* e, const DevState* st = nullptr) {
    DevState tmp;
    if (!st) { CK(e, hipMemcpy(&tmp, e->st, sizeof tmp, hipMemcpyDeviceToHost)); st = &tmp; }
    if (st->err & DEV_ERR_TOKEN) return fail(e, ASD_E_INVAL, "a token id outside the vocabulary reached the embedding");
    if (st->err & DEV_ERR_LOGITS) return fail(e, ASD_E_STATE, "a row of logits had no finite maximum (non-finite weights?)");
    return ASD_OK;
}

int check_tokens(asd_engine* e, const int32_t* t, int n) {
    for (int i = 0; i < n; ++i)
        if (t[i] < 0 || t[i] >= e->c.vocab) return fail(e, ASD_E_INVAL, "token id %d at index %d outside [0, %d)", t[i], i, e->c.vocab);
    return ASD_OK;
}

void drop_graphs(asd_engine* e) {
    for (auto& kv : e->graphs) hipGraphExecDestroy(kv.second);
    e->graphs.clear();
}

int capacity(const asd_engine* e) { return e->n_pages * e->c.page_tokens; }

// release what the engine owns on the host side (graphs, events, pinned state) and the engine itself
void destroy_host(asd_engine* e) {
    drop_graphs(e);
    for (hipEvent_t ev : e->ev) if (ev) hipEventDestroy(ev);
    if (e->h_st) hipHostFree(e->h_st);
    delete e;
}

// ------------------------------------------------------------------ prompt blocks
// Launch shape of a prompt GEMM class: NC 16-row chunks per workgroup and K slices (slices only for the two
// residual-add GEMMs).  The configuration's debug_tune (development aid) overrides, e.g. "pf_qkv=8,1;pf_o=8,2;pf_gu=4,1;pf_down=8,4".
PfCfg pf_pick(const char* tune, const char* name, int nc, int ks) {
    PfCfg g{nc, ks, 2, 0};
    int v[4] = {0, 0, 1, 0};
    const int n = tune_entry(tune, name, v, 4);
    if (n >= 2 && (v[0] == 2 || v[0] == 4 || v[0] == 8) && v[1] >= 1 && v[1] <= PF_MAX_KSPLIT && v[2] >= 1 && v[2] <= 4) { g.NC = v[0]; g.KS = v[1]; g.PD = v[2]; }
    if (n == 4 && v[3] >= 3 && v[3] <= 5) g.NA = v[3];
    return g;
}

constexpr int PF_NW = 4;                 // waves per workgroup of a prompt GEMM
template <int EPI> constexpr int pf_na() { return EPI == PF_GU ? 2 : 4; }     // weight tiles per wave (gate and up each, for PF_GU)

template <class T, int EPI, int NA> bool launch_pf_gemm_na(hipStream_t s, const PfCfg& g, PfArgs a, int n_chunks) {
    a.n_fb = (a.n_tiles + PF_NW * NA - 1) / (PF_NW * NA);
    a.n_rb = (n_chunks + g.NC - 1) / g.NC;
    a.ksplit = EPI == PF_RAW ? g.KS : 1;
    if (a.ksplit > a.KB) a.ksplit = a.KB;
    const unsigned grid = (unsigned)((a.n_fb + 7) / 8 * 8 * a.n_rb * a.ksplit);
#define PFK(nc, pd) if (g.NC == nc && g.PD == pd) { pf_gemm_kernel<T, EPI, NA, nc, PF_NW, pd><<<grid, PF_NW * 64, 0, s>>>(a); return true; }
    if constexpr (NA == pf_na<EPI>()) { PFK(2, 1) PFK(4, 1) PFK(8, 1) PFK(2, 2) PFK(4, 2) PFK(8, 2) PFK(2, 3) PFK(4, 3) PFK(2, 4) PFK(4, 4) }
    else { PFK(4, 2) }
#undef PFK
    return false;
}
// Tiles per wave of the prompt QKV GEMM.  Its workgroups cannot split K (the epilogue rotates and stores whole sums),
// so their number is feature blocks x row blocks, and with the default 4 tiles per wave that is 384 on the 7B shape:
// half the compute units hold two workgroups, half one, and the launch lasts as long as two.  Among 4, 3 and 5
// tiles per wave the one is taken that gives the busiest compute unit the least work (workgroups on it x tiles per
// wave): 7B 3 tiles (512 workgroups, two everywhere), 13B 4, 70B 5.  Which wave owns a tile does not enter any sum.
static int pf_qkv_na(const PfCfg& g, int n_tiles, int n_chunks) {
    if (g.NA) return g.NA;
    if (g.NC != 4 || g.PD != 2) return 4;
    const int units = device_units(), n_rb = (n_chunks + g.NC - 1) / g.NC;
    int best = 4, best_cost = 1 << 30;
    for (int na : {4, 3, 5}) {
        const int n_fb = (n_tiles + PF_NW * na - 1) / (PF_NW * na);
        const int cost = (n_fb * n_rb + units - 1) / units * na;
        if (cost < best_cost) { best = na; best_cost = cost; }
    }
    return best;
}
template <class T, int EPI> bool launch_pf_gemm_t(hipStream_t s, const PfCfg& g, PfArgs a, int n_chunks) {
    if constexpr (EPI == PF_QKV) {
        const int na = pf_qkv_na(g, a.n_tiles, n_chunks);
        if (na == 3) return launch_pf_gemm_na<T, EPI, 3>(s, g, a, n_chunks);
        if (na == 5) return launch_pf_gemm_na<T, EPI, 5>(s, g, a, n_chunks);
    }
    return launch_pf_gemm_na<T, EPI, pf_na<EPI>()>(s, g, a, n_chunks);
}
template <int EPI> bool launch_pf_gemm(asd_engine* e, const PfCfg& g, const PfArgs& a, int n_chunks) {
    return e->c.dtype == ASD_DT_BF16 ? launch_pf_gemm_t<BF16, EPI>(e->stream, g, a, n_chunks) : launch_pf_gemm_t<F32, EPI>(e->stream, g, a, n_chunks);
}

template <class T> void launch_pf_attn_t(asd_engine* e, const PfAttnArgs& a, int n_chunks) {
    const int H = e->c.head_dim;
    const dim3 grid((n_chunks + PF_ATT_NT - 1) / PF_ATT_NT, e->c.n_heads);
    if (H == 32) pf_attn_kernel<T, 32><<<grid, 256, 0, e->stream>>>(a);
    if (H == 64) pf_attn_kernel<T, 64><<<grid, 256, 0, e->stream>>>(a);
    if (H == 128) pf_attn_kernel<T, 128><<<grid, 256, 0, e->stream>>>(a);
}

template <class T> void launch_pf_rows_t(asd_engine* e, int what, int rows, int n_chunks, int ksplit, const float* gain, float* cos_row, int tail_row) {
    const asd_config& c = e->c;
    using El = typename T::elem;
    const int64_t xb_plane = (int64_t)PF_CHUNKS * e->KBd * 64 * e->KE, xb_chunk = (int64_t)e->KBd * 64 * e->KE;
    const float inv_d = 1.f / (float)c.d_model;
    if (what == 0)
        pf_embed_kernel<T><<<n_chunks * 16, 256, 0, e->stream>>>((const El*)e->embed, e->pf_tok, rows, c.d_model, gain, e->pf_xres, e->pf_xb,
                                                                 xb_plane, xb_chunk, e->pf_ssq, e->pf_rscale, inv_d, c.rms_eps);
    else if (what == 1)
        pf_resid_kernel<T><<<rows, 256, 0, e->stream>>>(e->pf_raw, ksplit, c.d_model, e->pf_xres, e->pf_xb, xb_plane, xb_chunk, gain, e->pf_ssq,
                                                        e->pf_rscale, cos_row, inv_d, c.rms_eps);
    else
        pf_tail_kernel<T><<<1, 256, 0, e->stream>>>(e->pf_xres, e->pf_ssq, tail_row, c.d_model, e->g_final, e->xres, e->xb,
                                                    (int64_t)e->KBd * 64 * e->KE, e->part);
}
void launch_pf_rows(asd_engine* e, int what, int rows, int n_chunks, int ksplit, const float* gain, float* cos_row, int tail_row) {
    if (e->c.dtype == ASD_DT_BF16) launch_pf_rows_t<BF16>(e, what, rows, n_chunks, ksplit, gain, cos_row, tail_row);
    else launch_pf_rows_t<F32>(e, what, rows, n_chunks, ksplit, gain, cos_row, tail_row);
}

// The whole prompt, block by block and layer by layer; leaves the last row's logits / greedy token in row 0 of the
// decode buffers and the cosine sums of all rows in cos_acc (the caller cleared it).  Enqueue only.
int prefill_blocks(asd_engine* e, const int32_t* tokens, int n, Profiler* profiler = nullptr) {
    const asd_config& c = e->c;
    const int L = c.n_layers, KE = e->KE;
    const double qd = (double)c.n_heads * c.head_dim, kvd = (double)c.n_kv_heads * c.head_dim;
    Prof pr{profiler, e->stream};
    auto wl = [&](PfArgs& a, const GemmCfg& cfg, int total_tiles, int KB) {
        a.n_tiles = total_tiles; a.KB = KB; a.w_tile_stride = cfg.kmajor ? 1 : KB; a.w_kb_stride = cfg.kmajor ? total_tiles : 1;
    };
    int rows = 0;
    for (int r0 = 0; r0 < n; r0 += rows) {
        rows = n - r0 < PF_ROWS ? n - r0 : PF_ROWS;
        const int n_chunks = (rows + 15) / 16;
        CK(e, hipMemcpyAsync(e->pf_tok, tokens + r0, (size_t)rows * 4, hipMemcpyHostToDevice, e->stream));
        set_state_kernel<<<1, 1, 0, e->stream>>>(e->st, r0, 0, 0, 0);
        pr.begin(ASD_PK_ROWS, 0);
        launch_pf_rows(e, 0, rows, n_chunks, 1, e->layers[0].g_attn, nullptr, 0);
        pr.end();
        // flops of each contraction over this block's rows (every weight multiply-add counted once), causal attention
        const double fl_row = 2.0 * rows, ctx_sum = (double)rows * r0 + 0.5 * rows * (rows + 1.0);

        PfArgs base{};
        base.rows = rows; base.rscale = e->pf_rscale; base.raw = e->pf_raw;
        base.pos0 = r0; base.rope = e->rope; base.q = e->pf_q; base.page_table = e->page_table;
        base.q_plane = (int64_t)PF_CHUNKS * e->KBq * 64 * KE; base.q_chunk = (int64_t)e->KBq * 64 * KE;
        base.n_h = c.n_heads; base.n_kv = c.n_kv_heads; base.h = c.head_dim; base.page_tokens = c.page_tokens;
        base.hmid = e->pf_hmid; base.hmid_plane = (int64_t)PF_CHUNKS * e->KBf * 64 * KE; base.hmid_chunk = (int64_t)e->KBf * 64 * KE;
        for (int l = 0; l < L; ++l) {
            const Layer& ly = e->layers[l];
            bool ok = true;
            PfArgs a = base;
            a.W = (const u32x4*)ly.wqkv; a.X = (const u32x4*)e->pf_xb; a.x_plane = (int64_t)PF_CHUNKS * e->KBd * 64; a.x_chunk = (int64_t)e->KBd * 64;
            wl(a, e->g_qkv, e->qkv_tiles, e->KBd);
            a.kv = e->kv + (size_t)l * e->kv_layer_bytes;
            pr.begin(ASD_PK_QKV, fl_row * c.d_model * (qd + 2 * kvd));
            ok = ok && launch_pf_gemm<PF_QKV>(e, e->pf_qkv, a, n_chunks);
            pr.end();

            PfAttnArgs t{};
            t.q = e->pf_q; t.out = e->pf_attn_out; t.q_plane = base.q_plane; t.q_chunk = base.q_chunk; t.kv = a.kv;
            t.page_table = e->page_table; t.pos0 = r0; t.rows = rows;
            t.n_h = c.n_heads; t.n_kv = c.n_kv_heads; t.h = c.head_dim; t.page_tokens = c.page_tokens;
            t.scale = 1.f / sqrtf((float)c.head_dim);
            pr.begin(ASD_PK_ATTN, 4.0 * qd * ctx_sum);
            if (c.dtype == ASD_DT_BF16) launch_pf_attn_t<BF16>(e, t, n_chunks); else launch_pf_attn_t<F32>(e, t, n_chunks);
            pr.end();

            PfArgs o = base;
            o.W = (const u32x4*)ly.wo; o.X = (const u32x4*)e->pf_attn_out; o.x_plane = (int64_t)PF_CHUNKS * e->KBq * 64; o.x_chunk = (int64_t)e->KBq * 64;
            wl(o, e->g_o, c.d_model / 16, e->KBq);
            pr.begin(ASD_PK_OPROJ, fl_row * qd * c.d_model);
            ok = ok && launch_pf_gemm<PF_RAW>(e, e->pf_o, o, n_chunks);
            pr.end();
            pr.begin(ASD_PK_ROWS, 0);
            launch_pf_rows(e, 1, rows, n_chunks, e->pf_o.KS < e->KBq ? e->pf_o.KS : e->KBq, ly.g_mlp, e->pf_cos_rows + (size_t)(2 * l) * PF_ROWS, 0);
            pr.end();

            PfArgs gu = base;
            gu.W = (const u32x4*)ly.wg; gu.W2 = (const u32x4*)ly.wu; gu.X = (const u32x4*)e->pf_xb; gu.x_plane = a.x_plane; gu.x_chunk = a.x_chunk;
            wl(gu, e->g_gu, c.d_ffn / 16, e->KBd);
            pr.begin(ASD_PK_GATEUP, fl_row * 2.0 * c.d_model * c.d_ffn);
            ok = ok && launch_pf_gemm<PF_GU>(e, e->pf_gu, gu, n_chunks);
            pr.end();

            PfArgs dn = base;
            dn.W = (const u32x4*)ly.wd; dn.X = (const u32x4*)e->pf_hmid; dn.x_plane = (int64_t)PF_CHUNKS * e->KBf * 64; dn.x_chunk = (int64_t)e->KBf * 64;
            wl(dn, e->g_down, c.d_model / 16, e->KBf);
            pr.begin(ASD_PK_DOWN, fl_row * (double)c.d_model * c.d_ffn);
            ok = ok && launch_pf_gemm<PF_RAW>(e, e->pf_down, dn, n_chunks);
            pr.end();
            pr.begin(ASD_PK_ROWS, 0);
            launch_pf_rows(e, 1, rows, n_chunks, e->pf_down.KS < e->KBf ? e->pf_down.KS : e->KBf, l + 1 < L ? e->layers[l + 1].g_attn : e->g_final,
                           e->pf_cos_rows + (size_t)(2 * l + 1) * PF_ROWS, 0);
            pr.end();
            if (!ok) return fail(e, ASD_E_STATE, "no prompt GEMM instance for this launch shape");
        }
        pf_cos_sum_kernel<<<2 * L, 256, 0, e->stream>>>(e->pf_cos_rows, rows, e->cos_acc);
        e->kv_len = r0 + rows;
    }
    // the last prompt row through the final norm and the LM head, as row 0 of a one-row pass
    pr.begin(ASD_PK_LMHEAD, 2.0 * c.d_model * c.vocab);
    launch_pf_rows(e, 2, rows, 0, 1, nullptr, nullptr, rows - 1);
    std::vector<PassOp> ops;
    build_pass(e, 1, 0, nullptr, n, chunks_for(n - 1), engine_out(e), ops);
    for (PassOp& op : ops) {
        if (op.type != OP_LM) continue;
        op.g.part_in = e->part; op.g.P_in = 1; op.g.fin_cos_rows = nullptr; op.g.fin_cos_acc = nullptr;
        if (!launch_gemm<EPI_LM>(e, e->g_lm, op.g)) return fail(e, ASD_E_STATE, "no kernel instance for the LM head");
    }
    finish_kernel<<<1, 64, 0, e->stream>>>((const AmaxCand*)e->amax_part, e->g_lm.grid, 1, c.vocab, e->argmax, FIN_NONE, 0, e->st, e->tokbuf, e->out_tokens);
    pr.end();
    hipError_t r = hipGetLastError();
    if (r != hipSuccess) return fail(e, ASD_E_HIP, "kernel launch: %s", hipGetErrorString(r));
    return ASD_OK;
}

}  // namespace

// =================================================================== C ABI
extern "C" {

size_t asd_arena_bytes(const asd_config* cfg) {
    if (!config_ok(cfg, nullptr)) return 0;
    return make_plan(*cfg).total;
}

const char* asd_last_error(const asd_engine* e) { return e ? e->err.c_str() : g_create_error.c_str(); }

int asd_create(const asd_config* cfg, void* device_arena, size_t arena_bytes, void* hip_stream, asd_engine** out) {
    std::string why;
    if (!out) return fail(nullptr, ASD_E_INVAL, "out is NULL");
    if (!config_ok(cfg, &why)) return fail(nullptr, ASD_E_INVAL, "invalid configuration: %s", why.c_str());
    if (!device_arena) return fail(nullptr, ASD_E_INVAL, "device_arena is NULL");
    if ((uintptr_t)device_arena % 256) return fail(nullptr, ASD_E_INVAL, "device_arena must be 256-byte aligned");
    Plan p = make_plan(*cfg);
    if (arena_bytes < p.total)
        return fail(nullptr, ASD_E_NOMEM, "arena too small: %zu bytes given, %zu needed", arena_bytes, p.total);
    asd_engine* e = new (std::nothrow) asd_engine();
    if (!e) return fail(nullptr, ASD_E_NOMEM, "host allocation failed");
    e->c = *cfg; e->stream = (hipStream_t)hip_stream; e->arena = (char*)device_arena; e->arena_bytes = arena_bytes;
    e->es = p.es; e->KE = p.KE; e->KBd = p.KBd; e->KBq = p.KBq; e->KBf = p.KBf;
    e->n_pages = p.n_pages; e->nc_stride = p.nc_stride; e->qkv_tiles = p.qkv_tiles;
    char* A = e->arena;
    e->embed = A + p.embed; e->lm = A + p.lm; e->g_final = (float*)(A + p.g_final);
    e->layers.resize(cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l) {
        char* B = A + p.layer0 + p.layer_stride * l;
        e->layers[l] = Layer{B + p.wqkv, B + p.wo, B + p.wg, B + p.wu, B + p.wd, (float*)(B + p.g_attn), (float*)(B + p.g_mlp)};
    }
    e->have.assign(12 + (size_t)cfg->n_layers * 12, 1);
    for (int t = 0; t <= ASD_T_LM_HEAD; ++t) {
        if (tensor_is_global(t)) e->have[t] = 0;
        else for (int l = 0; l < cfg->n_layers; ++l) e->have[12 + l * 12 + t] = 0;
    }
    e->kv = A + p.kv; e->kv_layer_bytes = p.kv_layer; e->page_table = (int32_t*)(A + p.page_table);
    e->xres = (float*)(A + p.xres); e->ssq = (float*)(A + p.ssq); e->part = (float*)(A + p.part);
    e->cos_rows = (float*)(A + p.cos_rows); e->logits = (float*)(A + p.logits); e->qlogits = (float*)(A + p.qlogits); e->last_logits_row = 0; e->o_part = (float*)(A + p.o_part);
    e->rope = (float*)(A + p.rope); e->ml_part = (float*)(A + p.ml_part); e->arrivals = (unsigned*)(A + p.arrivals);
    e->xb = A + p.xb; e->q = A + p.q; e->attn_out = A + p.attn_out; e->hmid = A + p.hmid;
    e->counters = (unsigned*)(A + p.counters); e->cos_acc = (double*)(A + p.cos_acc);
    e->amax_part = (AmaxPart*)(A + p.amax_part); e->argmax = (int32_t*)(A + p.argmax);
    e->tokbuf = (int32_t*)(A + p.tokbuf); e->out_tokens = (int32_t*)(A + p.out_tokens); e->st = (DevState*)(A + p.st);
    e->staging = A + p.staging; e->staging_bytes = p.staging_bytes;
    e->pf_tok = (int32_t*)(A + p.pf_tok); e->pf_xres = (float*)(A + p.pf_xres); e->pf_raw = (float*)(A + p.pf_raw);
    e->pf_ssq = (float*)(A + p.pf_ssq); e->pf_rscale = (float*)(A + p.pf_rscale); e->pf_cos_rows = (float*)(A + p.pf_cos_rows);
    e->pf_xb = A + p.pf_xb; e->pf_q = A + p.pf_q; e->pf_attn_out = A + p.pf_attn_out; e->pf_hmid = A + p.pf_hmid;
    e->tune = cfg->debug_tune ? cfg->debug_tune : "";
    e->c.debug_tune = nullptr;              // (the caller's string is not kept; e->tune is the copy)
    const char* tune = e->tune.empty() ? nullptr : e->tune.c_str();
    e->pf_qkv = pf_pick(tune, "pf_qkv", 4, 1); e->pf_o = pf_pick(tune, "pf_o", 4, 4);
    e->pf_gu = pf_pick(tune, "pf_gu", 4, 1); e->pf_down = pf_pick(tune, "pf_down", 4, 4);
    e->g_qkv = p.g_qkv; e->g_o = p.g_o; e->g_gu = p.g_gu; e->g_down = p.g_down; e->g_lm = p.g_lm;
    e->g_qkv_rows = pick_qkv_rows(e->g_qkv, e->qkv_tiles, tune);
    e->att_gh1 = (cfg->debug_flags & ASD_DBG_ATT_GH1) != 0;
    e->sample_mem = (cfg->debug_flags & ASD_DBG_SAMPLE_MEM) != 0;
    e->force_att_w4 = (cfg->debug_flags & ASD_DBG_ATT_W4) != 0;
    e->rs_pow2 = (cfg->debug_flags & ASD_DBG_RS_POW2) != 0;
    e->kv_len = 0;
    e->acs.assign(2 * (size_t)cfg->n_layers, 0.f);
    e->acs_sum.assign(2 * (size_t)cfg->n_layers, 0.0);
    e->acs_rows = 0;
    e->acs_valid = false;
    e->h_st = nullptr;

    {   // the static scratch of asd_forward_noalloc: resolve this device's address now, not in the middle of a caller's loop
        const hipError_t rs = scratch_ptr(&e->scratch);
        if (rs != hipSuccess) { delete e; return fail(nullptr, ASD_E_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(rs)); }
    }
    hipError_t r = hipHostMalloc((void**)&e->h_st, sizeof(DevState), hipHostMallocDefault);
    if (r != hipSuccess) { delete e; return fail(nullptr, ASD_E_HIP, "hipHostMalloc: %s", hipGetErrorString(r)); }
    for (int i = 0; i < 3 && r == hipSuccess; ++i) r = hipEventCreate(&e->ev[i]);
    if (r != hipSuccess) { destroy_host(e); return fail(nullptr, ASD_E_HIP, "hipEventCreate: %s", hipGetErrorString(r)); }
    // clear cache + workspace (everything after the weights), then build the tables
    r = hipMemsetAsync(A + p.kv, 0, p.total - p.kv, e->stream);
    if (r == hipSuccess) {
        const size_t nrope = (size_t)capacity(e) * (cfg->head_dim / 2);
        rope_table_kernel<<<(unsigned)((nrope + 255) / 256), 256, 0, e->stream>>>(e->rope, capacity(e), cfg->head_dim / 2,
                                                                                  (double)cfg->rope_theta);
        iota_kernel<<<(e->n_pages + 255) / 256, 256, 0, e->stream>>>(e->page_table, e->n_pages);
        r = hipStreamSynchronize(e->stream);
    }
    if (r != hipSuccess) {
        destroy_host(e);
        return fail(nullptr, ASD_E_HIP, "engine initialisation: %s", hipGetErrorString(r));
    }
    *out = e;
    return ASD_OK;
}

void asd_destroy(asd_engine* e) {
    if (!e) return;
    hipStreamSynchronize(e->stream);
    destroy_host(e);
}

int asd_set_weight(asd_engine* e, int32_t t, int32_t layer, const void* src, size_t bytes, int32_t src_on_device) {
    if (!e) return ASD_E_INVAL;
    TensorInfo ti;
    if (!src || !tensor_info(e->c, t, &ti)) return fail(e, ASD_E_INVAL, "bad tensor id or NULL source");
    if (!tensor_is_global(t) && (layer < 0 || layer >= e->c.n_layers)) return fail(e, ASD_E_INVAL, "layer %d out of range", layer);
    const size_t need = (size_t)ti.rows * ti.cols * (ti.norm ? 4 : e->es);
    if (bytes != need) return fail(e, ASD_E_INVAL, "tensor %d needs %zu bytes, got %zu", t, need, bytes);
    const TensorLoc loc = tensor_loc(e, t, layer);
    char* dst = loc.base;
    const hipMemcpyKind kind = src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    if (!ti.tiled) {
        CK(e, hipMemcpyAsync(dst, src, bytes, kind, e->stream));
    } else {
        const void* dsrc = src;
        if (!src_on_device) {
            CK(e, hipMemcpyAsync(e->staging, src, bytes, hipMemcpyHostToDevice, e->stream));
            dsrc = e->staging;
        }
        if (e->c.dtype == ASD_DT_BF16) launch_tile<BF16>(e, dsrc, dst, ti.rows, ti.cols, loc.tm, false);
        else launch_tile<F32>(e, dsrc, dst, ti.rows, ti.cols, loc.tm, false);
    }
    CK(e, hipStreamSynchronize(e->stream));
    e->have[have_slot(e, t, layer)] = 1;
    return ASD_OK;
}

int asd_get_weight(asd_engine* e, int32_t t, int32_t layer, void* dst, size_t bytes) {
    if (!e) return ASD_E_INVAL;
    TensorInfo ti;
    if (!dst || !tensor_info(e->c, t, &ti)) return fail(e, ASD_E_INVAL, "bad tensor id or NULL destination");
    if (!tensor_is_global(t) && (layer < 0 || layer >= e->c.n_layers)) return fail(e, ASD_E_INVAL, "layer %d out of range", layer);
    const size_t need = (size_t)ti.rows * ti.cols * (ti.norm ? 4 : e->es);
    if (bytes != need) return fail(e, ASD_E_INVAL, "tensor %d has %zu bytes, buffer has %zu", t, need, bytes);
    if (!e->have[have_slot(e, t, layer)]) return fail(e, ASD_E_STATE, "tensor %d of layer %d was never set", t, layer);
    const TensorLoc loc = tensor_loc(e, t, layer);
    char* src = loc.base;
    if (ti.tiled) {
        if (e->c.dtype == ASD_DT_BF16) launch_tile<BF16>(e, src, e->staging, ti.rows, ti.cols, loc.tm, true);
        else launch_tile<F32>(e, src, e->staging, ti.rows, ti.cols, loc.tm, true);
        src = e->staging;
    }
    CK(e, hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, e->stream));
    CK(e, hipStreamSynchronize(e->stream));
    return ASD_OK;
}

extern "C++" {
static float widen(uint16_t v) { const uint32_t u = (uint32_t)v << 16; float f; memcpy(&f, &u, 4); return f; }    // bf16 code -> fp32
static float widen(float v) { return v; }
template <class T>
static void untile_kv(const asd_engine* e, const std::vector<char>& block, int slot, float* k_row, float* v_row) {
    using E = typename T::elem;
    const int H = e->c.head_dim, PT = e->c.page_tokens, nkv = e->c.n_kv_heads;
    for (int kvh = 0; kvh < nkv; ++kvh) {
        const E* B = (const E*)block.data() + (size_t)kvh * 2 * PT * H;
        for (int d = 0; d < H; ++d) {
            if (k_row) k_row[kvh * H + d] = widen(B[kv_k_off<T>(slot, d, H)]);
            if (v_row) v_row[kvh * H + d] = widen(B[kv_v_off<T>(slot, d, H)]);
        }
    }
}
}   // extern "C++"

int asd_get_kv(asd_engine* e, int32_t layer, int32_t pos0, int32_t n, float* k_out, float* v_out) {
    if (!e) return ASD_E_INVAL;
    if (layer < 0 || layer >= e->c.n_layers) return fail(e, ASD_E_INVAL, "layer %d out of range", layer);
    if (pos0 < 0 || n < 0 || pos0 + n > capacity(e)) return fail(e, ASD_E_INVAL, "positions %d .. %d outside the cache capacity %d", pos0, pos0 + n, capacity(e));
    const int H = e->c.head_dim, PT = e->c.page_tokens, nkv = e->c.n_kv_heads;
    const size_t row = (size_t)nkv * H, page_bytes = (size_t)nkv * 2 * PT * H * e->es;
    CK(e, hipStreamSynchronize(e->stream));
    std::vector<int32_t> table(e->n_pages);
    CK(e, hipMemcpy(table.data(), e->page_table, table.size() * 4, hipMemcpyDeviceToHost));
    std::vector<char> block(page_bytes);
    int have = -1;
    for (int i = 0; i < n; ++i) {
        const int pos = pos0 + i, lp = pos / PT;
        if (lp != have) {
            const int page = table[lp];
            if (page < 0 || page >= e->n_pages) return fail(e, ASD_E_STATE, "page table entry %d is %d", lp, page);
            CK(e, hipMemcpy(block.data(), e->kv + (size_t)layer * e->kv_layer_bytes + (size_t)page * page_bytes, page_bytes, hipMemcpyDeviceToHost));
            have = lp;
        }
        float* kr = k_out ? k_out + (size_t)i * row : nullptr;
        float* vr = v_out ? v_out + (size_t)i * row : nullptr;
        if (e->c.dtype == ASD_DT_BF16) untile_kv<BF16>(e, block, pos % PT, kr, vr); else untile_kv<F32>(e, block, pos % PT, kr, vr);
    }
    return ASD_OK;
}

// host copy of the input generator's stream key and constants (pure integer / one sqrt / one pow)
static uint64_t h_mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31; return z;
}
static uint64_t h_stream(uint64_t seed, uint32_t tensor, uint32_t layer) {
    return h_mix64(h_mix64(seed + 0x9E3779B97F4A7C15ULL) ^ (((uint64_t)tensor << 32) | layer));
}

int asd_init_synthetic(asd_engine* e, uint64_t seed) {
    if (!e) return ASD_E_INVAL;
    const asd_config& c = e->c;
    const uint64_t G = 0x9E3779B97F4A7C15ULL;
    auto cst = [](double std) { return (float)(std / (65536.0 * std::sqrt(8.0 / 12.0))); };
    auto scale = [&](int j) {
        const uint64_t r = h_mix64(h_stream(seed, 101u, 0u) + (uint64_t)(j + 1) * G);
        const double u = (double)(r >> 11) * (1.0 / 9007199254740992.0);
        return std::pow(10.0, -3.0 * u);
    };
    auto gen = [&](int t, int layer, double std) {
        TensorInfo ti; tensor_info(c, t, &ti);
        const TensorLoc loc = tensor_loc(e, t, layer);
        char* dst = loc.base;
        const uint64_t st = h_stream(seed, (uint32_t)t, (uint32_t)layer);
        const size_t frags = ti.tiled ? (size_t)(ti.rows / 16) * loc.tm.KB * 64 : ((size_t)ti.rows * ti.cols + e->KE - 1) / e->KE;
        const unsigned grid = (unsigned)((frags + 255) / 256);
        if (c.dtype == ASD_DT_BF16)
            synth_weight_kernel<BF16><<<grid, 256, 0, e->stream>>>((uint16_t*)dst, ti.rows, ti.cols, loc.tm, st, cst(std), ti.tiled);
        else
            synth_weight_kernel<F32><<<grid, 256, 0, e->stream>>>((float*)dst, ti.rows, ti.cols, loc.tm, st, cst(std), ti.tiled);
    };
    auto ones = [&](float* p) { fill_f32_kernel<<<(c.d_model + 255) / 256, 256, 0, e->stream>>>(p, c.d_model, 1.f); };
    gen(ASD_T_EMBED, 0, 0.02); gen(ASD_T_LM_HEAD, 0, 0.02); ones(e->g_final);
    for (int l = 0; l < c.n_layers; ++l) {
        gen(ASD_T_WQ, l, 0.02); gen(ASD_T_WK, l, 0.02); gen(ASD_T_WV, l, 0.02);
        gen(ASD_T_WO, l, 0.02 * scale(2 * l));
        gen(ASD_T_WG, l, 0.02); gen(ASD_T_WU, l, 0.02);
        gen(ASD_T_WD, l, 0.02 * scale(2 * l + 1));
        ones(e->layers[l].g_attn); ones(e->layers[l].g_mlp);
    }
    CK(e, hipGetLastError());
    CK(e, hipStreamSynchronize(e->stream));
    std::fill(e->have.begin(), e->have.end(), 1);
    return ASD_OK;
}

int asd_load_weights_file(asd_engine* e, const char* path) {
    if (!e) return ASD_E_INVAL;
    if (!path) return fail(e, ASD_E_INVAL, "path is NULL");
    FILE* f = fopen(path, "rb");
    if (!f) return fail(e, ASD_E_IO, "cannot open %s", path);
    char magic[8];
    int32_t hdr[8];
    const asd_config& c = e->c;
    const int32_t want[8] = {c.n_layers, c.d_model, c.n_heads, c.n_kv_heads, c.head_dim, c.d_ffn, c.vocab, c.dtype};
    if (fread(magic, 1, 8, f) != 8 || memcmp(magic, "ASDW0001", 8) || fread(hdr, 4, 8, f) != 8) {
        fclose(f); return fail(e, ASD_E_IO, "%s: bad header", path);
    }
    if (memcmp(hdr, want, sizeof want)) { fclose(f); return fail(e, ASD_E_INVAL, "%s: shape differs from the engine's", path); }
    std::vector<char> buf;
    auto one = [&](int t, int layer) -> int {
        TensorInfo ti; tensor_info(c, t, &ti);
        const size_t bytes = (size_t)ti.rows * ti.cols * (ti.norm ? 4 : e->es);
        buf.resize(bytes);
        if (fread(buf.data(), 1, bytes, f) != bytes) return fail(e, ASD_E_IO, "%s: file too short", path);
        return asd_set_weight(e, t, layer, buf.data(), bytes, 0);
    };
    int rc = ASD_OK;
    const int gl[3] = {ASD_T_EMBED, ASD_T_FINAL_NORM, ASD_T_LM_HEAD};
    const int ly[9] = {ASD_T_ATTN_NORM, ASD_T_WQ, ASD_T_WK, ASD_T_WV, ASD_T_WO, ASD_T_MLP_NORM, ASD_T_WG, ASD_T_WU, ASD_T_WD};
    for (int i = 0; i < 3 && rc == ASD_OK; ++i) rc = one(gl[i], 0);
    for (int l = 0; l < c.n_layers && rc == ASD_OK; ++l)
        for (int i = 0; i < 9 && rc == ASD_OK; ++i) rc = one(ly[i], l);
    fclose(f);
    return rc;
}

int asd_set_page_table(asd_engine* e, const int32_t* table, int32_t n_pages) {
    if (!e) return ASD_E_INVAL;
    if (!table || n_pages != e->n_pages) return fail(e, ASD_E_INVAL, "page table must have %d entries", e->n_pages);
    if (e->kv_len != 0) return fail(e, ASD_E_STATE, "page table can only change while the cache is empty");
    std::vector<uint8_t> seen(n_pages, 0);
    for (int i = 0; i < n_pages; ++i) {
        if (table[i] < 0 || table[i] >= n_pages || seen[table[i]]) return fail(e, ASD_E_INVAL, "page table is not a permutation");
        seen[table[i]] = 1;
    }
    CK(e, hipMemcpyAsync(e->page_table, table, (size_t)n_pages * 4, hipMemcpyHostToDevice, e->stream));
    CK(e, hipStreamSynchronize(e->stream));
    drop_graphs(e);
    return ASD_OK;
}

int asd_reset(asd_engine* e) { if (!e) return ASD_E_INVAL; e->kv_len = 0; return ASD_OK; }
int asd_truncate(asd_engine* e, int32_t n) {
    if (!e) return ASD_E_INVAL;
    if (n < 0 || n > e->kv_len) return fail(e, ASD_E_INVAL, "truncate to %d outside [0, %d]", n, e->kv_len);
    e->kv_len = n; return ASD_OK;
}
int32_t asd_kv_len(const asd_engine* e) { return e ? e->kv_len : ASD_E_INVAL; }

int asd_admg2(const float* C2, int32_t L, float alpha, int32_t m, int32_t n, int32_t use_cs, float alpha_mlp, int32_t use_cs_mlp,
              uint8_t* mask) {
    if (!C2 || !mask || L < 1 || m < 0 || n < 0) return ASD_E_INVAL;
    if (use_cs && !(alpha > 0.f && alpha < 1.f)) return ASD_E_INVAL;
    if (use_cs_mlp && !(alpha_mlp > 0.f && alpha_mlp < 1.f)) return ASD_E_INVAL;
    for (int i = 0; i < L; ++i) {
        const bool free_to_go = i < L - n;                       // rule 2 keeps the last n layers
        const bool periodic = m > 0 && (i + 1) % m == 0;         // rule 1, layers counted from 1
        const bool similar = use_cs && C2[2 * i] >= alpha;       // CS thresholding
        const bool similar_mlp = use_cs_mlp && C2[2 * i + 1] >= alpha_mlp;
        mask[2 * i + 1] = free_to_go && (periodic || similar_mlp);
        mask[2 * i] = free_to_go && (similar || periodic);
    }
    return ASD_OK;
}

int asd_admg(const float* C, int32_t L, float alpha, int32_t m, int32_t n, int32_t use_cs, uint8_t* mask) {
    if (!C || L < 1) return ASD_E_INVAL;
    std::vector<float> c2(2 * (size_t)L, 0.f);
    for (int i = 0; i < L; ++i) c2[2 * i] = C[i];
    return asd_admg2(c2.data(), L, alpha, m, n, use_cs, 0.f, 0, mask);
}

// run rows [tokens, tokens+n) at the current cache end; results stay on the device
static int forward_rows(asd_engine* e, const int32_t* tokens, int n, const uint8_t* mask, Profiler* prof) {
    CK(e, hipMemcpyAsync(e->tokbuf, tokens, (size_t)n * 4, hipMemcpyHostToDevice, e->stream));
    set_state_kernel<<<1, 1, 0, e->stream>>>(e->st, e->kv_len, 0, 0, 0);
    return enqueue_forward(e, e->tokbuf, n, 0, mask, chunks_for(e->kv_len + n - 1), prof, e->kv_len + n);
}

int asd_forward(asd_engine* e, const int32_t* tokens, int32_t n_rows, int32_t pos0, const uint8_t* mask, int32_t commit,
                float* logits, float* cos, float* cos_rows, int32_t* argmax) {
    if (!e) return ASD_E_INVAL;
    if (!tokens) return fail(e, ASD_E_INVAL, "tokens is NULL");
    if (n_rows < 1 || n_rows > e->c.max_rows) return fail(e, ASD_E_INVAL, "n_rows %d outside [1, %d]", n_rows, e->c.max_rows);
    if (!weights_ready(e)) return fail(e, ASD_E_STATE, "weights are not fully loaded");
    if (pos0 != e->kv_len) return fail(e, ASD_E_STATE, "pos0 %d differs from the cache length %d", pos0, e->kv_len);
    if (pos0 + n_rows > capacity(e)) return fail(e, ASD_E_INVAL, "position %d exceeds the cache capacity %d", pos0 + n_rows, capacity(e));
    int rc = check_tokens(e, tokens, n_rows);
    if (rc) return rc;
    const int L2 = 2 * e->c.n_layers;
    CK(e, hipMemsetAsync(e->cos_acc, 0, (size_t)L2 * 8, e->stream));
    rc = forward_rows(e, tokens, n_rows, mask, nullptr);
    if (rc) return rc;
    std::vector<double> acc(L2);
    std::vector<float> rows((size_t)L2 * ASD_ROWS);
    std::vector<int32_t> am(ASD_ROWS);
    std::vector<float> lg;
    CK(e, hipMemcpyAsync(acc.data(), e->cos_acc, (size_t)L2 * 8, hipMemcpyDeviceToHost, e->stream));
    CK(e, hipMemcpyAsync(rows.data(), e->cos_rows, rows.size() * 4, hipMemcpyDeviceToHost, e->stream));
    CK(e, hipMemcpyAsync(am.data(), e->argmax, ASD_ROWS * 4, hipMemcpyDeviceToHost, e->stream));
    if (logits) {
        lg.resize((size_t)n_rows * e->c.vocab);
        CK(e, hipMemcpyAsync(lg.data(), e->logits, lg.size() * 4, hipMemcpyDeviceToHost, e->stream));
    }
    CK(e, hipStreamSynchronize(e->stream));
    rc = check_pass_error(e);
    if (rc) return rc;
    if (logits) memcpy(logits, lg.data(), lg.size() * 4);
    for (int j = 0; j < L2; ++j) {
        const bool skipped = mask && mask[j];
        if (cos) cos[j] = skipped ? 1.f : (float)(acc[j] / n_rows);
        if (cos_rows) for (int r = 0; r < n_rows; ++r) cos_rows[(size_t)r * L2 + j] = skipped ? 1.f : rows[(size_t)j * ASD_ROWS + r];
    }
    if (argmax) memcpy(argmax, am.data(), (size_t)n_rows * 4);
    if (commit) e->kv_len = pos0 + n_rows;
    return ASD_OK;
}

// The static scratch laid out for a pass of an engine's shape over a context of `groups` attention groups per head.
// Returns the bytes needed (the layout is valid when they fit ASD_SCRATCH_BYTES).
static size_t scratch_layout(const asd_engine* e, int groups, unsigned char* base, PassOut* o) {
    const asd_config& c = e->c;
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char* p = base + off; off = align_up(off + bytes); return p; };
    int pmax = e->g_o.grid > e->g_down.grid ? e->g_o.grid : e->g_down.grid;
    if (pmax < EMBED_SPLIT) pmax = EMBED_SPLIT;
    o->ssq = (float*)take(ASD_ROWS * 4);
    o->part = (float*)take((size_t)pmax * ASD_ROWS * 2 * 4);
    o->cos_rows = (float*)take((size_t)2 * c.n_layers * ASD_ROWS * 4);
    o->cos_acc = (double*)take((size_t)2 * c.n_layers * 8);
    o->arrivals = (unsigned*)take((size_t)c.n_heads * 4);
    o->amax_part = (AmaxPart*)take((size_t)e->g_lm.grid * ASD_ROWS * sizeof(AmaxPart));
    o->argmax = (int32_t*)take(ASD_ROWS * 4);
    o->ml_part = (float*)take((size_t)c.n_heads * groups * ASD_ROWS * 8);
    o->o_part = (float*)take((size_t)c.n_heads * groups * ASD_ROWS * c.head_dim * 4);
    o->nc_stride = groups;
    return off;
}

int asd_forward_noalloc(asd_engine* e, const int32_t* d_tokens, int32_t n_rows, int32_t pos0, const uint8_t* mask, int32_t commit,
                        float* d_logits, float* d_cos, int32_t* d_argmax) {
    if (!e) return ASD_E_INVAL;
    if (!d_tokens) return fail(e, ASD_E_INVAL, "d_tokens is NULL");
    if (n_rows < 1 || n_rows > e->c.max_rows) return fail(e, ASD_E_INVAL, "n_rows %d outside [1, %d]", n_rows, e->c.max_rows);
    if (!weights_ready(e)) return fail(e, ASD_E_STATE, "weights are not fully loaded");
    if (pos0 != e->kv_len) return fail(e, ASD_E_STATE, "pos0 %d differs from the cache length %d", pos0, e->kv_len);
    if (pos0 + n_rows > capacity(e)) return fail(e, ASD_E_INVAL, "position %d exceeds the cache capacity %d", pos0 + n_rows, capacity(e));
    const int L2 = 2 * e->c.n_layers;
    const int groups = (pos0 + n_rows + ATT_GROUP - 1) / ATT_GROUP;
    PassOut out{};
    const size_t need = scratch_layout(e, groups, e->scratch, &out);
    if (need > ASD_SCRATCH_BYTES)
        return fail(e, ASD_E_NOMEM, "a pass of this shape over %d positions needs %zu bytes of scratch, the static array holds %u",
                    pos0 + n_rows, need, (unsigned)ASD_SCRATCH_BYTES);
    out.logits = d_logits ? d_logits : e->logits;
    if (d_argmax) out.argmax = d_argmax;
    // what must start at zero: the running cosine sums and the heads' arrival counters (neighbours in the layout)
    const int nz = (int)(((unsigned char*)out.amax_part - (unsigned char*)out.cos_acc) / 4);
    zero_words_kernel<<<(nz + 255) / 256, 256, 0, e->stream>>>((uint32_t*)out.cos_acc, nz);
    set_state_kernel<<<1, 1, 0, e->stream>>>(e->st, e->kv_len, 0, 0, 0);
    const int rc = enqueue_forward(e, d_tokens, n_rows, 0, mask, chunks_for(e->kv_len + n_rows - 1), nullptr, e->kv_len + n_rows, FIN_NONE, 0, &out);
    if (rc) return rc;
    if (d_cos) {
        MaskBits mb{};
        for (int j = 0; j < L2; ++j) if (mask && mask[j]) mb.w[j >> 5] |= 1u << (j & 31);
        cos_mean_kernel<<<(L2 + 255) / 256, 256, 0, e->stream>>>(out.cos_acc, L2, n_rows, mb, d_cos);
    }
    const hipError_t r = hipGetLastError();
    if (r != hipSuccess) return fail(e, ASD_E_HIP, "kernel launch: %s", hipGetErrorString(r));
    if (commit) e->kv_len = pos0 + n_rows;
    return ASD_OK;
}

int asd_check(asd_engine* e) {
    if (!e) return ASD_E_INVAL;
    CK(e, hipStreamSynchronize(e->stream));
    return check_pass_error(e);
}

static int prefill_impl(asd_engine* e, const int32_t* tokens, int32_t n, int32_t* first_token, float* cos_out, float* last_logits, bool blocks) {
    if (!e) return ASD_E_INVAL;
    if (!tokens || !first_token) return fail(e, ASD_E_INVAL, "tokens or first_token is NULL");
    if (n < 1 || n > capacity(e)) return fail(e, ASD_E_INVAL, "prompt length %d outside [1, %d]", n, capacity(e));
    if (!weights_ready(e)) return fail(e, ASD_E_STATE, "weights are not fully loaded");
    int rc = check_tokens(e, tokens, n);
    if (rc) return rc;
    const int L2 = 2 * e->c.n_layers;
    e->kv_len = 0; e->acs_valid = false;
    CK(e, hipMemsetAsync(e->cos_acc, 0, (size_t)L2 * 8, e->stream));
    int last_row = 0;
    if (blocks) {
        rc = prefill_blocks(e, tokens, n);
        if (rc) return rc;
    } else {
        int rows = 0;
        for (int p = 0; p < n; p += rows) {
            rows = n - p < e->c.max_rows ? n - p : e->c.max_rows;
            rc = forward_rows(e, tokens + p, rows, nullptr, nullptr);
            if (rc) return rc;
            e->kv_len = p + rows;
        }
        last_row = rows - 1;
    }
    e->last_logits_row = last_row;
    std::vector<double> acc(L2);
    int32_t am[ASD_ROWS];
    CK(e, hipMemcpyAsync(acc.data(), e->cos_acc, (size_t)L2 * 8, hipMemcpyDeviceToHost, e->stream));
    CK(e, hipMemcpyAsync(am, e->argmax, ASD_ROWS * 4, hipMemcpyDeviceToHost, e->stream));
    std::vector<float> lg;
    if (last_logits) {
        lg.resize(e->c.vocab);
        CK(e, hipMemcpyAsync(lg.data(), e->logits + (size_t)last_row * e->c.vocab, lg.size() * 4, hipMemcpyDeviceToHost, e->stream));
    }
    CK(e, hipStreamSynchronize(e->stream));
    rc = check_pass_error(e);
    if (rc) return rc;
    for (int j = 0; j < L2; ++j) { e->acs[j] = (float)(acc[j] / n); e->acs_sum[j] = acc[j]; }
    e->acs_rows = n;
    e->acs_valid = true;
    if (cos_out) memcpy(cos_out, e->acs.data(), (size_t)L2 * 4);
    if (last_logits) memcpy(last_logits, lg.data(), lg.size() * 4);
    *first_token = am[last_row];
    return ASD_OK;
}

int asd_prefill(asd_engine* e, const int32_t* tokens, int32_t n, int32_t* first_token, float* cos_out, float* last_logits) {
    return prefill_impl(e, tokens, n, first_token, cos_out, last_logits, e && n > e->c.max_rows);
}

int asd_prefill_chunked(asd_engine* e, const int32_t* tokens, int32_t n, int32_t* first_token, float* cos_out, float* last_logits) {
    return prefill_impl(e, tokens, n, first_token, cos_out, last_logits, false);
}

// one draft/verify/accept cycle, enqueue only: kk draft steps with the masked model, then a (kk+1)-row verify
#define DECODE_BURST 16      // draft-free decode cycles enqueued between two looks at the device state

static int enqueue_drafts(asd_engine* e, int kk, const uint8_t* mask, int nc, int32_t ctx) {
    for (int j = 0; j < kk; ++j) {
        int rc = enqueue_forward(e, e->tokbuf + j, 1, j, mask, nc, nullptr, ctx, FIN_DRAFT, j);
        if (rc) return rc;
    }
    return ASD_OK;
}
static int enqueue_verify(asd_engine* e, int kk, int nc, int32_t ctx) {
    return enqueue_forward(e, e->tokbuf, kk + 1, 0, nullptr, nc, nullptr, ctx, FIN_ACCEPT, kk);
}

// sampling stream key: the synthetic-input generator's stream derivation for tensor id 102
static SampleArgs sample_args(asd_engine* e, float temperature, uint64_t seed) {
    SampleArgs a{};
    a.logits = e->logits; a.qlogits = e->qlogits; a.V = e->c.vocab; a.inv_T = 1.f / temperature;
    a.qstat = (double*)(e->qlogits + (size_t)ASD_ROWS * e->c.vocab);
    a.stream = h_stream(seed, 102u, 0u);
    a.st = e->st; a.tokbuf = e->tokbuf; a.out = e->out_tokens;
    return a;
}

// The sampling kernels hold a thread's share of a logit row in registers when the vocabulary allows it
// (ASD_DBG_SAMPLE_MEM, a test aid, forces the variant that re-reads memory: same arithmetic, same draws).
static bool sample_in_registers(const asd_engine* e) {
    return !e->sample_mem && e->c.vocab <= SAMPLE_SEG * SAMPLE_THREADS;
}
static void launch_sample_draft(asd_engine* e, const SampleArgs& sa, int j) {
    if (sample_in_registers(e)) sample_draft_kernel<SAMPLE_SEG><<<1, SAMPLE_THREADS, 0, e->stream>>>(sa, j);
    else sample_draft_kernel<0><<<1, SAMPLE_THREADS, 0, e->stream>>>(sa, j);
}
static void launch_sample_accept(asd_engine* e, const SampleArgs& sa, int kk) {
    if (sample_in_registers(e)) sample_accept_kernel<SAMPLE_SEG><<<1, SAMPLE_THREADS, 0, e->stream>>>(sa, kk);
    else sample_accept_kernel<0><<<1, SAMPLE_THREADS, 0, e->stream>>>(sa, kk);
}
static void launch_sample_plain(asd_engine* e, const SampleArgs& sa, int row, int64_t index) {
    if (sample_in_registers(e)) sample_plain_kernel<SAMPLE_SEG><<<1, SAMPLE_THREADS, 0, e->stream>>>(sa, row, index);
    else sample_plain_kernel<0><<<1, SAMPLE_THREADS, 0, e->stream>>>(sa, row, index);
}

// one sampled draft / verify / accept cycle, enqueue only
static int enqueue_sampled_drafts(asd_engine* e, int kk, const uint8_t* mask, int nc, int32_t ctx, const SampleArgs& sa) {
    for (int j = 0; j < kk; ++j) {
        int rc = enqueue_forward(e, e->tokbuf + j, 1, j, mask, nc, nullptr, ctx, FIN_NONE, 0);
        if (rc) return rc;
        launch_sample_draft(e, sa, j);
    }
    return ASD_OK;
}
static int enqueue_sampled_verify(asd_engine* e, int kk, int nc, int32_t ctx, const SampleArgs& sa) {
    int rc = enqueue_forward(e, e->tokbuf, kk + 1, 0, nullptr, nc, nullptr, ctx, FIN_NONE, 0);
    if (rc) return rc;
    launch_sample_accept(e, sa, kk);
    return ASD_OK;
}

int asd_spec_sample(asd_engine* e, const float* q_logits, const float* p_logits, int32_t kk, float temperature, uint64_t seed,
                    int64_t index0, int32_t* drafts_out, int32_t* n_accepted, int32_t* next_token) {
    if (!e) return ASD_E_INVAL;
    if (!p_logits || !n_accepted || !next_token || (kk > 0 && (!q_logits || !drafts_out)))
        return fail(e, ASD_E_INVAL, "NULL argument");
    if (kk < 0 || kk + 1 > e->c.max_rows) return fail(e, ASD_E_INVAL, "kk %d outside [0, %d]", kk, e->c.max_rows - 1);
    if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(e, ASD_E_INVAL, "temperature must be positive and finite");
    if (index0 < 0 || index0 > (1 << 30)) return fail(e, ASD_E_INVAL, "index0 out of range");
    const size_t V = e->c.vocab;
    const SampleArgs sa = sample_args(e, temperature, seed);
    set_state_kernel<<<1, 1, 0, e->stream>>>(e->st, e->kv_len, 0, kk + 1, 1, (int)index0);
    for (int j = 0; j < kk; ++j) {                 // each draft row takes the place a draft step's logits would have
        CK(e, hipMemcpyAsync(e->logits, q_logits + (size_t)j * V, V * 4, hipMemcpyHostToDevice, e->stream));
        launch_sample_draft(e, sa, j);
    }
    CK(e, hipMemcpyAsync(e->logits, p_logits, (size_t)(kk + 1) * V * 4, hipMemcpyHostToDevice, e->stream));
    launch_sample_accept(e, sa, kk);
    int32_t tb[ASD_ROWS + 1];
    CK(e, hipMemcpyAsync(tb, e->tokbuf, sizeof tb, hipMemcpyDeviceToHost, e->stream));
    CK(e, hipMemcpyAsync(e->h_st, e->st, sizeof(DevState), hipMemcpyDeviceToHost, e->stream));
    int32_t drafts[ASD_ROWS];
    // the accept step overwrote tokbuf[0] with the next token; the drafts are still in rows 1..kk
    CK(e, hipStreamSynchronize(e->stream));
    for (int j = 0; j < kk; ++j) drafts[j] = tb[j + 1];
    if (kk > 0) memcpy(drafts_out, drafts, (size_t)kk * 4);
    *n_accepted = e->h_st->accepted;
    *next_token = tb[0];
    return ASD_OK;
}

// Run `enqueue` on the engine's stream: eagerly, or (use_graphs) as a HIP graph captured once per key.
static int run_captured(asd_engine* e, bool use_graphs, const std::vector<int>& key, const std::function<int()>& enqueue) {
    if (!use_graphs) return enqueue();
    auto it = e->graphs.find(key);
    if (it == e->graphs.end()) {
        hipGraph_t g = nullptr;
        hipGraphExec_t ge = nullptr;
        CK(e, hipStreamBeginCapture(e->stream, hipStreamCaptureModeThreadLocal));
        const int rc = enqueue();
        hipError_t r2 = hipStreamEndCapture(e->stream, &g);
        if (rc) { if (g) hipGraphDestroy(g); return rc; }
        if (r2 != hipSuccess) return fail(e, ASD_E_HIP, "hipStreamEndCapture: %s", hipGetErrorString(r2));
        r2 = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
        hipGraphDestroy(g);
        if (r2 != hipSuccess) return fail(e, ASD_E_HIP, "hipGraphInstantiate: %s", hipGetErrorString(r2));
        it = e->graphs.emplace(key, ge).first;
    }
    CK(e, hipGraphLaunch(it->second, e->stream));
    return ASD_OK;
}

static int check_gen_params(asd_engine* e, const asd_gen_params* p) {
    if (p->mask_mode < 0 || p->mask_mode > 2) return fail(e, ASD_E_INVAL, "mask_mode must be 0, 1 or 2");
    if (p->mask_mode == 1 && !p->fixed_mask) return fail(e, ASD_E_INVAL, "mask_mode 1 needs fixed_mask");
    if (p->exit_mode != 0 && p->exit_mode != 1) return fail(e, ASD_E_INVAL, "exit_mode must be 0 or 1");
    if (p->exit_mode == 1) {
        const bool ok = p->beta1 >= 0.0 && p->beta1 <= 1.0 && p->beta2 >= 0.0 && p->beta2 <= 1.0 && p->eps >= 0.0 && std::isfinite(p->eps) &&
                        std::isfinite(p->gamma0) && std::isfinite(p->ar0) && std::isfinite(p->ar_target);
        if (!ok) return fail(e, ASD_E_INVAL, "adaptive draft exit: beta1, beta2 in [0, 1], eps >= 0, finite gamma0 / ar0 / ar_target");
    }
    if (p->temperature != 0.f) {
        if (!(p->temperature > 0.f) || !std::isfinite(p->temperature)) return fail(e, ASD_E_INVAL, "temperature must be >= 0 and finite");
        if (p->exit_mode != 0) return fail(e, ASD_E_INVAL, "the adaptive draft exit is available for greedy decoding only");
        if (p->sample_index0 < 0 || p->sample_index0 > (1 << 30)) return fail(e, ASD_E_INVAL, "sample_index0 out of range");
    }
    return ASD_OK;
}

int asd_decode(asd_engine* e, int32_t last_token, int32_t n_more, const asd_gen_params* p, int32_t* out, asd_gen_stats* stats,
               uint8_t* mask_used) {
    if (!e) return ASD_E_INVAL;
    if (!p || !out) return fail(e, ASD_E_INVAL, "params or out_tokens is NULL");
    if (n_more < 1) return fail(e, ASD_E_INVAL, "n_more must be >= 1");
    const int k = p->draft_len, L = e->c.n_layers, L2 = 2 * L;
    if (k < 0 || k + 1 > e->c.max_rows) return fail(e, ASD_E_INVAL, "draft_len %d outside [0, %d]", k, e->c.max_rows - 1);
    if (last_token < 0 || last_token >= e->c.vocab) return fail(e, ASD_E_INVAL, "last_token outside the vocabulary");
    if (!weights_ready(e)) return fail(e, ASD_E_STATE, "weights are not fully loaded");
    if (e->kv_len + n_more + k > capacity(e))
        return fail(e, ASD_E_INVAL, "cache capacity %d too small for %d + %d + %d positions", capacity(e), e->kv_len, n_more, k);
    int rc = check_gen_params(e, p);
    if (rc) return rc;
    std::vector<uint8_t> mask(L2, 0), mnew(L2, 0);
    const bool refresh = p->mask_mode == 2;
    std::vector<double> S;              // running sums of row cosines (mask refresh)
    std::vector<float> C(L2), cr;
    long n_rows = 0;
    if (p->mask_mode == 1) {
        for (int j = 0; j < L2; ++j) mask[j] = p->fixed_mask[j] ? 1 : 0;
    } else {
        if (!e->acs_valid) return fail(e, ASD_E_STATE, "mask_mode 0 / 2 needs the ACS of a preceding asd_prefill");
        if (asd_admg2(e->acs.data(), L, p->alpha, p->m, p->n, p->use_cs, p->alpha_mlp, p->use_cs_mlp, mask.data()))
            return fail(e, ASD_E_INVAL, "invalid ADMG parameters (thresholds in (0,1), m >= 0, n >= 0)");
        if (refresh) { S = e->acs_sum; n_rows = e->acs_rows; cr.resize((size_t)L2 * ASD_ROWS); }
    }
    if (mask != e->graph_mask) { drop_graphs(e); e->graph_mask = mask; }

    const auto t0 = std::chrono::steady_clock::now();
    const bool sampled = p->temperature > 0.f;
    const SampleArgs sa = sampled ? sample_args(e, p->temperature, p->seed) : SampleArgs{};
    set_state_kernel<<<1, 1, 0, e->stream>>>(e->st, e->kv_len, 0, n_more, 1, sampled ? (int)p->sample_index0 : 0);
    set_token_kernel<<<1, 1, 0, e->stream>>>(e->tokbuf, last_token);
    const bool graphs = p->use_graphs != 0;
    if (sampled && (e->graph_T != p->temperature || e->graph_seed != p->seed)) {        // both are baked into captured launches
        drop_graphs(e); e->graph_T = p->temperature; e->graph_seed = p->seed;
    }
    double gamma = p->gamma0, ar = p->ar0;
    long mask_changes = 0;
    int emitted = 0, accepted = 0;
    // Without drafts (and without a mask refresh) the host has nothing to decide between cycles: each one emits one
    // token and advances the cache by one, so cycles are enqueued DECODE_BURST at a time behind one another and the
    // host looks at the device state once per burst instead of once per token.
    const bool lockstep = k == 0 && !refresh;
    // phase accounting: GPU time between the stamps of every cycle, algorithmic bytes of its passes
    double ms_draft = 0.0, ms_verify = 0.0, bytes_draft = 0.0, bytes_verify = 0.0;
    auto add_bytes = [&](double& acc, const uint8_t* m, int ctx) {
        double cls[ASD_K_COUNT];
        pass_bytes(e, m, ctx, cls);
        for (int i = 0; i < ASD_K_COUNT; ++i) acc += cls[i];
    };
    while (emitted < n_more) {
        const int burst = lockstep ? (n_more - emitted < DECODE_BURST ? n_more - emitted : DECODE_BURST) : 1;
        CK(e, hipEventRecord(e->ev[0], e->stream));
        for (int b = 0; b + 1 < burst; ++b) {
            const int nc = chunks_for(e->kv_len + b), ctx = e->kv_len + b + 1;
            rc = sampled ? run_captured(e, graphs, {3, 0, nc}, [&] { return enqueue_sampled_verify(e, 0, nc, ctx, sa); })
                         : run_captured(e, graphs, {0, 0, nc}, [&] { return enqueue_verify(e, 0, nc, ctx); });
            if (rc) return rc;
            add_bytes(bytes_verify, nullptr, ctx);
        }
        const int ahead = burst - 1;                 // cycles already enqueued in this trip
        const int kk = k < n_more - emitted - 1 ? k : n_more - emitted - 1;
        const int nc = chunks_for(e->kv_len + ahead + kk), ctx = e->kv_len + ahead + kk + 1;
        int d = kk;
        if (sampled) {
            if (kk > 0) rc = run_captured(e, graphs, {4, kk, nc}, [&] { return enqueue_sampled_drafts(e, kk, mask.data(), nc, ctx, sa); });
            if (rc) return rc;
            CK(e, hipEventRecord(e->ev[1], e->stream));
            rc = run_captured(e, graphs, {3, kk, nc}, [&] { return enqueue_sampled_verify(e, kk, nc, ctx, sa); });
            if (rc) return rc;
        } else if (p->exit_mode == 0) {
            if (kk > 0) rc = run_captured(e, graphs, {5, kk, nc}, [&] { return enqueue_drafts(e, kk, mask.data(), nc, ctx); });
            if (rc) return rc;
            CK(e, hipEventRecord(e->ev[1], e->stream));
            rc = run_captured(e, graphs, {0, kk, nc}, [&] { return enqueue_verify(e, kk, nc, ctx); });
            if (rc) return rc;
        } else {
            // draft until the limit or a low-confidence draft; the host reads the confidence after every step
            d = 0;
            while (d < kk) {
                rc = run_captured(e, graphs, {1, d, nc},
                                  [&] { return enqueue_forward(e, e->tokbuf + d, 1, d, mask.data(), nc, nullptr, ctx, FIN_DRAFT, d); });
                if (rc) return rc;
                ++d;
                CK(e, hipMemcpyAsync(e->h_st, e->st, sizeof(DevState), hipMemcpyDeviceToHost, e->stream));
                CK(e, hipStreamSynchronize(e->stream));
                if ((double)e->h_st->conf < gamma) break;
            }
            CK(e, hipEventRecord(e->ev[1], e->stream));
            rc = run_captured(e, graphs, {2, d, nc},
                              [&] { return enqueue_forward(e, e->tokbuf, d + 1, 0, nullptr, nc, nullptr, ctx, FIN_ACCEPT, d); });
            if (rc) return rc;
        }
        CK(e, hipEventRecord(e->ev[2], e->stream));
        for (int j = 0; j < d; ++j) add_bytes(bytes_draft, mask.data(), e->kv_len + ahead + j + 1);
        add_bytes(bytes_verify, nullptr, e->kv_len + ahead + d + 1);
        CK(e, hipMemcpyAsync(e->h_st, e->st, sizeof(DevState), hipMemcpyDeviceToHost, e->stream));
        if (refresh) CK(e, hipMemcpyAsync(cr.data(), e->cos_rows, cr.size() * 4, hipMemcpyDeviceToHost, e->stream));
        CK(e, hipStreamSynchronize(e->stream));
        {
            float t_d = 0.f, t_v = 0.f;
            CK(e, hipEventElapsedTime(&t_d, e->ev[0], e->ev[1]));
            CK(e, hipEventElapsedTime(&t_v, e->ev[1], e->ev[2]));
            if (lockstep) ms_verify += (double)t_d + t_v; else { ms_draft += t_d; ms_verify += t_v; }
        }
        if (e->h_st->err) { const int rce = check_pass_error(e, e->h_st); if (rce) return rce; }
        if (e->h_st->emitted <= emitted || (lockstep && e->h_st->emitted != emitted + burst)) {
            const int rce = check_pass_error(e, e->h_st);
            return rce ? rce : fail(e, ASD_E_STATE, "decode cycle made no progress");
        }
        const int a = e->h_st->accepted - accepted;
        accepted = e->h_st->accepted;
        emitted = e->h_st->emitted;
        e->kv_len = e->h_st->pos;
        if (p->exit_mode == 1 && d > 0) {
            ar = p->beta1 * ar + (1.0 - p->beta1) * ((double)a / (double)d);
            const double gt = ar <= p->ar_target ? gamma + p->eps : gamma - p->eps;
            gamma = p->beta2 * gamma + (1.0 - p->beta2) * gt;
        }
        if (refresh) {
            // rows 0..a of the verification pass (a full-model pass) joined the sequence: extend the average
            for (int j = 0; j < L2; ++j)
                for (int i = 0; i <= a; ++i) S[j] += (double)cr[(size_t)j * ASD_ROWS + i];
            n_rows += a + 1;
            for (int j = 0; j < L2; ++j) C[j] = (float)(S[j] / (double)n_rows);
            asd_admg2(C.data(), L, p->alpha, p->m, p->n, p->use_cs, p->alpha_mlp, p->use_cs_mlp, mnew.data());
            if (mnew != mask) { mask = mnew; ++mask_changes; drop_graphs(e); e->graph_mask = mask; }
        }
    }
    CK(e, hipMemcpyAsync(out, e->out_tokens, (size_t)n_more * 4, hipMemcpyDeviceToHost, e->stream));
    CK(e, hipStreamSynchronize(e->stream));
    { const int rc2 = check_pass_error(e); if (rc2) return rc2; }
    const auto t1 = std::chrono::steady_clock::now();
    if (stats) {
        stats->cycles = e->h_st->cycles; stats->drafted = e->h_st->drafted; stats->accepted = e->h_st->accepted;
        stats->emitted = emitted; stats->ms_prefill = 0.0;
        stats->ms_decode = std::chrono::duration<double, std::milli>(t1 - t0).count();
        stats->mask_changes = mask_changes; stats->gamma = gamma; stats->ar = ar;
        stats->ms_draft = ms_draft; stats->ms_verify = ms_verify;
        stats->ms_other = stats->ms_decode - ms_draft - ms_verify;
        stats->bytes_draft = bytes_draft; stats->bytes_verify = bytes_verify;
    }
    if (mask_used) memcpy(mask_used, mask.data(), mask.size());
    return ASD_OK;
}

int asd_generate(asd_engine* e, const int32_t* prompt, int32_t n_prompt, int32_t n_new, const asd_gen_params* p, int32_t* out,
                 asd_gen_stats* stats, uint8_t* mask_used) {
    if (!e) return ASD_E_INVAL;
    if (!p || !out) return fail(e, ASD_E_INVAL, "params or out_tokens is NULL");
    if (n_new < 1) return fail(e, ASD_E_INVAL, "n_new must be >= 1");
    if (p->draft_len + 1 > e->c.max_rows) return fail(e, ASD_E_INVAL, "draft_len %d outside [0, %d]", p->draft_len, e->c.max_rows - 1);
    { const int rcp = check_gen_params(e, p); if (rcp) return rcp; }
    if (p->draft_len < 0 || n_prompt < 1 || n_prompt + n_new + p->draft_len > capacity(e))
        return fail(e, ASD_E_INVAL, "prompt %d + new %d + draft %d exceeds the cache capacity %d", n_prompt, n_new, p->draft_len, capacity(e));
    const auto t0 = std::chrono::steady_clock::now();
    int32_t t1 = 0;
    int rc = asd_prefill(e, prompt, n_prompt, &t1, nullptr, nullptr);
    if (rc) return rc;
    asd_gen_params pp = *p;
    if (p->temperature > 0.f) {           // the prompt pass's token is a plain draw with U(0, 2); decoding continues at index 1
        const SampleArgs sa = sample_args(e, p->temperature, p->seed);
        launch_sample_plain(e, sa, e->last_logits_row, 0);
        CK(e, hipMemcpyAsync(&t1, e->tokbuf, 4, hipMemcpyDeviceToHost, e->stream));
        CK(e, hipStreamSynchronize(e->stream));
        pp.sample_index0 = 1;
    }
    const double ms_pre = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    out[0] = t1;
    asd_gen_stats st{};
    if (n_new > 1) {
        rc = asd_decode(e, t1, n_new - 1, &pp, out + 1, &st, mask_used);
        if (rc) return rc;
    } else if (mask_used) {
        memset(mask_used, 0, 2 * (size_t)e->c.n_layers);
    }
    if (stats) { *stats = st; stats->emitted = st.emitted + 1; stats->ms_prefill = ms_pre; }
    return ASD_OK;
}

// ------------------------------------------------------------------ measurement helpers
static int bench_tokens(asd_engine* e, int n_rows) {
    int32_t t[ASD_ROWS];
    for (int i = 0; i < n_rows; ++i) t[i] = (int32_t)((1 + 7919 * i) % e->c.vocab);
    CK(e, hipMemcpyAsync(e->tokbuf, t, (size_t)n_rows * 4, hipMemcpyHostToDevice, e->stream));
    set_state_kernel<<<1, 1, 0, e->stream>>>(e->st, e->kv_len, 0, 0, 0);
    CK(e, hipStreamSynchronize(e->stream));
    return ASD_OK;
}

static int bench_checks(asd_engine* e, int n_rows) {
    if (n_rows < 1 || n_rows > e->c.max_rows) return fail(e, ASD_E_INVAL, "n_rows %d outside [1, %d]", n_rows, e->c.max_rows);
    if (!weights_ready(e)) return fail(e, ASD_E_STATE, "weights are not fully loaded");
    if (e->kv_len + n_rows > capacity(e)) return fail(e, ASD_E_INVAL, "no room for %d rows after %d cached positions", n_rows, e->kv_len);
    return ASD_OK;
}

int asd_time_pass(asd_engine* e, int32_t n_rows, const uint8_t* mask, int32_t reps, int32_t use_graph, double* ms_avg, double* bytes) {
    if (!e) return ASD_E_INVAL;
    if (!ms_avg || reps < 1) return fail(e, ASD_E_INVAL, "ms_avg is NULL or reps < 1");
    int rc = bench_checks(e, n_rows);
    if (rc) return rc;
    rc = bench_tokens(e, n_rows);
    if (rc) return rc;
    const int nc = chunks_for(e->kv_len + n_rows - 1), ctx = e->kv_len + n_rows;
    hipGraphExec_t ge = nullptr;
    if (use_graph) {
        hipGraph_t g = nullptr;
        CK(e, hipStreamBeginCapture(e->stream, hipStreamCaptureModeThreadLocal));
        rc = enqueue_forward(e, e->tokbuf, n_rows, 0, mask, nc, nullptr, ctx);
        hipError_t r2 = hipStreamEndCapture(e->stream, &g);
        if (rc) { if (g) hipGraphDestroy(g); return rc; }
        if (r2 != hipSuccess) return fail(e, ASD_E_HIP, "hipStreamEndCapture: %s", hipGetErrorString(r2));
        r2 = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
        hipGraphDestroy(g);
        if (r2 != hipSuccess) return fail(e, ASD_E_HIP, "hipGraphInstantiate: %s", hipGetErrorString(r2));
    }
    auto once = [&]() -> int {
        if (ge) { CK(e, hipGraphLaunch(ge, e->stream)); return ASD_OK; }
        return enqueue_forward(e, e->tokbuf, n_rows, 0, mask, nc, nullptr, ctx);
    };
    rc = once();                                   // warm-up
    hipEvent_t a = nullptr, b = nullptr;
    if (!rc) { hipEventCreate(&a); hipEventCreate(&b); hipEventRecord(a, e->stream); }
    for (int i = 0; i < reps && !rc; ++i) rc = once();
    float ms = 0.f;
    if (!rc) {
        hipEventRecord(b, e->stream);
        hipError_t r2 = hipEventSynchronize(b);
        if (r2 == hipSuccess) r2 = hipEventElapsedTime(&ms, a, b);
        if (r2 != hipSuccess) rc = fail(e, ASD_E_HIP, "event timing: %s", hipGetErrorString(r2));
    }
    if (a) hipEventDestroy(a);
    if (b) hipEventDestroy(b);
    if (ge) hipGraphExecDestroy(ge);
    if (rc) return rc;
    *ms_avg = (double)ms / reps;
    if (bytes) {
        double cls[ASD_K_COUNT];
        pass_bytes(e, mask, ctx, cls);
        *bytes = 0.0;
        for (int i = 0; i < ASD_K_COUNT; ++i) *bytes += cls[i];
    }
    return ASD_OK;
}

int asd_profile_forward(asd_engine* e, int32_t n_rows, const uint8_t* mask, asd_kernel_times* out) {
    if (!e) return ASD_E_INVAL;
    if (!out) return fail(e, ASD_E_INVAL, "out is NULL");
    int rc = bench_checks(e, n_rows);
    if (rc) return rc;
    rc = bench_tokens(e, n_rows);
    if (rc) return rc;
    const int nc = chunks_for(e->kv_len + n_rows - 1), ctx = e->kv_len + n_rows;
    rc = enqueue_forward(e, e->tokbuf, n_rows, 0, mask, nc, nullptr, ctx);     // warm-up
    if (rc) return rc;
    Profiler pf;
    rc = enqueue_forward(e, e->tokbuf, n_rows, 0, mask, nc, &pf, ctx);
    hipError_t r2 = hipStreamSynchronize(e->stream);
    memset(out, 0, sizeof *out);
    if (!rc && r2 == hipSuccess) {
        for (size_t i = 0; i < pf.cls.size(); ++i) {
            float ms = 0.f;
            hipEventElapsedTime(&ms, pf.ev[2 * i], pf.ev[2 * i + 1]);
            out->ms[pf.cls[i]] += ms; out->launches[pf.cls[i]] += 1; out->bytes[pf.cls[i]] += pf.bytes[i];
        }
        float tot = 0.f;
        if (!pf.ev.empty()) hipEventElapsedTime(&tot, pf.ev.front(), pf.ev.back());
        out->ms_total = tot;
    }
    for (hipEvent_t ev : pf.ev) hipEventDestroy(ev);
    if (rc) return rc;
    if (r2 != hipSuccess) return fail(e, ASD_E_HIP, "profiled pass: %s", hipGetErrorString(r2));
    return ASD_OK;
}

int asd_profile_prefill(asd_engine* e, const int32_t* tokens, int32_t n, asd_prefill_times* out) {
    if (!e) return ASD_E_INVAL;
    if (!tokens || !out) return fail(e, ASD_E_INVAL, "tokens or out is NULL");
    if (n <= e->c.max_rows || n > capacity(e)) return fail(e, ASD_E_INVAL, "prompt length %d outside (%d, %d]", n, e->c.max_rows, capacity(e));
    if (!weights_ready(e)) return fail(e, ASD_E_STATE, "weights are not fully loaded");
    int rc = check_tokens(e, tokens, n);
    if (rc) return rc;
    const int L2 = 2 * e->c.n_layers;
    e->kv_len = 0; e->acs_valid = false;
    CK(e, hipMemsetAsync(e->cos_acc, 0, (size_t)L2 * 8, e->stream));
    rc = prefill_blocks(e, tokens, n);                 // warm-up
    if (rc) return rc;
    e->kv_len = 0;
    CK(e, hipMemsetAsync(e->cos_acc, 0, (size_t)L2 * 8, e->stream));
    Profiler pf;
    rc = prefill_blocks(e, tokens, n, &pf);
    hipError_t r2 = hipStreamSynchronize(e->stream);
    memset(out, 0, sizeof *out);
    if (!rc && r2 == hipSuccess) {
        for (size_t i = 0; i < pf.cls.size(); ++i) {
            float ms = 0.f;
            hipEventElapsedTime(&ms, pf.ev[2 * i], pf.ev[2 * i + 1]);
            out->ms[pf.cls[i]] += ms; out->launches[pf.cls[i]] += 1; out->flops[pf.cls[i]] += pf.bytes[i];
        }
        float tot = 0.f;
        if (!pf.ev.empty()) hipEventElapsedTime(&tot, pf.ev.front(), pf.ev.back());
        out->ms_total = tot;
    }
    for (hipEvent_t ev : pf.ev) hipEventDestroy(ev);
    e->kv_len = 0;                                     // the cache content is the prompt's, but no ACS was kept: start over
    if (rc) return rc;
    if (r2 != hipSuccess) return fail(e, ASD_E_HIP, "profiled prompt pass: %s", hipGetErrorString(r2));
    return ASD_OK;
}

int asd_time_step_class(asd_engine* e, int32_t cls, int32_t n_rows, int32_t reps, double* us_avg, double* bytes_per_launch) {
    if (!e) return ASD_E_INVAL;
    if (!us_avg || reps < 1 || cls <= ASD_K_EMBED || cls >= ASD_K_FINISH)
        return fail(e, ASD_E_INVAL, "us_avg is NULL, reps < 1 or the class is not a timed step class");
    int rc = bench_checks(e, n_rows);
    if (rc) return rc;
    rc = bench_tokens(e, n_rows);
    if (rc) return rc;
    const int nc = chunks_for(e->kv_len + n_rows - 1), ctx = e->kv_len + n_rows;
    std::vector<PassOp> all, sel;
    const PassOut out = engine_out(e);
    build_pass(e, n_rows, 0, nullptr, ctx, nc, out, all);
    rc = launch_steps(e, all, e->tokbuf, n_rows, nullptr, nullptr, FIN_NONE, 0, out);     // valid inputs for every step
    if (rc) return rc;
    double bytes = 0.0;
    for (const PassOp& op : all) if (op.cls == cls) { sel.push_back(op); bytes += op.bytes; }
    if (sel.empty()) return fail(e, ASD_E_INVAL, "the pass has no step of class %d", cls);
    rc = launch_steps(e, sel, e->tokbuf, n_rows, nullptr, nullptr, FIN_NONE, 0, out);     // warm-up
    hipEvent_t a = nullptr, b = nullptr;
    if (!rc) { hipEventCreate(&a); hipEventCreate(&b); hipEventRecord(a, e->stream); }
    for (int i = 0; i < reps && !rc; ++i) rc = launch_steps(e, sel, e->tokbuf, n_rows, nullptr, nullptr, FIN_NONE, 0, out);
    float ms = 0.f;
    if (!rc) {
        hipEventRecord(b, e->stream);
        hipError_t r2 = hipEventSynchronize(b);
        if (r2 == hipSuccess) r2 = hipEventElapsedTime(&ms, a, b);
        if (r2 != hipSuccess) rc = fail(e, ASD_E_HIP, "event timing: %s", hipGetErrorString(r2));
    }
    if (a) hipEventDestroy(a);
    if (b) hipEventDestroy(b);
    if (rc) return rc;
    *us_avg = (double)ms * 1e3 / ((double)reps * sel.size());
    if (bytes_per_launch) *bytes_per_launch = bytes / sel.size();
    return ASD_OK;
}

int asd_copy_bench(asd_engine* e, size_t nbytes, int32_t reps, double* ms_avg) {
    if (!e) return ASD_E_INVAL;
    if (!ms_avg || reps < 1 || nbytes < 16 || nbytes % 16) return fail(e, ASD_E_INVAL, "nbytes must be a positive multiple of 16, reps >= 1");
    // source: the start of the arena (weights are only read); destination: the staging region
    if (nbytes > e->staging_bytes || nbytes > (size_t)(e->staging - e->arena)) return fail(e, ASD_E_INVAL, "nbytes exceeds the scratch region (%zu)", e->staging_bytes);
    hipEvent_t a, b;
    hipEventCreate(&a); hipEventCreate(&b);
    copy_kernel<<<2048, 256, 0, e->stream>>>((const u32x4*)e->arena, (u32x4*)e->staging, nbytes / 16);
    hipEventRecord(a, e->stream);
    for (int i = 0; i < reps; ++i) copy_kernel<<<2048, 256, 0, e->stream>>>((const u32x4*)e->arena, (u32x4*)e->staging, nbytes / 16);
    hipEventRecord(b, e->stream);
    hipError_t r = hipEventSynchronize(b);
    float ms = 0.f;
    if (r == hipSuccess) r = hipEventElapsedTime(&ms, a, b);
    hipEventDestroy(a); hipEventDestroy(b);
    if (r != hipSuccess) return fail(e, ASD_E_HIP, "copy benchmark: %s", hipGetErrorString(r));
    *ms_avg = (double)ms / reps;
    return ASD_OK;
}

}  // extern "C"
