// Host side of the EESD library: context, paged KV cache, pass drivers, the round's calls,
// the Beta-posterior controller and the generation loop.  C ABI in include/eesd.h.
#include "../../include/eesd.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "attention.hiph"
#include "common.hiph"
#include "gemm.hiph"
#include "sampling.hiph"

#define MAX_ROWS 16    // rows of a decoding pass: 1 (draft) .. k_cap + 1 (verify; 1 + k_cap * width in tree mode)
// pinned result words: [0] a, [1] y, [2] draft token, [3] token hooks, [4..4+MAX_ROWS) accepted rows, [24..24+MAX_ROWS+1) block tokens, [44] theta_M (float)
#define H_RESULT_INTS 48
#define H_ROWS_AT 4
#define H_TOKS_AT 24
#define H_THETA_AT 44
#define PREFILL_ROWS 128  // rows of a prefill block when the tiled MFMA product applies (row-major weights)
#define PREFILL_ROWS_WIDE 512   // the same on tile-major weights (gemm_pf_kernel)

// ---------------------------------------------------------------------------------------------
// tunables (benchmark sweeps)
// ---------------------------------------------------------------------------------------------
static int g_valu_nw = 0;      // waves per workgroup of the VALU product (0 = heuristic)
static int g_valu_tpw = 0;     // tasks per wave
static int g_valu_rp = 0;      // row pairs per task (1 or 2)
static int g_mfma_ksplit = 0;  // cross-workgroup K split of the residual products (0 = heuristic)
static int g_mfma_nw = 0;      // waves per workgroup of the MFMA product
static int g_attn_split = 0;   // keys per attention split
static int g_tile_kc = 0;      // column chunk of the tile kernel for verify-sized blocks: 256 / 512 (0 = by reduction length)
static int g_tile_nwt = 0;     // 4 / 8: tiles per workgroup of the tile kernel for verify-sized blocks (0 = by tile count)
static int g_fuse_norm = -1;   // residual -> next product hand-over without resid_norm_kernel: 1 both products, 2 attention output only, 3 FFN down only, 0 off, -1 by model width
static int g_nw_epi[4] = {0, 0, 0, 0};   // waves per workgroup of the per-tile product by epilogue (plain, resid, swiglu, qkv)
static int g_pf_kc = 0;        // 256: prefill blocks take 256-column chunks (default 128)
static int g_pf_rows = 0;      // rows of a prefill block on tile-major weights: 128 (gemm_tile_kernel), 256 or 512 (gemm_pf_kernel; 0 = 512), read by eesd_create
static int g_pf_ts = 0;        // gemm_pf_kernel: tile slots per workgroup for one-tile-per-group matrices (4 or 7; 0 = by tile count)
static int g_grp_minsteps = -1; // row-group kernel, residual products: 4 waves instead of 8 while a wave would get fewer 128-column steps than this (-1: built-in)
static int g_smp_spread = -1;      // draft-step sampling spread over 64 workgroups (three small kernels): 1 on, 0 off, -1 built-in (vocabularies of 4096 entries and more)
static int g_pf_nbw = 0;
static int g_pf_merge = -1;        // prefill GEMM: tails of 20-row groups gathered in one tile slot (0 off; -1 built-in: on)       // gemm_pf_kernel: 16-token blocks per wave (1, 2, 4; 0 = by rows and grid size)
static int g_mfma_tile = 0;    // 1: every block of <= 16 rows takes the LDS-shared tile kernel; 2: none does; 0: by rows and tile count
static int g_mfma_min_m = 1;   // AUTO: smallest M that takes the MFMA family on bf16 weights (measured: faster than the VALU family already at M = 1)

extern "C" int eesd_set_tunable(const char* name, int value) {
    if (!name) return EESD_EINVAL;
    struct { const char* n; int* p; } t[] = {{"valu_nw", &g_valu_nw}, {"valu_tpw", &g_valu_tpw}, {"valu_rp", &g_valu_rp},
                                             {"mfma_ksplit", &g_mfma_ksplit}, {"mfma_nw", &g_mfma_nw}, {"attn_split", &g_attn_split},
                                             {"mfma_min_m", &g_mfma_min_m}, {"mfma_tile", &g_mfma_tile}, {"pf_kc", &g_pf_kc}, {"pf_rows", &g_pf_rows}, {"pf_ts", &g_pf_ts}, {"pf_merge", &g_pf_merge}, {"smp_spread", &g_smp_spread}, {"grp_minsteps", &g_grp_minsteps}, {"pf_nbw", &g_pf_nbw}, {"nw_plain", &g_nw_epi[0]}, {"nw_resid", &g_nw_epi[1]}, {"nw_swiglu", &g_nw_epi[2]}, {"nw_qkv", &g_nw_epi[3]}, {"fuse_norm", &g_fuse_norm}, {"tile_kc", &g_tile_kc}, {"tile_nwt", &g_tile_nwt}};
    for (auto& e : t)
        if (!strcmp(e.n, name)) { *e.p = value; return EESD_OK; }
    return EESD_EINVAL;
}

// ---------------------------------------------------------------------------------------------
// counter-based uniforms: splitmix64 output function of a key built from
// (seed, stream, round, slot, sub); u = top 53 bits * 2^-53
// ---------------------------------------------------------------------------------------------
enum { STREAM_DRAFT = 1, STREAM_ACCEPT = 2, STREAM_RESAMPLE = 3, STREAM_TS_THETA = 4, STREAM_TS_CHI = 5 };

static inline uint64_t splitmix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static inline double uniform53(uint64_t seed, int stream, int64_t rnd, int slot, int sub) {
    uint64_t key = seed ^ ((uint64_t)(stream & 0xFF) << 56) ^ ((uint64_t)(rnd & 0xFFFFFF) << 32) ^
                   ((uint64_t)(slot & 0xFF) << 24) ^ (uint64_t)(sub & 0xFFFFFF);
    return (double)(splitmix64(key) >> 11) * (1.0 / 9007199254740992.0);
}

// ---------------------------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------------------------
enum State { ST_CREATED = 0, ST_READY, ST_VERIFIED, ST_ACCEPTED };

struct eesd_ctx {
    eesd_config cfg;
    std::vector<eesd_layer_weights> layers;
    eesd_weights w;
    hipStream_t stream;
    int device;
    std::string err;

    // sequence state
    State state;
    int kv_len;       // tokens whose K/V are valid in every cache
    int n_drafted;    // drafts since the last rollback
    int64_t round;    // 0 = prefill, 1.. = decoding rounds
    int last_a, last_y;
    std::vector<int32_t> forced;  // teacher-forced draft tokens (consumed front first)
    size_t forced_pos;

    // controller
    double alpha, beta;
    std::vector<int32_t> schedule;
    int64_t sched_round;
    eesd_stats stats;

    // paged KV cache
    int n_caches;            // L + 1
    int n_pages, page_tokens, page_shift;
    long long page_stride;   // elements
    size_t elem;             // bytes per cache element
    void* kv_pool;
    int32_t* d_table;        // device page table
    int32_t* h_table;        // pinned host mirror
    std::vector<int32_t> free_pages;
    int mapped_pages;

    // scratch (device)
    float *x, *q, *attn, *act, *logits, *p_rows, *q_logits, *q_rows, *part_o, *part_ml, *rope_cs, *part, *ssq;
    bool xb_has_ssq;       // c->xb holds gain * x (bf16) and c->ssq the partial sums of squares of x, instead of RMSNorm(x)
    bf16_t *xb, *ab, *actb;
    int32_t *blk_tok, *prompt_dev, *result_dev;
    int32_t *tree_blk;     // tree mode: tokens of the verify block's rows (pending token, then `width` children per depth)
    int32_t *h_result, *h_prompt;  // pinned
    // candidate tree
    bool tree_active;               // the rows being processed are tree nodes (verify in tree mode)
    unsigned short tree_mask[16];   // visible block rows per row
    unsigned char tree_depth[16];   // rotary offset per row
    std::vector<int32_t> last_tokens;   // tokens the last accept kept (drafts or tree nodes), without the next token
    // calibrated controller (Algorithm 3)
    bool cali_set;
    eesd_calibration cali;
    double cali_theta_hat, cali_weight;   // observed mean of chi and the observations behind it
    int64_t cali_n;                       // verifications so far
    float *h_t, *cali_u, *theta_dev;      // H_t^(T) [d], W^i H_t^(T) [d], theta_M
    bf16_t* h_tb;                         // bf16 copy of h_t (operand of the MFMA product)
    float* hn_rows;                       // verify_reuse: layer-N hidden state of every draft step's input row [k_cap][d]
    int launch_counts[20];   // product launches since creation, [kernel 0 VALU / 1 one workgroup per tile / 2 one workgroup per row group / 3 LDS-shared tiles / 4 prefill GEMM][epilogue]
    int max_splits;
    int n_cu;              // compute units of the device (fixes the row groups of the tile-major weight layout)
    int ssq_slots;         // partial sums of squares a residual product leaves per row
    int row_cap;           // rows the activation buffers hold (16, PREFILL_ROWS, or up to PREFILL_ROWS_WIDE with pf_wide)
    int part_rows;         // rows of one slab of the K-split partial sums
    char* spl_buf;      // chunk statistics of the sampling tails spread over workgroups (SPL_SCRATCH_BYTES)
    bf16_t *xpb, *abp, *actp;   // pf_wide: what xb, ab and actb hold for a prefill block, in operand order (written by the producers)
    bool pf_wide;          // prefill blocks go through gemm_pf_kernel (tile-major weights, every reduction a multiple of 256)
    hipEvent_t ev[4];

    // per-kernel timing of one class of product launches (benchmark hook)
    int prof_family, prof_epi, prof_in;   // family: -1 off, 0 VALU, 1 MFMA
    std::vector<hipEvent_t> prof_ev;      // start/stop pairs
    size_t prof_used;
};

static int fail(eesd_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIP_TRY(c, call)                                                                            \
    do {                                                                                            \
        hipError_t e__ = (call);                                                                    \
        if (e__ != hipSuccess) return fail((c), EESD_EDEVICE, "%s: %s", #call, hipGetErrorString(e__)); \
    } while (0)

static inline bool is_bf16(const eesd_ctx* c) { return c->cfg.dtype == EESD_DTYPE_BF16; }
// logits rows are fp32, or bf16 when the configuration asks the LM heads for bf16 logits
static inline bool lb16(const eesd_ctx* c) { return c->cfg.logits_bf16 == 1; }
static inline void* logit_row(const eesd_ctx* c, float* base, size_t row) { return (char*)base + row * (size_t)c->cfg.vocab * (lb16(c) ? 2 : 4); }

static KVView kv_view(const eesd_ctx* c, int cache) {
    KVView v;
    v.pool = c->kv_pool;
    v.table = c->d_table;
    v.page_stride = c->page_stride;
    long long blk = (long long)c->cfg.n_kv_heads * c->page_tokens * c->cfg.head_dim;
    v.k_off = (long long)(cache * 2) * blk;
    v.v_off = (long long)(cache * 2 + 1) * blk;
    v.page_tokens = c->page_tokens;
    v.page_shift = c->page_shift;
    v.n_kv_heads = c->cfg.n_kv_heads;
    v.head_dim = c->cfg.head_dim;
    v.v_transposed = is_bf16(c) ? 1 : 0;
    v.tiled = (is_bf16(c) && c->page_tokens % 32 == 0) ? 1 : 0;     // operand order: what the MFMA attention reads with contiguous lanes
    return v;
}

// compute units of the current device (cached per device)
static int device_cu_count() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (!cached[dev]) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev] = n;
    }
    return cached[dev];
}

// ---------------------------------------------------------------------------------------------
// kernel launchers
// ---------------------------------------------------------------------------------------------
// Dynamic LDS above the default limit has to be granted per kernel; remember what was granted.
static hipError_t allow_lds(const void* fn, size_t bytes) {
    static std::vector<std::pair<const void*, size_t>> done;
    static std::mutex mu;          // contexts of different threads share the list
    if (bytes <= 48 * 1024) return hipSuccess;
    std::lock_guard<std::mutex> lock(mu);
    for (auto& p : done)
        if (p.first == fn) {
            if (p.second >= bytes) return hipSuccess;
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e == hipSuccess) p.second = bytes;
            return e;
        }
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done.push_back({fn, bytes});
    return e;
}

template <typename WT, int MT, int EPI, int RP>
static hipError_t launch_valu_t(const GemmP& p, hipStream_t st) {
    int n_tasks = (p.out_rows / 2) / RP;
    size_t lds = ((size_t)MT * p.in_dim + MT) * sizeof(float);
    if (lds > 150 * 1024) return hipErrorInvalidValue;
    int nw = g_valu_nw ? g_valu_nw : ((lds > 40 * 1024 || sizeof(WT) == 2) ? 16 : 4);
    int tpw = g_valu_tpw ? g_valu_tpw : std::max(1, std::min(8, n_tasks / 8192));
    int grid = (n_tasks + nw * tpw - 1) / (nw * tpw);
    auto fn = gemm_valu_kernel<WT, MT, EPI, RP>;
    hipError_t e = allow_lds((const void*)fn, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(nw * 64), lds, st, p, n_tasks, tpw);
    return hipGetLastError();
}

template <typename WT, int EPI>
static hipError_t launch_valu_m(const GemmP& p, hipStream_t st) {
    bool rp2 = g_valu_rp ? g_valu_rp == 2 : true;
    // pairs per task must divide the pairs of a head half (QKV) and the pair count
    int n_pairs = p.out_rows / 2;
    if (EPI == EPI_QKV && ((p.head_dim / 2) % 2)) rp2 = false;
    if (n_pairs % 2) rp2 = false;
    if (p.M <= 1) return rp2 ? launch_valu_t<WT, 1, EPI, 2>(p, st) : launch_valu_t<WT, 1, EPI, 1>(p, st);
    if (p.M <= 2) return rp2 ? launch_valu_t<WT, 2, EPI, 2>(p, st) : launch_valu_t<WT, 2, EPI, 1>(p, st);
    if (p.M <= 4) return rp2 ? launch_valu_t<WT, 4, EPI, 2>(p, st) : launch_valu_t<WT, 4, EPI, 1>(p, st);
    if (p.M <= 8) return launch_valu_t<WT, 8, EPI, 1>(p, st);
    return launch_valu_t<WT, 16, EPI, 1>(p, st);
}

static size_t valu_lds_bytes(int M, int in) {
    int mt = M <= 1 ? 1 : M <= 2 ? 2 : M <= 4 ? 4 : M <= 8 ? 8 : 16;
    return ((size_t)mt * in + mt) * sizeof(float);
}

template <int EPI>
static hipError_t launch_valu(const GemmP& p, bool bf16, hipStream_t st) {
    return bf16 ? launch_valu_m<bf16_t, EPI>(p, st) : launch_valu_m<float, EPI>(p, st);
}

// cross-workgroup K split of a residual product (its partial sums are folded by resid_norm_kernel)
#define MFMA_MAX_KSPLIT 8
static int mfma_ksplit(int out_rows, int in_dim) {
    if (g_mfma_ksplit) return std::min(g_mfma_ksplit, MFMA_MAX_KSPLIT);
    const int n_tiles = out_rows / 16, steps = in_dim / 128;
    int ks = 1;
    while (ks < MFMA_MAX_KSPLIT && n_tiles * ks < 1024 && steps / (ks * 2) >= 4) ks *= 2;
    return ks;
}

#define GT_KC_MIN 256
static bool tile_shape_ok(int out_rows, int in_dim) { return (out_rows / 16) % 4 == 0 && in_dim % GT_KC_MIN == 0; }

template <int EPI, int NB, int KC, int NWT>
static hipError_t launch_tile_t(const GemmP& p, int ksplit, hipStream_t st) {
    size_t lds = (size_t)2 * NB * 16 * (KC + GT_PAD) * sizeof(bf16_t);
    auto fn = gemm_tile_kernel<EPI, NB, KC, NWT>;
    hipError_t e = allow_lds((const void*)fn, lds);
    if (e != hipSuccess) return e;
    const bool grouped = p.w_packed && p.n_groups != p.out_rows / 16;
    if (grouped && NWT < GRP_MAX_TILES) return hipErrorInvalidValue;
    GemmP pl = p;
    pl.nw = NWT; pl.ksplit = ksplit;
    hipLaunchKernelGGL(fn, dim3(grouped ? p.n_groups : p.out_rows / (16 * NWT), ksplit), dim3(64 * NWT), lds, st, pl);
    return hipGetLastError();
}

// one workgroup per row group (tile-major matrices dealt to one group per CU), blocks of <= 16 rows
template <int EPI>
static hipError_t launch_group(const GemmP& p, hipStream_t st) {
    if (EPI == EPI_RESID && p.y_partial) return hipErrorInvalidValue;
    const int units = p.out_rows / 4, max_units = (units + p.n_groups - 1) / p.n_groups;
    const int tmax = (max_units * 4 + 15) / 16;
    int nw = g_nw_epi[EPI] ? std::min(g_nw_epi[EPI], 8) : 8;
    const int steps = p.in_dim / 128;
    // residual products whose waves would get fewer than 14 steps each (13B shape: both; 70B shape: the attention output): 4 waves
    // (measured -1.1 us per 13B-shape layer, -0.3 us per 70B-shape layer)
    if (EPI == EPI_RESID && !g_nw_epi[EPI] && steps / 8 < (g_grp_minsteps < 0 ? 14 : g_grp_minsteps)) nw = 4;
    while (nw > 1 && steps / nw < 2) nw >>= 1;
    const size_t lds = (size_t)nw * tmax * 1024;
    GemmP pl = p;
    pl.nw = nw; pl.ksplit = 1;
    switch (tmax) {
        case 1: hipLaunchKernelGGL((gemm_group_kernel<EPI, 1>), dim3(p.n_groups), dim3(nw * 64), lds, st, pl); break;
        case 2: hipLaunchKernelGGL((gemm_group_kernel<EPI, 2>), dim3(p.n_groups), dim3(nw * 64), lds, st, pl); break;
        case 3: hipLaunchKernelGGL((gemm_group_kernel<EPI, 3>), dim3(p.n_groups), dim3(nw * 64), lds, st, pl); break;
        case 4: hipLaunchKernelGGL((gemm_group_kernel<EPI, 4>), dim3(p.n_groups), dim3(nw * 64), lds, st, pl); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// prefill blocks on tile-major weights: 8 waves x 16 NBW tokens against TS tile slots per workgroup
template <int EPI, int TS, int NBW>
static hipError_t launch_pf_t(const GemmP& p, int tg, int gx, int merged, hipStream_t st) {
    const size_t lds = (size_t)2 * PF_QC * TS * 1024;
    auto fn = gemm_pf_kernel<EPI, TS, NBW>;
    hipError_t e = allow_lds((const void*)fn, lds);
    if (e != hipSuccess) return e;
    const int gy = (p.M + PF_NW * 16 * NBW - 1) / (PF_NW * 16 * NBW);
    hipLaunchKernelGGL(fn, dim3((gx + 7) / 8 * 8 * gy), dim3(64 * PF_NW), lds, st, p, tg, gx, gy, merged);
    return hipGetLastError();
}
template <int EPI, int TS>
static hipError_t launch_pf_ts(const GemmP& p, int tg, int gx, int nbw, int merged, hipStream_t st) {
    if (nbw == 1) return launch_pf_t<EPI, TS, 1>(p, tg, gx, merged, st);
    if (nbw == 2) return launch_pf_t<EPI, TS, 2>(p, tg, gx, merged, st);
    if constexpr (TS <= 4) {   // 7 tile slots x 4 token blocks would not fit the register file
        if (nbw == 4) return launch_pf_t<EPI, TS, 4>(p, tg, gx, merged, st);
    }
    return hipErrorInvalidValue;
}
static bool pf_shape_ok(const GemmP& p) { return p.w_packed && p.in_dim % (32 * PF_QC) == 0 && p.M <= PREFILL_ROWS_WIDE && !p.y_partial && !p.ssq_in && !p.xb_out; }
// p.X: the block's rows in operand order (x_packed), or row-major, then xp: room for them in operand order (ceil(M / 16) * 16 * in_dim elements)
template <int EPI>
static hipError_t launch_pf(const GemmP& p_rows, bf16_t* xp, int n_cu, hipStream_t st) {
    if (!pf_shape_ok(p_rows) || (!xp && !p_rows.x_packed)) return hipErrorInvalidValue;
    GemmP p = p_rows;
    if (!p.x_packed) {
        hipLaunchKernelGGL(pack_act_kernel, dim3((p.in_dim / 8 + 255) / 256, (p.M + 15) / 16), dim3(256), 0, st, (const bf16_t*)p.X, p.ldx, p.M, p.in_dim, xp);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        p.X = xp;
        p.x_packed = 1;
    }
    const int n_tiles16 = p.out_rows / 16;
    int tg = 1, ts = 4, merged = 0;
    if (p.n_groups != n_tiles16) {
        // one row group per CU: 3 tiles per group - one group per workgroup; 1, 2 or 4 - four tile slots; groups of a
        // whole tile and a tail of 4 rows (plain and residual epilogues) - two groups per workgroup, their tails in one slot
        const int units = p.out_rows / 4, max_units = (units + p.n_groups - 1) / p.n_groups;
        tg = (max_units * 4 + 15) / 16;
        if (tg > GRP_MAX_TILES) return hipErrorInvalidValue;
        ts = tg == 3 ? 3 : 4;
        if ((EPI == EPI_PLAIN || EPI == EPI_RESID) && max_units == 5 && g_pf_merge != 0) { merged = 1; ts = 3; }
    } else {
        // one tile per group: 7 tiles per workgroup when there are very many (gate/up: 3584 = 2 x 256 x 7 at the 70B shape)
        ts = g_pf_ts ? g_pf_ts : (EPI == EPI_SWIGLU && n_tiles16 >= 4 * n_cu ? 7 : 4);
        if (ts != 4 && (ts != 7 || EPI != EPI_SWIGLU)) return hipErrorInvalidValue;
    }
    const int per_wg = merged ? ts - 1 : ts / tg;     // row groups of a workgroup
    const int gx = (p.n_groups + per_wg - 1) / per_wg;
    // tokens per wave: as many as the block has, fewer while the grid would leave CUs without a workgroup
    int nbw = p.M <= 128 ? 1 : (p.M <= 256 ? 2 : 4);
    if (ts == 7) nbw = std::min(nbw, 2);
    while (nbw > 1 && gx * ((p.M + 128 * nbw - 1) / (128 * nbw)) < n_cu) nbw >>= 1;
    if (g_pf_nbw) nbw = std::min(g_pf_nbw, ts == 7 ? 2 : 4);
    if (ts == 3) return launch_pf_ts<EPI, 3>(p, tg, gx, nbw, merged, st);
    if constexpr (EPI == EPI_SWIGLU) {
        if (ts == 7) return launch_pf_ts<EPI, 7>(p, tg, gx, nbw, 0, st);
    }
    return launch_pf_ts<EPI, 4>(p, tg, gx, nbw, 0, st);
}

template <int EPI>
static hipError_t launch_mfma(const GemmP& p, int ksplit, hipStream_t st, int* kernel_taken = nullptr, int n_cu = 0, bf16_t* xp = nullptr) {
    int taken_dummy;
    int& taken = kernel_taken ? *kernel_taken : taken_dummy;
    taken = 3;
    // Which kernel (measured per product at the 13B and 70B shapes): one workgroup per tile streams
    // fastest for few rows and for the products with few tiles (QKV, attention output, FFN down) at
    // any M <= 16; from 6 rows on (7 for the widest) the products with many tiles (gate/up, LM heads) gain more
    // from sharing the activation operand through LDS than they lose to its barriers, with 8 tiles
    // per workgroup when there are very many.  Prefill blocks (M > 16) always take the tile kernel.
    const int n_tiles16 = p.out_rows / 16;
    const bool partial = EPI == EPI_RESID && p.y_partial;
    if (p.M > 16 && n_cu > 0 && (xp || p.x_packed) && g_pf_rows != 128 && pf_shape_ok(p)) { taken = 4; return launch_pf<EPI>(p, xp, n_cu, st); }
    if (p.w_packed && p.n_groups != n_tiles16) {
        // one row group per CU: decoding blocks take the group kernel, prefill blocks the tile kernel with a wave per tile of the group
        if (p.M <= 16) { taken = 2; return launch_group<EPI>(p, st); }
        if (p.in_dim % GT_KC_MIN) return hipErrorInvalidValue;
        if (p.M <= 32) return launch_tile_t<EPI, 2, 256, 4>(p, ksplit, st);
        if (p.M <= 64) return launch_tile_t<EPI, 4, 256, 4>(p, ksplit, st);
        if (p.M <= 128) return g_pf_kc == 256 ? launch_tile_t<EPI, 8, 256, 4>(p, ksplit, st) : launch_tile_t<EPI, 8, 128, 4>(p, ksplit, st);
        return hipErrorInvalidValue;
    }
    bool use_tile = p.M > 16;
    if (p.M <= 16 && g_mfma_tile == 1) use_tile = true;
    // crossover rows (measured): row-major weights 6, 7 for the widest products; tile-major weights, whose
    // per-tile kernel leaves the activation rows in L2, 7 and 10
    const int tile_min_m = p.w_packed ? (n_tiles16 >= 3072 ? 10 : 7) : (n_tiles16 >= 3072 ? 7 : 6);
    if (p.M <= 16 && g_mfma_tile == 0) use_tile = p.M >= tile_min_m && n_tiles16 >= 1536 && !partial;
    if (EPI == EPI_RESID && p.xb_out) use_tile = false;   // the hand-over to the next product lives in the per-tile kernel
    if (use_tile && tile_shape_ok(p.out_rows, p.in_dim)) {
        if (p.M <= 16) {
            const bool w8 = (g_tile_nwt ? g_tile_nwt == 8 : n_tiles16 >= 3072) && n_tiles16 % 8 == 0;
            // 512-column chunks halve the barriers: measured -5 us per 70B-shape layer at 10-16 rows, +2.5 us at the 13B shape
            if ((g_tile_kc == 512 || (g_tile_kc == 0 && p.in_dim >= 8192)) && p.in_dim % 512 == 0)
                return w8 ? launch_tile_t<EPI, 1, 512, 8>(p, ksplit, st) : launch_tile_t<EPI, 1, 512, 4>(p, ksplit, st);
            return w8 ? launch_tile_t<EPI, 1, 256, 8>(p, ksplit, st) : launch_tile_t<EPI, 1, 256, 4>(p, ksplit, st);
        }
        if (p.M <= 32) return launch_tile_t<EPI, 2, 256, 4>(p, ksplit, st);
        if (p.M <= 64) return launch_tile_t<EPI, 4, 256, 4>(p, ksplit, st);
        // 128-row prefill blocks: 128-column chunks keep two workgroups on a CU (70 KB of LDS each),
        // which measured 1.3x faster than one workgroup with 256-column chunks
        if (p.M <= 128) return g_pf_kc == 256 ? launch_tile_t<EPI, 8, 256, 4>(p, ksplit, st) : launch_tile_t<EPI, 8, 128, 4>(p, ksplit, st);
        return hipErrorInvalidValue;
    }
    if (p.M > 16) return hipErrorInvalidValue;
    taken = 1;
    const int n_tiles = p.out_rows / 16, steps = p.in_dim / 128;
    int nw = g_nw_epi[EPI] ? g_nw_epi[EPI] : g_mfma_nw;
    if (!nw) {
        if (EPI == EPI_RESID && p.y_partial) {
            // K is already split over workgroups: 2-4 waves each, at least two 128-column steps per wave
            nw = 2;
            while (nw < 4 && n_tiles * ksplit * nw < 2560 && steps / (ksplit * nw * 2) >= 2) nw *= 2;
            if (steps / ksplit < 2) nw = 1;
        } else {
            // one workgroup per tile: many waves per tile keep the tail short when tiles / CU is
            // small or fractional (measured best at 8 for the QKV, gate/up and head products)
            nw = 8;
            // tile-major weights: the residual products that keep K whole (wide models) stream best
            // with 4 waves (measured -4 us per 70B layer; every other product stays at 8)
            if (p.w_packed && EPI == EPI_RESID && p.xb_out) nw = 4;
            while (nw > 1 && steps / nw < 4) nw >>= 1;
        }
    }
    nw = std::max(1, std::min(nw, 16));
    size_t lds = (size_t)nw * 64 * 16;
    GemmP pl = p;
    pl.nw = nw; pl.ksplit = ksplit;
    hipLaunchKernelGGL((gemm_mfma_kernel<EPI>), dim3(n_tiles, ksplit), dim3(nw * 64), lds, st, pl);
    return hipGetLastError();
}

static bool mfma_shape_ok(int out, int in, int epi, int head_dim) {
    if (in % 128) return false;
    if (epi == EPI_QKV) return head_dim % 16 == 0 && out % head_dim == 0;
    if (epi == EPI_SWIGLU) return (out / 2) % 8 == 0;
    return out % 16 == 0;
}

// true -> MFMA family
static bool pick_mfma(const eesd_ctx* c, int M) {
    if (!is_bf16(c)) return false;
    if (c->cfg.gemm_path == EESD_GEMM_VALU) return false;
    if (lb16(c)) return true;     // only the MFMA family writes bf16 logits
    if (c->cfg.gemm_path == EESD_GEMM_MFMA || c->cfg.weight_layout == EESD_WEIGHTS_TILED) return true;
    return M >= g_mfma_min_m;
}

#define PROF_MAX_PAIRS 8192

template <int EPI>
static int gemm_launch(eesd_ctx* c, bool mfma, const GemmP& p, int ksplit = 1) {
    bool prof = c->prof_family == (mfma ? 1 : 0) && c->prof_epi == EPI && (c->prof_in == 0 || c->prof_in == p.in_dim) &&
                p.M <= MAX_ROWS && c->prof_used < PROF_MAX_PAIRS;   // decoding passes only, not prefill blocks
    if (prof) {
        while (c->prof_ev.size() < 2 * (c->prof_used + 1)) {
            hipEvent_t e;
            HIP_TRY(c, hipEventCreate(&e));
            c->prof_ev.push_back(e);
        }
        HIP_TRY(c, hipEventRecord(c->prof_ev[2 * c->prof_used], c->stream));
    }
    if (mfma) {
        GemmP pm = p;
        pm.w_packed = c->cfg.weight_layout == EESD_WEIGHTS_TILED;
        pm.n_groups = pm.w_packed ? pack_n_groups(pm.out_rows, c->n_cu) : 0;
        int taken = 0;
        HIP_TRY(c, launch_mfma<EPI>(pm, ksplit, c->stream, &taken, c->n_cu, nullptr));
        ++c->launch_counts[taken * 4 + EPI];
    } else {
        HIP_TRY(c, launch_valu<EPI>(p, is_bf16(c), c->stream));
        ++c->launch_counts[EPI];
    }
    if (prof) {
        HIP_TRY(c, hipEventRecord(c->prof_ev[2 * c->prof_used + 1], c->stream));
        ++c->prof_used;
    }
    return EESD_OK;
}

// consumers of c->xb: tell the product whether the rows still need their 1/rms
static void take_xb(const eesd_ctx* c, GemmP& p) {
    if (c->xb_has_ssq) {
        p.ssq_in = c->ssq;
        p.ssq_tiles = c->ssq_slots;
        p.ssq_eps = c->cfg.rms_eps;
    }
}

// a RESID product of a decoding pass that hands its rows straight to the next product
static void fuse_next(eesd_ctx* c, GemmP& p, const void* gain) {
    p.xb_out = c->xb;
    p.ld_xb = c->cfg.d_model;
    p.gain_next = gain;
    p.ssq_out = c->ssq;
    p.ssq_tiles = c->ssq_slots;
}

static GemmP gemm_base(const void* W, const void* X, int ldx, int M, int out, int in) {
    GemmP p;
    memset(&p, 0, sizeof p);
    p.W = W; p.X = X; p.ldx = ldx; p.M = M; p.out_rows = out; p.in_dim = in;
    return p;
}

static int launch_attention(eesd_ctx* c, int cache, int M, int pos0, bool out_bf16) {
    const eesd_config& g = c->cfg;
    const bool kb = is_bf16(c);
    AttnP a;
    memset(&a, 0, sizeof a);
    a.Q = c->q;
    a.kv = kv_view(c, cache);
    a.M = M; a.pos0 = pos0;
    a.n_heads = g.n_heads; a.n_kv_heads = g.n_kv_heads; a.head_dim = g.head_dim;
    const int n_keys = pos0 + M;
    const int group = g.n_heads / g.n_kv_heads;
    // bf16: one wave per 16 query rows, all of a KV head's rows in one workgroup; fp32: 16 rows per workgroup
    const int qtiles = (M * group + 15) / 16;
    const int tile = kb ? 32 : ATT_TT;          // keys per inner step
    int split_len = g_attn_split;
    if (!split_len) {
        // enough waves to cover the chip, at least two steps per split when the cache is long
        int want = std::max(1, 2048 / std::max(1, g.n_kv_heads * qtiles));
        split_len = (n_keys + want - 1) / want;
        // bf16: one 32-key step per wave while the cache is short (measured 0.5 % of a layer better than two), two beyond
        split_len = std::max(kb ? (n_keys <= 1024 && M <= MAX_ROWS ? 32 : 64) : 2 * ATT_TT, split_len);
    }
    const int max_splits = std::max(1, std::min(c->max_splits, (MAX_ROWS * c->max_splits) / M));   // partial buffers hold 16 rows x max_splits
    // prefill blocks: the query tiles of a workgroup share the keys through LDS (attn_pf_kernel); key splits only while
    // the block alone leaves CUs without a workgroup
    const bool shared_keys = kb && M > MAX_ROWS && g.kv_page % 32 == 0 && !c->tree_active;
    if (shared_keys && !g_attn_split) {
        const int wgs = g.n_kv_heads * ((qtiles + 7) / 8);
        const int want = std::max(1, std::min(max_splits, (c->n_cu + wgs - 1) / wgs));
        split_len = std::max(64, (n_keys + want - 1) / want);
    }
    split_len = (split_len + tile - 1) / tile * tile;
    int n_splits = (n_keys + split_len - 1) / split_len;
    if (n_splits > max_splits) {
        split_len = ((n_keys + max_splits - 1) / max_splits + tile - 1) / tile * tile;
        n_splits = (n_keys + split_len - 1) / split_len;
    }
    a.n_splits = n_splits; a.split_len = split_len;
    a.scale = 1.0f / sqrtf((float)g.head_dim);
    a.out = out_bf16 ? (void*)c->ab : (void*)c->attn;
    a.out_bf16 = out_bf16;
    if (out_bf16 && M > MAX_ROWS && c->pf_wide) {   // prefill block: the output product reads its rows in operand order
        a.out = c->abp;
        a.out_packed = 1;
    }
    a.part_o = c->part_o; a.part_ml = c->part_ml;
    if (c->tree_active) {
        a.tree = 1;
        for (int r = 0; r < 16; ++r) a.tree_mask[r >> 2] |= (unsigned long long)c->tree_mask[r] << (16 * (r & 3));
    }
    if (kb) {
        dim3 grid(n_splits * g.n_kv_heads, (qtiles + 7) / 8);
        const int nwq = std::min(qtiles, 8);
        if (shared_keys) {
            if (g.head_dim == 128) hipLaunchKernelGGL((attn_pf_kernel<128>), grid, dim3(512), 0, c->stream, a);
            else hipLaunchKernelGGL((attn_pf_kernel<64>), grid, dim3(512), 0, c->stream, a);
        } else if (g.head_dim == 128) hipLaunchKernelGGL((attn_mfma_kernel<128>), grid, dim3(64 * nwq), 0, c->stream, a);
        else hipLaunchKernelGGL((attn_mfma_kernel<64>), grid, dim3(64 * nwq), 0, c->stream, a);
    } else {
        dim3 grid(n_splits * g.n_kv_heads, qtiles);
        if (g.head_dim == 128) hipLaunchKernelGGL((attn_split_kernel<float, 128>), grid, dim3(ATT_THREADS), 0, c->stream, a);
        else hipLaunchKernelGGL((attn_split_kernel<float, 64>), grid, dim3(ATT_THREADS), 0, c->stream, a);
    }
    HIP_TRY(c, hipGetLastError());
    if (n_splits > 1) {
        if (g.head_dim == 128) hipLaunchKernelGGL((attn_combine_kernel<128>), dim3(M * g.n_heads), dim3(128), 0, c->stream, a);
        else hipLaunchKernelGGL((attn_combine_kernel<64>), dim3(M * g.n_heads), dim3(64), 0, c->stream, a);
        HIP_TRY(c, hipGetLastError());
    }
    return EESD_OK;
}

static int launch_rmsnorm_bf16(eesd_ctx* c, const float* x, int M, const void* gain, bf16_t* out, int ld) {
    int d = c->cfg.d_model;
    if (out == c->xb) c->xb_has_ssq = false;
    bf16_t* xp = (out == c->xb && M > MAX_ROWS && c->pf_wide) ? c->xpb : nullptr;    // prefill block: its GEMMs read the rows in operand order
    hipLaunchKernelGGL((rmsnorm_bf16_kernel<bf16_t>), dim3(M), dim3(1024), 0, c->stream, x, d, (const bf16_t*)gain, c->cfg.rms_eps, d,
                       out, ld, xp);
    HIP_TRY(c, hipGetLastError());
    return EESD_OK;
}

static void fill_qkv(eesd_ctx* c, GemmP& p, int cache, int pos0, int head0) {
    p.Q = c->q;
    p.n_heads = c->cfg.n_heads; p.n_kv_heads = c->cfg.n_kv_heads; p.head_dim = c->cfg.head_dim;
    p.head0 = head0; p.pos0 = pos0; p.rope_cs = c->rope_cs;
    p.kv = kv_view(c, cache);
    p.kv_bf16 = is_bf16(c);
    if (c->tree_active) {
        p.tree = 1;
        for (int r = 0; r < 16; ++r) p.rope_off |= (unsigned long long)(c->tree_depth[r] & 15) << (4 * r);
    }
}

static int launch_resid_norm(eesd_ctx* c, int M, int ksplit, const void* gain) {
    const int d = c->cfg.d_model;
    bf16_t* xp = (M > MAX_ROWS && c->pf_wide) ? c->xpb : nullptr;
    hipLaunchKernelGGL((resid_norm_kernel<bf16_t>), dim3(M), dim3(1024), 0, c->stream, c->x, d, c->part, ksplit, c->part_rows, d, (const bf16_t*)gain,
                       c->cfg.rms_eps, d, c->xb, d, xp);
    HIP_TRY(c, hipGetLastError());
    return EESD_OK;
}

// One decoder layer on the M rows in c->x at positions pos0.. ; K/V go to `cache`.
// MFMA family: on entry c->xb holds RMSNorm(x; lw.attn_norm) in bf16; on exit it holds
// RMSNorm(x; next_gain) for whatever consumes the layer's output next.
static int run_layer(eesd_ctx* c, const eesd_layer_weights& lw, int cache, int M, int pos0, bool mfma, const void* next_gain) {
    const eesd_config& g = c->cfg;
    const int d = g.d_model, hd = g.head_dim, qd = g.n_heads * hd, f = g.d_ff;
    const int qkv_rows = (g.n_heads + 2 * g.n_kv_heads) * hd;
    int rc;
    if (mfma) {
        // Decoding blocks (<= 16 rows): the residual products keep K inside the workgroup and hand
        // gain * x and partial sums of squares to their consumer (no kernel in between).  Prefill
        // blocks split K over workgroups and fold the partial sums in resid_norm_kernel.
        // (measured: -10 us per 70B-shape layer; at d_model = 5120 the 320-tile FFN-down product loses more
        // without its K split than the small kernel costs, so narrow models hand over after the
        // attention output only: -2 us per 13B-shape layer)
        // (matrices dealt to one row group per CU always keep K whole and hand over: the group kernel has no other form)
        const bool fuse_ok = M <= MAX_ROWS;
        const bool grouped = c->cfg.weight_layout == EESD_WEIGHTS_TILED && pack_n_groups(d, c->n_cu) != d / 16;
        const bool fused_wo = fuse_ok && (grouped || g_fuse_norm < 0 ? true : (g_fuse_norm == 1 || g_fuse_norm == 2));
        const bool fused_down = fuse_ok && (grouped || (g_fuse_norm < 0 ? d / 16 >= 448 : (g_fuse_norm == 1 || g_fuse_norm == 3)));
        // prefill block on tile-major weights: GEMMs whose inputs the producers leave in operand order; a residual product
        // adds into the stream and a norm kernel follows
        const bool gemm_blk = M > MAX_ROWS && c->pf_wide;
        GemmP p = gemm_base(lw.wqkv, c->xb, d, M, qkv_rows, d);
        fill_qkv(c, p, cache, pos0, 0);
        take_xb(c, p);
        if (gemm_blk) { p.X = c->xpb; p.x_packed = 1; }
        if ((rc = gemm_launch<EPI_QKV>(c, true, p))) return rc;
        if ((rc = launch_attention(c, cache, M, pos0, true))) return rc;
        p = gemm_base(lw.wo, c->ab, qd, M, d, qd);
        if (gemm_blk) { p.X = c->abp; p.x_packed = 1; }
        if (gemm_blk) {
            p.Y = c->x; p.ldy = d;
            if ((rc = gemm_launch<EPI_RESID>(c, true, p))) return rc;
            if ((rc = launch_resid_norm(c, M, 0, lw.ffn_norm))) return rc;
            c->xb_has_ssq = false;
        } else if (fused_wo) {
            p.Y = c->x; p.ldy = d;
            fuse_next(c, p, lw.ffn_norm);
            if ((rc = gemm_launch<EPI_RESID>(c, true, p))) return rc;
            c->xb_has_ssq = true;
        } else {
            int ks = mfma_ksplit(d, qd);
            p.Y = c->part; p.ldy = d; p.y_partial = 1; p.part_rows = c->part_rows;
            if ((rc = gemm_launch<EPI_RESID>(c, true, p, ks))) return rc;
            if ((rc = launch_resid_norm(c, M, ks, lw.ffn_norm))) return rc;
            c->xb_has_ssq = false;
        }
        p = gemm_base(lw.w_gate_up, c->xb, d, M, 2 * f, d);
        p.Y = c->actb; p.ldy = f; p.y_bf16 = 1;
        take_xb(c, p);
        if (gemm_blk) { p.X = c->xpb; p.x_packed = 1; p.Y = c->actp; p.y_packed = 1; }
        if ((rc = gemm_launch<EPI_SWIGLU>(c, true, p))) return rc;
        p = gemm_base(lw.w_down, c->actb, f, M, d, f);
        if (gemm_blk) { p.X = c->actp; p.x_packed = 1; }
        if (gemm_blk) {
            p.Y = c->x; p.ldy = d;
            if ((rc = gemm_launch<EPI_RESID>(c, true, p))) return rc;
            if ((rc = launch_resid_norm(c, M, 0, next_gain))) return rc;
            c->xb_has_ssq = false;
        } else if (fused_down) {
            p.Y = c->x; p.ldy = d;
            fuse_next(c, p, next_gain);
            if ((rc = gemm_launch<EPI_RESID>(c, true, p))) return rc;
            c->xb_has_ssq = true;
        } else {
            int ks = mfma_ksplit(d, f);
            p.Y = c->part; p.ldy = d; p.y_partial = 1; p.part_rows = c->part_rows;
            if ((rc = gemm_launch<EPI_RESID>(c, true, p, ks))) return rc;
            if ((rc = launch_resid_norm(c, M, ks, next_gain))) return rc;
            c->xb_has_ssq = false;
        }
    } else {
        GemmP p = gemm_base(lw.wqkv, c->x, d, M, qkv_rows, d);
        p.gain = lw.attn_norm; p.eps = g.rms_eps;
        fill_qkv(c, p, cache, pos0, 0);
        if ((rc = gemm_launch<EPI_QKV>(c, false, p))) return rc;
        rc = launch_attention(c, cache, M, pos0, false);
        if (rc) return rc;
        p = gemm_base(lw.wo, c->attn, qd, M, d, qd);
        p.Y = c->x; p.ldy = d;
        if ((rc = gemm_launch<EPI_RESID>(c, false, p))) return rc;
        p = gemm_base(lw.w_gate_up, c->x, d, M, 2 * f, d);
        p.gain = lw.ffn_norm; p.eps = g.rms_eps;
        p.Y = c->act; p.ldy = f; p.y_bf16 = 0;
        if ((rc = gemm_launch<EPI_SWIGLU>(c, false, p))) return rc;
        p = gemm_base(lw.w_down, c->act, f, M, d, f);
        p.Y = c->x; p.ldy = d;
        if ((rc = gemm_launch<EPI_RESID>(c, false, p))) return rc;
    }
    return EESD_OK;
}

// Keys and values of the early-exit layer for the M rows in c->x (layer-N hidden states):
// only the k and v rows of its fused QKV matrix are streamed.
// MFMA family: c->xb holds RMSNorm(x; ee_layer.attn_norm) on entry.
static int run_ee_kv_fill(eesd_ctx* c, int M, int pos0, bool mfma) {
    const eesd_config& g = c->cfg;
    const int d = g.d_model, hd = g.head_dim;
    const size_t esz = is_bf16(c) ? 2 : 4;
    const char* wkv = (const char*)c->w.ee_layer.wqkv + (size_t)g.n_heads * hd * d * esz;
    const int rows = 2 * g.n_kv_heads * hd;
    int rc;
    if (mfma && c->cfg.weight_layout == EESD_WEIGHTS_TILED) {
        // tile-major: the whole fused matrix is given; tiles and groups of query heads are skipped
        GemmP p = gemm_base(c->w.ee_layer.wqkv, c->xb, d, M, (g.n_heads + 2 * g.n_kv_heads) * hd, d);
        fill_qkv(c, p, g.n_layers, pos0, 0);
        p.head_min = g.n_heads;
        take_xb(c, p);
        if (M > MAX_ROWS && c->pf_wide) { p.X = c->xpb; p.x_packed = 1; }
        if ((rc = gemm_launch<EPI_QKV>(c, true, p))) return rc;
    } else if (mfma) {
        GemmP p = gemm_base(wkv, c->xb, d, M, rows, d);
        fill_qkv(c, p, g.n_layers, pos0, g.n_heads);
        take_xb(c, p);
        if ((rc = gemm_launch<EPI_QKV>(c, true, p))) return rc;
    } else {
        GemmP p = gemm_base(wkv, c->x, d, M, rows, d);
        p.gain = c->w.ee_layer.attn_norm; p.eps = g.rms_eps;
        fill_qkv(c, p, g.n_layers, pos0, g.n_heads);
        if ((rc = gemm_launch<EPI_QKV>(c, false, p))) return rc;
    }
    return EESD_OK;
}

// logits[m][:] = RMSNorm(x[m]; norm) head^T for rows x0 .. x0+M-1 of c->x.
// MFMA family: the normalised rows are already in c->xb.
static int run_head(eesd_ctx* c, const void* norm, const void* head, int x0, int M, void* logits, bool mfma) {
    const eesd_config& g = c->cfg;
    const int d = g.d_model;
    int rc;
    if (mfma) {
        GemmP p = gemm_base(head, c->xb + (size_t)x0 * d, d, M, g.vocab, d);
        p.Y = logits; p.ldy = g.vocab; p.y_bf16 = lb16(c);
        take_xb(c, p);
        if (p.ssq_in) p.ssq_in += (size_t)x0 * p.ssq_tiles;   // partial sums are [row][tile]
        if ((rc = gemm_launch<EPI_PLAIN>(c, true, p))) return rc;
    } else {
        GemmP p = gemm_base(head, c->x + (size_t)x0 * d, d, M, g.vocab, d);
        p.gain = norm; p.eps = g.rms_eps;
        p.Y = logits; p.ldy = g.vocab;
        if ((rc = gemm_launch<EPI_PLAIN>(c, false, p))) return rc;
    }
    return EESD_OK;
}

static int launch_embed(eesd_ctx* c, const int32_t* tok_dev, int M) {
    const int d = c->cfg.d_model;
    dim3 grid((d + 255) / 256, M);
    if (is_bf16(c)) hipLaunchKernelGGL((embed_kernel<bf16_t>), grid, dim3(256), 0, c->stream, (const bf16_t*)c->w.tok_emb, tok_dev, d, c->x, d);
    else hipLaunchKernelGGL((embed_kernel<float>), grid, dim3(256), 0, c->stream, (const float*)c->w.tok_emb, tok_dev, d, c->x, d);
    HIP_TRY(c, hipGetLastError());
    return EESD_OK;
}

// x = embedding rows of the tokens and, for the MFMA family, xb = RMSNorm(x; first layer's gain): one kernel on bf16
// models (the sum of squares runs in the order of rmsnorm_bf16_kernel's waves - 16 wave sums added in order - so
// the result is that kernel's up to the order of additions inside a wave)
static int launch_embed_norm(eesd_ctx* c, const int32_t* tok_dev, int M, bool mfma) {
    const int d = c->cfg.d_model;
    if (mfma && is_bf16(c) && d % 8 == 0 && d <= RN_MAX_PIECES * 8 * EN_THREADS) {
        bf16_t* xp = (M > MAX_ROWS && c->pf_wide) ? c->xpb : nullptr;
        c->xb_has_ssq = false;
        hipLaunchKernelGGL(embed_norm_kernel, dim3(M), dim3(EN_THREADS), 0, c->stream, (const bf16_t*)c->w.tok_emb, tok_dev, c->x, d,
                           (const bf16_t*)c->layers[0].attn_norm, c->cfg.rms_eps, d, c->xb, d, xp);
        HIP_TRY(c, hipGetLastError());
        return EESD_OK;
    }
    int rc = launch_embed(c, tok_dev, M);
    if (rc) return rc;
    if (mfma && (rc = launch_rmsnorm_bf16(c, c->x, M, c->layers[0].attn_norm, c->xb, d))) return rc;
    return EESD_OK;
}

// Target forward over M rows whose tokens are tok_dev[0..M) at positions pos0.. :
// all L layers (plus the early-exit layer's K/V after layer N); leaves hidden states in c->x
// and, in the MFMA family, RMSNorm(x; final_norm) in c->xb.
static int run_target_rows(eesd_ctx* c, const int32_t* tok_dev, int M, int pos0, bool mfma) {
    const eesd_config& g = c->cfg;
    int rc = launch_embed_norm(c, tok_dev, M, mfma);
    if (rc) return rc;
    for (int l = 0; l < g.n_layers; ++l) {
        const bool ee_next = (l + 1 == g.n_draft_layers);
        const void* next_gain = ee_next ? c->w.ee_layer.attn_norm : (l + 1 < g.n_layers ? c->layers[l + 1].attn_norm : c->w.final_norm);
        if ((rc = run_layer(c, c->layers[l], l, M, pos0, mfma, next_gain))) return rc;
        if (ee_next) {
            if ((rc = run_ee_kv_fill(c, M, pos0, mfma))) return rc;
            // N < L always: the next target layer wants its own normalised copy
            if (mfma && (rc = launch_rmsnorm_bf16(c, c->x, M, c->layers[l + 1].attn_norm, c->xb, g.d_model))) return rc;
        }
    }
    return EESD_OK;
}

// The verify block [pending, d_1..d_K] when the K draft steps kept their layer-N hidden states
// (rows 0..K-1; their keys and values of layers 1..N and of the early-exit layer are in the caches
// already): layers 1..N and the early-exit K/V for the last draft token alone, then layers N+1..L
// on all K+1 rows.  Leaves what run_target_rows leaves.
static int run_target_rows_reusing(eesd_ctx* c, int K, int pos0) {
    const eesd_config& g = c->cfg;
    const int d = g.d_model, N = g.n_draft_layers, M = K + 1;
    const bool mfma1 = pick_mfma(c, 1), mfmaM = pick_mfma(c, M);
    int rc = launch_embed_norm(c, c->blk_tok + K, 1, mfma1);
    if (rc) return rc;
    for (int l = 0; l < N; ++l) {
        const void* next_gain = l + 1 < N ? c->layers[l + 1].attn_norm : c->w.ee_layer.attn_norm;
        if ((rc = run_layer(c, c->layers[l], l, 1, pos0 + K, mfma1, next_gain))) return rc;
    }
    if ((rc = run_ee_kv_fill(c, 1, pos0 + K, mfma1))) return rc;
    hipLaunchKernelGGL(assemble_rows_kernel, dim3((d + 255) / 256), dim3(256), 0, c->stream, c->x, c->hn_rows, K, d);
    HIP_TRY(c, hipGetLastError());
    if (mfmaM && (rc = launch_rmsnorm_bf16(c, c->x, M, c->layers[N].attn_norm, c->xb, d))) return rc;
    for (int l = N; l < g.n_layers; ++l) {
        const void* next_gain = l + 1 < g.n_layers ? c->layers[l + 1].attn_norm : c->w.final_norm;
        if ((rc = run_layer(c, c->layers[l], l, M, pos0, mfmaM, next_gain))) return rc;
    }
    return EESD_OK;
}

// ---------------------------------------------------------------------------------------------
// paged cache bookkeeping
// ---------------------------------------------------------------------------------------------
static int ensure_pages(eesd_ctx* c, int n_tokens) {
    int need = (n_tokens + c->page_tokens - 1) >> c->page_shift;
    if (need > c->n_pages) return fail(c, EESD_ERANGE, "KV cache full: %d tokens wanted, max_seq %d", n_tokens, c->cfg.max_seq);
    int first = c->mapped_pages;
    while (c->mapped_pages < need) {
        if (c->free_pages.empty()) return fail(c, EESD_ENOMEM, "KV page pool exhausted");
        c->h_table[c->mapped_pages++] = c->free_pages.back();
        c->free_pages.pop_back();
    }
    if (c->mapped_pages > first)
        HIP_TRY(c, hipMemcpyAsync(c->d_table + first, c->h_table + first, sizeof(int32_t) * (c->mapped_pages - first),
                                  hipMemcpyHostToDevice, c->stream));
    return EESD_OK;
}

// pages wholly past n_tokens go back to the pool (callers have synchronised the stream)
static void release_pages(eesd_ctx* c, int n_tokens) {
    int keep = (n_tokens + c->page_tokens - 1) >> c->page_shift;
    while (c->mapped_pages > keep) {
        --c->mapped_pages;
        c->free_pages.push_back(c->h_table[c->mapped_pages]);
        c->h_table[c->mapped_pages] = -1;
    }
}

// ---------------------------------------------------------------------------------------------
// controller (Section 3.3, Algorithm 2)
// ---------------------------------------------------------------------------------------------
// theta ~ Beta(a, b).  Integer parameters: the a-th smallest of a+b-1 uniforms (exact, needs
// comparisons only).  Otherwise the ratio of two Marsaglia-Tsang gamma variates.
static double gamma_mt(double shape, uint64_t seed, int64_t rnd, int slot, int& sub) {
    double boost = 1.0;
    if (shape < 1.0) {
        boost = pow(uniform53(seed, STREAM_TS_THETA, rnd, slot, sub++), 1.0 / shape);
        shape += 1.0;
    }
    const double d = shape - 1.0 / 3.0, cc = 1.0 / sqrt(9.0 * d);
    for (;;) {
        double u1 = uniform53(seed, STREAM_TS_THETA, rnd, slot, sub++), u2 = uniform53(seed, STREAM_TS_THETA, rnd, slot, sub++);
        double n = sqrt(-2.0 * log(1.0 - u1)) * cos(6.283185307179586 * u2);
        double v = 1.0 + cc * n;
        if (v <= 0.0) continue;
        v = v * v * v;
        double u = uniform53(seed, STREAM_TS_THETA, rnd, slot, sub++);
        if (log(1.0 - u) < 0.5 * n * n + d - d * v + d * log(v)) return boost * d * v;
    }
}

static double beta_draw_at(double a, double b, uint64_t seed, int64_t rnd, int slot) {
    if (a == floor(a) && b == floor(b) && a + b < 1e6) {
        int ia = (int)a, n = (int)(a + b) - 1;
        std::vector<double> us(n);
        for (int j = 0; j < n; ++j) us[j] = uniform53(seed, STREAM_TS_THETA, rnd, slot, j);
        std::nth_element(us.begin(), us.begin() + (ia - 1), us.end());
        return us[ia - 1];
    }
    int sub = 0;
    double x = gamma_mt(a, seed, rnd, slot, sub), y = gamma_mt(b, seed, rnd, slot, sub);
    return x / (x + y);
}

// Algorithm 2, steps 5-14 for one round: draft, draw theta from the posterior the round starts
// with, draw chi ~ Bernoulli(theta), stop on chi = 0 or at k_max drafts.
static int beta_ts_draw_k(double alpha, double beta, uint64_t seed, int64_t rnd, int k_max) {
    if (k_max < 1) k_max = 1;
    int k = 0;
    for (;;) {
        ++k;                                  // draft token k
        if (k >= k_max) return k_max;
        double theta = beta_draw_at(alpha, beta, seed, rnd, k);
        bool chi = uniform53(seed, STREAM_TS_CHI, rnd, k, 0) < theta;
        if (!chi) return k;
    }
}

// Eq. 3-4: alpha += r, beta += n - r (the two readings of n differ, see eesd_config.ts_update)
static void beta_ts_update(double* alpha, double* beta, int a, int K, int reading) {
    if (K < 1) return;
    int r = a;
    int n = reading == 0 ? std::min(a + 1, K) : std::min(a + 2, K);
    *alpha += r;
    *beta += n - r;
}

// K of the coming round.  Every theta of a round is drawn from the posterior the round starts
// with (Algorithm 2 indexes it by t), so K is known before the first draft step is launched.
static int draw_k(eesd_ctx* c, int k_max) {
    if (k_max < 1) k_max = 1;
    if (c->cfg.ts_mode == EESD_TS_FIXED) return std::min((int)c->cfg.k_cap, k_max);
    if (c->cfg.ts_mode == EESD_TS_SCHEDULE) {
        int k = c->cfg.k_cap;
        if (!c->schedule.empty()) k = c->schedule[std::min<size_t>((size_t)c->sched_round, c->schedule.size() - 1)];
        ++c->sched_round;
        return std::max(1, std::min(k, k_max));
    }
    return beta_ts_draw_k(c->alpha, c->beta, c->cfg.seed, c->round, k_max);
}

static void ts_update(eesd_ctx* c, int a, int K) { beta_ts_update(&c->alpha, &c->beta, a, K, c->cfg.ts_update); }

// ---- calibrated controller (Section 3.3 Eq. 6-8, Algorithm 3), host side ----
// standard normal from two counter-based uniforms (Box-Muller, cosine branch)
static double normal_draw(uint64_t seed, int64_t rnd, int slot) {
    const double u1 = uniform53(seed, STREAM_TS_THETA, rnd, slot, 0), u2 = uniform53(seed, STREAM_TS_THETA, rnd, slot, 1);
    return sqrt(-2.0 * log(1.0 - u1)) * cos(2.0 * M_PI * u2);
}

// theta ~ N(mu, sigma^2) with the posterior of Eq. 6-7; chi ~ Bernoulli(theta)
static bool cali_decide(double sigma_m, double sigma_s, double theta_hat, int64_t n, double theta_m, uint64_t seed, int64_t rnd, int slot,
                        double* theta_out) {
    const double sm2 = sigma_m * sigma_m, ss2 = sigma_s * sigma_s, dn = (double)n;
    const double mu = ss2 / (dn * sm2 + ss2) * theta_m + dn * sm2 / (dn * sm2 + ss2) * theta_hat;
    const double var = sm2 * ss2 / (ss2 + dn * sm2);
    const double theta = mu + sqrt(var) * normal_draw(seed, rnd, slot);
    if (theta_out) *theta_out = theta;
    return uniform53(seed, STREAM_TS_CHI, rnd, slot, 0) < theta;
}

// Eq. 8: running mean of the observed chi (reading 0: what the target judged; 1: as printed)
static void cali_update(double* theta_hat, double* weight, int64_t* n, int a, int K, int reading) {
    *n += 1;
    const int fresh = reading == 0 ? std::min(a + 1, K) : a;
    if (fresh) {
        *theta_hat = (*theta_hat * *weight + (double)a) / (*weight + (double)fresh);
        *weight += (double)fresh;
    }
}

// Host-only entry points (no GPU needed): the controller and the uniform generator as the
// library uses them, so that they can be checked without a device.
extern "C" double eesd_host_uniform(uint64_t seed, int32_t stream, int64_t round, int32_t slot, int32_t sub) {
    return uniform53(seed, stream, round, slot, sub);
}
extern "C" int eesd_host_draw_k(double alpha, double beta, uint64_t seed, int64_t round, int32_t k_max) {
    if (!(alpha > 0.0) || !(beta > 0.0)) return EESD_EINVAL;
    return beta_ts_draw_k(alpha, beta, seed, round, k_max);
}
// The element offsets of the two operand-order layouts, as the kernels compute them.
extern "C" int64_t eesd_host_layout_offset(int32_t what, int32_t a, int32_t b, int32_t n) {
    if (a < 0 || b < 0 || n < 1) return -1;
    if (what == 0) return n % 32 ? -1 : (int64_t)kv_tiled_k(a, b, n);       // key slot a (inside its page), channel b, head_dim n
    if (what == 1) return n % 32 ? -1 : (int64_t)kv_tiled_v(a, b, n);       // value slot a, channel b, head_dim n
    if (what == 2) return (int64_t)act_packed_offset(a, b, n);               // activation row a, column b, n = columns / 32
    if (what == 3 || what == 4) {                                             // row group a of a matrix of b rows on n CUs: first row / rows
        if (b < 16 || b % 16) return -1;
        const int groups = pack_n_groups(b, n);
        if (a >= groups) return -1;
        const GroupGeom gg = group_geom(a, groups, b);
        return what == 3 ? gg.row0 : gg.rows;
    }
    if (what == 5) return (b < 16 || b % 16) ? -1 : pack_n_groups(b, n);     // row groups of a matrix of b rows on n CUs
    return -1;
}
extern "C" int eesd_host_ts_update(double* alpha, double* beta, int32_t n_accepted, int32_t n_drafted, int32_t reading) {
    if (!alpha || !beta || n_accepted < 0 || n_accepted > n_drafted || reading < 0 || reading > 1) return EESD_EINVAL;
    beta_ts_update(alpha, beta, n_accepted, n_drafted, reading);
    return EESD_OK;
}

extern "C" int eesd_host_cali_decide(double sigma_m, double sigma_s, double theta_hat, int64_t n, double theta_m, uint64_t seed,
                                     int64_t round, int32_t slot, double* theta, int32_t* chi) {
    if (!chi || !(sigma_m > 0.0) || !(sigma_s > 0.0) || n < 0) return EESD_EINVAL;
    *chi = cali_decide(sigma_m, sigma_s, theta_hat, n, theta_m, seed, round, slot, theta) ? 1 : 0;
    return EESD_OK;
}
extern "C" int eesd_host_cali_update(double* theta_hat, double* weight, int64_t* n, int32_t n_accepted, int32_t n_drafted, int32_t reading) {
    if (!theta_hat || !weight || !n || n_accepted < 0 || n_drafted < n_accepted || reading < 0 || reading > 1) return EESD_EINVAL;
    cali_update(theta_hat, weight, n, n_accepted, n_drafted, reading);
    return EESD_OK;
}

static void finish_stats(eesd_ctx* c) {
    eesd_stats& s = c->stats;
    s.v_d = s.drafted ? (double)s.accepted / (double)s.drafted : 0.0;
    s.r_d = s.generated ? (double)s.accepted / (double)s.generated : 0.0;
    s.hm = (s.v_d + s.r_d) > 0 ? 2.0 * s.v_d * s.r_d / (s.v_d + s.r_d) * 100.0 : 0.0;
    s.alpha = c->alpha;
    s.beta = c->beta;
}

// ---------------------------------------------------------------------------------------------
// create / destroy
// ---------------------------------------------------------------------------------------------
static const char* k_no_ctx = "no context";

template <typename T>
static int dev_alloc(eesd_ctx* c, T** p, size_t n) {
    hipError_t e = hipMalloc((void**)p, n * sizeof(T));
    if (e != hipSuccess) return fail(c, EESD_ENOMEM, "hipMalloc(%zu bytes): %s", n * sizeof(T), hipGetErrorString(e));
    return EESD_OK;
}

extern "C" void eesd_destroy(eesd_ctx* c) {
    if (!c) return;
    hipStreamSynchronize(c->stream);
    void* dev[] = {c->kv_pool, c->d_table, c->x, c->q, c->attn, c->act, c->logits, c->p_rows, c->q_logits, c->q_rows, c->part_o,
                   c->part_ml, c->rope_cs, c->part, c->ssq, c->xb, c->xpb, c->abp, c->actp, c->spl_buf, c->ab, c->actb, c->blk_tok, c->prompt_dev, c->result_dev, c->tree_blk, c->h_t, c->cali_u, c->theta_dev, c->h_tb, c->hn_rows};
    for (void* p : dev)
        if (p) hipFree(p);
    if (c->h_table) hipHostFree(c->h_table);
    if (c->h_result) hipHostFree(c->h_result);
    if (c->h_prompt) hipHostFree(c->h_prompt);
    for (auto& e : c->ev)
        if (e) hipEventDestroy(e);
    for (auto& e : c->prof_ev) hipEventDestroy(e);
    delete c;
}

extern "C" int eesd_create(const eesd_config* cfg, const eesd_weights* w, void* hip_stream, eesd_ctx** out) {
    if (!cfg || !w || !out || !w->layers) return EESD_EINVAL;
    const eesd_config& g = *cfg;
    if (g.n_layers < 2 || g.n_draft_layers < 1 || g.n_draft_layers >= g.n_layers) return EESD_EINVAL;
    if (g.d_model < 8 || g.n_heads < 1 || g.n_kv_heads < 1 || g.n_heads % g.n_kv_heads) return EESD_EINVAL;
    if (g.head_dim != 64 && g.head_dim != 128) return EESD_EINVAL;
    if (g.d_ff < 8 || g.vocab < 2 || g.max_seq < 2 || g.k_cap < 1 || g.k_cap > ACC_MAX_K) return EESD_EINVAL;
    if (g.kv_page < 16 || (g.kv_page & (g.kv_page - 1))) return EESD_EINVAL;
    if (g.dtype != EESD_DTYPE_F32 && g.dtype != EESD_DTYPE_BF16) return EESD_EINVAL;
    if (!(g.temperature >= 0.0f) || !(g.ts_alpha0 > 0.0) || !(g.ts_beta0 > 0.0)) return EESD_EINVAL;
    if (g.ts_mode < 0 || g.ts_mode > 3 || g.ts_update < 0 || g.ts_update > 1 || g.gemm_path < 0 || g.gemm_path > 2) return EESD_EINVAL;
    if (g.tree_width < 0 || g.tree_width > TREE_MAX_WIDTH) return EESD_EINVAL;
    if (g.verify_reuse < 0 || g.verify_reuse > 1) return EESD_EINVAL;
    if (g.logits_bf16 < 0 || g.logits_bf16 > 1 || (g.logits_bf16 == 1 && (g.dtype != EESD_DTYPE_BF16 || g.gemm_path == EESD_GEMM_VALU))) return EESD_EINVAL;
    if (g.weight_layout != EESD_WEIGHTS_ROW_MAJOR && g.weight_layout != EESD_WEIGHTS_TILED) return EESD_EINVAL;
    if (g.weight_layout == EESD_WEIGHTS_TILED && (g.dtype != EESD_DTYPE_BF16 || g.gemm_path == EESD_GEMM_VALU)) return EESD_EINVAL;
    if (g.tree_width >= 2 && (g.temperature != 0.0f || 1 + g.k_cap * g.tree_width > MAX_ROWS)) return EESD_EINVAL;
    const int vec = g.dtype == EESD_DTYPE_BF16 ? 8 : 4;
    const int qd = g.n_heads * g.head_dim;
    if (g.d_model % vec || g.d_ff % vec || qd % vec || g.vocab % 4 || g.d_ff % 2) return EESD_EINVAL;
    if (g.dtype == EESD_DTYPE_BF16) {
        // the MFMA family needs 128-column steps and 32-row blocks
        if (g.d_model % 128 || g.d_ff % 128 || qd % 128 || g.vocab % 32 || g.d_model % 32 || (g.d_ff % 16)) return EESD_EINVAL;
        // one workgroup of the MFMA attention holds all query rows of a KV head: 16 rows x group <= 128
        if (g.n_heads / g.n_kv_heads > 8) return EESD_EINVAL;
        if (g.d_model > RN_MAX_PIECES * 8 * 1024) return EESD_EINVAL;
    }
    // whenever the VALU family may see a full block of rows its activations must fit in LDS
    if ((g.dtype == EESD_DTYPE_F32 || g.gemm_path == EESD_GEMM_VALU) &&
        valu_lds_bytes(MAX_ROWS, std::max(std::max(g.d_model, g.d_ff), qd)) > 150 * 1024)
        return EESD_EINVAL;
    if (valu_lds_bytes(1, std::max(std::max(g.d_model, g.d_ff), qd)) > 150 * 1024) return EESD_EINVAL;
    const void* ptrs[] = {w->tok_emb, w->final_norm, w->lm_head, w->ee_norm, w->ee_head, w->ee_layer.attn_norm, w->ee_layer.wqkv,
                          w->ee_layer.wo, w->ee_layer.ffn_norm, w->ee_layer.w_gate_up, w->ee_layer.w_down};
    for (const void* p : ptrs)
        if (!p) return EESD_EINVAL;
    for (int l = 0; l < g.n_layers; ++l) {
        const eesd_layer_weights& lw = w->layers[l];
        if (!lw.attn_norm || !lw.wqkv || !lw.wo || !lw.ffn_norm || !lw.w_gate_up || !lw.w_down) return EESD_EINVAL;
    }

    eesd_ctx* c = new (std::nothrow) eesd_ctx();
    if (!c) return EESD_ENOMEM;
    c->cfg = g;
    c->layers.assign(w->layers, w->layers + g.n_layers);
    c->w = *w;
    c->w.layers = c->layers.data();
    c->stream = (hipStream_t)hip_stream;
    c->state = ST_CREATED;
    c->kv_pool = nullptr; c->d_table = nullptr; c->h_table = nullptr;
    c->x = c->q = c->attn = c->act = c->logits = c->p_rows = c->q_logits = c->q_rows = c->part_o = c->part_ml = c->rope_cs = c->part = c->ssq = nullptr;
    c->xb_has_ssq = false;
    c->xb = c->ab = c->actb = c->xpb = c->abp = c->actp = nullptr;
    c->spl_buf = nullptr;
    c->blk_tok = c->prompt_dev = c->result_dev = c->tree_blk = nullptr;
    c->h_t = c->cali_u = c->theta_dev = nullptr; c->h_tb = nullptr; c->hn_rows = nullptr;
    c->cali_set = false; memset(&c->cali, 0, sizeof c->cali);
    c->cali_theta_hat = 0.0; c->cali_weight = 1.0; c->cali_n = 0;
    c->tree_active = false;
    c->h_result = c->h_prompt = nullptr;
    for (auto& e : c->ev) e = nullptr;
    c->alpha = g.ts_alpha0; c->beta = g.ts_beta0;
    c->sched_round = 0; c->round = 0; c->kv_len = 0; c->n_drafted = 0; c->forced_pos = 0;
    c->prof_family = -1; c->prof_epi = 0; c->prof_in = 0; c->prof_used = 0;
    memset(&c->stats, 0, sizeof c->stats);
    memset(c->launch_counts, 0, sizeof c->launch_counts);

    int rc = EESD_OK;
    auto bail = [&](int code) { std::string e = c->err; eesd_destroy(c); (void)e; return code; };
    if (hipGetDevice(&c->device) != hipSuccess) return bail(EESD_EDEVICE);

    // paged cache
    c->n_caches = g.n_layers + 1;
    c->page_tokens = g.kv_page;
    c->page_shift = 0;
    while ((1 << c->page_shift) < g.kv_page) ++c->page_shift;
    c->n_pages = (g.max_seq + g.kv_page - 1) / g.kv_page;
    c->elem = g.dtype == EESD_DTYPE_BF16 ? 2 : 4;
    c->page_stride = (long long)c->n_caches * 2 * g.n_kv_heads * g.kv_page * g.head_dim;
    size_t pool_bytes = (size_t)c->page_stride * c->n_pages * c->elem;
    if (hipMalloc(&c->kv_pool, pool_bytes) != hipSuccess) return bail(EESD_ENOMEM);
    if ((rc = dev_alloc(c, &c->d_table, c->n_pages))) return bail(rc);
    if (hipHostMalloc((void**)&c->h_table, sizeof(int32_t) * c->n_pages, hipHostMallocDefault) != hipSuccess) return bail(EESD_ENOMEM);
    if (hipHostMalloc((void**)&c->h_result, sizeof(int32_t) * H_RESULT_INTS, hipHostMallocDefault) != hipSuccess) return bail(EESD_ENOMEM);
    if (hipHostMalloc((void**)&c->h_prompt, sizeof(int32_t) * g.max_seq, hipHostMallocDefault) != hipSuccess) return bail(EESD_ENOMEM);
    // physical pages are handed out in reverse order, so logical != physical from the start
    for (int p = 0; p < c->n_pages; ++p) { c->free_pages.push_back(p); c->h_table[p] = -1; }
    c->mapped_pages = 0;

    const int d = g.d_model, f = g.d_ff, V = g.vocab;
    c->max_splits = 64;
    c->n_cu = device_cu_count();
    if (c->n_cu < 1) return bail(EESD_EDEVICE);
    {
        const bool grouped = g.weight_layout == EESD_WEIGHTS_TILED && pack_n_groups(d, c->n_cu) != d / 16;
        // a residual product leaves one partial sum of squares per row and tile: d / 16, or, dealt to one row group per CU,
        // (tiles of the largest group) per group
        const int tmax = ((((d / 4) + c->n_cu - 1) / c->n_cu) * 4 + 15) / 16;
        c->ssq_slots = grouped ? c->n_cu * tmax : d / 16;
    }
    {
        const int qkv_rows = (g.n_heads + 2 * g.n_kv_heads) * g.head_dim, kv_rows = 2 * g.n_kv_heads * g.head_dim;
        bool tiled = g.dtype == EESD_DTYPE_BF16 && g.gemm_path != EESD_GEMM_VALU && tile_shape_ok(qkv_rows, d) && tile_shape_ok(kv_rows, d) &&
                     tile_shape_ok(d, qd) && tile_shape_ok(2 * f, d) && tile_shape_ok(d, f) && tile_shape_ok(V, d);
        c->row_cap = tiled ? PREFILL_ROWS : MAX_ROWS;
        const int chunk = 32 * PF_QC;
        c->pf_wide = g.dtype == EESD_DTYPE_BF16 && g.gemm_path != EESD_GEMM_VALU && g.weight_layout == EESD_WEIGHTS_TILED && g_pf_rows != 128 &&
                     d % chunk == 0 && qd % chunk == 0 && f % chunk == 0 && d % 16 == 0 && f % 8 == 0;
        if (c->pf_wide) c->row_cap = g_pf_rows == 256 ? 256 : PREFILL_ROWS_WIDE;
        c->part_rows = std::min(c->row_cap, PREFILL_ROWS);
    }
    const size_t R = c->row_cap;
    if ((rc = dev_alloc(c, &c->x, R * d))) return bail(rc);
    if ((rc = dev_alloc(c, &c->q, R * qd))) return bail(rc);
    if ((rc = dev_alloc(c, &c->attn, R * qd))) return bail(rc);
    if ((rc = dev_alloc(c, &c->act, R * f))) return bail(rc);
    if ((rc = dev_alloc(c, &c->logits, (size_t)MAX_ROWS * V))) return bail(rc);
    if ((rc = dev_alloc(c, &c->p_rows, (size_t)MAX_ROWS * V))) return bail(rc);
    if ((rc = dev_alloc(c, &c->q_logits, (size_t)g.k_cap * V))) return bail(rc);
    if ((rc = dev_alloc(c, &c->q_rows, (size_t)g.k_cap * V))) return bail(rc);
    if ((rc = dev_alloc(c, &c->part_o, (size_t)MAX_ROWS * g.n_heads * c->max_splits * g.head_dim))) return bail(rc);
    if ((rc = dev_alloc(c, &c->part_ml, (size_t)MAX_ROWS * g.n_heads * c->max_splits * 2))) return bail(rc);
    if ((rc = dev_alloc(c, &c->part, (size_t)MFMA_MAX_KSPLIT * c->part_rows * d))) return bail(rc);
    if ((rc = dev_alloc(c, &c->ssq, (size_t)c->ssq_slots * MAX_ROWS))) return bail(rc);
    hipMemset(c->ssq, 0, sizeof(float) * c->ssq_slots * MAX_ROWS);
    if (c->pf_wide) {
        if ((rc = dev_alloc(c, &c->xpb, R * d))) return bail(rc);
        if ((rc = dev_alloc(c, &c->abp, R * qd))) return bail(rc);
        if ((rc = dev_alloc(c, &c->actp, R * f))) return bail(rc);
        // tokens past a block's last row keep whatever the buffers held: their products are never stored
        hipMemset(c->xpb, 0, sizeof(bf16_t) * R * d);
        hipMemset(c->abp, 0, sizeof(bf16_t) * R * qd);
        hipMemset(c->actp, 0, sizeof(bf16_t) * R * f);
    }
    if ((rc = dev_alloc(c, &c->xb, R * d))) return bail(rc);
    if ((rc = dev_alloc(c, &c->ab, R * qd))) return bail(rc);
    if ((rc = dev_alloc(c, &c->actb, R * f))) return bail(rc);
    if ((rc = dev_alloc(c, &c->spl_buf, (size_t)SPL_SCRATCH_BYTES))) return bail(rc);
    if ((rc = dev_alloc(c, &c->blk_tok, (size_t)MAX_ROWS + 1))) return bail(rc);
    if ((rc = dev_alloc(c, &c->prompt_dev, (size_t)g.max_seq))) return bail(rc);
    if ((rc = dev_alloc(c, &c->result_dev, (size_t)2 + MAX_ROWS))) return bail(rc);
    if ((rc = dev_alloc(c, &c->tree_blk, (size_t)MAX_ROWS + 1))) return bail(rc);
    if ((rc = dev_alloc(c, &c->h_t, (size_t)g.d_model))) return bail(rc);
    if ((rc = dev_alloc(c, &c->cali_u, (size_t)g.d_model))) return bail(rc);
    if ((rc = dev_alloc(c, &c->theta_dev, (size_t)4))) return bail(rc);
    if ((rc = dev_alloc(c, &c->h_tb, (size_t)g.d_model))) return bail(rc);
    if ((rc = dev_alloc(c, &c->hn_rows, (size_t)g.k_cap * g.d_model))) return bail(rc);
    // rows of the bf16 activation buffers past M are read (and ignored) by the MFMA product
    hipMemset(c->xb, 0, sizeof(bf16_t) * R * d);
    hipMemset(c->ab, 0, sizeof(bf16_t) * R * qd);
    hipMemset(c->actb, 0, sizeof(bf16_t) * R * f);
    hipMemset(c->d_table, 0, sizeof(int32_t) * c->n_pages);
    hipMemset(c->kv_pool, 0, pool_bytes);

    // rotary table: cos/sin(pos * base^(-2j/hd)) evaluated in double, stored fp32
    {
        const int half = g.head_dim / 2;
        std::vector<float> cs((size_t)g.max_seq * half * 2);
        for (int p = 0; p < g.max_seq; ++p)
            for (int j = 0; j < half; ++j) {
                double ang = (double)p * pow((double)g.rope_base, -2.0 * j / (double)g.head_dim);
                cs[((size_t)p * half + j) * 2] = (float)cos(ang);
                cs[((size_t)p * half + j) * 2 + 1] = (float)sin(ang);
            }
        if ((rc = dev_alloc(c, &c->rope_cs, cs.size()))) return bail(rc);
        if (hipMemcpy(c->rope_cs, cs.data(), cs.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return bail(EESD_EDEVICE);
    }
    for (auto& e : c->ev)
        if (hipEventCreate(&e) != hipSuccess) return bail(EESD_EDEVICE);
    if (hipDeviceSynchronize() != hipSuccess) return bail(EESD_EDEVICE);
    *out = c;
    return EESD_OK;
}

extern "C" const char* eesd_last_error(const eesd_ctx* c) { return c ? c->err.c_str() : k_no_ctx; }

extern "C" int eesd_get_stats(const eesd_ctx* c, eesd_stats* out) {
    if (!c || !out) return EESD_EINVAL;
    finish_stats(const_cast<eesd_ctx*>(c));
    *out = c->stats;
    return EESD_OK;
}

// ---------------------------------------------------------------------------------------------
// the calls of a round
// ---------------------------------------------------------------------------------------------
// the sampling kernels keep a vocabulary row in LDS when it fits
static int smp_use_lds(int V) { return V <= SMP_LDS_MAX_V; }
static size_t smp_lds_bytes(int V) { return smp_use_lds(V) ? (size_t)V * sizeof(float) : 0; }
template <typename F>
static hipError_t smp_allow(F fn, int V) { return allow_lds((const void*)fn, smp_lds_bytes(V)); }

static float inv_temperature(const eesd_ctx* c) { return c->cfg.temperature > 0.f ? 1.0f / c->cfg.temperature : 1.0f; }
static int greedy(const eesd_ctx* c) { return c->cfg.temperature == 0.f; }

// The predictor's H_t^(T): row `row` of the hidden states the last target pass left in c->x.
static int save_target_hidden(eesd_ctx* c, int row) {
    if (!c->cali_set) return EESD_OK;
    const int d = c->cfg.d_model;
    hipLaunchKernelGGL(save_hidden_kernel, dim3((d + 255) / 256), dim3(256), 0, c->stream, c->x + (size_t)row * d, c->h_t, c->h_tb, d);
    HIP_TRY(c, hipGetLastError());
    return EESD_OK;
}

static bool reuse_hn(const eesd_ctx* c) { return c->cfg.verify_reuse == 1 && c->cfg.tree_width < 2; }

static int tree_width(const eesd_ctx* c) { return c->cfg.tree_width >= 2 ? c->cfg.tree_width : 1; }
// most rows a verify block can have
static int rows_cap(const eesd_ctx* c) { return 1 + c->cfg.k_cap * tree_width(c); }

// softmax(row / T) -> probs, draw with u (greedy: argmax); the row is fp32 or bf16 logits
// whether a draft step at temperature > 0 samples with the three kernels spread over the chip (sampling.hiph)
static bool smp_spread(int V) { return V <= SPL_MAX_V && (g_smp_spread < 0 ? V >= 4096 : g_smp_spread != 0); }

template <typename LT>
static hipError_t launch_spread_sample(hipStream_t st, const LT* row, float* probs, int V, float inv_t, double u, int forced, SplScratch sc,
                                       int32_t* tok_out) {
    hipLaunchKernelGGL(softmax_part_kernel<LT>, dim3(SPL_CHUNKS), dim3(SPL_THREADS), 0, st, row, V, inv_t, sc);
    hipLaunchKernelGGL(softmax_norm_kernel<LT>, dim3(SPL_CHUNKS), dim3(SPL_THREADS), 0, st, row, probs, V, inv_t, sc);
    hipLaunchKernelGGL(sample_pick_kernel, dim3(1), dim3(64), 0, st, (const float*)probs, V, u, forced, sc, tok_out);
    return hipGetLastError();
}

// the verify side of the same: all K + 1 rows at once
template <typename LT>
static hipError_t launch_spread_accept(hipStream_t st, const LT* p_logits, float* p_rows, const float* q_rows, const int32_t* drafts, int K, int V,
                                       float inv_t, const AcceptU& uu, SplScratch sc, int32_t* result, int32_t* pending_out) {
    hipLaunchKernelGGL(softmax_part_kernel<LT>, dim3(SPL_CHUNKS, K + 1), dim3(SPL_THREADS), 0, st, p_logits, V, inv_t, sc);
    hipLaunchKernelGGL(accept_norm_kernel<LT>, dim3(SPL_CHUNKS, K + 1), dim3(SPL_THREADS), 0, st, p_logits, p_rows, q_rows, drafts, K, V, inv_t, uu, sc);
    hipLaunchKernelGGL(accept_pick_kernel, dim3(1), dim3(64), 0, st, (const float*)p_rows, q_rows, K, V, uu.u[K], sc, result, pending_out);
    return hipGetLastError();
}

static hipError_t launch_softmax_sample(eesd_ctx* c, const void* row, float* probs, double u, int forced, int32_t* tok_out) {
    const int V = c->cfg.vocab;
    if (!greedy(c) && smp_spread(V)) {
        const SplScratch sc = spl_scratch(c->spl_buf);
        return lb16(c) ? launch_spread_sample(c->stream, (const bf16_t*)row, probs, V, inv_temperature(c), u, forced, sc, tok_out)
                       : launch_spread_sample(c->stream, (const float*)row, probs, V, inv_temperature(c), u, forced, sc, tok_out);
    }
    if (lb16(c)) {
        hipError_t e = smp_allow(softmax_sample_kernel<bf16_t>, V);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(softmax_sample_kernel<bf16_t>, dim3(1), dim3(SMP_THREADS), smp_lds_bytes(V), c->stream, (const bf16_t*)row, probs, V,
                           inv_temperature(c), greedy(c), u, forced, tok_out, smp_use_lds(V));
    } else {
        hipError_t e = smp_allow(softmax_sample_kernel<float>, V);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(softmax_sample_kernel<float>, dim3(1), dim3(SMP_THREADS), smp_lds_bytes(V), c->stream, (const float*)row, probs, V,
                           inv_temperature(c), greedy(c), u, forced, tok_out, smp_use_lds(V));
    }
    return hipGetLastError();
}

static void reset_sequence(eesd_ctx* c) {
    release_pages(c, 0);
    c->kv_len = 0; c->n_drafted = 0; c->round = 0; c->sched_round = 0;
    c->alpha = c->cfg.ts_alpha0; c->beta = c->cfg.ts_beta0;
    c->forced.clear(); c->forced_pos = 0;
    memset(&c->stats, 0, sizeof c->stats);
    c->cali_theta_hat = c->cali.theta_hat0; c->cali_weight = 1.0; c->cali_n = 0;
}

extern "C" int eesd_prefill(eesd_ctx* c, const int32_t* prompt, int32_t n, int32_t* first_token) {
    if (!c) return EESD_EINVAL;
    if (!prompt || !first_token || n < 1) return fail(c, EESD_EINVAL, "prefill: null pointer or empty prompt");
    const eesd_config& g = c->cfg;
    if (n + rows_cap(c) > g.max_seq) return fail(c, EESD_ERANGE, "prefill: prompt of %d tokens + a verify block of %d rows exceeds max_seq %d", n, rows_cap(c), g.max_seq);
    for (int i = 0; i < n; ++i)
        if (prompt[i] < 0 || prompt[i] >= g.vocab) return fail(c, EESD_EINVAL, "prefill: token %d at %d outside [0,%d)", prompt[i], i, g.vocab);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    reset_sequence(c);
    c->state = ST_CREATED;
    memcpy(c->h_prompt, prompt, sizeof(int32_t) * n);
    HIP_TRY(c, hipMemcpyAsync(c->prompt_dev, c->h_prompt, sizeof(int32_t) * n, hipMemcpyHostToDevice, c->stream));
    int rc = ensure_pages(c, n);
    if (rc) return rc;
    int last_m = 0;
    bool last_mfma = false;
    for (int p0 = 0; p0 < n; p0 += c->row_cap) {
        int m = std::min(c->row_cap, n - p0);
        last_mfma = pick_mfma(c, m);
        rc = run_target_rows(c, c->prompt_dev + p0, m, p0, last_mfma);
        if (rc) return rc;
        last_m = m;
    }
    if ((rc = save_target_hidden(c, last_m - 1))) return rc;
    // logits of the last prompt position only (the family of the last block left its input ready)
    rc = run_head(c, c->w.final_norm, c->w.lm_head, last_m - 1, 1, c->logits, last_mfma);
    if (rc) return rc;
    double u = uniform53(g.seed, STREAM_RESAMPLE, 0, 0, 0);
    HIP_TRY(c, launch_softmax_sample(c, c->logits, c->p_rows, u, -1, c->blk_tok));
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipMemcpyAsync(c->h_result, c->blk_tok, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->kv_len = n;
    c->n_drafted = 0;
    c->round = 1;
    c->state = ST_READY;
    *first_token = c->h_result[0];
    return EESD_OK;
}

extern "C" int eesd_draft_step(eesd_ctx* c, int32_t* tok_or_null) {
    if (!c) return EESD_EINVAL;
    if (c->state != ST_READY) return fail(c, EESD_ESTATE, "draft_step: state is not ready");
    const eesd_config& g = c->cfg;
    const int i = c->n_drafted;
    if (i >= g.k_cap) return fail(c, EESD_ERANGE, "draft_step: k_cap = %d drafts already made", g.k_cap);
    const int pos = c->kv_len + i;
    if (c->kv_len + 1 + (i + 1) * tree_width(c) > g.max_seq)
        return fail(c, EESD_ERANGE, "draft_step: position %d does not leave room for verification (max_seq %d)", pos, g.max_seq);
    int rc = ensure_pages(c, pos + 1);
    if (rc) return rc;
    const bool mfma = pick_mfma(c, 1);
    if ((rc = launch_embed_norm(c, c->blk_tok + i, 1, mfma))) return rc;
    for (int l = 0; l < g.n_draft_layers; ++l) {
        const void* next_gain = l + 1 < g.n_draft_layers ? c->layers[l + 1].attn_norm : c->w.ee_layer.attn_norm;
        if ((rc = run_layer(c, c->layers[l], l, 1, pos, mfma, next_gain))) return rc;
    }
    if (reuse_hn(c)) {   // this row's layer-N hidden state is what verify would recompute
        hipLaunchKernelGGL(copy_row_kernel, dim3((g.d_model + 255) / 256), dim3(256), 0, c->stream, c->x, c->hn_rows + (size_t)i * g.d_model, g.d_model);
        HIP_TRY(c, hipGetLastError());
    }
    if ((rc = run_layer(c, c->w.ee_layer, g.n_layers, 1, pos, mfma, c->w.ee_norm))) return rc;
    void* ql = logit_row(c, c->q_logits, i);
    if ((rc = run_head(c, c->w.ee_norm, c->w.ee_head, 0, 1, ql, mfma))) return rc;
    const int width = tree_width(c);
    if (width > 1) {
        // the `width` most likely tokens are this depth's candidates; the first is drafted on from
        TreeForced tf;
        for (int j = 0; j < TREE_MAX_WIDTH; ++j) tf.tok[j] = -1;
        if (c->forced_pos + width <= c->forced.size()) {
            for (int j = 0; j < width; ++j) tf.tok[j] = c->forced[c->forced_pos + j];
            c->forced_pos += width;
        }
        if (lb16(c)) hipLaunchKernelGGL(top_candidates_kernel<bf16_t>, dim3(1), dim3(SMP_THREADS), 0, c->stream, (const bf16_t*)ql, g.vocab, width, tf,
                                        c->tree_blk + 1 + i * width, c->blk_tok + i + 1);
        else hipLaunchKernelGGL(top_candidates_kernel<float>, dim3(1), dim3(SMP_THREADS), 0, c->stream, (const float*)ql, g.vocab, width, tf,
                                c->tree_blk + 1 + i * width, c->blk_tok + i + 1);
    } else {
        int forced = -1;
        if (c->forced_pos < c->forced.size()) forced = c->forced[c->forced_pos++];
        double u = uniform53(g.seed, STREAM_DRAFT, c->round, i, 0);
        HIP_TRY(c, launch_softmax_sample(c, ql, c->q_rows + (size_t)i * g.vocab, u, forced, c->blk_tok + i + 1));
    }
    HIP_TRY(c, hipGetLastError());
    c->n_drafted = i + 1;
    if (tok_or_null) {
        HIP_TRY(c, hipMemcpyAsync(c->h_result + 2, c->blk_tok + i + 1, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        *tok_or_null = c->h_result[2];
    }
    return EESD_OK;
}

extern "C" int eesd_verify(eesd_ctx* c) {
    if (!c) return EESD_EINVAL;
    if (c->state != ST_READY) return fail(c, EESD_ESTATE, "verify: state is not ready");
    const eesd_config& g = c->cfg;
    const int width = tree_width(c);
    const int M = 1 + c->n_drafted * width;
    if (c->kv_len + M > g.max_seq) return fail(c, EESD_ERANGE, "verify: %d rows at %d exceed max_seq %d", M, c->kv_len, g.max_seq);
    int rc = ensure_pages(c, c->kv_len + M);
    if (rc) return rc;
    const bool mfma = pick_mfma(c, M);
    const int32_t* rows_tok = c->blk_tok;
    if (width > 1) {
        // rows: the pending token, then `width` children per depth; a node sees the pending token,
        // the first children of the depths above it, and itself
        HIP_TRY(c, hipMemcpyAsync(c->tree_blk, c->blk_tok, sizeof(int32_t), hipMemcpyDeviceToDevice, c->stream));
        memset(c->tree_mask, 0, sizeof c->tree_mask);
        memset(c->tree_depth, 0, sizeof c->tree_depth);
        c->tree_mask[0] = 1;
        unsigned chain = 1;   // row 0 and the first children so far
        for (int i = 0; i < c->n_drafted; ++i) {
            for (int j = 0; j < width; ++j) {
                const int r = 1 + i * width + j;
                c->tree_mask[r] = (unsigned short)(chain | (1u << r));
                c->tree_depth[r] = (unsigned char)(i + 1);
            }
            chain |= 1u << (1 + i * width);
        }
        c->tree_active = true;
        rows_tok = c->tree_blk;
    }
    if (reuse_hn(c) && c->n_drafted >= 1) rc = run_target_rows_reusing(c, c->n_drafted, c->kv_len);
    else rc = run_target_rows(c, rows_tok, M, c->kv_len, mfma);
    c->tree_active = false;
    if (rc) return rc;
    if ((rc = run_head(c, c->w.final_norm, c->w.lm_head, 0, M, c->logits, mfma))) return rc;
    c->state = ST_VERIFIED;
    return EESD_OK;
}

// Tree mode (greedy): the walk over the candidates, then the accepted nodes' keys and values are
// moved to the positions they now hold - both queued before the one synchronisation.
static int accept_tree(eesd_ctx* c, int32_t* n_accepted, int32_t* next_token) {
    const eesd_config& g = c->cfg;
    const int K = c->n_drafted, width = tree_width(c), M = 1 + K * width;
    if (lb16(c)) hipLaunchKernelGGL(accept_tree_kernel<bf16_t>, dim3(1), dim3(SMP_THREADS), 0, c->stream, (const bf16_t*)c->logits, c->tree_blk, K, width, g.vocab,
                                    c->result_dev, c->blk_tok);
    else hipLaunchKernelGGL(accept_tree_kernel<float>, dim3(1), dim3(SMP_THREADS), 0, c->stream, (const float*)c->logits, c->tree_blk, K, width, g.vocab,
                            c->result_dev, c->blk_tok);
    HIP_TRY(c, hipGetLastError());
    const int per = c->n_caches * g.n_kv_heads * g.head_dim;
    KVView v = kv_view(c, 0);
    if (is_bf16(c)) hipLaunchKernelGGL((kv_compact_kernel<bf16_t>), dim3((per + 255) / 256), dim3(256), 0, c->stream, v, c->n_caches, c->kv_len, c->result_dev);
    else hipLaunchKernelGGL((kv_compact_kernel<float>), dim3((per + 255) / 256), dim3(256), 0, c->stream, v, c->n_caches, c->kv_len, c->result_dev);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipMemcpyAsync(c->h_result, c->result_dev, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    if (K) HIP_TRY(c, hipMemcpyAsync(c->h_result + H_ROWS_AT, c->result_dev + 2, K * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->h_result + H_TOKS_AT, c->tree_blk, M * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->last_a = c->h_result[0];
    c->last_y = c->h_result[1];
    c->last_tokens.clear();
    for (int i = 0; i < c->last_a; ++i) c->last_tokens.push_back(c->h_result[H_TOKS_AT + c->h_result[H_ROWS_AT + i]]);
    c->state = ST_ACCEPTED;
    *n_accepted = c->last_a;
    *next_token = c->last_y;
    return EESD_OK;
}

extern "C" int eesd_accept(eesd_ctx* c, const double* uniforms_or_null, int32_t* n_accepted, int32_t* next_token) {
    if (!c) return EESD_EINVAL;
    if (!n_accepted || !next_token) return fail(c, EESD_EINVAL, "accept: null out pointer");
    if (c->state != ST_VERIFIED) return fail(c, EESD_ESTATE, "accept: nothing verified");
    const eesd_config& g = c->cfg;
    const int K = c->n_drafted;
    if (tree_width(c) > 1) return accept_tree(c, n_accepted, next_token);
    AcceptU uu;
    memset(&uu, 0, sizeof uu);
    for (int i = 0; i < K; ++i) uu.u[i] = uniforms_or_null ? uniforms_or_null[i] : uniform53(g.seed, STREAM_ACCEPT, c->round, i, 0);
    uu.u[K] = uniforms_or_null ? uniforms_or_null[K] : uniform53(g.seed, STREAM_RESAMPLE, c->round, 0, 0);
    for (int i = 0; i <= K; ++i)
        if (!(uu.u[i] >= 0.0 && uu.u[i] < 1.0)) return fail(c, EESD_EINVAL, "accept: uniform %d outside [0,1)", i);
    if (!greedy(c) && smp_spread(g.vocab)) {
        const SplScratch sc = spl_scratch(c->spl_buf);
        HIP_TRY(c, lb16(c) ? launch_spread_accept(c->stream, (const bf16_t*)c->logits, c->p_rows, c->q_rows, c->blk_tok + 1, K, g.vocab,
                                                  inv_temperature(c), uu, sc, c->result_dev, c->blk_tok)
                           : launch_spread_accept(c->stream, (const float*)c->logits, c->p_rows, c->q_rows, c->blk_tok + 1, K, g.vocab,
                                                  inv_temperature(c), uu, sc, c->result_dev, c->blk_tok));
    } else if (lb16(c)) {
        HIP_TRY(c, smp_allow(accept_kernel<bf16_t>, g.vocab));
        hipLaunchKernelGGL(accept_kernel<bf16_t>, dim3(1), dim3(SMP_THREADS), smp_lds_bytes(g.vocab), c->stream, (const bf16_t*)c->logits, c->p_rows, c->q_rows,
                           c->blk_tok + 1, K, g.vocab, inv_temperature(c), greedy(c), 1, uu, c->result_dev, c->blk_tok, smp_use_lds(g.vocab));
    } else {
        HIP_TRY(c, smp_allow(accept_kernel<float>, g.vocab));
        hipLaunchKernelGGL(accept_kernel<float>, dim3(1), dim3(SMP_THREADS), smp_lds_bytes(g.vocab), c->stream, (const float*)c->logits, c->p_rows, c->q_rows,
                           c->blk_tok + 1, K, g.vocab, inv_temperature(c), greedy(c), 1, uu, c->result_dev, c->blk_tok, smp_use_lds(g.vocab));
    }
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipMemcpyAsync(c->h_result, c->result_dev, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    if (K) HIP_TRY(c, hipMemcpyAsync(c->h_result + H_TOKS_AT, c->blk_tok + 1, K * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->last_a = c->h_result[0];
    c->last_y = c->h_result[1];
    c->last_tokens.assign(c->h_result + H_TOKS_AT, c->h_result + H_TOKS_AT + c->last_a);
    c->state = ST_ACCEPTED;
    *n_accepted = c->last_a;
    *next_token = c->last_y;
    return EESD_OK;
}

extern "C" int eesd_accepted_tokens(eesd_ctx* c, int32_t* toks, int32_t cap, int32_t* n) {
    if (!c) return EESD_EINVAL;
    if (!toks || !n) return fail(c, EESD_EINVAL, "accepted_tokens: null pointer");
    if (c->state != ST_ACCEPTED) return fail(c, EESD_ESTATE, "accepted_tokens: nothing accepted");
    if ((size_t)cap < c->last_tokens.size()) return fail(c, EESD_ERANGE, "accepted_tokens: room for %d of %d tokens", cap, (int)c->last_tokens.size());
    for (size_t i = 0; i < c->last_tokens.size(); ++i) toks[i] = c->last_tokens[i];
    *n = (int32_t)c->last_tokens.size();
    return EESD_OK;
}

// keeps n_accepted drafts of the round just judged (the caller has checked n_accepted)
static int commit_round(eesd_ctx* c, int n_accepted) {
    const int K = c->n_drafted;
    // the stream is idle here: eesd_accept synchronised it
    {   // the hidden state whose output is the next pending token: verify row of the last kept node
        int row = n_accepted;
        if (tree_width(c) > 1) row = n_accepted ? c->h_result[H_ROWS_AT + n_accepted - 1] : 0;
        int rc = save_target_hidden(c, row);
        if (rc) return rc;
        if (c->cali_set) cali_update(&c->cali_theta_hat, &c->cali_weight, &c->cali_n, n_accepted, K, c->cali.update);
    }
    c->kv_len += n_accepted + 1;
    release_pages(c, c->kv_len);
    // the pending token of the next round is already in blk_tok[0]: the accept kernel stored it
    ts_update(c, n_accepted, K);
    c->stats.rounds += 1;
    c->stats.drafted += K;
    c->stats.accepted += n_accepted;
    c->n_drafted = 0;
    c->round += 1;
    c->state = ST_READY;
    return EESD_OK;
}

extern "C" int eesd_rollback(eesd_ctx* c, int32_t n_accepted) {
    if (!c) return EESD_EINVAL;
    if (c->state != ST_ACCEPTED) return fail(c, EESD_ESTATE, "rollback: nothing accepted");
    // keeping more, or fewer, drafts than the accept rule kept would break the equality of the output
    // distribution with auto-regressive decoding (and the pending token belongs to position last_a)
    if (n_accepted != c->last_a)
        return fail(c, EESD_ERANGE, "rollback: n_accepted %d is not the %d drafts eesd_accept kept", n_accepted, c->last_a);
    return commit_round(c, n_accepted);
}

extern "C" int eesd_set_calibration(eesd_ctx* c, const eesd_calibration* cal) {
    if (!c) return EESD_EINVAL;
    if (!cal || !cal->w || !cal->wp) return fail(c, EESD_EINVAL, "set_calibration: null pointer");
    if (cal->n_mats < 1 || cal->n_mats > 10 || cal->update < 0 || cal->update > 1) return fail(c, EESD_EINVAL, "set_calibration: n_mats or update out of range");
    if (!(cal->sigma_m > 0.0) || !(cal->sigma_s > 0.0) || !(cal->theta_hat0 == cal->theta_hat0))
        return fail(c, EESD_EINVAL, "set_calibration: sigma_m and sigma_s must be positive");
    if (c->state != ST_CREATED && !(c->state == ST_READY && c->n_drafted == 0))
        return fail(c, EESD_ESTATE, "set_calibration: not between rounds");
    c->cali = *cal;
    c->cali_set = true;
    c->cali_theta_hat = cal->theta_hat0; c->cali_weight = 1.0; c->cali_n = 0;
    return EESD_OK;
}

extern "C" int eesd_cali_score(eesd_ctx* c, float* theta_m) {
    if (!c) return EESD_EINVAL;
    if (!theta_m) return fail(c, EESD_EINVAL, "cali_score: null pointer");
    if (!c->cali_set) return fail(c, EESD_ESTATE, "cali_score: no predictor installed");
    if (c->state != ST_READY || c->n_drafted < 1) return fail(c, EESD_ESTATE, "cali_score: no draft step made");
    const eesd_config& g = c->cfg;
    const int d = g.d_model, mat = std::min(c->n_drafted, (int)c->cali.n_mats) - 1;
    const bool mfma = pick_mfma(c, 1);
    const char* W = (const char*)c->cali.w + (size_t)mat * d * d * c->elem;
    GemmP p = mfma ? gemm_base(W, c->h_tb, d, 1, d, d) : gemm_base(W, c->h_t, d, 1, d, d);   // no norm: the hidden state as it is
    p.Y = c->cali_u; p.ldy = d;
    int rc = gemm_launch<EPI_PLAIN>(c, mfma, p);
    if (rc) return rc;
    // c->x row 0 still holds the hidden state the early-exit layer left for this draft step
    if (is_bf16(c)) hipLaunchKernelGGL((cali_score_kernel<bf16_t>), dim3(1), dim3(SMP_THREADS), 0, c->stream, (const bf16_t*)c->cali.wp, c->cali_u, c->x, d, c->theta_dev);
    else hipLaunchKernelGGL((cali_score_kernel<float>), dim3(1), dim3(SMP_THREADS), 0, c->stream, (const float*)c->cali.wp, c->cali_u, c->x, d, c->theta_dev);
    HIP_TRY(c, hipGetLastError());
    float* h_theta = (float*)(c->h_result + H_THETA_AT);
    HIP_TRY(c, hipMemcpyAsync(h_theta, c->theta_dev, sizeof(float), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    *theta_m = *h_theta;
    return EESD_OK;
}

extern "C" int eesd_set_draft_schedule(eesd_ctx* c, const int32_t* k_per_round, int32_t n_rounds) {
    if (!c) return EESD_EINVAL;
    if (n_rounds < 0 || (n_rounds > 0 && !k_per_round)) return fail(c, EESD_EINVAL, "schedule: null pointer");
    for (int i = 0; i < n_rounds; ++i)
        if (k_per_round[i] < 1 || k_per_round[i] > c->cfg.k_cap) return fail(c, EESD_ERANGE, "schedule: K[%d] = %d outside [1,%d]", i, k_per_round[i], c->cfg.k_cap);
    c->schedule.assign(k_per_round, k_per_round + n_rounds);
    c->sched_round = 0;
    return EESD_OK;
}

extern "C" int eesd_next_draft_len(eesd_ctx* c, int32_t k_max, int32_t* k_out) {
    if (!c || !k_out) return EESD_EINVAL;
    *k_out = draw_k(c, std::min((int)k_max, (int)c->cfg.k_cap));
    return EESD_OK;
}

extern "C" int eesd_debug_force_pending(eesd_ctx* c, int32_t tok);

static double ms_between(hipEvent_t a, hipEvent_t b) {
    float ms = 0.f;
    hipEventElapsedTime(&ms, a, b);
    return (double)ms;
}

extern "C" int eesd_generate(eesd_ctx* c, const int32_t* prompt, int32_t n_prompt, int32_t max_new, int32_t* out, int32_t* n_out,
                             eesd_stats* stats_or_null) {
    if (!c) return EESD_EINVAL;
    if (!prompt || !out || !n_out || max_new < 1) return fail(c, EESD_EINVAL, "generate: null pointer or max_new < 1");
    const eesd_config& g = c->cfg;
    if (n_prompt + max_new + rows_cap(c) > g.max_seq)
        return fail(c, EESD_ERANGE, "generate: %d prompt + %d new + a verify block of %d rows exceeds max_seq %d", n_prompt, max_new, rows_cap(c), g.max_seq);
    if (g.ts_mode == EESD_TS_CALI && !c->cali_set) return fail(c, EESD_ESTATE, "generate: ts_mode is EESD_TS_CALI but no predictor is installed");
    auto t_begin = std::chrono::steady_clock::now();
    int32_t tok;
    int rc = eesd_prefill(c, prompt, n_prompt, &tok);
    if (rc) return rc;
    auto t_prefill = std::chrono::steady_clock::now();
    int n = 0;
    out[n++] = tok;
    double ms_d = 0, ms_v = 0, ms_a = 0;
    while (n < max_new) {
        const int k_max = std::min((int)g.k_cap, max_new - n);
        const bool cali = g.ts_mode == EESD_TS_CALI;
        const int K = cali ? k_max : draw_k(c, k_max);
        HIP_TRY(c, hipEventRecord(c->ev[0], c->stream));
        for (int i = 0; i < K; ++i) {
            if ((rc = eesd_draft_step(c, nullptr))) return rc;
            if (cali && i + 1 < k_max) {
                // Algorithm 3: the predictor scores this step, the calibrated posterior decides whether to go on
                float theta_m;
                if ((rc = eesd_cali_score(c, &theta_m))) return rc;
                if (!cali_decide(c->cali.sigma_m, c->cali.sigma_s, c->cali_theta_hat, c->cali_n, (double)theta_m, g.seed, c->round, i + 1, nullptr))
                    break;
            }
        }
        HIP_TRY(c, hipEventRecord(c->ev[1], c->stream));
        if ((rc = eesd_verify(c))) return rc;
        HIP_TRY(c, hipEventRecord(c->ev[2], c->stream));
        // the block's tokens come back together with the decision: one synchronisation per round
        int32_t a, y;
        if ((rc = eesd_accept(c, nullptr, &a, &y))) return rc;
        HIP_TRY(c, hipEventRecord(c->ev[3], c->stream));
        HIP_TRY(c, hipEventSynchronize(c->ev[3]));
        ms_d += ms_between(c->ev[0], c->ev[1]);
        ms_v += ms_between(c->ev[1], c->ev[2]);
        ms_a += ms_between(c->ev[2], c->ev[3]);
        for (int i = 0; i < a && n < max_new; ++i) out[n++] = c->last_tokens[i];
        if (n < max_new) out[n++] = y;
        if ((rc = eesd_rollback(c, a))) return rc;
    }
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    auto t_end = std::chrono::steady_clock::now();
    c->stats.generated = n;
    c->stats.ms_draft = ms_d;
    c->stats.ms_verify = ms_v;
    c->stats.ms_accept = ms_a;
    double decode_ms = std::chrono::duration<double, std::milli>(t_end - t_prefill).count();
    c->stats.ms_other = std::max(0.0, decode_ms - ms_d - ms_v - ms_a);
    (void)t_begin;
    finish_stats(c);
    *n_out = n;
    if (stats_or_null) *stats_or_null = c->stats;
    return EESD_OK;
}

// ---------------------------------------------------------------------------------------------
// test and benchmark hooks
// ---------------------------------------------------------------------------------------------
extern "C" int eesd_debug_force_drafts(eesd_ctx* c, const int32_t* toks, int32_t n) {
    if (!c) return EESD_EINVAL;
    if (n < 0 || (n > 0 && !toks)) return fail(c, EESD_EINVAL, "force_drafts: null pointer");
    for (int i = 0; i < n; ++i)
        if (toks[i] < 0 || toks[i] >= c->cfg.vocab) return fail(c, EESD_EINVAL, "force_drafts: token out of range");
    c->forced.assign(toks, toks + n);
    c->forced_pos = 0;
    return EESD_OK;
}

extern "C" int eesd_debug_rollback(eesd_ctx* c, int32_t n_accepted, int32_t pending_tok) {
    if (!c) return EESD_EINVAL;
    if (c->state != ST_ACCEPTED) return fail(c, EESD_ESTATE, "debug_rollback: nothing accepted");
    if (n_accepted < 0 || n_accepted > c->n_drafted) return fail(c, EESD_ERANGE, "debug_rollback: n_accepted %d outside [0,%d]", n_accepted, c->n_drafted);
    if (tree_width(c) > 1 && n_accepted > c->last_a)
        return fail(c, EESD_ERANGE, "debug_rollback: tree mode keeps at most the %d accepted nodes", c->last_a);
    if (pending_tok < 0 || pending_tok >= c->cfg.vocab) return fail(c, EESD_EINVAL, "debug_rollback: token out of range");
    int rc = commit_round(c, n_accepted);
    if (rc) return rc;
    return eesd_debug_force_pending(c, pending_tok);
}

extern "C" int eesd_debug_force_pending(eesd_ctx* c, int32_t tok) {
    if (!c) return EESD_EINVAL;
    if (c->state != ST_READY || c->n_drafted != 0) return fail(c, EESD_ESTATE, "force_pending: state is not ready");
    if (tok < 0 || tok >= c->cfg.vocab) return fail(c, EESD_EINVAL, "force_pending: token out of range");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->h_result[3] = tok;
    HIP_TRY(c, hipMemcpyAsync(c->blk_tok, c->h_result + 3, sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return EESD_OK;
}

template <typename KT>
__global__ void kv_gather_kernel(KVView kv, bool is_v, int n_tokens, float* __restrict__ out) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    int row = kv.n_kv_heads * kv.head_dim;
    if (idx >= n_tokens * row) return;
    int t = idx / row, r = idx - t * row, h = r / kv.head_dim, c = r - h * kv.head_dim;
    long long off = is_v ? kv_v_elem(kv, h, t, c) : kv_k_elem(kv, h, t, c);
    out[idx] = load_as_f32<KT>((const KT*)kv.pool + off);
}

template <typename KT>
__global__ void kv_pattern_kernel(KVView kv, int n_tokens, unsigned salt) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    int row = kv.n_kv_heads * kv.head_dim;
    if (idx >= n_tokens * row) return;
    int t = idx / row, r = idx - t * row, h = r / kv.head_dim, c = r - h * kv.head_dim;
    unsigned x = (unsigned)idx * 2654435761u + salt;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    float kval = ((float)(x & 0xffff) / 65536.0f - 0.5f) * 2.0f;
    float vval = ((float)(x >> 16) / 65536.0f - 0.5f) * 2.0f;
    store_from_f32<KT>((KT*)kv.pool + kv_k_elem(kv, h, t, c), kval);
    store_from_f32<KT>((KT*)kv.pool + kv_v_elem(kv, h, t, c), vval);
}

extern "C" int eesd_debug_fill_cache(eesd_ctx* c, int32_t n_tokens, int32_t pending_tok) {
    if (!c) return EESD_EINVAL;
    const eesd_config& g = c->cfg;
    if (n_tokens < 1 || n_tokens + rows_cap(c) > g.max_seq) return fail(c, EESD_ERANGE, "fill_cache: %d tokens do not fit", n_tokens);
    if (pending_tok < 0 || pending_tok >= g.vocab) return fail(c, EESD_EINVAL, "fill_cache: token out of range");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    reset_sequence(c);
    int rc = ensure_pages(c, n_tokens);
    if (rc) return rc;
    int total = n_tokens * g.n_kv_heads * g.head_dim;
    for (int cache = 0; cache < c->n_caches; ++cache) {
        KVView v = kv_view(c, cache);
        if (is_bf16(c)) hipLaunchKernelGGL((kv_pattern_kernel<bf16_t>), dim3((total + 255) / 256), dim3(256), 0, c->stream, v, n_tokens, 977u * cache + 1u);
        else hipLaunchKernelGGL((kv_pattern_kernel<float>), dim3((total + 255) / 256), dim3(256), 0, c->stream, v, n_tokens, 977u * cache + 1u);
        HIP_TRY(c, hipGetLastError());
    }
    c->h_result[3] = pending_tok;
    HIP_TRY(c, hipMemcpyAsync(c->blk_tok, c->h_result + 3, sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->kv_len = n_tokens;
    c->round = 1;
    c->state = ST_READY;
    return EESD_OK;
}

// one row of bf16 logits, widened to fp32 on the host
static int read_bf16_row(eesd_ctx* c, const void* dev_row, float* host_dst) {
    std::vector<uint16_t> tmp(c->cfg.vocab);
    HIP_TRY(c, hipMemcpy(tmp.data(), dev_row, tmp.size() * 2, hipMemcpyDeviceToHost));
    for (size_t j = 0; j < tmp.size(); ++j) {
        uint32_t u = (uint32_t)tmp[j] << 16;
        memcpy(host_dst + j, &u, 4);
    }
    return EESD_OK;
}

extern "C" int eesd_debug_read(eesd_ctx* c, int what, int index, int32_t n_tokens, void* host_dst, size_t bytes) {
    if (!c) return EESD_EINVAL;
    if (!host_dst) return fail(c, EESD_EINVAL, "debug_read: null destination");
    const eesd_config& g = c->cfg;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const size_t row = sizeof(float) * g.vocab;
    switch (what) {
        case EESD_READ_DRAFT_LOGITS:
        case EESD_READ_DRAFT_PROBS: {
            if (index < 0 || index >= g.k_cap || bytes < row) return fail(c, EESD_ERANGE, "debug_read: bad draft slot or size");
            if (what == EESD_READ_DRAFT_LOGITS && lb16(c)) return read_bf16_row(c, logit_row(c, c->q_logits, index), (float*)host_dst);
            const float* src = (what == EESD_READ_DRAFT_LOGITS ? c->q_logits : c->q_rows) + (size_t)index * g.vocab;
            HIP_TRY(c, hipMemcpy(host_dst, src, row, hipMemcpyDeviceToHost));
            return EESD_OK;
        }
        case EESD_READ_VERIFY_LOGITS: {
            if (index < 0 || index >= MAX_ROWS || bytes < row) return fail(c, EESD_ERANGE, "debug_read: bad verify row or size");
            if (lb16(c)) return read_bf16_row(c, logit_row(c, c->logits, index), (float*)host_dst);
            HIP_TRY(c, hipMemcpy(host_dst, c->logits + (size_t)index * g.vocab, row, hipMemcpyDeviceToHost));
            return EESD_OK;
        }
        case EESD_READ_VERIFY_PROBS: {
            if (index < 0 || index >= MAX_ROWS || bytes < row) return fail(c, EESD_ERANGE, "debug_read: bad verify row or size");
            HIP_TRY(c, hipMemcpy(host_dst, c->p_rows + (size_t)index * g.vocab, row, hipMemcpyDeviceToHost));
            return EESD_OK;
        }
        case EESD_READ_LAUNCH_COUNTS: {
            if (bytes < sizeof c->launch_counts) return fail(c, EESD_ERANGE, "debug_read: destination too small");
            memcpy(host_dst, c->launch_counts, sizeof c->launch_counts);
            return EESD_OK;
        }
        case EESD_READ_KV_K:
        case EESD_READ_KV_V: {
            if (index < 0 || index >= c->n_caches) return fail(c, EESD_ERANGE, "debug_read: bad cache index");
            if (n_tokens < 1 || n_tokens > c->mapped_pages * c->page_tokens) return fail(c, EESD_ERANGE, "debug_read: tokens not mapped");
            size_t total = (size_t)n_tokens * g.n_kv_heads * g.head_dim;
            if (bytes < total * sizeof(float)) return fail(c, EESD_ERANGE, "debug_read: destination too small");
            float* tmp = nullptr;
            if (hipMalloc((void**)&tmp, total * sizeof(float)) != hipSuccess) return fail(c, EESD_ENOMEM, "debug_read: scratch");
            KVView v = kv_view(c, index);
            bool is_v = what == EESD_READ_KV_V;
            if (is_bf16(c)) hipLaunchKernelGGL((kv_gather_kernel<bf16_t>), dim3((total + 255) / 256), dim3(256), 0, c->stream, v, is_v, n_tokens, tmp);
            else hipLaunchKernelGGL((kv_gather_kernel<float>), dim3((total + 255) / 256), dim3(256), 0, c->stream, v, is_v, n_tokens, tmp);
            hipError_t e = hipGetLastError();
            if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
            if (e == hipSuccess) e = hipMemcpy(host_dst, tmp, total * sizeof(float), hipMemcpyDeviceToHost);
            hipFree(tmp);
            if (e != hipSuccess) return fail(c, EESD_EDEVICE, "debug_read: %s", hipGetErrorString(e));
            return EESD_OK;
        }
        case EESD_READ_TOKENS: {
            size_t need = sizeof(int32_t) * (c->n_drafted + 1);
            if (bytes < need) return fail(c, EESD_ERANGE, "debug_read: destination too small");
            HIP_TRY(c, hipMemcpy(host_dst, c->blk_tok, need, hipMemcpyDeviceToHost));
            return EESD_OK;
        }
        case EESD_READ_TREE_TOKENS: {
            size_t need = sizeof(int32_t) * (1 + c->n_drafted * tree_width(c));
            if (tree_width(c) < 2 || bytes < need) return fail(c, EESD_ERANGE, "debug_read: not in tree mode or destination too small");
            HIP_TRY(c, hipMemcpy(host_dst, c->tree_blk, need, hipMemcpyDeviceToHost));
            return EESD_OK;
        }
        case EESD_READ_CALI_STATE: {
            if (bytes < 3 * sizeof(double)) return fail(c, EESD_ERANGE, "debug_read: destination too small");
            double* dst = (double*)host_dst;
            dst[0] = c->cali_theta_hat; dst[1] = c->cali_weight; dst[2] = (double)c->cali_n;
            return EESD_OK;
        }
        case EESD_READ_KV_LEN: {
            if (bytes < sizeof(int32_t)) return fail(c, EESD_ERANGE, "debug_read: destination too small");
            *(int32_t*)host_dst = c->kv_len;
            return EESD_OK;
        }
        case EESD_READ_PAGE_TABLE: {
            if (bytes < sizeof(int32_t) * c->n_pages) return fail(c, EESD_ERANGE, "debug_read: destination too small");
            memcpy(host_dst, c->h_table, sizeof(int32_t) * c->n_pages);
            return EESD_OK;
        }
    }
    return fail(c, EESD_EINVAL, "debug_read: unknown selector %d", what);
}

// plain streaming copy with a name of its own, so that a hardware-counter run can be scaled by a
// kernel whose HBM traffic is known exactly (n bytes read, n bytes written)
__global__ void eesd_calibration_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

extern "C" int eesd_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (!dst || !src || bytes % 16) return EESD_EINVAL;
    hipLaunchKernelGGL(eesd_calibration_copy_kernel, dim3(4096), dim3(256), 0, (hipStream_t)hip_stream, (const uint4*)src, (uint4*)dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? EESD_OK : EESD_EDEVICE;
}

extern "C" int eesd_debug_profile_begin(eesd_ctx* c, int32_t family, int32_t epilogue_kind, int32_t in_dim) {
    if (!c) return EESD_EINVAL;
    if (family < 0 || family > 1 || epilogue_kind < 0 || epilogue_kind > 3 || in_dim < 0) return fail(c, EESD_EINVAL, "profile_begin: bad selector");
    c->prof_family = family; c->prof_epi = epilogue_kind; c->prof_in = in_dim; c->prof_used = 0;
    return EESD_OK;
}

extern "C" int eesd_debug_profile_end(eesd_ctx* c, int32_t* n_launches, double* total_ms) {
    if (!c) return EESD_EINVAL;
    if (!n_launches || !total_ms) return fail(c, EESD_EINVAL, "profile_end: null pointer");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    double ms = 0.0;
    for (size_t i = 0; i < c->prof_used; ++i) ms += ms_between(c->prof_ev[2 * i], c->prof_ev[2 * i + 1]);
    *n_launches = (int32_t)c->prof_used;
    *total_ms = ms;
    c->prof_family = -1;
    c->prof_used = 0;
    return EESD_OK;
}

// ---------------------------------------------------------------------------------------------
// stand-alone kernels
// ---------------------------------------------------------------------------------------------
extern "C" int eesd_op_accept(const float* p_rows, const float* q_rows, const int32_t* drafts, const double* uniforms, int32_t K,
                              int32_t vocab, int32_t greedy_flag, void* hip_stream, int32_t* result) {
    if (!p_rows || !result || K < 0 || K > ACC_MAX_K || vocab < 2) return EESD_EINVAL;
    if (K > 0 && !drafts) return EESD_EINVAL;
    if (!greedy_flag && (!uniforms || (K > 0 && !q_rows))) return EESD_EINVAL;
    AcceptU uu;
    memset(&uu, 0, sizeof uu);
    if (!greedy_flag)
        for (int i = 0; i <= K; ++i) {
            if (!(uniforms[i] >= 0.0 && uniforms[i] < 1.0)) return EESD_EINVAL;
            uu.u[i] = uniforms[i];
        }
    hipStream_t st = (hipStream_t)hip_stream;
    int32_t* d_res = nullptr;
    if (hipMalloc((void**)&d_res, 2 * sizeof(int32_t)) != hipSuccess) return EESD_ENOMEM;
    hipLaunchKernelGGL(accept_kernel<float>, dim3(1), dim3(SMP_THREADS), 0, st, (const float*)nullptr, const_cast<float*>(p_rows), q_rows, drafts, K,
                       vocab, 1.0f, greedy_flag, 0, uu, d_res, (int32_t*)nullptr, 0);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipMemcpy(result, d_res, 2 * sizeof(int32_t), hipMemcpyDeviceToHost);
    hipFree(d_res);
    return e == hipSuccess ? EESD_OK : EESD_EDEVICE;
}

extern "C" int eesd_op_accept_logits(const void* p_logits, int32_t logits_bf16, float* p_rows, const float* q_rows, const int32_t* drafts,
                                     const double* uniforms, int32_t K, int32_t vocab, float temperature, void* hip_stream, int32_t* result) {
    if (!p_logits || !result || K < 0 || K > ACC_MAX_K || vocab < 2 || !(temperature >= 0.f) || logits_bf16 < 0 || logits_bf16 > 1) return EESD_EINVAL;
    if (K > 0 && !drafts) return EESD_EINVAL;
    const int greedy_flag = temperature == 0.f;
    if (!greedy_flag && (!uniforms || !p_rows || (K > 0 && !q_rows))) return EESD_EINVAL;
    AcceptU uu;
    memset(&uu, 0, sizeof uu);
    if (!greedy_flag)
        for (int i = 0; i <= K; ++i) {
            if (!(uniforms[i] >= 0.0 && uniforms[i] < 1.0)) return EESD_EINVAL;
            uu.u[i] = uniforms[i];
        }
    hipStream_t st = (hipStream_t)hip_stream;
    int32_t* d_res = nullptr;
    if (hipMalloc((void**)&d_res, 256 + SPL_SCRATCH_BYTES) != hipSuccess) return EESD_ENOMEM;      // the result, then the spread kernels' chunk statistics
    const float inv_t = greedy_flag ? 1.0f : 1.0f / temperature;
    hipError_t e;
    if (!greedy_flag && smp_spread(vocab)) {
        const SplScratch sc = spl_scratch((char*)d_res + 256);
        e = logits_bf16 ? launch_spread_accept(st, (const bf16_t*)p_logits, p_rows, q_rows, drafts, K, vocab, inv_t, uu, sc, d_res, (int32_t*)nullptr)
                        : launch_spread_accept(st, (const float*)p_logits, p_rows, q_rows, drafts, K, vocab, inv_t, uu, sc, d_res, (int32_t*)nullptr);
    } else if (logits_bf16) {
        e = smp_allow(accept_kernel<bf16_t>, vocab);
        if (e == hipSuccess)
            hipLaunchKernelGGL(accept_kernel<bf16_t>, dim3(1), dim3(SMP_THREADS), smp_lds_bytes(vocab), st, (const bf16_t*)p_logits, p_rows, q_rows, drafts, K, vocab,
                               inv_t, greedy_flag, 1, uu, d_res, (int32_t*)nullptr, smp_use_lds(vocab));
    } else {
        e = smp_allow(accept_kernel<float>, vocab);
        if (e == hipSuccess)
            hipLaunchKernelGGL(accept_kernel<float>, dim3(1), dim3(SMP_THREADS), smp_lds_bytes(vocab), st, (const float*)p_logits, p_rows, q_rows, drafts, K, vocab,
                               inv_t, greedy_flag, 1, uu, d_res, (int32_t*)nullptr, smp_use_lds(vocab));
    }
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipMemcpy(result, d_res, 2 * sizeof(int32_t), hipMemcpyDeviceToHost);
    hipFree(d_res);
    return e == hipSuccess ? EESD_OK : EESD_EDEVICE;
}

extern "C" int eesd_op_softmax_sample(const float* logits, float* probs, int32_t vocab, float temperature, double u, void* hip_stream,
                                      int32_t* token) {
    if (!logits || !token || vocab < 2 || !(temperature >= 0.f) || !(u >= 0.0 && u < 1.0)) return EESD_EINVAL;
    if (temperature > 0.f && !probs) return EESD_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    int32_t* d_tok = nullptr;
    if (hipMalloc((void**)&d_tok, 256 + SPL_SCRATCH_BYTES) != hipSuccess) return EESD_ENOMEM;      // the token, then the spread kernels' chunk statistics
    hipError_t e = smp_allow(softmax_sample_kernel<float>, vocab);
    if (e == hipSuccess && temperature > 0.f && smp_spread(vocab)) {
        const SplScratch sc = spl_scratch((char*)d_tok + 256);
        e = launch_spread_sample(st, logits, probs, vocab, 1.0f / temperature, u, -1, sc, d_tok);
    } else if (e == hipSuccess) {
        hipLaunchKernelGGL(softmax_sample_kernel<float>, dim3(1), dim3(SMP_THREADS), smp_lds_bytes(vocab), st, logits, probs, vocab,
                           temperature > 0.f ? 1.0f / temperature : 1.0f, temperature == 0.f, u, -1, d_tok, smp_use_lds(vocab));
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipMemcpy(token, d_tok, sizeof(int32_t), hipMemcpyDeviceToHost);
    hipFree(d_tok);
    return e == hipSuccess ? EESD_OK : EESD_EDEVICE;
}

extern "C" int eesd_pack_weight(const void* src, void* dst, int32_t out_rows, int32_t in_dim, int32_t kind, int32_t head_dim, void* hip_stream) {
    if (!src || !dst || src == dst || out_rows < 16 || in_dim < 32 || in_dim % 32) return EESD_EINVAL;
    int epi;
    if (kind == EESD_PACK_PLAIN) epi = EPI_PLAIN;
    else if (kind == EESD_PACK_GATE_UP) epi = EPI_SWIGLU;
    else if (kind == EESD_PACK_QKV) epi = EPI_QKV;
    else return EESD_EINVAL;
    if (!mfma_shape_ok(out_rows, in_dim, epi, head_dim)) return EESD_EINVAL;
    if (out_rows % 16) return EESD_EINVAL;
    const int n_cu = device_cu_count();
    if (n_cu < 1) return EESD_EDEVICE;
    const int n_groups = pack_n_groups(out_rows, n_cu);
    hipLaunchKernelGGL(pack_weight_kernel, dim3(n_groups), dim3(256), 0, (hipStream_t)hip_stream, (const bf16_t*)src,
                       (bf16_t*)dst, out_rows, in_dim, epi, head_dim, n_groups);
    return hipGetLastError() == hipSuccess ? EESD_OK : EESD_EDEVICE;
}

extern "C" int eesd_op_gemm(const void* W, const float* X, float* Y, int32_t M, int32_t out, int32_t in, int32_t dtype, int32_t path,
                            int32_t weight_layout, void* hip_stream) {
    if (!W || !X || !Y || M < 1 || out < 2 || in < 8) return EESD_EINVAL;
    if (weight_layout != EESD_WEIGHTS_ROW_MAJOR && weight_layout != EESD_WEIGHTS_TILED) return EESD_EINVAL;
    // blocks of more than 128 rows exist on tile-major weights only (gemm_pf_kernel)
    const bool wide = weight_layout == EESD_WEIGHTS_TILED && in % (32 * PF_QC) == 0 && g_pf_rows != 128;
    if (M > (wide ? PREFILL_ROWS_WIDE : PREFILL_ROWS)) return EESD_EINVAL;
    if (weight_layout == EESD_WEIGHTS_TILED && (dtype != EESD_DTYPE_BF16 || path == EESD_GEMM_VALU)) return EESD_EINVAL;
    if (dtype != EESD_DTYPE_F32 && dtype != EESD_DTYPE_BF16) return EESD_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool b16 = dtype == EESD_DTYPE_BF16;
    bool mfma = b16 && (path == EESD_GEMM_MFMA || weight_layout == EESD_WEIGHTS_TILED || (path == EESD_GEMM_AUTO && M >= g_mfma_min_m));
    if (path == EESD_GEMM_MFMA && !b16) return EESD_EINVAL;
    if (mfma) {
        if (!mfma_shape_ok(out, in, EPI_PLAIN, 0)) return EESD_EINVAL;
        const int n_groups = weight_layout == EESD_WEIGHTS_TILED ? pack_n_groups(out, device_cu_count()) : 0;
        const bool grouped = n_groups && n_groups != out / 16;
        if (M > MAX_ROWS && (grouped ? in % GT_KC_MIN != 0 : !tile_shape_ok(out, in))) return EESD_EINVAL;
        // bf16 staging rows of the activations: one buffer per process, grown on demand, kept
        static bf16_t* xb = nullptr;
        static size_t xb_elems = 0;
        static std::mutex mu;      // guards the growth; calls that overlap on the GPU still share the rows (see the header)
        std::lock_guard<std::mutex> lock(mu);
        const size_t need = (size_t)2 * PREFILL_ROWS_WIDE * in;     // the rows, and the same in operand order for blocks of more than 16
        if (need > xb_elems) {
            if (hipDeviceSynchronize() != hipSuccess) return EESD_EDEVICE;
            if (xb) hipFree(xb);
            xb = nullptr; xb_elems = 0;
            if (hipMalloc((void**)&xb, need * sizeof(bf16_t)) != hipSuccess) return EESD_ENOMEM;
            if (hipMemset(xb, 0, need * sizeof(bf16_t)) != hipSuccess) return EESD_EDEVICE;
            xb_elems = need;
        }
        bf16_t* xp = xb + (size_t)PREFILL_ROWS_WIDE * in;
        hipLaunchKernelGGL(to_bf16_kernel, dim3((in + 255) / 256, M), dim3(256), 0, st, X, in, in, xb, in);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) {
            GemmP p = gemm_base(W, xb, in, M, out, in);
            p.Y = Y; p.ldy = out;
            p.w_packed = weight_layout == EESD_WEIGHTS_TILED;
            p.n_groups = n_groups;
            e = launch_mfma<EPI_PLAIN>(p, 1, st, nullptr, device_cu_count(), xp);
        }
        return e == hipSuccess ? EESD_OK : EESD_EDEVICE;
    }
    if (M > MAX_ROWS || in % (b16 ? 8 : 4) || out % 2 || valu_lds_bytes(M, in) > 150 * 1024) return EESD_EINVAL;
    GemmP p = gemm_base(W, X, in, M, out, in);
    p.Y = Y; p.ldy = out;
    hipError_t e = launch_valu<EPI_PLAIN>(p, b16, st);
    return e == hipSuccess ? EESD_OK : EESD_EDEVICE;
}

// ---------------------------------------------------------------------------------------------
// eesd_op_gemm without any allocation: the bf16 staging rows of the activations live in a fixed
// device array of this library instead of a buffer grown with hipMalloc.
// ---------------------------------------------------------------------------------------------
#define NOALLOC_MAX_ROWS MAX_ROWS
#define NOALLOC_MAX_IN 32768
static __device__ __align__(256) unsigned char scratch[(size_t)NOALLOC_MAX_ROWS * NOALLOC_MAX_IN * sizeof(bf16_t)];   // 1 MiB per GPU, held until the process ends
static void* g_scratch_ptr[64] = {nullptr};   // the array's address on each device

extern "C" int eesd_op_gemm_noalloc(const void* W, const float* X, float* Y, int32_t M, int32_t out, int32_t in, int32_t weight_layout,
                                    void* hip_stream) {
    if (!W || !X || !Y) return EESD_EINVAL;
    if (M < 1 || M > NOALLOC_MAX_ROWS || in < 128 || in > NOALLOC_MAX_IN) return EESD_ERANGE;   // beyond what the fixed staging array holds
    if (weight_layout != EESD_WEIGHTS_ROW_MAJOR && weight_layout != EESD_WEIGHTS_TILED) return EESD_EINVAL;
    if (!mfma_shape_ok(out, in, EPI_PLAIN, 0)) return EESD_EINVAL;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return EESD_EDEVICE;
    if (!g_scratch_ptr[dev]) {     // once per device, with that device current: every GPU holds its own copy of the array
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return EESD_EDEVICE;
        g_scratch_ptr[dev] = ptr;
    }
    bf16_t* xb = (bf16_t*)g_scratch_ptr[dev];
    const int n_cu = device_cu_count();
    if (n_cu < 1) return EESD_EDEVICE;
    hipStream_t st = (hipStream_t)hip_stream;
    // rows >= M of the staging array keep whatever the last call left: no kernel below stores a value computed from them
    hipLaunchKernelGGL(to_bf16_kernel, dim3((in + 255) / 256, M), dim3(256), 0, st, X, in, in, xb, in);
    if (hipGetLastError() != hipSuccess) return EESD_EDEVICE;
    GemmP p = gemm_base(W, xb, in, M, out, in);
    p.Y = Y; p.ldy = out;
    p.w_packed = weight_layout == EESD_WEIGHTS_TILED;
    p.n_groups = p.w_packed ? pack_n_groups(out, n_cu) : 0;
    return launch_mfma<EPI_PLAIN>(p, 1, st) == hipSuccess ? EESD_OK : EESD_EDEVICE;
}
