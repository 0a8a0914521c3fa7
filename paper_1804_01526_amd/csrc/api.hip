// Host side of the C ABI: geometry, argument validation, dispatch.
// Every check runs before anything is queued on the GPU, so the error paths
// behave the same on a machine without a GPU.
#include <string.h>

#include <atomic>

#include "hbfp_internal.h"

using namespace hbfp;

// ---- hbfp_encode_static: hbfp_encode for callers that cannot pass device scratch of their own.
// The table of block maxima of the two-pass conversions lives in this array.  Its name is a host-side stand-in: the
// address kernels can use comes from hipGetSymbolAddress, once per device (every device has its own copy).
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static int static_scratch(void **out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> address[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HBFP_ERR_LAUNCH;
    void *p = address[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HBFP_ERR_LAUNCH;
        address[dev].store(p, std::memory_order_release);       // a race stores the same address twice
    }
    *out = p;
    return HBFP_OK;
}


namespace {

int check_format(const hbfp_format *f) {
    if (!f) return HBFP_ERR_ARG;
    if (f->mant_bits < 2 || f->mant_bits > 16) return HBFP_ERR_FORMAT;
    if (f->rounding != HBFP_RNE && f->rounding != HBFP_STOCHASTIC) return HBFP_ERR_FORMAT;
    if (f->block_rows < 0 || f->block_cols < 0 || f->k_slot < 0) return HBFP_ERR_FORMAT;
    return HBFP_OK;
}

bool same_plan(const hbfp_tensor &a, const hbfp_tensor &b) {
    return a.rows == b.rows && a.kdim == b.kdim && a.kblock == b.kblock && a.kblock_pad == b.kblock_pad &&
           a.nblk == b.nblk && a.kpad == b.kpad && a.exp_ld == b.exp_ld && a.rblock == b.rblock && a.kshare == b.kshare &&
           a.src_rows == b.src_rows && a.src_cols == b.src_cols && a.contract_axis == b.contract_axis &&
           a.mant_bits == b.mant_bits && a.rounding == b.rounding && a.seed == b.seed &&
           a.mant_bytes == b.mant_bytes && a.exp_bytes == b.exp_bytes;
}

EncodeGeom geom_of(const hbfp_tensor &t, int64_t ld) {
    EncodeGeom g;
    g.src_rows = t.src_rows;
    g.src_cols = t.src_cols;
    g.ld = ld;
    g.axis = t.contract_axis;
    // exponent blocks in source coordinates: kshare stored blocks along k repeat one exponent
    const int64_t kext = t.kshare >= t.nblk ? t.kdim : t.kshare * t.kblock;
    if (t.contract_axis == 1) {
        g.br = t.rblock;
        g.bc = kext;
    } else {
        g.br = kext;
        g.bc = t.rblock;
    }
    g.kshare = t.kshare;
    g.nbr = ceil_div(g.src_rows, g.br);
    g.nbc = ceil_div(g.src_cols, g.bc);
    g.R = t.rows;
    g.K = t.kdim;
    g.kblock = t.kblock;
    g.kbp = t.kblock_pad;
    g.nblk = t.nblk;
    g.kpad = t.kpad;
    g.exp_ld = t.exp_ld;
    g.rblock = t.rblock;
    g.m = t.mant_bits;
    g.rounding = t.rounding;
    g.seed_lo = (uint32_t)t.seed;
    g.seed_hi = (uint32_t)(t.seed >> 32);
    return g;
}

// A descriptor is usable if it is exactly what hbfp_plan produces for its own key fields.
int check_tensor(const hbfp_tensor *t, bool need_ptrs) {
    if (!t) return HBFP_ERR_ARG;
    if (need_ptrs && (!t->mant || !t->exps)) return HBFP_ERR_ARG;
    if (t->src_rows <= 0 || t->src_cols <= 0 || (t->contract_axis != 0 && t->contract_axis != 1)) return HBFP_ERR_LAYOUT;
    hbfp_format f;
    f.mant_bits = t->mant_bits;
    f.rounding = t->rounding;
    f.seed = t->seed;
    if (t->kshare < 1) return HBFP_ERR_LAYOUT;
    f.k_slot = t->kshare > 1 ? t->kblock : 0;
    const int64_t kext = t->kshare == 1 ? t->kblock : (t->kshare >= t->nblk ? 0 : t->kshare * t->kblock);
    if (t->contract_axis == 1) {
        f.block_rows = t->rblock;
        f.block_cols = kext;
    } else {
        f.block_rows = kext;
        f.block_cols = t->rblock;
    }
    hbfp_tensor p;
    int rc = hbfp_plan(&f, t->src_rows, t->src_cols, t->contract_axis, &p);
    if (rc != HBFP_OK) return HBFP_ERR_LAYOUT;
    if (!same_plan(p, *t)) return HBFP_ERR_LAYOUT;
    if (need_ptrs && (((uintptr_t)t->mant & 15) || ((uintptr_t)t->exps & 3))) return HBFP_ERR_ARG;
    return HBFP_OK;
}

// Block shapes the single-pass kernels cover; everything else takes the max pass + quantise pass.
bool needs_tile_pass(const hbfp_tensor &t) {
    if (t.kshare > 1) return true;
    if (t.contract_axis == 1) return t.kblock > 128 || t.rblock > 32;
    return t.kblock > 64 || t.rblock > 64;
}

int check_pair(const hbfp_tensor *A, const hbfp_tensor *B) {
    int rc = check_tensor(A, true);
    if (rc != HBFP_OK) return rc;
    rc = check_tensor(B, true);
    if (rc != HBFP_OK) return rc;
    if (A->kdim != B->kdim || A->kblock != B->kblock) return HBFP_ERR_LAYOUT;
    const bool a8 = A->mant_bits <= 8, b8 = B->mant_bits <= 8;
    if (a8 != b8) return HBFP_ERR_FORMAT;
    if (A->mant_bits > 12 || B->mant_bits > 12) return HBFP_ERR_FORMAT;
    const int64_t qa = ((int64_t)1 << (A->mant_bits - 1)) - 1, qb = ((int64_t)1 << (B->mant_bits - 1)) - 1;
    // kblock * qa * qb must stay below 2^31 (int32 accumulators never overflow, Sec. 5.3)
    const int64_t lim = ((int64_t)1 << 31) - 1;
    if (A->kblock > lim / (qa * qb)) return HBFP_ERR_RANGE;
    return HBFP_OK;
}

GemmArgs gemm_args(const hbfp_tensor *A, const hbfp_tensor *B) {
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.mantA = A->mant;
    g.mantB = B->mant;
    g.expA = A->exps;
    g.expB = B->exps;
    g.M = A->rows;
    g.N = B->rows;
    g.kpad = A->kpad;
    g.expA_ld = A->exp_ld;
    g.expB_ld = B->exp_ld;
    g.nblk = A->nblk;
    g.kbp = A->kblock_pad;
    g.kblock = A->kblock;
    g.kdim = A->kdim;
    g.mA = A->mant_bits;
    g.mB = B->mant_bits;
    return g;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// the caller expects marked operands: prepare the 8-wave int8 kernel as the stand-by of the block-scaled product
bool fast_standby(const hbfp_tensor *A, const hbfp_tensor *B) { return ((A->hints | B->hints) & HBFP_HINT_HEAVY_TAILS) != 0; }

}  // namespace

extern "C" {

int hbfp_version(void) { return 100; }

const char *hbfp_status_string(int status) {
    switch (status) {
        case HBFP_OK: return "ok";
        case HBFP_ERR_ARG: return "bad argument";
        case HBFP_ERR_FORMAT: return "unsupported format";
        case HBFP_ERR_LAYOUT: return "operand layout mismatch";
        case HBFP_ERR_RANGE: return "int32 accumulator bound exceeded";
        case HBFP_ERR_LAUNCH: return "HIP runtime error";
        case HBFP_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
        default: return "unknown status";
    }
}

int hbfp_plan(const hbfp_format *fmt, int64_t rows, int64_t cols, int contract_axis, hbfp_tensor *out) {
    if (!fmt || !out || rows <= 0 || cols <= 0 || (contract_axis != 0 && contract_axis != 1)) return HBFP_ERR_ARG;
    int rc = check_format(fmt);
    if (rc != HBFP_OK) return rc;
    const int64_t br = (fmt->block_rows == 0 || fmt->block_rows > rows) ? rows : fmt->block_rows;
    const int64_t bc = (fmt->block_cols == 0 || fmt->block_cols > cols) ? cols : fmt->block_cols;
    memset(out, 0, sizeof *out);
    out->src_rows = rows;
    out->src_cols = cols;
    out->contract_axis = contract_axis;
    out->mant_bits = fmt->mant_bits;
    out->rounding = fmt->rounding;
    out->seed = fmt->rounding == HBFP_STOCHASTIC ? fmt->seed : 0;
    if (contract_axis == 1) {
        out->rows = rows;
        out->kdim = cols;
        out->kblock = bc;
        out->rblock = br;
    } else {
        out->rows = cols;
        out->kdim = rows;
        out->kblock = br;
        out->rblock = bc;
    }
    out->kshare = 1;
    if (fmt->k_slot > 0 && fmt->k_slot < out->kblock) {
        // stored blocks of k_slot elements repeat the exponent of the longer exponent block they lie in
        const int64_t kext = out->kblock;
        if (kext != out->kdim && kext % fmt->k_slot != 0) return HBFP_ERR_FORMAT;
        out->kblock = fmt->k_slot;
        out->kshare = kext == out->kdim ? ceil_div(out->kdim, out->kblock) : kext / out->kblock;
    }
    out->kblock_pad = out->kblock <= 32 ? 32 : out->kblock <= 64 ? 64 : round_up(out->kblock, 128);
    out->nblk = ceil_div(out->kdim, out->kblock);
    out->kpad = round_up(out->nblk * out->kblock_pad, 128);
    out->exp_ld = round_up(out->nblk, 4);
    out->mant_bytes = (uint64_t)out->rows * (uint64_t)out->kpad * (fmt->mant_bits <= 8 ? 1u : 2u);
    out->exp_bytes = (uint64_t)out->rows * (uint64_t)out->exp_ld;
    return HBFP_OK;
}

int hbfp_sizes(const hbfp_format *fmt, int64_t rows, int64_t cols, int contract_axis, size_t *mant_bytes, size_t *exp_bytes,
               int64_t *kpad) {
    hbfp_tensor t;
    const int rc = hbfp_plan(fmt, rows, cols, contract_axis, &t);
    if (rc != HBFP_OK) return rc;
    if (mant_bytes) *mant_bytes = (size_t)t.mant_bytes;
    if (exp_bytes) *exp_bytes = (size_t)t.exp_bytes;
    if (kpad) *kpad = t.kpad;
    return HBFP_OK;
}

int hbfp_encode_workspace(const hbfp_tensor *plan, size_t *bytes) {
    if (!plan || !bytes) return HBFP_ERR_ARG;
    int rc = check_tensor(plan, false);
    if (rc != HBFP_OK) return rc;
    if (!needs_tile_pass(*plan)) {
        *bytes = 0;
        return HBFP_OK;
    }
    const int64_t ntile = ceil_div(plan->rows, plan->rblock) * ceil_div(plan->nblk, plan->kshare);
    *bytes = align256((size_t)ntile * 4);
    return HBFP_OK;
}

// src [src_rows][ld] -> the buffers of t, in t's own layout and format
static int encode_planned(const float *src, int64_t ld, const hbfp_tensor *t, bool tile_pass, void *workspace, hipStream_t s) {
    if (t->rblock > 1 && tile_path_ok(&t, 1, nullptr, src, ld)) return launch_tile_encode(src, ld, 1.0f, nullptr, &t, 1, s);
    const EncodeGeom g = geom_of(*t, ld);
    if (tile_pass) return launch_encode_generic(src, g, t->mant, t->exps, (uint32_t *)workspace, s);
    if (t->contract_axis == 1) return launch_encode_row_fused(src, g, t->mant, t->exps, s);
    return launch_encode_col_fused(src, g, t->mant, t->exps, s);
}

int hbfp_encode(const float *src, int64_t rows, int64_t cols, int64_t ld, int contract_axis,
                const hbfp_format *fmt, hbfp_tensor *out, void *workspace, size_t ws_bytes, void *stream) {
    if (!src || !fmt || !out || rows <= 0 || cols <= 0 || ld < cols) return HBFP_ERR_ARG;
    hbfp_tensor p;
    int rc = hbfp_plan(fmt, rows, cols, contract_axis, &p);
    if (rc != HBFP_OK) return rc;
    if (!same_plan(p, *out)) return HBFP_ERR_LAYOUT;
    if (!out->mant || !out->exps) return HBFP_ERR_ARG;
    if (((uintptr_t)out->mant & 15) || ((uintptr_t)out->exps & 3) || ((uintptr_t)src & 3)) return HBFP_ERR_ARG;
    size_t need = 0;
    hbfp_encode_workspace(&p, &need);
    if (need) {
        if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
    }
    return encode_planned(src, ld, out, need != 0, workspace, (hipStream_t)stream);
}

size_t hbfp_encode_static_limit(void) { return kStaticScratchBytes; }

int hbfp_encode_static(const float *src, int64_t rows, int64_t cols, int64_t ld, int contract_axis, const hbfp_format *fmt,
                       hbfp_tensor *out, void *stream) {
    if (!src || !fmt || !out || rows <= 0 || cols <= 0 || ld < cols) return HBFP_ERR_ARG;
    hbfp_tensor p;
    int rc = hbfp_plan(fmt, rows, cols, contract_axis, &p);
    if (rc != HBFP_OK) return rc;
    if (!same_plan(p, *out)) return HBFP_ERR_LAYOUT;
    if (!out->mant || !out->exps) return HBFP_ERR_ARG;
    if (((uintptr_t)out->mant & 15) || ((uintptr_t)out->exps & 3) || ((uintptr_t)src & 3)) return HBFP_ERR_ARG;
    size_t need = 0;
    hbfp_encode_workspace(&p, &need);
    if (need > kStaticScratchBytes) return HBFP_ERR_WORKSPACE;     // more exponent blocks than the array holds
    void *table = nullptr;
    if (need) {
        rc = static_scratch(&table);
        if (rc != HBFP_OK) return rc;
    }
    // the first kernel of a two-pass conversion clears the entries it is going to use (a fill kernel, no memset node)
    return encode_planned(src, ld, out, need != 0, table, (hipStream_t)stream);
}

static int encode_multi_check(int n, const hbfp_tensor *const *outs, size_t *scratch) {
    if (n < 1 || n > 3 || !outs) return HBFP_ERR_ARG;
    *scratch = 0;
    for (int i = 0; i < n; ++i) {
        if (!outs[i]) return HBFP_ERR_ARG;
        int rc = check_tensor(outs[i], true);
        if (rc != HBFP_OK) return rc;
        if (outs[i]->src_rows != outs[0]->src_rows || outs[i]->src_cols != outs[0]->src_cols) return HBFP_ERR_LAYOUT;
        if (((uintptr_t)outs[i]->mant & 15) || ((uintptr_t)outs[i]->exps & 3)) return HBFP_ERR_ARG;
        size_t b = 0;
        hbfp_encode_workspace(outs[i], &b);
        *scratch = b > *scratch ? b : *scratch;
    }
    return HBFP_OK;
}

int hbfp_encode_multi_workspace(int n, const hbfp_tensor *const *outs, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    return encode_multi_check(n, outs, bytes);
}

int hbfp_encode_multi(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs,
                      void *workspace, size_t ws_bytes, void *stream) {
    size_t need = 0;
    int rc = encode_multi_check(n, outs, &need);
    if (rc != HBFP_OK) return rc;
    if (!src || ((uintptr_t)src & 3) || ld < outs[0]->src_cols) return HBFP_ERR_ARG;
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    if (n > 1 && tile_path_ok(outs, n, nullptr, src, ld)) return launch_tile_encode(src, ld, 1.0f, nullptr, outs, n, s);
    for (int i = 0; i < n; ++i) {
        rc = encode_planned(src, ld, outs[i], needs_tile_pass(*outs[i]), workspace, s);
        if (rc != HBFP_OK) return rc;
    }
    return HBFP_OK;
}

int hbfp_encode_packed_workspace(int n, const hbfp_tensor *const *outs, size_t *bytes) {
    return hbfp_encode_multi_workspace(n, outs, bytes);
}

static int pack_one(const hbfp_tensor *t, void *packed, hipStream_t s) {
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.mantA = t->mant;
    g.expA = t->exps;
    g.M = t->rows;
    g.kpad = t->kpad;
    g.expA_ld = t->exp_ld;
    g.kbp = t->kblock_pad;
    g.kblock = t->kblock;
    g.nblk = t->nblk;
    g.kdim = t->kdim;
    g.mA = g.mB = t->mant_bits;
    return bf_operand(t->mant_bits) ? launch_bf_pack(g, packed, nullptr, s)
           : t->mant_bits >= 10     ? launch_f16_planes_pack(g, packed, nullptr, s)
                                    : launch_mx_pack(g, packed, nullptr, s);
}

// argument checks of hbfp_encode_packed for one source; *need: bytes of its conversion's scratch
static int encode_packed_check(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed,
                               const size_t *packed_bytes, size_t *need) {
    int rc = encode_multi_check(n, outs, need);
    if (rc != HBFP_OK) return rc;
    if (!packed || !packed_bytes || !src || ((uintptr_t)src & 3) || ld < outs[0]->src_cols) return HBFP_ERR_ARG;
    for (int i = 0; i < n; ++i) {
        if (!packed[i]) continue;
        if ((uintptr_t)packed[i] & 255) return HBFP_ERR_ARG;
        if (outs[i]->mant_bits > 12) return HBFP_ERR_FORMAT;
        if (packed_bytes[i] < packed_operand_bytes(outs[i]->rows, outs[i]->kpad, outs[i]->mant_bits)) return HBFP_ERR_WORKSPACE;
        if (ceil_div(outs[i]->rows, 256) * 8 * ceil_div(outs[i]->kpad / 64, 4) > 0x7fffffff) return HBFP_ERR_ARG;
    }
    return HBFP_OK;
}

int hbfp_encode_packed(const float *src, int64_t ld, int n, const hbfp_tensor *const *outs, void *const *packed,
                       const size_t *packed_bytes, void *workspace, size_t ws_bytes, void *stream) {
    size_t need = 0;
    int rc = encode_packed_check(src, ld, n, outs, packed, packed_bytes, &need);
    if (rc != HBFP_OK) return rc;
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    if (encode_pack_ok(src, ld, n, outs, packed)) return launch_encode_pack(src, ld, n, outs, packed, s);
    rc = hbfp_encode_multi(src, ld, n, outs, workspace, ws_bytes, stream);
    for (int i = 0; i < n && rc == HBFP_OK; ++i)
        if (packed[i]) rc = pack_one(outs[i], packed[i], s);
    return rc;
}

int hbfp_encode_packed_batch_workspace(int njobs, const hbfp_encode_job *jobs, size_t *bytes) {
    if (!bytes || !jobs || njobs < 1 || njobs > HBFP_BATCH_MAX) return HBFP_ERR_ARG;
    *bytes = 0;
    for (int j = 0; j < njobs; ++j) {
        size_t b = 0;
        int rc = encode_multi_check(jobs[j].n, jobs[j].outs, &b);
        if (rc != HBFP_OK) return rc;
        *bytes = b > *bytes ? b : *bytes;       // the sources are converted one after the other when they need it
    }
    return HBFP_OK;
}

int hbfp_encode_packed_batch(int njobs, const hbfp_encode_job *jobs, void *workspace, size_t ws_bytes, void *stream) {
    if (!jobs || njobs < 1 || njobs > HBFP_BATCH_MAX) return HBFP_ERR_ARG;
    size_t need = 0;
    for (int j = 0; j < njobs; ++j) {
        size_t b = 0;
        if (jobs[j].reserved != 0) return HBFP_ERR_ARG;
        int rc = encode_packed_check(jobs[j].src, jobs[j].ld, jobs[j].n, jobs[j].outs, jobs[j].packed, jobs[j].packed_bytes, &b);
        if (rc != HBFP_OK) return rc;
        need = b > need ? b : need;
    }
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    // sources that the fused kernel takes, with equal rounding and limb counts, share launches; the others go one by one
    const float *src[HBFP_BATCH_MAX];
    int64_t ld[HBFP_BATCH_MAX];
    int n[HBFP_BATCH_MAX];
    const hbfp_tensor *const *outs[HBFP_BATCH_MAX];
    void *const *packed[HBFP_BATCH_MAX];
    bool done[HBFP_BATCH_MAX] = {};
    for (int j = 0; j < njobs; ++j) {
        if (done[j] || !encode_pack_ok(jobs[j].src, jobs[j].ld, jobs[j].n, jobs[j].outs, jobs[j].packed)) continue;
        int m = 0;
        for (int k = j; k < njobs; ++k) {
            if (done[k] || !encode_pack_ok(jobs[k].src, jobs[k].ld, jobs[k].n, jobs[k].outs, jobs[k].packed)) continue;
            src[m] = jobs[k].src, ld[m] = jobs[k].ld, n[m] = jobs[k].n, outs[m] = jobs[k].outs, packed[m] = jobs[k].packed;
            if (!encode_pack_batch_ok(m + 1, outs)) continue;
            done[k] = true;
            ++m;
        }
        int rc = launch_encode_pack_batch(m, src, ld, n, outs, packed, s);
        if (rc != HBFP_OK) return rc;
    }
    for (int j = 0; j < njobs; ++j) {
        if (done[j]) continue;
        int rc = hbfp_encode_packed(jobs[j].src, jobs[j].ld, jobs[j].n, jobs[j].outs, jobs[j].packed, jobs[j].packed_bytes, workspace,
                                    ws_bytes, stream);
        if (rc != HBFP_OK) return rc;
    }
    return HBFP_OK;
}

// a convolution with positive extents whose window fits the padded image at least once
static bool conv_geometry_ok(const hbfp_conv2d &c) {
    if (c.n <= 0 || c.h <= 0 || c.w <= 0 || c.c <= 0 || c.r <= 0 || c.s <= 0 || c.pad_h < 0 || c.pad_w < 0 || c.stride_h <= 0 ||
        c.stride_w <= 0 || c.c_block < 0)
        return false;
    return c.h + 2 * c.pad_h >= c.r && c.w + 2 * c.pad_w >= c.s;
}

// geometry and plan checks shared by hbfp_encode_im2col and its workspace query
static int im2col_check(const hbfp_conv2d *conv, const hbfp_tensor *out, bool need_ptrs, int64_t *ho, int64_t *wo, bool *per_image) {
    if (!conv) return HBFP_ERR_ARG;
    if (!conv_geometry_ok(*conv)) return HBFP_ERR_ARG;
    int rc = check_tensor(out, need_ptrs);
    if (rc != HBFP_OK) return rc;
    *ho = (conv->h + 2 * conv->pad_h - conv->r) / conv->stride_h + 1;
    *wo = (conv->w + 2 * conv->pad_w - conv->s) / conv->stride_w + 1;
    if (conv->h > 0x7fffffff || conv->w > 0x7fffffff || conv->c > 0x7fffffff || *ho * *wo > 0x7fffffff) return HBFP_ERR_ARG;
    if (out->src_rows != conv->n * *ho * *wo || out->src_cols != (int64_t)conv->r * conv->s * conv->c) return HBFP_ERR_LAYOUT;
    if (out->src_rows > 0x7fffffff || out->src_cols > 0x7fffffff) return HBFP_ERR_ARG;
    // one exponent per training input (Sec. 5.1): the rows of one image and the whole window share it
    *per_image = out->contract_axis == 1 && out->rblock == *ho * *wo && out->rblock > 1 && out->kshare >= out->nblk;
    if (!*per_image && (out->rblock != 1 || out->kshare != 1)) return HBFP_ERR_FORMAT;
    if (out->contract_axis == 1 ? (out->kblock > 128 || (out->kblock & 7) || (conv->c & 7) || (conv->c_block & 7)) : out->kblock > 64)
        return HBFP_ERR_FORMAT;
    if ((int64_t)conv->r * conv->s * (conv->c_block > 0 && conv->c_block < conv->c ? conv->c_block : conv->c) > 0x7fffffff) return HBFP_ERR_ARG;
    // the offset of a window entry from the corner pixel of the first window of its output row stays below 2^31 elements
    if ((((int64_t)conv->r + 1) * conv->w + conv->s) * conv->c > 0x7fffffff) return HBFP_ERR_ARG;
    return HBFP_OK;
}

int hbfp_encode_im2col_workspace(const hbfp_conv2d *conv, const hbfp_tensor *plan, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    int64_t ho = 0, wo = 0;
    bool per_image = false;
    const int rc = im2col_check(conv, plan, false, &ho, &wo, &per_image);
    if (rc != HBFP_OK) return rc;
    *bytes = per_image ? align256((size_t)conv->n * 4) : 0;
    return HBFP_OK;
}

int hbfp_encode_im2col(const float *x, const hbfp_conv2d *conv, const hbfp_tensor *out, void *workspace, size_t ws_bytes,
                       void *stream) {
    if (!x || ((uintptr_t)x & 15)) return HBFP_ERR_ARG;
    int64_t ho = 0, wo = 0;
    bool per_image = false;
    const int rc = im2col_check(conv, out, true, &ho, &wo, &per_image);
    if (rc != HBFP_OK) return rc;
    uint32_t *table = nullptr;
    if (per_image) {
        const size_t need = align256((size_t)conv->n * 4);
        if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
        table = (uint32_t *)workspace;
    }
    const EncodeGeom g = geom_of(*out, 0);
    return launch_encode_im2col(x, *conv, ho, wo, g, out->mant, out->exps, table, (hipStream_t)stream);
}

// arguments of a product whose operand A is gathered from `image` for M output rows
static GemmArgs conv_product_args(const hbfp_tensor *image, const hbfp_tensor *filters, int64_t M, float *C, int64_t ldc, float beta) {
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.mantA = image->mant;
    g.expA = image->exps;
    g.expA_ld = image->exp_ld;
    g.mantB = filters->mant;
    g.expB = filters->exps;
    g.expB_ld = filters->exp_ld;
    g.M = M;
    g.N = filters->rows;
    g.kpad = filters->kpad;
    g.nblk = filters->nblk;
    g.kbp = 32;
    g.kblock = image->kblock;
    g.mA = image->mant_bits;
    g.mB = filters->mant_bits;
    g.C = C;
    g.ldc = ldc;
    g.beta = beta;
    return g;
}

// geometry and operand checks shared by hbfp_gemm_conv2d and its workspace query.  *slot_order: -1 for the gather of 64
// channels of one tap per stage (blocks of 32, channels a multiple of 64, window entries tap by tap), else the order of k
// (0 tap by tap, 1 channel block by channel block) for the gather slot by slot.
static int conv_gemm_check(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, bool need_ptrs, int64_t *ho,
                           int64_t *wo, int *slot_order) {
    if (!image || !conv || !filters) return HBFP_ERR_ARG;
    if (!conv_geometry_ok(*conv)) return HBFP_ERR_ARG;
    int rc = check_tensor(image, need_ptrs);
    if (rc == HBFP_OK) rc = check_tensor(filters, need_ptrs);
    if (rc != HBFP_OK) return rc;
    *ho = (conv->h + 2 * conv->pad_h - conv->r) / conv->stride_h + 1;
    *wo = (conv->w + 2 * conv->pad_w - conv->s) / conv->stride_w + 1;
    const int64_t pixels = conv->n * conv->h * conv->w;
    if (conv->h > 0x7fffffff || conv->w > 0x7fffffff || conv->c > 0x7fffffff || pixels > 0x7fffffff || conv->n * *ho * *wo > 0x7fffffff)
        return HBFP_ERR_ARG;
    if (image->contract_axis != 1 || image->src_rows != pixels || image->src_cols != conv->c) return HBFP_ERR_LAYOUT;
    if (filters->contract_axis != 0 || filters->src_rows != (int64_t)conv->r * conv->s * conv->c) return HBFP_ERR_LAYOUT;
    if (image->mant_bits > 8 || filters->mant_bits > 8) return HBFP_ERR_FORMAT;
    // Both operands in stored blocks of 32 bytes that hold the same kblock <= 32 channels; how exponents are shared
    // beyond that (per pixel and block, per training input, filter tiles over the whole window) is the operands' business:
    // the product reads one exponent byte per row and stored block.
    const bool by_block = conv->c_block > 0 && conv->c_block < conv->c;
    if (image->kblock_pad != 32 || filters->kblock_pad != 32 || image->kblock != filters->kblock || conv->c % image->kblock ||
        (by_block && conv->c_block != image->kblock))
        return HBFP_ERR_FORMAT;
    *slot_order = by_block ? 1 : (image->kblock == 32 && !(conv->c & 63)) ? -1 : 0;
    return HBFP_OK;
}

// whether both operands of a convolution repeat their exponents over the r * s taps of a channel block (one exponent per
// training input against filter tiles over the whole window, window entries channel block by channel block): the
// product then scales each such run once (Sec. 4: the larger the tile, the fewer FP operations per fixed-point one)
static bool conv_runs(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, int slot_order) {
    const int64_t taps = (int64_t)conv->r * conv->s;
    return slot_order == 1 && taps > 1 && image->rblock == conv->h * conv->w && (filters->kshare >= filters->nblk || filters->kshare % taps == 0);
}

int hbfp_gemm_conv2d_workspace(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    int64_t ho = 0, wo = 0;
    int slot_order = -1;
    const int rc = conv_gemm_check(image, conv, filters, false, &ho, &wo, &slot_order);
    if (rc != HBFP_OK) return rc;
    *bytes = align256(gemm_conv_workspace(conv->n * ho * wo, filters->rows, filters->kpad, image->rows, (int)(conv->c / image->kblock)));
    return HBFP_OK;
}

int hbfp_gemm_conv2d(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, float *Y, int64_t ldy, float beta,
                     void *workspace, size_t ws_bytes, void *stream) {
    int64_t ho = 0, wo = 0;
    int slot_order = -1;
    int rc = conv_gemm_check(image, conv, filters, true, &ho, &wo, &slot_order);
    if (rc != HBFP_OK) return rc;
    if (!Y || ((uintptr_t)Y & 3) || ldy < filters->rows || (beta != 0.0f && beta != 1.0f)) return HBFP_ERR_ARG;
    size_t need = 0;
    hbfp_gemm_conv2d_workspace(image, conv, filters, &need);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
    const GemmArgs g = conv_product_args(image, filters, conv->n * ho * wo, Y, ldy, beta);
    return launch_gemm_conv_i8(g, *conv, ho, wo, image->kpad, workspace, (hipStream_t)stream, 1, 1, false, slot_order, (int)image->kblock,
                               conv_runs(image, conv, filters, slot_order) ? conv->r * conv->s : 0);
}

// hbfp_gemm_conv2d_bfp: [FP32 product, unless the kernel converts its accumulators][workspace of the convolution]
// [scratch of the conversion]
static int conv_bfp_plan(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, const hbfp_tensor *out, bool need_ptrs,
                         int64_t *ho, int64_t *wo, int *slot_order, bool *fused, size_t (&part)[3]) {
    int rc = conv_gemm_check(image, conv, filters, need_ptrs, ho, wo, slot_order);
    if (rc == HBFP_OK) rc = check_tensor(out, need_ptrs);
    if (rc != HBFP_OK) return rc;
    const int64_t M = conv->n * *ho * *wo, N = filters->rows;
    if (out->src_rows != M || out->src_cols != N) return HBFP_ERR_LAYOUT;
    *fused = conv_encoded_output_ok(M, N, filters->kpad, *out) && !conv_runs(image, conv, filters, *slot_order);
    part[0] = *fused ? 0 : align256((size_t)M * (size_t)N * 4);
    part[1] = align256(gemm_conv_workspace(M, N, filters->kpad, image->rows, (int)(conv->c / image->kblock)));
    size_t enc = 0;
    if (!*fused) hbfp_encode_workspace(out, &enc);
    part[2] = enc;
    return HBFP_OK;
}

int hbfp_gemm_conv2d_bfp_workspace(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, const hbfp_tensor *out,
                                   size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    int64_t ho = 0, wo = 0;
    int slot_order = -1;
    bool fused = false;
    size_t part[3];
    const int rc = conv_bfp_plan(image, conv, filters, out, false, &ho, &wo, &slot_order, &fused, part);
    if (rc != HBFP_OK) return rc;
    *bytes = part[0] + part[1] + part[2];
    return HBFP_OK;
}

int hbfp_gemm_conv2d_bfp(const hbfp_tensor *image, const hbfp_conv2d *conv, const hbfp_tensor *filters, const hbfp_tensor *out, int relu,
                         void *workspace, size_t ws_bytes, void *stream) {
    int64_t ho = 0, wo = 0;
    int slot_order = -1;
    bool fused = false;
    size_t part[3];
    int rc = conv_bfp_plan(image, conv, filters, out, true, &ho, &wo, &slot_order, &fused, part);
    if (rc != HBFP_OK) return rc;
    if (relu != 0 && relu != 1) return HBFP_ERR_ARG;
    if (!workspace || ws_bytes < part[0] + part[1] + part[2] || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t M = conv->n * ho * wo, N = filters->rows;
    float *C = (float *)workspace;
    char *ws_conv = (char *)workspace + part[0], *ws_enc = ws_conv + part[1];
    const GemmArgs g = conv_product_args(image, filters, M, fused ? nullptr : C, N, 0.0f);
    const int chain = conv_runs(image, conv, filters, slot_order) ? conv->r * conv->s : 0;
    rc = launch_gemm_conv_i8(g, *conv, ho, wo, image->kpad, ws_conv, s, 1, 1, false, slot_order, (int)image->kblock, chain,
                             fused ? out : nullptr, relu);
    if (rc != HBFP_OK || fused) return rc;
    if (relu) rc = launch_relu(C, M * N, s);
    if (rc != HBFP_OK) return rc;
    return encode_planned(C, N, out, part[2] != 0, ws_enc, s);
}

// The data gradient of a convolution of any stride: a stride-1 convolution of the zero-dilated output gradient with
// padding r - 1 - pad and the mirrored filter, computed for all h x w positions of the input.  The synthesized geometry
// describes that convolution: its image is dY as stored.
static int conv_dgrad_check(const hbfp_tensor *dy, const hbfp_conv2d *conv, const hbfp_tensor *filters, bool need_ptrs, hbfp_conv2d *as_forward,
                            int *slot_order) {
    if (!dy || !conv || !filters) return HBFP_ERR_ARG;
    if (!conv_geometry_ok(*conv)) return HBFP_ERR_ARG;
    int rc = check_tensor(dy, need_ptrs);
    if (rc == HBFP_OK) rc = check_tensor(filters, need_ptrs);
    if (rc != HBFP_OK) return rc;
    const int64_t ho = (conv->h + 2 * conv->pad_h - conv->r) / conv->stride_h + 1;
    const int64_t wo = (conv->w + 2 * conv->pad_w - conv->s) / conv->stride_w + 1;
    const int64_t f = dy->src_cols;
    if (conv->h > 0x7fffffff || conv->w > 0x7fffffff || conv->c > 0x7fffffff || f > 0x7fffffff || conv->n * conv->h * conv->w > 0x7fffffff ||
        conv->n * ho * wo > 0x7fffffff || conv->pad_h > 0xffff || conv->pad_w > 0xffff || conv->stride_h > 0xffff || conv->stride_w > 0xffff)
        return HBFP_ERR_ARG;
    if (dy->contract_axis != 1 || dy->src_rows != conv->n * ho * wo) return HBFP_ERR_LAYOUT;
    if (filters->contract_axis != 0 || filters->src_rows != (int64_t)conv->r * conv->s * f || filters->src_cols != conv->c) return HBFP_ERR_LAYOUT;
    if (dy->mant_bits > 8 || filters->mant_bits > 8) return HBFP_ERR_FORMAT;
    // as for hbfp_gemm_conv2d, with the filters of dy in the place of the channels (c_block counts filters here)
    const bool by_block = conv->c_block > 0 && conv->c_block < f;
    if (dy->kblock_pad != 32 || filters->kblock_pad != 32 || dy->kblock != filters->kblock || f % dy->kblock ||
        (by_block && conv->c_block != dy->kblock))
        return HBFP_ERR_FORMAT;
    *slot_order = by_block ? 1 : (dy->kblock == 32 && !(f & 63)) ? -1 : 0;
    *as_forward = *conv;
    as_forward->h = ho;
    as_forward->w = wo;
    as_forward->c = f;
    as_forward->pad_h = conv->r - 1 - conv->pad_h;
    as_forward->pad_w = conv->s - 1 - conv->pad_w;
    as_forward->stride_h = as_forward->stride_w = 1;
    return HBFP_OK;
}

int hbfp_gemm_conv2d_dgrad_workspace(const hbfp_tensor *dy, const hbfp_conv2d *conv, const hbfp_tensor *filters, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    hbfp_conv2d fw;
    int slot_order = -1;
    const int rc = conv_dgrad_check(dy, conv, filters, false, &fw, &slot_order);
    if (rc != HBFP_OK) return rc;
    *bytes = align256(gemm_conv_workspace(conv->n * conv->h * conv->w, filters->rows, filters->kpad, dy->rows, (int)(fw.c / dy->kblock)));
    return HBFP_OK;
}

int hbfp_gemm_conv2d_dgrad(const hbfp_tensor *dy, const hbfp_conv2d *conv, const hbfp_tensor *filters, float *dX, int64_t ldx, float beta,
                           void *workspace, size_t ws_bytes, void *stream) {
    hbfp_conv2d fw;
    int slot_order = -1;
    int rc = conv_dgrad_check(dy, conv, filters, true, &fw, &slot_order);
    if (rc != HBFP_OK) return rc;
    if (!dX || ((uintptr_t)dX & 3) || ldx < filters->rows || (beta != 0.0f && beta != 1.0f)) return HBFP_ERR_ARG;
    size_t need = 0;
    hbfp_gemm_conv2d_dgrad_workspace(dy, conv, filters, &need);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
    const GemmArgs g = conv_product_args(dy, filters, conv->n * conv->h * conv->w, dX, ldx, beta);
    // the slot-by-slot gather spreads dy out (zeros multiplied); the others go phase by phase where the window allows
    const bool by_phase = slot_order < 0 && conv_dgrad_by_phase(conv->r, conv->s, conv->stride_h, conv->stride_w);
    return launch_gemm_conv_i8(g, fw, conv->h, conv->w, dy->kpad, workspace, (hipStream_t)stream, conv->stride_h, conv->stride_w, by_phase,
                               slot_order, (int)dy->kblock);
}

int hbfp_decode(const hbfp_tensor *t, float *dst, int64_t ld, void *stream) {
    if (!dst) return HBFP_ERR_ARG;
    int rc = check_tensor(t, true);
    if (rc != HBFP_OK) return rc;
    if (ld < t->src_cols || ((uintptr_t)dst & 3)) return HBFP_ERR_ARG;
    return launch_decode(t, dst, ld, (hipStream_t)stream);
}

// hbfp_weight_update workspace: [FP32 weights after the step, src_rows x src_cols][scratch of the largest re-encode]
static int weight_update_plan(const hbfp_tensor *wide, const hbfp_tensor *na, const hbfp_tensor *nb, size_t *tmp_bytes,
                              size_t *total) {
    int rc = check_tensor(wide, true);
    if (rc != HBFP_OK) return rc;
    size_t scratch = 0;
    for (const hbfp_tensor *t : {wide, na, nb}) {
        if (!t) continue;
        rc = check_tensor(t, true);
        if (rc != HBFP_OK) return rc;
        if (t->src_rows != wide->src_rows || t->src_cols != wide->src_cols) return HBFP_ERR_LAYOUT;
        if (((uintptr_t)t->mant & 15) || ((uintptr_t)t->exps & 3)) return HBFP_ERR_ARG;
        size_t n = 0;
        hbfp_encode_workspace(t, &n);
        scratch = n > scratch ? n : scratch;
    }
    *tmp_bytes = align256((size_t)wide->src_rows * (size_t)wide->src_cols * 4);
    *total = *tmp_bytes + scratch;
    return HBFP_OK;
}

int hbfp_weight_update_workspace(const hbfp_tensor *wide, const hbfp_tensor *narrow_a, const hbfp_tensor *narrow_b,
                                 size_t *bytes) {
    if (!wide || !bytes) return HBFP_ERR_ARG;
    size_t tmp = 0;
    return weight_update_plan(wide, narrow_a, narrow_b, &tmp, bytes);
}

int hbfp_weight_update(const hbfp_tensor *wide, const float *delta, int64_t ld, float alpha,
                       const hbfp_tensor *narrow_a, const hbfp_tensor *narrow_b,
                       void *workspace, size_t ws_bytes, void *stream) {
    if (!wide || !delta || ((uintptr_t)delta & 3)) return HBFP_ERR_ARG;
    size_t tmp_bytes = 0, total = 0;
    int rc = weight_update_plan(wide, narrow_a, narrow_b, &tmp_bytes, &total);
    if (rc != HBFP_OK) return rc;
    if (ld < wide->src_cols) return HBFP_ERR_ARG;
    if (!workspace || ws_bytes < total || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    {   // all copies share a tile shape of at most 32 x 32: one kernel, the updated weights never leave the registers
        const hbfp_tensor *outs[3] = {wide, nullptr, nullptr};
        int n = 1;
        if (narrow_a) outs[n++] = narrow_a;
        if (narrow_b) outs[n++] = narrow_b;
        if (wide->rblock > 1 && tile_path_ok(outs, n, wide, delta, ld)) return launch_tile_encode(delta, ld, alpha, wide, outs, n, s);
    }
    float *w = (float *)workspace;
    void *scratch = (char *)workspace + tmp_bytes;
    const int64_t ldw = wide->src_cols;
    rc = launch_decode_axpy(wide, w, ldw, delta, ld, alpha, s);          // w = fma(alpha, delta, stored weight)
    if (rc != HBFP_OK) return rc;
    for (const hbfp_tensor *t : {wide, narrow_a, narrow_b}) {             // the wide copy first: it is the one read above
        if (!t) continue;
        rc = encode_planned(w, ldw, t, needs_tile_pass(*t), scratch, s);
        if (rc != HBFP_OK) return rc;
    }
    return HBFP_OK;
}

// 6..9-bit mantissas as bf16 numbers: asked for by name, or chosen where the 256 x 256 tiles pay (the shapes and block
// lengths for which the block-scaled kernel was measured ahead of the int8 kernels; the bf16 kernel is ahead of both there)
static bool use_bf(const GemmArgs &g, int kernel) {
    if (g.P || !gemm_bf_possible(g)) return false;
    return kernel == HBFP_KERNEL_BF16 || (kernel == HBFP_KERNEL_AUTO && gemm_mx_ok(g));
}

// 9..12-bit mantissas as FP16 numbers relative to their rows' largest exponents, on the same 256 x 256-tile kernel:
// asked for by name, or chosen for the shapes where those tiles pay when the bf16 kernel does not apply
static bool use_f16_planes(const GemmArgs &g, int kernel) {
    if (g.P || !gemm_f16_planes_possible(g)) return false;
    return kernel == HBFP_KERNEL_FP16_PLANES || (kernel == HBFP_KERNEL_AUTO && !use_bf(g, kernel) && gemm_mx_ok(g));
}

static bool use_scaled(const GemmArgs &g, int kernel) {
    if (g.P || kernel == HBFP_KERNEL_INT8 || kernel == HBFP_KERNEL_INT8_WIDE || kernel == HBFP_KERNEL_FP16 || kernel == HBFP_KERNEL_BF16 ||
        kernel == HBFP_KERNEL_FP16_PLANES)
        return false;
    if (use_bf(g, kernel) || use_f16_planes(g, kernel)) return false;
    return kernel == HBFP_KERNEL_SCALED ? gemm_mx_possible(g) : gemm_mx_ok(g);
}

int hbfp_gemm_select_workspace(const hbfp_tensor *A, const hbfp_tensor *B, int kernel, size_t *bytes) {
    if (!bytes || kernel < HBFP_KERNEL_AUTO || kernel > HBFP_KERNEL_FP16_PLANES) return HBFP_ERR_ARG;
    int rc = check_tensor(A, false);
    if (rc != HBFP_OK) return rc;
    rc = check_tensor(B, false);
    if (rc != HBFP_OK) return rc;
    *bytes = (A->mant_bits > 8 || B->mant_bits > 8) ? gemm_limb_workspace(A, B)
                                                     : gemm_i8_workspace(A->rows, B->rows, A->kpad, A->kblock_pad, A->exp_ld);
    const GemmArgs g = gemm_args(A, B);
    if (use_bf(g, kernel)) {                                     // [packed A][packed B]
        *bytes = packed_operand_bytes(g.M, g.kpad, g.mA) + packed_operand_bytes(g.N, g.kpad, g.mB);
        return HBFP_OK;
    }
    if (use_f16_planes(g, kernel)) {                             // [packed A][packed B]
        *bytes = f16_planes_bytes(g.M, g.kpad) + f16_planes_bytes(g.N, g.kpad);
        return HBFP_OK;
    }
    const size_t f16 = gemm_f16_workspace(A->rows, B->rows, A->kpad, A->kblock_pad, A->exp_ld > B->exp_ld ? A->exp_ld : B->exp_ld);
    if (kernel == HBFP_KERNEL_FP16 || (kernel == HBFP_KERNEL_AUTO && gemm_f16_possible(g))) {
        *bytes = f16;
        return HBFP_OK;
    }
    if (use_scaled(g, kernel))                                   // [packed A][packed B][int8 path behind the block-scaled kernel]
        *bytes = align256(*bytes) + mx_packed_bytes(g.M, g.kpad, g.mA) + mx_packed_bytes(g.N, g.kpad, g.mB);
    return HBFP_OK;
}

int hbfp_gemm_workspace(const hbfp_tensor *A, const hbfp_tensor *B, size_t *bytes) {
    return hbfp_gemm_select_workspace(A, B, HBFP_KERNEL_AUTO, bytes);
}

static int run_gemm(const hbfp_tensor *A, const hbfp_tensor *B, float *C, int64_t ldc, float beta, int32_t *P, int kernel,
                    void *workspace, size_t ws_bytes, void *stream) {
    int rc = check_pair(A, B);
    if (rc != HBFP_OK) return rc;
    GemmArgs g = gemm_args(A, B);
    g.C = C;
    g.ldc = ldc;
    g.beta = beta;
    g.P = P;
    if (kernel == HBFP_KERNEL_FP16 && !gemm_f16_possible(g)) return HBFP_ERR_FORMAT;
    if (kernel == HBFP_KERNEL_BF16 && !P && !gemm_bf_possible(g)) return HBFP_ERR_FORMAT;
    if (kernel == HBFP_KERNEL_FP16_PLANES && !P && !gemm_f16_planes_possible(g)) return HBFP_ERR_FORMAT;
    size_t need = 0;
    hbfp_gemm_select_workspace(A, B, kernel, &need);
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    if (kernel == HBFP_KERNEL_INT8_WIDE) {
        if (!gemm_wide_possible(g)) return HBFP_ERR_FORMAT;
        g.wide = 1;
    }
    if (use_bf(g, kernel)) {
        void *pa = workspace, *pb = (char *)workspace + packed_operand_bytes(g.M, g.kpad, g.mA);
        rc = launch_bf_pack(g, pa, pb, (hipStream_t)stream);
        const void *cpa = pa, *cpb = pb;
        return rc == HBFP_OK ? launch_bf_products(1, &g, &cpa, &cpb, (hipStream_t)stream) : rc;
    }
    if (use_f16_planes(g, kernel)) {
        void *pa = workspace, *pb = (char *)workspace + f16_planes_bytes(g.M, g.kpad);
        rc = launch_f16_planes_pack(g, pa, pb, (hipStream_t)stream);
        const void *cpa = pa, *cpb = pb;
        return rc == HBFP_OK ? launch_f16_planes_products(1, &g, &cpa, &cpb, (hipStream_t)stream) : rc;
    }
    // 9..12-bit mantissas are exact FP16 values: one FP16 matrix instruction per element pair instead of four or nine limb products
    if (kernel == HBFP_KERNEL_FP16 || (kernel == HBFP_KERNEL_AUTO && gemm_f16_possible(g)))
        return launch_gemm_f16(g, workspace, (hipStream_t)stream);
    if (use_scaled(g, kernel)) {
        // the block-scaled matrix instruction computes the product unless some exponent is out of its range;
        // the int8 kernels queue up behind it and run only in that case
        void *pa = workspace, *pb = (char *)workspace + mx_packed_bytes(g.M, g.kpad, g.mA);
        workspace = (char *)pb + mx_packed_bytes(g.N, g.kpad, g.mB);                  // what is left is the stand-by's
        rc = launch_mx_pack(g, pa, pb, (hipStream_t)stream);
        if (rc == HBFP_OK) rc = launch_mx_product(g, pa, pb, fast_standby(A, B) ? workspace : nullptr, (hipStream_t)stream);
        if (rc != HBFP_OK) return rc;
        g.run_a = (const int *)pa;
        g.run_b = (const int *)pb;
    }
    if (A->mant_bits > 8) return launch_gemm_limb(g, workspace, (hipStream_t)stream);
    return launch_gemm_i8(g, workspace, (hipStream_t)stream);
}

int hbfp_gemm_select(const hbfp_tensor *A, const hbfp_tensor *B, float *C, int64_t ldc, float beta, int kernel,
                     void *workspace, size_t ws_bytes, void *stream) {
    if (!A || !B || !C) return HBFP_ERR_ARG;
    if (beta != 0.0f && beta != 1.0f) return HBFP_ERR_ARG;
    if (kernel < HBFP_KERNEL_AUTO || kernel > HBFP_KERNEL_FP16_PLANES) return HBFP_ERR_ARG;
    if (ldc < B->rows || ((uintptr_t)C & 3)) return HBFP_ERR_ARG;
    return run_gemm(A, B, C, ldc, beta, nullptr, kernel, workspace, ws_bytes, stream);
}

int hbfp_gemm(const hbfp_tensor *A, const hbfp_tensor *B, float *C, int64_t ldc, float beta,
              void *workspace, size_t ws_bytes, void *stream) {
    return hbfp_gemm_select(A, B, C, ldc, beta, HBFP_KERNEL_AUTO, workspace, ws_bytes, stream);
}

// Checks the products of a batch and decides whether they share one launch of the bf16 or the block-scaled kernel; part[i] is
// product i's share of the workspace.
static int batch_plan(int n, const hbfp_tensor *const *A, const hbfp_tensor *const *B, int kernel, GemmArgs *g, size_t *part,
                      bool *grouped, int *group_kernel) {
    if (!A || !B || n < 1 || n > HBFP_BATCH_MAX) return HBFP_ERR_ARG;
    if (kernel < HBFP_KERNEL_AUTO || kernel > HBFP_KERNEL_FP16_PLANES) return HBFP_ERR_ARG;
    bool all_scaled = true, all_bf = true, bf_class = true, same = true;
    for (int i = 0; i < n; ++i) {
        if (!A[i] || !B[i]) return HBFP_ERR_ARG;
        const int rc = check_pair(A[i], B[i]);
        if (rc != HBFP_OK) return rc;
        g[i] = gemm_args(A[i], B[i]);
        all_scaled = all_scaled && use_scaled(g[i], kernel);
        all_bf = all_bf && use_bf(g[i], kernel);
        bf_class = bf_class && gemm_bf_possible(g[i]);
        same = same && (A[i]->mant_bits > 8) == (A[0]->mant_bits > 8) && mx_same_limbs(g[i], g[0]);
    }
    // products that would each take the bf16 or the block-scaled kernel anyway, or (automatic choice) that fill the chip
    // only together
    const bool together = kernel == HBFP_KERNEL_AUTO && gemm_mx_group_ok(n, g);
    *grouped = n > 1 && same && (all_scaled || all_bf || together);
    *group_kernel = !*grouped ? kernel : (all_bf || (together && bf_class)) ? HBFP_KERNEL_BF16 : HBFP_KERNEL_SCALED;
    for (int i = 0; i < n; ++i) {
        hbfp_gemm_select_workspace(A[i], B[i], *group_kernel, &part[i]);
        part[i] = align256(part[i]);
    }
    return HBFP_OK;
}

int hbfp_gemm_batch_workspace(int n, const hbfp_tensor *const *A, const hbfp_tensor *const *B, int kernel, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    GemmArgs g[HBFP_BATCH_MAX];
    size_t part[HBFP_BATCH_MAX];
    bool grouped = false;
    int group_kernel = kernel;
    const int rc = batch_plan(n, A, B, kernel, g, part, &grouped, &group_kernel);
    if (rc != HBFP_OK) return rc;
    *bytes = 0;
    for (int i = 0; i < n; ++i) *bytes += part[i];
    return HBFP_OK;
}

int hbfp_gemm_batch(int n, const hbfp_tensor *const *A, const hbfp_tensor *const *B, float *const *C, const int64_t *ldc,
                    float beta, int kernel, void *workspace, size_t ws_bytes, void *stream) {
    if (!C || !ldc) return HBFP_ERR_ARG;
    if (beta != 0.0f && beta != 1.0f) return HBFP_ERR_ARG;
    GemmArgs g[HBFP_BATCH_MAX];
    size_t part[HBFP_BATCH_MAX], need = 0;
    bool grouped = false;
    int group_kernel = kernel;
    int rc = batch_plan(n, A, B, kernel, g, part, &grouped, &group_kernel);
    if (rc != HBFP_OK) return rc;
    for (int i = 0; i < n; ++i) {
        if (!C[i] || ldc[i] < B[i]->rows || ((uintptr_t)C[i] & 3)) return HBFP_ERR_ARG;
        if (kernel == HBFP_KERNEL_INT8_WIDE && !gemm_wide_possible(g[i])) return HBFP_ERR_FORMAT;
        need += part[i];
        g[i].C = C[i];
        g[i].ldc = ldc[i];
        g[i].beta = beta;
    }
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    if (!grouped) {
        for (int i = 0; i < n; ++i) {
            rc = run_gemm(A[i], B[i], C[i], ldc[i], beta, nullptr, kernel, ws, part[i], stream);
            if (rc != HBFP_OK) return rc;
            ws += part[i];
        }
        return HBFP_OK;
    }
    const void *pa[HBFP_BATCH_MAX], *pb[HBFP_BATCH_MAX];
    if (group_kernel == HBFP_KERNEL_BF16) {
        for (int i = 0; i < n; ++i) {                                // product i: [packed A][packed B]
            char *a = ws, *b = a + packed_operand_bytes(g[i].M, g[i].kpad, g[i].mA);
            rc = launch_bf_pack(g[i], a, b, s);
            if (rc != HBFP_OK) return rc;
            pa[i] = a;
            pb[i] = b;
            ws += part[i];
        }
        return launch_bf_products(n, g, pa, pb, s);
    }
    void *standby[HBFP_BATCH_MAX];
    for (int i = 0; i < n; ++i) {                                    // product i: [packed A][packed B][int8 workspace]
        char *a = ws, *b = a + mx_packed_bytes(g[i].M, g[i].kpad, g[i].mA);
        standby[i] = b + mx_packed_bytes(g[i].N, g[i].kpad, g[i].mB);
        rc = launch_mx_pack(g[i], a, b, s);
        if (rc != HBFP_OK) return rc;
        pa[i] = a;
        pb[i] = b;
        ws += part[i];
    }
    void *fast[HBFP_BATCH_MAX];
    for (int i = 0; i < n; ++i) fast[i] = fast_standby(A[i], B[i]) ? standby[i] : nullptr;
    rc = launch_mx_products(n, g, pa, pb, fast, s);
    if (rc != HBFP_OK) return rc;
    for (int i = 0; i < n; ++i) {      // the int8 kernels stand by behind the group, one launch per product
        g[i].run_a = (const int *)pa[i];
        g[i].run_b = (const int *)pb[i];
        rc = A[i]->mant_bits > 8 ? launch_gemm_limb(g[i], standby[i], s) : launch_gemm_i8(g[i], standby[i], s);
        if (rc != HBFP_OK) return rc;
    }
    return HBFP_OK;
}

// Workspace of hbfp_gemm_bfp: [FP32 product M x N][workspace of the product][workspace of the conversion]
static int gemm_bfp_plan(const hbfp_tensor *A, const hbfp_tensor *B, const hbfp_tensor *out, int kernel, bool need_ptrs,
                         bool *fused, size_t part[3], int *kernel_used) {
    if (!A || !B || !out) return HBFP_ERR_ARG;
    if (kernel < HBFP_KERNEL_AUTO || kernel > HBFP_KERNEL_FP16_PLANES) return HBFP_ERR_ARG;
    int rc = need_ptrs ? check_pair(A, B) : check_tensor(A, false);
    if (rc == HBFP_OK && !need_ptrs) rc = check_tensor(B, false);
    if (rc == HBFP_OK) rc = check_tensor(out, need_ptrs);
    if (rc != HBFP_OK) return rc;
    if (out->src_rows != A->rows || out->src_cols != B->rows) return HBFP_ERR_LAYOUT;
    const GemmArgs g = gemm_args(A, B);
    *kernel_used = kernel;
    *fused = (use_scaled(g, kernel) || use_bf(g, kernel)) && mx_encoded_output_ok(*out);
    part[0] = align256((size_t)A->rows * (size_t)B->rows * sizeof(float));
    hbfp_gemm_select_workspace(A, B, kernel, &part[1]);
    part[1] = align256(part[1]);
    part[2] = 0;
    if (!*fused) hbfp_encode_workspace(out, &part[2]);
    part[2] = align256(part[2]);
    return HBFP_OK;
}

int hbfp_gemm_bfp_workspace(const hbfp_tensor *A, const hbfp_tensor *B, const hbfp_tensor *out, int kernel, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    bool fused = false;
    size_t part[3];
    const int rc = gemm_bfp_plan(A, B, out, kernel, false, &fused, part, &kernel);
    if (rc != HBFP_OK) return rc;
    *bytes = part[0] + part[1] + part[2];
    return HBFP_OK;
}

int hbfp_gemm_bfp(const hbfp_tensor *A, const hbfp_tensor *B, const hbfp_tensor *out, int relu, int kernel, void *workspace,
                  size_t ws_bytes, void *stream) {
    bool fused = false;
    size_t part[3];
    int rc = gemm_bfp_plan(A, B, out, kernel, true, &fused, part, &kernel);
    if (rc != HBFP_OK) return rc;
    if (relu != 0 && relu != 1) return HBFP_ERR_ARG;
    if (!workspace || ws_bytes < part[0] + part[1] + part[2] || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    float *C = (float *)workspace;
    char *ws_gemm = (char *)workspace + part[0], *ws_enc = ws_gemm + part[1];
    const int64_t M = A->rows, N = B->rows;
    if (!fused) {
        rc = run_gemm(A, B, C, N, 0.0f, nullptr, kernel, ws_gemm, part[1], stream);
        if (rc == HBFP_OK && relu) rc = launch_relu(C, M * N, s);
        if (rc != HBFP_OK) return rc;
        return encode_planned(C, N, out, part[2] != 0, ws_enc, s);
    }
    GemmArgs g = gemm_args(A, B);
    g.C = C;
    g.ldc = N;
    g.beta = 0.0f;
    if (use_bf(g, kernel)) {
        // the bf16 kernel converts its accumulators; for a marked operand it writes the FP32 product to the workspace
        // instead and the conversion behind it, which runs in that case only, produces the same output
        void *pa = ws_gemm, *pb = ws_gemm + packed_operand_bytes(g.M, g.kpad, g.mA);
        rc = launch_bf_pack(g, pa, pb, s);
        if (rc == HBFP_OK) rc = launch_bf_product_encoded(g, pa, pb, *out, relu, s);
        if (rc != HBFP_OK) return rc;
        return launch_mx_encode_standby(C, N, *out, relu, (const int *)pa, (const int *)pb, s);
    }
    // the block-scaled kernel converts its accumulators; should an exponent be outside its range, the int8 kernels behind
    // it write the FP32 product to the workspace and a conversion behind them produces the same output
    void *pa = ws_gemm, *pb = ws_gemm + mx_packed_bytes(g.M, g.kpad, g.mA);
    rc = launch_mx_pack(g, pa, pb, s);
    if (rc == HBFP_OK) rc = launch_mx_product_encoded(g, pa, pb, *out, relu, s);
    if (rc != HBFP_OK) return rc;
    g.run_a = (const int *)pa;
    g.run_b = (const int *)pb;
    void *standby = (char *)pb + mx_packed_bytes(g.N, g.kpad, g.mB);
    rc = A->mant_bits > 8 ? launch_gemm_limb(g, standby, s) : launch_gemm_i8(g, standby, s);
    if (rc != HBFP_OK) return rc;
    return launch_mx_encode_standby(C, N, *out, relu, g.run_a, g.run_b, s);
}

int hbfp_pack_bytes(const hbfp_tensor *t, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    const int rc = check_tensor(t, false);
    if (rc != HBFP_OK) return rc;
    if (t->mant_bits > 12) return HBFP_ERR_FORMAT;
    *bytes = packed_operand_bytes(t->rows, t->kpad, t->mant_bits);
    return HBFP_OK;
}

int hbfp_pack(const hbfp_tensor *t, void *packed, size_t bytes, void *stream) {
    int rc = check_tensor(t, true);
    if (rc != HBFP_OK) return rc;
    if (t->mant_bits > 12) return HBFP_ERR_FORMAT;
    if (!packed || ((uintptr_t)packed & 255)) return HBFP_ERR_ARG;
    if (bytes < packed_operand_bytes(t->rows, t->kpad, t->mant_bits)) return HBFP_ERR_WORKSPACE;
    if (ceil_div(t->rows, 256) * 8 * ceil_div(t->kpad / 64, 4) > 0x7fffffff) return HBFP_ERR_ARG;
    return pack_one(t, packed, (hipStream_t)stream);
}

// The packed form of an operand depends on its mantissa width alone (6..9 bits: bf16 planes, otherwise limb planes), so
// a product of packed operands runs on the bf16 kernel, on the block-scaled kernel, or, when the two forms meet, on the
// int8 kernels from the stored operands.
enum { kPackedMx = 0, kPackedBf = 1, kPackedMixed = 2, kPackedF16 = 3 };
static int packed_form(int mant_bits) { return bf_operand(mant_bits) ? 1 : mant_bits >= 10 ? 2 : 0; }
static int packed_kind(const hbfp_tensor *A, const hbfp_tensor *B) {
    const int a = packed_form(A->mant_bits), b = packed_form(B->mant_bits);
    return a != b ? kPackedMixed : a == 1 ? kPackedBf : a == 2 ? kPackedF16 : kPackedMx;
}

int hbfp_gemm_packed_workspace(const hbfp_tensor *A, const hbfp_tensor *B, size_t *bytes) {
    const int rc = hbfp_gemm_select_workspace(A, B, HBFP_KERNEL_INT8, bytes);
    if (rc == HBFP_OK && (packed_kind(A, B) == kPackedBf || packed_kind(A, B) == kPackedF16)) *bytes = 0;      // no stand-by kernels behind the bf16 / FP16 kernel
    return rc;
}

int hbfp_gemm_packed(const hbfp_tensor *A, const void *packed_a, const hbfp_tensor *B, const void *packed_b, float *C,
                     int64_t ldc, float beta, void *workspace, size_t ws_bytes, void *stream) {
    if (!A || !B || !C || !packed_a || !packed_b) return HBFP_ERR_ARG;
    if (beta != 0.0f && beta != 1.0f) return HBFP_ERR_ARG;
    if (((uintptr_t)packed_a & 255) || ((uintptr_t)packed_b & 255)) return HBFP_ERR_ARG;
    int rc = check_pair(A, B);
    if (rc != HBFP_OK) return rc;
    if (ldc < B->rows || ((uintptr_t)C & 3)) return HBFP_ERR_ARG;
    size_t need = 0;
    hbfp_gemm_packed_workspace(A, B, &need);
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    GemmArgs g = gemm_args(A, B);
    g.C = C;
    g.ldc = ldc;
    g.beta = beta;
    if (!gemm_mx_possible(g)) return HBFP_ERR_ARG;
    const int kind = packed_kind(A, B);
    if (kind == kPackedBf) rc = launch_bf_products(1, &g, &packed_a, &packed_b, (hipStream_t)stream);
    else if (kind == kPackedF16) rc = launch_f16_planes_products(1, &g, &packed_a, &packed_b, (hipStream_t)stream);
    else if (kind == kPackedMx) rc = launch_mx_product(g, packed_a, packed_b, fast_standby(A, B) ? workspace : nullptr, (hipStream_t)stream);
    if (rc != HBFP_OK || kind == kPackedBf || kind == kPackedF16) return rc;      // that kernel deals with marked operands itself
    if (kind != kPackedMixed) {      // the int8 kernels stand by; for a mixed pair they are the product
        g.run_a = (const int *)packed_a;
        g.run_b = (const int *)packed_b;
    }
    if (A->mant_bits > 8) return launch_gemm_limb(g, workspace, (hipStream_t)stream);
    return launch_gemm_i8(g, workspace, (hipStream_t)stream);
}

int hbfp_gemm_packed_batch_workspace(int n, const hbfp_tensor *const *A, const hbfp_tensor *const *B, size_t *bytes) {
    if (!bytes || !A || !B || n < 1 || n > HBFP_BATCH_MAX) return HBFP_ERR_ARG;
    *bytes = 0;
    for (int i = 0; i < n; ++i) {
        size_t part = 0;
        const int rc = hbfp_gemm_packed_workspace(A[i], B[i], &part);
        if (rc != HBFP_OK) return rc;
        *bytes += align256(part);
    }
    return HBFP_OK;
}

int hbfp_gemm_packed_batch(int n, const hbfp_tensor *const *A, const void *const *packed_a, const hbfp_tensor *const *B,
                           const void *const *packed_b, float *const *C, const int64_t *ldc, float beta, void *workspace,
                           size_t ws_bytes, void *stream) {
    if (!A || !B || !C || !ldc || !packed_a || !packed_b || n < 1 || n > HBFP_BATCH_MAX) return HBFP_ERR_ARG;
    if (beta != 0.0f && beta != 1.0f) return HBFP_ERR_ARG;
    GemmArgs g[HBFP_BATCH_MAX];
    size_t part[HBFP_BATCH_MAX], need = 0;
    for (int i = 0; i < n; ++i) {
        if (!A[i] || !B[i] || !C[i] || !packed_a[i] || !packed_b[i]) return HBFP_ERR_ARG;
        if (((uintptr_t)packed_a[i] & 255) || ((uintptr_t)packed_b[i] & 255) || ((uintptr_t)C[i] & 3)) return HBFP_ERR_ARG;
        int rc = check_pair(A[i], B[i]);
        if (rc != HBFP_OK) return rc;
        if (ldc[i] < B[i]->rows) return HBFP_ERR_ARG;
        rc = hbfp_gemm_packed_workspace(A[i], B[i], &part[i]);
        if (rc != HBFP_OK) return rc;
        part[i] = align256(part[i]);
        need += part[i];
        g[i] = gemm_args(A[i], B[i]);
        g[i].C = C[i];
        g[i].ldc = ldc[i];
        g[i].beta = beta;
        if (!gemm_mx_possible(g[i])) return HBFP_ERR_ARG;
        if ((A[i]->mant_bits > 8) != (A[0]->mant_bits > 8) || !mx_same_limbs(g[i], g[0])) return HBFP_ERR_FORMAT;
        if (packed_kind(A[i], B[i]) != packed_kind(A[0], B[0])) return HBFP_ERR_FORMAT;
    }
    const int kind = packed_kind(A[0], B[0]);
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    void *standby[HBFP_BATCH_MAX];
    {
        char *w = (char *)workspace;
        for (int i = 0; i < n; ++i) {
            standby[i] = part[i] && fast_standby(A[i], B[i]) ? w : nullptr;
            w += part[i];
        }
    }
    int rc = kind == kPackedBf    ? launch_bf_products(n, g, packed_a, packed_b, s)
             : kind == kPackedF16 ? launch_f16_planes_products(n, g, packed_a, packed_b, s)
             : kind == kPackedMx  ? launch_mx_products(n, g, packed_a, packed_b, standby, s)
                                  : HBFP_OK;
    if (rc != HBFP_OK || kind == kPackedBf || kind == kPackedF16) return rc;      // that kernel deals with marked operands itself
    char *ws = (char *)workspace;
    for (int i = 0; i < n; ++i) {      // the int8 kernels stand by behind the group, one launch per product
        if (kind != kPackedMixed) {
            g[i].run_a = (const int *)packed_a[i];
            g[i].run_b = (const int *)packed_b[i];
        }
        rc = A[i]->mant_bits > 8 ? launch_gemm_limb(g[i], ws, s) : launch_gemm_i8(g[i], ws, s);
        if (rc != HBFP_OK) return rc;
        ws += part[i];
    }
    return HBFP_OK;
}

int hbfp_gemm_partials(const hbfp_tensor *A, const hbfp_tensor *B, int32_t *P,
                       void *workspace, size_t ws_bytes, void *stream) {
    if (!A || !B || !P || ((uintptr_t)P & 3)) return HBFP_ERR_ARG;
    return run_gemm(A, B, nullptr, 0, 0.0f, P, HBFP_KERNEL_INT8, workspace, ws_bytes, stream);
}

int hbfp_gemm_partials_window(const hbfp_tensor *A, const hbfp_tensor *B, int64_t row0, int64_t rows, int64_t col0, int64_t cols,
                              int32_t *P, void *workspace, size_t ws_bytes, void *stream) {
    if (!A || !B || !P || ((uintptr_t)P & 3)) return HBFP_ERR_ARG;
    int rc = check_pair(A, B);
    if (rc != HBFP_OK) return rc;
    if (row0 < 0 || col0 < 0 || rows <= 0 || cols <= 0 || rows > A->rows || cols > B->rows || row0 > A->rows - rows || col0 > B->rows - cols)
        return HBFP_ERR_ARG;
    size_t need = 0;
    hbfp_gemm_select_workspace(A, B, HBFP_KERNEL_INT8, &need);      // that of the whole product covers any window
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return HBFP_ERR_WORKSPACE;
    // rows of an operand are kpad mantissas and exp_ld exponent bytes apart, so a window of the product is the
    // product of two operands that start further down and have fewer rows
    GemmArgs g = gemm_args(A, B);
    const int64_t es = A->mant_bits > 8 ? 2 : 1;
    g.mantA = (const char *)A->mant + row0 * A->kpad * es;
    g.mantB = (const char *)B->mant + col0 * B->kpad * es;
    g.expA = A->exps + row0 * A->exp_ld;
    g.expB = B->exps + col0 * B->exp_ld;
    g.M = rows;
    g.N = cols;
    g.P = P;
    if (A->mant_bits > 8) return launch_gemm_limb(g, workspace, (hipStream_t)stream);
    return launch_gemm_i8(g, workspace, (hipStream_t)stream);
}

// Layout of the hbfp_gemm_f32 workspace: [A mant][A exps][B mant][B exps][encode scratch][gemm scratch]
struct F32Plan {
    hbfp_tensor ta, tb;
    size_t off_am, off_ae, off_bm, off_be, off_enc, off_gemm, total;
};

static int plan_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                    const hbfp_format *fa, const hbfp_format *fb, F32Plan *p) {
    if (!fa || !fb || M <= 0 || N <= 0 || K <= 0) return HBFP_ERR_ARG;
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return HBFP_ERR_ARG;
    int rc = transA ? hbfp_plan(fa, K, M, 0, &p->ta) : hbfp_plan(fa, M, K, 1, &p->ta);
    if (rc != HBFP_OK) return rc;
    rc = transB ? hbfp_plan(fb, N, K, 1, &p->tb) : hbfp_plan(fb, K, N, 0, &p->tb);
    if (rc != HBFP_OK) return rc;
    if (p->ta.kblock != p->tb.kblock) return HBFP_ERR_LAYOUT;
    size_t ea = 0, eb = 0, gw = 0;
    hbfp_encode_workspace(&p->ta, &ea);
    hbfp_encode_workspace(&p->tb, &eb);
    rc = hbfp_gemm_workspace(&p->ta, &p->tb, &gw);
    if (rc != HBFP_OK) return rc;
    size_t o = 0;
    p->off_am = o; o += align256(p->ta.mant_bytes);
    p->off_ae = o; o += align256(p->ta.exp_bytes);
    p->off_bm = o; o += align256(p->tb.mant_bytes);
    p->off_be = o; o += align256(p->tb.exp_bytes);
    p->off_enc = o; o += align256(ea > eb ? ea : eb);
    p->off_gemm = o; o += align256(gw);
    p->total = o;
    return HBFP_OK;
}

int hbfp_gemm_f32_workspace(int transA, int transB, int64_t M, int64_t N, int64_t K,
                            const hbfp_format *fa, const hbfp_format *fb, size_t *bytes) {
    if (!bytes) return HBFP_ERR_ARG;
    F32Plan p;
    int rc = plan_f32(transA, transB, M, N, K, fa, fb, &p);
    if (rc != HBFP_OK) return rc;
    *bytes = p.total;
    return HBFP_OK;
}

int hbfp_gemm_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                  const float *A, int64_t lda, const float *B, int64_t ldb, float *C, int64_t ldc,
                  const hbfp_format *fa, const hbfp_format *fb,
                  void *workspace, size_t ws_bytes, void *stream) {
    if (!A || !B || !C) return HBFP_ERR_ARG;
    F32Plan p;
    int rc = plan_f32(transA, transB, M, N, K, fa, fb, &p);
    if (rc != HBFP_OK) return rc;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return HBFP_ERR_ARG;
    if (!workspace || ws_bytes < p.total || ((uintptr_t)workspace & 255)) return HBFP_ERR_WORKSPACE;
    char *w = (char *)workspace;
    p.ta.mant = w + p.off_am;
    p.ta.exps = (uint8_t *)(w + p.off_ae);
    p.tb.mant = w + p.off_bm;
    p.tb.exps = (uint8_t *)(w + p.off_be);
    rc = check_pair(&p.ta, &p.tb);  // mantissa classes and accumulator bound, before any launch
    if (rc != HBFP_OK) return rc;
    const size_t enc_bytes = p.off_gemm - p.off_enc, gemm_bytes = p.total - p.off_gemm;
    rc = transA ? hbfp_encode(A, K, M, lda, 0, fa, &p.ta, w + p.off_enc, enc_bytes, stream)
                : hbfp_encode(A, M, K, lda, 1, fa, &p.ta, w + p.off_enc, enc_bytes, stream);
    if (rc != HBFP_OK) return rc;
    rc = transB ? hbfp_encode(B, N, K, ldb, 1, fb, &p.tb, w + p.off_enc, enc_bytes, stream)
                : hbfp_encode(B, K, N, ldb, 0, fb, &p.tb, w + p.off_enc, enc_bytes, stream);
    if (rc != HBFP_OK) return rc;
    return hbfp_gemm(&p.ta, &p.tb, C, ldc, 0.0f, w + p.off_gemm, gemm_bytes, stream);
}

}  // extern "C"
