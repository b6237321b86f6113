// Row-tile inference kernel (cat_infer_kernel.h): variant selection on the host, launch.
#include "cat_infer_kernel.h"

#include "cat_infer.h"
#include "cat_tile_kernel.h"

namespace cat {

// centroid preparation shared with the tile kernels (cat_tile.hip)
cat_status launch_tile_prep_plain(cat_dtype dt, const float* cent, int64_t D, int32_t K, int32_t KT, int32_t P,
                                  int32_t nchunks, int rows_layout_f32, uint16_t* packA, float* cnorm, hipStream_t st);

namespace {

struct InferCfg {
    bool ok = false;
    int inst = -1;  // index into kInst
    int KT = 0, nsteps = 0;
    uint32_t xstride = 0, xpart = 0, off_s = 0, off_cnorm = 0, off_hist = 0, off_rep = 0, off_list = 0, off_misc = 0;
    size_t lds = 0;
};

struct Inst {
    bool bf16;
    int KW, SC, SPW, P, RGT, VPR;
    const void* fn[2][2];  // [mode: inference, assignment pass][tiles at a fixed stride, tiles handed out in order]
};

#define CAT_K(BF, KW, SC, SPW, P, RGT, VPR, DYN, MODE) (const void*)k_infer<BF, KW, SC, SPW, P, RGT, VPR, DYN, MODE>
#define CAT_INST(BF, KW, SC, SPW, P, RGT, VPR)                                                                         \
    {                                                                                                                  \
        BF, KW, SC, SPW, P, RGT, VPR, {                                                                                \
            {CAT_K(BF, KW, SC, SPW, P, RGT, VPR, false, INFER_APPLY), CAT_K(BF, KW, SC, SPW, P, RGT, VPR, true, INFER_APPLY)}, \
                {CAT_K(BF, KW, SC, SPW, P, RGT, VPR, false, INFER_ASSIGN), CAT_K(BF, KW, SC, SPW, P, RGT, VPR, true, INFER_ASSIGN)} \
        }                                                                                                              \
    }
// an instance whose inference variant would not fit the registers (the gamma / beta rows of bf16 data): assignment only
#define CAT_INST_ASSIGN(BF, KW, SC, SPW, P, RGT, VPR)                                                                  \
    {                                                                                                                  \
        BF, KW, SC, SPW, P, RGT, VPR, {                                                                                \
            {nullptr, nullptr},                                                                                        \
                {CAT_K(BF, KW, SC, SPW, P, RGT, VPR, false, INFER_ASSIGN), CAT_K(BF, KW, SC, SPW, P, RGT, VPR, true, INFER_ASSIGN)} \
        }                                                                                                              \
    }
// Instances.  The 8 waves of a workgroup are 8 / SC cluster shares (KW tiles of 16 clusters each) times SC channel
// shares (SPW steps of 32 channels each): an instance runs K <= 16 KW (8 / SC), D <= 32 SPW SC, rows of at most VPR
// KB.  For a shape several can run, the first in this list is taken (least padding work first).  A shape no instance
// holds takes the tile kernel.  Two centroid parts (hi + lo) wherever the wave's share fits 128 registers, else the
// hi part alone with the wider re-rank bound.
const Inst kInst[] = {
    // fp32 rows.  K <= 16
    CAT_INST(false, 1, 8, 1, 2, 1, 1), CAT_INST(false, 1, 8, 2, 2, 1, 2), CAT_INST(false, 1, 8, 4, 2, 1, 4),
    // K <= 32
    CAT_INST(false, 1, 4, 2, 2, 1, 1), CAT_INST(false, 1, 4, 4, 2, 1, 2), CAT_INST(false, 1, 4, 8, 2, 1, 4),
    // K <= 64
    CAT_INST(false, 1, 2, 4, 2, 1, 1), CAT_INST(false, 1, 2, 8, 2, 1, 2), CAT_INST(false, 1, 2, 16, 1, 1, 4),
    // K <= 128
    CAT_INST(false, 1, 1, 8, 2, 1, 1), CAT_INST(false, 1, 1, 16, 1, 1, 2),
    // bf16 rows (a vector holds 8 channels).  K <= 16, K <= 32, K <= 64, K <= 128
    CAT_INST(true, 1, 8, 2, 2, 1, 1), CAT_INST(true, 1, 8, 4, 2, 1, 2), CAT_INST_ASSIGN(true, 1, 8, 8, 2, 1, 4),
    CAT_INST(true, 1, 4, 4, 2, 1, 1), CAT_INST(true, 1, 4, 8, 2, 1, 2), CAT_INST_ASSIGN(true, 1, 4, 16, 2, 1, 4),
    CAT_INST(true, 1, 2, 8, 2, 1, 1), CAT_INST(true, 1, 2, 16, 2, 1, 2), CAT_INST_ASSIGN(true, 1, 2, 32, 1, 1, 4),
    CAT_INST(true, 1, 1, 16, 2, 1, 1), CAT_INST_ASSIGN(true, 1, 1, 32, 1, 1, 2),
};
constexpr int kNInst = sizeof(kInst) / sizeof(kInst[0]);

static inline uint32_t up16(size_t x) { return (uint32_t)((x + 15) & ~(size_t)15); }

InferCfg infer_config(int mode, bool lists, int64_t D, int32_t K, cat_dtype dt) {
    InferCfg c;
    const bool bf = dt == CAT_BF16;
    const int epl = bf ? 8 : 4, b = bf ? 2 : 4;
    if (D % epl || D > 8192 || K > 256) return c;
    const int nsteps = (int)((D + 31) / 32);
    const int vpr_need = (int)((D * b + 1023) / 1024);
    for (int i = 0; i < kNInst; i++) {
        const Inst& in = kInst[i];
        if (in.bf16 != bf || !in.fn[mode][0]) continue;
        const int KT = in.KW * (kInferWaves / in.SC);
        if (K > 16 * KT) continue;
        if (in.SPW * in.SC < nsteps || in.VPR < vpr_need) continue;
        const int rows = 16 * in.RGT;
        const int xp = (!bf && in.P == 2) ? 2 : 1;
        c.xstride = (uint32_t)(in.SPW * in.SC * 64 + 16);  // 32 channels of bf16 per step; + 16 bytes: rows 16 apart in banks
        c.xpart = (uint32_t)rows * c.xstride;
        c.off_s = up16((size_t)xp * c.xpart);
        c.off_cnorm = up16(c.off_s + (size_t)rows * in.SC * KT * 16 * 4);
        size_t off = c.off_cnorm + (size_t)KT * 16 * 4;
        if (mode == INFER_ASSIGN) {
            c.off_hist = up16(off);
            off = c.off_hist + (size_t)K * 4;
            c.off_rep = up16(off);
            off = c.off_rep + (size_t)K * 8;
            c.off_list = up16(off);
            off = c.off_list + (lists ? (size_t)1024 * 8 : 0);
            c.off_misc = up16(off);
            off = c.off_misc + 16 + 8 * kInferWaves;
        }
        c.lds = off;
        if (c.lds > 160 * 1024 - 256) continue;  // (the kernel has a few words of static LDS of its own)
        c.ok = true;
        c.inst = i;
        c.KT = KT;
        c.nsteps = nsteps;
        return c;
    }
    return c;
}

// error bound of the split arithmetic as a fraction of |x| |c| (see the tile kernel): 2^-16 per product with two
// parts per operand (one part: 2^-8), four such terms in a score difference, plus the fp32 accumulation of the
// MFMA partial sums of a wave and of the SC partial dot products
void rerank_bound(const Inst& in, const InferCfg& c, cat_dtype dt, float& tau, float& tau2) {
    const bool exact_x = dt == CAT_BF16;
    const int passes = in.P == 2 ? (exact_x ? 2 : 3) : 1;
    const float n_acc = (float)(passes * c.nsteps + in.SC + 8);
    const float split = in.P == 2 ? (exact_x ? 3.1e-5f : 9.4e-5f) : (exact_x ? 8.0e-3f : 1.6e-2f);
    tau = split + 4.f * n_acc * 5.96e-8f;
    tau2 = 4.0e-7f;
}

// persistent grid (as many workgroups as are resident at once), fixed stride or in-order hand-out, launch
cat_status launch_infer(InferParams& p, const Inst& in, const InferCfg& c, int mode, float* cnorm_ws, hipStream_t st) {
    static thread_local int cached_inst = -1, cached_mode = -1, cached_dev = -1, cached_lds = -1, per_cu = 1, ncu = 256;
    int dev = 0;
    CAT_HIP_TRY(hipGetDevice(&dev));
    if (cached_inst != c.inst || cached_mode != mode || cached_dev != dev || cached_lds != (int)c.lds) {
        int nb = 0, v = 0;
        CAT_HIP_TRY(hipFuncSetAttribute(in.fn[mode][0], hipFuncAttributeMaxDynamicSharedMemorySize, (int)c.lds));
        CAT_HIP_TRY(hipFuncSetAttribute(in.fn[mode][1], hipFuncAttributeMaxDynamicSharedMemorySize, (int)c.lds));
        CAT_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, in.fn[mode][0], kInferWaves * kWave, c.lds));
        CAT_HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
        per_cu = nb < 1 ? 1 : nb;
        ncu = v > 0 ? v : 256;
        cached_inst = c.inst;
        cached_mode = mode;
        cached_lds = (int)c.lds;
        cached_dev = dev;
    }
    const int64_t cap = (int64_t)ncu * per_cu;
    const unsigned blocks = (unsigned)(p.ntiles < cap ? p.ntiles : cap);
    // tiles in order pay from a few dozen tiles per workgroup on (the counters are cleared by a launch of their own)
    const bool dyn = p.ntiles >= 64 * (int64_t)blocks && p.ntiles < ((int64_t)1 << 31) - 8 * (int64_t)blocks;
    if (dyn) {
        p.counters = (unsigned int*)(cnorm_ws + 512);  // the norms take at most 256 of the 1024 floats
        cat_status fs = launch_fill_zero(p.counters, 8 * 16 * sizeof(unsigned int), st);
        if (fs != CAT_OK) return fs;
    }
    const bool prof = profile_on();
    if (prof) {
        cat_status ps = profile_mark(true, st);
        if (ps != CAT_OK) return ps;
    }
    void* args[] = {(void*)&p};
    CAT_HIP_TRY(hipLaunchKernel(in.fn[mode][dyn ? 1 : 0], dim3(blocks), dim3(kInferWaves * kWave), args, c.lds, st));
    CAT_LAUNCH_CHECK("k_infer");
    if (prof) return profile_mark(false, st);
    return CAT_OK;
}

}  // namespace

bool infer_supported(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    return N < ((int64_t)1 << 40) && infer_config(INFER_APPLY, false, D, K, dt).ok;
}

bool rowtile_assign_config(bool lists, int64_t N, int64_t D, int32_t K, cat_dtype dt, int* KT, int* P) {
    const InferCfg c = infer_config(INFER_ASSIGN, lists, D, K, dt);
    if (!c.ok || N >= ((int64_t)1 << 34)) return false;
    if (KT) *KT = c.KT;
    if (P) *P = kInst[c.inst].P;
    return true;
}

// One assignment pass with the bookkeeping of a Lloyd pass (the fields of the tile kernel's parameters).  packA and
// the norms must have been prepared with the cluster tiling and part count rowtile_assign_config reports, channels
// in plain order.
cat_status rowtile_assign(const TileParams& tp, cat_dtype dt, float* cnorm_ws, hipStream_t st) {
    const InferCfg c = infer_config(INFER_ASSIGN, tp.list != nullptr, tp.D, tp.K, dt);
    if (!c.ok) return set_error(CAT_ERR_UNSUPPORTED, "row-tile assignment kernel does not fit D=%lld K=%d", (long long)tp.D, (int)tp.K);
    const Inst& in = kInst[c.inst];
    InferParams p = {};
    p.lq = tp.lq;
    p.assign = tp.assign;
    p.N = tp.N;
    p.D = tp.D;
    const int rows = 16 * in.RGT;
    p.ntiles = (tp.N + rows - 1) / rows;
    p.K = tp.K;
    p.KT = c.KT;
    p.psteps = tp.nchunks * 4;
    p.packA = tp.packA;
    p.cnorm = tp.cnorm;
    p.cent = tp.cent;
    rerank_bound(in, c, dt, p.tau, p.tau2);
    p.xstride = c.xstride;
    p.xpart = c.xpart;
    p.off_s = c.off_s;
    p.off_cnorm = c.off_cnorm;
    p.counts = tp.counts;
    p.inertia = tp.inertia;
    p.rep = tp.rep;
    p.list = tp.list;
    p.list_count = tp.list_count;
    p.delta_mode = tp.delta_mode;
    p.list_cap = tp.list_cap;
    p.reverse = tp.reverse;
    p.skip_when_zero = tp.skip_when_zero;
    p.norm_part = tp.norm_part;
    p.norm_slices = tp.norm_slices;
    p.off_hist = c.off_hist;
    p.off_rep = c.off_rep;
    p.off_list = c.off_list;
    p.off_misc = c.off_misc;
    return launch_infer(p, in, c, INFER_ASSIGN, cnorm_ws, st);
}

cat_status infer_apply(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                       const float* gamma, const float* beta, void* corrected, int32_t* assign, const TileWs& ws,
                       hipStream_t st) {
    const InferCfg c = infer_config(INFER_APPLY, false, D, K, dt);
    if (!c.ok) return set_error(CAT_ERR_UNSUPPORTED, "row-tile inference kernel does not fit D=%lld K=%d", (long long)D, (int)K);
    const Inst& in = kInst[c.inst];
    // centroids: 16-byte aligned for the exact re-rank, else a copy in the workspace
    const float* cw = cent;
    if (((uintptr_t)cent & 15u) != 0) {
        cat_status s = launch_copy_words(cent, ws.cent, (int64_t)K * D, st);
        if (s != CAT_OK) return s;
        cw = ws.cent;
    }
    const int nchunks = (int)((D + 127) / 128);
    cat_status s = launch_tile_prep_plain(dt, cw, D, K, c.KT, in.P, nchunks, 0, ws.packA, ws.cnorm, st);
    if (s != CAT_OK) return s;
    InferParams p = {};
    p.lq = lq;
    p.out = corrected;
    p.assign = assign;
    p.N = N;
    p.D = D;
    const int rows = 16 * in.RGT;
    p.ntiles = (N + rows - 1) / rows;
    p.K = K;
    p.KT = c.KT;
    p.psteps = nchunks * 4;
    p.packA = ws.packA;
    p.cnorm = ws.cnorm;
    p.cent = cw;
    p.gamma = gamma;
    p.beta = beta;
    rerank_bound(in, c, dt, p.tau, p.tau2);
    p.xstride = c.xstride;
    p.xpart = c.xpart;
    p.off_s = c.off_s;
    p.off_cnorm = c.off_cnorm;
    return launch_infer(p, in, c, INFER_APPLY, ws.cnorm, st);
}

}  // namespace cat
