// Row-tile inference kernel (cat_infer_kernel.h): variant selection on the host, launch.
#include "cat_infer_kernel.h"

#include "cat_infer.h"

namespace cat {

// centroid preparation shared with the tile kernels (cat_tile.hip)
cat_status launch_tile_prep_plain(cat_dtype dt, const float* cent, int64_t D, int32_t K, int32_t KT, int32_t P,
                                  int32_t nchunks, int rows_layout_f32, uint16_t* packA, float* cnorm, hipStream_t st);

namespace {

struct InferCfg {
    bool ok = false;
    int inst = -1;  // index into kInst
    int KT = 0, nsteps = 0;
    bool ua = false;  // rows are not whole 16-byte groups
    uint32_t xstride = 0, xpart = 0, off_s = 0, off_cnorm = 0;
    size_t lds = 0;
};

struct Inst {
    bool bf16;
    int KW, SC, SPW, P, RGT, VPR;
    const void* fn;      // tiles at a fixed stride
    const void* fn_dyn;  // tiles handed out in order
    const void* fn_ua;   // the same two for rows that are not whole 16-byte groups
    const void* fn_ua_dyn;
};

#define CAT_INST(BF, KW, SC, SPW, P, RGT, VPR) \
    { BF, KW, SC, SPW, P, RGT, VPR, (const void*)k_infer<BF, KW, SC, SPW, P, RGT, VPR, false>, \
      (const void*)k_infer<BF, KW, SC, SPW, P, RGT, VPR, true>,                               \
      (const void*)k_infer<BF, KW, SC, SPW, P, RGT, VPR, false, true>,                        \
      (const void*)k_infer<BF, KW, SC, SPW, P, RGT, VPR, true, true> }
// (the word-by-word form of this instance does not fit the register file: rows that are not whole 16-byte groups take
// the streaming kernel there)
#define CAT_INST_ALIGNED_ONLY(BF, KW, SC, SPW, P, RGT, VPR) \
    { BF, KW, SC, SPW, P, RGT, VPR, (const void*)k_infer<BF, KW, SC, SPW, P, RGT, VPR, false>, \
      (const void*)k_infer<BF, KW, SC, SPW, P, RGT, VPR, true>, nullptr, nullptr }
// Instances.  The 8 waves of a workgroup are 8 / SC cluster shares (KW tiles of 16 clusters each) times SC channel
// shares (SPW steps of 32 channels each): an instance runs K <= 16 KW (8 / SC), D <= 32 SPW SC, rows of at most VPR
// KB.  For a shape several can run, the first in this list is taken (least padding work first).  A shape no instance
// holds takes the tile kernel.
const Inst kInst[] = {
    // K <= 16
    CAT_INST(false, 1, 8, 1, 2, 1, 1), CAT_INST(false, 1, 8, 2, 2, 1, 2), CAT_INST(false, 1, 8, 4, 2, 1, 4),
    // K <= 32
    CAT_INST(false, 1, 4, 2, 2, 1, 1), CAT_INST(false, 1, 4, 4, 2, 1, 2), CAT_INST(false, 1, 4, 8, 2, 1, 4),
    // K <= 64
    CAT_INST(false, 1, 2, 4, 2, 1, 1), CAT_INST(false, 1, 2, 8, 2, 1, 2), CAT_INST_ALIGNED_ONLY(false, 1, 2, 16, 1, 1, 4),
    // K <= 128 (from 16 steps on: hi part only, wider re-rank bound)
    CAT_INST(false, 1, 1, 8, 2, 1, 1), CAT_INST(false, 1, 1, 16, 1, 1, 2),
    // bf16 rows (a vector holds 8 channels; the gamma / beta rows take twice the registers of the row): K <= 16, 32, 64
    CAT_INST(true, 1, 8, 2, 2, 1, 1), CAT_INST(true, 1, 8, 4, 2, 1, 2),
    CAT_INST(true, 1, 4, 4, 2, 1, 1), CAT_INST(true, 1, 4, 8, 2, 1, 2),
    CAT_INST(true, 1, 2, 8, 2, 1, 1),
};
constexpr int kNInst = sizeof(kInst) / sizeof(kInst[0]);

static inline uint32_t up16(size_t x) { return (uint32_t)((x + 15) & ~(size_t)15); }

InferCfg infer_config(int64_t D, int32_t K, cat_dtype dt) {
    InferCfg c;
    const bool bf = dt == CAT_BF16;
    const int epl = bf ? 8 : 4, b = bf ? 2 : 4;
    // (rows that are not whole 16-byte groups run the word-by-word instances; bf16 rows are whole 4-byte words: D is even)
    if ((bf && D % 2) || D > 8192 || K > 256) return c;
    c.ua = D % epl != 0;
    const int nsteps = (int)((D + 31) / 32);
    const int vpr_need = (int)((D * b + 1023) / 1024);
    for (int i = 0; i < kNInst; i++) {
        const Inst& in = kInst[i];
        if (in.bf16 != bf) continue;
        const int KT = in.KW * (kInferWaves / in.SC);
        if (K > 16 * KT) continue;
        if (in.SPW * in.SC < nsteps || in.VPR < vpr_need) continue;
        if (c.ua && !in.fn_ua) continue;
        const int rows = 16 * in.RGT;
        const int xp = (!bf && in.P == 2) ? 2 : 1;
        c.xstride = (uint32_t)(in.SPW * in.SC * 64 + 16);  // 32 channels of bf16 per step; + 16 bytes: rows 16 apart in banks
        c.xpart = (uint32_t)rows * c.xstride;
        c.off_s = up16((size_t)xp * c.xpart);
        c.off_cnorm = up16(c.off_s + (size_t)rows * infer_dots_stride(in.SC * KT * 16) * 4);
        c.lds = c.off_cnorm + (size_t)KT * 16 * 4;
        if (c.lds > 160 * 1024) continue;
        c.ok = true;
        c.inst = i;
        c.KT = KT;
        c.nsteps = nsteps;
        return c;
    }
    return c;
}

}  // namespace

bool infer_supported(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    return N < ((int64_t)1 << 40) && infer_config(D, K, dt).ok;
}

cat_status infer_apply(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                       const float* gamma, const float* beta, void* corrected, int32_t* assign, const TileWs& ws,
                       hipStream_t st, bool out_bf16, double* inertia) {
    const InferCfg c = infer_config(D, K, dt);
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
    p.inertia = inertia;
    p.out_bf16 = (out_bf16 && dt == CAT_F32) ? 1 : 0;
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
    // (assignment only: the kernel still reads the parameter rows of the cluster it picks; any K x D array will do)
    p.gamma = corrected ? gamma : cw;
    p.beta = corrected ? beta : cw;
    // error bound of the split arithmetic as a fraction of |x| |c| (see the tile kernel): 2^-16 per product with two
    // parts per operand (one part: 2^-8), four such terms in a score difference, plus the fp32 accumulation of the
    // MFMA partial sums of a wave and of the S_c partial dot products
    const bool exact_x = dt == CAT_BF16;
    const int passes = in.P == 2 ? (exact_x ? 2 : 3) : 1;
    const float n_acc = (float)(passes * c.nsteps + in.SC + 8);
    const float split = in.P == 2 ? (exact_x ? 3.1e-5f : 9.4e-5f) : (exact_x ? 8.0e-3f : 1.6e-2f);
    p.tau = split + 4.f * n_acc * 5.96e-8f;
    p.tau2 = 4.0e-7f;
    p.xstride = c.xstride;
    p.xpart = c.xpart;
    p.off_s = c.off_s;
    p.off_cnorm = c.off_cnorm;

    static thread_local int cached_inst = -1, cached_lds = -1, cached_dev = -1, per_cu = 1, ncu = 256;
    const int inst_key = 2 * c.inst + (c.ua ? 1 : 0);
    int dev = 0;
    CAT_HIP_TRY(hipGetDevice(&dev));
    if (cached_inst != inst_key || cached_lds != (int)c.lds || cached_dev != dev) {
        int nb = 0, v = 0;
        const void* f0 = c.ua ? in.fn_ua : in.fn;
        const void* f1 = c.ua ? in.fn_ua_dyn : in.fn_dyn;
        CAT_HIP_TRY(hipFuncSetAttribute(f0, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c.lds));
        CAT_HIP_TRY(hipFuncSetAttribute(f1, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c.lds));
        CAT_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, f0, kInferWaves * kWave, c.lds));
        CAT_HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
        per_cu = nb < 1 ? 1 : nb;
        ncu = v > 0 ? v : 256;
        cached_inst = inst_key;
        cached_lds = (int)c.lds;
        cached_dev = dev;
    }
    const int64_t cap = (int64_t)ncu * per_cu;
    const unsigned blocks = (unsigned)(p.ntiles < cap ? p.ntiles : cap);
    // tiles in order pay from a few dozen tiles per workgroup on (the counters are cleared by a launch of their own)
    const bool dyn = p.ntiles >= 64 * (int64_t)blocks && p.ntiles < ((int64_t)1 << 31) - 8 * (int64_t)blocks;
    const void* fn = c.ua ? (dyn ? in.fn_ua_dyn : in.fn_ua) : (dyn ? in.fn_dyn : in.fn);
    if (dyn) {
        p.counters = (unsigned int*)(ws.cnorm + 512);  // the norms take at most 256 of the 1024 floats
        cat_status fs = launch_fill_zero(p.counters, 8 * 16 * sizeof(unsigned int), st);
        if (fs != CAT_OK) return fs;
    }
    const bool prof = profile_on();
    if (prof) {
        cat_status ps = profile_mark(true, st);
        if (ps != CAT_OK) return ps;
    }
    void* args[] = {(void*)&p};
    CAT_HIP_TRY(hipLaunchKernel(fn, dim3(blocks), dim3(kInferWaves * kWave), args, c.lds, st));
    CAT_LAUNCH_CHECK("k_infer");
    if (prof) return profile_mark(false, st);
    return CAT_OK;
}

}  // namespace cat
