// C ABI of the AQ-SGD boundary codec: argument checks and kernel dispatch.
// See include/aqsgd.h for the contract of every entry point.
#include <atomic>
#include <cstdlib>
#include <limits>
#include <vector>

#include "aqsgd_kernels.h"
#include "aqsgd_lowbit.h"
#include "aqsgd_topk.h"

namespace aqsgd {

thread_local ProfileRequest g_profile_request = {nullptr, nullptr};

// -- dtype fan-out (each dtype's kernels live in their own translation unit) ----
hipError_t launch_codec_jobs(int dtype, int rounding, int shape, bool three, const JobTable& t, hipStream_t s) {
    switch (dtype) {
    case AQSGD_F32:  return launch_codec_jobs_dt<AQSGD_F32>(rounding, shape, three, t, s);
    case AQSGD_F16:  return launch_codec_jobs_dt<AQSGD_F16>(rounding, shape, three, t, s);
    case AQSGD_BF16: return launch_codec_jobs_dt<AQSGD_BF16>(rounding, shape, three, t, s);
    default:         return hipErrorInvalidValue;
    }
}
hipError_t launch_dequant_jobs(int dtype, int unroll, const JobTable& t, hipStream_t s) {
    switch (dtype) {
    case AQSGD_F32:  return launch_dequant_jobs_dt<AQSGD_F32>(unroll, t, s);
    case AQSGD_F16:  return launch_dequant_jobs_dt<AQSGD_F16>(unroll, t, s);
    case AQSGD_BF16: return launch_dequant_jobs_dt<AQSGD_BF16>(unroll, t, s);
    default:         return hipErrorInvalidValue;
    }
}
hipError_t launch_quant_anyshape(int dtype, int bits, int rounding, const QuantJob& a, hipStream_t s) {
    switch (dtype) {
    case AQSGD_F32:  return launch_quant_anyshape_dt<AQSGD_F32>(bits, rounding, a, s);
    case AQSGD_F16:  return launch_quant_anyshape_dt<AQSGD_F16>(bits, rounding, a, s);
    case AQSGD_BF16: return launch_quant_anyshape_dt<AQSGD_BF16>(bits, rounding, a, s);
    default:         return hipErrorInvalidValue;
    }
}
hipError_t launch_dequant_anyshape(int dtype, const DequantJob& a, hipStream_t s) {
    switch (dtype) {
    case AQSGD_F32:  return launch_dequant_anyshape_dt<AQSGD_F32>(a, s);
    case AQSGD_F16:  return launch_dequant_anyshape_dt<AQSGD_F16>(a, s);
    case AQSGD_BF16: return launch_dequant_anyshape_dt<AQSGD_BF16>(a, s);
    default:         return hipErrorInvalidValue;
    }
}

hipError_t launch_lowbit(int dtype, int bits, int m_bits, int shape, bool sender, LaunchGeom g,
                         const LowbitArgs& a, hipStream_t s) {
    switch (dtype) {
    case AQSGD_F32:  return launch_lowbit_dt<AQSGD_F32>(bits, m_bits, shape, sender, g, a, s);
    case AQSGD_F16:  return launch_lowbit_dt<AQSGD_F16>(bits, m_bits, shape, sender, g, a, s);
    case AQSGD_BF16: return launch_lowbit_dt<AQSGD_BF16>(bits, m_bits, shape, sender, g, a, s);
    default:         return hipErrorInvalidValue;
    }
}

namespace {

// Launch-shape knobs.  They change how the work is cut into workgroups, never a
// result bit.  Defaults come from the environment, once, so a sweep needs no
// rebuild; aqsgd_set_launch_shape overrides them for the process.  Each knob is
// an atomic of its own: a call reads each one once, so a change made by another
// thread takes effect for whole calls only.
int env_int(const char* name, int fallback) {
    const char* v = std::getenv(name);
    if (!v || !*v) return fallback;
    char* end = nullptr;
    const long x = std::strtol(v, &end, 10);
    return (end && *end == '\0' && x > 0 && x < (1L << 30)) ? static_cast<int>(x) : fallback;
}

int64_t env_max_blocks() { return env_int("AQSGD_MAX_BLOCKS", 1 << 20); }
int env_dequant_unroll() {
    const int u = env_int("AQSGD_DEQUANT_UNROLL", 2);
    return (u == 1 || u == 2 || u == 4) ? u : 2;
}

std::atomic<int64_t>& max_blocks_knob() {
    static std::atomic<int64_t> v{env_max_blocks()};
    return v;
}
std::atomic<int>& dequant_unroll_knob() {
    static std::atomic<int> v{env_dequant_unroll()};
    return v;
}

// Workgroups per launch that carries several jobs; 0 = the library's own choice (see
// launch_budget).  For sweeps only: AQSGD_LAUNCH_BLOCKS in the environment.
int64_t env_launch_blocks() { return env_int("AQSGD_LAUNCH_BLOCKS", 0); }
std::atomic<int64_t>& launch_blocks_knob() {
    static std::atomic<int64_t> v{env_launch_blocks()};
    return v;
}

constexpr int64_t kMaxGridY = 65535;
constexpr int kMaxTeamChunks = 4096;     // 1024 lanes x 4 chunks x 8 elements = 32768 elements

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_desc(const aqsgd_desc* d, bool needs_buffer) {
    if (!d) return AQSGD_ERR_NULL;
    if (d->dtype != AQSGD_F32 && d->dtype != AQSGD_F16 && d->dtype != AQSGD_BF16) return AQSGD_ERR_DTYPE;
    if (d->rounding != AQSGD_ROUND_NEAREST && d->rounding != AQSGD_ROUND_STOCHASTIC) return AQSGD_ERR_DTYPE;
    if (!(d->bits == 2 || d->bits == 3 || d->bits == 4 || d->bits == 6 || d->bits == 8)) return AQSGD_ERR_BITS;
    if (d->batch < 0 || d->n_per <= 0) return AQSGD_ERR_SHAPE;
    if (d->group <= 0 || d->n_per % d->group != 0) return AQSGD_ERR_GROUP;
    if ((static_cast<int64_t>(d->group) * d->bits) % 8 != 0) return AQSGD_ERR_GROUP;
    const int64_t lim = std::numeric_limits<int64_t>::max() / 16;
    if (d->batch > std::numeric_limits<int32_t>::max()) return AQSGD_ERR_SHAPE;
    if (d->n_per > (int64_t{1} << 34)) return AQSGD_ERR_SHAPE;            // chunk index fits 32 bits
    if (d->batch > 0 && d->n_per > lim / d->batch) return AQSGD_ERR_SHAPE;
    if (needs_buffer) {
        if (d->n_samples <= 0 || d->n_per > lim / d->n_samples) return AQSGD_ERR_SHAPE;
    }
    return AQSGD_OK;
}

int team_shape_for(int cpg) {
    if (cpg <= 8) return kTeam8x1;
    if (cpg <= 16) return kTeam16x1;
    if (cpg <= 32) return kTeam32x1;
    if (cpg <= 64) return kTeam64x1;
    if (cpg <= 128) return kTeam64x2;
    if (cpg <= 192) return kTeam64x3;
    if (cpg <= 256) return kTeam64x4;
    if (cpg <= 512) return kTeam256x2;
    if (cpg <= 1024) return kTeam256x4;
    if (cpg <= 2048) return kTeam1024x2;
    return kTeam1024x4;
}

// Groups one step of a workgroup of the quantising kernel covers (its teams times the
// groups each takes, groups_per_team).
int groups_per_block_step(int shape) {
    switch (shape) {
    case kTeam8x1: return kBlock / 8 * groups_per_team(8, 1);
    case kTeam16x1: return kBlock / 16 * groups_per_team(16, 1);
    case kTeam32x1: return kBlock / 32 * groups_per_team(32, 1);
    case kTeam64x1: return kBlock / 64 * groups_per_team(64, 1);
    case kTeam64x2: case kTeam64x3: case kTeam64x4: return kBlock / 64;
    default: return 1;
    }
}

// Workgroups of one job: grid_y walks the samples, grid_x the pieces of a sample,
// bounded by `max_blocks` in all (the kernels loop over what is left).
LaunchGeom geometry(int64_t units_per_sample, int64_t units_per_block, int64_t batch, int64_t max_blocks) {
    LaunchGeom g;
    const int64_t gy = batch < kMaxGridY ? batch : kMaxGridY;
    int64_t gx = (units_per_sample + units_per_block - 1) / units_per_block;
    const int64_t cap = max_blocks / gy > 0 ? max_blocks / gy : 1;
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    g.grid_x = static_cast<uint32_t>(gx);
    g.grid_y = static_cast<uint32_t>(gy);
    return g;
}

int threads_of_shape(int shape) {
    switch (shape) {
    case kTeam1024x2: case kTeam1024x4: return 1024;
    default: return kBlock;
    }
}

// First-visit arguments of the *_seen entry points (all null / 0 otherwise).
struct SeenArgs {
    uint32_t* seen = nullptr;
    int32_t* first = nullptr;
    const void* full = nullptr;
    uint32_t stamp = 0;
};

// One message as the kernels see it.  Quantising side: aqsgd_encode, aqsgd_grad_quant.
struct QuantPlan {
    QuantJob job;
    int dtype, bits, rounding;
    int shape;                 // team shape, or -1: any-shape kernel (launched on its own)
};

QuantPlan plan_quant(const aqsgd_desc* d, int64_t batch, int64_t n_per, const void* src, const int64_t* ids,
                     void* m_buf, uint8_t* codes, float* scales, const SeenArgs& sa = SeenArgs()) {
    QuantPlan p;
    QuantJob& a = p.job;
    a.src = src; a.ids = ids; a.m_buf = m_buf; a.codes = codes; a.scales = scales;
    a.n_per = n_per; a.gps = n_per / d->group;
    a.batch = static_cast<int32_t>(batch); a.group = d->group; a.cpg = d->group / kChunk; a.bits = d->bits;
    a.grid_x = a.grid_y = 1; a.rcp_grid_x = 1.0f;
    a.seed = d->rng_seed; a.seen = sa.seen; a.first = sa.first; a.stamp = sa.stamp;
    p.dtype = d->dtype; p.bits = d->bits; p.rounding = d->rounding;
    p.shape = (d->group % kChunk == 0 && a.cpg <= kMaxTeamChunks) ? team_shape_for(a.cpg) : -1;
    return p;
}

// Dequantising side: aqsgd_decode, aqsgd_grad_dequant.
struct DequantPlan {
    DequantJob job;
    int dtype;
    bool flat;                 // false: any-shape kernel (launched on its own)
};

DequantPlan plan_dequant(const aqsgd_desc* d, int64_t batch, int64_t n_per, const uint8_t* codes,
                         const float* scales, const int64_t* ids, void* m_buf, void* out,
                         const SeenArgs& sa = SeenArgs()) {
    DequantPlan p;
    DequantJob& a = p.job;
    a.codes = codes; a.scales = scales; a.ids = ids; a.m_buf = m_buf; a.out = out; a.full = sa.full;
    a.n_per = n_per; a.gps = n_per / d->group; a.cps = n_per / kChunk;
    a.batch = static_cast<int32_t>(batch); a.group = d->group; a.cpg = d->group / kChunk; a.bits = d->bits;
    a.grid_x = a.grid_y = 1; a.rcp_grid_x = 1.0f;
    a.seen = sa.seen; a.stamp = sa.stamp;
    p.dtype = d->dtype;
    p.flat = d->group % kChunk == 0;
    return p;
}

// Workgroup budget of a launch led by quantising jobs of team shape `shape`.  A step of a
// small team (one chunk per lane) is short next to what opens a workgroup (job lookup,
// sample id, row addresses: dependent fetches), so a launch of many such workgroups keeps
// much of the chip in that opening; such launches get about as many workgroups as are
// resident at once (eight per compute unit) and each loops over several steps.  Measured
// on the 2-bit G = 128 and the 3-bit G = 64 boundaries: whole step 7-8 % shorter in the
// pipelined schedule, the launch on its own up to 7 % longer.  Launches of the wider
// shapes (a step is four chunks per lane or a whole workgroup's row) lose from it and
// keep one step per workgroup.
int64_t launch_budget(int shape, int64_t knob) {
    if (knob > 0) return knob;
    switch (shape) {
    case kTeam8x1: case kTeam16x1: case kTeam32x1: return 2048;
    default: return int64_t{1} << 40;
    }
}

// Workgroup numbers of a table whose jobs are all in: every job gets the grid its size
// asks for (at most max_blocks), and when the launch as a whole would pass
// `launch_blocks` workgroups the jobs share that budget in proportion to what they asked
// for (the kernels loop over what is left).  quant_step / dequant_step: groups, chunks one
// workgroup step covers.
void number_blocks(JobTable& t, int64_t quant_step, int64_t dequant_step, int64_t max_blocks,
                   int64_t launch_blocks) {
    int64_t want[kMaxQuantJobs + kMaxDequantJobs];
    int64_t total = 0;
    for (int k = 0; k < t.n_quant; ++k) {
        const LaunchGeom g = geometry(t.q[k].gps, quant_step, t.q[k].batch, max_blocks);
        total += want[k] = static_cast<int64_t>(g.grid_x) * g.grid_y;
    }
    for (int k = 0; k < t.n_dequant; ++k) {
        const LaunchGeom g = geometry(t.d[k].cps, dequant_step, t.d[k].batch, max_blocks);
        total += want[kMaxQuantJobs + k] = static_cast<int64_t>(g.grid_x) * g.grid_y;
    }
    const bool shrink = total > launch_blocks;
    auto share = [&](int64_t w) {
        if (!shrink) return max_blocks;
        const int64_t part = static_cast<int64_t>(static_cast<double>(launch_blocks) * static_cast<double>(w) /
                                                  static_cast<double>(total));
        return part < 1 ? int64_t{1} : (part < max_blocks ? part : max_blocks);
    };
    int64_t blocks = 0;
    for (int k = 0; k < t.n_quant; ++k) {
        QuantJob& a = t.q[k];
        const LaunchGeom g = geometry(a.gps, quant_step, a.batch, share(want[k]));
        a.grid_x = g.grid_x; a.grid_y = g.grid_y; a.rcp_grid_x = 1.0f / static_cast<float>(g.grid_x);
        t.q_block0[k] = static_cast<uint32_t>(blocks);
        blocks += static_cast<int64_t>(g.grid_x) * g.grid_y;
    }
    t.dequant_block0 = static_cast<uint32_t>(blocks);
    for (int k = 0; k < t.n_dequant; ++k) {
        DequantJob& a = t.d[k];
        const LaunchGeom g = geometry(a.cps, dequant_step, a.batch, share(want[kMaxQuantJobs + k]));
        a.grid_x = g.grid_x; a.grid_y = g.grid_y; a.rcp_grid_x = 1.0f / static_cast<float>(g.grid_x);
        t.d_block0[k] = static_cast<uint32_t>(blocks);
        blocks += static_cast<int64_t>(g.grid_x) * g.grid_y;
    }
    t.total_blocks = static_cast<uint32_t>(blocks);
}

// The launches of a set of independent messages: quantising jobs that share dtype,
// rounding mode and team shape go into one grid, together with the dequantising
// jobs of that dtype that are still waiting; dequantising jobs without such a host get a
// grid of their own; jobs that need the any-shape kernels are launched one by one.
int launch_plans(std::vector<QuantPlan>& qs, std::vector<DequantPlan>& ds, hipStream_t stream) {
    // a job's workgroup numbers must be exact in binary32 (place_in_job)
    const int64_t knob = max_blocks_knob().load(std::memory_order_relaxed);
    const int64_t max_blocks = knob < (int64_t{1} << 24) ? knob : (int64_t{1} << 24) - 1;
    const int unroll = dequant_unroll_knob().load(std::memory_order_relaxed);
    std::vector<bool> q_done(qs.size(), false), d_done(ds.size(), false);
    hipError_t err = hipSuccess;

    const int64_t launch_blocks = launch_blocks_knob().load(std::memory_order_relaxed);
    auto add_dequant = [&](JobTable& t, int dtype) {
        for (size_t k = 0; k < ds.size() && t.n_dequant < kMaxDequantJobs; ++k) {
            if (d_done[k] || !ds[k].flat || ds[k].dtype != dtype) continue;
            t.d[t.n_dequant++] = ds[k].job;
            d_done[k] = true;
        }
    };

    for (size_t i = 0; i < qs.size() && err == hipSuccess; ++i) {
        if (q_done[i]) continue;
        QuantPlan& lead = qs[i];
        if (lead.shape < 0) {                            // any-shape kernel, on its own
            const LaunchGeom g = geometry(lead.job.gps, kBlock, lead.job.batch, max_blocks);
            lead.job.grid_x = g.grid_x; lead.job.grid_y = g.grid_y;
            err = launch_quant_anyshape(lead.dtype, lead.bits, lead.rounding, lead.job, stream);
            q_done[i] = true;
            continue;
        }
        JobTable t;
        t.n_quant = t.n_dequant = 0;
        bool three = false;                              // a 3-bit job among them: the kernel variant that has those bodies
        for (size_t k = i; k < qs.size() && t.n_quant < kMaxQuantJobs; ++k) {
            const QuantPlan& c = qs[k];
            if (q_done[k] || c.shape != lead.shape || c.dtype != lead.dtype || c.rounding != lead.rounding)
                continue;
            three = three || c.bits == 3;
            t.q[t.n_quant++] = c.job;
            q_done[k] = true;
        }
        add_dequant(t, lead.dtype);
        number_blocks(t, groups_per_block_step(lead.shape),
                      static_cast<int64_t>(threads_of_shape(lead.shape)) * kHostedDequantUnroll, max_blocks,
                      launch_budget(lead.shape, launch_blocks));
        err = launch_codec_jobs(lead.dtype, lead.rounding, lead.shape, three, t, stream);
    }
    for (size_t i = 0; i < ds.size() && err == hipSuccess; ++i) {
        if (d_done[i]) continue;
        if (!ds[i].flat) {
            DequantJob& a = ds[i].job;
            const LaunchGeom g = geometry(a.gps, kBlock, a.batch, max_blocks);
            a.grid_x = g.grid_x; a.grid_y = g.grid_y;
            err = launch_dequant_anyshape(ds[i].dtype, a, stream);
            d_done[i] = true;
            continue;
        }
        JobTable t;
        t.n_quant = t.n_dequant = 0;
        add_dequant(t, ds[i].dtype);
        number_blocks(t, 1, static_cast<int64_t>(kBlock) * unroll, max_blocks, launch_budget(-1, launch_blocks));
        err = launch_dequant_jobs(ds[i].dtype, unroll, t, stream);
    }
    return err == hipSuccess ? AQSGD_OK : AQSGD_ERR_LAUNCH;
}

int launch_one(const QuantPlan& q, hipStream_t stream) {
    std::vector<QuantPlan> qs(1, q);
    std::vector<DequantPlan> ds;
    return launch_plans(qs, ds, stream);
}

int launch_one(const DequantPlan& d, hipStream_t stream) {
    std::vector<QuantPlan> qs;
    std::vector<DequantPlan> ds(1, d);
    return launch_plans(qs, ds, stream);
}

// Row copy for the uncompressed first visit of aqsgd_seed: m_buf[ids[i]] <- act[i].
// V = 16 bytes per lane and step (streaming accesses) when the row size allows it,
// else one element.
template <typename V>
__global__ __launch_bounds__(kBlock)
void seed_rows_kernel(const V* act, const int64_t* ids, V* m_buf, int64_t units_per_row, int batch) {
    for (int i = blockIdx.y; i < batch; i += gridDim.y) {
        const int64_t row = sample_id(ids, i);
        const V* src = act + static_cast<int64_t>(i) * units_per_row;
        V* dst = m_buf + row * units_per_row;
        for (int64_t c = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; c < units_per_row;
             c += static_cast<int64_t>(gridDim.x) * kBlock) {
            if constexpr (sizeof(V) == 16) {
                const V v = __builtin_nontemporal_load(src + c);
                store16_through(dst + c, v);
            } else {
                dst[c] = src[c];
            }
        }
    }
}

template <typename V>
hipError_t launch_seed_rows_as(const aqsgd_desc* d, int64_t row_bytes, const void* act, const int64_t* ids,
                               void* m_buf, hipStream_t s) {
    const int64_t units = row_bytes / static_cast<int64_t>(sizeof(V));
    const LaunchGeom g = geometry(units, static_cast<int64_t>(kBlock) * (sizeof(V) == 16 ? 2 : 4), d->batch,
                            max_blocks_knob().load(std::memory_order_relaxed));
    return launch_kernel(seed_rows_kernel<V>, dim3(g.grid_x, g.grid_y), dim3(kBlock), s,
                         static_cast<const V*>(act), ids, static_cast<V*>(m_buf), units,
                         static_cast<int>(d->batch));
}

hipError_t launch_seed_rows(const aqsgd_desc* d, const void* act, const int64_t* ids, void* m_buf,
                            hipStream_t s) {
    const int64_t eb = d->dtype == AQSGD_F32 ? 4 : 2;
    const int64_t row_bytes = d->n_per * eb;
    if (row_bytes % 16 == 0) return launch_seed_rows_as<u32x4_t>(d, row_bytes, act, ids, m_buf, s);
    if (eb == 4) return launch_seed_rows_as<uint32_t>(d, row_bytes, act, ids, m_buf, s);
    return launch_seed_rows_as<uint16_t>(d, row_bytes, act, ids, m_buf, s);
}

int check_encode(const aqsgd_desc* d, const void* act, const int64_t* ids, const void* m_buf,
                 const uint8_t* codes, const float* scales) {
    const int rc = check_desc(d, true);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    if (!act || !ids || !m_buf || !codes || !scales) return AQSGD_ERR_NULL;
    if (!aligned(act, 16) || !aligned(m_buf, 16) || !aligned(codes, 16) || !aligned(scales, 4) ||
        !aligned(ids, 8))
        return AQSGD_ERR_ALIGN;
    return AQSGD_OK;
}

int check_decode(const aqsgd_desc* d, const uint8_t* codes, const float* scales, const int64_t* ids,
                 const void* m_buf, const void* out) {
    const int rc = check_desc(d, true);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    if (!codes || !scales || !ids || !m_buf || !out) return AQSGD_ERR_NULL;
    if (!aligned(out, 16) || !aligned(m_buf, 16) || !aligned(codes, 16) || !aligned(scales, 4) ||
        !aligned(ids, 8))
        return AQSGD_ERR_ALIGN;
    return AQSGD_OK;
}

int check_grad_quant(const aqsgd_desc* d, const void* grad, const uint8_t* codes, const float* scales) {
    const int rc = check_desc(d, false);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    if (!grad || !codes || !scales) return AQSGD_ERR_NULL;
    if (!aligned(grad, 16) || !aligned(codes, 16) || !aligned(scales, 4)) return AQSGD_ERR_ALIGN;
    return AQSGD_OK;
}

int check_grad_dequant(const aqsgd_desc* d, const uint8_t* codes, const float* scales, const void* out) {
    const int rc = check_desc(d, false);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    if (!codes || !scales || !out) return AQSGD_ERR_NULL;
    if (!aligned(out, 16) || !aligned(codes, 16) || !aligned(scales, 4)) return AQSGD_ERR_ALIGN;
    return AQSGD_OK;
}

// The backward message has no per-sample rows to gather, and n_per is a multiple of
// the group, so the call tensor is treated as one long sample.
QuantPlan plan_grad_quant(const aqsgd_desc* d, const void* grad, uint8_t* codes, float* scales) {
    const int64_t n = d->batch * d->n_per;
    const bool flat = n <= (int64_t{1} << 34);
    return plan_quant(d, flat ? 1 : d->batch, flat ? n : d->n_per, grad, nullptr, nullptr, codes, scales);
}

DequantPlan plan_grad_dequant(const aqsgd_desc* d, const uint8_t* codes, const float* scales, void* out) {
    const int64_t n = d->batch * d->n_per;
    const bool flat = n <= (int64_t{1} << 34);
    return plan_dequant(d, flat ? 1 : d->batch, flat ? n : d->n_per, codes, scales, nullptr, nullptr, out);
}

int lowbit_shape_for(int cpg) {
    if (cpg <= 8) return kLb8x1;
    if (cpg <= 16) return kLb16x1;
    if (cpg <= 32) return kLb32x1;
    if (cpg <= 64) return kLb64x1;
    if (cpg <= 128) return kLb64x2;
    if (cpg <= 192) return kLb64x3;
    if (cpg <= 256) return kLb64x4;
    if (cpg <= 512) return kLb256x2;
    if (cpg <= 1024) return kLb256x4;
    return kLb1024x2;
}

int lowbit_teams_per_block(int shape) {
    switch (shape) {
    case kLb8x1: return kBlock / 8;
    case kLb16x1: return kBlock / 16;
    case kLb32x1: return kBlock / 32;
    case kLb64x1: case kLb64x2: case kLb64x3: case kLb64x4: return kBlock / 64;
    default: return 1;
    }
}

int check_lowbit(const aqsgd_desc* d, int32_t m_bits) {
    const int rc = check_desc(d, true);
    if (rc != AQSGD_OK) return rc;
    if (m_bits != 2 && m_bits != 8) return AQSGD_ERR_BITS;
    if (d->group % kChunk != 0 || d->group / kChunk > kMaxLowbitChunks) return AQSGD_ERR_GROUP;
    return AQSGD_OK;
}

int run_lowbit(const aqsgd_desc* d, int32_t m_bits, bool sender, const void* act, void* out,
               const int64_t* ids, uint8_t* m_codes, float* m_scales, uint8_t* codes, float* scales,
               hipStream_t stream) {
    LowbitArgs a;
    a.act = act; a.out = out; a.ids = ids; a.m_codes = m_codes; a.m_scales = m_scales;
    a.codes = codes; a.scales = scales;
    a.n_per = d->n_per; a.gps = d->n_per / d->group;
    a.batch = static_cast<int32_t>(d->batch); a.group = d->group; a.cpg = d->group / kChunk;
    a.stochastic = d->rounding == AQSGD_ROUND_STOCHASTIC; a.seed = d->rng_seed;
    const int shape = lowbit_shape_for(a.cpg);
    const hipError_t err = launch_lowbit(d->dtype, d->bits, m_bits, shape, sender,
                                         geometry(a.gps, lowbit_teams_per_block(shape), d->batch,
                                                  max_blocks_knob().load(std::memory_order_relaxed)),
                                         a, stream);
    return err == hipSuccess ? AQSGD_OK : AQSGD_ERR_LAUNCH;
}

int check_topk(const aqsgd_desc* d, int32_t keep) {
    const int rc = check_desc(d, false);
    if (rc != AQSGD_OK) return rc;
    if (d->bits != kTopkBits) return AQSGD_ERR_BITS;
    if (d->group % kChunk != 0 || d->group > kTopkMaxGroup) return AQSGD_ERR_GROUP;
    if (keep < 1 || keep > d->group) return AQSGD_ERR_SHAPE;
    return AQSGD_OK;
}

int run_topk(const aqsgd_desc* d, int32_t keep, bool sender, const void* grad, void* out, uint8_t* bitmap,
             uint8_t* codes, float* scales, hipStream_t stream) {
    TopkArgs a;
    a.grad = grad; a.out = out; a.bitmap = bitmap; a.codes = codes; a.scales = scales;
    a.n_groups = d->batch * (d->n_per / d->group);
    a.group = d->group; a.cpg = d->group / kChunk; a.keep = keep;
    a.stochastic = d->rounding == AQSGD_ROUND_STOCHASTIC; a.seed = d->rng_seed;
    const int cpl = a.cpg <= kWave ? 1 : (a.cpg <= 2 * kWave ? 2 : (a.cpg <= 3 * kWave ? 3 : 4));
    const LaunchGeom g = geometry(a.n_groups, kTopkBlock / kWave, 1,
                                  max_blocks_knob().load(std::memory_order_relaxed));
    const hipError_t err = launch_topk(d->dtype, cpl, sender, g.grid_x, a, stream);
    return err == hipSuccess ? AQSGD_OK : AQSGD_ERR_LAUNCH;
}

__global__ void check_ids_kernel(const int64_t* ids, int64_t batch, int64_t n_samples, int32_t* flag) {
    int bad = 0;
    for (int64_t i = threadIdx.x + static_cast<int64_t>(blockIdx.x) * blockDim.x; i < batch;
         i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
        const int64_t v = ids[i];
        if (v < 0 || v >= n_samples) bad |= 1;
        for (int64_t j = 0; j < i; ++j)
            if (ids[j] == v) bad |= 2;
    }
    if (bad) atomicOr(flag, bad);
}

}  // namespace
}  // namespace aqsgd

using namespace aqsgd;

extern "C" {

size_t aqsgd_codes_bytes(const aqsgd_desc* d) {
    if (check_desc(d, false) != AQSGD_OK) return 0;
    return static_cast<size_t>(d->batch) * static_cast<size_t>(d->n_per) * d->bits / 8;
}

size_t aqsgd_scales_count(const aqsgd_desc* d) {
    if (check_desc(d, false) != AQSGD_OK) return 0;
    return static_cast<size_t>(d->batch) * static_cast<size_t>(d->n_per / d->group);
}

int aqsgd_encode(const aqsgd_desc* d, const void* act, const int64_t* sample_ids, void* m_buf,
                 uint8_t* codes, float* scales, void* stream) {
    const int rc = check_encode(d, act, sample_ids, m_buf, codes, scales);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    return launch_one(plan_quant(d, d->batch, d->n_per, act, sample_ids, m_buf, codes, scales),
                      static_cast<hipStream_t>(stream));
}

int aqsgd_decode(const aqsgd_desc* d, const uint8_t* codes, const float* scales,
                 const int64_t* sample_ids, void* m_buf, void* out, void* stream) {
    const int rc = check_decode(d, codes, scales, sample_ids, m_buf, out);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    return launch_one(plan_dequant(d, d->batch, d->n_per, codes, scales, sample_ids, m_buf, out),
                      static_cast<hipStream_t>(stream));
}

int aqsgd_grad_quant(const aqsgd_desc* d, const void* grad, uint8_t* codes, float* scales,
                     void* stream) {
    const int rc = check_grad_quant(d, grad, codes, scales);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    return launch_one(plan_grad_quant(d, grad, codes, scales), static_cast<hipStream_t>(stream));
}

int aqsgd_grad_dequant(const aqsgd_desc* d, const uint8_t* codes, const float* scales, void* out,
                       void* stream) {
    const int rc = check_grad_dequant(d, codes, scales, out);
    if (rc != AQSGD_OK || d->batch == 0) return rc;
    return launch_one(plan_grad_dequant(d, codes, scales, out), static_cast<hipStream_t>(stream));
}

int aqsgd_run_jobs(const aqsgd_job* jobs, int32_t n_jobs, void* stream) {
    if (n_jobs < 0) return AQSGD_ERR_SHAPE;
    if (n_jobs == 0) return AQSGD_OK;
    if (!jobs) return AQSGD_ERR_NULL;
    std::vector<QuantPlan> qs;
    std::vector<DequantPlan> ds;
    for (int32_t k = 0; k < n_jobs; ++k) {               // every job is checked before anything is enqueued
        const aqsgd_job& j = jobs[k];
        const aqsgd_desc* d = &j.desc;
        int rc;
        switch (j.kind) {
        case AQSGD_JOB_ENCODE:
            rc = check_encode(d, j.src, j.sample_ids, j.m_buf, j.codes, j.scales);
            if (rc == AQSGD_OK && d->batch > 0)
                qs.push_back(plan_quant(d, d->batch, d->n_per, j.src, j.sample_ids, j.m_buf, j.codes, j.scales));
            break;
        case AQSGD_JOB_DECODE:
            rc = check_decode(d, j.codes, j.scales, j.sample_ids, j.m_buf, j.out);
            if (rc == AQSGD_OK && d->batch > 0)
                ds.push_back(plan_dequant(d, d->batch, d->n_per, j.codes, j.scales, j.sample_ids, j.m_buf, j.out));
            break;
        case AQSGD_JOB_GRAD_QUANT:
            rc = check_grad_quant(d, j.src, j.codes, j.scales);
            if (rc == AQSGD_OK && d->batch > 0) qs.push_back(plan_grad_quant(d, j.src, j.codes, j.scales));
            break;
        case AQSGD_JOB_GRAD_DEQUANT:
            rc = check_grad_dequant(d, j.codes, j.scales, j.out);
            if (rc == AQSGD_OK && d->batch > 0) ds.push_back(plan_grad_dequant(d, j.codes, j.scales, j.out));
            break;
        case AQSGD_JOB_ENCODE_SEEN: {
            rc = check_encode(d, j.src, j.sample_ids, j.m_buf, j.codes, j.scales);
            if (rc == AQSGD_OK && j.stamp == 0) rc = AQSGD_ERR_SHAPE;
            if (rc != AQSGD_OK || d->batch == 0) break;
            if (!j.seen || !j.first) { rc = AQSGD_ERR_NULL; break; }
            if (!aligned(j.first, 4) || !aligned(j.seen, 4)) { rc = AQSGD_ERR_ALIGN; break; }
            SeenArgs sa;
            sa.seen = j.seen; sa.first = j.first; sa.stamp = j.stamp;
            qs.push_back(plan_quant(d, d->batch, d->n_per, j.src, j.sample_ids, j.m_buf, j.codes, j.scales, sa));
            break;
        }
        case AQSGD_JOB_DECODE_SEEN: {
            rc = check_decode(d, j.codes, j.scales, j.sample_ids, j.m_buf, j.out);
            if (rc == AQSGD_OK && j.stamp == 0) rc = AQSGD_ERR_SHAPE;
            if (rc != AQSGD_OK || d->batch == 0) break;
            if (!j.seen || !j.full) { rc = AQSGD_ERR_NULL; break; }
            if (!aligned(j.full, 16) || !aligned(j.seen, 4)) { rc = AQSGD_ERR_ALIGN; break; }
            SeenArgs sa;
            sa.seen = j.seen; sa.full = j.full; sa.stamp = j.stamp;
            ds.push_back(plan_dequant(d, d->batch, d->n_per, j.codes, j.scales, j.sample_ids, j.m_buf, j.out, sa));
            break;
        }
        default:
            rc = AQSGD_ERR_SHAPE;
        }
        if (rc != AQSGD_OK) return rc;
    }
    return launch_plans(qs, ds, static_cast<hipStream_t>(stream));
}

int aqsgd_seed(const aqsgd_desc* d, const void* act, const int64_t* sample_ids, void* m_buf,
               void* stream) {
    const int rc = check_desc(d, true);
    if (rc != AQSGD_OK) return rc;
    if (d->batch == 0) return AQSGD_OK;
    if (!act || !sample_ids || !m_buf) return AQSGD_ERR_NULL;
    if (!aligned(act, 16) || !aligned(m_buf, 16) || !aligned(sample_ids, 8)) return AQSGD_ERR_ALIGN;
    const hipError_t err = launch_seed_rows(d, act, sample_ids, m_buf, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? AQSGD_OK : AQSGD_ERR_LAUNCH;
}

int aqsgd_encode_seen(const aqsgd_desc* d, const void* act, const int64_t* sample_ids, void* m_buf,
                      uint32_t* seen, uint32_t stamp, int32_t* first, uint8_t* codes, float* scales,
                      void* stream) {
    const int rc = check_encode(d, act, sample_ids, m_buf, codes, scales);
    if (rc != AQSGD_OK) return rc;
    if (stamp == 0) return AQSGD_ERR_SHAPE;
    if (d->batch == 0) return AQSGD_OK;
    if (!seen || !first) return AQSGD_ERR_NULL;
    if (!aligned(first, 4) || !aligned(seen, 4)) return AQSGD_ERR_ALIGN;
    SeenArgs sa;
    sa.seen = seen; sa.first = first; sa.stamp = stamp;
    return launch_one(plan_quant(d, d->batch, d->n_per, act, sample_ids, m_buf, codes, scales, sa),
                      static_cast<hipStream_t>(stream));
}

int aqsgd_decode_seen(const aqsgd_desc* d, const uint8_t* codes, const float* scales, const void* full,
                      const int64_t* sample_ids, void* m_buf, uint32_t* seen, uint32_t stamp, void* out,
                      void* stream) {
    const int rc = check_decode(d, codes, scales, sample_ids, m_buf, out);
    if (rc != AQSGD_OK) return rc;
    if (stamp == 0) return AQSGD_ERR_SHAPE;
    if (d->batch == 0) return AQSGD_OK;
    if (!seen || !full) return AQSGD_ERR_NULL;
    if (!aligned(full, 16) || !aligned(seen, 4)) return AQSGD_ERR_ALIGN;
    SeenArgs sa;
    sa.seen = seen; sa.full = full; sa.stamp = stamp;
    return launch_one(plan_dequant(d, d->batch, d->n_per, codes, scales, sample_ids, m_buf, out, sa),
                      static_cast<hipStream_t>(stream));
}

size_t aqsgd_lowbit_row_bytes(const aqsgd_desc* d, int32_t m_bits) {
    if (check_lowbit(d, m_bits) != AQSGD_OK) return 0;
    return static_cast<size_t>(d->n_per) * m_bits / 8;
}

int aqsgd_encode_lowbit(const aqsgd_desc* d, int32_t m_bits, const void* act, const int64_t* sample_ids,
                        uint8_t* m_codes, float* m_scales, uint8_t* codes, float* scales, void* stream) {
    const int rc = check_lowbit(d, m_bits);
    if (rc != AQSGD_OK) return rc;
    if (d->batch == 0) return AQSGD_OK;
    if (!act || !sample_ids || !m_codes || !m_scales || !codes || !scales) return AQSGD_ERR_NULL;
    if (!aligned(act, 16) || !aligned(m_codes, 16) || !aligned(codes, 16) || !aligned(scales, 4) ||
        !aligned(m_scales, 4) || !aligned(sample_ids, 8))
        return AQSGD_ERR_ALIGN;
    return run_lowbit(d, m_bits, true, act, nullptr, sample_ids, m_codes, m_scales, codes, scales,
                      static_cast<hipStream_t>(stream));
}

int aqsgd_decode_lowbit(const aqsgd_desc* d, int32_t m_bits, const uint8_t* codes, const float* scales,
                        const int64_t* sample_ids, uint8_t* m_codes, float* m_scales, void* out,
                        void* stream) {
    const int rc = check_lowbit(d, m_bits);
    if (rc != AQSGD_OK) return rc;
    if (d->batch == 0) return AQSGD_OK;
    if (!codes || !scales || !sample_ids || !m_codes || !m_scales || !out) return AQSGD_ERR_NULL;
    if (!aligned(out, 16) || !aligned(m_codes, 16) || !aligned(codes, 16) || !aligned(scales, 4) ||
        !aligned(m_scales, 4) || !aligned(sample_ids, 8))
        return AQSGD_ERR_ALIGN;
    return run_lowbit(d, m_bits, false, nullptr, out, sample_ids, m_codes, m_scales,
                      const_cast<uint8_t*>(codes), const_cast<float*>(scales), static_cast<hipStream_t>(stream));
}

size_t aqsgd_topk_bitmap_bytes(const aqsgd_desc* d) {
    if (check_topk(d, 1) != AQSGD_OK) return 0;
    return static_cast<size_t>(d->batch) * static_cast<size_t>(d->n_per) / 8;
}

size_t aqsgd_topk_codes_bytes(const aqsgd_desc* d, int32_t keep) {
    if (check_topk(d, keep) != AQSGD_OK) return 0;
    return static_cast<size_t>(d->batch) * static_cast<size_t>(d->n_per / d->group) * keep;
}

int aqsgd_grad_topk_quant(const aqsgd_desc* d, int32_t keep, const void* grad, uint8_t* bitmap,
                          uint8_t* codes, float* scales, void* stream) {
    const int rc = check_topk(d, keep);
    if (rc != AQSGD_OK) return rc;
    if (d->batch == 0) return AQSGD_OK;
    if (!grad || !bitmap || !codes || !scales) return AQSGD_ERR_NULL;
    if (!aligned(grad, 16) || !aligned(scales, 4) || (keep % 16 == 0 && !aligned(codes, 16)))
        return AQSGD_ERR_ALIGN;
    return run_topk(d, keep, true, grad, nullptr, bitmap, codes, scales, static_cast<hipStream_t>(stream));
}

int aqsgd_grad_topk_dequant(const aqsgd_desc* d, int32_t keep, const uint8_t* bitmap, const uint8_t* codes,
                            const float* scales, void* out, void* stream) {
    const int rc = check_topk(d, keep);
    if (rc != AQSGD_OK) return rc;
    if (d->batch == 0) return AQSGD_OK;
    if (!bitmap || !codes || !scales || !out) return AQSGD_ERR_NULL;
    if (!aligned(out, 16) || !aligned(scales, 4) || (keep % 16 == 0 && !aligned(codes, 16)))
        return AQSGD_ERR_ALIGN;
    return run_topk(d, keep, false, nullptr, out, const_cast<uint8_t*>(bitmap), const_cast<uint8_t*>(codes),
                    const_cast<float*>(scales), static_cast<hipStream_t>(stream));
}

int aqsgd_check_ids(const int64_t* sample_ids, int64_t batch, int64_t n_samples, int32_t* flag,
                    void* stream) {
    if (batch < 0 || n_samples < 0) return AQSGD_ERR_SHAPE;
    if (batch == 0) return AQSGD_OK;
    if (!sample_ids || !flag) return AQSGD_ERR_NULL;
    if (!aligned(sample_ids, 8) || !aligned(flag, 4)) return AQSGD_ERR_ALIGN;
    const int64_t blocks = (batch + kBlock - 1) / kBlock;
    const hipError_t err = launch_kernel(check_ids_kernel, dim3(static_cast<unsigned>(blocks < 1024 ? blocks : 1024)),
                                         dim3(kBlock), static_cast<hipStream_t>(stream), sample_ids, batch,
                                         n_samples, flag);
    return err == hipSuccess ? AQSGD_OK : AQSGD_ERR_LAUNCH;
}

int aqsgd_set_launch_shape(int64_t max_blocks, int32_t dequant_unroll) {
    if (max_blocks < 0 || max_blocks >= (int64_t{1} << 30)) return AQSGD_ERR_SHAPE;
    if (dequant_unroll != 0 && dequant_unroll != 1 && dequant_unroll != 2 && dequant_unroll != 4)
        return AQSGD_ERR_SHAPE;
    max_blocks_knob().store(max_blocks ? max_blocks : env_max_blocks(), std::memory_order_relaxed);
    dequant_unroll_knob().store(dequant_unroll ? dequant_unroll : env_dequant_unroll(),
                                std::memory_order_relaxed);
    return AQSGD_OK;
}

int aqsgd_profile_next_launch(void* start_event, void* stop_event) {
    g_profile_request.start = static_cast<hipEvent_t>(start_event);
    g_profile_request.stop = static_cast<hipEvent_t>(stop_event);
    return AQSGD_OK;
}

const char* aqsgd_strerror(int status) {
    switch (status) {
    case AQSGD_OK:         return "ok";
    case AQSGD_ERR_NULL:   return "a required pointer is NULL";
    case AQSGD_ERR_BITS:   return "bits must be 2, 3, 4, 6 or 8";
    case AQSGD_ERR_GROUP:  return "group must be positive, divide n_per, and hold whole bytes of codes";
    case AQSGD_ERR_DTYPE:  return "unknown dtype or rounding mode";
    case AQSGD_ERR_SHAPE:  return "a size, count, stamp or slot is negative, zero, too large or out of turn";
    case AQSGD_ERR_ALIGN:  return "a pointer misses its required alignment";
    case AQSGD_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case AQSGD_ERR_IO:     return "the file tier could not open, size, read or write its file";
    default:               return "unknown status";
    }
}

const char* aqsgd_version(void) { return "0.1.0"; }

}  // extern "C"
