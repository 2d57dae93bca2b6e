// Host side of libsconv: descriptor and CSR validation, canonical offset lowering
// (Figure 2's colidx -> f(c,r,s)), choice of a tiling, and packing of the nonzeros
// into the order and units the kernels read.  No device work happens here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

#include "sconv_internal.h"

namespace sconv {

int validate_desc(const sconv_desc &d)
{
    if (d.C < 1 || d.H < 1 || d.W < 1 || d.K < 1 || d.R < 1 || d.S < 1) return SCONV_ERR_DESC;
    if (d.stride < 1 || d.pad < 0 || d.groups < 1) return SCONV_ERR_DESC;
    if (d.C % d.groups || d.K % d.groups) return SCONV_ERR_DESC;
    if ((int64_t)d.H + 2 * (int64_t)d.pad < d.R || (int64_t)d.W + 2 * (int64_t)d.pad < d.S) return SCONV_ERR_DESC;
    // offsets inside one (padded) image and one group's CSR columns must fit int32
    const int64_t Hp = (int64_t)d.H + 2 * d.pad, Wp = (int64_t)d.W + 2 * d.pad;
    if ((int64_t)d.C * Hp * Wp >= (int64_t)1 << 30) return SCONV_ERR_RANGE;
    if ((int64_t)(d.C / d.groups) * d.R * d.S >= (int64_t)1 << 30) return SCONV_ERR_RANGE;
    if ((int64_t)d.K * (d.C / d.groups) * d.R * d.S >= (int64_t)1 << 31) return SCONV_ERR_RANGE;
    if (d.R > 255 || d.S > 255 || d.pad > 255) return SCONV_ERR_RANGE;
    return SCONV_OK;
}

// Figure 2's layout function on the zero-padded image.  CHW: f(c,r,s) = (c*Hp + r)*Wp + s.  HWC (channel
// innermost): f(c,r,s) = (r*Wp + s)*C + c.  Both are additive in the position, which is all Section 2.1 asks.
void lower_offsets(const sconv_desc &d, int layout, const int32_t *rowptr, const int32_t *colidx, int32_t *off)
{
    const Geometry g = geometry(d);
    for (int k = 0; k < d.K; ++k) {
        const int grp = k / g.Kg;
        for (int j = rowptr[k]; j < rowptr[k + 1]; ++j) {
            const int col = colidx[j];
            const int s = col % d.S, r = (col / d.S) % d.R, ch = grp * g.Cg + col / (d.S * d.R);
            off[j] = layout == SCONV_LAYOUT_HWC ? (r * g.Wp + s) * d.C + ch : (ch * g.Hp + r) * g.Wp + s;
        }
    }
}

static void lower(const sconv_desc &d, Canonical &c)
{
    c.off.resize(c.colidx.size());
    lower_offsets(d, SCONV_LAYOUT_CHW, c.rowptr.data(), c.colidx.data(), c.off.data());
}

int validate_csr(const sconv_desc &d, const int32_t *rowptr, const int32_t *colidx)
{
    const Geometry g = geometry(d);
    const int64_t ncol = (int64_t)g.Cg * d.R * d.S;
    if (rowptr[0] != 0) return SCONV_ERR_CSR;
    for (int k = 0; k < d.K; ++k)
        if (rowptr[k + 1] < rowptr[k]) return SCONV_ERR_CSR;
    if (rowptr[d.K] > 0 && !colidx) return SCONV_ERR_NULL;
    for (int k = 0; k < d.K; ++k) {
        if ((int64_t)rowptr[k + 1] - rowptr[k] > ncol) return SCONV_ERR_CSR;
        for (int32_t j = rowptr[k]; j < rowptr[k + 1]; ++j) {
            if (colidx[j] < 0 || colidx[j] >= ncol) return SCONV_ERR_CSR;
            if (j > rowptr[k] && colidx[j] <= colidx[j - 1]) return SCONV_ERR_CSR;
        }
    }
    return SCONV_OK;
}

int build_canonical_from_dense(const sconv_desc &d, const float *w, Canonical &out)
{
    const Geometry g = geometry(d);
    const int64_t ncol = (int64_t)g.Cg * d.R * d.S;
    out.rowptr.assign(d.K + 1, 0);
    out.colidx.clear();
    out.val.clear();
    for (int k = 0; k < d.K; ++k) {
        const float *row = w + (int64_t)k * ncol;
        for (int64_t j = 0; j < ncol; ++j) {
            if (row[j] == 0.0f) continue; // +0 and -0 are pruned; NaN compares unequal and stays
            out.colidx.push_back((int32_t)j);
            out.val.push_back(row[j]);
        }
        out.rowptr[k + 1] = (int32_t)out.colidx.size();
    }
    lower(d, out);
    return SCONV_OK;
}

int build_canonical_from_arrays(const sconv_desc &d, const int32_t *rowptr, const int32_t *colidx,
                                const float *values, Canonical &out)
{
    const int rc = validate_csr(d, rowptr, colidx);
    if (rc) return rc;
    const int32_t nnz = rowptr[d.K];
    if (nnz > 0 && !values) return SCONV_ERR_NULL;
    out.rowptr.assign(rowptr, rowptr + d.K + 1);
    out.colidx.assign(colidx, colidx + nnz);
    out.val.assign(values, values + nnz);
    lower(d, out);
    return SCONV_OK;
}

// ------------------------------------------------------------------ tiling

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Row pitch of the LDS plane.  W + pad columns are enough for the reads: one that runs into the right
// padding of a row (X >= W + pad) lands on column X - pitch < pad of the next row, left padding, zero as
// well.  The pitch must also hold a whole output row, which is wider than that when pad > S - 1, and a
// whole filter row, so that two taps never share a cell (images narrower than the filter: both taps would
// read nothing but padding, yet the packing could no longer be decoded).
// With strips, lane l of a chunk sits on cell (l / strip) * pitch + l % strip; a pitch congruent to the strip
// width modulo 16 makes that congruent to l, so that the 64 lanes of a 16-byte read fall on the LDS banks
// exactly as 64 consecutive cells do (the natural pitch costs a third of the read rate in bank conflicts).
static int lds_pitch(const sconv_desc &d, int strip = 0)
{
    const Geometry g = geometry(d);
    int pitch = std::max(std::max(d.W + d.pad, g.OW), d.S);
    while (strip && (pitch - strip) % 16) ++pitch;
    return pitch;
}

static int fill_tiling(const sconv_desc &d, const sconv_plan &p, LdsTiling &t, int phase_cg = 0)
{
    const Geometry g = geometry(d);
    if (d.stride != 1) return SCONV_ERR_PLAN;
    if (p.nt < 1 || p.cb < 1 || p.waves < 1 || p.waves > 16 || p.cg < 1 || p.rows_w < 1 || p.t < 1) return SCONV_ERR_PLAN;
    if (p.band < 0 || p.band > g.OH) return SCONV_ERR_PLAN;
    if (p.waves % p.cg) return SCONV_ERR_PLAN;
    t.p = p;
    if (!is_flat_kernel(p.kernel)) t.p.kernel = 1;
    const bool flat = is_flat_kernel(t.p.kernel), flow = t.p.kernel == 4;
    t.vec = (p.nt % 4 == 0) ? 4 : 1;
    if ((64 * t.vec) % p.nt) return SCONV_ERR_PLAN;
    if (p.strip < 0 || p.strip > 64 || (p.strip && !flat)) return SCONV_ERR_PLAN;
    if (flat) {
        if (p.nt != 4 || !lds2_kernel_available(p.t, p.rows_w, p.strip ? p.strip : 64)) return SCONV_ERR_PLAN;
    } else if (!lds_kernel_available(t.vec, p.t, p.rows_w)) {
        return SCONV_ERR_PLAN;
    }
    t.strip_rows = p.strip ? 64 / p.strip : 0;
    t.out_pos = 1;
    if (p.splits < 0 || (p.splits > 1 && !flat)) return SCONV_ERR_PLAN;
    if (t.p.splits == 0) t.p.splits = 1;
    if (t.p.band == 0) t.p.band = p.strip ? std::min(g.OH, p.cg * t.strip_rows) : g.OH;
    t.n_bands = ceil_div(g.OH, t.p.band);
    t.Wl = lds_pitch(d, p.strip);
    t.Hl = t.p.band + d.R - 1;
    t.plane_cells = t.Hl * t.Wl;
    t.pos_span = (t.p.band - 1) * t.Wl + g.OW;
    t.pos_per_chunk = 64 * t.vec / p.nt;
    t.n_chunks = ceil_div(t.pos_span, t.pos_per_chunk);
    if (p.strip) {
        // t strips of `strip` columns cover the width, cg blocks of strip_rows rows the band
        if (p.t * p.strip < g.OW || t.p.band > p.cg * t.strip_rows) return SCONV_ERR_PLAN;
        t.n_chunks = p.cg * p.t;
    } else if (t.n_chunks > p.cg * p.t) {
        return SCONV_ERR_PLAN;
    }
    if (p.cb > g.Cg) t.p.cb = g.Cg;
    t.nblk = ceil_div(g.Cg, t.p.cb);
    // A strided layer without padding can be staged straight from the caller's input when no channel block
    // straddles two phases (the virtual channels are ordered phase by phase, phase_cg real channels each)
    t.phase_cg = (phase_cg > 0 && flat && phase_cg % t.p.cb == 0) ? phase_cg : 0;
    if (t.p.splits > t.nblk) return SCONV_ERR_PLAN;
    // every part takes ceil(nblk / splits) blocks; fewer parts if the last ones would be empty
    t.p.splits = ceil_div(t.nblk, ceil_div(t.nblk, t.p.splits));
    t.rg = p.waves / p.cg;
    const int kt = t.rg * p.rows_w;
    t.nkt = ceil_div(g.Kg, kt);
    t.wave_slots = d.groups * t.nkt * t.rg;
    const int plane_floats = t.plane_cells * p.nt;
    t.n_slabs = ceil_div(plane_floats, 64);
    if (ceil_div(t.n_slabs, p.waves) > 4) return SCONV_ERR_PLAN; // slabs one wave stages per channel
    // LDS layout in floats: n_bufs x { [block: cb*plane_cells*nt] [zero page] }.  The zero
    // pages are cleared once per launch and never written.  A page serves three readers of the block in
    // front of it: the right padding of the very last row (pad*nt floats past the block), lanes past the
    // last valid position (their results are dropped), and the padding entries of the nonzero stream,
    // whose offset is the page's start, so that they multiply 0 by 0 for every lane and chunk: the page
    // has one cell more than the farthest cell a lane's chunk can start on (flat lanes: cg*t*64 cells;
    // strips: last row of the band, last column of the last strip).
    const int64_t block = (int64_t)t.p.cb * plane_floats;
    t.page_cells = p.strip ? (t.p.band - 1) * t.Wl + p.t * p.strip : p.cg * p.t * 64 * t.vec / p.nt;
    const int64_t page = (int64_t)t.page_cells * p.nt;
    if (page < (int64_t)d.pad * p.nt) return SCONV_ERR_PLAN;
    const int64_t stride = (block + page + 3) / 4 * 4;
    // barrier variant: two buffers; flow variant: its ring of buffers, and one counter per block behind them
    t.n_bufs = std::min(flow ? lds2_flow_bufs() : 2, t.nblk);
    const int64_t ctr_bytes = flow ? ((int64_t)t.nblk * 4 + 15) / 16 * 16 : 0;
    if (stride * t.n_bufs * 4 + ctr_bytes > 160 * 1024) return SCONV_ERR_PLAN;
    t.buf_stride_floats = (int)stride;
    t.ctr_bytes_at = flow ? (int)(stride * t.n_bufs * 4) : 0;
    t.lds_bytes = (int)(stride * t.n_bufs * 4 + ctr_bytes);
    t.zero_page = (unsigned)(block * 4);
    return SCONV_OK;
}

// Supported accumulator shapes; must match the instantiations in sconv_kernels.hip.
static const int kShapesV4[][2] = {{1, 8}, {2, 4}, {2, 8}, {3, 4}, {3, 6}, {3, 8}, {4, 4}, {4, 6}, {5, 4},
                                   {6, 2}, {6, 3}, {7, 2}, {7, 3}, {13, 1}, {14, 1}};
// read-ahead depth (stream entries in flight) of each shape above, as generated by gen_lds_loops.py
static const int kDepthV4[] = {4, 4, 2, 4, 2, 1, 2, 1, 1, 2, 1, 2, 1, 1, 1};

static int shape_depth(int vec, int t, int rows_w)
{
    if (vec != 4) return 1;
    for (size_t i = 0; i < sizeof(kDepthV4) / sizeof(kDepthV4[0]); ++i)
        if (kShapesV4[i][0] == t && kShapesV4[i][1] == rows_w) return kDepthV4[i];
    return 1;
}
static const int kShapesV1[][2] = {{1, 16}, {2, 16}, {3, 8}, {3, 16}, {4, 8}, {7, 8}, {13, 4}, {14, 4}};

bool lds_kernel_available(int vec, int t, int rows_w)
{
    if (vec == 4) {
        for (auto &s : kShapesV4)
            if (s[0] == t && s[1] == rows_w) return true;
    } else if (vec == 1) {
        for (auto &s : kShapesV1)
            if (s[0] == t && s[1] == rows_w) return true;
    }
    return false;
}

// Rough cost of a tiling in CU clocks; only used to rank candidates.
static double tiling_cost(const sconv_desc &d, const LdsTiling &t, int N, double avg_row_nnz)
{
    const Geometry g = geometry(d);
    const int n_tiles = ceil_div(N, t.p.nt);
    const double wgs = (double)n_tiles * d.groups * t.nkt * t.n_bands;
    const int by_lds = std::max(1, (160 * 1024) / (t.lds_bytes + 512));
    const int by_waves = std::max(1, 16 / t.p.waves);
    const int wpc = std::min(by_lds, by_waves);
    const double rows_per_wave = (double)g.Kg / (t.nkt * t.rg); // after dealing rows evenly
    // per-row streams: every (row, block) segment is padded to whole chunks of 4, 1.5 entries on average;
    // flat streams: every (wave, block) segment is padded to whole chunks of 8, 3.5 entries on average
    const bool flat = t.p.kernel == 3;
    const double seg_len = std::max(0.25, (flat ? rows_per_wave : 1.0) * avg_row_nnz / t.nblk);
    const double nnz_wave = rows_per_wave * avg_row_nnz * (seg_len + (flat ? 3.5 : 1.5)) / seg_len;
    const double fma_instr = t.p.t * t.vec;
    // SIMD-issue bound: waves on a SIMD run one after another; 4 clocks per wave instruction.
    // a shallow read-ahead ring leaves the wave waiting on LDS latency more often
    const double ring = 1.0 + 2.0 / (shape_depth(t.vec, t.p.t, t.p.rows_w) * t.p.t);
    const double simd = std::ceil(t.p.waves / 4.0) * nnz_wave * 4.0 * (fma_instr + 2.0) * ring;
    // LDS bound: clocks per wave read instruction.
    const double lds = t.p.waves * nnz_wave * t.p.t * (t.vec == 4 ? 4.3 : 2.4);
    // per segment fixed costs (pointer fetch, loop set-up, scalar latency), per wave, partly hidden
    const double seg = (double)t.nblk * (flat ? 4.0 : t.p.rows_w) * 60.0 * std::ceil(t.p.waves / 4.0);
    // loads stream in behind the multiply-adds; only the first block's load is exposed
    const double stage = (double)t.p.cb * t.plane_cells * t.p.nt * 4.0 / 32.0 + 3000.0 + t.nblk * 300.0;
    // fewer than four waves per SIMD hide each other's stalls less well
    const double occ = std::sqrt(16.0 / std::min(16, t.p.waves * wpc));
    const double wg = std::max(simd, lds) * occ + seg + stage;
    const double rounds = std::ceil(wgs / (256.0 * wpc));
    return rounds * wpc * wg;
}

// The same for the flat-stream kernel, in microseconds at 2.4 GHz; constants fitted to measured plan sweeps
// of the AlexNet layers at batch 256 (useful issue efficiency of the multiply-add loop, cost of a channel
// block's barrier and pipeline refill, cost of a workgroup's prologue and stores).
// wide: the layer's input is staged a cell per lane and its output stored four images at a time (feature-major
// activations): a block lands sooner and the stores of a workgroup take a fraction of the time.
static const double kWideFixed = 0.7;
static double tiling_cost_flat(const sconv_desc &d, const LdsTiling &t, int N, double avg_row_nnz, bool wide)
{
    const Geometry g = geometry(d);
    const int splits = std::max(1, t.p.splits);
    const int blocks = ceil_div(t.nblk, splits);              // channel blocks one workgroup walks
    const double wgs = (double)ceil_div(N, 4) * d.groups * t.nkt * t.n_bands * splits;
    const int by_lds = std::max(1, (160 * 1024) / (t.lds_bytes + 512));
    const int wpc = std::max(1, std::min(by_lds, 16 / t.p.waves));
    const double rows_wave = (double)g.Kg / (t.nkt * t.rg);
    const double entries = rows_wave * avg_row_nnz / splits + 1.5 * blocks; // segments are padded to fours
    const double cu_wgs = std::ceil(wgs / 256.0);             // workgroups one CU has to run ...
    const double m = std::min((double)wpc, cu_wgs);           // ... m of them side by side
    const double wps = t.p.waves * m / 4.0;                   // waves per SIMD
    double eff = wps >= 4 ? 0.78 : wps >= 3 ? 0.72 : wps >= 2 ? 0.68 : 0.42;
    // a shallow read-ahead ring (8 rows of 3 chunks leave registers for one entry ahead only) costs little: measured
    // on the 27x27 layer, 8 rows per wave beat 6 by 5 % in either variant, the longer streams outweighing it
    if (lds2_depth(t.p.t, t.p.rows_w) * t.p.t < 6) eff *= 0.99;
    const double simd_clk = t.p.waves * entries * (4.0 * t.p.t + 1.7); // VALU clocks per SIMD, one workgroup
    // per channel block: the barrier and the refill of the read pipeline, which a second workgroup on the CU
    // fills, and what the staging of the block (L2 to LDS, every workgroup its own copy) takes from the loop;
    // per workgroup: prologue and stores, partly filled by a second workgroup as well
    const double block_bytes = (double)t.p.cb * t.plane_cells * 16.0;
    // The flow variant pays no barrier: measured against the barrier variant on the same layers it gains about
    // 1000 clocks per block of the barrier variant (0.4-0.7 us per block on the 13x13 layers at any density)
    // and loses what its smaller blocks cost in padding.  Either variant issues the loads of the next block
    // when a block starts and cannot start that block before they have landed: a block lasts at least the
    // landing time, which binds at low density (measured: 3.3 us for 50 KB, 4.5 us for 74 KB per CU).
    const bool flow = t.p.kernel == 4;
    const double sync = flow ? 100.0 : 800.0 / m;
    // (a cell per lane: 0.7 us for the first bytes of a block, then 37 bytes per clock and CU)
    const double landing = wide ? 1700.0 + m * block_bytes / 37.0 : 4000.0 + m * block_bytes / 11.0;
    const double compute_block = m * simd_clk / eff / blocks;
    const double per_block = std::max(compute_block + sync + m * block_bytes / 120.0, landing);
    double group = blocks * per_block + (m >= 2 ? (t.p.waves >= 8 ? 8000.0 : 10500.0) : 14000.0) * (wide ? kWideFixed : 1.0);
    // Measured: the flow variant is the slower one (3-12 %) where a second workgroup on the CU already fills
    // the barrier's gaps and the blocks are only a few channels deep, where a block's arithmetic does not outlast its loads by a margin (its loads have
    // only the first chunks of a block to land in), and where there are too few blocks to rotate buffers.
    if (flow && ((m >= 2 && t.p.cb < 8) || blocks < 3 || compute_block < 1.5 * landing)) group *= 1.1;
    // (measured on the fully connected layers: with 16 waves 5-7 % behind the barrier variant and its larger blocks,
    // with 8 waves up to 10 % ahead)
    else if (flow && wide && t.p.waves >= 16) group *= 1.12;
    if (t.p.t >= 7) group /= 0.88;                            // shapes short of address registers
    double us = std::ceil(cu_wgs / m) * group / 2400.0;
    if (splits > 1) {
        // every part stores its partial results and a launch of its own adds them up
        const double out_bytes = 4.0 * N * d.K * g.OH * g.OW;
        us += 4.0 + splits * (out_bytes / (wide ? 6.0e6 : 3.5e6) + 0.3); // the reduction reads every part: bandwidth, and latency per part
    }
    return us;
}

static int search_lds_tilings(const sconv_desc &d, const sconv_plan &req, int N_hint, double avg_row_nnz, LdsTiling &out,
                              std::vector<std::pair<double, LdsTiling>> *all, int phase_cg = 0, bool wide = false);
// whether the library, left to itself, considers the flow variant of the flat-stream kernel
static const bool kFlowByDefault = true;

int make_lds_tiling(const sconv_desc &d, const sconv_plan &req, int N_hint, double avg_row_nnz, LdsTiling &out, int phase_cg, bool wide)
{
    return search_lds_tilings(d, req, N_hint, avg_row_nnz, out, nullptr, phase_cg, wide);
}

static bool same_tiling(const sconv_plan &a, const sconv_plan &b)
{
    return a.kernel == b.kernel && a.nt == b.nt && a.cb == b.cb && a.waves == b.waves && a.cg == b.cg &&
           a.rows_w == b.rows_w && a.t == b.t && a.band == b.band && a.strip == b.strip && a.splits == b.splits;
}

int rank_lds_tilings(const sconv_desc &d, const sconv_plan &req, int N_hint, double avg_row_nnz, int max_out,
                     std::vector<LdsTiling> &out, int phase_cg, bool wide)
{
    std::vector<std::pair<double, LdsTiling>> all;
    LdsTiling best;
    const int rc = search_lds_tilings(d, req, N_hint, avg_row_nnz, best, &all, phase_cg, wide);
    if (rc) return rc;
    std::stable_sort(all.begin(), all.end(), [](const std::pair<double, LdsTiling> &a, const std::pair<double, LdsTiling> &b) {
        return a.first < b.first;
    });
    out.clear();
    for (const auto &c : all) {
        if ((int)out.size() >= max_out) break;
        bool seen = false;
        for (const auto &o : out) seen = seen || same_tiling(o.p, c.second.p);
        if (!seen) out.push_back(c.second);
    }
    return out.empty() ? SCONV_ERR_PLAN : SCONV_OK;
}

static int search_lds_tilings(const sconv_desc &d, const sconv_plan &req, int N_hint, double avg_row_nnz, LdsTiling &out,
                              std::vector<std::pair<double, LdsTiling>> *all, int phase_cg, bool wide)
{
    const Geometry g = geometry(d);
    if (d.stride != 1) return SCONV_ERR_PLAN;
    const bool full = req.nt && req.cb && req.waves && req.cg && req.rows_w && req.t;
    if (full) {
        const int rc = fill_tiling(d, req, out, phase_cg);
        if (!rc && all) all->emplace_back(0.0, out);
        return rc;
    }
    if (req.strip && req.kernel && !is_flat_kernel(req.kernel)) return SCONV_ERR_PLAN;
    const int kinds[3] = {4, 3, 1};

    double best = -1;
    const int nts_big[] = {4, 8, 16}; // 8 and 16 only on request
    const int nts_small[] = {1, 2};
    const int *nts = N_hint >= 4 ? nts_big : nts_small;
    const int n_nts = N_hint >= 4 ? 3 : 2;
    // every (waves, rows_w, cb) for one choice of image tile, band, column group, chunk count and lane layout
    auto try_shapes = [&](int nt, int vec, int band, int cg, int T, int strip) {
        const int Wl = lds_pitch(d, strip);
        for (int waves : {4, 8, 16}) {
            if (req.waves && req.waves != waves) continue;
            if (waves % cg) continue;
            for (int ki = 0; ki < 3; ++ki)
            for (int rows_w = 1; rows_w <= 24; ++rows_w) {
                const int kind = kinds[ki];
                const bool flat = is_flat_kernel(kind);
                if (req.kernel && req.kernel != kind) continue;
                if (strip && !flat) continue;
                // left to itself the library uses flat streams for tiles of 4 images and per-row
                // streams only for the small-batch tiles the flat kernel does not cover
                if (!req.kernel && flat != (nt == 4)) continue;
                if (!req.kernel && kind == 4 && !kFlowByDefault) continue;
                if (flat ? (nt != 4 || !lds2_kernel_available(T, rows_w, strip ? strip : 64))
                         : !lds_kernel_available(vec, T, rows_w))
                    continue;
                if (req.rows_w && req.rows_w != rows_w) continue;
                for (int wpc_target : {1, 2, 4}) {
                    if (waves * wpc_target > 16) continue;
                    const int budget = 160 * 1024 / wpc_target - 256;
                    const int64_t per_ch = (int64_t)(band + d.R - 1) * Wl * nt * 4;
                    const int64_t page_cells = strip ? (band - 1) * Wl + T * strip : cg * T * 64 * vec / nt;
                    const int64_t fixed = page_cells * nt * 4 + 16;
                    int cb = g.Cg; // one block, one buffer, if it fits; else two buffers (flow: three)
                    if (fixed + per_ch * cb > budget) {
                        cb = (int)((budget / 2 - fixed) / per_ch);
                        // flow: as many buffers as the layer has blocks, up to its ring
                        for (int nb = 3; kind == 4 && nb <= lds2_flow_bufs() && (cb < 1 || ceil_div(g.Cg, cb) >= nb); ++nb)
                            cb = (int)(((budget - 128) / nb - fixed) / per_ch);
                    }
                    if (req.cb) cb = req.cb;
                    if (cb < 1) continue;
                    // even out the blocks
                    if (!req.cb) cb = ceil_div(g.Cg, ceil_div(g.Cg, cb));
                    // a strided layer staged straight from the input: blocks of whole phases' channels
                    if (!req.cb && phase_cg > 0 && flat) {
                        cb = std::min(cb, phase_cg);
                        while (phase_cg % cb) --cb;
                    }
                    // channel blocks of a tile shared by several workgroups, when there are too few tiles
                    static const int split_choices[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
                    for (int sp : split_choices) {
                        if (req.splits ? sp != 1 : (sp > 1 && !flat)) continue;
                        const int splits = req.splits ? req.splits : sp;
                        sconv_plan p = {kind, nt, cb, waves, cg, rows_w, T, band, strip, splits};
                        LdsTiling t;
                        if (fill_tiling(d, p, t, phase_cg) != SCONV_OK) continue;
                        if (!req.splits && t.p.splits != sp) continue; // the same as a smaller choice
                        const double c = flat ? tiling_cost_flat(d, t, N_hint, avg_row_nnz, wide)
                                                   : tiling_cost(d, t, N_hint, avg_row_nnz);
                        if (all) all->emplace_back(c, t);
                        if (best < 0 || c < best) {
                            best = c;
                            out = t;
                        }
                    }
                }
            }
        }
    };

    for (int a = 0; a < n_nts; ++a) {
        const int nt = nts[a];
        if (req.nt && req.nt != nt) continue;
        if (!req.nt && nt > 4) continue;
        if (nt > 1 && nt > N_hint) continue;
        const int vec = nt % 4 == 0 ? 4 : 1;
        int last_band = 0;
        for (int nb = 1; nb <= 8 && nb <= g.OH && !req.strip; ++nb) {
            const int band = req.band ? req.band : ceil_div(g.OH, nb);
            if (band == last_band) continue; // same band height as the previous count
            last_band = band;
            const int pos_span = (band - 1) * lds_pitch(d) + g.OW;
            const int n_chunks = ceil_div(pos_span, 64 * vec / nt);
            for (int cg = 1; cg <= 4; ++cg) {
                if (req.cg && req.cg != cg) continue;
                const int T = ceil_div(n_chunks, cg);
                if (req.t && req.t != T) continue;
                if (!req.cg && (cg - 1) * T >= n_chunks) continue; // a wave of the column group without positions
                try_shapes(nt, vec, band, cg, T, 0);
            }
            if (req.band) break;
        }
        // strips: t blocks of (64 / strip) rows x strip columns side by side, cg such rows of blocks
        if (nt != 4) continue;
        for (int strip : {7, 8, 9}) {
            if (req.strip && req.strip != strip) continue;
            const int T = ceil_div(g.OW, strip), bh = 64 / strip;
            if (req.t && req.t != T) continue;
            for (int cg = 1; cg <= 4; ++cg) {
                if (req.cg && req.cg != cg) continue;
                const int nb = ceil_div(g.OH, cg * bh);
                const int band = req.band ? req.band : ceil_div(g.OH, nb);
                if (band > cg * bh) continue;
                try_shapes(nt, vec, band, cg, T, strip);
            }
        }
    }
    return best < 0 ? SCONV_ERR_PLAN : SCONV_OK;
}

// ------------------------------------------------------------------ packing

// Rows of one group are dealt to the group's wave slots in descending order of their nonzero count,
// boustrophedon, so that every wave (which owns rows_w rows for the whole kernel) gets about the same
// number of nonzeros even when the row lengths are skewed; empty rows are dealt like any other row
// and simply produce empty segments.
int pack_lds(const sconv_desc &d, const Canonical &c, const LdsTiling &t, PackedLds &out)
{
    const Geometry g = geometry(d);
    const int rows_w = t.p.rows_w, cb = t.p.cb, nt = t.p.nt;
    const int waves_per_group = t.nkt * t.rg;
    out.t = t;
    out.row_of.assign((size_t)t.wave_slots * rows_w, -1);
    for (int grp = 0; grp < d.groups; ++grp) {
        std::vector<int> rows(g.Kg);
        std::iota(rows.begin(), rows.end(), grp * g.Kg);
        std::stable_sort(rows.begin(), rows.end(), [&](int a, int b) {
            return c.rowptr[a + 1] - c.rowptr[a] > c.rowptr[b + 1] - c.rowptr[b];
        });
        for (int i = 0; i < g.Kg; ++i) {
            const int round = i / waves_per_group, posn = i % waves_per_group;
            const int w = (round & 1) ? waves_per_group - 1 - posn : posn;
            if (round >= rows_w) return SCONV_ERR_PLAN; // cannot happen: nkt*rg*rows_w >= Kg
            out.row_of[((size_t)grp * waves_per_group + w) * rows_w + round] = rows[i];
        }
    }
    out.seg_ptr.assign((size_t)t.wave_slots * t.nblk * (rows_w + 1), 0);
    out.pairs.clear();
    out.pairs.reserve(c.val.size() + c.val.size() / 4);
    size_t real = 0;
    for (int ws = 0; ws < t.wave_slots; ++ws) {
        for (int b = 0; b < t.nblk; ++b) {
            int32_t *sp = &out.seg_ptr[((size_t)ws * t.nblk + b) * (rows_w + 1)];
            for (int i = 0; i < rows_w; ++i) {
                sp[i] = (int32_t)out.pairs.size();
                const int k = out.row_of[(size_t)ws * rows_w + i];
                if (k < 0) continue;
                const int grp = k / g.Kg;
                for (int j = c.rowptr[k]; j < c.rowptr[k + 1]; ++j) {
                    // canonical offset -> (absolute channel, r, s)
                    const int off = c.off[j];
                    const int s = off % g.Wp, r = (off / g.Wp) % g.Hp, ca = off / (g.Wp * g.Hp);
                    const int cl = ca - grp * g.Cg - b * cb;
                    if (cl < 0 || cl >= cb) continue;
                    const uint32_t byte_off = (uint32_t)(((int64_t)cl * t.plane_cells + r * t.Wl + s) * nt * 4);
                    uint32_t vb;
                    std::memcpy(&vb, &c.val[j], 4);
                    out.pairs.push_back((uint64_t)vb | ((uint64_t)byte_off << 32));
                    ++real;
                }
                // pad the segment to whole groups: value +0.0 at the all-zero page
                while ((out.pairs.size() - (size_t)sp[i]) % SCONV_PAIR_GROUP) out.pairs.push_back((uint64_t)t.zero_page << 32);
            }
            sp[rows_w] = (int32_t)out.pairs.size();
        }
    }
    if (real != c.val.size()) return SCONV_ERR_PLAN;
    // the kernel prefetches up to three chunks past the stream it is working on
    for (int i = 0; i < 3 * SCONV_PAIR_GROUP; ++i) out.pairs.push_back((uint64_t)t.zero_page << 32);
    return SCONV_OK;
}

// Rows of one group dealt to the group's wave slots for the flat-stream kernel.  Every wave of a workgroup
// meets the others at a barrier after each channel block, so what has to be even is the number of nonzeros a
// slot holds in EACH block, not only its total.  Greedy: rows in descending order of their nonzero count,
// each to the slot (with a free row) whose fullest block stays smallest, ties to the smaller total.  Rows
// without nonzeros are dealt like any other and fill what is left.
static int deal_rows(const sconv_desc &d, const Canonical &c, const LdsTiling &t, std::vector<int32_t> &row_of)
{
    const Geometry g = geometry(d);
    const int rows_w = t.p.rows_w, nblk = t.nblk, cb = t.p.cb;
    const int slots = t.nkt * t.rg;
    row_of.assign((size_t)t.wave_slots * rows_w, -1);
    std::vector<int> per_blk((size_t)g.Kg * nblk);
    std::vector<int64_t> load((size_t)slots * nblk), total(slots);
    std::vector<int> used(slots);
    for (int grp = 0; grp < d.groups; ++grp) {
        std::fill(per_blk.begin(), per_blk.end(), 0);
        for (int i = 0; i < g.Kg; ++i) {
            const int k = grp * g.Kg + i;
            for (int j = c.rowptr[k]; j < c.rowptr[k + 1]; ++j) {
                const int ca = c.off[j] / (g.Wp * g.Hp);
                per_blk[(size_t)i * nblk + (ca - grp * g.Cg) / cb]++;
            }
        }
        std::vector<int> rows(g.Kg);
        std::iota(rows.begin(), rows.end(), 0);
        std::stable_sort(rows.begin(), rows.end(), [&](int a, int b) {
            const int ka = grp * g.Kg + a, kb = grp * g.Kg + b;
            return c.rowptr[ka + 1] - c.rowptr[ka] > c.rowptr[kb + 1] - c.rowptr[kb];
        });
        std::fill(load.begin(), load.end(), 0);
        std::fill(total.begin(), total.end(), 0);
        std::fill(used.begin(), used.end(), 0);
        for (int i : rows) {
            const int *r = &per_blk[(size_t)i * nblk];
            int best = -1;
            int64_t best_max = 0, best_tot = 0;
            for (int s2 = 0; s2 < slots; ++s2) {
                if (used[s2] >= rows_w) continue;
                int64_t mx = 0;
                for (int b = 0; b < nblk; ++b) mx = std::max(mx, load[(size_t)s2 * nblk + b] + r[b]);
                if (best < 0 || mx < best_max || (mx == best_max && total[s2] < best_tot)) {
                    best = s2;
                    best_max = mx;
                    best_tot = total[s2];
                }
            }
            if (best < 0) return SCONV_ERR_PLAN; // cannot happen: slots * rows_w >= Kg
            for (int b = 0; b < nblk; ++b) {
                load[(size_t)best * nblk + b] += r[b];
                total[best] += r[b];
            }
            row_of[((size_t)grp * slots + best) * rows_w + used[best]++] = grp * g.Kg + i;
        }
    }
    return SCONV_OK;
}

int pack_flat(const sconv_desc &d, const Canonical &c, const LdsTiling &t, PackedFlat &out)
{
    const Geometry g = geometry(d);
    const int rows_w = t.p.rows_w, cb = t.p.cb;
    if (t.p.nt != 4 || rows_w * t.p.t * 4 > 256 || t.zero_page >= (1u << 20) || t.zero_page % 16) return SCONV_ERR_PLAN;
    out.t = t;
    int rc = deal_rows(d, c, t, out.row_of);
    if (rc) return rc;
    out.seg.assign((size_t)t.wave_slots * t.nblk * 2 + 2, 0); // one spare entry: the kernel looks one block ahead
    out.pairs.clear();
    out.pairs.reserve(c.val.size() + (size_t)t.wave_slots * t.nblk * 4);
    const uint64_t pad_entry = (uint64_t)((t.zero_page / 16) << 16) << 32;
    size_t real = 0;
    // nonzeros of a row by block: walk each row once per slot, bucketing by channel block
    std::vector<std::vector<uint64_t>> bucket(t.nblk);
    for (int ws = 0; ws < t.wave_slots; ++ws) {
        for (auto &b : bucket) b.clear();
        for (int i = 0; i < rows_w; ++i) {
            const int k = out.row_of[(size_t)ws * rows_w + i];
            if (k < 0) continue;
            const int grp = k / g.Kg;
            for (int j = c.rowptr[k]; j < c.rowptr[k + 1]; ++j) {
                const int off = c.off[j];
                const int s = off % g.Wp, r = (off / g.Wp) % g.Hp, ca = off / (g.Wp * g.Hp);
                const int cl_all = ca - grp * g.Cg;
                const int b = cl_all / cb, cl = cl_all - b * cb;
                const uint32_t byte_off = (uint32_t)(((int64_t)cl * t.plane_cells + r * t.Wl + s) * 16);
                if (byte_off >= t.zero_page) return SCONV_ERR_PLAN;
                uint32_t vb;
                std::memcpy(&vb, &c.val[j], 4);
                bucket[b].push_back((uint64_t)vb | ((uint64_t)(((byte_off / 16) << 16) | (uint32_t)(i * t.p.t * 4)) << 32));
                ++real;
            }
        }
        for (int b = 0; b < t.nblk; ++b) {
            // entries in ascending LDS offset: rows that share a column sit next to each other
            std::stable_sort(bucket[b].begin(), bucket[b].end(), [](uint64_t x, uint64_t y) { return (x >> 48) < (y >> 48); });
            // The segment in whole chunks of 8 entries.  Its length is first rounded up to a multiple of 4; an
            // odd number of fours puts the first four into a chunk of their own, whose other four entries the
            // kernel never executes (flag in bit 31 of the chunk count), so that at most 3 entries of a
            // segment are idle instead of 7.
            const size_t start = out.pairs.size();
            const size_t len = bucket[b].size(), fours = (len + 3) / 4;
            const bool half = fours % 2 == 1;
            size_t taken = 0;
            if (half) {
                for (; taken < 4 && taken < len; ++taken) out.pairs.push_back(bucket[b][taken]);
                while ((out.pairs.size() - start) % SCONV_FLAT_CHUNK) out.pairs.push_back(pad_entry);
            }
            out.pairs.insert(out.pairs.end(), bucket[b].begin() + (long)taken, bucket[b].end());
            while ((out.pairs.size() - start) % SCONV_FLAT_CHUNK) out.pairs.push_back(pad_entry);
            if (start * 8 >= ((uint64_t)1 << 32)) return SCONV_ERR_RANGE;
            const size_t chunks = (out.pairs.size() - start) / SCONV_FLAT_CHUNK;
            if (chunks >= ((size_t)1 << 24)) return SCONV_ERR_RANGE;
            out.seg[((size_t)ws * t.nblk + b) * 2] = (uint32_t)(start * 8);
            out.seg[((size_t)ws * t.nblk + b) * 2 + 1] = (uint32_t)chunks | (half ? 0x80000000u : 0u);
        }
    }
    if (real != c.val.size()) return SCONV_ERR_PLAN;
    // the kernel loads two chunks past the segment it is working on, and warms L2 with what follows those
    for (int i = 0; i < 3 * SCONV_FLAT_CHUNK + SCONV_FLAT_WARM_BYTES / 8; ++i) out.pairs.push_back(pad_entry);
    // store offsets of the positions a group of cg waves covers
    const int npos = t.p.cg * t.p.t * 64;
    out.store_tbl.assign(npos, -1);
    for (int pos = 0; pos < npos; ++pos) {
        int by = pos / t.Wl, ox = pos % t.Wl;
        if (t.p.strip) { // [wave of the column group][chunk = strip][lane = row * strip + column]
            const int cgi = pos / (t.p.t * 64), ch = pos / 64 % t.p.t, lane = pos % 64;
            const int br = lane / t.p.strip;
            by = br < t.strip_rows ? cgi * t.strip_rows + br : t.p.band;
            ox = ch * t.p.strip + lane % t.p.strip;
        }
        if (by < t.p.band && ox < g.OW) out.store_tbl[pos] = (by * g.OW + ox) * 4 * t.out_pos;
    }
    return SCONV_OK;
}

static void sort_rows_by_offset(const sconv_desc &d, std::vector<std::vector<std::pair<int32_t, float>>> &rows,
                                Canonical &out)
{
    out.rowptr.assign(d.K + 1, 0);
    out.off.clear();
    out.val.clear();
    out.colidx.clear();
    for (int k = 0; k < d.K; ++k) {
        auto &r = rows[k];
        std::stable_sort(r.begin(), r.end(), [](const std::pair<int32_t, float> &a, const std::pair<int32_t, float> &b) {
            return a.first < b.first;
        });
        for (auto &e : r) {
            out.off.push_back(e.first);
            out.val.push_back(e.second);
        }
        out.rowptr[k + 1] = (int32_t)out.off.size();
    }
}

int unpack_lds(const sconv_desc &d, const PackedLds &p, Canonical &out)
{
    const Geometry g = geometry(d);
    const LdsTiling &t = p.t;
    const int rows_w = t.p.rows_w;
    std::vector<std::vector<std::pair<int32_t, float>>> rows(d.K);
    for (int ws = 0; ws < t.wave_slots; ++ws) {
        for (int b = 0; b < t.nblk; ++b) {
            const int32_t *sp = &p.seg_ptr[((size_t)ws * t.nblk + b) * (rows_w + 1)];
            for (int i = 0; i < rows_w; ++i) {
                const int k = p.row_of[(size_t)ws * rows_w + i];
                if (k < 0) {
                    if (sp[i + 1] != sp[i]) return SCONV_ERR_CSR;
                    continue;
                }
                const int grp = k / g.Kg;
                for (int j = sp[i]; j < sp[i + 1]; ++j) {
                    const uint32_t vb = (uint32_t)(p.pairs[j] & 0xffffffffu);
                    const uint32_t byte_off = (uint32_t)(p.pairs[j] >> 32);
                    if (byte_off >= t.zero_page) continue; // group padding
                    const int cell = (int)(byte_off / (4u * t.p.nt));
                    const int cl = cell / t.plane_cells, rem = cell % t.plane_cells;
                    const int r = rem / t.Wl, s = rem % t.Wl;
                    const int ca = grp * g.Cg + b * t.p.cb + cl;
                    float v;
                    std::memcpy(&v, &vb, 4);
                    rows[k].push_back({((ca * g.Hp) + r) * g.Wp + s, v});
                }
            }
        }
    }
    sort_rows_by_offset(d, rows, out);
    return SCONV_OK;
}

int unpack_flat(const sconv_desc &d, const PackedFlat &p, Canonical &out)
{
    const Geometry g = geometry(d);
    const LdsTiling &t = p.t;
    const int rows_w = t.p.rows_w;
    std::vector<std::vector<std::pair<int32_t, float>>> rows(d.K);
    for (int ws = 0; ws < t.wave_slots; ++ws) {
        for (int b = 0; b < t.nblk; ++b) {
            const size_t start = p.seg[((size_t)ws * t.nblk + b) * 2] / 8;
            const size_t n = (size_t)(p.seg[((size_t)ws * t.nblk + b) * 2 + 1] & 0x7fffffffu) * SCONV_FLAT_CHUNK;
            for (size_t j = start; j < start + n; ++j) {
                const uint32_t vb = (uint32_t)(p.pairs[j] & 0xffffffffu);
                const uint32_t w1 = (uint32_t)(p.pairs[j] >> 32);
                const uint32_t byte_off = (w1 >> 16) * 16;
                if (byte_off >= t.zero_page) continue; // chunk padding
                const int i = (int)(w1 & 0xffffu) / (t.p.t * 4);
                if (i >= rows_w) return SCONV_ERR_CSR;
                const int k = p.row_of[(size_t)ws * rows_w + i];
                if (k < 0) return SCONV_ERR_CSR;
                const int grp = k / g.Kg;
                const int cell = (int)(byte_off / 16u);
                const int cl = cell / t.plane_cells, rem = cell % t.plane_cells;
                const int r = rem / t.Wl, sx = rem % t.Wl;
                const int ca = grp * g.Cg + b * t.p.cb + cl;
                float v;
                std::memcpy(&v, &vb, 4);
                rows[k].push_back({((ca * g.Hp) + r) * g.Wp + sx, v});
            }
        }
    }
    sort_rows_by_offset(d, rows, out);
    return SCONV_OK;
}

// ------------------------------------------------------------------ strided layers as phase images

void phase_desc(const sconv_desc &d, sconv_desc &v)
{
    const Geometry g = geometry(d);
    const int s = d.stride;
    v = d;
    v.C = d.C * s * s;
    v.R = ceil_div(d.R, s);
    v.S = ceil_div(d.S, s);
    v.H = g.OH + v.R - 1;
    v.W = g.OW + v.S - 1;
    v.stride = 1;
    v.pad = 0;
}

int phase_canonical(const sconv_desc &d, const Canonical &c, Canonical &vc)
{
    const Geometry g = geometry(d);
    sconv_desc v;
    phase_desc(d, v);
    const Geometry gv = geometry(v);
    const int s = d.stride;
    std::vector<std::vector<std::pair<int32_t, float>>> rows(d.K);
    for (int k = 0; k < d.K; ++k) {
        const int grp = k / g.Kg;
        for (int j = c.rowptr[k]; j < c.rowptr[k + 1]; ++j) {
            const int off = c.off[j];
            const int t = off % g.Wp, r = (off / g.Wp) % g.Hp, ca = off / (g.Wp * g.Hp);
            const int cl = ca - grp * g.Cg;
            const int va = grp * gv.Cg + ((r % s) * s + t % s) * g.Cg + cl; // phase by phase, the group's channels inside
            rows[k].push_back({(va * gv.Hp + r / s) * gv.Wp + t / s, c.val[j]});
        }
    }
    sort_rows_by_offset(v, rows, vc);
    // colidx of the virtual layer, for completeness: (v_local*R' + r')*S' + t'
    vc.colidx.resize(vc.off.size());
    for (int k = 0; k < d.K; ++k) {
        const int grp = k / g.Kg;
        for (int j = vc.rowptr[k]; j < vc.rowptr[k + 1]; ++j) {
            const int off = vc.off[j];
            const int t = off % gv.Wp, r = (off / gv.Wp) % gv.Hp, va = off / (gv.Wp * gv.Hp);
            vc.colidx[j] = ((va - grp * gv.Cg) * v.R + r) * v.S + t;
        }
    }
    return SCONV_OK;
}

int unphase_canonical(const sconv_desc &d, const Canonical &vc, Canonical &out)
{
    const Geometry g = geometry(d);
    sconv_desc v;
    phase_desc(d, v);
    const Geometry gv = geometry(v);
    const int s = d.stride;
    std::vector<std::vector<std::pair<int32_t, float>>> rows(d.K);
    for (int k = 0; k < d.K; ++k) {
        const int grp = k / g.Kg;
        for (int j = vc.rowptr[k]; j < vc.rowptr[k + 1]; ++j) {
            const int off = vc.off[j];
            const int t2 = off % gv.Wp, r2 = (off / gv.Wp) % gv.Hp, va = off / (gv.Wp * gv.Hp);
            const int vl = va - grp * gv.Cg;
            const int cl = vl % g.Cg, px = (vl / g.Cg) % s, py = vl / (g.Cg * s);
            const int r = r2 * s + py, t = t2 * s + px;
            if (r >= d.R || t >= d.S) return SCONV_ERR_CSR;
            rows[k].push_back({((grp * g.Cg + cl) * g.Hp + r) * g.Wp + t, vc.val[j]});
        }
    }
    sort_rows_by_offset(d, rows, out);
    return SCONV_OK;
}

// Direct kernel: per nonzero the value, the offset of (c, r-pad, s-pad) in the UNPADDED image
// (may be negative), and (r-pad, s-pad) for the bounds test that stands in for the zero padding.
int pack_direct(const sconv_desc &d, const Canonical &c, PackedDirect &out)
{
    const Geometry g = geometry(d);
    out.rowptr = c.rowptr;
    out.trip.resize(c.val.size() * 3);
    for (size_t j = 0; j < c.val.size(); ++j) {
        const int off = c.off[j];
        const int s = off % g.Wp, r = (off / g.Wp) % g.Hp, ca = off / (g.Wp * g.Hp);
        const int dr = r - d.pad, ds = s - d.pad;
        const int32_t goff = (ca * d.H + dr) * d.W + ds;
        uint32_t vb;
        std::memcpy(&vb, &c.val[j], 4);
        out.trip[3 * j + 0] = vb;
        out.trip[3 * j + 1] = (uint32_t)goff;
        out.trip[3 * j + 2] = ((uint32_t)(dr & 0xffff) << 16) | (uint32_t)(ds & 0xffff);
    }
    return SCONV_OK;
}

int unpack_direct(const sconv_desc &d, const PackedDirect &p, Canonical &out)
{
    const Geometry g = geometry(d);
    std::vector<std::vector<std::pair<int32_t, float>>> rows(d.K);
    for (int k = 0; k < d.K; ++k) {
        for (int j = p.rowptr[k]; j < p.rowptr[k + 1]; ++j) {
            const uint32_t vb = p.trip[3 * (size_t)j];
            const int32_t goff = (int32_t)p.trip[3 * (size_t)j + 1];
            const uint32_t rs = p.trip[3 * (size_t)j + 2];
            const int dr = (int16_t)(rs >> 16), ds = (int16_t)(rs & 0xffff);
            const int ca = (goff - dr * d.W - ds) / (d.H * d.W);
            float v;
            std::memcpy(&v, &vb, 4);
            rows[k].push_back({((ca * g.Hp) + dr + d.pad) * g.Wp + ds + d.pad, v});
        }
    }
    sort_rows_by_offset(d, rows, out);
    return SCONV_OK;
}

} // namespace sconv
