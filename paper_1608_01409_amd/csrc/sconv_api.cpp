// The extern "C" surface of libsconv (see include/sconv.h) and the roofline model of Section 2.2.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <map>
#include <new>
#include <utility>
#include <vector>

#include "sconv_internal.h"

using namespace sconv;

// An earlier packing of a handle, kept with its device copies: a caller that alternates between batch sizes
// gets it back instead of packing and uploading again.
struct StashedPacking {
    bool flat = false;
    PackedLds lds;
    PackedFlat lds_flat;
    DeviceLds dev;
    bool uploaded = false;
    // fully connected packings only
    int fc_n = 0, fc_tiles = 0;
    sconv_desc fc_desc;
};
static const size_t kStashed = 3; // packings kept besides the current one

static void release_arrays(DeviceLds &dev)
{
    release(dev.pairs);
    release(dev.seg_ptr);
    release(dev.row_of);
    release(dev.store_tbl);
    dev = DeviceLds();
}

struct sconv_csr {
    sconv_desc desc;
    Canonical canon;
    sconv_plan requested;    // what the caller asked for (zeros = choose)
    bool has_lds = false;    // one of the two LDS packings below is filled
    bool flat = false;       // ... the flat-stream one
    PackedLds lds;
    PackedFlat lds_flat;
    PackedDirect direct;
    DeviceLds dev_lds;
    DeviceDirect dev_direct;
    bool lds_uploaded = false, direct_uploaded = false;
    int planned_n = 0;       // batch size the current LDS tiling was chosen for
    std::map<int, sconv_plan> plan_of_n;     // tilings already chosen, by batch size
    std::vector<StashedPacking> stash;       // earlier packings, oldest first
    // the layer the LDS kernels run: the layer itself, or for stride > 1 its stride-1 form over phase images
    bool phased = false;
    sconv_desc kdesc;
    Canonical kcanon;        // filled only when phased
    void *phase_buf = nullptr;
    size_t phase_bytes = 0;
    void *part_buf = nullptr; // partial results of launches that split the channels over workgroups
    size_t part_bytes = 0;
    const Canonical &kc() const { return phased ? kcanon : canon; }
    // real channels per phase of a group when the phase images can be picked out of the caller's input while
    // staging (a strided layer without padding), else 0
    int phase_cg() const { return (phased && desc.pad == 0) ? desc.C / desc.groups : 0; }
    // fully connected use (sconv_fc_forward): the layer as a 1x1 convolution whose positions are the batch
    int fc_n = 0;            // batch size the arrays below were packed for
    int fc_tiles = 0;        // the batch is cut into this many tiles of fc_n / fc_tiles images
    sconv_desc fc_desc;
    PackedFlat fc_flat;
    DeviceLds fc_dev;
    bool fc_uploaded = false;
    std::vector<StashedPacking> fc_stash;
    std::map<int, sconv_plan> fc_plan_of_n;  // tilings sconv_fc_tune chose, by batch size
    size_t stash_cap = kStashed;             // packings kept besides the current one (more while tuning)
    int hip_err = 0;
};

static const LdsTiling &f_tiling(const sconv_csr *h) { return h->lds_flat.t; }

// Scratch owned by the handle, grown on demand.
static int grow(void **buf, size_t *have, size_t need, int *hip_err)
{
    if (need <= *have) return SCONV_OK;
    release(*buf);
    *buf = nullptr;
    *have = 0;
    const int rc = upload(nullptr, need, buf, hip_err);
    if (rc) return rc;
    *have = need;
    return SCONV_OK;
}

// A fixed piece of device memory handed out front to back (the entry point that must not allocate).
struct Workspace {
    char *base = nullptr;
    size_t bytes = 0, used = 0;
    void *take(size_t need)
    {
        const size_t at = (used + 255) & ~(size_t)255;
        if (at + need > bytes) return nullptr;
        used = at + need;
        return base + at;
    }
};

// The flat-stream kernel and, when the tiling splits the channels, the reduction of its partial results.
// The partial results go to scratch the handle owns and grows, or into `ws` when one is given.
static int run_flat(sconv_csr *h, const sconv_desc &kd, const LdsTiling &t, const DeviceLds &dev, const Lds2Layout &lay,
                    const float *in, float *out, int n_kernel, int64_t rows, int64_t inner, const Epilogue &ep, void *stream,
                    Workspace *ws = nullptr)
{
    if (t.p.splits <= 1) return launch_lds2(kd, t, dev, lay, in, out, n_kernel, ep, 0, stream, &h->hip_err);
    const int64_t total = rows * inner;
    const size_t need = (size_t)total * t.p.splits * sizeof(float);
    int rc;
    float *parts;
    if (ws) {
        parts = static_cast<float *>(ws->take(need));
        if (!parts) return SCONV_ERR_CAPACITY;
    } else {
        rc = grow(&h->part_buf, &h->part_bytes, need, &h->hip_err);
        if (rc) return rc;
        parts = static_cast<float *>(h->part_buf);
    }
    rc = launch_lds2(kd, t, dev, lay, in, parts, n_kernel, ep, total, stream, &h->hip_err);
    if (rc) return rc;
    return launch_reduce(parts, out, t.p.splits, rows, inner, h->desc.K, ep, stream, &h->hip_err);
}

static bool same_plan(const sconv_plan &a, const sconv_plan &b)
{
    return a.kernel == b.kernel && a.nt == b.nt && a.cb == b.cb && a.waves == b.waves && a.cg == b.cg &&
           a.rows_w == b.rows_w && a.t == b.t && a.band == b.band && a.strip == b.strip && a.splits == b.splits;
}

// Choose (or re-choose) the LDS tiling for batch size n and pack for it.  The best tiling depends on the
// batch: with few image tiles smaller workgroups are needed to occupy every CU.  The handle changes only
// once the new packing exists: after an error it still holds, and runs, the packing it had.
static const size_t kPlansRemembered = 64; // batch sizes whose tiling is kept; beyond that the table starts over

static int plan_lds(sconv_csr *h, int n, bool resident_only = false)
{
    const sconv_desc &d = h->kdesc;
    const double avg = d.K ? (double)h->canon.val.size() / d.K : 0.0;
    LdsTiling t;
    int rc;
    auto known = h->plan_of_n.find(n);
    const bool fresh = known == h->plan_of_n.end();
    if (fresh && resident_only) return SCONV_ERR_PLAN; // never planned for this batch size
    rc = make_lds_tiling(d, fresh ? h->requested : known->second, n, avg, t, h->phase_cg()); // a known tiling has every field: no search
    if (rc) return rc;
    auto remember = [&]() {
        if (!fresh) return;
        if (h->plan_of_n.size() >= kPlansRemembered) h->plan_of_n.clear();
        h->plan_of_n[n] = t.p;
    };
    if (h->has_lds && same_plan(t.p, h->flat ? h->lds_flat.t.p : h->lds.t.p)) {
        remember();
        h->planned_n = n;
        return SCONV_OK;
    }
    // an earlier packing for this tiling, device copies and all?
    size_t found = h->stash.size();
    for (size_t i = 0; i < h->stash.size(); ++i) {
        const StashedPacking &sp = h->stash[i];
        if (same_plan(t.p, sp.flat ? sp.lds_flat.t.p : sp.lds.t.p)) found = i;
    }
    StashedPacking next;
    if (found < h->stash.size()) {
        if (resident_only && !h->stash[found].uploaded) return SCONV_ERR_PLAN;
        next = std::move(h->stash[found]);
        h->stash.erase(h->stash.begin() + (long)found);
    } else if (resident_only) {
        return SCONV_ERR_PLAN; // the packing for this tiling has been dropped: it would have to be built and uploaded
    } else {
        next.flat = is_flat_kernel(t.p.kernel);
        rc = next.flat ? pack_flat(d, h->kc(), t, next.lds_flat) : pack_lds(d, h->kc(), t, next.lds);
        if (rc) return rc;
    }
    if (h->has_lds) { // set the current packing aside
        StashedPacking old;
        old.flat = h->flat;
        old.lds = std::move(h->lds);
        old.lds_flat = std::move(h->lds_flat);
        old.dev = h->dev_lds;
        old.uploaded = h->lds_uploaded;
        h->stash.push_back(std::move(old));
        // (resident_only: one packing left the stash and one entered it, so nothing has to go, and nothing may:
        // hipFree is not for that caller)
        while (!resident_only && h->stash.size() > h->stash_cap) { // hipFree waits for launches that still read the arrays
            release_arrays(h->stash.front().dev);
            h->stash.erase(h->stash.begin());
        }
    }
    h->flat = next.flat;
    h->lds = std::move(next.lds);
    h->lds_flat = std::move(next.lds_flat);
    h->dev_lds = next.dev;
    h->lds_uploaded = next.uploaded;
    h->has_lds = true;
    remember();
    h->planned_n = n;
    return SCONV_OK;
}

static int finish_create(sconv_csr *h, const sconv_plan *plan)
{
    std::memset(&h->requested, 0, sizeof(h->requested));
    if (plan) h->requested = *plan;
    if (h->requested.kernel < 0 || h->requested.kernel > 4) return SCONV_ERR_PLAN;
    const sconv_desc &d = h->desc;
    int rc = pack_direct(d, h->canon, h->direct);
    if (rc) return rc;
    h->kdesc = d;
    if (d.stride > 1 && h->requested.kernel != 2) {
        // phase images; layers whose virtual form is out of range keep the direct kernel
        sconv_desc v;
        phase_desc(d, v);
        if (validate_desc(v) == SCONV_OK && phase_canonical(d, h->canon, h->kcanon) == SCONV_OK) {
            h->kdesc = v;
            h->phased = true;
        }
    }
    if (h->requested.kernel != 2 && (d.stride == 1 || h->phased)) {
        // tuned for a large batch until the first forward call says otherwise; small ones go to the direct kernel
        rc = plan_lds(h, h->requested.nt ? h->requested.nt : 256);
        if (rc != SCONV_OK && h->requested.kernel != 0) return rc;
    } else if (h->requested.kernel == 1 || is_flat_kernel(h->requested.kernel)) {
        return SCONV_ERR_PLAN;
    }
    return SCONV_OK;
}

extern "C" int sconv_create_csr(const sconv_desc *desc, const float *dense_w, const sconv_plan *plan, sconv_csr **out)
{
    if (!desc || !dense_w || !out) return SCONV_ERR_NULL;
    *out = nullptr;
    int rc = validate_desc(*desc);
    if (rc) return rc;
    sconv_csr *h = new (std::nothrow) sconv_csr();
    if (!h) return SCONV_ERR_NOMEM;
    try {
        h->desc = *desc;
        rc = build_canonical_from_dense(*desc, dense_w, h->canon);
        if (!rc) rc = finish_create(h, plan);
    } catch (const std::bad_alloc &) {
        rc = SCONV_ERR_NOMEM;
    }
    if (rc) {
        delete h;
        return rc;
    }
    *out = h;
    return SCONV_OK;
}

extern "C" int sconv_create_csr_from_arrays(const sconv_desc *desc, const int32_t *rowptr, const int32_t *colidx,
                                            const float *values, const sconv_plan *plan, sconv_csr **out)
{
    if (!desc || !rowptr || !out) return SCONV_ERR_NULL;
    *out = nullptr;
    int rc = validate_desc(*desc);
    if (rc) return rc;
    sconv_csr *h = new (std::nothrow) sconv_csr();
    if (!h) return SCONV_ERR_NOMEM;
    try {
        h->desc = *desc;
        rc = build_canonical_from_arrays(*desc, rowptr, colidx, values, h->canon);
        if (!rc) rc = finish_create(h, plan);
    } catch (const std::bad_alloc &) {
        rc = SCONV_ERR_NOMEM;
    }
    if (rc) {
        delete h;
        return rc;
    }
    *out = h;
    return SCONV_OK;
}

extern "C" int sconv_lower_offsets(const sconv_desc *desc, int32_t layout, const int32_t *rowptr, const int32_t *colidx,
                                   int32_t *off, int32_t *step_y, int32_t *step_x)
{
    if (!desc || !rowptr) return SCONV_ERR_NULL;
    int rc = validate_desc(*desc);
    if (rc) return rc;
    if (layout != SCONV_LAYOUT_CHW && layout != SCONV_LAYOUT_HWC) return SCONV_ERR_DESC;
    rc = validate_csr(*desc, rowptr, colidx);
    if (rc) return rc;
    if (rowptr[desc->K] > 0 && !off) return SCONV_ERR_NULL;
    lower_offsets(*desc, layout, rowptr, colidx, off);
    const Geometry g = geometry(*desc);
    const int per_x = layout == SCONV_LAYOUT_HWC ? desc->C : 1;
    if (step_y) *step_y = desc->stride * g.Wp * per_x;
    if (step_x) *step_x = desc->stride * per_x;
    return SCONV_OK;
}

extern "C" int sconv_csr_info(const sconv_csr *h, int64_t *nnz, int32_t *out_h, int32_t *out_w, sconv_plan *plan)
{
    if (!h) return SCONV_ERR_NULL;
    const Geometry g = geometry(h->desc);
    if (nnz) *nnz = (int64_t)h->canon.val.size();
    if (out_h) *out_h = g.OH;
    if (out_w) *out_w = g.OW;
    if (plan) {
        std::memset(plan, 0, sizeof(*plan));
        if (h->has_lds)
            *plan = h->flat ? h->lds_flat.t.p : h->lds.t.p;
        else
            plan->kernel = 2;
    }
    return SCONV_OK;
}

extern "C" int sconv_csr_balance(const sconv_csr *h, sconv_balance *out)
{
    if (!h || !out) return SCONV_ERR_NULL;
    if (!h->has_lds || !h->flat) return SCONV_ERR_PLAN;
    const PackedFlat &f = h->lds_flat;
    const LdsTiling &t = f.t;
    std::memset(out, 0, sizeof(*out));
    out->nnz = (int64_t)h->canon.val.size();
    const int n_wg = t.wave_slots / t.rg; // groups * nkt workgroups' worth of row tiles
    double wg_sum = 0, wg_max = 0;
    for (int wg = 0; wg < n_wg; ++wg) {
        double wg_total = 0;
        for (int b = 0; b < t.nblk; ++b) {
            double sum = 0, mx = 0, simd[4] = {0, 0, 0, 0};
            int on_simd[4] = {0, 0, 0, 0};
            for (int r = 0; r < t.rg; ++r) {
                const uint32_t word = f.seg[((size_t)(wg * t.rg + r) * t.nblk + b) * 2 + 1];
                const double ch = (word & 0x7fffffffu) - ((word >> 31) ? 0.5 : 0.0); // a half chunk counts as half
                out->stream_entries += (int64_t)(ch * SCONV_FLAT_CHUNK + 0.5);
                sum += ch;
                mx = std::max(mx, ch);
                // the cg waves of a row group run the same stream; wave index = r * cg + column group
                for (int c = 0; c < t.p.cg; ++c) {
                    simd[(r * t.p.cg + c) & 3] += ch;
                    on_simd[(r * t.p.cg + c) & 3]++;
                }
            }
            double smx = 0;
            for (int q = 0; q < 4; ++q)
                if (on_simd[q]) smx = std::max(smx, simd[q] / on_simd[q]);
            out->wave_mean += sum / t.rg;
            out->wave_max += mx;
            out->simd_max += smx;
            wg_total += mx;
        }
        wg_sum += wg_total;
        wg_max = std::max(wg_max, wg_total);
    }
    out->workgroup_mean = n_wg ? wg_sum / n_wg : 0;
    out->workgroup_max = wg_max;
    return SCONV_OK;
}

static int export_canonical(const sconv_desc &d, const Canonical &c, int32_t *rowptr, int32_t *off, float *values,
                            int64_t *nnz_io)
{
    if (!nnz_io) return SCONV_ERR_NULL;
    const int64_t nnz = (int64_t)c.val.size();
    const int64_t cap = *nnz_io;
    *nnz_io = nnz;
    if (cap < nnz) return SCONV_ERR_CAPACITY;
    if (!rowptr || (nnz > 0 && (!off || !values))) return SCONV_ERR_NULL;
    std::memcpy(rowptr, c.rowptr.data(), sizeof(int32_t) * (d.K + 1));
    if (nnz) {
        std::memcpy(off, c.off.data(), sizeof(int32_t) * nnz);
        std::memcpy(values, c.val.data(), sizeof(float) * nnz);
    }
    return SCONV_OK;
}

extern "C" int sconv_csr_export(const sconv_csr *h, int32_t *rowptr, int32_t *off, float *values, int64_t *nnz_io)
{
    if (!h) return SCONV_ERR_NULL;
    return export_canonical(h->desc, h->canon, rowptr, off, values, nnz_io);
}

extern "C" int sconv_csr_unpack(const sconv_csr *h, int32_t which, int32_t *rowptr, int32_t *off, float *values,
                                int64_t *nnz_io)
{
    if (!h) return SCONV_ERR_NULL;
    Canonical c;
    int rc;
    try {
        if (which == 1) {
            if (!h->has_lds) return SCONV_ERR_PLAN;
            rc = h->flat ? unpack_flat(h->kdesc, h->lds_flat, c) : unpack_lds(h->kdesc, h->lds, c);
            if (!rc && h->phased) {
                Canonical real;
                rc = unphase_canonical(h->desc, c, real);
                c = std::move(real);
            }
        } else if (which == 2) {
            rc = unpack_direct(h->desc, h->direct, c);
        } else if (which == 3) {
            // the fully connected packing: offsets are feature * (positions per tile) in the wide image
            if (h->fc_n <= 0) return SCONV_ERR_PLAN;
            rc = unpack_flat(h->fc_desc, h->fc_flat, c);
            if (!rc) {
                const int w = h->fc_desc.W;
                for (auto &o : c.off) {
                    if (o % w) return SCONV_ERR_CSR;
                    o /= w;
                }
            }
        } else {
            return SCONV_ERR_PLAN;
        }
    } catch (const std::bad_alloc &) {
        return SCONV_ERR_NOMEM;
    }
    if (rc) return rc;
    return export_canonical(h->desc, c, rowptr, off, values, nnz_io);
}

static int forward_impl(sconv_csr *h, const float *in, float *out, int32_t N, const Epilogue &ep, void *hip_stream,
                        Workspace *ws = nullptr);

extern "C" int sconv_forward(sconv_csr *h, const float *in, float *out, int32_t N, void *hip_stream)
{
    return forward_impl(h, in, out, N, Epilogue(), hip_stream);
}

extern "C" int sconv_forward_fused(sconv_csr *h, const float *in, float *out, int32_t N, const float *bias, int32_t relu,
                                   void *hip_stream)
{
    Epilogue ep;
    ep.bias = bias;
    ep.relu = relu != 0;
    return forward_impl(h, in, out, N, ep, hip_stream);
}

// ws != nullptr: the caller forbids allocation.  Scratch then comes out of ws, and everything else the launch
// needs (the tiling for N, its packing, the device copies) must already exist: SCONV_ERR_PLAN otherwise.
static int forward_impl(sconv_csr *h, const float *in, float *out, int32_t N, const Epilogue &ep, void *hip_stream,
                        Workspace *ws)
{
    if (!h || !in || !out) return SCONV_ERR_NULL;
    if (N < 1) return SCONV_ERR_BATCH;
    const Geometry og = geometry(h->desc);
    const int64_t out_rows = (int64_t)N * h->desc.K, out_inner = (int64_t)og.OH * og.OW;
    bool use_lds = h->has_lds;
    // a tiling the library chose itself follows the batch size (only when none of its fields was requested)
    const sconv_plan &rq = h->requested;
    const bool free_choice = !rq.nt && !rq.cb && !rq.waves && !rq.cg && !rq.rows_w && !rq.t && !rq.band && !rq.strip && !rq.splits;
    // (batches below 4 use the tiling of batch 4: one tile of 4 images, not all of them present)
    const int n_plan = N < 4 ? 4 : N;
    if (use_lds && free_choice && n_plan != h->planned_n) {
        try {
            const int prc = plan_lds(h, n_plan, ws != nullptr);
            if (prc) return prc;
        } catch (const std::bad_alloc &) {
            return SCONV_ERR_NOMEM;
        }
    }
    if (ws && !(use_lds && h->flat && h->lds_uploaded)) return SCONV_ERR_PLAN;
    // the per-row-stream kernel's tiles of 4 images and more are no match for the direct kernel on 1-3 images
    if (use_lds && !h->flat && h->requested.kernel == 0 && N < 4 && h->lds.t.p.nt >= 4) use_lds = false;
    int rc;
    // the flat-stream kernel stages an unpadded strided layer straight from `in` when its blocks hold whole phases
    const bool stage_phases = use_lds && h->phased && h->flat && f_tiling(h).phase_cg > 0;
    if (use_lds && h->phased && !stage_phases) {
        // re-order the input into phase images (scratch owned by the handle, grown on demand)
        const size_t need = (size_t)N * h->kdesc.C * h->kdesc.H * h->kdesc.W * sizeof(float);
        float *phase;
        if (ws) {
            phase = static_cast<float *>(ws->take(need));
            if (!phase) return SCONV_ERR_CAPACITY;
        } else {
            rc = grow(&h->phase_buf, &h->phase_bytes, need, &h->hip_err);
            if (rc) return rc;
            phase = static_cast<float *>(h->phase_buf);
        }
        rc = launch_phase(h->desc, h->kdesc, in, phase, N, hip_stream, &h->hip_err);
        if (rc) return rc;
        in = phase;
    }
    if (use_lds && h->flat) {
        if (!h->lds_uploaded) {
            const PackedFlat &f = h->lds_flat;
            rc = upload(f.pairs.data(), f.pairs.size() * 8, &h->dev_lds.pairs, &h->hip_err);
            if (!rc) rc = upload(f.seg.data(), f.seg.size() * 4, &h->dev_lds.seg_ptr, &h->hip_err);
            if (!rc) rc = upload(f.row_of.data(), f.row_of.size() * 4, &h->dev_lds.row_of, &h->hip_err);
            if (!rc) rc = upload(f.store_tbl.data(), f.store_tbl.size() * 4, &h->dev_lds.store_tbl, &h->hip_err);
            if (rc) return rc;
            h->lds_uploaded = true;
            // set-up on this device: the address of the library's static scratch is looked up now, so that
            // sconv_forward_noalloc finds it known (a failure here is that entry point's to report)
            void *base;
            size_t bytes;
            int ignored = 0;
            (void)static_scratch(&base, &bytes, &ignored);
        }
        const LdsTiling &ft = f_tiling(h);
        Lds2Layout lay = nchw_layout(h->kdesc, ft);
        if (stage_phases) {
            // the input side of the layout is the caller's tensor; the output side is the same for both forms
            const int64_t HW = (int64_t)h->desc.H * h->desc.W;
            lay.phase_stride = h->desc.stride;
            lay.src_w = h->desc.W;
            lay.in_img = h->desc.C * HW; lay.in_tile = 4 * lay.in_img; lay.in_ch = HW; lay.in_pos = 1;
            lay.in_rec_fixed = 0; lay.in_rec_img = lay.in_img * 4; lay.in_rec_tile = 0;
        }
        return run_flat(h, h->kdesc, ft, h->dev_lds, lay, in, out, N, out_rows, out_inner, ep, hip_stream, ws);
    }
    if (use_lds) {
        if (!h->lds_uploaded) {
            rc = upload(h->lds.pairs.data(), h->lds.pairs.size() * 8, &h->dev_lds.pairs, &h->hip_err);
            if (!rc) rc = upload(h->lds.seg_ptr.data(), h->lds.seg_ptr.size() * 4, &h->dev_lds.seg_ptr, &h->hip_err);
            if (!rc) rc = upload(h->lds.row_of.data(), h->lds.row_of.size() * 4, &h->dev_lds.row_of, &h->hip_err);
            if (rc) return rc;
            h->lds_uploaded = true;
        }
        rc = launch_lds(h->kdesc, h->lds.t, h->dev_lds, in, out, N, hip_stream, &h->hip_err);
        return rc ? rc : launch_epilogue(out, out_rows, out_inner, h->desc.K, ep, hip_stream, &h->hip_err);
    }
    if (!h->direct_uploaded) {
        rc = upload(h->direct.rowptr.data(), h->direct.rowptr.size() * 4, &h->dev_direct.rowptr, &h->hip_err);
        if (!rc) rc = upload(h->direct.trip.data(), h->direct.trip.size() * 4, &h->dev_direct.trip, &h->hip_err);
        if (rc) return rc;
        h->direct_uploaded = true;
    }
    rc = launch_direct(h->desc, h->dev_direct, in, out, N, hip_stream, &h->hip_err);
    return rc ? rc : launch_epilogue(out, out_rows, out_inner, h->desc.K, ep, hip_stream, &h->hip_err);
}

extern "C" int sconv_forward_noalloc(sconv_csr *h, const float *in, float *out, int32_t N, void *hip_stream)
{
    if (!h) return SCONV_ERR_NULL;
    Workspace ws;
    void *base = nullptr;
    const int rc = static_scratch(&base, &ws.bytes, &h->hip_err);
    if (rc) return rc;
    ws.base = static_cast<char *>(base);
    return forward_impl(h, in, out, N, Epilogue(), hip_stream, &ws);
}

// ---- fully connected layers: out_t[K][N] = W[K][C] (CSR) x in_t[C][N] -------------------------------
//
// With the activations feature-major, four consecutive images of one feature are exactly one LDS cell of
// the flat-stream kernel and a feature's row is a channel plane: the product is the 1x1 convolution of a
// C-channel "image" of N/4 positions x 4 images, and the kernel runs it unchanged through other strides.

static bool is_fc(const sconv_desc &d)
{
    return d.H == 1 && d.W == 1 && d.R == 1 && d.S == 1 && d.stride == 1 && d.pad == 0 && d.groups == 1;
}

static void release_fc(sconv_csr *h)
{
    release(h->fc_dev.pairs);
    release(h->fc_dev.seg_ptr);
    release(h->fc_dev.row_of);
    release(h->fc_dev.store_tbl);
    h->fc_dev = DeviceLds();
    h->fc_uploaded = false;
}

// The layer as the flat-stream kernel sees it for a batch of N: `tiles` tiles of N / tiles images, f
// consecutive features forming one channel of f rows (a filter of f x 1 taps, one output row): the same
// arithmetic, but a channel plane is f times larger, so that every wave of a workgroup has a part of it
// to stage when the batch alone gives a plane of only a few hundred floats.
static int fc_mapping(const sconv_csr *h, int N, sconv_desc &kd, int &tiles)
{
    if (!is_fc(h->desc)) return SCONV_ERR_DESC;
    if (N < 4 || N % 4) return SCONV_ERR_BATCH;
    // one wave covers at most 4 x 256 images; larger batches are cut into equal tiles
    tiles = (N + 1023) / 1024;
    if (N % (4 * tiles)) return SCONV_ERR_BATCH;
    const int nc = N / tiles;
    int f = 1;
    if (tiles == 1)
        for (int c : {16, 8, 4, 2})
            if (h->desc.C % c == 0 && c * nc <= 1024) {
                f = c;
                break;
            }
    kd = h->desc;
    kd.C = h->desc.C / f;
    kd.H = f;
    kd.R = f;
    kd.W = nc / 4;
    return SCONV_OK;
}

// What the tiling search is asked for: the fields of the plan the handle was created with are honoured
// where they apply to this mapping.
static sconv_plan fc_request(const sconv_csr *h)
{
    sconv_plan req = h->requested;
    req.kernel = (req.kernel == 3 || req.kernel == 4) ? req.kernel : 0; // tiles of four images: a flat-stream variant either way
    req.nt = 4;
    req.band = 0;
    req.strip = 0;
    return req;
}

// Pack for a batch of N.  force: a complete tiling to use (sconv_fc_tune's candidates); otherwise the one
// tuned for N if there is one, otherwise the cost model's choice.
static int plan_fc(sconv_csr *h, int N, const sconv_plan *force = nullptr)
{
    sconv_desc kd;
    int tiles;
    int rc = fc_mapping(h, N, kd, tiles);
    if (rc) return rc;
    if (!force) {
        auto tuned = h->fc_plan_of_n.find(N);
        if (tuned != h->fc_plan_of_n.end()) force = &tuned->second;
    }
    if (N == h->fc_n && (!force || same_plan(*force, h->fc_flat.t.p))) return SCONV_OK;
    if (h->fc_n > 0) { // set the current packing aside; one for this batch size may be waiting there
        StashedPacking old;
        old.flat = true;
        old.lds_flat = std::move(h->fc_flat);
        old.dev = h->fc_dev;
        old.uploaded = h->fc_uploaded;
        old.fc_n = h->fc_n;
        old.fc_tiles = h->fc_tiles;
        old.fc_desc = h->fc_desc;
        h->fc_stash.push_back(std::move(old));
        h->fc_dev = DeviceLds();
        h->fc_uploaded = false;
        h->fc_n = 0;
        while (h->fc_stash.size() > h->stash_cap) {
            release_arrays(h->fc_stash.front().dev);
            h->fc_stash.erase(h->fc_stash.begin());
        }
    }
    for (size_t i = 0; i < h->fc_stash.size(); ++i) {
        StashedPacking &sp = h->fc_stash[i];
        if (sp.fc_n != N || (force && !same_plan(*force, sp.lds_flat.t.p))) continue;
        h->fc_flat = std::move(sp.lds_flat);
        h->fc_dev = sp.dev;
        h->fc_uploaded = sp.uploaded;
        h->fc_tiles = sp.fc_tiles;
        h->fc_desc = sp.fc_desc;
        h->fc_n = N;
        h->fc_stash.erase(h->fc_stash.begin() + (long)i);
        return SCONV_OK;
    }
    Canonical kc;
    kc.rowptr = h->canon.rowptr;
    kc.colidx = h->canon.colidx;
    kc.val = h->canon.val;
    kc.off.resize(h->canon.off.size());
    for (size_t j = 0; j < kc.off.size(); ++j) kc.off[j] = h->canon.off[j] * kd.W; // feature c = row c of the wide image
    const double avg = kd.K ? (double)kc.val.size() / kd.K : 0.0;
    LdsTiling t;
    rc = make_lds_tiling(kd, force ? *force : fc_request(h), 4 * tiles, avg, t, 0, true);
    if (rc) return rc;
    t.out_pos = 4; // the four images of a cell are consecutive in the output row
    rc = pack_flat(kd, kc, t, h->fc_flat);
    if (rc) return rc;
    h->fc_desc = kd;
    h->fc_tiles = tiles;
    h->fc_n = N;
    return SCONV_OK;
}

extern "C" int sconv_fc_plan(sconv_csr *h, int32_t N, sconv_plan *plan)
{
    if (!h || !plan) return SCONV_ERR_NULL;
    try {
        const int rc = plan_fc(h, N);
        if (rc) return rc;
    } catch (const std::bad_alloc &) {
        return SCONV_ERR_NOMEM;
    }
    *plan = h->fc_flat.t.p;
    return SCONV_OK;
}

extern "C" int sconv_fc_forward(sconv_csr *h, const float *in_t, float *out_t, int32_t N, const float *bias, int32_t relu,
                                void *hip_stream)
{
    if (!h || !in_t || !out_t) return SCONV_ERR_NULL;
    if (N < 1) return SCONV_ERR_BATCH;
    int rc;
    try {
        rc = plan_fc(h, N);
    } catch (const std::bad_alloc &) {
        return SCONV_ERR_NOMEM;
    }
    if (rc) return rc;
    if (!h->fc_uploaded) {
        const PackedFlat &f = h->fc_flat;
        rc = upload(f.pairs.data(), f.pairs.size() * 8, &h->fc_dev.pairs, &h->hip_err);
        if (!rc) rc = upload(f.seg.data(), f.seg.size() * 4, &h->fc_dev.seg_ptr, &h->hip_err);
        if (!rc) rc = upload(f.row_of.data(), f.row_of.size() * 4, &h->fc_dev.row_of, &h->hip_err);
        if (!rc) rc = upload(f.store_tbl.data(), f.store_tbl.size() * 4, &h->fc_dev.store_tbl, &h->hip_err);
        if (rc) {
            release_fc(h);
            return rc;
        }
        h->fc_uploaded = true;
    }
    const LdsTiling &t = h->fc_flat.t;
    const int64_t C = h->desc.C, K = h->desc.K, nc = N / h->fc_tiles;
    Lds2Layout lay;
    lay.in_tile = nc; lay.in_img = 1; lay.in_ch = (int64_t)h->fc_desc.H * N; lay.in_pos = 4;
    lay.in_rec_fixed = C * N * 4; lay.in_rec_img = 0; lay.in_rec_tile = nc * 4;
    lay.out_tile = nc; lay.out_band = 0; lay.out_row = N; lay.out_img = 1; lay.out_pos = 4;
    Epilogue ep;
    ep.bias = bias;
    ep.relu = relu != 0;
    return run_flat(h, h->fc_desc, t, h->fc_dev, lay, in_t, out_t, 4 * h->fc_tiles, K, N, ep, hip_stream);
}

// ---- measured choice of the tiling ----------------------------------------------------------------------

// Times run() after install(candidate) for every candidate and returns the index of the fastest in *best
// (-1 if none could be installed and run).  A candidate that cannot be packed or launched is skipped.
// All candidates are packed and uploaded first and stay in the handle's stash, so that the timed part only
// switches between them: the GPU's clocks drop while the host packs, and a candidate timed right after
// that would look 10-15 % slower than one timed later.
template <class Install, class Run>
static int time_candidates(sconv_csr *h, const std::vector<LdsTiling> &cands, Install install, Run run, void *stream, int *best)
{
    *best = -1;
    std::vector<size_t> ok;
    for (size_t i = 0; i < cands.size(); ++i)
        if (install(cands[i].p) == SCONV_OK && run() == SCONV_OK) ok.push_back(i);
    if (ok.empty()) return SCONV_OK;
    StreamTimer timer;
    int rc = timer_create(timer, &h->hip_err);
    if (rc) return rc;
    // `n` runs between two events, in milliseconds per run
    auto timed = [&](int n, float *ms) {
        int r = timer_start(timer, stream, &h->hip_err);
        for (int k = 0; k < n && !r; ++k) r = run();
        if (!r) r = timer_stop_ms(timer, stream, ms, &h->hip_err);
        *ms /= (float)n;
        return r;
    };
    // warm-up, about 30 ms of the first candidate
    float ms = 0, spent = 0;
    rc = install(cands[ok[0]].p);
    for (int k = 0; k < 200 && !rc && spent < 30.0f; ++k) {
        rc = timed(4, &ms);
        spent += 4 * ms;
    }
    // three rounds over the candidates, about 2 ms each; a candidate's time is its fastest round
    std::vector<float> t(ok.size(), std::numeric_limits<float>::max());
    for (int round = 0; round < 3 && !rc; ++round)
        for (size_t j = 0; j < ok.size() && !rc; ++j) {
            rc = install(cands[ok[j]].p);
            if (!rc) rc = timed(1, &ms);
            if (rc) break;
            const int reps = std::max(3, std::min(40, (int)(2.0f / std::max(ms, 0.01f))));
            rc = timed(reps, &ms);
            if (!rc) t[j] = std::min(t[j], ms);
        }
    timer_destroy(timer);
    if (rc) return rc;
    size_t arg = 0;
    for (size_t j = 1; j < ok.size(); ++j)
        if (t[j] < t[arg]) arg = j;
    // the timings repeat to 1-2 %: the cost model's own choice stands unless another is clearly faster
    if (ok[0] == 0 && t[arg] > 0.985f * t[0]) arg = 0;
    *best = (int)ok[arg];
    return SCONV_OK;
}

// The stash holds every candidate while they are timed; afterwards the oldest go.
struct StashRoom {
    sconv_csr *h;
    StashRoom(sconv_csr *handle, size_t n) : h(handle) { h->stash_cap = std::max(kStashed, n); }
    ~StashRoom()
    {
        h->stash_cap = kStashed;
        while (h->stash.size() > kStashed) {
            release_arrays(h->stash.front().dev);
            h->stash.erase(h->stash.begin());
        }
        while (h->fc_stash.size() > kStashed) {
            release_arrays(h->fc_stash.front().dev);
            h->fc_stash.erase(h->fc_stash.begin());
        }
    }
};

static int clamp_plans(int max_plans) { return max_plans < 1 ? 8 : std::min(max_plans, 32); }

extern "C" int sconv_rank_plans(const sconv_csr *h, int32_t N, int32_t max_plans, sconv_plan *plans, int32_t *count)
{
    if (!h || !plans || !count) return SCONV_ERR_NULL;
    *count = 0;
    if (N < 1) return SCONV_ERR_BATCH;
    if (!h->has_lds) return SCONV_ERR_PLAN;
    try {
        const double avg = h->kdesc.K ? (double)h->canon.val.size() / h->kdesc.K : 0.0;
        std::vector<LdsTiling> cands;
        const int rc = rank_lds_tilings(h->kdesc, h->requested, N < 4 ? 4 : N, avg, clamp_plans(max_plans), cands, h->phase_cg());
        if (rc) return rc;
        for (const LdsTiling &t : cands) plans[(*count)++] = t.p;
    } catch (const std::bad_alloc &) {
        return SCONV_ERR_NOMEM;
    }
    return SCONV_OK;
}

extern "C" int sconv_tune(sconv_csr *h, const float *in, float *out, int32_t N, int32_t max_plans, void *hip_stream)
{
    if (!h || !in || !out) return SCONV_ERR_NULL;
    if (N < 1) return SCONV_ERR_BATCH;
    const sconv_plan &rq = h->requested;
    const bool free_choice = !rq.nt && !rq.cb && !rq.waves && !rq.cg && !rq.rows_w && !rq.t && !rq.band && !rq.strip && !rq.splits;
    if (!h->has_lds || !free_choice) return SCONV_ERR_PLAN;
    const int n_plan = N < 4 ? 4 : N;
    const Epilogue none;
    try {
        const double avg = h->kdesc.K ? (double)h->canon.val.size() / h->kdesc.K : 0.0;
        std::vector<LdsTiling> cands;
        int rc = rank_lds_tilings(h->kdesc, h->requested, n_plan, avg, clamp_plans(max_plans), cands, h->phase_cg());
        if (rc) return rc;
        int best = -1;
        StashRoom room(h, cands.size());
        rc = time_candidates(
            h, cands,
            [&](const sconv_plan &p) {
                h->plan_of_n[n_plan] = p;
                return plan_lds(h, n_plan);
            },
            [&]() { return forward_impl(h, in, out, N, none, hip_stream); }, hip_stream, &best);
        // the fastest, or the cost model's choice if nothing could be timed
        h->plan_of_n[n_plan] = cands[best < 0 ? 0 : (size_t)best].p;
        const int prc = plan_lds(h, n_plan);
        if (rc) return rc;
        if (prc) return prc;
    } catch (const std::bad_alloc &) {
        return SCONV_ERR_NOMEM;
    }
    return forward_impl(h, in, out, N, none, hip_stream);
}

extern "C" int sconv_fc_tune(sconv_csr *h, const float *in_t, float *out_t, int32_t N, int32_t max_plans, void *hip_stream)
{
    if (!h || !in_t || !out_t) return SCONV_ERR_NULL;
    if (N < 1) return SCONV_ERR_BATCH;
    try {
        sconv_desc kd;
        int tiles;
        int rc = fc_mapping(h, N, kd, tiles);
        if (rc) return rc;
        const double avg = kd.K ? (double)h->canon.val.size() / kd.K : 0.0;
        std::vector<LdsTiling> cands;
        rc = rank_lds_tilings(kd, fc_request(h), 4 * tiles, avg, clamp_plans(max_plans), cands, 0, true);
        if (rc) return rc;
        int best = -1;
        StashRoom room(h, cands.size());
        h->fc_plan_of_n.erase(N);
        rc = time_candidates(
            h, cands, [&](const sconv_plan &p) { return plan_fc(h, N, &p); },
            [&]() { return sconv_fc_forward(h, in_t, out_t, N, nullptr, 0, hip_stream); }, hip_stream, &best);
        if (rc) return rc;
        h->fc_plan_of_n[N] = cands[best < 0 ? 0 : (size_t)best].p;
        rc = plan_fc(h, N); // while the candidates' packings are still at hand
        if (rc) return rc;
    } catch (const std::bad_alloc &) {
        return SCONV_ERR_NOMEM;
    }
    return sconv_fc_forward(h, in_t, out_t, N, nullptr, 0, hip_stream);
}

extern "C" int sconv_last_hip_error(const sconv_csr *h) { return h ? h->hip_err : 0; }

extern "C" void sconv_destroy_csr(sconv_csr *h)
{
    if (!h) return;
    release(h->dev_lds.pairs);
    release(h->dev_lds.seg_ptr);
    release(h->dev_lds.row_of);
    release(h->dev_lds.store_tbl);
    release(h->phase_buf);
    release(h->part_buf);
    release_fc(h);
    for (auto &sp : h->stash) release_arrays(sp.dev);
    for (auto &sp : h->fc_stash) release_arrays(sp.dev);
    release(h->dev_direct.rowptr);
    release(h->dev_direct.trip);
    delete h;
}

extern "C" const char *sconv_strerror(int status)
{
    switch (status) {
    case SCONV_OK: return "ok";
    case SCONV_ERR_NULL: return "a required pointer is NULL";
    case SCONV_ERR_DESC: return "bad layer descriptor";
    case SCONV_ERR_CSR: return "malformed CSR arrays";
    case SCONV_ERR_BATCH: return "batch size below 1, or not one the fully connected path takes (a multiple of 4 per tile)";
    case SCONV_ERR_CAPACITY: return "output buffer too small";
    case SCONV_ERR_PLAN: return "tiling not runnable for this layer";
    case SCONV_ERR_HIP: return "HIP call failed";
    case SCONV_ERR_NOMEM: return "out of host memory";
    case SCONV_ERR_RANGE: return "sizes exceed 32-bit offsets";
    default: return "unknown status";
    }
}

// ------------------------------------------------------------------------------------------------
// Section 2.2: t_dense = C/F, t_sparse_compute = alpha*x*C/F, t_sparse_bw = (S_A + beta*x*S_W)/B,
// speedup = t_dense / max(t_sparse_compute, t_sparse_bw).

extern "C" void sconv_machine_gfx950(sconv_machine *m)
{
    if (!m) return;
    // Achievable rates measured on one MI355X (see the benchmark report); not data-sheet peaks.
    m->dense_flops = 100e12;        // fp32 dense convolution / SGEMM proxy
    m->hbm_bytes_per_s = 4.9e12;    // device copy kernel (read + write), 1 GiB
    m->alpha = 0.0;                 // derive from the ceilings below
    m->beta = 2.0;
    m->fma_flops = 73.5e12;         // v_fma_f32, 256 CUs x 60 lanes-FMA/clk x 2.4 GHz x 2
    m->lds_bytes_per_s = 148e12;    // aligned ds_read_b128, 242 B/clk/CU
    m->lds_bytes_per_fma = 4.0;
    m->lane_efficiency = 0.73;      // 0.9 (lanes that are outputs) x 0.8 (issue slots left after address
                                    // arithmetic, LDS waits and barriers): CALIBRATED to the measured x = 1
                                    // plateau of 53-55 TFLOP/s, as the paper takes alpha from its measured plateau
    m->t_fixed = 11.4e-6;           // intercept of time against nonzeros on conv3's shape at batch 256
}

static int predict(const sconv_desc *desc, int32_t N, double density, const sconv_csr *h, const sconv_machine *m,
                   bool lowered, sconv_prediction *out);

extern "C" int sconv_model_predict(const sconv_desc *desc, int32_t N, double density, const sconv_csr *h,
                                   const sconv_machine *m, sconv_prediction *out)
{
    return predict(desc, N, density, h, m, false, out);
}

extern "C" int sconv_model_predict_lowered(const sconv_desc *desc, int32_t N, double density, const sconv_csr *h,
                                           const sconv_machine *m, sconv_prediction *out)
{
    return predict(desc, N, density, h, m, true, out);
}

static int predict(const sconv_desc *desc, int32_t N, double density, const sconv_csr *h, const sconv_machine *m,
                   bool lowered, sconv_prediction *out)
{
    if (!desc || !out) return SCONV_ERR_NULL;
    int rc = validate_desc(*desc);
    if (rc) return rc;
    if (N < 1) return SCONV_ERR_BATCH;
    sconv_machine def;
    if (!m) {
        sconv_machine_gfx950(&def);
        m = &def;
    }
    const Geometry g = geometry(*desc);
    const double cols = (double)g.Cg * desc->R * desc->S;
    double x = density;
    if (h) x = (double)h->canon.val.size() / ((double)desc->K * cols);
    if (!(x >= 0.0) || !(m->dense_flops > 0) || !(m->hbm_bytes_per_s > 0)) return SCONV_ERR_DESC;
    double alpha = m->alpha;
    if (!(alpha > 0)) {
        const double lds_flops = 2.0 * m->lds_bytes_per_s / m->lds_bytes_per_fma;
        const double f_sparse = m->lane_efficiency * std::fmin(m->fma_flops, lds_flops);
        if (!(f_sparse > 0)) return SCONV_ERR_DESC;
        alpha = m->dense_flops / f_sparse;
    }
    sconv_prediction p;
    p.flops_dense = 2.0 * desc->K * cols * g.OH * g.OW * N;
    // direct: every input element once; lowered: the (C*R*S) x (OH*OW) matrix the lowering writes out
    const double in_elems = lowered ? (double)desc->C * desc->R * desc->S * g.OH * g.OW : (double)desc->C * desc->H * desc->W;
    p.bytes_act = 4.0 * N * (in_elems + (double)desc->K * g.OH * g.OW);
    p.bytes_w = 4.0 * desc->K * cols;
    p.density = x;
    p.alpha = alpha;
    p.t_dense = p.flops_dense / m->dense_flops;
    p.t_sparse_compute = alpha * x * p.flops_dense / m->dense_flops;
    p.t_sparse_bw = (p.bytes_act + m->beta * x * p.bytes_w) / m->hbm_bytes_per_s;
    p.t_sparse = std::fmax(p.t_sparse_compute, p.t_sparse_bw) + (m->t_fixed > 0 ? m->t_fixed : 0.0);
    p.speedup = p.t_dense / p.t_sparse;
    p.effective_flops = p.flops_dense / p.t_sparse;
    p.actual_flops = x * p.flops_dense / p.t_sparse;
    const double denom = alpha * p.flops_dense / m->dense_flops - m->beta * p.bytes_w / m->hbm_bytes_per_s;
    p.x_upper = denom > 0 ? (p.bytes_act / m->hbm_bytes_per_s) / denom : std::numeric_limits<double>::infinity();
    p.x_lower = 1.0 / alpha;
    p.bandwidth_bound = p.t_sparse_bw > p.t_sparse_compute ? 1 : 0;
    *out = p;
    return SCONV_OK;
}

// Section 2.3's algorithm, one layer, one decision: exclude layers without a useful sparsity range at the
// start; stop pruning a layer once its sparsity reaches the upper bound of the range (density <= x_upper);
// give up on a layer whose sparsity has stabilised at or below the lower bound (density >= x_lower) and
// restore its dense weights; otherwise keep pruning.
extern "C" int sconv_gsl_decide(const sconv_desc *desc, int32_t N, double density, int32_t stabilized,
                                const sconv_machine *m, int32_t *action, sconv_prediction *pred)
{
    if (!action) return SCONV_ERR_NULL;
    if (!(density > 0.0) || density > 1.0) return SCONV_ERR_DESC;
    sconv_prediction p;
    const int rc = sconv_model_predict(desc, N, density, nullptr, m, &p);
    if (rc) return rc;
    if (pred) *pred = p;
    if (!(p.x_upper < p.x_lower))
        *action = SCONV_GSL_EXCLUDE;
    else if (density <= p.x_upper)
        *action = SCONV_GSL_STOP;
    else if (stabilized && density >= p.x_lower)
        *action = SCONV_GSL_RESTORE_DENSE;
    else
        *action = SCONV_GSL_PRUNE;
    return SCONV_OK;
}
