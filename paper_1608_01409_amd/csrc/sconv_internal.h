// Internal declarations shared by the host code and the kernel launchers of libsconv.
#pragma once

#include <cstdint>
#include <vector>

#include "sconv.h"

namespace sconv {

// Nonzeros per straight-line group of the LDS kernel; (row, block) segments are padded to a multiple.
#define SCONV_PAIR_GROUP 4

struct Geometry {
    int Cg, Kg, Hp, Wp, OH, OW;
};

inline Geometry geometry(const sconv_desc &d)
{
    Geometry g;
    g.Cg = d.C / d.groups;
    g.Kg = d.K / d.groups;
    g.Hp = d.H + 2 * d.pad;
    g.Wp = d.W + 2 * d.pad;
    g.OH = (g.Hp - d.R) / d.stride + 1;
    g.OW = (g.Wp - d.S) / d.stride + 1;
    return g;
}

// Tiling of the LDS kernel, derived from a sconv_plan and the layer.
//
// LDS holds one block of `cb` input channels of `nt` images as
// [channel][cell][image]: `cell` runs over a Hl x Wl plane of the zero-padded
// image, `image` is innermost so that a lane reading `vec` consecutive floats
// reads `vec` images at one cell, always at an aligned address.  The row pitch
// is Wl = max(W + pad, OW): a read that falls into the right padding of a row
// lands on the left padding of the next one, which is zero as well.
// A workgroup computes a band of `band` output rows starting at row y0 and
// stages rows y0 .. y0 + band + R - 2 of the padded image; y below is relative
// to y0, so the packed offsets are the same for every band.
// A nonzero (c,r,s) of a row then reads, for flat output index
// F = pos*nt + image with pos = y*Wl + x, the float at
//   ((c_local*plane_cells + r*Wl + s)*nt) + F,
// i.e. the packed byte offset plus a per-lane constant.
struct LdsTiling {
    sconv_plan p;
    int vec;            // floats per lane per chunk: 4 if nt % 4 == 0 else 1
    int Wl, Hl;         // plane pitch and rows (Hl = band + R - 1 rows of the padded image)
    int n_bands;        // ceil(OH / band): bands of output rows, one workgroup each
    int plane_cells;    // Hl * Wl
    int pos_span;       // (band-1)*Wl + OW: positions a tile computes
    int pos_per_chunk;  // 64*vec / nt
    int n_chunks;       // ceil(pos_span / pos_per_chunk), <= cg*t
    int nblk;           // ceil(Cg / cb)
    int rg;             // row groups = waves / cg
    int nkt;            // K tiles per group
    int wave_slots;     // groups * nkt * rg
    int n_slabs;        // 64-float slabs per channel plane (staging granule)
    int n_bufs;         // LDS block buffers: 2 (double-buffered; 3 for the flow variant) unless the layer has fewer blocks
    int ctr_bytes_at;   // flow variant: byte offset in LDS of its per-block counters (nblk dwords), else 0
    int phase_cg;       // > 0: stride-1 form of a strided, unpadded layer whose blocks hold whole phases' channels
                        // (that many real channels per phase): staged straight from the caller's input
    int buf_stride_floats; // floats from one buffer to the next: block + zero page, multiple of 4
    int lds_bytes;      // dynamic LDS per workgroup
    unsigned zero_page; // byte offset, relative to a buffer, of its all-zero page (padding entries)
    int page_cells;     // size of that page in cells of nt floats
    int strip_rows;     // strip layout: rows of the block of positions one chunk covers (64 / strip), else 0
    int out_pos;        // floats from one output position to the next in the caller's layout (1 for NCHW)
};

struct PackedLds {
    LdsTiling t;
    std::vector<uint64_t> pairs;   // low 32 bits: fp32 value bits; high 32: LDS byte offset
    std::vector<int32_t> seg_ptr;  // [wave_slot][nblk][rows_w + 1] -> index into pairs
    std::vector<int32_t> row_of;   // [wave_slot][rows_w] -> output channel or -1
};

// plan.kernel values that run the flat-stream kernel: 3 = a barrier per channel block, two block buffers;
// 4 = the flow variant, lds2_flow_bufs() buffers and per-block counters instead of barriers.  Same packing for both.
inline bool is_flat_kernel(int kernel) { return kernel == 3 || kernel == 4; }

// Packing for the flat-stream kernel (tiles of 4 images).  One stream per (wave slot, channel block)
// holding the nonzeros of all rows of the slot in that block, padded to whole chunks of 8 entries:
//   low 32 bits  fp32 value bits
//   high 32 bits (LDS byte offset / 16) << 16 | (row index inside the slot * t * 4)
// Padding entries have value +0.0 and point at the zero page.
#define SCONV_FLAT_CHUNK 8
// The kernel warms L2 with this many bytes of the stream beyond the point its scalar loads have reached (which is
// up to two chunks past a segment's end): the stream array carries that much padding behind its last segment.
#define SCONV_FLAT_WARM_BYTES 4096
struct PackedFlat {
    LdsTiling t;
    std::vector<uint64_t> pairs;
    std::vector<uint32_t> seg;       // [wave_slot][nblk] x (byte offset into pairs, number of chunks)
    std::vector<int32_t> row_of;     // [wave_slot][rows_w] -> output channel or -1
    std::vector<int32_t> store_tbl;  // [cg*t*64] -> (by*OW + ox)*4 inside a band, or -1
};

struct PackedDirect {
    std::vector<int32_t> rowptr;   // K+1
    std::vector<uint32_t> trip;    // 3 words per nonzero: value bits, goff, (dr<<16)|(ds&0xffff)
};

struct Canonical {
    std::vector<int32_t> rowptr, colidx, off;
    std::vector<float> val;
};

int validate_desc(const sconv_desc &d);
// rowptr starts at 0 and never falls, columns inside [0, Cg*R*S) and strictly ascending in each row
int validate_csr(const sconv_desc &d, const int32_t *rowptr, const int32_t *colidx);
// colidx -> off for a padded image stored in `layout` (a sconv_layout); the arrays are assumed valid
void lower_offsets(const sconv_desc &d, int layout, const int32_t *rowptr, const int32_t *colidx, int32_t *off);
int build_canonical_from_dense(const sconv_desc &d, const float *w, Canonical &out);
int build_canonical_from_arrays(const sconv_desc &d, const int32_t *rowptr, const int32_t *colidx,
                                const float *values, Canonical &out);

// Fill in a tiling for the LDS kernel (fields of `req` that are 0 are chosen).  N_hint is the
// batch size the choice is tuned for.  Returns SCONV_ERR_PLAN if the layer cannot use it.
// phase_cg > 0: d is the stride-1 form of a strided layer without padding, with that many real channels per
// phase; tilings whose blocks hold whole phases' channels can then be staged without the phase-image pass.
// wide: the input will be staged a cell per lane and the output stored four images at a time (feature-major
// activations); the cost model prices the landing of a block and the stores accordingly.
int make_lds_tiling(const sconv_desc &d, const sconv_plan &req, int N_hint, double avg_row_nnz, LdsTiling &out, int phase_cg = 0,
                    bool wide = false);
// The max_out distinct tilings the cost model ranks best, best first (out[0] is make_lds_tiling's choice).
int rank_lds_tilings(const sconv_desc &d, const sconv_plan &req, int N_hint, double avg_row_nnz, int max_out,
                     std::vector<LdsTiling> &out, int phase_cg = 0, bool wide = false);
// p.kernel selects the shape list: 1 = per-row streams, 3 = flat streams (nt must be 4)
bool lds_kernel_available(int vec, int t, int rows_w);

int pack_lds(const sconv_desc &d, const Canonical &c, const LdsTiling &t, PackedLds &out);
int unpack_lds(const sconv_desc &d, const PackedLds &p, Canonical &out);
int pack_flat(const sconv_desc &d, const Canonical &c, const LdsTiling &t, PackedFlat &out);
int unpack_flat(const sconv_desc &d, const PackedFlat &p, Canonical &out);
bool lds2_kernel_available(int t, int rows_w, int step); // step: 64 (flat lanes) or the strip width
int lds2_depth(int t, int rows_w);
int lds2_flow_bufs(); // block buffers the flow variant of the flat-stream kernel rotates through // read-ahead depth of a flat-stream shape, 0 if there is none
int pack_direct(const sconv_desc &d, const Canonical &c, PackedDirect &out);
int unpack_direct(const sconv_desc &d, const PackedDirect &p, Canonical &out);

// Strided layers on the LDS kernels.  With stride s the input rows that one filter row r touches are
// y*s + r: split r = r'*s + py and they become rows y + r' of the "phase image" py (every s-th row of the
// padded image, starting at py), and the same along x.  A strided layer is therefore a stride-1, pad-0 layer
// over Cg*s*s virtual channels (py, px, c: phase by phase) of size Hq x Wq = (OH + R' - 1) x (OW + S' - 1) with an R' x S'
// filter, R' = ceil(R/s): no input element is duplicated, only re-ordered (Section 2.1 allows any layout
// function f that is additive in the output position).  phase_desc gives that layer, phase_canonical its
// CSR; unphase_canonical maps offsets of the virtual layer back to the real one.
void phase_desc(const sconv_desc &d, sconv_desc &v);
int phase_canonical(const sconv_desc &d, const Canonical &c, Canonical &vc);
int unphase_canonical(const sconv_desc &d, const Canonical &vc, Canonical &out);

// Device side (sconv_kernels.hip)
struct DeviceLds {
    void *pairs = nullptr, *seg_ptr = nullptr, *row_of = nullptr, *store_tbl = nullptr;
};
struct DeviceDirect {
    void *rowptr = nullptr, *trip = nullptr;
};
int launch_lds(const sconv_desc &d, const LdsTiling &t, const DeviceLds &dev, const float *in, float *out,
               int N, void *stream, int *hip_err);
// Bias and ReLU applied to the outputs (bias null = none).
struct Epilogue {
    const float *bias = nullptr;
    bool relu = false;
};
// Where the flat-stream kernel finds its operands, in floats.  Input element (image i of tile m, channel c,
// position p = Y*W + X of the unpadded image): m*in_tile + i*in_img + c*in_ch + p*in_pos.  Output (image i
// of tile m, row k, band b, position q inside the band): m*out_tile + b*out_band + k*out_row + i*out_img +
// q*out_pos.  nchw_layout() gives the convolution's [N][C][H][W] -> [N][K][OH][OW].
struct Lds2Layout {
    // phase_stride > 1: the input is the strided layer's own [N][C][H][src_w] tensor and the kernel picks the
    // phase images out of it while staging (cell (Y, X) of phase (py, px) is input (Y*s + py, X*s + px));
    // the tiling's phase_cg real channels make up one phase of a group
    int phase_stride = 1, src_w = 0;
    int64_t in_tile, in_img, in_ch, in_pos;
    int64_t in_rec_fixed, in_rec_img, in_rec_tile; // bytes tile m with n valid images may read: fixed + n * img - m * tile
    int64_t out_tile, out_band, out_row, out_img, out_pos;
};
Lds2Layout nchw_layout(const sconv_desc &d, const LdsTiling &t);
// With t.p.splits > 1 `out` is a workspace of splits * split_stride floats that receives each part's partial
// results in the output's layout, and launch_reduce adds them up (and applies the epilogue) afterwards.
int launch_lds2(const sconv_desc &d, const LdsTiling &t, const DeviceLds &dev, const Lds2Layout &lay, const float *in,
                float *out, int N, const Epilogue &ep, int64_t split_stride, void *stream, int *hip_err);
int launch_reduce(const float *parts, float *out, int splits, int64_t rows, int64_t inner, int K, const Epilogue &ep,
                  void *stream, int *hip_err);
// out[n][k][..] = max(out + bias[k], 0) in place, for the paths that do not fuse it: rows of `inner` floats
int launch_epilogue(float *out, int64_t rows, int64_t inner, int K, const Epilogue &ep, void *stream, int *hip_err);

// in [N][C][H][W] -> q [N][C*s*s][Hq][Wq], zero padding written out
int launch_phase(const sconv_desc &d, const sconv_desc &v, const float *in, float *q, int N, void *stream, int *hip_err);
int launch_direct(const sconv_desc &d, const DeviceDirect &dev, const float *in, float *out, int N,
                  void *stream, int *hip_err);
// The library's static device scratch (SCONV_NOALLOC_SCRATCH_BYTES) on the current device: its address
// there, looked up once per device and remembered.
int static_scratch(void **base, size_t *bytes, int *hip_err);
int upload(const void *host, size_t bytes, void **dev, int *hip_err);
void release(void *dev);

// A pair of events that brackets work on one stream (for sconv_tune); stop waits for the stream.
struct StreamTimer {
    void *e0 = nullptr, *e1 = nullptr;
};
int timer_create(StreamTimer &t, int *hip_err);
int timer_start(StreamTimer &t, void *stream, int *hip_err);
int timer_stop_ms(StreamTimer &t, void *stream, float *ms, int *hip_err);
void timer_destroy(StreamTimer &t);

} // namespace sconv
