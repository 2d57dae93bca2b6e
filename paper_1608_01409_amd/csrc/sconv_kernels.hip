// HIP kernels for direct sparse convolution on gfx950 and their launchers.
//
// sconv_lds_kernel: the hot path for stride-1 layers (Section 2.1's loop nest with the input and
// output channels tiled and the weight matrix column-blocked, re-thought for CDNA4):
//   * a workgroup owns `nt` images and a tile of CSR rows (output channels) and walks the input
//     channels of its group in blocks of `cb`;
//   * each block is staged global -> LDS as [channel][cell][image], zero padding included; the image
//     index is innermost so that a lane's read of 4 images at one cell is one aligned ds_read_b128
//     whatever the nonzero's offset is;
//   * the nonzeros (value, LDS byte offset) of a wave's rows are wave-uniform: they come through
//     scalar loads and sit in SGPRs; lanes span (output position, image);
//   * accumulators stay in VGPRs across all channel blocks and are stored once.
// sconv_direct_kernel: any stride, small batches; reads the unpadded input straight from global
// memory with a bounds test standing in for the padding.
#include <hip/hip_runtime.h>

#include <mutex>
#include <set>
#include <utility>

#include "sconv_internal.h"

namespace sconv {

struct LdsArgs {
    const float *in;
    float *out;
    const unsigned *pairs; // (value bits, LDS byte offset) per nonzero
    const int *seg_ptr;
    const int *row_of;
    int N, C, H, W, K, OH, OW, pad, Cg, groups;
    int nt, cb, nblk, rg, cg, nkt;
    int band, n_bands; // output rows per workgroup, bands per image
    int Wl, plane_floats, n_slabs, buf_stride_floats, lds_floats;
    int n_tiles, units;
};

constexpr int kMaxSlabsPerWave = 4; // 64-float slabs of a channel plane one wave stages
typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void global_void_t;
constexpr int kGroup = SCONV_PAIR_GROUP; // nonzeros per straight-line group; segments are padded to it
using const_u32 = const __attribute__((address_space(4))) unsigned;

#include "sconv_lds_loops.inc"

template <int VEC>
struct VecT;
template <>
struct VecT<4> {
    using type = float4;
};
template <>
struct VecT<1> {
    using type = float;
};

template <int VEC, int T, int ROWS_W>
__global__ void __launch_bounds__(1024) sconv_lds_kernel(const LdsArgs a)
{
    using vec_t = typename VecT<VEC>::type;
    extern __shared__ float4 smem4[];
    float *lds = reinterpret_cast<float *>(smem4);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Consecutive workgroup ids land on different XCDs (each with its own L2); the workgroups that
    // share one image tile (same input, different rows) are given ids 8 apart so they meet in one L2.
    // workgroup id -> (image tile, unit): tiles 8 at a time, one per XCD; leftover tiles spread over all XCDs
    const int bid = blockIdx.x;
    const int full = (a.n_tiles >> 3) * 8 * a.units;
    int unit, tile;
    if (bid < full) {
        const int xcd = bid & 7, slot = bid >> 3;
        unit = slot % a.units;
        tile = (slot / a.units) * 8 + xcd;
    } else {
        const int j = bid - full;
        tile = (a.n_tiles >> 3) * 8 + j / a.units;
        unit = j % a.units;
    }
    if (tile >= a.n_tiles) return;
    const int gk = unit / a.n_bands, band_i = unit - gk * a.n_bands;
    const int g = gk / a.nkt, kt = gk - g * a.nkt;
    const int n0 = tile * a.nt;
    const int y0 = band_i * a.band; // first output row (= first row of the padded image) of this band
    const int rgi = __builtin_amdgcn_readfirstlane(wave / a.cg);
    const int cgi = wave - rgi * a.cg;
    const int wslot = __builtin_amdgcn_readfirstlane((g * a.nkt + kt) * a.rg + rgi);

    const int HW = a.H * a.W;
    const int CHW = a.C * HW;
    const float *in_tile = a.in + (size_t)n0 * CHW;

    // ---- staging set-up.  A channel plane in LDS is plane_floats = cells*nt floats, image innermost.  It is
    // filled 64 floats at a time by global_load_lds_dword: lane l of the instruction for slab s loads the
    // float (cell, image) = divmod(s*64 + l, nt) from its own global address and the hardware writes it to
    // LDS at (M0 base) + l*4, with no VGPR and no VALU work, asynchronously (vmcnt).  Lanes whose cell is
    // padding, whose image is past the batch or whose float is past the plane are masked off and their LDS
    // words keep the zero written once below.  A wave always stages the same slabs, so the per-lane source
    // offsets are computed once.
    const int n_waves = (int)blockDim.x >> 6;
    int src_off[kMaxSlabsPerWave];
#pragma unroll
    for (int j = 0; j < kMaxSlabsPerWave; ++j) {
        const int f = (wave + j * n_waves) * 64 + lane;
        const int cell = f / a.nt, img = f - cell * a.nt;
        const int Y = cell / a.Wl, X = cell - Y * a.Wl;
        const int iy = y0 + Y - a.pad, ix = X - a.pad;
        const bool ok = f < a.plane_floats && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W && n0 + img < a.N;
        src_off[j] = ok ? img * CHW + iy * a.W + ix : -1;
    }
    {
        float4 *z = reinterpret_cast<float4 *>(lds);
        for (int i = tid; i < a.lds_floats / 4; i += blockDim.x) z[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __syncthreads();

    auto stage = [&](int b, int buf) {
        const int c0 = g * a.Cg + b * a.cb;
        const int cb_here = min(a.cb, a.Cg - b * a.cb);
#pragma unroll
        for (int j = 0; j < kMaxSlabsPerWave; ++j) {
            const int slab = wave + j * n_waves;
            if (slab >= a.n_slabs) break;
            if (src_off[j] >= 0) {
                for (int cl = 0; cl < cb_here; ++cl) {
                    const float *src = in_tile + (size_t)(c0 + cl) * HW + src_off[j];
                    float *dst = lds + buf * a.buf_stride_floats + cl * a.plane_floats + slab * 64;
                    __builtin_amdgcn_global_load_lds((global_void_t *)src, (lds_void_t *)dst, 4, 0, 0);
                }
            }
        }
    };

    // acc[(i*T + t)*VEC + e]: row i of this wave, chunk t, image e of the lane's quad
    float acc[ROWS_W * T * VEC];
#pragma unroll
    for (int i = 0; i < ROWS_W * T * VEC; ++i) acc[i] = 0.f;

    const unsigned lane_byte0 = (unsigned)((cgi * T * 64 + lane) * VEC * 4);
    const char *lds_bytes = reinterpret_cast<const char *>(lds);
    // the nonzero stream is read-only for the whole launch: constant address space => scalar loads
    const_u32 *cp = (const_u32 *)(a.pairs);
    const_u32 *cseg = (const_u32 *)(a.seg_ptr);
    const_u32 *crow = (const_u32 *)(a.row_of);

    // Double-buffered: while block b is being multiplied out of buffer b&1, block b+1 streams into the
    // other buffer.  One barrier per block: past it every wave's loads of block b have landed and every
    // wave has finished with the buffer that block b+1 is about to overwrite.
    stage(0, 0);
    for (int b = 0; b < a.nblk; ++b) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (b + 1 < a.nblk) stage(b + 1, (b + 1) & 1);
        const unsigned lane_byte = lane_byte0 + (unsigned)((b & 1) * a.buf_stride_floats * 4);

        // Nonzeros of this wave's rows inside this channel block.  Every (row, block) segment is padded
        // on the host to whole chunks of kGroup entries (padding: value 0 at an all-zero LDS page).
        const_u32 *sp = cseg + ((size_t)wslot * a.nblk + b) * (ROWS_W + 1);
        int ptr[ROWS_W + 1];
#pragma unroll
        for (int i = 0; i <= ROWS_W; ++i) ptr[i] = (int)sp[i];
        if constexpr (VEC == 4) {
            int cnt[ROWS_W];
#pragma unroll
            for (int i = 0; i < ROWS_W; ++i) cnt[i] = (ptr[i + 1] - ptr[i]) / kGroup;
            if (ptr[ROWS_W] > ptr[0]) SegLoop<T, ROWS_W>::run(acc, a.pairs + 2 * (size_t)ptr[0], cnt, lane_byte);
        } else {
#pragma unroll
            for (int i = 0; i < ROWS_W; ++i) {
                for (int j = ptr[i]; j < ptr[i + 1]; ++j) {
                    const float w = __uint_as_float(cp[2 * j]);
                    const float *src = reinterpret_cast<const float *>(lds_bytes + (lane_byte + cp[2 * j + 1]));
#pragma unroll
                    for (int t = 0; t < T; ++t) acc[i * T + t] = fmaf(w, src[t * 64], acc[i * T + t]);
                }
            }
        }
    }

    // ---- epilogue: flat index F = pos*nt + image; a lane's VEC floats are VEC images at one position.
    const int OHW = a.OH * a.OW;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const int F0 = ((cgi * T + t) * 64 + lane) * VEC;
        const int pos = F0 / a.nt, nl = F0 - pos * a.nt;
        const int by = pos / a.Wl, ox = pos - by * a.Wl;
        const int oy = y0 + by;
        const bool valid = ox < a.OW && by < a.band && oy < a.OH;
#pragma unroll
        for (int i = 0; i < ROWS_W; ++i) {
            const int k = (int)crow[wslot * ROWS_W + i];
            if (k < 0) continue;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int n = n0 + nl + e;
                if (valid && n < a.N) a.out[((size_t)n * a.K + k) * OHW + oy * a.OW + ox] = acc[(i * T + t) * VEC + e];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// sconv_lds2_kernel: the flat-stream variant of the LDS-tiled kernel for tiles of 4 images.  Same
// tiling and LDS layout as above; what differs:
//   * the rows of a wave share one nonzero stream per channel block (entry = weight, LDS offset,
//     accumulator index), so nothing is padded per row and the rows of a wave need not be balanced;
//   * the accumulators are addressed through the VGPR index mode, so the whole tile (staging, channel
//     blocks, stores) runs inside one asm statement that owns a fixed block of registers;
//   * staging uses buffer loads into LDS whose range check returns 0 for the padding cells, so no
//     part of a plane is ever cleared and every cell of a block is rewritten with each block.
// Division of a small non-negative number by a divisor fixed per launch: a multiply-high with
// magic = ceil(2^32 / d), exact while n * d < 2^32 (the launcher checks the largest n of each use and passes
// magic = 0, meaning "divide", where that does not hold or d is 1).  The generic 32-bit division costs some 30
// instructions per use, and the kernel's first microsecond was mostly these.
struct FastDiv {
    unsigned d, magic;
};
static __device__ __forceinline__ int fdiv(int n, FastDiv f)
{
    return f.magic ? (int)__umulhi((unsigned)n, f.magic) : n / (int)f.d;
}
static FastDiv make_fastdiv(int d, int64_t n_max)
{
    FastDiv f;
    f.d = (unsigned)d;
    f.magic = (d > 1 && n_max * (int64_t)d < ((int64_t)1 << 32)) ? (unsigned)((((uint64_t)1 << 32) + d - 1) / (uint64_t)d) : 0u;
    return f;
}

struct Lds2Args {
    const float *in;
    float *out;
    const unsigned *pairs;   // stream entries
    const unsigned *seg;     // [wave slot][block] x (byte offset into pairs, chunks of 8 entries)
    const int *row_of;       // [wave slot][R]
    const int *store_tbl;    // [cg*T*64] byte offset (by*OW + ox)*4 of a position inside its band, or -1
    int cb, nblk, Cg, plane_bytes, buf_stride_bytes, HW4, OHW4, img_stride_bytes; // read by the asm
    int N, C, H, W, K, OH, OW, pad;
    int rg, cg, nkt, band, n_bands, Wl, plane_floats, n_slabs;
    int n_tiles, units, block_bytes, page_bytes, n_bufs;
    int strip, strip_rows;   // lanes of a wave span strip_rows x strip cells of the plane (0: 64 consecutive cells)
    // input addressing in floats: element (image i of the tile, channel c, row Y, column X of the unpadded
    // image) sits at tile * in_tile + i * in_img + c * (HW4 / 4) + (Y * W + X) * in_pos
    long long in_tile;
    int in_img, in_pos;
    long long in_rec_fixed, in_rec_img, in_rec_tile; // tile m with n valid images may read in_rec_fixed + n * in_rec_img - m * in_rec_tile bytes; past that, 0
    long long out_tile;      // floats from one tile's outputs to the next
    int out_band;            // floats from one band's outputs to the next (band * OW for NCHW)
    int out_pos4;            // bytes from one output position to the next (4 for NCHW); the store table holds multiples
    int splits, blk_split;   // workgroups along the input channels, channel blocks each of them takes
    long long split_stride;  // floats from one part's partial results to the next (out then is the workspace)
    const float *bias;       // [K] added to every output of row k, or null
    int relu;                // outputs below zero become zero
    int ctr_bytes_at;        // flow: LDS byte offset of the per-block landing counters (one dword per block)
    // strided layers staged straight from the caller's input (phase_stride > 1), else {huge, 1, 0, 0}: read by the asm
    int blocks_per_phase, phase_stride, src_row_bytes, phase_span_bytes; // phase_span = the group's channels of one phase
    int phase_cg;            // real channels per phase of a group
    int wide;                // the four images of a cell are adjacent in memory (16-byte aligned): staged a cell per lane
    FastDiv d_pcg, d_pstride;
    FastDiv d_units, d_splits, d_bands, d_nkt, d_cg, d_wl, d_strip; // the divisors of the index arithmetic below
};

typedef int int4v __attribute__((ext_vector_type(4)));

#include "sconv_lds2_asm.inc"

static_assert(offsetof(Lds2Args, pairs) == SCONV_LDS2_OFF_PAIRS, "asm reads pairs here");
static_assert(offsetof(Lds2Args, store_tbl) == SCONV_LDS2_OFF_TBL, "asm reads store_tbl here");
static_assert(offsetof(Lds2Args, cb) == SCONV_LDS2_OFF_CONSTS, "asm reads eight constants from here");
static_assert(offsetof(Lds2Args, img_stride_bytes) == SCONV_LDS2_OFF_CONSTS + 28, "layout of the constants");
static_assert(offsetof(Lds2Args, blocks_per_phase) == SCONV_LDS2_OFF_PHASE, "asm reads the four phase constants from here");
static_assert(SCONV_LDS2_WARM_BYTES == SCONV_FLAT_WARM_BYTES, "the host pads the stream by what the kernel reads ahead");
static_assert(offsetof(Lds2Args, phase_span_bytes) == SCONV_LDS2_OFF_PHASE + 12, "layout of the phase constants");

constexpr unsigned kSkipLane = 0xFFFFFFFFu; // lane past the end of a plane: writes nothing
constexpr unsigned kZeroLane = 0x80000000u; // padding cell: beyond num_records, the load returns 0

template <int T, int R, int STEP, bool FLOW>
__global__ void __launch_bounds__(1024) sconv_lds2_kernel(const Lds2Args a)
{
    extern __shared__ float4 smem4[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_waves = (int)blockDim.x >> 6;

    // Workgroup ids go round the 8 XCDs (each with its own L2).  Image tiles are taken 8 at a time, one per
    // XCD, so that the workgroups that stage the same input for different rows, bands and channel parts
    // meet in one L2; the tiles left over when their number is not a multiple of 8 are spread over all
    // XCDs unit by unit, so that a launch with few tiles still uses the whole chip.
    const int bid = blockIdx.x;
    const int full = (a.n_tiles >> 3) * 8 * a.units;
    int unit, tile;
    if (bid < full) {
        const int xcd = bid & 7, slot = bid >> 3;
        const int q = fdiv(slot, a.d_units);
        unit = slot - q * a.units;
        tile = q * 8 + xcd;
    } else {
        const int j = bid - full;
        const int q = fdiv(j, a.d_units);
        tile = (a.n_tiles >> 3) * 8 + q;
        unit = j - q * a.units;
    }
    if (tile >= a.n_tiles) return;
    const int us = fdiv(unit, a.d_splits), split = unit - us * a.splits;
    const int gk = fdiv(us, a.d_bands), band_i = us - gk * a.n_bands;
    const int g = fdiv(gk, a.d_nkt), kt = gk - g * a.nkt;
    const int n0 = tile * 4;
    const int y0 = band_i * a.band;
    const int blk0 = split * a.blk_split;                                 // first channel block of this workgroup
    const int nblk_here = min(a.blk_split, a.nblk - blk0);
    if (nblk_here <= 0) return; // the host never launches an empty part; the block loop needs one block at least
    const int ch0 = blk0 * a.cb, nch_here = min(nblk_here * a.cb, a.Cg - ch0);
    const int rgi = __builtin_amdgcn_readfirstlane(fdiv(wave, a.d_cg));
    const int cgi = wave - rgi * a.cg;
    const int wslot = __builtin_amdgcn_readfirstlane((g * a.nkt + kt) * a.rg + rgi);
    const int nimg = min(4, a.N - n0);

    // per-lane source offsets of the slabs this wave stages, relative to channel 0 of image n0.  A slab is what
    // one load instruction fills: 64 floats (16 cells, a float per lane), or 64 cells (a cell per lane) where the
    // four images of a cell are 16 adjacent, aligned bytes of the input (a.wide: feature-major activations).
    const bool wide = a.wide != 0;
    const int n_slabs = wide ? (a.plane_floats + 255) >> 8 : a.n_slabs;
    // Flow variant: the slabs go to the first waves of the workgroup only (four of them, or as many as four slabs each
    // require).  The SIMDs serve their oldest wave first, so the first waves run ahead and the last ones lag; a wave
    // without a share reports its (empty) landing on entering a block, and the block's counter no longer waits for the
    // slowest waves to be some chunks into the block before.  (Measured on the 13x13 layer with 4 rows per wave, 16
    // waves: 99.5 us with every wave staging, 98 with 12, 92.4 with 8, 91.1 with 4.)
    const int n_stagers = FLOW ? min(n_waves, max((n_slabs + 3) >> 2, 4)) : n_waves;
    unsigned voff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int slab_j = wave + j * n_stagers;
        const int f = wave >= n_stagers ? 0x40000000 : wide ? (slab_j * 64 + lane) * 4 : slab_j * 64 + lane;
        const int cell = f >> 2, img = f & 3;
        const int Y = fdiv(cell, a.d_wl), X = cell - Y * a.Wl;
        if (a.phase_stride > 1) {
            // cell (Y, X) of a phase image is element (Y*s, X*s) of the caller's plane, shifted by the phase,
            // which the scalar offset of the channel carries.  There is no padding (the host sends only unpadded
            // layers this way), and every cell a stored weight reads for a real output lies inside the image:
            // cells beyond it hold whatever follows in memory (zeros past the tensor's end, by the range check)
            // and are read only by lanes whose results are dropped.
            voff[j] = f >= a.plane_floats ? kSkipLane
                                          : (unsigned)(img * a.in_img + ((y0 + Y) * a.phase_stride * (a.src_row_bytes >> 2) + X * a.phase_stride)) * 4u;
            continue;
        }
        const int iy = y0 + Y - a.pad, ix = X - a.pad;
        const bool inside = iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
        voff[j] = f >= a.plane_floats ? kSkipLane
                  : inside            ? (unsigned)(img * a.in_img + (iy * a.W + ix) * a.in_pos) * 4u
                                      : kZeroLane;
    }
    int nslab = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) nslab += (wave < n_stagers && wave + j * n_stagers < n_slabs) ? 1 : 0;

    // the zero page behind each block buffer: cleared here, never written again
    {
        float4 *z = smem4;
        const int page4 = a.page_bytes >> 4;
        for (int b = 0; b < a.n_bufs; ++b)
            for (int i = tid; i < page4; i += blockDim.x) z[((b * a.buf_stride_bytes + a.block_bytes) >> 4) + i] = make_float4(0.f, 0.f, 0.f, 0.f);
        // A read into the right padding of a plane's last row lands on the first `pad` cells of the next
        // plane.  Staging writes zeros there (left padding), but a last block with fewer than cb channels
        // leaves the plane after its last channel unwritten: clear those cells of every plane once.
        const int per_plane = a.pad, total = a.n_bufs * a.cb * per_plane;
        for (int i = tid; i < total; i += blockDim.x) {
            const int cell = i % per_plane, pl = i / per_plane;
            const int b = pl / a.cb, cl = pl - b * a.cb;
            z[((b * a.buf_stride_bytes + cl * a.plane_bytes) >> 4) + cell] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        if (FLOW) {
            // the landing counters of this workgroup's blocks start at zero; this is the only barrier of the
            // kernel: behind it the zero pages and the counters are in place for every wave
            unsigned *ctr = reinterpret_cast<unsigned *>(reinterpret_cast<char *>(smem4) + a.ctr_bytes_at);
            for (int i = tid; i < nblk_here; i += blockDim.x) ctr[i] = 0u;
            __syncthreads();
        }
    }

    const float *in_tile = a.in + (size_t)tile * a.in_tile;
    const unsigned long long ip = (unsigned long long)in_tile;
    int4v rsrc;
    rsrc.x = __builtin_amdgcn_readfirstlane((int)(unsigned)ip);
    rsrc.y = __builtin_amdgcn_readfirstlane((int)(unsigned)(ip >> 32));   // stride 0
    rsrc.z = __builtin_amdgcn_readfirstlane((int)(a.in_rec_fixed + a.in_rec_img * nimg - a.in_rec_tile * tile)); // bytes past which loads return 0
    rsrc.w = 0x00020000;                                                   // raw 32-bit data format
    const unsigned long long op = (unsigned long long)(a.out + (size_t)split * a.split_stride + (size_t)tile * a.out_tile +
                                                       (size_t)band_i * a.out_band);
    const unsigned lim = (unsigned)(min(a.band, a.OH - y0) * a.OW * a.out_pos4);
    const unsigned ldsbase = (unsigned)(unsigned long long)(__attribute__((address_space(3))) void *)smem4;
    // cell of the plane this lane's chunk 0 sits on; chunk t is STEP cells further.  Flat: position p is
    // cell p.  Strips: lane = row * strip + column of a block of strip_rows x strip cells, the waves of a
    // column group stacked vertically; lanes outside the block or the band store nothing and read a cell of
    // the first row that falls on the same LDS banks as their own would (cell 0 for all of them costs every
    // read of the wave a bank conflict with the lane that owns that bank).
    int cell0 = cgi * T * 64 + lane;
    if (STEP != 64) {
        const int by = fdiv(lane, a.d_strip), bx = lane - by * a.strip;
        const int y = cgi * a.strip_rows + by;
        cell0 = y * a.Wl + bx;
        if (by >= a.strip_rows || y >= a.band) cell0 &= 15;
    }
    // scalar offset of the first channel this workgroup stages, and where it stands in its phase
    unsigned soff0 = (unsigned)((g * a.Cg + ch0) * a.HW4), blocks_to_wrap = 0x7fffffffu, px0 = 0;
    if (a.phase_stride > 1) {
        const int ph = fdiv(ch0, a.d_pcg), c0 = ch0 - ph * a.phase_cg, py = fdiv(ph, a.d_pstride), px = ph - py * a.phase_stride;
        soff0 = (unsigned)(g * a.phase_span_bytes + c0 * a.HW4 + py * a.src_row_bytes + px * 4);
        blocks_to_wrap = (unsigned)((a.phase_cg - c0) / a.cb);
        px0 = (unsigned)px;
    }
    const unsigned long long bias = (unsigned long long)a.bias;
    const unsigned flags = (unsigned)__builtin_amdgcn_readfirstlane((a.relu ? 1 : 0) | (wide ? 2 : 0));
    const unsigned slab_bytes = wide ? 1024u : 256u;
    Lds2Asm<T, R, STEP, FLOW>::run((unsigned long long)__builtin_amdgcn_kernarg_segment_ptr(), rsrc,
                       a.seg + ((size_t)wslot * a.nblk + blk0) * 2,
                       a.row_of + (size_t)wslot * R,
                       __builtin_amdgcn_readfirstlane((unsigned)op), __builtin_amdgcn_readfirstlane((unsigned)(op >> 32)),
                       (unsigned)__builtin_amdgcn_readfirstlane(soff0), (unsigned)nimg, lim,
                       __builtin_amdgcn_readfirstlane(ldsbase), (unsigned)wave * slab_bytes, (unsigned)n_stagers * slab_bytes,
                       (unsigned)__builtin_amdgcn_readfirstlane(nslab), (unsigned)(cell0 * 16), voff[0],
                       voff[1], voff[2], voff[3], (unsigned)((cgi * T * 64 + lane) * 4),
                       (unsigned)__builtin_amdgcn_readfirstlane(nch_here), (unsigned)__builtin_amdgcn_readfirstlane(nblk_here),
                       bias, flags, (unsigned)__builtin_amdgcn_readfirstlane(n_waves),
                       (unsigned)__builtin_amdgcn_readfirstlane(ldsbase + (unsigned)a.ctr_bytes_at),
                       (unsigned)__builtin_amdgcn_readfirstlane(blocks_to_wrap), (unsigned)__builtin_amdgcn_readfirstlane(px0));
}

// ------------------------------------------------------------------------------------------------

struct DirectArgs {
    const float *in;
    float *out;
    const int *rowptr;
    const uint32_t *trip;
    int N, C, H, W, K, OH, OW, stride, pad;
};

__global__ void __launch_bounds__(256) sconv_direct_kernel(const DirectArgs a)
{
    const int k = blockIdx.y;
    const int OHW = a.OH * a.OW;
    const long long total = (long long)a.N * OHW;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    const bool live = idx < total;
    const long long idc = live ? idx : total - 1;
    const int n = (int)(idc / OHW);
    const int rem = (int)(idc - (long long)n * OHW);
    const int oy = rem / a.OW, ox = rem - oy * a.OW;
    const int y0 = oy * a.stride, x0 = ox * a.stride;
    const float *src = a.in + (size_t)n * a.C * a.H * a.W + y0 * a.W + x0;
    float acc = 0.f;
    const int j0 = a.rowptr[k], j1 = a.rowptr[k + 1];
    for (int j = j0; j < j1; ++j) {
        const float w = __uint_as_float(a.trip[3 * (size_t)j]);
        const int goff = (int)a.trip[3 * (size_t)j + 1];
        const uint32_t rs = a.trip[3 * (size_t)j + 2];
        const int dr = (int)(short)(rs >> 16), ds = (int)(short)(rs & 0xffffu);
        const int iy = y0 + dr, ix = x0 + ds;
        const bool inside = iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
        const float v = inside ? src[goff] : 0.f;
        acc = fmaf(w, v, acc);
    }
    if (live) a.out[((size_t)n * a.K + k) * OHW + rem] = acc;
}

// ------------------------------------------------------------------------------------------------

// Scratch for the entry point that must not allocate: device memory the code object itself brings along,
// one copy per GPU the library runs on, held until the process ends.  Its name is a host-side stand-in, not
// a device address: host code only ever uses the address hipGetSymbolAddress reports for the current device.
static __device__ __align__(256) unsigned char scratch[SCONV_NOALLOC_SCRATCH_BYTES];

int static_scratch(void **base, size_t *bytes, int *hip_err)
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static void *ptr[kMaxDevices] = {};
    *base = nullptr;
    *bytes = 0;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> lock(guard);
        if (!ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e == hipSuccess && !p) e = hipErrorInvalidSymbol;
            if (e == hipSuccess) ptr[dev] = p;
        }
        if (e == hipSuccess) *base = ptr[dev];
    }
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    *bytes = SCONV_NOALLOC_SCRATCH_BYTES;
    return SCONV_OK;
}

int upload(const void *host, size_t bytes, void **dev, int *hip_err)
{
    *dev = nullptr;
    const size_t room = bytes ? bytes : 16; // keep a valid pointer for empty patterns
    hipError_t e = hipMalloc(dev, room);
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    if (host && bytes) {
        e = hipMemcpy(*dev, host, bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            *hip_err = (int)e;
            (void)hipFree(*dev);
            *dev = nullptr;
            return SCONV_ERR_HIP;
        }
    }
    return SCONV_OK;
}

void release(void *dev)
{
    if (dev) (void)hipFree(dev);
}

int timer_create(StreamTimer &t, int *hip_err)
{
    t.e0 = t.e1 = nullptr;
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) {
        e = hipEventCreate(&e1);
        if (e != hipSuccess) (void)hipEventDestroy(e0);
    }
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    t.e0 = e0;
    t.e1 = e1;
    return SCONV_OK;
}

int timer_start(StreamTimer &t, void *stream, int *hip_err)
{
    const hipError_t e = hipEventRecord(static_cast<hipEvent_t>(t.e0), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

int timer_stop_ms(StreamTimer &t, void *stream, float *ms, int *hip_err)
{
    hipError_t e = hipEventRecord(static_cast<hipEvent_t>(t.e1), static_cast<hipStream_t>(stream));
    if (e == hipSuccess) e = hipEventSynchronize(static_cast<hipEvent_t>(t.e1));
    if (e == hipSuccess) e = hipEventElapsedTime(ms, static_cast<hipEvent_t>(t.e0), static_cast<hipEvent_t>(t.e1));
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

void timer_destroy(StreamTimer &t)
{
    if (t.e0) (void)hipEventDestroy(static_cast<hipEvent_t>(t.e0));
    if (t.e1) (void)hipEventDestroy(static_cast<hipEvent_t>(t.e1));
    t.e0 = t.e1 = nullptr;
}

// A kernel may use more than 64 KB of dynamic LDS only after it has been allowed to, once per kernel and
// device.  The record of what has been allowed is the only state the library keeps outside its handles; it
// is guarded, so handles may be used from different threads.
static int allow_full_lds(const void *kern, int *hip_err)
{
    static std::mutex guard;
    static std::set<std::pair<const void *, int>> allowed;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> lock(guard);
        if (allowed.count({kern, dev})) return SCONV_OK;
        e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess) allowed.insert({kern, dev});
    }
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

template <int VEC, int T, int ROWS_W>
static int launch_lds_inst(const LdsArgs &a, int grid, int threads, int lds_bytes, hipStream_t s, int *hip_err)
{
    auto kern = sconv_lds_kernel<VEC, T, ROWS_W>;
    const int rc = allow_full_lds(reinterpret_cast<const void *>(kern), hip_err);
    if (rc) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds_bytes, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

#define SCONV_SHAPES_V1(X) \
    X(1, 1, 16) X(1, 2, 16) X(1, 3, 8) X(1, 3, 16) X(1, 4, 8) X(1, 7, 8) X(1, 13, 4) X(1, 14, 4)

int launch_lds(const sconv_desc &d, const LdsTiling &t, const DeviceLds &dev, const float *in, float *out,
               int N, void *stream, int *hip_err)
{
    const Geometry g = geometry(d);
    LdsArgs a;
    a.in = in;
    a.out = out;
    a.pairs = static_cast<const unsigned *>(dev.pairs);
    a.seg_ptr = static_cast<const int *>(dev.seg_ptr);
    a.row_of = static_cast<const int *>(dev.row_of);
    a.N = N; a.C = d.C; a.H = d.H; a.W = d.W; a.K = d.K; a.OH = g.OH; a.OW = g.OW; a.pad = d.pad;
    a.Cg = g.Cg; a.groups = d.groups;
    a.nt = t.p.nt; a.cb = t.p.cb; a.nblk = t.nblk; a.rg = t.rg; a.cg = t.p.cg; a.nkt = t.nkt;
    a.band = t.p.band; a.n_bands = t.n_bands;
    a.Wl = t.Wl; a.plane_floats = t.plane_cells * t.p.nt; a.n_slabs = t.n_slabs;
    a.buf_stride_floats = t.buf_stride_floats;
    a.lds_floats = t.lds_bytes / 4;
    a.n_tiles = (N + t.p.nt - 1) / t.p.nt;
    a.units = d.groups * t.nkt * t.n_bands;
    // the kernel's own assumptions, checked before anything is launched
    if ((t.n_slabs + t.p.waves - 1) / t.p.waves > kMaxSlabsPerWave) return SCONV_ERR_PLAN;
    if ((int64_t)t.p.nt * d.C * d.H * d.W >= ((int64_t)1 << 29)) return SCONV_ERR_RANGE;
    if (t.lds_bytes % 16 || t.lds_bytes > 160 * 1024) return SCONV_ERR_PLAN;
    const int64_t grid64 = (int64_t)a.n_tiles * a.units;
    if (grid64 > 0x7fffffff) return SCONV_ERR_RANGE;
    const int grid = (int)grid64, threads = t.p.waves * 64;
    hipStream_t s = static_cast<hipStream_t>(stream);
#define X(V, TT, RW) \
    if (t.vec == V && t.p.t == TT && t.p.rows_w == RW) return launch_lds_inst<V, TT, RW>(a, grid, threads, t.lds_bytes, s, hip_err);
    SCONV_SHAPES_V1(X)
#undef X
#define X(TT, RW) \
    if (t.vec == 4 && t.p.t == TT && t.p.rows_w == RW) return launch_lds_inst<4, TT, RW>(a, grid, threads, t.lds_bytes, s, hip_err);
    SCONV_ASM_SHAPES(X)
#undef X
    return SCONV_ERR_PLAN;
}

template <int T, int R, int STEP, bool FLOW>
static int launch_lds2_inst(const Lds2Args &a, int grid, int threads, int lds_bytes, hipStream_t s, int *hip_err)
{
    auto kern = sconv_lds2_kernel<T, R, STEP, FLOW>;
    const int rc = allow_full_lds(reinterpret_cast<const void *>(kern), hip_err);
    if (rc) return rc;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds_bytes, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

bool lds2_kernel_available(int t, int rows_w, int step)
{
#define X(TT, RW, ST) if (t == TT && rows_w == RW && step == ST) return true;
    SCONV_LDS2_SHAPES(X)
#undef X
    return false;
}

int lds2_flow_bufs() { return SCONV_LDS2_FLOW_BUFS; }

int lds2_depth(int t, int rows_w)
{
#define X(TT, RW, ST) if (t == TT && rows_w == RW && ST == 64) return Lds2Asm<TT, RW, ST, false>::kDepth;
    SCONV_LDS2_SHAPES(X)
#undef X
    return 0;
}

// Elementwise passes around the kernels that cannot fuse them.
__global__ void __launch_bounds__(256) sconv_epilogue_kernel(float *out, const float *bias, int relu, long long inner, int K, long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float v = out[i];
    if (bias) v += bias[(int)((i / inner) % K)];
    if (relu) v = fmaxf(v, 0.f);
    out[i] = v;
}

// out = sum of the parts' partial results (+ bias, ReLU): four floats per thread where the alignment allows.
__global__ void __launch_bounds__(256) sconv_reduce_kernel(const float *parts, float *out, int splits, long long total,
                                                           long long inner, int K, const float *bias, int relu)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    float v = 0.f;
    for (int s2 = 0; s2 < splits; ++s2) v += parts[(long long)s2 * total + i];
    if (bias) v += bias[(int)((i / inner) % K)];
    if (relu) v = fmaxf(v, 0.f);
    out[i] = v;
}

int launch_epilogue(float *out, int64_t rows, int64_t inner, int K, const Epilogue &ep, void *stream, int *hip_err)
{
    if (!ep.bias && !ep.relu) return SCONV_OK;
    const int64_t total = rows * inner, gx = (total + 255) / 256;
    if (gx > 0x7fffffff) return SCONV_ERR_RANGE;
    hipLaunchKernelGGL(sconv_epilogue_kernel, dim3((unsigned)gx), dim3(256), 0, static_cast<hipStream_t>(stream), out, ep.bias,
                       ep.relu ? 1 : 0, (long long)inner, K, (long long)total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

// The same, four outputs per thread, for rows whose length is a multiple of 4 (a float4 then lies in one row):
// the parts are added in the same order, so the results are the scalar kernel's bit for bit.
__global__ void __launch_bounds__(256) sconv_reduce4_kernel(const float4 *parts, float4 *out, int splits, long long total4,
                                                            long long inner4, int K, const float *bias, int relu)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total4) return;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s2 = 0; s2 < splits; ++s2) {
        const float4 p = parts[(long long)s2 * total4 + i];
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (bias) {
        const float b = bias[(int)((i / inner4) % K)];
        v.x += b; v.y += b; v.z += b; v.w += b;
    }
    if (relu) {
        v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
    }
    out[i] = v;
}

int launch_reduce(const float *parts, float *out, int splits, int64_t rows, int64_t inner, int K, const Epilogue &ep,
                  void *stream, int *hip_err)
{
    const int64_t total = rows * inner;
    const bool by4 = inner % 4 == 0 && ((uintptr_t)out & 15) == 0 && ((uintptr_t)parts & 15) == 0;
    const int64_t gx = ((by4 ? total / 4 : total) + 255) / 256;
    if (gx > 0x7fffffff) return SCONV_ERR_RANGE;
    if (by4)
        hipLaunchKernelGGL(sconv_reduce4_kernel, dim3((unsigned)gx), dim3(256), 0, static_cast<hipStream_t>(stream),
                           reinterpret_cast<const float4 *>(parts), reinterpret_cast<float4 *>(out), splits, (long long)(total / 4),
                           (long long)(inner / 4), K, ep.bias, ep.relu ? 1 : 0);
    else
        hipLaunchKernelGGL(sconv_reduce_kernel, dim3((unsigned)gx), dim3(256), 0, static_cast<hipStream_t>(stream), parts, out, splits,
                           (long long)total, (long long)inner, K, ep.bias, ep.relu ? 1 : 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

Lds2Layout nchw_layout(const sconv_desc &d, const LdsTiling &t)
{
    const Geometry g = geometry(d);
    Lds2Layout l;
    const int64_t HW = (int64_t)d.H * d.W, OHW = (int64_t)g.OH * g.OW;
    l.in_img = d.C * HW; l.in_tile = 4 * l.in_img; l.in_ch = HW; l.in_pos = 1;
    l.in_rec_fixed = 0; l.in_rec_img = l.in_img * 4; l.in_rec_tile = 0;
    l.out_img = d.K * OHW; l.out_tile = 4 * l.out_img; l.out_band = (int64_t)t.p.band * g.OW; l.out_row = OHW; l.out_pos = 1;
    return l;
}

int launch_lds2(const sconv_desc &d, const LdsTiling &t, const DeviceLds &dev, const Lds2Layout &lay, const float *in,
                float *out, int N, const Epilogue &ep, int64_t split_stride, void *stream, int *hip_err)
{
    const Geometry g = geometry(d);
    Lds2Args a;
    a.in = in;
    a.out = out;
    a.pairs = static_cast<const unsigned *>(dev.pairs);
    a.seg = static_cast<const unsigned *>(dev.seg_ptr);
    a.row_of = static_cast<const int *>(dev.row_of);
    a.store_tbl = static_cast<const int *>(dev.store_tbl);
    const int plane_floats = t.plane_cells * 4;
    a.cb = t.p.cb; a.nblk = t.nblk; a.Cg = g.Cg; a.plane_bytes = plane_floats * 4;
    a.buf_stride_bytes = t.buf_stride_floats * 4;
    a.N = N; a.C = d.C; a.H = d.H; a.W = d.W; a.K = d.K; a.OH = g.OH; a.OW = g.OW; a.pad = d.pad;
    a.rg = t.rg; a.cg = t.p.cg; a.nkt = t.nkt; a.band = t.p.band; a.n_bands = t.n_bands; a.Wl = t.Wl;
    a.plane_floats = plane_floats; a.n_slabs = t.n_slabs;
    a.n_tiles = (N + 3) / 4;
    a.splits = std::max(1, t.p.splits);
    a.blk_split = (t.nblk + a.splits - 1) / a.splits;
    if ((a.splits - 1) * a.blk_split >= t.nblk) return SCONV_ERR_PLAN; // a part without blocks
    a.units = d.groups * t.nkt * t.n_bands * a.splits;
    a.block_bytes = (int)t.zero_page;
    a.page_bytes = t.page_cells * 16;
    a.strip = t.p.strip; a.strip_rows = t.strip_rows;
    a.n_bufs = t.n_bufs;
    a.ctr_bytes_at = t.ctr_bytes_at;
    a.blocks_per_phase = 0x7fffffff; a.phase_stride = 1; a.src_row_bytes = 0; a.phase_span_bytes = 0; a.phase_cg = 0;
    a.d_pcg = make_fastdiv(1, 1); a.d_pstride = make_fastdiv(1, 1);
    if (lay.phase_stride > 1) {
        // d is the stride-1 form of the layer; the caller's tensor has C / s^2 channels of lay.in_ch floats
        if (t.phase_cg <= 0 || t.phase_cg % t.p.cb || d.pad != 0 || lay.in_pos != 1 || lay.src_w <= 0) return SCONV_ERR_PLAN;
        if (g.Cg != t.phase_cg * lay.phase_stride * lay.phase_stride) return SCONV_ERR_PLAN;
        a.phase_stride = lay.phase_stride;
        a.blocks_per_phase = t.phase_cg / t.p.cb;
        a.src_row_bytes = lay.src_w * 4;
        a.phase_span_bytes = (int)(t.phase_cg * lay.in_ch * 4);
        a.phase_cg = t.phase_cg;
        a.d_pcg = make_fastdiv(t.phase_cg, g.Cg);
        a.d_pstride = make_fastdiv(lay.phase_stride, lay.phase_stride * lay.phase_stride);
    }
    // a cell per lane instead of a float per lane where a cell's four images are 16 adjacent, aligned bytes and
    // no lane needs the zero fill of the padding
    a.wide = (lay.phase_stride == 1 && d.pad == 0 && lay.in_pos == 4 && lay.in_img == 1 && lay.in_ch % 4 == 0 && lay.in_tile % 4 == 0 &&
              reinterpret_cast<uintptr_t>(in) % 16 == 0 && N % 4 == 0) ? 1 : 0;
    // with several parts the kernel stores partial sums into the workspace `out` points to, part after part,
    // and the reduction that follows applies the epilogue
    a.split_stride = a.splits > 1 ? split_stride : 0;
    a.bias = a.splits == 1 ? ep.bias : nullptr;
    a.relu = (ep.relu && a.splits == 1) ? 1 : 0;
    // offsets the kernel keeps in 32 bits
    const int64_t lim32 = (int64_t)1 << 31;
    if (lay.in_img * 4 * 4 >= lim32 || lay.in_ch * 4 >= lim32 || lay.in_pos * 4 * d.H * d.W >= lim32) return SCONV_ERR_RANGE;
    if ((int64_t)d.C * lay.in_ch * 4 + 3 * lay.in_img * 4 >= lim32) return SCONV_ERR_RANGE;   // buffer offsets below 2^31 bytes
    if (lay.out_row * 4 >= lim32 || lay.out_img * 4 >= lim32 || lay.out_band >= lim32) return SCONV_ERR_RANGE;
    if ((int64_t)t.p.band * g.OW * lay.out_pos * 4 >= lim32) return SCONV_ERR_RANGE;
    a.in_tile = lay.in_tile; a.in_img = (int)lay.in_img; a.in_pos = (int)lay.in_pos; a.HW4 = (int)(lay.in_ch * 4);
    if (lay.in_rec_fixed + 4 * lay.in_rec_img >= lim32) return SCONV_ERR_RANGE;
    a.in_rec_fixed = lay.in_rec_fixed; a.in_rec_img = lay.in_rec_img; a.in_rec_tile = lay.in_rec_tile;
    if (lay.in_rec_fixed - lay.in_rec_tile * (a.n_tiles - 1) < 0) return SCONV_ERR_RANGE;
    a.out_tile = lay.out_tile; a.out_band = (int)lay.out_band; a.OHW4 = (int)(lay.out_row * 4);
    a.out_pos4 = (int)(lay.out_pos * 4);
    // what the kernel assumes, checked before anything is launched
    if (t.p.nt != 4 || t.vec != 4) return SCONV_ERR_PLAN;
    if ((t.n_slabs + t.p.waves - 1) / t.p.waves > 4) return SCONV_ERR_PLAN;
    if (t.lds_bytes % 16 || t.lds_bytes > 160 * 1024 || a.block_bytes % 16 || a.buf_stride_bytes % 16) return SCONV_ERR_PLAN;
    if (a.block_bytes + a.page_bytes > a.buf_stride_bytes) return SCONV_ERR_PLAN;
    if ((int64_t)a.buf_stride_bytes * t.n_bufs > t.lds_bytes) return SCONV_ERR_PLAN;
    if (t.p.rows_w * t.p.t * 4 > 256) return SCONV_ERR_PLAN;
    a.img_stride_bytes = (int)(lay.out_img * 4);
    const int64_t grid64 = (int64_t)a.n_tiles * a.units;
    if (grid64 > 0x7fffffff) return SCONV_ERR_RANGE;
    const int grid = (int)grid64, threads = t.p.waves * 64;
    // the largest dividend of each division in the kernel's index arithmetic
    a.d_units = make_fastdiv(a.units, grid64);
    a.d_splits = make_fastdiv(a.splits, a.units);
    a.d_bands = make_fastdiv(a.n_bands, a.units);
    a.d_nkt = make_fastdiv(a.nkt, a.units);
    a.d_cg = make_fastdiv(a.cg, 16);
    a.d_wl = make_fastdiv(a.Wl, (int64_t)4 * threads * 64);     // cells of the slabs a workgroup can stage
    a.d_strip = make_fastdiv(std::max(1, a.strip), 64);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int step = t.p.strip ? t.p.strip : 64;
    if (t.p.strip && (t.strip_rows < 1 || t.strip_rows * t.p.strip > 64 || t.p.band > t.p.cg * t.strip_rows)) return SCONV_ERR_PLAN;
    const bool flow = t.p.kernel == 4;
    if (flow != (t.ctr_bytes_at > 0) || (flow && t.ctr_bytes_at + 4 * t.nblk > t.lds_bytes)) return SCONV_ERR_PLAN;
    if (t.n_bufs != std::min(flow ? SCONV_LDS2_FLOW_BUFS : 2, t.nblk)) return SCONV_ERR_PLAN;
#define X(TT, RW, ST) \
    if (t.p.t == TT && t.p.rows_w == RW && step == ST) \
        return flow ? launch_lds2_inst<TT, RW, ST, true>(a, grid, threads, t.lds_bytes, s, hip_err) \
                    : launch_lds2_inst<TT, RW, ST, false>(a, grid, threads, t.lds_bytes, s, hip_err);
    SCONV_LDS2_SHAPES(X)
#undef X
    return SCONV_ERR_PLAN;
}

// Phase images of a strided layer: q[n][virtual channel of (c, py, px)][Y][X] = in_pad[n][c][Y*s + py][X*s + px], the
// zero padding written out.  One thread per element of q; consecutive threads write consecutive X.
struct PhaseArgs {
    const float *in;
    float *q;
    int C, Cg, H, W, s, pad, Hq, Wq;
    long long total;
};

__global__ void __launch_bounds__(256) sconv_phase_kernel(const PhaseArgs a)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.total) return;
    const int X = (int)(idx % a.Wq);
    long long rest = idx / a.Wq;
    const int Y = (int)(rest % a.Hq);
    rest /= a.Hq;
    const int cv = (int)(rest % (a.C * a.s * a.s));
    const long long n = rest / (a.C * a.s * a.s);
    // virtual channels run group by group, inside a group phase by phase, inside a phase over the group's channels
    const int per_group = a.Cg * a.s * a.s, grp = cv / per_group, rem = cv - grp * per_group;
    const int ph = rem / a.Cg, c = grp * a.Cg + rem - ph * a.Cg, py = ph / a.s, px = ph - py * a.s;
    const int iy = Y * a.s + py - a.pad, ix = X * a.s + px - a.pad;
    float v = 0.f;
    if (iy >= 0 && iy < a.H && ix >= 0 && ix < a.W) v = a.in[((n * a.C + c) * a.H + iy) * a.W + ix];
    a.q[idx] = v;
}

int launch_phase(const sconv_desc &d, const sconv_desc &v, const float *in, float *q, int N, void *stream, int *hip_err)
{
    PhaseArgs a;
    a.in = in;
    a.q = q;
    a.C = d.C; a.Cg = d.C / d.groups; a.H = d.H; a.W = d.W; a.s = d.stride; a.pad = d.pad; a.Hq = v.H; a.Wq = v.W;
    a.total = (long long)N * v.C * v.H * v.W;
    const long long gx = (a.total + 255) / 256;
    if (gx > 0x7fffffff) return SCONV_ERR_RANGE;
    hipLaunchKernelGGL(sconv_phase_kernel, dim3((unsigned)gx), dim3(256), 0, static_cast<hipStream_t>(stream), a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

int launch_direct(const sconv_desc &d, const DeviceDirect &dev, const float *in, float *out, int N,
                  void *stream, int *hip_err)
{
    const Geometry g = geometry(d);
    DirectArgs a;
    a.in = in;
    a.out = out;
    a.rowptr = static_cast<const int *>(dev.rowptr);
    a.trip = static_cast<const uint32_t *>(dev.trip);
    a.N = N; a.C = d.C; a.H = d.H; a.W = d.W; a.K = d.K; a.OH = g.OH; a.OW = g.OW; a.stride = d.stride; a.pad = d.pad;
    const int64_t total = (int64_t)N * g.OH * g.OW;
    const int64_t gx = (total + 255) / 256;
    if (gx > 0x7fffffff || d.K > 65535) return SCONV_ERR_RANGE;
    hipLaunchKernelGGL(sconv_direct_kernel, dim3((unsigned)gx, (unsigned)d.K), dim3(256), 0, static_cast<hipStream_t>(stream), a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        *hip_err = (int)e;
        return SCONV_ERR_HIP;
    }
    return SCONV_OK;
}

} // namespace sconv
