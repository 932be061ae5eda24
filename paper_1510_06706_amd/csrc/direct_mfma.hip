// Direct method on the fp32 matrix cores: forward and backward pass as an
// implicit GEMM whose reduction runs over (fan-in x kernel volume), i.e. the
// sum over the edges converging on a node is part of the GEMM's K loop.  The
// kernel is in direct_mfma_impl.h; this file holds the weight packer, the
// search for the workgroup's output box and the launch.  The backward pass is
// the same contraction with the roles of the two node sets swapped, the kernel
// reflected and the output gradient zero-extended by k-1 on every side
// (Section 3.1), which the halo loader and the weight packer provide; no
// separate kernel is needed.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "direct_mfma_tail_impl.h"

namespace znn {

namespace {

using conv::ConvFn;
using conv::ConvTile;

constexpr int kMaxTaps = 4096;

// Packs w[f'][f][k] for the kernel of direct_mfma_tail_impl.h: per (map group, chunk, tap) the NJ x 64 operands of
// the full tiles (lane l of tile jt: output-side map jt*16 + l%16, input-side map chunk*4 + l/16), then, with
// `tail`, [8 maps][4 input maps] for the 8-map block.  For the backward pass the two map indices trade places
// and the tap is reflected.
__global__ void __launch_bounds__(256)
k_pack_weights_tail(const float* __restrict__ w, float* __restrict__ wp, int f, int fo, int kz, int ky, int kx,
                    int backward, int NJ, int jgroups, int nchunk, int tail)
{
    const int taps = kz * ky * kx;
    const int WT = NJ * 64 + (tail ? conv::kTailPacked : 0);
    const long total = (long)jgroups * nchunk * taps * WT;
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int e = (int)(t % WT);
    long r = t / WT;
    const int tap = (int)(r % taps); r /= taps;
    const int ic = (int)(r % nchunk);
    const int jg = (int)(r / nchunk);
    int m, k;
    if (e < NJ * 64) {
        m = (jg * NJ + e / 64) * 16 + (e & 15);
        k = ic * 4 + ((e & 63) >> 4);
    } else {
        m = NJ * 16 + (e - NJ * 64) / 4;
        k = ic * 4 + (e & 3);
    }
    const int fM = backward ? f : fo, fK = backward ? fo : f;
    float v = 0.f;
    if (m < fM && k < fK) {
        if (!backward) {
            v = w[((long)m * f + k) * taps + tap];
        } else {
            const int c = tap % kx, b = (tap / kx) % ky, a = tap / (kx * ky);
            const int rt = ((kz - 1 - a) * ky + (ky - 1 - b)) * kx + (kx - 1 - c);
            v = w[((long)k * f + m) * taps + rt];
        }
    }
    wp[t] = v;
}

__global__ void __launch_bounds__(256)
k_conv_reduce(const float* __restrict__ partial, float* __restrict__ dst, long count, int splits)
{
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= count) return;
    float acc = partial[t];
    for (int s = 1; s < splits; ++s) acc += partial[(long)s * count + t];
    dst[t] = acc;
}

// Taps along x are walked in groups of U (direct_mfma_impl.h): the widest divisor of the
// kernel width that has an instance; 1 for sparse taps.
int group_width(int kx, int spx)
{
    if (tuning().conv_u1 || spx != 1) return 1;
    const int widths[6] = {11, 7, 5, 4, 3, 2};
    for (int i = 0; i < 6; ++i)
        if (kx % widths[i] == 0) return widths[i];
    return 1;
}

ConvFn pick_tail_kernel(int U, int nj, int nv, bool wl)
{
    switch (U) {
        case 1: return conv_tail_kernel_u1(nj, nv, wl);
        case 2: return conv_tail_kernel_u2(nj, nv, wl);
        case 3: return conv_tail_kernel_u3(nj, nv, wl);
        case 4: return conv_tail_kernel_u4(nj, nv, wl);
        case 5: return conv_tail_kernel_u5(nj, nv, wl);
        case 7: return conv_tail_kernel_u7(nj, nv, wl);
        case 11: return conv_tail_kernel_u11(nj, nv, wl);
    }
    return nullptr;
}

// The last 1..8 of the output-side maps as an 8-map block instead of a padded 16-row tile: one
// workgroup must hold all maps, and a lane's byte offset over the chunk's four source maps must fit
// 32 bits.
bool tail_applies(int fM, long svol)
{
    const int r = fM % 16;
    return !tuning().conv_no_tail && fM > 16 && fM / 16 <= 7 && r >= 1 && r <= conv::kTailMaps && svol * 16 < (1L << 32);
}

ConvFn pick_plain_kernel(int U, int nj, int nv, bool wl)
{
    switch (U) {
        case 1: return conv_plain_kernel_u1(nj, nv, wl);
        case 2: return conv_plain_kernel_u2(nj, nv, wl);
        case 3: return conv_plain_kernel_u3(nj, nv, wl);
        case 4: return conv_plain_kernel_u4(nj, nv, wl);
        case 5: return conv_plain_kernel_u5(nj, nv, wl);
        case 7: return conv_plain_kernel_u7(nj, nv, wl);
        case 11: return conv_plain_kernel_u11(nj, nv, wl);
    }
    return nullptr;
}

// Weights of one chunk in LDS: when they take at most 32 KiB.
bool weights_in_lds(int taps, int NJ, bool tail)
{
    return !tuning().conv_no_wl && (size_t)taps * (NJ * 64 + (tail ? conv::kTailPacked : 0)) * 4 <= 32 * 1024;
}

struct TileChoice {
    bool ok;
    int NJ, jgroups, NV;
    int Tz, Ty, Tx, HZ, HY, HX, MS;
    int cz, cy, cx;
    bool wl, dbuf;
    bool tail;          // NJ full tiles and an 8-map block (direct_mfma_tail_impl.h)
    int cps, splits;    // input-map chunks per workgroup and number of such shares
    size_t lds;
};

constexpr int kCUs = 256;
constexpr size_t kConvLdsMax = 64 * 1024;

// A layer with few output voxels leaves most compute units without a workgroup (and the rest
// with one wave per SIMD): below one workgroup per unit the input-map chunks are split over
// gridDim.z until about three per unit exist; the shares' partial sums are added in a fixed
// order afterwards.
void split_chunks(long blocks, int nchunk, int& cps, int& splits)
{
    long want = tuning().conv_no_split || blocks >= kCUs ? 1 : (3 * kCUs + blocks - 1) / blocks;
    if (want > nchunk) want = nchunk;
    cps = (int)(nchunk / want);        // rounded down: shares of equal length, a few more of them
    splits = (nchunk + cps - 1) / cps;
}

// Picks the tile box and the per-wave tile count so that the launch fills the
// 256 compute units in as few, as full rounds as possible.
TileChoice search_tile(int fM, int fK, int dz, int dy, int dx, int kz, int ky, int kx, int spz, int spy, int spx, bool tail)
{
    TileChoice best = {};
    best.ok = false;
    const int taps = kz * ky * kx;
    if (taps > kMaxTaps) return best;
    const int tiles = (fM + 15) / 16;
    const int jgroups = tail ? 1 : (tiles + 7) / 8;
    const int NJ = tail ? fM / 16 : (tiles + jgroups - 1) / jgroups;
    double best_cost = 1e300;
    const int nchunk = (fK + 3) / 4;
    // tuning aid: ZNN_CONV_TILE="NV,Tz,Ty,Tx" pins the configuration
    const int (&pin)[4] = tuning().conv_tile;
    const int nvs[6] = {2, 4, 5, 6, 7, 8};
    for (int ni = 0; ni < 6; ++ni) {
        const int NV = nvs[ni];
        if (tail ? !conv::tail_instance(NJ, NV) : !conv::plain_instance(NJ, NV)) continue;
        if (pin[0] && NV != pin[0]) continue;
        const int cap = 64 * NV;
        for (int Tx = 1; Tx <= dx && Tx <= cap; ++Tx) {
            for (int Ty = 1; Ty <= dy && Tx * Ty <= cap; ++Ty) {
                int Tz = cap / (Tx * Ty);
                if (Tz > dz) Tz = dz;
                if (Tz < 1) continue;
                if (pin[0]) {
                    if (Tx != pin[3] || Ty != pin[2] || pin[1] * Ty * Tx > cap) continue;
                    Tz = pin[1];
                }
                const int HZ = Tz + spz * (kz - 1), HY = Ty + spy * (ky - 1), HX = Tx + spx * (kx - 1);
                long hvol = (long)HZ * HY * HX;
                long MS = hvol;
                MS = (MS + 15) & ~15L;      // whole 64-word spans of 16 voxels x 4 maps
                const bool wl = weights_in_lds(taps, NJ, tail);
                // halo buffers (two that take turns if they fit, else one), the loader's table (one
                // map's box, padded to the workgroup size), the chunk's weights
                const long MSP = (MS + 255) & ~255L;
                const size_t wbytes = wl ? (size_t)taps * (NJ * 64 + (tail ? conv::kTailPacked : 0)) * 4 : 0;
                bool dbuf = true;
                size_t lds = (size_t)(8 * MS + MSP) * 4 + wbytes;
                if (lds > kConvLdsMax) { dbuf = false; lds = (size_t)(4 * MS + MSP) * 4 + wbytes; }
                if (lds > kConvLdsMax) continue;
                const int cz = (dz + Tz - 1) / Tz, cy = (dy + Ty - 1) / Ty, cx = (dx + Tx - 1) / Tx;
                const long blocks = (long)cz * cy * cx * jgroups;
                // shares of the input maps along gridDim.z when the output gives few workgroups (see below)
                int cps, splits;
                split_chunks(blocks, nchunk, cps, splits);
                // time ~ workgroups per compute unit (they share its matrix cores whether they run side
                // by side or one after the other) x (fixed cost of a workgroup + its chunks x (MFMA work +
                // halo fetch)); a unit with a single workgroup has one wave per SIMD and nothing to overlap
                // its waits with (measured on the 2D benchmark layer: 1.4x)
                const long groups = blocks * splits;
                const double rounds = (double)((groups + kCUs - 1) / kCUs) * (groups <= kCUs ? 1.4 : 1.0);
                // an 8-map block costs four short MFMAs per two voxel tiles (about 10 cycles each)
                const double mfma = (double)taps * (NJ * NV * 32.0 + (tail ? ((NV + 1) / 2) * 40.0 : 0.0));
                // halo fetch per chunk: hidden behind the taps with two buffers, else one exposed memory latency
                const double stage = dbuf ? 300.0 + (double)hvol * 4.0 / 256.0 * 2.0 : 1500.0 + (double)hvol * 4.0 / 256.0 * 6.0;
                const double fixed = 3000.0 + (double)MS / 256.0 * 300.0;      // launch, table, zero fill, epilogue
                // among boxes of equal cost the one that is longest along x: longer contiguous runs in the
                // epilogue's stores and in the halo fetch (config 2: 12x6x6 -> 6x6x12, 2 % faster)
                const double cost = rounds * (fixed + cps * (mfma + stage)) - 0.01 * Tx;
                if (cost < best_cost) {
                    best_cost = cost;
                    best.ok = true;
                    best.NJ = NJ; best.jgroups = jgroups; best.NV = NV;
                    best.Tz = Tz; best.Ty = Ty; best.Tx = Tx;
                    best.HZ = HZ; best.HY = HY; best.HX = HX; best.MS = (int)MS;
                    best.cz = cz; best.cy = cy; best.cx = cx;
                    best.wl = wl;
                    best.dbuf = dbuf;
                    best.tail = tail;
                    best.cps = cps; best.splits = splits;
                    best.lds = lds;
                }
            }
        }
    }
    return best;
}

// The search walks thousands of candidate boxes (a fraction of a millisecond on the host),
// and every call of a pass asks for the same answer up to three times: remembered per shape.
TileChoice choose_tile(int fM, int fK, int dz, int dy, int dx, int kz, int ky, int kx, int spz, int spy, int spx, long svol)
{
    struct Entry { int key[12]; TileChoice choice; };
    static std::mutex lock;
    static std::vector<Entry> memo;
    const bool tail = tail_applies(fM, svol);
    const int key[12] = {fM, fK, dz, dy, dx, kz, ky, kx, spz, spy, spx, tail ? 1 : 0};
    {
        std::lock_guard<std::mutex> hold(lock);
        for (const Entry& e : memo)
            if (memcmp(e.key, key, sizeof(key)) == 0) return e.choice;
    }
    Entry e;
    memcpy(e.key, key, sizeof(key));
    e.choice = search_tile(fM, fK, dz, dy, dx, kz, ky, kx, spz, spy, spx, tail);
    if (tail && !e.choice.ok) e.choice = search_tile(fM, fK, dz, dy, dx, kz, ky, kx, spz, spy, spx, false);
    std::lock_guard<std::mutex> hold(lock);
    if (memo.size() >= 256) memo.erase(memo.begin());
    memo.push_back(e);
    return e.choice;
}

size_t partial_bytes(const TileChoice& c, int fM, long dvol)
{
    return c.splits > 1 ? align256((size_t)c.splits * fM * dvol * sizeof(float)) : 0;
}

size_t packed_bytes(const TileChoice& c, int fK, int taps)
{
    const size_t per_tap = (size_t)c.NJ * 64 + (c.tail ? conv::kTailPacked : 0);
    return align256((size_t)c.jgroups * ((fK + 3) / 4) * taps * per_tap * sizeof(float));
}

TileChoice choose_for(const Geom& g, bool backward)
{
    return backward ? choose_tile(g.f, g.fo, g.nz, g.ny, g.nx, g.kz, g.ky, g.kx, g.spz, g.spy, g.spx, g.ovol())
                    : choose_tile(g.fo, g.f, g.oz, g.oy, g.ox, g.kz, g.ky, g.kx, g.spz, g.spy, g.spx, g.nvol());
}

}  // namespace

// The tiled path takes every shape whose halo box fits LDS; otherwise the caller falls back.
bool mfma_conv_supported(const Geom& g, bool backward)
{
    const TileChoice c = choose_for(g, backward);
    const long svol = backward ? g.ovol() : g.nvol();
    // the halo loader addresses the chunk's four source maps with one 32-bit byte offset
    return c.ok && svol < (1L << 28);
}

size_t mfma_conv_workspace(const Geom& g, bool backward)
{
    const TileChoice c = choose_for(g, backward);
    if (!c.ok) return 0;
    return packed_bytes(c, backward ? g.fo : g.f, (int)g.kvol()) +
           partial_bytes(c, backward ? g.f : g.fo, backward ? g.nvol() : g.ovol());
}

int mfma_conv(const Geom& g, bool backward, const float* src, const float* w, float* dst, void* ws,
              hipStream_t s)
{
    ConvTile P = {};
    P.src = src; P.dst = dst;
    P.kz = g.kz; P.ky = g.ky; P.kx = g.kx;
    P.spz = g.spz; P.spy = g.spy; P.spx = g.spx;
    if (!backward) {
        P.fK = g.f; P.fM = g.fo;
        P.sz = g.nz; P.sy = g.ny; P.sx = g.nx;
        P.pz = P.py = P.px = 0;
        P.dz = g.oz; P.dy = g.oy; P.dx = g.ox;
    } else {
        P.fK = g.fo; P.fM = g.f;
        P.sz = g.oz; P.sy = g.oy; P.sx = g.ox;
        P.pz = g.spz * (g.kz - 1); P.py = g.spy * (g.ky - 1); P.px = g.spx * (g.kx - 1);
        P.dz = g.nz; P.dy = g.ny; P.dx = g.nx;
    }
    const TileChoice c = choose_for(g, backward);
    if (!c.ok) return fail(ZNN_EUNSUPPORTED, "no tile configuration fits this shape");
    P.Tz = c.Tz; P.Ty = c.Ty; P.Tx = c.Tx;
    P.HZ = c.HZ; P.HY = c.HY; P.HX = c.HX; P.MS = c.MS;
    P.dHX = make_fastdiv((unsigned)c.HX); P.dHY = make_fastdiv((unsigned)c.HY); P.dHZ = make_fastdiv((unsigned)c.HZ);
    P.cz = c.cz; P.cy = c.cy; P.cx = c.cx;
    P.nchunk = (P.fK + 3) / 4;
    P.cps = c.cps;
    P.dbuf = c.dbuf ? 1 : 0;
    if (log_enabled())
        fprintf(stderr, "[znn] conv mfma (%s): NJ=%d%s jgroups=%d NV=%d U=%d tile=%dx%dx%d halo=%dx%dx%d blocks=%d splits=%d lds=%zu buffers=%d\n",
                backward ? "bwd" : "fwd", c.NJ, c.tail ? "+8" : "", c.jgroups, c.NV, group_width(g.kx, g.spx), c.Tz, c.Ty, c.Tx, c.HZ, c.HY, c.HX,
                c.cz * c.cy * c.cx, c.splits, c.lds, c.dbuf ? 2 : 1);
    const int taps = (int)g.kvol();
    float* wp = (float*)ws;
    P.wp = wp;
    P.partial = (float*)((char*)ws + packed_bytes(c, P.fK, taps));
    {
        const long total = (long)c.jgroups * P.nchunk * taps * (c.NJ * 64 + (c.tail ? conv::kTailPacked : 0));
        ZNN_LAUNCH("weight packing", s, k_pack_weights_tail, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                   w, wp, g.f, g.fo, g.kz, g.ky, g.kx, backward ? 1 : 0, c.NJ, c.jgroups, P.nchunk, c.tail ? 1 : 0);
    }
    int rc = check_launch("weight packing");
    if (rc != ZNN_OK) return rc;
    const int U = group_width(g.kx, g.spx);
    ConvFn fn = c.tail ? pick_tail_kernel(U, c.NJ, c.NV, c.wl) : pick_plain_kernel(U, c.NJ, c.NV, c.wl);
    if (!fn) return fail(ZNN_EUNSUPPORTED, "no kernel instance for tile %dx%d", c.NJ, c.NV);
    const long blocks = (long)c.cz * c.cy * c.cx;
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many tiles for one launch");
    ZNN_LAUNCH(backward ? "direct backward (MFMA)" : "direct forward (MFMA)", s, fn,
               dim3((unsigned)blocks, (unsigned)c.jgroups, (unsigned)c.splits), dim3(256), c.lds, P);
    rc = check_launch(backward ? "direct backward (MFMA)" : "direct forward (MFMA)");
    if (rc != ZNN_OK || c.splits == 1) return rc;
    const long count = (long)P.fM * P.dz * P.dy * P.dx;
    ZNN_LAUNCH("sum over input-map shares", s, k_conv_reduce, dim3((unsigned)((count + 255) / 256)), dim3(256), 0,
               (const float*)P.partial, dst, count, c.splits);
    return check_launch("sum over input-map shares");
}

}  // namespace znn
