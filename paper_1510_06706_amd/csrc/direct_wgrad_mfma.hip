// Direct method, kernel gradient (Section 3.2) on the fp32 matrix cores.
//
//   gw[j][i][a][b][c] = sum_v gout[j][v] * in[i][v + (kz-1-a, ky-1-b, kx-1-c)]
//
// is a GEMM whose reduction runs over the output voxels v:
//
//   D[m][n] += A[m][k] * B[k][n]      v_mfma_f32_16x16x4_f32
//     m : 16 output maps j                    (A = gout, from an LDS tile)
//     n : 16 columns of the flattened (c, i)  (B = in shifted by the tap, from an LDS tile)
//     k : 4 consecutive output voxels of one x-row
//
// A workgroup owns one (a, b) tap plane, a group of columns n = c*f + i and a
// share of the voxel rows (split-K).  Tiles of R voxel rows travel from global
// memory straight into LDS (global_load_lds, no registers in between) into one
// of two buffers, so the next tile is in flight while the waves run the MFMAs
// of the current one.  With few columns the waves share the column tiles and
// take alternate voxel steps of a tile (their accumulators are added in a fixed
// order through LDS); with many columns every wave owns columns of its own, so
// that a staged tile feeds four times the MFMAs.  One partial matrix per workgroup.  A second kernel adds the partial matrices in
// ascending split order, so the result is bit-reproducible (no atomics).
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "direct_wgrad_impl.h"

namespace znn {

namespace {

using wgrad::WgradFn;
using wgrad::WgradTile;
using wgrad::kBufFloats;
using wgrad::kMaxTiles;

// gw[j][i][a][b][c] = sum over splits of partial[s][ab][j][c*f + i], ascending s.
__global__ void __launch_bounds__(256)
k_wgrad_reduce(const float* __restrict__ partial, float* __restrict__ gw, int f, int fo, int kz, int ky, int kx,
               int ksplit, int Mpad, int Npad, int mapmajor)
{
    const int taps = kz * ky * kx;
    const long total = (long)fo * f * taps;
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int tap = (int)(t % taps);
    const long e = t / taps;
    const int i = (int)(e % f), j = (int)(e / f);
    const int c = tap % kx, ab = tap / kx;
    const int AB = kz * ky;
    const int n = mapmajor ? i * kx + c : c * f + i;
    float acc = 0.f;
    for (int s = 0; s < ksplit; ++s) acc += partial[((long)(s * AB + ab) * Mpad + j) * Npad + n];
    gw[t] = acc;
}

// The same for small layers with many splits, where one thread per element is a long chain of dependent
// additions on few threads: wave l of a workgroup sums the splits s = l, l + 4, ... of 64 elements, then the
// four sums are added in the order l = 0, 1, 2, 3 (fixed, so results are reproducible from run to run).
__global__ void __launch_bounds__(256)
k_wgrad_reduce4(const float* __restrict__ partial, float* __restrict__ gw, int f, int fo, int kz, int ky, int kx,
                int ksplit, int Mpad, int Npad, int mapmajor)
{
    __shared__ float part[4][64];
    const int taps = kz * ky * kx;
    const long total = (long)fo * f * taps;
    const int l = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long t = (long)blockIdx.x * 64 + lane;
    float acc = 0.f;
    if (t < total) {
        const int tap = (int)(t % taps);
        const long e = t / taps;
        const int i = (int)(e % f), j = (int)(e / f);
        const int c = tap % kx, ab = tap / kx;
        const int AB = kz * ky;
        const int n = mapmajor ? i * kx + c : c * f + i;
        for (int s = l; s < ksplit; s += 4) acc += partial[((long)(s * AB + ab) * Mpad + j) * Npad + n];
    }
    part[l][lane] = acc;
    __syncthreads();
    if (l == 0 && t < total) gw[t] = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
}

// ng column sets of kw waves each (direct_wgrad_impl.h).  Sixteen waves (4 x 4) were measured slower than
// eight on every benchmark shape and are not instantiated.
WgradFn pick_wgrad(int nj, int nt, int ng, int kw)
{
    if (ng == 2 && kw == 4) return nj <= 4 ? wgrad_kernel_h2a(nj, nt) : wgrad_kernel_h2b(nj, nt);
    if (ng == 1 && kw == 4) return nj <= 4 ? wgrad_kernel_h1a(nj, nt) : wgrad_kernel_h1b(nj, nt);
    if (ng == 4 && kw == 1) return nj <= 4 ? wgrad_kernel_n4a(nj, nt) : wgrad_kernel_n4b(nj, nt);
    if (ng == 8 && kw == 1) return nj <= 4 ? wgrad_kernel_n8a(nj, nt) : wgrad_kernel_n8b(nj, nt);
    return nullptr;
}

struct WgradChoice {
    bool ok;
    int NJ, JG, NT, G, NG, KW;
    int TX, XT, R, GS, IS, TXH;
    int Mpad, Npad;
    int tiles, tps, ksplit;
    int vec4, fast, mapmajor;
    size_t lds;
};


// Map stride in LDS: a multiple of 4 floats (16-byte loads land on 16-byte boundaries)
// whose residue modulo 32 spreads the 16 maps of an MFMA operand over the banks.
int pad_stride(int n)
{
    const int res = tuning().wgrad_stride_mod;
    while (n % 32 != res) ++n;
    return n;
}

// own: every wave owns columns (layers with many columns); else the waves of a set share its column tiles.
WgradChoice search_wgrad_layout(const Geom& g, bool own)
{
    WgradChoice c = {};
    c.ok = false;
    const int mt = (g.fo + 15) / 16;
    const int ncols = g.f * g.kx;
    const int nt_tot = (ncols + 15) / 16;
    const int allowed[11] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 13, 16};
    if (own) {
        // Many columns: waves with columns of their own.  Over the ways to cut the output maps into JG
        // groups of NJ tiles and the columns into G groups of OW * NT tiles, take the one with the least
        // issued MFMA work, weighted by how much of a staged tile each MFMA needs (the tile of a workgroup
        // holds NJ * 16 gout maps and OW * NT * 16 / kx input maps; the fewer MFMAs per staged map, the less
        // of the fetch hides behind them).
        double best = 1e300;
        const int OW = tuning().wgrad_own_waves;
        for (int JG = 1; JG <= mt; ++JG) {
            const int NJ = (mt + JG - 1) / JG;
            if (NJ > 8 || (JG > 1 && NJ * (JG - 1) >= mt)) continue;
            for (int G = 1; G <= nt_tot; ++G) {
                const int per_wave = ((nt_tot + G - 1) / G + OW - 1) / OW;
                int NT = 0;
                for (int k = 0; k < 11 && !NT; ++k)
                    if (allowed[k] >= per_wave) NT = allowed[k];
                if (!NT || !pick_wgrad(NJ, NT, OW, 1)) continue;
                if ((nt_tot + OW * NT - 1) / (OW * NT) != G) continue;     // fewer groups would do for this NT
                const double issued = (double)JG * NJ * G * OW * NT;
                const double per_map = (double)NJ * OW * NT / (NJ + (double)OW * NT / g.kx);
                const double cost = issued * (1.0 + 4.0 / per_map);
                if (cost < best) { best = cost; c.JG = JG; c.NJ = NJ; c.G = G; c.NT = NT; }
            }
        }
        if (best == 1e300) return c;
        c.NG = OW; c.KW = 1;
    } else {
        // at most six 16-map tiles per workgroup: with seven or eight the gout half of the LDS tile leaves
        // too few voxels per tile (config 5: 187 -> 160 ms with two groups of four)
        const int maxnj = tuning().wgrad_maxnj;
        c.JG = (mt + maxnj - 1) / maxnj;
        c.NJ = (mt + c.JG - 1) / c.JG;
        int nt_max = 1;
        for (int k = 0; k < 11; ++k)
            if (c.NJ * allowed[k] <= kMaxTiles) nt_max = allowed[k];
        c.G = (nt_tot + nt_max - 1) / nt_max;
        const int want = (nt_tot + c.G - 1) / c.G;
        c.NT = nt_max;
        for (int k = 10; k >= 0; --k)
            if (allowed[k] >= want && c.NJ * allowed[k] <= kMaxTiles) c.NT = allowed[k];
        c.G = (nt_tot + c.NT - 1) / c.NT;
        // eight waves: the column tiles of a group are dealt to two sets of four waves each
        c.NG = 1; c.KW = 4;
        if (tuning().wgrad_halves >= 2 && c.NT >= 2 && pick_wgrad(c.NJ, (c.NT + 1) / 2, 2, 4)) {
            c.NG = 2;
            c.NT = (c.NT + 1) / 2;
            c.G = (nt_tot + c.NT * c.NG - 1) / (c.NT * c.NG);
        }
    }
    if (!pick_wgrad(c.NJ, c.NT, c.NG, c.KW)) return c;
    c.Mpad = c.JG * c.NJ * 16;
    c.Npad = c.G * c.NT * c.NG * 16;
    // Column order.  With n = c*f + i (x-tap major) a column group spans all f input maps as soon as
    // it is wider than f, so the LDS tile of a layer with many input maps holds few voxels; with
    // n = i*kx + c (map major) a group holds only the maps of its own columns.  One group: the same
    // either way (tap major kept).  Several groups: map major.
    c.mapmajor = c.G > 1 ? 1 : 0;
    // widest x-tap span and largest input-map range over the column groups; whether every group's
    // tile starts at x-tap kx-1 (then rows of the in tile start 16-byte aligned)
    int cspan = 0, nmaps = 1;
    bool aligned_rows = true;
    for (int cg = 0; cg < c.G; ++cg) {
        const int n0 = cg * c.NT * c.NG * 16;
        const int n1 = n0 + c.NT * c.NG * 16 < ncols ? n0 + c.NT * c.NG * 16 : ncols;
        int cmin, cmax, maps;
        if (c.mapmajor) {
            const int imin = n0 / g.kx, imax = (n1 - 1) / g.kx;
            cmin = 0; cmax = g.kx - 1;
            if (imin == imax) { cmin = n0 % g.kx; cmax = (n1 - 1) % g.kx; }
            maps = imax - imin + 1;
        } else {
            cmin = n0 / g.f; cmax = (n1 - 1) / g.f;
            maps = cmax == cmin ? (n1 - 1) % g.f - n0 % g.f + 1 : g.f;
        }
        if (cmax - cmin > cspan) cspan = cmax - cmin;
        if (maps > nmaps) nmaps = maps;
        if (cmax != g.kx - 1) aligned_rows = false;
    }
    if (c.KW > 1 && (size_t)c.NJ * c.NT * c.NG * 64 * 4 > (size_t)kBufFloats) return c;   // cross-wave reduction needs this
    const int rows = g.oz * g.oy;
    const int nw = c.NG * c.KW;
    // 16-byte loads: groups of four x-neighbours must be wholly inside or outside the images and start on
    // multiples of four in both tensors
    const bool in16 = g.nx % 4 == 0 && aligned_rows;
    // fast tile loader (see the kernel): tiles of whole rows that do not straddle a z-plane, spans per wave
    // that fit its register arrays, a lane's offset from the tile origin (up to a whole group of maps) in 32 bits
    auto fast_tiles = [&](int R, int GS, int IS) {
        const long span_g = ((long)c.NJ * 16 * GS + 255) / 256, span_i = ((long)nmaps * IS + 255) / 256;
        return g.oy % R == 0 && (span_g + nw - 1) / nw <= wgrad::max_spans(nw, c.NJ) && (span_i + nw - 1) / nw <= wgrad::max_spans(nw, c.NJ) &&
               (double)g.fo * g.ovol() * 4.0 < 2147483648.0 && (double)g.f * g.nvol() * 4.0 < 2147483648.0 &&
               !tuning().wgrad_slow_loader;
    };
    // Rows of gout whose length is 2 modulo 4 (90, 246, ...): staged WITHOUT padding behind each row, a tile of
    // R whole rows (R even) is one contiguous run per map in global memory as in LDS, so 16-byte loads may
    // straddle rows; the voxel pairs of an MFMA step still lie inside one row.  Only with the fast loader.
    if (g.ox % 4 == 2 && in16 && g.ovol() % 4 == 0) {
        const int TX = g.ox, TXH = (TX + cspan * g.spx + 3) & ~3;
        for (int R = 2; R <= 32 && R <= rows; R += 2) {
            const int GS = pad_stride((R * TX + 7) & ~7), IS = pad_stride(R * TXH);
            if ((long)c.NJ * 16 * GS + (long)nmaps * IS + 64 > kBufFloats) break;
            if (!fast_tiles(R, GS, IS)) continue;
            c.XT = 1; c.TX = TX; c.TXH = TXH; c.R = R; c.GS = GS; c.IS = IS;
            c.vec4 = 1; c.fast = 1; c.ok = true;
        }
    }
    // otherwise: fewest x-segments whose tile fits a buffer, then as many rows as fit (the most that still
    // allow the fast loader if that is at least half as many)
    for (int XT = 1; XT <= g.ox && !c.ok; ++XT) {
        const int seg = (g.ox + XT - 1) / XT;
        int TX = (seg + 3) & ~3;
        if (TX % 8 != 0 && rows < 2) TX += 4;          // a single row must hold whole 8-voxel steps
        const int TXH = (TX + cspan * g.spx + 3) & ~3;
        const int vec4 = (g.ox % 4 == 0 && in16) ? 1 : 0;
        int bestR = 0, fastR = 0;
        for (int R = 1; R <= 32 && R <= rows; ++R) {
            // the MFMA loop walks 8 voxels per step; a tile that ends on half a step reads its last four
            // voxels from the zero padding behind the row (gout) and from whatever follows (in)
            const int GS = pad_stride((R * TX + 7) & ~7), IS = pad_stride(R * TXH);
            if ((long)c.NJ * 16 * GS + (long)nmaps * IS + 64 > kBufFloats) break;
            bestR = R;
            if (vec4 && XT == 1 && fast_tiles(R, GS, IS)) fastR = R;
        }
        if (bestR == 0) continue;
        c.fast = 2 * fastR >= bestR ? 1 : 0;
        if (c.fast) bestR = fastR;
        c.XT = XT; c.TX = TX; c.TXH = TXH; c.R = bestR;
        c.GS = pad_stride((bestR * TX + 7) & ~7); c.IS = pad_stride(bestR * TXH);
        c.vec4 = vec4;
        c.ok = true;
    }
    if (!c.ok) return c;
    c.lds = 2 * (size_t)kBufFloats * 4;
    c.tiles = ((rows + c.R - 1) / c.R) * c.XT;
    // one workgroup per compute unit: split the voxel range until the grid reaches 256
    const long other = (long)g.kz * g.ky * c.G * c.JG;
    long ks = 256 / other;
    if (ks < 1) ks = 1;
    if (ks > c.tiles) ks = c.tiles;
    c.tps = (int)((c.tiles + ks - 1) / ks);
    c.ksplit = (c.tiles + c.tps - 1) / c.tps;
    if ((long)g.kz * g.ky > 65535 || (long)c.G * c.JG > 65535) c.ok = false;
    // the tile loader addresses a map with a 32-bit byte offset
    if (g.nvol() >= (1L << 30) || g.ovol() >= (1L << 30)) c.ok = false;
    return c;
}

// With many columns the layout in which every wave owns columns stages fewer tiles per MFMA (config 4:
// 1.22 -> 1.03 ms); it is passed over when only the shared layout's tiles qualify for the fast loader
// (config 5: 82 ms shared with the fast loader, 102 ms with own columns and the general one).
WgradChoice search_wgrad(const Geom& g)
{
    const WgradChoice shared = search_wgrad_layout(g, false);
    const int nt_tot = (g.f * g.kx + 15) / 16;
    if (nt_tot < tuning().wgrad_own_columns_from) return shared;
    const WgradChoice own = search_wgrad_layout(g, true);
    if (!own.ok) return shared;
    if (!shared.ok) return own;
    return shared.fast && !own.fast ? shared : own;
}

// Every call of the pass asks for the same answer three times (supported?, workspace, launch):
// remembered per shape.
WgradChoice choose_wgrad(const Geom& g)
{
    struct Entry { int key[14]; WgradChoice choice; };
    static std::mutex lock;
    static std::vector<Entry> memo;
    const int key[14] = {g.f, g.fo, g.nz, g.ny, g.nx, g.kz, g.ky, g.kx, g.spz, g.spy, g.spx, g.oz, g.oy, g.ox};
    {
        std::lock_guard<std::mutex> hold(lock);
        for (const Entry& e : memo)
            if (memcmp(e.key, key, sizeof(key)) == 0) return e.choice;
    }
    Entry e;
    memcpy(e.key, key, sizeof(key));
    e.choice = search_wgrad(g);
    std::lock_guard<std::mutex> hold(lock);
    if (memo.size() >= 256) memo.erase(memo.begin());
    memo.push_back(e);
    return e.choice;
}

}  // namespace

bool mfma_wgrad_supported(const Geom& g) { return choose_wgrad(g).ok; }

size_t mfma_wgrad_workspace(const Geom& g)
{
    const WgradChoice c = choose_wgrad(g);
    if (!c.ok) return 0;
    return align256((size_t)c.ksplit * g.kz * g.ky * c.Mpad * c.Npad * sizeof(float));
}

int mfma_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s)
{
    const WgradChoice c = choose_wgrad(g);
    if (!c.ok) return fail(ZNN_EUNSUPPORTED, "no tile configuration fits this shape");
    WgradTile P = {};
    P.in = in; P.gout = gout; P.partial = (float*)ws;
    P.f = g.f; P.fo = g.fo;
    P.nz = g.nz; P.ny = g.ny; P.nx = g.nx;
    P.oz = g.oz; P.oy = g.oy; P.ox = g.ox;
    P.kz = g.kz; P.ky = g.ky; P.kx = g.kx;
    P.spz = g.spz; P.spy = g.spy; P.spx = g.spx;
    P.TX = c.TX; P.XT = c.XT; P.R = c.R;
    P.GS = c.GS; P.IS = c.IS; P.TXH = c.TXH;
    P.Mpad = c.Mpad; P.Npad = c.Npad;
    P.G = c.G;
    P.tiles = c.tiles; P.tps = c.tps;
    P.AB = g.kz * g.ky;
    P.vec4 = c.vec4;
    P.fast = c.fast;
    P.mapmajor = c.mapmajor;
    P.dGS = make_fastdiv(c.GS); P.dIS = make_fastdiv(c.IS);
    P.dTX = make_fastdiv(c.TX); P.dTXH = make_fastdiv(c.TXH); P.dOY = make_fastdiv(g.oy);
    if (log_enabled())
        fprintf(stderr, "[znn] wgrad mfma: NJ=%d JG=%d NT=%d waves=%dx%d G=%d TX=%d XT=%d R=%d lds=%zu ksplit=%d tiles=%d\n",
                c.NJ, c.JG, c.NT, c.NG, c.KW, c.G, c.TX, c.XT, c.R, c.lds, c.ksplit, c.tiles);
    WgradFn fn = pick_wgrad(c.NJ, c.NT, c.NG, c.KW);
    if (!fn) return fail(ZNN_EUNSUPPORTED, "no kernel instance for tile %dx%d", c.NJ, c.NT);
    ZNN_LAUNCH("direct kernel gradient (MFMA)", s, fn, dim3((unsigned)c.ksplit, (unsigned)P.AB, (unsigned)(c.G * c.JG)), dim3(64 * c.NG * c.KW), 0, P);
    int rc = check_launch("direct kernel gradient (MFMA)");
    if (rc != ZNN_OK) return rc;
    const long total = (long)g.fo * g.f * g.kvol();
    if (total < 65536 && c.ksplit >= 16)
        ZNN_LAUNCH("kernel gradient reduction", s, k_wgrad_reduce4, dim3((unsigned)((total + 63) / 64)), dim3(256), 0,
                           (const float*)ws, gw, g.f, g.fo, g.kz, g.ky, g.kx, c.ksplit, c.Mpad, c.Npad, c.mapmajor);
    else
        ZNN_LAUNCH("kernel gradient reduction", s, k_wgrad_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                           (const float*)ws, gw, g.f, g.fo, g.kz, g.ky, g.kx, c.ksplit, c.Mpad, c.Npad, c.mapmajor);
    return check_launch("kernel gradient reduction");
}

}  // namespace znn
