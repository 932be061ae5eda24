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
// share of the voxel rows (split-K).  Its four waves take alternate 4-voxel
// steps of every staged tile; their accumulators are added in a fixed order
// through LDS and written as one partial matrix per workgroup.  A second
// kernel adds the partial matrices in ascending split order, so the result is
// bit-reproducible (no atomics).
#include <cstdio>
#include <cstdlib>

#include "znn_internal.h"

namespace znn {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBatch = 8;

struct WgradTile {
    const float* in; const float* gout; float* partial;
    int f, fo;
    int nz, ny, nx;
    int oz, oy, ox;
    int kz, ky, kx;
    int TX, XT, R;      // x-segment width (multiple of 4), segments per row, rows per tile
    int GS, IS, TXH;    // LDS strides: gout map, in map, in row
    int Mpad, Npad;     // padded partial-matrix extents
    int G;              // column groups
    int tiles, tps;     // voxel tiles in total and per split
    int AB;             // kz * ky
    FastDiv dRT, dTX, dRTH, dTXH, dOY;   // R*TX, TX, R*TXH, TXH, oy
};

template <int NJ, int NT>
__global__ void __launch_bounds__(256, (NJ * NT <= 24 ? 2 : 1)) k_wgrad_mfma(WgradTile P)
{
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, grp = lane >> 4;
    const int s = blockIdx.x, ab = blockIdx.y;
    const int a = ab / P.ky, b = ab % P.ky;
    const int cg = blockIdx.z % P.G, jg = blockIdx.z / P.G;
    const int ncols = P.f * P.kx;
    const int n0 = cg * NT * 16;
    const int n1 = min(n0 + NT * 16, ncols);
    const int cmin = n0 / P.f, cmax = (n1 - 1) / P.f;
    int imin = 0, imax = P.f - 1;
    if (cmin == cmax) { imin = n0 % P.f; imax = (n1 - 1) % P.f; }
    const int nmaps = imax - imin + 1;
    const int TXH = P.TXH;
    float* gt = lds;                        // [NJ*16][GS]
    float* it = lds + NJ * 16 * P.GS;       // [nmaps][IS]

    int aoff[NJ], boff[NT];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt) aoff[jt] = (jt * 16 + col) * P.GS + grp;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int n = n0 + nt * 16 + col;
        int o = grp;
        if (n < n1) {
            const int c = n / P.f, i = n % P.f;
            o = (i - imin) * P.IS + (cmax - c) + grp;
        }
        boff[nt] = o;
    }

    floatx4 acc[NJ][NT];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[jt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int rows = P.oz * P.oy;
    const long oplane = (long)rows * P.ox;
    const long iplane = (long)P.ny * P.nx;
    const int t_end = min((s + 1) * P.tps, P.tiles);
    const int nks = P.R * P.TX / 4;

    for (int tile = s * P.tps; tile < t_end; ++tile) {
        const int xt = tile % P.XT, rt = tile / P.XT;
        const int rho0 = rt * P.R, xs0 = xt * P.TX;
        __syncthreads();
        // both tiles are fetched in batches of kBatch independent loads per thread
        {
            const unsigned total = (unsigned)(NJ * 16 * P.R * P.TX);
            const unsigned RT = (unsigned)(P.R * P.TX);
            for (unsigned base = threadIdx.x; base < total; base += 256 * kBatch) {
                float v[kBatch];
                int lo[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const unsigned idx = base + u * 256;
                    v[u] = 0.f; lo[u] = -1;
                    if (idx < total) {
                        const unsigned m = fdiv(idx, P.dRT), e = idx - m * RT;
                        const unsigned r = fdiv(e, P.dTX), x = e - r * P.TX;
                        const int j = jg * NJ * 16 + (int)m, rho = rho0 + (int)r, gx = xs0 + (int)x;
                        lo[u] = (int)(m * P.GS + e);
                        if (j < P.fo && rho < rows && gx < P.ox) v[u] = P.gout[j * oplane + (long)rho * P.ox + gx];
                    }
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u)
                    if (lo[u] >= 0) gt[lo[u]] = v[u];
            }
        }
        {
            const int xin0 = xs0 + (P.kx - 1 - cmax);
            const unsigned RTH = (unsigned)(P.R * TXH);
            const unsigned total = (unsigned)nmaps * RTH;
            for (unsigned base = threadIdx.x; base < total; base += 256 * kBatch) {
                float v[kBatch];
                int lo[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const unsigned idx = base + u * 256;
                    v[u] = 0.f; lo[u] = -1;
                    if (idx < total) {
                        const unsigned m = fdiv(idx, P.dRTH), e = idx - m * RTH;
                        const unsigned r = fdiv(e, P.dTXH), x = e - r * TXH;
                        const int rho = rho0 + (int)r, ix = xin0 + (int)x;
                        lo[u] = (int)(m * P.IS + e);
                        if (rho < rows && ix < P.nx) {
                            const int z = (int)fdiv((unsigned)rho, P.dOY), y = rho - z * P.oy;
                            v[u] = P.in[((long)(imin + (int)m) * P.nz + (z + P.kz - 1 - a)) * iplane +
                                        (long)(y + P.ky - 1 - b) * P.nx + ix];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u)
                    if (lo[u] >= 0) it[lo[u]] = v[u];
            }
        }
        __syncthreads();

        float an[NJ], bn[NT];
        {
            const int q = 4 * min(wave, nks - 1);
            const int r = (int)fdiv((unsigned)q, P.dTX), tx = q - r * P.TX;
            const int ao = r * P.TX + tx, bo = r * TXH + tx;
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt) an[jt] = gt[aoff[jt] + ao];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bn[nt] = it[boff[nt] + bo];
        }
        for (int ks = wave; ks < nks; ks += 4) {
            float av[NJ], bv[NT];
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt) av[jt] = an[jt];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bv[nt] = bn[nt];
            const int kn = ks + 4 < nks ? ks + 4 : ks;
            const int q = 4 * kn;
            const int r = (int)fdiv((unsigned)q, P.dTX), tx = q - r * P.TX;
            const int ao = r * P.TX + tx, bo = r * TXH + tx;
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt) an[jt] = gt[aoff[jt] + ao];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bn[nt] = it[boff[nt] + bo];
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[jt], bv[nt], acc[jt][nt], 0, 0, 0);
        }
    }

    // add the four waves' accumulators in the order 0 + 1 + 2 + 3
    floatx4* red = reinterpret_cast<floatx4*>(lds);
    for (int w = 1; w < 4; ++w) {
        __syncthreads();
        if (wave == w) {
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) red[(jt * NT + nt) * 64 + lane] = acc[jt][nt];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const floatx4 v = red[(jt * NT + nt) * 64 + lane];
                    acc[jt][nt] += v;
                }
        }
    }
    if (wave == 0) {
        float* out = P.partial + ((long)(s * P.AB + ab) * P.Mpad + jg * NJ * 16) * P.Npad + cg * NT * 16;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    out[(long)(jt * 16 + grp * 4 + r) * P.Npad + nt * 16 + col] = acc[jt][nt][r];
    }
}

// gw[j][i][a][b][c] = sum over splits of partial[s][ab][j][c*f + i], ascending s.
__global__ void __launch_bounds__(256)
k_wgrad_reduce(const float* __restrict__ partial, float* __restrict__ gw, int f, int fo, int kz, int ky, int kx,
               int ksplit, int Mpad, int Npad)
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
    const int n = c * f + i;
    float acc = 0.f;
    for (int s = 0; s < ksplit; ++s) acc += partial[((long)(s * AB + ab) * Mpad + j) * Npad + n];
    gw[t] = acc;
}

using WgradFn = void (*)(WgradTile);

constexpr int kMaxTiles = 40;   // accumulator tiles per wave (4 registers each)

template <int NJ, int NT> WgradFn inst()
{
    if constexpr (NJ * NT <= kMaxTiles) return k_wgrad_mfma<NJ, NT>;
    else return nullptr;
}

template <int NJ> WgradFn pick_nt(int nt)
{
    switch (nt) {
        case 1: return inst<NJ, 1>();
        case 2: return inst<NJ, 2>();
        case 3: return inst<NJ, 3>();
        case 4: return inst<NJ, 4>();
        case 5: return inst<NJ, 5>();
        case 6: return inst<NJ, 6>();
        case 7: return inst<NJ, 7>();
        case 8: return inst<NJ, 8>();
        case 10: return inst<NJ, 10>();
        case 13: return inst<NJ, 13>();
        case 16: return inst<NJ, 16>();
    }
    return nullptr;
}

WgradFn pick_wgrad(int nj, int nt)
{
    switch (nj) {
        case 1: return pick_nt<1>(nt);
        case 2: return pick_nt<2>(nt);
        case 3: return pick_nt<3>(nt);
        case 4: return pick_nt<4>(nt);
        case 5: return pick_nt<5>(nt);
        case 6: return pick_nt<6>(nt);
        case 7: return pick_nt<7>(nt);
        case 8: return pick_nt<8>(nt);
    }
    return nullptr;
}

struct WgradChoice {
    bool ok;
    int NJ, JG, NT, G;
    int TX, XT, R, GS, IS, TXH;
    int Mpad, Npad;
    int tiles, tps, ksplit;
    size_t lds;
};


int pad_stride(int n)   // smallest value >= n that is 4 modulo 32 (bank spread of 16 maps x 4 voxels)
{
    while (n % 32 != 4) ++n;
    return n;
}

int wgrad_occupancy()
{
    static const int occ = [] { const char* e = getenv("ZNN_WGRAD_OCC"); return e ? atoi(e) : 2; }();
    return occ;
}

WgradChoice choose_wgrad(const Geom& g)
{
    const int occ = wgrad_occupancy();
    const size_t lds_max = occ >= 2 ? 64 * 1024 : 128 * 1024;
    WgradChoice c = {};
    c.ok = false;
    const int mt = (g.fo + 15) / 16;
    c.JG = (mt + 7) / 8;
    c.NJ = (mt + c.JG - 1) / c.JG;
    const int ncols = g.f * g.kx;
    const int nt_tot = (ncols + 15) / 16;
    // occupancy 2 (two waves per SIMD, tiles overlap each other's staging) needs <= 24
    // accumulator tiles per wave; occupancy 1 allows 40 and fewer column groups.
    const int budget = occ >= 2 ? 24 : kMaxTiles;
    const int allowed[11] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 13, 16};
    int nt_max = 1;
    for (int k = 0; k < 11; ++k)
        if (c.NJ * allowed[k] <= budget) nt_max = allowed[k];
    c.G = (nt_tot + nt_max - 1) / nt_max;
    const int want = (nt_tot + c.G - 1) / c.G;
    c.NT = nt_max;
    for (int k = 10; k >= 0; --k)
        if (allowed[k] >= want && c.NJ * allowed[k] <= budget) c.NT = allowed[k];
    c.G = (nt_tot + c.NT - 1) / c.NT;
    if (!pick_wgrad(c.NJ, c.NT)) return c;
    c.Mpad = c.JG * c.NJ * 16;
    c.Npad = c.G * c.NT * 16;
    // widest x-tap span and largest input-map range over the column groups
    int cspan = 0, nmaps = 1;
    for (int cg = 0; cg < c.G; ++cg) {
        const int n0 = cg * c.NT * 16;
        const int n1 = n0 + c.NT * 16 < ncols ? n0 + c.NT * 16 : ncols;
        const int cmin = n0 / g.f, cmax = (n1 - 1) / g.f;
        const int span = cmax - cmin;
        const int maps = span == 0 ? (n1 - 1) % g.f - n0 % g.f + 1 : g.f;
        if (span > cspan) cspan = span;
        if (maps > nmaps) nmaps = maps;
    }
    const size_t red = (size_t)c.NJ * c.NT * 64 * sizeof(floatx4);
    const int rows = g.oz * g.oy;
    for (int XT = 1; XT <= g.ox; ++XT) {
        const int seg = (g.ox + XT - 1) / XT;
        const int TX = (seg + 3) & ~3;
        const int TXH = TX + cspan;
        int bestR = 0;
        for (int R = 1; R <= 16 && R <= rows && R * (TX + cspan) * nmaps < 60000; ++R) {
            const int GS = pad_stride(R * TX), IS = pad_stride(R * TXH);
            const size_t bytes = ((size_t)c.NJ * 16 * GS + (size_t)nmaps * IS) * 4;
            if (bytes <= lds_max) bestR = R;
        }
        if (bestR == 0) continue;
        c.XT = XT; c.TX = TX; c.TXH = TXH; c.R = bestR;
        c.GS = pad_stride(bestR * TX); c.IS = pad_stride(bestR * TXH);
        size_t bytes = ((size_t)c.NJ * 16 * c.GS + (size_t)nmaps * c.IS) * 4;
        if (bytes < red) bytes = red;
        if (bytes > lds_max) continue;
        c.lds = bytes;
        c.ok = true;
        break;
    }
    if (!c.ok) return c;
    c.tiles = ((rows + c.R - 1) / c.R) * c.XT;
    const long other = (long)g.kz * g.ky * c.G * c.JG;
    long ks = (512 + other - 1) / other;
    if (ks < 1) ks = 1;
    if (ks > c.tiles) ks = c.tiles;
    c.tps = (int)((c.tiles + ks - 1) / ks);
    c.ksplit = (c.tiles + c.tps - 1) / c.tps;
    if ((long)g.kz * g.ky > 65535 || (long)c.G * c.JG > 65535) c.ok = false;
    return c;
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
    P.TX = c.TX; P.XT = c.XT; P.R = c.R;
    P.GS = c.GS; P.IS = c.IS; P.TXH = c.TXH;
    P.Mpad = c.Mpad; P.Npad = c.Npad;
    P.G = c.G;
    P.tiles = c.tiles; P.tps = c.tps;
    P.AB = g.kz * g.ky;
    P.dRT = make_fastdiv(c.R * c.TX); P.dTX = make_fastdiv(c.TX);
    P.dRTH = make_fastdiv(c.R * c.TXH); P.dTXH = make_fastdiv(c.TXH); P.dOY = make_fastdiv(g.oy);
    if (log_enabled())
        fprintf(stderr, "[znn] wgrad mfma: NJ=%d JG=%d NT=%d G=%d TX=%d XT=%d R=%d lds=%zu ksplit=%d tiles=%d\n",
                c.NJ, c.JG, c.NT, c.G, c.TX, c.XT, c.R, c.lds, c.ksplit, c.tiles);
    WgradFn fn = pick_wgrad(c.NJ, c.NT);
    if (!fn) return fail(ZNN_EUNSUPPORTED, "no kernel instance for tile %dx%d", c.NJ, c.NT);
    if (c.lds > 64 * 1024 &&
        hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c.lds) != hipSuccess)
        return fail(ZNN_EHIP, "cannot reserve %zu bytes of LDS", c.lds);
    ZNN_LAUNCH("direct kernel gradient (MFMA)", s, fn, dim3((unsigned)c.ksplit, (unsigned)P.AB, (unsigned)(c.G * c.JG)), dim3(256), c.lds, P);
    int rc = check_launch("direct kernel gradient (MFMA)");
    if (rc != ZNN_OK) return rc;
    const long total = (long)g.fo * g.f * g.kvol();
    ZNN_LAUNCH("kernel gradient reduction", s, k_wgrad_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       (const float*)ws, gw, g.f, g.fo, g.kz, g.ky, g.kx, c.ksplit, c.Mpad, c.Npad);
    return check_launch("kernel gradient reduction");
}

}  // namespace znn
