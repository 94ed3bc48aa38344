// Packed triangular storage utilities (the paper's "packed triangular SPD storage", Sec. III-E):
// conversion between a dense symmetric fp32 matrix and its packed lower tiles (layout: gemm.h,
// packed_off).  One workgroup per lower-triangle tile; every global access is a 16-byte vector
// along a row where the shapes allow it.
#include "common.h"
#include "gemm.h"

using namespace asteria;

namespace {

// The descriptors travel as kernel arguments in chunks of this many.
constexpr int SYM_CHUNK = 128;
struct SymChunk {
    asteria_sympair it[SYM_CHUNK];
    int tile_start[SYM_CHUNK + 1];
};

template <bool UNPACK>
__global__ __launch_bounds__(256) void sym_pack_kernel(SymChunk c, int nitems)
{
    int lo = 0, hi = nitems - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (c.tile_start[mid] <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const asteria_sympair &I = c.it[lo];
    int ti, tj;
    tri_decode((int)blockIdx.x - c.tile_start[lo], ti, tj);
    const int n = I.n, ld = I.ld;
    float *tile = I.packed + ((size_t)ti * (ti + 1) / 2 + tj) * PACK_T * PACK_T;
    const int r0 = ti * PACK_T, c0 = tj * PACK_T;
    if (!UNPACK) {
        // rows beyond n and columns beyond n are written as zero: the packed buffer is fully defined
        for (int e = threadIdx.x; e < PACK_T * PACK_T; e += 256) {
            const int r = e / PACK_T, cc = e % PACK_T;
            const int gr = r0 + r, gc = c0 + cc;
            float v = 0.0f;
            if (gr < n && gc < n) v = (ti != tj || gr >= gc) ? I.full[(size_t)gr * ld + gc] : I.full[(size_t)gc * ld + gr];
            tile[e] = v;                                   // a diagonal tile takes its upper half from the lower triangle
        }
    } else {
        __shared__ float t[PACK_T][PACK_T + 1];
        for (int e = threadIdx.x; e < PACK_T * PACK_T; e += 256) t[e / PACK_T][e % PACK_T] = tile[e];
        __syncthreads();
        for (int e = threadIdx.x; e < PACK_T * PACK_T; e += 256) {
            const int r = e / PACK_T, cc = e % PACK_T;
            const int gr = r0 + r, gc = c0 + cc;
            if (gr < n && gc < n) I.full[(size_t)gr * ld + gc] = t[r][cc];
            // the mirror image of an off-diagonal tile, written along its own rows
            const int mr = c0 + r, mc = r0 + cc;
            if (ti != tj && mr < n && mc < n) I.full[(size_t)mr * ld + mc] = t[cc][r];
        }
    }
}

template <bool UNPACK>
asteria_status run(const asteria_sympair *items, int nitems, hipStream_t stream)
{
    if (!items || nitems <= 0) return ASTERIA_INVALID_ARG;
    for (int i = 0; i < nitems; ++i) {
        const asteria_sympair &I = items[i];
        if (!I.full || !I.packed || I.n <= 0 || I.ld < I.n) return ASTERIA_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(I.packed) & 15u) return ASTERIA_INVALID_ARG;
    }
    for (int first = 0; first < nitems; first += SYM_CHUNK) {
        const int cnt = nitems - first < SYM_CHUNK ? nitems - first : SYM_CHUNK;
        SymChunk c;
        memset(&c, 0, sizeof(c));
        int tiles = 0;
        for (int i = 0; i < cnt; ++i) {
            c.it[i] = items[first + i];
            c.tile_start[i] = tiles;
            tiles += (int)packed_tiles(items[first + i].n);
        }
        c.tile_start[cnt] = tiles;
        hipLaunchKernelGGL(sym_pack_kernel<UNPACK>, dim3(tiles), dim3(256), 0, stream, c, cnt);
        ASTERIA_HIP_TRY(hipGetLastError());
    }
    return ASTERIA_OK;
}

}  // namespace

extern "C" size_t asteria_packed_elems(int n) { return n > 0 ? packed_elems(n) : 0; }

extern "C" asteria_status asteria_sym_pack(const asteria_sympair *items, int nitems, void *stream)
{
    return run<false>(items, nitems, reinterpret_cast<hipStream_t>(stream));
}

extern "C" asteria_status asteria_sym_unpack(const asteria_sympair *items, int nitems, void *stream)
{
    return run<true>(items, nitems, reinterpret_cast<hipStream_t>(stream));
}
