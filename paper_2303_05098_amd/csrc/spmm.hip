// Y = A X for k right-hand sides at once, in every format: a second operation under the tuning interface, which the
// paper defines for SpMV and leaves open for further operations (Section VI-B).  X is n x k and Y is m x k, both
// row-major, so the k values a matrix entry needs are contiguous.
//
// The product is computed in column panels of width 8, 4, 2 or 1 (k = 13 is 8 + 4 + 1), the matrix streamed once per
// panel.  A panel row of X or Y is split into pieces of 16 bytes (V = 2 doubles or 4 floats) and a row of the matrix
// is owned by G = panel width / V neighbouring lanes, one piece each: a wave instruction that fetches X for one
// entry per row then reads whole 16-byte-per-lane runs, 64 / G rows of X with no byte fetched twice, and the G lanes
// of a row read the entry itself from the same address (one request).  With one lane per row and the whole panel in
// its registers (the first design) a lane needed four 16-byte loads per entry, each instruction touching 64 cache
// lines a quarter at a time: the L1's line rate, not the memory, bounded the product (8 columns of the 27-point
// stencil on 128^3 points: DIA 287 us, ELL 359 us, CSR 395 us).  Wider panels would not help: what limits the product
// beyond 8 columns is the footprint of the rows of X that neighbouring matrix rows share, which at 16 columns
// (128-byte rows) no longer fits the 4 MB L2 of an XCD for that stencil.
// Rows given by a row pointer (CSR, the CSR remainder of HDC, the sorted COO arrays with the positions of their row
// runs) reach the lanes through a per-wave LDS stage filled with coalesced loads, as in the conversion kernels.
// Every output is summed by one thread in a fixed order: results are bit-identical from run to run.  HYB and HDC run
// their second part in accumulate mode.
#include "dev_common.hpp"
#include "mo_internal.hpp"

namespace mo {

constexpr int MB = 256;
constexpr int SPMM_LONG_ROW = 64;   // rows longer than this are walked by the whole wave

// Lanes per matrix row for a panel of K columns: pieces of 16 bytes, at least one.
template <typename T, int K> struct Panel {
    static constexpr int V = K * (int)sizeof(T) >= 16 ? 16 / (int)sizeof(T) : K;   // columns per lane
    static constexpr int G = K / V;                                                // lanes per row
    static constexpr int ROWS = MB / G;                                            // rows per block of MB threads
};

// A 16-byte piece of a row of X as one load.  The rows of X are only as aligned as their element type (k = 13 columns
// of floats: 52-byte rows), which global loads of any width accept; written element by element the compiler fetches a
// piece of four floats as two 8-byte loads, and an 8-byte-per-lane load costs the memory pipeline as much as a 16-byte one.
typedef float flt4u __attribute__((ext_vector_type(4), aligned(4)));
typedef double dbl2u __attribute__((ext_vector_type(2), aligned(8)));
template <typename T, int V>
__device__ __forceinline__ void load_piece(const T *__restrict__ p, T (&out)[V])
{
    if constexpr (sizeof(T) == 4 && V == 4) {
        const flt4u w = *reinterpret_cast<const flt4u *>(p);
        out[0] = w.x; out[1] = w.y; out[2] = w.z; out[3] = w.w;
    } else if constexpr (sizeof(T) == 8 && V == 2) {
        const dbl2u w = *reinterpret_cast<const dbl2u *>(p);
        out[0] = w.x; out[1] = w.y;
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v) out[v] = p[v];
    }
}

template <typename T, int V>
__device__ __forceinline__ void fma_row(T (&acc)[V], T a, const T *__restrict__ xr)
{
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] += a * xr[v];
}

template <typename T, int V, bool ACC>
__device__ __forceinline__ void store_row(T *__restrict__ yr, const T (&acc)[V])
{
#pragma unroll
    for (int v = 0; v < V; ++v) yr[v] = ACC ? yr[v] + acc[v] : acc[v];
}

// The value that lane CC of the caller's group of G neighbouring lanes holds (G = 1, 2 or 4; groups never straddle a
// quad of lanes, so this is a quad permutation in the data path, no LDS traffic).
template <int G, int CC>
__device__ __forceinline__ int group_bcast_i32(int v)
{
    if constexpr (G == 1) return v;
    else {
        constexpr int hi = G == 4 ? CC : 2 + CC;                     // source of the quad's lanes 2 and 3
        constexpr int ctrl = CC | (CC << 2) | (hi << 4) | (hi << 6);   // quad_perm
        return __builtin_amdgcn_update_dpp(0, v, ctrl, 0xf, 0xf, true);
    }
}
template <int G, int CC>
__device__ __forceinline__ float group_bcast(float v) { return __builtin_bit_cast(float, group_bcast_i32<G, CC>(__builtin_bit_cast(int, v))); }
template <int G, int CC>
__device__ __forceinline__ int32_t group_bcast(int32_t v) { return group_bcast_i32<G, CC>(v); }
template <int G, int CC>
__device__ __forceinline__ double group_bcast(double v)
{
    int2v w = __builtin_bit_cast(int2v, v);
    w.x = group_bcast_i32<G, CC>(w.x);
    w.y = group_bcast_i32<G, CC>(w.y);
    return __builtin_bit_cast(double, w);
}
// f(cc, value held by lane cc of the group) for cc = 0 .. G-1, in this order
template <int G, typename A, typename F>
__device__ __forceinline__ void for_group(A v, F &&f)
{
    f(0, group_bcast<G, 0>(v));
    if constexpr (G >= 2) f(1, group_bcast<G, 1>(v));
    if constexpr (G == 4) { f(2, group_bcast<G, 2>(v)); f(3, group_bcast<G, 3>(v)); }
}

template <int G, typename A, typename B, typename F>
__device__ __forceinline__ void for_group2(A v, B w, F &&f)
{
    f(0, group_bcast<G, 0>(v), group_bcast<G, 0>(w));
    if constexpr (G >= 2) f(1, group_bcast<G, 1>(v), group_bcast<G, 1>(w));
    if constexpr (G == 4) { f(2, group_bcast<G, 2>(v), group_bcast<G, 2>(w)); f(3, group_bcast<G, 3>(v), group_bcast<G, 3>(w)); }
}

// HDC with short remainder rows: the lanes of row i add the row's run [p0, p1) of the CSR remainder after the diagonals
// (the callers read the two row pointers before the diagonals, so that they have arrived by now; an empty run when
// there is no remainder, or one that a kernel of its own adds).
template <typename T, int V>
__device__ __forceinline__ void add_remainder(T (&acc)[V], int32_t p0, int32_t p1, const int32_t *__restrict__ col,
                                              const T *__restrict__ val, const T *__restrict__ xc, int64_t ldk)
{
    for (int32_t p = p0; p < p1; ++p) fma_row<T, V>(acc, val[p], xc + (int64_t)col[p] * ldk);
}

constexpr int DIA_U = 8;   // slab values a lane holds per pass of the DIA kernels: DIA_U * G diagonals per pass

// x and y point at the first column of the panel; ldk = k is the distance between rows of X and of Y.
// The G lanes of a row share the loads of its slab values: lane cg fetches diagonals cg, cg + G, ... of a pass, all
// in flight together, and the group passes them round.  Slab positions whose column lies outside the matrix hold +0
// by construction, but X may hold anything there, so the value of X is selected away; the loads themselves carry no
// condition (row of X clamped), so they overlap.  Lanes of rows past the end compute on row m - 1 and store nothing.
template <typename T, int K>
__global__ __launch_bounds__(MB) void k_spmm_dia(const int32_t *__restrict__ off, const T *__restrict__ val, int64_t nd, int64_t ld,
                                                  int64_t m, int64_t n, int64_t ldk, const int32_t *__restrict__ rem_rp,
                                                  const int32_t *__restrict__ rem_col, const T *__restrict__ rem_val,
                                                  const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int V = Panel<T, K>::V, G = Panel<T, K>::G, XU = G == 1 ? 4 : G;   // XU rows of X in flight per lane
    const int64_t i0 = xcd_block(blockIdx.x, gridDim.x) * Panel<T, K>::ROWS + threadIdx.x / G;
    const int cg = (int)(threadIdx.x % G), c = cg * V;
    const int64_t i = i0 < m ? i0 : m - 1;
    T acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = (T)0;
    const T *vp = val + i;
    const T *xc = x + c;
    const int32_t p0 = rem_rp ? rem_rp[i] : 0, p1 = rem_rp ? rem_rp[i + 1] : 0;
    for (int64_t d0 = 0; d0 < nd; d0 += DIA_U * G) {
        T av[DIA_U];
#pragma unroll
        for (int u = 0; u < DIA_U; ++u) {
            const int64_t d = d0 + u * G + cg;
            av[u] = ld_stream(vp + (d < nd ? d : nd - 1) * ld);
        }
#pragma unroll
        for (int u = 0; u < DIA_U; u += XU / G) {   // XU diagonals at a time: their rows of X are fetched together
            if (d0 + u * G >= nd) break;
            T xr[XU][V], aa[XU];
#pragma unroll
            for (int w = 0; w < XU / G; ++w)
                for_group<G>(av[u + w], [&](int cc, T a) {
                    const int64_t d = d0 + (u + w) * G + cc;
                    const int64_t j = i + off[d < nd ? d : nd - 1];
                    const bool in = d < nd && j >= 0 && j < n;
                    const T *xp = xc + (in ? j : 0) * ldk;
                    aa[w * G + cc] = a;
                    load_piece<T, V>(xp, xr[w * G + cc]);
#pragma unroll
                    for (int v = 0; v < V; ++v) xr[w * G + cc][v] = in ? xr[w * G + cc][v] : (T)0;   // whatever X holds in the clamped row
                });
#pragma unroll
            for (int q = 0; q < XU; ++q) fma_row<T, V>(acc, aa[q], xr[q]);
        }
    }
    add_remainder<T, V>(acc, p0, p1, rem_col, rem_val, xc, ldk);
    if (i0 < m) store_row<T, V, false>(y + i * ldk + c, acc);
}

// DIA with windows of X in LDS (the idea of the SpMV kernel's window plan, made for blocks of SPMM_ROWS rows): offsets
// closer than one block of rows share a window; the block stages the windows' rows of X, K values each, in LDS once,
// with coalesced 16-byte pieces, and serves every diagonal from there instead of fetching K values per row and
// diagonal through the L1 / texture path, whose rate of bytes into registers is what bounds the direct kernel.
// SPMM_ROWS rows per block, G lanes per row as in the other kernels, so SPMM_ROWS * G threads; the lanes of a row
// read neighbouring pieces of LDS (no bank conflict).  Staged row e holds row e + delta of X, counted from the block's
// first matrix row, delta being one of two values per run of SPMM_ROWS staged rows (map: where the run's second window
// begins, delta before, delta from there on: uniform reads, so no thread waits for a table before it can ask for its
// pieces); columns outside [0, n) are staged as 0 and the slab holds +0 there, so the loop needs
// no bounds test.  A block's LDS footprint allows few waves per CU, so everything a thread needs from memory is
// requested before the barrier: the first DIA_U * G slab values of its row (shared among the row's lanes as in the
// direct kernel) and its pieces of the windows, WIN_SB at a time.  (A fixed grid of blocks that walk over tiles and
// request the next tile's pieces into registers while the current one is computed out of LDS was measured slower,
// 280 against 236 us for 8 columns of the 27-point stencil on 128^3 points: its registers allow three blocks per CU
// where the LDS allows four, and what counts is how much the resident blocks have in flight.)
constexpr int WIN_SB = 12;
template <typename T, int K>
__global__ __launch_bounds__(SPMM_ROWS * 4) void k_spmm_dia_win(const int32_t *__restrict__ xpos, const int32_t *__restrict__ map, int elems,
                                                                const T *__restrict__ val, int64_t nd, int64_t ld, int64_t m, int64_t n,
                                                                int64_t ldk, const int32_t *__restrict__ rem_rp,
                                                                const int32_t *__restrict__ rem_col, const T *__restrict__ rem_val,
                                                                const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int V = Panel<T, K>::V, G = Panel<T, K>::G;
    static_assert(G <= 4, "launch bounds assume at most four lanes per row");
    extern __shared__ __align__(16) unsigned char s_raw[];
    T *xs = reinterpret_cast<T *>(s_raw);
    const int64_t row0 = xcd_block(blockIdx.x, gridDim.x) * SPMM_ROWS;
    const int r = (int)threadIdx.x / G, cg = (int)threadIdx.x % G, c = cg * V;
    const int64_t i0 = row0 + r, i = i0 < m ? i0 : m - 1;
    const T *vp = val + i;
    const int32_t p0 = rem_rp ? rem_rp[i] : 0, p1 = rem_rp ? rem_rp[i + 1] : 0;
    T av[DIA_U];
#pragma unroll
    for (int u = 0; u < DIA_U; ++u) {
        const int64_t d = u * G + cg;
        av[u] = ld_stream(vp + (d < nd ? d : nd - 1) * ld);
    }
    const int nrun = (elems + SPMM_ROWS - 1) / SPMM_ROWS;
    for (int u0 = 0; u0 < nrun; u0 += WIN_SB) {   // thread (r, cg) stages piece cg of staged rows r, r + 64, ...
        T buf[WIN_SB][V];
        bool in[WIN_SB];
#pragma unroll
        for (int u = 0; u < WIN_SB; ++u) {
            const int uu = u0 + u < nrun ? u0 + u : nrun - 1;   // uniform: the three table reads are scalar loads
            const int e = uu * SPMM_ROWS + r, ec = e < elems ? e : elems - 1;
            const int mb = __builtin_amdgcn_readfirstlane(map[3 * uu]), da = __builtin_amdgcn_readfirstlane(map[3 * uu + 1]),
                      db = __builtin_amdgcn_readfirstlane(map[3 * uu + 2]);
            const int64_t j = row0 + ec + (ec < mb ? da : db);
            in[u] = j >= 0 && j < n;
            const T *xp = x + (in[u] ? j : 0) * ldk + c;
            load_piece<T, V>(xp, buf[u]);
        }
#pragma unroll
        for (int u = 0; u < WIN_SB; ++u) {
            const int e = (u0 + u) * SPMM_ROWS + r;
            if (u0 + u < nrun && e < elems) {
                T *dst = xs + (int64_t)e * K + c;
#pragma unroll
                for (int v = 0; v < V; ++v) dst[v] = in[u] ? buf[u][v] : (T)0;
            }
        }
    }
    __syncthreads();
    T acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = (T)0;
    const T *xl = xs + (int64_t)r * K + c;
    for (int64_t d0 = 0; d0 < nd; d0 += DIA_U * G) {
        if (d0 > 0) {
#pragma unroll
            for (int u = 0; u < DIA_U; ++u) {
                const int64_t d = d0 + u * G + cg;
                av[u] = ld_stream(vp + (d < nd ? d : nd - 1) * ld);
            }
        }
#pragma unroll
        for (int u = 0; u < DIA_U; ++u) {
            if (d0 + u * G >= nd) break;
            for_group<G>(av[u], [&](int cc, T a) {
                const int64_t d = d0 + u * G + cc;
                if (d < nd) fma_row<T, V>(acc, a, xl + (int64_t)xpos[d] * K);
            });
        }
    }
    add_remainder<T, V>(acc, p0, p1, rem_col, rem_val, x + c, ldk);
    if (i0 < m) store_row<T, V, false>(y + i * ldk + c, acc);
}

// Eight slots per pass; the G lanes of a row share the loads of the pass's columns and values (lane cg fetches slots
// cg, cg + G, ...) and pass them round, and the next pass's are requested before this pass's rows of X, so the two
// latencies overlap.  Padding slots carry column -1 and value +0: nothing is fetched for them (a matrix with rows of
// very different lengths is mostly padding in its last slots).  Lanes of rows past the end compute on row m - 1 and store nothing.
// coo_rp != nullptr: a HYB handle whose rows keep few entries in the COO part; the row's lanes add their own COO run.
template <typename T, int K>
__global__ __launch_bounds__(MB) void k_spmm_ell(const int32_t *__restrict__ col, const T *__restrict__ val, int64_t W, int64_t ld,
                                                  int64_t m, int64_t ldk, const int32_t *__restrict__ coo_rp,
                                                  const int32_t *__restrict__ ccol, const T *__restrict__ cval,
                                                  const T *__restrict__ x, T *__restrict__ y)
{
    constexpr int V = Panel<T, K>::V, G = Panel<T, K>::G, PASS = 8, EU = PASS / G;
    const int64_t i0 = xcd_block(blockIdx.x, gridDim.x) * Panel<T, K>::ROWS + threadIdx.x / G;
    const int cg = (int)(threadIdx.x % G), c = cg * V;
    const int64_t i = i0 < m ? i0 : m - 1;
    T acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = (T)0;
    const int32_t *cp = col + i;
    const T *vp = val + i;
    const T *xc = x + c;
    const int32_t p0 = coo_rp ? coo_rp[i] : 0, p1 = coo_rp ? coo_rp[i + 1] : 0;   // asked for now, needed after the slots
    int32_t nj[EU];
    T na[EU];
#pragma unroll
    for (int u = 0; u < EU; ++u) {
        const int64_t sl = u * G + cg;
        const int64_t sc = sl < W ? sl : (W > 0 ? W - 1 : 0);
        nj[u] = W > 0 ? ld_stream(cp + sc * ld) : -1;
        na[u] = W > 0 ? ld_stream(vp + sc * ld) : (T)0;
    }
    for (int64_t s0 = 0; s0 < W; s0 += PASS) {
        int32_t cj[EU];
        T ca[EU];
#pragma unroll
        for (int u = 0; u < EU; ++u) { cj[u] = nj[u]; ca[u] = na[u]; }
        if (s0 + PASS < W) {
#pragma unroll
            for (int u = 0; u < EU; ++u) {
                const int64_t sl = s0 + PASS + u * G + cg;
                const int64_t sc = sl < W ? sl : W - 1;
                nj[u] = ld_stream(cp + sc * ld);
                na[u] = ld_stream(vp + sc * ld);
            }
        }
        T xr[PASS][V], aa[PASS];
#pragma unroll
        for (int u = 0; u < EU; ++u)
            for_group2<G>(cj[u], ca[u], [&](int cc, int32_t j, T a) {
                const bool on = s0 + u * G + cc < W && j >= 0;
                aa[u * G + cc] = on ? a : (T)0;
#pragma unroll
                for (int v = 0; v < V; ++v) xr[u * G + cc][v] = (T)0;
                if (on) load_piece<T, V>(xc + (int64_t)j * ldk, xr[u * G + cc]);   // nothing is fetched for padding
            });
#pragma unroll
        for (int q = 0; q < PASS; ++q) fma_row<T, V>(acc, aa[q], xr[q]);
    }
    for (int32_t p = p0; p < p1; ++p) fma_row<T, V>(acc, cval[p], xc + (int64_t)ccol[p] * ldk);
    if (i0 < m) store_row<T, V, false>(y + i * ldk + c, acc);
}

// Rows by row pointer.  A wave owns 64 / G consecutive rows (G lanes each), whose entries are one contiguous run: it is
// staged in LDS in chunks of whole rows (as many consecutive rows as fit RCAP entries) and the lanes of a row walk it
// out of LDS, all reading the same entry and each its own piece of the row of X.  Rows of more than SPMM_LONG_ROW
// entries are left to the whole wave, so that one long row does not keep the other lanes waiting.  rp comes from a
// validated CSR or was built by the conversions, so it is non-decreasing; the conditions below still keep every
// LDS index inside the chunk.  The G lanes of a row hold the same lo / hi, so runs of rows begin and end on
// multiples of G lanes.  RCAP is the host's choice by the average length of the part's rows (launch_rows): the
// stage decides how many waves a CU holds (12 bytes per entry in fp64: 13 waves at 1024 entries, 26 at 512), and a
// wave that needs a second chunk for its 64 / G rows pays the stage's latency twice.
template <typename T, int K, bool ACC, int RCAP>
__global__ __launch_bounds__(MB) void k_spmm_rows(const int32_t *__restrict__ rp, const int32_t *__restrict__ col,
                                                   const T *__restrict__ val, int64_t m, int64_t ldk, const T *__restrict__ x,
                                                   T *__restrict__ y)
{
    constexpr int V = Panel<T, K>::V, G = Panel<T, K>::G;
    __shared__ int32_t s_col_all[(MB / WAVE) * RCAP];
    __shared__ T s_val_all[(MB / WAVE) * RCAP];
    int32_t *s_col = s_col_all + (threadIdx.x / WAVE) * RCAP;
    T *s_val = s_val_all + (threadIdx.x / WAVE) * RCAP;
    const int lane = lane_id();
    const int64_t i = xcd_block(blockIdx.x, gridDim.x) * Panel<T, K>::ROWS + threadIdx.x / G;
    const int c = (int)(threadIdx.x % G) * V;
    const T *xc = x + c;
    const bool rv = i < m;
    const int lo = rv ? rp[i] : 0, hi = rv ? rp[i + 1] : 0;
    T acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = (T)0;
    const bool is_long = rv && hi - lo > SPMM_LONG_ROW;
    const int nvalid = __popcll(ballot64(rv));
    int first = 0;
    while (first < nvalid) {
        const int start = __builtin_amdgcn_readlane(lo, first);
        const uint64_t fits = ballot64(rv && lo >= start && hi >= lo && hi - start <= RCAP) >> first;
        const int nrun = ~fits ? __ffsll((unsigned long long)~fits) - 1 : WAVE;
        if (nrun <= 0) { first += G; continue; }   // longer than a chunk: a long row, walked by the whole wave below
        const int last = first + nrun - 1;
        const int end = __builtin_amdgcn_readlane(hi, last);
        const int total = end - start;   // 0 .. RCAP
        if (total > 0) {   // (a single load per array for runs of at most 64 entries, as a branch of its own, cost 7 % on CSR)
            stage_to_lds(col + start, s_col, total, lane);
            stage_to_lds(val + start, s_val, total, lane);
        }
        if (!is_long && lane >= first && lane <= last && hi <= end) {
            constexpr int ROWS_U = V >= 8 ? 4 : 8;   // entries fetched together; fewer for wide pieces (registers)
            int p = lo - start;
            const int pe = hi - start;
            for (; p + ROWS_U <= pe; p += ROWS_U) {   // ROWS_U entries at a time: their LDS reads and their gathers of X overlap
                int32_t cj[ROWS_U];
                T aj[ROWS_U];
#pragma unroll
                for (int u = 0; u < ROWS_U; ++u) { cj[u] = s_col[p + u]; aj[u] = s_val[p + u]; }
                T xj[ROWS_U][V];
#pragma unroll
                for (int u = 0; u < ROWS_U; ++u) {
                    const T *xr = xc + (int64_t)cj[u] * ldk;
                    load_piece<T, V>(xr, xj[u]);
                }
#pragma unroll
                for (int u = 0; u < ROWS_U; ++u) fma_row<T, V>(acc, aj[u], xj[u]);
            }
            for (; p < pe; ++p) fma_row<T, V>(acc, s_val[p], xc + (int64_t)s_col[p] * ldk);
        }
        first = last + 1;
    }
    // Long rows: the 64 / G lane groups share the row's entries (loads straight from memory), the partial sums of the
    // lanes that hold the same piece are added across the wave in a fixed order, and the row's own lanes keep the result.
    uint64_t longmask = ballot64(is_long);
    while (longmask) {
        const int l = __ffsll((unsigned long long)longmask) - 1;   // first lane of the row's group: a multiple of G
        longmask &= ~(((uint64_t)(1u << G) - 1) << l);
        const int rlo = __builtin_amdgcn_readlane(lo, l), rhi = __builtin_amdgcn_readlane(hi, l);
        T part[V];
#pragma unroll
        for (int v = 0; v < V; ++v) part[v] = (T)0;
        for (int p = rlo + lane / G; p < rhi; p += WAVE / G) fma_row<T, V>(part, val[p], xc + (int64_t)col[p] * ldk);
#pragma unroll
        for (int v = 0; v < V; ++v) {
            T t = part[v];
            for (int o = WAVE / 2; o >= G; o >>= 1) t += __shfl_xor(t, o, WAVE);
            if (lane / G == l / G) acc[v] = t;
        }
    }
    if (rv && (!ACC || hi > lo)) store_row<T, V, ACC>(y + i * ldk + c, acc);
}

// One column panel of the DIA part (DIA, or HDC with kept diagonals).  windows: the kernel with staged windows of X.
// fused: the CSR remainder of an HDC handle is added by the same kernel.
template <typename T, int K>
static mo_status dia_panel(const mo_matrix &a, const T *x, T *y, int64_t ldk, bool windows, bool fused, hipStream_t s)
{
    const int32_t *rp = fused ? a.csr_row_ptr : nullptr;
    if (windows) {
        const size_t lds = (size_t)a.mm_lds_elems * K * sizeof(T);
        hipLaunchKernelGGL((k_spmm_dia_win<T, K>), dim3((unsigned)((a.m + SPMM_ROWS - 1) / SPMM_ROWS)), dim3(SPMM_ROWS * Panel<T, K>::G), lds, s,
                           a.mm_xpos, a.mm_map, (int)a.mm_lds_elems, (const T *)a.dia_val, a.nd, a.ld, a.m, a.n, ldk, rp, a.csr_col,
                           (const T *)a.csr_val, x, y);
    } else {
        constexpr int RPB = Panel<T, K>::ROWS;
        hipLaunchKernelGGL((k_spmm_dia<T, K>), dim3((unsigned)((a.m + RPB - 1) / RPB)), dim3(MB), 0, s, a.dia_off, (const T *)a.dia_val,
                           a.nd, a.ld, a.m, a.n, ldk, rp, a.csr_col, (const T *)a.csr_val, x, y);
    }
    MO_LAUNCH_CHECK();
    return MO_OK;
}

// The row-pointer kernel with the smallest stage (256, 512 or 1024 entries per wave) that holds a wave's 64 / G rows
// of average length with a tenth to spare.  Measured with 8 fp64 columns (16 rows per wave): the 27-point stencil (432
// entries per wave) 250 us at 512, 308 at 1024, 389 at 256.
template <typename T, int K, bool ACC>
static void launch_rows(const int32_t *rp, const int32_t *col, const T *val, int64_t m, int64_t part_nnz, int64_t ldk, const T *x, T *y,
                        hipStream_t s)
{
    constexpr int RPB = Panel<T, K>::ROWS, RPW = WAVE / Panel<T, K>::G;
    const unsigned grid = (unsigned)((m + RPB - 1) / RPB);
    const double need = 1.1 * (double)part_nnz / (double)(m > 0 ? m : 1) * RPW;
    if (need <= 256) hipLaunchKernelGGL((k_spmm_rows<T, K, ACC, 256>), dim3(grid), dim3(MB), 0, s, rp, col, val, m, ldk, x, y);
    else if (need <= 512) hipLaunchKernelGGL((k_spmm_rows<T, K, ACC, 512>), dim3(grid), dim3(MB), 0, s, rp, col, val, m, ldk, x, y);
    else hipLaunchKernelGGL((k_spmm_rows<T, K, ACC, 1024>), dim3(grid), dim3(MB), 0, s, rp, col, val, m, ldk, x, y);
}

// One column panel of everything that is not a DIA part.  after_dia: the DIA part of an HDC handle has already
// written this panel of Y, the remainder is added to it.
template <typename T, int K>
static mo_status rest_panel(const mo_matrix &a, const T *x, T *y, int64_t ldk, bool after_dia, hipStream_t s)
{
    constexpr int RPB = Panel<T, K>::ROWS;
    const unsigned grid = (unsigned)((a.m + RPB - 1) / RPB);
    switch (a.fmt) {
    case MO_DIA:
        return MO_OK;
    case MO_ELL:
    case MO_HYB:
    {
        const bool fused = a.fmt == MO_HYB && a.nnz_coo > 0 && a.hyb_max_surplus <= HYB_FUSED_MAX_SURPLUS && a.coo_rp;
        hipLaunchKernelGGL((k_spmm_ell<T, K>), dim3(grid), dim3(MB), 0, s, a.ell_col, (const T *)a.ell_val, a.k, a.ld, a.m, ldk,
                           fused ? a.coo_rp : (const int32_t *)nullptr, a.coo_col, (const T *)a.coo_val, x, y);
        MO_LAUNCH_CHECK();
        if (a.fmt == MO_HYB && a.nnz_coo > 0 && !fused) {
            launch_rows<T, K, true>(a.coo_rp, a.coo_col, (const T *)a.coo_val, a.m, a.nnz_coo, ldk, x, y, s);
            MO_LAUNCH_CHECK();
        }
        return MO_OK;
    }
    case MO_COO:
        launch_rows<T, K, false>(a.coo_rp, a.coo_col, (const T *)a.coo_val, a.m, a.nnz_coo, ldk, x, y, s);
        MO_LAUNCH_CHECK();
        return MO_OK;
    case MO_CSR:
        launch_rows<T, K, false>(a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, a.nnz_csr, ldk, x, y, s);
        MO_LAUNCH_CHECK();
        return MO_OK;
    case MO_HDC:
        if (!after_dia) {
            launch_rows<T, K, false>(a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, a.nnz_csr, ldk, x, y, s);
            MO_LAUNCH_CHECK();
        } else if (a.nnz_csr > 0) {
            launch_rows<T, K, true>(a.csr_row_ptr, a.csr_col, (const T *)a.csr_val, a.m, a.nnz_csr, ldk, x, y, s);
            MO_LAUNCH_CHECK();
        }
        return MO_OK;
    }
    return MO_E_FORMAT;
}

template <typename T>
static mo_status spmm_typed(const mo_matrix &a, const T *x, T *y, int k, hipStream_t s)
{
    const bool dia = a.fmt == MO_DIA || (a.fmt == MO_HDC && a.nd > 0);
    // HDC whose remainder rows are short (the rule of the SpMV dispatch): the DIA kernel adds them itself
    const bool fused = a.fmt == MO_HDC && a.nd > 0 && a.nnz_csr > 0 && a.csr_max_row <= HDC_FUSED_MAX_ROW;
    if (dia) {
        // Windows of X in LDS pay when diagonals share them: at most half as many staged rows as a row has diagonals
        // (27-point stencil on 128^3 points, 9.3 staged rows for 27 diagonals: 259 us with windows, 288 us without;
        // nine diagonals in five windows: 290 against 249 us), and when a panel of at least 4 columns (or all k of
        // them) fits the LDS budget; otherwise the slabs would be streamed too many times.
        int widest = 8;
        bool use_lds = a.mm_lds_elems > 0 && a.mm_lds_elems * 2 <= a.nd * (int64_t)SPMM_ROWS;
        if (use_lds) {
            while (widest > 1 && (size_t)a.mm_lds_elems * widest * sizeof(T) > (size_t)SPMM_WIN_BYTES) widest >>= 1;
            if ((size_t)a.mm_lds_elems * widest * sizeof(T) > (size_t)SPMM_WIN_BYTES || widest < (k < 4 ? k : 4)) { use_lds = false; widest = 8; }
        }
        for (int v0 = 0; v0 < k;) {
            const int left = k - v0 < widest ? k - v0 : widest;
            if (left >= 8) { MO_TRY((dia_panel<T, 8>(a, x + v0, y + v0, k, use_lds, fused, s))); v0 += 8; }
            else if (left >= 4) { MO_TRY((dia_panel<T, 4>(a, x + v0, y + v0, k, use_lds, fused, s))); v0 += 4; }
            else if (left >= 2) { MO_TRY((dia_panel<T, 2>(a, x + v0, y + v0, k, use_lds, fused, s))); v0 += 2; }
            else { MO_TRY((dia_panel<T, 1>(a, x + v0, y + v0, k, use_lds, fused, s))); v0 += 1; }
        }
        if (fused || a.fmt == MO_DIA) return MO_OK;
    }
    for (int v0 = 0; v0 < k;) {
        const int left = k - v0;
        if (left >= 8) { MO_TRY((rest_panel<T, 8>(a, x + v0, y + v0, k, dia, s))); v0 += 8; }
        else if (left >= 4) { MO_TRY((rest_panel<T, 4>(a, x + v0, y + v0, k, dia, s))); v0 += 4; }
        else if (left >= 2) { MO_TRY((rest_panel<T, 2>(a, x + v0, y + v0, k, dia, s))); v0 += 2; }
        else { MO_TRY((rest_panel<T, 1>(a, x + v0, y + v0, k, dia, s))); v0 += 1; }
    }
    return MO_OK;
}

mo_status spmm(const mo_matrix &a, const void *x, void *y, int k, hipStream_t s)
{
    return a.dtype == MO_F32 ? spmm_typed<float>(a, (const float *)x, (float *)y, k, s)
                             : spmm_typed<double>(a, (const double *)x, (double *)y, k, s);
}

}  // namespace mo
