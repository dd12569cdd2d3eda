// Fused multi-round kernel for gfx950 (MI355X): several consecutive averaging
// rounds of Moshpit All-Reduce (the loop of Alg. 1) in ONE pass over HBM.
//
// Columns never interact in a round (the convergence argument of App. C.2 is
// component-wise), and the rows that interact during rounds on F distinct grid
// axes are exactly the M^F vertices of an F-dimensional sub-grid.  So a tile
// made of the M^F rows of one sub-grid and W columns is closed under those
// rounds: it is read from HBM once, all fused rounds run on it in LDS, and it
// is written back once.  When F = d the sub-grid is the whole grid and any
// number of rounds can be fused.
//
// The arithmetic of a round is the one of the single-round kernel, bit for
// bit: values live in LDS in the storage type (so bfloat16 state is rounded
// after every round exactly as if it had gone through HBM), sums are binary32
// over a balanced tree of 16-position blocks, blocks added in ascending order,
// one division by the participant count.
//
// Schedule.  Persistent blocks, 16 waves per compute unit: two blocks of 512
// threads with 80 KiB of LDS each, or, when that lets more axes be fused, one
// block of 1024 threads with 160 KiB.  A thread owns 8 tile slots of 16 bytes
// (512 * 8 * 16 B = 64 KiB, or 128 KiB, of tile).  While the rounds of tile k
// run in LDS the 128-bit loads of tile k+1 are in flight into registers;
// afterwards every thread swaps its slots (tile k to HBM, tile k+1 into LDS)
// and the stores drain during the rounds of tile k+1.  A wave that issues
// vector memory instructions faster than the compute unit's share of HBM
// delivers stalls at the issue stage, and the round barriers pass that stall to
// the whole block; two blocks out of step with each other are what overlaps
// memory time with arithmetic.
//
// LDS layout (dynamic): [tile: rows x Wb bytes][2 x bitmaps: rounds x groups
// u64][byte offset of every local row][2 x row flags: rows bytes][2 x local-step
// flags: rows bytes][tile offset of
// the first row of every group per axis][pad][RN(1/k), k = 0..64][16 bytes of zeros][16 bytes
// of write-only trash].
#include "bf16_round.h"
#include "moshpit_internal.h"

namespace moshpit {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// BPC = blocks per compute unit (1 or 2): a block has 1024 / BPC threads and
// 160 / BPC KiB of LDS, so a compute unit always runs 16 waves on one or two tiles.
constexpr int threads_of(int bpc) { return 1024 / bpc; }
constexpr int lds_of(int bpc) { return 160 * 1024 / bpc; }
constexpr int kRcpBytes = 272;       // 65 reciprocals, padded to a multiple of 16 bytes
constexpr int kNormalOrZero = 0x168;  // v_cmp_class mask: -normal, -0, +0, +normal
constexpr int kMinSeg = 128;          // fewest bytes of a row in a tile
constexpr int kPrefetch = 8;          // 128-bit vectors per thread: 1024 * 8 * 16 B = 128 KiB of tile

// Block barrier that orders LDS traffic only.  __syncthreads() also waits for
// every outstanding global load and store of the wave (its fence covers global
// memory), which would serialise the tile prefetch and the store drain with
// the rounds running in LDS.  Threads of a block exchange data through LDS
// only, so waiting for the LDS counter before the barrier is sufficient.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Lane exchanges without a trip through LDS.  With rows of 16 lanes r0..r3,
//   swap16(a, b) = ([a.r0, b.r0, a.r2, b.r2], [a.r1, b.r1, a.r3, b.r3])
//   swap32(a, b) = ([a.r0, a.r1, b.r0, b.r1], [a.r2, a.r3, b.r2, b.r3])
// (v_permlane16_swap / v_permlane32_swap).  Adding the two results of a swap of
// two DIFFERENT values reduces both across a pair of rows at once and leaves
// one of them in each row of the pair: the transposing reduction used below.
struct LanePair { float first, second; };
__device__ __forceinline__ LanePair swap16(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return LanePair{__uint_as_float(r[0]), __uint_as_float(r[1])};
}
__device__ __forceinline__ LanePair swap32(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return LanePair{__uint_as_float(r[0]), __uint_as_float(r[1])};
}

// CV consecutive columns of one row in LDS, widened to binary32.
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <int DT, int CV> struct Cols;
template <> struct Cols<0, 4> {
    typedef float elem_t;
    static __device__ __forceinline__ void load(const elem_t *p, float (&f)[4])
    {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    static __device__ __forceinline__ void store(elem_t *p, const float (&f)[4])
    {
        *reinterpret_cast<f32x4 *>(p) = f32x4{f[0], f[1], f[2], f[3]};
    }
};
template <> struct Cols<0, 2> {
    typedef float elem_t;
    static __device__ __forceinline__ void load(const elem_t *p, float (&f)[2])
    {
        const f32x2 v = *reinterpret_cast<const f32x2 *>(p);
        f[0] = v.x; f[1] = v.y;
    }
    static __device__ __forceinline__ void store(elem_t *p, const float (&f)[2])
    {
        *reinterpret_cast<f32x2 *>(p) = f32x2{f[0], f[1]};
    }
};
template <> struct Cols<0, 1> {
    typedef float elem_t;
    static __device__ __forceinline__ void load(const elem_t *p, float (&f)[1]) { f[0] = *p; }
    static __device__ __forceinline__ void store(elem_t *p, const float (&f)[1]) { *p = f[0]; }
};
template <> struct Cols<1, 4> {
    typedef uint16_t elem_t;
    static __device__ __forceinline__ void load(const elem_t *p, float (&f)[4])
    {
        const u32x2 v = *reinterpret_cast<const u32x2 *>(p);
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(elem_t *p, const float (&f)[4])
    {
        *reinterpret_cast<u32x2 *>(p) = u32x2{bf16_pair(f[0], f[1]), bf16_pair(f[2], f[3])};
    }
};
template <> struct Cols<1, 2> {
    typedef uint16_t elem_t;
    static __device__ __forceinline__ void load(const elem_t *p, float (&f)[2])
    {
        const uint32_t v = *reinterpret_cast<const uint32_t *>(p);
        f[0] = __uint_as_float(v << 16); f[1] = __uint_as_float(v & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(elem_t *p, const float (&f)[2])
    {
        *reinterpret_cast<uint32_t *>(p) = bf16_pair(f[0], f[1]);
    }
};
template <> struct Cols<1, 1> {
    typedef uint16_t elem_t;
    static __device__ __forceinline__ void load(const elem_t *p, float (&f)[1])
    {
        f[0] = __uint_as_float(static_cast<uint32_t>(*p) << 16);
    }
    static __device__ __forceinline__ void store(elem_t *p, const float (&f)[1])
    {
        *p = bf16_one(f[0]);
    }
};

// One 16-byte tile slot (4 binary32 or 8 bfloat16 values) after a local step of
// Moshpit SGD (Alg. 2): x - gamma * g, formed in binary32 with one fused multiply-add
// per value and rounded to the storage type.
template <int DT> __device__ __forceinline__ u32x4 local_step(const u32x4 &x, const u32x4 &g, float gamma)
{
    if constexpr (DT == 0) {
        u32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            out[e] = __float_as_uint(__fmaf_rn(-gamma, __uint_as_float(g[e]), __uint_as_float(x[e])));
        return out;
    } else {
        u32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float lo = __fmaf_rn(-gamma, __uint_as_float(g[e] << 16), __uint_as_float(x[e] << 16));
            const float hi = __fmaf_rn(-gamma, __uint_as_float(g[e] & 0xffff0000u), __uint_as_float(x[e] & 0xffff0000u));
            out[e] = bf16_pair(lo, hi);
        }
        return out;
    }
}

// global row of local row lr: base + sum_f digit_f(lr) * gstride[f]
__device__ __forceinline__ int64_t global_row(const FusedPlan &p, int64_t base, int32_t lr)
{
    int64_t row = base;
    int32_t rest = lr;
    for (int f = 0; f < p.F; ++f) {
        const int32_t digit = rest % p.M;
        rest /= p.M;
        row += digit * p.gstride[f];
    }
    return row;
}

struct TileRef {
    int64_t plane;         // which sub-grid
    int64_t base;          // first global row of the sub-grid
    int64_t col0_bytes;    // first byte of the column slice within a row
    int32_t seg_bytes;     // bytes of the slice that exist (last slice may be short)
};

__device__ __forceinline__ TileRef tile_ref(const FusedPlan &p, int64_t w)
{
    TileRef t;
    const int64_t plane = w / p.tiles;
    const int64_t ctile = w - plane * p.tiles;
    t.plane = plane;
    t.base = 0;
    int64_t rest = plane;
    for (int o = 0; o < p.n_outer; ++o) {
        t.base += (rest % p.M) * p.ostride[o];
        rest /= p.M;
    }
    t.col0_bytes = ctile * p.Wb;
    const int64_t left = p.row_valid_bytes - t.col0_bytes;
    t.seg_bytes = static_cast<int32_t>(left < p.Wb ? left : p.Wb);
    return t;
}

// Sum of TREE positions j0..j0+TREE-1 of CV columns of a group, as the balanced
// tree ((x0+x1)+(x2+x3))+...; positions whose bit is clear (absent peers, and
// positions past the group, whose bits are never set) contribute an exact 0:
// their read is redirected to `zeros`, 16 bytes of LDS that hold 0, which costs
// one select per position instead of one per value.  Blocks of up to FLAT
// positions are read at once; larger trees are the sum of their two balanced
// halves, which bounds the register footprint.
template <int DT, int CV, int TREE, int FLAT>
__device__ __forceinline__ void tree_block(const typename Cols<DT, CV>::elem_t *col, int32_t step, int32_t j0,
                                           const typename Cols<DT, CV>::elem_t *zeros, uint32_t bits,
                                           float (&out)[CV])
{
    if constexpr (TREE > FLAT) {
        float lo[CV], hi[CV];
        tree_block<DT, CV, TREE / 2, FLAT>(col, step, j0, zeros, bits & ((1u << (TREE / 2)) - 1u), lo);
        tree_block<DT, CV, TREE / 2, FLAT>(col, step, j0 + TREE / 2, zeros, bits >> (TREE / 2), hi);
#pragma unroll
        for (int e = 0; e < CV; ++e) out[e] = lo[e] + hi[e];
    } else {
        float f[TREE][CV];
#pragma unroll
        for (int u = 0; u < TREE; ++u) {
            const bool on = (bits >> u) & 1u;
            Cols<DT, CV>::load(on ? col + (j0 + u) * step : zeros, f[u]);
        }
#pragma unroll
        for (int s = 1; s < TREE; s *= 2)
#pragma unroll
            for (int u = 0; u + s < TREE; u += 2 * s)
#pragma unroll
                for (int e = 0; e < CV; ++e) f[u][e] += f[u + s][e];
#pragma unroll
        for (int e = 0; e < CV; ++e) out[e] = f[0][e];
    }
}

// TREE = size of the summation block actually needed: 16 for M > 8, else the
// next power of two >= M (a 16-block padded with zeros gives the same bits).
// CV = columns one thread averages at a time; SPLIT = lanes of a wave that share
// the positions of one group (chosen so that every thread has work even when
// the tile is narrow).
template <int DT, int TREE, int CV, int SPLIT, int PER, int BPC>
__global__ __launch_bounds__(threads_of(BPC)) __attribute__((amdgpu_waves_per_eu(4, 4))) void fused_rounds_kernel(
    char *X, const uint8_t *__restrict__ masks, FusedPlan p)
{
    constexpr int kThreads = threads_of(BPC);
    typedef Cols<DT, CV> Q;
    typedef typename Q::elem_t elem_t;
    constexpr int FLAT = 16 / CV;
    extern __shared__ __align__(16) char lds[];
    char *tile = lds;
    const int32_t bm_count = p.rounds * p.groups;
    uint64_t *bitmaps0 = reinterpret_cast<uint64_t *>(lds + p.tile_bytes);
    int64_t *rowoff = reinterpret_cast<int64_t *>(bitmaps0 + 2 * bm_count);      // byte offset of local row lr
    uint8_t *rowflag0 = reinterpret_cast<uint8_t *>(rowoff + p.rows_padded);
    uint8_t *rowstep0 = rowflag0 + 2 * p.rows_padded;             // rows that take the local step (SGD pass)
    int32_t *lbase_tab = reinterpret_cast<int32_t *>(rowstep0 + 2 * p.rows_padded);
    float *rcp_tab = reinterpret_cast<float *>(lds + p.lds_bytes - 32 - kRcpBytes);  // RN(1 / k), k = 0..64
    elem_t *zeros = reinterpret_cast<elem_t *>(lds + p.lds_bytes - 32);            // 16 bytes that hold 0
    elem_t *trash = reinterpret_cast<elem_t *>(lds + p.lds_bytes - 16);            // 16 bytes nobody reads

    const int tid = threadIdx.x;

    // first local row of group gl on local axis f
    for (int32_t i = tid; i < p.F * p.groups; i += kThreads) {
        const int32_t f = i / p.groups, gl = i - f * p.groups;
        int32_t Sl = 1;
        for (int q = 0; q < f; ++q) Sl *= p.M;
        lbase_tab[i] = ((gl / Sl) * Sl * p.M + (gl % Sl)) * p.Wb;        // as a byte offset into the tile
    }
    for (int32_t lr = tid; lr < p.rows; lr += kThreads) rowoff[lr] = global_row(p, 0, lr) * p.row_bytes;
    if (tid < 4) reinterpret_cast<uint32_t *>(zeros)[tid] = 0u;
    if (tid <= 64) rcp_tab[tid] = tid == 0 ? 0.f : 1.f / static_cast<float>(tid);

    const int32_t Wv = p.Wb / 16;
    const int32_t W = p.Wb / static_cast<int32_t>(sizeof(elem_t));     // columns of a full tile

    // Participant bitmaps of every (round, group) of a sub-grid and per-row
    // "used" flags.  They depend on the sub-grid only, not on the column slice,
    // so a buffer is rebuilt only when the block moves to another sub-grid.
    // One thread per (round, row): independent byte loads, bits merged with LDS
    // atomics.
    int64_t tag0 = -1, tag1 = -1;                    // sub-grid held by buffer 0 / 1
    auto prepare = [&](const TileRef &t, int buf) {
        if ((buf == 0 ? tag0 : tag1) == t.plane) return;
        if (buf == 0) tag0 = t.plane; else tag1 = t.plane;
        unsigned long long *bm = reinterpret_cast<unsigned long long *>(bitmaps0 + buf * bm_count);
        uint8_t *flag = rowflag0 + buf * p.rows_padded;
        uint8_t *step = rowstep0 + buf * p.rows_padded;
        for (int32_t i = tid; i < bm_count; i += kThreads) bm[i] = 0ull;
        for (int32_t lr = tid; lr < p.rows; lr += kThreads) { flag[lr] = 0; step[lr] = 0; }
        lds_barrier();
        const int32_t pairs = p.rounds * p.rows;
        constexpr int kB = 8;
        for (int32_t i0 = tid; i0 < pairs; i0 += kThreads * kB) {
            uint8_t a[kB];
#pragma unroll
            for (int b = 0; b < kB; ++b) {
                const int32_t i = i0 + b * kThreads;
                a[b] = 0;
                if (i < pairs) {
                    const int32_t r = i / p.rows;
                    const int32_t lr = i - r * p.rows;
                    a[b] = masks == nullptr ? 1 : masks[static_cast<int64_t>(r) * p.N + global_row(p, t.base, lr)];
                }
            }
#pragma unroll
            for (int b = 0; b < kB; ++b) {
                const int32_t i = i0 + b * kThreads;
                if (i < pairs && a[b] != 0) {
                    const int32_t r = i / p.rows;
                    const int32_t lr = i - r * p.rows;
                    const int32_t lf = (p.local_axis0 + r) % p.F;
                    int32_t Sl = 1;
                    for (int q = 0; q < lf; ++q) Sl *= p.M;
                    const int32_t j = (lr / Sl) % p.M;
                    const int32_t gl = (lr / (Sl * p.M)) * Sl + lr % Sl;
                    atomicOr(&bm[r * p.groups + gl], 1ull << j);
                    flag[lr] = 1;                      // benign race: every writer stores 1
                    if (r == 0) step[lr] = 1;          // (one writer: the thread of (round 0, lr))
                }
            }
        }
        lds_barrier();
    };

    // Slot b of a thread is vector idx = tid + b * kThreads of the tile, i.e.
    // local row idx / Wv, vector idx % Wv; walked incrementally.  The opaque
    // copy of tid keeps this index arithmetic inside the tile loop instead of
    // having all of it hoisted into registers that live across the rounds.
    const int32_t slot_dq = kThreads / Wv, slot_dr = kThreads - slot_dq * Wv;

    // Issue the 128-bit loads of slots [b_lo, b_hi) of a tile into registers and
    // add them to the mask of slots in use.  The load is written as an asm
    // statement so that the compiler does not track it: for a load of its own,
    // issued in a loop into a register that an earlier iteration may have left
    // pending, it waits for ALL memory traffic first, which would serialise
    // every load behind the stores of the previous tile.  In exchange the wait
    // is ours to place: nothing may read or copy pre[] between fetch() and the
    // vmcnt(0) wait that precedes the swap (each pre[b] is an in-out operand, so
    // the load lands in the register that holds the variable).
    u32x4 pre[kPrefetch];
#pragma unroll
    for (int b = 0; b < kPrefetch; ++b) pre[b] = u32x4{0u, 0u, 0u, 0u};
    auto fetch = [&](const TileRef &t, int buf, int b_lo, int b_hi, uint32_t &used) {
        const uint8_t *flag = rowflag0 + buf * p.rows_padded;
        const int32_t seg_vec = t.seg_bytes / 16;
        const char *origin = X + t.base * p.row_bytes + t.col0_bytes;
        int32_t t_ = tid;
        asm volatile("" : "+v"(t_));
        int32_t lr = t_ / Wv, v = t_ - lr * Wv;
#pragma unroll
        for (int b = 0; b < kPrefetch; ++b) {
            if (b >= b_lo && b < b_hi && lr < p.rows && v < seg_vec && flag[lr]) {
                const char *src = origin + rowoff[lr] + v * 16;
                asm volatile("global_load_dwordx4 %0, %1, off nt" : "+v"(pre[b]) : "v"(src));
                used |= 1u << b;
            }
            v += slot_dr;
            lr += slot_dq;
            if (v >= Wv) { v -= Wv; lr += 1; }
        }
    };

    // The fused rounds of one tile, in LDS, with the bitmaps of buffer `buf`.
    // after_round(r) runs once the barrier of round r has been passed.
    auto compute = [&](const TileRef &t, int buf, auto after_round) {
        const uint64_t *bm = bitmaps0 + buf * bm_count;
        const int32_t cchunks = t.seg_bytes / (CV * static_cast<int32_t>(sizeof(elem_t)));
        // SPLIT adjacent lanes share one (group, column chunk) item and take
        // SPLIT equal parts of its positions
        // (sub is the slow lane index, so 8 consecutive lanes read 128 contiguous
        // bytes of one row: no LDS bank conflicts)
        constexpr int kItemThreads = kThreads / SPLIT;
        constexpr int kLanesPerSub = 64 / SPLIT;
        const int32_t sub = (tid & 63) / kLanesPerSub;
        const int32_t it0 = (tid >> 6) * kLanesPerSub + (tid & (kLanesPerSub - 1));
        const int32_t g_first = it0 / cchunks, c_first = it0 - g_first * cchunks;
        const int32_t dg = kItemThreads / cchunks, dc = kItemThreads - dg * cchunks;
        for (int32_t r = 0; r < p.rounds; ++r) {
            const int32_t lf = (p.local_axis0 + r) % p.F;
            int32_t Sl = 1;
            for (int q = 0; q < lf; ++q) Sl *= p.M;
            const int32_t step = Sl * W;
            const int32_t *lb = lbase_tab + lf * p.groups;
            const uint64_t *bmr = bm + r * p.groups;
            int32_t gl = g_first, cc = c_first;
            while (gl < p.groups) {
                const uint64_t live = bmr[gl];
                int32_t lbase = lb[gl];
                asm volatile("" : "+v"(lbase));        // keeps this read next to the bitmap's: one LDS latency, not two
                const int cnt = __popcll(live);
                if (cnt >= 2) {
                    [[maybe_unused]] float y = 0.f;    // RN(1 / cnt), read along with the rows
                    if constexpr (SPLIT == 1 && CV > 1) y = rcp_tab[cnt];
                    elem_t *col = reinterpret_cast<elem_t *>(tile + lbase) + cc * CV;
                    float acc[CV];
#pragma unroll
                    for (int e = 0; e < CV; ++e) acc[e] = 0.f;
                    elem_t *pos[SPLIT > 1 ? PER : 1];  // where this thread's positions are written back (SPLIT > 1)
                    if constexpr (SPLIT > 1) {
                        // M <= 32 here: SPLIT * PER = 16 or 32 positions (one or two
                        // 16-position blocks) cut into SPLIT balanced sub-trees of PER
                        // positions; the butterfly over the SPLIT lanes adds them in the
                        // order of the full tree.  All PER row reads are issued before
                        // the first use; the opaque copy of the row step keeps the
                        // per-position addresses out of registers that live across items.
                        int32_t st = step;
                        asm volatile("" : "+s"(st));
                        const int32_t j0 = sub * PER;
                        const uint32_t pbits = static_cast<uint32_t>(live >> j0) & ((1u << PER) - 1u);
                        elem_t *q = col + __mul24(j0, st);
                        float f[PER][CV];
#pragma unroll
                        for (int u = 0; u < PER; ++u) {
                            // absent peers and positions past the group read the zeros,
                            // and their (unconditional) store goes to the trash
                            const bool on = (pbits >> u) & 1u;
                            Q::load(on ? q : zeros, f[u]);
                            pos[u] = on ? q : trash;
                            q += st;
                        }
#pragma unroll
                        for (int w2 = 1; w2 < PER; w2 *= 2)
#pragma unroll
                            for (int u = 0; u + w2 < PER; u += 2 * w2)
#pragma unroll
                                for (int e = 0; e < CV; ++e) f[u][e] += f[u + w2][e];
                        // The SPLIT lanes of an item hold partial sums of its 4 columns.  They
                        // are added across lanes so that each lane ends with the total of ONE
                        // column (same order as the full tree: (s0 + s1) + (s2 + s3)), divides
                        // that one, and the quotients are handed round: 6 (4) exchanges and 1
                        // (2) divisions per lane instead of 8 (4) exchanges and 4 divisions.
                        static_assert(CV == 4, "lane-split items work on 4 columns");
                        const float k = static_cast<float>(cnt);
                        if constexpr (SPLIT == 4) {
                            const LanePair a = swap16(f[0][0], f[0][1]);    // rows 0, 2: column 0; rows 1, 3: column 1
                            const LanePair b = swap16(f[0][2], f[0][3]);    // rows 0, 2: column 2; rows 1, 3: column 3
                            const LanePair c = swap32(a.first + a.second, b.first + b.second);
                            const float mean = (0.f + (c.first + c.second)) / k;    // row r: column r
                            const LanePair eo = swap16(mean, mean);         // columns 0|2 and 1|3 of my half
                            const LanePair m02 = swap32(eo.first, eo.first);
                            const LanePair m13 = swap32(eo.second, eo.second);
                            acc[0] = m02.first; acc[1] = m13.first; acc[2] = m02.second; acc[3] = m13.second;
                        } else {
                            const LanePair a = swap32(f[0][0], f[0][1]);    // lower half: column 0, upper: column 1
                            const LanePair b = swap32(f[0][2], f[0][3]);    // lower half: column 2, upper: column 3
                            const float q01 = (0.f + (a.first + a.second)) / k;
                            const float q23 = (0.f + (b.first + b.second)) / k;
                            const LanePair m01 = swap32(q01, q01);
                            const LanePair m23 = swap32(q23, q23);
                            acc[0] = m01.first; acc[1] = m01.second; acc[2] = m23.first; acc[3] = m23.second;
                        }
                    } else if constexpr (TREE < 16) {
                        float t0[CV];
                        tree_block<DT, CV, TREE, FLAT>(col, step, 0, zeros, static_cast<uint32_t>(live), t0);
#pragma unroll
                        for (int e = 0; e < CV; ++e) acc[e] += t0[e];
                    } else {
                        for (int32_t j0 = 0; j0 < p.M; j0 += 16) {
                            const uint32_t bits = static_cast<uint32_t>(live >> j0) & 0xffffu;
                            if (bits == 0) continue;
                            float t16[CV];
                            tree_block<DT, CV, 16, FLAT>(col, step, j0, zeros, bits, t16);
#pragma unroll
                            for (int e = 0; e < CV; ++e) acc[e] += t16[e];
                        }
                    }
                    if constexpr (SPLIT == 1 && CV > 1) {
                        // acc / k for CV columns, sharing the reciprocal y = RN(1/k) (a table in
                        // LDS, filled by true divisions): q0 = RN(acc * y), the exact remainder
                        // r = acc - k * q0 (one fma), q = RN(q0 + r * y) is the correctly rounded
                        // quotient whenever nothing underflows.  A q that is not a normal number
                        // or zero (NaN from an infinite sum, subnormal) is redone with a true
                        // division.  With this guard the sequence was compared with the division
                        // for every count k <= 64 and all 2^32 binary32 numerators: the only
                        // difference is -0 / k, and acc is never -0 (it starts from +0).
                        const float k = static_cast<float>(cnt);
                        float quo[CV];
                        bool redo = false;
#pragma unroll
                        for (int e = 0; e < CV; ++e) {
                            const float q0 = __fmul_rn(acc[e], y);
                            const float r = __fmaf_rn(-k, q0, acc[e]);
                            quo[e] = __fmaf_rn(r, y, q0);
                            redo = redo || !__builtin_amdgcn_classf(quo[e], kNormalOrZero);
                        }
                        if (redo) {
#pragma unroll
                            for (int e = 0; e < CV; ++e) quo[e] = acc[e] / k;
                        }
#pragma unroll
                        for (int e = 0; e < CV; ++e) acc[e] = quo[e];
                    } else if constexpr (SPLIT == 1) {
                        acc[0] = acc[0] / static_cast<float>(cnt);
                    }
                    if constexpr (SPLIT > 1) {
#pragma unroll
                        for (int u = 0; u < PER; ++u) Q::store(pos[u], acc);
                    } else if constexpr (TREE < 16) {
                        // at most 8 positions: straight-line predicated stores
                        const uint32_t wbits = static_cast<uint32_t>(live);
#pragma unroll
                        for (int u = 0; u < TREE; ++u)
                            if ((wbits >> u) & 1u) Q::store(col + u * step, acc);
                    } else {
                        // unconditional stores, 16 positions at a time; those of absent
                        // peers and of positions past the group go to the trash
                        for (int32_t j0 = 0; j0 < p.M; j0 += 16) {
                            const uint32_t wbits = static_cast<uint32_t>(live >> j0);
#pragma unroll
                            for (int u = 0; u < 16; ++u)
                                Q::store(((wbits >> u) & 1u) ? col + (j0 + u) * step : trash, acc);
                        }
                    }
                }
                cc += dc;
                gl += dg;
                if (cc >= cchunks) { cc -= cchunks; gl += 1; }
            }
            lds_barrier();
            after_round(r);
        }
    };

    // Software pipeline over the block's tiles k = 0, 1, 2, ...  While tile k is
    // averaged in LDS, the loads of tile k+1 are issued into `pre` (before the
    // first round, or in `spread` portions after the first rounds).  Afterwards
    // tile k leaves LDS for HBM and tile k+1 enters LDS from `pre`; the stores
    // drain while tile k+1 is averaged.
    const int64_t stride = gridDim.x;
    int64_t w = blockIdx.x;
    if (w >= p.work_items) return;
    TileRef cur = tile_ref(p, w);
    int buf_cur = 0;
    prepare(cur, buf_cur);
    uint32_t used_cur = 0;
    fetch(cur, buf_cur, 0, kPrefetch, used_cur);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int b = 0; b < kPrefetch; ++b) asm volatile("" : "+v"(pre[b]));
#pragma unroll
    for (int b = 0; b < kPrefetch; ++b)
        if (used_cur & (1u << b)) *reinterpret_cast<u32x4 *>(tile + static_cast<int64_t>(tid + b * kThreads) * 16) = pre[b];
    // Moshpit SGD pass: the rows that are present in the pass's first round take their local
    // step on the way in.  A thread rewrites its own tile slots only, so no barrier is needed
    // between the tile's arrival in LDS and this.  (First tile of the block: gradient loads not
    // overlapped with anything.)
    if (p.grad != nullptr) {
        const uint8_t *step = rowstep0 + buf_cur * p.rows_padded;
        const char *g_origin = p.grad + cur.base * p.row_bytes + cur.col0_bytes;
        int32_t lr = tid / Wv, v = tid - lr * Wv;
#pragma unroll
        for (int b = 0; b < kPrefetch; ++b) {
            if ((used_cur & (1u << b)) && step[lr]) {
                u32x4 *slot = reinterpret_cast<u32x4 *>(tile + static_cast<int64_t>(tid + b * kThreads) * 16);
                const u32x4 g = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(g_origin + rowoff[lr] + v * 16));
                *slot = local_step<DT>(*slot, g, p.gamma);
            }
            v += slot_dr;
            lr += slot_dq;
            if (v >= Wv) { v -= Wv; lr += 1; }
        }
    }
    lds_barrier();

    while (true) {
        const bool has_next = w + stride < p.work_items;
        TileRef nxt = cur;
        int buf_next = buf_cur;
        uint32_t used_next = 0;
        if (has_next) {
            nxt = tile_ref(p, w + stride);
            buf_next = nxt.plane == cur.plane ? buf_cur : buf_cur ^ 1;
            prepare(nxt, buf_next);
        }
        // spread == 0: all slots of tile k+1 before the first round; otherwise slots
        // [r * kPrefetch / spread, (r + 1) * kPrefetch / spread) after round r < spread
        const int32_t spread = p.rounds < p.spread ? p.rounds : p.spread;
        if (has_next && p.spread == 0) fetch(nxt, buf_next, 0, kPrefetch, used_next);
        compute(cur, buf_cur, [&](int32_t r) {
            if (has_next && r < spread)
                fetch(nxt, buf_next, r * kPrefetch / spread, (r + 1) * kPrefetch / spread, used_next);
        });

        // Wait for the loads of tile k+1 (and, in passing, for the stores of tile
        // k-1); the empty asm statements keep every use of pre[] below the wait.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int b = 0; b < kPrefetch; ++b) asm volatile("" : "+v"(pre[b]));
        // Each thread owns the same tile slots for every tile, so it swaps tile
        // k out of LDS and tile k+1 in, slot by slot, without a barrier.
        constexpr int kHalf = kPrefetch / 2;
        {
            char *origin = X + cur.base * p.row_bytes + cur.col0_bytes;
            int32_t t_ = tid;
            asm volatile("" : "+v"(t_));
            int32_t lr = t_ / Wv, v = t_ - lr * Wv;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                u32x4 val[kHalf];
#pragma unroll
                for (int q = 0; q < kHalf; ++q) {
                    const int b = h * kHalf + q;
                    u32x4 *slot = reinterpret_cast<u32x4 *>(tile + static_cast<int64_t>(t_ + b * kThreads) * 16);
                    if (used_cur & (1u << b)) val[q] = *slot;
                    if (used_next & (1u << b)) *slot = pre[b];
                }
#pragma unroll
                for (int q = 0; q < kHalf; ++q) {
                    const int b = h * kHalf + q;
                    if (used_cur & (1u << b))
                        __builtin_nontemporal_store(val[q], reinterpret_cast<u32x4 *>(origin + rowoff[lr] + v * 16));
                    v += slot_dr;
                    lr += slot_dq;
                    if (v >= Wv) { v -= Wv; lr += 1; }
                }
            }
        }
        // Moshpit SGD pass: the rows of the incoming tile that are present in the pass's first
        // round take their local step, two slots at a time (few registers are free here): the
        // gradients are requested, waited for, and the slots rewritten in LDS by their owner.
        if (p.grad != nullptr && has_next) {
            const uint8_t *step = rowstep0 + buf_next * p.rows_padded;
            const char *g_origin = p.grad + nxt.base * p.row_bytes + nxt.col0_bytes;
            int32_t t_ = tid;
            asm volatile("" : "+v"(t_));
            int32_t lr = t_ / Wv, v = t_ - lr * Wv;
            constexpr int kBatch = 2;
#pragma unroll
            for (int b0 = 0; b0 < kPrefetch; b0 += kBatch) {
                u32x4 grad[kBatch];
                uint32_t stepping = 0;
#pragma unroll
                for (int q = 0; q < kBatch; ++q) {
                    if ((used_next & (1u << (b0 + q))) && step[lr]) {
                        grad[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(g_origin + rowoff[lr] + v * 16));
                        stepping |= 1u << q;
                    }
                    v += slot_dr;
                    lr += slot_dq;
                    if (v >= Wv) { v -= Wv; lr += 1; }
                }
#pragma unroll
                for (int q = 0; q < kBatch; ++q) {
                    if (stepping & (1u << q)) {
                        u32x4 *slot = reinterpret_cast<u32x4 *>(tile + static_cast<int64_t>(t_ + (b0 + q) * kThreads) * 16);
                        *slot = local_step<DT>(*slot, grad[q], p.gamma);
                    }
                }
            }
        }
        if (!has_next) break;
        lds_barrier();
        w += stride;
        cur = nxt;
        used_cur = used_next;
        buf_cur = buf_next;
    }
}

int tree_size(int32_t M) { return M > 8 ? 16 : M > 4 ? 8 : M > 2 ? 4 : 2; }

int64_t fixed_lds(int64_t rounds, int64_t rows, int64_t groups, int64_t F)
{
    const int64_t rows_padded = (rows + 15) / 16 * 16;
    // tables, slack, then (16-byte aligned) the reciprocals, 16 bytes of zeros, 16 bytes of write-only trash
    return (2 * rounds * groups * 8 + rows_padded * 8 + 4 * rows_padded + F * groups * 4 + 32 + 15) / 16 * 16 +
           kRcpBytes + 32;
}

}  // namespace

namespace {

bool plan_with(int bpc, int dtype, int64_t N, int32_t M, int32_t d, int64_t P, int64_t row_stride, const void *X,
               int64_t t0, int32_t rounds_wanted, FusedPlan *out)
{
    const int kThreads = threads_of(bpc);
    const int kLdsBytes = lds_of(bpc);
    const int64_t esize = dtype == 0 ? 4 : 2;
    const int64_t row_bytes = row_stride * esize;
    const int64_t valid = P * esize;
    if (rounds_wanted < 2) return false;
    if (reinterpret_cast<uintptr_t>(X) % 16 != 0 || row_bytes % 16 != 0 || valid % 16 != 0) return false;

    // widest sub-grid (most axes) whose rows still get >= 128 bytes each
    int F = 1;
    int64_t rows = M;
    while (F < d && F < rounds_wanted && F < kFusedMaxAxes) {
        const int64_t next = rows * M;
        const int64_t min_rounds = (F + 1 == d) ? 2 : (F + 1);
        if (next * kMinSeg + fixed_lds(min_rounds, next, next / M, F + 1) > kLdsBytes) break;
        if (next * kMinSeg > static_cast<int64_t>(kThreads) * kPrefetch * 16) break;
        rows = next;
        ++F;
    }
    if (F < 2) return false;                    // one axis per pass is the single-round kernel

    FusedPlan p{};
    p.N = N; p.M = M; p.F = F;
    p.rows = static_cast<int32_t>(rows);
    p.rows_padded = static_cast<int32_t>((rows + 15) / 16 * 16);
    p.groups = static_cast<int32_t>(rows / M);
    p.row_bytes = row_bytes;
    p.row_valid_bytes = valid;
    int32_t rounds = rounds_wanted;
    if (F < d) {
        rounds = F;                              // the tile is closed under exactly these F axes
        p.local_axis0 = 0;
        for (int f = 0; f < F; ++f) {
            int64_t S = 1;
            for (int64_t q = 0; q < (t0 + f) % d; ++q) S *= M;
            p.gstride[f] = S;
        }
        // outer axes: every grid axis not among the fused ones, ascending
        p.n_outer = 0;
        for (int a = 0; a < d; ++a) {
            bool inside = false;
            for (int f = 0; f < F; ++f) inside = inside || ((t0 + f) % d == a);
            if (inside) continue;
            int64_t S = 1;
            for (int q = 0; q < a; ++q) S *= M;
            p.ostride[p.n_outer++] = S;
        }
    } else {
        // whole grid in the tile: local axis f is grid axis f, any number of rounds
        p.local_axis0 = static_cast<int32_t>(t0 % d);
        int64_t S = 1;
        for (int f = 0; f < F; ++f) { p.gstride[f] = S; S *= M; }
        p.n_outer = 0;
        const int64_t max_rounds = 8192 / (static_cast<int64_t>(p.groups) * 8);    // <= 16 KiB of bitmaps
        if (rounds > max_rounds) rounds = static_cast<int32_t>(max_rounds);
        if (rounds < 2) return false;
    }
    p.rounds = rounds;
    // One block per compute unit means many rows of few bytes each (1024 x 128 B on a
    // 32 x 32 grid): HBM serves that pattern at little more than half the rate of the
    // single-round kernel, so a pass of only two rounds is slower than two single rounds
    // (measured: 10.6 ms against 9.0 ms on 16 GiB); from three rounds on the pass wins.
    if (bpc == 1 && rounds < 3) return false;
    // When the loads of the next tile are issued (measured on MI355X): two blocks per
    // compute unit do best issuing them all before the first round; a block that has the
    // compute unit to itself issues them in 2 or 4 portions, one after each of the first
    // rounds, once there are enough rounds to spread them over.
    p.spread = bpc == 1 ? (rounds >= 7 ? 4 : rounds >= 5 ? 2 : 0) : 0;
    const int64_t fixed = fixed_lds(rounds, rows, p.groups, F);
    int64_t budget = kLdsBytes - fixed;                          // LDS left for the tile ...
    const int64_t reg_tile = static_cast<int64_t>(kThreads) * kPrefetch * 16;   // ... and what the prefetch registers hold
    if (budget > reg_tile) budget = reg_tile;
    int64_t wb = budget / rows;
    wb = wb >= kMinSeg ? wb / kMinSeg * kMinSeg : 0;
    if (wb < kMinSeg) return false;
    if (wb > valid) wb = valid;                  // a multiple of 16 (checked above)
    // small states: narrower tiles so that every compute unit gets a few of them
    const int64_t planes_total = N / rows;
    while (wb >= 1024 && planes_total * ((valid + wb - 1) / wb) < 1024) wb = wb / 2 / 128 * 128;
    if (rows * (wb / 16) > static_cast<int64_t>(kThreads) * kPrefetch) return false;
    p.Wb = static_cast<int32_t>(wb);
    p.tile_bytes = static_cast<int32_t>(rows * wb);
    p.lds_bytes = static_cast<int32_t>(p.tile_bytes + fixed);
    p.tiles = (valid + wb - 1) / wb;
    p.planes = N / rows;
    p.work_items = p.planes * p.tiles;
    p.blocks_per_cu = bpc;
    *out = p;
    return true;
}

}  // namespace

// Two blocks per compute unit run out of step with each other, which hides a
// good part of the time a block spends issuing its loads and stores; one block
// per compute unit has twice the LDS for its tile and is taken when that lets
// more axes be fused (M^F rows of >= 128 bytes must fit).
bool plan_fused(int dtype, int64_t N, int32_t M, int32_t d, int64_t P, int64_t row_stride, const void *X,
                int64_t t0, int32_t rounds_wanted, FusedPlan *out)
{
    FusedPlan two{}, one{};
    const bool ok2 = plan_with(2, dtype, N, M, d, P, row_stride, X, t0, rounds_wanted, &two);
    const bool ok1 = plan_with(1, dtype, N, M, d, P, row_stride, X, t0, rounds_wanted, &one);
    if (!ok1 && !ok2) return false;
    *out = (ok2 && (!ok1 || two.F >= one.F)) ? two : one;
    return true;
}

namespace {

template <int BPC>
hipError_t launch_with(void *X, int dtype, const FusedPlan &plan, const uint8_t *masks, hipStream_t stream)
{
    constexpr int kThreads = threads_of(BPC);
    typedef void (*kernel_t)(char *, const uint8_t *, FusedPlan);
    // shape index: 0..2 = 1, 2, 4 columns per thread; 3..6 = 4 columns per thread with
    // (lanes per item, positions per lane) = (2,8) (unused) (4,4) (4,8)
#define MOSHPIT_ROW(DT, TR)                                                                                   \
    {fused_rounds_kernel<DT, TR, 1, 1, 0, BPC>, fused_rounds_kernel<DT, TR, 2, 1, 0, BPC>,                    \
     fused_rounds_kernel<DT, TR, 4, 1, 0, BPC>, nullptr, nullptr, nullptr, nullptr}
#define MOSHPIT_ROW16(DT)                                                                                     \
    {fused_rounds_kernel<DT, 16, 1, 1, 0, BPC>, fused_rounds_kernel<DT, 16, 2, 1, 0, BPC>,                    \
     fused_rounds_kernel<DT, 16, 4, 1, 0, BPC>, fused_rounds_kernel<DT, 16, 4, 2, 8, BPC>, nullptr,           \
     fused_rounds_kernel<DT, 16, 4, 4, 4, BPC>, fused_rounds_kernel<DT, 16, 4, 4, 8, BPC>}
    static const kernel_t table[2][4][7] = {
        {MOSHPIT_ROW(0, 2), MOSHPIT_ROW(0, 4), MOSHPIT_ROW(0, 8), MOSHPIT_ROW16(0)},
        {MOSHPIT_ROW(1, 2), MOSHPIT_ROW(1, 4), MOSHPIT_ROW(1, 8), MOSHPIT_ROW16(1)}};
#undef MOSHPIT_ROW
#undef MOSHPIT_ROW16
    const int tree = tree_size(plan.M);
    const int ti = tree == 2 ? 0 : tree == 4 ? 1 : tree == 8 ? 2 : 3;
    // Every thread should have an item: prefer 4 columns per thread; if the tile
    // is too narrow for that, let 2 or 4 lanes share a group's positions
    // (8 < M <= 32), else narrow the per-thread column group.
    const int64_t cols = plan.Wb / (dtype == 0 ? 4 : 2);
    const int64_t items4 = plan.groups * (cols / 4);
    int ci = 2;
    if (items4 < kThreads) {
        if (ti == 3 && plan.M <= 32) {
            const bool two_blocks = plan.M > 16;
            // (two 16-position blocks over 2 lanes would need 16 positions per lane: too many registers)
            if (two_blocks) ci = 6;
            else ci = items4 * 2 >= kThreads ? 3 : 5;
        } else {
            while (ci > 0 && plan.groups * (cols >> ci) < kThreads) --ci;
        }
    }
    const kernel_t kernel = table[dtype][ti][ci];
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kernel), lds_of(BPC));
    if (e != hipSuccess) return e;
    int compute_units = 0;
    e = current_compute_units(&compute_units);
    if (e != hipSuccess) return e;
    // persistent: BPC blocks per compute unit walk the tiles
    const int64_t slots = static_cast<int64_t>(compute_units) * BPC;
    const int64_t grid = plan.work_items < slots ? plan.work_items : slots;
    kernel<<<dim3(static_cast<uint32_t>(grid)), dim3(kThreads), plan.lds_bytes, stream>>>(static_cast<char *>(X), masks,
                                                                                         plan);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fused_rounds(void *X, int dtype, const FusedPlan &plan, const uint8_t *masks, hipStream_t stream)
{
    if (plan.blocks_per_cu == 2) return launch_with<2>(X, dtype, plan, masks, stream);
    if (plan.blocks_per_cu == 1) return launch_with<1>(X, dtype, plan, masks, stream);
    return hipErrorInvalidValue;
}

}  // namespace moshpit
