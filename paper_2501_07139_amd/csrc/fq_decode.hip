// Decode of a whole stack of blocks in ONE persistent launch (M = 1).
//
// Serving generates one token at a time (FlexQuant, arXiv 2501.07139, Section "Introduction"), so a stack
// forward is a chain of matrix-vector products, each of which needs the complete output of the one before:
// four dependent phases per block (q/k/v; o; gate/up; down).  As separate launches every phase pays the
// start of a kernel and, worse, the full memory latency before its first weights arrive.  Here one
// workgroup per compute unit stays resident for the whole stack:
//
//  - Eight compute wavefronts per workgroup each own a ring of 1 KiB pages in LDS that is filled by
//    copies from global memory straight into LDS.  The sequence of pages a wavefront will need (which
//    supertile rows of which matrix, phase after phase) is fixed by the bit vector, so the ring keeps
//    loading the next phases' weights while the current phase ends and the workgroups meet: the stream of
//    packed weights from HBM never stops at a phase boundary.
//  - A ninth wavefront does everything that must not queue behind those copies (a wavefront's memory
//    operations return in order): it sums the compute wavefronts' partial results, stores the phase's
//    outputs with write-through stores, arrives at the grid-wide barrier, waits for it, and copies the next
//    phase's input vectors into LDS with loads that bypass the per-XCD L2.  No cache-flushing fences.
//  - The barrier: eight arrival counters (one per XCD's workgroups), bumped by fire-and-forget atomics;
//    every workgroup polls all eight.  Every wait is bounded by the constant-rate timer; a workgroup that
//    gives up raises an error word and stops waiting for the rest of the launch, so the grid always drains.
//  - The grid is one workgroup per compute unit, which the occupancy query has confirmed can be resident
//    together; the row-wise glue of the block (rms, residual adds, silu*mul) runs in the staging of each
//    phase exactly as in the per-phase kernels, with the residual stream kept in registers.
//
// Work units are whole supertile rows (whole planes, contiguous in memory); a phase's units are dealt to the
// workgroups in contiguous runs balanced by bytes.  Inside a unit the eight wavefronts split the groups of
// 128 k into eight contiguous ranges; per (unit, group) item a wavefront copies the planes (one 1 KiB copy
// each) and the sixteen scales and zeros of every sub-block (one 4-byte-per-lane copy), and consumes items
// in order: wait until the item's copies have landed (the wait count is the number of younger copies in
// flight, selected by a branch tree since the instruction takes an immediate), read its own 16 bytes of
// every plane back from LDS, extract, four MFMAs per sub-block against the staged activations, one fused
// scale/zero step per sub-block.
#include "fq_device.h"
#include "fq_internal.h"
#include "fq_stage.h"

#include "fq.h"

#include <algorithm>
#include <mutex>

namespace {

constexpr int DW = 8;              // compute wavefronts per workgroup
constexpr int DTHREADS = 64 * (DW + 1);
constexpr int DCOMPUTE = 64 * DW;  // threads that stage and compute
constexpr int DNB = 16;            // blocks per launch at most (bounded by the kernel-argument size)
constexpr int PAGE = 1024;
constexpr int ROWS_MAX = 384;      // weight rows of one phase a workgroup finishes at most
constexpr int RES = 2;             // 16-byte chunks of the residual stream a thread keeps: hidden <= 8192
constexpr int TRIPS = 4;           // chunks of a staged row per thread at most: rows of <= 16384 elements
constexpr int NPG_MAX = 14;        // pages per ring at most
constexpr int NPG_MIN = 8;         // a ring holds at least the largest chunk (seven pages)
constexpr size_t LDS_LIMIT = 160 * 1024;
constexpr unsigned SYNC_STRIDE = 32; // dwords between two counters: each on its own 128-byte line
constexpr unsigned SYNC_ERR = 8 * SYNC_STRIDE;

struct DecodeBlock {
    const uint32_t *packed[7];
    const _Float16 *scales[7], *zeros[7];
    unsigned bits4, pad; // the seven bit-widths, four bits each (whole dwords: read through the scalar path)
};
__host__ __device__ constexpr int bits_at(unsigned bits4, int m) { return (int)((bits4 >> (4 * m)) & 15u); }

struct DecodeArgs {
    int H, F, nblocks;
    int first, last;   // this launch holds block 0 of the stack / the stack's last block
    int npg;           // pages per ring
    unsigned gen0;     // barriers passed by earlier launches of the same call
    unsigned long long give_up_ticks;
    const _Float16 *x_in;
    _Float16 *x_out;
    _Float16 *buf[8];  // q, k, v, o, g, p, d and the residual x1 handed from launch to launch
    unsigned *sync;    // eight arrival counters and an error word, SYNC_STRIDE dwords apart
    unsigned *host_err; // pinned host word raised when a workgroup gives up (may be null)
    unsigned off_raw, off_sums, off_red, off_part; // LDS byte offsets (the rings start at 0)
    DecodeBlock blk[DNB];
};
static_assert(sizeof(DecodeArgs) <= 4000, "kernel arguments");

__host__ __device__ constexpr int planes_of(int bits) { return bits == 3 ? 3 : (bits == 8 ? 2 : 1); }
__host__ __device__ constexpr int subs_of(int bits) { return bits == 2 ? 2 : (bits == 3 ? 4 : 1); }
__host__ __device__ constexpr int phase_first(int ph) { return ph == 0 ? 0 : (ph == 1 ? 3 : (ph == 2 ? 4 : 6)); }
__host__ __device__ constexpr int phase_count(int ph) { return ph == 0 ? 3 : (ph == 2 ? 2 : 1); }

// The units [u0, u1) of each matrix of a phase that workgroup `wg` of `grid` owns.  Every matrix is cut into
// `grid` contiguous runs of (nearly) equal length, so a workgroup's share of each matrix, and with it its
// bytes, is within one unit of the mean; the odd matrices are dealt in reverse workgroup order, so that the
// workgroups that took the longer runs of one matrix take the shorter runs of the next.
struct PhaseWork {
    int u0[3], u1[3];
};
// element j of a three-element array without indexing it by a run-time value (which would move the array
// to scratch memory)
__host__ __device__ inline int pick3(const int (&v)[3], int j) { return j == 0 ? v[0] : (j == 1 ? v[1] : v[2]); }

__host__ __device__ inline void phase_work(unsigned bits4, int ph, int N, int wg, int grid, PhaseWork &w)
{
    const int first = phase_first(ph), count = phase_count(ph);
    const unsigned rows16 = (unsigned)((N + 63) / 64 * 4); // sixteen-row sub-blocks of the padded matrix
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        // 1, 2 or 4 sub-blocks per unit: a shift, not a division
        const int b = bits_at(bits4, first + (j < count ? j : 0));
        const unsigned units = j < count ? rows16 >> (b == 2 ? 1 : (b == 3 ? 2 : 0)) : 0u;
        const unsigned i = (j & 1) ? (unsigned)(grid - 1 - wg) : (unsigned)wg;
        w.u0[j] = (int)(i * units / (unsigned)grid);
        w.u1[j] = (int)((i + 1) * units / (unsigned)grid);
    }
}

// ------------------------------------------------------------------ copies into LDS
// The compiler is not told that these write LDS: it would otherwise make every later LDS read wait for all
// of them.  The code below waits by count instead.  M0 holds the LDS address of lane 0's bytes.
// A uniform value as the scalar register operand the instructions below need.
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ bool uniform_bool(bool b) { return uniform32(b ? 1u : 0u) != 0u; }
__device__ __forceinline__ const void *uniform_ptr(const void *p)
{
    const uint64_t v = (uint64_t)(size_t)p;
    return reinterpret_cast<const void *>((size_t)(((uint64_t)uniform32((uint32_t)(v >> 32)) << 32) | uniform32((uint32_t)v)));
}

__device__ __forceinline__ void dma_page(uint32_t lds_addr, const void *base, uint32_t lane_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(uniform32(lds_addr)), "v"(lane_off),
                 "s"(uniform_ptr(base))
                 : "memory");
}

// the same through the L2-bypassing path: data another workgroup has just written
__device__ __forceinline__ void dma_page_fresh(uint32_t lds_addr, const void *base, uint32_t lane_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 sc1" ::"s"(uniform32(lds_addr)),
                 "v"(lane_off), "s"(uniform_ptr(base))
                 : "memory");
}

// sixteen bytes per lane, each lane with its own address
__device__ __forceinline__ void dma_words16(uint32_t lds_addr, const void *lane_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(uniform32(lds_addr)), "v"(lane_addr)
                 : "memory");
}

// Wait until at most n vector-memory operations of this wavefront are in flight, LO <= n <= HI.  The
// instruction takes an immediate, so a branch tree selects it; n is uniform.
template <int LO, int HI>
__device__ __forceinline__ void wait_vm_le(int n)
{
    if constexpr (LO == HI) {
        __builtin_amdgcn_s_waitcnt(gemv_wait_vmcnt(LO));
    } else {
        constexpr int MID = (LO + HI) / 2;
        if (n <= MID)
            wait_vm_le<LO, MID>(n);
        else
            wait_vm_le<MID + 1, HI>(n);
    }
}

// ------------------------------------------------------------------ the stream of pages of one wavefront
// A wavefront's share of a unit (its contiguous range of groups) is cut into chunks of up to chunk_groups
// groups.  A chunk is one page with the scales and zeros of its groups, then the groups' planes, which are
// contiguous in memory: after the first page the copies of a chunk differ only by an address increment.
// Every copy fills one ring page, so pages in the ring and copies in flight are the same count.
__host__ __device__ constexpr int chunk_groups(int bits) { return (bits == 2 || bits == 4) ? 4 : 2; }

struct Stream {
    int blk, ph, j, u;   // where the next chunk starts: block, phase, matrix of the phase, unit ...
    int g, g_end;        // ... and group; the end of this wavefront's range of groups
    PhaseWork w;
    bool done;
    // the matrix the cursor is in
    int bits, G;
    const char *packed;       // uniform
    const char *meta_lane;    // per lane: its 16 bytes of the scales/zeros of group 0 of sub-block v of unit 0
    bool meta_on;             // this lane fetches scales/zeros at all (sub-block v exists)
    int meta_q;               // its piece (16 bytes) within the chunk's groups
    // the chunk being copied
    int tiles_left;           // planes of the current chunk still to copy
    const char *tile_next;    // address of the next plane (uniform)
    // the ring
    int head;                 // slot of the next page to fill
    int inflight;             // pages filled (or being filled) and not yet released
};

struct Ctx {
    int wg, grid, wave, lane, npg;
    uint32_t lds0;             // LDS address of the dynamic segment
    uint32_t ring_addr;        // LDS address of this wavefront's ring ...
    const unsigned char *ring; // ... and the pointer to it
};

__device__ __forceinline__ int phase_k(const DecodeArgs &a, int ph) { return ph == 3 ? a.F : a.H; }
__device__ __forceinline__ int phase_n(const DecodeArgs &a, int ph) { return ph == 2 ? a.F : a.H; }
// the wavefront's contiguous share of the G groups
__device__ __forceinline__ int wave_g0(int G, int wave) { return (G * wave) / DW; }

// The cursor has entered matrix j of its phase: what the copies need of it.
__device__ __forceinline__ void stream_enter_matrix(const DecodeArgs &a, const Ctx &c, Stream &s)
{
    const int blk = (int)uniform32((uint32_t)s.blk), m = (int)uniform32((uint32_t)(phase_first(s.ph) + s.j));
    s.bits = bits_at(a.blk[blk].bits4, m);
    s.G = phase_k(a, s.ph) >> 7;
    s.packed = reinterpret_cast<const char *>(a.blk[blk].packed[m]);
    // lane = (2 v + part) * 2 CH + q: sub-block v, scales (part 0) or zeros (part 1), piece q of the chunk's groups
    const int CH = chunk_groups(s.bits), S = subs_of(s.bits);
    const int va = c.lane / (2 * CH), q = c.lane - va * 2 * CH, v = va >> 1;
    const char *const sc = reinterpret_cast<const char *>(a.blk[blk].scales[m]);
    const char *const zr = reinterpret_cast<const char *>(a.blk[blk].zeros[m]);
    s.meta_on = v < S;
    s.meta_q = q;
    s.meta_lane = ((va & 1) ? zr : sc) + (size_t)v * s.G * 32 + (size_t)q * 16;
}

// Moves the cursor to the next unit that exists (or sets done); the cursor's group range is reset.
__device__ __forceinline__ void stream_next_unit(const DecodeArgs &a, const Ctx &c, Stream &s, bool advance)
{
    if (advance)
        ++s.u;
    s.u = (int)uniform32((uint32_t)s.u);
    s.j = (int)uniform32((uint32_t)s.j);
    s.ph = (int)uniform32((uint32_t)s.ph);
    s.blk = (int)uniform32((uint32_t)s.blk);
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        s.w.u0[q] = (int)uniform32((uint32_t)s.w.u0[q]);
        s.w.u1[q] = (int)uniform32((uint32_t)s.w.u1[q]);
    }
    while (uniform_bool(!s.done)) {
        if (uniform_bool(s.j < phase_count(s.ph) && s.u < pick3(s.w.u1, s.j)))
            break;
        if (uniform_bool(s.j < phase_count(s.ph))) {
            ++s.j;
            if (s.j < phase_count(s.ph)) {
                s.u = pick3(s.w.u0, s.j);
                stream_enter_matrix(a, c, s);
            }
            continue;
        }
        if (++s.ph == 4) {
            s.ph = 0;
            ++s.blk;
        }
        if (uniform_bool(s.blk >= a.nblocks)) {
            s.done = true;
            return;
        }
        phase_work(a.blk[s.blk].bits4, s.ph, phase_n(a, s.ph), c.wg, c.grid, s.w);
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            s.w.u0[q] = (int)uniform32((uint32_t)s.w.u0[q]);
            s.w.u1[q] = (int)uniform32((uint32_t)s.w.u1[q]);
        }
        s.j = 0;
        s.u = s.w.u0[0];
        stream_enter_matrix(a, c, s);
    }
    s.G = (int)uniform32((uint32_t)s.G);
    s.g = wave_g0(s.G, c.wave);
    s.g_end = wave_g0(s.G, c.wave + 1);
}

// Issues copies while the ring has a free page.  Every counter of the cursor is passed through uniform32 when
// it changes: the values are the same in all lanes, and saying so at every step keeps the compiler from
// carrying them in vector registers and guarding the loop with lane masks.
__device__ __forceinline__ void stream_fill(const DecodeArgs &a, const Ctx &c, Stream &s)
{
    const int npg = c.npg;
    int inflight = (int)uniform32((uint32_t)s.inflight), head = (int)uniform32((uint32_t)s.head);
    int tiles_left = (int)uniform32((uint32_t)s.tiles_left);
    const char *tile_next = static_cast<const char *>(uniform_ptr(s.tile_next));
    for (;;) {
        // the planes of the current chunk: one copy each, addresses 1 KiB apart
        const int k = (int)uniform32((uint32_t)min(npg - inflight, tiles_left));
        for (int i = 0; uniform_bool(i < k); ++i) {
            dma_page(c.ring_addr + (uint32_t)head * PAGE, tile_next, (uint32_t)c.lane * 16u);
            tile_next = static_cast<const char *>(uniform_ptr(tile_next + PAGE));
            head = (int)uniform32((uint32_t)(head + 1 == npg ? 0 : head + 1));
        }
        inflight = (int)uniform32((uint32_t)(inflight + k));
        tiles_left = (int)uniform32((uint32_t)(tiles_left - k));
        if (uniform_bool(tiles_left > 0 || s.done || inflight >= npg))
            break;
        // a new chunk: first the page of scales and zeros
        if (uniform_bool(s.g >= s.g_end)) {
            stream_next_unit(a, c, s, true);
            continue;
        }
        const int bits = (int)uniform32((uint32_t)s.bits), G = (int)uniform32((uint32_t)s.G);
        const int P = planes_of(bits), S = subs_of(bits);
        const int g = (int)uniform32((uint32_t)s.g);
        const int n = (int)uniform32((uint32_t)min(chunk_groups(bits), s.g_end - g));
        const int u = (int)uniform32((uint32_t)s.u);
        if (s.meta_on && s.meta_q < 2 * n)
            dma_words16(c.ring_addr + (uint32_t)head * PAGE, s.meta_lane + ((size_t)u * S * G + g) * 32);
        head = (int)uniform32((uint32_t)(head + 1 == npg ? 0 : head + 1));
        inflight = (int)uniform32((uint32_t)(inflight + 1));
        tile_next = static_cast<const char *>(uniform_ptr(s.packed + ((size_t)u * G + g) * ((size_t)P * PAGE)));
        tiles_left = (int)uniform32((uint32_t)(n * P));
        s.g = (int)uniform32((uint32_t)(g + n));
    }
    s.inflight = inflight;
    s.head = head;
    s.tiles_left = tiles_left;
    s.tile_next = tile_next;
}

// ------------------------------------------------------------------ consuming one unit
struct Consumer {
    int page;    // ring slot of the oldest unconsumed page
    int slot;    // next free row of this phase in the reduction buffer
};

// The arithmetic of one group of a chunk for a matrix of BITS bits: per sub-block extract, four MFMAs
// against the staged activations, one scale/zero step.  plane: the lane's 16 bytes of every plane; meta:
// the chunk's page of scales and zeros; i: the group's place in the chunk.
template <int BITS>
__device__ __forceinline__ void group_math(const u4v (&plane)[planes_of(BITS)], const unsigned char *meta, int i,
                                           const h8 (&ax)[4], float xg, float cg, float eg, int r, float (&acc)[4])
{
    constexpr int S = subs_of(BITS), CH = chunk_groups(BITS);
#pragma unroll
    for (int u = 0; u < S; ++u) {
        uint32_t C[BITS], h[16];
#pragma unroll
        for (int q = 0; q < BITS; ++q) {
            const int j = BITS * u + q;
            const u4v pl = plane[j >> 2];
            C[q] = (j & 3) == 0 ? pl.x : ((j & 3) == 1 ? pl.y : ((j & 3) == 2 ? pl.z : pl.w));
        }
        extract_biased<BITS>(C, h);
        f4 p = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < 4; ++st)
            p = mfma16x16x32(ax[st], make_h8_bits(h[4 * st], h[4 * st + 1], h[4 * st + 2], h[4 * st + 3]), p);
        const float sf = (float)*reinterpret_cast<const _Float16 *>(meta + ((2 * u) * 2 * CH + 2 * i) * 16 + 2 * r);
        const float zf = (float)*reinterpret_cast<const _Float16 *>(meta + ((2 * u + 1) * 2 * CH + 2 * i) * 16 + 2 * r);
        // p = 2^E sum x code + 1024 sum x': back to the scale of x, bias and zero * sum x away, then scale
        acc[u] = fmaf(sf, fmaf(eg, p[0], -fmaf(zf, xg, cg)), acc[u]);
    }
}

// One unit (supertile row) of a matrix of BITS bits: this wavefront's groups of it, chunk by chunk.
template <int BITS>
__device__ __forceinline__ void consume_unit(const DecodeArgs &a, const Ctx &c, Stream &s, Consumer &k, int G, const h8 *xl,
                                             const float *xsum, const float *csum, const float *esc, float *red)
{
    constexpr int P = planes_of(BITS), S = subs_of(BITS), CH = chunk_groups(BITS);
    const int npg = c.npg;
    const int g0 = wave_g0(G, c.wave), g1 = wave_g0(G, c.wave + 1);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int cl = c.lane >> 4, r = c.lane & 15;
    for (int g = g0; uniform_bool(g < g1); g += CH) {
        const int n = (int)uniform32((uint32_t)min(CH, g1 - g)), pages = 1 + n * P;
        s.inflight = (int)uniform32((uint32_t)s.inflight);
        // the chunk's copies are the oldest in flight; all of them have been issued (the ring holds a chunk)
        wait_vm_le<0, NPG_MAX>(s.inflight - pages);
        asm volatile("" ::: "memory");
        int slot = k.page;
        const unsigned char *const meta = c.ring + slot * PAGE;
        auto next = [&](int sl) { return sl + 1 == npg ? 0 : sl + 1; };
        slot = next(slot);
        auto one_group = [&](int i) {
            u4v plane[P];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                plane[p] = *reinterpret_cast<const u4v *>(c.ring + slot * PAGE + c.lane * 16);
                slot = next(slot);
            }
            h8 ax[4];
#pragma unroll
            for (int st = 0; st < 4; ++st)
                ax[st] = xl[(g + i) * 16 + st * 4 + cl];
            group_math<BITS>(plane, meta, i, ax, xsum[g + i], csum[g + i], esc[g + i], r, acc);
        };
        if (n == CH) {
#pragma unroll 2
            for (int i = 0; i < CH; ++i)
                one_group(i);
        } else {
            for (int i = 0; i < n; ++i)
                one_group(i);
        }
        k.page = (int)uniform32((uint32_t)slot);
        asm volatile("" ::: "memory"); // the chunk's LDS reads stay ahead of the copies that refill its pages
        s.inflight -= pages;
        stream_fill(a, c, s);
    }
    if (c.lane < 16) {
#pragma unroll
        for (int u = 0; u < S; ++u)
            red[c.wave * ROWS_MAX + k.slot + 16 * u + c.lane] = acc[u];
    }
    k.slot += 16 * S;
}

// ------------------------------------------------------------------ grid-wide barrier (exchange wavefront only)
struct Grid {
    unsigned *sync, *host_err;
    unsigned per;   // workgroups behind each counter
    unsigned gen0;
    unsigned long long limit;
    bool dead;      // this workgroup has stopped waiting
};

__device__ __forceinline__ void grid_arrive(const Grid &g, int wg, int lane)
{
    if (lane == 0)
        __hip_atomic_fetch_add(g.sync + (wg & 7) * SYNC_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Waits until every workgroup has arrived k times (since the counters were cleared).  Bounded: after
// `limit` ticks of the constant-rate timer, or once any workgroup has given up, the wait ends, the error
// words are raised and this workgroup never waits again.
__device__ __forceinline__ void grid_wait(Grid &g, unsigned k, int lane)
{
    if (g.dead)
        return;
    const unsigned target = (g.gen0 + k) * g.per;
    const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
    for (;;) {
        unsigned v = target, e = 0;
        if (lane < 8)
            v = __hip_atomic_load(g.sync + lane * SYNC_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lane == 8)
            e = __hip_atomic_load(g.sync + SYNC_ERR, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool behind = (int)(v - target) < 0;
        if (__builtin_amdgcn_ballot_w64(behind) == 0)
            return;
        const bool late = __builtin_amdgcn_s_memrealtime() - t0 > g.limit;
        if (__builtin_amdgcn_ballot_w64(e != 0) != 0 || late) {
            g.dead = true;
            if (lane == 0) {
                __hip_atomic_store(g.sync + SYNC_ERR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (g.host_err)
                    __hip_atomic_store(g.host_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            return;
        }
        __builtin_amdgcn_s_sleep(2);
    }
}

// Sum over the compute threads, the same value in every compute thread.  The exchange wavefront passes the
// same barrier (exchange_main counts them).  part: two sets of DW partials used in turn.
__device__ __forceinline__ float wg_sum(float v, float *part, int which, int wave, int lane)
{
    v = row16_sum(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    if (lane == 0)
        part[which * DW + wave] = v;
    lds_barrier();
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < DW; ++w)
        sum += part[which * DW + w];
    return sum;
}

// Writes one staged chunk for the matrices of bit-width BITS: x * 2^(E - shift) and, once per group, 2^-E * 1024 * sum.
template <int BITS>
__device__ __forceinline__ void put_variant(h8 xe, int kc, int E, float einv, h8 *xl, float *csum)
{
    const h8 w = stage_scaled<BITS>(xe, (kc >> 2) & 3, E);
    xl[kc] = w;
    const float sc = row16_sum(gemv_sum(w));
    if ((kc & 15) == 0)
        csum[kc >> 4] = einv * (1024.0f * sc);
}

// The residual stream's chunk i of a thread, i a run-time (uniform) value: selected, not indexed, so that the
// array stays in registers.
__device__ __forceinline__ h8 get_res(const h8 (&v)[RES], int i) { return i == 0 ? v[0] : v[1]; }
__device__ __forceinline__ void set_res(h8 (&v)[RES], int i, h8 x)
{
    if (i == 0)
        v[0] = x;
    else if (i == 1)
        v[1] = x;
}

// LDS regions behind the rings.
struct Regions {
    unsigned char *raw; // input vectors as copied, later the staged x (one copy per distinct bit-width)
    float *xsum;        // [GP] sum of x over the group
    float *esc;         // [GP] 2^-E of the group
    float *csum;        // [3][GP] 2^-E * 1024 * sum of the staged x, per staged copy
    float *red;         // [DW][ROWS_MAX] partial results of the phase's rows
    float *part;        // [2][DW] partials of the block sums
    int GP;
};

__device__ __forceinline__ Regions regions_of(const DecodeArgs &a, unsigned char *smem)
{
    Regions r;
    r.raw = smem + a.off_raw;
    r.xsum = reinterpret_cast<float *>(smem + a.off_sums);
    r.GP = (a.H > a.F ? a.H : a.F) >> 7;
    r.esc = r.xsum + r.GP;
    r.csum = r.esc + r.GP;
    r.red = reinterpret_cast<float *>(smem + a.off_red);
    r.part = reinterpret_cast<float *>(smem + a.off_part);
    return r;
}

// How a phase's input is formed (the modes of the per-phase kernels):
//   phase 0: rms(x_in) in the stack's first block, else x = rms(x1 + d) kept as the block's input, then rms(x)
//   phase 1: rms(q + k + v)   phase 2: x1 = x + o kept, rms(x1)   phase 3: rms(silu(g) * p)
// Both kinds of wavefront pass these barriers per phase, in this order: input copied; one per block sum
// (two in phase 0 after the stack's first block); x staged; items done.

// ------------------------------------------------------------------ the eight compute wavefronts
__device__ __forceinline__ void compute_main(const DecodeArgs &a, unsigned char *smem, int wave, int lane)
{
    const int tid = threadIdx.x, grid = gridDim.x, wg = blockIdx.x;
    const Regions R = regions_of(a, smem);
    Ctx c;
    c.npg = a.npg;
    c.wg = wg;
    c.grid = grid;
    c.wave = wave;
    c.lane = lane;
    c.lds0 = (uint32_t)(size_t)smem;
    c.ring = smem + (size_t)wave * a.npg * PAGE;
    c.ring_addr = (uint32_t)(size_t)c.ring;

    Stream s;
    s.blk = 0;
    s.ph = 0;
    s.j = 0;
    s.done = false;
    s.head = s.inflight = s.tiles_left = 0;
    s.g = s.g_end = 0;
    s.tile_next = nullptr;
    phase_work(a.blk[0].bits4, 0, a.H, wg, grid, s.w);
    s.u = s.w.u0[0];
    stream_enter_matrix(a, c, s);
    stream_next_unit(a, c, s, false);
    stream_fill(a, c, s);
    Consumer k;
    k.page = 0;
    k.slot = 0;

    // the residual stream, replicated: thread t keeps chunks t and t + DCOMPUTE of x (block input) and x1
    h8 xcur[RES], x1r[RES];
#pragma unroll
    for (int i = 0; i < RES; ++i) {
        xcur[i] = h8{0, 0, 0, 0, 0, 0, 0, 0};
        x1r[i] = xcur[i];
    }
    int sums = 0;
    const int hchunks = a.H >> 3;

    for (int blk = 0; blk < a.nblocks; ++blk) {
        for (int ph = 0; ph < 4; ++ph) {
            const int K = phase_k(a, ph), N = phase_n(a, ph), G = K >> 7, chunks = K >> 3;
            const bool from_x_in = blk == 0 && ph == 0 && a.first, from_x1 = blk == 0 && ph == 0 && !a.first;
            lds_barrier(); // the input has been copied

            PhaseWork w;
            const unsigned bits4 = a.blk[blk].bits4;
            phase_work(bits4, ph, N, wg, grid, w);
            // distinct bit-widths among this workgroup's matrices of the phase: one staged copy of x each
            int vbits[3] = {0, 0, 0}, vof[3] = {0, 0, 0}, nvar = 0;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                if (j >= phase_count(ph) || w.u0[j] >= w.u1[j])
                    continue;
                const int b = bits_at(bits4, phase_first(ph) + j);
                int v = nvar; // index of the first variant with these bits, else a new one
#pragma unroll
                for (int q = 2; q >= 0; --q)
                    if (q < nvar && vbits[q] == b)
                        v = q;
#pragma unroll
                for (int q = 0; q < 3; ++q)
                    if (q == v && v == nvar)
                        vbits[q] = b;
                if (v == nvar)
                    ++nvar;
                vof[j] = v;
            }

            {
                // Two passes over this thread's chunks: sum of squares, then (the norm known) scale and stage.
                // Nothing but the residual stream is kept in registers between them: the cheap sums are formed
                // again, the silu products wait in the LDS slots of their inputs (32 bytes, which only this
                // thread touches).  The loops over the chunks are not unrolled: one chunk's registers at a time.
                const bool twice = ph == 0 && !from_x_in; // rms twice: the first result is the block's input, kept
                float ss = 0.f;
#pragma unroll 1
                for (int i = 0; i < TRIPS; ++i) {
                    const int kc = tid + DCOMPUTE * i;
                    if (kc >= chunks)
                        continue;
                    const h8 r0 = *reinterpret_cast<const h8 *>(R.raw + (size_t)kc * 16);
                    if (from_x_in) { // x = x_in
                        set_res(xcur, i, r0);
                        ss = gemv_sumsq(r0, ss);
                    } else if (ph == 0) { // x1 + d
                        if (from_x1)
                            set_res(x1r, i, *reinterpret_cast<const h8 *>(R.raw + (size_t)K * 2 + (size_t)kc * 16));
                        const h8 xa = get_res(x1r, i);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float t = (float)xa[e] + (float)r0[e];
                            ss = fmaf(t, t, ss);
                        }
                    } else if (ph == 1) {
                        const h8 r1 = *reinterpret_cast<const h8 *>(R.raw + (size_t)K * 2 + (size_t)kc * 16);
                        const h8 r2 = *reinterpret_cast<const h8 *>(R.raw + (size_t)K * 4 + (size_t)kc * 16);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float t = (float)r0[e] + (float)r1[e] + (float)r2[e];
                            ss = fmaf(t, t, ss);
                        }
                    } else if (ph == 2) { // x1 = x + o, an fp16 tensor
                        const h8 v = get_res(xcur, i) + r0;
                        set_res(x1r, i, v);
                        ss = gemv_sumsq(v, ss);
                    } else {
                        const h8 r1 = *reinterpret_cast<const h8 *>(R.raw + (size_t)K * 2 + (size_t)kc * 16);
                        float t[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float gv = (float)r0[e];
                            t[e] = gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv)) * (float)r1[e];
                            ss = fmaf(t[e], t[e], ss);
                        }
                        *reinterpret_cast<f4 *>(R.raw + (size_t)kc * 16) = f4{t[0], t[1], t[2], t[3]};
                        *reinterpret_cast<f4 *>(R.raw + (size_t)K * 2 + (size_t)kc * 16) = f4{t[4], t[5], t[6], t[7]};
                    }
                }
                const float inv1 = 1.0f / sqrtf(wg_sum(ss, R.part, sums++ & 1, wave, lane) / (float)K + 1e-5f);
                float inv2 = 1.0f;
                if (twice) {
                    float s2 = 0.f;
#pragma unroll 1
                    for (int i = 0; i < RES; ++i) {
                        const int kc = tid + DCOMPUTE * i;
                        if (kc >= chunks)
                            continue;
                        const h8 r0 = *reinterpret_cast<const h8 *>(R.raw + (size_t)kc * 16);
                        const h8 xa = get_res(x1r, i);
                        float t[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            t[e] = (float)xa[e] + (float)r0[e];
                        const h8 y = gemv_scaled(t, inv1);
                        set_res(xcur, i, y);
                        s2 = gemv_sumsq(y, s2);
                    }
                    inv2 = 1.0f / sqrtf(wg_sum(s2, R.part, sums++ & 1, wave, lane) / (float)K + 1e-5f);
                }
                // Every thread has read its chunks of the raw input (the block sum's barrier lies between), except
                // phase 1's sums and phase 3's products, which this thread reads back below before it overwrites
                // them: staged copy 0 of chunk kc lies in the slot of input 0's chunk kc, and the thread reads all
                // its inputs of a chunk before it stages that chunk.  Copies 1 and 2 (phases 0 and 2 only, whose
                // inputs are in registers by now) lie behind.
                h8 *const xl = reinterpret_cast<h8 *>(R.raw);
#pragma unroll 1
                for (int i = 0; i < TRIPS; ++i) {
                    const int kc = tid + DCOMPUTE * i;
                    if (kc >= chunks)
                        continue;
                    h8 xe;
                    if (ph == 0) {
                        xe = gemv_scaled(get_res(xcur, i), twice ? inv2 : inv1);
                    } else if (ph == 2) {
                        xe = gemv_scaled(get_res(x1r, i), inv1);
                    } else if (ph == 1) {
                        const h8 r0 = *reinterpret_cast<const h8 *>(R.raw + (size_t)kc * 16);
                        const h8 r1 = *reinterpret_cast<const h8 *>(R.raw + (size_t)K * 2 + (size_t)kc * 16);
                        const h8 r2 = *reinterpret_cast<const h8 *>(R.raw + (size_t)K * 4 + (size_t)kc * 16);
                        float t[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            t[e] = (float)r0[e] + (float)r1[e] + (float)r2[e];
                        xe = gemv_scaled(t, inv1);
                    } else {
                        const f4 lo = *reinterpret_cast<const f4 *>(R.raw + (size_t)kc * 16);
                        const f4 hi = *reinterpret_cast<const f4 *>(R.raw + (size_t)K * 2 + (size_t)kc * 16);
                        const float t[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        xe = gemv_scaled(t, inv1);
                    }
                    const int ex = min(max((int)(group_max_bits(xe) >> 10), 1), 30), E = 29 - ex;
                    const float einv = __builtin_bit_cast(float, (uint32_t)(127 - E) << 23);
                    const float sx = row16_sum(gemv_sum(xe));
                    if ((kc & 15) == 0) {
                        R.xsum[kc >> 4] = sx;
                        R.esc[kc >> 4] = einv;
                    }
                    for (int v = 0; v < nvar; ++v) { // one staged copy per distinct bit-width
                        h8 *xv = xl + (size_t)v * chunks;
                        float *cv = R.csum + v * R.GP;
                        switch (pick3(vbits, v)) {
                        case 2: put_variant<2>(xe, kc, E, einv, xv, cv); break;
                        case 3: put_variant<3>(xe, kc, E, einv, xv, cv); break;
                        case 4: put_variant<4>(xe, kc, E, einv, xv, cv); break;
                        default: put_variant<8>(xe, kc, E, einv, xv, cv); break;
                        }
                    }
                }
            }
            lds_barrier(); // x is staged

            k.slot = 0;
            for (int j = 0; j < phase_count(ph); ++j) {
                const int b = bits_at(bits4, phase_first(ph) + j), vj = pick3(vof, j);
                const h8 *xv = reinterpret_cast<const h8 *>(R.raw) + (size_t)vj * chunks;
                const float *cv = R.csum + vj * R.GP;
                for (int u = pick3(w.u0, j); u < pick3(w.u1, j); ++u) {
                    switch (b) { // uniform
                    case 2: consume_unit<2>(a, c, s, k, G, xv, R.xsum, cv, R.esc, R.red); break;
                    case 3: consume_unit<3>(a, c, s, k, G, xv, R.xsum, cv, R.esc, R.red); break;
                    case 4: consume_unit<4>(a, c, s, k, G, xv, R.xsum, cv, R.esc, R.red); break;
                    default: consume_unit<8>(a, c, s, k, G, xv, R.xsum, cv, R.esc, R.red); break;
                    }
                }
            }
            lds_barrier(); // the phase's partial results are in LDS
        }
    }

    // after the last block: the stack's output rms(x1 + d) (workgroup 0), or the residual for the next launch
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
    if (wg != 0)
        return;
    lds_barrier(); // d has been copied
    if (a.last) {
        float t32[RES][8];
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < RES; ++i) {
            const int kc = tid + DCOMPUTE * i;
            if (kc >= hchunks)
                continue;
            const h8 dv = *reinterpret_cast<const h8 *>(R.raw + (size_t)kc * 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                t32[i][e] = (float)x1r[i][e] + (float)dv[e];
                ss = fmaf(t32[i][e], t32[i][e], ss);
            }
        }
        const float inv = 1.0f / sqrtf(wg_sum(ss, R.part, sums++ & 1, wave, lane) / (float)a.H + 1e-5f);
#pragma unroll
        for (int i = 0; i < RES; ++i) {
            const int kc = tid + DCOMPUTE * i;
            if (kc < hchunks)
                *reinterpret_cast<h8 *>(a.x_out + (size_t)kc * 8) = gemv_scaled(t32[i], inv);
        }
    } else {
#pragma unroll
        for (int i = 0; i < RES; ++i) {
            const int kc = tid + DCOMPUTE * i;
            if (kc < hchunks)
                *reinterpret_cast<h8 *>(a.buf[7] + (size_t)kc * 8) = x1r[i];
        }
    }
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
}

// ------------------------------------------------------------------ the exchange wavefront
__device__ __forceinline__ void exchange_main(const DecodeArgs &a, unsigned char *smem, int lane)
{
    const int grid = gridDim.x, wg = blockIdx.x;
    const Regions R = regions_of(a, smem);
    const uint32_t raw_addr = (uint32_t)(size_t)smem + a.off_raw;
    Grid gb;
    gb.sync = a.sync;
    gb.host_err = a.host_err;
    gb.per = (unsigned)grid / 8u;
    gb.gen0 = a.gen0;
    gb.limit = a.give_up_ticks;
    gb.dead = false;

    auto fetch = [&](const _Float16 *src, int slot, int K) { // one input vector of K elements into raw slot `slot`
        const int chunks = K >> 3;
        for (int c0 = 0; c0 * 64 < chunks; ++c0)
            if (c0 * 64 + lane < chunks)
                dma_page_fresh(raw_addr + (uint32_t)(slot * K * 2 + c0 * PAGE), reinterpret_cast<const char *>(src) + (size_t)c0 * PAGE,
                               (uint32_t)lane * 16u);
    };

    for (int blk = 0; blk < a.nblocks; ++blk) {
        for (int ph = 0; ph < 4; ++ph) {
            const int K = phase_k(a, ph), N = phase_n(a, ph);
            const bool very_first = blk == 0 && ph == 0;
            // wait for the previous phase everywhere, then fetch this phase's input
            if (!very_first)
                grid_wait(gb, (unsigned)(blk * 4 + ph), lane);
            if (ph == 0) {
                fetch((very_first && a.first) ? a.x_in : a.buf[6], 0, K);
                if (very_first && !a.first)
                    fetch(a.buf[7], 1, K); // x1 of the previous launch
            } else if (ph == 1) {
                fetch(a.buf[0], 0, K);
                fetch(a.buf[1], 1, K);
                fetch(a.buf[2], 2, K);
            } else if (ph == 2) {
                fetch(a.buf[3], 0, K);
            } else {
                fetch(a.buf[4], 0, K);
                fetch(a.buf[5], 1, K);
            }
            __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
            lds_barrier(); // the input has been copied
            lds_barrier(); // block sum
            if (ph == 0 && !(very_first && a.first))
                lds_barrier(); // second block sum
            lds_barrier(); // x is staged
            lds_barrier(); // the phase's partial results are in LDS

            // finish the rows, publish them, arrive
            PhaseWork w;
            const unsigned bits4 = a.blk[blk].bits4;
            phase_work(bits4, ph, N, wg, grid, w);
            int slot = 0;
            for (int j = 0; j < phase_count(ph); ++j) {
                const int m = (int)uniform32((uint32_t)(phase_first(ph) + j));
                const int rows = 16 * subs_of(bits_at(bits4, m));
                unsigned short *out = reinterpret_cast<unsigned short *>(a.buf[m]);
                for (int u = pick3(w.u0, j); u < pick3(w.u1, j); ++u) {
                    const int n = u * rows + lane;
                    if (lane < rows && n < N) {
                        float sum = 0.f;
#pragma unroll
                        for (int wv = 0; wv < DW; ++wv)
                            sum += R.red[wv * ROWS_MAX + slot + lane];
                        const _Float16 hv = (_Float16)sum;
                        __hip_atomic_store(out + n, __builtin_bit_cast(unsigned short, hv), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                    }
                    slot += rows;
                }
            }
            __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0); // the stores have reached memory
            grid_arrive(gb, wg, lane);
        }
    }

    grid_wait(gb, (unsigned)(a.nblocks * 4), lane);
    if (wg != 0)
        return;
    if (a.last)
        fetch(a.buf[6], 0, a.H);
    __builtin_amdgcn_s_waitcnt(FQ_WAIT_VMCNT0);
    lds_barrier(); // d has been copied
    if (a.last)
        lds_barrier(); // block sum
}

__global__ __launch_bounds__(DTHREADS, 1) void decode_persist_kernel(const DecodeArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave < DW)
        compute_main(a, smem, wave, lane);
    else
        exchange_main(a, smem, lane);
}

__global__ void decode_clear_kernel(unsigned *sync)
{
    if (threadIdx.x < 9)
        sync[threadIdx.x * SYNC_STRIDE] = 0u;
}

// What the launcher has learnt about a device (fq_init, or the first use where allocating is allowed).
struct DecodeDevice {
    bool ready = false, usable = false;
    int cus = 0;
    unsigned *host_err = nullptr;     // pinned host word the kernel raises when a workgroup gives up ...
    unsigned *host_err_dev = nullptr; // ... and its device address
};
DecodeDevice g_dec[16];
std::mutex g_dec_guard;
unsigned long long g_give_up_ticks = 200000000ull; // two seconds of the 100 MHz timer
unsigned long long g_persistent_launches = 0;      // persistent launches queued by this process
int g_decode_mode = 0;                             // 0: per-phase launches (default), 1: persistent kernel where it applies

struct LdsPlan {
    int npg;
    unsigned off_raw, off_sums, off_red, off_part, total;
};

bool plan_lds(int H, int F, LdsPlan &p)
{
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    const size_t raw = up(std::max<size_t>((size_t)3 * H * 2, (size_t)2 * F * 2));
    const size_t sums = up((size_t)5 * (std::max(H, F) >> 7) * 4);
    const size_t red = (size_t)DW * ROWS_MAX * 4, part = 256;
    const size_t fixed = raw + sums + red + part;
    if (fixed >= LDS_LIMIT)
        return false;
    int npg = (int)((LDS_LIMIT - fixed) / ((size_t)DW * PAGE));
    npg = std::min(npg, NPG_MAX);
    if (npg < NPG_MIN)
        return false;
    p.npg = npg;
    p.off_raw = (unsigned)((size_t)DW * npg * PAGE);
    p.off_sums = (unsigned)(p.off_raw + raw);
    p.off_red = (unsigned)(p.off_sums + sums);
    p.off_part = (unsigned)(p.off_red + red);
    p.total = (unsigned)(p.off_part + part);
    return p.total <= LDS_LIMIT;
}

// Rows of a phase a workgroup finishes at most, for the phase's bit-widths: decides whether the reduction
// buffer holds them.  The answer depends on few things, so the last answers are kept.
int max_rows_per_workgroup(unsigned bits4, int ph, int N, int grid)
{
    struct Seen {
        unsigned key;
        int N, grid, rows;
    };
    static Seen seen[64];
    static int count = 0;
    static std::mutex guard;
    const int first = phase_first(ph), cnt = phase_count(ph);
    unsigned key = (unsigned)ph;
    for (int j = 0; j < cnt; ++j)
        key = key * 16u + (unsigned)bits_at(bits4, first + j);
    std::lock_guard<std::mutex> lock(guard);
    for (int i = 0; i < count; ++i)
        if (seen[i].key == key && seen[i].N == N && seen[i].grid == grid)
            return seen[i].rows;
    int worst = 0;
    for (int wg = 0; wg < grid; ++wg) {
        PhaseWork w;
        phase_work(bits4, ph, N, wg, grid, w);
        int rows = 0;
        for (int j = 0; j < cnt; ++j)
            rows += (w.u1[j] - w.u0[j]) * 16 * subs_of(bits_at(bits4, first + j));
        worst = std::max(worst, rows);
    }
    if (count < 64)
        seen[count++] = Seen{key, N, grid, worst};
    return worst;
}

int decode_prepare_locked(DecodeDevice &d, int dev, bool may_allocate)
{
    if (d.ready)
        return 0;
    if (!may_allocate)
        return -1;
    int n = 0;
    hipError_t e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess)
        return (int)e;
    d.cus = n;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(decode_persist_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_LIMIT);
    int per_cu = 0;
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_persist_kernel, DTHREADS, LDS_LIMIT);
    // the grid is one workgroup per compute unit and all of them must be resident together
    d.usable = e == hipSuccess && per_cu >= 1 && n >= 8 && n % 8 == 0;
    if (e != hipSuccess)
        (void)hipGetLastError(); // the per-phase launches serve instead
    if (d.usable) {
        void *h = nullptr, *hd = nullptr;
        if (hipHostMalloc(&h, 64, hipHostMallocMapped) == hipSuccess && hipHostGetDevicePointer(&hd, h, 0) == hipSuccess) {
            d.host_err = static_cast<unsigned *>(h);
            d.host_err_dev = static_cast<unsigned *>(hd);
            *d.host_err = 0;
        } else {
            (void)hipGetLastError();
            d.usable = false;
        }
    }
    d.ready = true;
    return 0;
}

DecodeDevice *decode_device(bool may_allocate, int *rc)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 16) {
        *rc = e != hipSuccess ? (int)e : (int)hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_dec_guard);
    *rc = decode_prepare_locked(g_dec[dev], dev, may_allocate);
    return *rc == 0 ? &g_dec[dev] : nullptr;
}

} // namespace

int fq_decode_prepare()
{
    int rc = 0;
    decode_device(true, &rc);
    return rc;
}

bool fq_decode_async_error()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16)
        return false;
    const DecodeDevice &d = g_dec[dev];
    return d.host_err && *reinterpret_cast<volatile unsigned *>(d.host_err) != 0;
}

void fq_decode_clear_async_error()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16)
        return;
    if (g_dec[dev].host_err)
        *reinterpret_cast<volatile unsigned *>(g_dec[dev].host_err) = 0;
}

unsigned long long fq_decode_set_give_up_ticks(unsigned long long ticks)
{
    const unsigned long long old = g_give_up_ticks;
    g_give_up_ticks = ticks;
    return old;
}

// 1 if fq_launch_decode_persist would run the persistent kernel for blocks of this size on the current
// device (prepared, resident grid possible, LDS plan fits); per-phase limits on the bit vector aside.
int fq_decode_available(int H, int F)
{
    if (H > 8 * DCOMPUTE * RES || F > 8 * DCOMPUTE * TRIPS || H <= 0 || F <= 0 || H % 128 || F % 128)
        return 0;
    int rc = 0;
    DecodeDevice *d = decode_device(false, &rc);
    LdsPlan lp;
    return d && d->usable && plan_lds(H, F, lp) ? lp.npg : 0;
}

void fq_decode_partition_of(unsigned bits4, int ph, int N, int wg, int grid, int *out6)
{
    PhaseWork w;
    phase_work(bits4, ph, N, wg, grid, w);
    for (int j = 0; j < 3; ++j) {
        out6[2 * j] = w.u0[j];
        out6[2 * j + 1] = w.u1[j];
    }
}

unsigned long long fq_decode_launches() { return g_persistent_launches; }

int fq_decode_set_mode(int mode)
{
    const int old = g_decode_mode;
    g_decode_mode = mode == 1 ? 1 : 0;
    return old;
}

// One token through L blocks in as few launches as the kernel-argument size allows.  Returns 0 when the work
// has been queued, -1 when the persistent kernel does not apply here (the caller then queues the per-phase
// launches), otherwise a hipError_t.
int fq_launch_decode_persist(const fq_layer *layers, int L, const uint8_t *bitvec, int H, int F, const void *x_in,
                             void *x_out, const fq_decode_buffers &b, bool may_allocate, fq_stream st)
{
    if (g_decode_mode != 1 || H > 8 * DCOMPUTE * RES || F > 8 * DCOMPUTE * TRIPS || H % 128 != 0 || F % 128 != 0)
        return -1;
    int rc = 0;
    DecodeDevice *d = decode_device(may_allocate, &rc);
    if (!d)
        return rc > 0 ? rc : -1;
    if (!d->usable)
        return -1;
    LdsPlan lp;
    if (!plan_lds(H, F, lp))
        return -1;
    const int grid = d->cus;
    auto pack_bits = [&](int l) {
        unsigned v = 0;
        for (int j = 0; j < 7; ++j)
            v |= (unsigned)bitvec[7 * l + j] << (4 * j);
        return v;
    };
    for (int l = 0; l < L; ++l)
        for (int ph = 0; ph < 4; ++ph)
            if (max_rows_per_workgroup(pack_bits(l), ph, ph == 2 ? F : H, grid) > ROWS_MAX)
                return -1;

    hipLaunchKernelGGL(decode_clear_kernel, dim3(1), dim3(64), 0, st, static_cast<unsigned *>(b.sync));
    if (hipError_t e = hipGetLastError(); e != hipSuccess)
        return (int)e;
    DecodeArgs a;
    a.H = H;
    a.F = F;
    a.npg = lp.npg;
    a.give_up_ticks = g_give_up_ticks;
    a.x_in = static_cast<const _Float16 *>(x_in);
    a.x_out = static_cast<_Float16 *>(x_out);
    void *const bufs[8] = {b.q, b.k, b.v, b.o, b.g, b.p, b.d, b.x1};
    for (int i = 0; i < 8; ++i)
        a.buf[i] = static_cast<_Float16 *>(bufs[i]);
    a.sync = static_cast<unsigned *>(b.sync);
    a.host_err = d->host_err_dev;
    a.off_raw = lp.off_raw;
    a.off_sums = lp.off_sums;
    a.off_red = lp.off_red;
    a.off_part = lp.off_part;
    unsigned gen = 0;
    for (int l0 = 0; l0 < L; l0 += DNB) {
        const int nb = std::min(DNB, L - l0);
        a.nblocks = nb;
        a.first = l0 == 0;
        a.last = l0 + nb == L;
        a.gen0 = gen;
        for (int i = 0; i < nb; ++i) {
            const fq_layer &ly = layers[l0 + i];
            for (int j = 0; j < 7; ++j) {
                const int bits = bitvec[7 * (l0 + i) + j], bi = fq_bits_index(bits);
                a.blk[i].packed[j] = static_cast<const uint32_t *>(ly.m[j].packed[bi]);
                a.blk[i].scales[j] = static_cast<const _Float16 *>(ly.m[j].scales[bi]);
                a.blk[i].zeros[j] = static_cast<const _Float16 *>(ly.m[j].zeros[bi]);
            }
            a.blk[i].bits4 = pack_bits(l0 + i);
            a.blk[i].pad = 0;
        }
        hipLaunchKernelGGL(decode_persist_kernel, dim3(grid), dim3(DTHREADS), lp.total, st, a);
        if (hipError_t e = hipGetLastError(); e != hipSuccess)
            return (int)e;
        ++g_persistent_launches;
        gen += (unsigned)nb * 4u;
    }
    return 0;
}
