// Stage 2: the min-plus recurrence over the latency-budget grid.
//
// Section 4.4 adds the pipeline's models one at a time and, for every budget,
// splits it between the current model and the rest.  With the candidate tables
// of stage 1 that is, for models s = S-1 .. 0 and budgets t = 0 .. T,
//
//     f[S][t] = 0
//     f[s][t] = min over candidates k with lt[s][k] <= t of
//               cost[s][k] + f[s+1][t - lt[s][k]]          (F_INF if none)
//
// (the suffix form: f[s][t] is the least cost of models s.. within t ticks, so
// that stage 3 can rebuild the choice forward from model 0).
//
// Mapping.  One workgroup per instance.  Lanes run over t and the candidate
// loop is wave-uniform: a candidate contributes f[s+1] shifted by lt, a
// unit-stride LDS read.  The row's entries (shift and cost packed into one dword)
// are staged in LDS once per model and every lane reads the same words (a
// broadcast, four entries at a time), so they arrive in VGPRs in order with the
// row reads.  There is no cross-lane traffic and no
// argmin bookkeeping in the loop: only f is kept, and stage 3 recovers the
// argmin from the stored rows.
//
// f is 16 bits wide (totals are bounded by THEMIS_COST_LIMIT), so a dword holds
// two cells and one v_pk_add_u16 + one v_pk_min_u16 relax two cells.  LDS reads
// are only fast at natural alignment (a misaligned ds_read is ~25x slower), and
// a shift by lt moves the row by an arbitrary number of 2-byte cells, so the
// previous row is kept in LDS once per residue of the shift: copy m is the row
// shifted by m cells, and a candidate reads the copy whose residue fits, always
// aligned.  Two copies with 32-bit reads (lt mod 2) are kept: four copies with
// 64-bit reads halve the LDS instructions but double the LDS footprint, and the
// resident wavefronts that costs weigh more (measured).  Rows of more than 16384
// cells go to the narrow kernel (two copies, static chunks).
// New values stay in registers while the old row is being read.
//
// The row is cut into positions of 512 cells.  A candidate only reaches the
// positions whose last cell is >= lt, and stage 1 ordered every row of the
// candidate table by lt / 512, so the candidates that reach position p are the
// first bcum[p+1] entries of the row: the inner loops run over a prefix with no
// test per candidate.  Work per position therefore grows with p; the wavefronts
// of a workgroup take positions from a counter, most expensive first (or, in the
// kernel for pruned rows, own a late and an early position each).  A stretch
// of F_INF in front of every copy serves the reads that reach below t = 0, and
// doubles as the harmless target of the entries that pad a group of four beyond
// the prefix.
//
// Scheduling.  Instances were listed by row length (work class) in stage 1.  A
// launch serves a group of classes with the geometry of the group's longest
// rows: a workgroup of exactly the wavefronts those need, and just enough
// workgroups to fill the chip.  Each workgroup starts on the list entry of its
// own index and then pulls further ones through an atomic cursor until the
// lists are exhausted, longest rows first, so the launch ends on the short
// ones.  Usually one launch serves every class; see make_plan().
#include <type_traits>
#include "instance_queue.h"
#include "themis_internal.h"

namespace themis {
namespace {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_add(uint32_t a, uint32_t b)
{
    u16x2 r = __builtin_bit_cast(u16x2, a) + __builtin_bit_cast(u16x2, b);
    return __builtin_bit_cast(uint32_t, r);
}

// a + (high half of e) in both cells: the operand-select bits of the packed add
// route the entry's cost to both lanes, so it need not be replicated first.
__device__ __forceinline__ uint32_t pk_add_hi(uint32_t a, uint32_t e)
{
    uint32_t r;
    asm("v_pk_add_u16 %0, %1, %2 op_sel:[0,1] op_sel_hi:[1,1]" : "=v"(r) : "v"(a), "v"(e));
    return r;
}

// base + 4 * (low half of e): one multiply-add on 16-bit operands
__device__ __forceinline__ uint32_t add_dwords_lo(uint32_t base, uint32_t e)
{
    uint32_t r;
    asm("v_mad_u32_u16 %0, %1, 4, %2" : "=v"(r) : "v"(e), "v"(base));
    return r;
}

__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{
    u16x2 r = __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
    return __builtin_bit_cast(uint32_t, r);
}

#define AS_LDS __attribute__((address_space(3)))

// The workgroup's dynamic LDS.  Functions kept out of line take their LDS
// pointers from here, not from their caller: a pointer that crosses a call is
// a generic one, and every access through it becomes a flat instruction (the
// volatile publishing stores even one that is waited for on the spot).
extern __shared__ uint32_t wide_lds[];

// LDS address (byte offset within the workgroup's allocation) of a pointer into it
__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(uintptr_t)(const AS_LDS char*)p;
}

// Entry idx of a row of bcum, for a wavefront-uniform idx.  The hardware has no
// 16-bit scalar loads, and a 16-bit read would become a vector load whose wait
// also waits for every vector load issued before it (the prefetched entries);
// so the dword that holds the entry is read through the scalar cache and the
// half picked.  Rows of bcum start on a dword boundary (their length is even).
__device__ __forceinline__ int bcum_at(const AS_CONST uint16_t* bc, int idx)
{
    const uint32_t pair = reinterpret_cast<const AS_CONST uint32_t*>(bc)[idx >> 1];
    return (int)((idx & 1) ? pair >> 16 : pair & 0xFFFFu);
}

// Entries of the row that can reach a position whose last cell is `last_cell`.
__device__ __forceinline__ int prefix_count(const AS_CONST uint16_t* bc, int last_cell)
{
    return bcum_at(bc, (last_cell >> BUCKET_SHIFT) + 1);
}

// ------------------------------------------------------------------ wide kernel
// Lane elements are pairs (2 cells, 4 bytes), four per position, read with
// ds_read_b32 from the copy lt mod 2.  A position is 512 cells and a lane keeps
// 4 dwords of it.
constexpr int POSC = BUCKET_CELLS;    // cells per position
constexpr int PADB = WIDE_PAD_BYTES;  // bytes of F_INF in front of every copy
constexpr int AD = 4;                 // accumulator dwords per lane per position
constexpr int COPIES = WIDE_COPIES;   // shifted copies of the row
constexpr int CAND_BUF = 512;         // entries of a row staged in LDS at a time
// Staged entries (the form the sweep reads from LDS) are one dword: the cost in
// the high half, and in the low half the shift in dwords plus SHIFT_BIAS, which
// makes it unsigned (shifts reach from -2 * 16384 bytes to +1 copy).
constexpr uint32_t SHIFT_BIAS = 8192;
static_assert(4 * SHIFT_BIAS >= 2 * WIDE_MAX_CELLS, "the bias covers the longest shift down");
static_assert(SHIFT_BIAS + (WIDE_PAD_BYTES + WIDE_MAX_CELLS * 2) / 4 < 65536,
              "biased shifts fit sixteen bits");
static_assert(4 * SHIFT_BIAS >= WIDE_PAD_BYTES + (WIDE_MAX_CELLS / BUCKET_CELLS - 1) * BUCKET_CELLS * 2,
              "the bias covers the parking shift of the last position");
static_assert(WIDE_CHUNK == 2 * POSC, "a wavefront holds two positions");
static_assert(PADB == POSC * 2, "the pad is as long as one position");
static_assert(16 * 64 * 16 / 32 * 4 <= 2 * PADB,
              "two copies hold a padded dword per cell of the longest row");

struct Geo {
    static constexpr int ELT = 4;                     // bytes per lane element
    static constexpr int NE = AD * 4 / ELT;           // lane elements per position
    // byte offset (inside a copy) of a lane's first element of position pos,
    // less the bias that staged entries carry in their shift
    static __device__ __forceinline__ uint32_t lane_byte(int pos, int lane)
    {
        return (uint32_t)(PADB + ELT * (pos * (64 * NE) + lane)) - 4u * SHIFT_BIAS;
    }
    // a staged entry (cost 0) whose shift lands the position's reads on the F_INF
    // pad of copy 0
    static __device__ __forceinline__ uint32_t park(int pos)
    {
        return SHIFT_BIAS - (uint32_t)((PADB + ELT * pos * (64 * NE)) / 4);
    }
    // Reads the first NEA of the lane's NE elements.  `at` is an LDS address (an
    // integer, so that the lane's base and the start of the copies fold into one
    // register outside the loop).
    template <int NEA>
    static __device__ __forceinline__ void read(uint32_t (&dst)[AD], uint32_t at)
    {
        const AS_LDS uint32_t* src = (const AS_LDS uint32_t*)(size_t)at;
#pragma unroll
        for (int u = 0; u < NEA; ++u) dst[u] = src[u * 64];
    }
    // Lane elements of position pos that hold any cell <= T (pos is one of the
    // row's positions, so at least one does): element q starts 64 * ELT / 2 cells
    // after element q - 1.
    static __device__ __forceinline__ int live_elements(int pos, int T)
    {
        const int n = (T - pos * POSC) / (64 * (ELT / 2)) + 1;
        return n < NE ? n : NE;
    }
};

// Sweep the first ke staged entries of a bucket-ordered row over one position.
// `ent` points at the staged entries in LDS; every lane reads the same words (a
// broadcast), so shift and cost arrive in VGPRs without touching the scalar
// unit, four entries per read.
//
// The loop is software-pipelined by hand: the row reads of entry k+D are issued
// before the arithmetic of entry k, into a ring of D+1 buffers, and the entries
// themselves are fetched one (D = 1) or two (D = 3) groups of four ahead, so a
// wavefront always has reads in flight while it works.  The scheduling barriers
// keep the compiler from undoing that order.  Entries at or beyond ke (the
// rest of the row, or the padding behind it) are parked on the F_INF pad, where
// they change nothing; with EXACT (D = 1) the last group of a prefix is instead
// straight-line code of exactly the entries left, picked by a switch: on pruned
// rows, where a position is a handful of entries, up to three idle ones at ten
// instructions each are a measurable share (on dense rows the extra code costs
// more than it saves).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int D, int NEA = Geo::NE, bool EXACT = false>
__device__ __forceinline__ void sweep(uint32_t (&acc)[AD], const char* ldsb, const uint32_t* ent,
                                      int ke, uint32_t byte_pos, uint32_t park)
{
    static_assert(D == 1 || D == 3, "the buffer ring must divide the group of four");
    using G = Geo;
    constexpr int ADA = NEA * (G::ELT / 4);  // accumulator dwords in use
    if (ke <= 0) return;
    constexpr int NQ = D == 1 ? 2 : 3;  // groups of entries held in registers
    const uint32_t lane_base = lds_address(ldsb) + byte_pos;
    const AS_LDS u32x4* const ent4 = (const AS_LDS u32x4*)(size_t)lds_address(ent);
    uint32_t buf[D + 1][AD];
    u32x4 q[NQ];

    auto issue = [&](uint32_t en, int slot) {
        G::template read<NEA>(buf[slot], add_dwords_lo(lane_base, en));
    };
    auto consume = [&](uint32_t en, int slot) {
        uint32_t t[AD];
        // all the adds, then all the mins: no add feeds the instruction after it
#pragma unroll
        for (int u = 0; u < ADA; ++u) t[u] = pk_add_hi(buf[slot][u], en);
#pragma unroll
        for (int u = 0; u < ADA; ++u) acc[u] = pk_min(acc[u], t[u]);
    };

#pragma unroll
    for (int r = 0; r < NQ - 1; ++r) q[r] = ent4[r];
#pragma unroll
    for (int z = 0; z < D; ++z) issue(z < ke ? q[0][z] : park, z);

    // One group: entries k0 .. k0+3 are relaxed while the reads of k0+D .. k0+3+D
    // are issued; `cur` is the register group that holds entries k0 .. k0+3.
    auto group = [&](int k0, int cur, bool tail) {
        q[(cur + NQ - 1) % NQ] = ent4[(k0 >> 2) + NQ - 1];
#pragma unroll
        for (int z = 0; z < 4; ++z) {
            const int x = z + D;
            uint32_t en = x < 4 ? q[cur][x & 3] : q[(cur + 1) % NQ][x & 3];
            if (tail) en = k0 + x < ke ? en : park;
            issue(en, x % (D + 1));
            __builtin_amdgcn_sched_barrier(0);
            consume(q[cur][z], z % (D + 1));
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // (EXACT) the last REM entries of the prefix
    auto rest = [&](int cur, auto rem) {
        constexpr int REM = decltype(rem)::value;
#pragma unroll
        for (int z = 0; z < REM; ++z) {
            const int x = z + D;
            if (x < REM) issue(q[cur][x & 3], x % (D + 1));
            __builtin_amdgcn_sched_barrier(0);
            consume(q[cur][z & 3], z % (D + 1));
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    for (int k0 = 0; k0 < ke; k0 += 4 * NQ) {
#pragma unroll
        for (int r = 0; r < NQ; ++r) {
            const int k = k0 + 4 * r;
            if (k >= ke) break;
            if (k + 4 + D <= ke)
                group(k, r, false);
            else if (EXACT && D == 1) {
                switch (ke - k) {
                case 1: rest(r, std::integral_constant<int, 1>{}); break;
                case 2: rest(r, std::integral_constant<int, 2>{}); break;
                case 3: rest(r, std::integral_constant<int, 3>{}); break;
                default: rest(r, std::integral_constant<int, 4>{}); break;
                }
            } else
                group(k, r, true);
        }
    }
}

// The same for a position of which only the first `nea` lane elements hold
// cells of the row (the top position of a row whose length is not a multiple of
// the position size): the elements beyond T are neither read nor relaxed.  The
// top position is the one every entry reaches, so on short rows this is a
// sizeable part of all the work.
template <int D, bool EXACT = false>
__device__ __forceinline__ void sweep_live(uint32_t (&acc)[AD], const char* ldsb,
                                           const uint32_t* ent, int ke, uint32_t byte_pos,
                                           uint32_t park, int nea)
{
    if (nea >= Geo::NE)
        sweep<D, Geo::NE, EXACT>(acc, ldsb, ent, ke, byte_pos, park);
    else if (nea == 1)
        sweep<D, 1, EXACT>(acc, ldsb, ent, ke, byte_pos, park);
    else if (nea == 2)
        sweep<D, 2, EXACT>(acc, ldsb, ent, ke, byte_pos, park);
    else
        sweep<D, 3, EXACT>(acc, ldsb, ent, ke, byte_pos, park);
}

// Whether every cell of position pos is a cell of the row (only the top position
// of a row can be cut short by T).  Uniform over the wavefront.
__device__ __forceinline__ bool whole_position(int pos, int T) { return (pos + 1) * POSC - 1 <= T; }

// Store a finished position to the HBM row (cells <= T only).
__device__ __forceinline__ void store_position(const uint32_t (&acc)[AD], uint16_t* out, int pos,
                                               int lane, int T)
{
    using G = Geo;
    uint32_t* const at = reinterpret_cast<uint32_t*>(out) + pos * (64 * G::NE) + lane;
    if (whole_position(pos, T)) {
#pragma unroll
        for (int q = 0; q < G::NE; ++q) at[q * 64] = acc[q];
        return;
    }
    const int room = T - (G::ELT / 2) * (pos * (64 * G::NE) + lane);  // cells up to T from the lane's first
#pragma unroll
    for (int q = 0; q < G::NE; ++q)
        if ((G::ELT / 2) * q * 64 <= room) at[q * 64] = acc[q];
}

// F_INF + cost back to F_INF
__device__ __forceinline__ void clamp_position(uint32_t (&acc)[AD])
{
#pragma unroll
    for (int u = 0; u < AD; ++u) acc[u] = pk_min(acc[u], F_INF2);
}

__device__ __forceinline__ void finish_position(uint32_t (&acc)[AD], uint16_t* out, int pos,
                                                int lane, int T)
{
    clamp_position(acc);
    store_position(acc, out, pos, lane, T);
}

// Write one lane element of the new row into the shifted LDS copies.  `at` is
// the element's LDS address in copy 0; copy m holds cell t at half-word
// (PADB/2 + t - m).  Each store must stay a naturally aligned access of exactly
// this width (merged neighbours would be misaligned, and a misaligned LDS access
// is many times slower), and it must be an LDS instruction: written as volatile
// stores through ordinary pointers they came out as flat stores, each one waited
// for before the next.  Hence the instructions themselves.  The compiler does
// not count them; publish_wait() before the barrier that ends the publishing.
// (OFF: a constant byte offset that rides in the instruction)
template <int OFF = 0>
__device__ __forceinline__ void lds_store_b32(uint32_t at, uint32_t v)
{
    asm volatile("ds_write_b32 %0, %1 offset:%2" : : "v"(at), "v"(v), "n"(OFF) : "memory");
}
// the low half of v at `at` + OFF, the high half GAP (a multiple of two) above it
template <int GAP, int OFF = 0>
__device__ __forceinline__ void lds_store_halves(uint32_t at, uint32_t v)
{
    asm volatile("ds_write_b16 %0, %1 offset:%2\n\tds_write_b16_d16_hi %0, %1 offset:%3"
                 :
                 : "v"(at), "v"(v), "n"(OFF), "n"(OFF + GAP)
                 : "memory");
}
__device__ __forceinline__ void publish_wait()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// `at`: the element's address in copy 0, less OFF; `at1`: the same in copy 1,
// two bytes lower
template <int OFF = 0>
__device__ __forceinline__ void publish_pair(uint32_t at, uint32_t at1, uint32_t v)
{
    lds_store_b32<OFF>(at, v);         // copy 0: c0 c1
    lds_store_halves<2, OFF>(at1, v);  // copy 1: c0 | c1 from two bytes below
}

// Write a finished position from the registers of the wavefront that computed
// it into the LDS copies (cells beyond T stay as they are; nothing reads them).
__device__ __forceinline__ void publish_position(const uint32_t (&acc)[AD], char* ldsb, int CSB,
                                                 int pos, int lane, int T)
{
    using G = Geo;
    static_assert(G::NE == 4, "unrolled by hand for the offsets");
    const int el = pos * (64 * G::NE) + lane;
    const uint32_t at = lds_address(ldsb) + (uint32_t)(PADB + G::ELT * el);
    const uint32_t at1 = at + (uint32_t)CSB - 2u;
    constexpr int STEP = 64 * G::ELT;  // bytes from one lane element to the next
    if (whole_position(pos, T)) {
        publish_pair<0 * STEP>(at, at1, acc[0]);
        publish_pair<1 * STEP>(at, at1, acc[1]);
        publish_pair<2 * STEP>(at, at1, acc[2]);
        publish_pair<3 * STEP>(at, at1, acc[3]);
        return;
    }
    const int room = T - (G::ELT / 2) * el;  // cells up to T from the lane's first
    if (0 * 64 * (G::ELT / 2) <= room) publish_pair<0 * STEP>(at, at1, acc[0]);
    if (1 * 64 * (G::ELT / 2) <= room) publish_pair<1 * STEP>(at, at1, acc[1]);
    if (2 * 64 * (G::ELT / 2) <= room) publish_pair<2 * STEP>(at, at1, acc[2]);
    if (3 * 64 * (G::ELT / 2) <= room) publish_pair<3 * STEP>(at, at1, acc[3]);
}

// Entries of one row held in registers on their way from HBM to the LDS
// staging buffer (loaded before a model's sweeps, stored after them).  They are
// held as loaded and every load is issued whatever the row's length (beyond it,
// slot 0 is read and dropped): a load under a test of its own, or one whose
// value is worked on at once, is waited for on the spot, and the sweeps would
// start after four memory latencies instead of hiding them.
constexpr int PREFETCH = 2;  // entries per thread

// An entry as the sweep wants it in LDS (see SHIFT_BIAS); the index is dropped.
// (The padding entries behind a row are only ever fetched, never relaxed: the
// sweep parks whatever lies at or beyond its end.)
__device__ __forceinline__ uint32_t staged(StepEntry se)
{
    return (se.ck << 16) | (((uint32_t)((int32_t)se.shift >> 2) + SHIFT_BIAS) & 0xFFFFu);
}

struct RowPrefetch {
    StepEntry e[PREFETCH];
    int cnt;  // entries of the row to stage (at most CAND_BUF); 16 padding entries follow
};

__device__ __forceinline__ void prefetch_row(RowPrefetch& pf, const StepEntry* grow, int cnt)
{
    pf.cnt = cnt;
#pragma unroll
    for (int j = 0; j < PREFETCH; ++j) {
        const int x = (int)threadIdx.x + j * (int)blockDim.x;
        pf.e[j] = grow[x < cnt ? x : 0];  // a row's stretch of the table has eight slots at least
    }
}

__device__ __forceinline__ void commit_row(const RowPrefetch& pf, const StepEntry* grow,
                                           uint32_t* cbuf)
{
    StepEntry none;
    none.shift = 0u;
    none.ck = 0u;
#pragma unroll
    for (int j = 0; j < PREFETCH; ++j) {
        const int x = (int)threadIdx.x + j * (int)blockDim.x;
        if (x < pf.cnt + 16) cbuf[x] = staged(x < pf.cnt ? pf.e[j] : none);
    }
    // whatever the registers did not cover
    for (int x = (int)threadIdx.x + PREFETCH * (int)blockDim.x; x < pf.cnt + 16;
         x += (int)blockDim.x) {
        StepEntry se = none;
        if (x < pf.cnt) se = grow[x];
        cbuf[x] = staged(se);
    }
}

// The first model of the recurrence by scatter and scan (see the call).  Kept
// out of line so that its registers do not weigh on the allocation of the sweep
// loop; every thread of the workgroup calls it.
__device__ __attribute__((noinline)) void first_model_by_scan(
    int CSB, const StepEntry* __restrict__ step_tab,
    const uint16_t* __restrict__ bcum, uint16_t* __restrict__ frow, int i, int S, int Kp, int nbs,
    int row_stride, int T, int npos, int cand_buf)
{
    // The model handled first (s = S-1) follows the all-zero row f[S], so its
    // row is a running minimum, f[S-1][t] = least cost among the entries with
    // lt <= t, and costs a scatter and a scan instead of a sweep per entry (in
    // the paper's own loop this is the step that starts from the single state
    // "nothing spent").  One dword per cell, laid over the row copies, takes
    // the least cost per latency; a min-scan over the cells makes the row.
    const int nt = (int)blockDim.x;
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t* const lds = wide_lds;
    char* const ldsb = reinterpret_cast<char*>(wide_lds);
    uint32_t* const cbuf = reinterpret_cast<uint32_t*>(ldsb + COPIES * CSB + 16);  // as in the kernel
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t row = (size_t)i * S + (S - 1);
    const StepEntry* const grow = step_tab + row * Kp;
    uint16_t* const out = frow + row * row_stride;
    const int n_all = bcum_at(as_constant(bcum + row * nbs), npos);  // all have lt <= T
    // One dword per cell over the first two copies, with a dword of padding per 32
    // cells: the scan below reads it with a stride of 16 cells per lane, which
    // unpadded lands on two LDS banks.  Every thread scans 16 cells; those beyond
    // T hold F_INF, so no cell needs a test of its own.
    uint32_t* const cell_min = lds;
    auto cell_at = [](int c) { return c + (c >> 5); };
    const int span = cell_at(16 * nt);  // dwords; fits two copies for up to 16 wavefronts

    // start fetching the next model's entries; they are stored after the scan
    RowPrefetch pf;
    const StepEntry* grow_next = grow;
    if (S > 1) {
        const int n_next = bcum_at(as_constant(bcum + (row - 1) * nbs), npos);
        grow_next = step_tab + (row - 1) * Kp;
        prefetch_row(pf, grow_next, n_next < cand_buf ? n_next : cand_buf);
    }
    for (int x = tid; x < span; x += nt) cell_min[x] = F_INF;
    __syncthreads();
    for (int e = tid; e < n_all; e += nt) {
        const StepEntry se = grow[e];
        atomicMin(&cell_min[cell_at((int)wide_lt_of_shift(se.shift, CSB))], se.ck & 0xFFFFu);
    }
    __syncthreads();
    const int c0 = tid * 16;
    uint32_t v[16];
    uint32_t run = F_INF;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const uint32_t x = cell_min[cell_at(c0 + j)];
        run = x < run ? x : run;
        v[j] = run;
    }
    // least cost of all earlier runs: scan over the lanes, then over the wavefronts
    uint32_t incl = run;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d, 64);
        if (lane >= d) incl = o < incl ? o : incl;
    }
    uint32_t before = __shfl_up(incl, 1, 64);
    if (lane == 0) before = F_INF;
    __syncthreads();  // cell_min has been read: the copies can be written
    if (lane == 63) cbuf[w] = incl;
    for (int x = tid; x < PADB / 4; x += nt) {
        lds[x] = F_INF2;
        lds[CSB / 4 + x] = F_INF2;
    }
    __syncthreads();
    for (int ww = 0; ww < w; ++ww) {
        const uint32_t o = cbuf[ww];
        before = o < before ? o : before;
    }
#pragma unroll
    for (int j = 0; j < 16; j += 2) {
        const int cell = c0 + j;
        if (cell <= T) {
            const uint32_t lo = v[j] < before ? v[j] : before;
            const uint32_t hi = v[j + 1] < before ? v[j + 1] : before;
            const uint32_t d = lo | (hi << 16);
            {
                const uint32_t at = lds_address(ldsb) + (uint32_t)(PADB + 2 * cell);
                publish_pair(at, at + (uint32_t)CSB - 2u, d);
            }
            *reinterpret_cast<uint32_t*>(out + cell) = d;
        }
    }
    publish_wait();
    __syncthreads();  // the wavefront totals in the staging buffer have been read
    if (S > 1) commit_row(pf, grow_next, cbuf);
}

// The answer of an instance without its last row (see the call).  Out of line
// for the same reason as first_model_by_scan(); every thread calls it.
__device__ __attribute__((noinline)) void answer_from_row_one(int CSB,
                                                              const StepEntry* __restrict__ grow,
                                                              int n_all, int cand_buf, int T,
                                                              int32_t* __restrict__ answer)
{
    char* const ldsb = reinterpret_cast<char*>(wide_lds);
    const uint32_t* const cbuf = reinterpret_cast<const uint32_t*>(ldsb + COPIES * CSB + 16);
    // Of the last row only two things are ever used: the least cost,
    // f[0][T], and the least budget that attains it.  Both follow from
    // row 1, which is in LDS, without building row 0:
    //   f[0][T] = min_k cost_k + f[1][T - lt_k]
    //   t*      = min_k lt_k + u_k,  u_k = first u with f[1][u] <= f[0][T] - cost_k
    // (rows never increase with the budget, so u_k is a binary search, and
    // c_k + f[1][u] cannot fall below the optimum for lt_k + u <= T; an
    // entry with no such u within T - lt_k does not attain it).
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t* const hdr = reinterpret_cast<uint32_t*>(ldsb + COPIES * CSB);  // [2], [3] are free
    const uint16_t* const row1 = reinterpret_cast<const uint16_t*>(ldsb + PADB);
    const int nt = (int)blockDim.x;
    if (tid == 0) {
        hdr[2] = 0xFFFFFFFFu;
        hdr[3] = 0xFFFFFFFFu;
    }
    __syncthreads();
    auto entry_of = [&](int x, uint32_t& lt, uint32_t& co) {
        const uint32_t e = x < cand_buf ? cbuf[x] : staged(grow[x]);
        co = e >> 16;
        lt = wide_lt_of_shift(4u * ((e & 0xFFFFu) - SHIFT_BIAS), CSB);
    };
    auto wave_min_into = [&](uint32_t v, uint32_t* dst) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const uint32_t o = __shfl_xor(v, d, 64);
            v = o < v ? o : v;
        }
        if (lane == 0) atomicMin(dst, v);
    };
    uint32_t mine = 0xFFFFFFFFu;
    for (int x = tid; x < n_all; x += nt) {
        uint32_t lt, co;
        entry_of(x, lt, co);
        const uint32_t rest = row1[T - (int)lt];
        const uint32_t v = rest >= F_INF ? F_INF : co + rest;
        mine = v < mine ? v : mine;
    }
    wave_min_into(mine, &hdr[2]);
    __syncthreads();
    const uint32_t best = hdr[2] < F_INF ? hdr[2] : F_INF;
    mine = 0xFFFFFFFFu;
    if (best < F_INF) {
        for (int x = tid; x < n_all; x += nt) {
            uint32_t lt, co;
            entry_of(x, lt, co);
            if (co > best) continue;
            const uint32_t need = best - co;
            int hi = T - (int)lt;
            if (row1[hi] > need) continue;  // this entry does not attain the optimum
            int lo = 0;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (row1[mid] <= need)
                    hi = mid;
                else
                    lo = mid + 1;
            }
            const uint32_t t = lt + (uint32_t)lo;
            mine = t < mine ? t : mine;
        }
    }
    wave_min_into(mine, &hdr[3]);
    __syncthreads();
    if (tid == 0) {
        answer[0] = (int32_t)best;
        answer[1] = best < F_INF ? (int32_t)hdr[3] : 0;
    }
}

// The positions of a row cost very different amounts of work (position p is
// reached by bcum[p+1] entries), so they are not dealt out in advance: the
// wavefronts of the workgroup take them one at a time from a counter in LDS,
// most expensive first.  A finished position goes to the HBM row at once; once
// every wavefront is done with the old row, the workgroup reads the new one
// back (it is still in L2) and spreads it over the LDS copies.  (Keeping a
// second set of copies to publish into directly costs more in occupancy than
// the round trip through L2 does.)  Pruned rows have a kernel of their own,
// k2_minplus_pruned below.
//
// Compiled for eight wavefronts per SIMD (64 VGPRs): the LDS footprints of the
// work classes are sized for 32 resident wavefronts per compute unit, which a
// few registers more would silently cut to 28.
//
// `shortcuts`: whether the first and the last model may take their shortcuts
// (off when this kernel serves a pruned problem that the kernel for pruned rows
// cannot take: the count of relaxations assumes every model of a pruned problem
// is swept).
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void k2_minplus_wide(
    const StepEntry* __restrict__ step_tab, const uint16_t* __restrict__ bcum,
    const int32_t* __restrict__ tmeta, const int32_t* __restrict__ order,
    int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow, int32_t* __restrict__ ans, int N,
    int S, int Kp, int nbs, int row_stride, int cls, int low_cls, int cand_buf, int shortcuts)
{
    using G = Geo;
    constexpr int DEPTH = 1;
    extern __shared__ uint32_t lds[];
    const int CSB = wide_copy_bytes(cls_waves(cls));  // bytes per copy: pad + the longest row
    const int SETB = COPIES * CSB;                    // bytes of all copies
    char* const ldsb = reinterpret_cast<char*>(lds);
    // after the copies: a dword for the instance queue, one for the position
    // counter, then the staging buffer for cand_buf (+16) candidate entries
    volatile uint32_t* const slot = reinterpret_cast<volatile uint32_t*>(ldsb + SETB);
    int* const next_pos = reinterpret_cast<int*>(ldsb + SETB + 4);
    uint32_t* const cbuf = reinterpret_cast<uint32_t*>(ldsb + SETB + 16);
    const uint32_t* const ent = cbuf;

    const int tid = threadIdx.x;
    const int lane = tid & 63;

    const int count = list_length(ctrl, cls, low_cls);
    int idx = -1;
    for (;;) {
        idx = next_index(slot, ctrl + N_CLS + cls, count, idx);
        if (idx < 0) break;
        const int i = list_entry(ctrl, order, N, cls, low_cls, idx);
        const int T = as_constant(tmeta)[i];
        const int npos = (T + POSC) / POSC;  // positions that hold cells 0..T

        // Whether the first and the last model are worth their shortcuts (below)
        // depends on how much sweeping they replace: entries times positions per
        // wavefront.  With a handful of entries (one-core solves) the plain sweeps
        // are cheaper than the scan and the searches.
        const int n_first = bcum_at(as_constant(bcum + ((size_t)i * S + (S - 1)) * nbs), npos);
        const bool scan_first = shortcuts && worth_shortcut(n_first, npos, (int)blockDim.x >> 6);
        if (!scan_first) {
            // rows before the first model: cells t < 0 are F_INF, cells t >= 0 are 0
            for (int x = tid; x < (PADB + npos * POSC * 2) / 4; x += (int)blockDim.x) {
#pragma unroll
                for (int m = 0; m < COPIES; ++m) {
                    const uint32_t h0 = 2 * x < PADB / 2 - m ? F_INF : 0u;
                    const uint32_t h1 = 2 * x + 1 < PADB / 2 - m ? F_INF : 0u;
                    lds[m * (CSB / 4) + x] = h0 | (h1 << 16);
                }
            }
            // entries of the first model
            const size_t row = (size_t)i * S + (S - 1);
            const int n_all = bcum_at(as_constant(bcum + row * nbs), npos);
            RowPrefetch pf;
            prefetch_row(pf, step_tab + row * Kp, n_all < cand_buf ? n_all : cand_buf);
            commit_row(pf, step_tab + row * Kp, cbuf);
            if (tid == 0) *next_pos = npos - 1;
        } else {
            first_model_by_scan(CSB, step_tab, bcum, frow, i, S, Kp, nbs, row_stride, T,
                                        npos, cand_buf);
            if (tid == 0) *next_pos = npos - 1;
        }
        __syncthreads();

        for (int s = scan_first ? S - 2 : S - 1; s >= 0; --s) {
            const size_t row = (size_t)i * S + s;
            const StepEntry* const grow = step_tab + row * Kp;
            const AS_CONST uint16_t* bc = as_constant(bcum + row * nbs);
            uint16_t* const out = frow + row * row_stride;
            const int n_all = bcum_at(bc, npos);  // entries that reach the top position: all feasible ones

            if (shortcuts && s == 0 && S > 1 && worth_shortcut(n_all, npos, (int)blockDim.x >> 6)) {
                answer_from_row_one(CSB, grow, n_all, cand_buf, T, ans + 2 * i);
                break;
            }

            // start fetching the next model's entries; they are stored after the sweeps
            RowPrefetch pf;
            const StepEntry* grow_next = grow;
            if (s > 0) {
                const int n_next = bcum_at(as_constant(bcum + (row - 1) * nbs), npos);
                grow_next = step_tab + (row - 1) * Kp;
                prefetch_row(pf, grow_next, n_next < cand_buf ? n_next : cand_buf);
            }

            const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
            const int nw = (int)blockDim.x >> 6;
            if (n_all <= cand_buf) {
                // the whole row is in the staging buffer (the usual case)
                for (;;) {
                    int p = 0;
                    if (lane == 0) p = atomicSub(next_pos, 1);
                    p = __builtin_amdgcn_readfirstlane(p);
                    if (p < 0) break;
                    uint32_t acc[AD];
#pragma unroll
                    for (int u = 0; u < AD; ++u) acc[u] = 0xFFFFFFFFu;
                    sweep_live<DEPTH>(acc, ldsb, ent, bcum_at(bc, p + 1), G::lane_byte(p, lane),
                                              G::park(p), G::live_elements(p, T));
                    finish_position(acc, out, p, lane, T);
                }
            } else {
                // a long row goes through the buffer in parts; every wavefront keeps
                // its positions (w, w + nw, ...) across the parts, with the partial
                // minimum parked in the HBM row in between
                for (int p0 = w; p0 < npos; p0 += nw) {
                    uint32_t acc[AD];
#pragma unroll
                    for (int u = 0; u < AD; ++u) acc[u] = 0xFFFFFFFFu;
                    finish_position(acc, out, p0, lane, T);  // start from "none"
                }
                for (int seg = 0; seg < n_all; seg += cand_buf) {
                    const int cnt = n_all - seg < cand_buf ? n_all - seg : cand_buf;
                    if (seg) {
                        __syncthreads();  // sweeps of the previous part are done
                        for (int x = tid; x < cnt + 16; x += (int)blockDim.x) {
                            StepEntry se;
                            se.shift = 0u;
                            se.ck = 0u;
                            if (x < cnt) se = grow[seg + x];
                            cbuf[x] = staged(se);
                        }
                        __syncthreads();
                    }
                    for (int p0 = w; p0 < npos; p0 += nw) {
                        const int n_p = bcum_at(bc, p0 + 1);
                        const int ke = n_p - seg < 0 ? 0 : (n_p - seg < cnt ? n_p - seg : cnt);
                        if (ke <= 0) continue;
                        uint32_t acc[AD];
#pragma unroll
                        for (int q = 0; q < G::NE; ++q) {
                            const int cell = (G::ELT / 2) * (p0 * (64 * G::NE) + q * 64 + lane);
                            acc[q] = cell <= T ? *reinterpret_cast<const uint32_t*>(out + cell)
                                               : F_INF2;
                        }
                        sweep<DEPTH>(acc, ldsb, ent, ke, G::lane_byte(p0, lane), G::park(p0));
                        finish_position(acc, out, p0, lane, T);
                    }
                }
            }
            if (s == 0) break;  // nothing reads the LDS copies of the last row

            __syncthreads();  // every wavefront is done with the old row; the new one is stored
            for (int el = tid; el * (G::ELT / 2) <= T; el += (int)blockDim.x) {
                const uint32_t at = lds_address(ldsb) + (uint32_t)(PADB + G::ELT * el);
                publish_pair(at, at + (uint32_t)CSB - 2u, *reinterpret_cast<const uint32_t*>(out + 2 * el));
            }
            // hand the next model its entries and its position counter
            commit_row(pf, grow_next, cbuf);
            if (tid == 0) *next_pos = npos - 1;
            publish_wait();
            __syncthreads();
        }
        __syncthreads();  // last row's reads are done before the LDS is re-initialised
    }
}

// ------------------------------------------------------- kernel for pruned rows
// With dominated candidates pruned, a row is a handful of entries, a position a
// few sweeps, and what is fixed per model weighs more than the sweeps.  So:
//
//  * every wavefront owns the w-th position from the top and, where the row has
//    more positions than the workgroup has wavefronts, one of the rest, dealt so
//    that the wavefront with the cheapest first position gets the dearest second
//    one; it keeps both results in registers and writes them into the LDS copies
//    itself after the barrier.  The HBM row is written for stage 3 only, and
//    nothing here reads it back or waits for its stores.
//  * the entries of as many of the pipeline's models as fit the staging buffer
//    together (usually all) are fetched at once: one memory latency per batch of
//    models, not one per model, whose wait would also wait for the row stores
//    issued before it (loads and stores retire through one counter).
//  * lane m of every wavefront keeps what the wavefront needs of the m-th model
//    in the order of the recurrence (model S-1-m): where its entries start and
//    how many of them reach each of the wavefront's two positions; a model's
//    sweeps take them from there with one cross-lane read each.
//
// For problems with Kp <= CAND_BUF (any single row fits the buffer) and at most
// 64 models; the launcher sends the others to k2_minplus_wide.  Measured on
// dense rows the dealt-out positions of that kernel are faster on four of five
// workloads, hence the two kernels.
template <bool CHUNKS>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void k2_minplus_pruned(
    const StepEntry* __restrict__ step_tab, const uint16_t* __restrict__ bcum,
    const int32_t* __restrict__ tmeta, const int32_t* __restrict__ order,
    int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow, int N, int S, int Kp, int nbs,
    int row_stride, int cls, int low_cls)
{
    using G = Geo;
    constexpr int DEPTH = 1;
    extern __shared__ uint32_t lds[];
    const int CSB = wide_copy_bytes(cls_waves(cls));  // bytes per copy: pad + the longest row
    const int SETB = COPIES * CSB;                    // bytes of all copies
    char* const ldsb = reinterpret_cast<char*>(lds);
    // after the copies: four dwords of thread 0's about the next instance (instance,
    // budget, list index; its chunk of the list), then the staging buffer for Kp
    // (+16) candidate entries
    volatile uint32_t* const slot = reinterpret_cast<volatile uint32_t*>(ldsb + SETB);
    uint32_t* const cbuf = reinterpret_cast<uint32_t*>(ldsb + SETB + 16);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = (int)blockDim.x >> 6;
    StepEntry none;
    none.shift = 0u;
    none.ck = 0u;

    // Instances come from the launch's list in the order of next_index().  What
    // identifies the next instance (list index, instance, budget) is a chain of
    // dependent memory latencies, several microseconds against the few an instance
    // of pruned rows takes; so thread 0 fetches it one link per model while the
    // workgroup works on the current instance, and hands it over through LDS.
    //
    // Pulls of short rows are in chunks: the cursor counts instances, and a pull
    // takes up to pull_max of them at once, fewer as the list runs out (a quarter
    // of what would be each workgroup's share of the rest), so that the last pulls
    // are single instances and the workgroups end level.  One address takes a
    // read-modify-write every twelve nanoseconds or so device-wide: a pull per
    // instance bounds a launch of many short rows by the cursor alone (86400 rows
    // of 2000 cells: 1.0 ms whatever the rows cost).  Workgroups of eight
    // wavefronts or more are few and their instances long: there single pulls
    // keep them level best, and their instantiation (CHUNKS false) is without the
    // chunk code, which costs the sweeps two registers (1.7 % there).
    const int pull_max = 16 / nw < 8 ? 16 / nw : 8;
    const int count = list_length(ctrl, cls, low_cls);
    int32_t* const cursor = ctrl + N_CLS + cls;
    const int dealt = static_rounds<true>(count, (int)gridDim.x) * (int)gridDim.x;
    // thread 0's chunk sits in LDS between its uses, not in registers the sweeps need:
    // (next list index of the chunk) << 4 | (instances left in it)
    if (CHUNKS && tid == 0) slot[3] = 0u;
    int idx = next_static_index<true>(count, -1);  // the first round is never pulled
    int i = -1, T = 0;
    if (idx >= 0) {
        i = list_entry(ctrl, order, N, cls, low_cls, idx);
        T = as_constant(tmeta)[i];
    }
    while (i >= 0) {
        // thread 0's fetch of the next instance, one link per call (every thread
        // calls, so that the link count stays uniform; `next` is thread 0's alone)
        idx = next_static_index<true>(count, idx);
        int link = 0, next = idx;
        auto pull_next = [&]() {
            if (link >= 3) return;
            if (tid == 0) {
                if (link == 0) {        // list index
                    if (next == -2) {
                        uint32_t chunk = CHUNKS ? slot[3] : 0u;
                        if (!CHUNKS) {
                            chunk = (uint32_t)(dealt + atomicAdd(cursor, 1)) << 4 | 1u;
                        } else if ((chunk & 15u) == 0u) {
                            // the cursor as last seen: where this workgroup's last chunk ended
                            const int seen = chunk ? (int)(chunk >> 4) : dealt;
                            int c = (count - seen) / (4 * (int)gridDim.x);
                            c = c < 1 ? 1 : (c > pull_max ? pull_max : c);
                            chunk = (uint32_t)(dealt + atomicAdd(cursor, c)) << 4 | (uint32_t)c;
                        }
                        next = (int)(chunk >> 4);
                        if (CHUNKS) slot[3] = chunk + 15u;  // index + 1, left - 1
                    }
                    slot[2] = (uint32_t)next;
                } else if (link == 1) {  // instance
                    int at = next;
                    next = -1;
                    for (int c = cls; c >= low_cls && at >= 0 && at < count; --c) {
                        const int n = as_constant(ctrl)[c];
                        if (at < n) {
                            next = order[(size_t)c * N + at];
                            break;
                        }
                        at -= n;
                    }
                } else {                 // budget
                    slot[0] = (uint32_t)next;
                    next = next >= 0 ? tmeta[next] : 0;
                }
            }
            ++link;
        };
        const int npos = (T + POSC) / POSC;  // positions that hold cells 0..T
        const int p_hi = npos - 1 - w;       // negative: none
        const int p_lo = npos - 2 * nw + w;  // negative: none

        int n_all_l = 0, n_hi_l = 0, n_lo_l = 0;
        if (lane < S) {
            const uint16_t* const bc = bcum + ((size_t)i * S + (size_t)(S - 1 - lane)) * nbs;
            n_all_l = bc[npos];  // entries that reach the top position: all feasible ones
            n_hi_l = bc[p_hi >= 0 ? p_hi + 1 : 0];
            n_lo_l = bc[p_lo >= 0 ? p_lo + 1 : 0];
        }
        // where each model's entries start when all are laid end to end, every row
        // starting on a group of four
        const int padded = (n_all_l + 3) & ~3;
        int end_l = padded;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(end_l, d, 64);
            if (lane >= d) end_l += o;
        }
        const int start_l = end_l - padded;

        // rows before the first model: cells t < 0 are F_INF, cells t >= 0 are 0
        for (int x = tid; x < (PADB + npos * POSC * 2) / 4; x += (int)blockDim.x) {
#pragma unroll
            for (int m = 0; m < COPIES; ++m) {
                const uint32_t h0 = 2 * x < PADB / 2 - m ? F_INF : 0u;
                const uint32_t h1 = 2 * x + 1 < PADB / 2 - m ? F_INF : 0u;
                lds[m * (CSB / 4) + x] = h0 | (h1 << 16);
            }
        }

        for (int m0 = 0; m0 < S;) {
            // the models m0 .. m1-1 fit the buffer together (a single one always does)
            const int base = __builtin_amdgcn_readlane(start_l, m0);
            const unsigned long long fit = __ballot(lane >= m0 && lane < S && end_l - base <= Kp);
            const int m1 = m0 + __builtin_popcountll(fit);
            for (int m = m0 + w; m < m1; m += nw) {
                const int n = __builtin_amdgcn_readlane(n_all_l, m);
                const int at = __builtin_amdgcn_readlane(start_l, m) - base;
                const StepEntry* const grow = step_tab + ((size_t)i * S + (size_t)(S - 1 - m)) * Kp;
                for (int e = lane; e < ((n + 3) & ~3); e += 64) {
                    StepEntry se = none;
                    if (e < n) se = grow[e];
                    cbuf[at + e] = staged(se);
                }
            }
            // the sweep fetches entries ahead of the end of its prefix
            if (tid < 16) cbuf[__builtin_amdgcn_readlane(end_l, m1 - 1) - base + tid] = staged(none);
            __syncthreads();

            for (int m = m0; m < m1; ++m) {
                const int s = S - 1 - m;
                pull_next();
                const uint32_t* const ent = cbuf + (__builtin_amdgcn_readlane(start_l, m) - base);
                uint16_t* const out = frow + ((size_t)i * S + s) * row_stride;
                uint32_t r_hi[AD], r_lo[AD];
                if (p_hi >= 0) {
#pragma unroll
                    for (int u = 0; u < AD; ++u) r_hi[u] = 0xFFFFFFFFu;
                    sweep_live<DEPTH, true>(r_hi, ldsb, ent, __builtin_amdgcn_readlane(n_hi_l, m),
                                      G::lane_byte(p_hi, lane), G::park(p_hi),
                                      G::live_elements(p_hi, T));
                    clamp_position(r_hi);
                }
                if (p_lo >= 0) {
#pragma unroll
                    for (int u = 0; u < AD; ++u) r_lo[u] = 0xFFFFFFFFu;
                    sweep<DEPTH, Geo::NE, true>(r_lo, ldsb, ent, __builtin_amdgcn_readlane(n_lo_l, m),
                                 G::lane_byte(p_lo, lane), G::park(p_lo));
                    clamp_position(r_lo);
                }
                if (s > 0) {  // nothing reads the LDS copies of the last row
                    lds_barrier();  // every wavefront is done with the old row
                    if (p_hi >= 0) publish_position(r_hi, ldsb, CSB, p_hi, lane, T);
                    if (p_lo >= 0) publish_position(r_lo, ldsb, CSB, p_lo, lane, T);
                }
                if (p_hi >= 0) store_position(r_hi, out, p_hi, lane, T);
                if (p_lo >= 0) store_position(r_lo, out, p_lo, lane, T);
                if (s > 0) lds_barrier();  // the new row is in the copies
            }
            m0 = m1;
        }
        // the links a short pipeline left over, then the hand-over
        pull_next();
        pull_next();
        pull_next();
        if (tid == 0) slot[1] = (uint32_t)next;
        __syncthreads();  // last row's reads are done before the LDS is re-initialised
        i = __builtin_amdgcn_readfirstlane((int)slot[0]);
        T = __builtin_amdgcn_readfirstlane((int)slot[1]);
        idx = __builtin_amdgcn_readfirstlane((int)slot[2]);
    }
}

// ---------------------------------------------------------------- narrow kernel
// Rows of up to 32768 cells: 16 wavefronts, each a contiguous chunk of 16
// dwords (32 cells) per lane, two copies read with ds_read_b32.
constexpr int NAR_NW = NAR_WAVES;
constexpr int NAR_U = NAR_CHUNK_DW / 64;     // dwords per lane
constexpr int NAR_CHUNK = NAR_CHUNK_DW;      // dwords per wavefront
constexpr int NAR_PADW = NAR_CHUNK;          // F_INF dwords in front of each copy
constexpr int NAR_BOFF = NAR_COPY_DW;        // dwords per copy, pad included

__global__ __launch_bounds__(NAR_NW * 64) void k2_minplus_narrow(
    const StepEntry* __restrict__ step_tab, const uint16_t* __restrict__ bcum,
    const int32_t* __restrict__ tmeta, const int32_t* __restrict__ order,
    int32_t* __restrict__ ctrl, uint16_t* __restrict__ frow, int N, int S, int Kp, int nbs,
    int row_stride)
{
    extern __shared__ uint32_t lds[];  // [A: pad + 16 chunks][B: pad + 16 chunks][slot]
    volatile uint32_t* const slot = lds + 2 * NAR_BOFF;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j0 = w * NAR_CHUNK;  // first dword of this wavefront's chunk
    const int count = as_constant(ctrl)[NARROW_CLS];
    const int32_t* const my_order = order + (size_t)NARROW_CLS * N;
    const int last_cell = 2 * (j0 + NAR_CHUNK) - 1;

    int idx = -1;
    for (;;) {
        idx = next_index(slot, ctrl + N_CLS + NARROW_CLS, count, idx);
        if (idx < 0) break;
        const int i = as_constant(my_order)[idx];
        const int T = as_constant(tmeta)[i];
        const int ndw = (T >> 1) + 1;  // dwords that hold cells 0..T
        const bool active = j0 < ndw;

        // copy A: dword j = cells (2j, 2j+1); copy B: dword j = cells (2j+1, 2j+2).
        // f[S][t] = 0 for t >= 0; pads F_INF; B's dword -1 is (cell -1, cell 0).
        for (int x = tid; x < NAR_BOFF; x += NAR_NW * 64) {
            lds[x] = x < NAR_PADW ? F_INF2 : 0u;
            lds[NAR_BOFF + x] = x < NAR_PADW - 1 ? F_INF2 : (x == NAR_PADW - 1 ? F_INF : 0u);
        }
        __syncthreads();

        for (int s = S - 1; s >= 0; --s) {
            uint32_t acc[NAR_U];
#pragma unroll
            for (int u = 0; u < NAR_U; ++u) acc[u] = 0xFFFFFFFFu;

            const size_t row = (size_t)i * S + s;
            if (active) {
                const AS_CONST StepEntry* ep = as_constant(step_tab + row * Kp);
                const int n = prefix_count(as_constant(bcum + row * nbs), last_cell > T ? T : last_cell);
                for (int k = 0; k < n; ++k) {
                    const uint32_t cost2 = (ep[k].ck & 0xFFFFu) * 0x10001u;
                    // shift = byte offset of the aligned source of dword 0 (copy A or B)
                    const uint32_t* src = lds + ((ep[k].shift >> 2) + j0 + lane);
#pragma unroll
                    for (int u = 0; u < NAR_U; ++u)
                        acc[u] = pk_min(acc[u], pk_add(src[u * 64], cost2));
                }
            }

            uint32_t* const out = reinterpret_cast<uint32_t*>(frow + row * row_stride);
#pragma unroll
            for (int u = 0; u < NAR_U; ++u) {
                acc[u] = pk_min(acc[u], F_INF2);
                const int j = j0 + u * 64 + lane;
                if (j < ndw) out[j] = acc[u];
            }
            if (s == 0) break;

            __syncthreads();
            if (active) {
                volatile uint16_t* const b16 = reinterpret_cast<volatile uint16_t*>(lds + NAR_BOFF);
#pragma unroll
                for (int u = 0; u < NAR_U; ++u) {
                    const int j = j0 + u * 64 + lane;
                    lds[NAR_PADW + j] = acc[u];
                    // B[j-1].hi = cell 2j, B[j].lo = cell 2j+1; two aligned 16-bit stores
                    b16[2 * (NAR_PADW + j) - 1] = (uint16_t)(acc[u] & 0xFFFFu);
                    b16[2 * (NAR_PADW + j)] = (uint16_t)(acc[u] >> 16);
                }
            }
            __syncthreads();
        }
        __syncthreads();
    }
}

int cu_count()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
        return 256;
    return n;
}

constexpr size_t LDS_PER_CU = 160 * 1024;

inline size_t wide_lds_bytes(int waves, int cand_buf)
{
    return (size_t)COPIES * wide_copy_bytes(waves) + 16 + (cand_buf + 16) * sizeof(uint32_t);
}

inline int wide_groups_per_cu(int waves, int cand_buf)
{
    int per_cu = (int)(LDS_PER_CU / wide_lds_bytes(waves, cand_buf));
    if (per_cu > 32 / waves) per_cu = 32 / waves;
    return per_cu < 1 ? 1 : per_cu;
}

// One launch of a wide kernel for the classes low .. c with the geometry of class
// c; `pruned_rows`: the kernel for pruned rows (the caller has checked its limits).
hipError_t launch_wide_class(const Layout& L_, char* ws, hipStream_t st, int c, int low, int cus,
                             bool pruned_rows)
{
    const int nwc = CLS_WAVES[c];
    const int cand_buf = L_.Kp < CAND_BUF ? L_.Kp : CAND_BUF;
    const size_t lds_bytes = wide_lds_bytes(nwc, cand_buf);
    const bool chunks = nwc < 8;  // see the kernel's pulls
    const void* const kernel =
        !pruned_rows ? reinterpret_cast<const void*>(&k2_minplus_wide)
        : chunks     ? reinterpret_cast<const void*>(&k2_minplus_pruned<true>)
                     : reinterpret_cast<const void*>(&k2_minplus_pruned<false>);
    hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(LDS_PER_CU - 1024));
    if (e != hipSuccess) return e;
    long long grid = (long long)cus * wide_groups_per_cu(nwc, cand_buf);
    if (grid > L_.N) grid = L_.N;
    if (pruned_rows) {
        auto launch = [&](auto kern) {
            hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(nwc * 64), lds_bytes, st,
                               (const StepEntry*)(ws + L_.step_off),
                               (const uint16_t*)(ws + L_.bcum_off),
                               (const int32_t*)(ws + L_.tmeta_off),
                               (const int32_t*)(ws + L_.order_off), (int32_t*)(ws + L_.ctrl_off),
                               (uint16_t*)(ws + L_.frow_off), L_.N, L_.S, L_.Kp, L_.nbs,
                               L_.row_stride, c, low);
        };
        if (chunks)
            launch(&k2_minplus_pruned<true>);
        else
            launch(&k2_minplus_pruned<false>);
    } else
        hipLaunchKernelGGL(k2_minplus_wide, dim3((unsigned)grid), dim3(nwc * 64), lds_bytes, st,
                           (const StepEntry*)(ws + L_.step_off), (const uint16_t*)(ws + L_.bcum_off),
                           (const int32_t*)(ws + L_.tmeta_off), (const int32_t*)(ws + L_.order_off),
                           (int32_t*)(ws + L_.ctrl_off), (uint16_t*)(ws + L_.frow_off),
                           (int32_t*)(ws + L_.ans_off), L_.N, L_.S, L_.Kp, L_.nbs, L_.row_stride, c,
                           low, cand_buf, L_.fixed_form ? 0 : 1);
    return hipGetLastError();
}

}  // namespace

MinplusPlan make_plan(const Layout& L_)
{
    MinplusPlan pl{};
    pl.cus = cu_count();
    pl.top = class_of_budget(L_.t_max);
    pl.top_wide = pl.top == NARROW_CLS ? N_WIDE_CLS - 1 : pl.top;
    // A batch that fills less than half of the chip even with workgroups of twice
    // the wavefronts gets that geometry: every wavefront then has one position of a
    // longest row instead of two, and a solve that is one latency chain (a handful
    // of instances) is about a quarter shorter.  (Not for step rows, whose kernel
    // works by budgets, not positions.)
    if (!L_.step_rows) {
        int boosted = pl.top_wide;
        const int want = 2 * CLS_WAVES[pl.top_wide] < 16 ? 2 * CLS_WAVES[pl.top_wide] : 16;
        while (CLS_WAVES[boosted] < want) ++boosted;
        const int cand_buf = L_.Kp < CAND_BUF ? L_.Kp : CAND_BUF;
        if (2LL * L_.N <= (long long)pl.cus * wide_groups_per_cu(CLS_WAVES[boosted], cand_buf))
            pl.top_wide = boosted;
    }
    // Heads of the class groups (bit c set = class c has a launch of its own).
    // One launch for everything is best until the batch is large and its longest
    // rows need twelve wavefronts or more; then the rows of up to eight chunks get
    // a launch with the eight-wavefront geometry (four workgroups per compute
    // unit), where short rows leave fewer wavefronts idle.  Measured: more heads
    // than that lose to the starts and thinning ends of the extra launches, except
    // on pruned rows, where a wavefront owns its positions (an idle one is not
    // made up for by the others taking more): there the twelve- and the
    // four-wavefront geometries get launches of their own as well.
    unsigned heads = 1u << pl.top_wide;
    constexpr int SECOND_HEAD = 5;  // CLS_WAVES[5] == 8
    static_assert(CLS_WAVES[SECOND_HEAD] == 8, "the second head is the eight-wavefront class");
    static_assert(CLS_WAVES[7] == 12 && CLS_WAVES[3] == 4, "the further heads for pruned rows");
    {
        const int cand_buf = L_.Kp < CAND_BUF ? L_.Kp : CAND_BUF;
        const long long resident =
            (long long)pl.cus * wide_groups_per_cu(CLS_WAVES[pl.top_wide], cand_buf);
        if (CLS_WAVES[pl.top_wide] >= 12 && L_.N >= 16 * resident) {
            heads |= 1u << SECOND_HEAD;
            if (L_.fixed_form) heads |= 1u << 7 | 1u << 3;
        }
    }
    pl.class_map = 0;
    int head = pl.top_wide;
    for (int c = pl.top_wide; c >= 0; --c) {
        if ((heads >> c) & 1u) head = c;
        pl.class_map |= (uint64_t)head << (4 * c);
    }
    return pl;
}

hipError_t launch_minplus(const themis_problem_t& p, const Layout& L_, char* ws, hipStream_t st)
{
    // the kernel for pruned rows stages whole rows and keeps one lane per model
    const bool pruned_rows = L_.fixed_form != 0 && L_.Kp <= CAND_BUF && L_.S <= 64;
    const MinplusPlan pl = make_plan(L_);
    hipError_t e;

    // longest rows first: they take longest, so they should not start last
    if (pl.top == NARROW_CLS) {
        size_t lds_bytes = (size_t)(2 * NAR_BOFF + 4) * sizeof(uint32_t);
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k2_minplus_narrow),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        int grid = L_.N < pl.cus ? L_.N : pl.cus;
        hipLaunchKernelGGL(k2_minplus_narrow, dim3(grid), dim3(NAR_NW * 64), lds_bytes, st,
                           (const StepEntry*)(ws + L_.step_off),
                           (const uint16_t*)(ws + L_.bcum_off), (const int32_t*)(ws + L_.tmeta_off),
                           (const int32_t*)(ws + L_.order_off), (int32_t*)(ws + L_.ctrl_off),
                           (uint16_t*)(ws + L_.frow_off), L_.N, L_.S, L_.Kp, L_.nbs,
                           L_.row_stride);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int c = pl.top_wide; c >= 0; --c) {
        if (head_of_class(c, pl.class_map) != c) continue;  // served by the launch of its head
        int low = c;
        while (low > 0 && head_of_class(low - 1, pl.class_map) == c) --low;
        if (p.prune & THEMIS_PRUNE_STEPS) {
            e = launch_steps_group(L_, ws, st, c, low, pl.cus);
            if (e != hipSuccess) return e;
            continue;
        }
        e = launch_wide_class(L_, ws, st, c, low, pl.cus, pruned_rows);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace themis
