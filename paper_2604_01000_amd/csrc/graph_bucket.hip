// Cut count of a partition over a CSR graph whose label vector is beyond every on-chip cache.
//
// What it computes (EmbedPart paper, Sec. "Partitioning quality metrics"): the number of stored entries
// (u, v) with pid(u) != pid(v), the numerator of the edge-cut ratio |C| / |E|.  Integer arithmetic only:
// the result does not depend on the order in which entries are met.
//
// Why a second path: the plain sweep (graph.hip) gathers pid(v) for every entry.  With 111 M vertices the
// byte copy of the labels is 111 MB, every gather misses the L2 and pulls a whole cache line over the
// fabric for one useful byte, and the sweep runs at the fabric's line rate (~50 G entries/s).  Here the
// entries are first bucketed by the vertex range of v, so that the labels a bucket needs are 256 KB (L2)
// and, in two pieces, 128 KB (LDS):
//   bucket_hist_kernel     entries per bucket (one streaming read of colidx)
//   bucket_scan_kernel     bucket offsets (each bucket starts on a 64-byte block), work items of the last pass
//   bucket_scatter_kernel  streams colidx with its rows' labels (blocks of 128 rows per wave) and
//                          writes one 32-bit record per entry, (v - bucket start) | pid(u) << shift, to
//                          the entry's bucket: a workgroup sorts a tile of 16,384 entries by bucket in LDS and
//                          every bucket's run leaves as a contiguous stream of whole 64-byte blocks, its place
//                          reserved with one integer atomic per bucket and tile
//   bucket_sweep_kernel    a workgroup takes 96 K records of one bucket into registers, walks the bucket's
//                          label slice through LDS 128 KB at a time and compares each record against the
//                          piece that holds its v
// Traffic: colidx twice, the records once out and once in, 4 bytes each: 16 bytes per entry in streams
// instead of one 128-byte line per entry.
#include <algorithm>
#include <atomic>

#include "kernels.h"

namespace ep {

namespace {

constexpr int kBlock = 256;
// Atomics on one cache line queue up behind each other: every bucket's cursor has a 128-byte line of its own.
constexpr int kCursorStride = 16;
constexpr int kAlign = 16;                 // records per 64-byte block: every write to the record buffer is whole blocks
constexpr int kScatterGridMax = 256;       // workgroups of the scatter pass (one per compute unit)
constexpr int kSliceShift = 17;            // label piece held in LDS: 2^17 bytes
constexpr int kSweepBlock = 1024;
constexpr int kSweepPerThread = 96;
constexpr int kChunk = kSweepBlock * kSweepPerThread;   // records per work item of the last pass
static_assert(kSweepPerThread % 4 == 0, "a thread takes its records four at a time");
constexpr int kSweepGrid = 1024;

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(kBlock) void bucket_clear_kernel(int nb, unsigned long long *__restrict__ hist,
                                                               unsigned long long *__restrict__ dropped) {
    const int t = blockIdx.x * kBlock + threadIdx.x;
    if (t < nb) hist[t] = 0;
    if (t == 0) *dropped = 0;
}

__global__ __launch_bounds__(kBlock) void bucket_hist_kernel(int64_t n, int64_t nnz, int shift, int nb,
                                                              const int32_t *__restrict__ colidx,
                                                              unsigned long long *__restrict__ hist) {
    __shared__ unsigned int h[kBucketsMax];
    for (int b = threadIdx.x; b < nb; b += kBlock) h[b] = 0;
    __syncthreads();
    const int64_t quads = nnz / 4, stride = (int64_t)gridDim.x * kBlock;
    for (int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x; q < quads; q += stride) {
        const i32x4 c = *reinterpret_cast<const i32x4 *>(colidx + 4 * q);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (c[t] >= 0 && c[t] < n) atomicAdd(&h[c[t] >> shift], 1u);
    }
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(nnz - 4 * quads)) {   // the last nnz % 4 entries
        const int32_t v = colidx[4 * quads + threadIdx.x];
        if (v >= 0 && v < n) atomicAdd(&h[v >> shift], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < nb; b += kBlock)
        if (h[b]) atomicAdd(&hist[b], (unsigned long long)h[b]);   // integers: the order does not matter
}

// base[b] = start of bucket b in the record buffer, cursor[b] = base[b], item_prefix[b] = number of
// kChunk-record work items before bucket b.  A bucket has room for its entries rounded up to whole blocks plus
// one block per workgroup of the scatter pass (the padded last flush of each).  One wave: lane l takes buckets
// kPerLaneBuckets l .. + kPerLaneBuckets - 1, the lanes' totals are scanned across the wave (one thread walking all
// buckets took 66 us of dependent memory round trips).
constexpr int kPerLaneBuckets = kBucketsMax / 64;
static_assert(kPerLaneBuckets * 64 == kBucketsMax, "the buckets divide over the lanes of one wave");
__global__ __launch_bounds__(64) void bucket_scan_kernel(int nb, int scatter_grid, const unsigned long long *__restrict__ hist,
                                                         int64_t *__restrict__ base, unsigned long long *__restrict__ cursor,
                                                         int64_t *__restrict__ item_prefix) {
    if (blockIdx.x != 0) return;
    const int lane = threadIdx.x, b0 = lane * kPerLaneBuckets;
    int64_t room[kPerLaneBuckets], mine_room = 0, mine_items = 0;
#pragma unroll
    for (int i = 0; i < kPerLaneBuckets; ++i) {
        const int b = b0 + i;
        const int64_t entries = b < nb ? (int64_t)hist[b] : 0;
        room[i] = b < nb ? (entries + kAlign - 1) / kAlign * kAlign + (int64_t)kAlign * scatter_grid : 0;
        mine_room += room[i];
        mine_items += (room[i] + kChunk - 1) / kChunk;
    }
    int64_t at = mine_room, items = mine_items;   // inclusive over the lanes, then made exclusive
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t up_room = __shfl_up(at, off, 64), up_items = __shfl_up(items, off, 64);
        if (lane >= off) {
            at += up_room;
            items += up_items;
        }
    }
    at -= mine_room;
    items -= mine_items;
#pragma unroll
    for (int i = 0; i < kPerLaneBuckets; ++i) {
        const int b = b0 + i;
        if (b <= nb) {   // b == nb: the totals
            base[b] = at;
            item_prefix[b] = items;
        }
        if (b < nb) cursor[b * kCursorStride] = (unsigned long long)at;
        at += room[i];
        items += (room[i] + kChunk - 1) / kChunk;
    }
    if (lane == 63 && nb == kBucketsMax) {   // the totals when every lane's buckets are real ones
        base[nb] = at;
        item_prefix[nb] = items;
    }
}

// A workgroup gathers a tile of up to kTile entries, sorts it by bucket in LDS and writes every bucket's run
// to the bucket's next free slots, reserved with one integer atomic per bucket and tile.
//   phase A  every wave streams its rows' entries (blocks of 128 rows, 256 entries per step, kTileSteps steps, the
//            next step's entries and the next block's offsets and labels in flight); an entry finds its row through
//            marks at the rows' first entries and a running maximum, takes its rank inside its bucket from an
//            LDS counter and stays in registers as (record, bucket | rank)
//   phase B  the counters are scanned (start of every bucket's run inside the tile) and thread b reserves the
//            run of bucket b in the record buffer
//   phase C  the records go to their sorted place in LDS, then every run leaves as one contiguous stream
constexpr int kScatterBlock = 1024;
constexpr int kScatterWaves = kScatterBlock / 64;
constexpr int kWindowRows = 128;   // rows per block of a wave: two per lane (a new block costs two memory latencies)
constexpr int kTileSteps = 4;
constexpr int kTile = kScatterWaves * kTileSteps * 256;
constexpr int kSpareWords = 320;   // > kScatterWaves * kTileSteps * 4: where records that count for nothing are put

template <typename RowT>
__global__ __launch_bounds__(kScatterBlock) void bucket_scatter_kernel(int64_t n, int64_t nnz, int shift, int nb,
                                                                        const RowT *__restrict__ rowptr,
                                                                        const int32_t *__restrict__ colidx,
                                                                        const uint8_t *__restrict__ label8,
                                                                        const int64_t *__restrict__ base,
                                                                        unsigned long long *__restrict__ cursor,
                                                                        uint32_t *__restrict__ records,
                                                                        unsigned long long *__restrict__ dropped) {
    static_assert(kScatterWaves == 16, "a wave's offset in the tile is summed over one row of 16 lanes");
    static_assert(kBucketsMax + 64 <= kScatterBlock, "one thread per bucket in the scan of a tile");
    __shared__ int32_t tile_cnt[kBucketsMax + 64];   // entries of the tile per bucket (+ one word per lane for entries
                                                     // that count for nothing: their rank is asked for all the same)
    __shared__ int32_t run_start[1024];              // start of every bucket's run in `sorted` (any 10-bit bucket number may
                                                     // be looked up; only those below nb hold something)
    __shared__ i32x4 run_meta[kBucketsMax];          // per bucket: run start, run length, records that leave with this
                                                     // tile, records that waited
    __shared__ int64_t run_dest[kBucketsMax];        // its place in the record buffer (-1: no room)
    __shared__ __attribute__((aligned(16))) int32_t mark_lds[kScatterWaves][256];   // per step: row number + 1 at a row's first entry
    __shared__ int32_t au_lds[kScatterWaves][kWindowRows + 1];   // [0]: for places before the block's first entry
    __shared__ int32_t wave_total[kScatterWaves];
    __shared__ int32_t any_work;
    // Records of earlier tiles that did not fill a whole 64-byte block of their bucket wait here for the next
    // tile, so that every write to the record buffer is a run of whole blocks at a block-aligned place (a
    // partial block costs the memory a read-modify-write).
    extern __shared__ __attribute__((aligned(16))) uint32_t scatter_lds[];
    uint32_t *sorted = scatter_lds;           // kTile records, sorted by bucket
    uint32_t *resid = scatter_lds + kTile + kSpareWords;   // nb * (kAlign - 1) records (between the two: the spare words)
    __shared__ int32_t resid_cnt[kBucketsMax];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int32_t *mk = mark_lds[wave];
    int32_t *aus = au_lds[wave];
    const int lane_before4 = ((lane + 63) & 63) << 2;   // byte address of lane - 1 for the lane exchange (lane 0: unused)
    const uint32_t n_ids = (uint32_t)min(n, (int64_t)1 << 31);          // a column c is a vertex iff (uint32_t)c < n_ids
    const uint32_t scrap_v = (uint32_t)(kBucketsMax + lane) << shift;   // "vertex" of the lane's own spare counter
    static_assert(kBucketsMax + 64 <= 1024, "bucket numbers, the spare ones included, take 10 bits of `where`");
    const int64_t row_blocks = (n + kWindowRows - 1) / kWindowRows;
    const int64_t rb_stride = (int64_t)gridDim.x * kScatterWaves;
    for (int b = threadIdx.x; b < kBucketsMax + 64; b += kScatterBlock) {
        tile_cnt[b] = 0;
        if (b < kBucketsMax) resid_cnt[b] = 0;
        else run_start[b] = kTile;   // the spare buckets: never written again (phase B writes below nb <= kBucketsMax)
    }
    if (threadIdx.x == 0) any_work = 0;
    __syncthreads();

    // this wave's position in its stream of entries
    int64_t rb = (int64_t)blockIdx.x * kScatterWaves + wave - rb_stride;   // current row block (none yet)
    int64_t p0 = 0, e_begin = 0, e_end = 0;   // next 256-entry step of the block, the block's entry range
    i32x4 ahead = {0, 0, 0, 0};               // this lane's four entries of the step at p0, loaded one step early
    unsigned long long lost = 0;

    // Every load of the stream is unconditional and branch-free, so that the compiler can count the accesses in
    // flight exactly: a wait for the entries loaded one step ago then leaves the step just issued in flight.  (Behind
    // a load under a branch every later wait is for all outstanding accesses, and the read-ahead is waited for as
    // soon as it is issued.)  The 256 entries of the step at p come through a buffer descriptor that ends at the
    // block's last entry: lanes past it get zeros, which no test below looks at (such an entry is not live).
    auto uniform64 = [](int64_t v) -> int64_t {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    auto load4 = [&](int64_t pstep) {   // pstep: first entry of the step, the same in every lane, a multiple of 4
        const int64_t ps = uniform64(pstep), pe = uniform64(min(e_end, nnz));
        const int64_t left = pe - ps;
        const int bytes = left <= 0 ? 0 : (int)(min(left, (int64_t)256) * 4);
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int32_t *>(colidx + (left <= 0 ? 0 : ps)), 0, bytes, 0x00020000);
        return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, 16 * lane, 0, 0));
    };
    // The offsets and labels of the wave's next row block are fetched one block ahead, into registers.
    constexpr int kPerLane = kWindowRows / 64;
    int64_t nrp[kPerLane], nrp_end = 0;
    int32_t nau[kPerLane];
    auto fetch_block = [&](int64_t b) {   // unconditional: rows past the graph read the last offset / a valid label
        const int64_t r0 = min(b, row_blocks) * kWindowRows;
#pragma unroll
        for (int q = 0; q < kPerLane; ++q) {
            nrp[q] = (int64_t)rowptr[min(r0 + 64 * q + lane, n)];
            nau[q] = (int32_t)label8[min(r0 + 64 * q + lane, n - 1)];
        }
        nrp_end = (int64_t)rowptr[min(r0 + kWindowRows, n)];
    };
    fetch_block(rb + rb_stride);
    const int64_t my_limit = (int)threadIdx.x < nb ? base[threadIdx.x + 1] : 0;   // end of the bucket thread t reserves in
    // The current block: the first entry of this lane's rows (row 64 q + lane of the block), and the number + 1 of
    // the last row that starts before the step at p0 (0: none yet).
    int64_t crp[kPerLane];
    uint32_t carry = 0;
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) crp[q] = 0;
    // the next row block of this wave that has entries; false when the wave has none left
    auto next_block = [&]() -> bool {
        for (;;) {
            rb += rb_stride;
            if (rb >= row_blocks) {
                p0 = e_begin = e_end = 0;
                return false;
            }
            const int64_t r0 = rb * kWindowRows;
            wave_fence();   // the labels of the previous block are no longer read
#pragma unroll
            for (int q = 0; q < kPerLane; ++q) {
                crp[q] = min(max(nrp[q], (int64_t)0), nnz);
                aus[1 + 64 * q + lane] = r0 + 64 * q + lane < n ? nau[q] : 255;
            }
            if (lane == 0) aus[0] = 255;
            const int64_t block_end = min(max(nrp_end, (int64_t)0), nnz);
            // (the old values are used up before the new loads are issued: loaded into other registers first, they
            // would have to be copied, and a copy waits for its load)
            __builtin_amdgcn_sched_barrier(0);
            fetch_block(rb + rb_stride);
            wave_fence();
            e_begin = uniform64(crp[0]);   // lane 0 holds the block's first row
            e_end = uniform64(block_end);
            p0 = e_begin & ~(int64_t)3;
            carry = 0;
            if (e_end > e_begin) {
                ahead = load4(p0);
                return true;
            }
        }
    };

    for (;;) {
        // ---- phase A ----
        uint32_t rec[kTileSteps * 4], where[kTileSteps * 4];   // where = 4 bucket | rank << 12; bucket >= kBucketsMax: no entry
        bool worked = false;
#pragma unroll
        for (int st = 0; st < kTileSteps; ++st) {
            bool have = p0 < e_end;
            if (!have) have = next_block();
#pragma unroll
            for (int t = 0; t < 4; ++t) where[4 * st + t] = (uint32_t)kBucketsMax << 2;   // a spare bucket, rank 0
            if (have) {   // uniform over the wave
                worked = true;
                const i32x4 c = ahead;
                ahead = load4(p0 + 256);   // the next step of this block, in flight while this one is ranked
                // The row of every entry without a search: rows that start inside the step leave their number + 1
                // at their first entry's place (of several rows at one place, all but the last are empty: the
                // largest number wins), and a running maximum over the step's 256 places, carried on from the
                // steps before, is the number + 1 of the last row that starts at or before a place.
                wave_fence();   // the previous step's marks have been read
                *reinterpret_cast<i32x4 *>(&mk[4 * lane]) = i32x4{0, 0, 0, 0};
                wave_fence();
#pragma unroll
                for (int q = 0; q < kPerLane; ++q) {
                    const int64_t s = crp[q] - p0;
                    if (s >= 0 && s < 256) atomicMax(&mk[(int)s], 64 * q + lane + 1);   // integer, LDS
                }
                wave_fence();
                const i32x4 m = *reinterpret_cast<const i32x4 *>(&mk[4 * lane]);
                uint32_t upto[4];   // running maximum inside the lane's four places
                upto[0] = (uint32_t)m[0];
#pragma unroll
                for (int t = 1; t < 4; ++t) upto[t] = max(upto[t - 1], (uint32_t)m[t]);
                const uint32_t incl = wave_inclusive_max(upto[3]);
                uint32_t before = (uint32_t)__builtin_amdgcn_ds_bpermute(lane_before4, (int)incl);   // the lanes before this one
                before = max(lane == 0 ? 0u : before, carry);
                carry = max(carry, (uint32_t)__builtin_amdgcn_readlane((int)incl, 63));
                // Which of the lane's places 4 lane + t hold entries of the block: lo <= place < hi, wave-uniform.
                const int lo = (int)min(max(e_begin - p0, (int64_t)0), (int64_t)256);
                const int hi = (int)min(max(e_end - p0, (int64_t)0), (int64_t)256);
                const uint32_t span = (uint32_t)max(hi - lo, 0);
                const int first_place = 4 * lane - lo;
                uint32_t lu[4], vv[4];   // vv: the column, or the lane's stand-in past all vertices for an entry that counts for nothing
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    lu[t] = (uint32_t)aus[max(before, upto[t])];   // row number + 1 <= kWindowRows; 0 only before the block's first entry
                    const bool ok = (uint32_t)(first_place + t) < span && (uint32_t)c[t] < n_ids;
                    vv[t] = ok ? (uint32_t)c[t] : scrap_v;
                }
                int rank[4];   // all four asked for at once (integer, LDS: the order inside a run is free)
#pragma unroll
                for (int t = 0; t < 4; ++t) rank[t] = atomicAdd(&tile_cnt[vv[t] >> shift], 1);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    rec[4 * st + t] = (vv[t] & ((1u << shift) - 1u)) | (lu[t] << shift);
                    where[4 * st + t] = ((vv[t] >> shift) << 2) | ((uint32_t)rank[t] << 12);
                }
                p0 += 256;
            }
        }
        if (worked && lane == 0) any_work = 1;
        __syncthreads();
        if (!any_work) break;   // uniform over the workgroup: no wave had a step
        // ---- phase B: exclusive scan of tile_cnt[0 .. nb), one counter per thread; reservations ----
        // The reservation of thread t's bucket is one integer atomic per bucket and tile; all of a tile's are in
        // flight together, and their answers (a round trip to the memory side) are looked at only after the
        // records have been sorted in LDS: the barriers in between wait for LDS traffic alone.
        const int t = threadIdx.x;
        unsigned long long pos = 0;
        int my_out = 0;
        {
            const int cnt = t < nb ? tile_cnt[t] : 0;
            const int incl = wave_inclusive_add(cnt);
            if (lane == 63) wave_total[wave] = incl;
            const int waited = t < nb ? resid_cnt[t] : 0;
            my_out = (waited + cnt) & ~(kAlign - 1);   // whole blocks of waiting + new records
            if (my_out > 0) pos = atomicAdd(&cursor[t * kCursorStride], (unsigned long long)my_out);
            __syncthreads();
            // every thread has read its counter and the flag: both start the next tile at zero (the barrier below
            // orders this before any wave's next phase A)
            if (t < kBucketsMax + 64) tile_cnt[t] = 0;
            if (t == 0) any_work = 0;
            int before = (lane & 15) < wave ? wave_total[lane & 15] : 0;   // summed over the 16 lanes of a row
            before += __builtin_amdgcn_update_dpp(0, before, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
            before += __builtin_amdgcn_update_dpp(0, before, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
            before += __builtin_amdgcn_update_dpp(0, before, 0x141, 0xF, 0xF, true);   // row_half_mirror
            before += __builtin_amdgcn_update_dpp(0, before, 0x140, 0xF, 0xF, true);   // row_mirror
            if (t < nb) {
                run_start[t] = before + incl - cnt;
                run_meta[t] = i32x4{before + incl - cnt, cnt, my_out, waited};
            }
        }
        __syncthreads();
        // ---- phase C ----
        {   // All look-ups of a thread's 16 records at once, then all writes.  A record that counts for nothing was
            // ranked on a spare counter (at most kTileSteps * 4 per thread and tile, one counter per lane number): the
            // spare buckets' runs all start at the spare words behind the tile, kScatterWaves * kTileSteps * 4 + 1 of them.
            uint32_t at[kTileSteps * 4];
#pragma unroll
            for (int i = 0; i < kTileSteps * 4; ++i)
                at[i] = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(run_start) + (where[i] & 0xFFCu));
#pragma unroll
            for (int i = 0; i < kTileSteps * 4; ++i) sorted[at[i] + (where[i] >> 12)] = rec[i];
        }
        {   // (straight-line code: the one wait for the answer sits on every path, and the write-out below, whose
            // stores must stay in flight from turn to turn, is not made to wait for it again)
            const bool fits = (int64_t)pos + my_out <= my_limit;   // never write past a bucket
            lost += (my_out > 0 && !fits) ? (unsigned long long)my_out : 0ull;
            run_dest[min(t, kBucketsMax - 1)] = (my_out > 0 && fits) ? (int64_t)pos : (int64_t)-1;
        }
        __syncthreads();
        // Four buckets per wave and turn, 16 lanes each: a run of this size is one or two 64-byte blocks, and a
        // whole wave per bucket spent most of its instructions on lanes with nothing to write.
        for (int b0 = 4 * wave; b0 < nb; b0 += 4 * kScatterWaves) {
            const int b = b0 + (lane >> 4), li = lane & 15;
            const bool valid = b < nb;
            const int bc = min(b, nb - 1);
            // the bucket's stream = the records that waited, then this tile's run; `out` of them leave
            const i32x4 meta = run_meta[bc];
            const int64_t dest = run_dest[bc];
            const int first = meta[0], cnt = meta[1], out = meta[2], waiting = meta[3];
            uint32_t *wait_b = resid + bc * (kAlign - 1);
            const int leaving = valid && dest >= 0 ? out : 0;   // a multiple of kAlign
            // (fewer than kAlign records wait, so only a lane's first record can be one of them)
            if (li < leaving) records[dest + li] = li < waiting ? wait_b[li] : sorted[first + li - waiting];
            for (int i = li + kAlign; i < leaving; i += kAlign) records[dest + i] = sorted[first + i - waiting];
            // What stays: with nothing gone the run joins the waiting records, else (out >= kAlign > waiting) the
            // tail of the run waits.
            const int keep = waiting + cnt - out;   // < kAlign
            const int moved = out == 0 ? cnt : keep;
            const int from = first + li + (out == 0 ? 0 : out - waiting), to = li + (out == 0 ? waiting : 0);
            wave_fence();
            if (valid && li < moved) wait_b[to] = sorted[from];
            if (valid && li == 0) resid_cnt[b] = keep;
        }
        // No barrier here: a wave that is done writing goes on to gather its part of the next tile.  What the next
        // tile shares with this write-out is touched only behind its first barrier (`sorted` and the run tables
        // two and three barriers on, resid_cnt of another wave's buckets in phase B), which every wave reaches
        // after its own write-out; the waiting records of a bucket stay with the same wave from tile to tile.
    }
    // what still waits leaves as one block per bucket, filled up with records that count for nothing
    for (int b = wave; b < nb; b += kScatterWaves) {
        const int waiting = resid_cnt[b];
        if (waiting == 0) continue;   // uniform over the wave
        unsigned long long pos = 0;
        if (lane == 0) pos = atomicAdd(&cursor[b * kCursorStride], (unsigned long long)kAlign);
        pos = __shfl(pos, 0, 64);
        if ((int64_t)pos + kAlign <= base[b + 1]) {
            if (lane < kAlign) records[pos + lane] = lane < waiting ? resid[b * (kAlign - 1) + lane] : (255u << shift);
        } else if (lane == 0) {
            lost += (unsigned long long)waiting;
        }
    }
    if (lost) atomicAdd(dropped, lost);
}

// Work item w = kChunk consecutive records of one bucket.  The records stay in registers while the bucket's
// label slice passes through LDS in pieces of 2^kSliceShift bytes.
__global__ __launch_bounds__(kSweepBlock) void bucket_sweep_kernel(int64_t n, int shift, int nb,
                                                                    const uint8_t *__restrict__ label8,
                                                                    const unsigned long long *__restrict__ cursor,
                                                                    const int64_t *__restrict__ base,
                                                                    const int64_t *__restrict__ item_prefix,
                                                                    const uint32_t *__restrict__ records,
                                                                    unsigned long long *__restrict__ out) {
    extern __shared__ __attribute__((aligned(16))) unsigned char slice[];   // 2^kSliceShift label bytes
    __shared__ int64_t prefix_lds[kBucketsMax + 1];
    __shared__ unsigned long long red[kSweepBlock / 64];
    for (int b = threadIdx.x; b <= nb; b += kSweepBlock) prefix_lds[b] = item_prefix[b];
    __syncthreads();
    const int64_t items = prefix_lds[nb];
    const uint32_t vmask = (1u << shift) - 1u;
    const int pieces = 1 << (shift - kSliceShift);
    unsigned long long cut = 0;
    for (int64_t w = blockIdx.x; w < items; w += gridDim.x) {
        int b = 0;   // the bucket of item w: the last b with item_prefix[b] <= w
        for (int step = kBucketsMax / 2; step > 0; step >>= 1)
            if (b + step < nb && prefix_lds[b + step] <= w) b += step;
        const int64_t first = base[b] + (w - prefix_lds[b]) * kChunk;
        const int64_t end = min((int64_t)cursor[b * kCursorStride], base[b + 1]);   // what the scatter pass wrote
        // The item's records, 16 bytes per lane and load, all loads of a thread in flight at once, through a buffer
        // descriptor that ends at the bucket's last record: what lies past it reads as zero and is replaced below
        // (only the last item of a bucket has such places) by a record that counts for nothing.
        uint32_t rec[kSweepPerThread];
        const int have = (int)min(max(end - first, (int64_t)0), (int64_t)kChunk);
#pragma unroll
        for (int q = 0; q < kSweepPerThread / 4; ++q) {   // (a descriptor per load: scalar work, and one offset register for all)
            const int here = min(max(have - q * 4 * kSweepBlock, 0), 4 * kSweepBlock);   // records of this load's 16 KB
            __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint32_t *>(records + (here ? first + (int64_t)q * 4 * kSweepBlock : 0)), 0, here * 4, 0x00020000);
            const u32x4 four = __builtin_amdgcn_raw_buffer_load_b128(rsrc, 16 * (int)threadIdx.x, 0, 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) rec[4 * q + j] = four[j];
        }
        if (have < kChunk) {   // uniform over the workgroup
#pragma unroll
            for (int q = 0; q < kSweepPerThread; ++q) {
                const int at = 4 * ((int)threadIdx.x + (q / 4) * kSweepBlock) + (q % 4);
                rec[q] = at < have ? rec[q] : (255u << shift);   // pid(u) = 255
            }
        }
        const int64_t v0 = (int64_t)b << shift;
        for (int piece = 0; piece < pieces; ++piece) {
            __syncthreads();   // the previous piece is no longer read
            const int64_t p0 = v0 + ((int64_t)piece << kSliceShift);
            {   // the piece's label bytes, two 16-byte loads of a thread in flight at a time, through a buffer descriptor
                // that ends at the word holding the last vertex (the range check works on whole words: a word cut
                // short would read as zero; the label array is followed by 256-byte aligned arrays of the same
                // workspace, and no record names a vertex past the last; words beyond the end read as zeros)
                constexpr int kLoads = (1 << kSliceShift) / 16 / kSweepBlock;
                static_assert(kLoads * kSweepBlock * 16 == (1 << kSliceShift), "whole loads per thread");
                const int64_t left = n - p0;
                const int bytes = left <= 0 ? 0 : (int)min((left + 3) & ~(int64_t)3, (int64_t)1 << kSliceShift);
                __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<uint8_t *>(label8 + (left <= 0 ? 0 : p0)), 0, bytes, 0x00020000);
                constexpr int kBatch = 2;   // (more at once do not fit beside the 96 records of a thread)
                static_assert(kLoads % kBatch == 0, "whole batches");
#pragma unroll
                for (int q0 = 0; q0 < kLoads; q0 += kBatch) {
                    u32x4 val[kBatch];
#pragma unroll
                    for (int q = 0; q < kBatch; ++q)
                        val[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, 16 * (int)(threadIdx.x + (q0 + q) * kSweepBlock), 0, 0);
#pragma unroll
                    for (int q = 0; q < kBatch; ++q)
                        reinterpret_cast<u32x4 *>(slice)[threadIdx.x + (q0 + q) * kSweepBlock] = val[q];
                }
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < kSweepPerThread; ++q) {
                asm volatile("" : "+v"(rec[q]));   // keeps the fields from being split out of all 64 records ahead of the loop (spills)
                const uint32_t vl = rec[q] & vmask;
                if ((int)(vl >> kSliceShift) == piece) {
                    const uint32_t lu = rec[q] >> shift, lv = slice[vl & ((1u << kSliceShift) - 1u)];
                    cut += (lu != 255u && lv != 255u && lu != lv) ? 1u : 0u;
                }
            }
        }
    }
    for (int off = 32; off > 0; off >>= 1) cut += __shfl_down(cut, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = cut;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long total = 0;
        for (int w = 0; w < kSweepBlock / 64; ++w) total += red[w];
        if (total) atomicAdd(out, total);
    }
}

// Dynamic LDS beyond 64 KB has to be allowed per kernel: done once per kernel and device (`done`: one word per
// kernel of this file, one bit per device).
int set_big_lds(const void *kern, std::atomic<uint64_t> &done, int bytes) {
    if (bytes + 16 * 1024 <= 64 * 1024) return EP_OK;   // room for the static LDS beside it
    int dev = 0;
    EP_HIP_TRY(hipGetDevice(&dev));
    const uint64_t bit = 1ull << (dev & 63);
    if (!(done.load(std::memory_order_acquire) & bit)) {
        EP_HIP_TRY(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
        done.fetch_or(bit, std::memory_order_release);
    }
    return EP_OK;
}
std::atomic<uint64_t> g_sweep_lds{0}, g_scatter_lds64{0}, g_scatter_lds32{0};

}  // namespace

BucketPlan bucket_plan(int64_t n, int64_t nnz, int32_t k) {
    BucketPlan pl{0, 0};
    // Worth it only when the byte labels are far beyond the L2 caches and the rows are not nearly empty.
    if (k > 255 || n < kBucketMinVertices || nnz < 4 * n) return pl;
    pl.shift = 18;   // 256 KB of labels per bucket: two LDS pieces in the last pass
    while (ceil_div(n, (int64_t)1 << pl.shift) > kBucketsMax) ++pl.shift;
    pl.nb = (int)ceil_div(n, (int64_t)1 << pl.shift);
    return pl;
}

int launch_cut_bucketed(int64_t n, int64_t nnz, const BucketPlan &pl, const void *rowptr, bool i64,
                        const int32_t *colidx, const GraphWs &w, unsigned long long *cut, hipStream_t s) {
    auto hist = reinterpret_cast<unsigned long long *>(w.bucket_hist);
    auto cursor = reinterpret_cast<unsigned long long *>(w.bucket_cursor);
    auto dropped = reinterpret_cast<unsigned long long *>(w.bucket_dropped);
    ProfScope prof(EP_PROF_EDGE_SWEEP, s);   // the four kernels together are this path's sweep
    bucket_clear_kernel<<<(unsigned)ceil_div(pl.nb, kBlock), kBlock, 0, s>>>(pl.nb, hist, dropped);
    EP_LAUNCH_CHECK();
    const unsigned hgrid = (unsigned)std::min<int64_t>(ceil_div(nnz / 4 + 1, kBlock * 8), 256 * 8);
    bucket_hist_kernel<<<hgrid, kBlock, 0, s>>>(n, nnz, pl.shift, pl.nb, colidx, hist);
    EP_LAUNCH_CHECK();
    const int64_t row_blocks = ceil_div(n, kWindowRows);
    const unsigned sgrid = (unsigned)std::min<int64_t>(ceil_div(row_blocks, kScatterWaves), kScatterGridMax);
    bucket_scan_kernel<<<1, 64, 0, s>>>(pl.nb, (int)sgrid, hist, w.bucket_base, cursor, w.bucket_items);
    EP_LAUNCH_CHECK();
    {
        // the tile (64 KB), the spare words and the waiting records (<= 30 KB) in dynamic LDS
        const int scatter_bytes = (kTile + kSpareWords + pl.nb * (kAlign - 1)) * 4;
        constexpr int kScatterLdsMax = (kTile + kSpareWords + kBucketsMax * (kAlign - 1)) * 4;
        if (i64) {
            int rc = set_big_lds(reinterpret_cast<const void *>(bucket_scatter_kernel<int64_t>), g_scatter_lds64, kScatterLdsMax);
            if (rc != EP_OK) return rc;
            bucket_scatter_kernel<int64_t><<<sgrid, kScatterBlock, scatter_bytes, s>>>(
                n, nnz, pl.shift, pl.nb, static_cast<const int64_t *>(rowptr), colidx, w.label8, w.bucket_base, cursor,
                w.bucket_records, dropped);
        } else {
            int rc = set_big_lds(reinterpret_cast<const void *>(bucket_scatter_kernel<int32_t>), g_scatter_lds32, kScatterLdsMax);
            if (rc != EP_OK) return rc;
            bucket_scatter_kernel<int32_t><<<sgrid, kScatterBlock, scatter_bytes, s>>>(
                n, nnz, pl.shift, pl.nb, static_cast<const int32_t *>(rowptr), colidx, w.label8, w.bucket_base, cursor,
                w.bucket_records, dropped);
        }
        EP_LAUNCH_CHECK();
        const int rc = set_big_lds(reinterpret_cast<const void *>(bucket_sweep_kernel), g_sweep_lds, 1 << kSliceShift);
        if (rc != EP_OK) return rc;
        bucket_sweep_kernel<<<kSweepGrid, kSweepBlock, 1 << kSliceShift, s>>>(n, pl.shift, pl.nb, w.label8, cursor,
                                                                              w.bucket_base, w.bucket_items,
                                                                              w.bucket_records, cut);
        EP_LAUNCH_CHECK();
    }
    return EP_OK;
}

size_t bucket_record_slots(int64_t nnz, const BucketPlan &pl) {
    return (size_t)nnz + (size_t)pl.nb * kAlign * (kScatterGridMax + 1) + kAlign;
}

}  // namespace ep
