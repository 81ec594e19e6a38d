// Long rows by column windows: a tiling of the reduction dimension for rows
// whose gathered operands would otherwise stream from HBM (in the spirit of the
// paper's Section 7.2, where tiling parameters are tuned apart from the
// synchronisation granularity).
//
// A row of many thousand stored entries gathers as many rows of B from all
// over the matrix; when B is far larger than an L2 (4 MB per die) every one of
// them comes from HBM, and a workload whose long rows hold most of the entries
// runs at the random-gather rate of HBM however the reduction is organised.
// Rows of B are reused *between* long rows, though: with 5,000 rows of 11,000
// entries over K = 500,000 columns every row of B is wanted about 110 times.
// This file cuts the columns into windows of about 2 MB of B and takes the work
// of the long rows window by window: the item (window w, long row r) is the run
// of r's entries whose column lies in w (columns are sorted inside a row, so it
// is one contiguous run).  Die w % 8 takes window w, and its workgroups walk the
// items window-major, so at any moment a die gathers from one or two windows,
// which its L2 holds.  Every item adds its partial row into C with atomic adds
// (the rows were zeroed before), which is what the "Atomics" output strategy of
// Section 6.2 does for a row that several groups produce.
//
// The row-split kernel then produces all other rows and leaves the long ones
// alone (`RowSkip`).  Everything is decided on the device, so the call stays
// asynchronous: the list of long rows and the window pointers live in a
// workspace of device memory that the caller hands in (sized by
// panel_workspace_bytes for a list of `cap` rows).  When the matrix has more long
// rows than the list holds, this path does nothing and the row-split kernel
// takes every row.
#include "sgap_common.hpp"
#include "sgap_lane_ops.hpp"
#include "sgap_row_split_impl.hpp"
#include "sgap_uniform.hpp"

namespace sgap {

constexpr int kPanelMaxWindows = 511;  // column windows at most
constexpr int kPanelDies = 8;          // dies of the chip (the window count is made a multiple of it)
constexpr int kRankMaxRows = 8192;     // lists up to this length are sorted by row length (their lengths fit in LDS)
constexpr int kSearchLanes = 4;        // lanes that look for one window pointer together

// The workspace: a header, the list of long rows, the same list sorted by length, the rows' lengths, and the
// window pointers.
struct PanelHeader {
    uint32_t count;     // long rows found (may exceed the list's capacity: then the path is off)
    uint32_t next[15];  // per die: the next item nobody has taken yet
    uint32_t pad[48];
};
struct PanelView {
    PanelHeader* head;
    int32_t* rows;   // [cap]
    int32_t* order;  // [cap] the long rows from the longest to the shortest: order[q] indexes rows[]
    int32_t* len;    // [cap] stored entries of rows[i]
    int32_t* ptr;    // [cap * (windows + 1)]: ptr[i * (windows + 1) + w] = first entry of long row i with column >= w * window_rows
    uint32_t cap;    // rows the list holds
};

int64_t panel_workspace_bytes(int64_t cap, int windows)
{
    const int64_t ints = 3 * cap + cap * (int64_t)(windows + 1);
    return (int64_t)sizeof(PanelHeader) + (ints * 4 + 255) / 256 * 256;
}

namespace {

PanelView panel_view(void* workspace, int64_t cap, int windows)
{
    PanelView v;
    char* base = static_cast<char*>(workspace);
    v.head = reinterpret_cast<PanelHeader*>(base);
    v.rows = reinterpret_cast<int32_t*>(base + sizeof(PanelHeader));
    v.order = v.rows + cap;
    v.len = v.order + cap;
    v.ptr = v.len + cap;
    v.cap = (uint32_t)cap;
    (void)windows;
    return v;
}

}  // namespace

__global__ void panel_reset_kernel(PanelView scr)
{
    if (blockIdx.x == 0 && threadIdx.x < 16) (&scr.head->count)[threadIdx.x] = 0;  // count and next[]
}

// A workgroup looks at kFindRows rows per thread and adds to the list's counter once: a returning atomic on one
// address takes about 0.1 us (they are carried out one after another, beyond the dies' L2s), and a matrix may have
// thousands of long rows (skewed, 5,000 of them: 44 us with one update per wavefront that found a row).
constexpr int kFindRows = 8;
__global__ __launch_bounds__(kBlock) void panel_find_rows_kernel(SpmmArgs a, PanelView scr, int32_t min_len)
{
    __shared__ uint32_t s_wave[kWavesPerBlock];
    __shared__ uint32_t s_base;
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int64_t row0 = (int64_t)blockIdx.x * (kBlock * kFindRows) + threadIdx.x;
    uint32_t mine = 0;  // bit j: row row0 + j * kBlock is long
    int32_t len[kFindRows];
#pragma unroll
    for (int j = 0; j < kFindRows; ++j) {
        const int64_t row = row0 + (int64_t)j * kBlock;
        len[j] = row < a.M ? a.rowptr[row + 1] - a.rowptr[row] : 0;
        if (row < a.M && len[j] >= min_len) mine |= 1u << j;
    }
    const uint32_t cnt = (uint32_t)__popc(mine);
    uint32_t incl = cnt;  // long rows of this and the lower lanes of the wavefront
#pragma unroll
    for (int d = 1; d < kWave; d *= 2) {
        const uint32_t t = (uint32_t)__shfl_up((int)incl, d, kWave);
        if (lane >= d) incl += t;
    }
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) {
            const uint32_t c = s_wave[w];
            s_wave[w] = total;
            total += c;
        }
        s_base = total ? atomicAdd(&scr.head->count, total) : 0u;
    }
    __syncthreads();
    uint32_t i = s_base + s_wave[wave] + incl - cnt;
#pragma unroll
    for (int j = 0; j < kFindRows; ++j) {
        if (!(mine & (1u << j))) continue;
        if (i < scr.cap) {
            scr.rows[i] = (int32_t)(row0 + (int64_t)j * kBlock);
            scr.len[i] = len[j];
        }
        ++i;
    }
}

// Window pointers of the long rows, and (zero_rows) zeros in their rows of C.  A list of at least `few_from`
// rows is panel_owner_kernel's, which finds the windows' ends itself while it walks a row and needs only the
// pointers of the first window of every die's share (and the row's end): those alone are written then.
__device__ __forceinline__ int panel_share_begin(int xcd, int windows, int xcds)
{
    return (int)((int64_t)xcd * windows / xcds);  // die x walks the windows [begin(x), begin(x + 1))
}

template <int VEC>
__device__ __forceinline__ void panel_pointers_body(const SpmmArgs& a, const PanelView& scr, int windows,
                                                    int32_t window_rows, int zero_rows, uint32_t few_from, int xcds,
                                                    bool ranked, uint32_t block, uint32_t blocks)
{
    const uint32_t n = scr.head->count;
    if (n == 0 || n > scr.cap) return;
    const int64_t threads = (int64_t)blocks * kBlock;
    const int64_t tid = (int64_t)block * kBlock + threadIdx.x;
    const int per_row = windows + 1;
    const bool few = n >= few_from;
    const int wanted = few ? xcds + 1 : per_row;
    const bool keep_order = !ranked || n > (uint32_t)kRankMaxRows;  // nobody sorts the list: the order of finding
    // kSearchLanes lanes look for one pointer together: each round they probe the stretch that is left at
    // kSearchLanes places and keep the piece in front of the first probe whose column is at or beyond the window's
    // first column (seven rounds of loads for a row of 20,000 entries, where one lane's bisection takes fifteen;
    // every round is a load from HBM, about a microsecond, and nothing else happens meanwhile.  More lanes per
    // pointer need fewer rounds but, for the 45,000 pointers of 5,000 long rows, more threads than are resident
    // at once: 16 lanes took longer than 4).  For any order of the columns the result is monotone in w, it is the row's first
    // entry for w = 0 and (w == windows) its end: the runs always partition the row.
    const int part = threadIdx.x % kSearchLanes;
    const int shift = (threadIdx.x % kWave) / kSearchLanes * kSearchLanes;
    const int64_t items = (int64_t)n * wanted;
    const int64_t rounds = (items * kSearchLanes + threads - 1) / threads;  // the same for every thread: ballots inside
    for (int64_t round = 0; round < rounds; ++round) {
        const int64_t t = (tid + round * threads) / kSearchLanes;
        const bool mine = t < items;
        const int i = mine ? (int)(t / wanted) : 0;
        const int w = !mine ? 0 : few ? panel_share_begin((int)(t % wanted), windows, xcds) : (int)(t % wanted);
        int32_t lo = 0, hi = 0;
        if (mine) {
            const int32_t row = scr.rows[i];
            lo = a.rowptr[row];
            hi = lo + scr.len[i];
            if (w >= windows) lo = hi;
        }
        const int64_t target = (int64_t)w * window_rows;
        while (__any(lo < hi)) {
            // probe j of kSearchLanes sits at lo + floor(span * (j + 1) / (kSearchLanes + 1)) < hi (in 32 bits)
            const uint32_t span = (uint32_t)(hi - lo);
            const uint32_t whole = span / (kSearchLanes + 1), rest = span % (kSearchLanes + 1);
            auto place = [&](int j) { return lo + (int32_t)(whole * (uint32_t)j + rest * (uint32_t)j / (kSearchLanes + 1)); };
            const bool at_or_beyond = lo < hi && a.colidx[place(part + 1)] >= target;
            const uint32_t found = (uint32_t)(__ballot(at_or_beyond) >> shift) & ((1u << kSearchLanes) - 1u);
            if (lo < hi) {
                const int first = found ? __ffs((int)found) - 1 : kSearchLanes;  // probes in front of it are below
                const int32_t new_lo = first > 0 ? place(first) + 1 : lo;
                const int32_t new_hi = first < kSearchLanes ? place(first + 1) : hi;
                lo = new_lo;
                hi = new_hi;
            }
        }
        if (mine && part == 0) {
            scr.ptr[(int64_t)i * per_row + w] = lo;
            if (keep_order && t % wanted == 0) scr.order[i] = i;
        }
    }
    if (!zero_rows) return;
    const int64_t chunks = a.N / VEC;  // N % VEC == 0
    Vec<VEC> z;
    z.zero();
    for (int64_t t = tid; t < (int64_t)n * chunks; t += threads) {
        const int i = (int)(t / chunks);
        const int64_t k = (t % chunks) * VEC;
        store_vec<VEC>(a.C + (int64_t)scr.rows[i] * a.N + k, z);
    }
}

// Value that lane `j` of the wavefront holds.  With one member per wavefront
// (UNIFORM) every lane asks for the same j, and the value comes back in a
// scalar register, so that the address arithmetic on it runs on the scalar unit.
template <bool UNIFORM>
__device__ __forceinline__ int32_t from_lane(int32_t v, int j)
{
    if constexpr (UNIFORM) return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(j));
    else return __shfl(v, j, kWave);
}

constexpr int kPanelDepth = 8;   // gathered rows of B in flight per lane
constexpr int kPanelClaim = 16;  // items a workgroup takes from its die's counter at a time
// Chunk lanes per column tile of the SpMM path: 64 lanes = 256 columns, the widest a wavefront covers.
// Narrower tiles would let a window hold more rows and so need fewer atomic pieces per row of C, but
// the narrower gathers cost more than that saves (skewed: 3.46 ms at 64 lanes, 3.69 at 32, 4.11 at 16).
constexpr int kPanelTileLanes = 64;

// acc += the entries [p0, p1) times the columns k0 .. k0 + LC*VEC of B, for this
// lane's member (the members split the entries) and chunk of columns.
template <int G, int LC, int VEC, bool OFF32>
__device__ __forceinline__ void panel_accumulate(const SpmmArgs& a, Vec<VEC>& acc, int32_t p0, int32_t p1, int64_t k0,
                                                 int lane)
{
    constexpr int D = kPanelDepth;
    const int member = lane / LC;
    const int chunk = lane % LC;
    const int64_t k = k0 + (int64_t)chunk * VEC;
    const bool k_ok = k < a.N;
    const BRow<OFF32> brow(a.B, a.N, k_ok ? k : 0);
    for (int32_t base = p0; base < p1; base += kWave) {
        // 64 entries with one coalesced load each for columns and values
        int32_t my_col = 0, my_val = 0;
        if (base + lane < p1) {
            my_col = load_stream(a.colidx + base + lane);
            my_val = __float_as_int(load_stream(a.vals + base + lane));
        }
        const int cnt = p1 - base < kWave ? p1 - base : kWave;
        // member m takes entries m, m + G, ... of the 64
        for (int j0 = 0; j0 < cnt; j0 += G * D) {
            int32_t col[D];
            float val[D];
            Vec<VEC> b[D];
#pragma unroll
            for (int u = 0; u < D; ++u) {
                const int j = j0 + u * G + member;
                col[u] = from_lane<G == 1>(my_col, j & (kWave - 1));
                val[u] = __int_as_float(from_lane<G == 1>(my_val, j & (kWave - 1)));
                if (j >= cnt) val[u] = 0.0f;
            }
#pragma unroll
            for (int u = 0; u < D; ++u) {
                b[u].zero();
                if (k_ok && j0 + u * G + member < cnt) b[u] = load_vec<VEC>(brow.at(col[u]));
            }
#pragma unroll
            for (int u = 0; u < D; ++u) acc.fma(val[u], b[u]);
        }
    }
}

// The members' partial sums of one row piece, tree-summed and added into C.
// Member 0's LC lanes hold the LC*VEC consecutive columns of the tile, VEC per
// lane.  An atomic instruction whose lanes are 16 bytes apart keeps the memory
// pipeline busy four times longer than one over consecutive words (451 against
// 115 clocks, measured), so the sums change hands first, which also makes the
// instructions as few as they can be: in round q lane l adds column q*64 + l,
// which lane (q*64 + l) / VEC holds (lanes 0 .. LC-1 are member 0).
template <int G, int LC, int VEC>
__device__ __forceinline__ void panel_flush(const SpmmArgs& a, Vec<VEC> acc, int64_t row, int64_t k0, int lane)
{
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc.v[v] = group_tree_sum<G, LC>(acc.v[v]);
    constexpr int PASS = LC * VEC;
#pragma unroll
    for (int q = 0; q < (PASS + kWave - 1) / kWave; ++q) {
        const int col = q * kWave + lane;  // column of the tile, counted from k0
        float mine = 0.0f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const float t = __shfl(acc.v[v], (col / VEC) & (kWave - 1), kWave);
            if (col % VEC == v) mine = t;
        }
        if (col < PASS && k0 + col < a.N) unsafeAtomicAdd(a.C + row * a.N + k0 + col, mine);
    }
}

// One item: the entries [p0, p1) of row `row` times the columns k0 .. k0 + LC*VEC
// of B, multiplied out by one wavefront whose 64 lanes are G members x LC chunk
// lanes.  p0, p1, row and k0 are the same in all lanes.
template <int G, int LC, int VEC, bool OFF32>
__device__ __forceinline__ void panel_item(const SpmmArgs& a, int32_t p0, int32_t p1, int64_t row, int64_t k0, int lane)
{
    Vec<VEC> acc;
    acc.zero();
    panel_accumulate<G, LC, VEC, OFF32>(a, acc, p0, p1, k0, lane);
    panel_flush<G, LC, VEC>(a, acc, row, k0, lane);
}

// B is cut into blocks of one window of rows by one tile of LC*VEC columns
// (one tile unless N > 256), about 2 MiB each.  Die x takes the blocks x,
// x + xcds, ... (window-major); its items (block, long row) are handed out to
// its workgroups kPanelClaim at a time from one counter, one item per
// wavefront.  Items differ in length by a factor of ten and more: with a fixed
// deal the wavefronts of a die drift more than a block apart, which the L2
// cannot hold (43 GB fetched instead of 1.8 GB on the skewed workload), and one
// item per claim makes the counter the bottleneck (a returning atomic on one
// address takes about 0.1 us).
template <int G, int LC, int VEC, bool OFF32>
__global__ __launch_bounds__(kBlock) void panel_long_rows_kernel(SpmmArgs a, PanelView scr, int windows, int xcds,
                                                                 uint32_t below)
{
    // below: the kernel runs only for lists of fewer rows (longer lists are panel_owner_kernel's)
    static_assert(G * LC == kWave, "one wavefront per item");
    __shared__ uint32_t s_claim;
    const uint32_t n = scr.head->count;
    if (n == 0 || n > scr.cap || n >= below) return;
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int per_row = windows + 1;
    const int xcd = blockIdx.x % xcds;
    const int tiles = (int)((a.N + LC * VEC - 1) / (LC * VEC));
    const int64_t blocks = (int64_t)windows * tiles;
    const int64_t my_blocks = xcd < blocks ? (blocks - xcd + xcds - 1) / xcds : 0;
    const uint32_t items = (uint32_t)(my_blocks * n);  // host: blocks * cap < 2^32
    for (;;) {
        __syncthreads();  // everyone has read the previous claim
        if (threadIdx.x == 0) s_claim = atomicAdd(&scr.head->next[xcd], (uint32_t)kPanelClaim);
        __syncthreads();
        const uint32_t claim = s_claim;
        if (claim >= items) break;  // the whole workgroup; the counter only grows, so every workgroup gets here
        for (int r = 0; r < kPanelClaim / kWavesPerBlock; ++r) {
            const uint32_t it = claim + (uint32_t)(r * kWavesPerBlock + wave);
            if (it >= items) break;
            const int64_t block = xcd + (int64_t)xcds * (it / n);
            const int w = (int)(block / tiles);
            const int64_t k0 = (block % tiles) * (LC * VEC);
            const int i = (int)(it % n);
            const int32_t p0 = scr.ptr[(int64_t)i * per_row + w];
            const int32_t p1 = scr.ptr[(int64_t)i * per_row + w + 1];
            if (p0 < p1) panel_item<G, LC, VEC, OFF32>(a, p0, p1, scr.rows[i], k0, lane);
        }
    }
}

// order[] = the long rows sorted by length, longest first (ties by their place in rows[]).  Every row counts
// the rows that come before it, sixteen lanes to a row, with all lengths in LDS; a list of more than
// kRankMaxRows rows keeps the order in which the rows were found (panel_pointers_kernel wrote it): with so
// many rows every wavefront owns several dozen and their lengths average out.
constexpr int kRankLanes = 16;
static_assert(kRankMaxRows % (kRankLanes * 4) == 0, "the padded list fits the LDS array");
__device__ __forceinline__ void panel_rank_body(const PanelView& scr, int32_t* s_len, uint32_t block)
{
    const uint32_t n = scr.head->count;
    constexpr uint32_t rows_per_block = kBlock / kRankLanes;
    if (n == 0 || n > scr.cap || n > (uint32_t)kRankMaxRows || block * rows_per_block >= n) return;
    // (padded to a multiple of the unrolled stride with lengths no row has: they come before nobody)
    constexpr uint32_t kStride = kRankLanes * 4;
    const uint32_t n_pad = (n + kStride - 1) / kStride * kStride;  // <= kRankMaxRows, a multiple of kStride
    constexpr int kAtOnce = 8;  // loads in flight per thread
    for (uint32_t j0 = threadIdx.x; j0 < n_pad; j0 += kAtOnce * kBlock) {
        int32_t len[kAtOnce];
#pragma unroll
        for (int u = 0; u < kAtOnce; ++u) {
            const uint32_t j = j0 + (uint32_t)u * kBlock;
            len[u] = j < n ? scr.len[j] : -1;
        }
#pragma unroll
        for (int u = 0; u < kAtOnce; ++u) {
            const uint32_t j = j0 + (uint32_t)u * kBlock;
            if (j < n_pad) s_len[j] = len[u];
        }
    }
    __syncthreads();
    const uint32_t i = block * rows_per_block + threadIdx.x / kRankLanes;
    const uint32_t part = threadIdx.x % kRankLanes;
    const int32_t mine = i < n ? s_len[i] : 0;
    uint32_t before = 0;
    for (uint32_t j0 = part; j0 < n_pad; j0 += kStride) {
        int32_t other[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) other[u] = s_len[j0 + u * kRankLanes];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            before += (other[u] > mine || (other[u] == mine && j0 + u * kRankLanes < i)) ? 1u : 0u;
    }
#pragma unroll
    for (int m = kRankLanes / 2; m >= 1; m /= 2) before += (uint32_t)__shfl_xor((int)before, m, kRankLanes);
    if (i < n && part == 0) scr.order[before] = (int32_t)i;
}

// One launch for both: the first pointer_blocks workgroups write the pointers (and the zeros), the others rank
// the rows; neither reads what the other writes.
template <int VEC>
__global__ __launch_bounds__(kBlock) void panel_pointers_kernel(SpmmArgs a, PanelView scr, int windows,
                                                                int32_t window_rows, int zero_rows, uint32_t few_from,
                                                                int xcds, uint32_t pointer_blocks)
{
    __shared__ int32_t s_len[kRankMaxRows];
    const bool ranked = gridDim.x > pointer_blocks;
    if (blockIdx.x < pointer_blocks)
        panel_pointers_body<VEC>(a, scr, windows, window_rows, zero_rows, few_from, xcds, ranked, blockIdx.x,
                                 pointer_blocks);
    else
        panel_rank_body(scr, s_len, blockIdx.x - pointer_blocks);
}

constexpr int kOwnerBlock = 1024;  // one workgroup of 16 wavefronts per compute unit
constexpr int kOwnerWaves = kOwnerBlock / kWave;
constexpr int kOwnerRows = 10;  // long rows a wavefront owns at a time
constexpr int kOwnerDepth = 8;  // gathered rows of B in flight per lane

// The same work (window, long row), but every long row has ONE owner wavefront per die, which keeps the row's
// sums in registers while its die walks its windows and adds them into C once at the end: 8 atomic row pieces per
// long row instead of one per window.  A die's share is a run of consecutive windows, so that its part of a row
// is one run of stored entries: a wavefront keeps a position per row, takes from there what lies in front of
// the current window's last column, and stays there until the next window (no pointer per window is needed, only
// the share's ends).  A die's wavefronts each own up to kOwnerRows rows (more rows: more passes) and take window
// after window in the same order, so that at any moment they gather from one or two windows, which the die's L2
// holds.  Two things keep them in step.  Rows are dealt from the longest to the shortest, back and forth over the
// wavefronts, so that all have about the same number of entries per window.  And a compute unit runs one
// workgroup of 16 wavefronts that meet at a barrier after every window: the hardware issues the memory
// instructions of the oldest wavefronts of a compute unit first, and without the barrier the youngest end up 1.5
// times slower and sixteen windows behind (measured), far more than an L2 holds.  Between compute units nothing
// but their equal shares of the work keeps the pace: they are alike, and each averages over 160 rows.
// One wavefront per row and 64 lanes on 64 column chunks: the entries are wave-uniform (sgap_uniform.hpp).
// Nothing here relies on sorted columns: an entry is taken in the first window of the share at which it is at
// the front of what is left and lies in front of the window's end, at the latest in the share's last window,
// which takes all that is left.
// Runs only when the list holds at least min_rows rows; with fewer, most wavefronts would own nothing and
// panel_long_rows_kernel (which then runs instead) keeps the whole chip busy.
template <int VEC, bool OFF32>
__global__ __launch_bounds__(kOwnerBlock) void panel_owner_kernel(const int32_t* __restrict__ colidx,
                                                                  const float* __restrict__ vals,
                                                                  const float* __restrict__ B, float* __restrict__ C,
                                                                  PanelView scr, int64_t K, int64_t N, int windows,
                                                                  int32_t window_rows, int xcds, uint32_t min_rows)
{
    constexpr int R = kOwnerRows;
    const uint32_t n = scr.head->count;
    if (n < min_rows || n > scr.cap) return;
    const int lane = threadIdx.x % kWave;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t xcd = blockIdx.x % xcds;
    const uint32_t waves = (gridDim.x / xcds) * kOwnerWaves;  // wavefronts of this die
    const uint32_t me = (blockIdx.x / xcds) * kOwnerWaves + wave;
    const uint32_t rounds = (n + waves - 1) / waves;           // rows a wavefront owns in all
    const int per_row = windows + 1;
    const int w_begin = panel_share_begin((int)xcd, windows, xcds);
    const int w_end = panel_share_begin((int)xcd + 1, windows, xcds);
    const int tiles = (int)((N + kWave * VEC - 1) / (kWave * VEC));
    SpmmArgs a;  // what panel_flush needs
    a.N = N;
    a.C = C;
    for (int tile = 0; tile < tiles; ++tile) {
        const int64_t k0 = (int64_t)tile * (kWave * VEC);
        const int64_t k = k0 + (int64_t)lane * VEC;
        const bool k_ok = k < N;
        const UniformRows<VEC, OFF32> rows(B, K, N, k_ok ? k : 0);
        for (uint32_t r0 = 0; r0 < rounds; r0 += R) {
            // lane l < 3R looks after one position of row slot l % R: where the slot's next entry is (l < R),
            // where the die's share of the row ends (R <= l < 2R), where the 64 entries start that the wavefront
            // holds of the row (2R <= l < 3R); lane l < R also knows the slot's row.
            // (A wavefront without rows in this pass walks along with nothing to do: it is needed at the barriers.)
            int32_t my_pos = 0;
            int32_t my_row = -1;
            {
                const uint32_t round = r0 + (uint32_t)(lane % R);
                const uint32_t q = round * waves + ((round & 1u) ? waves - 1u - me : me);
                if (lane < 3 * R && round < rounds && q < n) {
                    const int32_t i = scr.order[q];
                    my_pos = scr.ptr[(int64_t)i * per_row + (lane >= R && lane < 2 * R ? w_end : w_begin)];
                    my_row = scr.rows[i];
                }
            }
            Vec<VEC> acc[R];
            // 64 entries of every row slot stay in registers from window to window: a window ends somewhere
            // inside them, and the rest is the start of the slot's piece in the next window
            EntryChunk held[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                acc[r].zero();
                held[r] = load_chunk(colidx, vals, __builtin_amdgcn_readlane(my_pos, r),
                                     __builtin_amdgcn_readlane(my_pos, R + r), lane);
            }
            for (int w = w_begin; w < w_end; ++w) {
                const bool last = w + 1 == w_end;  // of the share: takes all that is left
                const int64_t limit64 = (int64_t)(w + 1) * window_rows;
                const int32_t limit = limit64 > 0x7fffffffLL ? 0x7fffffff : (int32_t)limit64;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    int32_t p = __builtin_amdgcn_readlane(my_pos, r);
                    const int32_t end = __builtin_amdgcn_readlane(my_pos, R + r);
                    int32_t base = __builtin_amdgcn_readlane(my_pos, 2 * R + r);
                    for (;;) {
                        // held[r] has the entries base .. base + 63 (none at or beyond end); p lies among them
                        const int from = p - base;
                        int to = end - base < kWave ? end - base : kWave;
                        if (to < from) to = from;
                        const bool whole = to == kWave && base + kWave < end;  // the row goes on behind them
                        if (!last) {
                            const unsigned long long beyond =
                                __ballot(lane >= from && lane < to && held[r].col >= limit);
                            if (beyond) to = __ffsll((long long)beyond) - 1;
                        }
                        // all of them taken and more to come: the next 64 are requested before these are multiplied
                        const bool refill = whole && to == kWave;
                        EntryChunk ahead = held[r];
                        if (refill) ahead = load_chunk(colidx, vals, base + kWave, end, lane);
                        if (to > from) chunk_accumulate<VEC, OFF32, kOwnerDepth>(rows, acc[r], held[r], from, to);
                        p = base + to;
                        if (!refill) break;
                        held[r] = ahead;
                        base += kWave;
                    }
                    if (lane == r) my_pos = p;
                    if (lane == 2 * R + r) my_pos = base;
                }
                __syncthreads();  // the compute unit's wavefronts take the next window together
            }
            // (the lane number through an opaque copy: the index arithmetic of the flush would otherwise be
            // hoisted in front of the walk and hold some thirty registers throughout it)
            int flush_lane = lane;
            asm volatile("" : "+v"(flush_lane));
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int32_t row = __builtin_amdgcn_readlane(my_row, r);
                if (row >= 0) panel_flush<1, kWave, VEC>(a, acc[r], row, k0, flush_lane);
            }
        }
    }
}

namespace {

template <int G, int LC, int VEC>
void launch_long_rows(const SpmmArgs& a, const PanelView& scr, int windows, int xcds, int compute_units,
                      uint32_t below, hipStream_t s)
{
    const bool off32 = offsets_fit_32(a);
    // workgroups of each instance that one compute unit holds at once: the grid must be resident as a whole
    auto resident = [](auto kernel) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, kBlock, 0) != hipSuccess || n < 1) n = 1;
        return n;
    };
    static const int per_cu_32 = resident(panel_long_rows_kernel<G, LC, VEC, true>);
    static const int per_cu_64 = resident(panel_long_rows_kernel<G, LC, VEC, false>);
    int grid = (off32 ? per_cu_32 : per_cu_64) * compute_units;
    grid -= grid % xcds;
    if (grid < xcds) grid = xcds;
    if (off32)
        hipLaunchKernelGGL((panel_long_rows_kernel<G, LC, VEC, true>), dim3(grid), dim3(kBlock), 0, s, a, scr, windows,
                           xcds, below);
    else
        hipLaunchKernelGGL((panel_long_rows_kernel<G, LC, VEC, false>), dim3(grid), dim3(kBlock), 0, s, a, scr, windows,
                           xcds, below);
}

// The owner kernel runs for lists of at least owner_min_rows rows (half the wavefronts of a die: with fewer rows
// than that most wavefronts would own nothing); below that the claiming kernel does.
uint32_t owner_min_rows(int xcds, int compute_units)
{
    int grid = compute_units;
    grid -= grid % xcds;
    if (grid < xcds) grid = xcds;
    return (uint32_t)(grid / xcds) * kOwnerWaves / 2;
}

template <int VEC>
void launch_owner_rows(const SpmmArgs& a, const PanelView& scr, int windows, int32_t window_rows, int xcds,
                       int compute_units, hipStream_t s)
{
    const bool off32 = offsets_fit_32(a);
    // one workgroup per compute unit (nothing depends on their all being resident: there is no waiting between them)
    int grid = compute_units;
    grid -= grid % xcds;
    if (grid < xcds) grid = xcds;
    const uint32_t min_rows = owner_min_rows(xcds, compute_units);
    if (off32)
        hipLaunchKernelGGL((panel_owner_kernel<VEC, true>), dim3(grid), dim3(kOwnerBlock), 0, s, a.colidx, a.vals, a.B,
                           a.C, scr, a.K, a.N, windows, window_rows, xcds, min_rows);
    else
        hipLaunchKernelGGL((panel_owner_kernel<VEC, false>), dim3(grid), dim3(kOwnerBlock), 0, s, a.colidx, a.vals, a.B,
                           a.C, scr, a.K, a.N, windows, window_rows, xcds, min_rows);
}

// Column windows of about window_bytes of B each, at most kPanelMaxWindows.
void plan_panels(int64_t K, int64_t N, int64_t window_bytes, int* windows, int32_t* window_rows)
{
    int64_t rows = window_bytes / (N * 4);
    if (rows < 1) rows = 1;
    int64_t w = (K + rows - 1) / rows;
    if (w > kPanelMaxWindows) {
        w = kPanelMaxWindows;
        rows = (K + w - 1) / w;
        w = (K + rows - 1) / rows;
    }
    // A multiple of kPanelDies windows of equal size: the dies walk equal shares of the windows, and with
    // 123 windows two of eight dies would walk 16 while the others walk 15 and wait.
    if (w > kPanelDies) {
        w = (w + kPanelDies - 1) / kPanelDies * kPanelDies;
        if (w > kPanelMaxWindows) w = kPanelMaxWindows / kPanelDies * kPanelDies;
        rows = (K + w - 1) / w;
        w = (K + rows - 1) / rows;
    }
    if (w < 1) w = 1;
    *windows = (int)w;
    *window_rows = (int32_t)rows;
}

// The preparation both operators share: list of the rows of at least min_len
// entries, their window pointers, and (zero_rows) zeros in their rows of C.
// owners: the list goes to panel_owner_kernel when it is long enough (the rows are ranked for it, and
// it needs the pointers of its xcds shares only).
void launch_panel_preparation(const SpmmArgs& a, const PanelView& scr, int windows, int32_t window_rows,
                              int32_t min_len, bool zero_rows, bool owners, int xcds, int compute_units,
                              hipStream_t s)
{
    const bool rank_rows = owners;
    const uint32_t few_from = owners ? owner_min_rows(xcds, compute_units) : 0xffffffffu;
    hipLaunchKernelGGL(panel_reset_kernel, dim3(1), dim3(kWave), 0, s, scr);
    constexpr int64_t rows_per_block = (int64_t)kBlock * kFindRows;
    hipLaunchKernelGGL(panel_find_rows_kernel, dim3((unsigned)((a.M + rows_per_block - 1) / rows_per_block)), dim3(kBlock),
                       0, s, a, scr, min_len);
    const uint32_t pointer_blocks = (uint32_t)compute_units * 4;
    uint32_t rank_blocks = 0;
    if (rank_rows) {
        const uint32_t rows = scr.cap < (uint32_t)kRankMaxRows ? scr.cap : (uint32_t)kRankMaxRows;
        rank_blocks = (rows + kBlock / kRankLanes - 1) / (kBlock / kRankLanes);
    }
    hipLaunchKernelGGL((panel_pointers_kernel<4>), dim3(pointer_blocks + rank_blocks), dim3(kBlock), 0, s, a, scr, windows,
                       window_rows, zero_rows ? 1 : 0, few_from, xcds, pointer_blocks);
}

// Lane layout of the SpMM window kernels: chunk lanes for the columns of a tile (at most kPanelTileLanes * 4
// columns), the rest of the 64 lanes split the entries; and the columns of B one item reads per row.
void spmm_panel_layout(int64_t N, int* wave_lc, int64_t* window_cols)
{
    int lc = 1;
    while (lc < kPanelTileLanes && (int64_t)lc * 4 < N) lc *= 2;
    *wave_lc = lc;
    *window_cols = (int64_t)lc * 4 < N ? (int64_t)lc * 4 : N;
}

}  // namespace

int64_t spmm_panels_workspace_bytes(int64_t K, int64_t N, int64_t window_bytes, int64_t cap)
{
    int wave_lc = 1, windows = 1;
    int64_t window_cols = 1;
    int32_t window_rows = 1;
    spmm_panel_layout(N > 0 ? N : 1, &wave_lc, &window_cols);
    plan_panels(K, window_cols, window_bytes, &windows, &window_rows);
    return panel_workspace_bytes(cap, windows);
}

int64_t sddmm_panels_workspace_bytes(int64_t K, int64_t J, int64_t window_bytes, int64_t cap)
{
    int windows = 1;
    int32_t window_rows = 1;
    plan_panels(K, J > 0 ? J : 1, window_bytes, &windows, &window_rows);
    return panel_workspace_bytes(cap, windows);
}

// Long rows (at least min_len entries) window by window, all other rows by the
// row-split kernel with g lanes per row.  Requires vec == 4 (N % 4 == 0, 16-byte
// aligned B and C) and a workspace of spmm_panels_workspace_bytes(K, N, window_bytes, cap)
// bytes.  lc and the other row-split arguments as for launch_row_split.
hipError_t launch_row_split_panels(const SpmmArgs& a, int g, int lc, int vec, int rows_per_slot, bool interleave,
                                   int tile_cols, int xcds, int compute_units, bool persistent, int block,
                                   int wave_vec, int32_t min_len, int64_t window_bytes, void* workspace, int64_t cap,
                                   hipStream_t s)
{
    if (vec != 4 || min_len < 1 || xcds < 1 || !workspace || cap < 1) return hipErrorInvalidValue;
    int wave_lc = 1, windows = 1;
    int64_t window_cols = 1;
    int32_t window_rows = 1;
    spmm_panel_layout(a.N, &wave_lc, &window_cols);
    plan_panels(a.K, window_cols, window_bytes, &windows, &window_rows);
    // the claiming kernel numbers its items (column tile, window, long row) with 32 bits
    if ((a.N + window_cols - 1) / window_cols * windows * cap > 0xffffffffLL)
        return launch_row_split(a, g, lc, vec, rows_per_slot, interleave, tile_cols, xcds, compute_units, persistent,
                                block, s);
    const PanelView scr = panel_view(workspace, cap, windows);
    // a wavefront per row with all 64 lanes on column chunks: worth it from 128 columns on
    const bool owners = wave_lc == kPanelTileLanes && a.N >= 128;
    launch_panel_preparation(a, scr, windows, window_rows, min_len, true, owners, xcds, compute_units, s);
    uint32_t below = 0xffffffffu;
    if (owners) {
        launch_owner_rows<4>(a, scr, windows, window_rows, xcds, compute_units, s);
        below = owner_min_rows(xcds, compute_units);
    }
    switch (wave_lc) {
        case 1: launch_long_rows<64, 1, 4>(a, scr, windows, xcds, compute_units, below, s); break;
        case 2: launch_long_rows<32, 2, 4>(a, scr, windows, xcds, compute_units, below, s); break;
        case 4: launch_long_rows<16, 4, 4>(a, scr, windows, xcds, compute_units, below, s); break;
        case 8: launch_long_rows<8, 8, 4>(a, scr, windows, xcds, compute_units, below, s); break;
        case 16: launch_long_rows<4, 16, 4>(a, scr, windows, xcds, compute_units, below, s); break;
        case 32: launch_long_rows<2, 32, 4>(a, scr, windows, xcds, compute_units, below, s); break;
        default: launch_long_rows<1, 64, 4>(a, scr, windows, xcds, compute_units, below, s); break;
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;

    const RowSkip skip{&scr.head->count, scr.cap, min_len};
    // serial strategy with one wavefront per rows_per_slot rows (sgap_wave_rows.hip)
    if (wave_vec > 0) return launch_wave_rows(a, wave_vec, rows_per_slot, xcds, &skip, s);
    row_split_detail::Launch<false, true> f{a, rows_per_slot, interleave ? 1 : 0, tile_cols, xcds, compute_units,
                                            offsets_fit_32(a), persistent, 0, block, s, skip};
    if (!dispatch_group(g, lc, vec, f)) return hipErrorInvalidValue;
    return hipGetLastError();
}

// ---- SDDMM ------------------------------------------------------------------

// One SDDMM item: out[p] = vals[p] * <X1[row, :], X2T[colidx[p], :]> for the
// entries [p0, p1) of a long row, by one wavefront of G members x LC chunk lanes
// (LC >= 8, J <= LC*4: a lane owns four columns).  The members split the entries
// eight at a time; a member's LC lanes hold partial dot products of its eight
// entries and sum them in log2(LC) exchange steps, the first three of which halve
// the number of values a lane carries (8, 4, 2, 1), so that the eight sums cost
// ten exchanges instead of 8 * log2(LC).  Afterwards lane c of a member holds the
// sum of entry c >> (log2(LC) - 3), and the lanes whose low bits are zero write.
template <int G, int LC>
__device__ __forceinline__ void panel_sddmm_item(const SpmmArgs& a, const float* __restrict__ X1,
                                                 float* __restrict__ out, int32_t p0, int32_t p1, int64_t row, int lane)
{
    constexpr int VEC = 4;
    constexpr int V = 8;  // entries per member and batch
    static_assert(LC >= 8 && G * LC == kWave, "eight values are halved three times");
    const int member = lane / LC;
    const int chunk = lane % LC;
    const int64_t J = a.N;
    const int64_t k = (int64_t)chunk * VEC;
    const bool k_ok = k < J;
    Vec<VEC> x1;
    x1.zero();
    if (k_ok) x1 = load_vec<VEC>(X1 + row * J + k);
    for (int32_t base = p0; base < p1; base += kWave) {
        int32_t my_col = 0, my_val = 0;
        if (base + lane < p1) {
            my_col = load_stream(a.colidx + base + lane);
            my_val = __float_as_int(load_stream(a.vals + base + lane));
        }
        const int cnt = p1 - base < kWave ? p1 - base : kWave;
        for (int j0 = 0; j0 < cnt; j0 += G * V) {
            // member m takes entries j0 + u*G + m, u < 8
            int32_t col[V];
            float val[V], part[V];
            Vec<VEC> x2[V];
#pragma unroll
            for (int u = 0; u < V; ++u) {
                const int j = j0 + u * G + member;
                col[u] = from_lane<G == 1>(my_col, j & (kWave - 1));
                val[u] = __int_as_float(from_lane<G == 1>(my_val, j & (kWave - 1)));
            }
#pragma unroll
            for (int u = 0; u < V; ++u) {
                x2[u].zero();
                if (k_ok && j0 + u * G + member < cnt) x2[u] = load_vec<VEC>(a.B + (int64_t)col[u] * J + k);
            }
#pragma unroll
            for (int u = 0; u < V; ++u) {
                part[u] = 0.0f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) part[u] = __builtin_fmaf(x1.v[v], x2[u].v[v], part[u]);
            }
            // 8 -> 4 -> 2 -> 1 values: the upper half of each pair of lane halves keeps the upper half of the values
            float four[4], two[2], one;
            {
                const bool up = (chunk & (LC / 2)) != 0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float keep = up ? part[u + 4] : part[u];
                    const float send = up ? part[u] : part[u + 4];
                    four[u] = keep + __shfl_xor(send, LC / 2, LC);
                }
            }
            {
                const bool up = (chunk & (LC / 4)) != 0;
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const float keep = up ? four[u + 2] : four[u];
                    const float send = up ? four[u] : four[u + 2];
                    two[u] = keep + __shfl_xor(send, LC / 4, LC);
                }
            }
            {
                const bool up = (chunk & (LC / 8)) != 0;
                const float keep = up ? two[1] : two[0];
                const float send = up ? two[0] : two[1];
                one = keep + __shfl_xor(send, LC / 8, LC);
            }
#pragma unroll
            for (int m = LC / 16; m >= 1; m /= 2) one += __shfl_xor(one, m, LC);
            // this lane's entry of the batch, and its value
            const int u_mine = chunk / (LC / 8);
            float val_mine = val[0];
#pragma unroll
            for (int u = 1; u < V; ++u)
                if (u == u_mine) val_mine = val[u];
            const int j = j0 + u_mine * G + member;
            if (chunk % (LC / 8) == 0 && j < cnt) out[base + j] = val_mine * one;
        }
    }
}

template <int G, int LC>
__global__ __launch_bounds__(kBlock) void panel_sddmm_kernel(SpmmArgs a, const float* __restrict__ X1,
                                                             float* __restrict__ out, PanelView scr, int windows,
                                                             int xcds)
{
    __shared__ uint32_t s_claim;
    const uint32_t n = scr.head->count;
    if (n == 0 || n > scr.cap) return;
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int per_row = windows + 1;
    const int xcd = blockIdx.x % xcds;
    const int64_t my_windows = xcd < windows ? (windows - xcd + xcds - 1) / xcds : 0;
    const uint32_t items = (uint32_t)(my_windows * n);
    for (;;) {  // claims as in panel_long_rows_kernel
        __syncthreads();
        if (threadIdx.x == 0) s_claim = atomicAdd(&scr.head->next[xcd], (uint32_t)kPanelClaim);
        __syncthreads();
        const uint32_t claim = s_claim;
        if (claim >= items) break;
        for (int r = 0; r < kPanelClaim / kWavesPerBlock; ++r) {
            const uint32_t it = claim + (uint32_t)(r * kWavesPerBlock + wave);
            if (it >= items) break;
            const int w = xcd + xcds * (int)(it / n);
            const int i = (int)(it % n);
            const int32_t p0 = scr.ptr[(int64_t)i * per_row + w];
            const int32_t p1 = scr.ptr[(int64_t)i * per_row + w + 1];
            if (p0 < p1) panel_sddmm_item<G, LC>(a, X1, out, p0, p1, scr.rows[i], lane);
        }
    }
}

namespace {

template <int G, int LC>
void launch_sddmm_long_rows(const SpmmArgs& a, const float* X1, float* out, const PanelView& scr, int windows, int xcds,
                            int compute_units, hipStream_t s)
{
    static const int per_cu = [] {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, panel_sddmm_kernel<G, LC>, kBlock, 0) != hipSuccess || n < 1)
            n = 1;
        return n;
    }();
    int grid = per_cu * compute_units;
    grid -= grid % xcds;
    if (grid < xcds) grid = xcds;
    hipLaunchKernelGGL((panel_sddmm_kernel<G, LC>), dim3(grid), dim3(kBlock), 0, s, a, X1, out, scr, windows, xcds);
}

}  // namespace

// a: M, K, N = J, rowptr, colidx, vals, B = X2T.  Requires 16-byte loads (J % 4 == 0,
// aligned X1 and X2T), 32 <= J <= 256 and a workspace of
// sddmm_panels_workspace_bytes(K, J, window_bytes, cap) bytes.
hipError_t launch_sddmm_panels(const SpmmArgs& a, const float* X1, float* out, int g, int per_lane, int xcds,
                               int compute_units, int64_t nnz_hint, int32_t min_len, int64_t window_bytes,
                               void* workspace, int64_t cap, hipStream_t s)
{
    if (a.N % 4 != 0 || a.N < 32 || a.N > 256 || min_len < 1 || xcds < 1 || !workspace || cap < 1)
        return hipErrorInvalidValue;
    int windows = 1;
    int32_t window_rows = 1;
    plan_panels(a.K, a.N, window_bytes, &windows, &window_rows);
    if ((int64_t)windows * cap > 0xffffffffLL) return hipErrorInvalidValue;
    const PanelView scr = panel_view(workspace, cap, windows);
    launch_panel_preparation(a, scr, windows, window_rows, min_len, false, false, 1, compute_units, s);
    int wave_lc = 8;
    while (wave_lc < kWave && (int64_t)wave_lc * 4 < a.N) wave_lc *= 2;
    switch (wave_lc) {
        case 8: launch_sddmm_long_rows<8, 8>(a, X1, out, scr, windows, xcds, compute_units, s); break;
        case 16: launch_sddmm_long_rows<4, 16>(a, X1, out, scr, windows, xcds, compute_units, s); break;
        case 32: launch_sddmm_long_rows<2, 32>(a, X1, out, scr, windows, xcds, compute_units, s); break;
        default: launch_sddmm_long_rows<1, 64>(a, X1, out, scr, windows, xcds, compute_units, s); break;
    }
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    return launch_sddmm_skip(a, X1, out, g, per_lane, compute_units, nnz_hint,
                             RowSkip{&scr.head->count, scr.cap, min_len}, s);
}

}  // namespace sgap
