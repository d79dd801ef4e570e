// Heavy-hitter retention and order-preserving cache compaction (Sec. 3.1 of arXiv 2506.01215:
// attention-based token eviction to the budget, retained tokens re-packed to consecutive
// positions; Sec. 4 setup: protected initial / recent tokens).
//
//   select_topk    (select.hip) exact top-B of the n candidate scores per KV head, lowest-index
//                  ties, protected first/last slots, kept slot indices ascending
//   evict_move_inplace K and V rows of the kept slots -> rows [0, new_len), one read + one write
//                      per moved row, ordered by per-tile flags (row sizes dividing 16 KB); the
//                      4-byte score / pos entries are staged by the selection's emission pass
//                      and written back by trailing workgroups of this kernel
//   evict_move<..>     fallback for other row sizes: K, V, score, pos through staging
// Rows whose slot does not change (kept_idx[r] == r, always a prefix) are not touched.
#include "common.h"

namespace reform {

hipError_t select_topk(const SelParams &p, hipStream_t st);

// kept_idx = 0..n-1 when nothing is evicted (n <= B).
__global__ void evict_identity(int32_t *kept, int Hkv, int B, int n)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    const int g = blockIdx.y;
    if (r < n) kept[(size_t)g * B + r] = r;
}

// grid (ceil(B*pieces/256), Hkv, 3): z = 0 moves K rows, z = 1 V rows (one 16-byte piece per
// thread), z = 2 the 4-byte score and pos entries (one row per thread).
template <bool TO_STAGE>
__global__ __launch_bounds__(256) void evict_move(EvictParams p)
{
    const int pieces = p.row_bytes >> 4;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const int g = blockIdx.y;
    if (blockIdx.z == 2) {
        const int r = (int)idx;
        if (idx >= p.B) return;
        const int src = p.kept[(size_t)g * p.B + r];
        if (src == r || (unsigned)src >= (unsigned)p.n) return;
        const size_t srow = (size_t)g * p.cap + (TO_STAGE ? src : r);
        const size_t trow = (size_t)g * p.B + r;
        if (TO_STAGE) {
            p.stage_score[trow] = p.score[srow];
            if (p.pos) p.stage_pos[trow] = p.pos[srow];
        } else {
            p.score[srow] = p.stage_score[trow];
            if (p.pos) p.pos[srow] = p.stage_pos[trow];
        }
        return;
    }
    const int r = (int)(idx / pieces), c = (int)(idx % pieces);
    if (r >= p.B) return;
    const int src = p.kept[(size_t)g * p.B + r];
    if (src == r || (unsigned)src >= (unsigned)p.n) return;
    const size_t srow = (size_t)g * p.cap + (TO_STAGE ? src : r);   // row in the cache arrays
    const size_t trow = (size_t)g * p.B + r;                        // row in the staging arrays
    char *cache = (char *)(blockIdx.z ? p.v : p.k) + srow * p.row_bytes + (size_t)c * 16;
    char *stage = (char *)(blockIdx.z ? p.stage_v : p.stage_k) + trow * p.row_bytes + (size_t)c * 16;
    if (TO_STAGE) *(v4u *)stage = *(const v4u *)cache;
    else *(v4u *)cache = *(const v4u *)stage;
}

// ------------------------------------------------------------------------------------------
// In-place, single-pass compaction of the K and V rows.  Destination row r takes source row
// kept[r] >= r, so a workgroup that writes dest rows [a, b) may destroy sources that other
// workgroups still have to read.  Who reads the rows [a, b)?  The dest rows rank(a)..rank(b)-1
// (rank(x) = number of kept slots below x), which lie in at most two tiles, both at or before the
// writer's own tile.  Protocol per tile of 16 KB:
//   1. take a ticket from the stream's atomic counter (stream = (head, K|V)): tiles of a stream are
//      handed out in ascending order, so every lower tile of the stream is already running when a
//      tile starts, whatever order the hardware dispatches workgroups in;
//   2. load the tile's source rows into registers and wait until the data has arrived;
//   3. publish flag[stream][tile] = 1 with a relaxed device-scope atomic store.  Nothing has to be
//      made visible except the flag itself (the tile has only READ so far, and its loads have
//      returned), so no release fence is used: on a multi-XCD part a device-scope release writes
//      back a whole L2 and made this kernel 4x slower than the staged copy;
//   4. poll (relaxed atomic loads) the flags of the <= 2 tiles that read rows [a, b) -- they never
//      wait before publishing, so this ends; the spin is bounded anyway and a timeout only raises
//      an error word.  The stores of step 5 are issued after the poll returned;
//   5. store the registers to rows [a, b).
// Traffic: every moved row is read once and written once.
constexpr int kTileBytes = kMoveTileBytes;
constexpr int kTilePieces = kTileBytes / 16 / 256;   // 16-byte pieces per thread
constexpr int kSyncLine = 32;        // ints per 128-byte line

__global__ __launch_bounds__(256) void evict_move_inplace(EvictParams p)
{
    __shared__ int sh[4];
    const int tid = threadIdx.x;
    const int nstreams = p.Hkv * 2;
    if ((int)blockIdx.x >= nstreams * p.ntile) {
        // trailing workgroups: the 4-byte score / pos entries come back from their staging rows
        // (filled by the selection's emission pass, which has finished before this kernel starts)
        const int sb = blockIdx.x - nstreams * p.ntile;
        const int per_head = (p.B + 255) / 256;
        const int g = sb / per_head, r = (sb % per_head) * 256 + tid;
        if (r >= p.B) return;
        const int src = p.kept[(size_t)g * p.B + r];
        if (src == r || (unsigned)src >= (unsigned)p.n) return;
        p.score[(size_t)g * p.cap + r] = p.stage_score[(size_t)g * p.B + r];
        if (p.pos) p.pos[(size_t)g * p.cap + r] = p.stage_pos[(size_t)g * p.B + r];
        return;
    }
    const int tr = kTileBytes / p.row_bytes;             // rows per tile
    const int pieces = p.row_bytes >> 4;
    // sync layout: [0] error word, then one ticket counter per stream (each on its own 128-byte
    // line: a single shared counter serialises 8192 atomics on one L2 address), then the flags
    const int stream = blockIdx.x % nstreams;
    int *counter = p.sync + kSyncLine * (1 + stream);
    int *flags = p.sync + kSyncLine * (1 + nstreams);
    if (tid == 0) sh[0] = atomicAdd(counter, 1);
    __syncthreads();
    const int tile = sh[0];                               // ascending within the stream
    const int g = stream >> 1;
    const int a = tile * tr, b = min(a + tr, p.B);
    if (a >= p.B) return;
    const int32_t *kept = p.kept + (size_t)g * p.B;
    int *flag = flags + (size_t)stream * p.ntile;
    char *base = (char *)((stream & 1) ? p.v : p.k) + (size_t)g * p.cap * p.row_bytes;

    // spin_limit 0 is the host's way to exercise the give-up branch: no tile publishes and every
    // wait on another tile expires on its first poll, so the kernel still runs to its end
    const bool publish = p.spin_limit > 0;
    if (kept[b - 1] == b - 1) {                           // kept[r] == r for every r < b: nothing moves
        if (tid == 0 && publish) __hip_atomic_store(&flag[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    v4u data[kTilePieces];
    int rows[kTilePieces];
#pragma unroll
    for (int i = 0; i < kTilePieces; ++i) {
        const int q = tid + 256 * i;
        const int r = a + q / pieces, c = q % pieces;
        rows[i] = r < b ? r : -1;
        if (r < b) {
            int src = kept[r];
            src = (unsigned)src < (unsigned)p.n ? src : r;
            data[i] = *(const v4u *)(base + (size_t)src * p.row_bytes + (size_t)c * 16);
        }
    }
    __builtin_amdgcn_s_waitcnt(0);                        // all loads of this wave have returned
    asm volatile("" ::: "memory");
    __syncthreads();                                      // ... and of every wave of the tile
    if (tid == 0) {
        if (publish) __hip_atomic_store(&flag[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // readers of rows [a, b): dest rows lo .. hi-1 with lo = rank(a), hi = rank(b)
        const int32_t *rank = p.sel.out_rank + (size_t)g * p.cap;
        const int lo = rank[a], hi = rank[b];             // b <= B < n: inside the candidate range
        if (hi > lo) {
            for (int t2 = lo / tr; t2 <= (hi - 1) / tr; ++t2) {
                if (t2 == tile) continue;
                int spins = 0;
                while (__hip_atomic_load(&flag[t2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
                    if (++spins > p.spin_limit) { atomicExch(p.sync, 1); break; }
                    __builtin_amdgcn_s_sleep(4);
                }
            }
        }
        asm volatile("" ::: "memory");
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kTilePieces; ++i) {
        if (rows[i] >= 0) {
            const int c = (tid + 256 * i) % pieces;
            *(v4u *)(base + (size_t)rows[i] * p.row_bytes + (size_t)c * 16) = data[i];
        }
    }
}

hipError_t evict_run(const EvictParams &p, hipStream_t st)
{
    const int pieces = p.row_bytes >> 4;
    if (p.sync) {
        // K/V rows in place.  The selection's own launches also clear the tickets and flags and
        // stage the 4-byte score / pos entries of the retained slots (8 bytes per row); trailing
        // workgroups of the move kernel bring them back.
        SelParams sel = p.sel;
        sel.out_val = p.stage_score;
        sel.side_src = p.pos;
        sel.side_dst = p.pos ? p.stage_pos : nullptr;
        sel.zero_extra = p.sync;
        sel.zero_extra_n = kSyncLine * (1 + p.Hkv * 2) + p.Hkv * 2 * p.ntile;
        sel.err = p.sync;                       // the call's status word
        hipError_t e = select_topk(sel, st);
        if (e != hipSuccess) return e;
        const int side_blocks = p.Hkv * ((p.B + 255) / 256);
        hipLaunchKernelGGL(evict_move_inplace, dim3(p.Hkv * 2 * p.ntile + side_blocks), dim3(256), 0, st, p);
        return hipGetLastError();
    }
    hipError_t e = select_topk(p.sel, st);
    if (e != hipSuccess) return e;
    const long items = (long)p.B * pieces;
    const dim3 grid((unsigned)((items + 255) / 256), p.Hkv, 3);
    hipLaunchKernelGGL(evict_move<true>, grid, dim3(256), 0, st, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(evict_move<false>, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t evict_fill_identity(int32_t *kept, int Hkv, int B, int n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(evict_identity, dim3((n + 255) / 256, Hkv), dim3(256), 0, st, kept, Hkv, B, n);
    return hipGetLastError();
}

}  // namespace reform
