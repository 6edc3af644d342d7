// Which lattice tiles of a group take part in the backward pass.
//
// Every entry of a lattice node's score gradient dh = gamma * softmax - posteriors (f^W_4) is at most the
// node's posterior gamma = exp(alpha + beta - ln P) in magnitude (the blank and label occupations are parts
// of gamma).  On long utterances gamma is far below the resolution of the sums the gradients are
// accumulated in for most of the lattice: the alignments that carry the probability pass through a narrow
// band.  A tile whose 64 nodes all have gamma < 2^-k contributes less than 2^-k per gradient entry and node
// and is left out; with k = 135 (the default where the fused backward kernel runs) everything such a tile would
// feed into the backward GEMMs is exactly zero as a bfloat16 value.  k_tile_flags marks the tiles that stay,
// k_compact_tiles lists them in their original order (so that every sum that is formed in a fixed order still is).
#include "device_common.h"

namespace rnnt {

namespace {

struct SelectArgs {
    SampleTable st;
    LatticeState ls;
    int s0, s1, tile0, tile1;
    float log_floor;     // ln of the smallest posterior that keeps a tile
    int* flags;          // [tiles of the call] 1 = the tile stays
    int* active;         // [tiles of the call] the group's entries, from tile0 on: tile ids that stay, ascending.
                         // May be the same array as flags: a round's flags are all read (barrier) before its list
                         // entries are written, and those land at or below the positions the round has read.
    int* n_active;       // one counter (this group's)
};

// one wavefront per tile, lane = tile row
__global__ __launch_bounds__(256) void k_tile_flags(SelectArgs a) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile = a.tile0 + (int)blockIdx.x * 4 + wave;
    if (tile >= a.tile1) return;
    const TilePos tp = locate_tile(a.st, a.s0, a.s1, tile);
    const int t = tp.t0 + (lane >> tp.us), u = tp.u0 + (lane & (tp.uw - 1));
    float lg = RNNT_NEG_INF;
    if (t < tp.T && u <= tp.U) {
        const long long idx = (a.st.row_off[tp.s] - a.ls.row_base) + (long long)t * (tp.U + 1) + u;
        lg = a.ls.alpha[idx] + a.ls.beta[idx] - a.ls.lnP[tp.s];
        if (a.ls.weight) lg += __logf(a.ls.weight[tp.s]);
    }
    const float m = wave_max(lg);           // NaN never compares below the floor: such a tile stays
    if (lane == 0) a.flags[tile] = (m < a.log_floor) ? 0 : 1;
}

// one workgroup per group: ordered compaction, 4096 tiles per round
constexpr int CT = 1024;
__global__ __launch_bounds__(CT) void k_compact_tiles(SelectArgs a) {
    __shared__ int wave_tot[CT / 64];
    __shared__ int round_tot;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    int running = 0;
    for (int base = a.tile0; base < a.tile1; base += 4 * CT) {
        const int first = base + 4 * tid;
        int f[4], mine = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[i] = (first + i < a.tile1) ? a.flags[first + i] : 0;
            mine += f[i];
        }
        // inclusive prefix over the workgroup
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o, 64);
            if (lane >= o) incl += v;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = 0;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        if (tid == CT - 1) round_tot = before + incl;
        int pos = a.tile0 + running + before + incl - mine;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (f[i]) a.active[pos++] = first + i;
        __syncthreads();
        running += round_tot;
        __syncthreads();
    }
    if (tid == 0) *a.n_active = running;
}

}  // namespace

hipError_t launch_select_tiles(const SampleTable& st, const LatticeState& ls, int s0, int s1, int tile0, int tile1,
                               float log_floor, int* flags, int* active, int* n_active, hipStream_t stream) {
    const int n = tile1 - tile0;
    if (n <= 0) return hipSuccess;
    SelectArgs a{st, ls, s0, s1, tile0, tile1, log_floor, flags, active, n_active};
    k_tile_flags<<<dim3((unsigned)((n + 3) / 4)), dim3(256), 0, stream>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    k_compact_tiles<<<dim3(1), dim3(CT), 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace rnnt
