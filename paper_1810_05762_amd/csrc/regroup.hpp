// Interaction groups chosen from where the agents are (Section 3.1: all agents share one scene;
// Section 4.1: the agents of the flagrun tasks collide with each other).
//
// A uniform grid over the ground plane; an agent's cell is that of its root body's world position;
// the agents are ordered along the Hilbert curve through the cells (ties: agent number), which puts
// agents that stand close together mostly close together in the order; windows of up to 256
// consecutive agents of that order are then split into groups by who is within reach of whom.
// The places of the launch (a workgroup holds consecutive places, a group consecutive places of a
// workgroup) are handed out in the resulting order.
// Every decision is taken in single precision with the operation order written out, so that a
// reference in plain C reaches the same order bit for bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sim355 {

#pragma clang fp contract(off)

// Position of cell (x, y), 16 bits each, along the Hilbert curve of order 16 (Hilbert 1891; the
// usual bit-by-bit form): from the top bit down, the quadrant (rx, ry) adds ((3 rx) xor ry) times
// the quadrant's size, and the coordinates inside it are reflected and exchanged so that the curve
// of the next level starts where this one enters the quadrant.
__device__ __forceinline__ uint32_t hilbert_index16(uint32_t x, uint32_t y) {
  uint32_t d = 0;
  for (uint32_t s = 32768u; s > 0; s >>= 1) {
    const uint32_t rx = (x & s) ? 1u : 0u, ry = (y & s) ? 1u : 0u;
    d += s * s * ((3u * rx) ^ ry);
    x &= s - 1u; y &= s - 1u;          // inside the quadrant
    if (ry == 0u) {
      if (rx == 1u) { x = (s - 1u) - x; y = (s - 1u) - y; }
      const uint32_t t = x; x = y; y = t;
    }
  }
  return d;
}

// cell index along one axis, moved into 0 .. 65535 (clamped; NaN goes to 0)
__device__ __forceinline__ uint32_t cell_coord(float p, float cell) {
  float c = floorf(p / cell);
  if (!(c >= -32768.0f)) c = -32768.0f;
  if (c > 32767.0f) c = 32767.0f;
  return (uint32_t)((int)c + 32768);
}

// world position of agent i's root body; state is [13][B][N], origins [N][3]
__device__ __forceinline__ void root_world(const float* __restrict__ state, const float* __restrict__ origins, int B, int N,
                                           int root, int i, float p[3]) {
  for (int c = 0; c < 3; ++c) p[c] = state[((size_t)c * B + root) * N + i] + origins[3 * i + c];
}

// words[i] = (position of agent i's cell along the curve) << 32 | i
__global__ void order_words_kernel(const float* __restrict__ state, const float* __restrict__ origins, int B, int N, int root,
                                   float cell, unsigned long long* __restrict__ words) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N) return;
  float p[3];
  root_world(state, origins, B, N, root, i, p);
  const uint32_t key = hilbert_index16(cell_coord(p[0], cell), cell_coord(p[1], cell));
  words[i] = ((unsigned long long)key << 32) | (unsigned)i;
}

// place_env[rank of words[i] among all words] = i.  The words are distinct (they end in the agent
// number), so the ranks are a permutation.  Quadratic in N on purpose: no scratch memory, a
// result that does not depend on scheduling, and a few milliseconds at 65536 agents.
__global__ void rank_places_kernel(const unsigned long long* __restrict__ words, int N, int32_t* __restrict__ place_env) {
  // A workgroup ranks 16 agents, 16 threads each: thread (agent a, part q) counts the smaller words
  // among those at positions q, q + 16, ... of every tile, and the 16 counts of an agent are added
  // up in LDS.  (One thread per agent left all but N / 256 compute units idle.)
  __shared__ unsigned long long tile[256];
  __shared__ int part_rank[16][17];
  const int al = threadIdx.x & 15, q = threadIdx.x >> 4;
  const int i = blockIdx.x * 16 + al;
  const unsigned long long mine = i < N ? words[i] : ~0ull;
  int rank = 0;
  for (int j0 = 0; j0 < N; j0 += 256) {
    const int j = j0 + threadIdx.x;
    tile[threadIdx.x] = j < N ? words[j] : ~0ull;     // (a padding word is smaller than nothing)
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) rank += tile[16 * k + q] < mine ? 1 : 0;
    __syncthreads();
  }
  part_rank[al][q] = rank;
  __syncthreads();
  if (q == 0 && i < N) {
    int r = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) r += part_rank[al][k];
    place_env[r] = i;
  }
}

// Second pass: the agents of a window of W consecutive places (W a multiple of the group size G, at
// most 256; one workgroup per window) are put into groups by who is close to whom rather than by
// their order along the curve.  Two agents are neighbours if their root bodies are within `reach`.
//  1. Clusters: in window order, every agent that is still free and has a free neighbour starts a
//     cluster, which takes, while it has fewer than G members, the first free agent (in window
//     order) that is a neighbour of any of its members.  What stays free has no free neighbour.
//  2. Packing: the clusters are laid out one after another; a cluster that does not fit into the
//     group being filled goes to the next one, and the gap is closed with free agents (in window
//     order) or, when they have run out, with the first members of that cluster.  The remaining
//     free agents follow.  Groups are every G consecutive agents of this layout.
// place_env holds the order along the curve on entry and the final places on return; a window
// only touches its own places.
constexpr int kWindow = 256;
__global__ void cluster_windows_kernel(const float* __restrict__ state, const float* __restrict__ origins, int B, int N,
                                       int root, int G, int W, float reach, int32_t* __restrict__ place_env) {
  __shared__ float wp[3][kWindow];
  __shared__ unsigned long long adj[kWindow][4];
  __shared__ unsigned long long has_nb[4];
  __shared__ int agent_of[kWindow];
  __shared__ short seq[kWindow], csize[kWindow / 2], pick[kWindow];
  const int lane = threadIdx.x, w0 = blockIdx.x * W;
  const int n = min(W, N - w0);
  float p[3] = {0.0f, 0.0f, 0.0f};
  if (lane < n) {
    agent_of[lane] = place_env[w0 + lane];
    root_world(state, origins, B, N, root, agent_of[lane], p);
  }
  wp[0][lane] = p[0]; wp[1][lane] = p[1]; wp[2][lane] = p[2];
  __syncthreads();
  const float r2 = reach * reach;
  unsigned long long mine[4] = {0ull, 0ull, 0ull, 0ull};
  if (lane < n)
    for (int k = 0; k < n; ++k) {
      const float dx = p[0] - wp[0][k], dy = p[1] - wp[1][k], dz = p[2] - wp[2][k];
      const float d2 = (dx * dx + dy * dy) + dz * dz;
      if (k != lane && d2 <= r2) mine[k >> 6] |= 1ull << (k & 63);
    }
  for (int w = 0; w < 4; ++w) adj[lane][w] = mine[w];
  // which agents have a neighbour at all: one word per wavefront
  {
    const unsigned long long hn = __ballot((mine[0] | mine[1] | mine[2] | mine[3]) != 0ull);
    if ((lane & 63) == 0) has_nb[lane >> 6] = hn;
  }
  __syncthreads();
  if (lane == 0) {
    // The sets of free agents and of a cluster's candidates live in registers (four 64-bit words
    // each, indexed through unrolled loops): this thread works alone, and a set kept in LDS would
    // cost it a round trip per look.
    unsigned long long fm[4], fr[4], hn[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int lo = 64 * w;
      fm[w] = n >= lo + 64 ? ~0ull : (n > lo ? (1ull << (n - lo)) - 1ull : 0ull);
      hn[w] = has_nb[w];
    }
    auto first_of = [&](const unsigned long long* m) -> int {
      int r = -1;
#pragma unroll
      for (int w = 3; w >= 0; --w) if (m[w]) r = 64 * w + __ffsll((long long)m[w]) - 1;
      return r;
    };
    auto clear_bit = [&](unsigned long long* m, int i) {
      const unsigned long long bit = 1ull << (i & 63);
#pragma unroll
      for (int w = 0; w < 4; ++w) m[w] &= ~((i >> 6) == w ? bit : 0ull);
    };
    // 1. clusters
    int n_seq = 0, n_cl = 0;
#pragma unroll
    for (int sw = 0; sw < 4; ++sw) {
      // seeds of this word in rising order: free agents that have neighbours at all (one without
      // any can neither start a cluster nor be taken by one)
      unsigned long long todo = fm[sw] & hn[sw];
      while (todo) {
        const int sb = __ffsll((long long)todo) - 1, seed = 64 * sw + sb;
        todo &= todo - 1ull;
        if (!((fm[sw] >> sb) & 1ull)) continue;          // taken by an earlier cluster meanwhile
        unsigned long long any = 0ull;
#pragma unroll
        for (int w = 0; w < 4; ++w) { fr[w] = adj[seed][w] & fm[w]; any |= fr[w]; }
        if (!any) continue;
        clear_bit(fm, seed);
        seq[n_seq++] = (short)seed;
        int cnt = 1;
        while (cnt < G) {
          const int nx = first_of(fr);
          if (nx < 0) break;
          clear_bit(fm, nx);
          seq[n_seq++] = (short)nx;
          ++cnt;
#pragma unroll
          for (int w = 0; w < 4; ++w) fr[w] = (fr[w] | adj[nx][w]) & fm[w];
        }
        csize[n_cl++] = (short)cnt;
      }
    }
    // 2. packing
    auto next_single = [&]() -> int {
      const int sgl = first_of(fm);
      if (sgl >= 0) clear_bit(fm, sgl);
      return sgl;
    };
    int out = 0, pos = 0, filled = 0;
    for (int c = 0; c < n_cl; ++c) {
      int sz = csize[c];
      if (filled + sz > G) {
        while (filled < G) {
          const int sgl = next_single();
          if (sgl < 0) break;
          pick[out++] = (short)sgl; ++filled;
        }
        for (; filled < G; ++filled, --sz) pick[out++] = seq[pos++];
        filled = 0;
      }
      for (int t = 0; t < sz; ++t) pick[out++] = seq[pos++];
      filled += sz;
      if (filled == G) filled = 0;
    }
    for (int sgl = next_single(); sgl >= 0; sgl = next_single()) pick[out++] = (short)sgl;
  }
  __syncthreads();
  if (lane < n) place_env[w0 + lane] = agent_of[pick[lane]];
}

// place_of[place_env[p]] = p (place_env null: the identity)
__global__ void invert_places_kernel(const int32_t* __restrict__ place_env, int N, int32_t* __restrict__ place_of) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < N) place_of[place_env ? place_env[p] : p] = p;
}

// counts[0] += agent pairs whose root bodies are within `reach`; counts[1] += those of them whose
// places lie in different groups of G
__global__ void near_pairs_kernel(const float* __restrict__ state, const float* __restrict__ origins, int B, int N, int root,
                                  const int32_t* __restrict__ place_of, int G, float reach,
                                  unsigned long long* __restrict__ counts) {
  __shared__ float tp[3][256];
  __shared__ int tg[256];
  const int i = blockIdx.x * 256 + threadIdx.x;
  float p[3] = {0.0f, 0.0f, 0.0f};
  int gi = -1;
  if (i < N) { root_world(state, origins, B, N, root, i, p); gi = place_of[i] / G; }
  const float r2 = reach * reach;
  unsigned near = 0, split = 0;
  for (int j0 = blockIdx.x * 256; j0 < N; j0 += 256) {   // (pairs i < j only: tiles from the thread's own on)
    const int j = j0 + threadIdx.x;
    float q[3] = {0.0f, 0.0f, 0.0f};
    if (j < N) root_world(state, origins, B, N, root, j, q);
    tp[0][threadIdx.x] = q[0]; tp[1][threadIdx.x] = q[1]; tp[2][threadIdx.x] = q[2];
    tg[threadIdx.x] = j < N ? place_of[j] / G : -1;
    __syncthreads();
    const int n_here = min(256, N - j0);
    if (i < N)
      for (int k = 0; k < n_here; ++k) {
        if (j0 + k <= i) continue;
        const float dx = p[0] - tp[0][k], dy = p[1] - tp[1][k], dz = p[2] - tp[2][k];
        const float d2 = (dx * dx + dy * dy) + dz * dz;
        if (d2 <= r2) { near += 1; split += tg[k] != gi ? 1 : 0; }
      }
    __syncthreads();
  }
  if (near) atomicAdd(&counts[0], (unsigned long long)near);
  if (split) atomicAdd(&counts[1], (unsigned long long)split);
}

// is place_env a permutation of 0 .. N-1?  seen[] starts at zero; flag[0] becomes 1 if not
__global__ void check_places_kernel(const int32_t* __restrict__ place_env, int N, int32_t* __restrict__ seen, int* __restrict__ flag) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= N) return;
  const int e = place_env[p];
  if (e < 0 || e >= N) { flag[0] = 1; return; }
  if (atomicAdd(&seen[e], 1) != 0) flag[0] = 1;
}

__global__ void fill_words_kernel(int32_t* __restrict__ dst, size_t n, int32_t value) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = value;
}

#pragma clang fp contract(fast)

}  // namespace sim355
