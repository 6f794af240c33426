// Data-driven neighbourhood graphs on the GPU (paper Sections 3.2.1-3.2.2, Algorithms 1 and 2):
//   pairwise squared node distances  ->  edge set (minimum spanning tree, or relative neighbourhood graph by the
//   blocker test)  ->  adjacency lists  ->  all-pairs hop counts G (float32, +inf where unreachable).
// Everything that decides an edge is float64 and uses direct differences, so the graphs agree with a float64
// host construction except on exact ties.  Work per rebuild at K = 1024: K^2 D distance flops, K^3 (max, min)
// operations for the blocker test, K breadth-first searches.
//   node_d2_kernel     d2[p][q] = sum_d (w_pd - w_qd)^2
//   boruvka_*          spanning tree for K <= 4096: <= log2 K rounds of (cheapest outgoing edge per node over all
//                      compute units, per-component minimum + merge in one workgroup)
//   mst_prim_kernel    spanning tree for larger K: Prim's method in one workgroup, K rounds of (arg-min, key update)
//   rng_near / rng_prefilter / rng_verify   pair (p, q) survives unless some r has max(d2[p][r], d2[q][r]) <
//                      d2[p][q]: every pair against 64 nodes near p first, the few pairs left against all nodes
//   csr_*              degree count, exclusive scan, ascending neighbour lists
//   bfs_kernel         one wavefront per source, frontier queue and distance row in LDS
#include "som_internal.hpp"

#include <math.h>

namespace som {

constexpr int kBoruvkaMaxNodes = 4096;   // 24 bytes of LDS per node in the merge kernel

// 32 x 32 pairs per workgroup, features staged through LDS 32 at a time; every pair sums over d in ascending order
__global__ void __launch_bounds__(256) node_d2_kernel(const float* __restrict__ W, int K, int D, double* __restrict__ d2)
{
    __shared__ float Wp[32][33];
    __shared__ float Wq[32][33];
    const int tid = threadIdx.x;
    const int p0 = blockIdx.x * 32, q0 = blockIdx.y * 32;
    const int pi = tid >> 5, qi = tid & 31;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    for (int d0 = 0; d0 < D; d0 += 32) {
        __syncthreads();
        for (int e = tid; e < 32 * 32; e += 256) {
            const int i = e >> 5, dd = e & 31;
            const bool in = d0 + dd < D;
            Wp[i][dd] = (in && p0 + i < K) ? W[(size_t)(p0 + i) * D + d0 + dd] : 0.0f;
            Wq[i][dd] = (in && q0 + i < K) ? W[(size_t)(q0 + i) * D + d0 + dd] : 0.0f;
        }
        __syncthreads();
        const int lim = (D - d0 < 32) ? D - d0 : 32;
        for (int dd = 0; dd < lim; ++dd) {
            const double b = (double)Wq[qi][dd];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const double df = (double)Wp[pi + 8 * t][dd] - b;
                s[t] = fma(df, df, s[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int p = p0 + pi + 8 * t, q = q0 + qi;
        if (p < K && q < K) d2[(size_t)p * K + q] = s[t];
    }
}

// adjacency matrix A (K x K bytes) <- minimum spanning tree.  Ties between equal keys go to the lowest node index.
__global__ void __launch_bounds__(1024) mst_prim_kernel(const double* __restrict__ d2, int K, unsigned char* __restrict__ A)
{
    extern __shared__ double prim_lds[];
    double* key = prim_lds;                                   // [K] cheapest connection to the tree
    int* from = reinterpret_cast<int*>(key + K);              // [K] its tree end
    __shared__ double red_v[16];
    __shared__ int red_i[16];
    __shared__ int chosen;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (size_t e = tid; e < (size_t)K * K; e += 1024) A[e] = 0;
    for (int v = tid; v < K; v += 1024) {
        key[v] = (v == 0) ? -1.0 : d2[v];                     // node 0 starts the tree; -1 marks "in tree"
        from[v] = 0;
    }
    __syncthreads();
    for (int round = 1; round < K; ++round) {
        double bv = INFINITY;
        int bi = 0x7fffffff;
        for (int v = tid; v < K; v += 1024) {
            const double k = key[v];
            if (k >= 0.0 && (k < bv || (k == bv && v < bi))) {
                bv = k;
                bi = v;
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double ov = __shfl_xor(bv, o);
            const int oi = __shfl_xor(bi, o);
            if (ov < bv || (ov == bv && oi < bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if (lane == 0) {
            red_v[wave] = bv;
            red_i[wave] = bi;
        }
        __syncthreads();
        if (tid == 0) {
            double mv = red_v[0];
            int mi = red_i[0];
            for (int w = 1; w < 16; ++w)
                if (red_v[w] < mv || (red_v[w] == mv && red_i[w] < mi)) {
                    mv = red_v[w];
                    mi = red_i[w];
                }
            chosen = mi;
            const int f = from[mi];
            A[(size_t)mi * K + f] = 1;
            A[(size_t)f * K + mi] = 1;
            key[mi] = -1.0;
        }
        __syncthreads();
        const int u = chosen;
        const double* row = d2 + (size_t)u * K;
        for (int v = tid; v < K; v += 1024) {
            const double k = key[v];
            const double c = row[v];
            if (k >= 0.0 && c < k) {
                key[v] = c;
                from[v] = u;
            }
        }
        __syncthreads();
    }
}

// ---- Boruvka's method for K <= 4096: every round each component picks its cheapest outgoing edge under the strict
// order (length, lower end, higher end) -- the order Kruskal's method would visit edges in, so the tree is the
// same one even when lengths tie -- and the components joined by the picked edges merge.  At most ceil(log2 K)
// rounds; a round is one scan over all pairs (all compute units) and one single-workgroup merge.

__device__ __forceinline__ bool edge_before(double wa, int la, int ha, double wb, int lb, int hb)
{
    return wa < wb || (wa == wb && (la < lb || (la == lb && ha < hb)));
}

// state[0] = number of components, comp[v] = label of v's component (the label is one of its nodes)
__global__ void __launch_bounds__(256) boruvka_init_kernel(int K, int* __restrict__ comp, int* __restrict__ state,
                                                           unsigned char* __restrict__ A)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e < (size_t)K * K) A[e] = 0;
    if (e < (size_t)K) comp[e] = (int)e;
    if (e == 0) state[0] = K;
}

// one wavefront per node v: cheapest edge to a node of another component
__global__ void __launch_bounds__(256) boruvka_scan_kernel(const double* __restrict__ d2, int K, const int* __restrict__ comp,
                                                           const int* __restrict__ state, double* __restrict__ best_w,
                                                           int* __restrict__ best_u)
{
    if (state[0] <= 1) return;
    const int v = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (v >= K) return;
    const int cv = comp[v];
    double bw = INFINITY;
    int bu = -1, blo = 0x7fffffff, bhi = 0x7fffffff;
    for (int u = lane; u < K; u += 64) {
        if (comp[u] == cv) continue;
        const double w = d2[(size_t)v * K + u];
        const int lo = v < u ? v : u, hi = v < u ? u : v;
        if (bu < 0 || edge_before(w, lo, hi, bw, blo, bhi)) {
            bw = w;
            bu = u;
            blo = lo;
            bhi = hi;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double ow = __shfl_xor(bw, o);
        const int ou = __shfl_xor(bu, o), olo = __shfl_xor(blo, o), ohi = __shfl_xor(bhi, o);
        if (ou >= 0 && (bu < 0 || edge_before(ow, olo, ohi, bw, blo, bhi))) {
            bw = ow;
            bu = ou;
            blo = olo;
            bhi = ohi;
        }
    }
    if (lane == 0) {
        best_w[v] = bw;
        best_u[v] = bu;
    }
}

// single workgroup: per-component minimum of the node picks, edges into A, merge of the joined components
__global__ void __launch_bounds__(1024) boruvka_merge_kernel(int K, int* __restrict__ comp, int* __restrict__ state,
                                                             const double* __restrict__ best_w, const int* __restrict__ best_u,
                                                             unsigned char* __restrict__ A)
{
    if (state[0] <= 1) return;
    extern __shared__ unsigned long long bor_lds[];
    unsigned long long* cw = bor_lds;                                 // [K] bit pattern of the cheapest length
    unsigned long long* ce = cw + K;                                  // [K] its ends, lower << 32 | higher
    int* parent = reinterpret_cast<int*>(ce + K);                     // [K]
    int* parent2 = parent + K;                                        // [K]
    __shared__ int count;
    const int tid = threadIdx.x;
    for (int c = tid; c < K; c += 1024) {
        cw[c] = ~0ull;
        ce[c] = ~0ull;
    }
    if (tid == 0) count = 0;
    __syncthreads();
    // lengths are non-negative doubles (or +inf): their bit patterns order like the values
    for (int v = tid; v < K; v += 1024)
        if (best_u[v] >= 0) atomicMin(&cw[comp[v]], (unsigned long long)__double_as_longlong(best_w[v]));
    __syncthreads();
    for (int v = tid; v < K; v += 1024) {
        const int u = best_u[v];
        if (u >= 0 && (unsigned long long)__double_as_longlong(best_w[v]) == cw[comp[v]]) {
            const unsigned long long lo = v < u ? v : u, hi = v < u ? u : v;
            atomicMin(&ce[comp[v]], (lo << 32) | hi);
        }
    }
    __syncthreads();
    for (int c = tid; c < K; c += 1024) {
        int par = c;
        if (comp[c] == c && ce[c] != ~0ull) {
            const int lo = (int)(ce[c] >> 32), hi = (int)(ce[c] & 0xffffffffull);
            A[(size_t)lo * K + hi] = 1;
            A[(size_t)hi * K + lo] = 1;
            par = (comp[lo] == c) ? comp[hi] : comp[lo];
        }
        parent[c] = par;
    }
    __syncthreads();
    // two components that picked each other (necessarily the same edge): the lower label becomes the root
    for (int c = tid; c < K; c += 1024) {
        const int par = parent[c];
        parent2[c] = (parent[par] == c && c < par) ? c : par;
    }
    __syncthreads();
    int* from = parent2;
    int* to = parent;
    for (int span = 1; span < K; span <<= 1) {
        for (int c = tid; c < K; c += 1024) to[c] = from[from[c]];
        __syncthreads();
        int* t = from;
        from = to;
        to = t;
    }
    int mine = 0;
    for (int v = tid; v < K; v += 1024) {
        const int root = from[comp[v]];      // from[] is not written any more; comp[v] is this thread's own entry
        comp[v] = root;
        if (root == v) ++mine;
    }
    if (mine) atomicAdd(&count, mine);
    __syncthreads();
    if (tid == 0) state[0] = count;
}

// Relative neighbourhood graph: pair (p, q) is an edge unless some third node r has
// max(d2[p][r], d2[q][r]) < d2[p][q].  Testing every r for every pair is K^3 / 2 comparisons, and almost every pair
// is blocked by a node close to one of its ends, so the test runs in three steps, all on the float64 distances:
//   rng_near_kernel       64 nodes near p for every p (the nearest one of every residue class modulo 64)
//   rng_prefilter_kernel  every pair against the 64 nodes near its lower end, nearest first; A = 1 where none blocks
//   rng_verify_kernel     the pairs left (the edges and a few more) against all nodes
// A blocker found in the second step is a blocker; a pair the second step leaves gets the complete test.  The
// result is the one the plain triple loop gives.
constexpr int kNear = 64;

__global__ void __launch_bounds__(256) rng_near_kernel(const double* __restrict__ d2, int K, int* __restrict__ near)
{
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= K) return;
    const double* row = d2 + (size_t)p * K;
    double bv = INFINITY;
    int br = -1;
    for (int r = lane; r < K; r += kNear) {
        const double v = row[r];
        if (r != p && v < bv) {
            bv = v;
            br = r;
        }
    }
    near[(size_t)p * kNear + lane] = br;
}

// one workgroup per lower end p; thread -> upper ends q = tid, tid + 256, ...
__global__ void __launch_bounds__(256) rng_prefilter_kernel(const double* __restrict__ d2, int K,
                                                            const int* __restrict__ near, unsigned char* __restrict__ A)
{
    __shared__ int nr_in[kNear], nr[kNear];
    __shared__ double dpr_in[kNear], dpr[kNear];
    const int tid = threadIdx.x, p = blockIdx.x;
    const double* rp = d2 + (size_t)p * K;
    if (tid < kNear) {
        const int r = near[(size_t)p * kNear + tid];
        nr_in[tid] = r;
        dpr_in[tid] = (r >= 0) ? rp[r] : INFINITY;
    }
    __syncthreads();
    if (tid < kNear) {
        // nearest first (rank by distance, then by place): the closest nodes block most pairs
        const double mine = dpr_in[tid];
        int rank = 0;
        for (int o = 0; o < kNear; ++o) rank += (dpr_in[o] < mine || (dpr_in[o] == mine && o < tid)) ? 1 : 0;
        nr[rank] = nr_in[tid];
        dpr[rank] = mine;
    }
    __syncthreads();
    for (int q = tid; q < K; q += 256) {
        if (q == p) A[(size_t)p * K + p] = 0;
        if (q <= p) continue;
        const double lim = rp[q];
        bool blocked = false;
        for (int o = 0; o < kNear && !blocked; ++o) {
            if (!(dpr[o] < lim)) break;                       // sorted: no later node is closer to p than the pair is long
            blocked = d2[(size_t)nr[o] * K + q] < lim;
        }
        const unsigned char keep = blocked ? 0 : 1;
        A[(size_t)p * K + q] = keep;
        A[(size_t)q * K + p] = keep;
    }
}

// one workgroup per lower end p; a wavefront takes the surviving pairs of 64 upper ends at a time, all its lanes
// scan the third nodes of one pair together
__global__ void __launch_bounds__(256) rng_verify_kernel(const double* __restrict__ d2, int K, unsigned char* __restrict__ A)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, p = blockIdx.x;
    const double* rp = d2 + (size_t)p * K;
    for (int qb = wave * 64; qb < K; qb += 256) {
        const int q = qb + lane;
        const bool alive = q > p && q < K && A[(size_t)p * K + q] != 0;
        unsigned long long mask = __ballot(alive);
        while (mask != 0ull) {
            const int qq = qb + (int)__ffsll((long long)mask) - 1;
            mask &= mask - 1ull;
            const double lim = rp[qq];
            const double* rq = d2 + (size_t)qq * K;
            bool found = false;
            // r = p and r = q give max = d2[p][q] itself, never strictly smaller: no masking needed
            for (int r0 = 0; r0 < K; r0 += 4 * 64) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int r = r0 + 64 * u + lane;
                    if (r < K) found = found || (fmax(rp[r], rq[r]) < lim);
                }
                if (__any(found)) break;
            }
            if (__any(found) && lane == 0) {
                A[(size_t)p * K + qq] = 0;
                A[(size_t)qq * K + p] = 0;
            }
        }
    }
}

__global__ void __launch_bounds__(256) csr_degree_kernel(const unsigned char* __restrict__ A, int K, int* __restrict__ deg)
{
    const int v = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (v >= K) return;
    int c = 0;
    for (int u = lane; u < K; u += 64) c += A[(size_t)v * K + u] ? 1 : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);
    if (lane == 0) deg[v] = c;
}

__global__ void __launch_bounds__(1024) csr_scan_kernel(const int* __restrict__ deg, int K, int* __restrict__ off)
{
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int per = (K + 1023) / 1024;
    int s = 0;
    for (int t = 0; t < per; ++t) {
        const int v = tid * per + t;
        if (v < K) s += deg[v];
    }
    part[tid] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const int add = (tid >= o) ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int run = part[tid] - s;
    for (int t = 0; t < per; ++t) {
        const int v = tid * per + t;
        if (v < K) {
            off[v] = run;
            run += deg[v];
        }
    }
    if (tid == 1023) off[K] = part[1023];
}

__global__ void __launch_bounds__(256) csr_fill_kernel(const unsigned char* __restrict__ A, int K,
                                                       const int* __restrict__ off, int* __restrict__ nbr)
{
    const int v = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (v >= K) return;
    int base = off[v];
    for (int u0 = 0; u0 < K; u0 += 64) {
        const int u = u0 + lane;
        const bool on = u < K && A[(size_t)v * K + u];
        const unsigned long long bal = __ballot(on);
        const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0));
        if (on) nbr[base + below] = u;
        base += __popcll(bal);
    }
}

// Hop counts from source = blockIdx.x to every node: one wavefront per source, no barriers.  dist[] (int32) and the
// visiting order (uint16 queue, every node enters once) live in LDS; the frontier is the queue segment
// [head, tail).  Lanes take one frontier node each and walk its neighbour list in step; a neighbour is claimed with
// a compare-and-swap on its distance, and the claimed ones of a step are appended through a ballot (the queue
// position is a wave-uniform register, not a counter in memory).  LDS operations of one wavefront execute in
// order, so a later step sees the earlier steps' claims and queue entries.
__global__ void __launch_bounds__(64) bfs_kernel(const int* __restrict__ off, const int* __restrict__ nbr, int K,
                                                 float* __restrict__ G)
{
    extern __shared__ int bfs_lds[];
    int* dist = bfs_lds;                                                       // [K]
    unsigned short* queue = reinterpret_cast<unsigned short*>(bfs_lds + K);    // [K]
    const int lane = threadIdx.x, src = blockIdx.x;
    for (int v = lane; v < K; v += 64) dist[v] = (v == src) ? 0 : -1;
    if (lane == 0) queue[0] = (unsigned short)src;
    int head = 0, tail = 1;
    for (int level = 0; head < tail; ++level) {
        const int end = tail;
        for (int base = head; base < end; base += 64) {
            const int i = base + lane;
            const bool has = i < end;
            const int v = has ? (int)queue[i] : 0;
            int e = has ? off[v] : 0;
            const int e1 = has ? off[v + 1] : 0;
            while (__any(e < e1)) {
                bool won = false;
                int u = 0;
                if (e < e1) {
                    u = nbr[e];
                    ++e;
                    won = atomicCAS(&dist[u], -1, level + 1) == -1;
                }
                const unsigned long long mask = __ballot(won);
                if (won) {
                    const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0));
                    queue[tail + below] = (unsigned short)u;
                }
                tail += __popcll(mask);
            }
        }
        head = end;
    }
    for (int v = lane; v < K; v += 64) {
        const int d = dist[v];
        G[(size_t)src * K + v] = d < 0 ? INFINITY : (float)d;
    }
}

} // namespace som

using namespace som;

extern "C" int som_topology(som_ctx* ctx, const float* W, int32_t K, int32_t D, int kind, float* G)
{
    if (!ctx) return SOM_EINVAL;
    if (!W || !G) return fail(ctx, SOM_EINVAL, "null W or G");
    if (K < 1 || D < 1) return fail(ctx, SOM_EINVAL, "K and D must be positive");
    if (kind != SOM_TOPOLOGY_MST && kind != SOM_TOPOLOGY_RNG) return fail(ctx, SOM_EINVAL, "unknown topology kind %d", kind);
    if (K > 12000) return fail(ctx, SOM_EINVAL, "K = %d is above the 12000 nodes the graph kernels hold in LDS", K);
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    const size_t kk = (size_t)K * K;
    const size_t need = kk * sizeof(double) + (size_t)K * sizeof(double) + ((size_t)4 * K + 8 + kk) * sizeof(int) + kk + 1024 +
                        (size_t)K * kNear * sizeof(int);
    if (need > ctx->topo_bytes) {
        if (ctx->topo_blob) {
            if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "sync before workspace growth")) return rc;
            (void)hipFree(ctx->topo_blob);
            ctx->topo_blob = nullptr;
            ctx->topo_bytes = 0;
        }
        if (hipMalloc(&ctx->topo_blob, need) != hipSuccess) {
            (void)hipGetLastError();
            return fail(ctx, SOM_ENOMEM, "cannot allocate %zu bytes for the topology workspace", need);
        }
        ctx->topo_bytes = need;
    }
    double* d2 = (double*)ctx->topo_blob;
    double* best_w = d2 + kk;
    int* deg = (int*)(best_w + K);
    int* off = deg + K;                                  // K + 1 entries
    int* comp = off + K + 2;
    int* best_u = comp + K;
    int* state = best_u + K;                             // 4 entries
    int* nbr = state + 4;                                // at most K * K entries
    unsigned char* A = (unsigned char*)(nbr + kk);
    int* near = (int*)(A + (kk + 1023) / 1024 * 1024);   // K * kNear entries (relative neighbourhood graph only)
    const dim3 tiles((K + 31) / 32, (K + 31) / 32);
    hipLaunchKernelGGL(node_d2_kernel, tiles, dim3(256), 0, ctx->stream, W, K, D, d2);
    if (int rc = check_hip(ctx, hipGetLastError(), "node distance launch")) return rc;
    if (kind == SOM_TOPOLOGY_MST && K <= kBoruvkaMaxNodes) {
        const size_t lds = (size_t)K * 24;
        if (lds > 48 * 1024) {
            if (int rc = check_hip(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(boruvka_merge_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kBoruvkaMaxNodes * 24), "raising the dynamic LDS limit")) return rc;
        }
        hipLaunchKernelGGL(boruvka_init_kernel, dim3((unsigned)((kk + 255) / 256)), dim3(256), 0, ctx->stream, K, comp, state, A);
        int rounds = 0;
        while ((1 << rounds) < K) ++rounds;              // the number of components at least halves every round
        for (int r = 0; r < rounds; ++r) {
            hipLaunchKernelGGL(boruvka_scan_kernel, dim3((K + 3) / 4), dim3(256), 0, ctx->stream, d2, K, comp, state, best_w, best_u);
            hipLaunchKernelGGL(boruvka_merge_kernel, dim3(1), dim3(1024), lds, ctx->stream, K, comp, state, best_w, best_u, A);
        }
    } else if (kind == SOM_TOPOLOGY_MST) {
        const size_t lds = (size_t)K * 12 + 16;
        if (lds > 48 * 1024) {
            if (int rc = check_hip(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(mst_prim_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024), "raising the dynamic LDS limit")) return rc;
        }
        hipLaunchKernelGGL(mst_prim_kernel, dim3(1), dim3(1024), lds, ctx->stream, d2, K, A);
    } else {
        hipLaunchKernelGGL(rng_near_kernel, dim3((K + 3) / 4), dim3(256), 0, ctx->stream, d2, K, near);
        hipLaunchKernelGGL(rng_prefilter_kernel, dim3(K), dim3(256), 0, ctx->stream, d2, K, near, A);
        hipLaunchKernelGGL(rng_verify_kernel, dim3(K), dim3(256), 0, ctx->stream, d2, K, A);
    }
    if (int rc = check_hip(ctx, hipGetLastError(), "edge kernel launch")) return rc;
    hipLaunchKernelGGL(csr_degree_kernel, dim3((K + 3) / 4), dim3(256), 0, ctx->stream, A, K, deg);
    hipLaunchKernelGGL(csr_scan_kernel, dim3(1), dim3(1024), 0, ctx->stream, deg, K, off);
    hipLaunchKernelGGL(csr_fill_kernel, dim3((K + 3) / 4), dim3(256), 0, ctx->stream, A, K, off, nbr);
    if (int rc = check_hip(ctx, hipGetLastError(), "adjacency launch")) return rc;
    // dist[K] int32 + queue[K] uint16 per wavefront (72 KB at the 12000-node limit)
    const size_t bfs_lds_bytes = ((size_t)K * 6 + 3) / 4 * 4;
    if (bfs_lds_bytes > 48 * 1024) {
        if (int rc = check_hip(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(bfs_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 12000 * 6), "raising the dynamic LDS limit")) return rc;
    }
    hipLaunchKernelGGL(bfs_kernel, dim3(K), dim3(64), bfs_lds_bytes, ctx->stream, off, nbr, K, G);
    return check_hip(ctx, hipGetLastError(), "hop-count launch");
}
