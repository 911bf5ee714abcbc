// libtva: greedy tree acceptance and commit of the accepted path's K/V rows (gfx950).
// Entry points and their meaning: include/tva_verify.h.
//
//   accept_kernel   one wave per sequence.  The walk from the root is a chain of dependent steps; each
//                   step's search for the matching child is the parallel part: the 64 lanes test 64
//                   candidate nodes at once and a ballot picks the lowest index.  Integer work,
//                   latency-bound (a few L2 round trips per accepted node).
//   commit_kernel   one workgroup per (path position, sequence): a row of K and a row of V, 16 bytes
//                   per lane, straight from the tree tensors to the cache.  HBM-bound in principle
//                   (read + write of 2 * Hkv * D * 2 bytes per accepted node), launch-bound at the
//                   sizes a decode step has.
//   compact_kernel  the same commit when the tree's K/V already sit in the cache behind the committed
//                   tokens: the accepted rows move down in place, one workgroup per sequence.
//   sample_kernel   acceptance by speculative sampling: one workgroup of 1024 threads per sequence.  The walk
//                   and the tests of the children are a chain of dependent steps that every thread takes in
//                   step (they read the same words); the data-parallel part is over the vocabulary: the
//                   sum of a distribution, the residual after a rejection, the draw of the last token --
//                   one streaming pass over V floats each.
//   row_sums_kernel the sums of all target rows of a small batch, ahead of the walk and with the whole chip: the
//                   walk then passes an accepted node with three loads instead of a pass over its row.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tva.h"
#include "tva_verify.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(64) accept_kernel(const int32_t *__restrict__ parent, const int32_t *__restrict__ cu_T,
                                                    const int32_t *__restrict__ draft, const int32_t *__restrict__ target,
                                                    int max_path, int32_t *__restrict__ path,
                                                    int32_t *__restrict__ path_len, int32_t *__restrict__ next_token) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int t0 = cu_T[b];
  const int T = cu_T[b + 1] - t0;
  if (T <= 0) {
    if (lane == 0) {
      path_len[b] = 0;
      next_token[b] = -1;
    }
    return;
  }
  int cur = 0, len = 1;
  if (lane == 0) path[(size_t)b * max_path] = 0;
  // every accepted node has a larger index than the one before, so at most T - 1 steps
  while (len < max_path) {
    const int want = target[t0 + cur];
    int found = -1;
    for (int base = cur + 1; base < T && found < 0; base += 64) {
      const int c = base + lane;
      const bool hit = c < T && parent[t0 + c] == cur && draft[t0 + c] == want;
      const uint64_t votes = __ballot(hit);
      if (votes) found = base + __builtin_ctzll(votes);
    }
    if (found < 0) break;
    cur = found;
    if (lane == 0) path[(size_t)b * max_path + len] = cur;
    ++len;
  }
  if (lane == 0) {
    path_len[b] = len;
    next_token[b] = target[t0 + cur];
  }
}

// ---- acceptance by speculative sampling ----
struct SampleParams {
  const int32_t *parent, *cu_T, *token;
  const float *p, *q, *u, *u_final;
  float *residual;
  int32_t *path, *path_len, *next_token, *err_flag;
  int V, max_path;
  // sums of the target rows, made ahead of the walk by row_sums_kernel, or NULL: row t's sum is the sum of
  // rowpart[t * pieces .. + pieces - 1]; rows 0 .. sum_T-1 have them
  const double *rowpart;
  // and, gathered by the same kernel, what a node's test as its parent's FIRST tested child reads: first[2 c] =
  // p[parent(c)][token(c)], first[2 c + 1] = q[parent(c)][token(c)] (a walk's reads of them would each be a cold,
  // dependent access to a row of its own)
  const float *first;
  int pieces, sum_T;
  int unit_rows;  // every target row is taken to sum to one: a freshly reached node's normaliser is 1, not summed
};

constexpr int kSampleThreads = 1024, kSampleWaves = kSampleThreads / 64;
constexpr int kSampleTreeLds = 1024;  // nodes of a tree whose parent, token and uniform number are kept in LDS

// One pass over a vocabulary-long row.  Wave w owns the contiguous segment [w * seg, (w + 1) * seg) and its lanes
// take consecutive elements (coalesced; VEC = 4: consecutive groups of four, which needs seg % 4 == 0 and rows
// aligned to 16 bytes); the row is elements lo .. V-1 (a slice of a longer one when several workgroups share a
// row).  load(v) fetches what element (group) v needs, use(v, t, x) handles it (it may store) and
// adds its weight to x; U fetches are issued before the first is used.  wsum[w] receives the segment's sum; the
// return value, the same in every thread, is their sum taken in segment order.
template <int VEC, int U, class L, class C>
__device__ __forceinline__ double segment_pass(int lo, int V, int seg, double *wsum, L load, C use) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int s0 = lo + wave * seg, s1 = s0 + seg < V ? s0 + seg : V;
  constexpr int step = 64 * VEC;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  for (int v = s0 + lane * VEC; v < s1; v += U * step) {
    decltype(load(0)) t[U];
#pragma unroll
    for (int k = 0; k < U; ++k)
      if (v + k * step < s1) t[k] = load(v + k * step);
#pragma unroll
    for (int k = 0; k < U; ++k)
      if (v + k * step < s1) use(v + k * step, t[k], acc[k & 3]);
  }
  double x = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  __syncthreads();  // (wsum may still be read from the pass before; stores of use() are visible after the next barrier)
  if (lane == 0) wsum[wave] = x;
  __syncthreads();
  double z = 0.0;
  for (int w = 0; w < kSampleWaves; ++w) z += wsum[w];
  return z;
}

struct Float4Pair {
  float4 a, c;
};
struct FloatPair {
  float a, c;
};

// the two passes: the sum of a row, and the residual max(0, from - Z q) written to r (from may be r itself)
template <int VEC>
__device__ __forceinline__ double row_sum(int V, int seg, double *wsum, const float *row) {
  if constexpr (VEC == 4) {
    return segment_pass<4, 8>(
        0, V, seg, wsum, [&](int v) { return *reinterpret_cast<const float4 *>(row + v); },  // (V % 4 == 0: no straddling)
        [&](int, const float4 &t, double &x) { x += ((double)t.x + (double)t.y) + ((double)t.z + (double)t.w); });
  } else {
    return segment_pass<1, 8>(
        0, V, seg, wsum, [&](int v) { return row[v]; }, [&](int, float t, double &x) { x += (double)t; });
  }
}

template <int VEC>
__device__ __forceinline__ double residual_pass(int V, int seg, double *wsum, const float *from, const float *q, double Z,
                                                float *r) {
  auto one = [&](float pv, float qv) {
    const double d = (double)pv - Z * (double)qv;
    return d > 0.0 ? (float)d : 0.f;
  };
  if constexpr (VEC == 4) {
    return segment_pass<4, 4>(
        0, V, seg, wsum,
        [&](int v) {
          return Float4Pair{*reinterpret_cast<const float4 *>(from + v), *reinterpret_cast<const float4 *>(q + v)};
        },
        [&](int v, const Float4Pair &t, double &x) {
          float4 o;
          o.x = one(t.a.x, t.c.x), o.y = one(t.a.y, t.c.y), o.z = one(t.a.z, t.c.z), o.w = one(t.a.w, t.c.w);
          *reinterpret_cast<float4 *>(r + v) = o;
          x += ((double)o.x + (double)o.y) + ((double)o.z + (double)o.w);
        });
  } else {
    return segment_pass<1, 4>(
        0, V, seg, wsum, [&](int v) { return FloatPair{from[v], q[v]}; },
        [&](int v, const FloatPair &t, double &x) {
          const float o = one(t.a, t.c);
          r[v] = o;
          x += (double)o;
        });
  }
}

// ---- the sums of all target rows, ahead of the walk ----
// A walk that accepts a child needs of the parent's row only its sum and two entries; summing the row is the pass
// that costs.  For a small batch (few trees, few nodes) the sums of ALL nodes' rows cost less when the whole chip
// makes them at once than the accepted nodes' rows do one after the other.  grid (pieces, rows): a workgroup adds
// the 8192 tokens of one piece of one row, in a fixed order; rows past cu_T[B] (a host count that was too large)
// are left alone.  The first workgroup also clears the n_sync arrival counters of the walk that follows (one
// launch less than with zero_sync_kernel).  One more workgroup per row (piece index = pieces) gathers the two
// entries of the parent's rows that the node's test reads.
constexpr int kRowPieceThreads = 256, kRowPiece = kRowPieceThreads * 32;

template <int VEC>
__global__ void __launch_bounds__(kRowPieceThreads) row_sums_kernel(const float *__restrict__ p, const int32_t *__restrict__ cu_T, int B,
                                                                    int V, double *__restrict__ rowpart, int *__restrict__ sync,
                                                                    int n_sync, const float *__restrict__ q,
                                                                    const int32_t *__restrict__ parent,
                                                                    const int32_t *__restrict__ token, float *__restrict__ first) {
  __shared__ double s_w[kRowPieceThreads / 64];
  const int tid = threadIdx.x, piece = blockIdx.x, row = blockIdx.y;
  const int pieces = (int)gridDim.x - 1;
  if (piece == 0 && row == 0)
    for (int i = tid; i < n_sync; i += kRowPieceThreads) sync[i] = 0;
  if (row >= cu_T[B]) return;
  if (piece == pieces) {
    if (tid != 0) return;
    // the tree that holds node `row`: the last b with cu_T[b] <= row (empty trees share their start with the next)
    int lo = 0, hi = B;  // cu_T[lo] <= row < cu_T[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (cu_T[mid] <= row) lo = mid;
      else hi = mid;
    }
    const int t0 = cu_T[lo], par = parent[row], x = token[row];
    float px = 0.f, qx = 0.f;
    if (par >= 0 && par < row - t0 && x >= 0 && x < V) {
      px = p[(size_t)(t0 + par) * V + x];
      qx = q[(size_t)(t0 + par) * V + x];
    }
    first[2 * (size_t)row] = px, first[2 * (size_t)row + 1] = qx;
    return;
  }
  const float *src = p + (size_t)row * V;
  const int base = piece * kRowPiece;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  if constexpr (VEC == 4) {
    float4 x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int v = base + i * (4 * kRowPieceThreads) + 4 * tid;
      x[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (v < V) x[i] = *reinterpret_cast<const float4 *>(src + v);  // (V % 4 == 0: no straddling)
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i & 3] += ((double)x[i].x + (double)x[i].y) + ((double)x[i].z + (double)x[i].w);
  } else {
    float x[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const int v = base + i * kRowPieceThreads + tid;
      x[i] = v < V ? src[v] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i & 3] += (double)x[i];
  }
  double z = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) z += __shfl_xor(z, o);
  if ((tid & 63) == 0) s_w[tid >> 6] = z;
  __syncthreads();
  if (tid == 0) rowpart[(size_t)row * pieces + piece] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

// the sum of row t from its pieces: the lanes of a wave fetch 64 of them at once (one round trip, not one per
// piece), and every thread adds them in the same order
__device__ __forceinline__ double summed_ahead(const SampleParams &p, int t) {
  const double *part = p.rowpart + (size_t)t * p.pieces;
  const int lane = threadIdx.x & 63;
  double z = 0.0;
  for (int base = 0; base < p.pieces; base += 64) {
    const double mine = base + lane < p.pieces ? part[base + lane] : 0.0;
    const int n = p.pieces - base < 64 ? p.pieces - base : 64;
    for (int j = 0; j < n; ++j) z += __shfl(mine, j);
  }
  return z;
}

// The last token, looked for inside [lo, hi): wsum holds the waves' sums of dist over their segments of that range
// (seg elements each), `before` is the weight in front of lo, `none` says that no place claimed the target (u_final
// was not below 1): then, and when rounding keeps the running sum below the target, it is the last token of the range
// that has weight.  The wave whose segment holds it walks the segment 64 elements at a time; its lane 0 stores it.
__device__ __forceinline__ void draw_in_range(const float *dist, int lo, int hi, int seg, const double *wsum, double before,
                                              double target, bool none, int32_t *out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int wclaim = -1, wlast = 0;
  {
    double pre = before;
    for (int i = 0; i < kSampleWaves; ++i) {
      const double nx = pre + wsum[i];
      if (wclaim < 0 && !none && nx > target) wclaim = i, before = pre;
      if (wsum[i] > 0.0) wlast = i;
      pre = nx;
    }
  }
  const bool wnone = wclaim < 0;
  if (wnone) wclaim = wlast;
  if (wave != wclaim) return;
  const int s0 = lo + wave * seg, s1 = s0 + seg < hi ? s0 + seg : hi;
  double acc = before;
  int tok = -1, last_pos = -1;
  for (int base = s0; base < s1; base += 64) {
    const int v = base + lane;
    const float f = v < s1 ? dist[v] : 0.f;
    double incl = (double)f;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double y = __shfl_up(incl, o);
      if (lane >= o) incl += y;
    }
    const unsigned long long heavy = __ballot(f > 0.f);
    if (heavy) last_pos = base + 63 - __builtin_clzll(heavy);
    const unsigned long long over = wnone ? 0ull : __ballot(acc + incl > target);
    if (over) {
      tok = base + __builtin_ctzll(over);
      break;
    }
    acc += __shfl(incl, 63);
  }
  if (lane == 0) *out = tok >= 0 ? tok : last_pos;
}

// The last token of a walk that ends at a node whose row was summed ahead (no pass has been made over it): the sums
// of the row's pieces, added in the order that made Z, say which piece of 8192 tokens holds it; this workgroup sums
// that piece by segments and draws inside it -- a pass over one piece, not over the row, and no wait for others.
template <int VEC>
__device__ __forceinline__ void draw_in_piece(const SampleParams &p, int t, const float *dist, double Z, double u_final, double *wsum,
                                              int32_t *out) {
  const int lane = threadIdx.x & 63;
  const double target = u_final * Z;
  const double *part = p.rowpart + (size_t)t * p.pieces;
  int k = -1, klast = 0;
  double pre = 0.0, before = 0.0;
  for (int base = 0; base < p.pieces; base += 64) {
    const double mine = base + lane < p.pieces ? part[base + lane] : 0.0;
    const int n = p.pieces - base < 64 ? p.pieces - base : 64;
    for (int j = 0; j < n; ++j) {
      const double v = __shfl(mine, j);
      const double nx = pre + v;
      if (k < 0 && nx > target) k = base + j, before = pre;
      if (v > 0.0) klast = base + j;
      pre = nx;
    }
  }
  const bool none = k < 0;
  if (none) k = klast;
  const int lo = k * kRowPiece, hi = lo + kRowPiece < p.V ? lo + kRowPiece : p.V;
  const int seg = ((hi - lo + kSampleWaves - 1) / kSampleWaves + VEC - 1) / VEC * VEC;
  if constexpr (VEC == 4) {
    segment_pass<4, 2>(
        lo, hi, seg, wsum, [&](int v) { return *reinterpret_cast<const float4 *>(dist + v); },
        [&](int, const float4 &x, double &a) { a += ((double)x.x + (double)x.y) + ((double)x.z + (double)x.w); });
  } else {
    segment_pass<1, 8>(
        lo, hi, seg, wsum, [&](int v) { return dist[v]; }, [&](int, float x, double &a) { a += (double)x; });
  }
  draw_in_range(dist, lo, hi, seg, wsum, before, target, none, out);
}

template <int VEC>
__global__ void __launch_bounds__(kSampleThreads) sample_kernel(const SampleParams p) {
  __shared__ double wsum[kSampleWaves];
  __shared__ int32_t s_parent[kSampleTreeLds], s_token[kSampleTreeLds];
  __shared__ float s_u[kSampleTreeLds];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int t0 = p.cu_T[b];
  const int T = p.cu_T[b + 1] - t0;
  if (T <= 0) {
    if (tid == 0) p.path_len[b] = 0, p.next_token[b] = -1;
    return;
  }
  // the tree's words, read once (the walk is a chain of dependent reads of them); a tree too long for that is
  // walked in global memory
  const int32_t *parent = p.parent + t0, *token = p.token + t0;
  const float *u = p.u + t0;
  if (T <= kSampleTreeLds) {
    for (int i = tid; i < T; i += kSampleThreads) s_parent[i] = parent[i], s_token[i] = token[i], s_u[i] = u[i];
    parent = s_parent, token = s_token, u = s_u;
    __syncthreads();
  }
  const int V = p.V;
  const int seg = ((V + kSampleWaves - 1) / kSampleWaves + VEC - 1) / VEC * VEC;
  float *const r = p.residual + (size_t)b * V;
  int cur = 0, len = 1;
  if (tid == 0) p.path[(size_t)b * p.max_path] = 0;
  const float *dist;  // what the next test or the last draw reads: the current node's target row, or the residual
  double Z;
  const bool ahead = p.rowpart != nullptr && t0 + T <= p.sum_T;  // this tree's row sums were made ahead of the walk
  bool segments;  // wsum holds the segments' sums of dist (the last draw starts from them)
  auto flag_sequence = [&]() {
    if (tid == 0 && p.err_flag) atomicCAS(p.err_flag, 0, 1 + b);
  };
  // the first child of `of` behind node `after` that carries a token (others are flagged and passed over: never
  // accepted, and they leave the residual alone), or -1; 64 candidates at a time, every wave finds the same one
  auto next_child = [&](int of, int after) -> int {
    for (int base = after + 1; base < T; base += 64) {
      const int i = base + lane;
      unsigned long long kids = __ballot(i < T && parent[i] == of);
      while (kids) {
        const int c = base + __builtin_ctzll(kids);
        kids &= kids - 1;
        const int x = token[c];
        if (x >= 0 && x < V) return c;
        flag_sequence();
      }
    }
    return -1;
  };
  while (true) {
    dist = p.p + (size_t)(t0 + cur) * V;
    const float *q = p.q + (size_t)(t0 + cur) * V;
    // the first child and the two entries its test reads: requested before the row's sum, used after it
    int c = len < p.max_path ? next_child(cur, cur) : -1;
    float rx0 = 0.f, qx = 0.f;
    if (c >= 0 && ahead) rx0 = p.first[2 * (size_t)(t0 + c)], qx = p.first[2 * (size_t)(t0 + c) + 1];
    else if (c >= 0) rx0 = dist[token[c]], qx = q[token[c]];
    if (p.unit_rows) Z = 1.0, segments = false;
    else if (ahead) Z = summed_ahead(p, t0 + cur), segments = false;
    else Z = row_sum<VEC>(V, seg, wsum, dist), segments = true;
    double rx = (double)rx0;
    bool accepted = false;
    while (c >= 0) {
      if (rx > 0.0 && (double)u[c] * (double)qx * Z <= rx) {
        cur = c;
        if (tid == 0) p.path[(size_t)b * p.max_path + len] = c;
        ++len;
        accepted = true;
        break;
      }
      // rejected: the residual max(0, r - Z q), unnormalised, and its sum; the next child's entry of the draft's
      // row (which stays as it is) is requested before the pass
      const int cn = next_child(cur, c);
      const int xn = cn >= 0 ? token[cn] : 0;
      if (cn >= 0) qx = q[xn];
      __syncthreads();  // every thread has read what it needs of the row before the residual is overwritten in place
      const double Zn = residual_pass<VEC>(V, seg, wsum, dist, q, Z, r);
      if (!(Zn > 0.0)) {
        // q was not a distribution the child could have been drawn from: flagged; the walk ends here
        flag_sequence();
        if (tid == 0) p.path_len[b] = len, p.next_token[b] = -1;
        return;
      }
      Z = Zn;
      dist = r;
      segments = true;
      c = cn;
      if (c >= 0) rx = (double)r[xn];
    }
    if (!accepted) break;
  }
  if (tid == 0) p.path_len[b] = len;
  // (the last draw divides by the sum of what it draws from: a row that was taken as summing to one is summed here --
  // from its pieces where those were made ahead -- and one whose pieces were not made ahead is passed over)
  if (!segments && ahead) return draw_in_piece<VEC>(p, t0 + cur, dist, summed_ahead(p, t0 + cur), (double)p.u_final[b], wsum, &p.next_token[b]);
  if (!segments) Z = row_sum<VEC>(V, seg, wsum, dist);
  // The last token: the smallest v whose cumulative weight exceeds u_final * Z.  The segments' sums of the pass
  // that produced Z say which segment holds it.
  draw_in_range(dist, 0, V, seg, wsum, 0.0, (double)p.u_final[b] * Z, false, &p.next_token[b]);
}

// ---- the same walk with the vocabulary of a sequence spread over W workgroups ----
// A sequence's passes wait for one another, and one workgroup streams a row at what one compute unit can (about
// 45 GB/s): with few sequences the chip idles.  Here workgroup w of a sequence's W takes the w-th slice of every
// row.  After its part of a pass it publishes its partial sum (and, after a residual pass, the residual's entry of
// the next child's token, if that lies in its slice), arrives at a counter, and waits for the W arrivals; then
// every workgroup adds the W partial sums in the same order and takes the same decision.  The wait is bounded:
// a workgroup that does not see the others within about a second flags the sequence and leaves (the launch keeps
// W x B within what the chip holds at once, so this happens only if something else is wrong).
constexpr int kCoopMaxW = 16;
constexpr int kCoopSpins = 1 << 20;

struct CoopParams {
  SampleParams s;
  int W;
  int arrivals;  // arrivals a wait expects: W (one more in the test of the bound: then no wait ever completes)
  int spins;     // polls after which a wait gives up
  int *sync;     // [B * 32]: one arrival counter per sequence, 128 bytes apart, zero at kernel start
  double *xchg;  // [B][2][kCoopMaxW + 1]: partial sums of the pass (two buffers in turn), and the exchanged entry
};

__global__ void zero_sync_kernel(int *sync, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) sync[i] = 0;
}

__device__ __forceinline__ void publish(double *dst, double x) {
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(dst), (unsigned long long)__double_as_longlong(x), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // written through before this thread goes on to the barrier
}
__device__ __forceinline__ double fetch(const double *src) {
  return __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<const unsigned long long *>(src), __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT));
}

template <int VEC>
__global__ void __launch_bounds__(kSampleThreads) sample_coop_kernel(const CoopParams cp) {
  const SampleParams &p = cp.s;
  __shared__ double wsum[kSampleWaves];
  __shared__ double s_part[kCoopMaxW + 1];
  __shared__ int s_abort;
  __shared__ int32_t s_parent[kSampleTreeLds], s_token[kSampleTreeLds];
  __shared__ float s_u[kSampleTreeLds];
  const int W = cp.W;
  const int b = blockIdx.x / W, w = blockIdx.x % W, tid = threadIdx.x, lane = tid & 63;
  const int t0 = p.cu_T[b];
  const int T = p.cu_T[b + 1] - t0;
  if (T <= 0) {
    if (w == 0 && tid == 0) p.path_len[b] = 0, p.next_token[b] = -1;
    return;
  }
  const int32_t *parent = p.parent + t0, *token = p.token + t0;
  const float *u = p.u + t0;
  if (T <= kSampleTreeLds) {
    for (int i = tid; i < T; i += kSampleThreads) s_parent[i] = parent[i], s_token[i] = token[i], s_u[i] = u[i];
    parent = s_parent, token = s_token, u = s_u;
  }
  if (tid == 0) s_abort = 0;
  __syncthreads();
  const int V = p.V;
  // this workgroup's slice of every row, and the waves' segments of it
  const int slice = ((V + W - 1) / W + VEC - 1) / VEC * VEC;
  const int lo = w * slice < V ? w * slice : V, hi = lo + slice < V ? lo + slice : V;
  const int seg = ((hi - lo + kSampleWaves - 1) / kSampleWaves + VEC - 1) / VEC * VEC;
  float *const r = p.residual + (size_t)b * V;
  int *const ctr = cp.sync + b * 32;
  double *const xbase = cp.xchg + (size_t)b * 2 * (kCoopMaxW + 1);
  int epoch = 0;

  // sum of the W partial sums, the same in every thread of every workgroup of the sequence; s_part[0 .. W-1] keeps
  // them, s_part[W] what was exchanged with them.  Returns a negative number if the others did not arrive.
  auto group_sum = [&](double local) -> double {
    double *x = xbase + (epoch & 1) * (kCoopMaxW + 1);
    ++epoch;
    if (tid == 0) publish(x + w, local);
    __syncthreads();  // (the thread that published the exchanged entry has waited for its store too)
    if (tid == 0) {
      __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int target = epoch * cp.arrivals;
      int spins = 0;
      while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
        __builtin_amdgcn_s_sleep(2);
        if (++spins > cp.spins) {
          s_abort = 1;
          break;
        }
      }
    }
    __syncthreads();
    if (s_abort) return -1.0;
    if (tid <= W) s_part[tid] = fetch(x + (tid < W ? tid : kCoopMaxW));
    __syncthreads();
    double z = 0.0;
    for (int i = 0; i < W; ++i) z += s_part[i];
    return z;
  };
  auto leave_flagged = [&]() {
    if (tid == 0 && p.err_flag) atomicCAS(p.err_flag, 0, 1 + b);
  };
  // the first child of `of` behind node `after` that carries a token (others are flagged and passed over), or -1
  auto next_child = [&](int of, int after) -> int {
    for (int base = after + 1; base < T; base += 64) {
      const int i = base + lane;
      unsigned long long kids = __ballot(i < T && parent[i] == of);
      while (kids) {
        const int c = base + __builtin_ctzll(kids);
        kids &= kids - 1;
        const int x = token[c];
        if (x >= 0 && x < V) return c;
        leave_flagged();
      }
    }
    return -1;
  };

  int cur = 0, len = 1;
  if (w == 0 && tid == 0) p.path[(size_t)b * p.max_path] = 0;
  const float *dist;
  double Z;
  // the sum of a row from the workgroups' sums of their slices (negative: the others did not arrive)
  auto row_total = [&](const float *row) -> double {
    double local;
    if constexpr (VEC == 4) {
      local = segment_pass<4, 8>(
          lo, hi, seg, wsum, [&](int v) { return *reinterpret_cast<const float4 *>(row + v); },
          [&](int, const float4 &t, double &x) { x += ((double)t.x + (double)t.y) + ((double)t.z + (double)t.w); });
    } else {
      local = segment_pass<1, 8>(
          lo, hi, seg, wsum, [&](int v) { return row[v]; }, [&](int, float t, double &x) { x += (double)t; });
    }
    return group_sum(local);
  };
  const bool ahead = p.rowpart != nullptr && t0 + T <= p.sum_T;  // this tree's row sums were made ahead of the walk
  bool segments;  // wsum and s_part hold the sums of dist's segments and slices (the last draw starts from them)
  while (true) {
    const float *prow = p.p + (size_t)(t0 + cur) * V;
    const float *q = p.q + (size_t)(t0 + cur) * V;
    dist = prow;
    double local;
    // the first child and the two entries its test reads: requested before the row's sum, used after it
    int c = len < p.max_path ? next_child(cur, cur) : -1;
    float rx0 = 0.f, qx = 0.f;
    if (c >= 0 && ahead) rx0 = p.first[2 * (size_t)(t0 + c)], qx = p.first[2 * (size_t)(t0 + c) + 1];
    else if (c >= 0) rx0 = prow[token[c]], qx = q[token[c]];
    if (p.unit_rows) Z = 1.0, segments = false;
    else if (ahead) Z = summed_ahead(p, t0 + cur), segments = false;
    else Z = row_total(prow), segments = true;
    if (Z < 0.0) return leave_flagged();
    bool accepted = false;
    {
      double rx = (double)rx0;
      while (c >= 0) {
        if (rx > 0.0 && (double)u[c] * (double)qx * Z <= rx) {
          cur = c;
          if (w == 0 && tid == 0) p.path[(size_t)b * p.max_path + len] = c;
          ++len;
          accepted = true;
          break;
        }
        // rejected: the residual max(0, r - Z q) over this workgroup's slice; the entry of the next child's token
        // goes to the others with the partial sum
        const int cn = next_child(cur, c);
        const int xn = cn >= 0 ? token[cn] : -1;
        if (cn >= 0) qx = q[xn];  // (the draft's row stays as it is: requested before the pass)
        double *xslot = xbase + (epoch & 1) * (kCoopMaxW + 1) + kCoopMaxW;
        const float *from = dist;
        const double Zq = Z;
        auto one = [&](float pv, float qv) {
          const double d = (double)pv - Zq * (double)qv;
          return d > 0.0 ? (float)d : 0.f;
        };
        __syncthreads();  // every thread has read what it needs of the row before the slice is overwritten in place
        if constexpr (VEC == 4) {
          local = segment_pass<4, 4>(
              lo, hi, seg, wsum,
              [&](int v) {
                return Float4Pair{*reinterpret_cast<const float4 *>(from + v), *reinterpret_cast<const float4 *>(q + v)};
              },
              [&](int v, const Float4Pair &t, double &acc) {
                float4 o;
                o.x = one(t.a.x, t.c.x), o.y = one(t.a.y, t.c.y), o.z = one(t.a.z, t.c.z), o.w = one(t.a.w, t.c.w);
                *reinterpret_cast<float4 *>(r + v) = o;
                if (xn >= v && xn < v + 4) publish(xslot, (double)(xn == v ? o.x : xn == v + 1 ? o.y : xn == v + 2 ? o.z : o.w));
                acc += ((double)o.x + (double)o.y) + ((double)o.z + (double)o.w);
              });
        } else {
          local = segment_pass<1, 4>(
              lo, hi, seg, wsum, [&](int v) { return FloatPair{from[v], q[v]}; },
              [&](int v, const FloatPair &t, double &acc) {
                const float o = one(t.a, t.c);
                r[v] = o;
                if (v == xn) publish(xslot, (double)o);
                acc += (double)o;
              });
        }
        const double Zn = group_sum(local);
        if (Zn < 0.0) return leave_flagged();
        if (!(Zn > 0.0)) {
          // q was not a distribution the child could have been drawn from: flagged; the walk ends here
          leave_flagged();
          if (w == 0 && tid == 0) p.path_len[b] = len, p.next_token[b] = -1;
          return;
        }
        Z = Zn;
        dist = r;
        segments = true;
        rx = s_part[W];
        c = cn;
      }
    }
    if (!accepted) break;
  }
  if (w == 0 && tid == 0) p.path_len[b] = len;
  if (!segments && ahead) {  // (the walk ends at a node whose row was summed ahead: one workgroup draws, from one piece of the row)
    if (w == 0) draw_in_piece<VEC>(p, t0 + cur, dist, summed_ahead(p, t0 + cur), (double)p.u_final[b], wsum, &p.next_token[b]);
    return;
  }
  if (!segments) {  // (a row taken as summing to one, its pieces not made ahead: the last draw sums it)
    Z = row_total(dist);
    if (Z < 0.0) return leave_flagged();
  }
  // The last token: the workgroup whose slice holds the smallest v with cumulative weight above u_final * Z, then
  // the wave of it whose segment does.
  const double target = (double)p.u_final[b] * Z;
  int claim = -1, last_heavy = 0;
  double before = 0.0;
  {
    double pre = 0.0;
    for (int i = 0; i < W; ++i) {
      const double nx = pre + s_part[i];
      if (claim < 0 && nx > target) claim = i, before = pre;
      if (s_part[i] > 0.0) last_heavy = i;
      pre = nx;
    }
  }
  const bool none = claim < 0;  // (u_final was not below 1: the last token that has weight)
  if (none) claim = last_heavy;
  if (w == claim) draw_in_range(dist, lo, hi, seg, wsum, before, target, none, &p.next_token[b]);
}

// Workgroups per sequence: as many as keep the launch within one workgroup per compute unit (all of them resident at
// once, which the waits between passes rely on), at most 16, a power of two, slices of 4096 tokens or more, and
// one only for vocabularies below 48 K: a wait between passes costs about 4.5 us, what one workgroup needs for
// a pass over 32 K tokens (measured: V = 32000 30.6 us with one workgroup, 35.3 with eight).  With the row sums made
// ahead of the walk only refusals still cost a pass and its wait, and sharing pays from 16 K tokens on (V = 32000,
// B = 1: 28.4 us with four workgroups against 31.2 with one; B = 4: 24.8 against 34.0).  Negative: a status.
int sample_workgroups(const tva_sample_args *a, bool ahead) {
  if (a->workgroups_per_sequence < 0 || a->workgroups_per_sequence > kCoopMaxW) return TVA_INVALID_ARG;
  if (!a->workspace || a->workgroups_per_sequence == 1) return 1;
  if (((uintptr_t)a->workspace & 7) || a->workspace_bytes < (size_t)a->B * 512) return TVA_WORKSPACE_TOO_SMALL;
  int W = 1;
  const int shared_from = ahead ? 16384 : 49152;
  while (a->V >= shared_from && 2 * W <= kCoopMaxW && (int64_t)a->B * 2 * W <= 256 && a->V / (2 * W) >= 4096) W *= 2;
  if (a->workgroups_per_sequence > 1) {
    W = a->workgroups_per_sequence;
    if ((int64_t)a->B * W > 256) return TVA_UNSUPPORTED;  // more than the chip holds at once
  }
  return W;
}

// Row sums ahead of the walk: where the host gave the number of nodes, the workspace has room behind the waits'
// words, and all rows together are few enough bytes (40 MB: 5 .. 8 us with the whole chip, what the passes over two
// accepted nodes' rows cost one after the other).
constexpr int64_t kRowSumsMaxBytes = 40 << 20;
inline int row_pieces(int V) { return (V + kRowPiece - 1) / kRowPiece; }
inline size_t row_sums_offset(int B) { return (size_t)B * 512; }
bool sums_ahead(const tva_sample_args *a) {
  if (a->sum_T <= 0 || !a->workspace || ((uintptr_t)a->workspace & 7)) return false;
  if ((int64_t)a->sum_T * a->V * (int64_t)sizeof(float) > kRowSumsMaxBytes || a->sum_T > 65535) return false;
  return a->workspace_bytes >= row_sums_offset(a->B) + (size_t)a->sum_T * (row_pieces(a->V) * sizeof(double) + 2 * sizeof(float));
}

struct CommitParams {
  const int32_t *cu_T, *L, *path, *path_len, *cu_L, *page_table;
  const char *k_tree, *v_tree;
  char *k_cache, *v_cache;
  int32_t *L_out, *err_flag;
  int Hkv, D, max_path, page_size, max_pages;
  int64_t stride_page, stride_tok, stride_head;  // elements
  int64_t layer_cache, layer_tree;                // bytes between the tensors of consecutive layers (blockIdx.z)
};

__global__ void __launch_bounds__(256) commit_kernel(const CommitParams p) {
  const int j = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
  const int n = p.path_len[b];
  const int Lb = p.L[b];
  if (j == 0 && layer == 0 && threadIdx.x == 0 && p.L_out) p.L_out[b] = Lb + (n < p.max_path ? n : p.max_path);
  if (j >= n || Lb < 0) return;
  const int node = p.path[(size_t)b * p.max_path + j];
  if (node < 0 || node >= p.cu_T[b + 1] - p.cu_T[b]) {  // not a node of this tree: nothing is copied
    if (threadIdx.x == 0 && p.err_flag) atomicCAS(p.err_flag, 0, 1 + b);
    return;
  }
  const int64_t src_row = (int64_t)p.cu_T[b] + node;
  const int pos = Lb + j;
  int64_t dst;  // element offset of (position, head 0, d 0)
  bool room;
  if (p.page_table) {
    const int pi = pos / p.page_size;
    room = pi < p.max_pages;
    const int page = room ? p.page_table[(int64_t)b * p.max_pages + pi] : 0;
    dst = (int64_t)page * p.stride_page + (int64_t)(pos - pi * p.page_size) * p.stride_tok;
  } else {
    room = (int64_t)p.cu_L[b] + pos < p.cu_L[b + 1];
    dst = ((int64_t)p.cu_L[b] + pos) * p.stride_tok;
  }
  if (!room) {
    if (threadIdx.x == 0 && p.err_flag) atomicCAS(p.err_flag, 0, 1 + b);
    return;
  }
  // 16-byte pieces: piece q of head g; the tree tensors are packed [node, Hkv, D]
  const int per_head = p.D / 8;
  const int pieces = p.Hkv * per_head;
  for (int q = threadIdx.x; q < 2 * pieces; q += blockDim.x) {
    const bool is_v = q >= pieces;
    const int r = is_v ? q - pieces : q;
    const int g = r / per_head, e = (r - g * per_head) * 8;
    const char *src = (is_v ? p.v_tree : p.k_tree) + layer * p.layer_tree + ((src_row * p.Hkv + g) * p.D + e) * 2;
    char *out = (is_v ? p.v_cache : p.k_cache) + layer * p.layer_cache + (dst + (int64_t)g * p.stride_head + e) * 2;
    *reinterpret_cast<u32x4 *>(out) = *reinterpret_cast<const u32x4 *>(src);
  }
}

// Tree K/V already in the cache behind the L_b committed tokens (tree node i at position L_b + i):
// the accepted nodes are moved down to positions L_b, L_b + 1, ...  One workgroup per sequence; a
// thread owns the same 16-byte pieces of every row and takes the path in order.  Step j reads
// position L_b + path[j] >= L_b + j and writes L_b + j, so a later step never reads what an earlier
// one wrote, and a read that a later step overwrites comes first in the same thread's program order.
__global__ void __launch_bounds__(256) compact_kernel(const CommitParams p) {
  const int b = blockIdx.x, layer = blockIdx.y;
  const int n = p.path_len[b] < p.max_path ? p.path_len[b] : p.max_path;
  const int Lb = p.L[b];
  const int T = p.cu_T[b + 1] - p.cu_T[b];
  if (layer == 0 && threadIdx.x == 0 && p.L_out) p.L_out[b] = Lb + n;
  if (Lb < 0) return;
  const int per_head = p.D / 8;
  const int pieces = p.Hkv * per_head;
  auto row_offset = [&](int pos) -> int64_t {  // element offset of (position, head 0, d 0)
    if (p.page_table) {
      const int pi = pos / p.page_size;
      const int page = p.page_table[(int64_t)b * p.max_pages + pi];
      return (int64_t)page * p.stride_page + (int64_t)(pos - pi * p.page_size) * p.stride_tok;
    }
    return ((int64_t)p.cu_L[b] + pos) * p.stride_tok;
  };
  for (int j = 0; j < n; ++j) {
    const int node = p.path[(size_t)b * p.max_path + j];
    if (node < j || node >= T || (p.page_table && (Lb + node) / p.page_size >= p.max_pages)) {
      // not a path of this tree (entries rise at least as fast as their position): stop here
      if (threadIdx.x == 0 && p.err_flag) atomicCAS(p.err_flag, 0, 1 + b);
      return;
    }
    if (node == j) continue;  // already in place
    const int64_t src = row_offset(Lb + node), dst = row_offset(Lb + j);
    for (int q = threadIdx.x; q < 2 * pieces; q += blockDim.x) {
      const bool is_v = q >= pieces;
      const int r = is_v ? q - pieces : q;
      const int g = r / per_head, e = (r - g * per_head) * 8;
      char *base = (is_v ? p.v_cache : p.k_cache) + layer * p.layer_cache;
      const int64_t inner = (int64_t)g * p.stride_head + e;
      *reinterpret_cast<u32x4 *>(base + (dst + inner) * 2) = *reinterpret_cast<const u32x4 *>(base + (src + inner) * 2);
    }
  }
}

}  // namespace

extern "C" {

int tva_accept_greedy(const int32_t *parent, const int32_t *cu_T, const int32_t *draft_token,
                      const int32_t *target_token, int32_t B, int32_t max_path, int32_t *path, int32_t *path_len,
                      int32_t *next_token, void *stream) {
  if (B < 0 || max_path < 1) return TVA_INVALID_ARG;
  if (B == 0) return TVA_OK;
  if (!parent || !cu_T || !draft_token || !target_token || !path || !path_len || !next_token) return TVA_INVALID_ARG;
  (void)hipGetLastError();  // the status below is this launch's
  hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, (hipStream_t)stream, parent, cu_T, draft_token, target_token,
                     max_path, path, path_len, next_token);
  return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

static int accept_sampling_impl(const tva_sample_args *a, void *stream, int missing_arrivals, int spins);

int tva_accept_sampling(const tva_sample_args *a, void *stream) { return accept_sampling_impl(a, stream, 0, kCoopSpins); }

int tva_accept_sampling_wait_bound_test(const tva_sample_args *a, int32_t spins, void *stream) {
  if (!a || spins < 1 || spins > kCoopSpins || !a->workspace || a->workgroups_per_sequence < 2) return TVA_INVALID_ARG;
  return accept_sampling_impl(a, stream, 1, spins);
}

static int accept_sampling_impl(const tva_sample_args *a, void *stream, int missing_arrivals, int spins) {
  if (!a || a->B < 0 || a->V < 1 || a->max_path < 1) return TVA_INVALID_ARG;
  if (a->B == 0) return TVA_OK;
  if (!a->parent || !a->cu_T || !a->draft_token || !a->p_target || !a->q_draft || !a->u || !a->u_final || !a->residual ||
      !a->path || !a->path_len || !a->next_token)
    return TVA_INVALID_ARG;
  SampleParams p;
  p.parent = a->parent, p.cu_T = a->cu_T, p.token = a->draft_token;
  p.p = a->p_target, p.q = a->q_draft, p.u = a->u, p.u_final = a->u_final;
  p.residual = a->residual;
  p.path = a->path, p.path_len = a->path_len, p.next_token = a->next_token, p.err_flag = a->err_flag;
  p.V = a->V, p.max_path = a->max_path;
  p.rowpart = nullptr, p.first = nullptr, p.pieces = row_pieces(a->V), p.sum_T = 0;
  p.unit_rows = a->unit_rows != 0;
  // groups of four need every row to start on 16 bytes
  const bool vec = a->V % 4 == 0 && (((uintptr_t)a->p_target | (uintptr_t)a->q_draft | (uintptr_t)a->residual) & 15) == 0;
  if (a->sum_T < 0) return TVA_INVALID_ARG;
  const bool ahead = sums_ahead(a);
  const int W = sample_workgroups(a, ahead);
  if (W < 0) return W;
  (void)hipGetLastError();  // the status below is these launches'
  hipStream_t st = (hipStream_t)stream;
  if (ahead) {
    double *rowpart = reinterpret_cast<double *>(static_cast<char *>(a->workspace) + row_sums_offset(a->B));
    int *sync = static_cast<int *>(a->workspace);
    const int n_sync = W > 1 ? a->B * 32 : 0;  // (the arrival counters of the walk start at zero)
    float *first = reinterpret_cast<float *>(rowpart + (size_t)a->sum_T * p.pieces);
    const dim3 grid(p.pieces + 1, a->sum_T);
    if (vec)
      hipLaunchKernelGGL(row_sums_kernel<4>, grid, dim3(kRowPieceThreads), 0, st, a->p_target, a->cu_T, a->B, a->V, rowpart, sync, n_sync,
                         a->q_draft, a->parent, a->draft_token, first);
    else
      hipLaunchKernelGGL(row_sums_kernel<1>, grid, dim3(kRowPieceThreads), 0, st, a->p_target, a->cu_T, a->B, a->V, rowpart, sync, n_sync,
                         a->q_draft, a->parent, a->draft_token, first);
    p.rowpart = rowpart, p.first = first, p.sum_T = a->sum_T;
  }
  if (W == 1) {
    if (vec) hipLaunchKernelGGL(sample_kernel<4>, dim3(a->B), dim3(kSampleThreads), 0, st, p);
    else hipLaunchKernelGGL(sample_kernel<1>, dim3(a->B), dim3(kSampleThreads), 0, st, p);
  } else {
    CoopParams cp;
    cp.s = p, cp.W = W, cp.arrivals = W + missing_arrivals, cp.spins = spins;
    cp.sync = static_cast<int *>(a->workspace);
    cp.xchg = reinterpret_cast<double *>(static_cast<char *>(a->workspace) + (size_t)a->B * 128);
    // the arrival counters start at zero (a kernel, not a memset node: the call may be captured into a graph)
    if (!ahead) hipLaunchKernelGGL(zero_sync_kernel, dim3((a->B * 32 + 255) / 256), dim3(256), 0, st, cp.sync, a->B * 32);
    if (vec) hipLaunchKernelGGL(sample_coop_kernel<4>, dim3(a->B * W), dim3(kSampleThreads), 0, st, cp);
    else hipLaunchKernelGGL(sample_coop_kernel<1>, dim3(a->B * W), dim3(kSampleThreads), 0, st, cp);
  }
  return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

size_t tva_sample_workspace_bytes(int32_t B) { return B < 0 ? (size_t)-1 : (size_t)B * 512; }

size_t tva_sample_workspace_bytes_rows(int32_t B, int32_t sum_T, int32_t V) {
  if (B < 0 || sum_T < 0 || V < 1) return (size_t)-1;
  return row_sums_offset(B) + (size_t)sum_T * (row_pieces(V) * sizeof(double) + 2 * sizeof(float));  // sums, then entries
}

size_t tva_sizeof_sample_args(void) { return sizeof(tva_sample_args); }

int tva_commit_path(const tva_commit_args *a, void *stream) {
  if (!a || a->B < 0 || a->Hkv < 1 || a->D < 8 || a->D % 8 || a->max_path < 1) return TVA_INVALID_ARG;
  if (a->B == 0) return TVA_OK;
  if (!a->cu_T || !a->L || !a->path || !a->path_len || !a->k_cache || !a->v_cache) return TVA_INVALID_ARG;
  if ((a->k_tree == nullptr) != (a->v_tree == nullptr)) return TVA_INVALID_ARG;
  const bool in_cache = a->k_tree == nullptr;
  const bool dense = a->cu_L != nullptr, paged = a->page_table != nullptr;
  if (dense == paged) return TVA_INVALID_ARG;
  if (paged && (a->page_size <= 0 || a->max_pages <= 0)) return TVA_INVALID_ARG;
  if ((a->stride_page | a->stride_tok | a->stride_head) % 8) return TVA_INVALID_ARG;
  if (a->stride_page < 0 || a->stride_tok < 0 || a->stride_head < 0) return TVA_INVALID_ARG;
  if (a->L_out == a->L) return TVA_INVALID_ARG;
  if (a->n_layers < 0 || a->layer_stride_cache < 0 || a->layer_stride_tree < 0 ||
      (a->layer_stride_cache | a->layer_stride_tree) % 8)
    return TVA_INVALID_ARG;
  const int layers = a->n_layers > 0 ? a->n_layers : 1;
  if (a->B > 65535 || layers > 65535) return TVA_UNSUPPORTED;
  CommitParams p;
  p.cu_T = a->cu_T; p.L = a->L; p.path = a->path; p.path_len = a->path_len;
  p.cu_L = a->cu_L; p.page_table = a->page_table;
  p.k_tree = (const char *)a->k_tree; p.v_tree = (const char *)a->v_tree;
  p.k_cache = (char *)a->k_cache; p.v_cache = (char *)a->v_cache;
  p.L_out = a->L_out; p.err_flag = a->err_flag;
  p.Hkv = a->Hkv; p.D = a->D; p.max_path = a->max_path;
  p.page_size = paged ? a->page_size : 1; p.max_pages = a->max_pages;
  p.stride_head = a->stride_head ? a->stride_head : a->D;
  p.stride_tok = a->stride_tok ? a->stride_tok : (int64_t)a->Hkv * a->D;
  p.stride_page = a->stride_page ? a->stride_page : (int64_t)p.page_size * p.stride_tok;
  p.layer_cache = a->layer_stride_cache * 2, p.layer_tree = a->layer_stride_tree * 2;
  (void)hipGetLastError();
  if (in_cache) hipLaunchKernelGGL(compact_kernel, dim3(a->B, layers), dim3(256), 0, (hipStream_t)stream, p);
  else hipLaunchKernelGGL(commit_kernel, dim3(a->max_path, a->B, layers), dim3(256), 0, (hipStream_t)stream, p);
  return hipPeekAtLastError() == hipSuccess ? TVA_OK : TVA_HIP_ERROR;
}

size_t tva_sizeof_commit_args(void) { return sizeof(tva_commit_args); }

}  // extern "C"
