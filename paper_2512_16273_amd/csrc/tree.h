// tslt_verify_tree: token-tree verification (Algorithm 8) with multi-candidate verification
// (Algorithm 5) at every non-leaf node.  Nodes are stored breadth-first (Section 4.1).
//
// Kernel M, one workgroup per (tree, non-leaf node): eval_row_on_set over the node's target row, then
// Algorithm 5 on the sparse representation.  With a sparse q_hat the distribution p^(i) is a vector
// a on the set and a scalar multiple c of p outside it, and the update p^(i+1) = norm(max(0, p^(i) -
// q_hat)) is a <- max(0, a - q_hat) / Z, c <- c / Z with Z = sum(max(0, a - q_hat)) + c * p_out: one
// dense pass per node, O(k * K) work for the k candidates.
// Kernel W, one wave per tree: the new-sequence search -- walk from the root through accepted
// children, write the accepted prefix, remember the node at which the walk stops.
// Kernels S and F: fp64 sweep and inverse CDF (rowops.h) for every node whose output has to be
// sampled -- a non-leaf node whose k candidates were all rejected draws from P^(k+1), a leaf from its
// target distribution.  Either every such node of the tree is sampled (node outputs requested) or
// only the node that ends the verified path.
#pragma once
#include "rowops.h"

namespace tslt {

constexpr int kMaxTreeDepth = 16;
constexpr int kMaxBranch = 16;

struct TreeParams {
  const void* target;
  int64_t B, V, row_stride;
  int n_nodes, n_int, depth;
  int expansion[kMaxTreeDepth];
  int offsets[kMaxTreeDepth + 2];     // first node of every layer; offsets[depth + 1] = n_nodes
  float rT, k2;
  const int32_t* q_idx;
  const float* q_logit;
  const int32_t* q_count;
  int k_cap;
  int wor;                // candidates were drawn without replacement: stage proposals are renormalised
  const int32_t* cand_tokens;
  const float* u_accept;
  const float* u_resample;
  int32_t* out_node_token;
  int32_t* out_node_slot;
  int32_t* out_seq;
  int32_t* out_len;
  float* out_ratio;
  float* out_beta;        // [B, n_nodes - 1] stage acceptance rate sum_x min(q^(i), p^(i)) of every tested candidate
  int32_t* status;
  // workspace
  int32_t* node_state;    // [B, n_int] 0 all candidates rejected, 1 a child accepted, 2 row unusable
  int32_t* node_slot;     // [B, n_int] accepted child number or -1
  int32_t* node_stages;   // [B, n_int] residual updates applied (candidates present and rejected)
  int32_t* node_status;   // [B, n_int]
  int32_t* term_node;     // [B] node at which the walk stops
  int32_t* seq_status;    // [B] status accumulated over the tree
  SegResult* segs;        // [B, tasks, n_seg + 2]
  double* subs;           // [B, tasks, n_seg, kSubChunks]
  int tasks;              // rows sampled per tree: n_nodes (all nodes) or 1 (path only)
  int all_nodes;
  int n_seg, n_seg_grid;
  int use_table;          // kernel S sums bf16 rows through the exp table
};

inline size_t tree_workspace_bytes(int64_t B, int64_t n_nodes, int64_t V, bool all_nodes) {
  const size_t n_seg = size_t(row_segments(V));
  const size_t tasks = all_nodes ? size_t(n_nodes) : 1;
  return align256(size_t(B) * n_nodes * 4) * 4 + align256(size_t(B) * 4) * 2 +
         align256(size_t(B) * tasks * (n_seg + 2) * sizeof(SegResult)) +
         align256(size_t(B) * tasks * n_seg * kSubChunks * sizeof(double));
}
inline void tree_carve_workspace(TreeParams& p, void* ws) {
  char* w = reinterpret_cast<char*>(ws);
  p.n_seg = row_segments(p.V);
  const size_t per = align256(size_t(p.B) * p.n_nodes * 4);
  p.node_state = reinterpret_cast<int32_t*>(w); w += per;
  p.node_slot = reinterpret_cast<int32_t*>(w); w += per;
  p.node_stages = reinterpret_cast<int32_t*>(w); w += per;
  p.node_status = reinterpret_cast<int32_t*>(w); w += per;
  p.term_node = reinterpret_cast<int32_t*>(w); w += align256(size_t(p.B) * 4);
  p.seq_status = reinterpret_cast<int32_t*>(w); w += align256(size_t(p.B) * 4);
  p.segs = reinterpret_cast<SegResult*>(w); w += align256(size_t(p.B) * p.tasks * (p.n_seg + 2) * sizeof(SegResult));
  p.subs = reinterpret_cast<double*>(w);
}

template <typename T> __device__ __forceinline__ const void* tree_row(const TreeParams& p, int64_t b, int node) {
  return reinterpret_cast<const char*>(p.target) +
         (size_t(b) * p.n_nodes + node) * size_t(p.row_stride) * ElemTraits<T>::kBytes;
}
__device__ __forceinline__ int tree_layer(const TreeParams& p, int node) {
  int l = 0;
  while (l < p.depth && node >= p.offsets[l + 1]) ++l;
  return l;
}
// first child of a non-leaf node: the i-th node of layer l owns nodes i*k .. i*k + k-1 of layer l+1
__device__ __forceinline__ int tree_first_child(const TreeParams& p, int node, int layer) {
  return p.offsets[layer + 1] + (node - p.offsets[layer]) * p.expansion[layer];
}

// ---------------------------------------------------------------------------------------------
// Kernel M: Algorithm 5 at one non-leaf node
// ---------------------------------------------------------------------------------------------
// Algorithm 5 at non-leaf node `node` of tree b, by all threads of a workgroup.  Writes the node's state,
// accepted child, number of updates and status to the workspace and the ratios of the candidates it
// tested; returns the state (0 all candidates rejected, 1 a child accepted, 2 row unusable) and, in
// `slot`, the accepted child.
template <typename T>
__device__ __forceinline__ int mcveri_node(const TreeParams& p, int64_t b, int node, VerifyShared& sh, int& slot, int& st) {
  const int tid = threadIdx.x;
  const int layer = tree_layer(p, node);
  const int k = p.expansion[layer];
  const int c0 = tree_first_child(p, node, layer);           // children are nodes c0 .. c0 + k - 1
  const int32_t* cand = p.cand_tokens + size_t(b) * (p.n_nodes - 1) + (c0 - 1);
  const float* u_acc = p.u_accept + size_t(b) * (p.n_nodes - 1) + (c0 - 1);
  float* ratio_out = p.out_ratio ? p.out_ratio + size_t(b) * (p.n_nodes - 1) + (c0 - 1) : nullptr;
  float* beta_out = p.out_beta ? p.out_beta + size_t(b) * (p.n_nodes - 1) + (c0 - 1) : nullptr;
  const void* row = tree_row<T>(p, b, node);
  const RowSplit rs = split_row<T>(row, p.V);
  const int64_t r = b * p.n_int + node;
  int count = p.q_count[r];
  count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
  double a_s[kSetPer], q_s[kSetPer], p_out;
  int yi[kSetPer];
  bool ok;
  eval_row_on_set<T>(row, rs, p.V, p.rT, p.k2, p.q_idx + size_t(r) * p.k_cap, p.q_logit + size_t(r) * p.k_cap, count, sh,
                     a_s, q_s, yi, p_out, ok, st);
  if (ratio_out && tid < k) ratio_out[tid] = NAN;              // candidates that are never tested
  if (beta_out && tid < k) beta_out[tid] = NAN;
  int accepted = -1, stages = 0;
  if (ok) {
    double c = 1.0;
    double qscale = 1.0, removed = 0.0;       // the stage's proposal is q_s * qscale
    for (int i = 0; i < k; ++i) {
      const int x = cand[i];
      if (x < 0) continue;                                      // absent candidate (block-uniform)
      if (tid == 0) { sh.bcast_d[0] = -1.0; sh.bcast_d[1] = 0.0; sh.bcast_i[0] = 0; }
      __syncthreads();
      int mine = -1;
#pragma unroll
      for (int q = 0; q < kSetPer; ++q)
        if (yi[q] == x && q_s[q] > 0.0 && atomicCAS(&sh.bcast_i[0], 0, 1) == 0) {
          sh.bcast_d[0] = a_s[q] / (q_s[q] * qscale);
          sh.bcast_d[1] = q_s[q];
          mine = q;
        }
      __syncthreads();
      const double ratio = sh.bcast_d[0];
      const double q_x = sh.bcast_d[1];
      const bool found = sh.bcast_i[0] != 0;
      __syncthreads();
      if (!found) st |= 4;
      if (ratio_out && tid == 0) ratio_out[i] = float(ratio);
      if (beta_out) {
        // Section 4.3's beta^(i): the mass that the stage's proposal and p^(i) share (all of it lies on the set)
        double shared = 0.0;
#pragma unroll
        for (int q = 0; q < kSetPer; ++q) {
          const double qq = q_s[q] * qscale;
          shared += (yi[q] >= 0) ? (a_s[q] < qq ? a_s[q] : qq) : 0.0;
        }
        shared = block_sum_f64<kWaves>(shared, sh.red);
        if (tid == 0) beta_out[i] = float(shared);
      }
      const double bound = ratio < 1.0 ? ratio : 1.0;
      if (found && double(u_acc[i]) < bound) { accepted = i; break; }
      // rejected: p <- norm(max(0, p - q)), q the proposal of this stage
      double part = 0.0;
#pragma unroll
      for (int q = 0; q < kSetPer; ++q) {
        const double d = a_s[q] - q_s[q] * qscale;
        a_s[q] = (yi[q] >= 0 && d > 0.0) ? d : 0.0;
        part += a_s[q];
      }
      const double Z = block_sum_f64<kWaves>(part, sh.red) + c * p_out;
      if (Z > 0.0) {
        const double inv_Z = 1.0 / Z;
#pragma unroll
        for (int q = 0; q < kSetPer; ++q) a_s[q] *= inv_Z;
        c *= inv_Z;
      }
      if (p.wor && found) {
        // drawn without replacement: x leaves the urn and what is left is renormalised
#pragma unroll
        for (int q = 0; q < kSetPer; ++q)
          if (q == mine) q_s[q] = 0.0;
        removed += q_x;
        const double rest = 1.0 - removed;
        qscale = rest > 0.0 ? 1.0 / rest : 0.0;
      }
      ++stages;
    }
  }
  const int state = !ok ? 2 : (accepted >= 0 ? 1 : 0);
  if (tid == 0) {
    p.node_state[r] = state;
    p.node_slot[r] = accepted;
    p.node_stages[r] = stages;
    p.node_status[r] = st;
  }
  slot = accepted;
  return state;
}

template <typename T>
__global__ __launch_bounds__(kBlock, kAccWavesPerSimd) void tree_mcveri_kernel(const TreeParams p) {
  __shared__ VerifyShared sh;
  const int64_t b = blockIdx.x / p.n_int;
  const int node = int(blockIdx.x - b * p.n_int);
  int slot, st;
  mcveri_node<T>(p, b, node, sh, slot, st);
}

// ---------------------------------------------------------------------------------------------
// Kernel L (only the verified path is wanted): one workgroup per tree walks from the root, running
// Algorithm 5 at each node it reaches and descending into the accepted child, so that depth + 1 target rows
// are read per tree instead of one per non-leaf node.  Uniforms are indexed by node, so the result is the
// one the all-nodes kernels give.  Leaves the stopping node to kernels S and F.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void tree_lazy_walk_kernel(const TreeParams p) {
  __shared__ VerifyShared sh;
  const int tid = threadIdx.x;
  const int64_t b = blockIdx.x;
  for (int i = tid; i < p.n_nodes - 1; i += kBlock) {
    if (p.out_ratio) p.out_ratio[size_t(b) * (p.n_nodes - 1) + i] = NAN;
    if (p.out_beta) p.out_beta[size_t(b) * (p.n_nodes - 1) + i] = NAN;
  }
  __syncthreads();
  int32_t* seq = p.out_seq + size_t(b) * (p.depth + 1);
  int node = 0, layer = 0, len = 0, st_all = 0;
  while (node < p.n_int) {
    int slot, st;
    const int state = mcveri_node<T>(p, b, node, sh, slot, st);
    st_all |= st;
    __syncthreads();
    if (state != 1) break;
    const int child = tree_first_child(p, node, layer) + slot;
    if (tid == 0) seq[len] = p.cand_tokens[size_t(b) * (p.n_nodes - 1) + (child - 1)];
    ++len;
    node = child;
    ++layer;
  }
  if (tid == 0) {
    p.term_node[b] = node;                 // its output is the last token; kernel F writes it
    p.out_len[b] = len + 1;
    for (int i = len + 1; i <= p.depth; ++i) seq[i] = -1;
    p.seq_status[b] = st_all;
  }
}


// ---------------------------------------------------------------------------------------------
// Kernel W: the new-sequence search, one wave per tree
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void tree_walk_kernel(const TreeParams p) {
  const int64_t b = blockIdx.x;
  const int lane = threadIdx.x;
  int st = 0;
  for (int n = lane; n < p.n_int; n += 64) st |= p.node_status[b * p.n_int + n];
  st = wave_or_i32(st);
  if (lane == 0) {
    int node = 0, layer = 0, len = 0;
    int32_t* seq = p.out_seq + size_t(b) * (p.depth + 1);
    while (node < p.n_int && p.node_state[b * p.n_int + node] == 1) {
      const int child = tree_first_child(p, node, layer) + p.node_slot[b * p.n_int + node];
      seq[len++] = p.cand_tokens[size_t(b) * (p.n_nodes - 1) + (child - 1)];
      node = child;
      ++layer;
    }
    p.term_node[b] = node;                 // its output is the last token; kernel F writes it
    p.out_len[b] = len + 1;
    for (int i = len + 1; i <= p.depth; ++i) seq[i] = -1;
    p.seq_status[b] = st;
  }
}

// ---------------------------------------------------------------------------------------------
// Kernels S and F: sample the output of the nodes that need it
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void tree_sweep_kernel(const TreeParams p) {
  __shared__ VerifyShared sh;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  double* table = nullptr;
  if constexpr (ExpTab<T>::kHas) {
    if (p.use_table) {
      table = reinterpret_cast<double*>(dyn_lds);
      build_exp_table<T>(table, p.rT, kBlock);
      __syncthreads();
    }
  }
  const int64_t n_items = p.B * p.tasks * p.n_seg_grid;
  for (int64_t item = blockIdx.x; item < n_items; item += gridDim.x) {      // persistent workgroups
    const int64_t task = item / p.n_seg_grid;                    // (b, t)
    const int seg = int(item - task * p.n_seg_grid);
    const int64_t b = task / p.tasks;
    const int node = p.all_nodes ? int(task - b * p.tasks) : p.term_node[b];
    if (node < p.n_int && p.node_state[b * p.n_int + node] != 0) continue;   // accepted a child, or unusable
    const void* row = tree_row<T>(p, b, node);
    const RowSplit rs = split_row<T>(row, p.V);
    // non-leaf rows were validated by kernel M; leaves are seen here for the first time
    sweep_group<T>(row, rs, seg, node >= p.n_int, p.rT, table, p.segs + size_t(task) * (p.n_seg + 2),
                     p.subs + size_t(task) * p.n_seg * kSubChunks, sh);
    __syncthreads();
  }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void tree_finish_kernel(const TreeParams p) {
  __shared__ VerifyShared sh;
  __shared__ double item_val[kMaxItems];
  const int tid = threadIdx.x;
  const int64_t task = blockIdx.x;
  const int64_t b = task / p.tasks;
  const int node = p.all_nodes ? int(task - b * p.tasks) : p.term_node[b];
  const bool leaf = node >= p.n_int;
  const int64_t r = b * p.n_int + (leaf ? 0 : node);
  const int state = leaf ? 0 : p.node_state[r];
  int token = -1, slot = -1, st = 0;
  if (state == 1) {
    // an accepted child: the node's output is that candidate
    slot = p.node_slot[r];
    const int layer = tree_layer(p, node);
    token = p.cand_tokens[size_t(b) * (p.n_nodes - 1) + (tree_first_child(p, node, layer) + slot - 1)];
  } else {
    FinishArgs a;
    a.row = tree_row<T>(p, b, node);
    a.rs = split_row<T>(a.row, p.V);
    a.n_seg_row = int((a.rs.nvec + kSegVecsTotal - 1) / kSegVecsTotal);
    a.V = p.V;
    a.rT = p.rT;
    a.segs = p.segs + size_t(task) * (p.n_seg + 2);
    a.subs = p.subs + size_t(task) * p.n_seg * kSubChunks;
    int count = leaf ? 0 : p.q_count[r];
    a.count = count < 0 ? 0 : (count > p.k_cap ? p.k_cap : count);
    a.qi = p.q_idx + size_t(r) * p.k_cap;
    a.ql = p.q_logit + size_t(r) * p.k_cap;
    a.stages = leaf ? 0 : p.node_stages[r];
    a.cands = nullptr;
    a.n_cands = 0;
    if (!leaf && p.wor) {
      const int layer = tree_layer(p, node);
      a.cands = p.cand_tokens + size_t(b) * (p.n_nodes - 1) + (tree_first_child(p, node, layer) - 1);
      a.n_cands = p.expansion[layer];
    }
    a.u = p.u_resample[size_t(b) * p.n_nodes + node];
    a.unusable = state == 2;
    a.item_val = item_val;
    a.table = nullptr;
    token = finish_core<T>(a, sh, st);
  }
  if (tid == 0) {
    if (p.out_node_token) p.out_node_token[size_t(b) * p.n_nodes + node] = token;
    if (p.out_node_slot) p.out_node_slot[size_t(b) * p.n_nodes + node] = slot;
    if (node == p.term_node[b]) p.out_seq[size_t(b) * (p.depth + 1) + (p.out_len[b] - 1)] = token;
    if (st) atomicOr(&p.seq_status[b], st);
  }
}

__global__ void tree_status_kernel(const TreeParams p) {
  const int64_t b = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (b < p.B && p.status) p.status[b] = p.seq_status[b];
}

template <typename T> hipError_t launch_verify_tree(TreeParams p, hipStream_t s) {
  hipError_t e;
  if (p.all_nodes) {
    hipLaunchKernelGGL(tree_mcveri_kernel<T>, dim3(unsigned(p.B * p.n_int)), dim3(kBlock), 0, s, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(tree_walk_kernel, dim3(unsigned(p.B)), dim3(64), 0, s, p);
  } else {
    hipLaunchKernelGGL(tree_lazy_walk_kernel<T>, dim3(unsigned(p.B)), dim3(kBlock), 0, s, p);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const int E = ElemTraits<T>::kPerVec;
  int n_seg = int((p.V / E + 1 + kSegVecsTotal - 1) / kSegVecsTotal);
  if (n_seg > p.n_seg) n_seg = p.n_seg;
  p.n_seg_grid = (n_seg + kGroupSegs - 1) / kGroupSegs;
  // the binary16 table would leave one workgroup of 256 threads per compute unit: bf16 rows only
  p.use_table = std::is_same<T, Bf16>::value && exp_table_usable<T>(p.rT) ? 1 : 0;
  const int64_t grid = std::min<int64_t>(p.B * p.tasks * p.n_seg_grid, sweep_grid_limit());
  hipLaunchKernelGGL(tree_sweep_kernel<T>, dim3(unsigned(grid)), dim3(kBlock), p.use_table ? ExpTab<T>::kBytes : 0, s, p);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(tree_finish_kernel<T>, dim3(unsigned(p.B * p.tasks)), dim3(kBlock), 0, s, p);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (p.status) {
    hipLaunchKernelGGL(tree_status_kernel, dim3(unsigned((p.B + 255) / 256)), dim3(256), 0, s, p);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace tslt
