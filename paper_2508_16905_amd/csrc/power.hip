// gfx950 kernels of the power iteration for the top-k eigenvalues of each layer's Hessian
// (Sec. 3.2, third equation): u <- H u / ||H u||, lambda ~ u^T H u / u^T u, carried out for k
// vectors at once with the earlier directions projected out in order (deflation).
//
// The caller supplies, per layer, the k current vectors u_j and the products w_j = H u_j.  The
// orthonormal basis that ordered Gram-Schmidt would produce from W = [w_0 .. w_{k-1}] is W R^-1,
// R being the Cholesky factor of the k x k Gram matrix W^T W.  That needs two streaming passes
// instead of k dependent ones:
//   Gram pass    reads U and W once: W^T W, u_j . w_j, u_j . u_j (fp64 sums, fixed order)
//   layer kernel k x k Cholesky, coefficients of R^-1, Rayleigh quotients, residuals (fp64)
//   apply pass   reads W again, writes q_j = sum_{i<=j} coef_ij w_i over u_j
// Both passes are HBM-bound: 8k bytes per element each.
#include "power.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "numerics.h"

namespace triaccel {

namespace {

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ constexpr int tri(int i, int j) { return j * (j + 1) / 2 + i; }  // i <= j

template <int K, bool FULL>
__device__ __forceinline__ void gram_chunk(const PowerDesc& pd, int64_t numel, int64_t base, double (&g)[K * (K + 1) / 2],
                                           double (&c)[K], double (&d)[K]) {
  // one row at a time: the 2k loads of a row are in flight together, and the accumulators leave
  // room for several wavefronts per SIMD to overlap their loads with the fp64 arithmetic
#pragma unroll 1
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + (int64_t)r * kRowElems + (int64_t)threadIdx.x * kVec;
    float u[K][4], w[K][4];
#pragma unroll
    for (int j = 0; j < K; ++j) {
      if constexpr (FULL) {
        load4<kFP32>(pd.u + (int64_t)j * pd.stride, idx, u[j]);
        load4<kFP32>(pd.hu + (int64_t)j * pd.stride, idx, w[j]);
      } else {
        load4_guard<kFP32>(pd.u + (int64_t)j * pd.stride, idx, numel, 0.0f, u[j]);
        load4_guard<kFP32>(pd.hu + (int64_t)j * pd.stride, idx, numel, 0.0f, w[j]);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
#pragma unroll
      for (int j = 0; j < K; ++j) {
        const double wj = (double)w[j][e], uj = (double)u[j][e];
        c[j] = fma(uj, wj, c[j]);
        d[j] = fma(uj, uj, d[j]);
#pragma unroll
        for (int i = 0; i <= j; ++i) g[tri(i, j)] = fma((double)w[i][e], wj, g[tri(i, j)]);
      }
    }
  }
}

// Gram pass: one workgroup per segment (kPowerSeg consecutive chunks of one tensor).
template <int K>
__global__ __launch_bounds__(kThreads) void k_power_gram(const TensorDesc* __restrict__ tds,
                                                         const PowerDesc* __restrict__ pds,
                                                         const SegRef* __restrict__ segs, double* __restrict__ partials) {
  constexpr int NG = K * (K + 1) / 2, PP = NG + 2 * K;
  const SegRef sr = segs[blockIdx.x];
  const int64_t numel = tds[sr.tensor].numel;
  const uint32_t n_chunks = tds[sr.tensor].n_chunks;
  const PowerDesc pd = pds[sr.tensor];
  double g[NG], c[K], d[K];
#pragma unroll
  for (int i = 0; i < NG; ++i) g[i] = 0.0;
#pragma unroll
  for (int j = 0; j < K; ++j) c[j] = d[j] = 0.0;
  const uint32_t c0 = sr.index * kPowerSeg;
  const uint32_t c1 = min(c0 + (uint32_t)kPowerSeg, n_chunks);
  for (uint32_t ch = c0; ch < c1; ++ch) {
    const int64_t base = (int64_t)ch * kChunk;
    if (base + kChunk <= numel) gram_chunk<K, true>(pd, numel, base, g, c, d);
    else gram_chunk<K, false>(pd, numel, base, g, c, d);
  }
  // lanes, then wavefronts, in a fixed order
  __shared__ double s_part[kThreads / kWave][PP];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    const double v = wave_sum_f64(g[i]);
    if (lane == 0) s_part[wave][i] = v;
  }
#pragma unroll
  for (int j = 0; j < K; ++j) {
    const double vc = wave_sum_f64(c[j]), vd = wave_sum_f64(d[j]);
    if (lane == 0) {
      s_part[wave][NG + j] = vc;
      s_part[wave][NG + K + j] = vd;
    }
  }
  __syncthreads();
  if (threadIdx.x < PP) {
    const int e = threadIdx.x;
    partials[(size_t)blockIdx.x * PP + e] = ((s_part[0][e] + s_part[1][e]) + s_part[2][e]) + s_part[3][e];
  }
}

// Per-layer kernel: one workgroup per tensor adds the segment partials (fixed order) and thread 0
// factorises the k x k Gram matrix.  A vector whose remainder after projecting out the earlier
// directions is numerically nothing (pivot <= 1e-12 of its own squared norm) gets a zero column.
template <int K>
__global__ __launch_bounds__(kThreads) void k_power_layer(const TensorDesc* __restrict__ tds,
                                                          const uint32_t* __restrict__ seg_first,
                                                          const double* __restrict__ partials, PowerLayer* state,
                                                          LayerDev* layers, int latch) {
  constexpr int NG = K * (K + 1) / 2, PP = NG + 2 * K;
  static_assert(PP <= kWave, "one lane per partial entry");
  const uint32_t l = blockIdx.x;
  const uint32_t n_segs = (tds[l].n_chunks + kPowerSeg - 1) / kPowerSeg;
  const double* p = partials + (size_t)seg_first[l] * PP;
  const int e = threadIdx.x & (kWave - 1), part = threadIdx.x / kWave;
  double acc = 0.0;
  if (e < PP)
    for (uint32_t s = part; s < n_segs; s += kThreads / kWave) acc += p[(size_t)s * PP + e];
  __shared__ double s_acc[kThreads / kWave][kWave];
  s_acc[part][e] = acc;
  __syncthreads();
  if (threadIdx.x != 0) return;
  double G[K][K], c[K], d[K];
  for (int j = 0; j < K; ++j) {
    for (int i = 0; i <= j; ++i) {
      const int t = tri(i, j);
      G[i][j] = G[j][i] = ((s_acc[0][t] + s_acc[1][t]) + s_acc[2][t]) + s_acc[3][t];
    }
    c[j] = ((s_acc[0][NG + j] + s_acc[1][NG + j]) + s_acc[2][NG + j]) + s_acc[3][NG + j];
    d[j] = ((s_acc[0][NG + K + j] + s_acc[1][NG + K + j]) + s_acc[2][NG + K + j]) + s_acc[3][NG + K + j];
  }
  PowerLayer& st = state[l];
  double R[K][K], T[K][K];
  uint32_t deficient = 0;
  double lam_max = 0.0;
  for (int j = 0; j < K; ++j) {
    // Rayleigh quotient and residual ||w - lambda u|| / ||u|| from the sums (zero iterate: both 0)
    double lam = 0.0, res = 0.0;
    if (d[j] > 0.0) {
      lam = c[j] / d[j];
      const double r2 = G[j][j] - 2.0 * lam * c[j] + lam * lam * d[j];
      res = sqrt(r2 > 0.0 ? r2 : 0.0) / sqrt(d[j]);
    }
    st.rayleigh[j] = (float)lam;
    st.resid[j] = (float)res;
    st.hnorm[j] = (float)sqrt(G[j][j]);
    lam_max = fmax(lam_max, fabs(lam));
    // column j of the Cholesky factor R (G = R^T R) ...
    for (int i = 0; i < j; ++i) {
      double s = 0.0;
      if (!((deficient >> i) & 1u)) {
        s = G[i][j];
        for (int q = 0; q < i; ++q) s -= R[q][i] * R[q][j];
        s /= R[i][i];
      }
      R[i][j] = s;
    }
    double piv = G[j][j];
    for (int q = 0; q < j; ++q) piv -= R[q][j] * R[q][j];
    const bool def = piv <= 1e-12 * G[j][j];
    R[j][j] = def ? 0.0 : sqrt(piv);
    if (def) deficient |= 1u << j;
    // ... and of its inverse: q_j = (w_j - sum_{p<j} R_pj q_p) / R_jj in terms of the w_i
    for (int i = 0; i <= j; ++i) {
      double s = 0.0;
      if (!def) {
        s = (i == j) ? 1.0 : 0.0;
        for (int q = i; q < j; ++q) s -= T[i][q] * R[q][j];
        s /= R[j][j];
      }
      T[i][j] = s;
    }
  }
  for (int i = 0; i < kMaxPowerK; ++i)
    for (int j = 0; j < kMaxPowerK; ++j) st.coef[i][j] = (i <= j && j < K) ? T[i][j] : 0.0;
  for (int j = K; j < kMaxPowerK; ++j) st.rayleigh[j] = st.resid[j] = st.hnorm[j] = 0.0f;
  st.deficient = deficient;
  st.lambda_max = (float)lam_max;
  if (latch) layers[l].lambda_power = (float)lam_max;
}

template <int K, bool FULL>
__device__ __forceinline__ void apply_chunk(const PowerDesc& pd, int64_t numel, int64_t base,
                                            const double (&t)[K * (K + 1) / 2]) {
#pragma unroll
  for (int r = 0; r < kRows; ++r) {
    const int64_t idx = base + (int64_t)r * kRowElems + (int64_t)threadIdx.x * kVec;
    if (!FULL && idx >= numel) continue;
    float w[K][4];
#pragma unroll
    for (int j = 0; j < K; ++j) {
      if constexpr (FULL) load4<kFP32>(pd.hu + (int64_t)j * pd.stride, idx, w[j]);
      else load4_guard<kFP32>(pd.hu + (int64_t)j * pd.stride, idx, numel, 0.0f, w[j]);
    }
#pragma unroll
    for (int j = 0; j < K; ++j) {
      float q[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        double acc = 0.0;
#pragma unroll
        for (int i = 0; i <= j; ++i) acc = fma(t[tri(i, j)], (double)w[i][e], acc);
        q[e] = (float)acc;
      }
      if constexpr (FULL) store4<kFP32>(pd.u + (int64_t)j * pd.stride, idx, q);
      else store4_guard<kFP32>(pd.u + (int64_t)j * pd.stride, idx, numel, q);
    }
  }
}

// Apply pass: one workgroup per chunk.
template <int K>
__global__ __launch_bounds__(kThreads) void k_power_apply(const TensorDesc* __restrict__ tds,
                                                          const PowerDesc* __restrict__ pds,
                                                          const ChunkRef* __restrict__ chunks,
                                                          const PowerLayer* __restrict__ state) {
  constexpr int NG = K * (K + 1) / 2;
  const ChunkRef cr = chunks[blockIdx.x];
  const int64_t numel = tds[cr.tensor].numel;
  const PowerDesc pd = pds[cr.tensor];
  double t[NG];
#pragma unroll
  for (int j = 0; j < K; ++j)
#pragma unroll
    for (int i = 0; i <= j; ++i) t[tri(i, j)] = state[cr.tensor].coef[i][j];
  const int64_t base = (int64_t)cr.index * kChunk;
  if (base + kChunk <= numel) apply_chunk<K, true>(pd, numel, base, t);
  else apply_chunk<K, false>(pd, numel, base, t);
}

template <int K>
hipError_t launch_k(const PowerTables& t, int latch, hipStream_t s, hipEvent_t* ev) {
  hipError_t e;
  if (ev && (e = hipEventRecord(ev[0], s)) != hipSuccess) return e;
  hipLaunchKernelGGL(k_power_gram<K>, dim3(t.total_segs), dim3(kThreads), 0, s, t.tensors, t.descs, t.segs, t.partials);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return e;
  hipLaunchKernelGGL(k_power_layer<K>, dim3(t.n_tensors), dim3(kThreads), 0, s, t.tensors, t.seg_first, t.partials,
                     t.state, t.layers, latch);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
  hipLaunchKernelGGL(k_power_apply<K>, dim3(t.total_chunks), dim3(kThreads), 0, s, t.tensors, t.descs, t.chunks,
                     t.state);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[3], s)) != hipSuccess) return e;
  return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// The iteration for callers that cannot allocate: every table and partial sum the kernels above
// use lives in one fixed device array.  Host code never uses the array's name as an address: the
// device address is looked up once per GPU (each GPU holds its own copy) and passed to the kernels.
// ---------------------------------------------------------------------------------------------
constexpr size_t align256(size_t b) { return (b + 255) & ~size_t(255); }
constexpr size_t kStaticMaxSegs = kStaticMaxChunks / kPowerSeg + kStaticMaxTensors;
constexpr size_t kOffTensors = 0;
constexpr size_t kOffDescs = kOffTensors + align256(sizeof(TensorDesc) * kStaticMaxTensors);
constexpr size_t kOffSegFirst = kOffDescs + align256(sizeof(PowerDesc) * kStaticMaxTensors);
constexpr size_t kOffChunks = kOffSegFirst + align256(sizeof(uint32_t) * kStaticMaxTensors);
constexpr size_t kOffSegs = kOffChunks + align256(sizeof(ChunkRef) * kStaticMaxChunks);
constexpr size_t kOffPartials = kOffSegs + align256(sizeof(SegRef) * kStaticMaxSegs);
constexpr size_t kOffState = kOffPartials + align256(sizeof(double) * power_partial_len(kMaxPowerK) * kStaticMaxSegs);
constexpr size_t kScratchBytes = kOffState + align256(sizeof(PowerLayer) * kStaticMaxTensors);
static_assert(kScratchBytes < (size_t(5) << 20), "the fixed array is meant to stay a few MiB");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU (null: not looked up yet)
std::mutex g_scratch_mutex;

struct StaticEntry {
  float* u;
  const float* hu;
  int64_t stride;
  int64_t numel;
  uint32_t first_chunk;
  uint32_t first_seg;
};
struct StaticBatchArg {
  uint32_t first;  // index of the batch's first tensor
  uint32_t count;
  StaticEntry e[kStaticBatch];
};
static_assert(sizeof(StaticBatchArg) <= 3072, "passed by value as a kernel argument");

// Table kernel: workgroup b writes the tables of tensor first + b (descriptor, chunk and segment lists).
__global__ __launch_bounds__(kThreads) void k_static_tables(StaticBatchArg a, unsigned char* base) {
  const StaticEntry en = a.e[blockIdx.x];
  const uint32_t l = a.first + blockIdx.x;
  const uint32_t nc = (uint32_t)((en.numel + kChunk - 1) / kChunk);
  const uint32_t ns = (nc + kPowerSeg - 1) / kPowerSeg;
  if (threadIdx.x == 0) {
    TensorDesc td{};
    td.numel = en.numel;
    td.first_chunk = en.first_chunk;
    td.n_chunks = nc;
    reinterpret_cast<TensorDesc*>(base + kOffTensors)[l] = td;
    reinterpret_cast<PowerDesc*>(base + kOffDescs)[l] = PowerDesc{en.u, en.hu, en.stride};
    reinterpret_cast<uint32_t*>(base + kOffSegFirst)[l] = en.first_seg;
  }
  ChunkRef* chunks = reinterpret_cast<ChunkRef*>(base + kOffChunks) + en.first_chunk;
  for (uint32_t c = threadIdx.x; c < nc; c += kThreads) chunks[c] = ChunkRef{l, c};
  SegRef* segs = reinterpret_cast<SegRef*>(base + kOffSegs) + en.first_seg;
  for (uint32_t q = threadIdx.x; q < ns; q += kThreads) segs[q] = SegRef{l, q};
}

__global__ void k_static_export(const PowerLayer* __restrict__ state, PowerInfoOut* __restrict__ out, int n) {
  const int l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= n) return;
  PowerInfoOut o;
  for (int j = 0; j < kMaxPowerK; ++j) {
    o.rayleigh[j] = state[l].rayleigh[j];
    o.resid[j] = state[l].resid[j];
    o.hnorm[j] = state[l].hnorm[j];
  }
  o.deficient = state[l].deficient;
  o.lambda_max = state[l].lambda_max;
  o.lambda_latched = 0.0f;
  out[l] = o;
}

}  // namespace

hipError_t power_static_prepare() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev]) return hipSuccess;
  void* p = nullptr;
  e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!p) return hipErrorInvalidSymbol;
  g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  return hipSuccess;
}

hipError_t launch_power_iter_static(const StaticTensor* tensors, int n, int k, PowerInfoOut* info, hipStream_t s) {
  hipError_t e = power_static_prepare();
  if (e != hipSuccess) return e;
  int dev = -1;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  unsigned char* base = g_scratch_ptr[dev];
  if (n == 0) return hipSuccess;
  // tables: the prefix sums are formed here, the lists are written on the device
  uint32_t chunk_pos = 0, seg_pos = 0;
  for (int first = 0; first < n; first += kStaticBatch) {
    StaticBatchArg a{};
    a.first = (uint32_t)first;
    a.count = (uint32_t)(n - first < kStaticBatch ? n - first : kStaticBatch);
    for (uint32_t i = 0; i < a.count; ++i) {
      const StaticTensor& t = tensors[first + (int)i];
      const uint32_t nc = (uint32_t)((t.numel + kChunk - 1) / kChunk);
      a.e[i] = StaticEntry{t.u, t.hu, t.stride, t.numel, chunk_pos, seg_pos};
      chunk_pos += nc;
      seg_pos += (nc + kPowerSeg - 1) / kPowerSeg;
    }
    hipLaunchKernelGGL(k_static_tables, dim3(a.count), dim3(kThreads), 0, s, a, base);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  PowerTables t{};
  t.tensors = reinterpret_cast<const TensorDesc*>(base + kOffTensors);
  t.chunks = reinterpret_cast<const ChunkRef*>(base + kOffChunks);
  t.layers = nullptr;  // only written when a value is latched into an optimizer handle: never here
  t.descs = reinterpret_cast<PowerDesc*>(base + kOffDescs);
  t.segs = reinterpret_cast<SegRef*>(base + kOffSegs);
  t.seg_first = reinterpret_cast<uint32_t*>(base + kOffSegFirst);
  t.partials = reinterpret_cast<double*>(base + kOffPartials);
  t.state = reinterpret_cast<PowerLayer*>(base + kOffState);
  t.n_tensors = (uint32_t)n;
  t.total_chunks = chunk_pos;
  t.total_segs = seg_pos;
  // every partial sum and every record the kernels read is written earlier in this same call, so
  // nothing in the array has to start at zero
  if ((e = launch_power_iter(t, k, 0, s, nullptr)) != hipSuccess) return e;
  hipLaunchKernelGGL(k_static_export, dim3((n + kWave - 1) / kWave), dim3(kWave), 0, s, t.state, info, n);
  return hipGetLastError();
}

hipError_t launch_power_iter(const PowerTables& t, int k, int latch, hipStream_t s, hipEvent_t* ev) {
  switch (k) {
    case 1: return launch_k<1>(t, latch, s, ev);
    case 2: return launch_k<2>(t, latch, s, ev);
    case 3: return launch_k<3>(t, latch, s, ev);
    case 4: return launch_k<4>(t, latch, s, ev);
    case 5: return launch_k<5>(t, latch, s, ev);
    case 6: return launch_k<6>(t, latch, s, ev);
    case 7: return launch_k<7>(t, latch, s, ev);
    case 8: return launch_k<8>(t, latch, s, ev);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace triaccel
