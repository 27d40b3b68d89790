// gfx950 kernels of the QODA hot path (arXiv 2505.14371): per-layer norms, stochastic quantization + code
// packing, fused decode + K-way mean + optimistic dual averaging update, and the histogram level fit.
//
// Execution shape of the norm and quantize passes: one workgroup = 256 threads = 4 wave64 = one tile of 16384
// coordinates of one (node, layer).  Wave w owns the 16 consecutive 256-coordinate blocks 16w..16w+15 of the tile; in a
// block, lane i owns coordinates 4i..4i+3 (one 128-bit load, 1 KB contiguous per wave).  Thread t = 64w+i is reduction
// slot t of the fixed-order fp64 sums.  The decode pass keeps the lane <-> coordinate mapping but runs in shorter
// workgroups (one octet per wave, see k_decode).  The packed message is lane-local: the codes of the 32 coordinates a lane
// owns in 8 consecutive blocks (an octet) are shifted into C1 = 1 + b 32-bit words per lane, and word r of the
// 64 lanes is one contiguous 256-byte store.
//
// Arithmetic that feeds an integer decision (level index, rounding direction, packed bits, histogram bin) is
// written as single IEEE operations with contraction off, so that it has one well-defined result.

#include "qoda_kernels.h"

namespace qoda {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));   // plain vector type: usable behind address-space pointers

__device__ __forceinline__ unsigned int f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(unsigned int u) { return __uint_as_float(u); }

constexpr float kFltMax = 3.402823466e+38f;
constexpr float kFltMin = 1.17549435e-38f;   // 2^-126, the smallest normal float

// Bits of the sticky device status word.
constexpr unsigned int kStatusNonFinite = 1u;   // a statistic is not a finite number in range
constexpr unsigned int kStatusTinyNorm = 2u;    // 0 < norm < 2^-126: 1/norm is not a float (the one case where the
                                                // quantizer of that vector is biased, Thm 5.1)

// largest float n >= 0 with n*n <= s (n*n is exact in fp64); 0 when s is not a finite number in range.
__device__ float sqrt_floor(double s) {
  const double lim = (double)kFltMax * (double)kFltMax;
  if (!(s >= 0.0) || !(s <= lim)) return 0.0f;
  const double r = sqrt(s);
  float n = (r >= (double)kFltMax) ? kFltMax : (float)r;
  for (int it = 0; it < 4 && (double)n * (double)n > s; ++it) n = u2f(f2u(n) - 1u);
  for (int it = 0; it < 4; ++it) {
    if (n == kFltMax) break;
    const float up = u2f(f2u(n) + 1u);
    if ((double)up * (double)up <= s) n = up; else break;
  }
  return n;
}

// largest finite float r >= 0 with x*r <= 1 (exact in fp64); 0 for x <= 0 or non-finite x.
__device__ float rcp_floor(float x) {
  if (!(x > 0.0f) || x > kFltMax) return 0.0f;
  float r = 1.0f / x;
  if (r > kFltMax) r = kFltMax;
  for (int it = 0; it < 4 && (double)x * (double)r > 1.0; ++it) r = u2f(f2u(r) - 1u);
  for (int it = 0; it < 4; ++it) {
    if (r == kFltMax) break;
    const float up = u2f(f2u(r) + 1u);
    if ((double)x * (double)up <= 1.0) r = up; else break;
  }
  return r;
}

// The same two functions for the per-bucket norms, where they run once per 128 coordinates and their cost shows:
// straight-line code for arguments in a comfortable range (sums of squares in [2^-200, 2^200]), the general
// routines otherwise.  Both return exactly what sqrt_floor / rcp_floor return (the definitions are by exact
// comparisons, so any way of finding the largest float that passes them gives the same bits).
__device__ __forceinline__ void norm_and_inverse(double s, float &n_out, float &r_out) {
  const long long bits = __double_as_longlong(s);
  const int e = (int)((bits >> 52) & 0x7FF) - 1023;
  if (e < -200 || e > 200) {   // zero, tiny, huge or not a number: the general path
    n_out = sqrt_floor(s);
    r_out = rcp_floor(n_out);
    return;
  }
  // s = sp * 4^k with sp in [1, 4): root in single precision, then the candidates around it are tested exactly
  const int k = e >> 1;
  const double sp = __longlong_as_double(bits - ((long long)(2 * k) << 52));
  const float r0 = __builtin_sqrtf((float)sp);   // within one unit of the last place of the true root of sp
  float n = u2f(f2u(r0) + 1u);
#pragma unroll
  for (int it = 0; it < 3; ++it) {
    const double nd = (double)n;
    if (nd * nd > sp) n = u2f(f2u(n) - 1u);
  }
  n = u2f(f2u(n) + ((unsigned int)k << 23));   // times 2^k: exact, the result is a normal number
  // reciprocal: hardware estimate, then the same exact test on the candidates around it
  const float q0 = __builtin_amdgcn_rcpf(n);
  float r = u2f(f2u(q0) + 1u);
  const double nd = (double)n;
#pragma unroll
  for (int it = 0; it < 3; ++it) {
    if (nd * (double)r > 1.0) r = u2f(f2u(r) - 1u);
  }
  n_out = n;
  r_out = r;
}

// Fixed halving tree over the 256 slots: p[i] += p[i+h], h = 128 .. 1.  The two cross-wave steps are one pass
// through shared memory, the six in-wave steps are shuffles (lane i < h adds lane i + h, exactly the tree).
// The total is valid in thread 0 only.
__device__ double block_tree(double v, double *red) {
  const int t = threadIdx.x;
  red[t] = v;
  __syncthreads();
  double r = 0.0;
  if (t < 64) {
    r = (red[t] + red[t + 128]) + (red[t + 64] + red[t + 192]);
#pragma unroll
    for (int h = 32; h >= 1; h >>= 1) r = r + __shfl_down(r, h, 64);
  }
  __syncthreads();   // red may be reused by the caller
  return r;
}

// The same shape with the maximum instead of the sum (the order does not matter for a maximum; v >= 0, never NaN).
__device__ double block_max(double v, double *red) {
  const int t = threadIdx.x;
  red[t] = v;
  __syncthreads();
  double r = 0.0;
  if (t < 64) {
    r = fmax(fmax(red[t], red[t + 128]), fmax(red[t + 64], red[t + 192]));
#pragma unroll
    for (int h = 32; h >= 1; h >>= 1) r = fmax(r, __shfl_down(r, h, 64));
  }
  __syncthreads();
  return r;
}

// ----- the three kinds of norm: statistic -> finite?, norm, reciprocal, fit weight
__device__ __forceinline__ bool stat_finite(double s, int kind) {
  const double fm = (double)kFltMax;
  return (s >= 0.0) && (s <= (kind == kNormL2 ? fm * fm : fm));
}
__device__ __forceinline__ float norm_of(double s, int kind) {
  return kind == kNormL2 ? sqrt_floor(s) : __double2float_rn(s);
}
__device__ __forceinline__ double weight_of(double s, int kind) { return kind == kNormL2 ? s : s * s; }
// largest magnitude from the running maximum of magnitude bit patterns: an infinity or a NaN pattern gives +infinity
__device__ __forceinline__ float magnitude_from_bits(unsigned int mb) { return u2f(mb > 0x7F7FFFFFu ? 0x7F800000u : mb); }

// rcp_floor for a norm in a comfortable range by straight-line code (estimate, then the exact test on the
// candidates around it), the general routine otherwise: the same bits either way.
__device__ __forceinline__ float inverse_of(float n) {
  const int e = (int)((f2u(n) >> 23) & 0xFF) - 127;
  if (e < -100 || e > 100) return rcp_floor(n);
  float r = u2f(f2u(__builtin_amdgcn_rcpf(n)) + 1u);
  const double nd = (double)n;
#pragma unroll
  for (int it = 0; it < 3; ++it) {
    if (nd * (double)r > 1.0) r = u2f(f2u(r) - 1u);
  }
  return r;
}

// Philox4x32-10 (Salmon et al., SC'11).
__device__ __forceinline__ void philox4x32_10(unsigned int c0, unsigned int c1, unsigned int c2, unsigned int c3,
                                               unsigned int k0, unsigned int k1, unsigned int out[4]) {
  constexpr unsigned long long M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull;
  constexpr unsigned int W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const unsigned long long p0 = M0 * (unsigned long long)c0;
    const unsigned long long p1 = M1 * (unsigned long long)c2;
    const unsigned int n0 = __builtin_amdgcn_bitop3_b32((unsigned int)(p1 >> 32), c1, k0, 0x96);   // 3-input xor
    const unsigned int n1 = (unsigned int)p1;
    const unsigned int n2 = __builtin_amdgcn_bitop3_b32((unsigned int)(p0 >> 32), c3, k1, 0x96);
    const unsigned int n3 = (unsigned int)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Loads through pointers read from device tables: tell the compiler they point to global memory.
template <class T>
__device__ __forceinline__ const __attribute__((address_space(1))) T *as_global(const T *p) {
  return (const __attribute__((address_space(1))) T *)p;
}

// Four coordinates e..e+3 of a layer of d entries; entries past the end read as +0.
__device__ __forceinline__ void load4(const float *__restrict__ v, long long e, long long d, float x[4]) {
  const auto *g = as_global(v);
  if (e + 4 <= d) {
    // every big array here is streamed once per pass: nontemporal accesses measurably raise the read rate
    const v4f q = __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) v4f *>(g + e));
    x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) x[j] = (e + j < d) ? g[e + j] : 0.0f;
  }
}

__device__ __forceinline__ void store4(float *__restrict__ v, long long e, long long d, const float x[4]) {
  auto *g = (__attribute__((address_space(1))) float *)v;
  if (e + 4 <= d) {
    v4f q;
    q.x = x[0]; q.y = x[1]; q.z = x[2]; q.w = x[3];
    __builtin_nontemporal_store(q, reinterpret_cast<__attribute__((address_space(1))) v4f *>(g + e));
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (e + j < d) g[e + j] = x[j];
  }
}

// ---- packed lane records (message body).  A lane's 32 codes of an octet (8 blocks x 4 coordinates, code
// number jj = 4*block + component, C1 bits each: sign | index << 1) form a little-endian bit string kept in C1
// 32-bit registers.  jj is a compile-time constant wherever these are called (fully unrolled loops), so every
// shift below is an immediate.
template <int C1>
__device__ __forceinline__ void insert_code(unsigned int (&D)[C1], unsigned int code, int jj) {
  const int pos = C1 * jj, r = pos >> 5, sh = pos & 31;
  D[r] |= code << sh;
  if (sh + C1 > 32) D[r + 1] |= code >> (32 - sh);
}

template <int C1>
__device__ __forceinline__ unsigned int extract_code(const unsigned int (&D)[C1], int jj) {
  const int pos = C1 * jj, r = pos >> 5, sh = pos & 31;
  unsigned int v = D[r] >> sh;
  if (sh + C1 > 32) v |= D[r + 1] << (32 - sh);
  return v & ((1u << C1) - 1u);
}

// Byte offset (code * 4) of code jj into a table of floats: two instructions (shift or funnel shift, mask).
template <int C1>
__device__ __forceinline__ unsigned int extract_off(const unsigned int (&D)[C1], int jj) {
  const int pos = C1 * jj, r = pos >> 5, sh = pos & 31;
  unsigned int v;
  if (sh + C1 <= 32) v = (sh >= 2) ? (D[r] >> (sh - 2)) : (D[r] << (2 - sh));
  else v = __builtin_amdgcn_alignbit(D[r + 1], D[r], sh - 2);   // straddles two words; then sh >= 23
  return v & (((1u << C1) - 1u) << 2);
}

__device__ __forceinline__ float lds_float_at(const float *table, unsigned int byte_off) {
  return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(table) + byte_off);
}

// Shift a C1-word little-endian bit string right by 8*C1 bits (one block pair's worth of codes).
template <int C1>
__device__ __forceinline__ void shift_out_pair(unsigned int (&D)[C1]) {
  constexpr int wq = (8 * C1) >> 5, bq = (8 * C1) & 31;
#pragma unroll
  for (int r = 0; r < C1; ++r) {
    const unsigned int lo = (r + wq < C1) ? D[r + wq] : 0u;
    const unsigned int hi = (r + wq + 1 < C1) ? D[r + wq + 1] : 0u;
    D[r] = (bq == 0) ? lo : ((lo >> bq) | (hi << (32 - bq)));
  }
}

// The C1 record words of lane i of one octet: word r is the 32-bit word r*64 + i of the octet's 256*C1 bytes.
template <int C1>
__device__ __forceinline__ void load_record(const unsigned char *octet, int i, unsigned int (&D)[C1]) {
  const auto *g = reinterpret_cast<const __attribute__((address_space(1))) unsigned int *>(as_global(octet));
#pragma unroll
  for (int r = 0; r < C1; ++r) D[r] = __builtin_nontemporal_load(g + r * 64 + i);
}

template <int C1>
__device__ __forceinline__ void store_record(unsigned char *octet, int i, const unsigned int (&D)[C1]) {
  auto *g = (__attribute__((address_space(1))) unsigned int *)octet;
#pragma unroll
  for (int r = 0; r < C1; ++r) __builtin_nontemporal_store(D[r], g + r * 64 + i);
}

}  // namespace

// ------------------------------------------------------------------------------------------------ zero fill
__global__ void k_zero_u32(unsigned int *p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

// ------------------------------------------------------------------------------------------------ pass 1
// Sum of squares of one tile in fp64 (Sec. 2.2, L2 norm before the root), optionally with the histogram of the
// top 11 magnitude bits of every coordinate (the distribution estimate of Alg. 1 line 4).
template <bool HIST, int KIND>
__global__ void __launch_bounds__(kThreads) k_sumsq(Dev a) {
  __shared__ double red[kThreads];
  __shared__ unsigned int lh[HIST ? kHistBins : 1];
  // a workgroup takes up to kSuperTile consecutive tiles of one layer, so that the histogram is flushed to
  // global memory (integer atomics on a few hot addresses) once per run instead of once per tile
  const int4 st = a.stiles[blockIdx.x];   // (layer, first chunk inside the layer, chunks)
  const int l = st.x;
  const int k = a.node0 + blockIdx.y;
  const int kr = k - a.row0;   // row of this node in the per-node scratch and pointer tables
  const LayerMeta m = a.meta[l];
  const float *__restrict__ v = a.grad[(size_t)kr * a.L + l];
  const int t = threadIdx.x;
  const int w = t >> 6, i = t & 63;
  if (HIST) {
    for (int b = t; b < kHistBins; b += kThreads) lh[b] = 0u;
    __syncthreads();
  }
  for (int cc = 0; cc < st.z; ++cc) {
    const int chunk = st.y + cc;
    const long long base = (long long)chunk * kChunkCoords + (long long)w * 16 * kBlockCoords + 4 * i;
    double acc = 0.0;
    unsigned int mb = 0u;   // KIND == kNormLinf: largest magnitude bit pattern
    if ((long long)(chunk + 1) * kChunkCoords <= m.d) {
      v4f q[16];
#pragma unroll
      for (int s = 0; s < 16; ++s)
        q[s] = __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) v4f *>(
            as_global(v) + base + (long long)s * kBlockCoords));
#pragma unroll
      for (int s = 0; s < 16; ++s) {
        const float x[4] = {q[s].x, q[s].y, q[s].z, q[s].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double xd = (double)x[j];
          if (KIND == kNormL2) acc = __builtin_fma(xd, xd, acc);   // the product is exact in fp64, so this equals acc + xd*xd
          else if (KIND == kNormL1) acc = acc + fabs(xd);
          else mb = max(mb, f2u(x[j]) & 0x7FFFFFFFu);
          if (HIST) atomicAdd(&lh[(f2u(x[j]) & 0x7FFFFFFFu) >> 20], 1u);
        }
      }
    } else {
      for (int s = 0; s < 16; ++s) {
        const long long e = base + (long long)s * kBlockCoords;
        if (e >= m.d) break;
        float x[4];
        load4(v, e, m.d, x);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double xd = (double)x[j];
          if (KIND == kNormL2) acc = __builtin_fma(xd, xd, acc);
          else if (KIND == kNormL1) acc = acc + fabs(xd);
          else mb = max(mb, f2u(x[j]) & 0x7FFFFFFFu);
          if (HIST && e + j < m.d) atomicAdd(&lh[(f2u(x[j]) & 0x7FFFFFFFu) >> 20], 1u);
        }
      }
    }
    const double total = (KIND == kNormLinf) ? block_max((double)magnitude_from_bits(mb), red) : block_tree(acc, red);
    if (t == 0) a.partial[(size_t)kr * a.G + m.first_chunk + chunk] = total;
  }
  if (HIST) {
    __syncthreads();
    unsigned int *gh = a.hist + ((size_t)k * a.L + l) * kHistBins;
    for (int b = t; b < kHistBins; b += kThreads) {
      const unsigned int c = lh[b];
      if (c) atomicAdd(&gh[b], c);
    }
  }
}

// Combine the tile sums of one (node, layer): slot j takes tiles j, j+256, ... in increasing order, then the
// halving tree; then norm = sqrt_floor(sum), inv = rcp_floor(norm).
__global__ void __launch_bounds__(kThreads) k_norm_finalize(Dev a) {
  __shared__ double red[kThreads];
  const int l = blockIdx.x;
  const int k = a.node0 + blockIdx.y - a.row0;   // row in the per-node scratch tables
  const LayerMeta m = a.meta[l];
  const double *p = a.partial + (size_t)k * a.G + m.first_chunk;
  double acc = 0.0;
  double s;
  if (a.kind == kNormLinf) {
    for (int c = threadIdx.x; c < m.nchunks; c += kThreads) acc = fmax(acc, p[c]);
    s = block_max(acc, red);
  } else {
    for (int c = threadIdx.x; c < m.nchunks; c += kThreads) acc = acc + p[c];
    s = block_tree(acc, red);
  }
  if (threadIdx.x == 0) {
    const bool finite = stat_finite(s, a.kind);
    const float n = finite ? norm_of(s, a.kind) : 0.0f;
    const size_t idx = (size_t)k * a.L + l;
    a.sumsq[idx] = s;
    a.norm[idx] = n;
    a.inv[idx] = rcp_floor(n);
    if (!finite) atomicOr(a.status, kStatusNonFinite);
    if (n > 0.0f && n < kFltMin) atomicOr(a.status, kStatusTinyNorm);
  }
}

// Whole-vector scope (the literal normalisation of Sec. 2.2 / Sec. 3.1): the L layer sums of a node are combined
// (slot j takes layers j, j+256, ... in increasing order, then the halving tree) and every layer of the node gets
// that sum, its root and the root's reciprocal.
__global__ void __launch_bounds__(kThreads) k_norm_vector(Dev a) {
  __shared__ double red[kThreads];
  __shared__ double tot[1];
  const int k = a.node0 + blockIdx.x - a.row0;   // row in the per-node scratch tables
  double acc = 0.0;
  double s;
  if (a.kind == kNormLinf) {
    for (int l = threadIdx.x; l < a.L; l += kThreads) acc = fmax(acc, a.sumsq[(size_t)k * a.L + l]);
    s = block_max(acc, red);
  } else {
    for (int l = threadIdx.x; l < a.L; l += kThreads) acc = acc + a.sumsq[(size_t)k * a.L + l];
    s = block_tree(acc, red);
  }
  if (threadIdx.x == 0) tot[0] = s;
  __syncthreads();
  const double total = tot[0];
  const bool finite = stat_finite(total, a.kind);
  const float n = finite ? norm_of(total, a.kind) : 0.0f;
  const float r = rcp_floor(n);
  for (int l = threadIdx.x; l < a.L; l += kThreads) {
    const size_t idx = (size_t)k * a.L + l;
    a.sumsq[idx] = total;
    a.norm[idx] = n;
    a.inv[idx] = r;
  }
  if (threadIdx.x == 0 && !finite) atomicOr(a.status, kStatusNonFinite);
  if (threadIdx.x == 0 && n > 0.0f && n < kFltMin) atomicOr(a.status, kStatusTinyNorm);
}

// ------------------------------------------------------------------------------------------------ pass 2
// Quantize + pack one tile (Sec. 3.1, Sec. 3.2) and accumulate the squared distance to the node's previous
// decoded message (the step-size term of eq. (general_stepsize)).
// Quantize the four coordinates a lane owns in one block (Sec. 3.1), append their codes to the record and add
// their squared distance to the previous decoded message (eq. (general_stepsize)).  jl0 = 0 or 4: position of
// the block inside its pair.
template <int C1, bool PREV>
__device__ __forceinline__ void quantize_block(const float (&x)[4], const unsigned int (&o)[4], int half, float inv,
                                               float norm, const unsigned char *lut, const float4 *tab,
                                               const float *tprev, unsigned int (&D)[C1], const unsigned int (&Dp)[C1],
                                               float &acc) {
  float u[4];
  int tau[4];
  float4 lv[4];                    // {l_tau, 1/gap, l_tau+1, -}; entry S-1 = {1, 0, +inf, -}
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    // min(|v| * inv, 1): the product is never negative or NaN for finite input, so the [0, 1] clamp of the
    // multiply instruction is the same thing
    u[j] = __builtin_amdgcn_fmed3f(fabsf(x[j]) * inv, 0.0f, 1.0f);
    tau[j] = lut[f2u(u[j]) >> 20];
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) lv[j] = tab[tau[j]];
  // The table gave tau at the lower edge of u's bin; a level inside the bin (never the case for fitted levels,
  // which sit on bin edges) makes some lanes walk on.  At u = 1 the walk ends on the entry of the last level
  // itself (xi = 0, never rounds up), which yields the same code and value as tau = S-2 rounding up.
  if (__ballot((lv[0].z <= u[0]) | (lv[1].z <= u[1]) | (lv[2].z <= u[2]) | (lv[3].z <= u[3])) != 0ull) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      while (lv[j].z <= u[j]) { ++tau[j]; lv[j] = tab[tau[j]]; }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int jl = 4 * half + j;                       // position of the coordinate inside the pair
    const unsigned int w16 = half ? (o[j] >> 16) : (o[j] & 0xFFFFu);
    const float xi = (u[j] - lv[j].x) * lv[j].y;
    // (w16 + 0.5) < xi * 65536  <=>  w16 < xi * 65536 - 0.5 : the scaling by 2^16 is exact, and the subtraction
    // is exact whenever its result is not negative, so one fused operation decides the same.
    const bool up = (float)w16 < __builtin_fmaf(xi, 65536.0f, -0.5f);
    const unsigned int h = (unsigned int)tau[j] + (up ? 1u : 0u);
    // norm * l_h, the value the decoder will rebuild (the +inf of the last entry is never selected: there xi = 0)
    const float mag = norm * (up ? lv[j].z : lv[j].x);
    const float cur = __builtin_copysignf(mag, x[j]);
    insert_code<C1>(D, (h << 1) | (f2u(x[j]) >> 31), 24 + jl);
    float diff = cur;   // PREV == false: no node has a previous message (first round, or the rule of eq. (Alt))
    if (PREV) diff = cur - lds_float_at(tprev, extract_off<C1>(Dp, jl));   // table all zero for a node without one
    acc = __builtin_fmaf(diff, diff, acc);
  }
}

__device__ __forceinline__ void load_block_fast(const float *__restrict__ v, long long B, int i, float (&x)[4]) {
  const v4f q = __builtin_nontemporal_load(
      reinterpret_cast<const __attribute__((address_space(1))) v4f *>(as_global(v) + B * kBlockCoords + 4 * i));
  x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
}

// One octet (8 blocks = 2048 coordinates) of one (node, layer) for one wave: 4 block pairs, each with one
// generator call and 8 coordinates per lane.  The lane record is built as a shift register: every pair shifts it
// right by 8*C1 bits and writes its 8 codes into the top quarter, so that after four pairs pair 0 sits at bit 0;
// the previous message's record is consumed from the bottom the same way.  The pair loop is deliberately not
// unrolled: unrolled, the compiler interleaves the pairs and needs more than 256 registers.  The next pair's
// gradient values are requested before the current pair is processed.
// FAST: the whole octet lies inside the layer (no bounds checks anywhere).
template <int C1, bool FAST, bool PREV>
__device__ __forceinline__ void quantize_octet(const Dev &a, const LayerMeta &m, int l, int k, long long O,
                                               const float *__restrict__ v, unsigned char *body,
                                               const unsigned char *prevbody, float inv, float norm,
                                               const unsigned char *lut, const float4 *tab, const float *tprev, int i,
                                               float &acc) {
  const unsigned int k0 = (unsigned int)a.seed, k1 = (unsigned int)(a.seed >> 32);
  unsigned int D[C1], Dp[C1];
#pragma unroll
  for (int r = 0; r < C1; ++r) { D[r] = 0u; Dp[r] = 0u; }
  if (PREV && prevbody != nullptr) load_record<C1>(prevbody + O * 256 * C1, i, Dp);
  float xa[4] = {0.0f, 0.0f, 0.0f, 0.0f}, xb[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (FAST) {
    load_block_fast(v, O * 8, i, xa);
    load_block_fast(v, O * 8 + 1, i, xb);
  }
#pragma unroll 1
  for (int pp = 0; pp < 4; ++pp) {
    const long long B0 = O * 8 + 2 * pp;   // block index inside the layer
    shift_out_pair<C1>(D);
    if (FAST || B0 < m.nblk) {
      float x0[4], x1[4];
      if (FAST) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { x0[j] = xa[j]; x1[j] = xb[j]; }
        if (pp < 3) {
          load_block_fast(v, B0 + 2, i, xa);
          load_block_fast(v, B0 + 3, i, xb);
        }
      } else {
        load4(v, B0 * kBlockCoords + 4 * i, m.d, x0);
#pragma unroll
        for (int j = 0; j < 4; ++j) x1[j] = 0.0f;
        if (B0 + 1 < m.nblk) load4(v, (B0 + 1) * kBlockCoords + 4 * i, m.d, x1);
      }
      unsigned int o[4];
      philox4x32_10((unsigned int)((B0 >> 1) * 64 + i), (unsigned int)l, a.round, (unsigned int)k, k0, k1, o);
      quantize_block<C1, PREV>(x0, o, 0, inv, norm, lut, tab, tprev, D, Dp, acc);
      // a block past the end of the layer is all padding: +0 inputs give code 0 and add nothing, as required
      quantize_block<C1, PREV>(x1, o, 1, inv, norm, lut, tab, tprev, D, Dp, acc);
    }
    if (PREV) shift_out_pair<C1>(Dp);
  }
  store_record<C1>(body + O * 256 * C1, i, D);
}

template <int C1, bool PREV>
__device__ __forceinline__ void quantize_tile(const Dev &a, const LayerMeta &m, int l, int k, int chunk,
                                              const unsigned char *lut, const float4 *tab, const float *tprev,
                                              double *red) {
  const int t = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int i = t & 63;
  const int kr = k - a.row0;   // row of this node in the per-node scratch and pointer tables
  const float *__restrict__ v = a.grad[(size_t)kr * a.L + l];
  unsigned char *body = a.msg[kr] + m.body_off;
  const unsigned char *prevbody = (a.prev != nullptr && a.prev[kr] != nullptr) ? a.prev[kr] + m.body_off : nullptr;
  const float inv = a.inv[(size_t)kr * a.L + l];
  const float norm = a.norm[(size_t)kr * a.L + l];
  const long long noct = (m.nblk + 7) >> 3;
  float acc = 0.0f;   // this slot's squared differences: an fp32 fused multiply-add chain in increasing coordinate
  for (int oo = 0; oo < 2; ++oo) {
    const long long O = (long long)chunk * 8 + w * 2 + oo;   // octet index inside the layer
    if (O >= noct) break;
    if ((O + 1) * 2048 <= m.d)
      quantize_octet<C1, true, PREV>(a, m, l, k, O, v, body, prevbody, inv, norm, lut, tab, tprev, i, acc);
    else
      quantize_octet<C1, false, PREV>(a, m, l, k, O, v, body, prevbody, inv, norm, lut, tab, tprev, i, acc);
  }
  const double total = block_tree((double)acc, red);
  if (t == 0) a.dpartial[(size_t)kr * a.G + blockIdx.x] = total;
}

template <int C1, bool PREV>
__global__ void __launch_bounds__(kThreads) k_quantize(Dev a) {
  __shared__ unsigned char lut[kLutSize];
  __shared__ float4 tab[kMaxPoints];
  __shared__ float tprev[2 * kMaxPoints];   // previous message's decode table indexed by code = sign | h << 1
  __shared__ double red[kThreads];
  const int2 tile = a.tiles[blockIdx.x];
  const int l = tile.x;
  const int k = a.node0 + blockIdx.y;
  const LayerMeta m = a.meta[l];
  if (m.planes != C1) return;   // layers of another code width are served by another instantiation
  const int t = threadIdx.x;
  const float *lev = a.lev + (size_t)m.type * kMaxPoints;
  const float *rg = a.rgap + (size_t)m.type * kMaxPoints;
  reinterpret_cast<unsigned int *>(lut)[t] = reinterpret_cast<const unsigned int *>(a.lut + (size_t)m.type * kLutSize)[t];
  const int kr = k - a.row0;
  const float norm = a.norm[(size_t)kr * a.L + l];
  const unsigned char *prevmsg = (a.prev != nullptr) ? a.prev[kr] : nullptr;
  if (t < m.S) {
    const float lj = lev[t];
    const float ln = (t + 1 < m.S) ? lev[t + 1] : __builtin_inff();   // the last entry stops every walk
    tab[t] = make_float4(lj, (t + 1 < m.S) ? rg[t] : 0.0f, ln, 0.0f);
  }
  if (tile.y == 0) {   // message header of this layer: {norm, levels[S]} (Sec. 3.2: the norm in C_q = 32 bits)
    float *h = reinterpret_cast<float *>(a.msg[kr] + m.hdr_off);
    for (int j = t; j <= m.S; j += kThreads) h[j] = (j == 0) ? norm : lev[j - 1];
  }
  for (int c = t; c < (1 << m.planes); c += kThreads) {   // codes past S-1 decode as the last level
    float pv = 0.0f;
    if (prevmsg) {
      const float *hp = reinterpret_cast<const float *>(prevmsg + m.hdr_off);
      const float mag = hp[0] * hp[1 + min(c >> 1, m.S - 1)];
      pv = (c & 1) ? -mag : mag;
    }
    tprev[c] = pv;
  }
  __syncthreads();
  quantize_tile<C1, PREV>(a, m, l, k, tile.y, lut, tab, tprev, red);
}

// ------------------------------------------------------------------------------------------------ bucket scope
// One norm per 128 consecutive coordinates (the experiments' setting, Sec. 7): the norms are computed by the wave
// that quantizes, so the gradient is read from memory once (the second touch of an octet, a few microseconds after
// the first, is served by the cache).
//
// Per-wave shared memory of the bucket-scope quantizer.
constexpr double kBucketRescueBelow = 7.888609052210118e-31;   // 2^-100

struct __attribute__((aligned(8))) BucketWave {
  // the lane's sum of its 4 squares (fp32 fused chain in coordinate order) for block bb, lane i, at index
  // 72*bb + i + i/8: one word of padding after every 8, so that the transposed read below (lane L reads the 8
  // consecutive entries 8L .. 8L+7, i.e. a stride of 9 words between lanes) spreads over all banks
  float psum[8 * 72];
  float norm[16];       // [8*half + block] of the current octet
  float inv[16];
  float pnorm[16];      // the previous message's norms of the same buckets
  unsigned int wfix[16];   // fit statistics: integer weight of the bucket (0: gathers nothing)
};

// The sums of squares of the 16 buckets of one octet once more with exact fp64 squares (a lane's chain
// acc = fma((double)x, (double)x, acc), then the same tree): the path taken when a single-precision result is below
// 2^-100 or not finite.  The 8 x 64 lane sums go through the wave's shared memory four blocks at a time (as doubles they
// fill the area the single-precision pass used).  Every lane of the wave must call this; the result is the sum of
// the lane's own bucket.
template <bool FAST>
__device__ __forceinline__ double bucket_sums_exact(const LayerMeta &m, long long O, const float *__restrict__ v,
                                                 float *psum, int i) {
  double *dsum = reinterpret_cast<double *>(psum);
  const int q = i >> 2, r = i & 3;
  const int bb = q >> 1, hf = q & 1;
  double s = 0.0;
  for (int half = 0; half < 2; ++half) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int b4 = 0; b4 < 4; ++b4) {
      const long long e = (O * 8 + 4 * half + b4) * kBlockCoords + 4 * i;
      float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (FAST || e < m.d) load4(v, e, FAST ? e + 4 : m.d, x);
      double acc = 0.0;
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = __builtin_fma((double)x[j], (double)x[j], acc);
      dsum[72 * b4 + i + (i >> 3)] = acc;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if ((bb >> 2) == half) {
      const double *p = &dsum[72 * (bb & 3) + 36 * hf + 9 * r];
      s = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
    }
  }
  s = s + __shfl_xor(s, 1, 64);
  s = s + __shfl_xor(s, 2, 64);
  return s;
}

// Sums of squares of the 16 buckets of one octet -> norm, inv (shared memory) and the octet's norm trailer.
// A lane's four squares are an fp32 fused chain; lane L then finishes bucket q = L/4 (block q/2, half q%2): it adds 8
// consecutive lane sums, widened to fp64, by the in-order binary tree, then the four lanes of the quad combine
// (neighbour, then pair), which continues the same tree.
// A single-precision result below 2^-100 (squares may have vanished) or not finite (squares may have overflowed) is
// replaced by the exact one (bucket_sums_exact).
// ex: weight scale of the layer's type for the fit statistics (kTypeSkip: none); best: running maximum of the bit
// patterns of the lane's bucket sums.
template <bool FAST, int KIND>
__device__ __forceinline__ void bucket_norms(const Dev &a, const LayerMeta &m, long long O, const float *__restrict__ v,
                                             float *trailer, const float *prev_trailer, BucketWave &bw, int i, int ex,
                                             unsigned long long &best) {
#pragma unroll
  for (int bb = 0; bb < 8; ++bb) {
    const long long e = (O * 8 + bb) * kBlockCoords + 4 * i;
    float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (FAST) {
      const v4f q = *reinterpret_cast<const __attribute__((address_space(1))) v4f *>(as_global(v) + e);
      x[0] = q.x; x[1] = q.y; x[2] = q.z; x[3] = q.w;
    } else if (e < m.d) {
      load4(v, e, m.d, x);
    }
    float acc = 0.0f;
    if (KIND == kNormL2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = __builtin_fmaf(x[j], x[j], acc);
    } else if (KIND == kNormL1) {
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = acc + fabsf(x[j]);
    } else {
      unsigned int mb = 0u;
#pragma unroll
      for (int j = 0; j < 4; ++j) mb = max(mb, f2u(x[j]) & 0x7FFFFFFFu);
      acc = magnitude_from_bits(mb);
    }
    bw.psum[72 * bb + i + (i >> 3)] = acc;
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const int q = i >> 2, r = i & 3;
  const int bb = q >> 1, hf = q & 1;
  const float *p = &bw.psum[72 * bb + 36 * hf + 9 * r];   // lanes 32*hf + 8*r .. +7 of block bb in the padded layout
  double s;
  if (KIND == kNormLinf) {
    const float mx = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])), fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
    s = (double)mx;
    s = fmax(s, __shfl_xor(s, 1, 64));
    s = fmax(s, __shfl_xor(s, 2, 64));
  } else {
    s = (((double)p[0] + (double)p[1]) + ((double)p[2] + (double)p[3])) +
        (((double)p[4] + (double)p[5]) + ((double)p[6] + (double)p[7]));
    s = s + __shfl_xor(s, 1, 64);
    s = s + __shfl_xor(s, 2, 64);
  }
  if (KIND == kNormL2) {
    const bool redo = !(s >= kBucketRescueBelow) || !(s <= 1.7976931348623157e308);
    if (__ballot(redo) != 0ull) {   // rare: all lanes of the wave take the exact path together
      const double exact = bucket_sums_exact<FAST>(m, O, v, bw.psum, i);
      if (redo) s = exact;
    }
  }
  const bool finite = stat_finite(s, KIND);
  float n = 0.0f, rinv = 0.0f;
  if (finite) {
    if (KIND == kNormL2) {
      norm_and_inverse(s, n, rinv);
    } else {
      n = __double2float_rn(s);
      rinv = inverse_of(n);
    }
  }
  if (!finite) atomicOr(a.status, kStatusNonFinite);
  if (n > 0.0f && n < kFltMin) atomicOr(a.status, kStatusTinyNorm);
  {
    const unsigned long long bits = finite ? (unsigned long long)__double_as_longlong(s) : 0x7FF0000000000000ull;
    best = bits > best ? bits : best;
  }
  unsigned int wf = 0u;
  if (ex != kTypeSkip && finite && rinv != 0.0f)
    wf = (unsigned int)fmin(floor(ldexp(weight_of(s, KIND), 23 - ex)), 1073741824.0);
  if (r == 0) {
    bw.norm[8 * hf + bb] = n;
    bw.inv[8 * hf + bb] = rinv;
    bw.wfix[8 * hf + bb] = wf;
    trailer[8 * hf + bb] = n;
  }
  if (i < 16) bw.pnorm[i] = prev_trailer ? prev_trailer[i] : 0.0f;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// quantize_block with the block's own (bucket) norm, reciprocal and previous norm; the tables hold plain levels.
constexpr int kBucketHistCopies = 4;   // power of two

template <int C1, bool PREV>
__device__ __forceinline__ void quantize_block_b(const float (&x)[4], const unsigned int (&o)[4], int half, float inv,
                                                 float norm, float pnorm, const unsigned char *lut, const float4 *tab,
                                                 const float *tprev, unsigned int (&D)[C1],
                                                 const unsigned int (&Dp)[C1], float &acc, unsigned int wfix,
                                                 unsigned long long *lh) {
  float u[4];
  int tau[4];
  float4 lv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    u[j] = __builtin_amdgcn_fmed3f(fabsf(x[j]) * inv, 0.0f, 1.0f);
    tau[j] = lut[f2u(u[j]) >> 20];
  }
  if (wfix != 0u) {   // a bucket with weight: the fit's grid histogram (integer adds)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if ((f2u(x[j]) & 0x7FF00000u) == 0u) continue;   // raw magnitude bin 0; also the +0 padding past the layer's end
      // u <= 1, so its bin never exceeds the last grid index: only the lower clamp is needed (saturating subtract)
      const unsigned int g = __builtin_elementwise_sub_sat(f2u(u[j]) >> 20, (unsigned int)kGridBase);
      atomicAdd(&lh[g * kBucketHistCopies], (unsigned long long)wfix);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) lv[j] = tab[tau[j]];
  if (__ballot((lv[0].z <= u[0]) | (lv[1].z <= u[1]) | (lv[2].z <= u[2]) | (lv[3].z <= u[3])) != 0ull) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      while (lv[j].z <= u[j]) { ++tau[j]; lv[j] = tab[tau[j]]; }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int jl = 4 * half + j;
    const unsigned int w16 = half ? (o[j] >> 16) : (o[j] & 0xFFFFu);
    const float xi = (u[j] - lv[j].x) * lv[j].y;
    const bool up = (float)w16 < __builtin_fmaf(xi, 65536.0f, -0.5f);
    const unsigned int h = (unsigned int)tau[j] + (up ? 1u : 0u);
    const float mag = norm * (up ? lv[j].z : lv[j].x);
    const float cur = __builtin_copysignf(mag, x[j]);
    insert_code<C1>(D, (h << 1) | (f2u(x[j]) >> 31), 24 + jl);
    float diff = cur;
    if (PREV) {
      const float pl = lds_float_at(tprev, extract_off<C1>(Dp, jl));   // +-level of the previous code
      const float pv = pnorm * pl;
      diff = cur - pv;
    }
    acc = __builtin_fmaf(diff, diff, acc);
  }
}

template <int C1, bool FAST, bool PREV, int KIND>
__device__ __forceinline__ void quantize_octet_b(const Dev &a, const LayerMeta &m, int l, int k, long long O,
                                                 const float *__restrict__ v, unsigned char *body,
                                                 const unsigned char *prevbody, const unsigned char *lut,
                                                 const float4 *tab, const float *tprev, BucketWave &bw, int i,
                                                 float &acc, int ex, unsigned long long &best,
                                                 unsigned long long *lh) {
  constexpr long long OS = 256 * C1 + 64;   // bytes per octet: codes, then the 16 bucket norms
  const unsigned int k0 = (unsigned int)a.seed, k1 = (unsigned int)(a.seed >> 32);
  unsigned char *oct = body + O * OS;
  const unsigned char *poct = prevbody ? prevbody + O * OS : nullptr;
  bucket_norms<FAST, KIND>(a, m, O, v, reinterpret_cast<float *>(oct + 256 * C1),
                     poct ? reinterpret_cast<const float *>(poct + 256 * C1) : nullptr, bw, i, ex, best);
  unsigned int D[C1], Dp[C1];
#pragma unroll
  for (int r = 0; r < C1; ++r) { D[r] = 0u; Dp[r] = 0u; }
  if (PREV && poct != nullptr) load_record<C1>(poct, i, Dp);
  float xa[4] = {0.0f, 0.0f, 0.0f, 0.0f}, xb[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (FAST) {
    load_block_fast(v, O * 8, i, xa);
    load_block_fast(v, O * 8 + 1, i, xb);
  }
  const int hf8 = (i >> 5) * 8;
#pragma unroll 1
  for (int pp = 0; pp < 4; ++pp) {
    const long long B0 = O * 8 + 2 * pp;
    shift_out_pair<C1>(D);
    if (FAST || B0 < m.nblk) {
      float x0[4], x1[4];
      if (FAST) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { x0[j] = xa[j]; x1[j] = xb[j]; }
        if (pp < 3) {
          load_block_fast(v, B0 + 2, i, xa);
          load_block_fast(v, B0 + 3, i, xb);
        }
      } else {
        load4(v, B0 * kBlockCoords + 4 * i, m.d, x0);
#pragma unroll
        for (int j = 0; j < 4; ++j) x1[j] = 0.0f;
        if (B0 + 1 < m.nblk) load4(v, (B0 + 1) * kBlockCoords + 4 * i, m.d, x1);
      }
      const float2 nn = *reinterpret_cast<const float2 *>(&bw.norm[hf8 + 2 * pp]);
      const float2 ii = *reinterpret_cast<const float2 *>(&bw.inv[hf8 + 2 * pp]);
      const float2 pn = *reinterpret_cast<const float2 *>(&bw.pnorm[hf8 + 2 * pp]);
      unsigned int o[4];
      philox4x32_10((unsigned int)((B0 >> 1) * 64 + i), (unsigned int)l, a.round, (unsigned int)k, k0, k1, o);
      const uint2 wf = *reinterpret_cast<const uint2 *>(&bw.wfix[hf8 + 2 * pp]);   // fit statistics: the buckets' weights
      quantize_block_b<C1, PREV>(x0, o, 0, ii.x, nn.x, pn.x, lut, tab, tprev, D, Dp, acc, wf.x, lh);
      quantize_block_b<C1, PREV>(x1, o, 1, ii.y, nn.y, pn.y, lut, tab, tprev, D, Dp, acc, wf.y, lh);
    }
    if (PREV) shift_out_pair<C1>(Dp);
  }
  store_record<C1>(oct, i, D);
}

template <int C1, bool PREV, int KIND>
__global__ void __launch_bounds__(kThreads) k_quantize_b(Dev a) {
  __shared__ unsigned char lut[kLutSize];
  __shared__ float4 tab[kMaxPoints];
  __shared__ float tprev[2 * kMaxPoints];   // +-level of the previous message, indexed by code = sign | h << 1
  __shared__ double red[kThreads];
  __shared__ BucketWave bws[kThreads / 64];
  // fit statistics of this run: weighted grid histogram, one copy per lane residue (a wave's lanes that meet in a
  // bin then collide a quarter as often), copies of a bin side by side
  __shared__ unsigned long long lh[kGridPoints * kBucketHistCopies];
  __shared__ unsigned long long wmax[kThreads / 64];
  // a workgroup takes a run of up to kSuperTile consecutive tiles of one layer: the tables are set up and the
  // statistics flushed once per run
  const int4 st = a.stiles[blockIdx.x];
  const int l = st.x;
  const int k = a.node0 + blockIdx.y;
  const LayerMeta m = a.meta[l];
  if (m.planes != C1) return;
  const int t = threadIdx.x;
  const float *lev = a.lev + (size_t)m.type * kMaxPoints;
  const float *rg = a.rgap + (size_t)m.type * kMaxPoints;
  reinterpret_cast<unsigned int *>(lut)[t] = reinterpret_cast<const unsigned int *>(a.lut + (size_t)m.type * kLutSize)[t];
  const int kr = k - a.row0;   // row in the pointer tables and in the per-tile scratch; the fit statistics use k
  const unsigned char *prevmsg = (a.prev != nullptr) ? a.prev[kr] : nullptr;
  const int ex = a.type_exp[m.type];
  if (t < m.S) {
    const float lj = lev[t];
    const float ln = (t + 1 < m.S) ? lev[t + 1] : __builtin_inff();
    tab[t] = make_float4(lj, (t + 1 < m.S) ? rg[t] : 0.0f, ln, 0.0f);
  }
  if (st.y == 0) {   // header of this layer: the norm entry is unused under bucket scope
    float *h = reinterpret_cast<float *>(a.msg[kr] + m.hdr_off);
    for (int j = t; j <= m.S; j += kThreads) h[j] = (j == 0) ? 0.0f : lev[j - 1];
  }
  for (int c = t; c < (1 << m.planes); c += kThreads) {
    float pl = 0.0f;
    if (prevmsg) {
      const float *hp = reinterpret_cast<const float *>(prevmsg + m.hdr_off);
      const float lvl = hp[1 + min(c >> 1, m.S - 1)];
      pl = (c & 1) ? -lvl : lvl;
    }
    tprev[c] = pl;
  }
  for (int j = t; j < kGridPoints * kBucketHistCopies; j += kThreads) lh[j] = 0ull;
  __syncthreads();
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int i = t & 63;
  unsigned long long *lhc = lh + (i & (kBucketHistCopies - 1));   // this lane's copy
  const float *__restrict__ v = a.grad[(size_t)kr * a.L + l];
  unsigned char *body = a.msg[kr] + m.body_off;
  const unsigned char *prevbody = prevmsg ? prevmsg + m.body_off : nullptr;
  const long long noct = (m.nblk + 7) >> 3;
  unsigned long long best = 0ull;
  for (int cc = 0; cc < st.z; ++cc) {
    const int chunk = st.y + cc;
    float acc = 0.0f;
    for (int oo = 0; oo < 2; ++oo) {
      const long long O = (long long)chunk * 8 + w * 2 + oo;
      if (O >= noct) break;
      if ((O + 1) * 2048 <= m.d)
        quantize_octet_b<C1, true, PREV, KIND>(a, m, l, k, O, v, body, prevbody, lut, tab, tprev, bws[w], i, acc, ex, best, lhc);
      else
        quantize_octet_b<C1, false, PREV, KIND>(a, m, l, k, O, v, body, prevbody, lut, tab, tprev, bws[w], i, acc, ex, best, lhc);
    }
    const double total = block_tree((double)acc, red);
    if (t == 0) a.dpartial[(size_t)kr * a.G + m.first_chunk + chunk] = total;
  }
  // statistics of the run: largest bucket sum (bit pattern of a non-negative double) and the histogram
#pragma unroll
  for (int sh = 1; sh < 64; sh *= 2) {
    const unsigned long long other = __shfl_xor(best, sh, 64);
    best = other > best ? other : best;
  }
  if (i == 0) wmax[w] = best;
  __syncthreads();
  const size_t idx = (size_t)k * a.L + l;
  if (t == 0) {
    for (int q = 1; q < kThreads / 64; ++q) best = wmax[q] > best ? wmax[q] : best;
    if (best) atomicMax(reinterpret_cast<unsigned long long *>(a.sumsq) + idx, best);
  }
  if (ex != kTypeSkip) {
    unsigned long long *gh = reinterpret_cast<unsigned long long *>(a.hist + idx * kHistBins);
    for (int j = t; j < kGridPoints; j += kThreads) {
      unsigned long long c = 0ull;
#pragma unroll
      for (int q = 0; q < kBucketHistCopies; ++q) c += lh[j * kBucketHistCopies + q];
      if (c) atomicAdd(&gh[j], c);
    }
  }
}

// delta_k: slot j takes the node's tiles j, j+256, ... (all layers, in order), then the halving tree.
__global__ void __launch_bounds__(kThreads) k_delta_finalize(Dev a) {
  __shared__ double red[kThreads];
  const int k = a.node0 + blockIdx.x;
  const int kr = k - a.row0;   // row in the per-node scratch and pointer tables
  const double *p = a.dpartial + (size_t)kr * a.G;
  double acc = 0.0;
  // the loads of a slot are independent of its running sum: requested 16 at a time, added in the slot's order
  int g = threadIdx.x;
  for (; g + 15 * kThreads < a.G; g += 16 * kThreads) {
    double v[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) v[q] = p[g + q * kThreads];
#pragma unroll
    for (int q = 0; q < 16; ++q) acc = acc + v[q];
  }
  for (; g < a.G; g += kThreads) acc = acc + p[g];
  const double s = block_tree(acc, red);
  if (threadIdx.x == 0) a.delta[k] = s;
  // layers without coordinates have no tile: their header entries (norm 0, levels) are written here
  for (int q = 0; q < a.n_empty; ++q) {
    const LayerMeta m = a.meta[a.empty_layers[q]];
    float *h = reinterpret_cast<float *>(a.msg[kr] + m.hdr_off);
    const float *lev = a.lev + (size_t)m.type * kMaxPoints;
    const float n0 = (a.scope == kScopeBucket) ? 0.0f : a.norm[(size_t)kr * a.L + a.empty_layers[q]];
    for (int j = threadIdx.x; j <= m.S; j += kThreads) h[j] = (j == 0) ? n0 : lev[j - 1];
  }
}

// ------------------------------------------------------------------------------------------------ step
// eq. (general_stepsize): acc += (sum_k delta_k) / K^2 ; eta = gamma = (1 + acc)^(-1/2), taken as
// rcp_floor(sqrt_floor(1 + acc)).
__global__ void k_step_scalars(Dev a) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double sum = a.delta[0];
  for (int k = 1; k < a.K; ++k) sum = sum + a.delta[k];
  const double acc = *a.acc + sum * a.invK2;
  *a.acc = acc;
  const float eta = rcp_floor(sqrt_floor(1.0 + acc));
  a.eta[0] = eta;
  a.eta[1] = eta;
  if (a.eta_out) { a.eta_out[0] = eta; a.eta_out[1] = eta; }
}

// eq. (Alt), Sec. 6: the rates for the update of this round from the sums over the rounds before it,
//   eta = (1 + lambda + mu)^(-1/2) as rcp_floor(sqrt_floor(.)),  gamma = (1 + lambda)^(q - 1/2),
// the power built from correctly rounded fp64 operations only: r_j = sqrt(r_{j-1}), r_0 = 1 + lambda, and
// (1 + lambda)^q = product of the r_j whose binary digit of q is set (j increasing).  Then lambda takes this
// round's sum_k ||Vhat_k||^2 / K^2 (the quantizer's distance output against an all-zero previous message).
__global__ void k_alt_scalars(Dev a) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const double lambda = a.alt_sums[0], mu = a.alt_sums[1];
  const float eta_prev = a.eta_out[0];
  const float eta = rcp_floor(sqrt_floor(1.0 + lambda + mu));
  const double base = 1.0 + lambda;
  double r = base, p = 1.0;
  for (int j = 1; j <= 32; ++j) {
    r = __dsqrt_rn(r);
    if ((a.q_digits >> (32 - j)) & 1u) p = p * r;
  }
  const float gamma = (float)__ddiv_rn(p, __dsqrt_rn(base));
  a.eta[0] = eta;
  a.eta[1] = gamma;
  a.eta[2] = eta_prev;
  a.eta_out[0] = eta;
  a.eta_out[1] = gamma;
  double sum = a.delta[0];
  for (int k = 1; k < a.K; ++k) sum = sum + a.delta[k];
  a.alt_sums[0] = lambda + sum * a.invK2;
}

// mu += ||X_t - X_{t+1}||^2: slot j takes the tiles j, j+256, ... (all layers, in order), then the halving tree.
__global__ void __launch_bounds__(kThreads) k_alt_finalize(Dev a) {
  __shared__ double red[kThreads];
  double acc = 0.0;
  int g = threadIdx.x;
  for (; g + 15 * kThreads < a.G; g += 16 * kThreads) {   // loads 16 at a time, sums in the slot's order
    double v[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) v[q] = a.dpartial[g + q * kThreads];
#pragma unroll
    for (int q = 0; q < 16; ++q) acc = acc + v[q];
  }
  for (; g < a.G; g += kThreads) acc = acc + a.dpartial[g];
  const double s = block_tree(acc, red);
  if (threadIdx.x == 0) a.alt_sums[1] = a.alt_sums[1] + s;
}

// DECODE + K-way mean (+ eq. (ODA) update unless MODE is kDecodeMean): one pass over Y, X_1 and the K messages.
// One octet per wave at a time: 32 running sums per lane, K records of C1 words, then 8 blocks of state.
// Under kDecodeUpdateAlt the lane also rebuilds X_t = X_1 + eta_prev * Y_t and adds (X_t - X_{t+1})^2 to its
// slot's fp32 fused chain (coordinates in increasing order, as in the quantizer's distance term).
// The 8 bucket norms a lane needs from one octet's trailer (its half's, blocks 0..7): two 128-bit loads.
__device__ __forceinline__ void load_bucket_norms(const unsigned char *trailer, int i, float (&n)[8]) {
  const auto *g = reinterpret_cast<const __attribute__((address_space(1))) v4f *>(as_global(trailer)) + 2 * (i >> 5);
  const v4f a = g[0], b = g[1];
  n[0] = a.x; n[1] = a.y; n[2] = a.z; n[3] = a.w; n[4] = b.x; n[5] = b.y; n[6] = b.z; n[7] = b.w;
}

template <int C1, int MODE, bool FAST, bool BUCKET>
__device__ __forceinline__ void decode_octet(const Dev &a, const LayerMeta &m, int l, long long O, const float *T, int i,
                                             float eta, float gamma, float eta_prev, float &accx) {
  constexpr int TS = 1 << C1;   // table entries per node, indexed by code = sign | h << 1
  constexpr long long OS = 256 * C1 + (BUCKET ? 64 : 0);   // bytes per octet (bucket scope: codes + 16 norms)
  const long long boff = m.body_off + O * OS;
  float sum[32];
  unsigned int Dc[C1], Dn[C1];
  float nc[8], nn[8];   // bucket scope: this node's and the next node's bucket norms for the lane's 8 blocks
  load_record<C1>(a.msgs_in[0] + boff, i, Dc);
  if (BUCKET) load_bucket_norms(a.msgs_in[0] + boff + 256 * C1, i, nc);
  for (int k = 0; k < a.K; ++k) {
#pragma unroll
    for (int r = 0; r < C1; ++r) Dn[r] = 0u;
    if (k + 1 < a.K) {
      load_record<C1>(a.msgs_in[k + 1] + boff, i, Dn);
      if (BUCKET) load_bucket_norms(a.msgs_in[k + 1] + boff + 256 * C1, i, nn);
    }
    const float *Tk = T + k * TS;
#pragma unroll
    for (int jj = 0; jj < 32; ++jj) {
      float val = lds_float_at(Tk, extract_off<C1>(Dc, jj));   // layer / vector scope: +-norm_k * level
      if (BUCKET) val = nc[jj >> 2] * val;                     // bucket scope: the table holds +-level
      sum[jj] = (k == 0) ? val : sum[jj] + val;
    }
#pragma unroll
    for (int r = 0; r < C1; ++r) Dc[r] = Dn[r];
    if (BUCKET) {
#pragma unroll
      for (int b = 0; b < 8; ++b) nc[b] = nn[b];
    }
  }
#pragma unroll
  for (int bb = 0; bb < 8; ++bb) {
    const long long B = O * 8 + bb;
    if (FAST || B < m.nblk) {
      const long long e = B * kBlockCoords + 4 * i;
      const long long dlim = FAST ? e + 4 : m.d;   // FAST: the whole block is inside the layer
      float mean[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) mean[j] = sum[4 * bb + j] * a.invK;
      if (MODE == kDecodeMean) {
        store4(a.mean_out[l], e, dlim, mean);
      } else if (MODE == kDecodeExtrapolate) {   // out = x - gamma * mean (x in a.x1, out in a.x_half)
        float x[4], out[4];
        load4(a.x1[l], e, dlim, x);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float gm = gamma * mean[j];
          out[j] = x[j] - gm;
        }
        store4(a.x_half[l], e, dlim, out);
      } else {
        float y[4], x1[4], xn[4], xh[4];
        load4(a.y[l], e, dlim, y);      // coordinates past the end of the layer read as 0 and add nothing below
        load4(a.x1[l], e, dlim, x1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float xt = 0.0f;
          if (MODE == kDecodeUpdateAlt) {
            const float ey_old = eta_prev * y[j];
            xt = x1[j] + ey_old;
          }
          y[j] = y[j] - mean[j];
          const float ey = eta * y[j];
          xn[j] = x1[j] + ey;
          const float gm = gamma * mean[j];
          xh[j] = xn[j] - gm;
          if (MODE == kDecodeUpdateAlt) {
            const float diff = xt - xn[j];
            accx = __builtin_fmaf(diff, diff, accx);
          }
        }
        store4(a.y[l], e, dlim, y);
        store4(a.x_half[l], e, dlim, xh);
        if (a.x_next) store4(a.x_next[l], e, dlim, xn);
      }
    }
  }
}

// The decode pass runs best in short workgroups of one octet per wave (measured against one tile per workgroup of
// four waves with two octets each: 6 % faster at K = 8, 4 % at K = 16): a workgroup has blockDim / 64 waves (1, 2 or 4)
// and takes that many consecutive octets of a tile.  Only the (Alt) variant keeps one workgroup of four waves per
// tile, two octets per wave: its squared-distance term is defined per slot and tile (a slot's chain runs through both
// octets of its wave).
template <int C1, int MODE, bool BUCKET>
__global__ void __launch_bounds__(kThreads) k_decode(Dev a) {
  extern __shared__ float T[];   // [K][2^C1]: +-norm_k * level_h (bucket scope: +-level_h) from the K message headers
  __shared__ double red[MODE == kDecodeUpdateAlt ? kThreads : 1];
  constexpr bool WHOLE = MODE == kDecodeUpdateAlt;
  const int nw = blockDim.x >> 6;
  const int PARTS = WHOLE ? 1 : 8 / nw;   // workgroups per tile
  const int g = blockIdx.x / PARTS, part = blockIdx.x - g * PARTS;
  const int2 tile = a.tiles[g];
  const int l = tile.x;
  const LayerMeta m = a.meta[l];
  if (m.planes != C1) return;
  const int TS = 1 << C1;
  for (int idx = threadIdx.x; idx < a.K * TS; idx += blockDim.x) {
    const int k = idx / TS, c = idx - k * TS;
    const float *hp = reinterpret_cast<const float *>(a.msgs_in[k] + m.hdr_off);
    const float lvl = hp[1 + min(c >> 1, m.S - 1)];
    const float mag = BUCKET ? lvl : hp[0] * lvl;
    T[idx] = (c & 1) ? -mag : mag;
  }
  __syncthreads();
  const int t = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int i = t & 63;
  float eta = 0.0f, gamma = 0.0f, eta_prev = 0.0f, accx = 0.0f;
  if (MODE == kDecodeUpdate || MODE == kDecodeUpdateAlt) { eta = a.eta[0]; gamma = a.eta[1]; }
  if (MODE == kDecodeUpdateAlt) eta_prev = a.eta[2];
  if (MODE == kDecodeExtrapolate) gamma = a.gamma_in[0];
  const long long noct = (m.nblk + 7) >> 3;
  for (int oo = 0; oo < (WHOLE ? 2 : 1); ++oo) {
    const long long O = (long long)tile.y * 8 + (WHOLE ? w * 2 + oo : part * nw + w);
    if (O >= noct) break;
    if ((O + 1) * 2048 <= m.d) decode_octet<C1, MODE, true, BUCKET>(a, m, l, O, T, i, eta, gamma, eta_prev, accx);
    else decode_octet<C1, MODE, false, BUCKET>(a, m, l, O, T, i, eta, gamma, eta_prev, accx);
  }
  if (MODE == kDecodeUpdateAlt) {
    const double total = block_tree((double)accx, red);
    if (t == 0) a.dpartial[g] = total;
  }
}

// ------------------------------------------------------------------------------------------------ code lengths
// Occurrences of every level index in the K messages, per type (the empirical p_j of Thm 5.3).  Every code of every
// octet is counted, padding included (index 0): the host subtracts the padding.  Each lane counts into its own column
// of a shared-memory table [index][lane], so no two lanes of a wave ever meet on an address.
template <int C1, bool BUCKET>
__global__ void __launch_bounds__(kThreads) k_index_hist(Dev a) {
  extern __shared__ unsigned int cnt[];   // [2^(C1-1)][64]
  constexpr int NI = 1 << (C1 - 1);
  constexpr long long OS = 256 * C1 + (BUCKET ? 64 : 0);
  const int4 st = a.stiles[blockIdx.x];   // a run of up to kSuperTile tiles of one layer: one flush per run
  const int l = st.x, k = blockIdx.y;
  const LayerMeta m = a.meta[l];
  if (m.planes != C1) return;
  const int t = threadIdx.x, w = t >> 6, i = t & 63;
  for (int q = t; q < NI * 64; q += kThreads) cnt[q] = 0u;
  __syncthreads();
  const long long noct = (m.nblk + 7) >> 3;
  for (int cc = 0; cc < st.z; ++cc)
    for (int oo = 0; oo < 2; ++oo) {
      const long long O = (long long)(st.y + cc) * 8 + w * 2 + oo;
      if (O >= noct) break;
      unsigned int D[C1];
      load_record<C1>(a.msgs_in[k] + m.body_off + O * OS, i, D);
#pragma unroll
      for (int jj = 0; jj < 32; ++jj) {
        const unsigned int h = extract_code<C1>(D, jj) >> 1;
        atomicAdd(&cnt[h * 64 + i], 1u);
      }
    }
  __syncthreads();
  for (int h = t; h < NI; h += kThreads) {
    unsigned long long sum = 0ull;
    for (int q = 0; q < 64; ++q) sum += cnt[h * 64 + ((q + h) & 63)];
    if (sum) atomicAdd(&a.index_counts[(size_t)m.type * 256 + h], sum);
  }
}

// ------------------------------------------------------------------------------------------------ level fit
// Largest squared norm of a type -> its binary exponent (fixed-point scale of the weights lambda_z).
__global__ void __launch_bounds__(kThreads) k_fit_typemax(Dev a) {
  __shared__ double red[kThreads];
  __shared__ int bad[1];
  const int mtype = blockIdx.x;
  if (threadIdx.x == 0) bad[0] = 0;
  for (int j = threadIdx.x; j < kGridPoints; j += kThreads) a.pooled[(size_t)mtype * kGridPoints + j] = 0ull;
  __syncthreads();
  double mx = 0.0;   // largest weight ||v||_q^2 of the type
  for (int idx = threadIdx.x; idx < a.K * a.L; idx += kThreads) {
    const int l = idx % a.L;
    if (a.meta[l].type != mtype) continue;
    const double s = a.sumsq[idx];
    if (!stat_finite(s, a.kind)) bad[0] = 1;
    else mx = fmax(mx, weight_of(s, a.kind));
  }
  red[threadIdx.x] = mx;
  __syncthreads();
  for (int h = kThreads / 2; h >= 1; h >>= 1) {
    if (threadIdx.x < h) red[threadIdx.x] = fmax(red[threadIdx.x], red[threadIdx.x + h]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double smax = red[0];
    int ex = kTypeSkip;
    if (!bad[0] && smax > 0.0) ex = (int)((__double_as_longlong(smax) >> 52) & 0x7FF) - 1023;
    a.type_exp[mtype] = ex;
  }
}

// Re-bin one (node, layer) histogram onto the normalised grid with weight floor(||v||_q^2 * 2^(23 - exponent)).
__global__ void __launch_bounds__(kThreads) k_fit_pool(Dev a) {
  const int l = blockIdx.x, k = blockIdx.y;
  const LayerMeta m = a.meta[l];
  const int ex = a.type_exp[m.type];
  if (ex == kTypeSkip) return;
  const size_t idx = (size_t)k * a.L + l;
  const unsigned long long wfix = (unsigned long long)floor(ldexp(weight_of(a.sumsq[idx], a.kind), 23 - ex));
  const float inv = a.inv[idx];
  if (wfix == 0ull || inv == 0.0f) return;
  const unsigned int *cnt = a.hist + idx * kHistBins;
  unsigned long long *W = a.pooled + (size_t)m.type * kGridPoints;
  for (int b = threadIdx.x; b < kHistBins; b += kThreads) {
    if (b == 0) continue;
    const unsigned int c = cnt[b];
    if (c == 0u) continue;
    const float mid = u2f(((unsigned int)b << 20) | (1u << 19));
    const float uc = fminf(mid * inv, 1.0f);
    int j = (int)(f2u(uc) >> 20) - kGridBase;
    j = max(0, min(j, kGridPoints - 1));
    atomicAdd(&W[j], wfix * (unsigned long long)c);
  }
}

// ---- level fit under bucket scope from given vectors: two passes over them (scale of the weights, then histogram).
// Statistic of the lane's bucket (half of block B) by the in-order binary tree, valid in all its 32 lanes.  Every lane
// of the wave must call this.
__device__ __forceinline__ double half_block_stat(const LayerMeta &m, const float *__restrict__ v, long long B, int i,
                                                  float (&x)[4], int kind) {
  const long long e = B * kBlockCoords + 4 * i;
#pragma unroll
  for (int j = 0; j < 4; ++j) x[j] = 0.0f;
  if (e < m.d) load4(v, e, m.d, x);
  if (kind == kNormLinf) {   // largest magnitude of the bucket
    unsigned int mb = 0u;
#pragma unroll
    for (int j = 0; j < 4; ++j) mb = max(mb, f2u(x[j]) & 0x7FFFFFFFu);
    double s = (double)magnitude_from_bits(mb);
#pragma unroll
    for (int w = 1; w < 32; w *= 2) s = fmax(s, __shfl_xor(s, w, 64));
    return s;
  }
  float acc = 0.0f;
  if (kind == kNormL2) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_fmaf(x[j], x[j], acc);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = acc + fabsf(x[j]);
  }
  double s = (double)acc;
#pragma unroll
  for (int w = 1; w < 32; w *= 2) s = s + __shfl_xor(s, w, 64);
  if (kind == kNormL2) {
    // below 2^-100 (squares may have vanished) or not finite (they may have overflowed): exact fp64 squares instead
    const bool redo = !(s >= kBucketRescueBelow) || !(s <= 1.7976931348623157e308);
    if (__ballot(redo) != 0ull) {
      double acc64 = 0.0;
#pragma unroll
      for (int j = 0; j < 4; ++j) acc64 = __builtin_fma((double)x[j], (double)x[j], acc64);
#pragma unroll
      for (int w = 1; w < 32; w *= 2) acc64 = acc64 + __shfl_xor(acc64, w, 64);
      if (redo) s = acc64;
    }
  }
  return s;
}

// Largest bucket statistic of every (node, layer), as the bit pattern of a non-negative double (ordered like
// an integer); one that is not a finite number in range leaves +infinity.  a.sumsq must be zero on entry.
__global__ void __launch_bounds__(kThreads) k_bucket_max(Dev a) {
  __shared__ unsigned long long wmax[kThreads / 64];
  const int4 st = a.stiles[blockIdx.x];
  const int l = st.x, k = blockIdx.y;
  const LayerMeta m = a.meta[l];
  const float *__restrict__ v = a.grad[(size_t)k * a.L + l];
  const int t = threadIdx.x, w = t >> 6, i = t & 63;
  unsigned long long best = 0ull;
  for (int cc = 0; cc < st.z; ++cc)
    for (int oo = 0; oo < 2; ++oo) {
      const long long O = (long long)(st.y + cc) * 8 + w * 2 + oo;
      for (int bb = 0; bb < 8; ++bb) {
        const long long B = O * 8 + bb;
        if (B >= m.nblk) break;   // the same for every lane of the wave
        float x[4];
        const double s = half_block_stat(m, v, B, i, x, a.kind);
        const bool finite = stat_finite(s, a.kind);
        const unsigned long long bits = finite ? (unsigned long long)__double_as_longlong(s) : 0x7FF0000000000000ull;
        best = bits > best ? bits : best;
      }
    }
  // both halves of the wave, then the four waves
  const unsigned long long other = __shfl_xor(best, 32, 64);
  best = other > best ? other : best;
  if (i == 0) wmax[w] = best;
  __syncthreads();
  if (t == 0) {
    for (int q = 1; q < kThreads / 64; ++q) best = wmax[q] > best ? wmax[q] : best;
    if (best) atomicMax(reinterpret_cast<unsigned long long *>(a.sumsq) + ((size_t)k * a.L + l), best);
  }
}

// Weighted histogram of the normalised magnitudes of the coordinates of every (node, layer) on the 257-point
// grid: weight floor(bucket sum * 2^(23 - exponent of the type)), integer adds, kept per (node, layer) in the first
// 257 64-bit words of its histogram area.
__global__ void __launch_bounds__(kThreads) k_bucket_hist(Dev a) {
  __shared__ unsigned long long lh[kGridPoints];
  const int4 st = a.stiles[blockIdx.x];
  const int l = st.x, k = blockIdx.y;
  const LayerMeta m = a.meta[l];
  const int ex = a.type_exp[m.type];
  if (ex == kTypeSkip) return;
  const float *__restrict__ v = a.grad[(size_t)k * a.L + l];
  const int t = threadIdx.x, w = t >> 6, i = t & 63;
  for (int j = t; j < kGridPoints; j += kThreads) lh[j] = 0ull;
  __syncthreads();
  for (int cc = 0; cc < st.z; ++cc)
    for (int oo = 0; oo < 2; ++oo) {
      const long long O = (long long)(st.y + cc) * 8 + w * 2 + oo;
      for (int bb = 0; bb < 8; ++bb) {
        const long long B = O * 8 + bb;
        if (B >= m.nblk) break;   // the same for every lane of the wave
        float x[4];
        const double s = half_block_stat(m, v, B, i, x, a.kind);
        const unsigned long long wfix = (unsigned long long)floor(ldexp(weight_of(s, a.kind), 23 - ex));
        const float inv = rcp_floor(norm_of(s, a.kind));
        if (wfix == 0ull || inv == 0.0f) continue;
        const long long e = B * kBlockCoords + 4 * i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (e + j >= m.d || ((f2u(x[j]) & 0x7FFFFFFFu) >> 20) == 0u) continue;
          const float uc = fminf(fabsf(x[j]) * inv, 1.0f);
          int g = (int)(f2u(uc) >> 20) - kGridBase;
          g = max(0, min(g, kGridPoints - 1));
          atomicAdd(&lh[g], wfix);
        }
      }
    }
  __syncthreads();
  unsigned long long *gh = reinterpret_cast<unsigned long long *>(a.hist + ((size_t)k * a.L + l) * kHistBins);
  for (int j = t; j < kGridPoints; j += kThreads) {
    const unsigned long long c = lh[j];
    if (c) atomicAdd(&gh[j], c);
  }
}

// Pool the per-(node, layer) grid histograms of a type.
__global__ void __launch_bounds__(kThreads) k_fit_pool_b(Dev a) {
  const int l = blockIdx.x, k = blockIdx.y;
  const LayerMeta m = a.meta[l];
  if (a.type_exp[m.type] == kTypeSkip) return;
  const unsigned long long *gh = reinterpret_cast<const unsigned long long *>(a.hist + ((size_t)k * a.L + l) * kHistBins);
  unsigned long long *W = a.pooled + (size_t)m.type * kGridPoints;
  for (int j = threadIdx.x; j < kGridPoints; j += kThreads) {
    const unsigned long long c = gh[j];
    if (c) atomicAdd(&W[j], c);
  }
}

__device__ __forceinline__ float grid_value(int j) { return u2f((unsigned int)(j + kGridBase) << 20); }

// Search tables of one type from its levels (in shared memory): reciprocal gaps and the bin -> index table.
__device__ void build_tables(const Dev &a, int mtype, int S, const float *slev) {
  float *rg = a.rgap + (size_t)mtype * kMaxPoints;
  unsigned char *lut = a.lut + (size_t)mtype * kLutSize;
  for (int j = threadIdx.x; j < kMaxPoints; j += (int)blockDim.x) rg[j] = (j < S - 1) ? rcp_floor(slev[j + 1] - slev[j]) : 0.0f;
  // entry q serves the values whose bit pattern >> 20 is q: tau at the lower edge of that bin.
  for (int q = threadIdx.x; q < kLutSize; q += (int)blockDim.x) {
    const float lo = u2f((unsigned int)q << 20);
    int tau = 0;
    if (q > 1016) {
      tau = S - 2;
    } else {
      for (int j = 1; j <= S - 2; ++j)
        if (slev[j] <= lo) tau = j;
    }
    lut[q] = (unsigned char)tau;
  }
}

__global__ void __launch_bounds__(kThreads) k_build_tables(Dev a, int mtype) {
  __shared__ float slev[kMaxPoints];
  const int S = a.type_points[mtype];
  for (int j = threadIdx.x; j < S; j += kThreads) slev[j] = a.lev[(size_t)mtype * kMaxPoints + j];
  __syncthreads();
  build_tables(a, mtype, S, slev);
}

// Exact minimisation of eq. (Qada2) over interior levels on the grid by dynamic programming; one workgroup per type.
// cost(a, b) = sum over bins i in [a, b) of W_i (g_b - mid_i)(mid_i - g_a), from prefix sums P0, P1, P2 of W, W*mid,
// W*mid^2 taken sequentially in increasing bin (fp64; the same operation order as the CPU checker).
struct __attribute__((aligned(32))) FitRow { double p0, p1, p2, g; };

__device__ __forceinline__ double fit_cost(const FitRow &ra, const FitRow &rb) {
  return ((ra.g + rb.g) * (rb.p1 - ra.p1) - (rb.p2 - ra.p2)) - (ra.g * rb.g) * (rb.p0 - ra.p0);
}

constexpr int kFitThreads = 1024;
constexpr int kFitLdsPoints = 128;  // up to this many level points the back-pointers stay in shared memory
// The cost of a pair (a, b) does not depend on the stage, so every thread computes the costs of its pairs once and
// keeps them in registers: grid index b (1..255, the only places an interior level can sit) has its b candidates
// a = 0..b-1 cut into segments of kFitSeg, one thread per segment -- 945 threads, at most kFitSeg costs each.  A stage
// is then one shared-memory read, one addition and one comparison per pair, and a second step in which the first
// thread of every b combines its segments in increasing a.
constexpr int kFitSeg = 40;
constexpr int kFitPad = 320;        // D rows are padded with +infinity: a segment may reach index 240 + 39

__global__ void __launch_bounds__(kFitThreads) k_fit_dp(Dev a) {
  __shared__ FitRow row[kGridPoints + 1];
  __shared__ double D[2][kFitPad];
  __shared__ double pbest[kFitThreads];   // first the per-bin terms of the prefix sums, then the segments' minima
  __shared__ int pa[kFitThreads];         // ... and where they are taken
  __shared__ float slev[kMaxPoints];
  __shared__ unsigned char sarg[kFitLdsPoints * 256];   // back-pointers of the stages, when S is small enough
  static_assert(3 * kGridPoints <= kFitThreads, "the per-bin terms share the segments' array");
  double (*wd)[kGridPoints] = reinterpret_cast<double (*)[kGridPoints]>(pbest);   // W, W*mid, (W*mid)*mid per bin
  double *rv = pbest;   // the last stage's candidates: after the stage loop
  int *ri = pa;
  const int mtype = blockIdx.x;
  if (a.type_exp[mtype] == kTypeSkip) return;   // all-zero or non-finite vectors: the type keeps its levels
  const int S = a.type_points[mtype];
  const int t = threadIdx.x;
  const unsigned long long *W = a.pooled + (size_t)mtype * kGridPoints;
  const int last = kGridPoints - 1;
  const double inf = __longlong_as_double(0x7FF0000000000000ll);
  for (int j = t; j < kGridPoints; j += kFitThreads) {
    const double wj = (double)W[j];
    const double mid = (j == last) ? 1.0 : (double)u2f(((unsigned int)(j + kGridBase) << 20) | (1u << 19));
    const double wm = wj * mid;
    wd[0][j] = wj;
    wd[1][j] = wm;
    wd[2][j] = wm * mid;
    row[j].g = (double)grid_value(j);
  }
  for (int j = t; j < 2 * kFitPad; j += kFitThreads) D[0][j] = inf;   // both rows: index 0, index `last`, the padding
  __syncthreads();
  // the three running sums, each by one thread of its own wave, bin after bin
  if ((t & 63) == 0 && t < 3 * 64) {
    const int f = t >> 6;
    const double *src = wd[f];
    double *dst = &row[0].p0 + f;   // p0, p1, p2 are the first three doubles of a row
    double p = 0.0;
    dst[0] = 0.0;
#pragma unroll 8
    for (int j = 0; j < kGridPoints; ++j) {
      p = p + src[j];
      dst[4 * (j + 1)] = p;
    }
    if (f == 0) row[kGridPoints].g = 0.0;
  }
  __syncthreads();
  if (row[kGridPoints].p0 == 0.0) return;   // no mass on the grid at all: the type keeps its levels
  short *arg = a.dp_arg + a.dp_arg_off[mtype];
  const bool lds_arg = S <= kFitLdsPoints;   // candidates a are at most 254: a byte each, 255 for "none"
  if (S > 2) {
    // level 1 at grid index b: cost of the bins below g_b against the levels 0 and g_b
    for (int b = t; b < kGridPoints; b += kFitThreads)
      D[1][b] = (b >= 1 && b <= last - (S - 2)) ? (row[b].g * row[b].p1 - row[b].p2) : inf;
    // this thread's grid index b, segment and number of segments of b (b = 0: no work): the indices
    // 40(g-1)+1 .. 40g have g segments each
    int b = 0, seg = 0, nseg = 0;
    {
      int base = 0;
      for (int g = 1; (g - 1) * kFitSeg + 1 <= last - 1; ++g) {
        const int r0 = (g - 1) * kFitSeg + 1, r1 = min(g * kFitSeg, last - 1);
        const int cnt = (r1 - r0 + 1) * g;
        if (t >= base && t < base + cnt) {
          const int o = t - base;
          b = r0 + o / g;
          seg = o - (o / g) * g;
          nseg = g;
        }
        base += cnt;
      }
    }
    const int a0 = seg * kFitSeg;
    double cost[kFitSeg];
    {
      const FitRow rb = row[b];
#pragma unroll
      for (int j = 0; j < kFitSeg; ++j) {
        const int aa = a0 + j;
        const FitRow ra = row[min(aa, last)];
        cost[j] = (aa <= b - 1) ? fit_cost(ra, rb) : inf;   // +infinity never wins a comparison below
        __builtin_amdgcn_sched_barrier(0);   // one pair at a time: 40 rows in flight would not fit the registers
      }
    }
    __syncthreads();
    for (int s = 2; s <= S - 2; ++s) {
      // D of the previous stage is +infinity wherever level s-1 cannot sit (in particular below index s-1), so the
      // candidates need no range test: min over a of D[a] + cost(a, b), the smallest a on equal cost
      const double *Dp = D[(s - 1) & 1] + a0;
      double *Dc = D[s & 1];
      double best = inf;
      int bj = 0;
#pragma unroll
      for (int j = 0; j < kFitSeg; ++j) {
        const double c = Dp[j] + cost[j];   // never a NaN: costs and D are finite or +infinity
        bj = (c < best) ? j : bj;
        best = fmin(best, c);
      }
      pbest[t] = best;
      pa[t] = a0 + bj;
      __syncthreads();
      if (b != 0 && seg == 0) {
        int besta = pa[t];
        for (int q = 1; q < nseg; ++q) {   // later segments hold larger a: they win only with a smaller cost
          const double ov = pbest[t + q];
          if (ov < best) { best = ov; besta = pa[t + q]; }
        }
        if (!(b >= s && b <= last - (S - 1 - s))) best = inf;   // level s cannot sit here
        Dc[b] = best;
        if (lds_arg) sarg[s * 256 + b] = (unsigned char)(best < inf ? besta : 255);
        else arg[(size_t)s * kGridPoints + b] = (short)(best < inf ? besta : -1);
      }
      __syncthreads();
    }
    // last level (1.0) at grid index `last`: one candidate per thread, then the smallest cost (ties: smallest index)
    {
      const double *Dp = D[(S - 2) & 1];
      double c = inf;
      if (t < kThreads && t >= S - 2 && t <= last - 1) {
        const FitRow ra = row[t], rb = row[last];
        c = Dp[t] + fit_cost(ra, rb);
      }
      if (t < kThreads) {
        rv[t] = c;
        ri[t] = (c < inf) ? t : 0x7FFFFFFF;
      }
      __syncthreads();
      for (int h = kThreads / 2; h >= 1; h >>= 1) {
        if (t < h) {
          const double ov = rv[t + h];
          const int oi = ri[t + h];
          if (ov < rv[t] || (ov == rv[t] && oi < ri[t])) { rv[t] = ov; ri[t] = oi; }
        }
        __syncthreads();
      }
    }
  }
  if (t == 0) {
    slev[0] = 0.0f;
    slev[S - 1] = 1.0f;
    if (S > 2) {
      int b = ri[0];
      for (int s = S - 2; s >= 1; --s) {
        b = max(1, min(b, last - 1));   // cannot trigger for finite costs; keeps a corrupted table in bounds
        slev[s] = grid_value(b);
        if (s >= 2) b = lds_arg ? (int)sarg[s * 256 + b] : (int)arg[(size_t)s * kGridPoints + b];
      }
    }
    for (int j = 0; j < S; ++j) a.lev[(size_t)mtype * kMaxPoints + j] = slev[j];
  }
  __syncthreads();
  build_tables(a, mtype, S, slev);
}

// ------------------------------------------------------------------------------------------------ calibration
// Plain 128-bit copy of n float4: the known-size kernel that hardware byte counters are calibrated against.
__global__ void __launch_bounds__(kThreads) k_copy_f4(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

// Streaming with the access type of the three big kernels: a workgroup takes tiles of 64 KiB; every thread issues 16
// nontemporal 128-bit loads per tile (1 KiB contiguous per wave and load) and STORES nontemporal 128-bit stores of
// values derived from them.  STORES = 0 measures the read-only ceiling (the norm pass), 16 a copy, values between
// the read/write mixes of the quantize pass (about 2) and of the decode + update pass (about 9).
template <int STORES>
__global__ void __launch_bounds__(kThreads) k_stream(const float *__restrict__ src, float *__restrict__ dst, size_t tiles,
                                                     float *sink) {
  const int t = threadIdx.x;
  float keep = 0.0f;
  for (size_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const size_t base = tile * kChunkCoords + (size_t)(t >> 6) * 16 * kBlockCoords + 4 * (t & 63);
    v4f q[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const auto *lp = reinterpret_cast<const __attribute__((address_space(1))) v4f *>(as_global(src) + base + (size_t)s * kBlockCoords);
      q[s] = __builtin_nontemporal_load(lp);
    }
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      if (s < STORES) {
        auto *sp = reinterpret_cast<__attribute__((address_space(1))) v4f *>((__attribute__((address_space(1))) float *)dst + base + (size_t)s * kBlockCoords);
        __builtin_nontemporal_store(q[s], sp);
      } else {
        keep += (q[s].x + q[s].y) + (q[s].z + q[s].w);
      }
    }
  }
  if (keep == 12345.678f) sink[0] = keep;   // keeps the loads alive; practically never true
}

// ------------------------------------------------------------------------------------------------ staging
// Small host arrays (pointer tables, level values) reach the device as kernel arguments and are written to their device
// table by the kernel itself: no staging buffer, no copy engine, no host memory that must outlive the call.
constexpr int kPackWords = 256;
struct WordPack { unsigned int w[kPackWords]; };

__global__ void __launch_bounds__(kPackWords) k_stage_words(unsigned int *dst, WordPack pack, int n) {
  const int t = threadIdx.x;
  if (t < n) dst[t] = pack.w[t];
}

// ------------------------------------------------------------------------------------------------ launchers
hipError_t launch_stage_words(void *dst_dev, const void *src_host, size_t nwords, hipStream_t s) {
  const unsigned int *src = static_cast<const unsigned int *>(src_host);
  unsigned int *dst = static_cast<unsigned int *>(dst_dev);
  for (size_t q = 0; q < nwords; q += kPackWords) {
    WordPack pack;
    const int m = (int)(nwords - q < (size_t)kPackWords ? nwords - q : (size_t)kPackWords);
    for (int j = 0; j < kPackWords; ++j) pack.w[j] = j < m ? src[q + j] : 0u;
    hipLaunchKernelGGL(k_stage_words, dim3(1), dim3(kPackWords), 0, s, dst + q, pack, m);
  }
  return hipGetLastError();
}

hipError_t launch_stage_pointers(void **dst_dev, const void *const *src_host, size_t n, hipStream_t s) {
  static_assert(sizeof(void *) == 2 * sizeof(unsigned int), "a pointer is two words");
  return launch_stage_words(dst_dev, src_host, 2 * n, s);
}

hipError_t launch_copy(const void *src, void *dst, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return hipSuccess;
  const size_t want = (n + kThreads * 4 - 1) / (kThreads * 4);
  const unsigned int blocks = (unsigned int)(want < 1048576 ? want : 1048576);
  hipLaunchKernelGGL(k_copy_f4, dim3(blocks), dim3(kThreads), 0, s, reinterpret_cast<const float4 *>(src),
                     reinterpret_cast<float4 *>(dst), n);
  return hipGetLastError();
}

hipError_t launch_stream(const void *src, void *dst, size_t bytes, int stores, void *sink, hipStream_t s) {
  const size_t tiles = bytes / (4 * (size_t)kChunkCoords);
  if (tiles == 0) return hipSuccess;
  const dim3 grid((unsigned int)(tiles < 65536 ? tiles : 65536)), block(kThreads);
  const float *a = static_cast<const float *>(src);
  float *b = static_cast<float *>(dst), *k = static_cast<float *>(sink);
  switch (stores) {
    case 0: hipLaunchKernelGGL((k_stream<0>), grid, block, 0, s, a, b, tiles, k); break;
    case 1: hipLaunchKernelGGL((k_stream<1>), grid, block, 0, s, a, b, tiles, k); break;
    case 2: hipLaunchKernelGGL((k_stream<2>), grid, block, 0, s, a, b, tiles, k); break;
    case 4: hipLaunchKernelGGL((k_stream<4>), grid, block, 0, s, a, b, tiles, k); break;
    case 8: hipLaunchKernelGGL((k_stream<8>), grid, block, 0, s, a, b, tiles, k); break;
    case 16: hipLaunchKernelGGL((k_stream<16>), grid, block, 0, s, a, b, tiles, k); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_zero_u32(unsigned int *p, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const unsigned int blocks = (unsigned int)((n + 1023) / 1024 < 65535 ? (n + 1023) / 1024 : 65535);
  hipLaunchKernelGGL(k_zero_u32, dim3(blocks), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

template <int KIND>
static void launch_sumsq_kind(const Dev &a, bool with_hist, hipStream_t s) {
  const dim3 grid(a.GS, a.nnodes), block(kThreads);
  if (with_hist) hipLaunchKernelGGL((k_sumsq<true, KIND>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((k_sumsq<false, KIND>), grid, block, 0, s, a);
}

hipError_t launch_sumsq(const Dev &a, bool with_hist, hipStream_t s) {
  if (a.GS == 0 || a.nnodes == 0) return hipSuccess;
  if (a.kind == kNormL2) launch_sumsq_kind<kNormL2>(a, with_hist, s);
  else if (a.kind == kNormL1) launch_sumsq_kind<kNormL1>(a, with_hist, s);
  else launch_sumsq_kind<kNormLinf>(a, with_hist, s);
  return hipGetLastError();
}

hipError_t launch_norm_finalize(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_norm_finalize, dim3(a.L, a.nnodes), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

// planes_mask: bit p set when some layer has code width p (2..9); one launch per width present.
template <int C1>
static void launch_quantize_width(const Dev &a, hipStream_t s) {
  const dim3 block(kThreads);
  const bool prev = a.prev != nullptr;   // no node has a previous message: the kernels skip that half of the work
  if (a.scope == kScopeBucket) {
    const dim3 grid(a.GS, a.nnodes);   // runs of tiles
    if (a.kind == kNormL2) {
      if (prev) hipLaunchKernelGGL((k_quantize_b<C1, true, kNormL2>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((k_quantize_b<C1, false, kNormL2>), grid, block, 0, s, a);
    } else if (a.kind == kNormL1) {
      if (prev) hipLaunchKernelGGL((k_quantize_b<C1, true, kNormL1>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((k_quantize_b<C1, false, kNormL1>), grid, block, 0, s, a);
    } else {
      if (prev) hipLaunchKernelGGL((k_quantize_b<C1, true, kNormLinf>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((k_quantize_b<C1, false, kNormLinf>), grid, block, 0, s, a);
    }
  } else {
    const dim3 grid(a.G, a.nnodes);
    if (prev) hipLaunchKernelGGL((k_quantize<C1, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((k_quantize<C1, false>), grid, block, 0, s, a);
  }
}

hipError_t launch_quantize(const Dev &a, unsigned int planes_mask, hipStream_t s) {
  if (a.G == 0 || a.nnodes == 0) return hipSuccess;
  if (planes_mask & (1u << 2)) launch_quantize_width<2>(a, s);
  if (planes_mask & (1u << 3)) launch_quantize_width<3>(a, s);
  if (planes_mask & (1u << 4)) launch_quantize_width<4>(a, s);
  if (planes_mask & (1u << 5)) launch_quantize_width<5>(a, s);
  if (planes_mask & (1u << 6)) launch_quantize_width<6>(a, s);
  if (planes_mask & (1u << 7)) launch_quantize_width<7>(a, s);
  if (planes_mask & (1u << 8)) launch_quantize_width<8>(a, s);
  if (planes_mask & (1u << 9)) launch_quantize_width<9>(a, s);
  return hipGetLastError();
}

hipError_t launch_delta_finalize(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_delta_finalize, dim3(a.nnodes), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_norm_vector(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_norm_vector, dim3(a.nnodes), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_step_scalars(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_step_scalars, dim3(1), dim3(64), 0, s, a);
  return hipGetLastError();
}

template <int C1, bool BUCKET>
static void launch_decode_scope(const Dev &a, int mode, size_t lds_bytes, hipStream_t s) {
  const dim3 whole(a.G), block(kThreads);                                           // one workgroup per tile
  // short workgroups: two waves, four where the K decode tables are large enough to limit the workgroups per CU
  const int nw = lds_bytes > 8192 ? 4 : kDecodeWaves;
  const dim3 parts((unsigned int)a.G * (8 / nw)), small(64 * nw);
  if (mode == kDecodeExtrapolate) hipLaunchKernelGGL((k_decode<C1, kDecodeExtrapolate, BUCKET>), parts, small, lds_bytes, s, a);
  else if (mode == kDecodeUpdateAlt) hipLaunchKernelGGL((k_decode<C1, kDecodeUpdateAlt, BUCKET>), whole, block, lds_bytes, s, a);
  else if (mode == kDecodeUpdate) hipLaunchKernelGGL((k_decode<C1, kDecodeUpdate, BUCKET>), parts, small, lds_bytes, s, a);
  else hipLaunchKernelGGL((k_decode<C1, kDecodeMean, BUCKET>), parts, small, lds_bytes, s, a);
}

template <int C1>
static void launch_decode_width(const Dev &a, int mode, size_t lds_bytes, hipStream_t s) {
  if (a.scope == kScopeBucket) launch_decode_scope<C1, true>(a, mode, lds_bytes, s);
  else launch_decode_scope<C1, false>(a, mode, lds_bytes, s);
}

hipError_t launch_decode(const Dev &a, int mode, unsigned int planes_mask, hipStream_t s) {
  if (a.G == 0) return hipSuccess;
  if (planes_mask & (1u << 2)) launch_decode_width<2>(a, mode, (size_t)a.K * 4 * sizeof(float), s);
  if (planes_mask & (1u << 3)) launch_decode_width<3>(a, mode, (size_t)a.K * 8 * sizeof(float), s);
  if (planes_mask & (1u << 4)) launch_decode_width<4>(a, mode, (size_t)a.K * 16 * sizeof(float), s);
  if (planes_mask & (1u << 5)) launch_decode_width<5>(a, mode, (size_t)a.K * 32 * sizeof(float), s);
  if (planes_mask & (1u << 6)) launch_decode_width<6>(a, mode, (size_t)a.K * 64 * sizeof(float), s);
  if (planes_mask & (1u << 7)) launch_decode_width<7>(a, mode, (size_t)a.K * 128 * sizeof(float), s);
  if (planes_mask & (1u << 8)) launch_decode_width<8>(a, mode, (size_t)a.K * 256 * sizeof(float), s);
  if (planes_mask & (1u << 9)) launch_decode_width<9>(a, mode, (size_t)a.K * 512 * sizeof(float), s);
  return hipGetLastError();
}

template <int C1>
static void launch_index_hist_width(const Dev &a, hipStream_t s) {
  const dim3 grid(a.GS, a.K), block(kThreads);
  const size_t lds = (size_t)(1 << (C1 - 1)) * 64 * sizeof(unsigned int);
  if (a.scope == kScopeBucket) hipLaunchKernelGGL((k_index_hist<C1, true>), grid, block, lds, s, a);
  else hipLaunchKernelGGL((k_index_hist<C1, false>), grid, block, lds, s, a);
}

hipError_t launch_index_hist(const Dev &a, unsigned int planes_mask, hipStream_t s) {
  if (a.G == 0) return hipSuccess;
  if (planes_mask & (1u << 2)) launch_index_hist_width<2>(a, s);
  if (planes_mask & (1u << 3)) launch_index_hist_width<3>(a, s);
  if (planes_mask & (1u << 4)) launch_index_hist_width<4>(a, s);
  if (planes_mask & (1u << 5)) launch_index_hist_width<5>(a, s);
  if (planes_mask & (1u << 6)) launch_index_hist_width<6>(a, s);
  if (planes_mask & (1u << 7)) launch_index_hist_width<7>(a, s);
  if (planes_mask & (1u << 8)) launch_index_hist_width<8>(a, s);
  if (planes_mask & (1u << 9)) launch_index_hist_width<9>(a, s);
  return hipGetLastError();
}

hipError_t launch_alt_scalars(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_alt_scalars, dim3(1), dim3(64), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_alt_finalize(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_alt_finalize, dim3(1), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bucket_max(const Dev &a, hipStream_t s) {
  if (a.GS == 0) return hipSuccess;
  hipLaunchKernelGGL(k_bucket_max, dim3(a.GS, a.K), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_bucket_hist(const Dev &a, hipStream_t s) {
  if (a.GS == 0) return hipSuccess;
  hipLaunchKernelGGL(k_bucket_hist, dim3(a.GS, a.K), dim3(kThreads), 0, s, a);
  hipLaunchKernelGGL(k_fit_pool_b, dim3(a.L, a.K), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_fit_pool_b(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_fit_pool_b, dim3(a.L, a.K), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_fit_typemax(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_fit_typemax, dim3(a.M), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_fit_pool(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_fit_pool, dim3(a.L, a.K), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_fit_dp(const Dev &a, hipStream_t s) {
  hipLaunchKernelGGL(k_fit_dp, dim3(a.M), dim3(kFitThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_build_tables(const Dev &a, int type, hipStream_t s) {
  hipLaunchKernelGGL(k_build_tables, dim3(1), dim3(kThreads), 0, s, a, type);
  return hipGetLastError();
}

}  // namespace qoda
