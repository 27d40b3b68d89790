// QODA CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// A plain, single-threaded, deliberately slow C++17 implementation of the per-round hot path of
// Quantized Optimistic Dual Averaging with layer-wise unbiased stochastic quantization
// (arXiv 2505.14371).  It exists so that the GPU library can be checked against something that a
// reader can verify against the paper by eye.  It shares no code with the GPU library; only tests,
// the smoke check and the bench's cpu_baseline leg may call it.
//
// What follows the paper, and where:
//   * vector representation (norm, signs, normalised magnitudes u_i)          -- Sec. 2.2
//   * level index tau(u), relative distance xi(u), random rounding q_l(u),
//     Q(v_i) = ||v|| * sign(v_i) * q_l(u_i), coordinates drawn independently  -- Sec. 3.1
//   * ENCODE / DECODE: 32-bit float norm, one sign bit, fixed-width level
//     index per coordinate (no entropy code, as in the experiments)           -- Sec. 3.2, App. C.1
//   * level fit: minimise sum_i int (l_{i+1}-u)(u-l_i) dF~(u), F~ the
//     norm^2-weighted pooled CDF of the sampled dual vectors                  -- Sec. 3.2, eq. (Qada2) and
//                                                                                 the weights lambda_z
//   * optimistic dual averaging update and adaptive step size                -- Sec. 4, eq. (ODA),
//                                                                                 eq. (general_stepsize), Alg. 1
//   * the alternative pair of step sizes lagged by two rounds                  -- Sec. 6, eq. (Alt)
//   * norm scopes (whole vector, buckets of 128), the extra-gradient leg,
//     index counts and code lengths (fixed width, entropy, Huffman)            -- Sec. 2.2, Sec. 7, Sec. 4,
//                                                                                 Thm 5.3 / App. C
//   * L^q normalisation for q = 1 and q -> infinity beside q = 2 (statistic,
//     norm, fit weight ||v||_q^2)                                              -- Sec. 2.2, Thm 5.1, eq. (Qada2)
//
// Pin status (see tests/test_oracle_*.py): every function below is pinned to something the paper or the
// mathematics fixes; the Philox generator also against the published known-answer vectors of its authors.
// The level fit minimises the paper's objective exactly on a histogram grid; the paper delegates the
// optimiser itself to third-party code it does not describe, so optimality relative to that code is
// "parity unpinned".
//
// Where the contract below is narrower than the textbook definition (step-size term, bucket sums, the histogram of
// the fit) the plain definition is at the end of this file, and the tests bound one against the other.
//
// Arithmetic contract (the GPU library follows the same written contract independently):
//   fp32 operations are single IEEE operations, never fused; sums that feed integer decisions are
//   taken in fp64 in a fixed "slot + halving tree" order; square roots and reciprocals that feed
//   integer decisions are defined by exact comparisons (largest float whose square / product does not
//   exceed the argument), so they do not depend on how well a sqrt or divide instruction rounds.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC qoda_oracle.cpp -o libqoda_oracle.so

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

constexpr int64_t kBlock = 256;     // coordinates per block (64 lanes x 4 consecutive coordinates)
constexpr int64_t kOctet = 2048;    // coordinates per packed record group (8 blocks)
constexpr int64_t kChunk = 16384;   // coordinates per reduction chunk (64 blocks)
constexpr int64_t kBucket = 128;    // coordinates per bucket when every bucket carries its own norm (Sec. 7)
// What one norm covers (Sec. 2.2 normalises "the vector"; Sec. 3 quantizes layer by layer; the experiments of
// Sec. 7 normalise buckets of 128 entries): a layer, the node's whole dual vector, or a bucket.
enum Scope { kScopeLayer = 0, kScopeVector = 1, kScopeBucket = 2 };
constexpr int kSlots = 256;         // reduction slots per chunk
constexpr int kHistBins = 2048;     // histogram bins on the top 11 magnitude bits of a float
constexpr int kGridBase = 760;      // (127-32)<<3 : bin of 2^-32 on the normalised grid
constexpr int kGridPoints = 257;    // normalised grid g_0=2^-32 ... g_256=1

inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float u2f(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

inline int index_bits(int S) {   // b = ceil(log2 S), at least 1
  int b = 1;
  while ((1 << b) < S) ++b;
  return b;
}

// ----- Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), written from the published construction.
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const uint64_t p0 = M0 * (uint64_t)c0;
    const uint64_t p1 = M1 * (uint64_t)c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The 16-bit uniform integer that decides coordinate e of (layer, round, node).
// One generator call serves 8 coordinates: the same lane position (e mod 256)/4 of two consecutive
// 256-coordinate blocks; the even block takes the low halves of the four output words, the odd block
// the high halves; word index = e mod 4.
uint32_t draw16(uint64_t seed, uint32_t round, uint32_t node, uint32_t layer, uint64_t e) {
  const uint32_t ctr[4] = {(uint32_t)(((e >> 9) << 6) | ((e >> 2) & 63u)), layer, round, node};
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  philox4x32_10(ctr, key, out);
  const uint32_t w = out[e & 3];
  return ((e >> 8) & 1) ? (w >> 16) : (w & 0xFFFFu);
}

// ----- canonical fp64 reductions.
// slot of coordinate e inside its chunk: block B = (e mod 16384)/256, slot = 64*(B/16) + (e mod 256)/4.
inline int slot_of(int64_t e) {
  const int64_t ec = e % kChunk;
  const int64_t B = ec / kBlock;
  return (int)(64 * (B / 16) + (ec % kBlock) / 4);
}

double halving_tree(double *p) {   // p has kSlots entries; destroys p
  for (int h = kSlots / 2; h >= 1; h /= 2)
    for (int i = 0; i < h; ++i) p[i] = p[i] + p[i + h];
  return p[0];
}

// Combine per-chunk sums: slot j takes chunks j, j+256, ... in increasing order, then the tree.
double combine_chunks(const std::vector<double> &chunk_sums) {
  double p[kSlots];
  for (int j = 0; j < kSlots; ++j) p[j] = 0.0;
  for (size_t c = 0; c < chunk_sums.size(); ++c) p[c % kSlots] = p[c % kSlots] + chunk_sums[c];
  return halving_tree(p);
}

// per-chunk sums of squares of one layer (products are exact in fp64).
void chunk_sumsq(const float *v, int64_t d, std::vector<double> &out) {
  const int64_t nchunks = (d + kChunk - 1) / kChunk;
  for (int64_t c = 0; c < nchunks; ++c) {
    double p[kSlots];
    for (int j = 0; j < kSlots; ++j) p[j] = 0.0;
    const int64_t e1 = std::min(d, (c + 1) * kChunk);
    for (int64_t e = c * kChunk; e < e1; ++e) {
      const double x = (double)v[e];
      p[slot_of(e)] = p[slot_of(e)] + x * x;
    }
    out.push_back(halving_tree(p));
  }
}

// ----- L^q normalisation (Sec. 2.2: u_i = |v_i| / ||v||_q).  Three kinds are defined here, named by q:
// kNormL2 (q = 2), kNormL1 (q = 1) and kNormLinf (the limit q -> infinity, stored as 0).  Each has a statistic s that
// is reduced over the vector (sum of squares, sum of magnitudes, largest magnitude), the norm derived from it, and
// the weight ||v||_q^2 that eq. (Qada2) gives the vector in the level fit.
constexpr int kNormLinf = 0, kNormL1 = 1, kNormL2 = 2;

// largest magnitude of v as a double; +infinity if an entry is an infinity or not a number (the integer order of the
// magnitude bits puts those above every finite value)
double max_magnitude(const float *v, int64_t d) {
  uint32_t mb = 0;
  for (int64_t e = 0; e < d; ++e) mb = std::max(mb, f2u(v[e]) & 0x7FFFFFFFu);
  return mb > 0x7F7FFFFFu ? std::numeric_limits<double>::infinity() : (double)u2f(mb);
}

// per-chunk sums of magnitudes of one layer, in the slot order of the sums of squares
void chunk_sumabs(const float *v, int64_t d, std::vector<double> &out) {
  const int64_t nchunks = (d + kChunk - 1) / kChunk;
  for (int64_t c = 0; c < nchunks; ++c) {
    double p[kSlots];
    for (int j = 0; j < kSlots; ++j) p[j] = 0.0;
    const int64_t e1 = std::min(d, (c + 1) * kChunk);
    for (int64_t e = c * kChunk; e < e1; ++e) p[slot_of(e)] = p[slot_of(e)] + (double)std::fabs(v[e]);
    out.push_back(halving_tree(p));
  }
}

// the statistic of one layer
double layer_stat(const float *v, int64_t d, int kind) {
  if (kind == kNormLinf) return max_magnitude(v, d);
  std::vector<double> cs;
  if (kind == kNormL1) chunk_sumabs(v, d, cs);
  else chunk_sumsq(v, d, cs);
  return combine_chunks(cs);
}

// statistics of parts -> statistic of the whole (vector scope combines its layers with this)
double combine_stats(const std::vector<double> &parts, int kind) {
  if (kind != kNormLinf) return combine_chunks(parts);
  double m = 0.0;
  for (double x : parts) m = (x > m || x != x) ? x : m;
  return m;
}

// a statistic whose norm is a finite float
bool stat_finite(double s, int kind) {
  const double fmax = (double)std::numeric_limits<float>::max();
  return (s >= 0.0) && (s <= (kind == kNormL2 ? fmax * fmax : fmax));
}

// largest float n >= 0 with n*n <= s (n*n is exact in fp64).  s must be finite and >= 0.
float sqrt_floor(double s) {
  if (!(s >= 0.0) || !(s <= (double)std::numeric_limits<float>::max() * (double)std::numeric_limits<float>::max()))
    return 0.0f;   // caller flags non-finite
  double r = std::sqrt(s);
  float n = (r >= (double)std::numeric_limits<float>::max()) ? std::numeric_limits<float>::max() : (float)r;
  for (int it = 0; it < 4 && (double)n * (double)n > s; ++it) n = u2f(f2u(n) - 1);
  for (int it = 0; it < 4; ++it) {
    if (n == std::numeric_limits<float>::max()) break;
    const float up = u2f(f2u(n) + 1);
    if ((double)up * (double)up <= s) n = up; else break;
  }
  return n;
}

// largest finite float r >= 0 with x*r <= 1 (x*r is exact in fp64); 0 for x <= 0 or non-finite x.
float rcp_floor(float x) {
  if (!(x > 0.0f) || std::isinf(x)) return 0.0f;
  float r = 1.0f / x;
  if (std::isinf(r)) r = std::numeric_limits<float>::max();
  for (int it = 0; it < 4 && (double)x * (double)r > 1.0; ++it) r = u2f(f2u(r) - 1);
  for (int it = 0; it < 4; ++it) {
    if (r == std::numeric_limits<float>::max()) break;
    const float up = u2f(f2u(r) + 1);
    if ((double)x * (double)up <= 1.0) r = up; else break;
  }
  return r;
}

// norm of a vector from its (finite) statistic: the floor root of a sum of squares; a sum of magnitudes rounded to
// the nearest float (one IEEE conversion); a largest magnitude is a float already
float norm_of(double s, int kind) { return kind == kNormL2 ? sqrt_floor(s) : (float)s; }

// ||v||_q^2 as a double: the sum of squares itself, else the statistic squared (one rounding)
double weight_of(double s, int kind) { return kind == kNormL2 ? s : s * s; }

// tau(u) = largest j in [0, S-2] with level[j] <= u   (Sec. 3.1; at u = 1 the last interval is taken)
int level_index(const float *lev, int S, float u) {
  int tau = 0;
  for (int j = 1; j <= S - 2; ++j)
    if (lev[j] <= u) tau = j;
  return tau;
}

struct Code { uint8_t sign; uint8_t h; };

// Q of one coordinate (Sec. 2.2 + Sec. 3.1): u = min(|v| * inv, 1); tau; xi; round up iff draw < xi.
Code quantize_coord(float v, float inv, const float *lev, int S, uint32_t w16) {
  const float u = std::fmin(std::fabs(v) * inv, 1.0f);
  const int tau = level_index(lev, S, u);
  const float rgap = rcp_floor(lev[tau + 1] - lev[tau]);
  const float xi = (u - lev[tau]) * rgap;
  const bool up = ((float)w16 + 0.5f) < xi * 65536.0f;
  Code c;
  c.sign = (uint8_t)(f2u(v) >> 31);
  c.h = (uint8_t)(tau + (up ? 1 : 0));
  return c;
}

inline float decode_value(uint8_t sign, int h, float norm, const float *lev, int S) {
  if (h > S - 1) h = S - 1;
  const float t = norm * lev[h];
  return sign ? -t : t;
}

// ----- message layout.
struct Layout {
  int L;
  int scope;
  std::vector<int64_t> d, noct, hdr_off, msg_off, ostride;   // ostride: bytes per octet of a layer's body
  std::vector<int> S, planes;
  int64_t header_bytes, message_bytes;
  int64_t total_chunks;
};

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// bytes of one octet of the body: 256*c1 bytes of codes, plus (bucket scope) the octet's 16 bucket norms
inline int64_t octet_stride(int planes, int scope) { return 256 * (int64_t)planes + (scope == kScopeBucket ? 64 : 0); }

Layout make_layout(int L, const int64_t *d, const int32_t *S, int scope) {
  Layout lay;
  lay.L = L;
  lay.scope = scope;
  int64_t h = 0;
  for (int l = 0; l < L; ++l) {
    lay.d.push_back(d[l]);
    lay.S.push_back(S[l]);
    lay.planes.push_back(1 + index_bits(S[l]));
    lay.noct.push_back((d[l] + kOctet - 1) / kOctet);
    lay.ostride.push_back(octet_stride(lay.planes[l], scope));
    lay.hdr_off.push_back(h);
    h += 4 * (1 + (int64_t)S[l]);
  }
  lay.header_bytes = round_up(h, 256);
  int64_t off = lay.header_bytes;
  int64_t chunks = 0;
  for (int l = 0; l < L; ++l) {
    lay.msg_off.push_back(off);
    off += lay.noct[l] * lay.ostride[l];
    chunks += (d[l] + kChunk - 1) / kChunk;
  }
  lay.message_bytes = round_up(off, 256);
  lay.total_chunks = chunks;
  return lay;
}

// Packed body of a layer (fixed width, c1 = 1 + b bits per coordinate, code = sign | index << 1).
// Coordinates are grouped in octets of 8 blocks (2048 coordinates).  Inside an octet, "lane" i = (e mod 256)/4
// owns the 32 coordinates {256*bb + 4*i + j : bb = 0..7, j = 0..3}, numbered jj = 4*bb + j; their codes form a
// little-endian bit string of 32*c1 bits (code jj at bits [c1*jj, c1*jj + c1)), i.e. c1 32-bit words per lane.
// Word r of lane i of octet O is the 32-bit word number O*64*c1 + r*64 + i of the layer's body, so that the 64
// lanes' words r are contiguous.  Padding coordinates carry code 0.
// Bucket scope: the 256*c1 code bytes of every octet are followed by its 16 bucket norms (fp32).  The bucket of
// block bb (0..7) and half hf (0: lanes 0..31, i.e. coordinates 0..127 of the block; 1: the rest) sits at position
// 8*hf + bb, so that the 8 norms a lane needs are contiguous.
inline void set_bit(uint8_t *layer_base, int c1, int64_t ostride, int64_t e, int t, bool v) {
  const int64_t O = e / kOctet;
  const int bb = (int)((e % kOctet) / kBlock), i = (int)((e % kBlock) / 4), j = (int)(e % 4);
  const int P = c1 * (4 * bb + j) + t;
  uint32_t *w = reinterpret_cast<uint32_t *>(layer_base + O * ostride) + ((int64_t)(P / 32) * 64 + i);
  if (v) *w |= (uint32_t)1 << (P % 32);
}
inline int get_bit(const uint8_t *layer_base, int c1, int64_t ostride, int64_t e, int t) {
  const int64_t O = e / kOctet;
  const int bb = (int)((e % kOctet) / kBlock), i = (int)((e % kBlock) / 4), j = (int)(e % 4);
  const int P = c1 * (4 * bb + j) + t;
  const uint32_t *w = reinterpret_cast<const uint32_t *>(layer_base + O * ostride) + ((int64_t)(P / 32) * 64 + i);
  return (int)((*w >> (P % 32)) & 1u);
}

void put_code(uint8_t *layer_base, int planes, int64_t ostride, int64_t e, Code c) {
  set_bit(layer_base, planes, ostride, e, 0, c.sign != 0);
  for (int p = 1; p < planes; ++p) set_bit(layer_base, planes, ostride, e, p, ((c.h >> (p - 1)) & 1) != 0);
}

Code get_code(const uint8_t *layer_base, int planes, int64_t ostride, int64_t e) {
  Code c;
  c.sign = (uint8_t)get_bit(layer_base, planes, ostride, e, 0);
  int h = 0;
  for (int p = 1; p < planes; ++p) h |= get_bit(layer_base, planes, ostride, e, p) << (p - 1);
  c.h = (uint8_t)h;
  return c;
}

// address of the stored norm of the bucket that holds coordinate e (bucket scope only)
inline float *bucket_norm_slot(uint8_t *layer_base, int planes, int64_t ostride, int64_t e) {
  const int64_t O = e / kOctet;
  const int bb = (int)((e % kOctet) / kBlock), hf = (int)((e % kBlock) / kBucket);
  return reinterpret_cast<float *>(layer_base + O * ostride + 256 * (int64_t)planes) + (8 * hf + bb);
}

// Sum of squares of one bucket (n <= 128 coordinates, missing ones count as 0): "lane" i = (e mod 128)/4 adds the
// squares of its four consecutive coordinates in order, the 32 lane sums are combined in fp64 by the in-order binary
// tree (lanes 0+1, 2+3, ...; then pairs of those; ...).  A lane first works in single precision (fused chain
// acc = fma(x, x, acc) from 0, then widened): relative error about 1e-7, which is all a bucket norm needs.  Single
// precision loses squares below 2^-149 and overflows above 2^128, and a norm that is too small makes u = |v|/norm
// exceed 1, which the clamp would turn into a bias (Thm 5.1 needs u <= 1 unclamped).  So whenever the single-precision
// result is below 2^-100 (zero included) or not a finite number, the lanes redo their chains in fp64, where every
// square is exact: acc = fma((double)x, (double)x, acc); same tree.
double bucket_sumsq_lanes(const float *v, int64_t n, bool exact) {
  double p[32];
  for (int i = 0; i < 32; ++i) {
    float acc32 = 0.0f;
    double acc64 = 0.0;
    for (int j = 0; j < 4; ++j) {
      const int64_t e = 4 * i + j;
      const float x = (e < n) ? v[e] : 0.0f;
      if (exact) acc64 = std::fma((double)x, (double)x, acc64);
      else acc32 = std::fmaf(x, x, acc32);
    }
    p[i] = exact ? acc64 : (double)acc32;
  }
  for (int w = 1; w < 32; w *= 2)
    for (int i = 0; i < 32; i += 2 * w) p[i] = p[i] + p[i + w];
  return p[0];
}

constexpr double kBucketRescueBelow = 7.888609052210118e-31;   // 2^-100

double bucket_sumsq(const float *v, int64_t n) {
  const double s = bucket_sumsq_lanes(v, n, false);
  const bool trusted = (s >= kBucketRescueBelow) && (s <= std::numeric_limits<double>::max());
  return trusted ? s : bucket_sumsq_lanes(v, n, true);
}

// The other kinds over a bucket, lane by lane as above: a lane adds its four magnitudes in order in fp32 from 0 (the
// lane sums are widened and combined by the same in-order tree), or takes their maximum.
double bucket_stat(const float *v, int64_t n, int kind) {
  if (kind == kNormL2) return bucket_sumsq(v, n);
  if (kind == kNormLinf) return max_magnitude(v, n);
  double p[32];
  for (int i = 0; i < 32; ++i) {
    float acc = 0.0f;
    for (int j = 0; j < 4; ++j) {
      const int64_t e = 4 * i + j;
      acc = acc + ((e < n) ? std::fabs(v[e]) : 0.0f);
    }
    p[i] = (double)acc;
  }
  for (int w = 1; w < 32; w *= 2)
    for (int i = 0; i < 32; i += 2 * w) p[i] = p[i] + p[i + w];
  return p[0];
}

struct HeaderView { float norm; const float *lev; };
inline HeaderView header_of(const uint8_t *msg, const Layout &lay, int l) {
  HeaderView h;
  const float *p = reinterpret_cast<const float *>(msg + lay.hdr_off[l]);
  h.norm = p[0];
  h.lev = p + 1;
  return h;
}

inline float grid_value(int j) { return u2f((uint32_t)(j + kGridBase) << 20); }
inline double grid_mid(int j) {
  if (j == kGridPoints - 1) return 1.0;
  return (double)u2f(((uint32_t)(j + kGridBase) << 20) | (1u << 19));
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------- scalar building blocks (exposed for the pins)
void oracle_philox4x32_10(const uint32_t *ctr, const uint32_t *key, uint32_t *out) { philox4x32_10(ctr, key, out); }
uint32_t oracle_draw16(uint64_t seed, uint32_t round, uint32_t node, uint32_t layer, uint64_t e) {
  return draw16(seed, round, node, layer, e);
}
float oracle_sqrt_floor(double s) { return sqrt_floor(s); }
float oracle_rcp_floor(float x) { return rcp_floor(x); }
int32_t oracle_level_index(const float *lev, int32_t S, float u) { return level_index(lev, S, u); }
int32_t oracle_index_bits(int32_t S) { return index_bits(S); }

// canonical sum of squares of one layer (Sec. 2.2, L2 norm before the square root).
double oracle_sumsq(const float *v, int64_t d) {
  std::vector<double> cs;
  chunk_sumsq(v, d, cs);
  return combine_chunks(cs);
}

// ---------------------------------------------------------------- one layer, unpacked (Sec. 3.1)
// Quantize coordinates [e0, e1) of a layer of d entries; inv is the layer's reciprocal norm.
void oracle_quantize_range(const float *v, int64_t e0, int64_t e1, float inv, const float *lev, int32_t S,
                           uint64_t seed, uint32_t round, uint32_t node, uint32_t layer, uint8_t *sign_out,
                           uint8_t *index_out) {
  for (int64_t e = e0; e < e1; ++e) {
    const Code c = quantize_coord(v[e], inv, lev, S, draw16(seed, round, node, layer, (uint64_t)e));
    sign_out[e - e0] = c.sign;
    index_out[e - e0] = c.h;
  }
}

// Same, but with the 16-bit draw supplied by the caller (used to enumerate every outcome in the pins).
void oracle_quantize_with_draws(const float *v, int64_t n, float inv, const float *lev, int32_t S,
                                const uint32_t *w16, uint8_t *sign_out, uint8_t *index_out) {
  for (int64_t e = 0; e < n; ++e) {
    const Code c = quantize_coord(v[e], inv, lev, S, w16[e]);
    sign_out[e] = c.sign;
    index_out[e] = c.h;
  }
}

void oracle_decode(const uint8_t *sign, const uint8_t *index, int64_t n, float norm, const float *lev, int32_t S,
                   float *out) {
  for (int64_t e = 0; e < n; ++e) out[e] = decode_value(sign[e], index[e], norm, lev, S);
}

// ---------------------------------------------------------------- message layout (Sec. 3.2, fixed width)
int64_t oracle_message_bytes(int32_t L, const int64_t *d, const int32_t *S, int32_t scope) {
  return make_layout(L, d, S, scope).message_bytes;
}
int64_t oracle_header_bytes(int32_t L, const int64_t *d, const int32_t *S, int32_t scope) {
  return make_layout(L, d, S, scope).header_bytes;
}
void oracle_layout(int32_t L, const int64_t *d, const int32_t *S, int32_t scope, int64_t *hdr_off, int64_t *msg_off) {
  const Layout lay = make_layout(L, d, S, scope);
  for (int l = 0; l < L; ++l) { hdr_off[l] = lay.hdr_off[l]; msg_off[l] = lay.msg_off[l]; }
}

// pack / unpack the codes of one layer into its body (region must hold ceil(d/2048) octets of the scope's stride).
// bucket scope: norms (ceil(d/128) floats, bucket order) are stored too / returned when the pointer is not NULL.
void oracle_pack_layer(const uint8_t *sign, const uint8_t *index, int64_t d, int32_t S, int32_t scope,
                       const float *bucket_norms, uint8_t *region) {
  const int planes = 1 + index_bits(S);
  const int64_t os = octet_stride(planes, scope);
  const int64_t noct = (d + kOctet - 1) / kOctet;
  std::memset(region, 0, (size_t)(noct * os));
  for (int64_t e = 0; e < d; ++e) { Code c; c.sign = sign[e]; c.h = index[e]; put_code(region, planes, os, e, c); }
  if (scope == kScopeBucket && bucket_norms)
    for (int64_t b = 0; b * kBucket < d; ++b) *bucket_norm_slot(region, planes, os, b * kBucket) = bucket_norms[b];
}
void oracle_unpack_layer(const uint8_t *region, int64_t d, int32_t S, int32_t scope, uint8_t *sign, uint8_t *index,
                         float *bucket_norms) {
  const int planes = 1 + index_bits(S);
  const int64_t os = octet_stride(planes, scope);
  for (int64_t e = 0; e < d; ++e) { const Code c = get_code(region, planes, os, e); sign[e] = c.sign; index[e] = c.h; }
  if (scope == kScopeBucket && bucket_norms)
    for (int64_t b = 0; b * kBucket < d; ++b)
      bucket_norms[b] = *bucket_norm_slot(const_cast<uint8_t *>(region), planes, os, b * kBucket);
}

double oracle_bucket_sumsq(const float *v, int64_t n) { return bucket_sumsq(v, n); }
// the statistic of a layer / of a bucket under the given kind of norm, and the norm and fit weight it yields
double oracle_norm_stat(const float *v, int64_t d, int32_t kind) { return layer_stat(v, d, kind); }
double oracle_bucket_stat(const float *v, int64_t n, int32_t kind) { return bucket_stat(v, n, kind); }
float oracle_norm_of(double s, int32_t kind) { return stat_finite(s, kind) ? norm_of(s, kind) : 0.0f; }
double oracle_weight_of(double s, int32_t kind) { return weight_of(s, kind); }

namespace {
constexpr int32_t kTypeSkip = 0x7fffffff;   // "this type has no weight scale": nothing is gathered / fitted for it

// Status bits returned by the routines below.
constexpr int32_t kStatusNonFinite = 1;   // a statistic is not a finite number in range: its vector's output is unspecified
constexpr int32_t kStatusTinyNorm = 2;    // 0 < norm < 2^-126: 1/norm is not a float, so u = |v| * inv falls short of
                                          // |v| / norm and E[Q(v)] = v (Thm 5.1) no longer holds for that vector

// integer weight of a bucket with sum of squares s under the scale 2^ex: floor(s * 2^(23 - ex)), capped at 2^30 (a
// scale taken from the previous round can be exceeded; the cap keeps every 64-bit total far from overflow)
inline uint64_t stat_weight(double s, int ex) {
  const double w = std::floor(std::ldexp(s, 23 - ex));
  return (uint64_t)std::fmin(w, 1073741824.0);
}

// the norm DECODE uses for coordinate e of layer l: the header's (layer and vector scope) or the bucket's
inline float stored_norm(const uint8_t *msg, const Layout &lay, int l, int64_t e) {
  if (lay.scope != kScopeBucket) return header_of(msg, lay, l).norm;
  return *bucket_norm_slot(const_cast<uint8_t *>(msg) + lay.msg_off[l], lay.planes[l], lay.ostride[l], e);
}

// DECODE of coordinate e of layer l of a stored message (Sec. 3.2): +-norm * level, with the message's own levels
inline float decoded_value(const uint8_t *msg, const Layout &lay, int l, int64_t e) {
  const HeaderView h = header_of(msg, lay, l);
  const Code c = get_code(msg + lay.msg_off[l], lay.planes[l], lay.ostride[l], e);
  return decode_value(c.sign, c.h, stored_norm(msg, lay, l, e), h.lev, lay.S[l]);
}

// Norm and reciprocal from a statistic (Sec. 2.2); raises the status bits above.
struct NormPair { float norm, inv; };
inline NormPair norm_pair(double stat, int kind, int32_t *status) {
  const bool finite = stat_finite(stat, kind);
  if (!finite) *status |= kStatusNonFinite;
  NormPair n;
  n.norm = finite ? norm_of(stat, kind) : 0.0f;
  n.inv = rcp_floor(n.norm);
  if (n.norm > 0.0f && n.norm < std::numeric_limits<float>::min()) *status |= kStatusTinyNorm;
  return n;
}

// || DECODE(msg) - DECODE(msg_prev) ||^2 (eq. (general_stepsize); msg_prev NULL: zeros) in the contract's order: per
// slot an fp32 fused chain over its coordinates of a chunk in increasing order, the 256 slots widened to fp64 and
// reduced by the tree, chunks numbered through all layers and combined like chunk sums.
double delta_between(const Layout &lay, const uint8_t *msg, const uint8_t *msg_prev) {
  std::vector<double> delta_chunks;
  for (int l = 0; l < lay.L; ++l) {
    const int64_t nchunks = (lay.d[l] + kChunk - 1) / kChunk;
    for (int64_t c = 0; c < nchunks; ++c) {
      float p32[kSlots];
      for (int j = 0; j < kSlots; ++j) p32[j] = 0.0f;
      const int64_t e1 = std::min(lay.d[l], (c + 1) * kChunk);   // padding coordinates carry code 0 and add nothing
      for (int64_t e = c * kChunk; e < e1; ++e) {
        const float cur = decoded_value(msg, lay, l, e);
        const float prev = msg_prev ? decoded_value(msg_prev, lay, l, e) : 0.0f;
        const float diff = cur - prev;
        p32[slot_of(e)] = std::fmaf(diff, diff, p32[slot_of(e)]);
      }
      double p[kSlots];
      for (int j = 0; j < kSlots; ++j) p[j] = (double)p32[j];
      delta_chunks.push_back(halving_tree(p));
    }
  }
  return combine_chunks(delta_chunks);
}

// Bucket scope: the level fit's statistics of one layer, gathered from the vectors a quantize pass sees (Alg. 1 runs
// lines 3-5 before the round's vectors exist, so the estimate can only come from earlier vectors).  hist (257, added
// to) receives the weight floor(sumsq_b * 2^(23 - ex)), capped at 2^30, at the grid bin of u for every coordinate whose
// raw magnitude bin is not 0; *bmax (maximised) the largest bucket statistic, +infinity if one is not finite.
void gather_bucket_stats(const float *v, int64_t d, int32_t ex, int norm_kind, uint64_t *hist, double *bmax) {
  for (int64_t e0 = 0; e0 < d; e0 += kBucket) {
    const int64_t n = std::min<int64_t>(kBucket, d - e0);
    const double s = bucket_stat(v + e0, n, norm_kind);
    const bool finite = stat_finite(s, norm_kind);
    const double sm = finite ? s : std::numeric_limits<double>::infinity();
    if (sm > *bmax) *bmax = sm;
    if (ex == kTypeSkip || !finite) continue;
    const uint64_t wfix = stat_weight(weight_of(s, norm_kind), ex);
    const float inv = rcp_floor(norm_of(s, norm_kind));
    if (wfix == 0 || inv == 0.0f) continue;
    for (int64_t q = e0; q < e0 + n; ++q) {
      if (((f2u(v[q]) & 0x7FFFFFFFu) >> 20) == 0) continue;
      const float uc = std::fmin(std::fabs(v[q]) * inv, 1.0f);
      int j = (int)(f2u(uc) >> 20) - kGridBase;
      if (j < 0) j = 0;
      if (j > kGridPoints - 1) j = kGridPoints - 1;
      hist[j] += wfix;
    }
  }
}
}  // namespace

// ---------------------------------------------------------------- ENCODE(Q(V_k)) for one node: Alg. 1 line 12
// grads[l]  : layer l of the node's dual vector.      levels[l] : the S[l] levels of layer l's type.
// msg       : message_bytes output.                    msg_prev  : previous-round message of this node or NULL.
// scope     : what one norm covers.  Layer: the layer's canonical statistic.  Vector: the canonical combination of
//             the L layer statistics (slot j takes layers j, j+256, ...; then the tree), used by every layer.
//             Bucket: every 128 consecutive coordinates of a layer (bucket_stat); the norms travel in the body.
// sumsq_out : L statistics (may be NULL): the layer's; under vector scope the whole vector's in every entry; under
//             bucket scope the largest bucket statistic of the layer.
// delta_out : || Vhat_{k,t+1/2} - Vhat_{k,t-1/2} ||^2 (the step-size term of eq. (general_stepsize)); prev = 0 if NULL.
// layer_exp : NULL, or (bucket scope) the weight scale of every layer's type: then stats_hist (L*257, added to) and
//             stats_max (L, maximised) receive the fit statistics of these vectors (gather_bucket_stats).
// returns the status bits (0: fine).
int32_t oracle_quantize(int32_t L, const int64_t *d, const int32_t *S, const float *const *levels,
                        const float *const *grads, uint64_t seed, uint32_t round, uint32_t node, int32_t scope,
                        uint8_t *msg, const uint8_t *msg_prev, double *sumsq_out, double *delta_out,
                        const int32_t *layer_exp, uint64_t *stats_hist, double *stats_max, int32_t norm_kind) {
  const Layout lay = make_layout(L, d, S, scope);
  std::memset(msg, 0, (size_t)lay.message_bytes);
  int32_t status = 0;
  // 1. the statistic every norm is derived from (Sec. 2.2)
  std::vector<double> stat(L, 0.0);
  if (scope != kScopeBucket) {
    for (int l = 0; l < L; ++l) stat[l] = layer_stat(grads[l], d[l], norm_kind);
    if (scope == kScopeVector) stat.assign(L, combine_stats(stat, norm_kind));
  }
  for (int l = 0; l < L; ++l) {
    // 2. header: the norm in 32 bits (Sec. 3.2; unused and 0 under bucket scope), then the levels in force
    NormPair n = {0.0f, 0.0f};
    if (scope != kScopeBucket) n = norm_pair(stat[l], norm_kind, &status);
    float *hdr = reinterpret_cast<float *>(msg + lay.hdr_off[l]);
    hdr[0] = n.norm;
    for (int j = 0; j < S[l]; ++j) hdr[1 + j] = levels[l][j];
    // 3. every coordinate: Q (Sec. 3.1) with its vector's norm, then its code into the body
    uint8_t *region = msg + lay.msg_off[l];
    for (int64_t e = 0; e < d[l]; ++e) {
      if (scope == kScopeBucket && e % kBucket == 0) {   // a new bucket: its own norm, stored after the octet's codes
        const double s = bucket_stat(grads[l] + e, std::min<int64_t>(kBucket, d[l] - e), norm_kind);
        n = norm_pair(s, norm_kind, &status);
        *bucket_norm_slot(region, lay.planes[l], lay.ostride[l], e) = n.norm;
        if (stat_finite(s, norm_kind) && s > stat[l]) stat[l] = s;
      }
      const Code code = quantize_coord(grads[l][e], n.inv, levels[l], S[l], draw16(seed, round, node, (uint32_t)l, (uint64_t)e));
      put_code(region, lay.planes[l], lay.ostride[l], e, code);
    }
    if (sumsq_out) sumsq_out[l] = stat[l];
    if (scope == kScopeBucket && layer_exp)
      gather_bucket_stats(grads[l], d[l], layer_exp[l], norm_kind, stats_hist + (size_t)l * kGridPoints, &stats_max[l]);
  }
  // 4. the step-size term, from the two messages as stored
  if (delta_out) *delta_out = delta_between(lay, msg, msg_prev);
  return status;
}

// ---------------------------------------------------------------- step-size term from two stored messages
// || DECODE(msg) - DECODE(msg_prev) ||^2 in the contract's order (msg_prev NULL: zeros): what oracle_quantize returns
// as delta, for a test that holds the messages of a full-size model but cannot quantize it on the CPU.
double oracle_delta_from_messages(int32_t L, const int64_t *d, const int32_t *S, int32_t scope, const uint8_t *msg,
                                  const uint8_t *msg_prev) {
  return delta_between(make_layout(L, d, S, scope), msg, msg_prev);
}

// ---------------------------------------------------------------- DECODE + mean over the K nodes: Alg. 1 lines 15-17
// mean_out[l][e] = ((Vhat_0 + Vhat_1) + ... + Vhat_{K-1}) * (1/K), all in fp32, k increasing.
void oracle_dequant_aggregate(int32_t L, const int64_t *d, const int32_t *S, int32_t scope, int32_t K,
                              const uint8_t *const *msgs, float *const *mean_out) {
  const Layout lay = make_layout(L, d, S, scope);
  const float invK = 1.0f / (float)K;
  for (int l = 0; l < L; ++l)
    for (int64_t e = 0; e < d[l]; ++e) {
      float sum = 0.0f;
      for (int k = 0; k < K; ++k) {
        const HeaderView h = header_of(msgs[k], lay, l);
        const Code c = get_code(msgs[k] + lay.msg_off[l], lay.planes[l], lay.ostride[l], e);
        const float val = decode_value(c.sign, c.h, stored_norm(msgs[k], lay, l, e), h.lev, S[l]);
        sum = (k == 0) ? val : sum + val;
      }
      mean_out[l][e] = sum * invK;
    }
}

// ---------------------------------------------------------------- step size: eq. (general_stepsize)
// acc <- acc + (delta_0 + ... + delta_{K-1}) / K^2 ;  eta = gamma = (1 + acc)^(-1/2), taken as
// rcp_floor(sqrt_floor(1 + acc)) so that it is defined by exact comparisons.
void oracle_step_size(int32_t K, const double *delta, double *acc, float *eta_out) {
  double sum = 0.0;
  for (int k = 0; k < K; ++k) sum = (k == 0) ? delta[k] : sum + delta[k];
  const double invK2 = 1.0 / ((double)K * (double)K);
  *acc = *acc + sum * invK2;
  *eta_out = rcp_floor(sqrt_floor(1.0 + *acc));
}

// ---------------------------------------------------------------- eq. (ODA) + Alg. 1 lines 10, 17, 18
// Y <- Y - mean ; X_next = X_1 + eta * Y ; X_half = X_next - gamma * mean   (next round's extrapolated point).
void oracle_oda_update(int64_t n, const float *mean, const float *x1, float *y, float *x_next, float *x_half,
                       float eta, float gamma) {
  for (int64_t e = 0; e < n; ++e) {
    const float yn = y[e] - mean[e];
    const float ey = eta * yn;
    const float xn = x1[e] + ey;
    const float gm = gamma * mean[e];
    y[e] = yn;
    if (x_next) x_next[e] = xn;
    x_half[e] = xn - gm;
  }
}

// ---------------------------------------------------------------- code-length accounting (Sec. 5 Thm 5.3, App. C.1, C.3)
// Occurrences of every level index among the real coordinates of one message, per type: counts[m*256 + h] += 1.
void oracle_index_counts(int32_t L, const int64_t *d, const int32_t *S, const int32_t *layer_type, int32_t scope,
                         const uint8_t *msg, uint64_t *counts) {
  const Layout lay = make_layout(L, d, S, scope);
  for (int l = 0; l < L; ++l)
    for (int64_t e = 0; e < d[l]; ++e) {
      const Code c = get_code(msg + lay.msg_off[l], lay.planes[l], lay.ostride[l], e);
      counts[(size_t)layer_type[l] * 256 + c.h] += 1;
    }
}

// Total length of an optimal prefix code (Huffman) for symbols with the given occurrence counts: sum_j c_j len_j.
// Built the plain way: repeatedly merge the two lightest subtrees; every merge adds the merged weight to the total.
// A single used symbol still takes one bit per occurrence.
double oracle_huffman_bits(const uint64_t *counts, int32_t n) {
  std::vector<double> w;
  for (int j = 0; j < n; ++j)
    if (counts[j]) w.push_back((double)counts[j]);
  if (w.empty()) return 0.0;
  if (w.size() == 1) return w[0];
  double total = 0.0;
  while (w.size() > 1) {
    std::sort(w.begin(), w.end());
    const double merged = w[0] + w[1];
    total += merged;
    w.erase(w.begin(), w.begin() + 2);
    w.push_back(merged);
  }
  return total;
}

// Bit counts for the coordinates behind `counts` (M types x 256 indices), with `num_norms` 32-bit norms sent:
//   out[0] fixed width, the format of this library: 32 num_norms + sum_m n_m (1 + ceil(log2 S_m));
//   out[1] the expression in the proof of Thm 5.3 with the empirical occurrence probabilities p_j = c_j / n_m:
//          32 num_norms + sum_m [ (n_m - c_0) + n_m (1 - sum_{j=1}^{alpha_m} p_j log2 p_j) ]   (alpha_m = S_m - 2:
//          the sum runs over the interior levels, as printed; one sign bit per non-zero entry);
//   out[2] entropy: 32 num_norms + (non-zeros) + sum_m n_m H_m, H_m = -sum_{j=0}^{S_m-1} p_j log2 p_j;
//   out[3] Huffman: 32 num_norms + (non-zeros) + sum_m (Huffman total of type m);
//   out[4] non-zero entries sum_m (n_m - c_0)  (the lemma on expected non-zeros, App. C.1);  out[5] coordinates.
void oracle_code_length(int32_t M, const int32_t *type_points, const uint64_t *counts, double num_norms, double *out) {
  double fixed = 32.0 * num_norms, paper = fixed, entropy = fixed, huff = fixed, nonzero = 0.0, coords = 0.0;
  for (int m = 0; m < M; ++m) {
    const uint64_t *c = counts + (size_t)m * 256;
    const int Sm = type_points[m];
    double n = 0.0;
    for (int j = 0; j < 256; ++j) n += (double)c[j];
    if (n == 0.0) continue;
    const double nz = n - (double)c[0];
    double h_all = 0.0, h_int = 0.0;
    for (int j = 0; j < 256; ++j) {
      if (!c[j]) continue;
      const double p = (double)c[j] / n;
      const double t = -p * std::log2(p);
      h_all += t;
      if (j >= 1 && j <= Sm - 2) h_int += t;
    }
    fixed += n * (1.0 + (double)index_bits(Sm));
    paper += nz + n * (1.0 + h_int);
    entropy += nz + n * h_all;
    huff += nz + oracle_huffman_bits(c, 256);
    nonzero += nz;
    coords += n;
  }
  out[0] = fixed; out[1] = paper; out[2] = entropy; out[3] = huff; out[4] = nonzero; out[5] = coords;
}

// ---------------------------------------------------------------- one plain step (extra-gradient leg, Sec. 4)
// out = x - gamma * mean.  An extra-gradient method, the two-call scheme the paper compares QODA with, applies it
// twice per round: X_{t+1/2} = X_t - gamma * mean_k Vhat_k(X_t), then X_{t+1} = X_t - gamma * mean_k Vhat_k(X_{t+1/2}).
void oracle_extrapolate(int64_t n, const float *mean, const float *x, float gamma, float *out) {
  for (int64_t e = 0; e < n; ++e) {
    const float gm = gamma * mean[e];
    out[e] = x[e] - gm;
  }
}

// ---------------------------------------------------------------- alternative step sizes: eq. (Alt), Sec. 6
// With lambda = sum_{s<=t-2} sum_k ||Vhat_{k,s+1/2}||^2 / K^2 and mu = sum_{s<=t-2} ||X_s - X_{s+1}||^2:
//   eta_t = (1 + lambda + mu)^(-1/2),  gamma_t = (1 + lambda)^(q - 1/2),  0 < q <= 1/4.
// (The main text and the appendix's choice of rates both sum the K squared norms; the appendix's lemma
// notation squares the norm of the sum instead.  The first form is taken here.)
// eta is taken as in eq. (general_stepsize): rcp_floor(sqrt_floor(.)).  The power with the free exponent q is
// built from correctly rounded operations only, so that it does not depend on a library's pow: q is cut to its
// first 32 binary digits q = sum_j b_j 2^-j, r_j = sqrt(r_{j-1}) with r_0 = 1 + lambda, (1+lambda)^q = product of
// the r_j with b_j = 1 (j increasing, fp64), gamma = fp32((1+lambda)^q / sqrt(1+lambda)).
void oracle_alt_step_size(double lambda, double mu, double q, float *eta_out, float *gamma_out) {
  *eta_out = rcp_floor(sqrt_floor(1.0 + lambda + mu));
  const double base = 1.0 + lambda;
  const uint64_t digits = (uint64_t)std::floor(std::ldexp(q, 32));   // b_1 is the most significant of 32 bits
  double r = base, p = 1.0;
  for (int j = 1; j <= 32; ++j) {
    r = std::sqrt(r);
    if ((digits >> (32 - j)) & 1u) p = p * r;
  }
  *gamma_out = (float)(p / std::sqrt(base));
}

// After round t: lambda <- lambda + (delta_0 + ... + delta_{K-1}) / K^2 with delta_k = ||Vhat_{k,t+1/2}||^2 (the
// quantizer's squared-distance output against an all-zero previous message), mu <- mu + ||X_t - X_{t+1}||^2.
void oracle_alt_advance(int32_t K, const double *delta, double dx2, double *lambda, double *mu) {
  double sum = 0.0;
  for (int k = 0; k < K; ++k) sum = (k == 0) ? delta[k] : sum + delta[k];
  const double invK2 = 1.0 / ((double)K * (double)K);
  *lambda = *lambda + sum * invK2;
  *mu = *mu + dx2;
}

// eq. (ODA) over all layers with the two rates of eq. (Alt), returning ||X_t - X_{t+1}||^2 where
// X_t = X_1 + eta_prev * Y_t is rebuilt from the state (the same two fp32 operations that produced it).
// The squared differences are summed like the step-size term of the main rule: per slot an fp32 fused chain in
// increasing coordinate, slots widened to fp64 and reduced by the tree, chunks numbered through all layers.
double oracle_oda_update_alt(int32_t L, const int64_t *d, const float *const *mean, const float *const *x1,
                             float *const *y, float *const *x_next /* may be NULL */, float *const *x_half,
                             float eta_prev, float eta, float gamma) {
  std::vector<double> chunks;
  for (int l = 0; l < L; ++l) {
    const int64_t nchunks = (d[l] + kChunk - 1) / kChunk;
    for (int64_t c = 0; c < nchunks; ++c) {
      float p32[kSlots];
      for (int j = 0; j < kSlots; ++j) p32[j] = 0.0f;
      const int64_t e1 = std::min(d[l], (c + 1) * kChunk);
      for (int64_t e = c * kChunk; e < e1; ++e) {
        const float ey_old = eta_prev * y[l][e];
        const float xt = x1[l][e] + ey_old;          // X_t
        const float yn = y[l][e] - mean[l][e];       // Y_{t+1}
        const float ey = eta * yn;
        const float xn = x1[l][e] + ey;              // X_{t+1}
        const float gm = gamma * mean[l][e];
        y[l][e] = yn;
        if (x_next) x_next[l][e] = xn;
        x_half[l][e] = xn - gm;                      // X_{t+3/2}
        const float diff = xt - xn;
        p32[slot_of(e)] = std::fmaf(diff, diff, p32[slot_of(e)]);
      }
      double p[kSlots];
      for (int j = 0; j < kSlots; ++j) p[j] = (double)p32[j];
      chunks.push_back(halving_tree(p));
    }
  }
  return combine_chunks(chunks);
}

// ---------------------------------------------------------------- level fit: eq. (Qada2), weights lambda_z
// The K nodes' current vectors are the Z samples.  Every coordinate of (node k, layer l) carries weight
// ||v_{k,l}||^2 (the factor that multiplies its normalised variance in eq. (MQV)/(Qada2)); layers of the
// same type pool.  The distribution is estimated by a histogram:
//   1. bin |v| of every coordinate on its top 11 magnitude bits (8 exponent + 3 mantissa bits): counts[k][l][2048];
//   2. map each bin's midpoint c to u = min(c * inv_norm, 1), re-bin u the same way onto the 257-point
//      grid g_j (g_0 = 2^-32, ..., g_256 = 1), adding weight wfix(k,l) * count, where
//      wfix = floor(sumsq(k,l) * 2^(23 - e)) and e is the binary exponent of the largest sumsq of the type;
//   3. minimise sum_i sum_{bins in [l_i, l_{i+1})} W_j (l_{i+1} - mid_j)(mid_j - l_i) exactly over interior
//      levels restricted to grid points, by dynamic programming (first level 0 and last level 1 are fixed).
// hist_out (optional): K*L*2048 uint32 counts.  pooled_out (optional): M*257 uint64 weights.
// levels_io: M pointers to S_m floats; a type whose vectors are all zero keeps its levels.
void oracle_histogram(const float *v, int64_t d, uint32_t *counts /* 2048, accumulated into */) {
  for (int64_t e = 0; e < d; ++e) counts[(f2u(v[e]) & 0x7FFFFFFFu) >> 20] += 1;
}

// objective of eq. (Qada2) for given levels on pooled grid weights W[257] (used by the fit and by its pins)
double oracle_fit_objective(const uint64_t *W, const float *lev, int32_t S) {
  double total = 0.0;
  for (int j = 0; j < kGridPoints - 1; ++j) {
    if (W[j] == 0) continue;
    const double u = grid_mid(j);
    const int tau = level_index(lev, S, (float)u);
    total += (double)W[j] * ((double)lev[tau + 1] - u) * (u - (double)lev[tau]);
  }
  return total;
}

void oracle_fit_dp(const uint64_t *W, int32_t S, float *lev_out) {
  const int J = kGridPoints;
  std::vector<double> P0(J + 1), P1(J + 1), P2(J + 1);
  P0[0] = P1[0] = P2[0] = 0.0;
  for (int j = 0; j < J; ++j) {
    const double w = (double)W[j];
    const double m = grid_mid(j);
    const double wm = w * m;
    P0[j + 1] = P0[j] + w;
    P1[j + 1] = P1[j] + wm;
    P2[j + 1] = P2[j] + wm * m;
  }
  auto cost0 = [&](int b) { return (double)grid_value(b) * P1[b] - P2[b]; };
  auto cost = [&](int a, int b) {
    const double ga = (double)grid_value(a), gb = (double)grid_value(b);
    return ((ga + gb) * (P1[b] - P1[a]) - (P2[b] - P2[a])) - (ga * gb) * (P0[b] - P0[a]);
  };
  lev_out[0] = 0.0f;
  lev_out[S - 1] = 1.0f;
  if (S == 2) return;
  const int last = J - 1;   // grid index of level S-1
  const double inf = std::numeric_limits<double>::infinity();
  // D[s][b]: best cost of bins below g_b with level s placed at grid index b, s = 1..S-2
  std::vector<std::vector<double>> D(S, std::vector<double>(J, inf));
  std::vector<std::vector<int>> arg(S, std::vector<int>(J, -1));
  for (int b = 1; b <= last - (S - 2); ++b) D[1][b] = cost0(b);
  for (int s = 2; s <= S - 2; ++s)
    for (int b = s; b <= last - (S - 1 - s); ++b) {
      double best = inf; int besta = -1;
      for (int a = s - 1; a <= b - 1; ++a) {
        const double c = D[s - 1][a] + cost(a, b);
        if (c < best) { best = c; besta = a; }
      }
      D[s][b] = best; arg[s][b] = besta;
    }
  double best = inf; int besta = -1;
  for (int a = S - 2; a <= last - 1; ++a) {
    const double c = D[S - 2][a] + cost(a, last);
    if (c < best) { best = c; besta = a; }
  }
  int b = besta;
  for (int s = S - 2; s >= 1; --s) {
    lev_out[s] = grid_value(b);
    b = arg[s][b];
  }
}

namespace {
inline bool any_weight(const std::vector<uint64_t> &W) {
  for (uint64_t w : W)
    if (w) return true;
  return false;
}
}  // namespace

int32_t oracle_fit_levels(int32_t L, const int64_t *d, const int32_t *layer_type, int32_t M, const int32_t *type_points,
                          int32_t K, int32_t scope, const float *const *grads /* K*L, entry k*L+l */,
                          float *const *levels_io, uint32_t *hist_out, uint64_t *pooled_out, int32_t norm_kind) {
  int32_t status = 0;
  if (scope == kScopeBucket) {
    // Every bucket is a vector of its own: weight = its sum of squares, normalisation = its norm.  Every coordinate
    // whose raw magnitude bin is not 0 goes straight onto the normalised grid:
    // W[bin(min(|v| * inv_b, 1))] += floor(sumsq_b * 2^(23 - e)), e = binary exponent of the type's largest bucket
    // sum.  There is no per-layer raw histogram in this scope (hist_out is left untouched).
    for (int m = 0; m < M; ++m) {
      std::vector<uint64_t> W(kGridPoints, 0);
      double smax = 0.0;
      bool finite = true;
      for (int l = 0; l < L; ++l) {
        if (layer_type[l] != m) continue;
        for (int k = 0; k < K; ++k)
          for (int64_t e = 0; e < d[l]; e += kBucket) {
            const double st = bucket_stat(grads[(size_t)k * L + l] + e, std::min<int64_t>(kBucket, d[l] - e), norm_kind);
            const double v = weight_of(st, norm_kind);
            if (!stat_finite(st, norm_kind)) finite = false;
            else if (v > smax) smax = v;
          }
      }
      if (!finite) status = 1;
      if (finite && smax > 0.0) {
        const int ex = std::ilogb(smax);
        for (int l = 0; l < L; ++l) {
          if (layer_type[l] != m) continue;
          for (int k = 0; k < K; ++k) {
            const float *g = grads[(size_t)k * L + l];
            for (int64_t e0 = 0; e0 < d[l]; e0 += kBucket) {
              const int64_t n = std::min<int64_t>(kBucket, d[l] - e0);
              const double sv = bucket_stat(g + e0, n, norm_kind);
              const uint64_t wfix = stat_weight(weight_of(sv, norm_kind), ex);
              const float inv = rcp_floor(norm_of(sv, norm_kind));
              if (wfix == 0 || inv == 0.0f) continue;
              for (int64_t e = e0; e < e0 + n; ++e) {
                if (((f2u(g[e]) & 0x7FFFFFFFu) >> 20) == 0) continue;
                const float uc = std::fmin(std::fabs(g[e]) * inv, 1.0f);
                int j = (int)(f2u(uc) >> 20) - kGridBase;
                if (j < 0) j = 0;
                if (j > kGridPoints - 1) j = kGridPoints - 1;
                W[j] += wfix;
              }
            }
          }
        }
        if (any_weight(W)) oracle_fit_dp(W.data(), type_points[m], levels_io[m]);   // no mass on the grid: keep the levels
      }
      if (pooled_out) std::memcpy(pooled_out + (size_t)m * kGridPoints, W.data(), kGridPoints * sizeof(uint64_t));
    }
    return status;
  }
  std::vector<double> s((size_t)K * L);
  std::vector<uint32_t> hist((size_t)K * L * kHistBins, 0);
  for (int k = 0; k < K; ++k) {
    for (int l = 0; l < L; ++l) {
      s[(size_t)k * L + l] = layer_stat(grads[(size_t)k * L + l], d[l], norm_kind);
      oracle_histogram(grads[(size_t)k * L + l], d[l], &hist[((size_t)k * L + l) * kHistBins]);
    }
    if (scope == kScopeVector) {   // one vector per node: its norm normalises, its squared norm weighs, every layer
      const std::vector<double> sums(s.begin() + (size_t)k * L, s.begin() + (size_t)(k + 1) * L);
      const double total = combine_stats(sums, norm_kind);
      for (int l = 0; l < L; ++l) s[(size_t)k * L + l] = total;
    }
  }
  if (hist_out) std::memcpy(hist_out, hist.data(), hist.size() * sizeof(uint32_t));
  for (int m = 0; m < M; ++m) {
    std::vector<uint64_t> W(kGridPoints, 0);
    double smax = 0.0;
    bool finite = true;
    for (int l = 0; l < L; ++l) {
      if (layer_type[l] != m) continue;
      for (int k = 0; k < K; ++k) {
        const double v = weight_of(s[(size_t)k * L + l], norm_kind);
        if (!stat_finite(s[(size_t)k * L + l], norm_kind)) finite = false;
        else if (v > smax) smax = v;
      }
    }
    if (!finite) status = 1;
    if (finite && smax > 0.0) {
      const int ex = std::ilogb(smax);
      for (int l = 0; l < L; ++l) {
        if (layer_type[l] != m) continue;
        for (int k = 0; k < K; ++k) {
          const double sv = s[(size_t)k * L + l];
          const uint64_t wfix = (uint64_t)std::floor(std::ldexp(weight_of(sv, norm_kind), 23 - ex));
          const float inv = rcp_floor(norm_of(sv, norm_kind));
          if (wfix == 0 || inv == 0.0f) continue;
          const uint32_t *cnt = &hist[((size_t)k * L + l) * kHistBins];
          for (int b = 1; b < kHistBins; ++b) {
            if (cnt[b] == 0) continue;
            const float c = u2f(((uint32_t)b << 20) | (1u << 19));
            const float uc = std::fmin(c * inv, 1.0f);
            int j = (int)(f2u(uc) >> 20) - kGridBase;
            if (j < 0) j = 0;
            if (j > kGridPoints - 1) j = kGridPoints - 1;
            W[j] += wfix * (uint64_t)cnt[b];
          }
        }
      }
      if (any_weight(W)) oracle_fit_dp(W.data(), type_points[m], levels_io[m]);   // no mass on the grid: keep the levels
    }
    if (pooled_out) std::memcpy(pooled_out + (size_t)m * kGridPoints, W.data(), kGridPoints * sizeof(uint64_t));
  }
  return status;
}

// The level fit from statistics gathered by oracle_quantize (bucket scope) over the K nodes of the previous round:
// pool the grid histograms of every type, fit (a type without a scale, or without any mass on the grid, keeps its levels),
// then derive the scale of the next gathering pass from the largest bucket sum of the type.
// hist: K*L*257 (entry (k*L + l)*257 + j), bmax: K*L, exp_io: M (in: the scale the histograms were gathered with).
int32_t oracle_fit_from_stats(int32_t L, const int32_t *layer_type, int32_t M, const int32_t *type_points, int32_t K,
                              const uint64_t *hist, const double *bmax, int32_t *exp_io, float *const *levels_io,
                              uint64_t *pooled_out, int32_t norm_kind) {
  int32_t status = 0;
  for (int m = 0; m < M; ++m) {
    std::vector<uint64_t> W(kGridPoints, 0);
    double smax = 0.0;
    bool finite = true;
    for (int l = 0; l < L; ++l) {
      if (layer_type[l] != m) continue;
      for (int k = 0; k < K; ++k) {
        const size_t idx = (size_t)k * L + l;
        for (int j = 0; j < kGridPoints; ++j) W[j] += hist[idx * kGridPoints + j];
        const double v = weight_of(bmax[idx], norm_kind);   // bmax holds the statistic; the scale is that of the weights
        if (!stat_finite(bmax[idx], norm_kind)) finite = false;
        else if (v > smax) smax = v;
      }
    }
    if (exp_io[m] != kTypeSkip && any_weight(W)) oracle_fit_dp(W.data(), type_points[m], levels_io[m]);
    if (pooled_out) std::memcpy(pooled_out + (size_t)m * kGridPoints, W.data(), kGridPoints * sizeof(uint64_t));
    if (!finite) status = 1;
    exp_io[m] = (finite && smax > 0.0) ? std::ilogb(smax) : kTypeSkip;
  }
  return status;
}

// ================================================================ plain definitions (references, no contract)
// The routines above fix precision and order of every operation so that two implementations can agree to the bit.
// Two of their quantities are narrower than the textbook definition, for the sake of a cheap GPU pass: the step-size
// term (single-precision chains inside a reduction slot) and the bucket sum of squares (single-precision chains inside
// a lane, where the result is in a safe range); the level fit works on a histogram instead of the samples themselves.
// What follows are the definitions themselves -- fp64 arithmetic, long double accumulators, plain coordinate order --
// for the tests that bound the contract's values against them.  Nothing here is called by the routines above.

// eq. (general_stepsize), one node's term: sum_i (Vhat_i - Vhat_prev_i)^2 over the decoded messages (prev NULL: 0).
double oracle_delta_plain(int32_t L, const int64_t *d, const int32_t *S, int32_t scope, const uint8_t *msg,
                          const uint8_t *msg_prev) {
  const Layout lay = make_layout(L, d, S, scope);
  long double total = 0.0L;
  for (int l = 0; l < L; ++l)
    for (int64_t e = 0; e < d[l]; ++e) {
      const double cur = (double)decoded_value(msg, lay, l, e);
      const double prev = msg_prev ? (double)decoded_value(msg_prev, lay, l, e) : 0.0;
      total += (long double)((cur - prev) * (cur - prev));
    }
  return (double)total;
}

// sum of squares of n coordinates (Sec. 2.2: the square of the L2 norm)
double oracle_sumsq_plain(const float *v, int64_t n) {
  long double total = 0.0L;
  for (int64_t e = 0; e < n; ++e) total += (long double)((double)v[e] * (double)v[e]);
  return (double)total;
}

namespace {
// ||v||_q for q = 2, 1, infinity, straight from the definition
double norm_plain(const float *v, int64_t n, int kind) {
  if (kind == kNormL2) return std::sqrt(oracle_sumsq_plain(v, n));
  long double total = 0.0L;
  double mx = 0.0;
  for (int64_t e = 0; e < n; ++e) {
    total += (long double)std::fabs((double)v[e]);
    mx = std::fmax(mx, std::fabs((double)v[e]));
  }
  return kind == kNormL1 ? (double)total : mx;
}

// sum_i (l_{tau+1} - u_i)(u_i - l_tau) with u_i = |v_i| / norm  (the normalised variance of eq. (Var))
long double normalised_variance(const float *v, int64_t n, double norm, const float *lev, int S) {
  long double total = 0.0L;
  if (!(norm > 0.0)) return total;
  for (int64_t e = 0; e < n; ++e) {
    const double u = std::fmin(std::fabs((double)v[e]) / norm, 1.0);
    int tau = 0;
    for (int j = 1; j <= S - 2; ++j)
      if ((double)lev[j] <= u) tau = j;
    total += (long double)(((double)lev[tau + 1] - u) * (u - (double)lev[tau]));
  }
  return total;
}
}  // namespace

// eq. (Var) for one vector with one level sequence: ||v||_q^2 * sum_i (l_{tau+1} - u_i)(u_i - l_tau).
double oracle_variance_plain(const float *v, int64_t n, const float *lev, int32_t S, int32_t norm_kind) {
  const double norm = norm_plain(v, n, norm_kind);
  return (double)((long double)(norm * norm) * normalised_variance(v, n, norm, lev, S));
}

// eq. (MQV): the total quantization variance of the K nodes' vectors under the given per-type levels -- what the level
// fit is meant to minimise.  A "vector" is what one norm covers: a layer, the node's whole dual vector, or a bucket.
double oracle_mqv_objective_plain(int32_t L, const int64_t *d, const int32_t *layer_type, const int32_t *type_points,
                                  int32_t K, int32_t scope, const float *const *grads /* K*L */,
                                  const float *const *levels /* M */, int32_t norm_kind) {
  long double total = 0.0L;
  for (int k = 0; k < K; ++k) {
    double vnorm = 0.0;
    if (scope == kScopeVector) {   // the norm of the concatenation of the node's layers
      long double acc = 0.0L;
      double mx = 0.0;
      for (int l = 0; l < L; ++l) {
        const double nl = norm_plain(grads[(size_t)k * L + l], d[l], norm_kind);
        if (norm_kind == kNormL2) acc += (long double)(nl * nl);
        else if (norm_kind == kNormL1) acc += (long double)nl;
        else mx = std::fmax(mx, nl);
      }
      vnorm = norm_kind == kNormL2 ? std::sqrt((double)acc) : (norm_kind == kNormL1 ? (double)acc : mx);
    }
    for (int l = 0; l < L; ++l) {
      const float *g = grads[(size_t)k * L + l];
      const float *lev = levels[layer_type[l]];
      const int S = type_points[layer_type[l]];
      if (scope == kScopeBucket) {
        for (int64_t e0 = 0; e0 < d[l]; e0 += kBucket) {
          const int64_t n = std::min<int64_t>(kBucket, d[l] - e0);
          const double nb = norm_plain(g + e0, n, norm_kind);
          total += (long double)(nb * nb) * normalised_variance(g + e0, n, nb, lev, S);
        }
      } else {
        const double nl = scope == kScopeVector ? vnorm : norm_plain(g, d[l], norm_kind);
        total += (long double)(nl * nl) * normalised_variance(g, d[l], nl, lev, S);
      }
    }
  }
  return (double)total;
}

}  // extern "C"
