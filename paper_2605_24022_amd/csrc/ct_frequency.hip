// Offline frequency-guided choice of the tokens to recompute (Sec. 4.1, Eq. 2-7).
//
// Scores.  The low-pass reconstruction of Eq. 2-4 is a forward FFT along the sequence, a mask
// and an inverse FFT, for every (head, dim) column of K and of V.  One workgroup takes a strip
// of 2*CP adjacent columns and all N tokens: two real columns ride as the real and imaginary
// part of one complex sequence (the mask is symmetric in +-frequency, so it commutes with that
// packing), which leaves CP complex sequences of length N.  They live in LDS for the whole
// transform; every pass is a Stockham (auto-sorting) radix-R step with R in {16, 8, 5, 4, 3, 2}:
// each thread pulls the R inputs of its butterflies into registers, the workgroup meets at a
// barrier, and the thread writes its R outputs to their natural-order places, so one LDS array
// serves as source and destination.  After the inverse passes the squared magnitudes of a
// token's row are summed over the strip (Eq. 5 needs the norm over all heads and dims) and
// accumulated over the strips a workgroup owns; a second small kernel adds the workgroups'
// partial sums in a fixed order, so the scores are reproducible bit for bit.
//
// Sequences longer than kFreqMaxTokens do not fit one workgroup's LDS: their transform is split as
// N = N1 N2 (token n = n1 N2 + n2, bin k = k1 + N1 k2) into length-N1 transforms over n1, a twiddle
// exp(-+2 pi i n2 k1 / N), and length-N2 transforms over n2, each done in LDS by the same passes,
// with one complex fp32 array of N x (row_elems / 2) per tensor in HBM between them:
//   A  (n2, strip):  x[n1 N2 + n2] -> FFT over n1 -> * twiddle -> Y[k1 N2 + n2]
//   B  (k1, strip):  Y[k1 N2 + .]  -> FFT over n2 -> mask bins k1 + N1 k2 -> inverse FFT over k2
//                    -> * conj twiddle -> Z[k1 N2 + n2]        (in place, contiguous rows)
//   C  (n2, strip):  Z[. N2 + n2]  -> inverse FFT over k1 -> squares summed per token.
//
// TopK (Eq. 7).  One workgroup per sequence: a 4 x 8-bit radix select over the order-preserving
// integer image of the scores finds the threshold value and how many of the tokens that tie with
// it still fit (lower index first); an ordered sweep then writes the chosen indices ascending.
#include "ct_internal.h"

namespace ct {

// One workgroup of 1024 threads per compute unit.  (Two of 512 threads with half the strip each
// were measured: no faster, the kernel is bound by vector instructions, not by waiting.)
constexpr int kFreqThreads = 1024;
constexpr int kFreqMaxElems = 16384;   // complex values of a strip held in LDS (16 per thread)
constexpr int kFreqMaxTokens = 4096;

struct FftPlan {
  int32_t n;          // tokens
  int32_t lg_cp;      // log2 of the complex sequences per strip
  int32_t n_pass;
  int32_t radix[12];
  int32_t cutoff;     // bins k with min(k, n - k) >= cutoff are zeroed
  int32_t strips;     // strips per tensor = row_elems / (2 CP)
  int32_t groups;     // workgroups per tensor; workgroup g owns strips g * (strips / groups) ... in order
};

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
// a * (sgn * i)
__device__ __forceinline__ float2 mul_si(float2 a, float sgn) { return make_float2(-sgn * a.y, sgn * a.x); }

// exp(sgn * 2 pi i m / 16), m constant after unrolling
__device__ __forceinline__ float2 w16(int m, float sgn) {
  constexpr float c[16] = {1.f, 0.9238795325112867f, 0.7071067811865476f, 0.3826834323650898f, 0.f,
                           -0.3826834323650898f, -0.7071067811865476f, -0.9238795325112867f, -1.f,
                           -0.9238795325112867f, -0.7071067811865476f, -0.3826834323650898f, 0.f,
                           0.3826834323650898f, 0.7071067811865476f, 0.9238795325112867f};
  return make_float2(c[m & 15], sgn * c[(m + 12) & 15]);   // sin(x) = cos(x - pi/2)
}

// In-register DFTs of length R: v[k] <- sum_n v[n] exp(sgn 2 pi i n k / R).
template <int R>
__device__ __forceinline__ void dft(float2 (&v)[R], float sgn);

template <>
__device__ __forceinline__ void dft<2>(float2 (&v)[2], float) {
  const float2 a = v[0], b = v[1];
  v[0] = cadd(a, b);
  v[1] = csub(a, b);
}
template <>
__device__ __forceinline__ void dft<4>(float2 (&v)[4], float sgn) {
  const float2 t0 = cadd(v[0], v[2]), t1 = csub(v[0], v[2]);
  const float2 t2 = cadd(v[1], v[3]), t3 = mul_si(csub(v[1], v[3]), sgn);
  v[0] = cadd(t0, t2);
  v[2] = csub(t0, t2);
  v[1] = cadd(t1, t3);
  v[3] = csub(t1, t3);
}
template <>
__device__ __forceinline__ void dft<3>(float2 (&v)[3], float sgn) {
  const float2 s = cadd(v[1], v[2]), d = csub(v[1], v[2]);
  const float2 m = make_float2(v[0].x - 0.5f * s.x, v[0].y - 0.5f * s.y);
  const float2 q = mul_si(make_float2(0.8660254037844386f * d.x, 0.8660254037844386f * d.y), sgn);
  v[0] = cadd(v[0], s);
  v[1] = cadd(m, q);
  v[2] = csub(m, q);
}
template <>
__device__ __forceinline__ void dft<5>(float2 (&v)[5], float sgn) {
  // pairs (1,4) and (2,3): sums feed the cosines, differences the sines
  const float c1 = 0.30901699437494745f, c2 = -0.8090169943749473f;
  const float s1 = 0.9510565162951535f, s2 = 0.5877852522924731f;
  const float2 a1 = cadd(v[1], v[4]), b1 = csub(v[1], v[4]);
  const float2 a2 = cadd(v[2], v[3]), b2 = csub(v[2], v[3]);
  const float2 x0 = v[0];
  const float2 p1 = make_float2(x0.x + c1 * a1.x + c2 * a2.x, x0.y + c1 * a1.y + c2 * a2.y);
  const float2 p2 = make_float2(x0.x + c2 * a1.x + c1 * a2.x, x0.y + c2 * a1.y + c1 * a2.y);
  const float2 q1 = mul_si(make_float2(s1 * b1.x + s2 * b2.x, s1 * b1.y + s2 * b2.y), sgn);
  const float2 q2 = mul_si(make_float2(s2 * b1.x - s1 * b2.x, s2 * b1.y - s1 * b2.y), sgn);
  v[0] = cadd(x0, cadd(a1, a2));
  v[1] = cadd(p1, q1);
  v[4] = csub(p1, q1);
  v[2] = cadd(p2, q2);
  v[3] = csub(p2, q2);
}
// R = R1 * 4 by one Cooley-Tukey split: input n = 4 n1 + n2, output k = k1 + R1 k2.
template <int R1>
__device__ __forceinline__ void dft_by4(float2 (&v)[R1 * 4], float sgn) {
  constexpr int R = R1 * 4;
  float2 y[R1][4];
#pragma unroll
  for (int n2 = 0; n2 < 4; ++n2) {
    float2 col[R1];
#pragma unroll
    for (int n1 = 0; n1 < R1; ++n1) col[n1] = v[4 * n1 + n2];
    dft<R1>(col, sgn);
#pragma unroll
    for (int k1 = 0; k1 < R1; ++k1) y[k1][n2] = (n2 * k1 == 0) ? col[k1] : cmul(col[k1], w16(n2 * k1 * (16 / R), sgn));
  }
#pragma unroll
  for (int k1 = 0; k1 < R1; ++k1) {
    dft<4>(y[k1], sgn);
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) v[k1 + R1 * k2] = y[k1][k2];
  }
}
template <>
__device__ __forceinline__ void dft<8>(float2 (&v)[8], float sgn) { dft_by4<2>(v, sgn); }
template <>
__device__ __forceinline__ void dft<16>(float2 (&v)[16], float sgn) { dft_by4<4>(v, sgn); }

// Place of element (token or bin n, sequence c) in LDS: one spare row per 16 rows keeps the
// first pass's strided writes off a common bank.
__device__ __forceinline__ int phys(int n, int c, int lg_cp) { return ((n + (n >> 4)) << lg_cp) + c; }

// One Stockham pass of radix R over all CP sequences.  ns = product of the radices of the
// passes before this one.  tw[t] = exp(-2 pi i t / n) for t < n / 2.
// N_CT > 0: the length (a power of two, with CP = kFreqMaxElems / N sequences per strip) and ns are known
// at compile time, which turns the index arithmetic into shifts and immediate offsets; N_CT = 0
// takes them at run time.
template <int R, int N_CT, int NS_CT>
__device__ __forceinline__ void stockham_pass(float2* data, const float2* tw, int n_rt, int lg_cp_rt, int ns_rt,
                                              float sgn) {
  constexpr bool FIXED = N_CT > 0;
  constexpr int ITER = (kFreqMaxElems / kFreqThreads + R - 1) / R;
  const int n = FIXED ? N_CT : n_rt;
  const int lg_cp = FIXED ? __builtin_ctz(kFreqMaxElems / (FIXED ? N_CT : 1)) : lg_cp_rt;
  const int ns = FIXED ? NS_CT : ns_rt;
  const int m = n / R;                 // butterflies per sequence
  const int nb = m << lg_cp;
  const int cmask = (1 << lg_cp) - 1;
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));        // addresses are computed here, not hoisted out of the strip loop
  float2 v[ITER][R];
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int b = tid + i * kFreqThreads;
    if (FIXED || b < nb) {
      const int j = b >> lg_cp, c = b & cmask;
      if (FIXED && (N_CT / R) % 16 == 0) {      // the stride is whole groups of 16 rows: constant offsets
        const float2* src = data + phys(j, c, lg_cp);
#pragma unroll
        for (int r = 0; r < R; ++r) v[i][r] = src[(r * (m + m / 16)) << lg_cp];
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) v[i][r] = data[phys(j + r * m, c, lg_cp)];
      }
    }
  }
  __syncthreads();
  const int tstep = n / (ns * R);
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int b = tid + i * kFreqThreads;
    if (FIXED || b < nb) {
      const int j = b >> lg_cp, c = b & cmask;
      const int hi = j / ns, k = j - hi * ns;
      if (ns > 1) {
        float2 w1 = tw[k * tstep];
        w1.y *= -sgn;                 // the table holds the forward (sgn = -1) twiddles
        float2 cur = w1, pw = w1;     // cur = w1^r; restarted from a repeated square at every power of two
#pragma unroll
        for (int r = 1; r < R; ++r) {
          if (r > 1) {
            if ((r & (r - 1)) == 0) {
              pw = cmul(pw, pw);
              cur = pw;
            } else {
              cur = cmul(cur, w1);
            }
          }
          v[i][r] = cmul(v[i][r], cur);
        }
      }
      dft<R>(v[i], sgn);
      const int j0 = hi * ns * R + k;
      if (FIXED && (NS_CT % 16 == 0 || (NS_CT == 1 && 16 % R == 0))) {
        // rows j0 + r ns: whole groups of 16 rows apart, or (ns = 1) inside one group
        float2* dst = data + phys(j0, c, lg_cp);
        const int stride = NS_CT == 1 ? 1 : ns + ns / 16;
#pragma unroll
        for (int r = 0; r < R; ++r) dst[(r * stride) << lg_cp] = v[i][r];
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) data[phys(j0 + r * ns, c, lg_cp)] = v[i][r];
      }
    }
  }
  __syncthreads();
}

// Run-time plan: any length of the form 2^a 3^b 5^c.
__device__ __forceinline__ void transform(float2* data, const float2* tw, const FftPlan& p, int n, int lg_cp,
                                          float sgn) {
  int ns = 1;
  for (int s = 0; s < p.n_pass; ++s) {
    const int r = p.radix[s];
    asm volatile("" : "+s"(n), "+s"(lg_cp));
    switch (r) {
      case 16: stockham_pass<16, 0, 0>(data, tw, n, lg_cp, ns, sgn); break;
      case 8: stockham_pass<8, 0, 0>(data, tw, n, lg_cp, ns, sgn); break;
      case 5: stockham_pass<5, 0, 0>(data, tw, n, lg_cp, ns, sgn); break;
      case 4: stockham_pass<4, 0, 0>(data, tw, n, lg_cp, ns, sgn); break;
      case 3: stockham_pass<3, 0, 0>(data, tw, n, lg_cp, ns, sgn); break;
      default: stockham_pass<2, 0, 0>(data, tw, n, lg_cp, ns, sgn); break;
    }
    ns *= r;
  }
}

// Compile-time plans for the power-of-two lengths 256 ... 4096 (three passes at most).
template <int N>
__device__ __forceinline__ void transform_fixed(float2* data, const float2* tw, float sgn) {
  constexpr int R0 = N == 512 ? 8 : 16;
  constexpr int R1 = (N == 512 || N == 1024) ? 8 : 16;
  constexpr int R2 = N / (R0 * R1);     // 1 (N = 256), 8 or 16
  stockham_pass<R0, N, 1>(data, tw, 0, 0, 0, sgn);
  stockham_pass<R1, N, R0>(data, tw, 0, 0, 0, sgn);
  if constexpr (R2 > 1) stockham_pass<R2, N, R0 * R1>(data, tw, 0, 0, 0, sgn);
}

// partial[((b * 2 + kv) * groups + g) * n + token] = sum over the workgroup's strips of
// |N x~|^2 (the 1/N of the inverse transform is applied by the finishing kernel).
template <int N_CT>
__global__ __launch_bounds__(kFreqThreads) void freq_energy_kernel(const uint16_t* __restrict__ k,
                                                                   const uint16_t* __restrict__ v,
                                                                   int64_t batch_stride, int32_t row_elems, int32_t n_work,
                                                                   FftPlan p, float* __restrict__ partial) {
  extern __shared__ float2 lds[];
  int n = N_CT > 0 ? N_CT : p.n, lg_cp = N_CT > 0 ? __builtin_ctz(kFreqMaxElems / (N_CT > 0 ? N_CT : 1)) : p.lg_cp;
  const int cp = 1 << lg_cp;
  float2* data = lds;
  float2* tw = lds + ((n + (n >> 4) + 1) << lg_cp);
  // workgroups that share 128-byte lines of the rows (adjacent strips) are given ids that differ
  // by 8, which puts them on the same XCD (and its L2) in the same wave of launches
  int w = blockIdx.x;
  const int own = p.strips / p.groups;                       // strips per workgroup
  const int per_line = cp * own >= 32 ? 1 : 32 / (cp * own);
  if (n_work % (8 * per_line) == 0 && p.groups % per_line == 0) {
    const int xcd = w & 7, slot = w >> 3;
    w = (slot / per_line) * (8 * per_line) + xcd * per_line + slot % per_line;
  }
  const int tensor = w / p.groups, g = w - tensor * p.groups;   // tensor = batch * 2 + kv
  const uint16_t* src = ((tensor & 1) ? v : k) + (int64_t)(tensor >> 1) * batch_stride;

  // only radices 8 and 16 occur in the compiled-in plans, so their first-power twiddles stop at n / 8
  const int tw_len = N_CT > 0 ? N_CT / 8 : (n + 1) / 2;
  for (int t = threadIdx.x; t < tw_len; t += kFreqThreads) {
    float s, c;
    const float turns = (float)t / (float)n;           // in [0, 1/2)
    sincospif(-2.f * turns, &s, &c);
    tw[t] = make_float2(c, s);
  }
  const int elems = n << lg_cp;
  constexpr int PER = kFreqMaxElems / kFreqThreads;
  // energy of the rows this thread owns (rows tid, tid + kFreqThreads, ...), summed over the strips
  constexpr int ROWS = kFreqMaxTokens / kFreqThreads;
  float acc[ROWS];
#pragma unroll
  for (int i = 0; i < ROWS; ++i) acc[i] = 0.f;

  for (int strip = g * own; strip < (g + 1) * own; ++strip) {
    // the sizes are made opaque once per strip, and once more before each stage, so that the
    // addresses of every stage are computed where they are used instead of being hoisted out of
    // the loop together (which overflows the 128 registers a 1024-thread workgroup leaves a lane)
    if (N_CT == 0) asm volatile("" : "+s"(n), "+s"(lg_cp));
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const uint32_t* base = reinterpret_cast<const uint32_t*>(src) + (int64_t)strip * cp;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = tid + i * kFreqThreads;
      if (e < elems) {
        const int row = e >> lg_cp, c = e & (cp - 1);
        const uint32_t pair = __builtin_nontemporal_load(base + (int64_t)row * (row_elems / 2) + c);
        data[phys(row, c, lg_cp)] = make_float2(bf16_lo(pair), bf16_hi(pair));
      }
    }
    __syncthreads();
    if constexpr (N_CT > 0) {
      transform_fixed<N_CT>(data, tw, -1.f);
    } else {
      asm volatile("" : "+s"(n), "+s"(lg_cp));
      transform(data, tw, p, n, lg_cp, -1.f);
      asm volatile("" : "+s"(n), "+s"(lg_cp));
    }
    // Eq. 3: bins from the cutoff on (and their mirror images) are zeroed
    {
      const int first = p.cutoff, last = p.cutoff == 0 ? n - 1 : n - p.cutoff;   // bins first..last go
      const int gone = last >= first ? last - first + 1 : 0;
      for (int e = threadIdx.x; e < (gone << lg_cp); e += kFreqThreads) {
        const int bin = first + (e >> lg_cp), c = e & (cp - 1);
        data[phys(bin, c, lg_cp)] = make_float2(0.f, 0.f);
      }
    }
    __syncthreads();
    if constexpr (N_CT > 0) {
      transform_fixed<N_CT>(data, tw, 1.f);
    } else {
      asm volatile("" : "+s"(n), "+s"(lg_cp));
      transform(data, tw, p, n, lg_cp, 1.f);
      asm volatile("" : "+s"(n), "+s"(lg_cp));
    }
    asm volatile("" : "+v"(tid));
    // Eq. 5: each thread adds up the squares of whole rows (all CP sequences of a token), the
    // sequences visited in an order rotated by the lane so that neighbours start on other banks
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
      const int row = tid + i * kFreqThreads;
      if (row < n) {
        const float2* line = data + phys(row, 0, lg_cp);
        float sq = 0.f;
        for (int q = 0; q < cp; ++q) {
          const float2 x = line[(q + tid) & (cp - 1)];
          sq = fmaf(x.x, x.x, fmaf(x.y, x.y, sq));
        }
        acc[i] += sq;
      }
    }
    __syncthreads();
  }
  float* out = partial + ((int64_t)tensor * p.groups + g) * n;
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    const int row = threadIdx.x + i * kFreqThreads;
    if (row < n) out[row] = acc[i];
  }
}

// ---- sequences beyond kFreqMaxTokens: N = N1 N2 through HBM -----------------------------------
constexpr int kFreqLongElems = 8192;   // complex values per workgroup in the long path (8 per thread)

__device__ __forceinline__ void build_twiddles(float2* tw, int n) {
  for (int t = threadIdx.x; t < (n + 1) / 2; t += kFreqThreads) {
    float s, c;
    sincospif(-2.f * ((float)t / (float)n), &s, &c);
    tw[t] = make_float2(c, s);
  }
}
// exp(sgn 2 pi i a b / n) for a b < 2^48, n < 2^24: the product is reduced exactly before it is rounded
__device__ __forceinline__ float2 long_twiddle(int a, int b, int n, float sgn) {
  const int t = (int)(((int64_t)a * b) % n);
  float s, c;
  sincospif(2.f * ((float)t / (float)n), &s, &c);
  return make_float2(c, sgn * s);
}

// A: one workgroup = one n2 and one strip of 2^lg complex columns (pairs of real columns).
__global__ __launch_bounds__(kFreqThreads) void freq_long_a_kernel(const uint16_t* __restrict__ src, int32_t width,
                                                                   FftPlan p1, int32_t n, int32_t n2_len,
                                                                   float2* __restrict__ scratch) {
  extern __shared__ float2 lds[];
  int n1 = p1.n, lg = p1.lg_cp;
  const int cp = 1 << lg;
  float2* data = lds;
  float2* tw = lds + ((n1 + (n1 >> 4) + 1) << lg);
  const int strips = width >> lg;
  const int strip = blockIdx.x % strips, n2 = blockIdx.x / strips;
  build_twiddles(tw, n1);
  const uint32_t* base = reinterpret_cast<const uint32_t*>(src) + (int64_t)strip * cp;
  for (int e = threadIdx.x; e < (n1 << lg); e += kFreqThreads) {
    const int row = e >> lg, c = e & (cp - 1);
    const uint32_t pair = __builtin_nontemporal_load(base + ((int64_t)row * n2_len + n2) * width + c);
    data[phys(row, c, lg)] = make_float2(bf16_lo(pair), bf16_hi(pair));
  }
  __syncthreads();
  transform(data, tw, p1, n1, lg, -1.f);
  float2* out = scratch + (int64_t)strip * cp;
  for (int e = threadIdx.x; e < (n1 << lg); e += kFreqThreads) {
    const int k1 = e >> lg, c = e & (cp - 1);
    out[((int64_t)k1 * n2_len + n2) * width + c] = cmul(data[phys(k1, c, lg)], long_twiddle(n2, k1, n, -1.f));
  }
}

// B: one workgroup = one k1 and one strip; rows k1 N2 ... k1 N2 + N2 - 1 of the scratch array, in place.
__global__ __launch_bounds__(kFreqThreads) void freq_long_b_kernel(float2* __restrict__ scratch, int32_t width, FftPlan p2,
                                                                   int32_t n, int32_t n1_len, int32_t cutoff) {
  extern __shared__ float2 lds[];
  int n2 = p2.n, lg = p2.lg_cp;
  const int cp = 1 << lg;
  float2* data = lds;
  float2* tw = lds + ((n2 + (n2 >> 4) + 1) << lg);
  const int strips = width >> lg;
  const int strip = blockIdx.x % strips, k1 = blockIdx.x / strips;
  build_twiddles(tw, n2);
  float2* rows = scratch + (int64_t)k1 * n2 * width + (int64_t)strip * cp;
  for (int e = threadIdx.x; e < (n2 << lg); e += kFreqThreads) {
    const int row = e >> lg, c = e & (cp - 1);
    data[phys(row, c, lg)] = rows[(int64_t)row * width + c];
  }
  __syncthreads();
  transform(data, tw, p2, n2, lg, -1.f);
  // Eq. 3: bin k = k1 + N1 k2 goes when cutoff <= k <= N - cutoff
  for (int e = threadIdx.x; e < (n2 << lg); e += kFreqThreads) {
    const int k2 = e >> lg, c = e & (cp - 1);
    const int k = k1 + n1_len * k2;
    if (k >= cutoff && k <= n - cutoff) data[phys(k2, c, lg)] = make_float2(0.f, 0.f);
  }
  __syncthreads();
  transform(data, tw, p2, n2, lg, 1.f);
  for (int e = threadIdx.x; e < (n2 << lg); e += kFreqThreads) {
    const int j = e >> lg, c = e & (cp - 1);
    rows[(int64_t)j * width + c] = cmul(data[phys(j, c, lg)], long_twiddle(j, k1, n, 1.f));
  }
}

// C: one workgroup = one n2 and one strip; partial[strip * n + token] = sum over the strip of |N x~|^2.
__global__ __launch_bounds__(kFreqThreads) void freq_long_c_kernel(const float2* __restrict__ scratch, int32_t width,
                                                                   FftPlan p1, int32_t n, int32_t n2_len,
                                                                   float* __restrict__ partial) {
  extern __shared__ float2 lds[];
  int n1 = p1.n, lg = p1.lg_cp;
  const int cp = 1 << lg;
  float2* data = lds;
  float2* tw = lds + ((n1 + (n1 >> 4) + 1) << lg);
  const int strips = width >> lg;
  const int strip = blockIdx.x % strips, n2 = blockIdx.x / strips;
  build_twiddles(tw, n1);
  const float2* in = scratch + (int64_t)strip * cp;
  for (int e = threadIdx.x; e < (n1 << lg); e += kFreqThreads) {
    const int k1 = e >> lg, c = e & (cp - 1);
    data[phys(k1, c, lg)] = in[((int64_t)k1 * n2_len + n2) * width + c];
  }
  __syncthreads();
  transform(data, tw, p1, n1, lg, 1.f);
  // Eq. 5: a token's squares over the strip, summed by one thread in a fixed order
  for (int row = threadIdx.x; row < n1; row += kFreqThreads) {
    const float2* line = data + phys(row, 0, lg);
    float sq = 0.f;
    for (int q = 0; q < cp; ++q) {
      const float2 x = line[(q + row) & (cp - 1)];
      sq = fmaf(x.x, x.x, fmaf(x.y, x.y, sq));
    }
    partial[(int64_t)strip * n + (int64_t)row * n2_len + n2] = sq;
  }
}

// Eq. 5-6: s_i = (||K~_i|| + ||V~_i||) / 2
__global__ __launch_bounds__(256) void freq_finish_kernel(const float* __restrict__ partial, int32_t n, int32_t groups,
                                                          int32_t n_batch, float* __restrict__ scores) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)n_batch * n) return;
  const int b = (int)(i / n), t = (int)(i - (int64_t)b * n);
  float sk = 0.f, sv = 0.f;
  for (int g = 0; g < groups; ++g) {
    sk += partial[((int64_t)(b * 2 + 0) * groups + g) * n + t];
    sv += partial[((int64_t)(b * 2 + 1) * groups + g) * n + t];
  }
  scores[i] = 0.5f * (sqrtf(sk) + sqrtf(sv)) / (float)n;
}

// ---- TopK ---------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t b = __float_as_uint(s);
  if (b == 0x80000000u) b = 0;                                   // -0 ties with +0
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);             // larger score <=> larger key
}

__global__ __launch_bounds__(1024) void topk_kernel(const float* __restrict__ scores, int32_t n, int32_t k,
                                                    int32_t* __restrict__ idx_out) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_need;
  __shared__ uint32_t wave_sum[2][16];
  __shared__ uint32_t carry[2];
  const float* s = scores + (int64_t)blockIdx.x * n;
  int32_t* out = idx_out + (int64_t)blockIdx.x * k;
  const int tid = threadIdx.x;
  if (k <= 0) return;
  // radix select, most significant byte first: after the loop `prefix` is the key of the k-th
  // largest score and `need` the number of tokens with exactly that key that are still taken
  uint32_t prefix = 0, need = (uint32_t)k;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t himask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
    for (int i = tid; i < n; i += 1024) {
      const uint32_t key = score_key(s[i]);
      if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {
      // the first wave walks the histogram from the top: lane l owns bins 4l .. 4l+3; a suffix
      // scan over the lanes gives the count above each lane's bins, and the one lane whose bins
      // take the running count to `need` publishes the bin and what is left to take inside it
      const uint32_t h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
      const uint32_t tot = h0 + h1 + h2 + h3;
      uint32_t incl = tot;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t y = __shfl_down(incl, off, 64);
        if (tid + off < 64) incl += y;
      }
      uint32_t above = incl - tot;
      if (above < need && need <= above + tot) {
        int bin = 4 * tid + 3;
        uint32_t left = need - above;
        if (h3 < left) { left -= h3; bin = 4 * tid + 2;
          if (h2 < left) { left -= h2; bin = 4 * tid + 1;
            if (h1 < left) { left -= h1; bin = 4 * tid; } } }
        sh_prefix = prefix | ((uint32_t)bin << shift);
        sh_need = left;
      }
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
    __syncthreads();
  }
  // ordered sweep: tokens above the threshold, and the first `need` tokens on it
  if (tid < 2) carry[tid] = 0;
  __syncthreads();
  const int lane = tid & 63, wv = tid >> 6;
  for (int i0 = 0; i0 < n; i0 += 1024) {
    const int i = i0 + tid;
    const uint32_t key = i < n ? score_key(s[i]) : 0u;
    const bool above = i < n && key > prefix;
    const bool tie = i < n && key == prefix;
    const uint64_t tie_ballot = __ballot(tie);
    const uint32_t tie_before = __popcll(tie_ballot & ((1ull << lane) - 1ull));
    if (lane == 0) wave_sum[0][wv] = __popcll(tie_ballot);
    __syncthreads();
    uint32_t tie_off = carry[0];
    for (int q = 0; q < wv; ++q) tie_off += wave_sum[0][q];
    const bool take = above || (tie && tie_off + tie_before < need);
    const uint64_t take_ballot = __ballot(take);
    const uint32_t take_before = __popcll(take_ballot & ((1ull << lane) - 1ull));
    if (lane == 0) wave_sum[1][wv] = __popcll(take_ballot);
    __syncthreads();
    uint32_t take_off = carry[1];
    for (int q = 0; q < wv; ++q) take_off += wave_sum[1][q];
    if (take) out[take_off + take_before] = i;
    __syncthreads();
    if (tid == 0) {
      uint32_t a = 0, b = 0;
      for (int q = 0; q < 16; ++q) {
        a += wave_sum[0][q];
        b += wave_sum[1][q];
      }
      carry[0] += a;
      carry[1] += b;
    }
    __syncthreads();
  }
}

// ---- host side ------------------------------------------------------------------------------
static bool factor_radices(int32_t n, FftPlan* p) {
  p->n = n;
  p->n_pass = 0;
  int rest = n;
  const int radices[6] = {16, 8, 4, 2, 3, 5};
  // powers of two first, largest radix first; a lone factor 2 after 16s is folded as 8 or 4
  for (int r : radices) {
    while (rest % r == 0 && rest > 1) {
      if (p->n_pass == 12) return false;
      p->radix[p->n_pass++] = r;
      rest /= r;
    }
  }
  return rest == 1;
}

static int32_t cutoff_bins(int32_t n, double alpha) {
  const int bins = n / 2 + 1;
  int c = (int)floor(alpha * bins + 1e-9);
  if (c < 0) c = 0;
  if (c > bins) c = bins;
  return c;
}

// Long sequences: N = N1 N2 with N1 <= N2 <= kFreqMaxTokens, N1 the largest such divisor.
struct LongPlan {
  FftPlan p1, p2;
  int32_t width;        // complex columns per row = row_elems / 2
  int32_t cutoff;
  size_t partial_bytes, scratch_bytes;
};
static bool make_long_plan(int32_t n, int32_t row_elems, double alpha, LongPlan* lp) {
  if (row_elems % 2 != 0 || n >= (1 << 24)) return false;
  int n1 = 0;
  for (int d = (int)floor(sqrt((double)n)); d >= 2; --d)
    if (n % d == 0) {
      if (n / d <= kFreqMaxTokens) n1 = d;
      break;                       // the largest divisor below the root; smaller ones have larger cofactors
    }
  if (n1 == 0) return false;
  *lp = LongPlan{};
  if (!factor_radices(n1, &lp->p1) || !factor_radices(n / n1, &lp->p2)) return false;
  lp->width = row_elems / 2;
  for (FftPlan* p : {&lp->p1, &lp->p2}) {
    int lg = 0;
    while (((int64_t)p->n << (lg + 1)) <= kFreqLongElems && lp->width % (2 << lg) == 0) ++lg;
    p->lg_cp = lg;
  }
  lp->cutoff = cutoff_bins(n, alpha);
  const size_t strips_c = (size_t)lp->width >> lp->p1.lg_cp;
  lp->partial_bytes = strips_c * n * sizeof(float);                            // per tensor
  lp->scratch_bytes = ((size_t)n * lp->width * sizeof(float2) + 255) & ~(size_t)255;
  return true;
}
static size_t long_lds_bytes(const FftPlan& p) {
  return ((size_t)((p.n + (p.n >> 4) + 1) << p.lg_cp) + (size_t)(p.n + 1) / 2) * sizeof(float2);
}

static bool make_plan(int32_t n, int32_t row_elems, double alpha, int32_t n_batch, FftPlan* p) {
  if (!factor_radices(n, p)) return false;
  int lg = 0;
  while ((2 << lg) <= 64 && (int64_t)n * (2 << lg) <= kFreqMaxElems && row_elems % (4 << lg) == 0) ++lg;
  if (row_elems % (2 << lg) != 0) return false;
  p->lg_cp = lg;
  p->cutoff = cutoff_bins(n, alpha);
  p->strips = row_elems / (2 << lg);
  // one strip per workgroup.  The split depends on the shape alone, not on the batch, so that a
  // sequence gets the same bits whatever it is batched with.
  (void)n_batch;
  p->groups = p->strips;
  return true;
}

static size_t freq_lds_bytes(const FftPlan& p, bool fixed) {
  return ((size_t)((p.n + (p.n >> 4) + 1) << p.lg_cp) + (size_t)(fixed ? p.n / 8 : (p.n + 1) / 2)) * sizeof(float2);
}

}  // namespace ct

using namespace ct;

extern "C" {

size_t ct_frequency_workspace_bytes(int32_t n_batch, int32_t n_tokens, int32_t row_elems) {
  FftPlan p;
  if (n_batch <= 0 || n_tokens <= 0 || row_elems <= 0) return 0;
  if (n_tokens > kFreqMaxTokens) {
    LongPlan lp;
    if (!make_long_plan(n_tokens, row_elems, 0.5, &lp)) return 0;
    return (((size_t)n_batch * 2 * lp.partial_bytes + 255) & ~(size_t)255) + lp.scratch_bytes;
  }
  if (!make_plan(n_tokens, row_elems, 0.5, n_batch, &p)) return 0;
  return (size_t)n_batch * 2 * p.groups * n_tokens * sizeof(float);
}

ct_status ct_frequency_scores(const void* k, const void* v, int32_t n_batch, int64_t batch_stride, int32_t n_tokens,
                              int32_t row_elems, double alpha, float* scores, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (n_batch < 0 || n_tokens < 0 || row_elems <= 0) return fail(CT_ERR_SHAPE, "negative size");
  if (n_batch == 0 || n_tokens == 0) return CT_OK;
  if (k == nullptr || v == nullptr || scores == nullptr) return fail(CT_ERR_NULL, "k, v and scores must be non-NULL");
  if (!(alpha >= 0.0 && alpha <= 1.0)) return fail(CT_ERR_RATIO, "alpha %g is outside [0, 1]", alpha);
  if (row_elems % 2 != 0) return fail(CT_ERR_SHAPE, "row_elems %d must be even", row_elems);
  if (n_batch > 1 && batch_stride < (int64_t)n_tokens * row_elems)
    return fail(CT_ERR_SHAPE, "batch_stride %lld is smaller than one sequence", (long long)batch_stride);
  hipStream_t s = (hipStream_t)stream;
  if (n_tokens > kFreqMaxTokens) {
    LongPlan lp;
    if (!make_long_plan(n_tokens, row_elems, alpha, &lp))
      return fail(CT_ERR_UNSUPPORTED,
                  "n_tokens %d: needs a divisor pair N1 N2 with both at most %d and no prime factor above 5, below 2^24",
                  n_tokens, kFreqMaxTokens);
    const size_t partial_all = ((size_t)n_batch * 2 * lp.partial_bytes + 255) & ~(size_t)255;
    const size_t need = partial_all + lp.scratch_bytes;
    if (workspace == nullptr || workspace_bytes < need)
      return fail(CT_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
    if (((uintptr_t)workspace & 255) != 0) return fail(CT_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    for (const void* fn : {(const void*)freq_long_a_kernel, (const void*)freq_long_b_kernel, (const void*)freq_long_c_kernel}) {
      hipError_t ea = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (ea != hipSuccess) return hip_fail(ea, "hipFuncSetAttribute(long-sequence frequency kernels)");
    }
    float* partial = (float*)workspace;
    float2* scratch = (float2*)((char*)workspace + partial_all);
    const int n1 = lp.p1.n, n2 = lp.p2.n;
    const unsigned grid_ac = (unsigned)((size_t)n2 * (lp.width >> lp.p1.lg_cp));
    const unsigned grid_b = (unsigned)((size_t)n1 * (lp.width >> lp.p2.lg_cp));
    const int groups = lp.width >> lp.p1.lg_cp;
    // one tensor at a time through the one scratch array (the launches of a stream run in order)
    for (int t = 0; t < n_batch * 2; ++t) {
      const uint16_t* src = (const uint16_t*)((t & 1) ? v : k) + (int64_t)(t >> 1) * batch_stride;
      launch_kernel(KC_FREQ, freq_long_a_kernel, dim3(grid_ac), dim3(kFreqThreads), (unsigned)long_lds_bytes(lp.p1), s, src,
                    lp.width, lp.p1, n_tokens, n2, scratch);
      launch_kernel(KC_FREQ, freq_long_b_kernel, dim3(grid_b), dim3(kFreqThreads), (unsigned)long_lds_bytes(lp.p2), s, scratch,
                    lp.width, lp.p2, n_tokens, n1, lp.cutoff);
      launch_kernel(KC_FREQ, freq_long_c_kernel, dim3(grid_ac), dim3(kFreqThreads), (unsigned)long_lds_bytes(lp.p1), s,
                    (const float2*)scratch, lp.width, lp.p1, n_tokens, n2,
                    partial + (size_t)t * (lp.partial_bytes / sizeof(float)));
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "long-sequence frequency score launch");
    const int64_t total = (int64_t)n_batch * n_tokens;
    launch_kernel(KC_FREQ, freq_finish_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                  (const float*)partial, n_tokens, groups, n_batch, scores);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "frequency score finish launch");
    return CT_OK;
  }
  FftPlan p;
  if (!make_plan(n_tokens, row_elems, alpha, n_batch, &p))
    return fail(CT_ERR_UNSUPPORTED, "n_tokens %d has a prime factor above 5", n_tokens);
  const size_t need = (size_t)n_batch * 2 * p.groups * n_tokens * sizeof(float);
  if (workspace == nullptr || workspace_bytes < need)
    return fail(CT_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
  // power-of-two lengths from 256 on whose strips hold the full kFreqMaxElems values take the kernel
  // with the plan compiled in; everything else the one that reads the plan at run time
  using Kernel = void (*)(const uint16_t*, const uint16_t*, int64_t, int32_t, int32_t, FftPlan, float*);
  Kernel kern = freq_energy_kernel<0>;
  if ((int64_t)n_tokens << p.lg_cp == kFreqMaxElems) {
    switch (n_tokens) {
      case 256: kern = freq_energy_kernel<256>; break;
      case 512: kern = freq_energy_kernel<512>; break;
      case 1024: kern = freq_energy_kernel<1024>; break;
      case 2048: kern = freq_energy_kernel<2048>; break;
      case 4096: kern = freq_energy_kernel<4096>; break;
      default: break;
    }
  }
  const size_t lds = freq_lds_bytes(p, kern != freq_energy_kernel<0>);
  hipError_t ea = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (ea != hipSuccess) return hip_fail(ea, "hipFuncSetAttribute(freq_energy_kernel)");
  const int n_work = n_batch * 2 * p.groups;
  launch_kernel(KC_FREQ, kern, dim3(n_work), dim3(kFreqThreads), (unsigned)lds, s, (const uint16_t*)k, (const uint16_t*)v,
                batch_stride, row_elems, n_work, p, (float*)workspace);
  const int64_t total = (int64_t)n_batch * n_tokens;
  launch_kernel(KC_FREQ, freq_finish_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                (const float*)workspace, n_tokens, p.groups, n_batch, scores);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "frequency score launch");
  return CT_OK;
}

ct_status ct_topk_indices(const float* scores, int32_t n_batch, int32_t n_tokens, int32_t k, int32_t* idx_out,
                          void* stream) {
  if (n_batch < 0 || n_tokens < 0 || k < 0) return fail(CT_ERR_SHAPE, "negative size");
  if (k > n_tokens) return fail(CT_ERR_SHAPE, "k %d exceeds n_tokens %d", k, n_tokens);
  if (n_batch == 0 || k == 0) return CT_OK;
  if (scores == nullptr || idx_out == nullptr) return fail(CT_ERR_NULL, "scores and idx_out must be non-NULL");
  hipStream_t s = (hipStream_t)stream;
  launch_kernel(KC_TOPK, topk_kernel, dim3(n_batch), dim3(1024), 0, s, scores, n_tokens, k, idx_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "topk launch");
  return CT_OK;
}

int32_t ct_frequency_n_selected(int32_t n_tokens, double ratio) {
  if (n_tokens <= 0 || !(ratio > 0.0)) return 0;
  if (ratio >= 1.0) return n_tokens;
  int64_t n = (int64_t)floor(ratio * (double)n_tokens + 1e-9);
  return (int32_t)(n < 1 ? 1 : n);
}

ct_status ct_select_frequency(const void* k, const void* v, int32_t n_batch, int64_t batch_stride, int32_t n_tokens,
                              int32_t row_elems, double alpha, double ratio, int32_t* idx_out, float* scores,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!(ratio >= 0.0 && ratio <= 1.0)) return fail(CT_ERR_RATIO, "ratio %g is outside [0, 1]", ratio);
  ct_status st = ct_frequency_scores(k, v, n_batch, batch_stride, n_tokens, row_elems, alpha, scores, workspace,
                                     workspace_bytes, stream);
  if (st != CT_OK) return st;
  return ct_topk_indices(scores, n_batch, n_tokens, ct_frequency_n_selected(n_tokens, ratio), idx_out, stream);
}

}  // extern "C"
